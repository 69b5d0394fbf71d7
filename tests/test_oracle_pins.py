"""Pins of the CPU oracle against what the paper and the mathematics fix.

Nothing here touches the GPU library.  Each pin uses something other than the
oracle's own code: a library routine (scipy pdist, numpy mean / median), an
exhaustive search over subsets, a hand-worked example, or an invariant.
"""
import itertools
import os

import numpy as np
import pytest
from scipy.spatial.distance import pdist, squareform

import oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(20190504)


# ----------------------------------------------------------------- parameters
# Section II-B: n >= 4f+3.  Algorithm 1: theta = n-2f-2, beta = theta-2f.
# Theorem 2 proof / Section II-B prose: n-2f rounds, m-2f values averaged.
@pytest.mark.parametrize("n,f,sel,alg1", [
    (11, 2, (7, 3), (5, 1)), (19, 4, (11, 3), (9, 1)), (27, 6, (15, 3), (13, 1)),
    (39, 9, (21, 3), (19, 1)), (51, 12, (27, 3), (25, 1)), (7, 1, (5, 3), (3, 1)),
    (9, 1, (7, 5), (5, 3)), (5, 0, (5, 5), (3, 3)), (3, 0, (3, 3), (1, 1)),
])
def test_params_closed_forms(n, f, sel, alg1):
    assert O.params(n, f, O.MODE_SELECTED) == sel
    assert O.params(n, f, O.MODE_ALG1) == alg1


@pytest.mark.parametrize("n,f", [(10, 2), (6, 1), (2, 0), (18, 4), (50, 12)])
def test_params_precondition(n, f):
    with pytest.raises(O.PreconditionError):
        O.params(n, f)
    with pytest.raises(O.PreconditionError):
        O.mbulyan(np.zeros((n, 4), np.float32), f)


def test_params_invalid():
    with pytest.raises(ValueError):
        O.params(5, -1)
    with pytest.raises(ValueError):
        O.params(0, 0)


# ------------------------------------------------------------------ distances
@pytest.mark.parametrize("n,d", [(2, 1), (5, 3), (11, 257), (39, 1000), (64, 33)])
def test_distances_match_scipy(n, d):
    G = rng.standard_normal((n, d)).astype(np.float32)
    D = O.pairwise_sqdist(G)
    ref = squareform(pdist(G.astype(np.float64), "sqeuclidean"))
    np.testing.assert_allclose(D, ref, rtol=1e-13, atol=0)
    assert np.array_equal(D, D.T)
    assert np.all(np.diag(D) == 0.0)


def test_distances_row_stride_and_chunks():
    wide = rng.standard_normal((7, 100)).astype(np.float32)
    view = wide[:, 10:70]                       # ld = 100 > d = 60
    ref = squareform(pdist(view.astype(np.float64), "sqeuclidean"))
    np.testing.assert_allclose(O.pairwise_sqdist(view), ref, rtol=1e-13)
    D = np.zeros((7, 7))
    for lo, hi in [(10, 30), (30, 31), (31, 70)]:   # ragged column chunks add up
        O.pairwise_sqdist(wide[:, lo:hi], D)
    np.testing.assert_allclose(D, ref, rtol=1e-13)


def test_distances_duplicates_exact_and_thread_independent():
    G = rng.standard_normal((9, 500)).astype(np.float32)
    G[7] = G[2]
    G[8] = G[2]
    D1 = O.pairwise_sqdist(G, nthreads=1)
    D4 = O.pairwise_sqdist(G, nthreads=4)
    assert np.array_equal(D1, D4)
    assert D1[2, 7] == 0.0 and D1[7, 8] == 0.0
    assert np.array_equal(D1[2], D1[7]) and np.array_equal(D1[2], D1[8])


def test_distances_closed_form():
    # rows a*ones: D = d*(a_i-a_j)^2 exactly for small integers
    a = np.array([0, 1, 3, -2, 7], np.float32)
    G = np.repeat(a[:, None], 1000, axis=1)
    D = O.pairwise_sqdist(G)
    assert np.array_equal(D, 1000.0 * (a[:, None] - a[None, :]).astype(np.float64) ** 2)


# --------------------------------------------------------------------- scores
def _random_dist(n):
    G = rng.standard_normal((n, 6))
    return squareform(pdist(G, "sqeuclidean"))


def _brute_scores(D, f, active):
    """Score by exhaustive search: the minimum, over all q-subsets of the other
    active gradients, of the summed squared distances (no sorting involved)."""
    n = D.shape[0]
    idx = [i for i in range(n) if active[i]]
    q = max(len(idx) - f - 2, 0)
    S = np.full(n, np.inf)
    for i in idx:
        others = [j for j in idx if j != i]
        S[i] = min(sum(D[i, j] for j in sub) for sub in itertools.combinations(others, q))
    return S, q


@pytest.mark.parametrize("n,f", [(3, 0), (5, 0), (7, 1), (8, 1), (8, 2), (6, 3)])
def test_scores_brute_force(n, f):
    for trial in range(5):
        D = _random_dist(n)
        active = np.ones(n, np.uint8)
        if trial >= 2:
            active[rng.choice(n, size=min(trial - 1, n - 1), replace=False)] = 0
        ref, _ = _brute_scores(D, f, active)
        got = O.krum_scores(D, f, active if trial else None)
        fin = np.isfinite(ref)
        assert np.array_equal(np.isfinite(got), fin)
        np.testing.assert_allclose(got[fin], ref[fin], rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------ selection
def _read_golden(name):
    rows = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            rows[key] = [float(v) for v in vals]
    return rows


def test_hand_worked_example():
    g = _read_golden("hand_1d_n7_f1.txt")
    G = np.array(g["x"], np.float32)[:, None]
    D = O.pairwise_sqdist(G)
    ext, sets, m, log = O.multikrum_select(D, 1, 5, want_scores=True)
    for t in range(5):
        assert np.array_equal(log[t], np.array(g[f"scores_round{t}"]))
    assert ext.tolist() == [int(v) for v in g["ext"]]
    assert m.tolist() == [int(v) for v in g["m"]]
    assert [sorted(np.flatnonzero(s).tolist()) for s in sets] == [[1, 2, 3, 4], [1, 3, 4], [1, 4], [4], []]
    out, ext2 = O.mbulyan(G, 1, O.MODE_SELECTED)
    assert ext2.tolist() == ext.tolist() and out[0] == np.float32(g["out_selected"][0])
    out, ext3 = O.mbulyan(G, 1, O.MODE_ALG1)
    assert ext3.tolist() == ext.tolist()[:3] and out[0] == np.float32(g["out_alg1"][0])


@pytest.mark.parametrize("n,f,theta", [(7, 1, 5), (8, 1, 6), (7, 0, 7), (8, 2, 3)])
def test_selection_brute_force(n, f, theta):
    """Every round: winner = exhaustive argmin of brute-force scores, averaged set =
    the q gradients that no other active gradient beats, removal of winners only."""
    for _ in range(4):
        D = _random_dist(n)
        ext, sets, m = O.multikrum_select(D, f, theta)
        active = np.ones(n, np.uint8)
        for t in range(theta):
            S, q = _brute_scores(D, f, active)
            better = [sum(1 for j in range(n) if active[j] and (S[j], j) < (S[i], i)) for i in range(n)]
            win = [i for i in range(n) if active[i] and better[i] == 0]
            assert win == [ext[t]]
            assert sorted(np.flatnonzero(sets[t]).tolist()) == sorted(
                i for i in range(n) if active[i] and better[i] < q)
            assert m[t] == q
            active[ext[t]] = 0


def test_selection_permutation_equivariance():
    n, f = 11, 2
    G = rng.standard_normal((n, 40)).astype(np.float32)
    out, ext = O.mbulyan(G, f)
    perm = rng.permutation(n)
    out_p, ext_p = O.mbulyan(G[perm], f)
    assert np.array_equal(perm[ext_p], ext)        # same workers, same order
    assert np.array_equal(out_p, out)              # sums are taken in sorted order
    out_a, ext_a = O.mbulyan(G, f, O.MODE_ALG1)
    out_ap, ext_ap = O.mbulyan(G[perm], f, O.MODE_ALG1)
    assert np.array_equal(perm[ext_ap], ext_a)
    np.testing.assert_allclose(out_ap, out_a, rtol=1e-6, atol=1e-7)
    assert np.array_equal(ext_a, ext[:len(ext_a)])  # both modes share the rounds


def test_score_ties_go_to_the_smaller_index():
    G = np.zeros((7, 3), np.float32)               # all identical: every score 0
    _, ext = O.mbulyan(G, 1)
    assert ext.tolist() == [0, 1, 2, 3, 4]


# ----------------------------------------------------------- coordinate phase
def _brute_closest_avg(vals, beta):
    """beta-subset minimising the sorted tuple of (|v-med| in fp32, rank), by search."""
    v = np.sort(np.asarray(vals, np.float32))
    th = len(v)
    med = v[th // 2] if th % 2 else np.float32(0.5) * np.float32(v[th // 2 - 1] + v[th // 2])
    delta = np.abs((v - med).astype(np.float32))
    best = min(itertools.combinations(range(th), beta),
               key=lambda sub: sorted((delta[p], p) for p in sub))
    return np.float32(sum(float(v[p]) for p in best) / beta)


@pytest.mark.parametrize("theta,beta", [(1, 1), (3, 1), (5, 3), (7, 3), (6, 2), (8, 4), (7, 7), (9, 5), (4, 1)])
def test_coordwise_brute_force(theta, beta):
    n, d = theta + 3, 64
    G = rng.standard_normal((n, d)).astype(np.float32)
    G[:, :8] = rng.integers(-3, 4, size=(n, 8))    # many exact ties
    ext = rng.permutation(n)[:theta].astype(np.int32)
    out = O.coordwise_selected(G, ext, beta)
    ref = np.array([_brute_closest_avg(G[ext, c], beta) for c in range(d)], np.float32)
    assert np.array_equal(out, ref)


def test_coordwise_special_cases_numpy():
    n, d = 15, 300
    G = (rng.standard_normal((n, d)) * 10).astype(np.float32)
    ext = rng.permutation(n)[:9].astype(np.int32)
    # beta = theta: plain mean of the extracted rows
    np.testing.assert_allclose(O.coordwise_selected(G, ext, 9),
                               G[ext].astype(np.float64).mean(0).astype(np.float32), rtol=1e-6, atol=1e-6)
    # beta = 1, odd theta: the coordinate-wise median
    assert np.array_equal(O.coordwise_selected(G, ext, 1), np.median(G[ext], axis=0))
    # even theta, beta = 2: the two middle values -> numpy's median
    ext8 = ext[:8]
    np.testing.assert_allclose(O.coordwise_selected(G, ext8, 2), np.median(G[ext8].astype(np.float64), axis=0),
                               rtol=1e-6, atol=1e-7)
    assert np.array_equal(O.coordwise_median(G), np.median(G, axis=0))
    np.testing.assert_allclose(O.coordwise_median(G[:14]), np.median(G[:14].astype(np.float64), axis=0),
                               rtol=1e-6, atol=1e-7)


def test_coordwise_invariants():
    n, d, theta, beta = 13, 500, 9, 5
    G = rng.standard_normal((n, d)).astype(np.float32)
    ext = rng.permutation(n)[:theta].astype(np.int32)
    out, scale = O.coordwise_selected(G, ext, beta, want_scale=True)
    assert np.all(out >= G[ext].min(0)) and np.all(out <= G[ext].max(0))
    assert np.all(scale >= np.abs(out) * (1 - 1e-6))
    # order of the extracted rows is irrelevant
    assert np.array_equal(O.coordwise_selected(G, ext[::-1], beta), out)
    # scaling by a power of two is exact
    assert np.array_equal(O.coordwise_selected(G * np.float32(8), ext, beta), out * np.float32(8))
    # negation mirrors the result unless a tie is broken towards the smaller value
    neg = O.coordwise_selected(-G, ext, beta)
    assert np.mean(neg == -out) > 0.99
    # rows outside ext do not matter
    G2 = G.copy()
    G2[np.setdiff1d(np.arange(n), ext)] = 1e9
    assert np.array_equal(O.coordwise_selected(G2, ext, beta), out)


def test_coordwise_tie_prefers_smaller_value():
    # values -1 0 1 around median 0, beta = 2: |.| ties, the smaller value wins
    G = np.array([[-1.0], [0.0], [1.0]], np.float32)
    out = O.coordwise_selected(G, np.arange(3, dtype=np.int32), 2)
    assert out[0] == np.float32(-0.5)


def test_alg1_reduces_to_selected_for_singleton_sets():
    n, d, theta, beta = 12, 200, 7, 3
    G = rng.standard_normal((n, d)).astype(np.float32)
    ext = rng.permutation(n)[:theta].astype(np.int32)
    sets = np.zeros((theta, n), np.uint8)
    sets[np.arange(theta), ext] = 1
    assert np.array_equal(O.coordwise_alg1(G, ext, sets, beta), O.coordwise_selected(G, ext, beta))


def test_alg1_against_numpy_formulation():
    n, d, theta, beta = 11, 300, 5, 1
    G = rng.standard_normal((n, d)).astype(np.float32)
    ext = rng.permutation(n)[:theta].astype(np.int32)
    sets = (rng.random((theta, n)) < 0.5).astype(np.uint8)
    sets[:, 0] = 1
    out, scale, margin, alt = O.coordwise_alg1(G, ext, sets, beta, want_extra=True)
    med = np.median(G[ext], axis=0)
    agr = np.stack([G[s.astype(bool)].astype(np.float64).mean(0) for s in sets]).astype(np.float32)
    delta = np.abs(agr - med[None, :])
    order = np.argsort(delta, axis=0, kind="stable")
    pick = np.take_along_axis(agr, order[:1], 0)[0]
    second = np.take_along_axis(agr, order[1:2], 0)[0]
    clear = margin > 1e-6
    assert clear.mean() > 0.95
    assert np.array_equal(out[clear], pick[clear])
    assert np.array_equal(alt[clear], second[clear])
    assert np.all(margin >= 0)


def _alg1_case(e_vals, groups):
    """(G, ext, sets) with d = 1: the extracted rows hold e_vals, every group of values gets rows of
    its own, and round t averages group t."""
    rows = list(e_vals)
    sets = []
    for g in groups:
        sets.append(list(range(len(rows), len(rows) + len(g))))
        rows += list(g)
    n, theta = len(rows), len(e_vals)
    assert theta == len(groups)
    G = np.array(rows, np.float32)[:, None]
    S = np.zeros((theta, n), np.uint8)
    for t, members in enumerate(sets):
        S[t, members] = 1
    return G, np.arange(theta, dtype=np.int32), S


def test_alg1_margin_and_alternative_hand_worked():
    """The runner-up aid of the Algorithm-1 comparison (margin, alt), for beta = 1 and beta > 1 and
    with averages that repeat, against cases worked by hand (tests/golden)."""
    seen = 0
    with open(os.path.join(GOLDEN, "hand_alg1_margin_alt.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            head, e_part, g_part, exp = [p.strip() for p in line.split("|")]
            name, beta = head.split()
            e_vals = [float(v) for v in e_part.split()]
            groups = [[float(v) for v in g.split()] for g in g_part.split(";")]
            want = [float(v) for v in exp.split()]
            G, ext, S = _alg1_case(e_vals, groups)
            out, scale, margin, alt = O.coordwise_alg1(G, ext, S, int(beta), want_extra=True)
            assert out[0] == pytest.approx(want[0], rel=3e-7), name
            assert margin[0] == want[1] or margin[0] == pytest.approx(want[1], rel=3e-7), name
            assert alt[0] == pytest.approx(want[2], rel=3e-7), name
            # the rows averaged into a round never enter the scale through their sign
            assert scale[0] == pytest.approx(max(np.mean(np.abs(g)) for g in groups), rel=1e-6), name
            seen += 1
    assert seen == 6


def test_alg1_acceptance_with_several_near_equidistant_averages():
    """oracle.alg1_accepts on hand-made coordinates (d = 1).  M = 10 (extracted values 9 10 11), scale = 12
    (the largest mean absolute value of a round's rows), so the noise band is 4e-6 * 12 = 4.8e-5.
    beta = 1, averages 10.001, 9.99898, 10.00104, 12: closenesses 1.00e-3, 1.02e-3, 1.04e-3, 2: the
    first three lie within the band of the best and are all acceptable, 12 is not, and neither is a
    value between two of them that no choice produces.
    beta = 2, same averages: the pairs among the first three are acceptable, a pair with 12 is not."""
    e_vals = [9.0, 10.0, 11.0]
    groups3 = [[10.001], [9.99898], [10.00104]]
    # a fourth round needs a fourth extracted value; keep M = 10 with extracted 9, 10, 10, 11 -> median 10
    G, ext, S = _alg1_case([9.0, 10.0, 10.0, 11.0], groups3 + [[12.0]])
    col = G[:, 0]
    a = [np.float32(10.001), np.float32(9.99898), np.float32(10.00104), np.float32(12.0)]
    for t in range(3):
        assert O.alg1_accepts(col, ext, S, 1, a[t])
    assert not O.alg1_accepts(col, ext, S, 1, a[3])
    assert not O.alg1_accepts(col, ext, S, 1, np.float32(10.0))          # the median itself is no average
    assert not O.alg1_accepts(col, ext, S, 1, np.float32(10.0005))
    for i, j in [(0, 1), (0, 2), (1, 2)]:
        assert O.alg1_accepts(col, ext, S, 2, np.float32((float(a[i]) + float(a[j])) / 2))
    assert not O.alg1_accepts(col, ext, S, 2, np.float32((float(a[0]) + 12.0) / 2))
    # a clear decision leaves no choice: averages 10.001, 9.9, 10.2 -> only the first for beta = 1
    G, ext, S = _alg1_case(e_vals, [[10.001], [9.9], [10.2]])
    assert O.alg1_accepts(G[:, 0], ext, S, 1, np.float32(10.001))
    assert not O.alg1_accepts(G[:, 0], ext, S, 1, np.float32(9.9))
    # and it agrees with out / alt of coordwise_alg1 on the hand-worked cases
    G, ext, S = _alg1_case([2.0, 4.0, 6.0], [[0.0, 10.0], [4.0, 6.0], [2.0, 4.0]])     # case B: out 3, alt 5, margin 0
    assert O.alg1_accepts(G[:, 0], ext, S, 1, np.float32(3.0)) and O.alg1_accepts(G[:, 0], ext, S, 1, np.float32(5.0))
    G, ext, S = _alg1_case([4.0, 5.5, 8.0], [[4.0, 6.0], [5.0], [6.0, 8.0]])            # case A: out 5, alt 7, margin 1
    assert O.alg1_accepts(G[:, 0], ext, S, 1, np.float32(5.0)) and not O.alg1_accepts(G[:, 0], ext, S, 1, np.float32(7.0))


def test_alg1_scale_is_the_conditioning_of_an_fp32_running_sum():
    """Why the Algorithm-1 output is compared on the scale "largest mean absolute value of the rows
    averaged into any G^agr[t][c]" and not on |G^agr|: an fp32 evaluation of the averages as
    running sums (the order a register-resident kernel uses: the rows of the last round's set,
    then one extracted row added per round from the last round back; Algorithm 1 only fixes the
    sets) is emulated here in numpy float32 and compared with the fp64 averages.  It stays within
    1e-5 of that scale at every coordinate and round, and it cannot stay within 1e-5 of
    |G^agr[t][c]| itself: where the rows cancel in the average the rounding of the partial sums is
    what is left."""
    n, f, d = 39, 9, 200_000
    theta, beta = O.params(n, f, O.MODE_ALG1)
    G = np.random.default_rng(5).standard_normal((n, d)).astype(np.float32)
    D = O.pairwise_sqdist(G)
    ext, sets, m = O.multikrum_select(D, f, theta)
    # the sets of consecutive rounds are nested when no score order changes; build them that way
    # from the oracle's last set so that the running-sum order is exactly the emulated one
    last = np.flatnonzero(sets[theta - 1])
    base = [r for r in last if r != ext[theta - 1]]
    nested = np.zeros((theta, n), np.uint8)
    for t in range(theta):
        nested[t, base] = 1
        nested[t, ext[t:]] = 1
    S = np.zeros(d, np.float32)
    for r in base:                                   # ascending row order
        S = (S + G[r]).astype(np.float32)
    worst_new, broke_old = 0.0, 0
    for t in range(theta - 1, -1, -1):
        S = (S + G[ext[t]]).astype(np.float32)
        mt = int(nested[t].sum())
        a32 = (S * np.float32(1.0 / mt)).astype(np.float32)
        rows = G[nested[t].astype(bool)].astype(np.float64)
        a64 = rows.mean(0)
        scale = np.abs(rows).mean(0)
        err = np.abs(a32.astype(np.float64) - a64)
        worst_new = max(worst_new, float(np.max(err / (1e-5 * np.maximum(np.abs(a64), scale)))))
        broke_old += int(np.sum(err > 1e-5 * np.abs(a64)))
    assert worst_new < 0.25          # a wide margin inside the bound the GPU tests use
    assert broke_old > 100           # the bound on |G^agr| alone is not one an fp32 sum can meet
    # and the oracle reports exactly that scale
    _, scale_o, _, _ = O.coordwise_alg1(G[:, :1000], ext, nested, beta, want_extra=True)
    ref = np.max([np.abs(G[nested[t].astype(bool), :1000]).mean(0) for t in range(theta)], axis=0)
    np.testing.assert_allclose(scale_o, ref, rtol=1e-6)


def test_same_side_rounding_tie_in_closeness():
    """Two different values on the left of the median whose fp32 differences to it round to the same
    number: the order (closeness, position) then prefers the smaller value.  (A kernel that walks
    outwards from the median prefers the nearer one; the two candidates differ by less than one ulp
    of that difference.)  median 2^25; 0.5 and 1 are both at fp32 distance 2^25 exactly."""
    big = np.float32(2.0 ** 25)
    assert np.float32(big - np.float32(0.5)) == big and np.float32(big - np.float32(1.0)) == big
    G = np.array([[0.5], [1.0], [big], [np.float32(2.0 ** 27)], [np.float32(2.0 ** 28)]], np.float32)
    out = O.coordwise_selected(G, np.arange(5, dtype=np.int32), 2)
    assert out[0] == np.float32((float(big) + 0.5) / 2)


# ------------------------------------------------------------------ whole GAR
def test_no_byzantine_is_plain_average():
    # f = 0: theta = beta = n, every gradient is extracted and averaged
    G = rng.standard_normal((9, 1000)).astype(np.float32)
    out, ext = O.mbulyan(G, 0)
    assert sorted(ext.tolist()) == list(range(9))
    np.testing.assert_allclose(out, G.astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("mode", [O.MODE_SELECTED, O.MODE_ALG1])
def test_identical_inputs_return_that_gradient(mode):
    row = rng.standard_normal(777).astype(np.float32)
    G = np.repeat(row[None, :], 11, axis=0)
    out, _ = O.mbulyan(G, 2, mode)
    np.testing.assert_allclose(out, row, rtol=2e-7, atol=0)


@pytest.mark.parametrize("n,f", [(7, 1), (11, 2), (19, 4)])
def test_output_stays_with_the_correct_gradients(n, f):
    """With at most f arbitrary rows among the theta >= 2f+1 extracted ones, the median lies within
    the range of the correct values (Theorem 2(i) argument).  A value among the beta closest to it is
    no farther from it than the beta-th closest correct value (there are theta-f >= beta correct
    ones), so it, and the average, lie within one width of that range on either side."""
    d = 400
    for trial in range(5):
        G = rng.standard_normal((n, d)).astype(np.float32)
        byz = rng.choice(n, size=f, replace=False)
        G[byz] = (rng.standard_normal((f, d)) * rng.choice([1e-3, 1.0, 1e4], size=(f, 1))).astype(np.float32)
        out, ext = O.mbulyan(G, f)
        good = np.setdiff1d(np.arange(n), byz)
        lo, hi = G[good].min(0), G[good].max(0)
        med = O.coordwise_selected(G, ext, 1)           # beta = 1, odd theta: the median itself
        assert np.all(med >= lo) and np.all(med <= hi)
        width = (hi - lo).astype(np.float64)
        assert np.all(out >= lo - width) and np.all(out <= hi + width)


def test_multikrum_aggregate_against_numpy():
    n, f, d = 11, 2, 500
    G = rng.standard_normal((n, d)).astype(np.float32)
    G[-f:] *= 30
    out, mask = O.multikrum_aggregate(G, f)
    D = squareform(pdist(G.astype(np.float64), "sqeuclidean"))
    S, q = _brute_scores(D, f, np.ones(n, np.uint8))
    best = np.argsort(S, kind="stable")[:n - f - 2]
    assert sorted(np.flatnonzero(mask).tolist()) == sorted(best.tolist()) and q == n - f - 2
    np.testing.assert_allclose(out, G[best].astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)
    with pytest.raises(O.PreconditionError):
        O.multikrum_aggregate(G[:6], 2)
