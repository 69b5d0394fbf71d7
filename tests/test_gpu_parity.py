"""Parity of the HIP library (through its C ABI) with the CPU oracle, step by step and end
to end, on seeded inputs that span several tiles and a ragged tail.

Bars: indices, masks and counts bit-exact; scores bit-exact when fed the oracle's distances;
distances within 1e-7 of the squared norms involved (Gram form) or 2e-6 relative (direct
form); outputs within 1e-5 of max(|reference|, mean |averaged values|), the conditioning scale of an
average evaluated in fp32.
"""
import sys

import numpy as np
import pytest
import torch

import alg1_check
import oracle as O
import paper_1905_04374_amd as mb
from progress import say
import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


ALGOS = [mb.DIST_DIRECT, mb.DIST_GRAM, mb.DIST_GRAM_BF16]



def gpu(x):
    return torch.as_tensor(x).to(DEV)


def assert_out_close(got, ref, scale, rtol=1e-5, what="out"):
    got = got.detach().cpu().numpy() if torch.is_tensor(got) else got
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    tol = rtol * np.maximum(np.abs(ref), scale).astype(np.float64) + 1e-37
    bad = np.flatnonzero(~(err <= tol))
    assert bad.size == 0, (f"{what}: {bad.size} of {ref.size} beyond tolerance; first {bad[:5]}, "
                           f"got {got[bad[:5]]}, ref {ref[bad[:5]]}, worst ratio {np.max(err / tol):.3g}")


def assert_dist_close(got, G, ref, algo):
    """|D - ref| <= 1e-7 (|x_i|^2 + |x_j|^2) for the Gram form (where that exceeds 2.6e-5 D the library
    runs its second pass and the bound is on the centred norms: tests/test_gpu_conditioning.py), 2e-6 D for
    the direct form.  1e-7 holds from ten thousand coordinates on; below, max(1e-7, 1e-5 / sqrt(d))."""
    got = got.cpu().numpy()
    sq = (G.astype(np.float64) ** 2).sum(1)
    if algo == mb.DIST_DIRECT:
        tol = 2e-6 * ref + 1e-30
    else:
        # rounding errors of independent signs: the bound falls with the square root of the number of
        # coordinates down to 1e-7 (measured: about 5e-6 / sqrt(d); 1e-8 at d >= 1e5); the fp32
        # matrix-core variant also rounds its products
        c = 1e-5 if algo == mb.DIST_GRAM_BF16 else 2e-5
        tol = max(1e-7, c / np.sqrt(G.shape[1])) * (sq[:, None] + sq[None, :]) + 1e-30
    err = np.abs(got - ref)
    assert np.all(err <= tol), f"dist: worst err/tol {np.max(err / tol):.3g}"
    assert np.array_equal(got, got.T) and np.all(np.diag(got) == 0.0)


# ------------------------------------------------------------------ distances
SHAPES = [(1, 5), (2, 1), (3, 31), (8, 128), (11, 1000), (16, 4096), (17, 4099), (19, 70001),
          (32, 33333), (39, 65537), (48, 8191), (51, 20000), (64, 12345)]


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("n,d", SHAPES)
def test_pairwise_sqdist(n, d, algo):
    say("pairwise_sqdist", n, d, algo)
    rng = np.random.default_rng(n * 1000 + d)
    G = (rng.standard_normal((n, d)) + 0.5).astype(np.float32)
    ref = O.pairwise_sqdist(G)
    got = mb.pairwise_sqdist(gpu(G), algo=algo)
    torch.cuda.synchronize()
    assert_dist_close(got, G, ref, algo)


@pytest.mark.parametrize("algo", ALGOS)
def test_pairwise_sqdist_strided_unaligned_and_chunked(algo):
    say("pairwise_sqdist strided", algo)
    rng = np.random.default_rng(5)
    wide = rng.standard_normal((13, 5003)).astype(np.float32)
    gw = gpu(wide)
    for lo, hi in [(0, 5003), (1, 4000), (3, 5002), (4, 1028)]:    # ld = 5003 (odd), shifted starts
        ref = O.pairwise_sqdist(wide[:, lo:hi])
        got = mb.pairwise_sqdist(gw[:, lo:hi], algo=algo)
        assert_dist_close(got, wide[:, lo:hi], ref, algo)
    # column chunks accumulate into one matrix
    ref = O.pairwise_sqdist(wide)
    D = None
    for lo, hi in [(0, 1000), (1000, 1001), (1001, 5003)]:
        chunk = gw[:, lo:hi].contiguous()
        D = mb.pairwise_sqdist(chunk, dist=D, accumulate=D is not None, algo=algo)
    assert_dist_close(D, wide, ref, algo)


@pytest.mark.parametrize("algo", [mb.DIST_GRAM, mb.DIST_GRAM_BF16])
def test_pairwise_sqdist_every_n_with_aligned_rows(algo):
    """Rows that start on 16-byte boundaries take the kernel that streams tiles of 128 columns into
    LDS: every n (every count of load instructions per wave, with and without a missing last row
    pair), one tile, a few tiles and many tiles per workgroup, each with an element tail."""
    say("pairwise_sqdist aligned rows, every n", algo)
    rng = np.random.default_rng(77)
    wide = (rng.standard_normal((64, 128 * 40 + 64)) + 0.25).astype(np.float32)   # ld % 4 == 0
    gw = gpu(wide)
    for n in range(1, 65):
        for d in (128, 128 * 3 + 77, 128 * 40 + 61):
            ref = O.pairwise_sqdist(wide[:n, :d])
            got = mb.pairwise_sqdist(gw[:n, :d], algo=algo)
            assert_dist_close(got, wide[:n, :d], ref, algo)


@pytest.mark.parametrize("algo", [mb.DIST_GRAM, mb.DIST_GRAM_BF16])
@pytest.mark.parametrize("n", [39, 51])
def test_pairwise_sqdist_aligned_rows_many_tiles_per_workgroup(n, algo):
    """More tiles than resident workgroups, so every workgroup walks its tile ring several times."""
    d = 128 * 5000 + 100
    say("pairwise_sqdist aligned rows, long", n, d, algo)
    G = torch.empty(n, d + 28, device=DEV).uniform_(-1.0, 1.0, generator=torch.Generator(DEV).manual_seed(n))[:, :d]
    assert G.data_ptr() % 16 == 0 and G.stride(0) % 4 == 0
    Gh = G.cpu().numpy()
    ref = O.pairwise_sqdist(np.ascontiguousarray(Gh))
    got = mb.pairwise_sqdist(G, algo=algo)
    assert_dist_close(got, Gh, ref, algo)


@pytest.mark.parametrize("algo", ALGOS)
def test_identical_rows_tie_exactly(algo):
    say("identical rows", algo)
    rng = np.random.default_rng(11)
    for d in (50021, 50020):                          # rows not aligned / aligned to 16 bytes
        G = rng.standard_normal((39, d)).astype(np.float32)
        G[33] = G[2]
        G[17] = G[2]
        G[38] = G[20]
        D = mb.pairwise_sqdist(gpu(G), algo=algo).cpu().numpy()
        assert D[2, 33] == 0.0 and D[2, 17] == 0.0 and D[17, 33] == 0.0 and D[20, 38] == 0.0
        assert np.array_equal(D[2], D[33]) and np.array_equal(D[2], D[17]) and np.array_equal(D[20], D[38])


@pytest.mark.parametrize("algo", ALGOS)
def test_distance_pass_is_deterministic(algo):
    say("determinism", algo)
    for d in (300_001, 300_032):                      # rows not aligned / aligned to 16 bytes
        G = gpu(W.make(2, "cpu", d=d))
        a = mb.pairwise_sqdist(G, algo=algo).clone()
        b = mb.pairwise_sqdist(G, algo=algo)
        assert torch.equal(a, b)


# --------------------------------------------------------- scores, selection
@pytest.mark.parametrize("n,f", [(3, 0), (7, 1), (11, 2), (19, 4), (39, 9), (51, 12), (64, 15), (64, 0), (20, 7)])
def test_krum_scores_and_selection_match_oracle(n, f):
    say("select", n, f)
    rng = np.random.default_rng(n * 100 + f)
    G = rng.standard_normal((n, 50)).astype(np.float32)
    if n >= 11:
        G[n - 1] = G[n - 2]            # an exact tie inside the matrix
    D = O.pairwise_sqdist(G)
    Dg = gpu(D)
    assert np.array_equal(mb.krum_scores(Dg, f).cpu().numpy(), O.krum_scores(D, f))
    active = (rng.random(n) < 0.7).astype(np.uint8)
    active[:2] = 1
    assert np.array_equal(mb.krum_scores(Dg, f, gpu(active)).cpu().numpy(), O.krum_scores(D, f, active))
    for theta in sorted({1, max(1, n - 2 * f - 2), max(1, n - 2 * f), n}):
        ext, sets, m = O.multikrum_select(D, f, theta)
        sel_g, sets_g, m_g = mb.multikrum_select(Dg, f, theta)
        assert sel_g.cpu().numpy().tolist() == ext.tolist()
        assert np.array_equal(sets_g.cpu().numpy(), sets)
        assert m_g.cpu().numpy().tolist() == m.tolist()


def test_selection_handles_nan_distances():
    say("select nan")
    D = O.pairwise_sqdist(np.random.default_rng(1).standard_normal((11, 20)).astype(np.float32))
    Dn = D.copy()
    Dn[4, :] = np.nan
    Dn[:, 4] = np.nan
    Dn[4, 4] = 0.0
    Di = np.where(np.isnan(Dn), np.inf, Dn)
    sel_g, _, _ = mb.multikrum_select(gpu(Dn), 2, 7)
    assert sel_g.cpu().numpy().tolist() == O.multikrum_select(Di, 2, 7)[0].tolist()


@pytest.mark.parametrize("n,f,d", [(3, 0, 7), (4, 0, 130), (11, 2, 5), (39, 9, 700), (64, 15, 130), (64, 15, 5000),
                                   (51, 12, 100_003), (27, 6, 65_536)])
def test_selection_from_rows_ordered_by_the_distance_pass(n, f, d):
    """A single-matrix aggregation lets the second distance pass order the rows of the distance matrix (one
    workgroup per row; several rows per workgroup when the launch has fewer workgroups than n, as for the
    short rows here) and the selection kernel start from them; the step entry points form and order the
    matrix inside the selection kernel.  Both ways give the same lists, with copies and a non-finite row in."""
    say("prepared rows", n, f, d)
    rng = np.random.default_rng(1000 * n + d)
    G = rng.standard_normal((n, d)).astype(np.float32)
    if n >= 11:
        G[n - 1] = G[n - 3]                    # copies: exact ties between scores
        G[n - 2] = G[n - 3]
        G[5, d // 2] = np.nan                  # a row at distance +inf from every other
    Gt = gpu(G)
    D = mb.pairwise_sqdist(Gt)
    for mode in (mb.MODE_SELECTED, mb.MODE_ALG1):
        theta, beta = mb.mbulyan_params(n, f, mode)
        if theta < 1 or beta < 1:
            continue
        out, sel = mb.mbulyan_aggregate_ex(Gt, f, mode=mode)
        sel2, sets2, _ = mb.multikrum_select(D, f, theta)
        assert sel.cpu().numpy().tolist() == sel2.cpu().numpy().tolist(), mode
        out2 = mb.coordwise_trimmed_avg(Gt, sel2, beta, agr_sets=sets2 if mode == mb.MODE_ALG1 else None)
        assert torch.equal(out, out2) or np.array_equal(out.cpu().numpy(), out2.cpu().numpy(), equal_nan=True)
    if n >= 2 * f + 3:
        _, mask = mb.multikrum_aggregate(Gt, f)
        _, sets1, _ = mb.multikrum_select(D, f, 1)
        assert np.array_equal(mask.cpu().numpy(), sets1.cpu().numpy()[0])


# ----------------------------------------------------------- coordinate pass
@pytest.mark.parametrize("theta,beta,d", [
    (1, 1, 100), (2, 1, 1000), (2, 2, 1000), (3, 1, 1000), (3, 3, 1024), (4, 2, 4097), (5, 3, 999),
    (6, 4, 5000), (7, 3, 100_000), (7, 7, 5001), (8, 3, 5000), (9, 5, 5000), (11, 3, 70_001), (13, 1, 3000),
    (15, 3, 50_000), (16, 6, 3000), (21, 3, 100_003), (21, 11, 3000), (27, 3, 40_000), (31, 31, 2000),
    (32, 10, 2000), (33, 3, 2000), (47, 17, 1500), (63, 3, 1500), (64, 34, 1500), (64, 64, 1027), (64, 1, 1027),
])
def test_coordwise_selected(theta, beta, d):
    say("coordwise_selected", theta, beta, d)
    rng = np.random.default_rng(theta * 1000 + beta)
    n = min(64, theta + 5)
    G = rng.standard_normal((n, d)).astype(np.float32)
    G[:, : d // 4] = rng.integers(-4, 5, size=(n, d // 4))      # exact ties and duplicates
    ext = rng.permutation(n)[:theta].astype(np.int32)
    ref, scale = O.coordwise_selected(G, ext, beta, want_scale=True)
    got = mb.coordwise_trimmed_avg(gpu(G), gpu(ext), beta)
    assert_out_close(got, ref, scale)


def test_coordwise_same_side_rounding_ties():
    """Two different values on one side of the median whose fp32 differences to it round to the same
    number: the oracle's order (closeness, position) takes the smaller one, the kernel's walk outwards
    from the median the nearer one.  Both are "closest" at the precision the closeness has; the two
    averages differ by less than an ulp of the median, far inside the general tolerance: here the
    bar is 2.5e-7 relative (2 ulps)."""
    say("coordwise same-side ties")
    rng = np.random.default_rng(14)
    d, theta = 4096, 5
    G = np.empty((theta, d), np.float32)
    big = (2.0 ** rng.integers(27, 40, size=d)).astype(np.float32)
    sign = rng.choice([-1.0, 1.0], size=d).astype(np.float32)
    G[0] = sign * 0.5 * rng.integers(1, 4, size=d)          # two small values on the same side of the median,
    G[1] = G[0] + sign * 0.25                                # half an ulp of (median - value) apart at most
    G[2] = sign * big                                        # the median
    G[3] = sign * big * 4
    G[4] = sign * big * 8
    assert np.all(np.abs(G[2] - G[0]).astype(np.float32) == np.abs(G[2] - G[1]).astype(np.float32))
    ext = np.arange(theta, dtype=np.int32)
    for beta in (2, 3):
        ref = O.coordwise_selected(G, ext, beta)
        got = mb.coordwise_trimmed_avg(gpu(G), gpu(ext), beta).cpu().numpy()
        assert np.all(np.abs(got.astype(np.float64) - ref) <= 2.5e-7 * np.abs(ref)), beta


def test_coordwise_selected_strided_unaligned():
    say("coordwise strided")
    rng = np.random.default_rng(8)
    wide = rng.standard_normal((15, 6007)).astype(np.float32)
    gw = gpu(wide)
    ext = rng.permutation(15)[:9].astype(np.int32)
    for lo, hi in [(0, 6007), (1, 6000), (2, 4099), (4, 1028)]:
        ref, scale = O.coordwise_selected(wide[:, lo:hi], ext, 5, want_scale=True)
        out = torch.empty(hi - lo + 3, device=DEV)[3 * (lo % 2):][: hi - lo]     # sometimes misaligned out
        mb.coordwise_trimmed_avg(gw[:, lo:hi], gpu(ext), 5, out=out)
        assert_out_close(out, ref, scale)


def test_coordwise_rejects_bad_indices_with_nan():
    say("coordwise bad idx")
    G = gpu(np.ones((7, 100), np.float32))
    out = mb.coordwise_trimmed_avg(G, gpu(np.array([0, 1, 9], np.int32)), 1)
    assert torch.isnan(out).all()
    # Algorithm-1 form: an index out of range, and an index extracted twice
    sets = gpu(np.ones((3, 7), np.uint8))
    for idx in ([0, 1, 9], [0, 1, -1], [2, 5, 2]):
        out = mb.coordwise_trimmed_avg(G, gpu(np.array(idx, np.int32)), 1, agr_sets=sets)
        assert torch.isnan(out).all(), idx
    out = mb.coordwise_trimmed_avg(G, gpu(np.array([2, 5, 3], np.int32)), 1, agr_sets=sets)
    assert torch.equal(out, torch.ones_like(out))


def test_coordwise_median():
    say("median")
    rng = np.random.default_rng(9)
    for n in (1, 2, 7, 11, 20, 39, 64):
        G = rng.standard_normal((n, 3001)).astype(np.float32)
        ref = O.coordwise_median(G)
        got = mb.coordwise_median(gpu(G)).cpu().numpy()
        assert_out_close(got, ref, np.abs(ref), rtol=1e-6, what=f"median n={n}")
        if n % 2:
            assert np.array_equal(got, ref)


def alg1_compare(got, G, ext, sets, beta):
    """How often the output is not the oracle's own choice but another legitimate one (see
    tests/alg1_check.py): on fp32 gradients a few per million coordinates (measured 10 and 80 of 2^24
    at full size); the tests fail above 1e-4 d."""
    return alg1_check.compare(got.cpu().numpy(), G, ext, sets, beta)[0]


@pytest.mark.parametrize("n,f,d", [(7, 1, 3000), (11, 2, 100_000), (13, 2, 5001), (19, 4, 30_000), (39, 9, 20_011),
                                   (51, 12, 9000), (64, 15, 3000), (64, 0, 2000)])
def test_coordwise_alg1(n, f, d):
    say("coordwise_alg1", n, f, d)
    rng = np.random.default_rng(n * 7 + f)
    G = rng.standard_normal((n, d)).astype(np.float32)
    theta, beta = O.params(n, f, O.MODE_ALG1)
    D = O.pairwise_sqdist(G)
    ext, sets, m = O.multikrum_select(D, f, theta)
    got = mb.coordwise_trimmed_avg(gpu(G), gpu(ext), beta, agr_sets=gpu(sets))
    flips = alg1_compare(got, G, ext, sets, beta)
    assert flips <= max(2, d // 10_000)


@pytest.mark.parametrize("n,theta,beta,d", [(9, 4, 1, 3001), (20, 7, 3, 5000), (39, 19, 1, 20_000), (64, 30, 2, 2000)])
def test_coordwise_alg1_arbitrary_sets(n, theta, beta, d):
    """Membership matrices that no run of multi-Krum would produce (rows enter and leave at will):
    the general path of the kernel, against the oracle's plain evaluation of the same sets."""
    say("coordwise_alg1 arbitrary sets", n, theta, beta, d)
    rng = np.random.default_rng(n * 31 + theta)
    G = rng.standard_normal((n, d)).astype(np.float32)
    ext = rng.permutation(n)[:theta].astype(np.int32)
    sets = (rng.random((theta, n)) < 0.4).astype(np.uint8)
    sets[np.arange(theta), ext] = 1
    sets[theta // 2] = 0                                     # an empty set averages to 0
    got = mb.coordwise_trimmed_avg(gpu(G), gpu(ext), beta, agr_sets=gpu(sets))
    flips = alg1_compare(got, G, ext, sets, beta)
    assert flips <= max(2, d // 10_000)


def test_coordwise_alg1_regular_sets_take_the_register_path():
    """Sets of the regular shape (each round's set = the previous one minus its winner), built by
    hand, so the register-only path is certainly the one compared."""
    say("coordwise_alg1 regular sets")
    rng = np.random.default_rng(77)
    n, theta, beta, d = 23, 9, 3, 10_007
    G = rng.standard_normal((n, d)).astype(np.float32)
    order = rng.permutation(n)
    ext = order[:theta].astype(np.int32)
    base = order[theta:theta + 5]
    sets = np.zeros((theta, n), np.uint8)
    for t in range(theta):
        sets[t, ext[t:]] = 1
        sets[t, base] = 1
    got = mb.coordwise_trimmed_avg(gpu(G), gpu(ext), beta, agr_sets=gpu(sets))
    flips = alg1_compare(got, G, ext, sets, beta)
    assert flips <= 2


# ------------------------------------------------------------------ whole GAR
@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("cfg,d,placement", [(1, None, "tail"), (1, None, "random"), (2, None, "tail"),
                                             (3, 300_007, "tail"), (4, 200_003, "random"), (5, 100_001, "tail")])
def test_aggregate_matches_oracle(cfg, d, placement, algo):
    say("aggregate", cfg, d, placement, algo)
    s = W.spec(cfg)
    Gt = W.make(cfg, DEV, d=d, placement=placement)
    G = Gt.cpu().numpy()
    ref, ext = O.mbulyan(G, s["f"])
    theta, beta = O.params(s["n"], s["f"])
    _, scale = O.coordwise_selected(G, ext, beta, want_scale=True)
    mb.mbulyan_set_dist_algo(algo)
    try:
        out, sel = mb.mbulyan_aggregate(Gt, s["f"])
        torch.cuda.synchronize()
    finally:
        mb.mbulyan_set_dist_algo(mb.DIST_AUTO)
    assert sel.cpu().numpy().tolist() == ext.tolist()
    assert_out_close(out, ref, scale)
    out2, sel2 = mb.mbulyan_aggregate(Gt, s["f"])
    if algo != mb.DIST_DIRECT:
        assert torch.equal(out, out2) and torch.equal(sel, sel2)      # run-to-run bit-identical


@pytest.mark.parametrize("cfg,d", [(1, None), (2, 400_000), (4, 100_003), (4, 4_500_000)])   # the last: above 2^22, the nested-sets kernel
def test_aggregate_alg1_mode(cfg, d):
    say("aggregate alg1", cfg, d)
    s = W.spec(cfg)
    n, f = s["n"], s["f"]
    Gt = W.make(cfg, DEV, d=d)
    G = Gt.cpu().numpy()
    theta, beta = O.params(n, f, O.MODE_ALG1)
    D = O.pairwise_sqdist(G)
    ext, sets, m = O.multikrum_select(D, f, theta)
    ws = torch.empty(mb.mbulyan_workspace_bytes(n, G.shape[1]), dtype=torch.uint8, device=DEV)
    out, sel = mb.mbulyan_aggregate_ex(Gt, f, mode=mb.MODE_ALG1, workspace=ws)
    assert sel.cpu().numpy().tolist() == ext.tolist()
    flips = alg1_compare(out, G, ext, sets, beta)
    assert flips <= max(2, G.shape[1] // 10_000)


def test_aggregate_chunked_equals_whole():
    say("chunked")
    s = W.spec(5)
    d = 150_001
    Gt = W.make(5, DEV, d=d)
    G = Gt.cpu().numpy()
    ref, ext = O.mbulyan(G, s["f"])
    _, scale = O.coordwise_selected(G, ext, 3, want_scale=True)
    cuts = [0, 40_000, 40_001, 100_004, d]
    chunks = [Gt[:, a:b].contiguous() for a, b in zip(cuts[:-1], cuts[1:])]
    outs, sel = mb.mbulyan_aggregate_chunked(chunks, s["f"])
    assert sel.cpu().numpy().tolist() == ext.tolist()
    assert_out_close(torch.cat(outs), ref, scale)
    views = [Gt[:, a:b] for a, b in zip(cuts[:-1], cuts[1:])]            # ld = d views, unaligned starts
    outs2, sel2 = mb.mbulyan_aggregate_chunked(views, s["f"])
    assert sel2.cpu().numpy().tolist() == ext.tolist()
    assert_out_close(torch.cat(outs2), ref, scale)


@pytest.mark.parametrize("in16", [False, True])
def test_aggregate_chunked_alg1_mode(in16):
    """Algorithm-1 mode over column chunks (one selection and one plan for all chunks) against the oracle
    on the whole matrix, and bit-identical to itself from call to call."""
    say("chunked alg1", in16)
    s = W.spec(3)
    n, f, d = s["n"], s["f"], 120_003
    Gt = W.make(3, DEV, d=d)
    if in16:
        Gt = Gt.to(torch.bfloat16)
    G = Gt.float().cpu().numpy()
    theta, beta = O.params(n, f, O.MODE_ALG1)
    ext, sets, m = O.multikrum_select(O.pairwise_sqdist(G), f, theta)
    cuts = [0, 50_000, 50_002, 90_001, d] if in16 else [0, 50_000, 50_001, 90_004, d]
    chunks = [Gt[:, a:b].contiguous() for a, b in zip(cuts[:-1], cuts[1:])]
    outs, sel = mb.mbulyan_aggregate_chunked(chunks, f, mode=mb.MODE_ALG1)
    assert sel.cpu().numpy().tolist() == ext.tolist()
    assert alg1_compare(torch.cat(outs), G, ext, sets, beta) <= max(2, d // 10_000)
    outs2, sel2 = mb.mbulyan_aggregate_chunked(chunks, f, mode=mb.MODE_ALG1)
    assert torch.equal(sel, sel2) and torch.equal(torch.cat(outs), torch.cat(outs2))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("n,f", [(11, 2), (13, 2), (17, 2), (39, 9), (40, 9)])   # beta 3, 5, 9, 3, 4 (selected)
def test_result_does_not_depend_on_alignment(n, f, dtype):
    """The same gradients in a contiguous, 16-byte aligned matrix and in one whose rows start at odd element
    offsets take different kernels (vector loads of two or four coordinates per lane, or element loads); the
    extracted list and every output bit must be the same, in both readings, also for the multi-Krum
    average and the median."""
    say("alignment", n, f, dtype)
    d = 40_001
    rng = np.random.default_rng(7 * n + f)
    mu = rng.standard_normal(d).astype(np.float32)
    G = np.stack([mu + 0.3 * (1 + 0.03 * w) * rng.standard_normal(d).astype(np.float32) for w in range(n)])
    A = gpu(G).to(dtype)
    wide = torch.zeros(n, d + 7, device=DEV, dtype=dtype)
    B = wide[:, 3:3 + d]                                # odd row stride, rows start 3 elements in
    B.copy_(A)
    for mode in (mb.MODE_SELECTED, mb.MODE_ALG1):
        oa, sa = mb.mbulyan_aggregate_ex(A, f, mode=mode)
        ob, sb = mb.mbulyan_aggregate_ex(B, f, mode=mode)
        assert torch.equal(sa, sb) and torch.equal(oa, ob), mode
    ma, ka = mb.multikrum_aggregate(A, f)
    mbb, kb = mb.multikrum_aggregate(B, f)
    assert torch.equal(ka, kb) and torch.equal(ma, mbb)
    assert torch.equal(mb.coordwise_median(A), mb.coordwise_median(B))


@pytest.mark.parametrize("in16", [False, True])
@pytest.mark.parametrize("mode", ["selected", "alg1"])
def test_scaling_by_a_power_of_two_is_exact(mode, in16):
    """Every operation of the path commutes exactly with a scaling of all gradients by a power of two
    (the bf16 pieces, the fp32 and fp64 sums, the comparisons, the weights 1/beta and 1/|set|): the
    same gradients are chosen and the output scales bit for bit.  Holds at any size."""
    say("scaling", mode, in16)
    s = W.spec(3)
    Gt = W.make(3, DEV, d=1_000_003)
    if in16:
        Gt = Gt.to(torch.bfloat16)
    m = mb.MODE_ALG1 if mode == "alg1" else mb.MODE_SELECTED
    out, sel = mb.mbulyan_aggregate_ex(Gt, s["f"], mode=m)
    for factor in (4.0, 0.125):
        out_s, sel_s = mb.mbulyan_aggregate_ex(Gt * factor, s["f"], mode=m)
        assert torch.equal(sel_s, sel)
        assert torch.equal(out_s, out * factor)
    mk, mask = mb.multikrum_aggregate(Gt, s["f"])
    mk_s, mask_s = mb.multikrum_aggregate(Gt * 4.0, s["f"])
    assert torch.equal(mask_s, mask) and torch.equal(mk_s, mk * 4.0)


def test_explicit_theta_beta_and_no_byzantine():
    say("explicit theta/beta, f=0")
    rng = np.random.default_rng(3)
    G = rng.standard_normal((9, 10_001)).astype(np.float32)
    out, sel = mb.mbulyan_aggregate(gpu(G), 0)
    assert sorted(sel.cpu().numpy().tolist()) == list(range(9))
    mean = G.astype(np.float64).mean(0)
    assert_out_close(out, mean.astype(np.float32), np.abs(G).mean(0))
    out, sel = mb.mbulyan_aggregate_ex(gpu(G), 1, theta=5, beta=2)
    D = O.pairwise_sqdist(G)
    ext, _, _ = O.multikrum_select(D, 1, 5)
    ref, scale = O.coordwise_selected(G, ext, 2, want_scale=True)
    assert sel.cpu().numpy().tolist() == ext.tolist()
    assert_out_close(out, ref, scale)


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("mode", ["selected", "alg1"])
def test_non_finite_byzantine_rows_are_never_chosen(algo, mode):
    """Byzantine rows full of NaN / inf have no finite distance to anyone: they are never a neighbour and never
    chosen, so the result is that of the same matrix with those rows moved far away (finite, 1e10)."""
    say("non-finite rows", algo, mode)
    s = W.spec(2)
    n, f = s["n"], s["f"]
    d = 40_003
    Gt = W.make(2, DEV, d=d)                       # Byzantine rows are the last f
    far = Gt.clone()
    bad = Gt.clone()
    for k in range(f):
        far[n - 1 - k] = 1e10 * (k + 1)
        bad[n - 1 - k] = [float("nan"), float("inf"), -float("inf")][k % 3]
    if f >= 2:
        bad[n - 2, ::2] = float("nan")             # a mixed row
    G = far.cpu().numpy()
    omode = O.MODE_ALG1 if mode == "alg1" else O.MODE_SELECTED
    theta, beta = O.params(n, f, omode)
    ext, sets, m = O.multikrum_select(O.pairwise_sqdist(G), f, theta)
    assert set(ext.tolist()).isdisjoint(range(n - f, n))
    mb.mbulyan_set_dist_algo(algo)
    try:
        out, sel = mb.mbulyan_aggregate_ex(bad, f, mode=mb.MODE_ALG1 if mode == "alg1" else mb.MODE_SELECTED)
        torch.cuda.synchronize()
    finally:
        mb.mbulyan_set_dist_algo(mb.DIST_AUTO)
    assert sel.cpu().numpy().tolist() == ext.tolist()
    assert torch.isfinite(out).all()
    if mode == "alg1":
        assert alg1_compare(out, G, ext, sets, beta) <= max(2, d // 10_000)
    else:
        ref, scale = O.coordwise_selected(G, ext, beta, want_scale=True)
        assert_out_close(out, ref, scale)
        ref, mask = O.multikrum_aggregate(G, f)
        out, mask_g = mb.multikrum_aggregate(bad, f)
        assert np.array_equal(mask_g.cpu().numpy(), mask) and not mask[n - f:].any()
        assert_out_close(out, ref, np.abs(G[mask.astype(bool)]).mean(0))


def test_multikrum_aggregate():
    say("multikrum_aggregate")
    for cfg, d in [(1, 50_001), (2, 20_000)]:
        s = W.spec(cfg)
        Gt = W.make(cfg, DEV, d=d)
        G = Gt.cpu().numpy()
        ref, mask = O.multikrum_aggregate(G, s["f"])
        out, mask_g = mb.multikrum_aggregate(Gt, s["f"])
        assert np.array_equal(mask_g.cpu().numpy(), mask)
        assert_out_close(out, ref, np.abs(G[mask.astype(bool)]).mean(0))


def test_aggregate_can_be_captured_in_a_graph():
    """An aggregation with a caller workspace allocates nothing and issues only kernels, so a
    stream capture records it.  Replays (with eager work and
    synchronisation in between, on fresh inputs) must equal the eager result each time."""
    say("graph capture")
    n, f, d = 19, 4, 200_000
    G = W.uniform(n, d, DEV, seed=1)
    ws = torch.empty(mb.mbulyan_workspace_bytes(n, d), dtype=torch.uint8, device=DEV)
    theta, _ = mb.mbulyan_params(n, f)
    out = torch.empty(d, device=DEV)
    sel = torch.empty(theta, device=DEV, dtype=torch.int32)
    for mode in (mb.MODE_SELECTED, mb.MODE_ALG1):
        th, _ = mb.mbulyan_params(n, f, mode)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            mb.mbulyan_aggregate_ex(G, f, mode=mode, out=out, selected_idx=sel[:th], workspace=ws)   # warm-up: one-time set-up
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                mb.mbulyan_aggregate_ex(G, f, mode=mode, out=out, selected_idx=sel[:th], workspace=ws)
        torch.cuda.synchronize()
        for rep in range(3):
            G.copy_(W.uniform(n, d, DEV, seed=2 + rep))
            eager, esel = mb.mbulyan_aggregate_ex(G, f, mode=mode, workspace=ws)
            torch.cuda.synchronize()
            out.zero_()
            sel.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager) and torch.equal(sel[:th], esel), (mode, rep)


def test_binding_refuses_buffers_the_kernels_would_overrun():
    """The C ABI sees pointers only; the binding is where a short, strided or misplaced buffer is caught."""
    say("binding checks")
    G = W.make(1, DEV, d=4096)
    with pytest.raises(ValueError):
        mb.mbulyan_aggregate(G, 2, out=torch.empty(4095, device=DEV))
    with pytest.raises(ValueError):
        mb.mbulyan_aggregate(G, 2, selected_idx=torch.empty(6, device=DEV, dtype=torch.int32))
    with pytest.raises(ValueError):
        mb.mbulyan_aggregate_ex(G, 2, out=torch.empty(8192, device=DEV)[::2])
    with pytest.raises(ValueError):
        mb.coordwise_median(G, out=torch.empty(100, device=DEV))
    with pytest.raises(ValueError):
        mb.pairwise_sqdist(G, dist=torch.empty(10, 11, device=DEV, dtype=torch.float64))
    with pytest.raises(TypeError):
        mb.mbulyan_aggregate(G, 2, out=torch.empty(4096))             # host memory


def test_stream_argument_is_honoured():
    say("stream")
    s = W.spec(1)
    Gt = W.make(1, DEV, d=65_536)
    ref, ext = O.mbulyan(Gt.cpu().numpy(), s["f"])
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        out, sel = mb.mbulyan_aggregate(Gt, s["f"])
    st.synchronize()
    assert sel.cpu().numpy().tolist() == ext.tolist()
    assert np.allclose(out.cpu().numpy(), ref, rtol=1e-5, atol=1e-6)


def test_timing_hooks():
    say("timing")
    Gt = W.make(1, DEV, d=65_536)
    mb.mbulyan_timing_reset()
    mb.mbulyan_timing_enable(True)
    for _ in range(3):
        mb.mbulyan_aggregate(Gt, 2)
    mb.mbulyan_timing_enable(False)
    t = mb.mbulyan_timing_read()
    assert t["dist"][1] == 3 and t["coord"][1] == 3 and t["select"][1] == 3 and t["reduce"][1] == 3
    assert all(0 < t[k][0] < 1000 for k in t)
    mb.mbulyan_timing_reset()
    assert mb.mbulyan_timing_read()["dist"] == (0.0, 0)
