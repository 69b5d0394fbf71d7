"""The distance pass where the Gram form cancels: gradients with a large common component, squared
norm : squared distance = 1e3 and 1e5 (the regime of Lemma 1's hypothesis: the gradient dominates
its noise).  Algorithm 1's score line and Eq. 4 define the score on |G_i - G_j|^2 itself, which is
what the oracle computes; here the distances are held to that definition *relative to the distance*:

    |D - D_ref| <= 1e-6 D_ref   for every pair of different rows,   0 exactly for copies,

and the extracted list must be the oracle's.  The uncentred Gram form alone cannot meet this (its
error is about 1e-8 of the norms: 1e-3 of D at the larger ratio, the size of the score gaps); the
library notices on the device and runs its second, centred pass.  Byzantine rows come last or
first: a pivot row fixed in advance (say row 0) would then be a Byzantine one.
"""
import sys

import numpy as np
import pytest
import torch

import oracle as O
import paper_1905_04374_amd as mb
from progress import say
import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"



def rel_err(Dg, D):
    off = D > 0
    assert np.all(Dg[~off] == 0.0), "copies must be at distance exactly 0"
    return float(np.max(np.abs(Dg - D)[off] / D[off]))


CASES = [(19, 4, 300_000), (39, 9, 200_064), (51, 12, 100_003)]   # the last: rows not 16-byte aligned


@pytest.mark.parametrize("byz_first", [False, True])
@pytest.mark.parametrize("kappa", [1e3, 1e5])
@pytest.mark.parametrize("n,f,d", CASES)
def test_distances_hold_relative_to_the_distance(n, f, d, kappa, byz_first):
    say("offset workload", n, f, d, kappa, byz_first)
    Gt = W.offset(n, f, d, kappa, DEV, byzantine_first=byz_first)
    G = Gt.cpu().numpy()
    D = O.pairwise_sqdist(G)
    sq = (G.astype(np.float64) ** 2).sum(1)
    hon = np.arange(f, n) if byz_first else np.arange(n - f)
    ratio = (sq[hon][:, None] + sq[hon][None, :]) / np.where(D[np.ix_(hon, hon)] > 0, D[np.ix_(hon, hon)], np.inf)
    assert ratio.max() > kappa            # the input is as ill-conditioned as it says
    for algo in (mb.DIST_GRAM_BF16, mb.DIST_GRAM, mb.DIST_DIRECT):
        Dg = mb.pairwise_sqdist(Gt, algo=algo).cpu().numpy()
        err = rel_err(Dg, D)
        say("  algo", algo, "max |D - D_ref| / D_ref", f"{err:.2e}")
        assert err <= (2e-6 if algo == mb.DIST_DIRECT else 1e-6), (algo, err)
        assert np.array_equal(Dg, Dg.T) and np.all(np.diag(Dg) == 0.0)
    # bf16 storage of the same gradients: another matrix (the rounding adds noise of its own), same bar
    G16 = Gt.to(torch.bfloat16)
    D16 = O.pairwise_sqdist(G16.float().cpu().numpy())
    err = rel_err(mb.pairwise_sqdist(G16).cpu().numpy(), D16)
    say("  bf16 gradients", f"{err:.2e}")
    assert err <= 1e-6
    # the whole rule: the extracted lists are the oracle's
    for mode, omode in ((mb.MODE_SELECTED, O.MODE_SELECTED), (mb.MODE_ALG1, O.MODE_ALG1)):
        theta, beta = O.params(n, f, omode)
        ext, sets, _ = O.multikrum_select(D, f, theta)
        out, sel = mb.mbulyan_aggregate_ex(Gt, f, mode=mode)
        assert sel.cpu().numpy().tolist() == ext.tolist(), (mode, sel.cpu().numpy().tolist(), ext.tolist())
        if omode == O.MODE_SELECTED:
            ref, scale = O.coordwise_selected(G, ext, beta, want_scale=True)
            errs = np.abs(out.cpu().numpy().astype(np.float64) - ref)
            assert np.all(errs <= 1e-5 * np.maximum(np.abs(ref), scale))


def test_chunks_are_refined_one_by_one():
    """Column chunks accumulate into one matrix; each chunk is checked and, if need be, centred on
    its own (any pivot gives the same distances), here with one well-conditioned chunk in between."""
    n, f = 27, 6
    say("offset workload in chunks")
    a = W.offset(n, f, 150_016, 1e5, DEV)
    b = W.make(3, DEV, d=80_000)                      # norms and distances of the same size
    c = W.offset(n, f, 90_001, 1e3, DEV, byzantine_first=False, seed=3)
    whole = torch.cat([a, b, c], dim=1)
    D = O.pairwise_sqdist(whole.cpu().numpy())
    Dg = None
    for chunk in (a, b, c):
        Dg = mb.pairwise_sqdist(chunk, dist=Dg, accumulate=Dg is not None)
    assert rel_err(Dg.cpu().numpy(), D) <= 1e-6
    theta, _ = O.params(n, f)
    ext, _, _ = O.multikrum_select(D, f, theta)
    outs, sel = mb.mbulyan_aggregate_chunked([a, b, c], f)
    assert sel.cpu().numpy().tolist() == ext.tolist()


def test_rows_that_nearly_coincide_are_not_taken_for_copies():
    """Two different rows whose distance is below the rounding of their norms: in the first pass
    G_ii + G_jj - 2 G_ij cancels (to anything from zero to twice the true value), but the rows are
    not bit-identical and must not be merged into one; the second pass resolves them (to 1e-7 of
    their centred norms).  A true copy stays at exactly 0 and shares its distance row."""
    say("near copies")
    n, d = 11, 100_000
    rng = np.random.default_rng(4)
    G = (rng.standard_normal((n, d)) * 0.01 + 1.0).astype(np.float32)  # common component 1, noise 0.01
    G[5] = G[2]                                                        # a copy
    G[7] = G[3] + (rng.standard_normal(d) * 1e-4).astype(np.float32)   # |x|^2 : D = 1e8
    D = O.pairwise_sqdist(G)
    assert D[2, 5] == 0.0 and 5e-4 < D[3, 7] < 2e-3
    for algo in (mb.DIST_GRAM_BF16, mb.DIST_GRAM):
        Dg = mb.pairwise_sqdist(torch.as_tensor(G).to(DEV), algo=algo).cpu().numpy()
        assert Dg[2, 5] == 0.0 and np.array_equal(Dg[2], Dg[5])
        centred = 2 * float(np.median(D[D > 0]))                       # |x_3 - x_p|^2 + |x_7 - x_p|^2, about
        assert abs(Dg[3, 7] - D[3, 7]) <= 1e-7 * centred, (Dg[3, 7], D[3, 7])
        assert Dg[3, 7] > 0.0 and not np.array_equal(Dg[3], Dg[7])
        other = D > 0
        other[3, 7] = other[7, 3] = False
        assert np.max(np.abs(Dg - D)[other] / D[other]) <= 1e-6


def test_a_huge_byzantine_row_harms_only_its_own_distances():
    """Rows as they are in the first pass: a row of norm 1e6 times the others' (first or last) leaves
    the distances among the others as accurate as without it."""
    say("huge row")
    n, f, d = 19, 4, 120_000
    Gt = W.offset(n, f, d, 1e3, DEV)
    for where in (0, n - 1):
        Gh = Gt.clone()
        Gh[where] = Gh[where] * 1e6 + 3e5
        G = Gh.cpu().numpy()
        D = O.pairwise_sqdist(G)
        Dg = mb.pairwise_sqdist(Gh).cpu().numpy()
        assert rel_err(Dg, D) <= 1e-6


def test_degenerate_inputs_through_the_two_pass_path():
    """Edge cases of the check that decides on the second pass: a single gradient, two gradients, all
    gradients identical (every pair a copy: nothing to flag), all zero, and an ill-conditioned input that
    also holds a non-finite Byzantine row (which must neither be chosen as the pivot nor break the check)."""
    say("degenerate inputs")
    d = 50_000
    rng = np.random.default_rng(6)
    # one gradient, two gradients (f = 0)
    one = (rng.standard_normal((1, d)) + 100.0).astype(np.float32)
    assert mb.pairwise_sqdist(torch.as_tensor(one).to(DEV)).cpu().numpy().tolist() == [[0.0]]
    two = np.stack([one[0], one[0] + (rng.standard_normal(d) * 1e-3).astype(np.float32)])
    D = O.pairwise_sqdist(two)
    Dg = mb.pairwise_sqdist(torch.as_tensor(two).to(DEV)).cpu().numpy()
    assert D[0, 1] > 0 and abs(Dg[0, 1] - D[0, 1]) <= 1e-6 * D[0, 1] and Dg[0, 0] == 0.0 and Dg[1, 1] == 0.0
    # all identical, large norm: every distance exactly 0, the rule returns that gradient
    same = np.repeat(one, 11, axis=0)
    assert not mb.pairwise_sqdist(torch.as_tensor(same).to(DEV)).cpu().numpy().any()
    for mode in (mb.MODE_SELECTED, mb.MODE_ALG1):
        out, sel = mb.mbulyan_aggregate_ex(torch.as_tensor(same).to(DEV), 2, mode=mode)
        assert sel.cpu().numpy().tolist() == list(range(sel.numel()))
        assert np.allclose(out.cpu().numpy(), one[0], rtol=3e-7, atol=0)
    # all zero
    zero = torch.zeros(7, d, device=DEV)
    assert not mb.pairwise_sqdist(zero).cpu().numpy().any()
    out, sel = mb.mbulyan_aggregate_ex(zero, 1)
    assert not out.cpu().numpy().any() and sel.cpu().numpy().tolist() == [0, 1, 2, 3, 4]
    # ill-conditioned and a non-finite row, first or last
    n, f = 19, 4
    base = W.offset(n, f, 100_000, 1e5, DEV)
    for where in (0, n - 1):
        bad, far = base.clone(), base.clone()
        bad[where, ::3] = float("nan")
        bad[where, 1::3] = float("inf")
        far[where] = 1e12
        G = far.cpu().numpy()
        Dref = O.pairwise_sqdist(G)
        Dg = mb.pairwise_sqdist(bad).cpu().numpy()
        keep = np.ones(n, bool)
        keep[where] = False
        sub, subg = Dref[np.ix_(keep, keep)], Dg[np.ix_(keep, keep)]
        assert np.max(np.abs(subg - sub)[sub > 0] / sub[sub > 0]) <= 1e-6
        assert np.all(np.isinf(Dg[where, keep])) and Dg[where, where] == 0.0
        theta, _ = O.params(n, f)
        ext, _, _ = O.multikrum_select(Dref, f, theta)
        _, sel = mb.mbulyan_aggregate_ex(bad, f)
        assert sel.cpu().numpy().tolist() == ext.tolist()
