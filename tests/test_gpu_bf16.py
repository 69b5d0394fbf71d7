"""Gradients stored as bf16: the bf16 entry points against the oracle on the widened values.

Every bf16 value is an fp32 value, so the oracle runs unchanged on `G.float()`; tolerances are those
of the fp32 entry points.  Inputs are the fp32 test matrices rounded to bf16 once, on the host.
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



def to_bf16(G):
    """(bf16 CUDA tensor, the same values as float32 numpy)"""
    t = torch.as_tensor(G).to(torch.bfloat16)
    return t.to(DEV), t.float().numpy()


def assert_dist_close(got, G, ref):
    got = got.cpu().numpy()
    sq = (G.astype(np.float64) ** 2).sum(1)
    tol = max(1e-7, 1e-5 / np.sqrt(G.shape[1])) * (sq[:, None] + sq[None, :]) + 1e-30
    err = np.abs(got - ref)
    assert np.all(err <= tol), f"dist: worst err/tol {np.max(err / tol):.3g}"
    assert np.array_equal(got, got.T) and np.all(np.diag(got) == 0.0)


def assert_out_close(got, ref, scale, rtol=1e-5):
    got = got.detach().cpu().numpy()
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    tol = rtol * np.maximum(np.abs(ref), scale).astype(np.float64) + 1e-37
    bad = np.flatnonzero(~(err <= tol))
    assert bad.size == 0, f"{bad.size} of {ref.size} beyond tolerance; first {bad[:5]}, worst {np.max(err / tol):.3g}"


def test_pairwise_sqdist_bf16_every_n():
    """Aligned rows (tiles of 256 columns streamed into LDS) with an element tail, every n."""
    say("pairwise_sqdist bf16, every n")
    rng = np.random.default_rng(91)
    wide_t, wide = to_bf16((rng.standard_normal((64, 256 * 24 + 72)) + 0.25).astype(np.float32))   # ld % 8 == 0
    for n in range(1, 65):
        for d in (256, 256 * 3 + 77, 256 * 24 + 61, 100):
            ref = O.pairwise_sqdist(np.ascontiguousarray(wide[:n, :d]))
            got = mb.pairwise_sqdist(wide_t[:n, :d])
            assert_dist_close(got, wide[:n, :d], ref)


def test_pairwise_sqdist_bf16_unaligned_and_chunked():
    say("pairwise_sqdist bf16 unaligned")
    rng = np.random.default_rng(92)
    wide_t, wide = to_bf16(rng.standard_normal((13, 5003)).astype(np.float32))     # ld odd
    for lo, hi in [(0, 5003), (1, 4000), (3, 5002), (8, 1032)]:
        ref = O.pairwise_sqdist(np.ascontiguousarray(wide[:, lo:hi]))
        got = mb.pairwise_sqdist(wide_t[:, lo:hi])
        assert_dist_close(got, wide[:, lo:hi], ref)
    ref = O.pairwise_sqdist(wide)
    D = None
    for lo, hi in [(0, 1000), (1000, 1001), (1001, 5003)]:
        D = mb.pairwise_sqdist(wide_t[:, lo:hi].contiguous(), dist=D, accumulate=D is not None)
    assert_dist_close(D, wide, ref)


@pytest.mark.parametrize("n", [39, 51])
def test_pairwise_sqdist_bf16_many_tiles_per_workgroup(n):
    d = 256 * 5000 + 100
    say("pairwise_sqdist bf16 long", n, d)
    Gt = torch.empty(n, d + 28, device=DEV).uniform_(-1.0, 1.0, generator=torch.Generator(DEV).manual_seed(n))
    Gt = Gt.to(torch.bfloat16)[:, :d]
    assert Gt.data_ptr() % 16 == 0 and Gt.stride(0) % 8 == 0
    Gh = Gt.float().cpu().numpy()
    ref = O.pairwise_sqdist(np.ascontiguousarray(Gh))
    got = mb.pairwise_sqdist(Gt)
    assert_dist_close(got, Gh, ref)
    again = mb.pairwise_sqdist(Gt)
    assert torch.equal(got, again)


def test_identical_rows_tie_exactly_bf16():
    say("identical rows bf16")
    rng = np.random.default_rng(93)
    for d in (50021, 50024):
        Gt, G = to_bf16(rng.standard_normal((39, d)).astype(np.float32))
        Gt[33] = Gt[2]
        Gt[17] = Gt[2]
        Gt[38] = Gt[20]
        D = mb.pairwise_sqdist(Gt).cpu().numpy()
        assert D[2, 33] == 0.0 and D[2, 17] == 0.0 and D[17, 33] == 0.0 and D[20, 38] == 0.0
        assert np.array_equal(D[2], D[33]) and np.array_equal(D[2], D[17]) and np.array_equal(D[20], D[38])


@pytest.mark.parametrize("theta,beta,d", [
    (1, 1, 100), (2, 2, 1000), (3, 1, 1000), (4, 2, 4097), (5, 3, 999), (7, 3, 100_000), (8, 3, 5000),
    (11, 3, 70_001), (15, 3, 50_000), (16, 6, 3000), (21, 3, 100_003), (21, 11, 3000), (27, 3, 40_000),
    (32, 10, 2000), (33, 3, 2000), (47, 17, 1500), (63, 3, 1500), (64, 34, 1500), (64, 1, 1027),
])
def test_coordwise_selected_bf16(theta, beta, d):
    """bf16 has 8 significand bits, so equal values and equal distances to the median are the rule
    here: the tie order is exercised throughout."""
    say("coordwise_selected bf16", theta, beta, d)
    rng = np.random.default_rng(theta * 1000 + beta + 7)
    n = min(64, theta + 5)
    Gt, G = to_bf16(rng.standard_normal((n, d)).astype(np.float32))
    ext = rng.permutation(n)[:theta].astype(np.int32)
    ref, scale = O.coordwise_selected(G, ext, beta, want_scale=True)
    got = mb.coordwise_trimmed_avg(Gt, torch.as_tensor(ext).to(DEV), beta)
    assert_out_close(got, ref, scale)


def test_coordwise_selected_bf16_strided_unaligned():
    say("coordwise bf16 strided")
    rng = np.random.default_rng(94)
    wide_t, wide = to_bf16(rng.standard_normal((15, 6007)).astype(np.float32))
    ext = rng.permutation(15)[:9].astype(np.int32)
    for lo, hi in [(0, 6007), (1, 6000), (2, 4099), (4, 1028)]:
        ref, scale = O.coordwise_selected(np.ascontiguousarray(wide[:, lo:hi]), ext, 5, want_scale=True)
        out = torch.empty(hi - lo + 3, device=DEV)[3 * (lo % 2):][: hi - lo]     # sometimes misaligned out
        mb.coordwise_trimmed_avg(wide_t[:, lo:hi], torch.as_tensor(ext).to(DEV), 5, out=out)
        assert_out_close(out, ref, scale)


@pytest.mark.parametrize("cfg,d,placement", [(1, None, "tail"), (1, None, "random"), (2, None, "tail"),
                                             (3, 300_008, "tail"), (4, 200_003, "random"), (5, 100_001, "tail")])
def test_aggregate_bf16_matches_oracle(cfg, d, placement):
    say("aggregate bf16", cfg, d, placement)
    s = W.spec(cfg)
    Gt = W.make(cfg, DEV, d=d, placement=placement).to(torch.bfloat16)
    G = Gt.float().cpu().numpy()
    ref, ext = O.mbulyan(G, s["f"])
    theta, beta = O.params(s["n"], s["f"])
    _, scale = O.coordwise_selected(G, ext, beta, want_scale=True)
    out, sel = mb.mbulyan_aggregate_ex(Gt, s["f"])
    torch.cuda.synchronize()
    assert sel.cpu().numpy().tolist() == ext.tolist()
    assert_out_close(out, ref, scale)
    out2, sel2 = mb.mbulyan_aggregate_ex(Gt, s["f"])
    assert torch.equal(out, out2) and torch.equal(sel, sel2)


def test_non_finite_byzantine_rows_are_never_chosen_bf16():
    """Rows full of NaN / inf are at distance +inf from everyone: the result is that of the same matrix with
    those rows moved far away (finite), for the whole rule and for the multi-Krum average."""
    say("non-finite rows bf16")
    s = W.spec(2)
    n, f = s["n"], s["f"]
    Gt = W.make(2, DEV, d=60_002).to(torch.bfloat16)       # Byzantine rows are the last f
    far, bad = Gt.clone(), Gt.clone()
    for k in range(f):
        far[n - 1 - k] = 1e10 * (k + 1)
        bad[n - 1 - k] = [float("nan"), float("inf"), -float("inf")][k % 3]
    bad[n - 2, 1::2] = float("nan")
    G = far.float().cpu().numpy()
    ref, ext = O.mbulyan(G, f)
    _, scale = O.coordwise_selected(G, ext, O.params(n, f)[1], want_scale=True)
    out, sel = mb.mbulyan_aggregate_ex(bad, f)
    assert sel.cpu().numpy().tolist() == ext.tolist()
    assert_out_close(out, ref, scale)
    ref, mask = O.multikrum_aggregate(G, f)
    out, mask_g = mb.multikrum_aggregate(bad, f)
    assert np.array_equal(mask_g.cpu().numpy(), mask) and not mask[n - f:].any()
    assert_out_close(out, ref, np.abs(G[mask.astype(bool)]).mean(0))


def test_aggregate_chunked_bf16_equals_whole():
    say("chunked bf16")
    s = W.spec(5)
    d = 300_000
    Gt = W.make(5, DEV, d=d).to(torch.bfloat16)
    whole, sel = mb.mbulyan_aggregate_ex(Gt, s["f"])
    cuts = [0, 70_001, 70_002, 200_000, d]
    chunks = [Gt[:, a:b].contiguous() for a, b in zip(cuts[:-1], cuts[1:])]
    outs, sel2 = mb.mbulyan_aggregate_chunked(chunks, s["f"])
    assert torch.equal(sel, sel2)
    assert torch.equal(whole, torch.cat(outs))
    G = Gt.float().cpu().numpy()
    ref, ext = O.mbulyan(G, s["f"])
    assert sel.cpu().numpy().tolist() == ext.tolist()


def test_multikrum_aggregate_bf16():
    say("multikrum_aggregate bf16")
    for cfg, d in [(1, 50_001), (2, 20_000), (4, 30_004)]:
        s = W.spec(cfg)
        Gt = W.make(cfg, DEV, d=d).to(torch.bfloat16)
        G = Gt.float().cpu().numpy()
        ref, mask = O.multikrum_aggregate(G, s["f"])
        out, mask_g = mb.multikrum_aggregate(Gt, s["f"])
        assert np.array_equal(mask_g.cpu().numpy(), mask)
        assert_out_close(out, ref, np.abs(G[mask.astype(bool)]).mean(0))


def test_coordwise_median_bf16():
    say("median bf16")
    rng = np.random.default_rng(95)
    for n in (1, 2, 7, 11, 20, 39, 64):
        Gt, G = to_bf16(rng.standard_normal((n, 3001)).astype(np.float32))
        ref = O.coordwise_median(G)
        got = mb.coordwise_median(Gt)
        assert_out_close(got, ref, np.abs(ref), rtol=1e-6)
        if n % 2:
            assert np.array_equal(got.cpu().numpy(), ref)


def alg1_compare(got, G, ext, sets, beta):
    """How often the output is not the oracle's own choice but another legitimate one (see
    tests/alg1_check.py).  With bf16 gradients this is not rare: values of 8 significant bits make
    averages that are *exactly* equidistant from the median (in exact arithmetic) about once in a
    thousand coordinates, and which of the two an evaluation takes then hangs on the last bit of
    the average (the oracle divides an fp64 sum, the kernel multiplies an fp32 sum by 1/m).  Measured:
    1e-4 d to 1e-3 d on the workloads below; the tests fail above 2e-3 d."""
    return alg1_check.compare(got.cpu().numpy(), G, ext, sets, beta)[0]


@pytest.mark.parametrize("n,f,d", [(7, 1, 3000), (11, 2, 100_000), (13, 2, 5001), (19, 4, 30_000), (39, 9, 20_011),
                                   (51, 12, 10_000), (64, 15, 4000)])
def test_coordwise_alg1_bf16(n, f, d):
    """Algorithm-1 form on bf16 gradients: sets from the oracle's selection on random data (the
    general membership changes) against the oracle on the widened values.  With 8 significand bits
    the averages tie often; the comparison allows the other candidate where the margin is tiny."""
    say("coordwise_alg1 bf16", n, f, d)
    rng = np.random.default_rng(n * 100 + f + 3)
    Gt, G = to_bf16(rng.standard_normal((n, d)).astype(np.float32))
    theta, beta = O.params(n, f, O.MODE_ALG1)
    D = O.pairwise_sqdist(G)
    ext, sets, m = O.multikrum_select(D, f, theta)
    got = mb.coordwise_trimmed_avg(Gt, torch.as_tensor(ext).to(DEV), beta, agr_sets=torch.as_tensor(sets).to(DEV))
    flips = alg1_compare(got, G, ext, sets, beta)
    assert flips <= max(4, d // 500)


@pytest.mark.parametrize("cfg,d", [(1, None), (2, 400_000), (4, 100_004), (4, 5_000_001)])
def test_aggregate_alg1_mode_bf16(cfg, d):
    """Whole rule in Algorithm-1 mode on the workloads rounded to bf16 (nested sets: above 2^22
    coordinates the kernel for that case runs, below it the general one)."""
    say("aggregate alg1 bf16", cfg, d)
    s = W.spec(cfg)
    Gt = W.make(cfg, DEV, d=d).to(torch.bfloat16)
    G = Gt.float().cpu().numpy()
    theta, beta = O.params(s["n"], s["f"], O.MODE_ALG1)
    D = O.pairwise_sqdist(G)
    ext, sets, m = O.multikrum_select(D, s["f"], theta)
    out, sel = mb.mbulyan_aggregate_ex(Gt, s["f"], mode=mb.MODE_ALG1)
    assert sel.cpu().numpy().tolist() == ext.tolist()
    flips = alg1_compare(out, G, ext, sets, beta)
    assert flips <= max(4, G.shape[1] // 500)
