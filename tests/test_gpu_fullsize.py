"""Parity at the full sizes of the workloads, in the launch configuration bench.py times
(mbulyan_aggregate_ex with a caller workspace; the chunked driver for workload 5).

Workloads 3 and 4 are compared with the oracle element by element over the whole output, and so is
workload 5 (n=51, d=1e9 in 4 chunks, 204 GB; the oracle needs a few minutes of host time for it).
"""
import os
import sys
import time

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



def check_chunk(got, ref, scale):
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    tol = 1e-5 * np.maximum(np.abs(ref), scale).astype(np.float64) + 1e-37
    worst = float(np.max(err / tol))
    assert worst <= 1.0, f"worst err/tol {worst:.3g} at {int(np.argmax(err / tol))}"
    return worst


def check_separation(D, f, theta, ext):
    """Scores of every round: the winner beats every gradient that is not a bit-identical copy
    of it by more than 1e-3 relative (otherwise the extracted list would hang on rounding)."""
    _, _, _, log = O.multikrum_select(D, f, theta, want_scores=True)
    worst = np.inf
    for t in range(theta):
        S, w = log[t], ext[t]
        for j in np.flatnonzero(np.isfinite(S)):
            if j != w and D[w, j] != 0.0:
                worst = min(worst, (S[j] - S[w]) / max(S[j], 1e-300))
    assert worst > 1e-3, f"scores separated by only {worst:.2e}"
    return worst


@pytest.mark.parametrize("cfg,dtype", [(3, "f32"), (4, "f32"), (4, "bf16")])
def test_full_size_single_buffer(cfg, dtype):
    """dtype bf16: the workload rounded to bf16 once, through the bf16 entry points; the oracle gets
    the widened values."""
    s = W.spec(cfg)
    n, f, d = s["n"], s["f"], s["d"]
    say("full size", cfg, dtype, n, f, d)
    theta, beta = O.params(n, f)
    Gt = W.make(cfg, DEV)
    if dtype == "bf16":
        G16 = torch.empty(n, d, device=DEV, dtype=torch.bfloat16)
        for r in range(n):
            G16[r].copy_(Gt[r])
        Gt = G16
    ws = torch.empty(mb.mbulyan_workspace_bytes(n, d), dtype=torch.uint8, device=DEV)
    out, sel = mb.mbulyan_aggregate_ex(Gt, f, workspace=ws)
    Dg = mb.pairwise_sqdist(Gt, workspace=ws).cpu().numpy()
    torch.cuda.synchronize()
    say("gpu done; copying", round(4e-9 * n * d, 1), "GB to the host")
    G = np.empty((n, d), np.float32)
    for r in range(n):
        G[r] = Gt[r].float().cpu().numpy()
    got = out.cpu().numpy()
    sel = sel.cpu().numpy()
    del Gt, out
    torch.cuda.empty_cache()
    t0 = time.time()
    D = O.pairwise_sqdist(G)
    say("oracle distances", round(time.time() - t0, 1), "s")
    ext, _, _ = O.multikrum_select(D, f, theta)
    gap = check_separation(D, f, theta, ext)
    assert sel.tolist() == ext.tolist()
    sq = np.array([float(np.dot(G[r, :1 << 20].astype(np.float64), G[r, :1 << 20])) for r in range(n)]) * (d / (1 << 20))
    assert np.all(np.abs(Dg - D) <= 1e-7 * (sq[:, None] + sq[None, :]))
    rel = np.abs(Dg - D)[D > 0] / D[D > 0]
    rel_norms = float(np.max(np.abs(Dg - D) / (sq[:, None] + sq[None, :])))
    t0 = time.time()
    worst = 0.0
    step = 1 << 24
    for lo in range(0, d, step):                       # oracle coordinate phase in slabs
        hi = min(d, lo + step)
        ref, scale = O.coordwise_selected(G[:, lo:hi], ext, beta, want_scale=True)
        worst = max(worst, check_chunk(got[lo:hi], ref, scale))
    say(f"cfg {cfg} {dtype}: selected {ext.tolist()}, score gap {gap:.2e}, dist err max {rel.max():.2e} of D, {rel_norms:.2e} of the norms, "
        f"out worst err/tol {worst:.3g}, oracle coordinate phase {time.time() - t0:.1f} s")


@pytest.mark.parametrize("cfg", [3, 4])
def test_full_size_alg1_mode(cfg):
    """Algorithm-1 mode at full size: extracted list exact, output compared over a sample of 2^24
    coordinates spread over the whole range (the oracle evaluates theta averages per coordinate)."""
    s = W.spec(cfg)
    n, f, d = s["n"], s["f"], s["d"]
    say("full size alg1", cfg, n, f, d)
    theta, beta = O.params(n, f, O.MODE_ALG1)
    Gt = W.make(cfg, DEV)
    ws = torch.empty(mb.mbulyan_workspace_bytes(n, d), dtype=torch.uint8, device=DEV)
    out, sel = mb.mbulyan_aggregate_ex(Gt, f, mode=mb.MODE_ALG1, workspace=ws)
    Dg = mb.pairwise_sqdist(Gt, workspace=ws).cpu().numpy()
    torch.cuda.synchronize()
    G = np.empty((n, d), np.float32)
    for r in range(n):
        G[r] = Gt[r].cpu().numpy()
    got = out.cpu().numpy()
    sel = sel.cpu().numpy()
    del Gt, out
    torch.cuda.empty_cache()
    D = O.pairwise_sqdist(G)
    ext, sets, m = O.multikrum_select(D, f, theta)
    assert sel.tolist() == ext.tolist()
    assert np.max(np.abs(Dg - D)[D > 0] / D[D > 0]) < 1e-5
    blocks = 64
    width = (1 << 24) // blocks
    flips = 0
    worst = 0.0
    for b in range(blocks):
        lo = (d - width) * b // (blocks - 1)
        fl, w = alg1_check.compare(got[lo:lo + width], G[:, lo:lo + width], ext, sets, beta, f"block {b}")
        flips += fl
        worst = max(worst, w)
    assert flips <= (1 << 24) // 10_000
    say(f"cfg {cfg} alg1: selected {ext.tolist()}, worst err/tol {worst:.3g}, ambiguous choices {flips} of {1 << 24}")


def test_full_size_chunked_both_modes():
    """Workload 5 at its full size (n = 51, d = 1e9 as four chunks of 51 GB), both readings of the rule
    on the same resident chunks.  The oracle's distances are accumulated once over all coordinates;
    the outputs are compared over every coordinate (theta = n-2f rows per coordinate) and, for the
    Algorithm-1 reading (theta averages of up to 37 rows per coordinate), over 64 blocks of 2^18
    coordinates spread over the four chunks.  MB_CFG5_REDUCED=1 runs a tenth of d (for a quick look)."""
    s = W.spec(5)
    n, f, nchunks = s["n"], s["f"], s["chunks"]
    d = s["d"] // 10 if os.environ.get("MB_CFG5_REDUCED") == "1" else s["d"]
    say("chunked", n, f, d, nchunks)
    theta, beta = O.params(n, f)
    theta1, beta1 = O.params(n, f, O.MODE_ALG1)
    bounds = [d * k // nchunks for k in range(nchunks + 1)]
    chunks = []
    for k in range(nchunks):
        g = torch.empty(n, bounds[k + 1] - bounds[k], device=DEV, dtype=torch.float32)
        W.fill(5, g, bounds[k])
        chunks.append(g)
    ws = torch.empty(mb.mbulyan_workspace_bytes(n, max(c.shape[1] for c in chunks)), dtype=torch.uint8, device=DEV)
    outs, sel = mb.mbulyan_aggregate_chunked(chunks, f, workspace=ws)
    outs1, sel1 = mb.mbulyan_aggregate_chunked(chunks, f, mode=mb.MODE_ALG1, workspace=ws)
    torch.cuda.synchronize()
    sel, sel1 = sel.cpu().numpy(), sel1.cpu().numpy()
    D = np.zeros((n, n))
    host = np.empty((n, chunks[0].shape[1]), np.float32)
    t0 = time.time()
    for k in range(nchunks):                           # distances accumulate over the chunks
        w = chunks[k].shape[1]
        for r in range(n):
            host[r, :w] = chunks[k][r].cpu().numpy()
        O.pairwise_sqdist(host[:, :w], D)
        say("oracle distances of chunk", k, round(time.time() - t0, 1), "s")
    ext, _, _ = O.multikrum_select(D, f, theta)
    ext1, sets1, _ = O.multikrum_select(D, f, theta1)
    gap = check_separation(D, f, theta, ext)
    assert sel.tolist() == ext.tolist()
    assert sel1.tolist() == ext1.tolist()
    worst, worst1, flips, sampled = 0.0, 0.0, 0, 0
    blocks, width = 16, 1 << 18
    for k in range(nchunks):
        w = chunks[k].shape[1]
        for r in range(n):
            host[r, :w] = chunks[k][r].cpu().numpy()
        got = outs[k].cpu().numpy()
        step = 1 << 24
        for lo in range(0, w, step):
            hi = min(w, lo + step)
            ref, scale = O.coordwise_selected(host[:, lo:hi], ext, beta, want_scale=True)
            worst = max(worst, check_chunk(got[lo:hi], ref, scale))
        got1 = outs1[k].cpu().numpy()
        wd = min(width, w)
        for b in range(blocks):
            lo = (w - wd) * b // (blocks - 1)
            fl, w1 = alg1_check.compare(got1[lo:lo + wd], host[:, lo:lo + wd], ext1, sets1, beta1, f"chunk {k} block {b}")
            flips += fl
            sampled += wd
            worst1 = max(worst1, w1)
        say("oracle coordinate phase of chunk", k, round(time.time() - t0, 1), "s")
    assert flips <= max(2, sampled // 10_000)
    say(f"cfg 5 (d={d}): selected {ext.tolist()}, score gap {gap:.2e}, out worst err/tol {worst:.3g}; "
        f"alg1: worst err/tol {worst1:.3g}, ambiguous choices {flips} of {sampled}")


def test_more_than_2_to_the_31_coordinates():
    """d = 2^31 + 2^27 + 77 per row (n = 11, 100 GB): every index computation has to be 64-bit.  The oracle
    cannot take the whole matrix in reasonable time, so: the distance matrix equals the one accumulated
    over four chunks (each below 2^31 columns, the path the other tests pin), the extracted list is the
    oracle's for that matrix, and the output is compared with the oracle on blocks of columns sampled
    over the whole range, the last block ending at d."""
    n, f = 11, 2
    d = (1 << 31) + (1 << 27) + 77
    say("d > 2^31", n, f, d)
    # one round fewer than the default: in the last default round (one neighbour each) two gradients
    # that are each other's nearest tie exactly, which is fine but not what check_separation expects
    theta, beta = 6, 2
    Gt = torch.empty(n, d, device=DEV, dtype=torch.float32)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(1905)
    step = 1 << 27
    noise = 1.0 + 0.05 * torch.arange(n, device=DEV, dtype=torch.float32)[:, None]   # a noise ladder: scores apart
    for lo in range(0, d, step):                       # filled in slabs: no d-sized temporaries
        hi = min(d, lo + step)
        mu = torch.randn(1, hi - lo, generator=gen, device=DEV)
        Gt[:, lo:hi] = mu + noise * torch.randn(n, hi - lo, generator=gen, device=DEV)
    ws = torch.empty(mb.mbulyan_workspace_bytes(n, d), dtype=torch.uint8, device=DEV)
    out, sel = mb.mbulyan_aggregate_ex(Gt, f, theta=theta, beta=beta, workspace=ws)
    D = mb.pairwise_sqdist(Gt, workspace=ws).cpu().numpy()
    torch.cuda.synchronize()
    cuts = [0, d // 4, d // 2, 3 * (d // 4) + 5, d]
    Dc = None
    for a, b in zip(cuts[:-1], cuts[1:]):
        Dc = mb.pairwise_sqdist(Gt[:, a:b], dist=Dc, accumulate=Dc is not None, workspace=ws)
    Dc = Dc.cpu().numpy()
    assert np.all(np.abs(D - Dc) <= 1e-9 * np.maximum(D, 1.0)), float(np.max(np.abs(D - Dc) / np.maximum(D, 1.0)))
    ext, _, _ = O.multikrum_select(D, f, theta)
    check_separation(D, f, theta, ext)
    assert sel.cpu().numpy().tolist() == ext.tolist()
    width = 1 << 20
    worst = 0.0
    for b in range(33):
        lo = (d - width) * b // 32
        G = Gt[:, lo:lo + width].cpu().numpy()
        ref, scale = O.coordwise_selected(np.ascontiguousarray(G), ext, beta, want_scale=True)
        worst = max(worst, check_chunk(out[lo:lo + width].cpu().numpy(), ref, scale))
    say(f"d = {d}: selected {ext.tolist()}, out worst err/tol {worst:.3g} on 33 blocks of 2^20 columns")
