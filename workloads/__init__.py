"""Seeded synthetic worker gradients (inputs only; none of the method's arithmetic).

The five workloads stand in for the paper's: n = 4f+3 workers, d from 1e5 to
1e9 coordinates, n-f "correct" gradients = a shared mean plus per-worker
noise, f Byzantine gradients following one attack each.  Both the GPU
library and the CPU oracle are fed from here, so that they see the same bits.

Columns are produced in fixed blocks of BLOCK coordinates, each block from
its own seed, so a matrix can be generated whole, in column chunks, or one
block at a time and always holds the same values for a given device type.

Correct worker w (w = 0..n-f-1) has noise sigma * (1 + LADDER * w): with equal
noise the Krum scores of the correct workers concentrate as d grows and their
order would be decided by rounding; the ladder keeps them apart.
"""
from __future__ import annotations

import torch

BLOCK = 1 << 20
LADDER = 0.02
BASE_SEED = 190504374

# n, f, d, number of column chunks the workload is processed in, noise sigma
CONFIGS = {
    1: dict(n=11, f=2, d=100_000, chunks=1, sigma=0.1),
    2: dict(n=19, f=4, d=1_000_000, chunks=1, sigma=0.5),
    3: dict(n=27, f=6, d=25_000_000, chunks=1, sigma=1.0),
    4: dict(n=39, f=9, d=250_000_000, chunks=1, sigma=0.3),
    5: dict(n=51, f=12, d=1_000_000_000, chunks=4, sigma=0.1),
}


def spec(cfg: int) -> dict:
    return dict(CONFIGS[cfg])


def row_order(cfg: int, placement: str = "tail", seed: int | None = None) -> torch.Tensor:
    """Row index of every logical worker: logical rows 0..n-f-1 are correct, the
    last f Byzantine.  'tail' keeps that order, 'random' shuffles it (seeded)."""
    n = CONFIGS[cfg]["n"]
    if placement == "tail":
        return torch.arange(n)
    g = torch.Generator().manual_seed((BASE_SEED if seed is None else seed) + 7919 * cfg)
    return torch.randperm(n, generator=g)


def _block(cfg: int, blk: int, device, seed: int) -> torch.Tensor:
    """The (n, BLOCK) block number blk of workload cfg, logical row order."""
    c = CONFIGS[cfg]
    n, f, sigma = c["n"], c["f"], c["sigma"]
    nc = n - f
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1_000_003 + cfg * 10_007 + blk)

    def randn(*shape):
        return torch.randn(*shape, generator=g, device=device, dtype=torch.float32)

    if cfg == 4:  # heavy-tailed mean: Student-t with 3 degrees of freedom
        z = randn(BLOCK)
        chi = randn(3, BLOCK).square_().sum(0).div_(3.0).sqrt_()
        mu = z / chi
    else:
        mu = randn(BLOCK)
    out = torch.empty(n, BLOCK, device=device, dtype=torch.float32)
    ladder = sigma * (1.0 + LADDER * torch.arange(nc, device=device, dtype=torch.float32))
    out[:nc] = randn(nc, BLOCK)
    out[:nc].mul_(ladder[:, None]).add_(mu[None, :])
    if cfg == 1:      # identical copies of -10 mu
        out[nc:] = (-10.0 * mu)[None, :]
    elif cfg == 2:    # large-norm noise, independent per row and coordinate
        out[nc:] = randn(f, BLOCK).mul_(100.0)
    elif cfg == 3:    # identical copies of mu - 1.5 std(correct), per coordinate
        out[nc:] = (mu - 1.5 * out[:nc].std(dim=0))[None, :]
    elif cfg == 4:    # identical copies of -4 mean(correct)
        out[nc:] = (-4.0 * out[:nc].mean(dim=0))[None, :]
    elif cfg == 5:    # half identical copies of -10 mu, half large-norm noise
        h = f // 2
        out[nc:nc + h] = (-10.0 * mu)[None, :]
        out[nc + h:] = randn(f - h, BLOCK).mul_(50.0)
    else:
        raise KeyError(cfg)
    return out


def fill(cfg: int, out: torch.Tensor, col0: int = 0, placement: str = "tail",
         seed: int | None = None) -> torch.Tensor:
    """Write columns [col0, col0 + out.shape[1]) of workload cfg into out (n, w)."""
    seed = BASE_SEED if seed is None else seed
    n = CONFIGS[cfg]["n"]
    assert out.shape[0] == n and out.dtype == torch.float32
    order = row_order(cfg, placement, seed).to(out.device)
    w = out.shape[1]
    c = col0
    while c < col0 + w:
        blk, off = divmod(c, BLOCK)
        take = min(BLOCK - off, col0 + w - c)
        b = _block(cfg, blk, out.device, seed)
        out[order, c - col0:c - col0 + take] = b[:, off:off + take]
        c += take
    return out


def make(cfg: int, device="cpu", d: int | None = None, col0: int = 0,
         placement: str = "tail", seed: int | None = None) -> torch.Tensor:
    """The first d columns from col0 (default: all of them) of workload cfg as an (n, d) tensor."""
    c = CONFIGS[cfg]
    d = c["d"] if d is None else d
    out = torch.empty(c["n"], d, device=device, dtype=torch.float32)
    return fill(cfg, out, col0, placement, seed)


def offset(n: int, f: int, d: int, kappa: float, device="cpu", byzantine_first: bool = False,
           sigma: float = 0.05, seed: int = 0) -> torch.Tensor:
    """Gradients that share a large common component, the regime the paper's convergence argument
    assumes (Lemma 1: the gradient dominates its noise): correct worker w = g + N(0, (sigma (1 +
    LADDER w))^2) with |g|^2 / d = (2 kappa - 1) sigma^2, so that squared norm : squared distance
    between two correct workers is about kappa : 1.  The f Byzantine rows: the first half identical
    copies of -2 g, the rest g + N(0, (20 sigma)^2) each.  They come last, or first when
    byzantine_first is set (row 0 is then a Byzantine one)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(BASE_SEED * 7 + 1009 * n + 31 * int(kappa) + seed)
    nc = n - f

    def randn(*shape):
        return torch.randn(*shape, generator=gen, device=device, dtype=torch.float32)

    out = torch.empty(n, d, device=device, dtype=torch.float32)
    gamma = sigma * (2.0 * kappa - 1.0) ** 0.5
    lo = 0
    while lo < d:                                   # in blocks: no n x d temporaries on top of the result
        w = min(BLOCK, d - lo)
        g = randn(w).mul_(gamma)
        blk = torch.empty(n, w, device=device, dtype=torch.float32)
        ladder = sigma * (1.0 + LADDER * torch.arange(nc, device=device, dtype=torch.float32))
        blk[:nc] = randn(nc, w).mul_(ladder[:, None]).add_(g[None, :])
        h = f // 2
        blk[nc:nc + h] = (-2.0 * g)[None, :]
        blk[nc + h:] = randn(f - h, w).mul_(20.0 * sigma).add_(g[None, :])
        if byzantine_first:
            blk = torch.cat([blk[nc:], blk[:nc]], dim=0)
        out[:, lo:lo + w] = blk
        lo += w
    return out


def uniform(n: int, d: int, device="cpu", seed: int = 0) -> torch.Tensor:
    """n gradients drawn independently from U(0,1)^d: the input of the paper's
    aggregation-time benchmark (Section V-A)."""
    g = torch.Generator(device=device)
    g.manual_seed(BASE_SEED + 31 * n + seed)
    return torch.rand(n, d, generator=g, device=device, dtype=torch.float32)
