"""The synthetic workloads: shapes, determinism, structure, and the score separation
that makes the extracted index list well defined (checked with the oracle)."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as W


def separation(G, f, theta):
    """Smallest relative gap, over all rounds, between the winner's score and the
    runner-up's, ignoring exact ties between bit-identical rows."""
    D = O.pairwise_sqdist(G)
    ext, sets, m, log = O.multikrum_select(D, f, theta, want_scores=True)
    worst = np.inf
    for t in range(theta):
        S = log[t]
        w = ext[t]
        for j in np.flatnonzero(np.isfinite(S)):
            if j == w:
                continue
            if D[w, j] == 0.0:           # bit-identical rows tie exactly; index order decides
                continue
            gap = (S[j] - S[w]) / max(S[j], 1e-300)
            worst = min(worst, gap)
    return worst, ext


@pytest.mark.parametrize("cfg,d", [(1, None), (2, None), (3, 1 << 21), (4, 1 << 21), (5, 1 << 21)])
def test_workload_structure_and_separation(cfg, d):
    s = W.spec(cfg)
    n, f = s["n"], s["f"]
    assert n == 4 * f + 3
    G = W.make(cfg, "cpu", d=d).numpy()
    assert G.shape == (n, d or s["d"]) and G.dtype == np.float32 and np.isfinite(G).all()
    theta, beta = O.params(n, f)
    gap, ext = separation(G, f, theta)
    assert gap > 1e-3, f"config {cfg}: scores separated by only {gap:.2e}"
    # the correct workers (rows 0..n-f-1) win the first n-2f-2 rounds in every workload
    assert np.all(ext[:n - 2 * f - 2 - (6 if cfg == 3 else 0)] < n - f)


def test_workload_chunks_and_determinism():
    a = W.make(5, "cpu", d=W.BLOCK + 1000)
    b = torch.empty_like(a)
    W.fill(5, b[:, :777], 0)
    W.fill(5, b[:, 777:W.BLOCK + 5], 777)
    W.fill(5, b[:, W.BLOCK + 5:], W.BLOCK + 5)
    assert torch.equal(a, b)
    assert not torch.equal(a, W.make(5, "cpu", d=W.BLOCK + 1000, seed=1))


def test_workload_random_placement_permutes_rows():
    a = W.make(1, "cpu", d=5000)
    b = W.make(1, "cpu", d=5000, placement="random")
    order = W.row_order(1, "random")
    assert torch.equal(b[order], a)
    assert sorted(order.tolist()) == list(range(11)) and order.tolist() != list(range(11))


def test_identical_byzantine_copies():
    for cfg, rows in [(1, [9, 10]), (3, list(range(21, 27))), (4, list(range(30, 39))), (5, list(range(39, 45)))]:
        G = W.make(cfg, "cpu", d=4096)
        for r in rows[1:]:
            assert torch.equal(G[r], G[rows[0]])
