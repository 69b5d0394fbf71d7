"""Many small seeded cases end to end: n, f, d, the kind of Byzantine rows, their placement, the reading of
Algorithm 1 and the storage format all drawn at random (fixed seeds), each compared with the oracle.

The inputs follow the recipe of the five workloads (correct worker w = shared mean + noise of standard
deviation sigma (1 + 0.03 w), so that the Krum scores of correct workers are separated), with Byzantine
rows of five kinds, copies among them.  Per case: the extracted list must be the oracle's wherever every
decision of the oracle is clearer than what the distance pass may be off by (else it must be valid on the
oracle's distances within that: 256 max(1e-7, 1e-5 / sqrt(d)) of a distance, the bound of a pair the first pass
is trusted on),
and the output must be the oracle's for the extracted list (the bars of tests/test_gpu_parity.py).
"""
import numpy as np
import pytest
import torch

import alg1_check
import oracle as O
import paper_1905_04374_amd as mb
from progress import say
from selection_check import replay

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
KINDS = ("copies of -3 mean", "large noise", "copies of a correct row", "near the mean", "mixed")


def make_case(rng):
    n = int(rng.choice([3, 4, 5, 7, 8, 11, 13, 16, 17, 19, 23, 27, 31, 32, 33, 39, 47, 48, 49, 51, 57, 64]))
    f = int(rng.integers(0, (n - 3) // 4 + 1))
    d = int(rng.choice([1, 2, 3, 7, 31, 128, 129, 255, 512, 1000, 1023, 2048, 4097, 10_000, 33_333, 70_001]))
    kind = KINDS[int(rng.integers(len(KINDS)))]
    sigma = float(rng.choice([0.05, 0.3, 1.0]))
    mu = rng.standard_normal(d).astype(np.float32)
    G = np.empty((n, d), np.float32)
    for w in range(n - f):
        G[w] = mu + (sigma * (1 + 0.03 * w)) * rng.standard_normal(d).astype(np.float32)
    mean = G[: n - f].mean(0)
    for b in range(f):
        k = kind if kind != "mixed" else KINDS[b % 4]
        if k == "copies of -3 mean":
            G[n - f + b] = -3 * mean
        elif k == "large noise":
            G[n - f + b] = 50 * rng.standard_normal(d).astype(np.float32)
        elif k == "copies of a correct row":
            G[n - f + b] = G[0]
        else:
            G[n - f + b] = mean + 0.01 * sigma * rng.standard_normal(d).astype(np.float32)
    if rng.random() < 0.5:
        G = G[rng.permutation(n)]
    return n, f, d, kind, np.ascontiguousarray(G)


@pytest.mark.parametrize("block", range(6))
def test_random_cases_end_to_end(block):
    rng = np.random.default_rng(4242 + block)
    clear_cases = 0
    for case in range(30):
        n, f, d, kind, G = make_case(rng)
        mode = (mb.MODE_SELECTED, mb.MODE_ALG1)[int(rng.integers(2))]
        omode = O.MODE_SELECTED if mode == mb.MODE_SELECTED else O.MODE_ALG1
        theta, beta = O.params(n, f, omode)
        if theta < 1 or beta < 1:
            continue
        storage = ("f32", "bf16", "fp16")[int(rng.integers(3))]
        Gt = torch.as_tensor(G).to(DEV)
        if storage != "f32":
            Gt = Gt.to(torch.bfloat16 if storage == "bf16" else torch.float16)
            G = Gt.float().cpu().numpy()              # the matrix the library sees
        say("random case", block, case, n, f, d, kind, "alg1" if omode else "selected", storage)
        D = O.pairwise_sqdist(G)
        ext, sets, _ = O.multikrum_select(D, f, theta)
        out, sel = mb.mbulyan_aggregate_ex(Gt, f, mode=mode)
        sel = sel.cpu().numpy()
        out = out.cpu().numpy()
        if omode == O.MODE_ALG1:
            Dg = mb.pairwise_sqdist(Gt)
            sel2, sets_g, _ = mb.multikrum_select(Dg, f, theta)
            assert sel2.cpu().numpy().tolist() == sel.tolist()
            sets_g = sets_g.cpu().numpy()
        else:
            sets_g = None
        tau = 256 * max(1e-7, 1e-5 / np.sqrt(d))
        clear = replay(D, f, sel, sets_g, tau)        # the library's list is valid on the oracle's distances
        if clear > tau:
            clear_cases += 1
            assert sel.tolist() == ext.tolist(), (n, f, d, kind, storage)
            if sets_g is not None:
                assert np.array_equal(sets_g, sets)
        if omode == O.MODE_SELECTED:
            ref, scale = O.coordwise_selected(G, sel, beta, want_scale=True)
            err = np.abs(out.astype(np.float64) - ref)
            tol = 1e-5 * np.maximum(np.abs(ref), scale) + 1e-37
            assert np.all(err <= tol), (n, f, d, kind, storage, float(np.max(err / tol)))
        else:
            flips, _ = alg1_check.compare(out, G, sel, sets_g, beta, f"case {block}.{case}")
            assert flips <= max(4, d // 500)
    say(f"block {block}: {clear_cases} cases with every oracle decision clearer than the distance bound")
    assert clear_cases >= 10
