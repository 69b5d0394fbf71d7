"""mbulyan_aggregate_host: gradients that stay in host memory, uploaded in column chunks (the upload of one
chunk overlapping the kernels of the one before; once if the matrix fits the device, else in two sweeps).
The distances accumulate over the same chunk boundaries as in the chunked device-resident entry point and
the coordinate kernels are the same, so the extracted list and the output must be bit-identical to it;
and the whole is compared with the oracle."""
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



@pytest.fixture(autouse=True)
def default_limit_afterwards():
    yield
    mb.mbulyan_host_resident_limit(-1)


@pytest.mark.parametrize("uploads", ["once", "twice"])
@pytest.mark.parametrize("pinned", [True, False])
@pytest.mark.parametrize("mode", [mb.MODE_SELECTED, mb.MODE_ALG1])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
def test_host_resident_gradients(dtype, mode, pinned, uploads):
    """uploads: the matrix fits the device and is uploaded once (the default for this size), or the two-sweep
    path that a matrix beyond the device takes, forced by a limit of 0."""
    say("host chunks", dtype, mode, pinned, uploads)
    mb.mbulyan_host_resident_limit(-1 if uploads == "once" else 0)
    s = W.spec(3)
    n, f = s["n"], s["f"]
    d, chunk_d = 700_013, 160_000                     # 5 chunks, the last one short and oddly sized
    G = W.make(3, "cpu", d=d).to(dtype)
    host = torch.empty(n, d + 24, dtype=dtype, pin_memory=pinned)[:, 8:8 + d]     # ld > d
    host.copy_(G)
    out, sel = mb.mbulyan_aggregate_host(host, f, chunk_d, mode=mode)
    # the device-resident chunked call on the same boundaries
    cuts = list(range(0, d, chunk_d)) + [d]
    chunks = [G[:, a:b].contiguous().to(DEV) for a, b in zip(cuts[:-1], cuts[1:])]
    outs, sel_dev = mb.mbulyan_aggregate_chunked(chunks, f, mode=mode)
    torch.cuda.synchronize()
    assert torch.equal(sel, sel_dev.cpu())
    assert torch.equal(out, torch.cat(outs).cpu())
    # and the oracle
    Gf = G.float().numpy()
    omode = O.MODE_ALG1 if mode == mb.MODE_ALG1 else O.MODE_SELECTED
    theta, beta = O.params(n, f, omode)
    ext, sets, _ = O.multikrum_select(O.pairwise_sqdist(Gf), f, theta)
    assert sel.tolist() == ext.tolist()
    if omode == O.MODE_SELECTED:
        ref, scale = O.coordwise_selected(Gf, ext, beta, want_scale=True)
        err = np.abs(out.numpy().astype(np.float64) - ref)
        assert np.all(err <= 1e-5 * np.maximum(np.abs(ref), scale))
    else:
        flips, _ = alg1_check.compare(out.numpy(), Gf, ext, sets, beta, "host chunks")
        assert flips <= max(4, d // (10_000 if dtype == torch.float32 else 500))


def test_host_entry_point_checks_its_arguments():
    host = torch.zeros(11, 1000)
    out = torch.empty(1000)
    lib = mb.lib
    args = lambda **k: [k.get("g", host.data_ptr()), k.get("storage", 0), k.get("n", 11), k.get("f", 2), k.get("d", 1000),
                        k.get("ld", 1000), k.get("mode", 0), k.get("chunk", 300), k.get("out", out.data_ptr()), None, None]
    assert lib.mbulyan_aggregate_host(*args(g=None)) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_host(*args(out=None)) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_host(*args(storage=3)) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_host(*args(ld=999)) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_host(*args(chunk=0)) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_host(*args(n=10)) == mb.MB_EPRECOND
    assert lib.mbulyan_aggregate_host(*args(n=65, f=0)) == mb.MB_EUNSUPPORTED
    assert lib.mbulyan_aggregate_host(*args(mode=4)) == mb.MB_EINVAL
