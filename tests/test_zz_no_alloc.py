"""mbulyan_aggregate_noalloc (the entry point for callers that cannot allocate: its workspace is a
static device array of the library) against mbulyan_aggregate_ex, through the raw C ABI.

Both run the same kernels, so the extracted list and the output must be bit-identical.  Two calls
in a row share the array, the second on a smaller input: nothing of the first call may leak into
the second.  Collected last on purpose (the file name), and it passes alone in a fresh process as
well as after the other tests.
"""
import ctypes as C
import sys

import pytest
import torch

import paper_1905_04374_amd as mb
from progress import say
import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"



def raw_noalloc(G, f, mode, out, sel):
    """The call as a C program would make it: plain pointers and sizes."""
    n, d = G.shape
    rc = mb.lib.mbulyan_aggregate_noalloc(C.c_void_p(G.data_ptr()), n, f, d, G.stride(0), mode,
                                          C.c_void_p(out.data_ptr()), C.c_void_p(sel.data_ptr()),
                                          C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == mb.MB_OK, mb.lib.mbulyan_strerror(rc)
    return out, sel


def buffers(G, f, mode):
    theta, _ = mb.mbulyan_params(G.shape[0], f, mode)
    return (torch.full((G.shape[1],), float("nan"), device=DEV),
            torch.full((theta,), -1, device=DEV, dtype=torch.int32))


def raw_ex(G, f, mode):
    n, d = G.shape
    theta, _ = mb.mbulyan_params(n, f, mode)
    ws = torch.empty(mb.mbulyan_workspace_bytes(n, d), dtype=torch.uint8, device=DEV)
    out = torch.empty(d, device=DEV)
    sel = torch.empty(theta, device=DEV, dtype=torch.int32)
    rc = mb.lib.mbulyan_aggregate_ex(C.c_void_p(G.data_ptr()), n, f, d, G.stride(0), mode, 0, 0,
                                     C.c_void_p(out.data_ptr()), C.c_void_p(sel.data_ptr()),
                                     C.c_void_p(ws.data_ptr()), ws.numel(),
                                     C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == mb.MB_OK, mb.lib.mbulyan_strerror(rc)
    torch.cuda.synchronize()
    return out, sel


@pytest.mark.parametrize("mode", [mb.MODE_SELECTED, mb.MODE_ALG1])
def test_noalloc_equals_aggregate_ex_twice_in_a_row(mode):
    # first a large call (n = 51: four row blocks, the most partial sums per workgroup; many tiles
    # per workgroup), then a smaller one (fewer rows, fewer workgroups) right behind it
    cases = [(5, 3_000_064), (2, 70_001), (1, 4096)]
    inputs = [(W.spec(cfg)["f"], W.make(cfg, DEV, d=d)) for cfg, d in cases]
    expect = [raw_ex(G, f, mode) for f, G in inputs]
    bufs = [buffers(G, f, mode) for f, G in inputs]
    # the first call on a device looks up the array's address (the runtime places the library's
    # device variables then): from the second call on nothing may be allocated
    raw_noalloc(inputs[-1][1], inputs[-1][0], mode, *buffers(inputs[-1][1], inputs[-1][0], mode))
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    for (cfg, d), (f, G), (out, sel) in zip(cases, inputs, bufs):
        say("noalloc", mode, cfg, d)
        raw_noalloc(G, f, mode, out, sel)            # back to back, no synchronisation in between
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert free_before - free_after < (1 << 20), "device memory was allocated during the calls"
    for (cfg, d), (out, sel), (ref, ref_sel) in zip(cases, bufs, expect):
        assert torch.equal(sel, ref_sel), (cfg, d, sel.tolist(), ref_sel.tolist())
        assert torch.equal(out, ref), (cfg, d)
    # and once more in the opposite order: small first, then large
    for (cfg, d), (f, G), (ref, ref_sel) in reversed(list(zip(cases, inputs, expect))):
        out, sel = raw_noalloc(G, f, mode, *buffers(G, f, mode))
        torch.cuda.synchronize()
        assert torch.equal(sel, ref_sel) and torch.equal(out, ref), (cfg, d)


def test_noalloc_rejects_what_it_cannot_hold_and_bad_arguments():
    one = C.c_void_p(256)   # never dereferenced: validation fails first
    lib = mb.lib
    assert lib.mbulyan_aggregate_noalloc(one, 65, 0, 100, 100, 0, one, None, None) == mb.MB_EUNSUPPORTED
    assert lib.mbulyan_aggregate_noalloc(one, 10, 2, 100, 100, 0, one, None, None) == mb.MB_EPRECOND
    assert lib.mbulyan_aggregate_noalloc(None, 11, 2, 100, 100, 0, one, None, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_noalloc(one, 11, 2, 100, 99, 0, one, None, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_noalloc(one, 11, 2, 100, 100, 0, None, None, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_noalloc(one, 11, 2, 100, 100, 5, one, None, None) == mb.MB_EINVAL


def test_noalloc_through_the_binding_with_a_strided_matrix():
    s = W.spec(3)
    wide = W.make(3, DEV, d=200_004)
    G = wide[:, 4:150_000]                            # ld > d
    ref, ref_sel = mb.mbulyan_aggregate_ex(G, s["f"])
    out = torch.empty(G.shape[1], device=DEV)
    sel = torch.empty(ref_sel.numel(), device=DEV, dtype=torch.int32)
    mb.mbulyan_aggregate_noalloc(G, s["f"], out, sel)
    torch.cuda.synchronize()
    assert torch.equal(sel, ref_sel) and torch.equal(out, ref)
