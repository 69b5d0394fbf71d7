"""ctypes binding of libmbulyan.so: argument marshalling only.

Every function has the name and meaning of the C entry point in
include/mbulyan.h; tensors are torch CUDA tensors (device memory), the stream
is torch's current stream unless given.  Nothing is computed here.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmbulyan.so")

MB_MAX_N = 64
MB_OK, MB_EINVAL, MB_EPRECOND, MB_EUNSUPPORTED, MB_EWORKSPACE, MB_EHIP = range(6)
MODE_SELECTED, MODE_ALG1 = 0, 1
DIST_AUTO, DIST_DIRECT, DIST_GRAM, DIST_GRAM_BF16 = 0, 1, 2, 3
STAGES = ("dist", "reduce", "select", "coord", "refine")

EXPORTS = [
    "mbulyan_strerror", "mbulyan_last_hip_error", "mbulyan_version", "mbulyan_params",
    "mbulyan_workspace_bytes", "mbulyan_set_dist_algo", "mbulyan_aggregate", "mbulyan_aggregate_ex",
    "mbulyan_aggregate_chunked", "pairwise_sqdist", "krum_scores", "multikrum_select",
    "coordwise_trimmed_avg", "multikrum_aggregate", "coordwise_median", "mbulyan_timing_enable",
    "mbulyan_timing_reset", "mbulyan_timing_read", "mbulyan_release",
    "pairwise_sqdist_bf16", "coordwise_trimmed_avg_bf16", "mbulyan_aggregate_bf16",
    "mbulyan_aggregate_chunked_bf16", "multikrum_aggregate_bf16", "coordwise_median_bf16",
    "mbulyan_aggregate_noalloc",
    "pairwise_sqdist_fp16", "coordwise_trimmed_avg_fp16", "mbulyan_aggregate_fp16",
    "mbulyan_aggregate_chunked_fp16", "multikrum_aggregate_fp16", "coordwise_median_fp16",
    "mbulyan_aggregate_host", "mbulyan_host_resident_limit",
]


class MBulyanError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"mbulyan status {status}: {message}")
        self.status = status


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python paper_1905_04374_amd/build.py` "
            "(there is no fallback implementation)")
    lib = C.CDLL(LIB_PATH)
    vp, i64, sz = C.c_void_p, C.c_int64, C.c_size_t
    ci = C.c_int
    lib.mbulyan_strerror.restype = C.c_char_p
    lib.mbulyan_strerror.argtypes = [ci]
    lib.mbulyan_version.restype = C.c_char_p
    lib.mbulyan_params.argtypes = [ci, ci, ci, C.POINTER(ci), C.POINTER(ci)]
    lib.mbulyan_workspace_bytes.argtypes = [ci, i64, C.POINTER(sz)]
    lib.mbulyan_set_dist_algo.argtypes = [ci]
    lib.mbulyan_aggregate.argtypes = [vp, ci, ci, i64, vp, vp, vp]
    lib.mbulyan_aggregate_ex.argtypes = [vp, ci, ci, i64, i64, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.mbulyan_aggregate_host.argtypes = [vp, ci, ci, ci, i64, i64, ci, i64, vp, vp, vp]
    lib.mbulyan_host_resident_limit.argtypes = [C.c_longlong]
    lib.mbulyan_aggregate_noalloc.argtypes = [vp, ci, ci, i64, i64, ci, vp, vp, vp]
    lib.mbulyan_aggregate_chunked.argtypes = [C.POINTER(vp), ci, C.POINTER(i64), C.POINTER(i64), ci, ci, ci,
                                              C.POINTER(vp), vp, vp, sz, vp]
    lib.pairwise_sqdist.argtypes = [vp, ci, i64, i64, vp, ci, ci, vp, sz, vp]
    lib.krum_scores.argtypes = [vp, ci, ci, vp, vp, vp]
    lib.multikrum_select.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp]
    lib.coordwise_trimmed_avg.argtypes = [vp, ci, i64, i64, vp, ci, ci, vp, vp, vp]
    lib.multikrum_aggregate.argtypes = [vp, ci, ci, i64, i64, vp, vp, vp, sz, vp]
    lib.coordwise_median.argtypes = [vp, ci, i64, i64, vp, vp]
    for sfx in ("bf16", "fp16"):
        getattr(lib, "pairwise_sqdist_" + sfx).argtypes = [vp, ci, i64, i64, vp, ci, vp, sz, vp]
        getattr(lib, "coordwise_trimmed_avg_" + sfx).argtypes = [vp, ci, i64, i64, vp, ci, ci, vp, vp, vp]
        getattr(lib, "mbulyan_aggregate_" + sfx).argtypes = [vp, ci, ci, i64, i64, ci, ci, ci, vp, vp, vp, sz, vp]
        getattr(lib, "mbulyan_aggregate_chunked_" + sfx).argtypes = [C.POINTER(vp), ci, C.POINTER(i64), C.POINTER(i64),
                                                                     ci, ci, ci, C.POINTER(vp), vp, vp, sz, vp]
        getattr(lib, "multikrum_aggregate_" + sfx).argtypes = [vp, ci, ci, i64, i64, vp, vp, vp, sz, vp]
        getattr(lib, "coordwise_median_" + sfx).argtypes = [vp, ci, i64, i64, vp, vp]
    lib.mbulyan_timing_enable.argtypes = [ci]
    lib.mbulyan_timing_read.argtypes = [C.POINTER(C.c_double), C.POINTER(i64)]
    return lib


lib = _load()


def _check(status: int):
    if status != MB_OK:
        msg = lib.mbulyan_strerror(status).decode()
        if status == MB_EHIP:
            msg += f" (hipError {lib.mbulyan_last_hip_error()})"
        raise MBulyanError(status, msg)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t: torch.Tensor | None, dtype, name: str, numel: int | None = None, like: torch.Tensor | None = None) -> int | None:
    """Pointer of a dense CUDA tensor of the given dtype.  The C ABI sees no sizes, so this is the
    only place that can refuse a buffer that is too short (numel), strided, or on another device than
    the gradients (like): the kernels would write past its end."""
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype:
        raise TypeError(f"{name} must be a CUDA tensor of dtype {dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name} holds {t.numel()} elements, {numel} are needed")
    if like is not None and t.device != like.device:
        raise ValueError(f"{name} is on {t.device}, the gradients on {like.device}")
    return t.data_ptr()


_SUFFIX = {torch.bfloat16: "bf16", torch.float16: "fp16"}


def _entry(name: str, grads: torch.Tensor):
    """The entry point for the storage format of grads: `name` itself for float32, its _bf16 / _fp16 form else."""
    sfx = _SUFFIX.get(grads.dtype)
    return getattr(lib, name + "_" + sfx) if sfx else getattr(lib, name)


def _matrix(grads: torch.Tensor, bf16_ok: bool = False):
    """(pointer, n, d, ld) of an (n, d) float32 CUDA tensor with unit column stride (bfloat16 or float16 where
    the entry point has 16-bit forms; ld is in elements)."""
    ok = (torch.float32, torch.bfloat16, torch.float16) if bf16_ok else (torch.float32,)
    if not grads.is_cuda or grads.dtype not in ok or grads.dim() != 2:
        raise TypeError("grads must be a 2-D CUDA tensor of " + " or ".join(str(t) for t in ok))
    n, d = grads.shape
    if d > 1 and grads.stride(1) != 1:
        raise ValueError("grads must have unit stride along the coordinates")
    ld = grads.stride(0) if n > 1 else max(d, 1)
    return grads.data_ptr(), n, d, ld


def version() -> str:
    return lib.mbulyan_version().decode()


def mbulyan_params(n: int, f: int, mode: int = MODE_SELECTED):
    th, be = C.c_int(), C.c_int()
    _check(lib.mbulyan_params(n, f, mode, C.byref(th), C.byref(be)))
    return th.value, be.value


def mbulyan_workspace_bytes(n: int, d: int) -> int:
    b = C.c_size_t()
    _check(lib.mbulyan_workspace_bytes(n, d, C.byref(b)))
    return b.value


def mbulyan_set_dist_algo(algo: int):
    _check(lib.mbulyan_set_dist_algo(algo))


def _ws(workspace):
    if workspace is None:
        return None, 0
    if not workspace.is_cuda or workspace.dtype != torch.uint8:
        raise TypeError("workspace must be a uint8 CUDA tensor")
    return workspace.data_ptr(), workspace.numel()


def mbulyan_aggregate(grads, f, out=None, selected_idx=None, stream=None):
    """GAR(f, grads) in MB_MODE_SELECTED with the library's workspace.  Returns (out, selected_idx)."""
    p, n, d, ld = _matrix(grads)
    if ld != d:
        raise ValueError("mbulyan_aggregate needs a dense matrix (ld == d); use mbulyan_aggregate_ex")
    theta, _ = mbulyan_params(n, f, MODE_SELECTED)
    if out is None:
        out = torch.empty(d, device=grads.device, dtype=torch.float32)
    if selected_idx is None:
        selected_idx = torch.empty(theta, device=grads.device, dtype=torch.int32)
    _check(lib.mbulyan_aggregate(p, n, f, d, _dev(out, torch.float32, "out", d, grads),
                                 _dev(selected_idx, torch.int32, "selected_idx", theta, grads), _stream(stream)))
    return out, selected_idx


def mbulyan_aggregate_ex(grads, f, mode=MODE_SELECTED, theta=0, beta=0, out=None, selected_idx=None,
                         workspace=None, stream=None):
    """grads may be bfloat16 or float16: the entry point for that storage runs, out stays float32."""
    p, n, d, ld = _matrix(grads, bf16_ok=True)
    th_def, _ = mbulyan_params(n, f, mode)
    th = theta or th_def
    if out is None:
        out = torch.empty(d, device=grads.device, dtype=torch.float32)
    if selected_idx is None:
        selected_idx = torch.empty(th, device=grads.device, dtype=torch.int32)
    wp, wb = _ws(workspace)
    if grads.dtype != torch.float32:
        _check(_entry("mbulyan_aggregate", grads)(p, n, f, d, ld, mode, theta, beta,
                                                  _dev(out, torch.float32, "out", d, grads),
                                                  _dev(selected_idx, torch.int32, "selected_idx", th, grads), wp, wb,
                                                  _stream(stream)))
        return out, selected_idx
    _check(lib.mbulyan_aggregate_ex(p, n, f, d, ld, mode, theta, beta, _dev(out, torch.float32, "out", d, grads),
                                    _dev(selected_idx, torch.int32, "selected_idx", th, grads), wp, wb, _stream(stream)))
    return out, selected_idx


def mbulyan_aggregate_noalloc(grads, f, out, selected_idx=None, mode=MODE_SELECTED, stream=None):
    """mbulyan_aggregate_ex on the library's static device array: the call allocates nothing, so the
    caller passes `out` (and `selected_idx`, if wanted).  Returns (out, selected_idx)."""
    p, n, d, ld = _matrix(grads)
    theta, _ = mbulyan_params(n, f, mode)
    _check(lib.mbulyan_aggregate_noalloc(p, n, f, d, ld, mode, _dev(out, torch.float32, "out", d, grads),
                                         _dev(selected_idx, torch.int32, "selected_idx", theta, grads),
                                         _stream(stream)))
    return out, selected_idx


def mbulyan_host_resident_limit(nbytes: int):
    """Host matrices up to this many bytes are uploaded once by mbulyan_aggregate_host (0: never; negative: the
    default, three quarters of the free device memory)."""
    _check(lib.mbulyan_host_resident_limit(int(nbytes)))


def mbulyan_aggregate_host(host_grads, f, chunk_d, mode=MODE_SELECTED, host_out=None, stream=None):
    """GAR(f, host_grads) for an (n, d) HOST tensor (float32, bfloat16 or float16; pinned memory lets the
    uploads overlap the kernels): uploaded in column chunks of chunk_d coordinates, twice.  Blocks until the
    result is in host_out.  Returns (host_out, selected_idx), both host tensors."""
    if host_grads.is_cuda or host_grads.dim() != 2 or host_grads.dtype not in (torch.float32, torch.bfloat16, torch.float16):
        raise TypeError("host_grads must be a 2-D host tensor of float32, bfloat16 or float16")
    n, d = host_grads.shape
    if d > 1 and host_grads.stride(1) != 1:
        raise ValueError("host_grads must have unit stride along the coordinates")
    ld = host_grads.stride(0) if n > 1 else max(d, 1)
    storage = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}[host_grads.dtype]
    theta, _ = mbulyan_params(n, f, mode)
    if host_out is None:
        host_out = torch.empty(d, dtype=torch.float32, pin_memory=host_grads.is_pinned())
    if host_out.is_cuda or host_out.dtype != torch.float32 or not host_out.is_contiguous() or host_out.numel() < d:
        raise ValueError("host_out must be a contiguous host float32 tensor of d elements")
    sel = torch.empty(theta, dtype=torch.int32)
    _check(lib.mbulyan_aggregate_host(host_grads.data_ptr(), storage, n, f, d, ld, mode, int(chunk_d),
                                      host_out.data_ptr(), sel.data_ptr(), _stream(stream)))
    return host_out, sel


def mbulyan_aggregate_chunked(chunks, f, mode=MODE_SELECTED, outs=None, selected_idx=None, workspace=None,
                              stream=None):
    """chunks: list of (n, d_c) float32 CUDA tensors, the column chunks of one matrix (all bfloat16
    or all float16 instead: the entry point for that storage)."""
    k = len(chunks)
    mats = [_matrix(c, bf16_ok=True) for c in chunks]
    in16 = chunks[0].dtype != torch.float32
    if any(c.dtype != chunks[0].dtype for c in chunks):
        raise TypeError("all chunks must have the same dtype")
    n = mats[0][1]
    if any(m[1] != n for m in mats):
        raise ValueError("all chunks must have the same number of rows")
    theta, _ = mbulyan_params(n, f, mode)
    if outs is None:
        outs = [torch.empty(m[2], device=chunks[0].device, dtype=torch.float32) for m in mats]
    if selected_idx is None:
        selected_idx = torch.empty(theta, device=chunks[0].device, dtype=torch.int32)
    cp = (C.c_void_p * k)(*[m[0] for m in mats])
    cd = (C.c_int64 * k)(*[m[2] for m in mats])
    cl = (C.c_int64 * k)(*[m[3] for m in mats])
    op = (C.c_void_p * k)(*[_dev(o, torch.float32, "out", m[2], chunks[0]) for o, m in zip(outs, mats)])
    wp, wb = _ws(workspace)
    if in16:
        _check(_entry("mbulyan_aggregate_chunked", chunks[0])(cp, k, cd, cl, n, f, mode, op,
                                                  _dev(selected_idx, torch.int32, "selected_idx", theta, chunks[0]),
                                                  wp, wb, _stream(stream)))
        return outs, selected_idx
    _check(lib.mbulyan_aggregate_chunked(cp, k, cd, cl, n, f, mode, op,
                                         _dev(selected_idx, torch.int32, "selected_idx", theta, chunks[0]), wp, wb,
                                         _stream(stream)))
    return outs, selected_idx


def pairwise_sqdist(grads, dist=None, accumulate=False, algo=DIST_AUTO, workspace=None, stream=None):
    """grads may be bfloat16 or float16: the entry point for that storage runs (Gram form, algo is not used)."""
    p, n, d, ld = _matrix(grads, bf16_ok=True)
    if dist is None:
        if accumulate:
            raise ValueError("accumulate needs an existing dist")
        dist = torch.empty(n, n, device=grads.device, dtype=torch.float64)
    wp, wb = _ws(workspace)
    if grads.dtype != torch.float32:
        _check(_entry("pairwise_sqdist", grads)(p, n, d, ld, _dev(dist, torch.float64, "dist", n * n, grads),
                                                int(accumulate), wp, wb, _stream(stream)))
        return dist
    _check(lib.pairwise_sqdist(p, n, d, ld, _dev(dist, torch.float64, "dist", n * n, grads), int(accumulate), algo,
                               wp, wb, _stream(stream)))
    return dist


def krum_scores(dist, f, active=None, scores=None, stream=None):
    n = dist.shape[0]
    if scores is None:
        scores = torch.empty(n, device=dist.device, dtype=torch.float64)
    _check(lib.krum_scores(_dev(dist, torch.float64, "dist", n * n), n, f, _dev(active, torch.uint8, "active", n, dist),
                           _dev(scores, torch.float64, "scores", n, dist), _stream(stream)))
    return scores


def multikrum_select(dist, f, theta, want_sets=True, stream=None):
    n = dist.shape[0]
    sel = torch.empty(max(theta, 0), device=dist.device, dtype=torch.int32)
    sets = torch.empty(max(theta, 0), n, device=dist.device, dtype=torch.uint8) if want_sets else None
    m = torch.empty(max(theta, 0), device=dist.device, dtype=torch.int32) if want_sets else None
    _check(lib.multikrum_select(_dev(dist, torch.float64, "dist", n * n), n, f, theta, _dev(sel, torch.int32, "sel"),
                                _dev(sets, torch.uint8, "agr_sets"), _dev(m, torch.int32, "m_out"),
                                _stream(stream)))
    return sel, sets, m


def coordwise_trimmed_avg(grads, selected_idx, beta, agr_sets=None, out=None, stream=None):
    """grads may be bfloat16 or float16."""
    p, n, d, ld = _matrix(grads, bf16_ok=True)
    if out is None:
        out = torch.empty(d, device=grads.device, dtype=torch.float32)
    theta = selected_idx.numel()
    sp = _dev(selected_idx, torch.int32, "selected_idx", None, grads)
    ap = _dev(agr_sets, torch.uint8, "agr_sets", theta * n, grads)
    fn = _entry("coordwise_trimmed_avg", grads)
    _check(fn(p, n, d, ld, sp, theta, beta, ap, _dev(out, torch.float32, "out", d, grads), _stream(stream)))
    return out


def multikrum_aggregate(grads, f, out=None, selected_mask=None, workspace=None, stream=None):
    """grads may be bfloat16 or float16."""
    p, n, d, ld = _matrix(grads, bf16_ok=True)
    if out is None:
        out = torch.empty(d, device=grads.device, dtype=torch.float32)
    if selected_mask is None:
        selected_mask = torch.empty(n, device=grads.device, dtype=torch.uint8)
    wp, wb = _ws(workspace)
    fn = _entry("multikrum_aggregate", grads)
    _check(fn(p, n, f, d, ld, _dev(out, torch.float32, "out", d, grads),
              _dev(selected_mask, torch.uint8, "selected_mask", n, grads), wp, wb, _stream(stream)))
    return out, selected_mask


def coordwise_median(grads, out=None, stream=None):
    """grads may be bfloat16 or float16."""
    p, n, d, ld = _matrix(grads, bf16_ok=True)
    if out is None:
        out = torch.empty(d, device=grads.device, dtype=torch.float32)
    fn = _entry("coordwise_median", grads)
    _check(fn(p, n, d, ld, _dev(out, torch.float32, "out", d, grads), _stream(stream)))
    return out


def mbulyan_timing_enable(on: bool, stages=None):
    """stages: names out of STAGES to time (each costs two event records per call); None: all of them."""
    mask = sum(1 << STAGES.index(s) for s in (STAGES if stages is None else stages)) if on else 0
    _check(lib.mbulyan_timing_enable(mask))


def mbulyan_timing_reset():
    _check(lib.mbulyan_timing_reset())


def mbulyan_timing_read():
    """{stage: (milliseconds, launches)} since the last reset (synchronises the recorded events)."""
    ms = (C.c_double * len(STAGES))()
    cnt = (C.c_int64 * len(STAGES))()
    _check(lib.mbulyan_timing_read(ms, cnt))
    return {s: (ms[i], cnt[i]) for i, s in enumerate(STAGES)}


def mbulyan_release():
    _check(lib.mbulyan_release())
