"""ctypes front end of the C oracle (test infrastructure only).

Arrays are numpy, host memory.  G is float32 of shape (n, d); a row stride
larger than d is allowed (pass a column slice of a wider C-contiguous array).
Each function cites the passage of the paper (arxiv 1905.04374) that its C
counterpart follows.
"""
import ctypes as C

import numpy as np

from .build import ensure_built

MODE_SELECTED = 0
MODE_ALG1 = 1
OK, EINVAL, EPRECOND = 0, -1, -2

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(ensure_built())
        f32p, f64p = C.POINTER(C.c_float), C.POINTER(C.c_double)
        i32p, u8p = C.POINTER(C.c_int32), C.POINTER(C.c_uint8)
        i64 = C.c_int64
        lib.orc_params.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
        lib.orc_pairwise_sqdist.argtypes = [f32p, C.c_int, i64, i64, f64p, C.c_int, C.c_int]
        lib.orc_pairwise_sqdist.restype = None
        lib.orc_krum_scores.argtypes = [f64p, C.c_int, C.c_int, u8p, f64p]
        lib.orc_krum_scores.restype = None
        lib.orc_multikrum_select.argtypes = [f64p, C.c_int, C.c_int, C.c_int, i32p, u8p, i32p, f64p]
        lib.orc_coordwise_selected.argtypes = [f32p, i64, i64, i32p, C.c_int, C.c_int, f32p, f32p, C.c_int]
        lib.orc_coordwise_selected.restype = None
        lib.orc_coordwise_alg1.argtypes = [f32p, C.c_int, i64, i64, i32p, u8p, C.c_int, C.c_int,
                                           f32p, f32p, f32p, f32p, C.c_int]
        lib.orc_coordwise_alg1.restype = None
        lib.orc_multikrum_aggregate.argtypes = [f32p, C.c_int, C.c_int, i64, i64, f32p, u8p, C.c_int]
        lib.orc_coordwise_median.argtypes = [f32p, C.c_int, i64, i64, f32p, C.c_int]
        lib.orc_coordwise_median.restype = None
        lib.orc_mbulyan.argtypes = [f32p, C.c_int, C.c_int, i64, i64, C.c_int, f32p, i32p, C.c_int]
        lib.orc_last_threads.restype = C.c_int
        _lib = lib
    return _lib


def _ptr(a, ty):
    return None if a is None else a.ctypes.data_as(C.POINTER(ty))


def _grads(G):
    """(array kept alive, n, d, ld) of a float32 (n, d) array with unit column stride."""
    G = np.asarray(G)
    if G.dtype != np.float32 or G.ndim != 2:
        raise TypeError("G must be a float32 array of shape (n, d)")
    if G.shape[1] > 1 and G.strides[1] != 4:
        G = np.ascontiguousarray(G)
    n, d = G.shape
    ld = G.strides[0] // 4 if n > 1 else max(d, 1)
    if ld < d:
        G = np.ascontiguousarray(G)
        ld = d
    return G, n, d, ld


class PreconditionError(ValueError):
    """n < 4f+3 (multi-Bulyan) or n < 2f+3 (multi-Krum), Section II-B."""


def _check(rc):
    if rc == EPRECOND:
        raise PreconditionError("precondition on (n, f) violated")
    if rc != OK:
        raise ValueError("invalid argument")


def last_threads():
    return _load().orc_last_threads()


def params(n, f, mode=MODE_SELECTED):
    """(theta, beta) of multi-Bulyan; Algorithm 1 (ALG1) / Theorem 2 proof (SELECTED)."""
    th, be = C.c_int(), C.c_int()
    _check(_load().orc_params(n, f, mode, C.byref(th), C.byref(be)))
    return th.value, be.value


def pairwise_sqdist(G, D=None, nthreads=0):
    """n x n squared l2 distances (Algorithm 1, multi-Krum score line).  If D is
    given the chunk's distances are added to it (column chunks)."""
    G, n, d, ld = _grads(G)
    acc = 1
    if D is None:
        D = np.zeros((n, n), np.float64)
        acc = 0
    assert D.dtype == np.float64 and D.shape == (n, n) and D.flags.c_contiguous
    _load().orc_pairwise_sqdist(_ptr(G, C.c_float), n, d, ld, _ptr(D, C.c_double), acc, nthreads)
    return D


def krum_scores(D, f, active=None):
    """Krum score of every active gradient (Algorithm 1, multi-Krum; Eq. 4)."""
    D = np.ascontiguousarray(D, np.float64)
    n = D.shape[0]
    if active is not None:
        active = np.ascontiguousarray(active, np.uint8)
    S = np.empty(n, np.float64)
    _load().orc_krum_scores(_ptr(D, C.c_double), n, f, _ptr(active, C.c_uint8), _ptr(S, C.c_double))
    return S


def multikrum_select(D, f, theta, want_scores=False):
    """theta rounds of multi-Krum (Algorithm 1, multi-Bulyan loop).
    Returns (ext[theta], agr_sets[theta, n], m[theta]) (+ score_log[theta, n])."""
    D = np.ascontiguousarray(D, np.float64)
    n = D.shape[0]
    ext = np.empty(theta, np.int32)
    sets = np.zeros((theta, n), np.uint8)
    m = np.empty(theta, np.int32)
    log = np.empty((theta, n), np.float64) if want_scores else None
    _check(_load().orc_multikrum_select(_ptr(D, C.c_double), n, f, theta, _ptr(ext, C.c_int32),
                                        _ptr(sets, C.c_uint8), _ptr(m, C.c_int32), _ptr(log, C.c_double)))
    return (ext, sets, m, log) if want_scores else (ext, sets, m)


def coordwise_selected(G, ext, beta, want_scale=False, nthreads=0):
    """Median, beta closest, average over the extracted rows (Section II-B)."""
    G, n, d, ld = _grads(G)
    ext = np.ascontiguousarray(ext, np.int32)
    assert ext.min(initial=0) >= 0 and ext.max(initial=0) < n
    out = np.empty(d, np.float32)
    scale = np.empty(d, np.float32) if want_scale else None
    _load().orc_coordwise_selected(_ptr(G, C.c_float), d, ld, _ptr(ext, C.c_int32), len(ext), beta,
                                   _ptr(out, C.c_float), _ptr(scale, C.c_float), nthreads)
    return (out, scale) if want_scale else out


def coordwise_alg1(G, ext, agr_sets, beta, want_extra=False, nthreads=0):
    """Algorithm 1 after the loop: median of G^ext, beta closest among G^agr, average.
    want_extra: also (scale, margin, alt)."""
    G, n, d, ld = _grads(G)
    ext = np.ascontiguousarray(ext, np.int32)
    sets = np.ascontiguousarray(agr_sets, np.uint8)
    theta = len(ext)
    assert sets.shape == (theta, n)
    out = np.empty(d, np.float32)
    scale = np.empty(d, np.float32) if want_extra else None
    margin = np.empty(d, np.float32) if want_extra else None
    alt = np.empty(d, np.float32) if want_extra else None
    _load().orc_coordwise_alg1(_ptr(G, C.c_float), n, d, ld, _ptr(ext, C.c_int32), _ptr(sets, C.c_uint8),
                               theta, beta, _ptr(out, C.c_float), _ptr(scale, C.c_float),
                               _ptr(margin, C.c_float), _ptr(alt, C.c_float), nthreads)
    return (out, scale, margin, alt) if want_extra else out


def alg1_accepts(col, ext, agr_sets, beta, got, noise_rel=4e-6, tol_rel=1e-5, max_subsets=20000):
    """Comparison aid for ONE coordinate of the Algorithm-1 phase (plain Python, slow): is `got` the
    average of beta entries of G^agr that an evaluation with relative rounding noise `noise_rel` could
    legitimately have found closest to the median?  `col` = the n values of the coordinate.

    Algorithm 1 takes the beta entries closest to M (Argpartition: ties open).  With closeness
    delta_t = |G^agr[t] - M| in fp32, delta* its beta-th smallest value and scale = the largest mean
    absolute value of the rows averaged into a round (what coordwise_alg1 reports): entries with
    delta_t < delta* - noise are in every legitimate choice, entries with delta_t <= delta* + noise may
    be, the others are not (noise = noise_rel * scale).  Accepted iff some such choice averages to
    `got` within tol_rel * max(|average|, scale).  Generalises margin / alt of coordwise_alg1 (one
    runner-up) to several averages nearly equidistant from the median."""
    import itertools
    col = np.asarray(col, np.float32)
    ext = np.asarray(ext)
    sets = np.asarray(agr_sets).astype(bool)
    theta = len(ext)
    e = np.sort(col[ext])
    med = e[theta // 2] if theta % 2 else np.float32(0.5) * np.float32(e[theta // 2 - 1] + e[theta // 2])
    a = np.zeros(theta, np.float32)
    scale = 0.0
    for t in range(theta):
        rows = col[sets[t]].astype(np.float64)
        if rows.size:
            a[t] = np.float32(rows.sum() / rows.size)
            scale = max(scale, float(np.abs(rows).sum() / rows.size))
    delta = np.abs((a - med).astype(np.float32)).astype(np.float64)
    star = np.sort(delta)[beta - 1]
    noise = noise_rel * scale
    must = [t for t in range(theta) if delta[t] < star - noise]
    pool = [t for t in range(theta) if delta[t] <= star + noise and t not in must]
    k = beta - len(must)
    if k < 0 or k > len(pool):
        return False
    base = float(np.sum(a[must].astype(np.float64)))
    for count, sub in enumerate(itertools.combinations(pool, k)):
        if count >= max_subsets:
            return False
        cand = (base + float(np.sum(a[list(sub)].astype(np.float64)))) / beta
        if abs(float(got) - cand) <= tol_rel * max(abs(cand), scale) + 1e-37:
            return True
    return False


def multikrum_aggregate(G, f, nthreads=0):
    """Multi-Krum GAR: average of the n-f-2 best-scored gradients.  (out, mask)."""
    G, n, d, ld = _grads(G)
    out = np.empty(d, np.float32)
    mask = np.zeros(n, np.uint8)
    _check(_load().orc_multikrum_aggregate(_ptr(G, C.c_float), n, f, d, ld, _ptr(out, C.c_float),
                                           _ptr(mask, C.c_uint8), nthreads))
    return out, mask


def coordwise_median(G, nthreads=0):
    """Coordinate-wise median of all rows (the Median GAR of Section V)."""
    G, n, d, ld = _grads(G)
    out = np.empty(d, np.float32)
    _load().orc_coordwise_median(_ptr(G, C.c_float), n, d, ld, _ptr(out, C.c_float), nthreads)
    return out


def mbulyan(G, f, mode=MODE_SELECTED, nthreads=0):
    """GAR(f, G) = multi-Bulyan (Algorithm 1).  Returns (out[d], ext[theta])."""
    G, n, d, ld = _grads(G)
    theta, _ = params(n, f, mode)
    out = np.empty(d, np.float32)
    ext = np.empty(theta, np.int32)
    _check(_load().orc_mbulyan(_ptr(G, C.c_float), n, f, d, ld, mode, _ptr(out, C.c_float),
                               _ptr(ext, C.c_int32), nthreads))
    return out, ext
