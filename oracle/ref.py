"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.
It loads oracle/libinshr_ref.so (plain C, built by oracle/build.py) and exchanges numpy arrays
with it.  It imports nothing from the HIP package.
"""
import ctypes as C

import numpy as np

from . import build as _build


class Config(C.Structure):
    _fields_ = [("bits", C.c_uint8), ("bins", C.c_uint16), ("prune_ppm", C.c_uint32),
                ("outlier_ppm", C.c_uint32)]


def _config(cfg):
    """cfg = (bits, prune_ppm, outlier_ppm) or (bits, prune_ppm, outlier_ppm, bins): with bins > 0
    the number of bins is that count, otherwise 2^bits."""
    b, p, o = cfg[:3]
    k = int(cfg[3]) if len(cfg) > 3 else 0
    return Config(int(b), k, int(p), int(o))


def bins_of(cfg):
    return int(cfg[3]) if len(cfg) > 3 and cfg[3] else 1 << int(cfg[0])


def symbol_bits(K):
    return int(lib().inshr_ref_symbol_bits(C.c_uint32(K)))


class Score(C.Structure):
    _fields_ = [("sse", C.c_double), ("sumsq", C.c_double), ("n_pruned", C.c_uint64),
                ("n_outlier", C.c_uint64), ("n_kept", C.c_uint64), ("cost_bits", C.c_uint64)]


class QInfo(C.Structure):
    _fields_ = [("n_pruned", C.c_uint64), ("n_outlier", C.c_uint64), ("n_kept", C.c_uint64),
                ("sym_bits", C.c_uint32), ("tau_prune_bits", C.c_uint32),
                ("tau_outlier_bits", C.c_uint32), ("sse", C.c_double), ("sumsq", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def _grid(grid):
    arr = (Config * len(grid))()
    for i, cfg in enumerate(grid):
        arr[i] = _config(cfg)
    return arr


class RefError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle error {code}")
        self.code = code


def pool_of(tensors):
    """Ascending magnitude images (uint32, -0.0 as +0.0) of all values of a group of tensors: the
    pooled order statistics that per-layer-type thresholds are read from (Sec. 4.2)."""
    mags = [np.ascontiguousarray(t, np.float32).ravel().view(np.uint32) & np.uint32(0x7fffffff) for t in tensors]
    return np.sort(np.concatenate(mags), kind="stable")


def quantize(x, cfg, pool=None):
    """cfg = (bits, prune_ppm, outlier_ppm[, bins]). Returns dict of numpy arrays and scalars.
    pool: pool_of(the tensors of x's layer type); thresholds are then the pooled quantiles."""
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    n = x.size
    o = cfg[2]
    K = bins_of(cfg)
    cap = n if pool is not None else max(1, n * int(o) // 1000000)
    sym = np.empty(n, np.uint16)
    bnd = np.empty(max(K - 1, 1), np.float32)
    cb = np.empty(K, np.float32)
    oi = np.empty(cap, np.uint32)
    ov = np.empty(cap, np.float32)
    info = QInfo()
    c = _config(cfg)
    pool = None if pool is None else np.ascontiguousarray(pool, np.uint32)
    rc = lib().inshr_ref_quantize_pooled(_p(x, C.c_float), C.c_uint64(n), _p(pool, C.c_uint32),
                                         C.c_uint64(0 if pool is None else pool.size), C.byref(c),
                                         _p(sym, C.c_uint16), _p(bnd, C.c_float), _p(cb, C.c_float),
                                         _p(oi, C.c_uint32), _p(ov, C.c_float), C.byref(info))
    if rc:
        raise RefError(rc)
    no = int(info.n_outlier)
    return dict(sym=sym, boundaries=bnd[:K - 1], codebook=cb, outlier_idx=oi[:no].copy(),
                outlier_val=ov[:no].copy(), n_pruned=int(info.n_pruned), n_outlier=no,
                n_kept=int(info.n_kept), sym_bits=int(info.sym_bits), K=K,
                tau_prune_bits=int(info.tau_prune_bits), tau_outlier_bits=int(info.tau_outlier_bits),
                sse=float(info.sse), sumsq=float(info.sumsq))


def quantize_sens(x, g, cfg, by_sens):
    """Partition by magnitude and sensitivity (Sec. 4.1-4.2): g = gradients, by_sens = the pruning
    metric is the sensitivity score.  Returns the dict of quantize plus tau_outlier_sens_bits."""
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    g = np.ascontiguousarray(g, dtype=np.float32).ravel()
    n = x.size
    if g.size != n:
        raise RefError(-5)
    K = bins_of(cfg)
    sym = np.empty(n, np.uint16)
    bnd = np.empty(max(K - 1, 1), np.float32)
    cb = np.empty(K, np.float32)
    oi = np.empty(n, np.uint32)
    ov = np.empty(n, np.float32)
    info = QInfo()
    tos = C.c_uint32(0)
    c = _config(cfg)
    rc = lib().inshr_ref_quantize_sens(_p(x, C.c_float), _p(g, C.c_float), C.c_uint64(n), C.byref(c),
                                       C.c_int(1 if by_sens else 0), _p(sym, C.c_uint16), _p(bnd, C.c_float),
                                       _p(cb, C.c_float), _p(oi, C.c_uint32), _p(ov, C.c_float),
                                       C.byref(info), C.byref(tos))
    if rc:
        raise RefError(rc)
    no = int(info.n_outlier)
    return dict(sym=sym, boundaries=bnd[:K - 1], codebook=cb, outlier_idx=oi[:no].copy(),
                outlier_val=ov[:no].copy(), n_pruned=int(info.n_pruned), n_outlier=no,
                n_kept=int(info.n_kept), sym_bits=int(info.sym_bits), K=K,
                tau_prune_bits=int(info.tau_prune_bits), tau_outlier_bits=int(info.tau_outlier_bits),
                tau_outlier_sens_bits=int(tos.value), sse=float(info.sse), sumsq=float(info.sumsq))


def bf16_round(x):
    """Protected values as Sec. 4.2 stores them: rounded to bfloat16 (returned as float32)."""
    x = np.ascontiguousarray(x, np.float32)
    f = lib().inshr_ref_bf16_round
    f.restype = C.c_float
    f.argtypes = [C.c_float]
    return np.array([f(float(v)) for v in x.ravel()], np.float32).reshape(x.shape)


def search(x, grid, eps, pool=None):
    """Returns (best, feasible, scores) with scores a list of dicts, one per grid entry.
    pool: as for quantize."""
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    g = _grid(grid)
    sc = (Score * len(grid))()
    best = C.c_uint32(0)
    feas = C.c_uint8(0)
    pool = None if pool is None else np.ascontiguousarray(pool, np.uint32)
    rc = lib().inshr_ref_search_pooled(_p(x, C.c_float), C.c_uint64(x.size), _p(pool, C.c_uint32),
                                       C.c_uint64(0 if pool is None else pool.size), g,
                                       C.c_uint32(len(grid)), C.c_double(eps), C.byref(best),
                                       C.byref(feas), sc)
    if rc:
        raise RefError(rc)
    scores = [dict(sse=s.sse, sumsq=s.sumsq, n_pruned=s.n_pruned, n_outlier=s.n_outlier,
                   n_kept=s.n_kept, cost_bits=s.cost_bits) for s in sc]
    return int(best.value), int(feas.value), scores


def dequantize(sym, bits, codebook, outlier_idx, outlier_val, K=None):
    """K: the number of bins when it is not 2^bits."""
    sym = np.ascontiguousarray(sym, np.uint16)
    cb = np.ascontiguousarray(codebook, np.float32)
    oi = np.ascontiguousarray(outlier_idx, np.uint32)
    ov = np.ascontiguousarray(outlier_val, np.float32)
    out = np.empty(sym.size, np.float32)
    rc = lib().inshr_ref_dequantize_k(_p(sym, C.c_uint16), C.c_uint64(sym.size),
                                      C.c_uint32(K if K else 1 << bits),
                                      _p(cb, C.c_float), _p(oi, C.c_uint32), _p(ov, C.c_float),
                                      C.c_uint64(oi.size), _p(out, C.c_float))
    if rc:
        raise RefError(rc)
    return out


def delta(s_prev, bits_prev, s_cur, bits_cur, K_prev=None, K_cur=None):
    """K_prev / K_cur: the numbers of bins when they are not 2^bits."""
    K_prev = K_prev if K_prev else 1 << bits_prev
    K_cur = K_cur if K_cur else 1 << bits_cur
    s_prev = np.ascontiguousarray(s_prev, np.uint16)
    s_cur = np.ascontiguousarray(s_cur, np.uint16)
    n = s_prev.size
    if s_cur.size != n:
        raise RefError(-5)
    d = np.empty(n, np.uint16)
    perm = np.empty(n, np.uint32)
    goff = np.empty(K_prev + 3, np.uint64)
    stream = np.empty(n, np.uint16)
    rc = lib().inshr_ref_delta_k(_p(s_prev, C.c_uint16), C.c_uint32(K_prev), _p(s_cur, C.c_uint16),
                                 C.c_uint32(K_cur), C.c_uint64(n), _p(d, C.c_uint16),
                                 _p(perm, C.c_uint32), _p(goff, C.c_uint64), _p(stream, C.c_uint16))
    if rc:
        raise RefError(rc)
    # the deltas lie in [0, B) with B = max(K_prev, K_cur) + 2 levels: same width as a symbol of the wider side
    return dict(delta=d, perm=perm, group_off=goff, stream=stream,
                delta_bits=symbol_bits(max(K_prev, K_cur)))


def reconstruct(s_prev, bits_prev, bits_cur, group_off, stream, K_prev=None, K_cur=None):
    K_prev = K_prev if K_prev else 1 << bits_prev
    K_cur = K_cur if K_cur else 1 << bits_cur
    s_prev = np.ascontiguousarray(s_prev, np.uint16)
    goff = np.ascontiguousarray(group_off, np.uint64)
    stream = np.ascontiguousarray(stream, np.uint16)
    out = np.empty(s_prev.size, np.uint16)
    rc = lib().inshr_ref_reconstruct_k(_p(s_prev, C.c_uint16), C.c_uint32(K_prev),
                                       C.c_uint32(K_cur), C.c_uint64(s_prev.size),
                                       _p(goff, C.c_uint64), _p(stream, C.c_uint16),
                                       _p(out, C.c_uint16))
    if rc:
        raise RefError(rc)
    return out


def pack(v, w):
    v = np.ascontiguousarray(v, np.uint16)
    words = np.empty((v.size * w + 63) // 64, np.uint64)
    rc = lib().inshr_ref_pack(_p(v, C.c_uint16), C.c_uint64(v.size), C.c_uint32(w),
                              _p(words, C.c_uint64))
    if rc:
        raise RefError(rc)
    return words


def unpack(words, n, w):
    words = np.ascontiguousarray(words, np.uint64)
    v = np.empty(n, np.uint16)
    rc = lib().inshr_ref_unpack(_p(words, C.c_uint64), C.c_uint64(n), C.c_uint32(w),
                                _p(v, C.c_uint16))
    if rc:
        raise RefError(rc)
    return v
