"""Thin Python binding of the C ABI in include/inshr.h (argument marshalling only).

Every step of search / quantize / delta runs in the HIP kernels of libinshr.so.  torch is used for
device memory and streams.  There is no CPU fallback: loading fails loudly when the library has
not been built (python -m paper_2306_11800_amd.build or __graft_entry__.build()).
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libinshr.so")

EXPORTS = ["inshr_create", "inshr_destroy", "inshr_strerror", "inshr_last_device_error",
           "inshr_sync", "inshr_lds_ordered", "inshr_sketch_quantiles", "inshr_search_sketch_grid", "inshr_search", "inshr_search_pooled", "inshr_quantize_sens", "inshr_quantize_bound", "inshr_quantize",
           "inshr_quantize_sketch", "inshr_search_sketch", "inshr_sketch_buckets",
           "inshr_delta_bound", "inshr_delta", "inshr_delta_static", "inshr_guided_search", "inshr_neighbourhood_search", "inshr_dequantize", "inshr_reconstruct",
           "inshr_entropy_encode", "inshr_entropy_decode",
           "inshr_profile", "inshr_profile_read"]

INSHR_REUSE_SEARCH = 1
INSHR_PROTECT_BF16 = 2
GROUP_OFF_ENTRIES = 259  # group offsets of a delta: (1 << 8) + 3, whatever the bits of prev


class CConfig(C.Structure):
    _fields_ = [("bits", C.c_uint8), ("bins", C.c_uint16), ("prune_ppm", C.c_uint32),
                ("outlier_ppm", C.c_uint32)]


def bins_of(cfg) -> int:
    """Number of bins of a configuration tuple (bits, prune_ppm, outlier_ppm[, bins])."""
    return int(cfg[3]) if len(cfg) > 3 and cfg[3] else 1 << int(cfg[0])


def symbol_bits(K: int) -> int:
    """Width of a symbol with K bins: K + 2 levels (pruned, protected, the bins)."""
    return max(1, (K + 1).bit_length())


class CTensor(C.Structure):
    _fields_ = [("data", C.c_void_p), ("n", C.c_uint64)]


class CScore(C.Structure):
    _fields_ = [("sse", C.c_double), ("sumsq", C.c_double), ("n_pruned", C.c_uint64),
                ("n_outlier", C.c_uint64), ("n_kept", C.c_uint64), ("cost_bits", C.c_uint64)]


class CSensInfo(C.Structure):
    _fields_ = [("tau_outlier_sens", C.c_float), ("sse", C.c_double), ("sumsq", C.c_double)]


class CQuantized(C.Structure):
    _fields_ = [("packed", C.c_void_p), ("packed_words", C.c_uint64), ("codebook", C.c_void_p),
                ("boundaries", C.c_void_p), ("outlier_idx", C.c_void_p), ("outlier_val", C.c_void_p),
                ("outlier_cap", C.c_uint64), ("n_pruned", C.c_uint64), ("n_outlier", C.c_uint64),
                ("n_kept", C.c_uint64), ("sym_bits", C.c_uint32), ("tau_prune", C.c_float),
                ("tau_outlier", C.c_float), ("n_bins", C.c_uint32)]


class CSketchParams(C.Structure):
    _fields_ = [("alpha", C.c_double), ("sigma", C.c_double), ("max_iter", C.c_uint32),
                ("uniforms", C.c_void_p)]


class CSketchInfo(C.Structure):
    _fields_ = [("n_buckets", C.c_uint32), ("rounds", C.c_uint32)]


class CSketchChoice(C.Structure):
    _fields_ = [("sse", C.c_double * 7), ("sumsq", C.c_double), ("rounds", C.c_uint32 * 7),
                ("best_bits", C.c_uint32), ("feasible", C.c_uint32)]


class CCodes(C.Structure):
    _fields_ = [("packed", C.c_void_p), ("sym_bits", C.c_uint32), ("bits", C.c_uint8),
                ("bins", C.c_uint16), ("n", C.c_uint64)]


class CKernelTime(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("total_ms", C.c_double), ("launches", C.c_uint64)]


class CDeltaOut(C.Structure):
    _fields_ = [("packed", C.c_void_p), ("packed_words", C.c_uint64), ("group_off", C.c_void_p),
                ("perm", C.c_void_p), ("delta_bits", C.c_uint32), ("group_off_entries", C.c_uint32)]


class CDequantIn(C.Structure):
    _fields_ = [("packed", C.c_void_p), ("codebook", C.c_void_p), ("outlier_idx", C.c_void_p),
                ("outlier_val", C.c_void_p), ("n_outlier", C.c_uint64), ("n", C.c_uint64),
                ("bits", C.c_uint8), ("protected_bf16", C.c_uint8), ("bins", C.c_uint16)]


class CEntropyStats(C.Structure):
    _fields_ = [("n_tokens", C.c_uint64), ("table_bytes", C.c_uint64), ("payload_bytes", C.c_uint64)]


class CCodesOut(C.Structure):
    _fields_ = [("packed", C.c_void_p), ("packed_words", C.c_uint64), ("bits", C.c_uint8),
                ("bins", C.c_uint16)]


_lib = None


def load_library() -> C.CDLL:
    """Load libinshr.so; raise if it is missing (the product path never falls back to the CPU)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2306_11800_amd.build`")
    lib = C.CDLL(LIB_PATH)
    lib.inshr_create.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.c_void_p, C.c_uint64]
    lib.inshr_destroy.argtypes = [C.c_void_p]
    lib.inshr_destroy.restype = None
    lib.inshr_strerror.argtypes = [C.c_int]
    lib.inshr_strerror.restype = C.c_char_p
    lib.inshr_last_device_error.argtypes = [C.c_void_p]
    lib.inshr_last_device_error.restype = C.c_char_p
    lib.inshr_sync.argtypes = [C.c_void_p]
    lib.inshr_lds_ordered.argtypes = [C.c_void_p]
    lib.inshr_search.argtypes = [C.c_void_p, C.POINTER(CTensor), C.c_uint32, C.POINTER(CConfig),
                                 C.c_uint32, C.c_double, C.POINTER(C.c_uint32),
                                 C.POINTER(C.c_uint8), C.POINTER(CScore)]
    lib.inshr_quantize_bound.argtypes = [C.c_uint64, C.POINTER(CConfig), C.POINTER(C.c_uint64),
                                         C.POINTER(C.c_uint64)]
    lib.inshr_quantize.argtypes = [C.c_void_p, C.POINTER(CTensor), C.POINTER(CConfig),
                                   C.POINTER(CQuantized), C.c_uint32, C.c_uint32]
    lib.inshr_quantize_sketch.argtypes = [C.c_void_p, C.POINTER(CTensor), C.POINTER(CConfig),
                                          C.POINTER(CSketchParams), C.POINTER(CQuantized),
                                          C.POINTER(CSketchInfo), C.c_uint32, C.c_uint32]
    lib.inshr_search_sketch.argtypes = [C.c_void_p, C.POINTER(CTensor), C.POINTER(CConfig),
                                        C.POINTER(CSketchParams), C.c_double, C.POINTER(CQuantized),
                                        C.POINTER(CSketchChoice), C.POINTER(CSketchInfo), C.c_uint32,
                                        C.c_uint32]
    lib.inshr_sketch_buckets.argtypes = [C.c_double, C.POINTER(C.c_int32), C.POINTER(C.c_uint32), C.c_void_p,
                                         C.c_void_p, C.c_uint32]
    lib.inshr_delta_bound.argtypes = [C.POINTER(CCodes), C.POINTER(CCodes), C.POINTER(C.c_uint64)]
    lib.inshr_delta.argtypes = [C.c_void_p, C.POINTER(CCodes), C.POINTER(C.c_void_p),
                                C.POINTER(CCodes), C.POINTER(CDeltaOut), C.c_uint32]
    lib.inshr_delta_static.argtypes = [C.c_void_p, C.POINTER(CCodes), C.POINTER(CCodes),
                                       C.POINTER(CDeltaOut), C.c_uint32]
    lib.inshr_search_pooled.argtypes = [C.c_void_p, C.POINTER(CTensor), C.POINTER(C.c_uint32), C.c_uint32,
                                        C.POINTER(CConfig), C.c_uint32, C.c_double, C.POINTER(C.c_uint32),
                                        C.POINTER(C.c_uint8), C.POINTER(CScore)]
    lib.inshr_quantize_sens.argtypes = [C.c_void_p, C.POINTER(CTensor), C.POINTER(C.c_void_p), C.POINTER(CConfig),
                                        C.POINTER(C.c_uint8), C.POINTER(CQuantized), C.POINTER(CSensInfo),
                                        C.c_uint32]
    lib.inshr_sketch_quantiles.argtypes = [C.c_void_p, C.POINTER(CTensor), C.c_uint32, C.POINTER(C.c_double),
                                           C.c_uint32, C.c_double, C.POINTER(C.c_double)]
    lib.inshr_search_sketch_grid.argtypes = [C.c_void_p, C.POINTER(CTensor), C.POINTER(CConfig), C.c_uint32,
                                             C.POINTER(CSketchParams), C.c_double, C.POINTER(CQuantized),
                                             C.POINTER(C.c_uint32), C.POINTER(CSketchChoice),
                                             C.POINTER(CSketchChoice), C.c_uint32]
    lib.inshr_guided_search.argtypes = [C.POINTER(CScore), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32),
                                        C.c_double, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32),
                                        C.POINTER(C.c_uint32), C.POINTER(C.c_uint8)]
    lib.inshr_neighbourhood_search.argtypes = [C.POINTER(CScore), C.POINTER(C.c_uint32),
                                               C.POINTER(C.c_uint32), C.c_uint32, C.c_uint32, C.c_double,
                                               C.POINTER(C.c_uint32), C.POINTER(C.c_uint32),
                                               C.POINTER(C.c_uint32)]
    lib.inshr_dequantize.argtypes = [C.c_void_p, C.POINTER(CDequantIn), C.POINTER(C.c_void_p),
                                     C.c_uint32]
    lib.inshr_reconstruct.argtypes = [C.c_void_p, C.POINTER(CCodes), C.POINTER(CDeltaOut),
                                      C.POINTER(CCodesOut), C.c_uint32]
    lib.inshr_entropy_encode.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p,
                                         C.c_uint32, C.c_void_p, C.c_uint64, C.POINTER(C.c_uint64),
                                         C.POINTER(CEntropyStats)]
    lib.inshr_entropy_decode.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32,
                                         C.c_void_p, C.c_void_p, C.c_void_p]
    lib.inshr_profile.argtypes = [C.c_void_p, C.c_int]
    lib.inshr_profile_read.argtypes = [C.c_void_p, C.POINTER(CKernelTime), C.c_uint32,
                                       C.POINTER(C.c_uint32)]
    _lib = lib
    return lib


class InshrError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"inshr error {code}: {text}")
        self.code = code


class Quantized:
    """Device-side result of quantizing one tensor.  The tensors are views of buffers allocated at
    the capacity inshr_quantize_bound gives; the views are made when they are asked for.  Counts,
    thresholds and the symbol width are read from the C struct that inshr_quantize filled."""
    __slots__ = ("n", "_bufs", "_ptrs", "_c", "_keep", "bf16")

    def __init__(self, n, bits, bufs, c_entry=None, keep=None, bins=0):
        if c_entry is None:
            c_entry = CQuantized()
        self.n = n
        self._bufs = bufs                                   # packed, codebook, boundaries, idx, val
        self._ptrs = tuple(b.data_ptr() for b in bufs)
        self._c = c_entry                                   # element of the CQuantized array
        self._keep = keep                                   # the array itself
        self.bf16 = False                                   # protected values stored as bfloat16
        c_entry.n_bins = bins if bins else 1 << bits
        c_entry.sym_bits = symbol_bits(c_entry.n_bins)

    sym_bits = property(lambda self: self._c.sym_bits)
    bits = property(lambda self: self._c.sym_bits - 1)      # of a power-of-two bin count
    K = property(lambda self: self._c.n_bins)               # number of bins
    n_pruned = property(lambda self: self._c.n_pruned)
    n_kept = property(lambda self: self._c.n_kept)
    tau_prune = property(lambda self: self._c.tau_prune)
    tau_outlier = property(lambda self: self._c.tau_outlier)

    @property
    def n_outlier(self):
        return self._c.n_outlier

    @n_outlier.setter
    def n_outlier(self, v):                  # (tests hand a wrong list length to the decoder)
        self._c.n_outlier = v

    @property
    def packed(self) -> torch.Tensor:        # int64 words (bit pattern of u64)
        return self._bufs[0][:(self.n * self.sym_bits + 63) // 64]

    @property
    def codebook(self) -> torch.Tensor:      # float32 [K]
        return self._bufs[1][:self.K]

    @property
    def boundaries(self) -> torch.Tensor:    # float32 [K-1]
        return self._bufs[2][:self.K - 1]

    @property
    def outlier_idx(self) -> torch.Tensor:   # int32 (bit pattern of u32) [n_outlier]
        return self._bufs[3][:self.n_outlier]

    @property
    def outlier_val(self) -> torch.Tensor:   # float32 [n_outlier], or bfloat16 when stored so
        if self.bf16:
            return self._bufs[4].view(torch.bfloat16)[:self.n_outlier]
        return self._bufs[4][:self.n_outlier]


class TensorBatch(list):
    """A list of tensors with its marshalled C array, for callers that pass the same tensors again
    and again (Context.batch).  The list must not be changed afterwards."""
    __slots__ = ("_ta",)


class QuantizedBatch(list):
    """The list inshr_quantize's binding returns; it keeps the C array of its entries so that a
    call with out=<this list> writes the same buffers again without marshalling them again."""
    __slots__ = ("_qa", "_sizes")


class DeltaBatch(list):
    __slots__ = ("_pa", "_ca", "_oa", "_prev", "_cur")


@dataclass
class Delta:
    n: int
    delta_bits: int
    packed: torch.Tensor        # int64 words
    group_off: torch.Tensor     # int64 [(1 << bits_prev) + 3]: a view of goff_buf
    perm: Optional[torch.Tensor]  # int32 (bit pattern of u32) [n] or None
    goff_buf: Optional[torch.Tensor] = None  # int64 [GROUP_OFF_ENTRIES]: room for any bits of prev


def _tensor_array(tensors: Sequence[torch.Tensor]):
    if isinstance(tensors, TensorBatch):
        return tensors._ta
    arr = (CTensor * len(tensors))()
    for i, t in enumerate(tensors):
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous float32 CUDA tensors")
        arr[i] = CTensor(t.data_ptr(), t.numel())
    return arr


def _config_array(cfgs):
    arr = (CConfig * len(cfgs))()
    for i, cfg in enumerate(cfgs):
        arr[i] = CConfig(int(cfg[0]), int(cfg[3]) if len(cfg) > 3 else 0, int(cfg[1]), int(cfg[2]))
    return arr


def cube_of(grid) -> Tuple[List[int], Tuple[int, int, int], tuple]:
    """Configuration cube (Sec. 5) of a full-factorial grid of (bits, prune_ppm, protect_ppm[, bins]):
    (cell_cfg, dims, axes) with axis 0 the numbers of bins ascending, axis 1 the prune fractions
    descending, axis 2 the protect fractions ascending."""
    ks = sorted({bins_of(g) for g in grid})
    ps = sorted({g[1] for g in grid}, reverse=True)
    os_ = sorted({g[2] for g in grid})
    where = {(bins_of(g), g[1], g[2]): i for i, g in enumerate(grid)}
    cells = [where[(k, p, o)] for k in ks for p in ps for o in os_]
    return cells, (len(ks), len(ps), len(os_)), (ks, ps, os_)


def _cube_args(scores, cell_cfg, dims):
    n = len(cell_cfg)
    if n != dims[0] * dims[1] * dims[2]:
        raise ValueError("cell_cfg does not fill the cube")
    return (C.c_uint32 * n)(*cell_cfg), (C.c_uint32 * 3)(*dims)


def guided_search(scores, cell_cfg, dims, eps: float):
    """inshr_guided_search on one row of a score table (a ctypes array of CScore).  Returns
    ((i, j, k), feasible, trials, visited[list of 0/1 per cell])."""
    lib = load_library()
    cc, dd = _cube_args(scores, cell_cfg, dims)
    best, feas, trials = C.c_uint32(), C.c_uint32(), C.c_uint32()
    vis = (C.c_uint8 * len(cell_cfg))()
    rc = lib.inshr_guided_search(scores, cc, dd, float(eps), C.byref(best), C.byref(feas), C.byref(trials), vis)
    if rc:
        raise InshrError(rc, "inshr_guided_search")
    b = best.value
    return (b >> 16, (b >> 8) & 255, b & 255), bool(feas.value), trials.value, list(vis)


def neighbourhood_search(scores, cell_cfg, dims, prev_cell, e: int, eps: float):
    """inshr_neighbourhood_search; prev_cell = (i, j, k).  Returns ((i, j, k), feasible, trials)."""
    lib = load_library()
    cc, dd = _cube_args(scores, cell_cfg, dims)
    best, feas, trials = C.c_uint32(), C.c_uint32(), C.c_uint32()
    pc = prev_cell[0] << 16 | prev_cell[1] << 8 | prev_cell[2]
    rc = lib.inshr_neighbourhood_search(scores, cc, dd, pc, int(e), float(eps), C.byref(best),
                                        C.byref(feas), C.byref(trials))
    if rc:
        raise InshrError(rc, "inshr_neighbourhood_search")
    b = best.value
    return (b >> 16, (b >> 8) & 255, b & 255), bool(feas.value), trials.value


class Context:
    """One device + one stream + scratch memory (inshr_ctx)."""

    def __init__(self, device: Optional[torch.device] = None, scratch_bytes: int = 0):
        self.lib = load_library()
        self.device = torch.device(device if device is not None else "cuda:0")
        idx = self.device.index if self.device.index is not None else 0
        self.stream = torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        rc = self.lib.inshr_create(C.byref(h), idx, C.c_void_p(self.stream.cuda_stream), scratch_bytes)
        if rc:
            raise InshrError(rc, self.lib.inshr_strerror(rc).decode())
        self.h = h
        self._bounds = {}

    def close(self):
        if getattr(self, "h", None):
            self.lib.inshr_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc:
            text = self.lib.inshr_strerror(rc).decode()
            extra = self.lib.inshr_last_device_error(self.h).decode()
            raise InshrError(rc, text + (f" ({extra})" if extra and rc in (-6, -7, -4, -2, -1) else ""))

    def sync(self):
        self._check(self.lib.inshr_sync(self.h))

    @property
    def lds_ordered(self) -> bool:
        """Whether equal symbols are ranked by returning LDS adds (True) or by ballots (False)."""
        return bool(self.lib.inshr_lds_ordered(self.h))

    def profile(self, enable: bool):
        self._check(self.lib.inshr_profile(self.h, 1 if enable else 0))

    def profile_read(self):
        """{kernel name: (total ms, launches)} since profile(True)."""
        n = C.c_uint32()
        arr = (CKernelTime * 64)()
        self._check(self.lib.inshr_profile_read(self.h, arr, 64, C.byref(n)))
        return {arr[i].name.decode(): (arr[i].total_ms, int(arr[i].launches))
                for i in range(min(n.value, 64))}

    def batch(self, tensors: Sequence[torch.Tensor]) -> TensorBatch:
        """The same tensors as a list that carries its C array (see TensorBatch)."""
        b = TensorBatch(tensors)
        b._ta = _tensor_array(list(tensors))
        return b

    # -- inshr_search ---------------------------------------------------------------------
    def search(self, tensors: Sequence[torch.Tensor], grid, eps: float, want_scores: bool = True,
               groups: Optional[Sequence[int]] = None):
        """Returns (best[list of int], feasible[list of int], scores or None) where scores is a
        ctypes array of CScore of length len(tensors) * len(grid), row-major by tensor.
        groups: one number per tensor; tensors with equal numbers share their thresholds
        (inshr_search_pooled)."""
        ta = _tensor_array(tensors)
        ga = _config_array(grid)
        nT, nC = len(tensors), len(grid)
        best = (C.c_uint32 * nT)()
        feas = (C.c_uint8 * nT)()
        scores = (CScore * (nT * nC))() if want_scores else None
        if groups is not None:
            if len(groups) != nT:
                raise ValueError("one group number per tensor")
            ga_ = (C.c_uint32 * nT)(*[int(g) for g in groups])
            self._check(self.lib.inshr_search_pooled(self.h, ta, ga_, nT, ga, nC, float(eps), best, feas, scores))
        else:
            self._check(self.lib.inshr_search(self.h, ta, nT, ga, nC, float(eps), best, feas, scores))
        return list(best), list(feas), scores

    # -- inshr_quantize -------------------------------------------------------------------
    def quantize(self, tensors: Sequence[torch.Tensor], cfgs, reuse_search: bool = False,
                 out: Optional[List[Quantized]] = None, protect_bf16: bool = False,
                 outlier_caps: Optional[Sequence[int]] = None) -> List[Quantized]:
        """`out` may carry the list an earlier call returned for tensors of the same sizes; its
        device buffers are then written again.  When that call sized them for the largest
        configuration (8 bits and the largest protect fraction in use), nothing is marshalled
        again."""
        nT = len(tensors)
        ta = _tensor_array(tensors)
        ca = _config_array(cfgs)
        flags = (INSHR_REUSE_SEARCH if reuse_search else 0) | (INSHR_PROTECT_BF16 if protect_bf16 else 0)
        if isinstance(out, QuantizedBatch) and out._sizes == tuple(t.numel() for t in tensors):
            # the C side checks every buffer against what the configuration needs
            self._check(self.lib.inshr_quantize(self.h, ta, ca, out._qa, nT, flags))
            for q in out:
                q.bf16 = protect_bf16
            return out
        qa = (CQuantized * nT)()
        res = QuantizedBatch()
        for i, (t, cfg) in enumerate(zip(tensors, cfgs)):
            n = t.numel()
            words, cap = self._bound(n, ca[i], cfg)
            if outlier_caps is not None:  # (after a search with shared thresholds a tensor's share
                cap = int(outlier_caps[i])  # of the protected values is not bounded by the fraction)
            e = qa[i]
            if out is not None:
                q = out[i]
                if q.n != n or q._bufs[0].numel() < words or q._bufs[3].numel() < cap:
                    raise ValueError("pre-allocated buffers are too small")
                q = Quantized(n, int(cfg[0]), q._bufs, e, qa, bins=bins_of(cfg))
            else:
                q = Quantized(n, int(cfg[0]), (
                    torch.empty(words, dtype=torch.int64, device=t.device),
                    torch.empty(256, dtype=torch.float32, device=t.device),
                    torch.empty(255, dtype=torch.float32, device=t.device),
                    torch.empty(max(cap, 1), dtype=torch.int32, device=t.device),
                    torch.empty(max(cap, 1), dtype=torch.float32, device=t.device)), e, qa, bins=bins_of(cfg))
            e.packed, e.codebook, e.boundaries, e.outlier_idx, e.outlier_val = q._ptrs
            e.packed_words = q._bufs[0].numel()
            e.outlier_cap = q._bufs[3].numel()
            res.append(q)
        res._qa = qa
        res._sizes = tuple(q.n for q in res)
        self._check(self.lib.inshr_quantize(self.h, ta, ca, qa, nT, flags))
        for q in res:
            q.bf16 = protect_bf16
        return res

    # -- inshr_sketch_quantiles ------------------------------------------------------------
    def sketch_quantiles(self, tensors: Sequence[torch.Tensor], q: Sequence[float], alpha: float = 0.01):
        """The sketch's estimates of the magnitudes of rank floor(q (n - 1)): list (per tensor) of lists."""
        nT, nq = len(tensors), len(q)
        ta = _tensor_array(tensors)
        qa = (C.c_double * nq)(*[float(v) for v in q])
        out = (C.c_double * (nT * nq))()
        self._check(self.lib.inshr_sketch_quantiles(self.h, ta, nT, qa, nq, float(alpha), out))
        return [[out[t * nq + k] for k in range(nq)] for t in range(nT)]

    # -- inshr_quantize_sens ---------------------------------------------------------------
    def quantize_sens(self, tensors: Sequence[torch.Tensor], grads: Sequence[torch.Tensor], cfgs,
                      by_sens: Sequence[bool]):
        """Partition by magnitude and sensitivity (gradients given).  Returns (list of Quantized,
        list of (tau_outlier_sens, sse, sumsq))."""
        nT = len(tensors)
        ta = _tensor_array(tensors)
        ca = _config_array(cfgs)
        gp = (C.c_void_p * nT)(*[g.data_ptr() for g in grads])
        bs = (C.c_uint8 * nT)(*[1 if b else 0 for b in by_sens])
        qa = (CQuantized * nT)()
        info = (CSensInfo * nT)()
        res = QuantizedBatch()
        for i, (t, g, cfg) in enumerate(zip(tensors, grads, cfgs)):
            n = t.numel()
            if g.numel() != n or g.dtype != torch.float32 or not g.is_contiguous():
                raise ValueError("one contiguous float32 gradient per tensor, of its size")
            words, cap = self._bound(n, ca[i], cfg)
            cap = 2 * cap + 1  # either metric may protect its fraction
            e = qa[i]
            q = Quantized(n, int(cfg[0]), (
                torch.empty(words, dtype=torch.int64, device=t.device),
                torch.empty(256, dtype=torch.float32, device=t.device),
                torch.empty(255, dtype=torch.float32, device=t.device),
                torch.empty(cap, dtype=torch.int32, device=t.device),
                torch.empty(cap, dtype=torch.float32, device=t.device)), e, qa, bins=bins_of(cfg))
            e.packed, e.codebook, e.boundaries, e.outlier_idx, e.outlier_val = q._ptrs
            e.packed_words = q._bufs[0].numel()
            e.outlier_cap = cap
            res.append(q)
        res._qa = qa
        res._sizes = tuple(q.n for q in res)
        self._check(self.lib.inshr_quantize_sens(self.h, ta, gp, ca, bs, qa, info, nT))
        return res, [(float(i.tau_outlier_sens), float(i.sse), float(i.sumsq)) for i in info]

    # -- inshr_quantize_sketch -------------------------------------------------------------
    def quantize_sketch(self, tensors: Sequence[torch.Tensor], cfgs, uniforms, alpha: float = 0.01,
                        sigma: float = 0.2, max_iter: int = 100, reuse_search: bool = False,
                        out: Optional[List[Quantized]] = None):
        """uniforms: numpy float64 array [len(tensors), 256] of numbers in [0, 1).  Returns
        (list of Quantized, list of (n_buckets, rounds)).  `out` may carry the list an earlier call
        returned for tensors of the same sizes; its buffers are then written again (the C side
        checks them against what the configurations need)."""
        import numpy as np
        nT = len(tensors)
        ta = _tensor_array(tensors)
        ca = _config_array(cfgs)
        u = np.ascontiguousarray(uniforms, dtype=np.float64)
        if u.shape != (nT, 256):
            raise ValueError("uniforms must have shape [len(tensors), 256]")
        reuse_out = isinstance(out, QuantizedBatch) and out._sizes == tuple(t.numel() for t in tensors)
        qa = out._qa if reuse_out else (CQuantized * nT)()
        res = out if reuse_out else QuantizedBatch()
        for i, (t, cfg) in enumerate(zip(tensors, cfgs)):
            if reuse_out:
                break
            n = t.numel()
            words, cap = self._bound(n, ca[i], cfg)
            e = qa[i]
            q = Quantized(n, int(cfg[0]), (
                torch.empty(words, dtype=torch.int64, device=t.device),
                torch.empty(256, dtype=torch.float32, device=t.device),
                torch.empty(255, dtype=torch.float32, device=t.device),
                torch.empty(max(cap, 1), dtype=torch.int32, device=t.device),
                torch.empty(max(cap, 1), dtype=torch.float32, device=t.device)), e, qa)
            e.packed, e.codebook, e.boundaries, e.outlier_idx, e.outlier_val = q._ptrs
            e.packed_words = q._bufs[0].numel()
            e.outlier_cap = q._bufs[3].numel()
            res.append(q)
        if not reuse_out:
            res._qa = qa
            res._sizes = tuple(q.n for q in res)
        par = CSketchParams(float(alpha), float(sigma), int(max_iter), u.ctypes.data)
        info = (CSketchInfo * nT)()
        self._check(self.lib.inshr_quantize_sketch(self.h, ta, ca, C.byref(par), qa, info, nT,
                                                   INSHR_REUSE_SEARCH if reuse_search else 0))
        return res, [(int(i.n_buckets), int(i.rounds)) for i in info]

    # -- inshr_search_sketch ---------------------------------------------------------------
    def search_sketch(self, tensors: Sequence[torch.Tensor], cfgs, uniforms, eps: float,
                      alpha: float = 0.01, sigma: float = 0.2, max_iter: int = 100,
                      reuse_search: bool = False, out: Optional[List[Quantized]] = None):
        """cfgs: (ignored bits, prune_ppm, outlier_ppm) per tensor.  Returns (list of Quantized with
        the chosen bits, list of dict(best_bits, feasible, sse[7], sumsq, rounds[7]), list of
        (n_buckets, rounds of the widest set)).  `out` may carry the list an earlier call returned
        for tensors of the same sizes and protect fractions; its buffers are then written again."""
        import numpy as np
        nT = len(tensors)
        ta = _tensor_array(tensors)
        wide = [(8, int(c[1]), int(c[2])) for c in cfgs]
        ca = _config_array(wide)
        u = np.ascontiguousarray(uniforms, dtype=np.float64)
        if u.shape != (nT, 256):
            raise ValueError("uniforms must have shape [len(tensors), 256]")
        reuse_out = isinstance(out, QuantizedBatch) and out._sizes == tuple(t.numel() for t in tensors)
        qa = out._qa if reuse_out else (CQuantized * nT)()
        res = out if reuse_out else QuantizedBatch()
        for i, (t, cfg) in enumerate(zip(tensors, wide)):
            if reuse_out:
                break  # the C side checks every buffer against what the configuration needs
            n = t.numel()
            words, cap = self._bound(n, ca[i], cfg)
            e = qa[i]
            q = Quantized(n, 8, (
                torch.empty(words, dtype=torch.int64, device=t.device),
                torch.empty(256, dtype=torch.float32, device=t.device),
                torch.empty(255, dtype=torch.float32, device=t.device),
                torch.empty(max(cap, 1), dtype=torch.int32, device=t.device),
                torch.empty(max(cap, 1), dtype=torch.float32, device=t.device)), e, qa)
            e.packed, e.codebook, e.boundaries, e.outlier_idx, e.outlier_val = q._ptrs
            e.packed_words = q._bufs[0].numel()
            e.outlier_cap = q._bufs[3].numel()
            res.append(q)
        if not reuse_out:
            res._qa = qa
            res._sizes = tuple(q.n for q in res)
        par = CSketchParams(float(alpha), float(sigma), int(max_iter), u.ctypes.data)
        info = (CSketchInfo * nT)()
        choice = (CSketchChoice * nT)()
        self._check(self.lib.inshr_search_sketch(self.h, ta, ca, C.byref(par), float(eps), qa, choice, info,
                                                 nT, INSHR_REUSE_SEARCH if reuse_search else 0))
        choices = [dict(best_bits=int(c.best_bits), feasible=bool(c.feasible), sse=list(c.sse),
                        sumsq=float(c.sumsq), rounds=list(c.rounds)) for c in choice]
        return res, choices, [(int(i.n_buckets), int(i.rounds)) for i in info]

    # -- inshr_search_sketch_grid ----------------------------------------------------------
    def search_sketch_grid(self, tensors: Sequence[torch.Tensor], pairs, uniforms, eps: float,
                           alpha: float = 0.01, sigma: float = 0.2, max_iter: int = 100):
        """pairs: (prune_ppm, outlier_ppm) tuples.  Returns (list of Quantized of the winners, list
        of winning pair indices, list of dicts of the winners' rows, table[t][q] of dicts)."""
        import numpy as np
        nT, nP = len(tensors), len(pairs)
        ta = _tensor_array(tensors)
        pa = _config_array([(8, int(p), int(o)) for p, o in pairs])
        u = np.ascontiguousarray(uniforms, dtype=np.float64)
        if u.shape != (nT, 256):
            raise ValueError("uniforms must have shape [len(tensors), 256]")
        o_max = max(int(o) for _, o in pairs)
        qa = (CQuantized * nT)()
        res = QuantizedBatch()
        for i, t in enumerate(tensors):
            n = t.numel()
            wide = (8, 0, o_max)
            words, cap = self._bound(n, _config_array([wide])[0], wide)
            e = qa[i]
            q = Quantized(n, 8, (
                torch.empty(words, dtype=torch.int64, device=t.device),
                torch.empty(256, dtype=torch.float32, device=t.device),
                torch.empty(255, dtype=torch.float32, device=t.device),
                torch.empty(max(cap, 1), dtype=torch.int32, device=t.device),
                torch.empty(max(cap, 1), dtype=torch.float32, device=t.device)), e, qa)
            e.packed, e.codebook, e.boundaries, e.outlier_idx, e.outlier_val = q._ptrs
            e.packed_words = q._bufs[0].numel()
            e.outlier_cap = q._bufs[3].numel()
            res.append(q)
        res._qa = qa
        res._sizes = tuple(q.n for q in res)
        par = CSketchParams(float(alpha), float(sigma), int(max_iter), u.ctypes.data)
        best = (C.c_uint32 * nT)()
        choice = (CSketchChoice * nT)()
        table = (CSketchChoice * (nT * nP))()
        self._check(self.lib.inshr_search_sketch_grid(self.h, ta, pa, nP, C.byref(par), float(eps), qa, best,
                                                      choice, table, nT))
        row = lambda c: dict(best_bits=int(c.best_bits), feasible=bool(c.feasible), sse=list(c.sse),
                             sumsq=float(c.sumsq), rounds=list(c.rounds))
        return (res, list(best), [row(c) for c in choice],
                [[row(table[t * nP + q]) for q in range(nP)] for t in range(nT)])

    def _bound(self, n, ccfg, cfg):
        key = (n, bins_of(cfg), int(cfg[1]), int(cfg[2]))
        hit = self._bounds.get(key)
        if hit is None:
            words, cap = C.c_uint64(), C.c_uint64()
            self._check(self.lib.inshr_quantize_bound(n, C.byref(ccfg), C.byref(words), C.byref(cap)))
            hit = self._bounds[key] = (words.value, cap.value)
        return hit

    # -- inshr_delta ----------------------------------------------------------------------
    def delta(self, prev: Sequence[Quantized], cur: Sequence[Quantized], want_perm: bool = False,
              prev_perm: Optional[Sequence[Optional[torch.Tensor]]] = None,
              out: Optional[List[Delta]] = None) -> List[Delta]:
        """Enqueues the delta of every (prev[i], cur[i]); call sync() before reading on the host.
        `out` may carry the list a previous call returned for the same shapes; with the same prev
        and cur lists as in that call only the symbol widths are marshalled again."""
        nT = len(prev)
        if (isinstance(out, DeltaBatch) and out._prev is prev and out._cur is cur and prev_perm is None
                and not want_perm):
            pa, ca, oa = out._pa, out._ca, out._oa
            for i in range(nT):
                pa[i].sym_bits, pa[i].bins = prev[i]._c.sym_bits, prev[i]._c.n_bins
                ca[i].sym_bits, ca[i].bins = cur[i]._c.sym_bits, cur[i]._c.n_bins
                if out[i].group_off.numel() != pa[i].bins + 3:  # prev was quantized again with other bins
                    out[i].group_off = out[i].goff_buf[:pa[i].bins + 3]
            self._check(self.lib.inshr_delta(self.h, pa, None, ca, oa, nT))
            for i in range(nT):
                out[i].delta_bits = int(oa[i].delta_bits)
            return out
        pa = (CCodes * nT)()
        ca = (CCodes * nT)()
        oa = (CDeltaOut * nT)()
        pp = (C.c_void_p * nT)() if prev_perm is not None else None
        res = DeltaBatch()
        for i, (p, c) in enumerate(zip(prev, cur)):
            pa[i] = CCodes(p._ptrs[0], p.sym_bits, 0, p.K, p.n)
            ca[i] = CCodes(c._ptrs[0], c.sym_bits, 0, c.K, c.n)
            key = (p.n, p.K, c.n, c.K)
            need = self._bounds.get(key)
            if need is None:
                words = C.c_uint64()
                self._check(self.lib.inshr_delta_bound(C.byref(pa[i]), C.byref(ca[i]), C.byref(words)))
                need = self._bounds[key] = words.value
            if out is not None:
                d = out[i]
            else:
                dev = p._bufs[0].device
                d = Delta(n=p.n, delta_bits=symbol_bits(max(p.K, c.K)),
                          packed=torch.empty(need, dtype=torch.int64, device=dev),
                          group_off=None, goff_buf=None,
                          perm=torch.empty(p.n, dtype=torch.int32, device=dev) if want_perm else None)
            if d.packed.numel() < need:
                raise ValueError("pre-allocated delta buffer is too small")
            if d.goff_buf is None or d.goff_buf.numel() < GROUP_OFF_ENTRIES:
                d.goff_buf = torch.empty(GROUP_OFF_ENTRIES, dtype=torch.int64, device=d.packed.device)
            d.group_off = d.goff_buf[:p.K + 3]
            oa[i].packed = d.packed.data_ptr()
            oa[i].packed_words = d.packed.numel()
            oa[i].group_off = d.goff_buf.data_ptr()
            oa[i].group_off_entries = d.goff_buf.numel()
            oa[i].perm = d.perm.data_ptr() if d.perm is not None else None
            if pp is not None:
                pp[i] = prev_perm[i].data_ptr() if prev_perm[i] is not None else None
            res.append(d)
        self._check(self.lib.inshr_delta(self.h, pa, pp, ca, oa, nT))
        for i in range(nT):
            res[i].delta_bits = int(oa[i].delta_bits)
        res._pa, res._ca, res._oa, res._prev, res._cur = pa, ca, oa, prev, cur
        return res

    def delta_static(self, prev: Sequence[Quantized], cur: Sequence[Quantized], out: List[Delta]) -> List[Delta]:
        """inshr_delta_static into the buffers of `out` (a list inshr_delta's binding returned for
        the same shapes): the library allocates nothing, and neither does this method on the device."""
        nT = len(prev)
        pa = (CCodes * nT)()
        ca = (CCodes * nT)()
        oa = (CDeltaOut * nT)()
        for i, (p, c, d) in enumerate(zip(prev, cur, out)):
            pa[i] = CCodes(p._ptrs[0], p.sym_bits, 0, p.K, p.n)
            ca[i] = CCodes(c._ptrs[0], c.sym_bits, 0, c.K, c.n)
            oa[i].packed = d.packed.data_ptr()
            oa[i].packed_words = d.packed.numel()
            oa[i].group_off = d.goff_buf.data_ptr()
            oa[i].group_off_entries = d.goff_buf.numel()
            oa[i].perm = d.perm.data_ptr() if d.perm is not None else None
        self._check(self.lib.inshr_delta_static(self.h, pa, ca, oa, nT))
        for i in range(nT):
            out[i].delta_bits = int(oa[i].delta_bits)
            out[i].group_off = out[i].goff_buf[:prev[i].K + 3]
        return out

    # -- inshr_dequantize -----------------------------------------------------------------
    def dequantize(self, qs: Sequence[Quantized],
                   out: Optional[Sequence[torch.Tensor]] = None) -> List[torch.Tensor]:
        """fp32 tensors decoded from the quantized form; returns after the work has completed."""
        nT = len(qs)
        ia = (CDequantIn * nT)()
        oa = (C.c_void_p * nT)()
        res = []
        for i, q in enumerate(qs):
            ia[i] = CDequantIn(q._ptrs[0], q._ptrs[1], q._ptrs[3], q._ptrs[4], q.n_outlier, q.n, 0,
                               1 if q.bf16 else 0, q.K)
            x = out[i] if out is not None else torch.empty(q.n, dtype=torch.float32,
                                                           device=q._bufs[0].device)
            if x.dtype != torch.float32 or x.numel() != q.n or not x.is_contiguous():
                raise ValueError("output must be a contiguous float32 tensor of n elements")
            oa[i] = x.data_ptr()
            res.append(x)
        self._check(self.lib.inshr_dequantize(self.h, ia, oa, nT))
        return res

    # -- inshr_reconstruct ----------------------------------------------------------------
    def reconstruct(self, prev: Sequence[Quantized], deltas: Sequence[Delta],
                    bits_cur: Sequence[int], bins_cur: Optional[Sequence[int]] = None) -> List[torch.Tensor]:
        """Packed symbols (int64 words) of the current checkpoint from the previous codes and the
        delta streams; returns after the work has completed.  bins_cur: the numbers of bins of the
        current checkpoint where they are not 2^bits."""
        nT = len(prev)
        pa = (CCodes * nT)()
        da = (CDeltaOut * nT)()
        ca = (CCodesOut * nT)()
        res = []
        for i, (p, d) in enumerate(zip(prev, deltas)):
            pa[i] = CCodes(p._ptrs[0], p.sym_bits, 0, p.K, p.n)
            Kc = int(bins_cur[i]) if bins_cur is not None and bins_cur[i] else 1 << int(bits_cur[i])
            da[i].packed = d.packed.data_ptr()
            da[i].packed_words = d.packed.numel()
            da[i].group_off = d.group_off.data_ptr() if d.group_off is not None else None
            da[i].perm = None
            da[i].delta_bits = d.delta_bits
            words = (p.n * symbol_bits(Kc) + 63) // 64
            w = torch.empty(words, dtype=torch.int64, device=p._bufs[0].device)
            ca[i] = CCodesOut(w.data_ptr(), words, 0, Kc)
            res.append(w)
        self._check(self.lib.inshr_reconstruct(self.h, pa, da, ca, nT))
        return res


# -- entropy stage of the delta: host memory, no device involved ------------------------------------
def sketch_buckets(alpha: float):
    """(i_lo, tops float32 array, values float64 array) of the bucket law for alpha (host only)."""
    import numpy as np
    lib = load_library()
    i_lo, n = C.c_int32(), C.c_uint32()
    rc = lib.inshr_sketch_buckets(float(alpha), C.byref(i_lo), C.byref(n), None, None, 0)
    if rc:
        raise InshrError(rc, lib.inshr_strerror(rc).decode())
    tops = np.empty(n.value, np.float32)
    values = np.empty(n.value, np.float64)
    rc = lib.inshr_sketch_buckets(float(alpha), C.byref(i_lo), C.byref(n), tops.ctypes.data, values.ctypes.data,
                                  n.value)
    if rc:
        raise InshrError(rc, lib.inshr_strerror(rc).decode())
    return int(i_lo.value), tops, values


def _host_ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def entropy_encode(group_off, delta_bits: int, packed=None, values=None):
    """Container bytes (numpy uint8) and (n_tokens, table_bytes, payload_bytes) for a delta stream in
    host memory: `packed` (numpy uint64 words as inshr_delta wrote them) or `values` (numpy uint16)."""
    import numpy as np
    lib = load_library()
    group_off = np.ascontiguousarray(group_off, dtype=np.uint64)
    n, n_groups = int(group_off[-1]), group_off.size - 1
    if packed is not None:
        packed = np.ascontiguousarray(packed, dtype=np.uint64)
    if values is not None:
        values = np.ascontiguousarray(values, dtype=np.uint16)
    stats, size = CEntropyStats(), C.c_uint64()
    out = np.empty(max(64, n // 4), dtype=np.uint8)
    for _ in range(2):
        rc = lib.inshr_entropy_encode(_host_ptr(packed), _host_ptr(values), n, delta_bits,
                                      _host_ptr(group_off), n_groups, _host_ptr(out), out.size,
                                      C.byref(size), C.byref(stats))
        if rc != -4:
            break
        out = np.empty(size.value, dtype=np.uint8)
    if rc:
        raise InshrError(rc, lib.inshr_strerror(rc).decode())
    return out[:size.value], (stats.n_tokens, stats.table_bytes, stats.payload_bytes)


def entropy_decode(data, n: int, delta_bits: int, n_groups: int, as_values: bool = False):
    """(stream, group_off): the stream as packed uint64 words, or as uint16 values."""
    import numpy as np
    lib = load_library()
    data = np.ascontiguousarray(data, dtype=np.uint8)
    goff = np.empty(n_groups + 1, dtype=np.uint64)
    packed = None if as_values else np.empty((n * delta_bits + 63) // 64, dtype=np.uint64)
    values = np.empty(n, dtype=np.uint16) if as_values else None
    rc = lib.inshr_entropy_decode(_host_ptr(data), data.size, n, delta_bits, n_groups,
                                  _host_ptr(packed), _host_ptr(values), _host_ptr(goff))
    if rc:
        raise InshrError(rc, lib.inshr_strerror(rc).decode())
    return (values if as_values else packed), goff
