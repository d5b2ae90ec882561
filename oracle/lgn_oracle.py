"""ctypes front end of the C oracle (`lgn_oracle.c`) -- TEST INFRASTRUCTURE ONLY.

Argument marshalling only: every number comes out of the C file, which states the passage of
the paper each function follows.  Tensors are numpy arrays: float32 for fp32 data, uint16 bit
patterns for bf16 data.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lgn_oracle.c")
_LIB = os.path.join(_HERE, "liblgn_oracle.so")

F32, BF16, F16 = 0, 1, 2
ROUND_NEAREST_EVEN, ROUND_STOCHASTIC = 0, 1
OUT_VALUE, OUT_CODE8, OUT_PACKED = 0, 1, 2
SCALE_QUANTILE, SCALE_MAX, SCALE_CENTER = 0, 1, 2
SIGMA_PAPER_LITERAL, SIGMA_BASE2 = 0, 1
ST_EMPTY, ST_SIGMA0, ST_NOTHING_TO_PRUNE, ST_NOT_CONVERGED = 1, 2, 4, 8
ST_ALPHA_BELOW_FP_RANGE, ST_HAS_NONFINITE = 16, 32


class Stats(C.Structure):
    _fields_ = [("n", C.c_uint64), ("nnz", C.c_uint64), ("n_nonfinite", C.c_uint64),
                ("mu", C.c_double), ("sigma", C.c_double),
                ("max_abs", C.c_float), ("min_abs_nz", C.c_float), ("status", C.c_uint32)]


class PruneParams(C.Structure):
    _fields_ = [("alpha", C.c_float), ("s_eff", C.c_double), ("s_pred", C.c_double),
                ("status", C.c_uint32)]


class FpParams(C.Structure):
    _fields_ = [("n_bits", C.c_int32), ("e_bits", C.c_int32), ("m_bits", C.c_int32),
                ("scale_exp", C.c_int32), ("eta", C.c_double), ("status", C.c_uint32)]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C11, -O2, OpenMP for the element loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-D_GNU_SOURCE", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        vp, u64, i32, dbl, f32, u32 = C.c_void_p, C.c_uint64, C.c_int, C.c_double, C.c_float, C.c_uint32
        L.orc_set_threads.argtypes = [i32]
        L.orc_get_threads.restype = i32
        L.orc_max_threads.restype = i32
        L.orc_stats.argtypes = [vp, u64, i32, C.POINTER(Stats)]
        L.orc_stats_masked.argtypes = [vp, vp, u64, i32, i32, C.POINTER(Stats)]
        L.orc_sparsity_of_alpha.argtypes = [dbl, dbl, dbl]
        L.orc_sparsity_of_alpha.restype = dbl
        L.orc_sparsity_of_log_alpha.argtypes = [dbl, dbl, dbl]
        L.orc_sparsity_of_log_alpha.restype = dbl
        L.orc_normal_quantile.argtypes = [dbl]
        L.orc_normal_quantile.restype = dbl
        L.orc_threshold.argtypes = [C.POINTER(Stats), dbl, i32, C.POINTER(PruneParams)]
        L.orc_expected_relative_error.argtypes = [dbl, i32, i32]
        L.orc_expected_relative_error.restype = dbl
        L.orc_fp_params.argtypes = [C.POINTER(Stats), i32, i32, i32, dbl, i32, C.POINTER(FpParams)]
        L.orc_philox4x32_10.argtypes = [C.POINTER(u32), C.POINTER(u32), C.POINTER(u32)]
        L.orc_random_word.argtypes = [u64, u64]
        L.orc_random_word.restype = u32
        L.orc_prune.argtypes = [vp, u64, i32, f32, u64, u64, vp]
        L.orc_decode.argtypes = [u32, i32, i32, i32]
        L.orc_decode.restype = dbl
        L.orc_packed_bytes.argtypes = [u64, i32]
        L.orc_packed_bytes.restype = u64
        L.orc_pack.argtypes = [vp, u64, i32, vp]
        L.orc_unpack.argtypes = [vp, u64, i32, vp]
        L.orc_fp_quantize.argtypes = [vp, u64, i32, i32, i32, i32, i32, u64, u64, vp, i32, vp]
        L.orc_prune_quantize.argtypes = [vp, u64, i32, f32, i32, i32, i32, i32, u64, u64, vp, i32, vp]
        L.orc_dequantize.argtypes = [vp, u64, i32, i32, i32, i32, vp]
        L.orc_quantize_one.argtypes = [f32, i32, i32, i32, i32, u32]
        L.orc_quantize_one.restype = u32
        L.orc_prune_one.argtypes = [f32, f32, u32]
        L.orc_prune_one.restype = f32
        L.orc_cosine_similarity.argtypes = [dbl, dbl, dbl]
        L.orc_cosine_similarity.restype = dbl
        L.orc_log_alpha_for_cosine.argtypes = [dbl, dbl, dbl]
        L.orc_log_alpha_for_cosine.restype = dbl
        L.orc_log_histogram.argtypes = [vp, u64, i32, vp]
        L.orc_truncation_k.argtypes = [vp, dbl, dbl, dbl]
        L.orc_truncation_k.restype = dbl
        L.orc_sparsity_allocate.argtypes = [vp, vp, i32, dbl, i32, vp, dbl, dbl, i32, vp, vp]
        L.orc_f16_to_float.argtypes = [C.c_uint16]
        L.orc_f16_to_float.restype = f32
        L.orc_float_to_f16.argtypes = [f32]
        L.orc_float_to_f16.restype = C.c_uint16
        L.orc_threshold_floor.argtypes = [i32, i32, vp, i32, vp]
        L.orc_alpha_below_fp_range.argtypes = [f32, i32, i32]
        L.orc_alpha_below_fp_range.restype = i32
        L.orc_prefix_chunks.argtypes = [u64]
        L.orc_prefix_chunks.restype = u64
        L.orc_prefix_bound_bytes.argtypes = [u64, i32]
        L.orc_prefix_bound_bytes.restype = u64
        L.orc_prefix_encode.argtypes = [vp, u64, i32, u32, vp, vp, vp]
        L.orc_prefix_encode.restype = u64
        L.orc_prefix_decode.argtypes = [vp, vp, u64, i32, u32, vp]
        L.orc_prefix_decode_sub.argtypes = [vp, vp, vp, u64, i32, u32, vp]
        _lib = L
    return _lib


def set_threads(t: int) -> None:
    lib().orc_set_threads(int(t))


def max_threads() -> int:
    return int(lib().orc_max_threads())


def _dtype_of(g: np.ndarray) -> int:
    if g.dtype == np.float32:
        return F32
    if g.dtype == np.uint16:
        return BF16
    if g.dtype == np.float16:
        return F16
    raise TypeError("oracle tensors are float32 (fp32), uint16 bit patterns (bf16) or float16 (fp16)")


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def stats(g: np.ndarray) -> Stats:
    g = np.ascontiguousarray(g).reshape(-1)
    st = Stats()
    lib().orc_stats(_ptr(g), g.size, _dtype_of(g), C.byref(st))
    return st


MASK_NONE, MASK_SAME_DTYPE, MASK_U8 = 0, 1, 2


def stats_masked(g: np.ndarray, mask: np.ndarray) -> Stats:
    """Statistics over the entries of g whose mask entry is non-zero (the right mode of a bi-modal
    gradient); the mask has g's dtype or is one byte per element."""
    g = np.ascontiguousarray(g).reshape(-1)
    mask = np.ascontiguousarray(mask).reshape(-1)
    assert mask.size == g.size
    kind = MASK_U8 if mask.dtype == np.uint8 else MASK_SAME_DTYPE
    assert kind == MASK_U8 or mask.dtype == g.dtype
    st = Stats()
    lib().orc_stats_masked(_ptr(g), _ptr(mask), g.size, _dtype_of(g), kind, C.byref(st))
    return st


def make_stats(n, nnz, mu, sigma, max_abs=0.0, min_abs_nz=0.0, n_nonfinite=0, status=0) -> Stats:
    return Stats(int(n), int(nnz), int(n_nonfinite), float(mu), float(sigma), float(max_abs),
                 float(min_abs_nz), int(status))


def sparsity_of_alpha(mu, sigma, alpha) -> float:
    return float(lib().orc_sparsity_of_alpha(mu, sigma, alpha))


def normal_quantile(q) -> float:
    return float(lib().orc_normal_quantile(q))


def threshold(st: Stats, target_sparsity: float, alpha_dtype: int = F32) -> PruneParams:
    p = PruneParams()
    lib().orc_threshold(C.byref(st), float(target_sparsity), int(alpha_dtype), C.byref(p))
    return p


def expected_relative_error(sigma, e_bits, m_bits) -> float:
    return float(lib().orc_expected_relative_error(float(sigma), int(e_bits), int(m_bits)))


def fp_params(st: Stats, n_bits: int, e_bits: int = -1, scale_mode: int = SCALE_QUANTILE,
              scale_arg: float = 0.997, sigma_units: int = SIGMA_PAPER_LITERAL) -> FpParams:
    f = FpParams()
    lib().orc_fp_params(C.byref(st), int(n_bits), int(e_bits), int(scale_mode), float(scale_arg),
                        int(sigma_units), C.byref(f))
    return f


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def random_word(seed, j) -> int:
    return int(lib().orc_random_word(int(seed), int(j)))


def prune(g: np.ndarray, alpha: float, seed: int, elem_offset: int = 0) -> np.ndarray:
    g = np.ascontiguousarray(g).reshape(-1)
    out = np.empty_like(g)
    lib().orc_prune(_ptr(g), g.size, _dtype_of(g), np.float32(alpha), int(seed), int(elem_offset),
                    _ptr(out))
    return out


def packed_bytes(n, n_bits) -> int:
    return int(lib().orc_packed_bytes(int(n), int(n_bits)))


def pack(codes: np.ndarray, n_bits: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8).reshape(-1)
    out = np.empty(packed_bytes(codes.size, n_bits), dtype=np.uint8)
    lib().orc_pack(_ptr(codes), codes.size, int(n_bits), _ptr(out))
    return out


def unpack(packed: np.ndarray, n: int, n_bits: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8).reshape(-1)
    out = np.empty(int(n), dtype=np.uint8)
    lib().orc_unpack(_ptr(packed), int(n), int(n_bits), _ptr(out))
    return out


def _alloc_out(g, out_kind, n_bits):
    if out_kind == OUT_VALUE:
        return np.empty_like(g), None
    if out_kind == OUT_CODE8:
        return np.empty(g.size, dtype=np.uint8), None
    return (np.empty(packed_bytes(g.size, n_bits), dtype=np.uint8),
            np.empty(g.size, dtype=np.uint8))


def fp_quantize(g: np.ndarray, e: int, m: int, s: int, rounding: int = ROUND_NEAREST_EVEN,
                seed: int = 0, elem_offset: int = 0, out_kind: int = OUT_VALUE) -> np.ndarray:
    g = np.ascontiguousarray(g).reshape(-1)
    out, scratch = _alloc_out(g, out_kind, 1 + e + m)
    lib().orc_fp_quantize(_ptr(g), g.size, _dtype_of(g), int(e), int(m), int(s), int(rounding),
                          int(seed), int(elem_offset), _ptr(out), int(out_kind),
                          _ptr(scratch) if scratch is not None else None)
    return out


def prune_quantize(g: np.ndarray, alpha: float, e: int, m: int, s: int,
                   rounding: int = ROUND_NEAREST_EVEN, seed: int = 0, elem_offset: int = 0,
                   out_kind: int = OUT_VALUE) -> np.ndarray:
    g = np.ascontiguousarray(g).reshape(-1)
    out, scratch = _alloc_out(g, out_kind, 1 + e + m)
    lib().orc_prune_quantize(_ptr(g), g.size, _dtype_of(g), np.float32(alpha), int(e), int(m),
                             int(s), int(rounding), int(seed), int(elem_offset), _ptr(out),
                             int(out_kind), _ptr(scratch) if scratch is not None else None)
    return out


def decode(code: int, e: int, m: int, s: int) -> float:
    return float(lib().orc_decode(int(code), int(e), int(m), int(s)))


def dequantize(codes: np.ndarray, e: int, m: int, s: int, dtype: int = F32) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8).reshape(-1)
    out = np.empty(codes.size, dtype={F32: np.float32, BF16: np.uint16, F16: np.float16}[dtype])
    lib().orc_dequantize(_ptr(codes), codes.size, int(e), int(m), int(s), int(dtype), _ptr(out))
    return out


def quantize_one(x, e, m, s, rounding=ROUND_NEAREST_EVEN, w=0) -> int:
    return int(lib().orc_quantize_one(np.float32(x), int(e), int(m), int(s), int(rounding),
                                      int(w) & 0xFFFFFFFF))


def prune_one(x, alpha, w) -> float:
    return float(lib().orc_prune_one(np.float32(x), np.float32(alpha), int(w) & 0xFFFFFFFF))


# ---- prefix code of the pruned tensor (appendix "Encoding") ----------------------------------
PREFIX_CHUNK = 4096


def _raw_view(a: np.ndarray, width: int) -> np.ndarray:
    a = np.ascontiguousarray(a).reshape(-1)
    if width == 32:
        return a.view(np.uint32)
    if width == 16:
        return a.view(np.uint16)
    return a.view(np.uint8)


def prefix_width(a: np.ndarray, n_bits: int = None) -> int:
    """Bits of an element's pattern: 32 (fp32), 16 (bf16 bit patterns) or N (FP-n codes)."""
    if a.dtype == np.float32:
        return 32
    if a.dtype in (np.uint16, np.float16):
        return 16
    assert a.dtype == np.uint8 and n_bits is not None
    return int(n_bits)


def prefix_special_of_alpha(alpha: float, width: int, fp16: bool = False) -> int:
    """Magnitude pattern of alpha as an fp32 (width 32), bf16 or fp16 (width 16) value."""
    if fp16:
        return int(np.float16(alpha).view(np.uint16)) & 0x7FFF
    b = int(np.float32(alpha).view(np.uint32)) & 0x7FFFFFFF
    return b if width == 32 else b >> 16


def prefix_special_of_code(alpha: float, e: int, m: int, s: int) -> int:
    """Magnitude code that alpha quantizes to with nearest rounding."""
    return quantize_one(abs(float(alpha)), e, m, s, ROUND_NEAREST_EVEN) & ((1 << (e + m)) - 1)


def prefix_bound_bytes(n: int, width: int) -> int:
    return int(lib().orc_prefix_bound_bytes(int(n), int(width)))


def prefix_encode(a: np.ndarray, special: int, n_bits: int = None, with_sub: bool = False):
    """Returns (stream bytes, table) for the prefix code, with with_sub also the bit lengths of the
    sub-blocks of 256 elements (16 per chunk); see orc_prefix_encode."""
    width = prefix_width(a, n_bits)
    raw = _raw_view(a, width)
    nchunks = int(lib().orc_prefix_chunks(raw.size))
    table = np.zeros(nchunks + 2, dtype=np.uint64)
    sub = np.zeros(16 * nchunks, dtype=np.uint16)
    nbytes = int(lib().orc_prefix_encode(_ptr(raw), raw.size, width, int(special), None, _ptr(table), None))
    stream = np.zeros(nbytes, dtype=np.uint8)
    lib().orc_prefix_encode(_ptr(raw), raw.size, width, int(special), _ptr(stream), _ptr(table),
                            _ptr(sub) if nchunks else None)
    return (stream, table, sub) if with_sub else (stream, table)


def prefix_decode_sub(stream: np.ndarray, table: np.ndarray, sub: np.ndarray, n: int, width: int,
                      special: int) -> np.ndarray:
    """Decodes sub-block by sub-block, each from the position the sub-block lengths give."""
    stream = np.ascontiguousarray(stream, dtype=np.uint8)
    table = np.ascontiguousarray(table, dtype=np.uint64)
    sub = np.ascontiguousarray(sub, dtype=np.uint16)
    out = np.empty(n, dtype={32: np.uint32, 16: np.uint16}.get(width, np.uint8))
    lib().orc_prefix_decode_sub(_ptr(stream), _ptr(table), _ptr(sub) if sub.size else None, int(n), int(width),
                                int(special), _ptr(out))
    return out


def prefix_decode(stream: np.ndarray, table: np.ndarray, n: int, width: int, special: int) -> np.ndarray:
    stream = np.ascontiguousarray(stream, dtype=np.uint8)
    table = np.ascontiguousarray(table, dtype=np.uint64)
    out = np.empty(n, dtype={32: np.uint32, 16: np.uint16}.get(width, np.uint8))
    lib().orc_prefix_decode(_ptr(stream), _ptr(table), int(n), int(width), int(special), _ptr(out))
    return out


# ---- cosine similarity of stochastic pruning, heterogeneous allocation -----------------------
HIST_BINS = 2048


class Alloc(C.Structure):
    _fields_ = [("sparsity", C.c_double), ("cosine", C.c_double), ("k", C.c_double),
                ("status", C.c_uint32), ("reserved", C.c_uint32)]


def cosine_similarity(sigma: float, log_alpha_rel: float, cutoff: float) -> float:
    """Closed-form cos(X, T(X)) for ln|x| - mu ~ N(0, sigma^2) truncated at `cutoff` above mu;
    log_alpha_rel = ln(alpha) - mu."""
    return float(lib().orc_cosine_similarity(float(sigma), float(log_alpha_rel), float(cutoff)))


def log_alpha_for_cosine(sigma: float, cutoff: float, min_cosine: float) -> float:
    return float(lib().orc_log_alpha_for_cosine(float(sigma), float(cutoff), float(min_cosine)))


def log_histogram(g: np.ndarray) -> np.ndarray:
    g = np.ascontiguousarray(g).reshape(-1)
    h = np.zeros(HIST_BINS, dtype=np.uint64)
    lib().orc_log_histogram(_ptr(g), g.size, _dtype_of(g), _ptr(h))
    return h


def truncation_k(hist, mu: float, sigma: float, q: float = 0.997) -> float:
    h = None if hist is None else _ptr(np.ascontiguousarray(hist, dtype=np.uint64))
    return float(lib().orc_truncation_k(h, float(mu), float(sigma), float(q)))


def sparsity_allocate(stats_list, hists, overall_sparsity: float, min_cosine, max_sparsity: float = 0.97,
                      quantile: float = 0.997, alpha_dtype: int = F32):
    """Layers deepest first; min_cosine has one entry per deep layer.  Returns (prune params, allocs)."""
    n = len(stats_list)
    st = (Stats * n)(*stats_list)
    mc = np.ascontiguousarray(min_cosine, dtype=np.float64)
    hs = None if hists is None else np.ascontiguousarray(hists, dtype=np.uint64).reshape(n, HIST_BINS)
    p = (PruneParams * n)()
    a = (Alloc * n)()
    lib().orc_sparsity_allocate(C.cast(st, C.c_void_p), _ptr(hs) if hs is not None else None, n,
                                float(overall_sparsity), int(mc.size), _ptr(mc) if mc.size else None,
                                float(max_sparsity), float(quantile), int(alpha_dtype),
                                C.cast(p, C.c_void_p), C.cast(a, C.c_void_p))
    return list(p), list(a)


def threshold_floor(e_bits: int, scale_exp: int, p_in: PruneParams = None, alpha_dtype: int = F32) -> PruneParams:
    """Pruning threshold raised to the format's smallest magnitude (stochastic underflow)."""
    out = PruneParams()
    lib().orc_threshold_floor(int(e_bits), int(scale_exp), C.byref(p_in) if p_in is not None else None,
                              int(alpha_dtype), C.byref(out))
    return out


def alpha_below_fp_range(alpha: float, e_bits: int, scale_exp: int) -> bool:
    """True if every survivor of pruning (+-alpha) would be flushed by the quantizer."""
    return bool(lib().orc_alpha_below_fp_range(np.float32(alpha), int(e_bits), int(scale_exp)))


def f16_to_float(h: int) -> float:
    return float(lib().orc_f16_to_float(int(h)))


def float_to_f16(x) -> int:
    return int(lib().orc_float_to_f16(np.float32(x)))
