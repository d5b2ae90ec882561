"""ctypes binding of `liblgn.so` (C interface: include/lgn.h).

Argument marshalling only.  Tensors are torch CUDA tensors (device memory), the parameter
structs live in device memory as small uint8 tensors, and every call is enqueued on torch's
current stream.  There is no CPU fallback: if the HIP library cannot be loaded the import of a
symbol fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from . import build as _build

# ---- constants of include/lgn.h ---------------------------------------------------------------
LGN_OK = 0
LGN_ERR_INVALID_ARG, LGN_ERR_UNSUPPORTED, LGN_ERR_WORKSPACE, LGN_ERR_DEVICE = -1, -2, -3, -4
LGN_F32, LGN_BF16, LGN_F16 = 0, 1, 2
LGN_ROUND_NEAREST_EVEN, LGN_ROUND_STOCHASTIC = 0, 1
LGN_OUT_VALUE, LGN_OUT_CODE8, LGN_OUT_PACKED = 0, 1, 2
LGN_SCALE_QUANTILE, LGN_SCALE_MAX, LGN_SCALE_CENTER = 0, 1, 2
LGN_SIGMA_PAPER_LITERAL, LGN_SIGMA_BASE2 = 0, 1
LGN_ST_EMPTY, LGN_ST_SIGMA0, LGN_ST_NOTHING_TO_PRUNE, LGN_ST_NOT_CONVERGED = 1, 2, 4, 8
LGN_ST_ALPHA_BELOW_FP_RANGE, LGN_ST_HAS_NONFINITE = 16, 32
LGN_PREFIX_CHUNK = 4096
LGN_PREFIX_SUB = 256
LGN_PREFIX_MAX_BLOCKS = 2048
LGN_MASK_NONE, LGN_MASK_SAME_DTYPE, LGN_MASK_U8 = 0, 1, 2
LGN_HIST_BINS = 2048
LGN_ALLOC_LOWERED, LGN_ALLOC_CAPPED = 1, 2
LGN_TUNE_STATS_KEEP_MB, LGN_TUNE_STATS_BLOCKS_PER_CU = 0, 1
LGN_TUNE_STREAM_PAIRS_PER_WAVE, LGN_TUNE_STREAM_BLOCKS_PER_CU = 2, 3
LGN_TUNE_STATS_STRICT_PUBLISH = 4


class LgnStats(C.Structure):
    _fields_ = [("n", C.c_uint64), ("nnz", C.c_uint64), ("n_nonfinite", C.c_uint64),
                ("mean_log2", C.c_double), ("m2_log2", C.c_double),
                ("mu", C.c_double), ("sigma", C.c_double),
                ("max_abs", C.c_float), ("min_abs_nz", C.c_float),
                ("status", C.c_uint32), ("reserved", C.c_uint32)]


class LgnPruneParams(C.Structure):
    _fields_ = [("alpha", C.c_float), ("status", C.c_uint32),
                ("s_eff", C.c_double), ("s_pred", C.c_double)]


class LgnFpParams(C.Structure):
    _fields_ = [("n_bits", C.c_int32), ("e_bits", C.c_int32), ("m_bits", C.c_int32),
                ("scale_exp", C.c_int32), ("eta", C.c_double),
                ("status", C.c_uint32), ("reserved", C.c_uint32)]


class LgnAlloc(C.Structure):
    _fields_ = [("sparsity", C.c_double), ("cosine", C.c_double), ("k", C.c_double),
                ("status", C.c_uint32), ("reserved", C.c_uint32)]


assert C.sizeof(LgnStats) == 72 and C.sizeof(LgnPruneParams) == 24 and C.sizeof(LgnFpParams) == 32
assert C.sizeof(LgnAlloc) == 32


class LgnBatchItem(C.Structure):
    _fields_ = [("g", C.c_void_p), ("out", C.c_void_p), ("n", C.c_uint64), ("seed", C.c_uint64),
                ("target_sparsity", C.c_double), ("n_bits", C.c_int32), ("e_bits", C.c_int32),
                ("st", C.c_void_p), ("p", C.c_void_p), ("f", C.c_void_p)]


assert C.sizeof(LgnBatchItem) == 72


class LgnError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"lgn error {code}: {text}")
        self.code = code


_lib = None

EXPORTS = ("lgn_workspace_bytes", "lgn_packed_bytes", "lgn_stats", "lgn_threshold",
           "lgn_fp_params", "lgn_prune", "lgn_fp_quantize", "lgn_prune_quantize_fused",
           "lgn_dequantize", "lgn_workspace_init", "lgn_stats_solve", "lgn_stats_masked", "lgn_prefix_encode",
           "lgn_prefix_decode", "lgn_log_histogram", "lgn_sparsity_allocate", "lgn_threshold_floor",
           "lgn_prefix_table_bytes", "lgn_prefix_bound_bytes", "lgn_set_tuning", "lgn_get_tuning",
           "lgn_stats_solve_static", "lgn_static_scratch_bytes",
           "lgn_batch_stats_solve", "lgn_batch_prune_quantize_fused",
           "lgn_last_error", "lgn_version")


def library_path() -> str:
    return _build.LIB


def load():
    """Load liblgn.so (building it first if it was never built).  Raises if that fails."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build(force=True)
    L = C.CDLL(_build.LIB)
    vp, u64, i32, dbl, sz = C.c_void_p, C.c_uint64, C.c_int, C.c_double, C.c_size_t
    L.lgn_workspace_bytes.argtypes = [u64, i32]
    L.lgn_workspace_bytes.restype = sz
    L.lgn_packed_bytes.argtypes = [u64, i32]
    L.lgn_packed_bytes.restype = sz
    L.lgn_stats.argtypes = [vp, u64, i32, vp, vp, sz, vp]
    L.lgn_threshold.argtypes = [vp, dbl, i32, vp, vp]
    L.lgn_fp_params.argtypes = [vp, i32, i32, i32, dbl, i32, vp, vp]
    L.lgn_prune.argtypes = [vp, u64, i32, vp, u64, u64, vp, vp]
    L.lgn_fp_quantize.argtypes = [vp, u64, i32, vp, i32, u64, u64, vp, i32, vp]
    L.lgn_prune_quantize_fused.argtypes = [vp, u64, i32, vp, vp, i32, u64, u64, vp, i32, vp]
    L.lgn_dequantize.argtypes = [vp, u64, i32, vp, i32, vp, vp]
    L.lgn_workspace_init.argtypes = [vp, sz, vp]
    L.lgn_stats_solve.argtypes = [vp, vp, i32, u64, i32, dbl, i32, i32, i32, i32, dbl, i32, vp, vp, vp, vp, sz, vp]
    L.lgn_stats_masked.argtypes = [vp, vp, i32, u64, i32, vp, vp, sz, vp]
    L.lgn_stats_solve_static.argtypes = [vp, vp, i32, u64, i32, dbl, i32, i32, i32, i32, dbl, i32, vp, vp, vp, vp]
    L.lgn_stats_solve_static.restype = i32
    L.lgn_static_scratch_bytes.restype = sz
    L.lgn_batch_stats_solve.argtypes = [vp, i32, i32, i32, i32, dbl, i32, vp, sz, vp]
    L.lgn_batch_stats_solve.restype = i32
    L.lgn_batch_prune_quantize_fused.argtypes = [vp, i32, i32, i32, i32, vp]
    L.lgn_batch_prune_quantize_fused.restype = i32
    L.lgn_last_error.restype = C.c_char_p
    L.lgn_version.restype = i32
    L.lgn_prefix_encode.argtypes = [vp, u64, i32, i32, vp, vp, vp, sz, vp, vp]
    L.lgn_prefix_decode.argtypes = [vp, vp, u64, i32, i32, vp, vp, vp, vp]
    L.lgn_prefix_table_bytes.argtypes = [u64]
    L.lgn_prefix_table_bytes.restype = sz
    L.lgn_prefix_bound_bytes.argtypes = [u64, i32]
    L.lgn_prefix_bound_bytes.restype = sz
    L.lgn_log_histogram.argtypes = [vp, u64, i32, vp, vp]
    L.lgn_sparsity_allocate.argtypes = [vp, vp, i32, dbl, i32, vp, dbl, dbl, i32, vp, vp, vp]
    L.lgn_threshold_floor.argtypes = [vp, vp, vp, vp]
    L.lgn_set_tuning.argtypes = [i32, C.c_long]
    L.lgn_set_tuning.restype = i32
    L.lgn_get_tuning.argtypes = [i32]
    L.lgn_get_tuning.restype = C.c_long
    # every entry point that can fail returns an LGN_* code; the sizes, the error text, the version and
    # the knob getter are set above
    not_status = {"lgn_workspace_bytes", "lgn_packed_bytes", "lgn_prefix_table_bytes", "lgn_prefix_bound_bytes",
                  "lgn_static_scratch_bytes", "lgn_last_error", "lgn_version", "lgn_get_tuning"}
    for name in EXPORTS:
        if name not in not_status:
            getattr(L, name).restype = i32
    _lib = L
    return L


def _check(rc):
    if rc != LGN_OK:
        raise LgnError(rc, load().lgn_last_error().decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor, dtype=None) -> int:
    if dtype is not None:
        return int(dtype)
    if t.dtype == torch.float32:
        return LGN_F32
    if t.dtype in (torch.bfloat16, torch.int16, torch.uint16):
        return LGN_BF16  # 16-bit integer tensors are taken as bf16 bit patterns
    if t.dtype == torch.float16:
        return LGN_F16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _flat(t: torch.Tensor) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError("tensors must live in device memory")
    if not t.is_contiguous():
        raise ValueError("tensors must be contiguous")
    return t


def _struct_buf(size, device):
    return torch.empty(size, dtype=torch.uint8, device=device)


_ws_cache = {}


def workspace(device) -> torch.Tensor:
    """Scratch tensor for lgn_stats / lgn_stats_solve, one per (device, current stream): calls on
    different streams may overlap in time and must not share the per-block records and the ticket.
    Allocated by torch and prepared with lgn_workspace_init on that same stream, so the preparation
    is ordered before the first use."""
    dev = torch.device(device)
    index = dev.index if dev.index is not None else torch.cuda.current_device()
    with torch.cuda.device(index):
        key = (index, torch.cuda.current_stream().cuda_stream)
        ws = _ws_cache.get(key)
        if ws is None:
            ws = torch.empty(lgn_workspace_bytes(0, LGN_F32), dtype=torch.uint8, device=f"cuda:{index}")
            lgn_workspace_init(ws)
            _ws_cache[key] = ws
    return ws


# ---- same names as the C interface ------------------------------------------------------------
def lgn_version() -> int:
    return int(load().lgn_version())


def lgn_set_tuning(knob: int, value: int) -> None:
    _check(load().lgn_set_tuning(int(knob), int(value)))


def lgn_get_tuning(knob: int) -> int:
    return int(load().lgn_get_tuning(int(knob)))


def lgn_workspace_bytes(n: int, dtype: int) -> int:
    return int(load().lgn_workspace_bytes(int(n), int(dtype)))


def lgn_packed_bytes(n: int, n_bits: int) -> int:
    return int(load().lgn_packed_bytes(int(n), int(n_bits)))


def lgn_stats(g: torch.Tensor, out: torch.Tensor = None, ws: torch.Tensor = None, dtype=None) -> torch.Tensor:
    g = _flat(g)
    if out is None:
        out = _struct_buf(C.sizeof(LgnStats), g.device)
    if ws is None:
        ws = workspace(g.device)
    _check(load().lgn_stats(g.data_ptr(), g.numel(), _dtype_code(g, dtype), out.data_ptr(),
                            ws.data_ptr(), ws.numel(), _stream()))
    return out


def lgn_workspace_init(ws: torch.Tensor) -> None:
    with torch.cuda.device(ws.device):
        _check(load().lgn_workspace_init(ws.data_ptr(), ws.numel(), _stream()))


def _mask_args(g: torch.Tensor, mask):
    """(pointer, kind) of an optional mask: a uint8 tensor or a tensor of g's element size."""
    if mask is None:
        return None, LGN_MASK_NONE
    mask = _flat(mask)
    if mask.numel() != g.numel():
        raise ValueError("mask and tensor differ in size")
    if mask.dtype == torch.uint8:
        return mask.data_ptr(), LGN_MASK_U8
    if mask.element_size() != g.element_size():
        raise TypeError("a mask is one byte per element or a tensor of the same type")
    return mask.data_ptr(), LGN_MASK_SAME_DTYPE


def lgn_stats_masked(g: torch.Tensor, mask: torch.Tensor, out: torch.Tensor = None,
                     ws: torch.Tensor = None, dtype=None) -> torch.Tensor:
    g = _flat(g)
    if out is None:
        out = _struct_buf(C.sizeof(LgnStats), g.device)
    if ws is None:
        ws = workspace(g.device)
    mp, mk = _mask_args(g, mask)
    _check(load().lgn_stats_masked(g.data_ptr(), mp, mk, g.numel(), _dtype_code(g, dtype), out.data_ptr(),
                                   ws.data_ptr(), ws.numel(), _stream()))
    return out


def lgn_stats_solve(g: torch.Tensor, target_sparsity: float = -1.0, alpha_dtype: int = LGN_F32,
                    n_bits: int = 0, e_bits: int = -1, scale_mode: int = LGN_SCALE_QUANTILE,
                    scale_arg: float = 0.997, sigma_units: int = LGN_SIGMA_PAPER_LITERAL,
                    st: torch.Tensor = None, p: torch.Tensor = None, f: torch.Tensor = None,
                    ws: torch.Tensor = None, dtype=None, mask: torch.Tensor = None):
    """One launch for lgn_stats + lgn_threshold + lgn_fp_params; returns (st, p, f) buffers
    (p is None without a target sparsity, f is None without n_bits)."""
    g = _flat(g)
    if st is None:
        st = _struct_buf(C.sizeof(LgnStats), g.device)
    if p is None and target_sparsity >= 0.0:
        p = _struct_buf(C.sizeof(LgnPruneParams), g.device)
    if f is None and n_bits:
        f = _struct_buf(C.sizeof(LgnFpParams), g.device)
    if ws is None:
        ws = workspace(g.device)
    mp, mk = _mask_args(g, mask)
    _check(load().lgn_stats_solve(g.data_ptr(), mp, mk, g.numel(), _dtype_code(g, dtype), float(target_sparsity),
                                  int(alpha_dtype), int(n_bits), int(e_bits), int(scale_mode),
                                  float(scale_arg), int(sigma_units), st.data_ptr(),
                                  p.data_ptr() if p is not None else None,
                                  f.data_ptr() if f is not None else None,
                                  ws.data_ptr(), ws.numel(), _stream()))
    return st, p, f


LGN_STATIC_MAX_ELEMENTS = 1 << 40


def lgn_static_scratch_bytes() -> int:
    return int(load().lgn_static_scratch_bytes())


def lgn_stats_solve_static(g: torch.Tensor, st: torch.Tensor, p: torch.Tensor = None, f: torch.Tensor = None,
                           target_sparsity: float = -1.0, alpha_dtype: int = LGN_F32, n_bits: int = 0,
                           e_bits: int = -1, scale_mode: int = LGN_SCALE_QUANTILE, scale_arg: float = 0.997,
                           sigma_units: int = LGN_SIGMA_PAPER_LITERAL, dtype=None, mask: torch.Tensor = None,
                           n: int = None):
    """lgn_stats_solve on the library's built-in scratch array.  The output structs are the
    caller's (this wrapper allocates nothing either); `n` overrides the element count."""
    g = _flat(g)
    mp, mk = _mask_args(g, mask)
    _check(load().lgn_stats_solve_static(g.data_ptr(), mp, mk, g.numel() if n is None else int(n),
                                         _dtype_code(g, dtype), float(target_sparsity), int(alpha_dtype),
                                         int(n_bits), int(e_bits), int(scale_mode), float(scale_arg),
                                         int(sigma_units), st.data_ptr(),
                                         p.data_ptr() if p is not None else None,
                                         f.data_ptr() if f is not None else None, _stream()))
    return st, p, f


class Batch:
    """A host array of lgn_batch_item_t plus the tensors it points to (kept alive with it)."""

    def __init__(self, items, dtype, device):
        self.count = len(items)
        self.array = (LgnBatchItem * max(self.count, 1))()
        self.tensors = items
        self.dtype = dtype
        self.device = device
        for i, it in enumerate(items):
            a = self.array[i]
            a.g, a.out = it["g"].data_ptr(), it["out"].data_ptr() if it.get("out") is not None else None
            a.n, a.seed = it["g"].numel(), int(it.get("seed", 0))
            a.target_sparsity = float(it.get("target_sparsity", -1.0))
            a.n_bits, a.e_bits = int(it.get("n_bits", 0)), int(it.get("e_bits", -1))
            a.st = it["st"].data_ptr()
            a.p = it["p"].data_ptr() if it.get("p") is not None else None
            a.f = it["f"].data_ptr() if it.get("f") is not None else None


def make_batch(items, dtype=None) -> Batch:
    """items: dicts with g (tensor), st and optionally out, p, f (device buffers), target_sparsity,
    n_bits, e_bits, seed.  Marshals them into the host descriptor array of the batched calls."""
    if not items:
        return Batch([], LGN_F32 if dtype is None else dtype, None)
    for it in items:
        _flat(it["g"])
    dt = _dtype_code(items[0]["g"], dtype)
    return Batch(items, dt, items[0]["g"].device)


def lgn_batch_stats_solve(batch: Batch, alpha_dtype: int = None, scale_mode: int = LGN_SCALE_QUANTILE,
                          scale_arg: float = 0.997, sigma_units: int = LGN_SIGMA_PAPER_LITERAL,
                          ws: torch.Tensor = None) -> None:
    if ws is None:
        ws = workspace(batch.device if batch.device is not None else "cuda")
    if alpha_dtype is None:
        alpha_dtype = batch.dtype
    _check(load().lgn_batch_stats_solve(C.addressof(batch.array), batch.count, int(batch.dtype), int(alpha_dtype),
                                        int(scale_mode), float(scale_arg), int(sigma_units), ws.data_ptr(),
                                        ws.numel(), _stream()))


def lgn_batch_prune_quantize_fused(batch: Batch, rounding: int = LGN_ROUND_NEAREST_EVEN,
                                   out_kind: int = LGN_OUT_CODE8) -> None:
    _check(load().lgn_batch_prune_quantize_fused(C.addressof(batch.array), batch.count, int(batch.dtype),
                                                 int(rounding), int(out_kind), _stream()))


def lgn_threshold(st: torch.Tensor, target_sparsity: float, alpha_dtype: int = LGN_F32,
                  out: torch.Tensor = None) -> torch.Tensor:
    if out is None:
        out = _struct_buf(C.sizeof(LgnPruneParams), st.device)
    _check(load().lgn_threshold(st.data_ptr(), float(target_sparsity), int(alpha_dtype),
                                out.data_ptr(), _stream()))
    return out


def lgn_threshold_floor(f: torch.Tensor, p: torch.Tensor = None, out: torch.Tensor = None) -> torch.Tensor:
    if out is None:
        out = _struct_buf(C.sizeof(LgnPruneParams), f.device)
    _check(load().lgn_threshold_floor(f.data_ptr(), p.data_ptr() if p is not None else None,
                                      out.data_ptr(), _stream()))
    return out


def lgn_fp_params(st: torch.Tensor, n_bits: int, e_bits: int = -1,
                  scale_mode: int = LGN_SCALE_QUANTILE, scale_arg: float = 0.997,
                  sigma_units: int = LGN_SIGMA_PAPER_LITERAL, out: torch.Tensor = None) -> torch.Tensor:
    if out is None:
        out = _struct_buf(C.sizeof(LgnFpParams), st.device)
    _check(load().lgn_fp_params(st.data_ptr(), int(n_bits), int(e_bits), int(scale_mode),
                                float(scale_arg), int(sigma_units), out.data_ptr(), _stream()))
    return out


def lgn_prune(g: torch.Tensor, p: torch.Tensor, seed: int, elem_offset: int = 0,
              out: torch.Tensor = None, dtype=None) -> torch.Tensor:
    g = _flat(g)
    if out is None:
        out = torch.empty_like(g)
    _check(load().lgn_prune(g.data_ptr(), g.numel(), _dtype_code(g, dtype), p.data_ptr(),
                            int(seed), int(elem_offset), out.data_ptr(), _stream()))
    return out


def _alloc_quant_out(g, out_kind, n_bits):
    if out_kind == LGN_OUT_VALUE:
        return torch.empty_like(g)
    if out_kind == LGN_OUT_CODE8:
        return torch.empty(g.numel(), dtype=torch.uint8, device=g.device)
    if n_bits is None:
        raise ValueError("n_bits is needed to size a PACKED output")
    nbytes = lgn_packed_bytes(g.numel(), n_bits)
    return torch.empty(nbytes, dtype=torch.uint8, device=g.device)


def lgn_fp_quantize(g: torch.Tensor, f: torch.Tensor, rounding: int = LGN_ROUND_NEAREST_EVEN,
                    seed: int = 0, elem_offset: int = 0, out: torch.Tensor = None,
                    out_kind: int = LGN_OUT_VALUE, n_bits: int = None, dtype=None) -> torch.Tensor:
    g = _flat(g)
    if out is None:
        out = _alloc_quant_out(g, out_kind, n_bits)
    _check(load().lgn_fp_quantize(g.data_ptr(), g.numel(), _dtype_code(g, dtype), f.data_ptr(),
                                  int(rounding), int(seed), int(elem_offset), out.data_ptr(),
                                  int(out_kind), _stream()))
    return out


def lgn_prune_quantize_fused(g: torch.Tensor, p: torch.Tensor, f: torch.Tensor,
                             rounding: int = LGN_ROUND_NEAREST_EVEN, seed: int = 0,
                             elem_offset: int = 0, out: torch.Tensor = None,
                             out_kind: int = LGN_OUT_VALUE, n_bits: int = None, dtype=None) -> torch.Tensor:
    g = _flat(g)
    if out is None:
        out = _alloc_quant_out(g, out_kind, n_bits)
    _check(load().lgn_prune_quantize_fused(g.data_ptr(), g.numel(), _dtype_code(g, dtype),
                                           p.data_ptr(), f.data_ptr(), int(rounding), int(seed),
                                           int(elem_offset), out.data_ptr(), int(out_kind),
                                           _stream()))
    return out


def lgn_dequantize(codes: torch.Tensor, n: int, in_kind: int, f: torch.Tensor,
                   dtype: int = LGN_F32, out: torch.Tensor = None) -> torch.Tensor:
    if out is None:
        out = torch.empty(int(n), dtype={LGN_F32: torch.float32, LGN_BF16: torch.bfloat16,
                                         LGN_F16: torch.float16}[dtype], device=codes.device)
    _check(load().lgn_dequantize(codes.data_ptr(), int(n), int(in_kind), f.data_ptr(), int(dtype),
                                 out.data_ptr(), _stream()))
    return out


def lgn_prefix_table_bytes(n: int) -> int:
    return int(load().lgn_prefix_table_bytes(int(n)))


def lgn_prefix_bound_bytes(n: int, width: int) -> int:
    return int(load().lgn_prefix_bound_bytes(int(n), int(width)))


def lgn_prefix_encode(x: torch.Tensor, in_kind: int, p: torch.Tensor = None, f: torch.Tensor = None,
                      out: torch.Tensor = None, table: torch.Tensor = None, width: int = None, dtype=None):
    """Returns (stream buffer, table).  The buffer is sized for the worst case unless `out` is given;
    the stream itself is the first table[nchunks] * 4 bytes of it."""
    x = _flat(x)
    n = x.numel()
    dt = LGN_F32 if in_kind == LGN_OUT_CODE8 else _dtype_code(x, dtype)
    if out is None:
        if width is None:
            width = 8 if in_kind == LGN_OUT_CODE8 else (32 if dt == LGN_F32 else 16)
        out = torch.empty(max(lgn_prefix_bound_bytes(n, width), 4), dtype=torch.uint8, device=x.device)
    if table is None:
        table = torch.empty(lgn_prefix_table_bytes(n) // 8, dtype=torch.int64, device=x.device)
    _check(load().lgn_prefix_encode(x.data_ptr(), n, int(in_kind), dt,
                                    p.data_ptr() if p is not None else None,
                                    f.data_ptr() if f is not None else None,
                                    out.data_ptr(), out.numel(), table.data_ptr(), _stream()))
    return out, table


def prefix_sub_lengths(table: torch.Tensor, n: int) -> torch.Tensor:
    """The 16-bit sub-block lengths (16 per chunk) stored behind the chunk table, as an int16 view."""
    nchunks = (int(n) + LGN_PREFIX_CHUNK - 1) // LGN_PREFIX_CHUNK
    first = (nchunks + 2 + LGN_PREFIX_MAX_BLOCKS) * 4          # in 16-bit units
    return table.view(torch.int16)[first:first + 16 * nchunks]


def lgn_prefix_decode(stream_buf: torch.Tensor, table: torch.Tensor, n: int, in_kind: int,
                      p: torch.Tensor = None, f: torch.Tensor = None, dtype: int = LGN_F32,
                      out: torch.Tensor = None) -> torch.Tensor:
    if out is None:
        tdt = torch.uint8 if in_kind == LGN_OUT_CODE8 else {LGN_F32: torch.float32, LGN_BF16: torch.bfloat16,
                                                            LGN_F16: torch.float16}[dtype]
        out = torch.empty(int(n), dtype=tdt, device=stream_buf.device)
    _check(load().lgn_prefix_decode(stream_buf.data_ptr(), table.data_ptr(), int(n), int(in_kind),
                                    int(dtype), p.data_ptr() if p is not None else None,
                                    f.data_ptr() if f is not None else None, out.data_ptr(), _stream()))
    return out


def lgn_log_histogram(g: torch.Tensor, out: torch.Tensor = None, dtype=None) -> torch.Tensor:
    g = _flat(g)
    if out is None:
        out = torch.empty(LGN_HIST_BINS, dtype=torch.int64, device=g.device)
    _check(load().lgn_log_histogram(g.data_ptr(), g.numel(), _dtype_code(g, dtype), out.data_ptr(), _stream()))
    return out


def lgn_sparsity_allocate(stats: torch.Tensor, hists, n_layers: int, overall_sparsity: float,
                          min_cosine: torch.Tensor = None, max_sparsity: float = 0.97,
                          quantile: float = 0.997, alpha_dtype: int = LGN_F32,
                          p_out: torch.Tensor = None, a_out: torch.Tensor = None):
    """stats: n_layers lgn_stats_t back to back (deepest layer first); hists: n_layers x 2048 int64
    or None; min_cosine: float64 tensor, one entry per deep layer.  Returns (p_out, a_out) buffers."""
    if p_out is None:
        p_out = torch.empty(max(n_layers, 1) * C.sizeof(LgnPruneParams), dtype=torch.uint8, device=stats.device)
    if a_out is None:
        a_out = torch.empty(max(n_layers, 1) * C.sizeof(LgnAlloc), dtype=torch.uint8, device=stats.device)
    n_deep = 0 if min_cosine is None else int(min_cosine.numel())
    if n_deep and min_cosine.dtype != torch.float64:
        raise TypeError("min_cosine must be float64")
    _check(load().lgn_sparsity_allocate(stats.data_ptr(), hists.data_ptr() if hists is not None else None,
                                        int(n_layers), float(overall_sparsity), n_deep,
                                        min_cosine.data_ptr() if n_deep else None, float(max_sparsity),
                                        float(quantile), int(alpha_dtype), p_out.data_ptr(), a_out.data_ptr(),
                                        _stream()))
    return p_out, a_out


def read_array(buf: torch.Tensor, cls, count: int):
    """`count` structs of type cls stored back to back in a device buffer."""
    raw = bytes(buf.cpu().numpy().tobytes())
    size = C.sizeof(cls)
    return [cls.from_buffer_copy(raw[i * size:(i + 1) * size]) for i in range(count)]


# ---- moving the small structs between host and device (tests, logging) ------------------------
def _read(buf: torch.Tensor, cls):
    raw = bytes(buf.cpu().numpy().tobytes())  # synchronises with the stream that wrote it
    return cls.from_buffer_copy(raw)


def read_stats(buf: torch.Tensor) -> LgnStats:
    return _read(buf, LgnStats)


def read_prune_params(buf: torch.Tensor) -> LgnPruneParams:
    return _read(buf, LgnPruneParams)


def read_fp_params(buf: torch.Tensor) -> LgnFpParams:
    return _read(buf, LgnFpParams)


def upload_struct(s: C.Structure, device="cuda") -> torch.Tensor:
    """Copy a host-side struct into a fresh device buffer (to feed hand-made parameters)."""
    import numpy as np
    arr = np.frombuffer(bytes(s), dtype=np.uint8).copy()
    return torch.from_numpy(arr).to(device)
