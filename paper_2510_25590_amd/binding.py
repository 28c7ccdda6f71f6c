"""Thin ctypes binding over libregione.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA tensors (used for device memory and streams only); every step of the
path runs in the library's HIP kernels.  The library is loaded on first use and the load
fails loudly if it has not been built (`python -m paper_2510_25590_amd.build`); there is no
fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libregione.so")

OK = 0
ERR_INVALID_ARG, ERR_BAD_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = -1, -2, -3, -4, -5
BF16, FP32 = 0, 1
BLOCK_DOUBLE, BLOCK_SINGLE = 0, 1
FLAG_STORE, FLAG_RETRIEVE = 1, 2
ACT_NONE, ACT_GELU_TANH, ACT_SILU = 0, 1, 2

EXPORTS = (
    "regione_last_error", "regione_create", "regione_destroy", "regione_partition", "regione_gather",
    "regione_scatter", "regione_attn_kvcache", "regione_linear", "regione_block_forward",
    "regione_velocity_decision_host", "regione_velocity_cache", "regione_profile_enable", "regione_profile_read",
    "regione_packed_weight_elems", "regione_pack_weight", "regione_tune_gemm", "regione_tune_attention",
    "regione_layernorm", "regione_stage_plan_host", "regione_cast", "regione_mask_cleanup", "regione_rope_table",
    "regione_vec_linear", "regione_timestep_embedding", "regione_block_forward_batched",
    "regione_sq_norms", "regione_gamma_fit_host", "regione_guidance_combine", "regione_rel_change",
    "regione_quantize_rows_fp8", "regione_pack_weight_fp8", "regione_linear_fp8", "regione_mfma_peak_probe",
    "regione_partition_static", "regione_rel_decision_host", "regione_rel_update_host", "regione_fresh_slots", "regione_time_bias",
    "regione_euler_rows", "regione_gather_pair", "regione_scatter_pair", "regione_velocity_head", "regione_region_step",
    "regione_block_forward_fp8",
)
STEP_FULL, STEP_FULL_STORE, STEP_REGION = 0, 1, 2
PROF_NAMES = ("partition", "rows", "layernorm", "gemm", "attention", "velocity")


class Dims(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("heads", C.c_int32), ("head_dim", C.c_int32), ("mlp", C.c_int32),
                ("max_fresh", C.c_int32), ("max_tokens", C.c_int32), ("compute_dtype", C.c_int32)]


_STREAM_FIELDS = ("w_qkv", "b_qkv", "w_o", "b_o", "w_1", "b_1", "w_2", "b_2",
                  "shift1", "scale1", "gate1", "shift2", "scale2", "gate2", "q_norm", "k_norm", "w_mod", "b_mod")


class StreamWeights(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in _STREAM_FIELDS]


class BlockWeights(C.Structure):
    _fields_ = [("txt", StreamWeights), ("img", StreamWeights), ("rope", C.c_void_p), ("rope_rows", C.c_int32), ("cond", C.c_void_p)]


_FP8_STREAM_FIELDS = ("w_qkv", "s_qkv", "w_o", "s_o", "w_1", "s_1", "w_2", "s_2")
_FP8_TAP_FIELDS = ("u1_codes", "u1_scale", "q", "attn", "a_codes", "a_scale", "h1", "u2_codes", "u2_scale", "m", "m_codes", "m_scale")


class StreamWeightsFp8(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in _FP8_STREAM_FIELDS]


class BlockWeightsFp8(C.Structure):
    _fields_ = [("txt", StreamWeightsFp8), ("img", StreamWeightsFp8)]


class Fp8Taps(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in _FP8_TAP_FIELDS]


class RegionStepArgs(C.Structure):
    """regione_region_step_args, field for field."""
    _fields_ = [("x_t", C.c_void_p), ("v", C.c_void_p), ("x_ref", C.c_void_p),
                ("n_tokens", C.c_int64), ("c", C.c_int32), ("dtype", C.c_int32), ("sigma_t", C.c_float), ("eta", C.c_float),
                ("score_opt", C.c_void_p), ("mask", C.c_void_p), ("e_index", C.c_void_p), ("u_index", C.c_void_p), ("n_edited_dev", C.c_void_p),
                ("h_full", C.c_void_p), ("h_dtype", C.c_int32), ("n_txt_fresh", C.c_int32),
                ("h_rows", C.c_void_p), ("h_rows_out", C.c_void_p), ("slots", C.c_void_p),
                ("n_blocks", C.c_int32), ("n_all", C.c_int32), ("slot_offset", C.c_int32), ("reserved", C.c_int32),
                ("blocks", C.POINTER(BlockWeights)), ("block_types", C.POINTER(C.c_int32)), ("k_caches", C.POINTER(C.c_void_p)), ("v_caches", C.POINTER(C.c_void_p)),
                ("w_head_packed", C.c_void_p), ("b_head_opt", C.c_void_p), ("dt", C.c_float), ("reserved2", C.c_int32),
                ("v_out_opt", C.c_void_p), ("c_a", C.c_void_p), ("x_e", C.c_void_p), ("x_next_full", C.c_void_p), ("h_next_full_opt", C.c_void_p)]


class AvdState(C.Structure):
    _fields_ = [("valid", C.c_int32), ("prod", C.c_double)]


class RelState(C.Structure):
    _fields_ = [("have_cache", C.c_int32), ("reuse_next", C.c_int32)]


class PlanStep(C.Structure):
    _fields_ = [("i", C.c_int32), ("kind", C.c_int32), ("seg_first", C.c_int32), ("seg_next", C.c_int32)]


class RegionEError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"regione error {code}: {message}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2510_25590_amd.build`")
        # torch ships its own HIP runtime; the library must bind to THAT copy (the tensors and streams it is handed live
        # there), so torch has to be loaded first: a process that loaded the library first would end up with two runtimes,
        # and the second one to initialise finds no device
        import torch  # noqa: F401
        _lib = C.CDLL(LIB_PATH)
        _lib.regione_last_error.restype = C.c_char_p
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        sig = {
            "regione_create": [C.POINTER(vp), C.POINTER(Dims), vp],
            "regione_destroy": [vp],
            "regione_partition": [vp, vp, vp, vp, i64, i32, i32, f32, f32, vp, vp, vp, vp, vp, C.POINTER(i32)],
            "regione_gather": [vp, vp, i32, i32, vp, vp, i64, vp],
            "regione_scatter": [vp, vp, i32, i32, vp, vp, i64, vp],
            "regione_attn_kvcache": [vp, vp, i32, vp, vp, i32, vp, vp, i32, vp, i32, i32, i32, f32, vp],
            "regione_linear": [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp],
            "regione_block_forward": [vp, C.POINTER(BlockWeights), i32, vp, vp, i32, i32, i32, vp, i32, vp, vp, i32, i32],
            "regione_block_forward_batched": [vp, C.POINTER(BlockWeights), i32, vp, vp, i32, i32, i32, i32, vp, i32, vp, vp, i32, i32],
            "regione_velocity_decision_host": [C.POINTER(f32), C.POINTER(f32), i32, f32, i32, C.POINTER(AvdState),
                                               C.POINTER(i32), C.POINTER(f32)],
            "regione_sq_norms": [vp, vp, i32, i64, i64, vp],
            "regione_guidance_combine": [vp, vp, vp, f32, vp, i64, i32],
            "regione_rel_change": [vp, vp, vp, i64, i32, vp, C.POINTER(C.c_double)],
            "regione_rel_decision_host": [C.POINTER(RelState), f32, C.POINTER(i32), C.POINTER(f32)],
            "regione_rel_update_host": [C.POINTER(RelState), C.POINTER(C.c_double), f32, C.POINTER(C.c_double)],
            "regione_fresh_slots": [vp, vp, vp, i64, i32, vp],
            "regione_time_bias": [vp, vp, vp, f32, vp, i32],
            "regione_euler_rows": [vp, vp, vp, vp, vp, i64, i32, i32, f32],
            "regione_gather_pair": [vp, vp, i32, i32, vp, vp, i32, i32, vp, vp, vp, i64],
            "regione_scatter_pair": [vp, vp, i32, i32, vp, vp, i32, i32, vp, vp, vp, i64],
            "regione_velocity_head": [vp, vp, vp, vp, i32, i32, i32, f32, vp, vp, vp, vp, vp, i32],
            "regione_region_step": [vp, C.POINTER(RegionStepArgs), C.POINTER(i32)],
            "regione_block_forward_fp8": [vp, C.POINTER(BlockWeights), C.POINTER(BlockWeightsFp8), i32, vp, vp, i32, i32, i32, vp, i32, vp, vp, i32, i32,
                                          C.POINTER(Fp8Taps)],
            "regione_partition_static": [vp, vp, vp, vp, i64, i32, i32, f32, f32, vp, vp, vp, vp, vp],
            "regione_gamma_fit_host": [C.POINTER(C.c_double), i32, C.POINTER(f32), i32, C.POINTER(f32)],
            "regione_velocity_cache": [vp, i32, f32, f32, vp, vp, vp, vp, vp, i64, i32, i32],
            "regione_pack_weight": [vp, vp, i32, i32, vp],
            "regione_mfma_peak_probe": [vp, i32, i32, i32, vp, C.POINTER(C.c_double)],
            "regione_quantize_rows_fp8": [vp, vp, i64, i32, vp, vp],
            "regione_pack_weight_fp8": [vp, vp, i32, i32, vp],
            "regione_linear_fp8": [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp],
            "regione_tune_gemm": [vp, i32, i32],
            "regione_tune_attention": [vp, i32],
            "regione_layernorm": [vp, vp, i32, i32, i32, vp, vp, vp],
            "regione_cast": [vp, vp, i32, vp, i32, i64],
            "regione_rope_table": [vp, vp, i64, i32, C.POINTER(i32), f32, vp],
            "regione_vec_linear": [vp, vp, i32, vp, vp, i32, i32, vp],
            "regione_timestep_embedding": [vp, C.c_double, i32, C.c_double, vp],
            "regione_mask_cleanup": [vp, vp, i32, i32, i32, vp, vp, vp, vp, C.POINTER(i32)],
            "regione_stage_plan_host": [i32, i32, i32, C.POINTER(i32), i32, C.POINTER(PlanStep), i32, C.POINTER(i32)],
            "regione_profile_enable": [vp, i32],
            "regione_profile_read": [vp, C.POINTER(C.c_double), C.POINTER(i64), i32],
        }
        for name, args in sig.items():
            fn = getattr(_lib, name)
            fn.argtypes = args
            fn.restype = C.c_int
        _lib.regione_packed_weight_elems.argtypes = [i32, i32]
        _lib.regione_packed_weight_elems.restype = C.c_int64
    return _lib


def _check(rc: int) -> None:
    if rc != OK:
        raise RegionEError(rc, lib().regione_last_error().decode())


def _p(t):
    """Device pointer of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


class Context:
    """Owns a regione_ctx bound to a torch stream (default: the current one)."""

    def __init__(self, hidden: int, heads: int, head_dim: int, mlp: int, max_fresh: int, max_tokens: int, stream=None,
                 compute_dtype: int = BF16):
        import torch
        self._torch = torch
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self.compute_dtype = compute_dtype
        self.torch_dtype = torch.float32 if compute_dtype == FP32 else torch.bfloat16   # storage type of activations, weights and caches
        self.dims = Dims(hidden, heads, head_dim, mlp, max_fresh, max_tokens, compute_dtype)
        handle = C.c_void_p()
        _check(lib().regione_create(C.byref(handle), C.byref(self.dims), C.c_void_p(self.stream.cuda_stream)))
        self.handle = handle

    def close(self):
        if getattr(self, "handle", None):
            lib().regione_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def make_stream_weights(tensors: dict) -> StreamWeights:
    """dict name -> torch CUDA tensor (missing names become NULL).  The caller keeps the tensors alive."""
    w = StreamWeights()
    for name in _STREAM_FIELDS:
        t = tensors.get(name)
        setattr(w, name, None if t is None else t.data_ptr())
    return w


def regione_partition(ctx, x_t, v, x_ref, n_tokens, c, dtype, sigma_t, eta, score, mask, e_index, u_index,
                      n_edited_dev, read_count: bool = True):
    host = C.c_int32(-1)
    _check(lib().regione_partition(ctx.handle, _p(x_t), _p(v), _p(x_ref), n_tokens, c, dtype, sigma_t, eta,
                                   _p(score), _p(mask), _p(e_index), _p(u_index), _p(n_edited_dev),
                                   C.byref(host) if read_count else None))
    return host.value if read_count else None


def regione_mask_cleanup(ctx, mask_in, grid_h, grid_w, n_images, mask_out, e_index, u_index, n_edited_dev, read_count: bool = True):
    host = C.c_int32(-1)
    _check(lib().regione_mask_cleanup(ctx.handle, _p(mask_in), grid_h, grid_w, n_images, _p(mask_out), _p(e_index), _p(u_index),
                                      _p(n_edited_dev), C.byref(host) if read_count else None))
    return host.value if read_count else None


def regione_gather(ctx, src, row_elems, dtype, index, n_dev, n_max, dst):
    _check(lib().regione_gather(ctx.handle, _p(src), row_elems, dtype, _p(index), _p(n_dev), n_max, _p(dst)))


def regione_scatter(ctx, dst_full, row_elems, dtype, index, n_dev, n_max, src):
    _check(lib().regione_scatter(ctx.handle, _p(dst_full), row_elems, dtype, _p(index), _p(n_dev), n_max, _p(src)))


def regione_attn_kvcache(ctx, q, n_q, k_fresh, v_fresh, n_fresh, k_cache, v_cache, n_c, cache_index, n_cache_index,
                         heads, d, scale, out):
    _check(lib().regione_attn_kvcache(ctx.handle, _p(q), n_q, _p(k_fresh), _p(v_fresh), n_fresh, _p(k_cache), _p(v_cache),
                                      n_c, _p(cache_index), n_cache_index, heads, d, scale, _p(out)))


def regione_linear(ctx, x, w, b, m, n, k, act, out_dtype, y):
    _check(lib().regione_linear(ctx.handle, _p(x), _p(w), _p(b), m, n, k, act, out_dtype, _p(y)))


def regione_block_forward(ctx, weights: BlockWeights, block_type, h_in, h_out, h_dtype, n_fresh, n_txt_fresh,
                          slot_index, slot_offset, k_cache, v_cache, n_all, flags):
    _check(lib().regione_block_forward(ctx.handle, C.byref(weights), block_type, _p(h_in), _p(h_out), h_dtype, n_fresh,
                                       n_txt_fresh, _p(slot_index), slot_offset, _p(k_cache), _p(v_cache), n_all, flags))


def regione_block_forward_fp8(ctx, weights: BlockWeights, weights8: BlockWeightsFp8, block_type, h_in, h_out, h_dtype, n_fresh, n_txt_fresh,
                              slot_index, slot_offset, k_cache, v_cache, n_all, flags, taps: "Fp8Taps | None" = None):
    _check(lib().regione_block_forward_fp8(ctx.handle, C.byref(weights), C.byref(weights8), block_type, _p(h_in), _p(h_out), h_dtype, n_fresh, n_txt_fresh,
                                           _p(slot_index), slot_offset, _p(k_cache), _p(v_cache), n_all, flags,
                                           None if taps is None else C.byref(taps)))


def make_stream_weights_fp8(ctx, tensors: dict):
    """dict with the bf16 row-major weights w_qkv, w_o, w_1, w_2 (CUDA tensors) -> (StreamWeightsFp8, tensors to keep
    alive): each is quantised with one scale per output feature (regione_quantize_rows_fp8) and packed
    (regione_pack_weight_fp8).  The unpacked codes are kept as well (tests feed them to the reference)."""
    import torch
    w8, keep = StreamWeightsFp8(), {}
    for name in ("w_qkv", "w_o", "w_1", "w_2"):
        if name not in tensors:          # a single-stream block has w_1 and w_2 only
            continue
        w = tensors[name].contiguous()
        n, k = w.shape
        codes = torch.empty((n, k), dtype=torch.uint8, device=w.device)
        scale = torch.empty(n, dtype=torch.float32, device=w.device)
        regione_quantize_rows_fp8(ctx, w, n, k, codes, scale)
        packed = torch.zeros(regione_packed_weight_elems(n, k), dtype=torch.uint8, device=w.device)
        regione_pack_weight_fp8(ctx, codes, n, k, packed)
        keep[name] = (packed, scale, codes)
        setattr(w8, name, packed.data_ptr())
        setattr(w8, "s_" + name[2:], scale.data_ptr())
    return w8, keep


def make_fp8_taps(tensors: dict) -> Fp8Taps:
    t = Fp8Taps()
    for name in _FP8_TAP_FIELDS:
        x = tensors.get(name)
        setattr(t, name, None if x is None else x.data_ptr())
    return t


def regione_block_forward_batched(ctx, weights: BlockWeights, block_type, h_in, h_out, h_dtype, n_branches, n_fresh, n_txt_fresh,
                                  slot_index, slot_offset, k_cache, v_cache, n_all, flags):
    _check(lib().regione_block_forward_batched(ctx.handle, C.byref(weights), block_type, _p(h_in), _p(h_out), h_dtype, n_branches, n_fresh,
                                               n_txt_fresh, _p(slot_index), slot_offset, _p(k_cache), _p(v_cache), n_all, flags))


def regione_rel_change(ctx, v_new, v_old, n_elems, dtype, out, read_back: bool = False):
    """With read_back the call waits for the stream and returns the two sums as a ctypes double[2]."""
    host = (C.c_double * 2)() if read_back else None
    _check(lib().regione_rel_change(ctx.handle, _p(v_new), _p(v_old), n_elems, dtype, _p(out), host))
    return host


def regione_rel_decision_host(state: RelState, decay: float):
    reuse, factor = C.c_int32(0), C.c_float(0.0)
    _check(lib().regione_rel_decision_host(C.byref(state), decay, C.byref(reuse), C.byref(factor)))
    return bool(reuse.value), factor.value


def regione_rel_update_host(state: RelState, sums, threshold: float) -> float:
    """sums: the ctypes double[2] of regione_rel_change(read_back=True), or None.  Returns the relative change."""
    rel = C.c_double(0.0)
    _check(lib().regione_rel_update_host(C.byref(state), sums, threshold, C.byref(rel)))
    return rel.value


def regione_fresh_slots(ctx, index, n_dev, n_max, n_txt, slots):
    _check(lib().regione_fresh_slots(ctx.handle, _p(index), _p(n_dev), n_max, n_txt, _p(slots)))


def regione_gather_pair(ctx, src_a, row_elems_a, dtype_a, dst_a, src_b, row_elems_b, dtype_b, dst_b, index, n_dev, n_max):
    _check(lib().regione_gather_pair(ctx.handle, _p(src_a), row_elems_a, dtype_a, _p(dst_a), _p(src_b), row_elems_b, dtype_b, _p(dst_b),
                                     _p(index), _p(n_dev), n_max))


def regione_scatter_pair(ctx, dst_full_a, row_elems_a, dtype_a, src_a, dst_full_b, row_elems_b, dtype_b, src_b, index, n_dev, n_max):
    _check(lib().regione_scatter_pair(ctx.handle, _p(dst_full_a), row_elems_a, dtype_a, _p(src_a), _p(dst_full_b), row_elems_b, dtype_b, _p(src_b),
                                      _p(index), _p(n_dev), n_max))


def regione_velocity_head(ctx, h_rows, w_head, b_head, n, c, hidden, dt, v_out, c_a, x_e, x_full, index, dtype):
    _check(lib().regione_velocity_head(ctx.handle, _p(h_rows), _p(w_head), _p(b_head), n, c, hidden, float(dt), _p(v_out), _p(c_a), _p(x_e),
                                       _p(x_full), _p(index), dtype))


def make_region_step_args(*, x_t, v, x_ref, n_tokens, c, dtype, sigma_t, eta, score, mask, e_index, u_index, n_edited_dev,
                          h_full, h_dtype, n_txt_fresh, h_rows, h_rows_out, slots, blocks, block_types, k_caches, v_caches, n_all, slot_offset,
                          w_head, b_head, dt, v_out, c_a, x_e, x_next_full, h_next_full):
    """Fills a RegionStepArgs from tensors; blocks: list of BlockWeights, k_caches / v_caches: lists of tensors.  The
    returned object keeps the host arrays it points to alive (attribute `_keep`)."""
    n_blocks = len(blocks)
    a = RegionStepArgs()
    arr_b = (BlockWeights * max(n_blocks, 1))(*blocks)
    arr_t = (C.c_int32 * max(n_blocks, 1))(*block_types)
    arr_k = (C.c_void_p * max(n_blocks, 1))(*[t.data_ptr() for t in k_caches])
    arr_v = (C.c_void_p * max(n_blocks, 1))(*[t.data_ptr() for t in v_caches])
    a._keep = (arr_b, arr_t, arr_k, arr_v)
    ptr = lambda t: None if t is None else t.data_ptr()
    a.x_t, a.v, a.x_ref = ptr(x_t), ptr(v), ptr(x_ref)
    a.n_tokens, a.c, a.dtype, a.sigma_t, a.eta = n_tokens, c, dtype, sigma_t, eta
    a.score_opt, a.mask, a.e_index, a.u_index, a.n_edited_dev = ptr(score), ptr(mask), ptr(e_index), ptr(u_index), ptr(n_edited_dev)
    a.h_full, a.h_dtype, a.n_txt_fresh = ptr(h_full), h_dtype, n_txt_fresh
    a.h_rows, a.h_rows_out, a.slots = ptr(h_rows), ptr(h_rows_out), ptr(slots)
    a.n_blocks, a.n_all, a.slot_offset = n_blocks, n_all, slot_offset
    a.blocks = C.cast(arr_b, C.POINTER(BlockWeights)); a.block_types = C.cast(arr_t, C.POINTER(C.c_int32))
    a.k_caches = C.cast(arr_k, C.POINTER(C.c_void_p)); a.v_caches = C.cast(arr_v, C.POINTER(C.c_void_p))
    a.w_head_packed, a.b_head_opt, a.dt = ptr(w_head), ptr(b_head), dt
    a.v_out_opt, a.c_a, a.x_e, a.x_next_full, a.h_next_full_opt = ptr(v_out), ptr(c_a), ptr(x_e), ptr(x_next_full), ptr(h_next_full)
    return a


def regione_region_step(ctx, args: RegionStepArgs) -> int:
    """One region-aware step in one call; returns the edited-token count."""
    n = C.c_int32(0)
    _check(lib().regione_region_step(ctx.handle, C.byref(args), C.byref(n)))
    return n.value


def regione_euler_rows(ctx, x_full, v_full, index, n_dev, n_max, c, dtype, dt):
    _check(lib().regione_euler_rows(ctx.handle, _p(x_full), _p(v_full), _p(index), _p(n_dev), n_max, c, dtype, float(dt)))


def regione_time_bias(ctx, b, b_time, t, out, n):
    _check(lib().regione_time_bias(ctx.handle, _p(b), _p(b_time), float(t), _p(out), n))


def regione_partition_static(stream, x_t, v, x_ref, n_tokens, c, dtype, sigma_t, eta, score, mask, e_index, u_index, n_edited_dev):
    """The partition without a context (allocates nothing); stream: a torch stream or None for the default stream."""
    _check(lib().regione_partition_static(None if stream is None else C.c_void_p(stream.cuda_stream), _p(x_t), _p(v), _p(x_ref),
                                          n_tokens, c, dtype, sigma_t, eta, _p(score), _p(mask), _p(e_index), _p(u_index), _p(n_edited_dev)))


def regione_guidance_combine(ctx, v_cond, v_uncond, scale, out, n_elems, dtype):
    _check(lib().regione_guidance_combine(ctx.handle, _p(v_cond), _p(v_uncond), scale, _p(out), n_elems, dtype))


def regione_sq_norms(ctx, x, dtype, n_vectors, vec_elems, out):
    _check(lib().regione_sq_norms(ctx.handle, _p(x), dtype, n_vectors, vec_elems, _p(out)))


def regione_gamma_fit_host(sq_norms, t):
    """sq_norms: host array [n_samples, T+1] of float64; t: T+1 floats.  Returns the list gamma[0..T]."""
    import numpy as np
    a = np.ascontiguousarray(sq_norms, dtype=np.float64)
    n_samples, cols = a.shape
    T = cols - 1
    tt = (C.c_float * (T + 1))(*[float(v) for v in t])
    out = (C.c_float * (T + 1))()
    _check(lib().regione_gamma_fit_host(a.ctypes.data_as(C.POINTER(C.c_double)), n_samples, tt, T, out))
    return list(out)


def regione_velocity_decision_host(t, gamma, n_steps, delta, j, state: AvdState):
    """t, gamma: sequences of n_steps+1 floats.  Returns (reuse, factor) and updates `state`."""
    arr_t = (C.c_float * len(t))(*[float(x) for x in t])
    arr_g = (C.c_float * len(gamma))(*[float(x) for x in gamma])
    reuse, factor = C.c_int32(0), C.c_float(0.0)
    _check(lib().regione_velocity_decision_host(arr_t, arr_g, n_steps, delta, j, C.byref(state), C.byref(reuse), C.byref(factor)))
    return bool(reuse.value), factor.value


def regione_velocity_cache(ctx, reuse, factor, dt, v_fresh, c_a, v_out, x_e, n_dev, n_max, c, dtype):
    _check(lib().regione_velocity_cache(ctx.handle, int(bool(reuse)), factor, dt, _p(v_fresh), _p(c_a), _p(v_out), _p(x_e),
                                        _p(n_dev), n_max, c, dtype))


def regione_rope_table(ctx, pos_ids, n, axes_dims, theta, table):
    """pos_ids: CUDA int32 [n, len(axes_dims)]; table: CUDA float32 [n, sum(axes_dims)] (cos | sin)."""
    dims = (C.c_int32 * len(axes_dims))(*axes_dims)
    _check(lib().regione_rope_table(ctx.handle, _p(pos_ids), n, len(axes_dims), dims, theta, _p(table)))


def regione_vec_linear(ctx, x, pre_act, w, b, n, k, y):
    _check(lib().regione_vec_linear(ctx.handle, _p(x), pre_act, _p(w), _p(b), n, k, _p(y)))


def regione_timestep_embedding(ctx, t, dim, max_period, out):
    _check(lib().regione_timestep_embedding(ctx.handle, float(t), dim, float(max_period), _p(out)))


def regione_cast(ctx, src, src_dtype, dst, dst_dtype, n_elems):
    _check(lib().regione_cast(ctx.handle, _p(src), src_dtype, _p(dst), dst_dtype, n_elems))


def regione_layernorm(ctx, h, h_dtype, n, hidden, shift, scale, u):
    _check(lib().regione_layernorm(ctx.handle, _p(h), h_dtype, n, hidden, _p(shift), _p(scale), _p(u)))


def regione_stage_plan_host(T: int, t_st: int, t_sm: int, forced_k):
    """Returns the steps of Algorithm 1 in the order they run, as a list of PlanStep."""
    forced = [int(k) for k in forced_k]
    arr = (C.c_int32 * max(len(forced), 1))(*forced)
    steps = (PlanStep * (T + 1))()
    n = C.c_int32(0)
    _check(lib().regione_stage_plan_host(T, t_st, t_sm, arr, len(forced), steps, T + 1, C.byref(n)))
    return [steps[k] for k in range(n.value)]


def regione_profile_enable(ctx, on: bool):
    _check(lib().regione_profile_enable(ctx.handle, int(bool(on))))


def regione_profile_read(ctx):
    """Returns {class name: (total milliseconds, launch groups)} since the last read."""
    n = len(PROF_NAMES)
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _check(lib().regione_profile_read(ctx.handle, ms, cnt, n))
    return {name: (ms[i], cnt[i]) for i, name in enumerate(PROF_NAMES)}


def regione_packed_weight_elems(n: int, k: int) -> int:
    return int(lib().regione_packed_weight_elems(n, k))


def regione_pack_weight(ctx, w, n, k, w_packed):
    _check(lib().regione_pack_weight(ctx.handle, _p(w), n, k, _p(w_packed)))


def regione_mfma_peak_probe(ctx, fmt: int, iters: int, n_workgroups: int, out) -> float:
    """Enqueues the probe; returns the floating point operations of the launch."""
    flops = C.c_double(0.0)
    _check(lib().regione_mfma_peak_probe(ctx.handle, fmt, iters, n_workgroups, _p(out), C.byref(flops)))
    return flops.value


def regione_quantize_rows_fp8(ctx, x, rows, cols, q, scale):
    _check(lib().regione_quantize_rows_fp8(ctx.handle, _p(x), rows, cols, _p(q), _p(scale)))


def regione_pack_weight_fp8(ctx, wq, n, k, wq_packed):
    _check(lib().regione_pack_weight_fp8(ctx.handle, _p(wq), n, k, _p(wq_packed)))


def regione_linear_fp8(ctx, xq, x_scale, wq_packed, w_scale, b, m, n, k, act, out_dtype, y):
    _check(lib().regione_linear_fp8(ctx.handle, _p(xq), _p(x_scale), _p(wq_packed), _p(w_scale), _p(b), m, n, k, act, out_dtype, _p(y)))


def regione_tune_gemm(ctx, wave_tile_blocks: int, k_splits: int):
    _check(lib().regione_tune_gemm(ctx.handle, wave_tile_blocks, k_splits))


def regione_tune_attention(ctx, key_splits: int):
    _check(lib().regione_tune_attention(ctx.handle, key_splits))


def pack_weight(ctx, w):
    """Convenience: packs a row-major CUDA tensor [n, k] of the context's storage type into a new tensor in the library's layout."""
    import torch
    n, k = w.shape
    assert w.dtype == ctx.torch_dtype, (w.dtype, ctx.torch_dtype)
    out = torch.empty(regione_packed_weight_elems(n, k), dtype=w.dtype, device=w.device)
    regione_pack_weight(ctx, w.contiguous(), n, k, out)
    return out
