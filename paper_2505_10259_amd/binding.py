"""ctypes binding of libspecverify.so: the same names as include/specverify.h, argument
marshalling only.  Every step of the draft/verify path runs inside the library's HIP kernels;
there is no Python or CPU fallback — if the library is missing, importing raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SO_PATH = os.path.join(_HERE, "libspecverify.so")

SPEC_OK = 0
SPEC_ERR_ARG, SPEC_ERR_SHAPE, SPEC_ERR_BUDGET, SPEC_ERR_CAPACITY, SPEC_ERR_HIP, SPEC_ERR_STATE = -1, -2, -3, -4, -5, -6
SPEC_F32, SPEC_BF16 = 0, 1
SPEC_GREEDY, SPEC_SAMPLE = 0, 1
SPEC_FLAG_NO_OVERLAP, SPEC_FLAG_SIMPLE_KERNELS, SPEC_FLAG_POISON_RELEASED, SPEC_FLAG_PIN_ATTENTION = 1, 2, 4, 8

EXPORTS = [
    "spec_layer_blob_elems", "spec_global_blob_elems", "spec_plan_residency", "spec_host_alloc",
    "spec_host_free", "spec_init", "spec_destroy", "spec_last_error", "spec_prefill", "spec_kv_import",
    "spec_reset", "spec_draft", "spec_verify", "spec_sync", "spec_step", "spec_get_lengths",
    "spec_get_tokens", "spec_get_stats", "spec_reset_stats", "spec_debug_logits",
    "spec_debug_draft_logits", "spec_accept", "spec_philox_uniforms", "spec_layer_forward",
    "spec_debug_routing", "spec_gemm", "spec_debug_gemm", "spec_measure_link", "spec_profile_enable", "spec_profile_read",
    "spec_plan_paraspec", "spec_plan_evaluate", "spec_plan_placement", "spec_debug_force_routing",
    "spec_layer_forward_static",
]
PROF_CLASSES = ["norm", "qkv", "rope", "attn", "oproj", "route", "moe1", "moe2", "head", "accept", "draft"]


class spec_model_shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim",
                                         "d_ff", "vocab", "n_experts", "top_k", "attn_only", "dtype")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class spec_host_weights(C.Structure):
    _fields_ = [("layer_blobs", C.POINTER(C.c_void_p)), ("global_blob", C.c_void_p)]


class spec_runtime_cfg(C.Structure):
    _fields_ = [("hbm_weight_budget_bytes", C.c_int64), ("n_sub_batches", C.c_int32),
                ("batch_max", C.c_int32), ("k_max", C.c_int32), ("ctx_max", C.c_int32),
                ("page_tokens", C.c_int32), ("mode", C.c_int32), ("temperature", C.c_float),
                ("seed", C.c_uint64), ("n_ring_slots", C.c_int32), ("flags", C.c_int32),
                ("prefill_chunk", C.c_int32), ("compute_stream", C.c_void_p), ("copy_stream", C.c_void_p),
                ("draft_stream", C.c_void_p), ("n_piece_slots", C.c_int32), ("prefill_group_rows", C.c_int32)]


class spec_stats(C.Structure):
    _fields_ = [("bytes_streamed", C.c_int64), ("layers_streamed", C.c_int64),
                ("resident_layers", C.c_int64), ("hbm_weight_bytes", C.c_int64), ("rounds", C.c_int64),
                ("committed_tokens", C.c_int64), ("accept_hist", C.c_int64 * 17), ("copy_busy_ms", C.c_double),
                ("pinned_piece_bytes", C.c_int64)]


class spec_placement(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("resident_layers", "pinned_piece_bytes", "streamed_bytes_per_pass",
                                         "ring_bytes", "fixed_bytes")] + \
               [("n_slots", C.c_int32), ("piece_staging", C.c_int32)]


_PLANNER_INTS = ("n_layer", "n_layer_streamed", "l_input", "n_generate", "bs_max", "n_cand_max")
_PLANNER_DOUBLES = ("p_accept", "t_c2g_para", "t_gpu_prefill_comp", "t_ffn_c2g", "t_ffn_gpu", "t_attention_unit",
                    "t_draft_prefill", "t_draft_decoding", "gpu_mem_capacity", "v_target_prefill", "v_target_kv",
                    "v_target_ffn", "v_draft", "v_draft_kv", "t_ffn_gpu_per_token", "t_draft_per_seq",
                    "t_prefill_comp_per_seq", "v_target_kv_decoding")


class spec_planner_profile(C.Structure):
    _fields_ = [(n, C.c_int32) for n in _PLANNER_INTS] + [(n, C.c_double) for n in _PLANNER_DOUBLES]


class spec_plan(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("feasible", "bs", "bs_prefill", "bs_draft", "n_cand", "n_iter")] + \
               [(n, C.c_double) for n in ("throughput", "expected_tokens", "t_prefill", "t_round",
                                          "t_target_decoding", "t_draft", "v_prefill", "v_decoding")]


class SpecError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"specverify error {code}: {msg}")
        self.code = code


def _load() -> C.CDLL:
    if not os.path.exists(SO_PATH):
        from .build import build
        build()
    # PyTorch ships its own copy of the HIP runtime; it must be the one already mapped when this
    # library is loaded (loading the system copy first leaves torch without a visible GPU), so that
    # torch tensors/streams and the library share one runtime.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(SO_PATH)
    vp, i32, i64, u32, u64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64, C.c_float
    P = C.POINTER
    sig = {
        "spec_layer_blob_elems": (i64, [P(spec_model_shape)]),
        "spec_global_blob_elems": (i64, [P(spec_model_shape)]),
        "spec_plan_residency": (i64, [P(spec_model_shape), P(spec_model_shape), i64, i32, P(i64)]),
        "spec_host_alloc": (i32, [C.c_size_t, P(vp)]),
        "spec_host_free": (i32, [vp]),
        "spec_init": (i32, [P(spec_model_shape), P(spec_model_shape), P(spec_host_weights),
                            P(spec_host_weights), P(spec_runtime_cfg), P(vp)]),
        "spec_destroy": (None, [vp]),
        "spec_last_error": (C.c_char_p, [vp]),
        "spec_prefill": (i32, [vp, i32, vp, vp, i32, i32]),
        "spec_kv_import": (i32, [vp, i32, i32, vp, vp, i32, i32]),
        "spec_reset": (i32, [vp, i32]),
        "spec_draft": (i32, [vp, i32, i32, vp]),
        "spec_verify": (i32, [vp, i32, vp, i32, vp, vp]),
        "spec_sync": (i32, [vp, i32]),
        "spec_step": (i32, [vp, i32]),
        "spec_get_lengths": (i32, [vp, i32, vp]),
        "spec_get_tokens": (i32, [vp, i32, i32, vp, i32, P(i32)]),
        "spec_get_stats": (i32, [vp, P(spec_stats)]),
        "spec_reset_stats": (i32, [vp]),
        "spec_debug_logits": (i32, [vp, i32, vp]),
        "spec_debug_draft_logits": (i32, [vp, i32, vp]),
        "spec_accept": (i32, [vp, vp, vp, vp, vp, f32, u64, u32, u32, i32, i32, i32, vp, vp, vp]),
        "spec_philox_uniforms": (i32, [u64, u32, u32, i32, i32, vp, vp]),
        "spec_layer_forward": (i32, [vp, i32, i32, vp, i32, vp]),
        "spec_layer_forward_static": (i32, [vp, i32, i32, vp, i32, vp]),
        "spec_debug_routing": (i32, [vp, i32, vp, vp, i32]),
        "spec_gemm": (i32, [vp, vp, vp, i32, i32, i32, i32, i32, vp]),
        "spec_debug_gemm": (i32, [vp, vp, vp, i32, i32, i32, i32, i32, vp]),
        "spec_measure_link": (i32, [C.c_size_t, i32, P(C.c_double)]),
        "spec_profile_enable": (i32, [vp, u32]),
        "spec_profile_read": (i32, [vp, P(C.c_double), P(i64), i32]),
        "spec_plan_paraspec": (i32, [P(spec_planner_profile), P(spec_plan)]),
        "spec_plan_evaluate": (i32, [P(spec_planner_profile), i32, i32, i32, i32, P(spec_plan)]),
        "spec_plan_placement": (i32, [P(spec_model_shape), P(spec_model_shape), P(spec_runtime_cfg), P(spec_placement)]),
        "spec_debug_force_routing": (i32, [vp, i32, vp, i32]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


lib = _load()


def _ptr(x) -> Optional[int]:
    """Device/host address of a torch tensor, numpy array, int or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return x.data_ptr()          # torch.Tensor


def _check(rc: int, ctx=None):
    if rc < 0:
        raise SpecError(rc, (lib.spec_last_error(ctx) or b"").decode())
    return rc


def make_shape(s) -> spec_model_shape:
    """C struct from any object with the ModelShape attribute names."""
    return spec_model_shape(s.n_layers, s.d_model, s.n_q_heads, s.n_kv_heads, s.head_dim, s.d_ff, s.vocab,
                            s.n_experts, s.top_k, int(s.attn_only), SPEC_BF16 if s.dtype == "bf16" else SPEC_F32,
                            s.rope_theta, s.rms_eps)


def make_host_weights(layer_ptrs: Sequence[int], global_ptr: int):
    arr = (C.c_void_p * max(1, len(layer_ptrs)))(*layer_ptrs)
    hw = spec_host_weights(C.cast(arr, C.POINTER(C.c_void_p)), global_ptr)
    hw._keep = arr
    return hw


# ---- same-name wrappers ---------------------------------------------------------------------
def spec_layer_blob_elems(shape) -> int:
    return _check(lib.spec_layer_blob_elems(C.byref(make_shape(shape))))


def spec_global_blob_elems(shape) -> int:
    return _check(lib.spec_global_blob_elems(C.byref(make_shape(shape))))


def spec_plan_residency(target, draft, budget: int, n_ring_slots: int = 0):
    out = C.c_int64(0)
    d = C.byref(make_shape(draft)) if draft is not None else None
    r = _check(lib.spec_plan_residency(C.byref(make_shape(target)), d, budget, n_ring_slots, C.byref(out)))
    return r, out.value


def spec_plan_placement(target, draft, *, hbm_weight_budget_bytes: int, n_ring_slots: int = 0, n_piece_slots: int = 0,
                        flags: int = 0) -> dict:
    cfg = spec_runtime_cfg()
    cfg.hbm_weight_budget_bytes, cfg.n_ring_slots, cfg.n_piece_slots, cfg.flags = hbm_weight_budget_bytes, n_ring_slots, n_piece_slots, flags
    out = spec_placement()
    d = C.byref(make_shape(draft)) if draft is not None else None
    _check(lib.spec_plan_placement(C.byref(make_shape(target)), d, C.byref(cfg), C.byref(out)))
    return {n: getattr(out, n) for n, _ in spec_placement._fields_}


def spec_host_alloc(nbytes: int) -> int:
    p = C.c_void_p()
    _check(lib.spec_host_alloc(nbytes, C.byref(p)))
    return p.value


def spec_host_free(ptr: int) -> None:
    _check(lib.spec_host_free(ptr))


class PinnedArena:
    """Pinned host arrays from spec_host_alloc, freed together."""

    def __init__(self):
        self._ptrs = []

    def alloc(self, n_elems: int, dtype) -> np.ndarray:
        dt = np.dtype(dtype)
        nbytes = max(1, n_elems * dt.itemsize)
        p = spec_host_alloc(nbytes)
        self._ptrs.append(p)
        buf = (C.c_char * nbytes).from_address(p)
        return np.frombuffer(buf, dtype=dt, count=n_elems)

    def free(self):
        for p in self._ptrs:
            spec_host_free(p)
        self._ptrs = []


def spec_init(target, draft, target_w: spec_host_weights, draft_w: Optional[spec_host_weights], *,
              hbm_weight_budget_bytes: int = 0, n_sub_batches: int = 1, batch_max: int, k_max: int,
              ctx_max: int, page_tokens: int = 0, mode: int = SPEC_GREEDY, temperature: float = 1.0,
              seed: int = 0, n_ring_slots: int = 0, flags: int = 0, prefill_chunk: int = 0,
              compute_stream=None, copy_stream=None, draft_stream=None, n_piece_slots: int = 0,
              prefill_group_rows: int = 0) -> int:
    cfg = spec_runtime_cfg(hbm_weight_budget_bytes, n_sub_batches, batch_max, k_max, ctx_max, page_tokens,
                           mode, temperature, seed, n_ring_slots, flags, prefill_chunk, compute_stream,
                           copy_stream, draft_stream, n_piece_slots, prefill_group_rows)
    ctx = C.c_void_p()
    ts = make_shape(target)
    ds = make_shape(draft) if draft is not None else None
    _check(lib.spec_init(C.byref(ts), C.byref(ds) if ds is not None else None, C.byref(target_w),
                         C.byref(draft_w) if draft_w is not None else None, C.byref(cfg), C.byref(ctx)))
    return ctx.value


def spec_destroy(ctx: int) -> None:
    lib.spec_destroy(ctx)


def spec_last_error(ctx=None) -> str:
    return (lib.spec_last_error(ctx) or b"").decode()


def spec_prefill(ctx, sub: int, prompts: Sequence[np.ndarray], max_new: int) -> None:
    cu = np.zeros(len(prompts) + 1, dtype=np.int32)
    cu[1:] = np.cumsum([len(p) for p in prompts])
    flat = np.ascontiguousarray(np.concatenate([np.asarray(p, dtype=np.int32) for p in prompts]))
    _check(lib.spec_prefill(ctx, sub, flat.ctypes.data, cu.ctypes.data, len(prompts), max_new), ctx)


def spec_kv_import(ctx, sub, layer, k_ctx_dev, v_ctx_dev, B, ctx_len) -> None:
    _check(lib.spec_kv_import(ctx, sub, layer, _ptr(k_ctx_dev), _ptr(v_ctx_dev), B, ctx_len), ctx)


def spec_reset(ctx, sub) -> None:
    _check(lib.spec_reset(ctx, sub), ctx)


def spec_draft(ctx, sub, k, draft_tokens_dev=None) -> None:
    _check(lib.spec_draft(ctx, sub, k, _ptr(draft_tokens_dev)), ctx)


def spec_verify(ctx, sub, draft_tokens_dev, k, n_accepted_dev=None, next_token_dev=None) -> None:
    _check(lib.spec_verify(ctx, sub, _ptr(draft_tokens_dev), k, _ptr(n_accepted_dev), _ptr(next_token_dev)), ctx)


def spec_sync(ctx, sub=-1) -> None:
    _check(lib.spec_sync(ctx, sub), ctx)


def spec_step(ctx, k) -> None:
    _check(lib.spec_step(ctx, k), ctx)


def spec_get_lengths(ctx, sub, B) -> np.ndarray:
    out = np.zeros(B, dtype=np.int32)
    _check(lib.spec_get_lengths(ctx, sub, out.ctypes.data), ctx)
    return out


def spec_get_tokens(ctx, sub, seq, cap) -> np.ndarray:
    out = np.zeros(cap, dtype=np.int32)
    n = C.c_int32(0)
    _check(lib.spec_get_tokens(ctx, sub, seq, out.ctypes.data, cap, C.byref(n)), ctx)
    return out[:min(cap, n.value)]


def spec_get_stats(ctx) -> dict:
    st = spec_stats()
    _check(lib.spec_get_stats(ctx, C.byref(st)), ctx)
    d = {n: getattr(st, n) for n, _ in spec_stats._fields_ if n != "accept_hist"}
    d["accept_hist"] = list(st.accept_hist)
    return d


def spec_reset_stats(ctx) -> None:
    _check(lib.spec_reset_stats(ctx), ctx)


def spec_debug_logits(ctx, sub, out_dev) -> None:
    _check(lib.spec_debug_logits(ctx, sub, _ptr(out_dev)), ctx)


def spec_debug_draft_logits(ctx, sub, out_dev) -> None:
    _check(lib.spec_debug_draft_logits(ctx, sub, _ptr(out_dev)), ctx)


def spec_accept(p_logits, q_logits, draft_tokens, u_accept, u_resample, temperature, seed, rnd, seq_base,
                B, k, V, n_accepted, next_token, stream=None) -> None:
    _check(lib.spec_accept(_ptr(p_logits), _ptr(q_logits), _ptr(draft_tokens), _ptr(u_accept), _ptr(u_resample),
                           temperature, seed, rnd, seq_base, B, k, V, _ptr(n_accepted), _ptr(next_token), stream))


def spec_philox_uniforms(seed, rnd, seq_base, B, k, out_dev, stream=None) -> None:
    _check(lib.spec_philox_uniforms(seed, rnd, seq_base, B, k, _ptr(out_dev), stream))


def spec_layer_forward(ctx, sub, layer, x_in_dev, n_new, x_out_dev) -> None:
    _check(lib.spec_layer_forward(ctx, sub, layer, _ptr(x_in_dev), n_new, _ptr(x_out_dev)), ctx)


def spec_layer_forward_static(ctx, sub, layer, x_in_dev, n_new, x_out_dev) -> None:
    _check(lib.spec_layer_forward_static(ctx, sub, layer, _ptr(x_in_dev), n_new, _ptr(x_out_dev)), ctx)


def spec_debug_routing(ctx, sub, ids_dev, weights_dev, T) -> None:
    _check(lib.spec_debug_routing(ctx, sub, _ptr(ids_dev), _ptr(weights_dev), T), ctx)


def spec_debug_force_routing(ctx, sub, ids_dev, rows_per_layer) -> None:
    _check(lib.spec_debug_force_routing(ctx, sub, _ptr(ids_dev), rows_per_layer), ctx)


def spec_gemm(A_dev, W_dev, C_dev, M, N, K, dtype, flags=0, stream=None) -> None:
    _check(lib.spec_gemm(_ptr(A_dev), _ptr(W_dev), _ptr(C_dev), M, N, K, dtype, flags, stream))


def spec_debug_gemm(A_dev, W_dev, C_dev, M, N, K, tile_rows, tile_cols, stream=None) -> None:
    _check(lib.spec_debug_gemm(_ptr(A_dev), _ptr(W_dev), _ptr(C_dev), M, N, K, tile_rows, tile_cols, stream))


def spec_measure_link(nbytes: int, reps: int = 4) -> float:
    out = C.c_double(0.0)
    _check(lib.spec_measure_link(nbytes, reps, C.byref(out)))
    return out.value


def spec_profile_enable(ctx, classes=None) -> None:
    """classes: iterable of names from PROF_CLASSES (None = all, empty = off)."""
    names = PROF_CLASSES if classes is None else list(classes)
    mask = 0
    for n in names:
        mask |= 1 << PROF_CLASSES.index(n)
    _check(lib.spec_profile_enable(ctx, mask), ctx)


def spec_profile_read(ctx, reset: bool = True) -> dict:
    ms = (C.c_double * len(PROF_CLASSES))()
    n = (C.c_int64 * len(PROF_CLASSES))()
    _check(lib.spec_profile_read(ctx, ms, n, int(reset)), ctx)
    return {name: {"ms": ms[i], "launches": n[i]} for i, name in enumerate(PROF_CLASSES)}


def _planner_profile(profile: dict) -> spec_planner_profile:
    pr = spec_planner_profile()
    for n in _PLANNER_INTS:
        setattr(pr, n, int(profile[n]))
    for n in _PLANNER_DOUBLES:
        setattr(pr, n, float(profile.get(n, 0.0)))
    return pr


def _plan_dict(pl: spec_plan) -> dict:
    return {n: getattr(pl, n) for n, _ in spec_plan._fields_}


def spec_plan_paraspec(profile: dict) -> dict:
    """profile: the fields of spec_planner_profile by name (the optional ones default to 0)."""
    pl = spec_plan()
    _check(lib.spec_plan_paraspec(C.byref(_planner_profile(profile)), C.byref(pl)), None)
    return _plan_dict(pl)


def spec_plan_evaluate(profile: dict, bs: int, bs_prefill: int, bs_draft: int, n_cand: int) -> dict:
    pl = spec_plan()
    _check(lib.spec_plan_evaluate(C.byref(_planner_profile(profile)), bs, bs_prefill, bs_draft, n_cand, C.byref(pl)), None)
    return _plan_dict(pl)
