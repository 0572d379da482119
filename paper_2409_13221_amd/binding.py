"""ctypes binding of librlhf.so: the same names as include/rlhf.h and include/rlhf_ops.h.

Argument marshalling only -- every step of the stage runs in the library's HIP kernels.
torch is used for device memory (weights are torch tensors whose data_ptr() is borrowed by
the library) and numpy for the host arrays the ABI fills.  There is no fallback: if the
shared library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librlhf.so")

RLHF_OK, RLHF_EINVAL, RLHF_ENOMEM, RLHF_ESTATE, RLHF_EDEVICE, RLHF_ENONFINITE = 0, -1, -2, -3, -4, -5
RLHF_ACTOR, RLHF_REF, RLHF_CRITIC, RLHF_REWARD = 0, 1, 2, 3
RLHF_FP32, RLHF_BF16 = 0, 1
_STATUS = {0: "OK", -1: "EINVAL", -2: "ENOMEM", -3: "ESTATE", -4: "EDEVICE", -5: "ENONFINITE"}


def RLHF_ROLE_BIT(role: int) -> int:
    return 1 << role


class RlhfError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"RLHF_{_STATUS.get(code, code)}: {msg}")
        self.code = code


class rlhf_model_cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim",
                                         "ffn", "vocab", "dtype")] + [("rms_eps", C.c_float),
                                                                      ("rope_base", C.c_float)]


class rlhf_engine_cfg(C.Structure):
    _fields_ = [("page_tokens", C.c_int32), ("kv_pool_bytes", C.c_int64), ("max_samples", C.c_int32),
                ("max_ctx", C.c_int32), ("max_active", C.c_int32), ("max_batch_tokens", C.c_int32),
                ("eos_id", C.c_int32), ("stop_on_eos", C.c_int32), ("corun_decode_cus", C.c_int32),
                ("optimistic_admission", C.c_int32), ("decode_stream", C.c_void_p),
                ("score_stream", C.c_void_p), ("half_weight_copies", C.c_int32)]


class rlhf_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("embed", "wqkv", "wo", "w_gate_up", "w_down", "g_attn", "g_mlp",
                                          "g_final", "head")]


class rlhf_step_info(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("step", "n_admitted", "n_prefill_tokens", "n_decoded", "n_active",
                                         "n_preempted")]


class rlhf_stage_opts(C.Structure):
    _fields_ = [("fused", C.c_int32), ("R_t", C.c_int32), ("score_chunk_tokens", C.c_int32),
                ("role_mask", C.c_uint32), ("trace_active", C.c_void_p), ("trace_decoded", C.c_void_p),
                ("trace_step_ms", C.c_void_p), ("trace_step_bytes", C.c_void_p),
                ("trace_prefill_tokens", C.c_void_p), ("trace_cap", C.c_int32)]


class rlhf_stage_stats(C.Structure):
    _fields_ = [("n_steps", C.c_int32), ("n_batches", C.c_int32), ("generated_tokens", C.c_int64),
                ("scored_tokens", C.c_int64), ("prefill_tokens", C.c_int64), ("wall_ms", C.c_double),
                ("decode_stream_ms", C.c_double), ("score_stream_ms", C.c_double),
                ("decode_weight_bytes", C.c_int64), ("decode_kv_bytes", C.c_int64), ("fused_used", C.c_int32)]


class rlhf_results(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("gen_len", "resp_offsets", "tokens", "lp_actor", "lp_actor_rescored",
                                          "lp_ref", "values", "reward")] + [("packed_capacity", C.c_int64)]


class rlhf_snapshot(C.Structure):
    _fields_ = ([(n, C.c_int32) for n in ("step", "n_samples", "n_waiting", "n_active", "n_retired", "n_batches",
                                          "n_free", "reserved_pages", "pool_pages", "max_pages")]
                + [(n, C.c_void_p) for n in ("active", "ctx", "gen_len", "n_pages", "page_table", "free_list",
                                             "retired", "batch_offsets", "batch_step")]
                + [(n, C.c_int32) for n in ("cap_samples", "cap_max_pages", "cap_pool_pages")])


class rlhf_kernel_profile(C.Structure):
    _fields_ = [("launches", C.c_int64), ("sampled", C.c_int64), ("sampled_ms", C.c_double),
                ("sampled_bytes", C.c_double), ("sampled_flops", C.c_double), ("total_bytes", C.c_double),
                ("total_flops", C.c_double), ("dropped", C.c_int64), ("bracket_overhead_ms", C.c_double)]


KERNEL_CLASSES = ("gemm_decode", "gemm_batch", "attn_decode", "attn_batch")

_lib = None


def lib() -> C.CDLL:
    """Load librlhf.so (built in-tree by paper_2409_13221_amd.build).  Fails loudly."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2409_13221_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32
        L.rlhf_create.argtypes = [C.POINTER(rlhf_model_cfg), C.POINTER(rlhf_engine_cfg), C.POINTER(vp)]
        L.rlhf_destroy.argtypes = [vp]
        L.rlhf_destroy.restype = None
        L.rlhf_last_error.argtypes = [vp]
        L.rlhf_last_error.restype = C.c_char_p
        L.rlhf_load_weights.argtypes = [vp, C.c_int, C.POINTER(rlhf_weights)]
        L.rlhf_submit.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
        L.rlhf_generate_step.argtypes = [vp, C.POINTER(rlhf_step_info)]
        L.rlhf_retire.argtypes = [vp, vp, C.POINTER(i32)]
        L.rlhf_migrate.argtypes = [vp, vp, i32, i32]
        L.rlhf_score.argtypes = [vp, i32, vp, u32, i32]
        L.rlhf_run_stage.argtypes = [vp, C.POINTER(rlhf_stage_opts), C.POINTER(rlhf_stage_stats)]
        L.rlhf_get_results.argtypes = [vp, C.POINTER(rlhf_results)]
        L.rlhf_debug_snapshot.argtypes = [vp, C.POINTER(rlhf_snapshot)]
        L.rlhf_sync.argtypes = [vp]
        L.rlhf_compute_gae.argtypes = [vp, C.c_float, C.c_float, C.c_float, vp, vp, i64]
        L.rlhf_profile_begin.argtypes = [vp, i32]
        L.rlhf_profile_end.argtypes = [vp, C.POINTER(rlhf_kernel_profile)]
        L.rlhf_op_gemm_nsplit.argtypes = [C.c_int] * 5
        L.rlhf_op_gemm.argtypes = [C.c_int, C.c_int, vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, vp]
        L.rlhf_op_paged_decode_attention.argtypes = [C.c_int, vp, vp, vp, C.c_int, vp, vp, vp, vp, vp] + [C.c_int] * 7 + [vp]
        L.rlhf_op_paged_decode_attention_noalloc.argtypes = [C.c_int, vp, vp, vp, C.c_int, vp, vp, vp] + [C.c_int] * 7 + [vp]
        L.rlhf_op_varlen_attention.argtypes = [C.c_int, vp, vp, vp, vp, vp, vp] + [C.c_int] * 4 + [vp]
        L.rlhf_op_flash_attention.argtypes = [vp] * 7 + [C.c_int] * 5 + [vp]
        L.rlhf_op_gemm_swiglu.argtypes = [C.c_int, vp, vp, vp, C.c_int, C.c_int, C.c_int, vp]
        L.rlhf_op_gemm_rope.argtypes = [C.c_int] + [vp] * 9 + [C.c_int] * 7 + [vp]
        f32 = C.c_float
        L.rlhf_op_rmsnorm.argtypes = [C.c_int, vp, vp, C.c_int, i64, vp, vp, vp, C.c_int, C.c_int, f32, vp]
        L.rlhf_op_rope_kv.argtypes = [C.c_int, vp, C.c_int, i64] + [vp] * 7 + [C.c_int] * 6 + [vp]
        L.rlhf_op_swiglu.argtypes = [C.c_int, vp, C.c_int, i64, vp, C.c_int, C.c_int, vp]
        L.rlhf_op_pick_scratch_floats.argtypes = [C.c_int]
        L.rlhf_op_pick_scratch_floats.restype = i64
        L.rlhf_op_pick.argtypes = [vp, C.c_int, i64, C.c_int, C.c_int] + [vp] * 8
        L.rlhf_op_gather_lp.argtypes = [vp, C.c_int, i64, C.c_int, C.c_int] + [vp] * 5
        L.rlhf_op_head_dot.argtypes = [C.c_int, C.c_int, vp, vp, C.c_int, C.c_int, vp, vp, vp]
        L.rlhf_op_lm_head_logprob_scratch_floats.argtypes = [C.c_int, C.c_int]
        L.rlhf_op_lm_head_logprob_scratch_floats.restype = i64
        L.rlhf_op_lm_head_logprob.argtypes = [C.c_int] + [vp] * 7 + [C.c_int] * 3 + [vp]
        L.rlhf_op_lm_head_logprob.restype = C.c_int
        L.rlhf_op_gemm_tall_grid.argtypes = [C.c_int, C.c_int]
        L.rlhf_op_gemm_tall_grid.restype = C.c_int
        L.rlhf_op_gemm_tall_tile.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.rlhf_op_gemm_tall_tile.restype = C.c_int
        L.rlhf_op_bf16_to_half.argtypes = [vp, vp, i64, vp]
        L.rlhf_op_bf16_to_half.restype = C.c_int
        for name in ("rlhf_op_rmsnorm", "rlhf_op_rope_kv", "rlhf_op_swiglu", "rlhf_op_pick", "rlhf_op_gather_lp",
                     "rlhf_op_head_dot"):
            getattr(L, name).restype = C.c_int
        for name in ("rlhf_create", "rlhf_load_weights", "rlhf_submit", "rlhf_generate_step", "rlhf_retire",
                     "rlhf_migrate", "rlhf_score", "rlhf_run_stage", "rlhf_get_results", "rlhf_debug_snapshot", "rlhf_sync",
                     "rlhf_profile_begin", "rlhf_profile_end", "rlhf_compute_gae",
                     "rlhf_op_gemm_nsplit", "rlhf_op_gemm", "rlhf_op_paged_decode_attention",
                     "rlhf_op_paged_decode_attention_noalloc",
                     "rlhf_op_varlen_attention", "rlhf_op_flash_attention", "rlhf_op_gemm_swiglu",
                     "rlhf_op_gemm_rope"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(ctx, rc: int):
    if rc != RLHF_OK:
        raise RlhfError(rc, lib().rlhf_last_error(ctx).decode())


def _np(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


# ------------------------------------------------------------------------------ stage API

def model_cfg_of(m) -> rlhf_model_cfg:
    """rlhf_model_cfg from any object with the fields of workload.ModelCfg."""
    return rlhf_model_cfg(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn, m.vocab,
                          RLHF_FP32 if m.dtype == "fp32" else RLHF_BF16, m.rms_eps, m.rope_base)


def rlhf_create(model: rlhf_model_cfg, engine: rlhf_engine_cfg) -> C.c_void_p:
    ctx = C.c_void_p()
    rc = lib().rlhf_create(C.byref(model), C.byref(engine), C.byref(ctx))
    _check(None, rc)
    return ctx


def rlhf_destroy(ctx) -> None:
    lib().rlhf_destroy(ctx)


def rlhf_last_error(ctx) -> str:
    return lib().rlhf_last_error(ctx).decode()


def rlhf_load_weights(ctx, role: int, tensors: Dict[str, "torch.Tensor"]) -> None:
    """tensors: name -> contiguous device tensor (the layout of rlhf_weights).  The caller keeps
    them alive until rlhf_destroy."""
    w = rlhf_weights()
    for name, _ in rlhf_weights._fields_:
        t = tensors[name]
        if not t.is_contiguous() or not t.is_cuda:
            raise ValueError(f"weight {name} must be a contiguous device tensor")
        setattr(w, name, t.data_ptr())
    _check(ctx, lib().rlhf_load_weights(ctx, role, C.byref(w)))


def rlhf_submit(ctx, prompt_tokens, prompt_offsets, max_new, forced_len=None, forced_tokens=None,
                forced_offsets=None) -> None:
    pt, po, mn = _np(prompt_tokens, np.int32), _np(prompt_offsets, np.int64), _np(max_new, np.int32)
    fl = None if forced_len is None else _np(forced_len, np.int32)
    ft = None if forced_tokens is None else _np(forced_tokens, np.int32)
    fo = None if forced_offsets is None else _np(forced_offsets, np.int64)
    _check(ctx, lib().rlhf_submit(ctx, len(mn), _p(pt), _p(po), _p(mn), _p(fl), _p(ft), _p(fo)))


def rlhf_generate_step(ctx) -> rlhf_step_info:
    info = rlhf_step_info()
    _check(ctx, lib().rlhf_generate_step(ctx, C.byref(info)))
    return info


def rlhf_retire(ctx, capacity: int) -> np.ndarray:
    ids = np.zeros(max(capacity, 1), np.int32)
    n = C.c_int32()
    _check(ctx, lib().rlhf_retire(ctx, _p(ids), C.byref(n)))
    return ids[:n.value].copy()


def rlhf_migrate(ctx, sample_ids: Sequence[int], to_back: bool = False) -> None:
    ids = _np(sample_ids, np.int32)
    _check(ctx, lib().rlhf_migrate(ctx, _p(ids), len(ids), int(to_back)))


def rlhf_score(ctx, sample_ids: Sequence[int], role_mask: int, on_score_stream: bool = True) -> None:
    ids = _np(sample_ids, np.int32)
    _check(ctx, lib().rlhf_score(ctx, len(ids), _p(ids), role_mask, int(on_score_stream)))


def rlhf_run_stage(ctx, fused: bool, R_t: int, score_chunk_tokens: int, role_mask: int,
                   trace_cap: int = 0, trace_time: bool = False):
    """fused: True, False, or "auto" (the library picks the plan).  Returns (rlhf_stage_stats, trace dict or None)."""
    o = rlhf_stage_opts(2 if fused == "auto" else int(fused), R_t, score_chunk_tokens, role_mask, None, None, None,
                        None, None, 0)
    tr = None
    if trace_cap > 0:
        tr = {"active": np.zeros(trace_cap, np.int32), "decoded": np.zeros(trace_cap, np.int32),
              "step_bytes": np.zeros(trace_cap, np.int64), "prefill_tokens": np.zeros(trace_cap, np.int32)}
        o.trace_active, o.trace_decoded, o.trace_cap = _p(tr["active"]), _p(tr["decoded"]), trace_cap
        o.trace_step_bytes, o.trace_prefill_tokens = _p(tr["step_bytes"]), _p(tr["prefill_tokens"])
        if trace_time:
            tr["step_ms"] = np.zeros(trace_cap, np.float32)
            o.trace_step_ms = _p(tr["step_ms"])
    st = rlhf_stage_stats()
    _check(ctx, lib().rlhf_run_stage(ctx, C.byref(o), C.byref(st)))
    if tr is not None:
        tr = {k: v[:st.n_steps] for k, v in tr.items()}
    return st, tr


def rlhf_get_results(ctx, n: int, packed_capacity: int) -> Dict[str, np.ndarray]:
    out = {"gen_len": np.zeros(n, np.int32), "resp_offsets": np.zeros(n + 1, np.int64),
           "tokens": np.zeros(packed_capacity, np.int32)}
    for k in ("lp_actor", "lp_actor_rescored", "lp_ref", "values"):
        out[k] = np.full(packed_capacity, np.nan, np.float32)
    out["reward"] = np.full(n, np.nan, np.float32)
    r = rlhf_results()
    for name, _ in rlhf_results._fields_[:-1]:
        setattr(r, name, _p(out[name]))
    r.packed_capacity = packed_capacity
    _check(ctx, lib().rlhf_get_results(ctx, C.byref(r)))
    total = int(out["resp_offsets"][-1])
    for k in ("tokens", "lp_actor", "lp_actor_rescored", "lp_ref", "values"):
        out[k] = out[k][:total]
    return out


def rlhf_debug_snapshot(ctx, cap_samples: int, cap_max_pages: int, cap_pool_pages: int) -> dict:
    a = {k: np.full(cap_samples, -1, np.int32) for k in ("active", "ctx", "gen_len", "n_pages", "retired",
                                                         "batch_step")}
    a["page_table"] = np.full(cap_samples * cap_max_pages, -1, np.int32)
    a["free_list"] = np.full(max(cap_pool_pages, 1), -1, np.int32)
    a["batch_offsets"] = np.zeros(cap_samples + 1, np.int32)
    s = rlhf_snapshot()
    for k, v in a.items():
        setattr(s, k, _p(v))
    s.cap_samples, s.cap_max_pages, s.cap_pool_pages = cap_samples, cap_max_pages, cap_pool_pages
    _check(ctx, lib().rlhf_debug_snapshot(ctx, C.byref(s)))
    n = s.n_samples
    pt = a["page_table"].reshape(cap_samples, cap_max_pages)
    retired = a["retired"][:s.n_retired].tolist()
    bo = a["batch_offsets"][:s.n_batches + 1].tolist()
    return {
        "step": s.step, "n_waiting": s.n_waiting, "reserved": s.reserved_pages, "pool_pages": s.pool_pages,
        "active": a["active"][:s.n_active].tolist(),
        "ctx": a["ctx"][:n].tolist(), "gen_len": a["gen_len"][:n].tolist(),
        "pages": [pt[i, :a["n_pages"][i]].tolist() for i in range(n)],
        "free": a["free_list"][:s.n_free].tolist(),
        "retired": retired,
        "batches": [retired[bo[b]:bo[b + 1]] for b in range(s.n_batches)],
        "batch_step": a["batch_step"][:s.n_batches].tolist(),
    }


def rlhf_sync(ctx) -> None:
    _check(ctx, lib().rlhf_sync(ctx))


def rlhf_compute_gae(ctx, gamma: float, lam: float, kl_coef: float, packed_capacity: int):
    """Returns (advantages, returns), float32 arrays of packed_capacity entries (the caller
    trims them with resp_offsets)."""
    adv = np.full(packed_capacity, np.nan, np.float32)
    ret = np.full(packed_capacity, np.nan, np.float32)
    _check(ctx, lib().rlhf_compute_gae(ctx, gamma, lam, kl_coef, _p(adv), _p(ret), packed_capacity))
    return adv, ret


def rlhf_profile_begin(ctx, sample_every: int = 1) -> None:
    _check(ctx, lib().rlhf_profile_begin(ctx, sample_every))


def rlhf_profile_end(ctx) -> Dict[str, dict]:
    arr = (rlhf_kernel_profile * 4)()
    _check(ctx, lib().rlhf_profile_end(ctx, arr))
    return {name: {f: getattr(arr[k], f) for f, _ in rlhf_kernel_profile._fields_}
            for k, name in enumerate(KERNEL_CLASSES)}


# ------------------------------------------------------------------------- kernel-level API

def _dt(t) -> int:
    import torch
    return RLHF_BF16 if t.dtype == torch.bfloat16 else RLHF_FP32


def _stream_ptr():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _op_check(rc: int, what: str):
    if rc != RLHF_OK:
        raise RlhfError(rc, what)


def _half_code(A, W) -> int:
    """act_half argument of the fused-epilogue GEMMs: 0 bf16 x bf16, 1 half x bf16, 2 half x half copy."""
    import torch
    if W.dtype == torch.float16:
        assert A.dtype == torch.float16
        return 2
    return int(A.dtype == torch.float16)


def rlhf_op_bf16_to_half(W):
    """IEEE-half copy of a bfloat16 tensor, converted by the library's own kernel."""
    import torch
    assert W.dtype == torch.bfloat16 and W.is_contiguous() and W.numel() % 2 == 0
    out = torch.empty_like(W, dtype=torch.float16)
    _op_check(lib().rlhf_op_bf16_to_half(W.data_ptr(), out.data_ptr(), W.numel(), _stream_ptr()), "rlhf_op_bf16_to_half")
    return out


def rlhf_op_gemm_nsplit(dtype: int, M: int, N: int, K: int, max_split: int) -> int:
    return lib().rlhf_op_gemm_nsplit(dtype, M, N, K, max_split)


def rlhf_op_gemm(A, W, C_out, nsplit: int, variant: int = 0) -> None:
    """W [N,K] (bf16 or fp32), A [M,K] of W's dtype or float16 (with bf16 W), C_out float32
    [nsplit, M, N]; on torch's current stream."""
    import torch
    M, K = A.shape
    N = W.shape[0]
    assert W.shape[1] == K and tuple(C_out.shape) == (nsplit, M, N) and A.is_contiguous() and W.is_contiguous()
    half = A.dtype == torch.float16
    assert half or A.dtype == W.dtype
    wcode = 2 if W.dtype == torch.float16 else _dt(W)            # float16 W: a half copy of bf16 weights
    _op_check(lib().rlhf_op_gemm(wcode, int(half), A.data_ptr(), W.data_ptr(), C_out.data_ptr(), M, N, K, nsplit,
                                 variant, _stream_ptr()), "rlhf_op_gemm")


def rlhf_op_paged_decode_attention(q, pool, page_table, row_sample, ctx_len, out, part_acc, part_ml, layer: int,
                                   nsplit: int, n_layers: int, n_q_heads: int, n_kv_heads: int, head_dim: int):
    import torch
    rows = q.shape[0]
    _op_check(lib().rlhf_op_paged_decode_attention(
        2 if q.dtype == torch.float16 else _dt(q), q.data_ptr(), pool.data_ptr(), page_table.data_ptr(), page_table.shape[1], row_sample.data_ptr(),
        ctx_len.data_ptr(), out.data_ptr(), part_acc.data_ptr() if part_acc is not None else None,
        part_ml.data_ptr() if part_ml is not None else None, rows, layer, nsplit, n_layers, n_q_heads,
        n_kv_heads, head_dim, _stream_ptr()), "rlhf_op_paged_decode_attention")


def rlhf_op_paged_decode_attention_noalloc(q, pool, page_table, row_sample, ctx_len, out, layer: int, nsplit: int,
                                           n_layers: int, n_q_heads: int, n_kv_heads: int, head_dim: int):
    """The same attention with the library's built-in scratch for the split partials (no allocation)."""
    import torch
    rc = lib().rlhf_op_paged_decode_attention_noalloc(
        2 if q.dtype == torch.float16 else _dt(q), q.data_ptr(), pool.data_ptr(), page_table.data_ptr(),
        page_table.shape[1], row_sample.data_ptr(), ctx_len.data_ptr(), out.data_ptr(), q.shape[0], layer, nsplit,
        n_layers, n_q_heads, n_kv_heads, head_dim, _stream_ptr())
    if rc != RLHF_OK:
        raise RlhfError(rc, lib().rlhf_last_error(None).decode())


def rlhf_op_varlen_attention(q, k, v, row_start, row_pos, out, n_q_heads: int, n_kv_heads: int, head_dim: int):
    """float32 q, k, v; out float16 or float32."""
    import torch
    assert q.dtype == k.dtype == v.dtype == torch.float32 and out.dtype in (torch.float16, torch.float32)
    _op_check(lib().rlhf_op_varlen_attention(int(out.dtype == torch.float16), q.data_ptr(), k.data_ptr(), v.data_ptr(), row_start.data_ptr(),
                                             row_pos.data_ptr(), out.data_ptr(), q.shape[0], n_q_heads, n_kv_heads,
                                             head_dim, _stream_ptr()), "rlhf_op_varlen_attention")


def rlhf_op_flash_attention(q, k, v, seq_lens, out, n_q_heads: int, n_kv_heads: int, head_dim: int):
    """float16 q [T, Hq*hd], k, v [T, Hkv*hd], out like q; sequences of seq_lens packed back to back."""
    import torch
    assert q.dtype == k.dtype == v.dtype == out.dtype == torch.float16
    ts, tq, tl, start = [], [], [], 0
    for L in seq_lens:
        for q0 in range(0, L, 128):
            ts.append(start); tq.append(q0); tl.append(L)
        start += L
    dev = lambda a: torch.tensor(a, dtype=torch.int32, device=q.device)
    d_ts, d_tq, d_tl = dev(ts), dev(tq), dev(tl)
    _op_check(lib().rlhf_op_flash_attention(q.data_ptr(), k.data_ptr(), v.data_ptr(), d_ts.data_ptr(), d_tq.data_ptr(),
                                            d_tl.data_ptr(), out.data_ptr(), len(ts), q.shape[0], n_q_heads,
                                            n_kv_heads, head_dim, _stream_ptr()), "rlhf_op_flash_attention")
    return d_ts, d_tq, d_tl          # keep alive until the stream has run


def rlhf_op_gemm_swiglu(A, W_gate_up, act) -> None:
    """A [M,K] float16 or bfloat16, W_gate_up bfloat16 [2f, K], act [M, f] of A's dtype."""
    import torch
    M, K = A.shape
    f = W_gate_up.shape[0] // 2
    assert W_gate_up.dtype in (torch.bfloat16, torch.float16) and act.dtype == A.dtype and tuple(act.shape) == (M, f)
    _op_check(lib().rlhf_op_gemm_swiglu(_half_code(A, W_gate_up), A.data_ptr(), W_gate_up.data_ptr(),
                                        act.data_ptr(), M, f, K, _stream_ptr()), "rlhf_op_gemm_swiglu")


def rlhf_op_gemm_rope(A, W_qkv, pos, table, q, k=None, v=None, pool=None, kv_dst=None, layer=0, n_layers=1,
                      n_q_heads=1, n_kv_heads=1, head_dim=64, check_indices=True) -> None:
    """A [M,K] float16 or bfloat16, W_qkv bfloat16 [(Hq+2Hkv)*hd, K], pos / kv_dst int32 [M], table float32
    [max_pos, hd/2, 2]; q, k, v (and pool) of A's dtype.  check_indices reads pos and kv_dst back to the host
    (a synchronisation) to make sure they stay inside table and pool; a caller that has checked them itself
    and times the kernel passes False."""
    import torch
    M, K = A.shape
    assert W_qkv.dtype in (torch.bfloat16, torch.float16) and tuple(W_qkv.shape) == ((n_q_heads + 2 * n_kv_heads) * head_dim, K)
    assert pos.dtype == torch.int32 and pos.numel() == M and table.dtype == torch.float32
    assert tuple(table.shape[1:]) == (head_dim // 2, 2)
    assert not check_indices or (0 <= int(pos.min()) and int(pos.max()) < table.shape[0])
    assert q.dtype == A.dtype and tuple(q.shape) == (M, n_q_heads * head_dim)
    for t in (k, v):
        assert t is None or (t.dtype == A.dtype and tuple(t.shape) == (M, n_kv_heads * head_dim))
    if pool is not None:
        assert pool.dtype == A.dtype and kv_dst is not None and kv_dst.dtype == torch.int32 and kv_dst.numel() == M
        page_elems = n_layers * 2 * n_kv_heads * 16 * head_dim
        assert pool.numel() % page_elems == 0
        assert not check_indices or (0 <= int(kv_dst.min()) and int(kv_dst.max()) < pool.numel() // page_elems * 16)
    ptr = lambda t: None if t is None else t.data_ptr()
    _op_check(lib().rlhf_op_gemm_rope(_half_code(A, W_qkv), A.data_ptr(), W_qkv.data_ptr(), pos.data_ptr(),
                                      ptr(kv_dst), table.data_ptr(), q.data_ptr(), ptr(k), ptr(v), ptr(pool), M, K,
                                      layer, n_layers, n_q_heads, n_kv_heads, head_dim, _stream_ptr()),
              "rlhf_op_gemm_rope")


def _act_code(t) -> int:
    import torch
    return {torch.float32: RLHF_FP32, torch.bfloat16: RLHF_BF16, torch.float16: 2}[t.dtype]


def _ptr(t):
    return None if t is None else t.data_ptr()


def rlhf_op_rmsnorm(h, part, g, xn, eps: float, row_idx=None) -> None:
    """h float32 [*, d] (updated in place when row_idx is None); part float32 [nsplit, rows_h, d] or None;
    g float32 [d]; xn [rows, d] float32 / bfloat16 / float16."""
    rows, d = xn.shape
    nsplit = 0 if part is None else part.shape[0]
    sstride = 0 if part is None else part.stride(0)
    _op_check(lib().rlhf_op_rmsnorm(_act_code(xn), h.data_ptr(), _ptr(part), nsplit, sstride, _ptr(row_idx),
                                    g.data_ptr(), xn.data_ptr(), rows, d, eps, _stream_ptr()), "rlhf_op_rmsnorm")


def rlhf_op_rope_kv(qkv, pos, table, q, k=None, v=None, pool=None, kv_dst=None, layer=0, n_layers=1, n_q_heads=1,
                    n_kv_heads=1, head_dim=64) -> None:
    """qkv float32 [nsplit, rows, (Hq+2Hkv)*hd]; q, k, v, pool of one activation dtype."""
    nsplit, rows, width = qkv.shape
    assert width == (n_q_heads + 2 * n_kv_heads) * head_dim and tuple(q.shape) == (rows, n_q_heads * head_dim)
    assert int(pos.max()) < table.shape[0] and int(pos.min()) >= 0
    if pool is not None:
        page_elems = n_layers * 2 * n_kv_heads * 16 * head_dim
        assert 0 <= int(kv_dst.min()) and int(kv_dst.max()) < pool.numel() // page_elems * 16
    _op_check(lib().rlhf_op_rope_kv(_act_code(q), qkv.data_ptr(), nsplit, qkv.stride(0), pos.data_ptr(), _ptr(kv_dst),
                                    table.data_ptr(), q.data_ptr(), _ptr(k), _ptr(v), _ptr(pool), layer, rows,
                                    n_layers, n_q_heads, n_kv_heads, head_dim, _stream_ptr()), "rlhf_op_rope_kv")


def rlhf_op_swiglu(gu, act) -> None:
    """gu float32 [nsplit, rows, 2*ffn]; act [rows, ffn]."""
    nsplit, rows, two_f = gu.shape
    assert tuple(act.shape) == (rows, two_f // 2)
    _op_check(lib().rlhf_op_swiglu(_act_code(act), gu.data_ptr(), nsplit, gu.stride(0), act.data_ptr(), rows,
                                   two_f // 2, _stream_ptr()), "rlhf_op_swiglu")


def rlhf_op_pick(logits, forced, tokens, tok_dst, lp, lp_dst, picked=None) -> None:
    """logits float32 [nsplit, rows, vocab]; forced int32 [rows] or None; tokens int32 buffer indexed by
    tok_dst [rows]; lp float32 buffer indexed by lp_dst [rows]."""
    import torch
    nsplit, rows, vocab = logits.shape
    assert int(tok_dst.max()) < tokens.numel() and int(lp_dst.max()) < lp.numel()
    scratch = torch.empty(max(1, lib().rlhf_op_pick_scratch_floats(rows)), device=logits.device)
    _op_check(lib().rlhf_op_pick(logits.data_ptr(), nsplit, logits.stride(0), rows, vocab, _ptr(forced),
                                 tokens.data_ptr(), tok_dst.data_ptr(), lp.data_ptr(), lp_dst.data_ptr(),
                                 _ptr(picked), scratch.data_ptr(), _stream_ptr()), "rlhf_op_pick")
    torch.cuda.current_stream().synchronize()          # scratch is released on return


def rlhf_op_gather_lp(logits, tokens, target_idx, out, out_dst) -> None:
    nsplit, rows, vocab = logits.shape
    assert int(target_idx.max()) < tokens.numel() and int(out_dst.max()) < out.numel()
    _op_check(lib().rlhf_op_gather_lp(logits.data_ptr(), nsplit, logits.stride(0), rows, vocab, tokens.data_ptr(),
                                      target_idx.data_ptr(), out.data_ptr(), out_dst.data_ptr(), _stream_ptr()),
              "rlhf_op_gather_lp")


def rlhf_op_head_dot(xn, w, out, out_dst) -> None:
    rows, d = xn.shape
    assert w.numel() == d and int(out_dst.max()) < out.numel()
    _op_check(lib().rlhf_op_head_dot(_act_code(xn), _dt(w), xn.data_ptr(), w.data_ptr(), rows, d, out.data_ptr(),
                                     out_dst.data_ptr(), _stream_ptr()), "rlhf_op_head_dot")


def rlhf_op_lm_head_logprob(A, W_head, tokens, target_idx, out, out_dst, scratch=None):
    """A [M, K] float16 / bfloat16, W_head bfloat16 [vocab, K]; out[out_dst[m]] = log-prob of token
    tokens[target_idx[m]] under row m's logits.  Returns the scratch tensor (keep it alive until the
    stream has run)."""
    import torch
    M, K = A.shape
    vocab = W_head.shape[0]
    assert W_head.dtype in (torch.bfloat16, torch.float16) and W_head.shape[1] == K and A.is_contiguous() and W_head.is_contiguous()
    assert int(target_idx.max()) < tokens.numel() and int(out_dst.max()) < out.numel()
    need = lib().rlhf_op_lm_head_logprob_scratch_floats(M, vocab)
    if scratch is None:
        scratch = torch.empty(max(need, 1), device=A.device)
    assert scratch.numel() >= need
    _op_check(lib().rlhf_op_lm_head_logprob(_half_code(A, W_head), A.data_ptr(), W_head.data_ptr(),
                                            tokens.data_ptr(), target_idx.data_ptr(), out.data_ptr(), out_dst.data_ptr(),
                                            scratch.data_ptr(), M, vocab, K, _stream_ptr()), "rlhf_op_lm_head_logprob")
    return scratch


def rlhf_op_gemm_tall_grid(tiles_m: int, tiles_n: int) -> int:
    return lib().rlhf_op_gemm_tall_grid(tiles_m, tiles_n)


def rlhf_op_gemm_tall_tile(bid: int, tiles_m: int, tiles_n: int):
    """(tm, tn) of workgroup bid, or None if it has no tile."""
    tm, tn = C.c_int(), C.c_int()
    rc = lib().rlhf_op_gemm_tall_tile(bid, tiles_m, tiles_n, C.byref(tm), C.byref(tn))
    if rc < 0:
        raise RlhfError(rc, "rlhf_op_gemm_tall_tile")
    return (tm.value, tn.value) if rc == 1 else None
