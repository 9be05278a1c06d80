"""ctypes binding of libmimose.so: same names as the C ABI, marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmimose.so")

MIMOSE_OK = 0
MIMOSE_ERR_INVALID_ARG = -1
MIMOSE_ERR_OOM_BUDGET = -2
MIMOSE_ERR_BUDGET_INFEASIBLE = -3
MIMOSE_ERR_HIP = -4
MIMOSE_ERR_NOT_READY = -5
ERR_NAMES = {0: "OK", -1: "INVALID_ARG", -2: "OOM_BUDGET", -3: "BUDGET_INFEASIBLE", -4: "HIP", -5: "NOT_READY"}

Q_LAYER_KEPT, Q_LAYER_BOUNDARY, Q_LAYER_BWD, Q_EMBED, Q_HEAD, Q_FIXED, Q_LAYER_TIME = range(7)


class mimose_model_cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "hidden", "n_heads", "ffn", "vocab", "max_seq",
                 "dtype", "causal", "pre_ln", "gelu_tanh", "head")] + \
               [("ln_eps", C.c_float)] + \
               [(n, C.c_int32) for n in ("sheltered_steps", "bucket_tol_permille", "poly_order", "size_quantum")] + \
               [("reserve_bytes", C.c_uint64), ("guard_bytes", C.c_uint64)] + \
               [("ffn_by_layer", C.c_int32 * 64), ("cost_aware", C.c_int32), ("reserved_", C.c_int32)]


class mimose_stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in
                ("steps", "sheltered_steps", "cache_hits", "cache_misses", "cache_entries",
                 "planner_ns_last", "planner_ns_total", "recomputed_layers_last", "recomputed_layers_total")] + \
               [(n, C.c_double) for n in
                ("useful_flops_last", "recompute_flops_last", "useful_flops_total", "recompute_flops_total")] + \
               [(n, C.c_uint64) for n in
                ("peak_bytes_last", "peak_bytes_max", "predicted_peak_last", "fixed_bytes", "budget_bytes",
                 "plan_gen_count", "plan_gen_ns_total", "plan_gen_ns_min", "plan_gen_ns_max", "replans")]

    def as_dict(self) -> dict:
        return {n: getattr(self, n) for n, _ in self._fields_}


class mimose_adamw_cfg(C.Structure):
    _fields_ = [(n, C.c_float) for n in ("lr", "beta1", "beta2", "eps", "weight_decay")]


class MimoseError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libmimose: {ERR_NAMES.get(code, code)}: {msg}")
        self.code = code


_lib = None
_vp, _i32, _i64, _u64, _f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float

# name -> (restype, argtypes); every symbol include/mimose.h declares
SIGNATURES = {
    "mimose_init": (C.c_int, [C.POINTER(mimose_model_cfg), _u64, _vp, _u64, _vp, C.POINTER(_vp)]),
    "mimose_param_count": (C.c_int, [_vp, C.POINTER(_i32)]),
    "mimose_param_info": (C.c_int, [_vp, _i32, C.POINTER(C.c_char_p), C.POINTER(_i64), C.POINTER(_i32)]),
    "mimose_load_param": (C.c_int, [_vp, _i32, _vp, _u64]),
    "mimose_train_step": (C.c_int, [_vp, _vp, _vp, _i32, _i32, C.POINTER(_f32), C.POINTER(_u64), C.POINTER(_u64)]),
    "mimose_train_step_padded": (C.c_int, [_vp, _vp, _vp, _vp, _i32, _i32, C.POINTER(_f32), C.POINTER(_u64),
                                           C.POINTER(_u64)]),
    "mimose_sync_loss": (C.c_int, [_vp, C.POINTER(_f32)]),
    "mimose_set_collector": (C.c_int, [_vp, _i32]),
    "mimose_set_dropout": (C.c_int, [_vp, _f32, _f32, _u64, _u64]),
    "mimose_op_dropout": (C.c_int, [_i32, _vp, _vp, _i32, _vp, _i64, _f32, _u64, C.c_uint32, C.c_uint32, _vp]),
    "mimose_dry_step": (C.c_int, [_vp, _i32, _i32, C.POINTER(_u64), C.POINTER(_u64)]),
    "mimose_get_grad": (C.c_int, [_vp, _i32, _vp, _u64]),
    "mimose_get_param": (C.c_int, [_vp, _i32, _vp, _u64]),
    "mimose_optimizer_init": (C.c_int, [_vp, _vp]),
    "mimose_optimizer_step": (C.c_int, [_vp]),
    "mimose_force_plan": (C.c_int, [_vp, _i64]),
    "mimose_set_plan_mode": (C.c_int, [_vp, _i32]),
    "mimose_planner_feed": (C.c_int, [_vp, _i32, _i32, _i32, _i32, _u64]),
    "mimose_planner_end_step": (C.c_int, [_vp, _i32, _i32]),
    "mimose_planner_query": (C.c_int, [_vp, _i32, _i32, C.POINTER(_u64), C.POINTER(_u64)]),
    "mimose_profile_enable": (C.c_int, [_vp, _i32]),
    "mimose_profile_read": (C.c_int, [_vp, _i32, C.POINTER(_u64), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "mimose_get_layer_times": (C.c_int, [_vp, _vp]),
    "mimose_get_step_memory": (C.c_int, [_vp, C.POINTER(_u64), C.POINTER(_u64), C.POINTER(_u64), _vp, _vp, _vp]),
    "mimose_get_stats": (C.c_int, [_vp, C.POINTER(mimose_stats)]),
    "mimose_last_error": (C.c_char_p, [_vp]),
    "mimose_destroy": (None, [_vp]),
    "mimose_op_gemm": (C.c_int, [_i32, _vp, _i64, _i32, _vp, _i64, _i32, _vp, _i64, _i32, _i32, _i32, _i32,
                                 _vp, _vp, _i64, _vp, _i32, _vp, _vp, _u64, _vp]),
    "mimose_op_gemm_workspace_bytes": (_u64, [_i32, _i32]),
    "mimose_op_gemm_long_k_workspace_bytes": (_u64, [_i32]),
    "mimose_op_layernorm_fwd": (C.c_int, [_i32, _vp, _i32, _vp, _vp, _vp, _i32, _i32, _f32, _vp]),
    "mimose_op_layernorm_bwd": (C.c_int, [_i32, _vp, _i32, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _f32,
                                          _vp]),
    "mimose_op_partial_rows": (_i32, [_i32]),
    "mimose_op_layernorm_bwd_noalloc": (C.c_int, [_i32, _vp, _i32, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _f32,
                                                  _vp]),
    "mimose_op_layernorm_bwd_noalloc_max_floats": (_u64, []),
    "mimose_op_gelu_bwd": (C.c_int, [_i32, _vp, _vp, _i64, _i32, _vp]),
    "mimose_op_attention_fwd": (C.c_int, [_i32, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _f32, _u64, C.c_uint32,
                                          C.c_uint32, _vp]),
    "mimose_op_attention_bwd": (C.c_int, [_i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _f32,
                                          _u64, C.c_uint32, C.c_uint32, _vp]),
    "mimose_op_softmax_xent": (C.c_int, [_i32, _vp, _i64, _vp, _vp, _vp, _i32, _i32, _i32, _vp]),
    "mimose_op_embed_fwd": (C.c_int, [_i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _f32, _i32, _vp]),
    "mimose_op_embed_bwd": (C.c_int, [_i32, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _i32, _i32, _i32, _i32, _vp]),
}


def load_library():
    """Loads libmimose.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2209_02478_amd.build`")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _ptr(x) -> Optional[int]:
    """Address of a torch tensor (device or host), numpy array, int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return x.data_ptr()


def _check(code: int, ctx=None):
    if code != MIMOSE_OK:
        msg = load_library().mimose_last_error(ctx)
        raise MimoseError(code, msg.decode() if msg else "")


def make_cfg(shape: dict, **planner) -> mimose_model_cfg:
    """shape: dict with the model fields (dtype as 'fp32' / 'bf16' or 0 / 1)."""
    c = mimose_model_cfg()
    for k in ("n_layers", "hidden", "n_heads", "ffn", "vocab", "max_seq", "causal", "pre_ln", "gelu_tanh", "head"):
        setattr(c, k, int(shape[k]))
    dt = shape.get("dtype", 0)
    c.dtype = {"fp32": 0, "bf16": 1}.get(dt, dt)
    c.ln_eps = float(shape.get("ln_eps", 1e-5))
    for l, w in enumerate(shape.get("ffn_by_layer", ()) or ()):
        c.ffn_by_layer[l] = int(w)
    for k, v in planner.items():
        setattr(c, k, v)
    return c


# ---------------------------------------------------------------- C ABI, same names
def mimose_init(cfg: mimose_model_cfg, mem_budget_bytes: int, arena=None, arena_bytes: int = 0, hip_stream=None):
    lib = load_library()
    out = _vp()
    if arena is not None and not isinstance(arena, int):
        arena_bytes = arena_bytes or arena.numel() * arena.element_size()
    code = lib.mimose_init(C.byref(cfg), mem_budget_bytes, _ptr(arena), arena_bytes, _ptr(hip_stream), C.byref(out))
    _check(code, None)
    return out


def mimose_param_count(ctx) -> int:
    n = _i32()
    _check(load_library().mimose_param_count(ctx, C.byref(n)), ctx)
    return n.value


def mimose_param_info(ctx, i: int) -> Tuple[str, Tuple[int, ...]]:
    name = C.c_char_p()
    shape = (_i64 * 4)()
    nd = _i32()
    _check(load_library().mimose_param_info(ctx, i, C.byref(name), shape, C.byref(nd)), ctx)
    return name.value.decode(), tuple(shape[k] for k in range(nd.value))


def mimose_load_param(ctx, i: int, host_fp32: np.ndarray):
    a = np.ascontiguousarray(host_fp32, dtype=np.float32)
    _check(load_library().mimose_load_param(ctx, i, a.ctypes.data, a.size), ctx)


def mimose_train_step(ctx, tokens: np.ndarray, labels: np.ndarray, wait: bool = True):
    """wait=False passes loss = NULL: the iteration is queued, the loss returned is None."""
    t = np.ascontiguousarray(tokens, dtype=np.int32)
    l = np.ascontiguousarray(labels, dtype=np.int32)
    B, L = t.shape
    loss, peak, plan = _f32(), _u64(), _u64()
    _check(load_library().mimose_train_step(ctx, t.ctypes.data, l.ctypes.data, B, L, C.byref(loss) if wait else None,
                                            C.byref(peak), C.byref(plan)), ctx)
    return (loss.value if wait else None), peak.value, plan.value


def mimose_sync_loss(ctx) -> float:
    loss = _f32()
    _check(load_library().mimose_sync_loss(ctx, C.byref(loss)), ctx)
    return loss.value


def mimose_train_step_padded(ctx, tokens: np.ndarray, labels: np.ndarray, lengths: np.ndarray, wait: bool = True):
    t = np.ascontiguousarray(tokens, dtype=np.int32)
    l = np.ascontiguousarray(labels, dtype=np.int32)
    n = np.ascontiguousarray(lengths, dtype=np.int32)
    B, L = t.shape
    if n.shape != (B,):
        raise ValueError("lengths must have one entry per sample")
    loss, peak, plan = _f32(), _u64(), _u64()
    _check(load_library().mimose_train_step_padded(ctx, t.ctypes.data, l.ctypes.data, n.ctypes.data, B, L,
                                                   C.byref(loss) if wait else None, C.byref(peak), C.byref(plan)), ctx)
    return (loss.value if wait else None), peak.value, plan.value


def mimose_dry_step(ctx, B: int, L: int) -> Tuple[int, int]:
    peak, plan = _u64(), _u64()
    _check(load_library().mimose_dry_step(ctx, B, L, C.byref(peak), C.byref(plan)), ctx)
    return peak.value, plan.value


def mimose_get_grad(ctx, i: int, n_elems: int) -> np.ndarray:
    out = np.empty(n_elems, dtype=np.float32)
    _check(load_library().mimose_get_grad(ctx, i, out.ctypes.data, n_elems), ctx)
    return out


def mimose_get_param(ctx, i: int, n_elems: int) -> np.ndarray:
    out = np.empty(n_elems, dtype=np.float32)
    _check(load_library().mimose_get_param(ctx, i, out.ctypes.data, n_elems), ctx)
    return out


def mimose_optimizer_init(ctx, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
    cfg = mimose_adamw_cfg(lr, beta1, beta2, eps, weight_decay)
    _check(load_library().mimose_optimizer_init(ctx, C.addressof(cfg)), ctx)


def mimose_optimizer_step(ctx):
    _check(load_library().mimose_optimizer_step(ctx), ctx)


def mimose_force_plan(ctx, plan: int):
    _check(load_library().mimose_force_plan(ctx, plan), ctx)


PLAN_MODES = {"input_aware": 0, "static_max": 1, "all": 2, "none": 3}


def mimose_set_plan_mode(ctx, mode: int):
    _check(load_library().mimose_set_plan_mode(ctx, mode), ctx)


COLLECTORS = {"marks": 0, "two_forwards": 1}


def mimose_set_collector(ctx, mode: int):
    _check(load_library().mimose_set_collector(ctx, mode), ctx)


def mimose_planner_feed(ctx, B: int, L: int, quantity: int, layer: int, nbytes: int):
    _check(load_library().mimose_planner_feed(ctx, B, L, quantity, layer, nbytes), ctx)


def mimose_planner_end_step(ctx, B: int, L: int):
    _check(load_library().mimose_planner_end_step(ctx, B, L), ctx)


def mimose_planner_query(ctx, B: int, L: int) -> Tuple[int, int]:
    plan, peak = _u64(), _u64()
    _check(load_library().mimose_planner_query(ctx, B, L, C.byref(plan), C.byref(peak)), ctx)
    return plan.value, peak.value


KERNEL_CLASSES = ("gemm", "attention_fwd", "attention_bwd", "layernorm_fwd", "layernorm_bwd", "gelu_bwd",
                  "softmax_xent", "embed_fwd")


def mimose_profile_enable(ctx, on: int):
    _check(load_library().mimose_profile_enable(ctx, on), ctx)


def mimose_profile_read(ctx, kernel_class: int) -> Tuple[int, float, float]:
    n, ms, work = _u64(), C.c_double(), C.c_double()
    _check(load_library().mimose_profile_read(ctx, kernel_class, C.byref(n), C.byref(ms), C.byref(work)), ctx)
    return n.value, ms.value, work.value


def mimose_get_step_memory(ctx, n_layers: int) -> dict:
    F, e, g = _u64(), _u64(), _u64()
    a, b, w = (np.zeros(n_layers, dtype=np.uint64) for _ in range(3))
    _check(load_library().mimose_get_step_memory(ctx, C.byref(F), C.byref(e), C.byref(g), a.ctypes.data,
                                                 b.ctypes.data, w.ctypes.data), ctx)
    return dict(F=F.value, e=e.value, g=g.value, a=[int(v) for v in a], b=[int(v) for v in b],
                w=[int(v) for v in w])


def mimose_get_layer_times(ctx, n_layers: int) -> list:
    t = np.zeros(n_layers, dtype=np.uint64)
    _check(load_library().mimose_get_layer_times(ctx, t.ctypes.data), ctx)
    return [int(v) for v in t]


def mimose_get_stats(ctx) -> dict:
    s = mimose_stats()
    _check(load_library().mimose_get_stats(ctx, C.byref(s)), ctx)
    return s.as_dict()


def mimose_last_error(ctx) -> str:
    m = load_library().mimose_last_error(ctx)
    return m.decode() if m else ""


def mimose_destroy(ctx):
    load_library().mimose_destroy(ctx)


# kernel-level entry points: device tensors in, same argument order as the header
def mimose_op_gemm(dtype, A, lda, a_kmajor, B, ldb, b_kmajor, Cm, ldc, c_f32, M, N, K, bias=None, resid=None, ldr=0,
                   gelu_out=None, gelu=0, a_rowsum=None, workspace=None, workspace_bytes=0, stream=None):
    _check(load_library().mimose_op_gemm(dtype, _ptr(A), lda, a_kmajor, _ptr(B), ldb, b_kmajor, _ptr(Cm), ldc, c_f32,
                                         M, N, K, _ptr(bias), _ptr(resid), ldr, _ptr(gelu_out), gelu, _ptr(a_rowsum),
                                         _ptr(workspace), workspace_bytes, _ptr(stream)))


def mimose_op_gemm_workspace_bytes(M: int, N: int) -> int:
    return load_library().mimose_op_gemm_workspace_bytes(M, N)


def mimose_op_gemm_long_k_workspace_bytes(N: int) -> int:
    return load_library().mimose_op_gemm_long_k_workspace_bytes(N)


def mimose_op_layernorm_fwd(dtype, x, x_f32, gamma, beta, y, T, H, eps, stream=None):
    _check(load_library().mimose_op_layernorm_fwd(dtype, _ptr(x), x_f32, _ptr(gamma), _ptr(beta), _ptr(y), T, H, eps,
                                                  _ptr(stream)))


def mimose_op_layernorm_bwd(dtype, dy, dy_f32, x, x_f32, gamma, dx, add, dgamma, dbeta, partial, T, H, eps,
                            stream=None):
    _check(load_library().mimose_op_layernorm_bwd(dtype, _ptr(dy), dy_f32, _ptr(x), x_f32, _ptr(gamma), _ptr(dx),
                                                  _ptr(add), _ptr(dgamma), _ptr(dbeta), _ptr(partial), T, H, eps,
                                                  _ptr(stream)))


def mimose_op_partial_rows(T: int) -> int:
    return load_library().mimose_op_partial_rows(T)


def mimose_op_layernorm_bwd_noalloc(dtype, dy, dy_f32, x, x_f32, gamma, dx, add, dgamma, dbeta, T, H, eps, stream=None):
    _check(load_library().mimose_op_layernorm_bwd_noalloc(dtype, _ptr(dy), dy_f32, _ptr(x), x_f32, _ptr(gamma), _ptr(dx),
                                                          _ptr(add), _ptr(dgamma), _ptr(dbeta), T, H, eps, _ptr(stream)))


def mimose_op_layernorm_bwd_noalloc_max_floats() -> int:
    return load_library().mimose_op_layernorm_bwd_noalloc_max_floats()


def mimose_op_gelu_bwd(dtype, d, pre, n, tanh_form, stream=None):
    _check(load_library().mimose_op_gelu_bwd(dtype, _ptr(d), _ptr(pre), n, tanh_form, _ptr(stream)))


def mimose_op_attention_fwd(dtype, qkv, ctx_out, lse, B, L, n_heads, head_dim, causal, stream=None, lengths=None,
                            p_drop=0.0, seed=0, site=0, step=0):
    _check(load_library().mimose_op_attention_fwd(dtype, _ptr(qkv), _ptr(ctx_out), _ptr(lse), _ptr(lengths), B, L,
                                                  n_heads, head_dim, causal, p_drop, seed, site, step, _ptr(stream)))


def mimose_op_attention_bwd(dtype, qkv, ctx_in, dctx, lse, delta, dqkv, B, L, n_heads, head_dim, causal, stream=None,
                            lengths=None, p_drop=0.0, seed=0, site=0, step=0):
    _check(load_library().mimose_op_attention_bwd(dtype, _ptr(qkv), _ptr(ctx_in), _ptr(dctx), _ptr(lse), _ptr(delta),
                                                  _ptr(dqkv), _ptr(lengths), B, L, n_heads, head_dim, causal, p_drop,
                                                  seed, site, step, _ptr(stream)))


def mimose_op_dropout(dtype, dst, src, io_f32, resid, n, p, seed, site, step, stream=None):
    _check(load_library().mimose_op_dropout(dtype, _ptr(dst), _ptr(src), int(io_f32), _ptr(resid), n, p, seed, site, step,
                                            _ptr(stream)))


def mimose_set_dropout(ctx, p_hidden: float, p_attn: float, seed: int, first_step: int = 0):
    _check(load_library().mimose_set_dropout(ctx, p_hidden, p_attn, seed, first_step), ctx)


def mimose_op_softmax_xent(dtype, logits, ld, labels, row_loss, loss, T, V, n_valid, stream=None):
    _check(load_library().mimose_op_softmax_xent(dtype, _ptr(logits), ld, _ptr(labels), _ptr(row_loss), _ptr(loss),
                                                 T, V, n_valid, _ptr(stream)))


def mimose_op_embed_fwd(dtype, ids, tok, pos, gamma, beta, sum_out, y, B, L, H, eps, has_ln, stream=None):
    _check(load_library().mimose_op_embed_fwd(dtype, _ptr(ids), _ptr(tok), _ptr(pos), _ptr(gamma), _ptr(beta),
                                              _ptr(sum_out), _ptr(y), B, L, H, eps, has_ln, _ptr(stream)))


def mimose_op_embed_bwd(dtype, d, ids, order, seg, n_seg, dtok, dpos, B, L, H, max_seq, stream=None):
    _check(load_library().mimose_op_embed_bwd(dtype, _ptr(d), _ptr(ids), _ptr(order), _ptr(seg), n_seg, _ptr(dtok),
                                              _ptr(dpos), B, L, H, max_seq, _ptr(stream)))


# ---------------------------------------------------------------- convenience wrapper
class Mimose:
    """Owns a context and (optionally) the torch-allocated device arena behind it."""

    def __init__(self, shape: dict, budget_bytes: int = 0, arena_bytes: int = 0, device: Optional[str] = "cuda:0",
                 **planner):
        self.cfg = make_cfg(shape, **planner)
        self.arena = None
        stream = None
        if device is not None:
            import torch
            if not torch.cuda.is_available():
                raise RuntimeError("a device context needs a GPU; pass device=None for a host-only context")
            nbytes = arena_bytes or budget_bytes
            if nbytes <= 0:
                raise ValueError("arena_bytes or budget_bytes must be given for a device context")
            self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
            stream = torch.cuda.current_stream(device).cuda_stream
            base = self.arena.data_ptr()
            aligned = (base + 255) // 256 * 256
            self.ctx = mimose_init(self.cfg, budget_bytes, aligned, nbytes, stream)
        else:
            self.ctx = mimose_init(self.cfg, budget_bytes, None, 0, None)
        self.names: List[str] = []
        self.shapes: Dict[str, Tuple[int, ...]] = {}
        for i in range(mimose_param_count(self.ctx)):
            n, s = mimose_param_info(self.ctx, i)
            self.names.append(n)
            self.shapes[n] = s

    def load_params(self, params: Dict[str, np.ndarray]):
        for i, n in enumerate(self.names):
            a = params[n]
            assert tuple(a.shape) == self.shapes[n], (n, a.shape, self.shapes[n])
            mimose_load_param(self.ctx, i, a)

    def train_step(self, tokens, labels, lengths=None, wait=True):
        if lengths is not None:
            return mimose_train_step_padded(self.ctx, tokens, labels, lengths, wait)
        return mimose_train_step(self.ctx, tokens, labels, wait)

    def sync_loss(self) -> float:
        return mimose_sync_loss(self.ctx)

    def set_dropout(self, p_hidden, p_attn=0.0, seed=0, first_step=0):
        mimose_set_dropout(self.ctx, p_hidden, p_attn, seed, first_step)

    def dry_step(self, B, L):
        return mimose_dry_step(self.ctx, B, L)

    def grads(self) -> Dict[str, np.ndarray]:
        return {n: mimose_get_grad(self.ctx, i, int(np.prod(self.shapes[n]))).reshape(self.shapes[n])
                for i, n in enumerate(self.names)}

    def force_plan(self, plan: int):
        mimose_force_plan(self.ctx, plan)

    def optimizer_init(self, **hyper):
        mimose_optimizer_init(self.ctx, **hyper)

    def optimizer_step(self):
        mimose_optimizer_step(self.ctx)

    def params(self) -> Dict[str, np.ndarray]:
        return {n: mimose_get_param(self.ctx, i, int(np.prod(self.shapes[n]))).reshape(self.shapes[n])
                for i, n in enumerate(self.names)}

    def set_plan_mode(self, mode):
        mimose_set_plan_mode(self.ctx, PLAN_MODES[mode] if isinstance(mode, str) else int(mode))

    def set_collector(self, mode):
        mimose_set_collector(self.ctx, COLLECTORS[mode] if isinstance(mode, str) else mode)

    def stats(self) -> dict:
        return mimose_get_stats(self.ctx)

    def step_memory(self) -> dict:
        return mimose_get_step_memory(self.ctx, self.cfg.n_layers)

    def layer_times(self) -> list:
        return mimose_get_layer_times(self.ctx, self.cfg.n_layers)

    def close(self):
        if self.ctx is not None:
            mimose_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


__all__ = [n for n in dir() if n.startswith("mimose_") or n.startswith("MIMOSE_") or n.startswith("Q_")] + \
          ["Mimose", "MimoseError", "make_cfg", "load_library", "LIB_PATH", "SIGNATURES", "ERR_NAMES", "KERNEL_CLASSES", "PLAN_MODES", "COLLECTORS"]
