"""ctypes binding of libflowprefill.so: the same entry points as include/flowprefill.h, argument
marshalling only.  Every operator runs in the library's HIP kernels; torch is used by callers for
device memory and streams.  There is no fallback: if the compiled library is missing, importing
this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflowprefill.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2602_16603_amd.csrc.build` "
        "(there is no CPU fallback for the prefill path)")

lib = C.CDLL(LIB_PATH)

FP_OK, FP_DONE, FP_PREEMPTED = 0, 1, 2
FP_ERR_INVALID, FP_ERR_OOM, FP_ERR_STATE, FP_ERR_DEVICE = -1, -2, -3, -4
FP_DTYPE_F32, FP_DTYPE_BF16 = 0, 1
FP_OPS_PER_LAYER = 9
FP_BOUNDARY_EVERY_OP, FP_BOUNDARY_PAPER_OPS, FP_BOUNDARY_LAYER, FP_BOUNDARY_NONE = 0x1FF, 0x15A, 0x100, 0x0
OP_NAMES = ("rmsnorm_attn", "qkv_proj", "rope_kvwrite", "attn", "o_proj", "rmsnorm_mlp",
            "gate_up_proj", "silu_mul", "down_proj")
MOE_OP_NAMES = OP_NAMES[:6] + ("gate", "experts_up", "experts_down")


class fp_shape(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32),
                ("kv_block_tokens", C.c_int32), ("kv_num_blocks", C.c_int64),
                ("max_position", C.c_int32), ("n_experts", C.c_int32), ("top_k", C.c_int32)]


class fp_layer_weights(C.Structure):
    _fields_ = [("attn_norm", C.c_void_p), ("w_qkv", C.c_void_p), ("w_o", C.c_void_p),
                ("mlp_norm", C.c_void_p), ("w_gate_up", C.c_void_p), ("w_down", C.c_void_p),
                ("w_router", C.c_void_p)]


_P = C.c_void_p
_I32P = C.POINTER(C.c_int32)
_SIGS = {
    "fp_model_create": (C.c_int, [C.POINTER(fp_shape), C.POINTER(fp_layer_weights), _P, C.POINTER(_P)]),
    "fp_model_destroy": (None, [_P]),
    "fp_kv_alloc": (C.c_int, [_P, C.c_int32, _I32P]),
    "fp_kv_free": (C.c_int, [_P, C.c_int32, _I32P]),
    "fp_model_kv_pools": (C.c_int, [_P, C.POINTER(_P), C.POINTER(_P)]),
    "fp_prefill_begin": (C.c_int, [_P, _P, _I32P, C.c_int32, _I32P, _I32P, C.c_int32, C.c_uint32, C.POINTER(_P)]),
    "fp_prefill_advance": (C.c_int, [_P, C.c_int32, _I32P]),
    "fp_prefill_set_launch_ahead": (C.c_int, [_P, C.c_int32]),
    "fp_preempt": (C.c_int, [_P]),
    "fp_preempt_signal": (C.c_int, [_P]),
    "fp_preempt_wait": (C.c_int, [_P]),
    "fp_resume": (C.c_int, [_P]),
    "fp_prefill_cursor": (C.c_int, [_P, _I32P, _I32P]),
    "fp_prefill_hidden": (C.c_int, [_P, C.POINTER(_P)]),
    "fp_prefill_kv": (C.c_int, [_P, C.c_int32, C.POINTER(_P), C.POINTER(_P), C.POINTER(_I32P)]),
    "fp_prefill_block_tables": (C.c_int, [_P, C.POINTER(_I32P), _I32P]),
    "fp_prefill_kv_gather": (C.c_int, [_P, C.c_int32, C.c_int32, _P, _P]),
    "fp_prefill_set_timing": (C.c_int, [_P, C.c_int32]),
    "fp_prefill_op_times": (C.c_int, [_P, C.POINTER(C.c_float), C.c_int32, _I32P]),
    "fp_prefill_moe_routing": (C.c_int, [_P, C.c_int32, _P, _P]),
    "fp_prefill_end": (None, [_P]),
    "fp_op_gemm": (C.c_int, [C.c_int32, _P, _P, _P, C.c_int64, C.c_int64, C.c_int64, C.c_int32, _P]),
    "fp_op_gemm_ws": (C.c_int, [C.c_int32, _P, _P, _P, C.c_int64, C.c_int64, C.c_int64, C.c_int32, _P, C.c_int64, _P]),
    "fp_op_gemm_tail": (C.c_int, [C.c_int32, _P, _P, _P, C.c_int64, C.c_int64, C.c_int64, C.c_int32, _P, C.c_int64,
                                  C.c_int32, _P, _P, C.c_float, _P]),
    "fp_op_gemm_noalloc": (C.c_int, [C.c_int32, _P, _P, _P, C.c_int64, C.c_int64, C.c_int64, C.c_int32, _P]),
    "fp_op_gemm_workspace_bytes": (C.c_int64, [C.c_int32, C.c_int64, C.c_int64, C.c_int64]),
    "fp_op_rmsnorm": (C.c_int, [C.c_int32, _P, _P, _P, C.c_int64, C.c_int64, C.c_float, _P]),
    "fp_op_silu_mul": (C.c_int, [C.c_int32, _P, _P, C.c_int64, C.c_int64, _P]),
    "fp_op_gemm_swiglu": (C.c_int, [_P, _P, _P, C.c_int64, C.c_int64, C.c_int64, _P]),
    "fp_sched_create": (C.c_int, [C.c_int64, C.POINTER(C.c_double), C.c_int32, C.c_int32, C.c_int32, C.POINTER(_P)]),
    "fp_sched_destroy": (None, [_P]),
    "fp_sched_arrive": (C.c_int, [_P, C.c_int64, C.c_int64, C.c_double, C.c_double]),
    "fp_sched_complete": (C.c_int, [_P, C.c_int64]),
    "fp_sched_retire": (C.c_int, [_P, C.c_int64]),
    "fp_sched_round": (C.c_int, [_P, C.c_double, _P]),
    "fp_sched_predict": (C.c_double, [_P, C.c_int64]),
    "fp_diag_mfma_ceiling": (C.c_int, [C.c_int32, _P, C.POINTER(C.c_double)]),
    "fp_last_error": (C.c_char_p, []),
    "fp_version": (C.c_char_p, []),
}
EXPORTED = tuple(_SIGS)
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


class FlowPrefillError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.fp_last_error()
        super().__init__(f"{where}: status {status}: {msg.decode() if msg else ''}")


def _check(status: int, where: str) -> int:
    if status < 0:
        raise FlowPrefillError(status, where)
    return status


def _i32(values: Optional[Sequence[int]]):
    if values is None:
        return None, None
    arr = np.ascontiguousarray(np.asarray(values, dtype=np.int32))
    return arr, arr.ctypes.data_as(_I32P)


# ---------------------------------------------------------------------------------------------
# Same-named thin wrappers
# ---------------------------------------------------------------------------------------------

def fp_version() -> str:
    return lib.fp_version().decode()


def fp_last_error() -> str:
    return lib.fp_last_error().decode()


def fp_model_create(shape: fp_shape, layers: Sequence[Dict[str, int]], hip_stream: int = 0) -> int:
    """layers: per layer a dict name -> device address (int)."""
    arr = (fp_layer_weights * len(layers))()
    for i, w in enumerate(layers):
        for name, _ in fp_layer_weights._fields_:
            setattr(arr[i], name, int(w.get(name, 0)))          # w_router: mixture-of-experts models only
    out = _P()
    _check(lib.fp_model_create(C.byref(shape), arr, _P(hip_stream), C.byref(out)), "fp_model_create")
    return out.value


def fp_model_destroy(model: int) -> None:
    lib.fp_model_destroy(_P(model))


def fp_kv_alloc(model: int, n: int) -> np.ndarray:
    ids = np.empty(max(n, 1), dtype=np.int32)
    _check(lib.fp_kv_alloc(_P(model), n, ids.ctypes.data_as(_I32P)), "fp_kv_alloc")
    return ids[:n]


def fp_kv_free(model: int, ids: Sequence[int]) -> None:
    arr, ptr = _i32(ids)
    _check(lib.fp_kv_free(_P(model), len(arr), ptr), "fp_kv_free")


def fp_model_kv_pools(model: int):
    k, v = _P(), _P()
    _check(lib.fp_model_kv_pools(_P(model), C.byref(k), C.byref(v)), "fp_model_kv_pools")
    return k.value, v.value


def fp_prefill_begin(model: int, hidden_in: int, cu_seqlens: Sequence[int],
                     cached_lens: Optional[Sequence[int]] = None,
                     block_tables: Optional[np.ndarray] = None,
                     boundary_mask: int = FP_BOUNDARY_EVERY_OP) -> int:
    cu, cu_p = _i32(cu_seqlens)
    n_seqs = len(cu) - 1
    _c, c_p = _i32(cached_lens)
    max_blocks = 0
    bt_p = None
    if block_tables is not None:
        bt = np.ascontiguousarray(np.asarray(block_tables, dtype=np.int32)).reshape(n_seqs, -1)
        max_blocks = bt.shape[1]
        bt_p = bt.ctypes.data_as(_I32P)
    out = _P()
    _check(lib.fp_prefill_begin(_P(model), _P(hidden_in), cu_p, n_seqs, c_p, bt_p, max_blocks,
                                C.c_uint32(boundary_mask), C.byref(out)), "fp_prefill_begin")
    return out.value


def fp_prefill_advance(task: int, max_ops: int = 2 ** 31 - 1):
    """Returns (status, ops_done)."""
    done = C.c_int32(0)
    st = _check(lib.fp_prefill_advance(_P(task), max_ops, C.byref(done)), "fp_prefill_advance")
    return st, done.value


def fp_prefill_set_launch_ahead(task: int, k: int) -> None:
    _check(lib.fp_prefill_set_launch_ahead(_P(task), k), "fp_prefill_set_launch_ahead")


def fp_preempt(task: int) -> int:
    return _check(lib.fp_preempt(_P(task)), "fp_preempt")


def fp_preempt_signal(task: int) -> int:
    return _check(lib.fp_preempt_signal(_P(task)), "fp_preempt_signal")


def fp_preempt_wait(task: int) -> int:
    return _check(lib.fp_preempt_wait(_P(task)), "fp_preempt_wait")


def fp_resume(task: int) -> None:
    _check(lib.fp_resume(_P(task)), "fp_resume")


def fp_prefill_cursor(task: int):
    layer, op = C.c_int32(), C.c_int32()
    _check(lib.fp_prefill_cursor(_P(task), C.byref(layer), C.byref(op)), "fp_prefill_cursor")
    return layer.value, op.value


def fp_prefill_hidden(task: int) -> int:
    p = _P()
    _check(lib.fp_prefill_hidden(_P(task), C.byref(p)), "fp_prefill_hidden")
    return p.value


def fp_prefill_block_tables(task: int, n_seqs: int) -> np.ndarray:
    ptr, mb = _I32P(), C.c_int32()
    _check(lib.fp_prefill_block_tables(_P(task), C.byref(ptr), C.byref(mb)), "fp_prefill_block_tables")
    if n_seqs == 0:
        return np.zeros((0, mb.value), dtype=np.int32)
    return np.ctypeslib.as_array(ptr, shape=(n_seqs, mb.value)).copy()


def fp_prefill_kv(task: int, layer: int, n_seqs: int):
    """-> (k_pool address of that layer, v_pool address of that layer, block tables [n_seqs, max_blocks])."""
    k, v, ptr = _P(), _P(), _I32P()
    _check(lib.fp_prefill_kv(_P(task), layer, C.byref(k), C.byref(v), C.byref(ptr)), "fp_prefill_kv")
    return k.value, v.value, fp_prefill_block_tables(task, n_seqs)


def fp_prefill_kv_gather(task: int, layer: int, seq: int, k_out: int, v_out: int) -> None:
    _check(lib.fp_prefill_kv_gather(_P(task), layer, seq, _P(k_out), _P(v_out)), "fp_prefill_kv_gather")


def fp_prefill_set_timing(task: int, on: bool) -> None:
    _check(lib.fp_prefill_set_timing(_P(task), 1 if on else 0), "fp_prefill_set_timing")


def fp_prefill_op_times(task: int, n: int) -> List[float]:
    buf = (C.c_float * max(n, 1))()
    cnt = C.c_int32()
    _check(lib.fp_prefill_op_times(_P(task), buf, n, C.byref(cnt)), "fp_prefill_op_times")
    return [buf[i] for i in range(cnt.value)]


def fp_prefill_end(task: int) -> None:
    lib.fp_prefill_end(_P(task))


def fp_op_gemm(dtype: int, a: int, w: int, c: int, m: int, n: int, k: int, residual: bool,
               hip_stream: int = 0) -> None:
    _check(lib.fp_op_gemm(dtype, _P(a), _P(w), _P(c), m, n, k, 1 if residual else 0, _P(hip_stream)),
           "fp_op_gemm")


def fp_op_gemm_ws(dtype: int, a: int, w: int, c: int, m: int, n: int, k: int, residual: bool,
                  workspace: int, workspace_bytes: int, hip_stream: int = 0) -> None:
    _check(lib.fp_op_gemm_ws(dtype, _P(a), _P(w), _P(c), m, n, k, 1 if residual else 0, _P(workspace),
                             workspace_bytes, _P(hip_stream)), "fp_op_gemm_ws")


FP_TAIL_RMSNORM, FP_TAIL_SWIGLU = 1, 2


def fp_op_gemm_tail(a: int, w: int, c: int, m: int, n: int, k: int, residual: bool, workspace: int,
                    workspace_bytes: int, tail: int, gain: int, tail_out: int, eps: float = 0.0,
                    hip_stream: int = 0) -> None:
    _check(lib.fp_op_gemm_tail(FP_DTYPE_BF16, _P(a), _P(w), _P(c), m, n, k, 1 if residual else 0, _P(workspace),
                               workspace_bytes, tail, _P(gain), _P(tail_out), C.c_float(eps), _P(hip_stream)),
           "fp_op_gemm_tail")


FP_NOALLOC_SCRATCH_BYTES = 32 * 1024 * 1024


def fp_op_gemm_noalloc(dtype: int, a: int, w: int, c: int, m: int, n: int, k: int, residual: bool,
                       hip_stream: int = 0) -> None:
    _check(lib.fp_op_gemm_noalloc(dtype, _P(a), _P(w), _P(c), m, n, k, 1 if residual else 0, _P(hip_stream)),
           "fp_op_gemm_noalloc")


def fp_op_gemm_workspace_bytes(dtype: int, m: int, n: int, k: int) -> int:
    return int(lib.fp_op_gemm_workspace_bytes(dtype, m, n, k))


def fp_op_rmsnorm(dtype: int, x_f32: int, gain: int, out: int, t: int, d: int, eps: float,
                  hip_stream: int = 0) -> None:
    _check(lib.fp_op_rmsnorm(dtype, _P(x_f32), _P(gain), _P(out), t, d, C.c_float(eps), _P(hip_stream)),
           "fp_op_rmsnorm")


def fp_prefill_moe_routing(task: int, layer: int, ids_out: int, weights_out: int) -> None:
    _check(lib.fp_prefill_moe_routing(_P(task), layer, _P(ids_out), _P(weights_out)), "fp_prefill_moe_routing")


def fp_diag_mfma_ceiling(milliseconds: int = 200, hip_stream: int = 0) -> float:
    out = C.c_double()
    _check(lib.fp_diag_mfma_ceiling(milliseconds, _P(hip_stream), C.byref(out)), "fp_diag_mfma_ceiling")
    return out.value


def fp_op_silu_mul(dtype: int, gu: int, out: int, t: int, f: int, hip_stream: int = 0) -> None:
    _check(lib.fp_op_silu_mul(dtype, _P(gu), _P(out), t, f, _P(hip_stream)), "fp_op_silu_mul")


def fp_op_gemm_swiglu(a: int, w_gate_up: int, out: int, m: int, f: int, k: int, hip_stream: int = 0) -> None:
    _check(lib.fp_op_gemm_swiglu(_P(a), _P(w_gate_up), _P(out), m, f, k, _P(hip_stream)), "fp_op_gemm_swiglu")


def make_shape(spec, dtype: int, kv_num_blocks: int, max_position: int) -> fp_shape:
    """fp_shape from an inputs.ShapeSpec-like object (plain attribute copy)."""
    return fp_shape(spec.n_layers, spec.hidden, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                    spec.ffn, spec.rms_eps, spec.rope_theta, dtype, 16, kv_num_blocks, max_position,
                    getattr(spec, "n_experts", 0), getattr(spec, "top_k", 0))


# ---- event-driven scheduler (host-only) ----
FP_SCHED_SEDF, FP_SCHED_EDF, FP_SCHED_FCFS = 0, 1, 2
FP_SCHED_NONE, FP_SCHED_SUBMIT, FP_SCHED_RESUME = 0, 1, 2
FP_SCHED_MAX_BATCH = 64


class SchedDecision(C.Structure):
    _fields_ = [("preempt_id", C.c_int64), ("action", C.c_int32), ("n_batch", C.c_int32),
                ("head_id", C.c_int64), ("batch_ids", C.c_int64 * FP_SCHED_MAX_BATCH)]


def fp_sched_create(token_budget: int, ttft_coef, policy: int = FP_SCHED_SEDF, batching: bool = True) -> int:
    coef = (C.c_double * len(ttft_coef))(*[float(c) for c in ttft_coef])
    out = _P()
    _check(lib.fp_sched_create(int(token_budget), coef, len(ttft_coef), policy, int(batching), C.byref(out)),
           "fp_sched_create")
    return out.value


def fp_sched_destroy(sched: int) -> None:
    lib.fp_sched_destroy(_P(sched))


def fp_sched_arrive(sched: int, id: int, n_tokens: int, arrival: float, ttft_slo: float) -> None:
    _check(lib.fp_sched_arrive(_P(sched), id, n_tokens, arrival, ttft_slo), "fp_sched_arrive")


def fp_sched_complete(sched: int, head_id: int) -> None:
    _check(lib.fp_sched_complete(_P(sched), head_id), "fp_sched_complete")


def fp_sched_retire(sched: int, id: int) -> None:
    _check(lib.fp_sched_retire(_P(sched), id), "fp_sched_retire")


def fp_sched_round(sched: int, now: float):
    """-> (preempt_id or None, action, head_id or None, [batch ids])"""
    d = SchedDecision()
    _check(lib.fp_sched_round(_P(sched), now, C.byref(d)), "fp_sched_round")
    return (None if d.preempt_id < 0 else d.preempt_id, d.action, None if d.head_id < 0 else d.head_id,
            [d.batch_ids[i] for i in range(d.n_batch)])


def fp_sched_predict(sched: int, n_tokens: int) -> float:
    return lib.fp_sched_predict(_P(sched), n_tokens)

