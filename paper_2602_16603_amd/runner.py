"""Torch-side plumbing around the C-ABI binding: device buffers for weights and hidden states,
the stream handle, and copies of results back into torch tensors.  No arithmetic of the method
lives here; every operator runs inside libflowprefill.so.
"""
from __future__ import annotations

import ctypes as C
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import binding as B

_hip = None


def _hip_runtime():
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
        _hip.hipMemcpy.restype = C.c_int
        _hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
    return _hip


def copy_from_device_ptr(ptr: int, shape: Sequence[int], dtype: torch.dtype) -> torch.Tensor:
    """A fresh torch tensor holding a copy of `prod(shape)` elements at device address `ptr`."""
    out = torch.empty(tuple(shape), dtype=dtype, device="cuda")
    if out.numel():
        rc = _hip_runtime().hipMemcpy(out.data_ptr(), ptr, out.numel() * out.element_size(), 3)
        if rc != 0:
            raise RuntimeError(f"hipMemcpy failed with {rc}")
    return out


TORCH_DTYPE = {B.FP_DTYPE_F32: torch.float32, B.FP_DTYPE_BF16: torch.bfloat16}


class PrefillModel:
    """Owns the device weights (kept alive for the model's life) and the fp_model handle."""

    def __init__(self, spec, weights: List[Dict[str, torch.Tensor]], dtype: int,
                 kv_num_blocks: int, max_position: int, stream: Optional[torch.cuda.Stream] = None):
        self.spec = spec
        self.dtype = dtype
        self.torch_dtype = TORCH_DTYPE[dtype]
        self.stream = stream
        self.weights = []
        for w in weights:
            dev = {k: v.to(device="cuda", dtype=self.torch_dtype).contiguous() for k, v in w.items()}
            self.weights.append(dev)
        torch.cuda.synchronize()
        shape = B.make_shape(spec, dtype, kv_num_blocks, max_position)
        ptrs = [{k: v.data_ptr() for k, v in w.items()} for w in self.weights]
        self.handle = B.fp_model_create(shape, ptrs, stream.cuda_stream if stream is not None else 0)

    def begin(self, hidden: torch.Tensor, lengths: Sequence[int],
              cached: Optional[Sequence[int]] = None, block_tables: Optional[np.ndarray] = None,
              boundary_mask: int = B.FP_BOUNDARY_EVERY_OP) -> "PrefillTask":
        return PrefillTask(self, hidden, lengths, cached, block_tables, boundary_mask)

    def close(self) -> None:
        if self.handle:
            B.fp_model_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class PrefillTask:
    """One execution task (submit / advance / preempt / resume), a thin veneer over fp_prefill_*."""

    def __init__(self, model: PrefillModel, hidden: torch.Tensor, lengths: Sequence[int],
                 cached, block_tables, boundary_mask: int):
        self.model = model
        self.lengths = [int(n) for n in lengths]
        self.cached = [0] * len(self.lengths) if cached is None else [int(c) for c in cached]
        self.cu = [0]
        for n in self.lengths:
            self.cu.append(self.cu[-1] + n)
        assert hidden.is_cuda and hidden.dtype == model.torch_dtype and hidden.is_contiguous()
        assert tuple(hidden.shape) == (self.cu[-1], model.spec.hidden)
        torch.cuda.current_stream().synchronize()   # hidden was produced on torch's stream
        self._hidden_in = hidden                    # read asynchronously by the library: keep it alive
        self.handle = B.fp_prefill_begin(model.handle, hidden.data_ptr(), self.cu,
                                         None if cached is None else self.cached, block_tables,
                                         boundary_mask)

    def advance(self, max_ops: int = 2 ** 31 - 1) -> Tuple[int, int]:
        return B.fp_prefill_advance(self.handle, max_ops)

    def run_to_completion(self) -> None:
        st, _ = self.advance()
        if st != B.FP_DONE:
            raise RuntimeError(f"prefill stopped with status {st}")

    def preempt(self) -> int:
        return B.fp_preempt(self.handle)

    def resume(self) -> None:
        B.fp_resume(self.handle)

    def cursor(self) -> Tuple[int, int]:
        return B.fp_prefill_cursor(self.handle)

    def hidden(self) -> torch.Tensor:
        """Copy of the fp32 residual stream [T, d]."""
        return copy_from_device_ptr(B.fp_prefill_hidden(self.handle),
                                    (self.cu[-1], self.model.spec.hidden), torch.float32)

    def kv(self, layer: int, seq: int) -> Tuple[torch.Tensor, torch.Tensor]:
        """(K rotated, V) of one sequence, [len, Hkv, D] in the storage dtype."""
        n = self.cached[seq] + self.lengths[seq]
        sp = self.model.spec
        k = torch.empty((n, sp.n_kv_heads, sp.head_dim), dtype=self.model.torch_dtype, device="cuda")
        v = torch.empty_like(k)
        torch.cuda.synchronize()
        if n:
            B.fp_prefill_kv_gather(self.handle, layer, seq, k.data_ptr(), v.data_ptr())
        return k, v

    def moe_routing(self, layer: int) -> Tuple[torch.Tensor, torch.Tensor]:
        """(expert ids [T, top_k] int32, weights [T, top_k] fp32) chosen by layer `layer`'s router."""
        k = self.model.spec.top_k
        ids = torch.empty((self.cu[-1], k), dtype=torch.int32, device="cuda")
        wts = torch.empty((self.cu[-1], k), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        B.fp_prefill_moe_routing(self.handle, layer, ids.data_ptr(), wts.data_ptr())
        return ids, wts

    def kv_pools(self, layer: int) -> Tuple[int, int, np.ndarray]:
        """(device address of the layer's K pool slice, of its V pool slice, block tables)."""
        return B.fp_prefill_kv(self.handle, layer, len(self.lengths))

    def block_tables(self) -> np.ndarray:
        return B.fp_prefill_block_tables(self.handle, len(self.lengths))

    def end(self) -> None:
        if self.handle:
            B.fp_prefill_end(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.end()
        except Exception:
            pass
