"""fp_op_gemm_noalloc -- the entry point for callers that cannot allocate -- through the C ABI
against fp_op_gemm_ws (caller workspace, same kernels): bit-identical outputs on two calls in a
row, the second with a smaller problem that leaves most of the static scratch holding the first
call's partial sums; sizes beyond the static scratch are refused with nothing launched."""
import pytest
import torch

from oracle import prefill_oracle as O
from paper_2602_16603_amd import inputs as I
from tests.util import TOL, max_rel_err

pytestmark = pytest.mark.gpu


def _binding():
    from paper_2602_16603_amd import binding
    return binding


def _run_pair(B, m, n, k, residual, seed):
    a = I.normal_tensor((m, k), 1.0, seed, torch.bfloat16, "cuda")
    w = I.normal_tensor((n, k), 0.05, seed + 1, torch.bfloat16, "cuda")
    td = torch.float32 if residual else torch.bfloat16
    g = 2
    bufs = []
    for _ in range(2):
        buf = torch.full((m + 2 * g, n), 7.0, dtype=td, device="cuda")
        if residual:
            buf[g:g + m] = I.normal_tensor((m, n), 1.0, seed + 2, torch.float32, "cuda")
        bufs.append(buf)
    x0 = bufs[0][g:g + m].clone()
    ws_bytes = B.fp_op_gemm_workspace_bytes(1, m, n, k)
    ws = torch.empty((max(ws_bytes, 256),), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    print(f"  noalloc gemm m={m} n={n} k={k} residual={residual} scratch wanted={ws_bytes}", flush=True)
    B.fp_op_gemm_noalloc(1, a.data_ptr(), w.data_ptr(), bufs[0][g:g + m].data_ptr(), m, n, k, residual)
    B.fp_op_gemm_ws(1, a.data_ptr(), w.data_ptr(), bufs[1][g:g + m].data_ptr(), m, n, k, residual,
                    ws.data_ptr(), ws_bytes)
    torch.cuda.synchronize()
    assert torch.equal(bufs[0], bufs[1])                       # same bits, guard rows (7.0) included
    ref = O.linear(a.cpu(), w.cpu())
    if residual:
        ref = ref + x0.cpu().double()
    assert max_rel_err(bufs[0][g:g + m], ref) <= TOL["bf16"]
    return ws_bytes


@pytest.mark.parametrize("residual", [False, True])
def test_two_calls_in_a_row_second_one_smaller(residual):
    B = _binding()
    big = _run_pair(B, 256, 4096, 4096, residual, seed=61)     # 32 MiB of partial sums: all of the scratch
    small = _run_pair(B, 130, 2056, 2048, residual, seed=64)   # a few MiB: the rest keeps the first call's sums
    assert 0 < small < big <= B.FP_NOALLOC_SCRATCH_BYTES
    unsplit = _run_pair(B, 2304, 2816, 192, residual, seed=67) # a problem that needs no scratch at all
    assert unsplit == 0


def test_sizes_beyond_the_static_scratch_are_refused():
    B = _binding()
    m, n, k = 1000, 4096, 4096                                  # wants 62.5 MiB of partial sums
    assert B.fp_op_gemm_workspace_bytes(1, m, n, k) > B.FP_NOALLOC_SCRATCH_BYTES
    a = torch.zeros((m, k), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((n, k), dtype=torch.bfloat16, device="cuda")
    c = torch.full((m, n), 3.0, dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    with pytest.raises(B.FlowPrefillError) as e:
        B.fp_op_gemm_noalloc(1, a.data_ptr(), w.data_ptr(), c.data_ptr(), m, n, k, False)
    assert e.value.status == B.FP_ERR_INVALID and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert torch.all(c == 3.0)                                  # nothing was launched
    with pytest.raises(B.FlowPrefillError):
        B.fp_op_gemm_noalloc(1, a.data_ptr(), w.data_ptr(), c.data_ptr(), m, n, 12, False)   # K % 8
