"""Single-operator parity: each HIP kernel, called through the C ABI, against the oracle's plain
definition on the same seeded inputs (sizes span several tiles and ragged tails)."""
import pytest
import torch

from oracle import prefill_oracle as O
from paper_2602_16603_amd import inputs as I
from tests.util import TOL, max_rel_err

pytestmark = pytest.mark.gpu

DT = {"fp32": (0, torch.float32), "bf16": (1, torch.bfloat16)}


def _binding():
    from paper_2602_16603_amd import binding
    return binding


@pytest.mark.parametrize("name", ["bf16", "fp32"])
@pytest.mark.parametrize("m,n,k", [
    (1, 8, 8), (37, 520, 264), (256, 512, 256), (300, 1408, 256), (256, 256, 704),
    (1000, 256, 704), (513, 776, 1000), (4113, 4096, 512),
])
def test_gemm_matches_definition(name, m, n, k):
    B = _binding()
    code, td = DT[name]
    print(f"gemm {name} m={m} n={n} k={k}", flush=True)
    a = I.normal_tensor((m, k), 1.0, 11, td, "cuda")
    w = I.normal_tensor((n, k), 0.05, 12, td, "cuda")
    c = torch.full((m, n), float("nan"), dtype=td, device="cuda")
    torch.cuda.synchronize()
    B.fp_op_gemm(code, a.data_ptr(), w.data_ptr(), c.data_ptr(), m, n, k, False)
    torch.cuda.synchronize()
    ref = O.linear(a.cpu(), w.cpu())
    assert max_rel_err(c, ref) <= TOL[name]


@pytest.mark.parametrize("name", ["bf16", "fp32"])
@pytest.mark.parametrize("m,n,k", [(300, 264, 520), (4113, 4096, 256)])
def test_gemm_residual_accumulates_into_fp32(name, m, n, k):
    B = _binding()
    code, td = DT[name]
    print(f"gemm-residual {name} m={m} n={n} k={k}", flush=True)
    a = I.normal_tensor((m, k), 1.0, 13, td, "cuda")
    w = I.normal_tensor((n, k), 0.05, 14, td, "cuda")
    x = I.normal_tensor((m, n), 1.0, 15, torch.float32, "cuda")
    x0 = x.clone()
    torch.cuda.synchronize()
    B.fp_op_gemm(code, a.data_ptr(), w.data_ptr(), x.data_ptr(), m, n, k, True)
    torch.cuda.synchronize()
    ref = x0.cpu().double() + O.linear(a.cpu(), w.cpu())
    assert max_rel_err(x, ref) <= TOL[name]


@pytest.mark.parametrize("residual", [False, True])
@pytest.mark.parametrize("m,n,k", [
    (2304, 2816, 64), (2304, 2816, 128), (2304, 2816, 192), (2560, 2560, 448), (2560, 2560, 576),
    (2560, 2560, 1088), (2561, 2568, 704), (2049, 3080, 1600),
])
def test_gemm_fast_path_trip_counts_and_ragged_edges(residual, m, n, k):
    """The 256x256-tile MFMA kernel on every path of its K loop (1, 2, 3, 7, 9, 11, 17 and 25
    k-tiles: single tiles, pairs, the eight-tile trip and their mixes), with a last row tile of
    one row and a last column tile of eight columns; rows behind the output must stay untouched."""
    B = _binding()
    print(f"gemm fast path residual={residual} m={m} n={n} k={k}", flush=True)
    a = I.normal_tensor((m, k), 1.0, 21, torch.bfloat16, "cuda")
    w = I.normal_tensor((n, k), 0.05, 22, torch.bfloat16, "cuda")
    td = torch.float32 if residual else torch.bfloat16
    guard = 300
    buf = torch.full((m + guard, n), 7.0, dtype=td, device="cuda")
    if residual:
        buf[:m] = I.normal_tensor((m, n), 1.0, 23, torch.float32, "cuda")
    x0 = buf[:m].clone()
    torch.cuda.synchronize()
    B.fp_op_gemm(1, a.data_ptr(), w.data_ptr(), buf.data_ptr(), m, n, k, residual)
    torch.cuda.synchronize()
    ref = O.linear(a.cpu(), w.cpu())
    if residual:
        ref = ref + x0.cpu().double()
    assert max_rel_err(buf[:m], ref) <= TOL["bf16"]
    assert torch.all(buf[m:] == 7.0)


@pytest.mark.parametrize("residual", [False, True])
@pytest.mark.parametrize("m,n,k", [
    (512, 6144, 64), (300, 6152, 128), (257, 6152, 192), (512, 6152, 448), (257, 6152, 576), (130, 12296, 704),
    (257, 6152, 1088), (1, 12296, 1600),
])
def test_gemm_narrow_tile_trip_counts_and_ragged_edges(residual, m, n, k):
    """The 128-column tile that requests of up to two row tiles run on, uncut (no workspace), on
    every path of its K loop (1, 2, 3, 7, 9, 11, 17 and 25 k-tiles), with a last row tile of one
    row and a last column tile of eight columns; rows behind the output must stay untouched."""
    B = _binding()
    assert B.fp_op_gemm_workspace_bytes(1, m, n, k) == 0 or k >= 1024   # (short K: not cut even with a workspace)
    print(f"gemm narrow tile residual={residual} m={m} n={n} k={k}", flush=True)
    a = I.normal_tensor((m, k), 1.0, 24, torch.bfloat16, "cuda")
    w = I.normal_tensor((n, k), 0.05, 25, torch.bfloat16, "cuda")
    td = torch.float32 if residual else torch.bfloat16
    guard = 300
    buf = torch.full((m + guard, n), 7.0, dtype=td, device="cuda")
    if residual:
        buf[:m] = I.normal_tensor((m, n), 1.0, 26, torch.float32, "cuda")
    x0 = buf[:m].clone()
    torch.cuda.synchronize()
    B.fp_op_gemm(1, a.data_ptr(), w.data_ptr(), buf.data_ptr(), m, n, k, residual)
    torch.cuda.synchronize()
    ref = O.linear(a.cpu(), w.cpu())
    if residual:
        ref = ref + x0.cpu().double()
    assert max_rel_err(buf[:m], ref) <= TOL["bf16"]
    assert torch.all(buf[m:] == 7.0)


def _random_gemm_shapes(count, seed):
    import random
    rng = random.Random(seed)
    ms = [1, 7, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 511, 513, 777, 1024, 1500, 2049, 2560, 3001]
    ns = [8, 16, 64, 120, 128, 136, 248, 256, 264, 512, 520, 1000, 1024, 2048, 2056, 3072, 4104]
    ks = [8, 16, 24, 64, 72, 128, 192, 256, 320, 512, 1024, 1088, 2048, 4096]
    out = []
    while len(out) < count:
        m, n, k = rng.choice(ms), rng.choice(ns), rng.choice(ks)
        if m * n * k <= 6e9:
            out.append((m, n, k, rng.random() < 0.5))
    return out


@pytest.mark.parametrize("m,n,k,residual", _random_gemm_shapes(32, 20260216))
def test_gemm_seeded_random_shapes(m, n, k, residual):
    """Shapes drawn (seeded) across the dispatches of the bf16 GEMM that need no workspace -- the
    small-problem kernel and the 256x256-tile kernel -- with ragged rows, columns and K; rows
    before and behind the output must stay untouched.  (The split-K form is reached through
    fp_op_gemm_ws: test_gemm_split_k_with_workspace.)"""
    B = _binding()
    print(f"gemm random m={m} n={n} k={k} residual={residual}", flush=True)
    a = I.normal_tensor((m, k), 1.0, 31, torch.bfloat16, "cuda")
    w = I.normal_tensor((n, k), 0.05, 32, torch.bfloat16, "cuda")
    td = torch.float32 if residual else torch.bfloat16
    g = 3
    buf = torch.full((m + 2 * g, n), 7.0, dtype=td, device="cuda")
    if residual:
        buf[g:g + m] = I.normal_tensor((m, n), 1.0, 33, torch.float32, "cuda")
    x0 = buf[g:g + m].clone()
    out = buf[g:g + m]
    torch.cuda.synchronize()
    B.fp_op_gemm(1, a.data_ptr(), w.data_ptr(), out.data_ptr(), m, n, k, residual)
    torch.cuda.synchronize()
    ref = O.linear(a.cpu(), w.cpu())
    if residual:
        ref = ref + x0.cpu().double()
    assert max_rel_err(out, ref) <= TOL["bf16"]
    assert torch.all(buf[:g] == 7.0) and torch.all(buf[g + m:] == 7.0)


@pytest.mark.parametrize("residual", [False, True])
@pytest.mark.parametrize("m,n,k", [
    (256, 6144, 4096), (1, 4096, 4096), (130, 4096, 14336), (1000, 4096, 4096), (512, 6144, 4096),
    (513, 4104, 1024), (200, 14336, 4096), (64, 5120, 27648), (777, 2056, 2048),
])
def test_gemm_split_k_with_workspace(residual, m, n, k):
    """Short requests (the 128-1024-token prompts of the trace) leave too few output tiles to fill
    the chip; with a workspace the GEMM is cut over K and a second kernel adds the partial sums in
    a fixed order.  Ragged M and N, guard rows before and behind the output, the workspace's own
    guard region untouched, the result against the definition and against the uncut form."""
    B = _binding()
    ws_bytes = B.fp_op_gemm_workspace_bytes(1, m, n, k)
    print(f"gemm split-K m={m} n={n} k={k} residual={residual} workspace={ws_bytes}", flush=True)
    assert ws_bytes > 0, "shape chosen for the split-K path does not split"
    a = I.normal_tensor((m, k), 1.0, 35, torch.bfloat16, "cuda")
    w = I.normal_tensor((n, k), 0.05, 36, torch.bfloat16, "cuda")
    td = torch.float32 if residual else torch.bfloat16
    g = 3
    buf = torch.full((m + 2 * g, n), 7.0, dtype=td, device="cuda")
    if residual:
        buf[g:g + m] = I.normal_tensor((m, n), 1.0, 37, torch.float32, "cuda")
    x0 = buf[g:g + m].clone()
    plain = x0.clone()
    out = buf[g:g + m]
    pad = 4096
    ws = torch.full((ws_bytes + pad,), 0x5A, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    B.fp_op_gemm_ws(1, a.data_ptr(), w.data_ptr(), out.data_ptr(), m, n, k, residual, ws.data_ptr(), ws_bytes)
    B.fp_op_gemm(1, a.data_ptr(), w.data_ptr(), plain.data_ptr(), m, n, k, residual)
    torch.cuda.synchronize()
    ref = O.linear(a.cpu(), w.cpu())
    if residual:
        ref = ref + x0.cpu().double()
    assert max_rel_err(out, ref) <= TOL["bf16"]
    assert max_rel_err(out, plain.cpu().double()) <= 1e-2          # same sums, another fp32 order
    assert torch.all(buf[:g] == 7.0) and torch.all(buf[g + m:] == 7.0)
    assert torch.all(ws[ws_bytes:] == 0x5A)
    again = x0.clone()                                              # fixed-order reduction: repeats bit for bit
    B.fp_op_gemm_ws(1, a.data_ptr(), w.data_ptr(), again.data_ptr(), m, n, k, residual, ws.data_ptr(), ws_bytes)
    torch.cuda.synchronize()
    assert torch.equal(again, out)


@pytest.mark.parametrize("m,n,k", [(256, 4096, 4096), (1000, 4096, 14336), (130, 5120, 27648), (1, 4096, 4096), (513, 2056, 2048)])
def test_split_k_reduction_fused_with_rmsnorm_equals_the_two_operators(m, n, k):
    """Residual projection cut over K whose reduction kernel also normalises the updated row: the
    residual and the normalised rows carry the bits of fp_op_gemm_ws followed by fp_op_rmsnorm,
    and agree with the definition."""
    B = _binding()
    ws_bytes = B.fp_op_gemm_workspace_bytes(1, m, n, k)
    assert ws_bytes > 0
    a = I.normal_tensor((m, k), 1.0, 45, torch.bfloat16, "cuda")
    w = I.normal_tensor((n, k), 0.02, 46, torch.bfloat16, "cuda")
    gain = (1.0 + I.normal_tensor((n,), 0.1, 47, torch.float32, "cuda")).to(torch.bfloat16)
    x0 = I.normal_tensor((m, n), 1.0, 48, torch.float32, "cuda")
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda")
    x_two, x_fused = x0.clone(), x0.clone()
    h_two = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    h_fused = torch.full((m + 2, n), 7.0, dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    B.fp_op_gemm_ws(1, a.data_ptr(), w.data_ptr(), x_two.data_ptr(), m, n, k, True, ws.data_ptr(), ws_bytes)
    B.fp_op_rmsnorm(1, x_two.data_ptr(), gain.data_ptr(), h_two.data_ptr(), m, n, 1e-5)
    B.fp_op_gemm_tail(a.data_ptr(), w.data_ptr(), x_fused.data_ptr(), m, n, k, True, ws.data_ptr(), ws_bytes,
                      B.FP_TAIL_RMSNORM, gain.data_ptr(), h_fused[1:].data_ptr(), 1e-5)
    torch.cuda.synchronize()
    assert torch.equal(x_fused, x_two) and torch.equal(h_fused[1:m + 1], h_two)
    assert torch.all(h_fused[0] == 7.0) and torch.all(h_fused[m + 1] == 7.0)
    x_ref = x0.cpu().double() + O.linear(a.cpu(), w.cpu())
    assert max_rel_err(x_fused, x_ref) <= TOL["bf16"]
    assert max_rel_err(h_fused[1:m + 1], O.rmsnorm(x_ref, gain.cpu(), 1e-5)) <= TOL["bf16"]


@pytest.mark.parametrize("m,f,k", [(256, 7168, 4096), (100, 2048, 4096), (64, 6912, 5120)])
def test_split_k_reduction_fused_with_swiglu_equals_the_two_operators(m, f, k):
    """gate_up projection cut over K whose reduction kernel applies SiLU(gate)*up: the bits of
    fp_op_gemm_ws into [M, 2F] followed by fp_op_silu_mul, without that intermediate."""
    B = _binding()
    ws_bytes = B.fp_op_gemm_workspace_bytes(1, m, 2 * f, k)
    assert ws_bytes > 0
    a = I.normal_tensor((m, k), 1.0, 49, torch.bfloat16, "cuda")
    w = I.normal_tensor((2 * f, k), 0.02, 50, torch.bfloat16, "cuda")
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda")
    gu = torch.empty((m, 2 * f), dtype=torch.bfloat16, device="cuda")
    two = torch.empty((m, f), dtype=torch.bfloat16, device="cuda")
    fused = torch.full((m + 1, f), 7.0, dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    B.fp_op_gemm_ws(1, a.data_ptr(), w.data_ptr(), gu.data_ptr(), m, 2 * f, k, False, ws.data_ptr(), ws_bytes)
    B.fp_op_silu_mul(1, gu.data_ptr(), two.data_ptr(), m, f)
    B.fp_op_gemm_tail(a.data_ptr(), w.data_ptr(), 0, m, 2 * f, k, False, ws.data_ptr(), ws_bytes,
                      B.FP_TAIL_SWIGLU, 0, fused.data_ptr())
    torch.cuda.synchronize()
    assert torch.equal(fused[:m], two) and torch.all(fused[m] == 7.0)
    ref = O.silu_mul(O.linear(a.cpu(), w.cpu()))
    assert max_rel_err(fused[:m], ref) <= TOL["bf16"]


def test_fused_tail_is_refused_when_the_problem_is_not_cut():
    B = _binding()
    m, n, k = 4096, 4096, 4096                        # fills the chip with output tiles: no split-K, no tail
    a = torch.zeros((m, k), dtype=torch.bfloat16, device="cuda")
    x = torch.zeros((m, n), dtype=torch.float32, device="cuda")
    ws = torch.empty((1 << 20,), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.FlowPrefillError) as e:
        B.fp_op_gemm_tail(a.data_ptr(), a.data_ptr(), x.data_ptr(), m, n, k, True, ws.data_ptr(), 1 << 20,
                          B.FP_TAIL_RMSNORM, a.data_ptr(), a.data_ptr(), 1e-5)
    assert e.value.status == B.FP_ERR_INVALID


@pytest.mark.parametrize("name", ["bf16", "fp32"])
@pytest.mark.parametrize("t,d", [(1, 256), (77, 4096), (5, 5120), (3, 8200), (2, 20000)])
def test_rmsnorm_matches_definition(name, t, d):
    B = _binding()
    code, td = DT[name]
    x = I.normal_tensor((t, d), 3.0, 16, torch.float32, "cuda")
    g = (1.0 + I.normal_tensor((d,), 0.1, 17, torch.float32, "cuda")).to(td)
    out = torch.empty((t, d), dtype=td, device="cuda")
    torch.cuda.synchronize()
    B.fp_op_rmsnorm(code, x.data_ptr(), g.data_ptr(), out.data_ptr(), t, d, 1e-5)
    torch.cuda.synchronize()
    ref = O.rmsnorm(x.cpu(), g.cpu(), 1e-5)
    assert max_rel_err(out, ref) <= TOL[name]


@pytest.mark.parametrize("name", ["bf16", "fp32"])
@pytest.mark.parametrize("t,f", [(1, 8), (33, 704), (7, 14336)])
def test_silu_mul_matches_definition(name, t, f):
    B = _binding()
    code, td = DT[name]
    gu = I.normal_tensor((t, 2 * f), 2.0, 18, td, "cuda")
    out = torch.empty((t, f), dtype=td, device="cuda")
    torch.cuda.synchronize()
    B.fp_op_silu_mul(code, gu.data_ptr(), out.data_ptr(), t, f)
    torch.cuda.synchronize()
    ref = O.silu_mul(gu.cpu())
    assert max_rel_err(out, ref) <= TOL[name]


@pytest.mark.parametrize("m,f,k", [(8192, 14336, 4096), (1000, 14336, 4096), (3000, 1000, 256), (700, 27648, 5120),
                                   (2304, 1536, 64), (2305, 1544, 576),
                                   (256, 14336, 4096), (130, 14336, 4096), (200, 6152, 1024), (500, 3080, 512)])
def test_fused_gate_up_swiglu_equals_the_two_operators(m, f, k):
    """The gate_up GEMM with SiLU(gate)*up in its epilogue gives the bits of the GEMM followed by
    the stand-alone silu_mul (ragged M, an FFN width that is not a multiple of the 128-column
    tile, both 8B and 32B shapes; the last four shapes run on the 64-column tile of short
    requests), and both agree with the definition."""
    B = _binding()
    a = I.normal_tensor((m, k), 1.0, 40, torch.bfloat16, "cuda")
    w = I.normal_tensor((2 * f, k), 0.02, 41, torch.bfloat16, "cuda")
    gu = torch.empty((m, 2 * f), dtype=torch.bfloat16, device="cuda")
    two = torch.empty((m, f), dtype=torch.bfloat16, device="cuda")
    fused = torch.full((m, f), float("nan"), dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    B.fp_op_gemm(1, a.data_ptr(), w.data_ptr(), gu.data_ptr(), m, 2 * f, k, False)
    B.fp_op_silu_mul(1, gu.data_ptr(), two.data_ptr(), m, f)
    B.fp_op_gemm_swiglu(a.data_ptr(), w.data_ptr(), fused.data_ptr(), m, f, k)
    torch.cuda.synchronize()
    assert torch.equal(fused, two)
    rows = torch.tensor(sorted(r for r in {0, 1, 255, 256, m // 2, m - 1} if r < m))
    ref = O.silu_mul(O.linear(a[rows].cpu().double(), w.cpu().double()))
    assert max_rel_err(fused[rows], ref) <= TOL["bf16"]


def test_fused_swiglu_rejects_small_problems():
    B = _binding()
    a = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.FlowPrefillError):
        B.fp_op_gemm_swiglu(a.data_ptr(), a.data_ptr(), a.data_ptr(), 16, 64, 64)


def test_bad_sizes_are_rejected_not_launched():
    B = _binding()
    a = torch.zeros(64, device="cuda")
    with pytest.raises(B.FlowPrefillError):
        B.fp_op_gemm(1, a.data_ptr(), a.data_ptr(), a.data_ptr(), 4, 8, 12, False)   # K % 8
    with pytest.raises(B.FlowPrefillError):
        B.fp_op_gemm(1, a.data_ptr(), a.data_ptr(), a.data_ptr(), 0, 8, 8, False)
    with pytest.raises(B.FlowPrefillError):
        B.fp_op_rmsnorm(1, a.data_ptr(), a.data_ptr(), a.data_ptr(), 1, 12, 1e-5)


def test_mfma_ceiling_diagnostic_reports_a_plausible_rate():
    """The register-only MFMA loop cannot beat the vendor's dense bf16 peak and, on an idle chip,
    does not fall below a third of it."""
    B = _binding()
    rate = B.fp_diag_mfma_ceiling(100)
    assert 800.0 < rate < 2600.0
    with pytest.raises(B.FlowPrefillError):
        B.fp_diag_mfma_ceiling(0)
