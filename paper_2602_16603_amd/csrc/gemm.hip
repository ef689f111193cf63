// Dense projections of the prefill layer: C[M,N] = A[M,K] * W[N,K]^T (both operands K-major),
// FlowPrefill Eq. (1) and the operators qkv_proj / o_proj / gate_up_proj / down_proj of
// Section 5.1.  bf16 path: MFMA 32x32x16 tiles with fp32 accumulation, LDS-staged and
// double-buffered.  fp32 path: a plain LDS-tiled FMA kernel (debug).
#include <algorithm>

#include "common.h"
#include "kernels.h"

namespace fp {

// ------------------------------------------------------------------------------------------
// Workgroup -> output tile mapping.  Hardware deals consecutive workgroup ids round-robin over
// the 8 XCDs, each with its own L2.  The map gives every XCD a contiguous run of logical tiles
// and walks that run in column-panels of `kGroupM` tile rows, so the ~32 tiles an XCD has in
// flight share a small set of A row-panels and W row-panels in its L2.
// ------------------------------------------------------------------------------------------
constexpr int kXcds = 8;
constexpr int kGroupM = 8;

__device__ __forceinline__ void tile_of_workgroup(int wg, int tiles_m, int tiles_n, int& tm,
                                                  int& tn) {
  const int total = tiles_m * tiles_n;
  const int xcd = wg % kXcds;
  const int local = wg / kXcds;
  const int base = total / kXcds, rem = total % kXcds;
  const int logical = xcd * base + min(xcd, rem) + local;
  const int per_group = kGroupM * tiles_n;
  const int group = logical / per_group;
  const int in_group = logical - group * per_group;
  const int gm = min(kGroupM, tiles_m - group * kGroupM);
  tm = group * kGroupM + in_group % gm;
  tn = in_group / gm;
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA GEMM.  WGM x WGN waves; each wave owns a (BM/WGM)x(BN/WGN) block of 32x32 MFMA
// accumulators.  K is consumed 64 at a time.  LDS rows hold 64 bf16 = eight 16-byte chunks.  The
// gfx950 LDS has 64 four-byte banks (256 B per clock for reads); a ds_read_b128 is served one
// half-wave after the other and a half-wave costs max(2, most lanes on one 16-byte bank group)
// clocks.  Two consecutive 128-byte rows fill one bank period, so chunk c of row r is stored at
// chunk position c ^ ((r >> 1) & 7): the 32 rows a half-wave reads then put exactly two lanes on
// every bank group (measured: full rate, against half rate with key r & 7).
// ------------------------------------------------------------------------------------------
constexpr int kBK = 64;

template <int ROWS, int NT>
__device__ __forceinline__ void load_tile_global(const bf16* __restrict__ src, int64_t ld,
                                                 int row0, int row_max, int k0, int K, int tid,
                                                 u32x4 (&regs)[ROWS * 8 / NT]) {
#pragma unroll
  for (int i = 0; i < ROWS * 8 / NT; ++i) {
    const int c = tid + i * NT;
    const int row = c >> 3, ch = c & 7;
    const int grow = min(row0 + row, row_max);
    const int k = k0 + ch * 8;
    if (k < K)
      regs[i] = *reinterpret_cast<const u32x4*>(src + (int64_t)grow * ld + k);
    else
      regs[i] = u32x4{0, 0, 0, 0};
  }
}

template <int ROWS, int NT>
__device__ __forceinline__ void store_tile_lds(bf16* dst, int tid, const u32x4 (&regs)[ROWS * 8 / NT]) {
#pragma unroll
  for (int i = 0; i < ROWS * 8 / NT; ++i) {
    const int c = tid + i * NT;
    const int row = c >> 3, ch = c & 7;
    *reinterpret_cast<u32x4*>(dst + row * kBK + ((ch ^ ((row >> 1) & 7)) << 3)) = regs[i];
  }
}

template <int BM, int BN, int WGM, int WGN, bool RESID>
__global__ __launch_bounds__(WGM * WGN * 64) void gemm_bf16_kernel(const bf16* __restrict__ A,
                                                           const bf16* __restrict__ W,
                                                           void* __restrict__ Cout, int M, int N,
                                                           int K, int tiles_m, int tiles_n) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / 32, TN = WTN / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16* sA = reinterpret_cast<bf16*>(smem_raw);            // [2][BM*64]
  bf16* sB = sA + 2 * BM * kBK;                            // [2][BN*64]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  int tile_m, tile_n;
  tile_of_workgroup(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4 ra[BM * 8 / NT], rb[BN * 8 / NT];
  const int kt_count = (K + kBK - 1) / kBK;
  load_tile_global<BM, NT>(A, K, m0, M - 1, 0, K, tid, ra);
  load_tile_global<BN, NT>(W, K, n0, N - 1, 0, K, tid, rb);
  store_tile_lds<BM, NT>(sA, tid, ra);
  store_tile_lds<BN, NT>(sB, tid, rb);
  __syncthreads();

  const int frag_row = lane & 31, frag_half = lane >> 5;
  for (int kt = 0; kt < kt_count; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < kt_count) {
      load_tile_global<BM, NT>(A, K, m0, M - 1, (kt + 1) * kBK, K, tid, ra);
      load_tile_global<BN, NT>(W, K, n0, N - 1, (kt + 1) * kBK, K, tid, rb);
    }
    const bf16* cA = sA + cur * BM * kBK;
    const bf16* cB = sB + cur * BN * kBK;
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      bf16x8 fa[TM], fb[TN];
      const int ch = kk * 2 + frag_half;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = wm * WTM + i * 32 + frag_row;
        fa[i] = *reinterpret_cast<const bf16x8*>(cA + row * kBK + ((ch ^ ((row >> 1) & 7)) << 3));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int row = wn * WTN + j * 32 + frag_row;
        fb[j] = *reinterpret_cast<const bf16x8*>(cB + row * kBK + ((ch ^ ((row >> 1) & 7)) << 3));
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < kt_count) {
      store_tile_lds<BM, NT>(sA + (cur ^ 1) * BM * kBK, tid, ra);
      store_tile_lds<BN, NT>(sB + (cur ^ 1) * BN * kBK, tid, rb);
    }
    __syncthreads();
  }

  // Epilogue.  Accumulator register r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l%32] of its
  // 32x32 block: the 32 lanes of a half-wave write 32 consecutive columns of one row.
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn * WTN + j * 32 + frag_row;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
        if (m < M && n < N) {
          if (RESID) {
            float* c = reinterpret_cast<float*>(Cout) + (int64_t)m * N + n;
            *c = *c + acc[i][j][r];
          } else {
            reinterpret_cast<bf16*>(Cout)[(int64_t)m * N + n] = static_cast<bf16>(acc[i][j][r]);
          }
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Ping-pong bf16 MFMA GEMM (the fast path; K % 64 == 0).
//
// 256x256 output tile, K consumed 64 at a time, 512 threads = 8 waves.  The hardware places the
// waves of a workgroup round-robin on the CU's four SIMDs, so waves w and w+4 share a SIMD.  The
// two wave groups {0..3} and {4..7} run the same loop half an iteration apart: while one group
// issues its 32 MFMAs from registers ("compute phase"), the other pulls its MFMA operands for
// the same k-tile out of LDS ("memory phase"); one s_barrier ends every phase.  The matrix pipe
// of each SIMD therefore always has a wave with all operands resident, independent of how the
// compiler schedules inside a phase.
//
// Global -> LDS goes through the DMA path (buffer_load_dwordx4 ... lds: no VGPR staging, no
// ds_write).  A DMA instruction writes lane i's 16 bytes at base + 16*i, i.e. one wave fills
// eight consecutive 128-byte LDS rows; the LDS swizzle is obtained by permuting which 16-byte
// global chunk each lane fetches.  Two LDS stages (A and B, 32 KB each per stage).  Group 1
// does all the loading: during its compute phase of k-tile t -- the first moment at which both
// groups have finished reading stage t%2 -- it refills that stage with k-tile t+2, one DMA
// instruction per two MFMAs, and awaits it at the end of its next memory phase, i.e. before the
// barrier that lets group 0 start reading k-tile t+2.  Stages are separate __shared__ arrays so
// that the compiler can tell that DMA in flight to one stage does not alias LDS reads of the
// other (otherwise it would serialise them with vmcnt(0)).  Operand panels are addressed through
// raw buffer descriptors sized to the valid rows, so row tails of A and W read as zero.
// ------------------------------------------------------------------------------------------
constexpr int kWaitVm0 = 0x0F70;   // s_waitcnt vmcnt(0)           (expcnt/lgkmcnt untouched)
constexpr int kWaitLgkm0 = 0xC07F; // s_waitcnt lgkmcnt(0)         (vmcnt/expcnt untouched)

struct PpFrags {
  bf16x8 a[4][4];   // [32-row block][k-step]
  bf16x8 b[2][4];
};

// Raw buffer descriptor over `bytes` bytes at `base` (stride 0, 32-bit offsets, reads past the
// end return zero -- which is how row tails of A and W are zero-filled).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t pp_panel_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// SPLITW (the fused SwiGLU GEMM): a wave's 64 LDS rows of W are 32 gate rows followed by the 32
// up rows of the same FFN columns; they come through two descriptors (rw, rw2), each shifted so
// that the per-lane offsets of instructions 0..3 address the right rows of its panel.
template <bool SPLITW>
__device__ __forceinline__ void pp_issue_tile(__amdgpu_buffer_rsrc_t ra, __amdgpu_buffer_rsrc_t rw,
                                              __amdgpu_buffer_rsrc_t rw2, int kbyte,
                                              const uint32_t (&voff)[8], bf16* sA, bf16* sB, int w4) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int base_row = (w4 * 8 + j) * 8;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        ra, (__attribute__((address_space(3))) void*)(sA + base_row * kBK), 16, voff[j], kbyte, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        (SPLITW && j >= 4) ? rw2 : rw, (__attribute__((address_space(3))) void*)(sB + base_row * kBK), 16,
        voff[SPLITW ? (j & 3) : j], kbyte, 0, 0);
  }
}

__device__ __forceinline__ void pp_read_frags(const bf16* sA, const bf16* sB, int a_row0,
                                              int b_row0, int key, int half, PpFrags& f) {
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const int pch = ((kk * 2 + half) ^ key) << 3;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      f.a[i][kk] = *reinterpret_cast<const bf16x8*>(sA + (a_row0 + i * 32) * kBK + pch);
#pragma unroll
    for (int j = 0; j < 2; ++j)
      f.b[j][kk] = *reinterpret_cast<const bf16x8*>(sB + (b_row0 + j * 32) * kBK + pch);
  }
}

// Compute phase: the 32 MFMAs of one k-tile.  In the loading group (`load` set, wave-uniform)
// the 16 DMA instructions of one whole k-tile (8 for A, 8 for W per wave of the group) are
// slotted in one per two MFMAs, so the address unit (16 clocks per dwordx4 instruction) never
// backs up into the wave's in-order issue.  The branches are scalar and keep MFMAs and loads in
// source order without further scheduling directives.
template <bool SPLITW>
__device__ __forceinline__ void pp_mfma_and_loads(const PpFrags& f, f32x16 (&acc)[4][2], bool load,
                                                  __amdgpu_buffer_rsrc_t ra, __amdgpu_buffer_rsrc_t rw,
                                                  __amdgpu_buffer_rsrc_t rw2, int kbyte,
                                                  const uint32_t (&voff)[8], bf16* sA, bf16* sB, int w4) {
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[j][kk], f.a[i][kk], acc[i][j], 0, 0, 0);
      if (load) {
        const int slot = kk * 4 + i;            // 0..15: slots 0..7 load A rows, 8..15 load W rows
        const int base_row = (w4 * 8 + (slot & 7)) * 8;
        if (slot < 8)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(
              ra, (__attribute__((address_space(3))) void*)(sA + base_row * kBK), 16, voff[slot & 7], kbyte, 0, 0);
        else
          __builtin_amdgcn_raw_ptr_buffer_load_lds(
              (SPLITW && (slot & 7) >= 4) ? rw2 : rw, (__attribute__((address_space(3))) void*)(sB + base_row * kBK),
              16, voff[SPLITW ? (slot & 3) : (slot & 7)], kbyte, 0, 0);
      }
    }
}

__device__ __forceinline__ void pp_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
}

// EPI selects the epilogue: bf16 store, fp32 residual read-modify-write, (split-K) fp32 partial
// sums to a workspace [split][M][N] that splitk_reduce_kernel adds up in a fixed order, or the
// fused SwiGLU: W is [2N][K] = [gate rows | up rows], the tile covers 128 FFN columns, each
// wave's two 32-column accumulator blocks are gate and up of the same columns, and the output
// [M][N] is silu(bf16(gate)) * bf16(up) -- the values, rounding included, that the separate
// gate_up GEMM + silu_mul operators produce, without the [M][2N] round trip through HBM.
enum { kEpiBf16 = 0, kEpiResidual = 1, kEpiPartial = 2, kEpiSwiGLU = 3 };

//
// GROUPED (mixture-of-experts): the launch covers many independent problems that share N and K.
// groups[0] = number of row tiles; entry i (three ints from groups[1 + 3 i]) = {expert, first
// row, rows (<= 256)}: the tile multiplies rows [first, first + rows) of A with expert's weight
// matrix (W holds the experts' matrices back to back) into the same rows of C.  The grid is sized
// for the worst case on the host; workgroups past groups[0] row tiles return at once.
template <int EPI, bool GROUPED = false>
__global__ __launch_bounds__(512) void gemm_bf16_pp_kernel(const bf16* __restrict__ A,
                                                           const bf16* __restrict__ W,
                                                           void* __restrict__ Cout, int M, int N,
                                                           int K, int tiles_m, int tiles_n,
                                                           int kt_per_split,
                                                           const int32_t* __restrict__ groups) {
  constexpr bool RESID = EPI == kEpiResidual;
  constexpr bool SWIGLU = EPI == kEpiSwiGLU;
  constexpr int BM = 256, BN = SWIGLU ? 128 : 256;   // output columns per tile
  __shared__ __attribute__((aligned(1024))) bf16 sA0[BM * kBK];
  __shared__ __attribute__((aligned(1024))) bf16 sA1[BM * kBK];
  __shared__ __attribute__((aligned(1024))) bf16 sB0[256 * kBK];
  __shared__ __attribute__((aligned(1024))) bf16 sB1[256 * kBK];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int group = wave >> 2;
  const int wm = wave & 1, wn = wave >> 1;           // 2 x 4 waves, wave tile 128 x 64
  int tile_m, tile_n;
  const int n_tiles = tiles_m * tiles_n;
  const int split = GROUPED ? 0 : blockIdx.x / n_tiles;   // which K range (0 unless split-K)
  if (GROUPED) {
    const int ti = blockIdx.x / tiles_n;
    if (ti >= groups[0]) return;                     // whole workgroup, before any barrier
    const int expert = groups[1 + 3 * ti], first = groups[2 + 3 * ti];
    M = groups[3 + 3 * ti];
    A += (int64_t)first * K;
    W += (int64_t)expert * (EPI == kEpiSwiGLU ? 2 : 1) * N * K;
    Cout = reinterpret_cast<char*>(Cout) + (int64_t)first * N * (EPI == kEpiBf16 || EPI == kEpiSwiGLU ? 2 : 4);
    tile_m = 0;
    tile_n = blockIdx.x - ti * tiles_n;
  } else {
    tile_of_workgroup(blockIdx.x - split * n_tiles, tiles_m, tiles_n, tile_m, tile_n);
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int kt_first = split * kt_per_split;
  const int kt_count = min(kt_per_split, K / kBK - kt_first);
  const int kbyte0 = kt_first * kBK * 2;

  // Per-lane byte offsets of the DMA sources inside the tile's row panel (the same for the A
  // and the W panel: both have K as row stride).  The four waves of group 1 load whole k-tiles:
  // wave w4 covers rows [64*w4, 64*w4+64) of each operand, 8 rows per instruction.
  const int w4 = wave & 3;
  uint32_t voff[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int row = (w4 * 8 + j) * 8 + (lane >> 3);
    const int ch = (lane & 7) ^ ((row >> 1) & 7);
    voff[j] = (uint32_t)((row * K + ch * 8) * 2);
  }
  const __amdgpu_buffer_rsrc_t rsrc_a =
      pp_panel_rsrc(A + (int64_t)m0 * K, (uint32_t)(min(BM, M - m0) * K * 2));
  // SwiGLU: gate rows n0 + 32*w4 .. +31 and up rows N + n0 + 32*w4 .. +31 sit at LDS rows 64*w4 ..
  // of the W stage; shifting each panel's base back by 32*w4 rows makes voff[0..3] (built for LDS
  // rows 64*w4 + 0..31) address them, and the bound moves with it.
  const int w_shift = SWIGLU ? 32 * w4 : 0;
  const uint32_t w_bytes = (uint32_t)((w_shift + min(BN, N - n0)) * K * 2);
  const __amdgpu_buffer_rsrc_t rsrc_w = pp_panel_rsrc(W + ((int64_t)n0 - w_shift) * K, w_bytes);
  const __amdgpu_buffer_rsrc_t rsrc_w2 =
      pp_panel_rsrc(W + ((int64_t)N + n0 - w_shift) * K, SWIGLU ? w_bytes : 0u);

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  if (group == 1) {
    pp_issue_tile<SWIGLU>(rsrc_a, rsrc_w, rsrc_w2, kbyte0, voff, sA0, sB0, w4);
    if (kt_count > 1) pp_issue_tile<SWIGLU>(rsrc_a, rsrc_w, rsrc_w2, kbyte0 + kBK * 2, voff, sA1, sB1, w4);
    __builtin_amdgcn_s_waitcnt(kWaitVm0);
  }
  pp_barrier();

  const int frag_row = lane & 31, half = lane >> 5;
  const int key = (lane >> 1) & 7;
  const int a_row0 = wm * 128 + frag_row, b_row0 = wn * 64 + frag_row;
  PpFrags f;

  // One iteration = memory phase + compute phase of k-tile t on the given stage.
  auto iteration = [&](int t, bf16* sA, bf16* sB, bf16* sA_other, bf16* sB_other) {
    // -- memory phase --
    pp_read_frags(sA, sB, a_row0, b_row0, key, half, f);
    if (group == 1) __builtin_amdgcn_s_waitcnt(kWaitVm0);   // k-tile t+1, issued one iteration ago
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    pp_barrier();
    // -- compute phase --
    // Both groups have finished reading this stage (group 0 one phase ago, group 1 just now):
    // group 1 refills it with k-tile t+2 while it computes.
    pp_mfma_and_loads<SWIGLU>(f, acc, group == 1 && t + 2 < kt_count, rsrc_a, rsrc_w, rsrc_w2,
                              kbyte0 + (t + 2) * kBK * 2, voff, sA, sB, w4);
    pp_barrier();
  };

  if (group == 1) pp_barrier();                          // run half an iteration behind group 0
  for (int t = 0; t < kt_count; t += 2) {
    iteration(t, sA0, sB0, sA1, sB1);
    if (t + 1 < kt_count) iteration(t + 1, sA1, sB1, sA0, sB0);
  }
  if (group == 0) pp_barrier();

  // Epilogue.  The MFMAs take the W fragment as their row operand, so each 32x32 accumulator is
  // a block of C^T: lane l holds output row m = l%32 and, per register quad a, the four
  // consecutive columns n = 8a + 4*(l/32) + (0..3).
  // Each wave stages its block through its own 16 KB of the (now idle) LDS stages so that global
  // memory sees whole 128-byte row segments (8 full cache lines per instruction) instead of the
  // 8/16-byte pieces the accumulator layout would give.
  bf16* region = (wave >> 1) == 0 ? sA0 : (wave >> 1) == 1 ? sA1 : (wave >> 1) == 2 ? sB0 : sB1;
  region += (wave & 1) * (128 * 64);
  if (SWIGLU) {
    // acc[i][0] = gate, acc[i][1] = up for output columns n0 + 32*wn + (0..31).  Staged as
    // [128 rows][4 chunks of 8 bf16], chunk c of row r at position c ^ ((r>>2)&3), then stored as
    // 64-byte row segments with 16-byte accesses.
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = i * 32 + frag_row;
      const int rkey = (row >> 2) & 3;
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        bf16x4 v;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const float g = static_cast<float>(static_cast<bf16>(acc[i][0][4 * a + b]));
          const float u = static_cast<float>(static_cast<bf16>(acc[i][1][4 * a + b]));
          v[b] = static_cast<bf16>(silu_mul_f32(g, u));
        }
        *reinterpret_cast<bf16x4*>(region + row * 32 + ((a ^ rkey) << 3) + 4 * half) = v;
      }
    }
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);     // own wave's LDS writes have landed; no other wave touches the region
    bf16* cbase = reinterpret_cast<bf16*>(Cout) + (int64_t)(m0 + wm * 128) * N + n0 + wn * 32;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int idx = lane + it * 64;
      const int row = idx >> 2, ch = idx & 3;
      const u32x4 v = *reinterpret_cast<const u32x4*>(region + row * 32 + ((ch ^ ((row >> 2) & 3)) << 3));
      if (m0 + wm * 128 + row < M && n0 + wn * 32 + ch * 8 < N)
        *reinterpret_cast<u32x4*>(cbase + (int64_t)row * N + ch * 8) = v;
    }
  } else if (EPI != kEpiBf16) {
    // fp32 residual (read-modify-write) or split-K partial (plain store into this split's
    // [M][N] slab): two passes of 32 columns, staged as [128 rows][8 chunks of 4 floats], chunk c
    // of row r at position c ^ ((r>>1)&7).
    float* stage = reinterpret_cast<float*>(region);
    float* cf = reinterpret_cast<float*>(Cout) + (EPI == kEpiPartial ? (int64_t)split * M * N : 0) +
                (int64_t)(m0 + wm * 128) * N + n0 + wn * 64;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = i * 32 + frag_row;
        const int rkey = (row >> 1) & 7;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          f32x4 v;
#pragma unroll
          for (int b = 0; b < 4; ++b) v[b] = acc[i][j][4 * a + b];
          *reinterpret_cast<f32x4*>(stage + row * 32 + (((2 * a + half) ^ rkey) << 2)) = v;
        }
      }
      __builtin_amdgcn_s_waitcnt(kWaitLgkm0);   // own wave's LDS writes have landed; no other wave touches the region
#pragma unroll
      for (int it = 0; it < 16; ++it) {
        const int idx = lane + it * 64;
        const int row = idx >> 3, ch = idx & 7;
        f32x4 v = *reinterpret_cast<const f32x4*>(stage + row * 32 + ((ch ^ ((row >> 1) & 7)) << 2));
        if (m0 + wm * 128 + row < M && n0 + wn * 64 + j * 32 + ch * 4 < N) {   // N % 8 == 0: quads all-in or all-out
          f32x4* c = reinterpret_cast<f32x4*>(cf + (int64_t)row * N + j * 32 + ch * 4);
          if (RESID) {
            const f32x4 x = *c;
#pragma unroll
            for (int b = 0; b < 4; ++b) v[b] += x[b];
          }
          *c = v;
        }
      }
    }
  } else {
    // bf16 output: staged as [128 rows][8 chunks of 8 bf16], chunk c of row r at position
    // c ^ ((r>>1)&7), then stored as whole 128-byte rows with 16-byte accesses.
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = i * 32 + frag_row;
      const int rkey = (row >> 1) & 7;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          bf16x4 v;
#pragma unroll
          for (int b = 0; b < 4; ++b) v[b] = static_cast<bf16>(acc[i][j][4 * a + b]);
          *reinterpret_cast<bf16x4*>(region + row * 64 + (((j * 4 + a) ^ rkey) << 3) + 4 * half) = v;
        }
    }
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);     // own wave's LDS writes have landed; no other wave touches the region
    bf16* cbase = reinterpret_cast<bf16*>(Cout) + (int64_t)(m0 + wm * 128) * N + n0 + wn * 64;
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const int idx = lane + it * 64;
      const int row = idx >> 3, ch = idx & 7;
      const u32x4 v = *reinterpret_cast<const u32x4*>(region + row * 64 + ((ch ^ ((row >> 1) & 7)) << 3));
      if (m0 + wm * 128 + row < M && n0 + wn * 64 + ch * 8 < N)
        *reinterpret_cast<u32x4*>(cbase + (int64_t)row * N + ch * 8) = v;
    }
  }
}

// Split-K reduction: out[m][n] = sum over splits (in index order: deterministic) of the fp32
// partials, added into the fp32 residual or rounded to bf16.  One thread per 8 outputs.
template <bool RESID>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part,
                                                            void* __restrict__ out, int64_t mn8,
                                                            int64_t mn, int splits) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= mn8) return;
  f32x8 acc = Vec8<float>::load(part + i * 8);
  for (int z = 1; z < splits; ++z) {
    const f32x8 v = Vec8<float>::load(part + z * mn + i * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += v[e];
  }
  if (RESID) {
    float* o = reinterpret_cast<float*>(out) + i * 8;
    const f32x8 x = Vec8<float>::load(o);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += x[e];
    Vec8<float>::store(o, acc);
  } else {
    Vec8<bf16>::store(reinterpret_cast<bf16*>(out) + i * 8, acc);
  }
}

// How many K ranges to cut a problem into so that a launch has about one workgroup per CU:
// only when the 256x256 tiles alone leave most of the chip idle, and never below 8 k-tiles
// (512 columns) per range.  1 = no split.
static int pp_splits(int64_t m, int64_t n, int64_t k) {
  const int64_t tiles = ((m + 255) / 256) * ((n + 255) / 256);
  if (tiles <= 0 || tiles >= 160) return 1;
  int s = (int)std::min<int64_t>(16, 256 / tiles);
  while (s > 1 && (k / kBK) / s < 8) --s;
  return s;
}

bool gemm_swiglu_fusable(int dtype, int64_t m, int64_t f, int64_t k) {
  if (dtype != 1 || k % kBK != 0 || f % 8 != 0 || m <= 0) return false;
  const int64_t tiles = ((m + 255) / 256) * ((f + 127) / 128);
  return tiles >= 96 && pp_splits(m, 2 * f, k) == 1;
}

void launch_gemm_swiglu(const void* a, const void* w_gate_up, void* out, int64_t m, int64_t f,
                        int64_t k, hipStream_t s) {
  const int tiles_m = (int)((m + 255) / 256), tiles_n = (int)((f + 127) / 128);
  gemm_bf16_pp_kernel<kEpiSwiGLU><<<dim3((unsigned)(tiles_m * tiles_n)), 512, 0, s>>>(
      (const bf16*)a, (const bf16*)w_gate_up, out, (int)m, (int)f, (int)k, tiles_m, tiles_n,
      (int)(k / kBK), nullptr);
}

void launch_gemm_grouped(const void* a, const void* w, void* c, int64_t n, int64_t k, int swiglu,
                         const int32_t* groups, int max_row_tiles, hipStream_t s) {
  const int tiles_n = (int)(swiglu ? (n + 127) / 128 : (n + 255) / 256);
  const dim3 grid((unsigned)(max_row_tiles * tiles_n));
  if (swiglu)
    gemm_bf16_pp_kernel<kEpiSwiGLU, true><<<grid, 512, 0, s>>>((const bf16*)a, (const bf16*)w, c, 0, (int)n,
                                                              (int)k, max_row_tiles, tiles_n, (int)(k / kBK), groups);
  else
    gemm_bf16_pp_kernel<kEpiBf16, true><<<grid, 512, 0, s>>>((const bf16*)a, (const bf16*)w, c, 0, (int)n,
                                                            (int)k, max_row_tiles, tiles_n, (int)(k / kBK), groups);
}

size_t gemm_workspace_bytes(int dtype, int64_t m, int64_t n, int64_t k) {
  if (dtype != 1 || k % kBK != 0) return 0;
  const int s = pp_splits(m, n, k);
  return s > 1 ? (size_t)s * m * n * sizeof(float) : 0;
}

template <bool RESID>
static void launch_bf16_pp(const bf16* a, const bf16* w, void* c, int m, int n, int k, int splits,
                           float* workspace, hipStream_t s) {
  const int tiles_m = (m + 255) / 256, tiles_n = (n + 255) / 256;
  const int kt = k / kBK;
  if (splits <= 1) {
    gemm_bf16_pp_kernel<RESID ? kEpiResidual : kEpiBf16>
        <<<dim3((unsigned)(tiles_m * tiles_n)), 512, 0, s>>>(a, w, c, m, n, k, tiles_m, tiles_n, kt, nullptr);
    return;
  }
  const int per = (kt + splits - 1) / splits;
  const int used = (kt + per - 1) / per;             // every launched split has at least one k-tile
  gemm_bf16_pp_kernel<kEpiPartial><<<dim3((unsigned)(tiles_m * tiles_n * used)), 512, 0, s>>>(
      a, w, workspace, m, n, k, tiles_m, tiles_n, per, nullptr);
  const int64_t mn = (int64_t)m * n;
  splitk_reduce_kernel<RESID><<<dim3((unsigned)((mn / 8 + 255) / 256)), 256, 0, s>>>(workspace, c, mn / 8,
                                                                                   mn, used);
}

template <int BM, int BN, int WGM, int WGN, bool RESID>
static void launch_bf16_cfg(const bf16* a, const bf16* w, void* c, int m, int n, int k,
                            hipStream_t s) {
  const int tiles_m = (m + BM - 1) / BM, tiles_n = (n + BN - 1) / BN;
  const size_t smem = (size_t)2 * (BM + BN) * kBK * sizeof(bf16);
  static bool attr_set = false;   // per instantiation
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<BM, BN, WGM, WGN, RESID>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    attr_set = true;
  }
  gemm_bf16_kernel<BM, BN, WGM, WGN, RESID><<<dim3((unsigned)(tiles_m * tiles_n)), WGM * WGN * 64, smem, s>>>(
      a, w, c, m, n, k, tiles_m, tiles_n);
}

// ------------------------------------------------------------------------------------------
// fp32 debug GEMM: 64x64 tile, 256 threads, 4x4 outputs per thread, K step 16, plain FMAs.
// ------------------------------------------------------------------------------------------
template <bool RESID>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A,
                                                       const float* __restrict__ W,
                                                       float* __restrict__ C, int M, int N,
                                                       int K) {
  __shared__ float sA[16][64 + 1];
  __shared__ float sW[16][64 + 1];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256;          // 0..1023 = 64 rows x 16 k
      const int row = e >> 4, kk = e & 15;
      const int gm = m0 + row, gn = n0 + row, gk = k0 + kk;
      sA[kk][row] = (gm < M && gk < K) ? A[(int64_t)gm * K + gk] : 0.f;
      sW[kk][row] = (gn < N && gk < K) ? W[(int64_t)gn * K + gk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = sA[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = sW[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) {
        float* c = C + (int64_t)m * N + n;
        *c = RESID ? (*c + acc[i][j]) : acc[i][j];
      }
    }
}

void launch_gemm(int dtype, const void* a, const void* w, void* c, int64_t m, int64_t n,
                 int64_t k, int residual, void* workspace, size_t workspace_bytes, hipStream_t s) {
  if (m == 0 || n == 0) return;
  if (dtype == 0) {
    dim3 grid((unsigned)((n + 63) / 64), (unsigned)((m + 63) / 64));
    if (residual)
      gemm_f32_kernel<true><<<grid, 256, 0, s>>>((const float*)a, (const float*)w, (float*)c,
                                                  (int)m, (int)n, (int)k);
    else
      gemm_f32_kernel<false><<<grid, 256, 0, s>>>((const float*)a, (const float*)w, (float*)c,
                                                   (int)m, (int)n, (int)k);
    return;
  }
  const bf16* pa = (const bf16*)a;
  const bf16* pw = (const bf16*)w;
  // K a multiple of 64 and enough 256x256 tiles (or enough K to split) to occupy the chip: the
  // ping-pong DMA kernel, split over K when the caller's workspace allows.  Otherwise (tiny or
  // odd-K problems): the register-staged kernel on 128x128 tiles.
  const int64_t big_tiles = ((m + 255) / 256) * ((n + 255) / 256);
  int splits = k % kBK == 0 ? pp_splits(m, n, k) : 1;
  if (splits > 1 && (size_t)splits * m * n * sizeof(float) > workspace_bytes) splits = 1;
  if (k % kBK == 0 && big_tiles * splits >= 96) {
    if (residual) launch_bf16_pp<true>(pa, pw, c, (int)m, (int)n, (int)k, splits, (float*)workspace, s);
    else launch_bf16_pp<false>(pa, pw, c, (int)m, (int)n, (int)k, splits, (float*)workspace, s);
  } else {
    if (residual) launch_bf16_cfg<128, 128, 2, 2, true>(pa, pw, c, (int)m, (int)n, (int)k, s);
    else launch_bf16_cfg<128, 128, 2, 2, false>(pa, pw, c, (int)m, (int)n, (int)k, s);
  }
}

// ------------------------------------------------------------------------------------------
// Diagnostic: what the matrix pipes sustain on this chip with nothing else in the way -- a loop of
// v_mfma_f32_32x32x16_bf16 on eight independent accumulators from registers, random operands
// (the data the pipes chew on changes the power they draw, and with it the clock), two waves per
// SIMD on every CU.  The GEMM and attention kernels are judged against this as well as against
// the vendor peak.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void mfma_ceiling_kernel(float* __restrict__ sink, int iters) {
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  bf16x8 a, b;
  uint32_t h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    h = h * 1664525u + 1013904223u;
    a[e] = static_cast<bf16>((float)((h >> 8) & 0xFFFF) / 65536.0f - 0.5f);
    h = h * 1664525u + 1013904223u;
    b[e] = static_cast<bf16>((float)((h >> 8) & 0xFFFF) / 65536.0f - 0.5f);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// Launches the loop on `blocks` workgroups of 8 waves; returns the FLOPs one launch performs.
double launch_mfma_ceiling(float* sink, int blocks, int iters, hipStream_t s) {
  mfma_ceiling_kernel<<<dim3((unsigned)blocks), 512, 0, s>>>(sink, iters);
  return (double)blocks * 8.0 * (double)iters * 8.0 * 2.0 * 32.0 * 32.0 * 16.0;
}

}  // namespace fp
