// Dense projections of the prefill layer: C[M,N] = A[M,K] * W[N,K]^T (both operands K-major),
// FlowPrefill Eq. (1) and the operators qkv_proj / o_proj / gate_up_proj / down_proj of
// Section 5.1.  bf16 path: MFMA tiles with fp32 accumulation, LDS-staged and double-buffered (the
// fast kernel on 16x16x32, the small-problem kernel on 32x32x16).  fp32 path: a plain LDS-tiled
// FMA kernel (debug).
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
// bf16 MFMA GEMM for tiny or odd-K problems (register-staged loads).  WGM x WGN waves; each wave
// owns a (BM/WGM)x(BN/WGN) block of 32x32 MFMA accumulators.  K is consumed 64 at a time.  LDS rows hold 64 bf16 = eight 16-byte chunks.  The
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
// bf16 MFMA GEMM, one wave per SIMD (the fast path; K % 64 == 0).
//
// 256x256 output tile, K consumed 64 at a time, 256 threads = 4 waves, one per SIMD, each with the
// whole 512-register budget: a wave owns a 128x128 block of the tile, 8x8 accumulators of 16x16 =
// 256 accumulator registers, multiplied with v_mfma_f32_16x16x32_bf16 (on random operands the
// register-only loop of this instruction sustains 2.0-2.1 PFLOP/s where 32x32x16 sustains
// 1.8-1.9: the chip is power limited and the smaller accumulator costs less energy per FLOP).
// The wave's instruction stream is software-pipelined by k-step (32 of K = 64 MFMAs = 1024
// matrix-pipe cycles): every LDS fragment read of the next k-step and every global load sits
// alone behind an MFMA, inside the 16 cycles the matrix pipe is busy with it; one s_barrier per
// k-tile.  The loop body is straight-line code on purpose: the compiler keeps the 256
// accumulators in place in the accumulation registers only while no control flow crosses them, so
// "nothing left to fetch" is expressed through an empty buffer descriptor, never through a branch.
//
// Global -> LDS goes through the DMA path (buffer_load_dwordx4 ... lds: no VGPR staging, no
// ds_write).  A DMA instruction writes lane i's 16 bytes at base + 16*i, i.e. one wave fills
// eight consecutive 128-byte LDS rows; the LDS swizzle is obtained by permuting which 16-byte
// global chunk each lane fetches.  Two LDS stages (A and W, 32 KB each per stage) as four
// separate __shared__ arrays, so that the compiler can tell that DMA in flight to one stage does
// not alias LDS reads of the other (otherwise it would serialise them with vmcnt(0)).  Wave w
// fetches rows [64w, 64w+64) of both operands, 16 instructions per k-tile, all in the k-step after
// the barrier that frees the stage; the other k-step gives them time to land.  Operand panels are addressed through raw buffer descriptors
// sized to the valid rows, so row tails of A and W read as zero.
//
// L2 warm-up.  The 32 workgroups running on one XCD share operand panels (8 tile rows x 4 tile
// columns under tile_of_workgroup), run in step, and would all ask the XCD's L2 for the same
// 128-byte lines within a few hundred cycles: one request misses and every sharer's request
// queues behind that miss (measured: 480 cycles average L2 read latency in gate_up_proj, 3300
// cycles per k-tile in down_proj).  Instead each workgroup asks for its share of the lines three
// k-tiles ahead of the DMA -- every 4th row of its A panel (wave 0) and every 8th row of its W
// panel (wave 1), the shares rotating with the k-tile -- with a one-dword-per-lane load into a
// dummy LDS pad, so the DMA requests of all sharers find the line resident (2180-2240 cycles per
// k-tile for both projections).  The pad load is the last VMEM instruction before the wave's
// wait, which therefore asks for "all but one" and never blocks on it.
// ------------------------------------------------------------------------------------------
constexpr int kWaitVm0 = 0x0F70;   // s_waitcnt vmcnt(0)           (expcnt/lgkmcnt untouched)
constexpr int kWaitVm1 = 0x0F71;   // s_waitcnt vmcnt(1)
constexpr int kWaitVm13 = 0x0F7D;  // s_waitcnt vmcnt(13)
constexpr int kWaitVm17 = 0x4F71;  // s_waitcnt vmcnt(17)
constexpr int kWaitLgkm0 = 0xC07F; // s_waitcnt lgkmcnt(0)         (vmcnt/expcnt untouched)
constexpr int kWarmAhead = 3;      // k-tiles between the L2 warm-up load and the DMA of the same lines
constexpr uint32_t kOffOutOfRange = 0x80000000u;   // a byte offset no descriptor here covers

typedef float f32x4_acc __attribute__((ext_vector_type(4)));
template <int NJ>
struct W4Frags {     // MFMA operands of one k-step (32 of K): eight 16-row blocks of A and NJ of W
  bf16x8 a[8];
  bf16x8 b[NJ];
};

// Raw buffer descriptor over `bytes` bytes at `base` (stride 0, 32-bit offsets, reads past the
// end return zero -- which is how row tails of A and W are zero-filled -- and writes past the end
// are dropped).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t panel_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ void w4_dma(__amdgpu_buffer_rsrc_t r, bf16* lds_rows, uint32_t voff, int kbyte) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void*)lds_rows, 16, voff, kbyte, 0, 0);
}

// One k-step: 8 NJ MFMAs from `cur` (A block s against the NJ W blocks, s = 0..7; NJ = 8: the
// 256-column tile described here, NJ = 4: the 128-column tile of short requests, with half the W
// fragments and DMA instructions in the same slots).  Every other
// instruction sits alone behind an MFMA: READS fragment reads of the next k-step per A block (2:
// spread over the k-step; 4: all in its first half, for the k-step that ends at the barrier, so
// that the wait in front of the barrier finds them done), in the order of their first use (all of
// W, then A blocks 0..7); if DMA, two of the wave's 16 DMA instructions per A block (0..7: its A
// rows, 8..15: its W rows, 8 rows of 128 bytes each).
// The MFMA is written as inline assembly to accumulate in place: the compiler leaves the
// destination of this 4-pass instruction free to differ from its accumulator input, which
// overflows the completely used accumulation registers (the 8-pass 32x32x16 is tied by itself).
// No accumulator is touched twice within 64 MFMAs, and LDS results reach the operands through
// the s_waitcnt the compiler places for the asm inputs, so no software-managed hazard arises.
template <int READS, bool DMA, int NJ>
__device__ __forceinline__ void w4_block(f32x4_acc (&acc)[8][NJ], const W4Frags<NJ>& cur, W4Frags<NJ>& nxt,
                                         const bf16* rA, const bf16* rB, int pch,
                                         __amdgpu_buffer_rsrc_t rs_a, __amdgpu_buffer_rsrc_t rs_w, bf16* dA,
                                         bf16* dB, const uint32_t (&voff_a)[8], const uint32_t (&voff)[8], int kbyte) {
#pragma unroll
  for (int s = 0; s < 8; ++s) {
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[s][j]) : "v"(cur.b[j]), "v"(cur.a[s]));
      if (j < READS) {
        const int r = s * READS + j;
        if (r < NJ + 8) {
          if (r < NJ) nxt.b[r] = *reinterpret_cast<const bf16x8*>(rB + r * 16 * kBK + pch);
          else nxt.a[r - NJ] = *reinterpret_cast<const bf16x8*>(rA + (r - NJ) * 16 * kBK + pch);
        }
      }
      if (DMA && (j == NJ / 2 || j == NJ / 2 + NJ / 4)) {
        const int d = 2 * s + (j != NJ / 2);
        if (d < 8) w4_dma(rs_a, dA + d * 8 * kBK, voff_a[d], kbyte);
        else if (d - 8 < NJ) w4_dma(rs_w, dB + (d - 8) * 8 * kBK, voff[d - 8], kbyte);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

__device__ __forceinline__ void w4_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
}

// EPI selects the epilogue: bf16 store, fp32 residual read-modify-write, (split-K) fp32 partial
// sums to a workspace [split][M][N] that splitk_reduce_kernel adds up in a fixed order, or the
// fused SwiGLU: W is [2N][K] = [gate rows | up rows], the tile covers 128 FFN columns, the 128 W
// rows a wave multiplies are 64 gate rows followed by the 64 up rows of the same columns, so its
// accumulator blocks [i][0..1] and [i][2..3] are gate and up of the same output elements, and the
// output [M][N] is silu(bf16(gate)) * bf16(up) -- the values, rounding included, that the
// separate gate_up GEMM + silu_mul operators produce, without the [M][2N] round trip through HBM.
enum { kEpiBf16 = 0, kEpiResidual = 1, kEpiPartial = 2, kEpiSwiGLU = 3 };

//
// GROUPED (mixture-of-experts): the launch covers many independent problems that share N and K.
// groups[0] = number of row tiles; entry i (three ints from groups[1 + 3 i]) = {expert, first
// row, rows (<= 256)}: the tile multiplies rows [first, first + rows) of A with expert's weight
// matrix (W holds the experts' matrices back to back) into the same rows of C.  The grid is sized
// for the worst case on the host; workgroups past groups[0] row tiles return at once.
// With a_rows != null the rows of A are GATHERED: row r of the launch's row space is row a_rows[r]
// of A (the tokens routed to an expert, fetched by the DMA from where they lie -- no gathered copy
// of the activations is ever written); the kernel's M argument then holds the number of rows of A.
//
// NJ = 4: the tile is half as wide (128 W rows per stage, wave tile 128 x 64).  A request of a few
// hundred tokens has one or two row tiles: the narrow tile doubles the number of output tiles, so
// the chip is occupied with half as many K ranges -- half the fp32 partial sums through memory,
// and the fused gate_up projection of a 256-token request needs no K ranges at all (measured: a
// 256-token request through the 8B-shaped stack 7.3 -> 6.5 ms; from three row tiles on the MFMAs
// bound the launch and the wide tile's operand reuse wins).
template <int EPI, bool GROUPED = false, int NJ = 8>
__global__ __launch_bounds__(256) void gemm_bf16_w4_kernel(const bf16* __restrict__ A,
                                                           const bf16* __restrict__ W,
                                                           void* __restrict__ Cout, int M, int N,
                                                           int K, int tiles_m, int tiles_n,
                                                           int kt_per_split,
                                                           const int32_t* __restrict__ groups,
                                                           const int32_t* __restrict__ a_rows) {
  constexpr bool RESID = EPI == kEpiResidual;
  constexpr bool SWIGLU = EPI == kEpiSwiGLU;
  constexpr int WR = 32 * NJ;                        // W rows per stage (256 or 128)
  constexpr int Q = WR / 4;                          // of which each wave fetches this many
  constexpr int BM = 256, BN = SWIGLU ? WR / 2 : WR; // output columns per tile
  __shared__ __attribute__((aligned(1024))) bf16 sA0[BM * kBK];
  __shared__ __attribute__((aligned(1024))) bf16 sA1[BM * kBK];
  __shared__ __attribute__((aligned(1024))) bf16 sB0[256 * kBK];   // (32 KB each also when WR = 128: the epilogue
  __shared__ __attribute__((aligned(1024))) bf16 sB1[256 * kBK];   //  stages 32 KB per wave through them)
  __shared__ __attribute__((aligned(256))) uint32_t sWarm[4 * 64];   // landing pad of the L2 warm-up loads

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 1, wn = wave >> 1;           // 2 x 2 waves, wave tile 128 x WR/2 (SwiGLU: 128 x WR/4 outputs)
  int tile_m, tile_n, share_m;
  int a_total_rows = 0;
  const int n_tiles = tiles_m * tiles_n;
  const int split = GROUPED ? 0 : blockIdx.x / n_tiles;   // which K range (0 unless split-K)
  if (GROUPED) {
    // Consecutive workgroup ids go to the 8 XCDs in turn, each with its own L2.  Every XCD takes a
    // contiguous run of the row-tile table (row tiles of one expert are neighbours in it) and walks
    // it row tile by row tile, all column tiles of a row tile in a row: the workgroups an XCD has
    // in flight then share the A panel of their row tile (all column tiles) and the W panels of
    // their expert (its two or three row tiles) through that L2, instead of each fetching both
    // panels from the fabric.
    const int n_row_tiles = groups[0];
    const int quota = (n_row_tiles + kXcds - 1) / kXcds;
    const int in_xcd = blockIdx.x / kXcds;
    const int ti = (blockIdx.x % kXcds) * quota + in_xcd / tiles_n;
    if (in_xcd / tiles_n >= quota || ti >= n_row_tiles) return;   // whole workgroup, before any barrier
    const int expert = groups[1 + 3 * ti], first = groups[2 + 3 * ti];
    a_total_rows = M;                                // gathered mode: the caller passes the rows of A here
    M = groups[3 + 3 * ti];
    if (a_rows) a_rows += first;                     // row r of the tile is row a_rows[r] of A
    else A += (int64_t)first * K;
    W += (int64_t)expert * (SWIGLU ? 2 : 1) * N * K;
    Cout = reinterpret_cast<char*>(Cout) + (int64_t)first * N * (EPI == kEpiBf16 || SWIGLU ? 2 : 4);
    tile_m = 0;
    tile_n = in_xcd % tiles_n;
    share_m = ti;
  } else {
    tile_of_workgroup(blockIdx.x - split * n_tiles, tiles_m, tiles_n, tile_m, tile_n);
    share_m = tile_m;
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int kt_first = split * kt_per_split;
  const int kt_count = min(kt_per_split, K / kBK - kt_first);
  const int kbyte0 = kt_first * kBK * 2;

  // DMA sources.  Wave w fetches LDS rows [64w, 64w+64) of each operand, 8 rows per instruction;
  // voff[j] is lane's byte offset inside the wave's 64-row panel for instruction j (the same for A
  // and W: both have K as row stride): row 8j + lane/8, 16-byte chunk (lane%8) ^ swizzle key.
  uint32_t voff[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int row = j * 8 + (lane >> 3);
    const int ch = (lane & 7) ^ ((row >> 1) & 7);
    voff[j] = (uint32_t)((row * K + ch * 8) * 2);
  }
  // A rows of the same lanes: the same offsets, unless the rows are gathered (then absolute
  // offsets into all of A, rows past the tile's end pointing outside the descriptor).
  uint32_t voff_a[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) voff_a[j] = voff[j];
  const bool gathered = GROUPED && a_rows != nullptr;
  if (gathered) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int row = 64 * wave + j * 8 + (lane >> 3);          // tile_m = 0 in grouped launches
      const int ch = (lane & 7) ^ ((row >> 1) & 7);
      const int src = row < M ? a_rows[row] : -1;
      voff_a[j] = src >= 0 ? (uint32_t)((src * K + ch * 8) * 2) : kOffOutOfRange;
    }
  }
  // Plain: W rows n0 + Q w ..; SwiGLU: LDS rows 2Q wn + (0..Q-1) are gate rows n0 + Q wn + (0..Q-1),
  // rows 2Q wn + Q + (0..Q-1) the up rows N + the same -- waves 2*wn and 2*wn+1 fetch them.
  const int w_col0 = SWIGLU ? n0 + Q * (wave >> 1) : n0 + Q * wave;
  const int64_t w_row0 = SWIGLU ? (int64_t)(wave & 1) * N + w_col0 : w_col0;
  const int a_panel_rows = __builtin_amdgcn_readfirstlane(min(64, max(0, M - m0 - 64 * wave)));
  const int w_rows = __builtin_amdgcn_readfirstlane(min(Q, max(0, N - w_col0)));
  const __amdgpu_buffer_rsrc_t rsrc_a =
      gathered ? panel_rsrc(A, (uint32_t)(a_total_rows * K * 2))
               : panel_rsrc(A + (int64_t)(m0 + 64 * wave) * K, (uint32_t)(a_panel_rows * K * 2));
  const __amdgpu_buffer_rsrc_t rsrc_w = panel_rsrc(W + w_row0 * K, (uint32_t)(w_rows * K * 2));
  const __amdgpu_buffer_rsrc_t rsrc_none = panel_rsrc(A, 0u);
  bf16* const dA0 = sA0 + 64 * wave * kBK;
  bf16* const dA1 = sA1 + 64 * wave * kBK;
  bf16* const dB0 = sB0 + Q * wave * kBK;
  bf16* const dB1 = sB1 + Q * wave * kBK;

  // L2 warm-up sources: wave 0 lane l -> A row 4l + share, wave 1 lane l < 32 -> W-stage row 8l +
  // share (SwiGLU: stage row r is gate row n0 + Q*(r/2Q) + r%Q, or the up row N + that, for
  // r%2Q >= Q).  The share is added through the scalar offset.
  uint32_t* const warm = sWarm + 64 * wave;
  const int warm_rows_a = __builtin_amdgcn_readfirstlane(min(BM, M - m0));
  const int warm_rows_w = __builtin_amdgcn_readfirstlane(SWIGLU ? N + min(BN, N - n0) : min(BN, N - n0));
  const __amdgpu_buffer_rsrc_t rsrc_warm_a = panel_rsrc(A + (int64_t)m0 * K, (uint32_t)(warm_rows_a * K * 2));
  const __amdgpu_buffer_rsrc_t rsrc_warm_w = panel_rsrc(W + (int64_t)n0 * K, (uint32_t)(warm_rows_w * K * 2));
  // (gathered rows are not contiguous: their lines are not warmed)
  const __amdgpu_buffer_rsrc_t rsrc_warm = wave == 0 ? (gathered ? rsrc_none : rsrc_warm_a) : wave == 1 ? rsrc_warm_w : rsrc_none;
  // Grouped launches: a W panel is shared by the two or three row tiles of its expert only, so
  // there every workgroup takes a quarter of the W lines (all 64 lanes, every 4th row) instead of
  // an eighth.
  constexpr int kWShares = GROUPED ? 4 : 8;
  const int warm_mask = wave == 0 ? 3 : kWShares - 1;
  const int warm_id = wave == 0 ? (tile_n & 3) : (share_m & (kWShares - 1));
  uint32_t voff_warm;
  {
    const int r0 = lane * kWShares;                  // wave 1: W-stage row of this lane's share 0
    const int64_t wrow = SWIGLU ? (int64_t)((r0 / Q) & 1) * N + Q * (r0 / (2 * Q)) + (r0 % Q) : r0;
    voff_warm = wave == 0 ? (uint32_t)(lane * 4 * K * 2) : r0 < WR ? (uint32_t)(wrow * K * 2) : kOffOutOfRange;
  }

  // MFMA fragment addresses: lane reads row (lane%16) of each 16-row block, k-chunk 4*ks + lane/16
  // of k-step ks, at its swizzled position.
  const int frag_row = lane & 15, quad = lane >> 4;
  const int key = (lane >> 1) & 7;
  const int pch0 = ((0 + quad) ^ key) << 3, pch1 = ((4 + quad) ^ key) << 3;
  const bf16* const rA0 = sA0 + (wm * 128 + frag_row) * kBK;
  const bf16* const rA1 = sA1 + (wm * 128 + frag_row) * kBK;
  const bf16* const rB0 = sB0 + (wn * (WR / 2) + frag_row) * kBK;
  const bf16* const rB1 = sB1 + (wn * (WR / 2) + frag_row) * kBK;

#define W4_WARM(u)                                                                                            \
  __builtin_amdgcn_raw_ptr_buffer_load_lds((u) < kt_count ? rsrc_warm : rsrc_none,                            \
                                           (__attribute__((address_space(3))) void*)warm, 4, voff_warm,       \
                                           kbyte0 + (u) * kBK * 2 + ((warm_id - (u)) & warm_mask) * K * 2, 0, 0)
  // Prologue: k-tile 0 into stage 0 (awaited), k-tile 1 into stage 1 (in flight), then one warm-up
  // load, so that "all but one" is the right wait from the first barrier on.
#pragma unroll
  for (int s = 0; s < 8; ++s) w4_dma(rsrc_a, dA0 + s * 8 * kBK, voff_a[s], kbyte0);
#pragma unroll
  for (int s = 0; s < NJ; ++s) w4_dma(rsrc_w, dB0 + s * 8 * kBK, voff[s], kbyte0);
  {
    const __amdgpu_buffer_rsrc_t ra1 = kt_count > 1 ? rsrc_a : rsrc_none, rw1 = kt_count > 1 ? rsrc_w : rsrc_none;
#pragma unroll
    for (int s = 0; s < 8; ++s) w4_dma(ra1, dA1 + s * 8 * kBK, voff_a[s], kbyte0 + kBK * 2);
#pragma unroll
    for (int s = 0; s < NJ; ++s) w4_dma(rw1, dB1 + s * 8 * kBK, voff[s], kbyte0 + kBK * 2);
  }
  W4_WARM(kWarmAhead - 1);
  __builtin_amdgcn_sched_barrier(0);
  // Cleared while the first k-tile is on its way.
  f32x4_acc acc[8][NJ];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) asm volatile("" : "+a"(acc[i][j]));   // materialise the zeros here, not at first use
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(NJ == 8 ? kWaitVm17 : kWaitVm13);   // all but k-tile 1 (8 + NJ) and the warm-up load
  w4_barrier();
  W4Frags<NJ> f0, f1;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    if (s < NJ) f0.b[s] = *reinterpret_cast<const bf16x8*>(rB0 + s * 16 * kBK + pch0);
    f0.a[s] = *reinterpret_cast<const bf16x8*>(rA0 + s * 16 * kBK + pch0);
  }
  __builtin_amdgcn_sched_barrier(0);

  // k-tile t on stage c (the other stage: o).  On entry f0 holds k-step 0 of tile t and tile t+1 is
  // in flight to stage o.  k-step 0 reads k-step 1's fragments; then everything but the last
  // warm-up load must have landed; the barrier tells all waves that tile t+1 is complete and stage
  // c is free; k-step 1 (fed from registers) refills stage c with tile t+2, asks for the wave's
  // share of tile t+3's lines, and starts reading tile t+1.
#define W4_TILE(t, c, o)                                                                                      \
  {                                                                                                           \
    const int t2_ = (t) + 2;                                                                                  \
    w4_block<4, false, NJ>(acc, f0, f1, rA##c, rB##c, pch1, rsrc_none, rsrc_none, dA##c, dB##c, voff_a, voff, 0); \
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);                                                                   \
    __builtin_amdgcn_s_waitcnt(kWaitVm1);                                                                     \
    w4_barrier();                                                                                             \
    w4_block<2, true, NJ>(acc, f1, f0, rA##o, rB##o, pch0, t2_ < kt_count ? rsrc_a : rsrc_none,                   \
                      t2_ < kt_count ? rsrc_w : rsrc_none, dA##c, dB##c, voff_a, voff, kbyte0 + t2_ * kBK * 2); \
    W4_WARM((t) + kWarmAhead);                                                                                \
    __builtin_amdgcn_sched_barrier(0);                                                                        \
  }
  // Eight k-tiles per trip: the taken branch at the end of a trip costs the matrix pipe about 200
  // cycles.
  int t = 0;
  for (; t + 7 < kt_count; t += 8) {
    W4_TILE(t, 0, 1);
    W4_TILE(t + 1, 1, 0);
    W4_TILE(t + 2, 0, 1);
    W4_TILE(t + 3, 1, 0);
    W4_TILE(t + 4, 0, 1);
    W4_TILE(t + 5, 1, 0);
    W4_TILE(t + 6, 0, 1);
    W4_TILE(t + 7, 1, 0);
  }
  for (; t + 1 < kt_count; t += 2) {
    W4_TILE(t, 0, 1);
    W4_TILE(t + 1, 1, 0);
  }
  if (t < kt_count) W4_TILE(t, 0, 1);
#undef W4_TILE
#undef W4_WARM
  __builtin_amdgcn_s_waitcnt(kWaitVm0);      // the trailing (empty) DMA writes have landed
  __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
  w4_barrier();                              // before the stages are reused for the epilogue
  // The compiler does not know that the assembly above writes the accumulators with MFMA latency:
  // keep the first read of them away from the last MFMA by more than any such hazard asks for
  // (the waits and the barrier above already take longer; this makes it independent of them).
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");

  // Epilogue.  The MFMAs take the W fragment as their row operand, so each 16x16 accumulator is a
  // block of C^T: accumulator [i][j] of lane l holds output row m = 16i + l%16 and the four
  // consecutive columns n = 16j + 4*(l/16) + (0..3).  The wave stages its block through its own
  // 32 KB of the (now idle) LDS stages so that global memory sees whole row segments of 128-256
  // bytes.  Global accesses go through a buffer descriptor over the wave's valid rows (rows past M
  // fall outside it, columns past N get an out-of-range offset): no branches, so the stores -- and
  // the residual reads, 16 row segments at a time -- are in flight together instead of one after
  // the other.
  bf16* region = wave == 0 ? sA0 : wave == 1 ? sA1 : wave == 2 ? sB0 : sB1;
  const int rows_valid = __builtin_amdgcn_readfirstlane(min(128, max(0, M - m0 - wm * 128)));
  if (SWIGLU) {
    // Accumulators [i][0..NJ/2-1] are gate, [i][NJ/2..NJ-1] up of outputs n0 + (WR/4)*wn + (0..WR/4-1):
    // staged as [128 rows][CH = NJ chunks of 8 bf16], chunk c of row r at position c ^ ((r>>1) & (CH-1)).
    constexpr int CH = NJ;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = i * 16 + frag_row;
      const int rkey = (row >> 1) & (CH - 1);
#pragma unroll
      for (int j = 0; j < NJ / 2; ++j) {
        bf16x4 v;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const float g = static_cast<float>(static_cast<bf16>(acc[i][j][b]));
          const float u = static_cast<float>(static_cast<bf16>(acc[i][NJ / 2 + j][b]));
          v[b] = static_cast<bf16>(silu_mul_f32(g, u));
        }
        *reinterpret_cast<bf16x4*>(region + row * (CH * 8) + (((2 * j + (quad >> 1)) ^ rkey) << 3) + 4 * (quad & 1)) = v;
      }
    }
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);     // own wave's LDS writes have landed; no other wave touches the region
    bf16* cb = reinterpret_cast<bf16*>(Cout) + (int64_t)(m0 + wm * 128) * N;
    const __amdgpu_buffer_rsrc_t rc = panel_rsrc(cb, (uint32_t)(rows_valid * N * 2));
    const int col = n0 + wn * (CH * 8) + (lane % CH) * 8;
    const uint32_t cbyte = col < N ? (uint32_t)(((lane / CH) * N + col) * 2) : kOffOutOfRange;
#pragma unroll
    for (int it = 0; it < 2 * CH; ++it) {
      const int idx = lane + it * 64;
      const int row = idx / CH, ch = idx % CH;
      const u32x4 v = *reinterpret_cast<const u32x4*>(region + row * (CH * 8) + ((ch ^ ((row >> 1) & (CH - 1))) << 3));
      __builtin_amdgcn_raw_buffer_store_b128(v, rc, cbyte, it * (64 / CH) * N * 2, 0);
    }
  } else if (EPI == kEpiBf16) {
    // [128 rows][CH = 2 NJ chunks of 8 bf16], chunk c of row r at position c ^ (r & (CH-1)).
    constexpr int CH = 2 * NJ;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = i * 16 + frag_row;
      const int rkey = row & (CH - 1);
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        bf16x4 v;
#pragma unroll
        for (int b = 0; b < 4; ++b) v[b] = static_cast<bf16>(acc[i][j][b]);
        *reinterpret_cast<bf16x4*>(region + row * (CH * 8) + (((2 * j + (quad >> 1)) ^ rkey) << 3) + 4 * (quad & 1)) = v;
      }
    }
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    bf16* cb = reinterpret_cast<bf16*>(Cout) + (int64_t)(m0 + wm * 128) * N;
    const __amdgpu_buffer_rsrc_t rc = panel_rsrc(cb, (uint32_t)(rows_valid * N * 2));
    const int col = n0 + wn * (CH * 8) + (lane % CH) * 8;
    const uint32_t cbyte = col < N ? (uint32_t)(((lane / CH) * N + col) * 2) : kOffOutOfRange;
#pragma unroll
    for (int it = 0; it < 2 * CH; ++it) {
      const int idx = lane + it * 64;
      const int row = idx / CH, ch = idx % CH;
      const u32x4 v = *reinterpret_cast<const u32x4*>(region + row * (CH * 8) + ((ch ^ (row & (CH - 1))) << 3));
      __builtin_amdgcn_raw_buffer_store_b128(v, rc, cbyte, it * (64 / CH) * N * 2, 0);
    }
  } else {
    // fp32 residual (read-modify-write) or split-K partial (plain store into this split's [M][N]
    // slab): two passes of 64 columns, staged as [128 rows][16 chunks of 4 floats], chunk c of row r
    // at position c ^ (r & 15).
    float* stage = reinterpret_cast<float*>(region);
    float* cf = reinterpret_cast<float*>(Cout) + (EPI == kEpiPartial ? (int64_t)split * M * N : 0) +
                (int64_t)(m0 + wm * 128) * N;
    const __amdgpu_buffer_rsrc_t rc = panel_rsrc(cf, (uint32_t)(rows_valid * N * 4));
    const int col0 = n0 + wn * (WR / 2) + (lane & 15) * 4;
#pragma unroll
    for (int jp = 0; jp < NJ / 4; ++jp) {
      const int col = col0 + jp * 64;
      const uint32_t cbyte = col < N ? (uint32_t)(((lane >> 4) * N + col) * 4) : kOffOutOfRange;   // N % 8 == 0: quads all-in or all-out
      f32x4 x[16];
      if (RESID) {
#pragma unroll
        for (int it = 0; it < 16; ++it)
          x[it] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rc, cbyte, it * 4 * N * 4, 0));
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int row = i * 16 + frag_row;
        const int rkey = row & 15;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          f32x4 v;
#pragma unroll
          for (int b = 0; b < 4; ++b) v[b] = acc[i][jp * 4 + jj][b];
          *reinterpret_cast<f32x4*>(stage + row * 64 + (((jj * 4 + quad) ^ rkey) << 2)) = v;
        }
      }
      __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        if (RESID && h == 1) {
#pragma unroll
          for (int it = 0; it < 16; ++it)
            x[it] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rc, cbyte, (16 + it) * 4 * N * 4, 0));
        }
#pragma unroll
        for (int it = 0; it < 16; ++it) {
          const int idx = lane + (h * 16 + it) * 64;
          const int row = idx >> 4, ch = idx & 15;
          f32x4 v = *reinterpret_cast<const f32x4*>(stage + row * 64 + ((ch ^ (row & 15)) << 2));
          if (RESID) {
#pragma unroll
            for (int b = 0; b < 4; ++b) v[b] += x[it][b];
          }
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), rc, cbyte, (h * 16 + it) * 4 * N * 4, 0);
        }
      }
      __builtin_amdgcn_s_waitcnt(kWaitLgkm0);   // the stage is rewritten by the next pass
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

// Split-K reduction of a gate_up projection fused with SiLU(gate)*up: part [splits][M][2F] fp32
// -> out [M][F].  Gate and up sums are rounded to bf16 first, so the result has the bits of
// splitk_reduce_kernel<false> into [M][2F] followed by the stand-alone silu_mul operator, without
// that intermediate.  One thread per 8 outputs.
__global__ __launch_bounds__(256) void splitk_reduce_swiglu_kernel(const float* __restrict__ part,
                                                                   bf16* __restrict__ out, int64_t m,
                                                                   int64_t f, int splits) {
  const int64_t f8 = f / 8;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= m * f8) return;
  const int64_t r = i / f8, c = i - r * f8;
  const int64_t mn = m * 2 * f;
  const float* row = part + r * 2 * f + c * 8;
  f32x8 g = Vec8<float>::load(row), u = Vec8<float>::load(row + f);
  for (int z = 1; z < splits; ++z) {
    const f32x8 gz = Vec8<float>::load(row + z * mn), uz = Vec8<float>::load(row + z * mn + f);
#pragma unroll
    for (int e = 0; e < 8; ++e) { g[e] += gz[e]; u[e] += uz[e]; }
  }
  f32x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e)
    o[e] = silu_mul_f32(static_cast<float>(static_cast<bf16>(g[e])), static_cast<float>(static_cast<bf16>(u[e])));
  Vec8<bf16>::store(out + r * f + c * 8, o);
}

// Split-K reduction of a residual projection fused with the RMSNorm that follows it: one
// 256-thread workgroup per token row adds the partial sums (in index order) and the residual,
// writes the new residual row, and normalises it from registers into h -- the arithmetic, in the
// order, of splitk_reduce_kernel<true> followed by the stand-alone RMSNorm operator, which then
// has nothing left to do.  Rows of up to kTailNormCols columns.
constexpr int kTailNormVec = 4;
constexpr int kTailNormCols = 256 * 8 * kTailNormVec;
__global__ __launch_bounds__(256) void splitk_reduce_norm_kernel(const float* __restrict__ part,
                                                                 float* __restrict__ x,
                                                                 const bf16* __restrict__ gain,
                                                                 bf16* __restrict__ h, int64_t mn, int n,
                                                                 int splits, float eps) {
  __shared__ float partial[4];
  const int tid = threadIdx.x;
  const int64_t at = (int64_t)blockIdx.x * n;
  const int n8 = n / 8;
  f32x8 held[kTailNormVec];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < kTailNormVec; ++i) {
    const int c = tid + i * 256;
    if (c < n8) {
      const f32x8 xv = Vec8<float>::load(x + at + c * 8);
      f32x8 acc = Vec8<float>::load(part + at + c * 8);
      int z = 1;
      for (; z + 3 < splits; z += 4) {               // four loads in flight; added in index order
        const f32x8 v0 = Vec8<float>::load(part + z * mn + at + c * 8);
        const f32x8 v1 = Vec8<float>::load(part + (z + 1) * mn + at + c * 8);
        const f32x8 v2 = Vec8<float>::load(part + (z + 2) * mn + at + c * 8);
        const f32x8 v3 = Vec8<float>::load(part + (z + 3) * mn + at + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = ((acc[e] + v0[e]) + v1[e]) + v2[e] + v3[e];
      }
      for (; z < splits; ++z) {
        const f32x8 v = Vec8<float>::load(part + z * mn + at + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += v[e];
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += xv[e];
      Vec8<float>::store(x + at + c * 8, acc);
      held[i] = acc;
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += acc[e] * acc[e];
    }
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) partial[tid >> 6] = ss;
  __syncthreads();
  const float total = partial[0] + partial[1] + partial[2] + partial[3];
  const float inv = 1.0f / sqrtf(total / (float)n + eps);
#pragma unroll
  for (int i = 0; i < kTailNormVec; ++i) {
    const int c = tid + i * 256;
    if (c < n8) {
      const f32x8 g = Vec8<bf16>::load(gain + c * 8);
      f32x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = held[i][e] * inv * g[e];
      Vec8<bf16>::store(h + at + c * 8, o);
    }
  }
}

// Tile width and number of K ranges for a problem.  Enough 256-column tiles to occupy the chip, or
// more than two row tiles (then the MFMAs bound the launch and the wide tile's operand reuse
// counts: measured at 768 tokens and up): the 256-column tile.  Otherwise the 128-column tile.
// Either is cut over K only as far as it takes to reach about one workgroup per CU, and never
// below 8 k-tiles (512 columns) per range.
struct W4Shape {
  int nj;       // W blocks per wave tile: 8 (256-column tile) or 4 (128-column tile)
  int splits;   // 1 = no split
};
static W4Shape w4_shape(int64_t m, int64_t n, int64_t k) {
  const int64_t tiles_m = (m + 255) / 256;
  const int64_t wide = tiles_m * ((n + 255) / 256);
  if (wide >= 160) return {8, 1};
  const bool narrow = tiles_m <= 2;
  const int64_t tiles = std::max<int64_t>(1, narrow ? tiles_m * ((n + 127) / 128) : wide);
  int s = (int)std::max<int64_t>(1, std::min<int64_t>(16, 256 / tiles));
  while (s > 1 && (k / kBK) / s < 8) --s;
  return {narrow ? 4 : 8, s};
}

// Tile of the fused gate_up projection: 128 FFN columns when that occupies the chip or the
// request has more than two row tiles, else 64.
static int swiglu_nj(int64_t m, int64_t f) {
  const int64_t tiles_m = (m + 255) / 256;
  return tiles_m <= 2 && tiles_m * ((f + 127) / 128) < 160 ? 4 : 8;
}

bool gemm_swiglu_fusable(int dtype, int64_t m, int64_t f, int64_t k) {
  if (dtype != 1 || k % kBK != 0 || f % 8 != 0 || m <= 0) return false;
  if ((f + 256) * k * 2 >= (int64_t)kOffOutOfRange) return false;   // the kernel's 32-bit offsets into the [gate | up] panel
  const int cols = swiglu_nj(m, f) * 16;
  return ((m + 255) / 256) * ((f + cols - 1) / cols) >= 96;
}

void launch_gemm_swiglu(const void* a, const void* w_gate_up, void* out, int64_t m, int64_t f,
                        int64_t k, hipStream_t s) {
  const int nj = swiglu_nj(m, f);
  const int tiles_m = (int)((m + 255) / 256), tiles_n = (int)((f + nj * 16 - 1) / (nj * 16));
  const dim3 grid((unsigned)(tiles_m * tiles_n));
  if (nj == 8)
    gemm_bf16_w4_kernel<kEpiSwiGLU><<<grid, 256, 0, s>>>((const bf16*)a, (const bf16*)w_gate_up, out, (int)m, (int)f,
                                                         (int)k, tiles_m, tiles_n, (int)(k / kBK), nullptr, nullptr);
  else
    gemm_bf16_w4_kernel<kEpiSwiGLU, false, 4><<<grid, 256, 0, s>>>((const bf16*)a, (const bf16*)w_gate_up, out, (int)m,
                                                                   (int)f, (int)k, tiles_m, tiles_n, (int)(k / kBK),
                                                                   nullptr, nullptr);
}

void launch_gemm_grouped(const void* a, const void* w, void* c, int64_t n, int64_t k, int swiglu,
                         const int32_t* groups, int max_row_tiles, const int32_t* a_rows, int64_t a_total_rows,
                         hipStream_t s) {
  const int tiles_n = (int)(swiglu ? (n + 127) / 128 : (n + 255) / 256);
  const dim3 grid((unsigned)((max_row_tiles + kXcds - 1) / kXcds * kXcds * tiles_n));   // a whole number of row tiles per XCD
  const int m_arg = a_rows ? (int)a_total_rows : 0;
  if (swiglu)
    gemm_bf16_w4_kernel<kEpiSwiGLU, true><<<grid, 256, 0, s>>>((const bf16*)a, (const bf16*)w, c, m_arg, (int)n,
                                                              (int)k, max_row_tiles, tiles_n, (int)(k / kBK), groups, a_rows);
  else
    gemm_bf16_w4_kernel<kEpiBf16, true><<<grid, 256, 0, s>>>((const bf16*)a, (const bf16*)w, c, m_arg, (int)n,
                                                            (int)k, max_row_tiles, tiles_n, (int)(k / kBK), groups, a_rows);
}

size_t gemm_workspace_bytes(int dtype, int64_t m, int64_t n, int64_t k) {
  if (dtype != 1 || k % kBK != 0) return 0;
  const int s = w4_shape(m, n, k).splits;
  return s > 1 ? (size_t)s * m * n * sizeof(float) : 0;
}

// tail: what follows the split-K reduction in the same kernel (kTailNone: nothing).
template <bool RESID, int NJ>
static void launch_bf16_w4(const bf16* a, const bf16* w, void* c, int m, int n, int k, int splits,
                           float* workspace, const GemmTail& tail, hipStream_t s) {
  constexpr int BN = 32 * NJ;
  const int tiles_m = (m + 255) / 256, tiles_n = (n + BN - 1) / BN;
  const int kt = k / kBK;
  if (splits <= 1) {
    gemm_bf16_w4_kernel<RESID ? kEpiResidual : kEpiBf16, false, NJ>
        <<<dim3((unsigned)(tiles_m * tiles_n)), 256, 0, s>>>(a, w, c, m, n, k, tiles_m, tiles_n, kt, nullptr, nullptr);
    return;
  }
  const int per = (kt + splits - 1) / splits;
  const int used = (kt + per - 1) / per;             // every launched split has at least one k-tile
  gemm_bf16_w4_kernel<kEpiPartial, false, NJ><<<dim3((unsigned)(tiles_m * tiles_n * used)), 256, 0, s>>>(
      a, w, workspace, m, n, k, tiles_m, tiles_n, per, nullptr, nullptr);
  const int64_t mn = (int64_t)m * n;
  if (RESID && tail.kind == kTailRmsNorm)
    splitk_reduce_norm_kernel<<<dim3((unsigned)m), 256, 0, s>>>(workspace, (float*)c, (const bf16*)tail.gain,
                                                               (bf16*)tail.out, mn, n, used, tail.eps);
  else if (!RESID && tail.kind == kTailSwiGLU)
    splitk_reduce_swiglu_kernel<<<dim3((unsigned)(((int64_t)m * (n / 2) / 8 + 255) / 256)), 256, 0, s>>>(
        workspace, (bf16*)tail.out, m, n / 2, used);
  else
    splitk_reduce_kernel<RESID><<<dim3((unsigned)((mn / 8 + 255) / 256)), 256, 0, s>>>(workspace, c, mn / 8,
                                                                                     mn, used);
}

template <int BM, int BN, int WGM, int WGN, bool RESID>
static void launch_bf16_cfg(const bf16* a, const bf16* w, void* c, int m, int n, int k,
                            hipStream_t s) {
  const int tiles_m = (m + BM - 1) / BM, tiles_n = (n + BN - 1) / BN;
  const size_t smem = (size_t)2 * (BM + BN) * kBK * sizeof(bf16);
  // Once per instantiation; a function-local static is initialised exactly once even when several
  // threads launch at the same time.
  static const hipError_t attr_set =
      hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<BM, BN, WGM, WGN, RESID>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  (void)attr_set;
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

// Tile and number of K ranges launch_gemm uses with that much workspace (splits 1 = uncut; 0 = the
// problem does not run on the fast kernel at all).
static W4Shape w4_plan(int dtype, int64_t m, int64_t n, int64_t k, size_t workspace_bytes) {
  if (dtype != 1 || k % kBK != 0 || n % 8 != 0 || n > (1 << 21) || k > (1 << 21)) return {8, 0};
  // (the size limits keep the fast kernel's 32-bit buffer offsets below kOffOutOfRange)
  W4Shape p = w4_shape(m, n, k);
  if (p.splits > 1 && (size_t)p.splits * m * n * sizeof(float) > workspace_bytes) p.splits = 1;
  const int64_t tiles = ((m + 255) / 256) * ((n + 32 * p.nj - 1) / (32 * p.nj));
  if (tiles * p.splits < 96) p.splits = 0;
  return p;
}

bool gemm_tail_fusable(int dtype, int64_t m, int64_t n, int64_t k, size_t workspace_bytes, int tail_kind) {
  if (w4_plan(dtype, m, n, k, workspace_bytes).splits <= 1) return false;   // tails ride on the split-K reduction
  if (tail_kind == kTailRmsNorm) return n <= kTailNormCols;
  if (tail_kind == kTailSwiGLU) return n % 16 == 0;
  return false;
}

void launch_gemm(int dtype, const void* a, const void* w, void* c, int64_t m, int64_t n,
                 int64_t k, int residual, void* workspace, size_t workspace_bytes, hipStream_t s,
                 const GemmTail* tail) {
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
  // one-wave-per-SIMD DMA kernel, split over K when the caller's workspace allows.  Otherwise (tiny or
  // odd-K problems): the register-staged kernel on 128x128 tiles.
  const W4Shape plan = w4_plan(dtype, m, n, k, workspace_bytes);
  const int splits = plan.splits;
  const GemmTail none{};
  const GemmTail& tl = tail && gemm_tail_fusable(dtype, m, n, k, workspace_bytes, tail->kind) ? *tail : none;
  if (splits >= 1 && plan.nj == 8) {
    if (residual) launch_bf16_w4<true, 8>(pa, pw, c, (int)m, (int)n, (int)k, splits, (float*)workspace, tl, s);
    else launch_bf16_w4<false, 8>(pa, pw, c, (int)m, (int)n, (int)k, splits, (float*)workspace, tl, s);
  } else if (splits >= 1) {
    if (residual) launch_bf16_w4<true, 4>(pa, pw, c, (int)m, (int)n, (int)k, splits, (float*)workspace, tl, s);
    else launch_bf16_w4<false, 4>(pa, pw, c, (int)m, (int)n, (int)k, splits, (float*)workspace, tl, s);
  } else {
    if (residual) launch_bf16_cfg<128, 128, 2, 2, true>(pa, pw, c, (int)m, (int)n, (int)k, s);
    else launch_bf16_cfg<128, 128, 2, 2, false>(pa, pw, c, (int)m, (int)n, (int)k, s);
  }
}

// ------------------------------------------------------------------------------------------
// Diagnostic: what the matrix pipes sustain on this chip with nothing else in the way -- a loop of
// v_mfma_f32_16x16x32_bf16 (the instruction of the GEMM; on random operands it sustains about 12 %
// more than v_mfma_f32_32x32x16_bf16, which attention uses) on 32 independent accumulators from
// registers, random operands (the data the pipes chew on changes the power they draw, and with it
// the clock), two waves per SIMD on every CU.  The GEMM and attention kernels are judged against
// this as well as against the vendor peak.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void mfma_ceiling_kernel(float* __restrict__ sink, int iters) {
  f32x4_acc acc[32];
#pragma unroll
  for (int i = 0; i < 32; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[i][r] = 0.f;
  bf16x8 a[4], b[8];
  uint32_t h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
#pragma unroll
  for (int f = 0; f < 12; ++f) {
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      h = h * 1664525u + 1013904223u;
      v[e] = static_cast<bf16>((float)((h >> 8) & 0xFFFF) / 65536.0f - 0.5f);
    }
    if (f < 4) a[f] = v; else b[f - 4] = v;
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
        acc[i * 8 + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i * 8 + j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 32; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) s += acc[i][r];
  sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// Launches the loop on `blocks` workgroups of 8 waves; returns the FLOPs one launch performs.
double launch_mfma_ceiling(float* sink, int blocks, int iters, hipStream_t s) {
  mfma_ceiling_kernel<<<dim3((unsigned)blocks), 512, 0, s>>>(sink, iters);
  return (double)blocks * 8.0 * (double)iters * 32.0 * 2.0 * 16.0 * 16.0 * 32.0;
}

}  // namespace fp
