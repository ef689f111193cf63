// Dense projections of the prefill layer: C[M,N] = A[M,K] * W[N,K]^T (both operands K-major),
// FlowPrefill Eq. (1) and the operators qkv_proj / o_proj / gate_up_proj / down_proj of
// Section 5.1.  bf16 path: MFMA 32x32x16 tiles with fp32 accumulation, LDS-staged and
// double-buffered.  fp32 path: a plain LDS-tiled FMA kernel (debug).
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
// bf16 MFMA GEMM.  256 threads = 4 waves in a 2x2 grid; each wave owns a (BM/2)x(BN/2) block of
// 32x32 MFMA accumulators.  K is consumed 64 at a time.  LDS rows hold 64 bf16 = eight 16-byte
// chunks; chunk c of row r is stored at chunk position c ^ (r & 7) so that the eight lanes of a
// ds_read_b128 phase hit distinct banks.
// ------------------------------------------------------------------------------------------
constexpr int kBK = 64;

template <int ROWS>
__device__ __forceinline__ void load_tile_global(const bf16* __restrict__ src, int64_t ld,
                                                 int row0, int row_max, int k0, int K, int tid,
                                                 u32x4 (&regs)[ROWS / 32]) {
#pragma unroll
  for (int i = 0; i < ROWS / 32; ++i) {
    const int c = tid + i * 256;
    const int row = c >> 3, ch = c & 7;
    const int grow = min(row0 + row, row_max);
    const int k = k0 + ch * 8;
    if (k < K)
      regs[i] = *reinterpret_cast<const u32x4*>(src + (int64_t)grow * ld + k);
    else
      regs[i] = u32x4{0, 0, 0, 0};
  }
}

template <int ROWS>
__device__ __forceinline__ void store_tile_lds(bf16* dst, int tid, const u32x4 (&regs)[ROWS / 32]) {
#pragma unroll
  for (int i = 0; i < ROWS / 32; ++i) {
    const int c = tid + i * 256;
    const int row = c >> 3, ch = c & 7;
    *reinterpret_cast<u32x4*>(dst + row * kBK + ((ch ^ (row & 7)) << 3)) = regs[i];
  }
}

template <int BM, int BN, bool RESID>
__global__ __launch_bounds__(256, 1) void gemm_bf16_kernel(const bf16* __restrict__ A,
                                                           const bf16* __restrict__ W,
                                                           void* __restrict__ Cout, int M, int N,
                                                           int K, int tiles_m, int tiles_n) {
  constexpr int WTM = BM / 2, WTN = BN / 2, TM = WTM / 32, TN = WTN / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16* sA = reinterpret_cast<bf16*>(smem_raw);            // [2][BM*64]
  bf16* sB = sA + 2 * BM * kBK;                            // [2][BN*64]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
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

  u32x4 ra[BM / 32], rb[BN / 32];
  const int kt_count = (K + kBK - 1) / kBK;
  load_tile_global<BM>(A, K, m0, M - 1, 0, K, tid, ra);
  load_tile_global<BN>(W, K, n0, N - 1, 0, K, tid, rb);
  store_tile_lds<BM>(sA, tid, ra);
  store_tile_lds<BN>(sB, tid, rb);
  __syncthreads();

  const int frag_row = lane & 31, frag_half = lane >> 5;
  for (int kt = 0; kt < kt_count; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < kt_count) {
      load_tile_global<BM>(A, K, m0, M - 1, (kt + 1) * kBK, K, tid, ra);
      load_tile_global<BN>(W, K, n0, N - 1, (kt + 1) * kBK, K, tid, rb);
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
        fa[i] = *reinterpret_cast<const bf16x8*>(cA + row * kBK + ((ch ^ (row & 7)) << 3));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int row = wn * WTN + j * 32 + frag_row;
        fb[j] = *reinterpret_cast<const bf16x8*>(cB + row * kBK + ((ch ^ (row & 7)) << 3));
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < kt_count) {
      store_tile_lds<BM>(sA + (cur ^ 1) * BM * kBK, tid, ra);
      store_tile_lds<BN>(sB + (cur ^ 1) * BN * kBK, tid, rb);
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

template <int BM, int BN, bool RESID>
static void launch_bf16_cfg(const bf16* a, const bf16* w, void* c, int m, int n, int k,
                            hipStream_t s) {
  const int tiles_m = (m + BM - 1) / BM, tiles_n = (n + BN - 1) / BN;
  const size_t smem = (size_t)2 * (BM + BN) * kBK * sizeof(bf16);
  static bool attr_set = false;   // per instantiation
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<BM, BN, RESID>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    attr_set = true;
  }
  gemm_bf16_kernel<BM, BN, RESID><<<dim3((unsigned)(tiles_m * tiles_n)), 256, smem, s>>>(
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
                 int64_t k, int residual, hipStream_t s) {
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
  // 256x256 tiles when they fill the chip (>= one tile per CU); else 128x128 tiles.
  const int64_t big_tiles = ((m + 255) / 256) * ((n + 255) / 256);
  if (big_tiles >= 256) {
    if (residual) launch_bf16_cfg<256, 256, true>(pa, pw, c, (int)m, (int)n, (int)k, s);
    else launch_bf16_cfg<256, 256, false>(pa, pw, c, (int)m, (int)n, (int)k, s);
  } else {
    if (residual) launch_bf16_cfg<128, 128, true>(pa, pw, c, (int)m, (int)n, (int)k, s);
    else launch_bf16_cfg<128, 128, false>(pa, pw, c, (int)m, (int)n, (int)k, s);
  }
}

}  // namespace fp
