// Causal variable-length grouped-query attention over the paged KV cache
// (FlowPrefill Eq. (2) with the causal mask and KV-cache reuse of Section 3.1; operator `attn`
// of Section 5.1).  bf16 path: flash-style tiling, MFMA 32x32x16 for both contractions, fp32
// online softmax.  fp32 path: one wave per (token, head), plain FMAs (debug).
#include "common.h"
#include "kernels.h"

namespace fp {


// ------------------------------------------------------------------------------------------
// bf16 kernel.
//
// One workgroup = 8 waves = one (sequence, query tile of 256 rows, query head); each wave owns
// 32 query rows.  Two waves share a SIMD, so one wave's softmax arithmetic (VALU, exp) overlaps
// the other's MFMAs.  Keys are consumed 64 at a time (four 16-token cache blocks) from a ring of
// three LDS stages filled by DMA (buffer_load ... lds): tile t+2 is requested while tile t is
// being consumed, by waves 0..3 only, after their own P V -- they win MFMA arbitration, finish a
// tile first and would otherwise idle at the barrier, so the ~500 cycles the eight waves' 32 KB of
// requests need on the CU's 64 B/clk vector-memory path stay off the critical path.  (Loading
// through registers at the top of the tile, with the block-table look-up in front, kept every
// wave in instruction issue for 1500 of 4900 cycles per tile.)
//
// The score tile is computed TRANSPOSED, S^T = K Q^T: the MFMA accumulator layout then gives
// each lane one query column and 16 key rows per 32-key block, so the row maximum and row sum of
// the softmax are in-lane reductions plus one exchange with lane^32 (v_permlane32_swap), the
// rescale factor is a per-lane scalar, and exp(S^T) converted to bf16 is already laid out as the
// B operand of the second MFMA, O^T += V^T P^T -- no LDS round trip for P.  The row sum is taken
// over those bf16 values (the denominator then matches the numerator's weights exactly), one
// two-element dot product per packed pair; the row maximum takes one three-operand max per two
// scores.  Every VALU instruction costs issue cycles next to the other wave's MFMAs.
//
// Accumulator row i = 8a + 4h + b (a = reg/4, h = lane/32, b = reg%4) of a 32-row block, while
// the B operand wants k = 8h + e.  Loading key pi(i) into MFMA row i, pi = swap of bits 2 and 3,
// makes registers 8*a1 .. 8*a1+7 of a lane hold the 8 consecutive keys 16*a1 + 8h + (0..7): one
// B operand per 16-key chunk, matching V^T read in natural key order.
//
// The running maximum is applied lazily: the exponent reference m_use is only moved (and O, l
// rescaled) when some row's maximum has grown by more than 2^8 since the reference was set, so
// exp2 arguments stay <= 8 and almost every tile skips the D/32*16 rescale multiplies.  The
// query fragments are scaled by log2(e)/sqrt(D) once, and the score MFMAs start from an
// accumulator holding -m_use instead of zero: they deliver s - m_use, the exp2 argument,
// directly, which takes one FMA per score out of the VALU-bound softmax.
//
// LDS layouts (16-byte chunks).  Measured on gfx950: 64 banks; a ds_read_b128 is served one
// half-wave after the other, and a half-wave costs max(2, most lanes on one 16-byte bank group)
// clocks -- so a pattern is conflict-free when each half-wave puts at most two lanes on any
// 16-byte slot modulo 256 bytes:
//   K tile [64 keys][D]      chunk c of key row r stored at c ^ key(r), key chosen so that the
//                            16 rows one read phase touches fall on 16 distinct bank groups
//   V tile [4 blocks][D][16] the two 16-byte halves of channel row d swapped when d & 8
// ------------------------------------------------------------------------------------------
constexpr int kKT = 64;   // keys per tile

__device__ __forceinline__ float xhalf_max(float v) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float v) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
// acc + a + b on a packed bf16 pair (v_dot2c_f32_bf16 against (1, 1)).
__device__ __forceinline__ float pair_sum(bf16 a, bf16 b, float acc) {
  const bf16x2 p = {a, b};
  const bf16x2 one = {(__bf16)1.0f, (__bf16)1.0f};
  return __builtin_amdgcn_fdot2_f32_bf16(p, one, acc, false);
}

// LDS swizzle key of the K tile as a function of the MFMA row (= lane & 31) that reads it.
template <int D> __device__ __forceinline__ int k_key_of_lane(int lq) {
  return D == 128 ? (lq & 15) : ((lq >> 1) & 7);
}
__device__ __forceinline__ int pi_swap23(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

// DMA of one loader wave's share of a 64-key tile: IPW 1 KB instructions each for K and V.  One
// descriptor per instruction, over exactly the (block, kv head) slab it reads; a block past the
// end of the sequence gets an empty descriptor, so its rows arrive as zeros.
// Workgroup barrier without the memory fence of __syncthreads (the fence would wait for the DMA
// just issued for a later tile); callers wait for exactly the DMA they need before it.
__device__ __forceinline__ void tile_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
}

template <int D, int IPW>
__device__ __forceinline__ void dma_kv_tile(int j0, int tile, int total, const int32_t* bt,
                                            bf16* k_head, bf16* v_head, int64_t block_elems,
                                            const uint32_t (&koff)[IPW], const uint32_t (&voff)[IPW],
                                            bf16* dK, bf16* dV) {
  constexpr int IPB = D / 32;                // instructions per 16-token block
#pragma unroll
  for (int u = 0; u < IPW; ++u) {
    const int j = j0 + u;
    const int lb = tile * 4 + j / IPB;
    const bool valid = lb * kKvBlock < total;
    const int64_t blk = valid ? bt[lb] : 0;
    const int bytes = valid ? kKvBlock * D * 2 : 0;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        __builtin_amdgcn_make_buffer_rsrc(k_head + blk * block_elems, 0, bytes, 0x00020000),
        (__attribute__((address_space(3))) void*)(dK + j * 512), 16, koff[u], 0, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        __builtin_amdgcn_make_buffer_rsrc(v_head + blk * block_elems, 0, bytes, 0x00020000),
        (__attribute__((address_space(3))) void*)(dV + j * 512), 16, voff[u], 0, 0, 0);
  }
}

template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void attn_bf16_kernel(
    const bf16* __restrict__ qkv, const bf16* __restrict__ k_pool, const bf16* __restrict__ v_pool,
    bf16* __restrict__ o, int n_q_heads, int n_kv_heads, int64_t kv_num_blocks, int layer,
    const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ cached_lens,
    const int32_t* __restrict__ block_tables, int max_blocks,
    const int32_t* __restrict__ attn_items, float scale_log2) {
  static_assert(NW == 8, "work split assumes 8 waves");
  constexpr int BQW = NW * 32;
  constexpr int CPR = D / 8;                 // 16-byte chunks per key row
  constexpr int DB = D / 32;                 // 32-channel blocks of the output
  constexpr int KK = D / 16;                 // MFMA k-steps of the score contraction
  constexpr int NI = D / 8;                  // 1 KB DMA instructions per 64-key tile (K and V each)
  constexpr int NL = 4;                      // loader waves
  constexpr int IPW = NI / NL;               // DMA instructions per loader wave (K and V each)
  constexpr int RPI = 512 / D;               // key rows per K instruction
  constexpr int IPB = NI / 4;                // instructions per 16-token block
  constexpr int TILE = kKT * D;              // elements per tile buffer
  constexpr int kWaitOwnDma = 0x0F70 | (2 * IPW);   // vmcnt(2*IPW): all but the newest tile's DMA

  __shared__ __attribute__((aligned(1024))) bf16 sK0[TILE];
  __shared__ __attribute__((aligned(1024))) bf16 sK1[TILE];
  __shared__ __attribute__((aligned(1024))) bf16 sK2[TILE];
  __shared__ __attribute__((aligned(1024))) bf16 sV0[TILE];
  __shared__ __attribute__((aligned(1024))) bf16 sV1[TILE];
  __shared__ __attribute__((aligned(1024))) bf16 sV2[TILE];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31, lh = lane >> 5;
  const int group = n_q_heads / n_kv_heads;
  const int w = blockIdx.x;
  const int kvh = w % n_kv_heads;
  const int rest = w / n_kv_heads;
  const int head = kvh * group + rest % group;
  const int item = rest / group;
  const int s = attn_items[2 * item];
  const int qt = attn_items[2 * item + 1];

  const int seq_lo = cu_seqlens[s];
  const int n_new = cu_seqlens[s + 1] - seq_lo;
  const int cached = cached_lens[s];
  const int total = cached + n_new;
  const int q_row0 = qt * BQW;
  const int wq0 = q_row0 + wave * 32;
  const int kv_len = cached + min(n_new, q_row0 + BQW);
  const int n_tiles = (kv_len + kKT - 1) / kKT;
  const int64_t width = (int64_t)(n_q_heads + 2 * n_kv_heads) * D;
  const int32_t* bt = block_tables + (int64_t)s * max_blocks;
  const int64_t block_elems = (int64_t)n_kv_heads * kKvBlock * D;           // one block, all kv heads
  const int64_t head_elems = ((int64_t)layer * kv_num_blocks * n_kv_heads + kvh) * (kKvBlock * D);
  bf16* const k_head = const_cast<bf16*>(k_pool) + head_elems;              // block 0 of this layer, this kv head
  bf16* const v_head = const_cast<bf16*>(v_pool) + head_elems;
  const bool loader = wave < NL;

  // Per-lane source offsets inside one (block, kv head) slab (16 x D elements) for this wave's DMA
  // instructions.  A DMA instruction writes lane i's 16 bytes at LDS base + 16 i, so the LDS
  // swizzles are obtained by permuting which 16-byte source chunk each lane fetches.
  uint32_t koff[IPW], voff[IPW];
#pragma unroll
  for (int u = 0; u < IPW; ++u) {
    const int j = (wave & (NL - 1)) * IPW + u;          // instruction index within the tile
    const int row = j * RPI + lane / CPR;               // key row of the tile this lane fills
    const int pch = lane % CPR;
    const int src = pch ^ k_key_of_lane<D>(pi_swap23(row & 31));
    koff[u] = (uint32_t)((row % kKvBlock) * D * 2 + src * 16);
    const int q = (j % IPB) * 64 + lane;                // 16-byte slot inside the block's V slab
    const int d = q >> 1, hp = q & 1;
    voff[u] = (uint32_t)((d * 2 + (hp ^ ((d >> 3) & 1))) * 16);
  }
  auto dma_tile = [&](int tile, bf16* dK, bf16* dV) {
    dma_kv_tile<D, IPW>((wave & (NL - 1)) * IPW, tile, total, bt, k_head, v_head, block_elems, koff, voff, dK, dV);
  };

  // ---- query fragments (B operand of S^T = K Q^T), resident for the whole kernel ----
  bf16x8 qf[KK];
  {
    const int row = min(wq0 + lq, n_new - 1);
    const bf16* src = qkv + (int64_t)(seq_lo + row) * width + head * D + lh * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      // Scores come out of the MFMA already in exp2 units: q is scaled by log2(e)/sqrt(D) here,
      // once, instead of every score in every tile.
      const f32x8 q = __builtin_convertvector(*reinterpret_cast<const bf16x8*>(src + kk * 16), f32x8);
      f32x8 qs;
#pragma unroll
      for (int e = 0; e < 8; ++e) qs[e] = q[e] * scale_log2;
      qf[kk] = __builtin_convertvector(qs, bf16x8);
    }
  }

  f32x16 oacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
  float m_use = -INFINITY;      // exponent reference of this lane's query (exp2 units)
  float l_run = 0.f, l_run2 = 0.f;   // this lane's half of the row sum, in two running parts
  // -m_use in all 16 accumulator slots: the score MFMAs start from it, so they deliver s - m_use,
  // the exp2 argument, directly.  Rewritten only when the reference moves.
  f32x16 neg_m;
#pragma unroll
  for (int r = 0; r < 16; ++r) neg_m[r] = 0.f;

  const int wave_q_min = cached + wq0;               // smallest query position of the wave
  const int wave_q_max = cached + wq0 + 31;          // largest
  const int qpos = cached + wq0 + lq;
  const int pi_row = pi_swap23(lq);
  const int k_swz = k_key_of_lane<D>(lq);
  const float lazy_gap = 8.0f;                        // 2^8 of head-room
  const bool wave_valid = wq0 < n_new;

  // One tile: scores, softmax, P V from stage (cK, cV); the loader waves then start the DMA of
  // tile t + 2 into (nK, nV), the stage every wave finished reading before the previous barrier.
  auto tile_step = [&](int t, const bf16* cK, const bf16* cV, bf16* nK, bf16* nV) __attribute__((always_inline)) {
    const int key0 = t * kKT;
    if (key0 <= wave_q_max && wave_valid) {
      f32x16 sacc[2];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
        const bf16* krow = cK + (rb * 32 + pi_row) * D;
        bf16x8 kf[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
          kf[kk] = *reinterpret_cast<const bf16x8*>(krow + (((kk * 2 + lh) ^ k_swz) << 3));
        __builtin_amdgcn_sched_barrier(0);
        sacc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0], qf[0], neg_m, 0, 0, 0);
#pragma unroll
        for (int kk = 1; kk < KK; ++kk)
          sacc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], sacc[rb], 0, 0, 0);
      }
      if (key0 + kKT - 1 > wave_q_min) {              // tile straddles the diagonal: mask
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + rb * 32 + 16 * (r >> 3) + 8 * lh + (r & 7);
            sacc[rb][r] = key <= qpos ? sacc[rb][r] : -INFINITY;
          }
      }
      // sacc = s - m_use.  The first tile (m_use = -inf encoded as neg_m = 0) and any tile whose
      // row maximum exceeds the reference by more than the head-room move the reference.
      float mx0 = -INFINITY, mx1 = -INFINITY;         // one three-operand max per two scores
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        mx0 = max3(mx0, sacc[0][r], sacc[0][r + 1]);
        mx1 = max3(mx1, sacc[1][r], sacc[1][r + 1]);
      }
      const float mx = xhalf_max(fmaxf(mx0, mx1));
      // Key 0 is visible to every query, so mx is finite from the first tile on.
      if (__any(m_use == -INFINITY || mx > lazy_gap)) {
        const float shift = m_use == -INFINITY ? mx : fmaxf(mx, 0.f);   // new reference - old reference
        const float base = m_use == -INFINITY ? 0.f : m_use;
        const float alpha = m_use == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(-shift);
        m_use = base + shift;
        l_run *= alpha;
        l_run2 *= alpha;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int r = 0; r < 16; ++r) sacc[rb][r] -= shift;
#pragma unroll
        for (int r = 0; r < 16; ++r) neg_m[r] = -m_use;
      }
      // The row sum is taken over the bf16-rounded probabilities, the values P V multiplies by:
      // one two-element dot product with (1, 1) per packed pair instead of one add per score.
      bf16x8 pf[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        f32x8 pv;
#pragma unroll
        for (int e = 0; e < 8; ++e) pv[e] = __builtin_amdgcn_exp2f(sacc[c >> 1][8 * (c & 1) + e]);
        pf[c] = __builtin_convertvector(pv, bf16x8);
        l_run = pair_sum(pf[c][0], pf[c][1], l_run);
        l_run2 = pair_sum(pf[c][2], pf[c][3], l_run2);
        l_run = pair_sum(pf[c][4], pf[c][5], l_run);
        l_run2 = pair_sum(pf[c][6], pf[c][7], l_run2);
      }
#pragma unroll
      for (int i = 0; i < DB; ++i) {
        const int d = i * 32 + lq;
        const int phys = d * 2 + (lh ^ ((d >> 3) & 1));
        bf16x8 vf[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
          vf[c] = *reinterpret_cast<const bf16x8*>(cV + c * (D * kKvBlock) + (phys << 3));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c = 0; c < 4; ++c)
          oacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[c], pf[c], oacc[i], 0, 0, 0);
      }
    }
    if (loader) {
      if (t + 2 < n_tiles) {
        dma_tile(t + 2, nK, nV);
        __builtin_amdgcn_s_waitcnt(kWaitOwnDma);     // tile t+1's DMA (issued a tile ago) has landed
      } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);
      }
    }
    tile_barrier();
  };

  if (loader) {
    dma_tile(0, sK0, sV0);
    if (1 < n_tiles) dma_tile(1, sK1, sV1);
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
  tile_barrier();
  for (int t = 0; t < n_tiles; t += 3) {
    tile_step(t, sK0, sV0, sK2, sV2);
    if (t + 1 < n_tiles) tile_step(t + 1, sK1, sV1, sK0, sV0);
    if (t + 2 < n_tiles) tile_step(t + 2, sK2, sV2, sK1, sV1);
  }

  // ---- normalise, stage through LDS, store rows with 16-byte accesses ----
  bf16* stage = ((wave >> 1) == 0 ? sK0 : (wave >> 1) == 1 ? sK1 : (wave >> 1) == 2 ? sK2 : sV0) + (wave & 1) * (32 * D);
  {
    const float l_tot = xhalf_sum(l_run + l_run2);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int d = i * 32 + 8 * a + 4 * lh;
        bf16x4 v4;
#pragma unroll
        for (int b = 0; b < 4; ++b) v4[b] = static_cast<bf16>(oacc[i][4 * a + b] * inv);
        const int dch = d >> 3;
        *reinterpret_cast<bf16x4*>(stage + lq * D + ((dch ^ (lq & 7)) << 3) + (d & 7)) = v4;
      }
  }
  __syncthreads();
  const int64_t o_width = (int64_t)n_q_heads * D;
#pragma unroll
  for (int i = 0; i < 32 * CPR / 64; ++i) {
    const int idx = lane + i * 64;
    const int row = idx / CPR, dch = idx % CPR;
    if (wq0 + row < n_new) {
      u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * D + ((dch ^ (row & 7)) << 3));
      *reinterpret_cast<u32x4*>(o + (int64_t)(seq_lo + wq0 + row) * o_width + head * D + dch * 8) = v;
    }
  }
}

// ------------------------------------------------------------------------------------------
// fp32 debug kernel: one wave per (token, query head).  Lane l walks keys l, l+64, ... keeping
// its own running max / sum / weighted value sum; the 64 partial states are merged at the end.
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(64) void attn_f32_kernel(
    const float* __restrict__ qkv, const float* __restrict__ k_pool,
    const float* __restrict__ v_pool, float* __restrict__ o, int n_q_heads, int n_kv_heads,
    int64_t kv_num_blocks, int layer, const int32_t* __restrict__ tok_seq,
    const int32_t* __restrict__ tok_pos, const int32_t* __restrict__ block_tables, int max_blocks,
    float scale) {
  const int t = blockIdx.x, head = blockIdx.y, lane = threadIdx.x;
  const int s = tok_seq[t], pos = tok_pos[t];
  const int kvh = head / (n_q_heads / n_kv_heads);
  const int64_t width = (int64_t)(n_q_heads + 2 * n_kv_heads) * D;
  const float* q = qkv + (int64_t)t * width + head * D;
  const int32_t* bt = block_tables + (int64_t)s * max_blocks;
  float qv[D];
#pragma unroll
  for (int d = 0; d < D; ++d) qv[d] = q[d];
  float acc[D];
#pragma unroll
  for (int d = 0; d < D; ++d) acc[d] = 0.f;
  float m = -INFINITY, l = 0.f;
  for (int key = lane; key <= pos; key += 64) {
    const int64_t blk = bt[key / kKvBlock];
    const int64_t base = (((int64_t)layer * kv_num_blocks + blk) * n_kv_heads + kvh) *
                         (int64_t)(kKvBlock * D);
    const float* kr = k_pool + base + (key % kKvBlock) * D;
    float sc = 0.f;
#pragma unroll
    for (int d = 0; d < D; ++d) sc = fmaf(qv[d], kr[d], sc);
    sc *= scale;
    const float m_new = fmaxf(m, sc);
    const float alpha = __expf(m - m_new);
    const float p = __expf(sc - m_new);
    l = l * alpha + p;
    const float* vr = v_pool + base + (key % kKvBlock);
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] = acc[d] * alpha + p * vr[d * kKvBlock];
    m = m_new;
  }
  const float m_all = wave_max(m);
  const float w = (m == -INFINITY) ? 0.f : __expf(m - m_all);
  const float l_all = wave_sum(l * w);
  float* orow = o + (int64_t)t * n_q_heads * D + head * D;
#pragma unroll
  for (int d = 0; d < D; ++d) {
    const float v = wave_sum(acc[d] * w);
    if (lane == 0) orow[d] = v / l_all;
  }
}

int attention_q_tile_rows(int head_dim) { (void)head_dim; return 8 * 32; }

template <int D>
static void launch_attn_bf16(const void* qkv, const void* k_pool, const void* v_pool, void* o,
                             const Geometry& g, const BatchMeta& m, int layer, hipStream_t s) {
  constexpr int NW = 8;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)D);
  dim3 grid((unsigned)((int64_t)m.n_attn_items * g.n_q_heads));
  attn_bf16_kernel<D, NW><<<grid, NW * 64, 0, s>>>(
      (const bf16*)qkv, (const bf16*)k_pool, (const bf16*)v_pool, (bf16*)o, g.n_q_heads,
      g.n_kv_heads, g.kv_num_blocks, layer, m.cu_seqlens, m.cached_lens, m.block_tables,
      m.max_blocks, m.attn_items, scale_log2);
}

template <int D>
static void launch_attn_f32(const void* qkv, const void* k_pool, const void* v_pool, void* o,
                            const Geometry& g, const BatchMeta& m, int layer, hipStream_t s) {
  dim3 grid((unsigned)m.n_tokens, (unsigned)g.n_q_heads);
  attn_f32_kernel<D><<<grid, 64, 0, s>>>((const float*)qkv, (const float*)k_pool,
                                         (const float*)v_pool, (float*)o, g.n_q_heads,
                                         g.n_kv_heads, g.kv_num_blocks, layer, m.tok_seq,
                                         m.tok_pos, m.block_tables, m.max_blocks,
                                         1.0f / sqrtf((float)D));
}

void launch_attention(int dtype, const void* qkv, const void* k_pool, const void* v_pool,
                      void* o, const Geometry& g, const BatchMeta& m, int layer, hipStream_t s) {
  if (m.n_tokens == 0) return;
  if (dtype == 1) {
    if (m.n_attn_items == 0) return;
    if (g.head_dim == 128) launch_attn_bf16<128>(qkv, k_pool, v_pool, o, g, m, layer, s);
    else launch_attn_bf16<64>(qkv, k_pool, v_pool, o, g, m, layer, s);
  } else {
    switch (g.head_dim) {
      case 16: launch_attn_f32<16>(qkv, k_pool, v_pool, o, g, m, layer, s); break;
      case 32: launch_attn_f32<32>(qkv, k_pool, v_pool, o, g, m, layer, s); break;
      case 64: launch_attn_f32<64>(qkv, k_pool, v_pool, o, g, m, layer, s); break;
      default: launch_attn_f32<128>(qkv, k_pool, v_pool, o, g, m, layer, s); break;
    }
  }
}

}  // namespace fp
