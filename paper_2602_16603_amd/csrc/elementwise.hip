// HBM-bound operators of the prefill layer: residual initialisation, RMSNorm, rotary embedding
// with paged KV-cache write, SiLU(gate)*up.  All are coalesced, 16-byte-vectorised and do their
// arithmetic in fp32 (FlowPrefill Section 2.1: "FFN and residual connections"; the operators
// between the five core operators of Section 5.1).
#include "common.h"
#include "kernels.h"

namespace fp {

template <typename T> using vec8 = T __attribute__((ext_vector_type(8)));

// ------------------------------------------------------------------------------------------
// hidden_in (storage dtype) -> fp32 residual stream
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void to_residual_kernel(const T* __restrict__ in,
                                                          float* __restrict__ x, int64_t n8) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  f32x8 v = Vec8<T>::load(in + i * 8);
  Vec8<float>::store(x + i * 8, v);
}

void launch_to_residual(int dtype, const void* in, float* x, int64_t n_elems, hipStream_t s) {
  int64_t n8 = n_elems / 8;
  if (n8 == 0) return;
  dim3 grid((unsigned)((n8 + 255) / 256));
  if (dtype == 1)
    to_residual_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)in, x, n8);
  else
    to_residual_kernel<float><<<grid, 256, 0, s>>>((const float*)in, x, n8);
}

// ------------------------------------------------------------------------------------------
// RMSNorm: out = x * rsqrt(mean(x^2) + eps) * gain.  One 256-thread workgroup per token row;
// the row stays in registers between the sum-of-squares pass and the scaling pass (one HBM
// read), for rows up to 256*8*kMaxVec elements; longer rows are re-read.
// ------------------------------------------------------------------------------------------
constexpr int kNormMaxVec = 4;   // 256 threads * 8 elems * 4 = 8192 columns held in registers

template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x,
                                                      const T* __restrict__ gain,
                                                      T* __restrict__ out, int64_t d, float eps) {
  __shared__ float partial[4];
  const int tid = threadIdx.x;
  const float* row = x + (int64_t)blockIdx.x * d;
  T* orow = out + (int64_t)blockIdx.x * d;
  const int64_t n8 = d / 8;
  f32x8 held[kNormMaxVec];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < kNormMaxVec; ++i) {
    int64_t c = tid + (int64_t)i * 256;
    if (c < n8) {
      held[i] = Vec8<float>::load(row + c * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += held[i][e] * held[i][e];
    }
  }
  for (int64_t c = tid + (int64_t)kNormMaxVec * 256; c < n8; c += 256) {
    f32x8 v = Vec8<float>::load(row + c * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += v[e] * v[e];
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) partial[tid >> 6] = ss;
  __syncthreads();
  float total = partial[0] + partial[1] + partial[2] + partial[3];
  float inv = 1.0f / sqrtf(total / (float)d + eps);
#pragma unroll
  for (int i = 0; i < kNormMaxVec; ++i) {
    int64_t c = tid + (int64_t)i * 256;
    if (c < n8) {
      f32x8 g = Vec8<T>::load(gain + c * 8);
      f32x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = held[i][e] * inv * g[e];
      Vec8<T>::store(orow + c * 8, o);
    }
  }
  for (int64_t c = tid + (int64_t)kNormMaxVec * 256; c < n8; c += 256) {
    f32x8 v = Vec8<float>::load(row + c * 8);
    f32x8 g = Vec8<T>::load(gain + c * 8);
    f32x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = v[e] * inv * g[e];
    Vec8<T>::store(orow + c * 8, o);
  }
}

void launch_rmsnorm(int dtype, const float* x, const void* gain, void* out, int64_t t, int64_t d,
                    float eps, hipStream_t s) {
  if (t == 0) return;
  dim3 grid((unsigned)t);
  if (dtype == 1)
    rmsnorm_kernel<bf16><<<grid, 256, 0, s>>>(x, (const bf16*)gain, (bf16*)out, d, eps);
  else
    rmsnorm_kernel<float><<<grid, 256, 0, s>>>(x, (const float*)gain, (float*)out, d, eps);
}

// ------------------------------------------------------------------------------------------
// SiLU(gate) * up : gu [T, 2F] -> out [T, F]; gate = columns [0,F), up = columns [F,2F).
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void silu_mul_kernel(const T* __restrict__ gu,
                                                       T* __restrict__ out, int64_t t, int64_t f) {
  const int64_t f8 = f / 8;
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= t * f8) return;
  int64_t r = i / f8, c = i - r * f8;
  const T* row = gu + r * 2 * f;
  f32x8 g = Vec8<T>::load(row + c * 8);
  f32x8 u = Vec8<T>::load(row + f + c * 8);
  f32x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = silu_mul_f32(g[e], u[e]);
  Vec8<T>::store(out + r * f + c * 8, o);
}

void launch_silu_mul(int dtype, const void* gu, void* out, int64_t t, int64_t f, hipStream_t s) {
  int64_t n = t * (f / 8);
  if (n == 0) return;
  dim3 grid((unsigned)((n + 255) / 256));
  if (dtype == 1)
    silu_mul_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)gu, (bf16*)out, t, f);
  else
    silu_mul_kernel<float><<<grid, 256, 0, s>>>((const float*)gu, (float*)out, t, f);
}

// ------------------------------------------------------------------------------------------
// Rotary embedding + paged KV-cache write, one launch.
//   the first n_kv_items workgroups: one (sequence, logical block) each -- copy the raw values of
//                                 that block's new tokens into the V pool
//                                 [layer][block][Hkv][D][16] (transposed inside the block so the
//                                 attention kernel can read 8 consecutive keys of one channel
//                                 as a 16-byte MFMA operand); they take longest and go first;
//   the following T workgroups:   one token each -- rotate its Hq query heads in place in the
//                                 qkv buffer, rotate its Hkv key heads and store them into the
//                                 K pool [layer][block][Hkv][16][D].
// Pair (j, j+D/2) is rotated by angle pos * theta^(-2j/D); cos/sin come from a table computed in
// fp64 on the host.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void rope_kvwrite_kernel(
    T* __restrict__ qkv, const float* __restrict__ rope_cos, const float* __restrict__ rope_sin,
    int n_q_heads, int n_kv_heads, int head_dim, int64_t kv_num_blocks, int layer,
    T* __restrict__ k_pool, T* __restrict__ v_pool, int n_tokens,
    const int32_t* __restrict__ tok_seq, const int32_t* __restrict__ tok_pos,
    const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ cached_lens,
    const int32_t* __restrict__ block_tables, int max_blocks,
    const int32_t* __restrict__ kv_items) {
  const int tid = threadIdx.x;
  const int half = head_dim / 2;
  const int64_t width = (int64_t)(n_q_heads + 2 * n_kv_heads) * head_dim;
  const int n_kv_items = (int)gridDim.x - n_tokens;
  if ((int)blockIdx.x >= n_kv_items) {
    const int t = (int)blockIdx.x - n_kv_items;
    const int s = tok_seq[t];
    const int pos = tok_pos[t];
    const int64_t blk = block_tables[(int64_t)s * max_blocks + pos / kKvBlock];
    T* row = qkv + (int64_t)t * width;
    const float* cs = rope_cos + (int64_t)pos * half;
    const float* sn = rope_sin + (int64_t)pos * half;
    const int per_head = half / 8;
    const int units = (n_q_heads + n_kv_heads) * per_head;
    for (int u = tid; u < units; u += 256) {
      const int h = u / per_head;
      const int j = (u - h * per_head) * 8;
      T* base = row + (int64_t)h * head_dim;
      f32x8 a = Vec8<T>::load(base + j);
      f32x8 b = Vec8<T>::load(base + half + j);
      f32x8 c = Vec8<float>::load(cs + j);
      f32x8 sv = Vec8<float>::load(sn + j);
      f32x8 ra, rb;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        ra[e] = a[e] * c[e] - b[e] * sv[e];
        rb[e] = b[e] * c[e] + a[e] * sv[e];
      }
      if (h < n_q_heads) {
        Vec8<T>::store(base + j, ra);
        Vec8<T>::store(base + half + j, rb);
      } else {
        const int kh = h - n_q_heads;
        T* dst = k_pool + ((((int64_t)layer * kv_num_blocks + blk) * n_kv_heads + kh) * kKvBlock +
                           (pos % kKvBlock)) * head_dim;
        Vec8<T>::store(dst + j, ra);
        Vec8<T>::store(dst + half + j, rb);
      }
    }
    return;
  }
  // ---- value block role ----
  const int item = blockIdx.x;
  const int s = kv_items[2 * item];
  const int lb = kv_items[2 * item + 1];
  const int cached = cached_lens[s];
  const int seq_lo = cu_seqlens[s];
  const int n_new = cu_seqlens[s + 1] - seq_lo;
  const int64_t blk = block_tables[(int64_t)s * max_blocks + lb];
  const int p_lo = max(lb * kKvBlock, cached);
  const int p_hi = min(lb * kKvBlock + kKvBlock, cached + n_new);
  const bool full = (p_hi - p_lo) == kKvBlock;
  const int units = n_kv_heads * head_dim / 8;
  const int64_t v_off = (int64_t)(n_q_heads + n_kv_heads) * head_dim;
  for (int u = tid; u < units; u += 256) {
    const int kh = u / (head_dim / 8);
    const int d0 = (u - kh * (head_dim / 8)) * 8;
    T* dst = v_pool + (((int64_t)layer * kv_num_blocks + blk) * n_kv_heads + kh) *
                          ((int64_t)head_dim * kKvBlock) + (int64_t)d0 * kKvBlock;
    if (full) {
      vec8<T> v[kKvBlock];
#pragma unroll
      for (int tk = 0; tk < kKvBlock; ++tk) {
        const int64_t trow = seq_lo + (p_lo + tk - cached);
        v[tk] = *reinterpret_cast<const vec8<T>*>(qkv + trow * width + v_off + kh * head_dim + d0);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        vec8<T> lo, hi;
#pragma unroll
        for (int tk = 0; tk < 8; ++tk) {
          lo[tk] = v[tk][e];
          hi[tk] = v[tk + 8][e];
        }
        *reinterpret_cast<vec8<T>*>(dst + e * kKvBlock) = lo;
        *reinterpret_cast<vec8<T>*>(dst + e * kKvBlock + 8) = hi;
      }
    } else {
      for (int p = p_lo; p < p_hi; ++p) {
        const int64_t trow = seq_lo + (p - cached);
        vec8<T> v = *reinterpret_cast<const vec8<T>*>(qkv + trow * width + v_off + kh * head_dim + d0);
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[e * kKvBlock + (p % kKvBlock)] = v[e];
      }
    }
  }
}

void launch_rope_kvwrite(int dtype, void* qkv, const float* rope_cos, const float* rope_sin,
                         const Geometry& g, const BatchMeta& m, int layer, void* k_pool,
                         void* v_pool, hipStream_t s) {
  if (m.n_tokens == 0) return;
  dim3 grid((unsigned)(m.n_tokens + m.n_kv_items));
  if (dtype == 1)
    rope_kvwrite_kernel<bf16><<<grid, 256, 0, s>>>(
        (bf16*)qkv, rope_cos, rope_sin, g.n_q_heads, g.n_kv_heads, g.head_dim, g.kv_num_blocks,
        layer, (bf16*)k_pool, (bf16*)v_pool, m.n_tokens, m.tok_seq, m.tok_pos, m.cu_seqlens,
        m.cached_lens, m.block_tables, m.max_blocks, m.kv_items);
  else
    rope_kvwrite_kernel<float><<<grid, 256, 0, s>>>(
        (float*)qkv, rope_cos, rope_sin, g.n_q_heads, g.n_kv_heads, g.head_dim, g.kv_num_blocks,
        layer, (float*)k_pool, (float*)v_pool, m.n_tokens, m.tok_seq, m.tok_pos, m.cu_seqlens,
        m.cached_lens, m.block_tables, m.max_blocks, m.kv_items);
}

// ------------------------------------------------------------------------------------------
// Gather one sequence's keys/values of one layer from the paged pools into contiguous
// [len, Hkv, D] buffers (what a prefill instance hands to a decode instance, and what the
// parity tests compare).  One thread per 8 channels.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void kv_gather_kernel(const T* __restrict__ k_pool,
                                                        const T* __restrict__ v_pool,
                                                        T* __restrict__ k_out, T* __restrict__ v_out,
                                                        int len, int n_kv_heads, int head_dim,
                                                        int64_t kv_num_blocks, int layer,
                                                        const int32_t* __restrict__ table) {
  const int per_tok = n_kv_heads * head_dim / 8;
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)len * per_tok) return;
  const int p = (int)(i / per_tok);
  const int u = (int)(i - (int64_t)p * per_tok);
  const int kh = u / (head_dim / 8), d0 = (u % (head_dim / 8)) * 8;
  const int64_t blk = table[p / kKvBlock];
  const int64_t base = (((int64_t)layer * kv_num_blocks + blk) * n_kv_heads + kh) *
                       ((int64_t)head_dim * kKvBlock);
  const int slot = p % kKvBlock;
  vec8<T> kv = *reinterpret_cast<const vec8<T>*>(k_pool + base + (int64_t)slot * head_dim + d0);
  vec8<T> vv;
#pragma unroll
  for (int e = 0; e < 8; ++e) vv[e] = v_pool[base + (int64_t)(d0 + e) * kKvBlock + slot];
  const int64_t dst = ((int64_t)p * n_kv_heads + kh) * head_dim + d0;
  *reinterpret_cast<vec8<T>*>(k_out + dst) = kv;
  *reinterpret_cast<vec8<T>*>(v_out + dst) = vv;
}

void launch_kv_gather(int dtype, const void* k_pool, const void* v_pool, void* k_out, void* v_out,
                      int len, const Geometry& g, int layer, const int32_t* table_dev,
                      hipStream_t s) {
  if (len == 0) return;
  const int64_t n = (int64_t)len * g.n_kv_heads * g.head_dim / 8;
  dim3 grid((unsigned)((n + 255) / 256));
  if (dtype == 1)
    kv_gather_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)k_pool, (const bf16*)v_pool,
                                                (bf16*)k_out, (bf16*)v_out, len, g.n_kv_heads,
                                                g.head_dim, g.kv_num_blocks, layer, table_dev);
  else
    kv_gather_kernel<float><<<grid, 256, 0, s>>>((const float*)k_pool, (const float*)v_pool,
                                                 (float*)k_out, (float*)v_out, len, g.n_kv_heads,
                                                 g.head_dim, g.kv_num_blocks, layer, table_dev);
}

}  // namespace fp
