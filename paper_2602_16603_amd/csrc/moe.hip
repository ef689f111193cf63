// Mixture-of-experts FFN support (FlowPrefill Section 7, "Mixture-of-Experts (MoE) models": the
// `gate` operator -- a gated router -- and the `experts` operator -- several expert FFNs).
// Router: softmax over all experts of h W_r^T, the top_k most probable experts per token (ties:
// lower index), probabilities renormalised over the selected ones.  The expert FFNs run as two
// grouped GEMMs over per-expert row ranges (the first gathers the routed tokens' activations by
// index; the second one's rows are then combined, weighted, into the residual stream).  The arithmetic of a token never depends on where in an
// expert's row range it lands, so the (atomic, run-to-run varying) slot order does not reach the
// results.
#include "common.h"
#include "kernels.h"

namespace fp {

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* __restrict__ p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

void launch_fill_zero(void* p, int64_t n_dwords, hipStream_t s) {
  if (n_dwords <= 0) return;
  fill_zero_kernel<<<dim3((unsigned)((n_dwords + 255) / 256)), 256, 0, s>>>((uint32_t*)p, n_dwords);
}

// Router: one wave per token (16 waves per workgroup, 4 tokens per wave): probabilities, top_k
// selection, renormalised weights.  n_experts <= 256 (lane l holds experts l, l+64, l+128, l+192),
// top_k <= 8.  Every chosen (token, expert) pair also takes a rank among the workgroup's pairs of
// that expert (an LDS counter), and the workgroup leaves its per-expert counts in
// block_counts[block][expert]: the row plan below needs no global atomics (65536 of them on 128
// addresses cost more than the rest of the operator).
constexpr int kRouteTokensPerBlock = 64;

__global__ __launch_bounds__(1024) void moe_route_kernel(const float* __restrict__ logits,
                                                         int32_t* __restrict__ ids,
                                                         float* __restrict__ wts,
                                                         int32_t* __restrict__ rank_in_block,
                                                         int32_t* __restrict__ block_counts,
                                                         int n_tokens, int n_experts, int top_k) {
  __shared__ int hist[256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x < 256) hist[threadIdx.x] = 0;
  __syncthreads();
  for (int q = 0; q < 4; ++q) {
    const int t = blockIdx.x * kRouteTokensPerBlock + wave * 4 + q;
    if (t >= n_tokens) break;                       // wave-uniform
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane + 64 * i;
      p[i] = e < n_experts ? logits[(int64_t)t * n_experts + e] : -INFINITY;
    }
    float mx = fmaxf(fmaxf(p[0], p[1]), fmaxf(p[2], p[3]));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      p[i] = lane + 64 * i < n_experts ? expf(p[i] - mx) : -1.0f;   // -1: never selected
      sum += fmaxf(p[i], 0.f);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = p[i] >= 0.f ? p[i] * inv : -1.0f;

    float chosen_p[8];
    int chosen_e[8];
    float total = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (j < top_k) {
        float bv = p[0];
        int be = lane;
#pragma unroll
        for (int i = 1; i < 4; ++i)
          if (p[i] > bv) { bv = p[i]; be = lane + 64 * i; }        // own experts ascend with i: ties keep the lower
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
          const float ov = __shfl_xor(bv, o);
          const int oe = __shfl_xor(be, o);
          if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; }
        }
        chosen_p[j] = bv;
        chosen_e[j] = be;
        total += bv;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (be == lane + 64 * i) p[i] = -1.0f;                    // taken
      }
    }
    if (lane == 0) {
      const float norm = 1.0f / total;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (j < top_k) {
          ids[(int64_t)t * top_k + j] = chosen_e[j];
          wts[(int64_t)t * top_k + j] = chosen_p[j] * norm;
          rank_in_block[(int64_t)t * top_k + j] = atomicAdd(&hist[chosen_e[j]], 1);
        }
    }
  }
  __syncthreads();
  if (threadIdx.x < n_experts) block_counts[(int64_t)blockIdx.x * n_experts + threadIdx.x] = hist[threadIdx.x];
}

// One workgroup: per-expert totals and row offsets, the route workgroups' counts turned into
// their first row inside each expert's range (in place), and the grouped GEMMs' row-tile table.
//   plan[0 .. E) offsets;   groups[0] = row tiles, then {expert, first row, rows} per 256-row tile
__global__ __launch_bounds__(256) void moe_plan_kernel(int32_t* __restrict__ plan,
                                                       int32_t* __restrict__ block_counts,
                                                       int32_t* __restrict__ groups, int n_experts,
                                                       int n_blocks) {
  __shared__ int s_cnt[256], s_off[257], s_tile[257];
  const int e = threadIdx.x;
  int total = 0;
  if (e < n_experts)
    for (int b0 = 0; b0 < n_blocks; b0 += 16) {    // 16 loads in flight, then their prefix, then 16 stores
      int c[16];
#pragma unroll
      for (int i = 0; i < 16; ++i)
        c[i] = b0 + i < n_blocks ? block_counts[(int64_t)(b0 + i) * n_experts + e] : 0;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        if (b0 + i < n_blocks) block_counts[(int64_t)(b0 + i) * n_experts + e] = total;
        total += c[i];
      }
    }
  s_cnt[e] = total;
  __syncthreads();
  if (e == 0) {                                   // 256 LDS steps: cheaper than a parallel scan is worth
    int off = 0, tiles = 0;
    for (int i = 0; i < n_experts; ++i) {
      s_off[i] = off;
      s_tile[i] = tiles;
      off += s_cnt[i];
      tiles += (s_cnt[i] + 255) >> 8;
    }
    groups[0] = tiles;
  }
  __syncthreads();
  if (e < n_experts) {
    plan[e] = s_off[e];
    const int c = s_cnt[e];
    int n = s_tile[e];
    for (int m = 0; m < c; m += 256, ++n) {
      groups[1 + 3 * n] = e;
      groups[2 + 3 * n] = s_off[e] + m;
      groups[3 + 3 * n] = min(256, c - m);
    }
  }
}

// One thread per (token, choice): the pair's row = expert's offset + its route workgroup's first
// row for that expert + its rank there; leaves the row in slot_of and the token in row_token[row]
// (the index the grouped GEMM gathers the activations by -- they are never copied).
__global__ __launch_bounds__(256) void moe_index_kernel(const int32_t* __restrict__ ids,
                                                        const int32_t* __restrict__ plan,
                                                        const int32_t* __restrict__ block_counts,
                                                        int32_t* __restrict__ slot_of,
                                                        int32_t* __restrict__ row_token, int n_pairs,
                                                        int top_k, int n_experts) {
  const int pair = blockIdx.x * 256 + threadIdx.x;
  if (pair >= n_pairs) return;
  const int token = pair / top_k;
  const int e = ids[pair];
  const int slot = plan[e] + block_counts[(int64_t)(token / kRouteTokensPerBlock) * n_experts + e] + slot_of[pair];
  slot_of[pair] = slot;
  row_token[slot] = token;
}

// x[t] += sum_j wts[t][j] * y[slot_of[t][j]], j ascending, fp32.
__global__ __launch_bounds__(256) void moe_combine_kernel(float* __restrict__ x,
                                                          const bf16* __restrict__ y,
                                                          const int32_t* __restrict__ slot_of,
                                                          const float* __restrict__ wts, int64_t n_tokens,
                                                          int top_k, int d) {
  const int64_t d8 = d / 8;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_tokens * d8) return;
  const int64_t t = i / d8, c = i - t * d8;
  f32x8 acc = Vec8<float>::load(x + t * d + c * 8);
  for (int j = 0; j < top_k; ++j) {
    const float w = wts[t * top_k + j];
    const f32x8 v = Vec8<bf16>::load(y + (int64_t)slot_of[t * top_k + j] * d + c * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = fmaf(w, v[e], acc[e]);
  }
  Vec8<float>::store(x + t * d + c * 8, acc);
}

int moe_route_blocks(int64_t n_tokens) { return (int)((n_tokens + kRouteTokensPerBlock - 1) / kRouteTokensPerBlock); }

void launch_moe_route(const float* logits, int32_t* ids, float* wts, int32_t* slot_of, int32_t* plan,
                      int32_t* block_counts, int32_t* groups, int64_t n_tokens, int n_experts, int top_k,
                      hipStream_t s) {
  const int n_blocks = moe_route_blocks(n_tokens);
  moe_route_kernel<<<dim3((unsigned)n_blocks), 1024, 0, s>>>(logits, ids, wts, slot_of, block_counts, (int)n_tokens,
                                                           n_experts, top_k);
  moe_plan_kernel<<<1, 256, 0, s>>>(plan, block_counts, groups, n_experts, n_blocks);
}

void launch_moe_index(const int32_t* ids, const int32_t* plan, const int32_t* block_counts,
                      int32_t* slot_of, int32_t* row_token, int64_t n_tokens, int top_k, int n_experts,
                      hipStream_t s) {
  const int64_t pairs = n_tokens * top_k;
  moe_index_kernel<<<dim3((unsigned)((pairs + 255) / 256)), 256, 0, s>>>(ids, plan, block_counts, slot_of, row_token,
                                                                        (int)pairs, top_k, n_experts);
}

void launch_moe_combine(float* x, const void* y, const int32_t* slot_of, const float* wts,
                        int64_t n_tokens, int top_k, int d, hipStream_t s) {
  const int64_t n = n_tokens * (d / 8);
  moe_combine_kernel<<<dim3((unsigned)((n + 255) / 256)), 256, 0, s>>>(x, (const bf16*)y, slot_of, wts, n_tokens,
                                                                       top_k, d);
}

}  // namespace fp
