// Host-callable launchers of the prefill operators.  Each launches on the given stream and
// returns without synchronising; hipGetLastError is left for the caller to check.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fp {

// Static geometry of the model that the kernels need.
struct Geometry {
  int32_t hidden, n_q_heads, n_kv_heads, head_dim, ffn;
  int64_t kv_num_blocks;
  int32_t qkv_width() const { return (n_q_heads + 2 * n_kv_heads) * head_dim; }
};

// Per-task device-side description of the packed batch.
struct BatchMeta {
  int32_t n_tokens;             // T
  int32_t n_seqs;
  int32_t max_blocks;           // row length of block_tables
  const int32_t* tok_seq;       // device [T]   sequence of each packed token
  const int32_t* tok_pos;       // device [T]   absolute position (cached_len + index in chunk)
  const int32_t* cu_seqlens;    // device [n_seqs+1]
  const int32_t* cached_lens;   // device [n_seqs]
  const int32_t* block_tables;  // device [n_seqs, max_blocks]
  const int32_t* kv_items;      // device [n_kv_items][2]  (seq, logical block) touched by new tokens
  int32_t n_kv_items;
  const int32_t* attn_items;    // device [n_attn_items][2] (seq, query tile), longest first
  int32_t n_attn_items;
};

// Rows of queries one attention workgroup owns on the bf16 path (the runtime sizes attn_items
// with it).
int attention_q_tile_rows(int head_dim);

void launch_to_residual(int dtype, const void* in, float* x, int64_t n_elems, hipStream_t s);
void launch_rmsnorm(int dtype, const float* x, const void* gain, void* out, int64_t t, int64_t d,
                    float eps, hipStream_t s);
void launch_silu_mul(int dtype, const void* gu, void* out, int64_t t, int64_t f, hipStream_t s);
// qkv [T, qkv_width] in place for the query columns; rotated keys and raw values go to the pools.
void launch_rope_kvwrite(int dtype, void* qkv, const float* rope_cos, const float* rope_sin,
                         const Geometry& g, const BatchMeta& m, int layer, void* k_pool,
                         void* v_pool, hipStream_t s);
void launch_attention(int dtype, const void* qkv, const void* k_pool, const void* v_pool,
                      void* o, const Geometry& g, const BatchMeta& m, int layer, hipStream_t s);
// C[M,N] = A[M,K] W[N,K]^T  (residual == 0, C in the storage dtype), or C_f32 += ... (residual).
// `workspace` (device, may be null) holds split-K partial sums for problems too small to fill the
// chip with output tiles alone; gemm_workspace_bytes says how much such a problem wants (0 if
// it would not split).  Without enough workspace the problem runs unsplit.
// `tail` (may be null): the operator that follows the projection, carried out by the split-K
// reduction kernel when -- and only when -- gemm_tail_fusable says so for the same arguments
// (short requests: one launch and one pass over the data fewer):
//   kTailRmsNorm  residual projections: tail.out [M,N] (storage dtype) = rmsnorm(updated C row) * tail.gain
//   kTailSwiGLU   gate_up projection (N = 2F, gate columns first): tail.out [M,F] = silu(gate) * up and C
//                 is NOT written
// with the bits the stand-alone operators give.
enum { kTailNone = 0, kTailRmsNorm = 1, kTailSwiGLU = 2 };
struct GemmTail {
  int kind = kTailNone;
  const void* gain = nullptr;
  void* out = nullptr;
  float eps = 0.f;
};
bool gemm_tail_fusable(int dtype, int64_t m, int64_t n, int64_t k, size_t workspace_bytes, int tail_kind);
void launch_gemm(int dtype, const void* a, const void* w, void* c, int64_t m, int64_t n,
                 int64_t k, int residual, void* workspace, size_t workspace_bytes, hipStream_t s,
                 const GemmTail* tail = nullptr);
size_t gemm_workspace_bytes(int dtype, int64_t m, int64_t n, int64_t k);
// Fused gate_up projection + SiLU(gate)*up (bf16): out[m][f] from a[m][k] and w_gate_up[2f][k]
// (gate rows first), bit-identical to launch_gemm into [m][2f] followed by launch_silu_mul.
// Only for problems gemm_swiglu_fusable accepts (K % 64 == 0, f % 8 == 0, enough tiles to fill the
// chip without splitting K).
bool gemm_swiglu_fusable(int dtype, int64_t m, int64_t f, int64_t k);
void launch_gemm_swiglu(const void* a, const void* w_gate_up, void* out, int64_t m, int64_t f,
                        int64_t k, hipStream_t s);
// Grouped bf16 GEMM for mixture-of-experts layers (K % 64 == 0, n % 8 == 0): `groups` (device) =
// {row tiles, then {expert, first row, rows <= 256} per row tile}; row tile i multiplies those
// rows with expert's matrix of w ([experts][n][k], or [experts][2n][k] gate rows then up rows when
// swiglu) into the same rows of c [*, n] (bf16; swiglu: silu(gate)*up).  The rows are rows of a
// [*, k] itself (a_rows == null) or, gathered, rows a_rows[first row + r] of a [a_total_rows, k]
// (a_total_rows * k < 2^30).  The grid covers max_row_tiles row tiles; the surplus exits.
void launch_gemm_grouped(const void* a, const void* w, void* c, int64_t n, int64_t k, int swiglu,
                         const int32_t* groups, int max_row_tiles, const int32_t* a_rows,
                         int64_t a_total_rows, hipStream_t s);

// Gathers positions 0..len-1 of one sequence (block table row `table_dev`, device) of one layer
// into contiguous k_out/v_out [len, Hkv, D].
void launch_kv_gather(int dtype, const void* k_pool, const void* v_pool, void* k_out, void* v_out,
                      int len, const Geometry& g, int layer, const int32_t* table_dev,
                      hipStream_t s);

// Mixture-of-experts FFN (bf16 path).  plan = device int32 [n_experts] (row offset of every
// expert); block_counts = device int32 [moe_route_blocks(T)][n_experts]; slot_of = device int32
// [T*top_k] (rank inside the route workgroup after launch_moe_route, final row after
// launch_moe_gather); groups = device int32 [1 + 3 * (T*top_k/256 + n_experts)]: the row-tile
// table launch_gemm_grouped reads.
void launch_fill_zero(void* p, int64_t n_dwords, hipStream_t s);
int moe_route_blocks(int64_t n_tokens);
void launch_moe_route(const float* logits, int32_t* ids, float* wts, int32_t* slot_of, int32_t* plan,
                      int32_t* block_counts, int32_t* groups, int64_t n_tokens, int n_experts, int top_k,
                      hipStream_t s);
void launch_moe_index(const int32_t* ids, const int32_t* plan, const int32_t* block_counts,
                      int32_t* slot_of, int32_t* row_token, int64_t n_tokens, int top_k, int n_experts,
                      hipStream_t s);
void launch_moe_combine(float* x, const void* y, const int32_t* slot_of, const float* wts,
                        int64_t n_tokens, int top_k, int d, hipStream_t s);

// Register-only MFMA loop (diagnostic); sink = device float[blocks * 512]; returns FLOPs per launch.
double launch_mfma_ceiling(float* sink, int blocks, int iters, hipStream_t s);

// Sets the calling thread's fp_last_error() text (for translation units other than the runtime).
void set_last_error(const char* message);

}  // namespace fp
