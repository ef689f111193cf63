/*
 * flowprefill.h -- C ABI of the op-preemptible transformer prefill for AMD MI355X (gfx950).
 *
 * The library runs the prefill forward pass of a dense pre-norm decoder (RMSNorm, fused QKV
 * projection, rotary embedding + paged KV-cache write, causal variable-length GQA attention,
 * output projection, RMSNorm, fused gate/up projection, SiLU*up, down projection) as a
 * sequence of individually launched HIP kernels, with a cooperative preemption check at every
 * operator boundary.  It follows FlowPrefill (arxiv 2602.16603):
 *   - Section 2.1, Eq. (1)-(2): what a layer computes;
 *   - Section 5.1 "Operator-Level Preemption": checks between the core operators qkv_proj, attn,
 *     o_proj, gate_up_proj, down_proj; on a signal the runtime lets the operator in flight
 *     finish, acknowledges, and suspends the task with its state kept; latency is bounded by
 *     one operator;
 *   - Section 4 "Execution Pool": at most one task runs; preempted tasks keep their state until
 *     resumed; the pool obeys three commands -- submit, preempt, resume.
 * submit = fp_prefill_begin + fp_prefill_advance, preempt = fp_preempt, resume = fp_resume +
 * fp_prefill_advance.
 *
 * Conventions
 *   - Every pointer argument says "host" or "device".  Device pointers are plain HIP device
 *     addresses on the current device.  The library never frees caller memory.
 *   - All tensors are row-major and token-major.  Weights are [out, in]; y = x W^T.
 *     w_qkv rows: [Hq*D query rows | Hkv*D key rows | Hkv*D value rows]; w_gate_up rows:
 *     [F gate rows | F up rows].
 *   - dtype FP_DTYPE_F32: weights, input hidden states, KV cache and all intermediates are
 *     fp32 (debug path).  FP_DTYPE_BF16: weights, input hidden states, intermediates and KV
 *     cache are bf16; accumulation, softmax, norm and SiLU arithmetic is fp32.  In BOTH modes the
 *     residual stream is kept in fp32 and fp_prefill_hidden returns fp32.
 *   - Every function returns fp_status; negative values are errors and leave the handle as it
 *     was.  fp_last_error() gives a thread-local message for the last error on this thread.
 *   - No C++ exception crosses this boundary.
 *
 * One layer is 9 operators (cursor positions 0..8):
 *   0 rmsnorm_attn  1 qkv_proj  2 rope_kvwrite  3 attn  4 o_proj(+residual)
 *   5 rmsnorm_mlp   6 gate_up_proj  7 silu_mul  8 down_proj(+residual)
 * The paper's five boundaries are after positions 1, 3, 4, 6, 8.
 *
 * Mixture-of-experts models (Section 7: the FFN becomes the two operators `gate` and `experts`)
 * keep the nine positions; 6-8 become
 *   6 gate          router logits, softmax over all experts, top_k experts per token (ties: lower
 *                   index), probabilities renormalised over the selected experts
 *   7 experts_up    tokens gathered per expert; gate/up projection + SiLU*up of every expert
 *   8 experts_down  down projection of every expert; weighted sum into the residual stream
 * so the paper's boundaries (after gate, after experts) are again positions 6 and 8.
 */
#ifndef FLOWPREFILL_H
#define FLOWPREFILL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fp_model fp_model;     /* immutable after create                                  */
typedef struct fp_prefill fp_prefill; /* one execution task of the Execution Pool (Section 4)    */

typedef enum {
  FP_OK = 0,          /* advanced; more operators remain                                         */
  FP_DONE = 1,        /* all n_layers*9 operators finished and the stream is drained             */
  FP_PREEMPTED = 2,   /* parked at an operator boundary; device quiesced; acknowledgement sent   */
  FP_ERR_INVALID = -1,
  FP_ERR_OOM = -2,
  FP_ERR_STATE = -3,  /* call not legal in the handle's state (e.g. resume of a running task)    */
  FP_ERR_DEVICE = -4
} fp_status;

enum { FP_DTYPE_F32 = 0, FP_DTYPE_BF16 = 1 };
enum { FP_OPS_PER_LAYER = 9 };

/* boundary_mask: bit i set = a preemption check sits after operator i of every layer.          */
#define FP_BOUNDARY_EVERY_OP 0x1FFu /* all nine operators                                        */
#define FP_BOUNDARY_PAPER_OPS 0x15Au /* after qkv_proj, attn, o_proj, gate_up_proj, down_proj    */
#define FP_BOUNDARY_LAYER 0x100u    /* only after down_proj (layer-level preemption, Fig. 5)     */
#define FP_BOUNDARY_NONE 0x0u       /* none: a preempt request waits for completion (chunk-level)*/

typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn;
  float rms_eps, rope_theta;
  int32_t dtype;            /* FP_DTYPE_*                                                        */
  int32_t kv_block_tokens;  /* tokens per KV block; must be 16                                   */
  int64_t kv_num_blocks;    /* size of the block pool; one block id addresses all layers         */
  int32_t max_position;     /* RoPE table length = largest sequence length (prefix + new tokens) */
  int32_t n_experts;        /* 0 = dense FFN.  > 0: mixture-of-experts FFN (Section 7), bf16 only: */
  int32_t top_k;            /*   top_k of n_experts experts per token, `ffn` = one expert's width  */
} fp_shape;

/* Device pointers, BORROWED: the caller owns them and keeps them alive and unchanged for the
 * life of the model.  attn_norm/mlp_norm [hidden]; w_qkv [(Hq+2Hkv)*D, hidden]; w_o [hidden,
 * Hq*D]; w_gate_up [2*ffn, hidden]; w_down [hidden, ffn]; element type per fp_shape.dtype.
 * All must be 16-byte aligned.                                                                   */
typedef struct {
  const void *attn_norm, *w_qkv, *w_o, *mlp_norm, *w_gate_up, *w_down;
  const void* w_router;     /* mixture-of-experts models only (else NULL): [n_experts, hidden];
                             * then w_gate_up is [n_experts, 2*ffn, hidden] and w_down
                             * [n_experts, hidden, ffn], one expert after the other            */
} fp_layer_weights;

/* Creates a model: validates the shape (hidden, Hq*D, ffn multiples of 8; head_dim 64 or 128 on
 * the bf16 path; Hq multiple of Hkv), builds the RoPE cos/sin table on the host in fp64 and
 * uploads it as fp32, and allocates the paged KV pool:
 *   K pool [n_layers][kv_num_blocks][Hkv][16 tokens][D]   (keys after rotation)
 *   V pool [n_layers][kv_num_blocks][Hkv][D][16 tokens]   (values, transposed inside a block)
 * `layers` is a host array of n_layers entries.  `hip_stream` is the hipStream_t every kernel of
 * this model's tasks is launched on (NULL = the default stream).  Errors: FP_ERR_INVALID,
 * FP_ERR_OOM, FP_ERR_DEVICE.                                                                      */
fp_status fp_model_create(const fp_shape* shape, const fp_layer_weights* layers /*host*/,
                          void* hip_stream, fp_model** out);
/* Frees the pool, the tables, cached workspaces and pooled events.  All tasks must have been
 * ended: while any task of the model is alive the call frees nothing, leaves the model usable and
 * sets fp_last_error() (the tasks' buffers live in the model's pools).                            */
void fp_model_destroy(fp_model* model);

/* KV block allocator of the pool (host bookkeeping only).  fp_kv_alloc writes n distinct free
 * block ids to ids_out (host) or fails with FP_ERR_OOM taking none.  fp_kv_free returns them.    */
fp_status fp_kv_alloc(fp_model* model, int32_t n, int32_t* ids_out /*host*/);
fp_status fp_kv_free(fp_model* model, int32_t n, const int32_t* ids /*host*/);
/* Device base addresses of the whole K and V pools (layouts above; layer 0 first).              */
fp_status fp_model_kv_pools(const fp_model* model, const void** k_pool /*device*/,
                            const void** v_pool /*device*/);

/* "submit" (Section 4; Alg. 2 submit_new_execution): creates a task for a request set of n_seqs
 * prompts (or prompt chunks) packed token-major.
 *   hidden_in    device [T, hidden] in the storage dtype, T = cu_seqlens[n_seqs]; widened into
 *                the task's own fp32 residual buffer by a kernel this call enqueues on the
 *                model's stream WITHOUT waiting for it: the caller keeps hidden_in valid and
 *                unchanged until the first fp_prefill_advance on the task has returned (or the
 *                stream has otherwise drained); the library never writes it.
 *   cu_seqlens   host [n_seqs+1], non-decreasing, cu_seqlens[0] = 0.  Empty sequences allowed.
 *   cached_lens  host [n_seqs] tokens of each sequence already in the cache (earlier chunks), or
 *                NULL for all zero.  Token i of sequence s has position cached_lens[s] + i.
 *   block_tables host [n_seqs, max_blocks] physical block ids covering positions
 *                0 .. cached_lens[s]+len_s-1 of each sequence (entry b holds positions
 *                16b..16b+15); NULL = the library allocates blocks from the pool (then
 *                cached_lens must be NULL/zero) and frees them in fp_prefill_end.
 *   boundary_mask which operator boundaries carry a preemption check (FP_BOUNDARY_*).
 * The task starts idle with its cursor at (layer 0, op 0).  Errors: FP_ERR_INVALID (bad
 * lengths, block id out of range, position beyond max_position), FP_ERR_OOM, FP_ERR_DEVICE.      */
fp_status fp_prefill_begin(fp_model* model, const void* hidden_in /*device*/,
                           const int32_t* cu_seqlens /*host*/, int32_t n_seqs,
                           const int32_t* cached_lens /*host or NULL*/,
                           const int32_t* block_tables /*host or NULL*/, int32_t max_blocks,
                           uint32_t boundary_mask, fp_prefill** out);

/* Runs up to max_ops operators from the cursor, one kernel launch sequence per operator, with a
 * check of the preemption signal at each enabled boundary (Section 5.1).  Returns when the
 * operators it issued have completed on the device:
 *   FP_OK         max_ops operators ran, more remain;
 *   FP_DONE       the last operator of the last layer has completed;
 *   FP_PREEMPTED  a signal was seen at a boundary: signal cleared, acknowledgement sent, task
 *                 parked (fp_resume needed before the next advance).
 * *ops_done (host, may be NULL) receives the number of operators executed by this call.
 * Only one thread may be inside advance for a given task; fp_preempt may be called from
 * another thread meanwhile.  FP_ERR_STATE if the task is parked or already done.                 */
fp_status fp_prefill_advance(fp_prefill* task, int32_t max_ops, int32_t* ops_done /*host*/);

/* How many operators may be enqueued on the stream beyond the one known complete.  With k >= 1
 * the host launches an operator only once all but the last k-1 of the operators enqueued before
 * it have completed (operators that launch nothing -- their work rides in a neighbour's kernel --
 * take no place in that window), so a signal is honoured within k operators.  Default 2 (no
 * launch bubble; at most the running and one queued operator finish before the acknowledgement).  k = 0 removes the bound (and the per-operator event): the
 * host enqueues as fast as it can and a signal is honoured only after everything enqueued so far
 * has run -- meant for short requests whose operators last tens of microseconds.                 */
fp_status fp_prefill_set_launch_ahead(fp_prefill* task, int32_t k);

/* "preempt" (Section 5.1, Fig. 6): thread-safe.  Sets the task's signal and blocks until the
 * runtime acknowledges at the next enabled boundary with the device quiesced (FP_PREEMPTED), or
 * until the task completes first (FP_DONE).  On an idle task (no advance in flight) parks it at
 * once.  FP_ERR_STATE if already parked.  fp_preempt = fp_preempt_signal + fp_preempt_wait; the
 * split lets a caller time exactly the signal -> acknowledgement interval (Section 6.4).         */
fp_status fp_preempt(fp_prefill* task);
fp_status fp_preempt_signal(fp_prefill* task);
fp_status fp_preempt_wait(fp_prefill* task);

/* "resume" (Alg. 2 resume_execution): parked -> idle; the next advance continues from the
 * cursor with the task's workspace and KV blocks untouched.  FP_ERR_STATE unless parked.         */
fp_status fp_resume(fp_prefill* task);

/* Cursor = the next operator to run: layer in [0, n_layers], op in [0, 9).  (n_layers, 0) = done.
 * The layer/operator cursor is part of the preserved state of a task (Section 4, Execution Pool).
 * Thread-safe: may be polled from any thread while another one is inside fp_prefill_advance.     */
fp_status fp_prefill_cursor(const fp_prefill* task, int32_t* layer /*host*/, int32_t* op /*host*/);

/* The fp32 residual stream [T, hidden] (device, owned by the task, valid until fp_prefill_end).
 * After FP_DONE it is the stack's output; at a layer boundary it is that layer's input.          */
fp_status fp_prefill_hidden(const fp_prefill* task, const void** dev_ptr);

/* The preserved KV state of a task (Section 4, "Execution Pool": a preempted task keeps its
 * partial KV cache until it is resumed; Section 3.1: later chunks and the decode phase read it):
 * device base addresses of layer `layer`'s slice of the paged pools,
 *   *k_pool [kv_num_blocks][Hkv][16][D], *v_pool [kv_num_blocks][Hkv][D][16] (storage dtype),
 * and the task's block tables, host [n_seqs, max_blocks] (row s, entry b = physical block of
 * positions 16b..16b+15 of sequence s; max_blocks from fp_prefill_block_tables).  All three stay
 * owned by the model / the task and are valid until fp_prefill_end.  Blocks of layers the cursor
 * has not passed yet hold whatever the pool held before.  Does not synchronise: read the device
 * memory only while the task is not running (parked, idle between advance calls, or done).
 * FP_ERR_INVALID for a null argument or a layer outside [0, n_layers).                           */
fp_status fp_prefill_kv(const fp_prefill* task, int32_t layer, const void** k_pool /*device*/,
                        const void** v_pool /*device*/, const int32_t** block_tables_host);

/* The task's block tables (host [n_seqs, max_blocks], owned by the task) and max_blocks.         */
fp_status fp_prefill_block_tables(const fp_prefill* task, const int32_t** tables_host,
                                  int32_t* max_blocks /*host*/);

/* Copies positions 0 .. cached_lens[seq]+len_seq-1 of sequence `seq`, layer `layer`, out of the
 * paged pools into the caller's contiguous device buffers k_out, v_out [len, Hkv, D] (storage
 * dtype): keys as cached (rotated), values raw.  This is the hand-over format for a decode
 * instance and what parity tests compare.  Synchronises the stream before returning.             */
fp_status fp_prefill_kv_gather(const fp_prefill* task, int32_t layer, int32_t seq,
                               void* k_out /*device*/, void* v_out /*device*/);

/* Device time of each operator of the task's most recent advance call, in milliseconds, when
 * per-op timing was switched on with fp_prefill_set_timing(task, 1) before that call.  Writes
 * min(n, ops of that call) entries to ms_out (host) and the count to *n_out.                     */
fp_status fp_prefill_set_timing(fp_prefill* task, int32_t on);
fp_status fp_prefill_op_times(fp_prefill* task, float* ms_out /*host*/, int32_t n,
                              int32_t* n_out /*host*/);

/* Mixture-of-experts models: copies layer `layer`'s routing decision -- expert ids [T, top_k]
 * (int32, most probable first) and renormalised weights [T, top_k] (fp32) -- to device buffers.
 * Valid once the cursor has passed that layer's gate operator (FP_ERR_STATE before); waits for
 * the stream.  Tests use it to hand the same decision to a reference when two experts are a
 * rounding error apart.                                                                          */
fp_status fp_prefill_moe_routing(fp_prefill* task, int32_t layer, int32_t* ids_out /*device*/,
                                 float* weights_out /*device*/);

/* Ends a task in any state except while an advance is running: returns its workspace to the
 * model's cache and frees the KV blocks the library allocated for it.  "Running" lasts until
 * fp_prefill_advance has RETURNED in its thread: after fp_preempt reports FP_PREEMPTED from
 * another thread, wait for that advance call to return before ending the task.                   */
void fp_prefill_end(fp_prefill* task);

/* Single-operator entry points used by the unit tests and the roofline measurement: each
 * launches exactly the kernel the prefill path uses for that operator on `hip_stream` and
 * returns without synchronising.  Pointers are device pointers; dtype is FP_DTYPE_*.
 *   fp_op_gemm     C[M,N] (+)= A[M,K] W[N,K]^T.  residual=0: C in the storage dtype is
 *                  overwritten; residual=1: C is fp32 and accumulated into (x += ...).
 *   fp_op_rmsnorm  out[T,d] (storage dtype) = rmsnorm(x[T,d] fp32) * gain[d]
 *   fp_op_silu_mul out[T,F] = silu(gu[:, :F]) * gu[:, F:]
 *   fp_op_gemm_swiglu  bf16 only: out[M,F] = silu(G) * U with [G | U] = A[M,K] W[2F,K]^T rounded
 *                  to bf16 (W rows: F gate rows, then F up rows) -- the gate_up projection with
 *                  the activation fused into its epilogue, the form the prefill path uses for
 *                  operators 6+7 when the problem fills the chip (the SwiGLU MLP of the operator
 *                  list in Section 5.1); same bits as fp_op_gemm followed by fp_op_silu_mul.
 *                  FP_ERR_INVALID for shapes the fused kernel does not take (K % 64, F % 8, fewer
 *                  than 96 output tiles of 256 x 128): callers then use the two-operator form.
 *   fp_op_gemm_ws  fp_op_gemm with a caller-provided device workspace (256-byte aligned): problems
 *                  with too few output tiles to fill the chip are then cut over K, the fp32 partial
 *                  sums go to the workspace and a second kernel adds them in a fixed order -- the
 *                  form the prefill path uses for the 128-1024-token requests of the evaluation
 *                  trace (Section 6.1, Table 1).  fp_op_gemm_workspace_bytes says how much such a
 *                  problem wants (0: it would not be cut); with less, or with fp_op_gemm, the
 *                  problem runs uncut.  Results of the cut and uncut forms differ by fp32 rounding
 *                  order only.
 * FP_ERR_INVALID on misaligned or non-positive sizes (K and N multiples of 8).                   */
fp_status fp_op_gemm(int32_t dtype, const void* a, const void* w, void* c, int64_t m, int64_t n,
                     int64_t k, int32_t residual, void* hip_stream);
fp_status fp_op_gemm_ws(int32_t dtype, const void* a, const void* w, void* c, int64_t m, int64_t n,
                        int64_t k, int32_t residual, void* workspace /*device*/,
                        int64_t workspace_bytes, void* hip_stream);
int64_t fp_op_gemm_workspace_bytes(int32_t dtype, int64_t m, int64_t n, int64_t k);

/* The short-request form of two operator pairs of the layer (the operators between the core
 * operators of Section 5.1; requests of 128-1024 tokens, Section 6.1): when a projection is cut
 * over K, the kernel that adds the partial sums also carries out the operator that follows, so
 * that operator launches nothing (its cursor position and boundary remain).  bf16 only.
 *   FP_TAIL_RMSNORM  residual = 1: c (fp32 [M,N]) += A W^T, then tail_out [M,N] (bf16) =
 *                    rmsnorm(updated row of c, eps) * gain[N]           (o_proj / down_proj + RMSNorm)
 *   FP_TAIL_SWIGLU   residual = 0, N = 2F, gate columns first: tail_out [M,F] (bf16) =
 *                    silu(bf16(gate)) * bf16(up); c is not written and may be NULL  (gate_up_proj + SiLU*up)
 * Same bits as fp_op_gemm_ws followed by fp_op_rmsnorm / fp_op_silu_mul.  FP_ERR_INVALID, with
 * nothing launched, when the problem would not be cut over K with this workspace (see
 * fp_op_gemm_workspace_bytes), N > 8192 for FP_TAIL_RMSNORM, or on the size errors of fp_op_gemm.   */
enum { FP_TAIL_RMSNORM = 1, FP_TAIL_SWIGLU = 2 };
fp_status fp_op_gemm_tail(int32_t dtype, const void* a, const void* w, void* c, int64_t m, int64_t n,
                          int64_t k, int32_t residual, void* workspace /*device*/, int64_t workspace_bytes,
                          int32_t tail, const void* gain /*device, FP_TAIL_RMSNORM*/,
                          void* tail_out /*device*/, float eps, void* hip_stream);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): fp_op_gemm_ws without a workspace argument.  The split-K partial sums go
 * to a static device array of FP_NOALLOC_SCRATCH_BYTES inside the library (each GPU the library
 * runs on holds its own copy until the process ends); the call allocates and frees nothing --
 * no hipMalloc, no hipFree, no allocating library routine.  Same kernels and the same bits as
 * fp_op_gemm_ws given fp_op_gemm_workspace_bytes of workspace.  The first call on a device looks
 * the array's address up once (hipGetSymbolAddress); make that call outside a capture.
 * FP_ERR_INVALID, with nothing launched, when the problem wants more scratch than the array holds
 * (fp_op_gemm_workspace_bytes(...) > FP_NOALLOC_SCRATCH_BYTES) or on the size errors of fp_op_gemm.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams or threads) race on it; the array keeps the previous call's contents between calls and
 * none of it needs to start at zero.                                                              */
#define FP_NOALLOC_SCRATCH_BYTES (32 * 1024 * 1024)
fp_status fp_op_gemm_noalloc(int32_t dtype, const void* a, const void* w, void* c, int64_t m,
                             int64_t n, int64_t k, int32_t residual, void* hip_stream);
fp_status fp_op_rmsnorm(int32_t dtype, const void* x_f32, const void* gain, void* out,
                        int64_t t, int64_t d, float eps, void* hip_stream);
fp_status fp_op_silu_mul(int32_t dtype, const void* gu, void* out, int64_t t, int64_t f,
                         void* hip_stream);
fp_status fp_op_gemm_swiglu(const void* a, const void* w_gate_up, void* out, int64_t m, int64_t f,
                            int64_t k, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Event-driven scheduler (Section 5.2): S-EDF priority (Eq. (3)), SLO-aware batching
 * (Algorithm 1) and the scheduling round of Algorithm 2.  Host-only bookkeeping: it decides which
 * commands (preempt / submit / resume) the caller should issue to the execution pool; it never
 * touches the GPU.  Times are seconds on any one monotonic clock of the caller's choosing.
 *
 *   fp_sched_create   token_budget = G of Algorithm 1.  ttft_coef[0..n_coef-1] (host): the
 *                     offline-fitted polynomial of Section 6.3, predicted TTFT in seconds of an
 *                     execution of n tokens = sum_i coef[i] * n^i.  policy: FP_SCHED_SEDF
 *                     (Eq. (3)), FP_SCHED_EDF (1/deadline: the chunked-prefill + EDF baseline of
 *                     Section 6.1) or FP_SCHED_FCFS (arrival order, never preempts).  batching != 0
 *                     enables Algorithm 1.
 *   fp_sched_arrive   a new request joins the waiting queue Q_w; deadline = arrival + ttft_slo.
 *   fp_sched_complete the running execution E (batch head `head_id` and every request batched
 *                     under it) has finished.  FP_ERR_STATE if head_id is not the running one.
 *   fp_sched_retire   a preempted execution turned out to be finished (fp_preempt returned
 *                     FP_DONE: the command raced with completion); it leaves Q_p.  FP_ERR_STATE if
 *                     `id` is not in the preempted queue.
 *   fp_sched_round    one iteration of Algorithm 2's loop at time `now` (call it after every
 *                     arrival or completion event).  On return *decision says what to do, in this
 *                     order: if preempt_id >= 0 preempt that execution (it moves to Q_p); then
 *                     action FP_SCHED_SUBMIT: start one execution for the n_batch requests
 *                     batch_ids[] (head first; they leave Q_w), or FP_SCHED_RESUME: resume
 *                     head_id (it leaves Q_p), or FP_SCHED_NONE.  The state already reflects the
 *                     decision when the call returns.  At most FP_SCHED_MAX_BATCH requests are
 *                     batched.
 *   fp_sched_predict  the polynomial's value for n tokens.
 * Readings of the paper: sgn(0) = +1; equal priorities are ordered by earlier arrival, then
 * smaller id; the running execution is not a batching candidate; Algorithm 1 scans all
 * candidates in priority order with the strict comparisons as printed; a preempted request's
 * estimate is the polynomial at its full token count.
 * Not thread-safe: one scheduler thread, as in the paper.                                       */
typedef struct fp_sched fp_sched;
enum { FP_SCHED_SEDF = 0, FP_SCHED_EDF = 1, FP_SCHED_FCFS = 2 };
enum { FP_SCHED_NONE = 0, FP_SCHED_SUBMIT = 1, FP_SCHED_RESUME = 2 };
enum { FP_SCHED_MAX_BATCH = 64 };
typedef struct {
  int64_t preempt_id;                      /* -1: nothing to preempt                            */
  int32_t action;                          /* FP_SCHED_NONE / _SUBMIT / _RESUME                 */
  int32_t n_batch;                         /* number of ids in batch_ids (SUBMIT only)          */
  int64_t head_id;                         /* the execution that runs next (-1 if NONE)         */
  int64_t batch_ids[FP_SCHED_MAX_BATCH];
} fp_sched_decision;

fp_status fp_sched_create(int64_t token_budget, const double* ttft_coef, int32_t n_coef,
                          int32_t policy, int32_t batching, fp_sched** out);
void fp_sched_destroy(fp_sched* sched);
fp_status fp_sched_arrive(fp_sched* sched, int64_t id, int64_t n_tokens, double arrival,
                          double ttft_slo);
fp_status fp_sched_complete(fp_sched* sched, int64_t head_id);
fp_status fp_sched_retire(fp_sched* sched, int64_t id);
fp_status fp_sched_round(fp_sched* sched, double now, fp_sched_decision* decision);
double fp_sched_predict(const fp_sched* sched, int64_t n_tokens);

/* Diagnostic for the roofline report: runs a register-only loop of the bf16 MFMA instruction the
 * GEMM kernel uses (16x16x32; random operands, two waves per SIMD on every CU) for about
 * `milliseconds` and writes the rate of the last launch, in TFLOP/s, to *tflops_out (host).  This
 * is what the matrix pipes sustain on the chip at hand at the clock it holds under that load.
 * Allocates and frees a small device buffer; synchronises `hip_stream`.                          */
fp_status fp_diag_mfma_ceiling(int32_t milliseconds, void* hip_stream, double* tflops_out /*host*/);

const char* fp_last_error(void);
const char* fp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FLOWPREFILL_H */
