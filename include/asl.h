/*
 * libasl -- the per-layer token-importance pass of Adaptive Selection Layer (ASL) token pruning
 * (arXiv 2601.07667), as hand-written HIP kernels for gfx950 (MI355X) behind a C ABI.
 *
 * The calls follow the problem statement of the paper's Alg. 1 (GetRanks: Q, K, V, layer_idx,
 * window W, pooling kernel S, KV budget, rank cache) and Alg. 2 (SelectTokens: layer_idx,
 * KV budget, W, L_min, L_obs, tau, rank cache, init_var).
 *
 * Conventions for every entry point
 *  - Pointers named q_obs, k, v, lse*, u, p_head, s_all, scores, rank*, idx*, *_ptrs, state, out
 *    are DEVICE pointers owned by the caller.  `params` and `ctx` are HOST pointers.  The library
 *    owns only the workspace inside asl_ctx (allocated by asl_create; no allocation afterwards).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work
 *    and return; they never synchronise.  Calls sharing a ctx share its workspace: calls of the
 *    same family must not overlap.  The families use disjoint workspace regions, so one call each
 *    of {asl_score_layer, asl_pool}, {asl_rank, asl_rankvar, asl_rank_stat}, {asl_select_topk} and
 *    {asl_gather_kv} may run concurrently on different streams of the ctx's device (e.g. ranking
 *    and top-k of the same scores side by side).
 *  - Return value: ASL_OK or a negative asl_status.  Arguments are validated on the host before
 *    any launch; asl_last_error() gives a message for the last failure on that ctx.
 *  - Notation: Hq query heads, Hk KV heads, G = Hq/Hk, d head dim, N sequence length,
 *    W window, T = N - W past tokens, S pooling kernel, k = min(budget, N) - W.
 *  - Tie rule everywhere: among equal scores the lower token index ranks first / is kept.
 *    NaN scores give an unspecified (but memory-safe) order.
 */
#ifndef ASL_H_
#define ASL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct asl_ctx asl_ctx;

typedef enum {
  ASL_OK = 0,
  ASL_EINVAL = -1,        /* bad argument (null pointer, shape, budget <= W, even S, ...) */
  ASL_ENOMEM = -2,        /* workspace allocation failed / problem larger than the ctx was made for */
  ASL_EHIP = -3,          /* a HIP runtime call failed */
  ASL_EUNSUPPORTED = -4   /* valid but not implemented (dtype, misaligned strides, sizes past limits) */
} asl_status;

typedef enum { ASL_BF16 = 0, ASL_F32 = 1 } asl_dtype;

/* Problem statement (Alg. 1 inputs; Alg. 2 shares budget and window). */
typedef struct {
  int32_t n_q_heads;      /* Hq                                            */
  int32_t n_kv_heads;     /* Hk, Hq % Hk == 0                              */
  int32_t head_dim;       /* d                                             */
  int32_t seq_len;        /* N = N_q (keys == queries during prefill)      */
  int32_t window;         /* W, 1 <= W < N                                 */
  int32_t pool_kernel;    /* S, odd, >= 1                                  */
  int32_t budget;         /* KV budget, > W;  k = min(budget, N) - W       */
  int32_t dtype;          /* asl_dtype of q_obs, k, v                      */
  int64_t k_stride_head;  /* element strides of K [Hk, N, d]; d contiguous */
  int64_t k_stride_tok;
  int64_t v_stride_head;  /* same for V                                    */
  int64_t v_stride_tok;
  float scale;            /* logit scale; <= 0 means 1/sqrt(d)             */
  int32_t flags;          /* ASL_FLAG_* bits, normally 0                   */
} asl_params;

/* Score with the plain fp32-FMA kernels even where the MFMA kernels apply (an on-GPU cross-check). */
#define ASL_FLAG_GENERIC_SCORE 1
/* asl_layer_step only: run top-k + compaction on the context's second stream and return without
 * waiting for it (see asl_layer_step and asl_join). */
#define ASL_FLAG_DEFER_JOIN 2

/* Cross-layer state of Alg. 2 (init_var and the fill level of the rank cache).  24-byte device
 * struct owned by the caller; all-zero bytes = fresh sequence.  The library updates it. */
typedef struct {
  double init_var;        /* var_top at the first evaluated layer (Sec. 4.1, relative variance) */
  int32_t init_set;       /* 0 until init_var has been set                                      */
  int32_t n_valid_rows;   /* filled rows of the rank ring, <= L_obs                             */
  int32_t last_layer;     /* layer index of the newest row (valid when n_valid_rows > 0)        */
  int32_t reserved;
} asl_state;

/* Result of the statistic (Alg. 2 steps 4-10), written to device memory. */
typedef struct {
  double var_top;         /* mean over the union of the per-token rank variance               */
  double rel_var;         /* var_top / init_var (IEEE: NaN or inf when init_var == 0)         */
  uint64_t numerator;     /* sum over the union of  n * sum R^2 - (sum R)^2  (exact)          */
  int32_t union_size;     /* |top(L)|                                                         */
  int32_t n_rows;         /* rank rows used (n)                                               */
  int32_t evaluated;      /* 0 when layer_idx < L_min or fewer than two rows were available   */
  int32_t selected;       /* 1 iff evaluated and rel_var < tau                                */
} asl_stat;

/* Create a context on `device` with a workspace large enough for any call with
 * seq_len <= max_seq_len, n_kv_heads <= max_kv_heads and Hq*W <= max_q_rows.
 * Errors: ASL_EINVAL (null/negative), ASL_EHIP, ASL_ENOMEM. */
asl_status asl_create(asl_ctx** out, int device, int32_t max_seq_len, int32_t max_kv_heads,
                      int32_t max_q_rows);
asl_status asl_destroy(asl_ctx* ctx);
/* Message of the last failure on ctx (ctx-owned string, valid until the next call on ctx). */
const char* asl_last_error(const asl_ctx* ctx);
/* Bytes of device workspace asl_create would allocate for these limits. */
size_t asl_workspace_bytes(int32_t max_seq_len, int32_t max_kv_heads, int32_t max_q_rows);

/* Alg. 1 steps 5-8 and the Sec. 4.1 "scores" equation.
 *   q_obs  [Hq, W, d] contiguous: the last W query rows of every head.
 *   k      [Hk, N, d] with the strides in params (16-byte aligned rows).
 *   lse    [Hq, W] f32 or NULL: natural-log-sum-exp of each window row's masked, scaled logits
 *          (what the layer's attention kernel produces).  When given, K is streamed once;
 *          when NULL the row normalisers are computed here with an extra pass over K.
 *   p_head [Hk, T] f32 out: pooled, group-summed scores P.
 *   s_all  [T]     f32 out: sum of P over the KV heads (the vector that is ranked).
 * Logits are scaled q.k with the causal mask on the last W x W block; softmax over all N keys;
 * column sums over the W rows and the G heads of a group, past columns only; AvgPool1D(S,
 * stride 1, zero pad floor(S/2), divisor S).  bf16 inputs with d in {64, 128} and G*W <= 512 use
 * bf16 MFMA with fp32 accumulation; other shapes take plain fp32-FMA kernels, which are meant for
 * small problems (ASL_EUNSUPPORTED when Hq*W*N*d exceeds 6e11).  Softmax and sums are fp32 and
 * deterministic (fixed reduction order, no float atomics). */
asl_status asl_score_layer(asl_ctx* ctx, const asl_params* params, const void* q_obs,
                           const void* k, const float* lse, float* p_head, float* s_all,
                           void* stream);

/* The normaliser of Alg. 1 step 5's softmax on its own: lse_out[h, i] = natural-log-sum-exp over
 * all N keys of window row i of query head h's scaled, causally masked logits (the first of
 * asl_score_layer's two passes over K; fp32, deterministic).
 *   q_obs, k as in asl_score_layer;  lse_out [Hq, W] f32 out.
 * Handing lse_out back to asl_score_layer as `lse` gives the scores of the self-contained call up
 * to the fp32 rounding of the logarithm's change of base (relative differences of a few 1e-6).
 * For callers that score one K against the same window more than once, and as the reference for
 * an attention kernel that produces these values itself. */
asl_status asl_window_lse(asl_ctx* ctx, const asl_params* params, const void* q_obs, const void* k,
                          float* lse_out, void* stream);

/* Alg. 1 step 7 on its own: zero-padded moving average, kernel S (odd), stride 1, along T.
 *   u [rows, T] f32 in; p_out [rows, T] f32 out; s_out [T] f32 out or NULL (sum of the pooled rows). */
asl_status asl_pool(asl_ctx* ctx, const float* u, int32_t rows, int32_t T, int32_t S,
                    float* p_out, float* s_out, void* stream);

/* Alg. 1 step 11, RankDesc: rank_out[t] = #{t': s[t'] > s[t]} + #{t' < t: s[t'] == s[t]}.
 *   s [T] f32 in; rank_out [T] int32 out (a permutation of 0..T-1). */
asl_status asl_rank(asl_ctx* ctx, const float* s, int32_t T, int32_t* rank_out, void* stream);

/* asl_rank for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  It needs no context: the sort's scratch buffers
 * live in a static device array inside the library (about 4.1 MiB on every GPU the library runs
 * on, held until the process ends), so the call allocates nothing, on the device or through any
 * library.  Same result as asl_rank, bit for bit.
 *   s [T] f32 in, rank_out [T] int32 out: device pointers on the CURRENT device; T <=
 *   ASL_RANK_STATIC_MAX_T, larger T returns ASL_ENOMEM (message from asl_static_last_error, a
 *   thread-local string).  The work is enqueued on `stream`.
 * All calls on one GPU share that GPU's scratch array: calls that overlap on one GPU (different
 * streams or threads) race; serialise them.  The array's device address is looked up on the first
 * call per device (or by asl_create on that device); make that first call outside stream capture. */
#define ASL_RANK_STATIC_MAX_T 262144
asl_status asl_rank_static(const float* s, int32_t T, int32_t* rank_out, void* stream);
const char* asl_static_last_error(void);

/* Alg. 2 steps 4-10 on a rank ring that already holds this layer's row.
 *   rank_ring [l_obs, T] int32; the rows in use are those of layers
 *   layer_idx - state->n_valid_rows + 1 .. layer_idx, layer l living in row l % l_obs.
 *   Union = tokens with rank < k in any used row; var_top = mean population variance of their
 *   ranks; first evaluation sets state->init_var; selected = (var_top / init_var < tau).
 *   With layer_idx < l_min or fewer than two rows: out->evaluated = 0 and nothing else changes.
 *   On selection the ring is released (state->n_valid_rows = 0).
 *   `out` may be device memory or page-locked host memory that the device can address (the
 *   kernel then writes the record straight to the host; read it after synchronising the stream).
 * Limits: n^2 * T^3 / 4 must fit in 64 bits (ASL_EUNSUPPORTED otherwise). */
asl_status asl_rankvar(asl_ctx* ctx, const int32_t* rank_ring, int32_t l_obs, int32_t T,
                       int32_t layer_idx, int32_t l_min, int32_t k, double tau,
                       asl_state* state, asl_stat* out, void* stream);

/* Alg. 1 step 11 + Alg. 2: rank s_all into ring row layer_idx % l_obs, then the statistic as
 * asl_rankvar with k = min(budget - W, T).  The host reads *out after synchronising the stream.
 * The new row continues the rows already held iff layer_idx == state->last_layer + 1, or
 * layer_idx == state->last_layer + 1 - l_obs (the replay of a captured sequence of l_obs layers,
 * which overwrites the same ring rows in the same order); any other layer index restarts the ring
 * from this one row.  Zero the state to start a new sequence. */
asl_status asl_rank_stat(asl_ctx* ctx, const asl_params* params, const float* s_all,
                         int32_t layer_idx, int32_t l_min, int32_t l_obs, double tau,
                         int32_t* rank_ring, asl_state* state, asl_stat* out, void* stream);

/* Alg. 1 steps 9-10 (rows = Hk on p_head) or Alg. 2 steps 11-12 (rows = 1 on s_all):
 *   scores  [rows, T] f32 in.
 *   idx_out [rows, k + W] int32 out: the k highest-scoring past tokens of each row in ascending
 *   token order, followed by the window tokens T .. T+W-1. */
asl_status asl_select_topk(asl_ctx* ctx, const asl_params* params, const float* scores,
                           int32_t rows, int32_t* idx_out, void* stream);

/* Alg. 1 step 12: K[I], V[I].
 *   idx [idx_rows, n_idx] int32, idx_rows in {1, Hk} (one shared row or one per KV head),
 *   every entry in [0, N) (caller's contract; asl_select_topk output satisfies it).
 *   k_out, v_out [Hk, n_idx, d] dense, same dtype as k, v.  v / v_out may both be NULL. */
asl_status asl_gather_kv(asl_ctx* ctx, const asl_params* params, const void* k, const void* v,
                         const int32_t* idx, int32_t idx_rows, int32_t n_idx, void* k_out,
                         void* v_out, void* stream);

/* Alg. 1 step 12 for many layers in one launch (Sec. 4.2 "Decoding": every layer before the
 * selection layer keeps a compressed KV cache, each layer's cache being its own allocation).
 *   k_ptrs, v_ptrs         DEVICE arrays of n_layers device pointers, layer l's K (V) [Hk, N, d]
 *                          with the strides in params (the same for every layer); 16-byte aligned.
 *   idx                    [n_layers, idx_rows, n_idx] int32, idx_rows in {1, Hk}, entries in [0, N).
 *   k_out_ptrs, v_out_ptrs DEVICE arrays of n_layers device pointers to dense [Hk, n_idx, d] outputs.
 * v_ptrs / v_out_ptrs may both be NULL.  The pointer arrays are read by the kernel only: nothing
 * is copied or allocated by the call (capturable in a HIP graph).  n_layers <= 16384. */
asl_status asl_gather_kv_layers(asl_ctx* ctx, const asl_params* params, const void* const* k_ptrs,
                                const void* const* v_ptrs, const int32_t* idx, int32_t idx_rows,
                                int32_t n_idx, int32_t n_layers, void* const* k_out_ptrs,
                                void* const* v_out_ptrs, void* stream);

/* Token propagation at the selection layer (Sec. 4.2 "Prefilling": only the selected tokens go on
 * to the deeper layers; Alg. 2's select_idx applied to the hidden states): dst[i,:] = src[idx[i],:].
 *   src rows of row_bytes bytes, src_row_stride_bytes apart; idx [n_idx] int32, entries in range
 *   (caller's contract); dst [n_idx, row_bytes] dense.  16-byte aligned rows, pointers, stride. */
asl_status asl_gather_rows(asl_ctx* ctx, const void* src, int64_t src_row_stride_bytes, int32_t row_bytes,
                           const int32_t* idx, int32_t n_idx, void* dst, void* stream);

/* One layer of Alg. 1 + Alg. 2 in a single call: asl_score_layer, asl_rank_stat, asl_select_topk
 * (Hk per-head rows + the all-head row) and asl_gather_kv (per-head rows), with the same results as
 * the single calls.  After the scoring, ranking and top-k + compaction are independent; the call
 * runs them side by side in four launches on `stream`, launch i carrying pass i of the ranking sort
 * in some workgroups and stage i of the top-k / compaction in the others, followed by the statistic.
 *   scores  [Hk+1, T] f32 out: rows 0..Hk-1 = P (per KV head), row Hk = s (all heads).
 *   idx_out [Hk+1, k+W] int32 out: rows 0..Hk-1 = Alg. 1's per-head I, row Hk = Alg. 2's select_idx
 *           (to be used only when out->selected is set).
 *   k_out, v_out [Hk, k+W, d] out: K[I], V[I] per head; pass k_out = NULL to skip the compaction.
 * The ctx must have been created with max_kv_heads >= Hk + 1.  Other arguments as in the single
 * calls.  Not to be overlapped with any other call on the same ctx.
 * With ASL_FLAG_DEFER_JOIN in params->flags (and for sizes the four launches do not take) ranking +
 * statistic run on `stream` and top-k + compaction on a second stream owned by the ctx.  With the
 * flag the call returns as soon as ranking + statistic are queued; idx_out, k_out and v_out are then
 * complete only after asl_join.  The next asl_layer_step on the ctx joins by itself before it
 * overwrites `scores` (so in a layer loop the top-k + compaction of one layer overlaps the scoring
 * of the next); until the join, `scores`, k, v and the three outputs of the deferred call must not
 * be written or freed, and no other entry point may be used on the ctx.  Call asl_join before
 * reading the outputs and before ending a stream capture (asl_destroy waits for the second stream
 * by itself). */
asl_status asl_layer_step(asl_ctx* ctx, const asl_params* params, const void* q_obs, const void* k,
                          const void* v, const float* lse, int32_t layer_idx, int32_t l_min,
                          int32_t l_obs, double tau, float* scores, int32_t* rank_ring,
                          asl_state* state, asl_stat* out, int32_t* idx_out, void* k_out, void* v_out,
                          void* stream);

/* Makes `stream` wait for the second-stream work of the last asl_layer_step issued with
 * ASL_FLAG_DEFER_JOIN (no-op if there is none).  Sec. 4.2 "Prefilling": only the decision is needed
 * before the next layer starts; the compacted KV of a layer is needed at decoding time. */
asl_status asl_join(asl_ctx* ctx, void* stream);

/* Health check (not a step of the paper's method).  The workgroups of a ranking or statistic
 * launch hand counts to each other inside the launch and wait for them with a bounded number
 * of polls; a workgroup whose wait runs out raises a fault word in the workspace and writes no
 * results (every wave still exits).  This call waits for the device to go idle, returns the word
 * in *fault_out (0 = no wait ever ran out) and clears it.  Results of calls issued since the last
 * check are valid iff it reads 0.  Synchronises: not for the hot loop. */
asl_status asl_device_fault(asl_ctx* ctx, int32_t* fault_out);

/* Measurement aid (not a step of the paper's method; for callers that time the kernels of the
 * calls above).  Kernel ids: 0 score row statistics (pass 1), 1 its combine, 2 score column sums
 * (pass 2), 3 pool, 4 sort histogram, 5 sort scatter, 6 rank-variance finalisation (or the
 * below-L_min skip), 7 rank-variance partial sums, 8 select histogram, 9 select write, 10 gather,
 * 11 plain-FMA score kernels, 12 the four launches of asl_layer_step that carry sort passes and
 * top-k / compaction stages together.  (Each sort pass is one kernel, recorded under 5, id 4 is unused;
 * 8 covers the top-k's bound and filter kernels, 9 its finishing kernel; the statistic is one
 * kernel, 7; 6 is the below-L_min skip.)
 * asl_profile_enable: launches whose id bit is set in kernel_mask carry a HIP event pair that the
 *   runtime stamps with the kernel's start and end on the device (the call's stream; not under
 *   stream capture), up to max_records launches (further ones run unrecorded); mask 0 turns
 *   it off and frees the events.  Allocates host memory and events: not for the hot loop.
 * asl_profile_collect: waits for the recorded events of kernel_id and returns their summed
 *   duration in milliseconds and their number; kernel_id -1 clears the records instead. */
asl_status asl_profile_enable(asl_ctx* ctx, uint32_t kernel_mask, int32_t max_records);
asl_status asl_profile_collect(asl_ctx* ctx, int32_t kernel_id, double* total_ms, int32_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* ASL_H_ */
