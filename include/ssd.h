/* libssd - the target-model verification step of Speech Speculative Decoding (SSD) on one MI355X.
 *
 * Notation follows the paper with one renaming to avoid its p/q clash with the usual convention:
 *   pt = the target model's distribution (the paper's q^s), pd = the draft model's (the paper's p^d),
 *   K  = number of draft tokens per cycle (the paper's L_d), beta = tolerance factor.
 *
 * One SSD cycle (Alg. 1): the draft model proposes x_1..x_K autoregressively with full rows pd_1..pd_K
 * (Eq. 2-3, ssd_draft_step); the target model scores [pending, x_1..x_K] in one causal pass giving
 * pt_1..pt_{K+1} (Eq. 4); x_i is accepted while r_i < min(1, pt_i(x_i)/pd_i(x_i)) + beta (Eq. 5); at the
 * first rejection a token is drawn from normalize(max(0, pt_i - pd_i)) (Eq. 6), and if all K are accepted
 * a bonus token is drawn from pt_{K+1}; the sequence grows by n_accepted + 1 tokens (ssd_verify).
 * The KV cache, its paging and the rollback of rejected positions are this library's mechanics; the
 * paper speaks only of a growing prefix.
 *
 * Conventions for every call
 *   - Pointers named dev_* are DEVICE pointers owned by the caller; everything else is host memory.
 *     The library allocates no device memory: weights, KV pool and workspaces are caller buffers that
 *     the handles borrow until they are destroyed.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work and
 *     return; outputs are valid after the stream is synchronised.  Calls on one handle must be issued on
 *     one stream (or be externally ordered).
 *   - Return value: SSD_OK (0) or a negative error code; ssd_last_error() gives a message for the last
 *     failure on the calling thread.  Arguments are validated on the host before anything is launched;
 *     nothing throws or aborts across this boundary.
 *   - Sequence state (length, pending token(s), block table) lives on the device so that cycles can be
 *     chained without a host round trip.  The host keeps an upper bound of every length and synchronises
 *     the stream only when that bound would exhaust the pool, or when asked for the state.
 */
#ifndef SSD_H
#define SSD_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

#define SSD_OK      0
#define SSD_EINVAL (-1)   /* bad argument (null, out of range, shape mismatch, state mismatch) */
#define SSD_ENOMEM (-2)   /* KV pool or a caller buffer too small for the request */
#define SSD_EHIP   (-3)   /* a HIP call failed */
#define SSD_ENOSUP (-4)   /* shape not supported by the kernels */

#define SSD_DTYPE_FP32 0
#define SSD_DTYPE_BF16 1
#define SSD_MAX_K      15  /* draft tokens per cycle */
#define SSD_DRAFT_SLOT0 (SSD_MAX_K + 1)  /* first random-counter slot of the draft's draws (see ssd_sample_config) */

typedef struct ssd_model ssd_model;   /* a decoder: shape + device weights in the layout the kernels stream */
typedef struct ssd_kv    ssd_kv;      /* a paged KV cache + per-sequence state + activation workspace    */

/* Decoder shape.  Pre-norm blocks: RMSNorm, QKV projection (+bias), rotary embedding on the pairs
 * (i, i+head_dim/2), grouped-query attention scaled by 1/sqrt(head_dim), output projection, RMSNorm,
 * SwiGLU feed-forward; final RMSNorm and an untied output head over `vocab` speech tokens.  `n_embed`
 * >= vocab rows of input embedding (rows >= vocab are the text ids of the prompt, Sec. 2.1). */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, n_embed;
  int32_t dtype;        /* SSD_DTYPE_*: storage type of matrices, embeddings and the KV cache */
  int32_t qkv_bias;     /* 0/1 */
  float   rope_base, rms_eps;
} ssd_model_config;

/* Sampling of one model.  pt and pd are post-warp distributions: logits / temperature, then top-k
 * (ties at the k-th value: lower index survives), then softmax; greedy != 0 replaces the row by a one-hot
 * at the arg-max (lowest index).  Uniforms come from Philox-4x32-10 keyed by `seed` with counter
 * (slot, sequence, step_lo, step_hi).  A verification uses slots 0..K-1 for r_1..r_K and slot K for the emitted
 * token; draft step i of the same cycle draws x_{i+1} with slot SSD_DRAFT_SLOT0 + i.  Eq. 5 compares r_i with a
 * ratio that depends on x_i, and Alg. 1 draws r_i afresh, so the two must be independent: with the slot ranges
 * disjoint they are even when draft and target are given the same seed. */
typedef struct {
  float    beta;          /* tolerance factor of Eq. 5, >= 0 (used by ssd_verify only) */
  float    temperature;   /* > 0 */
  int32_t  top_k;         /* 0 = off */
  int32_t  greedy;        /* 0/1 */
  uint64_t seed;
} ssd_sample_config;

/* ---- model ------------------------------------------------------------------------------------------
 * dev_weights: array (host) of 3 + 8*n_layers device pointers in canonical layout, linear weights
 * row-major [out_features, in_features]:
 *   [0] embed [n_embed, d]   [1] final_norm gain [d] fp32   [2] head [vocab, d]
 *   per layer l at 3+8l: ln1 gain [d] fp32, wqkv [(nq+2nkv)*hd, d] (query heads, key heads, value heads),
 *   bqkv [(nq+2nkv)*hd] fp32 (NULL if !qkv_bias), wo [d, nq*hd], ln2 gain [d] fp32, wgate [ffn, d],
 *   wup [ffn, d], wdown [d, ffn].   Matrices/embeddings have the config's dtype.
 * They are read only by the work this call enqueues (it repacks them into dev_model_ws, which must hold
 * ssd_model_workspace_bytes() and stay alive as long as the model).  `max_positions` bounds every
 * sequence length + rows (size of the rotary table).  Requirements (else SSD_ENOSUP): head_dim in
 * {32,64,128}; n_q_heads % n_kv_heads == 0; for bf16 d_model, n_q_heads*head_dim and d_ffn multiples of
 * 32; vocab <= 16384. */
size_t ssd_model_workspace_bytes(const ssd_model_config* cfg, int max_positions);
int    ssd_model_create(const ssd_model_config* cfg, const void* const* dev_weights, int n_weights,
                        int max_positions, void* dev_model_ws, size_t ws_bytes, void* stream, ssd_model** out);
int    ssd_model_destroy(ssd_model* m);

/* ---- KV cache + sequence state ----------------------------------------------------------------------
 * Pool layout (dtype elements): keys [layer][0][block][kv_head][token_in_block][head_dim], stored after the
 * rotary embedding; values [layer][1][block][kv_head][head_dim][token_in_block] (token-minor, the order the
 * matrix-core attention reads them in).  The pool must hold finite values (e.g. zeros) when handed over.  `max_rows` bounds the rows of one forward per sequence (K+1 for verify, the
 * chunk of a prefill); max_seqs*max_rows <= 1024.  `pending_cap` is 1 for a target cache and 2 for a draft
 * cache (a draft may owe two tokens after a fully accepted cycle).  Blocks are handed out lowest id first;
 * see ssd_kv_state for the exact bookkeeping.  dev_ws must hold ssd_kv_workspace_bytes(). */
size_t ssd_kv_pool_bytes(const ssd_model* m, int n_blocks, int block_tokens);
size_t ssd_kv_workspace_bytes(const ssd_model* m, int max_seqs, int max_rows, int n_blocks, int max_blocks_per_seq);
int    ssd_kv_create(const ssd_model* m, int max_seqs, int max_rows, int n_blocks, int block_tokens,
                     int max_blocks_per_seq, int pending_cap, void* dev_pool, size_t pool_bytes,
                     void* dev_ws, size_t ws_bytes, void* stream, ssd_kv** out);
int    ssd_kv_destroy(ssd_kv* kv);

/* Reset sequence `seq`, run tokens[0..n-2] through the model into its cache (length = n-1) and make
 * tokens[n-1] the pending token: the "prompt" T_in of Alg. 1.  n >= 1. */
int ssd_prefill(ssd_model* m, ssd_kv* kv, int seq, const int32_t* dev_tokens, int n, void* stream);

/* ---- the three calls of the hot path ------------------------------------------------------------------
 * ssd_draft_step (Eq. 2-3): for sequences 0..n_seqs-1 of the draft cache feed the pending token(s), give the
 * warped distribution pd (full fp32 row, written to dev_probs_out + b*probs_stride) and a token drawn
 * from it with uniform slot SSD_DRAFT_SLOT0 + draft_idx (written to dev_token_out[b*token_stride]); the token becomes the
 * new pending token and the length grows by the rows fed.  Strides are in elements. */
int ssd_draft_step(ssd_model* draft, ssd_kv* kv_d, int n_seqs, const ssd_sample_config* cfg,
                   uint64_t step_ctr, int draft_idx, int32_t* dev_token_out, int token_stride,
                   float* dev_probs_out, size_t probs_stride, void* stream);

/* ssd_verify (Eq. 4-6, Alg. 1 loop body after drafting) for sequences 0..n_seqs-1 of the target cache.
 *   prefix_len      host array [n_seqs] or NULL.  When given, each entry must equal the cached length of
 *                   the sequence (forces a stream synchronisation to check; SSD_EINVAL on mismatch).
 *   dev_draft_tokens [n_seqs, K] int32, dev_draft_probs [n_seqs, K, V] fp32 row-major (both may be NULL
 *                   when K == 0, which is a plain autoregressive step).
 *   step_ctr        the cycle index used in the random counter.
 *   dev_n_accepted  [n_seqs] int32 out: number of accepted draft tokens n in 0..K.
 *   dev_next_token  [n_seqs] int32 out: the resampled (n < K) or bonus (n == K) token.
 *   dev_target_probs_opt [n_seqs, K+1, V] fp32 out or NULL; dev_logits_opt likewise (pre-warp logits).
 * On completion each sequence's length is len + 1 + n, its pending token is next_token, the keys/values of
 * the rejected positions are dead (overwritten by the next call) and blocks wholly past the new length
 * are back on the free stack.  SSD_ENOMEM if the pool cannot hold K+1 more positions per sequence. */
int ssd_verify(ssd_model* target, ssd_kv* kv, int n_seqs, const int32_t* prefix_len,
               const int32_t* dev_draft_tokens, const float* dev_draft_probs, int K,
               const ssd_sample_config* cfg, uint64_t step_ctr,
               int32_t* dev_n_accepted, int32_t* dev_next_token,
               float* dev_target_probs_opt, float* dev_logits_opt, void* stream);

/* ssd_verify_noalloc: ssd_verify for callers that cannot allocate device memory at all or that forbid the library to
 * - code under HIP graph capture, tight serving loops, harnesses without hipMalloc.  Same work, same results and
 * same state changes as ssd_verify(target, kv, n_seqs, NULL, ..., NULL, NULL, stream); the difference is where the
 * call's staging lives: the logits rows, the probability rows and the commit's arrival counter are kept in a
 * static device array inside the library (SSD_NOALLOC_MAX_ELEMS floats each for logits and probabilities, about
 * 2 MiB in all, held by every GPU the library runs on until the process ends) instead of in the cache's workspace.
 * The call allocates and frees nothing, on the device or through any library.  n_seqs * (K+1) * vocab beyond
 * SSD_NOALLOC_MAX_ELEMS is refused with SSD_ENOMEM before anything is launched.  Every call on one GPU shares
 * that GPU's array: calls that overlap on one GPU (two streams, two threads) race; calls in stream order do not,
 * and what a call needs zeroed it zeroes itself. */
#define SSD_NOALLOC_MAX_ELEMS (1u << 18)
int ssd_verify_noalloc(ssd_model* target, ssd_kv* kv, int n_seqs, const int32_t* dev_draft_tokens,
                       const float* dev_draft_probs, int K, const ssd_sample_config* cfg, uint64_t step_ctr,
                       int32_t* dev_n_accepted, int32_t* dev_next_token, void* stream);

/* ssd_kv_rollback: truncate sequence `seq` to `new_len` cached positions (<= its current length), free the
 * blocks wholly past it and set the single pending token.  Used for the draft cache after a rejection.
 * The length lives on the device and the call does not wait for it: a new_len beyond the host's upper bound of the
 * length is refused at once (SSD_EINVAL); one between the device's length and that bound is refused by the kernel -
 * the sequence stays as it was - and the NEXT call on this cache returns SSD_EINVAL (see ssd_kv_clear_error). */
int ssd_kv_rollback(ssd_kv* kv, int seq, int new_len, int pending_token, void* stream);

/* Device-side form for the draft cache after a verify of K >= 1 drafts, no host round trip: for each
 * sequence, n < K: truncate to the target's new length and pend next_token; n == K: keep the length and pend
 * [x_K, next_token] (x_K was sampled but never fed to the draft). */
int ssd_kv_follow(ssd_kv* kv_d, int n_seqs, int K, const int32_t* dev_n_accepted,
                  const int32_t* dev_next_token, const int32_t* dev_draft_tokens, void* stream);

/* ---- one SSD cycle as a replayable graph (Alg. 1 loop body) ---------------------------------------------------
 * K draft steps (Eq. 2-3), the verification (Eq. 4-6) and the draft cache following the decision, captured once as
 * a HIP graph and replayed by ssd_cycle_launch: nothing a replay needs is a kernel argument that changes from cycle
 * to cycle (the cycle index of the random counter and the launch numbers of the forward kernels are read from
 * device memory and advanced by the cycle's own kernels).  The caller's buffers (dev_draft_tokens [n_seqs,K],
 * dev_draft_probs [n_seqs,K,V], dev_n_accepted [n_seqs], dev_next_token [n_seqs]) are rewritten by every replay and
 * must outlive the handle.  The cycle index starts at first_step.  Launch shapes are captured for lengths up to 256
 * positions beyond the current ones; ssd_cycle_launch captures again (synchronising the stream) when the host's
 * bound of a length outgrows that, so a replay never runs with a stale shape.  Both caches must run the barrier-free
 * forward kernel (bf16 storage, head_dim 64, at most 16 rows per launch), else SSD_ENOSUP.  `stream` of
 * ssd_cycle_launch must not be the default (NULL) stream, which HIP cannot capture (SSD_EINVAL).  Between replays
 * the caches may be used through the other calls as well, on the same stream. */
typedef struct ssd_cycle ssd_cycle;
int ssd_cycle_create(ssd_model* target, ssd_kv* kv, ssd_model* draft, ssd_kv* kv_d, int n_seqs, int K,
                     const ssd_sample_config* cfg, const ssd_sample_config* dcfg, int32_t* dev_draft_tokens,
                     float* dev_draft_probs, int32_t* dev_n_accepted, int32_t* dev_next_token, uint64_t first_step,
                     void* stream, ssd_cycle** out);
int ssd_cycle_launch(ssd_cycle* c, void* stream);
int ssd_cycle_captures(const ssd_cycle* c);     /* how many times the graph has been captured so far */
int ssd_cycle_destroy(ssd_cycle* c);

/* ---- the acceptance step alone (Eq. 5-6), for decision parity with given probabilities and uniforms ----
 * dev_pt [B, K+1, V], dev_pd [B, K, V], dev_tokens [B, K], dev_uniforms [B, K+1] (r_1..r_K then the
 * sampling uniform; values k * 2^-24).  Outputs [B]: n accepted, emitted token, flag (1 = the residual had
 * zero mass and the token was drawn from pt_i instead). */
int ssd_verify_from_probs(const float* dev_pt, const float* dev_pd, const int32_t* dev_tokens,
                          const float* dev_uniforms, int B, int K, int V, float beta,
                          int32_t* dev_n_accepted, int32_t* dev_next_token, int32_t* dev_flags, void* stream);

/* Warp + softmax alone (temperature, top-k, greedy as in ssd_sample_config): dev_logits [rows, V] ->
 * dev_probs [rows, V]. */
int ssd_warp_probs(const float* dev_logits, int rows, int V, const ssd_sample_config* cfg,
                   float* dev_probs, void* stream);

/* ---- introspection (synchronises `stream`) -------------------------------------------------------------
 * Bookkeeping contract: a forward that writes R rows makes each sequence (ascending) own
 * ceil((len+R)/block_tokens) blocks, popping the free stack; a commit or rollback to new_len pushes back the
 * blocks with table index >= ceil(new_len/block_tokens), highest index first.  `free_stack` is returned bottom
 * first (the last entry is popped next).  dev_error_flag: bit 0 = the device allocator ran out of blocks, bit 1 = a
 * persistent forward kernel gave up (a bounded wait timed out, or the launch numbering ran out), bit 2 = a rollback
 * beyond the cached length was refused.  Any output pointer may be NULL. */
int ssd_kv_state(ssd_kv* kv, int seq, void* stream, int32_t* len, int32_t* n_pending, int32_t pending[2],
                 int32_t* n_owned, int32_t* block_table, int block_table_cap);
int ssd_kv_free_stack(ssd_kv* kv, void* stream, int32_t* free_stack, int cap, int32_t* n_free, int32_t* dev_error_flag);

/* ---- errors raised on the device ------------------------------------------------------------------------------
 * Every wait inside the persistent forward kernels is bounded.  When one gives up, every workgroup leaves, the
 * kernel that follows the forward commits NOTHING (lengths, pending tokens and blocks stay as they were; the
 * outputs of that call are void) and the error reaches the host through a host-mapped word: the next call on that
 * cache - and every one after it - returns SSD_EHIP until ssd_kv_clear_error.  The same path reports a refused
 * rollback (SSD_EINVAL), pool exhaustion found by the device allocator (SSD_ENOMEM), and an exhausted launch
 * numbering (SSD_EHIP; the library renumbers by itself long before that unless its calls are replayed from a graph
 * it did not capture).  ssd_kv_clear_error re-zeroes the words the kernels synchronise through, clears the flags
 * and restarts the numbering, in stream order; sequence state is kept.  Not allowed inside a stream capture. */
int ssd_kv_clear_error(ssd_kv* kv, void* stream);

/* Test hooks: force, from the host, conditions that otherwise need a fault.  SSD_HOOK_TIMEOUT raises the device's
 * timeout word, so that every bounded wait of later forwards gives up at once and all kernels still exit normally.
 * SSD_HOOK_LAUNCH_NUMBER sets the number the next forward on the cache reads (1 .. 2^25-2), on device and host;
 * SSD_HOOK_LAUNCH_NUMBER_DEVICE_ONLY sets it on the device alone (up to 2^25-1, the value at which forwards refuse
 * to run), as a graph replayed past the limit would leave it. */
#define SSD_HOOK_TIMEOUT 1
#define SSD_HOOK_LAUNCH_NUMBER 2
#define SSD_HOOK_LAUNCH_NUMBER_DEVICE_ONLY 3
int ssd_kv_test_hook(ssd_kv* kv, int what, long long value, void* stream);

/* ---- measurement ---------------------------------------------------------------------------------------
 * Between ssd_profile_begin(kind) and ssd_profile_end() every launch of the named kernel family is bracketed
 * by a pair of HIP events on its stream (this perturbs the pipeline slightly, so it is meant for a pass of its
 * own, not for the region whose throughput is reported).  ssd_profile_end synchronises and returns the summed
 * kernel time in milliseconds and the number of launches.  Kinds: 0 QKV GEMM, 1 attention (chunks + combine),
 * 2 output-projection GEMM, 3 gate/up GEMM + SwiGLU, 4 down GEMM, 5 head GEMM, 6 the persistent whole-forward
 * kernel (used instead of 0-5 when the shape allows it). */
int ssd_profile_begin(int kind);
int ssd_profile_end(double* total_ms, int* launches);

/* Which kernels ran the last decoder forward on `kv` (host bookkeeping, no synchronisation):
 * 0 none yet, 1 one launch per operator (fp32 storage, more than 16 rows, head_dim other than 64),
 * 2 one persistent kernel with grid barriers between phases, 3 one persistent kernel whose phases are ordered by
 * tagged data words (the default for bf16 storage and at most 16 rows; the environment variable
 * SSD_FORWARD=barrier, read at ssd_kv_create, selects 2 instead; 2 is also what runs when a launch exceeds the
 * limits of 3), 4 the same kernel with the attention of a short prefix
 * (at most 1520 cached positions) done by one workgroup per row tile instead of 256-key parts (the default for caches
 * created with pending_cap 2; SSD_ATTN_WHOLE=1 selects it for every cache, 0 for none). */
int ssd_kv_last_forward_path(const ssd_kv* kv);

/* Phase trace of the persistent forward kernels, recorded only by builds with -DSSD_TRACE (otherwise SSD_ENOSUP
 * and the kernels carry no clock reads): with enable != 0 every later forward on `kv` records, per
 * workgroup, 100 MHz wall-clock samples.  When `out` is non-NULL the samples of the last forward are copied out
 * first (synchronises `stream`): rows of 512 entries per workgroup, *n_wgs workgroups, cap >= 512 * workgroups.
 * Barrier kernel: out[wg*512 + 2*b] = arrival and [.. + 2*b+1] = release of grid barrier b for b < *n_samples / 2.
 * Barrier-free kernel: entry 1 = entry of the workgroup, entry 0 = past the start barrier; entries 2 + 10*layer + 2*k and + 1 = operands staged / outputs stored of phase
 * k (0 QKV, 1 attention, 2 output projection, 3 MLP, 4 partial sum), 0 where the workgroup has no item. */
int ssd_trace_barriers(ssd_kv* kv, int enable, void* stream, unsigned long long* out, int cap, int* n_wgs,
                       int* n_samples);

const char* ssd_strerror(int code);
const char* ssd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
