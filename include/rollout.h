/*
 * librollout -- the rollout phase of length-aware (SortedRL-style) RL training on one MI355X.
 *
 * The four core calls follow the paper's statement of the problem (Fig. 2 steps 1-4, Sec. 3.1-3.3):
 * a controller feeds more prompts than the engine has running slots (oversubscription), the engine
 * decodes one token per running request per step, finished short rollouts leave the batch early and
 * are handed back in length-ordered update groups, freed slots are refilled from the queue, and
 * unfinished rollouts stay cached across update boundaries (partial mode).
 *
 * Conventions
 *   - Plain C ABI.  Every call returns 0 (ROLLOUT_OK) or a negative ROLLOUT_E* code;
 *     rollout_last_error() gives a library-owned message valid until the next call on that ctx.
 *   - Pointers are HOST pointers unless the name ends in _dev (device memory on cfg.device).
 *   - The library copies what it is given; the caller keeps ownership of every buffer it passes
 *     in and of every output buffer it provides.  One ctx is used from one thread at a time.
 *   - Everything runs in hand-written HIP kernels on the ctx's own stream; there is no CPU
 *     fallback: without a usable GPU rollout_init fails with ROLLOUT_EDEVICE.
 */
#ifndef ROLLOUT_H
#define ROLLOUT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rollout_ctx rollout_ctx; /* opaque */

enum {
  ROLLOUT_OK = 0,
  ROLLOUT_EINVAL = -1,  /* bad argument / unsupported configuration */
  ROLLOUT_ENOMEM = -2,  /* KV pool cannot hold one maximum-length rollout, or allocation failed */
  ROLLOUT_EBUSY = -3,   /* grouped-loading gate closed, or sequence table full */
  ROLLOUT_ERANGE = -4,  /* prompt too long, token id out of range, output buffer too small */
  ROLLOUT_EDEVICE = -5  /* HIP error; the ctx is unusable afterwards */
};

enum { ROLLOUT_EOS_FORCED_ONLY = 0, ROLLOUT_EOS_NATURAL_OR_FORCED = 1 };
/* Sec. 3.2: partial mode keeps unfinished rollouts (tokens, log-probs, KV) across update boundaries;
 * on-policy mode terminates them at a boundary and re-queues their prompts; SYNC is the canonical
 * baseline the paper compares against (a batch is admitted only when every slot is empty). */
enum { ROLLOUT_MODE_PARTIAL = 0, ROLLOUT_MODE_ONPOLICY = 1, ROLLOUT_MODE_SYNC = 2 };
enum { ROLLOUT_FLUSH = 1 };
enum {
  ROLLOUT_DEBUG_NO_MODEL = 1,   /* scheduler kernels only: every non-forced token is 0 */
  ROLLOUT_DEBUG_TIME_ATTN = 2   /* bracket each decode-attention kernel launch (not its merge) with HIP events */
};

typedef struct rollout_cfg {
  /* policy shape (pre-norm decoder, GQA, rotate-half RoPE, SwiGLU, untied LM head) */
  uint32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_theta;
  uint32_t qkv_bias;          /* 0/1 */
  uint32_t weight_dtype;      /* element type of the weights blob: 0 = fp32 (rounded to bf16 at init), 1 = bf16 */
  uint32_t weights_on_device; /* 0 = `weights` is a host pointer, 1 = device pointer */
  /* engine */
  uint32_t max_slots;         /* Q: running-queue size (Sec. 4.4.1) */
  uint32_t page_tokens;       /* must be 16 */
  uint64_t kv_pool_bytes;     /* 0 = size the pool for max_slots maximum-length rollouts */
  uint32_t max_prompt_len, max_new_tokens;
  uint32_t max_seqs;          /* capacity of the sequence table = most submitted-but-unharvested rollouts */
  int32_t eos_id;
  uint32_t eos_mode;          /* ROLLOUT_EOS_* */
  uint32_t mode;              /* ROLLOUT_MODE_* */
  int32_t max_staleness;      /* update boundaries a KV cache may survive; -1 = unlimited */
  uint32_t grouped_loading;   /* 1 = rollout_submit refused until the previous group is fully harvested (Sec. 3.1) */
  uint32_t debug_flags;       /* ROLLOUT_DEBUG_* */
  uint64_t page_seed;         /* seeds the initial order of the page free list */
  int32_t device;             /* HIP device ordinal */
  uint32_t reserved;
  /* sampling (Sec. 4.1 collects several sampled responses per prompt: rollout_submit_n) */
  float temperature;          /* 0 = greedy argmax; > 0 = draw from softmax(logits / temperature) by Gumbel-max */
  uint32_t reserved2;
  uint64_t sample_seed;       /* key of the counter-based generator; the counter is (vocab index, token index, seq_id) */
} rollout_cfg;

typedef struct rollout_step_info {
  uint64_t step;                   /* index of the step just executed */
  uint32_t n_ran;                  /* r_s: slots that produced a token this step (prefill or decode) */
  uint32_t n_active;               /* running requests after the step */
  uint32_t n_finished_unharvested;
  uint32_t n_queued;
  uint32_t free_pages;
  uint32_t n_admitted;             /* admitted (prefilled) this step */
  uint32_t n_finished_step;
  uint32_t n_preempted_step;
  uint64_t ctx_tokens;             /* cached tokens over the running requests after the step: what the next step's
                                      decode attention reads (times the per-token KV bytes) */
  /* the work this step did (Sec. 2.2: a step streams the weights once, the KV caches of its decode rows, and computes
   * the prefill of the slots it refilled) */
  uint32_t n_decode_rows;          /* rows that decoded one token on top of their cache (n_ran - n_admitted) */
  uint32_t prefill_tokens;         /* token positions prefilled for the slots admitted this step */
  uint64_t decode_ctx_tokens;      /* cached tokens the decode rows attended over, per layer */
  uint64_t prefill_ctx_pairs;      /* sum over the prefilled positions of their causal context length (query-key pairs
                                      of the prefill attention, per layer and head) */
} rollout_step_info;

typedef struct rollout_traj {
  uint64_t seq_id;           /* submission order, 0-based */
  uint32_t slot;             /* slot of the (last) admission */
  uint32_t completion_step;
  uint32_t gen_len;
  uint32_t group_idx;        /* running index of the update group this record belongs to */
  uint64_t tok_off;          /* offset of its gen_len tokens (and log-probs) in tok_buf / logp_buf */
  uint32_t n_preempt;
  uint32_t policy_version;   /* update boundaries (policy versions) passed when its last token was produced; compare with
                                rollout_stats_t.version at the harvest to see how stale a finished rollout is */
} rollout_traj;

typedef struct rollout_stats_t {
  uint64_t steps;
  uint64_t busy;             /* sum_s r_s */
  uint64_t idle;             /* sum_s (Q - r_s): numerator of eq. 4 with dt = 1 step */
  uint64_t steps_q, idle_q;  /* the same restricted to steps that began with a non-empty queue */
  uint64_t gen_tokens, discarded_tokens, prefill_tokens;
  uint64_t n_preempt, n_stale, version;
  uint64_t n_pages, max_pages_used;
  /* filled when ROLLOUT_DEBUG_TIME_ATTN is set: decode-attention launches of decode rows only */
  uint64_t attn_launches;
  uint64_t attn_kv_tokens;   /* sum over those launches of the cached tokens attended (all kv heads share it) */
  double attn_ms;            /* summed HIP-event time of those launches */
  double wall_ms_steps;      /* host wall time spent inside rollout_step */
} rollout_stats_t;

/* Fig. 2 / Sec. 3.3: build the engine.  `weights` holds, in this order,
 *   embed[V,D], per layer { attn_norm[D], wq[Hq*d,D], wk[Hkv*d,D], wv[Hkv*d,D], (bq,bk,bv if qkv_bias),
 *   wo[D,Hq*d], ffn_norm[D], w_gate[F,D], w_up[F,D], w_down[D,F] }, final_norm[D], lm_head[V,D],
 * every matrix row-major [out, in].  The blob is copied (and repacked) before the call returns.
 * Errors: EINVAL (null / unsupported shape: head_dim must be 32 or 128, Hq/Hkv in {1,4,5}, page_tokens 16,
 * max_slots <= 1024, d_model, d_ffn multiples of 64, d_model <= 8192, d_ffn <= 2^20, vocab <= 2^24), ENOMEM, EDEVICE. */
int rollout_init(rollout_ctx** out, const void* weights, size_t weights_bytes, const rollout_cfg* cfg);

/* Sec. 3.2 / Sec. 3.3: install the policy produced by the trainer's update (same shape, same blob format and location
 * as at rollout_init).  Call it between steps, normally right after a rollout_harvest that returned groups.  Running
 * rollouts keep their tokens, log-probs and KV pages: tokens generated afterwards use the new weights on top of the
 * cache they already have, and their log-probs are recorded under the policy that produced them, so a harvested
 * trajectory carries the concatenation of old- and new-policy segments (the pi_old of eq. 1).  With
 * max_staleness >= 0 the boundary of that harvest has already released the caches that are too old; they are rebuilt
 * under the new weights by re-prefill.  Errors: EINVAL (blob size does not match the shape; the ctx is unusable
 * afterwards), ENOMEM, EDEVICE. */
int rollout_update_weights(rollout_ctx*, const void* weights, size_t weights_bytes);

/* Fig. 2 step 1 "feed prompts": append n prompts to the FIFO queue.  tokens = concatenated ids,
 * offsets[n+1] delimits them, target_len[i] > 0 forces EOS as the target_len-th generated token
 * (Sec. 4.4.1 pins per-sample lengths this way), 0 = no forced length.  first_seq_id (nullable) receives the id
 * of the first prompt; ids are consecutive.  Nothing is consumed on error.
 * Errors: ERANGE (empty or over-long prompt, id outside [0, vocab), target_len > max_new_tokens),
 * EBUSY (grouped loading: previous group not fully harvested; or more than max_seqs unharvested). */
int rollout_submit(rollout_ctx*, const int32_t* tokens, const uint32_t* offsets, const uint32_t* target_len,
                   uint32_t n, uint64_t* first_seq_id);

/* Sec. 4.1 (several responses are drawn for every prompt): like rollout_submit, but each of the n prompts starts k
 * rollouts.  target_len has n*k entries, prompt-major; seq ids follow the same order (prompt i, response r ->
 * first_seq_id + i*k + r).  The k rollouts of a prompt share the KV pages the prompt fills completely, except the page
 * holding its last token: floor((prompt_len - 1) / 16) pages.  The first of them to be admitted allocates and
 * prefills the whole prompt; one admitted while a sibling is running allocates only its private tail and prefills
 * from the first unshared position; shared pages return to the pool when the last running sibling leaves (finish,
 * preemption, staleness or on-policy termination), and a rollout that attached takes the shared part's policy
 * version as its own for the staleness rule.  With temperature 0 the k responses are identical.  k = 1, or a prompt
 * of at most 16 tokens, shares nothing.  Errors as rollout_submit; EINVAL for k = 0; n*k counts against max_seqs. */
int rollout_submit_n(rollout_ctx*, const int32_t* tokens, const uint32_t* offsets, const uint32_t* target_len,
                     uint32_t n, uint32_t k, uint64_t* first_seq_id);

/* One global decode step (Sec. 3.1): refill free slots from the queue head (prefill), decode one token for
 * every other running request, emit (forced EOS / greedy argmax, lowest index on ties / a Gumbel-max draw when
 * cfg.temperature > 0: argmax_j logits_j / T - log(-log u_j), u_j from Philox4x32-10), evict finished
 * rollouts and free their pages, grow pages (preempting the shortest rollout if the pool is empty).
 * info is nullable. */
int rollout_step(rollout_ctx*, rollout_step_info* info);

/* Fig. 2 steps 3-4 "collect" and "sort and feed training batches": cut the finished-unharvested rollouts,
 * sorted by (completion_step, gen_len, seq_id), into complete groups of group_size; with ROLLOUT_FLUSH and
 * nothing queued or running the remainder forms a last short group.  recs[0..n_recs) are in that order;
 * tokens (and log-probs when logp_buf != NULL) are packed at recs[i].tok_off.  Each returned group is one
 * update boundary (policy version += 1); caches older than max_staleness are then released for re-prefill
 * (partial mode) or unfinished rollouts are discarded and re-queued (on-policy mode).
 * If recs_cap or tok_cap is too small: ERANGE, n_recs / tok_needed report the sizes, nothing is consumed. */
int rollout_harvest(rollout_ctx*, uint32_t group_size, uint32_t flags, rollout_traj* recs, uint32_t recs_cap,
                    int32_t* tok_buf, float* logp_buf, uint64_t tok_cap, uint32_t* n_groups, uint32_t* n_recs,
                    uint64_t* tok_needed);

/* Eq. 4 counters and friends. */
int rollout_stats(rollout_ctx*, rollout_stats_t* out);

/* Teacher forcing for parity tests: like rollout_step, but slot i emits forced_tok[i] when it is >= 0
 * (forced_tok has max_slots entries), and logits_out (nullable, host, max_slots * vocab floats) receives
 * the fp32 logits row of every slot that ran (other rows are left untouched). */
int rollout_step_forced(rollout_ctx*, const int32_t* forced_tok, float* logits_out, rollout_step_info* info);

/* Sec. 4.1 "incomplete request state retrieval": copy out the partial trajectory of any sequence.
 * state: 0 queued, 1 active, 2 finished, 3 harvested.  tok_buf/logp_buf nullable; cap in elements. */
int rollout_peek(rollout_ctx*, uint64_t seq_id, int32_t* tok_buf, float* logp_buf, uint32_t cap,
                 uint32_t* gen_len, uint32_t* state, int32_t* slot);

/* Debug: page ids currently held by a slot (n = 0 if the slot is empty). */
int rollout_slot_pages(rollout_ctx*, uint32_t slot, int32_t* pages, uint32_t cap, uint32_t* n);

const char* rollout_last_error(rollout_ctx*);
void rollout_destroy(rollout_ctx*);

/* ---- the ragged paged GQA decode-attention kernel alone (Sec. 2.2: rollout is bound by streaming KV caches) ----
 * KV pool layout (bf16): for page p and kv head g, a block of 2 * 16 * head_dim elements at
 *   ((p * n_kv_heads + g) * 2 * 16 * head_dim):  K as [head_dim/8][16 tokens][8 dims], then
 *   V as [2 token-halves][head_dim][8 tokens].
 * All pointers are device pointers; `stream` is a hipStream_t (NULL = default stream). */

/* Bytes of a pool of n_pages pages (one layer). */
uint64_t rollout_attn_pool_bytes(uint32_t n_pages, uint32_t n_kv_heads, uint32_t head_dim);

/* Scatter n_tok rows of k, v (bf16 [n_tok, Hkv, d]) into the pool: row t belongs to sequence tok_seq_dev[t]
 * at position tok_pos_dev[t]; page_table_dev is int32 [n_seqs, max_pages]. */
int rollout_attn_write_kv(void* pool_dev, uint32_t n_kv_heads, uint32_t head_dim, const void* k_dev,
                          const void* v_dev, const int32_t* tok_seq_dev, const int32_t* tok_pos_dev,
                          const int32_t* page_table_dev, uint32_t max_pages, uint64_t n_tok, void* stream);

/* Workspace bytes rollout_attn_plan / rollout_attn_decode need for n sequences whose lengths sum to total_ctx. */
uint64_t rollout_attn_workspace_bytes(uint32_t n, uint64_t total_ctx, uint32_t n_q_heads, uint32_t head_dim);

/* Build the work list for context lengths ctx_len (host int32 [n], each >= 1) at the head of workspace_dev: one item
 * (one workgroup per kv head) per four consecutive chunks of a sequence.  The chunk (cached tokens per wavefront, a
 * multiple of 64 in 128..1024) is chosen from the total context as the largest that still leaves every resident
 * wavefront slot of the chip a span or two; it is returned in chunk_tokens and must be passed to rollout_attn_decode; n_work receives the number
 * of items.  Also zeroes the per-(sequence, kv head) arrival counters with which the work items of a long sequence
 * find out which of them finishes last and merges their partial results; every rollout_attn_decode leaves them at
 * zero again, so one plan serves any number of launches -- but launches that overlap in time must not share a
 * workspace.  Synchronous (blocking host-to-device copies). */
int rollout_attn_plan(const int32_t* ctx_len, uint32_t n, uint32_t n_q_heads, uint32_t n_kv_heads, uint32_t head_dim,
                      void* workspace_dev, uint64_t workspace_bytes, uint32_t* n_work, uint32_t* chunk_tokens);

/* o[i] = softmax(q[i] K_i^T / sqrt(d)) V_i for the n planned sequences: q_dev bf16 [n, Hq, d]; out_dev fp32
 * [n, Hq, d] if out_fp32 else bf16.  Only enqueues kernels on `stream`; never synchronises or allocates.
 * Errors: EINVAL (null pointer, unsupported head_dim / group size, bad chunk_tokens). */
int rollout_attn_decode(const void* pool_dev, uint32_t n_q_heads, uint32_t n_kv_heads, uint32_t head_dim,
                        const void* q_dev, const int32_t* page_table_dev, uint32_t max_pages, uint32_t n,
                        uint32_t n_work, uint32_t chunk_tokens, void* out_dev, int out_fp32, void* workspace_dev,
                        void* stream);

/* ---- the bf16 MFMA projection GEMM alone: c[M,N] (fp32) = a[M,K] (bf16, row-major) * w[N,K]^T (bf16) ----
 * The kernels read w in a packed fragment layout (tiles of 32 rows x 64 columns stored in the order the MFMA
 * operand loads consume them, rows padded to a multiple of 32); rollout_gemm_pack_weights converts a row-major
 * [N, K] matrix into rollout_gemm_packed_bytes(N, K) bytes at packed_dev.  K must be a multiple of 64, K <= 2^20,
 * M and N <= 2^24 (EINVAL otherwise).
 * workspace_dev needs rollout_gemm_workspace_bytes(M, N, K) bytes.  All calls only enqueue on `stream`. */
uint64_t rollout_gemm_packed_bytes(uint32_t N, uint32_t K);
int rollout_gemm_pack_weights(const void* w_dev, void* packed_dev, uint32_t N, uint32_t K, void* stream);
uint64_t rollout_gemm_workspace_bytes(uint32_t M, uint32_t N, uint32_t K);
int rollout_gemm_bf16(const void* a_dev, const void* w_packed_dev, float* c_dev, uint32_t M, uint32_t N, uint32_t K,
                      void* workspace_dev, uint64_t workspace_bytes, void* stream);

/* rollout_gemm_bf16 for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same kernels,
 * same result bit for bit.  The split-K partial sums go to a fixed array of rollout_gemm_static_scratch_bytes()
 * (32 MiB) inside the library's device image; every GPU the library runs on holds its own copy until the process
 * ends.  The call runs on the current device, allocates nothing (no hipMalloc / hipFree, no allocating library
 * routine) and only enqueues on `stream`.  Errors: EINVAL as rollout_gemm_bf16 (K not a multiple of 64, a dimension
 * beyond the maxima above); ERANGE when rollout_gemm_splits(M, N, K) * M * N * 4 bytes exceed the array -- a second line
 * of defence: the library never launches more than 256 workgroups of a split-K product (splits x 128-column tiles x
 * 256-row blocks), which bounds the partial sums of every shape by 256 x 256 x 128 fp32 = the array's 32 MiB (the O
 * projection of the 8B shape at 256 rows, 8 splits, fills it exactly); EDEVICE.  All calls on one GPU
 * share that GPU's array, which keeps the last call's contents (every split overwrites its whole partial, nothing
 * needs clearing): calls that overlap on one GPU -- different streams or threads -- race, so serialise them. */
uint64_t rollout_gemm_static_scratch_bytes(void);
int rollout_gemm_bf16_static(const void* a_dev, const void* w_packed_dev, float* c_dev, uint32_t M, uint32_t N, uint32_t K,
                             void* stream);

/* The gate/up projection with its SwiGLU epilogue alone (the largest weight stream of a decode step, Sec. 2.2):
 * act[M, F] (bf16) = silu(a Wg^T) * (a Wu^T), a bf16 [M, K].  w_packed_dev is rollout_gemm_pack_weights applied to the
 * [2F, K] matrix whose rows interleave gate and up in blocks of 16: rows 32q .. 32q+15 = Wg rows 16q .. 16q+15,
 * rows 32q+16 .. 32q+31 = Wu rows 16q .. 16q+15 (so one wavefront's 32 output columns hold gate and up of the same
 * 16 features).  F must be a multiple of 16, K of 64.  Enqueue only; needs no workspace. */
int rollout_gemm_swiglu_bf16(const void* a_dev, const void* w_packed_dev, void* act_dev, uint32_t M, uint32_t F, uint32_t K,
                             void* stream);

/* Name of the kernel instantiation rollout_gemm_bf16 (swiglu = 0; N output columns) or rollout_gemm_swiglu_bf16
 * (swiglu = 1; N = 2F) launches for this shape, e.g. "k_gemm_bf16_deep<1>"; the engine's projections go through the
 * same selection, so a parity test can state which instantiation it covers.  splits = the number of K splits
 * (0 = what rollout_gemm_bf16 picks, i.e. rollout_gemm_splits; the engine uses that for the QKV, O and down
 * projections and 1 for the LM head; ignored with swiglu).  Library-owned, thread-local string, valid until the
 * next call; "" (resp. 0) for an unsupported shape. */
const char* rollout_gemm_kernel_name(uint32_t M, uint32_t N, uint32_t K, uint32_t splits, int swiglu);
uint32_t rollout_gemm_splits(uint32_t M, uint32_t N, uint32_t K);

/* ---- plain streaming kernels: dst = src, and a pure read of src (16-byte accesses, grid-stride).  They exist to
 * calibrate the memory-traffic counters against a known byte count and to measure the practical HBM ceiling that the
 * KV and weight streams of the rollout step (Sec. 2.2) are compared with.  bytes must be a multiple of 16;
 * sink_dev needs 4 writable bytes.  Enqueue only. */
int rollout_stream_copy(const void* src_dev, void* dst_dev, uint64_t bytes, void* stream);
int rollout_stream_read(const void* src_dev, uint64_t bytes, void* sink_dev, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ROLLOUT_H */
