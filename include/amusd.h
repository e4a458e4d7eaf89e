/*
 * amusd.h - C ABI of the MI355X (gfx950) verify-pass library.
 *
 * The library implements the per-model steps of asynchronous speculative
 * decoding (Algorithm 1 of the AMUSD paper): VerifyTokens with the mismatch
 * test and the verified-token cache update, GenerateToken, and the rollback of
 * a key-value cache, for Llama-style decoders (the model family of the paper's
 * Section IV-A), plus drivers that run the loops on those steps.
 *
 * Conventions
 *   - Every function returns AMUSD_OK (0) or a negative AMUSD_E_* code; it
 *     never throws or aborts.  On error the model's state is unchanged (amusd_prefill runs several passes:
 *     if one fails, the cache length is restored to what it was before the call).
 *   - All pointers are owned by the caller.  The library copies what it needs:
 *     after a successful amusd_model_set_tensor / amusd_model_load the caller
 *     may free the weight buffers.  Output scalars/arrays are HOST memory and
 *     are valid when the call returns (calls are synchronous for the host).
 *   - A model is bound to one HIP stream given at creation; all its device work
 *     is enqueued there.  Calls on one model must not overlap; calls on
 *     different models may run concurrently from different host threads.
 *   - Token ids are int32 in [0, vocab).  Positions count tokens from 0.
 *   - A pass is a chain of ~6 short dependent kernels per layer, each of which starts by reading its arguments.
 *     The quoted latencies hold with the HIP runtime keeping kernel arguments in device memory
 *     (HIP_FORCE_DEV_KERNARG=1 in the environment before the process's first HIP call; the Python binding sets
 *     it when imported first); with arguments in host memory every kernel waits for PCIe and an 8B-shape pass
 *     takes about 12 % longer.  The library itself cannot change this setting.
 *
 * Per-sequence state: kv_len (tokens in the sequence's cache) and p_next, the
 * model's greedy token for position kv_len (known once the cache is non-empty).
 * A model holds max_seqs independent sequences (one by default); the calls
 * without a sequence argument act on sequence 0.
 */
#ifndef AMUSD_H
#define AMUSD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AMUSD_OK            0
#define AMUSD_E_ARG        -1   /* null pointer, k out of [1,max_k], unsupported or inconsistent config */
#define AMUSD_E_RANGE      -2   /* ctx_len / new_len outside [0, kv_len] (a cache cannot be rolled forward) */
#define AMUSD_E_CAPACITY   -3   /* the call would need more than max_ctx positions */
#define AMUSD_E_TOKEN      -4   /* token id outside [0, vocab) */
#define AMUSD_E_STATE      -5   /* model not finalized / tensor missing / p_next unknown (empty cache) */
#define AMUSD_E_HIP        -6   /* HIP runtime failure (no device, out of memory, launch error) */
#define AMUSD_E_NOMEM      -7   /* host allocation failure */

#define AMUSD_DTYPE_FP32    0
#define AMUSD_DTYPE_BF16    1   /* weights bf16; the cache, queries and attention probabilities are kept as IEEE half
                                  * (same 2 bytes, three more mantissa bits): keys, values and queries are assumed to
                                  * lie within +-65504 and are clamped to that range when stored */

#define AMUSD_MAX_K        16   /* rows of one pass: the 16-row matrix-core tile */
#define AMUSD_MAX_SEQS   4096   /* sequences (key-value caches) one model can hold */

/* Tensor ids for amusd_model_set_tensor.  Matrices are row-major
 * [out_features, in_features] in the model's dtype (bf16 bit patterns or
 * fp32); gains are [d_model] in the same dtype. */
enum {
    AMUSD_T_EMBED = 0,      /* [vocab, d_model]                  (no layer) */
    AMUSD_T_LM_HEAD = 1,    /* [vocab, d_model]                  (no layer) */
    AMUSD_T_FINAL_NORM = 2, /* [d_model]                         (no layer) */
    AMUSD_T_WQ = 3,         /* [n_q_heads*head_dim, d_model]     per layer  */
    AMUSD_T_WK = 4,         /* [n_kv_heads*head_dim, d_model]               */
    AMUSD_T_WV = 5,         /* [n_kv_heads*head_dim, d_model]               */
    AMUSD_T_WO = 6,         /* [d_model, n_q_heads*head_dim]                */
    AMUSD_T_WG = 7,         /* [d_ffn, d_model]   gate projection           */
    AMUSD_T_WU = 8,         /* [d_ffn, d_model]   up projection             */
    AMUSD_T_WD = 9,         /* [d_model, d_ffn]   down projection           */
    AMUSD_T_NORM_ATTN = 10, /* [d_model]                                    */
    AMUSD_T_NORM_MLP = 11,  /* [d_model]                                    */
    AMUSD_T_COUNT = 12
};

/* Options for amusd_set_option. */
enum {
    AMUSD_OPT_KEEP_LOGITS = 0, /* 1: each pass also stores its fp32 logits (test hook), default 0 */
    AMUSD_OPT_TIME_STAGE = 2    /* AMUSD_STAGE_* to bracket with HIP events in every pass, -1: none (default) */
};

/* Stages of a pass, for AMUSD_OPT_TIME_STAGE / amusd_stage_time. */
enum {
    AMUSD_STAGE_EMBED = 0, AMUSD_STAGE_QKV = 1, AMUSD_STAGE_ATTENTION = 2, AMUSD_STAGE_ATTN_MERGE = 3,
    AMUSD_STAGE_OPROJ = 4, AMUSD_STAGE_GATEUP = 5, AMUSD_STAGE_DOWN = 6, AMUSD_STAGE_LMHEAD = 7,
    AMUSD_STAGE_ACCEPT = 8, AMUSD_STAGE_COUNT = 9
};

typedef struct amusd_model amusd_model; /* opaque, owned by the library */

/* Decoder shape.  Requirements: n_q_heads / n_kv_heads is 1, 2, 4 or 8; head_dim is 64 or
 * 128; d_model, n_q_heads*head_dim and d_ffn are multiples of 32 (bf16) or 16
 * (fp32); vocab and d_ffn multiples of 16; 1 <= max_k <= AMUSD_MAX_K;
 * 0 <= max_seqs <= AMUSD_MAX_SEQS. */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t max_ctx;   /* capacity of the key-value cache, in positions */
    int32_t max_k;     /* largest number of rows a pass will be given */
    int32_t dtype;     /* AMUSD_DTYPE_* : storage type of weights and of the cache */
    float rope_theta;  /* rotary base: pair i of a head turns by pos * theta^(-2i/head_dim) */
    float rms_eps;     /* added to the mean square inside every RMSNorm */
    int32_t max_seqs;  /* independent sequences, each with a cache of max_ctx positions; 0 means 1 */
} amusd_config;

/* All weights at once, for amusd_model_load.  The per-layer members are arrays
 * of n_layers pointers. */
typedef struct {
    const void *embed, *lm_head, *final_norm;
    const void *const *wq, *const *wk, *const *wv, *const *wo, *const *wg, *const *wu, *const *wd,
        *const *norm_attn, *const *norm_mlp;
    int32_t on_device; /* 0: the pointers are host memory; 1: device memory */
} amusd_weights;

typedef struct {
    int32_t rounds;          /* verify passes run */
    int32_t rollbacks;       /* passes that ended in a mismatch (rollback flag raised) */
    int32_t draft_steps;     /* draft-model steps run, including those rolled back */
    int32_t accepted_total;  /* sum of accept_len over all passes */
    int32_t accept_hist[AMUSD_MAX_K + 1]; /* passes by accept_len */
    double wall_ms;          /* host wall-clock time of the loop, prompt prefill excluded */
} amusd_loop_stats;

/* ---- model set-up (Algorithm 1, "Require": the draft and verify models) --------------------- */

/* Allocates a model of the given shape on the current HIP device: weight
 * storage (re-laid out for the kernels), a zeroed cache of max_ctx positions,
 * rotary tables and scratch.  hip_stream is a hipStream_t (NULL: the default
 * stream).  *out is set only on success and released by amusd_model_free. */
int amusd_model_create(const amusd_config *cfg, void *hip_stream, amusd_model **out);

/* Copies one tensor into the model.  `layer` is ignored for the three global
 * tensors.  data points to host (on_device=0) or device (on_device=1) memory
 * of exactly the tensor's size; it is not referenced after the call returns. */
int amusd_model_set_tensor(amusd_model *m, int32_t tensor_id, int32_t layer, const void *data, int32_t on_device);

/* Checks that every tensor has been set and makes the model usable.
 * AMUSD_E_STATE names a missing tensor through amusd_last_error. */
int amusd_model_finalize(amusd_model *m);

/* create + set every tensor + finalize. */
int amusd_model_load(const amusd_config *cfg, const amusd_weights *w, void *hip_stream, amusd_model **out);

int amusd_model_free(amusd_model *m);

/* ---- the steps of Algorithm 1 ------------------------------------------------------------- */

/* Cache initialisation with the prompt (Algorithm 1, the state set-up before the two loops): appends n
 * tokens (host array) at
 * positions kv_len .. kv_len+n-1 unconditionally, several rows per pass, and
 * returns in *next_token the greedy token after the last one.  next_token may
 * be NULL.  Errors: ARG, TOKEN, CAPACITY. */
int amusd_prefill(amusd_model *m, const int32_t *tokens, int32_t n, int32_t *next_token);

/* VerifyTokens + mismatch test + cache update (Algorithm 1, VerifyProcess).
 * First truncates the cache to ctx_len (must be in [0, kv_len]; at ctx_len = 0 the model's token for
 * position 0 is unknown unless amusd_set_next gave it, and the call fails with STATE).  Row j feeds
 * draft[j] (host array of k ids) at position ctx_len+j and attends to the
 * ctx_len cached positions plus rows 0..j.  With g[j] the arg-max token of row
 * j (lowest id on ties) and target = [p(ctx_len), g[0], .., g[k-2]], where
 * p(ctx_len) is the model's stored greedy token for that position:
 *   *accept_len = length of the longest prefix with draft[i] == target[i];
 *   *next_token = target[accept_len] if accept_len < k, else g[k-1].
 * Afterwards kv_len = ctx_len + accept_len and p_next = *next_token.
 * Errors: ARG (k), RANGE (ctx_len), CAPACITY (ctx_len+k > max_ctx), TOKEN, STATE. */
int amusd_verify(amusd_model *m, int32_t ctx_len, const int32_t *draft, int32_t k,
                 int32_t *accept_len, int32_t *next_token);

/* amusd_verify for callers that cannot allocate device memory while they run (code under HIP graph capture
 * around it, tight serving loops, harnesses that forbid allocation calls): the same pass with the same
 * arguments, results and errors, bit for bit, but the buffers a pass keeps between its stages (residual stream,
 * GEMM inputs, queries, attention partials, arg-max partials) live in one statically allocated device array of
 * AMUSD_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process ends, instead of in the
 * model's own workspace.  The call makes no allocation of any kind (device, pinned or through another library).
 * A model whose workspace does not fit (amusd_static_scratch_bytes above the limit: many sequences per pass,
 * very wide models) is refused with AMUSD_E_CAPACITY and unchanged state.  All models on one GPU share the
 * array and it keeps the last call's contents (the region is cleared when another model used it last), so two
 * amusd_verify_static calls that overlap in time on one GPU race, also when they are for different models on
 * different streams.  Inputs (weights, cache, drafts) and outputs are where amusd_verify has them. */
#define AMUSD_STATIC_SCRATCH_BYTES (16 * 1024 * 1024)
int amusd_verify_static(amusd_model *m, int32_t ctx_len, const int32_t *draft, int32_t k,
                        int32_t *accept_len, int32_t *next_token);
/* Bytes of the static array a pass of this model needs (a negative error code if m is NULL). */
int64_t amusd_static_scratch_bytes(const amusd_model *m);

/* GenerateToken (Algorithm 1, DraftProcess): feeds p_next at position kv_len,
 * appends its keys/values (kv_len grows by one) and returns the new p_next in
 * *token_out.  Same kernels as a pass with k = 1.  Errors: STATE, CAPACITY. */
int amusd_draft_step(amusd_model *m, int32_t *token_out);

/* Cache rollback (Algorithm 1, the draft side's reaction to the rollback flag; also how the verify cache
 * drops rejected rows): sets kv_len = new_len in O(1), no data is
 * moved; p_next becomes the greedy token recorded for position new_len.
 * Errors: RANGE unless 0 <= new_len <= kv_len. */
int amusd_kv_rollback(amusd_model *m, int32_t new_len);

/* Replaces p_next (the token the next amusd_draft_step feeds): how the draft
 * model receives the verifier's token after a rollback.  Errors: TOKEN. */
int amusd_set_next(amusd_model *m, int32_t token);

/* Current cache length, or a negative error code if m is NULL. */
int amusd_kv_len(const amusd_model *m);

/* Current p_next in *token (-1 if unknown).  */
int amusd_get_next(const amusd_model *m, int32_t *token);

/* ---- several sequences sharing one weight stream -------------------------------------------- */
/* Not in the paper: VerifyTokens reads every weight once for k rows, so the
 * rows of one pass may as well belong to different sequences.  Each sequence
 * `seq` in [0, max_seqs) has its own cache, kv_len and p_next; one pass serves
 * up to 16 rows in total.  A sequence's results are bit-identical to those of
 * the same call made for it alone. */

/* amusd_prefill / amusd_kv_rollback / amusd_set_next / amusd_kv_len /
 * amusd_get_next for sequence `seq`.  Errors as those, plus ARG for a bad seq. */
int amusd_seq_prefill(amusd_model *m, int32_t seq, const int32_t *tokens, int32_t n, int32_t *next_token);
int amusd_seq_rollback(amusd_model *m, int32_t seq, int32_t new_len);
int amusd_seq_set_next(amusd_model *m, int32_t seq, int32_t token);
int amusd_seq_len(const amusd_model *m, int32_t seq);
int amusd_seq_get_next(const amusd_model *m, int32_t seq, int32_t *token);

/* amusd_verify for n_seq distinct sequences in one pass.  seq_ids, ctx_len, k,
 * accept_len and next_token are host arrays of n_seq entries; drafts holds the
 * sequences' draft tokens back to back (k[0] ids of seq_ids[0], then k[1] of
 * seq_ids[1], ...).  Sequence i is handled exactly as amusd_verify(ctx_len[i],
 * its drafts, k[i]) would.  Errors: ARG (n_seq outside [1,16], a repeated or
 * bad sequence id, k[i] < 1, sum of k above max_k), RANGE, CAPACITY, TOKEN,
 * STATE; on error no sequence has changed. */
int amusd_verify_batch(amusd_model *m, int32_t n_seq, const int32_t *seq_ids, const int32_t *ctx_len,
                       const int32_t *k, const int32_t *drafts, int32_t *accept_len, int32_t *next_token);

/* amusd_draft_step for n_seq distinct sequences in one pass (one row each);
 * tokens_out[i] is sequence seq_ids[i]'s new p_next.  Errors: ARG (n_seq above
 * max_k or 16, repeated or bad id), STATE, CAPACITY. */
int amusd_draft_step_batch(amusd_model *m, int32_t n_seq, const int32_t *seq_ids, int32_t *tokens_out);

/* ---- drivers on the same steps -------------------------------------------------------------- */

/* Algorithm 1 as a whole: DraftProcess and VerifyProcess run concurrently on
 * two host threads, each driving its model on that model's stream, sharing
 * the draft buffer D, the verified buffer V, p_d, p_v and the rollback flag R
 * (single writer each).  Both caches must be empty or are reset; both are
 * first filled with the prompt.  Writes the n_new tokens that follow the
 * prompt to out_tokens (host) - by construction the verify model's greedy
 * continuation.  A verify window is min(available drafts, k_max) rows.
 * stats may be NULL.  The two models must share the vocabulary. */
int amusd_generate_async(amusd_model *draft, amusd_model *verify, const int32_t *prompt, int32_t n_prompt,
                         int32_t n_new, int32_t k_max, int32_t *out_tokens, amusd_loop_stats *stats);

/* Synchronous speculative decoding (the paper's baseline, Section III-A):
 * alternate a draft phase of k_max-1 draft steps and one verify pass, on one
 * host thread. */
int amusd_generate_sync(amusd_model *draft, amusd_model *verify, const int32_t *prompt, int32_t n_prompt,
                        int32_t n_new, int32_t k_max, int32_t *out_tokens, amusd_loop_stats *stats);

/* Plain autoregressive decoding with one model (the paper's other baseline):
 * prefill, then one single-row pass per token. */
int amusd_generate_greedy(amusd_model *m, const int32_t *prompt, int32_t n_prompt, int32_t n_new,
                          int32_t *out_tokens, amusd_loop_stats *stats);

/* ---- inspection (tests, benchmark) ---------------------------------------------------------- */

int amusd_set_option(amusd_model *m, int32_t option, int32_t value);

/* fp32 logits of the last pass, rows 0..rows-1, to host memory [rows, vocab]
 * (a batched pass keeps its sequences' rows back to back, in call order).
 * Needs AMUSD_OPT_KEEP_LOGITS = 1 before that pass.  Errors: ARG, STATE. */
int amusd_get_logits(amusd_model *m, float *out, int32_t rows);

/* g[0..rows) of the last pass (arg-max token of each row) to host memory. */
int amusd_get_greedy(amusd_model *m, int32_t *out, int32_t rows);

/* Device time of the last pass in milliseconds, from HIP events recorded on
 * the model's stream around the pass's kernels (first launch to last end). */
int amusd_last_pass_ms(amusd_model *m, float *ms);

/* Accumulated device time (HIP events on the model's stream, one pair around
 * every launch of the stage selected with AMUSD_OPT_TIME_STAGE) and number of
 * launches since the option was last set.  Also reports the algorithmic bytes
 * one such launch reads from device memory (weights of the stage for one
 * layer; for the attention stage the cache rows of the last pass). */
int amusd_stage_time(amusd_model *m, double *total_ms, int64_t *launches, int64_t *bytes_per_launch);

/* Copies rows [pos0, pos0+n) of layer `layer`'s cached keys (which=0) or
 * values (which=1) of sequence 0 to host fp32 [n_kv_heads, n, head_dim], undoing the
 * library's internal layout.  Test hook. */
int amusd_get_kv(amusd_model *m, int32_t layer, int32_t which, int32_t pos0, int32_t n, float *out);
/* The same for sequence `seq`. */
int amusd_seq_get_kv(amusd_model *m, int32_t seq, int32_t layer, int32_t which, int32_t pos0, int32_t n, float *out);

/* Bytes of weights one pass streams from device memory, and bytes of cache it
 * reads at the given context and k (the algorithmic traffic used for roofline
 * accounting). */
int64_t amusd_weight_bytes_per_pass(const amusd_model *m);
int64_t amusd_kv_bytes_per_pass(const amusd_model *m, int32_t ctx_len, int32_t k);

/* Plain device-to-device copy kernel of `bytes` bytes (a multiple of 16; both
 * pointers device memory, 16-byte aligned) on the given HIP stream.  Not part
 * of the method: a kernel of exactly known traffic (bytes read + bytes written)
 * against which profiler byte counters are calibrated. */
int amusd_calibration_copy(void *dst, const void *src, int64_t bytes, void *hip_stream);

/* Enqueues n_kernels bare streaming kernels on the given HIP stream, each reading bytes_per_kernel bytes (a
 * positive multiple of 2 MiB: 256 workgroups x 512 threads x 16 bytes) from `buf` (device memory of buf_bytes >=
 * bytes_per_kernel; successive kernels take successive regions, wrapping around) with the load pattern of the
 * projection stages and none of their arithmetic, and each depending on the one before.  scratch: 3 KiB of
 * zeroed device memory.  Not part of the method: it measures what a chain of dependent kernels of a given size
 * can reach on the machine, the yardstick the stage timings are held against.  The caller times the stream. */
int amusd_calibration_chain(const void *buf, int64_t buf_bytes, int64_t bytes_per_kernel, int32_t n_kernels,
                            void *scratch, void *hip_stream);

/* Static description of a code; amusd_last_error gives the calling thread's
 * most recent detailed message (e.g. the HIP error string). */
const char *amusd_strerror(int code);
const char *amusd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* AMUSD_H */
