/*
 * sled.h -- C ABI of the MI355X (gfx950) library for the server-side batched
 * verification step of SLED (arXiv 2506.09397).
 *
 * The paper's server queues verification requests from many edge devices, batches
 * them, runs ONE forward pass of a shared target LLM over every request's draft
 * tokens and applies the speculative-decoding acceptance rule (Sec. 3.1, Sec. 3.2,
 * Sec. 3.4).  This library is that step and nothing else:
 *
 *   sled_verify_batch   target logits for a ragged batch of requests, each scored on
 *                       top of its own cached context (Sec. 3.1: all drafts in a single
 *                       forward pass; Sec. 3.4 batching of heterogeneous devices)
 *   sled_accept         accepted-prefix length and one corrective / bonus token per
 *                       request (Eq. 1 and the resampling rule of Sec. 3.1; the
 *                       feedback message of Sec. 3.2)
 *   sled_kv_append      bring a request's context K/V into the server-side cache, or
 *                       commit the K/V of the tokens just accepted (the iterate-until-
 *                       done loop of Sec. 3.2)
 *   sled_prefill        (beyond the step) a request's prompt through the same kernels into
 *                       its cache
 *
 * General rules
 *   - Plain C.  Every function returns SLED_OK (0) or a negative error code; nothing
 *     throws or aborts.  sled_last_error() gives a message for the calling thread.
 *   - Pointers marked "dev" are device (HBM) pointers owned by the caller; the library
 *     never frees or keeps them beyond the work it enqueues.  Pointers marked "host"
 *     are ordinary host memory, read before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All device
 *     work is enqueued on it and the calls return without waiting for it, except where
 *     stated.  Calls that touch the same pool must be issued on one stream or be ordered
 *     by the caller.
 *   - The library owns what sits behind its handles: packed weights, the paged K/V pool.
 *   - Handles are not thread-safe; use one thread per handle or lock outside.
 *
 * Request layout.  Request i has L_i context tokens in the pool, one pending token (the
 * last committed token, whose K/V is not cached yet) and k_i draft tokens.  Its
 * n_i = k_i + 1 query tokens [pending, draft_1 .. draft_k] sit at positions
 * L_i .. L_i + k_i.  A batch packs all requests' query tokens back to back:
 * T = sum_i (k_i + 1) rows, request-major.  Logits row j of a request is the target
 * distribution of the token that follows its j-th query token: row j-1 judges draft j,
 * row k_i yields the bonus token.
 */
#ifndef SLED_H
#define SLED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SLED_API __attribute__((visibility("default")))

/* ---- status codes -------------------------------------------------------------- */
#define SLED_OK       0
#define SLED_EINVAL  (-1)   /* bad pointer, shape, range or unsupported configuration  */
#define SLED_ENOMEM  (-2)   /* page pool or request table exhausted, or allocation failed */
#define SLED_ESTATE  (-3)   /* call out of order (e.g. commit without a preceding verify) */
#define SLED_EHIP    (-4)   /* the HIP runtime reported an error                         */

/* ---- enums --------------------------------------------------------------------- */
#define SLED_F32   0        /* weights, activations and K/V stored as float32 */
#define SLED_BF16  1        /* stored as bfloat16; sums, softmax, residual stream, logits in float32 */

#define SLED_GREEDY 0       /* exact match against the target's argmax chain */
#define SLED_SAMPLE 1       /* speculative sampling, Eq. 1 */

/* tensor ids for sled_model_load; linear weights are [out_features, in_features] row-major */
#define SLED_T_EMBED    0   /* [vocab, d_model]                         (layer ignored) */
#define SLED_T_WQ       1   /* [n_q_heads*head_dim, d_model]                            */
#define SLED_T_WK       2   /* [n_kv_heads*head_dim, d_model]                           */
#define SLED_T_WV       3   /* [n_kv_heads*head_dim, d_model]                           */
#define SLED_T_WO       4   /* [d_model, n_q_heads*head_dim]                            */
#define SLED_T_WGATE    5   /* [d_ffn, d_model]                                         */
#define SLED_T_WUP      6   /* [d_ffn, d_model]                                         */
#define SLED_T_WDOWN    7   /* [d_model, d_ffn]                                         */
#define SLED_T_G_ATTN   8   /* [d_model] RMSNorm gain before attention                  */
#define SLED_T_G_MLP    9   /* [d_model] RMSNorm gain before the MLP                    */
#define SLED_T_G_FINAL 10   /* [d_model] final RMSNorm gain             (layer ignored) */
#define SLED_T_LM_HEAD 11   /* [vocab, d_model]                         (layer ignored) */
/* models with 8- or 4-bit weights (sled_model_set_weight_bits): SLED_T_SCALE + a matrix id names that matrix's
 * scales -- 8 bits: per-output-row, float32 [rows]; 4 bits: per row and block of 32 inputs, uint8 [rows, in / 32] */
#define SLED_T_SCALE  100

typedef struct sled_model  sled_model;
typedef struct sled_kvpool sled_kvpool;

/* LLaMA-family decoder (Sec. 4): pre-norm, RMSNorm, rotary embedding with the half-split
 * pairing (i, i + head_dim/2), grouped-query attention (query head h reads kv head
 * h / (n_q_heads/n_kv_heads)), SwiGLU, no biases, untied LM head. */
typedef struct sled_shape {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t dtype;        /* SLED_F32 or SLED_BF16 */
    float   rms_eps;
    float   rope_theta;
    int32_t page_size;    /* tokens per K/V page; must be 16 */
    int32_t k_max;        /* largest number of draft tokens in one request (<= 15) */
} sled_shape;

/* ---- model --------------------------------------------------------------------- */

/* Allocates device storage for all weights of `shape` in the library's packed layout.
 * Supported: SLED_BF16 with head_dim 128, d_model, d_ffn and n_q_heads*head_dim multiples
 * of 256, vocab a multiple of 32, (n_q_heads/n_kv_heads)*(k_max+1) <= 80; SLED_F32 with head_dim 64 or 128.
 * Errors: SLED_EINVAL (unsupported shape), SLED_ENOMEM. */
SLED_API int sled_model_create(const sled_shape* shape /*host*/, sled_model** out);

/* Repacks one tensor from the caller's row-major array `src` (dev, model dtype) into the
 * model.  `layer` in [0, n_layers) for per-layer tensors.  Asynchronous on `stream`; `src`
 * may be freed once the stream has passed this point.  Errors: SLED_EINVAL. */
SLED_API int sled_model_load(sled_model* m, int tensor_id, int layer, const void* src /*dev*/, void* stream);

/* bits = 8: the projection matrices (WQ .. WDOWN, LM_HEAD) are stored as 8-bit floats -- FP8 E4M3 in the OCP
 * encoding, which gfx950 widens to bf16 in hardware -- with one float32 scale per output row,
 * W[n][k] = fp8[n][k] * scale[n]: weight-only quantisation, the 8-bit point of the paper's bit-width sweep
 * (Sec. 4.3).  Activations, K/V cache and arithmetic stay as in a bf16 model (an FP8 value is exact in bf16; the
 * scale is applied to the float32 accumulator), so the weight stream halves and nothing else changes.
 * Call it right after sled_model_create, before any sled_model_load: the matrices' device storage is given back and
 * allocated anew at bits/8 bytes per weight (a 70B-shaped model takes 141, 71 or 37 GB), so whatever was loaded
 * before is lost, and after SLED_ENOMEM the model can only be destroyed.  The matrices are then loaded as FP8 bytes
 * [out, in] (dev) and their scales under SLED_T_SCALE + id.  NaN encodings are the caller's to avoid.  bf16
 * models whose projection widths are multiples of 64 only.  bits = 16 restores the default.
 * bits = 4: the 4-bit point of the same sweep, in the MXFP4 arrangement -- FP4 E2M1 codes (0, 0.5, 1, 1.5, 2, 3, 4, 6
 * and their negatives; bit 3 is the sign), two per byte with the even input index in the low nibble, and one
 * E8M0 scale byte e per output row and block of 32 inputs, W[n][k] = fp4[n][k] * 2^(e[n][k / 32] - 127).  gfx950
 * widens two codes to bf16 and applies the block scale in one instruction, exactly; the rest as for 8 bits.
 * Matrices are loaded as uint8 [out, in / 2] (dev), scales under SLED_T_SCALE + id as uint8 [out, in / 32]; scale
 * bytes must lie in 1 .. 254 (0 reads as a zero scale, 255 is NaN in E8M0).  Input widths multiples of 32.
 * Errors: SLED_EINVAL, SLED_ENOMEM. */
SLED_API int sled_model_set_weight_bits(sled_model* m, int bits);

/* on != 0: the logits of a request no longer depend, not even in the last bit, on which other requests share its
 * batch or on how many rows the batch has -- so a greedy text is the same however the server happens to batch it.
 * The projections then keep one workgroup shape at every batch size and attention sums a request's keys in fixed
 * runs of 768 tokens instead of runs balanced over the CUs for the batch at hand; both cost speed on large or
 * uneven batches.  Set it before sizing workspaces (sled_verify_workspace_bytes depends on it).  Default: off. */
SLED_API int sled_model_set_batch_invariant(sled_model* m, int on);

SLED_API int sled_model_destroy(sled_model* m);

/* ---- paged K/V pool -------------------------------------------------------------- */

/* A pool of `n_pages` pages of 16 tokens (all layers, K and V) shared by up to
 * `max_requests` open requests.  The paper leaves server-side K/V caching to future work
 * (Sec. 5); keeping each device's context resident between rounds is this library's
 * reading of "each request carries its context".  K is stored already rotated. */
SLED_API int sled_kvpool_create(const sled_model* m, int64_t n_pages, int max_requests, sled_kvpool** out);

/* Opens an empty request (L = 0) and returns its id.  Host bookkeeping only: nothing is enqueued and nothing is
 * waited for (the device-side length of the slot is reset by the first append, verify or prefill that names the
 * request, on that call's stream).  Errors: SLED_ENOMEM. */
SLED_API int sled_kvpool_open(sled_kvpool* p, int* req_id /*host out*/);

/* Returns the request's pages to the pool.  Host bookkeeping only, no wait: the pages may be handed to another
 * request at once, which is safe because all calls on one pool are issued on one stream (or ordered by the caller),
 * so whatever still reads the pages runs before whatever writes them next.  A verify of this request that has
 * not been committed is dropped.  Errors: SLED_EINVAL (unknown id). */
SLED_API int sled_kvpool_close(sled_kvpool* p, int req_id);

/* The one call of the pool that waits: synchronises `stream`, then writes the exact committed context length of
 * each listed request to lens (host out, B ints) and tightens the host-side page accounting to it.  Rows staged by
 * a verify that is not committed yet keep their pages, so the call may come between a verify and its commit.
 * No other call needs it: a commit sends the exact lengths back to the host behind itself, and a later call on
 * the pool picks them up, once they have arrived, without waiting. */
SLED_API int sled_kvpool_lengths(sled_kvpool* p, int B, const int* req_ids /*host*/, int* lens /*host out*/, void* stream);

SLED_API int sled_kvpool_destroy(sled_kvpool* p);

/* Two uses, chosen by accept_len:
 *
 * (1) accept_len == NULL: append n_tokens[i] tokens of externally produced K/V to request
 *     req_ids[i].  k_src[i] and v_src[i] (host arrays of B dev pointers) each point to
 *     [n_layers, n_tokens[i], n_kv_heads, head_dim] in the model dtype; K already rotated
 *     for positions L_i .. L_i + n_tokens[i] - 1.  L_i grows by n_tokens[i].
 *
 * (2) accept_len != NULL (dev, B int32, as written by sled_accept): commit the K/V that the
 *     last sled_verify_batch staged for these requests: the pending token and the first
 *     accept_len[i] drafts become context, L_i += accept_len[i] + 1.  No data moves; the
 *     rejected tokens' slots are overwritten by the next verify.  n_tokens, k_src, v_src
 *     are ignored.  The requests must be among those of the last verify, each at most once
 *     (SLED_ESTATE otherwise); they may be committed in several calls, accept_len[i] always belonging
 *     to req_ids[i] of the call at hand.  Page accounting on the host assumes every staged row was
 *     accepted until the exact lengths, copied back asynchronously behind the commit, have arrived.
 *
 * Errors: SLED_EINVAL, SLED_ENOMEM (no free page), SLED_ESTATE. */
SLED_API int sled_kv_append(sled_kvpool* p, int B, const int* req_ids /*host*/, const int* n_tokens /*host*/,
                   const void* const* k_src /*host array of dev ptrs*/, const void* const* v_src,
                   const int32_t* accept_len /*dev or NULL*/, void* stream);

/* The way out of the cache (sled_kv_append with k_src/v_src is the way in): copies the K/V of positions
 * first_token .. first_token + n_tokens - 1 of a request to k_dst and v_dst (dev, each
 * [n_layers, n_tokens, n_kv_heads, head_dim] in the model dtype, K rotated as stored).  Positions may reach past the
 * committed length into the rows a verify has staged (that is how a caller looks at what a step wrote), but not past
 * the request's pages.  For moving a device's context to another server, and for inspection.  Asynchronous on
 * `stream`.  Errors: SLED_EINVAL. */
SLED_API int sled_kv_read(sled_kvpool* p, int req_id, int first_token, int n_tokens, void* k_dst /*dev out*/,
                 void* v_dst /*dev out*/, void* stream);

/* ---- the verification step ------------------------------------------------------- */

/* Bytes of scratch sled_verify_batch needs for batches of at most B_max requests, T_max
 * packed rows and ctx_tokens_max total context tokens (sum of L_i + k_i + 1). */
SLED_API size_t sled_verify_workspace_bytes(const sled_model* m, int B_max, int T_max, int64_t ctx_tokens_max);

/* Planning aids (host only: no GPU is touched, no model needed).  They return what a step will do, so that a caller
 * can size batches -- and so that the choices can be tested.
 *
 * sled_attention_partition: how the attention of a verification step (Sec. 3.4: requests of different lengths in one
 * batch) is cut into work items, one per workgroup.  n_pages[B]: the K/V pages each request holds in the step
 * (ceil((L_i + k_i + 1) / 16)).  Every (request, kv head) splits its pages evenly into ceil(n_pages[i] /
 * *pages_per_item) items; *n_items is their total.  The bound is chosen by playing the launch through (256 CUs, work
 * items handed out in order, longest requests first): at least 32 pages per item unless the request is shorter, at
 * most eight items per (request, kv head).  Models in batch-invariant mode use fixed runs of 48 pages instead.
 *
 * sled_projection_slices: the number of K slices (partial sums that a row kernel or the attention prologue adds up)
 * a projection of n_out outputs over n_in inputs runs with in a step of T packed rows of a bf16 model, and the most it
 * may ever use (which sizes the workspace).  n_out a multiple of 32, n_in of 256. */
SLED_API int sled_attention_partition(int n_kv_heads, int B, const int* n_pages /*host*/, int* pages_per_item /*host out*/,
                             int* n_items /*host out*/);
SLED_API int sled_projection_slices(int n_out, int n_in, int T, int* slices /*host out*/, int* max_slices /*host out*/);

/* One batched verification forward.
 *   req_ids[B], k[B]   host; 0 <= k[i] <= k_max (k[i] = 0 is a plain decode step); a request
 *                      may appear only once in a batch
 *   tokens[T]          dev int32, packed [pending, draft_1..draft_k] per request; ids outside
 *                      [0, vocab) are clamped into range
 *   logits[T, vocab]   dev float32 out, row-major, row order = tokens order
 *   workspace          dev scratch of at least sled_verify_workspace_bytes(...) bytes,
 *                      256-byte aligned; contents are undefined afterwards
 * Stages the new tokens' K/V in the requests' tail slots (positions L_i .. L_i + k_i) but does
 * not change L_i: a verify that is never committed leaves the pool logically unchanged and can
 * simply be issued again (the retry of Sec. 3.3).  Results for a request do not depend on the
 * other requests in the batch.
 * Errors: SLED_EINVAL (bad k, unknown or duplicate request, small workspace), SLED_ENOMEM
 * (no free page for the staged tokens). */
SLED_API int sled_verify_batch(sled_model* m, sled_kvpool* p, int B, const int* req_ids /*host*/, const int* k /*host*/,
                      const int32_t* tokens /*dev*/, float* logits /*dev*/,
                      void* workspace /*dev*/, size_t workspace_bytes, void* stream);

/* Context ingest through the target model itself: runs n_tokens prompt tokens of ONE request through the
 * same kernels as the verification step, on top of whatever the request has cached, writes their K/V into the
 * request's pages and commits them (L += n_tokens).  This is how a device's prompt p^n reaches the server-side
 * cache (Sec. 3.2: the tokenised prompt is what a device holds before it drafts); the other way in is
 * sled_kv_append with externally produced K/V.
 *   tokens[n_tokens]     dev int32, the tokens at positions L .. L + n_tokens - 1
 *   logits_last[vocab]   dev float32 out or NULL: logits of the last token, i.e. the target's distribution of
 *                        the first token to generate (the last prompt token may instead be kept back as the
 *                        pending token of the first verification)
 *   workspace            dev scratch, 256-byte aligned; any size that sled_verify_workspace_bytes returns for
 *                        B_max >= 1 will do: the prompt is cut into slices of as many blocks of k_max + 1 rows
 *                        as the workspace holds (larger workspace, fewer and larger slices)
 * Rows that an earlier, uncommitted sled_verify_batch staged for the request are overwritten (that request can then no
 * longer be committed; the other requests of that verify can).
 * Errors: SLED_EINVAL, SLED_ENOMEM (no free page). */
SLED_API int sled_prefill(sled_model* m, sled_kvpool* p, int req_id, int n_tokens, const int32_t* tokens /*dev*/,
                 float* logits_last /*dev or NULL*/, void* workspace /*dev*/, size_t workspace_bytes, void* stream);

/* Bytes of scratch sled_accept needs for T packed rows. */
SLED_API size_t sled_accept_workspace_bytes(int B, int T, int vocab);

/* Acceptance on given logits (usable without a model).
 *   mode          SLED_GREEDY: accept_len[i] = number of leading drafts equal to the argmax of
 *                 their judging row (lowest id on ties); out_token[i] = argmax of the row after
 *                 the last accepted draft.
 *                 SLED_SAMPLE: with p = softmax(logits_row / temperature), draft d judged by
 *                 that row is accepted iff u_acc * q(d) <= p(d) (probability min(1, p/q), Eq. 1);
 *                 at the first rejection out_token is drawn from max(0, p - q) normalised, by
 *                 inverse CDF over ascending token ids with u_smp[i]; if no draft is rejected
 *                 the bonus token is drawn the same way from the last row's p.
 *   k[B]          host
 *   logits[T,V]   dev float32; tokens[T] dev int32 (same packing as sled_verify_batch)
 *   draft_q       dev float32 [sum k, V] probabilities, one row per draft, request-major
 *                 (SLED_SAMPLE only; may be NULL for SLED_GREEDY, as may u_acc, u_smp)
 *   u_acc[sum k], u_smp[B]  dev float32 uniforms in [0, 1)
 *   accept_len[B], out_token[B]  dev int32 out; 0 <= accept_len[i] <= k[i]
 * Inputs must be finite.  Errors: SLED_EINVAL. */
SLED_API int sled_accept(int mode, int B, const int* k /*host*/, int vocab, float temperature,
                const float* logits /*dev*/, const int32_t* tokens /*dev*/,
                const float* draft_q /*dev*/, const float* u_acc /*dev*/, const float* u_smp /*dev*/,
                int32_t* accept_len /*dev out*/, int32_t* out_token /*dev out*/,
                void* workspace /*dev*/, size_t workspace_bytes, void* stream);

/* sled_accept for callers that cannot allocate device memory -- code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc: same arguments and results as sled_accept without the workspace.  The row
 * statistics go to a fixed 256 KiB array of device memory inside the library (one copy per GPU, held until the process
 * ends); the call allocates nothing and frees nothing.  Limit: T <= 16384 packed rows (the array holds 16384 row-segment
 * statistics, and T rows are scanned in at most ceil(8192 / T) segments each); beyond it the call fails with
 * SLED_EINVAL and sled_accept is the one to use.  All calls
 * on one GPU share that array and it keeps the last call's contents (nothing in it needs clearing): calls that
 * overlap on one GPU -- two streams, two threads -- race; issue them on one stream.  Errors: SLED_EINVAL, SLED_EHIP. */
SLED_API int sled_accept_static(int mode, int B, const int* k /*host*/, int vocab, float temperature,
                       const float* logits /*dev*/, const int32_t* tokens /*dev*/,
                       const float* draft_q /*dev*/, const float* u_acc /*dev*/, const float* u_smp /*dev*/,
                       int32_t* accept_len /*dev out*/, int32_t* out_token /*dev out*/, void* stream);

/* sled_accept in sampling mode with the draft distributions given sparsely: draft j's distribution q_j is
 * q_probs[j][i] on token q_ids[j][i] (i < q_m) and zero elsewhere.  This is exact, not an approximation, when
 * the device drew its draft from that very distribution -- e.g. from its top-q_m tokens renormalised -- because
 * Eq. 1 and the residual norm(max(0, p - q)) only ever need the q the draft was drawn from; it replaces V floats
 * per draft token on the uplink (Sec. 3.2 wants tokens, not activations, to travel) by q_m (id, probability) pairs.
 *   q_ids[sum k, q_m]     dev int32; distinct within a row; an id outside [0, vocab) marks padding
 *   q_probs[sum k, q_m]   dev float32; a probability of 0 marks padding
 *   q_rest[sum k]         dev float32 or NULL.  NULL: q is zero off the list (the device drafted from the listed
 *                         tokens alone, e.g. its top q_m renormalised).  Otherwise the pairs carry the drafter's
 *                         probabilities as they were and q_rest[j] is the mass of everything it did not list, which
 *                         both sides take to be spread evenly over the unlisted tokens:
 *                         q_j(v) = q_rest[j] / (vocab - listed) for v off the list.  Exact when the device drew
 *                         its draft from that reconstruction (top entries as they are, with probability q_rest an
 *                         unlisted token chosen uniformly); it distorts the drafter less than renormalising, so
 *                         more drafts are accepted, at the price of a second pass over the rejecting row.
 *   1 <= q_m <= 1024
 * Everything else as sled_accept (mode SLED_SAMPLE).  A drafted token that is not among its row's ids has the
 * probability of an unlisted token (0 without q_rest: it is then accepted, product form of Eq. 1). */
SLED_API int sled_accept_sparse(int B, const int* k /*host*/, int vocab, float temperature, const float* logits /*dev*/,
                       const int32_t* tokens /*dev*/, int q_m, const int32_t* q_ids /*dev*/, const float* q_probs /*dev*/,
                       const float* q_rest /*dev or NULL*/, const float* u_acc /*dev*/, const float* u_smp /*dev*/, int32_t* accept_len /*dev out*/,
                       int32_t* out_token /*dev out*/, void* workspace /*dev*/, size_t workspace_bytes, void* stream);

/* Confidence score of every row of a logits matrix: conf[t] = max_v softmax(logits[t] / temperature)[v], the quantity
 * the paper's dynamic drafting compares with its threshold c_th (Eq. 2: below it a device asks for verification,
 * at or above it drafts another token), and top[t] = the token that attains it (lowest id among ties).  One pass
 * over the logits, the same row scan that sled_accept starts with -- for a drafter that runs next to the server, or
 * to tell a device how sure the target was of the token it sent back.
 *   logits[T, V]  dev float32, finite;  conf[T] dev float32 out;  top[T] dev int32 out or NULL
 *   workspace     dev scratch, 256-byte aligned, sled_accept_workspace_bytes(1, T, vocab) bytes
 * Errors: SLED_EINVAL. */
SLED_API int sled_row_confidence(int T, int vocab, float temperature, const float* logits /*dev*/, float* conf /*dev out*/,
                        int32_t* top /*dev out or NULL*/, void* workspace /*dev*/, size_t workspace_bytes, void* stream);

/* ---- kernel timing (measurement aid) ---------------------------------------------- */

/* Kernel classes of one verification step. */
#define SLED_PROF_PROJ  0   /* projection GEMMs: QKV, O, gate/up, down, LM head (weight stream)    */
#define SLED_PROF_ATTN  1   /* verify attention over the paged K/V cache (K/V stream) + its merge  */
#define SLED_PROF_ROWS  2   /* row operators: embedding, split-K reduce, RMSNorm, rotary, K/V store */
#define SLED_PROF_N     3

/* With on != 0, every following sled_verify_batch on this model brackets each kernel launch with
 * HIP events on the caller's stream (this costs a few microseconds per launch: never leave it on
 * in a throughput run).  sled_profile_read waits for `stream`, adds up the elapsed time and the
 * number of launches of each class since the last read, writes them to ms[SLED_PROF_N] and
 * launches[SLED_PROF_N] (host out) and starts over.  Errors: SLED_EINVAL, SLED_EHIP. */
SLED_API int sled_profile_enable(sled_model* m, int on);
SLED_API int sled_profile_read(sled_model* m, void* stream, float* ms /*host out*/, int* launches /*host out*/);

/* ---- errors ---------------------------------------------------------------------- */
SLED_API const char* sled_strerror(int code);
SLED_API const char* sled_last_error(void);   /* message of the last failing call on this thread */

#ifdef __cplusplus
}
#endif
#endif /* SLED_H */
