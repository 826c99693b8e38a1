/*
 * flame_gr.h - C ABI of the MI355X (gfx950) generative-recommendation forward.
 *
 * The library scores a jagged batch of requests.  A request is one user history of L_i items
 * followed by M_i upstream candidate items ("single user, multiple items" per request: Section 1
 * and Section 3.2 of the FLAME paper); candidates are appended after the behaviour sequence
 * (Section 2.1) and a customised attention mask lets every candidate be scored in the same pass,
 * independently of the other candidates (Section 3.2).  The number of candidates differs from
 * request to request (Section 3.3), hence the offset arrays.  Inputs arrive as embeddings that
 * the CPU side has already looked up (Section 2.3: embedding look-up is CPU work), and no device
 * memory is allocated on the request path (Section 3.3: run-time allocation is what the
 * explicit-shape executors remove): every workspace is sized at flame_gr_create.
 *
 * Per layer the forward computes, for the merged token matrix X (history rows then candidate
 * rows of each request):
 *     [U V Q K] = silu(X W1^T + b1)
 *     O_r(head h) = sum over allowed keys c of silu(alpha <Q_r,K_c>_h + rab[l,h,bucket(p_r-p_c)]) V_c(h)
 *     X <- X + (LayerNorm(O) * U) W2^T + b2
 * and finally score_j = <w_s, X_{cand j}> + b_s.  A history row r may look at keys c <= r of its
 * own request; a candidate row may look at the whole history of its request and at itself.
 * History token t has position t, every candidate has position L_i.
 *
 * Conventions
 *   - Every function returns 0 on success or a negative flame_gr_status.  Nothing throws, aborts
 *     or prints.  flame_gr_last_error gives a message for the most recent failure on a handle
 *     (or, with a NULL handle, for the most recent failing flame_gr_create on this thread).
 *   - "device" pointers are HIP device memory on the device that was current at create time;
 *     "host" pointers are ordinary host memory.  Calls that enqueue work for a handle while another
 *     device is current are INVALID_ARGUMENT.  The caller owns every pointer it passes; the
 *     library owns the handle and its workspaces.
 *   - A handle is used by one host thread at a time.
 *   - With dtype FLAME_GR_BF16 every embedding and weight pointer must be 16-byte aligned (the kernels
 *     read 8 elements at a time; rows are multiples of 128 bytes because d % 64 == 0); a misaligned
 *     pointer is INVALID_ARGUMENT.
 *
 * Arithmetic of the two element types
 *   - FLAME_GR_F32: fp32 operands, fp32 accumulation, plain FMA kernels.
 *   - FLAME_GR_BF16 names the STORAGE type at this boundary: embeddings, W1, b1, ln_g, ln_b, W2, b2 and w_s
 *     arrive as bf16.  Inside, the matrix instructions run on IEEE binary16 (fp16) operands with fp32
 *     accumulation: embeddings and projection matrices are converted bf16 -> fp16 once, and the
 *     intermediates U, V, Q, K, O and the gated rows are stored as fp16 (11 significant bits against the 8 of
 *     bf16: the deep workloads need them).  The residual stream is held as TWO fp16 words per element, fp16(X) (which is
 *     also the projection's operand) and fp16(X - fp16(X)): 22 significant bits, added up in fp32.  LayerNorm
 *     statistics, SiLU / softmax arguments, bias adds and the score head are fp32; rab, temperature and b_s are fp32 inputs.
 *   - Range of that path.  Every fp16 store SATURATES at +-65504 (the largest finite fp16) instead of
 *     producing inf, so the workspaces always hold finite values: the tiled kernels multiply rows outside
 *     a query's mask by a zero weight, which is only harmless while those rows are finite.  Consequences
 *     the caller must know: bf16 inputs and activations beyond +-65504 in magnitude are clamped silently
 *     (the un-normalised SiLU attention sums up to L_i terms per output, so this is reachable with
 *     embeddings of order 1e2 and long histories; the scores then stay finite but are no longer the
 *     model's); weights below 2^-14 in magnitude become fp16 subnormals (absolute error <= 3e-8); and a
 *     NaN in an input is NOT propagated faithfully: the saturating store turns it into -65504, so the
 *     request that holds it gets finite but meaningless scores.  In no case does a value of one
 *     request, however large, change another request's scores.
 */
#ifndef FLAME_GR_H
#define FLAME_GR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct flame_gr flame_gr_t; /* opaque */

typedef enum {
  FLAME_GR_OK = 0,
  FLAME_GR_INVALID_ARGUMENT = -1, /* null pointer, bad offsets, bad configuration */
  FLAME_GR_CAPACITY_EXCEEDED = -2, /* batch larger than the capacity given at create */
  FLAME_GR_HIP_ERROR = -3,         /* a HIP runtime call failed */
  FLAME_GR_BAD_HANDLE = -4,        /* NULL or destroyed handle */
  FLAME_GR_UNSUPPORTED = -5        /* shape outside what the kernels are built for */
} flame_gr_status;

/* Element type of embeddings and weights at this boundary.  FLAME_GR_BF16 is a storage type: see "Arithmetic
 * of the two element types" above for what the kernels compute in (fp16 operands, fp32 accumulation) and
 * for the saturation at +-65504 that goes with it. */
typedef enum { FLAME_GR_F32 = 0, FLAME_GR_BF16 = 1 } flame_gr_dtype;

/* Attention weights of a query row r over its allowed keys c, with logit z_rc = alpha <Q_r,K_c> +
 * rab[l,h,bucket(p_r-p_c)]:
 *   FLAME_GR_ATTN_SILU     w_rc = silu(z_rc), pointwise (the block stated at the top of this header);
 *   FLAME_GR_ATTN_SOFTMAX  w_rc = softmax over c of z_rc / tau[l,h]: the softmax attention with an adaptive
 *                          temperature coefficient of the paper's own model (Section 2.1), tau > 0 a weight
 *                          per layer and head. */
typedef enum { FLAME_GR_ATTN_SILU = 0, FLAME_GR_ATTN_SOFTMAX = 1 } flame_gr_attn_kind;

/* Model shape and capacity.  Fixed for the life of a handle. */
typedef struct {
  int32_t n_layers;      /* >= 1 */
  int32_t d_model;       /* d; multiple of n_heads.  bf16: d % 64 == 0 and d/n_heads in {32,64} */
  int32_t n_heads;       /* H */
  int32_t n_buckets;     /* relative-position buckets: power of two, >= 2 */
  int32_t max_rel_dist;  /* D: power of two >= n_buckets/2; distances >= D share the last bucket */
  int32_t dtype;         /* flame_gr_dtype of embeddings and weights (rab and b_s are always fp32); with
                            FLAME_GR_BF16 the arithmetic inside is fp16 x fp16 -> fp32, stores saturate at +-65504 */
  float ln_eps;          /* LayerNorm epsilon; 0 selects 1e-6 */
  float attn_scale;      /* alpha; 0 selects 1.0 */
  int32_t max_requests;      /* capacity: requests per forward */
  int32_t max_total_tokens;  /* capacity: sum over requests of (L_i + M_i) per forward; FLAME_GR_BF16: the
                                padded workspace must stay below 2^26 rows, else UNSUPPORTED */
  int32_t max_seq_tokens;    /* 0 = unlimited; else a request with L_i + M_i above this is split by
                                candidates into chunks (largest first), each chunk re-running the
                                history, as the descending-size split of Section 3.3 does */
  int32_t n_streams;         /* 0 or 1 = everything on the caller's stream; k > 1 = requests are
                                partitioned into k cost-balanced groups that run on k internal
                                streams, joined to the caller's stream by events (Section 3.3) */
  int32_t attn_kind;         /* flame_gr_attn_kind */
  int32_t kv_cache;          /* 0 = one-pass forward only; 1 = also allocate a K and a V plane per layer so
                                that flame_gr_prefill and flame_gr_score can keep the history keys and
                                values of every layer */
  int32_t latency_mode;      /* 0 = kernels configured for throughput (batches that fill the chip);
                                1 = the MFMA attention kernel in its latency configuration, for handles that
                                serve one or a few requests per call: pairs of wavefronts split the keys of a
                                query tile, which halves the chain of dependent key tiles that bounds a small
                                batch's run time.  Partial sums are grouped differently: scores agree with
                                mode 0 to rounding (same error bars), not bit for bit.  No effect on fp32 handles */
  int32_t weights_static;    /* 0 = the caller may change the weight values between calls: every call derives its
                                operand copies (fp16 conversions, packed layouts, the bias table by distance) again;
                                1 = the caller promises that the device contents behind the weight pointers do not
                                change while the same pointers are passed: the copies are derived on the first call
                                and again only when a pointer of the weights struct differs from the previous call.
                                Saves a few small kernels per call, which counts for single requests and small batches */
} flame_gr_config;

/* Model weights: device pointers, caller-owned, read-only, element type = config.dtype unless
 * stated.  All matrices are row-major with the input feature contiguous (y = x W^T). */
typedef struct {
  const void *w1;     /* [n_layers][4*d][d]   output rows ordered U | V | Q | K */
  const void *b1;     /* [n_layers][4*d] */
  const float *rab;   /* [n_layers][n_heads][n_buckets]   fp32 */
  const void *ln_g;   /* [n_layers][d] */
  const void *ln_b;   /* [n_layers][d] */
  const void *w2;     /* [n_layers][d][d] */
  const void *b2;     /* [n_layers][d] */
  const void *w_s;    /* [d]   (may be NULL for flame_gr_forward_hidden) */
  float b_s;
  const float *temperature; /* [n_layers][n_heads] fp32, > 0; read only with FLAME_GR_ATTN_SOFTMAX */
} flame_gr_weights;

/* Create a handle on the current HIP device and allocate all workspaces for the given capacity.
 * Errors: INVALID_ARGUMENT (bad shape), UNSUPPORTED (shape the bf16 kernels do not cover),
 * HIP_ERROR (no device / out of memory).  *out is set to NULL on failure. */
int flame_gr_create(const flame_gr_config *cfg, flame_gr_t **out);

/* Score one jagged batch (the problem statement of Sections 1 and 3.2-3.3).
 *   weights          host struct of device pointers (see above)
 *   history_emb      device [sum L_i][d], rows of request i at history_offsets[i]..[i+1]
 *   history_offsets  HOST   int32 [n_requests+1], [0] == 0, non-decreasing
 *   cand_emb         device [sum M_i][d]
 *   cand_offsets     HOST   int32 [n_requests+1], [0] == 0, non-decreasing
 *   scores           device fp32 [sum M_i], written in cand_offsets order
 *   stream           hipStream_t (or NULL for the default stream)
 * The call validates and plans on the host, stages the plan through pinned memory, enqueues all
 * kernels and returns; scores are valid once `stream` has been synchronised.  L_i = 0, M_i = 0
 * and n_requests = 0 are legal.  Embedding pointers may be NULL when the matching total is 0.
 * The host offset arrays may be reused as soon as the call returns.  The device buffers must stay
 * alive and unmodified until the stream has passed the call.  Two forwards on one handle are
 * serialised by the library (the second waits for the first on the device).
 * Errors: BAD_HANDLE, INVALID_ARGUMENT (offsets not starting at 0 or decreasing, null pointers),
 * CAPACITY_EXCEEDED, HIP_ERROR.  On error nothing is enqueued. */
int flame_gr_forward(flame_gr_t *h, const flame_gr_weights *weights,
                     const void *history_emb, const int32_t *history_offsets,
                     const void *cand_emb, const int32_t *cand_offsets,
                     int32_t n_requests, float *scores, void *stream);

/* As flame_gr_forward, but instead of scores the call delivers the candidates' final residual rows
 * (the input of the score head): hidden is device fp32 [sum M_i][d] in cand_offsets order.  This is
 * what a stage above the block stack consumes, e.g. the fusion of several sub-sequence blocks
 * (flame_climber_head).  weights->w_s is not read.  UNSUPPORTED when max_seq_tokens splits a request. */
int flame_gr_forward_hidden(flame_gr_t *h, const flame_gr_weights *weights,
                            const void *history_emb, const int32_t *history_offsets,
                            const void *cand_emb, const int32_t *cand_offsets,
                            int32_t n_requests, float *hidden, void *stream);

/* Explicit-shape executor (Section 3.3): with the batch shape fixed, the whole forward is recorded
 * once into a HIP graph and later requests of that shape replay it with one call instead of one
 * launch per kernel.  A handle holds up to FLAME_GR_MAX_GRAPHS such graphs (`slot`), e.g. one per
 * candidate-count profile, all working in the handle's one set of workspaces.
 *
 * flame_gr_capture takes the arguments of flame_gr_forward: it synchronises the handle's earlier
 * work, uploads the plan into tables owned by the slot, derives the weight copies and records the
 * kernels; nothing is scored yet.  record_stream is the hipStream_t to record on (it is synchronised
 * and idle when the call returns; the legacy default stream cannot record) or NULL for a stream
 * that the handle creates for the purpose: a caller that counts its streams against the hardware
 * queues passes the stream it will replay on.  The graph is bound to the shape (the
 * offsets) and to the device buffers history_emb, cand_emb, scores and the weight pointers: the
 * caller refreshes the contents of history_emb / cand_emb in place before each replay.  The derived
 * weight copies belong to the handle and are rewritten by every capture and every eager call from the
 * weights passed there: keep to one set of weight values per handle, and capture again after changing
 * them.  This setup call may allocate (graph objects, the slot's tables, one stream);
 * flame_gr_replay does not.  Needs n_streams <= 1 (UNSUPPORTED otherwise) and at least one candidate.
 * Capturing into a used slot replaces its graph.
 *
 * flame_gr_replay enqueues the captured forward of `slot` on `stream` (hipStream_t or NULL); scores
 * are valid once the stream has been synchronised.  Calls on one handle are serialised on the device
 * like forwards.  INVALID_ARGUMENT if the slot holds no graph. */
#define FLAME_GR_MAX_GRAPHS 16
int flame_gr_capture(flame_gr_t *h, int32_t slot, const flame_gr_weights *weights,
                     const void *history_emb, const int32_t *history_offsets,
                     const void *cand_emb, const int32_t *cand_offsets,
                     int32_t n_requests, float *scores, void *record_stream);
int flame_gr_replay(flame_gr_t *h, int32_t slot, void *stream);

/* Two-stage scoring with a history key/value cache: the paradigm that Section 5 leaves for future
 * work, expecting it to pay for long contexts and larger models.  Because a history row never looks
 * at a candidate (mask of Section 3.2), the history part of every layer does not depend on the
 * candidates: flame_gr_prefill runs it once and keeps K and V of the history rows of every layer on
 * the device, and flame_gr_score then runs only the candidate rows against them, as often as the
 * caller has candidate batches for the same users.  Scores equal those of flame_gr_forward on the
 * same inputs bit for bit.  Needs a handle created with kv_cache = 1 and dtype FLAME_GR_BF16
 * (UNSUPPORTED otherwise).
 *
 * flame_gr_prefill
 *   history_emb, history_offsets, n_requests, stream   as in flame_gr_forward
 *   cand_capacity    HOST int32 [n_requests]: the largest candidate count that a later
 *                    flame_gr_score may bring for each request (rows are reserved for it; the
 *                    capacity checks of create apply to L_i + cand_capacity[i], and a request is
 *                    never split: L_i + cand_capacity[i] above a non-zero max_seq_tokens is
 *                    UNSUPPORTED)
 * The cache (K and V of every layer: 2 x n_layers x rows x d fp16 elements beside the one-pass
 * workspaces) belongs to the handle and is replaced by the next flame_gr_prefill; one-pass forwards
 * and replays on the same handle leave it intact. */
int flame_gr_prefill(flame_gr_t *h, const flame_gr_weights *weights, const void *history_emb,
                     const int32_t *history_offsets, const int32_t *cand_capacity, int32_t n_requests,
                     void *stream);

/* flame_gr_score: score candidates of the requests of the last flame_gr_prefill on this handle.
 *   weights          the same weights as at prefill (device contents unchanged since then)
 *   cand_emb         device [sum M_i][d]
 *   cand_offsets     HOST   int32 [n_requests+1], M_i <= cand_capacity[i]; M_i = 0 is legal
 *   n_requests       must equal that of the prefill
 *   scores           device fp32 [sum M_i]
 * May be called any number of times after one prefill; calls are serialised on the device like
 * forwards.  Errors: as flame_gr_forward, plus INVALID_ARGUMENT when no prefill is valid or
 * n_requests differs, CAPACITY_EXCEEDED when M_i exceeds its reserved capacity. */
int flame_gr_score(flame_gr_t *h, const flame_gr_weights *weights, const void *cand_emb,
                   const int32_t *cand_offsets, int32_t n_requests, float *scores, void *stream);

/* For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  flame_gr_forward_static is flame_gr_forward without a handle: the same kernels, with every
 * workspace (residual stream, activation planes, converted weights, bias and bucket tables, plan tables) carved
 * out of one static device array of FLAME_GR_STATIC_SCRATCH_MIB MiB that the library's code object holds on each
 * GPU it runs on until the process ends.  The call makes no hipMalloc / hipFree / hipHostMalloc, creates no
 * stream or event, issues no memcpy or memset: plan tables travel as kernel arguments, the bucket table is
 * computed on the device, and only kernels are enqueued on `stream` (so the call can be captured).  Host-side
 * planning uses the C++ heap, as in flame_gr_forward.
 *   cfg      as for flame_gr_create; the capacity fields (max_requests, max_total_tokens) are ignored: the
 *            capacity is the static array.  n_streams > 1 and kv_cache are UNSUPPORTED
 *   others   as for flame_gr_forward
 * A batch and model that need more than the array (flame_gr_static_scratch_bytes tells how much: about
 * 14*d bytes per padded row plus 10*d*d*n_layers bytes of converted weights with FLAME_GR_BF16) is
 * CAPACITY_EXCEEDED, with the two sizes in the message; nothing is enqueued then.  The device address of the
 * array is looked up once per device (hipGetSymbolAddress, with that device current) and kept.
 * All calls on one GPU share that GPU's array, which keeps the last call's contents: a call rewrites every row
 * it reads (and clears the spare rows behind its batch), so earlier calls cannot influence its scores, but two
 * calls that overlap in time on one GPU (different streams, or the same graph launched twice concurrently)
 * race on the array: serialise them.  Scores equal those of flame_gr_forward on the same inputs bit for bit.
 * Errors are reported like those of flame_gr_create: flame_gr_last_error(NULL) on the calling thread. */
#define FLAME_GR_STATIC_SCRATCH_MIB 64
int flame_gr_forward_static(const flame_gr_config *cfg, const flame_gr_weights *weights,
                            const void *history_emb, const int32_t *history_offsets,
                            const void *cand_emb, const int32_t *cand_offsets,
                            int32_t n_requests, float *scores, void *stream);

/* Bytes of the static array that flame_gr_forward_static needs for this model and a batch of `padded_rows`
 * workspace rows (the sum over requests of history and candidate lengths, each rounded up to a multiple of 64;
 * with max_seq_tokens splitting, over chunks).  HOST arithmetic only. */
int flame_gr_static_scratch_bytes(const flame_gr_config *cfg, int64_t padded_rows, int64_t *bytes);

/* Release the handle and its workspaces (synchronises the device work of the handle first).
 * NULL is a no-op that returns 0. */
int flame_gr_destroy(flame_gr_t *h);

/* Message for the last error on `h` (never NULL; "" if none).  The string is owned by the handle
 * (or by the thread, for h == NULL) and valid until the next call on it. */
const char *flame_gr_last_error(const flame_gr_t *h);

/* ------------------------------------------------------------------------------------------
 * Host-only helpers: integer planning logic, usable without a GPU.  They expose what the forward
 * uses internally so that it can be compared bit for bit with an independent implementation.
 * ------------------------------------------------------------------------------------------ */

/* bucket(delta) for delta = 0..max_rel_dist-1 into out[max_rel_dist] (HOST).  The near half of the
 * table is exact (delta < n_buckets/2 maps to itself); above it every octave up to max_rel_dist is
 * cut into 2^m equal sub-buckets, m the largest value such that all octaves fit in the far half. */
int flame_gr_host_bucket_table(int32_t n_buckets, int32_t max_rel_dist, int32_t *out);

/* Attention mask and bucket index of one request with L history items and M candidates (the mask
 * of Section 3.2), as HOST arrays of (L+M)*(L+M) entries, row = query, column = key:
 * mask 1 = allowed; bucket = bucket(p_r - p_c) on allowed pairs and -1 elsewhere (may be NULL). */
int flame_gr_host_mask(int32_t L, int32_t M, int32_t n_buckets, int32_t max_rel_dist,
                       uint8_t *mask, int32_t *bucket);

/* Plan of a batch without running it (all arrays HOST).
 *   tok_off   [n_requests+1]  start of each request in the merged token order (history_offsets +
 *                             cand_offsets), i.e. the logical, unpadded layout
 *   n_segments                number of scheduled segments (>= n_requests when requests are split)
 *   seg       [cap_segments][6] per segment: request, hist_len, cand_begin (first candidate of
 *                             the request handled by this segment), cand_len, row_start (first
 *                             row of the segment in the library's padded workspace), stream group
 * seg may be NULL to query n_segments only.  Errors as flame_gr_forward. */
int flame_gr_host_plan(const flame_gr_config *cfg, const int32_t *history_offsets,
                       const int32_t *cand_offsets, int32_t n_requests, int32_t *tok_off,
                       int32_t *n_segments, int32_t *seg, int32_t cap_segments);

/* Rows of every per-token workspace that flame_gr_create allocates for this configuration (HOST output):
 * max_total_tokens, plus room for padding each request's history and candidate part to multiples of 64
 * rows, rounded up to 256, plus 256 spare rows.  The spare rows are never part of a plan: a batch whose
 * padded rows (flame_gr_host_plan: row_start + padded lengths of the last segment) would reach into them
 * is CAPACITY_EXCEEDED, which can only happen when max_seq_tokens splits requests (every chunk repeats the
 * history).  Device memory per row with FLAME_GR_BF16: 14*d bytes (the residual as two
 * fp16 words, four fp16 planes, the attention output; 16*d for model widths whose output projection is not fused),
 * 28*d with FLAME_GR_F32, plus 4*d*n_layers with kv_cache. */
int flame_gr_host_workspace_rows(const flame_gr_config *cfg, int64_t *rows);

/* Plan of the two-stage path: as flame_gr_host_plan, but with candidate rows reserved for
 * cand_capacity[i] (HOST int32 [n_requests]) candidates per request, the layout that flame_gr_prefill
 * (with all candidate counts 0) and flame_gr_score (with the actual counts) build.  Segment rows and
 * stream groups depend on history_offsets and cand_capacity only; requests are never split. */
int flame_gr_host_plan_reserved(const flame_gr_config *cfg, const int32_t *history_offsets,
                                const int32_t *cand_offsets, const int32_t *cand_capacity,
                                int32_t n_requests, int32_t *n_segments, int32_t *seg,
                                int32_t cap_segments);

/* ------------------------------------------------------------------------------------------
 * Debug / parity exports (device work; not on the timed path).
 * ------------------------------------------------------------------------------------------ */

/* Select a layer (0-based) whose intermediates the next forwards keep, or -1 to stop capturing.
 * Allocates the capture buffers (this call may allocate; forward still does not). */
int flame_gr_debug_capture(flame_gr_t *h, int32_t layer);

/* After a forward with capture on and a stream synchronisation: copy one captured tensor of the
 * whole batch to HOST fp32 [sum(L_i+M_i)][d], rows in merged token order (request by request,
 * history then candidates; padding rows removed).  which: 0=U 1=V 2=Q 3=K 4=O (attention output
 * before LayerNorm) 5=X (residual stream after the layer).  Only valid if no request was split. */
int flame_gr_debug_stage(flame_gr_t *h, int32_t which, float *host_out);

/* Evaluate on the device the mask and bucket of one request of shape (L, M); HOST outputs as
 * flame_gr_host_mask.  This runs a small kernel of its own: it shares the visible-history rule and the
 * bucket table with the attention kernels, not their tile-level masking (which key tiles a wavefront
 * skips, where it applies the per-element predicate).  That logic is verified separately, by counting the
 * visible keys per row through the attention kernels' output with indicator values. */
int flame_gr_debug_device_mask(flame_gr_t *h, int32_t L, int32_t M, uint8_t *mask, int32_t *bucket);

/* Per-kernel timing for measurements.  With enable != 0 every kernel launch of the following
 * forwards is bracketed by HIP events on the stream it is launched on (this serialises nothing but
 * adds event overhead, so leave it off when timing whole forwards). */
int flame_gr_debug_profile(flame_gr_t *h, int32_t enable);

/* Summed milliseconds and launch counts, by kernel kind, of all forwards since profiling was
 * enabled or last read: HOST arrays of 7 entries in the order assemble, bias expansion, UVQK
 * projection, attention, LayerNorm-gate, output projection, score head.  Waits for the last forward
 * to finish, then resets the sums. */
int flame_gr_debug_profile_read(flame_gr_t *h, float *ms_by_kind, int32_t *launches_by_kind);

#ifdef __cplusplus
}
#endif
#endif /* FLAME_GR_H */
