/*
 * flame_dso.h - C ABI of the request orchestrator in front of the GR forward (flame_gr.h).
 *
 * The paper's Dynamic Stream Orchestrator (Section 3.3): upstream services send one user at a time
 * with a varying number of candidates.  Instead of one dynamic-shape engine, a set of executors is
 * built ahead of time for a few candidate-count profiles: an executor owns pre-allocated input and
 * output buffers, a stream, and the forward of its explicit shapes captured as graphs.  Free
 * executors wait in an index queue.  A request is split by candidate count in descending profile
 * order, every chunk is handed to a free executor, and the executor's index returns to the queue
 * once its work has completed.  Inputs travel through pinned host buffers that belong to the
 * executors (the "pinned data transfer" of Section 3.1), so a chunk's upload overlaps the compute
 * of the chunks before it on other streams.
 *
 * (Mode 1 of three; modes 0 and 2 are described at flame_dso_config.)
 * Here an executor is a flame_gr handle with one captured HIP graph per profile (flame_gr_capture,
 * one slot each, all bound to the executor's one set of buffers), a pinned input buffer, a device
 * input buffer, a device and a pinned score buffer, a stream and an event.  Because every executor
 * can replay every profile there is one queue, not one per profile: a burst of one candidate count
 * never waits while executors of another profile idle.  Every chunk re-runs the user's history (as
 * the split of Section 3.3 does).
 *
 * Conventions as in flame_gr.h: 0 or a negative flame_gr_status is returned, nothing throws.  All
 * embedding and score pointers of this header are HOST pointers (any host memory).  One host thread
 * drives an orchestrator; the library starts no threads of its own.
 */
#ifndef FLAME_DSO_H
#define FLAME_DSO_H

#include <stdint.h>

#include "flame_gr.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct flame_dso flame_dso_t; /* opaque */

typedef struct {
  int32_t hist_len;              /* L: every request brings exactly this many history items (the
                                    explicit shape of every executor) */
  int32_t n_profiles;            /* 1..16 */
  const int32_t *profiles;       /* HOST [n_profiles]: candidate counts, strictly ascending, >= 1;
                                    at most FLAME_GR_MAX_GRAPHS when explicit_shapes = 1 */
  int32_t n_executors;           /* 1..256 executors (each with its own stream and buffers) */
  int32_t explicit_shapes;       /* 1: the executors described above (graph replay, a chunk with fewer
                                       candidates than its profile is padded with rows whose scores are
                                       dropped).
                                    0: the baseline the paper calls implicit shape: the same pool and
                                       buffers, but every executor takes any candidate count up to the
                                       largest profile and runs the dynamic-shape flame_gr_forward
                                       (planned and launched kernel by kernel per request); a request
                                       is split only above the largest profile.
                                    2: jagged micro-batches, the re-design that jagged kernels allow: requests
                                       of any candidate counts gather in an executor's pinned buffer and are
                                       scored by ONE jagged flame_gr_forward when max_batch requests have
                                       gathered, when the buffer is full, when a gathered ticket is waited
                                       for, or on flame_dso_flush / flame_dso_drain.  No padding, no
                                       profiles (they only bound the buffer: max_batch x largest profile
                                       candidate rows); kernels see batches large enough to fill the chip */
  int32_t max_batch;             /* mode 2 only: 1..256 requests per micro-batch */
} flame_dso_config;

/* Build all executors on the current device: model->max_requests / max_total_tokens / n_streams /
 * kv_cache are ignored (each executor is sized for its own shape).  `weights` are device pointers
 * as in flame_gr.h; their values are frozen into the executors here (create again after a change).
 * Errors: INVALID_ARGUMENT, UNSUPPORTED (model shape), HIP_ERROR.  *out = NULL on failure; the
 * message is available from flame_dso_last_error(NULL). */
int flame_dso_create(const flame_gr_config *model, const flame_gr_weights *weights,
                     const flame_dso_config *cfg, flame_dso_t **out);

/* Enqueue one request.
 *   history_emb  HOST [hist_len][d] of the model dtype
 *   cand_emb     HOST [n_cand][d]
 *   n_cand       >= 1
 *   scores       HOST fp32 [n_cand]: filled by the flame_dso_wait that retires the request (or by a
 *                later submit that needs one of its executors); must stay valid until then
 *   ticket       receives a handle for flame_dso_wait
 * The call copies the embeddings into the executors' pinned buffers (both host arrays may be reused
 * when it returns), enqueues upload, forward and download on the executors' streams and returns
 * without waiting for the GPU, unless every executor is busy: then it first waits for the one that
 * was handed out earliest. */
int flame_dso_submit(flame_dso_t *dso, const void *history_emb, const void *cand_emb, int32_t n_cand,
                     float *scores, int64_t *ticket);

/* Mode 2 only: as flame_dso_submit for a request whose history has hist_len items, 0 <= hist_len <= the
 * hist_len of create (which then is the capacity per request of an executor's buffers): jagged kernels take
 * any mix of history lengths in one micro-batch.  UNSUPPORTED in modes 0 and 1, CAPACITY_EXCEEDED beyond
 * the capacity. */
int flame_dso_submit_jagged(flame_dso_t *dso, const void *history_emb, int32_t hist_len, const void *cand_emb,
                            int32_t n_cand, float *scores, int64_t *ticket);

/* Block until every chunk of `ticket` has completed and its scores are in the caller's array.
 * Waiting twice for a ticket, or for one already retired by executor reuse, returns at once. */
int flame_dso_wait(flame_dso_t *dso, int64_t ticket);

/* Mode 2: send the gathering micro-batch to the GPU now (no-op otherwise or when nothing gathers). */
int flame_dso_flush(flame_dso_t *dso);

/* Wait for everything submitted so far. */
int flame_dso_drain(flame_dso_t *dso);

/* Destroy the orchestrator (drains first).  NULL is a no-op. */
int flame_dso_destroy(flame_dso_t *dso);

const char *flame_dso_last_error(const flame_dso_t *dso);

/* Host-only: the routing rule.  Splits n_cand into chunks (profile, count) in descending profile
 * order: the largest profile is taken while at least that many candidates remain; a remainder r is
 * then either padded up to the smallest profile >= r or split further as (largest profile <= r) +
 * remainder, whichever costs less by the forward's cost model 10 N d^2 + 4 P d per chunk (N = rows,
 * P = allowed query-key pairs; every chunk repeats the history).  With explicit_shapes = 0 a chunk
 * is min(remaining, largest profile) candidates and its profile entry is -1.
 *   chunks  HOST [cap_chunks][2]: profile index, candidates taken by the chunk
 * Errors: INVALID_ARGUMENT, CAPACITY_EXCEEDED (cap_chunks too small; *n_chunks holds the need). */
int flame_dso_route(const int32_t *profiles, int32_t n_profiles, int32_t hist_len, int32_t d_model,
                    int32_t explicit_shapes, int32_t n_cand, int32_t *chunks, int32_t cap_chunks,
                    int32_t *n_chunks);

/* Counters since create: HOST int64 [4] = requests submitted, chunks dispatched, candidate rows
 * computed including padding, times a submit had to wait for a busy executor. */
int flame_dso_stats(const flame_dso_t *dso, int64_t *out);

#ifdef __cplusplus
}
#endif
#endif /* FLAME_DSO_H */
