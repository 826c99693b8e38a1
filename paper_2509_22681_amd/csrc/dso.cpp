// Request orchestrator (flame_dso.h): explicit-shape executors with captured graphs, an executor
// index queue, descending-size split routing, pinned staging (Sections 3.1 and 3.3 of the paper).
//
// Three modes: explicit shapes (one captured graph per profile on every executor), implicit shapes (the paper's
// baseline: eager dynamic-shape forward per request), and jagged micro-batches (several pending requests of any
// candidate counts scored by one jagged forward: what the jagged kernels make possible in place of shape
// profiles).
//
// Single host thread, no threads of its own: completion is tracked with one event per executor,
// and an executor's index goes back to the queue when its event is found complete (on wait, drain,
// or when a submit finds the queue empty).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <deque>
#include <new>
#include <string>
#include <vector>

#include "../../include/flame_dso.h"

namespace {

constexpr uint32_t kDsoMagic = 0x464c4453u;  // "FLDS"
thread_local std::string g_dso_create_error;

struct Pending { int64_t ticket = -1; float *dst = nullptr; int32_t m = 0; };

struct Executor {
  flame_gr_t *h = nullptr;
  int32_t cap = 0;          // candidate rows of the buffers (largest profile x requests per batch)
  int32_t n_req = 0, n_cand = 0, n_hist = 0;   // jagged mode: requests, candidate rows and history rows gathered so far
  std::vector<Pending> batch;             // jagged mode: what the gathered requests are owed (reserved at create)
  std::vector<int32_t> hoff, coff;        // jagged mode: offsets of the gathered batch (reserved at create)
  hipStream_t stream = nullptr;
  hipEvent_t done = nullptr;
  char *pin_in = nullptr, *dev_in = nullptr;
  float *dev_scores = nullptr, *pin_scores = nullptr;
  bool busy = false;
  Pending pending;
};

// cost of one chunk of p candidates behind a history of L items (the planner's model)
int64_t chunk_cost(int64_t L, int64_t p, int64_t d) {
  const int64_t N = L + p, P = L * (L + 1) / 2 + p * (L + 1);
  return 10 * N * d * d + 4 * P * d;
}

struct Piece { int32_t profile, count; };

// Remainder r < largest profile: pad up, or take the largest profile below and go on.
int64_t route_remainder(const std::vector<int32_t> &prof, int64_t L, int64_t d, int32_t r, std::vector<Piece> &out) {
  if (r <= 0) return 0;
  int up = -1, down = -1;
  for (int i = 0; i < (int)prof.size(); ++i) {
    if (prof[i] >= r && up < 0) up = i;
    if (prof[i] <= r) down = i;
  }
  std::vector<Piece> a, b;
  int64_t ca = -1, cb = -1;
  if (up >= 0) { a.push_back(Piece{up, r}); ca = chunk_cost(L, prof[up], d); }
  if (down >= 0 && prof[down] < r) {
    b.push_back(Piece{down, prof[down]});
    cb = chunk_cost(L, prof[down], d) + route_remainder(prof, L, d, r - prof[down], b);
  }
  const bool take_a = ca >= 0 && (cb < 0 || ca <= cb);
  const std::vector<Piece> &pick = take_a ? a : b;
  out.insert(out.end(), pick.begin(), pick.end());
  return take_a ? ca : cb;
}

int route(const std::vector<int32_t> &prof, int32_t L, int32_t d, bool explicit_shapes, int32_t M, std::vector<Piece> &out) {
  out.clear();
  const int32_t top = prof.back();
  if (!explicit_shapes) {
    for (int32_t r = M; r > 0; r -= std::min(r, top)) out.push_back(Piece{-1, std::min(r, top)});
    return 0;
  }
  int32_t r = M;
  while (r >= top) { out.push_back(Piece{(int32_t)prof.size() - 1, top}); r -= top; }
  route_remainder(prof, L, d, r, out);
  return 0;
}

bool profiles_ok(const int32_t *p, int32_t n) {
  if (!p || n < 1 || n > 16) return false;
  for (int i = 0; i < n; ++i)
    if (p[i] < 1 || (i && p[i] <= p[i - 1])) return false;
  return true;
}

}  // namespace

struct flame_dso {
  uint32_t magic = kDsoMagic;
  flame_gr_config model{};
  flame_gr_weights weights{};
  bool explicit_shapes = true;
  bool jagged = false;
  int32_t max_batch = 1;
  int gathering = -1;       // jagged mode: executor that collects the next batch, -1 if none
  int32_t L = 0, d = 0;
  size_t elt = 2;
  std::vector<int32_t> profiles;
  std::vector<Executor> ex;
  std::deque<int> free_q, busy_q;  // executor indices: free ones, and busy ones in the order they were handed out
  int64_t next_ticket = 1;
  int64_t stats[4] = {0, 0, 0, 0};
  std::string err;
};

namespace {

bool live(const flame_dso *d) { return d && d->magic == kDsoMagic; }

#define DSO_HIP(dso, expr)                                                   \
  do {                                                                       \
    hipError_t e_ = (expr);                                                  \
    if (e_ != hipSuccess) {                                                  \
      (dso)->err = std::string(#expr) + ": " + hipGetErrorString(e_);        \
      return FLAME_GR_HIP_ERROR;                                             \
    }                                                                        \
  } while (0)

// The executor's work is complete: deliver its scores and put its index back into the queue.
int retire(flame_dso *d, int idx) {
  Executor &e = d->ex[idx];
  if (!e.busy) return FLAME_GR_OK;
  DSO_HIP(d, hipEventSynchronize(e.done));
  if (d->jagged) {
    int32_t at = 0;
    for (const Pending &p : e.batch) {
      std::memcpy(p.dst, e.pin_scores + at, (size_t)p.m * sizeof(float));
      at += p.m;
    }
    e.batch.clear();
    e.n_req = e.n_cand = e.n_hist = 0;
  } else {
    std::memcpy(e.pending.dst, e.pin_scores, (size_t)e.pending.m * sizeof(float));
  }
  e.busy = false;
  e.pending = Pending();
  d->busy_q.erase(std::find(d->busy_q.begin(), d->busy_q.end(), idx));
  d->free_q.push_back(idx);
  return FLAME_GR_OK;
}

// Jagged mode: send the gathered batch of executor idx to the GPU as one jagged forward.
int flush(flame_dso *d, int idx) {
  Executor &e = d->ex[idx];
  d->gathering = -1;
  if (e.n_req == 0) { d->free_q.push_front(idx); return FLAME_GR_OK; }
  const size_t row = (size_t)d->d * d->elt;
  const size_t hist_region = (size_t)d->max_batch * d->L * row;
  e.busy = true;
  d->busy_q.push_back(idx);
  ++d->stats[1];
  d->stats[2] += e.n_cand;
  if (e.n_hist > 0) DSO_HIP(d, hipMemcpyAsync(e.dev_in, e.pin_in, (size_t)e.n_hist * row, hipMemcpyHostToDevice, e.stream));
  DSO_HIP(d, hipMemcpyAsync(e.dev_in + hist_region, e.pin_in + hist_region, (size_t)e.n_cand * row, hipMemcpyHostToDevice, e.stream));
  int rc = flame_gr_forward(e.h, &d->weights, e.dev_in, e.hoff.data(), e.dev_in + hist_region, e.coff.data(), e.n_req,
                            e.dev_scores, e.stream);
  if (rc) { d->err = std::string("executor: ") + flame_gr_last_error(e.h); return rc; }
  DSO_HIP(d, hipMemcpyAsync(e.pin_scores, e.dev_scores, (size_t)e.n_cand * sizeof(float), hipMemcpyDeviceToHost, e.stream));
  DSO_HIP(d, hipEventRecord(e.done, e.stream));
  return FLAME_GR_OK;
}

// A free executor, waiting for the one handed out earliest if none is free.
int acquire(flame_dso *d, int *idx) {
  if (d->free_q.empty()) {
    ++d->stats[3];
    int rc = retire(d, d->busy_q.front());
    if (rc) return rc;
  }
  *idx = d->free_q.front();
  d->free_q.pop_front();
  return FLAME_GR_OK;
}

void release_all(flame_dso *d) {
  for (Executor &e : d->ex) {
    if (e.stream) (void)hipStreamSynchronize(e.stream);
    if (e.h) (void)flame_gr_destroy(e.h);
    if (e.stream) (void)hipStreamDestroy(e.stream);
    if (e.done) (void)hipEventDestroy(e.done);
    if (e.pin_in) (void)hipHostFree(e.pin_in);
    if (e.pin_scores) (void)hipHostFree(e.pin_scores);
    (void)hipFree(e.dev_in);
    (void)hipFree(e.dev_scores);
  }
  d->ex.clear();
}

}  // namespace

extern "C" {

const char *flame_dso_last_error(const flame_dso_t *d) {
  if (!d) return g_dso_create_error.c_str();
  if (!live(d)) return "bad handle";
  return d->err.c_str();
}

int flame_dso_route(const int32_t *profiles, int32_t n_profiles, int32_t hist_len, int32_t d_model,
                    int32_t explicit_shapes, int32_t n_cand, int32_t *chunks, int32_t cap_chunks, int32_t *n_chunks) {
  if (!profiles_ok(profiles, n_profiles) || hist_len < 0 || d_model < 1 || n_cand < 0 || !n_chunks || cap_chunks < 0 ||
      (cap_chunks > 0 && !chunks))
    return FLAME_GR_INVALID_ARGUMENT;
  std::vector<Piece> pieces;
  route(std::vector<int32_t>(profiles, profiles + n_profiles), hist_len, d_model, explicit_shapes != 0, n_cand, pieces);
  *n_chunks = (int32_t)pieces.size();
  if ((int32_t)pieces.size() > cap_chunks) return FLAME_GR_CAPACITY_EXCEEDED;
  for (size_t i = 0; i < pieces.size(); ++i) { chunks[2 * i] = pieces[i].profile; chunks[2 * i + 1] = pieces[i].count; }
  return FLAME_GR_OK;
}

int flame_dso_create(const flame_gr_config *model, const flame_gr_weights *weights, const flame_dso_config *cfg,
                     flame_dso_t **out) {
  if (out) *out = nullptr;
  auto bad = [&](const char *m) { g_dso_create_error = m; return (int)FLAME_GR_INVALID_ARGUMENT; };
  if (!model || !weights || !cfg || !out) return bad("a pointer argument is NULL");
  if (!profiles_ok(cfg->profiles, cfg->n_profiles)) return bad("profiles must be 1..16 strictly ascending positive counts");
  if (cfg->hist_len < 0) return bad("hist_len < 0");
  if (cfg->n_executors < 1 || cfg->n_executors > 256) return bad("n_executors must be in [1, 256]");
  if (cfg->explicit_shapes < 0 || cfg->explicit_shapes > 2) return bad("explicit_shapes must be 0, 1 or 2");
  if (cfg->explicit_shapes == 1 && cfg->n_profiles > FLAME_GR_MAX_GRAPHS) return bad("more profiles than graph slots per executor");
  if (cfg->explicit_shapes == 2 && (cfg->max_batch < 1 || cfg->max_batch > 256)) return bad("max_batch must be in [1, 256]");
  flame_dso *d = new (std::nothrow) flame_dso();
  if (!d) { g_dso_create_error = "out of host memory"; return FLAME_GR_HIP_ERROR; }
  d->model = *model;
  d->weights = *weights;
  d->explicit_shapes = cfg->explicit_shapes == 1;
  d->jagged = cfg->explicit_shapes == 2;
  d->max_batch = d->jagged ? cfg->max_batch : 1;
  d->L = cfg->hist_len;
  d->d = model->d_model;
  d->elt = model->dtype == FLAME_GR_BF16 ? 2 : 4;
  d->profiles.assign(cfg->profiles, cfg->profiles + cfg->n_profiles);
  auto fail = [&](int code, const std::string &m) {
    g_dso_create_error = m;
    release_all(d);
    d->magic = 0;
    delete d;
    return code;
  };
#define CR(expr)                                                                                          \
  do {                                                                                                    \
    hipError_t e_ = (expr);                                                                               \
    if (e_ != hipSuccess) return fail(FLAME_GR_HIP_ERROR, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)
  const size_t row = (size_t)d->d * d->elt;
  d->ex.reserve(cfg->n_executors);
  for (int k = 0; k < cfg->n_executors; ++k) {
    d->ex.emplace_back();
    Executor &e = d->ex.back();
    e.cap = d->profiles.back() * d->max_batch;
    e.batch.reserve(d->max_batch);
    e.hoff.reserve(d->max_batch + 1);
    e.coff.reserve(d->max_batch + 1);
    flame_gr_config c = *model;
    c.max_requests = d->max_batch;
    c.max_total_tokens = d->max_batch * d->L + e.cap;
    c.max_seq_tokens = 0;
    c.n_streams = 0;
    c.kv_cache = 0;
    c.weights_static = 1;     // the orchestrator's weights are fixed at its creation
    int rc = flame_gr_create(&c, &e.h);
    if (rc) return fail(rc, std::string("executor create: ") + flame_gr_last_error(nullptr));
    const size_t in_bytes = ((size_t)d->max_batch * d->L + e.cap) * row;
    CR(hipStreamCreateWithFlags(&e.stream, hipStreamNonBlocking));
    CR(hipEventCreateWithFlags(&e.done, hipEventDisableTiming));
    CR(hipHostMalloc((void **)&e.pin_in, in_bytes, hipHostMallocDefault));
    CR(hipHostMalloc((void **)&e.pin_scores, (size_t)e.cap * sizeof(float), hipHostMallocDefault));
    CR(hipMalloc((void **)&e.dev_in, in_bytes));
    CR(hipMalloc((void **)&e.dev_scores, (size_t)e.cap * sizeof(float)));
    // padded candidate rows of a chunk are computed and dropped: they must hold finite values
    CR(hipMemset(e.dev_in, 0, in_bytes));
    CR(hipMemset(e.dev_scores, 0, (size_t)e.cap * sizeof(float)));
    if (d->explicit_shapes)
      for (int p = 0; p < cfg->n_profiles; ++p) {      // one graph per profile, all on this executor's buffers
        const int32_t hoff[2] = {0, d->L}, coff[2] = {0, d->profiles[p]};
        rc = flame_gr_capture(e.h, p, weights, e.dev_in, hoff, e.dev_in + (size_t)d->L * row, coff, 1, e.dev_scores, e.stream);
        if (rc) return fail(rc, std::string("executor capture: ") + flame_gr_last_error(e.h));
      }
    d->free_q.push_back(k);
  }
  CR(hipDeviceSynchronize());
#undef CR
  *out = d;
  return FLAME_GR_OK;
}

static int submit_request(flame_dso_t *d, const void *history_emb, int32_t hist_len, const void *cand_emb, int32_t n_cand,
                          float *scores, int64_t *ticket) {
  d->err.clear();
  auto bad = [&](const char *m) { d->err = m; return (int)FLAME_GR_INVALID_ARGUMENT; };
  if (n_cand < 1) return bad("n_cand must be >= 1");
  if (!cand_emb || !scores || !ticket) return bad("cand_emb, scores or ticket is NULL");
  if (hist_len > 0 && !history_emb) return bad("history_emb is NULL");
  std::vector<Piece> pieces;
  route(d->profiles, hist_len, d->d, d->explicit_shapes, n_cand, pieces);
  const int64_t t = d->next_ticket++;
  const size_t row = (size_t)d->d * d->elt;
  const size_t hist_bytes = (size_t)hist_len * row;
  int32_t taken = 0;
  ++d->stats[0];
  if (d->jagged) {
    // every piece (the whole request unless it exceeds the largest profile) joins the gathering batch
    const size_t hist_region = (size_t)d->max_batch * d->L * row;
    for (const Piece &pc : pieces) {
      if (d->gathering >= 0 && d->ex[d->gathering].n_cand + pc.count > d->ex[d->gathering].cap) {
        int rc = flush(d, d->gathering);
        if (rc) return rc;
      }
      if (d->gathering < 0) {
        int rc = acquire(d, &d->gathering);
        if (rc) return rc;
        Executor &g = d->ex[d->gathering];
        g.hoff.assign(1, 0);
        g.coff.assign(1, 0);
      }
      Executor &e = d->ex[d->gathering];
      if (hist_bytes) std::memcpy(e.pin_in + (size_t)e.n_hist * row, history_emb, hist_bytes);
      std::memcpy(e.pin_in + hist_region + (size_t)e.n_cand * row, (const char *)cand_emb + (size_t)taken * row, (size_t)pc.count * row);
      e.batch.push_back(Pending{t, scores + taken, pc.count});
      ++e.n_req;
      e.n_cand += pc.count;
      e.n_hist += hist_len;
      e.hoff.push_back(e.n_hist);
      e.coff.push_back(e.n_cand);
      taken += pc.count;
      if (e.n_req == d->max_batch) {
        int rc = flush(d, d->gathering);
        if (rc) return rc;
      }
    }
    *ticket = t;
    return FLAME_GR_OK;
  }
  for (const Piece &pc : pieces) {
    int idx;
    {
      int rc = acquire(d, &idx);
      if (rc) return rc;
    }
    Executor &e = d->ex[idx];
    const int32_t m = pc.count;
    if (hist_bytes) std::memcpy(e.pin_in, history_emb, hist_bytes);
    std::memcpy(e.pin_in + hist_bytes, (const char *)cand_emb + (size_t)taken * row, (size_t)m * row);
    e.busy = true;
    e.pending = Pending{t, scores + taken, m};
    d->busy_q.push_back(idx);
    ++d->stats[1];
    d->stats[2] += d->explicit_shapes ? d->profiles[pc.profile] : m;
    DSO_HIP(d, hipMemcpyAsync(e.dev_in, e.pin_in, hist_bytes + (size_t)m * row, hipMemcpyHostToDevice, e.stream));
    int rc;
    if (d->explicit_shapes) {
      rc = flame_gr_replay(e.h, pc.profile, e.stream);
    } else {
      const int32_t hoff[2] = {0, d->L}, coff[2] = {0, m};
      rc = flame_gr_forward(e.h, &d->weights, e.dev_in, hoff, e.dev_in + hist_bytes, coff, 1, e.dev_scores, e.stream);
    }
    if (rc) { d->err = std::string("executor: ") + flame_gr_last_error(e.h); return rc; }
    DSO_HIP(d, hipMemcpyAsync(e.pin_scores, e.dev_scores, (size_t)m * sizeof(float), hipMemcpyDeviceToHost, e.stream));
    DSO_HIP(d, hipEventRecord(e.done, e.stream));
    taken += m;
  }
  *ticket = t;
  return FLAME_GR_OK;
}

int flame_dso_submit(flame_dso_t *d, const void *history_emb, const void *cand_emb, int32_t n_cand, float *scores,
                     int64_t *ticket) {
  if (!live(d)) return FLAME_GR_BAD_HANDLE;
  return submit_request(d, history_emb, d->L, cand_emb, n_cand, scores, ticket);
}

int flame_dso_submit_jagged(flame_dso_t *d, const void *history_emb, int32_t hist_len, const void *cand_emb, int32_t n_cand,
                            float *scores, int64_t *ticket) {
  if (!live(d)) return FLAME_GR_BAD_HANDLE;
  if (!d->jagged) { d->err = "histories of other lengths need the jagged micro-batch mode"; return FLAME_GR_UNSUPPORTED; }
  if (hist_len < 0 || hist_len > d->L) { d->err = "hist_len must be in [0, the hist_len given at create]"; return FLAME_GR_CAPACITY_EXCEEDED; }
  return submit_request(d, history_emb, hist_len, cand_emb, n_cand, scores, ticket);
}

int flame_dso_wait(flame_dso_t *d, int64_t ticket) {
  if (!live(d)) return FLAME_GR_BAD_HANDLE;
  d->err.clear();
  if (ticket < 1 || ticket >= d->next_ticket) { d->err = "unknown ticket"; return FLAME_GR_INVALID_ARGUMENT; }
  auto holds = [&](const Executor &e) {
    if (!d->jagged) return e.pending.ticket == ticket;
    for (const Pending &p : e.batch)
      if (p.ticket == ticket) return true;
    return false;
  };
  // a request that still sits in the gathering batch goes to the GPU now
  if (d->gathering >= 0 && holds(d->ex[d->gathering])) {
    int rc = flush(d, d->gathering);
    if (rc) return rc;
  }
  for (int i = 0; i < (int)d->ex.size(); ++i)
    if (d->ex[i].busy && holds(d->ex[i])) {
      int rc = retire(d, i);
      if (rc) return rc;
    }
  return FLAME_GR_OK;
}

int flame_dso_drain(flame_dso_t *d) {
  if (!live(d)) return FLAME_GR_BAD_HANDLE;
  d->err.clear();
  if (d->gathering >= 0) {
    int rc = flush(d, d->gathering);
    if (rc) return rc;
  }
  for (int i = 0; i < (int)d->ex.size(); ++i) {
    int rc = retire(d, i);
    if (rc) return rc;
  }
  return FLAME_GR_OK;
}

int flame_dso_flush(flame_dso_t *d) {
  if (!live(d)) return FLAME_GR_BAD_HANDLE;
  d->err.clear();
  return d->gathering >= 0 ? flush(d, d->gathering) : (int)FLAME_GR_OK;
}

int flame_dso_stats(const flame_dso_t *d, int64_t *out) {
  if (!live(d)) return FLAME_GR_BAD_HANDLE;
  if (!out) return FLAME_GR_INVALID_ARGUMENT;
  std::memcpy(out, d->stats, sizeof(d->stats));
  return FLAME_GR_OK;
}

int flame_dso_destroy(flame_dso_t *d) {
  if (!d) return FLAME_GR_OK;
  if (!live(d)) return FLAME_GR_BAD_HANDLE;
  (void)flame_dso_drain(d);
  release_all(d);
  d->magic = 0;
  delete d;
  return FLAME_GR_OK;
}

}  // extern "C"
