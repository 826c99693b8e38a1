// C ABI of the GR forward (flame_gr.h): handle, validation, plan staging, kernel sequencing.
//
// A handle is the analogue of the paper's executor (Section 3.3): pre-allocated buffers plus
// streams, created once; the request path allocates nothing.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>
#include <utility>
#include <string>
#include <vector>

#include "../../include/flame_gr.h"
#include "kernels.h"
#include "plan.h"

using namespace flame;

namespace {

constexpr uint32_t kMagic = 0x464c4752u;  // "FLGR"
constexpr int kStageSlots = 2;
constexpr size_t kStageOneCopyBytes = 64 << 10;   // plan tables up to this size are staged with one copy
constexpr int kMaxGroups = 16;
constexpr int kMaxGraphs = FLAME_GR_MAX_GRAPHS;
enum { KIND_ASSEMBLE = 0, KIND_BIAS, KIND_UVQK, KIND_ATTN, KIND_LNGATE, KIND_OUTPROJ, KIND_SCORE, KIND_COUNT };

thread_local std::string g_create_error;

struct StageLayout {  // byte offsets inside one staging buffer (host pinned and device mirror)
  size_t blocks, items, cand_items, cand_blocks, hist_items, hist_blocks, total;
};

// What a pass covers: the whole batch, or one stage of the two-stage path (Section 5).
enum PassMode { PASS_FULL = 0, PASS_HISTORY, PASS_CANDIDATES };

struct ProfEvent { hipEvent_t a, b; int kind; };

// One captured forward: the graph and the plan tables its kernels read (its own copy, so that eager
// passes and the other graphs of the handle, which stage their own plans, leave it intact).
struct CapturedGraph {
  hipGraphExec_t exec = nullptr;
  char *tables = nullptr;
  bool valid = false;
};

}  // namespace

struct flame_gr {
  uint32_t magic = kMagic;
  flame_gr_config cfg{};
  Shape sh{};
  int device = 0;
  int n_groups = 1;
  int q_tile = 0;
  int64_t ws_rows = 0;
  size_t elt = 4;
  std::string err;
  // workspaces (device)
  float *X = nullptr;                                                    // residual stream, fp32 path
  void *Xb = nullptr, *Xl = nullptr;                                     // residual stream, MFMA path: fp16(X) (k-tile blocked) and fp16(X - Xb)
  void *planes = nullptr, *O = nullptr, *G = nullptr;
  void *W1h = nullptr, *W2h = nullptr, *W2p = nullptr;                   // fp16 copies of the projection matrices (W2p: fragment-major)
  float *bias = nullptr;
  float *tscale = nullptr;                                               // softmax: logit scale per layer and head
  int32_t *bucket_tab = nullptr;
  // plan staging
  StageLayout lay{};
  char *stage_host[kStageSlots] = {};
  hipEvent_t stage_done[kStageSlots] = {};
  bool stage_used[kStageSlots] = {};
  int stage_next = 0;
  char *stage_dev = nullptr;
  // streams / events
  hipStream_t gstream[kMaxGroups] = {};
  hipEvent_t ev_fork = nullptr, ev_join[kMaxGroups] = {}, ev_done = nullptr;
  bool has_prev = false;
  // weights_static: the pointers the derived copies were made from
  bool derived_valid = false;
  flame_gr_weights derived_from{};
  // last plan (kept for the debug exports)
  Plan plan;
  // explicit-shape executor: the one-pass forward of one fixed batch, captured as a HIP graph
  hipStream_t cap_stream = nullptr;
  CapturedGraph graphs[kMaxGraphs];
  // two-stage path: what the last prefill cached (layer l keeps V and K at kv + l * 2 * plane_bytes)
  size_t plane_bytes = 0;
  char *kv = nullptr;
  bool kv_valid = false;
  std::vector<int32_t> kv_hoff, kv_cap;
  // debug capture
  int capture_layer = -1;
  void *cap_planes = nullptr, *cap_O = nullptr;
  float *cap_X = nullptr;
  bool cap_valid = false;
  // per-kernel timing
  bool profiling = false;
  std::vector<ProfEvent> prof_pool;
  size_t prof_used = 0;
};

namespace {

#define HIP_TRY(h, expr)                                                                   \
  do {                                                                                     \
    hipError_t e_ = (expr);                                                                \
    if (e_ != hipSuccess) {                                                                \
      (h)->err = std::string(#expr) + ": " + hipGetErrorString(e_);                        \
      return FLAME_GR_HIP_ERROR;                                                           \
    }                                                                                      \
  } while (0)

bool live(const flame_gr *h) { return h && h->magic == kMagic; }

// A handle's buffers live on the device that was current at create: work for it is enqueued there only.
bool on_own_device(flame_gr *h) {
  int dev = -1;
  if (hipGetDevice(&dev) == hipSuccess && dev == h->device) return true;
  h->err = "the handle was created on another device than the current one";
  return false;
}

// IEEE binary16 -> float on the host (debug export only)
float half_bits_to_float(uint16_t b) {
  const uint32_t sign = (uint32_t)(b & 0x8000u) << 16;
  uint32_t exp = (b >> 10) & 0x1f, man = b & 0x3ffu, out;
  if (exp == 0) {
    if (man == 0) out = sign;
    else {
      int sh = 0;
      while (!(man & 0x400u)) { man <<= 1; ++sh; }
      out = sign | ((uint32_t)(113 - sh) << 23) | ((man & 0x3ffu) << 13);
    }
  } else if (exp == 31) out = sign | 0x7f800000u | (man << 13);
  else out = sign | ((exp + 112) << 23) | (man << 13);
  float f;
  std::memcpy(&f, &out, 4);
  return f;
}

void free_all(flame_gr *h) {
  (void)hipFree(h->X); (void)hipFree(h->Xb); (void)hipFree(h->Xl); (void)hipFree(h->planes); (void)hipFree(h->kv); (void)hipFree(h->O); (void)hipFree(h->G);
  (void)hipFree(h->bias); (void)hipFree(h->tscale); (void)hipFree(h->bucket_tab); (void)hipFree(h->stage_dev);
  (void)hipFree(h->W1h); (void)hipFree(h->W2h); (void)hipFree(h->W2p);
  (void)hipFree(h->cap_planes); (void)hipFree(h->cap_O); (void)hipFree(h->cap_X);
  for (int i = 0; i < kStageSlots; ++i) {
    if (h->stage_host[i]) (void)hipHostFree(h->stage_host[i]);
    if (h->stage_done[i]) (void)hipEventDestroy(h->stage_done[i]);
  }
  for (int g = 0; g < kMaxGroups; ++g) {
    if (h->gstream[g]) (void)hipStreamDestroy(h->gstream[g]);
    if (h->ev_join[g]) (void)hipEventDestroy(h->ev_join[g]);
  }
  for (CapturedGraph &g : h->graphs) {
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
    (void)hipFree(g.tables);
  }
  if (h->cap_stream) (void)hipStreamDestroy(h->cap_stream);
  if (h->ev_fork) (void)hipEventDestroy(h->ev_fork);
  if (h->ev_done) (void)hipEventDestroy(h->ev_done);
  for (auto &p : h->prof_pool) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
}

// Bracket one launch with events when profiling is on.
struct Timed {
  flame_gr *h; hipStream_t s; ProfEvent *pe = nullptr;
  Timed(flame_gr *h_, int kind, hipStream_t s_) : h(h_), s(s_) {
    if (!h->profiling) return;
    if (h->prof_used == h->prof_pool.size()) {
      ProfEvent p{};
      if (hipEventCreate(&p.a) != hipSuccess || hipEventCreate(&p.b) != hipSuccess) return;
      h->prof_pool.push_back(p);
    }
    pe = &h->prof_pool[h->prof_used++];
    pe->kind = kind;
    (void)hipEventRecord(pe->a, s);
  }
  ~Timed() { if (pe) (void)hipEventRecord(pe->b, s); }
};

// The layer sequence of one stream group.  PASS_FULL: all rows, one set of planes reused by every
// layer.  PASS_HISTORY / PASS_CANDIDATES: the history rows (resp. candidate rows) only, every layer
// on its own set of planes, so that the candidate pass finds K and V of the history rows of layer l
// where the history pass left them.
void run_group(flame_gr *h, const flame_gr_weights &w, const Group &G, const void *hist, const void *cand,
               float *scores, hipStream_t s, PassMode mode, float *hidden = nullptr) {
  const Shape &sh = h->sh;
  const int dt = h->cfg.dtype;
  const int d = sh.d;
  const size_t e = h->elt;
  const RowBlock *blocks = (const RowBlock *)(h->stage_dev + h->lay.blocks);
  const AttnItem *items = (const AttnItem *)(h->stage_dev + h->lay.items);
  const AttnItem *citems = (const AttnItem *)(h->stage_dev + h->lay.cand_items);
  const int32_t *cblks = (const int32_t *)(h->stage_dev + h->lay.cand_blocks);
  const AttnItem *hitems = (const AttnItem *)(h->stage_dev + h->lay.hist_items);
  const int32_t *hblks = (const int32_t *)(h->stage_dev + h->lay.hist_blocks);
  const int n_blk = G.blk_end - G.blk_begin;
  const int32_t *cl = cblks + G.cblk_begin;
  const int n_cblk = G.cblk_end - G.cblk_begin;
  const int32_t *hl = hblks + G.hblk_begin;
  const int n_hblk = G.hblk_end - G.hblk_begin;
  // the rows of this pass outside the last layer: a contiguous block range, or a list
  const int32_t *pass_list = mode == PASS_FULL ? nullptr : mode == PASS_HISTORY ? hl : cl;
  const int pass_n = mode == PASS_FULL ? n_blk : mode == PASS_HISTORY ? n_hblk : n_cblk;
  const int pass_first = mode == PASS_FULL ? G.blk_begin : 0;
  if (pass_n == 0) return;
  { Timed t(h, KIND_ASSEMBLE, s); launch_assemble(dt, blocks, pass_list, pass_n, pass_first, hist, cand, h->X, h->Xb, d, s); }
  const int64_t plane = sh.ws_rows * d;
  for (int l = 0; l < sh.n_layers; ++l) {
    const bool capture = mode == PASS_FULL && h->capture_layer == l;
    const bool last = (l == sh.n_layers - 1) && !capture;
    // one-pass: the four planes of the handle, reused by every layer; two-stage: U and Q there, V and K in the
    // layer's own pair of planes, where the candidate pass finds the history rows that the history pass left
    char *planes = (char *)h->planes;
    PlanePtrs pp{planes, planes + h->plane_bytes, planes + 2 * h->plane_bytes, planes + 3 * h->plane_bytes};
    if (mode != PASS_FULL) {
      pp.v = h->kv + (size_t)l * 2 * h->plane_bytes;
      pp.k = h->kv + ((size_t)l * 2 + 1) * h->plane_bytes;
    }
    const char *w1 = (const char *)(dt == FLAME_GR_BF16 ? h->W1h : w.w1) + (size_t)l * 4 * d * d * e;
    const char *b1 = (const char *)w.b1 + (size_t)l * 4 * d * e;
    const char *w2 = (const char *)(dt == FLAME_GR_BF16 ? h->W2h : w.w2) + (size_t)l * d * d * e;
    const char *b2 = (const char *)w.b2 + (size_t)l * d * e;
    const char *lg = (const char *)w.ln_g + (size_t)l * d * e;
    const char *lb = (const char *)w.ln_b + (size_t)l * d * e;
    const float *bias_l = h->bias + (size_t)l * sh.H * sh.D;
    const float *tscale_l = h->tscale ? h->tscale + (size_t)l * sh.H : nullptr;
    // In the last layer only candidate rows feed the scores, and history rows never look at
    // candidates: history rows need K and V only, attention and the output projection run on
    // candidate rows only.
    if (dt == FLAME_GR_BF16) {
      Timed t(h, KIND_UVQK, s);
      if (mode == PASS_FULL && last) {
        launch_uvqk_bf16(h->Xb, w1, b1, pp, nullptr, n_blk, G.blk_begin, 0xA, sh, s);  // V, K: all rows
        launch_uvqk_bf16(h->Xb, w1, b1, pp, cl, n_cblk, 0, 0x5, sh, s);                // U, Q: candidates
      } else {
        launch_uvqk_bf16(h->Xb, w1, b1, pp, pass_list, pass_n, pass_first, mode == PASS_HISTORY && last ? 0xA : 0xF, sh, s);
      }
    } else {
      Timed t(h, KIND_UVQK, s);
      launch_uvqk_f32(h->X, (const float *)w1, (const float *)b1, (float *)planes, G.blk_begin, n_blk, sh, s);
    }
    if (mode == PASS_HISTORY && last) break;  // the history rows of the last layer end at K and V
    {
      Timed t(h, KIND_ATTN, s);
      const AttnItem *it = items + G.item_begin;
      int n_it = G.item_end - G.item_begin;
      if (mode == PASS_HISTORY) { it = hitems + G.hitem_begin; n_it = G.hitem_end - G.hitem_begin; }
      else if (mode == PASS_CANDIDATES || last) { it = citems + G.citem_begin; n_it = G.citem_end - G.citem_begin; }
      if (dt == FLAME_GR_BF16) launch_attn_bf16(pp, bias_l, tscale_l, h->O, it, n_it, sh, s);
      else launch_attn_f32((const float *)planes, bias_l, tscale_l, (float *)h->O, it, n_it, h->q_tile, sh, s);
    }
    const int32_t *bl = mode == PASS_FULL ? (last ? cl : nullptr) : pass_list;
    const int nb = mode == PASS_FULL ? (last ? n_cblk : n_blk) : pass_n;
    const int bf = mode == PASS_FULL && !last ? G.blk_begin : 0;
    if (dt == FLAME_GR_BF16 && k3_fused_supported(d)) {
      Timed t(h, KIND_OUTPROJ, s);
      launch_k3_fused(h->O, planes, lg, lb, (const char *)h->W2p + (size_t)l * d * d * e, b2, h->Xb, h->Xl, l == 0, blocks, bl, nb, bf, sh, s);
    } else {
      {
        Timed t(h, KIND_LNGATE, s);
        launch_ln_gate(dt, h->O, planes, lg, lb, h->G, blocks, bl, nb, bf, d, sh.eps, s);
      }
      Timed t(h, KIND_OUTPROJ, s);
      if (dt == FLAME_GR_BF16) launch_outproj_bf16(h->G, w2, b2, h->Xb, h->Xl, l == 0, bl, nb, bf, sh, s);
      else launch_outproj_f32((const float *)h->G, (const float *)w2, (const float *)b2, h->X, bl, nb, bf, sh, s);
    }
    if (capture && h->cap_planes) {
      const size_t r0 = (size_t)G.row_begin * d, nr = (size_t)(G.row_end - G.row_begin) * d;
      for (int p = 0; p < 4; ++p) {
        if (dt == FLAME_GR_BF16 && p == 1) {
          // V is stored feature-major ([d][ws_rows]): this group's tokens are a column range
          const size_t off = ((size_t)plane + (size_t)G.row_begin) * e, pitch = (size_t)sh.ws_rows * e;
          (void)hipMemcpy2DAsync((char *)h->cap_planes + off, pitch, (char *)h->planes + off, pitch,
                                 (size_t)(G.row_end - G.row_begin) * e, (size_t)d, hipMemcpyDeviceToDevice, s);
        } else {
          (void)hipMemcpyAsync((char *)h->cap_planes + ((size_t)p * plane + r0) * e, (char *)h->planes + ((size_t)p * plane + r0) * e, nr * e, hipMemcpyDeviceToDevice, s);
        }
      }
      (void)hipMemcpyAsync((char *)h->cap_O + r0 * e, (char *)h->O + r0 * e, nr * e, hipMemcpyDeviceToDevice, s);
      if (dt == FLAME_GR_BF16) launch_residual_to_f32(h->Xb, h->Xl, h->cap_X, G.row_begin, G.row_end, d, s);
      else (void)hipMemcpyAsync(h->cap_X + r0, h->X + r0, nr * sizeof(float), hipMemcpyDeviceToDevice, s);
    }
  }
  if (mode == PASS_HISTORY) return;
  {
    Timed t(h, KIND_SCORE, s);
    if (hidden) launch_gather_hidden(h->X, h->Xb, h->Xl, blocks, cl, n_cblk, hidden, d, s);
    else launch_scores(dt, h->X, h->Xb, h->Xl, w.w_s, w.b_s, blocks, cl, n_cblk, scores, d, s);
  }
}

// What the kernels read in place of the caller's weights: fp16 copies of the projection matrices in
// the operand layouts of the GEMMs (MFMA path), and the bias table indexed by distance.
bool same_weight_pointers(const flame_gr_weights &a, const flame_gr_weights &b) {
  return a.w1 == b.w1 && a.w2 == b.w2 && a.rab == b.rab && a.temperature == b.temperature;   // what the copies are made from
}

void derive_weights(flame_gr *h, const flame_gr_weights *w, hipStream_t s) {
  if (h->cfg.weights_static && h->derived_valid && same_weight_pointers(h->derived_from, *w)) return;
  h->derived_from = *w;
  h->derived_valid = true;
  if (h->cfg.dtype == FLAME_GR_BF16) {
    const int dm = h->sh.d;
    launch_bf16_to_f16(w->w1, h->W1h, (int64_t)h->sh.n_layers * 4 * dm, dm, true, s);
    if (k3_fused_supported(dm)) launch_pack_w2(w->w2, h->W2p, dm, h->sh.n_layers, s);
    else launch_bf16_to_f16(w->w2, h->W2h, (int64_t)h->sh.n_layers * dm, dm, true, s);
  }
  launch_expand_bias(w->rab, h->bucket_tab, h->bias, h->sh.n_layers * h->sh.H, h->sh.n_buckets, h->sh.D,
                     h->cfg.dtype == FLAME_GR_BF16 ? 0.5f : 1.0f, s);
  // softmax: exponent = logit / tau.  The MFMA kernel holds halved logits and uses the base-2 exponential.
  if (h->sh.softmax)
    launch_logit_scale(w->temperature, h->tscale, h->sh.n_layers * h->sh.H,
                       h->cfg.dtype == FLAME_GR_BF16 ? 2.0f * 1.4426950408889634f : 1.0f, s);
}

// Stage h->plan through pinned memory, refresh the derived weights and run `mode` on every stream group.
int enqueue_pass(flame_gr *h, const flame_gr_weights *w, const void *history_emb, const void *cand_emb, float *scores,
                 hipStream_t s0, PassMode mode, float *hidden = nullptr) {
  const Plan &P = h->plan;
  // stage the plan: one pinned buffer
  const int slot = h->stage_next;
  h->stage_next = (slot + 1) % kStageSlots;
  if (h->stage_used[slot]) HIP_TRY(h, hipEventSynchronize(h->stage_done[slot]));
  char *sh_ = h->stage_host[slot];
  // a pass on another stream must not overtake the previous one on this handle
  if (h->has_prev) HIP_TRY(h, hipStreamWaitEvent(s0, h->ev_done, 0));
  // The tables are copied separately, only as far as they are filled and only those the pass reads; on a handle whose
  // tables are small altogether (one or a few requests) they leave as one copy instead, what lies between them included:
  // every copy is a few microseconds in front of the first kernel.
  const bool one_copy = h->lay.total <= kStageOneCopyBytes;
  size_t staged_end = 0;
  auto stage = [&](size_t off, const void *src, size_t bytes) -> hipError_t {
    if (bytes == 0) return hipSuccess;
    std::memcpy(sh_ + off, src, bytes);
    if (one_copy) { staged_end = std::max(staged_end, off + bytes); return hipSuccess; }
    return hipMemcpyAsync(h->stage_dev + off, sh_ + off, bytes, hipMemcpyHostToDevice, s0);
  };
  HIP_TRY(h, stage(h->lay.blocks, P.blocks.data(), P.blocks.size() * sizeof(RowBlock)));
  if (mode == PASS_FULL) HIP_TRY(h, stage(h->lay.items, P.items.data(), P.items.size() * sizeof(AttnItem)));
  if (mode != PASS_HISTORY) {
    HIP_TRY(h, stage(h->lay.cand_items, P.cand_items.data(), P.cand_items.size() * sizeof(AttnItem)));
    HIP_TRY(h, stage(h->lay.cand_blocks, P.cand_blocks.data(), P.cand_blocks.size() * sizeof(int32_t)));
  }
  if (mode == PASS_HISTORY) {
    HIP_TRY(h, stage(h->lay.hist_items, P.hist_items.data(), P.hist_items.size() * sizeof(AttnItem)));
    HIP_TRY(h, stage(h->lay.hist_blocks, P.hist_blocks.data(), P.hist_blocks.size() * sizeof(int32_t)));
  }
  if (one_copy && staged_end > 0) HIP_TRY(h, hipMemcpyAsync(h->stage_dev, sh_, staged_end, hipMemcpyHostToDevice, s0));
  HIP_TRY(h, hipEventRecord(h->stage_done[slot], s0));
  h->stage_used[slot] = true;
  {
    // the caller owns the weights and may have changed them: derive on every pass (unless declared static)
    Timed t(h, KIND_BIAS, s0);
    derive_weights(h, w, s0);
  }
  if (h->n_groups == 1) {
    run_group(h, *w, P.groups[0], history_emb, cand_emb, scores, s0, mode, hidden);
  } else {
    HIP_TRY(h, hipEventRecord(h->ev_fork, s0));
    for (int g = 0; g < h->n_groups; ++g) {
      if (P.groups[g].blk_end == P.groups[g].blk_begin) continue;
      HIP_TRY(h, hipStreamWaitEvent(h->gstream[g], h->ev_fork, 0));
      run_group(h, *w, P.groups[g], history_emb, cand_emb, scores, h->gstream[g], mode, hidden);
      HIP_TRY(h, hipEventRecord(h->ev_join[g], h->gstream[g]));
      HIP_TRY(h, hipStreamWaitEvent(s0, h->ev_join[g], 0));
    }
  }
  HIP_TRY(h, hipEventRecord(h->ev_done, s0));
  h->has_prev = true;
  hipError_t le = hipGetLastError();
  if (le != hipSuccess) { h->err = std::string("kernel launch: ") + hipGetErrorString(le); return FLAME_GR_HIP_ERROR; }
  return FLAME_GR_OK;
}

// Plan tables of a workspace of nblk 64-row blocks, back to back in one buffer.
StageLayout stage_layout(size_t nblk) {
  StageLayout lay{};
  lay.blocks = 0;
  lay.items = lay.blocks + nblk * sizeof(RowBlock);
  lay.cand_items = lay.items + nblk * sizeof(AttnItem);
  lay.cand_blocks = lay.cand_items + nblk * sizeof(AttnItem);
  lay.hist_items = lay.cand_blocks + nblk * sizeof(int32_t);
  lay.hist_blocks = lay.hist_items + nblk * sizeof(AttnItem);
  lay.total = lay.hist_blocks + nblk * sizeof(int32_t);
  return lay;
}

// The MFMA path reads embeddings and weights 16 bytes at a time.
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool pointers_aligned(const flame_gr *h, const flame_gr_weights *w, const void *hist, const void *cand) {
  if (h->cfg.dtype != FLAME_GR_BF16) return true;
  return aligned16(hist) && aligned16(cand) && aligned16(w->w1) && aligned16(w->b1) && aligned16(w->ln_g) && aligned16(w->ln_b) &&
         aligned16(w->w2) && aligned16(w->b2) && aligned16(w->w_s);
}

// w_s may be absent when the caller asks for hidden rows instead of scores
bool weights_complete(const flame_gr *h, const flame_gr_weights *w, bool need_score_head = true) {
  return w->w1 && w->b1 && w->rab && w->ln_g && w->ln_b && w->w2 && w->b2 && (w->w_s || !need_score_head) &&
         (w->temperature || !h->sh.softmax);
}

}  // namespace

extern "C" {

const char *flame_gr_last_error(const flame_gr_t *h) {
  if (!h) return g_create_error.c_str();
  if (!live(h)) return "bad handle";
  return h->err.c_str();
}

int flame_gr_create(const flame_gr_config *cfg_in, flame_gr_t **out) {
  if (out) *out = nullptr;
  if (!cfg_in || !out) { g_create_error = "cfg or out is NULL"; return FLAME_GR_INVALID_ARGUMENT; }
  flame_gr_config cfg = *cfg_in;
  if (cfg.ln_eps == 0.f) cfg.ln_eps = 1e-6f;
  if (cfg.attn_scale == 0.f) cfg.attn_scale = 1.0f;
  int rc = validate_config(cfg, g_create_error);
  if (rc) return rc;
  flame_gr *h = new (std::nothrow) flame_gr();
  if (!h) { g_create_error = "out of host memory"; return FLAME_GR_HIP_ERROR; }
  h->cfg = cfg;
  h->n_groups = cfg.n_streams > 1 ? cfg.n_streams : 1;
  h->q_tile = cfg.dtype == FLAME_GR_BF16 ? kAttnQTileBf16 : kAttnQTileF32;
  h->elt = cfg.dtype == FLAME_GR_BF16 ? 2 : 4;
  h->ws_rows = workspace_rows(cfg);
  h->sh = Shape{cfg.d_model, cfg.n_heads, cfg.d_model / cfg.n_heads, cfg.n_layers, cfg.n_buckets,
                cfg.max_rel_dist, cfg.ln_eps, cfg.attn_scale, h->ws_rows, cfg.attn_kind == FLAME_GR_ATTN_SOFTMAX ? 1 : 0,
                cfg.latency_mode ? 1 : 0};
  auto fail = [&](const std::string &m, int code) {
    g_create_error = m;
    free_all(h);
    h->magic = 0;
    delete h;
    return code;
  };
#define CR(expr)                                                                            \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) return fail(std::string(#expr) + ": " + hipGetErrorString(e_), FLAME_GR_HIP_ERROR); \
  } while (0)
  CR(hipGetDevice(&h->device));
  if (h->sh.latency && cfg.dtype == FLAME_GR_BF16) CR(attn_latency_setup(h->sh));
  const size_t rows = (size_t)h->ws_rows, d = (size_t)cfg.d_model, e = h->elt;
  const bool mfma_path = cfg.dtype == FLAME_GR_BF16;
  if (!mfma_path) CR(hipMalloc(&h->X, rows * d * sizeof(float)));
  h->plane_bytes = rows * d * e;
  CR(hipMalloc(&h->planes, 4 * h->plane_bytes));
  if (cfg.kv_cache) CR(hipMalloc((void **)&h->kv, (size_t)cfg.n_layers * 2 * h->plane_bytes));
  CR(hipMalloc(&h->O, rows * d * e));
  const bool need_g = !mfma_path || !k3_fused_supported(cfg.d_model);      // the fused K3 keeps the gated rows in LDS
  if (need_g) CR(hipMalloc(&h->G, rows * d * e));
  if (mfma_path) {
    CR(hipMalloc(&h->Xb, rows * d * e));
    CR(hipMalloc(&h->Xl, rows * d * e));
    CR(hipMalloc(&h->W1h, (size_t)cfg.n_layers * 4 * d * d * e));
    CR(hipMalloc(&h->W2h, (size_t)cfg.n_layers * d * d * e));
    CR(hipMalloc(&h->W2p, (size_t)cfg.n_layers * d * d * e));
  }
  CR(hipMalloc(&h->bias, (size_t)cfg.n_layers * cfg.n_heads * cfg.max_rel_dist * sizeof(float)));
  CR(hipMalloc(&h->bucket_tab, (size_t)cfg.max_rel_dist * sizeof(int32_t)));
  if (h->sh.softmax) CR(hipMalloc(&h->tscale, (size_t)cfg.n_layers * cfg.n_heads * sizeof(float)));
  // Every workspace starts finite: rows that a batch leaves as padding are read (and multiplied
  // by zero weights) by the tiled kernels.
  if (h->X) CR(hipMemset(h->X, 0, rows * d * sizeof(float)));
  CR(hipMemset(h->planes, 0, 4 * h->plane_bytes));
  if (h->kv) CR(hipMemset(h->kv, 0, (size_t)cfg.n_layers * 2 * h->plane_bytes));
  CR(hipMemset(h->O, 0, rows * d * e));
  if (h->G) CR(hipMemset(h->G, 0, rows * d * e));
  if (h->Xb) CR(hipMemset(h->Xb, 0, rows * d * e));
  if (h->Xl) CR(hipMemset(h->Xl, 0, rows * d * e));
  {
    std::vector<int32_t> tab(cfg.max_rel_dist);
    bucket_table(cfg.n_buckets, cfg.max_rel_dist, tab.data());
    CR(hipMemcpy(h->bucket_tab, tab.data(), tab.size() * sizeof(int32_t), hipMemcpyHostToDevice));
  }
  h->lay = stage_layout(rows / kRowAlign);
  CR(hipMalloc(&h->stage_dev, h->lay.total));
  for (int i = 0; i < kStageSlots; ++i) {
    CR(hipHostMalloc((void **)&h->stage_host[i], h->lay.total, hipHostMallocDefault));
    CR(hipEventCreateWithFlags(&h->stage_done[i], hipEventDisableTiming));
  }
  CR(hipEventCreateWithFlags(&h->ev_fork, hipEventDisableTiming));
  CR(hipEventCreateWithFlags(&h->ev_done, hipEventDisableTiming));
  if (h->n_groups > 1)
    for (int g = 0; g < h->n_groups; ++g) {
      CR(hipStreamCreateWithFlags(&h->gstream[g], hipStreamNonBlocking));
      CR(hipEventCreateWithFlags(&h->ev_join[g], hipEventDisableTiming));
    }
  CR(hipDeviceSynchronize());
#undef CR
  *out = h;
  return FLAME_GR_OK;
}

int flame_gr_destroy(flame_gr_t *h) {
  if (!h) return FLAME_GR_OK;
  if (!live(h)) return FLAME_GR_BAD_HANDLE;
  if (h->has_prev) (void)hipEventSynchronize(h->ev_done);
  for (int g = 0; g < kMaxGroups; ++g)
    if (h->gstream[g]) (void)hipStreamSynchronize(h->gstream[g]);
  free_all(h);
  h->magic = 0;
  delete h;
  return FLAME_GR_OK;
}

static int forward_common(flame_gr_t *h, const flame_gr_weights *w, const void *history_emb,
                          const int32_t *history_offsets, const void *cand_emb, const int32_t *cand_offsets,
                          int32_t n_requests, float *scores, float *hidden, void *stream_v) {
  if (!live(h)) return FLAME_GR_BAD_HANDLE;
  h->err.clear();
  if (!on_own_device(h)) return FLAME_GR_INVALID_ARGUMENT;
  auto bad = [&](const char *m) { h->err = m; return (int)FLAME_GR_INVALID_ARGUMENT; };
  const bool want_hidden = scores == nullptr && hidden != nullptr;
  if (!w) return bad("weights is NULL");
  if (n_requests < 0) return bad("n_requests < 0");
  if (n_requests > 0 && (!history_offsets || !cand_offsets)) return bad("offset arrays are NULL");
  Plan plan;
  int rc = build_plan(h->cfg, history_offsets, cand_offsets, n_requests, h->q_tile, h->n_groups, h->ws_rows, plan, h->err);
  if (rc) return rc;
  if (want_hidden && plan.split) { h->err = "hidden rows are not available for split requests"; return FLAME_GR_UNSUPPORTED; }
  const int64_t sumL = n_requests ? history_offsets[n_requests] : 0, sumM = n_requests ? cand_offsets[n_requests] : 0;
  if (sumL > 0 && !history_emb) return bad("history_emb is NULL");
  if (sumM > 0 && (!cand_emb || (!scores && !hidden))) return bad("cand_emb or the output array is NULL");
  if (plan.total_rows > 0 && !weights_complete(h, w, !want_hidden)) return bad("a weight pointer is NULL");
  if (!pointers_aligned(h, w, history_emb, cand_emb)) return bad("bf16 embeddings and weights must be 16-byte aligned");
  h->plan = std::move(plan);
  h->cap_valid = false;
  if (h->plan.total_rows == 0) return FLAME_GR_OK;
  rc = enqueue_pass(h, w, history_emb, cand_emb, scores, (hipStream_t)stream_v, PASS_FULL, want_hidden ? hidden : nullptr);
  if (rc) return rc;
  h->cap_valid = h->capture_layer >= 0 && h->cap_planes;
  return FLAME_GR_OK;
}

int flame_gr_forward(flame_gr_t *h, const flame_gr_weights *w, const void *history_emb,
                     const int32_t *history_offsets, const void *cand_emb, const int32_t *cand_offsets,
                     int32_t n_requests, float *scores, void *stream_v) {
  if (live(h) && n_requests > 0 && cand_offsets && cand_offsets[n_requests] > 0 && !scores) {
    h->err = "cand_emb or scores is NULL";
    return FLAME_GR_INVALID_ARGUMENT;
  }
  return forward_common(h, w, history_emb, history_offsets, cand_emb, cand_offsets, n_requests, scores, nullptr, stream_v);
}

int flame_gr_forward_hidden(flame_gr_t *h, const flame_gr_weights *w, const void *history_emb,
                            const int32_t *history_offsets, const void *cand_emb, const int32_t *cand_offsets,
                            int32_t n_requests, float *hidden, void *stream_v) {
  if (live(h) && n_requests > 0 && cand_offsets && cand_offsets[n_requests] > 0 && !hidden) {
    h->err = "cand_emb or hidden is NULL";
    return FLAME_GR_INVALID_ARGUMENT;
  }
  return forward_common(h, w, history_emb, history_offsets, cand_emb, cand_offsets, n_requests, nullptr, hidden, stream_v);
}

int flame_gr_capture(flame_gr_t *h, int32_t slot, const flame_gr_weights *w, const void *history_emb,
                     const int32_t *history_offsets, const void *cand_emb, const int32_t *cand_offsets,
                     int32_t n_requests, float *scores, void *record_stream) {
  if (!live(h)) return FLAME_GR_BAD_HANDLE;
  h->err.clear();
  if (!on_own_device(h)) return FLAME_GR_INVALID_ARGUMENT;
  auto bad = [&](const char *m) { h->err = m; return (int)FLAME_GR_INVALID_ARGUMENT; };
  if (slot < 0 || slot >= kMaxGraphs) return bad("graph slot out of range");
  if (h->n_groups != 1) { h->err = "capture needs a handle without internal stream groups (n_streams <= 1)"; return FLAME_GR_UNSUPPORTED; }
  if (h->capture_layer >= 0) { h->err = "capture is not available while a debug layer capture is selected"; return FLAME_GR_UNSUPPORTED; }
  if (!w) return bad("weights is NULL");
  if (n_requests < 0) return bad("n_requests < 0");
  if (n_requests > 0 && (!history_offsets || !cand_offsets)) return bad("offset arrays are NULL");
  Plan plan;
  int rc = build_plan(h->cfg, history_offsets, cand_offsets, n_requests, h->q_tile, 1, h->ws_rows, plan, h->err);
  if (rc) return rc;
  const int64_t sumL = n_requests ? history_offsets[n_requests] : 0, sumM = n_requests ? cand_offsets[n_requests] : 0;
  if (sumM == 0) return bad("nothing to capture: the batch has no candidates");
  if (sumL > 0 && !history_emb) return bad("history_emb is NULL");
  if (!cand_emb || !scores) return bad("cand_emb or scores is NULL");
  if (!weights_complete(h, w)) return bad("a weight pointer is NULL");
  if (!pointers_aligned(h, w, history_emb, cand_emb)) return bad("bf16 embeddings and weights must be 16-byte aligned");
  // setup, outside the graph: wait for earlier work on the handle, then upload the plan and derive the weights
  if (h->has_prev) HIP_TRY(h, hipEventSynchronize(h->ev_done));
  CapturedGraph &cg = h->graphs[slot];
  cg.valid = false;
  h->cap_valid = false;
  if (cg.exec) { HIP_TRY(h, hipGraphExecDestroy(cg.exec)); cg.exec = nullptr; }
  if (!cg.tables) HIP_TRY(h, hipMalloc((void **)&cg.tables, h->lay.total));
  hipStream_t cs = (hipStream_t)record_stream;
  if (!cs) {
    if (!h->cap_stream) HIP_TRY(h, hipStreamCreateWithFlags(&h->cap_stream, hipStreamNonBlocking));
    cs = h->cap_stream;
  }
  h->plan = std::move(plan);
  const Plan &P = h->plan;
  auto upload = [&](size_t off, const void *src, size_t bytes) -> hipError_t {
    return bytes ? hipMemcpy(cg.tables + off, src, bytes, hipMemcpyHostToDevice) : hipSuccess;
  };
  HIP_TRY(h, upload(h->lay.blocks, P.blocks.data(), P.blocks.size() * sizeof(RowBlock)));
  HIP_TRY(h, upload(h->lay.items, P.items.data(), P.items.size() * sizeof(AttnItem)));
  HIP_TRY(h, upload(h->lay.cand_items, P.cand_items.data(), P.cand_items.size() * sizeof(AttnItem)));
  HIP_TRY(h, upload(h->lay.cand_blocks, P.cand_blocks.data(), P.cand_blocks.size() * sizeof(int32_t)));
  derive_weights(h, w, cs);
  HIP_TRY(h, hipStreamSynchronize(cs));
  // the layer sequence, recorded instead of run (kernel launches only: no copies, no memsets), reading this slot's tables
  const bool prof = h->profiling;
  char *const eager_tables = h->stage_dev;
  h->profiling = false;
  h->stage_dev = cg.tables;
  hipGraph_t graph = nullptr;
  hipError_t e = hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal);
  if (e == hipSuccess) {
    run_group(h, *w, P.groups[0], history_emb, cand_emb, scores, cs, PASS_FULL);
    e = hipStreamEndCapture(cs, &graph);
  }
  h->stage_dev = eager_tables;
  h->profiling = prof;
  if (e == hipSuccess) e = hipGraphInstantiate(&cg.exec, graph, nullptr, nullptr, 0);
  if (graph) (void)hipGraphDestroy(graph);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    cg.exec = nullptr;
    h->err = std::string("graph capture: ") + hipGetErrorString(e);
    return FLAME_GR_HIP_ERROR;
  }
  cg.valid = true;
  return FLAME_GR_OK;
}

int flame_gr_replay(flame_gr_t *h, int32_t slot, void *stream_v) {
  if (!live(h)) return FLAME_GR_BAD_HANDLE;
  h->err.clear();
  if (!on_own_device(h)) return FLAME_GR_INVALID_ARGUMENT;
  if (slot < 0 || slot >= kMaxGraphs) { h->err = "graph slot out of range"; return FLAME_GR_INVALID_ARGUMENT; }
  if (!h->graphs[slot].valid) { h->err = "no captured forward in this slot"; return FLAME_GR_INVALID_ARGUMENT; }
  hipStream_t s0 = (hipStream_t)stream_v;
  if (h->has_prev) HIP_TRY(h, hipStreamWaitEvent(s0, h->ev_done, 0));
  HIP_TRY(h, hipGraphLaunch(h->graphs[slot].exec, s0));
  HIP_TRY(h, hipEventRecord(h->ev_done, s0));
  h->has_prev = true;
  h->cap_valid = false;
  return FLAME_GR_OK;
}

int flame_gr_prefill(flame_gr_t *h, const flame_gr_weights *w, const void *history_emb,
                     const int32_t *history_offsets, const int32_t *cand_capacity, int32_t n_requests,
                     void *stream_v) {
  if (!live(h)) return FLAME_GR_BAD_HANDLE;
  h->err.clear();
  if (!on_own_device(h)) return FLAME_GR_INVALID_ARGUMENT;
  auto bad = [&](const char *m) { h->err = m; return (int)FLAME_GR_INVALID_ARGUMENT; };
  if (!h->cfg.kv_cache) { h->err = "handle was created without kv_cache"; return FLAME_GR_UNSUPPORTED; }
  if (!w) return bad("weights is NULL");
  if (n_requests < 0) return bad("n_requests < 0");
  if (n_requests > 0 && (!history_offsets || !cand_capacity)) return bad("history_offsets or cand_capacity is NULL");
  const std::vector<int32_t> no_cands((size_t)n_requests + 1, 0);
  Plan plan;
  int rc = build_plan(h->cfg, history_offsets, no_cands.data(), n_requests, h->q_tile, h->n_groups, h->ws_rows, plan,
                      h->err, cand_capacity);
  if (rc) return rc;
  const int64_t sumL = n_requests ? history_offsets[n_requests] : 0;
  if (sumL > 0 && !history_emb) return bad("history_emb is NULL");
  if (sumL > 0 && !weights_complete(h, w)) return bad("a weight pointer is NULL");
  if (!pointers_aligned(h, w, history_emb, nullptr)) return bad("bf16 embeddings and weights must be 16-byte aligned");
  h->plan = std::move(plan);
  h->cap_valid = false;
  h->kv_valid = false;
  h->kv_hoff.assign(history_offsets, history_offsets + (n_requests ? n_requests + 1 : 0));
  h->kv_cap.assign(cand_capacity, cand_capacity + n_requests);
  if (sumL > 0) {
    rc = enqueue_pass(h, w, history_emb, nullptr, nullptr, (hipStream_t)stream_v, PASS_HISTORY);
    if (rc) return rc;
  }
  h->kv_valid = true;
  return FLAME_GR_OK;
}

int flame_gr_score(flame_gr_t *h, const flame_gr_weights *w, const void *cand_emb, const int32_t *cand_offsets,
                   int32_t n_requests, float *scores, void *stream_v) {
  if (!live(h)) return FLAME_GR_BAD_HANDLE;
  h->err.clear();
  if (!on_own_device(h)) return FLAME_GR_INVALID_ARGUMENT;
  auto bad = [&](const char *m) { h->err = m; return (int)FLAME_GR_INVALID_ARGUMENT; };
  if (!h->cfg.kv_cache) { h->err = "handle was created without kv_cache"; return FLAME_GR_UNSUPPORTED; }
  if (!h->kv_valid) return bad("no valid prefill on this handle");
  if (!w) return bad("weights is NULL");
  if (n_requests != (int32_t)h->kv_cap.size()) return bad("n_requests differs from the prefill");
  if (n_requests > 0 && !cand_offsets) return bad("cand_offsets is NULL");
  Plan plan;
  int rc = build_plan(h->cfg, h->kv_hoff.data(), cand_offsets, n_requests, h->q_tile, h->n_groups, h->ws_rows, plan,
                      h->err, h->kv_cap.data());
  if (rc) return rc;
  const int64_t sumM = n_requests ? cand_offsets[n_requests] : 0;
  if (sumM > 0 && (!cand_emb || !scores)) return bad("cand_emb or scores is NULL");
  if (sumM > 0 && !weights_complete(h, w)) return bad("a weight pointer is NULL");
  if (!pointers_aligned(h, w, nullptr, cand_emb)) return bad("bf16 embeddings and weights must be 16-byte aligned");
  h->plan = std::move(plan);
  h->cap_valid = false;
  if (sumM == 0) return FLAME_GR_OK;
  return enqueue_pass(h, w, nullptr, cand_emb, scores, (hipStream_t)stream_v, PASS_CANDIDATES);
}

}  // extern "C"

// ---------------------------------------------------------------------------------------------
// The forward in a static workspace, for callers that cannot allocate.
// ---------------------------------------------------------------------------------------------
namespace {
constexpr size_t kStaticScratchBytes = (size_t)FLAME_GR_STATIC_SCRATCH_MIB << 20;
constexpr int kMaxDevices = 64;
}  // namespace

// Every workspace of flame_gr_forward_static lives here: one copy per GPU, held until the process ends.  On the
// host this name is only a handle for hipGetSymbolAddress; kernels get the device address obtained there.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

std::mutex g_scratch_mu;
unsigned char *g_scratch_ptr[kMaxDevices] = {};

// Device address of this device's copy of `scratch` (looked up once per device, with that device current).
int static_scratch_base(int dev, unsigned char **out) {
  if (dev < 0 || dev >= kMaxDevices) { g_create_error = "device index out of range for the static workspace"; return FLAME_GR_UNSUPPORTED; }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      g_create_error = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e);
      return FLAME_GR_HIP_ERROR;
    }
    g_scratch_ptr[dev] = (unsigned char *)p;
  }
  *out = g_scratch_ptr[dev];
  return FLAME_GR_OK;
}

struct Carver {   // offsets of consecutive 256-byte aligned pieces
  size_t off = 0;
  size_t take(size_t bytes) { const size_t o = off; off = (off + bytes + 255) & ~(size_t)255; return o; }
};

}  // namespace

extern "C" {

int flame_gr_static_scratch_bytes(const flame_gr_config *cfg_in, int64_t padded_rows, int64_t *bytes) {
  if (!cfg_in || !bytes || padded_rows < 0) { g_create_error = "cfg or bytes is NULL, or padded_rows < 0"; return FLAME_GR_INVALID_ARGUMENT; }
  flame_gr_config cfg = *cfg_in;
  cfg.max_requests = 0; cfg.max_total_tokens = 0;      // capacities play no part here
  std::string err;
  const int rc = validate_config(cfg, err);
  if (rc) { g_create_error = err; return rc; }
  const bool bf = cfg.dtype == FLAME_GR_BF16;
  const size_t rows = (size_t)((padded_rows + 255) / 256 * 256 + kSpareRows), d = (size_t)cfg.d_model, e = bf ? 2 : 4;
  const size_t L = (size_t)cfg.n_layers;
  Carver c;
  c.take(bf ? 2 * rows * d * e : rows * d * sizeof(float)); // residual: Xh and Xl (MFMA path) or fp32 X
  c.take(4 * rows * d * e);                                 // U, V, Q, K
  c.take(rows * d * e);                                     // O
  if (!bf || !k3_fused_supported(cfg.d_model)) c.take(rows * d * e);   // G
  if (bf) {
    c.take(L * 4 * d * d * e);                              // W1 as fp16, k-tile blocked
    c.take(L * d * d * e);                                  // W2 as fp16 (blocked or fragment-packed)
  }
  c.take(L * (size_t)cfg.n_heads * (size_t)cfg.max_rel_dist * sizeof(float));   // bias by distance
  c.take((size_t)cfg.max_rel_dist * sizeof(int32_t));       // bucket table
  c.take(L * (size_t)cfg.n_heads * sizeof(float));          // softmax logit scales
  c.take(stage_layout(rows / kRowAlign).total);             // plan tables
  *bytes = (int64_t)c.off;
  return FLAME_GR_OK;
}

int flame_gr_forward_static(const flame_gr_config *cfg_in, const flame_gr_weights *w, const void *history_emb,
                            const int32_t *history_offsets, const void *cand_emb, const int32_t *cand_offsets,
                            int32_t n_requests, float *scores, void *stream_v) {
  auto bad = [&](const char *m) { g_create_error = m; return (int)FLAME_GR_INVALID_ARGUMENT; };
  if (!cfg_in) return bad("cfg is NULL");
  if (!w) return bad("weights is NULL");
  if (n_requests < 0) return bad("n_requests < 0");
  if (n_requests > 0 && (!history_offsets || !cand_offsets)) return bad("offset arrays are NULL");
  flame_gr h;                                     // lives for this call only; owns nothing on the device
  h.cfg = *cfg_in;
  flame_gr_config &cfg = h.cfg;
  if (cfg.ln_eps == 0.f) cfg.ln_eps = 1e-6f;
  if (cfg.attn_scale == 0.f) cfg.attn_scale = 1.0f;
  if (cfg.n_streams > 1 || cfg.kv_cache) { g_create_error = "the static workspace serves one stream and no K/V cache (n_streams <= 1, kv_cache = 0)"; return FLAME_GR_UNSUPPORTED; }
  // the capacity of this entry point is the static workspace, not the capacity fields of the configuration
  cfg.max_requests = n_requests;
  cfg.max_total_tokens = n_requests ? history_offsets[n_requests] + cand_offsets[n_requests] : 0;
  if (cfg.max_total_tokens < 0) return bad("offsets must be non-decreasing");
  int rc = validate_config(cfg, g_create_error);
  if (rc) return rc;
  const bool bf = cfg.dtype == FLAME_GR_BF16;
  h.n_groups = 1;
  h.q_tile = bf ? kAttnQTileBf16 : kAttnQTileF32;
  h.elt = bf ? 2 : 4;
  rc = build_plan(cfg, history_offsets, cand_offsets, n_requests, h.q_tile, 1, (int64_t)1 << 40, h.plan, g_create_error);
  if (rc) return rc;
  const Plan &P = h.plan;
  const int64_t sumL = n_requests ? history_offsets[n_requests] : 0, sumM = n_requests ? cand_offsets[n_requests] : 0;
  if (sumL > 0 && !history_emb) return bad("history_emb is NULL");
  if (sumM > 0 && (!cand_emb || !scores)) return bad("cand_emb or scores is NULL");
  if (P.total_rows == 0) return FLAME_GR_OK;
  if (!weights_complete(&h, w) || (cfg.attn_kind == FLAME_GR_ATTN_SOFTMAX && !w->temperature)) return bad("a weight pointer is NULL");
  if (!pointers_aligned(&h, w, history_emb, cand_emb)) return bad("bf16 embeddings and weights must be 16-byte aligned");
  // size check first: host arithmetic only
  int64_t need = 0;
  rc = flame_gr_static_scratch_bytes(&cfg, P.total_rows, &need);
  if (rc) return rc;
  if ((size_t)need > kStaticScratchBytes) {
    g_create_error = "batch and model need " + std::to_string(need) + " bytes of workspace; the static workspace holds " +
                     std::to_string(kStaticScratchBytes) + " (use a handle: flame_gr_create / flame_gr_forward)";
    return FLAME_GR_CAPACITY_EXCEEDED;
  }
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { g_create_error = "hipGetDevice failed"; return FLAME_GR_HIP_ERROR; }
  unsigned char *base = nullptr;
  rc = static_scratch_base(dev, &base);
  if (rc) return rc;
  // the same pieces, in the same order, as flame_gr_static_scratch_bytes
  h.device = dev;
  h.ws_rows = ((int64_t)P.total_rows + 255) / 256 * 256 + kSpareRows;
  h.sh = Shape{cfg.d_model, cfg.n_heads, cfg.d_model / cfg.n_heads, cfg.n_layers, cfg.n_buckets,
               cfg.max_rel_dist, cfg.ln_eps, cfg.attn_scale, h.ws_rows, cfg.attn_kind == FLAME_GR_ATTN_SOFTMAX ? 1 : 0,
               cfg.latency_mode ? 1 : 0};
  const size_t rows = (size_t)h.ws_rows, d = (size_t)cfg.d_model, e = h.elt, L = (size_t)cfg.n_layers;
  Carver c;
  if (bf) {
    h.Xb = base + c.take(2 * rows * d * e);
    h.Xl = (char *)h.Xb + rows * d * e;
  } else {
    h.X = (float *)(base + c.take(rows * d * sizeof(float)));
  }
  h.plane_bytes = rows * d * e;
  h.planes = base + c.take(4 * h.plane_bytes);
  h.O = base + c.take(rows * d * e);
  if (!bf || !k3_fused_supported(cfg.d_model)) h.G = base + c.take(rows * d * e);
  if (bf) {
    h.W1h = base + c.take(L * 4 * d * d * e);
    void *w2 = base + c.take(L * d * d * e);
    h.W2h = w2;
    h.W2p = w2;                                   // one of the two layouts is used, by the model width
  }
  h.bias = (float *)(base + c.take(L * (size_t)cfg.n_heads * (size_t)cfg.max_rel_dist * sizeof(float)));
  h.bucket_tab = (int32_t *)(base + c.take((size_t)cfg.max_rel_dist * sizeof(int32_t)));
  h.tscale = (float *)(base + c.take(L * (size_t)cfg.n_heads * sizeof(float)));
  if (!h.sh.softmax) h.tscale = nullptr;
  h.lay = stage_layout(rows / kRowAlign);
  h.stage_dev = (char *)(base + c.take(h.lay.total));
  if ((int64_t)c.off != need) { g_create_error = "internal: static workspace layout mismatch"; return FLAME_GR_HIP_ERROR; }
  if (h.sh.latency && bf && attn_latency_setup(h.sh) != hipSuccess) { g_create_error = "attention kernel setup failed"; return FLAME_GR_HIP_ERROR; }
  hipStream_t s = (hipStream_t)stream_v;
  // plan tables as kernel arguments, bucket table computed on the device: no copies, no memsets, no events
  launch_upload_words(P.blocks.data(), P.blocks.size() * sizeof(RowBlock), h.stage_dev + h.lay.blocks, s);
  launch_upload_words(P.items.data(), P.items.size() * sizeof(AttnItem), h.stage_dev + h.lay.items, s);
  launch_upload_words(P.cand_items.data(), P.cand_items.size() * sizeof(AttnItem), h.stage_dev + h.lay.cand_items, s);
  launch_upload_words(P.cand_blocks.data(), P.cand_blocks.size() * sizeof(int32_t), h.stage_dev + h.lay.cand_blocks, s);
  launch_bucket_table(cfg.n_buckets, cfg.max_rel_dist, h.bucket_tab, s);
  derive_weights(&h, w, s);
  // The array keeps the last call's contents, laid out for another batch: every row of this batch's blocks is
  // rewritten by the kernels below, and the rows behind them, which whole-tile key loads may read, are cleared.
  if (bf) launch_clear_spare((char *)h.planes + 3 * h.plane_bytes, (char *)h.planes + h.plane_bytes, cfg.d_model, h.ws_rows,
                             P.total_rows, (int)(h.ws_rows - P.total_rows), s);
  run_group(&h, *w, P.groups[0], history_emb, cand_emb, scores, s, PASS_FULL);
  const hipError_t le = hipGetLastError();
  h.magic = 0;
  if (le != hipSuccess) { g_create_error = std::string("kernel launch: ") + hipGetErrorString(le); return FLAME_GR_HIP_ERROR; }
  return FLAME_GR_OK;
}

// ---------------------------------------------------------------------------------------------
// host-only helpers
// ---------------------------------------------------------------------------------------------
int flame_gr_host_bucket_table(int32_t n_buckets, int32_t max_rel_dist, int32_t *out) {
  flame_gr_config c{};
  c.n_layers = 1; c.d_model = 1; c.n_heads = 1; c.n_buckets = n_buckets; c.max_rel_dist = max_rel_dist;
  std::string err;
  if (!out) return FLAME_GR_INVALID_ARGUMENT;
  int rc = validate_config(c, err);
  if (rc) { g_create_error = err; return rc; }
  bucket_table(n_buckets, max_rel_dist, out);
  return FLAME_GR_OK;
}

int flame_gr_host_mask(int32_t L, int32_t M, int32_t n_buckets, int32_t max_rel_dist, uint8_t *mask, int32_t *bucket) {
  if (L < 0 || M < 0 || !mask) return FLAME_GR_INVALID_ARGUMENT;
  std::vector<int32_t> tab;
  if (bucket) {
    tab.resize(max_rel_dist > 0 ? max_rel_dist : 0);
    int rc = flame_gr_host_bucket_table(n_buckets, max_rel_dist, tab.data());
    if (rc) return rc;
  }
  const int64_t N = (int64_t)L + M;
  for (int64_t r = 0; r < N; ++r)
    for (int64_t c = 0; c < N; ++c) {
      const bool ok = allowed((int32_t)r, (int32_t)c, L);
      mask[r * N + c] = ok;
      if (bucket) {
        const int32_t pr = r < L ? (int32_t)r : L, pc = c < L ? (int32_t)c : L;
        int32_t delta = pr - pc;
        if (delta > max_rel_dist - 1) delta = max_rel_dist - 1;
        bucket[r * N + c] = ok ? tab[delta] : -1;
      }
    }
  return FLAME_GR_OK;
}

static int host_plan(const flame_gr_config *cfg_in, const int32_t *history_offsets, const int32_t *cand_offsets,
                     const int32_t *cand_capacity, int32_t n_requests, int32_t *tok_off, int32_t *n_segments,
                     int32_t *seg, int32_t cap_segments) {
  if (!cfg_in) return FLAME_GR_INVALID_ARGUMENT;
  flame_gr_config cfg = *cfg_in;
  std::string err;
  int rc = validate_config(cfg, err);
  if (!rc) {
    Plan P;
    const int q_tile = cfg.dtype == FLAME_GR_BF16 ? kAttnQTileBf16 : kAttnQTileF32;
    rc = build_plan(cfg, history_offsets, cand_offsets, n_requests, q_tile, cfg.n_streams > 1 ? cfg.n_streams : 1,
                    workspace_rows(cfg), P, err, cand_capacity);
    if (!rc) {
      if (tok_off) std::memcpy(tok_off, P.tok_off.data(), P.tok_off.size() * sizeof(int32_t));
      if (n_segments) *n_segments = (int32_t)P.segs.size();
      if (seg) {
        if ((int32_t)P.segs.size() > cap_segments) { g_create_error = "cap_segments too small"; return FLAME_GR_CAPACITY_EXCEEDED; }
        for (size_t i = 0; i < P.segs.size(); ++i) {
          const Segment &s = P.segs[i];
          int32_t *o = seg + 6 * i;
          o[0] = s.req; o[1] = s.L; o[2] = s.cand_begin; o[3] = s.M; o[4] = s.row_start; o[5] = s.group;
        }
      }
    }
  }
  if (rc) g_create_error = err;
  return rc;
}

int flame_gr_host_workspace_rows(const flame_gr_config *cfg_in, int64_t *rows) {
  if (!cfg_in || !rows) { g_create_error = "cfg or rows is NULL"; return FLAME_GR_INVALID_ARGUMENT; }
  std::string err;
  const int rc = validate_config(*cfg_in, err);
  if (rc) { g_create_error = err; return rc; }
  *rows = workspace_rows(*cfg_in);
  return FLAME_GR_OK;
}

int flame_gr_host_plan(const flame_gr_config *cfg_in, const int32_t *history_offsets, const int32_t *cand_offsets,
                       int32_t n_requests, int32_t *tok_off, int32_t *n_segments, int32_t *seg, int32_t cap_segments) {
  return host_plan(cfg_in, history_offsets, cand_offsets, nullptr, n_requests, tok_off, n_segments, seg, cap_segments);
}

int flame_gr_host_plan_reserved(const flame_gr_config *cfg_in, const int32_t *history_offsets,
                                const int32_t *cand_offsets, const int32_t *cand_capacity, int32_t n_requests,
                                int32_t *n_segments, int32_t *seg, int32_t cap_segments) {
  if (n_requests > 0 && !cand_capacity) { g_create_error = "cand_capacity is NULL"; return FLAME_GR_INVALID_ARGUMENT; }
  static const int32_t none = 0;
  return host_plan(cfg_in, history_offsets, cand_offsets, n_requests > 0 ? cand_capacity : &none, n_requests, nullptr,
                   n_segments, seg, cap_segments);
}

// ---------------------------------------------------------------------------------------------
// debug exports
// ---------------------------------------------------------------------------------------------
int flame_gr_debug_capture(flame_gr_t *h, int32_t layer) {
  if (!live(h)) return FLAME_GR_BAD_HANDLE;
  if (layer >= h->cfg.n_layers) { h->err = "layer out of range"; return FLAME_GR_INVALID_ARGUMENT; }
  h->capture_layer = layer < 0 ? -1 : layer;
  h->cap_valid = false;
  if (layer >= 0 && !h->cap_planes) {
    const size_t n = (size_t)h->ws_rows * h->sh.d;
    HIP_TRY(h, hipMalloc(&h->cap_planes, 4 * n * h->elt));
    HIP_TRY(h, hipMalloc(&h->cap_O, n * h->elt));
    HIP_TRY(h, hipMalloc((void **)&h->cap_X, n * sizeof(float)));
  }
  return FLAME_GR_OK;
}

int flame_gr_debug_stage(flame_gr_t *h, int32_t which, float *host_out) {
  if (!live(h)) return FLAME_GR_BAD_HANDLE;
  if (!h->cap_valid) { h->err = "no captured forward"; return FLAME_GR_INVALID_ARGUMENT; }
  if (which < 0 || which > 5 || !host_out) { h->err = "bad stage selector"; return FLAME_GR_INVALID_ARGUMENT; }
  if (h->plan.split) { h->err = "stage export needs unsplit requests"; return FLAME_GR_UNSUPPORTED; }
  HIP_TRY(h, hipEventSynchronize(h->ev_done));
  const size_t d = h->sh.d, rows = (size_t)h->plan.total_rows, e = h->elt, wsr = (size_t)h->ws_rows;
  const bool bf = h->cfg.dtype == FLAME_GR_BF16;
  const bool transposed = bf && which == 1;
  std::vector<char> raw;
  size_t esz = which == 5 ? 4 : e;
  if (transposed) {
    raw.resize(wsr * d * e);
    HIP_TRY(h, hipMemcpy(raw.data(), (char *)h->cap_planes + wsr * d * e, raw.size(), hipMemcpyDeviceToHost));
  } else {
    raw.resize(rows * d * esz);
    const void *src = which < 4 ? (const void *)((char *)h->cap_planes + (size_t)which * wsr * d * e)
                      : which == 4 ? h->cap_O : (const void *)h->cap_X;
    HIP_TRY(h, hipMemcpy(raw.data(), src, raw.size(), hipMemcpyDeviceToHost));
  }
  // the MFMA path stores Q times alpha/2: report the plain tensor
  const float unscale = bf && which == 2 ? 2.0f / h->sh.alpha : 1.0f;
  auto get = [&](size_t row, size_t k) -> float {
    if (esz == 4) return ((const float *)raw.data())[row * d + k];
    const uint16_t *p = (const uint16_t *)raw.data();
    return unscale * half_bits_to_float(transposed ? p[k * wsr + row] : p[row * d + k]);
  };
  // segments are in workspace order; the output is in request order (merged token offsets)
  for (const Segment &s : h->plan.segs) {
    float *dst = host_out + (size_t)h->plan.tok_off[s.req] * d;
    for (int32_t t = 0; t < s.L; ++t)
      for (size_t k = 0; k < d; ++k) dst[(size_t)t * d + k] = get((size_t)s.row_start + t, k);
    for (int32_t j = 0; j < s.M; ++j)
      for (size_t k = 0; k < d; ++k) dst[(size_t)(s.L + j) * d + k] = get((size_t)s.row_start + s.Lp + j, k);
  }
  return FLAME_GR_OK;
}

int flame_gr_debug_device_mask(flame_gr_t *h, int32_t L, int32_t M, uint8_t *mask, int32_t *bucket) {
  if (!live(h)) return FLAME_GR_BAD_HANDLE;
  if (L < 0 || M < 0 || !mask) { h->err = "bad arguments"; return FLAME_GR_INVALID_ARGUMENT; }
  const size_t n = (size_t)(L + M) * (L + M);
  if (n == 0) return FLAME_GR_OK;
  uint8_t *dm = nullptr;
  int32_t *db = nullptr;
  HIP_TRY(h, hipMalloc((void **)&dm, n));
  if (bucket) {
    hipError_t e_ = hipMalloc((void **)&db, n * sizeof(int32_t));
    if (e_ != hipSuccess) { (void)hipFree(dm); h->err = "hipMalloc failed"; return FLAME_GR_HIP_ERROR; }
  }
  launch_debug_mask(L, M, h->bucket_tab, h->sh.D, dm, db, nullptr);
  hipError_t e1 = hipMemcpy(mask, dm, n, hipMemcpyDeviceToHost);
  hipError_t e2 = bucket ? hipMemcpy(bucket, db, n * sizeof(int32_t), hipMemcpyDeviceToHost) : hipSuccess;
  (void)hipFree(dm);
  (void)hipFree(db);
  if (e1 != hipSuccess || e2 != hipSuccess) { h->err = "debug mask copy failed"; return FLAME_GR_HIP_ERROR; }
  return FLAME_GR_OK;
}

int flame_gr_debug_profile(flame_gr_t *h, int32_t enable) {
  if (!live(h)) return FLAME_GR_BAD_HANDLE;
  h->profiling = enable != 0;
  h->prof_used = 0;
  return FLAME_GR_OK;
}

int flame_gr_debug_profile_read(flame_gr_t *h, float *ms_by_kind, int32_t *launches_by_kind) {
  if (!live(h)) return FLAME_GR_BAD_HANDLE;
  if (!ms_by_kind || !launches_by_kind) { h->err = "NULL output"; return FLAME_GR_INVALID_ARGUMENT; }
  for (int k = 0; k < KIND_COUNT; ++k) { ms_by_kind[k] = 0.f; launches_by_kind[k] = 0; }
  if (h->has_prev) HIP_TRY(h, hipEventSynchronize(h->ev_done));
  for (size_t i = 0; i < h->prof_used; ++i) {
    float ms = 0.f;
    HIP_TRY(h, hipEventElapsedTime(&ms, h->prof_pool[i].a, h->prof_pool[i].b));
    ms_by_kind[h->prof_pool[i].kind] += ms;
    launches_by_kind[h->prof_pool[i].kind] += 1;
  }
  h->prof_used = 0;
  return FLAME_GR_OK;
}

}  // extern "C"
