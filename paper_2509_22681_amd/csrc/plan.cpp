// Host-side planner: see plan.h.
#include "plan.h"

#include <algorithm>
#include <numeric>

namespace flame {

static bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }
static int ilog2(int64_t v) {
  int e = 0;
  while ((int64_t(1) << (e + 1)) <= v) ++e;
  return e;
}
static int32_t round_up(int32_t v, int32_t a) { return (v + a - 1) / a * a; }

int validate_config(const flame_gr_config &c, std::string &err) {
  auto bad = [&](const char *m) { err = m; return (int)FLAME_GR_INVALID_ARGUMENT; };
  if (c.n_layers < 1) return bad("n_layers must be >= 1");
  if (c.d_model < 1 || c.n_heads < 1 || c.d_model % c.n_heads) return bad("d_model must be a positive multiple of n_heads");
  if (!is_pow2(c.n_buckets) || c.n_buckets < 2) return bad("n_buckets must be a power of two >= 2");
  if (!is_pow2(c.max_rel_dist) || c.max_rel_dist < c.n_buckets / 2) return bad("max_rel_dist must be a power of two >= n_buckets/2");
  if (ilog2(c.max_rel_dist) - ilog2(c.n_buckets / 2) > c.n_buckets / 2) return bad("max_rel_dist has more octaves above n_buckets/2 than the far half of the table has buckets");
  if (c.dtype != FLAME_GR_F32 && c.dtype != FLAME_GR_BF16) return bad("dtype must be FLAME_GR_F32 or FLAME_GR_BF16");
  if (c.ln_eps < 0.f || c.attn_scale < 0.f) return bad("ln_eps and attn_scale must be >= 0");
  if (c.max_requests < 0 || c.max_total_tokens < 0 || c.max_seq_tokens < 0) return bad("capacities must be >= 0");
  if (c.n_streams < 0 || c.n_streams > 16) return bad("n_streams must be in [0, 16]");
  if (c.kv_cache != 0 && c.kv_cache != 1) return bad("kv_cache must be 0 or 1");
  if (c.latency_mode != 0 && c.latency_mode != 1) return bad("latency_mode must be 0 or 1");
  if (c.weights_static != 0 && c.weights_static != 1) return bad("weights_static must be 0 or 1");
  if (c.attn_kind != FLAME_GR_ATTN_SILU && c.attn_kind != FLAME_GR_ATTN_SOFTMAX) return bad("attn_kind must be FLAME_GR_ATTN_SILU or FLAME_GR_ATTN_SOFTMAX");
  if (c.kv_cache && c.dtype != FLAME_GR_BF16) {
    err = "the two-stage path (kv_cache) is built for the bf16 kernels only";
    return FLAME_GR_UNSUPPORTED;
  }
  if (c.dtype == FLAME_GR_BF16) {
    int dh = c.d_model / c.n_heads;
    if (c.d_model % 64 || !(dh == 32 || dh == 64)) {
      err = "bf16 path needs d_model % 64 == 0 and head width 32 or 64";
      return FLAME_GR_UNSUPPORTED;
    }
    // the attention kernel reaches the 32 rows of a V^T request with 32-bit byte offsets from a 64-bit base
    if (workspace_rows(c) >= (int64_t)1 << 26) {
      err = "bf16 path: max_total_tokens (plus padding) must stay below 2^26 rows";
      return FLAME_GR_UNSUPPORTED;
    }
  } else if (c.d_model / c.n_heads > 256) {
    err = "fp32 path needs head width <= 256";
    return FLAME_GR_UNSUPPORTED;
  }
  return FLAME_GR_OK;
}

int32_t bucket_of(int32_t delta, int32_t nb, int32_t D) {
  const int32_t half = nb / 2;
  if (delta > D - 1) delta = D - 1;
  if (delta < half) return delta;
  const int lo = ilog2(half), hi = ilog2(D);
  const int octaves = std::max(hi - lo, 0);
  int sub = lo;  // log2 of sub-buckets per octave
  while (sub > 0 && octaves * (1 << sub) > half) --sub;
  const int oct = ilog2(delta);
  return half + (oct - lo) * (1 << sub) + ((delta - (1 << oct)) >> (oct - sub));
}

void bucket_table(int32_t nb, int32_t D, int32_t *out) {
  for (int32_t t = 0; t < D; ++t) out[t] = bucket_of(t, nb, D);
}

int64_t workspace_rows(const flame_gr_config &c) {
  int64_t rows = (int64_t)c.max_total_tokens + 2ll * (kRowAlign - 1) * std::max(c.max_requests, 1);
  rows = (rows + 255) / 256 * 256 + kSpareRows;  // spare rows that no plan uses: whole-tile loads stay inside
  return rows;
}

int build_plan(const flame_gr_config &cfg, const int32_t *hoff, const int32_t *coff, int32_t B,
               int32_t q_tile, int32_t n_groups, int64_t ws_rows, Plan &p, std::string &err,
               const int32_t *cand_capacity) {
  auto fail = [&](int code, const std::string &m) { err = m; return code; };
  if (B < 0) return fail(FLAME_GR_INVALID_ARGUMENT, "n_requests < 0");
  if (B > 0 && (!hoff || !coff)) return fail(FLAME_GR_INVALID_ARGUMENT, "offset arrays are NULL");
  if (B > cfg.max_requests) return fail(FLAME_GR_CAPACITY_EXCEEDED, "n_requests exceeds max_requests");
  p = Plan();
  p.tok_off.assign(B + 1, 0);
  if (B > 0 && (hoff[0] != 0 || coff[0] != 0)) return fail(FLAME_GR_INVALID_ARGUMENT, "offsets must start at 0");
  int64_t cap_sum = 0;
  for (int i = 0; i < B; ++i) {
    if (hoff[i + 1] < hoff[i] || coff[i + 1] < coff[i])
      return fail(FLAME_GR_INVALID_ARGUMENT, "offsets must be non-decreasing (request " + std::to_string(i) + ")");
    cap_sum += cand_capacity ? std::max(cand_capacity[i], 0) : 0;
    int64_t t = (int64_t)hoff[i + 1] + (cand_capacity ? cap_sum : (int64_t)coff[i + 1]);
    if (t > cfg.max_total_tokens) return fail(FLAME_GR_CAPACITY_EXCEEDED, "total tokens exceed max_total_tokens");
    p.tok_off[i + 1] = (int32_t)t;
  }
  if (n_groups < 1) n_groups = 1;
  const int64_t d = cfg.d_model;

  // 1. segments (descending-size split of over-long requests)
  for (int i = 0; i < B; ++i) {
    const int32_t L = hoff[i + 1] - hoff[i], M = coff[i + 1] - coff[i];
    if (cand_capacity) {
      // reserved layout: one segment per request, candidate rows for the capacity
      const int32_t C = cand_capacity[i];
      if (C < 0) return fail(FLAME_GR_INVALID_ARGUMENT, "negative candidate capacity (request " + std::to_string(i) + ")");
      if (M > C) return fail(FLAME_GR_CAPACITY_EXCEEDED, "request " + std::to_string(i) + " has more candidates than its reserved capacity");
      if (cfg.max_seq_tokens > 0 && L + C > cfg.max_seq_tokens)
        return fail(FLAME_GR_UNSUPPORTED, "a request with reserved candidates would need splitting (max_seq_tokens)");
      Segment s{};
      s.req = i; s.L = L; s.cand_begin = 0; s.M = M;
      s.Lp = round_up(L, kRowAlign); s.Mp = round_up(C, kRowAlign);
      const int64_t N = (int64_t)L + C;
      const int64_t P = (int64_t)L * (L + 1) / 2 + (int64_t)C * (L + 1);
      s.cost = 10 * N * d * d + 4 * P * d;
      p.segs.push_back(s);
      continue;
    }
    int32_t cap = M;
    if (cfg.max_seq_tokens > 0 && L + M > cfg.max_seq_tokens && M > 0) {
      cap = cfg.max_seq_tokens - L;
      if (cap < 1) return fail(FLAME_GR_CAPACITY_EXCEEDED, "history of request " + std::to_string(i) + " leaves no room for a candidate within max_seq_tokens");
    }
    int32_t done = 0;
    do {
      Segment s{};
      s.req = i; s.L = L; s.cand_begin = done; s.M = std::min(cap, M - done);
      s.Lp = round_up(L, kRowAlign); s.Mp = round_up(s.M, kRowAlign);
      const int64_t N = (int64_t)L + s.M;
      const int64_t P = (int64_t)L * (L + 1) / 2 + (int64_t)s.M * (L + 1);
      s.cost = 10 * N * d * d + 4 * P * d;
      p.segs.push_back(s);
      done += s.M;
      if (done < M) p.split = true;
    } while (done < M);
  }

  // 2. stream groups: longest-processing-time first onto the least loaded group
  std::vector<int> order(p.segs.size());
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return p.segs[a].cost > p.segs[b].cost; });
  std::vector<int64_t> load(n_groups, 0);
  for (int idx : order) {
    int g = (int)(std::min_element(load.begin(), load.end()) - load.begin());
    p.segs[idx].group = g;
    load[g] += p.segs[idx].cost;
  }
  std::vector<Segment> sorted;
  sorted.reserve(p.segs.size());
  for (int g = 0; g < n_groups; ++g)
    for (int idx : order)
      if (p.segs[idx].group == g) sorted.push_back(p.segs[idx]);
  p.segs.swap(sorted);

  // 3. rows, blocks, work items
  p.groups.assign(n_groups, Group{});
  int64_t row = 0;
  size_t si = 0;
  for (int g = 0; g < n_groups; ++g) {
    Group &G = p.groups[g];
    G.row_begin = (int32_t)row;
    G.blk_begin = (int32_t)p.blocks.size();
    G.item_begin = (int32_t)p.items.size();
    G.citem_begin = (int32_t)p.cand_items.size();
    G.cblk_begin = (int32_t)p.cand_blocks.size();
    G.hitem_begin = (int32_t)p.hist_items.size();
    G.hblk_begin = (int32_t)p.hist_blocks.size();
    for (; si < p.segs.size() && p.segs[si].group == g; ++si) {
      Segment &s = p.segs[si];
      // The last kSpareRows rows of the workspace stay out of every plan: key tiles of up to 128 rows are loaded
      // whole, so the tile that starts inside the last segment may reach that far past its end.  (Unsplit
      // batches within the create-time capacities always fit; a split batch repeats histories and may not.)
      if (row + s.Lp + s.Mp > ws_rows - kSpareRows) return fail(FLAME_GR_CAPACITY_EXCEEDED, "padded batch does not fit the workspace sized at create");
      s.row_start = (int32_t)row;
      for (int32_t b = 0; b < s.Lp; b += kRowAlign) {
        p.hist_blocks.push_back((int32_t)p.blocks.size());
        p.blocks.push_back(RowBlock{hoff[s.req] + b, std::min(kRowAlign, s.L - b), 0, (int32_t)si});
      }
      for (int32_t b = 0; b < s.Mp; b += kRowAlign) {
        // reserved rows past the actual candidates form blocks without valid rows: not in the work lists
        const int32_t nv = std::max(0, std::min(kRowAlign, s.M - b));
        if (nv > 0) p.cand_blocks.push_back((int32_t)p.blocks.size());
        p.blocks.push_back(RowBlock{coff[s.req] + s.cand_begin + b, nv, 1, (int32_t)si});
      }
      // candidate tiles first (they see the whole history), then history tiles from the end
      for (int32_t j = 0; j < s.M; j += q_tile) {
        AttnItem it{s.row_start + s.Lp + j, std::min(q_tile, s.M - j), s.row_start, s.L, s.L, 1, s.L, 0};
        p.items.push_back(it);
        p.cand_items.push_back(it);
      }
      for (int32_t q0 = (s.L - 1) / q_tile * q_tile; s.L > 0 && q0 >= 0; q0 -= q_tile) {
        const int32_t nq = std::min(q_tile, s.L - q0);
        AttnItem it{s.row_start + q0, nq, s.row_start, s.L, q0, 0, q0 + nq, 0};
        p.items.push_back(it);
        p.hist_items.push_back(it);
      }
      row += s.Lp + s.Mp;
      p.total_cands += s.M;
    }
    G.row_end = (int32_t)row;
    G.blk_end = (int32_t)p.blocks.size();
    G.item_end = (int32_t)p.items.size();
    G.citem_end = (int32_t)p.cand_items.size();
    G.cblk_end = (int32_t)p.cand_blocks.size();
    G.hitem_end = (int32_t)p.hist_items.size();
    G.hblk_end = (int32_t)p.hist_blocks.size();
  }
  p.total_rows = (int32_t)row;
  return FLAME_GR_OK;
}

}  // namespace flame
