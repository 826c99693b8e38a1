// Host-side planner of the jagged GR forward: integer work only, no HIP.
//
// A batch of requests (history length L_i, candidate count M_i: Sections 1 and 3.3 of the paper)
// becomes a list of segments laid out in one padded token workspace, plus the work lists the
// kernels consume.  The mask and the relative-position bucket function (Section 3.2's customised
// mask; bucket function as documented in flame_gr.h) also live here so that host tests can
// compare them bit for bit with an independent implementation.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/flame_gr.h"

namespace flame {

constexpr int kRowAlign = 64;  // history part and candidate part of a segment start on multiples of this
constexpr int kSpareRows = 256;  // rows at the end of every workspace that no plan places a segment in

struct Segment {
  int32_t req;        // request index in the caller's batch
  int32_t L;          // history length
  int32_t cand_begin; // first candidate (relative to the request) handled here
  int32_t M;          // number of candidates handled here
  int32_t row_start;  // first workspace row (history row 0)
  int32_t Lp;         // L rounded up to kRowAlign: candidates start at row_start + Lp
  int32_t Mp;         // M rounded up to kRowAlign
  int32_t group;      // stream group
  int64_t cost;       // model cost, 10*N*d^2 + 4*P*d
};

// One 64-row block of the workspace: where its rows come from.
struct RowBlock {
  int32_t src_row;  // first source row in history_emb (kind 0) or cand_emb (kind 1)
  int32_t n_valid;  // rows [0, n_valid) of the block are real tokens, the rest is zero padding
  int32_t kind;     // 0 history, 1 candidate
  int32_t seg;      // owning segment
};

// One attention work item: a tile of query rows of one segment (all heads run it).
struct AttnItem {
  int32_t q_row;    // workspace row of the first query
  int32_t n_q;      // valid query rows in the tile (<= tile height)
  int32_t kv_row;   // workspace row of the segment's history row 0
  int32_t L;        // history length of the segment
  int32_t q_pos;    // position of the first query row: its history index, or L for candidate tiles
  int32_t is_cand;  // 1: rows are candidates (see all L history keys + themselves)
  int32_t n_kv;     // number of history keys the tile can see (causal upper bound)
  int32_t pad;
};

struct Group {
  int32_t row_begin, row_end;          // workspace rows [begin, end) of this stream group (multiples of 64)
  int32_t blk_begin, blk_end;          // RowBlock range
  int32_t item_begin, item_end;        // AttnItem range, all layers but the last
  int32_t citem_begin, citem_end;      // AttnItem range of candidate tiles only (last layer, score stage)
  int32_t cblk_begin, cblk_end;        // range in cand_blocks (last-layer row pruning, score head, score stage)
  int32_t hitem_begin, hitem_end;      // AttnItem range of history tiles only (prefill stage)
  int32_t hblk_begin, hblk_end;        // range in hist_blocks (prefill stage)
};

struct Plan {
  std::vector<int32_t> tok_off;        // logical merged offsets, [B+1]
  std::vector<Segment> segs;           // in workspace order
  std::vector<RowBlock> blocks;        // total_rows / 64 entries
  std::vector<AttnItem> items;         // per group: cost-descending
  std::vector<AttnItem> cand_items;    // candidate tiles only
  std::vector<int32_t> cand_blocks;    // indices of candidate RowBlocks with valid rows, per group contiguous
  std::vector<AttnItem> hist_items;    // history tiles only
  std::vector<int32_t> hist_blocks;    // indices of history RowBlocks, per group contiguous
  std::vector<Group> groups;
  int32_t total_rows = 0;
  int64_t total_cands = 0;
  bool split = false;                  // some request was split into several segments
};

// Validation + planning.  q_tile = query rows per attention item.  Returns a flame_gr_status;
// on failure `err` holds the reason.
int validate_config(const flame_gr_config &cfg, std::string &err);
// cand_capacity (optional, [B]): rows are reserved for that many candidates per request (>= the actual
// count), and layout and stream groups depend on the capacities only, not on the actual counts: the plans
// of a prefill (no candidates yet) and of the score calls that follow it then agree on every row.
int build_plan(const flame_gr_config &cfg, const int32_t *hoff, const int32_t *coff, int32_t B,
               int32_t q_tile, int32_t n_groups, int64_t ws_rows, Plan &plan, std::string &err,
               const int32_t *cand_capacity = nullptr);

// bucket(delta) for delta in [0, D)
void bucket_table(int32_t n_buckets, int32_t D, int32_t *out);
int32_t bucket_of(int32_t delta, int32_t n_buckets, int32_t D);

// The mask predicate, on (row, col) token indices of a request with L history items.
inline bool allowed(int32_t r, int32_t c, int32_t L) {
  return r < L ? (c <= r) : (c < L || c == r);
}

// Workspace rows needed for a capacity (used at create).
int64_t workspace_rows(const flame_gr_config &cfg);

}  // namespace flame
