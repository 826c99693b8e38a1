// Jagged masked pointwise-SiLU attention with relative-position bias, fp16 MFMA (fp32 accumulation), gfx950.
//
// For every query row r of a request and every head:
//     O_r = sum over allowed keys c of silu(<Q_r, K_c> + bias[p_r - p_c]) V_c
// Q arrives multiplied by alpha*log2(e), the bias table by log2(e) and V by ln(2), so the logits are
// directly exp2 arguments: silu costs exp2, add, rcp, mul and the scale factors cancel in O.  History rows look at keys 0..r, candidate rows look at the
// whole history and at themselves: the customised mask of Section 3.2 that lets all candidates of
// a request be scored in one pass.  No score matrix is materialised: like a flash-attention tile
// loop, but the pointwise SiLU needs neither running maximum nor rescaling.
//
// Work decomposition: one workgroup = (query tile of 128 rows, head); 4 wavefronts, 32 query rows
// each; keys are walked in tiles of 64 staged through LDS (double buffered).
//
// Register-level formulation: the products are computed transposed,
//     S^T[kv][q] = K Q^T      (A operand = K rows, B operand = Q rows)
//     O^T[d][q] += V^T P^T    (A operand = V^T rows, B operand = P^T)
// so that the accumulator of the first product, where a lane holds one query column and 16 key
// rows, already has the register layout of the second product's B operand.  The only thing to
// arrange is which key goes to which MFMA row: feeding key row pi(m) = m with bits 2 and 3 swapped
// into MFMA row m makes accumulator elements 8s..8s+7 of a lane hold keys 16s+8*(lane/32)+0..7, which
// is exactly the k order of a 16-deep B operand.  V is stored feature-major by the projection
// kernel, so V^T tiles are plain row loads.
#include "device_common.h"
#include "kernels.h"

namespace flame {

namespace {

constexpr int QT = kAttnQTileBf16;  // query rows per workgroup (4 wavefronts x 32)
static_assert(QT == 128, "4 wavefronts of 32 query rows");
constexpr int KT = 64;       // keys per tile
constexpr int PAD = 8;       // fp16 elements of LDS row padding
constexpr int BW = 192;      // bias window per key tile, stored by decreasing distance:
                             // slot u holds bias[q_first + 127 - k0 - u], u = 0..191

__device__ __forceinline__ int pi32(int m) {  // swap bits 2 and 3
  return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1);
}

// eight attention weights -> fp16 B-operand fragment (v_cvt_pk_f16_f32, round to nearest even).
// A weight beyond the fp16 range becomes inf; the output store saturates, so nothing non-finite is
// ever written to the workspace.
__device__ __forceinline__ f16x8 pack8(const float *v) {
  f16x8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = (half_t)v[i];
  return r;
}

template <int DH>
__global__ __launch_bounds__(256) void attn_bf16_kernel(const half_t *__restrict__ planes, const float *__restrict__ bias_lh,
                                                        half_t *__restrict__ O, const AttnItem *__restrict__ items,
                                                        int H, int d, int D, int64_t ws_rows) {
  constexpr int KS = DH / 16;          // k-steps of the Q K^T product
  constexpr int DB = DH / 32;          // 32-row blocks of O^T
  constexpr int NCH = DH / 32;         // 16-byte chunks per thread for one K (or V^T) tile
  __shared__ __attribute__((aligned(16))) half_t sK[2][KT][DH + PAD];
  __shared__ __attribute__((aligned(16))) half_t sVt[2][DH][KT + PAD];
  __shared__ float sBias[2][BW];

  const int head = blockIdx.x % H;
  const AttnItem it = items[blockIdx.x / H];
  const int tid = threadIdx.x, lane = tid & 63;
  // wavefront index as a scalar: every branch on it is then a uniform (scalar) branch
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lhalf = lane >> 5;

  const int64_t plane = ws_rows * d;
  const half_t *Vt = planes + 1 * plane + (int64_t)head * DH * ws_rows;   // [DH][ws_rows]
  const half_t *Qp = planes + 2 * plane + head * DH;                      // [row][d]
  const half_t *Kp = planes + 3 * plane + head * DH;
  const float *bias = bias_lh + (int64_t)head * D;

  // this wavefront's 32 query rows
  const int q_local0 = wave * 32;
  const bool wave_active = q_local0 < it.n_q;
  const int my_q_local = q_local0 + l32;
  const bool row_valid = my_q_local < it.n_q;
  const int64_t my_row = it.q_row + (row_valid ? my_q_local : it.n_q - 1);   // clamped for loads
  // position of my query row; number of history keys it may see
  const int q_index = it.is_cand ? it.L : it.q_pos + my_q_local;
  const int n_vis = visible_history(it.is_cand, q_index, it.L);
  const int wave_vis_min = it.is_cand ? it.L : it.q_pos + q_local0 + 1;
  const int wave_vis_max = it.is_cand ? it.L : it.q_pos + q_local0 + 32;

  // Q fragments (B operand of S^T): row = my query, k = 16*s + 8*lhalf + 0..7
  f16x8 fq[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) fq[s] = *(const f16x8 *)(Qp + my_row * d + s * 16 + lhalf * 8);

  f32x16 oacc[DB];
#pragma unroll
  for (int b = 0; b < DB; ++b)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[b][e] = 0.f;

  const int n_tiles = (it.n_kv + KT - 1) / KT;
  const int q_first = it.is_cand ? it.L : it.q_pos;     // position of query row 0 of the workgroup tile

  // global -> register -> LDS staging of one key tile: per-thread source pointers at tile 0 and LDS
  // destinations are fixed; every iteration prefetches unconditionally (the last one re-reads its
  // own tile) so that the staging registers never live across a branch.
  const half_t *gK[NCH];
  const half_t *gV[NCH];
  int oK[NCH], oV[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = tid + i * 256;
    const int r = c / (DH / 8), c8 = c % (DH / 8);
    gK[i] = Kp + (int64_t)(it.kv_row + r) * d + c8 * 8;
    oK[i] = r * (DH + PAD) + c8 * 8;
    const int rr = c >> 3, cc = c & 7;
    gV[i] = Vt + (int64_t)rr * ws_rows + it.kv_row + cc * 8;
    oV[i] = rr * (KT + PAD) + cc * 8;
  }
  const int bias_t = tid < BW ? tid : BW - 1;
  const int delta0 = q_first + (QT - 1) - bias_t;       // distance held by window slot bias_t for tile 0
  uint4 rk[NCH], rv[NCH];
  float rbias;
#define ATTN_LOAD_TILE(T)                                                                   \
  {                                                                                         \
    const int k0_ = (T) * KT;                                                               \
    _Pragma("unroll") for (int i = 0; i < NCH; ++i) {                                       \
      rk[i] = *(const uint4 *)(gK[i] + (int64_t)k0_ * d);                                   \
      rv[i] = *(const uint4 *)(gV[i] + k0_);                                                \
    }                                                                                       \
    int dl_ = delta0 - k0_;                                                                 \
    dl_ = dl_ < 0 ? 0 : (dl_ > D - 1 ? D - 1 : dl_);                                        \
    rbias = bias[dl_];                                                                      \
  }
#define ATTN_STORE_TILE(BUF)                                                                \
  {                                                                                         \
    _Pragma("unroll") for (int i = 0; i < NCH; ++i) {                                       \
      *(uint4 *)(&sK[BUF][0][0] + oK[i]) = rk[i];                                           \
      *(uint4 *)(&sVt[BUF][0][0] + oV[i]) = rv[i];                                          \
    }                                                                                       \
    sBias[BUF][bias_t] = rbias;                                                             \
  }

  if (n_tiles > 0) {
    ATTN_LOAD_TILE(0);
    ATTN_STORE_TILE(0);
  }
  __syncthreads();

  // window slot of (my row, key 0 of the tile); keys further right sit at increasing slots
  const int bias_base = (QT - 1) - (it.is_cand ? 0 : my_q_local) + 8 * lhalf;

  for (int t = 0; t < n_tiles; ++t) {
    const int buf = t & 1;
    const int k0 = t * KT;
    const int tn = t + 1 < n_tiles ? t + 1 : t;
    ATTN_LOAD_TILE(tn);
    __builtin_amdgcn_sched_barrier(0);   // the prefetch stays ahead of the tile's arithmetic
    if (wave_active && k0 < wave_vis_max) {
      // ---- S^T = K Q^T + bias, two blocks of 32 keys
      f32x16 sacc[2];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[j][e] = sBias[buf][bias_base + 32 * j + 16 * (e >> 3) + (e & 7)];
#pragma unroll
      for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const f16x8 fk = *(const f16x8 *)&sK[buf][32 * j + pi32(l32)][s * 16 + lhalf * 8];
          sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fk, fq[s], sacc[j], 0, 0, 0);
        }
      // ---- P^T = silu(S^T), masked where the tile reaches past what a row may see
      const bool need_mask = k0 + KT > wave_vis_min;
      f16x8 fp[4];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        float p[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) p[e] = silu_log2_domain(sacc[j][e]);
        if (need_mask) {
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int kv = k0 + 32 * j + 16 * (e >> 3) + 8 * lhalf + (e & 7);
            p[e] = kv < n_vis ? p[e] : 0.f;
          }
        }
        fp[2 * j] = pack8(p);
        fp[2 * j + 1] = pack8(p + 8);
      }
      // ---- O^T += V^T P^T
#pragma unroll
      for (int s2 = 0; s2 < 4; ++s2)
#pragma unroll
        for (int b = 0; b < DB; ++b) {
          const f16x8 fv = *(const f16x8 *)&sVt[buf][32 * b + l32][s2 * 16 + lhalf * 8];
          oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fv, fp[s2], oacc[b], 0, 0, 0);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    ATTN_STORE_TILE(buf ^ 1);
    __syncthreads();
  }
#undef ATTN_LOAD_TILE
#undef ATTN_STORE_TILE

  // ---- candidates: the row itself is one more key, at distance 0.  Each wavefront multiplies its
  // 32 candidate rows against themselves and keeps the diagonal.
  if (it.is_cand && wave_active) {
    const int64_t base_row = it.q_row + q_local0;        // multiple of 32 inside the padded workspace
    f32x16 sacc;
    const float b0 = bias[0];
#pragma unroll
    for (int e = 0; e < 16; ++e) sacc[e] = b0;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const f16x8 fk = *(const f16x8 *)(Kp + (base_row + pi32(l32)) * d + s * 16 + lhalf * 8);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(fk, fq[s], sacc, 0, 0, 0);
    }
    float p[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int kv_local = 16 * (e >> 3) + 8 * lhalf + (e & 7);
      p[e] = (kv_local == l32 && row_valid) ? silu_log2_domain(sacc[e]) : 0.f;
    }
    f16x8 fp[2] = {pack8(p), pack8(p + 8)};
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int b = 0; b < DB; ++b) {
        const f16x8 fv = *(const f16x8 *)(Vt + (int64_t)(32 * b + l32) * ws_rows + base_row + s2 * 16 + lhalf * 8);
        oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fv, fp[s2], oacc[b], 0, 0, 0);
      }
  }

  // ---- write O[q][head*DH + dd]; accumulator element e of block b: dd = 32b + 8*(e/4) + 4*lhalf + e%4
  if (row_valid) {
    half_t *orow = O + (it.q_row + my_q_local) * (int64_t)d + head * DH;
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f16x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = to_f16_sat(oacc[b][4 * g + i]);
        *(f16x4 *)(orow + 32 * b + 8 * g + 4 * lhalf) = v;
      }
  }
}

}  // namespace

void launch_attn_bf16(const void *planes, const float *bias_lh, void *O, const AttnItem *items, int n_items,
                      const Shape &sh, hipStream_t s) {
  if (n_items <= 0) return;
  const int grid = n_items * sh.H;
#define ATTN_CASE(DHV) attn_bf16_kernel<DHV><<<grid, 256, 0, s>>>((const half_t *)planes, bias_lh, (half_t *)O, items, sh.H, sh.d, sh.D, sh.ws_rows)
  if (sh.dh == 32) ATTN_CASE(32);
  else if (sh.dh == 64) ATTN_CASE(64);
  else ATTN_CASE(128);
#undef ATTN_CASE
}

}  // namespace flame
