// Jagged masked pointwise-SiLU attention with relative-position bias, fp16 MFMA (fp32 accumulation), gfx950.
//
// For every query row r of a request and every head:
//     O_r = sum over allowed keys c of silu(<Q_r, K_c> + bias[p_r - p_c]) V_c
// Q arrives multiplied by alpha/2 and the bias table by 1/2, so the kernel sees halved logits s = x/2
// (both factors are powers of two for the usual alpha: no rounding).  History rows look at keys 0..r,
// candidate rows look at the whole history and at themselves: the customised mask of Section 3.2
// that lets all candidates of a request be scored in one pass.  No score matrix is materialised:
// like a flash-attention tile loop, but the pointwise SiLU needs neither running maximum nor
// rescaling.
//
// Work decomposition: one workgroup = (query tile of 128 rows, head); 4 wavefronts of 32 query rows
// (one 32-row MFMA block each: about 160 registers per lane and 51 KB of LDS per workgroup, so three
// workgroups = three wavefronts per SIMD fit a CU; the kernel is bound by MFMA + VALU issue, and a third
// wavefront per SIMD fills part of the issue slots that two leave empty: measured 1.46x from one to two,
// 1.04x from two to three, the latter net of twice the K/V tile traffic of 256-row query tiles).  Keys
// are walked in tiles of 64.  A tile (K rows, V^T rows and the window of the bias table it needs) is
// brought into a ring of three LDS stages by LDS-DMA loads (global_load_lds: no staging registers, no
// LDS store instructions), requested two tiles ahead right after the barrier that opens the current
// tile.  LDS rows are unpadded (a DMA instruction fills 1 KB of consecutive LDS) and 16-byte chunks are
// XOR-swizzled so that 16 consecutive lanes of a fragment read fall into 16 different slots of the 256
// bytes the LDS serves per clock.
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
//
// SiLU: two routes to the same fp16 weights.  If every logit of a wavefront's 32x64 block satisfies
// |x| <= 2 (masked positions included), a polynomial whose correction term runs in packed fp16 (within one
// fp16 ulp of the exact weight); otherwise the exact exp2/rcp form in fp32.  The mask is applied to the
// fp32 weights of either route, on boundary tiles only.
//
// Bias: each key tile brings a window of the per-distance table (by decreasing distance, fp32) into
// LDS; a lane's 8 consecutive entries per accumulator half-block are read straight into the
// accumulator registers, so the bias add costs LDS bandwidth but no VALU instruction (on this
// chip VALU and MFMA work of one SIMD largely serialise, so every VALU instruction saved counts).
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace flame {

namespace {

constexpr int QT = kAttnQTileBf16;  // query rows per workgroup: four groups of 32 (one 32-row MFMA block each)
static_assert(QT == 128, "4 groups of 32 query rows");
constexpr int NSTAGE = 3;           // LDS stages (ring)
constexpr int KH = 64;              // keys per half tile (one pass of the register-level loop)

// SiLU for small arguments: the polynomial of device_common.h, silu(x) = x/2 + x^2 (a1 + a3 x^2 + a5 x^4).  On the halved
// logit s = x/2, with t = s^2:
//   silu(x) = s + q,   q = t (4 a1 + 16 a3 t + 64 a5 t^2).
// t and the bracket are evaluated in packed fp16 (one multiply and two fused multiply-adds per pair of
// weights); the last step is a mixed-precision fused multiply-add per weight, fp16 t times fp16 bracket
// plus the fp32 logit itself, rounded to fp16 once, like the weight of the exact route.
constexpr float kPolyT2 = 1.0f;                                  // bound on t = s^2  (|x| <= 2)
// Second segment, |x| <= 4 (t <= 4): silu(x) = s + t (B0 + B1 t + B2 t^2 + B3 t^3 + B4 t^4), minimax-weighted fit of
// (silu(2 s) - s) / t on 0 <= t <= 4 (error of silu below 5.4e-4).
constexpr float kMidT2 = 4.0f;
__device__ constexpr float kMidB[5] = {0.9926417973f, -0.3010154918f, 0.0835130618f, -0.0141349725f, 0.0010234216f};
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

// SOFTMAX = false: the weights are silu(logit), pointwise.  SOFTMAX = true: the weights of a query row are
// softmax over its allowed keys of logit / tau (tau per layer and head); the kernel keeps a running maximum and
// sum per row and rescales its output accumulators when the maximum moves (one pass over the keys).  The logit
// in the accumulators is halved, so the exponent fed to the base-2 exponential is accumulator * tscale_h[head]
// with tscale = 2 log2(e) / tau.  The 64 keys of a half tile of one query sit in two lanes (lane and lane ^ 32),
// which exchange their maxima with one half-swap; their partial sums are only added at the end.
//
// KSPLIT = false is the throughput configuration described at the top: 4 wavefronts, key tiles of 64, three
// workgroups per CU.  KSPLIT = true is the latency configuration for batches too small to fill the chip, where a
// workgroup sits alone on its CU and its run time is the chain of key tiles of its longest row: 8 wavefronts, key
// tiles of 128, and each group of 32 query rows is served by a PAIR of wavefronts that take one 64-key half of every
// tile each (two wavefronts per SIMD, so one's MFMAs run under the other's VALU work) and add their partial outputs
// through LDS at the end, in a fixed order.  The chain is half as many steps and the sums are grouped differently,
// so the two configurations agree to rounding, not bit for bit.
template <int DH, bool SOFTMAX, bool KSPLIT>
__global__ __launch_bounds__(KSPLIT ? 512 : 256, KSPLIT ? 1 : 3) void attn_mfma_kernel(PlanePtrs planes, const float *__restrict__ bias_lh,
                                                           const float *__restrict__ tscale_h,
                                                           half_t *__restrict__ O, const AttnItem *__restrict__ items,
                                                           int H, int d, int D, int64_t ws_rows) {
  constexpr int NW = KSPLIT ? 8 : 4;   // wavefronts per workgroup
  constexpr int KT = KSPLIT ? 128 : 64;   // keys per LDS stage
  constexpr int BW = QT + KT;          // bias window per key tile: slot u holds bias[q_first + QT-1 - k0 - u]
  static_assert(BW <= 64 * NW, "one 64-slot window request per wavefront");
  constexpr int KS = DH / 16;          // k-steps of the Q K^T product
  constexpr int DB = DH / 32;          // 32-row blocks of O^T
  constexpr int KCH = DH / 8;          // 16-byte chunks per K row (8 or 4)
  constexpr int KSH = KCH == 8 ? 1 : 2;            // K rows per 256 bytes = 1 << KSH
  constexpr int VCH = KT / 8;          // 16-byte chunks per V^T row (16 or 8)
  constexpr int VSH = VCH == 16 ? 0 : 1;           // V^T rows per 256 bytes = 1 << VSH
  constexpr int K_BYTES = KT * DH * 2;             // K tile [KT keys][DH]
  constexpr int V_BYTES = DH * KT * 2;             // V^T tile [DH][KT keys]
  constexpr int W_BYTES = NW * 256;                // bias window: 64 slots per wavefront (BW <= 64 NW of them are used)
  constexpr int STAGE = K_BYTES + V_BYTES + W_BYTES;
  static_assert(K_BYTES % 1024 == 0 && V_BYTES % 1024 == 0 && STAGE % 256 == 0, "stage parts start on 256-byte boundaries");
  static_assert(QT * DH * 2 <= NSTAGE * STAGE, "output patches fit in the tile buffers");
  // the stages; the output patches of the wavefronts reuse them once the key loop is over.  The latency
  // configuration needs more than the 64 KB a static array may have and takes its stages from dynamic LDS.
  extern __shared__ __attribute__((aligned(256))) char lds_dynamic[];
  __shared__ __attribute__((aligned(256))) char lds_static[KSPLIT ? 256 : NSTAGE * STAGE];
  char *const lds = KSPLIT ? lds_dynamic : lds_static;

  const int head = blockIdx.x % H;
  const AttnItem it = items[blockIdx.x / H];
  const int tid = threadIdx.x, lane = tid & 63;
  // wavefront index as a scalar: every branch on it is then a uniform (scalar) branch
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lhalf = lane >> 5;

  const half_t *Vt = (const half_t *)planes.v + (int64_t)head * DH * ws_rows;   // [DH][ws_rows]
  const half_t *Qp = (const half_t *)planes.q + head * DH;                      // [row][d]
  const half_t *Kp = (const half_t *)planes.k + head * DH;
  const float *bias = bias_lh + (int64_t)head * D;

  // this wavefront's 32 query rows and (latency configuration) its half of every key tile
  const int q_group = KSPLIT ? wave >> 1 : wave;
  const int k_half = KSPLIT ? wave & 1 : 0;
  const int q_local0 = q_group * 32;
  const bool wave_active = q_local0 < it.n_q;
  const int my_q_local = q_local0 + l32;
  const bool row_valid = my_q_local < it.n_q;
  f16x8 fq[KS];                        // Q fragments (B operand of S^T): row = my query, k = 16*s + 8*lhalf + 0..7
  int n_vis;
  int64_t q_row_clamped;
  {
    const int64_t row = it.q_row + (row_valid ? my_q_local : it.n_q - 1);   // clamped for loads
    const int q_index = it.is_cand ? it.L : it.q_pos + my_q_local;
    n_vis = visible_history(it.is_cand, q_index, it.L);
    q_row_clamped = row;
  }
  const int wave_vis_min = it.is_cand ? it.L : it.q_pos + q_local0 + 1;
  const int wave_vis_max = it.is_cand ? it.L : it.q_pos + q_local0 + 32;

  f32x16 oacc[DB];
#pragma unroll
  for (int b = 0; b < DB; ++b)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[b][e] = 0.f;
  // softmax state of my query row (both lanes of a pair hold the same maximum; each holds the sum over its keys)
  // Finite stand-ins for -inf, so that no inf - inf can arise: a masked key's raw logit is kNeg; the running
  // maximum starts below kNeg * tscale for any sensible temperature, so a row whose keys so far were all masked
  // holds weights exp2(0) that the first real maximum scales to zero (every row sees key 0 of tile 0 or itself).
  constexpr float kNeg = -1.0e30f;
  const float ts = SOFTMAX ? tscale_h[head] : 0.f;
  float m_run = -3.0e38f, l_run = 0.f;

  const int n_tiles = (it.n_kv + KT - 1) / KT;
  const int q_first = it.is_cand ? it.L : it.q_pos;     // position of query row 0 of the workgroup tile

  // ---- LDS-DMA sources.  One instruction of a wavefront fills 1 KB of LDS, lane p at byte 16 p.
  // K tile: 1 KB = 64 / KCH rows; lane p owns physical chunk p % KCH of row p / KCH and fetches the logical
  // chunk the swizzle maps there (chunk ^ key, key = row bits above the rows that share 256 bytes).
  // V^T tile: 1 KB = 64 / VCH feature rows of 2 KT bytes, same scheme.
  // Instruction I = wave + 4 i of either tile belongs to this wavefront.
  typedef __attribute__((address_space(1))) const void gvoid;
  typedef __attribute__((address_space(3))) void lvoid;
  // Instruction I of a tile belongs to wavefront I % NW; going from I to I + NW leaves the swizzle key
  // unchanged, so a wavefront keeps one lane pointer per tile kind (for the tile to request next) and adds
  // scalar offsets for its further instructions.  Bias window: slots 64 w .. 64 w + 63 by wavefront w.
  constexpr int NKI = K_BYTES / 1024, NVI = V_BYTES / 1024;
  static_assert(NKI % NW == 0 && NVI % NW == 0, "every wavefront issues the same number of requests per tile");
  static_assert((NW * (64 / KCH)) % (KCH << KSH) == 0 && (NW * (64 / VCH)) % (VCH << VSH) == 0, "swizzle keys do not depend on the instruction");
  constexpr int REQ = NKI / NW + NVI / NW + 1;       // requests per wavefront and tile
  // Addresses are a wave-uniform base (advanced per tile with scalar arithmetic) plus a 32-bit lane offset that
  // never changes: the request instruction takes them as scalar base + vector offset, and a tile costs no
  // vector address arithmetic.  (Lane offsets stay below 2^32: at most 64 rows of d, resp. DH rows of ws_rows.)
  const char *bK = (const char *)(Kp + (int64_t)it.kv_row * d);
  const char *bV = (const char *)(Vt + it.kv_row);
  uint32_t oK, oV;
  // (candidate tiles shift the window by one slot: all their rows read it at the same slots, which then start on a
  // 16-byte boundary and leave as four-float reads)
  const int dW0 = q_first + (QT - 1) + (it.is_cand ? 1 : 0) - (wave * 64 + lane);   // distance held by window slot 64 w + lane in tile 0
  int sW = 0;                                                 // keys the next tile to request lies behind tile 0 (scalar)
  {
    const int row = wave * (64 / KCH) + lane / KCH;
    const int c = (lane % KCH) ^ ((row >> KSH) & (KCH - 1));
    oK = (uint32_t)(row * d + c * 8) * 2u;
  }
  {
    const int row = wave * (64 / VCH) + lane / VCH;
    const int c = (lane % VCH) ^ ((row >> VSH) & (VCH - 1));
    oV = (uint32_t)((int64_t)row * ws_rows + c * 8) * 2u;
  }
  auto request_tile = [&](int stage) {
    char *sb = lds + stage * STAGE;
    // (the empty asm keeps the widening of the offsets next to the requests: hoisted out of the loop, the
    // compiler would add full 64-bit vector addresses per request again)
    asm volatile("" : "+v"(oK), "+v"(oV));
#pragma unroll
    for (int i = 0; i < NKI / NW; ++i)
      __builtin_amdgcn_global_load_lds((gvoid *)(bK + (int64_t)(i * NW * (64 / KCH)) * d * 2 + oK), (lvoid *)(sb + (wave + NW * i) * 1024), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < NVI / NW; ++i)
      __builtin_amdgcn_global_load_lds((gvoid *)(bV + (int64_t)(i * NW * (64 / VCH)) * ws_rows * 2 + oV), (lvoid *)(sb + K_BYTES + (wave + NW * i) * 1024), 16, 0, 0);
    // every wavefront issues one window request, so that all of them have the same number of requests in
    // flight per tile (slots past the window are filled too and never read)
    uint32_t oW = (uint32_t)max(0, min(D - 1, dW0 - sW)) * 4u;
    asm volatile("" : "+v"(oW));
    __builtin_amdgcn_global_load_lds((gvoid *)((const char *)bias + oW), (lvoid *)(sb + K_BYTES + V_BYTES + wave * 256), 4, 0, 0);
  };
  auto next_tile = [&]() {
    bK += (int64_t)KT * d * 2;
    bV += KT * 2;
    sW += KT;
  };

  // Window slot of (my row, key 0 of the tile) is QT-1 - m + 8*lhalf with m the row's index in the
  // workgroup tile; keys further right sit at increasing slots.  Candidate rows all sit at the same distance
  // from a key (m = 0), and their window is shifted by one slot: QT + 8*lhalf, a 16-byte boundary.
  const int bias_idx = it.is_cand ? QT + 8 * lhalf : (QT - 1) - my_q_local + 8 * lhalf;
  // fragment byte offsets inside a stage.  K (A operand of S^T): MFMA row m takes key pi32(m); per 32-key
  // block j the row advances by 32 (key bits 0..4 unchanged, so the swizzle key is the same).  V^T (A
  // operand of O^T): row = feature 32 b + l32, chunk = key / 8.
  // The swizzled chunk (c ^ key) << 4 never carries into the row bits, so an address is
  // (row base | key << 4) ^ (c << 4): one XOR with a constant per fragment.
  const int krow = pi32(l32);
  const int ka0 = (krow * (DH * 2)) | (((((krow >> KSH) & (KCH - 1)) ^ lhalf) << 4));
  const int va0 = (K_BYTES + l32 * (KT * 2)) | (((((l32 >> VSH) & (VCH - 1)) ^ lhalf) << 4));

  // Ring of NSTAGE = 3 stages, requests two tiles ahead.  Past the last tile the requests repeat the last
  // tile (into a free stage), so that "at most REQ requests outstanding" always means "tile t has landed".
  if (n_tiles > 0) {
    request_tile(0);
    if (n_tiles > 1) next_tile();
    request_tile(1);
  }
  // The query fragments are requested behind the first two tiles, not ahead of them: the tiles are what the first
  // step waits for.  (The waits below count requests in order: with at most REQ outstanding, the query loads and
  // every tile before the newest have landed.)
#pragma unroll
  for (int s = 0; s < KS; ++s) fq[s] = *(const f16x8 *)(Qp + q_row_clamped * d + s * 16 + lhalf * 8);
  // One key tile.  The stage is a compile-time constant (the tile loop below is unrolled over the ring), so
  // every fragment address is a fixed lane offset plus an immediate and costs no instruction.
  auto tile_step = [&](auto stage_c, const int t) {
    constexpr int ST = decltype(stage_c)::value;
    const char *sb = lds + ST * STAGE;
    // tile t has landed for this wavefront; past the barrier it has landed for all of them, and everybody
    // has left tile t-1, whose stage the next request overwrites
    if (REQ == 5) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
    else if (REQ == 3) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    if (t + 2 < n_tiles) next_tile();
    request_tile((ST + 2) % NSTAGE);
    __builtin_amdgcn_sched_barrier(0);   // the requests stay ahead of the tile's arithmetic
#pragma unroll 1
    for (int u = KSPLIT ? k_half : 0; u < (KSPLIT ? k_half + 1 : KT / KH); ++u) {
    const int k0 = t * KT + u * KH;
    if (wave_active && k0 < wave_vis_max) {
      const char *kb = sb + u * (KH * DH * 2);                 // K rows of this half tile
      const int vau = va0 ^ (u << 7);                          // V^T: chunks 8 u .. 8 u + 7 of each row
      const bool need_mask = k0 + KH > wave_vis_min;
      // key 32 j + 16 (e >> 3) + 8 lhalf + (e & 7) of this half tile is visible to my row iff its constant part is below vis_lim
      const int vis_lim = n_vis - k0 - 8 * lhalf;
      {
        // ---- S^T = K Q^T: blocks [j], j = 32-key half of the half tile.  Fragment reads run one group
        // ahead of the MFMAs that use them (and the first V^T group is fetched behind the last K group),
        // so LDS latency hides behind matrix work instead of being paid once per group.
        f32x16 sacc[2];
        {
          // one address register, the 32 reads use immediate offsets (the empty asm keeps the compiler
          // from folding constant parts of the address into every read as a separate add)
          typedef const __attribute__((address_space(3))) float *lds_cfloat;
          lds_cfloat bp = (lds_cfloat)(sb + K_BYTES + V_BYTES) + (bias_idx + u * KH);
          asm volatile("" : "+v"(bp));
          if (it.is_cand) {
            typedef const __attribute__((address_space(3))) f32x4 *lds_cf4;
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
              for (int g = 0; g < 4; ++g) {
                const f32x4 v = *(lds_cf4)(bp + 32 * j + 16 * (g >> 1) + 4 * (g & 1));
#pragma unroll
                for (int q = 0; q < 4; ++q) sacc[j][4 * g + q] = v[q];
              }
          } else {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
              for (int e = 0; e < 16; ++e) sacc[j][e] = bp[32 * j + 16 * (e >> 3) + (e & 7)];
          }
        }
        f16x8 fk[2][2], fv[2][DB];
#pragma unroll
        for (int j = 0; j < 2; ++j) fk[0][j] = *(const f16x8 *)(kb + j * (32 * DH * 2) + ka0);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          if (s + 1 < KS) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
              fk[(s + 1) & 1][j] = *(const f16x8 *)(kb + j * (32 * DH * 2) + (ka0 ^ ((s + 1) << 5)));
          } else {
#pragma unroll
            for (int b = 0; b < DB; ++b) fv[0][b] = *(const f16x8 *)(sb + b * (32 * KT * 2) + vau);
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int j = 0; j < 2; ++j)
            sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fk[s & 1][j], fq[s], sacc[j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
        // ---- P^T = silu(S^T) (the bias is already in the accumulators), or the softmax numerators
        f16x8 fp[4];
        bool fast = SOFTMAX;
        if constexpr (SOFTMAX) {
          // maximum of the raw (halved) logits first: the temperature scale is positive, so it commutes with the max.
          // Maxima and sums are taken in four independent chains (the 32 values of a lane would otherwise form one
          // chain of dependent instructions).
          if (need_mask) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
              for (int e = 0; e < 16; ++e) {
                sacc[j][e] = 32 * j + 16 * (e >> 3) + (e & 7) < vis_lim ? sacc[j][e] : kNeg;
              }
          }
          // maximum of the lane's 32 logits as a tree of three-input maxima, 10 + 4 + 2 instructions.  (Written as
          // instructions: for fmaxf on accumulator values the compiler first emits one canonicalising v_max_f32 per
          // value, 53 instructions in all.)
          float l1[10], l2[4];
#pragma unroll
          for (int k = 0; k < 10; ++k) {
            const int e = 3 * k;   // values 0..29 in the order sacc[0][0..15], sacc[1][0..13]
            l1[k] = max3_f32(sacc[e >> 4][e & 15], sacc[(e + 1) >> 4][(e + 1) & 15], sacc[(e + 2) >> 4][(e + 2) & 15]);
          }
#pragma unroll
          for (int k = 0; k < 3; ++k) l2[k] = max3_f32(l1[3 * k], l1[3 * k + 1], l1[3 * k + 2]);
          l2[3] = max3_f32(l1[9], sacc[1][14], sacc[1][15]);
          const float l3 = max3_f32(l2[0], l2[1], l2[2]);
          const float mt = max3_f32(l3, l2[3], l2[3]);
          const float m_new = fmaxf(m_run, pair_max(mt) * ts);
          // the accumulators are rescaled only when some row of the wavefront has a new maximum (rare after the
          // first tiles); the branch is uniform over the wavefront
          if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {
            const float sc = __builtin_amdgcn_exp2f(m_run - m_new);
            l_run *= sc;
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
              for (int e = 0; e < 16; ++e) oacc[b][e] *= sc;
            m_run = m_new;
          }
          const float nm = -m_new;
          float psum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            float w[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) w[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[j][e], ts, nm));
#pragma unroll
            for (int e = 0; e < 16; ++e) psum[e & 3] += w[e];
            fp[2 * j] = pack8(w);
            fp[2 * j + 1] = pack8(w + 8);
          }
          const float ps = (psum[0] + psum[1]) + (psum[2] + psum[3]);
          l_run += ps;
        } else {
          f16x2 th[2][8];
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              const f16x2 yh = f16x2{(half_t)sacc[j][2 * i], (half_t)sacc[j][2 * i + 1]};
              th[j][i] = yh * yh;
            }
          // maximum of the 16 pairs with the packed three-input maximum (NaN-propagating): 5 + 2 + 1 instructions
          auto max3 = [](f16x2 a, f16x2 b, f16x2 c) { return __builtin_elementwise_maximum(__builtin_elementwise_maximum(a, b), c); };
          const f16x2 m0 = max3(th[0][0], th[0][1], th[0][2]), m1 = max3(th[0][3], th[0][4], th[0][5]);
          const f16x2 m2 = max3(th[0][6], th[0][7], th[1][0]), m3 = max3(th[1][1], th[1][2], th[1][3]);
          const f16x2 m4 = max3(th[1][4], th[1][5], th[1][6]);
          const f16x2 m = __builtin_elementwise_maximum(max3(m0, m1, m2), max3(m3, m4, th[1][7]));
          const bool bad = !((float)m[0] <= kPolyT2 && (float)m[1] <= kPolyT2);     // NaN counts as bad
          const bool bad_mid = !((float)m[0] <= kMidT2 && (float)m[1] <= kMidT2);
          fast = __builtin_amdgcn_ballot_w64(bad) == 0;
          const bool mid = !fast && __builtin_amdgcn_ballot_w64(bad_mid) == 0;
          if (mid) {
            // 2 < max |x| <= 4 somewhere in the block: the same form with a polynomial of degree 4 in t fitted on
            // |x| <= 4 (approximation error below 5.4e-4; two more packed multiply-adds per pair of weights than the
            // short polynomial, still no transcendental).  The exp2 / rcp route is left for blocks with |x| > 4.
#pragma unroll
            for (int j = 0; j < 2; ++j) {
              const f16x2 d4 = {(half_t)kMidB[4], (half_t)kMidB[4]}, d3 = {(half_t)kMidB[3], (half_t)kMidB[3]};
              const f16x2 d2 = {(half_t)kMidB[2], (half_t)kMidB[2]}, d1 = {(half_t)kMidB[1], (half_t)kMidB[1]};
              const f16x2 d0 = {(half_t)kMidB[0], (half_t)kMidB[0]};
              f16x2 r[8];
#pragma unroll
              for (int i = 0; i < 8; ++i) r[i] = __builtin_elementwise_fma(d4, th[j][i], d3);
#pragma unroll
              for (int i = 0; i < 8; ++i) r[i] = __builtin_elementwise_fma(r[i], th[j][i], d2);
#pragma unroll
              for (int i = 0; i < 8; ++i) r[i] = __builtin_elementwise_fma(r[i], th[j][i], d1);
#pragma unroll
              for (int i = 0; i < 8; ++i) r[i] = __builtin_elementwise_fma(r[i], th[j][i], d0);
              float w[16];
#pragma unroll
              for (int i = 0; i < 8; ++i) {
                w[2 * i] = __builtin_fmaf((float)th[j][i][0], (float)r[i][0], sacc[j][2 * i]);
                w[2 * i + 1] = __builtin_fmaf((float)th[j][i][1], (float)r[i][1], sacc[j][2 * i + 1]);
              }
              if (need_mask) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                  w[e] = 32 * j + 16 * (e >> 3) + (e & 7) < vis_lim ? w[e] : 0.f;
                }
              }
              __builtin_amdgcn_sched_barrier(0);
              fp[2 * j] = pack8(w);
              fp[2 * j + 1] = pack8(w + 8);
            }
            fast = true;      // the weights are made
          } else if (fast) {
            // stage by stage over eight independent pairs, so that no instruction waits for the one before
#pragma unroll
            for (int j = 0; j < 2; ++j) {
              constexpr float b1 = 4.0f * kPolyA1, b3 = 16.0f * kPolyA3, b5 = 64.0f * kPolyA5;
              const f16x2 c5 = {(half_t)b5, (half_t)b5}, c3 = {(half_t)b3, (half_t)b3}, c1 = {(half_t)b1, (half_t)b1};
              f16x2 r[8];
#pragma unroll
              for (int i = 0; i < 8; ++i) r[i] = __builtin_elementwise_fma(c5, th[j][i], c3);
#pragma unroll
              for (int i = 0; i < 8; ++i) r[i] = __builtin_elementwise_fma(r[i], th[j][i], c1);
              float w[16];
#pragma unroll
              for (int i = 0; i < 8; ++i) {
                w[2 * i] = __builtin_fmaf((float)th[j][i][0], (float)r[i][0], sacc[j][2 * i]);
                w[2 * i + 1] = __builtin_fmaf((float)th[j][i][1], (float)r[i][1], sacc[j][2 * i + 1]);
              }
              if (need_mask) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                  w[e] = 32 * j + 16 * (e >> 3) + (e & 7) < vis_lim ? w[e] : 0.f;
                }
              }
              __builtin_amdgcn_sched_barrier(0);
              fp[2 * j] = pack8(w);
              fp[2 * j + 1] = pack8(w + 8);
            }
          }
        }
        if (!fast) {
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            float p[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) p[e] = silu_half_domain(sacc[j][e]);
            if (need_mask) {
#pragma unroll
              for (int e = 0; e < 16; ++e) {
                p[e] = 32 * j + 16 * (e >> 3) + (e & 7) < vis_lim ? p[e] : 0.f;
              }
            }
            fp[2 * j] = pack8(p);
            fp[2 * j + 1] = pack8(p + 8);
          }
        }
        // ---- O^T += V^T P^T; V^T fragments read one group ahead
#pragma unroll
        for (int s2 = 0; s2 < 4; ++s2) {
          if (s2 + 1 < 4) {
#pragma unroll
            for (int b = 0; b < DB; ++b)
              fv[(s2 + 1) & 1][b] = *(const f16x8 *)(sb + b * (32 * KT * 2) + (vau ^ ((s2 + 1) << 5)));
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int b = 0; b < DB; ++b)
            oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fv[s2 & 1][b], fp[s2], oacc[b], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    }
  };
  static_assert(NSTAGE == 3, "the tile loop is unrolled over a ring of three stages");
  for (int t = 0; t < n_tiles; t += NSTAGE) {
    tile_step(std::integral_constant<int, 0>{}, t);
    if (t + 1 < n_tiles) tile_step(std::integral_constant<int, 1>{}, t + 1);
    if (t + 2 < n_tiles) tile_step(std::integral_constant<int, 2>{}, t + 2);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the repeated requests of the tail have landed
  __builtin_amdgcn_s_barrier();          // everybody has left the last tile: the stages become output patches

  // ---- latency configuration: the wavefront with the second key half hands its partial output (and its softmax
  // state) to its partner through LDS, behind the output patches; the partner goes on alone.
  if constexpr (KSPLIT) {
    constexpr int PART = DB * 16 * 64 * 4;            // bytes of one wavefront's accumulators
    char *area = lds + 4 * (32 * DH * 2) + q_group * (PART + 512);
    if (k_half == 1) {
#pragma unroll
      for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 v = {oacc[b][4 * g], oacc[b][4 * g + 1], oacc[b][4 * g + 2], oacc[b][4 * g + 3]};
          *(f32x4 *)(area + ((b * 4 + g) * 64 + lane) * 16) = v;
        }
      if constexpr (SOFTMAX) *(float2 *)(area + PART + lane * 8) = float2{m_run, l_run};
    }
    __builtin_amdgcn_s_barrier();
    if (k_half == 1) return;
    float s_mine = 1.f, s_other = 1.f;
    if constexpr (SOFTMAX) {
      const float2 ml = *(const float2 *)(area + PART + lane * 8);
      const float m_new = fmaxf(m_run, ml.x);
      s_mine = __builtin_amdgcn_exp2f(m_run - m_new);
      s_other = __builtin_amdgcn_exp2f(ml.x - m_new);
      l_run = l_run * s_mine + ml.y * s_other;
      m_run = m_new;
    }
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 v = *(const f32x4 *)(area + ((b * 4 + g) * 64 + lane) * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          oacc[b][4 * g + i] = SOFTMAX ? oacc[b][4 * g + i] * s_mine + v[i] * s_other : oacc[b][4 * g + i] + v[i];
      }
  }

  // ---- candidates: the row itself is one more key, at distance 0.  The wavefront multiplies its 32
  // candidate rows against themselves and keeps the diagonal.
  if (it.is_cand && wave_active) {
    const float b0 = bias[0];
    const int64_t base_row = it.q_row + q_local0;   // multiple of 32 inside the padded workspace
    f32x16 sacc;
#pragma unroll
    for (int e = 0; e < 16; ++e) sacc[e] = b0;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const f16x8 fk = *(const f16x8 *)(Kp + (base_row + pi32(l32)) * d + s * 16 + lhalf * 8);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(fk, fq[s], sacc, 0, 0, 0);
    }
    float p[16];
    if constexpr (SOFTMAX) {
      // the diagonal element of my query sits in one lane of the pair
      float ys = kNeg;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int kv_local = 16 * (e >> 3) + 8 * lhalf + (e & 7);
        ys = kv_local == l32 ? sacc[e] * ts : ys;
      }
      const bool mine = ys > kNeg;
      const float m_new = fmaxf(m_run, pair_max(ys));
      const float sc = __builtin_amdgcn_exp2f(m_run - m_new);
      const float pself = mine ? __builtin_amdgcn_exp2f(ys - m_new) : 0.f;
      m_run = m_new;
      l_run = l_run * sc + pself;
#pragma unroll
      for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[b][e] *= sc;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int kv_local = 16 * (e >> 3) + 8 * lhalf + (e & 7);
        p[e] = (kv_local == l32 && row_valid) ? pself : 0.f;
      }
    } else {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int kv_local = 16 * (e >> 3) + 8 * lhalf + (e & 7);
      p[e] = (kv_local == l32 && row_valid) ? silu_half_domain(sacc[e]) : 0.f;
    }
    }
    const f16x8 fps[2] = {pack8(p), pack8(p + 8)};
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int b = 0; b < DB; ++b) {
        const f16x8 fv = *(const f16x8 *)(Vt + (int64_t)(32 * b + l32) * ws_rows + base_row + s2 * 16 + lhalf * 8);
        oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fv, fps[s2], oacc[b], 0, 0, 0);
      }
  }

  // ---- write O[q][head*DH + dd]; accumulator element e of block b: dd = 32b + 8*(e/4) + 4*lhalf + e%4.
  // Only two lanes share a query row there (16 contiguous bytes per row and store instruction, and the
  // write path is bound by the number of requests), so each wavefront transposes its 32 x DH patch
  // through LDS (16-byte chunks XOR-swizzled by row; every wavefront is past the barrier that closes the key
  // loop, nobody reads the tile buffers any more) and stores 16 bytes per lane, a whole head row of
  // 2*DH bytes per group of lanes.
  if constexpr (SOFTMAX) {
    const float lt = pair_sum(l_run);
    const float inv = lt > 0.f ? 1.0f / lt : 0.f;
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[b][e] *= inv;
  }
  {
    constexpr int CPR = DH / 8;                       // 16-byte chunks per patch row
    constexpr int RPI = 64 / CPR;                     // patch rows per store instruction
    char *pb = lds + q_group * (32 * DH * 2);
    auto pkey = [](int row) { return CPR == 8 ? (row >> 1) & 7 : (row >> 2) & 3; };   // spreads 16 rows over 256 bytes
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f16x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = to_f16_sat(oacc[b][4 * g + i]);
        const int c = 4 * b + g;
        *(f16x4 *)(pb + l32 * (DH * 2) + ((c ^ pkey(l32)) << 4) + 8 * lhalf) = v;
      }
    const int rl = lane / CPR, c = lane % CPR;
    half_t *obase = O + (int64_t)it.q_row * d + head * DH + c * 8;
#pragma unroll
    for (int t = 0; t < 32 / RPI; ++t) {
      const int row = t * RPI + rl;
      const f16x8 v = *(const f16x8 *)(pb + row * (DH * 2) + ((c ^ pkey(row)) << 4));
      if (q_local0 + row < it.n_q) __builtin_nontemporal_store(v, (f16x8 *)(obase + (int64_t)(q_local0 + row) * d));
    }
  }
}

}  // namespace

// The latency configuration needs its LDS limit raised once per kernel instance (a function attribute, no
// allocation); handles in latency mode do it when they are created, outside any stream capture.
template <int DH>
constexpr int key_split_lds_bytes() { return NSTAGE * (2 * 128 * DH * 2 + 8 * 256); }

template <int DH, bool SM>
static hipError_t key_split_setup() {
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_mfma_kernel<DH, SM, true>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, key_split_lds_bytes<DH>());
  return attr;
}

template <int DH, bool SM>
static void launch_key_split(int grid, PlanePtrs planes, const float *bias_lh, const float *tscale_h, half_t *O,
                             const AttnItem *items, const Shape &sh, hipStream_t s) {
  (void)key_split_setup<DH, SM>();
  attn_mfma_kernel<DH, SM, true><<<grid, 512, key_split_lds_bytes<DH>(), s>>>(planes, bias_lh, tscale_h, O, items, sh.H, sh.d, sh.D, sh.ws_rows);
}

hipError_t attn_latency_setup(const Shape &sh) {
  if (sh.softmax) return sh.dh == 32 ? key_split_setup<32, true>() : key_split_setup<64, true>();
  return sh.dh == 32 ? key_split_setup<32, false>() : key_split_setup<64, false>();
}

void launch_attn_bf16(PlanePtrs planes, const float *bias_lh, const float *tscale_h, void *O, const AttnItem *items,
                      int n_items, const Shape &sh, hipStream_t s) {
  if (n_items <= 0) return;
  const int grid = n_items * sh.H;
  if (sh.latency) {
    if (sh.softmax) {
      if (sh.dh == 32) launch_key_split<32, true>(grid, planes, bias_lh, tscale_h, (half_t *)O, items, sh, s);
      else launch_key_split<64, true>(grid, planes, bias_lh, tscale_h, (half_t *)O, items, sh, s);
    } else {
      if (sh.dh == 32) launch_key_split<32, false>(grid, planes, bias_lh, tscale_h, (half_t *)O, items, sh, s);
      else launch_key_split<64, false>(grid, planes, bias_lh, tscale_h, (half_t *)O, items, sh, s);
    }
    return;
  }
#define ATTN_CASE(DHV, SM) attn_mfma_kernel<DHV, SM, false><<<grid, 256, 0, s>>>(planes, bias_lh, tscale_h, (half_t *)O, items, sh.H, sh.d, sh.D, sh.ws_rows)
  if (sh.softmax) {
    if (sh.dh == 32) ATTN_CASE(32, true);
    else ATTN_CASE(64, true);
  } else {
    if (sh.dh == 32) ATTN_CASE(32, false);
    else ATTN_CASE(64, false);
  }
#undef ATTN_CASE
}

}  // namespace flame
