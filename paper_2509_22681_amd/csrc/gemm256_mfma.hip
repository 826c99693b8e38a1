// K1 for wide models (d % 256 == 0): [U V Q K] = silu(X W1^T + b1) on 256 x 256 x 32 tiles.
//
// On gfx950 the matrix pipe outruns everything that feeds it: a CU's LDS delivers about 128 B/clk and
// its vector-memory path 64 B/clk against 4096 fp16 flop/clk, and VALU work of a SIMD largely
// serialises with its MFMA work, so a second resident workgroup does not hide an epilogue.  The
// tile is therefore as large as registers allow: 256 threads = 4 wavefronts (2 x 2), each owning
// 128 x 128 outputs as 4 x 4 blocks of v_mfma_f32_32x32x16_f16 (256 accumulator registers per lane,
// one workgroup per CU).  Per 16-deep step a wavefront reads 8 KB of fragments for 16 MFMAs - half
// the LDS bytes per flop of a 128 x 64 patch - and the block re-reads half the operand bytes per
// flop of a 256 x 128 tile.
//
// Pipeline: k advances in steps of 32 through a ring of three LDS stages and two register sets.  In
// iteration kt the global loads of tile kt+3 are issued first (they stay in flight for two
// iterations: with one wavefront per SIMD nothing else hides memory latency), tile kt is multiplied
// (fragments of the next 16-deep step - and, at the end, of the next tile - are read while the current
// MFMAs run), then tile kt+2 is written to the stage that tile kt-1 vacated; one barrier per iteration.
//
// Epilogue: accumulators start at the bias; SiLU; operand order chosen per plane so that each lane
// stores 8 contiguous bytes (row-major planes: 4 features of a token; the feature-major V plane:
// 4 tokens of a feature).
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace flame {

namespace {

constexpr int BM = 256, BN = 256, BK = 32;
constexpr int RB = BM / kRowAlign;
constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;   // 32 KB
constexpr int NSTAGE = 3;

struct PlaneSel256 { int id[4]; int n; };

// byte offset of 16-byte chunk c (0..3) of tile row `row` inside one operand of a stage: rows are
// 64 bytes, two per 128-byte line, chunks XOR-swizzled with the line index
__device__ __forceinline__ int lds_off(int row, int c) {
  const int line = row >> 1;
  const int slot = ((row & 1) << 2) | c;
  return line * 128 + ((slot ^ (line & 7)) << 4);
}

// One 256 x 256 tile: main loop and epilogue, instantiated per operand order.
// FM (feature-major, the V plane): activations are the A operand and each lane ends up with 4 consecutive
// tokens of one feature; otherwise W1 rows are the A operand and each lane holds 4 consecutive features
// of one token.
template <bool FM>
__device__ __forceinline__ void tile_body(char *smem, const half_t *__restrict__ A, const half_t *__restrict__ Wn0,
                                          const uint32_t (&aoff)[4], uint32_t boff, int o0, const int (&f0)[2], const int (&g0)[2],
                                          const int (&blk)[RB], const bf16_t *__restrict__ bias, half_t *__restrict__ planes,
                                          int plane, int n_in_plane, int n0, int K, int d, int64_t ws_rows, float alpha,
                                          int wm, int wn, int l32, int lhalf) {
  f32x16 acc[4][4];                          // [row block i][column block j]
  {
    // accumulators start at the bias of their feature
    if (FM) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float bv = to_f32(bias[n0 + wn * 128 + j * 32 + l32]);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[i][j][e] = bv;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const bf16x4 bv = *(const bf16x4 *)(bias + n0 + wn * 128 + j * 32 + 8 * g + 4 * lhalf);
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[i][j][4 * g + q] = (float)bv[q];
        }
    }

    const int nk = K / BK;                    // even (K % 64 == 0)
    uint4 ra[2][4], rb[2][4];                 // two tiles in flight: set = tile & 1
    auto issue = [&](auto setc, int tile) {
      constexpr int set = decltype(setc)::value;
      const int kk = (tile < nk ? tile : nk - 1) * BK;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ra[set][i] = *(const uint4 *)(A + aoff[i] + kk);
        rb[set][i] = *(const uint4 *)(Wn0 + (size_t)i * 64 * K + boff + kk);
      }
    };
    auto commit = [&](auto setc, int stage) {
      constexpr int set = decltype(setc)::value;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *(uint4 *)(smem + stage * STAGE + o0 + i * 4096) = ra[set][i];
        *(uint4 *)(smem + stage * STAGE + A_BYTES + o0 + i * 4096) = rb[set][i];
      }
    };
    // prologue: tiles 0 and 1 into stages 0 and 1, tile 2 in flight
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    issue(S0{}, 0);
    issue(S1{}, 1);
    commit(S0{}, 0);
    commit(S1{}, 1);
    issue(S0{}, 2);
    __syncthreads();

    f16x8 fa[2][4], fb[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      fa[0][i] = *(const f16x8 *)(smem + f0[0] + i * 2048);
      fb[0][i] = *(const f16x8 *)(smem + A_BYTES + g0[0] + i * 2048);
    }
    // One iteration: tile kt is multiplied from stage st; tile kt+3 is requested into register set
    // (kt+1)&1 and stays in flight for two iterations; tile kt+2 (set kt&1) is written to the stage that
    // tile kt-1 vacated.
    auto iteration = [&](auto parc, int kt, int st) {
      constexpr int par = decltype(parc)::value;
      const int st1 = st + 1 >= NSTAGE ? st + 1 - NSTAGE : st + 1;      // stage of tile kt+1
      const int st2 = st1 + 1 >= NSTAGE ? st1 + 1 - NSTAGE : st1 + 1;   // stage that receives tile kt+2
      issue(std::integral_constant<int, par ^ 1>{}, kt + 3);
      __builtin_amdgcn_sched_barrier(0);
      // step 0: fetch step-1 fragments of this tile, multiply step 0
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        fa[1][i] = *(const f16x8 *)(smem + st * STAGE + f0[1] + i * 2048);
        fb[1][i] = *(const f16x8 *)(smem + st * STAGE + A_BYTES + g0[1] + i * 2048);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = FM ? __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[0][i], fb[0][j], acc[i][j], 0, 0, 0)
                         : __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[0][j], fa[0][i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      // step 1: fetch step-0 fragments of the next tile (already complete in its stage), multiply step 1
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        fa[0][i] = *(const f16x8 *)(smem + st1 * STAGE + f0[0] + i * 2048);
        fb[0][i] = *(const f16x8 *)(smem + st1 * STAGE + A_BYTES + g0[0] + i * 2048);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = FM ? __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[1][i], fb[1][j], acc[i][j], 0, 0, 0)
                         : __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[1][j], fa[1][i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      commit(std::integral_constant<int, par>{}, st2);
      __syncthreads();
    };
    int st = 0;
    for (int kt = 0; kt < nk; kt += 2) {
      iteration(S0{}, kt, st);
      st = st + 1 >= NSTAGE ? 0 : st + 1;
      iteration(S1{}, kt + 1, st);
      st = st + 1 >= NSTAGE ? 0 : st + 1;
    }
  }

  // Epilogue.  Accumulator element e of a 32x32 block sits at (A-operand row 8*(e/4) + 4*(lane/32) + e%4,
  // B-operand row lane%32): four consecutive e are four consecutive A-operand rows.
  half_t *P = planes + (int64_t)plane * ws_rows * d;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int tr = wm * 128 + i * 32;
    const int rblk = blk[tr >> 6];
    if (rblk < 0) continue;
    const int64_t row_base = (int64_t)rblk * kRowAlign + (tr & 63);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int nb0 = n_in_plane + wn * 128 + j * 32;
      if (!FM) {
        // Q leaves this kernel multiplied by alpha * log2(e), V by ln 2 (the attention kernel works in
        // the exp2 domain)
        const float sc = plane == 2 ? alpha * kLog2e : 1.0f;
        half_t *prow = P + (row_base + l32) * d + nb0 + 4 * lhalf;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f16x4 o;
#pragma unroll
          for (int q = 0; q < 4; ++q) o[q] = to_f16_sat(silu_fast(acc[i][j][4 * g + q]) * sc);
          *(f16x4 *)(prow + 8 * g) = o;
        }
      } else {
        half_t *pcol = P + (int64_t)(nb0 + l32) * ws_rows + row_base + 4 * lhalf;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f16x4 o;
#pragma unroll
          for (int q = 0; q < 4; ++q) o[q] = to_f16_sat(silu_fast(acc[i][j][4 * g + q]) * kLn2);
          *(f16x4 *)(pcol + 8 * g) = o;
        }
      }
    }
  }
}

__global__ __launch_bounds__(256, 1) void uvqk256_kernel(
    const half_t *__restrict__ A, const half_t *__restrict__ W, const bf16_t *__restrict__ bias, half_t *__restrict__ planes,
    const int32_t *__restrict__ blk_list, int blk_first, int n_blk, int n_row_tiles, int n_col_tiles, int K, int d,
    int64_t ws_rows, PlaneSel256 sel, float alpha) {
  extern __shared__ __attribute__((aligned(128))) char smem[];   // NSTAGE * STAGE

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lhalf = lane >> 5;

  // workgroup id -> (row tile, column tile), XCD-aware: XCD x takes row tiles congruent to x mod 8 and
  // walks all column tiles of a row tile before the next one
  int row_tile, col_tile;
  {
    constexpr int NXCD = 8;
    const int wg = blockIdx.x, xcd = wg % NXCD, j = wg / NXCD;
    const int full = (n_row_tiles / NXCD) * NXCD;
    const int rt = (j / n_col_tiles) * NXCD + xcd;
    if (rt < full) {
      row_tile = rt;
      col_tile = j % n_col_tiles;
    } else {
      const int t = wg - full * n_col_tiles;
      row_tile = full + t / n_col_tiles;
      col_tile = t % n_col_tiles;
    }
  }
  const int tiles_per_plane = d / BN;
  const int plane = sel.id[col_tile / tiles_per_plane];
  const int n_in_plane = (col_tile % tiles_per_plane) * BN;
  const int n0 = plane * d + n_in_plane;
  int blk[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    const int t = row_tile * RB + r;
    blk[r] = t < n_blk ? (blk_list ? blk_list[t] : blk_first + t) : -1;
  }

  // global -> register staging: 16-byte chunks, 4 per 32-wide row; thread t stages chunk t & 3 of tile rows
  // (t >> 2) + 64 i, i = 0..3, of both operands.  Offsets in elements from the operand bases; in LDS the
  // four rows are 4096 bytes apart (the swizzle only involves the low bits of the line index).
  const int r0 = tid >> 2, ch = tid & 3;
  uint32_t aoff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int b = blk[i] >= 0 ? blk[i] : blk[0];
    aoff[i] = (uint32_t)(((int64_t)b * kRowAlign + r0) * K + ch * 8);
  }
  const uint32_t boff = (uint32_t)(r0 * K + ch * 8);
  const half_t *Wn0 = W + (int64_t)n0 * K;
  const int o0 = lds_off(r0, ch);
  // fragment byte offsets inside an operand for 16-deep step 0 and 1; blocks i are 2048 bytes apart
  int f0[2], g0[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    f0[ks] = lds_off(wm * 128 + l32, ks * 2 + lhalf);
    g0[ks] = lds_off(wn * 128 + l32, ks * 2 + lhalf);
  }

  if (plane == 1)
    tile_body<true>(smem, A, Wn0, aoff, boff, o0, f0, g0, blk, bias, planes, plane, n_in_plane, n0, K, d, ws_rows, alpha, wm, wn, l32, lhalf);
  else
    tile_body<false>(smem, A, Wn0, aoff, boff, o0, f0, g0, blk, bias, planes, plane, n_in_plane, n0, K, d, ws_rows, alpha, wm, wn, l32, lhalf);
}

}  // namespace

// Not dispatched yet: measured slower than the 256 x 128 two-workgroup kernel (register staging of two
// tiles in flight spills); kept for the LDS-DMA version of the pipeline.
bool uvqk256_supported(int d) { (void)d; return false; }

void launch_uvqk256(const void *Xh, const void *W1h, const void *b1, void *planes, const int32_t *blk_list, int n_blk,
                    int blk_first, int plane_mask, const Shape &sh, hipStream_t s) {
  if (n_blk <= 0 || !(plane_mask & 0xF)) return;
  PlaneSel256 sel{};
  for (int p = 0; p < 4; ++p)
    if (plane_mask & (1 << p)) sel.id[sel.n++] = p;
  const int row_tiles = (n_blk + RB - 1) / RB;
  const int col_tiles = sel.n * (sh.d / BN);
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void *)uvqk256_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, NSTAGE * STAGE);
    attr_set = true;
  }
  uvqk256_kernel<<<row_tiles * col_tiles, 256, NSTAGE * STAGE, s>>>((const half_t *)Xh, (const half_t *)W1h, (const bf16_t *)b1,
                                                                    (half_t *)planes, blk_list, blk_first, n_blk, row_tiles, col_tiles,
                                                                    sh.d, sh.d, sh.ws_rows, sel, sh.alpha);
}

}  // namespace flame
