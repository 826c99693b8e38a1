// MFMA projections of the GR block for gfx950 (fp16 operands, fp32 accumulation):
//   K1  [U V Q K] = silu(X W1^T + b1)            (SiLU fused as the GEMM epilogue)
//   K3b X <- X + G W2^T + b2, Xh = fp16(X)       (residual fused as the GEMM epilogue)
// Both are C[m][n] = sum_k A[m][k] W[n][k] with A and W row-major, k contiguous.
//
// Tiling: 256 threads = 4 wavefronts in a 2x2 arrangement, block tile 128 x BN x 64, each
// wavefront owns a 64 x (BN/2) patch built from v_mfma_f32_32x32x16_f16 blocks; global -> register
// -> LDS double buffering overlaps the loads of tile k+1 with the MFMAs of tile k (the role the
// cp.async pipeline plays in Section 3.2).  Rows are addressed through 64-row blocks so that the
// same kernel runs on a contiguous range or on a list of candidate blocks (last-layer pruning).
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace flame {

namespace {

constexpr int BM = 128;
constexpr int BK = 64;
constexpr int LDS_PAD = 8;              // fp16 elements; keeps 16-byte alignment, spreads banks
constexpr int LDS_LD = BK + LDS_PAD;    // 72

struct PlaneSel { int id[4]; int n; };

template <int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(
    const half_t *__restrict__ A, const half_t *__restrict__ W, const bf16_t *__restrict__ bias,
    half_t *__restrict__ planes, float *__restrict__ X, half_t *__restrict__ Xh,
    const int32_t *__restrict__ blk_list, int blk_first, int n_blk, int n_row_tiles, int n_col_tiles, int K, int d,
    int64_t ws_rows, PlaneSel sel, float alpha) {
  constexpr int WN = BN / 2;            // wavefront patch width
  constexpr int NB = WN / 32;           // 32-wide MFMA blocks per wavefront in n
  __shared__ __attribute__((aligned(16))) half_t sA[2][BM][LDS_LD];
  __shared__ __attribute__((aligned(16))) half_t sB[2][BN][LDS_LD];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lhalf = lane >> 5;

  // Workgroup id -> (row tile, column tile).  Consecutive workgroup ids go round-robin over the 8
  // XCDs, each with its own L2: XCD x takes the row tiles congruent to x mod 8 and walks through all
  // column tiles of one row tile before the next, so an activation tile is fetched from HBM once
  // and then served from that XCD's L2, while the (small) weight matrix stays resident in all L2s.
  int row_tile, col_tile;
  {
    constexpr int NXCD = 8;
    const int wg = blockIdx.x, xcd = wg % NXCD, j = wg / NXCD;
    const int full = (n_row_tiles / NXCD) * NXCD;       // row tiles that split evenly over the XCDs
    const int rt = (j / n_col_tiles) * NXCD + xcd;
    if (rt < full) {
      row_tile = rt;
      col_tile = j % n_col_tiles;
    } else {                                            // the tail is dealt out in plain order
      const int t = wg - full * n_col_tiles;
      row_tile = full + t / n_col_tiles;
      col_tile = t % n_col_tiles;
    }
  }
  // column tile -> (plane, offset inside the plane)
  int plane = 0, n_in_plane = 0, n0;
  if (EPI == 0) {
    const int tiles_per_plane = d / BN;
    plane = sel.id[col_tile / tiles_per_plane];
    n_in_plane = (col_tile % tiles_per_plane) * BN;
    n0 = plane * d + n_in_plane;
  } else {
    n0 = col_tile * BN;
  }
  // the two 64-row blocks of this row tile (-1: absent)
  int blk[2];
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int t = row_tile * 2 + r;
    blk[r] = t < n_blk ? (blk_list ? blk_list[t] : blk_first + t) : -1;
  }
  const int blk_safe1 = blk[1] >= 0 ? blk[1] : blk[0];

  // global -> register staging: 16-byte chunks, 8 per 64-wide row.  Per-thread source pointers
  // (at k = 0) and LDS destinations are fixed for the whole loop.
  constexpr int A_CH = BM * 8 / 256, B_CH = BN * 8 / 256;
  const half_t *gA[A_CH];
  const half_t *gB[B_CH];
  int oA[A_CH], oB[B_CH];               // element offsets inside one LDS buffer
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int c = tid + i * 256, r = c >> 3, c8 = c & 7;
    const int64_t row = (int64_t)(r < 64 ? blk[0] : blk_safe1) * kRowAlign + (r & 63);
    gA[i] = A + row * K + c8 * 8;
    oA[i] = r * LDS_LD + c8 * 8;
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int c = tid + i * 256, r = c >> 3, c8 = c & 7;
    gB[i] = W + (int64_t)(n0 + r) * K + c8 * 8;
    oB[i] = r * LDS_LD + c8 * 8;
  }

  f32x16 acc[2][NB];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // The V plane is produced transposed (feature-major) because the attention kernel consumes V as
  // the A operand of O^T = V^T P^T: swapping the MFMA operands yields C^T in registers for free.
  const bool transposed = (EPI == 0) && plane == 1;

  // The operand order is fixed per workgroup; the loop is instantiated once per order so that no
  // branch sits between the MFMAs.
  auto main_loop = [&](auto swapped) {
    constexpr bool SW = decltype(swapped)::value;
    uint4 ra[A_CH], rb[B_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) ra[i] = *(const uint4 *)gA[i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) rb[i] = *(const uint4 *)gB[i];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) *(uint4 *)(&sA[0][0][0] + oA[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) *(uint4 *)(&sB[0][0][0] + oB[i]) = rb[i];
    __syncthreads();
    const int nk = K / BK;
    for (int kt = 0; kt < nk; ++kt) {
      const int buf = kt & 1;
      // prefetch the next k tile into registers (the last iteration re-reads its own tile: no branch)
      const int kn = (kt + 1 < nk ? kt + 1 : kt) * BK;
#pragma unroll
      for (int i = 0; i < A_CH; ++i) ra[i] = *(const uint4 *)(gA[i] + kn);
#pragma unroll
      for (int i = 0; i < B_CH; ++i) rb[i] = *(const uint4 *)(gB[i] + kn);
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        f16x8 fa[2], fb[NB];
#pragma unroll
        for (int i = 0; i < 2; ++i) fa[i] = *(const f16x8 *)&sA[buf][wm * 64 + i * 32 + l32][ks * 16 + lhalf * 8];
#pragma unroll
        for (int j = 0; j < NB; ++j) fb[j] = *(const f16x8 *)&sB[buf][wn * WN + j * 32 + l32][ks * 16 + lhalf * 8];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < NB; ++j)
            acc[i][j] = SW ? __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[j], fa[i], acc[i][j], 0, 0, 0)
                           : __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      }
      // the other buffer was last read before the previous barrier: safe to overwrite
#pragma unroll
      for (int i = 0; i < A_CH; ++i) *(uint4 *)(&sA[buf ^ 1][0][0] + oA[i]) = ra[i];
#pragma unroll
      for (int i = 0; i < B_CH; ++i) *(uint4 *)(&sB[buf ^ 1][0][0] + oB[i]) = rb[i];
      __syncthreads();
    }
  };
  if (transposed) main_loop(std::true_type{});
  else main_loop(std::false_type{});

  // epilogue.  Accumulator element e of a 32x32 block: column = lane % 32, row = 8*(e/4) + 4*(lane/32) + e%4
  // (rows are tokens and columns features, or the reverse for the transposed plane).
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int rblk = blk[wm];             // wavefront rows wm*64 .. +63 lie in one 64-row block
    if (rblk < 0) continue;
    const int64_t row_base = (int64_t)rblk * kRowAlign + i * 32;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int nb0 = wn * WN + j * 32;   // column offset of this block inside the tile
      if (EPI == 0) {
        half_t *P = planes + (int64_t)plane * ws_rows * d;
        if (!transposed) {
          const int n = n_in_plane + nb0 + l32;
          const float bv = to_f32(bias[plane * d + n]);
          // Q leaves this kernel multiplied by alpha * log2(e): the attention logits are then
          // directly the arguments of exp2 (V carries the inverse factor ln 2).
          const float sc = plane == 2 ? alpha * kLog2e : 1.0f;
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int m = 8 * (e >> 2) + 4 * lhalf + (e & 3);
            P[(row_base + m) * d + n] = to_f16_sat(silu_fast(acc[i][j][e] + bv) * sc);
          }
        } else {
          const int64_t m = row_base + l32;
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int n = n_in_plane + nb0 + 8 * (e >> 2) + 4 * lhalf + (e & 3);
            const float bv = to_f32(bias[plane * d + n]);
            P[(int64_t)n * ws_rows + m] = to_f16_sat(silu_fast(acc[i][j][e] + bv) * kLn2);
          }
        }
      } else {
        const int n = n0 + nb0 + l32;
        const float bv = to_f32(bias[n]);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int64_t m = row_base + 8 * (e >> 2) + 4 * lhalf + (e & 3);
          const float v = X[m * d + n] + acc[i][j][e] + bv;
          X[m * d + n] = v;
          Xh[m * d + n] = to_f16_sat(v);
        }
      }
    }
  }
}

}  // namespace

void launch_uvqk_bf16(const void *Xh, const void *W1h, const void *b1, void *planes, const int32_t *blk_list,
                      int n_blk, int blk_first, int plane_mask, const Shape &sh, hipStream_t s) {
  if (n_blk <= 0 || !(plane_mask & 0xF)) return;
  PlaneSel sel{};
  for (int p = 0; p < 4; ++p)
    if (plane_mask & (1 << p)) sel.id[sel.n++] = p;
  const int row_tiles = (n_blk + 1) / 2;
  if (sh.d % 128 == 0) {
    const int col_tiles = sel.n * (sh.d / 128);
    gemm_bf16_kernel<128, 0><<<row_tiles * col_tiles, 256, 0, s>>>((const half_t *)Xh, (const half_t *)W1h, (const bf16_t *)b1, (half_t *)planes,
                                                  nullptr, nullptr, blk_list, blk_first, n_blk, row_tiles, col_tiles, sh.d, sh.d, sh.ws_rows, sel, sh.alpha);
  } else {
    const int col_tiles = sel.n * (sh.d / 64);
    gemm_bf16_kernel<64, 0><<<row_tiles * col_tiles, 256, 0, s>>>((const half_t *)Xh, (const half_t *)W1h, (const bf16_t *)b1, (half_t *)planes,
                                                 nullptr, nullptr, blk_list, blk_first, n_blk, row_tiles, col_tiles, sh.d, sh.d, sh.ws_rows, sel, sh.alpha);
  }
}

void launch_outproj_bf16(const void *G, const void *W2h, const void *b2, float *X, void *Xh, const int32_t *blk_list,
                         int n_blk, int blk_first, const Shape &sh, hipStream_t s) {
  if (n_blk <= 0) return;
  PlaneSel sel{};
  const int row_tiles = (n_blk + 1) / 2;
  if (sh.d % 128 == 0) {
    const int col_tiles = sh.d / 128;
    gemm_bf16_kernel<128, 1><<<row_tiles * col_tiles, 256, 0, s>>>((const half_t *)G, (const half_t *)W2h, (const bf16_t *)b2, nullptr, X, (half_t *)Xh,
                                                  blk_list, blk_first, n_blk, row_tiles, col_tiles, sh.d, sh.d, sh.ws_rows, sel, 1.0f);
  } else {
    const int col_tiles = sh.d / 64;
    gemm_bf16_kernel<64, 1><<<row_tiles * col_tiles, 256, 0, s>>>((const half_t *)G, (const half_t *)W2h, (const bf16_t *)b2, nullptr, X, (half_t *)Xh,
                                                 blk_list, blk_first, n_blk, row_tiles, col_tiles, sh.d, sh.d, sh.ws_rows, sel, 1.0f);
  }
}

}  // namespace flame
