// MFMA projections of the GR block for gfx950 (fp16 operands, fp32 accumulation):
//   K1  [U V Q K] = silu(X W1^T + b1)            (SiLU fused as the GEMM epilogue)
//   K3b X <- X + G W2^T + b2                     (residual fused as the GEMM epilogue; X is held as the two fp16 words
//                                                 Xh = fp16(X), k-tile blocked, and Xl = fp16(X - Xh), row-major)
// Both are C[m][n] = sum_k A[m][k] W[n][k] with A and W row-major, k contiguous.
//
// Tiling.  A 128x128 tile re-reads 1 byte of operand per 64 flop, which at MFMA speed is twice what
// the L2 delivers (measured about 19 TB/s), so the block tile is 256 x BN (BN = 128 where d allows):
// 256 threads = 4 wavefronts in a 2x2 arrangement, each owning 128 x BN/2 as 4 x (BN/64) blocks of
// v_mfma_f32_32x32x16_f16.  Two workgroups share a CU: with K = d as short as 512 the fixed cost of a
// tile (pipeline fill, epilogue) is a third of its time and only another resident workgroup hides it
// (a 256 x 256 tile at one workgroup per CU measured slower for exactly that reason).
//
// Pipeline (the role the cp.async pipeline plays in Section 3.2): k advances in steps of 32 through a
// ring of three LDS stages filled by LDS-DMA loads (global_load_lds_dwordx4: no staging registers,
// lane i of an instruction lands at base + 16 i).  Iteration kt waits for its own DMA of tile kt, passes
// one barrier (tile kt complete for everybody, tile kt-1 vacated by everybody), requests tile kt+2
// into the vacated stage - two iterations of flight time - and multiplies tile kt; the fragment reads
// of the second 16-deep step are issued behind the first MFMAs of the first step, so that they run
// under matrix work and nothing waits on them early.  LDS rows are 64 bytes; 16-byte chunks are
// XOR-swizzled over 128-byte lines (each DMA lane fetches the chunk that belongs in its slot), which
// makes the fragment reads bank-conflict free without padding.
//
// Rows are addressed through 64-row blocks so that the same kernel runs on a contiguous range or on
// a list of candidate blocks (last-layer pruning).
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace flame {

namespace {

constexpr int BM = 256;
constexpr int BK = 32;
constexpr int RB = BM / kRowAlign;      // 64-row blocks per row tile

struct PlaneSel { int id[4]; int n; };

// byte offset of 16-byte chunk c (0..3) of tile row `row` inside one LDS operand.  Four 64-byte rows share a 256-byte
// group: row bits 0..1 pick the quarter, and the chunk index is XORed with row bits 2..3.  The LDS serves 256 bytes
// = 16 lanes x 16 bytes per clock from 64 banks, and the 16 lanes of a ds_read_b128 that it serves together are not
// 16 consecutive ones: measured on this chip (chip_microbench, the four ds_read_b128 lines), lanes {0-3, 12-15, 20-23,
// 24-27} go together, then {4-7, 8-11, 16-19, 28-31}, and likewise in the upper half of the wavefront.  With this key
// both fragment row orders used below (identity, and sigma32: lane m reads row 16 bit2(m) + 4 (m / 8) + m % 4) put
// the four quads of such a group into four different key values, i.e. 16 different slots: 240 and 225 bytes per clock
// and CU.  (A key with row bit 3 ^ bit 4 in place of bit 3, which is free of conflicts for 16 consecutive lanes,
// measured 127.)
__device__ __forceinline__ int lds_key(int row) { return (row >> 2) & 3; }
__device__ __forceinline__ int lds_off(int row, int c) {
  return (row >> 2) * 256 + ((((row & 3) << 2) | (c ^ lds_key(row))) << 4);
}
// XOR key of the chunk index in an epilogue patch whose rows hold CPR 16-byte chunks (8: 128-byte rows,
// two per 256-byte group; 4: 64-byte rows, four per group): 16 consecutive rows of one chunk column use
// every slot of the 256 bytes once.
template <int CPR>
__device__ __forceinline__ int patch_key(int row) { return CPR == 8 ? (row >> 1) & 7 : (row >> 2) & 3; }

// Row order of the MFMA A operand.  Accumulator element e of lane (l32, lhalf) belongs to A-operand
// row 8*(e/4) + 4*lhalf + e%4.  Feeding tile row sigma32(m) = 16*bit2(m) + 4*(m/8) + m%4 into A-operand
// row m turns that into tile row 16*lhalf + e: a lane then owns 16 consecutive outputs (features of
// one token, or tokens of one feature for the feature-major plane) and stores them as two 16-byte
// words, two lanes covering a contiguous 64 bytes.
__device__ __forceinline__ int sigma32(int m) { return ((m & 4) << 2) | ((m >> 3) << 2) | (m & 3); }

template <int BN, int EPI>
__global__ __launch_bounds__(256, 2) void gemm_mfma_kernel(
    const half_t *__restrict__ A, const half_t *__restrict__ W, const bf16_t *__restrict__ bias,
    PlanePtrs planes, half_t *__restrict__ Xl, half_t *__restrict__ Xh, int lo_is_zero,
    const int32_t *__restrict__ blk_list, int blk_first, int n_blk, int n_row_tiles, int n_col_tiles, int K, int d,
    int64_t ws_rows, PlaneSel sel, float alpha, bool a_blocked) {
  constexpr int WN = BN / 2;            // wavefront patch: 128 rows x WN columns
  constexpr int MB = 4;                 // 32-row MFMA blocks per wavefront
  constexpr int NB = WN / 32;           // 32-column MFMA blocks per wavefront
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  constexpr int NSTAGE = 3;
  __shared__ __attribute__((aligned(128))) char smem[NSTAGE * STAGE];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
  // the 64-row blocks of this row tile (-1: absent; loads then fall back to the first block)
  int blk[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    const int t = row_tile * RB + r;
    blk[r] = t < n_blk ? (blk_list ? blk_list[t] : blk_first + t) : -1;
  }

  // LDS-DMA sources.  One instruction of a wavefront fills 1 KB = four 256-byte groups = 16 tile rows;
  // lane p owns physical slot p & 15 of group p >> 4 and must fetch the chunk the swizzle maps there:
  // row = 4 * group + (slot >> 2), chunk = (slot & 3) ^ key(row).  Instruction q of wavefront w covers tile
  // rows 16 * (4 q + w) .. + 15 (A: q = 0..3, one 64-row block each; B: q < BN / 64).
  constexpr int A_Q = BM / 64, B_Q = BN / 64;
  const int rloc = 16 * wave + 4 * (lane >> 4) + ((lane & 15) >> 2);
  const int dch = (lane & 3) ^ lds_key(rloc);
  // W is k-tile blocked (64 rows x 32 k = 2048 contiguous elements, whole 128-byte lines per request);
  // A is blocked too when it is the activation copy Xh, row-major when it is G.
  // Every request address is a wave-uniform base (64-row block and k tile: scalar arithmetic) plus a fixed 32-bit
  // lane offset in bytes, which is the scalar-base form of the request instruction: no vector address
  // arithmetic per k tile.  (Lane offsets are below 64 rows x K elements.)
  const char *abase[A_Q];
#pragma unroll
  for (int q = 0; q < A_Q; ++q) {
    const int b = blk[q] >= 0 ? blk[q] : blk[0];
    abase[q] = (const char *)(A + (int64_t)b * kRowAlign * K);
  }
  uint32_t alane = (uint32_t)(a_blocked ? rloc * 32 + dch * 8 : rloc * K + dch * 8) * 2u;
  const int a_kstep = (a_blocked ? 64 * BK : BK) * 2;                 // bytes per k tile
  const char *Wn0 = (const char *)(W + (int64_t)n0 * K);  // n0 % 64 == 0: a block boundary
  uint32_t blane = (uint32_t)(rloc * 32 + dch * 8) * 2u;
  // Operand order.  Row-major outputs (U, Q, K planes, X) want each lane to hold 4 consecutive
  // features of one token, which is the transposed accumulator: W rows as the A operand.  The V
  // plane is stored feature-major for the attention kernel (V^T is its A operand) and wants 4
  // consecutive tokens of one feature: activations as the A operand.
  const bool feature_major = (EPI == 0) && plane == 1;
  // Accumulators.  In the projection (EPI 0) they start from the bias, which then costs no instruction per
  // output: accumulator element e of block (i, j) is feature 32 j + 16 lhalf + e of the wavefront's columns
  // in the row-major planes, and feature 32 j + l32 (all elements alike) in the feature-major plane.
  f32x16 acc[MB][NB];
  if (EPI == 0) {
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const bf16_t *bp = bias + plane * d + n_in_plane + wn * WN + 32 * j;
      if (!feature_major) {
        const bf16x8 b0v = *(const bf16x8 *)(bp + 16 * lhalf), b1v = *(const bf16x8 *)(bp + 16 * lhalf + 8);
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[i][j][e] = (float)(e < 8 ? b0v[e & 7] : b1v[e & 7]);
      } else {
        const float bv = to_f32(bp[l32]);
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[i][j][e] = bv;
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  }
  // fragment byte offsets inside a stage for the two 16-deep steps (32-row blocks are 2048 bytes apart);
  // the operand that plays A is read in sigma32 row order
  int f0[2], g0[2];
  {
    const int ra = feature_major ? sigma32(l32) : l32, rb = feature_major ? l32 : sigma32(l32);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      f0[ks] = lds_off(wm * 128 + ra, ks * 2 + lhalf);
      g0[ks] = A_BYTES + lds_off(wn * WN + rb, ks * 2 + lhalf);
    }
  }

  typedef __attribute__((address_space(1))) const void gvoid;
  typedef __attribute__((address_space(3))) void lvoid;
  auto main_loop = [&](auto fm) {
    constexpr bool FM = decltype(fm)::value;
    const int nk = K / BK;
    const int k_rot = (n0 / BN) % nk;              // tied to the output columns, not to the launch's tile numbering
    auto request = [&](int tile, int stage) {            // A_Q + B_Q DMA instructions per wavefront
      // The workgroups that share a row tile (one per column tile) run at the same time on one XCD.  Each walks k
      // from a different starting tile (rotation by its column tile), so that they touch different lines of the
      // shared activations at any moment: one of them misses L2 on a line, the others hit it later, instead of
      // all of them missing together.
      int kt_ = (tile < nk ? tile : nk - 1) + k_rot;
      kt_ = kt_ >= nk ? kt_ - nk : kt_;
      // (the empty asm keeps the widening of the lane offsets next to the requests; hoisted out of the loop the
      // compiler would go back to full 64-bit vector addresses)
      asm volatile("" : "+v"(alane), "+v"(blane));
#pragma unroll
      for (int q = 0; q < A_Q; ++q)
        __builtin_amdgcn_global_load_lds((gvoid *)(abase[q] + (int64_t)kt_ * a_kstep + alane), (lvoid *)(smem + stage * STAGE + (4 * q + wave) * 1024), 16, 0, 0);
#pragma unroll
      for (int q = 0; q < B_Q; ++q)
        __builtin_amdgcn_global_load_lds((gvoid *)(Wn0 + ((size_t)q * 64 * K + (size_t)kt_ * (64 * BK)) * 2 + blane),
                                         (lvoid *)(smem + stage * STAGE + A_BYTES + (4 * q + wave) * 1024), 16, 0, 0);
    };
#define GEMM_MFMA(S, i, j)                                                                              \
  acc[i][j] = FM ? __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[S][i], fb[S][j], acc[i][j], 0, 0, 0)         \
                 : __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[S][j], fa[S][i], acc[i][j], 0, 0, 0)
    request(0, 0);
    request(1, 1);
    f16x8 fa[2][MB], fb[2][NB];
    // One k tile.  The stage is a compile-time constant (the loop below is unrolled over the ring), so the
    // fragment reads are a fixed lane offset plus an immediate and need no address instruction.
    auto k_step = [&](auto stage_c, const int kt) {
      constexpr int ST = decltype(stage_c)::value;
      // tile kt has landed for this wavefront once at most the requests of tile kt+1 are outstanding
      if (A_Q + B_Q == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      request(kt + 2, (ST + 2) % NSTAGE);
      const char *sp = smem + ST * STAGE;
#pragma unroll
      for (int i = 0; i < MB; ++i) fa[0][i] = *(const f16x8 *)(sp + f0[0] + i * 2048);
#pragma unroll
      for (int j = 0; j < NB; ++j) fb[0][j] = *(const f16x8 *)(sp + g0[0] + j * 2048);
      __builtin_amdgcn_sched_barrier(0);
      GEMM_MFMA(0, 0, 0);
      GEMM_MFMA(0, 1, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < MB; ++i) fa[1][i] = *(const f16x8 *)(sp + f0[1] + i * 2048);
#pragma unroll
      for (int j = 0; j < NB; ++j) fb[1][j] = *(const f16x8 *)(sp + g0[1] + j * 2048);
      __builtin_amdgcn_sched_barrier(0);
      GEMM_MFMA(0, 2, 0);
      GEMM_MFMA(0, 3, 0);
#pragma unroll
      for (int j = 1; j < NB; ++j)
#pragma unroll
        for (int i = 0; i < MB; ++i) GEMM_MFMA(0, i, j);
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int i = 0; i < MB; ++i) GEMM_MFMA(1, i, j);
      __builtin_amdgcn_sched_barrier(0);
    };
    static_assert(NSTAGE == 3, "the k loop is unrolled over a ring of three stages");
    for (int kt = 0; kt < nk; kt += NSTAGE) {
      k_step(std::integral_constant<int, 0>{}, kt);
      if (kt + 1 < nk) k_step(std::integral_constant<int, 1>{}, kt + 1);
      if (kt + 2 < nk) k_step(std::integral_constant<int, 2>{}, kt + 2);
    }
#undef GEMM_MFMA
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the clamped tail requests must not outlive the workgroup's LDS
  };
  if (feature_major) main_loop(std::true_type{});
  else main_loop(std::false_type{});

  // Epilogue.  With the sigma32 row order accumulator element e of a 32x32 block sits at (A-operand
  // tile row 16*lhalf + e, B-operand tile row l32).
  const int b0 = wm ? blk[2] : blk[0], b1 = wm ? blk[3] : blk[1];    // the two 64-row blocks of this wavefront's 128 rows
  if (EPI == 0) {
    // Only two lanes share an output row in the accumulator layout, so direct stores would reach the
    // L2 as 32-byte pieces, and the write path is then bound by the number of requests.  The
    // wavefront's patch goes through LDS instead (the operand ring is free by now; each wavefront
    // owns a private slice of it, chunks XOR-swizzled by row so that writes and reads are conflict free) and leaves as 16 bytes per lane with
    // whole 128-byte lines per output row.
    __builtin_amdgcn_s_barrier();                     // every wavefront has finished reading the ring
    char *pb = smem + wave * (128 * WN * 2);
    half_t *P = (half_t *)(plane == 0 ? planes.u : plane == 1 ? planes.v : plane == 2 ? planes.q : planes.k);
    if (!feature_major) {
      // patch[128 tokens][WN features]; lane holds token 32i + l32, features 32j + 16*lhalf + 0..15
      // (the bias is already in the accumulators).  Q leaves this kernel multiplied by alpha / 2: the
      // attention kernel works on halved logits; the other planes are stored plain.
      constexpr int CPR = WN / 8;                     // 16-byte chunks per patch row
      auto to_patch = [&](auto scaled) {
        const float sc = alpha * 0.5f;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
#pragma unroll
          for (int i = 0; i < MB; ++i) {
            const int row = 32 * i + l32;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
              f16x8 o;
#pragma unroll
              for (int q = 0; q < 8; ++q) {
                const float w = silu_fast(acc[i][j][8 * g + q]);
                o[q] = to_f16_sat(decltype(scaled)::value ? w * sc : w);
              }
              const int c = 4 * j + 2 * lhalf + g;
              *(f16x8 *)(pb + row * (WN * 2) + ((c ^ patch_key<CPR>(row)) << 4)) = o;
            }
          }
        }
      };
      if (plane == 2) to_patch(std::true_type{});
      else to_patch(std::false_type{});
      constexpr int RPI = 64 / CPR;                   // patch rows per store instruction
      const int rl = lane / CPR, c = lane % CPR;
      // Store instruction `it` takes patch rows it * RPI + rl.  No address arithmetic per instruction: the
      // patch address is a fixed lane offset plus an immediate (rows RPI apart share their swizzle key, except
      // that with 8 chunks per row every other instruction flips bit 2 of it), and the global address is a
      // scalar base (64-row block, row group, column: wave-uniform) plus the fixed lane offset of (rl, c).
      static_assert(CPR == 8 || CPR == 4, "patch rows of 128 or 64 bytes");
      constexpr int FLIP = CPR == 8 ? 64 : 0;
      const int lds0 = rl * (WN * 2) + ((c ^ patch_key<CPR>(rl)) << 4);
      uint32_t goff = (uint32_t)(rl * d + c * 8) * 2u;
      const char *gcol = (const char *)(P + n_in_plane + wn * WN);
      // the two 64-row blocks of the patch in turn: all reads of a block first, then its stores
      constexpr int NI = 64 / RPI;                    // store instructions per 64-row block
#pragma unroll
      for (int hb = 0; hb < 2; ++hb) {
        const int rblk = hb ? b1 : b0;
        if (rblk < 0) continue;
        const char *gblk = gcol + (int64_t)rblk * kRowAlign * d * 2;
        f16x8 v[NI];
#pragma unroll
        for (int k = 0; k < NI; ++k) {
          const int it = hb * NI + k;
          v[k] = *(const f16x8 *)(pb + it * RPI * (WN * 2) + (lds0 ^ ((it & 1) ? FLIP : 0)));
        }
        asm volatile("" : "+v"(goff));   // keeps the widening of the offset next to the stores (scalar base + offset form)
#pragma unroll
        for (int k = 0; k < NI; ++k)
          __builtin_nontemporal_store(v[k], (f16x8 *)(gblk + (int64_t)(k * RPI) * d * 2 + goff));
      }
    } else {
      // patch[WN features][128 tokens]; lane holds feature 32j + l32, tokens 32i + 16*lhalf + 0..15
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int fr = 32 * j + l32;
#pragma unroll
        for (int i = 0; i < MB; ++i) {
#pragma unroll
          for (int g = 0; g < 2; ++g) {
            f16x8 o;
#pragma unroll
            for (int q = 0; q < 8; ++q) o[q] = to_f16_sat(silu_fast(acc[i][j][8 * g + q]));
            const int c = 4 * i + 2 * lhalf + g;
            *(f16x8 *)(pb + fr * 256 + (((c ^ fr) & 15) << 4)) = o;
          }
        }
      }
      const int rl = lane >> 4, c = lane & 15;
      const int rblk = c >= 8 ? b1 : b0;
      // Store instruction `it` takes feature rows 4 it + rl.  As above: the patch address is a fixed lane offset
      // XOR a constant (the swizzle key of row 4 it + rl is that of rl XOR 4 it) plus an immediate, the global
      // address a scalar base (feature row group) plus a fixed lane offset (row rl, token block and chunk of c).
      const int lds0 = rl * 256 + ((c ^ rl) << 4);
      uint32_t goff = (uint32_t)((int64_t)rl * ws_rows + (int64_t)(rblk < 0 ? 0 : rblk) * kRowAlign + (c & 7) * 8) * 2u;
      const char *gfeat = (const char *)(P + (int64_t)(n_in_plane + wn * WN) * ws_rows);
      if (rblk >= 0) {
        constexpr int NI = 8;                           // reads in flight before their stores
#pragma unroll
        for (int i0 = 0; i0 < WN / 4; i0 += NI) {
          f16x8 v[NI];
#pragma unroll
          for (int k = 0; k < NI; ++k) {
            const int it = i0 + k;
            v[k] = *(const f16x8 *)(pb + it * 1024 + (lds0 ^ (((4 * it) & 15) << 4)));
          }
          asm volatile("" : "+v"(goff));
#pragma unroll
          for (int k = 0; k < NI; ++k)
            __builtin_nontemporal_store(v[k], (f16x8 *)(gfeat + (int64_t)(4 * (i0 + k)) * ws_rows * 2 + goff));
        }
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      const int rblk = i >= 2 ? b1 : b0;              // 32-row block i lies inside one 64-row block
      if (rblk < 0) continue;
      const int64_t m = (int64_t)rblk * kRowAlign + (i & 1) * 32 + l32;
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int nn = n0 + wn * WN + j * 32 + 16 * lhalf;
#pragma unroll
        for (int g = 0; g < 2; ++g) {
          const bf16x8 bv = *(const bf16x8 *)(bias + nn + 8 * g);
          const f16x8 h8 = *(const f16x8 *)(Xh + blocked_index(m, nn + 8 * g, d));
          f16x8 l8;
#pragma unroll
          for (int q = 0; q < 8; ++q) l8[q] = (half_t)0.f;
          if (!lo_is_zero) l8 = *(const f16x8 *)(Xl + m * d + nn + 8 * g);
          f16x8 o, ol;
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            const float x = ((float)h8[q] + (float)l8[q]) + (acc[i][j][8 * g + q] + (float)bv[q]);
            o[q] = to_f16_sat(x);
            ol[q] = to_f16_sat(x - (float)o[q]);
          }
          *(f16x8 *)(Xl + m * d + nn + 8 * g) = ol;
          *(f16x8 *)(Xh + blocked_index(m, nn + 8 * g, d)) = o;
        }
      }
    }
  }
}


}  // namespace

void launch_uvqk_bf16(const void *Xh, const void *W1h, const void *b1, PlanePtrs planes, const int32_t *blk_list,
                      int n_blk, int blk_first, int plane_mask, const Shape &sh, hipStream_t s) {
  if (n_blk <= 0 || !(plane_mask & 0xF)) return;
  PlaneSel sel{};
  for (int p = 0; p < 4; ++p)
    if (plane_mask & (1 << p)) sel.id[sel.n++] = p;
  const int row_tiles = (n_blk + RB - 1) / RB;
  if (sh.d % 128 == 0) {
    const int col_tiles = sel.n * (sh.d / 128);
    gemm_mfma_kernel<128, 0><<<row_tiles * col_tiles, 256, 0, s>>>((const half_t *)Xh, (const half_t *)W1h, (const bf16_t *)b1,
                                                                   planes, nullptr, nullptr, 0, blk_list, blk_first, n_blk,
                                                                   row_tiles, col_tiles, sh.d, sh.d, sh.ws_rows, sel, sh.alpha, true);
  } else {
    const int col_tiles = sel.n * (sh.d / 64);
    gemm_mfma_kernel<64, 0><<<row_tiles * col_tiles, 256, 0, s>>>((const half_t *)Xh, (const half_t *)W1h, (const bf16_t *)b1,
                                                                  planes, nullptr, nullptr, 0, blk_list, blk_first, n_blk,
                                                                  row_tiles, col_tiles, sh.d, sh.d, sh.ws_rows, sel, sh.alpha, true);
  }
}

void launch_outproj_bf16(const void *G, const void *W2h, const void *b2, void *Xh, void *Xl, bool lo_is_zero, const int32_t *blk_list,
                         int n_blk, int blk_first, const Shape &sh, hipStream_t s) {
  if (n_blk <= 0) return;
  PlaneSel sel{};
  const int row_tiles = (n_blk + RB - 1) / RB;
  if (sh.d % 128 == 0) {
    const int col_tiles = sh.d / 128;
    gemm_mfma_kernel<128, 1><<<row_tiles * col_tiles, 256, 0, s>>>((const half_t *)G, (const half_t *)W2h, (const bf16_t *)b2, PlanePtrs{}, (half_t *)Xl,
                                                                   (half_t *)Xh, lo_is_zero ? 1 : 0, blk_list, blk_first, n_blk, row_tiles, col_tiles,
                                                                   sh.d, sh.d, sh.ws_rows, sel, 1.0f, false);
  } else {
    const int col_tiles = sh.d / 64;
    gemm_mfma_kernel<64, 1><<<row_tiles * col_tiles, 256, 0, s>>>((const half_t *)G, (const half_t *)W2h, (const bf16_t *)b2, PlanePtrs{}, (half_t *)Xl,
                                                                  (half_t *)Xh, lo_is_zero ? 1 : 0, blk_list, blk_first, n_blk, row_tiles, col_tiles,
                                                                  sh.d, sh.d, sh.ws_rows, sel, 1.0f, false);
  }
}

}  // namespace flame
