// Fusion of the sub-sequence blocks and the task head of the paper's model (flame_climber.h):
//   g_b = sigmoid([H_0 | ... | H_{Nb-1}] Wg_b^T + cg_b),  F = sum_b g_b * H_b,
//   p_t = sigmoid(<v_t, relu(F A_t^T + a_t)> + c_t).
// Both products run on the fp32 matrix instruction (32 x 32 x 2, fp32 operands and accumulator, the same
// arithmetic as a chain of FMAs) whenever d is a multiple of 32 and the operands are 16-byte aligned: a
// wavefront owns a 32 x 32 output tile and feeds the instruction straight from global memory, one 16-byte
// load per operand and lane for four instructions, no LDS staging.  Other shapes take fp32 FMA kernels with
// LDS tiling (64 x 64 output tile, 64-deep k chunks, 256 threads each owning a 4 x 4 patch).
#include <hip/hip_runtime.h>

#include "../../include/flame_climber.h"

namespace {

constexpr int kMaxBlocks = FLAME_CLIMBER_MAX_BLOCKS;

struct HiddenPtrs { const float *h[kMaxBlocks]; };

__device__ __forceinline__ float sigmoid_f32(float x) { return 1.0f / (1.0f + expf(-x)); }

constexpr int KC = 64;   // k chunk: deep enough that a workgroup's chain of dependent global loads stays short

// One k chunk of a 64 x 64 tile product: sA/sW hold [k][row] and [k][column]; every thread owns a 4 x 4 patch.
__device__ __forceinline__ void tile_fma(const float (*sA)[64 + 1], const float (*sW)[64 + 1], int tx, int ty, float (&acc)[4][4]) {
#pragma unroll 8
  for (int k = 0; k < KC; ++k) {
    float a[4], w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i] = sA[k][ty * 4 + i]; w[i] = sW[k][tx * 4 + i]; }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
  }
}

// Fill one operand chunk: rows r0 .. r0+63 of a row-major matrix with row pitch `pitch`, columns k0 .. k0+63
// (zero outside n_rows / n_cols).  Thread (kk = tid & 63, rq = tid >> 6) takes column kk of rows rq, rq+4, ...:
// 16 independent loads per thread, 256 contiguous bytes per row and wavefront.
__device__ __forceinline__ void fill_chunk(float (*dst)[64 + 1], const float *__restrict__ src, int64_t r0, int64_t n_rows,
                                           int64_t pitch, int k0, int n_cols) {
  const int kk = threadIdx.x & 63, rq = threadIdx.x >> 6;
  const bool kin = k0 + kk < n_cols;
  float v[16];
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int64_t r = r0 + rq + 4 * q;
    v[q] = (kin && r < n_rows) ? src[r * pitch + k0 + kk] : 0.f;
  }
#pragma unroll
  for (int q = 0; q < 16; ++q) dst[kk][rq + 4 * q] = v[q];
}

// F[r][f] for a 64 x 64 tile: for every block b one GEMM over the concatenation [H_0 | ... | H_{Nb-1}] (walked
// source block by source block), closed by the gate and the product with H_b.
__global__ __launch_bounds__(256) void fuse_kernel(HiddenPtrs H, int n_blocks, const float *__restrict__ wg,
                                                   const float *__restrict__ cg, float *__restrict__ F, int64_t rows, int d) {
  __shared__ float sA[KC][64 + 1];
  __shared__ float sW[KC][64 + 1];
  const int64_t row0 = (int64_t)blockIdx.x * 64;
  const int f0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int K = n_blocks * d;
  float fused[4][4] = {};
  for (int b = 0; b < n_blocks; ++b) {
    const float *W = wg + (int64_t)b * d * K;          // [d][K]
    float acc[4][4] = {};
    for (int sb = 0; sb < n_blocks; ++sb)
      for (int k0 = 0; k0 < d; k0 += KC) {
        fill_chunk(sA, H.h[sb], row0, rows, d, k0, d);
        fill_chunk(sW, W + (int64_t)sb * d, f0, d, K, k0, d);
        __syncthreads();
        tile_fma(sA, sW, tx, ty, acc);
        __syncthreads();
      }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int f = f0 + tx * 4 + j;
        const int64_t r = row0 + ty * 4 + i;
        if (f < d && r < rows) fused[i][j] = fmaf(sigmoid_f32(acc[i][j] + cg[b * d + f]), H.h[b][r * d + f], fused[i][j]);
      }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int f = f0 + tx * 4 + j;
      const int64_t r = row0 + ty * 4 + i;
      if (f < d && r < rows) F[r * d + f] = fused[i][j];
    }
}

// probs[r][t] for 64 rows and one task: the expert layer is walked in chunks of 64 units; every thread keeps
// the partial <v, relu(.)> of its 4 rows over its 4 units per chunk, the 16 threads of a row are summed at the
// end through LDS in a fixed order.
__global__ __launch_bounds__(256) void expert_kernel(const float *__restrict__ F, const float *__restrict__ a_w,
                                                     const float *__restrict__ a_b, const float *__restrict__ v,
                                                     const float *__restrict__ c, float *__restrict__ probs, int64_t rows,
                                                     int d, int E, int T) {
  __shared__ float sA[KC][64 + 1];
  __shared__ float sW[KC][64 + 1];
  const int64_t row0 = (int64_t)blockIdx.x * 64;
  const int t = blockIdx.y;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const float *W = a_w + (int64_t)t * E * d;            // [E][d]
  float part[4] = {0.f, 0.f, 0.f, 0.f};
  for (int e0 = 0; e0 < E; e0 += 64) {
    float acc[4][4] = {};
    for (int k0 = 0; k0 < d; k0 += KC) {
      fill_chunk(sA, F, row0, rows, d, k0, d);
      fill_chunk(sW, W, e0, E, d, k0, d);
      __syncthreads();
      tile_fma(sA, sW, tx, ty, acc);
      __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int e = e0 + tx * 4 + j;
      if (e < E) {
        const float ab = a_b[t * E + e], ve = v[t * E + e];
#pragma unroll
        for (int i = 0; i < 4; ++i) part[i] = fmaf(fmaxf(acc[i][j] + ab, 0.f), ve, part[i]);
      }
    }
  }
  // sum over the 16 threads of a row, through a slice of sA (free by now)
  float (*sR)[16 + 1] = (float (*)[16 + 1])&sA[0][0];
#pragma unroll
  for (int i = 0; i < 4; ++i) sR[ty * 4 + i][tx] = part[i];
  __syncthreads();
  if (threadIdx.x < 64) {
    const int64_t r = row0 + threadIdx.x;
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) s += sR[threadIdx.x][k];
    if (r < rows) probs[r * T + t] = sigmoid_f32(s + c[t]);
  }
}

typedef float f32x16 __attribute__((ext_vector_type(16)));

// The fp32 matrix instruction computes acc[i][j] += sum over its two k slots of A[i][k] W[j][k] for 32 rows i and
// 32 rows j: lane l supplies row l & 31 of both operands, k slot l >> 5.  A lane reads 4 consecutive floats of
// its row at offset 4 * (l >> 5) of every group of 8: the two lane halves then hold the k slots {8s + t} and
// {8s + 4 + t} of instruction t of step s.  Accumulator element e of a lane is output row
// 8 * (e / 4) + 4 * (l >> 5) + e % 4, column l & 31.
__device__ __forceinline__ void mfma_step(const float4 a, const float4 w, f32x16 &acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, w.x, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, w.y, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, w.z, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, w.w, acc, 0, 0, 0);
}

// Both kernels below stream ALL their steps (every gate block, every group of expert units) through one ring of
// PD float4 pairs per lane: as soon as step s has been issued, its slot is refilled with the operands of step
// s + PD, across the boundaries between products, so the memory latency is paid once per kernel and not once
// per product.  Refilling after the use (not before) lets old and new value share registers; the request
// cursor stops at the last step instead of being guarded, so the loop body has no branch; the scheduling
// barriers keep the compiler from moving the requests down to their first use.  Products end on a multiple of
// PD steps (d a multiple of 8 * PD).
constexpr int PD = 4;

// Fusion on the matrix instruction: workgroup = 32 rows x (4 wavefronts x 32 features).  Rows and features
// past the end are clamped for the loads and dropped at the store.  No barrier: a wavefront with no feature
// tile leaves at once.
__global__ __launch_bounds__(256) void fuse_mfma_kernel(HiddenPtrs H, int n_blocks, const float *__restrict__ wg,
                                                        const float *__restrict__ cg, float *__restrict__ F, int64_t rows, int d) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, lh = lane >> 5;
  const int f0 = (blockIdx.y * 4 + wave) * 32;
  if (f0 >= d) return;
  const int64_t row0 = (int64_t)blockIdx.x * 32;
  const int64_t aoff = min(row0 + l32, rows - 1) * d + 4 * lh;
  const int wrow = min(f0 + l32, d - 1);
  const int K = n_blocks * d;
  const int sd = d >> 3;             // steps per source block
  const int spb = n_blocks * sd;     // steps per gate block
  const int total = n_blocks * spb;
  const float *wbase = wg + (int64_t)wrow * K + 4 * lh;
  const int64_t wpitch = (int64_t)d * K;
  // request cursor: gate block pb, source block psb, step pk in the source block, step pr in the gate block
  int pb = 0, psb = 0, pk = 0, pr = 0, pq = 0;
  const float *hp = H.h[0] + aoff;
  const float *wp = wbase;
  auto fetch = [&](float4 &a, float4 &w) {
    a = *(const float4 *)(hp + 8 * pk);
    w = *(const float4 *)(wp + 8 * pr);
    if (pq < total - 1) {
      ++pq;
      ++pr;
      if (++pk == sd) {
        pk = 0;
        if (++psb == n_blocks) {
          psb = 0;
          pr = 0;
          ++pb;
          wp = wbase + pb * wpitch;
        }
        hp = H.h[psb] + aoff;
      }
    }
  };
  // operands of the gate of block cb: its bias and this lane's 16 elements of H_cb, requested a product ahead
  const int f = f0 + l32;
  const bool fin = f < d;
  float hb[16], bias;
  auto fetch_gate = [&](int cb) {
    bias = cg[cb * d + wrow];
    const float *Hb = H.h[cb];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int64_t r = min(row0 + 8 * (e >> 2) + 4 * lh + (e & 3), rows - 1);
      hb[e] = Hb[r * d + wrow];
    }
  };
  float4 a[PD], w[PD];
#pragma unroll
  for (int p = 0; p < PD; ++p) fetch(a[p], w[p]);
  fetch_gate(0);
  f32x16 fused = {}, acc = {};
  int cb = 0, left = spb;
  for (int s0 = 0; s0 < total; s0 += PD) {
#pragma unroll
    for (int p = 0; p < PD; ++p) {
      mfma_step(a[p], w[p], acc);
      __builtin_amdgcn_sched_barrier(0);
      fetch(a[p], w[p]);
      __builtin_amdgcn_sched_barrier(0);
    }
    left -= PD;
    if (left == 0) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        fused[e] = fmaf(sigmoid_f32(acc[e] + bias), hb[e], fused[e]);
        acc[e] = 0.f;
      }
      // the next gate's operands reuse hb's registers: requested after the use above, and without a branch
      // (after the last gate the request repeats itself), so that the barrier holds them in place
      __builtin_amdgcn_sched_barrier(0);
      cb = min(cb + 1, n_blocks - 1);
      fetch_gate(cb);
      left = spb;
    }
  }
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int64_t r = row0 + 8 * (e >> 2) + 4 * lh + (e & 3);
    if (fin && r < rows) F[r * d + f] = fused[e];
  }
}

// Task head on the matrix instruction: workgroup = 32 rows of one task; wavefront w takes the expert units
// [32 (w + 4 j), +32) and keeps <v, relu(.)> of its 16 rows over its units in registers.  The sum over the
// units of a row (32 lanes x 4 wavefronts) goes through LDS in a fixed order.
__global__ __launch_bounds__(256) void expert_mfma_kernel(const float *__restrict__ F, const float *__restrict__ a_w,
                                                          const float *__restrict__ a_b, const float *__restrict__ v,
                                                          const float *__restrict__ c, float *__restrict__ probs, int64_t rows,
                                                          int d, int E, int T) {
  __shared__ float red[4][32][32 + 1];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l32 = lane & 31, lh = lane >> 5;
  const int64_t row0 = (int64_t)blockIdx.x * 32;
  const int t = blockIdx.y;
  const float *pa = F + min(row0 + l32, rows - 1) * d + 4 * lh;
  const int sd = d >> 3;
  const int nseg = wave * 32 < E ? (E - wave * 32 + 127) / 128 : 0;   // groups of 32 units this wavefront owns
  const int total = nseg * sd;
  float part[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) part[e] = 0.f;
  if (nseg > 0) {
    auto unit_of = [&](int j) { return min(wave * 32 + 128 * j + l32, E - 1); };
    auto wrow_of = [&](int j) { return a_w + ((int64_t)t * E + unit_of(j)) * d + 4 * lh; };
    int pj = 0, pk = 0, pq = 0;
    const float *wp = wrow_of(0);
    auto fetch = [&](float4 &a, float4 &w) {
      a = *(const float4 *)(pa + 8 * pk);
      w = *(const float4 *)(wp + 8 * pk);
      if (pq < total - 1) {
        ++pq;
        if (++pk == sd) {
          pk = 0;
          wp = wrow_of(++pj);
        }
      }
    };
    float ab, ve;
    bool live;   // units past E are computed on clamped operands and weighted 0
    auto fetch_unit = [&](int j) {
      ab = a_b[t * E + unit_of(j)];
      ve = v[t * E + unit_of(j)];
      live = wave * 32 + 128 * j + l32 < E;
    };
    float4 a[PD], w[PD];
#pragma unroll
    for (int p = 0; p < PD; ++p) fetch(a[p], w[p]);
    fetch_unit(0);
    f32x16 acc = {};
    int cj = 0, left = sd;
    for (int s0 = 0; s0 < total; s0 += PD) {
#pragma unroll
      for (int p = 0; p < PD; ++p) {
        mfma_step(a[p], w[p], acc);
        __builtin_amdgcn_sched_barrier(0);
        fetch(a[p], w[p]);
        __builtin_amdgcn_sched_barrier(0);
      }
      left -= PD;
      if (left == 0) {
        const float vl = live ? ve : 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          part[e] = fmaf(fmaxf(acc[e] + ab, 0.f), vl, part[e]);
          acc[e] = 0.f;
        }
        __builtin_amdgcn_sched_barrier(0);
        cj = min(cj + 1, nseg - 1);
        fetch_unit(cj);
        left = sd;
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 16; ++e) red[wave][8 * (e >> 2) + 4 * lh + (e & 3)][l32] = part[e];
  __syncthreads();
  // thread (row = tid / 8, seg = tid % 8) sums columns [4 seg, +4) of the four wavefronts, then the 8 threads of a row
  const int rr = threadIdx.x >> 3, seg = threadIdx.x & 7;
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w)
#pragma unroll
    for (int q = 0; q < 4; ++q) s += red[w][rr][seg * 4 + q];
  s += __shfl_xor(s, 1);
  s += __shfl_xor(s, 2);
  s += __shfl_xor(s, 4);
  const int64_t r = row0 + rr;
  if (seg == 0 && r < rows) probs[r * T + t] = sigmoid_f32(s + c[t]);
}

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

thread_local const char *g_head_error = "";

}  // namespace

extern "C" {

const char *flame_climber_last_error(void) { return g_head_error; }

int flame_climber_head(const flame_climber_head_config *cfg, const flame_climber_head_weights *w,
                       const float *const *hidden, int64_t n_rows, float *fused, float *probs, void *stream) {
  auto bad = [&](const char *m) { g_head_error = m; return (int)FLAME_GR_INVALID_ARGUMENT; };
  g_head_error = "";
  if (!cfg || !w || !hidden) return bad("a pointer argument is NULL");
  if (cfg->n_blocks < 1 || cfg->n_blocks > kMaxBlocks) return bad("n_blocks must be in [1, FLAME_CLIMBER_MAX_BLOCKS]");
  if (cfg->d_model < 1 || cfg->n_tasks < 1 || cfg->n_tasks > 64 || cfg->expert_width < 1) return bad("d_model, n_tasks (1..64) and expert_width must be positive");
  if (n_rows < 0 || n_rows > (int64_t)1 << 31) return bad("n_rows out of range");
  if (n_rows == 0) return FLAME_GR_OK;
  if (!w->wg || !w->cg || !w->a_w || !w->a_b || !w->v || !w->c) return bad("a weight pointer is NULL");
  if (!fused || !probs) return bad("fused or probs is NULL");
  HiddenPtrs H{};
  for (int b = 0; b < cfg->n_blocks; ++b) {
    if (!hidden[b]) return bad("a hidden pointer is NULL");
    H.h[b] = hidden[b];
  }
  hipStream_t s = (hipStream_t)stream;
  bool mfma = cfg->d_model % (8 * PD) == 0 && aligned16(w->wg) && aligned16(w->a_w) && aligned16(fused);
  for (int b = 0; b < cfg->n_blocks; ++b) mfma = mfma && aligned16(hidden[b]);
  if (mfma) {
    const unsigned tiles32 = (unsigned)((n_rows + 31) / 32);
    fuse_mfma_kernel<<<dim3(tiles32, (cfg->d_model + 127) / 128), 256, 0, s>>>(H, cfg->n_blocks, w->wg, w->cg, fused, n_rows, cfg->d_model);
    expert_mfma_kernel<<<dim3(tiles32, cfg->n_tasks), 256, 0, s>>>(fused, w->a_w, w->a_b, w->v, w->c, probs, n_rows, cfg->d_model,
                                                                   cfg->expert_width, cfg->n_tasks);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { g_head_error = hipGetErrorString(e); return FLAME_GR_HIP_ERROR; }
    return FLAME_GR_OK;
  }
  const unsigned row_tiles = (unsigned)((n_rows + 63) / 64);
  fuse_kernel<<<dim3(row_tiles, (cfg->d_model + 63) / 64), 256, 0, s>>>(H, cfg->n_blocks, w->wg, w->cg, fused, n_rows, cfg->d_model);
  expert_kernel<<<dim3(row_tiles, cfg->n_tasks), 256, 0, s>>>(fused, w->a_w, w->a_b, w->v, w->c, probs, n_rows, cfg->d_model,
                                                            cfg->expert_width, cfg->n_tasks);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { g_head_error = hipGetErrorString(e); return FLAME_GR_HIP_ERROR; }
  return FLAME_GR_OK;
}

// Host-only: the sub-sequence of block b out of n_blocks of a history of L items.
int flame_climber_block_range(int32_t L, int32_t n_blocks, int32_t b, int32_t *begin, int32_t *end) {
  if (L < 0 || n_blocks < 1 || b < 0 || b >= n_blocks || !begin || !end) return FLAME_GR_INVALID_ARGUMENT;
  *begin = (int32_t)((int64_t)b * L / n_blocks);
  *end = (int32_t)((int64_t)(b + 1) * L / n_blocks);
  return FLAME_GR_OK;
}

}  // extern "C"
