// Fusion of the sub-sequence blocks and the task head of the paper's model (flame_climber.h):
//   g_b = sigmoid([H_0 | ... | H_{Nb-1}] Wg_b^T + cg_b),  F = sum_b g_b * H_b,
//   p_t = sigmoid(<v_t, relu(F A_t^T + a_t)> + c_t).
// fp32 FMA kernels with LDS tiling (64 x 64 output tile, 64-deep k chunks, 256 threads each owning a
// 4 x 4 patch): correct and allocation-free, not tuned - at the paper's shapes this stage is a few
// per cent of the block stacks' work.
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
