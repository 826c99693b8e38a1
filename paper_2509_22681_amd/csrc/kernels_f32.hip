// fp32 instantiation of the GR block: plain FMA kernels with LDS tiling.  This path exists for
// the 1e-4 parity case and for any shape the MFMA path does not cover; it is not tuned.
#include "device_common.h"
#include "kernels.h"

namespace flame {

// ---------------------------------------------------------------------------------------------
// C[m][n] = sum_k A[m][k] W[n][k] + bias[n] over 64-row blocks, 64x64 tile, 16-deep k chunks,
// 256 threads each owning a 4x4 patch.  EPI 0: silu -> planes[n / d][m][n % d].
// EPI 1: X[m][n] += value (residual update in place).
// ---------------------------------------------------------------------------------------------
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ A, const float *__restrict__ W,
                                                       const float *__restrict__ bias, float *__restrict__ out,
                                                       const int32_t *__restrict__ blk_list, int blk_first,
                                                       int K, int Ncols, int d, int64_t plane_stride) {
  __shared__ float sA[16][64 + 1];
  __shared__ float sW[16][64 + 1];
  const int blk = blk_list ? blk_list[blockIdx.x] : blk_first + blockIdx.x;
  const int64_t row0 = (int64_t)blk * kRowAlign;
  const int n0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int i = threadIdx.x; i < 64 * 16; i += 256) {
      const int r = i >> 4, k = i & 15;
      sA[k][r] = (k0 + k < K) ? A[(row0 + r) * K + k0 + k] : 0.f;
      sW[k][r] = (k0 + k < K && n0 + r < Ncols) ? W[(int64_t)(n0 + r) * K + k0 + k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = sA[k][ty * 4 + i]; w[i] = sW[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      const int64_t m = row0 + ty * 4 + i;
      if (n >= Ncols) continue;
      const float v = acc[i][j] + bias[n];
      if (EPI == 0) out[(int64_t)(n / d) * plane_stride + m * d + (n % d)] = silu_f32(v);
      else out[m * Ncols + n] += v;
    }
}

void launch_uvqk_f32(const float *X, const float *W1, const float *b1, float *planes, int blk_first, int n_blk,
                     const Shape &sh, hipStream_t s) {
  if (n_blk <= 0) return;
  dim3 grid(n_blk, (4 * sh.d + 63) / 64);
  gemm_f32_kernel<0><<<grid, 256, 0, s>>>(X, W1, b1, planes, nullptr, blk_first, sh.d, 4 * sh.d, sh.d, sh.ws_rows * sh.d);
}

void launch_outproj_f32(const float *G, const float *W2, const float *b2, float *X, const int32_t *blk_list,
                        int n_blk, int blk_first, const Shape &sh, hipStream_t s) {
  if (n_blk <= 0) return;
  dim3 grid(n_blk, (sh.d + 63) / 64);
  gemm_f32_kernel<1><<<grid, 256, 0, s>>>(G, W2, b2, X, blk_list, blk_first, sh.d, sh.d, sh.d, 0);
}

// ---------------------------------------------------------------------------------------------
// Attention, one wavefront per query row.  Keys are taken 64 at a time: lane c computes
// silu(alpha <Q_r,K_c> + bias[p_r - p_c]) for its key, the 64 weights go through LDS, then lane j
// accumulates sum_c weight_c V_c[j].  Fixed summation order: results are run-to-run identical.
// ---------------------------------------------------------------------------------------------
template <bool SOFTMAX>
__global__ __launch_bounds__(256) void attn_f32_kernel(const float *__restrict__ U_V_Q_K, const float *__restrict__ bias_lh,
                                                       const float *__restrict__ tscale_h,
                                                       float *__restrict__ O, const AttnItem *__restrict__ items,
                                                       int q_tile, int d, int dh, int D, float alpha, int64_t plane_stride) {
  __shared__ float sQ[4][256];
  __shared__ float sP[4][64];
  const AttnItem it = items[blockIdx.x];
  const int h = blockIdx.y;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const float *Vp = U_V_Q_K + 1 * plane_stride + h * dh;
  const float *Qp = U_V_Q_K + 2 * plane_stride + h * dh;
  const float *Kp = U_V_Q_K + 3 * plane_stride + h * dh;
  const float *bias = bias_lh + (int64_t)h * D;
  for (int qi = wave; qi < it.n_q; qi += 4) {
    const int64_t qrow = it.q_row + qi;
    const int q_index = it.is_cand ? it.L : it.q_pos + qi;
    const int n_vis = visible_history(it.is_cand, q_index, it.L);
    for (int k = lane; k < dh; k += 64) sQ[wave][k] = Qp[qrow * d + k];
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    // softmax: running maximum and sum of the row (in units of the scaled logit), a finite stand-in for -inf
    constexpr float kNeg = -1.0e30f;
    const float ts = SOFTMAX ? tscale_h[h] : 0.f;
    float m_run = kNeg, l_run = 0.f;
    // history keys, then (candidates only) the row itself as one more key at distance 0
    const int n_keys = n_vis + (it.is_cand ? 1 : 0);
    for (int c0 = 0; c0 < n_keys; c0 += 64) {
      const int c = c0 + lane;
      float p = 0.f, z = kNeg;
      if (c < n_keys) {
        const bool self = c >= n_vis;
        const int64_t krow = self ? qrow : (int64_t)it.kv_row + c;
        const int delta = self ? 0 : q_index - c;
        float dot = 0.f;
        for (int k = 0; k < dh; ++k) dot = fmaf(sQ[wave][k], Kp[krow * d + k], dot);
        const float logit = alpha * dot + bias[delta < D ? delta : D - 1];
        if (SOFTMAX) z = logit * ts;
        else p = silu_f32(logit);
      }
      if (SOFTMAX) {
        const float m_new = fmaxf(m_run, wave_max(z));
        const float sc = expf(m_run - m_new);
        p = c < n_keys ? expf(z - m_new) : 0.f;
        l_run = l_run * sc + wave_sum(p);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] *= sc;
        m_run = m_new;
      }
      sP[wave][lane] = p;
      const int cn = min(64, n_keys - c0);
      for (int cc = 0; cc < cn; ++cc) {
        const bool self = c0 + cc >= n_vis;
        const int64_t vrow = self ? qrow : (int64_t)it.kv_row + c0 + cc;
        const float pw = sP[wave][cc];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int k = lane + j * 64;
          if (k < dh) acc[j] = fmaf(pw, Vp[vrow * d + k], acc[j]);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = lane + j * 64;
      if (k < dh) O[qrow * d + h * dh + k] = SOFTMAX ? acc[j] / l_run : acc[j];
    }
  }
}

void launch_attn_f32(const float *planes, const float *bias_lh, const float *tscale_h, float *O, const AttnItem *items,
                     int n_items, int q_tile, const Shape &sh, hipStream_t s) {
  if (n_items <= 0) return;
  dim3 grid(n_items, sh.H);
  if (sh.softmax)
    attn_f32_kernel<true><<<grid, 256, 0, s>>>(planes, bias_lh, tscale_h, O, items, q_tile, sh.d, sh.dh, sh.D, sh.alpha, sh.ws_rows * sh.d);
  else
    attn_f32_kernel<false><<<grid, 256, 0, s>>>(planes, bias_lh, tscale_h, O, items, q_tile, sh.d, sh.dh, sh.D, sh.alpha, sh.ws_rows * sh.d);
}

}  // namespace flame
