// Small bandwidth-bound kernels of the GR forward: input assembly, bias-table expansion,
// LayerNorm * U gating, score head, and the debug evaluation of the mask predicate.
#include "device_common.h"
#include "kernels.h"

namespace flame {

// ---------------------------------------------------------------------------------------------
// Assembly: the token matrix of a request is its history rows followed by its candidate rows
// (Section 2.1: candidates are appended after the behaviour sequence).  One workgroup per 64-row
// block of the padded workspace; rows past n_valid are zero so that they stay finite downstream.
// fp32 path: X is row-major fp32.  MFMA path: the residual is held as two fp16 words, Xh = fp16(X) (k-tile blocked, the
// projection's operand) and Xl = fp16(X - Xh); embeddings are exact in Xh, so assembly writes Xh only and the first layer
// treats Xl as zero.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void assemble_kernel(const RowBlock *__restrict__ blocks, const int32_t *__restrict__ list, int blk_begin,
                                                       const T *__restrict__ hist, const T *__restrict__ cand,
                                                       float *__restrict__ X, half_t *__restrict__ Xh, int d) {
  const int b = list ? list[blockIdx.x] : blk_begin + blockIdx.x;
  const RowBlock rb = blocks[b];
  const T *src = rb.kind ? cand : hist;
  const int64_t dst0 = (int64_t)b * kRowAlign * d;
  const int n = kRowAlign * d;
  const int nv = rb.n_valid * d;
  for (int i = threadIdx.x; i < n; i += 256) {
    float v = 0.f;
    if (i < nv) v = to_f32(src[(int64_t)rb.src_row * d + i]);
    X[dst0 + i] = v;
    if (Xh) Xh[blocked_index((int64_t)b * kRowAlign + i / d, i % d, d)] = to_f16_sat(v);
  }
}

// bf16 inputs: 16 bytes per lane, each 64-row block cut into gridDim.y row slices so that a small batch
// still spreads over many compute units and no lane walks a long chain of dependent loads.
__global__ __launch_bounds__(256) void assemble_bf16_kernel(const RowBlock *__restrict__ blocks, const int32_t *__restrict__ list,
                                                            int blk_begin, const bf16_t *__restrict__ hist,
                                                            const bf16_t *__restrict__ cand, half_t *__restrict__ Xh, int d) {
  const int b = list ? list[blockIdx.x] : blk_begin + blockIdx.x;
  const RowBlock rb = blocks[b];
  const bf16_t *src = rb.kind ? cand : hist;
  const int cpr = d / 8;                                   // 16-byte chunks per row
  const int rows = kRowAlign / gridDim.y, r0 = blockIdx.y * rows;
  const int64_t row_base = (int64_t)b * kRowAlign;
#pragma unroll 4
  for (int i = threadIdx.x; i < rows * cpr; i += 256) {
    const int r = r0 + i / cpr, c = i % cpr;
    bf16x8 v;
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = (bf16_t)0.f;
    if (r < rb.n_valid) v = *(const bf16x8 *)(src + ((int64_t)rb.src_row + r) * d + c * 8);
    f16x8 o;
#pragma unroll
    for (int k = 0; k < 8; ++k) o[k] = to_f16_sat((float)v[k]);
    *(f16x8 *)(Xh + blocked_index(row_base + r, c * 8, d)) = o;
  }
}

void launch_assemble(int dtype, const RowBlock *blocks, const int32_t *list, int n, int first, const void *hist,
                     const void *cand, float *X, void *Xh, int d, hipStream_t s) {
  if (n <= 0) return;
  if (dtype == FLAME_GR_BF16)
    assemble_bf16_kernel<<<dim3(n, 4), 256, 0, s>>>(blocks, list, first, (const bf16_t *)hist, (const bf16_t *)cand, (half_t *)Xh, d);
  else
    assemble_kernel<float><<<n, 256, 0, s>>>(blocks, list, first, (const float *)hist, (const float *)cand, X, nullptr, d);
}

// ---------------------------------------------------------------------------------------------
// bias[lh][delta] = rab[lh][bucket(delta)]: the attention kernels index the bias by distance.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void expand_bias_kernel(const float *__restrict__ rab, const int32_t *__restrict__ tab,
                                                          float *__restrict__ bias, int nb, int D, float scale) {
  const int lh = blockIdx.y;
  for (int t = blockIdx.x * 256 + threadIdx.x; t < D; t += gridDim.x * 256)
    bias[(int64_t)lh * D + t] = rab[(int64_t)lh * nb + tab[t]] * scale;
}

void launch_expand_bias(const float *rab, const int32_t *bucket_tab, float *bias, int n_lh, int n_buckets,
                        int D, float scale, hipStream_t s) {
  dim3 grid((D + 255) / 256 > 64 ? 64 : (D + 255) / 256, n_lh);
  expand_bias_kernel<<<grid, 256, 0, s>>>(rab, bucket_tab, bias, n_buckets, D, scale);
}

__global__ __launch_bounds__(256) void logit_scale_kernel(const float *__restrict__ temperature, float *__restrict__ out, int n,
                                                          float factor) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) out[i] = factor / temperature[i];
}

void launch_logit_scale(const float *temperature, float *out, int n, float factor, hipStream_t s) {
  if (n > 0) logit_scale_kernel<<<(n + 255) / 256, 256, 0, s>>>(temperature, out, n, factor);
}

// ---------------------------------------------------------------------------------------------
// The candidates' final residual rows, in candidate order (the input of a fusion / head stage).
// ---------------------------------------------------------------------------------------------
// Xh != nullptr: the residual is the pair (Xh blocked, Xl row-major) of the MFMA path, else fp32 X.
__global__ __launch_bounds__(256) void gather_hidden_kernel(const float *__restrict__ X, const half_t *__restrict__ Xh,
                                                            const half_t *__restrict__ Xl, const RowBlock *__restrict__ blocks,
                                                            const int32_t *__restrict__ cand_blocks, float *__restrict__ hidden, int d) {
  const int b = cand_blocks[blockIdx.x];
  const RowBlock rb = blocks[b];
  const int n = rb.n_valid * d;
  const int64_t row0 = (int64_t)b * kRowAlign;
  float *dst = hidden + (int64_t)rb.src_row * d;
  for (int i = threadIdx.x; i < n; i += 256) {
    if (Xh) dst[i] = (float)Xh[blocked_index(row0 + i / d, i % d, d)] + (float)Xl[row0 * d + i];
    else dst[i] = X[row0 * d + i];
  }
}

void launch_gather_hidden(const float *X, const void *Xh, const void *Xl, const RowBlock *blocks, const int32_t *cand_blocks, int n_cblk,
                          float *hidden, int d, hipStream_t s) {
  if (n_cblk > 0) gather_hidden_kernel<<<n_cblk, 256, 0, s>>>(X, (const half_t *)Xh, (const half_t *)Xl, blocks, cand_blocks, hidden, d);
}

// Debug capture: the residual rows [row_begin, row_end) of the MFMA path as fp32 (Xh + Xl, exact).
__global__ __launch_bounds__(256) void residual_to_f32_kernel(const half_t *__restrict__ Xh, const half_t *__restrict__ Xl,
                                                              float *__restrict__ out, int64_t first, int64_t n, int d) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t e = first + i;
    out[e] = (float)Xh[blocked_index(e / d, (int)(e % d), d)] + (float)Xl[e];
  }
}

void launch_residual_to_f32(const void *Xh, const void *Xl, float *out, int64_t row_begin, int64_t row_end, int d, hipStream_t s) {
  const int64_t n = (row_end - row_begin) * d;
  if (n <= 0) return;
  const int grid = (int)((n + 255) / 256 > 4096 ? 4096 : (n + 255) / 256);
  residual_to_f32_kernel<<<grid, 256, 0, s>>>((const half_t *)Xh, (const half_t *)Xl, out, row_begin * d, n, d);
}

// ---------------------------------------------------------------------------------------------
// bf16 -> fp16 copy of the projection matrices.  The MFMA path works on fp16 operands: with eight
// to sixteen layers the 2^-9 rounding of bf16 intermediates alone puts about 1e-2 rms (5e-2 worst
// case) on the scores, fp16's 2^-12 keeps them ten times closer; weights of magnitude >= 2^-14 are
// represented exactly either way.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bf16_to_f16_kernel(const bf16_t *__restrict__ in, half_t *__restrict__ out, int64_t n8,
                                                          int K, bool blocked) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (int64_t)gridDim.x * 256) {
    const bf16x8 v = ((const bf16x8 *)in)[i];
    f16x8 o;
#pragma unroll
    for (int k = 0; k < 8; ++k) o[k] = to_f16_sat((float)v[k]);
    const int64_t e = i * 8;                              // 8 consecutive k of one row stay together
    *(f16x8 *)(out + (blocked ? blocked_index(e / K, (int)(e % K), K) : e)) = o;
  }
}

void launch_bf16_to_f16(const void *in, void *out, int64_t rows, int K, bool blocked, hipStream_t s) {
  const int64_t n8 = rows * K / 8;   // K % 64 == 0 in the MFMA path
  if (n8 <= 0) return;
  int grid = (int)((n8 + 255) / 256 > 2048 ? 2048 : (n8 + 255) / 256);
  bf16_to_f16_kernel<<<grid, 256, 0, s>>>((const bf16_t *)in, (half_t *)out, n8, K, blocked);
}

// ---------------------------------------------------------------------------------------------
// G = (LayerNorm_d(O) * gamma + beta) * U.  One wavefront per row, statistics in fp32 by wavefront
// reduction (mean first, then the centred second moment: biased variance).
// ---------------------------------------------------------------------------------------------
template <typename T, typename TW, int MAXV>   // T: activations (O, U, G); TW: stored weights (gamma, beta)
__global__ __launch_bounds__(256) void ln_gate_kernel(const T *__restrict__ O, const T *__restrict__ U,
                                                      const TW *__restrict__ gamma, const TW *__restrict__ beta,
                                                      T *__restrict__ G, const RowBlock *__restrict__ blocks,
                                                      const int32_t *__restrict__ blk_list, int blk_first, int d,
                                                      float eps) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int rb = blockIdx.x >> 4;                       // 16 workgroups of 4 rows per 64-row block
  const int blk = blk_list ? blk_list[rb] : blk_first + rb;
  const int in_blk = (blockIdx.x & 15) * 4 + wave;
  const int64_t row = (int64_t)blk * kRowAlign + in_blk;
  if (in_blk >= blocks[blk].n_valid) {                  // padding row: keep it finite (zero branch)
    for (int k = lane; k < d; k += 64) G[row * d + k] = from_f32<T>(0.f);
    return;
  }
  const T *o = O + row * d;
  float v[MAXV];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int k = lane + i * 64;
    v[i] = k < d ? to_f32(o[k]) : 0.f;
    sum += v[i];
  }
  const float mu = wave_sum(sum) / (float)d;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int k = lane + i * 64;
    const float c = k < d ? v[i] - mu : 0.f;
    sq += c * c;
  }
  const float rstd = rsqrtf(wave_sum(sq) / (float)d + eps);
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int k = lane + i * 64;
    if (k < d) {
      const float y = ((v[i] - mu) * rstd * to_f32(gamma[k]) + to_f32(beta[k])) * to_f32(U[row * d + k]);
      G[row * d + k] = from_f32<T>(y);
    }
  }
}

template <typename T, typename TW>
static void ln_gate_dispatch(const void *O, const void *U, const void *g, const void *b, void *G,
                             const RowBlock *blocks, const int32_t *blk_list, int n_blk, int blk_first, int d, float eps, hipStream_t s) {
  const int grid = n_blk * 16;
#define LN_CASE(MV) ln_gate_kernel<T, TW, MV><<<grid, 256, 0, s>>>((const T *)O, (const T *)U, (const TW *)g, (const TW *)b, (T *)G, blocks, blk_list, blk_first, d, eps)
  if (d <= 64) LN_CASE(1);
  else if (d <= 128) LN_CASE(2);
  else if (d <= 256) LN_CASE(4);
  else if (d <= 512) LN_CASE(8);
  else if (d <= 1024) LN_CASE(16);
  else LN_CASE(64);
#undef LN_CASE
}

void launch_ln_gate(int dtype, const void *O, const void *U, const void *gamma, const void *beta, void *G,
                    const RowBlock *blocks, const int32_t *blk_list, int n_blk, int blk_first, int d, float eps, hipStream_t s) {
  if (n_blk <= 0) return;
  if (dtype == FLAME_GR_BF16) ln_gate_dispatch<half_t, bf16_t>(O, U, gamma, beta, G, blocks, blk_list, n_blk, blk_first, d, eps, s);
  else ln_gate_dispatch<float, float>(O, U, gamma, beta, G, blocks, blk_list, n_blk, blk_first, d, eps, s);
}

// ---------------------------------------------------------------------------------------------
// Score head: one logit per candidate row, written in the caller's candidate order.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void score_kernel(const float *__restrict__ X, const half_t *__restrict__ Xh,
                                                    const half_t *__restrict__ Xl, const T *__restrict__ w_s, float b_s,
                                                    const RowBlock *__restrict__ blocks, const int32_t *__restrict__ cblk,
                                                    float *__restrict__ scores, int d) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int blk = cblk[blockIdx.x >> 4];
  const RowBlock rb = blocks[blk];
  const int i = (blockIdx.x & 15) * 4 + wave;
  if (i >= rb.n_valid) return;
  const int64_t row = (int64_t)blk * kRowAlign + i;
  float acc = 0.f;
  if constexpr (sizeof(T) == 2) {
    // MFMA path: 8 features per lane and step, 16-byte loads (8 consecutive k sit together in the blocked word too)
    for (int k = lane * 8; k < d; k += 512) {
      const f16x8 h8 = *(const f16x8 *)(Xh + blocked_index(row, k, d)), l8 = *(const f16x8 *)(Xl + row * d + k);
      const bf16x8 w8 = *(const bf16x8 *)(w_s + k);
#pragma unroll
      for (int q = 0; q < 8; ++q) acc += ((float)h8[q] + (float)l8[q]) * (float)w8[q];
    }
  } else {
    for (int k = lane; k < d; k += 64) acc += X[row * d + k] * to_f32(w_s[k]);
  }
  acc = wave_sum(acc);
  if (lane == 0) scores[rb.src_row + i] = acc + b_s;
}

void launch_scores(int dtype, const float *X, const void *Xh, const void *Xl, const void *w_s, float b_s, const RowBlock *blocks,
                   const int32_t *cand_blocks, int n_cblk, float *scores, int d, hipStream_t s) {
  if (n_cblk <= 0) return;
  if (dtype == FLAME_GR_BF16)
    score_kernel<bf16_t><<<n_cblk * 16, 256, 0, s>>>(nullptr, (const half_t *)Xh, (const half_t *)Xl, (const bf16_t *)w_s, b_s, blocks, cand_blocks, scores, d);
  else
    score_kernel<float><<<n_cblk * 16, 256, 0, s>>>(X, nullptr, nullptr, (const float *)w_s, b_s, blocks, cand_blocks, scores, d);
}

// ---------------------------------------------------------------------------------------------
// Helpers of the entry point that works in a static workspace (no allocation, no copies): the bucket
// table computed on the device, plan tables delivered as kernel arguments, and the spare rows behind
// a batch cleared (whole-tile key loads may read them; they must hold finite values).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int ilog2_dev(int v) { return 31 - __builtin_clz(v); }

// Same integers as the host planner's bucket function (documented in flame_gr.h).
__global__ __launch_bounds__(256) void bucket_table_kernel(int nb, int D, int32_t *__restrict__ out) {
  const int half = nb / 2;
  const int lo = ilog2_dev(half), hi = ilog2_dev(D);
  const int octaves = hi > lo ? hi - lo : 0;
  int sub = lo;
  while (sub > 0 && octaves * (1 << sub) > half) --sub;
  for (int t = blockIdx.x * 256 + threadIdx.x; t < D; t += gridDim.x * 256) {
    int b = t;
    if (t >= half) {
      const int oct = ilog2_dev(t);
      b = half + (oct - lo) * (1 << sub) + ((t - (1 << oct)) >> (oct - sub));
    }
    out[t] = b;
  }
}

void launch_bucket_table(int n_buckets, int D, int32_t *out, hipStream_t s) {
  const int grid = (D + 255) / 256 > 64 ? 64 : (D + 255) / 256;
  bucket_table_kernel<<<grid, 256, 0, s>>>(n_buckets, D, out);
}

__global__ __launch_bounds__(256) void upload_words_kernel(UploadWords src, int n, uint32_t *__restrict__ dst) {
  for (int i = threadIdx.x; i < n; i += 256) dst[i] = src.w[i];
}

void launch_upload_words(const void *host_src, size_t bytes, void *dst, hipStream_t s) {
  const uint32_t *src = (const uint32_t *)host_src;
  uint32_t *out = (uint32_t *)dst;
  size_t n = bytes / 4;                        // every plan table is an array of 32-bit integers
  while (n > 0) {
    UploadWords u;
    const int m = (int)(n < (size_t)UploadWords::kWords ? n : (size_t)UploadWords::kWords);
    for (int i = 0; i < m; ++i) u.w[i] = src[i];
    upload_words_kernel<<<1, 256, 0, s>>>(u, m, out);
    src += m; out += m; n -= m;
  }
}

// K plane rows [row0, row0 + n) and the same token columns of the feature-major V plane <- 0
__global__ __launch_bounds__(256) void clear_spare_kernel(half_t *__restrict__ K, half_t *__restrict__ Vt, int d, int64_t ws_rows,
                                                          int64_t row0, int n) {
  const int64_t total = (int64_t)n * d;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    K[row0 * d + i] = (half_t)0.f;
    Vt[(i / n) * ws_rows + row0 + i % n] = (half_t)0.f;
  }
}

void launch_clear_spare(void *K, void *Vt, int d, int64_t ws_rows, int64_t row0, int n, hipStream_t s) {
  if (n <= 0) return;
  const int64_t total = (int64_t)n * d;
  const int grid = (int)((total + 255) / 256 > 1024 ? 1024 : (total + 255) / 256);
  clear_spare_kernel<<<grid, 256, 0, s>>>((half_t *)K, (half_t *)Vt, d, ws_rows, row0, n);
}

// ---------------------------------------------------------------------------------------------
// Debug: the mask predicate and bucket table as the attention kernels see them.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void debug_mask_kernel(int L, int M, const int32_t *__restrict__ tab, int D,
                                                         uint8_t *__restrict__ mask, int32_t *__restrict__ bucket) {
  const int N = L + M;
  const int64_t total = (int64_t)N * N;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int r = (int)(i / N), c = (int)(i % N);
    const int is_cand = r >= L;
    const int q_index = is_cand ? L : r;
    bool ok;
    int delta;
    if (c < L) {
      ok = c < visible_history(is_cand, q_index, L);
      delta = q_index - c;
    } else {
      ok = is_cand && c == r;   // among candidate keys a candidate sees itself only
      delta = 0;
    }
    mask[i] = ok ? 1 : 0;
    if (bucket) bucket[i] = ok ? tab[delta < D ? delta : D - 1] : -1;
  }
}

void launch_debug_mask(int L, int M, const int32_t *bucket_tab, int D, uint8_t *mask, int32_t *bucket, hipStream_t s) {
  const int64_t total = (int64_t)(L + M) * (L + M);
  if (total == 0) return;
  int grid = (int)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
  debug_mask_kernel<<<grid, 256, 0, s>>>(L, M, bucket_tab, D, mask, bucket);
}

}  // namespace flame
