// Launch interface between the host API and the gfx950 kernels.  All pointers are device
// pointers unless stated; every launcher only enqueues work on `s`.
#pragma once
#include <hip/hip_runtime.h>

#include "plan.h"

namespace flame {

// Shapes every launcher needs.
struct Shape {
  int d, H, dh, n_layers, n_buckets, D;
  float eps, alpha;
  int64_t ws_rows;  // rows of every workspace matrix (plane stride = ws_rows * d)
  int softmax;      // attention weights: 0 = pointwise SiLU, 1 = softmax with a temperature per layer and head
  int latency;      // MFMA attention: 0 = throughput configuration, 1 = latency configuration (pairs of wavefronts split the keys)
};

// ---- shared small kernels (misc.hip) --------------------------------------------------------
// rows of blocks <- embeddings: fp32 X in the fp32 path, the k-tile blocked fp16 word Xh in the MFMA path (whose residual is
// the pair Xh = fp16(X), Xl = fp16(X - Xh); embeddings are exact in Xh and Xl is not written); padding rows zeroed.
// The n blocks are list[0..n) if list is given, else first..first+n.
void launch_assemble(int dtype, const RowBlock *blocks, const int32_t *list, int n, int first, const void *hist,
                     const void *cand, float *X, void *Xh, int d, hipStream_t s);
// fp16 copy of a bf16 matrix of `rows` rows of K elements (K % 8 == 0); blocked: written in the k-tile
// blocked layout of the GEMM operands (rows % 64 == 0, K % 32 == 0), else element for element
void launch_bf16_to_f16(const void *in, void *out, int64_t rows, int K, bool blocked, hipStream_t s);
// bias[lh][delta] = scale * rab[lh][bucket_tab[delta]] for all layers and heads (scale = 1/2 in the
// MFMA path, whose attention kernel works on halved logits; 1 in the fp32 path).
void launch_expand_bias(const float *rab, const int32_t *bucket_tab, float *bias, int n_lh,
                        int n_buckets, int D, float scale, hipStream_t s);
// G = (LayerNorm(O) * gamma + beta) * U, one row at a time (element type of O, U, G = dtype);
// padding rows of a block get G = 0 so that they stay finite through the layers.
void launch_ln_gate(int dtype, const void *O, const void *U, const void *gamma, const void *beta,
                    void *G, const RowBlock *blocks, const int32_t *blk_list, int n_blk, int blk_first, int d,
                    float eps, hipStream_t s);
// scores[src_row + i] = <X[row], w_s> + b_s for the valid rows of every candidate block (MFMA path: X = Xh + Xl).
void launch_scores(int dtype, const float *X, const void *Xh, const void *Xl, const void *w_s, float b_s, const RowBlock *blocks,
                   const int32_t *cand_blocks, int n_cblk, float *scores, int d, hipStream_t s);
// out[i] = factor / temperature[i] (the per-layer, per-head logit scale of the softmax attention).
void launch_logit_scale(const float *temperature, float *out, int n, float factor, hipStream_t s);
// hidden[(src_row + i) * d ..] = X[row] for the valid rows of every candidate block (fp32).
// (Xh given: the residual is the pair Xh, Xl of the MFMA path; else fp32 X)
void launch_gather_hidden(const float *X, const void *Xh, const void *Xl, const RowBlock *blocks, const int32_t *cand_blocks, int n_cblk,
                          float *hidden, int d, hipStream_t s);
// out[row][k] = Xh + Xl as fp32 for rows [row_begin, row_end) (debug capture of the MFMA path's residual)
void launch_residual_to_f32(const void *Xh, const void *Xl, float *out, int64_t row_begin, int64_t row_end, int d, hipStream_t s);
// bucket(delta) for delta in [0, D), computed on the device (the integers of plan.h's bucket_of)
void launch_bucket_table(int n_buckets, int D, int32_t *out, hipStream_t s);
// Host words -> device memory without a copy engine or staging buffer: the words travel as kernel arguments
// (UploadWords::kWords per launch; bytes % 4 == 0).  For small tables on paths that may not allocate or copy.
struct UploadWords {
  static constexpr int kWords = 960;
  uint32_t w[kWords];
};
void launch_upload_words(const void *host_src, size_t bytes, void *dst, hipStream_t s);
// rows [row0, row0 + n) of the row-major K plane and of the feature-major V plane (d features) <- 0
void launch_clear_spare(void *K, void *Vt, int d, int64_t ws_rows, int64_t row0, int n, hipStream_t s);
// mask / bucket of one request evaluated with the device predicate (debug export).
void launch_debug_mask(int L, int M, const int32_t *bucket_tab, int D, uint8_t *mask, int32_t *bucket,
                       hipStream_t s);

// ---- fp32 path (kernels_f32.hip): plain FMA kernels, correctness first ------------------------
// planes[p][row][n] = silu(X W1^T + b1), p = U,V,Q,K; rows = 64-row blocks [blk_first, blk_first+n_blk)
void launch_uvqk_f32(const float *X, const float *W1, const float *b1, float *planes, int blk_first,
                     int n_blk, const Shape &sh, hipStream_t s);
// tscale_h (softmax only): per head, the factor from the logit the kernel forms to the exponent it feeds to
// its exponential: 1 / tau here (natural exponential of the full logit).
void launch_attn_f32(const float *planes, const float *bias_lh, const float *tscale_h, float *O, const AttnItem *items,
                     int n_items, int q_tile, const Shape &sh, hipStream_t s);
// X[row] += G[row] W2^T + b2 for the rows of the listed blocks (blk_list == nullptr: contiguous)
void launch_outproj_f32(const float *G, const float *W2, const float *b2, float *X,
                        const int32_t *blk_list, int n_blk, int blk_first, const Shape &sh, hipStream_t s);

// The four activation planes of a layer (MFMA path), each [ws_rows][d] fp16 (V feature-major [d][ws_rows]).  The
// one-pass forward keeps them in one allocation; the two-stage path points v and k at the layer's cache.
struct PlanePtrs { void *u, *v, *q, *k; };

// ---- bf16-storage path (gemm_mfma.hip, attn_mfma.hip): fp16 MFMA kernels, fp32 accumulation --------
// Activations (Xh, planes, O, G) and the converted matrices W1h/W2h are fp16; biases stay bf16.
// Xh, W1h and W2h are k-tile blocked (device_common.h: blocked_index); planes, O and G are row-major.
// U, Q, K planes row-major [row][d]; the V plane is written transposed, Vt[n][row] (row stride ws_rows).
// plane_mask bit p set = compute plane p (U=1, V=2, Q=4, K=8).
void launch_uvqk_bf16(const void *Xh, const void *W1h, const void *b1, PlanePtrs planes, const int32_t *blk_list,
                      int n_blk, int blk_first, int plane_mask, const Shape &sh, hipStream_t s);
// tscale_h (softmax only): 2 log2(e) / tau per head (the kernel holds halved logits and uses the base-2 exponential).
void launch_attn_bf16(PlanePtrs planes, const float *bias_lh, const float *tscale_h, void *O, const AttnItem *items,
                      int n_items, const Shape &sh, hipStream_t s);
// Prepares the latency configuration of the attention kernel for this shape (raises its LDS limit); once per handle.
hipError_t attn_latency_setup(const Shape &sh);
// X[row] += G W2h^T + b2 on the residual pair (Xh, Xl); lo_is_zero: Xl is not read (first layer)
void launch_outproj_bf16(const void *G, const void *W2h, const void *b2, void *Xh, void *Xl, bool lo_is_zero,
                         const int32_t *blk_list, int n_blk, int blk_first, const Shape &sh, hipStream_t s);

// K3 fused (k3_mfma.hip): LayerNorm * U gate + output projection + residual in one kernel, for
// d in {128, 192, 256, 384, 512}; W2p is the fragment-major packed fp16 copy of W2 written by launch_pack_w2.
bool k3_fused_supported(int d);
void launch_pack_w2(const void *W2, void *W2p, int d, int n_layers, hipStream_t s);
// (residual pair Xh, Xl as above; lo_is_zero: Xl is not read)
void launch_k3_fused(const void *O, const void *U, const void *gamma, const void *beta, const void *W2p_layer, const void *b2,
                     void *Xh, void *Xl, bool lo_is_zero, const RowBlock *blocks, const int32_t *blk_list, int n_blk, int blk_first,
                     const Shape &sh, hipStream_t s);

constexpr int kAttnQTileBf16 = 128;  // query rows per attention work item, MFMA path
constexpr int kAttnQTileF32 = 64;    // fp32 path

}  // namespace flame
