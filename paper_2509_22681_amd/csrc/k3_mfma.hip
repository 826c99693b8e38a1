// K3 of the GR block, fused: X <- X + (LayerNorm_d(O) * U) W2^T + b2.
//
// The residual stream X lives in HBM as two fp16 words per element: Xh = fp16(X), the k-tile blocked operand copy that the
// next layer's projection reads anyway, and Xl = fp16(X - Xh) (row-major), together 22 significant bits, so that
// this kernel reads 4 and writes 4 bytes per element instead of reading 4 and writing 6 (fp32 X plus the operand copy).
//
// LayerNorm, the U gate, the output projection and the residual run in one kernel (the fusion of
// layer normalisation with the following linear projection that Section 3.2 describes), so the
// gated activations never travel through HBM.  The kernel is HBM-bound by construction (per row it
// must read O and U and read-modify-write X: 12 bytes per element against 2*d flops), so the
// design aims at streaming, not at MFMA utilisation:
//   * one workgroup = one 64-row block of the workspace, all d output features (d <= 512 per pass);
//   * phase 1: each wavefront normalises 16 rows (one row per wavefront-wide 16-byte load, statistics
//     by wavefront reduction in fp32: mean, then centred second moment) and writes the gated fp16 rows
//     into LDS, 16-byte chunks XOR-swizzled with the row's low four bits so that the MFMA operand reads are
//     conflict free (the LDS serves 16 lanes x 16 bytes per clock from 64 banks);
//   * phase 2: each wavefront owns d/4 output features; the W2 operand comes straight from L2 in a
//     fragment-major packed layout (one coalesced 1 KB read per MFMA operand, prepared once per forward
//     by pack_w2_kernel), so LDS holds only the activations and two workgroups fit on a CU;
//   * phase 3: residual add in fp32 (X = Xh + Xl, exact in fp32) and split into the two fp16 words again, after a
//     transposition of the accumulators through LDS so that the residual is read and written in whole lines.
#include "device_common.h"
#include "kernels.h"

namespace flame {

namespace {

// W2p[ks][cb][lane][0..7] = W2[32*cb + lane%32][16*ks + 8*(lane/32) + 0..7]  (bf16 -> fp16)
__global__ __launch_bounds__(256) void pack_w2_kernel(const bf16_t *__restrict__ W2, half_t *__restrict__ W2p, int d, int n_layers) {
  const int64_t per_layer = (int64_t)d * d / 8;            // 16-byte chunks
  const int64_t total = per_layer * n_layers;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t l = i / per_layer, c = i % per_layer;
    const int lane = (int)(c & 63);
    const int64_t t = c >> 6;
    const int cb = (int)(t % (d / 32)), ks = (int)(t / (d / 32));
    const bf16x8 v = *(const bf16x8 *)(W2 + l * d * d + (int64_t)(32 * cb + (lane & 31)) * d + 16 * ks + 8 * (lane >> 5));
    f16x8 o;
#pragma unroll
    for (int k = 0; k < 8; ++k) o[k] = to_f16_sat((float)v[k]);
    *(f16x8 *)(W2p + (l * per_layer + c) * 8) = o;
  }
}

// NWV wavefronts per workgroup, NBW 32-feature blocks per wavefront: d = 32 * NBW * NWV (four wavefronts for
// d = 128, 256, 512; three for d = 96, 192, 384).  The 64 rows of the block are dealt out RPW per wavefront in
// phase 1 (with three wavefronts the last one has rows to spare, which it skips).
// CS workgroups share a row block (blockIdx.y): each repeats phase 1 and takes 1/CS of every wavefront's feature
// blocks through phases 2 and 3.  CS = 2 is for launches with few row blocks, where a workgroup sits alone on its
// CU and its run time, not the chip's bandwidth, is what counts; every output element is computed exactly as with
// CS = 1.
template <int NWV, int NBW, int CS>
__global__ __launch_bounds__(64 * NWV, 2) void k3_fused_kernel(const half_t *__restrict__ O, const half_t *__restrict__ U,
                                                          const bf16_t *__restrict__ gamma, const bf16_t *__restrict__ beta,
                                                          const half_t *__restrict__ W2p, const bf16_t *__restrict__ b2,
                                                          half_t *__restrict__ Xh, half_t *__restrict__ Xl, int lo_is_zero,
                                                          const RowBlock *__restrict__ blocks, const int32_t *__restrict__ blk_list,
                                                          int blk_first, float eps) {
  constexpr int d = 32 * NBW * NWV;
  constexpr int RB4 = 4;                         // rows per batch of phase 1
  constexpr int RPW = (kRowAlign + NWV * RB4 - 1) / (NWV * RB4) * RB4;   // rows per wavefront in phase 1 (16, or 24 of which 64 exist)
  constexpr bool EVEN = RPW * NWV == kRowAlign;
  constexpr int NCHUNK = d / 8;                  // 16-byte chunks per row
  // Swizzle key of the gated rows in LDS.  A row of d fp16 is NCHUNK chunks; the MFMA operand reads take one chunk
  // column of 16 consecutive rows.  With NCHUNK a multiple of 16 the row pitch is a multiple of 256 bytes and the
  // low four row bits spread those reads over the 16 slots; with NCHUNK = 24 (d = 192, pitch 384 bytes: odd and
  // even rows already sit 128 bytes apart) three bits of row / 2 do, and the XOR stays inside a group of 8 chunks.
  auto gkey = [](int r) { return NCHUNK % 16 == 0 ? r & 15 : (r >> 1) & 7; };
  constexpr int CPL = (NCHUNK + 63) / 64;        // chunks per lane in phase 1
  extern __shared__ __attribute__((aligned(16))) char smem[];   // sG: 64 rows x d fp16, swizzled

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lhalf = lane >> 5;
  const int blk = blk_list ? blk_list[blockIdx.x] : blk_first + blockIdx.x;
  const int n_valid = blocks[blk].n_valid;
  const int64_t row0 = (int64_t)blk * kRowAlign;

  // ---- phase 1: G = (LN(O) * gamma + beta) * U -> LDS
  float g[CPL][8], bt[CPL][8];
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const int ch = lane + 64 * c;
    if (ch < NCHUNK) {
      const bf16x8 gv = *(const bf16x8 *)(gamma + ch * 8), bv = *(const bf16x8 *)(beta + ch * 8);
#pragma unroll
      for (int k = 0; k < 8; ++k) { g[c][k] = (float)gv[k]; bt[c][k] = (float)bv[k]; }
    }
  }
  // Rows are taken four at a time, and the loads of the next four are issued before the current
  // four are normalised: with one row in flight per wavefront the kernel would run at the latency,
  // not the bandwidth, of HBM.
  f16x8 ov[2][RB4][CPL], uv[2][RB4][CPL];
  auto issue = [&](int set, int batch) {
#pragma unroll
    for (int q = 0; q < RB4; ++q)
#pragma unroll
      for (int c = 0; c < CPL; ++c) {
        const int ch = lane + 64 * c;
        if (ch < NCHUNK) {
          const int rr = wave * RPW + batch * RB4 + q;
          const int64_t off = (row0 + (EVEN || rr < kRowAlign ? rr : kRowAlign - 1)) * d + ch * 8;
          ov[set][q][c] = __builtin_nontemporal_load((const f16x8 *)(O + off));
          uv[set][q][c] = __builtin_nontemporal_load((const f16x8 *)(U + off));
        }
      }
  };
  issue(0, 0);
#pragma unroll
  for (int batch = 0; batch < RPW / RB4; ++batch) {
    const int set = batch & 1;
    if (batch + 1 < RPW / RB4) issue(set ^ 1, batch + 1);
    __builtin_amdgcn_sched_barrier(0);
    // the four rows go through each step together, so that their reduction chains overlap
    float v[RB4][CPL][8], mu[RB4], rstd[RB4];
#pragma unroll
    for (int q = 0; q < RB4; ++q) {
      float sum = 0.f;
#pragma unroll
      for (int c = 0; c < CPL; ++c)
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          v[q][c][k] = lane + 64 * c < NCHUNK ? (float)ov[set][q][c][k] : 0.f;
          sum += v[q][c][k];
        }
      mu[q] = sum;
    }
#pragma unroll
    for (int q = 0; q < RB4; ++q) mu[q] = wave_sum(mu[q]) * (1.0f / d);
#pragma unroll
    for (int q = 0; q < RB4; ++q) {
      float sq = 0.f;
#pragma unroll
      for (int c = 0; c < CPL; ++c)
        if (lane + 64 * c < NCHUNK) {
#pragma unroll
          for (int k = 0; k < 8; ++k) { const float t = v[q][c][k] - mu[q]; sq += t * t; }
        }
      rstd[q] = sq;
    }
#pragma unroll
    for (int q = 0; q < RB4; ++q) rstd[q] = rsqrtf(wave_sum(rstd[q]) * (1.0f / d) + eps);
#pragma unroll
    for (int q = 0; q < RB4; ++q) {
      const int r = wave * RPW + batch * RB4 + q;
      if (!EVEN && r >= kRowAlign) continue;       // a spare row of the last wavefront
      const bool pad = r >= n_valid;               // padding rows carry a zero branch so that they stay finite
#pragma unroll
      for (int c = 0; c < CPL; ++c) {
        const int ch = lane + 64 * c;
        if (ch < NCHUNK) {
          f16x8 o;
#pragma unroll
          for (int k = 0; k < 8; ++k)
            o[k] = pad ? (half_t)0.f : to_f16_sat(((v[q][c][k] - mu[q]) * rstd[q] * g[c][k] + bt[c][k]) * (float)uv[set][q][c][k]);
          *(f16x8 *)(smem + r * (d * 2) + ((ch ^ gkey(r)) << 4)) = o;
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  __syncthreads();

  // ---- phase 2: acc[token][feature] over k; features of this wavefront: wave*32*NBW .. +32*NBW-1
  static_assert(NBW % CS == 0, "feature blocks of a wavefront divide among the workgroups of a row block");
  constexpr int NB2 = NBW / CS;                  // feature blocks per wavefront in this workgroup
  const int fb0 = wave * NBW + (CS > 1 ? (int)blockIdx.y * NB2 : 0);   // first of them
  f32x16 acc[2][NB2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < NB2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  constexpr int NKS = d / 16;
  // The W2 fragments come from L2, whose latency is several times the 8 MFMAs of a k-step: they are requested
  // PD - 1 k-steps ahead into a register ring (scheduling barriers keep the compiler from sinking the requests
  // back to their first use); the activations come from LDS, one step ahead.
  constexpr int PD = 4;
  static_assert(NKS % PD == 0, "k-steps are walked in groups of the ring depth");
  const half_t *wp = W2p + ((int64_t)fb0 * 64 + lane) * 8;      // + (ks * (d/32) + j) * 512
  f16x8 fw[PD][NB2], fa[2][2];
#pragma unroll
  for (int p = 0; p < PD - 1; ++p)
#pragma unroll
    for (int j = 0; j < NB2; ++j) fw[p][j] = *(const f16x8 *)(wp + ((int64_t)p * (d / 32) + j) * 512);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = 32 * i + l32;
    fa[0][i] = *(const f16x8 *)(smem + r * (d * 2) + ((lhalf ^ gkey(r)) << 4));
  }
  __builtin_amdgcn_sched_barrier(0);
  for (int ks0 = 0; ks0 < NKS; ks0 += PD) {
#pragma unroll
    for (int u = 0; u < PD; ++u) {
      const int ks = ks0 + u;
      const int cur = u & 1, nxt = cur ^ 1;
      const int kw = ks + PD - 1 < NKS ? ks + PD - 1 : NKS - 1;
      const int kn = ks + 1 < NKS ? ks + 1 : ks;
#pragma unroll
      for (int j = 0; j < NB2; ++j) fw[(u + PD - 1) % PD][j] = *(const f16x8 *)(wp + ((int64_t)kw * (d / 32) + j) * 512);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int r = 32 * i + l32;
        fa[nxt][i] = *(const f16x8 *)(smem + r * (d * 2) + (((2 * kn + lhalf) ^ gkey(r)) << 4));
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NB2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw[u][j], fa[cur][i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- phase 3: residual.  In the accumulators a lane holds one token and scattered features, and only
  // two lanes share a row, so direct X accesses would be 32-byte pieces (the memory path is bound by the
  // number of requests, not only by bytes).  Each wavefront passes its 32 x (32 NBW) patch through a
  // private slice of the now free LDS (16-byte chunks XOR-swizzled by row) and then walks it row by
  // row: 16 bytes per lane, whole lines of X, 64-byte runs of the blocked fp16 copy.
  __syncthreads();                                  // every wavefront has finished reading G
  constexpr int WF = 32 * NB2;                      // features per wavefront (in this workgroup)
  constexpr int CPR = WF / 4;                       // 16-byte fp32 chunks per patch row
  constexpr int RPI = 64 / CPR;                     // patch rows per instruction
  constexpr int NIT = 32 / RPI;
  char *pb = smem + wave * (32 * WF * 4);
  // chunk XOR key: 16 consecutive rows of one chunk column use each of the 16 slots of 256 bytes once
  auto pkey = [](int row) { return CPR == 8 ? (row >> 1) & 7 : row & 15; };
  const int rl = lane / CPR, cc = lane % CPR;
  const int n = fb0 * 32 + 4 * cc;                  // this lane's 4 features in the read-out
  f32x4 bvf;
  {
    const bf16x4 bv = *(const bf16x4 *)(b2 + n);
#pragma unroll
    for (int q = 0; q < 4; ++q) bvf[q] = (float)bv[q];
  }
  constexpr int XB = NIT < 8 ? NIT : 8;             // residual rows requested ahead
  // lo_is_zero: the first layer, whose input rows are embeddings (exact in Xh): Xl is not read, only written
  f16x4 xh[XB], xl[XB];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int64_t m0 = row0 + 32 * i + rl;
    auto load = [&](int t, int it) {
      const int64_t m = m0 + (int64_t)it * RPI;
      xh[t] = __builtin_nontemporal_load((const f16x4 *)(Xh + blocked_index(m, n, d)));
      xl[t] = f16x4{(half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f};
      if (!lo_is_zero) xl[t] = __builtin_nontemporal_load((const f16x4 *)(Xl + m * d + n));
    };
#pragma unroll
    for (int t = 0; t < XB; ++t) load(t, t);
#pragma unroll
    for (int j = 0; j < NB2; ++j)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        const int c = 8 * j + 2 * gq + lhalf;
        const f32x4 v = {acc[i][j][4 * gq], acc[i][j][4 * gq + 1], acc[i][j][4 * gq + 2], acc[i][j][4 * gq + 3]};
        *(f32x4 *)(pb + l32 * (WF * 4) + ((c ^ pkey(l32)) << 4)) = v;
      }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int row = it * RPI + rl;
      const f32x4 v = *(const f32x4 *)(pb + row * (WF * 4) + ((cc ^ pkey(row)) << 4));
      const f16x4 h4 = xh[it % XB], l4 = xl[it % XB];
      if (it + XB < NIT) load(it % XB, it + XB);
      f16x4 oh, ol;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float x = ((float)h4[q] + (float)l4[q]) + (v[q] + bvf[q]);
        oh[q] = to_f16_sat(x);
        ol[q] = to_f16_sat(x - (float)oh[q]);
      }
      const int64_t m = row0 + 32 * i + row;
      __builtin_nontemporal_store(oh, (f16x4 *)(Xh + blocked_index(m, n, d)));
      __builtin_nontemporal_store(ol, (f16x4 *)(Xl + m * d + n));
    }
  }
}

}  // namespace

bool k3_fused_supported(int d) { return d == 128 || d == 192 || d == 256 || d == 384 || d == 512; }

void launch_pack_w2(const void *W2, void *W2p, int d, int n_layers, hipStream_t s) {
  const int64_t total = (int64_t)d * d / 8 * n_layers;
  int grid = (int)((total + 255) / 256 > 2048 ? 2048 : (total + 255) / 256);
  pack_w2_kernel<<<grid, 256, 0, s>>>((const bf16_t *)W2, (half_t *)W2p, d, n_layers);
}

void launch_k3_fused(const void *O, const void *U, const void *gamma, const void *beta, const void *W2p_layer, const void *b2,
                     void *Xh, void *Xl, bool lo_is_zero, const RowBlock *blocks, const int32_t *blk_list, int n_blk, int blk_first,
                     const Shape &sh, hipStream_t s) {
  if (n_blk <= 0) return;
  const size_t lds = (size_t)kRowAlign * sh.d * 2;
  // few row blocks: two workgroups per block (see the kernel), as long as the launch still fits the chip once over
  const bool split = n_blk <= 128;
#define K3_CASE(NWV, NB, CSV) k3_fused_kernel<NWV, NB, CSV><<<dim3(n_blk, CSV), 64 * NWV, lds, s>>>((const half_t *)O, (const half_t *)U, (const bf16_t *)gamma, (const bf16_t *)beta, \
    (const half_t *)W2p_layer, (const bf16_t *)b2, (half_t *)Xh, (half_t *)Xl, lo_is_zero ? 1 : 0, blocks, blk_list, blk_first, sh.eps)
  const bool split4 = n_blk <= 64;
  if (sh.d == 512) { if (split4) K3_CASE(4, 4, 4); else if (split) K3_CASE(4, 4, 2); else K3_CASE(4, 4, 1); }
  else if (sh.d == 384) { if (split4) K3_CASE(3, 4, 4); else if (split) K3_CASE(3, 4, 2); else K3_CASE(3, 4, 1); }
  else if (sh.d == 256) { if (split) K3_CASE(4, 2, 2); else K3_CASE(4, 2, 1); }
  else if (sh.d == 192) { if (split) K3_CASE(3, 2, 2); else K3_CASE(3, 2, 1); }
  else K3_CASE(4, 1, 1);
#undef K3_CASE
}

}  // namespace flame
