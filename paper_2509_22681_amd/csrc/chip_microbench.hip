// Box measurements that the kernel designs argue from: what one MI355X sustains for the building blocks of the
// GR forward.  A standalone program (built by build.py next to the library, not part of it):
//     paper_2509_22681_amd/chip_microbench            prints one line per measurement
// Measurements: matrix-instruction rate with operands in registers (constant data) and read from LDS (random data);
// whether matrix and vector instructions of one SIMD overlap (same wavefront, and two wavefronts of different roles);
// issue cost of the vector instructions the attention SiLU is made of; LDS fragment-read rate with and without the
// XOR swizzle; device copy and fill rates; kernel launch latency.  Every kernel also reports the shader clock it ran
// at (cycle counter against the constant-rate wall clock), because the chip lowers its clock under matrix load.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define CK(x)                                                                      \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);        \
      exit(1);                                                                     \
    }                                                                              \
  } while (0)

constexpr int kCU = 256;

// clocks[0] += shader cycles, clocks[1] += wall ticks (100 MHz) of workgroup 0, wavefront 0
struct ClockProbe {
  long long c0, w0;
  __device__ void start() { c0 = clock64(); w0 = wall_clock64(); }
  __device__ void stop(long long *out, int probe_thread = 0) {
    if (blockIdx.x == 0 && (int)threadIdx.x == probe_thread) { out[0] = clock64() - c0; out[1] = wall_clock64() - w0; }
  }
};

// ---- matrix instructions, operands in registers -------------------------------------------------------------
__global__ __launch_bounds__(256) void mfma_reg_kernel(float *out, int iters, long long *clk) {
  ClockProbe p; p.start();
  f16x8 a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(1.0f + i); b[i] = (_Float16)(0.5f * i); }
  f32x16 acc[8];
  for (int j = 0; j < 8; ++j) for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
  for (int j = 0; j < 8; ++j) for (int e = 0; e < 16; ++e) s += acc[j][e];
  if (s == 12345.678f) out[0] = s;
  p.stop(clk);
}

// ---- matrix instructions fed from LDS (the way the GEMM and attention kernels run them) ----------------------
// per iteration and wavefront: 8 matrix instructions (4 x 2 blocks), 6 fragment reads prefetched one iteration ahead
// IDLE > 0: every wavefront sleeps 64 * IDLE cycles after each group of 8 matrix instructions (256 cycles of the pipe), which
// lowers the duty of the matrix pipe with nothing else running: how the clock answers tells how much of the chip's power is
// there whether or not the pipe works.
template <bool RANDOM, int IDLE = 0>
__global__ __launch_bounds__(256, 2) void mfma_lds_kernel(float *out, int iters, const _Float16 *src, long long *clk) {
  __shared__ __attribute__((aligned(16))) _Float16 lds[2][6 * 512 * 4];     // 2 x 24 KB
  const int tid = threadIdx.x, lane = tid & 63;
  for (int i = tid; i < 2 * 6 * 512 * 4 / 8; i += 256)
    ((f16x8 *)&lds[0][0])[i] = RANDOM ? ((const f16x8 *)src)[i] : f16x8{1, 2, 3, 4, 5, 6, 7, 8};
  __syncthreads();
  ClockProbe p; p.start();
  f16x8 f[2][6];
  for (int r = 0; r < 6; ++r) f[0][r] = *(const f16x8 *)((const char *)&lds[0][0] + lane * 16 + r * 4096 + (tid >> 6) * 1024);
  f32x16 acc[4][2];
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 2; ++j) for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  const char *base = (const char *)&lds[0][0] + lane * 16;
  for (int it = 0; it < iters; it += 2) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      __builtin_amdgcn_sched_barrier(0);
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[q][0], f[q][4], acc[0][0], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[q][1], f[q][4], acc[1][0], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int r = 0; r < 6; ++r) f[q ^ 1][r] = *(const f16x8 *)(base + ((it + q) & 1) * 24576 + r * 4096 + (tid >> 6) * 1024);
      __builtin_amdgcn_sched_barrier(0);
      acc[2][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[q][2], f[q][4], acc[2][0], 0, 0, 0);
      acc[3][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[q][3], f[q][4], acc[3][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[q][0], f[q][5], acc[0][1], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[q][1], f[q][5], acc[1][1], 0, 0, 0);
      acc[2][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[q][2], f[q][5], acc[2][1], 0, 0, 0);
      acc[3][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f[q][3], f[q][5], acc[3][1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (IDLE > 0) __builtin_amdgcn_s_sleep(IDLE);
    }
  }
  float s = 0.f;
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 2; ++j) for (int e = 0; e < 16; ++e) s += acc[i][j][e];
  if (s == 12345.678f) out[0] = s;
  p.stop(clk);
}

// ---- do matrix and vector instructions of one SIMD overlap? --------------------------------------------------
// A workgroup of 8 wavefronts, two per SIMD.  ROLES: wavefronts 0..3 run only matrix instructions, 4..7 only vector
// FMAs (bit 0: matrix wavefronts active, bit 1: vector wavefronts active).  !ROLES: every wavefront runs the two
// kinds interleaved in one instruction stream (MODE bit 0 / bit 1 select which kind is present).
template <bool ROLES>
__global__ __launch_bounds__(512) void overlap_kernel(float *out, int iters, int mode, long long *clk) {
  ClockProbe p; p.start();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const bool do_m = (mode & 1) && (!ROLES || wave < 4);
  const bool do_v = (mode & 2) && (!ROLES || wave >= 4);
  f16x8 a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(1.0f + i + threadIdx.x * 0.001f); b[i] = (_Float16)(0.5f * i); }
  f32x16 acc[4];
  for (int j = 0; j < 4; ++j) for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  float v[16];
  for (int i = 0; i < 16; ++i) v[i] = 1.0f + threadIdx.x * 1e-3f + i * 0.01f;
  // per iteration: 4 matrix instructions (4 x 32 cycles of the matrix pipe) and/or 32 vector FMAs
  if (do_m && do_v) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[j], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[(8 * j + i) & 15] = __builtin_fmaf(v[(8 * j + i) & 15], 1.0001f, 0.0001f);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
      }
    }
  } else if (do_m) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[j], 0, 0, 0);
    }
  } else if (do_v) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 32; ++i) v[i & 15] = __builtin_fmaf(v[i & 15], 1.0001f, 0.0001f);
    }
  }
  float s = 0.f;
  for (int j = 0; j < 4; ++j) for (int e = 0; e < 16; ++e) s += acc[j][e];
  for (int i = 0; i < 16; ++i) s += v[i];
  if (s == 12345.678f) out[0] = s;
  p.stop(clk, (ROLES && !(mode & 1)) ? 256 : 0);      // a wavefront that did work
}

// ---- issue cost of vector instructions -----------------------------------------------------------------------
// KIND 0 v_fma_f32, 1 v_pk_fma_f16, 2 v_exp_f32, 3 v_rcp_f32, 4 v_cvt_pk_f16_f32 (two fp32 -> packed fp16), 5 v_pk_mul_f16,
// 6 v_max3_f32, 7 v_fma_mix_f32 (fp16 x fp16 + fp32)
template <int KIND>
__global__ __launch_bounds__(256) void valu_kernel(float *out, int iters, long long *clk) {
  ClockProbe p; p.start();
  float v[16];
  f16x2 h[16];
  for (int i = 0; i < 16; ++i) { v[i] = 1.0f + threadIdx.x * 1e-3f + i * 0.01f; h[i] = f16x2{(_Float16)v[i], (_Float16)(0.5f * v[i])}; }
  const f16x2 c1 = {(_Float16)0.999f, (_Float16)1.001f}, c2 = {(_Float16)0.001f, (_Float16)-0.001f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      const int r = i & 15;
      if (KIND == 0) v[r] = __builtin_fmaf(v[r], 1.0001f, 0.0001f);
      else if (KIND == 1) h[r] = __builtin_elementwise_fma(h[r], c1, c2);
      else if (KIND == 2) v[r] = __builtin_amdgcn_exp2f(v[r]);
      else if (KIND == 3) v[r] = __builtin_amdgcn_rcpf(v[r]);
      else if (KIND == 4) asm volatile("v_cvt_pk_f16_f32 %0, %1, %2" : "=v"(h[r]) : "v"(v[r]), "v"(v[(r + 1) & 15]));
      else if (KIND == 5) h[r] = h[r] * c1;
      else if (KIND == 6) asm volatile("v_max3_f32 %0, %1, %2, %3" : "=v"(v[r]) : "v"(v[r]), "v"(v[(r + 1) & 15]), "v"(v[(r + 2) & 15]));
      else asm volatile("v_fma_mix_f32 %0, %1, %2, %0 op_sel_hi:[1,1,0]" : "+v"(v[r]) : "v"(h[r]), "v"(h[(r + 1) & 15]));
    }
  }
  float s = 0.f;
  for (int i = 0; i < 16; ++i) s += v[i] + (float)h[i][0] + (float)h[i][1];
  if (s == 12345.678f) out[0] = s;
  p.stop(clk);
}

// ---- LDS fragment reads: 16-byte reads of 32 rows x 2 chunk columns, rows of 64 bytes ----------------------------
// ORDER 0: unswizzled; 1: the swizzle, rows in lane order; 2: the same swizzle with the rows in the order in which the
// projection kernel's second operand is read (lane m reads row 16 bit2(m) + 4 (m / 8) + m % 4); 3: another key.
template <int ORDER>
__global__ __launch_bounds__(256, 2) void lds_kernel(float *out, int iters, long long *clk) {
  __shared__ __attribute__((aligned(16))) char lds[65536];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 65536 / 16; i += 256) ((f16x8 *)lds)[i] = f16x8{1, 2, 3, 4, 5, 6, 7, 8};
  __syncthreads();
  ClockProbe p; p.start();
  const int m = lane & 31, c = lane >> 5;
  const int row = ORDER == 2 ? (((m & 4) << 2) | ((m >> 3) << 2) | (m & 3)) : m;
  // 64-byte rows, four to a 256-byte group; swizzled: chunk index XOR row bits 2 and 3 (ORDER 3: bit 3 XOR bit 4 instead
  // of bit 3, which is free of conflicts if 16 consecutive lanes are served per clock, and is not on this chip)
  const int key = ORDER == 3 ? ((row >> 2) & 1) | ((((row >> 3) ^ (row >> 4)) & 1) << 1) : (row >> 2) & 3;
  const int off = ORDER ? (row >> 2) * 256 + ((((row & 3) << 2) | (c ^ key)) << 4) : row * 64 + c * 16;
  // LDS addresses are the low 32 bits of the generic pointer
  const uint32_t a0 = (uint32_t)(uintptr_t)(lds + wave * 16384 + off);
  f16x8 r[8];
  for (int i = 0; i < 8; ++i) r[i] = f16x8{0, 0, 0, 0, 0, 0, 0, 0};
  for (int it = 0; it < iters; ++it) {
    asm volatile("ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:2048\n ds_read_b128 %2, %8 offset:4096\n ds_read_b128 %3, %8 offset:6144\n"
                 "ds_read_b128 %4, %8 offset:8192\n ds_read_b128 %5, %8 offset:10240\n ds_read_b128 %6, %8 offset:12288\n ds_read_b128 %7, %8 offset:14336\n"
                 "s_waitcnt lgkmcnt(0)"
                 : "=v"(r[0]), "=v"(r[1]), "=v"(r[2]), "=v"(r[3]), "=v"(r[4]), "=v"(r[5]), "=v"(r[6]), "=v"(r[7]) : "v"(a0));
  }
  f16x8 acc = r[0] + r[1] + r[2] + r[3] + r[4] + r[5] + r[6] + r[7];
  float s = 0.f;
  for (int i = 0; i < 8; ++i) s += (float)acc[i];
  if (s == 12345.678f) out[0] = s;
  p.stop(clk);
}

// ---- HBM --------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void copy_kernel(const uint4 *__restrict__ in, uint4 *__restrict__ outp, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) outp[i] = in[i];
}
__global__ __launch_bounds__(256) void fill_kernel(uint4 *__restrict__ outp, size_t n16) {
  const uint4 v = {1, 2, 3, 4};
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) outp[i] = v;
}
__global__ void empty_kernel() {}

template <typename F>
static float time_ms(F f, int reps = 3) {
  hipEvent_t a, b;
  CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  f(); CK(hipDeviceSynchronize());
  float best = 1e30f;
  for (int r = 0; r < reps; ++r) {
    CK(hipEventRecord(a)); f(); CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
    float ms; CK(hipEventElapsedTime(&ms, a, b));
    if (ms < best) best = ms;
  }
  CK(hipEventDestroy(a)); CK(hipEventDestroy(b));
  return best;
}

static double g_wall_khz = 100000.0;   // rate of wall_clock64()
static double shader_ghz(long long *dclk) {
  long long h[2];
  CK(hipMemcpy(h, dclk, sizeof(h), hipMemcpyDeviceToHost));
  return h[1] > 0 ? (double)h[0] / ((double)h[1] / g_wall_khz * 1e6) : 0.0;
}

int main() {
  hipDeviceProp_t prop;
  CK(hipGetDeviceProperties(&prop, 0));
  {
    int khz = 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, 0) == hipSuccess && khz > 0) g_wall_khz = khz;
  }
  printf("device: %s, %d CUs, clock %d kHz, wall clock %.0f kHz\n", prop.gcnArchName, prop.multiProcessorCount, prop.clockRate, g_wall_khz);
  float *o; CK(hipMalloc(&o, 64));
  long long *clk; CK(hipMalloc(&clk, 16)); CK(hipMemset(clk, 0, 16));
  const int iters = 20000;

  for (int occ : {1, 2}) {
    const float ms = time_ms([&] { mfma_reg_kernel<<<kCU * occ, 256>>>(o, iters, clk); });
    const double fl = (double)kCU * occ * 4 * iters * 8 * 32768.0;
    printf("mfma_f32_32x32x16_f16, register operands, constant data, %d wavefront(s) per SIMD: %.1f TFLOP/s at %.2f GHz\n", occ,
           fl / ms * 1e-9, shader_ghz(clk));
  }
  {
    _Float16 *src; CK(hipMalloc(&src, 49152));
    std::vector<_Float16> hsrc(24576);
    srand(1);
    for (auto &x : hsrc) x = (_Float16)((rand() % 2001 - 1000) * 0.001f);
    CK(hipMemcpy(src, hsrc.data(), 49152, hipMemcpyHostToDevice));
    for (int rnd = 0; rnd < 2; ++rnd) {
      const float ms = rnd ? time_ms([&] { mfma_lds_kernel<true><<<kCU * 2, 256>>>(o, iters, src, clk); })
                           : time_ms([&] { mfma_lds_kernel<false><<<kCU * 2, 256>>>(o, iters, src, clk); });
      const double fl = (double)kCU * 2 * 4 * iters * 8 * 32768.0;
      printf("mfma fed by 6 LDS fragment reads per 8 instructions, %s data, 2 wavefronts per SIMD: %.1f TFLOP/s at %.2f GHz\n",
             rnd ? "random" : "constant", fl / ms * 1e-9, shader_ghz(clk));
    }
    // the same random-data stream at reduced duty of the matrix pipe
    {
      const int it2 = iters / 4;
      const double fl = (double)kCU * 2 * 4 * it2 * 8 * 32768.0;
      const float m1 = time_ms([&] { mfma_lds_kernel<true, 4><<<kCU * 2, 256>>>(o, it2, src, clk); });
      const double g1 = shader_ghz(clk);
      const float m2 = time_ms([&] { mfma_lds_kernel<true, 12><<<kCU * 2, 256>>>(o, it2, src, clk); });
      const double g2 = shader_ghz(clk);
      const float m3 = time_ms([&] { mfma_lds_kernel<true, 28><<<kCU * 2, 256>>>(o, it2, src, clk); });
      const double g3 = shader_ghz(clk);
      // duty = matrix cycles / all cycles of a SIMD = flop / (1024 SIMDs x 1024 flop per cycle x cycles)
      auto duty = [&](float ms, double ghz) { return fl / (1024.0 * 1024.0 * ms * 1e-3 * ghz * 1e9); };
      printf("random data, wavefronts sleeping 256 / 768 / 1792 cycles per 8 instructions: %.1f TFLOP/s at %.2f GHz (pipe duty %.2f), "
             "%.1f at %.2f GHz (%.2f), %.1f at %.2f GHz (%.2f)\n",
             fl / m1 * 1e-9, g1, duty(m1, g1), fl / m2 * 1e-9, g2, duty(m2, g2), fl / m3 * 1e-9, g3, duty(m3, g3));
    }
    CK(hipFree(src));
  }
  {
    float t[4];
    double g[4];
    for (int mode = 1; mode <= 3; ++mode) {
      t[mode] = time_ms([&] { overlap_kernel<true><<<kCU, 512>>>(o, iters, mode, clk); });
      g[mode] = shader_ghz(clk);
    }
    printf("two wavefronts per SIMD with separate roles (per iteration 4 mfma | 32 v_fma_f32): mfma alone %.3f ms (%.2f GHz), "
           "valu alone %.3f ms (%.2f GHz), both %.3f ms (%.2f GHz); sum %.3f, max %.3f\n",
           t[1], g[1], t[2], g[2], t[3], g[3], t[1] + t[2], t[1] > t[2] ? t[1] : t[2]);
    for (int mode = 1; mode <= 3; ++mode) {
      t[mode] = time_ms([&] { overlap_kernel<false><<<kCU, 512>>>(o, iters, mode, clk); });
      g[mode] = shader_ghz(clk);
    }
    printf("two wavefronts per SIMD, each interleaving 1 mfma : 8 v_fma_f32: mfma alone %.3f ms (%.2f GHz), valu alone %.3f ms "
           "(%.2f GHz), both %.3f ms (%.2f GHz); sum %.3f, max %.3f\n",
           t[1], g[1], t[2], g[2], t[3], g[3], t[1] + t[2], t[1] > t[2] ? t[1] : t[2]);
  }
  {
    const char *names[] = {"v_fma_f32", "v_pk_fma_f16", "v_exp_f32", "v_rcp_f32", "v_cvt_pk_f16_f32", "v_pk_mul_f16", "v_max3_f32",
                           "v_fma_mix_f32"};
    for (int kind = 0; kind < 8; ++kind) {
      printf("%s, cycles per wavefront instruction per SIMD at 1, 2, 3, 4 wavefronts per SIMD:", names[kind]);
      for (int occ = 1; occ <= 4; ++occ) {
        float ms = 0.f;
        const int grid = kCU * occ;
        switch (kind) {
          case 0: ms = time_ms([&] { valu_kernel<0><<<grid, 256>>>(o, iters, clk); }); break;
          case 1: ms = time_ms([&] { valu_kernel<1><<<grid, 256>>>(o, iters, clk); }); break;
          case 2: ms = time_ms([&] { valu_kernel<2><<<grid, 256>>>(o, iters, clk); }); break;
          case 3: ms = time_ms([&] { valu_kernel<3><<<grid, 256>>>(o, iters, clk); }); break;
          case 4: ms = time_ms([&] { valu_kernel<4><<<grid, 256>>>(o, iters, clk); }); break;
          case 5: ms = time_ms([&] { valu_kernel<5><<<grid, 256>>>(o, iters, clk); }); break;
          case 6: ms = time_ms([&] { valu_kernel<6><<<grid, 256>>>(o, iters, clk); }); break;
          default: ms = time_ms([&] { valu_kernel<7><<<grid, 256>>>(o, iters, clk); }); break;
        }
        const double ghz = shader_ghz(clk);
        printf(" %.2f", ms * 1e-3 * ghz * 1e9 / ((double)iters * 32 * occ));
      }
      printf("\n");
    }
  }
  for (int sw = 0; sw < 4; ++sw) {
    const int it2 = 20000;
    const float ms = sw == 3 ? time_ms([&] { lds_kernel<3><<<kCU * 2, 256>>>(o, it2, clk); })
                     : sw == 2 ? time_ms([&] { lds_kernel<2><<<kCU * 2, 256>>>(o, it2, clk); })
                     : sw    ? time_ms([&] { lds_kernel<1><<<kCU * 2, 256>>>(o, it2, clk); })
                             : time_ms([&] { lds_kernel<0><<<kCU * 2, 256>>>(o, it2, clk); });
    const double ghz = shader_ghz(clk);
    const double bytes = (double)kCU * 2 * 256 * 16 * 8 * it2;
    printf("ds_read_b128 of 64-byte rows, %s: %.1f bytes per cycle per CU at %.2f GHz\n", sw == 3 ? "XOR-swizzled with row bit 3 ^ bit 4 in the key" : sw == 2 ? "XOR-swizzled, rows in the permuted order of the projection kernel's second operand" : sw ? "XOR-swizzled" : "unswizzled",
           bytes / (ms * 1e-3 * ghz * 1e9) / kCU, ghz);
  }
  {
    const size_t bytes = (size_t)1 << 30;
    uint4 *a, *b;
    CK(hipMalloc(&a, bytes)); CK(hipMalloc(&b, bytes));
    CK(hipMemset(a, 1, bytes));
    const float tc = time_ms([&] { copy_kernel<<<2048, 256>>>(a, b, bytes / 16); });
    const float tf = time_ms([&] { fill_kernel<<<2048, 256>>>(b, bytes / 16); });
    printf("device copy of 1 GiB: %.3f ms, %.0f GB/s read + written; fill of 1 GiB: %.3f ms, %.0f GB/s\n", tc, 2.0 * bytes / tc * 1e-6,
           tf, bytes / tf * 1e-6);
    CK(hipFree(a)); CK(hipFree(b));
  }
  {
    const float ms = time_ms([&] { for (int i = 0; i < 1000; ++i) empty_kernel<<<1, 64>>>(); });
    printf("empty kernel, 1000 launches back to back: %.2f us per launch\n", ms);
  }
  return 0;
}
