// Device-side helpers shared by the gfx950 kernels of the GR forward.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace flame {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 half_t;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
__device__ __forceinline__ float to_f32(half_t v) { return (float)v; }

// fp16 storage of an fp32 value: round to nearest even, saturating at the largest finite fp16 so
// that an out-of-range activation degrades gracefully instead of turning into inf (and then NaN).
__device__ __forceinline__ half_t to_f16_sat(float v) {
  return (half_t)__builtin_fminf(__builtin_fmaxf(v, -65504.f), 65504.f);
}

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }  // round to nearest even
template <> __device__ __forceinline__ half_t from_f32<half_t>(float v) { return to_f16_sat(v); }

// silu(x) = x / (1 + exp(-x)).  exp2 of a large positive argument gives +inf and the quotient 0,
// of a large negative one gives 0 and the quotient x: both limits are the right ones.
__device__ __forceinline__ float silu_f32(float x) {
  return x / (1.0f + __expf(-x));
}

// Faster variant: hardware exp2 and reciprocal (about 1 ulp each), same limits.
__device__ __forceinline__ float silu_fast(float x) {
  float e = __builtin_amdgcn_exp2f(x * -1.4426950408889634f);
  return x * __builtin_amdgcn_rcpf(1.0f + e);
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// SiLU of an argument that arrives halved: returns silu(x) for s = x / 2.  The attention kernel keeps
// its logits in this form (the factor 1/2 is folded into Q and into the bias table, both exactly):
// silu(x) = x/2 + x^2 r(x^2) then starts from the logit itself, see the polynomial route there.
__device__ __forceinline__ float silu_half_domain(float s) {
  // x / (1 + e^-x) = s / (1/2 + 2^(-2 log2(e) s - 1)): fma, exp2, add, rcp, mul
  return s * __builtin_amdgcn_rcpf(0.5f + __builtin_amdgcn_exp2f(__builtin_fmaf(s, -2.0f * kLog2e, -1.0f)));
}

// SiLU for small arguments.  silu(x) - x/2 is even: silu(x) = x/2 + x^2 r(x^2) with r(u) ~ a1 + a3 u + a5 u^2 (weighted
// least-squares fit of (silu(x) - x/2) / x^2 on [-2, 2]; approximation error below 5.3e-4 at |x| = 2, below 1e-4 for
// |x| <= 1.5 and below 1e-5 for |x| <= 1).
constexpr float kPolyA1 = 0.24916259f, kPolyA3 = -0.01916112f, kPolyA5 = 0.00112581f;

// max(|a|, |b|, |c|) and max(a, b, c) in one instruction each (absolute values are operand modifiers)
__device__ __forceinline__ float max3_abs_f32(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, |%1|, |%2|, |%3|" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}
__device__ __forceinline__ float max3_f32(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}

// "k-tile blocked" layout of the fp16 GEMM operands (the activation copy Xh and the converted weight
// matrices): inside every block of 64 rows the 32-wide k slices follow one another,
// [row / 64][k / 32][row % 64][k % 32], so the 64 rows x 32 k slice a GEMM k-tile needs is 4 KB of
// contiguous memory and is fetched as whole 128-byte lines.  (Row-major rows of d elements would hand
// the L1 two 64-byte requests per line, and the number of requests in flight is what bounds it.)
__device__ __forceinline__ int64_t blocked_index(int64_t row, int k, int K) {
  return (row >> 6) * 64 * K + (int64_t)(k >> 5) * 2048 + (row & 63) * 32 + (k & 31);
}

// Number of history keys a query row may look at (the mask of the single-user-multiple-items
// scoring pass): a history row at index q sees keys 0..q, a candidate row sees all L.
__device__ __forceinline__ int visible_history(int is_cand, int q_index, int L) {
  return is_cand ? L : q_index + 1;
}

// Sum over the 64 lanes, delivered to every lane: the butterfly v += v[lane ^ o] for o = 32, 16, 8, 4, 2, 1,
// without the LDS crossbar.  The two widest steps use the half- and row-swap instructions of gfx950 (each
// returns both halves of the exchange, whose sum is the butterfly step in either half); the others are DPP
// operands of the add.  After the step for o, lanes that differ only in bits >= o hold equal values, so a row
// rotation by 4 (resp. 2) reaches a lane that holds exactly what lane ^ 4 (resp. lane ^ 2) holds: every lane
// gets the bits the plain butterfly would give.
__device__ __forceinline__ float wave_sum(float v) {
  {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  }
  {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  }
  v += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x128, 0xf, 0xf, false));  // row_ror:8
  v += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x124, 0xf, 0xf, false));  // row_ror:4
  v += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x4e, 0xf, 0xf, false));   // quad_perm 2,3,0,1
  v += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0xb1, 0xf, 0xf, false));   // quad_perm 1,0,3,2
  return v;
}

// Maximum over the 64 lanes, delivered to every lane (same exchange pattern as wave_sum).
__device__ __forceinline__ float wave_max(float v) {
  {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  }
  {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  }
  v = fmaxf(v, __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x128, 0xf, 0xf, false)));
  v = fmaxf(v, __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x124, 0xf, 0xf, false)));
  v = fmaxf(v, __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x4e, 0xf, 0xf, false)));
  v = fmaxf(v, __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0xb1, 0xf, 0xf, false)));
  return v;
}

// Exchange between the two lanes that share a query column of a 32x32 accumulator block (lane and lane ^ 32):
// both get the maximum, resp. the sum, of their two values.
__device__ __forceinline__ float pair_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

}  // namespace flame
