// Small device helpers shared by the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace d2o {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) double f64x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// Storage element traits: float and bf16 (held as uint16_t).
template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static __device__ __forceinline__ double to_f64(float x) { return double(x); }
  static __device__ __forceinline__ float to_f32(float x) { return x; }
  static __device__ __forceinline__ float from_f64(double x) { return float(x); }
  static __device__ __forceinline__ float from_f32(float x) { return x; }
};
template <>
struct Elem<uint16_t> {
  static __device__ __forceinline__ float to_f32(uint16_t x) { return __uint_as_float(uint32_t(x) << 16); }
  static __device__ __forceinline__ double to_f64(uint16_t x) { return double(to_f32(x)); }
  // fp64 -> bf16, round to nearest even, in one rounding (no detour through fp32 rounding):
  // bf16 keeps 7 of the 52 fraction bits; values are far from bf16's exponent limits.
  static __device__ __forceinline__ uint16_t from_f64(double x) {
    unsigned long long b = (unsigned long long)__double_as_longlong(x);
    const unsigned long long lsb = (b >> 45) & 1ull;
    b = (b + ((1ull << 44) - 1ull) + lsb) & ~((1ull << 45) - 1ull);
    const float f = float(__longlong_as_double((long long)b));  // exact: 8 significant bits
    return uint16_t(__float_as_uint(f) >> 16);
  }
  static __device__ __forceinline__ uint16_t from_f32(float x) {
    uint32_t b = __float_as_uint(x);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return uint16_t(b >> 16);
  }
};

// ---- fp8 cache rows: d codes of the 8-bit format E4M3 (1 sign, 4 exponent bits with bias 7, 3
// fraction bits, subnormals, largest magnitude 448, no infinities) and one power of two per row;
// a row's values are code * 2^e.
template <>
struct Elem<uint8_t> {  // the code alone, without the row's power of two
  static __device__ __forceinline__ float to_f32(uint8_t x) { return __builtin_amdgcn_cvt_f32_fp8(int(x), 0); }
  static __device__ __forceinline__ double to_f64(uint8_t x) { return double(to_f32(x)); }
};
__device__ __forceinline__ double pow2_f64(int e) { return __hiloint2double((1023 + e) << 20, 0); }   // |e| < 1023
__device__ __forceinline__ float pow2_f32(int e) { return __uint_as_float(uint32_t(127 + e) << 23); }  // |e| < 127
// The row's exponent: the smallest e with amax * 2^-e <= 448 (448 = 0.875 * 2^9), not below -120
// (one signed byte holds it); 0 for an all-zero row.
__device__ __forceinline__ int fp8_row_exponent(double amax) {
  if (!(amax > 0.0)) return 0;
  int ex;
  const double fr = frexp(amax, &ex);
  return max((fr <= 0.875 ? ex - 9 : ex - 8), -120);
}
// y (|y| <= 448) to the nearest E4M3 value, ties to the even fraction; exact arithmetic throughout.
__device__ __forceinline__ uint8_t fp8_encode(double y) {
  const double ay = fabs(y);
  int ex;
  (void)frexp(ay, &ex);                       // ay in [2^(ex-1), 2^ex); ex = 0 for ay = 0
  const int E = max(ex - 1, -6);              // the subnormal range counts as binade -6
  const double q = ldexp(rint(ldexp(ay, 3 - E)), E - 3);
  if (q == 0.0) return 0;                     // (no negative zero)
  int eq;
  (void)frexp(q, &eq);
  const int Eq = eq - 1;                      // rounding may have carried into the next binade
  const uint32_t code = Eq < -6 ? uint32_t(ldexp(q, 9)) : (uint32_t(Eq + 7) << 3) | uint32_t(ldexp(q, 3 - Eq) - 8.0);
  return uint8_t(code | (y < 0.0 ? 0x80u : 0u));
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ int wave_min(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, 64));
  return v;
}

// Wavefront reductions on the data-parallel-primitive path (register-to-register lane
// permutations, no LDS round trip): four butterfly steps inside each row of 16 lanes, then the
// four row results are combined through scalar registers.  Every lane gets the result; the
// combination tree is fixed.
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7 - i within 8
constexpr int kDppMirror = 0x140;      // lane i <-> 15 - i within 16
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  const int lo = dpp_i32<CTRL>(__double2loint(v)), hi = dpp_i32<CTRL>(__double2hiint(v));
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double lane_f64(double v, int lane) {
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), lane),
                          __builtin_amdgcn_readlane(__double2loint(v), lane));
}
__device__ __forceinline__ double fast_wave_max(double v) {
  v = fmax(v, dpp_f64<kDppXor1>(v));
  v = fmax(v, dpp_f64<kDppXor2>(v));
  v = fmax(v, dpp_f64<kDppHalfMirror>(v));
  v = fmax(v, dpp_f64<kDppMirror>(v));
  return fmax(fmax(lane_f64(v, 0), lane_f64(v, 16)), fmax(lane_f64(v, 32), lane_f64(v, 48)));
}
__device__ __forceinline__ double fast_wave_sum(double v) {
  v += dpp_f64<kDppXor1>(v);
  v += dpp_f64<kDppXor2>(v);
  v += dpp_f64<kDppHalfMirror>(v);
  v += dpp_f64<kDppMirror>(v);
  return (lane_f64(v, 0) + lane_f64(v, 16)) + (lane_f64(v, 32) + lane_f64(v, 48));
}
__device__ __forceinline__ int fast_wave_min(int v) {
  v = min(v, dpp_i32<kDppXor1>(v));
  v = min(v, dpp_i32<kDppXor2>(v));
  v = min(v, dpp_i32<kDppHalfMirror>(v));
  v = min(v, dpp_i32<kDppMirror>(v));
  return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
             min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

// Sum over each row of 16 lanes with the same four butterfly steps; every lane of the row gets
// the row's sum.
__device__ __forceinline__ double row16_sum(double v) {
  v += dpp_f64<kDppXor1>(v);
  v += dpp_f64<kDppXor2>(v);
  v += dpp_f64<kDppHalfMirror>(v);
  v += dpp_f64<kDppMirror>(v);
  return v;
}

// Workgroup barrier for exchanges through LDS only: it waits for the wavefront's LDS traffic,
// not for its outstanding global loads and stores (which __syncthreads would drain first).
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Deterministic block-wide sum (fixed tree): every thread gets the total.
// `buf` holds one double per wave; blockDim.x must be a multiple of 64 and <= 1024.
__device__ __forceinline__ double block_sum(double v, double* buf) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) buf[w] = v;
  __syncthreads();
  double t = 0.0;
  for (int i = 0; i < nw; ++i) t += buf[i];
  return t;
}

}  // namespace d2o
