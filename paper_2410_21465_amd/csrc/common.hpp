// Device-side helpers shared by the ShadowKV HIP kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace skv {

typedef uint16_t bf16_t;
constexpr int kWave = 64;

// ---- bf16 <-> fp32 / fp64 ---------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }

// fp32 -> bf16, round to nearest even (NaN stays NaN).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// fp64 -> bf16 with a single rounding: truncate to fp32, make the result odd if
// anything was lost (round-to-odd keeps the sticky information), then round the
// fp32 to bf16 nearest-even.  fp32 carries 16 more fraction bits than bf16, so
// the second rounding sees exactly what a direct rounding would.
__device__ __forceinline__ bf16_t f64_to_bf16(double x) {
  float f = __double2float_rz(x);
  if ((double)f != x) f = __uint_as_float(__float_as_uint(f) | 1u);
  return f32_to_bf16(f);
}

// ---- order-preserving key of a double (larger value <=> larger key, never 0 for
// finite or infinite inputs).  -0.0 is folded onto +0.0 first.
__device__ __forceinline__ uint64_t f64_key(double x) {
  x += 0.0;
  uint64_t u = (uint64_t)__double_as_longlong(x);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

// ---- wave-level helpers -----------------------------------------------------
__device__ __forceinline__ double shfl_xor_f64(double v, int mask) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_xor(lo, mask, kWave);
  hi = __shfl_xor(hi, mask, kWave);
  return __hiloint2double(hi, lo);
}

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int mask) {
  uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
  lo = (uint32_t)__shfl_xor((int)lo, mask, kWave);
  hi = (uint32_t)__shfl_xor((int)hi, mask, kWave);
  return ((uint64_t)hi << 32) | lo;
}

// sum over the 16 lanes that share lane/16 (result in all 16)
__device__ __forceinline__ double sum16_f64(double v) {
  v += shfl_xor_f64(v, 8);
  v += shfl_xor_f64(v, 4);
  v += shfl_xor_f64(v, 2);
  v += shfl_xor_f64(v, 1);
  return v;
}
__device__ __forceinline__ float sum16_f32(float v) {
  v += __shfl_xor(v, 8, kWave);
  v += __shfl_xor(v, 4, kWave);
  v += __shfl_xor(v, 2, kWave);
  v += __shfl_xor(v, 1, kWave);
  return v;
}
__device__ __forceinline__ double wave_max_f64(double v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmax(v, shfl_xor_f64(v, m));
  return v;
}
__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += shfl_xor_f64(v, m);
  return v;
}

// Load ELEMS consecutive bf16 (ELEMS in {4, 6, 8}) from a 4-byte aligned address
// (16-byte aligned when ELEMS == 8) and widen them to fp32.
template <int ELEMS>
__device__ __forceinline__ void load_bf16_row(const bf16_t* __restrict__ p, float (&x)[ELEMS]) {
  static_assert(ELEMS == 4 || ELEMS == 6 || ELEMS == 8, "unsupported slice width");
  if constexpr (ELEMS == 8) {
    uint4 w = *reinterpret_cast<const uint4*>(p);
    x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x); x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
    x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z); x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
  } else if constexpr (ELEMS == 6) {
    const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
    uint32_t a = q[0], b = q[1], c = q[2];
    x[0] = bf16_lo(a); x[1] = bf16_hi(a); x[2] = bf16_lo(b); x[3] = bf16_hi(b);
    x[4] = bf16_lo(c); x[5] = bf16_hi(c);
  } else {
    uint2 w = *reinterpret_cast<const uint2*>(p);
    x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x); x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
  }
}

// Store ELEMS consecutive bf16 given as fp32 (round to nearest even).
template <int ELEMS>
__device__ __forceinline__ void store_bf16_row(bf16_t* __restrict__ p, const bf16_t (&h)[ELEMS]) {
  uint32_t* q = reinterpret_cast<uint32_t*>(p);
#pragma unroll
  for (int i = 0; i < ELEMS / 2; ++i) q[i] = (uint32_t)h[2 * i] | ((uint32_t)h[2 * i + 1] << 16);
}

}  // namespace skv
