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

// ---- FP8 E5M2 storage of the KV cache (section "Precision Sensitivity") --------------------
// One byte per element: sign, 5 exponent bits (bias 15), 2 fraction bits, subnormals, infinities and
// NaNs as in IEEE 754 -- the upper byte of a half.  Widening is exact; the conversion unit takes two
// bytes of a 32-bit word at a time (v_cvt_pk_f32_bf8; checked on the chip against the format's
// definition for all 256 codes).
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void e5m2x4_to_f32(uint32_t w, float* x) {
  const f32x2_t lo = __builtin_amdgcn_cvt_pk_f32_bf8((int)w, false);
  const f32x2_t hi = __builtin_amdgcn_cvt_pk_f32_bf8((int)w, true);
  x[0] = lo[0]; x[1] = lo[1]; x[2] = hi[0]; x[3] = hi[1];
}
__device__ __forceinline__ float e5m2_to_f32(uint8_t v) { return __builtin_amdgcn_cvt_f32_bf8((int)v, 0); }
// two E5M2 values (bytes 2*PAIR and 2*PAIR+1 of w) as a pair of bf16 bit patterns: every E5M2 value is
// exact in bf16, so the upper halves of the fp32 patterns are the answer
template <int PAIR>
__device__ __forceinline__ uint32_t e5m2x2_to_bf16x2(uint32_t w) {
  const f32x2_t f = __builtin_amdgcn_cvt_pk_f32_bf8((int)w, PAIR != 0);
  return (__float_as_uint(f[0]) >> 16) | (__float_as_uint(f[1]) & 0xffff0000u);
}

// fp64 -> E5M2 with a single rounding (nearest, ties to even; beyond the largest finite value 57344
// the result is infinity, as in IEEE 754): fp64 -> fp32 by truncation with a sticky last bit, then
// the fp32 is rounded at its 21st fraction bit, in integer arithmetic so that a carry moves into the
// exponent by itself; below 2^-14 the codes are equally spaced (2^-16).
__device__ __forceinline__ uint8_t f64_to_e5m2(double x) {
  float f = __double2float_rz(x);
  if ((double)f != x) f = __uint_as_float(__float_as_uint(f) | 1u);
  const uint32_t u = __float_as_uint(f);
  const uint32_t sign = (u >> 24) & 0x80u, a = u & 0x7fffffffu;
  if (a > 0x7f800000u) return (uint8_t)(sign | 0x7fu);
  if (a >= 0x38800000u) {  // |f| >= 2^-14: a normal E5M2 number, or overflow
    const uint32_t r = (a + 0xfffffu + ((a >> 21) & 1u)) >> 21;  // 8 exponent bits | 2 fraction bits
    const int e = (int)(r >> 2) - 127 + 15;
    if (e >= 31) return (uint8_t)(sign | 0x7cu);
    return (uint8_t)(sign | ((uint32_t)e << 2) | (r & 3u));
  }
  return (uint8_t)(sign | (uint32_t)rintf(__uint_as_float(a) * 65536.0f));  // 0..4; 4 is the smallest normal
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

// ---- wave-wide scans and reductions on the DPP path (data-parallel primitives: a VALU operand taken from another
// lane, no LDS round trip as with the shuffle builtins).  Pattern: inclusive scan inside each row of 16 lanes with
// row_shr 1, 2, 4, 8 (lanes without a source take the identity), then lane 15 of rows 0 and 2 into rows 1 and 3
// (row_bcast:15), then lane 31 into rows 2 and 3 (row_bcast:31).  Lane 63 ends with the reduction over the wave.
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t identity, uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)x, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ double dpp_f64(double identity, double x) {
  const int lo = __builtin_amdgcn_update_dpp(__double2loint(identity), __double2loint(x), CTRL, ROW_MASK, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(__double2hiint(identity), __double2hiint(x), CTRL, ROW_MASK, 0xf, false);
  return __hiloint2double(hi, lo);
}
#define SKV_WAVE_SCAN(T, DPP, OP, ID)                                        \
  x = OP(x, DPP<0x111>(ID, x)); x = OP(x, DPP<0x112>(ID, x));                \
  x = OP(x, DPP<0x114>(ID, x)); x = OP(x, DPP<0x118>(ID, x));                \
  x = OP(x, DPP<0x142, 0xa>(ID, x)); x = OP(x, DPP<0x143, 0xc>(ID, x));
__device__ __forceinline__ uint32_t op_add(uint32_t a, uint32_t b) { return a + b; }
__device__ __forceinline__ uint32_t op_min(uint32_t a, uint32_t b) { return a < b ? a : b; }
__device__ __forceinline__ uint32_t op_max(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t op_and(uint32_t a, uint32_t b) { return a & b; }
__device__ __forceinline__ uint32_t op_or(uint32_t a, uint32_t b) { return a | b; }
__device__ __forceinline__ uint32_t last_lane_u32(uint32_t x) { return (uint32_t)__builtin_amdgcn_readlane((int)x, kWave - 1); }
// inclusive prefix sum over the wave's lanes
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t x) { SKV_WAVE_SCAN(uint32_t, dpp_u32, op_add, 0u) return x; }
// reductions over the wave, result in every lane (through a scalar register)
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x) { SKV_WAVE_SCAN(uint32_t, dpp_u32, op_min, 0xffffffffu) return last_lane_u32(x); }
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) { SKV_WAVE_SCAN(uint32_t, dpp_u32, op_max, 0u) return last_lane_u32(x); }
__device__ __forceinline__ uint32_t wave_and_u32(uint32_t x) { SKV_WAVE_SCAN(uint32_t, dpp_u32, op_and, 0xffffffffu) return last_lane_u32(x); }
__device__ __forceinline__ uint32_t wave_or_u32(uint32_t x) { SKV_WAVE_SCAN(uint32_t, dpp_u32, op_or, 0u) return last_lane_u32(x); }
__device__ __forceinline__ double last_lane_f64(double x) {
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), kWave - 1),
                          __builtin_amdgcn_readlane(__double2loint(x), kWave - 1));
}
__device__ __forceinline__ double wave_max_f64_dpp(double x) {
  SKV_WAVE_SCAN(double, dpp_f64, fmax, -INFINITY)
  return last_lane_f64(x);
}
// (the order of the additions is fixed by the pattern: the same inputs give the same bits on every run)
__device__ __forceinline__ double op_addd(double a, double b) { return a + b; }
__device__ __forceinline__ double wave_sum_f64_dpp(double x) {
  SKV_WAVE_SCAN(double, dpp_f64, op_addd, 0.0)
  return last_lane_f64(x);
}
#undef SKV_WAVE_SCAN
// the same two through the shuffle path (butterfly order)
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

// 32-bit words that hold EPL consecutive elements of EB bytes
template <int EPL, int EB>
struct RawWords { static constexpr int n = (EPL * EB + 3) / 4; };

// EPL consecutive stored elements (EPL in {4, 6, 8}) as fp32
template <int EPL, int EB>
__device__ __forceinline__ void unpack_kv(const uint32_t (&w)[RawWords<EPL, EB>::n], float (&x)[EPL]) {
  if constexpr (EB == 2) {
#pragma unroll
    for (int i = 0; i < EPL / 2; ++i) { x[2 * i] = bf16_lo(w[i]); x[2 * i + 1] = bf16_hi(w[i]); }
  } else {
    e5m2x4_to_f32(w[0], x);
    if constexpr (EPL == 8) e5m2x4_to_f32(w[1], x + 4);
    if constexpr (EPL == 6) {
      const f32x2_t t = __builtin_amdgcn_cvt_pk_f32_bf8((int)w[1], false);
      x[4] = t[0]; x[5] = t[1];
    }
  }
}
// p: address of the first of the EPL elements (EPL * EB bytes apart from lane to lane)
template <int EPL, int EB>
__device__ __forceinline__ void load_raw(const uint8_t* __restrict__ p, uint32_t (&w)[RawWords<EPL, EB>::n]) {
  if constexpr (EPL * EB == 16) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  } else if constexpr (EPL * EB == 12) {
    const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
    w[0] = q[0]; w[1] = q[1]; w[2] = q[2];
  } else if constexpr (EPL * EB == 8) {
    const uint2 v = *reinterpret_cast<const uint2*>(p);
    w[0] = v.x; w[1] = v.y;
  } else if constexpr (EPL * EB == 6) {   // 2-byte aligned only
    const uint16_t* q = reinterpret_cast<const uint16_t*>(p);
    w[0] = (uint32_t)q[0] | ((uint32_t)q[1] << 16); w[1] = q[2];
  } else {
    w[0] = *reinterpret_cast<const uint32_t*>(p);
  }
}
// Raw words of EPL stored elements back to memory (same alignment rules as load_raw).
template <int EPL, int EB>
__device__ __forceinline__ void store_raw(uint8_t* __restrict__ p, const uint32_t (&w)[RawWords<EPL, EB>::n]) {
  if constexpr (EPL * EB == 16) {
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  } else if constexpr (EPL * EB == 12) {
    uint32_t* q = reinterpret_cast<uint32_t*>(p);
    q[0] = w[0]; q[1] = w[1]; q[2] = w[2];
  } else if constexpr (EPL * EB == 8) {
    *reinterpret_cast<uint2*>(p) = make_uint2(w[0], w[1]);
  } else if constexpr (EPL * EB == 6) {
    uint16_t* q = reinterpret_cast<uint16_t*>(p);
    q[0] = (uint16_t)w[0]; q[1] = (uint16_t)(w[0] >> 16); q[2] = (uint16_t)w[1];
  } else {
    *reinterpret_cast<uint32_t*>(p) = w[0];
  }
}
// EPL fp64 values rounded once to the storage type, packed as raw words
template <int EPL, int EB>
__device__ __forceinline__ void pack_kv(const double (&x)[EPL], uint32_t (&w)[RawWords<EPL, EB>::n]) {
#pragma unroll
  for (int i = 0; i < RawWords<EPL, EB>::n; ++i) w[i] = 0u;
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    if constexpr (EB == 2) w[e / 2] |= (uint32_t)f64_to_bf16(x[e]) << (16 * (e & 1));
    else w[e / 4] |= (uint32_t)f64_to_e5m2(x[e]) << (8 * (e & 3));
  }
}
// one stored element as fp32 / one fp64 value rounded once into its place
template <int EB>
__device__ __forceinline__ float kv_elem(const void* base, size_t i) {
  if constexpr (EB == 2) return bf16_to_f32(static_cast<const bf16_t*>(base)[i]);
  else return e5m2_to_f32(static_cast<const uint8_t*>(base)[i]);
}
template <int EB>
__device__ __forceinline__ void kv_store_elem(void* base, size_t i, double x) {
  if constexpr (EB == 2) static_cast<bf16_t*>(base)[i] = f64_to_bf16(x);
  else static_cast<uint8_t*>(base)[i] = f64_to_e5m2(x);
}

// Store ELEMS consecutive bf16 given as fp32 (round to nearest even).
template <int ELEMS>
__device__ __forceinline__ void store_bf16_row(bf16_t* __restrict__ p, const bf16_t (&h)[ELEMS]) {
  uint32_t* q = reinterpret_cast<uint32_t*>(p);
#pragma unroll
  for (int i = 0; i < ELEMS / 2; ++i) q[i] = (uint32_t)h[2 * i] | ((uint32_t)h[2 * i + 1] << 16);
}

}  // namespace skv
