// Workgroup-wide exact selection of the `k` largest 64-bit keys (ArgTopK of both
// algorithms of the paper; ties go to the lower index).
//
// Every thread of an NT-thread workgroup holds E keys in blocked order: element
// (tid, e) has order index tid * E + e.  Key 0 means "absent".  The method is a
// most-significant-digit radix select (8-bit digits, LDS histograms private to each
// wave) that first skips the bit prefix all keys share, and stops as soon as the
// digit bin that straddles the k-th position is needed in full.  After that a
// single ordered scan gives every thread the output slot of its selected elements,
// so the result is written in ascending order index without atomics.
#pragma once
#include "common.hpp"

namespace skv {

template <int NT>
struct SelectSmem {
  static constexpr int NW = NT / kWave;
  uint32_t hist[NW][256];
  uint64_t red_and[NW];
  uint64_t red_or[NW];
  uint32_t wave_tot[NW];
  uint32_t bin, above, cnt;
};

// Exclusive prefix sum of `v` over the workgroup in thread order; needs sm.wave_tot.
template <int NT>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, SelectSmem<NT>& sm) {
  constexpr int NW = NT / kWave;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  uint32_t incl = v;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    uint32_t t = (uint32_t)__shfl_up((int)incl, off, kWave);
    if (lane >= off) incl += t;
  }
  if (lane == kWave - 1) sm.wave_tot[wave] = incl;
  __syncthreads();
  uint32_t base = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w)
    if (w < wave) base += sm.wave_tot[w];
  __syncthreads();
  return base + incl - v;
}

// Value of an order-preserving key (inverse of f64_key).
__device__ __forceinline__ double f64_from_key(uint64_t key) {
  const uint64_t u = (key >> 63) ? (key & 0x7fffffffffffffffull) : ~key;
  return __longlong_as_double((long long)u);
}

// Threshold search among the present (non-zero) keys: on return the k largest are those whose bits
// under det_mask exceed det_val, plus `need` of those that equal it.  Returns true when all of the
// equal ones are wanted (or none is left to want), false when the keys ran out of bits first, i.e.
// more than `need` keys are identical.
template <int NT, int E>
__device__ bool radix_threshold(const uint64_t (&key)[E], uint32_t k, SelectSmem<NT>& sm, uint64_t& det_val,
                                uint64_t& det_mask, uint32_t& need) {
  constexpr int NW = NT / kWave;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;

  // 1. bits shared by every present key
  uint64_t a = ~0ull, o = 0ull;
#pragma unroll
  for (int e = 0; e < E; ++e)
    if (key[e]) { a &= key[e]; o |= key[e]; }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) { a &= shfl_xor_u64(a, m); o |= shfl_xor_u64(o, m); }
  if (lane == 0) { sm.red_and[wave] = a; sm.red_or[wave] = o; }
  __syncthreads();
  a = ~0ull; o = 0ull;
#pragma unroll
  for (int w = 0; w < NW; ++w) { a &= sm.red_and[w]; o |= sm.red_or[w]; }
  __syncthreads();

  const uint64_t diff = a ^ o;
  int nb = diff ? 64 - __clzll((long long)diff) : 0;   // undetermined low bits
  det_mask = nb >= 64 ? 0ull : ~((1ull << nb) - 1ull);  // bits fixed so far
  det_val = a & det_mask;
  need = k;

  // 2. radix passes, most significant undetermined digit first
  while (nb > 0 && need > 0) {
    const int w = nb < 8 ? nb : 8;
    const int shift = nb - w;
    const uint32_t dmask = (1u << w) - 1u;
    for (int i = threadIdx.x; i < NW * 256; i += NT) (&sm.hist[0][0])[i] = 0u;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < E; ++e)
      if (key[e] && (key[e] & det_mask) == det_val)
        atomicAdd(&sm.hist[wave][(uint32_t)(key[e] >> shift) & dmask], 1u);
    __syncthreads();
    if (wave == 0) {
      uint32_t c[4], tot = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int b = 255 - 4 * lane - i;
        uint32_t sct = 0;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) sct += sm.hist[ww][b];
        c[i] = sct; tot += sct;
      }
      uint32_t incl = tot;
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        uint32_t t = (uint32_t)__shfl_up((int)incl, off, kWave);
        if (lane >= off) incl += t;
      }
      const uint32_t excl = incl - tot;
      if (excl < need && need <= incl) {
        uint32_t run = excl;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (need <= run + c[i]) { sm.bin = 255 - 4 * lane - i; sm.above = run; sm.cnt = c[i]; break; }
          run += c[i];
        }
      }
    }
    __syncthreads();
    const uint32_t bin = sm.bin, cnt = sm.cnt;
    need -= sm.above;
    det_val |= (uint64_t)bin << shift;
    det_mask |= (uint64_t)dmask << shift;
    nb = shift;
    __syncthreads();
    if (cnt == need) return true;  // the whole bin is wanted: no need to look at lower digits
  }
  return need == 0;
}

// On return: bit e of sel_mask is set iff element (tid, e) is among the k largest
// (k must not exceed the number of present keys); out_pos is the number of
// selected elements that precede this thread's in order index.
//
// SPREAD (keys made by f64_key from scores): such keys put the exponent field first, and one
// element in another binade than the rest costs a whole radix pass that tells nothing.  The search
// then runs on the key of (score - 1024) instead, a monotone map that lays the scores of a softmax
// out linearly (one shared exponent, 2^-42 apart); only if more elements than wanted share that
// coarse key -- scores closer than 2^-42 -- is the search repeated among them on the exact keys, so
// the result is the exact order in every case.
template <int NT, int E, bool SPREAD = false>
__device__ void block_select_topk(const uint64_t (&key)[E], int k, SelectSmem<NT>& sm,
                                  uint32_t& sel_mask, int& out_pos) {
  static_assert(E <= 32, "selection mask is 32 bits wide");
  uint64_t det_val, det_mask;
  uint32_t need;
  uint32_t gt = 0, eq = 0;
  if constexpr (SPREAD) {
    uint64_t k1[E];
#pragma unroll
    for (int e = 0; e < E; ++e) k1[e] = key[e] ? f64_key(f64_from_key(key[e]) - 1024.0) : 0ull;
    const bool done = radix_threshold<NT, E>(k1, (uint32_t)k, sm, det_val, det_mask, need);
#pragma unroll
    for (int e = 0; e < E; ++e) {
      if (!k1[e]) continue;
      const uint64_t m = k1[e] & det_mask;
      if (m > det_val) gt |= 1u << e;
      else if (m == det_val) eq |= 1u << e;
    }
    if (!done) {  // more than `need` elements share the coarse key: settle it among them on the exact keys
      uint64_t k2[E];
#pragma unroll
      for (int e = 0; e < E; ++e) k2[e] = (eq & (1u << e)) ? key[e] : 0ull;
      radix_threshold<NT, E>(k2, need, sm, det_val, det_mask, need);
      eq = 0;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        if (!k2[e]) continue;
        const uint64_t m = k2[e] & det_mask;
        if (m > det_val) gt |= 1u << e;
        else if (m == det_val) eq |= 1u << e;
      }
    }
  } else {
    radix_threshold<NT, E>(key, (uint32_t)k, sm, det_val, det_mask, need);
#pragma unroll
    for (int e = 0; e < E; ++e) {
      if (!key[e]) continue;
      const uint64_t m = key[e] & det_mask;
      if (m > det_val) gt |= 1u << e;
      else if (m == det_val) eq |= 1u << e;
    }
  }
  // place: the greater ones are in; of the equal ones the first `need` in order index are in
  const uint32_t cg = (uint32_t)__popc(gt), ce = (uint32_t)__popc(eq);
  const uint32_t excl = block_exclusive_scan<NT>((cg << 16) | ce, sm);
  const uint32_t pre_g = excl >> 16, pre_e = excl & 0xffffu;
  out_pos = (int)(pre_g + (pre_e < need ? pre_e : need));
  uint32_t sel = gt, rank = pre_e;
#pragma unroll
  for (int e = 0; e < E; ++e)
    if (eq & (1u << e)) { if (rank < need) sel |= 1u << e; ++rank; }
  sel_mask = sel;
}

}  // namespace skv
