// Workgroup-wide exact selection of the `k` largest keys (ArgTopK of both
// algorithms of the paper; ties go to the lower index).
//
// Every thread of an NT-thread workgroup holds E keys in blocked order: element
// (tid, e) has order index tid * E + e.  Key 0 means "absent".  Keys are unsigned
// integers of 32 or 64 bits whose order is the order wanted.  The method is a
// most-significant-digit radix select (8-bit digits, LDS histograms private to each
// wave) that first skips the bit prefix all keys share, and stops as soon as the
// digit bin that straddles the k-th position is needed in full.  After that a
// single ordered scan gives every thread the output slot of its selected elements,
// so the result is written in ascending order index without atomics.
//
// banded_select_topk (further down) is the form the decode step uses: the search runs on
// 32-bit keys made from the stored fp32 logits, and wherever those cannot decide -- an
// element left out lies within the rounding error of the k-th one -- the elements near the
// boundary are scored again exactly (fp64, from the landmarks) and the boundary is settled
// on those scores, so the selected set is the one an fp64 ranking gives.
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

template <typename K>
__device__ __forceinline__ int key_clz(K v) {   // v != 0
  if constexpr (sizeof(K) == 8) return __clzll((long long)v);
  else return __clz((int)v);
}

// Exclusive prefix sum of `v` over the workgroup in thread order; needs sm.wave_tot.
template <int NT>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, SelectSmem<NT>& sm) {
  constexpr int NW = NT / kWave;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const uint32_t incl = wave_incl_scan_u32(v);
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
template <int NT, int E, typename K>
__device__ bool radix_threshold(const K (&key)[E], uint32_t k, SelectSmem<NT>& sm, K& det_val, K& det_mask,
                                uint32_t& need) {
  constexpr int NW = NT / kWave;
  constexpr int BITS = 8 * (int)sizeof(K);
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;

  // 1. bits shared by every present key
  K a = (K)~(K)0, o = 0;
#pragma unroll
  for (int e = 0; e < E; ++e)
    if (key[e]) { a &= key[e]; o |= key[e]; }
  if constexpr (sizeof(K) == 8) {   // bitwise: the two halves reduce independently
    a = (K)(((uint64_t)wave_and_u32((uint32_t)((uint64_t)a >> 32)) << 32) | wave_and_u32((uint32_t)a));
    o = (K)(((uint64_t)wave_or_u32((uint32_t)((uint64_t)o >> 32)) << 32) | wave_or_u32((uint32_t)o));
  } else {
    a = (K)wave_and_u32((uint32_t)a);
    o = (K)wave_or_u32((uint32_t)o);
  }
  if (lane == 0) { sm.red_and[wave] = a; sm.red_or[wave] = o; }
  __syncthreads();
  a = (K)~(K)0; o = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) { a &= (K)sm.red_and[w]; o |= (K)sm.red_or[w]; }
  __syncthreads();

  const K diff = a ^ o;
  int nb = diff ? BITS - key_clz<K>(diff) : 0;                   // undetermined low bits
  det_mask = nb >= BITS ? (K)0 : (K)~((((K)1) << nb) - (K)1);     // bits fixed so far
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
      const uint32_t incl = wave_incl_scan_u32(tot);
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
    det_val |= (K)bin << shift;
    det_mask |= (K)dmask << shift;
    nb = shift;
    __syncthreads();
    if (cnt == need) return true;  // the whole bin is wanted: no need to look at lower digits
  }
  return need == 0;
}

// Elements above the threshold / equal to it, as bit masks over the thread's E elements (branch-free on purpose:
// with a branch per element the compiler kept the two masks in scratch memory).
template <int E, typename K>
__device__ __forceinline__ void classify(const K (&key)[E], K det_val, K det_mask, uint32_t& gt_out, uint32_t& eq_out) {
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const K m = key[e] & det_mask;
    const bool present = key[e] != 0;
    gt |= (uint32_t)(present & (m > det_val)) << e;
    eq |= (uint32_t)(present & (m == det_val)) << e;
  }
  gt_out |= gt; eq_out |= eq;
}

// Placement: the greater ones are in; of the equal ones the first `need` in order index are in.
// out_pos = number of selected elements that precede this thread's in order index.
template <int NT, int E>
__device__ __forceinline__ void place_selected(uint32_t gt, uint32_t eq, uint32_t need, SelectSmem<NT>& sm,
                                               uint32_t& sel_mask, int& out_pos) {
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
    const bool done = radix_threshold<NT, E, uint64_t>(k1, (uint32_t)k, sm, det_val, det_mask, need);
    classify<E, uint64_t>(k1, det_val, det_mask, gt, eq);
    if (!done) {  // more than `need` elements share the coarse key: settle it among them on the exact keys
      uint64_t k2[E];
#pragma unroll
      for (int e = 0; e < E; ++e) k2[e] = (eq & (1u << e)) ? key[e] : 0ull;
      radix_threshold<NT, E, uint64_t>(k2, need, sm, det_val, det_mask, need);
      eq = 0;
      classify<E, uint64_t>(k2, det_val, det_mask, gt, eq);
    }
  } else {
    radix_threshold<NT, E, uint64_t>(key, (uint32_t)k, sm, det_val, det_mask, need);
    classify<E, uint64_t>(key, det_val, det_mask, gt, eq);
  }
  place_selected<NT, E>(gt, eq, need, sm, sel_mask, out_pos);
}

// ---- selection on approximate scores with an exact boundary -----------------------------------------
// Fixed-point search key of a log-domain softmax score z (z <= 0 up to rounding): (z + 128) * 2^25, clamped to
// [1, 2^32 - 1].  Linear in z (every digit tells something), 3e-8 apart.  Scores below -128 share key 1.
constexpr double kKeyOffset = 128.0, kKeyScale = 33554432.0;   // 2^25
__device__ __forceinline__ uint32_t score_key32(double z) {
  const double x = (z + kKeyOffset) * kKeyScale;
  return x >= 4294967295.0 ? 0xffffffffu : x >= 1.0 ? (uint32_t)x : 1u;   // (NaN ends at 1)
}
__device__ __forceinline__ double score_from_key32(uint32_t key) { return (double)key / kKeyScale - kKeyOffset; }

// ---- threshold search on 32-bit score keys: one histogram pass, then the boundary bin ranked from a list ----
// The histogram's 2048 bins count down from `key_top`, a key no element exceeds (the largest score of the unit):
// the upper 1024 bins are 2^19 key units wide (1/64 in the score) and cover the 16 below the top, where the
// threshold of a softmax that is not extremely peaked lies; the lower 1024 are 2^22 wide (1/8) and cover the rest
// of the key range.  Wave 0 walks the histogram from the top to the bin that straddles the k-th position.  The few
// keys in that bin are put on a list and ranked against each other (larger key first, equal keys by order
// index): no further passes.  A boundary bin with more keys than the list holds falls back to radix passes among
// them.
constexpr int kHistBins = 2048, kFineShift = 19, kCoarseShift = 22;
constexpr int kListCap = 512;
template <int NT>
struct Select32Smem {
  static constexpr int NW = NT / kWave;
  union {
    SelectSmem<NT> radix;        // fallback passes, and the exact (64-bit) search of the banded selection
    uint32_t hist[kHistBins];
  };
  uint32_t list_key[kListCap], list_ord[kListCap];
  uint64_t list_z[kListCap];   // exact scores (as keys) of the elements near the boundary
  uint32_t list_n, bin, above, cnt;
  uint32_t red[2 * NW];
};
// Must run (and be followed by a barrier) before threshold32.
template <int NT>
__device__ __forceinline__ void threshold32_prepare(Select32Smem<NT>& sm) {
  for (int i = threadIdx.x; i < kHistBins; i += NT) sm.hist[i] = 0u;
  if (threadIdx.x == 0) sm.list_n = 0u;
}
__device__ __forceinline__ uint32_t hist_bin(uint32_t key, uint32_t key_top) {
  const uint32_t d = key < key_top ? key_top - key : 0u;            // distance below the top
  const uint32_t fine = (uint32_t)(kHistBins / 2) << kFineShift;    // 2^29: the part the fine bins cover
  if (d < fine) return (uint32_t)kHistBins - 1u - (d >> kFineShift);
  const uint32_t c = (d - fine) >> kCoarseShift;                    // at most (2^32 - 2^29) >> 22 = 896
  return (uint32_t)(kHistBins / 2) - 1u - c;
}

// smallest key that falls into `bin` (inverse of hist_bin at the bin's lower edge; 0 when the edge is below every key)
__device__ __forceinline__ uint32_t hist_bin_floor(uint32_t bin, uint32_t key_top) {
  const uint32_t fine = (uint32_t)(kHistBins / 2) << kFineShift;
  uint64_t d_max;   // largest distance below the top that still maps to `bin`
  if (bin >= (uint32_t)(kHistBins / 2)) d_max = (((uint64_t)kHistBins - bin) << kFineShift) - 1u;
  else d_max = (uint64_t)fine + ((((uint64_t)(kHistBins / 2) - bin)) << kCoarseShift) - 1u;
  return d_max >= key_top ? 0u : key_top - (uint32_t)d_max;
}

// On return: `gt` = elements certainly among the k largest keys, `eq` = elements of which the first `need` in order
// index are also in.  Returns false when `eq` holds more than `need` elements (identical keys; fallback path only).
// When the boundary bin holds at most 64 keys (the usual case) every wave ranks them in its own registers and
// `tu_known` is set: t_key = smallest key taken, u_key = largest key left out, or an upper bound on it (the
// largest key that can lie below the boundary bin) when nothing of the bin is left out; 0 = nothing below.
template <int NT, int E>
__device__ bool threshold32(const uint32_t (&key)[E], uint32_t k, uint32_t key_top, Select32Smem<NT>& sm, uint32_t& gt,
                            uint32_t& eq, uint32_t& need, bool& tu_known, uint32_t& t_key, uint32_t& u_key) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  uint32_t bins[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    bins[e] = hist_bin(key[e], key_top);
    if (key[e]) atomicAdd(&sm.hist[bins[e]], 1u);
  }
  __syncthreads();
  if (wave == 0) {
    // lane l owns the 32 bins from hi = 2047 - 32 l downwards
    constexpr int PER = kHistBins / kWave;
    const int hi = kHistBins - 1 - PER * lane;
    uint32_t c[PER], tot = 0;
#pragma unroll
    for (int j = 0; j < PER / 4; ++j) {
      const uint4 v = *reinterpret_cast<const uint4*>(&sm.hist[hi - 3 - 4 * j]);
      c[4 * j] = v.w; c[4 * j + 1] = v.z; c[4 * j + 2] = v.y; c[4 * j + 3] = v.x;   // descending bins
      tot += v.x + v.y + v.z + v.w;
    }
    const uint32_t incl = wave_incl_scan_u32(tot), excl = incl - tot;
    if (excl < k && k <= incl) {
      uint32_t run = excl;
      bool found = false;
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        if (!found && k <= run + c[i]) { sm.bin = (uint32_t)(hi - i); sm.above = run; sm.cnt = c[i]; found = true; }
        run += c[i];
      }
    }
  }
  __syncthreads();
  const uint32_t bin = sm.bin, cnt = sm.cnt;
  need = k - sm.above;
  uint32_t cand = 0;
  gt = 0; eq = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const bool present = key[e] != 0u;
    gt |= (uint32_t)(present & (bins[e] > bin)) << e;
    cand |= (uint32_t)(present & (bins[e] == bin)) << e;
  }
  tu_known = false;
  if (cnt > (uint32_t)kWave && cnt == need) { eq = cand; return true; }      // the whole bin is wanted
  if (cnt <= (uint32_t)kListCap) {
#pragma unroll
    for (int e = 0; e < E; ++e)
      if (cand & (1u << e)) {
        const uint32_t slot = atomicAdd(&sm.list_n, 1u);
        sm.list_key[slot] = key[e];
        sm.list_ord[slot] = threadIdx.x * E + e;
      }
    __syncthreads();
    if (cnt <= (uint32_t)kWave) {
      // every wave ranks the list in its registers: lane i holds entry i and counts the entries ahead of it
      const uint32_t kv = (uint32_t)lane < cnt ? sm.list_key[lane] : 0u, ov = (uint32_t)lane < cnt ? sm.list_ord[lane] : 0xffffffffu;
      uint32_t ahead = 0;
      for (uint32_t j = 0; j < cnt; ++j) {
        const uint32_t kj = (uint32_t)__builtin_amdgcn_readlane((int)kv, (int)j), oj = (uint32_t)__builtin_amdgcn_readlane((int)ov, (int)j);
        ahead += (kj > kv) | ((kj == kv) & (oj < ov));
      }
      const int it = __ffsll((unsigned long long)__ballot((uint32_t)lane < cnt && ahead == need - 1u)) - 1;   // last one taken
      t_key = (uint32_t)__builtin_amdgcn_readlane((int)kv, it);
      const uint32_t t_ord = (uint32_t)__builtin_amdgcn_readlane((int)ov, it);
      if (cnt > need) {
        const int iu = __ffsll((unsigned long long)__ballot((uint32_t)lane < cnt && ahead == need)) - 1;      // first one left out
        u_key = (uint32_t)__builtin_amdgcn_readlane((int)kv, iu);
      } else {
        const uint32_t fl = hist_bin_floor(bin, key_top);
        u_key = fl > 1u ? fl - 1u : 0u;
      }
      tu_known = true;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const bool in = (key[e] > t_key) | ((key[e] == t_key) & (threadIdx.x * E + e <= t_ord));
        gt |= (uint32_t)(((cand >> e) & 1u) & in) << e;
      }
      need = 0;
      return true;
    }
    // a longer list: every thread walks it once (broadcast reads) and counts, for each of its own candidates, the
    // entries ahead of it.  Equal keys on both sides of the boundary are ranked by order index here; the caller sees them
    // as a taken and a left-out element with the same key and settles them on exact scores.
    if (__builtin_amdgcn_readfirstlane(__any(cand != 0u))) {
      uint32_t ahead[E];
#pragma unroll
      for (int e = 0; e < E; ++e) ahead[e] = 0u;
      for (uint32_t j = 0; j < cnt; ++j) {
        const uint32_t kj = sm.list_key[j], oj = sm.list_ord[j];
#pragma unroll
        for (int e = 0; e < E; ++e)
          ahead[e] += (kj > key[e]) | ((kj == key[e]) & (oj < threadIdx.x * E + e));
      }
#pragma unroll
      for (int e = 0; e < E; ++e) gt |= (uint32_t)(((cand >> e) & 1u) & (ahead[e] < need)) << e;
    }
    need = 0;
    return true;
  }
  // more keys in the boundary bin than the list holds: radix passes among them
  uint32_t k2[E];
#pragma unroll
  for (int e = 0; e < E; ++e) k2[e] = (cand & (1u << e)) ? key[e] : 0u;
  __syncthreads();   // the histogram's memory becomes the radix histograms
  uint32_t det_val, det_mask;
  const bool all_wanted = radix_threshold<NT, E, uint32_t>(k2, need, sm.radix, det_val, det_mask, need);
  classify<E, uint32_t>(k2, det_val, det_mask, gt, eq);
  return all_wanted;
}

// The k largest of the exact scores z, found through 32-bit keys of approximate scores z~ (key = score_key32(z~)):
//   |z~ - z| <= u_rel * (|z~| + lmax)  for every element, where lmax bounds the magnitude of what was subtracted
//   from the stored logit to make the score (the head's log-sum-exp).
// The search finds the k-th largest key T.  With D = that bound taken at |T| + 1, plus the key's own resolution,
// every element whose key is more than 2D above T is in the exact top k, every one more than 2D below is not
// (for elements within 1 of T the bound at |T| + 1 covers them; further down the distance grows faster than the
// bound, as long as 2D < 0.45 -- beyond that every element counts as near).  If no element left out is within 2D
// of T the selection by keys is the exact one.  Otherwise the elements within 2D of T are scored again exactly
// (fp64) and the search is repeated on exact 64-bit keys with the elements above the band forced in.
//   row_of(e)       what the exact scorers take for element e (its landmark row)
//   score_wave(r)   exact score of row r, computed by the calling wave together (same r in every lane)
//   score_thread(r) the same by one thread alone (only used when the elements near the boundary outnumber the list)
//   early(sel)      called once the selection is known and before the output positions are (the fast case only)
// Needs threshold32_prepare and a barrier before it; `key_top` is a key no element exceeds.
template <int NT, int E, class RowOf, class ScoreWave, class ScoreThread, class Early>
__device__ void banded_select_topk(const uint32_t (&key)[E], int k, uint32_t key_top, Select32Smem<NT>& sm, double lmax,
                                   double u_rel, RowOf row_of, ScoreWave score_wave, ScoreThread score_thread,
                                   Early early, uint32_t& sel_mask, int& out_pos) {
  constexpr int NW = NT / kWave;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  uint32_t gt, eq, need, kmin, kmax;
  bool tu_known;
  const bool decided = threshold32<NT, E>(key, (uint32_t)k, key_top, sm, gt, eq, need, tu_known, kmin, kmax);
  if (!tu_known) {
    // smallest key taken, largest key left out (when `decided`, every element of eq is taken)
    kmin = 0xffffffffu; kmax = 0u;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const bool taken = ((gt | eq) >> e) & 1u;
      const uint32_t lo = taken ? key[e] : 0xffffffffu, hi = taken ? 0u : key[e];   // absent keys are 0: never taken
      kmin = lo < kmin ? lo : kmin;
      kmax = hi > kmax ? hi : kmax;
    }
    kmin = wave_min_u32(kmin);
    kmax = wave_max_u32(kmax);
    if (lane == 0) { sm.red[wave] = kmin; sm.red[NW + wave] = kmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const uint32_t a = sm.red[w], b = sm.red[NW + w];
      kmin = a < kmin ? a : kmin; kmax = b > kmax ? b : kmax;
    }
  }
  const double T = score_from_key32(kmin);
  double band = 2.0 * (u_rel * (fabs(T) + 1.0 + lmax) + 2.0 / kKeyScale);
  // keys at the ends of the fixed-point range stand for scores that may lie anywhere beyond them: with the
  // threshold within 1 of the lower end (or at the upper end) the keys decide nothing
  const bool blind = !(band < 0.45) || kmin < (uint32_t)kKeyScale + 2u || kmin == 0xffffffffu;
  const bool near_miss = kmax != 0u && score_from_key32(kmax) >= T - band;
  if (decided && !blind && !near_miss) {
    early(gt | eq);
    place_selected<NT, E>(gt, eq, need, sm.radix, sel_mask, out_pos);
    return;
  }
  // the boundary is not decided by the keys: exact scores for every element near it
  if (blind) band = INFINITY;
  uint32_t above = 0, near = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const double z = score_from_key32(key[e]);
    const bool present = key[e] != 0u, hi = z > T + band;
    above |= (uint32_t)(present & hi) << e;
    near |= (uint32_t)(present & !hi & (z >= T - band)) << e;
  }
  if (threadIdx.x == 0) { sm.list_n = 0u; sm.above = 0u; }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < E; ++e)
    if (near & (1u << e)) {
      const uint32_t slot = atomicAdd(&sm.list_n, 1u);
      if (slot < (uint32_t)kListCap) { sm.list_ord[slot] = threadIdx.x * E + e; sm.list_key[slot] = (uint32_t)row_of(e); }
    }
  {
    const uint32_t n_mine = wave_incl_scan_u32((uint32_t)__popc(above));
    if (lane == kWave - 1 && n_mine) atomicAdd(&sm.above, n_mine);
  }
  __syncthreads();
  const uint32_t n_near = sm.list_n, n_above = sm.above;
  if (n_near <= (uint32_t)kWave) {
    // the usual case, a handful of elements: one wave per row for the exact scores, then every wave ranks them in
    // its registers (larger score first, equal scores by order index) and every thread decides its own elements
    for (uint32_t i = wave; i < n_near; i += NW) {
      const double ze = score_wave((int)sm.list_key[i]);
      if (lane == 0) sm.list_z[i] = f64_key(ze);
    }
    __syncthreads();
    const uint32_t want = (uint32_t)k - n_above;    // places left for the elements near the boundary (>= 1)
    const uint64_t zv = (uint32_t)lane < n_near ? sm.list_z[lane] : 0ull;
    const uint32_t ov = (uint32_t)lane < n_near ? sm.list_ord[lane] : 0xffffffffu;
    uint32_t ahead = 0;
    for (uint32_t j = 0; j < n_near; ++j) {
      const uint64_t zj = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(zv >> 32), (int)j) << 32) |
                          (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)zv, (int)j);
      const uint32_t oj = (uint32_t)__builtin_amdgcn_readlane((int)ov, (int)j);
      ahead += (zj > zv) | ((zj == zv) & (oj < ov));
    }
    const unsigned long long taken = __ballot((uint32_t)lane < n_near && ahead < want);
    uint32_t gt2 = above;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      if (!(near & (1u << e))) continue;
      const uint32_t ord = threadIdx.x * E + e;
      for (uint32_t j = 0; j < n_near; ++j)
        if ((uint32_t)__builtin_amdgcn_readlane((int)ov, (int)j) == ord && ((taken >> j) & 1ull)) gt2 |= 1u << e;
    }
    place_selected<NT, E>(gt2, 0u, 0u, sm.radix, sel_mask, out_pos);
    return;
  }
  uint64_t k2[E];
#pragma unroll
  for (int e = 0; e < E; ++e) k2[e] = (above & (1u << e)) ? f64_key(1.0) : 0ull;   // in (exact scores never reach 1)
  if (n_near <= (uint32_t)kListCap) {
    // the waves share the rows out among themselves, each scoring a row together
    for (uint32_t i = wave; i < n_near; i += NW) {
      const double ze = score_wave((int)sm.list_key[i]);
      if (lane == 0) sm.list_z[i] = f64_key(ze < 0.5 ? ze : 0.5);
    }
    __syncthreads();
    if (__builtin_amdgcn_readfirstlane(__any(near != 0u))) {
      for (uint32_t j = 0; j < n_near; ++j) {
        const uint32_t oj = sm.list_ord[j];
        const uint64_t zj = sm.list_z[j];
#pragma unroll
        for (int e = 0; e < E; ++e)
          if (oj == threadIdx.x * E + e) k2[e] = zj;
      }
    }
  } else {
#pragma unroll
    for (int e = 0; e < E; ++e)
      if (near & (1u << e)) {
        const double ze = score_thread(row_of(e));
        k2[e] = f64_key(ze < 0.5 ? ze : 0.5);
      }
  }
  __syncthreads();   // the histogram's memory is reused
  block_select_topk<NT, E, false>(k2, k, sm.radix, sel_mask, out_pos);
}

}  // namespace skv
