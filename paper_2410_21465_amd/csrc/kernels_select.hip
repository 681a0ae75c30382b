// ArgTopK of the decoding algorithm (group score of every landmark slot -> k chunks)
// and of the pre-filling algorithm (lowest minimum cosine -> o outlier chunks).
//
// Decoding algorithm: `select_logits_kernel` ranks the slots of a unit in one workgroup (up to 32768 of them;
// longer units in slices whose survivors `merge_logits_kernel` ranks) on 32-bit keys of the scores made from
// the stored fp32 logits, with the boundary settled on exact fp64 scores wherever those keys cannot decide.
// Pre-filling algorithm and the ArgTopK entry point (fp64 scores in an array): `select_slices` ranks one slice
// of NT*E candidates per workgroup and keeps min(k, slice) of them; `select_merge` ranks the survivors of all
// slices of a unit.  With a single slice the first kernel writes the final ids itself.
#include "kernels.hpp"
#include "select.hpp"
#include "attn_kernels.hpp"
#include <cstdlib>

namespace skv {

constexpr int kSelNT = 512;

// Log-sum-exp of each query head of the unit from the per-tile (max, sum) pairs the scoring
// kernel left behind.  Sums and the logarithm are fp64; the rescaling factors exp(m_t - m) go
// through the fp32 exp2 unit exactly as they did when the scoring kernel formed the pairs (relative
// error ~1e-7 on terms that are summed, an order below the 1e-6 at which two scores count as tied).
// Every (max, sum) pair is read once.
__device__ __forceinline__ double exp_neg_fast(double x) {
  return (double)__builtin_amdgcn_exp2f((float)(x * 1.4426950408889634074));
}
// NB of a lane's pairs are requested together (long contexts have many tiles per head).  The lane's first pair of
// the wave's first head is requested by the caller (ahead of everything else the kernel loads: the normalisers are
// on the critical path) and handed in.  Ends with a barrier.
__device__ __forceinline__ double2 lse_pair(const double2* __restrict__ p, int n_tiles, int t) {
  double2 v = p[min(t, n_tiles - 1)];
  if (t >= n_tiles) v = make_double2(-INFINITY, 0.0);   // tiles past the end count as empty
  return v;
}
// zmax_sm[g] = largest score of head g (its largest logit minus its log-sum-exp).
template <int NT, int NB>
__device__ void unit_lse(const double2* __restrict__ part, int n_tiles, int G, double* lse_sm, float* lsef_sm,
                         float* zmax_sm, double2 first) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  for (int g = wave; g < G; g += NT / kWave) {
    const double2* p = part + (size_t)g * n_tiles;
    double m = -INFINITY, s = 0.0;   // running (max, sum exp(. - max)) of this lane's tiles
    // the pairs are folded in the order lane, lane + 64, ... whatever the batching
    for (int t0 = lane; t0 < n_tiles; t0 += NB * kWave) {
      double2 v[NB];
      const bool have_first = g == wave && t0 == lane;
#pragma unroll
      for (int u = 0; u < NB; ++u) v[u] = (u == 0 && have_first) ? first : lse_pair(p, n_tiles, t0 + u * kWave);
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        if (v[u].x > m) { s = s * exp_neg_fast(m - v[u].x) + v[u].y; m = v[u].x; }
        else if (v[u].x != -INFINITY) s += v[u].y * exp_neg_fast(v[u].x - m);
      }
    }
    const double mw = wave_max_f64_dpp(m);
    s = (m == -INFINITY) ? 0.0 : s * exp_neg_fast(m - mw);
    s = wave_sum_f64_dpp(s);
    if (lane == 0) { const double ls = log(s), l = mw + ls; lse_sm[g] = l; lsef_sm[g] = (float)l; zmax_sm[g] = (float)-ls; }
  }
  __syncthreads();
}

// ---- ArgTopK of the decoding algorithm: group scores from the stored logits --------------------------
// score(slot) = max over the group's heads of (logit - lse_head).  The scoring kernel stores the logit rounded
// to fp32; the search runs on keys of approximate scores formed from those in fp32 -- stored logit minus the
// normaliser rounded to fp32: three roundings of 2^-24 each, on the logit (at most |score| + |lse|), on the
// normaliser and on the difference, together at most 2 * 2^-24 * (|score| + max |lse|) -- and
// banded_select_topk settles whatever they cannot decide on exact scores, for which `exact_group_score`
// forms the logit again from q and the landmark row in fp64 (sequential sum, like the plain definition).
constexpr double kScoreRelErr = 2.0002 / 16777216.0;   // 2 * 2^-24 with a little room for the bound's own arithmetic

// (calls, not inlined: they are rare and should not cost the common path registers; operands by value)
struct ExactOperands {
  const bf16_t* q;     // the unit's G query heads, [G, d]
  const uint8_t* L;    // the unit's landmarks, [nc_stride, d]
  int d, kv_bytes, G;
  double scale;
};
__device__ __forceinline__ ExactOperands exact_operands(const SelectArgs& a, int unit) {
  ExactOperands x;
  x.q = a.q + (size_t)unit * a.G * a.d;
  x.L = static_cast<const uint8_t*>(a.landmarks) + (size_t)unit * a.nc_stride * a.d * a.kv_bytes;
  x.d = a.d; x.kv_bytes = a.kv_bytes; x.G = a.G; x.scale = a.scale;
  return x;
}
// by one thread: the sum runs over the elements in order
template <int EB>
__device__ __forceinline__ double exact_group_score_eb(const ExactOperands& a, int j, const double* lse_sm) {
  const uint8_t* row = a.L + (size_t)j * a.d * EB;
  double best = -INFINITY;
  for (int g = 0; g < a.G; ++g) {
    const bf16_t* qg = a.q + (size_t)g * a.d;
    double dot = 0.0;
    for (int x = 0; x < a.d; ++x) dot = fma((double)bf16_to_f32(qg[x]), (double)kv_elem<EB>(row, x), dot);
    const double z = __dsub_rn(__dmul_rn(dot, a.scale), lse_sm[g]);
    best = z > best ? z : best;
  }
  return best;
}
__device__ __noinline__ double exact_group_score(ExactOperands a, int j, const double* lse_sm) {
  return a.kv_bytes == 1 ? exact_group_score_eb<1>(a, j, lse_sm) : exact_group_score_eb<2>(a, j, lse_sm);
}
// by a wave together: lane l takes elements 2l and 2l+1 (d <= 128), the partial sums are added across the wave.
// The products are exact and the sums stay within fp64's 53 bits for any data that makes sense, so the order of
// the additions does not show.  Returns the score in every lane.
template <int EB>
__device__ __forceinline__ double wave_group_score_eb(const ExactOperands& a, int j, const double* lse_sm) {
  const int lane = threadIdx.x & (kWave - 1);
  const uint8_t* row = a.L + (size_t)j * a.d * EB;
  const bool act = 2 * lane < a.d;
  const double l0 = act ? (double)kv_elem<EB>(row, 2 * lane) : 0.0, l1 = act ? (double)kv_elem<EB>(row, 2 * lane + 1) : 0.0;
  double best = -INFINITY;
  for (int g = 0; g < a.G; ++g) {
    const bf16_t* qg = a.q + (size_t)g * a.d;
    const double q0 = act ? (double)bf16_to_f32(qg[2 * lane]) : 0.0, q1 = act ? (double)bf16_to_f32(qg[2 * lane + 1]) : 0.0;
    const double dot = wave_sum_f64_dpp(fma(q1, l1, q0 * l0));
    const double z = __dsub_rn(__dmul_rn(dot, a.scale), lse_sm[g]);
    best = z > best ? z : best;
  }
  return best;
}
__device__ __noinline__ double wave_group_score(ExactOperands a, int j, const double* lse_sm) {
  return a.kv_bytes == 1 ? wave_group_score_eb<1>(a, j, lse_sm) : wave_group_score_eb<2>(a, j, lse_sm);
}

// One workgroup ranks NT*E slots of a unit (all of them when the unit has a single slice).  Thread t owns the
// E consecutive slots from base + t*E: their logits come in as 16-byte pieces, GB heads at a time, the first
// batch requested before the normalisers are formed.
// RD != 0: workgroups past the slices attend over the resident rows of the unit (head dimension RD, REB bytes
// per stored element), four query heads each: work that needs no selection, on compute units this launch would
// leave idle.
template <int NT, int E, int RD = 0, int REB = 2>
__global__ __launch_bounds__(NT) void select_logits_kernel(SelectArgs a, ResidentArgs r) {
  // RD != 0 (single slice per unit): a flat grid, the selection's workgroups first (they are dispatched first and
  // are the longer ones), then (unit, head block) of the resident rows
  if constexpr (RD != 0) {
    if ((int)blockIdx.x >= r.units) {
      const int idx = (int)blockIdx.x - r.units;
      resident_rows_attention<RD, REB, NT>(r, idx % r.units, idx / r.units * 4);
      return;
    }
  }
  constexpr int GB = E <= 4 ? 16 : E <= 8 ? 8 : E <= 16 ? 4 : 2;   // heads per batch: 64 logits in flight per thread
  __shared__ Select32Smem<NT> sm;
  __shared__ double lse_sm[64];
  const int unit = RD != 0 ? blockIdx.x : blockIdx.y, slice = RD != 0 ? 0 : blockIdx.x;
  const int base = slice * a.slice_len;
  const int n_here = min(a.slice_len, a.n - base);
  const int k_here = min(a.k, n_here);
  const int j0 = base + threadIdx.x * E;
  // One byte offset per thread serves every load (uniform row base + this offset + a constant).  No load is
  // predicated: the logits array is followed by slice_len floats of padding, so a thread past the end of a row
  // reads something readable, and its keys are cleared below.
  const char* lg = reinterpret_cast<const char*>(a.logits + (size_t)unit * a.G * a.ld);
  const uint32_t off0 = (uint32_t)j0 * 4u, row_bytes = (uint32_t)a.ld * 4u;

  float pre[GB][E];
  auto request = [&](int gb) {
#pragma unroll
    for (int g = 0; g < GB; ++g) {
      const char* row = lg + (size_t)((uint32_t)min(gb + g, a.G - 1) * row_bytes);
#pragma unroll
      for (int x = 0; x < E / 4; ++x) {
        const float4 v = *reinterpret_cast<const float4*>(row + off0 + 16u * x);
        pre[g][4 * x] = v.x; pre[g][4 * x + 1] = v.y; pre[g][4 * x + 2] = v.z; pre[g][4 * x + 3] = v.w;
      }
    }
  };
  // the normalisers first (they are on the critical path), then the logits
  __shared__ float lsef_sm[64];
  const double2* part = a.partials + (size_t)unit * a.G * a.n_tiles;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  __shared__ float zmax_sm[64];
  double2 first = make_double2(-INFINITY, 0.0);
  if (wave < a.G) first = lse_pair(part + (size_t)wave * a.n_tiles, a.n_tiles, lane);
  request(0);
  threshold32_prepare<NT>(sm);
  if (a.n_tiles > 64) unit_lse<NT, 4>(part, a.n_tiles, a.G, lse_sm, lsef_sm, zmax_sm, first);
  else unit_lse<NT, 1>(part, a.n_tiles, a.G, lse_sm, lsef_sm, zmax_sm, first);
  double lmax = 0.0;
  float zmax = -INFINITY;
  for (int g = 0; g < a.G; ++g) { lmax = fmax(lmax, fabs(lse_sm[g])); zmax = fmaxf(zmax, zmax_sm[g]); }
  // a key no slot of the unit exceeds: the largest score, with room for the roundings of the fp32 scores
  const uint32_t key_top = score_key32((double)zmax + 1e-3 + 4.0 * kScoreRelErr * ((double)fabsf(zmax) + lmax));
  if (a.n_slices > 1 && slice == 0 && (int)threadIdx.x < a.G) a.lse_out[(size_t)unit * a.G + threadIdx.x] = lse_sm[threadIdx.x];
  if (a.n_slices > 1 && slice == 0 && threadIdx.x == 0) a.key_top_out[unit] = key_top;

  // approximate group score of each slot in fp32: the maximum over the heads of (stored logit - normaliser)
  float zf[E];
#pragma unroll
  for (int e = 0; e < E; ++e) zf[e] = -INFINITY;
  for (int gb = 0; gb < a.G; gb += GB) {
    if (gb) request(gb);
#pragma unroll
    for (int g = 0; g < GB; ++g) {
      if (gb + g < a.G) {
        const float l = lsef_sm[gb + g];
#pragma unroll
        for (int e = 0; e < E; ++e) zf[e] = fmaxf(zf[e], pre[g][e] - l);
      }
    }
  }
  uint32_t key[E];
#pragma unroll
  for (int e = 0; e < E; ++e) key[e] = j0 + e < a.n ? score_key32((double)zf[e]) : 0u;

  // reported ids of the selected slots (single slice): requested as soon as the selection is known
  int id[E];
  bool have_ids = false;
  auto request_ids = [&](uint32_t m) {
    have_ids = true;
    if (a.n_slices != 1) return;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      id[e] = j0 + e;
      if ((m & (1u << e)) && a.id_map) id[e] = a.id_map[(size_t)unit * a.id_stride + j0 + e];
    }
  };
  uint32_t sel; int pos;
  const ExactOperands xo = exact_operands(a, unit);
  banded_select_topk<NT, E>(key, k_here, key_top, sm, lmax, kScoreRelErr, [&](int e) { return j0 + e; },
                            [&](int j) { return wave_group_score(xo, j, lse_sm); },
                            [&](int j) { return exact_group_score(xo, j, lse_sm); }, request_ids, sel, pos);
  if (!have_ids) request_ids(sel);

  if (a.n_slices == 1) {
#pragma unroll
    for (int e = 0; e < E; ++e)
      if ((sel & (1u << e)) && pos < k_here) {
        a.out_ids[(size_t)unit * a.k + pos] = id[e];
        if (a.out_ids2) a.out_ids2[(size_t)unit * a.k + pos] = id[e];
        ++pos;
      }
  } else {
    const size_t off = (size_t)unit * a.cand_stride + (size_t)slice * min(a.k, a.slice_len);
    uint32_t* ck = reinterpret_cast<uint32_t*>(a.cand_key);
#pragma unroll
    for (int e = 0; e < E; ++e)
      if ((sel & (1u << e)) && pos < k_here) {
        ck[off + pos] = key[e];
        a.cand_idx[off + pos] = j0 + e;
        ++pos;
      }
  }
}

// Survivors of the slices (or of a middle level) ranked by one workgroup.  MID: one workgroup per (group of
// survivors, unit) keeps the k best of its group as new survivors; otherwise one workgroup per unit writes the ids.
template <int NT, int E, bool MID>
__global__ __launch_bounds__(NT) void merge_logits_kernel(SelectArgs a) {
  __shared__ Select32Smem<NT> sm;
  __shared__ double lse_sm[64];
  const int unit = MID ? blockIdx.y : blockIdx.x;
  const int per = min(a.k, a.slice_len);
  const int n_last = a.n - (a.n_slices - 1) * a.slice_len;
  const int n_first = (a.n_slices - 1) * per + min(a.k, n_last);  // survivors of the slices
  const uint32_t* ck = reinterpret_cast<const uint32_t*>(a.cand_key) + (size_t)unit * a.cand_stride;
  const int32_t* ci = a.cand_idx + (size_t)unit * a.cand_stride;
  int n_cand = n_first, k_here = a.k;
  if constexpr (MID) {
    const int g0 = blockIdx.x * a.group_cands;
    ck += g0; ci += g0;
    n_cand = min(a.group_cands, n_first - g0);
    k_here = min(a.k, n_cand);
  } else if (a.n_groups > 0) {  // the middle level ran: its survivors are packed k per group
    ck += a.cand2_off; ci += a.cand2_off;
    const int n_last_group = n_first - (a.n_groups - 1) * a.group_cands;
    n_cand = (a.n_groups - 1) * a.k + min(a.k, n_last_group);
  }
  uint32_t key[E];
  int idx[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int c = threadIdx.x * E + e;
    key[e] = c < n_cand ? ck[c] : 0u;
    idx[e] = c < n_cand ? ci[c] : 0;
  }
  if ((int)threadIdx.x < a.G) lse_sm[threadIdx.x] = a.lse_out[(size_t)unit * a.G + threadIdx.x];
  const uint32_t key_top = a.key_top_out[unit];
  threshold32_prepare<NT>(sm);
  __syncthreads();
  double lmax = 0.0;
  for (int g = 0; g < a.G; ++g) lmax = fmax(lmax, fabs(lse_sm[g]));

  int id[E];
  bool have_ids = false;
  auto request_ids = [&](uint32_t m) {
    have_ids = true;
    if (MID) return;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      id[e] = idx[e];
      if ((m & (1u << e)) && a.id_map) id[e] = a.id_map[(size_t)unit * a.id_stride + idx[e]];
    }
  };
  uint32_t sel; int pos;
  const ExactOperands xo = exact_operands(a, unit);
  banded_select_topk<NT, E>(key, k_here, key_top, sm, lmax, kScoreRelErr, [&](int e) { return idx[e]; },
                            [&](int j) { return wave_group_score(xo, j, lse_sm); },
                            [&](int j) { return exact_group_score(xo, j, lse_sm); }, request_ids, sel, pos);
  if (!have_ids) request_ids(sel);
  if constexpr (MID) {
    const size_t off = (size_t)unit * a.cand_stride + a.cand2_off + (size_t)blockIdx.x * a.k;
    uint32_t* co = reinterpret_cast<uint32_t*>(a.cand_key);
#pragma unroll
    for (int e = 0; e < E; ++e)
      if ((sel & (1u << e)) && pos < k_here) {
        co[off + pos] = key[e];
        a.cand_idx[off + pos] = idx[e];
        ++pos;
      }
  } else {
    // survivors are in ascending index within a slice / group and slices / groups are in order, so the
    // output is in ascending index here as well
#pragma unroll
    for (int e = 0; e < E; ++e)
      if ((sel & (1u << e)) && pos < a.k) {
        a.out_ids[(size_t)unit * a.k + pos] = id[e];
        if (a.out_ids2) a.out_ids2[(size_t)unit * a.k + pos] = id[e];
        ++pos;
      }
  }
}

// ---- ArgTopK on an array of fp64 scores (outlier chunks of the pre-filling algorithm, shadowkv_argtopk) ----
template <int E>
__global__ __launch_bounds__(kSelNT) void select_slices(SelectArgs a) {
  __shared__ SelectSmem<kSelNT> sm;
  const int unit = blockIdx.y, slice = blockIdx.x;
  const int base = slice * a.slice_len;
  const int n_here = min(a.slice_len, a.n - base);
  const int k_here = min(a.k, n_here);

  uint64_t key[E];
  const double* sc = a.scores + (size_t)unit * a.n;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int j = base + threadIdx.x * E + e;
    key[e] = j < a.n ? f64_key(a.sign * sc[j]) : 0ull;
  }

  uint32_t sel; int pos;
  block_select_topk<kSelNT, E, true>(key, k_here, sm, sel, pos);

  if (a.n_slices == 1) {
#pragma unroll
    for (int e = 0; e < E; ++e)
      if ((sel & (1u << e)) && pos < k_here) {
        const int j = base + threadIdx.x * E + e;
        const int id = a.id_map ? a.id_map[(size_t)unit * a.id_stride + j] : j;
        a.out_ids[(size_t)unit * a.k + pos] = id;
        if (a.out_ids2) a.out_ids2[(size_t)unit * a.k + pos] = id;
        ++pos;
      }
  } else {
    const size_t off = (size_t)unit * a.cand_stride + (size_t)slice * min(a.k, a.slice_len);
#pragma unroll
    for (int e = 0; e < E; ++e)
      if ((sel & (1u << e)) && pos < k_here) {
        a.cand_key[off + pos] = key[e];
        a.cand_idx[off + pos] = base + threadIdx.x * E + e;
        ++pos;
      }
  }
}

// Array source.  MID: one workgroup per (group of survivors, unit) keeps the k best of its group as new
// survivors; otherwise one workgroup per unit ranks the survivors (of the slices, or of the middle level) and
// writes the final ids.
template <int E, bool MID>
__global__ __launch_bounds__(kSelNT) void select_merge(SelectArgs a) {
  __shared__ SelectSmem<kSelNT> sm;
  const int unit = MID ? blockIdx.y : blockIdx.x;
  const int per = min(a.k, a.slice_len);
  const int n_last = a.n - (a.n_slices - 1) * a.slice_len;
  const int n_first = (a.n_slices - 1) * per + min(a.k, n_last);  // survivors of the slices
  const uint64_t* ck = a.cand_key + (size_t)unit * a.cand_stride;
  const int32_t* ci = a.cand_idx + (size_t)unit * a.cand_stride;
  int n_cand = n_first, k_here = a.k;
  if constexpr (MID) {
    const int g0 = blockIdx.x * a.group_cands;
    ck += g0; ci += g0;
    n_cand = min(a.group_cands, n_first - g0);
    k_here = min(a.k, n_cand);
  } else if (a.n_groups > 0) {  // the middle level ran: its survivors are packed k per group
    ck += a.cand2_off; ci += a.cand2_off;
    const int n_last_group = n_first - (a.n_groups - 1) * a.group_cands;
    n_cand = (a.n_groups - 1) * a.k + min(a.k, n_last_group);
  }
  uint64_t key[E];
  int idx[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int c = threadIdx.x * E + e;
    key[e] = c < n_cand ? ck[c] : 0ull;
    idx[e] = c < n_cand ? ci[c] : 0;
  }
  uint32_t sel; int pos;
  block_select_topk<kSelNT, E, true>(key, k_here, sm, sel, pos);
  if constexpr (MID) {
    const size_t off = (size_t)unit * a.cand_stride + a.cand2_off + (size_t)blockIdx.x * a.k;
#pragma unroll
    for (int e = 0; e < E; ++e)
      if ((sel & (1u << e)) && pos < k_here) {
        a.cand_key[off + pos] = key[e];
        a.cand_idx[off + pos] = idx[e];
        ++pos;
      }
  } else {
    // survivors are in ascending index within a slice / group and slices / groups are in order, so the
    // output is in ascending index here as well
#pragma unroll
    for (int e = 0; e < E; ++e)
      if ((sel & (1u << e)) && pos < a.k) {
        const int id = a.id_map ? a.id_map[(size_t)unit * a.id_stride + idx[e]] : idx[e];
        a.out_ids[(size_t)unit * a.k + pos] = id;
        if (a.out_ids2) a.out_ids2[(size_t)unit * a.k + pos] = id;
        ++pos;
      }
  }
}

// ---- host side ----------------------------------------------------------------
// Array source: smallest per-thread element count whose slice plan fits the merge kernels (512-thread
// workgroups).  More than 4096 survivors go through the middle level in groups of 2048 (k <= 2048) or 16384.
static bool plan_select_array(int n, int k, SelectPlan* plan) {
  static const int es[] = {4, 8, 16, 32};
  const long cap = (long)kSelNT * 32;  // what one workgroup can rank
  for (int e : es) {
    const int slice_len = kSelNT * e;
    const int n_slices = (n + slice_len - 1) / slice_len;
    const long per = k < slice_len ? k : slice_len;
    const long cand = (long)n_slices * per;
    *plan = SelectPlan{};
    plan->nt = plan->merge_nt = plan->mid_nt = kSelNT;
    plan->e = e; plan->slice_len = slice_len; plan->n_slices = n_slices;
    if (n_slices == 1) return true;
    auto fit = [](long c) { int me = 1; while ((long)kSelNT * me < c) me *= 2; return me; };
    // middle level (more than 4096 survivors): groups of whole slices, at most `cap` survivors in, k out
    if (cand > 4096) {
      long group = k <= 2048 ? 2048 : cap;
      group = group / per * per;
      const long n_groups = group > 0 ? (cand + group - 1) / group : 0;
      const long cand2 = n_groups * k;
      if (group >= 2 * per && n_groups >= 2 && cand2 <= 4096) {
        plan->group_cands = (int)group; plan->n_groups = (int)n_groups; plan->cand2_off = (int)cand;
        plan->cand_stride = (int)(cand + cand2);
        plan->mid_e = fit(group); plan->merge_e = fit(cand2);
        return true;
      }
    }
    if (cand <= cap) {
      plan->cand_stride = (int)cand; plan->merge_e = fit(cand);
      return true;
    }
  }
  return false;
}

// Logits source: one workgroup ranks up to 16384 slots without spilling registers (1024 threads x 16; 32768 with
// spills), so a unit of that size needs a single launch; small problems take 256 threads.  Longer units are cut
// into slices whose survivors (k each) are ranked by one more workgroup, through a middle level if even those
// exceed what one workgroup holds.  With few units the slices are made short (4096 or 8192 slots) so that more
// workgroups share the work, as long as one workgroup can still rank their survivors.
static void shape_for(long n, int* nt, int* e) {
  if (n <= 1024) { *nt = 256; *e = 4; return; }
  if (n <= 2048) { *nt = 256; *e = 8; return; }
  *nt = 1024; *e = 4;
  while ((long)*nt * *e < n) *e *= 2;
}
static bool plan_select_logits(int n, int k, int units, SelectPlan* plan) {
  const long cap = 1024l * 32, easy = 1024l * 16;
  *plan = SelectPlan{};
  if (n <= cap) {
    shape_for(n, &plan->nt, &plan->e);
    plan->slice_len = plan->nt * plan->e; plan->n_slices = 1;
    return true;
  }
  plan->nt = 1024; plan->e = 16;
  for (int e : {4, 8}) {   // shorter slices while the chip is far from full and the survivors stay easy to rank
    const long sl = 1024l * e, ns = (n + sl - 1) / sl;
    if ((long)units * ns <= 512 && ns * (k < sl ? k : sl) <= easy) { plan->e = e; break; }
  }
  plan->slice_len = plan->nt * plan->e;
  plan->n_slices = (n + plan->slice_len - 1) / plan->slice_len;
  const long per = k < plan->slice_len ? k : plan->slice_len;
  const long cand = (long)plan->n_slices * per;
  if (cand <= cap) {
    plan->cand_stride = (int)cand;
    shape_for(cand, &plan->merge_nt, &plan->merge_e);
    return true;
  }
  const long group = cap / per * per;   // whole slices per group
  if (group < 2 * per) return false;
  const long n_groups = (cand + group - 1) / group, cand2 = n_groups * k;
  if (cand2 > cap) return false;
  plan->group_cands = (int)group; plan->n_groups = (int)n_groups; plan->cand2_off = (int)cand;
  plan->cand_stride = (int)(cand + cand2);
  shape_for(group, &plan->mid_nt, &plan->mid_e);
  shape_for(cand2, &plan->merge_nt, &plan->merge_e);
  return true;
}

bool plan_select(int n, int k, int src, int units, SelectPlan* plan) {
  return src == kSrcLogits ? plan_select_logits(n, k, units, plan) : plan_select_array(n, k, plan);
}

static hipError_t launch_slices_array(const SelectArgs& a, int e, int units, hipStream_t st) {
  dim3 grid(a.n_slices, units), block(kSelNT);
  switch (e) {
    case 4: hipLaunchKernelGGL((select_slices<4>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((select_slices<8>), grid, block, 0, st, a); break;
    case 16: hipLaunchKernelGGL((select_slices<16>), grid, block, 0, st, a); break;
    case 32: hipLaunchKernelGGL((select_slices<32>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <bool MID>
static hipError_t launch_merge_array(const SelectArgs& a, int e, dim3 grid, hipStream_t st) {
  dim3 block(kSelNT);
  switch (e) {
    case 1: hipLaunchKernelGGL((select_merge<1, MID>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((select_merge<2, MID>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((select_merge<4, MID>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((select_merge<8, MID>), grid, block, 0, st, a); break;
    case 16: hipLaunchKernelGGL((select_merge<16, MID>), grid, block, 0, st, a); break;
    case 32: hipLaunchKernelGGL((select_merge<32, MID>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// the (threads, keys per thread) shapes shape_for() hands out
#define SKV_FOR_SHAPE(nt_, e_, WHAT)                                   \
  do {                                                                 \
    if ((nt_) == 256 && (e_) == 4) { WHAT(256, 4); }                   \
    else if ((nt_) == 256 && (e_) == 8) { WHAT(256, 8); }              \
    else if ((nt_) == 1024 && (e_) == 4) { WHAT(1024, 4); }            \
    else if ((nt_) == 1024 && (e_) == 8) { WHAT(1024, 8); }            \
    else if ((nt_) == 1024 && (e_) == 16) { WHAT(1024, 16); }          \
    else if ((nt_) == 1024 && (e_) == 32) { WHAT(1024, 32); }          \
    else return hipErrorInvalidValue;                                  \
  } while (0)

// The resident rows ride the selection only where that costs nothing: a single slice per unit ranked by 1024
// threads (one workgroup per compute unit), head dimension 128, and room on the chip for the extra workgroups.
bool resident_fits(const SelectPlan& plan, int units, int G, int d) {
  return plan.nt == 1024 && plan.e == 16 && plan.n_slices == 1 && d == 128 && (long)units * (1 + (G + 3) / 4) <= 256;
}
static hipError_t launch_slices_logits(const SelectArgs& a, int nt, int e, int units, hipStream_t st,
                                       const ResidentArgs* res, int kv_bytes) {
  if (res) {
    dim3 grid(units * (1 + res->head_blocks));
    if (kv_bytes == 1) hipLaunchKernelGGL((select_logits_kernel<1024, 16, 128, 1>), grid, dim3(1024), 0, st, a, *res);
    else hipLaunchKernelGGL((select_logits_kernel<1024, 16, 128, 2>), grid, dim3(1024), 0, st, a, *res);
    return hipGetLastError();
  }
  dim3 grid(a.n_slices, units);
  const ResidentArgs none{};
#define SKV_L(NT_, E_) hipLaunchKernelGGL((select_logits_kernel<NT_, E_>), grid, dim3(NT_), 0, st, a, none)
  SKV_FOR_SHAPE(nt, e, SKV_L);
#undef SKV_L
  return hipGetLastError();
}
template <bool MID>
static hipError_t launch_merge_logits(const SelectArgs& a, int nt, int e, dim3 grid, hipStream_t st) {
#define SKV_M(NT_, E_) hipLaunchKernelGGL((merge_logits_kernel<NT_, E_, MID>), grid, dim3(NT_), 0, st, a)
  SKV_FOR_SHAPE(nt, e, SKV_M);
#undef SKV_M
  return hipGetLastError();
}

hipError_t launch_select(const SelectArgs& a0, const SelectPlan& plan, int src, int units, hipStream_t st,
                         const ResidentArgs* res, int d, int kv_bytes) {
  if (res && (src != kSrcLogits || !resident_fits(plan, units, a0.G, d))) return hipErrorInvalidValue;
  SelectArgs a = a0;
  a.group_cands = plan.group_cands; a.n_groups = plan.n_groups; a.cand2_off = plan.cand2_off;
  const bool lg = src == kSrcLogits;
  hipError_t err = lg ? launch_slices_logits(a, plan.nt, plan.e, units, st, res, kv_bytes) : launch_slices_array(a, plan.e, units, st);
  if (err != hipSuccess || a.n_slices == 1) return err;
  if (plan.n_groups > 0) {
    err = lg ? launch_merge_logits<true>(a, plan.mid_nt, plan.mid_e, dim3(plan.n_groups, units), st)
             : launch_merge_array<true>(a, plan.mid_e, dim3(plan.n_groups, units), st);
    if (err != hipSuccess) return err;
  }
  return lg ? launch_merge_logits<false>(a, plan.merge_nt, plan.merge_e, dim3(units), st)
            : launch_merge_array<false>(a, plan.merge_e, dim3(units), st);
}

}  // namespace skv
