// ArgTopK of the decoding algorithm (group score of every landmark slot -> k chunks)
// and of the pre-filling algorithm (lowest minimum cosine -> o outlier chunks).
//
// Two kernels: `select_slices` ranks one slice of NT*E candidates per workgroup and
// keeps min(k, slice) of them; `select_merge` ranks the survivors of all slices of a
// unit.  With a single slice the first kernel writes the final ids itself.
#include "kernels.hpp"
#include "select.hpp"
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
// NB of a lane's pairs are requested together (long contexts have many tiles per head).
template <int NB>
__device__ void unit_lse(const double2* __restrict__ part, int n_tiles, int G, double* lse_sm) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  for (int g = wave; g < G; g += kSelNT / kWave) {
    const double2* p = part + (size_t)g * n_tiles;
    double m = -INFINITY, s = 0.0;   // running (max, sum exp(. - max)) of this lane's tiles
    // tiles past the end read the last pair and count as empty; the pairs are folded in the order
    // lane, lane + 64, ... whatever the batching
    for (int t0 = lane; t0 < n_tiles; t0 += NB * kWave) {
      double2 v[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int t = t0 + u * kWave;
        v[u] = p[min(t, n_tiles - 1)];
        if (t >= n_tiles) v[u] = make_double2(-INFINITY, 0.0);
      }
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        if (v[u].x > m) { s = s * exp_neg_fast(m - v[u].x) + v[u].y; m = v[u].x; }
        else if (v[u].x != -INFINITY) s += v[u].y * exp_neg_fast(v[u].x - m);
      }
    }
    const double mw = wave_max_f64(m);
    s = (m == -INFINITY) ? 0.0 : s * exp_neg_fast(m - mw);
    s = wave_sum_f64(s);
    if (lane == 0) lse_sm[g] = mw + log(s);
  }
  __syncthreads();
}

// WIDE > 0: the variants for more than 4 query heads per KV head or more than 64 score tiles per head (they spend
// registers on loads in flight that the common case does not need).
template <int E, int SRC, int WIDE>
__global__ __launch_bounds__(kSelNT) void select_slices(SelectArgs a) {
  __shared__ SelectSmem<kSelNT> sm;
  __shared__ double lse_sm[64];
  const int unit = blockIdx.y, slice = blockIdx.x;
  const int base = slice * a.slice_len;
  const int n_here = min(a.slice_len, a.n - base);
  const int k_here = min(a.k, n_here);

  uint64_t key[E];
  if constexpr (SRC == kSrcLogits) {
    // the logits of the first heads are requested before the normalisers are formed (the two do not
    // depend on each other), the remaining heads of a large group afterwards
    constexpr int GP = 4;
    const double* lg = a.logits + (size_t)unit * a.G * a.n;
    const int j0 = base + threadIdx.x * E;
    double pre[GP][E];
#pragma unroll
    for (int g = 0; g < GP; ++g) {
      const double* row = lg + (size_t)min(g, a.G - 1) * a.n;
#pragma unroll
      for (int e = 0; e < E; ++e) pre[g][e] = row[min(j0 + e, a.n - 1)];
    }
    unit_lse<WIDE == 0 ? 1 : WIDE == 1 ? 4 : 8>(a.partials + (size_t)unit * a.G * a.n_tiles, a.n_tiles, a.G, lse_sm);
#pragma unroll
    for (int e = 0; e < E; ++e) key[e] = 0ull;
#pragma unroll
    for (int g = 0; g < GP; ++g) {
      if (g < a.G) {
        const double l = lse_sm[g];
#pragma unroll
        for (int e = 0; e < E; ++e)
          if (j0 + e < a.n) {
            const uint64_t kk = f64_key(pre[g][e] - l);
            key[e] = kk > key[e] ? kk : key[e];   // max over the heads of the group
          }
      }
    }
    // the remaining heads of a large group: with few keys per thread a batch of 32 logits is requested
    // before it is used; the wide variants have no registers to spare and take one head at a time
    constexpr int GB = WIDE == 0 ? 1 : E <= 4 ? (WIDE == 1 ? 4 : 12) : E <= 8 ? 4 : 1;
    for (int gb = GP; gb < a.G; gb += GB) {
      double more[GB][E];
#pragma unroll
      for (int g = 0; g < GB; ++g) {
        const double* row = lg + (size_t)min(gb + g, a.G - 1) * a.n;
#pragma unroll
        for (int e = 0; e < E; ++e) more[g][e] = GB > 1 ? row[min(j0 + e, a.n - 1)] : (j0 + e < a.n ? row[j0 + e] : 0.0);
      }
#pragma unroll
      for (int g = 0; g < GB; ++g) {
        if (gb + g < a.G) {
          const double l = lse_sm[gb + g];
#pragma unroll
          for (int e = 0; e < E; ++e)
            if (j0 + e < a.n) {
              const uint64_t kk = f64_key(more[g][e] - l);
              key[e] = kk > key[e] ? kk : key[e];
            }
        }
      }
    }
  } else {
    const double* sc = a.scores + (size_t)unit * a.n;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int j = base + threadIdx.x * E + e;
      key[e] = j < a.n ? f64_key(a.sign * sc[j]) : 0ull;
    }
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

// MID: one workgroup per (group of survivors, unit) keeps the k best of its group as new survivors;
// otherwise one workgroup per unit ranks the survivors (of the slices, or of the middle level) and
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
// Smallest per-thread element count whose slice plan fits the merge kernels.  More than 4096
// survivors go through the middle level in groups of 2048 (k <= 2048) or 16384.
bool plan_select(int n, int k, SelectPlan* plan) {
  static const int es[] = {4, 8, 16, 32};
  // tuning override: keys per thread of the slices (read once)
  static const int forced = [] { const char* ov = std::getenv("SHADOWKV_SELECT_E"); return ov ? std::atoi(ov) : 0; }();
  const long cap = (long)kSelNT * 32;  // what one workgroup can rank
  for (int e : es) {
    if (forced && e != forced && e != 32) continue;
    const int slice_len = kSelNT * e;
    const int n_slices = (n + slice_len - 1) / slice_len;
    const long per = k < slice_len ? k : slice_len;
    const long cand = (long)n_slices * per;
    *plan = SelectPlan{};
    plan->e = e; plan->slice_len = slice_len; plan->n_slices = n_slices;
    if (n_slices == 1) return true;
    auto fit = [](long c) { int me = 1; while ((long)kSelNT * me < c) me *= 2; return me; };
    // middle level (more than 4096 survivors): groups of whole slices, at most `cap` survivors in, k out
    if (cand > 4096 && !forced) {
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

template <int SRC, int WIDE>
static hipError_t launch_slices_w(const SelectArgs& a, int e, int units, hipStream_t st) {
  dim3 grid(a.n_slices, units), block(kSelNT);
  switch (e) {
    case 4: hipLaunchKernelGGL((select_slices<4, SRC, WIDE>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((select_slices<8, SRC, WIDE>), grid, block, 0, st, a); break;
    case 16: hipLaunchKernelGGL((select_slices<16, SRC, WIDE>), grid, block, 0, st, a); break;
    case 32: hipLaunchKernelGGL((select_slices<32, SRC, WIDE>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
template <int SRC>
static hipError_t launch_slices(const SelectArgs& a, int e, int units, hipStream_t st) {
  // 0: the common case; 1: 5 to 8 heads per KV head or more than 64 score tiles per head; 2: more than 8 heads
  if (SRC == kSrcLogits && a.G > 8) return launch_slices_w<SRC, 2>(a, e, units, st);
  if (SRC == kSrcLogits && (a.G > 4 || a.n_tiles > 64)) return launch_slices_w<SRC, 1>(a, e, units, st);
  return launch_slices_w<SRC, 0>(a, e, units, st);
}

template <bool MID>
static hipError_t launch_merge(const SelectArgs& a, int e, dim3 grid, hipStream_t st) {
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

hipError_t launch_select(const SelectArgs& a0, const SelectPlan& plan, int src, int units, hipStream_t st) {
  SelectArgs a = a0;
  a.group_cands = plan.group_cands; a.n_groups = plan.n_groups; a.cand2_off = plan.cand2_off;
  hipError_t err = src == kSrcLogits ? launch_slices<kSrcLogits>(a, plan.e, units, st)
                                     : launch_slices<kSrcArray>(a, plan.e, units, st);
  if (err != hipSuccess || a.n_slices == 1) return err;
  if (plan.n_groups > 0) {
    err = launch_merge<true>(a, plan.mid_e, dim3(plan.n_groups, units), st);
    if (err != hipSuccess) return err;
  }
  return launch_merge<false>(a, plan.merge_e, dim3(units), st);
}

}  // namespace skv
