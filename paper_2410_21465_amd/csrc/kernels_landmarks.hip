// Pre-filling algorithm after the SVD: C = Reduce(K^RoPE) (chunk means),
// S = CosineSimilarity(C, K^RoPE), Min over each chunk -- one streaming pass over the
// post-RoPE keys -- then, once the o lowest chunks are known, L = C without them
// (ascending chunk order) and the gather of the outlier chunks' keys and values.
//
// chunk_stats: 16 lanes own one chunk (d/16 columns each, all c rows), so the mean needs
// no cross-lane traffic.  For c <= 8 the rows stay in registers (one pass over HBM).  The
// per-row dot products <mean, k_t> and squared norms are partial sums over a lane's columns;
// a transposed butterfly over the 16 lanes (DPP pairings xor 8, 7, 2, 1) leaves row t's dot
// in lane t and its squared norm in lane t+8, so each cosine -- an fp64 sqrt and divide -- is
// evaluated once, not 16 times.  Everything is fp64: the minimum cosine decides an index set
// against an fp64 reference.
#include "kernels.hpp"

namespace skv {

// 64-bit DPP move: value of the lane that the control word pairs this lane with (same 16-lane row)
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, false);
  return __hiloint2double(hi, lo);
}
constexpr int kDppXor8 = 0x128;  // row_ror:8
constexpr int kDppXor7 = 0x141;  // row_half_mirror: lane x <-> 7 - x inside each group of 8
constexpr int kDppXor2 = 0x4E;   // quad_perm [2,3,0,1]
constexpr int kDppXor1 = 0xB1;   // quad_perm [1,0,3,2]

__device__ __forceinline__ double allsum16_f64(double v) {
  v += dpp_f64<0x128>(v);
  v += dpp_f64<0x124>(v);
  v += dpp_f64<0x122>(v);
  v += dpp_f64<0x121>(v);
  return v;
}
__device__ __forceinline__ double allmin16_f64(double v) {
  v = fmin(v, dpp_f64<kDppXor8>(v));
  v = fmin(v, dpp_f64<kDppXor7>(v));
  v = fmin(v, dpp_f64<kDppXor2>(v));
  v = fmin(v, dpp_f64<kDppXor1>(v));
  return v;
}

// One butterfly stage: N values in, N/2 out.  Lanes whose selector bit is set keep the upper half.
template <int N, int CTRL>
__device__ __forceinline__ void scatter_stage(const double (&in)[N], double (&out)[N / 2], bool upper) {
#pragma unroll
  for (int i = 0; i < N / 2; ++i) {
    const double keep = upper ? in[N / 2 + i] : in[i];
    const double send = upper ? in[i] : in[N / 2 + i];
    out[i] = keep + dpp_f64<CTRL>(send);
  }
}
// Sum of v[i] over the 16 lanes of a row, delivered to lane i (i = lane % 16).
__device__ __forceinline__ double reduce_scatter16_f64(const double (&v)[16], int sub) {
  double a[8], b[4], c[2], d[1];
  scatter_stage<16, kDppXor8>(v, a, (sub & 8) != 0);
  scatter_stage<8, kDppXor7>(a, b, (sub & 4) != 0);
  scatter_stage<4, kDppXor2>(b, c, (sub & 2) != 0);
  scatter_stage<2, kDppXor1>(c, d, (sub & 1) != 0);
  return d[0];
}

// REG: the chunk's rows are kept in registers (c <= 8); otherwise they are read twice.
// EB: bytes per stored element (2 = bf16, 1 = FP8 E5M2); the means are written in the same type.
template <int D, bool REG, int EB>
__global__ __launch_bounds__(256) void chunk_stats_kernel(const uint8_t* __restrict__ k_rope,
                                                          uint8_t* __restrict__ chunk_mean,
                                                          double* __restrict__ chunk_min_cos, int s, int c,
                                                          int n_ch) {
  constexpr int EPL = D / 16;
  constexpr int RW = RawWords<EPL, EB>::n;
  const int unit = blockIdx.y;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int sub = lane & 15, cg = lane >> 4;
  const int j = blockIdx.x * 16 + wave * 4 + cg;
  const bool ok = j < n_ch;
  const uint8_t* base = k_rope + (((size_t)unit * s + (size_t)(ok ? j : 0) * c) * D + sub * EPL) * EB;

  uint32_t raw[REG ? 8 : 1][RW];
  double mean[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) mean[e] = 0.0;
  if constexpr (REG) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
#pragma unroll
      for (int e = 0; e < RW; ++e) raw[t][e] = 0u;   // all-zero bits are 0.0 in either type
      if (t < c) load_raw<EPL, EB>(base + (size_t)t * D * EB, raw[t]);
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      float x[EPL];
      unpack_kv<EPL, EB>(raw[t], x);
#pragma unroll
      for (int e = 0; e < EPL; ++e) mean[e] += (double)x[e];
    }
  } else {
    for (int t = 0; t < c; ++t) {
      float x[EPL];
      load_raw<EPL, EB>(base + (size_t)t * D * EB, raw[0]);
      unpack_kv<EPL, EB>(raw[0], x);
#pragma unroll
      for (int e = 0; e < EPL; ++e) mean[e] += (double)x[e];
    }
  }
  // sum / c: the multiplication by 1/c is exact (and identical to the division) when c is a power of two
  const bool pow2 = (c & (c - 1)) == 0;
  const double inv_c = 1.0 / (double)c;
  double cn2 = 0.0;
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    mean[e] = pow2 ? mean[e] * inv_c : mean[e] / (double)c;
    cn2 = fma(mean[e], mean[e], cn2);
  }
  const double cn = fmax(sqrt(allsum16_f64(cn2)), 1e-8);

  double mn = INFINITY;
  if constexpr (REG) {
    double v[16];  // v[t] = partial <mean, k_t>, v[8 + t] = partial |k_t|^2
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      double dot = 0.0, kn2 = 0.0;
      float x[EPL];
      unpack_kv<EPL, EB>(raw[t], x);
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const double xd = (double)x[e];
        dot = fma(mean[e], xd, dot);
        kn2 = fma(xd, xd, kn2);
      }
      v[t] = dot; v[8 + t] = kn2;
    }
    const double mine = reduce_scatter16_f64(v, sub);   // lane t: dot_t, lane 8+t: |k_t|^2
    const double kn2 = dpp_f64<kDppXor8>(mine);
    double cs = INFINITY;
    if (sub < c) cs = mine / (cn * fmax(sqrt(kn2), 1e-8));
    mn = allmin16_f64(cs);
  } else {
    for (int t = 0; t < c; ++t) {
      float x[EPL];
      load_raw<EPL, EB>(base + (size_t)t * D * EB, raw[0]);
      unpack_kv<EPL, EB>(raw[0], x);
      double dot = 0.0, kn2 = 0.0;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const double xd = (double)x[e];
        dot = fma(mean[e], xd, dot);
        kn2 = fma(xd, xd, kn2);
      }
      dot = allsum16_f64(dot);
      kn2 = allsum16_f64(kn2);
      mn = fmin(mn, dot / (cn * fmax(sqrt(kn2), 1e-8)));
    }
  }
  if (ok) {
    uint32_t hm[RW];
    pack_kv<EPL, EB>(mean, hm);
    store_raw<EPL, EB>(chunk_mean + (((size_t)unit * n_ch + j) * D + sub * EPL) * EB, hm);
    if (sub == 0) chunk_min_cos[(size_t)unit * n_ch + j] = mn;
  }
}

// L <- C \ Gather(C, I): landmark slot s -> chunk s + t, t = number of outliers i with id_i - i <= s
// (ids ascending), found by bisection.  A workgroup copies 128 consecutive slots.
template <int D, int EB>
__global__ __launch_bounds__(256) void compact_landmarks_kernel(const uint8_t* __restrict__ chunk_mean,
                                                                const int32_t* __restrict__ outlier_ids,
                                                                uint8_t* __restrict__ landmarks,
                                                                int32_t* __restrict__ landmark_chunk_ids, int n_ch,
                                                                int o, int nc_stride) {
  constexpr int EPL = D / 16;
  __shared__ int32_t oid[1024];
  const int unit = blockIdx.y, n_c = n_ch - o;
  for (int i = threadIdx.x; i < o; i += 256) oid[i] = outlier_ids[(size_t)unit * o + i] - i;
  __syncthreads();
  const int sub = threadIdx.x & 15;
#pragma unroll 2
  for (int it = 0; it < 8; ++it) {
    const int slot = blockIdx.x * 128 + it * 16 + (threadIdx.x >> 4);
    if (slot >= n_c) break;
    int lo = 0, hi = o;  // first index with oid[i] > slot
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (oid[mid] <= slot) lo = mid + 1; else hi = mid;
    }
    const int j = slot + lo;
    uint32_t row[RawWords<EPL, EB>::n];
    load_raw<EPL, EB>(chunk_mean + (((size_t)unit * n_ch + j) * D + sub * EPL) * EB, row);
    store_raw<EPL, EB>(landmarks + (((size_t)unit * nc_stride + slot) * D + sub * EPL) * EB, row);
    if (sub == 0) landmark_chunk_ids[(size_t)unit * nc_stride + slot] = j;
  }
}

__global__ __launch_bounds__(256) void gather_outliers_kernel(const uint4* __restrict__ k_rope,
                                                              const uint4* __restrict__ v,
                                                              const int32_t* __restrict__ outlier_ids,
                                                              uint4* __restrict__ k_outlier,
                                                              uint4* __restrict__ v_outlier, int o,
                                                              int vec_per_chunk, size_t vec_per_unit,
                                                              size_t vec_per_unit_v) {
  const int unit = blockIdx.y, i = blockIdx.x;
  const int last_chunk = (int)(vec_per_unit / vec_per_chunk) - 1;
  const int id = min(max(outlier_ids[(size_t)unit * o + i], 0), last_chunk);
  const size_t src = (size_t)unit * vec_per_unit + (size_t)id * vec_per_chunk;
  const size_t dst = ((size_t)unit * o + i) * vec_per_chunk;
  for (int x = threadIdx.x; x < vec_per_chunk; x += 256) {
    k_outlier[dst + x] = k_rope[src + x];
    if (v) v_outlier[dst + x] = v[(size_t)unit * vec_per_unit_v + (size_t)id * vec_per_chunk + x];
  }
}

hipError_t launch_chunk_stats(const void* k_rope, int kv_bytes, void* chunk_mean, double* chunk_min_cos, int units, int d,
                              int s, int c, hipStream_t st) {
  const int n_ch = s / c;
  dim3 grid((n_ch + 15) / 16, units), block(256);
  const uint8_t* kr = static_cast<const uint8_t*>(k_rope);
  uint8_t* cm = static_cast<uint8_t*>(chunk_mean);
#define SKV_STATS(D_, EB_)                                                                                         \
  do {                                                                                                             \
    if (c <= 8) hipLaunchKernelGGL((chunk_stats_kernel<D_, true, EB_>), grid, block, 0, st, kr, cm, chunk_min_cos, s, c, n_ch); \
    else hipLaunchKernelGGL((chunk_stats_kernel<D_, false, EB_>), grid, block, 0, st, kr, cm, chunk_min_cos, s, c, n_ch);       \
  } while (0)
  switch (d * 4 + kv_bytes) {
    case 64 * 4 + 2: SKV_STATS(64, 2); break;
    case 96 * 4 + 2: SKV_STATS(96, 2); break;
    case 128 * 4 + 2: SKV_STATS(128, 2); break;
    case 64 * 4 + 1: SKV_STATS(64, 1); break;
    case 96 * 4 + 1: SKV_STATS(96, 1); break;
    case 128 * 4 + 1: SKV_STATS(128, 1); break;
    default: return hipErrorInvalidValue;
  }
#undef SKV_STATS
  return hipGetLastError();
}

hipError_t launch_compact_landmarks(const void* chunk_mean, int kv_bytes, const int32_t* outlier_ids, void* landmarks,
                                    int32_t* landmark_chunk_ids, int units, int d, int n_ch, int o, int nc_stride,
                                    hipStream_t st) {
  const int n_c = n_ch - o;
  if (n_c <= 0) return hipSuccess;
  dim3 grid((n_c + 127) / 128, units), block(256);
  const uint8_t* cm = static_cast<const uint8_t*>(chunk_mean);
  uint8_t* lm = static_cast<uint8_t*>(landmarks);
#define SKV_COMPACT(D_, EB_)                                                                                     \
  hipLaunchKernelGGL((compact_landmarks_kernel<D_, EB_>), grid, block, 0, st, cm, outlier_ids, lm, landmark_chunk_ids, \
                     n_ch, o, nc_stride)
  switch (d * 4 + kv_bytes) {
    case 64 * 4 + 2: SKV_COMPACT(64, 2); break;
    case 96 * 4 + 2: SKV_COMPACT(96, 2); break;
    case 128 * 4 + 2: SKV_COMPACT(128, 2); break;
    case 64 * 4 + 1: SKV_COMPACT(64, 1); break;
    case 96 * 4 + 1: SKV_COMPACT(96, 1); break;
    case 128 * 4 + 1: SKV_COMPACT(128, 1); break;
    default: return hipErrorInvalidValue;
  }
#undef SKV_COMPACT
  return hipGetLastError();
}

hipError_t launch_gather_outliers(const void* k_rope, const void* v, int kv_bytes, const int32_t* outlier_ids,
                                  void* k_outlier, void* v_outlier, int units, int d, int s, int s_cap, int c,
                                  int o, hipStream_t st) {
  if (o <= 0) return hipSuccess;
  dim3 grid(o, units), block(256);
  hipLaunchKernelGGL(gather_outliers_kernel, grid, block, 0, st, reinterpret_cast<const uint4*>(k_rope),
                     reinterpret_cast<const uint4*>(v), outlier_ids, reinterpret_cast<uint4*>(k_outlier),
                     reinterpret_cast<uint4*>(v_outlier), o, c * d * kv_bytes / 16, (size_t)s * d * kv_bytes / 16,
                     (size_t)s_cap * d * kv_bytes / 16);
  return hipGetLastError();
}

}  // namespace skv
