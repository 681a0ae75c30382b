// Pre-filling algorithm after the SVD: C = Reduce(K^RoPE) (chunk means),
// S = CosineSimilarity(C, K^RoPE), Min over each chunk -- one streaming pass over the
// post-RoPE keys -- then, once the o lowest chunks are known, L = C without them
// (ascending chunk order) and the gather of the outlier chunks' keys and values.
//
// chunk_stats: 16 lanes own one chunk (d/16 columns each, all c rows), so the mean needs
// no cross-lane traffic; the per-token dot products and norms are reduced over the 16
// lanes in fp64 (the minimum cosine decides an index set against an fp64 reference).
#include "kernels.hpp"

namespace skv {

template <int D>
__global__ __launch_bounds__(256) void chunk_stats_kernel(const bf16_t* __restrict__ k_rope,
                                                          bf16_t* __restrict__ chunk_mean,
                                                          double* __restrict__ chunk_min_cos, int s, int c,
                                                          int n_ch) {
  constexpr int EPL = D / 16;
  const int unit = blockIdx.y;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int sub = lane & 15, cg = lane >> 4;
  const int j = blockIdx.x * 16 + wave * 4 + cg;
  const bool ok = j < n_ch;
  const bf16_t* base = k_rope + ((size_t)unit * s + (size_t)(ok ? j : 0) * c) * D + sub * EPL;

  double mean[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) mean[e] = 0.0;
  for (int t = 0; t < c; ++t) {
    float x[EPL];
    load_bf16_row<EPL>(base + (size_t)t * D, x);
#pragma unroll
    for (int e = 0; e < EPL; ++e) mean[e] += (double)x[e];
  }
  double cn2 = 0.0;
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    mean[e] = mean[e] / (double)c;
    cn2 = fma(mean[e], mean[e], cn2);
  }
  const double cn = fmax(sqrt(sum16_f64(cn2)), 1e-8);
  double mn = INFINITY;
  for (int t = 0; t < c; ++t) {
    float x[EPL];
    load_bf16_row<EPL>(base + (size_t)t * D, x);
    double dot = 0.0, kn2 = 0.0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const double xd = (double)x[e];
      dot = fma(mean[e], xd, dot);
      kn2 = fma(xd, xd, kn2);
    }
    dot = sum16_f64(dot);
    kn2 = sum16_f64(kn2);
    const double cs = dot / (cn * fmax(sqrt(kn2), 1e-8));
    mn = fmin(mn, cs);
  }
  if (ok) {
    bf16_t hm[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) hm[e] = f64_to_bf16(mean[e]);
    store_bf16_row<EPL>(chunk_mean + ((size_t)unit * n_ch + j) * D + sub * EPL, hm);
    if (sub == 0) chunk_min_cos[(size_t)unit * n_ch + j] = mn;
  }
}

// L <- C \ Gather(C, I): landmark slot -> the slot-th chunk that is not an outlier.
template <int D>
__global__ __launch_bounds__(256) void compact_landmarks_kernel(const bf16_t* __restrict__ chunk_mean,
                                                                const int32_t* __restrict__ outlier_ids,
                                                                bf16_t* __restrict__ landmarks,
                                                                int32_t* __restrict__ landmark_chunk_ids, int n_ch,
                                                                int o) {
  constexpr int EPL = D / 16;
  __shared__ int32_t oid[1024];
  const int unit = blockIdx.y, n_c = n_ch - o;
  for (int i = threadIdx.x; i < o; i += 256) oid[i] = outlier_ids[(size_t)unit * o + i];
  __syncthreads();
  const int sub = threadIdx.x & 15;
  const int slot = blockIdx.x * 16 + (threadIdx.x >> 4);
  if (slot >= n_c) return;
  int j = slot;
  for (int i = 0; i < o && oid[i] <= j; ++i) ++j;  // ids ascending: skip every outlier at or below j
  const bf16_t* src = chunk_mean + ((size_t)unit * n_ch + j) * D + sub * EPL;
  bf16_t* dst = landmarks + ((size_t)unit * n_c + slot) * D + sub * EPL;
  const uint32_t* s32 = reinterpret_cast<const uint32_t*>(src);
  uint32_t* d32 = reinterpret_cast<uint32_t*>(dst);
#pragma unroll
  for (int e = 0; e < EPL / 2; ++e) d32[e] = s32[e];
  if (sub == 0) landmark_chunk_ids[(size_t)unit * n_c + slot] = j;
}

__global__ __launch_bounds__(256) void gather_outliers_kernel(const uint4* __restrict__ k_rope,
                                                              const uint4* __restrict__ v,
                                                              const int32_t* __restrict__ outlier_ids,
                                                              uint4* __restrict__ k_outlier,
                                                              uint4* __restrict__ v_outlier, int o,
                                                              int vec_per_chunk, size_t vec_per_unit) {
  const int unit = blockIdx.y, i = blockIdx.x;
  const int last_chunk = (int)(vec_per_unit / vec_per_chunk) - 1;
  const int id = min(max(outlier_ids[(size_t)unit * o + i], 0), last_chunk);
  const size_t src = (size_t)unit * vec_per_unit + (size_t)id * vec_per_chunk;
  const size_t dst = ((size_t)unit * o + i) * vec_per_chunk;
  for (int x = threadIdx.x; x < vec_per_chunk; x += 256) {
    k_outlier[dst + x] = k_rope[src + x];
    if (v) v_outlier[dst + x] = v[src + x];
  }
}

hipError_t launch_chunk_stats(const bf16_t* k_rope, bf16_t* chunk_mean, double* chunk_min_cos, int units, int d,
                              int s, int c, hipStream_t st) {
  const int n_ch = s / c;
  dim3 grid((n_ch + 15) / 16, units), block(256);
  switch (d) {
    case 64: hipLaunchKernelGGL((chunk_stats_kernel<64>), grid, block, 0, st, k_rope, chunk_mean, chunk_min_cos, s, c, n_ch); break;
    case 96: hipLaunchKernelGGL((chunk_stats_kernel<96>), grid, block, 0, st, k_rope, chunk_mean, chunk_min_cos, s, c, n_ch); break;
    case 128: hipLaunchKernelGGL((chunk_stats_kernel<128>), grid, block, 0, st, k_rope, chunk_mean, chunk_min_cos, s, c, n_ch); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_compact_landmarks(const bf16_t* chunk_mean, const int32_t* outlier_ids, bf16_t* landmarks,
                                    int32_t* landmark_chunk_ids, int units, int d, int n_ch, int o, hipStream_t st) {
  const int n_c = n_ch - o;
  if (n_c <= 0) return hipSuccess;
  dim3 grid((n_c + 15) / 16, units), block(256);
  switch (d) {
    case 64: hipLaunchKernelGGL((compact_landmarks_kernel<64>), grid, block, 0, st, chunk_mean, outlier_ids, landmarks, landmark_chunk_ids, n_ch, o); break;
    case 96: hipLaunchKernelGGL((compact_landmarks_kernel<96>), grid, block, 0, st, chunk_mean, outlier_ids, landmarks, landmark_chunk_ids, n_ch, o); break;
    case 128: hipLaunchKernelGGL((compact_landmarks_kernel<128>), grid, block, 0, st, chunk_mean, outlier_ids, landmarks, landmark_chunk_ids, n_ch, o); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_gather_outliers(const bf16_t* k_rope, const bf16_t* v, const int32_t* outlier_ids,
                                  bf16_t* k_outlier, bf16_t* v_outlier, int units, int d, int s, int c, int o,
                                  hipStream_t st) {
  if (o <= 0) return hipSuccess;
  dim3 grid(o, units), block(256);
  hipLaunchKernelGGL(gather_outliers_kernel, grid, block, 0, st, reinterpret_cast<const uint4*>(k_rope),
                     reinterpret_cast<const uint4*>(v), outlier_ids, reinterpret_cast<uint4*>(k_outlier),
                     reinterpret_cast<uint4*>(v_outlier), o, c * d * 2 / 16, (size_t)s * d * 2 / 16);
  return hipGetLastError();
}

}  // namespace skv
