// Landmark scoring: P = Q L^T * scale for every landmark slot (first line of the
// decoding algorithm), streamed once from HBM for all heads of a KV group.
//
// The scores decide an index set that has to match an fp64 reference, so products
// (exact in fp32 for bf16 inputs) are accumulated in fp64 -- v_fma_f64 issues at the
// same rate as scalar fp32 FMA on this chip, and the kernel stays bound by the L read.
//
// Layout: 16 lanes share one landmark row (D/16 contiguous elements each), a wave
// covers 4 rows per load and 64 rows in all, a workgroup 256 rows.  Besides the
// logits the kernel leaves, per (head, tile), the pair (max, sum exp(p - max)) from
// which the selection kernel forms each head's log-sum-exp.
#include "kernels.hpp"

namespace skv {

template <int D, int GH>
__global__ __launch_bounds__(256) void score_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ L,
                                                    double* __restrict__ logits, double2* __restrict__ partials,
                                                    int hq, int hkv, int G, int n_c, int n_tiles, double scale) {
  constexpr int EPL = D / 16;
  __shared__ double sp[4][GH][kWave];
  __shared__ double2 wred[4][GH];
  const int unit = blockIdx.y, tile = blockIdx.x, g0 = blockIdx.z * GH;
  const int b = unit / hkv, h = unit % hkv;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int sub = lane & 15, rg = lane >> 4;
  const size_t head0 = (size_t)b * hq + (size_t)h * G + g0;

  double qv[GH][EPL];
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    float x[EPL];
    load_bf16_row<EPL>(q + (head0 + g) * D + sub * EPL, x);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qv[g][e] = (double)x[e];
  }

  const bf16_t* Lu = L + (size_t)unit * n_c * D;
  const int row0 = tile * kScoreTile + wave * kWave;
#pragma unroll 4
  for (int it = 0; it < 16; ++it) {
    const int rw = it * 4 + rg;
    const int row = row0 + rw;
    double acc[GH];
#pragma unroll
    for (int g = 0; g < GH; ++g) acc[g] = 0.0;
    if (row < n_c) {
      float x[EPL];
      load_bf16_row<EPL>(Lu + (size_t)row * D + sub * EPL, x);
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const double xd = (double)x[e];
#pragma unroll
        for (int g = 0; g < GH; ++g) acc[g] = fma(xd, qv[g][e], acc[g]);
      }
    }
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      const double t = sum16_f64(acc[g]);
      if (sub == g) sp[wave][g][rw] = row < n_c ? t * scale : -INFINITY;
    }
  }
  __syncthreads();

  // one lane per row from here on: coalesced logit stores, wave-wide (max, sum exp)
  const int row = row0 + lane;
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    const double p = sp[wave][g][lane];
    if (row < n_c) logits[(head0 + g) * n_c + row] = p;
    const double m = wave_max_f64(p);
    const double e = (row < n_c) ? exp(p - m) : 0.0;
    const double s = wave_sum_f64(e);
    if (lane == 0) wred[wave][g] = make_double2(m, s);
  }
  __syncthreads();
  if (threadIdx.x < GH) {
    const int g = threadIdx.x;
    double M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmax(M, wred[w][g].x);
    double S = 0.0;
#pragma unroll
    for (int w = 0; w < 4; ++w)
      if (wred[w][g].x != -INFINITY) S += wred[w][g].y * exp(wred[w][g].x - M);
    partials[(head0 + g) * n_tiles + tile] = make_double2(M, S);
  }
}

template <int D>
static hipError_t launch_score_d(const bf16_t* q, const bf16_t* L, double* logits, double2* partials, int batch,
                                 int hq, int hkv, int n_c, double scale, hipStream_t st) {
  const int G = hq / hkv;
  const int n_tiles = (n_c + kScoreTile - 1) / kScoreTile;
  const int gh = (G % 8 == 0) ? 8 : (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
  dim3 grid(n_tiles, batch * hkv, G / gh), block(256);
#define SKV_SCORE(GH_)                                                                                   \
  hipLaunchKernelGGL((score_kernel<D, GH_>), grid, block, 0, st, q, L, logits, partials, hq, hkv, G, n_c, \
                     n_tiles, scale)
  switch (gh) {
    case 8: SKV_SCORE(8); break;
    case 4: SKV_SCORE(4); break;
    case 2: SKV_SCORE(2); break;
    default: SKV_SCORE(1); break;
  }
#undef SKV_SCORE
  return hipGetLastError();
}

hipError_t launch_score(const bf16_t* q, const bf16_t* landmarks, double* logits, double2* partials, int batch,
                        int hq, int hkv, int d, int n_c, double scale, hipStream_t st) {
  switch (d) {
    case 64: return launch_score_d<64>(q, landmarks, logits, partials, batch, hq, hkv, n_c, scale, st);
    case 96: return launch_score_d<96>(q, landmarks, logits, partials, batch, hq, hkv, n_c, scale, st);
    case 128: return launch_score_d<128>(q, landmarks, logits, partials, batch, hq, hkv, n_c, scale, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace skv
