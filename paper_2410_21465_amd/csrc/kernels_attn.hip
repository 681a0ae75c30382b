// Softmax attention of each query head over K = [K_outlier ; RoPE(K_sparse) ; K_recent],
// V = [V_outlier ; V_sparse ; V_recent] (last lines of the decoding algorithm and the
// "standard attention computation for the top-k chunks and predefined outliers").
//
// Split-K flash-decode: the T attended tokens of a (batch, KV head) unit are cut into
// splits; one workgroup streams one split for up to 8 query heads of the GQA group at a
// time, so K and V rows are read once per group rather than once per head.  16 lanes
// share a token row (d/16 contiguous elements each); every lane keeps an online-softmax
// state (running max in log2 units, sum, d/16 output columns) per head, merged across
// the row groups by shuffles, across waves through LDS, and across splits by the small
// combine kernel.  Rebuilt keys arrive as fp32 (their bf16 rounding alone would use up
// most of the output tolerance); values of the selected chunks are read either from the
// staging buffer or in place from the HBM value store through the chunk ids.
#include "kernels.hpp"

namespace skv {

template <int ELEMS>
__device__ __forceinline__ void load_f32_row(const float* __restrict__ p, float (&x)[ELEMS]) {
  if constexpr (ELEMS == 8) {
    const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  } else if constexpr (ELEMS == 6) {
    const float2 a = reinterpret_cast<const float2*>(p)[0], b = reinterpret_cast<const float2*>(p)[1],
                 c = reinterpret_cast<const float2*>(p)[2];
    x[0] = a.x; x[1] = a.y; x[2] = b.x; x[3] = b.y; x[4] = c.x; x[5] = c.y;
  } else {
    const float4 a = reinterpret_cast<const float4*>(p)[0];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
  }
}

template <int D, int GH>
__global__ __launch_bounds__(256) void attn_split_kernel(AttnArgs a) {
  constexpr int EPL = D / 16;
  __shared__ float sm_acc[4][GH][D];
  __shared__ float sm_m[4][GH], sm_l[4][GH];
  const int unit = blockIdx.y, split = blockIdx.x, g0 = blockIdx.z * GH;
  const int G = a.hq / a.hkv, b = unit / a.hkv, h = unit % a.hkv;
  const size_t head0 = (size_t)b * a.hq + (size_t)h * G + g0;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int sub = lane & 15, rg = lane >> 4;
  const int oc = a.o * a.c, kc = a.k * a.c, T = oc + kc + a.w;
  const int i_begin = split * a.split_len;
  const int i_end = min(T, i_begin + a.split_len);

  float qv[GH][EPL];
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    float x[EPL];
    load_bf16_row<EPL>(a.q + (head0 + g) * D + sub * EPL, x);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qv[g][e] = x[e] * a.scale_log2;
  }
  float m[GH], l[GH], acc[GH][EPL];
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }

  const int n_iter = (i_end - i_begin + 15) / 16;
  for (int it = 0; it < n_iter; ++it) {
    const int i = i_begin + it * 16 + wave * 4 + rg;
    const bool ok = i < i_end;
    float kx[EPL], vx[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) { kx[e] = 0.f; vx[e] = 0.f; }
    if (ok) {
      if (i < oc) {
        const size_t row = (size_t)unit * oc + i;
        load_bf16_row<EPL>(a.k_outlier + row * D + sub * EPL, kx);
        load_bf16_row<EPL>(a.v_outlier + row * D + sub * EPL, vx);
      } else if (i < oc + kc) {
        const int j = i - oc;
        const size_t row = (size_t)unit * kc + j;
        load_f32_row<EPL>(a.k_sparse + row * D + sub * EPL, kx);
        if (a.v_sparse) {
          load_bf16_row<EPL>(a.v_sparse + row * D + sub * EPL, vx);
        } else {
          const int ch = j / a.c, t = j - ch * a.c;
          const int id = min(max(a.sel_ids[(size_t)unit * a.k + ch], 0), a.s / a.c - 1);
          const size_t tok = (size_t)id * a.c + t;
          load_bf16_row<EPL>(a.v_store + ((size_t)unit * a.s + tok) * D + sub * EPL, vx);
        }
      } else {
        const size_t row = (size_t)unit * a.w + (i - oc - kc);
        load_bf16_row<EPL>(a.k_local + row * D + sub * EPL, kx);
        load_bf16_row<EPL>(a.v_local + row * D + sub * EPL, vx);
      }
    }
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) dot = fmaf(kx[e], qv[g][e], dot);
      dot = sum16_f32(dot);
      if (ok) {
        const float mn = fmaxf(m[g], dot);
        const float corr = exp2f(m[g] - mn);
        const float p = exp2f(dot - mn);
        l[g] = l[g] * corr + p;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, vx[e], acc[g][e] * corr);
        m[g] = mn;
      }
    }
  }

  // merge the four row groups of the wave
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    float mt = fmaxf(m[g], __shfl_xor(m[g], 16, kWave));
    mt = fmaxf(mt, __shfl_xor(mt, 32, kWave));
    const float sc = (m[g] == -INFINITY) ? 0.f : exp2f(m[g] - mt);
    float lv = l[g] * sc;
    lv += __shfl_xor(lv, 16, kWave);
    lv += __shfl_xor(lv, 32, kWave);
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float v = acc[g][e] * sc;
      v += __shfl_xor(v, 16, kWave);
      v += __shfl_xor(v, 32, kWave);
      if (rg == 0) sm_acc[wave][g][sub * EPL + e] = v;
    }
    if (lane == 0) { sm_m[wave][g] = mt; sm_l[wave][g] = lv; }
  }
  __syncthreads();
  // merge the four waves and write this split's partial state
  for (int idx = threadIdx.x; idx < GH * D; idx += 256) {
    const int g = idx / D, e = idx - g * D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, sm_m[w][g]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float sc = (sm_m[w][g] == -INFINITY) ? 0.f : exp2f(sm_m[w][g] - M);
      num = fmaf(sm_acc[w][g][e], sc, num);
      den = fmaf(sm_l[w][g], sc, den);
    }
    const size_t pidx = (head0 + g) * a.n_splits + split;
    a.part_acc[pidx * D + e] = num;
    if (e == 0) a.part_ml[pidx] = make_float2(M, den);
  }
}

template <int D>
__global__ __launch_bounds__(D) void attn_combine_kernel(const float* __restrict__ part_acc,
                                                         const float2* __restrict__ part_ml,
                                                         bf16_t* __restrict__ out, int n_splits) {
  const size_t head = blockIdx.x;
  const int e = threadIdx.x;
  const float2* ml = part_ml + head * n_splits;
  float M = -INFINITY;
  for (int sp = 0; sp < n_splits; ++sp) M = fmaxf(M, ml[sp].x);
  float num = 0.f, den = 0.f;
  for (int sp = 0; sp < n_splits; ++sp) {
    const float sc = exp2f(ml[sp].x - M);
    num = fmaf(part_acc[(head * n_splits + sp) * D + e], sc, num);
    den = fmaf(ml[sp].y, sc, den);
  }
  out[head * D + e] = f32_to_bf16(num / den);
}

template <int D>
static hipError_t launch_attention_d(const AttnArgs& a, hipStream_t st) {
  const int G = a.hq / a.hkv;
  const int gh = (G % 8 == 0) ? 8 : (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
  dim3 grid(a.n_splits, a.batch * a.hkv, G / gh), block(256);
  switch (gh) {
    case 8: hipLaunchKernelGGL((attn_split_kernel<D, 8>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((attn_split_kernel<D, 4>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((attn_split_kernel<D, 2>), grid, block, 0, st, a); break;
    default: hipLaunchKernelGGL((attn_split_kernel<D, 1>), grid, block, 0, st, a); break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_combine_kernel<D>), dim3(a.batch * a.hq), dim3(D), 0, st, a.part_acc, a.part_ml, a.out,
                     a.n_splits);
  return hipGetLastError();
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t st) {
  switch (a.d) {
    case 64: return launch_attention_d<64>(a, st);
    case 96: return launch_attention_d<96>(a, st);
    case 128: return launch_attention_d<128>(a, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace skv
