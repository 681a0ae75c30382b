// Sparse attention of the decode step, fused with the key rebuild:
//   K = [K_outlier ; RoPE(Gather(A, I) B) ; K_recent],  V = [V_outlier ; Gather(V, I) ; V_recent],
//   out_g = softmax(q_g K^T * scale) V      (last lines of the decoding algorithm and the "standard
//   attention computation for the top-k chunks and predefined outliers").
//
// Split-K flash-decode.  The selected tokens of a (batch, KV head) unit are cut into splits; one
// workgroup owns one split plus an equal share of the unit's resident tokens (outliers, recent),
// for up to 4 query heads of the GQA group (8 made the kernel spill), so K and V are touched once per four heads.
//   * resident rows: K rows are read as stored (bf16);
//   * selected rows: the keys never exist in memory.  Each wave gathers 16 rows of A straight
//     into MFMA operand layout, multiplies by B^T staged in LDS (v_mfma_f32_16x16x32_bf16, fp32
//     accumulate), rotates the accumulators in registers (the RoPE partner i + d/2 of a column
//     sits in the same lane, d/32 column blocks away), and forms q.K from the same registers; a
//     16-lane DPP reduction gives every lane the logits of its rows.
// 16 lanes share a V row (d/16 columns each) and every lane keeps an online-softmax state
// (running max in log2 units, sum, its output columns) per head; states are merged across the
// four row groups of a wave by shuffles, across waves through LDS, across splits by the small
// combine kernel.  Keeping the rebuilt keys in fp32
// registers matters: rounding them to bf16 alone would use up most of the output tolerance.
// RoPE angle: position * frequency in fp64 revolutions, reduced to [-0.5, 0.5], then the
// hardware sin/cos of 2*pi*x -- accurate at positions beyond 2^20.  When the chunk size is a
// multiple of 4 the four rows a lane holds per tile are consecutive tokens: one such angle per
// tile and frequency is stepped by one position three times.
// Latency: the first token (and value row) of every chunk a split touches is staged in LDS once,
// and a wave requests the A rows and value rows of its next 16-row block before it works on the
// current one, with a fixed number of unconditional loads per block so that the wait before the
// MFMAs covers only the current block's loads.
// When the selected values are not readable yet (they are being gathered on another stream) the
// work is done in two kernels: this one with KEYS_ONLY (no selected value touched, logits stored),
// then sparse_values_kernel.
// Storage of the KV-cache tensors: EB = 2 bytes per element (bf16) or 1 (FP8 E5M2, section "Precision
// Sensitivity").  E5M2 elements are widened exactly -- to bf16 pairs for the matrix-core operands (the
// chip's own FP8 matrix instruction accumulates with about 16 bits, measured, against 24 of the bf16
// one, so it is not used), to fp32 for the vector work; the arithmetic after that is the same.
// This file holds the templates; kernels_attn.hip instantiates them for bf16, kernels_attn_fp8.hip for E5M2.
#pragma once
#include "kernels.hpp"

namespace skv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short bf16x4;

// Sum over the 16 lanes of a DPP row, result in every lane: four rotate-and-add steps, each a
// single VALU instruction with a DPP operand (row_ror:n), no LDS traffic.
template <int N>
__device__ __forceinline__ float row_ror_f32(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x120 + N, 0xf, 0xf, false));
}
// GH independent sums, interleaved so that no DPP operand was written by the instruction just before it.
template <int GH>
__device__ __forceinline__ void allsum16_vec(float (&v)[GH]) {
#pragma unroll
  for (int g = 0; g < GH; ++g) v[g] += row_ror_f32<8>(v[g]);
#pragma unroll
  for (int g = 0; g < GH; ++g) v[g] += row_ror_f32<4>(v[g]);
#pragma unroll
  for (int g = 0; g < GH; ++g) v[g] += row_ror_f32<2>(v[g]);
#pragma unroll
  for (int g = 0; g < GH; ++g) v[g] += row_ror_f32<1>(v[g]);
}

// 8 consecutive stored elements as the bf16x8 operand of the matrix instruction
template <int EB>
struct AFrag;
template <>
struct AFrag<2> {
  uint4 raw;
  __device__ __forceinline__ void load(const uint8_t* p) { raw = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ bf16x8 operand(bool zero) const {
    uint4 wv = zero ? make_uint4(0u, 0u, 0u, 0u) : raw;
    return *reinterpret_cast<bf16x8*>(&wv);
  }
};
template <>
struct AFrag<1> {
  uint2 raw;
  __device__ __forceinline__ void load(const uint8_t* p) { raw = *reinterpret_cast<const uint2*>(p); }
  __device__ __forceinline__ bf16x8 operand(bool zero) const {
    uint4 wv = make_uint4(e5m2x2_to_bf16x2<0>(raw.x), e5m2x2_to_bf16x2<1>(raw.x), e5m2x2_to_bf16x2<0>(raw.y),
                          e5m2x2_to_bf16x2<1>(raw.y));
    if (zero) wv = make_uint4(0u, 0u, 0u, 0u);
    return *reinterpret_cast<bf16x8*>(&wv);
  }
};

// Online-softmax state of one lane: NR rows at a time are folded in with one rescale per head.
template <int GH, int EPL, int EB>
struct OnlineSoftmax {
  float m[GH], l[GH], acc[GH][EPL];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }
  }
  // lg[row][g]: logits in log2 units, -inf for masked rows; vraw[row]: the lane's V columns (bf16 pairs)
  template <int NR>
  __device__ __forceinline__ void fold(const float (&lg)[NR][GH], const uint32_t (&vraw)[NR][RawWords<EPL, EB>::n]) {
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      float mn = m[g];
#pragma unroll
      for (int i = 0; i < NR; ++i) mn = fmaxf(mn, lg[i][g]);
      if (mn != -INFINITY) {
        const float corr = __builtin_amdgcn_exp2f(m[g] - mn);
        m[g] = mn;
        l[g] *= corr;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] *= corr;
      }
    }
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      float vx[EPL];
      unpack_kv<EPL, EB>(vraw[i], vx);
#pragma unroll
      for (int g = 0; g < GH; ++g) {
        // masked rows carry -inf and contribute exp2(-inf) = 0; a still-empty state uses 0 as reference
        const float p = __builtin_amdgcn_exp2f(lg[i][g] - (m[g] == -INFINITY ? 0.f : m[g]));
        l[g] += p;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, vx[e], acc[g][e]);
      }
    }
  }
};

// Value chunks copied by the first workgroups of the key-phase launch (see GatherArgs).  A zero-copy
// reader like gather_values_kernel: 16 bytes per lane, whole chunks contiguous, four independent loads in
// flight per thread; a fixed, small number of workgroups loops over the work, so that the rest of the chip
// is left to the key phase that runs beside it.
__device__ __forceinline__ void gather_chunks(const GatherArgs& g, int block) {
  constexpr int U = 4;  // loads in flight per thread
  const int vpc = g.vec_per_chunk;
  const int sub = block % g.blocks_per_unit;
  const int stride = g.blocks_per_unit * 256;
  for (int unit = block / g.blocks_per_unit; unit < g.units; unit += g.unit_step) {
    const int n_chunks = g.miss_slots ? min(max(g.n_miss[unit], 0), g.k) : g.k;
    const int total = n_chunks * vpc;
    const int32_t* ids = g.ids + (size_t)unit * (g.miss_slots ? g.slots_per_unit : g.k);
    const uint4* src_u = g.store + (size_t)unit * g.vec_per_unit_store;
    uint4* dst_u = g.dst + (size_t)unit * g.slots_per_unit * vpc;
    for (int v0 = sub * 256 + (int)threadIdx.x; v0 < total; v0 += stride * U) {
      // every load is issued (positions past the end repeat the first one and are not stored); named
      // variables rather than arrays, which the compiler kept in scratch memory here
      auto fetch = [&](int u, uint4& buf, int& at) {
        const int v = v0 + u * stride;
        const int vc = v < total ? v : v0;
        const int i = vc / vpc, off = vc - i * vpc;
        const int slot = g.miss_slots ? min(max(g.miss_slots[(size_t)unit * g.k + i], 0), g.slots_per_unit - 1) : i;
        buf = src_u[(size_t)min(max(ids[slot], 0), g.last_chunk) * vpc + off];
        at = v < total ? slot * vpc + off : -1;
      };
      uint4 b0, b1, b2, b3;
      int a0, a1, a2, a3;
      fetch(0, b0, a0); fetch(1, b1, a1); fetch(2, b2, a2); fetch(3, b3, a3);
      if (a0 >= 0) dst_u[a0] = b0;
      if (a1 >= 0) dst_u[a1] = b1;
      if (a2 >= 0) dst_u[a2] = b2;
      if (a3 >= 0) dst_u[a3] = b3;
    }
  }
}

// Attention of four query heads of one unit over the unit's resident rows [outliers ; recent] alone, by a whole
// workgroup of NT threads: the part of the decode step's attention that needs no selected chunk.  It can therefore
// run beside the selection (the first level of the selection rides a launch that leaves half the chip idle, and the
// extra workgroups of that launch call this), after which the attention kernel proper skips these rows.  Writes one
// partial state (m, l, acc[d]) per head at index `part_slot` of the head's n_part states.
// Heads past the group repeat its last head and are not written.  16 lanes share a row (d/16 columns each), a wave
// takes eight rows per step.
template <int D, int EB, int NT>
__device__ void resident_rows_attention(const ResidentArgs& r, int unit, int g0) {
  constexpr int GH = 4, EPL = D / 16, RW = RawWords<EPL, EB>::n, NW = NT / kWave;
  __shared__ float sm_acc[NW][GH][D];
  __shared__ float sm_m[NW][GH], sm_l[NW][GH];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int sub = lane & 15, rg = lane >> 4;
  const int G = r.hq / r.hkv, b = unit / r.hkv, h = unit % r.hkv;
  const size_t head0 = (size_t)b * r.hq + (size_t)h * G + g0;
  const int nv = min(GH, G - g0);
  const int n_res = r.oc + r.w;
  OnlineSoftmax<GH, EPL, EB> st;
  st.init();
  float qv[GH][EPL];
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    float x[EPL];
    load_bf16_row<EPL>(r.q + (head0 + min(g, nv - 1)) * D + sub * EPL, x);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qv[g][e] = x[e] * r.scale_log2;
  }
  for (int i0 = wave * 8; i0 < n_res; i0 += NW * 8) {
    uint32_t kraw[2][RW], vraw[2][RW];
    bool ok[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const int i = i0 + 4 * x + rg;
      ok[x] = i < n_res;
      const int ic = min(i, n_res - 1);
      const uint8_t *kp, *vp;
      if (ic < r.oc) {
        kp = static_cast<const uint8_t*>(r.k_outlier) + ((size_t)unit * r.oc + ic) * D * EB;
        vp = static_cast<const uint8_t*>(r.v_outlier) + ((size_t)unit * r.oc + ic) * D * EB;
      } else {
        kp = static_cast<const uint8_t*>(r.k_local) + ((size_t)unit * r.w + (ic - r.oc)) * D * EB;
        vp = static_cast<const uint8_t*>(r.v_local) + ((size_t)unit * r.w + (ic - r.oc)) * D * EB;
      }
      load_raw<EPL, EB>(kp + sub * EPL * EB, kraw[x]);
      load_raw<EPL, EB>(vp + sub * EPL * EB, vraw[x]);
    }
    float lg[2][GH];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      float kx[EPL], dot[GH];
      unpack_kv<EPL, EB>(kraw[x], kx);
#pragma unroll
      for (int g = 0; g < GH; ++g) {
        dot[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) dot[g] = fmaf(kx[e], qv[g][e], dot[g]);
      }
      allsum16_vec<GH>(dot);
#pragma unroll
      for (int g = 0; g < GH; ++g) lg[x][g] = ok[x] ? dot[g] : -INFINITY;
    }
    st.template fold<2>(lg, vraw);
  }
  // merge: row groups of the wave, then the waves of the workgroup
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    float mt = fmaxf(st.m[g], __shfl_xor(st.m[g], 16, kWave));
    mt = fmaxf(mt, __shfl_xor(mt, 32, kWave));
    const float sc = (st.m[g] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st.m[g] - mt);
    float lv = st.l[g] * sc;
    lv += __shfl_xor(lv, 16, kWave);
    lv += __shfl_xor(lv, 32, kWave);
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float v = st.acc[g][e] * sc;
      v += __shfl_xor(v, 16, kWave);
      v += __shfl_xor(v, 32, kWave);
      if (rg == 0) sm_acc[wave][g][sub * EPL + e] = v;
    }
    if (lane == 0) { sm_m[wave][g] = mt; sm_l[wave][g] = lv; }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < nv * D; idx += NT) {
    const int g = idx / D, e = idx - g * D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) M = fmaxf(M, sm_m[w][g]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float sc = (sm_m[w][g] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sm_m[w][g] - M);
      num = fmaf(sm_acc[w][g][e], sc, num);
      den = fmaf(sm_l[w][g], sc, den);
    }
    const size_t pidx = (head0 + g) * r.n_part + r.part_slot;
    r.part_acc[pidx * D + e] = num;
    if (e == 0) r.part_ml[pidx] = make_float2(M, den);
  }
}

// KSMAX = number of 32-wide rank steps the A prefetch buffer is sized for (5: r <= 160, 8: r <= 256).
// KEYS_ONLY: the selected values are still on their way (a gather on another stream).  The kernel
// then does everything that needs no selected value -- the resident rows in full, and for the
// selected rows the key rebuild, RoPE and q.K -- and leaves the logits of the selected rows in
// `logit_buf` for sparse_values_kernel, which runs once the values have arrived.
template <int D, int GH, int KSMAX, bool FAST4, bool KEYS_ONLY, int EB>
__global__ __launch_bounds__(256, 2) void sparse_attn_kernel(AttnArgs a) {
  constexpr int EPL = D / 16, NB = D / 16, HB = NB / 2;
  constexpr int RW = RawWords<EPL, EB>::n;
  constexpr int NT = FAST4 ? 1 : 4;  // token positions a lane keeps per block (FAST4: the first of 4 consecutive)
  extern __shared__ __align__(16) bf16_t Bt[];  // [D][rp], element (n, kk) = B[kk][n]; then int tokb[]
  __shared__ float sm_acc[4][GH][D];
  __shared__ float sm_m[4][GH], sm_l[4][GH];
  // KEYS_ONLY: a flat grid, the gather's workgroups first (they are dispatched first), then (split, unit, head block)
  // the unit is the fastest-varying index of the grid: workgroups go to the chip's eight XCDs in turn, so the
  // splits of a unit (same B, same chunk ids) meet in one XCD's L2 when the unit count is a multiple of 8
  int unit = blockIdx.x, split = blockIdx.y, g0 = blockIdx.z * GH;
  if constexpr (KEYS_ONLY) {
    if ((int)blockIdx.x < a.gather.n_blocks) {
      gather_chunks(a.gather, blockIdx.x);
      return;
    }
    const int idx = blockIdx.x - a.gather.n_blocks, units = a.batch * a.hkv;
    unit = idx % units;
    split = (idx / units) % a.n_splits;
    g0 = idx / (a.n_splits * units) * GH;
  }
  const int G = a.hq / a.hkv, b = unit / a.hkv, h = unit % a.hkv;
  const size_t head0 = (size_t)b * a.hq + (size_t)h * G + g0;
  const int nv = min(GH, G - g0);   // heads of this block that exist (the last block of a group may be partly empty:
                                    // its surplus heads repeat the last real one and are never written)
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform: keeps the row loops scalar
  const int sub = lane & 15, rg = lane >> 4;
  const int oc = a.o * a.c, kc = a.k * a.c;
  const int r = a.r, rp = a.rp, r32 = a.r32;
  const int s_begin = split * a.sparse_split_len;
  const int s_end = min(kc, s_begin + a.sparse_split_len);
  const int cshift = a.c_shift;  // log2(c) when c is a power of two, else -1
  auto chunk_of = [&](int i) { return cshift >= 0 ? i >> cshift : i / a.c; };
  const int ch_begin = chunk_of(s_begin);

  // ---- first token of every selected chunk this split touches, into LDS.  Ids are clamped: a bad id
  //      can never address outside A or V.
  //      Next to it the first row of the chunk's values inside the buffer they are read from: the store
  //      itself, the staged copy (chunk i at slot i), or a value cache (chunk i at slot v_slots[i]).
  int* tokb = reinterpret_cast<int*>(Bt + (size_t)D * rp);
  int* vrowb = tokb + (a.sparse_split_len / a.c + 2);
  const uint8_t* vbase = a.v_sparse ? static_cast<const uint8_t*>(a.v_sparse) + (size_t)unit * a.v_unit_rows * D * EB
                                    : static_cast<const uint8_t*>(a.v_store) + (size_t)unit * a.s_cap * D * EB;
  if (s_begin < s_end) {
    const int last_chunk = a.s / a.c - 1;
    const int32_t* ids = a.sel_ids + (size_t)unit * a.k;
    const int n_ch = chunk_of(s_end - 1) - ch_begin + 1;
    const int last_slot = a.v_unit_rows / a.c - 1;
    for (int idx = threadIdx.x; idx < n_ch; idx += 256) {
      const int tb = min(max(ids[ch_begin + idx], 0), last_chunk) * a.c;
      tokb[idx] = tb;
      int vb = tb;
      if (a.v_sparse) {
        const int slot = a.v_slots ? a.v_slots[(size_t)unit * a.k + ch_begin + idx] : ch_begin + idx;
        vb = min(max(slot, 0), last_slot) * a.c;
      }
      vrowb[idx] = vb;
    }
  }
  __syncthreads();

  // ---- one 16-row block of selected tokens: the lane's A row in MFMA operand layout (row = lane % 16)
  //      and the V slices of the four rows whose logits it will hold (accumulator layout: rows 4*(lane/16)+j).
  //      Rows past the end of the split are clamped onto its last rows; their logits are masked later.
  const int ksteps = r32 / 32;
  auto load_block = [&](int row0, AFrag<EB> (&af)[KSMAX], uint32_t (&vraw)[4][RW], int (&tok)[NT], bool (&okr)[NT]) {
    {
      const int i = min(row0 + sub, s_end - 1);
      const int ch = chunk_of(i);
      const size_t n = (size_t)(tokb[ch - ch_begin] + (i - ch * a.c));
      const uint8_t* arow = static_cast<const uint8_t*>(a.A) + ((size_t)b * a.s_cap + n) * r * EB;
      // every load is issued (a fixed number in flight per block); rank positions past r read the row's
      // last 8 elements instead and are zeroed when the block is taken up
#pragma unroll
      for (int ks = 0; ks < KSMAX; ++ks) {
        const int kk = ks * 32 + rg * 8;
        af[ks].load(arow + (size_t)min(kk, r - 8) * EB);
      }
    }
    if constexpr (FAST4) {
      const int i0 = row0 + rg * 4;
      okr[0] = i0 < s_end;
      const int ic = min(i0, s_end - 4);
      const int ch = chunk_of(ic);
      const int n0 = tokb[ch - ch_begin] + (ic - ch * a.c);
      tok[0] = n0;
      if constexpr (!KEYS_ONLY) {
        const uint8_t* vp = vbase + ((size_t)(vrowb[ch - ch_begin] + (ic - ch * a.c)) * D + sub * EPL) * EB;
#pragma unroll
        for (int j = 0; j < 4; ++j) load_raw<EPL, EB>(vp + (size_t)j * D * EB, vraw[j]);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = row0 + rg * 4 + j;
        okr[j] = i < s_end;
        const int ic = min(i, s_end - 1);
        const int ch = chunk_of(ic);
        const int n = tokb[ch - ch_begin] + (ic - ch * a.c);
        tok[j] = n;
        if constexpr (!KEYS_ONLY) {
          const uint8_t* vp = vbase + (size_t)(vrowb[ch - ch_begin] + (ic - ch * a.c)) * D * EB;
          load_raw<EPL, EB>(vp + sub * EPL * EB, vraw[j]);
        }
      }
    }
  };

  // first block of this wave: in flight while B^T is staged and the resident rows are processed
  AFrag<EB> afN[KSMAX];
  uint32_t vN[4][RW];
  int tokN[NT];
  bool okN[NT];
  if (s_begin < s_end) load_block(s_begin + wave * 16, afN, vN, tokN, okN);

  // ---- B^T of this KV head into LDS (zero beyond rank r).  A wave reads 16 rank rows x 64 bytes
  //      per load and scatters them as 16-bit LDS writes.
  {
    constexpr int NBI = (KSMAX * 32 * (D / 8) + 255) / 256;  // 16-byte pieces per thread
    const uint8_t* Bu = static_cast<const uint8_t*>(a.B) + (size_t)unit * r * D * EB;
    const int pieces = r32 * (D / 8);
    uint4 bw[NBI];
    int dst[NBI];
#pragma unroll
    for (int it = 0; it < NBI; ++it) {
      const int idx = min((int)threadIdx.x + it * 256, pieces - 1);
      const int n8 = (idx & 3) + 4 * (idx / (4 * r32)), kk = (idx >> 2) % r32;
      const uint8_t* src = Bu + ((size_t)min(kk, r - 1) * D + n8 * 8) * EB;
      if constexpr (EB == 2) {
        bw[it] = *reinterpret_cast<const uint4*>(src);
      } else {   // 8 bytes -> the same 8 elements as bf16 bit patterns
        const uint2 v = *reinterpret_cast<const uint2*>(src);
        bw[it] = make_uint4(v.x, v.y, 0u, 0u);
      }
      dst[it] = kk < r ? n8 * 8 * rp + kk : -(n8 * 8 * rp + kk) - 1;  // negative: store zeros
    }
    if constexpr (EB == 1) {
#pragma unroll
      for (int it = 0; it < NBI; ++it)
        bw[it] = make_uint4(e5m2x2_to_bf16x2<0>(bw[it].x), e5m2x2_to_bf16x2<1>(bw[it].x), e5m2x2_to_bf16x2<0>(bw[it].y),
                            e5m2x2_to_bf16x2<1>(bw[it].y));
    }
#pragma unroll
    for (int it = 0; it < NBI; ++it) {
      // (threads past the last piece repeat it: same values to the same place, no branch)
      const bool real = dst[it] >= 0;
      const int at = real ? dst[it] : -(dst[it] + 1);
      const uint32_t w4[4] = {real ? bw[it].x : 0u, real ? bw[it].y : 0u, real ? bw[it].z : 0u, real ? bw[it].w : 0u};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        Bt[at + (2 * i) * rp] = (bf16_t)(w4[i] & 0xffffu);
        Bt[at + (2 * i + 1) * rp] = (bf16_t)(w4[i] >> 16);
      }
    }
  }

  OnlineSoftmax<GH, EPL, EB> st;
  st.init();

  // ---------------- this split's share of the resident tokens: [outliers ; recent] ----------------
  {
    float qv[GH][EPL];
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      float x[EPL];
      load_bf16_row<EPL>(a.q + (head0 + min(g, nv - 1)) * D + sub * EPL, x);
#pragma unroll
      for (int e = 0; e < EPL; ++e) qv[g][e] = x[e] * a.scale_log2;
    }
    const int n_res = a.skip_resident ? 0 : oc + a.w;   // (skipped: another launch has attended over them)
    const int i_begin = min(n_res, split * a.res_split_len);
    const int i_end = min(n_res, i_begin + a.res_split_len);
    // two rows per lane group and step: rows i0 + rg and i0 + 4 + rg; the next step's rows are loaded
    // before the current ones are used
    auto load_res = [&](int i0, uint32_t (&kraw)[2][RW], uint32_t (&vraw)[2][RW], bool (&ok)[2]) {
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const int i = i0 + 4 * x + rg;
        ok[x] = i < i_end;
        const int ic = min(i, i_end - 1);
        const uint8_t *kp, *vp;
        if (ic < oc) {
          kp = static_cast<const uint8_t*>(a.k_outlier) + ((size_t)unit * oc + ic) * D * EB;
          vp = static_cast<const uint8_t*>(a.v_outlier) + ((size_t)unit * oc + ic) * D * EB;
        } else {
          kp = static_cast<const uint8_t*>(a.k_local) + ((size_t)unit * a.w + (ic - oc)) * D * EB;
          vp = static_cast<const uint8_t*>(a.v_local) + ((size_t)unit * a.w + (ic - oc)) * D * EB;
        }
        load_raw<EPL, EB>(kp + sub * EPL * EB, kraw[x]);
        load_raw<EPL, EB>(vp + sub * EPL * EB, vraw[x]);
      }
    };
    auto fold_res = [&](const uint32_t (&kraw)[2][RW], const uint32_t (&vraw)[2][RW], const bool (&ok)[2]) {
      float lg[2][GH];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        float kx[EPL], dot[GH];
        unpack_kv<EPL, EB>(kraw[x], kx);
#pragma unroll
        for (int g = 0; g < GH; ++g) {
          dot[g] = 0.f;
#pragma unroll
          for (int e = 0; e < EPL; ++e) dot[g] = fmaf(kx[e], qv[g][e], dot[g]);
        }
        allsum16_vec<GH>(dot);
#pragma unroll
        for (int g = 0; g < GH; ++g) lg[x][g] = ok[x] ? dot[g] : -INFINITY;
      }
      st.template fold<2>(lg, vraw);
    };
    if (i_begin < i_end) {
      uint32_t kN[2][RW], vN2[2][RW];
      bool okN2[2];
      load_res(i_begin + wave * 8, kN, vN2, okN2);
      for (int i0 = i_begin + wave * 8; i0 < i_end; i0 += 32) {
        uint32_t kC[2][RW], vC[2][RW];
        bool okC[2];
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          okC[x] = okN2[x];
#pragma unroll
          for (int e = 0; e < RW; ++e) { kC[x][e] = kN[x][e]; vC[x][e] = vN2[x][e]; }
        }
        load_res(i0 + 32, kN, vN2, okN2);  // rows past the end are clamped and masked
        fold_res(kC, vC, okC);
      }
    }
  }

  // ---------------- selected chunks: rebuild keys on the matrix cores ----------------
  {
    // q in accumulator-column layout (column nb*16 + sub), pre-scaled to log2 units
    float qc[GH][NB];
#pragma unroll
    for (int g = 0; g < GH; ++g)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        qc[g][nb] = bf16_to_f32(a.q[(head0 + min(g, nv - 1)) * D + nb * 16 + sub]) * a.scale_log2;
    double frev[HB];
#pragma unroll
    for (int nb = 0; nb < HB; ++nb) {
      const int f = nb * 16 + sub;
      frev[nb] = a.inv_freq_dev ? (double)a.inv_freq_dev[f] * 0.15915494309189533577 : a.freqs.rev[f];
    }
    const double pos0 = a.pos_offset ? (double)a.pos_offset[b] : 0.0;
    float cd[HB], sd[HB];  // one-position rotation step per frequency (FAST4)
    if constexpr (FAST4) {
#pragma unroll
      for (int nb = 0; nb < HB; ++nb) {
        double rv = frev[nb];
        rv -= rint(rv);
        cd[nb] = __builtin_amdgcn_cosf((float)rv);
        sd[nb] = __builtin_amdgcn_sinf((float)rv);
      }
    }
    __syncthreads();  // B^T is in place

    auto compute_block = [&](int row0, const bf16x8 (&af)[KSMAX], const uint32_t (&vraw)[4][RW],
                             const int (&tok)[NT], const bool (&okr)[NT]) {
      // -- K tile = A_sel * B on the matrix cores
      f32x4 acc[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KSMAX; ++ks) {
        if (ks < ksteps) {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(&Bt[(nb * 16 + sub) * rp + ks * 32 + rg * 8]);
            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[ks], bfrag, acc[nb], 0, 0, 0);
          }
        }
      }
      // -- RoPE and q.K row by row; the logits of the 4 rows x GH heads stay in registers
      float lg[4][GH];
      float cs[HB], sn[HB];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool ok = okr[FAST4 ? 0 : j];
        if (!FAST4 || j == 0) {
          const double pos = pos0 + (double)tok[FAST4 ? 0 : j];
#pragma unroll
          for (int nb = 0; nb < HB; ++nb) {
            double rev = pos * frev[nb];
            rev -= rint(rev);
            const float rv = (float)rev;  // revolutions in [-0.5, 0.5]
            sn[nb] = __builtin_amdgcn_sinf(rv);
            cs[nb] = __builtin_amdgcn_cosf(rv);
          }
        } else {
#pragma unroll
          for (int nb = 0; nb < HB; ++nb) {
            const float c1 = cs[nb] * cd[nb] - sn[nb] * sd[nb];
            sn[nb] = sn[nb] * cd[nb] + cs[nb] * sd[nb];
            cs[nb] = c1;
          }
        }
        float kr[NB];
#pragma unroll
        for (int nb = 0; nb < HB; ++nb) {
          const float x0 = acc[nb][j], x1 = acc[nb + HB][j];
          kr[nb] = x0 * cs[nb] - x1 * sn[nb];
          kr[nb + HB] = x1 * cs[nb] + x0 * sn[nb];
        }
        if (a.k_sparse_out && ok && g0 == 0) {
          float* orow = a.k_sparse_out + ((size_t)unit * kc + (row0 + rg * 4 + j)) * D;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) orow[nb * 16 + sub] = kr[nb];
        }
        float dot[GH];
#pragma unroll
        for (int g = 0; g < GH; ++g) {
          dot[g] = 0.f;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) dot[g] = fmaf(kr[nb], qc[g][nb], dot[g]);
        }
        allsum16_vec<GH>(dot);
#pragma unroll
        for (int g = 0; g < GH; ++g) lg[j][g] = ok ? dot[g] : -INFINITY;
      }
      if constexpr (KEYS_ONLY) {
        // rows 4*rg + j of the block: lane sub = j stores that row's logit for every head
        if (sub < 4) {
          const int i = row0 + rg * 4 + sub;
          if (i < s_end) {
#pragma unroll
            for (int g = 0; g < GH; ++g) {
              float v = lg[0][g];
#pragma unroll
              for (int j = 1; j < 4; ++j) v = sub == j ? lg[j][g] : v;
              if (g < nv) a.logit_buf[(head0 + g) * (size_t)kc + i] = v;
            }
          }
        }
      } else {
        st.template fold<4>(lg, vraw);
      }
    };

    // the four waves take 16-row blocks in turn; the next block of a wave is requested before the
    // current one is used (past the end of the split the request re-reads the split's last rows)
    for (int row0 = s_begin + wave * 16; row0 < s_end; row0 += 64) {
      bf16x8 afC[KSMAX];
      uint32_t vC[4][RW];
      int tokC[NT];
      bool okC[NT];
#pragma unroll
      for (int ks = 0; ks < KSMAX; ++ks) afC[ks] = afN[ks].operand(ks * 32 + rg * 8 >= r);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < RW; ++e) vC[j][e] = vN[j][e];
#pragma unroll
      for (int j = 0; j < NT; ++j) { tokC[j] = tokN[j]; okC[j] = okN[j]; }
      load_block(row0 + 64, afN, vN, tokN, okN);
      compute_block(row0, afC, vC, tokC, okC);
    }
  }

  // ---------------- merge: row groups of the wave, waves of the workgroup ----------------
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    float mt = fmaxf(st.m[g], __shfl_xor(st.m[g], 16, kWave));
    mt = fmaxf(mt, __shfl_xor(mt, 32, kWave));
    const float sc = (st.m[g] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st.m[g] - mt);
    float lv = st.l[g] * sc;
    lv += __shfl_xor(lv, 16, kWave);
    lv += __shfl_xor(lv, 32, kWave);
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float v = st.acc[g][e] * sc;
      v += __shfl_xor(v, 16, kWave);
      v += __shfl_xor(v, 32, kWave);
      if (rg == 0) sm_acc[wave][g][sub * EPL + e] = v;
    }
    if (lane == 0) { sm_m[wave][g] = mt; sm_l[wave][g] = lv; }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < nv * D; idx += 256) {
    const int g = idx / D, e = idx - g * D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, sm_m[w][g]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float sc = (sm_m[w][g] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sm_m[w][g] - M);
      num = fmaf(sm_acc[w][g][e], sc, num);
      den = fmaf(sm_l[w][g], sc, den);
    }
    const size_t pidx = (head0 + g) * a.n_part + split;
    a.part_acc[pidx * D + e] = num;
    if (e == 0) a.part_ml[pidx] = make_float2(M, den);
  }
}

// The fused kernel again, with the work of a block of selected rows divided between two kinds of waves (NKW waves
// rebuild keys, NVW waves attend), for groups of four query heads and chunk sizes that are
// multiples of four.  The single-role kernel above keeps per lane the A fragments, the MFMA accumulators, the
// rotation state, the queries, the value rows AND the online-softmax state of four heads: 242 registers, two waves
// per SIMD, each going through all phases of a block in turn, and it moves the scattered 2-2.5 KB pieces of A and V
// at 3.1-3.7 TB/s where the bare gather reaches 5.4 TB/s.  Here
//   * a key wave owns 16 rows per step: A rows -> MFMA (B^T in LDS) -> RoPE in place -> q.K (queries from LDS, two
//     heads at a time) -> the 16 x 4 logits into a two-deep ring in LDS; the A rows of its next block are requested
//     before it starts on the current one (two sets of fragments);
//   * a value wave takes the blocks that key waves vw, vw + NVW, ... produced one step earlier: logits from the ring,
//     value rows requested two blocks ahead (they depend on nothing but the selection), online softmax, P.V on the
//     matrix cores;
//     it also takes this split's share of the resident rows first, when no other launch has done them;
//   * one barrier per step orders the ring.
// Each role fits 128 registers, so 16 waves share a compute unit: 12 key + 4 value waves in one 1024-thread
// workgroup per compute unit (with softmax x V on the matrix cores a value wave keeps up with three key waves;
// waves i and i + 4 of a workgroup share a SIMD, so every SIMD gets three key waves and one value wave).
template <int D, int KSMAX, int EB, int ABUF, int NKW, int NVW>
__global__ __launch_bounds__(64 * (NKW + NVW), 4) void sparse_attn_roles_kernel(AttnArgs a) {
  constexpr int GH = 4, EPL = D / 16, NB = D / 16, HB = NB / 2;
  constexpr int RW = RawWords<EPL, EB>::n;
  constexpr int NT = 64 * (NKW + NVW), RPS = 16 * NKW, BPV = NKW / NVW;   // threads; rows per step; blocks per value wave and step
  static_assert(NKW % NVW == 0, "every value wave takes the same number of blocks per step");
  extern __shared__ __align__(16) bf16_t Bt[];  // [D][rp], element (n, kk) = B[kk][n]; then int tokb[], vrowb[]
  __shared__ __align__(16) float lgs[2][RPS][GH]; // logits (log2 units) of the rows of one step, -inf past the end
  __shared__ __align__(16) float qs[GH][D];       // the block's queries, scaled to log2 units
  __shared__ double frev_s[D / 2];                // rotary frequencies in revolutions per position
  __shared__ float cd_s[D / 2], sd_s[D / 2];      // cos / sin of one position step
  __shared__ float sm_acc[NVW][GH][D];
  __shared__ float sm_m[NVW][GH], sm_l[NVW][GH];
  const int unit = blockIdx.x, split = blockIdx.y, g0 = blockIdx.z * GH;
  const int G = a.hq / a.hkv, b = unit / a.hkv, h = unit % a.hkv;
  const size_t head0 = (size_t)b * a.hq + (size_t)h * G + g0;
  const int nv = min(GH, G - g0);
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int sub = lane & 15, rg = lane >> 4;
  const int oc = a.o * a.c, kc = a.k * a.c;
  const int r = a.r, rp = a.rp, r32 = a.r32;
  const int s_begin = split * a.sparse_split_len;
  const int s_end = min(kc, s_begin + a.sparse_split_len);
  const int cshift = a.c_shift;
  auto chunk_of = [&](int i) { return cshift >= 0 ? i >> cshift : i / a.c; };
  const int ch_begin = chunk_of(s_begin);
  const int n_it = (s_end - s_begin + RPS - 1) / RPS;

  int* tokb = reinterpret_cast<int*>(Bt + (size_t)D * rp);
  int* vrowb = tokb + (a.sparse_split_len / a.c + 2);
  const uint8_t* vbase = a.v_sparse ? static_cast<const uint8_t*>(a.v_sparse) + (size_t)unit * a.v_unit_rows * D * EB
                                    : static_cast<const uint8_t*>(a.v_store) + (size_t)unit * a.s_cap * D * EB;
  if (s_begin < s_end) {
    const int last_chunk = a.s / a.c - 1;
    const int32_t* ids = a.sel_ids + (size_t)unit * a.k;
    const int n_ch = chunk_of(s_end - 1) - ch_begin + 1;
    const int last_slot = a.v_unit_rows / a.c - 1;
    for (int idx = threadIdx.x; idx < n_ch; idx += NT) {
      const int tb = min(max(ids[ch_begin + idx], 0), last_chunk) * a.c;
      tokb[idx] = tb;
      int vb = tb;
      if (a.v_sparse) {
        const int slot = a.v_slots ? a.v_slots[(size_t)unit * a.k + ch_begin + idx] : ch_begin + idx;
        vb = min(max(slot, 0), last_slot) * a.c;
      }
      vrowb[idx] = vb;
    }
  }
  for (int idx = threadIdx.x; idx < GH * D; idx += NT) {
    const int g = idx / D, e = idx - g * D;
    qs[g][e] = bf16_to_f32(a.q[(head0 + min(g, nv - 1)) * D + e]) * a.scale_log2;
  }
  if (threadIdx.x < D / 2) {
    double rv = a.inv_freq_dev ? (double)a.inv_freq_dev[threadIdx.x] * 0.15915494309189533577 : a.freqs.rev[threadIdx.x];
    frev_s[threadIdx.x] = rv;
    rv -= rint(rv);
    cd_s[threadIdx.x] = __builtin_amdgcn_cosf((float)rv);
    sd_s[threadIdx.x] = __builtin_amdgcn_sinf((float)rv);
  }
  // ---- B^T of this KV head into LDS (zero beyond rank r), by all the waves
  {
    constexpr int NBI = (KSMAX * 32 * (D / 8) + NT - 1) / NT;  // 16-byte pieces per thread
    const uint8_t* Bu = static_cast<const uint8_t*>(a.B) + (size_t)unit * r * D * EB;
    const int pieces = r32 * (D / 8);
    uint4 bw[NBI];
    int dst[NBI];
#pragma unroll
    for (int it = 0; it < NBI; ++it) {
      const int idx = min((int)threadIdx.x + it * NT, pieces - 1);
      const int n8 = (idx & 3) + 4 * (idx / (4 * r32)), kk = (idx >> 2) % r32;
      const uint8_t* src = Bu + ((size_t)min(kk, r - 1) * D + n8 * 8) * EB;
      if constexpr (EB == 2) {
        bw[it] = *reinterpret_cast<const uint4*>(src);
      } else {
        const uint2 v = *reinterpret_cast<const uint2*>(src);
        bw[it] = make_uint4(v.x, v.y, 0u, 0u);
      }
      dst[it] = kk < r ? n8 * 8 * rp + kk : -(n8 * 8 * rp + kk) - 1;  // negative: store zeros
    }
    if constexpr (EB == 1) {
#pragma unroll
      for (int it = 0; it < NBI; ++it)
        bw[it] = make_uint4(e5m2x2_to_bf16x2<0>(bw[it].x), e5m2x2_to_bf16x2<1>(bw[it].x), e5m2x2_to_bf16x2<0>(bw[it].y),
                            e5m2x2_to_bf16x2<1>(bw[it].y));
    }
#pragma unroll
    for (int it = 0; it < NBI; ++it) {
      const bool real = dst[it] >= 0;
      const int at = real ? dst[it] : -(dst[it] + 1);
      const uint32_t w4[4] = {real ? bw[it].x : 0u, real ? bw[it].y : 0u, real ? bw[it].z : 0u, real ? bw[it].w : 0u};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        Bt[at + (2 * i) * rp] = (bf16_t)(w4[i] & 0xffffu);
        Bt[at + (2 * i + 1) * rp] = (bf16_t)(w4[i] >> 16);
      }
    }
  }
  __syncthreads();   // tables, queries and B^T are in place

  if (wave < NKW) {
    // =========================== key waves ===========================
    const int kw = wave;
    const int ksteps = r32 / 32;
    const double pos0 = a.pos_offset ? (double)a.pos_offset[b] : 0.0;
    // two sets of A fragments: the rows of the next block are requested before the current block is worked on
    AFrag<EB> afA[KSMAX], afB[KSMAX];
    int tokA = 0, tokB = 0;
    auto load_a = [&](int row0, AFrag<EB> (&af)[KSMAX], int& tok0) {
      const int i = min(row0 + sub, s_end - 1);
      const int ch = chunk_of(i);
      const size_t n = (size_t)(tokb[ch - ch_begin] + (i - ch * a.c));
      const uint8_t* arow = static_cast<const uint8_t*>(a.A) + ((size_t)b * a.s_cap + n) * r * EB;
#pragma unroll
      for (int ks = 0; ks < KSMAX; ++ks) af[ks].load(arow + (size_t)min(ks * 32 + rg * 8, r - 8) * EB);
      const int ic = min(row0 + rg * 4, s_end - 4);   // first of this lane's four consecutive tokens
      const int ch4 = chunk_of(ic);
      tok0 = tokb[ch4 - ch_begin] + (ic - ch4 * a.c);
    };
    auto work = [&](int it, AFrag<EB> (&af)[KSMAX], int& tok_af) {
      const int row0 = s_begin + it * RPS + kw * 16;
      const int tok_cur = tok_af;
      f32x4 acc[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KSMAX; ++ks) {
        if (ks < ksteps) {
          const bf16x8 afrag = af[ks].operand(ks * 32 + rg * 8 >= r);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(&Bt[(nb * 16 + sub) * rp + ks * 32 + rg * 8]);
            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, bfrag, acc[nb], 0, 0, 0);
          }
        }
      }
      if (ABUF == 1 && it + 1 < n_it) load_a(row0 + RPS, af, tok_af);   // one set of fragments: consumed, so reload
      // RoPE in place: one accurate angle per frequency for the first of the lane's four tokens, stepped by
      // one position for the others
      {
        float cs[HB], sn[HB];
        const double pos = pos0 + (double)tok_cur;
#pragma unroll
        for (int nb = 0; nb < HB; ++nb) {
          double rev = pos * frev_s[nb * 16 + sub];
          rev -= rint(rev);
          const float rv = (float)rev;
          sn[nb] = __builtin_amdgcn_sinf(rv);
          cs[nb] = __builtin_amdgcn_cosf(rv);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (j > 0) {
#pragma unroll
            for (int nb = 0; nb < HB; ++nb) {
              const float cd = cd_s[nb * 16 + sub], sd = sd_s[nb * 16 + sub];
              const float c1 = cs[nb] * cd - sn[nb] * sd;
              sn[nb] = sn[nb] * cd + cs[nb] * sd;
              cs[nb] = c1;
            }
          }
#pragma unroll
          for (int nb = 0; nb < HB; ++nb) {
            const float x0 = acc[nb][j], x1 = acc[nb + HB][j];
            acc[nb][j] = x0 * cs[nb] - x1 * sn[nb];
            acc[nb + HB][j] = x1 * cs[nb] + x0 * sn[nb];
          }
        }
      }
      // q.K, two heads at a time; lane sub == 0 of a row group stores the logits of its four rows
#pragma unroll
      for (int hp = 0; hp < GH / 2; ++hp) {
        float qv[2][NB];
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) qv[g][nb] = qs[2 * hp + g][nb * 16 + sub];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float dot[2] = {0.f, 0.f};
#pragma unroll
          for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) dot[g] = fmaf(acc[nb][j], qv[g][nb], dot[g]);
          allsum16_vec<2>(dot);
          if (sub == 0) {
            const bool ok = row0 + rg * 4 + j < s_end;
            float2 v = make_float2(dot[0], dot[1]);
            if (!ok) v = make_float2(-INFINITY, -INFINITY);
            *reinterpret_cast<float2*>(&lgs[it & 1][kw * 16 + rg * 4 + j][2 * hp]) = v;
          }
        }
      }
    };
    // (blocks that start past the end of the split are skipped by both kinds of waves)
    if (n_it > 0) load_a(s_begin + kw * 16, afA, tokA);
    if constexpr (ABUF == 1) {
      for (int it = 0; it <= n_it; ++it) {
        if (it < n_it && s_begin + it * RPS + kw * 16 < s_end) work(it, afA, tokA);
        __syncthreads();
      }
    } else {
      for (int it = 0; it <= n_it; it += 2) {
        if (it < n_it) {
          if (it + 1 < n_it) load_a(s_begin + (it + 1) * RPS + kw * 16, afB, tokB);
          if (s_begin + it * RPS + kw * 16 < s_end) work(it, afA, tokA);
        }
        __syncthreads();
        if (it + 1 <= n_it) {
          if (it + 1 < n_it) {
            if (it + 2 < n_it) load_a(s_begin + (it + 2) * RPS + kw * 16, afA, tokA);
            if (s_begin + (it + 1) * RPS + kw * 16 < s_end) work(it + 1, afB, tokB);
          }
          __syncthreads();
        }
      }
    }
    __syncthreads();   // (pairs with the value waves' barrier before the merge)
    return;
  }

  // =========================== value waves ===========================
  const int vw = wave - NKW;
  OnlineSoftmax<GH, EPL, EB> st;
  st.init();
  auto load_v = [&](int row0, uint32_t (&vraw)[4][RW]) {
    const int ic = min(row0 + rg * 4, s_end - 4);
    const int ch = chunk_of(ic);
    const uint8_t* vp = vbase + ((size_t)(vrowb[ch - ch_begin] + (ic - ch * a.c)) * D + sub * EPL) * EB;
#pragma unroll
    for (int j = 0; j < 4; ++j) load_raw<EPL, EB>(vp + (size_t)j * D * EB, vraw[j]);
  };
  // ---- this split's share of the resident rows [outliers ; recent], unless another launch has done them
  if (!a.skip_resident) {
    float qv[GH][EPL];
#pragma unroll
    for (int g = 0; g < GH; ++g)
#pragma unroll
      for (int e = 0; e < EPL; ++e) qv[g][e] = qs[g][sub * EPL + e];
    const int n_res = oc + a.w;
    const int i_begin = min(n_res, split * a.res_split_len);
    const int i_end = min(n_res, i_begin + a.res_split_len);
    for (int i0 = i_begin + vw * 8; i0 < i_end; i0 += 8 * NVW) {
      uint32_t kraw[2][RW], vraw[2][RW];
      bool ok[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const int i = i0 + 4 * x + rg;
        ok[x] = i < i_end;
        const int ic = min(i, i_end - 1);
        const uint8_t *kp, *vp;
        if (ic < oc) {
          kp = static_cast<const uint8_t*>(a.k_outlier) + ((size_t)unit * oc + ic) * D * EB;
          vp = static_cast<const uint8_t*>(a.v_outlier) + ((size_t)unit * oc + ic) * D * EB;
        } else {
          kp = static_cast<const uint8_t*>(a.k_local) + ((size_t)unit * a.w + (ic - oc)) * D * EB;
          vp = static_cast<const uint8_t*>(a.v_local) + ((size_t)unit * a.w + (ic - oc)) * D * EB;
        }
        load_raw<EPL, EB>(kp + sub * EPL * EB, kraw[x]);
        load_raw<EPL, EB>(vp + sub * EPL * EB, vraw[x]);
      }
      float lg[2][GH];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        float kx[EPL], dot[GH];
        unpack_kv<EPL, EB>(kraw[x], kx);
#pragma unroll
        for (int g = 0; g < GH; ++g) {
          dot[g] = 0.f;
#pragma unroll
          for (int e = 0; e < EPL; ++e) dot[g] = fmaf(kx[e], qv[g][e], dot[g]);
        }
        allsum16_vec<GH>(dot);
#pragma unroll
        for (int g = 0; g < GH; ++g) lg[x][g] = ok[x] ? dot[g] : -INFINITY;
      }
      st.template fold<2>(lg, vraw);
    }
  }
  // ---- selected rows: softmax x V on the matrix cores.
  // out[head][col] += sum_rows p[row][head] V[row][col] per block of 16 rows is a 16x16x16 product per output
  // column block, with the heads (padded from 4 to 16) as the rows of the left operand: lane (sub, rg) supplies
  // p of head sub for rows 4 rg .. 4 rg + 3 (only sub < 4 is real; the other lanes repeat head sub & 3 and feed
  // output rows nobody reads) and V of rows 4 rg .. 4 rg + 3 at ONE column.  Which column an operand lane stands
  // for is free as long as the output is read the same way: taking element e of the lane's EPL contiguous columns
  // for product number e, the lane's row pieces are used as loaded (a byte permute gathers element e of the four
  // rows), and lanes rg == 0 end up with out[head i][sub * EPL + e] in oacc[e][i] -- the columns they own in the
  // vector form as well.  p is fed as two bf16 terms (the top 16 bits of the fp32 value, 2^-16 relative), V is
  // bf16 as stored (E5M2 widens exactly).  The running maximum of every head is kept in every lane; the sum of p
  // in the lanes sub < 4 for the rows they fed.
  f32x4 oacc[EPL];
  float mh[GH], lpart = 0.f;
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    // what the resident rows left in the vector form: common maximum, sums over the row groups
    float mt = fmaxf(st.m[g], __shfl_xor(st.m[g], 16, kWave));
    mt = fmaxf(mt, __shfl_xor(mt, 32, kWave));
    const float sc = (st.m[g] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st.m[g] - mt);
    float lv = st.l[g] * sc;
    lv += __shfl_xor(lv, 16, kWave);
    lv += __shfl_xor(lv, 32, kWave);
    mh[g] = mt;
    if (rg == 0 && sub == g) lpart = lv;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float v = st.acc[g][e] * sc;
      v += __shfl_xor(v, 16, kWave);
      v += __shfl_xor(v, 32, kWave);
      oacc[e][g] = rg == 0 ? v : 0.f;
    }
  }
  {
    uint32_t v0[4][RW], v1[4][RW];
    const int hsel = sub & 3;   // the head whose weights this lane forms
    // this wave's blocks in the order it meets them: number q is block vw + (q % BPV) * NVW of step q / BPV
    const int n_q = n_it * BPV;
    auto row_of_q = [&](int q) { return s_begin + (q / BPV) * RPS + (vw + (q % BPV) * NVW) * 16; };
    if (n_q > 0) load_v(row_of_q(0), v0);
    if (n_q > 1) load_v(row_of_q(1), v1);
    for (int it = 0; it <= n_it; ++it) {
      for (int jj = 0; it >= 1 && jj < BPV; ++jj) {
        const int q = (it - 1) * BPV + jj;   // logits finished by the key waves in the previous step
        const int lrow = (vw + jj * NVW) * 16;
        if (row_of_q(q) < s_end) {
        float lgv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) lgv[i] = lgs[(it - 1) & 1][lrow + rg * 4 + i][hsel];
        // maximum of each head over the block: the lane's four rows, the four row groups, then every head of the
        // quad into every lane
        float bm = fmaxf(fmaxf(lgv[0], lgv[1]), fmaxf(lgv[2], lgv[3]));
        bm = fmaxf(bm, __shfl_xor(bm, 16, kWave));
        bm = fmaxf(bm, __shfl_xor(bm, 32, kWave));
        float corr[GH], m_own = -INFINITY, corr_own = 1.f;
        bool moved = false;
        const int bmi = __float_as_int(bm);
        const float bq[GH] = {__int_as_float(__builtin_amdgcn_update_dpp(0, bmi, 0x00, 0xf, 0xf, false)),
                              __int_as_float(__builtin_amdgcn_update_dpp(0, bmi, 0x55, 0xf, 0xf, false)),
                              __int_as_float(__builtin_amdgcn_update_dpp(0, bmi, 0xaa, 0xf, 0xf, false)),
                              __int_as_float(__builtin_amdgcn_update_dpp(0, bmi, 0xff, 0xf, 0xf, false))};
#pragma unroll
        for (int g = 0; g < GH; ++g) {
          const float bg = bq[g];   // lane g of the quad, into every lane of the quad
          const float mn = fmaxf(mh[g], bg);
          corr[g] = (mn == mh[g]) ? 1.f : __builtin_amdgcn_exp2f(mh[g] - mn);   // (-inf -> value: 2^-inf = 0)
          moved |= mn != mh[g];
          mh[g] = mn;
          if (hsel == g) { m_own = mn; corr_own = corr[g]; }
        }
        if (__any(moved)) {
          lpart *= corr_own;
#pragma unroll
          for (int e = 0; e < EPL; ++e)
#pragma unroll
            for (int g = 0; g < GH; ++g) oacc[e][g] *= corr[g];
        }
        const float m_ref = m_own == -INFINITY ? 0.f : m_own;
        uint32_t ph[4], pl[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float pv = __builtin_amdgcn_exp2f(lgv[i] - m_ref);   // rows past the end carry -inf: 0
          lpart += pv;
          ph[i] = __float_as_uint(pv) & 0xffff0000u;
          pl[i] = __float_as_uint(pv - __uint_as_float(ph[i]));
        }
        bf16x4 a_hi, a_lo;
        {
          const uint32_t h01 = __builtin_amdgcn_perm(ph[1], ph[0], 0x07060302u), h23 = __builtin_amdgcn_perm(ph[3], ph[2], 0x07060302u);
          const uint32_t l01 = __builtin_amdgcn_perm(pl[1], pl[0], 0x07060302u), l23 = __builtin_amdgcn_perm(pl[3], pl[2], 0x07060302u);
          const uint2 hv = make_uint2(h01, h23), lv2 = make_uint2(l01, l23);
          a_hi = *reinterpret_cast<const bf16x4*>(&hv);
          a_lo = *reinterpret_cast<const bf16x4*>(&lv2);
        }
        uint32_t bw[4][EPL / 2];   // the four rows as bf16 pairs
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
          for (int w = 0; w < EPL / 2; ++w) {
            if constexpr (EB == 2) bw[j][w] = v0[j][w];
            else bw[j][w] = (w & 1) ? e5m2x2_to_bf16x2<1>(v0[j][w / 2]) : e5m2x2_to_bf16x2<0>(v0[j][w / 2]);
          }
        }
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;   // the upper / lower element of a pair
          const uint2 bv = make_uint2(__builtin_amdgcn_perm(bw[1][e / 2], bw[0][e / 2], sel),
                                      __builtin_amdgcn_perm(bw[3][e / 2], bw[2][e / 2], sel));
          const bf16x4 bfrag = *reinterpret_cast<const bf16x4*>(&bv);
          oacc[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_hi, bfrag, oacc[e], 0, 0, 0);
          oacc[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_lo, bfrag, oacc[e], 0, 0, 0);
        }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int e = 0; e < RW; ++e) v0[j][e] = v1[j][e];
        if (q + 2 < n_q) load_v(row_of_q(q + 2), v1);   // (rows past the end are clamped inside)
      }
      __syncthreads();
    }
  }
  // ---- merge: the value waves through LDS
  lpart += __shfl_xor(lpart, 16, kWave);
  lpart += __shfl_xor(lpart, 32, kWave);
  if (rg == 0) {
#pragma unroll
    for (int g = 0; g < GH; ++g)
#pragma unroll
      for (int e = 0; e < EPL; ++e) sm_acc[vw][g][sub * EPL + e] = oacc[e][g];
    if (sub < GH) { sm_l[vw][sub] = lpart; }
  }
  if (lane == 0) {
#pragma unroll
    for (int g = 0; g < GH; ++g) sm_m[vw][g] = mh[g];
  }
  __syncthreads();
  for (int idx = threadIdx.x - 64 * NKW; idx < nv * D; idx += 64 * NVW) {
    const int g = idx / D, e = idx - g * D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NVW; ++w) M = fmaxf(M, sm_m[w][g]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < NVW; ++w) {
      const float sc = (sm_m[w][g] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sm_m[w][g] - M);
      num = fmaf(sm_acc[w][g][e], sc, num);
      den = fmaf(sm_l[w][g], sc, den);
    }
    const size_t pidx = (head0 + g) * a.n_part + split;
    a.part_acc[pidx * D + e] = num;
    if (e == 0) a.part_ml[pidx] = make_float2(M, den);
  }
}

// Second phase of the two-phase path: out-contribution of the selected rows from their stored logits
// (log2 units) and their values.  A workgroup takes pv_split_len consecutive selected rows of a unit for
// GH heads: 16 lanes share a row (d/16 columns each), 16 rows at a time; the maximum of each head over
// the workgroup's rows is formed first, so a single pass accumulates sum 2^(l - m) v.  Writes one
// partial state (m, l, acc[d]) per head behind those of the first phase.
template <int D, int GH, int EB>
__global__ __launch_bounds__(256) void sparse_values_kernel(AttnArgs a) {
  constexpr int EPL = D / 16;
  constexpr int RW = RawWords<EPL, EB>::n;
  __shared__ float sm_max[16][GH];
  __shared__ float sm_l[16][GH];
  __shared__ float sm_acc[16][GH][D];
  const int unit = blockIdx.y, split = blockIdx.x, g0 = blockIdx.z * GH;
  const int G = a.hq / a.hkv, b = unit / a.hkv, h = unit % a.hkv;
  const size_t head0 = (size_t)b * a.hq + (size_t)h * G + g0;
  const int nv = min(GH, G - g0);   // heads of this block that exist; surplus ones repeat the last real one
  const int sub = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const int kc = a.k * a.c;
  const int r_begin = split * a.pv_split_len, r_end = min(kc, r_begin + a.pv_split_len);
  const float* lg = a.logit_buf + head0 * (size_t)kc;
  const uint8_t* vbase = static_cast<const uint8_t*>(a.v_sparse) + (size_t)unit * a.v_unit_rows * D * EB;
  const int last_slot = a.v_unit_rows / a.c - 1;

  // per-head maximum over the workgroup's rows
  float mx[GH];
#pragma unroll
  for (int g = 0; g < GH; ++g) mx[g] = -INFINITY;
  for (int i = r_begin + threadIdx.x; i < r_end; i += 256)
#pragma unroll
    for (int g = 0; g < GH; ++g) mx[g] = fmaxf(mx[g], lg[(size_t)min(g, nv - 1) * kc + i]);
#pragma unroll
  for (int g = 0; g < GH; ++g) {
#pragma unroll
    for (int m = 8; m >= 1; m >>= 1) mx[g] = fmaxf(mx[g], __shfl_xor(mx[g], m, kWave));
    if (sub == 0) sm_max[grp][g] = mx[g];
  }
  __syncthreads();
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    float m = -INFINITY;
#pragma unroll
    for (int w = 0; w < 16; ++w) m = fmaxf(m, sm_max[w][g]);
    mx[g] = m;
  }

  float l[GH], acc[GH][EPL];
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }
  for (int i0 = r_begin + grp; i0 < r_end; i0 += 64) {   // four rows per lane group in flight
    uint32_t vraw[4][RW];
    float p[4][GH];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int i = i0 + 16 * x;
      const int ic = min(i, r_end - 1);
      const int ch = ic / a.c, t = ic - ch * a.c;
      const int slot = a.v_slots ? a.v_slots[(size_t)unit * a.k + ch] : ch;
      load_raw<EPL, EB>(vbase + (((size_t)min(max(slot, 0), last_slot) * a.c + t) * D + sub * EPL) * EB, vraw[x]);
#pragma unroll
      for (int g = 0; g < GH; ++g) p[x][g] = i < r_end ? lg[(size_t)min(g, nv - 1) * kc + ic] : -INFINITY;
    }
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      float vx[EPL];
      unpack_kv<EPL, EB>(vraw[x], vx);
#pragma unroll
      for (int g = 0; g < GH; ++g) {
        const float w = __builtin_amdgcn_exp2f(p[x][g] - mx[g]);   // -inf for rows past the end: 0
        l[g] += w;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(w, vx[e], acc[g][e]);
      }
    }
  }
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    if (sub == 0) sm_l[grp][g] = l[g];
#pragma unroll
    for (int e = 0; e < EPL; ++e) sm_acc[grp][g][sub * EPL + e] = acc[g][e];
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < nv * D; idx += 256) {
    const int g = idx / D, e = idx - g * D;
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) { num += sm_acc[w][g][e]; den += sm_l[w][g]; }
    const size_t pidx = (head0 + g) * a.n_part + a.n_splits + split;
    a.part_acc[pidx * D + e] = num;
    if (e == 0) {
      float m = -INFINITY;
#pragma unroll
      for (int w = 0; w < 16; ++w) m = fmaxf(m, sm_max[w][g]);
      a.part_ml[pidx] = make_float2(m, den);
    }
  }
}

// Merge of the per-split states of one head: out = sum_s acc_s 2^(m_s - M) / sum_s l_s 2^(m_s - M).
// A separate launch on purpose: a device-scope release inside the attention kernel would make every
// workgroup write back its XCD's L2, which costs far more than this kernel.
constexpr int kCombineNY = 4;
template <int D>
__global__ __launch_bounds__(D * kCombineNY) void attn_combine_kernel(const float* __restrict__ part_acc,
                                                                      const float2* __restrict__ part_ml,
                                                                      bf16_t* __restrict__ out, int n_splits) {
  // thread (e, y): output column e, the y-th quarter of the partial states (long contexts with few units have
  // dozens of them per head); eight loads are issued together, the folding order is fixed
  __shared__ float sm_M[kCombineNY], sm_den[kCombineNY], sm_num[kCombineNY][D];
  const size_t head = blockIdx.x;
  const int e = threadIdx.x, y = threadIdx.y;
  const int per = (n_splits + kCombineNY - 1) / kCombineNY;
  const int s_begin = min(n_splits, y * per), s_end = min(n_splits, s_begin + per);
  const float2* ml = part_ml + head * n_splits;
  const float* pa = part_acc + head * n_splits * D + e;
  float M = -INFINITY;
  for (int s0 = s_begin; s0 < s_end; s0 += 8) {
    float mx[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) mx[u] = ml[min(s0 + u, s_end - 1)].x;
#pragma unroll
    for (int u = 0; u < 8; ++u) M = fmaxf(M, mx[u]);
  }
  if (e == 0) sm_M[y] = M;
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kCombineNY; ++j) M = fmaxf(M, sm_M[j]);
  float num = 0.f, den = 0.f;
  for (int s0 = s_begin; s0 < s_end; s0 += 8) {
    float2 st[8];
    float av[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int sp = min(s0 + u, s_end - 1);
      st[u] = ml[sp];
      av[u] = pa[(size_t)sp * D];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (s0 + u < s_end) {
        const float sc = (st[u].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st[u].x - M);
        num = fmaf(av[u], sc, num);
        den = fmaf(st[u].y, sc, den);
      }
    }
  }
  sm_num[y][e] = num;
  if (e == 0) sm_den[y] = den;
  __syncthreads();
  if (y == 0) {
    num = sm_num[0][e]; den = sm_den[0];
#pragma unroll
    for (int j = 1; j < kCombineNY; ++j) { num += sm_num[j][e]; den += sm_den[j]; }
    out[head * D + e] = f32_to_bf16(num / den);
  }
}

template <int D, int GH, int KSMAX, bool FAST4, bool KEYS_ONLY, int EB>
static hipError_t launch_sparse(const AttnArgs& a, dim3 grid, size_t lds, hipStream_t st) {
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sparse_attn_kernel<D, GH, KSMAX, FAST4, KEYS_ONLY, EB>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((sparse_attn_kernel<D, GH, KSMAX, FAST4, KEYS_ONLY, EB>), grid, dim3(256), lds, st, a);
  return hipGetLastError();
}

template <int D, int GH, bool KEYS_ONLY, int EB>
static hipError_t launch_sparse_ks(const AttnArgs& a, dim3 grid, size_t lds, hipStream_t st) {
  const bool fast4 = a.c % 4 == 0;
  if (a.r32 <= 160)
    return fast4 ? launch_sparse<D, GH, 5, true, KEYS_ONLY, EB>(a, grid, lds, st)
                 : launch_sparse<D, GH, 5, false, KEYS_ONLY, EB>(a, grid, lds, st);
  return fast4 ? launch_sparse<D, GH, 8, true, KEYS_ONLY, EB>(a, grid, lds, st)
               : launch_sparse<D, GH, 8, false, KEYS_ONLY, EB>(a, grid, lds, st);
}

template <int D, int KSMAX, int EB>
static hipError_t launch_roles(const AttnArgs& a, dim3 grid, size_t lds, hipStream_t st) {
  constexpr int NKW = 12, NVW = 4;
  if (lds > 32 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sparse_attn_roles_kernel<D, KSMAX, EB, 1, NKW, NVW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((sparse_attn_roles_kernel<D, KSMAX, EB, 1, NKW, NVW>), grid, dim3(64 * (NKW + NVW)), lds, st, a);
  return hipGetLastError();
}

template <int D, bool KEYS_ONLY, int EB>
static hipError_t launch_keys_d(const AttnArgs& a, hipStream_t st) {
  const int G = a.hq / a.hkv;
  const int gh = attention_heads_per_group(G);
  // B^T (as bf16 whatever the storage), then the first token and the first value row of each chunk a split touches
  const size_t lds = (size_t)D * a.rp * sizeof(bf16_t) + 2 * ((size_t)a.sparse_split_len / a.c + 2) * sizeof(int);
  const int zb = (G + gh - 1) / gh;   // head blocks per unit (the last one may be partly empty)
  dim3 grid(a.batch * a.hkv, a.n_splits, zb);
  if (KEYS_ONLY) grid = dim3((unsigned)(a.gather.n_blocks + (long)a.n_splits * a.batch * a.hkv * zb));
  // values readable now, four heads per block, chunks of a multiple of four tokens: the kernel with key waves and
  // value waves
  if (attention_has_roles(G, a.c, a.k, a.k_sparse_out != nullptr, KEYS_ONLY))
    return a.r32 <= 160 ? launch_roles<D, 5, EB>(a, grid, lds, st) : launch_roles<D, 8, EB>(a, grid, lds, st);
  switch (gh) {
    case 4: return launch_sparse_ks<D, 4, KEYS_ONLY, EB>(a, grid, lds, st);
    case 2: return launch_sparse_ks<D, 2, KEYS_ONLY, EB>(a, grid, lds, st);
    default: return launch_sparse_ks<D, 1, KEYS_ONLY, EB>(a, grid, lds, st);
  }
}

template <int D>
static hipError_t launch_combine_d(const AttnArgs& a, hipStream_t st) {
  hipLaunchKernelGGL((attn_combine_kernel<D>), dim3(a.batch * a.hq), dim3(D, kCombineNY), 0, st, a.part_acc, a.part_ml, a.out,
                     a.n_part);
  return hipGetLastError();
}

template <int D, int EB>
static hipError_t launch_values_d(const AttnArgs& a, hipStream_t st) {
  const int G = a.hq / a.hkv;
  const int gh = attention_heads_per_group(G);
  dim3 grid(a.n_pv_splits, a.batch * a.hkv, (G + gh - 1) / gh);
  switch (gh) {
    case 4: hipLaunchKernelGGL((sparse_values_kernel<D, 4, EB>), grid, dim3(256), 0, st, a); break;
    case 2: hipLaunchKernelGGL((sparse_values_kernel<D, 2, EB>), grid, dim3(256), 0, st, a); break;
    default: hipLaunchKernelGGL((sparse_values_kernel<D, 1, EB>), grid, dim3(256), 0, st, a); break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_combine_d<D>(a, st);
}

// The three launches for one storage type; each translation unit instantiates one EB.
// Fused path: everything in one kernel (values already readable), then the merge of the splits.
template <int EB>
hipError_t launch_attention_eb(const AttnArgs& a, hipStream_t st) {
  hipError_t e;
  switch (a.d) {
    case 64: e = launch_keys_d<64, false, EB>(a, st); return e != hipSuccess ? e : launch_combine_d<64>(a, st);
    case 96: e = launch_keys_d<96, false, EB>(a, st); return e != hipSuccess ? e : launch_combine_d<96>(a, st);
    case 128: e = launch_keys_d<128, false, EB>(a, st); return e != hipSuccess ? e : launch_combine_d<128>(a, st);
    default: return hipErrorInvalidValue;
  }
}
// Two-phase path for values that arrive through a gather on another stream: this part needs none of them ...
template <int EB>
hipError_t launch_attention_keys_eb(const AttnArgs& a, hipStream_t st) {
  switch (a.d) {
    case 64: return launch_keys_d<64, true, EB>(a, st);
    case 96: return launch_keys_d<96, true, EB>(a, st);
    case 128: return launch_keys_d<128, true, EB>(a, st);
    default: return hipErrorInvalidValue;
  }
}
// ... and this part runs once they are there (softmax of the stored logits times the values, merge of all parts).
template <int EB>
hipError_t launch_attention_values_eb(const AttnArgs& a, hipStream_t st) {
  switch (a.d) {
    case 64: return launch_values_d<64, EB>(a, st);
    case 96: return launch_values_d<96, EB>(a, st);
    case 128: return launch_values_d<128, EB>(a, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace skv
