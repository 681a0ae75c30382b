// Launch interfaces of the ShadowKV HIP kernels (internal; the public ABI is
// include/shadowkv.h).  Every launcher only enqueues on the given stream and
// returns hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "common.hpp"

namespace skv {

constexpr int kMaxHalfDim = 64;   // head_dim <= 128
constexpr int kScoreTile = 256;   // landmark rows per scoring workgroup

// Rotary frequencies, in revolutions per position (inv_freq / 2 pi), fp64, by value.
struct RopeFreqs {
  double rev[kMaxHalfDim];
};

// ---- landmark scoring (decoding algorithm, P = Q L^T / sqrt(d)) ----------------
// logits [b*h_q, ld] fp32 (the fp64 sum rounded once; ld = n_c rounded up to a multiple of 4); partials [b*h_q, n_tiles] (max, sum exp(p - max))
// per tile, fp64.
// landmarks [units, nc_stride, d]: n_c valid rows per unit.
// kv_bytes (here and below): bytes per element of the KV-cache tensors, 2 = bf16, 1 = FP8 E5M2.
hipError_t launch_score(const bf16_t* q, const void* landmarks, int kv_bytes, float* logits, int ld, double2* partials,
                        int batch, int hq, int hkv, int d, int n_c, int nc_stride, double scale, hipStream_t st);

// ---- ArgTopK -------------------------------------------------------------------
// Attention over the resident rows [outliers ; recent] of every unit, done by extra workgroups of the selection's
// first launch (see resident_rows_attention in attn_kernels.hpp).
struct ResidentArgs {
  const bf16_t* q;          // [b, h_q, d]
  const void* k_outlier;    // [units, o*c, d]
  const void* v_outlier;
  const void* k_local;      // [units, w, d]
  const void* v_local;
  float* part_acc;          // [b*h_q, n_part, d]
  float2* part_ml;          // [b*h_q, n_part]
  int hq, hkv, oc, w, n_part, part_slot;
  int head_blocks;          // blocks of four heads per unit
  int units;
  float scale_log2;
};
constexpr int kSrcLogits = 0;  // key = max over the group of (logit - lse)
constexpr int kSrcArray = 1;   // key = sign * scores[unit, j]

struct SelectArgs {
  const float* logits;      // kSrcLogits: [units*G, ld] stored logits (fp32 roundings of the fp64 sums), ld % 4 == 0
  const double2* partials;  //             [units*G, n_tiles]
  int n_tiles, G, ld;
  // kSrcLogits, for exact scores at the selection boundary: the operands of the logits and a place for the
  // heads' log-sum-exp (written by the first level, read by the later ones)
  const bf16_t* q;          // [units*G, d]
  const void* landmarks;    // [units, nc_stride, d]
  int d, kv_bytes, nc_stride;
  double scale;
  double* lse_out;          // [units*G]
  uint32_t* key_top_out;    // [units] search key no slot of the unit exceeds
  const double* scores;     // kSrcArray: [units, n]
  double sign;
  int n, k, slice_len, n_slices, cand_stride;
  int group_cands, n_groups, cand2_off;  // middle level (0 groups = none): see SelectPlan
  uint64_t* cand_key;       // [units, cand_stride] survivors of the slices (kSrcLogits: 32-bit keys in the same space)
  int32_t* cand_idx;
  const int32_t* id_map;    // optional [units, id_stride]: index -> reported id
  int id_stride;
  int32_t* out_ids;         // [units, k], ascending index order
  int32_t* out_ids2;        // optional copy
};
// Survivors of the slices are ranked by one workgroup per unit when it can hold them; otherwise groups of them
// (group_cands each) are first cut down to k per group by a middle level whose output lives behind the slices'
// survivors in the same arrays (offset cand2_off inside a unit's stride).  nt / e: threads per workgroup and
// keys per thread of each level.
struct SelectPlan {
  int nt, e, slice_len, n_slices, cand_stride, merge_nt, merge_e;
  int group_cands, n_groups, cand2_off, mid_nt, mid_e;
};
bool plan_select(int n, int k, int src, int units, SelectPlan* plan);
// res (may be NULL): resident-row attention to ride the first launch; only for shapes resident_fits() accepts
hipError_t launch_select(const SelectArgs& a, const SelectPlan& plan, int src, int units, hipStream_t st,
                         const ResidentArgs* res = nullptr, int d = 0, int kv_bytes = 2);
bool resident_fits(const SelectPlan& plan, int units, int G, int d);

// ---- value chunk gather (V_sparse = Gather(V_store, I)) -----------------------------
// store [units, s_cap, d] of which s tokens are valid
hipError_t launch_gather_values(const void* store, const int32_t* sel_ids, void* v_sparse, int kv_bytes, int units,
                                int d, int s, int s_cap, int c, int k, hipStream_t st);

// ---- chunk cache of the offloaded values: index scan, fetch of the missing chunks ------
constexpr int kMaxCacheSlots = 8192;  // slots per unit the index-scan kernel handles (256 threads x 32, LDS)
// cache_ids [units, S], stamps [units, S + 1] (entry S = the unit's clock), sel_slots / miss_slots [units, k]
hipError_t launch_cache_update(const int32_t* sel_ids, int32_t* cache_ids, int32_t* stamps, int32_t* sel_slots,
                               int32_t* miss_slots, int32_t* n_miss, int32_t* n_miss_copy, int units, int k, int S,
                               hipStream_t st);
hipError_t launch_gather_missing(const void* store, const int32_t* cache_ids, const int32_t* miss_slots,
                                 const int32_t* n_miss, void* v_cache, int kv_bytes, int units, int d, int s, int s_cap,
                                 int c, int k, int S, hipStream_t st);
hipError_t launch_fill_i32(int32_t* p, size_t n, int32_t value, hipStream_t st);

// ---- attention over [outliers ; recent] and [selected chunks], keys rebuilt in-kernel ----
// K_sparse = RoPE(Gather(A, I) B) is formed per 16-row block on the matrix cores and consumed
// from registers.  Split i covers selected rows [i*sparse_split_len, ...) and resident rows
// [i*res_split_len, ...); a combine kernel merges the splits into `out`.
// A gather of value chunks that rides in the same launch as the key phase of the attention (the first
// `n_blocks` workgroups of that launch do it; 0: none).  Plain: chunk ids[unit][i] of the store goes to
// slot i of dst.  With a chunk cache (miss_slots != NULL): for i < n_miss[unit], the chunk named by
// ids[unit][slot], slot = miss_slots[unit][i], goes to that slot of dst.
struct GatherArgs {
  const uint4* store;         // [units, vec_per_unit_store] 16-byte vectors (HBM or device-readable pinned host memory)
  uint4* dst;                 // [units, slots_per_unit, vec_per_chunk]
  const int32_t* ids;         // plain: [units, k] selected chunk ids; cache: [units, slots_per_unit] chunk id held by each slot
  const int32_t* miss_slots;  // cache only: [units, k]
  const int32_t* n_miss;      // cache only: [units]
  int n_blocks, blocks_per_unit, unit_step;
  int units, k, slots_per_unit, vec_per_chunk, last_chunk;
  size_t vec_per_unit_store;
};
void plan_gather(GatherArgs* g);  // fills n_blocks, blocks_per_unit, unit_step from the sizes

struct AttnArgs {
  const bf16_t* q;          // [b, h_q, d]
  int kv_bytes;             // storage of the tensors below that are void*: 2 = bf16, 1 = FP8 E5M2
  const void* A;            // [b, s_cap, r]
  const void* B;            // [units, r, d]
  const void* k_outlier;    // [units, o*c, d]
  const void* v_outlier;
  const void* k_local;      // [units, w, d]
  const void* v_local;
  const void* v_sparse;     // staged [units, v_unit_rows, d], or NULL: read v_store through sel_ids
  const int32_t* v_slots;   // optional [units, k]: chunk slot of selected chunk i inside v_sparse (NULL: slot i)
  int v_unit_rows;          // rows per unit of v_sparse (k*c, or slots*c of a value cache)
  const void* v_store;      // [units, s_cap, d] (HBM, or device-readable pinned host memory)
  const int32_t* sel_ids;   // [units, k] true chunk ids
  const int32_t* pos_offset;  // [b] or NULL
  const float* inv_freq_dev;  // optional [d/2]
  float* k_sparse_out;      // optional [units, k*c, d]: copy of the rebuilt keys (diagnostics)
  float* part_acc;          // [b*h_q, n_splits, d]
  float2* part_ml;          // [b*h_q, n_splits] (max in log2 units, sum)
  bf16_t* out;              // [b, h_q, d]
  int batch, hq, hkv, d, s, c, o, k, w, r, r32, rp;
  int s_cap;                // tokens A and v_store are laid out for (>= s)
  int res_split_len, sparse_split_len, n_splits;
  float* logit_buf;         // two-phase path: [b*h_q, k*c] logits of the selected rows (log2 units)
  int pv_split_len, n_pv_splits;  // two-phase path: selected rows per workgroup of the second phase
  int n_part;               // partial states per head: n_splits (+ n_pv_splits on the two-phase path, + 1 with skip_resident)
  int skip_resident;        // the resident rows [outliers ; recent] are attended over elsewhere (state at index n_part - 1)
  int c_shift;              // log2(c) when c is a power of two, else -1
  float scale_log2;         // softmax scale * log2(e)
  RopeFreqs freqs;
  GatherArgs gather;        // key phase of the two-phase path only: value gather done by the same launch
};
// Query heads per attention workgroup: four wherever the group has at least three heads (a group of 3, 5, 6 or 7
// leaves part of its last block empty, which costs less than rebuilding the keys once more per head or pair).
inline int attention_heads_per_group(int G) { return G >= 3 ? 4 : G; }
// Shapes the kernel with key waves and value waves takes: values readable in place, four heads per block, chunks
// of a multiple of four tokens, no diagnostic copy of the keys.
inline bool attention_has_roles(int G, int c, int k, bool keep_keys, bool keys_only) {
  return !keys_only && attention_heads_per_group(G) == 4 && c % 4 == 0 && !keep_keys && (long)k * c >= 4;
}
hipError_t launch_attention(const AttnArgs& a, hipStream_t st);         // values readable now: one fused kernel
hipError_t launch_attention_keys(const AttnArgs& a, hipStream_t st);    // two-phase path, before the values arrive
hipError_t launch_attention_values(const AttnArgs& a, hipStream_t st);  // two-phase path, after

// ---- pre-filling algorithm: chunk means, min cosine, compaction, outlier gather -------
hipError_t launch_chunk_stats(const void* k_rope, int kv_bytes, void* chunk_mean, double* chunk_min_cos, int units, int d,
                              int s, int c, hipStream_t st);
hipError_t launch_compact_landmarks(const void* chunk_mean, int kv_bytes, const int32_t* outlier_ids, void* landmarks,
                                    int32_t* landmark_chunk_ids, int units, int d, int n_ch, int o, int nc_stride,
                                    hipStream_t st);
hipError_t launch_gather_outliers(const void* k_rope, const void* v, int kv_bytes, const int32_t* outlier_ids,
                                  void* k_outlier, void* v_outlier, int units, int d, int s, int s_cap, int c,
                                  int o, hipStream_t st);

// ---- generated tokens: one more chunk of context (low-rank states K' Psi, landmark, values) ----
hipError_t launch_append_chunk(const void* k_pre, const void* k_rope, const void* v, const void* B, void* A,
                               void* landmarks, int32_t* landmark_chunk_ids, void* value_store, int kv_bytes, int batch,
                               int hkv, int d, int s, int s_cap, int c, int r, int o, hipStream_t st);

// ---- pre-filling algorithm, first line: A, B <- SVD(K) truncated to rank r (kernels_factorize.hip) ----
struct FactorizePlan {
  int m, mp;                // subspace width r + oversample (at most D), and the same rounded up to even
  int nb;                   // 64-column blocks of the Gram matrix
  int n_splits, tokens_per_split;
  size_t part, G, Xt, Yt, W, V, Wsel, Psi_t, total;  // workspace offsets (bytes)
};
FactorizePlan plan_factorize(int batch, int s, int D, int r, int oversample);
// k_pre [b, s, h_kv*d]; A [b, s_cap, r]; B [b, h_kv, r, d]; psi_out optional [b, r, D] fp64 (right singular vectors
// as rows, after the sign convention); sigma_out optional [b, r] fp64 (singular values, strongest first)
hipError_t launch_factorize(const void* k_pre, int kv_bytes, void* A, void* B, double* psi_out, double* sigma_out,
                            char* ws, const FactorizePlan& pl, int batch, int hkv, int d, int s, int s_cap, int r,
                            int n_iter, int n_sweeps, hipStream_t st);

}  // namespace skv
