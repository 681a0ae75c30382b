// C ABI of libshadowkv (see include/shadowkv.h): argument validation, workspace layout,
// and the enqueue order of the kernels.  Nothing here touches the GPU before the
// arguments have been accepted.
#include "../../include/shadowkv.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "kernels.hpp"

using namespace skv;

// Scratch memory of shadowkv_decode_step_static: what the other decode entry points take as `workspace`.
// One copy per GPU the library is loaded on, held until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; the device address it yields (per device) is what the kernels are given.
constexpr size_t kStaticScratchBytes = (size_t)96 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local char g_err[512] = "";

void set_err(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}

int fail_inval(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return SHADOWKV_EINVAL;
}

int fail_hip(const char* what, hipError_t e) {
  set_err("%s: %s", what, hipGetErrorString(e));
  return SHADOWKV_EHIP;
}

constexpr size_t kAlign = 256;
size_t up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Shape {
  int b, hq, hkv, G, d, s, c, r, o, k, w, n_ch, n_c, units;
  int cap, nc_cap;  // tokens / landmark rows the context arrays are laid out for
  int eb;           // bytes per element of the KV-cache tensors (2 = bf16, 1 = FP8 E5M2)
  bool stage, keep_keys;
};

// Shape rules shared by both entry points.  Returns SHADOWKV_OK or EINVAL with a reason.
int check_params(const shadowkv_params* p, bool decode, Shape* sh) {
  if (!p) return fail_inval("params is NULL");
  if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1)
    return fail_inval("batch, n_q_heads, n_kv_heads must be >= 1");
  if (p->n_q_heads % p->n_kv_heads) return fail_inval("n_q_heads must be a multiple of n_kv_heads");
  if (p->n_q_heads / p->n_kv_heads > 64) return fail_inval("group size above 64 is not supported");
  if (p->head_dim != 64 && p->head_dim != 96 && p->head_dim != 128)
    return fail_inval("head_dim must be 64, 96 or 128");
  if (p->chunk_size < 1 || p->chunk_size > 64) return fail_inval("chunk_size must be in [1, 64]");
  if (p->ctx_len < p->chunk_size || p->ctx_len % p->chunk_size)
    return fail_inval("ctx_len must be a positive multiple of chunk_size");
  const long n_ch = p->ctx_len / p->chunk_size;
  if (p->n_outlier_chunks < 0 || p->n_outlier_chunks > 1024 || p->n_outlier_chunks > n_ch)
    return fail_inval("n_outlier_chunks must be in [0, min(1024, ctx_len/chunk_size)]");
  const long units = (long)p->batch * p->n_kv_heads;
  if (units > 65535) return fail_inval("batch * n_kv_heads above 65535 is not supported");
  if (p->value_location != SHADOWKV_VALUES_DEVICE && p->value_location != SHADOWKV_VALUES_HOST)
    return fail_inval("value_location must be SHADOWKV_VALUES_DEVICE or SHADOWKV_VALUES_HOST");
  if (p->kv_dtype != SHADOWKV_KV_BF16 && p->kv_dtype != SHADOWKV_KV_FP8_E5M2)
    return fail_inval("kv_dtype must be SHADOWKV_KV_BF16 or SHADOWKV_KV_FP8_E5M2");
  sh->eb = p->kv_dtype == SHADOWKV_KV_FP8_E5M2 ? 1 : 2;
  sh->b = p->batch; sh->hq = p->n_q_heads; sh->hkv = p->n_kv_heads; sh->G = sh->hq / sh->hkv;
  sh->d = p->head_dim; sh->s = p->ctx_len; sh->c = p->chunk_size; sh->o = p->n_outlier_chunks;
  sh->n_ch = (int)n_ch; sh->n_c = (int)n_ch - sh->o; sh->units = (int)units;
  if (p->ctx_capacity != 0 && (p->ctx_capacity < p->ctx_len || p->ctx_capacity % p->chunk_size))
    return fail_inval("ctx_capacity must be 0 or a multiple of chunk_size that is >= ctx_len");
  sh->cap = p->ctx_capacity ? p->ctx_capacity : p->ctx_len;
  sh->nc_cap = sh->cap / sh->c - sh->o;
  sh->r = p->rank; sh->k = p->topk_chunks; sh->w = p->local_len;
  sh->stage = p->value_location == SHADOWKV_VALUES_HOST || (p->flags & SHADOWKV_FLAG_STAGE_VALUES);
  sh->keep_keys = (p->flags & SHADOWKV_FLAG_KEEP_REBUILT_KEYS) != 0;
  if (!decode) return SHADOWKV_OK;
  if (p->rank < 8 || p->rank > 256 || p->rank % 8) return fail_inval("rank must be a multiple of 8 in [8, 256]");
  if (p->local_len < 0) return fail_inval("local_len must be >= 0");
  if (p->topk_chunks < 1 || p->topk_chunks > sh->n_c)
    return fail_inval("topk_chunks must be in [1, ctx_len/chunk_size - n_outlier_chunks]");
  if ((long)p->topk_chunks * p->chunk_size > (1l << 24)) return fail_inval("topk_chunks * chunk_size too large");
  if (!(p->softmax_scale >= 0.0) || !std::isfinite(p->softmax_scale))
    return fail_inval("softmax_scale must be finite and >= 0");
  if (!p->inv_freq && !(p->rope_theta > 0.0 && std::isfinite(p->rope_theta)))
    return fail_inval("rope_theta must be finite and > 0 when inv_freq is NULL");
  SelectPlan plan;
  if (!plan_select(sh->n_c, sh->k, kSrcLogits, sh->units, &plan))
    return fail_inval("topk_chunks / landmark count combination exceeds the selection kernels' capacity");
  return SHADOWKV_OK;
}

// Split plan of the attention kernel: the selected rows are cut into splits that are multiples of
// 32 rows (two MFMA row blocks); every split also takes an equal share of the resident
// rows (outliers + recent tokens).
struct AttnPlan {
  int res_split_len, sparse_split_len, n_splits, z;
  int pv_split_len, n_pv_splits;  // second phase of the two-phase path (values gathered meanwhile)
};
AttnPlan plan_attention(const Shape& sh, bool with_cache = false) {
  AttnPlan ap;
  ap.z = (sh.G + attention_heads_per_group(sh.G) - 1) / attention_heads_per_group(sh.G);
  const long groups = (long)sh.units * ap.z;
  const long kc = (long)sh.k * sh.c, n_res = (long)sh.o * sh.c + sh.w;
  // the largest split (fewest B^T stagings) that still gives >= 512 workgroups; the kernel with key and value
  // waves runs one 1024-thread workgroup per compute unit: 256 of them fill the chip
  const bool roles = attention_has_roles(sh.G, sh.c, sh.k, sh.keep_keys, sh.stage || with_cache);
  const long want = roles ? 256 : 512;
  long len = 32;
  for (long cand : {1024l, 512l, 256l, 128l, 64l}) if (kc * groups / cand >= want) { len = cand; break; }
  // tuning override: rows per split (read once)
  static const long forced = [] { const char* ov = std::getenv("SHADOWKV_SPARSE_SPLIT"); return ov ? std::atol(ov) : 0l; }();
  if (forced >= 32 && forced <= 1024 && forced % 32 == 0) len = forced;
  while ((kc + len - 1) / len > 65535) len *= 2;   // the splits are a grid dimension
  ap.sparse_split_len = (int)len;
  ap.n_splits = (int)((kc + len - 1) / len);
  ap.res_split_len = (int)((n_res + ap.n_splits - 1) / ap.n_splits);
  ap.pv_split_len = 256;
  ap.n_pv_splits = (int)((kc + ap.pv_split_len - 1) / ap.pv_split_len);
  return ap;
}

struct DecodeLayout {
  size_t logits, partials, lse, key_top, cand_key, cand_idx, sel_ids, miss_slots, sel_slots, n_miss, logit_buf, k_sparse, v_sparse, part_acc, part_ml, total;
  SelectPlan sel;
  AttnPlan attn;
  int n_tiles, ld;   // score tiles per head; floats per row of the logits (n_c rounded up to a multiple of 4)
};
DecodeLayout decode_layout(const Shape& sh) {
  DecodeLayout L{};
  plan_select(sh.n_c, sh.k, kSrcLogits, sh.units, &L.sel);
  L.attn = plan_attention(sh);
  L.n_tiles = (sh.n_c + kScoreTile - 1) / kScoreTile;
  const size_t heads = (size_t)sh.b * sh.hq, rows = (size_t)sh.units * sh.k * sh.c;
  size_t off = 0;
  L.ld = (sh.n_c + 3) / 4 * 4;
  // (+ one slice of padding: the selection reads whole slices without bounds checks)
  L.logits = off; off += up((heads * L.ld + (size_t)L.sel.slice_len) * sizeof(float));
  L.partials = off; off += up(heads * L.n_tiles * sizeof(double2));
  L.lse = off; off += up(heads * sizeof(double));
  L.key_top = off; off += up((size_t)sh.units * sizeof(uint32_t));
  L.cand_key = off; off += up((size_t)sh.units * L.sel.cand_stride * sizeof(uint64_t));
  L.cand_idx = off; off += up((size_t)sh.units * L.sel.cand_stride * sizeof(int32_t));
  L.sel_ids = off; off += up((size_t)sh.units * sh.k * sizeof(int32_t));
  L.miss_slots = off; off += up((size_t)sh.units * sh.k * sizeof(int32_t));  // chunk cache: slots to fill
  L.sel_slots = off; off += up((size_t)sh.units * sh.k * sizeof(int32_t));   // chunk cache: slot of each selected chunk
  L.n_miss = off; off += up((size_t)sh.units * sizeof(int32_t));
  L.logit_buf = off; off += up(heads * rows / sh.units * sizeof(float));  // two-phase path: [b*h_q, k*c]
  L.k_sparse = off; off += sh.keep_keys ? up(rows * sh.d * sizeof(float)) : 0;
  L.v_sparse = off; off += sh.stage ? up(rows * sh.d * sh.eb) : 0;
  // (a step with a value cache plans its splits for the two-phase kernels: room for whichever has more)
  const AttnPlan cached = plan_attention(sh, true);
  const size_t n_part = (size_t)std::max(L.attn.n_splits, cached.n_splits) + L.attn.n_pv_splits;
  L.part_acc = off; off += up(heads * n_part * sh.d * sizeof(float));
  L.part_ml = off; off += up(heads * n_part * sizeof(float2));
  L.total = off;
  return L;
}

// Whether the resident rows (outliers, recent tokens) are attended over by extra workgroups of the selection launch.
bool resident_rows_in_selection(const Shape& sh, const DecodeLayout& L, bool with_cache) {
  return !with_cache && !sh.stage && !sh.keep_keys && sh.o * sh.c + sh.w > 0 && resident_fits(L.sel, sh.units, sh.G, sh.d);
}

struct BuildLayout {
  size_t chunk_mean, min_cos, cand_key, cand_idx, total;
  SelectPlan sel;
};
bool build_layout(const Shape& sh, BuildLayout* L) {
  *L = BuildLayout{};
  if (sh.o > 0 && !plan_select(sh.n_ch, sh.o, kSrcArray, sh.units, &L->sel)) return false;
  size_t off = 0;
  L->chunk_mean = off; off += up((size_t)sh.units * sh.n_ch * sh.d * sh.eb);
  L->min_cos = off; off += up((size_t)sh.units * sh.n_ch * sizeof(double));
  L->cand_key = off; off += up((size_t)sh.units * L->sel.cand_stride * sizeof(uint64_t));
  L->cand_idx = off; off += up((size_t)sh.units * L->sel.cand_stride * sizeof(int32_t));
  L->total = off;
  return true;
}

int check_workspace(void* ws, size_t have, size_t need) {
  if (!ws) { set_err("workspace is NULL"); return SHADOWKV_EWORKSPACE; }
  if (reinterpret_cast<uintptr_t>(ws) % kAlign) { set_err("workspace must be 256-byte aligned"); return SHADOWKV_EWORKSPACE; }
  if (have < need) { set_err("workspace too small: %zu bytes given, %zu needed", have, need); return SHADOWKV_EWORKSPACE; }
  return SHADOWKV_OK;
}

// Fork/join events, one pair per device, created on first use.
std::mutex g_mu;
constexpr int kMaxDev = 16;
hipEvent_t g_fork[kMaxDev] = {}, g_join[kMaxDev] = {};
bool g_have[kMaxDev] = {};

int get_events(hipEvent_t* fork, hipEvent_t* join) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip("hipGetDevice", e);
  if (dev < 0 || dev >= kMaxDev) return fail_inval("device index %d out of range", dev);
  if (!g_have[dev]) {
    e = hipEventCreateWithFlags(&g_fork[dev], hipEventDisableTiming);
    if (e != hipSuccess) return fail_hip("hipEventCreate", e);
    e = hipEventCreateWithFlags(&g_join[dev], hipEventDisableTiming);
    if (e != hipSuccess) { (void)hipEventDestroy(g_fork[dev]); return fail_hip("hipEventCreate", e); }
    g_have[dev] = true;
  }
  *fork = g_fork[dev]; *join = g_join[dev];
  return SHADOWKV_OK;
}

// Device address of `scratch` on the current device, looked up once per device.
void* g_scratch_ptr[kMaxDev] = {};
bool g_scratch_have[kMaxDev] = {};

int static_scratch(void** ptr) {
  std::lock_guard<std::mutex> lk(g_mu);
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip("hipGetDevice", e);
  if (dev < 0 || dev >= kMaxDev) return fail_inval("device index %d out of range", dev);
  if (!g_scratch_have[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip("hipGetSymbolAddress(scratch)", e);
    if (!p || reinterpret_cast<uintptr_t>(p) % kAlign) {
      set_err("static scratch has no usable device address");
      return SHADOWKV_EHIP;
    }
    g_scratch_ptr[dev] = p;
    g_scratch_have[dev] = true;
  }
  *ptr = g_scratch_ptr[dev];
  return SHADOWKV_OK;
}

// Optional per-stage timing: HIP events recorded on the caller's stream at the stage
// boundaries of every decode step between profile_begin and profile_end.
constexpr int kStages = 4;  // score | select | staged value gather (+ join) | attention with key rebuild
struct Profile {
  bool on = false;
  int max_steps = 0, n_steps = 0;
  std::vector<hipEvent_t> ev;  // [max_steps][kStages + 1]
} g_prof;

void prof_mark(hipStream_t st, int step, int boundary) {
  if (step >= 0) (void)hipEventRecord(g_prof.ev[(size_t)step * (kStages + 1) + boundary], st);
}

}  // namespace

extern "C" {

int shadowkv_profile_begin(int max_steps) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (g_prof.on) return fail_inval("profiling is already on");
  if (max_steps < 1 || max_steps > 100000) return fail_inval("max_steps must be in [1, 100000]");
  g_prof.ev.assign((size_t)max_steps * (kStages + 1), nullptr);
  for (auto& e : g_prof.ev) {
    hipError_t err = hipEventCreate(&e);
    if (err != hipSuccess) {
      for (auto& d : g_prof.ev) if (d) (void)hipEventDestroy(d);
      g_prof.ev.clear();
      return fail_hip("hipEventCreate", err);
    }
  }
  g_prof.on = true; g_prof.max_steps = max_steps; g_prof.n_steps = 0;
  return SHADOWKV_OK;
}

int shadowkv_profile_end(double* stage_ms, int* n_steps) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_prof.on) return fail_inval("profiling is not on");
  int rc = SHADOWKV_OK;
  if (stage_ms) for (int i = 0; i < kStages; ++i) stage_ms[i] = 0.0;
  for (int s = 0; s < g_prof.n_steps && rc == SHADOWKV_OK; ++s) {
    hipEvent_t* e = &g_prof.ev[(size_t)s * (kStages + 1)];
    hipError_t err = hipEventSynchronize(e[kStages]);
    if (err != hipSuccess) { rc = fail_hip("hipEventSynchronize", err); break; }
    for (int i = 0; i < kStages; ++i) {
      float ms = 0.f;
      err = hipEventElapsedTime(&ms, e[i], e[i + 1]);
      if (err != hipSuccess) { rc = fail_hip("hipEventElapsedTime", err); break; }
      if (stage_ms) stage_ms[i] += ms;
    }
  }
  if (n_steps) *n_steps = g_prof.n_steps;
  for (auto& d : g_prof.ev) if (d) (void)hipEventDestroy(d);
  g_prof.ev.clear();
  g_prof.on = false;
  return rc;
}

int shadowkv_version(void) { return 400; }

const char* shadowkv_status_string(int status) {
  switch (status) {
    case SHADOWKV_OK: return "ok";
    case SHADOWKV_EINVAL: return "invalid argument";
    case SHADOWKV_EWORKSPACE: return "workspace missing, misaligned or too small";
    case SHADOWKV_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

const char* shadowkv_last_error(void) { return g_err; }

void shadowkv_shutdown(void) {
  std::lock_guard<std::mutex> lk(g_mu);
  int cur = 0;
  if (hipGetDevice(&cur) != hipSuccess) cur = -1;
  for (int d = 0; d < kMaxDev; ++d)
    if (g_have[d]) {
      if (hipSetDevice(d) == hipSuccess) { (void)hipEventDestroy(g_fork[d]); (void)hipEventDestroy(g_join[d]); }
      g_have[d] = false;
    }
  if (cur >= 0) (void)hipSetDevice(cur);
}

int shadowkv_validate_params(const shadowkv_params* params, int for_decode) {
  Shape sh;
  return check_params(params, for_decode != 0, &sh);
}

size_t shadowkv_decode_workspace_bytes(const shadowkv_params* params) {
  Shape sh;
  if (check_params(params, true, &sh) != SHADOWKV_OK) return 0;
  return decode_layout(sh).total;
}

int shadowkv_decode_plan(const shadowkv_params* params, int32_t* plan) {
  Shape sh;
  const int rc = check_params(params, true, &sh);
  if (rc != SHADOWKV_OK) return rc;
  if (!plan) return fail_inval("plan is NULL");
  const DecodeLayout L = decode_layout(sh);
  plan[0] = L.attn.n_splits;
  plan[1] = L.attn.sparse_split_len;
  plan[2] = resident_rows_in_selection(sh, L, false) ? 1 : 0;
  plan[3] = attention_has_roles(sh.G, sh.c, sh.k, sh.keep_keys, sh.stage) ? 1 : 0;
  plan[4] = L.sel.nt;
  plan[5] = L.sel.e;
  plan[6] = L.sel.n_slices == 1 ? 1 : (L.sel.n_groups > 0 ? 3 : 2);
  plan[7] = L.ld;
  return SHADOWKV_OK;
}

size_t shadowkv_build_workspace_bytes(const shadowkv_params* params) {
  Shape sh;
  BuildLayout L;
  if (check_params(params, false, &sh) != SHADOWKV_OK || !build_layout(sh, &L)) return 0;
  return L.total;
}

void* shadowkv_decode_workspace_view(const shadowkv_params* params, void* workspace, int which) {
  Shape sh;
  if (!workspace || check_params(params, true, &sh) != SHADOWKV_OK) return nullptr;
  const DecodeLayout L = decode_layout(sh);
  char* ws = static_cast<char*>(workspace);
  switch (which) {
    case 0: return sh.keep_keys ? ws + L.k_sparse : nullptr;
    case 1: return sh.stage ? ws + L.v_sparse : nullptr;
    case 2: return ws + L.sel_ids;
    case 3: return ws + L.logits;
    case 4: return ws + L.miss_slots;
    case 5: return ws + L.sel_slots;
    default: return nullptr;
  }
}

int shadowkv_build_landmarks(const shadowkv_params* params, const shadowkv_kv* k_rope, const shadowkv_kv* v,
                             shadowkv_kv* landmarks, int32_t* landmark_chunk_ids, int32_t* outlier_chunk_ids,
                             shadowkv_kv* k_outlier, shadowkv_kv* v_outlier, void* workspace,
                             size_t workspace_bytes, void* stream) {
  Shape sh;
  int rc = check_params(params, false, &sh);
  if (rc != SHADOWKV_OK) return rc;
  if (!k_rope) return fail_inval("k_rope is NULL");
  if (sh.n_c > 0 && (!landmarks || !landmark_chunk_ids)) return fail_inval("landmarks / landmark_chunk_ids is NULL");
  if (sh.o > 0 && (!outlier_chunk_ids || !k_outlier)) return fail_inval("outlier outputs are NULL with n_outlier_chunks > 0");
  if (sh.o > 0 && v && !v_outlier) return fail_inval("v given but v_outlier is NULL");
  if (!aligned16(k_rope) || !aligned16(v) || !aligned16(landmarks) || !aligned16(k_outlier) || !aligned16(v_outlier))
    return fail_inval("tensor pointers must be 16-byte aligned");
  BuildLayout L;
  if (!build_layout(sh, &L)) return fail_inval("n_outlier_chunks / chunk count exceeds the selection kernels' capacity");
  rc = check_workspace(workspace, workspace_bytes, L.total);
  if (rc != SHADOWKV_OK) return rc;

  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  void* chunk_mean = ws + L.chunk_mean;
  double* min_cos = reinterpret_cast<double*>(ws + L.min_cos);
  hipError_t e = launch_chunk_stats(k_rope, sh.eb, chunk_mean, min_cos, sh.units, sh.d, sh.s, sh.c, st);
  if (e != hipSuccess) return fail_hip("chunk_stats", e);
  if (sh.o > 0) {
    SelectArgs a{};
    a.scores = min_cos; a.sign = -1.0;  // ArgTopK(-Min(S), o)
    a.n = sh.n_ch; a.k = sh.o;
    a.slice_len = L.sel.slice_len; a.n_slices = L.sel.n_slices; a.cand_stride = L.sel.cand_stride;
    a.cand_key = reinterpret_cast<uint64_t*>(ws + L.cand_key);
    a.cand_idx = reinterpret_cast<int32_t*>(ws + L.cand_idx);
    a.out_ids = outlier_chunk_ids;
    e = launch_select(a, L.sel, kSrcArray, sh.units, st);
    if (e != hipSuccess) return fail_hip("select outliers", e);
    e = launch_gather_outliers(k_rope, v, sh.eb, outlier_chunk_ids, k_outlier, v_outlier, sh.units, sh.d, sh.s, sh.cap,
                               sh.c, sh.o, st);
    if (e != hipSuccess) return fail_hip("gather outliers", e);
  }
  e = launch_compact_landmarks(chunk_mean, sh.eb, outlier_chunk_ids, landmarks, landmark_chunk_ids, sh.units, sh.d,
                               sh.n_ch, sh.o, sh.nc_cap, st);
  if (e != hipSuccess) return fail_hip("compact landmarks", e);
  return SHADOWKV_OK;
}

// Value cache handed to a cached step (all device pointers).
struct CacheIO {
  int slots;             // S >= k slots per unit
  void* values;          // [units, S*c, d] in the storage type of the KV cache
  int32_t* chunk_ids;    // [units, S], -1 = empty
  int32_t* stamps;       // [units, S + 1]: last use of each slot, then the unit's clock
  int32_t* miss_count;   // optional [units]
};

static int decode_impl(const shadowkv_params* params, const shadowkv_bf16* q, const shadowkv_kv* A,
                       const shadowkv_kv* B, const shadowkv_kv* landmarks, const int32_t* landmark_chunk_ids,
                       const shadowkv_kv* k_outlier, const shadowkv_kv* v_outlier,
                       const shadowkv_kv* k_local, const shadowkv_kv* v_local,
                       const shadowkv_kv* value_store, const int32_t* pos_offset, const CacheIO* cache,
                       shadowkv_bf16* out, int32_t* out_chunk_ids, void* workspace, size_t workspace_bytes,
                       void* stream, void* side_stream) {
  Shape sh;
  int rc = check_params(params, true, &sh);
  if (rc != SHADOWKV_OK) return rc;
  if (!q || !A || !B || !landmarks || !landmark_chunk_ids || !value_store || !out)
    return fail_inval("q, A, B, landmarks, landmark_chunk_ids, value_store and out must not be NULL");
  if (sh.o > 0 && (!k_outlier || !v_outlier)) return fail_inval("k_outlier / v_outlier is NULL with n_outlier_chunks > 0");
  if (sh.w > 0 && (!k_local || !v_local)) return fail_inval("k_local / v_local is NULL with local_len > 0");
  if (!aligned16(q) || !aligned16(A) || !aligned16(B) || !aligned16(landmarks) || !aligned16(k_outlier) ||
      !aligned16(v_outlier) || !aligned16(k_local) || !aligned16(v_local) || !aligned16(value_store) || !aligned16(out))
    return fail_inval("tensor pointers must be 16-byte aligned");
  if (cache) {
    if (!cache->values || !cache->chunk_ids || !cache->stamps)
      return fail_inval("value_cache, cache_chunk_ids and cache_stamps must not be NULL");
    if (!aligned16(cache->values)) return fail_inval("value_cache must be 16-byte aligned");
    if (cache->slots < sh.k || cache->slots > kMaxCacheSlots)
      return fail_inval("cache_slots %d must be in [topk_chunks = %d, %d]", cache->slots, sh.k, kMaxCacheSlots);
  }
  DecodeLayout L = decode_layout(sh);
  if (cache) L.attn = plan_attention(sh, true);
  rc = check_workspace(workspace, workspace_bytes, L.total);
  if (rc != SHADOWKV_OK) return rc;

  hipStream_t st = static_cast<hipStream_t>(stream);
  hipStream_t side = static_cast<hipStream_t>(side_stream);
  const bool fork = (sh.stage || cache) && side && side != st;
  char* ws = static_cast<char*>(workspace);
  float* logits = reinterpret_cast<float*>(ws + L.logits);
  double2* partials = reinterpret_cast<double2*>(ws + L.partials);
  int32_t* sel_ids = reinterpret_cast<int32_t*>(ws + L.sel_ids);
  void* v_sparse = sh.stage ? ws + L.v_sparse : nullptr;
  const double scale = params->softmax_scale != 0.0 ? params->softmax_scale : 1.0 / std::sqrt((double)sh.d);

  RopeFreqs freqs;
  for (int i = 0; i < sh.d / 2; ++i)
    freqs.rev[i] = std::pow(params->rope_theta, -2.0 * (double)i / (double)sh.d) / 6.283185307179586476925;
  for (int i = sh.d / 2; i < kMaxHalfDim; ++i) freqs.rev[i] = 0.0;

  std::lock_guard<std::mutex> lk(g_mu);  // one enqueue sequence at a time (the events are shared)
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  if (fork) {
    rc = get_events(&ev_fork, &ev_join);
    if (rc != SHADOWKV_OK) return rc;
  }

  const int pstep = (g_prof.on && g_prof.n_steps < g_prof.max_steps) ? g_prof.n_steps++ : -1;
  prof_mark(st, pstep, 0);
  // 1. P = Q L^T / sqrt(d), per-tile softmax statistics
  hipError_t e = launch_score(q, landmarks, sh.eb, logits, L.ld, partials, sh.b, sh.hq, sh.hkv, sh.d, sh.n_c, sh.nc_cap, scale, st);
  if (e != hipSuccess) return fail_hip("score", e);
  prof_mark(st, pstep, 1);
  // 2. softmax normaliser per head, max over the group, ArgTopK -> true chunk ids
  SelectArgs a{};
  a.logits = logits; a.partials = partials; a.n_tiles = L.n_tiles; a.G = sh.G; a.ld = L.ld;
  a.q = q; a.landmarks = landmarks; a.d = sh.d; a.kv_bytes = sh.eb; a.nc_stride = sh.nc_cap; a.scale = scale;
  a.lse_out = reinterpret_cast<double*>(ws + L.lse);
  a.key_top_out = reinterpret_cast<uint32_t*>(ws + L.key_top);
  a.n = sh.n_c; a.k = sh.k;
  a.slice_len = L.sel.slice_len; a.n_slices = L.sel.n_slices; a.cand_stride = L.sel.cand_stride;
  a.cand_key = reinterpret_cast<uint64_t*>(ws + L.cand_key);
  a.cand_idx = reinterpret_cast<int32_t*>(ws + L.cand_idx);
  a.id_map = landmark_chunk_ids; a.id_stride = sh.nc_cap;
  a.out_ids = sel_ids; a.out_ids2 = out_chunk_ids;
  // values readable in place: the attention over the resident rows [outliers ; recent] needs nothing of the
  // selection and rides its launch where that launch leaves room (its state is the last of each head's partials)
  const bool res_early = resident_rows_in_selection(sh, L, cache != nullptr);
  ResidentArgs ra{};
  if (res_early) {
    ra.q = q; ra.k_outlier = k_outlier; ra.v_outlier = v_outlier; ra.k_local = k_local; ra.v_local = v_local;
    ra.part_acc = reinterpret_cast<float*>(ws + L.part_acc);
    ra.part_ml = reinterpret_cast<float2*>(ws + L.part_ml);
    ra.hq = sh.hq; ra.hkv = sh.hkv; ra.oc = sh.o * sh.c; ra.w = sh.w;
    ra.n_part = L.attn.n_splits + 1; ra.part_slot = L.attn.n_splits;
    ra.head_blocks = (sh.G + 3) / 4; ra.units = sh.units;
    ra.scale_log2 = (float)(scale * 1.4426950408889634074);
  }
  e = launch_select(a, L.sel, kSrcLogits, sh.units, st, res_early ? &ra : nullptr, sh.d, sh.eb);
  if (e != hipSuccess) return fail_hip("select chunks", e);
  prof_mark(st, pstep, 2);
  AttnArgs t{};
  t.kv_bytes = sh.eb;
  t.q = q; t.A = A; t.B = B; t.k_outlier = k_outlier; t.v_outlier = v_outlier;
  t.k_local = k_local; t.v_local = v_local; t.v_store = value_store;
  t.sel_ids = sel_ids; t.pos_offset = pos_offset; t.inv_freq_dev = params->inv_freq;
  t.k_sparse_out = sh.keep_keys ? reinterpret_cast<float*>(ws + L.k_sparse) : nullptr;
  t.part_acc = reinterpret_cast<float*>(ws + L.part_acc);
  t.part_ml = reinterpret_cast<float2*>(ws + L.part_ml);
  t.logit_buf = reinterpret_cast<float*>(ws + L.logit_buf);
  t.out = out;
  t.s_cap = sh.cap;
  t.batch = sh.b; t.hq = sh.hq; t.hkv = sh.hkv; t.d = sh.d; t.s = sh.s; t.c = sh.c; t.o = sh.o; t.k = sh.k; t.w = sh.w;
  t.r = sh.r; t.r32 = (sh.r + 31) / 32 * 32; t.rp = t.r32 + 16;  // row pitch = 16 mod 32 elements: the 16-byte operand reads of a wave then spread evenly over the LDS banks (measured: twice the rate of +8)
  t.res_split_len = L.attn.res_split_len; t.sparse_split_len = L.attn.sparse_split_len; t.n_splits = L.attn.n_splits;
  t.pv_split_len = L.attn.pv_split_len; t.n_pv_splits = L.attn.n_pv_splits;
  t.v_unit_rows = sh.k * sh.c;
  t.c_shift = -1;
  for (int sft = 0; sft < 7; ++sft) if ((1 << sft) == sh.c) t.c_shift = sft;
  t.scale_log2 = (float)(scale * 1.4426950408889634074);
  t.freqs = freqs;

  if (!cache && !sh.stage) {
    // 3./4. values readable in place: one fused kernel rebuilds and rotates the keys and attends over
    //       [outliers ; selected ; recent]
    prof_mark(st, pstep, 3);
    t.n_part = t.n_splits + (res_early ? 1 : 0);
    t.skip_resident = res_early ? 1 : 0;
    e = launch_attention(t, st);
    if (e != hipSuccess) return fail_hip("attention", e);
    prof_mark(st, pstep, 4);
    return SHADOWKV_OK;
  }

  // 3. the selected values have to be brought in by a gather (all of them, or with a cache only the
  //    missing chunks).  It runs on the side stream while this stream does everything that needs none of
  //    them: the resident rows, and key rebuild + RoPE + q.K of the selected rows.
  int32_t* miss_slots = reinterpret_cast<int32_t*>(ws + L.miss_slots);
  int32_t* n_miss = reinterpret_cast<int32_t*>(ws + L.n_miss);
  int32_t* sel_slots = reinterpret_cast<int32_t*>(ws + L.sel_slots);
  if (cache) {
    e = launch_cache_update(sel_ids, cache->chunk_ids, cache->stamps, sel_slots, miss_slots, n_miss, cache->miss_count,
                            sh.units, sh.k, cache->slots, st);
    if (e != hipSuccess) return fail_hip("cache update", e);
  }
  // With a side stream the gather is a launch of its own there; without one it is done by the first
  // workgroups of the key-phase launch (no events between streams, and the step stays on one stream).
  const int vec_per_chunk = sh.c * sh.d * sh.eb / 16;
  if (fork) {
    if ((e = hipEventRecord(ev_fork, st)) != hipSuccess) return fail_hip("hipEventRecord", e);
    if ((e = hipStreamWaitEvent(side, ev_fork, 0)) != hipSuccess) return fail_hip("hipStreamWaitEvent", e);
  } else {
    GatherArgs& g = t.gather;
    g.store = static_cast<const uint4*>(value_store);
    g.units = sh.units; g.k = sh.k; g.vec_per_chunk = vec_per_chunk; g.last_chunk = sh.s / sh.c - 1;
    g.vec_per_unit_store = (size_t)sh.cap * sh.d * sh.eb / 16;
    if (cache) {
      g.dst = static_cast<uint4*>(cache->values); g.ids = cache->chunk_ids; g.miss_slots = miss_slots; g.n_miss = n_miss;
      g.slots_per_unit = cache->slots;
    } else {
      g.dst = static_cast<uint4*>(v_sparse); g.ids = sel_ids; g.miss_slots = nullptr; g.n_miss = nullptr;
      g.slots_per_unit = sh.k;
    }
    plan_gather(&g);
  }
  e = hipSuccess;
  if (cache) {
    if (fork)
      e = launch_gather_missing(value_store, cache->chunk_ids, miss_slots, n_miss, cache->values, sh.eb, sh.units, sh.d,
                                sh.s, sh.cap, sh.c, sh.k, cache->slots, side);
    t.v_sparse = cache->values; t.v_slots = sel_slots; t.v_unit_rows = cache->slots * sh.c;
  } else {
    if (fork)
      e = launch_gather_values(value_store, sel_ids, v_sparse, sh.eb, sh.units, sh.d, sh.s, sh.cap, sh.c, sh.k, side);
    t.v_sparse = v_sparse;
  }
  if (e != hipSuccess) return fail_hip("gather values", e);
  t.n_part = t.n_splits + t.n_pv_splits;
  e = launch_attention_keys(t, st);
  if (e != hipSuccess) return fail_hip("attention (keys)", e);
  if (fork) {
    if ((e = hipEventRecord(ev_join, side)) != hipSuccess) return fail_hip("hipEventRecord", e);
    if ((e = hipStreamWaitEvent(st, ev_join, 0)) != hipSuccess) return fail_hip("hipStreamWaitEvent", e);
  }
  prof_mark(st, pstep, 3);
  // 4. softmax of the stored logits times the gathered values, merge with the resident part
  e = launch_attention_values(t, st);
  if (e != hipSuccess) return fail_hip("attention (values)", e);
  prof_mark(st, pstep, 4);
  return SHADOWKV_OK;
}

int shadowkv_decode_step(const shadowkv_params* params, const shadowkv_bf16* q, const shadowkv_kv* A,
                         const shadowkv_kv* B, const shadowkv_kv* landmarks, const int32_t* landmark_chunk_ids,
                         const shadowkv_kv* k_outlier, const shadowkv_kv* v_outlier,
                         const shadowkv_kv* k_local, const shadowkv_kv* v_local,
                         const shadowkv_kv* value_store, const int32_t* pos_offset, shadowkv_bf16* out,
                         int32_t* out_chunk_ids, void* workspace, size_t workspace_bytes, void* stream,
                         void* side_stream) {
  return decode_impl(params, q, A, B, landmarks, landmark_chunk_ids, k_outlier, v_outlier, k_local, v_local,
                     value_store, pos_offset, nullptr, out, out_chunk_ids, workspace, workspace_bytes, stream,
                     side_stream);
}

size_t shadowkv_static_scratch_bytes(void) { return kStaticScratchBytes; }

int shadowkv_decode_step_static(const shadowkv_params* params, const shadowkv_bf16* q, const shadowkv_kv* A,
                                const shadowkv_kv* B, const shadowkv_kv* landmarks, const int32_t* landmark_chunk_ids,
                                const shadowkv_kv* k_outlier, const shadowkv_kv* v_outlier,
                                const shadowkv_kv* k_local, const shadowkv_kv* v_local,
                                const shadowkv_kv* value_store, const int32_t* pos_offset, shadowkv_bf16* out,
                                int32_t* out_chunk_ids, void* stream) {
  // the size check comes first: a shape that does not fit is rejected before anything touches the GPU
  Shape sh;
  int rc = check_params(params, true, &sh);
  if (rc != SHADOWKV_OK) return rc;
  const size_t need = decode_layout(sh).total;
  if (need > kStaticScratchBytes) {
    set_err("shape needs %zu bytes of scratch, the static scratch holds %zu: use shadowkv_decode_step with a workspace",
            need, kStaticScratchBytes);
    return SHADOWKV_EWORKSPACE;
  }
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != SHADOWKV_OK) return rc;
  return decode_impl(params, q, A, B, landmarks, landmark_chunk_ids, k_outlier, v_outlier, k_local, v_local,
                     value_store, pos_offset, nullptr, out, out_chunk_ids, ws, kStaticScratchBytes, stream, nullptr);
}

int shadowkv_decode_step_cached(const shadowkv_params* params, const shadowkv_bf16* q, const shadowkv_kv* A,
                                const shadowkv_kv* B, const shadowkv_kv* landmarks,
                                const int32_t* landmark_chunk_ids, const shadowkv_kv* k_outlier,
                                const shadowkv_kv* v_outlier, const shadowkv_kv* k_local,
                                const shadowkv_kv* v_local, const shadowkv_kv* value_store,
                                const int32_t* pos_offset, int32_t cache_slots, shadowkv_kv* value_cache,
                                int32_t* cache_chunk_ids, int32_t* cache_stamps, int32_t* out_miss_count,
                                shadowkv_bf16* out, int32_t* out_chunk_ids, void* workspace, size_t workspace_bytes,
                                void* stream, void* side_stream) {
  CacheIO c{cache_slots, value_cache, cache_chunk_ids, cache_stamps, out_miss_count};
  return decode_impl(params, q, A, B, landmarks, landmark_chunk_ids, k_outlier, v_outlier, k_local, v_local,
                     value_store, pos_offset, &c, out, out_chunk_ids, workspace, workspace_bytes, stream, side_stream);
}

int shadowkv_append_chunk(const shadowkv_params* params, const shadowkv_kv* k_pre, const shadowkv_kv* k_rope,
                          const shadowkv_kv* v, const shadowkv_kv* B, shadowkv_kv* A, shadowkv_kv* landmarks,
                          int32_t* landmark_chunk_ids, shadowkv_kv* value_store, void* stream) {
  Shape sh;
  int rc = check_params(params, false, &sh);
  if (rc != SHADOWKV_OK) return rc;
  if (params->rank < 8 || params->rank > 256 || params->rank % 8)
    return fail_inval("rank must be a multiple of 8 in [8, 256]");
  if (sh.s + sh.c > sh.cap)
    return fail_inval("no room for another chunk: ctx_len %d + chunk_size %d exceeds ctx_capacity %d", sh.s, sh.c, sh.cap);
  if (!k_pre || !k_rope || !v || !B || !A || !landmarks || !landmark_chunk_ids || !value_store)
    return fail_inval("k_pre, k_rope, v, B, A, landmarks, landmark_chunk_ids and value_store must not be NULL");
  if (!aligned16(k_pre) || !aligned16(k_rope) || !aligned16(v) || !aligned16(B) || !aligned16(A) ||
      !aligned16(landmarks) || !aligned16(value_store))
    return fail_inval("tensor pointers must be 16-byte aligned");
  hipError_t e = launch_append_chunk(k_pre, k_rope, v, B, A, landmarks, landmark_chunk_ids, value_store, sh.eb, sh.b,
                                     sh.hkv, sh.d, sh.s, sh.cap, sh.c, sh.r, sh.o, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip("append chunk", e);
  return SHADOWKV_OK;
}

constexpr int kFactorOversample = 32;  // extra vectors carried by the subspace iteration
constexpr int kFactorSweeps = 9;       // Jacobi sweeps of the Ritz step (converged to rounding after 7-8 for m <= 288)
constexpr int kFactorIters = 16;       // default number of subspace iterations

size_t shadowkv_factorize_workspace_bytes(const shadowkv_params* params) {
  Shape sh;
  if (check_params(params, false, &sh) != SHADOWKV_OK) return 0;
  if (params->rank < 8 || params->rank > 256 || params->rank % 8 || params->rank > sh.hkv * sh.d) return 0;
  return plan_factorize(sh.b, sh.s, sh.hkv * sh.d, params->rank, kFactorOversample).total;
}

int shadowkv_factorize_keys(const shadowkv_params* params, const shadowkv_kv* k_pre, shadowkv_kv* A, shadowkv_kv* B,
                            double* psi_out, double* sigma_out, int32_t n_iter, void* workspace, size_t workspace_bytes,
                            void* stream) {
  Shape sh;
  int rc = check_params(params, false, &sh);
  if (rc != SHADOWKV_OK) return rc;
  if (params->rank < 8 || params->rank > 256 || params->rank % 8)
    return fail_inval("rank must be a multiple of 8 in [8, 256]");
  if (params->rank > sh.hkv * sh.d) return fail_inval("rank %d exceeds the key width %d", params->rank, sh.hkv * sh.d);
  if (n_iter < 0 || n_iter > 1000) return fail_inval("n_iter must be in [0, 1000] (0 = default)");
  if (!k_pre || !A || !B) return fail_inval("k_pre, A and B must not be NULL");
  if (!aligned16(k_pre) || !aligned16(A) || !aligned16(B) || !aligned16(psi_out))
    return fail_inval("tensor pointers must be 16-byte aligned");
  const FactorizePlan pl = plan_factorize(sh.b, sh.s, sh.hkv * sh.d, params->rank, kFactorOversample);
  rc = check_workspace(workspace, workspace_bytes, pl.total);
  if (rc != SHADOWKV_OK) return rc;
  hipError_t e = launch_factorize(k_pre, sh.eb, A, B, psi_out, sigma_out, static_cast<char*>(workspace), pl, sh.b, sh.hkv,
                                  sh.d, sh.s, sh.cap, params->rank, n_iter ? n_iter : kFactorIters, kFactorSweeps,
                                  static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip("factorize keys", e);
  return SHADOWKV_OK;
}

size_t shadowkv_argtopk_workspace_bytes(int32_t units, int32_t n, int32_t k) {
  SelectPlan plan;
  if (units < 1 || units > 65535 || n < 1 || k < 1 || k > n || !plan_select(n, k, kSrcArray, units, &plan)) return 0;
  const size_t bytes = up((size_t)units * plan.cand_stride * sizeof(uint64_t)) +
                       up((size_t)units * plan.cand_stride * sizeof(int32_t));
  return bytes ? bytes : kAlign;
}

int shadowkv_argtopk(const double* scores, int32_t units, int32_t n, int32_t k, double sign, int32_t* out_ids,
                     void* workspace, size_t workspace_bytes, void* stream) {
  if (!scores || !out_ids) return fail_inval("scores and out_ids must not be NULL");
  if (units < 1 || units > 65535 || n < 1 || k < 1 || k > n) return fail_inval("need 1 <= k <= n and 1 <= units <= 65535");
  if (sign != 1.0 && sign != -1.0) return fail_inval("sign must be +1 or -1");
  SelectPlan plan;
  if (!plan_select(n, k, kSrcArray, units, &plan)) return fail_inval("n / k combination exceeds the selection kernels' capacity");
  int rc = check_workspace(workspace, workspace_bytes, shadowkv_argtopk_workspace_bytes(units, n, k));
  if (rc != SHADOWKV_OK) return rc;
  char* ws = static_cast<char*>(workspace);
  SelectArgs a{};
  a.scores = scores; a.sign = sign; a.n = n; a.k = k;
  a.slice_len = plan.slice_len; a.n_slices = plan.n_slices; a.cand_stride = plan.cand_stride;
  a.cand_key = reinterpret_cast<uint64_t*>(ws);
  a.cand_idx = reinterpret_cast<int32_t*>(ws + up((size_t)units * plan.cand_stride * sizeof(uint64_t)));
  a.out_ids = out_ids;
  hipError_t e = launch_select(a, plan, kSrcArray, units, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip("argtopk", e);
  return SHADOWKV_OK;
}

size_t shadowkv_value_cache_bytes(const shadowkv_params* params, int32_t cache_slots) {
  Shape sh;
  if (check_params(params, true, &sh) != SHADOWKV_OK) return 0;
  if (cache_slots < sh.k || cache_slots > kMaxCacheSlots) return 0;
  return (size_t)sh.units * cache_slots * sh.c * sh.d * sh.eb;
}

int shadowkv_value_cache_reset(const shadowkv_params* params, int32_t cache_slots, int32_t* cache_chunk_ids,
                               int32_t* cache_stamps, void* stream) {
  Shape sh;
  int rc = check_params(params, true, &sh);
  if (rc != SHADOWKV_OK) return rc;
  if (cache_slots < sh.k || cache_slots > kMaxCacheSlots)
    return fail_inval("cache_slots %d must be in [topk_chunks = %d, %d]", cache_slots, sh.k, kMaxCacheSlots);
  if (!cache_chunk_ids || !cache_stamps) return fail_inval("cache_chunk_ids / cache_stamps is NULL");
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = launch_fill_i32(cache_chunk_ids, (size_t)sh.units * cache_slots, -1, st);
  if (e == hipSuccess) e = launch_fill_i32(cache_stamps, (size_t)sh.units * (cache_slots + 1), 0, st);
  if (e != hipSuccess) return fail_hip("cache reset", e);
  return SHADOWKV_OK;
}

}  // extern "C"
