// C ABI of the FastGen hot path: argument validation, workspace carve-up, launch order.
// See include/fastgen.h for the contract of every entry point.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>

#include "fg_common.h"
#include "fg_internal.h"

// Scratch of fastgen_profile_static, the entry point that allocates nothing: one copy of this
// array lives on every GPU the library runs on, from module load until the process ends. In
// host code the name `scratch` is only a handle for hipGetSymbolAddress; the device address it
// yields (one per GPU) is what kernels and copies receive.
static constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];   // device address of `scratch`, per GPU (NULL: not asked yet)
static std::mutex g_scratch_mu;
static thread_local char g_static_err[256] = "";

namespace {

constexpr size_t kAlign = 256;
constexpr int FG_MAX_TOKENS = 131072;  // longest sequence (prompt + generated) a unit may reach

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

bool config_ok(const fg_config* c, char* why, size_t why_len) {
#define FG_REQUIRE(cond, msg)                 \
  if (!(cond)) {                              \
    if (why) snprintf(why, why_len, "%s", msg); \
    return false;                             \
  }
  FG_REQUIRE(c != nullptr, "config is NULL");
  FG_REQUIRE(c->num_units > 0 && c->num_units <= (1 << 24), "num_units out of range");
  FG_REQUIRE(c->num_seqs > 0 && c->num_units % c->num_seqs == 0, "num_seqs must divide num_units");
  FG_REQUIRE(c->head_dim == 64 || c->head_dim == 128, "head_dim must be 64 or 128");
  FG_REQUIRE(c->dtype == FG_F32 || c->dtype == FG_BF16, "dtype must be FG_F32 or FG_BF16");
  FG_REQUIRE(c->prompt_len >= 1 && c->prompt_len <= FG_MAX_TOKENS, "prompt_len out of range");
  FG_REQUIRE(c->max_new_tokens >= 0 && c->max_new_tokens <= FG_MAX_TOKENS, "max_new_tokens out of range");
  // the kernels index a unit's rows with 32-bit byte offsets (16 heads x 131072 rows x 512 B is
  // below 2^31) and the read-back kernel keeps a bitmap of n + S positions in shared memory
  FG_REQUIRE(c->prompt_len + c->max_new_tokens <= FG_MAX_TOKENS,
             "prompt_len + max_new_tokens must not exceed 131072");
  FG_REQUIRE(c->T > 0.0 && c->T <= 1.0, "T must be in (0, 1]");
  FG_REQUIRE(c->r_l >= 0.0 && c->r_l <= 1.0, "r_l must be in [0, 1]");
  FG_REQUIRE(c->r_f >= 0.0 && c->r_f <= 1.0, "r_f must be in [0, 1]");
  FG_REQUIRE(c->softmax_scale >= 0.f && isfinite(c->softmax_scale), "softmax_scale must be >= 0");
  FG_REQUIRE(c->forced_policy >= -1 && c->forced_policy <= 4, "forced_policy must be -1..4");
  FG_REQUIRE(c->cache_tokens >= 0, "cache_tokens must be >= 0");
  {
    // the flat work list of the decode kernels (one item per 128 or 256 reserved slots) is a 32-bit grid
    const long long full = (long long)c->prompt_len + c->max_new_tokens;
    const long long pool = c->cache_tokens > 0 ? c->cache_tokens : (long long)c->num_units * full;
    FG_REQUIRE(pool / fg_decode_chunk(c->prompt_len, c->max_new_tokens) + c->num_units < (1ll << 31) - 1, "cache pool too large for the decode work list");
  }
  FG_REQUIRE(c->group_size >= 0 && c->group_size <= 16, "group_size must be 0..16");
  bool any = false;
  for (int i = 0; i < 4; ++i) {
    FG_REQUIRE(c->family[i] >= 0 && c->family[i] <= 15, "family entries must be FG_COMP_* masks (0..15)");
    any = any || c->family[i] != 0;
  }
  FG_REQUIRE(!any || c->forced_policy < 0 || c->forced_policy == 4 || c->family[c->forced_policy] != 0,
             "forced_policy names an unused family entry");
#undef FG_REQUIRE
  return true;
}

// component masks of policy ids 0..3: the configured table, or the family of Eq. 2
void family_of(const fg_config& c, int* out) {
  const bool any = c.family[0] || c.family[1] || c.family[2] || c.family[3];
  const int eq2[4] = {FG_COMP_SPECIAL, FG_COMP_SPECIAL | FG_COMP_PUNCT,
                      FG_COMP_SPECIAL | FG_COMP_PUNCT | FG_COMP_FREQUENT,
                      FG_COMP_SPECIAL | FG_COMP_PUNCT | FG_COMP_FREQUENT | FG_COMP_LOCAL};
  for (int i = 0; i < 4; ++i) out[i] = any ? c.family[i] : eq2[i];
}

int group_of(const fg_config& c) { return c.group_size > 1 ? c.group_size : 1; }

// Regions that fastgen_profile writes (the profiling scratch and the per-unit results); they
// come first in the workspace. Returns the bytes they take.
size_t layout_profile_part(const fg_config& c, fg_layout& L) {
  const size_t G = (size_t)group_of(c);
  const size_t U = (size_t)c.num_units, n = (size_t)c.prompt_len;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  L.rowstat = take(U * G * n * 8);
  L.colsum = take(U * n * 8);
  L.bandcol = take(U * n * 8);
  L.keep = take(U * n);
  L.slot = take(U * n * 4);
  L.policy = take(U * 4);
  L.recov = take(U * 5 * 8);
  L.kcount = take(U * 5 * 4);
  L.cap = take(U * 4);
  L.off = take((U + 1) * 8);
  L.len = take(U * 4);
  L.flags = take(8 * 4);
  return o;
}

fg_layout make_layout(const fg_config& c) {
  fg_layout L;
  memset(&L, 0, sizeof(L));
  const size_t G = (size_t)group_of(c);
  const size_t U = (size_t)c.num_units, n = (size_t)c.prompt_len, d = (size_t)c.head_dim;
  const size_t e = c.dtype == FG_BF16 ? 2 : 4;
  const size_t full = n + (size_t)c.max_new_tokens;
  const size_t pool = c.cache_tokens > 0 ? (size_t)c.cache_tokens : U * full;
  L.pool_tokens = (int64_t)pool;
  L.chunk = fg_decode_chunk(c.prompt_len, c.max_new_tokens);
  L.max_chunks = (int64_t)(pool / (size_t)L.chunk + U);
  size_t o = layout_profile_part(c, L);
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  L.ck = take(pool * d * e);
  L.cv = take(pool * d * e);
  L.cscore = take(pool * 8);
  L.cpos = take(pool * 4);
  L.ccls = take(pool);
  L.clogit = take(pool * G * 8);
  L.chunk_off = take((U + 1) * 4);
  L.item_unit = take((size_t)L.max_chunks * 32);
  L.part = take((size_t)L.max_chunks * G * (d + 2) * 4);
  L.total = o;
  return L;
}

fg_status fail(fastgen_ctx* ctx, fg_status st, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return st;
}

// failure of a call that has no context: the message is kept per host thread
__attribute__((format(printf, 2, 3))) fg_status sfail(fg_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_static_err, sizeof(g_static_err), fmt, ap);
  va_end(ap);
  return st;
}

fg_status hip_fail(fastgen_ctx* ctx, hipError_t e, const char* where) {
  return fail(ctx, FG_EHIP, "%s: %s", where, hipGetErrorString(e));
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <class T>
T* at(fastgen_ctx* ctx, size_t off) { return reinterpret_cast<T*>(ctx->ws + off); }

// Device-time accounting of the kernel groups of one API call: consecutive groups share the
// event between them (an event record costs several microseconds on the stream).
struct PhaseChain {
  fastgen_ctx* ctx; hipStream_t s; bool on; int last = -1, open_phase = -1, open_a = -1;
  PhaseChain(fastgen_ctx* c, hipStream_t st, bool enabled) : ctx(c), s(st), on(enabled) {}
  int record() {
    hipEvent_t e;
    if (!ctx->spare.empty()) { e = ctx->spare.back(); ctx->spare.pop_back(); }
    else if (hipEventCreate(&e) != hipSuccess) { on = false; return -1; }
    (void)hipEventRecord(e, s);
    ctx->events.push_back(e);
    return (int)ctx->events.size() - 1;
  }
  void begin(int phase) {
    if (!on) return;
    open_a = last >= 0 ? last : record();
    open_phase = phase;
  }
  void end() {
    if (!on || open_phase < 0) return;
    const int b = record();
    if (b >= 0 && open_a >= 0) ctx->pending.push_back({open_phase, open_a, b});
    last = b;
    open_phase = -1;
  }
};

// The kernels of stage 1a in launch order, over scratch regions `L` inside `ws`. Shared by
// fastgen_profile (regions in the caller's workspace) and fastgen_profile_static (regions in
// the library's own static device array).
hipError_t launch_profile_path(const fg_config& c, const fg_layout& L, char* ws, float scale, int w,
                               const void* Q, const void* K, const uint8_t* token_class,
                               const float* lse_opt, int32_t* policy, double* recovery,
                               int32_t* kept_count, hipStream_t s, PhaseChain& tm, const char** where) {
  auto at = [&](size_t off) { return ws + off; };
  fg_profile_args pa;
  pa.Q = Q; pa.K = K;
  pa.rowstat = reinterpret_cast<float2*>(at(L.rowstat));
  pa.colsum = reinterpret_cast<double*>(at(L.colsum));
  pa.bandcol = reinterpret_cast<double*>(at(L.bandcol));
  pa.U = c.num_units; pa.n = c.prompt_len; pa.d = c.head_dim; pa.w = w; pa.G = group_of(c);
  pa.scale = scale;
  hipError_t e;
  *where = "fastgen_profile(row log-sum-exp sweep)";
  tm.begin(FG_PHASE_SWEEP1);
  if (lse_opt) e = fg_launch_lse_to_rowstat(lse_opt, pa.rowstat, (size_t)c.num_units * pa.G * c.prompt_len, s);
  else e = (c.dtype == FG_BF16) ? fg_launch_profile_bf16(pa, 1, s) : fg_launch_profile_f32(pa, 1, s);
  tm.end();
  if (e != hipSuccess) return e;
  *where = "fastgen_profile(column sweep)";
  tm.begin(FG_PHASE_SWEEP2);
  e = (c.dtype == FG_BF16) ? fg_launch_profile_bf16(pa, 2, s) : fg_launch_profile_f32(pa, 2, s);
  tm.end();
  if (e != hipSuccess) return e;

  fg_select_args sa;
  sa.colsum = pa.colsum; sa.bandcol = pa.bandcol; sa.token_class = token_class;
  sa.keep = reinterpret_cast<uint8_t*>(at(L.keep)); sa.slot = reinterpret_cast<int32_t*>(at(L.slot));
  sa.policy = reinterpret_cast<int32_t*>(at(L.policy)); sa.recov = reinterpret_cast<double*>(at(L.recov));
  sa.kcount = reinterpret_cast<int32_t*>(at(L.kcount)); sa.cap = reinterpret_cast<int32_t*>(at(L.cap));
  sa.len = reinterpret_cast<int32_t*>(at(L.len));
  sa.policy_out = policy; sa.recov_out = recovery; sa.kcount_out = kept_count;
  sa.U = c.num_units; sa.n = c.prompt_len; sa.units_per_seq = c.num_units / c.num_seqs;
  sa.w = w; sa.S = c.max_new_tokens; sa.T = c.T; sa.r_f = c.r_f; sa.G = pa.G;
  sa.forced_policy = c.forced_policy;
  family_of(c, sa.family);
  *where = "fastgen_profile(select)";
  tm.begin(FG_PHASE_SELECT);
  e = fg_launch_select(sa, s);
  tm.end();
  return e;
}

float scale_of(const fg_config& c) {
  return c.softmax_scale > 0.f ? c.softmax_scale : 1.0f / sqrtf((float)c.head_dim);
}

int window_of(const fg_config& c) {
  const int w = fg_budget(c.r_l, c.prompt_len);
  return w < 1 ? 1 : w;
}

}  // namespace

extern "C" {

size_t fastgen_workspace_bytes(const fg_config* cfg) {
  if (!config_ok(cfg, nullptr, 0)) return 0;
  return make_layout(*cfg).total;
}

fg_status fastgen_create(const fg_config* cfg, void* workspace, size_t bytes, fastgen_ctx** out) {
  if (!out) return FG_EINVAL;
  *out = nullptr;
  char why[128];
  if (!config_ok(cfg, why, sizeof(why))) return FG_EINVAL;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0) return FG_EINVAL;
  fg_layout lay = make_layout(*cfg);
  if (bytes < lay.total) return FG_ENOMEM;
  fastgen_ctx* ctx = new (std::nothrow) fastgen_ctx();
  if (!ctx) return FG_ENOMEM;
  ctx->timing = 0;
  ctx->cfg = *cfg;
  ctx->lay = lay;
  ctx->ws = static_cast<char*>(workspace);
  ctx->scale = scale_of(*cfg);
  ctx->w = window_of(*cfg);
  ctx->stage = 0;
  ctx->steps_done = 0;
  ctx->err[0] = '\0';
  *out = ctx;
  return FG_OK;
}

fg_status fastgen_destroy(fastgen_ctx* ctx) {
  if (!ctx) return FG_OK;
  for (auto e : ctx->events) (void)hipEventDestroy(e);
  for (auto e : ctx->spare) (void)hipEventDestroy(e);
  delete ctx;
  return FG_OK;
}

fg_status fastgen_enable_timing(fastgen_ctx* ctx, int enable) {
  if (!ctx) return FG_EINVAL;
  ctx->timing = enable < 0 ? 0 : enable;
  return FG_OK;
}

fg_status fastgen_read_timing(fastgen_ctx* ctx, double* ms, int64_t* launches) {
  if (!ctx) return FG_EINVAL;
  if (!ms) return fail(ctx, FG_EINVAL, "fastgen_read_timing: ms is required");
  for (int i = 0; i < FG_NUM_PHASES; ++i) { ms[i] = 0.0; if (launches) launches[i] = 0; }
  fg_status st = FG_OK;
  for (auto& r : ctx->pending) {
    float t = 0.f;
    hipError_t e = hipEventSynchronize(ctx->events[r.b]);
    if (e == hipSuccess) e = hipEventElapsedTime(&t, ctx->events[r.a], ctx->events[r.b]);
    if (e != hipSuccess) st = hip_fail(ctx, e, "fastgen_read_timing");
    else { ms[r.phase] += (double)t; if (launches) launches[r.phase] += 1; }
  }
  for (auto e : ctx->events) ctx->spare.push_back(e);
  ctx->events.clear();
  ctx->pending.clear();
  return st;
}

fg_status fastgen_classify(const int32_t* token_ids, int64_t count, const int32_t* special_ids,
                           int32_t num_special, const int32_t* punct_ids, int32_t num_punct,
                           uint8_t* token_class, void* stream) {
  if (count < 0 || count > ((int64_t)1 << 38)) return sfail(FG_EINVAL, "fastgen_classify: count out of range");
  if (num_special < 0 || num_special > FG_MAX_CLASS_IDS || num_punct < 0 || num_punct > FG_MAX_CLASS_IDS)
    return sfail(FG_EINVAL, "fastgen_classify: an id list holds at most %d entries", FG_MAX_CLASS_IDS);
  if ((num_special > 0 && !special_ids) || (num_punct > 0 && !punct_ids))
    return sfail(FG_EINVAL, "fastgen_classify: an id list is NULL but its count is not 0");
  if (count == 0) return FG_OK;
  if (!token_ids || !token_class) return sfail(FG_EINVAL, "fastgen_classify: token_ids and token_class are required");
  fg_classify_args a;
  memset(&a, 0, sizeof(a));
  a.token_ids = token_ids; a.token_class = token_class; a.count = count;
  a.num_special = num_special; a.num_punct = num_punct;
  for (int i = 0; i < num_special; ++i) a.special[i] = special_ids[i];
  for (int i = 0; i < num_punct; ++i) a.punct[i] = punct_ids[i];
  const hipError_t e = fg_launch_classify(a, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return sfail(FG_EHIP, "fastgen_classify: %s", hipGetErrorString(e));
  return FG_OK;
}

fg_status fastgen_profile(fastgen_ctx* ctx, const void* Q, const void* K, const uint8_t* token_class,
                          const float* lse_opt, int32_t* policy, double* recovery,
                          int32_t* kept_count, void* stream) {
  if (!ctx) return FG_EINVAL;
  if (!Q || !K || !token_class) return fail(ctx, FG_EINVAL, "fastgen_profile: Q, K and token_class are required");
  if (!aligned16(Q) || !aligned16(K)) return fail(ctx, FG_EINVAL, "fastgen_profile: Q and K must be 16-byte aligned");
  if (ctx->stage != 0) return fail(ctx, FG_ESTATE, "fastgen_profile: context already profiled");
  hipStream_t s = static_cast<hipStream_t>(stream);
  PhaseChain tm(ctx, s, ctx->timing != 0);
  const char* where = "";
  const hipError_t e = launch_profile_path(ctx->cfg, ctx->lay, ctx->ws, ctx->scale, ctx->w, Q, K, token_class,
                                           lse_opt, policy, recovery, kept_count, s, tm, &where);
  if (e != hipSuccess) return hip_fail(ctx, e, where);
  ctx->stage = 1;
  return FG_OK;
}

fg_status fastgen_profile_static(const fg_config* cfg, const void* Q, const void* K,
                                 const uint8_t* token_class, const float* lse_opt, int32_t* policy,
                                 double* recovery, int32_t* kept_count, void* stream) {
  char why[128] = "";
  if (!config_ok(cfg, why, sizeof(why))) return sfail(FG_EINVAL, "fastgen_profile_static: %s", why);
  if (!Q || !K || !token_class) return sfail(FG_EINVAL, "fastgen_profile_static: Q, K and token_class are required");
  if (!aligned16(Q) || !aligned16(K)) return sfail(FG_EINVAL, "fastgen_profile_static: Q and K must be 16-byte aligned");
  fg_layout L;
  memset(&L, 0, sizeof(L));
  const size_t need = layout_profile_part(*cfg, L);
  if (need > kStaticScratchBytes)
    return sfail(FG_ENOMEM, "fastgen_profile_static: this shape needs %zu bytes of scratch, the static array holds %zu",
                 need, kStaticScratchBytes);
  // device address of this GPU's copy of the array (asked once per device, with it current)
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return sfail(FG_EHIP, "fastgen_profile_static(hipGetDevice): %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return sfail(FG_EINVAL, "fastgen_profile_static: device index %d not supported", dev);
  void* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p)
        return sfail(FG_EHIP, "fastgen_profile_static(hipGetSymbolAddress): %s", hipGetErrorString(e));
      g_scratch_ptr[dev] = p;
    }
    base = g_scratch_ptr[dev];
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  PhaseChain tm(nullptr, s, false);
  const char* where = "";
  // every region the kernels read is written first by an earlier kernel of this call for all
  // U * n entries in use, so nothing left over from the previous call needs clearing
  e = launch_profile_path(*cfg, L, static_cast<char*>(base), scale_of(*cfg), window_of(*cfg), Q, K, token_class,
                          lse_opt, policy, recovery, kept_count, s, tm, &where);
  if (e != hipSuccess) return sfail(FG_EHIP, "%s: %s", where, hipGetErrorString(e));
  return FG_OK;
}

fg_status fastgen_compact(fastgen_ctx* ctx, const void* K, const void* V, void* stream) {
  if (!ctx) return FG_EINVAL;
  if (!K || !V) return fail(ctx, FG_EINVAL, "fastgen_compact: K and V are required");
  if (!aligned16(K) || !aligned16(V)) return fail(ctx, FG_EINVAL, "fastgen_compact: K and V must be 16-byte aligned");
  if (ctx->stage != 1) return fail(ctx, FG_ESTATE, "fastgen_compact: needs fastgen_profile first (once)");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const fg_config& c = ctx->cfg;
  const fg_layout& L = ctx->lay;
  PhaseChain tm(ctx, s, ctx->timing != 0);
  tm.begin(FG_PHASE_COMPACT);
  hipError_t e = fg_launch_offsets(at<int32_t>(ctx, L.cap), at<int32_t>(ctx, L.len), at<int32_t>(ctx, L.policy),
                                   at<int64_t>(ctx, L.off), at<int32_t>(ctx, L.chunk_off), at<int32_t>(ctx, L.item_unit),
                                   at<int32_t>(ctx, L.flags), c.num_units, L.pool_tokens,
                                   L.max_chunks, L.chunk, s);
  if (e != hipSuccess) return hip_fail(ctx, e, "fastgen_compact(offsets)");
  fg_compact_args ca;
  ca.K = K; ca.V = V;
  ca.colsum = at<double>(ctx, L.colsum); ca.keep = at<uint8_t>(ctx, L.keep);
  ca.slot = at<int32_t>(ctx, L.slot); ca.cap = at<int32_t>(ctx, L.cap);
  ca.off = at<int64_t>(ctx, L.off); ca.len = at<int32_t>(ctx, L.len);
  ca.flags = at<int32_t>(ctx, L.flags);
  ca.ck = at<void>(ctx, L.ck); ca.cv = at<void>(ctx, L.cv);
  ca.cscore = at<double>(ctx, L.cscore); ca.cpos = at<int32_t>(ctx, L.cpos);
  ca.ccls = at<uint8_t>(ctx, L.ccls);
  ca.U = c.num_units; ca.n = c.prompt_len; ca.d = c.head_dim;
  ca.esize = c.dtype == FG_BF16 ? 2 : 4;
  ca.units_per_seq = c.num_units / c.num_seqs;
  ca.pool_tokens = L.pool_tokens;
  e = fg_launch_compact(ca, s);
  tm.end();
  if (e != hipSuccess) return hip_fail(ctx, e, "fastgen_compact(gather)");
  ctx->stage = 2;
  ctx->steps_done = 0;
  return FG_OK;
}

static fg_status decode_step_impl(fastgen_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                                  const uint8_t* class_new, void* out, double* probe, void* stream) {
  if (!ctx) return FG_EINVAL;
  if (!q || !k_new || !v_new || !class_new || !out)
    return fail(ctx, FG_EINVAL, "fastgen_decode_step: q, k_new, v_new, class_new and out are required");
  if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(out))
    return fail(ctx, FG_EINVAL, "fastgen_decode_step: q, k_new, v_new, out must be 16-byte aligned");
  if (ctx->stage != 2) return fail(ctx, FG_ESTATE, "fastgen_decode_step: needs fastgen_compact first");
  const fg_config& c = ctx->cfg;
  if (ctx->steps_done >= c.max_new_tokens)
    return fail(ctx, FG_ECAP, "fastgen_decode_step: max_new_tokens (%d) steps already done", c.max_new_tokens);
  const fg_layout& L = ctx->lay;
  fg_decode_args da;
  da.q = q; da.k_new = k_new; da.v_new = v_new; da.class_new = class_new; da.out = out;
  da.policy = at<int32_t>(ctx, L.policy); da.cap = at<int32_t>(ctx, L.cap);
  da.off = at<int64_t>(ctx, L.off); da.len = at<int32_t>(ctx, L.len);
  da.flags = at<int32_t>(ctx, L.flags);
  da.ck = at<void>(ctx, L.ck); da.cv = at<void>(ctx, L.cv);
  da.cscore = at<double>(ctx, L.cscore); da.cpos = at<int32_t>(ctx, L.cpos);
  da.ccls = at<uint8_t>(ctx, L.ccls); da.clogit = at<double>(ctx, L.clogit);
  da.chunk_off = at<int32_t>(ctx, L.chunk_off); da.item_unit = at<int32_t>(ctx, L.item_unit);
  da.part = at<float>(ctx, L.part);
  da.U = c.num_units; da.n = c.prompt_len; da.d = c.head_dim; da.dtype = c.dtype;
  da.units_per_seq = c.num_units / c.num_seqs; da.w = ctx->w; da.step = ctx->steps_done;
  da.G = group_of(c);
  da.r_f = c.r_f; da.scale = ctx->scale; da.max_chunks = L.max_chunks; da.chunk = L.chunk;
  da.probe = probe;
  family_of(c, da.family);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  PhaseChain tm(ctx, s, ctx->timing == 1 || (ctx->timing > 1 && ctx->steps_done % ctx->timing == 0));
  tm.begin(FG_PHASE_DECODE_ATTN);
  e = fg_launch_decode_attn(da, s);
  tm.end();
  if (e != hipSuccess) return hip_fail(ctx, e, "fastgen_decode_step(attention)");
  tm.begin(FG_PHASE_DECODE_UPDATE);
  e = fg_launch_decode_update(da, s);
  tm.end();
  if (e != hipSuccess) return hip_fail(ctx, e, "fastgen_decode_step(update)");
  ctx->steps_done += 1;
  return FG_OK;
}

fg_status fastgen_decode_step(fastgen_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                              const uint8_t* class_new, void* out, void* stream) {
  return decode_step_impl(ctx, q, k_new, v_new, class_new, out, nullptr, stream);
}

fg_status fastgen_decode_step_probe(fastgen_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                                    const uint8_t* class_new, void* out, double* step_recovery,
                                    void* stream) {
  if (!ctx) return FG_EINVAL;
  if (!step_recovery) return fail(ctx, FG_EINVAL, "fastgen_decode_step_probe: step_recovery is required");
  return decode_step_impl(ctx, q, k_new, v_new, class_new, out, step_recovery, stream);
}

fg_status fastgen_export_state(fastgen_ctx* ctx, int32_t* lengths, int64_t* offsets, int32_t* positions,
                               double* scores, void* keys, void* values, int32_t* status,
                               void* stream) {
  if (!ctx) return FG_EINVAL;
  if (ctx->stage != 2) return fail(ctx, FG_ESTATE, "fastgen_export_state: needs fastgen_compact first");
  if ((positions || scores || keys || values) && !offsets)
    return fail(ctx, FG_EINVAL, "fastgen_export_state: packed outputs need `offsets`");
  const fg_config& c = ctx->cfg;
  const fg_layout& L = ctx->lay;
  fg_export_args ea;
  ea.off = at<int64_t>(ctx, L.off); ea.len = at<int32_t>(ctx, L.len);
  ea.flags = at<int32_t>(ctx, L.flags);
  ea.ck = at<void>(ctx, L.ck); ea.cv = at<void>(ctx, L.cv);
  ea.cscore = at<double>(ctx, L.cscore); ea.cpos = at<int32_t>(ctx, L.cpos);
  ea.lengths = lengths; ea.offsets = offsets; ea.positions = positions; ea.scores = scores;
  ea.keys = keys; ea.values = values; ea.status = status;
  ea.U = c.num_units; ea.d = c.head_dim; ea.esize = c.dtype == FG_BF16 ? 2 : 4;
  ea.max_pos = c.prompt_len + c.max_new_tokens;
  hipError_t e = fg_launch_export(ea, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(ctx, e, "fastgen_export_state");
  return FG_OK;
}

const char* fastgen_last_error(const fastgen_ctx* ctx) { return ctx ? ctx->err : g_static_err; }

const char* fastgen_version(void) { return "fastgen-mi355x 0.2 (gfx950)"; }

}  // extern "C"
