// C-ABI of the LASER-KV block-selection library: argument checks, workspace, launch sequence.
#include "../../include/laserkv.h"
#include "../../include/laserkv_profile.h"
#include "laserkv_kernels.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

namespace {

constexpr int kMaxBlock = 16384;
constexpr int kMaxRows = 1024;   // G * W
constexpr int kMaxPlanes = 512;  // L * K

char g_error[512] = "";

constexpr int kMaxDevices = 64;

}  // namespace

// Workspace of laserkv_compress_block_static: one copy per GPU, held until the process ends.  The name is
// a host-side stand-in; host code uses the per-device address from hipGetSymbolAddress (static_device()).
static __device__ __align__(256) unsigned char scratch[LKV_STATIC_SCRATCH_BYTES];

struct laserkv_ctx {
  laserkv_config cfg;
  int device;
  int n_cu;
  int group;
  int elem_size;
  // device workspace
  int max_ranges;    // key ranges per (head, query-row group) the workspace is sized for
  float2* part;      // [H_kv, m_pad, max_ranges]
  float* s_part;     // [n_qgroups_max, H_kv, max_block]
  float* s_exact;    // [H_kv, max_block]
  int32_t* cnt;      // [n_qgroups_max, H_kv, max_block] count parts
  int32_t* cnt_sum;  // [H_kv, max_block] summed counts (stage output)
  uint32_t* qhist;   // [H_kv, L, 2^K / 2, n_qgroups] or null when the tables are too large
  uint32_t* sync;    // single sweep: [0] epoch, [1] finished workgroups, [64 ..] per-table flags [H_kv, L]; null without qhist
  uint16_t* sig_k;   // [H_kv, max_block, L]
  uint16_t* sig_q;   // [H_q, max_window, L]
  int m_pad;
  bool owns_workspace;   // the buffers above came from hipMalloc and are freed by laserkv_destroy
  const float* row_lse;  // laserkv_set_row_lse: applies to every following scoring call until reset
  bool row_lse_complete; // the rows' complete log-sum-exp (laserkv_set_row_lse_complete) rather than outside keys only
  int only_kernel;   // >= 0: launch only this kernel kind (laserkv_profile_isolate); -1 normally
  // tuning switches, read from the environment once when the context is created
  int sweep_wg_per_cu;   // LASERKV_SWEEP_WG_PER_CU: sweep workgroups aimed at per compute unit (default 1)
  int append_split;      // LASERKV_APPEND_SPLIT: select+append workgroups per head (default: n_cu / heads)
  int single_spin;       // LASERKV_SINGLE_SPIN: polls of a histogram flag before a workgroup computes the table itself
                         // (default 64; negative: the single sweep is not used)
  char error[512];
  // per-kernel event timing (benchmarks only)
  bool profiling;
  std::vector<hipEvent_t>* ev_pool;   // pairs: [2*i] start, [2*i+1] stop
  std::vector<int>* ev_kind;          // kernel id of recorded pair i
};

namespace {

int fail(laserkv_ctx* ctx, int code, const char* fmt, ...) {
  char* dst = ctx ? ctx->error : g_error;
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(dst, 512, fmt, ap);
  va_end(ap);
  return code;
}

int fail_hip(laserkv_ctx* ctx, hipError_t e, const char* what) {
  return fail(ctx, LKV_EHIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  if (!v || !*v) return dflt;
  return atoi(v);
}

int bits_for(int64_t v) {
  int b = 1;
  while ((int64_t(1) << b) <= v) ++b;
  return b;
}

// Runs `launch` bracketed by an event pair when the context is profiling.
template <typename F>
hipError_t timed(laserkv_ctx* ctx, int kind, hipStream_t st, F launch) {
  if (ctx->only_kernel >= 0 && ctx->only_kernel != kind) return hipSuccess;  // benchmark isolation
  if (!ctx->profiling || ctx->ev_kind->size() >= LKV_PROFILE_MAX_LAUNCHES) return launch();
  const size_t i = ctx->ev_kind->size();
  while (ctx->ev_pool->size() < 2 * (i + 1)) {
    hipEvent_t ev;
    hipError_t e = hipEventCreate(&ev);
    if (e != hipSuccess) return e;
    ctx->ev_pool->push_back(ev);
  }
  hipError_t e = hipEventRecord((*ctx->ev_pool)[2 * i], st);
  if (e != hipSuccess) return e;
  e = launch();
  if (e != hipSuccess) return e;
  e = hipEventRecord((*ctx->ev_pool)[2 * i + 1], st);
  if (e != hipSuccess) return e;
  ctx->ev_kind->push_back(kind);
  return hipSuccess;
}


// Configuration limits shared by every entry point that takes a laserkv_config.
int check_config(const laserkv_config& c, const char* who) {
  if (c.n_kv_heads < 1 || c.n_q_heads < c.n_kv_heads || c.n_q_heads % c.n_kv_heads)
    return fail(nullptr, LKV_EINVAL, "%s: n_kv_heads must divide n_q_heads", who);
  if (c.head_dim != 64 && c.head_dim != 128) return fail(nullptr, LKV_EINVAL, "%s: head_dim must be 64 or 128", who);
  if (c.dtype != LKV_F32 && c.dtype != LKV_BF16) return fail(nullptr, LKV_EINVAL, "%s: unknown dtype", who);
  if (c.lsh_tables < 1 || c.lsh_bits < 1 || c.lsh_bits > 16 || c.lsh_tables * c.lsh_bits > kMaxPlanes)
    return fail(nullptr, LKV_EINVAL, "%s: need 1 <= K <= 16 and L*K <= %d", who, kMaxPlanes);
  if (c.max_block < 1 || c.max_block > kMaxBlock) return fail(nullptr, LKV_EINVAL, "%s: max_block must be 1..%d", who, kMaxBlock);
  if (c.max_window < 1 || (int64_t)(c.n_q_heads / c.n_kv_heads) * c.max_window > kMaxRows)
    return fail(nullptr, LKV_EINVAL, "%s: G * max_window must be 1..%d", who, kMaxRows);
  if (c.max_ctx_keys < 0) return fail(nullptr, LKV_EINVAL, "%s: max_ctx_keys < 0", who);
  return LKV_OK;
}

// The device workspace of a configuration: nine buffers, in the order of WsIndex.
constexpr int kWsBuffers = 9;
enum WsIndex { WS_PART, WS_S_PART, WS_S_EXACT, WS_CNT, WS_CNT_SUM, WS_SIG_K, WS_SIG_Q, WS_QHIST, WS_SYNC };
struct WsPlan {
  int m_pad, max_ranges;
  size_t bytes[kWsBuffers];  // 0: buffer not used by this configuration
  size_t total() const {
    size_t t = 0;
    for (size_t b : bytes) t += (b + 255) & ~(size_t)255;
    return t;
  }
};

void plan_workspace(const laserkv_config& c, bool allow_qhist, WsPlan& w) {
  const int group = c.n_q_heads / c.n_kv_heads;
  const int m_rows = group * c.max_window;
  const int rows_per_group = lkv::sweep_rows_per_group();
  w.m_pad = (m_rows + rows_per_group - 1) / rows_per_group * rows_per_group;
  const size_t n_qg_max = w.m_pad / rows_per_group;
  // a key range never has fewer than 32 keys (wide rows and many planes shrink it that far), and the
  // look-back keys have ranges of their own
  w.max_ranges = ((c.max_block + 31) / 32 + (c.max_ctx_keys + 31) / 32 + 7) & ~7;
  // histograms of the query codes (one per query-row group) are kept in global memory between the two
  // sweeps when a head's tables fit 512 KiB per group
  const size_t hist_bytes_head = ((size_t)c.lsh_tables << c.lsh_bits) * 2;
  const bool use_qhist = allow_qhist && hist_bytes_head <= 512 * 1024;
  const size_t hk = c.n_kv_heads, sb = c.max_block;
  w.bytes[WS_PART] = hk * w.max_ranges * w.m_pad * sizeof(float2);
  w.bytes[WS_S_PART] = n_qg_max * hk * sb * sizeof(float);
  w.bytes[WS_S_EXACT] = hk * sb * sizeof(float);
  w.bytes[WS_CNT] = n_qg_max * hk * sb * sizeof(int32_t);
  w.bytes[WS_CNT_SUM] = hk * sb * sizeof(int32_t);
  w.bytes[WS_SIG_K] = hk * sb * c.lsh_tables * sizeof(uint16_t);
  w.bytes[WS_SIG_Q] = (size_t)c.n_q_heads * c.max_window * c.lsh_tables * sizeof(uint16_t);
  w.bytes[WS_QHIST] = use_qhist ? n_qg_max * hk * hist_bytes_head : 0;
  // the single sweep's per-table flags and its two launch counters (zero before the first launch)
  w.bytes[WS_SYNC] = use_qhist ? (hk * c.lsh_tables + 64) * sizeof(uint32_t) : 0;
}

void init_ctx_fields(laserkv_ctx* ctx, const laserkv_config& c) {
  ctx->cfg = c;
  ctx->only_kernel = -1;
  ctx->group = c.n_q_heads / c.n_kv_heads;
  ctx->elem_size = c.dtype == LKV_BF16 ? 2 : 4;
  ctx->sweep_wg_per_cu = 1;
}

void bind_workspace(laserkv_ctx* ctx, const WsPlan& w, void* const ptr[kWsBuffers]) {
  ctx->m_pad = w.m_pad;
  ctx->max_ranges = w.max_ranges;
  ctx->part = (float2*)ptr[WS_PART];
  ctx->s_part = (float*)ptr[WS_S_PART];
  ctx->s_exact = (float*)ptr[WS_S_EXACT];
  ctx->cnt = (int32_t*)ptr[WS_CNT];
  ctx->cnt_sum = (int32_t*)ptr[WS_CNT_SUM];
  ctx->sig_k = (uint16_t*)ptr[WS_SIG_K];
  ctx->sig_q = (uint16_t*)ptr[WS_SIG_Q];
  ctx->qhist = (uint32_t*)ptr[WS_QHIST];
  ctx->sync = (uint32_t*)ptr[WS_SYNC];
}

}  // namespace

extern "C" {

const char* laserkv_last_error(const laserkv_ctx* ctx) { return ctx ? ctx->error : g_error; }

int64_t laserkv_budget(int64_t s_block, int64_t l_ctx, int64_t r_num, int64_t r_den) {
  if (s_block <= 0 || l_ctx <= 0 || r_num < 0 || r_den <= 0) return -1;
  const __int128 num = (__int128)2 * r_num * s_block * l_ctx;
  const __int128 den = (__int128)r_den * (s_block + l_ctx);
  return (int64_t)(num / den);
}

int laserkv_partition(int32_t B, int32_t n, double alpha, int32_t s_t,
                      int32_t* n_anchor, int32_t* n_local, int32_t* k_exact, int32_t* k_lsh) {
  if (!n_anchor || !n_local || !k_exact || !k_lsh) return fail(nullptr, LKV_EINVAL, "partition: null output");
  if (n < 2) return fail(nullptr, LKV_EINVAL, "partition: protection divisor n must be >= 2 (got %d)", n);
  if (!(alpha >= 0.0 && alpha <= 1.0)) return fail(nullptr, LKV_EINVAL, "partition: alpha must lie in [0, 1]");
  if (B < 0 || s_t < 1) return fail(nullptr, LKV_EINVAL, "partition: need B >= 0 and s_t >= 1");
  const int32_t b_t = B < s_t ? B : s_t;
  const int32_t a = b_t / n;
  const int32_t b_long = b_t - 2 * a;
  const int32_t ke = (int32_t)std::floor(alpha * (double)b_long);
  *n_anchor = a;
  *n_local = a;
  *k_exact = ke;
  *k_lsh = b_long - ke;
  return LKV_OK;
}

int laserkv_create(const laserkv_config* cfg, laserkv_ctx** out) {
  if (!cfg || !out) return fail(nullptr, LKV_EINVAL, "create: null argument");
  const laserkv_config& c = *cfg;
  int rc = check_config(c, "create");
  if (rc != LKV_OK) return rc;

  laserkv_ctx* ctx = new (std::nothrow) laserkv_ctx();
  if (!ctx) return fail(nullptr, LKV_ENOMEM, "create: host allocation failed");
  memset(ctx, 0, sizeof(*ctx));
  init_ctx_fields(ctx, c);
  ctx->ev_pool = new (std::nothrow) std::vector<hipEvent_t>();
  ctx->ev_kind = new (std::nothrow) std::vector<int>();
  if (!ctx->ev_pool || !ctx->ev_kind) {
    laserkv_destroy(ctx);
    return fail(nullptr, LKV_ENOMEM, "create: host allocation failed");
  }
  hipError_t e = hipGetDevice(&ctx->device);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&ctx->n_cu, hipDeviceAttributeMultiprocessorCount, ctx->device);
  if (e != hipSuccess) {
    laserkv_destroy(ctx);
    return fail_hip(nullptr, e, "create: device query");
  }
  e = lkv::init_kernel_attributes();
  if (e == hipSuccess) e = lkv::init_attend_attributes();
  if (e == hipSuccess) e = lkv::init_single_attributes();
  if (e != hipSuccess) {
    laserkv_destroy(ctx);
    return fail_hip(nullptr, e, "create: kernel attribute");
  }
  ctx->sweep_wg_per_cu = env_int("LASERKV_SWEEP_WG_PER_CU", 1);
  if (ctx->sweep_wg_per_cu < 1) ctx->sweep_wg_per_cu = 1;
  ctx->append_split = env_int("LASERKV_APPEND_SPLIT", 0);
  ctx->single_spin = env_int("LASERKV_SINGLE_SPIN", 64);
  WsPlan ws;
  plan_workspace(c, env_int("LASERKV_NO_QHIST", 0) == 0, ws);
  void* ptr[kWsBuffers] = {};
  for (int i = 0; i < kWsBuffers; ++i) {
    if (!ws.bytes[i]) continue;
    e = hipMalloc(&ptr[i], ws.bytes[i]);
    if (e != hipSuccess) {
      for (int j = 0; j < i; ++j)
        if (ptr[j]) (void)hipFree(ptr[j]);
      laserkv_destroy(ctx);
      return fail(nullptr, LKV_ENOMEM, "create: hipMalloc of %zu bytes failed: %s", ws.bytes[i], hipGetErrorString(e));
    }
  }
  bind_workspace(ctx, ws, ptr);
  ctx->owns_workspace = true;
  // LASERKV_POISON_WORKSPACE=1 (tests): fill the fresh workspace with a non-zero pattern, so that a kernel
  // reading what no kernel wrote shows up in the results instead of meeting zeros by luck
  if (env_int("LASERKV_POISON_WORKSPACE", 0)) {
    for (int i = 0; i < kWsBuffers; ++i)
      if (e == hipSuccess && ptr[i]) e = hipMemset(ptr[i], 0xA5, ws.bytes[i]);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
      laserkv_destroy(ctx);
      return fail_hip(nullptr, e, "create: workspace fill");
    }
  }
  if (ptr[WS_SYNC]) {
    e = hipMemset(ptr[WS_SYNC], 0, ws.bytes[WS_SYNC]);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
      laserkv_destroy(ctx);
      return fail_hip(nullptr, e, "create: clearing the flags of the single sweep");
    }
  }
  *out = ctx;
  return LKV_OK;
}

void laserkv_destroy(laserkv_ctx* ctx) {
  if (!ctx) return;
  void* ptrs[] = {ctx->part, ctx->s_part, ctx->s_exact, ctx->cnt, ctx->cnt_sum, ctx->qhist, ctx->sig_k, ctx->sig_q, ctx->sync};
  if (ctx->owns_workspace)
    for (void* p : ptrs)
      if (p) (void)hipFree(p);
  if (ctx->ev_pool)
    for (hipEvent_t ev : *ctx->ev_pool) (void)hipEventDestroy(ev);
  delete ctx->ev_pool;
  delete ctx->ev_kind;
  delete ctx;
}

}  // extern "C"

namespace {

// Steps a1-a4, and a5 in the same last kernel when `fused` is given.
int select_impl(laserkv_ctx* ctx,
                const void* q_win, int64_t q_stride_head, int64_t q_stride_tok,
                const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                const void* k_ctx, int64_t c_stride_head, int64_t c_stride_tok,
                const void* hyperplanes,
                int32_t s_t, int32_t w, int32_t t_ctx,
                int64_t block_pos0, int64_t q_pos0, int32_t causal,
                int32_t n_anchor, int32_t n_local, int32_t k_exact, int32_t k_lsh,
                int32_t* keep_idx,
                float* dbg_s_exact, uint16_t* dbg_sig_k, uint16_t* dbg_sig_q, int32_t* dbg_count,
                const lkv::AppendParams* fused, void* hip_stream,
                float* acc_score = nullptr, int32_t* acc_count = nullptr, int accumulate = 0) {
  // acc_score != null: scoring only (steps a1-a3), summed over the heads into the accumulators
  if (!ctx) return fail(nullptr, LKV_EINVAL, "select_block: null context");
  const laserkv_config& c = ctx->cfg;
  const int es = ctx->elem_size, d = c.head_dim, G = ctx->group;
  if (!q_win || !k_blk || !hyperplanes || (!keep_idx && !acc_score)) return fail(ctx, LKV_EINVAL, "select_block: null tensor");
  if (s_t < 1 || s_t > c.max_block) return fail(ctx, LKV_EINVAL, "select_block: s_t=%d outside 1..max_block=%d", s_t, c.max_block);
  if (w < 1 || w > c.max_window) return fail(ctx, LKV_EINVAL, "select_block: w=%d outside 1..max_window=%d", w, c.max_window);
  if (t_ctx < 0 || t_ctx > c.max_ctx_keys) return fail(ctx, LKV_EINVAL, "select_block: t_ctx=%d outside 0..max_ctx_keys=%d", t_ctx, c.max_ctx_keys);
  if ((t_ctx > 0) != (k_ctx != nullptr)) return fail(ctx, LKV_EINVAL, "select_block: k_ctx must be given iff t_ctx > 0");
  if (n_anchor < 0 || n_local < 0 || k_exact < 0 || k_lsh < 0) return fail(ctx, LKV_EINVAL, "select_block: negative budget");
  if ((int64_t)n_anchor + n_local > s_t) return fail(ctx, LKV_EINVAL, "select_block: protected sets exceed the block");
  if ((int64_t)k_exact + k_lsh > (int64_t)s_t - n_anchor - n_local)
    return fail(ctx, LKV_EINVAL, "select_block: recall budget exceeds the candidate set");
  if (q_pos0 == LKV_WINDOW_AT_BLOCK_END) q_pos0 = block_pos0 + s_t - w;
  if (causal && q_pos0 < block_pos0) return fail(ctx, LKV_EINVAL, "select_block: causal window must not start before the block");
  const int64_t row_elems = d;
  auto bad_stride = [&](int64_t sh, int64_t st) { return st < row_elems || sh < 0 || ((st * es) & 15) || ((sh * es) & 15); };
  if (bad_stride(q_stride_head, q_stride_tok) || bad_stride(k_stride_head, k_stride_tok) ||
      (t_ctx > 0 && bad_stride(c_stride_head, c_stride_tok)))
    return fail(ctx, LKV_EINVAL, "select_block: strides must cover a row and keep rows 16-byte aligned");
  if ((int64_t)s_t * k_stride_tok * es >= (int64_t(1) << 31) || (int64_t)t_ctx * c_stride_tok * es >= (int64_t(1) << 31))
    return fail(ctx, LKV_EINVAL, "select_block: a head's keys must span less than 2 GiB");
  if (!aligned16(q_win) || !aligned16(k_blk) || !aligned16(hyperplanes) || (k_ctx && !aligned16(k_ctx)))
    return fail(ctx, LKV_EINVAL, "select_block: tensors must be 16-byte aligned");

  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const int m_rows = G * w;
  // With the rows' complete log-sum-exp from the caller the look-back keys have nothing left to contribute
  // (they only ever entered the normaliser): they are not read.
  const bool lse_complete = ctx->row_lse && ctx->row_lse_complete;
  if (lse_complete) {
    t_ctx = 0;
    k_ctx = nullptr;
  }
  const int n_keys = t_ctx + s_t;

  lkv::PassParams sp;
  sp.q = {(const char*)q_win, q_stride_head * es, q_stride_tok * es};
  sp.kb = {(const char*)k_blk, k_stride_head * es, k_stride_tok * es};
  sp.kc = {(const char*)k_ctx, c_stride_head * es, c_stride_tok * es};
  sp.planes = (const char*)hyperplanes;
  sp.q_linear = (q_stride_head >= (int64_t)w * q_stride_tok && (int64_t)G * q_stride_head * es < (int64_t(1) << 31)) ? 1 : 0;
  sp.group = G;
  sp.w = w;
  sp.m_rows = m_rows;
  sp.s_t = s_t;
  sp.t_ctx = t_ctx;
  sp.w_magic = (uint32_t)(((uint64_t(1) << 32) + (uint64_t)w - 1) / (uint64_t)w);
  const int n_qg = (m_rows + lkv::sweep_rows_per_group() - 1) / lkv::sweep_rows_per_group();
  sp.n_qgroups = n_qg;
  sp.n_kv_heads = c.n_kv_heads;
  // Key ranges, about one workgroup per compute unit and query-row group.  Sweep 1: ranges of nk keys, each
  // entirely look-back keys or entirely block keys.  Sweep 2 scores block keys only and has ranges of its
  // own: one round of workgroups if such ranges fit the LDS, else two, three, ... whole rounds.
  const int wg_target = ctx->n_cu * ctx->sweep_wg_per_cu;
  int nr0 = wg_target / (c.n_kv_heads * n_qg);
  if (nr0 < 1) nr0 = 1;
  int nk = ((n_keys + nr0 - 1) / nr0 + 31) / 32 * 32;
  if (nk > lkv::score_max_range()) nk = lkv::score_max_range();
  // the query-code job of a sweep-1 workgroup: ceil(L / n_ranges) tables, floor(32 / K) whole tables per
  // plane tile, and (when they fit 32 KiB of LDS) their histograms
  sp.q_tab_per_tile = 32 / c.lsh_bits;
  for (;;) {
    sp.keys_per_range = sp.blk_per_range = sp.ctx_per_range = nk;
    sp.n_ctx_ranges = (t_ctx + nk - 1) / nk;
    sp.n_ranges = sp.n_ctx_ranges + (s_t + nk - 1) / nk;
    sp.q_tab_per_wg = (c.lsh_tables + sp.n_ranges - 1) / sp.n_ranges;
    sp.q_tiles = (sp.q_tab_per_wg + sp.q_tab_per_tile - 1) / sp.q_tab_per_tile;
    const size_t hist_words = ((size_t)sp.q_tab_per_wg << c.lsh_bits) / 2;
    sp.hist_lds_words = (ctx->qhist && hist_words * 4 <= 32 * 1024) ? (int)(hist_words ? hist_words : 1) : 0;
    if (nk <= 32 || lkv::sweep_lds_bytes(c.dtype, d, false, nk, sp.q_tiles, sp.hist_lds_words) <= 150 * 1024) break;
    nk -= 32;
  }
  sp.n_parts = sp.n_ranges;
  {
    auto fits2 = [&](int blk) { return blk <= lkv::score_max_range() && lkv::sweep_lds_bytes(c.dtype, d, true, blk, 0, 0) <= 160 * 1024; };
    int blk = 32;
    bool ok = false;
    for (int rounds = 1; rounds <= 64 && !ok; ++rounds) {
      blk = ((s_t + nr0 * rounds - 1) / (nr0 * rounds) + 31) / 32 * 32;
      ok = fits2(blk);
      if (blk == 32) break;
    }
    while (!ok && blk > 32) ok = fits2(blk -= 32);
    sp.s2_blk_per_range = blk;
    sp.s2_ranges = (s_t + blk - 1) / blk;
  }
  if (lkv::sweep_lds_bytes(c.dtype, d, false, nk, sp.q_tiles, sp.hist_lds_words) > 160 * 1024)
    return fail(ctx, LKV_EINVAL, "select_block: s_t + t_ctx = %d keys are too few to spread %d tables of %d bits over "
                "(the query-code job of one key range exceeds the LDS)", n_keys, c.lsh_tables, c.lsh_bits);
  if (sp.n_ranges > ctx->max_ranges) return fail(ctx, LKV_EINVAL, "select_block: internal range split too fine");
  sp.causal = causal ? 1 : 0;
  int64_t lim0 = (int64_t)t_ctx + (q_pos0 - block_pos0);
  if (lim0 > (1 << 30)) lim0 = 1 << 30;
  sp.lim0 = (int)lim0;
  sp.scale2 = (float)(1.4426950408889634 / std::sqrt((double)d));
  sp.part = ctx->part;
  sp.m_pad = ctx->m_pad;
  sp.r_pad = (sp.n_ranges + 7) & ~7;
  sp.s_part = ctx->s_part;
  sp.row_lse = ctx->row_lse;
  sp.lse_complete = lse_complete ? 1 : 0;
  sp.n_tables = c.lsh_tables;
  sp.n_bits = c.lsh_bits;
  sp.n_planes = c.lsh_tables * c.lsh_bits;
  sp.tables_per_split = (c.lsh_tables + n_qg - 1) / n_qg;
  sp.sig_k = ctx->sig_k;
  sp.sig_q = ctx->sig_q;
  sp.cnt = ctx->cnt;
  sp.qhist = sp.hist_lds_words ? ctx->qhist : nullptr;

  lkv::CountParams cp;
  cp.sig_k = ctx->sig_k;
  cp.sig_q = ctx->sig_q;
  cp.cnt = ctx->cnt;
  cp.group = G;
  cp.w = w;
  cp.s_t = s_t;
  cp.n_tables = c.lsh_tables;
  cp.n_bits = c.lsh_bits;
  {
    // tables per group: keep the histogram within 64 KiB of LDS (one table at K = 16 takes 128 KiB)
    int tg = (64 * 1024) / ((1 << c.lsh_bits) * 2);
    if (tg < 1) tg = 1;
    if (tg > c.lsh_tables) tg = c.lsh_tables;
    cp.tables_per_group = tg;
    const int n_tg = (c.lsh_tables + tg - 1) / tg;
    // Several table groups per workgroup (taken one after the other) save global atomics; as many as
    // still leave about one workgroup per compute unit with key ranges of at least 1024 keys.
    int gpw = 1;
    while (gpw * 2 <= n_tg && (int64_t)c.n_kv_heads * ((n_tg + 2 * gpw - 1) / (2 * gpw)) * ((s_t + 1023) / 1024) >= wg_target) gpw *= 2;
    cp.groups_per_wg = gpw;
    const int n_wg_t = (n_tg + gpw - 1) / gpw;
    int n_kr = wg_target / (c.n_kv_heads * n_wg_t);
    if (n_kr < 1) n_kr = 1;
    int kpr = ((s_t + n_kr - 1) / n_kr + 1023) / 1024 * 1024;
    if (kpr > lkv::count_max_keys_per_range()) kpr = lkv::count_max_keys_per_range();
    // the workgroup stages its tables' codes of all window queries and of its keys in LDS beside the histogram:
    // fewer table groups per workgroup, then shorter key ranges, until that fits
    while (lkv::count_lds_bytes(c.lsh_bits, tg, gpw, m_rows, kpr) > 156 * 1024 && gpw > 1) gpw /= 2;
    while (lkv::count_lds_bytes(c.lsh_bits, tg, gpw, m_rows, kpr) > 156 * 1024 && kpr > 64) kpr /= 2;
    cp.groups_per_wg = gpw;
    cp.keys_per_range = kpr;
  }

  lkv::SelectParams lp;
  lp.s_part = ctx->s_part;
  lp.n_qgroups = n_qg;
  lp.n_kv_heads = c.n_kv_heads;
  lp.inv_m = 1.0f / (float)m_rows;
  lp.cnt = ctx->cnt;
  // sweep 2 writes a count part only for the query-row groups that own tables (the first ones); the
  // stand-alone count kernel sums into part 0
  lp.n_cnt_parts = sp.qhist ? (c.lsh_tables + sp.tables_per_split - 1) / sp.tables_per_split : 1;
  lp.cnt_out = dbg_count ? ctx->cnt_sum : nullptr;      // stage outputs are written only on request
  lp.s_t = s_t;
  lp.n_anchor = n_anchor;
  lp.n_local = n_local;
  lp.k_exact = k_exact;
  lp.k_lsh = k_lsh;
  lp.cnt_bits = bits_for((int64_t)m_rows * c.lsh_tables);
  lp.s_exact = dbg_s_exact ? ctx->s_exact : nullptr;
  lp.keep = keep_idx;

  // With complete row statistics from the caller nothing depends on a first pass over all keys: one sweep
  // hashes, scores and counts (keys read once), where the shape allows it (the GQA group's window rows in one
  // workgroup, histograms of the window-row codes resident in global memory, rows of at most 256 bytes).
  lkv::SingleParams sg = {};
  bool single = lse_complete && ctx->qhist && ctx->sync && ctx->single_spin >= 0 && sp.q_linear &&
                lkv::single_supports(c.dtype, d) && m_rows <= lkv::single_max_rows();
  if (single) {
    int snk = (int)(((int64_t)s_t * c.n_kv_heads + ctx->n_cu - 1) / ctx->n_cu + 31) / 32 * 32;
    snk = std::max(32, std::min(snk, lkv::single_max_keys()));
    for (;; snk -= 32) {
      sg.keys_per_range = snk;
      sg.n_ranges = (s_t + snk - 1) / snk;
      sg.q_tab_per_wg = (c.lsh_tables + sg.n_ranges - 1) / sg.n_ranges;
      sg.q_tiles = (sg.q_tab_per_wg + sp.q_tab_per_tile - 1) / sp.q_tab_per_tile;
      const bool fits = sg.q_tiles <= lkv::single_max_qtiles() &&
                        lkv::single_lds_bytes(c.dtype, d, snk, sg.q_tiles, sg.q_tab_per_wg, c.lsh_bits, c.lsh_tables) <= 160 * 1024;
      if (fits || snk <= 32) {
        single = fits;
        break;
      }
    }
  }
  if (single) {
    sg.q = sp.q;
    sg.kb = sp.kb;
    sg.planes = sp.planes;
    sg.group = G;
    sg.w = w;
    sg.w_magic = sp.w_magic;
    sg.m_rows = m_rows;
    sg.s_t = s_t;
    sg.n_kv_heads = c.n_kv_heads;
    sg.causal = sp.causal;
    sg.lim0 = sp.lim0;
    sg.scale2 = sp.scale2;
    sg.row_lse = ctx->row_lse;
    sg.n_tables = c.lsh_tables;
    sg.n_bits = c.lsh_bits;
    sg.n_planes = sp.n_planes;
    sg.q_tab_per_tile = sp.q_tab_per_tile;
    sg.s_part = ctx->s_part;
    sg.cnt = ctx->cnt;
    sg.sig_k = dbg_sig_k ? ctx->sig_k : nullptr;
    sg.sig_q = ctx->sig_q;
    sg.qhist = ctx->qhist;
    sg.sync = ctx->sync;
    sg.flags = ctx->sync + 64;
    sg.spin_limit = ctx->single_spin;
    lp.n_qgroups = 1;
    lp.n_cnt_parts = 1;
  }

  hipError_t e;
  const int nh = c.n_kv_heads, dt = c.dtype;
  if (single) {
    if ((e = timed(ctx, LKV_KERN_SINGLE, st, [&] { return lkv::launch_single(dt, d, sg, st); })) != hipSuccess)
      return fail_hip(ctx, e, "select_block: single sweep (SimHash codes + pooled probabilities + collision counts)");
  } else {
    if ((e = timed(ctx, LKV_KERN_SWEEP1, st, [&] { return lkv::launch_sweep1(dt, d, sp, st); })) != hipSuccess)
      return fail_hip(ctx, e, "select_block: sweep 1 (row statistics + SimHash codes)");
    if ((e = timed(ctx, LKV_KERN_SWEEP2, st, [&] { return lkv::launch_sweep2(dt, d, sp, st); })) != hipSuccess)
      return fail_hip(ctx, e, "select_block: sweep 2 (pooled probabilities)");
    if (!sp.qhist && (e = timed(ctx, LKV_KERN_COUNT, st, [&] { return lkv::launch_count(cp, nh, st); })) != hipSuccess)
      return fail_hip(ctx, e, "select_block: count kernel");
  }
  if (acc_score) {
    lkv::AccumParams acp;
    acp.s_part = ctx->s_part;
    acp.cnt = ctx->cnt;
    acp.n_qgroups = lp.n_qgroups;
    acp.n_cnt_parts = lp.n_cnt_parts;
    acp.n_kv_heads = c.n_kv_heads;
    acp.s_t = s_t;
    acp.inv_m = lp.inv_m;
    acp.score = acc_score;
    acp.count = acc_count;
    acp.accumulate = accumulate;
    if ((e = timed(ctx, LKV_KERN_SELECT, st, [&] { return lkv::launch_accumulate(acp, st); })) != hipSuccess)
      return fail_hip(ctx, e, "score_block: accumulation kernel");
  } else if (fused) {
    lkv::AppendParams ap = *fused;
    ap.keep = keep_idx;
    const int n_cu = ctx->n_cu, split = ctx->append_split;
    if ((e = timed(ctx, LKV_KERN_SELECT, st, [&] { return lkv::launch_select_append(lp, ap, n_cu, split, st); })) != hipSuccess)
      return fail_hip(ctx, e, "compress_block: select + append kernel");
  } else if ((e = timed(ctx, LKV_KERN_SELECT, st, [&] { return lkv::launch_select(lp, st); })) != hipSuccess) {
    return fail_hip(ctx, e, "select_block: select kernel");
  }

  const size_t hk = c.n_kv_heads;
  if (dbg_s_exact && (e = hipMemcpyAsync(dbg_s_exact, ctx->s_exact, hk * s_t * sizeof(float), hipMemcpyDeviceToDevice, st)) != hipSuccess)
    return fail_hip(ctx, e, "select_block: copy of S_exact");
  if (dbg_sig_k && (e = hipMemcpyAsync(dbg_sig_k, ctx->sig_k, hk * s_t * c.lsh_tables * sizeof(uint16_t), hipMemcpyDeviceToDevice, st)) != hipSuccess)
    return fail_hip(ctx, e, "select_block: copy of key signatures");
  if (dbg_sig_q && (e = hipMemcpyAsync(dbg_sig_q, ctx->sig_q, (size_t)c.n_q_heads * w * c.lsh_tables * sizeof(uint16_t), hipMemcpyDeviceToDevice, st)) != hipSuccess)
    return fail_hip(ctx, e, "select_block: copy of query signatures");
  if (dbg_count && (e = hipMemcpyAsync(dbg_count, ctx->cnt_sum, hk * s_t * sizeof(int32_t), hipMemcpyDeviceToDevice, st)) != hipSuccess)
    return fail_hip(ctx, e, "select_block: copy of counts");
  return LKV_OK;
}

// Checks the append arguments and fills the kernel parameter block (keep is set by the caller).
int append_params(laserkv_ctx* ctx,
                  const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                  const void* v_blk, int64_t v_stride_head, int64_t v_stride_tok,
                  int32_t b_t, int32_t s_t, int64_t block_pos0,
                  void* k_cache, void* v_cache, int64_t cache_stride_head,
                  int64_t* cache_pos, int64_t pos_stride_head,
                  int64_t cache_len, int64_t cache_cap, lkv::AppendParams& ap) {
  const laserkv_config& c = ctx->cfg;
  const int es = ctx->elem_size, d = c.head_dim;
  if (!k_blk || !v_blk || !k_cache || !v_cache || !cache_pos) return fail(ctx, LKV_EINVAL, "append: null tensor");
  if (s_t < 1 || b_t < 0 || b_t > s_t) return fail(ctx, LKV_EINVAL, "append: need 0 <= b_t <= s_t");
  if (cache_len < 0 || cache_cap < 0) return fail(ctx, LKV_EINVAL, "append: negative cache length or capacity");
  if (cache_len + b_t > cache_cap) return fail(ctx, LKV_ECAP, "append: %lld + %d rows exceed the capacity %lld", (long long)cache_len, b_t, (long long)cache_cap);
  auto bad_stride = [&](int64_t sh, int64_t st) { return st < d || sh < 0 || ((st * es) & 15) || ((sh * es) & 15); };
  if (bad_stride(k_stride_head, k_stride_tok) || bad_stride(v_stride_head, v_stride_tok))
    return fail(ctx, LKV_EINVAL, "append: strides must cover a row and keep rows 16-byte aligned");
  if (cache_stride_head < cache_cap * d || ((cache_stride_head * es) & 15)) return fail(ctx, LKV_EINVAL, "append: cache head stride too small or misaligned");
  if (pos_stride_head < cache_cap) return fail(ctx, LKV_EINVAL, "append: position head stride below the capacity");
  if (!aligned16(k_blk) || !aligned16(v_blk) || !aligned16(k_cache) || !aligned16(v_cache))
    return fail(ctx, LKV_EINVAL, "append: tensors must be 16-byte aligned");
  ap.kb = {(const char*)k_blk, k_stride_head * es, k_stride_tok * es};
  ap.vb = {(const char*)v_blk, v_stride_head * es, v_stride_tok * es};
  ap.keep = nullptr;
  ap.keep_stride_head = b_t;
  ap.b_t = b_t;
  ap.s_t = s_t;
  ap.row_bytes = d * es;
  ap.k_cache = (char*)k_cache;
  ap.v_cache = (char*)v_cache;
  ap.cache_stride_head = cache_stride_head * es;
  ap.cache_pos = cache_pos;
  ap.pos_stride_head = pos_stride_head;
  ap.cache_len = cache_len;
  ap.block_pos0 = block_pos0;
  return LKV_OK;
}

}  // namespace

extern "C" {

int laserkv_select_block(laserkv_ctx* ctx,
                         const void* q_win, int64_t q_stride_head, int64_t q_stride_tok,
                         const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                         const void* k_ctx, int64_t c_stride_head, int64_t c_stride_tok,
                         const void* hyperplanes,
                         int32_t s_t, int32_t w, int32_t t_ctx,
                         int64_t block_pos0, int64_t q_pos0, int32_t causal,
                         int32_t n_anchor, int32_t n_local, int32_t k_exact, int32_t k_lsh,
                         int32_t* keep_idx,
                         float* dbg_s_exact, uint16_t* dbg_sig_k, uint16_t* dbg_sig_q, int32_t* dbg_count,
                         void* hip_stream) {
  return select_impl(ctx, q_win, q_stride_head, q_stride_tok, k_blk, k_stride_head, k_stride_tok,
                     k_ctx, c_stride_head, c_stride_tok, hyperplanes, s_t, w, t_ctx, block_pos0, q_pos0, causal,
                     n_anchor, n_local, k_exact, k_lsh, keep_idx, dbg_s_exact, dbg_sig_k, dbg_sig_q, dbg_count,
                     nullptr, hip_stream);
}

int laserkv_append(laserkv_ctx* ctx,
                   const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                   const void* v_blk, int64_t v_stride_head, int64_t v_stride_tok,
                   const int32_t* keep_idx, int32_t b_t, int32_t s_t, int64_t block_pos0,
                   void* k_cache, void* v_cache, int64_t cache_stride_head,
                   int64_t* cache_pos, int64_t pos_stride_head,
                   int64_t cache_len, int64_t cache_cap,
                   void* hip_stream) {
  if (!ctx) return fail(nullptr, LKV_EINVAL, "append: null context");
  if (!keep_idx) return fail(ctx, LKV_EINVAL, "append: null tensor");
  lkv::AppendParams ap;
  const int rc = append_params(ctx, k_blk, k_stride_head, k_stride_tok, v_blk, v_stride_head, v_stride_tok, b_t, s_t,
                               block_pos0, k_cache, v_cache, cache_stride_head, cache_pos, pos_stride_head, cache_len,
                               cache_cap, ap);
  if (rc != LKV_OK) return rc;
  ap.keep = keep_idx;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const int nh = ctx->cfg.n_kv_heads;
  hipError_t e = timed(ctx, LKV_KERN_APPEND, st, [&] { return lkv::launch_append(ap, nh, st); });
  if (e != hipSuccess) return fail_hip(ctx, e, "append: gather kernel");
  return LKV_OK;
}

int laserkv_compress_block(laserkv_ctx* ctx,
                           const void* q_win, int64_t q_stride_head, int64_t q_stride_tok,
                           const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                           const void* v_blk, int64_t v_stride_head, int64_t v_stride_tok,
                           const void* k_ctx, int64_t c_stride_head, int64_t c_stride_tok,
                           const void* hyperplanes,
                           int32_t s_t, int32_t w, int32_t t_ctx,
                           int64_t block_pos0, int64_t q_pos0, int32_t causal,
                           int32_t n_anchor, int32_t n_local, int32_t k_exact, int32_t k_lsh,
                           int32_t* keep_idx,
                           void* k_cache, void* v_cache, int64_t cache_stride_head,
                           int64_t* cache_pos, int64_t pos_stride_head,
                           int64_t cache_len, int64_t cache_cap,
                           void* hip_stream) {
  if (!ctx) return fail(nullptr, LKV_EINVAL, "compress_block: null context");
  const int64_t b_t = (int64_t)n_anchor + n_local + k_exact + k_lsh;
  if (n_anchor < 0 || n_local < 0 || k_exact < 0 || k_lsh < 0 || b_t > s_t) return fail(ctx, LKV_EINVAL, "compress_block: budget does not fit the block");
  lkv::AppendParams ap;
  const int rc = append_params(ctx, k_blk, k_stride_head, k_stride_tok, v_blk, v_stride_head, v_stride_tok, (int32_t)b_t, s_t,
                               block_pos0, k_cache, v_cache, cache_stride_head, cache_pos, pos_stride_head, cache_len,
                               cache_cap, ap);
  if (rc != LKV_OK) return rc;
  return select_impl(ctx, q_win, q_stride_head, q_stride_tok, k_blk, k_stride_head, k_stride_tok,
                     k_ctx, c_stride_head, c_stride_tok, hyperplanes, s_t, w, t_ctx, block_pos0, q_pos0, causal,
                     n_anchor, n_local, k_exact, k_lsh, keep_idx, nullptr, nullptr, nullptr, nullptr, &ap, hip_stream);
}

int laserkv_set_row_lse(laserkv_ctx* ctx, const float* row_lse) {
  if (!ctx) return fail(nullptr, LKV_EINVAL, "set_row_lse: null context");
  if (row_lse && (reinterpret_cast<uintptr_t>(row_lse) & 3)) return fail(ctx, LKV_EINVAL, "set_row_lse: misaligned pointer");
  ctx->row_lse = row_lse;
  ctx->row_lse_complete = false;
  return LKV_OK;
}

int laserkv_set_row_lse_complete(laserkv_ctx* ctx, const float* row_lse) {
  if (!ctx) return fail(nullptr, LKV_EINVAL, "set_row_lse_complete: null context");
  if (row_lse && (reinterpret_cast<uintptr_t>(row_lse) & 3)) return fail(ctx, LKV_EINVAL, "set_row_lse_complete: misaligned pointer");
  ctx->row_lse = row_lse;
  ctx->row_lse_complete = row_lse != nullptr;
  return LKV_OK;
}

// Shared by laserkv_attend_cache (no block keys) and laserkv_attend_block.
static bool attend_sizes_ok(const laserkv_ctx* ctx, int64_t n_q, int64_t n_q_max, int64_t cache_len, int64_t s_t) {
  return ctx && n_q >= 1 && n_q <= n_q_max && cache_len >= 0 && s_t >= 0 && s_t <= ctx->cfg.max_block &&
         cache_len * ctx->cfg.head_dim * ctx->elem_size < (int64_t(1) << 31);
}

static int64_t attend_workspace_need(const laserkv_ctx* ctx, int n_q, int64_t cache_len, int s_t, bool with_lse_only) {
  const int m_rows = ctx->group * n_q;
  lkv::AttendPlan plan;
  lkv::attend_plan(m_rows, cache_len, s_t, ctx->cfg.n_kv_heads, ctx->n_cu, &plan);
  size_t need = lkv::attend_workspace_bytes(plan, m_rows, ctx->cfg.n_kv_heads, ctx->cfg.head_dim);
  if (with_lse_only) {
    lkv::AttendPlan lplan;
    lkv::attend_lse_plan(m_rows, cache_len, ctx->cfg.n_kv_heads, ctx->n_cu, &lplan);
    need = std::max(need, (size_t)ctx->cfg.n_kv_heads * lplan.n_parts * m_rows * 8 + 256);
  }
  return (int64_t)need;
}

int64_t laserkv_attend_workspace_bytes(const laserkv_ctx* ctx, int32_t n_q, int64_t cache_len) {
  if (!ctx || !attend_sizes_ok(ctx, n_q, ctx->cfg.max_window, cache_len, 0)) return -1;
  return attend_workspace_need(ctx, n_q, cache_len, 0, true);  // enough for the call with or without `out`
}

int64_t laserkv_attend_block_workspace_bytes(const laserkv_ctx* ctx, int32_t n_q, int64_t cache_len, int32_t s_t) {
  if (!ctx || !attend_sizes_ok(ctx, n_q, ctx->cfg.max_block, cache_len, s_t)) return -1;
  return attend_workspace_need(ctx, n_q, cache_len, s_t, false);
}

static int attend_impl(laserkv_ctx* ctx, const char* fn, int64_t n_q_max,
                       const void* q, int64_t q_stride_head, int64_t q_stride_tok, int32_t n_q,
                       const void* k_cache, const void* v_cache, int64_t cache_stride_head, int64_t cache_len,
                       const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                       const void* v_blk, int64_t v_stride_head, int64_t v_stride_tok,
                       int32_t s_t, int64_t diag64,
                       float* out, float* out_lse, bool lse_only,
                       void* workspace, int64_t workspace_bytes, void* hip_stream) {
  const laserkv_config& c = ctx->cfg;
  const int es = ctx->elem_size, d = c.head_dim;
  if (!q || !out_lse || !workspace) return fail(ctx, LKV_EINVAL, "%s: null tensor", fn);
  if (!attend_sizes_ok(ctx, n_q, n_q_max, cache_len, s_t))
    return fail(ctx, LKV_EINVAL, "%s: n_q must be 1..%lld, s_t 0..max_block (%d), cache_len >= 0 with cache_len * d * elem size < 2^31",
                fn, (long long)n_q_max, c.max_block);
  if (cache_len > 0 && (!k_cache || (!v_cache && !lse_only))) return fail(ctx, LKV_EINVAL, "%s: null cache", fn);
  if (q_stride_tok < d || q_stride_head < 0 || ((q_stride_tok * es) & 15) || ((q_stride_head * es) & 15))
    return fail(ctx, LKV_EINVAL, "%s: query strides must cover a row and keep rows 16-byte aligned", fn);
  if (cache_stride_head < cache_len * d || ((cache_stride_head * es) & 15))
    return fail(ctx, LKV_EINVAL, "%s: cache head stride too small or misaligned", fn);
  if (s_t > 0) {
    if (!k_blk || !v_blk) return fail(ctx, LKV_EINVAL, "%s: null block tensor", fn);
    if (k_stride_tok < d || v_stride_tok < d || k_stride_head < 0 || v_stride_head < 0 || ((k_stride_tok * es) & 15) ||
        ((v_stride_tok * es) & 15) || ((k_stride_head * es) & 15) || ((v_stride_head * es) & 15))
      return fail(ctx, LKV_EINVAL, "%s: block strides must cover a row and keep rows 16-byte aligned", fn);
    // the kernels address rows up to a chunk past the block with 32-bit byte offsets
    if (((int64_t)s_t + 256) * std::max(k_stride_tok, v_stride_tok) * es >= (int64_t(1) << 31))
      return fail(ctx, LKV_EINVAL, "%s: (s_t + 256) * token stride * elem size must stay below 2^31", fn);
    if (!aligned16(k_blk) || !aligned16(v_blk)) return fail(ctx, LKV_EINVAL, "%s: block tensors must be 16-byte aligned", fn);
  }
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) ||
      (reinterpret_cast<uintptr_t>(out_lse) & 3u) || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return fail(ctx, LKV_EINVAL, "%s: tensors must be 16-byte aligned (out_lse 4, workspace 256)", fn);
  const int m_rows = ctx->group * n_q;
  lkv::AttendPlan plan;
  if (lse_only) lkv::attend_lse_plan(m_rows, cache_len, c.n_kv_heads, ctx->n_cu, &plan);
  else lkv::attend_plan(m_rows, cache_len, s_t, c.n_kv_heads, ctx->n_cu, &plan);
  const size_t need = lse_only ? (size_t)c.n_kv_heads * plan.n_parts * m_rows * 8 + 256
                               : lkv::attend_workspace_bytes(plan, m_rows, c.n_kv_heads, d);
  if (workspace_bytes < (int64_t)need)
    return fail(ctx, LKV_EINVAL, "%s: workspace of %lld bytes, %zu needed", fn, (long long)workspace_bytes, need);
  lkv::AttendParams p = {};
  p.q = {(const char*)q, q_stride_head * es, q_stride_tok * es};
  p.group = ctx->group;
  p.n_q = n_q;
  p.nq_magic = n_q > 1 ? (uint32_t)(((uint64_t(1) << 32) + n_q - 1) / n_q) : 0u;
  p.m_rows = m_rows;
  p.k_cache = (const char*)k_cache;
  p.v_cache = (const char*)v_cache;
  p.cache_stride_head = cache_stride_head * es;
  p.row_bytes = d * es;
  p.cache_len = (int)cache_len;
  p.k_blk = (const char*)k_blk;
  p.v_blk = (const char*)v_blk;
  p.kb_stride_head = k_stride_head * es;
  p.vb_stride_head = v_stride_head * es;
  p.kb_stride_row = (int)(k_stride_tok * es);
  p.vb_stride_row = (int)(v_stride_tok * es);
  p.s_t = s_t;
  p.diag = (int)std::max<int64_t>(-(int64_t(1) << 30), std::min<int64_t>(diag64, int64_t(1) << 30));
  p.keys_per_split = plan.keys_per_split;
  p.blk_keys_per_split = plan.blk_keys_per_split;
  p.n_splits = plan.n_splits;
  p.direct = plan.direct;
  p.wprt_log = plan.wprt_log;
  p.n_parts = plan.n_parts;
  p.n_qgroups = plan.n_qgroups;
  p.n_kv_heads = c.n_kv_heads;
  p.scale2 = (float)(1.4426950408889634 / sqrt((double)d));
  const size_t rows = (size_t)c.n_kv_heads * plan.n_parts * m_rows;
  p.part_o = lse_only ? nullptr : reinterpret_cast<float*>(workspace);
  p.part_ml = lse_only ? reinterpret_cast<float2*>(workspace)
                       : reinterpret_cast<float2*>(reinterpret_cast<char*>(workspace) + ((rows * d * 4 + 255) & ~(size_t)255));
  p.out = out;
  p.out_lse = out_lse;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  hipError_t e = timed(ctx, LKV_KERN_ATTEND, st, [&] {
    return lse_only ? lkv::launch_attend_lse((int)c.dtype, d, p, st) : lkv::launch_attend((int)c.dtype, d, p, st);
  });
  if (e != hipSuccess) return fail(ctx, LKV_EHIP, "%s: kernels: %s", fn, hipGetErrorString(e));
  return LKV_OK;
}

int laserkv_attend_cache(laserkv_ctx* ctx,
                         const void* q, int64_t q_stride_head, int64_t q_stride_tok, int32_t n_q,
                         const void* k_cache, const void* v_cache, int64_t cache_stride_head, int64_t cache_len,
                         float* out, float* out_lse,
                         void* workspace, int64_t workspace_bytes,
                         void* hip_stream) {
  if (!ctx) return fail(nullptr, LKV_EINVAL, "attend_cache: null context");
  return attend_impl(ctx, "attend_cache", ctx->cfg.max_window, q, q_stride_head, q_stride_tok, n_q, k_cache, v_cache,
                     cache_stride_head, cache_len, nullptr, 0, 0, nullptr, 0, 0, 0, 0, out, out_lse, out == nullptr,
                     workspace, workspace_bytes, hip_stream);
}

int laserkv_attend_block(laserkv_ctx* ctx,
                         const void* q, int64_t q_stride_head, int64_t q_stride_tok, int32_t n_q,
                         const void* k_cache, const void* v_cache, int64_t cache_stride_head, int64_t cache_len,
                         const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                         const void* v_blk, int64_t v_stride_head, int64_t v_stride_tok,
                         int32_t s_t, int64_t block_pos0, int64_t q_pos0, int32_t causal,
                         float* out, float* out_lse,
                         void* workspace, int64_t workspace_bytes,
                         void* hip_stream) {
  if (!ctx) return fail(nullptr, LKV_EINVAL, "attend_block: null context");
  if (!out) return fail(ctx, LKV_EINVAL, "attend_block: null output");
  // key i (position block_pos0 + i) is visible to query j (position q_pos0 + j) iff i <= q_pos0 - block_pos0 + j
  const int64_t diag = causal ? q_pos0 - block_pos0 : (int64_t(1) << 30);
  return attend_impl(ctx, "attend_block", ctx->cfg.max_block, q, q_stride_head, q_stride_tok, n_q, k_cache, v_cache,
                     cache_stride_head, cache_len, k_blk, k_stride_head, k_stride_tok, v_blk, v_stride_head, v_stride_tok,
                     s_t, diag, out, out_lse, false, workspace, workspace_bytes, hip_stream);
}

int laserkv_score_block(laserkv_ctx* ctx,
                        const void* q_win, int64_t q_stride_head, int64_t q_stride_tok,
                        const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                        const void* k_ctx, int64_t c_stride_head, int64_t c_stride_tok,
                        const void* hyperplanes,
                        int32_t s_t, int32_t w, int32_t t_ctx,
                        int64_t block_pos0, int64_t q_pos0, int32_t causal,
                        float* score_acc, int32_t* count_acc, int32_t accumulate,
                        void* hip_stream) {
  if (!ctx) return fail(nullptr, LKV_EINVAL, "score_block: null context");
  if (!score_acc || !count_acc) return fail(ctx, LKV_EINVAL, "score_block: null accumulator");
  return select_impl(ctx, q_win, q_stride_head, q_stride_tok, k_blk, k_stride_head, k_stride_tok,
                     k_ctx, c_stride_head, c_stride_tok, hyperplanes, s_t, w, t_ctx, block_pos0, q_pos0, causal,
                     0, 0, 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, hip_stream,
                     score_acc, count_acc, accumulate ? 1 : 0);
}

int laserkv_select_consensus(laserkv_ctx* ctx, const float* score_acc, const int32_t* count_acc, int32_t s_t,
                             int32_t n_anchor, int32_t n_local, int32_t k_exact, int32_t k_lsh,
                             int32_t* keep_idx, void* hip_stream) {
  if (!ctx) return fail(nullptr, LKV_EINVAL, "select_consensus: null context");
  if (!score_acc || !count_acc || !keep_idx) return fail(ctx, LKV_EINVAL, "select_consensus: null tensor");
  if (s_t < 1 || s_t > ctx->cfg.max_block) return fail(ctx, LKV_EINVAL, "select_consensus: s_t=%d outside 1..max_block=%d", s_t, ctx->cfg.max_block);
  if (n_anchor < 0 || n_local < 0 || k_exact < 0 || k_lsh < 0) return fail(ctx, LKV_EINVAL, "select_consensus: negative budget");
  if ((int64_t)n_anchor + n_local > s_t) return fail(ctx, LKV_EINVAL, "select_consensus: protected sets exceed the block");
  if ((int64_t)k_exact + k_lsh > (int64_t)s_t - n_anchor - n_local)
    return fail(ctx, LKV_EINVAL, "select_consensus: recall budget exceeds the candidate set");
  if (!aligned16(score_acc) || !aligned16(count_acc)) return fail(ctx, LKV_EINVAL, "select_consensus: accumulators must be 16-byte aligned");
  lkv::SelectParams lp;
  lp.s_part = score_acc;
  lp.n_qgroups = 1;
  lp.n_kv_heads = 1;
  lp.inv_m = 1.0f;
  lp.cnt = count_acc;
  lp.n_cnt_parts = 1;
  lp.cnt_out = nullptr;
  lp.s_t = s_t;
  lp.n_anchor = n_anchor;
  lp.n_local = n_local;
  lp.k_exact = k_exact;
  lp.k_lsh = k_lsh;
  lp.cnt_bits = 31;  // the kernel reads the largest count and uses only the digits it needs
  lp.s_exact = nullptr;
  lp.keep = keep_idx;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  hipError_t e = timed(ctx, LKV_KERN_SELECT, st, [&] { return lkv::launch_select(lp, st); });
  if (e != hipSuccess) return fail_hip(ctx, e, "select_consensus: select kernel");
  return LKV_OK;
}

int laserkv_append_shared(laserkv_ctx* ctx,
                          const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                          const void* v_blk, int64_t v_stride_head, int64_t v_stride_tok,
                          const int32_t* keep_idx, int32_t b_t, int32_t s_t, int64_t block_pos0,
                          void* k_cache, void* v_cache, int64_t cache_stride_head,
                          int64_t* cache_pos, int64_t pos_stride_head,
                          int64_t cache_len, int64_t cache_cap,
                          void* hip_stream) {
  if (!ctx) return fail(nullptr, LKV_EINVAL, "append_shared: null context");
  if (!keep_idx) return fail(ctx, LKV_EINVAL, "append_shared: null tensor");
  lkv::AppendParams ap;
  const int rc = append_params(ctx, k_blk, k_stride_head, k_stride_tok, v_blk, v_stride_head, v_stride_tok, b_t, s_t,
                               block_pos0, k_cache, v_cache, cache_stride_head, cache_pos, pos_stride_head, cache_len,
                               cache_cap, ap);
  if (rc != LKV_OK) return rc;
  ap.keep = keep_idx;
  ap.keep_stride_head = 0;  // one index list for every head
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const int nh = ctx->cfg.n_kv_heads;
  hipError_t e = timed(ctx, LKV_KERN_APPEND, st, [&] { return lkv::launch_append(ap, nh, st); });
  if (e != hipSuccess) return fail_hip(ctx, e, "append_shared: gather kernel");
  return LKV_OK;
}

int laserkv_profile_isolate(laserkv_ctx* ctx, int32_t kernel_id) {
  if (!ctx) return fail(nullptr, LKV_EINVAL, "profile_isolate: null context");
  if (kernel_id >= LKV_N_KERNELS) return fail(ctx, LKV_EINVAL, "profile_isolate: no kernel kind %d", kernel_id);
  ctx->only_kernel = kernel_id < 0 ? -1 : kernel_id;
  return LKV_OK;
}

int laserkv_profile_begin(laserkv_ctx* ctx) {
  if (!ctx) return fail(nullptr, LKV_EINVAL, "profile_begin: null context");
  ctx->ev_kind->clear();
  ctx->profiling = true;
  return LKV_OK;
}

int laserkv_profile_end(laserkv_ctx* ctx, double* ms_per_kernel, int64_t* launches) {
  if (!ctx || !ms_per_kernel || !launches) return fail(ctx, LKV_EINVAL, "profile_end: null argument");
  if (!ctx->profiling) return fail(ctx, LKV_EINVAL, "profile_end: profile_begin was not called");
  ctx->profiling = false;
  for (int k = 0; k < LKV_N_KERNELS; ++k) {
    ms_per_kernel[k] = 0.0;
    launches[k] = 0;
  }
  for (size_t i = 0; i < ctx->ev_kind->size(); ++i) {
    hipError_t e = hipEventSynchronize((*ctx->ev_pool)[2 * i + 1]);
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, (*ctx->ev_pool)[2 * i], (*ctx->ev_pool)[2 * i + 1]);
    if (e != hipSuccess) {
      ctx->ev_kind->clear();
      return fail_hip(ctx, e, "profile_end: event timing");
    }
    ms_per_kernel[(*ctx->ev_kind)[i]] += ms;
    launches[(*ctx->ev_kind)[i]] += 1;
  }
  ctx->ev_kind->clear();
  return LKV_OK;
}

}  // extern "C"

namespace {

struct StaticDevice {
  bool ready;
  unsigned char* scratch;  // device address of this GPU's copy of the scratch array
  int n_cu;
};
StaticDevice g_static[kMaxDevices];
std::mutex g_static_mutex;

// Once per device, with that device current: the address of its scratch array, its compute-unit count and
// the kernels' LDS attributes.  Nothing here allocates device memory.
int static_device(StaticDevice** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(nullptr, e, "compress_block_static: hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, LKV_EINVAL, "compress_block_static: device %d not supported", dev);
  std::lock_guard<std::mutex> lock(g_static_mutex);
  StaticDevice& sd = g_static[dev];
  if (!sd.ready) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return fail_hip(nullptr, e, "compress_block_static: hipGetSymbolAddress");
    int n_cu = 0;
    e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return fail_hip(nullptr, e, "compress_block_static: device query");
    e = lkv::init_kernel_attributes();
    if (e != hipSuccess) return fail_hip(nullptr, e, "compress_block_static: kernel attribute");
    sd.scratch = static_cast<unsigned char*>(ptr);
    sd.n_cu = n_cu;
    sd.ready = true;
  }
  *out = &sd;
  return LKV_OK;
}

}  // namespace

extern "C" {

int laserkv_static_init(void) {
  StaticDevice* sd = nullptr;
  return static_device(&sd);
}

size_t laserkv_static_workspace_bytes(const laserkv_config* cfg) {
  if (!cfg || check_config(*cfg, "static_workspace_bytes") != LKV_OK) return 0;
  WsPlan ws;
  plan_workspace(*cfg, true, ws);
  return ws.total();
}

int laserkv_compress_block_static(const laserkv_config* cfg,
                                  const void* q_win, int64_t q_stride_head, int64_t q_stride_tok,
                                  const void* k_blk, int64_t k_stride_head, int64_t k_stride_tok,
                                  const void* v_blk, int64_t v_stride_head, int64_t v_stride_tok,
                                  const void* k_ctx, int64_t c_stride_head, int64_t c_stride_tok,
                                  const void* hyperplanes,
                                  int32_t s_t, int32_t w, int32_t t_ctx,
                                  int64_t block_pos0, int64_t q_pos0, int32_t causal,
                                  int32_t n_anchor, int32_t n_local, int32_t k_exact, int32_t k_lsh,
                                  int32_t* keep_idx,
                                  void* k_cache, void* v_cache, int64_t cache_stride_head,
                                  int64_t* cache_pos, int64_t pos_stride_head,
                                  int64_t cache_len, int64_t cache_cap,
                                  void* hip_stream) {
  if (!cfg) return fail(nullptr, LKV_EINVAL, "compress_block_static: null configuration");
  int rc = check_config(*cfg, "compress_block_static");
  if (rc != LKV_OK) return rc;
  WsPlan ws;
  plan_workspace(*cfg, true, ws);
  if (ws.total() > LKV_STATIC_SCRATCH_BYTES)
    return fail(nullptr, LKV_EINVAL, "compress_block_static: this configuration needs %zu bytes of workspace, the static "
                "scratch holds %zu (use laserkv_create + laserkv_compress_block)", ws.total(), (size_t)LKV_STATIC_SCRATCH_BYTES);
  StaticDevice* sd = nullptr;
  rc = static_device(&sd);
  if (rc != LKV_OK) return rc;
  // a context on the stack whose workspace is carved out of this GPU's scratch array
  laserkv_ctx ctx;
  memset(&ctx, 0, sizeof(ctx));
  init_ctx_fields(&ctx, *cfg);
  hipError_t e = hipGetDevice(&ctx.device);
  if (e != hipSuccess) return fail_hip(nullptr, e, "compress_block_static: hipGetDevice");
  ctx.n_cu = sd->n_cu;
  void* ptr[kWsBuffers];
  size_t off = 0;
  for (int i = 0; i < kWsBuffers; ++i) {
    ptr[i] = ws.bytes[i] ? sd->scratch + off : nullptr;
    off += (ws.bytes[i] + 255) & ~(size_t)255;
  }
  bind_workspace(&ctx, ws, ptr);
  rc = laserkv_compress_block(&ctx, q_win, q_stride_head, q_stride_tok, k_blk, k_stride_head, k_stride_tok,
                              v_blk, v_stride_head, v_stride_tok, k_ctx, c_stride_head, c_stride_tok, hyperplanes,
                              s_t, w, t_ctx, block_pos0, q_pos0, causal, n_anchor, n_local, k_exact, k_lsh, keep_idx,
                              k_cache, v_cache, cache_stride_head, cache_pos, pos_stride_head, cache_len, cache_cap,
                              hip_stream);
  if (rc != LKV_OK) memcpy(g_error, ctx.error, sizeof(g_error));  // the stack context is gone after return
  return rc;
}

}  // extern "C"
