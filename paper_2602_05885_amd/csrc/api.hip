// Host side of the C ABI: argument validation, workspace planning, kernel sequencing.
// Nothing here synchronises with the device or allocates device memory.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/pg_head.h"
#include "gemm_core.h"
#include "kernels.h"

namespace {

thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

constexpr size_t ALIGN = 256;
constexpr uint64_t FOUR_GIB = 1ull << 32;
constexpr uint64_t DS_BUDGET = 2ull << 30;   // bytes per orientation of the dS chunk scratch
constexpr double LOG2E = 1.4426950408889634;

// Tuning knob: PG_HEAD_DS_BUDGET_BYTES overrides the size of the dS chunk scratch (and with
// it the number of vocab chunks of the backward pass).
uint64_t ds_budget() {
  if (const char* e = std::getenv("PG_HEAD_DS_BUDGET_BYTES")) {
    const unsigned long long v = std::strtoull(e, nullptr, 10);
    if (v > 0) return v;
  }
  return DS_BUDGET;
}

inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

// Leading dimension of the caller-owned W^T cache [d, ld]: the vocabulary rounded up to whole tiles.
inline int64_t wt_cache_ld(int64_t V) { return pg::pad_ld((V + 255) / 256 * 256); }

struct Plan {
  int64_t T = 0, d = 0, V = 0;
  int is_f32 = 0;
  int t_cap = 0;       // T rounded up to 256
  int kd = 0;          // contraction length of the logits (d, or 3d for the split fp32 path)
  int tiles_v = 0;     // 256-row vocab tiles
  int tiles_t = 0;
  int chunk_tiles = 0; // vocab tiles per backward chunk
  int nchunks = 0;
  int vc = 0;          // chunk_tiles * 256
  int ld_v = 0;        // leading dimension of the [*, vc] scratch matrices
  int ld_t = 0;        // leading dimension of the [*, t_cap] scratch matrices
  int queue_words = 0; // tile-queue counters (8 per persistent launch)
  size_t ctl, counters, queue, flag, c_tok, a_tok, rows, pos, yc, zy, lse2, coefc, lossterm;
  size_t part_m, part_s, part_u, Hc, HcT, Wc, dS, dST, WT, dHacc, rstd_c = 0, norm_partial = 0;
  size_t HcT_lo = 0, dS_lo = 0, dST_lo = 0, WT_lo = 0;   // fp32 heads only
  size_t total = 0;
};

int32_t check_params(const pg_params* p) {
  if (!p) return fail(PG_ERR_INVALID_ARG, "params is NULL");
  if (p->dtype != PG_DTYPE_BF16 && p->dtype != PG_DTYPE_F32) return fail(PG_ERR_INVALID_ARG, "unknown dtype %d", p->dtype);
  if (!(p->temperature > 0.f) || !std::isfinite(p->temperature))
    return fail(PG_ERR_INVALID_ARG, "temperature must be finite and > 0");
  if (p->mismatch_mode < 0 || p->mismatch_mode > 2) return fail(PG_ERR_INVALID_ARG, "unknown mismatch_mode %d", p->mismatch_mode);
  if (!(p->clip_eps_lo >= 0.f) || !(p->clip_eps_hi >= 0.f)) return fail(PG_ERR_INVALID_ARG, "clip eps must be >= 0");
  if (p->mismatch_mode == PG_MISMATCH_GEOMETRIC && !(p->geo_lo <= p->geo_hi))
    return fail(PG_ERR_INVALID_ARG, "geo_lo must be <= geo_hi");
  if (p->mismatch_mode == PG_MISMATCH_TRUNCATE && !(p->trunc_c > 0.f))
    return fail(PG_ERR_INVALID_ARG, "trunc_c must be > 0");
  if (!(p->veto_ratio >= 0.f)) return fail(PG_ERR_INVALID_ARG, "veto_ratio must be >= 0");
  if (p->dW_dtype != 0 && p->dW_dtype != 1) return fail(PG_ERR_INVALID_ARG, "unknown dW_dtype %d", p->dW_dtype);
  if (p->n_samples < 0) return fail(PG_ERR_INVALID_ARG, "n_samples must be >= 0");
  if (p->w_transposed_valid != 0 && p->w_transposed_valid != 1) return fail(PG_ERR_INVALID_ARG, "w_transposed_valid must be 0 or 1");
  if (p->w_transposed && (reinterpret_cast<uintptr_t>(p->w_transposed) & 15u)) return fail(PG_ERR_INVALID_ARG, "w_transposed must be 16-byte aligned");
  return PG_OK;
}

int32_t make_plan(int64_t T, int64_t d, int64_t V, int32_t S, const pg_params* p, int which, Plan& pl) {
  int32_t rc = check_params(p);
  if (rc) return rc;
  if (which != PG_CALL_LOGPROB_FWD && which != PG_CALL_LOSS_FWD_BWD && which != PG_CALL_LOSS_FWD_BWD_NORMED)
    return fail(PG_ERR_INVALID_ARG, "unknown call id %d", which);
  if (T < 0 || d < 1 || V < 1 || S < 0) return fail(PG_ERR_INVALID_ARG, "negative or zero extent (T=%lld d=%lld V=%lld S=%d)", (long long)T, (long long)d, (long long)V, S);
  if (d % 64 != 0) return fail(PG_ERR_UNSUPPORTED_SHAPE, "d=%lld is not a multiple of 64", (long long)d);
  if (T > (1ll << 30) || V > (1ll << 30)) return fail(PG_ERR_UNSUPPORTED_SHAPE, "T or V too large");
  pl.T = T; pl.d = d; pl.V = V;
  pl.is_f32 = p->dtype == PG_DTYPE_F32;
  const int64_t t_cap = (T + 255) / 256 * 256;
  const int64_t kd = pl.is_f32 ? 3 * d : d;
  const int64_t tiles_v = (V + 255) / 256;
  // a tile's 256 operand rows are addressed through one 32-bit buffer range
  if ((uint64_t)kd * 2 * 256 >= FOUR_GIB) return fail(PG_ERR_UNSUPPORTED_SHAPE, "d=%lld: 256 operand rows reach 4 GiB", (long long)d);
  if ((uint64_t)(t_cap + 64) * 2 * 256 >= FOUR_GIB) return fail(PG_ERR_UNSUPPORTED_SHAPE, "T=%lld: 256 rows of a [*, T] scratch matrix reach 4 GiB", (long long)T);
  // tile indices and queue tickets are 32-bit, with 3 bits of a ticket naming the XCD
  if (tiles_v * (t_cap / 256) >= (1ll << 28))
    return fail(PG_ERR_UNSUPPORTED_SHAPE, "T=%lld x V=%lld: more than 2^28 logits tiles", (long long)T, (long long)V);
  pl.t_cap = (int)t_cap; pl.kd = (int)kd; pl.tiles_v = (int)tiles_v; pl.tiles_t = (int)(t_cap / 256);

  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  pl.ctl = take(sizeof(pg::Ctl));
  pl.counters = take(8 * sizeof(unsigned long long));
  pl.flag = take((size_t)T);
  pl.c_tok = take((size_t)T * 4);
  pl.a_tok = take((size_t)T * 4);
  pl.rows = take((size_t)t_cap * 4);
  pl.pos = take((size_t)T * 4);
  pl.yc = take((size_t)t_cap * 4);
  pl.zy = take((size_t)t_cap * 4);
  pl.lse2 = take((size_t)t_cap * 4);
  pl.coefc = take((size_t)t_cap * 4);
  pl.lossterm = take((size_t)t_cap * 4);
  pl.part_m = take((size_t)tiles_v * t_cap * 4);
  pl.part_s = take((size_t)tiles_v * t_cap * 4);
  pl.part_u = take((size_t)tiles_v * t_cap * 4);
  pl.Hc = take((size_t)t_cap * kd * 2);
  pl.Wc = pl.is_f32 ? take((size_t)V * kd * 2) : 0;
  pl.queue_words = pg::QUEUE_SET_WORDS * pg::queue_sets(0);
  if (which == PG_CALL_LOSS_FWD_BWD_NORMED) {
    if (d > pg::NORM_MAX_D) return fail(PG_ERR_UNSUPPORTED_SHAPE, "d=%lld: the fused normalisation takes d <= %d", (long long)d, pg::NORM_MAX_D);
    pl.rstd_c = take((size_t)t_cap * 4);
    pl.norm_partial = take((size_t)pg::NORM_STRIPS * d * 4);
  }
  if (which != PG_CALL_LOGPROB_FWD) {
    int64_t max_tiles = t_cap > 0 ? (int64_t)(ds_budget() / ((uint64_t)t_cap * 2 * 256)) : tiles_v;
    if (max_tiles < 1) max_tiles = 1;
    if (max_tiles > tiles_v) max_tiles = tiles_v;
    // Chunk size: within the scratch budget, the size whose dW launches (chunk_tiles x ceil(d/256)
    // tiles each, over 256 compute units) waste the fewest partly filled rounds; every extra chunk
    // is charged half a round for its launches and its pass over the dH accumulator.
    int64_t chunk_tiles = max_tiles;
    if (tiles_v > max_tiles) {
      const int64_t td = (d + 255) / 256;
      double best = 1e30;
      for (int64_t ct = max_tiles; ct >= 1 && ct * 3 >= max_tiles * 2; --ct) {
        const int64_t nch = (tiles_v + ct - 1) / ct;
        const int64_t last = tiles_v - (nch - 1) * ct;
        const double cost = (double)((nch - 1) * ((ct * td + 255) / 256) + (last * td + 255) / 256) + 0.5 * (double)nch;
        if (cost < best) { best = cost; chunk_tiles = ct; }
      }
    }
    const int64_t nchunks = (tiles_v + chunk_tiles - 1) / chunk_tiles;
    const int64_t vc = chunk_tiles * 256;
    const int64_t ld_v = pg::pad_ld(vc), ld_t = pg::pad_ld(t_cap);
    if ((uint64_t)ld_v * 2 * 256 >= FOUR_GIB || (uint64_t)ld_t * 2 * 256 >= FOUR_GIB)
      return fail(PG_ERR_UNSUPPORTED_SHAPE, "256 rows of a backward scratch matrix reach 4 GiB");
    pl.nchunks = (int)nchunks; pl.chunk_tiles = (int)chunk_tiles; pl.vc = (int)vc;
    pl.ld_v = (int)ld_v; pl.ld_t = (int)ld_t;
    pl.HcT = take((size_t)d * ld_t * 2);
    pl.dS = take((size_t)t_cap * ld_v * 2);
    pl.dST = take((size_t)vc * ld_t * 2);
    pl.WT = take((size_t)d * ld_v * 2);
    if (pl.is_f32) {   // bf16 remainders of the four backward operands
      pl.HcT_lo = take((size_t)d * ld_t * 2);
      pl.dS_lo = take((size_t)t_cap * ld_v * 2);
      pl.dST_lo = take((size_t)vc * ld_t * 2);
      pl.WT_lo = take((size_t)d * ld_v * 2);
    }
    pl.dHacc = take((size_t)t_cap * d * 4);
    pl.queue_words = pg::QUEUE_SET_WORDS * pg::queue_sets((int)nchunks);
  }
  pl.queue = take((size_t)pl.queue_words * sizeof(unsigned));
  pl.total = off > 0 ? off : ALIGN;
  return PG_OK;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int32_t ensure_init() {
  static bool done[64] = {};
  static std::mutex mu;
  std::lock_guard<std::mutex> lock(mu);
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return fail(PG_ERR_HIP, "hipGetDevice failed");
  if (dev < 0 || dev >= 64) return fail(PG_ERR_HIP, "device index %d out of range", dev);
  if (!done[dev]) {
    hipError_t e = pg::init_gemm_kernels();
    if (e != hipSuccess) return fail(PG_ERR_HIP, "kernel attribute setup failed: %s", hipGetErrorString(e));
    done[dev] = true;
  }
  return PG_OK;
}

// ---- scratch of the entry point that allocates nothing (pg_monitors_static) ----
// The monitors' partial sums ([6][MON_BLOCKS] fp64, 48 KiB) in a file-scope device array: every GPU
// the library runs on holds its own copy, at its own address, until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; kernels get the resolved address.
constexpr size_t MON_SCRATCH_DOUBLES = (size_t)6 * pg::MON_BLOCKS;
static __device__ __align__(256) double scratch[MON_SCRATCH_DOUBLES];

// Device address of `scratch` on the current device, resolved once per device.
int32_t monitors_scratch(double** out) {
  static double* ptr[64] = {};
  static std::mutex mu;
  std::lock_guard<std::mutex> lock(mu);
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return fail(PG_ERR_HIP, "hipGetDevice failed");
  if (dev < 0 || dev >= 64) return fail(PG_ERR_HIP, "device index %d out of range", dev);
  if (!ptr[dev]) {
    double* p = nullptr;
    hipError_t e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(PG_ERR_HIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return PG_OK;
}

// Launch errors.  hipGetLastError() would also return (and clear) an error that some earlier HIP
// call of the caller left behind, and blame it on this call; instead the error state is looked at
// without clearing it, before the first launch and after the last one, and only a state that
// changed in between is reported.  An error present on entry is left for the caller to find.
struct LaunchGuard {
  hipError_t before;
  LaunchGuard() : before(hipPeekAtLastError()) {}
  int32_t check(const char* what) const {
    const hipError_t e = hipPeekAtLastError();
    if (e != hipSuccess && e != before) return fail(PG_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return PG_OK;
  }
};

int32_t check_monitor_args(const float* logp_train, const uint8_t* loss_mask, int64_t T, const void* dH, int32_t dH_dtype,
                           int64_t dH_elems, const void* dW, int32_t dW_dtype, int64_t dW_elems, const double* out) {
  if (T < 0 || dH_elems < 0 || dW_elems < 0) return fail(PG_ERR_INVALID_ARG, "negative extent");
  if (!out) return fail(PG_ERR_INVALID_ARG, "out must not be NULL");
  if (T > 0 && (!logp_train || !loss_mask)) return fail(PG_ERR_INVALID_ARG, "logp_train and loss_mask must not be NULL when T > 0");
  if ((dH && dH_dtype != 0 && dH_dtype != 1) || (dW && dW_dtype != 0 && dW_dtype != 1))
    return fail(PG_ERR_INVALID_ARG, "gradient dtype must be 0 (bf16) or 1 (fp32)");
  if ((dH && misaligned(dH)) || (dW && misaligned(dW))) return fail(PG_ERR_INVALID_ARG, "dH and dW must be 16-byte aligned");
  return PG_OK;
}

// ---- optional per-kernel timing (measurement hook; off by default) ----
// When enabled, every launch of the three MFMA kernels is bracketed by a pair of events on the
// caller's stream, taken from a pool created up front.  Not thread-safe.
struct Profiler {
  bool on = false;
  std::vector<hipEvent_t> ev;     // 2 per recorded launch
  std::vector<int> cls;           // kernel class per recorded launch
  size_t cap = 0;
} g_prof;

struct ProfScope {
  hipStream_t st;
  bool active;
  ProfScope(int cls, hipStream_t s) : st(s), active(false) {
    if (g_prof.on && g_prof.cls.size() < g_prof.cap) {
      active = true;
      (void)hipEventRecord(g_prof.ev[2 * g_prof.cls.size()], st);
      g_prof.cls.push_back(cls);
    }
  }
  ~ProfScope() {
    if (active) (void)hipEventRecord(g_prof.ev[2 * (g_prof.cls.size() - 1) + 1], st);
  }
};

template <typename T>
T* at(void* ws, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(ws) + off); }

// Steps shared by both calls: pre-pass, operand staging, forward contraction, combine.
// y_offset: first vocab row of W within the whole vocabulary (0 unless W is a vocab shard).  With
// comb.partials_in set, the contraction is skipped and the rows' states come from there.
void run_forward(const Plan& pl, const pg_params& p, void* ws, const void* H, const void* W, const int32_t* y,
                 int64_t y_offset, const pg::PrepArgs& prep, pg::CombineArgs comb, bool need_HT, hipStream_t st,
                 const pg::NormFuse* norm = nullptr) {
  pg::launch_prepass(prep, st);
  const void* Wop = W;
  if (pl.is_f32) {
    pg::launch_split_w(static_cast<const float*>(W), at<__bf16>(ws, pl.Wc), pl.V, (int)pl.d, st);
    Wop = at<__bf16>(ws, pl.Wc);
  }
  pg::GatherArgs g{};
  g.H = H; g.y = y; g.d = (int)pl.d; g.t_cap = pl.t_cap; g.is_f32 = pl.is_f32;
  g.rows = at<int>(ws, pl.rows); g.Hc = at<__bf16>(ws, pl.Hc);
  g.HcT = need_HT ? at<__bf16>(ws, pl.HcT) : nullptr;
  g.HcT_lo = need_HT && pl.is_f32 ? at<__bf16>(ws, pl.HcT_lo) : nullptr;
  g.yc = at<int>(ws, pl.yc); g.ctl = at<pg::Ctl>(ws, pl.ctl); g.ld_t = pl.ld_t;
  g.y_offset = (int)y_offset; g.V = (int)pl.V;
  if (norm) pg::launch_norm_gather(g, *norm, st);
  else pg::launch_gather(g, st);

  pg::FwdArgs f{};
  f.W = Wop; f.Hc = at<__bf16>(ws, pl.Hc);
  f.w_rows = (int)pl.V; f.h_rows = pl.t_cap;
  f.ldw = pl.kd; f.ldh = pl.kd; f.K = pl.kd; f.V = (int)pl.V;
  f.tiles_v = pl.tiles_v; f.tiles_t = pl.tiles_t; f.t_cap = pl.t_cap;
  f.scale = (float)(LOG2E / (double)p.temperature);
  f.yc = at<int>(ws, pl.yc); f.zy = at<float>(ws, pl.zy);
  f.part_m = at<float>(ws, pl.part_m); f.part_s = at<float>(ws, pl.part_s); f.part_u = at<float>(ws, pl.part_u);
  f.ctl = at<pg::Ctl>(ws, pl.ctl);
  f.queue = at<unsigned>(ws, pl.queue);
  if (!comb.partials_in) { ProfScope ps(PG_KERNEL_FWD, st); pg::launch_lmhead_fwd(f, st); }

  comb.tiles_v = comb.partials_in ? 0 : pl.tiles_v; comb.t_cap = pl.t_cap;
  comb.part_m = f.part_m; comb.part_s = f.part_s; comb.part_u = f.part_u;
  comb.zy = f.zy; comb.rows = at<int>(ws, pl.rows); comb.lse2 = at<float>(ws, pl.lse2);
  comb.ctl = f.ctl;
  pg::launch_combine(comb, st);
}

pg::PrepArgs base_prep(const Plan& pl, void* ws) {
  pg::PrepArgs a{};
  a.T = (int)pl.T; a.t_cap = pl.t_cap;
  a.flag = at<uint8_t>(ws, pl.flag); a.c_tok = at<float>(ws, pl.c_tok); a.a_tok = at<float>(ws, pl.a_tok);
  a.rows = at<int>(ws, pl.rows); a.pos = at<int>(ws, pl.pos); a.zy = at<float>(ws, pl.zy);
  a.counters = at<unsigned long long>(ws, pl.counters); a.ctl = at<pg::Ctl>(ws, pl.ctl);
  a.queue = at<unsigned>(ws, pl.queue); a.queue_words = pl.queue_words;
  return a;
}

int32_t turn_advantage(const float* rewards, const uint8_t* valid, int32_t P, int32_t K, int32_t Tmax, float gamma,
                       double* returns_out, double* adv_out, int32_t* group_n_out, int group_mean, void* stream,
                       const char* what) {
  if (!rewards || !valid || !adv_out) return fail(PG_ERR_INVALID_ARG, "rewards, valid and adv_out must not be NULL");
  if (P < 1 || K < 1 || Tmax < 1) return fail(PG_ERR_INVALID_ARG, "P, K, Tmax must be >= 1");
  if ((int64_t)P * K * Tmax > (1ll << 30)) return fail(PG_ERR_UNSUPPORTED_SHAPE, "P*K*Tmax too large");
  if (!std::isfinite(gamma)) return fail(PG_ERR_INVALID_ARG, "gamma must be finite");
  const LaunchGuard guard;
  pg::TrlooArgs a{rewards, valid, P, K, Tmax, gamma, returns_out, adv_out, group_n_out, group_mean};
  pg::launch_trloo(a, static_cast<hipStream_t>(stream));
  return guard.check(what);
}

// W as one vocab shard of a larger head: rows [v_offset, v_offset + V) of the vocabulary, the rows'
// softmax states merged over all shards (nullptr: W is the whole head and the forward
// contraction runs here), and whether dH (a partial sum over this shard) is written as fp32.
// The normalisation fused around the head (pg_loss_fwd_bwd_normed): H of the call is X.
struct NormIn {
  const void* gamma;
  float eps;
  float* dgamma;
};

struct Shard {
  const float* partials = nullptr;
  int64_t v_offset = 0;
  int dH_f32 = 0;
  const char* what = nullptr;
};

// Loss forward + backward shared by the policy-gradient call (sft = 0) and the SFT
// cross-entropy call (sft = 1: no segments, no advantages, no mismatch correction).
int32_t loss_fwd_bwd(int sft, const void* H, const void* W, const int32_t* y, const uint8_t* loss_mask,
                     const int32_t* cu_seqlens, int32_t S, const double* adv, const int32_t* seg_sample,
                     const uint8_t* sample_keep, const float* old_logp, const float* rollout_logp, int64_t T, int64_t d,
                     int64_t V, const pg_params* h_params, float* loss_out, void* dH, void* dW, float* logp_out,
                     float* entropy_out, int64_t* counters_out, void* workspace, size_t workspace_bytes, void* stream,
                     const Shard& shard, const NormIn* norm = nullptr);

}  // namespace

extern "C" {

const char* pg_last_error(void) { return g_err; }

int32_t pg_init(void) {
  int32_t rc = ensure_init();
  if (rc) return rc;
  double* unused = nullptr;
  return monitors_scratch(&unused);
}

int32_t pg_profile_enable(int32_t on, int32_t max_launches) {
  for (hipEvent_t e : g_prof.ev) (void)hipEventDestroy(e);
  g_prof.ev.clear(); g_prof.cls.clear(); g_prof.cap = 0; g_prof.on = false;
  if (!on) return PG_OK;
  if (max_launches < 1 || max_launches > (1 << 20)) return fail(PG_ERR_INVALID_ARG, "max_launches out of range");
  g_prof.ev.resize(2 * (size_t)max_launches);
  for (auto& e : g_prof.ev)
    if (hipEventCreate(&e) != hipSuccess) return fail(PG_ERR_HIP, "hipEventCreate failed");
  g_prof.cls.reserve(max_launches);
  g_prof.cap = (size_t)max_launches;
  g_prof.on = true;
  return PG_OK;
}

int32_t pg_profile_read(double* h_ms, int64_t* h_launches) {
  if (!h_ms || !h_launches) return fail(PG_ERR_INVALID_ARG, "output arrays must not be NULL");
  for (int k = 0; k < PG_KERNEL_CLASSES; ++k) { h_ms[k] = 0.0; h_launches[k] = 0; }
  for (size_t i = 0; i < g_prof.cls.size(); ++i) {
    if (hipEventSynchronize(g_prof.ev[2 * i + 1]) != hipSuccess) return fail(PG_ERR_HIP, "hipEventSynchronize failed");
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]) != hipSuccess)
      return fail(PG_ERR_HIP, "hipEventElapsedTime failed");
    h_ms[g_prof.cls[i]] += ms;
    h_launches[g_prof.cls[i]] += 1;
  }
  g_prof.cls.clear();
  return PG_OK;
}

size_t pg_workspace_bytes(int64_t T, int64_t d, int64_t V, int32_t S, const pg_params* h_params, int32_t which_call) {
  Plan pl;
  if (make_plan(T, d, V, S, h_params, which_call, pl) != PG_OK) return 0;
  return pl.total;
}

size_t pg_w_transposed_bytes(int64_t d, int64_t V) {
  if (d < 1 || V < 1 || d % 64 != 0 || V > (1ll << 30)) return 0;
  const int64_t ld = wt_cache_ld(V);
  if ((uint64_t)ld * 2 * 256 >= FOUR_GIB) return 0;
  return align_up((size_t)d * (size_t)ld * 2);
}

int64_t pg_backward_chunk_rows(int64_t T, int64_t d, int64_t V, int32_t S, const pg_params* h_params) {
  Plan pl;
  if (make_plan(T, d, V, S, h_params, PG_CALL_LOSS_FWD_BWD, pl) != PG_OK) return 0;
  return pl.vc;
}

int32_t trloo_advantage(const float* rewards, const uint8_t* valid, int32_t P, int32_t K, int32_t Tmax, float gamma,
                        double* returns_out, double* adv_out, int32_t* group_n_out, void* stream) {
  return turn_advantage(rewards, valid, P, K, Tmax, gamma, returns_out, adv_out, group_n_out, 0, stream, "trloo_advantage");
}

int32_t grpo_advantage(const float* rewards, const uint8_t* valid, int32_t P, int32_t K, int32_t Tmax, float gamma,
                       double* returns_out, double* adv_out, int32_t* group_n_out, void* stream) {
  return turn_advantage(rewards, valid, P, K, Tmax, gamma, returns_out, adv_out, group_n_out, 1, stream, "grpo_advantage");
}

int32_t pg_logprob_fwd(const void* H, const void* W, const int32_t* y, const uint8_t* row_mask, int64_t T, int64_t d,
                       int64_t V, const pg_params* h_params, float* logp_out, float* entropy_out, float* lse_out,
                       void* workspace, size_t workspace_bytes, void* stream) {
  Plan pl;
  int32_t rc = make_plan(T, d, V, 0, h_params, PG_CALL_LOGPROB_FWD, pl);
  if (rc) return rc;
  if (T == 0) return PG_OK;
  if (!H || !W || !y || !logp_out || !workspace) return fail(PG_ERR_INVALID_ARG, "H, W, y, logp_out and workspace must not be NULL");
  if (misaligned(H) || misaligned(W) || misaligned(workspace)) return fail(PG_ERR_INVALID_ARG, "H, W and workspace must be 16-byte aligned");
  if (workspace_bytes < pl.total) return fail(PG_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, pl.total);
  if ((rc = ensure_init())) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);

  const LaunchGuard guard;

  pg::PrepArgs prep = base_prep(pl, workspace);
  prep.mask = row_mask;
  prep.out0 = logp_out; prep.out1 = entropy_out; prep.out2 = lse_out;
  pg::CombineArgs comb{};
  comb.logp_out = logp_out; comb.ent_out = entropy_out; comb.lse_out = lse_out;
  comb.with_loss = 0;
  run_forward(pl, *h_params, workspace, H, W, y, 0, prep, comb, false, st);
  return guard.check("pg_logprob_fwd");
}

int32_t pg_loss_fwd_bwd(const void* H, const void* W, const int32_t* y, const uint8_t* loss_mask,
                        const int32_t* cu_seqlens, int32_t S, const double* adv, const int32_t* seg_sample,
                        const uint8_t* sample_keep, const float* old_logp, const float* rollout_logp, int64_t T,
                        int64_t d, int64_t V, const pg_params* h_params, float* loss_out, void* dH, void* dW,
                        float* logp_out, float* entropy_out, int64_t* counters_out, void* workspace,
                        size_t workspace_bytes, void* stream) {
  return loss_fwd_bwd(0, H, W, y, loss_mask, cu_seqlens, S, adv, seg_sample, sample_keep, old_logp, rollout_logp, T, d, V,
                      h_params, loss_out, dH, dW, logp_out, entropy_out, counters_out, workspace, workspace_bytes, stream,
                      Shard{});
}

int32_t pg_loss_fwd_bwd_normed(const void* X, const void* gamma, float norm_eps, const void* W, const int32_t* y,
                               const uint8_t* loss_mask, const int32_t* cu_seqlens, int32_t S, const double* adv,
                               const int32_t* seg_sample, const uint8_t* sample_keep, const float* old_logp,
                               const float* rollout_logp, int64_t T, int64_t d, int64_t V, const pg_params* h_params,
                               float* loss_out, void* dX, float* dgamma_out, void* dW, float* logp_out,
                               float* entropy_out, int64_t* counters_out, void* workspace, size_t workspace_bytes,
                               void* stream) {
  const NormIn norm{gamma, norm_eps, dgamma_out};
  return loss_fwd_bwd(0, X, W, y, loss_mask, cu_seqlens, S, adv, seg_sample, sample_keep, old_logp, rollout_logp, T, d, V,
                      h_params, loss_out, dX, dW, logp_out, entropy_out, counters_out, workspace, workspace_bytes, stream,
                      Shard{}, &norm);
}

int32_t pg_head_shard_fwd(const void* H, const void* W_shard, const int32_t* y, const uint8_t* row_mask, int64_t T,
                          int64_t d, int64_t V_shard, int64_t v_offset, const pg_params* h_params, float* partials_out,
                          void* workspace, size_t workspace_bytes, void* stream) {
  Plan pl;
  int32_t rc = make_plan(T, d, V_shard, 0, h_params, PG_CALL_LOGPROB_FWD, pl);
  if (rc) return rc;
  if (v_offset < 0 || v_offset > (1ll << 30)) return fail(PG_ERR_INVALID_ARG, "v_offset out of range");
  if (T == 0) return PG_OK;
  if (!H || !W_shard || !y || !partials_out || !workspace)
    return fail(PG_ERR_INVALID_ARG, "H, W_shard, y, partials_out and workspace must not be NULL");
  if (misaligned(H) || misaligned(W_shard) || misaligned(workspace) || misaligned(partials_out))
    return fail(PG_ERR_INVALID_ARG, "H, W_shard, partials_out and workspace must be 16-byte aligned");
  if (workspace_bytes < pl.total) return fail(PG_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, pl.total);
  if ((rc = ensure_init())) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);

  const LaunchGuard guard;

  pg::launch_fill_zero_bytes(partials_out, (size_t)T * 4 * sizeof(float), st);   // rows that are masked out stay empty
  pg::PrepArgs prep = base_prep(pl, workspace);
  prep.mask = row_mask;
  pg::CombineArgs comb{};
  comb.with_loss = 0;
  comb.partials_out = partials_out;
  run_forward(pl, *h_params, workspace, H, W_shard, y, v_offset, prep, comb, false, st);
  return guard.check("pg_head_shard_fwd");
}

int32_t pg_head_partials_merge(const float* a, const float* b, float* out, int64_t T, void* stream) {
  if (T < 0) return fail(PG_ERR_INVALID_ARG, "T must be >= 0");
  if (T == 0) return PG_OK;
  if (!a || !b || !out) return fail(PG_ERR_INVALID_ARG, "a, b and out must not be NULL");
  if (misaligned(a) || misaligned(b) || misaligned(out)) return fail(PG_ERR_INVALID_ARG, "a, b and out must be 16-byte aligned");
  const LaunchGuard guard;
  pg::launch_merge_partials(a, b, out, T, static_cast<hipStream_t>(stream));
  return guard.check("pg_head_partials_merge");
}

int32_t pg_head_partials_finish(const float* partials, int64_t T, float* logp_out, float* entropy_out, float* lse_out,
                                void* stream) {
  if (T < 0) return fail(PG_ERR_INVALID_ARG, "T must be >= 0");
  if (T == 0) return PG_OK;
  if (!partials || !logp_out) return fail(PG_ERR_INVALID_ARG, "partials and logp_out must not be NULL");
  if (misaligned(partials)) return fail(PG_ERR_INVALID_ARG, "partials must be 16-byte aligned");
  const LaunchGuard guard;
  pg::launch_finish_partials(partials, T, logp_out, entropy_out, lse_out, static_cast<hipStream_t>(stream));
  return guard.check("pg_head_partials_finish");
}

int32_t pg_loss_shard_bwd(const void* H, const void* W_shard, const int32_t* y, const uint8_t* loss_mask,
                          const int32_t* cu_seqlens, int32_t S, const double* adv, const int32_t* seg_sample,
                          const uint8_t* sample_keep, const float* old_logp, const float* rollout_logp,
                          const float* partials, int64_t T, int64_t d, int64_t V_shard, int64_t v_offset, const pg_params* h_params, float* loss_out, void* dH_partial,
                          int32_t dH_f32, void* dW_shard, float* logp_out, float* entropy_out, int64_t* counters_out,
                          void* workspace, size_t workspace_bytes, void* stream) {
  if (v_offset < 0 || v_offset > (1ll << 30)) return fail(PG_ERR_INVALID_ARG, "v_offset out of range");
  if (dH_f32 != 0 && dH_f32 != 1) return fail(PG_ERR_INVALID_ARG, "dH_f32 must be 0 or 1");
  if (T > 0 && !partials) return fail(PG_ERR_INVALID_ARG, "partials must not be NULL");
  if (misaligned(partials)) return fail(PG_ERR_INVALID_ARG, "partials must be 16-byte aligned");
  Shard sh;
  sh.partials = partials; sh.v_offset = v_offset; sh.dH_f32 = dH_f32; sh.what = "pg_loss_shard_bwd";
  return loss_fwd_bwd(0, H, W_shard, y, loss_mask, cu_seqlens, S, adv, seg_sample, sample_keep, old_logp, rollout_logp, T,
                      d, V_shard, h_params, loss_out, dH_partial, dW_shard, logp_out, entropy_out, counters_out, workspace,
                      workspace_bytes, stream, sh);
}

int32_t pg_sft_fwd_bwd(const void* H, const void* W, const int32_t* y, const uint8_t* loss_mask, int64_t T, int64_t d,
                       int64_t V, const pg_params* h_params, float* loss_out, void* dH, void* dW, float* logp_out,
                       float* entropy_out, int64_t* counters_out, void* workspace, size_t workspace_bytes,
                       void* stream) {
  return loss_fwd_bwd(1, H, W, y, loss_mask, nullptr, 0, nullptr, nullptr, nullptr, nullptr, nullptr, T, d, V, h_params,
                      loss_out, dH, dW, logp_out, entropy_out, counters_out, workspace, workspace_bytes, stream, Shard{});
}

int32_t turn_reward(const uint8_t* correct, const float* t_reference, const float* t_kernel, const float* t_generated,
                    const float* t_total, int64_t n, float speedup_cap, float* rewards_out, float* pr_out,
                    void* stream) {
  if (n < 0) return fail(PG_ERR_INVALID_ARG, "n must be >= 0");
  if (n == 0) return PG_OK;
  if (!correct || !t_reference || !t_kernel || !rewards_out)
    return fail(PG_ERR_INVALID_ARG, "correct, t_reference, t_kernel and rewards_out must not be NULL");
  if ((t_generated == nullptr) != (t_total == nullptr))
    return fail(PG_ERR_INVALID_ARG, "t_generated and t_total must be given together");
  if (!(speedup_cap > 0.f) || !std::isfinite(speedup_cap)) return fail(PG_ERR_INVALID_ARG, "speedup_cap must be finite and > 0");
  const LaunchGuard guard;
  pg::RewardArgs a{correct, t_reference, t_kernel, t_generated, t_total, (long long)n, speedup_cap, rewards_out, pr_out};
  pg::launch_turn_reward(a, static_cast<hipStream_t>(stream));
  return guard.check("turn_reward");
}

int32_t prs_retain(const float* pr, const uint8_t* valid, int64_t n, float tau, float s, int32_t hard, uint64_t seed,
                   uint8_t* keep_out, float* p_out, void* stream) {
  if (n < 0) return fail(PG_ERR_INVALID_ARG, "n must be >= 0");
  if (n == 0) return PG_OK;
  if (!pr || !keep_out) return fail(PG_ERR_INVALID_ARG, "pr and keep_out must not be NULL");
  if (!(s > 0.f) || !std::isfinite(s) || !std::isfinite(tau)) return fail(PG_ERR_INVALID_ARG, "tau must be finite and s finite and > 0");
  const LaunchGuard guard;
  pg::PrsArgs a{pr, valid, (long long)n, tau, s, hard != 0, (unsigned long long)seed, keep_out, p_out};
  pg::launch_prs_retain(a, static_cast<hipStream_t>(stream));
  return guard.check("prs_retain");
}

size_t pg_monitors_workspace_bytes(void) { return (size_t)6 * pg::MON_BLOCKS * sizeof(double); }

int32_t pg_monitors(const float* logp_train, const float* logp_rollout, const float* entropy, const uint8_t* loss_mask,
                    int64_t T, const void* dH, int32_t dH_dtype, int64_t dH_elems, const void* dW, int32_t dW_dtype,
                    int64_t dW_elems, double* out, void* workspace, size_t workspace_bytes, void* stream) {
  int32_t rc = check_monitor_args(logp_train, loss_mask, T, dH, dH_dtype, dH_elems, dW, dW_dtype, dW_elems, out);
  if (rc) return rc;
  if (!workspace) return fail(PG_ERR_INVALID_ARG, "workspace must not be NULL");
  if (reinterpret_cast<uintptr_t>(workspace) & 7u) return fail(PG_ERR_INVALID_ARG, "workspace must be 8-byte aligned");
  if (workspace_bytes < pg_monitors_workspace_bytes())
    return fail(PG_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, pg_monitors_workspace_bytes());
  const LaunchGuard guard;
  pg::MonitorArgs a{logp_train, logp_rollout, entropy, loss_mask, (long long)T, dH, dH_dtype, (long long)dH_elems,
                    dW, dW_dtype, (long long)dW_elems, static_cast<double*>(workspace), out};
  pg::launch_monitors(a, static_cast<hipStream_t>(stream));
  return guard.check("pg_monitors");
}

int32_t pg_monitors_static(const float* logp_train, const float* logp_rollout, const float* entropy,
                           const uint8_t* loss_mask, int64_t T, const void* dH, int32_t dH_dtype, int64_t dH_elems,
                           const void* dW, int32_t dW_dtype, int64_t dW_elems, double* out, void* stream) {
  int32_t rc = check_monitor_args(logp_train, loss_mask, T, dH, dH_dtype, dH_elems, dW, dW_dtype, dW_elems, out);
  if (rc) return rc;
  if (T > PG_MONITORS_STATIC_MAX_ROWS || dH_elems > PG_MONITORS_STATIC_MAX_ELEMS || dW_elems > PG_MONITORS_STATIC_MAX_ELEMS)
    return fail(PG_ERR_UNSUPPORTED_SHAPE,
                "pg_monitors_static takes at most %lld rows and %lld elements per gradient (got T=%lld, dH_elems=%lld, "
                "dW_elems=%lld); use pg_monitors with a caller-owned workspace beyond that",
                (long long)PG_MONITORS_STATIC_MAX_ROWS, (long long)PG_MONITORS_STATIC_MAX_ELEMS, (long long)T,
                (long long)dH_elems, (long long)dW_elems);
  double* partial = nullptr;
  if ((rc = monitors_scratch(&partial))) return rc;
  const LaunchGuard guard;
  // every one of the 6 x MON_BLOCKS partial sums is rewritten by each call (one workgroup per
  // column), so nothing of the previous call's contents has to be cleared
  pg::MonitorArgs a{logp_train, logp_rollout, entropy, loss_mask, (long long)T, dH, dH_dtype, (long long)dH_elems,
                    dW, dW_dtype, (long long)dW_elems, partial, out};
  pg::launch_monitors(a, static_cast<hipStream_t>(stream));
  return guard.check("pg_monitors_static");
}

int32_t pg_rmsnorm_fwd(const void* X, const void* gamma, int64_t T, int64_t d, float eps, int32_t dtype, void* H_out,
                       float* rstd_out, void* stream) {
  if (T < 0 || d < 1) return fail(PG_ERR_INVALID_ARG, "T must be >= 0 and d >= 1");
  if (dtype != PG_DTYPE_BF16 && dtype != PG_DTYPE_F32) return fail(PG_ERR_INVALID_ARG, "unknown dtype %d", dtype);
  if (d % 8 != 0 || d > pg::NORM_MAX_D)
    return fail(PG_ERR_UNSUPPORTED_SHAPE, "d=%lld must be a multiple of 8 and at most %d", (long long)d, pg::NORM_MAX_D);
  if (!(eps >= 0.f) || !std::isfinite(eps)) return fail(PG_ERR_INVALID_ARG, "eps must be finite and >= 0");
  if (T == 0) return PG_OK;
  if (!X || !gamma || !H_out) return fail(PG_ERR_INVALID_ARG, "X, gamma and H_out must not be NULL");
  if (misaligned(X) || misaligned(gamma) || misaligned(H_out)) return fail(PG_ERR_INVALID_ARG, "X, gamma and H_out must be 16-byte aligned");
  const LaunchGuard guard;
  pg::NormArgs a{};
  a.X = X; a.gamma = gamma; a.T = T; a.d = (int)d; a.eps = eps; a.is_f32 = dtype == PG_DTYPE_F32;
  a.H = H_out; a.rstd_out = rstd_out;
  pg::launch_rmsnorm_fwd(a, static_cast<hipStream_t>(stream));
  return guard.check("pg_rmsnorm_fwd");
}

size_t pg_rmsnorm_bwd_workspace_bytes(int64_t d) {
  if (d < 1 || d % 8 != 0 || d > pg::NORM_MAX_D) return 0;
  return (size_t)pg::NORM_STRIPS * (size_t)d * sizeof(float);
}

int32_t pg_rmsnorm_bwd(const void* X, const void* gamma, const void* dH, int64_t T, int64_t d, float eps, int32_t dtype,
                       void* dX_out, float* dgamma_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (T < 0 || d < 1) return fail(PG_ERR_INVALID_ARG, "T must be >= 0 and d >= 1");
  if (dtype != PG_DTYPE_BF16 && dtype != PG_DTYPE_F32) return fail(PG_ERR_INVALID_ARG, "unknown dtype %d", dtype);
  if (d % 8 != 0 || d > pg::NORM_MAX_D)
    return fail(PG_ERR_UNSUPPORTED_SHAPE, "d=%lld must be a multiple of 8 and at most %d", (long long)d, pg::NORM_MAX_D);
  if (!(eps >= 0.f) || !std::isfinite(eps)) return fail(PG_ERR_INVALID_ARG, "eps must be finite and >= 0");
  if (!dgamma_out || !workspace) return fail(PG_ERR_INVALID_ARG, "dgamma_out and workspace must not be NULL");
  if (T > 0 && (!X || !gamma || !dH || !dX_out)) return fail(PG_ERR_INVALID_ARG, "X, gamma, dH and dX_out must not be NULL");
  if (misaligned(X) || misaligned(gamma) || misaligned(dH) || misaligned(dX_out) || misaligned(workspace))
    return fail(PG_ERR_INVALID_ARG, "X, gamma, dH, dX_out and workspace must be 16-byte aligned");
  if (workspace_bytes < pg_rmsnorm_bwd_workspace_bytes(d))
    return fail(PG_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, pg_rmsnorm_bwd_workspace_bytes(d));
  const LaunchGuard guard;
  pg::NormArgs a{};
  a.X = X; a.gamma = gamma; a.T = T; a.d = (int)d; a.eps = eps; a.is_f32 = dtype == PG_DTYPE_F32;
  a.dH = dH; a.dX = dX_out; a.partial = static_cast<float*>(workspace); a.dgamma = dgamma_out;
  pg::launch_rmsnorm_bwd(a, static_cast<hipStream_t>(stream));
  return guard.check("pg_rmsnorm_bwd");
}

}  // extern "C"

namespace {

int32_t loss_fwd_bwd(int sft, const void* H, const void* W, const int32_t* y, const uint8_t* loss_mask,
                     const int32_t* cu_seqlens, int32_t S, const double* adv, const int32_t* seg_sample,
                     const uint8_t* sample_keep, const float* old_logp, const float* rollout_logp, int64_t T, int64_t d,
                     int64_t V, const pg_params* h_params, float* loss_out, void* dH, void* dW, float* logp_out,
                     float* entropy_out, int64_t* counters_out, void* workspace, size_t workspace_bytes, void* stream,
                     const Shard& shard, const NormIn* norm) {
  Plan pl;
  int32_t rc = make_plan(T, d, V, S, h_params, norm ? PG_CALL_LOSS_FWD_BWD_NORMED : PG_CALL_LOSS_FWD_BWD, pl);
  if (rc) return rc;
  const pg_params& p = *h_params;
  if (!W || !loss_out || !dW) return fail(PG_ERR_INVALID_ARG, "W, loss_out and dW must not be NULL");
  if (misaligned(W) || misaligned(dW)) return fail(PG_ERR_INVALID_ARG, "W and dW must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t dw_elem = p.dW_dtype ? 2 : 4;
  if (norm) {
    if (!norm->gamma || !norm->dgamma) return fail(PG_ERR_INVALID_ARG, "gamma and dgamma_out must not be NULL");
    if (misaligned(norm->gamma)) return fail(PG_ERR_INVALID_ARG, "gamma must be 16-byte aligned");
    if (!(norm->eps >= 0.f) || !std::isfinite(norm->eps)) return fail(PG_ERR_INVALID_ARG, "norm_eps must be finite and >= 0");
  }
  if (T == 0) {   // empty microbatch: zero loss, zero gradient
    const LaunchGuard guard;
    if (norm) pg::launch_fill_f32(norm->dgamma, (size_t)d, 0.f, st);
    pg::launch_fill_f32(loss_out, 1, 0.f, st);
    if (counters_out) pg::launch_fill_zero_bytes(counters_out, 8 * sizeof(int64_t), st);
    if (!p.accumulate_dW) pg::launch_fill_zero_bytes(dW, (size_t)V * d * dw_elem, st);
    return guard.check(shard.what ? shard.what : sft ? "pg_sft_fwd_bwd (empty)" : "pg_loss_fwd_bwd (empty)");
  }
  if (!H || !y || !loss_mask || !dH || !workspace)
    return fail(PG_ERR_INVALID_ARG, "H, y, loss_mask, dH and workspace must not be NULL");
  if (!sft) {
    if (!cu_seqlens || !adv) return fail(PG_ERR_INVALID_ARG, "cu_seqlens and adv must not be NULL");
    if (S < 1) return fail(PG_ERR_INVALID_ARG, "S must be >= 1 when T > 0");
    if (p.mismatch_mode != PG_MISMATCH_NONE && (!old_logp || !rollout_logp))
      return fail(PG_ERR_INVALID_ARG, "mismatch correction needs old_logp and rollout_logp");
  }
  if (misaligned(H) || misaligned(dH) || misaligned(workspace)) return fail(PG_ERR_INVALID_ARG, "H, dH and workspace must be 16-byte aligned");
  if (workspace_bytes < pl.total) return fail(PG_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, pl.total);
  if ((rc = ensure_init())) return rc;
  void* ws = workspace;
  const LaunchGuard guard;

  pg::PrepArgs prep = base_prep(pl, ws);
  prep.mask = loss_mask; prep.cu = cu_seqlens; prep.S = S; prep.adv = adv; prep.seg_sample = seg_sample;
  prep.sample_keep = sample_keep; prep.n_samples = p.n_samples;
  prep.old_logp = old_logp; prep.rollout_logp = rollout_logp;
  prep.mismatch_mode = sft ? PG_MISMATCH_NONE : p.mismatch_mode; prep.geo_lo = p.geo_lo; prep.geo_hi = p.geo_hi;
  prep.veto_ratio = p.veto_ratio; prep.trunc_c = p.trunc_c; prep.norm_override = p.norm_override;
  prep.out0 = logp_out; prep.out1 = entropy_out; prep.out2 = nullptr;

  pg::CombineArgs comb{};
  comb.logp_out = logp_out; comb.ent_out = entropy_out; comb.lse_out = nullptr;
  comb.with_loss = sft ? 2 : 1; comb.old_logp = old_logp;
  comb.c_tok = at<float>(ws, pl.c_tok); comb.a_tok = at<float>(ws, pl.a_tok);
  comb.eps_lo = p.clip_eps_lo; comb.eps_hi = p.clip_eps_hi; comb.inv_tau = 1.f / p.temperature;
  comb.coefc = at<float>(ws, pl.coefc); comb.lossterm = at<float>(ws, pl.lossterm);
  comb.counters = at<unsigned long long>(ws, pl.counters);
  comb.partials_in = shard.partials;
  pg::NormFuse nf{};
  if (norm) {
    nf.X = H; nf.gamma = norm->gamma; nf.eps = norm->eps; nf.dgamma = norm->dgamma;
    nf.rstd_c = at<float>(ws, pl.rstd_c); nf.partial = at<float>(ws, pl.norm_partial);
  }
  run_forward(pl, p, ws, H, W, y, shard.v_offset, prep, comb, true, st, norm ? &nf : nullptr);

  pg::FinishArgs fin{at<float>(ws, pl.lossterm), at<unsigned long long>(ws, pl.counters), loss_out,
                     reinterpret_cast<long long*>(counters_out), at<pg::Ctl>(ws, pl.ctl)};
  pg::launch_finish(fin, st);

  // ---- backward, one vocab chunk at a time ----
  const void* Wop = pl.is_f32 ? static_cast<const void*>(at<__bf16>(ws, pl.Wc)) : W;
  const pg::Ctl* ctl = at<pg::Ctl>(ws, pl.ctl);
  const int d_i = (int)pl.d;
  for (int c = 0; c < pl.nchunks; ++c) {
    const int v0 = c * pl.vc;
    if (v0 >= pl.V) break;
    const int rows_valid = (int)((pl.V - v0) < pl.vc ? (pl.V - v0) : pl.vc);
    const int tiles_c = (rows_valid + 255) / 256;
    const int kc = tiles_c * 256;

    // W^T of this chunk: in the workspace, or a column range of the caller's cache (filled here unless valid)
    __bf16* wt = at<__bf16>(ws, pl.WT);
    int ld_wt = pl.ld_v;
    if (p.w_transposed) {
      wt = static_cast<__bf16*>(p.w_transposed) + v0;
      ld_wt = (int)wt_cache_ld(pl.V);
    }
    if (!p.w_transposed || !p.w_transposed_valid) pg::launch_transpose_w(W, pl.is_f32, pl.V, d_i, d_i, v0, kc, ld_wt, wt, st);
    if (pl.is_f32)   // the remainders W - bf16(W) are columns [d, 2d) of the split operand
      pg::launch_transpose_w(at<__bf16>(ws, pl.Wc) + d_i, 0, pl.V, d_i, pl.kd, v0, kc, pl.ld_v, at<__bf16>(ws, pl.WT_lo), st);

    pg::DlogitsArgs g{};
    g.W = Wop; g.Hc = at<__bf16>(ws, pl.Hc);
    g.w_rows = (int)pl.V; g.h_rows = pl.t_cap;
    g.ldw = pl.kd; g.ldh = pl.kd; g.K = pl.kd; g.V = (int)pl.V; g.v0 = v0; g.ld_s = pl.ld_v; g.ld_t = pl.ld_t;
    g.tiles_v = tiles_c; g.tiles_t = pl.tiles_t; g.t_cap = pl.t_cap;
    g.scale = (float)(LOG2E / (double)p.temperature);
    g.yc = at<int>(ws, pl.yc); g.lse2 = at<float>(ws, pl.lse2); g.coefc = at<float>(ws, pl.coefc);
    g.dS = at<__bf16>(ws, pl.dS); g.dST = at<__bf16>(ws, pl.dST); g.ctl = ctl;
    if (pl.is_f32) { g.dS_lo = at<__bf16>(ws, pl.dS_lo); g.dST_lo = at<__bf16>(ws, pl.dST_lo); }
    pg::Rechunk rc{};
    rc.enabled = pl.nchunks > 1; rc.chunk = c; rc.tiles_v_all = pl.tiles_v; rc.ld_s_all = (int)pg::pad_ld((int64_t)pl.tiles_v * 256);
    rc.cap_s = (long long)pl.t_cap * pl.ld_v; rc.cap_t = (long long)pl.vc * pl.ld_t;
    g.rc = rc;
    unsigned* const queues = at<unsigned>(ws, pl.queue) + pg::QUEUE_SET_WORDS * (1 + 4 * c);
    g.queue = queues; g.queue_lo = queues + 3 * pg::QUEUE_SET_WORDS;
    { ProfScope ps(PG_KERNEL_DLOGITS, st); pg::launch_lmhead_dlogits(g, st); }

    pg::StoreArgs w{};   // dW[v0 + m, :] = sum_t dS^T[m, t] H^T[:, t]
    w.A = at<__bf16>(ws, pl.dST); w.B = at<__bf16>(ws, pl.HcT);
    if (pl.is_f32) { w.A_lo = at<__bf16>(ws, pl.dST_lo); w.B_lo = at<__bf16>(ws, pl.HcT_lo); w.ldb_lo = pl.ld_t; }
    w.a_rows = pl.vc; w.b_rows = d_i;
    w.lda = pl.ld_t; w.ldb = pl.ld_t; w.M = rows_valid; w.N = d_i; w.K = pl.t_cap;
    w.tiles_m = tiles_c; w.tiles_n = (d_i + 255) / 256;
    w.C = static_cast<char*>(dW) + (size_t)v0 * pl.d * dw_elem; w.ldc = d_i;
    w.accumulate = p.accumulate_dW; w.out_bf16 = p.dW_dtype; w.k_from_ctl = 1; w.m_from_ctl = 0; w.ctl = ctl;
    w.queue = queues + pg::QUEUE_SET_WORDS;
    w.rc = rc; w.rc_role = 1; w.v0 = v0;
    { ProfScope ps(PG_KERNEL_DW, st); pg::launch_gemm_store(w, st); }

    pg::StoreArgs h{};   // dHacc[t, :] (+)= sum_v dS[t, v] W^T[:, v]
    h.A = at<__bf16>(ws, pl.dS); h.B = wt;
    if (pl.is_f32) { h.A_lo = at<__bf16>(ws, pl.dS_lo); h.B_lo = at<__bf16>(ws, pl.WT_lo); h.ldb_lo = pl.ld_v; }
    h.a_rows = pl.t_cap; h.b_rows = d_i;
    h.lda = pl.ld_v; h.ldb = ld_wt; h.M = pl.t_cap; h.N = d_i; h.K = kc;
    h.tiles_m = pl.tiles_t; h.tiles_n = (d_i + 255) / 256;
    h.C = at<float>(ws, pl.dHacc); h.ldc = d_i;
    h.accumulate = c > 0; h.out_bf16 = 0; h.k_from_ctl = 0; h.m_from_ctl = 1; h.split_k = 1; h.ctl = ctl;
    h.queue = queues + 2 * pg::QUEUE_SET_WORDS;
    h.rc = rc; h.rc_role = 2; h.v0 = v0;
    { ProfScope ps(PG_KERNEL_DH, st); pg::launch_gemm_store(h, st); }
  }

  const int kc0 = (int)(((pl.V < pl.vc ? pl.V : pl.vc) + 255) / 256 * 256);      // contraction length of the first chunk
  pg::ScatterArgs sc{at<float>(ws, pl.dHacc), at<int>(ws, pl.pos), dH, (int)pl.T, d_i, pl.is_f32 || shard.dH_f32,
                     1, pl.t_cap, (d_i + 255) / 256, kc0 / 64, ctl};
  if (norm) pg::launch_scatter_dx_norm(sc, nf, st);
  else pg::launch_scatter_dh(sc, st);
  return guard.check(shard.what ? shard.what : sft ? "pg_sft_fwd_bwd" : norm ? "pg_loss_fwd_bwd_normed" : "pg_loss_fwd_bwd");
}

}  // namespace
