// Argument blocks and launchers of the device kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pg {

struct Ctl;

// Tile-queue counters in the workspace: one set of 8 (one per XCD) for every persistent launch of a
// call (the forward, then recompute / dW / dH / remainder recompute of every vocab chunk), all cleared
// by the pre-pass.
constexpr int QUEUE_SET_WORDS = 8;
inline int queue_sets(int nchunks) { return 1 + 4 * nchunks; }

// Scratch leading dimensions (multiples of 64 elements = 128 bytes) are made an odd number of
// 128-byte lines, so that the rows of a tile spread over the memory channels instead of
// landing on a few of them (power-of-two strides measured 3 % slower).
__host__ __device__ inline long long pad_ld(long long n) { return ((n / 64) % 2 == 0) ? n + 64 : n; }

// Few active rows (most samples rejected: known only on the device).  The chunk scratch is sized for
// t_cap rows; when the rows that are really active are so few that dS of the WHOLE vocabulary fits it, the
// first chunk's recompute launch covers the whole vocabulary (the same buffers, laid out as
// [n_pad, ld_s_all] and [V_pad, pad_ld(n_pad)]: 14 rounds of tiles in one launch instead of seven launches
// of 2.1 rounds at the 14B head with 1536 rows) and the later chunks' recompute launches return at once;
// the dW and dH launches keep their chunks and read their rows of the wide dS^T, their columns of the wide
// dS.  Every kernel takes the decision from the same device-side values, and a tile's arithmetic does not
// depend on it.
struct Rechunk {
  int enabled;          // the backward was planned in more than one vocab chunk
  int chunk;            // this launch's chunk
  int tiles_v_all;      // 256-row vocab tiles of the whole head
  int ld_s_all;         // pad_ld(256 tiles_v_all)
  long long cap_s;      // elements of the dS scratch
  long long cap_t;      // elements of the dS^T scratch
};
__device__ inline bool rechunk_all(const Rechunk& r, int n_pad, int& ld_t_all) {
  ld_t_all = (int)pad_ld(n_pad);
  return r.enabled && n_pad > 0 && (long long)n_pad * r.ld_s_all <= r.cap_s &&
         (long long)r.tiles_v_all * 256 * ld_t_all <= r.cap_t;
}

// ---- MFMA kernels ---------------------------------------------------------------------
struct FwdArgs {
  const void* W;        // [V, ldw] bf16
  const void* Hc;       // [t_cap, ldh] bf16, compacted rows, zero padded
  int w_rows, h_rows;   // rows that exist in W / Hc (loads beyond them give 0)
  int ldw, ldh;         // elements
  int K;                // contraction length (multiple of 64)
  int V;
  int tiles_v, tiles_t; // tile counts (tiles_t from t_cap; tiles beyond n_pad exit)
  int t_cap;
  float scale;          // log2(e) / tau
  const int* yc;        // [t_cap] compacted token ids (-1 on padding)
  float* zy;            // [t_cap] scaled logit of the sampled token
  float* part_m;        // [tiles_v, t_cap] each
  float* part_s;
  float* part_u;
  const Ctl* ctl;
  unsigned* queue;      // [8] tile counters of this launch's queue, zero at launch
};

struct DlogitsArgs {
  const void* W;
  const void* Hc;
  int w_rows, h_rows;   // rows that exist in W / Hc (loads beyond them give 0)
  int ldw, ldh;
  int K;
  int V;
  int v0;               // first vocab row of this chunk
  int ld_s;             // leading dimension of dS   (>= chunk capacity)
  int ld_t;             // leading dimension of dS^T (>= t_cap)
  int tiles_v, tiles_t; // tiles of this chunk
  int t_cap;
  float scale;
  const int* yc;
  const float* lse2;    // [t_cap] log2-domain logsumexp
  const float* coefc;   // [t_cap] coef / tau (0 on padding)
  __bf16* dS;           // [t_cap, ld_s]
  __bf16* dST;          // [vc, ld_t]
  __bf16* dS_lo;        // fp32 heads: the bf16 remainders dS - bf16(dS), same two layouts; else null
  __bf16* dST_lo;
  const Ctl* ctl;
  unsigned* queue;      // [8] tile counters of this launch's queue, zero at launch
  unsigned* queue_lo;   // [8] the same for the launch that stores the remainders
  Rechunk rc;
};

struct StoreArgs {
  const void* A;        // [M, lda] bf16
  const void* B;        // [N, ldb] bf16
  const void* A_lo;     // fp32 heads: bf16 remainders of A and B (same shapes; A_lo with A's leading dimension,
  const void* B_lo;     // B_lo with ldb_lo); the contraction then adds A B_lo and A_lo B to A B.  Both null otherwise.
  int ldb_lo;
  int a_rows, b_rows;   // rows that exist in A / B (loads beyond them give 0)
  int lda, ldb;
  int M, N, K;
  int tiles_m, tiles_n;
  void* C;              // [M, ldc] fp32 or bf16
  int ldc;
  int accumulate;
  int out_bf16;
  int k_from_ctl;       // contraction length = padded active-token count
  int m_from_ctl;       // row extent        = padded active-token count
  int split_k;          // with m_from_ctl: cut K into dh_split() parts, part p writes rows p n_pad + m
  const Ctl* ctl;
  unsigned* queue;      // [8] tile counters of this launch's queue, zero at launch
  Rechunk rc;           // see there; rc_role 0: not a chunked launch, 1: dW of a chunk, 2: dH of a chunk
  int rc_role;
  int v0;               // first vocab row of the chunk: its rows of the whole-vocabulary dS^T, its columns of dS
};

hipError_t init_gemm_kernels();
void launch_lmhead_fwd(const FwdArgs& a, hipStream_t s);
void launch_lmhead_dlogits(const DlogitsArgs& a, hipStream_t s);
void launch_gemm_store(const StoreArgs& a, hipStream_t s);

// ---- row / vector kernels ----------------------------------------------------------------
struct TrlooArgs {
  const float* rewards;
  const uint8_t* valid;
  int P, K, Tmax;
  float gamma;
  double* returns_out;
  double* adv_out;
  int* group_n_out;
  int group_mean;      // 0: leave-one-out baseline (Eq. 5), 1: group-mean baseline (Eq. 3)
};
void launch_trloo(const TrlooArgs& a, hipStream_t s);

struct PrepArgs {
  // inputs
  const uint8_t* mask;       // [T] loss / row mask (nullable = all ones)
  const int* cu;             // [S+1] (nullable: no segments, every row its own weight 1)
  int S;
  const double* adv;
  const int* seg_sample;
  const uint8_t* sample_keep; // indexed like adv (nullable = keep all): 0 drops the segment
  int n_samples;             // entries of adv / sample_keep (0 = unknown: indices are not range-checked)
  const float* old_logp;
  const float* rollout_logp;
  int T, t_cap;
  int mismatch_mode;
  float geo_lo, geo_hi, veto_ratio, trunc_c, norm_override;
  // workspace
  uint8_t* flag;             // [T]
  float* c_tok;              // [T]
  float* a_tok;              // [T]
  int* rows;                 // [t_cap]
  int* pos;                  // [T]
  float* zy;                 // [t_cap]
  unsigned long long* counters; // [8]
  unsigned* queue;           // [queue_words] tile-queue counters of the persistent kernels, cleared here
  int queue_words;
  Ctl* ctl;
  // per-row outputs to clear
  float* out0; float* out1; float* out2;
};
void launch_prepass(const PrepArgs& a, hipStream_t s);

struct GatherArgs {
  const void* H;        // [T, d] bf16 or fp32
  const int* y;
  int d, t_cap;
  int is_f32;
  const int* rows;
  __bf16* Hc;           // [t_cap, ldh]   bf16: ldh = d;  fp32: ldh = 3d = [hi | hi | lo]
  __bf16* HcT;          // [d, ld_t] (nullable): transpose of the bf16 operand / of the hi parts
  __bf16* HcT_lo;       // [d, ld_t] (nullable, fp32 only): transpose of the lo parts
  int ld_t;
  int* yc;              // y - y_offset where that lies in [0, V), else -1
  int y_offset, V;      // first vocab row and number of vocab rows of the weight operand
  const Ctl* ctl;
};
void launch_gather(const GatherArgs& a, hipStream_t s);
// HcT[j, i] = Hc[i, j] over d columns of row stride ldh, for the live rows
void launch_transpose_hc(const __bf16* Hc, int ldh, __bf16* HcT, const GatherArgs& g, hipStream_t s);

// fp32 head weight -> [V, 3d] bf16 = [hi | lo | hi]
void launch_split_w(const float* W, __bf16* Wc, int64_t V, int d, hipStream_t s);

struct CombineArgs {
  int tiles_v, t_cap;
  const float* part_m; const float* part_s; const float* part_u;
  const float* zy;
  const int* rows;
  float* lse2;
  float* logp_out; float* ent_out; float* lse_out;      // original-row indexed, nullable
  // loss epilogue: 0 none, 1 clipped surrogate, 2 cross-entropy (l = -logp, dl/dlogp = -1)
  int with_loss;
  const float* old_logp;     // original-row indexed, nullable
  const float* c_tok; const float* a_tok;
  float eps_lo, eps_hi, inv_tau;
  float* coefc;              // [t_cap]
  float* lossterm;           // [t_cap]
  unsigned long long* counters;
  // vocab-sharded head: partials_out != null writes the merged state of the row as
  // (m, s, u, z_y) in natural-log units at [row][4] and stops; partials_in != null takes the
  // row's state from there (the state merged over all shards) instead of from part_*.
  float* partials_out;
  const float* partials_in;
  const Ctl* ctl;
};
void launch_combine(const CombineArgs& a, hipStream_t s);

struct FinishArgs {
  const float* lossterm;
  const unsigned long long* counters;
  float* loss_out;
  long long* counters_out;
  const Ctl* ctl;
};
void launch_finish(const FinishArgs& a, hipStream_t s);

// W[v0 .. v0+cols) x d  ->  WT [d, ldt] bf16 (zeros for v >= V)
void launch_transpose_w(const void* W, int is_f32, int64_t V, int d, int ldw, int v0, int cols, int ldt, __bf16* WT,
                        hipStream_t s);

struct ScatterArgs {
  const float* acc;     // [t_cap, d]
  const int* pos;       // [T]
  void* dH;             // [T, d]
  int T, d;
  int out_f32;
  // split-K slabs of the accumulator (see dh_split): 0 = one slab; else the arguments of dh_split
  // as the first chunk's contraction saw them
  int split_k, t_cap, tiles_n, k_stages;
  const Ctl* ctl;
};
void launch_scatter_dh(const ScatterArgs& a, hipStream_t s);

// RMS normalisation fused around the head (h = x rstd gamma in front of it, its backward behind dH):
// the forward is applied while the active rows are compacted, the backward while dH is scattered.
struct NormFuse {
  const void* X;        // [T, d] bf16 or fp32: the rows in front of the normalisation
  const void* gamma;    // [d] same dtype
  float eps;
  float* rstd_c;        // [t_cap] workspace: 1 / rms of every compacted row
  float* partial;       // [NORM_STRIPS, d] workspace: dgamma partial sums
  float* dgamma;        // [d] output
};
// Hc[i, :] = normalised row rows[i] of X (zeros on padding), yc[i] as launch_gather; then Hc -> HcT.
void launch_norm_gather(const GatherArgs& g, const NormFuse& n, hipStream_t s);
// dX[t, :] = RMSNorm backward of the accumulated dH row of t (zeros for rows that are not active); dgamma.
void launch_scatter_dx_norm(const ScatterArgs& a, const NormFuse& n, hipStream_t s);

// out[t] = merge(a[t], b[t]) of two per-row softmax states (m, s, u, z_y), [T][4] each.
void launch_merge_partials(const float* a, const float* b, float* out, long long T, hipStream_t s);
// logsumexp = m + ln s, log-prob = z_y - logsumexp, entropy = ln s - u / s per row; 0 on empty rows.
void launch_finish_partials(const float* parts, long long T, float* logp, float* ent, float* lse, hipStream_t s);

// ---- stages around the path -------------------------------------------------------------
struct RewardArgs {
  const uint8_t* correct;
  const float* t_reference; const float* t_kernel;
  const float* t_generated; const float* t_total;   // both nullable
  long long n;
  float cap;
  float* rewards_out;
  float* pr_out;                                    // nullable
};
void launch_turn_reward(const RewardArgs& a, hipStream_t s);

struct PrsArgs {
  const float* pr;
  const uint8_t* valid;     // nullable
  long long n;
  float tau, s;
  int hard;
  unsigned long long seed;
  uint8_t* keep_out;
  float* p_out;             // nullable
};
void launch_prs_retain(const PrsArgs& a, hipStream_t s);

constexpr int MON_BLOCKS = 1024;     // partial sums per reduced quantity
struct MonitorArgs {
  const float* logp_train; const float* logp_rollout; const float* entropy;
  const uint8_t* mask;
  long long T;
  const void* dH; int dH_f32; long long dH_elems;
  const void* dW; int dW_f32; long long dW_elems;
  double* partial;          // [6][MON_BLOCKS]
  double* out;              // [8]
};
void launch_monitors(const MonitorArgs& a, hipStream_t s);

constexpr int NORM_STRIPS = 1024;    // row strips of the RMSNorm backward (one workgroup and one dgamma partial each)
constexpr int NORM_MAX_D = 8192;     // both kernels keep a row in registers (backward: 4 x 8 columns per thread of 256)
struct NormArgs {
  const void* X;        // [T, d] bf16 or fp32
  const void* gamma;    // [d]    same dtype
  long long T;
  int d;                // multiple of 8
  float eps;
  int is_f32;
  // forward
  void* H;              // [T, d] same dtype
  float* rstd_out;      // [T], nullable
  // backward
  const void* dH;       // [T, d] same dtype
  void* dX;             // [T, d] same dtype
  float* partial;       // [NORM_STRIPS, d]
  float* dgamma;        // [d]
};
void launch_rmsnorm_fwd(const NormArgs& a, hipStream_t s);
void launch_rmsnorm_bwd(const NormArgs& a, hipStream_t s);

void launch_fill_f32(float* p, size_t n, float v, hipStream_t s);
void launch_fill_zero_bytes(void* p, size_t nbytes, hipStream_t s);   // nbytes multiple of 4

}  // namespace pg
