// Vector / row kernels around the MFMA kernels: TRLOO advantages, mismatch pre-pass, row
// compaction, operand staging, the per-row softmax combine with the surrogate epilogue,
// and the final scatter of dH.  None of them is bandwidth- or flop-significant next to the
// contractions; they are written for determinism (fixed reduction orders, integer atomics
// only) and to keep the host out of the loop (no synchronisation, counts stay on device).
#include "kernels.h"
#include "gemm_core.h"

namespace pg {

// ------------------------------------------------------------------ fills
__global__ void fill_f32_kernel(float* p, size_t n, float v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}
void launch_fill_f32(float* p, size_t n, float v, hipStream_t s) {
  if (!p || n == 0) return;
  const int grid = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  hipLaunchKernelGGL(fill_f32_kernel, dim3(grid), dim3(256), 0, s, p, n, v);
}
void launch_fill_zero_bytes(void* p, size_t nbytes, hipStream_t s) {
  launch_fill_f32(reinterpret_cast<float*>(p), nbytes / 4, 0.f, s);
}

// ------------------------------------------------------------------ TRLOO (Sec. 4.2, Eq. 2, 3 and 5)
// A segmented group reduction: one wavefront per (prompt, turn) group, its 64 lanes striding over the
// K rollouts (the group's members lie Tmax elements apart in the [P, K, Tmax] tensors).  Every lane
// evaluates the returns of its rollouts once, by Horner's rule from the last turn backwards, and keeps
// them in registers (up to TRLOO_HELD per lane, i.e. K <= 64 TRLOO_HELD; beyond that they are evaluated
// again in the second sweep); the group's sum and count are then reduced across the wavefront by a
// butterfly of shuffles, whose order is fixed, so results repeat bit for bit.  fp64 throughout.  The
// leave-one-out mean is (sum - own) / (N - 1), the group mean of the comparison baseline sum / N.
constexpr int TRLOO_HELD = 4;

__device__ __forceinline__ double turn_return(const float* r, int t, int Tmax, double gamma) {
  double g = 0.0;
  for (int tp = Tmax - 1; tp >= t; --tp) g = (double)r[tp] + gamma * g;
  return g;
}

__global__ __launch_bounds__(256) void trloo_kernel(TrlooArgs a) {
  const int lane = threadIdx.x & 63;
  const int g = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);      // wavefront-uniform
  if (g >= a.P * a.Tmax) return;
  const int p = g / a.Tmax, t = g % a.Tmax;
  const double gamma = (double)a.gamma;
  double held[TRLOO_HELD];
  double sum = 0.0;
  int n = 0;
  for (int k = lane, i = 0; k < a.K; k += 64, ++i) {
    const size_t base = ((size_t)p * a.K + k) * a.Tmax;
    const double G = turn_return(a.rewards + base, t, a.Tmax, gamma);
    if (i < TRLOO_HELD) held[i] = G;
    if (a.returns_out) a.returns_out[base + t] = G;
    if (a.valid[base + t]) { sum += G; ++n; }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    sum += __shfl_xor(sum, off);
    n += __shfl_xor(n, off);
  }
  if (lane == 0 && a.group_n_out) a.group_n_out[g] = n;
  for (int k = lane, i = 0; k < a.K; k += 64, ++i) {
    const size_t base = ((size_t)p * a.K + k) * a.Tmax;
    double A = 0.0;
    if (a.valid[base + t]) {
      const double G = i < TRLOO_HELD ? held[i] : turn_return(a.rewards + base, t, a.Tmax, gamma);
      if (a.group_mean) A = G - sum / (double)n;                    // Eq. (3); n >= 1 here
      else if (n >= 2) A = G - (sum - G) / (double)(n - 1);         // Eq. (5)
    }
    a.adv_out[base + t] = A;
  }
}
void launch_trloo(const TrlooArgs& a, hipStream_t s) {
  const int n = a.P * a.Tmax;                                       // groups, 4 per workgroup
  hipLaunchKernelGGL(trloo_kernel, dim3((n + 3) / 4), dim3(256), 0, s, a);
}

// ------------------------------------------------------------------ pre-pass
__global__ void prep_init_kernel(PrepArgs a) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < 8) a.counters[i] = 0ull;
  for (int w = i; w < a.queue_words; w += gridDim.x * blockDim.x) a.queue[w] = 0u;
  if (i < a.t_cap) a.zy[i] = 0.f;
  if (i < a.T) {
    if (a.out0) a.out0[i] = 0.f;
    if (a.out1) a.out1[i] = 0.f;
    if (a.out2) a.out2[i] = 0.f;
    if (a.cu) {
      a.flag[i] = 0;
    } else {
      a.flag[i] = a.mask ? (a.mask[i] != 0) : 1;
      a.c_tok[i] = 1.f;
      a.a_tok[i] = 0.f;
    }
  }
}

// One workgroup per segment (= one training sample): Sec. 5.1's geometric-mean ratio and
// token veto over the sample's loss tokens, decided in fp64, then per-row weights.  A sample
// whose keep flag is 0 (Sec. 5.2's rejection sampling), or whose index lies outside the
// advantage table, is skipped before any of that.
__global__ __launch_bounds__(256) void prep_segment_kernel(PrepArgs a) {
  __shared__ double sh_sum[256];
  __shared__ double sh_min[256];
  __shared__ int sh_n[256];
  __shared__ int sh_keep;
  const int s = blockIdx.x, tid = threadIdx.x;
  int lo = a.cu[s], hi = a.cu[s + 1];
  lo = max(lo, 0);
  hi = min(hi, a.T);
  const bool mm = a.mismatch_mode != 0;
  // table entry of this segment; an index outside the tables drops the segment and reads nothing
  const int idx = a.seg_sample ? a.seg_sample[s] : s;
  const bool in_table = a.n_samples <= 0 || (idx >= 0 && idx < a.n_samples);
  double sum = 0.0, mn = 1.0e300;
  int n = 0;
  for (int t = lo + tid; t < hi; t += 256) {
    if (a.mask[t]) {
      ++n;
      if (mm) {
        const double dl = (double)a.old_logp[t] - (double)a.rollout_logp[t];
        sum += dl;
        mn = fmin(mn, dl);
      }
    }
  }
  sh_sum[tid] = sum; sh_min[tid] = mn; sh_n[tid] = n;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (tid < w) {
      sh_sum[tid] += sh_sum[tid + w];
      sh_min[tid] = fmin(sh_min[tid], sh_min[tid + w]);
      sh_n[tid] += sh_n[tid + w];
    }
    __syncthreads();
  }
  if (tid == 0) {
    int keep = 1;
    const int nn = sh_n[0];
    const bool dropped = !in_table || (a.sample_keep && !a.sample_keep[idx]);
    if (dropped) {            // filtered out before training (PRS): as if the sample had no loss rows
      keep = 0;
      if (nn > 0) atomicAdd(&a.counters[7], 1ull);
    } else if (nn > 0) {
      atomicAdd(&a.counters[6], (unsigned long long)nn);
      if (mm) {
        const bool vetoed = (a.veto_ratio > 0.f) && (exp(sh_min[0]) < (double)a.veto_ratio);
        if (vetoed) { atomicAdd(&a.counters[4], 1ull); keep = 0; }
        if (a.mismatch_mode == 1) {
          const double w = exp(sh_sum[0] / (double)nn);
          const bool inside = ((double)a.geo_lo <= w) && (w <= (double)a.geo_hi);
          if (!inside) { atomicAdd(&a.counters[3], 1ull); keep = 0; }
        }
      }
    }
    sh_keep = keep;
  }
  __syncthreads();
  const int keep = sh_keep;
  const float A = in_table ? (float)a.adv[idx] : 0.f;
  unsigned long long ntr = 0;
  for (int t = lo + tid; t < hi; t += 256) {
    const bool act = a.mask[t] && keep;
    float c = 0.f;
    if (act) {
      c = 1.f;
      if (a.mismatch_mode == 2) {
        const double ratio = exp((double)a.old_logp[t] - (double)a.rollout_logp[t]);
        if (ratio > (double)a.trunc_c) { ++ntr; c = a.trunc_c; } else { c = (float)ratio; }
      }
    }
    a.flag[t] = act;
    a.c_tok[t] = c;
    a.a_tok[t] = A;
  }
  if (ntr) atomicAdd(&a.counters[5], ntr);
}

// Single workgroup: exclusive scan of the active flags -> compacted row list, inverse map,
// counts and the loss normaliser.
__global__ __launch_bounds__(1024) void prep_compact_kernel(PrepArgs a) {
  __shared__ int sh[1024];
  const int tid = threadIdx.x;
  const int chunk = (a.T + 1023) / 1024;
  const int lo = min(a.T, tid * chunk), hi = min(a.T, lo + chunk);
  int cnt = 0;
  for (int t = lo; t < hi; ++t) cnt += a.flag[t] ? 1 : 0;
  sh[tid] = cnt;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    const int v = (tid >= off) ? sh[tid - off] : 0;
    __syncthreads();
    sh[tid] += v;
    __syncthreads();
  }
  int idx = sh[tid] - cnt;
  for (int t = lo; t < hi; ++t) {
    if (a.flag[t]) { a.rows[idx] = t; a.pos[t] = idx; ++idx; } else { a.pos[t] = -1; }
  }
  if (tid == 1023) {
    const int total = sh[1023];
    a.ctl->n_active = total;
    a.ctl->n_pad = (total + 255) / 256 * 256;
    a.ctl->norm = a.norm_override > 0.f ? a.norm_override : (float)max(total, 1);
    a.ctl->pad_ = 0;
    a.counters[0] = (unsigned long long)total;
    if (!a.cu) a.counters[6] = (unsigned long long)total;   // no segments: every flagged row is a loss row
  }
}

void launch_prepass(const PrepArgs& a, hipStream_t s) {
  const int n = a.t_cap > 8 ? a.t_cap : 8;
  hipLaunchKernelGGL(prep_init_kernel, dim3((n + 255) / 256), dim3(256), 0, s, a);
  if (a.cu && a.S > 0) hipLaunchKernelGGL(prep_segment_kernel, dim3(a.S), dim3(256), 0, s, a);
  hipLaunchKernelGGL(prep_compact_kernel, dim3(1), dim3(1024), 0, s, a);
}

// ------------------------------------------------------------------ operand staging
__device__ __forceinline__ void split_bf16(float x, __bf16& hi, __bf16& lo) {
  hi = (__bf16)x;
  lo = (__bf16)(x - (float)hi);
}

// ---- 64 x 64 bf16 tile transposition through LDS with 16-byte global accesses ----
// Rows are staged with a stride of 68 elements (34 words): 8-byte aligned for the row writes and
// odd enough in words that the column reads of the transposed phase spread over the banks.
constexpr int TT_LD = 68;

// thread t: 16-byte chunk t&7 of rows (t>>3) and (t>>3)+32
__device__ __forceinline__ void tt_put(uint16_t* tile, int row, int chunk, const i32x4& v) {
  uint2* p = reinterpret_cast<uint2*>(tile + row * TT_LD + chunk * 8);
  p[0] = make_uint2((uint32_t)v[0], (uint32_t)v[1]);
  p[1] = make_uint2((uint32_t)v[2], (uint32_t)v[3]);
}
// column `col`, rows chunk*8 .. chunk*8+7, packed as one 16-byte row piece of the transpose
__device__ __forceinline__ i32x4 tt_get(const uint16_t* tile, int col, int chunk) {
  uint32_t w[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const uint32_t lo = tile[(chunk * 8 + 2 * e) * TT_LD + col];
    const uint32_t hi = tile[(chunk * 8 + 2 * e + 1) * TT_LD + col];
    w[e] = lo | (hi << 16);
  }
  i32x4 v;
  v[0] = (int)w[0]; v[1] = (int)w[1]; v[2] = (int)w[2]; v[3] = (int)w[3];
  return v;
}

// 64 compacted rows x 64 columns per workgroup: copies (or splits) H rows into the compacted,
// zero-padded operand and writes its transpose for the dW contraction.
__global__ __launch_bounds__(256) void gather_kernel(GatherArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[64 * TT_LD];
  const Ctl ctl = *a.ctl;
  const int i0 = blockIdx.x * 64, j0 = blockIdx.y * 64;
  if (i0 >= ctl.n_pad) return;
  const int tid = threadIdx.x;
  if (blockIdx.y == 0 && tid < 64) {
    const int i = i0 + tid;
    int yl = -1;
    if (i < ctl.n_active) {
      yl = a.y[a.rows[i]] - a.y_offset;
      if (yl < 0 || yl >= a.V) yl = -1;
    }
    a.yc[i] = yl;
  }
  if (!a.is_f32) {
    const int chunk = tid & 7;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int r = (tid >> 3) + 32 * p;
      const int i = i0 + r;
      i32x4 v = {0, 0, 0, 0};
      if (i < ctl.n_active)
        v = *reinterpret_cast<const i32x4*>(reinterpret_cast<const __bf16*>(a.H) + (size_t)a.rows[i] * a.d + j0 + chunk * 8);
      *reinterpret_cast<i32x4*>(a.Hc + (size_t)i * a.d + j0 + chunk * 8) = v;
      tt_put(tile, r, chunk, v);
    }
    if (!a.HcT) return;
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int jj = (tid >> 3) + 32 * p;
      *reinterpret_cast<i32x4*>(a.HcT + (size_t)(j0 + jj) * a.ld_t + i0 + chunk * 8) = tt_get(tile, jj, chunk);
    }
    return;
  }
  // fp32 inputs: split into bf16 hi + lo parts, [hi | hi | lo] along k
  __bf16* tl = reinterpret_cast<__bf16*>(tile);
  const int ldh = 3 * a.d;
  const int r = tid >> 2, c0 = (tid & 3) * 16;
  const int i = i0 + r;
  const bool live = i < ctl.n_active;
  const size_t src = live ? (size_t)a.rows[i] * a.d + j0 + c0 : 0;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    __bf16 hi = (__bf16)0.f, lo = (__bf16)0.f;
    if (live) split_bf16(reinterpret_cast<const float*>(a.H)[src + e], hi, lo);
    const size_t o = (size_t)i * ldh + j0 + c0 + e;
    a.Hc[o] = hi;
    a.Hc[o + a.d] = hi;
    a.Hc[o + 2 * a.d] = lo;
    tl[r * TT_LD + c0 + e] = hi;
  }
  if (!a.HcT) return;
  __syncthreads();
  const int j = tid >> 2;
#pragma unroll
  for (int e = 0; e < 16; ++e) a.HcT[(size_t)(j0 + j) * a.ld_t + i0 + c0 + e] = tl[(c0 + e) * TT_LD + j];
}
void launch_gather(const GatherArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(gather_kernel, dim3(a.t_cap / 64, a.d / 64), dim3(256), 0, s, a);
  if (a.HcT_lo) launch_transpose_hc(a.Hc + 2 * a.d, 3 * a.d, a.HcT_lo, a, s);
}

__global__ void split_w_kernel(const float* W, __bf16* Wc, size_t n, int d) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    const size_t v = i / d, k = i % d;
    __bf16 hi, lo;
    split_bf16(W[i], hi, lo);
    __bf16* o = Wc + v * 3 * (size_t)d + k;
    o[0] = hi; o[d] = lo; o[2 * (size_t)d] = hi;
  }
}
void launch_split_w(const float* W, __bf16* Wc, int64_t V, int d, hipStream_t s) {
  const size_t n = (size_t)V * d;
  const int grid = (int)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
  hipLaunchKernelGGL(split_w_kernel, dim3(grid), dim3(256), 0, s, W, Wc, n, d);
}

// W rows [v0, v0+cols) (row stride ldw elements) -> WT[j][v - v0] (bf16; fp32 weights are rounded), zeros for v >= V.
__global__ __launch_bounds__(256) void transpose_w_kernel(const void* W, int is_f32, long long V, int ldw, int v0,
                                                          int ldt, __bf16* WT) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[64 * TT_LD];
  const int vt = blockIdx.x * 64, j0 = blockIdx.y * 64;
  const int tid = threadIdx.x;
  const int chunk = tid & 7;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int r = (tid >> 3) + 32 * p;
    const long long v = (long long)v0 + vt + r;
    i32x4 x = {0, 0, 0, 0};
    if (v < V) {
      const size_t o = (size_t)v * ldw + j0 + chunk * 8;
      if (is_f32) {
        const float* src = reinterpret_cast<const float*>(W) + o;
        bf16x8 h;
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = (__bf16)src[e];
        x = __builtin_bit_cast(i32x4, h);
      } else {
        x = *reinterpret_cast<const i32x4*>(reinterpret_cast<const __bf16*>(W) + o);
      }
    }
    tt_put(tile, r, chunk, x);
  }
  __syncthreads();
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int jj = (tid >> 3) + 32 * p;
    *reinterpret_cast<i32x4*>(WT + (size_t)(j0 + jj) * ldt + vt + chunk * 8) = tt_get(tile, jj, chunk);
  }
}
void launch_transpose_w(const void* W, int is_f32, int64_t V, int d, int ldw, int v0, int cols, int ldt, __bf16* WT,
                        hipStream_t s) {
  hipLaunchKernelGGL(transpose_w_kernel, dim3(cols / 64, d / 64), dim3(256), 0, s, W, is_f32, (long long)V, ldw, v0,
                     ldt, WT);
}

// ------------------------------------------------------------------ combine + surrogate
// Merges the per-vocab-tile softmax partials of every compacted row with the online merge rule
// (m, s, u) + (m2, s2, u2), emits log-prob / entropy / logsumexp, and for the loss call evaluates
// the clipped surrogate and the coefficient that scales (onehot - softmax) in the backward.
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs a) {
  // 64 tokens per workgroup; the four wavefronts each merge every fourth vocab tile's partial
  // state (online, fixed order), then wavefront 0 merges the four results and finishes the row.
  __shared__ float sh[3][3][64];
  const Ctl ctl = *a.ctl;
  const int lane = threadIdx.x & 63, part = threadIdx.x >> 6;
  const int i = blockIdx.x * 64 + lane;
  if (blockIdx.x * 64 >= ctl.n_pad) return;      // whole workgroup beyond the padded rows
  float M = -1.0e30f, s = 0.f, u = 0.f;
  for (int k = part; k < a.tiles_v; k += 4) {
    const size_t o = (size_t)k * a.t_cap + i;
    const float m2 = a.part_m[o], s2 = a.part_s[o], u2 = a.part_u[o];
    const float mm = fmaxf(M, m2);
    const float a1 = __builtin_amdgcn_exp2f(M - mm), a2 = __builtin_amdgcn_exp2f(m2 - mm);
    u = a1 * (u + (M - mm) * s) + a2 * (u2 + (m2 - mm) * s2);
    s = a1 * s + a2 * s2;
    M = mm;
  }
  if (part > 0) { sh[part - 1][0][lane] = M; sh[part - 1][1][lane] = s; sh[part - 1][2][lane] = u; }
  __syncthreads();
  if (part > 0) return;
#pragma unroll
  for (int w = 0; w < 3; ++w) {
    const float m2 = sh[w][0][lane], s2 = sh[w][1][lane], u2 = sh[w][2][lane];
    const float mm = fmaxf(M, m2);
    const float a1 = __builtin_amdgcn_exp2f(M - mm), a2 = __builtin_amdgcn_exp2f(m2 - mm);
    u = a1 * (u + (M - mm) * s) + a2 * (u2 + (m2 - mm) * s2);
    s = a1 * s + a2 * s2;
    M = mm;
  }
  const float LN2 = 0.693147180559945309f, LOG2E = 1.44269504088896341f;
  if (a.partials_out) {      // this shard's state of the row, natural-log units
    if (i < ctl.n_active)
      *reinterpret_cast<float4*>(a.partials_out + (size_t)a.rows[i] * 4) = make_float4(M * LN2, s, u * LN2, a.zy[i] * LN2);
    return;
  }
  float zy = a.zy[i];
  if (a.partials_in) {       // state merged over all shards; padded rows get lse = 0
    M = 0.f; s = 1.f; u = 0.f; zy = 0.f;
    if (i < ctl.n_active) {
      const float4 q = *reinterpret_cast<const float4*>(a.partials_in + (size_t)a.rows[i] * 4);
      M = q.x * LOG2E; s = q.y; u = q.z * LOG2E; zy = q.w * LOG2E;
    }
  }
  const float log2s = __builtin_amdgcn_logf(s);     // v_log_f32: log2
  const float lse2 = M + log2s;
  a.lse2[i] = lse2;
  if (i >= ctl.n_active) {
    if (a.with_loss) { a.coefc[i] = 0.f; a.lossterm[i] = 0.f; }
    return;
  }
  const int row = a.rows[i];
  const float logp = (zy - lse2) * LN2;
  if (a.logp_out) a.logp_out[row] = logp;
  if (a.ent_out) a.ent_out[row] = (log2s - u / s) * LN2;
  if (a.lse_out) a.lse_out[row] = lse2 * LN2;
  if (!a.with_loss) return;
  if (a.with_loss == 2) {            // cross-entropy: l = -logp, dl/dlogp = -1
    a.coefc[i] = -1.f / ctl.norm * a.inv_tau;
    a.lossterm[i] = -logp;
    return;
  }
  const float A = a.a_tok[row], c = a.c_tok[row];
  const float r = a.old_logp ? expf(logp - a.old_logp[row]) : 1.f;
  const float lo = 1.f - a.eps_lo, hi = 1.f + a.eps_hi;
  const float rc = fminf(fmaxf(r, lo), hi);
  float l = -fminf(r * A, rc * A);
  const bool flows = (A >= 0.f && r <= hi) || (A < 0.f && r >= lo);
  float g = flows ? -A * r : 0.f;
  if (r != r) { l = r; g = r; }      // fminf / fmaxf drop a NaN operand: a NaN ratio must reach the loss
  if (A >= 0.f && r > hi) atomicAdd(&a.counters[1], 1ull);
  if (A < 0.f && r < lo) atomicAdd(&a.counters[2], 1ull);
  a.coefc[i] = c * g / ctl.norm * a.inv_tau;
  a.lossterm[i] = c * l;
}
void launch_combine(const CombineArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(combine_kernel, dim3(a.t_cap / 64), dim3(256), 0, s, a);
}

// Single workgroup, fixed order, fp64: loss = (sum_t c_t l_t) / norm; publishes the counters.
__global__ __launch_bounds__(1024) void finish_kernel(FinishArgs a) {
  __shared__ double sh[1024];
  const Ctl ctl = *a.ctl;
  const int tid = threadIdx.x;
  double acc = 0.0;
  for (int i = tid; i < ctl.n_active; i += 1024) acc += (double)a.lossterm[i];
  sh[tid] = acc;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if (tid < w) sh[tid] += sh[tid + w];
    __syncthreads();
  }
  if (tid == 0 && a.loss_out) *a.loss_out = (float)(sh[0] / (double)ctl.norm);
  if (tid < 8 && a.counters_out) a.counters_out[tid] = (long long)a.counters[tid];
}
void launch_finish(const FinishArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(1024), 0, s, a);
}

// ------------------------------------------------------------------ dH scatter
// dH[t,:] = accumulated row of its compacted position, or zeros for rows that are not active.
__global__ __launch_bounds__(256) void scatter_dh_kernel(ScatterArgs a) {
  const int t = blockIdx.x;
  const int p = a.pos[t];
  const float* src = a.acc + (size_t)(p < 0 ? 0 : p) * a.d;
  const int n_pad = a.ctl->n_pad;
  const int ks = a.split_k ? dh_split(n_pad, a.t_cap, a.tiles_n, a.k_stages) : 1;
  const size_t slab = (size_t)n_pad * a.d;
  for (int j = threadIdx.x * 4; j < a.d; j += 256 * 4) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (p >= 0) {
      v = *reinterpret_cast<const float4*>(src + j);
      for (int q = 1; q < ks; ++q) {               // split-K slabs, added in a fixed order
        const float4 w = *reinterpret_cast<const float4*>(src + q * slab + j);
        v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
      }
    }
    if (a.out_f32) {
      *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.dH) + (size_t)t * a.d + j) = v;
    } else {
      bf16x4 o;
      o[0] = (__bf16)v.x; o[1] = (__bf16)v.y; o[2] = (__bf16)v.z; o[3] = (__bf16)v.w;
      *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(a.dH) + (size_t)t * a.d + j) = o;
    }
  }
}
// ------------------------------------------------------------------ vocab-sharded head
// The reduction operator of the exchange between vocab shards: per row, the softmax states
// (m, s, u) of two disjoint vocab ranges merge by the online-softmax rule and the sampled
// token's logit (held by one shard, 0 elsewhere) by addition.  Rows nobody computed are all
// zeros and stay so.  out may alias a or b.
__global__ void merge_partials_kernel(const float* a, const float* b, float* out, long long T) {
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  const float4 p = *reinterpret_cast<const float4*>(a + t * 4), q = *reinterpret_cast<const float4*>(b + t * 4);
  float4 r;
  if (p.y == 0.f) {          // empty state on one side: the other side unchanged
    r = make_float4(q.x, q.y, q.z, p.w + q.w);
  } else if (q.y == 0.f) {
    r = make_float4(p.x, p.y, p.z, p.w + q.w);
  } else {
    const float mm = fmaxf(p.x, q.x);
    const float a1 = expf(p.x - mm), a2 = expf(q.x - mm);
    r.x = mm;
    r.y = a1 * p.y + a2 * q.y;
    r.z = a1 * (p.z + (p.x - mm) * p.y) + a2 * (q.z + (q.x - mm) * q.y);
    r.w = p.w + q.w;
  }
  *reinterpret_cast<float4*>(out + t * 4) = r;
}
void launch_merge_partials(const float* a, const float* b, float* out, long long T, hipStream_t s) {
  if (T <= 0) return;
  hipLaunchKernelGGL(merge_partials_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, s, a, b, out, T);
}

__global__ void finish_partials_kernel(const float* parts, long long T, float* logp, float* ent, float* lse) {
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  const float4 p = *reinterpret_cast<const float4*>(parts + t * 4);
  float lp = 0.f, en = 0.f, ls = 0.f;
  if (p.y != 0.f) {
    const float lns = logf(p.y);
    ls = p.x + lns;
    lp = p.w - ls;
    en = lns - p.z / p.y;
  }
  if (logp) logp[t] = lp;
  if (ent) ent[t] = en;
  if (lse) lse[t] = ls;
}
void launch_finish_partials(const float* parts, long long T, float* logp, float* ent, float* lse, hipStream_t s) {
  if (T <= 0) return;
  hipLaunchKernelGGL(finish_partials_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, s, parts, T, logp, ent, lse);
}

void launch_scatter_dh(const ScatterArgs& a, hipStream_t s) {
  if (a.T <= 0) return;
  hipLaunchKernelGGL(scatter_dh_kernel, dim3(a.T), dim3(256), 0, s, a);
}

// ------------------------------------------------------------------ rewards (Eq. 1, Eq. 6-7)
__global__ void turn_reward_kernel(RewardArgs a) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= a.n) return;
  double R = 0.0, pr = 0.0;
  if (a.correct[i]) {
    const double speedup = fmin((double)a.t_reference[i] / (double)a.t_kernel[i], (double)a.cap);
    R = 1.0 + speedup;
    if (a.t_generated) {
      pr = (double)a.t_generated[i] / (double)a.t_total[i];
      R += pr;
    }
  }
  a.rewards_out[i] = (float)R;
  if (a.pr_out) a.pr_out[i] = (float)pr;
}
void launch_turn_reward(const RewardArgs& a, hipStream_t s) {
  if (a.n <= 0) return;
  hipLaunchKernelGGL(turn_reward_kernel, dim3((unsigned)((a.n + 255) / 256)), dim3(256), 0, s, a);
}

// ------------------------------------------------------------------ PRS (Sec. 5.2, Eq. 8)
// Philox-4x32 with 10 rounds (Salmon et al., SC'11), one block per sample; only the first
// output word is used.
__device__ __forceinline__ uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                       uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c0;
}

__global__ void prs_retain_kernel(PrsArgs a) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= a.n) return;
  const double pr = (double)a.pr[i];
  double p = (pr - (double)a.tau) / (double)a.s;
  p = fmin(fmax(p, 0.0), 1.0);
  bool keep = false;
  if (!a.valid || a.valid[i]) {
    if (a.hard) {
      keep = pr >= (double)a.tau;
    } else {
      const uint32_t x = philox4x32_10_word0((uint32_t)i, (uint32_t)((unsigned long long)i >> 32), 0u, 0u,
                                             (uint32_t)a.seed, (uint32_t)(a.seed >> 32));
      const double u = ((double)x + 0.5) * (1.0 / 4294967296.0);
      keep = u < p;
    }
  }
  a.keep_out[i] = keep ? 1 : 0;
  if (a.p_out) a.p_out[i] = (float)p;
}
void launch_prs_retain(const PrsArgs& a, hipStream_t s) {
  if (a.n <= 0) return;
  hipLaunchKernelGGL(prs_retain_kernel, dim3((unsigned)((a.n + 255) / 256)), dim3(256), 0, s, a);
}

// ------------------------------------------------------------------ monitors (Sec. 5.1)
// Stage 1: MON_BLOCKS workgroups; workgroup b sums a fixed, contiguous slice of every input in
// fp64 (tree reduction in a fixed order).  Stage 2: one workgroup folds the partials, again in a
// fixed order, and writes the six monitors.
__device__ __forceinline__ double block_sum_256(double v, double* sh) {
  const int tid = threadIdx.x;
  sh[tid] = v;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (tid < w) sh[tid] += sh[tid + w];
    __syncthreads();
  }
  const double r = sh[0];
  __syncthreads();
  return r;
}

__device__ __forceinline__ double sumsq_slice(const void* p, int is_f32, long long n, int b, int tid) {
  // slice b of MON_BLOCKS, in units of 8 elements so that loads stay 16-byte aligned
  const long long units = (n + 7) / 8, per = (units + MON_BLOCKS - 1) / MON_BLOCKS;
  const long long u0 = (long long)b * per, u1 = u0 + per < units ? u0 + per : units;
  double acc = 0.0;
  for (long long u = u0 + tid; u < u1; u += 256) {
    const long long e0 = u * 8;
    if (e0 + 8 <= n) {
      if (is_f32) {
        const float4 x = reinterpret_cast<const float4*>(p)[u * 2], y = reinterpret_cast<const float4*>(p)[u * 2 + 1];
        acc += (double)x.x * x.x + (double)x.y * x.y + (double)x.z * x.z + (double)x.w * x.w +
               (double)y.x * y.x + (double)y.y * y.y + (double)y.z * y.z + (double)y.w * y.w;
      } else {
        const bf16x8 x = reinterpret_cast<const bf16x8*>(p)[u];
#pragma unroll
        for (int e = 0; e < 8; ++e) { const double v = (double)(float)x[e]; acc += v * v; }
      }
    } else {
      for (long long e = e0; e < n; ++e) {
        const double v = is_f32 ? (double)reinterpret_cast<const float*>(p)[e]
                                : (double)(float)reinterpret_cast<const __bf16*>(p)[e];
        acc += v * v;
      }
    }
  }
  return acc;
}

__global__ __launch_bounds__(256) void monitors_partial_kernel(MonitorArgs a) {
  __shared__ double sh[256];
  const int b = blockIdx.x, tid = threadIdx.x;
  const long long per = (a.T + MON_BLOCKS - 1) / MON_BLOCKS;
  const long long t0 = (long long)b * per, t1 = t0 + per < a.T ? t0 + per : a.T;
  double s_ent = 0.0, s_tr = 0.0, s_ro = 0.0, s_n = 0.0;
  for (long long t = t0 + tid; t < t1; t += 256) {
    if (a.mask[t]) {
      s_n += 1.0;
      s_tr += (double)a.logp_train[t];
      if (a.logp_rollout) s_ro += (double)a.logp_rollout[t];
      if (a.entropy) s_ent += (double)a.entropy[t];
    }
  }
  const double r0 = block_sum_256(s_ent, sh), r1 = block_sum_256(s_tr, sh), r2 = block_sum_256(s_ro, sh),
               r5 = block_sum_256(s_n, sh);
  const double r3 = a.dH ? block_sum_256(sumsq_slice(a.dH, a.dH_f32, a.dH_elems, b, tid), sh) : 0.0;
  const double r4 = a.dW ? block_sum_256(sumsq_slice(a.dW, a.dW_f32, a.dW_elems, b, tid), sh) : 0.0;
  if (tid == 0) {
    a.partial[0 * MON_BLOCKS + b] = r0; a.partial[1 * MON_BLOCKS + b] = r1; a.partial[2 * MON_BLOCKS + b] = r2;
    a.partial[3 * MON_BLOCKS + b] = r3; a.partial[4 * MON_BLOCKS + b] = r4; a.partial[5 * MON_BLOCKS + b] = r5;
  }
}

__global__ __launch_bounds__(256) void monitors_final_kernel(MonitorArgs a) {
  __shared__ double sh[256];
  __shared__ double tot[6];
  const int tid = threadIdx.x;
  for (int q = 0; q < 6; ++q) {
    double v = 0.0;
    for (int b = tid; b < MON_BLOCKS; b += 256) v += a.partial[q * MON_BLOCKS + b];
    const double r = block_sum_256(v, sh);
    if (tid == 0) tot[q] = r;
  }
  __syncthreads();
  if (tid == 0) {
    const double n = tot[5], den = n > 0.0 ? n : 1.0;
    a.out[0] = a.entropy ? tot[0] / den : 0.0;
    a.out[1] = exp(-tot[1] / den);
    a.out[2] = a.logp_rollout ? exp(-tot[2] / den) : 0.0;
    a.out[3] = sqrt(tot[3]);
    a.out[4] = sqrt(tot[4]);
    a.out[5] = n;
    a.out[6] = 0.0;
    a.out[7] = 0.0;
  }
}
void launch_monitors(const MonitorArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(monitors_partial_kernel, dim3(MON_BLOCKS), dim3(256), 0, s, a);
  hipLaunchKernelGGL(monitors_final_kernel, dim3(1), dim3(256), 0, s, a);
}

// ------------------------------------------------------------------ RMSNorm in front of the head
// h = x * rstd * gamma, rstd = 1 / sqrt(mean x^2 + eps).  One wavefront per row, 16-byte (bf16) or
// 32-byte (fp32) accesses of 8 consecutive elements per lane and step; fp32 arithmetic, the sum of
// squares reduced in a fixed butterfly order.  Both kernels hold the current row in registers and
// read every element once; they are HBM-bound.
template <bool F32>
__device__ __forceinline__ void load8(const void* p, long long elem, float (&v)[8]) {
  if (F32) {
    const float4 a = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p) + elem);
    const float4 b = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p) + elem + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  } else {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const __bf16*>(p) + elem);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (float)a[e];
  }
}
template <bool F32>
__device__ __forceinline__ void store8(void* p, long long elem, const float (&v)[8]) {
  if (F32) {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(p) + elem) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(p) + elem + 4) = make_float4(v[4], v[5], v[6], v[7]);
  } else {
    bf16x8 a;
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = (__bf16)v[e];
    *reinterpret_cast<bf16x8*>(reinterpret_cast<__bf16*>(p) + elem) = a;
  }
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int sh = 32; sh >= 1; sh >>= 1) v += __shfl_xor(v, sh);
  return v;
}
// Forward: a lane keeps its (up to) NORM_FC x 8 elements of the row in registers between the sum
// of squares and the scaling, so every element of X is read from memory once.  All loads of the
// row are issued before the first use, so they are in flight together.
constexpr int NORM_FC = NORM_MAX_D / 512;          // 8-column steps per lane

template <bool F32> struct Raw8;
template <> struct Raw8<true> { float4 a, b; };
template <> struct Raw8<false> { bf16x8 v; };
__device__ __forceinline__ void raw_load(const void* p, long long elem, Raw8<true>& r) {
  r.a = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p) + elem);
  r.b = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p) + elem + 4);
}
__device__ __forceinline__ void raw_load(const void* p, long long elem, Raw8<false>& r) {
  r.v = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const __bf16*>(p) + elem);
}
__device__ __forceinline__ void raw_unpack(const Raw8<true>& r, float (&v)[8]) {
  v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w; v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
}
__device__ __forceinline__ void raw_unpack(const Raw8<false>& r, float (&v)[8]) {
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (float)r.v[e];
}

template <bool F32>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(NormArgs a) {
  const int lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= a.T) return;
  Raw8<F32> raw[NORM_FC];
#pragma unroll
  for (int q = 0; q < NORM_FC; ++q) {
    const int c = lane * 8 + q * 512;
    if (c < a.d) raw_load(a.X, row * a.d + c, raw[q]);
  }
  float ss = 0.f;
#pragma unroll
  for (int q = 0; q < NORM_FC; ++q) {
    const int c = lane * 8 + q * 512;
    if (c < a.d) {
      float x[8];
      raw_unpack(raw[q], x);
#pragma unroll
      for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
    }
  }
  ss = wave_sum(ss);
  const float rstd = 1.f / sqrtf(ss / (float)a.d + a.eps);
  if (a.rstd_out && lane == 0) a.rstd_out[row] = rstd;
#pragma unroll
  for (int q = 0; q < NORM_FC; ++q) {
    const int c = lane * 8 + q * 512;
    if (c < a.d) {
      float x[8], g[8], h[8];
      raw_unpack(raw[q], x);
      load8<F32>(a.gamma, c, g);
#pragma unroll
      for (int e = 0; e < 8; ++e) h[e] = x[e] * rstd * g[e];
      store8<F32>(a.H, row * a.d + c, h);
    }
  }
}
void launch_rmsnorm_fwd(const NormArgs& a, hipStream_t s) {
  if (a.T <= 0) return;
  const unsigned grid = (unsigned)((a.T + 3) / 4);
  if (a.is_f32) hipLaunchKernelGGL(rmsnorm_fwd_kernel<true>, dim3(grid), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(rmsnorm_fwd_kernel<false>, dim3(grid), dim3(256), 0, s, a);
}

// Backward: dx = rstd (gamma g - xhat mean(gamma g xhat)), xhat = x rstd; dgamma = sum_rows g xhat.
// Workgroup b takes the rows b, b + NORM_STRIPS, b + 2 NORM_STRIPS, ... (so the workgroups running at
// one time read and write neighbouring rows: 4 % faster than a contiguous strip per workgroup); a thread
// owns the same (up to) 4 x 8 columns of every row, holds x and g of the current row in registers
// (each element is read once) and keeps the dgamma partial sums of its columns in registers.  The
// two row sums (x^2 and gamma g x) are reduced over the workgroup together, in a fixed order.  The
// workgroups' partials are folded by the second kernel.
constexpr int NORM_NC = NORM_MAX_D / 2048;         // 8-column steps per thread at the largest d
static_assert(NORM_NC == 4, "the launcher instantiates 1..4 steps");

__device__ __forceinline__ float block_sum4(float v, float* red, int lane, int wave) {
  v = wave_sum(v);
  if (lane == 0) red[wave] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// Keeps the register values of a packed row opaque to the optimiser between the two passes over a row, so that
// the unpacked fp32 copies of the first pass are not kept alive across the reduction (they are unpacked again).
__device__ __forceinline__ void opaque(Raw8<true>& r) { asm volatile("" : "+v"(r.a.x), "+v"(r.a.y), "+v"(r.a.z), "+v"(r.a.w), "+v"(r.b.x), "+v"(r.b.y), "+v"(r.b.z), "+v"(r.b.w)); }
__device__ __forceinline__ void opaque(Raw8<false>& r) {
  i32x4 v = __builtin_bit_cast(i32x4, r.v);
  asm volatile("" : "+v"(v));
  r.v = __builtin_bit_cast(bf16x8, v);
}

// NC: 8-column steps per thread, ceil(d / 2048).  Rows stay in registers as loaded (bf16 rows packed) and are
// unpacked on the fly in both passes: with three steps and bf16 rows the kernel fits 4 workgroups on a
// compute unit, each with one row of X and dH in flight ahead of the one it works on.
template <bool F32, int NC>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(NormArgs a) {
  __shared__ float red[2][8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long long r0 = blockIdx.x, r1 = a.T;      // rows r0, r0 + NORM_STRIPS, ...
  float dg[NC][8];
  Raw8<F32> g_raw[NC] = {};
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    const int c = tid * 8 + q * 2048;
#pragma unroll
    for (int e = 0; e < 8; ++e) dg[q][e] = 0.f;
    if (c < a.d) raw_load(a.gamma, c, g_raw[q]);
  }
  const float inv_d = 1.f / (float)a.d;
  // The next row's loads are issued before the current row's workgroup reduction, so a
  // workgroup always has one row of X and dH in flight while it works on the previous one.
  Raw8<F32> xr[NC] = {}, gr_raw[NC] = {}, xn[NC] = {}, gn[NC] = {};
  auto fetch = [&](long long row, Raw8<F32> (&xa)[NC], Raw8<F32> (&ga)[NC]) {
#pragma unroll
    for (int q = 0; q < NC; ++q) {
      const int c = tid * 8 + q * 2048;
      if (c < a.d) {
        raw_load(a.X, row * a.d + c, xa[q]);
        raw_load(a.dH, row * a.d + c, ga[q]);
      }
    }
  };
  if (r0 < r1) fetch(r0, xr, gr_raw);
  int parity = 0;
  for (long long row = r0; row < r1; row += NORM_STRIPS, parity ^= 1) {
    if (row + NORM_STRIPS < r1) fetch(row + NORM_STRIPS, xn, gn);
    // sum x^2 and sum gamma g x in one workgroup reduction: mean_j(gamma_j g_j xhat_j) = rstd mean_j(gamma_j g_j x_j)
    float ss = 0.f, sd = 0.f;
#pragma unroll
    for (int q = 0; q < NC; ++q) {
      const int c = tid * 8 + q * 2048;
      if (c < a.d) {
        float x[8], gr[8], g[8];
        raw_unpack(xr[q], x);
        raw_unpack(gr_raw[q], gr);
        raw_unpack(g_raw[q], g);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          ss = fmaf(x[e], x[e], ss);
          sd = fmaf(g[e] * gr[e], x[e], sd);
        }
      }
    }
    ss = wave_sum(ss);
    sd = wave_sum(sd);
    float* rb = red[parity];                // alternating buffers: one barrier per row is enough
    if (lane == 0) { rb[wave] = ss; rb[4 + wave] = sd; }
    __syncthreads();
    const float rstd = 1.f / sqrtf(((rb[0] + rb[1]) + (rb[2] + rb[3])) * inv_d + a.eps);
    const float dot = ((rb[4] + rb[5]) + (rb[6] + rb[7])) * rstd * inv_d;
#pragma unroll
    for (int q = 0; q < NC; ++q) {
      const int c = tid * 8 + q * 2048;
      if (c < a.d) {
        opaque(xr[q]);
        opaque(gr_raw[q]);
        float x[8], gr[8], g[8], dx[8];
        raw_unpack(xr[q], x);
        raw_unpack(gr_raw[q], gr);
        raw_unpack(g_raw[q], g);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = x[e] * rstd;
          dx[e] = rstd * (g[e] * gr[e] - xh * dot);
          dg[q][e] = fmaf(gr[e], xh, dg[q][e]);
        }
        store8<F32>(a.dX, row * a.d + c, dx);
      }
    }
#pragma unroll
    for (int q = 0; q < NC; ++q) { xr[q] = xn[q]; gr_raw[q] = gn[q]; }
  }
  float* part = a.partial + (size_t)blockIdx.x * a.d;
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    const int c = tid * 8 + q * 2048;
    if (c < a.d) {
      *reinterpret_cast<float4*>(part + c) = make_float4(dg[q][0], dg[q][1], dg[q][2], dg[q][3]);
      *reinterpret_cast<float4*>(part + c + 4) = make_float4(dg[q][4], dg[q][5], dg[q][6], dg[q][7]);
    }
  }
}

// dgamma[c] = sum over the strips' partials, in a fixed order: workgroup = 32 columns x 8 strip
// groups; group k adds strips k, k+8, ... in four interleaved chains, then the groups are folded.
__global__ __launch_bounds__(256) void rmsnorm_dgamma_kernel(NormArgs a) {
  __shared__ float sh[8][32];
  const int col = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + col;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (c < a.d) {
    for (int b = grp; b < NORM_STRIPS; b += 32)
#pragma unroll
      for (int k = 0; k < 4; ++k) acc[k] += a.partial[(size_t)(b + 8 * k) * a.d + c];
  }
  sh[grp][col] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
  __syncthreads();
  if (grp == 0 && c < a.d) {
    float v = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) v += sh[k][col];
    a.dgamma[c] = v;
  }
}
static_assert(NORM_STRIPS % 32 == 0, "strip groups");

template <bool F32>
static void launch_rmsnorm_bwd_rows(const NormArgs& a, hipStream_t s) {
  switch ((a.d + 2047) / 2048) {     // 8-column steps per thread; d <= NORM_MAX_D is checked by the caller
    case 1: hipLaunchKernelGGL((rmsnorm_bwd_kernel<F32, 1>), dim3(NORM_STRIPS), dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL((rmsnorm_bwd_kernel<F32, 2>), dim3(NORM_STRIPS), dim3(256), 0, s, a); break;
    case 3: hipLaunchKernelGGL((rmsnorm_bwd_kernel<F32, 3>), dim3(NORM_STRIPS), dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL((rmsnorm_bwd_kernel<F32, NORM_NC>), dim3(NORM_STRIPS), dim3(256), 0, s, a); break;
  }
}
void launch_rmsnorm_bwd(const NormArgs& a, hipStream_t s) {
  if (a.is_f32) launch_rmsnorm_bwd_rows<true>(a, s);
  else launch_rmsnorm_bwd_rows<false>(a, s);
  hipLaunchKernelGGL(rmsnorm_dgamma_kernel, dim3((a.d + 31) / 32), dim3(256), 0, s, a);
}


// ------------------------------------------------------------------ RMSNorm fused around the head
// Forward, fused into the row compaction: one wavefront per compacted row reads the row of X once,
// keeps it in registers between the sum of squares and the scaling (as rmsnorm_fwd_kernel), rounds
// h = x rstd gamma to bf16 (fp32 inputs: splits it into bf16 hi + lo parts, [hi | hi | lo] along k) and
// writes it as the head's compacted operand row; rows that are not active are never read.
template <bool F32>
__global__ __launch_bounds__(256) void norm_gather_kernel(GatherArgs a, NormFuse n) {
  const Ctl ctl = *a.ctl;
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= ctl.n_pad) return;
  const bool live = i < ctl.n_active;
  const int t = live ? a.rows[i] : 0;
  if (lane == 0) {
    int yl = -1;
    if (live) {
      yl = a.y[t] - a.y_offset;
      if (yl < 0 || yl >= a.V) yl = -1;
    }
    a.yc[i] = yl;
  }
  Raw8<F32> raw[NORM_FC];
  if (live) {
#pragma unroll
    for (int q = 0; q < NORM_FC; ++q) {
      const int c = lane * 8 + q * 512;
      if (c < a.d) raw_load(n.X, (long long)t * a.d + c, raw[q]);
    }
  }
  float ss = 0.f;
  if (live) {
#pragma unroll
    for (int q = 0; q < NORM_FC; ++q) {
      const int c = lane * 8 + q * 512;
      if (c < a.d) {
        float x[8];
        raw_unpack(raw[q], x);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
      }
    }
  }
  ss = wave_sum(ss);
  const float rstd = live ? 1.f / sqrtf(ss / (float)a.d + n.eps) : 0.f;
  if (lane == 0) n.rstd_c[i] = rstd;
  const int ldh = F32 ? 3 * a.d : a.d;
#pragma unroll
  for (int q = 0; q < NORM_FC; ++q) {
    const int c = lane * 8 + q * 512;
    if (c < a.d) {
      float h[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      if (live) {
        float x[8], g[8];
        raw_unpack(raw[q], x);
        load8<F32>(n.gamma, c, g);
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = x[e] * rstd * g[e];
      }
      __bf16* o = a.Hc + (size_t)i * ldh + c;
      if (F32) {
        bf16x8 hi, lo;
#pragma unroll
        for (int e = 0; e < 8; ++e) { __bf16 x, y; split_bf16(h[e], x, y); hi[e] = x; lo[e] = y; }
        *reinterpret_cast<bf16x8*>(o) = hi;
        *reinterpret_cast<bf16x8*>(o + a.d) = hi;
        *reinterpret_cast<bf16x8*>(o + 2 * a.d) = lo;
      } else {
        bf16x8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (__bf16)h[e];
        *reinterpret_cast<bf16x8*>(o) = v;
      }
    }
  }
}

// HcT[j, i] = Hc[i, j] for d columns of row stride ldh (the bf16 operand; the hi or the lo parts of a split fp32 one).
__global__ __launch_bounds__(256) void transpose_hc_kernel(const __bf16* Hc, int ldh, __bf16* HcT, int ld_t, const Ctl* ctlp) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[64 * TT_LD];
  const int i0 = blockIdx.x * 64, j0 = blockIdx.y * 64;
  if (i0 >= ctlp->n_pad) return;
  const int tid = threadIdx.x, chunk = tid & 7;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int r = (tid >> 3) + 32 * p;
    tt_put(tile, r, chunk, *reinterpret_cast<const i32x4*>(Hc + (size_t)(i0 + r) * ldh + j0 + chunk * 8));
  }
  __syncthreads();
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int jj = (tid >> 3) + 32 * p;
    *reinterpret_cast<i32x4*>(HcT + (size_t)(j0 + jj) * ld_t + i0 + chunk * 8) = tt_get(tile, jj, chunk);
  }
}

void launch_transpose_hc(const __bf16* Hc, int ldh, __bf16* HcT, const GatherArgs& g, hipStream_t s) {
  hipLaunchKernelGGL(transpose_hc_kernel, dim3(g.t_cap / 64, g.d / 64), dim3(256), 0, s, Hc, ldh, HcT, g.ld_t, g.ctl);
}

void launch_norm_gather(const GatherArgs& g, const NormFuse& n, hipStream_t s) {
  if (g.is_f32) hipLaunchKernelGGL(norm_gather_kernel<true>, dim3(g.t_cap / 4), dim3(256), 0, s, g, n);
  else hipLaunchKernelGGL(norm_gather_kernel<false>, dim3(g.t_cap / 4), dim3(256), 0, s, g, n);
  if (g.HcT) launch_transpose_hc(g.Hc, g.is_f32 ? 3 * g.d : g.d, g.HcT, g, s);
  if (g.HcT_lo) launch_transpose_hc(g.Hc + 2 * g.d, 3 * g.d, g.HcT_lo, g, s);
}

// Backward, fused into the scatter of dH: workgroup b takes the T-rows b, b + NORM_STRIPS, ... (as
// rmsnorm_bwd_kernel) and a thread the same (up to) 4 x 8 columns of every row.  For an active row
// the accumulated fp32 gradient g of its compacted position (split-K slabs added in order) and the
// row of X are read once, rstd comes from the forward,
//   dx = rstd (gamma g - xhat mean_j(gamma_j g_j xhat_j)),  xhat = x rstd,
// and g xhat is added to the thread's dgamma partial sums; rows that are not active are written as
// zeros and nothing of theirs is read.  The workgroups' partials are folded by rmsnorm_dgamma_kernel.
template <bool F32, int NC>
__global__ __launch_bounds__(256) void scatter_dx_norm_kernel(ScatterArgs a, NormFuse n) {
  __shared__ float red[2][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long long T = a.T;
  const int n_pad = a.ctl->n_pad;
  const int ks = a.split_k ? dh_split(n_pad, a.t_cap, a.tiles_n, a.k_stages) : 1;
  const size_t slab = (size_t)n_pad * a.d;
  float dg[NC][8];
  Raw8<F32> gam_raw[NC] = {};
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    const int c = tid * 8 + q * 2048;
#pragma unroll
    for (int e = 0; e < 8; ++e) dg[q][e] = 0.f;
    if (c < a.d) raw_load(n.gamma, c, gam_raw[q]);
  }
  const float inv_d = 1.f / (float)a.d;
  // Row r of the workgroup is T-row blockIdx.x + r NORM_STRIPS; the inputs of the next one (its compacted
  // position, rstd, the row of X and the first slab of the accumulator) are requested before the current
  // row's reduction.  An inactive row (position < 0) needs no input.
  Raw8<F32> xc[NC] = {}, xn[NC] = {};
  Raw8<true> gc[NC] = {}, gn[NC] = {};
  auto fetch = [&](long long row, Raw8<F32> (&xa)[NC], Raw8<true> (&ga)[NC], int& p, float& rstd) {
    p = a.pos[row];                                 // uniform over the workgroup
    if (p < 0) return;
    rstd = n.rstd_c[p];
#pragma unroll
    for (int q = 0; q < NC; ++q) {
      const int c = tid * 8 + q * 2048;
      if (c < a.d) {
        raw_load(n.X, row * a.d + c, xa[q]);
        raw_load(a.acc, (long long)p * a.d + c, ga[q]);
      }
    }
  };
  int pc = -1, parity = 0;
  float rc = 0.f;
  long long row = blockIdx.x;
  if (row < T) fetch(row, xc, gc, pc, rc);
  for (; row < T; row += NORM_STRIPS) {
    int pn = -1;
    float rn = 0.f;
    if (row + NORM_STRIPS < T) fetch(row + NORM_STRIPS, xn, gn, pn, rn);
    if (pc < 0) {
#pragma unroll
      for (int q = 0; q < NC; ++q) {
        const int c = tid * 8 + q * 2048;
        const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (c < a.d) store8<F32>(a.dH, row * a.d + c, z);
      }
    } else {
      const float rstd = rc;
      float dot = 0.f;
#pragma unroll
      for (int q = 0; q < NC; ++q) {
        const int c = tid * 8 + q * 2048;
        if (c < a.d) {
          float x[8], g[8], gam[8];
          raw_unpack(xc[q], x);
          raw_unpack(gc[q], g);
          raw_unpack(gam_raw[q], gam);
          if (ks > 1) {
            for (int s2 = 1; s2 < ks; ++s2) {       // split-K slabs, added in a fixed order
              float w[8];
              load8<true>(a.acc, (long long)(s2 * slab) + (long long)pc * a.d + c, w);
#pragma unroll
              for (int e = 0; e < 8; ++e) g[e] += w[e];
            }
            gc[q].a = make_float4(g[0], g[1], g[2], g[3]);
            gc[q].b = make_float4(g[4], g[5], g[6], g[7]);
          }
#pragma unroll
          for (int e = 0; e < 8; ++e) dot = fmaf(gam[e] * g[e], x[e] * rstd, dot);
        }
      }
      dot = wave_sum(dot);
      float* rb = red[parity];                      // alternating buffers: one barrier per row is enough
      parity ^= 1;
      if (lane == 0) rb[wave] = dot;
      __syncthreads();
      dot = ((rb[0] + rb[1]) + (rb[2] + rb[3])) * inv_d;
#pragma unroll
      for (int q = 0; q < NC; ++q) {
        const int c = tid * 8 + q * 2048;
        if (c < a.d) {
          opaque(xc[q]);
          float x[8], g[8], gam[8], dx[8];
          raw_unpack(xc[q], x);
          raw_unpack(gc[q], g);
          raw_unpack(gam_raw[q], gam);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float xh = x[e] * rstd;
            dx[e] = rstd * (gam[e] * g[e] - xh * dot);
            dg[q][e] = fmaf(g[e], xh, dg[q][e]);
          }
          store8<F32>(a.dH, row * a.d + c, dx);
        }
      }
    }
#pragma unroll
    for (int q = 0; q < NC; ++q) { xc[q] = xn[q]; gc[q] = gn[q]; }
    pc = pn; rc = rn;
  }
  float* part = n.partial + (size_t)blockIdx.x * a.d;
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    const int c = tid * 8 + q * 2048;
    if (c < a.d) {
      *reinterpret_cast<float4*>(part + c) = make_float4(dg[q][0], dg[q][1], dg[q][2], dg[q][3]);
      *reinterpret_cast<float4*>(part + c + 4) = make_float4(dg[q][4], dg[q][5], dg[q][6], dg[q][7]);
    }
  }
}

template <bool F32>
static void launch_scatter_dx_norm_rows(const ScatterArgs& a, const NormFuse& n, hipStream_t s) {
  switch ((a.d + 2047) / 2048) {     // 8-column steps per thread; d <= NORM_MAX_D is checked by the caller
    case 1: hipLaunchKernelGGL((scatter_dx_norm_kernel<F32, 1>), dim3(NORM_STRIPS), dim3(256), 0, s, a, n); break;
    case 2: hipLaunchKernelGGL((scatter_dx_norm_kernel<F32, 2>), dim3(NORM_STRIPS), dim3(256), 0, s, a, n); break;
    case 3: hipLaunchKernelGGL((scatter_dx_norm_kernel<F32, 3>), dim3(NORM_STRIPS), dim3(256), 0, s, a, n); break;
    default: hipLaunchKernelGGL((scatter_dx_norm_kernel<F32, NORM_NC>), dim3(NORM_STRIPS), dim3(256), 0, s, a, n); break;
  }
}
void launch_scatter_dx_norm(const ScatterArgs& a, const NormFuse& n, hipStream_t s) {
  if (a.out_f32) launch_scatter_dx_norm_rows<true>(a, n, s);
  else launch_scatter_dx_norm_rows<false>(a, n, s);
  NormArgs f{};
  f.d = a.d; f.partial = n.partial; f.dgamma = n.dgamma;
  hipLaunchKernelGGL(rmsnorm_dgamma_kernel, dim3((a.d + 31) / 32), dim3(256), 0, s, f);
}

}  // namespace pg
