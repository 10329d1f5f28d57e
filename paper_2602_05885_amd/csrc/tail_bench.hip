// Stand-alone timeline of one vocab chunk's three persistent launches at the 14B head shape (d=5120,
// 32 768 tokens, a chunk of 89 vocab tiles): the recompute (logits tile -> dS in both orientations), the dW
// contraction and the dH contraction, each as the library launches it (one workgroup per compute unit,
// tiles from the per-XCD queue), with the 100 MHz wall clock read inside the kernel
//   * per workgroup at its start, at the start of its last tile and at its end: how long the workgroups
//     idle at the end of a launch, per XCD, and how long the last tile was;
//   * for the recompute, per tile at the end of the main loop and at the end of the epilogue, for the first
//     TL_TILES tiles of every workgroup: whether the epilogue (two 128 KB store bursts per tile) is slower
//     while all workgroups still run in step (first tiles of a launch) than after they have drifted apart.
// The kernels are the library's own tile bodies and queue (kernels_gemm.hip is included), wrapped with the
// clock reads.  Usage: tail_bench [repetitions]   (default 2)
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "kernels_gemm.hip"
using namespace pg;

#define CK(x)                                                                 \
  do {                                                                        \
    hipError_t e_ = (x);                                                      \
    if (e_ != hipSuccess) {                                                   \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
      exit(1);                                                                \
    }                                                                         \
  } while (0)

constexpr int TL_TILES = 40;   // tiles of every workgroup whose epilogue is timed (a workgroup does about 44)

namespace pg {

__device__ __forceinline__ unsigned long long wall() { return __builtin_amdgcn_s_memrealtime(); }

// per workgroup: start, end, start of the last tile, (XCD << 32) | tiles done
__device__ __forceinline__ void put_summary(unsigned long long* pr, unsigned long long t0, unsigned long long tlast, int xcd, int n) {
  if (threadIdx.x == 0) {
    pr[blockIdx.x * 4] = t0; pr[blockIdx.x * 4 + 1] = wall(); pr[blockIdx.x * 4 + 2] = tlast;
    pr[blockIdx.x * 4 + 3] = ((unsigned long long)xcd << 32) | (unsigned)n;
  }
}

__global__ __launch_bounds__(NTHREADS) void store_timeline_kernel(StoreArgs a, unsigned long long* pr) {
  const unsigned long long t0 = wall();
  const Ctl ctl = *a.ctl;
  StoreShape sh;
  sh.init(a, ctl);
  TileQueue Q;
  Q.init(a.queue, sh.total, 1);
  volatile int* claim = reinterpret_cast<volatile int*>(g_smem + CLAIM_OFF);
  int n = 0;
  unsigned long long tlast = t0;
  drain_queue(Q, true, claim, [&](int b, auto&& after_loop, auto&& before_stores) {
    ++n; tlast = wall();
    gemm_store_tile(a, sh, ctl.n_pad, b, after_loop, before_stores);
  });
  put_summary(pr, t0, tlast, Q.home, n);
}

__global__ __launch_bounds__(NTHREADS) void dlogits_timeline_kernel(DlogitsArgs a, unsigned long long* pr, unsigned long long* tl) {
  const unsigned long long t0 = wall();
  const Ctl ctl = *a.ctl;
  const int tiles_t = min(a.tiles_t, ctl.n_pad / BN);
  TileQueue Q;
  Q.init(a.queue, a.tiles_v * tiles_t, 0);
  volatile int* claim = reinterpret_cast<volatile int*>(g_smem + CLAIM_OFF);
  int n = 0;
  unsigned long long tlast = t0;
  drain_queue(Q, true, claim, [&](int b, auto&& after_loop, auto&& before_stores) {
    const int k = n;
    int tm, tn;
    ++n; tlast = wall();
    map_tile(b, a.tiles_v, tiles_t, tm, tn);
    unsigned long long* rec = tl + ((size_t)blockIdx.x * TL_TILES + k) * 3;
    dlogits_tile<false>(a, tm, tn, [&]() { after_loop(); if (threadIdx.x == 0 && k < TL_TILES) rec[1] = wall(); }, before_stores);
    if (threadIdx.x == 0 && k < TL_TILES) { rec[0] = tlast; rec[2] = wall(); }
  });
  put_summary(pr, t0, tlast, Q.home, n);
}

__global__ void fill_kernel(__bf16* p, size_t n, unsigned seed, float scale) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    unsigned x = (unsigned)(i * 2654435761u) ^ seed;
    x ^= x >> 16; x *= 0x85ebca6bu; x ^= x >> 13; x *= 0xc2b2ae35u; x ^= x >> 16;
    p[i] = (__bf16)(((float)(x & 0xffff) / 65536.f - 0.5f) * scale);
  }
}

}  // namespace pg

static void report(const char* name, const std::vector<unsigned long long>& t, int grid, float ms, double flops) {
  unsigned long long s0 = ~0ull, e1 = 0;
  for (int b = 0; b < grid; ++b) { s0 = std::min(s0, t[b * 4]); e1 = std::max(e1, t[b * 4 + 1]); }
  double idle = 0, lastlen = 0;
  int tiles = 0;
  for (int b = 0; b < grid; ++b) {
    idle += e1 - t[b * 4 + 1]; lastlen += t[b * 4 + 1] - t[b * 4 + 2]; tiles += (int)(t[b * 4 + 3] & 0xffffffffu);
  }
  const double span = (double)(e1 - s0);
  printf("[%-9s] %.3f ms per launch (%.1f TFLOP/s), %d tiles; a workgroup idles %.1f us at the end on average (%.2f%% of the launch); "
         "its last tile took %.1f us\n", name, ms, flops / ms / 1e9, tiles, idle / grid * 0.01, idle / grid / span * 100, lastlen / grid * 0.01);
  for (int x = 0; x < 8; ++x) {
    double mn = 1e30, mx = 0;
    int n = 0, tl = 0;
    for (int b = 0; b < grid; ++b)
      if ((int)(t[b * 4 + 3] >> 32) == x) {
        const double v = (t[b * 4 + 1] - s0) * 0.01;
        mn = std::min(mn, v); mx = std::max(mx, v); ++n; tl += (int)(t[b * 4 + 3] & 0xffffffffu);
      }
    if (n) printf("    XCD %d: %2d workgroups, %4d tiles, done %.0f .. %.0f us after the launch started\n", x, n, tl, mn, mx);
  }
  fflush(stdout);
}

int main(int argc, char** argv) {
  const int reps = argc > 1 ? atoi(argv[1]) : 2;
  const int T = 32768, d = 5120, vc = 22784, V = 151936;     // one full chunk of the headline plan: 89 vocab tiles
  CK(init_gemm_kernels());
  CK(hipFuncSetAttribute(reinterpret_cast<const void*>(store_timeline_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, PERSISTENT_LDS_BYTES));
  CK(hipFuncSetAttribute(reinterpret_cast<const void*>(dlogits_timeline_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, PERSISTENT_LDS_BYTES));
  int cus = 0;
  CK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
  const int grid = std::max(8, cus / 8 * 8);
  const int ld_t = T + 64, ld_v = vc + 64;     // odd numbers of 128-byte lines, as the library pads them
  __bf16 *dST, *HcT, *dS, *WT, *W, *Hc;
  float *dW, *dH, *lse2, *coefc;
  int* yc;
  Ctl* ctl;
  unsigned* queue;
  unsigned long long *pr, *tl;
  CK(hipMalloc(&dST, (size_t)vc * ld_t * 2)); CK(hipMalloc(&HcT, (size_t)d * ld_t * 2));
  CK(hipMalloc(&dS, (size_t)T * ld_v * 2)); CK(hipMalloc(&WT, (size_t)d * ld_v * 2));
  CK(hipMalloc(&W, (size_t)V * d * 2)); CK(hipMalloc(&Hc, (size_t)T * d * 2));
  CK(hipMalloc(&dW, (size_t)vc * d * 4)); CK(hipMalloc(&dH, (size_t)T * d * 4));
  CK(hipMalloc(&yc, T * 4)); CK(hipMalloc(&lse2, T * 4)); CK(hipMalloc(&coefc, T * 4));
  CK(hipMalloc(&ctl, sizeof(Ctl))); CK(hipMalloc(&queue, 64));
  CK(hipMalloc(&pr, (size_t)grid * 4 * 8)); CK(hipMalloc(&tl, (size_t)grid * TL_TILES * 3 * 8));
  Ctl h{T, T, 1.f, 0};
  CK(hipMemcpy(ctl, &h, sizeof h, hipMemcpyHostToDevice));
  fill_kernel<<<1024, 256>>>(dST, (size_t)vc * ld_t, 1u, 1e-3f);
  fill_kernel<<<1024, 256>>>(HcT, (size_t)d * ld_t, 2u, 3.4f);
  fill_kernel<<<1024, 256>>>(dS, (size_t)T * ld_v, 3u, 1e-3f);
  fill_kernel<<<1024, 256>>>(WT, (size_t)d * ld_v, 4u, 0.07f);
  fill_kernel<<<1024, 256>>>(W, (size_t)V * d, 5u, 0.07f);      // W ~ U(-0.035, 0.035): standard deviation 0.02
  fill_kernel<<<1024, 256>>>(Hc, (size_t)T * d, 6u, 3.4f);      // H ~ U(-1.7, 1.7): unit RMS
  CK(hipMemset(dH, 0, (size_t)T * d * 4));
  CK(hipMemset(yc, 0, T * 4));
  {
    std::vector<float> l(T, 17.0f), c(T, 3e-5f);                // a plausible log2-sum-exp and loss coefficient per row
    CK(hipMemcpy(lse2, l.data(), T * 4, hipMemcpyHostToDevice));
    CK(hipMemcpy(coefc, c.data(), T * 4, hipMemcpyHostToDevice));
  }
  CK(hipDeviceSynchronize());

  StoreArgs w{};      // dW chunk: [vc, d] = dS^T [vc, T] x H^T [d, T]
  w.A = dST; w.B = HcT; w.a_rows = vc; w.b_rows = d; w.lda = ld_t; w.ldb = ld_t; w.M = vc; w.N = d; w.K = T;
  w.tiles_m = vc / 256; w.tiles_n = d / 256; w.C = dW; w.ldc = d; w.k_from_ctl = 1; w.ctl = ctl; w.queue = queue;
  StoreArgs g{};      // dH: [T, d] += dS [T, vc] x W^T [d, vc]
  g.A = dS; g.B = WT; g.a_rows = T; g.b_rows = d; g.lda = ld_v; g.ldb = ld_v; g.M = T; g.N = d; g.K = vc;
  g.tiles_m = T / 256; g.tiles_n = d / 256; g.C = dH; g.ldc = d; g.accumulate = 1; g.m_from_ctl = 1; g.split_k = 1; g.ctl = ctl; g.queue = queue;
  DlogitsArgs r{};    // recompute of the chunk's logits, dS and dS^T out
  r.W = W; r.Hc = Hc; r.w_rows = V; r.h_rows = T; r.ldw = d; r.ldh = d; r.K = d; r.V = V; r.v0 = vc; r.ld_s = ld_v; r.ld_t = ld_t;
  r.tiles_v = vc / 256; r.tiles_t = T / 256; r.t_cap = T; r.scale = 1.4427f; r.yc = yc; r.lse2 = lse2; r.coefc = coefc;
  r.dS = dS; r.dST = dST; r.ctl = ctl; r.queue = queue;

  const double fl = 2.0 * vc * (double)T * d;
  std::vector<unsigned long long> t((size_t)grid * 4), v((size_t)grid * TL_TILES * 3);
  const char* names[3] = {"dW", "dH", "recompute"};
  for (int rep = 0; rep < reps; ++rep)
    for (int which = 0; which < 3; ++which) {
      hipEvent_t e0, e1;
      CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
      CK(hipMemset(tl, 0, v.size() * 8));
      for (int it = 0; it < 4; ++it) {         // three launches to settle the clock, the fourth is reported
        CK(hipMemsetAsync(queue, 0, 64, 0));
        if (it == 3) CK(hipEventRecord(e0));
        if (which == 0) hipLaunchKernelGGL(store_timeline_kernel, dim3(grid), dim3(NTHREADS), PERSISTENT_LDS_BYTES, 0, w, pr);
        else if (which == 1) hipLaunchKernelGGL(store_timeline_kernel, dim3(grid), dim3(NTHREADS), PERSISTENT_LDS_BYTES, 0, g, pr);
        else hipLaunchKernelGGL(dlogits_timeline_kernel, dim3(grid), dim3(NTHREADS), PERSISTENT_LDS_BYTES, 0, r, pr, tl);
        if (it == 3) CK(hipEventRecord(e1));
      }
      float ms = 0;
      CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
      CK(hipMemcpy(t.data(), pr, t.size() * 8, hipMemcpyDeviceToHost));
      report(names[which], t, grid, ms, fl);
      if (which == 2) {
        CK(hipMemcpy(v.data(), tl, v.size() * 8, hipMemcpyDeviceToHost));
        for (int k = 0; k < TL_TILES; k += (k < 4 ? 1 : 8)) {
          double ml = 0, ep = 0;
          int n = 0;
          for (int b = 0; b < grid; ++b) {
            const unsigned long long* p = &v[((size_t)b * TL_TILES + k) * 3];
            if (p[2]) { ml += p[1] - p[0]; ep += p[2] - p[1]; ++n; }
          }
          if (n) printf("    tile %2d of every workgroup: main loop %.2f us, epilogue %.2f us\n", k, ml / n * 0.01, ep / n * 0.01);
        }
        fflush(stdout);
      }
    }
  return 0;
}
