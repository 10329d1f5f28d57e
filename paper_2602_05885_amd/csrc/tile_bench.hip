// Stand-alone benchmark of the tile engine (gemm_core.h): the main loop alone, finished with a
// checksum instead of an epilogue, at the three contraction shapes of the 14B head
// (logits: M=V, N=tokens, K=d;  dW chunk: M=vc, N=d, K=tokens;  dH chunk: M=tokens, N=d, K=vc).
// Usage: tile_bench [iters [shape]]   iters timed launches per shape (default 3); shape 0..2 runs
// that shape only, shape 3 only the register-resident MFMA loop, shape 4 the logits contraction over all
// 32768 tokens in one launch (297 rounds of tiles instead of 74).  It first verifies a small ragged
// product against a naive kernel, then times the MFMA instruction alone (operands and accumulators
// in registers, no memory traffic: the rate the matrix pipes sustain on this chip, which the
// published peak is compared with) and then the three shapes.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "gemm_core.h"
using namespace pg;

#define CK(x)                                                                 \
  do {                                                                        \
    hipError_t e_ = (x);                                                      \
    if (e_ != hipSuccess) {                                                   \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
      exit(1);                                                                \
    }                                                                         \
  } while (0)

extern __shared__ __attribute__((aligned(16))) char g_smem[];

__global__ __launch_bounds__(NTHREADS) void tile_kernel(const __bf16* A, const __bf16* B, float* out, int M, int N,
                                                        int K, int tiles_m, int tiles_n, int store_full) {
  int tm, tn;
  if (!map_tile(blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  TileLoader LA, LB;
  LA.init(A, M, tm * BM, K, 0u, tid);
  LB.init(B, N, tn * BN, K, 0u, tid);
  f32x4 acc[GM][GN];
  zero_acc(acc);
  mainloop(LA, LB, K / BK, g_smem, acc);
  if (store_full) {
    for (int j = 0; j < GN; ++j) {
      const int n = tn * BN + wn * WCOLS + j * 16 + (lane & 15);
      for (int i = 0; i < GM; ++i)
        for (int r = 0; r < 4; ++r) {
          const int m = tm * BM + wm * WROWS + i * 16 + acc_row(r, lane);
          if (m < M && n < N) out[(size_t)m * N + n] = acc[i][j][r];
        }
    }
  } else {
    float s = 0.f;
    for (int i = 0; i < GM; ++i)
      for (int j = 0; j < GN; ++j)
        for (int r = 0; r < 4; ++r) s += acc[i][j][r];
    out[(size_t)blockIdx.x * NTHREADS + tid] = s;
  }
}

// The engine's per-wavefront register tile (4 x 8 MFMA tiles, 8 wavefronts per workgroup, one
// workgroup per CU) with every operand already in registers.  clk[0..1] = shader-clock and
// 100 MHz wall-clock ticks of workgroup 0 over the loop.
// random_operands = 0: small multiples of 0.01 / 0.02 (few mantissa bits set); 1: hashed values
// with full-entropy mantissas in (-1, 1), the kind of data the contractions see.
__device__ __forceinline__ float hashed_unit(unsigned x) {
  x ^= x >> 16; x *= 0x85ebca6bu; x ^= x >> 13; x *= 0xc2b2ae35u; x ^= x >> 16;
  return (float)(x & 0xffffff) / 8388608.f - 1.f;
}
__global__ __launch_bounds__(NTHREADS) void mfma_only_kernel(float* out, int iters, long long* clk, int random_operands) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[GM], b[GN];
  for (int i = 0; i < GM; ++i)
    for (int e = 0; e < 8; ++e)
      a[i][e] = random_operands ? (__bf16)hashed_unit(threadIdx.x * 64 + i * 8 + e)
                                : (__bf16)(0.01f * (float)((lane * 7 + e * 3 + i) % 17 - 8));
  for (int j = 0; j < GN; ++j)
    for (int e = 0; e < 8; ++e)
      b[j][e] = random_operands ? (__bf16)(0.05f * hashed_unit(0x9e3779b9u + threadIdx.x * 64 + j * 8 + e))
                                : (__bf16)(0.02f * (float)((lane * 5 + e + j) % 13 - 6));
  f32x4 acc[GM][GN];
  zero_acc(acc);
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < GN; ++j)
#pragma unroll
      for (int i = 0; i < GM; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  float s = 0.f;
  for (int i = 0; i < GM; ++i)
    for (int j = 0; j < GN; ++j)
      for (int r = 0; r < 4; ++r) s += acc[i][j][r];
  out[(size_t)blockIdx.x * NTHREADS + threadIdx.x] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
}

__global__ void naive_kernel(const __bf16* A, const __bf16* B, float* out, int M, int N, int K) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x, m = blockIdx.y;
  if (n >= N || m >= M) return;
  float s = 0.f;
  for (int k = 0; k < K; ++k) s += (float)A[(size_t)m * K + k] * (float)B[(size_t)n * K + k];
  out[(size_t)m * N + n] = s;
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

static void launch(const __bf16* A, const __bf16* B, float* out, int M, int N, int K, int full) {
  const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
  hipLaunchKernelGGL(tile_kernel, dim3(grid_for_tiles(tiles_m, tiles_n)), dim3(NTHREADS), GEMM_LDS_BYTES, 0, A, B, out,
                     M, N, K, tiles_m, tiles_n, full);
}

int main(int argc, char** argv) {
  const int iters = argc > 1 ? atoi(argv[1]) : 3;
  const int only = argc > 2 ? atoi(argv[2]) : -1;
  CK(hipFuncSetAttribute(reinterpret_cast<const void*>(tile_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                         GEMM_LDS_BYTES));
  {  // correctness on a ragged shape
    const int M = 700, N = 520, K = 320;
    __bf16 *A, *B;
    float *out, *ref;
    CK(hipMalloc(&A, (size_t)M * K * 2)); CK(hipMalloc(&B, (size_t)N * K * 2));
    CK(hipMalloc(&out, (size_t)M * N * 4)); CK(hipMalloc(&ref, (size_t)M * N * 4));
    fill_kernel<<<256, 256>>>(A, (size_t)M * K, 1u, 2.f);
    fill_kernel<<<256, 256>>>(B, (size_t)N * K, 2u, 2.f);
    naive_kernel<<<dim3((N + 255) / 256, M), 256>>>(A, B, ref, M, N, K);
    CK(hipMemset(out, 0xff, (size_t)M * N * 4));
    launch(A, B, out, M, N, K, 1);
    CK(hipDeviceSynchronize());
    std::vector<float> h((size_t)M * N), r((size_t)M * N);
    CK(hipMemcpy(h.data(), out, h.size() * 4, hipMemcpyDeviceToHost));
    CK(hipMemcpy(r.data(), ref, r.size() * 4, hipMemcpyDeviceToHost));
    size_t bad = 0;
    double maxerr = 0;
    for (size_t i = 0; i < h.size(); ++i) {
      const double e = fabs((double)h[i] - r[i]);
      if (!(e < 1e-2)) ++bad;
      if (e > maxerr) maxerr = e;
    }
    printf("[check] M=%d N=%d K=%d maxerr=%.3e bad=%zu %s\n", M, N, K, maxerr, bad, bad ? "FAIL" : "ok");
    fflush(stdout);
    CK(hipFree(A)); CK(hipFree(B)); CK(hipFree(out)); CK(hipFree(ref));
    if (bad) return 1;
  }
  if (only < 0 || only == 3) {  // the MFMA instruction alone, one workgroup per CU and four per CU
    float* out;
    long long* clk;
    const int n_it = 20000;
    CK(hipMalloc(&out, (size_t)1024 * NTHREADS * 4)); CK(hipMalloc(&clk, 16));
    for (int pass = 0; pass < 6; ++pass) {
      const int wg_per_cu = 1 + (pass & 1);
      const int random_operands = pass >= 4;
      const int grid = 256 * wg_per_cu;
      mfma_only_kernel<<<grid, NTHREADS>>>(out, n_it / 2, clk, random_operands);   // long enough for the clock to settle
      CK(hipDeviceSynchronize());
      hipEvent_t e0, e1;
      CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
      CK(hipEventRecord(e0));
      mfma_only_kernel<<<grid, NTHREADS>>>(out, n_it, clk, random_operands);
      CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
      float ms;
      CK(hipEventElapsedTime(&ms, e0, e1));
      long long h[2];
      CK(hipMemcpy(h, clk, 16, hipMemcpyDeviceToHost));
      const double fl = (double)grid * (NTHREADS / 64) * n_it * (GM * GN) * 16384.0;
      printf("[mfma ] registers only, %s operands, %d workgroup(s) of %d wavefronts per CU: %.3f ms  %.1f TFLOP/s  "
             "(%.1f%% of 2500)  shader clock %.3f GHz\n", random_operands ? "random" : "small-integer", wg_per_cu,
             NTHREADS / 64, ms, fl / ms / 1e9, fl / ms / 1e9 / 25.0, h[1] ? (double)h[0] / (double)h[1] * 0.1 : 0.0);
      fflush(stdout);
    }
    CK(hipFree(out)); CK(hipFree(clk));
  }
  struct Shape { const char* name; int M, N, K; } shapes[] = {
      {"logits  (V x tokens x d)", 151936, 8192, 5120},
      {"dW chunk (vc x d x tokens)", 21760, 5120, 32768},
      {"dH chunk (tokens x d x vc)", 32768, 5120, 21760},
      {"logits, 32768 tokens (297 rounds)", 151936, 32768, 5120}};
  for (int si = 0; si < 4; ++si) {
    if (only < 0 && si == 3) continue;    // the long logits launch runs only when asked for (shape 4)
    if (only >= 0 && si != (only == 4 ? 3 : only)) continue;
    const Shape s = shapes[si];
    __bf16 *A, *B;
    float* out;
    CK(hipMalloc(&A, (size_t)s.M * s.K * 2)); CK(hipMalloc(&B, (size_t)s.N * s.K * 2));
    const int grid = grid_for_tiles((s.M + 255) / 256, (s.N + 255) / 256);
    CK(hipMalloc(&out, (size_t)grid * NTHREADS * 4));
    fill_kernel<<<1024, 256>>>(A, (size_t)s.M * s.K, 1u, 0.1f);
    fill_kernel<<<1024, 256>>>(B, (size_t)s.N * s.K, 2u, 2.f);
    for (int w = 0; w < 2; ++w) launch(A, B, out, s.M, s.N, s.K, 0);
    CK(hipDeviceSynchronize());
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    CK(hipEventRecord(e0));
    for (int w = 0; w < iters; ++w) launch(A, B, out, s.M, s.N, s.K, 0);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    ms /= iters;
    const double fl = 2.0 * s.M * s.N * s.K;
    printf("[time ] %-28s M=%d N=%d K=%d  %.3f ms  %.1f TFLOP/s  (%.1f%% of 2500)\n", s.name, s.M, s.N, s.K, ms,
           fl / ms / 1e9, fl / ms / 1e9 / 25.0);
    fflush(stdout);
    CK(hipFree(A)); CK(hipFree(B)); CK(hipFree(out));
  }
  return 0;
}
