// 256x256x64 bf16 MFMA tile engine for gfx950 (CDNA4), shared by the three contractions
// of the policy-gradient head:
//   logits^T = W H^T        (forward statistics, and the backward's recompute)
//   dW       = dS^T H
//   dH       = dS W
// Every contraction is brought to the form C[m,n] = sum_k A[m,k] B[n,k] with both
// operands k-contiguous in memory, so one main loop serves all of them.
//
// Work split: WM x WN wavefronts per workgroup; each wavefront owns a (256/WM) x (256/WN)
// block of MFMA 32x32x16 tiles.  The M side of the MFMA is the "vocab-like" operand so
// that a lane's 16 accumulators of one MFMA tile share one n (token): row statistics over
// the vocabulary reduce inside a lane first.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pg {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;

constexpr int BM = 256;           // tile rows   (A rows)
constexpr int BN = 256;           // tile cols   (B rows)
constexpr int BK = 64;            // k-slab per pipeline stage
constexpr int SLAB_BYTES = BM * BK * 2;          // one operand slab: 256 rows x 128 B
constexpr int STAGE_BYTES = 2 * SLAB_BYTES;      // A slab + B slab
constexpr int EPI_STRIDE = 528;                  // epilogue staging: 256 bf16 per row + 16 B pad
constexpr int GEMM_LDS_BYTES = 256 * EPI_STRIDE; // 132 KiB >= the 128 KiB double-buffered main loop
static_assert(GEMM_LDS_BYTES >= 2 * STAGE_BYTES, "LDS budget");

// Wavefront layout of a workgroup.  DIRECT selects global->LDS loads that bypass registers.
template <int WM_, int WN_, bool DIRECT_, bool SCHED_ = false>
struct Cfg {
  static constexpr int WM = WM_, WN = WN_;
  static constexpr int NW = WM * WN;          // wavefronts
  static constexpr int NT = NW * 64;          // threads
  static constexpr int FM = BM / WM / 32;     // MFMA tiles per wavefront along m
  static constexpr int FN = BN / WN / 32;     //                      ... along n
  static constexpr int WROWS = BM / WM;       // rows of the wavefront's block
  static constexpr int WCOLS = BN / WN;
  static constexpr bool DIRECT = DIRECT_;
  static constexpr bool SCHED = SCHED_;       // pin the LDS-read / MFMA interleave
  static constexpr int CHUNKS = 2048 / NT;    // 16-byte chunks per thread per slab
};

// ---- control block written by the row-compaction kernel (device memory) ----
struct Ctl {
  int n_active;   // number of compacted rows
  int n_pad;      // n_active rounded up to a multiple of 256
  float norm;     // loss normaliser
  int pad_;
};

// ---- buffer resources: loads beyond num_bytes return 0, which pads ragged tiles ----
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t num_bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, num_bytes, 0x00020000);
}

// ---- workgroup -> tile mapping -------------------------------------------------
// Workgroups are dealt round-robin to the 8 XCDs, each with a private L2.  The tile
// space is cut into super-blocks of 4 (m) x 8 (n) tiles; the 32 workgroups that run
// together on one XCD take one super-block, so each A slab is reused by 8 and each B
// slab by 4 workgroups out of that XCD's L2.  The 8 XCDs work on 8 neighbouring
// super-blocks along m (same 8 n-tiles), which share their B rows in the last-level cache.
constexpr int SB_M = 4, SB_N = 8;

__host__ __device__ inline int grid_for_tiles(int tiles_m, int tiles_n) {
  int nsb = ((tiles_m + SB_M - 1) / SB_M) * ((tiles_n + SB_N - 1) / SB_N);
  int nsb_pad = (nsb + 7) / 8 * 8;
  return nsb_pad * SB_M * SB_N;
}

__device__ __forceinline__ bool map_tile(int bid, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int nsb_m = (tiles_m + SB_M - 1) / SB_M;
  const int nsb_n = (tiles_n + SB_N - 1) / SB_N;
  const int xcd = bid & 7;
  const int q = bid >> 3;
  const int sb = (q / (SB_M * SB_N)) * 8 + xcd;
  const int w = q % (SB_M * SB_N);
  if (sb >= nsb_m * nsb_n) return false;
  const int sbm = sb % nsb_m, sbn = sb / nsb_m;
  tm = sbm * SB_M + (w % SB_M);
  tn = sbn * SB_N + (w / SB_M);
  return tm < tiles_m && tn < tiles_n;
}

// ---- operand slabs in LDS ----------------------------------------------------------
// Row r (one of 256) holds its 64 k-values as eight 16-byte chunks; chunk c is stored at
// position c ^ ((r >> 1) & 7).  A 16-lane group of an operand read (16 consecutive rows,
// same logical chunk) then touches 16 distinct bank groups.
//
// Register-staged loads: thread t owns chunk (row t/8 + (NT/8) i, logical chunk t%8).
// Direct loads: one wavefront instruction fills 1024 contiguous LDS bytes (8 rows); lane l
// lands at row l/8, position l%8, so it fetches the logical chunk (l%8) ^ ((row>>1)&7).
template <class C>
struct TileLoader {
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t voff[C::CHUNKS];
};

template <class C>
__device__ __forceinline__ void init_loader(TileLoader<C>& L, const void* base, uint32_t num_bytes, int row0,
                                            int ld_elems, int tid) {
  L.rsrc = make_rsrc(base, num_bytes);
#pragma unroll
  for (int i = 0; i < C::CHUNKS; ++i) {
    int row, chunk;
    if (C::DIRECT) {
      const int lane = tid & 63, wave = tid >> 6;
      row = (i * C::NW + wave) * 8 + (lane >> 3);
      chunk = (lane & 7) ^ ((row >> 1) & 7);
    } else {
      row = (tid >> 3) + (C::NT / 8) * i;
      chunk = tid & 7;
    }
    L.voff[i] = (uint32_t)(row0 + row) * (uint32_t)ld_elems * 2u + (uint32_t)chunk * 16u;
  }
}

template <class C>
__device__ __forceinline__ void load_slab_regs(const TileLoader<C>& L, uint32_t k_byte_off, i32x4 (&regs)[C::CHUNKS]) {
#pragma unroll
  for (int i = 0; i < C::CHUNKS; ++i)
    regs[i] = __builtin_amdgcn_raw_buffer_load_b128(L.rsrc, L.voff[i], k_byte_off, 0);
}

template <class C>
__device__ __forceinline__ void store_slab_regs(char* slab, int tid, const i32x4 (&regs)[C::CHUNKS]) {
  const int r = tid >> 3, c = tid & 7;
  char* p = slab + r * 128 + ((c ^ ((r >> 1) & 7)) << 4);
#pragma unroll
  for (int i = 0; i < C::CHUNKS; ++i) *reinterpret_cast<i32x4*>(p + i * (C::NT / 8) * 128) = regs[i];
}

typedef __attribute__((address_space(3))) void lds_void;

template <class C>
__device__ __forceinline__ void load_slab_direct(const TileLoader<C>& L, uint32_t k_byte_off, char* slab, int wave) {
#pragma unroll
  for (int i = 0; i < C::CHUNKS; ++i) {
    char* dst = slab + (i * C::NW + wave) * 1024;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(L.rsrc, (lds_void*)dst, 16, L.voff[i], k_byte_off, 0, 0);
  }
}

__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0) only

// Scheduling hint: NR LDS reads spread evenly between NM MFMAs (read, then its share of MFMAs).
template <int Q, int NR, int NM>
struct Interleave {
  static __device__ __forceinline__ void run() {
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, (NM * (Q + 1)) / NR - (NM * Q) / NR, 0);
    Interleave<Q + 1, NR, NM>::run();
  }
};
template <int NR, int NM>
struct Interleave<NR, NR, NM> {
  static __device__ __forceinline__ void run() {}
};

// One 64-deep k-slab of MFMAs for this wavefront, with the operand fragments of the next
// 16-deep step fetched from LDS while the current step's MFMAs issue.
template <class C>
__device__ __forceinline__ void compute_stage(const char* stage, uint32_t a_row_off, uint32_t b_row_off,
                                              const uint32_t (&koff)[4], f32x16 (&acc)[C::FM][C::FN]) {
  bf16x8 a[2][C::FM], b[2][C::FN];
#pragma unroll
  for (int i = 0; i < C::FM; ++i)
    a[0][i] = *reinterpret_cast<const bf16x8*>(stage + a_row_off + i * (32 * 128) + koff[0]);
#pragma unroll
  for (int j = 0; j < C::FN; ++j)
    b[0][j] = *reinterpret_cast<const bf16x8*>(stage + b_row_off + j * (32 * 128) + koff[0]);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int cur = ks & 1, nxt = cur ^ 1;
    if (ks < 3) {
#pragma unroll
      for (int i = 0; i < C::FM; ++i)
        a[nxt][i] = *reinterpret_cast<const bf16x8*>(stage + a_row_off + i * (32 * 128) + koff[ks + 1]);
#pragma unroll
      for (int j = 0; j < C::FN; ++j)
        b[nxt][j] = *reinterpret_cast<const bf16x8*>(stage + b_row_off + j * (32 * 128) + koff[ks + 1]);
    }
#pragma unroll
    for (int i = 0; i < C::FM; ++i)
#pragma unroll
      for (int j = 0; j < C::FN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
    if (C::SCHED && ks < 3) {
      // interleave: one LDS read, then its share of MFMAs
      Interleave<0, C::FM + C::FN, C::FM * C::FN>::run();
    }
  }
}

// Accumulates C(256x256) += A(256 x K) B(256 x K)^T for this workgroup's tile.
// acc[i][j] is the MFMA tile at rows wm*WROWS+i*32, cols wn*WCOLS+j*32 of the workgroup tile.
template <class C>
__device__ __forceinline__ void mainloop(const TileLoader<C>& LA, const TileLoader<C>& LB, int nk, char* smem,
                                         f32x16 (&acc)[C::FM][C::FN]) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int lrow = lane & 31;
  const int xr = (lane >> 1) & 7;
  const uint32_t a_row_off = (uint32_t)(wm * C::WROWS + lrow) * 128u;
  const uint32_t b_row_off = (uint32_t)(wn * C::WCOLS + lrow) * 128u + SLAB_BYTES;
  uint32_t koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) koff[ks] = (uint32_t)(((ks * 2 + (lane >> 5)) ^ xr) << 4);

  if (nk <= 0) return;
  if constexpr (C::DIRECT) {
    load_slab_direct<C>(LA, 0, smem, wave);
    load_slab_direct<C>(LB, 0, smem + SLAB_BYTES, wave);
    wait_vmem_all();
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      char* cur = smem + (kt & 1) * STAGE_BYTES;
      char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
      if (kt + 1 < nk) {
        load_slab_direct<C>(LA, (uint32_t)(kt + 1) * (BK * 2), nxt, wave);
        load_slab_direct<C>(LB, (uint32_t)(kt + 1) * (BK * 2), nxt + SLAB_BYTES, wave);
      }
      compute_stage<C>(cur, a_row_off, b_row_off, koff, acc);
      wait_vmem_all();
      __syncthreads();
    }
  } else {
    i32x4 ra[C::CHUNKS], rb[C::CHUNKS];
    load_slab_regs<C>(LA, 0, ra);
    load_slab_regs<C>(LB, 0, rb);
    store_slab_regs<C>(smem, tid, ra);
    store_slab_regs<C>(smem + SLAB_BYTES, tid, rb);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      char* cur = smem + (kt & 1) * STAGE_BYTES;
      char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
      const bool more = kt + 1 < nk;
      if (more) {
        load_slab_regs<C>(LA, (uint32_t)(kt + 1) * (BK * 2), ra);
        load_slab_regs<C>(LB, (uint32_t)(kt + 1) * (BK * 2), rb);
      }
      compute_stage<C>(cur, a_row_off, b_row_off, koff, acc);
      if (more) {
        store_slab_regs<C>(nxt, tid, ra);
        store_slab_regs<C>(nxt + SLAB_BYTES, tid, rb);
      }
      __syncthreads();
    }
  }
}

// Row (m) index inside a 32x32 MFMA tile of accumulator register r for this lane;
// the column (n) is lane & 31.
__device__ __forceinline__ int acc_row(int r, int lane) { return ((r >> 2) << 3) + ((lane >> 5) << 2) + (r & 3); }

template <int FM, int FN>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[FM][FN]) {
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
}

}  // namespace pg
