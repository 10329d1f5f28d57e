// 256x256x64 bf16 MFMA tile engine for gfx950 (CDNA4), shared by the three contractions
// of the policy-gradient head:
//   logits^T = W H^T        (forward statistics, and the backward's recompute)
//   dW       = dS^T H
//   dH       = dS W
// Every contraction is brought to the form C[m,n] = sum_k A[m,k] B[n,k] with both
// operands k-contiguous in memory, so one main loop serves all of them.
//
// Shape of the engine (each choice measured on MI355X):
//   * 8 wavefronts per workgroup as 4 (m) x 2 (n), two per SIMD, each owning a 64 x 128 block
//     = 4 x 8 MFMA 16x16x32 tiles (128 fp32 accumulators per lane).  Two wavefronts per SIMD
//     hide each other's LDS and barrier latency; one wavefront per SIMD with a 128 x 128 block
//     was 30 % slower with compiler-scheduled code.
//   * v_mfma_f32_16x16x32_bf16 rather than 32x32x16: same LDS traffic per flop, half the
//     accumulator traffic; the chip is power-limited under MFMA load and sustains a higher
//     clock with it (+6 % end to end, +13 % on a pure MFMA stream).
//   * operand slabs go global -> LDS directly (buffer_load ... lds, 16 B per lane), two
//     64-deep stages of 64 KiB.
//   * a wavefront that issues a burst of such loads is held at the issue stage while the
//     texture-address unit works through them (16 cycles per 1 KiB load, 64 loads per stage), and
//     its MFMAs wait behind them.  The loads are therefore trickled out one per 64-cycle step over
//     the whole stage, which a two-barrier stage schedule makes legal: the A slab of a stage is
//     dead once the register-resident A fragments have been read (barrier X after step 4), the
//     B slab once the last streamed B fragment has been read (barrier Y, two steps before the end
//     of the stage).  Measured +10..13 % over issuing a stage's loads in one burst.
//   * inside a stage the LDS->register traffic is software-pipelined by hand (A fragments
//     resident, B fragments streamed two steps ahead, the first fragments of the next stage
//     fetched behind barrier Y under the last two steps' MFMAs) and pinned with sched_barrier.
//   * the M side of the MFMA is the "vocab-like" operand, so a lane's accumulators of one
//     MFMA tile share one n (token): row statistics over the vocabulary reduce inside a lane
//     first, then across the four 16-lane groups, then across wavefronts through LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pg {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int BM = 256;           // tile rows   (A rows)
constexpr int BN = 256;           // tile cols   (B rows)
constexpr int BK = 64;            // k-slab per pipeline stage
constexpr int WM = 4, WN = 2;     // wavefront grid
constexpr int NW = WM * WN;
constexpr int NTHREADS = NW * 64;
constexpr int WROWS = BM / WM;    // 64 rows per wavefront
constexpr int WCOLS = BN / WN;    // 128 cols per wavefront
constexpr int GM = WROWS / 16;    // 4 MFMA tiles along m
constexpr int GN = WCOLS / 16;    // 8 MFMA tiles along n
constexpr int SLAB_BYTES = BM * BK * 2;          // one operand slab: 256 rows x 128 B
constexpr int STAGE_BYTES = 2 * SLAB_BYTES;      // A slab + B slab
constexpr int CHUNKS = 32 / NW;                  // direct loads per wavefront per slab (1 KiB each)
// Epilogue staging rows (256 bf16 + pad).  The pad makes the lanes of a half-wavefront hit distinct
// banks: rows written 16 at a time with 8-byte elements want a row pitch of 4 banks (mod 64),
// rows written 8 at a time with 32 bytes per row want 8 banks.
constexpr int EPI_STRIDE = 528;                  // 132 dwords
constexpr int EPI_STRIDE_T = 544;                // 136 dwords
constexpr int GEMM_LDS_BYTES = 256 * EPI_STRIDE_T; // 136 KiB >= the 128 KiB double-buffered main loop
static_assert(GEMM_LDS_BYTES >= 2 * STAGE_BYTES, "LDS budget");
static_assert(GM == 4 && GN == 8, "the main loop's 16-step schedule is written for 4 x 8 MFMA tiles per wavefront");

// ---- control block written by the row-compaction kernel (device memory) ----
struct Ctl {
  int n_active;   // number of compacted rows
  int n_pad;      // n_active rounded up to a multiple of 256
  float norm;     // loss normaliser
  int pad_;
};

// ---- workgroup -> tile mapping -------------------------------------------------
// Workgroups are dealt round-robin to the 8 XCDs, each with a private L2.  The flattened tile
// order (panels of 8 n-tiles; inside a panel, groups of 4 m-tiles, so 32 consecutive tiles form
// a 4 x 8 block whose A slabs are shared by 8 and B slabs by 4 workgroups) is cut into 8 equal
// contiguous ranges, one per XCD: the 32 workgroups resident on an XCD work on one such block
// out of that XCD's L2, and every XCD gets the same number of tiles to within one.
constexpr int SB_M = 4, SB_N = 8;

__host__ __device__ inline int grid_for_tiles(int tiles_m, int tiles_n) {
  const int total = tiles_m * tiles_n;
  return ((total + 7) / 8) * 8;
}

// (host-callable too, like the queue's share() below: a host test sweeps them over tile counts and checks
// that every tile is handed out exactly once)
__host__ __device__ inline int imin(int a, int b) { return a < b ? a : b; }
__host__ __device__ inline int imax(int a, int b) { return a > b ? a : b; }

__host__ __device__ inline bool map_tile(int bid, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int total = tiles_m * tiles_n;   // may be smaller than what the grid was sized for
  const int per = (total + 7) / 8;
  const int xcd = bid & 7, q = bid >> 3;
  const int t = xcd * per + q;
  if (q >= per || t >= total) return false;
  const int panel_tiles = SB_N * tiles_m;
  const int p = t / panel_tiles;
  const int w = imin(SB_N, tiles_n - p * SB_N);
  const int idx = t - p * panel_tiles;
  const int mg = idx / (SB_M * w);
  const int rig = imin(SB_M, tiles_m - mg * SB_M);
  const int rem = idx - mg * SB_M * w;
  tm = mg * SB_M + rem % rig;
  tn = p * SB_N + rem / rig;
  return true;
}

// The same flattened order dealt to the XCDs in units of 32 consecutive tiles (one 4 x 8 block):
// the eight XCDs then work on eight neighbouring blocks of one n-panel at the same time and the
// panel's B slabs are fetched from HBM once for all of them (they meet in the memory-side cache).
// The last (< 256) tiles are split evenly.  Pays when the n-panel (B rows x K) is too large to
// stay cached while an XCD walks the whole M extent on its own: measured +1..3 % on the dW and
// dH contractions, -1.5 % on the logits contraction (whose token panels do stay cached).
__host__ __device__ inline bool map_tile_interleaved(int bid, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int total = tiles_m * tiles_n;
  const int full = (total / 256) * 256;
  const int xcd = bid & 7, q = bid >> 3;
  int t;
  if (q < full / 8) {
    t = ((q >> 5) * 8 + xcd) * 32 + (q & 31);
  } else {
    const int rem = total - full, per = (rem + 7) / 8, qq = q - full / 8;
    t = full + xcd * per + qq;
    if (qq >= per || t >= total) return false;
  }
  const int panel_tiles = SB_N * tiles_m;
  const int p = t / panel_tiles;
  const int w = imin(SB_N, tiles_n - p * SB_N);
  const int idx = t - p * panel_tiles;
  const int mg = idx / (SB_M * w);
  const int rig = imin(SB_M, tiles_m - mg * SB_M);
  const int rem = idx - mg * SB_M * w;
  tm = mg * SB_M + rem % rig;
  tn = p * SB_N + rem / rig;
  return true;
}

// Split-K factor of the dH contraction.  Its row extent is the padded number of active tokens,
// known only on the device; when those rows give fewer tiles than the chip has compute units
// (a microbatch most of whose samples were rejected), the contraction length is cut into ks
// parts that run side by side.  Part p accumulates into its own slab of n_pad rows of the
// [t_cap, d] accumulator (so ks n_pad <= t_cap), and the final scatter adds the slabs in order.
// Every kernel derives ks from the same device-side values, so the decomposition, and with it
// the summation order, is fixed for given inputs.
__host__ __device__ inline int dh_split(int n_pad, int t_cap, int tiles_n, int k_stages) {
  if (n_pad <= 0) return 1;
  const int tiles = (n_pad / 256) * tiles_n;
  int ks = 256 / (tiles > 0 ? tiles : 1);
  if (ks > t_cap / n_pad) ks = t_cap / n_pad;
  if (ks > k_stages / 8) ks = k_stages / 8;        // every part keeps at least 8 stages
  if (ks > 8) ks = 8;
  return ks < 1 ? 1 : ks;
}

// ---- operand slabs in LDS ----------------------------------------------------------
// Row r (one of 256) holds its 64 k-values as eight 16-byte chunks; chunk c is stored at
// position c ^ ((r >> 1) & 7): a 16-lane group of an operand read (16 consecutive rows, same
// logical chunk) then touches 16 distinct bank groups (measured: zero bank conflicts).
// One wavefront load instruction fills 1024 contiguous LDS bytes (8 rows); lane l lands at row
// l/8, position l%8, so it fetches the logical chunk (l%8) ^ ((row>>1)&7) of that row.
// Loads beyond the buffer resource's size return 0, which pads ragged tiles.
static_assert(BM == BN, "one loader serves both operands");
struct TileLoader {
  const void* base;
  uint32_t bytes;
  uint32_t voff[CHUNKS];

  // Buffer resource over the operand; with on == false its range is empty, so loads through it
  // fetch nothing and deliver zeros (used to switch the loads off beyond the last stage without
  // a branch in the schedule).
  __device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc(bool on) const {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, on ? bytes : 0u, 0x00020000);
  }

  // The resource covers only the (up to) 256 rows of this tile, from byte k_byte0 of its first
  // row to the end of its last existing row, so operands of any size can be addressed (a
  // resource's range and the lane offsets are 32-bit) and rows beyond rows_total read as 0.
  __device__ __forceinline__ void init(const void* base_, int rows_total, int row0, int ld_elems, uint32_t k_byte0,
                                       int tid) {
    const int rows = min(max(rows_total - row0, 0), BM);
    const uint64_t b = reinterpret_cast<uint64_t>(base_) + (uint64_t)row0 * (uint64_t)ld_elems * 2u + k_byte0;
    // the tile index is the same for the whole workgroup: keep the resource in scalar registers
    // (left to itself the compiler treats it as per-lane and loops over every load)
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    base = reinterpret_cast<const void*>(((uint64_t)hi << 32) | lo);
    bytes = __builtin_amdgcn_readfirstlane(rows > 0 ? (uint32_t)rows * (uint32_t)ld_elems * 2u - k_byte0 : 0u);
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int row = (i * NW + wave) * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      voff[i] = (uint32_t)row * (uint32_t)ld_elems * 2u + (uint32_t)chunk * 16u;
    }
  }

  // global -> LDS, bypassing registers: chunk i (1 KiB = 8 rows) of this wavefront's share of one
  // operand slab.  `wave` must be wave-uniform (it addresses LDS through M0).
  __device__ __forceinline__ void issue1(__amdgpu_buffer_rsrc_t r, int i, uint32_t k_byte_off, char* slab,
                                         int wave) const {
    char* dst = slab + (i * NW + wave) * 1024;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void*)dst, 16, voff[i], k_byte_off, 0, 0);
  }
};

// Accumulates C(256x256) += A(256 x K) B(256 x K)^T for this workgroup's tile, K = 64 nk.
// acc[i][j] is the 16x16 MFMA tile at rows wm*64+i*16, cols wn*128+j*16 of the workgroup tile;
// within it, register r of lane l is row 4*(l>>4)+r, column l&15.
//
// A stage (64 of k) is 16 steps s = (ks, j) of 4 MFMAs.  Per wavefront and stage:
//   steps 0..1   second half of the B loads of stage kt+1 (the first half went out in the
//                previous tail), A fragments of the second k-half
//   step  4      barrier X: every A read of this stage is complete -> its A slab is free
//   steps 5..8   A loads of stage kt+2 into that slab, one per step
//   step  13     barrier Y: every B read of this stage is complete and stage kt+1 has landed
//                (the wavefront leaves only its 4 newest loads, the A loads of kt+2, in flight)
//   steps 14,15  "tail": first half of the B loads of stage kt+2, first LDS reads of stage kt+1,
//                under the last 8 MFMAs of stage kt
// On return every load has landed and every wavefront has passed a barrier, so the caller may
// reuse the LDS.  The barriers carry their own waits; the "memory" clobber keeps LDS accesses on
// their side of them.
__device__ __forceinline__ void mainloop(const TileLoader& LA, const TileLoader& LB, int nk, char* smem,
                                         f32x4 (&acc)[GM][GN]) {
  constexpr int NS = 2 * GN;          // steps per stage
  constexpr int TAIL = 2;             // steps behind barrier Y
  constexpr int XS = 4;               // barrier X follows this step
  constexpr int BH = CHUNKS / 2;      // B loads per half
  static_assert(CHUNKS == 4 && BH <= XS && XS + CHUNKS < NS - TAIL, "load schedule");
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int lrow = lane & 15;
  const int xr = (lane >> 1) & 7;
  const uint32_t a_off = (uint32_t)(wm * WROWS + lrow) * 128u;
  const uint32_t b_off = (uint32_t)(wn * WCOLS + lrow) * 128u + SLAB_BYTES;
  uint32_t koff[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) koff[ks] = (uint32_t)(((ks * 4 + (lane >> 4)) ^ xr) << 4);
  if (nk <= 0) return;

  bf16x8 a[2][GM], bq[4];
  auto rdA = [&](const char* st, int ks, int i) -> bf16x8 {
    return *reinterpret_cast<const bf16x8*>(st + a_off + i * (16 * 128) + koff[ks]);
  };
  auto rdB = [&](const char* st, int s) -> bf16x8 {   // B fragment of step s
    return *reinterpret_cast<const bf16x8*>(st + b_off + (s % GN) * (16 * 128) + koff[s / GN]);
  };

  {  // prologue: stage 0 complete, A and the first half of B of stage 1
    const __amdgpu_buffer_rsrc_t ra = LA.rsrc(true), rb = LB.rsrc(true);
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) LA.issue1(ra, i, 0, smem, wave);
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) LB.issue1(rb, i, 0, smem + SLAB_BYTES, wave);
    const __amdgpu_buffer_rsrc_t ra1 = LA.rsrc(nk > 1), rb1 = LB.rsrc(nk > 1);
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) LA.issue1(ra1, i, BK * 2, smem + STAGE_BYTES, wave);
#pragma unroll
    for (int i = 0; i < BH; ++i) LB.issue1(rb1, i, BK * 2, smem + STAGE_BYTES + SLAB_BYTES, wave);
  }
  asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");   // all but the CHUNKS + BH newest
  bq[0] = rdB(smem, 0);
#pragma unroll
  for (int i = 0; i < GM; ++i) a[0][i] = rdA(smem, 0, i);
  bq[1] = rdB(smem, 1);

  for (int kt = 0; kt < nk; ++kt) {
    char* cur = smem + (kt & 1) * STAGE_BYTES;
    char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
    const uint32_t kb1 = (uint32_t)(kt + 1) * (BK * 2), kb2 = (uint32_t)(kt + 2) * (BK * 2);
    const __amdgpu_buffer_rsrc_t rb1 = LB.rsrc(kt + 1 < nk);
    const __amdgpu_buffer_rsrc_t ra2 = LA.rsrc(kt + 2 < nk), rb2 = LB.rsrc(kt + 2 < nk);
#pragma unroll
    for (int s = 0; s < NS - TAIL; ++s) {
      const int ks = s / GN, j = s % GN;
      bq[(s + 2) & 3] = rdB(cur, s + 2);
      if (s < GM) a[1][s] = rdA(cur, 1, s);
      if (s < BH) LB.issue1(rb1, BH + s, kb1, nxt + SLAB_BYTES, wave);
      if (s > XS && s <= XS + CHUNKS) LA.issue1(ra2, s - XS - 1, kb2, cur, wave);
#pragma unroll
      for (int i = 0; i < GM; ++i)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks][i], bq[s & 3], acc[i][j], 0, 0, 0);
      // barrier X: all LDS reads but the newest one (a B fragment) are complete
      if (s == XS) asm volatile("s_waitcnt lgkmcnt(1)\n\ts_barrier" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);   // keep this read/load/MFMA interleave as written
    }
    // barrier Y
    asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
    for (int m = 0; m < TAIL * GM; ++m) {
      const int s = NS - TAIL + m / GM, i = m % GM;
      const int ks = s / GN, j = s % GN;
      if (m == 0) bq[0] = rdB(nxt, 0);
      else if (m <= GM) a[0][m - 1] = rdA(nxt, 0, m - 1);
      else if (m == GM + 1) bq[1] = rdB(nxt, 1);
      if (m % GM == 0) LB.issue1(rb2, m / GM, kb2, cur + SLAB_BYTES, wave);
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks][i], bq[s & 3], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---- the same main loop as a stream of tiles (persistent workgroups) -------------------------------
// A persistent workgroup walks a sequence of tiles that share the operands' leading dimensions
// and the contraction length.  The per-lane offsets are then the same for every tile (OperandLanes);
// what changes from tile to tile is the wave-uniform base address and byte range (TileSrc).  The
// stage schedule above keeps two stages of loads in flight, and across a tile boundary those are
// simply the first two stages of the next tile: the load stream never drains, the next tile's
// stage 0 has landed and most of its stage 1 is in flight when the current tile's last MFMA
// retires, and the epilogue runs with those loads in flight.  The epilogue must therefore not touch
// the two stage buffers (the first 2 x STAGE_BYTES of the dynamic LDS).
struct OperandLanes {
  uint32_t voff[CHUNKS];
  __device__ __forceinline__ void init(int ld_elems, int tid) {
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int row = (i * NW + wave) * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ ((row >> 1) & 7);
      voff[i] = (uint32_t)row * (uint32_t)ld_elems * 2u + (uint32_t)chunk * 16u;
    }
  }
};

struct TileSrc {
  uint32_t lo, hi, bytes;       // wave-uniform (scalar registers)
  // rows [row0, row0 + 256) of an operand with rows_total rows of ld_elems elements, from byte
  // k_byte0 of each row on; rows beyond rows_total read as zero; bytes = 0 switches the loads off
  __device__ __forceinline__ void set(const void* base_, int rows_total, int row0, int ld_elems, uint32_t k_byte0) {
    const int rows = min(max(rows_total - row0, 0), BM);
    const uint64_t b = reinterpret_cast<uint64_t>(base_) + (uint64_t)row0 * (uint64_t)ld_elems * 2u + k_byte0;
    lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
    hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    bytes = __builtin_amdgcn_readfirstlane(rows > 0 ? (uint32_t)rows * (uint32_t)ld_elems * 2u - k_byte0 : 0u);
  }
  __device__ __forceinline__ void off() { lo = 0; hi = 0; bytes = 0; }
  __device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc() const {
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((uint64_t)hi << 32) | lo), 0, bytes, 0x00020000);
  }
};

__device__ __forceinline__ void issue_lds(__amdgpu_buffer_rsrc_t r, const OperandLanes& L, int i, uint32_t k_byte_off,
                                          char* slab, int wave) {
  char* dst = slab + (i * NW + wave) * 1024;
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void*)dst, 16, L.voff[i], k_byte_off, 0, 0);
}

// Buffer resource and k byte offset of stage g (counted from this tile's stage 0) of the stream:
// stages 0 .. nk-1 belong to this tile, nk and nk+1 to the next one (nk >= 2).  All of it is
// wave-uniform and stays in scalar registers; the sources are passed as plain values for that.
__device__ __forceinline__ void pick_stage(const TileSrc cur, const TileSrc nxt, int g, int nk,
                                           __amdgpu_buffer_rsrc_t& r, uint32_t& kb) {
  const bool ahead = g >= nk;
  kb = (uint32_t)(ahead ? g - nk : g) * (BK * 2);
  TileSrc t;
  t.lo = __builtin_amdgcn_readfirstlane(ahead ? +nxt.lo : +cur.lo);
  t.hi = __builtin_amdgcn_readfirstlane(ahead ? +nxt.hi : +cur.hi);
  t.bytes = __builtin_amdgcn_readfirstlane(ahead ? +nxt.bytes : +cur.bytes);
  r = t.rsrc();
}

// One tile of the stream: acc += A(256 x K) B(256 x K)^T with K = 64 nk.
//   A0, B0    operand sources of this tile; A1, B1 of the next one (bytes = 0 where the stream
//             ends).  A tile of a single stage (nk = 1) cannot run ahead by two stages: the caller
//             then passes switched-off next sources, cold = true for every tile, and waits for
//             vmcnt(0) and a barrier before the next call.
//   cold      the stream starts here: nothing of this tile is in flight yet
//   par0      stage buffer (0 / 1) that holds, or will hold, this tile's stage 0; the next tile's is
//             (par0 + nk) & 1
// On return the first two stages of the next tile are in the stage buffers or on their way (this
// wavefront's newest CHUNKS + BH loads may still be in flight) and nobody reads the buffers until the
// next call's opening barrier.
__device__ __forceinline__ void mainloop_stream(const OperandLanes& VA, const OperandLanes& VB, const TileSrc A0,
                                                const TileSrc B0, const TileSrc A1, const TileSrc B1, int nk,
                                                bool cold, int par0, char* smem,
                                                f32x4 (&acc)[GM][GN]) {
  constexpr int NS = 2 * GN, TAIL = 2, XS = 4, BH = CHUNKS / 2;
  static_assert(CHUNKS == 4 && BH <= XS && XS + CHUNKS < NS - TAIL, "load schedule");
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int lrow = lane & 15;
  const int xr = (lane >> 1) & 7;
  const uint32_t a_off = (uint32_t)(wm * WROWS + lrow) * 128u;
  const uint32_t b_off = (uint32_t)(wn * WCOLS + lrow) * 128u + SLAB_BYTES;
  uint32_t koff[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) koff[ks] = (uint32_t)(((ks * 4 + (lane >> 4)) ^ xr) << 4);

  bf16x8 a[2][GM], bq[4];
  auto rdA = [&](const char* st, int ks, int i) -> bf16x8 {
    return *reinterpret_cast<const bf16x8*>(st + a_off + i * (16 * 128) + koff[ks]);
  };
  auto rdB = [&](const char* st, int s) -> bf16x8 {
    return *reinterpret_cast<const bf16x8*>(st + b_off + (s % GN) * (16 * 128) + koff[s / GN]);
  };

  if (cold) {   // stage 0 complete, A and the first half of B of stage 1
    char* s0 = smem + par0 * STAGE_BYTES;
    char* s1 = smem + (par0 ^ 1) * STAGE_BYTES;
    __amdgpu_buffer_rsrc_t ra, rb;
    uint32_t kb;
    pick_stage(A0, A1, 0, nk, ra, kb);
    pick_stage(B0, B1, 0, nk, rb, kb);
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) issue_lds(ra, VA, i, 0, s0, wave);
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) issue_lds(rb, VB, i, 0, s0 + SLAB_BYTES, wave);
    pick_stage(A0, A1, 1, nk, ra, kb);
    pick_stage(B0, B1, 1, nk, rb, kb);
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) issue_lds(ra, VA, i, kb, s1, wave);
#pragma unroll
    for (int i = 0; i < BH; ++i) issue_lds(rb, VB, i, kb, s1 + SLAB_BYTES, wave);
  }
  // stage 0 has landed: all but this wavefront's CHUNKS + BH newest loads are complete
  asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");
  {
    const char* s0 = smem + par0 * STAGE_BYTES;
    bq[0] = rdB(s0, 0);
#pragma unroll
    for (int i = 0; i < GM; ++i) a[0][i] = rdA(s0, 0, i);
    bq[1] = rdB(s0, 1);
  }

  for (int kt = 0; kt < nk; ++kt) {
    char* cur = smem + ((par0 + kt) & 1) * STAGE_BYTES;
    char* nxt = smem + ((par0 + kt + 1) & 1) * STAGE_BYTES;
    __amdgpu_buffer_rsrc_t rb1, ra2, rb2;
    uint32_t kb1, kb2, kb2b;
    pick_stage(B0, B1, kt + 1, nk, rb1, kb1);
    pick_stage(A0, A1, kt + 2, nk, ra2, kb2);
    pick_stage(B0, B1, kt + 2, nk, rb2, kb2b);
#pragma unroll
    for (int s = 0; s < NS - TAIL; ++s) {
      const int ks = s / GN, j = s % GN;
      bq[(s + 2) & 3] = rdB(cur, s + 2);
      if (s < GM) a[1][s] = rdA(cur, 1, s);
      if (s < BH) issue_lds(rb1, VB, BH + s, kb1, nxt + SLAB_BYTES, wave);
      if (s > XS && s <= XS + CHUNKS) issue_lds(ra2, VA, s - XS - 1, kb2, cur, wave);
#pragma unroll
      for (int i = 0; i < GM; ++i)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks][i], bq[s & 3], acc[i][j], 0, 0, 0);
      if (s == XS) asm volatile("s_waitcnt lgkmcnt(1)\n\ts_barrier" ::: "memory");   // barrier X
      __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");          // barrier Y
#pragma unroll
    for (int m = 0; m < TAIL * GM; ++m) {
      const int s = NS - TAIL + m / GM, i = m % GM;
      const int ks = s / GN, j = s % GN;
      if (m == 0) bq[0] = rdB(nxt, 0);
      else if (m <= GM) a[0][m - 1] = rdA(nxt, 0, m - 1);
      else if (m == GM + 1) bq[1] = rdB(nxt, 1);
      if (m % GM == 0) issue_lds(rb2, VB, m / GM, kb2b, cur + SLAB_BYTES, wave);
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks][i], bq[s & 3], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// ---- tile queue of the persistent kernels ----------------------------------------------------------
// The eight XCDs of the chip run at different clocks under load (each has its own frequency
// control: 1.58 to 1.80 GHz were measured side by side in one launch), so an equal share of the
// tiles per XCD (which is what the hardware dispatcher hands out: workgroup b runs on XCD b mod 8)
// makes a launch as slow as its slowest XCD.  The MFMA kernels are therefore persistent (one
// workgroup per compute unit) and take their tiles from a queue: XCD y owns the tiles that the
// XCD-aware order (map_tile / map_tile_interleaved) gives to the workgroups b = 8 i + y,
// i = 0 .. n_y - 1; its workgroups take them in that order with one atomic increment of cnt[y], and
// once its share is used up they take tiles from the XCD that has most left.  Which workgroup
// computes a tile does not change the tile's result, so results stay bitwise repeatable.
// cnt[0..7] must be zero at launch.
struct TileQueue {
  unsigned* cnt;
  int total;          // tiles of the launch
  int interleaved;    // 0: map_tile order, 1: map_tile_interleaved order
  int home;           // XCD this workgroup runs on

  __device__ __forceinline__ void init(unsigned* cnt_, int total_, int interleaved_) {
    cnt = cnt_; total = total_; interleaved = interleaved_;
    unsigned x;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
    home = (int)(x & 7u);
  }
  // n_y: how many workgroup indices b = 8 i + y map to a tile
  __host__ __device__ inline int share(int y) const {
    if (!interleaved) {
      const int per = (total + 7) / 8;
      return imin(imax(total - y * per, 0), per);
    }
    const int full = (total / 256) * 256, rem = total - full, per = (rem + 7) / 8;
    return full / 8 + imin(imax(rem - y * per, 0), per);
  }
  // the workgroup index that map_tile / map_tile_interleaved would have seen for entry i of XCD y
  static __host__ __device__ inline int encode(int y, int i) { return (i << 3) | y; }

  // Issues the claim on the home share; the ticket is resolved later, so that the atomic's latency
  // hides behind whatever runs in between.  (atomicInc with the largest bound is an add of one; unlike
  // atomicAdd the compiler does not turn it into a wave-wide reduction that needs the result at once.)
  __device__ __forceinline__ unsigned ticket() const { return atomicInc(cnt + home, 0xffffffffu); }

  // Workgroup index (see encode) of the claimed tile, or -1 when no tile is left anywhere.  Every failed
  // attempt means one more XCD's share is used up, so the loop ends after at most nine rounds.
  // steal = false confines every XCD to its own share (used by the measurement tool only).
  __device__ __forceinline__ int resolve(unsigned tk, bool steal = true) const {
    if ((int)min(tk, 0x40000000u) < share(home)) return encode(home, (int)tk);
    if (!steal) return -1;
    for (int attempt = 0; attempt < 9; ++attempt) {
      int best = -1, best_left = 0;
      for (int y = 0; y < 8; ++y) {
        const unsigned c = __hip_atomic_load(cnt + y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int left = share(y) - (int)min(c, 0x40000000u);
        if (left > best_left) { best_left = left; best = y; }
      }
      if (best < 0) return -1;
      const unsigned t = atomicInc(cnt + best, 0xffffffffu);
      if ((int)min(t, 0x40000000u) < share(best)) return encode(best, (int)t);
    }
    return -1;
  }
};

// Thread 0 claims, everybody learns the claim through one LDS word.  `slot` must lie outside whatever the
// kernel's epilogue uses; the call contains a workgroup barrier (LDS only: vector memory operations
// in flight are not waited for).
__device__ __forceinline__ int queue_broadcast(volatile int* slot, int value_of_thread0) {
  if (threadIdx.x == 0) *slot = value_of_thread0;
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  const int v = __builtin_amdgcn_readfirstlane(*slot);
  return v;
}

// Row (m) index inside a 16x16 MFMA tile of accumulator register r for this lane;
// the column (n) is lane & 15.
__device__ __forceinline__ int acc_row(int r, int lane) { return ((lane >> 4) << 2) + r; }

__device__ __forceinline__ void zero_acc(f32x4 (&acc)[GM][GN]) {
#pragma unroll
  for (int i = 0; i < GM; ++i)
#pragma unroll
    for (int j = 0; j < GN; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
}

}  // namespace pg
