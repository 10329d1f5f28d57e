// The three MFMA kernels of the policy-gradient head (see gemm_core.h for the tile engine).
//
// Accumulator layout they all rely on: acc[i][j][r] of lane l is
//   engine row     wm*64  + i*16 + 4*(l>>4) + r      (i < 4, r < 4)
//   engine column  wn*128 + j*16 + (l & 15)          (j < 8)
// so one lane holds 16 rows of each of its 8 columns, and the four 16-lane groups of a
// wavefront hold the other 48 rows of the same columns.  The two logits kernels put the
// vocabulary on the rows (a token's statistics then reduce inside a lane first); the store
// kernel puts the output's contiguous dimension there (4 consecutive elements per lane).
#include <cstdlib>

#include "kernels.h"
#include "gemm_core.h"

namespace pg {

extern __shared__ __attribute__((aligned(16))) char g_smem[];

// Softmax partial state in the log2 domain: t = z * log2(e) / tau,
// m = max t, s = sum 2^(t-m), u = sum 2^(t-m) (t-m).
__device__ __forceinline__ void merge_state(float& m, float& s, float& u, float m2, float s2, float u2) {
  const float mm = fmaxf(m, m2);
  const float a1 = __builtin_amdgcn_exp2f(m - mm), a2 = __builtin_amdgcn_exp2f(m2 - mm);
  u = a1 * (u + (m - mm) * s) + a2 * (u2 + (m2 - mm) * s2);
  s = a1 * s + a2 * s2;
  m = mm;
}

// Finite stand-in for -inf (keeps 0 * (t - m) finite).  A power of two, so that its product
// with the logit scale is exact and "t - max" of an all-masked column is exactly zero.
constexpr float NEG_BIG = -0x1p100f;

// ------------------------------------------------------------------------------------
// Forward: a tile is 256 vocab rows x 256 compacted tokens.  The logits live only in the
// accumulators; what leaves the kernel is one (m, s, u) triple per token and vocab tile, plus the
// scaled logit of the sampled token.
// Persistent: one workgroup per compute unit takes tiles from the XCD-aware queue (gemm_core.h)
// until none is left.  The operand loads of the next tile run ahead through the tile boundary
// (mainloop_stream), so the statistics epilogue of a tile executes while the first two stages of
// the next one arrive, and a tile costs no launch, no cold prologue and no drain.  A workgroup
// always knows its next tile (the loads need it) and has the claim for the one after that in
// flight.  LDS: the two stage buffers, then the cross-wavefront merge array, the sampled-token ids
// of the tile (double-buffered; loaded one tile ahead so that the epilogue waits on no global load)
// and the words that hand the claimed tiles to all wavefronts.
// ------------------------------------------------------------------------------------
constexpr int FWD_RED_OFF = 2 * STAGE_BYTES;                 // [WM][256 tokens][3] floats
constexpr int FWD_STASH_OFF = FWD_RED_OFF + WM * 256 * 3 * 4; // [2][256] ints
constexpr int FWD_CLAIM_OFF = FWD_STASH_OFF + 2 * 256 * 4;    // [4] ints
constexpr int FWD_LDS_BYTES = FWD_CLAIM_OFF + 16;

// PROBE = true (the stand-alone measurement tool only) records wall-clock and shader-clock stamps of
// tiles PROBE_FIRST .. PROBE_FIRST + PROBE_TILES - 1 of every workgroup in tl[wg][tile][4] (main loop
// start, main loop end, epilogue end, shader clock at the epilogue's end) and lets the tool switch the
// stealing between XCDs off; the library instantiates PROBE = false, which compiles to none of it.
constexpr int PROBE_FIRST = 150, PROBE_TILES = 16;

template <bool PROBE>
__device__ __forceinline__ void lmhead_fwd_body(const FwdArgs& a, bool steal, unsigned long long* tl) {
  const Ctl ctl = *a.ctl;
  const int tiles_t = min(a.tiles_t, ctl.n_pad / BN);          // live token tiles: known only on the device
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  TileQueue Q;
  Q.init(a.queue, a.tiles_v * tiles_t, 0);
  float* red = reinterpret_cast<float*>(g_smem + FWD_RED_OFF);
  int* stash = reinterpret_cast<int*>(g_smem + FWD_STASH_OFF);
  volatile int* claim = reinterpret_cast<volatile int*>(g_smem + FWD_CLAIM_OFF);

  // the first two tiles
  if (tid == 0) {
    const unsigned k0 = Q.ticket(), k1 = Q.ticket();
    claim[0] = Q.resolve(k0, steal);
    claim[1] = Q.resolve(k1, steal);
  }
  __syncthreads();
  const int b_cur = __builtin_amdgcn_readfirstlane(claim[0]), b_nxt = __builtin_amdgcn_readfirstlane(claim[1]);
  if (b_cur < 0) return;
  int tm, tn, tm1 = 0, tn1 = 0;
  map_tile(b_cur, a.tiles_v, tiles_t, tm, tn);
  bool more = b_nxt >= 0;
  if (more) map_tile(b_nxt, a.tiles_v, tiles_t, tm1, tn1);
  OperandLanes VA, VB;
  VA.init(a.ldw, tid);
  VB.init(a.ldh, tid);
  const bool ahead = a.K / BK >= 2;        // single-stage tiles cannot run two stages ahead
  TileSrc A0, B0, A1, B1;
  A0.set(a.W, a.w_rows, tm * BM, a.ldw, 0u);
  B0.set(a.Hc, a.h_rows, tn * BN, a.ldh, 0u);
  A1.set(a.W, (more && ahead) ? a.w_rows : 0, tm1 * BM, a.ldw, 0u);
  B1.set(a.Hc, (more && ahead) ? a.h_rows : 0, tn1 * BN, a.ldh, 0u);
  const int nk = a.K / BK;
  if (tid < BN) stash[tid] = a.yc[tn * BN + tid];     // visible to everybody behind the main loop's barriers
  int par = 0;

  for (int n = 0;; ++n) {
    const int* ys = stash + (n & 1) * BN;
    f32x4 acc[GM][GN];
    zero_acc(acc);
    const bool probe = PROBE && tl && tid == 0 && n >= PROBE_FIRST && n < PROBE_FIRST + PROBE_TILES;
    unsigned long long* stamp = probe ? tl + ((size_t)blockIdx.x * PROBE_TILES + (n - PROBE_FIRST)) * 4 : nullptr;
    if (probe) stamp[0] = wall_clock64();
    mainloop_stream(VA, VB, A0, B0, A1, B1, nk, n == 0 || !ahead, par, g_smem, acc);
    par = (par + nk) & 1;
    if (probe) stamp[1] = wall_clock64();
    if (!ahead) asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    // claim the tile after the next one: issued here, behind the main loop's last loads (memory
    // operations return in order, an atomic in front of them would hold up their completion), and
    // picked up at the end of the epilogue.  (Left uninitialised on the other threads on purpose: a
    // merged value would make the compiler wait for the atomic right here.)
    unsigned ticket;
    if (tid == 0 && more) ticket = Q.ticket();
    // the next tile's token ids: fetched now, parked in LDS before this tile's stores are issued, so
    // that neither this epilogue nor the next one waits on memory
    int y_next = 0;
    if (more && tid < BN) y_next = a.yc[tn1 * BN + tid];

    const int v_base = tm * BM + wm * WROWS;            // first vocab row of this wavefront's block
    const bool ragged = (tm * BM + BM > a.V);
#pragma unroll
    for (int j = 0; j < GN; ++j) {
      const int tok_l = wn * WCOLS + j * 16 + (lane & 15);
      const int tok = tn * BN + tok_l;
      float mr = NEG_BIG;
#pragma unroll
      for (int i = 0; i < GM; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (ragged && (v_base + i * 16 + acc_row(r, lane) >= a.V)) acc[i][j][r] = NEG_BIG;
          mr = fmaxf(mr, acc[i][j][r]);
        }
      float mx = mr * a.scale;
      const float nmx = -mx;
      float s = 0.f, u = 0.f;
#pragma unroll
      for (int i = 0; i < GM; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float dlt = fmaf(acc[i][j][r], a.scale, nmx);
          const float e = __builtin_amdgcn_exp2f(dlt);
          s += e;
          u = fmaf(e, dlt, u);
        }
      const int ytok = ys[tok_l];
      const int yrel = ytok - v_base;
      const bool mine = (yrel >= 0) && (yrel < WROWS) && (ytok < a.V) && (((yrel >> 2) & 3) == (lane >> 4));
      if (__any(mine)) {
        float zy = 0.f;
#pragma unroll
        for (int i = 0; i < GM; ++i)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (yrel == i * 16 + acc_row(r, lane)) zy = acc[i][j][r] * a.scale;
        if (mine) a.zy[tok] = zy;
      }
#pragma unroll
      for (int sh = 16; sh <= 32; sh <<= 1) {
        const float m2 = __shfl_xor(mx, sh), s2 = __shfl_xor(s, sh), u2 = __shfl_xor(u, sh);
        merge_state(mx, s, u, m2, s2, u2);
      }
      if (lane < 16) {
        float* p = red + (wm * 256 + tok_l) * 3;
        p[0] = mx; p[1] = s; p[2] = u;
      }
    }
    if (tid == 0) claim[2] = more ? Q.resolve(ticket, steal) : -1;
    // LDS-only synchronisation: a full __syncthreads() would also wait for the next tile's loads
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const int b_nn = __builtin_amdgcn_readfirstlane(claim[2]);
    if (tid < BN) {
      stash[((n + 1) & 1) * BN + tid] = y_next;
      const float* p0 = red + tid * 3;
      float m = p0[0], s = p0[1], u = p0[2];
#pragma unroll
      for (int w = 1; w < WM; ++w) {
        const float* p1 = red + (w * 256 + tid) * 3;
        merge_state(m, s, u, p1[0], p1[1], p1[2]);
      }
      const size_t o = (size_t)tm * a.t_cap + (size_t)tn * BN + tid;
      a.part_m[o] = m; a.part_s[o] = s; a.part_u[o] = u;
    }
    if (probe) { stamp[2] = wall_clock64(); stamp[3] = clock64(); }
    if (!more) break;
    tm = tm1; tn = tn1;
    A0.set(a.W, a.w_rows, tm * BM, a.ldw, 0u);
    B0.set(a.Hc, a.h_rows, tn * BN, a.ldh, 0u);
    more = b_nn >= 0;
    if (more) map_tile(b_nn, a.tiles_v, tiles_t, tm1, tn1);
    A1.set(a.W, (more && ahead) ? a.w_rows : 0, tm1 * BM, a.ldw, 0u);
    B1.set(a.Hc, (more && ahead) ? a.h_rows : 0, tn1 * BN, a.ldh, 0u);
  }
}

__global__ __launch_bounds__(NTHREADS) void lmhead_fwd_kernel(FwdArgs a) { lmhead_fwd_body<false>(a, true, nullptr); }

// ------------------------------------------------------------------------------------
// Backward recompute: the same contraction, finished with
//   dS[t,v] = c_t * (onehot(y_t)[v] - 2^(t2 - lse2_t)),  c_t = coef_t / tau,
// rounded to bf16 and written for one vocab chunk in both orientations
// (dS [t_cap, ld_s] for dH, dS^T [vc, ld_t] for dW).  Both go through an LDS transposition
// stage so that global stores are 16 B per lane and 512 B per row.
// ------------------------------------------------------------------------------------
// Where the persistent kernels keep the word that hands a claimed tile to all wavefronts: behind the
// recompute epilogue's staging area (the largest LDS user).
constexpr int CLAIM_OFF = GEMM_LDS_BYTES;
constexpr int PERSISTENT_LDS_BYTES = CLAIM_OFF + 16;

// Takes tiles from the queue until it has none for this workgroup: with steal = false the XCD's own
// share only, with steal = true the own share first and then whatever is left on other XCDs.
// tile(b, after_loop, before_stores) computes the tile with workgroup index b (TileQueue::encode) and
// calls the two hooks once each, on every thread: after_loop behind its main loop's last load (the
// claim for the next tile is issued there: memory operations return in order, an atomic in front of
// the loads would hold up their completion), before_stores at a point that at least one workgroup
// barrier separates from the end of the tile and that lies before the tile's own global stores
// (the claim is picked up there; later it would wait for those stores to complete).
template <class TileFn>
__device__ __forceinline__ void drain_queue(const TileQueue& Q, bool steal, volatile int* claim, TileFn&& tile) {
  const int tid = threadIdx.x;
  int b = queue_broadcast(claim, tid == 0 ? Q.resolve(Q.ticket(), steal) : 0);
  while (b >= 0) {
    // (ticket is left uninitialised on the other threads on purpose: a merged value would make the
    // compiler wait for the atomic where it is issued)
    unsigned ticket;
    tile(b, [&]() { if (tid == 0) ticket = Q.ticket(); }, [&]() { if (tid == 0) claim[0] = Q.resolve(ticket, steal); });
    b = __builtin_amdgcn_readfirstlane(claim[0]);
    // every wavefront is done with the tile's LDS before the next tile's loads land in it
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  }
}

template <bool LO, class AfterLoop, class BeforeStores>
__device__ __forceinline__ void dlogits_tile(const DlogitsArgs& a, int tm, int tn, AfterLoop&& after_loop,
                                             BeforeStores&& before_stores) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  TileLoader LA, LB;
  LA.init(a.W, a.w_rows, a.v0 + tm * BM, a.ldw, 0u, tid);
  LB.init(a.Hc, a.h_rows, tn * BN, a.ldh, 0u, tid);
  f32x4 acc[GM][GN];
  zero_acc(acc);
  mainloop(LA, LB, a.K / BK, g_smem, acc);
  after_loop();

  const int v_base = a.v0 + tm * BM + wm * WROWS;     // global vocab index
  const bool ragged = (a.v0 + tm * BM + BM > a.V);

  // dS = c (onehot - p) is formed as  -sign(c) 2^(t2 - lse2 + log2|c|)  for every element (one fma
  // and one exp2 each; c = 0 gives 2^-inf = 0), the one-hot term c is added to the single element
  // that holds the sampled token (rare, wave-uniform branch), and the sign goes on with the bf16
  // packing.  pk[i][j][h] holds rows 2h, 2h+1 of this lane's 4-row group as a bf16 pair.
  // For an fp32 head a second launch (LO) recomputes the tile and stores the remainders dS - bf16(dS).
  uint32_t pk[GM][GN][2];
#pragma unroll
  for (int j = 0; j < GN; ++j) {
    const int tok = tn * BN + wn * WCOLS + j * 16 + (lane & 15);
    const float c = a.coefc[tok];
    const float k2 = __builtin_amdgcn_logf(fabsf(c)) - a.lse2[tok];
    const uint32_t sgn = c > 0.f ? 0x80008000u : 0u;
    const int yrel = a.yc[tok] - v_base;
    const bool mine = (yrel >= 0) && (yrel < WROWS) && (((yrel >> 2) & 3) == (lane >> 4));
    const bool any_mine = __any(mine);
#pragma unroll
    for (int i = 0; i < GM; ++i) {
      float g[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) g[r] = __builtin_amdgcn_exp2f(fmaf(acc[i][j][r], a.scale, k2));
      if (any_mine) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (yrel == i * 16 + acc_row(r, lane)) g[r] -= fabsf(c);     // sign is applied below
      }
      if (ragged) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (v_base + i * 16 + acc_row(r, lane) >= a.V) g[r] = 0.f;
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
        bf16x2 two;
        two[0] = (__bf16)g[2 * h];
        two[1] = (__bf16)g[2 * h + 1];
        if constexpr (LO) {
          two[0] = (__bf16)(g[2 * h] - (float)two[0]);
          two[1] = (__bf16)(g[2 * h + 1] - (float)two[1]);
        }
        pk[i][j][h] = __builtin_bit_cast(uint32_t, two) ^ sgn;
      }
    }
  }

  // ---- orientation 1: dS[tok][v], staged as rows of 256 v ----
  char* st = g_smem;
#pragma unroll
  for (int j = 0; j < GN; ++j) {
    const int tok_l = wn * WCOLS + j * 16 + (lane & 15);
#pragma unroll
    for (int i = 0; i < GM; ++i) {
      const int v_l = wm * WROWS + i * 16 + ((lane >> 4) << 2);
      uint2 two = make_uint2(pk[i][j][0], pk[i][j][1]);
      *reinterpret_cast<uint2*>(st + tok_l * EPI_STRIDE + v_l * 2) = two;
    }
  }
  before_stores();
  __syncthreads();
  {
    const int chunk = tid & 31, r0 = tid >> 5;
    __bf16* dst = (LO ? a.dS_lo : a.dS) + ((size_t)tn * BN) * a.ld_s + (size_t)tm * BM + chunk * 8;
#pragma unroll 4
    for (int ps = 0; ps < 256 / (NTHREADS / 32); ++ps) {
      const int row = r0 + ps * (NTHREADS / 32);
      const i32x4 v = *reinterpret_cast<const i32x4*>(st + row * EPI_STRIDE + chunk * 16);
      __builtin_nontemporal_store(v, reinterpret_cast<i32x4*>(dst + (size_t)row * a.ld_s));
    }
  }
  __syncthreads();
  // ---- orientation 2: dS^T[v][tok], staged as rows of 256 tokens ----
  // A quad of lanes holds a 4 (vocab rows) x 4 (tokens) block, one token per lane.  Two
  // butterfly exchanges inside the quad turn it so that lane q holds row q of all four tokens,
  // which then goes to LDS as one 8-byte store (instead of sixteen 2-byte ones per block).
  {
    const int q = lane & 3;
    const uint32_t sel = (q & 1) ? 0x03020706u : 0x05040100u;   // v_perm byte selectors, see below
    const bool upper = q >= 2;
    const int row_l = wm * WROWS + ((lane >> 4) << 2) + q;
    const int tok0_l = wn * WCOLS + (((lane & 15) >> 2) << 2);
#pragma unroll
    for (int j = 0; j < GN; ++j) {
#pragma unroll
      for (int i = 0; i < GM; ++i) {
        const uint32_t w0 = pk[i][j][0], w1 = pk[i][j][1];        // rows (0,1), (2,3) of my token
        // neighbour in the lane pair: even lanes keep the even row of both tokens, odd lanes the odd row
        const uint32_t p0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w0, 0xB1, 0xf, 0xf, false);
        const uint32_t p1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w1, 0xB1, 0xf, 0xf, false);
        const uint32_t x0 = __builtin_amdgcn_perm(p0, w0, sel);   // row (q&1),   tokens of my pair
        const uint32_t x1 = __builtin_amdgcn_perm(p1, w1, sel);   // row 2+(q&1), tokens of my pair
        // other pair of the quad: lanes 0,1 collect rows 0,1 and lanes 2,3 rows 2,3 of all four tokens
        const uint32_t send = upper ? x0 : x1;
        const uint32_t recv = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send, 0x4E, 0xf, 0xf, false);
        const uint2 two = upper ? make_uint2(recv, x1) : make_uint2(x0, recv);
        *reinterpret_cast<uint2*>(st + (row_l + i * 16) * EPI_STRIDE_T + (tok0_l + j * 16) * 2) = two;
      }
    }
  }
  __syncthreads();
  {
    const int chunk = tid & 31, r0 = tid >> 5;
    __bf16* dst = (LO ? a.dST_lo : a.dST) + ((size_t)tm * BM) * a.ld_t + (size_t)tn * BN + chunk * 8;
#pragma unroll 4
    for (int ps = 0; ps < 256 / (NTHREADS / 32); ++ps) {
      const int row = r0 + ps * (NTHREADS / 32);
      const i32x4 v = *reinterpret_cast<const i32x4*>(st + row * EPI_STRIDE_T + chunk * 16);
      __builtin_nontemporal_store(v, reinterpret_cast<i32x4*>(dst + (size_t)row * a.ld_t));
    }
  }
}

template <bool LO>
__global__ __launch_bounds__(NTHREADS) void lmhead_dlogits_kernel(DlogitsArgs a) {
  const Ctl ctl = *a.ctl;
  int ld_t_all;
  if (rechunk_all(a.rc, ctl.n_pad, ld_t_all)) {         // few active rows: the first chunk's launch covers the vocabulary
    if (a.rc.chunk > 0) return;
    a.v0 = 0; a.tiles_v = a.rc.tiles_v_all; a.ld_s = a.rc.ld_s_all; a.ld_t = ld_t_all;
  }
  const int tiles_t = min(a.tiles_t, ctl.n_pad / BN);   // live token tiles: known only on the device
  TileQueue Q;
  Q.init(a.queue, a.tiles_v * tiles_t, 0);
  volatile int* claim = reinterpret_cast<volatile int*>(g_smem + CLAIM_OFF);
  // persistent: one workgroup per compute unit takes tiles from the XCD-aware queue until none is left
  drain_queue(Q, true, claim, [&](int b, auto&& after_loop, auto&& before_stores) {
    int tm, tn;
    map_tile(b, a.tiles_v, tiles_t, tm, tn);
    dlogits_tile<LO>(a, tm, tn, after_loop, before_stores);
  });
}

// ------------------------------------------------------------------------------------
// Plain contraction with a store epilogue: C[m,n] (+)= sum_k A[m,k] B[n,k].
// Used for dW (A = dS^T chunk, B = H^T, k = compacted tokens) and for dH
// (A = dS chunk, B = W^T chunk, k = vocab chunk).  The extent marked by k_from_ctl /
// m_from_ctl is the device-side padded token count.
// ------------------------------------------------------------------------------------
// The engine's row side (4 consecutive rows per lane and MFMA tile) is given the B matrix, so that a
// lane owns 4 consecutive n of one m and C[m, n..n+3] leaves as one 16-byte (fp32) or 8-byte (bf16)
// access; N is a multiple of 4.  (Accumulating with fp32 adds performed at the L2 instead of the
// read-modify-write below was measured 6 % slower on the dH contraction.)
template <typename OutT>
__device__ __forceinline__ void store_tile(const StoreArgs& a, int tm, int tn, int m_lim, f32x4 (&acc)[GM][GN]) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  OutT* C = reinterpret_cast<OutT*>(a.C);
#pragma unroll
  for (int j = 0; j < GN; ++j) {
    const int m = tm * BM + wn * WCOLS + j * 16 + (lane & 15);
    if (m >= m_lim) continue;
#pragma unroll
    for (int i = 0; i < GM; ++i) {
      const int n0 = tn * BN + wm * WROWS + i * 16 + ((lane >> 4) << 2);
      if (n0 >= a.N) continue;
      OutT* p = C + (size_t)m * a.ldc + n0;
      f32x4 v = acc[i][j];
      if constexpr (sizeof(OutT) == 4) {
        if (a.accumulate) v += *reinterpret_cast<const f32x4*>(p);
        *reinterpret_cast<f32x4*>(p) = v;
      } else {
        if (a.accumulate) {
          const bf16x4 old = *reinterpret_cast<const bf16x4*>(p);
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] += (float)old[r];
        }
        bf16x4 o;
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = (__bf16)v[r];
        *reinterpret_cast<bf16x4*>(p) = o;
      }
    }
  }
}

// The run-time extents of a store contraction (the padded active-token count is known only on the device).
struct StoreShape {
  int m_lim, tiles_m, K, ks, total;
  __device__ __forceinline__ void init(const StoreArgs& a, const Ctl& ctl) {
    m_lim = a.m_from_ctl ? min(a.M, ctl.n_pad) : a.M;
    tiles_m = min(a.tiles_m, (m_lim + BM - 1) / BM);
    K = a.k_from_ctl ? ctl.n_pad : a.K;
    ks = (a.split_k && a.m_from_ctl) ? dh_split(ctl.n_pad, a.M, a.tiles_n, K / BK) : 1;
    total = tiles_m * ks * a.tiles_n;
  }
};

template <class AfterLoop, class BeforeStores>
__device__ __forceinline__ void gemm_store_tile(StoreArgs a, const StoreShape& sh, int n_pad, int b, AfterLoop&& after_loop,
                                                BeforeStores&& before_stores) {
  const int tid = threadIdx.x;
  int tm, tn;
  map_tile_interleaved(b, sh.tiles_m * sh.ks, a.tiles_n, tm, tn);
  const int part = tm / sh.tiles_m;                    // 0 unless the contraction is split
  tm -= part * sh.tiles_m;
  const int s0 = (int)((long long)part * (sh.K / BK) / sh.ks), s1 = (int)((long long)(part + 1) * (sh.K / BK) / sh.ks);
  const uint32_t kb = (uint32_t)s0 * BK * 2u;          // byte offset of this part's first k

  // (a tile here is hundreds of stages long: the claim for the next one simply travels under the main loop)
  after_loop();
  TileLoader LA, LB;
  LA.init(a.B, a.b_rows, tn * BN, a.ldb, kb, tid);     // engine rows <- n
  LB.init(a.A, a.a_rows, tm * BM, a.lda, kb, tid);     // engine columns <- m
  f32x4 acc[GM][GN];
  zero_acc(acc);
  mainloop(LA, LB, s1 - s0, g_smem, acc);
  if (a.A_lo) {   // split fp32 operands: add the two cross terms (the product of the remainders is dropped)
    __syncthreads();
    LA.init(a.B_lo, a.b_rows, tn * BN, a.ldb_lo, kb, tid);
    mainloop(LA, LB, s1 - s0, g_smem, acc);
    __syncthreads();
    LA.init(a.B, a.b_rows, tn * BN, a.ldb, kb, tid);
    LB.init(a.A_lo, a.a_rows, tm * BM, a.lda, kb, tid);
    mainloop(LA, LB, s1 - s0, g_smem, acc);
  }
  before_stores();
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // the claim is visible behind this barrier
  a.C = static_cast<char*>(a.C) + (size_t)part * n_pad * a.ldc * (a.out_bf16 ? 2 : 4);
  if (a.out_bf16)
    store_tile<__bf16>(a, tm, tn, sh.m_lim, acc);
  else
    store_tile<float>(a, tm, tn, sh.m_lim, acc);
}

__global__ __launch_bounds__(NTHREADS) void gemm_store_kernel(StoreArgs a) {
  const Ctl ctl = *a.ctl;
  int ld_t_all;
  if (a.rc_role && rechunk_all(a.rc, ctl.n_pad, ld_t_all)) {   // few active rows, see Rechunk
    if (a.rc_role == 1) {          // dW: this chunk's rows of the dS^T that spans the whole vocabulary
      a.A = static_cast<const char*>(a.A) + (size_t)a.v0 * ld_t_all * 2;
      if (a.A_lo) a.A_lo = static_cast<const char*>(a.A_lo) + (size_t)a.v0 * ld_t_all * 2;
      a.lda = ld_t_all;
    } else {                       // dH: this chunk's columns of the dS rows that span the whole vocabulary
      a.A = static_cast<const char*>(a.A) + (size_t)a.v0 * 2;
      if (a.A_lo) a.A_lo = static_cast<const char*>(a.A_lo) + (size_t)a.v0 * 2;
      a.lda = a.rc.ld_s_all;
    }
  }
  StoreShape sh;
  sh.init(a, ctl);
  TileQueue Q;
  Q.init(a.queue, sh.total, 1);
  volatile int* claim = reinterpret_cast<volatile int*>(g_smem + CLAIM_OFF);
  // persistent: one workgroup per compute unit takes tiles from the XCD-aware queue until none is left
  drain_queue(Q, true, claim, [&](int b, auto&& after_loop, auto&& before_stores) {
    gemm_store_tile(a, sh, ctl.n_pad, b, after_loop, before_stores);
  });
}

// ---- host-side launchers -------------------------------------------------------------
// Workgroups of a persistent launch: one per compute unit, a multiple of the 8 XCDs.
static int g_persistent_grid = 256;

hipError_t init_gemm_kernels() {
  hipError_t e;
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(lmhead_fwd_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               FWD_LDS_BYTES)) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(lmhead_dlogits_kernel<false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, PERSISTENT_LDS_BYTES)) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(lmhead_dlogits_kernel<true>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, PERSISTENT_LDS_BYTES)) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_store_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               PERSISTENT_LDS_BYTES)) != hipSuccess) return e;
  int dev = 0, cus = 0;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
  g_persistent_grid = cus >= 8 ? (cus / 8) * 8 : 8;
  return hipSuccess;
}

// The grid covers the host-side maximum of tiles (the live extent is known only on the device) but
// never more than one workgroup per compute unit.
static int persistent_grid(int tiles_m, int tiles_n) { return min(grid_for_tiles(tiles_m, tiles_n), g_persistent_grid); }

void launch_lmhead_fwd(const FwdArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(lmhead_fwd_kernel, dim3(persistent_grid(a.tiles_v, a.tiles_t)), dim3(NTHREADS), FWD_LDS_BYTES, s, a);
}
void launch_lmhead_dlogits(const DlogitsArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(lmhead_dlogits_kernel<false>, dim3(persistent_grid(a.tiles_v, a.tiles_t)), dim3(NTHREADS), PERSISTENT_LDS_BYTES, s, a);
  if (a.dS_lo) {   // fp32 head: the remainders, from a second pass over the same tiles with a queue of its own
    DlogitsArgs lo = a;
    lo.queue = a.queue_lo;
    hipLaunchKernelGGL(lmhead_dlogits_kernel<true>, dim3(persistent_grid(a.tiles_v, a.tiles_t)), dim3(NTHREADS), PERSISTENT_LDS_BYTES, s, lo);
  }
}
void launch_gemm_store(const StoreArgs& a, hipStream_t s) {
  // (a split contraction's parts share the row extent: parts x live rows never exceed tiles_m tiles)
  hipLaunchKernelGGL(gemm_store_kernel, dim3(persistent_grid(a.tiles_m, a.tiles_n)), dim3(NTHREADS), PERSISTENT_LDS_BYTES, s, a);
}

}  // namespace pg
