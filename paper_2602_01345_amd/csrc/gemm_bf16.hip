// bf16 matrix-core GEMM of the pruned block's four projections (Sec. 3.3, "Residual Cache
// Reuse", first equation: Layer_j on the kept rows):  out = epilogue(A W^T),
// A [M, K] activations, W [Nout, K] weights, both K-contiguous, fp32 accumulation.
//
// gfx950 design:
//  * v_mfma_f32_32x32x16_bf16; a workgroup owns a BM x BN tile, WM x WN waves own
//    (BM/WM) x (BN/WN) sub-tiles, the K loop advances 64 elements (128 bytes per row).
//  * Global -> LDS copies bypass the registers (global_load_lds_dwordx4): a wave instruction
//    drops 8 rows x 128 bytes straight into LDS.  Because the LDS side of that instruction is
//    lane-linear, the bank-conflict-avoiding XOR swizzle is applied on the global side: the
//    lane that fills 16-byte slot p of row r fetches chunk p ^ ((r >> 1) & 7) of that row, and
//    the MFMA operand reads look the chunk up at the same swizzled slot.
//  * An NST-stage LDS ring (2 to 6 stages, per tile configuration): the loads of tiles t+1 .. t+NST-1 are in
//    flight while tile t feeds the MFMAs; one bare barrier per K step with explicit vmcnt / lgkmcnt waits.
//  * Workgroup ids are remapped so that each XCD (ids are dealt round-robin to the 8 XCDs) works
//    on a contiguous run of tiles, ordered in bands of 8 tile rows, so that the tiles in flight on
//    one XCD form a compact rectangle and share A rows and W columns in that XCD's L2.
#include "common.h"
#include "epilogue.h"
#include "nova_internal.h"

namespace {

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// s_waitcnt with only vmcnt = n constrained (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
#define WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

// LDS byte offset of 16-byte chunk `c` of tile row `r`; a row holds BK elements (64 or 128 bytes).
// The XOR term changes with every group of rows that shares a bank window, so that 16 consecutive
// rows reading the same chunk index hit 16 different 16-byte bank groups.
template <int BK>
__device__ __forceinline__ int swz(int r, int c) {
  if (BK == 64) return r * 128 + ((c ^ ((r >> 1) & 7)) << 4);
  return r * 64 + ((c ^ ((r >> 2) & 3)) << 4);
}

// Whether a workgroup walks several tiles (one workgroup per CU): the modes whose epilogue needs no LDS, large
// tiles only; with a residual the prefetched residual chunks of a wave's MFMA tiles must leave room in the
// register file for the next tile's addresses (at most 4 MFMA tiles per wave).
constexpr bool persistent_tiles(int mfma_tiles_per_wave, bool stagger, int mode) {
  if (stagger) return false;
  if (mode == EPI_GELU || mode == EPI_GELU_TANH || mode == EPI_PLAIN) return true;
  return (mode == EPI_ATTN_OUT || mode == EPI_RESIDUAL) && mfma_tiles_per_wave <= 4;
}

template <int BM, int BN, int WM, int WN, int BK, int NST, bool STAGGER, int MODE>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_kernel(const bf16_t* __restrict__ A,
                                                                const bf16_t* __restrict__ W, int M, int Nout,
                                                                int K, int m_base, int tiles_m, int tiles_n,
                                                                int kslices, EpiParams<bf16_t> ep) {
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;      // MFMA tiles per wave
  constexpr int ROW_BYTES = BK * 2;
  constexpr int CH = ROW_BYTES / 16;                       // 16-byte chunks per tile row
  constexpr int RPI = 64 / CH;                             // tile rows filled by one wave load instruction
  constexpr int LA = BM / RPI / NW, LB = BN / RPI / NW;    // load instructions per wave per stage
  constexpr int LPW = LA + LB;
  constexpr int KS = BK / 16;                              // MFMA K steps per stage
  constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES, STAGE = A_BYTES + B_BYTES;
  constexpr int CT_PITCH = BN + 8;                         // epilogue staging tile pitch (elements)
  constexpr int CT_BYTES = BM * CT_PITCH * 2;
  constexpr int LDS_BYTES = NST * STAGE > CT_BYTES ? NST * STAGE : CT_BYTES;
  static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "tile rows must split over the waves");
  static_assert((NST - 2) * LPW < 64, "vmcnt is a 6-bit counter");
  __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS fill addresses stay scalar
  const int wm = wave / WN, wn = wave % WN;

  // ---- workgroup id -> tile, XCD-contiguous, M fastest -------------------------------
  // kslices > 1 (EPI_PARTIAL only): the grid is kslices copies of the tile grid, copy s sums K slice s
  // PERSIST (the modes whose epilogue needs no LDS, large tiles): the grid is one workgroup per CU and a
  // workgroup takes the tiles L, L + gridDim.x, ...; the first K stages of its next tile are requested
  // before the epilogue of the current one, so their latency passes behind the epilogue.
  constexpr bool PERSIST = persistent_tiles(BM / WM / 32 * (BN / WN / 32), STAGGER, MODE);
  const int nblk = tiles_m * tiles_n;
  const int kslice = PERSIST ? 0 : blockIdx.x / nblk;
  int L = blockIdx.x - kslice * nblk;
  // ---- global -> LDS: instruction i of this wave fills tile rows (i * NW + wave) * RPI + lane / CH
  const int lr = lane / CH, lp = lane % CH;
  const bf16_t* ga[LA];
  const bf16_t* gb[LB];
  int tn = 0, m0 = 0, n0 = 0;
  auto set_tile = [&](int Lt) {
    // Lt -> tile, XCD-contiguous (gridDim.x is a multiple of 8 when a workgroup takes several tiles, so all of
    // them have its XCD's residue)
    const int xcd = Lt & 7, j = Lt >> 3;
    const int base = nblk >> 3, rem = nblk & 7;
    const int id = xcd * base + min(xcd, rem) + j;
    // bands of GM tile rows, column by column inside a band: the workgroups an XCD runs at the same
    // time then cover a compact GM x (slots / GM) rectangle and share A and W tiles in its L2
    constexpr int GM = 8;
    const int band = id / (GM * tiles_n), in_band = id - band * (GM * tiles_n);
    const int first_m = band * GM, rows = min(tiles_m - first_m, GM);
    tn = in_band / rows;
    const int tm = first_m + (in_band - tn * rows);
    m0 = m_base + tm * BM;                                 // this launch covers rows [m_base, M)
    n0 = tn * BN;
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int r = (i * NW + wave) * RPI + lr;
      const int c = (swz<BK>(r, lp) - r * ROW_BYTES) >> 4;   // chunk of the row that lands in slot lp
      ga[i] = A + (int64_t)min(m0 + r, M - 1) * K + c * 8;   // rows past the edge re-read the last row
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const int r = (i * NW + wave) * RPI + lr;
      const int c = (swz<BK>(r, lp) - r * ROW_BYTES) >> 4;
      gb[i] = W + (int64_t)min(n0 + r, Nout - 1) * K + c * 8;
    }
  };
  set_tile(L);
  if (ep.k_rows) {
    // Per-image keep counts: the rows are B segments of ep.k slots and image b fills only the first k_rows[b] of
    // its segment.  A tile none of whose rows is a live slot has nothing to compute (launches with per-image counts
    // give every tile its own workgroup, so leaving here skips exactly this tile).  The whole workgroup leaves
    // together, before the first barrier.
    const int m_hi = min(m0 + BM, M);
    bool live = false;
    for (int b = m0 / ep.k; b * ep.k < m_hi; ++b)
      live = live || max(m0 - b * ep.k, 0) < image_count(ep.k_rows, b, ep.k);
    if (!live) return;
  }
  // load instructions lo..hi-1 (A first, then W) of the tile at K offset k0 into `stage`
  auto issue = [&](int stage, int k0, int lo, int hi) {
    char* sa = lds + stage * STAGE;
    char* sb = sa + A_BYTES;
#pragma unroll
    for (int i = 0; i < LA; ++i)
      if (i >= lo && i < hi)
        __builtin_amdgcn_global_load_lds((gptr_t)(ga[i] + k0), (lptr_t)(sa + (i * NW + wave) * RPI * ROW_BYTES), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < LB; ++i)
      if (LA + i >= lo && LA + i < hi)
        __builtin_amdgcn_global_load_lds((gptr_t)(gb[i] + k0), (lptr_t)(sb + (i * NW + wave) * RPI * ROW_BYTES), 16, 0, 0);
  };

  f32x16 acc[TM][TN];

  const int KT = K / BK / kslices;                         // K steps of this workgroup's slice
  const int k_begin = kslice * KT * BK;
  // With few rows every tile column is streamed by one workgroup (or a few that share it), and all
  // of them would walk K in step: the same 128-byte slice of every weight row at the same time,
  // rows a power-of-two stride apart, i.e. a handful of memory channels.  Each tile column
  // therefore starts its (cyclic) walk over K at its own offset.
  const int kt_first = STAGGER ? (int)(((int64_t)tn * KT) / tiles_n) : 0;
  auto k_of = [&](int t) { const int q = t + kt_first; return k_begin + (q >= KT ? q - KT : q) * BK; };
  // prologue: NST-1 K stages in flight
  auto prologue = [&]() {
#pragma unroll
    for (int t = 0; t < NST - 1; ++t)
      if (t < KT) issue(t, k_of(t), 0, LPW);
  };
  prologue();

  const int half = lane >> 5, r32 = lane & 31;
  const int arow0 = wm * (BM / WM) + r32;   // tile row of this lane's A operand in MFMA tile 0
  const int brow0 = wn * (BN / WN) + r32;
  // swizzled byte offsets of this lane's operand chunk for the 16-wide K steps of a stage
  int aoff[KS], boff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    aoff[ks] = swz<BK>(arow0, ks * 2 + half);
    boff[ks] = swz<BK>(brow0, ks * 2 + half);
  }
  // Operand fragments are double buffered in registers and the schedule is pinned with
  // sched_barrier: the LDS reads of K step ks+1 are issued right after the first MFMA of K step
  // ks, so the remaining MFMAs of that step cover their latency.  The reads of the next stage's
  // first K step are issued right after the barrier, under the MFMAs of this stage's last K step.
  bf16x8 a[2][TM], b[2][TN];
  auto read_frags = [&](int buf, int stage, int ks) {
    const char* sa = lds + stage * STAGE;
    const char* sb = sa + A_BYTES;
#pragma unroll
    for (int i = 0; i < TM; ++i) a[buf][i] = *reinterpret_cast<const bf16x8*>(sa + aoff[ks] + i * 32 * ROW_BYTES);
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) b[buf][jn] = *reinterpret_cast<const bf16x8*>(sb + boff[ks] + jn * 32 * ROW_BYTES);
  };
  // MFMAs lo..hi-1 (flattened over the wave's TM x TN tiles) of one K step
  auto mfmas = [&](int buf, int lo, int hi) {
#pragma unroll
    for (int t = 0; t < TM * TN; ++t)
      if (t >= lo && t < hi) acc[t / TN][t % TN] = mfma32(b[buf][t % TN], a[buf][t / TN], acc[t / TN][t % TN]);
  };
  constexpr int LEAD = 1;                   // MFMAs issued before the next K step's LDS reads
  static_assert(KS % 2 == 0, "fragment buffers alternate per K step");

  bool first_tile = true;
  for (;;) {   // tiles of this workgroup (one, unless PERSIST)
  // wait for the first K stage.  After a prefetch the epilogue's own loads and stores are in flight as well and
  // the counter does not tell them apart: wait for everything.
  if (first_tile && KT >= NST - 1) { WAIT_VMCNT((NST - 2) * LPW); } else { WAIT_VMCNT(0); }
  first_tile = false;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int jn = 0; jn < TN; ++jn)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][jn][r] = 0.f;
  int stage = 0, fill = NST - 1;            // stage being computed / stage being refilled
  read_frags(0, 0, 0);
  for (int kt = 0; kt < KT; ++kt) {
    // the stage refilled now was read during the previous iteration and freed by its barrier
    const bool more = kt + NST - 1 < KT;
    constexpr int LPS = (LPW + KS - 2) / (KS - 1);   // fill instructions issued per K step (all but the last step)
#pragma unroll
    for (int ks = 0; ks < KS - 1; ++ks) {
      mfmas(ks & 1, 0, LEAD);
      __builtin_amdgcn_sched_barrier(0);
      if (more) issue(fill, k_of(kt + NST - 1), ks * LPS, ks + 2 == KS ? LPW : (ks + 1) * LPS);
      read_frags((ks + 1) & 1, stage, ks + 1);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(ks & 1, LEAD, TM * TN);
      __builtin_amdgcn_sched_barrier(0);
    }
    // tile kt+1 must have landed (younger tiles may stay in flight) and this wave's reads of
    // the current stage must be complete before anyone may refill it
    if (more) { WAIT_VMCNT((NST - 2) * LPW); } else { WAIT_VMCNT(0); }
    __builtin_amdgcn_s_waitcnt(0xC07F);     // lgkmcnt(0)
    // a bare barrier: __syncthreads() would add a wait for ALL outstanding loads, i.e. also for the
    // tiles requested for later iterations, and a ring deeper than two stages would gain nothing
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    const int next = stage + 1 == NST ? 0 : stage + 1;
    mfmas((KS - 1) & 1, 0, LEAD);
    __builtin_amdgcn_sched_barrier(0);
    if (kt + 1 < KT) read_frags(0, next, 0);
    __builtin_amdgcn_sched_barrier(0);
    mfmas((KS - 1) & 1, LEAD, TM * TN);
    __builtin_amdgcn_sched_barrier(0);
    stage = next;
    fill = fill + 1 == NST ? 0 : fill + 1;
  }
  if constexpr (MODE == EPI_ENTROPY) {
    // The accumulators (+ bias) are logits that never leave the chip: each lane reduces the columns
    // it holds of a token row to (max, S, T), the two half-waves and then the waves that share the
    // row merge their partials, and one (m, S, T) per row and column tile goes to memory.
    constexpr float kLog2e = 1.4426950408889634f;
    f32x4* lp = reinterpret_cast<f32x4*>(lds);           // [WN][BM]; the stage ring is free after the last barrier
    float bias[TN][16];
#pragma unroll
    for (int jn = 0; jn < TN; ++jn)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int col = n0 + wn * (BN / WN) + jn * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
        bias[jn][r] = col >= Nout ? -INFINITY : (ep.bias ? (float)ep.bias[col] : 0.0f);   // -inf masks the edge
      }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      float m = -INFINITY;
#pragma unroll
      for (int jn = 0; jn < TN; ++jn)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          acc[i][jn][r] += bias[jn][r];
          m = fmaxf(m, acc[i][jn][r]);
        }
      float S = 0.0f, T = 0.0f;
      if (m != -INFINITY) {
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float d = fmaxf(acc[i][jn][r] - m, -200.0f);     // e^-200 == 0: masked columns add nothing
            const float e = __builtin_amdgcn_exp2f(d * kLog2e);
            S += e;
            T = fmaf(-d, e, T);
          }
      }
      entropy_merge(m, S, T, __shfl_xor(m, 32, 64), __shfl_xor(S, 32, 64), __shfl_xor(T, 32, 64));
      if (half == 0) lp[wn * BM + wm * (BM / WM) + i * 32 + r32] = f32x4{m, S, T, 0.0f};
    }
    __syncthreads();
    for (int row = tid; row < BM; row += NW * 64) {
      const f32x4 a = lp[row];
      float pm = a[0], pS = a[1], pT = a[2];
#pragma unroll
      for (int w = 1; w < WN; ++w) {
        const f32x4 b2 = lp[w * BM + row];
        entropy_merge(pm, pS, pT, b2[0], b2[1], b2[2]);
      }
      if (m0 + row < M) ep.ent_part[(int64_t)tn * M + m0 + row] = f32x4{pm, pS, pT, 0.0f};
    }
    return;
  }
  // The MFMAs ran with the weight rows as the A operand, so a lane owns token l % 32 of each MFMA
  // tile and, per register group r / 4, four consecutive output features.
  if constexpr (MODE == EPI_PARTIAL) {
    float* pp = ep.part + ((int64_t)kslice * (M - m_base) - m_base) * Nout;     // [slice][row - m_base][Nout]
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = m0 + wm * (BM / WM) + i * 32 + r32;
#pragma unroll
      for (int jn = 0; jn < TN; ++jn)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int col = n0 + wn * (BN / WN) + jn * 32 + 8 * g4 + 4 * half;
          if (row < M && col < Nout) {
            f32x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[i][jn][g4 * 4 + e];
            *reinterpret_cast<f32x4*>(pp + (int64_t)row * Nout + col) = v;
          }
        }
    }
    return;
  } else if constexpr (MODE != EPI_QKV) {
    const int em0 = m0, en0 = n0;            // origin of the tile whose accumulators are written out below
    // ---- direct epilogue (everything but the QKV projection): no LDS staging.  A lane owns token l % 32
    // and, per register group g4, four consecutive features (8 g4 + 4 half ..); swapping the upper lanes'
    // group g4 with the lower lanes' group g4 + 1 (v_permlane32_swap) leaves every lane with eight
    // consecutive features of its token: 16-byte residual / gate loads and one 16-byte store, and the two
    // halves of the wave cover 32 contiguous bytes of each row.
    constexpr bool HAS_RES = MODE == EPI_ATTN_OUT || MODE == EPI_RESIDUAL;
    // The residual chunks are requested first, so that their latency (two dependent loads for the
    // gathered residual) passes behind the conversion work.
    bf16x8 rs[HAS_RES ? TM * TN * 2 : 1];
    if constexpr (HAS_RES) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = em0 + wm * (BM / WM) + i * 32 + r32;
        int64_t roff = (int64_t)row * ep.ldo;
        if (MODE == EPI_ATTN_OUT && row < M)
          roff = ((int64_t)(row / ep.k) * ep.Ntok + min(max(ep.idx[row], 0), ep.Ntok - 1)) * ep.C;
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
          for (int gp = 0; gp < 2; ++gp) {
            const int col = en0 + wn * (BN / WN) + jn * 32 + 8 * (2 * gp + half);
            if (row < M && col < Nout) rs[(i * TN + jn) * 2 + gp] = *reinterpret_cast<const bf16x8*>(ep.res + roff + col);
          }
      }
    }
    bf16x4 bvec[TN][4];                       // this lane's bias entries, packed
#pragma unroll
    for (int jn = 0; jn < TN; ++jn)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int col = en0 + wn * (BN / WN) + jn * 32 + 8 * g4 + 4 * half;
        bf16x4 bv = {(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
        if (ep.bias && col < Nout) bv = *reinterpret_cast<const bf16x4*>(ep.bias + col);
        bvec[jn][g4] = bv;
      }
    bool more_tiles = false;
    if constexpr (PERSIST) {
      // Every wave has passed the last barrier of the K loop, nobody reads the ring any more: request the
      // first stages of this workgroup's next tile now.  They are requested after the epilogue's own loads
      // (loads complete in order, so those do not wait for the tile data) and land behind the conversion work.
      if (L + (int)gridDim.x < nblk) {
        more_tiles = true;
        L += gridDim.x;
        set_tile(L);
        prologue();
      }
    }
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
      const int cb = en0 + wn * (BN / WN) + jn * 32;                   // first feature of this 32-column block
      float bias[16];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
        for (int e = 0; e < 4; ++e) bias[g4 * 4 + e] = (float)bvec[jn][g4][e];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = em0 + wm * (BM / WM) + i * 32 + r32;
#pragma unroll
        for (int gp = 0; gp < 2; ++gp) {                              // register groups (2 gp, 2 gp + 1)
          u32x2 lo, hi;                                               // packed bf16 pairs of the two groups
#pragma unroll
          for (int g = 0; g < 2; ++g) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float v = acc[i][jn][(2 * gp + g) * 4 + e] + bias[(2 * gp + g) * 4 + e];
              if (MODE == EPI_GELU) v = gelu_erf(v);
              if (MODE == EPI_GELU_TANH) v = gelu_tanh(v);
              if (MODE == EPI_PLAIN) v *= ep.q_scale;
              o[e] = (bf16_t)v;
            }
            (g == 0 ? lo : hi) = __builtin_bit_cast(u32x2, o);
          }
          u32x4 out16;
#pragma unroll
          for (int w2 = 0; w2 < 2; ++w2) {
            const auto sw = __builtin_amdgcn_permlane32_swap(lo[w2], hi[w2], false, false);
            out16[w2] = sw[0];          // lower lanes: own group 2 gp;       upper lanes: lower partner's group 2 gp + 1
            out16[2 + w2] = sw[1];      // lower lanes: upper partner's 2 gp; upper lanes: own group 2 gp + 1
          }
          const int col = cb + 8 * (2 * gp + half);                   // eight consecutive features from here
          if (row < M && col < Nout) {
            if constexpr (HAS_RES) {
              // the projection (+ bias) is rounded to bf16 before the gate and the residual are applied
              const bf16x8 v = __builtin_bit_cast(bf16x8, out16);
              const bf16x8 r = rs[(i * TN + jn) * 2 + gp];
              bf16x8 o;
              if (ep.gate) {
                const bf16x8 gt = *reinterpret_cast<const bf16x8*>(ep.gate + (int64_t)(row / ep.k) * ep.gate_pitch + col);
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = (bf16_t)fmaf((float)gt[e], (float)v[e], (float)r[e]);
              } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = (bf16_t)((float)v[e] + (float)r[e]);
              }
              *reinterpret_cast<bf16x8*>(ep.out + (int64_t)row * ep.ldo + col) = o;
            } else {
              *reinterpret_cast<u32x4*>(ep.out + (int64_t)row * ep.ldo + col) = out16;
            }
          }
        }
      }
    }
    if (more_tiles) continue;
    return;
  }
  break;   // the QKV projection: staged epilogue below
  }
  // ---- QKV epilogue, stage 1: accumulators (+ bias) -> bf16 tile in LDS, row-major (the value columns are
  // written transposed, which needs the whole tile at hand) ---------------------------------------------
  constexpr int NT = NW * 64;
  constexpr int CPR = BN / 8;                       // chunks per tile row
  constexpr int RPP = NT / CPR;                     // tile rows covered per pass
  constexpr int NI = BM / RPP;                      // tile rows per thread
  static_assert(NT % CPR == 0 && BM % RPP == 0, "chunk walk tiles the output tile");
  bf16_t* ct = reinterpret_cast<bf16_t*>(lds);
#pragma unroll
  for (int jn = 0; jn < TN; ++jn)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int lc = wn * (BN / WN) + jn * 32 + 8 * g4 + 4 * half;   // first of 4 consecutive features
      const int col = n0 + lc;
      const float qs = col < ep.C ? ep.q_scale : 1.0f;   // query features (C is a multiple of 8: all four or none)
      float bias[4] = {0.f, 0.f, 0.f, 0.f};
      if (ep.bias && col < Nout) {
        const bf16x4 bv = *reinterpret_cast<const bf16x4*>(ep.bias + col);
#pragma unroll
        for (int e = 0; e < 4; ++e) bias[e] = (float)bv[e];
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int lrw = wm * (BM / WM) + i * 32 + r32;
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (bf16_t)((acc[i][jn][g4 * 4 + e] + bias[e]) * qs);
        *reinterpret_cast<bf16x4*>(ct + lrw * CT_PITCH + lc) = o;
      }
    }
  __syncthreads();

  // ---- stage 2: 16-byte row chunks out of LDS, coalesced global stores ----------------------
  // A thread keeps one column chunk and walks down the tile rows, so everything that depends on
  // the column (q / key / value split, head, channel) is computed once.
  {
    const int cc = tid % CPR, r_first = tid / CPR;
    const int col = n0 + cc * 8;
    const int sel = col / ep.C, cf = col - sel * ep.C;
    const int head = cf / ep.dh, d = cf - head * ep.dh;
    if (col < Nout && sel != 2) {
#pragma unroll
      for (int it = 0; it < NI; ++it) {
        const int lrw = r_first + it * RPP;
        const int row = m0 + lrw;
        if (row >= M) break;
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(ct + lrw * CT_PITCH + cc * 8);
        if (sel == 0) {
          *reinterpret_cast<bf16x8*>(ep.out + (int64_t)row * ep.ldo + cf) = v;
        } else {
          const int bb = row / ep.k, s = row - bb * ep.k;
          if (s < image_count(ep.k_rows, bb, ep.k))      // slots past an image's keep count append nothing
            *reinterpret_cast<bf16x8*>(ep.kc + (((int64_t)bb * ep.heads + head) * ep.cap +
                                                image_prior(ep.kv_rows, bb, ep.P) + s) * ep.dh + d) = v;
        }
      }
    }
  }
  if (MODE == EPI_QKV) {
    // value columns: the cache is key-minor, so a thread keeps one tile row (token) and walks
    // the value columns; consecutive lanes hold consecutive tokens -> consecutive addresses
    const int v_lo = max(2 * ep.C - n0, 0);          // first tile column that is a value feature
    const int v_hi = min(BN, Nout - n0);
    if (v_hi > v_lo) {
      constexpr int CG = NT / BM;                    // column groups walked in parallel
      static_assert(NT % BM == 0, "one thread per tile row and column group");
      const int lrw = tid % BM, cg = tid / BM;
      const int row = m0 + lrw;
      const int bb = row < M ? row / ep.k : 0, s = row - bb * ep.k;
      if (row < M && s < image_count(ep.k_rows, bb, ep.k)) {
        bf16_t* vrow = ep.vc + (int64_t)bb * ep.heads * ep.dh * ep.cap + image_prior(ep.kv_rows, bb, ep.P) + s;
        const int cf0 = n0 - 2 * ep.C;               // value feature of tile column 0
        for (int lc = v_lo + cg; lc < v_hi; lc += CG)
          vrow[(int64_t)(cf0 + lc) * ep.cap] = ct[lrw * CT_PITCH + lc];   // (head * dh + d) * cap
      }
    }
  }
}

template <int BM, int BN, int WM, int WN, int BK, int NST, bool STAGGER, int MODE>
hipError_t launch_cfg(hipStream_t st, const bf16_t* A, const bf16_t* W, int m_base, int M, int Nout, int K,
                      const EpiParams<bf16_t>& ep, int slots, int kslices = 1) {
  const int tiles_m = (M - m_base + BM - 1) / BM, tiles_n = (Nout + BN - 1) / BN;   // rows [m_base, M)
  // the kernel's PERSIST modes walk several tiles per workgroup: one workgroup per CU then (a multiple of 8, so
  // that a workgroup's tiles share its XCD)
  constexpr bool PERSIST = persistent_tiles(BM / WM / 32 * (BN / WN / 32), STAGGER, MODE);
  int grid = tiles_m * tiles_n * kslices;
  // (not with per-image keep counts: a workgroup that finds its tile without a live row leaves at once)
  if (PERSIST && slots > 0 && slots % 8 == 0 && grid > slots && !ep.k_rows) grid = slots;
  gemm_bf16_kernel<BM, BN, WM, WN, BK, NST, STAGGER, MODE><<<grid, WM * WN * 64, 0, st>>>(
      A, W, M, Nout, K, m_base, tiles_m, tiles_n, kslices, ep);
  return hipGetLastError();
}

// Second pass of a K-sliced launch: out = residual-epilogue(sum of the slices + bias) for rows [m_base, M);
// MODE is EPI_RESIDUAL (residual row = output row) or EPI_ATTN_OUT (residual row gathered through the kept indices).
// One thread per 8 output features.
template <int MODE>
__global__ __launch_bounds__(256) void gemm_reduce_kernel(const float* __restrict__ part, int kslices, int m_base,
                                                          int M, int Nout, EpiParams<bf16_t> ep) {
  const int cpr = Nout / 8;
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= (int64_t)(M - m_base) * cpr) return;
  const int row = m_base + (int)(v / cpr), col = (int)(v % cpr) * 8;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < kslices; ++s) {
    const float* p = part + ((int64_t)s * (M - m_base) + row - m_base) * Nout + col;
    const f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { acc[e] += a[e]; acc[4 + e] += b[e]; }
  }
  bf16x8 bias;
#pragma unroll
  for (int e = 0; e < 8; ++e) bias[e] = (bf16_t)0.f;
  if (ep.bias) bias = *reinterpret_cast<const bf16x8*>(ep.bias + col);
  int64_t roff = (int64_t)row * ep.ldo;
  if (MODE == EPI_ATTN_OUT) roff = ((int64_t)(row / ep.k) * ep.Ntok + min(max(ep.idx[row], 0), ep.Ntok - 1)) * ep.C;
  const bf16x8 r = *reinterpret_cast<const bf16x8*>(ep.res + roff + col);
  bf16x8 o;
  if (ep.gate) {
    const bf16x8 gt = *reinterpret_cast<const bf16x8*>(ep.gate + (int64_t)(row / ep.k) * ep.gate_pitch + col);
#pragma unroll
    for (int e = 0; e < 8; ++e)      // the projection (+ bias) is rounded to bf16 first, as in the fused epilogue
      o[e] = (bf16_t)fmaf((float)gt[e], (float)(bf16_t)(acc[e] + (float)bias[e]), (float)r[e]);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (bf16_t)((float)(bf16_t)(acc[e] + (float)bias[e]) + (float)r[e]);
  }
  *reinterpret_cast<bf16x8*>(ep.out + (int64_t)row * ep.ldo + col) = o;
}

// Tile configurations (NOVA_GEMM_CFG forces one, for tuning):
//   0: 128x128x64, 4 waves of 64x64, 2 LDS stages, two workgroups per CU
//   1: 256x256x64, 8 waves of 128x64, 2 stages
//   2: 256x128x64, 8 waves of 64x64, 3 stages
//   3: 64x32x64, 2 waves of 32x32, 6 stages, staggered K walk          (M <= 64)
//   4: 128x32x64, 4 waves of 32x32, 4 stages, staggered K walk         (M <= 256; M <= 512 for a narrow output and short K)
//   5: 128x128x64, 8 waves of 64x32, 3 stages, one workgroup per CU (two waves per SIMD hide the LDS waits that
//      four waves of 64x64 expose: 3-10 % faster at every shape measured)
//   6: 256x256x32, 8 waves of 128x64, 3 stages
// Without a forced choice the launcher prices the candidates 2, 5 and 6 with a small model fitted
// to measurements on MI355X (M = 1.6k..4.9k, N and K = 2k..8k): a launch takes
// ceil(tiles / CUs) rounds, a round costs the tile's flops at the rate one workgroup sustains when
// every CU holds one, plus a fixed prologue/epilogue time.  Large tiles win when their tile count
// fills whole rounds; the one-workgroup 128x128 kernel wins when there are few tiles (narrow
// outputs, late blocks with few kept tokens).
constexpr int kNumCfgs = 7;

struct Candidate {
  int cfg, bm, bn;
  double rate;   // flop/s of one resident workgroup with all CUs busy
};

static const Candidate kCands[] = {{2, 256, 128, 3.3e12}, {5, 128, 128, 3.2e12}, {6, 256, 256, 3.6e12}};
constexpr double kFixed = 8e-6;          // per round of workgroups: launch ramp, prologue, epilogue

// Modelled time of one launch over M rows with candidate c: whole rounds over the CUs, each a tile's flops at the
// candidate's sustained rate plus the fixed time.  A projection done by one launch of a single round that fills
// only a fraction f of the CUs is shorter (the busy CUs share L2 and memory with fewer others): taken as
// max(0.85, 1.1 f) of a whole round (`alone`).  Measured over the 32 blocks of the largest workload this helps the
// K = 2048 projections; for the parts of a two-launch plan it misleads and is not applied.  K = 8192 has its own fit.
double model_time(const Candidate& c, double slots, int M, int Nout, int K, bool alone = false) {
  const double tiles = (double)((M + c.bm - 1) / c.bm) * ((Nout + c.bn - 1) / c.bn);
  const double t_tile = 2.0 * c.bm * c.bn * K / c.rate;
  if (alone && K < 4096 && tiles < slots)   // a whole projection that fills only a fraction of the CUs
    return t_tile * std::max(0.85, std::min(1.0, 1.1 * tiles / slots)) + kFixed;
  // K = 8192 (the FFN down projection), one partly filled round: measured 99 ... 131 us for 80 ... 256 tiles of
  // 256 x 128 and 70 ... 79 us for 144 ... 256 tiles of 128 x 128, i.e. 0.8 of the fit above at a full round and
  // a weak dependence on the fill
  if (K >= 4096 && tiles < slots) return (t_tile + kFixed) * 0.8 * (0.65 + 0.35 * tiles / slots);
  return std::ceil(tiles / slots) * (t_tile + kFixed) * (K >= 4096 ? 0.8 : 1.0);
}

// Whether M rows of this projection go to the narrow-tile kernels (see pick_cfg).
bool narrow_tiles(int M, int Nout, int K) { return M <= 256 || (M <= 512 && Nout < 4096 && K < 4096); }

int pick_cfg(const nova_ctx* ctx, int M, int Nout, int K, double* t_out = nullptr, bool alone = true) {
  if (ctx && ctx->gemm_cfg >= 0 && ctx->gemm_cfg < kNumCfgs) return ctx->gemm_cfg;
  // few rows (the early, small scales): the weights are streamed once and the output has too few
  // large tiles to occupy the CUs, so narrow tiles spread the weight stream over many workgroups
  // (from 257 rows on only for a narrow output with a short K, the attention output projection: measured at 288 ...
  // 512 rows, 128 x 32 tiles against 128 x 128: QKV 32-35 / 27 us, FFN1 32-39 / 25-27 us, FFN2 45-49 / 28-34 us
  // (the latter with K slices), O-proj 17-19 / 23 us)
  if (M <= 64) return 3;
  if (narrow_tiles(M, Nout, K)) return 4;
  const double slots = ctx ? ctx->num_cus : 256;
  int best = 2;
  double best_t = 1e30;
  for (const Candidate& c : kCands) {
    const double t = model_time(c, slots, M, Nout, K, alone);
    if (t < best_t) { best_t = t; best = c.cfg; }
  }
  if (t_out) *t_out = best_t;
  return best;
}

// A launch plan: one configuration for all rows, or two launches -- typically (nearly) whole rounds of large
// tiles over the first rows and the best single configuration for the rows left over, so that only a small
// remainder pays for a ragged last round.  Returns the number of parts; part i covers rows [m_base[i], m_end[i]) with cfg[i].
struct Plan {
  int n;
  int m_base[2], m_end[2], cfg[2];
};
Plan plan_rows(const nova_ctx* ctx, int mode, int M, int Nout, int K) {
  Plan p;
  double t_single = 1e30;
  p.n = 1; p.m_base[0] = 0; p.m_end[0] = M; p.cfg[0] = pick_cfg(ctx, M, Nout, K, &t_single);
  const bool forced = ctx && ctx->gemm_cfg >= 0 && ctx->gemm_cfg < kNumCfgs;
  if (forced || mode == EPI_ENTROPY || M <= 512 || (ctx && ctx->gemm_parts == 0)) return p;   // one launch
  const int slots = ctx ? ctx->num_cus : 256;
  double best = t_single * 0.97;                          // a second launch has to pay for itself
  for (const Candidate& c : kCands) {
    for (int rows = 1; rows * c.bm < M; ++rows) {         // tile rows in the first part
      const int m1 = rows * c.bm;
      double t_rest = 0.0;
      const int cfg_rest = pick_cfg(ctx, M - m1, Nout, K, &t_rest, false);
      if (narrow_tiles(M - m1, Nout, K)) {
        // the narrow-tile kernels stream the weights once: measured 16 / 21 / 35 us for <= 128 / 256 / 512 rows of
        // a 2048 x 8192 projection, in proportion to the weight bytes, never under 15 us
        const int mr = M - m1;
        const double w_time = 2.0 * Nout * (double)K / 3.2e12 * (mr <= 128 ? 1.0 : mr <= 256 ? 1.45 : 3.0);
        t_rest = std::max(15e-6, 6e-6 + w_time) + (K >= 4096 ? 5e-6 : 0.0);
      }
      const double t = model_time(c, slots, m1, Nout, K) + t_rest + 3e-6;
      if (t < best) {
        best = t;
        p.n = 2;
        p.m_base[0] = 0; p.m_end[0] = m1; p.cfg[0] = c.cfg;
        p.m_base[1] = m1; p.m_end[1] = M; p.cfg[1] = cfg_rest;
      }
    }
  }
  return p;
}

template <int MODE>
hipError_t launch_part(hipStream_t st, int cfg, const bf16_t* A, const bf16_t* W, int m_base, int M, int Nout, int K,
                       const EpiParams<bf16_t>& ep, int slots, int cus, int ksplit) {
  if constexpr (MODE == EPI_RESIDUAL) {
    // A long K and a narrow output with large tiles (the FFN down projection once few tokens are kept): the tiles
    // fill less than half of the CUs.  K is cut into 2 or 4 slices summed by as many workgroups per tile, fp32
    // partial sums go to the scratch buffer and the second pass adds them and applies the epilogue.  The scratch
    // buffer holds 4 x rows x C floats, hence Nout == C and at most four slices.
    if ((cfg == 2 || cfg == 5 || cfg == 6) && ep.part && ksplit != 0 && K >= 4096 && Nout == ep.C && Nout % 8 == 0) {
      const int bm = cfg == 5 ? 128 : 256, bn = cfg == 6 ? 256 : 128, bk = cfg == 6 ? 32 : 64;
      const int tiles = ((M - m_base + bm - 1) / bm) * ((Nout + bn - 1) / bn);
      int ks = 1;
      if (ksplit > 0) ks = ksplit;
      else while (ks < 4 && tiles * ks * 2 <= cus) ks *= 2;
      if ((ks == 2 || ks == 4) && K % (ks * bk) == 0 && K / (ks * bk) >= 16 &&
          (int64_t)ks * (M - m_base) * Nout <= ep.part_floats) {
        hipError_t e;
        if (cfg == 2) e = launch_cfg<256, 128, 4, 2, 64, 3, false, EPI_PARTIAL>(st, A, W, m_base, M, Nout, K, ep, 0, ks);
        else if (cfg == 5) e = launch_cfg<128, 128, 2, 4, 64, 3, false, EPI_PARTIAL>(st, A, W, m_base, M, Nout, K, ep, 0, ks);
        else e = launch_cfg<256, 256, 2, 4, 32, 3, false, EPI_PARTIAL>(st, A, W, m_base, M, Nout, K, ep, 0, ks);
        if (e != hipSuccess) return e;
        const int64_t nvec = (int64_t)(M - m_base) * (Nout / 8);
        gemm_reduce_kernel<MODE><<<(unsigned)((nvec + 255) / 256), 256, 0, st>>>(ep.part, ks, m_base, M, Nout, ep);
        return hipGetLastError();
      }
    }
  }
  if constexpr (MODE == EPI_RESIDUAL || MODE == EPI_ATTN_OUT) {
    // Few rows and a narrow output (the two projections back to C of the small scales and of row remainders): a
    // tile column is one workgroup, too few to stream the weights at speed.  K is cut into slices summed by more
    // workgroups (at least eight K steps per slice); a second small pass adds the slices and applies the epilogue.
    const int wgs = ((M - m_base + (cfg == 3 ? 63 : 127)) / (cfg == 3 ? 64 : 128)) * ((Nout + 31) / 32);
    if ((cfg == 3 || cfg == 4) && ep.part && wgs <= 128 && K >= 2048 && K % (4 * 64) == 0 && Nout % 8 == 0 &&
        (int64_t)4 * (M - m_base) * Nout <= ep.part_floats) {
      const int ks = 4;
      const hipError_t e =
          cfg == 3 ? launch_cfg<64, 32, 2, 1, 64, 6, true, EPI_PARTIAL>(st, A, W, m_base, M, Nout, K, ep, 0, ks)
                   : launch_cfg<128, 32, 4, 1, 64, 4, true, EPI_PARTIAL>(st, A, W, m_base, M, Nout, K, ep, 0, ks);
      if (e != hipSuccess) return e;
      const int64_t nvec = (int64_t)(M - m_base) * (Nout / 8);
      gemm_reduce_kernel<MODE><<<(unsigned)((nvec + 255) / 256), 256, 0, st>>>(ep.part, ks, m_base, M, Nout, ep);
      return hipGetLastError();
    }
  }
  switch (cfg) {
    case 0: return launch_cfg<128, 128, 2, 2, 64, 2, false, MODE>(st, A, W, m_base, M, Nout, K, ep, slots);
    case 1: return launch_cfg<256, 256, 2, 4, 64, 2, false, MODE>(st, A, W, m_base, M, Nout, K, ep, slots);
    case 3: return launch_cfg<64, 32, 2, 1, 64, 6, true, MODE>(st, A, W, m_base, M, Nout, K, ep, slots);
    case 4: return launch_cfg<128, 32, 4, 1, 64, 4, true, MODE>(st, A, W, m_base, M, Nout, K, ep, slots);
    case 5: return launch_cfg<128, 128, 2, 4, 64, 3, false, MODE>(st, A, W, m_base, M, Nout, K, ep, slots);
    case 6: return launch_cfg<256, 256, 2, 4, 32, 3, false, MODE>(st, A, W, m_base, M, Nout, K, ep, slots);
    default: return launch_cfg<256, 128, 4, 2, 64, 3, false, MODE>(st, A, W, m_base, M, Nout, K, ep, slots);
  }
}

template <int MODE>
hipError_t launch_mode(const nova_ctx* ctx, hipStream_t st, const bf16_t* A, const bf16_t* W, int M, int Nout,
                       int K, const EpiParams<bf16_t>& ep) {
  const Plan p = plan_rows(ctx, MODE, M, Nout, K);
  for (int i = 0; i < p.n; ++i) {
    const int cus = ctx ? ctx->num_cus : 256;
    const hipError_t e = launch_part<MODE>(st, p.cfg[i], A, W, p.m_base[i], p.m_end[i], Nout, K, ep,
                                           (ctx && ctx->gemm_persist == 0) ? 0 : cus, cus,
                                           ctx ? ctx->gemm_ksplit : -1);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace

// Output columns per tile of the configuration launch_gemm_bf16 uses for this shape.
int gemm_bf16_tile_cols(const nova_ctx* ctx, int M, int Nout, int K) {
  switch (pick_cfg(ctx, M, Nout, K)) {
    case 0: case 5: return 128;
    case 1: case 6: return 256;
    case 3: case 4: return 32;
    default: return 128;
  }
}

hipError_t launch_gemm_bf16(const nova_ctx* ctx, hipStream_t st, int mode, const void* A, const void* W, int M,
                            int Nout, int K, const EpiParams<bf16_t>& ep) {
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* w = static_cast<const bf16_t*>(W);
  switch (mode) {
    case EPI_QKV: return launch_mode<EPI_QKV>(ctx, st, a, w, M, Nout, K, ep);
    case EPI_ATTN_OUT: return launch_mode<EPI_ATTN_OUT>(ctx, st, a, w, M, Nout, K, ep);
    case EPI_GELU: return launch_mode<EPI_GELU>(ctx, st, a, w, M, Nout, K, ep);
    case EPI_GELU_TANH: return launch_mode<EPI_GELU_TANH>(ctx, st, a, w, M, Nout, K, ep);
    case EPI_PLAIN: return launch_mode<EPI_PLAIN>(ctx, st, a, w, M, Nout, K, ep);
    case EPI_ENTROPY: return launch_mode<EPI_ENTROPY>(ctx, st, a, w, M, Nout, K, ep);
    default: return launch_mode<EPI_RESIDUAL>(ctx, st, a, w, M, Nout, K, ep);
  }
}
