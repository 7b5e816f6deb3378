// Flash-style attention of the kept queries over the prior-scale KV cache plus the kept
// current keys (Sec. 3.3, "Residual Cache Reuse", first equation on the kept rows; Sec. 3.2:
// attention is the cost that pruning saves).  bf16 operands, fp32 softmax and accumulation.
//
// Everything is computed transposed so that one lane owns one query column:
//   S^T = K Q^T    A operand = key rows from LDS, B operand = query fragments held in registers
//   O^T += V^T P^T A operand = value-cache columns from LDS (the value cache is stored key-minor
//                  for exactly this read), B operand = the probabilities just computed, already
//                  sitting in the lane layout the MFMA wants
// so the online-softmax state (reference point and sum) is one scalar per lane and query group, and
// no data is exchanged between lanes except one max/sum swap between the two half-waves.
// The query rows arrive multiplied by (score scale * log2 e): the MFMA sums are scores in log2 units, the
// softmax reference enters as the accumulator input of the score MFMAs and moves only when a score lies far
// above it, so per score the common case is one exp2, one add and half a conversion (see the tile body).
//
// A workgroup is NW (4 or 8) waves; a wave owns NQ groups of 32 queries (every K / V fragment read from LDS
// feeds NQ MFMAs).  K and V tiles of 64 keys stream through an NST-stage LDS ring filled by
// direct global->LDS loads; the bank-conflict XOR swizzle is applied on the global side of those
// loads.  Workgroup ids are remapped so that all query blocks of one (batch row, head) run on the
// same XCD at about the same time and share that head's K/V in its L2.
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "nova_internal.h"

namespace {

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

#define WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

constexpr int BKV = 64;              // keys per tile
constexpr int kMaxSplit = 4;         // the partial-result workspace holds kMaxSplit partials per item on average; the
                                     // items of the last round alone are cut, into up to 16 key runs each

// MFMA row i of a 32-key block reads key pi(i), chosen so that the 8 scores a lane ends up holding
// in registers 0..7 (and 8..15) belong to 8 consecutive keys: exactly the 8-key run the P^T operand
// of the second MFMA needs from that lane.
__device__ __forceinline__ int key_of_mfma_row(int i) {
  const int base = i & 16, t = i & 15;
  return base + 8 * ((t >> 2) & 1) + 4 * (t >> 3) + (t & 3);
}

// byte offset of 16-byte chunk c of row r in a swizzled tile whose rows are ROWB bytes
template <int ROWB>
__device__ __forceinline__ int swz(int r, int c) {
  if (ROWB == 256) return r * 256 + ((c ^ (r & 15)) << 4);
  return r * 128 + ((c ^ ((r >> 1) & 7)) << 4);
}

template <int DH, int NQ, int NST, int OCC, int NW>
__global__ __launch_bounds__(NW * 64, OCC) void attention_bf16_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc, const bf16_t* __restrict__ vc, int k, int C,
    int heads, int cap, int kv_total_uniform, int nqb, int n_whole, int nsplit,
    bf16_t* __restrict__ out, float* __restrict__ part_o, float* __restrict__ part_ml,
    const int32_t* __restrict__ k_rows, const int32_t* __restrict__ kv_rows, int P, int self_keys) {
  constexpr int KROWB = DH * 2;                  // bytes per key row of the K tile
  constexpr int KCH = KROWB / 16;                // chunks per key row
  constexpr int K_BYTES = BKV * KROWB;
  constexpr int V_BYTES = DH * 128;              // DH rows of 64 keys
  constexpr int STAGE = K_BYTES + V_BYTES;
  constexpr int KSTEPS = DH / 16;                // MFMAs along dh for S^T
  constexpr int DB = DH / 32;                    // 32-row blocks of O^T
  constexpr int K_RPI = 1024 / KROWB;            // K rows filled per wave load instruction
  constexpr int LK = BKV / K_RPI / NW;    // K load instructions per wave per tile
  constexpr int LV = DH / 8 / NW;         // V load instructions per wave per tile (8 rows each)
  constexpr int LPW = LK + LV;
  constexpr int BQ = NW * NQ * 32;        // queries per workgroup
  static_assert((NST - 2) * LPW < 64, "vmcnt is a 6-bit counter");
  __shared__ __attribute__((aligned(1024))) char lds[NST * STAGE];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5, col = lane & 31;

  // ---- workgroup id -> item (batch row * heads + head, query block) and key split ---------------
  // The first n_whole workgroups take one item each over all keys (whole rounds over the CUs); the items
  // left over for the last, partly filled round are cut into nsplit equal runs of key tiles each, the runs
  // of an item being neighbours.  Within either group the ids are made XCD-contiguous (the hardware deals
  // consecutive workgroups to the 8 XCDs in turn), so that the query blocks of one (batch row, head) read
  // its keys and values through one L2.
  auto xcd_contiguous = [](int L, int n) {
    const int xcd = L & 7, j = L >> 3;
    return xcd * (n >> 3) + min(xcd, n & 7) + j;
  };
  const bool whole = (int)blockIdx.x < n_whole;
  const int pidx = whole ? 0 : xcd_contiguous(blockIdx.x - n_whole, gridDim.x - n_whole);   // index of the partial result
  const int item = whole ? xcd_contiguous(blockIdx.x, n_whole) : n_whole + pidx / nsplit;
  const int split = whole ? 0 : pidx % nsplit;
  const int nparts = whole ? 1 : nsplit;
  const int bh = item / nqb, qb = item - bh * nqb;
  const int b = bh / heads, head = bh - b * heads;
  const bf16_t* Kg = kc + (int64_t)bh * cap * DH;          // [cap][DH]
  const bf16_t* Vg = vc + (int64_t)bh * DH * (int64_t)cap; // [DH][cap]
  // Per-image keep counts: image b's queries are slots [0, kq) of its k-slot segment and its keys are its own
  // prior rows plus its own kq kept rows (self-attention; a cross-attention call has the same keys for every image).
  const int kq = image_count(k_rows, b, k);
  const int kv_total = self_keys && (k_rows || kv_rows) ? image_prior(kv_rows, b, P) + kq : kv_total_uniform;
  if (qb * (NW * NQ * 32) >= kq) {
    // no live query in this block (the whole workgroup leaves, before any barrier): an uncut item zeroes its
    // rows of the output, the rows of a cut item are zeroed by the merge pass
    if (whole) {
      constexpr int CPR = DH / 8;                            // 16-byte chunks per row of this head
      const int r0 = qb * (NW * NQ * 32), r1 = min(r0 + NW * NQ * 32, k);
      for (int i = tid; i < (r1 - r0) * CPR; i += NW * 64) {
        const int r = r0 + i / CPR, c = i % CPR;
        *reinterpret_cast<u32x4*>(out + ((int64_t)b * k + r) * C + head * DH + c * 8) = u32x4{0u, 0u, 0u, 0u};
      }
    }
    return;
  }

  // ---- query fragments (B operand): lane = query column, 8 dh elements per K step ----------
  bf16x8 qf[NQ][KSTEPS];
  int qi[NQ];
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    qi[g] = qb * BQ + (wave * NQ + g) * 32 + col;
    const int qrow = min(qi[g], kq - 1);                   // clamped past the last live query; never stored
    const bf16_t* qp = q + ((int64_t)b * k + qrow) * C + head * DH + half * 8;
#pragma unroll
    for (int t = 0; t < KSTEPS; ++t) qf[g][t] = *reinterpret_cast<const bf16x8*>(qp + t * 16);
  }

  // ---- global -> LDS fills -------------------------------------------------------------------
  const int klr = lane / KCH, klp = lane % KCH;            // K: row within the instruction, slot
  const int vlr = lane >> 3, vlp = lane & 7;               // V: 8 rows x 8 slots per instruction
  int koff[LK], voff[LV];                                  // element offsets from the tile origin
#pragma unroll
  for (int i = 0; i < LK; ++i) {
    const int r = (i * NW + wave) * K_RPI + klr;
    const int c = (swz<KROWB>(r, klp) - r * KROWB) >> 4;
    koff[i] = r * DH + c * 8;
  }
#pragma unroll
  for (int i = 0; i < LV; ++i) {
    const int r = (i * NW + wave) * 8 + vlr;
    const int c = (swz<128>(r, vlp) - r * 128) >> 4;
    voff[i] = r * cap + c * 8;                             // row r of the tile is dh index r
  }
  auto issue = [&](int stage, int key0) {
    char* sk = lds + stage * STAGE;
    char* sv = sk + K_BYTES;
    const bf16_t* kt = Kg + (int64_t)key0 * DH;
    const bf16_t* vt = Vg + key0;
#pragma unroll
    for (int i = 0; i < LK; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(kt + koff[i]), (lptr_t)(sk + (i * NW + wave) * 1024), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < LV; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(vt + voff[i]), (lptr_t)(sv + (i * NW + wave) * 1024), 16, 0, 0);
  };
  // The last tile may reach past the valid keys.  Scores of those keys are masked below; the value
  // columns must be exactly zero (0 * garbage could be NaN), so the wave that filled a row zeroes
  // the invalid tail of that row once its own fill has landed.
  auto zero_value_tail = [&](int stage, int key0) {
    char* sv = lds + stage * STAGE + K_BYTES;
    const int first_bad = kv_total - key0;                 // 1..63 here
#pragma unroll
    for (int i = 0; i < LV; ++i) {
      const int r = (i * NW + wave) * 8 + vlr;
      for (int key = first_bad + vlp; key < BKV; key += 8)
        *reinterpret_cast<bf16_t*>(sv + swz<128>(r, key >> 3) + (key & 7) * 2) = (bf16_t)0.0f;
    }
  };

  f32x16 o[NQ][DB];
#pragma unroll
  for (int g = 0; g < NQ; ++g)
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[g][d][r] = 0.f;
  // Softmax state per query (= per lane).  The query rows arrive multiplied by (score scale * log2 e), so the
  // MFMA sums are scores in log2 units.  m_run is the reference point the probabilities are taken against,
  // 2^(score - m_run); neg_m holds -m_run in all 16 registers of an accumulator block and is the accumulator
  // input of the first score MFMA of every tile, so the scores come out of the matrix core with the reference
  // already subtracted.  Reference 0 until the first tile has set it.
  float m_run[NQ], l_run[NQ];
  f32x16 neg_m[NQ];
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    m_run[g] = 0.f; l_run[g] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) neg_m[g][r] = 0.f;
  }

  // this workgroup's run of key tiles [t_begin, t_end)
  const int ntiles_all = (kv_total + BKV - 1) / BKV;
  const int tps = (ntiles_all + nparts - 1) / nparts;
  const int t_begin = split * tps;
  const int ntiles = min(ntiles_all, t_begin + tps);       // exclusive end
  if (t_begin >= ntiles_all) {
    // an empty key run (only with per-image counts: this image has fewer key tiles than the launch was planned
    // for): an all-zero partial with reference -inf, which the merge pass weighs with 0.  Leaves before any barrier.
#pragma unroll
    for (int g = 0; g < NQ; ++g) {
      if (qi[g] >= kq) continue;
      const int64_t prow = (int64_t)pidx * BQ + (qi[g] - qb * BQ);
      for (int d = half * (DH / 2); d < (half + 1) * (DH / 2); d += 4)
        *reinterpret_cast<f32x4*>(part_o + prow * DH + d) = f32x4{0.f, 0.f, 0.f, 0.f};
      if (half == 0) { part_ml[prow * 2] = -INFINITY; part_ml[prow * 2 + 1] = 0.f; }
    }
    return;
  }
#pragma unroll
  for (int t = 0; t < NST - 1; ++t)
    if (t_begin + t < ntiles) issue(t, (t_begin + t) * BKV);
  if (ntiles - t_begin >= NST - 1) { WAIT_VMCNT((NST - 2) * LPW); } else { WAIT_VMCNT(0); }
  if (t_begin + 1 == ntiles_all && kv_total < ntiles_all * BKV) zero_value_tail(0, t_begin * BKV);
  __syncthreads();

  // The last query block of an (image, head) is ragged: waves with no kept query leave the matrix core and the
  // vector units to the other workgroup of the CU.
  const bool wave_live = qb * BQ + wave * NQ * 32 < kq;
  // A-operand row of this lane inside a 32-key block (see key_of_mfma_row)
  const int krow = key_of_mfma_row(col);
  // One 64-key tile.  TAIL (last tile only) masks the scores of keys past kv_total.  stage_v is the ring stage
  // the tile sits in: a compile-time constant with a two-stage ring (the tile loop is unrolled by two, so that
  // every LDS address is a per-lane offset plus an immediate), a run-time value otherwise.
  auto tile_body = [&](auto tail_tag, auto stage_v, int t) {
    constexpr bool TAIL = decltype(tail_tag)::value;
    const int stage = stage_v;
    const int fill = stage == 0 ? NST - 1 : stage - 1;    // the stage freed by the previous tile
    const int key0 = t * BKV;
    const bool more = t + NST - 1 < ntiles;
    if (more) issue(fill, (t + NST - 1) * BKV);
    const char* sk = lds + stage * STAGE;
    const char* sv = sk + K_BYTES;

    if (wave_live) {   // a wave whose queries all lie past the last kept row only helps to fill and to synchronise
    // ---- S^T tile: 64 keys x 32 queries per group, two 32-key blocks -------------------------
    // Key fragments travel through a two-deep register ring of GF fragments.  The schedule is
    // pinned: first MFMA of a group, then the LDS reads of the next group, then the group's other
    // MFMAs -- so the wait in front of the next group finds its fragments (almost) landed.
    constexpr int NF = 2 * KSTEPS;            // fragments per tile; fragment f = (kb = f / KSTEPS, ks = f % KSTEPS)
    constexpr int GF = 4;                     // fragments per group
    static_assert(NF % GF == 0, "groups tile the fragments");
    f32x16 s[NQ][2];
    bf16x8 kf[2][GF];
    auto read_k = [&](int buf, int f0) {
#pragma unroll
      for (int i = 0; i < GF; ++i) {
        const int f = f0 + i;
        kf[buf][i] = *reinterpret_cast<const bf16x8*>(sk + swz<KROWB>((f / KSTEPS) * 32 + krow, (f % KSTEPS) * 2 + half));
      }
    };
    auto mfma_k = [&](int buf, int f0, int lo, int hi) {
#pragma unroll
      for (int i = 0; i < GF; ++i)
        if (i >= lo && i < hi) {
          const int f = f0 + i;
#pragma unroll
          for (int g = 0; g < NQ; ++g)
            s[g][f / KSTEPS] = mfma32(kf[buf][i], qf[g][f % KSTEPS], f % KSTEPS == 0 ? neg_m[g] : s[g][f / KSTEPS]);
        }
    };
    read_k(0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int grp = 0; grp < NF / GF; ++grp) {
      mfma_k(grp & 1, grp * GF, 0, 1);
      __builtin_amdgcn_sched_barrier(0);
      if (grp + 1 < NF / GF) read_k((grp + 1) & 1, (grp + 1) * GF);
      __builtin_amdgcn_sched_barrier(0);
      mfma_k(grp & 1, grp * GF, 1, GF);
      __builtin_amdgcn_sched_barrier(0);
    }

    // Value fragments go through the same kind of register ring: one group = four fragments = the DB fragments
    // of 4 / DB runs of 16 keys.  The first group is requested here, so that it lands behind the softmax
    // arithmetic.
    constexpr int KGG = 4 / DB;               // key runs per group
    constexpr int NG = 4 / KGG;               // groups per tile
    bf16x8 vf[2][4];
    bf16x8 p[NQ][4];                          // probabilities, in the B-operand layout of the value MFMAs
    auto read_v = [&](int buf, int grp) {
#pragma unroll
      for (int f = 0; f < 4; ++f) {
        const int kg = grp * KGG + f / DB, d = f % DB;
        vf[buf][f] = *reinterpret_cast<const bf16x8*>(sv + swz<128>(d * 32 + col, kg * 2 + half));
      }
    };
    auto mfma_v = [&](int buf, int grp, int lo, int hi) {
#pragma unroll
      for (int f = 0; f < 4; ++f)
        if (f >= lo && f < hi) {
          const int kg = grp * KGG + f / DB, d = f % DB;
#pragma unroll
          for (int g = 0; g < NQ; ++g) o[g][d] = mfma32(vf[buf][f], p[g][kg], o[g][d]);
        }
    };
    // (only where the register budget allows it: one query group per wave and at most two workgroups per CU;
    // otherwise the fragments are read in front of their MFMAs)
    constexpr bool VRING = NQ == 1 && OCC <= 2;
    if constexpr (VRING) {
      read_v(0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }

    // ---- online softmax; register r of block kb is key key0 + kb*32 + 16*(r/8) + 8*half + r%8 ---
    // s holds score - m_run.  m_run is a reference point, not necessarily the maximum: the tile's
    // probabilities 2^s are taken against it as it stands, and only when a lane's sum of them says that some
    // score lies far above it -- or on the first tile of the run, which sets it -- is the true maximum of the
    // tile computed, the accumulators rescaled and the tile's probabilities taken again.  Any common
    // reference cancels in o / l at the end; a term of at most kBig keeps every sum far inside the fp32
    // range.  In the common case the softmax is one exp2, one add and half a conversion per score.
    constexpr float kBig = 1024.0f;
#pragma unroll
    for (int g = 0; g < NQ; ++g) {
      if (TAIL) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + kb * 32 + 16 * (r >> 3) + 8 * half + (r & 7);
            s[g][kb][r] = key < kv_total ? s[g][kb][r] : -INFINITY;
          }
      }
      float psum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float e = __builtin_amdgcn_exp2f(s[g][kb][r]);
          psum += e;
          p[g][kb * 2 + (r >> 3)][r & 7] = (bf16_t)e;
        }
      const bool first = t == t_begin;
      if (__any(!(psum <= kBig)) || first) {    // !(<=) is also true for inf and NaN
        float tmax = -INFINITY;                 // of score - m_run
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[g][kb][r]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, NOVA_WAVE));    // finite: every tile holds a valid key
        // the reference moves by shift >= 0 (on the first tile: to the tile's maximum, whatever its sign;
        // nothing has been accumulated yet, so there is nothing to rescale)
        const float shift = first ? tmax : fmaxf(tmax, 0.f);
        const float alpha = first ? 0.f : __builtin_amdgcn_exp2f(-shift);
        l_run[g] *= alpha;
#pragma unroll
        for (int d = 0; d < DB; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[g][d][r] *= alpha;
        m_run[g] += shift;
#pragma unroll
        for (int r = 0; r < 16; ++r) neg_m[g][r] = -m_run[g];
        psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float e = __builtin_amdgcn_exp2f(s[g][kb][r] - shift);
            psum += e;
            p[g][kb * 2 + (r >> 3)][r & 7] = (bf16_t)e;
          }
      }
      l_run[g] += psum;
    }

    // ---- O^T += V^T P^T : DH rows x 32 queries per group, 4 runs of 16 keys --------------------
    // pinned like the score MFMAs: first MFMA of a run, the reads of the next run, the run's other MFMAs
    if constexpr (VRING) {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int grp = 0; grp < NG; ++grp) {
        mfma_v(grp & 1, grp, 0, 1);
        __builtin_amdgcn_sched_barrier(0);
        if (grp + 1 < NG) read_v((grp + 1) & 1, grp + 1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_v(grp & 1, grp, 1, 4);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int grp = 0; grp < NG; ++grp) {
        read_v(0, grp);
        mfma_v(0, grp, 0, 4);
      }
    }
    }   // wave_live

    // tile t+1 must have landed; this wave's LDS reads of the current stage must be complete
    if (more) { WAIT_VMCNT((NST - 2) * LPW); } else { WAIT_VMCNT(0); }
    if (t + 2 == ntiles_all && (t + 2) * BKV > kv_total) zero_value_tail(stage + 1 == NST ? 0 : stage + 1, (t + 1) * BKV);
    __builtin_amdgcn_s_waitcnt(0xC07F);     // lgkmcnt(0)
    // a bare barrier: __syncthreads() would also wait for the tiles requested for later iterations
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
  if constexpr (NST == 2) {
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    int t = t_begin;
    for (; t + 2 < ntiles; t += 2) {
      tile_body(std::false_type{}, S0{}, t);
      tile_body(std::false_type{}, S1{}, t + 1);
    }
    if (t + 2 == ntiles) {
      tile_body(std::false_type{}, S0{}, t);
      tile_body(std::true_type{}, S1{}, t + 1);
    } else {
      tile_body(std::true_type{}, S0{}, t);
    }
  } else {
    int stage = 0;
    for (int t = t_begin; t + 1 < ntiles; ++t) {
      tile_body(std::false_type{}, stage, t);
      stage = stage + 1 == NST ? 0 : stage + 1;
    }
    tile_body(std::true_type{}, stage, ntiles - 1);
  }

#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    const float l_tot = l_run[g] + __shfl_xor(l_run[g], 32, NOVA_WAVE);
    if (qi[g] >= k) continue;
    const int64_t row = (int64_t)b * k + qi[g];
    if (qi[g] >= kq) {
      // a slot past this image's keep count: zeros (an uncut item; the merge pass does it for cut ones)
      if (nparts == 1) {
        bf16_t* op = out + row * C + head * DH;
#pragma unroll
        for (int d = 0; d < DB; ++d)
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) *reinterpret_cast<u32x2*>(op + d * 32 + r4 * 8 + half * 4) = u32x2{0u, 0u};
      }
      continue;
    }
    if (nparts == 1) {
      const float inv = 1.0f / l_tot;
      bf16_t* op = out + row * C + head * DH;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (bf16_t)(o[g][d][r4 * 4 + e] * inv);
          *reinterpret_cast<bf16x4*>(op + d * 32 + r4 * 8 + half * 4) = v;
        }
    } else {
      // unnormalised partial sums of this key split, [partial][query of the block][DH], merged by
      // attention_combine_kernel
      const int64_t prow = (int64_t)pidx * BQ + (qi[g] - qb * BQ);
      float* po = part_o + prow * DH;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = o[g][d][r4 * 4 + e];
          *reinterpret_cast<f32x4*>(po + d * 32 + r4 * 8 + half * 4) = v;
        }
      if (half == 0) {
        float* pm = part_ml + prow * 2;
        pm[0] = m_run[g];
        pm[1] = l_tot;
      }
    }
  }
}

// Merge of the key splits of the items that were cut: out = sum_s w_s O_s / sum_s w_s l_s with
// w_s = 2^((m_s - max_s m_s) c).  The partials of cut item i (counted from n_whole) are [nsplit][BQ][DH] from
// partial index i * nsplit on.  One thread per 4 output features; a workgroup covers kCombineRows queries
// of one item.
constexpr int kCombineRows = 8;
template <int DH, int BQ>
__global__ __launch_bounds__(kCombineRows * (DH / 4)) void attention_combine_kernel(
    const float* __restrict__ part_o, const float* __restrict__ part_ml, int k, int C, int heads, int nqb,
    int n_whole, int nsplit, bf16_t* __restrict__ out, const int32_t* __restrict__ k_rows) {
  constexpr int CHUNKS = BQ / kCombineRows;                         // workgroups per item
  const int ci = blockIdx.x / CHUNKS, chunk = blockIdx.x - ci * CHUNKS;
  const int item = n_whole + ci;
  const int bh = item / nqb, qb = item - bh * nqb;
  const int b = bh / heads, head = bh - b * heads;
  const int qr = chunk * kCombineRows + threadIdx.x / (DH / 4);     // query of the block
  const int c = (threadIdx.x % (DH / 4)) * 4;
  const int qrow = qb * BQ + qr;
  if (qrow >= k) return;
  if (qrow >= image_count(k_rows, b, k)) {                          // a slot past its image's keep count: zeros
    *reinterpret_cast<u32x2*>(out + ((int64_t)b * k + qrow) * C + head * DH + c) = u32x2{0u, 0u};
    return;
  }
  const int64_t p0 = (int64_t)ci * nsplit;                          // first partial of this item
  float mmax = -INFINITY;
  for (int s = 0; s < nsplit; ++s) mmax = fmaxf(mmax, part_ml[((p0 + s) * BQ + qr) * 2]);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float* pm = part_ml + ((p0 + s) * BQ + qr) * 2;
    const float w = __builtin_amdgcn_exp2f(pm[0] - mmax);        // references are in log2 units
    l = fmaf(w, pm[1], l);
    const f32x4 o = *reinterpret_cast<const f32x4*>(part_o + ((p0 + s) * BQ + qr) * DH + c);
    acc += w * o;
  }
  const float inv = 1.0f / l;
  bf16x4 r;
#pragma unroll
  for (int e = 0; e < 4; ++e) r[e] = (bf16_t)(acc[e] * inv);
  *reinterpret_cast<bf16x4*>(out + ((int64_t)b * k + qrow) * C + head * DH + c) = r;
}

template <int DH, int NQ, int NST, int OCC, int NW>
hipError_t launch_cfg(const nova_ctx* ctx, hipStream_t st, const bf16_t* q, const bf16_t* kc, const bf16_t* vc, int B,
                      int k, int C, int heads, int cap, int kv_total, bf16_t* out, float* part_o,
                      float* part_ml, int64_t part_floats, const int32_t* k_rows, const int32_t* kv_rows, int P,
                      int self_keys) {
  constexpr int BQ = NW * NQ * 32;
  const int nqb = (k + BQ - 1) / BQ;
  const int items = nqb * heads * B;                      // (batch row, head, query block)
  const int slots = (ctx ? ctx->num_cus : 256) * OCC;
  const int ntiles = (kv_total + BKV - 1) / BKV;
  // Items are equally long, so whole rounds over the workgroup slots run uncut; only the last, partly filled
  // round is worth cutting into runs of key tiles (finer granularity at the price of partial results for those
  // items and a small merge pass).  Its time is modelled in units of one item with every slot busy.  Measured:
  // a workgroup that has its CU to itself runs kSolo times faster, and partial results cost about 5 % of an
  // item per extra run for the share of the rows that has them.  Three ways to run the last round:
  //   (i)   uncut;
  //   (ii)  every item cut into s runs;
  //   (iii) two resident workgroups per CU only: one uncut item per CU first, the others cut into s runs that
  //         fill the second slots (and leave the uncut workgroup alone on its CU once they are done).
  // The partial workspace holds part_floats / (BQ * DH) partial results.
  constexpr float kSolo = 1.8f;
  int n_whole = items, nsplit = 1;
  if (part_o && part_ml) {
    const int cus = slots / OCC;
    const int rest = items % slots;                       // items of the last round (0: nothing to cut)
    auto usable = [&](int s, int cut) {                   // every run owns at least one tile; partials fit
      return s >= 1 && (s - 1) * ((ntiles + s - 1) / s) < ntiles && (int64_t)cut * s * BQ * DH <= part_floats;
    };
    if (rest > 0) {
      float best = rest <= cus ? 1.0f / kSolo : 1.0f;     // (i)
      int best_whole = rest;                              // uncut items of the last round
      const int forced = ctx && ctx->attn_split >= 2 ? ctx->attn_split : 0;
      if (forced) best = 1e30f;
      for (int s = forced ? forced : 2; s <= (forced ? forced : 16); ++s) {
        if (!forced && ntiles / s < 8) break;
        if (usable(s, rest)) {                            // (ii)
          const int pieces = rest * s;
          const float run = pieces <= cus ? 1.0f / (s * kSolo) : (float)((pieces + slots - 1) / slots) / s;
          const float cost = run + 0.05f * (s - 1) * (float)rest / (float)items;
          if (cost < best - 1e-6f) { best = cost; nsplit = s; best_whole = 0; }
        }
        if (OCC == 2 && rest > cus && usable(s, rest - cus)) {   // (iii)
          const float paired = (float)(((rest - cus) * s + cus - 1) / cus) / s;    // second-slot time of the busiest CU
          const float run = paired <= 1.0f ? paired + (1.0f - paired) / kSolo : 1.0f + (paired - 1.0f) / kSolo;
          const float cost = run + 0.05f * (s - 1) * (float)(rest - cus) / (float)items;
          if (cost < best - 1e-6f) { best = cost; nsplit = s; best_whole = cus; }
        }
      }
      if (nsplit > 1) n_whole = items - rest + best_whole;
    }
  }
  const int grid = n_whole + (items - n_whole) * nsplit;
  attention_bf16_kernel<DH, NQ, NST, OCC, NW><<<grid, NW * 64, 0, st>>>(
      q, kc, vc, k, C, heads, cap, kv_total, nqb, n_whole, nsplit, out, part_o, part_ml, k_rows, kv_rows, P, self_keys);
  if (nsplit > 1)
    attention_combine_kernel<DH, BQ><<<(items - n_whole) * (BQ / kCombineRows), kCombineRows * (DH / 4), 0, st>>>(
        part_o, part_ml, k, C, heads, nqb, n_whole, nsplit, out, k_rows);
  return hipGetLastError();
}

}  // namespace

int attention_max_split() { return kMaxSplit; }

hipError_t launch_attention_bf16(const nova_ctx* ctx, hipStream_t st, const void* qv, const void* kcv,
                                 const void* vcv, int B, int k, int C, int heads, int cap, int kv_total,
                                 void* outv, float* part_o, float* part_ml, int64_t part_floats,
                                 const int32_t* k_rows, const int32_t* kv_rows, int P, int self_keys) {
  const bf16_t* q = static_cast<const bf16_t*>(qv);
  const bf16_t* kc = static_cast<const bf16_t*>(kcv);
  const bf16_t* vc = static_cast<const bf16_t*>(vcv);
  bf16_t* out = static_cast<bf16_t*>(outv);
  const int dh = C / heads;
  // One group of 32 queries per wave (two workgroups per CU, so that one wave's softmax overlaps
  // another wave's MFMAs); two groups per wave (half the LDS reads per MFMA, one workgroup per
  // CU) can be forced for tuning.
  int nq = ctx ? ctx->attn_cfg : -1;
  // 1: 4 waves x 32 queries, two workgroups per CU (default); 2: 4 waves x 64 queries; 3: 8 waves x 32 queries,
  // deeper ring; 4 (dh = 64 only): as 1 with three workgroups per CU and no value-fragment ring
  if (nq < 1 || nq > 4) nq = 1;
#define ATT_LAUNCH(DH_, NQ_, NST_, OCC_, NW_)                                                                       \
  return launch_cfg<DH_, NQ_, NST_, OCC_, NW_>(ctx, st, q, kc, vc, B, k, C, heads, cap, kv_total, out, \
                                               part_o, part_ml, part_floats, k_rows, kv_rows, P, self_keys)
  if (dh == 64) {
    if (nq == 1) ATT_LAUNCH(64, 1, 2, 2, 4);
    if (nq == 4) ATT_LAUNCH(64, 1, 2, 3, 4);
    if (nq == 3) ATT_LAUNCH(64, 1, 4, 2, 8);
    ATT_LAUNCH(64, 2, 3, 1, 4);
  }
  if (nq == 1) ATT_LAUNCH(128, 1, 2, 2, 4);
  if (nq == 3) ATT_LAUNCH(128, 1, 3, 1, 8);
  ATT_LAUNCH(128, 2, 3, 1, 4);
#undef ATT_LAUNCH
}
