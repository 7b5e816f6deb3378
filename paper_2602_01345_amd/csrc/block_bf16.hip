// bf16 matrix-core path of the pruned block (Sec. 3.3, "Residual Cache Reuse", first
// equation, evaluated on the kept rows only; Sec. 3.2: attention is the cost pruning saves).
//
//   gather+LN -> QKV GEMM (epilogue appends K/V to the caches) -> flash-style attention
//   -> O-proj GEMM (+ residual) -> LN -> FFN1 GEMM (+GELU) -> FFN2 GEMM (+ residual)
//
// GEMMs: y = u W^T with both operands K-contiguous, so every MFMA operand is one 16-byte
// LDS read.  v_mfma_f32_32x32x16_bf16, fp32 accumulate, 128x128x64 tiles, 4 waves (2x2) of
// 64x64, double-buffered LDS with the next tile's global loads in flight during the MFMAs.
//
// Attention: everything is computed transposed so that one lane owns one query column:
//   S^T = K Q^T   (A operand = key rows from LDS, B operand = query fragments in registers)
//   O^T += V^T P^T (A operand = value columns from LDS -- the value cache is stored key-minor
//                   for exactly this read -- B operand = the probabilities just computed,
//                   already sitting in the lane layout the MFMA wants)
// The online-softmax state (max, sum) is then one scalar per lane.
#include "common.h"
#include "epilogue.h"
#include "nova_internal.h"

namespace {

// ------------------------------------------------------------------------------------
// MFMA operand / result lane layout (wave64, 32x32x16 bf16):
//   A: lane l holds A[row = l % 32][k = 8 * (l / 32) + 0..7]
//   B: lane l holds B[k = 8 * (l / 32) + 0..7][col = l % 32]
//   D: lane l, register r holds D[row = 8 * (r / 4) + 4 * (l / 32) + r % 4][col = l % 32]
// ------------------------------------------------------------------------------------
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// =============================== attention =========================================
constexpr int ATT_THREADS = 256;     // 4 waves, 32 queries each
constexpr int ATT_BQ = 128;          // queries per workgroup
constexpr int ATT_BKV = 64;          // keys per LDS tile
constexpr int VPITCH = ATT_BKV + 8;  // value tile row pitch (elements)

// MFMA row i of a 32-key block reads key pi(i), chosen so that the 8 scores a lane ends up
// holding in registers 0..7 (and 8..15) belong to 8 consecutive keys: exactly the 8-key run the
// P^T operand of the second MFMA needs from that lane.
__device__ __forceinline__ int key_of_mfma_row(int i) {
  const int base = i & 16, t = i & 15;
  return base + 8 * ((t >> 2) & 1) + 4 * (t >> 3) + (t & 3);
}

template <int DH>
__global__ __launch_bounds__(ATT_THREADS) void attention_bf16_kernel(const bf16_t* __restrict__ q,
                                                                     const bf16_t* __restrict__ kc,
                                                                     const bf16_t* __restrict__ vc, int k, int C,
                                                                     int heads, int cap, int kv_total,
                                                                     float scale_log2, bf16_t* __restrict__ out) {
  constexpr int KPITCH = DH + 8;
  constexpr int KSTEPS = DH / 16;              // MFMAs along dh for S^T
  constexpr int DB = DH / 32;                  // 32-row blocks of O^T
  constexpr int KCH = ATT_BKV * DH / 8;        // 16-byte chunks in a key tile (= value tile)
  constexpr int CPT = KCH / ATT_THREADS;       // chunks per thread
  __shared__ __attribute__((aligned(16))) bf16_t Ks[2][ATT_BKV * KPITCH];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[2][DH * VPITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int head = blockIdx.y, b = blockIdx.z;
  const int64_t bh = (int64_t)b * heads + head;
  const bf16_t* Kg = kc + bh * cap * DH;              // [cap][DH]
  const bf16_t* Vg = vc + bh * DH * (int64_t)cap;     // [DH][cap]

  // this lane's query (clamped past the edge; such columns are never stored)
  const int qi = blockIdx.x * ATT_BQ + wave * 32 + col;
  const int qrow = min(qi, k - 1);
  const bf16_t* qp = q + ((int64_t)b * k + qrow) * C + head * DH + half * 8;
  bf16x8 qf[KSTEPS];
#pragma unroll
  for (int t = 0; t < KSTEPS; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(qp + t * 16);

  bf16x8 rk[CPT], rv[CPT];
  auto gload = [&](int key0) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + i * ATT_THREADS;
      // key tile: chunk c -> key c / (DH/8), part c % (DH/8); contiguous in memory
      rk[i] = *reinterpret_cast<const bf16x8*>(Kg + (int64_t)key0 * DH + (int64_t)c * 8);
      // value tile: chunk c -> dh row c / 8, 8 keys at (c % 8) * 8
      const int d = c >> 3, part = c & 7;
      bf16x8 v = *reinterpret_cast<const bf16x8*>(Vg + (int64_t)d * cap + key0 + part * 8);
      if (key0 + ATT_BKV > kv_total) {            // last tile: columns past the end must be exactly zero
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (key0 + part * 8 + e >= kv_total) v[e] = (bf16_t)0.0f;
      }
      rv[i] = v;
    }
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + i * ATT_THREADS;
      const int key = c / (DH / 8), kpart = c % (DH / 8);
      *reinterpret_cast<bf16x8*>(&Ks[buf][key * KPITCH + kpart * 8]) = rk[i];
      const int d = c >> 3, part = c & 7;
      *reinterpret_cast<bf16x8*>(&Vs[buf][d * VPITCH + part * 8]) = rv[i];
    }
  };

  f32x16 o[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
  float m_run = -INFINITY;     // running max of the raw scores (same in both half-lanes of a query)
  float l_run = 0.f;           // this lane's share of the running sum

  const int ntiles = (kv_total + ATT_BKV - 1) / ATT_BKV;
  gload(0);
  lstore(0);
  __syncthreads();
  const int krow_off = key_of_mfma_row(col) * KPITCH + half * 8;
  for (int t = 0; t < ntiles; ++t) {
    const int buf = t & 1, key0 = t * ATT_BKV;
    if (t + 1 < ntiles) gload(key0 + ATT_BKV);

    // ---- S^T tile: 64 keys x 32 queries, two 32-key blocks -------------------------
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[buf][kb * 32 * KPITCH + krow_off + ks * 16]);
        s[kb] = mfma32(a, qf[ks], s[kb]);
      }
    }
    // register r of block kb belongs to key  key0 + kb*32 + 16*(r/8) + 8*half + r%8
    float tmax = -INFINITY;
    const bool tail = key0 + ATT_BKV > kv_total;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (tail) {
          const int key = key0 + kb * 32 + 16 * (r >> 3) + 8 * half + (r & 7);
          s[kb][r] = key < kv_total ? s[kb][r] : -INFINITY;
        }
        tmax = fmaxf(tmax, s[kb][r]);
      }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, NOVA_WAVE));
    const float m_new = fmaxf(m_run, tmax);             // finite: every tile holds at least one valid key
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2);
    const float mb = m_new * scale_log2;
    float psum = 0.f;
    bf16x8 p[4];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float e = __builtin_amdgcn_exp2f(fmaf(s[kb][r], scale_log2, -mb));
        psum += e;
        p[kb * 2 + (r >> 3)][r & 7] = (bf16_t)e;
      }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[d][r] *= alpha;

    // ---- O^T += V^T P^T : DH rows x 32 queries, 4 groups of 16 keys -----------------
#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
      for (int d = 0; d < DB; ++d) {
        bf16x8 a = *reinterpret_cast<const bf16x8*>(&Vs[buf][(d * 32 + col) * VPITCH + g * 16 + half * 8]);
        o[d] = mfma32(a, p[g], o[d]);
      }
    }
    if (t + 1 < ntiles) lstore(buf ^ 1);
    __syncthreads();
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, NOVA_WAVE);
  const float inv = 1.0f / l_tot;
  if (qi < k) {
    bf16_t* op = out + ((int64_t)b * k + qi) * C + head * DH;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (bf16_t)(o[d][g * 4 + j] * inv);
        *reinterpret_cast<bf16x4*>(op + d * 32 + g * 8 + half * 4) = v;
      }
  }
}

}  // namespace

hipError_t launch_block_bf16(nova_ctx* ctx, hipStream_t st, const nova_block_shape& s,
                             const nova_block_weights& w, const void* xv, const int32_t* idx, void* kcv,
                             void* vcv, void* yv, const BlockWorkspace& ws) {
  const int M = s.B * s.k, C = s.C, F = s.C * s.ffn_mult, dh = s.C / s.heads;
  const bf16_t* x = static_cast<const bf16_t*>(xv);
  bf16_t* kc = static_cast<bf16_t*>(kcv);
  bf16_t* vc = static_cast<bf16_t*>(vcv);
  bf16_t* y = static_cast<bf16_t*>(yv);
  bf16_t* u = reinterpret_cast<bf16_t*>(ws.u);
  bf16_t* q = reinterpret_cast<bf16_t*>(ws.q);
  bf16_t* attn = reinterpret_cast<bf16_t*>(ws.attn);
  bf16_t* x1 = reinterpret_cast<bf16_t*>(ws.x1);
  bf16_t* hid = reinterpret_cast<bf16_t*>(ws.hid);

  hipError_t e;
  {
    StageTimer t(ctx, st, NOVA_STAGE_GATHER_LN);
    e = launch_gather_ln(st, NOVA_BF16, x, idx, M, s.k, s.N, C, u);
  }
  if (e != hipSuccess) return e;

  EpiParams<bf16_t> ep = {};
  ep.C = C; ep.heads = s.heads; ep.dh = dh; ep.cap = s.kv_capacity; ep.P = s.kv_len; ep.k = s.k;
  ep.idx = idx; ep.Ntok = s.N;

  ep.bias = static_cast<const bf16_t*>(w.b_qkv); ep.out = q; ep.ldo = C; ep.kc = kc; ep.vc = vc;
  {
    StageTimer t(ctx, st, NOVA_STAGE_QKV);
    e = launch_gemm_bf16(ctx, st, EPI_QKV, u, w.w_qkv, M, 3 * C, C, ep);
  }

  const int kv_total = s.kv_len + s.k;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)dh);
  dim3 agrid((s.k + ATT_BQ - 1) / ATT_BQ, s.heads, s.B);
  {
    StageTimer t(ctx, st, NOVA_STAGE_ATTENTION);
    if (dh == 64)
      attention_bf16_kernel<64><<<agrid, ATT_THREADS, 0, st>>>(q, kc, vc, s.k, C, s.heads, s.kv_capacity, kv_total,
                                                               scale_log2, attn);
    else
      attention_bf16_kernel<128><<<agrid, ATT_THREADS, 0, st>>>(q, kc, vc, s.k, C, s.heads, s.kv_capacity,
                                                                kv_total, scale_log2, attn);
  }

  ep.bias = static_cast<const bf16_t*>(w.b_o); ep.out = x1; ep.ldo = C; ep.res = x;
  {
    StageTimer t(ctx, st, NOVA_STAGE_OPROJ);
    e = launch_gemm_bf16(ctx, st, EPI_ATTN_OUT, attn, w.w_o, M, C, C, ep);
  }
  {
    StageTimer t(ctx, st, NOVA_STAGE_LN2);
    e = launch_gather_ln(st, NOVA_BF16, x1, nullptr, M, s.k, s.N, C, u);
  }
  if (e != hipSuccess) return e;

  ep.bias = static_cast<const bf16_t*>(w.b_fc1); ep.out = hid; ep.ldo = F;
  {
    StageTimer t(ctx, st, NOVA_STAGE_FFN1);
    e = launch_gemm_bf16(ctx, st, EPI_GELU, u, w.w_fc1, M, F, C, ep);
  }

  ep.bias = static_cast<const bf16_t*>(w.b_fc2); ep.out = y; ep.ldo = C; ep.res = x1;
  {
    StageTimer t(ctx, st, NOVA_STAGE_FFN2);
    e = launch_gemm_bf16(ctx, st, EPI_RESIDUAL, hid, w.w_fc2, M, C, F, ep);
  }
  return hipGetLastError();
}
