// Per-row state and row walk of the token-entropy reduction (Sec. 3.3, "Adaptive Acceleration Activation", entropy
// equation), used by the entropy kernels in entropy.hip.
//
// With S = sum_v e^{x_v - m} and T = sum_v (m - x_v) e^{x_v - m}:  H = ln S + T / S.  Both terms are non-negative, so
// nothing cancels.  To keep relative accuracy when H is tiny (one dominant logit) the elements equal to the running
// maximum m are counted, not summed: S = cnt + R with R = sum over x_v < m, and H = log1p(R + cnt - 1) + T / (R + cnt).
#pragma once
#include "common.h"

namespace entropy_core {

constexpr int kWavesPerBlock = 4;
constexpr int kWavesPerSimd = 3;   // resident waves per SIMD the grid is sized for (measured best of 1..8)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kClamp = -200.0f;   // e^-200 == 0 in fp32; keeps (m - x) * e finite for x = -inf
constexpr float kClampNat = -140.0f; // likewise for the per-element path (natural units; 2^(-140 log2 e) flushes to 0)


// Wave-wide sum / maximum on the DPP cross-lane paths of the vector ALU (quads, half rows, rows of 16, then the two
// row broadcasts), read back from lane 63 as a wave-uniform scalar: six dependent vector instructions and no trip
// through the LDS crossbar, which is what a butterfly of lane shuffles costs six times over.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_or(float v, float identity) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum_uniform(float v) {
  v += dpp_or<0xB1, 0xF>(v, 0.0f);          // quad_perm [1,0,3,2]
  v += dpp_or<0x4E, 0xF>(v, 0.0f);          // quad_perm [2,3,0,1]
  v += dpp_or<0x141, 0xF>(v, 0.0f);         // row_half_mirror
  v += dpp_or<0x140, 0xF>(v, 0.0f);         // row_mirror: every lane holds the sum of its row of 16
  v += dpp_or<0x142, 0xA>(v, 0.0f);         // row_bcast15 into rows 1 and 3
  v += dpp_or<0x143, 0xC>(v, 0.0f);         // row_bcast31 into rows 2 and 3: lane 63 holds the total
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max_uniform(float v) {
  v = fmaxf(v, dpp_or<0xB1, 0xF>(v, -INFINITY));
  v = fmaxf(v, dpp_or<0x4E, 0xF>(v, -INFINITY));
  v = fmaxf(v, dpp_or<0x141, 0xF>(v, -INFINITY));
  v = fmaxf(v, dpp_or<0x140, 0xF>(v, -INFINITY));
  v = fmaxf(v, dpp_or<0x142, 0xA>(v, -INFINITY));
  v = fmaxf(v, dpp_or<0x143, 0xC>(v, -INFINITY));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// ln(1 + x) for x >= 0 to a few fp32 ulps, on the native log2 unit: a short alternating series where 1 + x would
// round away most of x, else ln(u) with u = fl(1 + x) plus the first-order term for what that rounding dropped.
__device__ __forceinline__ float log1p_pos(float x) {
  if (x < 0.0625f) {
    float p = fmaf(x, 1.0f / 7.0f, -1.0f / 6.0f);
    p = fmaf(p, x, 1.0f / 5.0f);
    p = fmaf(p, x, -1.0f / 4.0f);
    p = fmaf(p, x, 1.0f / 3.0f);
    p = fmaf(p, x, -1.0f / 2.0f);
    p = fmaf(p, x, 1.0f);
    return p * x;                              // next term x^8 / 8: below 2e-10 of the result
  }
  const float u = 1.0f + x;
  const float lost = x - (u - 1.0f);
  return fmaf(__builtin_amdgcn_logf(u), 0.6931471805599453f, lost * __builtin_amdgcn_rcpf(u));
}

struct Row {
  float m;        // running maximum, wave uniform (-inf before the first element)
  float R, T;     // per-lane partial sums against m, excluding elements equal to m
  float cS, cT;   // wave-uniform sums of elements that once equalled the maximum
  int cnt;        // wave-uniform count of elements equal to the current m
  bool nan;       // wave-uniform: a NaN logit has been seen (the row's entropy is NaN)

  __device__ __forceinline__ void init() { m = -INFINITY; R = T = cS = cT = 0.f; cnt = 0; nan = false; }

  // new wave-uniform maximum M >= every element seen so far and in the coming chunk
  __device__ __forceinline__ void rebase(float M) {
    if (M > m) {
      if (m != -INFINITY) {
        float d = m - M;                                 // < 0
        float dc = (d < kClamp) ? kClamp : d;
        float f = __builtin_amdgcn_exp2f(dc * kLog2e);
        // every earlier term e^{x-m} becomes f e^{x-m}; (m-x) grows by -d
        T = f * fmaf(-dc, R, T);
        R = f * R;
        float S_old = cS + (float)cnt;
        cT = f * fmaf(-dc, S_old, cT);
        cS = f * S_old;
        cnt = 0;
      }
      m = M;
    }
  }

  __device__ __forceinline__ void add(float x) {
    const float d = x - m;                    // <= 0; exactly 0 for an element equal to m; -inf for x = -inf
    // counted on the scalar unit.  "not less than 0" is "equal to 0" for every number and also true for NaN: a NaN
    // logit shows up as an unexpected count, which sends the chunk through a NaN check (walk_rows)
    cnt += __popcll(__ballot(!(d < 0.0f)));
    // One integer minimum on the bit pattern does three things: non-positive floats order as integers the other way
    // round (more negative float = larger integer) and +0 is integer 0, the largest of all, so min(bits(d),
    // bits(-140)) maps d = 0 (an element equal to m: counted, not summed) and every d < -140 (-inf included) to -140
    // and leaves the rest alone; e^-140 is 0 in fp32 (so are all terms below e^-104), and -140 * 0 is 0 where
    // -inf * 0 would be NaN.  A NaN is mapped as well: NaN logits are caught through the count (see above).
    const float dc = __int_as_float(min(__float_as_int(d), __float_as_int(kClampNat)));
    const float e = __builtin_amdgcn_exp2f(dc * kLog2e);
    R += e;
    T = fmaf(-dc, e, T);                      // (m - x) e^{x - m}
  }

  // lanes that must not contribute (tail) call this instead, keeping ballots uniform
  __device__ __forceinline__ void add_masked(float x, bool valid) {
    float d = x - m;
    d = (d < kClamp) ? kClamp : d;
    bool is_max = valid && (d == 0.0f);
    float e = __builtin_amdgcn_exp2f(d * kLog2e);
    cnt += __popcll(__ballot(is_max));
    e = (is_max || !valid) ? 0.0f : e;
    float t = valid ? -d : 0.0f;
    R += e;
    T = fmaf(t, e, T);
  }

  __device__ __forceinline__ float finish() const {
    float Rw = wave_sum_uniform(R) + cS;
    float Tw = wave_sum_uniform(T) + cT;
    // S = cnt + Rw, one maximum instance split off for log1p
    float extra = Rw + (float)(cnt - 1);
    float H = log1p_pos(extra) + Tw * __builtin_amdgcn_rcpf(1.0f + extra);
    // empty or all -inf row, a +inf logit (inf - inf): undefined; NaN logit
    if (m == -INFINITY || m == INFINITY || cnt < 1 || nan) H = __builtin_nanf("");
    return (H < 0.0f) ? 0.0f : H;                             // NaN passes through
  }
};

// Regular rows (every lane owns CH full 16-byte vectors in every chunk, no scalar tail): the wave visits rows
// first_row, first_row + row_step, ... (my_rows of them) as a sequence of chunks and keeps one chunk of look-ahead in
// registers: the loads of chunk i+1 are in flight while the exp/accumulate work of chunk i runs, so the memory
// stream and the ALU work overlap inside every wave.  on_row(row, H) is called by the whole wave, H wave-uniform.
template <typename T, int CH, typename OnRow>
__device__ __forceinline__ void walk_rows(const T* __restrict__ logits, int64_t first_row, int64_t row_step,
                                          int64_t my_rows, int nchunk, int64_t stride, int lane, OnRow on_row) {
  using VT = Vec16<T>;
  constexpr int VN = VT::N;
  if (my_rows <= 0) return;
  VT bufA[CH], bufB[CH];
  auto load = [&](VT (&buf)[CH], int64_t row, int chunk) {
    const T* p = logits + row * stride + ((int64_t)chunk * CH * NOVA_WAVE + lane) * VN;
#pragma unroll
    for (int c = 0; c < CH; ++c) buf[c].load(p + c * NOVA_WAVE * VN);
  };
  auto process = [&](Row& st, const VT (&buf)[CH]) {
    float cm = -INFINITY;
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
      for (int i = 0; i < VN; ++i) cm = fmaxf(cm, buf[c].get(i));
    const float M = wave_max_uniform(cm);
    st.rebase(M);
    const int before = st.cnt;
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
      for (int i = 0; i < VN; ++i) st.add(buf[c].get(i));
    // The maximum drops NaNs and add() counts them as if they were maxima.  A chunk without ties and without NaNs
    // counts exactly one element when its maximum is the running maximum and none otherwise; anything else (ties are
    // common with bf16 logits, NaNs are not) pays for one unordered compare per pair of elements.
    if (st.cnt - before != (M == st.m ? 1 : 0)) {
      bool unordered = false;
#pragma unroll
      for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int i = 0; i < VN; i += 2) unordered = unordered || __builtin_isunordered(buf[c].get(i), buf[c].get(i + 1));
      if (__any(unordered)) st.nan = true;
    }
  };
  auto finish_row = [&](int64_t row, Row& st) {
    on_row(row, st.finish());
    st.init();
  };
  // item = (row, chunk); the items of this wave are walked row-major with the two buffers alternating.  Every
  // load below is unconditional straight-line code (the odd tail is peeled), so the compiler's vmcnt bookkeeping
  // lets the look-ahead loads stay in flight.
  struct Cursor { int64_t row; int chunk; };
  auto advance = [&](Cursor c) {
    ++c.chunk;
    if (c.chunk == nchunk) { c.chunk = 0; c.row += row_step; }
    return c;
  };
  const int64_t n = my_rows * nchunk;
  Row st;
  st.init();
  Cursor ca = {first_row, 0};
  load(bufA, ca.row, ca.chunk);
  int64_t i = 0;
  for (; i + 2 < n; i += 2) {
    const Cursor cb = advance(ca);
    load(bufB, cb.row, cb.chunk);
    process(st, bufA);
    if (ca.chunk == nchunk - 1) finish_row(ca.row, st);
    ca = advance(cb);
    load(bufA, ca.row, ca.chunk);
    process(st, bufB);
    if (cb.chunk == nchunk - 1) finish_row(cb.row, st);
  }
  if (i + 1 < n) {
    const Cursor cb = advance(ca);
    load(bufB, cb.row, cb.chunk);
    process(st, bufA);
    if (ca.chunk == nchunk - 1) finish_row(ca.row, st);
    process(st, bufB);
    if (cb.chunk == nchunk - 1) finish_row(cb.row, st);
  } else {
    process(st, bufA);
    if (ca.chunk == nchunk - 1) finish_row(ca.row, st);
  }
}

// Chunk size for regular rows: V / (elements of one 16-byte vector per lane) sweeps per row, split into nchunk chunks
// of CH sweeps.  Returns 0 when the rows are not regular (V not a multiple of a sweep, or unaligned).
template <typename T>
__host__ inline int regular_sweeps(const void* logits, int V, int64_t stride) {
  constexpr int VN = Vec16<T>::N;
  const bool vec_ok = ((reinterpret_cast<uintptr_t>(logits) & 15) == 0) && ((stride * (int64_t)sizeof(T)) % 16 == 0);
  return (vec_ok && V % (NOVA_WAVE * VN) == 0) ? V / (NOVA_WAVE * VN) : 0;
}

}  // namespace entropy_core
