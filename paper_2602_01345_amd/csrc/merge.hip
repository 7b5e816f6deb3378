// Residual cache reuse (Sec. 3.3, "Residual Cache Reuse", second and third equations):
// kept tokens take the block's output; pruned tokens take their input plus the prior
// scale's residual cache interpolated to the current grid; the new residual cache is
// output minus input everywhere.
//
// Bandwidth-bound streaming kernel.  One wave64 owns one row of C channels and moves it in 16-byte vectors; all
// loads of a sweep are issued before the first use.  The launch has one wave per token (it serves the pruned
// tokens: a wave whose mask byte says "kept" leaves at once) followed by one wave per kept slot (b, s), which
// copies row s of the block's output to token kept_idx[b, s] -- so nobody has to look up where in the kept
// list a token sits.  Per-image keep counts: slots past an image's count (or holding -1) leave at once.
// The bilinear taps (half-pixel centres) are wave-uniform and evaluated in fp32.  Other interpolation
// kernels (nearest cell, cubic convolution) go through a generic separable-taps kernel further down.
#include "common.h"
#include "nova_internal.h"

namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kUnroll = 4;

struct Taps {
  int i0, i1;
  float w1;
};

__device__ __forceinline__ Taps axis_taps(int dst, int n_in, int n_out) {
  float src = ((float)dst + 0.5f) * ((float)n_in / (float)n_out) - 0.5f;
  src = src < 0.0f ? 0.0f : src;
  int i0 = (int)floorf(src);
  i0 = i0 > n_in - 1 ? n_in - 1 : i0;
  Taps t;
  t.i0 = i0;
  t.i1 = i0 + 1 > n_in - 1 ? n_in - 1 : i0 + 1;
  t.w1 = src - (float)i0;
  return t;
}

// The wave's job: a pruned token (tok >= 0, slot < 0), a kept slot (both >= 0), or nothing (tok < 0).
struct MergeItem {
  int b, tok;
  int64_t slot;      // row of y_kept, or -1
};
__device__ __forceinline__ MergeItem merge_item(int B, int N, int k, const int32_t* __restrict__ idx,
                                                const uint8_t* __restrict__ mask, const int32_t* __restrict__ k_rows) {
  const int wave = threadIdx.x / NOVA_WAVE;
  const int64_t item = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  const int64_t n_tok = (int64_t)B * N;
  MergeItem it = {0, -1, -1};
  if (item < n_tok) {
    it.b = (int)(item / N);
    // kept tokens are written by their slot's wave (with k == 0 there are no slots: every token takes this path)
    if (!mask[item] || k == 0) it.tok = (int)(item - (int64_t)it.b * N);
  } else if (item - n_tok < (int64_t)B * k) {
    const int64_t slot = item - n_tok;
    it.b = (int)(slot / k);
    const int s = (int)(slot - (int64_t)it.b * k);
    const int t = s < image_count(k_rows, it.b, k) ? idx[slot] : -1;
    if (t >= 0 && t < N) { it.tok = t; it.slot = slot; }
  }
  return it;
}

// kept token: the block's output, copied; residual = output - input
template <typename T>
__device__ __forceinline__ void merge_kept_row(const T* __restrict__ yr, const T* __restrict__ xr, T* __restrict__ outr,
                                               T* __restrict__ cnr, int nvec, int lane) {
  using VT = Vec16<T>;
  constexpr int VN = VT::N;
  for (int v0 = 0; v0 < nvec; v0 += kUnroll * NOVA_WAVE) {
    VT vy[kUnroll], vx[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      int vi = v0 + u * NOVA_WAVE + lane;
      if (vi < nvec) { vy[u].load(yr + vi * VN); vx[u].load(xr + vi * VN); }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      int vi = v0 + u * NOVA_WAVE + lane;
      if (vi < nvec) {
        vy[u].store(outr + vi * VN);
        if (cnr) {
          VT c;
#pragma unroll
          for (int e = 0; e < VN; ++e) c.set(e, vy[u].get(e) - vx[u].get(e));
          c.store(cnr + vi * VN);
        }
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kWavesPerBlock* NOVA_WAVE) void merge_kernel(
    int B, int C, int h, int w, int hp, int wp, int k, const T* __restrict__ x, const T* __restrict__ y,
    const int32_t* __restrict__ idx, const uint8_t* __restrict__ mask, const T* __restrict__ cache_prev,
    T* __restrict__ out, T* __restrict__ cache_new, const int32_t* __restrict__ k_rows) {
  using VT = Vec16<T>;
  constexpr int VN = VT::N;
  const int lane = threadIdx.x & (NOVA_WAVE - 1);
  const int N = h * w;
  const MergeItem it = merge_item(B, N, k, idx, mask, k_rows);
  if (it.tok < 0) return;
  const int b = it.b, i = it.tok;
  const int64_t row = (int64_t)b * N + i;
  const int nvec = C / VN;                                           // C % VN == 0 (checked by the host)
  const T* xr = x + row * C;
  T* outr = out + row * C;
  T* cnr = cache_new ? cache_new + row * C : nullptr;

  if (it.slot >= 0) {
    merge_kept_row<T>(y + it.slot * C, xr, outr, cnr, nvec, lane);
    return;
  }

  if (!cache_prev) {
    // no prior cache was given (legal only when every token is kept): a row the mask still
    // marks as pruned passes through unchanged with a zero residual
    for (int vi = lane; vi < nvec; vi += NOVA_WAVE) {
      VT v, z;
      v.load(xr + vi * VN);
#pragma unroll
      for (int e = 0; e < VN; ++e) z.set(e, 0.0f);
      v.store(outr + vi * VN);
      if (cnr) z.store(cnr + vi * VN);
    }
    return;
  }
  const int oy = i / w, ox = i - oy * w;
  const Taps ty = axis_taps(oy, hp, h);
  const Taps tx = axis_taps(ox, wp, w);
  const T* base = cache_prev + (int64_t)b * hp * wp * C;
  const T* c00 = base + ((int64_t)ty.i0 * wp + tx.i0) * C;
  const T* c01 = base + ((int64_t)ty.i0 * wp + tx.i1) * C;
  const T* c10 = base + ((int64_t)ty.i1 * wp + tx.i0) * C;
  const T* c11 = base + ((int64_t)ty.i1 * wp + tx.i1) * C;
  const float wy1 = ty.w1, wy0 = 1.0f - ty.w1, wx1 = tx.w1, wx0 = 1.0f - tx.w1;

  for (int v0 = 0; v0 < nvec; v0 += kUnroll * NOVA_WAVE) {
    VT vx[kUnroll], a00[kUnroll], a01[kUnroll], a10[kUnroll], a11[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      int vi = v0 + u * NOVA_WAVE + lane;
      if (vi < nvec) {
        vx[u].load(xr + vi * VN);
        a00[u].load(c00 + vi * VN); a01[u].load(c01 + vi * VN);
        a10[u].load(c10 + vi * VN); a11[u].load(c11 + vi * VN);
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      int vi = v0 + u * NOVA_WAVE + lane;
      if (vi < nvec) {
        VT o, c;
#pragma unroll
        for (int e = 0; e < VN; ++e) {
          // rows first (y), then columns (x), as separable linear interpolation
          float top = a00[u].get(e) * wy0 + a10[u].get(e) * wy1;
          float bot = a01[u].get(e) * wy0 + a11[u].get(e) * wy1;
          float up = top * wx0 + bot * wx1;
          o.set(e, vx[u].get(e) + up);
          c.set(e, up);
        }
        o.store(outr + vi * VN);
        if (cnr) c.store(cnr + vi * VN);
      }
    }
  }
}

// ---- other interpolation kernels: NT taps per axis (1 = nearest cell, 4 = cubic convolution) -------------
template <int NT>
struct AxisTaps {
  int i[NT];
  float w[NT];
};

// nearest: the source cell that contains the output cell's centre, min(floor((dst + 1/2) n_in / n_out), n_in - 1),
// in integer arithmetic (centres on a cell boundary must not depend on rounding)
__device__ __forceinline__ AxisTaps<1> nearest_taps(int dst, int n_in, int n_out) {
  AxisTaps<1> t;
  const int64_t q = ((int64_t)(2 * dst + 1) * n_in) / (2 * (int64_t)n_out);
  t.i[0] = (int)(q > n_in - 1 ? n_in - 1 : q);
  t.w[0] = 1.0f;
  return t;
}

// cubic convolution, kernel parameter a = -3/4, half-pixel centres, taps floor(src) - 1 .. floor(src) + 2
// clamped to the grid
__device__ __forceinline__ AxisTaps<4> cubic_taps(int dst, int n_in, int n_out) {
  constexpr float a = -0.75f;
  const float src = ((float)dst + 0.5f) * ((float)n_in / (float)n_out) - 0.5f;
  const float fl = floorf(src);
  const float t = src - fl;
  const int i0 = (int)fl;
  auto near = [](float d) { return ((a + 2.0f) * d - (a + 3.0f)) * d * d + 1.0f; };          // |d| <= 1
  auto far = [](float d) { return ((a * d - 5.0f * a) * d + 8.0f * a) * d - 4.0f * a; };     // 1 < |d| < 2
  AxisTaps<4> r;
  r.w[0] = far(t + 1.0f); r.w[1] = near(t); r.w[2] = near(1.0f - t); r.w[3] = far(2.0f - t);
#pragma unroll
  for (int j = 0; j < 4; ++j) r.i[j] = min(max(i0 - 1 + j, 0), n_in - 1);
  return r;
}

template <typename T, int NT>
__global__ __launch_bounds__(kWavesPerBlock* NOVA_WAVE) void merge_taps_kernel(
    int B, int C, int h, int w, int hp, int wp, int k, const T* __restrict__ x, const T* __restrict__ y,
    const int32_t* __restrict__ idx, const uint8_t* __restrict__ mask, const T* __restrict__ cache_prev,
    T* __restrict__ out, T* __restrict__ cache_new, const int32_t* __restrict__ k_rows) {
  using VT = Vec16<T>;
  constexpr int VN = VT::N;
  const int lane = threadIdx.x & (NOVA_WAVE - 1);
  const int N = h * w;
  const MergeItem it = merge_item(B, N, k, idx, mask, k_rows);
  if (it.tok < 0) return;
  const int b = it.b, i = it.tok;
  const int64_t row = (int64_t)b * N + i;
  const int nvec = C / VN;
  const T* xr = x + row * C;
  T* outr = out + row * C;
  T* cnr = cache_new ? cache_new + row * C : nullptr;

  if (it.slot >= 0) {
    merge_kept_row<T>(y + it.slot * C, xr, outr, cnr, nvec, lane);
    return;
  }
  if (!cache_prev) {              // legal only when every token is kept: pass through, zero residual
    for (int vi = lane; vi < nvec; vi += NOVA_WAVE) {
      VT v, z;
      v.load(xr + vi * VN);
#pragma unroll
      for (int e = 0; e < VN; ++e) z.set(e, 0.0f);
      v.store(outr + vi * VN);
      if (cnr) z.store(cnr + vi * VN);
    }
    return;
  }
  const int oy = i / w, ox = i - oy * w;
  AxisTaps<NT> ty, tx;
  if constexpr (NT == 1) { ty = nearest_taps(oy, hp, h); tx = nearest_taps(ox, wp, w); }
  else { ty = cubic_taps(oy, hp, h); tx = cubic_taps(ox, wp, w); }
  const T* base = cache_prev + (int64_t)b * hp * wp * C;
  for (int vi = lane; vi < nvec; vi += NOVA_WAVE) {
    VT vx;
    vx.load(xr + vi * VN);
    float up[VN];
#pragma unroll
    for (int e = 0; e < VN; ++e) up[e] = 0.0f;
#pragma unroll
    for (int jx = 0; jx < NT; ++jx) {
      float col[VN];                                     // rows first (y), then columns (x)
#pragma unroll
      for (int e = 0; e < VN; ++e) col[e] = 0.0f;
#pragma unroll
      for (int jy = 0; jy < NT; ++jy) {
        VT a;
        a.load(base + ((int64_t)ty.i[jy] * wp + tx.i[jx]) * C + vi * VN);
#pragma unroll
        for (int e = 0; e < VN; ++e) col[e] = fmaf(a.get(e), ty.w[jy], col[e]);
      }
#pragma unroll
      for (int e = 0; e < VN; ++e) up[e] = fmaf(col[e], tx.w[jx], up[e]);
    }
    VT o, c;
#pragma unroll
    for (int e = 0; e < VN; ++e) { o.set(e, vx.get(e) + up[e]); c.set(e, up[e]); }
    o.store(outr + vi * VN);
    if (cnr) c.store(cnr + vi * VN);
  }
}

template <typename T>
hipError_t launch_t(hipStream_t st, int interp, int B, int C, int h, int w, int hp, int wp, int k, const void* x,
                    const void* y, const int32_t* idx, const uint8_t* mask, const void* cache_prev, void* out,
                    void* cache_new, const int32_t* k_rows) {
  const int64_t rows = (int64_t)B * h * w + (int64_t)B * k;          // one wave per token, then one per kept slot
  const unsigned grid = (unsigned)((rows + kWavesPerBlock - 1) / kWavesPerBlock);
  const T* xt = static_cast<const T*>(x);
  const T* yt = static_cast<const T*>(y);
  const T* ct = static_cast<const T*>(cache_prev);
  T* ot = static_cast<T*>(out);
  T* nt = static_cast<T*>(cache_new);
  if (interp == NOVA_INTERP_NEAREST)
    merge_taps_kernel<T, 1><<<grid, kWavesPerBlock * NOVA_WAVE, 0, st>>>(B, C, h, w, hp, wp, k, xt, yt, idx, mask, ct,
                                                                       ot, nt, k_rows);
  else if (interp == NOVA_INTERP_BICUBIC)
    merge_taps_kernel<T, 4><<<grid, kWavesPerBlock * NOVA_WAVE, 0, st>>>(B, C, h, w, hp, wp, k, xt, yt, idx, mask, ct,
                                                                       ot, nt, k_rows);
  else
    merge_kernel<T><<<grid, kWavesPerBlock * NOVA_WAVE, 0, st>>>(B, C, h, w, hp, wp, k, xt, yt, idx, mask, ct, ot, nt,
                                                                 k_rows);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_merge(hipStream_t st, int dtype, int interp, int B, int C, int h, int w, int hp, int wp, int k,
                        const void* x, const void* y, const int32_t* idx, const uint8_t* mask,
                        const void* cache_prev, void* out, void* cache_new, const int32_t* k_rows) {
  if (dtype == NOVA_BF16)
    return launch_t<bf16_t>(st, interp, B, C, h, w, hp, wp, k, x, y, idx, mask, cache_prev, out, cache_new, k_rows);
  return launch_t<float>(st, interp, B, C, h, w, hp, wp, k, x, y, idx, mask, cache_prev, out, cache_new, k_rows);
}
