// Residual cache reuse (Sec. 3.3, "Residual Cache Reuse", second and third equations):
// kept tokens take the block's output; pruned tokens take their input plus the prior
// scale's residual cache interpolated to the current grid; the new residual cache is
// output minus input everywhere.
//
// Bandwidth-bound streaming kernel.  One wave64 owns one token row of C channels and
// moves it in 16-byte vectors; all loads of a sweep are issued before the first use.
// The bilinear taps (half-pixel centres) are wave-uniform and evaluated in fp32.  Other interpolation
// kernels (nearest cell, cubic convolution) go through a generic separable-taps kernel further down.
#include "common.h"
#include "nova_internal.h"

namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kUnroll = 4;

// Position of kept token i in the ascending kept list of its image = the number of kept tokens in front of it.
// When the image's mask row is 16-byte aligned and a whole number of 16-byte chunks, the wave counts the
// non-zero mask bytes before i, 16 per lane and step: independent loads, one round trip to memory.  Otherwise a
// binary search over the index list (log2 k dependent loads).  Both give the same number for a consistent
// (index list, mask) pair.  Wave-uniform result.
__device__ __forceinline__ int kept_rank(const uint8_t* __restrict__ mrow, const int32_t* __restrict__ list, int N,
                                         int k, int i, int lane) {
  if ((reinterpret_cast<uintptr_t>(mrow) & 15) == 0 && N % 16 == 0) {
    int cnt = 0;
    constexpr int kChunks = 4;                             // chunks per lane requested together
    for (int base = 0; base < i; base += kChunks * NOVA_WAVE * 16) {
      u32x4 v[kChunks];
#pragma unroll
      for (int u = 0; u < kChunks; ++u) {
        const int j0 = base + (u * NOVA_WAVE + lane) * 16;
        v[u] = u32x4{0u, 0u, 0u, 0u};
        if (j0 < i) v[u] = *reinterpret_cast<const u32x4*>(mrow + j0);
      }
#pragma unroll
      for (int u = 0; u < kChunks; ++u) {
        const int j0 = base + (u * NOVA_WAVE + lane) * 16;
        const int valid = min(16, i - j0);                 // bytes of this chunk that lie in front of i (<= 0: none)
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const int nv = min(max(valid - 4 * d, 0), 4);
          const uint32_t keep = nv >= 4 ? 0xffffffffu : ((1u << (8 * nv)) - 1u);
          const uint32_t wd = v[u][d] & keep;
          const uint32_t nz = (((wd & 0x7f7f7f7fu) + 0x7f7f7f7fu) | wd) & 0x80808080u;   // top bit of every non-zero byte
          cnt += __popc(nz);
        }
      }
    }
#pragma unroll
    for (int o = NOVA_WAVE / 2; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, NOVA_WAVE);
    return min(cnt, k - 1);
  }
  int lo = 0, hi = k - 1;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (list[mid] < i) lo = mid + 1; else hi = mid;
  }
  return lo;
}

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

template <typename T>
__global__ __launch_bounds__(kWavesPerBlock* NOVA_WAVE) void merge_kernel(
    int B, int C, int h, int w, int hp, int wp, int k, const T* __restrict__ x, const T* __restrict__ y,
    const int32_t* __restrict__ idx, const uint8_t* __restrict__ mask, const T* __restrict__ cache_prev,
    T* __restrict__ out, T* __restrict__ cache_new) {
  using VT = Vec16<T>;
  constexpr int VN = VT::N;
  const int lane = threadIdx.x & (NOVA_WAVE - 1);
  const int wave = threadIdx.x / NOVA_WAVE;
  const int N = h * w;
  const int64_t row = (int64_t)blockIdx.x * kWavesPerBlock + wave;   // b * N + i
  if (row >= (int64_t)B * N) return;
  const int b = (int)(row / N);
  const int i = (int)(row - (int64_t)b * N);
  const int nvec = C / VN;                                           // C % VN == 0 (checked by the host)
  const T* xr = x + row * C;
  T* outr = out + row * C;
  T* cnr = cache_new ? cache_new + row * C : nullptr;

  if (mask[row] && k > 0) {
    const int lo = kept_rank(mask + (int64_t)b * N, idx + (int64_t)b * k, N, k, i, lane);
    const T* yr = y + ((int64_t)b * k + lo) * C;
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
    T* __restrict__ out, T* __restrict__ cache_new) {
  using VT = Vec16<T>;
  constexpr int VN = VT::N;
  const int lane = threadIdx.x & (NOVA_WAVE - 1);
  const int wave = threadIdx.x / NOVA_WAVE;
  const int N = h * w;
  const int64_t row = (int64_t)blockIdx.x * kWavesPerBlock + wave;   // b * N + i
  if (row >= (int64_t)B * N) return;
  const int b = (int)(row / N);
  const int i = (int)(row - (int64_t)b * N);
  const int nvec = C / VN;
  const T* xr = x + row * C;
  T* outr = out + row * C;
  T* cnr = cache_new ? cache_new + row * C : nullptr;

  if (mask[row] && k > 0) {       // kept token: the block's output, copied; residual = output - input
    const int lo = kept_rank(mask + (int64_t)b * N, idx + (int64_t)b * k, N, k, i, lane);
    const T* yr = y + ((int64_t)b * k + lo) * C;
    for (int vi = lane; vi < nvec; vi += NOVA_WAVE) {
      VT vy, vx, c;
      vy.load(yr + vi * VN); vx.load(xr + vi * VN);
      vy.store(outr + vi * VN);
      if (cnr) {
#pragma unroll
        for (int e = 0; e < VN; ++e) c.set(e, vy.get(e) - vx.get(e));
        c.store(cnr + vi * VN);
      }
    }
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
                    void* cache_new) {
  const int64_t rows = (int64_t)B * h * w;
  const unsigned grid = (unsigned)((rows + kWavesPerBlock - 1) / kWavesPerBlock);
  const T* xt = static_cast<const T*>(x);
  const T* yt = static_cast<const T*>(y);
  const T* ct = static_cast<const T*>(cache_prev);
  T* ot = static_cast<T*>(out);
  T* nt = static_cast<T*>(cache_new);
  if (interp == NOVA_INTERP_NEAREST)
    merge_taps_kernel<T, 1><<<grid, kWavesPerBlock * NOVA_WAVE, 0, st>>>(B, C, h, w, hp, wp, k, xt, yt, idx, mask, ct,
                                                                       ot, nt);
  else if (interp == NOVA_INTERP_BICUBIC)
    merge_taps_kernel<T, 4><<<grid, kWavesPerBlock * NOVA_WAVE, 0, st>>>(B, C, h, w, hp, wp, k, xt, yt, idx, mask, ct,
                                                                       ot, nt);
  else
    merge_kernel<T><<<grid, kWavesPerBlock * NOVA_WAVE, 0, st>>>(B, C, h, w, hp, wp, k, xt, yt, idx, mask, ct, ot, nt);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_merge(hipStream_t st, int dtype, int interp, int B, int C, int h, int w, int hp, int wp, int k,
                        const void* x, const void* y, const int32_t* idx, const uint8_t* mask,
                        const void* cache_prev, void* out, void* cache_new) {
  if (dtype == NOVA_BF16)
    return launch_t<bf16_t>(st, interp, B, C, h, w, hp, wp, k, x, y, idx, mask, cache_prev, out, cache_new);
  return launch_t<float>(st, interp, B, C, h, w, hp, wp, k, x, y, idx, mask, cache_prev, out, cache_new);
}
