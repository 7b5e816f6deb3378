// Row gather + LayerNorm (no affine, biased variance, eps 1e-6) feeding the block's
// two projections; optionally modulated per image, LN(x) (1 + scale[b]) + shift[b].  One wave64 per row; mean and
// variance are two separate fp32 passes over the row, which is read once and held in registers when it fits
// (else three reads, the second and third from the cache); the output is rounded once to the storage type.
#include "common.h"
#include "nova_internal.h"

namespace {

constexpr int kWavesPerBlock = 4;
constexpr float kEps = 1e-6f;
constexpr int kRegVecs = 8;        // 16-byte vectors per lane a row may take to be kept in registers

template <typename T>
__global__ __launch_bounds__(kWavesPerBlock* NOVA_WAVE) void gather_ln_kernel(
    const T* __restrict__ src, const int32_t* __restrict__ idx, int M, int k, int N, int C,
    const T* __restrict__ shift, const T* __restrict__ scale, int mod_pitch, T* __restrict__ dst,
    const int32_t* __restrict__ k_rows, const int32_t* __restrict__ kv_rows, int32_t* __restrict__ kv_next, int P) {
  using VT = Vec16<T>;
  constexpr int VN = VT::N;
  const int lane = threadIdx.x & (NOVA_WAVE - 1);
  const int m = blockIdx.x * kWavesPerBlock + threadIdx.x / NOVA_WAVE;
  if (kv_next && blockIdx.x == 0) {
    // per-image cache lengths after this block: prior rows + kept rows.  Written by this launch (the second
    // LayerNorm: everything that reads the old lengths has run), so the output may be the input array.
    const int B = M / k;
    for (int b = threadIdx.x; b < B; b += kWavesPerBlock * NOVA_WAVE)
      kv_next[b] = image_prior(kv_rows, b, P) + image_count(k_rows, b, k);
  }
  if (m >= M) return;
  if (k_rows && m % k >= image_count(k_rows, m / k, k)) {
    // a slot past its image's keep count: zeros, so that everything downstream of it stays finite
    VT z;
#pragma unroll
    for (int e = 0; e < VN; ++e) z.set(e, 0.0f);
    for (int vi = lane; vi < C / VN; vi += NOVA_WAVE) z.store(dst + (int64_t)m * C + vi * VN);
    return;
  }
  int64_t srow = m;
  if (idx) {
    const int b = m / k;
    const int t = min(max(idx[m], 0), N - 1);   // idx is [B, k] and m = b * k + s; clamped, never out of bounds
    srow = (int64_t)b * N + t;
  }
  const T* p = src + srow * C;
  T* q = dst + (int64_t)m * C;
  const int nvec = C / VN;

  if (nvec <= kRegVecs * NOVA_WAVE) {
    // the row fits the wave's registers (C <= 4096 bf16 / 2048 fp32): read once; the same sums in the same
    // order as the three-pass form below
    VT v[kRegVecs];
#pragma unroll
    for (int u = 0; u < kRegVecs; ++u) {
      const int vi = u * NOVA_WAVE + lane;
      if (vi < nvec) v[u].load(p + vi * VN);
    }
    float sum = 0.f;
#pragma unroll
    for (int u = 0; u < kRegVecs; ++u)
      if (u * NOVA_WAVE + lane < nvec) {
#pragma unroll
        for (int e = 0; e < VN; ++e) sum += v[u].get(e);
      }
    const float mean = wave_sum(sum) / (float)C;
    float sq = 0.f;
#pragma unroll
    for (int u = 0; u < kRegVecs; ++u)
      if (u * NOVA_WAVE + lane < nvec) {
#pragma unroll
        for (int e = 0; e < VN; ++e) { float d = v[u].get(e) - mean; sq = fmaf(d, d, sq); }
      }
    const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)C + kEps);
    const T* sh = shift ? shift + (int64_t)(m / k) * mod_pitch : nullptr;
    const T* sc = shift ? scale + (int64_t)(m / k) * mod_pitch : nullptr;
#pragma unroll
    for (int u = 0; u < kRegVecs; ++u) {
      const int vi = u * NOVA_WAVE + lane;
      if (vi < nvec) {
        VT o;
        if (shift) {
          VT a, g; a.load(sh + vi * VN); g.load(sc + vi * VN);
#pragma unroll
          for (int e = 0; e < VN; ++e) o.set(e, fmaf((v[u].get(e) - mean) * rstd, 1.0f + g.get(e), a.get(e)));
        } else {
#pragma unroll
          for (int e = 0; e < VN; ++e) o.set(e, (v[u].get(e) - mean) * rstd);
        }
        o.store(q + vi * VN);
      }
    }
    return;
  }

  float sum = 0.f;
  for (int vi = lane; vi < nvec; vi += NOVA_WAVE) {
    VT v; v.load(p + vi * VN);
#pragma unroll
    for (int e = 0; e < VN; ++e) sum += v.get(e);
  }
  const float mean = wave_sum(sum) / (float)C;
  float sq = 0.f;
  for (int vi = lane; vi < nvec; vi += NOVA_WAVE) {
    VT v; v.load(p + vi * VN);
#pragma unroll
    for (int e = 0; e < VN; ++e) { float d = v.get(e) - mean; sq = fmaf(d, d, sq); }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)C + kEps);
  if (shift) {          // modulation vectors of image m / k (both given or neither)
    const T* sh = shift + (int64_t)(m / k) * mod_pitch;
    const T* sc = scale + (int64_t)(m / k) * mod_pitch;
    for (int vi = lane; vi < nvec; vi += NOVA_WAVE) {
      VT v, o, a, g; v.load(p + vi * VN); a.load(sh + vi * VN); g.load(sc + vi * VN);
#pragma unroll
      for (int e = 0; e < VN; ++e) o.set(e, fmaf((v.get(e) - mean) * rstd, 1.0f + g.get(e), a.get(e)));
      o.store(q + vi * VN);
    }
    return;
  }
  for (int vi = lane; vi < nvec; vi += NOVA_WAVE) {
    VT v, o; v.load(p + vi * VN);
#pragma unroll
    for (int e = 0; e < VN; ++e) o.set(e, (v.get(e) - mean) * rstd);
    o.store(q + vi * VN);
  }
}

}  // namespace

hipError_t launch_gather_ln(hipStream_t st, int dtype, const void* src, const int32_t* idx, int M, int k,
                            int N, int C, const void* shift, const void* scale, int mod_pitch, void* dst,
                            const int32_t* k_rows, const int32_t* kv_rows, int32_t* kv_next, int P) {
  const unsigned grid = (unsigned)((M + kWavesPerBlock - 1) / kWavesPerBlock);
  if (dtype == NOVA_BF16)
    gather_ln_kernel<bf16_t><<<grid, kWavesPerBlock * NOVA_WAVE, 0, st>>>(
        static_cast<const bf16_t*>(src), idx, M, k, N, C, static_cast<const bf16_t*>(shift),
        static_cast<const bf16_t*>(scale), mod_pitch, static_cast<bf16_t*>(dst), k_rows, kv_rows, kv_next, P);
  else
    gather_ln_kernel<float><<<grid, kWavesPerBlock * NOVA_WAVE, 0, st>>>(
        static_cast<const float*>(src), idx, M, k, N, C, static_cast<const float*>(shift),
        static_cast<const float*>(scale), mod_pitch, static_cast<float*>(dst), k_rows, kv_rows, kv_next, P);
  return hipGetLastError();
}
