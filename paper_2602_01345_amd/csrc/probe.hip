// Instrumentation, not part of the hot path: three plain kernels that measure what this chip
// sustains, so that roofline fractions can be read against an achievable figure as well as the
// published one -- a streaming read, a streaming copy (16 bytes per lane, grid-stride) and a loop of
// independent bf16 MFMAs with no memory traffic, on constant operands and on operands loaded once from the
// caller's buffer (what the matrix cores sustain depends on the data: random operands switch more bits per
// MFMA, draw more power and run at a lower clock).  The caller times them with events.
#include "common.h"
#include "nova_internal.h"

namespace {

constexpr int kUnroll = 4;

__global__ __launch_bounds__(256) void probe_read_kernel(const f32x4* __restrict__ src, int64_t nvec,
                                                         float* __restrict__ sink) {
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  const int64_t stride = (int64_t)gridDim.x * 256 * kUnroll;
  for (int64_t i = (int64_t)blockIdx.x * 256 * kUnroll + threadIdx.x; i < nvec; i += stride) {
    f32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = i + u * 256 < nvec ? src[i + u * 256] : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc += v[u];
  }
  // keeps the loads alive; true for no real input
  if (acc[0] + acc[1] + acc[2] + acc[3] == 12345.678f) sink[0] = 1.0f;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst,
                                                         int64_t nvec) {
  const int64_t stride = (int64_t)gridDim.x * 256 * kUnroll;
  for (int64_t i = (int64_t)blockIdx.x * 256 * kUnroll + threadIdx.x; i < nvec; i += stride) {
    f32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (i + u * 256 < nvec) v[u] = src[i + u * 256];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (i + u * 256 < nvec) dst[i + u * 256] = v[u];
  }
}

// 8 waves per CU, each issuing `iters` rounds of 32 MFMAs over four independent accumulators
__global__ __launch_bounds__(512, 1) void probe_mfma_kernel(int iters, float* __restrict__ sink) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (bf16_t)(0.001f * (float)(threadIdx.x & 63) + (float)i);
    b[i] = (bf16_t)(0.5f * (float)i);
  }
  f32x16 c[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) c[t][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 32; ++u) c[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[u & 3], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c[t][r];
  if (s == 12345.678f) sink[0] = s;
}

// the same loop with every lane's operand fragments read once from memory (eight 16-byte vectors per lane)
__global__ __launch_bounds__(512, 1) void probe_mfma_data_kernel(const bf16x8* __restrict__ src, int iters,
                                                                 float* __restrict__ sink) {
  const int64_t t = (int64_t)blockIdx.x * 512 + threadIdx.x;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = src[t * 8 + i];
    b[i] = src[t * 8 + 4 + i];
  }
  f32x16 c[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) c[u][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 32; ++u) c[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u & 3], b[(u >> 2) & 3], c[u & 3], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c[u][r];
  if (s == 12345.678f) sink[0] = s;
}

}  // namespace

hipError_t launch_probe_read(hipStream_t st, int num_cus, const void* src, int64_t bytes, float* sink) {
  probe_read_kernel<<<num_cus * 16, 256, 0, st>>>(static_cast<const f32x4*>(src), bytes / 16, sink);
  return hipGetLastError();
}

hipError_t launch_probe_copy(hipStream_t st, int num_cus, const void* src, void* dst, int64_t bytes) {
  probe_copy_kernel<<<num_cus * 16, 256, 0, st>>>(static_cast<const f32x4*>(src), static_cast<f32x4*>(dst), bytes / 16);
  return hipGetLastError();
}

hipError_t launch_probe_mfma(hipStream_t st, int num_cus, int iters, float* sink) {
  probe_mfma_kernel<<<num_cus, 512, 0, st>>>(iters, sink);
  return hipGetLastError();
}

hipError_t launch_probe_mfma_data(hipStream_t st, int num_cus, const void* src, int iters, float* sink) {
  probe_mfma_data_kernel<<<num_cus, 512, 0, st>>>(static_cast<const bf16x8*>(src), iters, sink);
  return hipGetLastError();
}
