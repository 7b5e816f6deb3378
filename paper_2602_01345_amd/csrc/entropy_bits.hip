// Token entropy of a bitwise token head (the Infinity-style backbones of Sec. 4; entropy equation of
// Sec. 3.3 applied to a token that is d independent binary choices): H = sum over the d bits of the
// binary entropy of softmax(l0, l1).  With z = l1 - l0, a = |z| and q = e^-a:
//   h = ln(1 + q) + a q / (1 + q)        (no cancellation; -> 0 as a grows, ln 2 at a = 0)
// The input is a few bytes per token (2 d logits), so one thread owns one token and walks its bits
// with 16-byte loads; the rows of a wave stay in L1 between the iterations.
#include "common.h"
#include "nova_internal.h"

namespace {

__device__ __forceinline__ float binary_entropy_from_logits(float l0, float l1) {
  float a = fabsf(l1 - l0);
  a = a > 200.0f ? 200.0f : a;                       // e^-200 == 0: also covers an infinite logit; NaN stays NaN
  const float q = __expf(-a);
  return log1pf(q) + a * q / (1.0f + q);
}

template <typename T>
__global__ __launch_bounds__(256) void entropy_bits_kernel(const T* __restrict__ logits, int64_t rows, int d,
                                                           float* __restrict__ H) {
  using VT = Vec16<T>;
  constexpr int VN = VT::N;                          // elements per 16-byte vector (even)
  const int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= rows) return;
  const T* p = logits + row * 2 * (int64_t)d;
  const int n = 2 * d;
  float h = 0.0f;
  int i = 0;
  if ((reinterpret_cast<uintptr_t>(p) & 15) == 0) {
    for (; i + VN <= n; i += VN) {
      VT v;
      v.load(p + i);
#pragma unroll
      for (int e = 0; e < VN; e += 2) h += binary_entropy_from_logits(v.get(e), v.get(e + 1));
    }
  }
  for (; i < n; i += 2) h += binary_entropy_from_logits((float)p[i], (float)p[i + 1]);
  H[row] = h;
}

}  // namespace

hipError_t launch_entropy_bits(hipStream_t st, const void* logits, int dtype, int64_t rows_per_batch, int batch,
                               int d, float* H, float* mean) {
  const int64_t rows = rows_per_batch * batch;
  const int grid = (int)((rows + 255) / 256);
  if (dtype == NOVA_BF16)
    entropy_bits_kernel<bf16_t><<<grid, 256, 0, st>>>(static_cast<const bf16_t*>(logits), rows, d, H);
  else
    entropy_bits_kernel<float><<<grid, 256, 0, st>>>(static_cast<const float*>(logits), rows, d, H);
  if (mean) return launch_row_mean(st, H, rows_per_batch, batch, mean);
  return hipGetLastError();
}
