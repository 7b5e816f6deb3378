// Entropy-guided token selection: per batch row keep the k tokens that come first in
// the order (entropy descending, index ascending)  (Sec. 3.3, "Dual-Linkage
// Acceleration", final sentence; Sec. 3.2, the highest-entropy tokens are maintained).
//
// One 1024-thread workgroup per batch row.  Entropies are mapped to 32-bit keys whose
// unsigned order is the required numeric order (NaN lowest, -0 == +0), staged in LDS,
// and the k-th largest key is found by a 4-pass, 8-bit MSB radix select on LDS
// histograms (select_core.h).  Every key above the threshold is kept; of the keys equal to it the
// first (k - #above) in index order are kept.  Two block-wide prefix sums over
// contiguous index ranges turn that rule into the ascending index list and the mask.
// Integer compares only: the result equals a stable sort bit for bit.
#include "common.h"
#include "nova_internal.h"
#include "select_core.h"

namespace {

using namespace select_core;

constexpr int kThreads = 1024;
constexpr int kLdsKeys = 8192;   // rows up to this many tokens are staged in LDS

template <bool STAGED>
__global__ __launch_bounds__(kThreads) void select_kernel(const float* __restrict__ H, int N, int k_uniform,
                                                          const int32_t* __restrict__ k_per_row,
                                                          int pitch, int32_t* __restrict__ idx,
                                                          uint8_t* __restrict__ mask) {
  __shared__ uint32_t keys_lds[STAGED ? kLdsKeys : 1];
  __shared__ Scratch<kThreads> sc;

  const int tid = threadIdx.x;
  const int b = blockIdx.x;
  const float* h = H + (int64_t)b * N;

  int k = k_uniform;
  if (k_per_row) {
    k = k_per_row[b];
    k = k < 0 ? 0 : (k > N ? N : k);
    k = k > pitch ? pitch : k;
  }

  if (STAGED) {
    for (int i = tid; i < N; i += kThreads) keys_lds[i] = sort_key(h[i]);
    __syncthreads();
  }
  auto key_at = [&](int i) -> uint32_t { return STAGED ? keys_lds[i] : sort_key(h[i]); };

  uint32_t thr = 0, remaining = 0;
  if (k > 0 && k < N) thr = radix_select<kThreads, 32>(key_at, N, k, sc, &remaining);
  compact<kThreads>(key_at, N, thr, remaining, k == N, k == 0, pitch, idx + (int64_t)b * pitch, mask + (int64_t)b * N,
                    sc.wave_sums);
}

}  // namespace

hipError_t launch_select(hipStream_t st, const float* H, int B, int N, int k, const int32_t* k_per_row,
                         int32_t* idx, uint8_t* mask) {
  if (N <= kLdsKeys)
    select_kernel<true><<<B, kThreads, 0, st>>>(H, N, k, k_per_row, k, idx, mask);
  else
    select_kernel<false><<<B, kThreads, 0, st>>>(H, N, k, k_per_row, k, idx, mask);
  return hipGetLastError();
}
