// Ratio controllers (Sec. 3.3, "Adaptive Acceleration Activation": growth rate, early baseline,
// smoothed growth, activation scale; "Dual-Linkage Acceleration": scale-linkage and layer-linkage
// reduction ratios).  The scale-level quantities are a handful of scalars per image and are
// computed on the host; the layer-level ratio sits between two device kernels of every block
// (entropy before it, selection after it), so it runs on the device and hands nova_select its
// per-row keep counts directly.
#include <cmath>

#include "common.h"
#include "nova_internal.h"

namespace {

__global__ __launch_bounds__(256) void layer_ratio_kernel(const float* __restrict__ mean_entropy,
                                                          float* __restrict__ entropy_sum,
                                                          const float* __restrict__ ratio_t, int j, int B, int N,
                                                          float* __restrict__ ratio_tj,
                                                          int32_t* __restrict__ k_per_row) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const float h = mean_entropy[b];
  const float rt = ratio_t[b];
  float r = rt;
  float sum = 0.0f;
  if (j >= 2) {
    sum = entropy_sum[b];
    const float mu = sum / (float)(j - 1);
    if (mu != 0.0f) {
      const float delta = (h - mu) / mu;
      r = rt - delta * rt;
    }
  }
  entropy_sum[b] = sum + h;
  ratio_tj[b] = r;
  // NaN falls through both comparisons of the clamp as 0: every token is kept
  const float rc = fminf(fmaxf(r, 0.0f), 1.0f);
  k_per_row[b] = N - (int)floorf(rc * (float)N);
}

}  // namespace

hipError_t launch_layer_ratio(hipStream_t st, const float* mean_entropy, float* entropy_sum, const float* ratio_t,
                              int j, int B, int N, float* ratio_tj, int32_t* k_per_row) {
  const int threads = 256;
  layer_ratio_kernel<<<(B + threads - 1) / threads, threads, 0, st>>>(mean_entropy, entropy_sum, ratio_t, j, B, N,
                                                                     ratio_tj, k_per_row);
  return hipGetLastError();
}

extern "C" {

int nova_activation_scale(const double* hbar, int T, int t_est, double alpha, int* t_star) {
  if (!t_star || T < 0 || t_est < 2 || (T > 0 && !hbar)) return NOVA_ERR_INVALID_ARG;
  *t_star = 0;
  if (T < t_est + 1) return NOVA_OK;            // the baseline window plus one candidate scale
  // eta: the growth rates of the window telescope, but they are summed one by one as defined
  double eta = 0.0;
  for (int t = 2; t <= t_est; ++t) eta += hbar[t - 1] - hbar[t - 2];
  eta /= (double)(t_est - 1);
  for (int t = t_est + 1; t <= T; ++t) {
    const double g_t = hbar[t - 1] - hbar[t - 2], g_prev = hbar[t - 2] - hbar[t - 3];
    if (0.5 * (g_t + g_prev) <= alpha * eta) {
      *t_star = t;
      break;
    }
  }
  return NOVA_OK;
}

int nova_scale_ratio(int t, int t_star, double g_t, double tau, double lambda, double* ratio) {
  if (!ratio || tau == 0.0) return NOVA_ERR_INVALID_ARG;
  const double z = (double)(t - (t_star + 1)) / tau;
  *ratio = 1.0 / (1.0 + std::exp(-z)) - lambda * std::tanh(g_t);
  return NOVA_OK;
}

}  // extern "C"
