// Token predictive entropy H = -sum_v p(v) ln p(v), p = softmax(logits)
// (Sec. 3.3, "Adaptive Acceleration Activation", entropy equation; the optional
// per-batch-row mean is the scale mean entropy of the same section).
//
// Bandwidth-bound: every logit is read from HBM exactly once.  One wave64 owns one row at a
// time and walks several rows.  A row is consumed in chunks of CH 16-byte vectors per lane; the
// next chunk (of this or the next row) is already in flight while the current one is reduced.
// Per chunk the wave agrees on a running maximum m, so all lanes accumulate against the same m
// and the final combine is a plain wave sum.
//
// With S = sum_v e^{x_v - m} and T = sum_v (m - x_v) e^{x_v - m}:  H = ln S + T / S.
// Both terms are non-negative, so nothing cancels.  To keep relative accuracy when H
// is tiny (one dominant logit) the elements equal to m are counted, not summed:
// S = cnt + R with R = sum over x_v < m, and H = log1p(R + cnt - 1) + T / (R + cnt).
#include <algorithm>

#include "common.h"
#include "entropy_core.h"
#include "nova_internal.h"

namespace {

using namespace entropy_core;

// Any shape: one row per wave, lanes past the row's end masked.
template <typename T, int CH>
__global__ __launch_bounds__(kWavesPerBlock* NOVA_WAVE) void entropy_generic_kernel(
    const T* __restrict__ logits, int64_t rows, int V, int64_t stride, float* __restrict__ H, int vec_ok) {
  using VT = Vec16<T>;
  constexpr int VN = VT::N;
  const int lane = threadIdx.x & (NOVA_WAVE - 1);
  const int wave = threadIdx.x / NOVA_WAVE;
  const int64_t row = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  if (row >= rows) return;                       // whole wave leaves together
  const T* p = logits + row * stride;

  Row st;
  st.init();

  int done = 0;
  if (vec_ok) {
    const int nvec = V / VN;                     // full 16-byte vectors in the row
    for (int v0 = 0; v0 < nvec; v0 += CH * NOVA_WAVE) {
      VT buf[CH];
      bool have[CH];
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        int vi = v0 + c * NOVA_WAVE + lane;
        have[c] = vi < nvec;
        if (have[c]) buf[c].load(p + (int64_t)vi * VN);
      }
      float cm = -INFINITY;
      bool unordered = false;                    // the maximum drops NaNs: they are caught here
#pragma unroll
      for (int c = 0; c < CH; ++c)
        if (have[c]) {
#pragma unroll
          for (int i = 0; i < VN; i += 2) {
            const float x0 = buf[c].get(i), x1 = buf[c].get(i + 1);
            cm = fmaxf(cm, fmaxf(x0, x1));
            unordered = unordered || __builtin_isunordered(x0, x1);
          }
        }
      if (__any(unordered)) st.nan = true;
      st.rebase(wave_max(cm));
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        // have[c] is false only in the last, partial sweep; keep ballots wave-wide
        if (__all(have[c])) {
#pragma unroll
          for (int i = 0; i < VN; ++i) st.add(buf[c].get(i));
        } else if (__any(have[c])) {
#pragma unroll
          for (int i = 0; i < VN; ++i) st.add_masked(have[c] ? buf[c].get(i) : 0.0f, have[c]);
        }
      }
    }
    done = nvec * VN;
  }
  // scalar tail (or the whole row when it is not 16-byte aligned)
  for (int e0 = done; e0 < V; e0 += NOVA_WAVE) {
    int ei = e0 + lane;
    bool valid = ei < V;
    float x = valid ? ld_f32(p + ei) : -INFINITY;
    st.rebase(wave_max(x));
    st.add_masked(valid ? x : 0.0f, valid);
  }

  float h = st.finish();
  if (lane == 0) H[row] = h;
}


// Regular rows: each wave walks rows  w, w + nwaves, ...  (entropy_core.h: walk_rows).
template <typename T, int CH>
__global__ __launch_bounds__(kWavesPerBlock* NOVA_WAVE) void entropy_kernel(
    const T* __restrict__ logits, int64_t rows, int nchunk, int64_t stride, float* __restrict__ H) {
  const int lane = threadIdx.x & (NOVA_WAVE - 1);
  const int64_t w0 = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / NOVA_WAVE;
  const int64_t nwaves = (int64_t)gridDim.x * kWavesPerBlock;
  if (w0 >= rows) return;                        // whole wave leaves together
  walk_rows<T, CH>(logits, w0, nwaves, (rows - w0 + nwaves - 1) / nwaves, nchunk, stride, lane,
                   [&](int64_t row, float h) { if (lane == 0) H[row] = h; });
}

// Scale mean entropy of one image per workgroup: mean[b] = (sum_i H[b, i]) / N with a fixed summation order
// (thread t adds its contiguous share of the elements in index order, then a fixed tree over the threads), so the
// result is the same bits on every run: the layer-linkage ratio turns it into an integer keep count.  A NaN
// entropy gives NaN.
constexpr int kMeanThreads = 256;
__global__ __launch_bounds__(kMeanThreads) void row_mean_kernel(const float* __restrict__ H, int64_t rows_per_batch,
                                                                float* __restrict__ mean) {
  __shared__ float part[kMeanThreads];
  const float* h = H + (int64_t)blockIdx.x * rows_per_batch;
  float s = 0.0f;
  const int64_t ipt = (rows_per_batch + kMeanThreads - 1) / kMeanThreads;
  const int64_t i0 = std::min<int64_t>(threadIdx.x * ipt, rows_per_batch), i1 = std::min<int64_t>(i0 + ipt, rows_per_batch);
  for (int64_t i = i0; i < i1; ++i) s += h[i];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int o = kMeanThreads / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) mean[blockIdx.x] = part[0] / (float)rows_per_batch;
}

template <typename T, int CH>
void launch_regular(hipStream_t st, int num_cus, const T* logits, int64_t rows, int nchunk, int64_t stride, float* H) {
  // at most kWavesPerSimd resident waves per SIMD, each walking several rows
  const int64_t max_blocks = (int64_t)num_cus * 4 * kWavesPerSimd / kWavesPerBlock;
  const unsigned grid = (unsigned)std::min<int64_t>((rows + kWavesPerBlock - 1) / kWavesPerBlock, max_blocks);
  entropy_kernel<T, CH><<<grid, kWavesPerBlock * NOVA_WAVE, 0, st>>>(logits, rows, nchunk, stride, H);
}

template <typename T>
hipError_t launch_t(hipStream_t st, int num_cus, const T* logits, int64_t rows_per_batch, int batch, int V,
                    int64_t stride, float* H, float* mean) {
  constexpr int VN = Vec16<T>::N;
  const int64_t rows = rows_per_batch * batch;
  const int vec_ok = ((reinterpret_cast<uintptr_t>(logits) & 15) == 0) &&
                     ((stride * (int64_t)sizeof(T)) % 16 == 0);
  const int per_sweep = NOVA_WAVE * VN;            // elements one 16-byte vector per lane covers
  if (vec_ok && V % per_sweep == 0) {
    const int sweeps = V / per_sweep;
    if (sweeps % 4 == 0) launch_regular<T, 4>(st, num_cus, logits, rows, sweeps / 4, stride, H);
    else if (sweeps % 2 == 0) launch_regular<T, 2>(st, num_cus, logits, rows, sweeps / 2, stride, H);
    else launch_regular<T, 1>(st, num_cus, logits, rows, sweeps, stride, H);
  } else {
    const unsigned grid = (unsigned)((rows + kWavesPerBlock - 1) / kWavesPerBlock);
    entropy_generic_kernel<T, 8><<<grid, kWavesPerBlock * NOVA_WAVE, 0, st>>>(logits, rows, V, stride, H, vec_ok);
  }
  if (mean) return launch_row_mean(st, H, rows_per_batch, batch, mean);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_row_mean(hipStream_t st, const float* H, int64_t rows_per_batch, int batch, float* mean) {
  row_mean_kernel<<<batch, kMeanThreads, 0, st>>>(H, rows_per_batch, mean);
  return hipGetLastError();
}

hipError_t launch_entropy(hipStream_t st, int num_cus, const void* logits, int dtype, int64_t rows_per_batch,
                          int batch, int V, int64_t stride, float* H, float* mean) {
  if (dtype == NOVA_BF16)
    return launch_t<bf16_t>(st, num_cus, static_cast<const bf16_t*>(logits), rows_per_batch, batch, V, stride, H,
                            mean);
  return launch_t<float>(st, num_cus, static_cast<const float*>(logits), rows_per_batch, batch, V, stride, H, mean);
}
