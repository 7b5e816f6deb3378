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
#include "nova_internal.h"

namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kWavesPerSimd = 3;   // resident waves per SIMD the grid is sized for (measured best of 1..8)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kClamp = -200.0f;   // e^-200 == 0 in fp32; keeps (m - x) * e finite for x = -inf

struct Row {
  float m;        // running maximum, wave uniform (-inf before the first element)
  float R, T;     // per-lane partial sums against m, excluding elements equal to m
  float cS, cT;   // wave-uniform sums of elements that once equalled the maximum
  int cnt;        // wave-uniform count of elements equal to the current m

  __device__ __forceinline__ void init() { m = -INFINITY; R = T = cS = cT = 0.f; cnt = 0; }

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
    const float d = x - m;                    // <= 0; -inf for x = -inf; NaN for NaN
    const bool is_max = (d == 0.0f);
    float e = __builtin_amdgcn_exp2f(d * kLog2e);
    cnt += __popcll(__ballot(is_max));
    e = is_max ? 0.0f : e;
    R += e;
    // (m - x) * e with the legacy multiply's 0 * inf = 0, so x = -inf (e = 0) adds nothing; NaN stays NaN
    float t;
    asm("v_mul_legacy_f32 %0, -%1, %2" : "=v"(t) : "v"(d), "v"(e));
    T += t;
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
    float Rw = wave_sum(R) + cS;
    float Tw = wave_sum(T) + cT;
    // S = cnt + Rw, one maximum instance split off for log1p
    float extra = Rw + (float)(cnt - 1);
    float H = log1pf(extra) + Tw / (1.0f + extra);
    if (m == -INFINITY || cnt < 1) H = __builtin_nanf("");   // empty or all -inf row: undefined
    return (H < 0.0f) ? 0.0f : H;                             // NaN passes through
  }
};

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
#pragma unroll
      for (int c = 0; c < CH; ++c)
        if (have[c]) {
#pragma unroll
          for (int i = 0; i < VN; ++i) cm = fmaxf(cm, buf[c].get(i));
        }
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


// Regular rows (every lane owns CH full 16-byte vectors in every chunk, no scalar tail): each wave
// walks rows  w, w + nwaves, ...  as a sequence of chunks and keeps one chunk of look-ahead in
// registers: the loads of chunk i+1 are in flight while the exp/accumulate work of chunk i runs, so
// the memory stream and the ALU work overlap inside every wave instead of alternating chip-wide.
template <typename T, int CH>
__global__ __launch_bounds__(kWavesPerBlock* NOVA_WAVE) void entropy_kernel(
    const T* __restrict__ logits, int64_t rows, int nchunk, int64_t stride, float* __restrict__ H) {
  using VT = Vec16<T>;
  constexpr int VN = VT::N;
  const int lane = threadIdx.x & (NOVA_WAVE - 1);
  const int64_t w0 = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / NOVA_WAVE;
  const int64_t nwaves = (int64_t)gridDim.x * kWavesPerBlock;
  if (w0 >= rows) return;                        // whole wave leaves together

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
    st.rebase(wave_max(cm));
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
      for (int i = 0; i < VN; ++i) st.add(buf[c].get(i));
  };
  auto finish_row = [&](int64_t row, Row& st) {
    const float h = st.finish();
    if (lane == 0) H[row] = h;
    st.init();
  };

  // item = (row, chunk); the items of this wave are walked row-major with the two buffers
  // alternating.  Every load below is unconditional straight-line code (the odd tail is peeled), so
  // the compiler's vmcnt bookkeeping lets the look-ahead loads stay in flight.
  struct Cursor { int64_t row; int chunk; };
  auto advance = [&](Cursor c) {
    ++c.chunk;
    if (c.chunk == nchunk) { c.chunk = 0; c.row += nwaves; }
    return c;
  };
  const int64_t my_rows = (rows - w0 + nwaves - 1) / nwaves;
  const int64_t n = my_rows * nchunk;
  Row st;
  st.init();
  Cursor ca = {w0, 0};
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

// Scale mean entropy of one image per workgroup: mean[b] = (sum_i H[b, i]) / N with a fixed summation order
// (thread t adds elements t, t + 256, ... in turn, then a fixed tree over the threads), so the result is the same
// bits on every run -- the layer-linkage ratio turns it into an integer keep count.  A NaN entropy gives NaN.
constexpr int kMeanThreads = 256;
__global__ __launch_bounds__(kMeanThreads) void row_mean_kernel(const float* __restrict__ H, int64_t rows_per_batch,
                                                                float* __restrict__ mean) {
  __shared__ float part[kMeanThreads];
  const float* h = H + (int64_t)blockIdx.x * rows_per_batch;
  float s = 0.0f;
  for (int64_t i = threadIdx.x; i < rows_per_batch; i += kMeanThreads) s += h[i];
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
