// Entropy-guided token selection: per batch row keep the k tokens that come first in
// the order (entropy descending, index ascending)  (Sec. 3.3, "Dual-Linkage
// Acceleration", final sentence; Sec. 3.2, the highest-entropy tokens are maintained).
//
// One 1024-thread workgroup per batch row.  Entropies are mapped to 32-bit keys whose
// unsigned order is the required numeric order (NaN lowest, -0 == +0), staged in LDS,
// and the k-th largest key is found by a 4-pass, 8-bit MSB radix select on LDS
// histograms.  Entropies of one row share their leading bits, so in the first passes
// nearly all keys fall into one or two bins: a single histogram would serialise its
// atomics on one address.  Each bin therefore has 32 counters, one per LDS bank, and a
// lane adds to the counter of its own bank; the 32 counters are summed (and cleared)
// after the pass.  Every key above the threshold is kept; of the keys equal to it the
// first (k - #above) in index order are kept.  Two block-wide prefix sums over
// contiguous index ranges turn that rule into the ascending index list and the mask.
// Integer compares only: the result equals a stable sort bit for bit.
#include "common.h"
#include "nova_internal.h"

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / NOVA_WAVE;
constexpr int kLdsKeys = 8192;   // rows up to this many tokens are staged in LDS
constexpr int kCopies = 32;      // counters per histogram bin, one per LDS bank
static_assert(kThreads == 256 * 4, "the counter sum below gives four threads to every bin");

__device__ __forceinline__ uint32_t sort_key(float h) {
  uint32_t b = __float_as_uint(h);
  if ((b & 0x7fffffffu) > 0x7f800000u) return 0u;       // NaN: below every number
  if (b == 0x80000000u) b = 0u;                         // -0 == +0
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);    // -inf -> 0x007fffff > 0
}

// exclusive prefix sum of v over the block's threads, in thread order; total in *total
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_sums, uint32_t* total) {
  const int lane = threadIdx.x & (NOVA_WAVE - 1);
  const int wave = threadIdx.x / NOVA_WAVE;
  uint32_t inc = v;
#pragma unroll
  for (int o = 1; o < NOVA_WAVE; o <<= 1) {
    uint32_t t = __shfl_up(inc, o, NOVA_WAVE);
    if (lane >= o) inc += t;
  }
  __syncthreads();                       // wave_sums may still be read from a previous scan
  if (lane == NOVA_WAVE - 1) wave_sums[wave] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    uint32_t s = wave_sums[w];
    if (w < wave) base += s;
    tot += s;
  }
  *total = tot;
  return base + inc - v;
}

template <bool STAGED>
__global__ __launch_bounds__(kThreads) void select_kernel(const float* __restrict__ H, int N, int k_uniform,
                                                          const int32_t* __restrict__ k_per_row,
                                                          int pitch, int32_t* __restrict__ idx,
                                                          uint8_t* __restrict__ mask) {
  __shared__ uint32_t keys_lds[STAGED ? kLdsKeys : 1];
  __shared__ uint32_t hist[256];
  __shared__ uint32_t hist_banked[256 * kCopies];   // [bin][copy]: copy = lane % 32 = the LDS bank
  __shared__ uint32_t wave_sums[kWaves];
  __shared__ uint32_t sh_bin, sh_remaining;

  const int tid = threadIdx.x;
  const int lane = tid & (NOVA_WAVE - 1);
  const int wave = tid / NOVA_WAVE;
  const int b = blockIdx.x;
  const float* h = H + (int64_t)b * N;
  int32_t* out_idx = idx + (int64_t)b * pitch;
  uint8_t* out_mask = mask + (int64_t)b * N;

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

  // ---- k-th largest key by MSB radix select --------------------------------
  uint32_t prefix = 0, prefix_mask = 0, remaining = (uint32_t)k;
  bool keep_all_ge = true;     // false when k == 0: nothing is kept
  if (k == 0) keep_all_ge = false;
  if (k > 0 && k < N) {
    for (int i = tid; i < 256 * kCopies; i += kThreads) hist_banked[i] = 0;
    for (int shift = 24; shift >= 0; shift -= 8) {
      __syncthreads();
      for (int i = tid; i < N; i += kThreads) {
        uint32_t key = key_at(i);
        if ((key & prefix_mask) == prefix)
          atomicAdd(&hist_banked[((key >> shift) & 255u) * kCopies + (lane & (kCopies - 1))], 1u);
      }
      __syncthreads();
      {
        // four threads per bin, eight counters each (walked from a bin-dependent start, so that the lanes of a
        // wave touch all banks); the counters are left at zero for the next pass
        const int bin = tid >> 2, q = tid & 3;
        uint32_t s = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int c = bin * kCopies + q * 8 + ((j + bin) & 7);
          s += hist_banked[c];
          hist_banked[c] = 0;
        }
        s += __shfl_xor(s, 1, NOVA_WAVE);
        s += __shfl_xor(s, 2, NOVA_WAVE);
        if (q == 0) hist[bin] = s;
      }
      __syncthreads();
      if (wave == 0) {
        uint32_t h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
        uint32_t s = h0 + h1 + h2 + h3;
        uint32_t suf = s;                        // sum over lanes >= this one (higher bins)
#pragma unroll
        for (int o = 1; o < NOVA_WAVE; o <<= 1) {
          uint32_t t = __shfl_down(suf, o, NOVA_WAVE);
          if (lane + o < NOVA_WAVE) suf += t;
        }
        uint32_t above = suf - s;
        if (above < remaining && remaining <= suf) {       // exactly one lane
          uint32_t r = remaining - above;
          uint32_t bin;
          if (r <= h3) { bin = 3; }
          else { r -= h3; if (r <= h2) { bin = 2; } else { r -= h2; if (r <= h1) { bin = 1; } else { r -= h1; bin = 0; } } }
          sh_bin = 4u * lane + bin;
          sh_remaining = r;
        }
      }
      __syncthreads();
      prefix |= sh_bin << shift;
      prefix_mask |= 255u << shift;
      remaining = sh_remaining;
      // hist and sh_* are rewritten only behind further barriers of the next pass
    }
  } else if (k == N) {
    prefix = 0; remaining = 0;       // every key >= 0: all kept through the "above" rule below
  }
  // threshold = prefix; keys > prefix kept; first `remaining` keys == prefix kept (k in (0,N));
  // for k == N treat everything as "above".
  const bool all = (k == N);

  // ---- compaction over contiguous index ranges -----------------------------
  const int ipt = (N + kThreads - 1) / kThreads;
  const int i0 = min(tid * ipt, N), i1 = min(i0 + ipt, N);
  uint32_t n_gt = 0, n_eq = 0;
  if (keep_all_ge) {
    for (int i = i0; i < i1; ++i) {
      uint32_t key = key_at(i);
      n_gt += (all || key > prefix);
      n_eq += (!all && key == prefix);
    }
  }
  uint32_t tot;
  uint32_t eq_before = block_exclusive_scan(n_eq, wave_sums, &tot);
  uint32_t eq_take = 0;
  if (eq_before < remaining) eq_take = min(n_eq, remaining - eq_before);
  uint32_t pos = block_exclusive_scan(n_gt + eq_take, wave_sums, &tot);
  uint32_t eq_seen = eq_before;
  for (int i = i0; i < i1; ++i) {
    bool keep = false;
    if (keep_all_ge) {
      uint32_t key = key_at(i);
      if (all || key > prefix) keep = true;
      else if (key == prefix) { keep = eq_seen < remaining; ++eq_seen; }
    }
    out_mask[i] = keep ? 1 : 0;
    if (keep && pos < (uint32_t)pitch) out_idx[pos++] = i;   // pos < k <= pitch by construction
  }
  // unused tail of the row's index list
  for (int i = (int)tot + tid; i < pitch; i += kThreads) out_idx[i] = -1;
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
