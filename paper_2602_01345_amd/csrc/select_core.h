// Building blocks of the entropy-guided token selection (Sec. 3.3, "Dual-Linkage Acceleration", final sentence: the
// lowest-entropy tokens are pruned; Sec. 3.2: the highest-entropy tokens are maintained), written over the number
// of threads of the workgroup that runs them.  Everything is integer work on order-preserving keys:
// the result equals a stable sort (entropy descending, index ascending) bit for bit.
#pragma once
#include "common.h"

namespace select_core {


// 32-bit key whose unsigned order is the required numeric order: NaN lowest, -0 == +0
__device__ __forceinline__ uint32_t sort_key(float h) {
  uint32_t b = __float_as_uint(h);
  if ((b & 0x7fffffffu) > 0x7f800000u) return 0u;       // NaN: below every number
  if (b == 0x80000000u) b = 0u;                         // -0 == +0
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);    // -inf -> 0x007fffff > 0
}

// LDS scratch of one workgroup of NT threads; COPIES counters per histogram bin (32 = one per LDS bank)
template <int NT, int COPIES = 32>
struct Scratch {
  uint32_t hist[256];
  uint32_t hist_banked[256 * COPIES];    // [bin][copy]: copy = lane % COPIES
  uint32_t wave_sums[NT / NOVA_WAVE];
  uint32_t bin, remaining;
};

// exclusive prefix sum of v over the block's threads, in thread order; total in *total
template <int NT>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_sums, uint32_t* total) {
  constexpr int kWaves = NT / NOVA_WAVE;
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

// The k-th largest of the N keys key_at(0..N-1), 0 < k < N, by a 4-pass, 8-bit MSB radix select on LDS histograms:
// returns the threshold key; *remaining_out = how many of the keys equal to it are kept (the first ones in index
// order).  Keys of one image share their leading bits, so in the first passes nearly all keys fall into one or two
// bins: a single histogram would serialise its atomics on one address.  Each bin therefore has COPIES counters (32:
// one per LDS bank) and a lane adds to the counter of its own bank; the counters are summed (and cleared) after the
// pass.  Called by all NT threads of the workgroup.
template <int NT, int COPIES, typename KeyAt>
__device__ __forceinline__ uint32_t radix_select(KeyAt key_at, int N, int k, Scratch<NT, COPIES>& sc,
                                                 uint32_t* remaining_out) {
  constexpr int kCopies = COPIES;
  static_assert(NT == 256 || NT == 1024, "the counter sum below gives NT / 256 threads to every bin");
  constexpr int TPB = NT / 256;          // threads per bin in the counter sum
  const int tid = threadIdx.x;
  const int lane = tid & (NOVA_WAVE - 1);
  const int wave = tid / NOVA_WAVE;
  uint32_t prefix = 0, prefix_mask = 0, remaining = (uint32_t)k;
  for (int i = tid; i < 256 * kCopies; i += NT) sc.hist_banked[i] = 0;
  for (int shift = 24; shift >= 0; shift -= 8) {
    __syncthreads();
    for (int i = tid; i < N; i += NT) {
      uint32_t key = key_at(i);
      if ((key & prefix_mask) == prefix)
        atomicAdd(&sc.hist_banked[((key >> shift) & 255u) * kCopies + (lane & (kCopies - 1))], 1u);
    }
    __syncthreads();
    {
      // TPB threads per bin, COPIES / TPB counters each (walked from a bin-dependent start, so that the lanes of a
      // wave touch all banks); the counters are left at zero for the next pass
      constexpr int CPT = kCopies / TPB;
      const int bin = tid / TPB, q = tid % TPB;
      uint32_t s = 0;
#pragma unroll
      for (int j = 0; j < CPT; ++j) {
        const int c = bin * kCopies + q * CPT + ((j + bin) & (CPT - 1));
        s += sc.hist_banked[c];
        sc.hist_banked[c] = 0;
      }
#pragma unroll
      for (int o = 1; o < TPB; o <<= 1) s += __shfl_xor(s, o, NOVA_WAVE);
      if (q == 0) sc.hist[bin] = s;
    }
    __syncthreads();
    if (wave == 0) {
      uint32_t h0 = sc.hist[4 * lane], h1 = sc.hist[4 * lane + 1], h2 = sc.hist[4 * lane + 2], h3 = sc.hist[4 * lane + 3];
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
        sc.bin = 4u * lane + bin;
        sc.remaining = r;
      }
    }
    __syncthreads();
    prefix |= sc.bin << shift;
    prefix_mask |= 255u << shift;
    remaining = sc.remaining;
    // hist and bin / remaining are rewritten only behind further barriers of the next pass
  }
  *remaining_out = remaining;
  return prefix;
}

// Writes the ascending kept-index list and the mask of one image from the selection rule: every key above `thr` is
// kept, of the keys equal to it the first `remaining` in index order; all = keep everything, none = keep nothing.
// Two block-wide prefix sums over contiguous index ranges.  Entries [kept, pitch) of the index row are set to -1.
template <int NT, typename KeyAt>
__device__ __forceinline__ void compact(KeyAt key_at, int N, uint32_t thr, uint32_t remaining, bool all, bool none,
                                        int pitch, int32_t* __restrict__ out_idx, uint8_t* __restrict__ out_mask,
                                        uint32_t* wave_sums) {
  const int tid = threadIdx.x;
  const int ipt = (N + NT - 1) / NT;
  const int i0 = min(tid * ipt, N), i1 = min(i0 + ipt, N);
  uint32_t n_gt = 0, n_eq = 0;
  if (!none) {
    for (int i = i0; i < i1; ++i) {
      uint32_t key = key_at(i);
      n_gt += (all || key > thr);
      n_eq += (!all && key == thr);
    }
  }
  uint32_t tot;
  uint32_t eq_before = block_exclusive_scan<NT>(n_eq, wave_sums, &tot);
  uint32_t eq_take = 0;
  if (eq_before < remaining) eq_take = min(n_eq, remaining - eq_before);
  uint32_t pos = block_exclusive_scan<NT>(n_gt + eq_take, wave_sums, &tot);
  uint32_t eq_seen = eq_before;
  for (int i = i0; i < i1; ++i) {
    bool keep = false;
    if (!none) {
      uint32_t key = key_at(i);
      if (all || key > thr) keep = true;
      else if (key == thr) { keep = eq_seen < remaining; ++eq_seen; }
    }
    out_mask[i] = keep ? 1 : 0;
    if (keep && pos < (uint32_t)pitch) out_idx[pos++] = i;   // pos < k <= pitch by construction
  }
  // unused tail of the row's index list
  for (int i = (int)tot + tid; i < pitch; i += NT) out_idx[i] = -1;
}

}  // namespace select_core
