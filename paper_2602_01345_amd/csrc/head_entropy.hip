// Token entropy straight from a linear prediction head (Sec. 4, "Entropy Computation Overhead":
// the entropy is taken from the distributions decoding produces anyway; Sec. 3.3, "Adaptive
// Acceleration Activation": the entropy equation).  logits = hidden W^T + b are formed tile by tile
// on the matrix cores and reduced on the spot, so the [tokens, V] logits never reach HBM: the GEMM's
// entropy epilogue leaves one (max, S, T) partial per row and column tile, and the kernel here
// merges a row's partials: H = ln S + T / S with S = sum e^(x-m), T = sum (m-x) e^(x-m).
#include "common.h"
#include "epilogue.h"
#include "nova_internal.h"

namespace {

__global__ __launch_bounds__(256) void head_entropy_combine_kernel(const f32x4* __restrict__ part, int tiles_n,
                                                                   int M, float* __restrict__ H) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= M) return;
  const f32x4 a = part[row];
  float m = a[0], S = a[1], T = a[2];
  for (int t = 1; t < tiles_n; ++t) {
    const f32x4 b = part[(int64_t)t * M + row];
    entropy_merge(m, S, T, b[0], b[1], b[2]);
  }
  float h = logf(S) + T / S;
  h = h < 0.0f ? 0.0f : h;
  H[row] = h;
}

// Scratch of the allocation-free entry point (nova_head_entropy_static): the per-tile entropy partials live in
// this array instead of a caller's workspace.  Every GPU the library runs on holds its own copy at its own
// address; the array's name is only a host-side handle, the device address comes from hipGetSymbolAddress.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};       // device address of `scratch` on each device, set by head_entropy_static_init

}  // namespace

hipError_t head_entropy_static_init(int device) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  if (g_scratch_ptr[device]) return hipSuccess;
  int cur = -1;
  hipError_t e = hipGetDevice(&cur);
  if (e != hipSuccess) return e;
  if (cur != device && (e = hipSetDevice(device)) != hipSuccess) return e;
  void* p = nullptr;
  e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
  if (cur != device) (void)hipSetDevice(cur);
  if (e != hipSuccess) return e;
  g_scratch_ptr[device] = p;
  return hipSuccess;
}

void* head_entropy_static_scratch(int device) {
  return device >= 0 && device < kMaxDevices ? g_scratch_ptr[device] : nullptr;
}

size_t head_entropy_static_capacity() { return kStaticScratchBytes; }

// Bytes of partials the launch below really writes for this shape: one 16-byte partial per row and per column
// tile of the GEMM configuration the launcher picks.
size_t head_entropy_partial_bytes(const nova_ctx* ctx, int M, int V, int C) {
  const int bn = gemm_bf16_tile_cols(ctx, M, V, C);
  return (size_t)((V + bn - 1) / bn) * (size_t)M * sizeof(f32x4);
}

size_t head_entropy_workspace_bytes(int M, int V) {
  // one 16-byte partial per row and column tile; the narrowest tile configuration has 32 columns
  return (size_t)((V + 31) / 32) * (size_t)M * sizeof(f32x4);
}

hipError_t launch_head_entropy(const nova_ctx* ctx, hipStream_t st, const void* hidden, const void* w_head,
                               const void* b_head, int rows_per_batch, int batch, int C, int V, float* H,
                               float* mean, void* workspace) {
  const int M = rows_per_batch * batch;
  EpiParams<bf16_t> ep{};
  ep.bias = static_cast<const bf16_t*>(b_head);
  ep.ent_part = static_cast<f32x4*>(workspace);
  hipError_t e = launch_gemm_bf16(ctx, st, EPI_ENTROPY, hidden, w_head, M, V, C, ep);
  if (e != hipSuccess) return e;
  const int bn = gemm_bf16_tile_cols(ctx, M, V, C);
  head_entropy_combine_kernel<<<(M + 255) / 256, 256, 0, st>>>(ep.ent_part, (V + bn - 1) / bn, M, H);
  if (mean) return launch_row_mean(st, H, rows_per_batch, batch, mean);
  return hipGetLastError();
}
