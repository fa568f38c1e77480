// Tiled 3x3 forward, bf16 storage: the instantiations that read bf16 rows, and the widening of the kernel tensors.
// The kernel is in fwd_tiled3x3_kernel.h, the choice of its form in fwd_tiled3x3_launch.h.
#include "fwd_tiled3x3_launch.h"

namespace tconv {
namespace {

// bf16 kernel tensors are widened to fp32 once, into the workspace
__global__ __launch_bounds__(256) void bf16_to_f32_kernel(const bf16_t* __restrict__ src,
                                                          float* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    dst[i] = __uint_as_float(((unsigned)src[i]) << 16);
}

void widen(const void* src, float* dst, size_t n, hipStream_t s) {
  size_t blocks = (n + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(bf16_to_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const bf16_t*)src, dst, n);
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

}  // namespace

// workspace: fp32 copies of the kernel tensors (forward_tiled3x3_workspace)
hipError_t launch_forward_tiled3x3_bf16(const Params& p, const FwdArgs& a, void* workspace, hipStream_t s) {
  const size_t nw = (size_t)p.C_out * p.K;
  float* wa = (float*)workspace;
  float* wb = (float*)((char*)wa + align256(nw * 4));
  const float* wmin_f = nullptr;
  const float* wmax_f = nullptr;
  if (p.mode == TCONV_PARALLEL) {
    widen(a.w_min, wa, nw, s);
    widen(a.w_max, wb, nw, s);
    wmin_f = wa; wmax_f = wb;
  } else {
    widen(mode_has_max(p.mode) ? a.w_max : a.w_min, wa, nw, s);
    wmin_f = wmax_f = wa;
  }
  return launch_mode<bf16_t>(p, a.x, wmin_f, wmax_f, a, s);
}

}  // namespace tconv
