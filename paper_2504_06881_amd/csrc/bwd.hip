// Backward kernels: both route the output gradient through the saved winning-tap
// indices (sub-gradient of max / min: the whole gradient of a branch goes to the one
// x element and the one kernel element that produced the extremum).  Neither does
// any arithmetic beyond adds, so both are bound by reading gy and idx from HBM.
//
//   backward_input : grad_x[n, c*, ih*, iw*] += g_b   (scatter, hardware fp32 atomics)
//   backward_weight: grad_w_b[c_out, k*]    += g_b   (per-c_out LDS histogram, then flush)
//
// g_min = alpha[c_out]*gy and g_max = beta[c_out]*gy in compound / parallel mode
// (paper Sec. 3.3 definitions), g = gy in max / min mode.
#include "tconv_internal.h"

namespace tconv {

// Zero n floats: float4 stores over the 16-byte-aligned body, scalar stores for the ragged ends.
__global__ __launch_bounds__(256) void fill_zero_kernel(float* __restrict__ p, size_t n) {
  const size_t mis = (16 - ((uintptr_t)p & 15u)) & 15u;  // bytes up to the next 16-byte boundary
  size_t head = mis / 4;
  if (head > n) head = n;
  const size_t n4 = (n - head) / 4;
  const size_t tail0 = head + n4 * 4;
  float4* body = (float4*)(p + head);
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride)
    body[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  if (blockIdx.x == 0) {
    if (threadIdx.x < head) p[threadIdx.x] = 0.f;
    if (tail0 + threadIdx.x < n) p[tail0 + threadIdx.x] = 0.f;
  }
}

// A kernel rather than hipMemsetAsync, so that the call can sit inside a captured graph.
static void fill_zero(float* p, size_t n, hipStream_t s) {
  if (n == 0) return;
  size_t blocks = (n / 4 + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (blocks == 0) blocks = 1;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, n);
}

template <int MODE>
__global__ __launch_bounds__(256) void bwd_input_scatter_kernel(Params p, BwdArgs a,
                                                                float* __restrict__ grad_x) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX);
  constexpr bool DO_MAX = (MODE != TCONV_MIN);
  constexpr bool SCALED = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= total) return;
  const int ow = (int)(o % p.Wo);
  const int oh = (int)((o / p.Wo) % p.Ho);
  const int co = (int)((o / ((size_t)p.Wo * p.Ho)) % p.C_out);
  const int n = (int)(o / ((size_t)p.Wo * p.Ho * p.C_out));
  const float g = a.gy[o];
  float* gxn = grad_x + (size_t)n * p.C_in * p.H * p.W;
  const int kk = p.KH * p.KW;
  if (DO_MIN) {
    const int k = a.idx_min[o];
    const int c = k / kk, r = k - c * kk, i = r / p.KW, j = r - i * p.KW;
    const int ih = oh * p.sh - p.ph + i * p.dh, iw = ow * p.sw - p.pw + j * p.dw;
    const float gm = SCALED ? __fmul_rn(a.alpha ? a.alpha[co] : 1.0f, g) : g;
    if ((unsigned)c < (unsigned)p.C_in && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W)
      atomicAdd(gxn + ((size_t)c * p.H + ih) * p.W + iw, gm);
  }
  if (DO_MAX) {
    const int k = a.idx_max[o];
    const int c = k / kk, r = k - c * kk, i = r / p.KW, j = r - i * p.KW;
    const int ih = oh * p.sh - p.ph + i * p.dh, iw = ow * p.sw - p.pw + j * p.dw;
    const float gm = SCALED ? __fmul_rn(a.beta ? a.beta[co] : 1.0f, g) : g;
    if ((unsigned)c < (unsigned)p.C_in && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W)
      atomicAdd(gxn + ((size_t)c * p.H + ih) * p.W + iw, gm);
  }
}

hipError_t launch_backward_input(const Params& p, const BwdArgs& a, float* grad_x, hipStream_t s) {
  fill_zero(grad_x, (size_t)p.N * p.C_in * p.H * p.W, s);
  const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  switch (p.mode) {
    case TCONV_MAX:
      hipLaunchKernelGGL(bwd_input_scatter_kernel<TCONV_MAX>, dim3(blocks), dim3(256), 0, s, p, a, grad_x);
      break;
    case TCONV_MIN:
      hipLaunchKernelGGL(bwd_input_scatter_kernel<TCONV_MIN>, dim3(blocks), dim3(256), 0, s, p, a, grad_x);
      break;
    default:  // compound and parallel route gradients identically
      hipLaunchKernelGGL(bwd_input_scatter_kernel<TCONV_COMPOUND>, dim3(blocks), dim3(256), 0, s, p, a, grad_x);
      break;
  }
  return hipGetLastError();
}

// One block = one output channel x one slice of the batch.  The block keeps a K-bin
// fp32 histogram per destination tensor in LDS, adds every (n, oh, ow) item of its
// slice with LDS atomics, then flushes the non-zero bins with global atomics.
// NHIST = 1: a single destination (max, min, and compound where both branches share
// one grad_w); NHIST = 2: parallel (min branch -> grad_w_min, max branch -> grad_w_max).
template <int MODE>
__global__ __launch_bounds__(256) void bwd_weight_hist_kernel(Params p, BwdArgs a,
                                                              float* __restrict__ gw_min,
                                                              float* __restrict__ gw_max,
                                                              int n_per_block) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX);
  constexpr bool DO_MAX = (MODE != TCONV_MIN);
  constexpr bool SCALED = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  constexpr int NHIST = (MODE == TCONV_PARALLEL) ? 2 : 1;
  extern __shared__ float hist[];  // NHIST * K floats
  const int co = blockIdx.x;
  const int n0 = blockIdx.y * n_per_block;
  const int n1 = min(n0 + n_per_block, p.N);
  const int K = p.K;
  for (int k = threadIdx.x; k < NHIST * K; k += blockDim.x) hist[k] = 0.f;
  __syncthreads();
  float* hmin = hist;
  float* hmax = hist + (NHIST - 1) * K;
  const float ca = SCALED ? (a.alpha ? a.alpha[co] : 1.0f) : 1.0f;
  const float cb = SCALED ? (a.beta ? a.beta[co] : 1.0f) : 1.0f;
  const int plane = p.Ho * p.Wo;
  for (int n = n0; n < n1; ++n) {
    const size_t base = ((size_t)n * p.C_out + co) * plane;
    for (int q = threadIdx.x; q < plane; q += blockDim.x) {
      const float g = a.gy[base + q];
      if (DO_MIN) {
        const int k = a.idx_min[base + q];
        if ((unsigned)k < (unsigned)K) atomicAdd(hmin + k, SCALED ? __fmul_rn(ca, g) : g);
      }
      if (DO_MAX) {
        const int k = a.idx_max[base + q];
        if ((unsigned)k < (unsigned)K) atomicAdd(hmax + k, SCALED ? __fmul_rn(cb, g) : g);
      }
    }
  }
  __syncthreads();
  float* dmin = (MODE == TCONV_MAX) ? gw_max : gw_min;  // NHIST == 1: the single destination
  for (int k = threadIdx.x; k < K; k += blockDim.x) {
    const float v = hist[k];
    if (v != 0.f) atomicAdd(dmin + (size_t)co * K + k, v);
    if (NHIST == 2) {
      const float v2 = hmax[k];
      if (v2 != 0.f) atomicAdd(gw_max + (size_t)co * K + k, v2);
    }
  }
}

// Fallback for K too large for an LDS histogram: straight global atomics.
template <int MODE>
__global__ __launch_bounds__(256) void bwd_weight_scatter_kernel(Params p, BwdArgs a,
                                                                 float* __restrict__ gw_min,
                                                                 float* __restrict__ gw_max) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX);
  constexpr bool DO_MAX = (MODE != TCONV_MIN);
  constexpr bool SCALED = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= total) return;
  const int co = (int)((o / ((size_t)p.Wo * p.Ho)) % p.C_out);
  const float g = a.gy[o];
  if (DO_MIN) {
    const int k = a.idx_min[o];
    const float gm = SCALED ? __fmul_rn(a.alpha ? a.alpha[co] : 1.0f, g) : g;
    if ((unsigned)k < (unsigned)p.K) atomicAdd(gw_min + (size_t)co * p.K + k, gm);
  }
  if (DO_MAX) {
    const int k = a.idx_max[o];
    const float gm = SCALED ? __fmul_rn(a.beta ? a.beta[co] : 1.0f, g) : g;
    if ((unsigned)k < (unsigned)p.K) atomicAdd(gw_max + (size_t)co * p.K + k, gm);
  }
}

hipError_t launch_backward_weight(const Params& p, const BwdArgs& a, float* grad_w_min,
                                  float* grad_w_max, hipStream_t s) {
  const size_t wn = (size_t)p.C_out * p.K;
  float* gmin = grad_w_min;
  float* gmax = grad_w_max;
  if (p.mode == TCONV_COMPOUND) gmin = gmax = (grad_w_min ? grad_w_min : grad_w_max);
  if (p.mode != TCONV_MAX) fill_zero(gmin, wn, s);
  if (p.mode == TCONV_MAX || p.mode == TCONV_PARALLEL) fill_zero(gmax, wn, s);

  const int nhist = (p.mode == TCONV_PARALLEL) ? 2 : 1;
  const size_t lds = (size_t)nhist * p.K * sizeof(float);
  if (lds <= 64 * 1024) {
    // enough blocks to fill 256 CUs several times over, but at least one image per block
    int slices = (4096 + p.C_out - 1) / p.C_out;
    if (slices > p.N) slices = p.N;
    if (slices < 1) slices = 1;
    const int n_per_block = (p.N + slices - 1) / slices;
    slices = (p.N + n_per_block - 1) / n_per_block;
    dim3 grid(p.C_out, slices);
    switch (p.mode) {
      case TCONV_MAX:
        hipLaunchKernelGGL(bwd_weight_hist_kernel<TCONV_MAX>, grid, dim3(256), lds, s, p, a, gmin, gmax, n_per_block);
        break;
      case TCONV_MIN:
        hipLaunchKernelGGL(bwd_weight_hist_kernel<TCONV_MIN>, grid, dim3(256), lds, s, p, a, gmin, gmax, n_per_block);
        break;
      case TCONV_COMPOUND:
        hipLaunchKernelGGL(bwd_weight_hist_kernel<TCONV_COMPOUND>, grid, dim3(256), lds, s, p, a, gmin, gmax, n_per_block);
        break;
      default:
        hipLaunchKernelGGL(bwd_weight_hist_kernel<TCONV_PARALLEL>, grid, dim3(256), lds, s, p, a, gmin, gmax, n_per_block);
        break;
    }
  } else {
    const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    switch (p.mode) {
      case TCONV_MAX:
        hipLaunchKernelGGL(bwd_weight_scatter_kernel<TCONV_MAX>, dim3(blocks), dim3(256), 0, s, p, a, gmin, gmax);
        break;
      case TCONV_MIN:
        hipLaunchKernelGGL(bwd_weight_scatter_kernel<TCONV_MIN>, dim3(blocks), dim3(256), 0, s, p, a, gmin, gmax);
        break;
      default:
        hipLaunchKernelGGL(bwd_weight_scatter_kernel<TCONV_COMPOUND>, dim3(blocks), dim3(256), 0, s, p, a, gmin, gmax);
        break;
    }
  }
  return hipGetLastError();
}

}  // namespace tconv
