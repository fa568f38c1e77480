// Three-dimensional tropical convolution layers (paper Sec. 3.2, three-dimensional base operators MinPlus3d /
// MaxPlus3d and layers (iii) - (vi); Sec. 3.3 compound / parallel) on volumes x [N, C_in, D, H, W] with kernels
// [C_out, C_in, KD, KH, KW].  The saved winner is the flattened tap k = ((c*KD + a)*KH + i)*KW + j.
//
// These are plain kernels for any window, stride, padding and dilation: one thread per output in the forward
// pass (consecutive threads own consecutive ow, so reads of x and all writes are coalesced), a scatter with
// float atomics for the input gradient.  The kernel gradient needs no geometry (it is a histogram of the
// winners per output channel) and runs on the two-dimensional histogram kernel.  fp32 only.
#include "tconv_internal.h"

namespace tconv {
namespace {

// One pass over the window of every input channel for both branches.  Inside a channel strict compares in
// ascending tap order keep the lowest tap; across channels strict compares in ascending order keep the lowest
// channel, which for the full-window layers is the lowest k overall.
template <int MODE>
__global__ __launch_bounds__(256) void fwd3d_kernel(Params3 p, const float* __restrict__ x,
                                                    const float* __restrict__ w_min,
                                                    const float* __restrict__ w_max,
                                                    const float* __restrict__ alpha,
                                                    const float* __restrict__ beta, float* __restrict__ y,
                                                    float* __restrict__ y_min, float* __restrict__ y_max,
                                                    int32_t* __restrict__ idx_min, int32_t* __restrict__ idx_max) {
  constexpr bool DO_MIN = mode_has_min(MODE), DO_MAX = mode_has_max(MODE);
  constexpr bool MIN_OUTER_MAX = (MODE == TCONV_MINPLUS_MAX);  // layer (iii): max over channels of the min-plus operator
  constexpr bool MAX_OUTER_MIN = (MODE == TCONV_MAXPLUS_MIN);  // layer (vi)
  const size_t ovol = (size_t)p.Do * p.Ho * p.Wo;
  const size_t total = (size_t)p.N * p.C_out * ovol;
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= total) return;
  const int ow = (int)(o % p.Wo);
  const int oh = (int)((o / p.Wo) % p.Ho);
  const int od = (int)((o / ((size_t)p.Wo * p.Ho)) % p.Do);
  const int co = (int)((o / ovol) % p.C_out);
  const int n = (int)(o / (ovol * p.C_out));
  const size_t vol = (size_t)p.D * p.H * p.W;
  const int KK = p.KD * p.KH * p.KW;
  const float* xn = x + (size_t)n * p.C_in * vol;
  const float* wa = DO_MIN ? w_min + (size_t)co * p.K : nullptr;
  const float* wb = DO_MAX ? w_max + (size_t)co * p.K : nullptr;
  const int id0 = od * p.sd - p.pd, ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
  float bmin = MIN_OUTER_MAX ? -INFINITY : INFINITY, bmax = MAX_OUTER_MIN ? INFINITY : -INFINITY;
  int kmin = 0, kmax = 0;
  for (int c = 0; c < p.C_in; ++c) {
    const float* xc = xn + (size_t)c * vol;
    float vmin = INFINITY, vmax = -INFINITY;  // identities of the inner operators
    int tmin = 0, tmax = 0, t = 0;
    for (int a = 0; a < p.KD; ++a) {
      const int id = id0 + a * p.dd;
      const bool dv = (id >= 0 && id < p.D);
      for (int i = 0; i < p.KH; ++i) {
        const int ih = ih0 + i * p.dh;
        const bool rv = dv && (ih >= 0 && ih < p.H);
        for (int j = 0; j < p.KW; ++j, ++t) {
          const int iw = iw0 + j * p.dw;
          if (!rv || iw < 0 || iw >= p.W) continue;
          const float xv = xc[((size_t)id * p.H + ih) * p.W + iw];
          if (DO_MIN) {
            const float s = __fadd_rn(xv, wa[c * KK + t]);
            if (s < vmin) { vmin = s; tmin = t; }
          }
          if (DO_MAX) {
            const float s = __fadd_rn(xv, wb[c * KK + t]);
            if (s > vmax) { vmax = s; tmax = t; }
          }
        }
      }
    }
    if (DO_MIN && (MIN_OUTER_MAX ? (vmin > bmin) : (vmin < bmin))) { bmin = vmin; kmin = c * KK + tmin; }
    if (DO_MAX && (MAX_OUTER_MIN ? (vmax < bmax) : (vmax > bmax))) { bmax = vmax; kmax = c * KK + tmax; }
  }
  float out;
  if (!DO_MIN) out = bmax;
  else if (!DO_MAX) out = bmin;
  else out = combine(alpha ? alpha[co] : 1.0f, bmin, beta ? beta[co] : 1.0f, bmax);
  y[o] = out;
  if (DO_MIN) {
    if (y_min) y_min[o] = bmin;
    idx_min[o] = kmin;
  }
  if (DO_MAX) {
    if (y_max) y_max[o] = bmax;
    idx_max[o] = kmax;
  }
}

// grad_x[n, c*, id*, ih*, iw*] += g_b for every output and live branch (zero-filled first).  MODE is a backward
// mode: MAX, MIN, COMPOUND or PARALLEL.
template <int MODE>
__global__ __launch_bounds__(256) void bwd3d_input_kernel(Params3 p, BwdArgs a, float* __restrict__ grad_x) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool SCALED = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  const size_t ovol = (size_t)p.Do * p.Ho * p.Wo;
  const size_t total = (size_t)p.N * p.C_out * ovol;
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= total) return;
  const int ow = (int)(o % p.Wo);
  const int oh = (int)((o / p.Wo) % p.Ho);
  const int od = (int)((o / ((size_t)p.Wo * p.Ho)) % p.Do);
  const int co = (int)((o / ovol) % p.C_out);
  const int n = (int)(o / (ovol * p.C_out));
  const size_t vol = (size_t)p.D * p.H * p.W;
  const int KHW = p.KH * p.KW, KK = p.KD * KHW;
  float* gxn = grad_x + (size_t)n * p.C_in * vol;
  const float g = a.gy[o];
  auto deposit = [&](int k, float v) {
    const int c = k / KK, t = k - c * KK, ta = t / KHW, r = t - ta * KHW, ti = r / p.KW, tj = r - ti * p.KW;
    const int id = od * p.sd - p.pd + ta * p.dd, ih = oh * p.sh - p.ph + ti * p.dh, iw = ow * p.sw - p.pw + tj * p.dw;
    // a winner written by the forward pass is inside the volume; the test keeps a corrupted index in bounds
    if ((unsigned)c < (unsigned)p.C_in && (unsigned)id < (unsigned)p.D && (unsigned)ih < (unsigned)p.H &&
        (unsigned)iw < (unsigned)p.W)
      atomicAdd(gxn + (size_t)c * vol + ((size_t)id * p.H + ih) * p.W + iw, v);
  };
  if (DO_MIN) deposit(a.idx_min[o], (SCALED && a.alpha) ? a.alpha[co] * g : g);
  if (DO_MAX) deposit(a.idx_max[o], (SCALED && a.beta) ? a.beta[co] * g : g);
}

__global__ __launch_bounds__(256) void fill3d_zero_kernel(float* __restrict__ p, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0.f;
}

template <int MODE>
hipError_t launch_fwd(const Params3& p, const FwdArgs& a, hipStream_t s) {
  const size_t total = (size_t)p.N * p.C_out * p.Do * p.Ho * p.Wo;
  hipLaunchKernelGGL(fwd3d_kernel<MODE>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p, (const float*)a.x,
                     (const float*)a.w_min, (const float*)a.w_max, a.alpha, a.beta, (float*)a.y, (float*)a.y_min,
                     (float*)a.y_max, a.idx_min, a.idx_max);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_forward_3d(const Params3& p, const FwdArgs& a, hipStream_t s) {
  switch (p.mode) {
    case TCONV_MAX: return launch_fwd<TCONV_MAX>(p, a, s);
    case TCONV_MIN: return launch_fwd<TCONV_MIN>(p, a, s);
    case TCONV_COMPOUND: return launch_fwd<TCONV_COMPOUND>(p, a, s);
    case TCONV_PARALLEL: return launch_fwd<TCONV_PARALLEL>(p, a, s);
    case TCONV_MINPLUS_MAX: return launch_fwd<TCONV_MINPLUS_MAX>(p, a, s);
    default: return launch_fwd<TCONV_MAXPLUS_MIN>(p, a, s);
  }
}

// p.mode is a backward mode here (the mixed layers arrive as MIN / MAX)
hipError_t launch_backward_input_3d(const Params3& p, const BwdArgs& a, float* grad_x, hipStream_t s) {
  const size_t nx = (size_t)p.N * p.C_in * p.D * p.H * p.W;
  size_t zb = (nx + 255) / 256;
  if (zb > 8192) zb = 8192;
  hipLaunchKernelGGL(fill3d_zero_kernel, dim3((unsigned)zb), dim3(256), 0, s, grad_x, nx);
  const size_t total = (size_t)p.N * p.C_out * p.Do * p.Ho * p.Wo;
  const dim3 grid((unsigned)((total + 255) / 256));
  switch (p.mode) {
    case TCONV_MAX: hipLaunchKernelGGL(bwd3d_input_kernel<TCONV_MAX>, grid, dim3(256), 0, s, p, a, grad_x); break;
    case TCONV_MIN: hipLaunchKernelGGL(bwd3d_input_kernel<TCONV_MIN>, grid, dim3(256), 0, s, p, a, grad_x); break;
    case TCONV_COMPOUND: hipLaunchKernelGGL(bwd3d_input_kernel<TCONV_COMPOUND>, grid, dim3(256), 0, s, p, a, grad_x); break;
    default: hipLaunchKernelGGL(bwd3d_input_kernel<TCONV_PARALLEL>, grid, dim3(256), 0, s, p, a, grad_x); break;
  }
  return hipGetLastError();
}

}  // namespace tconv
