// Generic forward kernel: one thread per output element, any kernel size, stride,
// padding and dilation.  It exists for the shapes the tiled 3x3 kernel does not
// cover (and as the first correct GPU path); consecutive threads own consecutive
// ow, so x reads and all output writes are coalesced.
//
// Operator: paper Sec. 3.1 layers (iv) MinPlus-Min-Conv2d / (v) MaxPlus-Max-Conv2d
// (one extremum over all C_in*KH*KW taps) and the Sec. 3.3 compound / parallel
// combinations.  Padded taps are skipped (they hold the semiring identity and can
// never win) or, with zero padding (App. A.1.1: the unfold formulation pads with zeros), enter with input value +0;
// strict compares while k ascends keep the lowest winning tap.  The epilogue (bias, folded batch norm, residual;
// App. A.2, Sec. 5 TCNN BasicBlock) is applied to the combined output only.
#include "tconv_internal.h"

namespace tconv {

template <int MODE, typename T>
__global__ __launch_bounds__(256) void fwd_generic_kernel(Params p, FwdArgs a) {
  const T* __restrict__ x = (const T*)a.x;
  const T* __restrict__ w_min = (const T*)a.w_min;
  const T* __restrict__ w_max = (const T*)a.w_max;
  const float* __restrict__ alpha = a.alpha;
  const float* __restrict__ beta = a.beta;
  T* __restrict__ y = (T*)a.y;
  T* __restrict__ y_min = (T*)a.y_min;
  T* __restrict__ y_max = (T*)a.y_max;
  int32_t* __restrict__ idx_min = a.idx_min;
  int32_t* __restrict__ idx_max = a.idx_max;
  constexpr bool DO_MIN = (MODE != TCONV_MAX);
  constexpr bool DO_MAX = (MODE != TCONV_MIN);
  const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= total) return;
  const int ow = (int)(o % p.Wo);
  const int oh = (int)((o / p.Wo) % p.Ho);
  const int co = (int)((o / ((size_t)p.Wo * p.Ho)) % p.C_out);
  const int n = (int)(o / ((size_t)p.Wo * p.Ho * p.C_out));

  const T* xn = x + (size_t)n * p.C_in * p.H * p.W;
  const T* wmn = DO_MIN ? w_min + (size_t)co * p.K : nullptr;
  const T* wmx = DO_MAX ? w_max + (size_t)co * p.K : nullptr;

  float bmax = -INFINITY, bmin = INFINITY;
  int imax = 0, imin = 0;
  const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
  int k = 0;
  for (int c = 0; c < p.C_in; ++c) {
    const T* xc = xn + (size_t)c * p.H * p.W;
    for (int i = 0; i < p.KH; ++i) {
      const int ih = ih0 + i * p.dh;
      const bool rv = (ih >= 0 && ih < p.H);
      for (int j = 0; j < p.KW; ++j, ++k) {
        const int iw = iw0 + j * p.dw;
        const bool inside = rv && iw >= 0 && iw < p.W;
        if (!inside && !p.pad_zero) continue;
        const float xv = inside ? ld_f32(xc, (size_t)ih * p.W + iw) : 0.0f;
        if (MODE == TCONV_PARALLEL) {
          const float s1 = candidate<T>(xv, ld_f32(wmn, k));
          const float s2 = candidate<T>(xv, ld_f32(wmx, k));
          if (s1 < bmin) { bmin = s1; imin = k; }
          if (s2 > bmax) { bmax = s2; imax = k; }
        } else {
          const float s = candidate<T>(xv, ld_f32(DO_MAX ? wmx : wmn, k));
          if (DO_MAX && s > bmax) { bmax = s; imax = k; }
          if (DO_MIN && s < bmin) { bmin = s; imin = k; }
        }
      }
    }
  }
  float out;
  if (MODE == TCONV_MAX) out = bmax;
  else if (MODE == TCONV_MIN) out = bmin;
  else out = combine(alpha ? alpha[co] : 1.0f, bmin, beta ? beta[co] : 1.0f, bmax);
  st_f32(y, o, apply_epilogue<T>(out, a, co, o));
  if (DO_MIN) {
    if (y_min) st_f32(y_min, o, bmin);
    idx_min[o] = imin;
  }
  if (DO_MAX) {
    if (y_max) st_f32(y_max, o, bmax);
    idx_max[o] = imax;
  }
}

// Mixed layers (paper Sec. 3.1 (iii) MinPlus-Max-Conv2d, (vi) MaxPlus-Min-Conv2d): the window of every
// input channel is reduced on its own (strict compares, ascending taps: lowest tap), then the channel
// results with the opposite operator (strict compares, ascending channels: lowest channel).
template <bool OUTER_MAX, typename T>
__global__ __launch_bounds__(256) void fwd_mixed_generic_kernel(Params p, FwdArgs a) {
  const T* __restrict__ x = (const T*)a.x;
  const T* __restrict__ w = (const T*)(OUTER_MAX ? a.w_min : a.w_max);
  T* __restrict__ y = (T*)a.y;
  T* __restrict__ y_branch = (T*)(OUTER_MAX ? a.y_min : a.y_max);
  int32_t* __restrict__ idx = OUTER_MAX ? a.idx_min : a.idx_max;
  const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= total) return;
  const int ow = (int)(o % p.Wo);
  const int oh = (int)((o / p.Wo) % p.Ho);
  const int co = (int)((o / ((size_t)p.Wo * p.Ho)) % p.C_out);
  const int n = (int)(o / ((size_t)p.Wo * p.Ho * p.C_out));
  const T* xn = x + (size_t)n * p.C_in * p.H * p.W;
  const T* wr = w + (size_t)co * p.K;
  const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
  float best = OUTER_MAX ? -INFINITY : INFINITY;
  int ibest = 0, k = 0;
  for (int c = 0; c < p.C_in; ++c) {
    const T* xc = xn + (size_t)c * p.H * p.W;
    float v = OUTER_MAX ? INFINITY : -INFINITY;  // identity of the inner operator
    int kv = k;
    for (int i = 0; i < p.KH; ++i) {
      const int ih = ih0 + i * p.dh;
      const bool rv = (ih >= 0 && ih < p.H);
      for (int j = 0; j < p.KW; ++j, ++k) {
        const int iw = iw0 + j * p.dw;
        const bool inside = rv && iw >= 0 && iw < p.W;
        if (!inside && !p.pad_zero) continue;
        const float s = candidate<T>(inside ? ld_f32(xc, (size_t)ih * p.W + iw) : 0.0f, ld_f32(wr, k));
        if (OUTER_MAX ? (s < v) : (s > v)) { v = s; kv = k; }
      }
    }
    if (OUTER_MAX ? (v > best) : (v < best)) { best = v; ibest = kv; }
  }
  st_f32(y, o, apply_epilogue<T>(best, a, co, o));
  if (y_branch) st_f32(y_branch, o, best);
  idx[o] = ibest;
}

template <bool OUTER_MAX, typename T>
static hipError_t launch_mixed(const Params& p, const FwdArgs& a, hipStream_t s) {
  const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL((fwd_mixed_generic_kernel<OUTER_MAX, T>), dim3(blocks), dim3(256), 0, s, p, a);
  return hipGetLastError();
}

template <int MODE, typename T>
static hipError_t launch_t(const Params& p, const FwdArgs& a, hipStream_t s) {
  const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL((fwd_generic_kernel<MODE, T>), dim3(blocks), dim3(256), 0, s, p, a);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_m(const Params& p, const FwdArgs& a, hipStream_t s) {
  switch (p.mode) {
    case TCONV_MAX: return launch_t<TCONV_MAX, T>(p, a, s);
    case TCONV_MIN: return launch_t<TCONV_MIN, T>(p, a, s);
    case TCONV_COMPOUND: return launch_t<TCONV_COMPOUND, T>(p, a, s);
    case TCONV_PARALLEL: return launch_t<TCONV_PARALLEL, T>(p, a, s);
    case TCONV_MINPLUS_MAX: return launch_mixed<true, T>(p, a, s);
    default: return launch_mixed<false, T>(p, a, s);
  }
}

hipError_t launch_forward_generic(const Params& p, int dtype, const FwdArgs& a, hipStream_t s) {
  if (dtype == TCONV_F16) return launch_m<f16_t>(p, a, s);
  return dtype == TCONV_BF16 ? launch_m<bf16_t>(p, a, s) : launch_m<float>(p, a, s);
}

}  // namespace tconv
