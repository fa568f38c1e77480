// Forward kernel for one-row inputs with a long window: the raw-waveform stems of one-dimensional networks
// (paper Sec. 3.2, MinPlus1d / MaxPlus1d and the one-dimensional layers (iv) / (v); Sec. 3.3 compound and
// parallel combinations), e.g. 1 -> 64 channels, kernel length 80, stride 4.  Few input channels, so the
// two-dimensional design (input channels as the long axis) has nothing to iterate over; here the window is.
//
// A workgroup owns 256 consecutive outputs of one sequence and RT_TN output channels; a lane owns one output
// position.  The input span of the workgroup is staged once in LDS, de-interleaved by the stride
// (xs[r][m] = x[first + S*m + r]), so that for every tap the 64 lanes of a wave read 64 consecutive words.
// Kernel values are wave-uniform (scalar loads).  The loop walks the window in chunks of RT_CH = 8 taps: 8 adds,
// a v_min3 / v_max3 tree, then one compare, one select and one min / max per chunk, channel and branch keep the
// extremum and the CHUNK that first reached it (strict compares, chunks ascending).  Afterwards the 8 taps of
// that chunk are recomputed from LDS (input and a chunk-major copy of the kernels) and the first tap whose sum
// equals the extremum is the winner: the lowest flattened tap, as everywhere else.  Padding and the taps
// past the window end are NaN, which v_min3 / v_max3 ignore and no compare selects.
#include <type_traits>

#include "tconv_internal.h"

namespace tconv {
namespace {

constexpr int RT_TN = 8;    // output channels per workgroup
constexpr int RT_CH = 8;    // taps per tracked chunk (a multiple of every supported stride)
constexpr int RT_BL = 256;  // outputs (threads) per workgroup
constexpr int RT_M = 320;   // words per LDS row: 256 lanes + up to 64 steps of the window
constexpr int RT_WS = 9;    // LDS words per chunk of kernel values (odd: the chunks of different lanes spread over the banks)
constexpr size_t RT_LDS_MAX = 48 * 1024;

__device__ __forceinline__ float min8(const float* s) {
  return fminf(fminf(fminf(fminf(s[0], s[1]), s[2]), fminf(s[3], s[4])), fminf(fminf(s[5], s[6]), s[7]));
}
__device__ __forceinline__ float max8(const float* s) {
  return fmaxf(fmaxf(fmaxf(fmaxf(s[0], s[1]), s[2]), fmaxf(s[3], s[4])), fmaxf(fmaxf(s[5], s[6]), s[7]));
}

template <int MODE, int S>
__global__ __launch_bounds__(RT_BL) void fwd_row_kernel(Params p, const float* __restrict__ x,
                                                        const float* __restrict__ w_min,
                                                        const float* __restrict__ w_max,
                                                        const float* __restrict__ alpha,
                                                        const float* __restrict__ beta, float* __restrict__ y,
                                                        float* __restrict__ y_min, float* __restrict__ y_max,
                                                        int32_t* __restrict__ idx_min, int32_t* __restrict__ idx_max,
                                                        int nch, unsigned inv_nch) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO_W = (MODE == TCONV_PARALLEL);
  static_assert(RT_CH % S == 0, "a chunk starts at the first row of the de-interleaved tile");
  HIP_DYNAMIC_SHARED(float, lds)
  const int K = p.KW, G = p.C_in * nch;
  float* xs = lds;                       // [C_in][S][RT_M]
  float* ws = lds + p.C_in * S * RT_M;   // [kernel set][RT_TN][G][RT_WS]
  const int tid = threadIdx.x;
  const int n = blockIdx.z, co0 = blockIdx.y * RT_TN, l0 = blockIdx.x * RT_BL;
  const float nan = __uint_as_float(0x7fc00000u);

  // input span of the workgroup, every input channel
  const float* xn = x + (size_t)n * p.C_in * p.W;
  const int first = l0 * S - p.pw;
  for (int ci = 0; ci < p.C_in; ++ci)
    for (int e = tid; e < S * RT_M; e += RT_BL) {
      const int pos = first + e;
      float v = nan;
      if (pos >= 0 && pos < p.W) v = xn[(size_t)ci * p.W + pos];
      xs[(ci * S + (e % S)) * RT_M + e / S] = v;
    }
  // chunk-major copy of the kernels of the workgroup's channels (read only when the winners are resolved)
  for (int set = 0; set < (TWO_W ? 2 : 1); ++set) {
    const float* wsrc = (set == 0 && DO_MIN) ? w_min : w_max;
    for (int c = 0; c < RT_TN; ++c) {
      const int co = min(co0 + c, p.C_out - 1);
      for (int ci = 0; ci < p.C_in; ++ci)
        for (int t = tid; t < nch * RT_CH; t += RT_BL) {
          float v = nan;
          if (t < K) v = wsrc[((size_t)co * p.C_in + ci) * K + t];
          ws[((set * RT_TN + c) * G + ci * nch + t / RT_CH) * RT_WS + t % RT_CH] = v;
        }
    }
  }
  __syncthreads();

  float bmin[RT_TN], bmax[RT_TN];
  int cmin[RT_TN], cmax[RT_TN];  // winning chunk: channel * nch + chunk
#pragma unroll
  for (int c = 0; c < RT_TN; ++c) {
    bmin[c] = INFINITY; bmax[c] = -INFINITY;
    cmin[c] = 0; cmax[c] = 0;
  }

  for (int ci = 0; ci < p.C_in; ++ci) {
    for (int ch = 0; ch < nch; ++ch) {
      const int k0 = ch * RT_CH, g = ci * nch + ch;
      const float* xr = xs + ci * S * RT_M + tid + ch * (RT_CH / S);
      auto chunk = [&](auto full_c) {
        constexpr bool FULL = decltype(full_c)::value;
        float xv[RT_CH];
#pragma unroll
        for (int j = 0; j < RT_CH; ++j) {
          xv[j] = xr[(j % S) * RT_M + j / S];
          if (!FULL && k0 + j >= K) xv[j] = nan;
        }
        // kernel values of channel slot c (a surplus slot reads the last channel and stores nothing).  With two
        // kernels they are requested one channel ahead, so that the scalar loads run under the arithmetic of
        // the channel before; with one kernel the higher occupancy of the plain order hides them better.
        float wa[2][RT_CH], wb[2][RT_CH];
        auto load_w = [&](int c) {
          const int co = min(co0 + c, p.C_out - 1);
          const size_t wb0 = ((size_t)co * p.C_in + ci) * K;
#pragma unroll
          for (int j = 0; j < RT_CH; ++j) {
            const int t = FULL ? k0 + j : min(k0 + j, K - 1);
            if (DO_MIN) wa[c & 1][j] = w_min[wb0 + t];
            if (DO_MAX && MODE != TCONV_COMPOUND) wb[c & 1][j] = w_max[wb0 + t];
          }
        };
        if (TWO_W) load_w(0);
#pragma unroll
        for (int c = 0; c < RT_TN; ++c) {
          if (!TWO_W) load_w(c);
          else if (c + 1 < RT_TN) load_w(c + 1);
          float s1[RT_CH], s2[RT_CH];
#pragma unroll
          for (int j = 0; j < RT_CH; ++j) {
            if (DO_MIN) s1[j] = __fadd_rn(xv[j], wa[c & 1][j]);
            if (DO_MAX) s2[j] = (MODE == TCONV_COMPOUND) ? s1[j] : __fadd_rn(xv[j], wb[c & 1][j]);
          }
          if (DO_MIN) {
            const float m = min8(s1);
            cmin[c] = (m < bmin[c]) ? g : cmin[c];
            bmin[c] = fminf(bmin[c], m);
          }
          if (DO_MAX) {
            const float m = max8(s2);
            cmax[c] = (m > bmax[c]) ? g : cmax[c];
            bmax[c] = fmaxf(bmax[c], m);
          }
        }
      };
      if (k0 + RT_CH <= K) chunk(std::true_type{});
      else chunk(std::false_type{});
    }
  }

  // exact tap: the first of the 8 taps of the winning chunk whose sum equals the extremum.  An extremum that
  // never left its start value (inputs of -inf / +inf only) keeps tap 0, as a strict compare from tap 0 does.
  auto refine = [&](int set, int c, int g, float best, float start) -> int {
    const int ci = (p.C_in > 1) ? (int)(inv_nch ? __umulhi((unsigned)g, inv_nch) : (unsigned)g) : 0;
    const int ch = g - ci * nch;
    const float* xr = xs + ci * S * RT_M + tid + ch * (RT_CH / S);
    const float* wr = ws + ((set * RT_TN + c) * G + g) * RT_WS;
    const int k0 = ci * K + ch * RT_CH;
    int res = k0;
#pragma unroll
    for (int j = RT_CH - 1; j >= 0; --j) {
      const float sum = __fadd_rn(xr[(j % S) * RT_M + j / S], wr[j]);
      res = (sum == best) ? k0 + j : res;
    }
    return best == start ? 0 : res;
  };

  const int l = l0 + tid;
  const bool ok = l < p.Wo;
#pragma unroll
  for (int c = 0; c < RT_TN; ++c) {
    const int co = co0 + c;
    if (co >= p.C_out) break;
    const size_t o = ((size_t)n * p.C_out + co) * p.Wo + l;
    int imin = 0, imax = 0;
    if (DO_MIN) imin = refine(0, c, cmin[c], bmin[c], INFINITY);
    if (DO_MAX) imax = refine(TWO_W ? 1 : 0, c, cmax[c], bmax[c], -INFINITY);
    float out;
    if (!DO_MIN) out = bmax[c];
    else if (!DO_MAX) out = bmin[c];
    else out = combine(alpha ? alpha[co] : 1.0f, bmin[c], beta ? beta[co] : 1.0f, bmax[c]);
    if (ok) {
      y[o] = out;
      if (DO_MIN) {
        if (y_min) y_min[o] = bmin[c];
        idx_min[o] = imin;
      }
      if (DO_MAX) {
        if (y_max) y_max[o] = bmax[c];
        idx_max[o] = imax;
      }
    }
  }
}

int chunks_of(const Params& p) { return (p.KW + RT_CH - 1) / RT_CH; }

size_t lds_bytes(const Params& p) {
  const size_t sets = p.mode == TCONV_PARALLEL ? 2 : 1;
  return ((size_t)p.C_in * p.sw * RT_M + sets * RT_TN * p.C_in * chunks_of(p) * RT_WS) * sizeof(float);
}

template <int MODE, int S>
hipError_t launch_s(const Params& p, const FwdArgs& a, hipStream_t s) {
  const int nch = chunks_of(p);
  const unsigned inv = nch > 1 ? (unsigned)(0x100000000ull / (unsigned)nch) + 1u : 0u;
  const dim3 grid((unsigned)((p.Wo + RT_BL - 1) / RT_BL), (unsigned)((p.C_out + RT_TN - 1) / RT_TN), (unsigned)p.N);
  hipLaunchKernelGGL((fwd_row_kernel<MODE, S>), grid, dim3(RT_BL), lds_bytes(p), s, p, (const float*)a.x,
                     (const float*)a.w_min, (const float*)a.w_max, a.alpha, a.beta, (float*)a.y, (float*)a.y_min,
                     (float*)a.y_max, a.idx_min, a.idx_max, nch, inv);
  return hipGetLastError();
}

template <int MODE>
hipError_t launch_m(const Params& p, const FwdArgs& a, hipStream_t s) {
  switch (p.sw) {
    case 1: return launch_s<MODE, 1>(p, a, s);
    case 2: return launch_s<MODE, 2>(p, a, s);
    case 4: return launch_s<MODE, 4>(p, a, s);
    default: return launch_s<MODE, 8>(p, a, s);
  }
}

}  // namespace

// One-row input, window of at least 8 taps without dilation, stride 1, 2, 4 or 8, full-window modes, fp32,
// and few enough input channels that the input span and the kernels of a workgroup fit its LDS.
bool forward_row_supported(const Params& p, int dtype) {
  if (dtype != TCONV_F32 || p.mode > TCONV_PARALLEL || p.pad_zero) return false;
  if (p.H != 1 || p.KH != 1 || p.ph != 0 || p.dw != 1 || p.KW < RT_CH) return false;
  if (p.sw != 1 && p.sw != 2 && p.sw != 4 && p.sw != 8) return false;
  if ((chunks_of(p) * RT_CH - 1) / p.sw > RT_M - RT_BL - 1) return false;  // the last lane's window ends inside its LDS row
  if (lds_bytes(p) > RT_LDS_MAX) return false;
  return p.N <= 65535 && (p.C_out + RT_TN - 1) / RT_TN <= 65535;
}

hipError_t launch_forward_row(const Params& p, const FwdArgs& a, hipStream_t s) {
  switch (p.mode) {
    case TCONV_MAX: return launch_m<TCONV_MAX>(p, a, s);
    case TCONV_MIN: return launch_m<TCONV_MIN>(p, a, s);
    case TCONV_COMPOUND: return launch_m<TCONV_COMPOUND>(p, a, s);
    default: return launch_m<TCONV_PARALLEL>(p, a, s);
  }
}

}  // namespace tconv
