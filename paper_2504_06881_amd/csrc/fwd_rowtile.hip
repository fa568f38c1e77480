// Tiled forward kernel for tropical convolutions with windows other than 3x3 on gfx950 (fp32): 5x5 and 7x7 windows
// (the LeNet layers of the paper's Table 1, an ImageNet-style 7x7 stride-2 stem, Sec. 5), 1 x 1, and any KH x KW with
// KW <= 7, stride 1 or 2 along the row, dilation 1 along the row.
//
// Operator: paper Sec. 3.1 layers (iv) / (v) and the Sec. 3.3 compound / parallel combinations, as in the 3x3 kernel:
// one rounded fp32 add per candidate, max / min over all C_in*KH*KW taps, lowest flattened tap on ties.
//
// Scheme (compiler-scheduled, no hand-written blocks): a lane owns PX consecutive output pixels of a row (8 at stride
// 1, 4 at stride 2) and 4 output channels; the running extrema stay in registers for the whole K loop.  The K loop
// walks kernel ROWS: step st = c*KH + i covers the KW taps k = st*KW + j.  Per step a lane loads the one input row
// segment its pixels read ((PX-1)*S + KW values, next step's segment one step ahead into a second register set),
// padding becomes NaN (which max and min drop), the KW kernel values of each of the lane's output channels are
// wave-uniform scalars, and per (pixel, channel, branch) the step costs KW adds (shared by both branches in compound
// mode), ceil(KW/2) three-operand max / min, one compare and one select that record the STEP at which the extremum
// improved.  The epilogue re-evaluates the KW taps of the recorded step and takes the first that equals the extremum.
#include <stdlib.h>

#include "tile_common.h"

namespace tconv {
namespace {

using namespace tile;

constexpr int TN = 4;  // output channels per lane

template <int MODE, int KW, int S>
__global__ __launch_bounds__(WAVES * 64, 2) void fwd_rowtile_kernel(
    Params p, const float* __restrict__ x, const float* __restrict__ w_min, const float* __restrict__ w_max,
    const float* __restrict__ alpha, const float* __restrict__ beta, float* __restrict__ y,
    float* __restrict__ y_min, float* __restrict__ y_max, int32_t* __restrict__ idx_min,
    int32_t* __restrict__ idx_max, int segs, int n_units, int n_groups, int n_blocks, int core_lo, int core_hi,
    unsigned inv_kh) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr int PX = (S == 1) ? 8 : 4;
  constexpr int XR = (PX - 1) * S + KW;  // input columns a lane touches per row

  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: every XCD gets a contiguous run of
  // workgroup numbers, so that the channel blocks of a pixel block (consecutive numbers) read their input lines
  // through one L2.  The grid is padded to a multiple of 8; the kernel has no barrier.
  const int per_xcd = (n_blocks + 7) >> 3;
  const int bid = (int)(blockIdx.x & 7u) * per_xcd + (int)(blockIdx.x >> 3);
  if (bid >= n_blocks || (int)(blockIdx.x >> 3) >= per_xcd) return;
  const int gblocks = (n_groups + WAVES - 1) / WAVES;
  const int ublock = bid / gblocks;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int group = (bid - ublock * gblocks) * WAVES + wave;
  if (group >= n_groups) return;  // whole wave leaves
  const int co0 = group * TN;
  const int lane = threadIdx.x & 63;
  const int unit_raw = ublock * 64 + lane;
  const bool unit_ok = unit_raw < n_units;
  const int unit = unit_ok ? unit_raw : n_units - 1;  // surplus lanes recompute the last unit, store nothing
  const int seg = unit % segs;
  const int oh = (unit / segs) % p.Ho;
  const int n = unit / (segs * p.Ho);
  const int ow_nom = seg * PX;
  const int ow0 = min(ow_nom, p.Wo - PX);  // the last segment of a row is shifted left
  const int first_q = unit_ok ? ow_nom - ow0 : PX;

  const int iw0 = ow0 * S - p.pw;  // input column of register column 0
  const int ih0 = oh * p.sh - p.ph;
  const size_t HW = (size_t)p.H * p.W;
  const unsigned HWb = (unsigned)(HW * sizeof(float));
  const rsrc_t xres = make_rsrc(x, (unsigned)((size_t)p.N * p.C_in * HW * sizeof(float)));
  const unsigned nbase = (unsigned)((size_t)n * p.C_in * HW * sizeof(float));
  // per register column: clamped byte offset inside a row, and all-ones where the column is padding
  unsigned coff[XR], mcol[XR];
#pragma unroll
  for (int e = 0; e < XR; ++e) {
    const int iw = iw0 + e;
    mcol[e] = (iw >= 0 && iw < p.W) ? 0u : 0xffffffffu;
    coff[e] = (unsigned)min(max(iw, 0), p.W - 1) * 4u;
  }
  const int nst = p.C_in * p.KH;  // steps: (channel, kernel row) pairs in k order

  // Register columns [core_lo, core_hi) lie inside the row for every lane (core_lo = the left padding; the host
  // derives both from the geometry): they are read in runs of four with 16-byte loads, the columns left and right
  // of them one by one from clamped positions.  The run boundaries depend on core_lo, a wave-uniform run-time value,
  // while register numbers must be constants: one statically laid out variant per left padding 0..3, chosen by a
  // uniform branch (wider paddings: every column on its own).
  const unsigned cb0 = (unsigned)(iw0 * 4);  // byte offset of register column 0 (may wrap; only used inside the core)
  auto load_cols = [&](float (&xs)[XR], unsigned roff, unsigned soff, auto loc) {
    constexpr int LO = decltype(loc)::value;
#pragma unroll
    for (int e = 0; e < (LO < XR ? LO : XR); ++e) xs[e] = load_one<float>(xres, roff + coff[e], soff);
    static_steps<LO, XR, 4>([&](auto ec) {
      constexpr int e = decltype(ec)::value;
      if (e + 4 <= XR && e + 4 <= core_hi) {  // wave-uniform
        if constexpr (e + 4 <= XR) load_run<4, float>(&xs[e], xres, roff + cb0 + 4u * e, soff);
      } else {
#pragma unroll
        for (int t = e; t < (e + 4 < XR ? e + 4 : XR); ++t) xs[t] = load_one<float>(xres, roff + coff[t], soff);
      }
    });
  };
  // row segment of step (c, i); returns the row's padding mask
  auto load_row = [&](float (&xs)[XR], int c, int i) -> unsigned {
    const int ih = ih0 + i * p.dh;
    const unsigned roff = nbase + (unsigned)(min(max(ih, 0), p.H - 1) * p.W) * 4u;
    const unsigned soff = (unsigned)min(c, p.C_in - 1) * HWb;
    switch (core_lo) {  // wave-uniform
      case 0: load_cols(xs, roff, soff, std::integral_constant<int, 0>{}); break;
      case 1: load_cols(xs, roff, soff, std::integral_constant<int, 1>{}); break;
      case 2: load_cols(xs, roff, soff, std::integral_constant<int, 2>{}); break;
      case 3: load_cols(xs, roff, soff, std::integral_constant<int, 3>{}); break;
      default: load_cols(xs, roff, soff, std::integral_constant<int, XR>{}); break;
    }
    return (ih >= 0 && ih < p.H) ? 0u : 0xffffffffu;
  };
  auto mask_row = [&](float (&xs)[XR], unsigned mrow) {
#pragma unroll
    for (int e = 0; e < XR; ++e) xs[e] = nan_or(xs[e], mrow | mcol[e]);
  };

  float bmax[TN][PX], bmin[TN][PX];
  int imax[TN][PX], imin[TN][PX];
#pragma unroll
  for (int t = 0; t < TN; ++t)
#pragma unroll
    for (int q = 0; q < PX; ++q) {
      bmax[t][q] = -INFINITY; bmin[t][q] = INFINITY;
      imax[t][q] = 0; imin[t][q] = 0;
    }

  // one step: KW taps for every pixel and output channel of the lane
  auto step = [&](const float (&xs)[XR], int st) {
#pragma unroll
    for (int t = 0; t < TN; ++t) {
      const int co = min(co0 + t, p.C_out - 1);
      const float* wa = DO_MIN ? w_min + (size_t)co * p.K + (size_t)st * KW : nullptr;
      const float* wb = DO_MAX ? w_max + (size_t)co * p.K + (size_t)st * KW : nullptr;
      float ka[KW], kb[KW];
#pragma unroll
      for (int j = 0; j < KW; ++j) {
        if (DO_MIN) ka[j] = wa[j];
        if (DO_MAX) kb[j] = wb[j];
      }
#pragma unroll
      for (int q = 0; q < PX; ++q) {
        float sa[KW], sb[KW];
#pragma unroll
        for (int j = 0; j < KW; ++j) {
          const float xv = xs[q * S + j];
          if (DO_MIN) sa[j] = __fadd_rn(xv, ka[j]);
          if (DO_MAX) sb[j] = (MODE == TCONV_COMPOUND) ? sa[j] : __fadd_rn(xv, kb[j]);
        }
        if (DO_MIN) {
          float m = bmin[t][q];
#pragma unroll
          for (int j = 0; j + 1 < KW; j += 2) m = fminf(fminf(m, sa[j]), sa[j + 1]);
          if (KW & 1) m = fminf(m, sa[KW - 1]);
          imin[t][q] = (m < bmin[t][q]) ? st : imin[t][q];
          bmin[t][q] = m;
        }
        if (DO_MAX) {
          float m = bmax[t][q];
#pragma unroll
          for (int j = 0; j + 1 < KW; j += 2) m = fmaxf(fmaxf(m, sb[j]), sb[j + 1]);
          if (KW & 1) m = fmaxf(m, sb[KW - 1]);
          imax[t][q] = (m > bmax[t][q]) ? st : imax[t][q];
          bmax[t][q] = m;
        }
      }
    }
  };

  {
    float xa[XR], xb[XR];
    int c = 0, i = 0;  // step st = c*KH + i
    unsigned ma = load_row(xa, 0, 0), mb = 0;
    for (int st = 0; st < nst; st += 2) {
      int c1 = c, i1 = i + 1;
      if (i1 == p.KH) { i1 = 0; ++c1; }
      mb = load_row(xb, c1, i1);  // past the last step: a clamped, unused reload
      mask_row(xa, ma);
      step(xa, st);
      if (st + 1 < nst) {  // wave-uniform
        c = c1; i = i1 + 1;
        if (i == p.KH) { i = 0; ++c; }
        ma = load_row(xa, c, i);
        mask_row(xb, mb);
        step(xb, st + 1);
      }
    }
  }

  // ---- epilogue: first tap of the recorded step that equals the extremum, combine, store
  const size_t plane = (size_t)p.Ho * p.Wo;
  const rsrc_t wres_min = make_rsrc(DO_MIN ? w_min : w_max, (unsigned)((size_t)p.C_out * p.K * sizeof(float)));
  const rsrc_t wres_max = make_rsrc(DO_MAX ? w_max : w_min, (unsigned)((size_t)p.C_out * p.K * sizeof(float)));
  // (the step unflattens with a multiply-high: inv_kh = floor(2^32 / KH) + 1 is exact for st * KH < 2^32; KH = 1: 0)
  auto refine = [&](rsrc_t wres, unsigned cobase, auto qc, int st, float best) -> int {
    constexpr int q = decltype(qc)::value;
    const int c = inv_kh ? (int)__umulhi((unsigned)st, inv_kh) : st;
    const int i = st - c * p.KH;
    const int ih = ih0 + i * p.dh;  // inside the image: the recorded step improved the extremum
    const unsigned roff = nbase + (unsigned)c * HWb + (unsigned)(min(max(ih, 0), p.H - 1) * p.W) * 4u;
    float xv[KW], wv[KW];
    load_run<KW, float>(wv, wres, cobase + (unsigned)(st * KW) * 4u, 0u);
    if (q * S >= core_lo && q * S + KW <= core_hi) {  // wave-uniform: the pixel's window is inside the row
      load_run<KW, float>(xv, xres, roff + cb0 + 4u * (q * S), 0u);
    } else {
#pragma unroll
      for (int j = 0; j < KW; ++j) xv[j] = nan_or(load_one<float>(xres, roff + coff[q * S + j], 0u), mcol[q * S + j]);
    }
    int r = 0;
#pragma unroll
    for (int j = KW - 1; j >= 0; --j) r = (__fadd_rn(xv[j], wv[j]) == best) ? j : r;
    return st * KW + r;
  };
#pragma unroll
  for (int t = 0; t < TN; ++t) {
    const int co = co0 + t;
    if (co >= p.C_out) break;  // wave-uniform
    const size_t ob = ((size_t)n * p.C_out + co) * plane + (size_t)oh * p.Wo + ow0;
    float ca = 1.f, cb = 1.f;
    if (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL) {
      if (alpha) ca = alpha[co];
      if (beta) cb = beta[co];
    }
    int ridx[PX];
    float out[PX];
    const unsigned cobase = (unsigned)((size_t)co * p.K * sizeof(float));
    if (DO_MIN) {
      static_steps<0, PX, 1>([&](auto qc) {
        constexpr int q = decltype(qc)::value;
        ridx[q] = refine(wres_min, cobase, qc, imin[t][q], bmin[t][q]);
      });
      store_row<PX>(idx_min + ob, ridx, first_q);
      if (y_min) store_row<PX>(y_min + ob, bmin[t], first_q);
    }
    if (DO_MAX) {
      static_steps<0, PX, 1>([&](auto qc) {
        constexpr int q = decltype(qc)::value;
        ridx[q] = refine(wres_max, cobase, qc, imax[t][q], bmax[t][q]);
      });
      store_row<PX>(idx_max + ob, ridx, first_q);
      if (y_max) store_row<PX>(y_max + ob, bmax[t], first_q);
    }
#pragma unroll
    for (int q = 0; q < PX; ++q) {
      if (!DO_MIN) out[q] = bmax[t][q];
      else if (!DO_MAX) out[q] = bmin[t][q];
      else out[q] = combine(ca, bmin[t][q], cb, bmax[t][q]);
    }
    store_row<PX>(y + ob, out, first_q);
  }
}

template <int MODE, int KW, int S>
hipError_t launch_k(const Params& p, const FwdArgs& a, hipStream_t s) {
  constexpr int PX = (S == 1) ? 8 : 4;
  const int segs = (p.Wo + PX - 1) / PX;
  const long long n_units = (long long)p.N * p.Ho * segs;
  const int n_groups = (p.C_out + TN - 1) / TN;
  const long long blocks = ((n_units + 63) / 64) * ((n_groups + WAVES - 1) / WAVES);
  const long long grid = ((blocks + 7) / 8) * 8;
  if (grid > 0x7ffffff0LL) return hipErrorInvalidValue;
  // register columns inside the row for every lane: a lane's column e is input column ow0 * S - pad_w + e with
  // 0 <= ow0 <= W_out - PX
  constexpr int XR = (PX - 1) * S + KW;
  const int core_lo = p.pw < XR ? p.pw : XR;
  long long hi = (long long)p.W + p.pw - (long long)(p.Wo - PX) * S;
  const int core_hi = (int)(hi < core_lo ? core_lo : (hi > XR ? XR : hi));
  const unsigned inv_kh = p.KH > 1 ? (unsigned)(0x100000000ULL / (unsigned long long)p.KH) + 1u : 0u;
  hipLaunchKernelGGL((fwd_rowtile_kernel<MODE, KW, S>), dim3((unsigned)grid), dim3(WAVES * 64), 0, s, p,
                     (const float*)a.x, (const float*)a.w_min, (const float*)a.w_max, a.alpha, a.beta, (float*)a.y,
                     (float*)a.y_min, (float*)a.y_max, a.idx_min, a.idx_max, segs, (int)n_units, n_groups, (int)blocks,
                     core_lo, core_hi, inv_kh);
  return hipGetLastError();
}

template <int MODE, int KW>
hipError_t launch_s(const Params& p, const FwdArgs& a, hipStream_t s) {
  return p.sw == 1 ? launch_k<MODE, KW, 1>(p, a, s) : launch_k<MODE, KW, 2>(p, a, s);
}

template <int MODE>
hipError_t launch_kw(const Params& p, const FwdArgs& a, hipStream_t s) {
  switch (p.KW) {
    case 1: return launch_s<MODE, 1>(p, a, s);
    case 2: return launch_s<MODE, 2>(p, a, s);
    case 3: return launch_s<MODE, 3>(p, a, s);
    case 4: return launch_s<MODE, 4>(p, a, s);
    case 5: return launch_s<MODE, 5>(p, a, s);
    case 6: return launch_s<MODE, 6>(p, a, s);
    default: return launch_s<MODE, 7>(p, a, s);
  }
}

}  // namespace

// fp32 storage, the four full-window modes, identity padding, KW <= 7, stride 1 or 2 and dilation 1 along the row
// (any stride and dilation along the column), at least one full pixel segment per output row, tensors addressable
// with 32-bit byte offsets.  One-row inputs with long windows have a kernel of their own.
bool forward_rowtile_supported(const Params& p, int dtype) {
  if (dtype != TCONV_F32 || p.mode > TCONV_PARALLEL || p.pad_zero) return false;
  if (p.KW < 1 || p.KW > 7 || p.dw != 1 || (p.sw != 1 && p.sw != 2)) return false;
  if (p.Wo < (p.sw == 1 ? 8 : 4)) return false;
  if ((size_t)p.N * p.C_in * p.H * p.W * 4 >= 0xfffff000ull) return false;
  if ((size_t)p.C_out * p.K * 4 >= 0xfffff000ull) return false;
  if ((long long)p.C_in * p.KH >= (1LL << 28)) return false;
  if ((long long)p.C_in * p.KH * p.KH >= (1LL << 32)) return false;  // a step unflattens with a multiply-high
  return true;
}

hipError_t launch_forward_rowtile(const Params& p, const FwdArgs& a, hipStream_t s) {
  switch (p.mode) {
    case TCONV_MAX: return launch_kw<TCONV_MAX>(p, a, s);
    case TCONV_MIN: return launch_kw<TCONV_MIN>(p, a, s);
    case TCONV_COMPOUND: return launch_kw<TCONV_COMPOUND>(p, a, s);
    default: return launch_kw<TCONV_PARALLEL>(p, a, s);
  }
}

}  // namespace tconv
