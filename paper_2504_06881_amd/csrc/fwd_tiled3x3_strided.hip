// Tiled forward kernel for 3x3, STRIDE-2 tropical convolutions on gfx950 (compiler-scheduled variant).
//
// Operator: paper Sec. 3.1 layers (iv) / (v) (one min / max over all C_in*9 taps of x + w) and the
// Sec. 3.3 compound / parallel combinations.  Same lane geometry as the stride-1 kernel (a lane owns
// 8 consecutive output pixels x 4 output channels, kernel values wave-uniform in SGPRs, x rows in
// VGPRs with padding turned into NaN), but a stride-2 lane touches 17 input columns per row, which
// leaves no room for the stride-1 kernel's two-channel register blocks.  Here the inner loop walks
// pairs of consecutive taps ("steps"): 2 adds, then per branch one v_max3/v_min3, one compare and
// one select recording the STEP; the exact tap (first or second of the step) is recovered after
// the K loop by re-evaluating the step's first tap.  Steps partition k in ascending order and
// updates are strict, so the recorded step holds the lowest winning k.
#include <stdlib.h>

#include "tile_common.h"

namespace tconv {
namespace {

using namespace tile;

template <int MODE, int S, int D, int TN, typename T>
struct Tile {
  static constexpr bool DO_MIN = (MODE != TCONV_MAX);
  static constexpr bool DO_MAX = (MODE != TCONV_MIN);
  static constexpr bool TWO_W = (MODE == TCONV_PARALLEL);
  static constexpr int XR = 7 * S + 2 * D + 1;  // input columns a lane touches per row
  static constexpr int NC = 7 * S + 1;          // core columns [D, D+NC): always inside the row

  float bmax[TN][PX], bmin[TN][PX];
  int imax[TN][PX], imin[TN][PX];

  __device__ __forceinline__ void init() {
#pragma unroll
    for (int c = 0; c < TN; ++c)
#pragma unroll
      for (int q = 0; q < PX; ++q) {
        bmax[c][q] = -INFINITY; bmin[c][q] = INFINITY;
        imax[c][q] = 0; imin[c][q] = 0;
      }
  }

  // One row of one channel: core run + clamped halo singles, then NaN out what is padding.
  // ro is the lane's byte offset of the first core column (iw0 + D) of the (clamped) row, soff the
  // wave-uniform byte offset of the channel; hoff[h] are the clamped byte offsets of the 2D halo
  // columns relative to ro (possibly negative; the 32-bit sum ro + hoff[h] never is);
  // mrow / mhalo are all-ones where the row / halo column is padding.
  __device__ __forceinline__ void load_row(float (&xr)[XR], rsrc_t r, unsigned ro, unsigned soff,
                                           const int (&hoff)[2 * D], unsigned mrow,
                                           const unsigned (&mhalo)[2 * D]) {
    load_run<NC, T>(&xr[D], r, ro, soff);
#pragma unroll
    for (int h = 0; h < D; ++h) {
      xr[h] = load_one<T>(r, ro + (unsigned)hoff[h], soff);
      xr[D + NC + h] = load_one<T>(r, ro + (unsigned)hoff[D + h], soff);
    }
#pragma unroll
    for (int o = 0; o < XR; ++o) {
      unsigned m = mrow;
      if (o < D) m |= mhalo[o];
      if (o >= D + NC) m |= mhalo[o - NC];
      xr[o] = nan_or(xr[o], m);
    }
  }

  // One step = two consecutive taps (a, b) for all pixels and channels of the lane.
  __device__ __forceinline__ void step(const float (&xa)[PX], const float (&xb)[PX],
                                       const float (&wa_min)[TN], const float (&wb_min)[TN],
                                       const float (&wa_max)[TN], const float (&wb_max)[TN], int t) {
#pragma unroll
    for (int c = 0; c < TN; ++c) {
      // one scheduling region per output channel: bounds the temporaries the scheduler keeps live
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = 0; q < PX; ++q) {
        if (TWO_W) {
          const float sa1 = xa[q] + wa_min[c], sb1 = xb[q] + wb_min[c];
          const float sa2 = xa[q] + wa_max[c], sb2 = xb[q] + wb_max[c];
          const float nmn = fminf(fminf(bmin[c][q], sa1), sb1);
          imin[c][q] = (nmn < bmin[c][q]) ? t : imin[c][q];
          bmin[c][q] = nmn;
          const float nmx = fmaxf(fmaxf(bmax[c][q], sa2), sb2);
          imax[c][q] = (nmx > bmax[c][q]) ? t : imax[c][q];
          bmax[c][q] = nmx;
        } else {
          const float sa = xa[q] + (DO_MAX ? wa_max[c] : wa_min[c]);
          const float sb = xb[q] + (DO_MAX ? wb_max[c] : wb_min[c]);
          if (DO_MAX) {
            const float nmx = fmaxf(fmaxf(bmax[c][q], sa), sb);
            imax[c][q] = (nmx > bmax[c][q]) ? t : imax[c][q];
            bmax[c][q] = nmx;
          }
          if (DO_MIN) {
            const float nmn = fminf(fminf(bmin[c][q], sa), sb);
            imin[c][q] = (nmn < bmin[c][q]) ? t : imin[c][q];
            bmin[c][q] = nmn;
          }
        }
      }
    }
  }

  // Last tap of an odd K: a step with a single candidate.
  __device__ __forceinline__ void step1(const float (&xa)[PX], const float (&wa_min)[TN],
                                        const float (&wa_max)[TN], int t) {
#pragma unroll
    for (int c = 0; c < TN; ++c)
#pragma unroll
      for (int q = 0; q < PX; ++q) {
        if (DO_MIN) {
          const float s = xa[q] + ((TWO_W || !DO_MAX) ? wa_min[c] : wa_max[c]);  // compound: shared kernel
          const float nmn = fminf(bmin[c][q], s);
          imin[c][q] = (nmn < bmin[c][q]) ? t : imin[c][q];
          bmin[c][q] = nmn;
        }
        if (DO_MAX) {
          const float s = xa[q] + wa_max[c];
          const float nmx = fmaxf(bmax[c][q], s);
          imax[c][q] = (nmx > bmax[c][q]) ? t : imax[c][q];
          bmax[c][q] = nmx;
        }
      }
  }
};

// The 8 x values of tap (i, j) within a channel's three row registers.
template <int S, int D, int XR>
__device__ __forceinline__ void tap_x(float (&out)[PX], const float (&row)[XR], int j) {
#pragma unroll
  for (int q = 0; q < PX; ++q) out[q] = row[q * S + j * D];
}

template <typename T>
__device__ __forceinline__ float wld(const T* w, int k);
template <>
__device__ __forceinline__ float wld<float>(const float* w, int k) { return w[k]; }
template <>
__device__ __forceinline__ float wld<bf16_t>(const bf16_t* w, int k) {
  return __uint_as_float(((unsigned)w[k]) << 16);
}

template <int MODE, int S, int D, int TN, typename T>
__global__ __launch_bounds__(WAVES * 64, 2) void fwd_tiled3x3_kernel(
    Params p, const T* __restrict__ x, const T* __restrict__ w_min, const T* __restrict__ w_max,
    const float* __restrict__ alpha, const float* __restrict__ beta, T* __restrict__ y,
    T* __restrict__ y_min, T* __restrict__ y_max, int32_t* __restrict__ idx_min,
    int32_t* __restrict__ idx_max, int segs, int n_units, int n_groups, int dbg) {
  using TL = Tile<MODE, S, D, TN, T>;
  constexpr bool DO_MIN = TL::DO_MIN, DO_MAX = TL::DO_MAX, TWO_W = TL::TWO_W;
  constexpr int XR = TL::XR, NC = TL::NC;

  // ---- which c_out group (wave-uniform) and which pixel segment (per lane)
  const int gblocks = (n_groups + WAVES - 1) / WAVES;
  const int ublock = blockIdx.x / gblocks;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int group = (blockIdx.x - ublock * gblocks) * WAVES + wave;
  if (group >= n_groups) return;  // whole wave leaves; the kernel has no barrier
  const int co0 = group * TN;
  const int lane = threadIdx.x & 63;
  const int unit_raw = ublock * 64 + lane;
  const bool unit_ok = unit_raw < n_units;
  const int unit = unit_ok ? unit_raw : n_units - 1;  // surplus lanes recompute the last unit, store nothing
  const int seg = unit % segs;
  const int oh = (unit / segs) % p.Ho;
  const int n = unit / (segs * p.Ho);
  // the last segment of a row is shifted left so that every lane owns 8 real pixels;
  // pixels it shares with its neighbour are computed twice and stored once
  const int ow_nom = seg * PX;
  const int ow0 = min(ow_nom, p.Wo - PX);
  const int first_q = ow_nom - ow0;  // pixels q < first_q belong to the previous segment

  // ---- channel-independent addressing and padding masks
  const int iw0 = ow0 * S - p.pw;
  const size_t HW = (size_t)p.H * p.W;
  const rsrc_t xres = make_rsrc(x, (unsigned)((size_t)p.N * p.C_in * HW * sizeof(T)));
  // per-lane byte offsets (32-bit: the tensor is below 4 GiB) added to a wave-uniform channel base
  unsigned roff[3];
  unsigned mrow[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int ih = oh * S - p.ph + i * D;
    const bool v = (ih >= 0 && ih < p.H);
    mrow[i] = v ? 0u : 0xffffffffu;
    const int ihc = min(max(ih, 0), p.H - 1);
    // offset of the lane's first CORE column (iw0 + D >= 0 because pad_w <= D): never negative
    roff[i] = (unsigned)(((size_t)n * p.C_in * HW + (size_t)ihc * p.W + (size_t)(iw0 + D)) * sizeof(T));
  }
  int hoff[2 * D];
  unsigned mhalo[2 * D];
#pragma unroll
  for (int h = 0; h < 2 * D; ++h) {
    const int o = (h < D) ? h : h + NC;
    const int iw = iw0 + o;
    const bool v = (iw >= 0 && iw < p.W);
    mhalo[h] = v ? 0u : 0xffffffffu;
    hoff[h] = (min(max(iw, 0), p.W - 1) - (iw0 + D)) * (int)sizeof(T);  // relative to the core start
  }

  // ---- kernel rows of this wave's TN output channels (wave-uniform pointers)
  const T* wr_min[TN];
  const T* wr_max[TN];
#pragma unroll
  for (int c = 0; c < TN; ++c) {
    const int co = min(co0 + c, p.C_out - 1);
    wr_min[c] = DO_MIN ? w_min + (size_t)co * p.K : nullptr;
    wr_max[c] = DO_MAX ? w_max + (size_t)co * p.K : nullptr;
  }

  TL acc;
  acc.init();

  // ---- main loop over channel pairs: 18 taps = 9 steps.  Software pipeline, in program order:
  //  * the six input rows of a pair (2 channels x 3 kernel rows; tap t lives in row slot t/3)
  //    sit in six register slots; a slot is re-loaded for the NEXT pair right after the step
  //    that last reads it, and its padding mask is applied just before its first use;
  //  * the kernel values of a step (2 taps x TN channels, SGPRs) are fetched one step ahead.
  const int npairs = (dbg & 2) ? 0 : (p.C_in >> 1);
  constexpr int WMN = (TWO_W || !DO_MAX) ? TN : 1;
  constexpr int WMX = DO_MAX ? TN : 1;
  float xs[6][XR];
  auto issue_row = [&](int slot, int cp) {
    const unsigned soff = (unsigned)((size_t)(2 * cp + slot / 3) * HW * sizeof(T));  // wave-uniform
    const unsigned ro = roff[slot % 3];
    load_run<NC, T>(&xs[slot][D], xres, ro, soff);
#pragma unroll
    for (int h = 0; h < D; ++h) {
      xs[slot][h] = load_one<T>(xres, ro + (unsigned)hoff[h], soff);
      xs[slot][D + NC + h] = load_one<T>(xres, ro + (unsigned)hoff[D + h], soff);
    }
  };
  auto finalize_row = [&](int slot) {
    const unsigned mr = mrow[slot % 3];
#pragma unroll
    for (int o = 0; o < XR; ++o) {
      unsigned m = mr;
      if (o < D) m |= mhalo[o];
      if (o >= D + NC) m |= mhalo[o - NC];
      xs[slot][o] = nan_or(xs[slot][o], m);
    }
  };
  auto load_w = [&](float (&wmn)[WMN][2], float (&wmx)[WMX][2], int k) {
#pragma unroll
    for (int c = 0; c < TN; ++c) {
      if (DO_MAX) { wmx[c][0] = wld<T>(wr_max[c], k); wmx[c][1] = wld<T>(wr_max[c], k + 1); }
      if (TWO_W || !DO_MAX) { wmn[c][0] = wld<T>(wr_min[c], k); wmn[c][1] = wld<T>(wr_min[c], k + 1); }
    }
  };
  float wc_mn[WMN][2], wc_mx[WMX][2];
  if (npairs > 0) {
#pragma unroll
    for (int r = 0; r < 6; ++r) issue_row(r, 0);
    load_w(wc_mn, wc_mx, 0);
  }
  for (int cp = 0; cp < npairs; ++cp) {
    const int cpn = min(cp + 1, npairs - 1);  // past the end: re-load the last pair (unused, in bounds)
    const int t0 = cp * 9;
#pragma unroll
    for (int s = 0; s < 9; ++s) {
      const int ta = 2 * s, tb = 2 * s + 1;
      float wn_mn[WMN][2], wn_mx[WMX][2];
      load_w(wn_mn, wn_mx, (s < 8) ? cp * 18 + 2 * s + 2 : cpn * 18);
#pragma unroll
      for (int r = 0; r < 6; ++r)
        if ((3 * r) / 2 == s) finalize_row(r);
      float xa[PX], xb[PX];
      tap_x<S, D, XR>(xa, xs[ta / 3], ta % 3);
      tap_x<S, D, XR>(xb, xs[tb / 3], tb % 3);
      float wa1[TN], wb1[TN], wa2[TN], wb2[TN];
#pragma unroll
      for (int c = 0; c < TN; ++c) {
        wa2[c] = DO_MAX ? wc_mx[DO_MAX ? c : 0][0] : 0.f;
        wb2[c] = DO_MAX ? wc_mx[DO_MAX ? c : 0][1] : 0.f;
        wa1[c] = (TWO_W || !DO_MAX) ? wc_mn[(TWO_W || !DO_MAX) ? c : 0][0] : 0.f;
        wb1[c] = (TWO_W || !DO_MAX) ? wc_mn[(TWO_W || !DO_MAX) ? c : 0][1] : 0.f;
      }
      acc.step(xa, xb, wa1, wb1, wa2, wb2, t0 + s);
#pragma unroll
      for (int r = 0; r < 6; ++r)
        if ((3 * r + 2) / 2 == s) issue_row(r, cpn);
      __builtin_amdgcn_sched_barrier(0);  // keep the hand-made pipeline: nothing moves across a step
#pragma unroll
      for (int c = 0; c < TN; ++c) {
        if (DO_MAX) { wc_mx[c][0] = wn_mx[c][0]; wc_mx[c][1] = wn_mx[c][1]; }
        if (TWO_W || !DO_MAX) { wc_mn[c][0] = wn_mn[c][0]; wc_mn[c][1] = wn_mn[c][1]; }
      }
    }
  }
  if (p.C_in & 1) {  // odd C_in: the last channel alone, 4 full steps and a single-candidate step
    const int cl = p.C_in - 1;
    float wmn[TWO_W || !DO_MAX ? TN : 1][9], wmx[DO_MAX ? TN : 1][9];
#pragma unroll
    for (int c = 0; c < TN; ++c)
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        if (DO_MAX) wmx[c][t] = wld<T>(wr_max[c], cl * 9 + t);
        if (TWO_W || !DO_MAX) wmn[c][t] = wld<T>(wr_min[c], cl * 9 + t);
      }
    float xs1[3][XR];
#pragma unroll
    for (int i = 0; i < 3; ++i)
      acc.load_row(xs1[i], xres, roff[i], (unsigned)((size_t)cl * HW * sizeof(T)), hoff, mrow[i], mhalo);
    const int t0 = npairs * 9;
#pragma unroll
    for (int s = 0; s < 5; ++s) {
      const int ta = 2 * s, tb = 2 * s + 1;
      float xa[PX], xb[PX];
      float wa1[TN], wb1[TN], wa2[TN], wb2[TN];
      tap_x<S, D, XR>(xa, xs1[ta / 3], ta % 3);
#pragma unroll
      for (int c = 0; c < TN; ++c) {
        wa2[c] = DO_MAX ? wmx[c][ta] : 0.f;
        wa1[c] = (TWO_W || !DO_MAX) ? wmn[TWO_W || !DO_MAX ? c : 0][ta] : 0.f;
      }
      if (s < 4) {
        tap_x<S, D, XR>(xb, xs1[tb / 3], tb % 3);
#pragma unroll
        for (int c = 0; c < TN; ++c) {
          wb2[c] = DO_MAX ? wmx[c][tb] : 0.f;
          wb1[c] = (TWO_W || !DO_MAX) ? wmn[TWO_W || !DO_MAX ? c : 0][tb] : 0.f;
        }
        acc.step(xa, xb, wa1, wb1, wa2, wb2, t0 + s);
      } else {
        acc.step1(xa, wa1, wa2, t0 + s);
      }
    }
  }

  // ---- epilogue: exact tap index of every extremum, combine, store.  Branch-free per item;
  // each lane writes its 8 consecutive outputs of a (channel, tensor) with two 16-byte stores.
  if (!unit_ok) return;
  const size_t xn_off = (size_t)n * p.C_in * HW;
  const int ih_base = oh * S - p.ph;
  auto refine = [&](int t, float best, const T* wrow, int q) -> int {
    const int ka = 2 * t, kb = ka + 1;
    const int c = ka / 9, r = ka - 9 * c, i = r / 3, j = r - 3 * i;
    const int ih = ih_base + i * D, iw = (ow0 + q) * S - p.pw + j * D;
    const bool v = (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W);
    const int ihc = min(max(ih, 0), p.H - 1), iwc = min(max(iw, 0), p.W - 1);
    const float xv = load_one<T>(xres, (unsigned)((xn_off + (size_t)c * HW + (size_t)ihc * p.W + iwc) * sizeof(T)), 0u);
    const float sa = __fadd_rn(xv, wld<T>(wrow, ka));
    const bool first = (v && sa == best) || (kb >= p.K) || (dbg & 1);
    return first ? ka : kb;
  };
  const size_t plane = (size_t)p.Ho * p.Wo;
#pragma unroll
  for (int c = 0; c < TN; ++c) {
    const int co = co0 + c;
    if (co >= p.C_out) break;  // wave-uniform
    const size_t ob = ((size_t)n * p.C_out + co) * plane + (size_t)oh * p.Wo + ow0;
    float ca = 1.f, cb = 1.f;
    if (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL) {
      if (alpha) ca = alpha[co];
      if (beta) cb = beta[co];
    }
    int ridx[PX];
    float out[PX];
    if (DO_MIN) {
#pragma unroll
      for (int q = 0; q < PX; ++q) ridx[q] = refine(acc.imin[c][q], acc.bmin[c][q], wr_min[c], q);
      store_row(idx_min + ob, ridx, first_q);
      if (y_min) store_row(y_min + ob, acc.bmin[c], first_q);
    }
    if (DO_MAX) {
#pragma unroll
      for (int q = 0; q < PX; ++q) ridx[q] = refine(acc.imax[c][q], acc.bmax[c][q], wr_max[c], q);
      store_row(idx_max + ob, ridx, first_q);
      if (y_max) store_row(y_max + ob, acc.bmax[c], first_q);
    }
#pragma unroll
    for (int q = 0; q < PX; ++q) {
      if (MODE == TCONV_MAX) out[q] = acc.bmax[c][q];
      else if (MODE == TCONV_MIN) out[q] = acc.bmin[c][q];
      else out[q] = combine(ca, acc.bmin[c][q], cb, acc.bmax[c][q]);
    }
    store_row(y + ob, out, first_q);
  }
}

template <int MODE, int S, int D, int TN, typename T>
hipError_t launch_one(const Params& p, const FwdArgs& a, hipStream_t s) {
  const int segs = (p.Wo + PX - 1) / PX;
  const long long n_units = (long long)p.N * p.Ho * segs;
  const int n_groups = (p.C_out + TN - 1) / TN;
  const long long ublocks = (n_units + 63) / 64;
  const long long gblocks = (n_groups + WAVES - 1) / WAVES;
  const long long blocks = ublocks * gblocks;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  const char* e = getenv("TCONV_DEBUG_FLAGS");
  const int dbg = e ? atoi(e) : 0;
  hipLaunchKernelGGL((fwd_tiled3x3_kernel<MODE, S, D, TN, T>), dim3((unsigned)blocks),
                     dim3(WAVES * 64), 0, s, p, (const T*)a.x, (const T*)a.w_min,
                     (const T*)a.w_max, a.alpha, a.beta, (T*)a.y, (T*)a.y_min, (T*)a.y_max,
                     a.idx_min, a.idx_max, segs, (int)n_units, n_groups, dbg);
  return hipGetLastError();
}

template <int MODE, typename T>
hipError_t launch_geo(const Params& p, const FwdArgs& a, hipStream_t s) {
  return launch_one<MODE, 2, 1, 4, T>(p, a, s);
}

template <typename T>
hipError_t launch_mode(const Params& p, const FwdArgs& a, hipStream_t s) {
  switch (p.mode) {
    case TCONV_MAX: return launch_geo<TCONV_MAX, T>(p, a, s);
    case TCONV_MIN: return launch_geo<TCONV_MIN, T>(p, a, s);
    case TCONV_COMPOUND: return launch_geo<TCONV_COMPOUND, T>(p, a, s);
    default: return launch_geo<TCONV_PARALLEL, T>(p, a, s);
  }
}

}  // namespace

// 3x3 kernels with stride 2 and dilation 1 on both axes, horizontal padding at most 1 (so the core
// columns of every lane lie inside the row), and at least one full 8-pixel segment per output row.
bool forward_tiled_strided_supported(const Params& p, int dtype) {
  if (p.KH != 3 || p.KW != 3) return false;
  if (p.sh != 2 || p.sw != 2 || p.dh != 1 || p.dw != 1) return false;
  if (p.pw > p.dw) return false;
  if (p.Wo < PX) return false;
  // lanes address x with 32-bit byte offsets
  const size_t esz = (dtype == TCONV_BF16) ? 2 : 4;
  if ((size_t)p.N * p.C_in * p.H * p.W * esz >= 0xfffff000ull) return false;
  return true;
}

hipError_t launch_forward_tiled_strided(const Params& p, int dtype, const FwdArgs& a, hipStream_t s) {
  return dtype == TCONV_BF16 ? launch_mode<bf16_t>(p, a, s) : launch_mode<float>(p, a, s);
}

}  // namespace tconv
