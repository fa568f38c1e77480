// Three-dimensional tropical convolution layers (paper Sec. 3.2, three-dimensional base operators MinPlus3d /
// MaxPlus3d and layers (iii) - (vi); Sec. 3.3 compound / parallel) on volumes x [N, C_in, D, H, W] with kernels
// [C_out, C_in, KD, KH, KW].  The saved winner is the flattened tap k = ((c*KD + a)*KH + i)*KW + j.
//
// These are plain kernels for any window, stride, padding and dilation: one thread per output in the forward
// pass (consecutive threads own consecutive ow, so reads of x and all writes are coalesced), a scatter with
// float atomics for the input gradient.  The kernel gradient needs no geometry (it is a histogram of the
// winners per output channel) and runs on the two-dimensional histogram kernel.  fp32 only.
#include <stdlib.h>
#include <string.h>

#include "tile_common.h"

namespace tconv {
namespace {

using namespace tile;

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


// ---------------------------------------------------------------------------------- 3 x 3 x 3, stride 1, dilation 1

// Register-resident kernel for the common volumetric window.  A lane owns 4 consecutive outputs of one row and
// TN3 = 4 output channels (the 4 waves of a workgroup take different channel groups of the same outputs, so
// their input lines meet in the L1); per input channel it loads the 9 input rows under its outputs once
// (3 depths x 3 heights x 6 columns, padding as NaN, which v_max3 / v_min3 ignore) and reuses them for 27 taps x
// 4 outputs x 4 channels.  Kernel values are wave-uniform (scalar loads).  The loop tracks the winning ROW of
// three taps (channel, depth tap, height tap: one v_min3 / v_max3, one compare and one select per row, output
// and branch, strict compares in ascending order); afterwards only the three taps of that row are looked at
// again and the first that equals the extremum is the winner.  (Tracking just the channel, as the
// two-dimensional kernel does, costs 27 scattered loads per output and branch afterwards, which at the
// few channels of volumetric nets outweighs the loop.)  Full-window modes, horizontal padding 0 or 1.
constexpr int TN3 = 4;

__device__ __forceinline__ unsigned fast_div3(unsigned u, unsigned inv) { return inv ? __umulhi(u, inv) : u; }

template <int MODE>
__global__ __launch_bounds__(WAVES * 64) void fwd3d_k3_kernel(Params3 p, const float* __restrict__ x,
                                                              const float* __restrict__ w_min,
                                                              const float* __restrict__ w_max,
                                                              const float* __restrict__ alpha,
                                                              const float* __restrict__ beta, float* __restrict__ y,
                                                              float* __restrict__ y_min, float* __restrict__ y_max,
                                                              int32_t* __restrict__ idx_min,
                                                              int32_t* __restrict__ idx_max, int segs,
                                                              unsigned n_units, unsigned inv_segs, unsigned inv_ho,
                                                              unsigned inv_do, int gblocks, unsigned inv_gblocks,
                                                              int n_blocks, int xcd_runs) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  // Workgroup number = pixel block * gblocks + output-channel block.  Workgroups are dealt round-robin to the 8
  // XCDs, each with its own L2; with xcd_runs every XCD gets a contiguous run of numbers, so that the channel
  // blocks of a pixel block (same input lines) run at the same time behind one L2.  The grid is padded to a
  // multiple of 8; the kernel has no barrier.
  const int per_xcd = (n_blocks + 7) >> 3;
  const int bid = xcd_runs ? (int)(blockIdx.x & 7u) * per_xcd + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  if (bid >= n_blocks) return;
  const unsigned ub = fast_div3((unsigned)bid, inv_gblocks);
  const int gb = bid - (int)ub * gblocks;
  const int co0 = (gb * WAVES + wave) * TN3;
  if (co0 >= p.C_out) return;  // whole wave
  const unsigned u_raw = ub * 64u + lane;
  const bool unit_ok = u_raw < n_units;
  const unsigned u = unit_ok ? u_raw : n_units - 1;  // surplus lanes recompute the last unit and store nothing
  const unsigned t1 = fast_div3(u, inv_segs);
  const int seg = (int)(u - t1 * (unsigned)segs);
  const unsigned t2 = fast_div3(t1, inv_ho);
  const int oh = (int)(t1 - t2 * (unsigned)p.Ho);
  const unsigned n = fast_div3(t2, inv_do);
  const int od = (int)(t2 - n * (unsigned)p.Do);
  const int ow0 = min(seg * 4, p.Wo - 4);
  const int first_q = unit_ok ? seg * 4 - ow0 : 4;

  // channel-independent addressing: 9 rows (depth a, height i), 6 columns
  const size_t vol = (size_t)p.D * p.H * p.W;
  const float* xn = x + (size_t)n * p.C_in * vol;
  int roff[9];
  bool rok[9];
#pragma unroll
  for (int a = 0; a < 3; ++a)
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int id = od - p.pd + a, ih = oh - p.ph + i;
      rok[a * 3 + i] = (id >= 0 && id < p.D && ih >= 0 && ih < p.H);
      roff[a * 3 + i] = (min(max(id, 0), p.D - 1) * p.H + min(max(ih, 0), p.H - 1)) * p.W;
    }
  int coff[6];
  bool cok[6];
#pragma unroll
  for (int k = 0; k < 6; ++k) {
    const int iw = ow0 - p.pw + k;
    cok[k] = (iw >= 0 && iw < p.W);
    coff[k] = min(max(iw, 0), p.W - 1);
  }

  const int core0 = ow0 - p.pw + 1;  // first of the four columns that are always in range

  float bmax[TN3][4], bmin[TN3][4];
  int cmax[TN3][4], cmin[TN3][4];  // winning row: channel * 9 + depth tap * 3 + height tap
#pragma unroll
  for (int c = 0; c < TN3; ++c)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      bmax[c][q] = -INFINITY; bmin[c][q] = INFINITY;
      cmax[c][q] = 0; cmin[c][q] = 0;
    }

  for (int ci = 0; ci < p.C_in; ++ci) {
    const float* xc = xn + (size_t)ci * vol;
    float xs[9][6];
#pragma unroll
    for (int r = 0; r < 9; ++r) {
      // columns 1..4 (the pixels themselves shifted by 1 - pw) always lie inside the row for pw <= 1
      const f4u core = *(const f4u*)(xc + roff[r] + core0);
      const float h0 = xc[roff[r] + coff[0]], h5 = xc[roff[r] + coff[5]];
      const float nan = __uint_as_float(0x7fc00000u);
      xs[r][0] = (rok[r] && cok[0]) ? h0 : nan;
      xs[r][1] = rok[r] ? core.x : nan;
      xs[r][2] = rok[r] ? core.y : nan;
      xs[r][3] = rok[r] ? core.z : nan;
      xs[r][4] = rok[r] ? core.w : nan;
      xs[r][5] = (rok[r] && cok[5]) ? h5 : nan;
    }
#pragma unroll
    for (int c = 0; c < TN3; ++c) {
      const int co = min(co0 + c, p.C_out - 1);  // a surplus channel slot recomputes the last channel, stores nothing
      const float* wa = DO_MIN ? w_min + ((size_t)co * p.C_in + ci) * 27 : nullptr;
      const float* wb = DO_MAX ? w_max + ((size_t)co * p.C_in + ci) * 27 : nullptr;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int r = 0; r < 9; ++r) {
          float s1[3], s2[3];
#pragma unroll
          for (int j = 0; j < 3; ++j) {
            if (DO_MIN) s1[j] = __fadd_rn(xs[r][q + j], wa[r * 3 + j]);
            if (DO_MAX) s2[j] = (MODE == TCONV_COMPOUND) ? s1[j] : __fadd_rn(xs[r][q + j], wb[r * 3 + j]);
          }
          const int row = ci * 9 + r;
          if (DO_MIN) {
            const float rm = fminf(fminf(s1[0], s1[1]), s1[2]);  // NaN (a row wholly in the padding) never wins
            cmin[c][q] = (rm < bmin[c][q]) ? row : cmin[c][q];
            bmin[c][q] = fminf(bmin[c][q], rm);
          }
          if (DO_MAX) {
            const float rM = fmaxf(fmaxf(s2[0], s2[1]), s2[2]);
            cmax[c][q] = (rM > bmax[c][q]) ? row : cmax[c][q];
            bmax[c][q] = fmaxf(bmax[c][q], rM);
          }
        }
      }
    }
  }

  // exact tap: the first of the three taps of the winning row whose sum equals the extremum
  auto refine = [&](const float* w, int co, int row, float best, int q) -> int {
    const int cs = min(row / 9, p.C_in - 1), r = row - (row / 9) * 9, a = r / 3, i = r - a * 3;
    const int id = min(max(od - p.pd + a, 0), p.D - 1), ih = min(max(oh - p.ph + i, 0), p.H - 1);
    const float* xr = xn + (size_t)cs * vol + ((size_t)id * p.H + ih) * p.W;
    const float* wr = w + ((size_t)co * p.C_in + cs) * 27 + r * 3;
    int res = cs * 27 + r * 3;
#pragma unroll
    for (int j = 2; j >= 0; --j) {
      const int iw = ow0 - p.pw + q + j;
      const float sum = __fadd_rn(xr[min(max(iw, 0), p.W - 1)], wr[j]);
      res = (iw >= 0 && iw < p.W && sum == best) ? cs * 27 + r * 3 + j : res;
    }
    return res;
  };
  const size_t ovol = (size_t)p.Do * p.Ho * p.Wo;
#pragma unroll
  for (int c = 0; c < TN3; ++c) {
    const int co = co0 + c;
    if (co >= p.C_out) break;  // wave-uniform
    const size_t ob = ((size_t)n * p.C_out + co) * ovol + ((size_t)od * p.Ho + oh) * p.Wo + ow0;
    float ca = 1.f, cb = 1.f;
    if (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL) {
      if (alpha) ca = alpha[co];
      if (beta) cb = beta[co];
    }
    int ridx[4];
    float out[4];
    if (DO_MIN) {
      for (int q = 0; q < 4; ++q) ridx[q] = refine(w_min, co, cmin[c][q], bmin[c][q], q);
      store_row<4>(idx_min + ob, ridx, first_q);
      if (y_min) store_row<4>(y_min + ob, bmin[c], first_q);
    }
    if (DO_MAX) {
      for (int q = 0; q < 4; ++q) ridx[q] = refine(w_max, co, cmax[c][q], bmax[c][q], q);
      store_row<4>(idx_max + ob, ridx, first_q);
      if (y_max) store_row<4>(y_max + ob, bmax[c], first_q);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (!DO_MIN) out[q] = bmax[c][q];
      else if (!DO_MAX) out[q] = bmin[c][q];
      else out[q] = combine(ca, bmin[c][q], cb, bmax[c][q]);
    }
    store_row<4>(y + ob, out, first_q);
  }
}

bool k3_ok(const Params3& p) {
  if (p.KD != 3 || p.KH != 3 || p.KW != 3) return false;
  if (p.sd != 1 || p.sh != 1 || p.sw != 1 || p.dd != 1 || p.dh != 1 || p.dw != 1) return false;
  if (p.mode > TCONV_PARALLEL || p.Wo < 4 || p.pw > 1) return false;
  const long long segs = (p.Wo + 3) / 4, units = (long long)p.N * p.Do * p.Ho * segs;
  const long long dmax = segs > p.Ho ? (segs > p.Do ? segs : p.Do) : (p.Ho > p.Do ? p.Ho : p.Do);
  if (units * dmax >= 0xffffffffLL) return false;                    // multiply-high quotients stay exact
  if ((long long)p.D * p.H * p.W >= 0x7fffffffLL) return false;      // 32-bit offsets inside a channel volume
  const long long gblocks = ((p.C_out + TN3 - 1) / TN3 + WAVES - 1) / WAVES;
  return ((units + 63) / 64) * gblocks < 0x7ffffff0LL / gblocks;  // workgroup numbers fit, their quotient by gblocks stays exact
}

unsigned inv3(int d) { return d > 1 ? (unsigned)(0x100000000ull / (unsigned)d) + 1u : 0u; }

template <int MODE>
hipError_t launch_k3(const Params3& p, const FwdArgs& a, hipStream_t s) {
  const int segs = (p.Wo + 3) / 4;
  const unsigned n_units = (unsigned)((long long)p.N * p.Do * p.Ho * segs);
  const int gblocks = ((p.C_out + TN3 - 1) / TN3 + WAVES - 1) / WAVES;
  const long long n_blocks = (long long)((n_units + 63) / 64) * gblocks;
  const long long w_bytes = (long long)p.C_out * p.K * (long long)sizeof(float) * (MODE == TCONV_PARALLEL ? 2 : 1);
  const char* xe = getenv("TCONV_XCD_RUNS");
  const int xcd_runs = xe ? atoi(xe) : (w_bytes <= 2LL * 1024 * 1024 ? 1 : 0);  // as for the two-dimensional kernel
  const dim3 grid((unsigned)(((n_blocks + 7) / 8) * 8));
  hipLaunchKernelGGL(fwd3d_k3_kernel<MODE>, grid, dim3(WAVES * 64), 0, s, p, (const float*)a.x, (const float*)a.w_min,
                     (const float*)a.w_max, a.alpha, a.beta, (float*)a.y, (float*)a.y_min, (float*)a.y_max, a.idx_min,
                     a.idx_max, segs, n_units, inv3(segs), inv3(p.Ho), inv3(p.Do), gblocks, inv3(gblocks),
                     (int)n_blocks, xcd_runs);
  return hipGetLastError();
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


// Input gradient without global atomics: a workgroup owns a box of TD depth slices x TH rows (all columns) of one
// image for a chunk of CC input channels, keeps their sums in LDS as fp64 ([CC][TD][TH][W]) and scans every output
// whose window can reach the box: the output depths and rows around it, all output columns and channels.  An
// output is taken if its winner lands inside the box.  Every input element belongs to exactly one workgroup, so
// plain stores finish the job (no zero fill).  The box is as cubic as LDS allows: an output is visited by
// (TD + reach) / TD x (TH + reach) / TH workgroups.  Item and element numbers unflatten by multiply-high
// (inv = floor(2^32 / d) + 1, exact while number * d < 2^32; the host passes 0 where that cannot be shown, then
// the kernel divides).  K27: the 3 x 3 x 3 window, whose tap numbers unflatten by constants.
__device__ __forceinline__ unsigned divq(unsigned u, unsigned d, unsigned inv) {
  return inv ? __umulhi(u, inv) : (d == 1 ? u : u / d);
}

template <int MODE, bool K27>
__global__ __launch_bounds__(1024) void bwd3d_input_tile_kernel(Params3 p, BwdArgs a, float* __restrict__ grad_x, int TD,
                                                                int TH, int CC, int tiles_d, int tiles_h, int chunks,
                                                                int n_blocks, int fast, unsigned inv_wo, unsigned inv_w,
                                                                unsigned inv_th, unsigned inv_td) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool SCALED = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  HIP_DYNAMIC_SHARED(double, tile3)
  const int bd = blockDim.x;
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: give every XCD a contiguous run of boxes,
  // so that neighbouring boxes (which scan the same gy / idx lines) share one L2.
  const int per_xcd = (n_blocks + 7) >> 3;
  int b = (int)(blockIdx.x & 7u) * per_xcd + (int)(blockIdx.x >> 3);
  if (b >= n_blocks) return;  // padding of the grid: the whole workgroup leaves before any barrier
  const int ch = b % chunks; b /= chunks;
  const int th = b % tiles_h; b /= tiles_h;
  const int td = b % tiles_d;
  const int n = b / tiles_d;
  const int d0 = td * TD, h0 = th * TH, c0 = ch * CC;
  const int tsz = CC * TD * TH * p.W;
  for (int e = threadIdx.x; e < tsz; e += bd) tile3[e] = 0.0;
  __syncthreads();

  const int KD = K27 ? 3 : p.KD, KH = K27 ? 3 : p.KH, KW = K27 ? 3 : p.KW, KHW = KH * KW, KK = KD * KHW;
  // output depths and rows whose window can reach the box
  const int nd = d0 + p.pd - (KD - 1) * p.dd, nh = h0 + p.ph - (KH - 1) * p.dh;
  const int od_lo = nd <= 0 ? 0 : (nd + p.sd - 1) / p.sd, oh_lo = nh <= 0 ? 0 : (nh + p.sh - 1) / p.sh;
  const int od_hi = min(p.Do - 1, (d0 + TD - 1 + p.pd) / p.sd), oh_hi = min(p.Ho - 1, (h0 + TH - 1 + p.ph) / p.sh);
  const int RH = max(oh_hi - oh_lo + 1, 0);
  const int P = RH * p.Wo;          // pixels per output depth and channel
  const int per_od = p.C_out * P;   // items per output depth: (co, oh, ow), ow fastest
  const unsigned inv_p = (fast && P > 1) ? 0xffffffffu / (unsigned)P + 1u : 0u;
  const size_t ovol = (size_t)p.Do * p.Ho * p.Wo;
  for (int od = od_lo; od <= od_hi && P > 0; ++od) {
    const int bdz = od * p.sd - p.pd - d0;
    const size_t obase = (size_t)n * p.C_out * ovol + (size_t)od * p.Ho * p.Wo;
    constexpr int UB = 4;  // items per thread in flight
    for (int it0 = threadIdx.x; it0 < per_od; it0 += bd * UB) {
      float gv[UB];
      int kmn[UB], kmx[UB], cov[UB], bhv[UB], bwv[UB];
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        const int it = min(it0 + u * bd, per_od - 1);
        const int co = P > 1 ? (int)divq((unsigned)it, (unsigned)P, inv_p) : it;
        const int px = it - co * P;
        const int r = (int)divq((unsigned)px, (unsigned)p.Wo, fast ? inv_wo : 0u);
        const int ow = px - r * p.Wo, oh = oh_lo + r;
        const size_t o = obase + (size_t)co * ovol + (size_t)oh * p.Wo + ow;
        gv[u] = a.gy[o];
        if (DO_MIN) kmn[u] = a.idx_min[o];
        if (DO_MAX) kmx[u] = a.idx_max[o];
        cov[u] = co;
        bhv[u] = oh * p.sh - p.ph - h0;
        bwv[u] = ow * p.sw - p.pw;
      }
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        if (it0 + u * bd >= per_od) break;
        const int bh = bhv[u], bw = bwv[u];
        auto deposit = [&](int k, double v) {
          const int c = k / KK, tt = k - c * KK, ka = tt / KHW, rr = tt - ka * KHW, ki = rr / KW, kj = rr - ki * KW;
          const int dz = bdz + ka * p.dd, ih = bh + ki * p.dh, iw = bw + kj * p.dw, cc = c - c0;
          if ((unsigned)dz < (unsigned)TD && (unsigned)ih < (unsigned)TH && (unsigned)iw < (unsigned)p.W &&
              (unsigned)cc < (unsigned)CC && d0 + dz < p.D && h0 + ih < p.H)
            atomicAdd(&tile3[((cc * TD + dz) * TH + ih) * p.W + iw], v);
        };
        const double g = (double)gv[u];
        if (DO_MIN) deposit(kmn[u], (SCALED && a.alpha) ? (double)a.alpha[cov[u]] * g : g);
        if (DO_MAX) deposit(kmx[u], (SCALED && a.beta) ? (double)a.beta[cov[u]] * g : g);
      }
    }
  }
  __syncthreads();
  const size_t vol = (size_t)p.D * p.H * p.W;
  float* gxn = grad_x + (size_t)n * p.C_in * vol;
  for (int e = threadIdx.x; e < tsz; e += bd) {
    const unsigned t1 = divq((unsigned)e, (unsigned)p.W, inv_w), t2 = divq(t1, (unsigned)TH, inv_th);
    const unsigned cc = divq(t2, (unsigned)TD, inv_td);
    const int iw = e - (int)t1 * p.W, ih = (int)t1 - (int)t2 * TH, dz = (int)t2 - (int)cc * TD;
    if (d0 + dz < p.D && h0 + ih < p.H && c0 + (int)cc < p.C_in)
      gxn[(size_t)(c0 + cc) * vol + ((size_t)(d0 + dz) * p.H + (h0 + ih)) * p.W + iw] = (float)tile3[e];
  }
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

static bool use_k3(const Params3& p) {
  const char* e = getenv("TCONV_FORWARD_KERNEL");
  return k3_ok(p) && !(e && strcmp(e, "generic") == 0);
}

const char* forward_3d_kernel_name(const Params3& p) { return use_k3(p) ? "k3x3x3" : "generic3d"; }

hipError_t launch_forward_3d(const Params3& p, const FwdArgs& a, hipStream_t s) {
  if (use_k3(p)) {
    switch (p.mode) {
      case TCONV_MAX: return launch_k3<TCONV_MAX>(p, a, s);
      case TCONV_MIN: return launch_k3<TCONV_MIN>(p, a, s);
      case TCONV_COMPOUND: return launch_k3<TCONV_COMPOUND>(p, a, s);
      default: return launch_k3<TCONV_PARALLEL>(p, a, s);
    }
  }
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
  // LDS box [CC][TD][TH][W] of doubles: all channels if a 2 x 2 box of them fits, else chunks of channels; then the
  // depth x row shape that lets the fewest workgroups visit an output
  size_t budget = 72 * 1024;  // two workgroups of 1024 threads per compute unit
  if (const char* eb = getenv("TCONV_BWD3_LDS_KB")) budget = (size_t)atoi(eb) * 1024;  // testing aid: smaller boxes
  const size_t row_bytes = (size_t)p.W * sizeof(double);
  const char* e = getenv("TCONV_FORWARD_KERNEL");
  const bool plain = e && strcmp(e, "generic") == 0;
  if (!plain && row_bytes <= budget) {
    const int min_rows = (p.D < 2 ? p.D : 2) * (p.H < 2 ? p.H : 2);
    int CC = p.C_in;
    while (CC > 1 && (size_t)CC * row_bytes * min_rows > budget) CC = (CC + 1) / 2;
    const int rows = (int)(budget / ((size_t)CC * row_bytes));  // (depth, row) pairs that fit
    const double ed = (double)(p.KD - 1) * p.dd, eh = (double)(p.KH - 1) * p.dh;
    int TD = 1, TH = 1;
    double best = 1e30;
    for (int td = 1; td <= p.D && td <= rows; ++td) {
      int thh = rows / td;
      if (thh > p.H) thh = p.H;
      const double cost = (td + ed) / td * (thh + eh) / thh;
      if (cost < best - 1e-9) { best = cost; TD = td; TH = thh; }
    }
    const int tiles_d = (p.D + TD - 1) / TD, tiles_h = (p.H + TH - 1) / TH, chunks = (p.C_in + CC - 1) / CC;
    TD = (p.D + tiles_d - 1) / tiles_d;  // even boxes
    TH = (p.H + tiles_h - 1) / tiles_h;
    const long long blocks = (long long)p.N * tiles_d * tiles_h * chunks;
    const long long tsz = (long long)CC * TD * TH * p.W;
    if (blocks <= 0x7ffffff0LL && tsz < 0x7fffffffLL) {
      const size_t lds = (size_t)tsz * sizeof(double);
      const dim3 grid((unsigned)(((blocks + 7) / 8) * 8));  // the kernel renumbers the workgroups per XCD
      const bool k27 = (p.KD == 3 && p.KH == 3 && p.KW == 3);
      // multiply-high quotients: items it < C_out * P with P <= Ho * Wo pixels; elements e < tsz
      const long long pmax = (long long)p.Ho * p.Wo;
      const int fast = ((long long)p.C_out * pmax < 0x100000000LL / pmax) ? 1 : 0;
      const long long dmax = p.W > TH ? (p.W > TD ? p.W : TD) : (TH > TD ? TH : TD);
      const bool fast_e = tsz * dmax < 0x100000000LL;
      const unsigned inv_wo = fast ? inv3(p.Wo) : 0u;
      const unsigned inv_w = fast_e ? inv3(p.W) : 0u, inv_th = fast_e ? inv3(TH) : 0u, inv_td = fast_e ? inv3(TD) : 0u;
      const int threads = 1024;
#define TCONV_LAUNCH_BWD3(M)                                                                                       \
  do {                                                                                                             \
    if (k27) hipLaunchKernelGGL((bwd3d_input_tile_kernel<M, true>), grid, dim3(threads), lds, s, p, a, grad_x, TD, TH, \
                                CC, tiles_d, tiles_h, chunks, (int)blocks, fast, inv_wo, inv_w, inv_th, inv_td);   \
    else hipLaunchKernelGGL((bwd3d_input_tile_kernel<M, false>), grid, dim3(threads), lds, s, p, a, grad_x, TD, TH,    \
                            CC, tiles_d, tiles_h, chunks, (int)blocks, fast, inv_wo, inv_w, inv_th, inv_td);       \
  } while (0)
      switch (p.mode) {
        case TCONV_MAX: TCONV_LAUNCH_BWD3(TCONV_MAX); break;
        case TCONV_MIN: TCONV_LAUNCH_BWD3(TCONV_MIN); break;
        case TCONV_COMPOUND: TCONV_LAUNCH_BWD3(TCONV_COMPOUND); break;
        default: TCONV_LAUNCH_BWD3(TCONV_PARALLEL); break;
      }
#undef TCONV_LAUNCH_BWD3
      return hipGetLastError();
    }
  }
  // rows too long for the LDS tile: zero fill and scatter with global atomics
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
