// Backward kernels: both route the output gradient through the saved winning-tap
// indices (sub-gradient of max / min: the whole gradient of a branch goes to the one
// x element and the one kernel element that produced the extremum).  Neither does
// any arithmetic beyond adds, so both are bound by reading gy and idx from HBM.
//
//   backward_input : grad_x[n, c*, ih*, iw*] += g_b   (input tile in LDS as fp64, ds_add_f64, plain stores)
//   backward_weight: grad_w_b[c_out, k*]    += g_b   (per-c_out LDS histogram, then flush)
// Both accumulate in fp64 in LDS (see below).
//
// g_min = alpha[c_out]*gy and g_max = beta[c_out]*gy in compound / parallel mode
// (paper Sec. 3.3 definitions), g = gy in max / min mode.
#include <stdlib.h>
#include <string.h>

#include <math.h>

#include <mutex>

#include "tile_common.h"

namespace tconv {

// ---- accumulation in LDS.  On gfx950 an LDS fp32 atomic add (ds_add_f32) runs about 9-12x slower than
// the 64-bit LDS atomics (measured with random addresses, cycles per wave instruction: ds_add_f32 ~190,
// ds_add_u64 ~16, ds_add_f64 ~22).  Both backward kernels therefore accumulate in fp64 with ds_add_f64:
// every term is the exact double product coef*gy, the order-dependence of the sum is at the 1e-16
// level, and each sum is rounded to fp32 once at the end.

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

// Tiled backward-input: no global atomics.  One workgroup owns an INPUT tile (CC channels x TH x TW
// pixels of one image) in LDS, scans every output whose window can reach the tile (the tile grown by
// the kernel extent, all C_out channels, every live branch), adds the gradients that land inside
// with fp64 LDS atomics and finally writes the tile to grad_x with plain coalesced stores.  Every input
// element belongs to exactly one workgroup, so grad_x needs no zero fill.  The price is re-reading
// gy / idx for the halo: (TH+e)(TW+e)/(TH*TW) times the algorithmic bytes (times the number of
// channel chunks when C_in*TH*TW does not fit in LDS); neighbouring tiles share those lines in L2.
// A winner k unflattens with two divisions; for the 3 x 3 window they are by constants, otherwise by
// multiply-high with inv = floor(2^32 / d) + 1 (exact while k * d < 2^32; inv = 0: plain division, which
// this target expands into dozens of vector instructions and which then dominates the kernel).
__device__ __forceinline__ int unflatten_div(int u, int d, unsigned inv) {
  return inv ? (int)__umulhi((unsigned)u, inv) : (d == 1 ? u : u / d);
}

// The kernel is bound by vector-instruction issue, not by LDS or memory (counters: the vector ALUs busy two thirds
// of the time, LDS a quarter), so its index arithmetic is kept off the slow paths: no division by a run-time value
// inside a loop (a 3 x 3 winner unflattens with full-rate 24-bit multiplies: k / 9 = (k * 58255) >> 19 while
// k < 73700, r / 3 = (r * 11) >> 5 for r < 9; the tile is written out with incremental coordinates and one
// multiply-high), and gy / idx are read through buffer resources of the image with 32-bit offsets.
template <int MODE, bool K3>
__global__ __launch_bounds__(1024) void bwd_input_tile_kernel(Params p, BwdArgs a,
                                                              float* __restrict__ grad_x, int TH,
                                                              int TW, int CC, int tiles_h,
                                                              int tiles_w, int chunks, unsigned inv_kk,
                                                              unsigned inv_kw, unsigned inv_tw, int k24) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX);
  constexpr bool DO_MAX = (MODE != TCONV_MIN);
  constexpr bool SCALED = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  HIP_DYNAMIC_SHARED(double, acc)  // [CC][TH][TW] fp64 sums
  const int bd = blockDim.x;
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Give every XCD a contiguous
  // run of tiles, so that the tiles of one image (which share halo rows of gy / idx) meet in one L2.
  const int nblk = p.N * tiles_h * tiles_w * chunks;
  const int per_xcd = (nblk + 7) / 8;
  int b = (int)(blockIdx.x % 8u) * per_xcd + (int)(blockIdx.x / 8u);
  if (b >= nblk || (int)(blockIdx.x / 8u) >= per_xcd) return;  // whole workgroup leaves before any barrier
  const int ch = b % chunks; b /= chunks;
  const int tw = b % tiles_w; b /= tiles_w;
  const int th = b % tiles_h;
  const int n = b / tiles_h;
  const int h0 = th * TH, w0 = tw * TW, c0 = ch * CC;
  const int tsz = CC * TH * TW;
  for (int e = threadIdx.x; e < tsz; e += bd) acc[e] = 0.0;

  // outputs whose window can reach the tile
  const int KHs = K3 ? 3 : p.KH, KWs = K3 ? 3 : p.KW, KK = KHs * KWs;
  const int nh = h0 + p.ph - (KHs - 1) * p.dh, nw = w0 + p.pw - (KWs - 1) * p.dw;
  const int oh_lo = nh <= 0 ? 0 : (nh + p.sh - 1) / p.sh;
  const int ow_lo = nw <= 0 ? 0 : (nw + p.sw - 1) / p.sw;
  const int oh_hi = min(p.Ho - 1, (h0 + TH - 1 + p.ph) / p.sh);
  const int ow_hi = min(p.Wo - 1, (w0 + TW - 1 + p.pw) / p.sw);
  const int RH = max(oh_hi - oh_lo + 1, 0), RW = max(ow_hi - ow_lo + 1, 0);
  const int P = RH * RW;  // output pixels scanned per output channel
  const int plane = p.Ho * p.Wo;

  if (P > 0) {
    // the outputs of image n, [C_out][plane]: 32-bit byte offsets (the host checks that they fit)
    const unsigned img_bytes = (unsigned)((size_t)p.C_out * plane * sizeof(float));
    const size_t img_off = (size_t)n * p.C_out * plane;
    const tile::rsrc_t r_gy = tile::make_rsrc(a.gy + img_off, img_bytes);
    const tile::rsrc_t r_mn = tile::make_rsrc((DO_MIN ? a.idx_min : a.idx_max) + img_off, img_bytes);
    const tile::rsrc_t r_mx = tile::make_rsrc((DO_MAX ? a.idx_max : a.idx_min) + img_off, img_bytes);
    const unsigned plane_bytes = (unsigned)plane * 4u;
    // A thread keeps ONE scanned pixel and walks output channels: with P <= bd pixels the threads form G = bd / P
    // channel groups (group g takes channels g, g + G, ...; bd - G * P threads idle), otherwise one group whose
    // threads loop over the pixels.  Consecutive threads read consecutive pixels of a plane row, and everything
    // that depends on the pixel only (its offset, where its taps fall in the tile) is computed once.
    const int G = max(bd / P, 1);
    const int cg = (int)threadIdx.x / P;  // 0 for every thread when P > bd
    constexpr int UB = 4;                 // items per thread in flight (12 independent loads)
    float gv[UB];
    int kmn[UB], kmx[UB];
    auto issue = [&](unsigned voff, int co0) {
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        const unsigned off = voff + __umul24((unsigned)min(co0 + u * G, p.C_out - 1), plane_bytes);
        gv[u] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r_gy, off, 0, 0));
        if (DO_MIN) kmn[u] = (int)__builtin_amdgcn_raw_buffer_load_b32(r_mn, off, 0, 0);
        if (DO_MAX) kmx[u] = (int)__builtin_amdgcn_raw_buffer_load_b32(r_mx, off, 0, 0);
      }
    };
    auto pixel = [&](int px, int& bh, int& bw, unsigned& voff) {
      const int prow = px / RW;
      const int oh = oh_lo + prow, ow = ow_lo + (px - prow * RW);
      bh = oh * p.sh - p.ph - h0; bw = ow * p.sw - p.pw - w0;  // tap (0, 0) relative to the tile
      voff = (unsigned)(oh * p.Wo + ow) * 4u;
    };
    const bool active = cg < G;
    int px = (int)threadIdx.x - cg * P, bh = 0, bw = 0;
    unsigned voff = 0;
    if (active) {  // the first loads go out before the tile is known to be zero: they do not touch LDS
      pixel(px, bh, bw, voff);
      issue(voff, cg);
    }
    __syncthreads();
    if (active) {
      // LDS element a winner lands on, -1: outside this workgroup's tile
      auto target = [&](int k) -> int {
        int c, i, j;
        if (K3 && k24) {
          c = (int)(__umul24((unsigned)k, 58255u) >> 19);
          const int r = k - __mul24(c, 9);
          i = (int)(__umul24((unsigned)r, 11u) >> 5);
          j = r - __mul24(i, 3);
        } else {
          c = K3 ? k / KK : unflatten_div(k, KK, inv_kk);
          const int r = k - c * KK;
          i = K3 ? r / KWs : unflatten_div(r, KWs, inv_kw);
          j = r - i * KWs;
        }
        const int ih = bh + __mul24(i, p.dh), iw = bw + __mul24(j, p.dw), cc = c - c0;
        const bool in = (unsigned)ih < (unsigned)TH && (unsigned)iw < (unsigned)TW && (unsigned)cc < (unsigned)CC;
        return in ? __mul24(__mul24(cc, TH) + ih, TW) + iw : -1;
      };
      for (;;) {
        for (int co0 = cg; co0 < p.C_out; co0 += G * UB) {
          if (co0 != cg) issue(voff, co0);
#pragma unroll
          for (int u = 0; u < UB; ++u) {
            const int co = co0 + u * G;
            if (co < p.C_out) {
              const double g = (double)gv[u];
              if (DO_MIN) {
                const int t = target(kmn[u]);
                if (t >= 0) atomicAdd(&acc[t], (SCALED && a.alpha) ? (double)a.alpha[co] * g : g);
              }
              if (DO_MAX) {
                const int t = target(kmx[u]);
                if (t >= 0) atomicAdd(&acc[t], (SCALED && a.beta) ? (double)a.beta[co] * g : g);
              }
            }
          }
        }
        px += bd;
        if (px >= P) break;
        pixel(px, bh, bw, voff);
        issue(voff, cg);
      }
    }
    __syncthreads();
  } else {
    __syncthreads();
  }
  // Write the tile (all zeros when no output reaches it).  Element e = (cc * TH + ih) * TW + iw; a thread's
  // elements are bd apart, so (cc * TH + ih, iw) advance by a fixed step with one carry.
  const size_t HW = (size_t)p.H * p.W;
  float* gxn = grad_x + (size_t)n * p.C_in * HW;
  const int d_row = bd / TW, d_col = bd - d_row * TW;  // uniform
  int row = TW == 1 ? (int)threadIdx.x : (int)__umulhi(threadIdx.x, inv_tw);  // cc * TH + ih; exact: threadIdx.x * TW < 2^32
  int iw = (int)threadIdx.x - row * TW;
  {
    // rows of the tile are numbered cc * TH + ih; split once per thread and carry from there on
    int cc = row / TH, ih = row - cc * TH;
    const int d_cc = d_row / TH, d_ih = d_row - d_cc * TH;
    for (int e = threadIdx.x; e < tsz; e += bd) {
      if (h0 + ih < p.H && w0 + iw < p.W && c0 + cc < p.C_in)
        gxn[(unsigned)((c0 + cc) * (int)HW + (h0 + ih) * p.W + (w0 + iw))] = (float)acc[e];
      iw += d_col; ih += d_ih; cc += d_cc;
      if (iw >= TW) { iw -= TW; ++ih; }
      if (ih >= TH) { ih -= TH; ++cc; }
    }
  }
}

// Input gradient of one-row inputs (sequences: H = 1, KH = 1).  Same ownership as the tiled kernel - a workgroup
// owns CC channels x TW positions of one sequence in LDS as fp64 and scans every output that can reach them -
// but a thread keeps ONE output position and walks the output channels.  On sequences the winners of the
// channels of a position coincide massively (a peak of the input wins in every window that covers it and for
// most kernels), and as LDS atomics on one address serialise, the pixel-major order of the tiled kernel is
// bound by them.  Here a thread adds up the run of equal targets in a register and issues one atomic per run.
template <int MODE>
__global__ __launch_bounds__(1024) void bwd_input_row_kernel(Params p, BwdArgs a, float* __restrict__ grad_x, int TW,
                                                             int CC, int tiles_w, int chunks, unsigned inv_kw) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX);
  constexpr bool DO_MAX = (MODE != TCONV_MIN);
  constexpr bool SCALED = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  HIP_DYNAMIC_SHARED(double, acc)  // [CC][TW]
  const int bd = blockDim.x, tid = threadIdx.x;
  int b = blockIdx.x;
  const int ch = b % chunks; b /= chunks;
  const int tw = b % tiles_w;
  const int n = b / tiles_w;
  const int w0 = tw * TW, c0 = ch * CC, tsz = CC * TW;
  for (int e = tid; e < tsz; e += bd) acc[e] = 0.0;
  __syncthreads();

  // output positions whose window can reach the tile
  const int nw = w0 + p.pw - (p.KW - 1) * p.dw;
  const int ow_lo = nw <= 0 ? 0 : (nw + p.sw - 1) / p.sw;
  const int ow_hi = min(p.Wo - 1, (w0 + TW - 1 + p.pw) / p.sw);
  const int P = max(ow_hi - ow_lo + 1, 0);
  if (P > 0) {
    // P >= bd: a thread takes positions tid, tid + bd, ... and all channels; P < bd: bd / P groups of threads
    // share the positions and deal the channels among them (surplus threads idle)
    const int groups = max(bd / P, 1);
    const int cg = tid / P;
    if (cg < groups) {
      for (int px = tid - cg * P; px < P; px += bd) {
        const int ow = ow_lo + px;
        const int bw = ow * p.sw - p.pw - w0;
        const size_t base = (size_t)n * p.C_out * p.Wo + ow;
        int am = -1, aM = -1;      // pending LDS element of the min / max branch, -1: none
        double sm = 0.0, sM = 0.0;
        auto target = [&](int k) -> int {
          const int c = inv_kw ? (int)__umulhi((unsigned)k, inv_kw) : (p.KW == 1 ? k : k / p.KW);
          const int j = k - c * p.KW, iw = bw + j * p.dw, cc = c - c0;
          return ((unsigned)iw < (unsigned)TW && (unsigned)cc < (unsigned)CC) ? cc * TW + iw : -1;
        };
        constexpr int UB = 4;
        for (int co0 = cg; co0 < p.C_out; co0 += groups * UB) {
          float gv[UB];
          int kmn[UB], kmx[UB];
#pragma unroll
          for (int u = 0; u < UB; ++u) {
            const int co = min(co0 + u * groups, p.C_out - 1);
            const size_t o = base + (size_t)co * p.Wo;
            gv[u] = a.gy[o];
            if (DO_MIN) kmn[u] = a.idx_min[o];
            if (DO_MAX) kmx[u] = a.idx_max[o];
          }
#pragma unroll
          for (int u = 0; u < UB; ++u) {
            const int co = co0 + u * groups;
            if (co >= p.C_out) break;
            const double g = (double)gv[u];
            if (DO_MIN) {
              const int t = target(kmn[u]);
              if (t != am) {
                if (am >= 0) atomicAdd(&acc[am], sm);
                am = t; sm = 0.0;
              }
              sm += (SCALED && a.alpha) ? (double)a.alpha[co] * g : g;
            }
            if (DO_MAX) {
              const int t = target(kmx[u]);
              if (t != aM) {
                if (aM >= 0) atomicAdd(&acc[aM], sM);
                aM = t; sM = 0.0;
              }
              sM += (SCALED && a.beta) ? (double)a.beta[co] * g : g;
            }
          }
        }
        if (DO_MIN && am >= 0) atomicAdd(&acc[am], sm);
        if (DO_MAX && aM >= 0) atomicAdd(&acc[aM], sM);
      }
    }
  }
  __syncthreads();
  float* gxn = grad_x + (size_t)n * p.C_in * p.W;
  for (int e = tid; e < tsz; e += bd) {
    const int iw = e % TW, cc = e / TW;
    if (w0 + iw < p.W && c0 + cc < p.C_in) gxn[(size_t)(c0 + cc) * p.W + (w0 + iw)] = (float)acc[e];
  }
}

// Tile shape for bwd_input_tile_kernel: minimise (channel chunks) x (halo re-read factor) under the
// LDS budget, with a penalty for rows too short to coalesce.
struct BwdInTile { int TH, TW, CC, tiles_h, tiles_w, chunks; };

// LDS bytes of a candidate: the tile.
static size_t bwd_input_lds_bytes(const Params& p, int CC, int TH, int TW) {
  (void)p;
  return (size_t)CC * TH * TW * sizeof(double);
}

// Cost of a candidate: (channel chunks) x halo^0.55 / utilisation^0.15 / (how evenly the workgroups fill 256 compute
// units, one resident workgroup each).  halo = scanned output pixels per owned input pixel (ragged last tiles scan
// nearly as much as full ones but own less), utilisation = share of the 1024 threads that own a scanned pixel (whole
// channel groups of P threads, see the kernel).  The exponents are fitted to measured times of two tile shapes each
// on the 32 x 32 and the 56 x 56 benchmark layers (64 channels): a tile's fixed work - zeroing, the write-out, the
// first load latency - does not grow with either.
static BwdInTile search_bwd_input_tile(const Params& p, size_t lds_budget) {
  BwdInTile best = {0, 0, 0, 0, 0, 0};
  double best_cost = 1e30;
  const int eh = (p.KH - 1) * p.dh, ew = (p.KW - 1) * p.dw;
  for (int chunks = 1; chunks <= p.C_in; chunks *= 2) {
    const int CC = (p.C_in + chunks - 1) / chunks;
    const int real_chunks = (p.C_in + CC - 1) / CC;
    // one-row inputs (sequences) have no second axis to grow the tile along: they take long rows instead
    const int tw_max = p.H == 1 ? 4096 : 128;
    for (int TWc = 8; TWc <= tw_max; TWc += (TWc < 64 ? 4 : (TWc < 256 ? 32 : 512))) {
      const int TW = TWc < p.W ? TWc : p.W;
      const int th_max = p.H < 64 ? p.H : 64;
      for (int TH = th_max; TH >= 1; --TH) {
        if (bwd_input_lds_bytes(p, CC, TH, TW) > lds_budget) continue;
        const long long RH = min((long long)p.Ho, (long long)(TH - 1 + eh) / p.sh + 1);
        const long long RW = min((long long)p.Wo, (long long)(TW - 1 + ew) / p.sw + 1);
        const long long P = RH * RW;  // output pixels an interior tile scans per output channel
        const int tiles_h = (p.H + TH - 1) / TH, tiles_w = (p.W + TW - 1) / TW;
        const double halo = (double)P * p.sh * p.sw / ((double)TH * TW) * ((double)tiles_h * TH / p.H) *
                            ((double)tiles_w * TW / p.W);
        const double util =
            P <= 1024 ? (double)(P * (1024 / P)) / 1024.0 : (double)P / (double)(((P + 1023) / 1024) * 1024);
        double cost = (double)real_chunks * pow(halo, 0.55) / pow(util, 0.15);
        if (RW < 16) cost *= 1.5;  // rows too short to coalesce
        const double wgs = (double)p.N * tiles_h * tiles_w * real_chunks;
        const double rounds = (double)(((long long)wgs + 255) / 256);
        cost *= rounds * 256.0 / wgs;  // idle compute units in the last round (or in the only one)
        if (cost < best_cost - 1e-12) {
          best_cost = cost;
          best = {TH, TW, CC, tiles_h, tiles_w, real_chunks};
        }
        if (TH * 2 < th_max && TH * 4 * (long long)TW * CC * 8 < (long long)lds_budget) break;  // far below the budget
      }
      if (TW == p.W) break;
    }
    if (CC == 1) break;
  }
  return best;
}

// The search runs once per layer shape and LDS budget (a few thousand candidates); later launches look the tile up.
static BwdInTile choose_bwd_input_tile(const Params& p, size_t lds_budget) {
  struct Entry { int key[14]; size_t budget; BwdInTile tile; };
  static std::mutex mu;
  static Entry cache[64];
  static int n_cached = 0;
  const int key[14] = {p.N, p.C_in, p.H, p.W, p.C_out, p.KH, p.KW, p.sh, p.sw, p.ph, p.pw, p.dh, p.dw, p.Ho * 65536 + p.Wo};
  {
    std::lock_guard<std::mutex> lock(mu);
    for (int e = 0; e < n_cached; ++e)
      if (cache[e].budget == lds_budget && memcmp(cache[e].key, key, sizeof(key)) == 0) return cache[e].tile;
  }
  const BwdInTile t = search_bwd_input_tile(p, lds_budget);
  {
    std::lock_guard<std::mutex> lock(mu);
    Entry& e = cache[n_cached < 64 ? n_cached++ : (key[0] + key[1] + key[2]) & 63];
    memcpy(e.key, key, sizeof(key));
    e.budget = lds_budget;
    e.tile = t;
  }
  return t;
}

// One-row inputs: positions per tile and channels per chunk, block size fitted to the scanned outputs.
static bool launch_backward_input_row(const Params& p, const BwdArgs& a, float* grad_x, hipStream_t s) {
  if (p.H != 1 || p.KH != 1 || p.Ho != 1) return false;
  if (const char* e = getenv("TCONV_BWD_ROW")) if (atoi(e) == 0) return false;
  const int TW = p.W < 2048 ? p.W : 2048;
  const size_t budget = 48 * 1024;
  int CC = (int)(budget / ((size_t)TW * sizeof(double)));
  if (CC < 1) return false;
  if (CC > p.C_in) CC = p.C_in;
  const int chunks = (p.C_in + CC - 1) / CC, tiles_w = (p.W + TW - 1) / TW;
  const long long blocks = (long long)p.N * tiles_w * chunks;
  if (blocks > 0x7fffffffLL) return false;
  const long long pmax = ((long long)TW - 1 + (long long)(p.KW - 1) * p.dw) / p.sw + 1;  // outputs that can reach a tile
  const int threads = pmax >= 1024 ? 1024 : (int)((pmax + 63) / 64) * 64;
  const unsigned inv_kw =
      (p.KW > 1 && (long long)p.K * p.KW < 0x100000000LL) ? (unsigned)(0x100000000ULL / (unsigned)p.KW) + 1u : 0u;
  const size_t lds = (size_t)CC * TW * sizeof(double);
#define TCONV_LAUNCH_BWD_ROW(M)                                                                                  \
  hipLaunchKernelGGL(bwd_input_row_kernel<M>, dim3((unsigned)blocks), dim3(threads), lds, s, p, a, grad_x, TW, CC, \
                     tiles_w, chunks, inv_kw)
  switch (p.mode) {
    case TCONV_MAX: TCONV_LAUNCH_BWD_ROW(TCONV_MAX); break;
    case TCONV_MIN: TCONV_LAUNCH_BWD_ROW(TCONV_MIN); break;
    default: TCONV_LAUNCH_BWD_ROW(TCONV_COMPOUND); break;  // compound and parallel route gradients identically
  }
#undef TCONV_LAUNCH_BWD_ROW
  return true;
}

hipError_t launch_backward_input(const Params& p, const BwdArgs& a, float* grad_x, hipStream_t s) {
  if (launch_backward_input_row(p, a, grad_x, s)) return hipGetLastError();
  // One workgroup per compute unit with nearly all of its 160 KB of LDS: measured faster than two half-size tiles on
  // every benchmark layer (a larger tile re-reads less halo; 30 / 60 / 78 / 100 / 156 KB: 76 / 53 / 49 / 47 / 45 us on
  // the cfg2 layer, 167 / 86 / 75 / 67 / 55 us on cfg4b)
  size_t LDS_BUDGET = 156 * 1024;
  if (const char* e = getenv("TCONV_BWD_LDS_KB")) LDS_BUDGET = (size_t)atoi(e) * 1024;
  const BwdInTile t = choose_bwd_input_tile(p, LDS_BUDGET);
  const long long blocks = (long long)p.N * t.tiles_h * t.tiles_w * t.chunks;
  // the tile kernel addresses the outputs of one image and the elements of one input image with 32 bits
  const bool fits32 = (size_t)p.C_out * p.Ho * p.Wo * sizeof(float) < 0xfffff000ull &&
                      (size_t)p.C_in * p.H * p.W < 0x7fffffffull && (size_t)p.Ho * p.Wo * 4 < (1u << 24) &&
                      p.C_out < (1 << 24);
  if (t.TH >= 1 && blocks <= 0x7fffffffLL && fits32) {
    const size_t lds = bwd_input_lds_bytes(p, t.CC, t.TH, t.TW);
    const long long grid_blocks = ((blocks + 7) / 8) * 8;  // the kernel remaps blockIdx per XCD
    const bool k3 = (p.KH == 3 && p.KW == 3);
    const long long kk = (long long)p.KH * p.KW;
    const auto inv_of = [](long long d, long long umax) -> unsigned {  // 0: the kernel divides plainly
      return (d > 1 && umax * d < 0x100000000LL) ? (unsigned)(0x100000000ULL / (unsigned long long)d) + 1u : 0u;
    };
    const unsigned inv_kk = inv_of(kk, p.K), inv_kw = inv_of(p.KW, kk);
    const unsigned inv_tw = (unsigned)(0x100000000ULL / (unsigned long long)t.TW) + 1u;  // exact for thread numbers
    const int k24 = p.K < 73700 ? 1 : 0;  // the 24-bit unflattening of a 3 x 3 winner is exact below that
#define TCONV_LAUNCH_BWD_IN(M, K3)                                                              \
  hipLaunchKernelGGL((bwd_input_tile_kernel<M, K3>), dim3((unsigned)grid_blocks), dim3(1024), lds, s, p, a, \
                     grad_x, t.TH, t.TW, t.CC, t.tiles_h, t.tiles_w, t.chunks, inv_kk, inv_kw, inv_tw, k24)
    switch (p.mode) {
      case TCONV_MAX: if (k3) TCONV_LAUNCH_BWD_IN(TCONV_MAX, true); else TCONV_LAUNCH_BWD_IN(TCONV_MAX, false); break;
      case TCONV_MIN: if (k3) TCONV_LAUNCH_BWD_IN(TCONV_MIN, true); else TCONV_LAUNCH_BWD_IN(TCONV_MIN, false); break;
      default:  // compound and parallel route gradients identically
        if (k3) TCONV_LAUNCH_BWD_IN(TCONV_COMPOUND, true); else TCONV_LAUNCH_BWD_IN(TCONV_COMPOUND, false);
        break;
    }
#undef TCONV_LAUNCH_BWD_IN
    return hipGetLastError();
  }
  // fallback: zero fill + global atomics
  fill_zero(grad_x, (size_t)p.N * p.C_in * p.H * p.W, s);
  const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
  const unsigned sblocks = (unsigned)((total + 255) / 256);
  switch (p.mode) {
    case TCONV_MAX:
      hipLaunchKernelGGL(bwd_input_scatter_kernel<TCONV_MAX>, dim3(sblocks), dim3(256), 0, s, p, a, grad_x);
      break;
    case TCONV_MIN:
      hipLaunchKernelGGL(bwd_input_scatter_kernel<TCONV_MIN>, dim3(sblocks), dim3(256), 0, s, p, a, grad_x);
      break;
    default:
      hipLaunchKernelGGL(bwd_input_scatter_kernel<TCONV_COMPOUND>, dim3(sblocks), dim3(256), 0, s, p, a, grad_x);
      break;
  }
  return hipGetLastError();
}

// One block = one output channel x one slice of the batch.  The block keeps a K-bin fp64 histogram
// per destination tensor in LDS, adds every (n, oh, ow) item of its slice with LDS atomics, then
// flushes the non-zero bins (rounded to fp32 once) with global atomics.
// NHIST = 1: a single destination (max, min, and compound where both branches share
// one grad_w); NHIST = 2: parallel (min branch -> grad_w_min, max branch -> grad_w_max).
// EXTRA (two-stage form only): the same pass also sums gy, gy * y_min and gy * y_max over the slice (the gradients
// of a bias and of the combine coefficients, Sec. 3.3) into three more fp64 slots behind the histogram.
struct ParamExtras {
  const float* y_min;  // EXTRA == 1: the branch outputs as the forward pass stored them; NULL: no grad_alpha
  const float* y_max;  //             NULL: no grad_beta
  // EXTRA == 2: no stored branch outputs; an output's y_min / y_max is formed again from its winner,
  // fl(x[winner] + w[winner]), the very add the forward pass made (a padded winner, possible under zero padding only,
  // reads x as +0)
  const float* x;
  const float* w_min;
  const float* w_max;
  int want_alpha, want_beta;
  int k3;            // 3 x 3 window with K < 73700
  unsigned inv_wo;   // 2^32 / W_out + 1 where that divides every pixel number of a plane exactly, else 0
  // where the three extra sums go when the batch is not sliced (one workgroup per output channel writes its results)
  float* grad_bias;
  float* grad_alpha;
  float* grad_beta;
};
constexpr int N_EXTRA = 3;  // bias, alpha, beta

template <int MODE, int EXTRA>
__global__ __launch_bounds__(1024) void bwd_weight_hist_kernel(Params p, BwdArgs a,
                                                              float* __restrict__ gw_min,
                                                              float* __restrict__ gw_max,
                                                              int n_per_block, double* __restrict__ partial,
                                                              ParamExtras ex) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX);
  constexpr bool DO_MAX = (MODE != TCONV_MIN);
  constexpr bool SCALED = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  constexpr int NHIST = (MODE == TCONV_PARALLEL) ? 2 : 1;
  HIP_DYNAMIC_SHARED(double, hist)  // NHIST * K sums; EXTRA: + 3 totals + 3 x 16 per-wave sums
  const int co = blockIdx.x;
  const int n0 = blockIdx.y * n_per_block;
  const int n1 = min(n0 + n_per_block, p.N);
  const int K = p.K;
  const int bd = blockDim.x;
  for (int k = threadIdx.x; k < NHIST * K; k += bd) hist[k] = 0.0;
  __syncthreads();
  double* hmin = hist;
  double* hmax = hist + (NHIST - 1) * K;
  const float ca = SCALED ? (a.alpha ? a.alpha[co] : 1.0f) : 1.0f;
  const float cb = SCALED ? (a.beta ? a.beta[co] : 1.0f) : 1.0f;
  const int plane = p.Ho * p.Wo;
  const int n_start = n0 + threadIdx.x / plane, q_start = threadIdx.x % plane;
  const int dn = bd / plane, dq = bd % plane;
  double s_bias = 0.0, s_alpha = 0.0, s_beta = 0.0;
  // items (image, pixel) of this slice, pixel-major; four per thread in flight
  {
    constexpr int UB = 4;
    int n = n_start, q = q_start;
    while (n < n1) {
      size_t ov[UB];
      bool okv[UB];
      float gv[UB], ymn[UB], ymx[UB];
      int kmn[UB], kmx[UB], nv[UB], qv[UB];
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        okv[u] = n < n1;
        nv[u] = okv[u] ? n : n0;
        qv[u] = q;
        ov[u] = ((size_t)(okv[u] ? n : n0) * p.C_out + co) * plane + q;
        q += dq;
        n += dn;
        if (q >= plane) { q -= plane; ++n; }
      }
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        gv[u] = a.gy[ov[u]];
        if (DO_MIN) kmn[u] = a.idx_min[ov[u]];
        if (DO_MAX) kmx[u] = a.idx_max[ov[u]];
        if (EXTRA == 1 && ex.y_min) ymn[u] = ex.y_min[ov[u]];
        if (EXTRA == 1 && ex.y_max) ymx[u] = ex.y_max[ov[u]];
      }
      if (EXTRA == 2) {
        const int KK = p.KH * p.KW;
        auto branch_output = [&](int nn, int qq, int k, const float* w) -> float {
          if ((unsigned)k >= (unsigned)K) return 0.f;  // a corrupted index stays in bounds (and adds nothing below)
          int c, i, j;
          if (ex.k3) {  // 3 x 3 windows, K < 73700: the winner unflattens with 24-bit multiplies (exact in that range)
            c = (int)(__umul24((unsigned)k, 58255u) >> 19);
            const int r = k - __mul24(c, 9);
            i = (int)(__umul24((unsigned)r, 11u) >> 5);
            j = r - __mul24(i, 3);
          } else {
            c = k / KK;
            const int r = k - c * KK;
            i = r / p.KW;
            j = r - i * p.KW;
          }
          const int oh = ex.inv_wo ? (int)__umulhi((unsigned)qq, ex.inv_wo) : qq / p.Wo, ow = qq - oh * p.Wo;
          const int ih = oh * p.sh - p.ph + i * p.dh, iw = ow * p.sw - p.pw + j * p.dw;
          const bool inside = (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
          const float xv = inside ? ex.x[((size_t)nn * p.C_in + c) * ((size_t)p.H * p.W) + (size_t)ih * p.W + iw] : 0.f;
          return __fadd_rn(xv, w[(size_t)co * K + k]);
        };
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          if (DO_MIN && ex.want_alpha) ymn[u] = branch_output(nv[u], qv[u], kmn[u], ex.w_min);
          if (DO_MAX && ex.want_beta) ymx[u] = branch_output(nv[u], qv[u], kmx[u], ex.w_max);
        }
      }
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        if (!okv[u]) continue;
        if (EXTRA) {
          const double g = (double)gv[u];
          s_bias += g;
          if (EXTRA == 1 ? ex.y_min != nullptr : (DO_MIN && ex.want_alpha)) s_alpha += g * (double)ymn[u];
          if (EXTRA == 1 ? ex.y_max != nullptr : (DO_MAX && ex.want_beta)) s_beta += g * (double)ymx[u];
        }
        if (DO_MIN && (unsigned)kmn[u] < (unsigned)K)
          atomicAdd(hmin + kmn[u], SCALED ? (double)ca * (double)gv[u] : (double)gv[u]);
        if (DO_MAX && (unsigned)kmx[u] < (unsigned)K)
          atomicAdd(hmax + kmx[u], SCALED ? (double)cb * (double)gv[u] : (double)gv[u]);
      }
    }
  }
  if (EXTRA) {  // a wave's three sums (butterfly), then the 16 waves' in wave order: a fixed order of additions
    double* wsum = hist + NHIST * K + N_EXTRA;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      s_bias += __shfl_xor(s_bias, off);
      s_alpha += __shfl_xor(s_alpha, off);
      s_beta += __shfl_xor(s_beta, off);
    }
    if ((threadIdx.x & 63) == 0) {
      const int w = threadIdx.x >> 6;
      wsum[w] = s_bias; wsum[16 + w] = s_alpha; wsum[32 + w] = s_beta;
    }
  }
  __syncthreads();
  if (EXTRA) {
    if (threadIdx.x < N_EXTRA) {
      const double* wsum = hist + NHIST * K + N_EXTRA + 16 * threadIdx.x;
      double t = 0.0;
      for (int w = 0; w < bd / 64; ++w) t += wsum[w];
      hist[NHIST * K + threadIdx.x] = t;
    }
    __syncthreads();
  }
  if (partial && gridDim.y == 1) {
    // the batch is not sliced (at least 512 output channels): this workgroup's sums are the result, rounded once as the
    // second stage would round them; no partial histograms, no second kernel
    float* d0 = (MODE == TCONV_MAX) ? gw_max : gw_min;
    for (int k = threadIdx.x; k < K; k += bd) {
      d0[(size_t)co * K + k] = (float)hist[k];
      if (NHIST == 2) gw_max[(size_t)co * K + k] = (float)hmax[k];
    }
    if (EXTRA && threadIdx.x < N_EXTRA) {
      float* const d = threadIdx.x == 0 ? ex.grad_bias : (threadIdx.x == 1 ? ex.grad_alpha : ex.grad_beta);
      if (d) d[co] = (float)hist[NHIST * K + threadIdx.x];
    }
    return;
  }
  if (partial) {  // two-stage form: the fp64 histogram of this (batch slice, channel) as it is; a second kernel adds the slices
    const int NH = NHIST * K + (EXTRA ? N_EXTRA : 0);
    double* dst = partial + ((size_t)blockIdx.y * p.C_out + co) * (size_t)NH;
    for (int k = threadIdx.x; k < NH; k += bd) dst[k] = hist[k];
    return;
  }
  float* dmin = (MODE == TCONV_MAX) ? gw_max : gw_min;  // NHIST == 1: the single destination
  for (int k = threadIdx.x; k < K; k += bd) {
    const double v = hist[k];
    if (v != 0.0) atomicAdd(dmin + (size_t)co * K + k, (float)v);
    if (NHIST == 2) {
      const double v2 = hmax[k];
      if (v2 != 0.0) atomicAdd(gw_max + (size_t)co * K + k, (float)v2);
    }
  }
}

// Second stage of the deterministic kernel gradient: grad_w[co, k] = the partial histograms of the batch slices
// added in ascending slice order in fp64, rounded to fp32 once.  Writes every element: no zero fill, no atomics.
__global__ __launch_bounds__(256) void bwd_weight_reduce_kernel(const double* __restrict__ partial,
                                                                float* __restrict__ dst0, float* __restrict__ dst1,
                                                                int nhist, int K, int C_out, int slices) {
  const size_t total = (size_t)C_out * K, per_slice = total * nhist;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
    const size_t co = e / (size_t)K, k = e - co * K;
    for (int h = 0; h < nhist; ++h) {
      const double* src = partial + (co * nhist + h) * (size_t)K + k;
      double v = 0.0;
      // the loads of 8 slices go out together (the adds keep their order): this kernel is a chain of load latencies
#pragma unroll 8
      for (int sl = 0; sl < slices; ++sl) v += src[(size_t)sl * per_slice];
      (h == 0 ? dst0 : dst1)[e] = (float)v;
    }
  }
}

// The same second stage for the pass that also carries the three extra sums: a slice's record per output channel is
// nhist * K bins followed by the sums of gy, gy * y_min, gy * y_max.
__global__ __launch_bounds__(256) void bwd_params_reduce_kernel(const double* __restrict__ partial,
                                                                float* __restrict__ dst0, float* __restrict__ dst1,
                                                                float* __restrict__ grad_bias,
                                                                float* __restrict__ grad_alpha,
                                                                float* __restrict__ grad_beta, int nhist, int K,
                                                                int C_out, int slices) {
  const size_t NH = (size_t)nhist * K + N_EXTRA, total = (size_t)C_out * NH;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
    const size_t co = e / NH, r = e - co * NH;
    const double* src = partial + e;
    double v = 0.0;
#pragma unroll 8
    for (int sl = 0; sl < slices; ++sl) v += src[(size_t)sl * total];
    if (r < (size_t)K) dst0[co * K + r] = (float)v;
    else if (r < (size_t)nhist * K) dst1[co * K + (r - K)] = (float)v;
    else {
      float* const d = (r == (size_t)nhist * K) ? grad_bias : (r == (size_t)nhist * K + 1) ? grad_alpha : grad_beta;
      if (d) d[co] = (float)v;
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

// Batch slices of the histogram kernel: about two 1024-thread workgroups per compute unit in all.
static int weight_slices(const Params& p, int* n_per_block) {
  int slices = (512 + p.C_out - 1) / p.C_out;
  if (slices > p.N) slices = p.N;
  if (slices < 1) slices = 1;
  *n_per_block = (p.N + slices - 1) / slices;
  return (p.N + *n_per_block - 1) / *n_per_block;
}

static bool weight_hist_fits(const Params& p) {
  const int nhist = (p.mode == TCONV_PARALLEL) ? 2 : 1;
  return (size_t)nhist * p.K * sizeof(double) <= 64 * 1024;
}

// Scratch of the deterministic (two-stage) kernel gradient: one fp64 histogram per (batch slice, output channel,
// destination tensor).  0: the layer's histogram does not fit LDS and the scatter kernel (global atomics) runs.
size_t backward_weight_workspace(const Params& p) {
  if (!weight_hist_fits(p)) return 0;
  int npb = 0;
  const int slices = weight_slices(p, &npb);
  const int nhist = (p.mode == TCONV_PARALLEL) ? 2 : 1;
  return (size_t)slices * p.C_out * nhist * p.K * sizeof(double);
}

hipError_t launch_backward_weight(const Params& p, const BwdArgs& a, float* grad_w_min,
                                  float* grad_w_max, double* partial, hipStream_t s) {
  const size_t wn = (size_t)p.C_out * p.K;
  float* gmin = grad_w_min;
  float* gmax = grad_w_max;
  if (p.mode == TCONV_COMPOUND) gmin = gmax = (grad_w_min ? grad_w_min : grad_w_max);
  const bool hist = weight_hist_fits(p);
  if (!hist) partial = nullptr;
  if (!partial) {  // the atomic forms add into zero-filled tensors
    if (p.mode != TCONV_MAX) fill_zero(gmin, wn, s);
    if (p.mode == TCONV_MAX || p.mode == TCONV_PARALLEL) fill_zero(gmax, wn, s);
  }

  const int nhist = (p.mode == TCONV_PARALLEL) ? 2 : 1;
  const size_t lds = (size_t)nhist * p.K * sizeof(double);
  if (hist) {
    // two 1024-thread workgroups per CU; few slices keep the second stage (or the flush atomics) small
    int n_per_block = 0;
    const int slices = weight_slices(p, &n_per_block);
    dim3 grid(p.C_out, slices);
    switch (p.mode) {
      case TCONV_MAX:
        hipLaunchKernelGGL((bwd_weight_hist_kernel<TCONV_MAX, 0>), grid, dim3(1024), lds, s, p, a, gmin, gmax, n_per_block, partial, ParamExtras{});
        break;
      case TCONV_MIN:
        hipLaunchKernelGGL((bwd_weight_hist_kernel<TCONV_MIN, 0>), grid, dim3(1024), lds, s, p, a, gmin, gmax, n_per_block, partial, ParamExtras{});
        break;
      case TCONV_COMPOUND:
        hipLaunchKernelGGL((bwd_weight_hist_kernel<TCONV_COMPOUND, 0>), grid, dim3(1024), lds, s, p, a, gmin, gmax, n_per_block, partial, ParamExtras{});
        break;
      default:
        hipLaunchKernelGGL((bwd_weight_hist_kernel<TCONV_PARALLEL, 0>), grid, dim3(1024), lds, s, p, a, gmin, gmax, n_per_block, partial, ParamExtras{});
        break;
    }
    if (partial && slices > 1) {  // one slice: the histogram kernel has written the result itself
      size_t blocks = (wn + 255) / 256;
      if (blocks > 2048) blocks = 2048;
      float* d0 = (p.mode == TCONV_MAX) ? gmax : gmin;
      hipLaunchKernelGGL(bwd_weight_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, partial, d0, gmax, nhist, p.K,
                         p.C_out, slices);
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

// ---- every parameter gradient of a layer from one pass over gy: the kernel gradient(s) as launch_backward_weight
// writes them in its two-stage form, and from the same loads grad_bias[c] = sum gy, grad_alpha[c] = sum gy * y_min,
// grad_beta[c] = sum gy * y_max (each optional).  One histogram kernel and one reduction instead of three kernels
// and three reductions: a training step of a small layer is a chain of launch latencies, not of bytes.
// 0: no fused form for this layer (window too large for an on-chip histogram); the caller runs the separate kernels.
size_t backward_params_workspace(const Params& p) {
  if (!weight_hist_fits(p)) return 0;
  int npb = 0;
  const int slices = weight_slices(p, &npb);
  const int nhist = (p.mode == TCONV_PARALLEL) ? 2 : 1;
  return (size_t)slices * p.C_out * ((size_t)nhist * p.K + N_EXTRA) * sizeof(double);
}

hipError_t launch_backward_params(const Params& p, const BwdArgs& a, const float* y_min, const float* y_max,
                                  const float* x, const float* w_min, const float* w_max, float* grad_w_min,
                                  float* grad_w_max, float* grad_alpha, float* grad_beta, float* grad_bias,
                                  double* partial, hipStream_t s) {
  float* gmin = grad_w_min;
  float* gmax = grad_w_max;
  if (p.mode == TCONV_COMPOUND) gmin = gmax = (grad_w_min ? grad_w_min : grad_w_max);
  const int nhist = (p.mode == TCONV_PARALLEL) ? 2 : 1;
  const size_t lds = ((size_t)nhist * p.K + N_EXTRA + 16 * N_EXTRA) * sizeof(double);
  int n_per_block = 0;
  const int slices = weight_slices(p, &n_per_block);
  const dim3 grid(p.C_out, slices);
  const bool recompute = x != nullptr;  // the branch outputs again from the winners instead of stored tensors
  const long long plane = (long long)p.Ho * p.Wo;
  const unsigned inv_wo = (p.Wo > 1 && plane * p.Wo < 0x100000000LL) ? (unsigned)(0x100000000ULL / (unsigned)p.Wo) + 1u : 0u;
  const ParamExtras ex = {(!recompute && grad_alpha) ? y_min : nullptr, (!recompute && grad_beta) ? y_max : nullptr,
                          x, w_min, w_max, (recompute && grad_alpha) ? 1 : 0, (recompute && grad_beta) ? 1 : 0,
                          (p.KH == 3 && p.KW == 3 && p.K < 73700) ? 1 : 0, inv_wo, grad_bias, grad_alpha, grad_beta};
#define TCONV_LAUNCH_PARAMS(M)                                                                                       \
  do {                                                                                                               \
    if (recompute)                                                                                                   \
      hipLaunchKernelGGL((bwd_weight_hist_kernel<M, 2>), grid, dim3(1024), lds, s, p, a, gmin, gmax, n_per_block,    \
                         partial, ex);                                                                               \
    else                                                                                                             \
      hipLaunchKernelGGL((bwd_weight_hist_kernel<M, 1>), grid, dim3(1024), lds, s, p, a, gmin, gmax, n_per_block,    \
                         partial, ex);                                                                               \
  } while (0)
  switch (p.mode) {
    case TCONV_MAX: TCONV_LAUNCH_PARAMS(TCONV_MAX); break;
    case TCONV_MIN: TCONV_LAUNCH_PARAMS(TCONV_MIN); break;
    case TCONV_COMPOUND: TCONV_LAUNCH_PARAMS(TCONV_COMPOUND); break;
    default: TCONV_LAUNCH_PARAMS(TCONV_PARALLEL); break;
  }
#undef TCONV_LAUNCH_PARAMS
  if (slices == 1) return hipGetLastError();  // one slice: the histogram kernel has written the results itself
  const size_t total = (size_t)p.C_out * ((size_t)nhist * p.K + N_EXTRA);
  size_t blocks = (total + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  float* d0 = (p.mode == TCONV_MAX) ? gmax : gmin;
  hipLaunchKernelGGL(bwd_params_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, partial, d0, gmax, grad_bias,
                     grad_alpha, grad_beta, nhist, p.K, p.C_out, slices);
  return hipGetLastError();
}

// ---- the kernel gradient for callers that cannot hand over a workspace: the partial histograms live in a fixed
// array in device memory that belongs to the library (each GPU the library runs on holds its own copy until the
// process ends).  In host code the array's name is only a stand-in for that per-device copy; its device address is
// asked for once per device and that pointer is what the kernels get.
constexpr size_t STATIC_SCRATCH_BYTES = 32u << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

size_t backward_weight_static_limit() { return STATIC_SCRATCH_BYTES; }

// The scratch array's address on the current device (NULL and an error code if the runtime refuses).
static hipError_t static_scratch(double** out) {
  constexpr int MAX_DEV = 64;
  static std::mutex lock;
  static void* ptrs[MAX_DEV] = {};
  *out = nullptr;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEV) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> g(lock);
  if (!ptrs[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    ptrs[dev] = ptr;
  }
  *out = (double*)ptrs[dev];
  return hipSuccess;
}

// Deterministic kernel gradient with the library's own scratch.  hipErrorOutOfMemory: the layer needs more than the
// array holds (nothing was enqueued).  Every partial histogram is written before it is read, so the array needs no
// clearing between calls; two calls in flight on one GPU at the same time would share it and race.
hipError_t launch_backward_weight_static(const Params& p, const BwdArgs& a, float* grad_w_min, float* grad_w_max,
                                         hipStream_t s) {
  const size_t need = backward_weight_workspace(p);
  if (need > STATIC_SCRATCH_BYTES) return hipErrorOutOfMemory;
  double* partial = nullptr;
  if (need > 0) {
    const hipError_t e = static_scratch(&partial);
    if (e != hipSuccess) return e;
  }
  return launch_backward_weight(p, a, grad_w_min, grad_w_max, partial, s);
}

// ---- gradient of the combine step (paper Sec. 3.3: y = alpha*y_min + beta*y_max with learnable alpha,
// beta, one pair per output channel here): grad_alpha[c] = sum over (n, oh, ow) of gy*y_min, grad_beta[c]
// the same with y_max.  HBM bound: gy and the branch outputs are read once.  Workgroup = one output
// channel x a slice of the batch; fp64 partial sums per thread, reduced through LDS, one fp32 atomic per
// workgroup and output into the zero-filled result.
template <typename TY>
__global__ __launch_bounds__(256) void bwd_alpha_beta_kernel(Params p, const float* __restrict__ gy,
                                                             const TY* __restrict__ y_min,
                                                             const TY* __restrict__ y_max,
                                                             float* __restrict__ grad_alpha,
                                                             float* __restrict__ grad_beta, int n_per_block,
                                                             double* __restrict__ partial) {
  const int co = blockIdx.x;
  const int n0 = blockIdx.y * n_per_block;
  const int n1 = min(n0 + n_per_block, p.N);
  const size_t plane = (size_t)p.Ho * p.Wo;
  double sa = 0.0, sb = 0.0;
  // fp32 planes of a multiple of four elements are read 16 bytes at a time (plane bases are then 16-byte aligned
  // when the tensors are); a thread's terms are added in a fixed order either way
  const bool vec4 = sizeof(TY) == 4 && (plane & 3) == 0 &&
                    ((((uintptr_t)gy | (uintptr_t)y_min | (uintptr_t)y_max) & 15) == 0);
  for (int n = n0; n < n1; ++n) {
    const size_t base = ((size_t)n * p.C_out + co) * plane;
    if (vec4) {
      const float4* g4 = (const float4*)(gy + base);
      const float4* a4 = (const float4*)((const float*)y_min + base);
      const float4* b4 = (const float4*)((const float*)y_max + base);
#pragma unroll 2
      for (size_t i = threadIdx.x; i < plane / 4; i += blockDim.x) {
        const float4 g = g4[i];
        if (grad_alpha) {
          const float4 v = a4[i];
          sa += (double)g.x * (double)v.x; sa += (double)g.y * (double)v.y;
          sa += (double)g.z * (double)v.z; sa += (double)g.w * (double)v.w;
        }
        if (grad_beta) {
          const float4 v = b4[i];
          sb += (double)g.x * (double)v.x; sb += (double)g.y * (double)v.y;
          sb += (double)g.z * (double)v.z; sb += (double)g.w * (double)v.w;
        }
      }
      continue;
    }
    for (size_t i = threadIdx.x; i < plane; i += blockDim.x) {
      const float g = gy[base + i];
      if (grad_alpha) sa += (double)g * (double)ld_f32(y_min, base + i);
      if (grad_beta) sb += (double)g * (double)ld_f32(y_max, base + i);
    }
  }
  __shared__ double red[2][256];
  red[0][threadIdx.x] = sa;
  red[1][threadIdx.x] = sb;
  __syncthreads();
  for (int h = 128; h > 0; h >>= 1) {
    if ((int)threadIdx.x < h) {
      red[0][threadIdx.x] += red[0][threadIdx.x + h];
      red[1][threadIdx.x] += red[1][threadIdx.x + h];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    if (partial) {  // two-stage form: this slice's fp64 sums; ab_reduce_kernel adds the slices
      partial[((size_t)blockIdx.y * p.C_out + co) * 2] = red[0][0];
      partial[((size_t)blockIdx.y * p.C_out + co) * 2 + 1] = red[1][0];
    } else {
      if (grad_alpha) atomicAdd(grad_alpha + co, (float)red[0][0]);
      if (grad_beta) atomicAdd(grad_beta + co, (float)red[1][0]);
    }
  }
}

// Second stage: the slices' sums in ascending slice order, in fp64, rounded to fp32 once.
__global__ __launch_bounds__(256) void ab_reduce_kernel(const double* __restrict__ partial, float* __restrict__ grad_alpha,
                                                        float* __restrict__ grad_beta, int C_out, int slices) {
  const int co = blockIdx.x * blockDim.x + threadIdx.x;
  if (co >= C_out) return;
  double sa = 0.0, sb = 0.0;
#pragma unroll 8
  for (int sl = 0; sl < slices; ++sl) {
    const double2 v = *(const double2*)(partial + ((size_t)sl * C_out + co) * 2);
    sa += v.x;
    sb += v.y;
  }
  if (grad_alpha) grad_alpha[co] = (float)sa;
  if (grad_beta) grad_beta[co] = (float)sb;
}

static int ab_slices(const Params& p, int* n_per_block) {
  // about eight 256-thread workgroups per compute unit (these kernels stream their operands once and need the
  // loads of many waves in flight), each with at least one image
  int slices = (2048 + p.C_out - 1) / p.C_out;
  if (slices > p.N) slices = p.N;
  if (slices > 65535) slices = 65535;
  *n_per_block = (p.N + slices - 1) / slices;
  return (p.N + *n_per_block - 1) / *n_per_block;
}

// Scratch of the deterministic form: two fp64 sums per (batch slice, output channel).
size_t backward_alpha_beta_workspace(const Params& p) {
  int npb = 0;
  return (size_t)ab_slices(p, &npb) * p.C_out * 2 * sizeof(double);
}

hipError_t launch_backward_alpha_beta(const Params& p, int dtype, const float* gy, const void* y_min,
                                      const void* y_max, float* grad_alpha, float* grad_beta, double* partial,
                                      hipStream_t s) {
  if (!partial) {
    if (grad_alpha) fill_zero(grad_alpha, (size_t)p.C_out, s);
    if (grad_beta) fill_zero(grad_beta, (size_t)p.C_out, s);
  }
  int n_per_block = 0;
  const int slices = ab_slices(p, &n_per_block);
  const dim3 grid((unsigned)p.C_out, (unsigned)slices);
  if (dtype == TCONV_F16)
    hipLaunchKernelGGL(bwd_alpha_beta_kernel<f16_t>, grid, dim3(256), 0, s, p, gy, (const f16_t*)y_min,
                       (const f16_t*)y_max, grad_alpha, grad_beta, n_per_block, partial);
  else if (dtype == TCONV_BF16)
    hipLaunchKernelGGL(bwd_alpha_beta_kernel<bf16_t>, grid, dim3(256), 0, s, p, gy, (const bf16_t*)y_min,
                       (const bf16_t*)y_max, grad_alpha, grad_beta, n_per_block, partial);
  else
    hipLaunchKernelGGL(bwd_alpha_beta_kernel<float>, grid, dim3(256), 0, s, p, gy, (const float*)y_min,
                       (const float*)y_max, grad_alpha, grad_beta, n_per_block, partial);
  if (partial)
    hipLaunchKernelGGL(ab_reduce_kernel, dim3((unsigned)((p.C_out + 255) / 256)), dim3(256), 0, s, partial, grad_alpha,
                       grad_beta, p.C_out, slices);
  return hipGetLastError();
}

// ---- gradient of the epilogue's bias: grad_bias[c] = sum over (n, oh, ow) of gy.  Same layout of workgroups and the
// same two forms (fp32 atomic per workgroup, or fp64 partial sums added by ab_reduce_kernel) as the kernel above.
__global__ __launch_bounds__(256) void bwd_bias_kernel(Params p, const float* __restrict__ gy,
                                                       float* __restrict__ grad_bias, int n_per_block,
                                                       double* __restrict__ partial) {
  const int co = blockIdx.x;
  const int n0 = blockIdx.y * n_per_block;
  const int n1 = min(n0 + n_per_block, p.N);
  const size_t plane = (size_t)p.Ho * p.Wo;
  double sa = 0.0;
  const bool vec4 = (plane & 3) == 0 && (((uintptr_t)gy & 15) == 0);
  for (int n = n0; n < n1; ++n) {
    const size_t base = ((size_t)n * p.C_out + co) * plane;
    if (vec4) {
      const float4* g4 = (const float4*)(gy + base);
#pragma unroll 2
      for (size_t i = threadIdx.x; i < plane / 4; i += blockDim.x) {
        const float4 g = g4[i];
        sa += (double)g.x; sa += (double)g.y; sa += (double)g.z; sa += (double)g.w;
      }
      continue;
    }
    for (size_t i = threadIdx.x; i < plane; i += blockDim.x) sa += (double)gy[base + i];
  }
  __shared__ double red[256];
  red[threadIdx.x] = sa;
  __syncthreads();
  for (int h = 128; h > 0; h >>= 1) {
    if ((int)threadIdx.x < h) red[threadIdx.x] += red[threadIdx.x + h];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    if (partial) {
      partial[((size_t)blockIdx.y * p.C_out + co) * 2] = red[0];
      partial[((size_t)blockIdx.y * p.C_out + co) * 2 + 1] = 0.0;
    } else {
      atomicAdd(grad_bias + co, (float)red[0]);
    }
  }
}

hipError_t launch_backward_bias(const Params& p, const float* gy, float* grad_bias, double* partial, hipStream_t s) {
  if (!partial) fill_zero(grad_bias, (size_t)p.C_out, s);
  int n_per_block = 0;
  const int slices = ab_slices(p, &n_per_block);
  hipLaunchKernelGGL(bwd_bias_kernel, dim3((unsigned)p.C_out, (unsigned)slices), dim3(256), 0, s, p, gy, grad_bias,
                     n_per_block, partial);
  if (partial)
    hipLaunchKernelGGL(ab_reduce_kernel, dim3((unsigned)((p.C_out + 255) / 256)), dim3(256), 0, s, partial, grad_bias,
                       (float*)nullptr, p.C_out, slices);
  return hipGetLastError();
}

}  // namespace tconv
