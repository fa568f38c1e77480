// Tiled forward kernel for 3x3, stride-1 tropical convolutions on gfx950: a VALU "semiring GEMM".
//
// Operator: paper Sec. 3.1 layers (iv) / (v) (one min / max over all C_in*9 taps of x + w) and the
// Sec. 3.3 compound (one shared add feeds both reductions, Sec. 3.5 closing remark) and parallel
// combinations.  The semiring has no multiply, so the matrix cores do not apply; the kernel is
// built for the vector ALUs:
//
//  * A lane owns a row segment of 8 consecutive output pixels and 4 output channels: 32 running
//    extrema per branch stay in VGPRs for the whole K loop.  The 4 waves of a workgroup share the
//    pixel segments (same x lines in L1) and differ in output-channel group.  No LDS, no barrier.
//  * Kernel values are wave-uniform: scalar loads straight from the OIHW tensor (k is contiguous
//    per c_out) put the 18 values of a channel pair in SGPRs, where they are the scalar operand
//    of v_add_f32 - no repacking pass, no VGPRs, no LDS.
//  * Implicit im2col: per channel a lane loads 3 rows x (8 + 2*dil) input values once (raw buffer
//    loads: wave-uniform descriptor + 32-bit lane offset + uniform channel offset) and reuses them
//    for 9 taps x 8 pixels x 4 channels.  Padding becomes NaN with one OR per loaded value;
//    v_max/v_min/v_max3/v_min3 return the non-NaN operand, so a padded tap never wins in either
//    branch and costs nothing in the inner loop.
//  * Inner blocks (tile_blocks_gfx950.h, hand-scheduled): one accumulator walks two channels
//    (18 taps) with 18 adds, v_max3/v_min3 chains, and 2 compares + 2 selects per branch that
//    record the winning CHANNEL.  After the K loop the epilogue re-evaluates the 9 taps of that
//    channel and takes the first that equals the extremum: exactly the lowest winning tap.
//  * Register-resident software pipeline: the six x rows of a channel pair occupy six register
//    slots.  Pixels are walked left to right, so the low columns of every slot die first; they
//    are re-loaded for the NEXT channel pair in the middle of the current one, the high columns
//    at its end, and each half is masked just before its first use.
#include <stdlib.h>

#include "tile_common.h"
// after tile_common.h: the blocks header relies on the HIP runtime declarations included there
#include <tile_blocks_gfx950.h>

namespace tconv {
namespace {

using namespace tile;

constexpr int TN = 4;  // output channels per lane

// 9 x values of pixel q for the 3x3 taps of one channel: rows[i][q + j*D]
template <int D, int XR>
__device__ __forceinline__ void taps_of(float (&out)[9], const float (&rows)[6][XR], int ch, int q) {
#pragma unroll
  for (int i = 0; i < 3; ++i)
#pragma unroll
    for (int j = 0; j < 3; ++j) out[i * 3 + j] = rows[ch * 3 + i][q + j * D];
}

template <int MODE, int D, typename TO>
__global__ __launch_bounds__(WAVES * 64, 2) void fwd_tiled3x3_s1_kernel(
    Params p, const float* __restrict__ x, const float* __restrict__ w_min,
    const float* __restrict__ w_max, const float* __restrict__ alpha,
    const float* __restrict__ beta, TO* __restrict__ y, TO* __restrict__ y_min,
    TO* __restrict__ y_max, int32_t* __restrict__ idx_min, int32_t* __restrict__ idx_max, int segs,
    int n_units, int n_groups, int dbg) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr int XR = 8 + 2 * D;  // input columns a lane touches per row
  constexpr int H1 = D + 4;      // columns [0, H1): left halo + first half of the core
  constexpr int P1 = D + 3;      // first-half columns are dead once pixel P1 is done
  constexpr int P2 = 4 - D;      // second-half columns are first read by pixel P2

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
  const int first_q = ow_nom - ow0;

  // ---- channel-independent addressing and padding masks
  const int iw0 = ow0 - p.pw;  // input column of register column 0
  const size_t HW = (size_t)p.H * p.W;
  const rsrc_t xres = make_rsrc(x, (unsigned)((size_t)p.N * p.C_in * HW * sizeof(float)));
  unsigned roff[3];  // byte offset of the first core column (iw0 + D >= 0) of each (clamped) row
  unsigned mrow[3];  // all-ones where the row is padding
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int ih = oh - p.ph + i * D;
    mrow[i] = (ih >= 0 && ih < p.H) ? 0u : 0xffffffffu;
    const int ihc = min(max(ih, 0), p.H - 1);
    roff[i] = (unsigned)(((size_t)n * p.C_in * HW + (size_t)ihc * p.W + (size_t)(iw0 + D)) * sizeof(float));
  }
  int hoff[2 * D];         // clamped byte offsets of the halo columns relative to roff
  unsigned mhalo[2 * D];   // all-ones where the halo column is padding
#pragma unroll
  for (int h = 0; h < 2 * D; ++h) {
    const int o = (h < D) ? h : h + 8;
    const int iw = iw0 + o;
    mhalo[h] = (iw >= 0 && iw < p.W) ? 0u : 0xffffffffu;
    hoff[h] = (min(max(iw, 0), p.W - 1) - (iw0 + D)) * (int)sizeof(float);
  }

  // ---- kernel rows of this wave's output channels (wave-uniform)
  const float* wr_min[TN];
  const float* wr_max[TN];
#pragma unroll
  for (int c = 0; c < TN; ++c) {
    const int co = min(co0 + c, p.C_out - 1);
    wr_min[c] = DO_MIN ? w_min + (size_t)co * p.K : nullptr;
    wr_max[c] = DO_MAX ? w_max + (size_t)co * p.K : nullptr;
  }

  float bmax[TN][PX], bmin[TN][PX];
  int imax[TN][PX], imin[TN][PX];
#pragma unroll
  for (int c = 0; c < TN; ++c)
#pragma unroll
    for (int q = 0; q < PX; ++q) {
      bmax[c][q] = -INFINITY; bmin[c][q] = INFINITY;
      imax[c][q] = 0; imin[c][q] = 0;
    }

  // ---- main loop over channel pairs (cA = 2*du, cB = 2*du + 1; an odd C_in gets a virtual last
  // channel whose x is all NaN)
  const int ndu = (dbg & 2) ? 0 : (p.C_in + 1) >> 1;
  float xs[6][XR];  // slot = 3*(channel parity) + kernel row

  auto chan_soff = [&](int c) -> unsigned {  // wave-uniform byte offset of channel c (clamped)
    return (unsigned)((size_t)min(c, p.C_in - 1) * HW * sizeof(float));
  };
  auto issue_first = [&](int du) {  // left halo + first 4 core columns of all six rows
#pragma unroll
    for (int sl = 0; sl < 6; ++sl) {
      const unsigned soff = chan_soff(2 * du + sl / 3);
      const unsigned ro = roff[sl % 3];
      load_run<4, float>(&xs[sl][D], xres, ro, soff);
#pragma unroll
      for (int h = 0; h < D; ++h) xs[sl][h] = load_one<float>(xres, ro + (unsigned)hoff[h], soff);
    }
  };
  auto issue_second = [&](int du) {  // last 4 core columns + right halo
#pragma unroll
    for (int sl = 0; sl < 6; ++sl) {
      const unsigned soff = chan_soff(2 * du + sl / 3);
      const unsigned ro = roff[sl % 3];
      load_run<4, float>(&xs[sl][D + 4], xres, ro + 16u, soff);
#pragma unroll
      for (int h = 0; h < D; ++h) xs[sl][D + 8 + h] = load_one<float>(xres, ro + (unsigned)hoff[D + h], soff);
    }
  };
  auto mask_cols = [&](int lo, int hi, unsigned mB) {  // padding -> NaN for columns [lo, hi)
#pragma unroll
    for (int sl = 0; sl < 6; ++sl) {
      const unsigned mr = mrow[sl % 3] | (sl >= 3 ? mB : 0u);
#pragma unroll
      for (int o = 0; o < XR; ++o) {
        if (o < lo || o >= hi) continue;
        unsigned m = mr;
        if (o < D) m |= mhalo[o];
        if (o >= D + 8) m |= mhalo[o - 8];
        xs[sl][o] = nan_or(xs[sl][o], m);
      }
    }
  };
  // 18 kernel values (channels cA, cB) of output channel slot c; the offsets are laundered so that
  // every block re-loads them (SGPRs are too few to keep all four channels' values live)
  auto load_w = [&](float (&wv)[18], const float* row, int cA, int cB) {
    const float* pa = row + launder_uniform(cA * 9);
    const float* pb = row + launder_uniform(cB * 9);
#pragma unroll
    for (int t = 0; t < 9; ++t) { wv[t] = pa[t]; wv[9 + t] = pb[t]; }
  };

  if (ndu > 0) {
    issue_first(0);
    issue_second(0);
  }
  for (int du = 0; du < ndu; ++du) {
    const int dn = min(du + 1, ndu - 1);  // past the end: re-load the last pair (unused, in bounds)
    const int cA = 2 * du, cBv = 2 * du + 1;
    const int cB = min(cBv, p.C_in - 1);
    const unsigned mB = (cBv < p.C_in) ? 0u : 0xffffffffu;
    const int tA = cA, tB = cBv;
    mask_cols(0, H1, mB);
    if (MODE == TCONV_COMPOUND) {
      float wc[18], wn[18];
      load_w(wc, wr_max[0], cA, cB);
#pragma unroll
      for (int q = 0; q < PX; ++q) {
        if (q == P2) mask_cols(H1, XR, mB);
        float xA[9], xB[9];
        taps_of<D, XR>(xA, xs, 0, q);
        taps_of<D, XR>(xB, xs, 1, q);
#pragma unroll
        for (int c = 0; c < TN; ++c) {
          load_w(wn, wr_max[(c + 1) % TN], cA, cB);
          float wA[9], wB[9];
#pragma unroll
          for (int t = 0; t < 9; ++t) { wA[t] = wc[t]; wB[t] = wc[9 + t]; }
          blk_both(bmax[c][q], bmin[c][q], imax[c][q], imin[c][q], xA, xB, wA, wB, tA, tB);
#pragma unroll
          for (int t = 0; t < 18; ++t) wc[t] = wn[t];
        }
        if (q == P1) issue_first(dn);
      }
    } else {
      // single-branch blocks cover two pixels; parallel mode runs a max block and a min block
      constexpr int NB = (MODE == TCONV_PARALLEL) ? 2 : 1;
      float wc[18], wn[18];
      load_w(wc, DO_MAX ? wr_max[0] : wr_min[0], cA, cB);
#pragma unroll
      for (int q = 0; q < PX; q += 2) {
        if (q == (P2 & ~1)) mask_cols(H1, XR, mB);
        float xA0[9], xB0[9], xA1[9], xB1[9];
        taps_of<D, XR>(xA0, xs, 0, q);
        taps_of<D, XR>(xB0, xs, 1, q);
        taps_of<D, XR>(xA1, xs, 0, q + 1);
        taps_of<D, XR>(xB1, xs, 1, q + 1);
#pragma unroll
        for (int c = 0; c < TN; ++c)
#pragma unroll
          for (int b = 0; b < NB; ++b) {
            const bool is_max = (MODE == TCONV_MAX) || (MODE == TCONV_PARALLEL && b == 0);
            // next block in program order: other branch of the same channel, or next channel
            const int cn = (b == NB - 1) ? (c + 1) % TN : c;
            const bool next_is_max = (MODE == TCONV_MAX) || (MODE == TCONV_PARALLEL && ((b + 1) % NB) == 0);
            load_w(wn, next_is_max ? wr_max[cn] : wr_min[cn], cA, cB);
            float wA[9], wB[9];
#pragma unroll
            for (int t = 0; t < 9; ++t) { wA[t] = wc[t]; wB[t] = wc[9 + t]; }
            if (is_max)
              blk_max2(bmax[c][q], imax[c][q], bmax[c][q + 1], imax[c][q + 1], xA0, xB0, xA1, xB1, wA, wB, tA, tB);
            else
              blk_min2(bmin[c][q], imin[c][q], bmin[c][q + 1], imin[c][q + 1], xA0, xB0, xA1, xB1, wA, wB, tA, tB);
#pragma unroll
            for (int t = 0; t < 18; ++t) wc[t] = wn[t];
          }
        if (q == (P1 & ~1)) issue_first(dn);
      }
    }
    issue_second(dn);
  }

  // ---- epilogue: exact tap of every extremum (first tap of the winning channel, in k order, whose
  // sum equals it), combine, store.  Each lane writes its 8 consecutive outputs with 16-byte stores.
  // The winning-channel ids are parked in LDS (a private 16-byte-per-lane slot per row: no barrier)
  // so that the gather batches below have registers to land in.
  constexpr int NBR = (DO_MIN && DO_MAX) ? 2 : 1;
  __shared__ int4 stash[WAVES][NBR][TN][2][64];
#pragma unroll
  for (int c = 0; c < TN; ++c)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if (DO_MIN) stash[wave][0][c][h][lane] = make_int4(imin[c][4 * h], imin[c][4 * h + 1], imin[c][4 * h + 2], imin[c][4 * h + 3]);
      if (DO_MAX) stash[wave][NBR - 1][c][h][lane] = make_int4(imax[c][4 * h], imax[c][4 * h + 1], imax[c][4 * h + 2], imax[c][4 * h + 3]);
    }
  auto unstash = [&](int br, int c, int (&ids)[PX]) {
    const int4 a0 = stash[wave][br][c][0][lane], a1 = stash[wave][br][c][1][lane];
    ids[0] = a0.x; ids[1] = a0.y; ids[2] = a0.z; ids[3] = a0.w;
    ids[4] = a1.x; ids[5] = a1.y; ids[6] = a1.z; ids[7] = a1.w;
  };
  if (!unit_ok) return;
  const size_t wbytes = (size_t)p.C_out * p.K * sizeof(float);
  const rsrc_t wres_min = make_rsrc(DO_MIN ? w_min : w_max, (unsigned)wbytes);
  const rsrc_t wres_max = make_rsrc(DO_MAX ? w_max : w_min, (unsigned)wbytes);
  const size_t xn_off = (size_t)n * p.C_in * HW;
  int ihc[3];
  bool rv[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int ih = oh - p.ph + i * D;
    rv[i] = (ih >= 0 && ih < p.H);
    ihc[i] = min(max(ih, 0), p.H - 1);
  }
  // Exact taps for RB pixels of one (channel, branch) row at a time: first ALL gathers of the batch
  // are issued (9 kernel values and a 3 x (2D+1) input patch per item), only then any is consumed,
  // so the batch pays one memory latency instead of one per item.  Border pixels load their patch
  // from a start clamped into the row and pick the taps with a per-lane shift.
  constexpr int L = 2 * D + 1;           // contiguous input columns spanned by the 3 taps of a row
  constexpr int RB = (D == 1) ? 4 : 2;   // items per batch (register budget)
  auto refine_batch = [&](const int (&cs_row)[PX], const float (&best_row)[PX], rsrc_t wres, int co, int q0,
                          int (&res)[PX]) {
    float wv[RB][9];
    float run[RB][3][L];
    int csv[RB], shv[RB];
#pragma unroll
    for (int u = 0; u < RB; ++u) {
      const int q = q0 + u;
      const int cs = min(cs_row[q], p.C_in - 1);  // a virtual channel never wins; keep the address in range
      csv[u] = cs;
      load_run<9, float>(wv[u], wres, (unsigned)(((size_t)co * p.K + (size_t)cs * 9) * sizeof(float)), 0u);
      const int iwq = ow0 + q - p.pw;
      const bool inner = (q >= D && q <= 7 - D);  // every tap column of this pixel lies inside the row
      const int start = inner ? iwq : min(max(iwq, 0), p.W - L);
      shv[u] = iwq - start;
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        const size_t rbase = xn_off + (size_t)cs * HW + (size_t)ihc[i] * p.W;
        load_run<L, float>(run[u][i], xres, (unsigned)((rbase + start) * sizeof(float)), 0u);
      }
    }
    __builtin_amdgcn_sched_barrier(0);  // keep the gathers of the batch ahead of every use
#pragma unroll
    for (int u = 0; u < RB; ++u) {
      const int q = q0 + u;
      const bool inner = (q >= D && q <= 7 - D);
      const int iwq = ow0 + q - p.pw;
      int r = csv[u] * 9;
#pragma unroll
      for (int i = 2; i >= 0; --i)
#pragma unroll
        for (int j = 2; j >= 0; --j) {
          float xv;
          bool ok = rv[i];
          if (inner) {
            xv = run[u][i][j * D];
          } else {
            const int col = j * D + shv[u];  // position of the tap inside the loaded run
            xv = run[u][i][0];
#pragma unroll
            for (int t = 1; t < L; ++t) xv = (col == t) ? run[u][i][t] : xv;
            const int iw = iwq + j * D;
            ok = ok && (iw >= 0 && iw < p.W);
          }
          const float sum = __fadd_rn(xv, wv[u][i * 3 + j]);
          r = (ok && sum == best_row[q]) ? csv[u] * 9 + i * 3 + j : r;
        }
      res[q] = (dbg & 1) ? csv[u] * 9 : r;
    }
    __builtin_amdgcn_sched_barrier(0);  // the next batch starts after this one has retired its registers
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
    int ridx[PX], cids[PX];
    float out[PX];
    if (DO_MIN) {
      unstash(0, c, cids);
#pragma unroll
      for (int q = 0; q < PX; q += RB) refine_batch(cids, bmin[c], wres_min, co, q, ridx);
      store_row(idx_min + ob, ridx, first_q);
      if (y_min) store_row(y_min + ob, bmin[c], first_q);
    }
    if (DO_MAX) {
      unstash(NBR - 1, c, cids);
#pragma unroll
      for (int q = 0; q < PX; q += RB) refine_batch(cids, bmax[c], wres_max, co, q, ridx);
      store_row(idx_max + ob, ridx, first_q);
      if (y_max) store_row(y_max + ob, bmax[c], first_q);
    }
#pragma unroll
    for (int q = 0; q < PX; ++q) {
      if (MODE == TCONV_MAX) out[q] = bmax[c][q];
      else if (MODE == TCONV_MIN) out[q] = bmin[c][q];
      else out[q] = combine(ca, bmin[c][q], cb, bmax[c][q]);
    }
    store_row(y + ob, out, first_q);
  }
}

// bf16 storage is widened to fp32 once, into the workspace, so that the main kernel always reads fp32
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

template <int MODE, int D, typename TO>
hipError_t launch_one(const Params& p, const float* x, const float* w_min, const float* w_max,
                      const FwdArgs& a, hipStream_t s) {
  const int segs = (p.Wo + PX - 1) / PX;
  const long long n_units = (long long)p.N * p.Ho * segs;
  const int n_groups = (p.C_out + TN - 1) / TN;
  const long long ublocks = (n_units + 63) / 64;
  const long long gblocks = (n_groups + WAVES - 1) / WAVES;
  const long long blocks = ublocks * gblocks;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  const char* e = getenv("TCONV_DEBUG_FLAGS");
  const int dbg = e ? atoi(e) : 0;
  hipLaunchKernelGGL((fwd_tiled3x3_s1_kernel<MODE, D, TO>), dim3((unsigned)blocks), dim3(WAVES * 64),
                     0, s, p, x, w_min, w_max, a.alpha, a.beta, (TO*)a.y, (TO*)a.y_min, (TO*)a.y_max,
                     a.idx_min, a.idx_max, segs, (int)n_units, n_groups, dbg);
  return hipGetLastError();
}

template <int MODE, typename TO>
hipError_t launch_dil(const Params& p, const float* x, const float* w_min, const float* w_max,
                      const FwdArgs& a, hipStream_t s) {
  return p.dh == 1 ? launch_one<MODE, 1, TO>(p, x, w_min, w_max, a, s)
                   : launch_one<MODE, 2, TO>(p, x, w_min, w_max, a, s);
}

template <typename TO>
hipError_t launch_mode(const Params& p, const float* x, const float* w_min, const float* w_max,
                       const FwdArgs& a, hipStream_t s) {
  switch (p.mode) {
    case TCONV_MAX: return launch_dil<TCONV_MAX, TO>(p, x, w_min, w_max, a, s);
    case TCONV_MIN: return launch_dil<TCONV_MIN, TO>(p, x, w_min, w_max, a, s);
    case TCONV_COMPOUND: return launch_dil<TCONV_COMPOUND, TO>(p, x, w_min, w_max, a, s);
    default: return launch_dil<TCONV_PARALLEL, TO>(p, x, w_min, w_max, a, s);
  }
}

bool stride1_supported(const Params& p) {
  if (p.KH != 3 || p.KW != 3) return false;
  if (p.sh != 1 || p.sw != 1 || p.dh != p.dw || (p.dh != 1 && p.dh != 2)) return false;
  if (p.pw > p.dw) return false;  // the 8 core columns of every lane must lie inside the row
  if (p.Wo < PX) return false;    // at least one full 8-pixel segment per output row
  // lanes address x and the kernels (as fp32) with 32-bit byte offsets
  if ((size_t)p.N * p.C_in * p.H * p.W * 4 >= 0xfffff000ull) return false;
  if ((size_t)p.C_out * p.K * 4 >= 0xfffff000ull) return false;
  return true;
}

}  // namespace

bool forward_tiled3x3_supported(const Params& p, int dtype) {
  return stride1_supported(p) || forward_tiled_strided_supported(p, dtype);
}

// Workspace of the tiled path: only bf16 storage with the stride-1 kernel needs one (fp32 copies
// of x and of the kernel tensors).
size_t forward_tiled3x3_workspace(const Params& p, int dtype) {
  if (dtype != TCONV_BF16 || !stride1_supported(p)) return 0;
  const size_t nx = (size_t)p.N * p.C_in * p.H * p.W, nw = (size_t)p.C_out * p.K;
  return align256(nx * 4) + align256(nw * 4) * (p.mode == TCONV_PARALLEL ? 2 : 1);
}

hipError_t launch_forward_tiled3x3(const Params& p, int dtype, const FwdArgs& a, void* workspace,
                                   hipStream_t s) {
  if (!stride1_supported(p)) return launch_forward_tiled_strided(p, dtype, a, s);
  if (dtype != TCONV_BF16)
    return launch_mode<float>(p, (const float*)a.x, (const float*)a.w_min, (const float*)a.w_max, a, s);
  const size_t nx = (size_t)p.N * p.C_in * p.H * p.W, nw = (size_t)p.C_out * p.K;
  float* xf = (float*)workspace;
  float* wa = (float*)((char*)workspace + align256(nx * 4));
  float* wb = (float*)((char*)wa + align256(nw * 4));
  widen(a.x, xf, nx, s);
  const float* wmin_f = nullptr;
  const float* wmax_f = nullptr;
  if (p.mode == TCONV_PARALLEL) {
    widen(a.w_min, wa, nw, s);
    widen(a.w_max, wb, nw, s);
    wmin_f = wa; wmax_f = wb;
  } else {
    widen(p.mode == TCONV_MIN ? a.w_min : a.w_max, wa, nw, s);
    wmin_f = wmax_f = wa;
  }
  return launch_mode<bf16_t>(p, xf, wmin_f, wmax_f, a, s);
}

}  // namespace tconv
