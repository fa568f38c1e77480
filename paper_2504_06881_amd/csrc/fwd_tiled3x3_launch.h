// Host-side choice of the tiled 3x3 forward kernel's form (output channels per lane, bf16 row loads, the forms in
// code objects of their own) as templates over the storage type: fp32 storage and bf16 storage instantiate them in
// separate translation units.
#pragma once
#include "fwd_tiled3x3_kernel.h"

namespace tconv {
namespace {

// workgroups the chip holds at once (two per compute unit); the unit count is asked for once per process
// (every device of a node is the same part)
inline long long resident_workgroups() {
  static const int cus = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
      n = 256;
    return n;
  }();
  return 2LL * cus;
}

template <int MODE, int S, int D, typename TO>
hipError_t launch_one(const Params& p, const void* x, const float* w_min, const float* w_max,
                      const FwdArgs& a, hipStream_t s) {
  // 4 output channels per lane reuse every loaded input value twice as often as 2, but a layer whose
  // grid leaves half of the wave slots empty runs faster on twice as many, half as long waves
  // (measured: not so at stride 2, whose loads per arithmetic instruction are already twice as many,
  // unless three quarters are empty)
  constexpr int PX = (S == 1) ? 8 : 4;
  const long long n_units = (long long)p.N * p.Ho * ((p.Wo + PX - 1) / PX);
  const long long blocks4 = ((n_units + 63) / 64) * ((((long long)p.C_out + 3) / 4 + WAVES - 1) / WAVES);
  int tn = (blocks4 * (S == 1 ? 2 : 4) <= resident_workgroups() && p.C_out > 2) ? 2 : 4;
  if (const char* e = getenv("TCONV_FWD_TN")) {  // tuning aid
    if (atoi(e) == 2 || atoi(e) == 4) tn = atoi(e);
  }
  // bf16 rows whose core columns start at even elements for every lane: W even (rows, channels and images start
  // even), an even first output column of every segment (W_out even) and an even left margin D - pad_w
  // fp32 rows at stride 2 whose right halo column (register column 8 of the widest-placed segment, input column
  // 2 * (W_out - 4) - pad_w + 8) is inside the row: read in one run with the core columns
  // (bf16 rows at stride 2: both: the run of 8 then starts at an even element and is four dwords)
  const bool wide2 = S == 2 && 2 * p.Wo - p.pw <= p.W - 1 && !getenv("TCONV_FWD_NARROW2");
  const bool xa = (sizeof(TO) == 2 && S == 1 && p.W % 2 == 0 && p.Wo % 2 == 0 && (D - p.pw) % 2 == 0) ||
                  (sizeof(TO) == 4 && wide2) || (sizeof(TO) == 2 && wide2 && p.W % 2 == 0 && (D - p.pw) % 2 == 0);
  // the form that splits the input channels over the waves of a workgroup lives in a code object of its own
  if (forward_tiled3x3_ks_wanted(p, blocks4, resident_workgroups()))
    return launch_forward_tiled3x3_ks(p, sizeof(TO) == 2, xa, x, w_min, w_max, a, s);
  if constexpr (sizeof(TO) == 2) {
    if (xa) {
      if (p.pad_zero)
        return tn == 2 ? launch_tn<MODE, S, D, 2, true, TO, true>(p, x, w_min, w_max, a, s)
                       : launch_tn<MODE, S, D, 4, true, TO, true>(p, x, w_min, w_max, a, s);
      return tn == 2 ? launch_tn<MODE, S, D, 2, false, TO, true>(p, x, w_min, w_max, a, s)
                     : launch_tn<MODE, S, D, 4, false, TO, true>(p, x, w_min, w_max, a, s);
    }
  }
  if constexpr (sizeof(TO) == 4 && S == 2) {
    if (xa) {
      if (p.pad_zero)
        return tn == 2 ? launch_tn<MODE, S, D, 2, true, TO, true>(p, x, w_min, w_max, a, s)
                       : launch_tn<MODE, S, D, 4, true, TO, true>(p, x, w_min, w_max, a, s);
      return tn == 2 ? launch_tn<MODE, S, D, 2, false, TO, true>(p, x, w_min, w_max, a, s)
                     : launch_tn<MODE, S, D, 4, false, TO, true>(p, x, w_min, w_max, a, s);
    }
  }
  if (p.pad_zero)
    return tn == 2 ? launch_tn<MODE, S, D, 2, true, TO>(p, x, w_min, w_max, a, s)
                   : launch_tn<MODE, S, D, 4, true, TO>(p, x, w_min, w_max, a, s);
  return tn == 2 ? launch_tn<MODE, S, D, 2, false, TO>(p, x, w_min, w_max, a, s)
                 : launch_tn<MODE, S, D, 4, false, TO>(p, x, w_min, w_max, a, s);
}

template <int MODE, typename TO>
hipError_t launch_geo(const Params& p, const void* x, const float* w_min, const float* w_max,
                      const FwdArgs& a, hipStream_t s) {
  if (p.sh == 2) return launch_one<MODE, 2, 1, TO>(p, x, w_min, w_max, a, s);
  return p.dh == 1 ? launch_one<MODE, 1, 1, TO>(p, x, w_min, w_max, a, s)
                   : launch_one<MODE, 1, 2, TO>(p, x, w_min, w_max, a, s);
}

template <typename TO>
hipError_t launch_mode(const Params& p, const void* x, const float* w_min, const float* w_max,
                       const FwdArgs& a, hipStream_t s) {
  switch (p.mode) {
    case TCONV_MAX: return launch_geo<TCONV_MAX, TO>(p, x, w_min, w_max, a, s);
    case TCONV_MIN: return launch_geo<TCONV_MIN, TO>(p, x, w_min, w_max, a, s);
    case TCONV_COMPOUND: return launch_geo<TCONV_COMPOUND, TO>(p, x, w_min, w_max, a, s);
    case TCONV_PARALLEL: return launch_geo<TCONV_PARALLEL, TO>(p, x, w_min, w_max, a, s);
    case TCONV_MINPLUS_MAX: return launch_geo<TCONV_MINPLUS_MAX, TO>(p, x, w_min, w_max, a, s);
    default: return launch_geo<TCONV_MAXPLUS_MIN, TO>(p, x, w_min, w_max, a, s);
  }
}

}  // namespace
}  // namespace tconv
