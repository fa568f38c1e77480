// Tiled 3x3 forward, the form in which the four waves of a workgroup split the input channels of one group of four
// output channels (four times as many, a quarter as long workgroups).  Instantiations and their choice; the kernel is
// in fwd_tiled3x3_kernel.h.
#include "fwd_tiled3x3_kernel.h"

namespace tconv {
namespace {

template <int MODE, int S, int D, typename TO, bool XA>
hipError_t launch_ks(const Params& p, const void* x, const float* w_min, const float* w_max, const FwdArgs& a,
                     hipStream_t s) {
  return p.pad_zero ? launch_tn<MODE, S, D, 4, true, TO, XA, true>(p, x, w_min, w_max, a, s)
                    : launch_tn<MODE, S, D, 4, false, TO, XA, true>(p, x, w_min, w_max, a, s);
}

// xa: bf16 rows whose core columns start at even elements for every lane (stride 1), fp32 rows whose right halo
// column is inside the row for every lane (stride 2); the caller has checked
template <int MODE, typename TO>
hipError_t launch_ks_geo(const Params& p, bool xa, const void* x, const float* w_min, const float* w_max,
                         const FwdArgs& a, hipStream_t s) {
  if (p.sh == 2)
    return xa ? launch_ks<MODE, 2, 1, TO, true>(p, x, w_min, w_max, a, s)
              : launch_ks<MODE, 2, 1, TO, false>(p, x, w_min, w_max, a, s);
  if constexpr (sizeof(TO) == 2) {
    if (xa)
      return p.dh == 1 ? launch_ks<MODE, 1, 1, TO, true>(p, x, w_min, w_max, a, s)
                       : launch_ks<MODE, 1, 2, TO, true>(p, x, w_min, w_max, a, s);
  }
  return p.dh == 1 ? launch_ks<MODE, 1, 1, TO, false>(p, x, w_min, w_max, a, s)
                   : launch_ks<MODE, 1, 2, TO, false>(p, x, w_min, w_max, a, s);
}

template <typename TO>
hipError_t launch_ks_mode(const Params& p, bool xa, const void* x, const float* w_min, const float* w_max,
                          const FwdArgs& a, hipStream_t s) {
  switch (p.mode) {
    case TCONV_MAX: return launch_ks_geo<TCONV_MAX, TO>(p, xa, x, w_min, w_max, a, s);
    case TCONV_MIN: return launch_ks_geo<TCONV_MIN, TO>(p, xa, x, w_min, w_max, a, s);
    case TCONV_COMPOUND: return launch_ks_geo<TCONV_COMPOUND, TO>(p, xa, x, w_min, w_max, a, s);
    case TCONV_PARALLEL: return launch_ks_geo<TCONV_PARALLEL, TO>(p, xa, x, w_min, w_max, a, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

// Where it applies: fp32 and bf16 storage, modes max / min / compound / parallel, one channel pair per wave or more (chosen by
// itself from two pairs per wave), more than two output channels.  Where it pays: workgroups of the plain form all run equally long, so a grid of them occupies
// the chip in whole rounds of `resident` workgroups; the split form has four times as many, a quarter as long
// workgroups and costs a few per cent in the exchange and in set-up done four times.  It is chosen unless the plain
// grid fills its rounds to 95 % (measured, plain -> split, ms: 3.06 rounds 0.936 -> 0.849, 1.75 rounds 0.610 -> 0.547,
// 0.875 rounds 0.961 -> 0.853, a quarter round 0.111 -> 0.075; 2.0 rounds 0.439 -> 0.462 and 1.587 -> 1.630, 4.0 rounds
// 1.499 -> 1.494).  TCONV_FWD_KSPLIT=1 asks for it wherever it applies, 0 never (tuning and testing aid).
bool forward_tiled3x3_ks_wanted(const Params& p, long long plain_workgroups, long long resident) {
  if (p.mode > TCONV_PARALLEL || p.C_in < 2 * tile::WAVES || p.C_out <= 2) return false;
  if (const char* e = getenv("TCONV_FWD_KSPLIT")) return atoi(e) == 1;
  if (p.C_in < 4 * tile::WAVES) return false;
  const long long rounds = (plain_workgroups + resident - 1) / resident;
  return plain_workgroups * 100 < rounds * resident * 95;
}

hipError_t launch_forward_tiled3x3_ks(const Params& p, bool bf16, bool xa, const void* x, const float* w_min,
                                      const float* w_max, const FwdArgs& a, hipStream_t s) {
  return bf16 ? launch_ks_mode<bf16_t>(p, xa, x, w_min, w_max, a, s)
              : launch_ks_mode<float>(p, xa, x, w_min, w_max, a, s);
}

}  // namespace tconv
