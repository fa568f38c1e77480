// Tiled forward for 3x3 tropical convolutions (paper Sec. 3.1 layers (iii)-(vi), Sec. 3.3 compound and parallel):
// which layers it takes, its workspace, and the fp32-storage instantiations of the plain form.  The kernel is in
// fwd_tiled3x3_kernel.h, the choice of its form in fwd_tiled3x3_launch.h.
#include "fwd_tiled3x3_launch.h"

namespace tconv {
namespace {

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

}  // namespace

// 3x3 kernels with equal stride and dilation on both axes, (stride, dilation) in {(1,1), (1,2), (2,1)},
// horizontal padding at most the dilation (so that the core columns of every lane lie inside the row),
// at least one full pixel segment per output row, tensors addressable with 32-bit byte offsets.
bool forward_tiled3x3_supported(const Params& p, int dtype) {
  if (dtype == TCONV_F16) return false;  // binary16 arithmetic has kernels of its own
  if (p.KH != 3 || p.KW != 3) return false;
  if (p.sh != p.sw || p.dh != p.dw) return false;
  const bool geo = (p.sh == 1 && (p.dh == 1 || p.dh == 2)) || (p.sh == 2 && p.dh == 1);
  if (!geo) return false;
  if (p.pw > p.dw) return false;
  if (p.Wo < (p.sh == 1 ? 8 : 4)) return false;
  if (p.W < 2 * p.dw + 1) return false;  // the epilogue loads 2*dil + 1 consecutive columns of a row
  if (p.C_in > 65535) return false;      // winning channels are parked as 16-bit values
  if ((size_t)p.N * p.C_in * p.H * p.W * (dtype == TCONV_BF16 ? 2 : 4) >= 0xfffff000ull) return false;
  if ((size_t)p.C_out * p.K * 4 >= 0xfffff000ull) return false;
  if ((size_t)p.N * p.C_out * p.Ho * p.Wo * 4 >= 0xfffff000ull) return false;  // a lane's output offset is 32 bits
  return true;
}

// Workspace of the tiled path: only bf16 storage needs one, for fp32 copies of the kernel tensors (scalar loads take
// whole dwords at dword-aligned addresses; the tensors are small).  x is read as bf16 by the kernel itself.
size_t forward_tiled3x3_workspace(const Params& p, int dtype) {
  if (dtype != TCONV_BF16) return 0;
  const size_t nw = (size_t)p.C_out * p.K;
  return align256(nw * 4) * (p.mode == TCONV_PARALLEL ? 2 : 1);
}

// whether launch_forward_tiled3x3 will run the form that splits the input channels over the waves (host only)
bool forward_tiled3x3_splits(const Params& p, int dtype) {
  if (dtype != TCONV_F32 && dtype != TCONV_BF16) return false;
  const int px = p.sh == 1 ? 8 : 4;
  const long long n_units = (long long)p.N * p.Ho * ((p.Wo + px - 1) / px);
  const long long blocks4 = ((n_units + 63) / 64) * ((((long long)p.C_out + 3) / 4 + WAVES - 1) / WAVES);
  return forward_tiled3x3_ks_wanted(p, blocks4, resident_workgroups());
}

hipError_t launch_forward_tiled3x3(const Params& p, int dtype, const FwdArgs& a, void* workspace,
                                   hipStream_t s) {
  if (dtype == TCONV_BF16) return launch_forward_tiled3x3_bf16(p, a, workspace, s);
  return launch_mode<float>(p, a.x, (const float*)a.w_min, (const float*)a.w_max, a, s);
}

}  // namespace tconv
