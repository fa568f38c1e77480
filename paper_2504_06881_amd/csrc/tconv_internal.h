// Internal declarations shared by the HIP translation units of libtconv (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tconv.h"

namespace tconv {

// Launch-time view of a validated descriptor.
struct Params {
  int N, C_in, H, W;
  int C_out, KH, KW;
  int sh, sw, ph, pw, dh, dw;
  int Ho, Wo;
  int K;     // C_in*KH*KW
  int mode;  // enum tconv_mode
  int pad_zero;  // 0: out-of-image taps never win (semiring identity); 1: they are candidates with input value +0
};

// Which kernel / index / output side a mode uses.  The mixed layers are single-branch: (iii) MinPlus-Max
// lives on the min side (its operator is min-plus), (vi) MaxPlus-Min on the max side.
__host__ __device__ constexpr bool mode_has_min(int m) { return m != TCONV_MAX && m != TCONV_MAXPLUS_MIN; }
__host__ __device__ constexpr bool mode_has_max(int m) { return m != TCONV_MIN && m != TCONV_MINPLUS_MAX; }
// The backward pass of a mixed layer is the one of the plain single-branch layer on the same side: the
// whole gradient of an output goes through its one winning tap, whatever reduction picked it.
constexpr int backward_mode(int m) {
  return m == TCONV_MINPLUS_MAX ? TCONV_MIN : (m == TCONV_MAXPLUS_MIN ? TCONV_MAX : m);
}

// Launch-time view of a validated three-dimensional descriptor.
struct Params3 {
  int N, C_in, D, H, W;
  int C_out, KD, KH, KW;
  int sd, sh, sw, pd, ph, pw, dd, dh, dw;
  int Do, Ho, Wo;
  int K;     // C_in*KD*KH*KW
  int mode;  // enum tconv_mode
};

struct FwdArgs {
  const void* x;
  const void* w_min;  // kernel of the min-plus branch (compound: the shared kernel)
  const void* w_max;  // kernel of the max-plus branch (compound: the shared kernel)
  const float* alpha;
  const float* beta;
  void* y;
  void* y_min;
  void* y_max;
  int32_t* idx_min;
  int32_t* idx_max;
  // epilogue on the combined output y (each NULL = step left out), applied in this order:
  const float* bias;      // [C_out]: y + bias
  const float* scale;     // [C_out]: y * scale + shift (shift NULL = 0), a batch norm folded for inference
  const float* shift;
  const void* residual;   // [N, C_out, H_out, W_out] in the storage dtype: y + residual
};

struct BwdArgs {
  const float* gy;
  const float* alpha;
  const float* beta;
  const int32_t* idx_min;
  const int32_t* idx_max;
};

// Sum-channel layers (fp32): inputs of both passes, and the gradient request of the backward pass.
struct SumArgs {
  const float* x;
  const float* w_min;  // W1, kernel of the min-plus branch (compound: the shared kernel)
  const float* w_max;  // W2, kernel of the max-plus branch (compound: the shared kernel)
  const float* alpha;  // [C_in, C_out] or NULL
  const float* beta;
  float* y;            // forward only
};

struct SumGrads {
  const float* gy;
  float* grad_x;
  float* grad_w_min;
  float* grad_w_max;
  float* grad_alpha;
  float* grad_beta;
};

// Depthwise layers (fp32): C_out = mult * C_in, output channel co reads input channel co / mult; kernels
// [C_out, 1, KH, KW], alpha / beta [C_out]; idx: one byte per output, low nibble = winning tap of the min-plus
// branch, high nibble = of the max-plus branch.
struct DwArgs {
  const float* x;
  const float* w_min;
  const float* w_max;
  const float* alpha;
  const float* beta;
  float* y;      // forward only
  uint8_t* idx;  // written by forward (optional there), read by backward
};

struct DwGrads {
  const float* gy;
  float* grad_x;
  float* grad_w_min;
  float* grad_w_max;
  float* grad_alpha;
  float* grad_beta;
};

// bf16 storage helpers: exact widening, round-to-nearest-even narrowing.
typedef unsigned short bf16_t;

__device__ __forceinline__ float ld_f32(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float ld_f32(const bf16_t* p, size_t i) {
  return __uint_as_float(((unsigned)p[i]) << 16);
}
__device__ __forceinline__ void st_f32(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st_f32(bf16_t* p, size_t i, float v) {
  unsigned u = __float_as_uint(v);
  if ((u & 0x7f800000u) != 0x7f800000u) u += 0x7fffu + ((u >> 16) & 1u);
  p[i] = (bf16_t)(u >> 16);
}

// binary16 storage: exact widening, round-to-nearest-even narrowing (v_cvt_f16_f32 under the default rounding mode).
typedef _Float16 f16_t;
__device__ __forceinline__ float ld_f32(const f16_t* p, size_t i) { return (float)p[i]; }
__device__ __forceinline__ void st_f32(f16_t* p, size_t i, float v) { p[i] = (f16_t)v; }

// One candidate: x + w rounded once, in the arithmetic type of the storage type - fp32 for fp32 and bf16 storage,
// binary16 for binary16 storage (both operands are exactly representable there; the sum is one v_add_f16).
template <typename T>
__device__ __forceinline__ float candidate(float x, float w) {
  if constexpr (sizeof(T) == 2 && !__is_same(T, bf16_t)) return (float)((f16_t)x + (f16_t)w);
  else return __fadd_rn(x, w);
}

// alpha*y_min + beta*y_max with each product and the sum rounded separately (no FMA).
__device__ __forceinline__ float combine(float a, float ymin, float b, float ymax) {
  return __fadd_rn(__fmul_rn(a, ymin), __fmul_rn(b, ymax));
}

// The epilogue of one output: bias, affine, residual, every operation rounded to fp32 on its own.
template <typename T>
__device__ __forceinline__ float apply_epilogue(float t, const FwdArgs& a, int co, size_t o) {
  if (a.bias) t = __fadd_rn(t, a.bias[co]);
  if (a.scale) t = __fadd_rn(__fmul_rn(t, a.scale[co]), a.shift ? a.shift[co] : 0.0f);
  if (a.residual) t = __fadd_rn(t, ld_f32((const T*)a.residual, o));
  return t;
}

// Kernel launchers (each returns hipGetLastError() after its launches).
hipError_t launch_forward_generic(const Params& p, int dtype, const FwdArgs& a, hipStream_t s);
bool forward_tiled3x3_supported(const Params& p, int dtype);
size_t forward_tiled3x3_workspace(const Params& p, int dtype);  // bytes of device scratch it needs
hipError_t launch_forward_tiled3x3(const Params& p, int dtype, const FwdArgs& a, void* workspace,
                                   hipStream_t s);
// its bf16-storage instantiations (a translation unit of their own); workspace as forward_tiled3x3_workspace says
hipError_t launch_forward_tiled3x3_bf16(const Params& p, const FwdArgs& a, void* workspace, hipStream_t s);
// the form of the tiled 3x3 kernel that splits the input channels over the waves of a workgroup (fp32 and bf16 storage,
// the four full-window modes; a code object of its own; xa: bf16 rows read as dword pairs).  plain_workgroups: the grid of the plain form with 4 output
// channels per lane, resident: the workgroups the chip holds at once
bool forward_tiled3x3_ks_wanted(const Params& p, long long plain_workgroups, long long resident);
bool forward_tiled3x3_splits(const Params& p, int dtype);  // the tiled path will take that form (host only)
hipError_t launch_forward_tiled3x3_ks(const Params& p, bool bf16, bool xa, const void* x, const float* w_min,
                                      const float* w_max, const FwdArgs& a, hipStream_t s);
// binary16 arithmetic (TCONV_F16) on the packed 16-bit vector instructions
bool forward_tiled3x3_f16_supported(const Params& p, int dtype);
size_t forward_tiled3x3_f16_workspace(const Params& p);
hipError_t launch_forward_tiled3x3_f16(const Params& p, const FwdArgs& a, void* workspace, hipStream_t s);
// windows other than 3x3 (KW <= 7), fp32: kernel rows walked with the input row segment in registers
bool forward_rowtile_supported(const Params& p, int dtype);
hipError_t launch_forward_rowtile(const Params& p, const FwdArgs& a, hipStream_t s);
bool forward_row_supported(const Params& p, int dtype);  // one-row inputs with a long window
hipError_t launch_forward_row(const Params& p, const FwdArgs& a, hipStream_t s);
hipError_t launch_backward_input(const Params& p, const BwdArgs& a, float* grad_x, hipStream_t s);
hipError_t launch_backward_bias(const Params& p, const float* gy, float* grad_bias, double* partial, hipStream_t s);
// every parameter gradient from one pass (fp32 branch outputs; partial: backward_params_workspace(p) bytes, not 0).
// x != NULL: the branch outputs are not read but formed again from the winners, fl(x[winner] + w[winner]) (fp32 x and
// kernels; y_min / y_max ignored).
size_t backward_params_workspace(const Params& p);
hipError_t launch_backward_params(const Params& p, const BwdArgs& a, const float* y_min, const float* y_max,
                                  const float* x, const float* w_min, const float* w_max, float* grad_w_min,
                                  float* grad_w_max, float* grad_alpha, float* grad_beta, float* grad_bias,
                                  double* partial, hipStream_t s);
// partial: device scratch of backward_weight_workspace(p) bytes for the deterministic two-stage form (fp64 partial
// histograms per batch slice, added in a fixed order, one rounding), or NULL: fp32 atomics into zero-filled tensors
size_t backward_weight_workspace(const Params& p);
hipError_t launch_backward_weight(const Params& p, const BwdArgs& a, float* grad_w_min,
                                  float* grad_w_max, double* partial, hipStream_t s);
// the same with the library's own fixed scratch array (no workspace argument, nothing allocated);
// hipErrorOutOfMemory when the layer needs more than backward_weight_static_limit() bytes
size_t backward_weight_static_limit();
hipError_t launch_backward_weight_static(const Params& p, const BwdArgs& a, float* grad_w_min, float* grad_w_max,
                                         hipStream_t s);
size_t backward_alpha_beta_workspace(const Params& p);
hipError_t launch_backward_alpha_beta(const Params& p, int dtype, const float* gy, const void* y_min,
                                      const void* y_max, float* grad_alpha, float* grad_beta, double* partial,
                                      hipStream_t s);

// Sum-channel layers.  dtype TCONV_BF16: x, the kernels and y are bf16 behind the float pointers of SumArgs, workspace
// holds sum_workspace(p, dtype, backward) bytes; forward then only where sum_forward_supported says so.
size_t sum_workspace(const Params& p, int dtype, bool backward);
bool sum_forward_supported(const Params& p, int dtype);
hipError_t launch_sum_forward(const Params& p, int dtype, const SumArgs& a, void* workspace, hipStream_t s);
hipError_t launch_sum_backward(const Params& p, int dtype, const SumArgs& a, const SumGrads& g, void* workspace,
                               hipStream_t s);
const char* sum_forward_kernel_name(const Params& p);

hipError_t launch_forward_3d(const Params3& p, const FwdArgs& a, hipStream_t s);
hipError_t launch_backward_input_3d(const Params3& p, const BwdArgs& a, float* grad_x, hipStream_t s);
const char* forward_3d_kernel_name(const Params3& p);

hipError_t launch_depthwise_forward(const Params& p, const DwArgs& a, hipStream_t s);
hipError_t launch_depthwise_backward(const Params& p, const DwArgs& a, const DwGrads& g, hipStream_t s);
const char* depthwise_forward_kernel_name(const Params& p);

}  // namespace tconv
