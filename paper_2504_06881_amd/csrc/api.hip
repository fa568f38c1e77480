// C-ABI entry points of libtconv: argument validation and kernel selection only.
// Every step of the hot path runs in the HIP kernels of this library; there is
// no host-side or CPU implementation behind these calls.
#include <stdlib.h>
#include <string.h>

#include "tconv_internal.h"

using namespace tconv;

namespace {

// True if some window of one axis has no tap inside the input.  With pad <= dil * (k - 1) and a non-empty output
// every window's span overlaps the input, and where the input is at least as long as the dilation one of the
// window's taps then lies inside it.  A shorter input can be straddled: at most one tap of a window can be inside,
// the one at the window start's residue modulo the dilation, and the residues repeat with period dil / gcd(stride, dil).
bool axis_has_empty_window(long long in, long long k, long long st, long long pd, long long dl, long long out) {
  if (k == 1 || in >= dl) return false;
  long long a = st, b = dl;
  while (b) { const long long t = a % b; a = b; b = t; }
  const long long period = dl / a, n = out < period ? out : period;
  for (long long o = 0; o < n; ++o)
    if (((o * st - pd) % dl + dl) % dl >= in) return true;
  return false;
}

// Validates the descriptor and fills the launch-time view.
int make_params(const tconv_desc* d, Params* p) {
  if (!d) return TCONV_E_INVAL;
  if (d->N < 1 || d->C_in < 1 || d->H < 1 || d->W < 1 || d->C_out < 1 || d->KH < 1 || d->KW < 1)
    return TCONV_E_INVAL;
  if (d->stride_h < 1 || d->stride_w < 1 || d->dil_h < 1 || d->dil_w < 1 || d->pad_h < 0 ||
      d->pad_w < 0)
    return TCONV_E_INVAL;
  if (d->mode < TCONV_MAX || d->mode > TCONV_MAXPLUS_MIN) return TCONV_E_INVAL;
  if (d->dtype != TCONV_F32 && d->dtype != TCONV_BF16 && d->dtype != TCONV_F16) return TCONV_E_INVAL;
  if (d->pad_mode != TCONV_PAD_IDENTITY && d->pad_mode != TCONV_PAD_ZERO) return TCONV_E_INVAL;
  const long long eh = (long long)d->dil_h * (d->KH - 1), ew = (long long)d->dil_w * (d->KW - 1);
  // a window must never lie wholly in the padding (kept for zero padding too: one rule for both modes)
  if (d->pad_h > eh || d->pad_w > ew) return TCONV_E_SHAPE;
  const long long nh = (long long)d->H + 2LL * d->pad_h - eh - 1;
  const long long nw = (long long)d->W + 2LL * d->pad_w - ew - 1;
  if (nh < 0 || nw < 0) return TCONV_E_SHAPE;
  const long long Ho = nh / d->stride_h + 1, Wo = nw / d->stride_w + 1;
  const long long K = (long long)d->C_in * d->KH * d->KW;
  const long long lim = 0x7fffffffLL;
  if (K > lim || (long long)d->N * d->C_in * d->H * d->W > lim ||
      (long long)d->N * d->C_out * Ho * Wo > lim || (long long)d->C_out * K > lim)
    return TCONV_E_SHAPE;
  // ... nor may its taps straddle an input shorter than the dilation
  if (axis_has_empty_window(d->H, d->KH, d->stride_h, d->pad_h, d->dil_h, Ho) ||
      axis_has_empty_window(d->W, d->KW, d->stride_w, d->pad_w, d->dil_w, Wo))
    return TCONV_E_SHAPE;
  p->N = d->N; p->C_in = d->C_in; p->H = d->H; p->W = d->W;
  p->C_out = d->C_out; p->KH = d->KH; p->KW = d->KW;
  p->sh = d->stride_h; p->sw = d->stride_w; p->ph = d->pad_h; p->pw = d->pad_w;
  p->dh = d->dil_h; p->dw = d->dil_w;
  p->Ho = (int)Ho; p->Wo = (int)Wo; p->K = (int)K; p->mode = d->mode;
  p->pad_zero = d->pad_mode == TCONV_PAD_ZERO ? 1 : 0;
  return TCONV_OK;
}

// TCONV_FORWARD_KERNEL=generic forces the generic kernel (tuning / testing aid).
bool generic_forced() {
  const char* e = getenv("TCONV_FORWARD_KERNEL");
  return e && strcmp(e, "generic") == 0;
}

// Optional scratch of the parameter gradients: NULL selects the atomic form, a buffer must hold `need` bytes and be
// 8-byte aligned.  Returns false on a buffer that is too small or misaligned.
bool take_partial(void* workspace, size_t workspace_bytes, size_t need, double** partial) {
  *partial = nullptr;
  if (!workspace || need == 0) return true;
  if (workspace_bytes < need || ((uintptr_t)workspace & 7u)) return false;
  *partial = (double*)workspace;
  return true;
}

// A launcher reports hipGetLastError() after its launches.  That status is sticky per host thread: drop whatever an
// earlier, unrelated call of the caller left behind, so that TCONV_E_LAUNCH always speaks of this call's launches.
void own_status() { (void)hipGetLastError(); }

bool use_tiled(const Params& p, int dtype) { return forward_tiled3x3_supported(p, dtype) && !generic_forced(); }

bool use_tiled16(const Params& p, int dtype) { return forward_tiled3x3_f16_supported(p, dtype) && !generic_forced(); }

bool use_row(const Params& p, int dtype) {
  return !use_tiled(p, dtype) && forward_row_supported(p, dtype) && !generic_forced();
}

bool use_rowtile(const Params& p, int dtype) {
  return !use_tiled(p, dtype) && !use_tiled16(p, dtype) && !use_row(p, dtype) && forward_rowtile_supported(p, dtype) &&
         !generic_forced();
}

}  // namespace

extern "C" {

int tconv_out_shape(const tconv_desc* desc, int32_t* H_out, int32_t* W_out) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!H_out || !W_out) return TCONV_E_INVAL;
  *H_out = p.Ho;
  *W_out = p.Wo;
  return TCONV_OK;
}

namespace {
// tconv_backward_params: the one-pass form wants fp32 branch outputs and a window whose histogram fits LDS; otherwise
// the separate kernels run, the kernel gradient's scratch first and the two-sums-per-slice scratch behind it
bool params_one_pass(const Params& p, int dtype) { return dtype == TCONV_F32 && backward_params_workspace(p) != 0; }
size_t params_split_offset(const Params& p) { return (backward_weight_workspace(p) + 255) & ~(size_t)255; }
size_t params_workspace(const Params& p, int dtype) {
  if (params_one_pass(p, dtype)) return backward_params_workspace(p);
  return params_split_offset(p) + backward_alpha_beta_workspace(p);
}
}  // namespace

int tconv_workspace_bytes(const tconv_desc* desc, int32_t op, size_t* bytes) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!bytes || op < TCONV_OP_FORWARD || op > TCONV_OP_BACKWARD_PARAMS) return TCONV_E_INVAL;
  *bytes = 0;
  if (op == TCONV_OP_BACKWARD_BIAS) *bytes = backward_alpha_beta_workspace(p);  // the same slices, two sums each
  // forward: only the tiled kernel with bf16 storage stages anything (fp32 copies of x and the kernels)
  if (op == TCONV_OP_FORWARD && use_tiled(p, desc->dtype)) *bytes = forward_tiled3x3_workspace(p, desc->dtype);
  // the binary16 tiled kernel: the kernel tensors re-laid in output-channel pairs
  if (op == TCONV_OP_FORWARD && use_tiled16(p, desc->dtype)) *bytes = forward_tiled3x3_f16_workspace(p);
  // the deterministic forms of the parameter gradients: fp64 partial sums per batch slice
  if (op == TCONV_OP_BACKWARD_WEIGHT || op == TCONV_OP_BACKWARD) {
    p.mode = backward_mode(p.mode);
    *bytes = backward_weight_workspace(p);
  }
  if (op == TCONV_OP_BACKWARD_ALPHA_BETA && (p.mode == TCONV_COMPOUND || p.mode == TCONV_PARALLEL))
    *bytes = backward_alpha_beta_workspace(p);
  if (op == TCONV_OP_BACKWARD_PARAMS) {
    p.mode = backward_mode(p.mode);
    *bytes = params_workspace(p, desc->dtype);
  }
  return TCONV_OK;
}

int tconv_forward(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                  const float* alpha, const float* beta, void* y, void* y_min, void* y_max,
                  int32_t* idx_min, int32_t* idx_max, void* workspace, size_t workspace_bytes,
                  void* hip_stream) {
  return tconv_forward_fused(desc, x, w_min, w_max, alpha, beta, nullptr, y, y_min, y_max, idx_min, idx_max, workspace,
                             workspace_bytes, hip_stream);
}

int tconv_forward_fused(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                        const float* alpha, const float* beta, const tconv_epilogue* epilogue, void* y, void* y_min,
                        void* y_max, int32_t* idx_min, int32_t* idx_max, void* workspace, size_t workspace_bytes,
                        void* hip_stream) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!x || !y) return TCONV_E_INVAL;
  FwdArgs a = {x, w_min, w_max, alpha, beta, y, y_min, y_max, idx_min, idx_max};
  if (p.pad_zero && p.mode > TCONV_PARALLEL) return TCONV_E_UNSUPPORTED;  // the mixed layers keep identity padding
  if (desc->dtype == TCONV_F16 && p.mode > TCONV_PARALLEL) return TCONV_E_UNSUPPORTED;  // and fp32 / bf16 storage
  if (epilogue && desc->dtype == TCONV_F16 &&
      (epilogue->bias || epilogue->scale || epilogue->shift || epilogue->residual))
    return TCONV_E_UNSUPPORTED;  // the binary16 contract has no epilogue
  if (epilogue) {
    if (epilogue->shift && !epilogue->scale) return TCONV_E_INVAL;
    a.bias = epilogue->bias; a.scale = epilogue->scale; a.shift = epilogue->shift; a.residual = epilogue->residual;
  }
  if (p.mode == TCONV_COMPOUND) a.w_min = a.w_max = (w_min ? w_min : w_max);
  const bool do_min = mode_has_min(p.mode), do_max = mode_has_max(p.mode);
  if (do_min && (!a.w_min || !idx_min)) return TCONV_E_INVAL;
  if (do_max && (!a.w_max || !idx_max)) return TCONV_E_INVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  hipError_t e;
  // the tiled kernel reads bf16 rows as whole dwords: x dword-aligned, and an even element count so that no dword
  // reaches past the tensor; anything else goes to the kernels that read value by value
  const bool bf16_dwords = desc->dtype != TCONV_BF16 ||
                           (((uintptr_t)x & 3u) == 0 && (((size_t)p.N * p.C_in * p.H * p.W) & 1u) == 0);
  if (use_tiled(p, desc->dtype) && bf16_dwords) {
    const size_t need = forward_tiled3x3_workspace(p, desc->dtype);
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u)))
      return TCONV_E_WORKSPACE;
    own_status();
    e = launch_forward_tiled3x3(p, desc->dtype, a, workspace, s);
  } else if (use_tiled16(p, desc->dtype)) {
    const size_t need = forward_tiled3x3_f16_workspace(p);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u)) return TCONV_E_WORKSPACE;
    own_status();
    e = launch_forward_tiled3x3_f16(p, a, workspace, s);
  } else if (use_row(p, desc->dtype) && !a.bias && !a.scale && !a.residual) {  // the row kernel has no epilogue
    own_status();
    e = launch_forward_row(p, a, s);
  } else if (use_rowtile(p, desc->dtype) && !a.bias && !a.scale && !a.residual) {  // nor has the row-tiled kernel
    own_status();
    e = launch_forward_rowtile(p, a, s);
  } else {
    own_status();
    e = launch_forward_generic(p, desc->dtype, a, s);
  }
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv_backward_input(const tconv_desc* desc, const float* gy, const float* alpha,
                         const float* beta, const int32_t* idx_min, const int32_t* idx_max,
                         float* grad_x, void* workspace, size_t workspace_bytes, void* hip_stream) {
  (void)workspace; (void)workspace_bytes;
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!gy || !grad_x) return TCONV_E_INVAL;
  p.mode = backward_mode(p.mode);
  if (p.mode != TCONV_MAX && !idx_min) return TCONV_E_INVAL;
  if (p.mode != TCONV_MIN && !idx_max) return TCONV_E_INVAL;
  BwdArgs a = {gy, alpha, beta, idx_min, idx_max};
  own_status();
  const hipError_t e = launch_backward_input(p, a, grad_x, (hipStream_t)hip_stream);
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv_backward_weight(const tconv_desc* desc, const float* gy, const float* alpha,
                          const float* beta, const int32_t* idx_min, const int32_t* idx_max,
                          float* grad_w_min, float* grad_w_max, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!gy) return TCONV_E_INVAL;
  p.mode = backward_mode(p.mode);
  if (p.mode != TCONV_MAX && !idx_min) return TCONV_E_INVAL;
  if (p.mode != TCONV_MIN && !idx_max) return TCONV_E_INVAL;
  switch (p.mode) {
    case TCONV_MAX: if (!grad_w_max) return TCONV_E_INVAL; break;
    case TCONV_MIN: if (!grad_w_min) return TCONV_E_INVAL; break;
    case TCONV_COMPOUND: if (!grad_w_min && !grad_w_max) return TCONV_E_INVAL; break;
    default: if (!grad_w_min || !grad_w_max) return TCONV_E_INVAL; break;
  }
  double* partial = nullptr;
  if (!take_partial(workspace, workspace_bytes, backward_weight_workspace(p), &partial)) return TCONV_E_WORKSPACE;
  BwdArgs a = {gy, alpha, beta, idx_min, idx_max};
  own_status();
  const hipError_t e = launch_backward_weight(p, a, grad_w_min, grad_w_max, partial, (hipStream_t)hip_stream);
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv_backward_weight_noalloc(const tconv_desc* desc, const float* gy, const float* alpha, const float* beta,
                                  const int32_t* idx_min, const int32_t* idx_max, float* grad_w_min,
                                  float* grad_w_max, void* hip_stream) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!gy) return TCONV_E_INVAL;
  p.mode = backward_mode(p.mode);
  if (p.mode != TCONV_MAX && !idx_min) return TCONV_E_INVAL;
  if (p.mode != TCONV_MIN && !idx_max) return TCONV_E_INVAL;
  switch (p.mode) {
    case TCONV_MAX: if (!grad_w_max) return TCONV_E_INVAL; break;
    case TCONV_MIN: if (!grad_w_min) return TCONV_E_INVAL; break;
    case TCONV_COMPOUND: if (!grad_w_min && !grad_w_max) return TCONV_E_INVAL; break;
    default: if (!grad_w_min || !grad_w_max) return TCONV_E_INVAL; break;
  }
  if (backward_weight_workspace(p) > backward_weight_static_limit()) return TCONV_E_WORKSPACE;
  BwdArgs a = {gy, alpha, beta, idx_min, idx_max};
  own_status();
  const hipError_t e = launch_backward_weight_static(p, a, grad_w_min, grad_w_max, (hipStream_t)hip_stream);
  if (e == hipErrorOutOfMemory) return TCONV_E_WORKSPACE;
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv_backward(const tconv_desc* desc, const float* gy, const float* alpha, const float* beta,
                   const int32_t* idx_min, const int32_t* idx_max, float* grad_x, float* grad_w_min,
                   float* grad_w_max, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!gy || !grad_x) return TCONV_E_INVAL;
  p.mode = backward_mode(p.mode);
  if (p.mode != TCONV_MAX && !idx_min) return TCONV_E_INVAL;
  if (p.mode != TCONV_MIN && !idx_max) return TCONV_E_INVAL;
  switch (p.mode) {
    case TCONV_MAX: if (!grad_w_max) return TCONV_E_INVAL; break;
    case TCONV_MIN: if (!grad_w_min) return TCONV_E_INVAL; break;
    case TCONV_COMPOUND: if (!grad_w_min && !grad_w_max) return TCONV_E_INVAL; break;
    default: if (!grad_w_min || !grad_w_max) return TCONV_E_INVAL; break;
  }
  double* partial = nullptr;
  if (!take_partial(workspace, workspace_bytes, backward_weight_workspace(p), &partial)) return TCONV_E_WORKSPACE;
  BwdArgs a = {gy, alpha, beta, idx_min, idx_max};
  own_status();
  // the kernel gradient first: it reads gy / idx in the order the forward pass wrote them; the input gradient, which
  // follows on the same stream, finds what the last-level cache still holds of them
  hipError_t e = launch_backward_weight(p, a, grad_w_min, grad_w_max, partial, (hipStream_t)hip_stream);
  if (e == hipSuccess) e = launch_backward_input(p, a, grad_x, (hipStream_t)hip_stream);
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv_backward_bias(const tconv_desc* desc, const float* gy, float* grad_bias, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!gy || !grad_bias) return TCONV_E_INVAL;
  double* partial = nullptr;
  if (!take_partial(workspace, workspace_bytes, backward_alpha_beta_workspace(p), &partial)) return TCONV_E_WORKSPACE;
  own_status();
  const hipError_t e = launch_backward_bias(p, gy, grad_bias, partial, (hipStream_t)hip_stream);
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv_backward_alpha_beta(const tconv_desc* desc, const float* gy, const void* y_min,
                              const void* y_max, float* grad_alpha, float* grad_beta, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (p.mode != TCONV_COMPOUND && p.mode != TCONV_PARALLEL) return TCONV_E_INVAL;
  if (!gy || (!grad_alpha && !grad_beta)) return TCONV_E_INVAL;
  if ((grad_alpha && !y_min) || (grad_beta && !y_max)) return TCONV_E_INVAL;
  double* partial = nullptr;
  if (!take_partial(workspace, workspace_bytes, backward_alpha_beta_workspace(p), &partial)) return TCONV_E_WORKSPACE;
  own_status();
  const hipError_t e = launch_backward_alpha_beta(p, desc->dtype, gy, y_min, y_max, grad_alpha, grad_beta, partial,
                                                  (hipStream_t)hip_stream);
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv_backward_params(const tconv_desc* desc, const float* gy, const float* alpha, const float* beta,
                          const int32_t* idx_min, const int32_t* idx_max, const void* y_min, const void* y_max,
                          float* grad_w_min, float* grad_w_max, float* grad_alpha, float* grad_beta,
                          float* grad_bias, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!gy) return TCONV_E_INVAL;
  if ((grad_alpha || grad_beta) && p.mode != TCONV_COMPOUND && p.mode != TCONV_PARALLEL) return TCONV_E_INVAL;
  if ((grad_alpha && !y_min) || (grad_beta && !y_max)) return TCONV_E_INVAL;
  p.mode = backward_mode(p.mode);
  if (p.mode != TCONV_MAX && !idx_min) return TCONV_E_INVAL;
  if (p.mode != TCONV_MIN && !idx_max) return TCONV_E_INVAL;
  switch (p.mode) {
    case TCONV_MAX: if (!grad_w_max) return TCONV_E_INVAL; break;
    case TCONV_MIN: if (!grad_w_min) return TCONV_E_INVAL; break;
    case TCONV_COMPOUND: if (!grad_w_min && !grad_w_max) return TCONV_E_INVAL; break;
    default: if (!grad_w_min || !grad_w_max) return TCONV_E_INVAL; break;
  }
  double* partial = nullptr;
  if (!take_partial(workspace, workspace_bytes, params_workspace(p, desc->dtype), &partial)) return TCONV_E_WORKSPACE;
  const BwdArgs a = {gy, alpha, beta, idx_min, idx_max};
  hipStream_t s = (hipStream_t)hip_stream;
  own_status();
  if (partial && params_one_pass(p, desc->dtype)) {
    const hipError_t e = launch_backward_params(p, a, (const float*)y_min, (const float*)y_max, nullptr, nullptr, nullptr,
                                                grad_w_min, grad_w_max, grad_alpha, grad_beta, grad_bias, partial, s);
    return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
  }
  // the separate kernels, each in its deterministic form when there is scratch; the two small reductions share theirs
  // (they follow each other on the stream)
  double* const part_w = (partial && backward_weight_workspace(p)) ? partial : nullptr;
  double* const part_ab = partial ? (double*)((char*)partial + params_split_offset(p)) : nullptr;
  hipError_t e = launch_backward_weight(p, a, grad_w_min, grad_w_max, part_w, s);
  if (e == hipSuccess && (grad_alpha || grad_beta))
    e = launch_backward_alpha_beta(p, desc->dtype, gy, y_min, y_max, grad_alpha, grad_beta, part_ab, s);
  if (e == hipSuccess && grad_bias) e = launch_backward_bias(p, gy, grad_bias, part_ab, s);
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv_backward_params_recompute(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                                    const float* gy, const float* alpha, const float* beta, const int32_t* idx_min,
                                    const int32_t* idx_max, float* grad_w_min, float* grad_w_max, float* grad_alpha,
                                    float* grad_beta, float* grad_bias, void* workspace, size_t workspace_bytes,
                                    void* hip_stream) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!gy || !x) return TCONV_E_INVAL;
  if ((grad_alpha || grad_beta) && p.mode != TCONV_COMPOUND && p.mode != TCONV_PARALLEL) return TCONV_E_INVAL;
  const int fwd_mode = p.mode;
  p.mode = backward_mode(p.mode);
  if (p.mode != TCONV_MAX && !idx_min) return TCONV_E_INVAL;
  if (p.mode != TCONV_MIN && !idx_max) return TCONV_E_INVAL;
  const void* wa = w_min;
  const void* wb = w_max;
  if (fwd_mode == TCONV_COMPOUND) wa = wb = (w_min ? w_min : w_max);
  if (grad_alpha && !wa) return TCONV_E_INVAL;
  if (grad_beta && !wb) return TCONV_E_INVAL;
  switch (p.mode) {
    case TCONV_MAX: if (!grad_w_max) return TCONV_E_INVAL; break;
    case TCONV_MIN: if (!grad_w_min) return TCONV_E_INVAL; break;
    case TCONV_COMPOUND: if (!grad_w_min && !grad_w_max) return TCONV_E_INVAL; break;
    default: if (!grad_w_min || !grad_w_max) return TCONV_E_INVAL; break;
  }
  // fp32 storage, a window whose histogram fits LDS, and the scratch of the one-pass form
  if (desc->dtype != TCONV_F32 || !params_one_pass(p, desc->dtype)) return TCONV_E_UNSUPPORTED;
  double* partial = nullptr;
  if (!take_partial(workspace, workspace_bytes, params_workspace(p, desc->dtype), &partial) || !partial)
    return TCONV_E_WORKSPACE;
  const BwdArgs a = {gy, alpha, beta, idx_min, idx_max};
  own_status();
  const hipError_t e = launch_backward_params(p, a, nullptr, nullptr, (const float*)x, (const float*)wa, (const float*)wb,
                                              grad_w_min, grad_w_max, grad_alpha, grad_beta, grad_bias, partial,
                                              (hipStream_t)hip_stream);
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv_sum_workspace_bytes(const tconv_desc* desc, int backward, size_t* bytes) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!bytes || p.mode > TCONV_PARALLEL) return TCONV_E_INVAL;
  if (desc->dtype != TCONV_F32 && desc->dtype != TCONV_BF16) return TCONV_E_UNSUPPORTED;
  *bytes = sum_workspace(p, desc->dtype, backward != 0);
  return TCONV_OK;
}

int tconv_sum_forward(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                      const float* alpha, const float* beta, void* y, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!x || !y) return TCONV_E_INVAL;
  if (p.mode > TCONV_PARALLEL) return TCONV_E_INVAL;  // the mixed layers have no channel sum
  if ((desc->dtype != TCONV_F32 && desc->dtype != TCONV_BF16) || p.pad_zero) return TCONV_E_UNSUPPORTED;
  if (!sum_forward_supported(p, desc->dtype)) return TCONV_E_UNSUPPORTED;
  const size_t need = sum_workspace(p, desc->dtype, false);
  if (need && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))) return TCONV_E_WORKSPACE;
  SumArgs a = {(const float*)x, (const float*)w_min, (const float*)w_max, alpha, beta, (float*)y};
  if (p.mode == TCONV_COMPOUND) a.w_min = a.w_max = (const float*)(w_min ? w_min : w_max);
  if (p.mode != TCONV_MAX && !a.w_min) return TCONV_E_INVAL;
  if (p.mode != TCONV_MIN && !a.w_max) return TCONV_E_INVAL;
  own_status();
  const hipError_t e = launch_sum_forward(p, desc->dtype, a, workspace, (hipStream_t)hip_stream);
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv_sum_backward(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                       const float* alpha, const float* beta, const float* gy, float* grad_x,
                       float* grad_w_min, float* grad_w_max, float* grad_alpha, float* grad_beta,
                       void* workspace, size_t workspace_bytes, void* hip_stream) {
  Params p;
  const int rc = make_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!x || !gy) return TCONV_E_INVAL;
  if (p.mode > TCONV_PARALLEL) return TCONV_E_INVAL;  // the mixed layers have no channel sum
  if ((desc->dtype != TCONV_F32 && desc->dtype != TCONV_BF16) || p.pad_zero) return TCONV_E_UNSUPPORTED;
  const size_t need = sum_workspace(p, desc->dtype, true);
  if (need && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))) return TCONV_E_WORKSPACE;
  const bool two = p.mode == TCONV_COMPOUND || p.mode == TCONV_PARALLEL;
  if (!two && (grad_alpha || grad_beta)) return TCONV_E_INVAL;
  if (!grad_x && !grad_w_min && !grad_w_max && !grad_alpha && !grad_beta) return TCONV_E_INVAL;
  SumArgs a = {(const float*)x, (const float*)w_min, (const float*)w_max, alpha, beta, nullptr};
  if (p.mode == TCONV_COMPOUND) a.w_min = a.w_max = (const float*)(w_min ? w_min : w_max);
  if (p.mode != TCONV_MAX && !a.w_min) return TCONV_E_INVAL;
  if (p.mode != TCONV_MIN && !a.w_max) return TCONV_E_INVAL;
  const SumGrads g = {gy, grad_x, grad_w_min, grad_w_max, grad_alpha, grad_beta};
  own_status();
  const hipError_t e = launch_sum_backward(p, desc->dtype, a, g, workspace, (hipStream_t)hip_stream);
  if (e == hipErrorInvalidValue) return TCONV_E_UNSUPPORTED;  // rows or kernel window too large for the LDS kernels
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

const char* tconv_sum_forward_kernel_name(const tconv_desc* desc) {
  Params p;
  if (make_params(desc, &p) != TCONV_OK || p.mode > TCONV_PARALLEL) return nullptr;
  return sum_forward_kernel_name(p);
}

// Depthwise layers: C_out a multiple of C_in, one of the four base modes, fp32 storage.
static int depthwise_params(const tconv_desc* desc, Params* p) {
  const int rc = make_params(desc, p);
  if (rc != TCONV_OK) return rc;
  if (p->mode > TCONV_PARALLEL) return TCONV_E_INVAL;
  if (p->C_out % p->C_in != 0) return TCONV_E_SHAPE;
  if (desc->dtype != TCONV_F32 || p->pad_zero) return TCONV_E_UNSUPPORTED;
  return TCONV_OK;
}

int tconv_depthwise_forward(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                            const float* alpha, const float* beta, void* y, uint8_t* idx, void* workspace,
                            size_t workspace_bytes, void* hip_stream) {
  (void)workspace; (void)workspace_bytes;
  Params p;
  const int rc = depthwise_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!x || !y) return TCONV_E_INVAL;
  if (idx && p.KH * p.KW > 16) return TCONV_E_UNSUPPORTED;  // a winning tap must fit a nibble
  DwArgs a = {(const float*)x, (const float*)w_min, (const float*)w_max, alpha, beta, (float*)y, idx};
  if (p.mode == TCONV_COMPOUND) a.w_min = a.w_max = (const float*)(w_min ? w_min : w_max);
  if (p.mode != TCONV_MAX && !a.w_min) return TCONV_E_INVAL;
  if (p.mode != TCONV_MIN && !a.w_max) return TCONV_E_INVAL;
  own_status();
  const hipError_t e = launch_depthwise_forward(p, a, (hipStream_t)hip_stream);
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv_depthwise_backward(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                             const float* alpha, const float* beta, const float* gy, const uint8_t* idx,
                             float* grad_x, float* grad_w_min, float* grad_w_max, float* grad_alpha,
                             float* grad_beta, void* workspace, size_t workspace_bytes, void* hip_stream) {
  (void)workspace; (void)workspace_bytes;
  Params p;
  const int rc = depthwise_params(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!gy || !idx) return TCONV_E_INVAL;
  if (p.KH * p.KW > 16) return TCONV_E_UNSUPPORTED;
  const bool two = p.mode == TCONV_COMPOUND || p.mode == TCONV_PARALLEL;
  if (!two && (grad_alpha || grad_beta)) return TCONV_E_INVAL;
  if (!grad_x && !grad_w_min && !grad_w_max && !grad_alpha && !grad_beta) return TCONV_E_INVAL;
  DwArgs a = {(const float*)x, (const float*)w_min, (const float*)w_max, alpha, beta, nullptr,
              const_cast<uint8_t*>(idx)};
  if (p.mode == TCONV_COMPOUND) a.w_min = a.w_max = (const float*)(w_min ? w_min : w_max);
  if (grad_alpha || grad_beta) {  // the branch outputs are re-evaluated at the winners
    if (!x) return TCONV_E_INVAL;
    if ((p.mode != TCONV_MAX && !a.w_min) || (p.mode != TCONV_MIN && !a.w_max)) return TCONV_E_INVAL;
  }
  const DwGrads g = {gy, grad_x, grad_w_min, grad_w_max, grad_alpha, grad_beta};
  own_status();
  const hipError_t e = launch_depthwise_backward(p, a, g, (hipStream_t)hip_stream);
  if (e == hipErrorInvalidValue) return TCONV_E_UNSUPPORTED;
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

const char* tconv_depthwise_forward_kernel_name(const tconv_desc* desc) {
  Params p;
  if (depthwise_params(desc, &p) != TCONV_OK) return nullptr;
  return depthwise_forward_kernel_name(p);
}

// The two-dimensional view of a one-dimensional layer (same memory, same flattened tap numbers).
static int view_2d(const tconv1d_desc* d, tconv_desc* v) {
  if (!d) return TCONV_E_INVAL;
  if (d->N < 1 || d->C_in < 1 || d->L < 1 || d->C_out < 1 || d->K < 1 || d->stride < 1 || d->dil < 1 || d->pad < 0)
    return TCONV_E_INVAL;
  const bool full_window = d->mode >= TCONV_MAX && d->mode <= TCONV_PARALLEL;
  // three consecutive channels as the three rows of an image: the 3 x 3 window of "channel" c' covers the taps
  // of channels 3c', 3c'+1, 3c'+2, and k = ((c'*3 + i)*3 + j) = (3c' + i)*3 + j is the 1-D tap number
  const bool rows3 = full_window && d->K == 3 && d->dil == 1 && (d->stride == 1 || d->stride == 2) && d->pad <= 1 &&
                     d->C_in % 3 == 0;
  if (rows3) {
    const tconv_desc t = {d->N, d->C_in / 3, 3, d->L, d->C_out, 3, 3, d->stride, d->stride, 0, d->pad, 1, 1, d->mode,
                          d->dtype};
    *v = t;
  } else {
    const tconv_desc t = {d->N, d->C_in, 1, d->L, d->C_out, 1, d->K, 1, d->stride, 0, d->pad, 1, d->dil, d->mode,
                          d->dtype};
    *v = t;
  }
  return TCONV_OK;
}

int tconv1d_out_len(const tconv1d_desc* desc, int32_t* L_out) {
  tconv_desc v;
  int32_t ho = 0;
  const int rc = view_2d(desc, &v);
  return rc != TCONV_OK ? rc : tconv_out_shape(&v, &ho, L_out);
}

int tconv1d_workspace_bytes(const tconv1d_desc* desc, int32_t op, size_t* bytes) {
  tconv_desc v;
  const int rc = view_2d(desc, &v);
  return rc != TCONV_OK ? rc : tconv_workspace_bytes(&v, op, bytes);
}

int tconv1d_forward(const tconv1d_desc* desc, const void* x, const void* w_min, const void* w_max,
                    const float* alpha, const float* beta, void* y, void* y_min, void* y_max,
                    int32_t* idx_min, int32_t* idx_max, void* workspace, size_t workspace_bytes,
                    void* hip_stream) {
  tconv_desc v;
  const int rc = view_2d(desc, &v);
  if (rc != TCONV_OK) return rc;
  return tconv_forward(&v, x, w_min, w_max, alpha, beta, y, y_min, y_max, idx_min, idx_max, workspace,
                       workspace_bytes, hip_stream);
}

int tconv1d_backward_input(const tconv1d_desc* desc, const float* gy, const float* alpha, const float* beta,
                           const int32_t* idx_min, const int32_t* idx_max, float* grad_x, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
  tconv_desc v;
  const int rc = view_2d(desc, &v);
  if (rc != TCONV_OK) return rc;
  return tconv_backward_input(&v, gy, alpha, beta, idx_min, idx_max, grad_x, workspace, workspace_bytes, hip_stream);
}

int tconv1d_backward_weight(const tconv1d_desc* desc, const float* gy, const float* alpha, const float* beta,
                            const int32_t* idx_min, const int32_t* idx_max, float* grad_w_min,
                            float* grad_w_max, void* workspace, size_t workspace_bytes, void* hip_stream) {
  tconv_desc v;
  const int rc = view_2d(desc, &v);
  if (rc != TCONV_OK) return rc;
  return tconv_backward_weight(&v, gy, alpha, beta, idx_min, idx_max, grad_w_min, grad_w_max, workspace,
                               workspace_bytes, hip_stream);
}

const char* tconv1d_forward_kernel_name(const tconv1d_desc* desc) {
  tconv_desc v;
  if (view_2d(desc, &v) != TCONV_OK) return nullptr;
  return tconv_forward_kernel_name(&v);
}

// Validates a three-dimensional descriptor and fills the launch-time view.
static int make_params3(const tconv3d_desc* d, Params3* p) {
  if (!d) return TCONV_E_INVAL;
  if (d->N < 1 || d->C_in < 1 || d->D < 1 || d->H < 1 || d->W < 1 || d->C_out < 1 || d->KD < 1 || d->KH < 1 || d->KW < 1)
    return TCONV_E_INVAL;
  if (d->stride_d < 1 || d->stride_h < 1 || d->stride_w < 1 || d->dil_d < 1 || d->dil_h < 1 || d->dil_w < 1 ||
      d->pad_d < 0 || d->pad_h < 0 || d->pad_w < 0)
    return TCONV_E_INVAL;
  if (d->mode < TCONV_MAX || d->mode > TCONV_MAXPLUS_MIN) return TCONV_E_INVAL;
  if (d->dtype != TCONV_F32 && d->dtype != TCONV_BF16) return TCONV_E_INVAL;
  const long long in[3] = {d->D, d->H, d->W}, k[3] = {d->KD, d->KH, d->KW};
  const long long st[3] = {d->stride_d, d->stride_h, d->stride_w}, pd[3] = {d->pad_d, d->pad_h, d->pad_w};
  const long long dl[3] = {d->dil_d, d->dil_h, d->dil_w};
  long long out[3];
  for (int a = 0; a < 3; ++a) {
    const long long ext = dl[a] * (k[a] - 1);
    if (pd[a] > ext) return TCONV_E_SHAPE;  // a window could lie wholly in the padding
    const long long n = in[a] + 2 * pd[a] - ext - 1;
    if (n < 0) return TCONV_E_SHAPE;
    out[a] = n / st[a] + 1;
  }
  const long long K = (long long)d->C_in * d->KD * d->KH * d->KW, lim = 0x7fffffffLL;
  if (K > lim || (long long)d->N * d->C_in * d->D * d->H * d->W > lim ||
      (long long)d->N * d->C_out * out[0] * out[1] * out[2] > lim || (long long)d->C_out * K > lim)
    return TCONV_E_SHAPE;
  for (int a = 0; a < 3; ++a)  // the taps of a window must not straddle an input shorter than the dilation either
    if (axis_has_empty_window(in[a], k[a], st[a], pd[a], dl[a], out[a])) return TCONV_E_SHAPE;
  if (d->dtype != TCONV_F32) return TCONV_E_UNSUPPORTED;
  p->N = d->N; p->C_in = d->C_in; p->D = d->D; p->H = d->H; p->W = d->W;
  p->C_out = d->C_out; p->KD = d->KD; p->KH = d->KH; p->KW = d->KW;
  p->sd = d->stride_d; p->sh = d->stride_h; p->sw = d->stride_w;
  p->pd = d->pad_d; p->ph = d->pad_h; p->pw = d->pad_w;
  p->dd = d->dil_d; p->dh = d->dil_h; p->dw = d->dil_w;
  p->Do = (int)out[0]; p->Ho = (int)out[1]; p->Wo = (int)out[2];
  p->K = (int)K; p->mode = d->mode;
  return TCONV_OK;
}

// What the two-dimensional histogram kernel needs to know of a three-dimensional layer: outputs per (image, channel)
// and taps per channel, not the geometry.
static Params histogram_view(const Params3& p3, int mode) {
  Params p = {};
  p.N = p3.N; p.C_out = p3.C_out; p.Ho = p3.Do * p3.Ho; p.Wo = p3.Wo; p.K = p3.K; p.mode = mode;
  return p;
}

int tconv3d_workspace_bytes(const tconv3d_desc* desc, int32_t op, size_t* bytes) {
  Params3 p3;
  const int rc = make_params3(desc, &p3);
  if (rc != TCONV_OK) return rc;
  if (!bytes || op < TCONV_OP_FORWARD || op > TCONV_OP_BACKWARD) return TCONV_E_INVAL;
  *bytes = (op == TCONV_OP_BACKWARD_WEIGHT) ? backward_weight_workspace(histogram_view(p3, backward_mode(p3.mode))) : 0;
  return TCONV_OK;
}

int tconv3d_out_shape(const tconv3d_desc* desc, int32_t* D_out, int32_t* H_out, int32_t* W_out) {
  Params3 p;
  const int rc = make_params3(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!D_out || !H_out || !W_out) return TCONV_E_INVAL;
  *D_out = p.Do; *H_out = p.Ho; *W_out = p.Wo;
  return TCONV_OK;
}

const char* tconv3d_forward_kernel_name(const tconv3d_desc* desc) {
  Params3 p;
  if (make_params3(desc, &p) != TCONV_OK) return nullptr;
  return forward_3d_kernel_name(p);
}

int tconv3d_forward(const tconv3d_desc* desc, const void* x, const void* w_min, const void* w_max,
                    const float* alpha, const float* beta, void* y, void* y_min, void* y_max,
                    int32_t* idx_min, int32_t* idx_max, void* workspace, size_t workspace_bytes,
                    void* hip_stream) {
  (void)workspace; (void)workspace_bytes;
  Params3 p;
  const int rc = make_params3(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!x || !y) return TCONV_E_INVAL;
  FwdArgs a = {x, w_min, w_max, alpha, beta, y, y_min, y_max, idx_min, idx_max};
  if (p.mode == TCONV_COMPOUND) a.w_min = a.w_max = (w_min ? w_min : w_max);
  if (mode_has_min(p.mode) && (!a.w_min || !idx_min)) return TCONV_E_INVAL;
  if (mode_has_max(p.mode) && (!a.w_max || !idx_max)) return TCONV_E_INVAL;
  own_status();
  const hipError_t e = launch_forward_3d(p, a, (hipStream_t)hip_stream);
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv3d_backward_input(const tconv3d_desc* desc, const float* gy, const float* alpha, const float* beta,
                           const int32_t* idx_min, const int32_t* idx_max, float* grad_x, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
  (void)workspace; (void)workspace_bytes;
  Params3 p;
  const int rc = make_params3(desc, &p);
  if (rc != TCONV_OK) return rc;
  if (!gy || !grad_x) return TCONV_E_INVAL;
  p.mode = backward_mode(p.mode);
  if (p.mode != TCONV_MAX && !idx_min) return TCONV_E_INVAL;
  if (p.mode != TCONV_MIN && !idx_max) return TCONV_E_INVAL;
  BwdArgs a = {gy, alpha, beta, idx_min, idx_max};
  own_status();
  const hipError_t e = launch_backward_input_3d(p, a, grad_x, (hipStream_t)hip_stream);
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

int tconv3d_backward_weight(const tconv3d_desc* desc, const float* gy, const float* alpha, const float* beta,
                            const int32_t* idx_min, const int32_t* idx_max, float* grad_w_min,
                            float* grad_w_max, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Params3 p3;
  const int rc = make_params3(desc, &p3);
  if (rc != TCONV_OK) return rc;
  if (!gy) return TCONV_E_INVAL;
  const int mode = backward_mode(p3.mode);
  if (mode != TCONV_MAX && !idx_min) return TCONV_E_INVAL;
  if (mode != TCONV_MIN && !idx_max) return TCONV_E_INVAL;
  switch (mode) {
    case TCONV_MAX: if (!grad_w_max) return TCONV_E_INVAL; break;
    case TCONV_MIN: if (!grad_w_min) return TCONV_E_INVAL; break;
    case TCONV_COMPOUND: if (!grad_w_min && !grad_w_max) return TCONV_E_INVAL; break;
    default: if (!grad_w_min || !grad_w_max) return TCONV_E_INVAL; break;
  }
  // The kernel gradient is a histogram of the winners per output channel: it needs the number of outputs per
  // (image, channel) and the number of taps, not the geometry, so the two-dimensional kernel takes it as is.
  const Params p = histogram_view(p3, mode);
  double* partial = nullptr;
  if (!take_partial(workspace, workspace_bytes, backward_weight_workspace(p), &partial)) return TCONV_E_WORKSPACE;
  BwdArgs a = {gy, alpha, beta, idx_min, idx_max};
  own_status();
  const hipError_t e = launch_backward_weight(p, a, grad_w_min, grad_w_max, partial, (hipStream_t)hip_stream);
  return e == hipSuccess ? TCONV_OK : TCONV_E_LAUNCH;
}

const char* tconv_status_string(int status) {
  switch (status) {
    case TCONV_OK: return "ok";
    case TCONV_E_INVAL: return "invalid argument (NULL required pointer, non-positive size, bad mode, dtype or op)";
    case TCONV_E_SHAPE: return "unsupported shape (empty output, a window with no tap inside the input, or a tensor of 2^31 or more elements)";
    case TCONV_E_WORKSPACE: return "workspace missing or too small";
    case TCONV_E_UNSUPPORTED: return "no kernel for this request in this build";
    case TCONV_E_LAUNCH: return "HIP kernel launch failed";
    default: return "unknown status";
  }
}

const char* tconv_forward_kernel_name(const tconv_desc* desc) {
  Params p;
  if (make_params(desc, &p) != TCONV_OK) return nullptr;
  if (use_tiled16(p, desc->dtype)) return "tiled3x3_f16";
  if (use_tiled(p, desc->dtype)) return forward_tiled3x3_splits(p, desc->dtype) ? "tiled3x3_split" : "tiled3x3";
  if (use_row(p, desc->dtype)) return "row1d";
  return use_rowtile(p, desc->dtype) ? "rowtile" : "generic";
}

}  // extern "C"
