/*
 * tconv.h - C ABI of the MI355X (gfx950) tropical convolution library.
 *
 * Operator family (paper Sec. 3.1 and 3.3).  For every output element
 * (n, c_out, oh, ow) and every live branch the library reduces over all
 * K = C_in*KH*KW taps of the window
 *
 *     y_max = max_k ( x[n, c, ih, iw] + w_max[c_out, c, i, j] )     max-plus, layer (v) MaxPlus-Max-Conv2d
 *     y_min = min_k ( x[n, c, ih, iw] + w_min[c_out, c, i, j] )     min-plus, layer (iv) MinPlus-Min-Conv2d
 *
 * with k = (c*KH + i)*KW + j, ih = oh*stride_h - pad_h + i*dil_h, iw likewise
 * (cross-correlation, as the discrete operators of Sec. 3.1 are written), and
 *
 *     compound:  y = alpha[c_out]*y_min + beta[c_out]*y_max,  ONE kernel feeds both branches
 *     parallel:  y = alpha[c_out]*y_min + beta[c_out]*y_max,  kernel g1 = w_min, g2 = w_max
 *
 * (Sec. 3.3, Definitions "compound" and "parallel"; alpha = beta = 1 gives the
 * direct-summation variants of App. B.4).  The mixed layers of Sec. 3.1 reduce the
 * window of every input channel with one operator and the channel results with the other:
 *
 *     minplus_max:  y = max_c ( min_{i,j} ( x + w_min ) )     layer (iii) MinPlus-Max-Conv2d
 *     maxplus_min:  y = min_c ( max_{i,j} ( x + w_max ) )     layer (vi)  MaxPlus-Min-Conv2d
 *
 * with winner k = c* *KH*KW + t*: the lowest tap t* of the inner reduction inside the lowest
 * channel c* of the outer one.  Padding holds the semiring identity
 * (-inf for max-plus, +inf for min-plus, Sec. 3.1): a padded tap never wins.
 * Ties keep the lowest k.  Every x + w is one rounded fp32 add; the combine is
 * two rounded fp32 products and one rounded fp32 sum (no fused multiply-add).
 * Backward routes the whole output gradient of a branch through its winning
 * tap (the saved idx), scaled by alpha (min branch) / beta (max branch) in
 * compound and parallel mode and unscaled in max / min mode.
 *
 * Conventions shared by every entry point
 *   - Tensors are contiguous, x / grad_x NCHW, kernels OIHW, outputs NCHW
 *     [N, C_out, H_out, W_out].  All tensor pointers are DEVICE pointers owned by
 *     the caller; `desc` and the size outputs are HOST pointers.  The library
 *     allocates nothing and keeps no state between calls.
 *   - dtype selects the storage type of x, kernels, y, y_min, y_max (fp32 or
 *     bf16; bf16 is widened exactly, all arithmetic and the index decision are
 *     fp32, results are rounded to nearest-even on store).  gy, grad_x, grad_w,
 *     alpha, beta are always fp32; idx_* are int32 in [0, K).
 *   - Domain: finite values, no negative zero in x or the kernels.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on that stream and return; outputs are overwritten.
 *   - Return value: TCONV_OK (0) or a negative tconv_status.  The library never
 *     aborts, throws or prints.  On error nothing has been enqueued.
 */
#ifndef TCONV_H
#define TCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum tconv_mode {
  TCONV_MAX = 0,         /* Sec. 3.1 layer (v)  MaxPlus-Max-Conv2d                                   */
  TCONV_MIN = 1,         /* Sec. 3.1 layer (iv) MinPlus-Min-Conv2d                                   */
  TCONV_COMPOUND = 2,    /* Sec. 3.3 compound: one shared kernel, alpha*min + beta*max               */
  TCONV_PARALLEL = 3,    /* Sec. 3.3 parallel: two kernels, alpha*min + beta*max                     */
  TCONV_MINPLUS_MAX = 4, /* Sec. 3.1 layer (iii) MinPlus-Max-Conv2d: max over c_in of the min-plus operator;
                            single branch on the MIN side (w_min, idx_min, y_min, grad_w_min)       */
  TCONV_MAXPLUS_MIN = 5  /* Sec. 3.1 layer (vi) MaxPlus-Min-Conv2d: min over c_in of the max-plus operator;
                            single branch on the MAX side (w_max, idx_max, y_max, grad_w_max)       */
};
enum tconv_dtype {
  TCONV_F32 = 0,
  TCONV_BF16 = 1,  /* storage only: widened exactly, all arithmetic and the index decision in fp32 */
  TCONV_F16 = 2    /* IEEE binary16 storage AND arithmetic (the packed 16-bit path): every candidate x + w is ONE add
                      rounded to binary16 (nearest even), the comparisons are on those binary16 sums, ties keep the
                      lowest k; the combine is evaluated in fp32 from the binary16 extrema (two rounded products, one
                      rounded sum) and rounded to binary16 once.  tconv_forward / tconv_backward* / the one-dimensional
                      entry points only; no epilogue (TCONV_E_UNSUPPORTED elsewhere).  Results differ from the fp32
                      layers by construction: it is a different numeric contract, not an approximation of theirs. */
};
enum tconv_pad_mode {
  TCONV_PAD_IDENTITY = 0,  /* padding holds the semiring identity (Sec. 3.1): a padded tap never wins            */
  TCONV_PAD_ZERO = 1       /* padding holds zeros (App. A.1.1, the unfold formulation pads the input with zeros):
                              a padded tap is a candidate of value fl(0 + w[k]); it can win, its index is saved
                              like any other, and in the backward pass its gradient reaches the kernel only     */
};
enum tconv_op {
  TCONV_OP_FORWARD = 0,
  TCONV_OP_BACKWARD_INPUT = 1,
  TCONV_OP_BACKWARD_WEIGHT = 2,
  TCONV_OP_BACKWARD_ALPHA_BETA = 3,
  TCONV_OP_BACKWARD = 4,  /* tconv_backward: both gradients in one call */
  TCONV_OP_BACKWARD_BIAS = 5,
  TCONV_OP_BACKWARD_PARAMS = 6  /* tconv_backward_params: every parameter gradient in one call */
};

enum tconv_status {
  TCONV_OK = 0,
  TCONV_E_INVAL = -1,       /* NULL required pointer, non-positive dim, stride < 1, dil < 1, pad < 0, bad mode / dtype / op */
  TCONV_E_SHAPE = -2,       /* H_out or W_out < 1, a window with no tap inside the input (pad > dil*(k-1), or dilated taps that straddle an input shorter than the dilation), a tensor with >= 2^31 elements */
  TCONV_E_WORKSPACE = -3,   /* workspace NULL or smaller than tconv_workspace_bytes() reports */
  TCONV_E_UNSUPPORTED = -4, /* valid request this build has no kernel for */
  TCONV_E_LAUNCH = -5       /* the HIP runtime refused a launch (hipGetLastError) */
};

typedef struct tconv_desc {
  int32_t N, C_in, H, W;    /* input  [N, C_in, H, W]                 */
  int32_t C_out, KH, KW;    /* kernel [C_out, C_in, KH, KW]           */
  int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
  int32_t mode;             /* enum tconv_mode                        */
  int32_t dtype;            /* enum tconv_dtype                       */
  int32_t pad_mode;         /* enum tconv_pad_mode; the full-window layers (modes max .. parallel of tconv_forward*,
                               tconv_backward*) take both, the mixed modes and every other entry point
                               TCONV_PAD_IDENTITY only (TCONV_E_UNSUPPORTED)                                    */
} tconv_desc;

/* H_out = floor((H + 2*pad_h - dil_h*(KH-1) - 1)/stride_h) + 1, W_out likewise.  Host only. */
int tconv_out_shape(const tconv_desc* desc, int32_t* H_out, int32_t* W_out);

/* Scratch bytes `op` (enum tconv_op) needs (forward) or can use (the parameter gradients, where a workspace selects
 * the deterministic summation) for this descriptor; may be 0.  Host only. */
int tconv_workspace_bytes(const tconv_desc* desc, int32_t op, size_t* bytes);

/*
 * Forward (Sec. 3.1 layers (iii) - (vi); Sec. 3.3 compound / parallel).
 *   x        [N, C_in, H, W], dtype.
 *   w_min    kernel of the min-plus branch, w_max of the max-plus branch, dtype.
 *            max: w_max required (w_min ignored); min: w_min required;
 *            compound: the one shared kernel through either pointer (w_min wins if both set);
 *            parallel: both required (g1 = w_min, g2 = w_max);
 *            minplus_max: as min (w_min, idx_min, optional y_min); maxplus_min: as max.
 *   alpha, beta  fp32 [C_out] or NULL (= all ones); ignored in max / min mode.
 *   y        required; combined output (max / min: the single branch), dtype.
 *   y_min, y_max  optional branch outputs (NULL = not written), dtype.
 *   idx_min, idx_max  int32, required for every live branch: lowest winning tap k.
 *   workspace  device scratch of at least tconv_workspace_bytes(desc, TCONV_OP_FORWARD) bytes,
 *            256-byte aligned (may be NULL when that is 0).
 */
int tconv_forward(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                  const float* alpha, const float* beta, void* y, void* y_min, void* y_max,
                  int32_t* idx_min, int32_t* idx_max, void* workspace, size_t workspace_bytes,
                  void* hip_stream);

/*
 * Forward with the layer's epilogue fused into the kernel that produces y.  The layers of the paper derive from the
 * framework's convolution base class (App. A.2), which carries an optional bias, and its residual blocks (Sec. 5,
 * "TCNN BasicBlock": tropical conv -> batch norm -> tropical conv -> batch norm -> shortcut add, no activation) follow
 * every tropical layer with a batch norm and, at the end of the block, the shortcut.  With t the combined output of
 * tconv_forward, the call stores
 *     t1 = bias  ? fl(t + bias[c_out])                              : t
 *     t2 = scale ? fl(fl(t1 * scale[c_out]) + shift[c_out])         : t1      (shift NULL = zeros)
 *     y  = residual ? fl(t2 + residual[n, c_out, oh, ow])           : t2
 * every operation rounded to fp32 on its own (then to the storage dtype).  scale / shift are a batch norm folded for
 * inference, scale = gamma / sqrt(var + eps), shift = beta - mean * scale; forming them is the caller's business.
 * y_min, y_max, idx_min, idx_max are those of the bare layer.  `epilogue` is a HOST pointer to a struct of DEVICE
 * pointers (bias, scale, shift fp32 [C_out]; residual in the storage dtype, same shape as y; it may alias nothing the
 * call writes); NULL, or all members NULL, makes the call identical to tconv_forward.  Everything else as there.
 * Backward: the epilogue is affine, so the caller feeds tconv_backward* with gy scaled per channel (pass
 * alpha * scale and beta * scale as coefficients in compound / parallel mode), adds gy to the shortcut's gradient,
 * and gets grad_bias from tconv_backward_bias.
 */
typedef struct tconv_epilogue {
  const float* bias;
  const float* scale;
  const float* shift;
  const void* residual;
} tconv_epilogue;

int tconv_forward_fused(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                        const float* alpha, const float* beta, const tconv_epilogue* epilogue, void* y, void* y_min,
                        void* y_max, int32_t* idx_min, int32_t* idx_max, void* workspace, size_t workspace_bytes,
                        void* hip_stream);

/*
 * Gradient of the epilogue's bias: grad_bias[c_out] = sum over (n, oh, ow) of gy (gy as it arrives at the bias add,
 * fp32).  fp32 [C_out], overwritten.  workspace optional, tconv_workspace_bytes(desc, TCONV_OP_BACKWARD_BIAS): with
 * it the batch slices are added in a fixed order in fp64 (deterministic), without it with fp32 atomics.
 */
int tconv_backward_bias(const tconv_desc* desc, const float* gy, float* grad_bias, void* workspace,
                        size_t workspace_bytes, void* hip_stream);

/*
 * Backward w.r.t. the input: grad_x[n, c*, ih*, iw*] += g_b for every output and
 * live branch b, (c*, i*, j*) = unflatten(idx_b); g_min = alpha*gy, g_max = beta*gy
 * (compound / parallel), g = gy (max / min; minplus_max is treated as min, maxplus_min as
 * max: one winner per output carries the whole gradient).  grad_x fp32 [N, C_in, H, W] is
 * overwritten.  The sums are accumulated in fp64 in an unspecified order and rounded
 * to fp32 once.
 */
int tconv_backward_input(const tconv_desc* desc, const float* gy, const float* alpha,
                         const float* beta, const int32_t* idx_min, const int32_t* idx_max,
                         float* grad_x, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward w.r.t. the kernel(s): grad_w_b[c_out, k*] += g_b summed over (n, oh, ow).
 * max, maxplus_min: grad_w_max; min, minplus_max: grad_w_min; parallel: both; compound: both branches add
 * into ONE tensor, grad_w_min if non-NULL else grad_w_max.  fp32 OIHW, overwritten.
 *   workspace  optional.  With a buffer of tconv_workspace_bytes(desc, TCONV_OP_BACKWARD_WEIGHT) bytes (8-byte
 *            aligned; TCONV_E_WORKSPACE if smaller) the sums are DETERMINISTIC: fp64 partial histograms per batch
 *            slice, added in a fixed order and rounded to fp32 once.  With NULL (or when that size is 0: a window
 *            too large for an on-chip histogram) the batch slices are combined with fp32 atomics in an unspecified
 *            order, so the last bits vary from run to run.
 */
int tconv_backward_weight(const tconv_desc* desc, const float* gy, const float* alpha,
                          const float* beta, const int32_t* idx_min, const int32_t* idx_max,
                          float* grad_w_min, float* grad_w_max, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/*
 * tconv_backward_weight for callers that cannot allocate or pass device scratch: code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation.  Same arguments without the workspace pair, same deterministic
 * result bit for bit as tconv_backward_weight with a workspace: the fp64 partial histograms go to a fixed array of
 * 32 MiB of device memory that the library owns (each GPU the library runs on holds one until the process ends).
 * The call allocates nothing and frees nothing.  TCONV_E_WORKSPACE: the layer needs more than 32 MiB of partial
 * histograms (tconv_workspace_bytes(desc, TCONV_OP_BACKWARD_WEIGHT) tells how much); nothing was enqueued.
 * All calls on one GPU share the array: it needs no clearing between calls (every element is written before it is
 * read), but two calls whose kernels overlap in time on one GPU (different streams, different threads) race.
 */
int tconv_backward_weight_noalloc(const tconv_desc* desc, const float* gy, const float* alpha, const float* beta,
                                  const int32_t* idx_min, const int32_t* idx_max, float* grad_w_min,
                                  float* grad_w_max, void* hip_stream);

/*
 * Both gradients of the layer in one call: grad_x as tconv_backward_input writes it and the kernel gradient(s) as
 * tconv_backward_weight writes them, from the same gy / idx (every argument as in those two calls; grad_x and the
 * kernel gradient(s) of the mode are all required).  workspace: as for tconv_backward_weight, sized by
 * tconv_workspace_bytes(desc, TCONV_OP_BACKWARD).  The two kernels run back to back on the stream, so the second
 * reads gy / idx while the last-level cache still holds what fits of them.
 */
int tconv_backward(const tconv_desc* desc, const float* gy, const float* alpha, const float* beta,
                   const int32_t* idx_min, const int32_t* idx_max, float* grad_x, float* grad_w_min,
                   float* grad_w_max, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward w.r.t. the combine coefficients (Sec. 3.3: y = alpha*y_min + beta*y_max with learnable
 * alpha, beta; one pair per output channel): grad_alpha[c] = sum over (n, oh, ow) of gy*y_min,
 * grad_beta[c] = the same with y_max.  Compound and parallel mode only (TCONV_E_INVAL otherwise).
 *   gy       fp32 [N, C_out, H_out, W_out].
 *   y_min, y_max  the branch outputs of tconv_forward, dtype; y_min is required when grad_alpha is
 *            requested, y_max when grad_beta is.
 *   grad_alpha, grad_beta  fp32 [C_out], overwritten; either may be NULL (not computed), not both.
 * Partial sums are fp64.  workspace is optional: with a buffer of tconv_workspace_bytes(desc,
 * TCONV_OP_BACKWARD_ALPHA_BETA) bytes (8-byte aligned) the per-workgroup sums are added in a fixed order in fp64 and
 * rounded once (deterministic); with NULL they are added with fp32 atomics in an unspecified order.
 */
int tconv_backward_alpha_beta(const tconv_desc* desc, const float* gy, const void* y_min,
                              const void* y_max, float* grad_alpha, float* grad_beta, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/*
 * Every parameter gradient of a layer in one call, from one pass over gy where the layer allows it: the kernel
 * gradient(s) of tconv_backward_weight (Sec. 3.2: the winner of every output receives its gradient), grad_alpha /
 * grad_beta of tconv_backward_alpha_beta (Sec. 3.3: the combine is linear in its coefficients) and grad_bias of
 * tconv_backward_bias, each argument as in those calls.  grad_alpha, grad_beta (compound and parallel mode only) and
 * grad_bias are optional (NULL: not computed); the kernel gradient(s) of the mode are required.
 *   workspace  optional, tconv_workspace_bytes(desc, TCONV_OP_BACKWARD_PARAMS) bytes, 8-byte aligned
 *            (TCONV_E_WORKSPACE if smaller).  With it every result is a sum of fp64 partial sums per batch slice added
 *            in a fixed order and rounded to fp32 once, and for fp32 storage and windows whose histogram fits on chip
 *            (3x3 layers up to 455 input channels, 910 with one kernel tensor) one kernel reads gy, the winner indices and the branch outputs
 *            ONCE for all of them, followed by one reduction - three launches fewer than the separate calls, which is
 *            what a training step of a small layer is made of.  With NULL, or for other layers, the separate kernels
 *            run (NULL: their fp32-atomic forms).
 */
int tconv_backward_params(const tconv_desc* desc, const float* gy, const float* alpha, const float* beta,
                          const int32_t* idx_min, const int32_t* idx_max, const void* y_min, const void* y_max,
                          float* grad_w_min, float* grad_w_max, float* grad_alpha, float* grad_beta,
                          float* grad_bias, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * tconv_backward_params without stored branch outputs, for a forward pass that was given y_min = y_max = NULL (12
 * instead of 20 bytes written per output, which is what layers with few input channels wait for): an output's
 * y_min / y_max is formed again from its winner, fl(x[winner] + w[winner]), the very add the forward pass made
 * (Sec. 3.1: the output of a branch IS its winning candidate), so every gradient equals tconv_backward_params' bit
 * for bit.  x, w_min, w_max as in tconv_forward (COMPOUND: the one kernel tensor in either pointer); the other
 * arguments as in tconv_backward_params.  fp32 storage, windows whose histogram fits LDS (else
 * TCONV_E_UNSUPPORTED), and the workspace is required: tconv_workspace_bytes(desc, TCONV_OP_BACKWARD_PARAMS)
 * bytes (else TCONV_E_WORKSPACE).
 */
int tconv_backward_params_recompute(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                                    const float* gy, const float* alpha, const float* beta, const int32_t* idx_min,
                                    const int32_t* idx_max, float* grad_w_min, float* grad_w_max, float* grad_alpha,
                                    float* grad_beta, float* grad_bias, void* workspace, size_t workspace_bytes,
                                    void* hip_stream);

/*
 * Sum-channel layers.  Base operators of Sec. 3.1 for one
 * input channel: MinPlus2d / MaxPlus2d = the minimum / maximum of x + w over the KH x KW window.
 *   mode MIN       layer (i)  MinPlus-Sum-Conv2d:  y = sum over c_in of MinPlus2d(x, w_min)
 *   mode MAX       layer (ii) MaxPlus-Sum-Conv2d:  y = sum over c_in of MaxPlus2d(x, w_max)
 *   mode COMPOUND  y = sum over c_in of ( alpha[c_in, c_out]*MinPlus2d(x, W) + beta[c_in, c_out]*MaxPlus2d(x, W) )
 *   mode PARALLEL  the same with W1 = w_min in the min-plus and W2 = w_max in the max-plus operator
 * (the two-parameter layers of Sec. 3.5 and 3.6; a one-parameter layer is this one with
 * beta = 1 - alpha, and its gradient is grad_alpha - grad_beta).
 *   alpha, beta  fp32 [C_in, C_out] (element c_in*C_out + c_out) or NULL (= all ones); not used in MIN / MAX.
 *   y        [N, C_out, H_out, W_out] in the storage type, overwritten.
 * Padded taps are skipped; a channel's term is fl(fl(alpha*m) + fl(beta*M)); the terms are added in
 * ascending c_in starting from +0, every add rounded to fp32, so the result is reproducible bit for bit.
 * dtype TCONV_BF16 (storage of x, the kernels and y, as in the conventions above: widened exactly, fp32
 * arithmetic, y rounded to nearest-even once, after the channel sum): forward for the geometries of the
 * "sum_tiled3x3" kernel (else TCONV_E_UNSUPPORTED), backward for every geometry; both need a workspace
 * (device, 256-byte aligned) of tconv_sum_workspace_bytes bytes, else TCONV_E_WORKSPACE.  fp32 needs none.
 */
/* Workspace of tconv_sum_forward (backward == 0) or tconv_sum_backward (backward != 0), in *bytes (host). */
int tconv_sum_workspace_bytes(const tconv_desc* desc, int backward, size_t* bytes);

int tconv_sum_forward(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                      const float* alpha, const float* beta, void* y, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/*
 * Backward of tconv_sum_forward.  The window winners are re-computed from x and the kernels (no index
 * tensors are kept; ties: lowest tap of the window).  With g = gy[n, c_out, oh, ow], for every
 * (c_in, c_out, pixel) the min-plus winner (ih*, iw*, tap t*) receives
 *   grad_x[n, c_in, ih*, iw*] += alpha*g,  grad_w_min[c_out, c_in, t*] += alpha*g,  grad_alpha[c_in, c_out] += g*m
 * and the max-plus winner the same with beta, grad_w_max, grad_beta, M (coefficients 1 in MIN / MAX
 * mode; COMPOUND adds both branches into ONE kernel gradient, grad_w_min if non-NULL else grad_w_max).
 * Every gradient pointer may be NULL (not computed), not all of them; grad_alpha / grad_beta must be
 * NULL in MIN / MAX mode.  gy and all gradients fp32 (also with bf16 storage of x and the kernels),
 * overwritten; sums are kept in fp64 inside a workgroup and combined in fp32 in an unspecified order.
 * TCONV_E_UNSUPPORTED: rows longer than about 5000 elements or kernel windows of more than 62 taps.
 */
int tconv_sum_backward(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                       const float* alpha, const float* beta, const float* gy, float* grad_x,
                       float* grad_w_min, float* grad_w_max, float* grad_alpha, float* grad_beta,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* Name of the forward kernel tconv_sum_forward selects: "sum_tiled3x3" or "sum_generic".  Host only. */
const char* tconv_sum_forward_kernel_name(const tconv_desc* desc);

/*
 * Depthwise layers (fp32 only; TCONV_E_UNSUPPORTED for bf16).  The MobileNetV2 variants of Sec. 5 put a
 * tropical layer in place of every depthwise convolution: output channel co reads the single input
 * channel co / mult, mult = C_out / C_in (TCONV_E_SHAPE unless C_out is a multiple of C_in), so the layer
 * is the base operator of Sec. 3.1 per channel, combined as in Sec. 3.5 / 3.6:
 *   m = min over the window of x[n, co / mult] + w_min[co],  M = max over the window of x + w_max[co]
 *   mode MAX: y = M;  MIN: y = m;  COMPOUND (one kernel) / PARALLEL (two): y = alpha[co]*m + beta[co]*M
 *   x [N, C_in, H, W];  w_min, w_max [C_out, 1, KH, KW] (same rules as tconv_forward for which is needed);
 *   alpha, beta fp32 [C_out] or NULL (= ones), ignored in MAX / MIN mode;  y [N, C_out, H_out, W_out].
 * Padded taps are skipped, ties keep the lowest tap t = i*KW + j, every x + w is one rounded fp32 add and
 * y = fl(fl(alpha*m) + fl(beta*M)).  Modes above PARALLEL: TCONV_E_INVAL.
 *   idx      uint8 [N, C_out, H_out, W_out], optional in forward (NULL: inference, nothing saved),
 *            required in backward: low nibble = winning tap of the min-plus branch, high nibble = of the
 *            max-plus branch (0 for a branch the mode does not have).  TCONV_E_UNSUPPORTED if KH*KW > 16.
 */
int tconv_depthwise_forward(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                            const float* alpha, const float* beta, void* y, uint8_t* idx, void* workspace,
                            size_t workspace_bytes, void* hip_stream);

/*
 * Backward of the depthwise layer through the saved winners, with g = gy[n, co, oh, ow]:
 *   grad_x[n, co / mult, ih*, iw*] += alpha[co]*g (min winner), += beta[co]*g (max winner); g itself in
 *   MAX / MIN mode.  Summed in fp32 in a fixed order (a gather: no atomics), overwritten.
 *   grad_w_min[co, t*] += alpha[co]*g, grad_w_max likewise with beta (COMPOUND: both into ONE tensor,
 *   grad_w_min if non-NULL else grad_w_max);  grad_alpha[co] = sum g*m, grad_beta[co] = sum g*M (COMPOUND /
 *   PARALLEL only, TCONV_E_INVAL otherwise; they need x and the kernels, which may be NULL when neither is
 *   requested).  Partial sums in fp32 / fp64 inside a workgroup, fp32 atomics across workgroups; overwritten.
 * Any gradient pointer may be NULL (not computed); at least one must be given.
 */
int tconv_depthwise_backward(const tconv_desc* desc, const void* x, const void* w_min, const void* w_max,
                             const float* alpha, const float* beta, const float* gy, const uint8_t* idx,
                             float* grad_x, float* grad_w_min, float* grad_w_max, float* grad_alpha,
                             float* grad_beta, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Name of the forward kernel tconv_depthwise_forward selects: "dw_tiled3x3", "dw_rows3x3" or "dw_generic".  Host only. */
const char* tconv_depthwise_forward_kernel_name(const tconv_desc* desc);

/*
 * One-dimensional layers (Sec. 3.2, one-dimensional base operators MinPlus1d / MaxPlus1d and layers (iii) - (vi);
 * Sec. 3.3 compound / parallel): the same operator family on x [N, C_in, L] with kernels [C_out, C_in, K] and
 * outputs [N, C_out, L_out], L_out = floor((L + 2*pad - dil*(K-1) - 1)/stride) + 1.  The saved winner is the
 * flattened tap k = c*K + i.  Every argument has the meaning, the rules and the error behaviour of its
 * two-dimensional counterpart above (tconv_out_shape, tconv_workspace_bytes, tconv_forward,
 * tconv_backward_input, tconv_backward_weight, tconv_forward_kernel_name); the Sum-channel and depthwise entry
 * points take a one-dimensional layer as the two-dimensional one with H = 1, KH = 1.
 * These calls only choose a two-dimensional view of the same memory: in general the one-row image
 * [N, C_in, 1, L] with a 1 x K kernel; for K = 3, dil = 1, stride 1 or 2, pad <= 1, C_in a multiple of 3 and a
 * full-window mode the image [N, C_in/3, 3, L] with a 3 x 3 kernel and no vertical padding, whose three rows are
 * three consecutive channels: same candidates, same k, and the tiled 3 x 3 kernels apply.  The one-row image has
 * a forward kernel of its own for long windows over few channels (waveform stems: K >= 8, dil = 1, stride 1, 2,
 * 4 or 8, full-window modes, fp32) and an input-gradient kernel of its own.
 */
typedef struct tconv1d_desc {
  int32_t N, C_in, L;       /* input  [N, C_in, L]                    */
  int32_t C_out, K;         /* kernel [C_out, C_in, K]                */
  int32_t stride, pad, dil;
  int32_t mode;             /* enum tconv_mode                        */
  int32_t dtype;            /* enum tconv_dtype                       */
} tconv1d_desc;

int tconv1d_out_len(const tconv1d_desc* desc, int32_t* L_out);
int tconv1d_workspace_bytes(const tconv1d_desc* desc, int32_t op, size_t* bytes);
int tconv1d_forward(const tconv1d_desc* desc, const void* x, const void* w_min, const void* w_max,
                    const float* alpha, const float* beta, void* y, void* y_min, void* y_max,
                    int32_t* idx_min, int32_t* idx_max, void* workspace, size_t workspace_bytes,
                    void* hip_stream);
int tconv1d_backward_input(const tconv1d_desc* desc, const float* gy, const float* alpha, const float* beta,
                           const int32_t* idx_min, const int32_t* idx_max, float* grad_x, void* workspace,
                           size_t workspace_bytes, void* hip_stream);
int tconv1d_backward_weight(const tconv1d_desc* desc, const float* gy, const float* alpha, const float* beta,
                            const int32_t* idx_min, const int32_t* idx_max, float* grad_w_min,
                            float* grad_w_max, void* workspace, size_t workspace_bytes, void* hip_stream);
const char* tconv1d_forward_kernel_name(const tconv1d_desc* desc);

/*
 * Three-dimensional layers (Sec. 3.2, three-dimensional base operators MinPlus3d / MaxPlus3d and layers (iii) - (vi);
 * Sec. 3.3 compound / parallel), fp32 only (TCONV_E_UNSUPPORTED for bf16): x [N, C_in, D, H, W], kernels
 * [C_out, C_in, KD, KH, KW], outputs [N, C_out, D_out, H_out, W_out]; per axis
 * out = floor((in + 2*pad - dil*(k-1) - 1)/stride) + 1.  The saved winner is the flattened tap
 * k = ((c*KD + a)*KH + i)*KW + j.  Arguments, rules and error behaviour as for tconv_out_shape, tconv_forward,
 * tconv_backward_input and tconv_backward_weight.  Only tconv3d_backward_weight uses a workspace, and optionally:
 * tconv3d_workspace_bytes(desc, TCONV_OP_BACKWARD_WEIGHT) bytes select the deterministic kernel gradient, as in two
 * dimensions; every other op reports 0.
 */
typedef struct tconv3d_desc {
  int32_t N, C_in, D, H, W;      /* input  [N, C_in, D, H, W]            */
  int32_t C_out, KD, KH, KW;     /* kernel [C_out, C_in, KD, KH, KW]     */
  int32_t stride_d, stride_h, stride_w, pad_d, pad_h, pad_w, dil_d, dil_h, dil_w;
  int32_t mode;                  /* enum tconv_mode                      */
  int32_t dtype;                 /* enum tconv_dtype                     */
} tconv3d_desc;

int tconv3d_out_shape(const tconv3d_desc* desc, int32_t* D_out, int32_t* H_out, int32_t* W_out);
int tconv3d_workspace_bytes(const tconv3d_desc* desc, int32_t op, size_t* bytes);
/* "k3x3x3" (3 x 3 x 3 window, stride 1, dilation 1, horizontal padding <= 1, a full-window mode) or "generic3d". */
const char* tconv3d_forward_kernel_name(const tconv3d_desc* desc);
int tconv3d_forward(const tconv3d_desc* desc, const void* x, const void* w_min, const void* w_max,
                    const float* alpha, const float* beta, void* y, void* y_min, void* y_max,
                    int32_t* idx_min, int32_t* idx_max, void* workspace, size_t workspace_bytes,
                    void* hip_stream);
int tconv3d_backward_input(const tconv3d_desc* desc, const float* gy, const float* alpha, const float* beta,
                           const int32_t* idx_min, const int32_t* idx_max, float* grad_x, void* workspace,
                           size_t workspace_bytes, void* hip_stream);
int tconv3d_backward_weight(const tconv3d_desc* desc, const float* gy, const float* alpha, const float* beta,
                            const int32_t* idx_min, const int32_t* idx_max, float* grad_w_min,
                            float* grad_w_max, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Static, NUL-terminated description of a tconv_status value.  Host only. */
const char* tconv_status_string(int status);

/*
 * Name of the forward kernel tconv_forward would launch for this descriptor
 * ("tiled3x3"; "tiled3x3_split" - the same kernel with the input channels split over the waves of a workgroup, chosen
 * where whole rounds of plain workgroups would fill the chip badly; "tiled3x3_f16" - binary16 arithmetic on the packed
 * 16-bit vector instructions; "row1d" - one-row
 * inputs with a window of 8 taps or more; "rowtile" - other windows up to 7 taps wide, fp32; or "generic"), for
 * tests and benchmarks.  Host only; NULL on a bad descriptor.
 */
const char* tconv_forward_kernel_name(const tconv_desc* desc);

#ifdef __cplusplus
}
#endif
#endif /* TCONV_H */
