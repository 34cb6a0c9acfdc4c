/*
 * glowmi -- the lowered Convolution / FullyConnected hot path of the Glow paper (arXiv 1805.00907)
 * as hand-written HIP kernels for AMD MI355X (gfx950), behind a plain C ABI.
 *
 * What the calls compute
 * ----------------------
 * After the paper's node-lowering phase (Section 3.4) a network's dense layers are a matrix
 * multiplication followed by a broadcasted add of the bias, and the element-wise operators that
 * follow are executed in the same pass over the data (Section 5.2, operator stacking).  Each entry
 * point below is one such stack: contraction + bias + optional Relu (the max0 instruction of the
 * Section 3.5 listing), in fp32 and in the quantized int8 form of Section 4.
 *
 * Conventions common to every call
 * --------------------------------
 *  - Every tensor pointer is a DEVICE pointer to a dense, row-major buffer owned by the caller.
 *    Inputs are never written.  Outputs must not overlap inputs or the workspace.
 *  - x, w, y (and a, the FC input) must be 16-byte aligned, bias 4-byte aligned (any 4-byte
 *    boundary will do), else GLOWMI_ERR_ALIGN.  bias may be NULL (treated as zeros).
 *  - Calls are asynchronous on `stream`, never synchronise the device and never allocate.
 *  - `workspace` is optional scratch in device memory (16-byte aligned).  With NULL / 0 bytes the
 *    call still computes the same result to the same accuracy; with at least
 *    glowmi_*_workspace_bytes() bytes the library may split the reduction dimension over more
 *    workgroups (small-M layers) and, for large fp32 contractions, repack both operands there (two
 *    fp16 pieces per value, 4 bytes per element: see "Results" below), which is faster.  A workspace
 *    smaller than that figure is not used at all.  The contents on entry do not matter and are
 *    undefined on return.  Two calls that share a workspace must be ordered on one stream.
 *  - Arguments are validated on the host before anything is launched.  On any error nothing is
 *    launched, y is untouched, the status says why and glowmi_last_error() gives a sentence.
 *  - Every tensor must hold fewer than 2^31 elements (GLOWMI_ERR_UNSUPPORTED otherwise).
 *  - Results: fp32 entry points accumulate in fp32 (order unspecified).  Products are fp32 products:
 *    either the fp32 matrix cores' own, or -- large contractions with a workspace -- formed on the
 *    fp16 matrix cores from operands cut into two fp16 pieces each: a tensor (for the input of a 3x3 tile
 *    kernel: each patch a workgroup stages) is scaled by the power of two that brings its largest magnitude
 *    under 2^15 (exact), a scaled value v becomes h1 = fp16(v) and
 *    H2 = fp16((v - h1) * 2^11), 22 significant bits together, and a product is the three piece products
 *    h1 h1' + 2^-11 (h1 H2' + H2 h1'), multiplied exactly and accumulated in fp32; a product is then
 *    within 3 * 2^-22 of |x*y|, a few fp32 roundings.  Either way |result - exact| stays within a few
 *    2^-22 * (|A||W| + |bias|) componentwise for tensors whose elements lie within 2^28 of the largest
 *    magnitude they are scaled by; smaller elements keep 11 significant bits and the product of two such elements,
 *    one from each operand, is dropped, which adds at most 2^-38 * max|A| * max|W| * (reduction length).
 *    Scaling an operand by a power of two scales the result by it and changes nothing else.  With
 *    non-finite inputs the outputs they reach are non-finite (an infinity may come out as NaN); on the
 *    fp16 matrix cores outputs they do not reach may turn into NaN as well, up to every output of the
 *    call (no scale fits a tensor or patch that holds one), but never into wrong finite values.  The int8
 *    entry points are exact integer arithmetic and reproducible bit for bit.
 */
#ifndef GLOWMI_H
#define GLOWMI_H

#include <stddef.h>
#include <stdint.h>

#include <hip/hip_runtime_api.h> /* hipStream_t */

#ifdef __cplusplus
extern "C" {
#endif

typedef enum glowmi_status {
  GLOWMI_OK = 0,
  GLOWMI_ERR_NULL = 1,        /* a required pointer is NULL                                   */
  GLOWMI_ERR_SHAPE = 2,       /* non-positive extent, groups not dividing channels, empty output */
  GLOWMI_ERR_UNSUPPORTED = 3, /* valid request outside what the kernels cover (e.g. >= 2^31 elements) */
  GLOWMI_ERR_ALIGN = 4,       /* pointer alignment                                             */
  GLOWMI_ERR_QUANT = 5,       /* scale not finite and positive, offset outside [-128,127], multiplier out of range */
  GLOWMI_ERR_HIP = 6          /* the HIP runtime refused the launch                            */
} glowmi_status;

/* The element-wise chain fused behind the contraction. */
typedef enum glowmi_act {
  GLOWMI_ACT_NONE = 0,
  GLOWMI_ACT_RELU = 1 /* max(v, 0); on a quantized tensor: max(q, y.offset) (Section 4.3, same-scale max) */
} glowmi_act;

/*
 * Convolution geometry.  Input is <n x h x w x c> (Section 3.5 listing), the filter is
 * [k][r][s][c/groups] = [depth, filter_x, filter_y, channel] (filter-layout figure of Section 5.2),
 * the output is <n x oh x ow x k> with
 *     oh = floor((h + pad_t + pad_b - r) / stride_h) + 1,   ow likewise
 * (the listing's [kernel stride pad depth] parameters; its 28 -> 28 and 28 -> 9 examples).
 * Padding is zero padding of the real-valued input.  No filter flip: output (oh, ow) reads input
 * row oh*stride_h - pad_t + r and column ow*stride_w - pad_l + s.  groups splits input and output
 * channels into that many contiguous blocks (a reading: the paper has no grouped convolution).
 */
typedef struct glowmi_conv_desc {
  int32_t n, h, w, c;
  int32_t k, r, s;
  int32_t stride_h, stride_w;
  int32_t pad_t, pad_l, pad_b, pad_r;
  int32_t groups;
} glowmi_conv_desc;

/* Quantized tensor type of Section 4.1: int8 codes q with value = (q - offset) * scale. */
typedef struct glowmi_qparam {
  float scale;    /* finite, > 0 */
  int32_t offset; /* in [-128, 127] */
} glowmi_qparam;

/* Output extents for a descriptor; returns GLOWMI_ERR_SHAPE if the descriptor is invalid. Host only. */
glowmi_status glowmi_conv_out_shape(const glowmi_conv_desc* d, int32_t* oh, int32_t* ow);

/*
 * fp32 Convolution + bias + activation (Sections 3.1, 3.5, 5.2).
 *   x [n][h][w][c], w [k][r][s][c/groups], bias [k] or NULL, y [n][oh][ow][k], all float, device.
 */
glowmi_status glowmi_conv2d(const float* x, const float* w, const float* bias, float* y,
                            const glowmi_conv_desc* d, glowmi_act act, void* workspace,
                            size_t workspace_bytes, hipStream_t stream);
size_t glowmi_conv2d_workspace_bytes(const glowmi_conv_desc* d);

/*
 * fp32 FullyConnected as lowered in Section 3.4: y = a * w (MatMul), + bias broadcast over rows
 * (BatchedAdd), then the activation.
 *   a [M][K], w [K][N], bias [N] or NULL, y [M][N], all float, device.
 */
glowmi_status glowmi_fc(const float* a, const float* w, const float* bias, float* y, int32_t M,
                        int32_t K, int32_t N, glowmi_act act, void* workspace,
                        size_t workspace_bytes, hipStream_t stream);
size_t glowmi_fc_workspace_bytes(int32_t M, int32_t K, int32_t N);

/*
 * glowmi_fc for callers that cannot allocate and have no workspace to hand over: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and checks as glowmi_fc,
 * and the kernels and results glowmi_fc gives with a workspace that holds its split-reduction partial sums
 * (operands are never repacked here: the fp32 matrix-core kernels are used whatever the size); the partial
 * sums go to a buffer that is part of the library image (a static array in device memory of
 * glowmi_fc_noalloc_max_scratch_bytes() = 8 MiB, one copy per GPU the library is used on, held until
 * the process ends).  The call allocates nothing and calls no allocating routine.
 *   - A shape whose partial sums need more than that is rejected with GLOWMI_ERR_UNSUPPORTED and a message;
 *     nothing is launched.
 *   - Every call on one GPU shares that GPU's buffer: calls must be ordered on one stream (or otherwise
 *     serialised); calls that overlap on one GPU race.  Nothing in the buffer needs to start at zero
 *     (every partial sum is written before it is read), so its stale contents are harmless.
 */
glowmi_status glowmi_fc_noalloc(const float* a, const float* w, const float* bias, float* y, int32_t M,
                                int32_t K, int32_t N, glowmi_act act, hipStream_t stream);
size_t glowmi_fc_noalloc_max_scratch_bytes(void);

/*
 * Quantized Convolution (Section 4.1 tensor type; Section 4.3: the rescale to the output range is
 * folded into the operation, and Relu is a plain integer max because both sides share a scale).
 *   acc   = sum over taps inside the image of (x - xq.offset) * (w - wq.offset)  + bias     (int32)
 *   y     = saturate( round(acc * xq.scale * wq.scale / yq.scale) + yq.offset )  to [lo, 127]
 *   lo    = max(-128, yq.offset) with GLOWMI_ACT_RELU, else -128
 * bias is int32 with scale xq.scale*wq.scale and offset 0 (or NULL).  The multiplier
 * Mr = xq.scale*wq.scale/yq.scale is evaluated in double on the host and applied as an integer:
 * Mr = f * 2^e with f in [0.5, 1); mant = round(f * 2^31) (renormalised if that is 2^31);
 * shift = 31 - e, which must lie in [1, 62] (GLOWMI_ERR_QUANT otherwise);
 *   round(acc * Mr) := (acc * mant + 2^(shift-1)) >> shift    (64-bit, arithmetic shift: ties go up).
 * The int32 accumulator must not overflow.  A code minus its offset reaches 128 + |offset| in magnitude
 * (255 at the extreme offsets), so the sum of products of a reduction of depth D = r*s*c/groups is
 * bounded by D * (128 + |x.offset|) * (128 + |w.offset|); the call is rejected with
 * GLOWMI_ERR_UNSUPPORTED when that bound exceeds 2^31 - 2^27 or when D > 65535.  The 2^27 left over is
 * room for |bias| plus the rescaled addend of a chain: contents of device memory the host cannot see,
 * so keeping them inside it is the caller's contract (an overflow is not detected on the device).
 *   x int8 [n][h][w][c], w int8 [k][r][s][c/groups], bias int32 [k], y int8 [n][oh][ow][k], device.
 */
glowmi_status glowmi_qconv2d(const int8_t* x, glowmi_qparam xq, const int8_t* w, glowmi_qparam wq,
                             const int32_t* bias, int8_t* y, glowmi_qparam yq,
                             const glowmi_conv_desc* d, glowmi_act act, void* workspace,
                             size_t workspace_bytes, hipStream_t stream);
size_t glowmi_qconv2d_workspace_bytes(const glowmi_conv_desc* d);

/*
 * Quantized FullyConnected: the Section 3.4 lowering on Section 4.1 tensors, same arithmetic as
 * glowmi_qconv2d.   a int8 [M][K], w int8 [K][N], bias int32 [N] or NULL, y int8 [M][N], device.
 */
glowmi_status glowmi_qfc(const int8_t* a, glowmi_qparam aq, const int8_t* w, glowmi_qparam wq,
                         const int32_t* bias, int8_t* y, glowmi_qparam yq, int32_t M, int32_t K,
                         int32_t N, glowmi_act act, void* workspace, size_t workspace_bytes,
                         hipStream_t stream);
size_t glowmi_qfc_workspace_bytes(int32_t M, int32_t K, int32_t N);

/*
 * The element-wise chain behind the contraction when one of its links has a tensor operand.
 * Section 5.2 (operator stacking): consecutive data-parallel operators work on one memory location one
 * after the other instead of each making its own pass; the code-generation figure of Section 5.3 shows
 * an element-wise Add fused with a max.  Here the chain is
 *     bias add  ->  + addend (optional)  ->  act
 * i.e. y = act(contraction + bias + addend): the tail of a residual block in one pass.
 *   addend    device tensor with the shape, layout and element type of y (float for glowmi_conv2d_chain,
 *             int8 for glowmi_qconv2d_chain), 16-byte aligned; NULL removes the link (the call is then
 *             glowmi_conv2d / glowmi_qconv2d).  addend may be y itself (in-place accumulate into the
 *             residual); any other overlap with y is not allowed.
 *   addend_q  quantized form only: the addend's scale/offset.  Following Section 4.3 (a rescale node in
 *             front of the add, folded into the producer) the addend is brought to the accumulator's
 *             scale x.scale*w.scale before the single requantize:
 *                 acc += round((addend - addend_q.offset) * Mres),  Mres = addend_q.scale / (x.scale*w.scale)
 *             with Mres evaluated in double and applied as mant * 2^-shift exactly like the output
 *             multiplier (31-bit mantissa, ties go up); the shift must lie in [12, 62], i.e. Mres < 2^19,
 *             so that the term of the largest code difference (255) stays below 2^27
 *             (GLOWMI_ERR_QUANT otherwise).  The sum must still fit int32 (caller's contract).
 */
typedef struct glowmi_chain {
  const void* addend;
  glowmi_qparam addend_q;
  glowmi_act act;
} glowmi_chain;

/* glowmi_conv2d with the chain above.  chain must not be NULL.  Workspace as for glowmi_conv2d. */
glowmi_status glowmi_conv2d_chain(const float* x, const float* w, const float* bias, float* y,
                                  const glowmi_conv_desc* d, const glowmi_chain* chain, void* workspace,
                                  size_t workspace_bytes, hipStream_t stream);
/* glowmi_qconv2d with the chain above.  chain must not be NULL.  Workspace as for glowmi_qconv2d. */
glowmi_status glowmi_qconv2d_chain(const int8_t* x, glowmi_qparam xq, const int8_t* w, glowmi_qparam wq,
                                   const int32_t* bias, int8_t* y, glowmi_qparam yq,
                                   const glowmi_conv_desc* d, const glowmi_chain* chain, void* workspace,
                                   size_t workspace_bytes, hipStream_t stream);

/*
 * Filters transformed ahead of time.  Section 5.3 (the filter-layout figure and the three kinds of
 * convolution): the weights of a layer are constants, so the compiler changes their memory layout once, at
 * compile time, into the form the selected convolution reads.  The form here is the one every fp32 kernel on
 * the fp16 matrix cores reads: the weights scaled by the power of two that follows from their largest
 * magnitude and cut into two fp16 pieces each (see "Results" above), kept as two planes of fp16, a convolution
 * filter in its own [k][r][s][c/groups] order, a FullyConnected weight transposed to [N][K], followed by a
 * trailer that holds the largest magnitude.  glowmi_conv2d / glowmi_fc make these planes inside every call
 * (in the workspace); a caller that keeps the weights fixed makes them once and hands them to the *_packed
 * entry points, which are otherwise the same calls: bit for bit the same results where the same kernel serves
 * both, and within the accuracy stated at the top where a layer takes the fp16 kernels only once its weights
 * need no cutting.
 *   glowmi_conv2d_filter_planes_bytes / glowmi_fc_filter_planes_bytes
 *       bytes of the planes (4 per weight, rounded up to 256, plus 4096 of trailer), or 0 when the shape has no plane form
 *       (c/groups, or K of a FullyConnected layer, not a multiple of 8; more than 2^28 weights; bad descriptor).
 *   glowmi_conv2d_pack_filter / glowmi_fc_pack_filter
 *       write the planes of `w` to `planes` (device, 16-byte aligned, planes_bytes >= the figure above;
 *       GLOWMI_ERR_UNSUPPORTED when that figure is 0, GLOWMI_ERR_SHAPE when planes_bytes is too small).
 *       Asynchronous on `stream`; `w` is not written.
 *   glowmi_conv2d_packed / glowmi_fc_packed
 *       glowmi_conv2d_chain / glowmi_fc with `w_planes` = the planes made from this very `w` for this very
 *       descriptor (or K, N); the library cannot check that and results are undefined otherwise.  `w` itself
 *       is still required: layers that take a kernel which does not read planes use it, and ignore w_planes.
 *       w_planes = NULL makes the call the plain one.  chain of glowmi_conv2d_packed must not be NULL.
 *       GLOWMI_ERR_ALIGN for w_planes not 16-byte aligned, GLOWMI_ERR_UNSUPPORTED for w_planes != NULL on a
 *       shape without a plane form.
 *   glowmi_conv2d_packed_workspace_bytes / glowmi_fc_packed_workspace_bytes
 *       the workspace of a *_packed call with w_planes != NULL.  On the same kernel it is the plain call's
 *       minus the weights' planes (a 3x3 layer on the tile kernels needs none at all); a layer that only pays
 *       for the fp16 kernels once its weights need no cutting (a FullyConnected of a few hundred rows) takes
 *       them here and not in the plain call, and then asks for room for the input's planes.
 */
size_t glowmi_conv2d_filter_planes_bytes(const glowmi_conv_desc* d);
glowmi_status glowmi_conv2d_pack_filter(const float* w, const glowmi_conv_desc* d, void* planes,
                                        size_t planes_bytes, hipStream_t stream);
size_t glowmi_conv2d_packed_workspace_bytes(const glowmi_conv_desc* d);
glowmi_status glowmi_conv2d_packed(const float* x, const float* w, const void* w_planes, const float* bias,
                                   float* y, const glowmi_conv_desc* d, const glowmi_chain* chain,
                                   void* workspace, size_t workspace_bytes, hipStream_t stream);
size_t glowmi_fc_filter_planes_bytes(int32_t K, int32_t N);
glowmi_status glowmi_fc_pack_filter(const float* w, int32_t K, int32_t N, void* planes, size_t planes_bytes,
                                    hipStream_t stream);
size_t glowmi_fc_packed_workspace_bytes(int32_t M, int32_t K, int32_t N);
glowmi_status glowmi_fc_packed(const float* a, const float* w, const void* w_planes, const float* bias,
                               float* y, int32_t M, int32_t K, int32_t N, glowmi_act act, void* workspace,
                               size_t workspace_bytes, hipStream_t stream);

/*
 * General element-wise chains.  Section 5.2: whenever data-parallel operators follow one another they
 * are stacked and executed in one pass over the data, whatever they are; the fixed chain above is the
 * most common instance.  Here the caller gives the run of operators that follows the contraction as a
 * list of up to GLOWMI_MAX_CHAIN_OPS ops, applied IN ORDER to every output element after the bias:
 *     GLOWMI_OP_ADD_TENSOR  v += tensor[element]        tensor: device, shape/layout/type of y, 16-byte
 *                                                       aligned; may be y itself, no other overlap with y
 *     GLOWMI_OP_MUL_SCALAR  v *= a
 *     GLOWMI_OP_MAX_SCALAR  v  = max(v, a)              (a = 0: Relu)
 *     GLOWMI_OP_CLIP        v  = min(max(v, a), b)      a <= b
 * There is no separate activation: n_ops = 0 is the bare contraction + bias.
 *
 * fp32 (glowmi_conv2d_chainv): each op is evaluated in fp32 on the accumulator in registers; a, b must
 * not be NaN.
 *
 * Quantized (glowmi_qconv2d_chainv), a reading, since the paper only says that rescale nodes convert
 * between ranges (Section 4.3): the chain runs on the int32 accumulator, whose real value is acc * s with
 * s = x.scale * w.scale at first (formed in double).
 *     MUL_SCALAR (a > 0 required)  s becomes s * a; the integer is untouched (exact)
 *     MAX_SCALAR / CLIP            the bounds are put on the accumulator's grid, T = floor(a / s + 0.5)
 *                                  saturated to int32, then plain integer max / min
 *     ADD_TENSOR                   acc += round((tensor - tensor_q.offset) * tensor_q.scale / s), multiplier
 *                                  in the mantissa/shift form of glowmi_chain (shift in [12, 62])
 *     at the end                   y = saturate(round(acc * s_final / y.scale) + y.offset) to [-128, 127]
 * Lists that are one of the fixed shapes ({}, {max 0}, {add}, {add, max 0}) give exactly the results of
 * glowmi_(q)conv2d(_chain) and take the same kernels; any other list runs on the generic tiled kernels.
 * Errors: GLOWMI_ERR_UNSUPPORTED for n_ops > GLOWMI_MAX_CHAIN_OPS or an unknown kind, GLOWMI_ERR_NULL /
 * GLOWMI_ERR_ALIGN for a tensor, GLOWMI_ERR_QUANT for scalars or scales outside the stated ranges
 * (quantized) and GLOWMI_ERR_SHAPE for NaN scalars or a > b (fp32).  Workspace: at least
 * glowmi_(q)conv2d_chainv_workspace_bytes() for the same descriptor and list, or NULL.
 */
typedef enum glowmi_op_kind {
  GLOWMI_OP_ADD_TENSOR = 1,
  GLOWMI_OP_MUL_SCALAR = 2,
  GLOWMI_OP_MAX_SCALAR = 3,
  GLOWMI_OP_CLIP = 4
} glowmi_op_kind;

#define GLOWMI_MAX_CHAIN_OPS 4

typedef struct glowmi_chain_op {
  glowmi_op_kind kind;
  float a, b;              /* scalars of MUL / MAX / CLIP                                   */
  const void* tensor;      /* ADD_TENSOR operand                                            */
  glowmi_qparam tensor_q;  /* quantized form: its scale/offset                              */
} glowmi_chain_op;

glowmi_status glowmi_conv2d_chainv(const float* x, const float* w, const float* bias, float* y,
                                   const glowmi_conv_desc* d, const glowmi_chain_op* ops, int32_t n_ops,
                                   void* workspace, size_t workspace_bytes, hipStream_t stream);
size_t glowmi_conv2d_chainv_workspace_bytes(const glowmi_conv_desc* d, const glowmi_chain_op* ops, int32_t n_ops);
glowmi_status glowmi_qconv2d_chainv(const int8_t* x, glowmi_qparam xq, const int8_t* w, glowmi_qparam wq,
                                    const int32_t* bias, int8_t* y, glowmi_qparam yq, const glowmi_conv_desc* d,
                                    const glowmi_chain_op* ops, int32_t n_ops, void* workspace,
                                    size_t workspace_bytes, hipStream_t stream);
size_t glowmi_qconv2d_chainv_workspace_bytes(const glowmi_conv_desc* d, const glowmi_chain_op* ops, int32_t n_ops);

/*
 * A straight sequence of convolution layers (with their stacked chains) run back to back on one
 * stream out of ONE caller-provided arena.  The paper's low-level IR marks the lifetime of every
 * activation (alloc/dealloc, Section 3.5) and all of them are then allocated statically in a single
 * buffer (Section 5.3); in a straight sequence two alternately used regions hold every intermediate.
 * The arena also carries the split-reduction workspace.  Layer i reads layer i-1's output (layer 0
 * reads x); the last layer writes y.  add_input != 0 adds the sequence input x (an identity shortcut;
 * shapes must match) in that layer's chain before its activation: 1x1 -> 3x3 -> 1x1 with add_input on
 * the last layer is a residual bottleneck block in three launches.  Nothing is synchronised or
 * allocated, so the whole sequence can be captured in a HIP graph (fewer launches is the other gain
 * the paper names for stacking on GPUs, Section 5.2).
 *   w, bias: device pointers, float / float for glowmi_seq_conv2d, int8 / int32 for glowmi_seq_qconv2d.
 *   wq, yq:  quantized form only: the filter's and the layer output's scale/offset; a layer's input
 *            type is the previous layer's yq (xq for layer 0); the shortcut is x with xq.
 *   arena:   device memory, 16-byte aligned, at least glowmi_seq_arena_bytes(); contents undefined after.
 * Errors: GLOWMI_ERR_SHAPE when consecutive layers (or the shortcut) do not fit, GLOWMI_ERR_ALIGN when
 * the arena is too small or misaligned, otherwise the status of the failing layer call.
 */
typedef struct glowmi_seq_layer {
  glowmi_conv_desc desc;
  const void* w;
  const void* bias;
  glowmi_qparam wq, yq;
  glowmi_act act;
  int32_t add_input;
} glowmi_seq_layer;

size_t glowmi_seq_arena_bytes(const glowmi_seq_layer* layers, int32_t n, int32_t quantized);
glowmi_status glowmi_seq_conv2d(const float* x, const glowmi_seq_layer* layers, int32_t n, float* y, void* arena,
                                size_t arena_bytes, hipStream_t stream);
glowmi_status glowmi_seq_qconv2d(const int8_t* x, glowmi_qparam xq, const glowmi_seq_layer* layers, int32_t n,
                                 int8_t* y, void* arena, size_t arena_bytes, hipStream_t stream);

/*
 * Conversions at the borders of the integer islands of Section 4.2, on the device, so that quantized
 * layers can be chained without the host.  count elements, device pointers, 16-byte aligned, the
 * output must not overlap the input (except glowmi_rescale, which may run in place: out == in).
 *   glowmi_quantize    q = saturate(round(v / scale) + offset), the inverse of the Section 4.1 formula;
 *                      the quotient is formed in double and rounded to nearest, ties to even.
 *   glowmi_dequantize  v = (q - offset) * scale                                   (Section 4.1).
 *   glowmi_rescale     the rescale node of Section 4.3: the same real values on another scale/offset,
 *                      out = saturate(round((in - from.offset) * from.scale / to.scale) + to.offset), the
 *                      multiplier applied in the integer form of glowmi_qconv2d (ties go up).
 */
glowmi_status glowmi_quantize(const float* x, int8_t* q, size_t count, glowmi_qparam qp, hipStream_t stream);
glowmi_status glowmi_dequantize(const int8_t* q, float* x, size_t count, glowmi_qparam qp, hipStream_t stream);
glowmi_status glowmi_rescale(const int8_t* in, glowmi_qparam from, int8_t* out, glowmi_qparam to, size_t count,
                             hipStream_t stream);

/*
 * Host-side, compile-time transformation (the paper merges batch normalization into the preceding
 * convolution before code generation, Section 5.3): fold y = gamma * (conv - mean) / sqrt(var + eps)
 * + beta into the filter and bias,
 *     w_out[k][...] = w[k][...] * gamma[k] / sqrt(var[k] + eps)
 *     bias_out[k]   = (bias[k] - mean[k]) * gamma[k] / sqrt(var[k] + eps) + beta[k]
 * so that glowmi_conv2d on (w_out, bias_out) computes convolution + batch normalization.
 * ALL POINTERS ARE HOST POINTERS.  w, w_out: k filters of elems_per_filter floats (r*s*c/groups);
 * bias may be NULL (zeros); w_out may be w and bias_out may be bias.  Evaluated in double, rounded once.
 */
glowmi_status glowmi_fold_batchnorm(const float* w, const float* bias, const float* gamma, const float* beta,
                                    const float* mean, const float* var, float eps, int32_t k,
                                    int64_t elems_per_filter, float* w_out, float* bias_out);

/* Host helper: the integer multiplier/shift the quantized entry points derive from three scales. */
glowmi_status glowmi_requant_params(float x_scale, float w_scale, float y_scale, int32_t* mant,
                                    int32_t* shift);

/* Host helper: mant/shift of Mres = r_scale / (x_scale * w_scale), the addend rescale of glowmi_chain. */
glowmi_status glowmi_rescale_params(float r_scale, float x_scale, float w_scale, int32_t* mant,
                                    int32_t* shift);

/*
 * Tuning knobs for experiments and tests: force a tile variant, or lower the size threshold of a
 * specialised kernel so that a small test shape reaches it.  name is the knob's name without prefix
 * (e.g. "F32_TILE", "I8_K3_MIN_BLOCKS"); the same knobs are seeded ONCE, at the library's first use,
 * from environment variables GLOWMI_<name>.  Every setting computes the same result (int8: bit for
 * bit; fp32: within the accuracy stated at the top of this file, the kernels differ in rounding order and
 * in which matrix cores form the products: "F32_P3", "F32_K3", "F32_K3C64", "F32_PW_BF16",
 * "F32_SMALLC_BF16" (the first-layer kernel's piece-product form, whatever the pieces' type) = 0 keep a layer on the
 * fp32 matrix cores; "F32_K3V" = 0 keeps the 3x3 kernel on its
 * fixed 16 x 16 pixel tile and "F32_K3_TH" / "F32_K3_TW" force a tile of that many rows / columns, at most 256
 * pixels, 64 columns and (rows + 2) x (columns + 4) <= 360, else ignored; "DW" = 0 keeps depthwise 3x3 layers,
 * groups == c == k, off their own kernel, 2 / 3 make its threads walk one / two output rows at a time); only the
 * choice of kernel changes.
 * glowmi_tuning_reset() returns every knob to "the planner's own choice" (it does not re-read the
 * environment).  Not thread-safe against concurrent launches that should see a consistent setting.
 * GLOWMI_ERR_UNSUPPORTED for an unknown name.
 */
glowmi_status glowmi_tuning_set(const char* name, int32_t value);
void glowmi_tuning_reset(void);

const char* glowmi_status_string(glowmi_status s);
/* Message of the last failing call on the calling thread ("" if none). Valid until the next call. */
const char* glowmi_last_error(void);
/* Name of the kernel variant the last successful call on this thread launched (for profiling). */
const char* glowmi_last_variant(void);

#ifdef __cplusplus
}
#endif
#endif /* GLOWMI_H */
