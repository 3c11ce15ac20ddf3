/* qasr.h -- C ABI of the integer-only ASR encoder library for AMD MI355X (gfx950).
 *
 * The library executes the INT8 inference path of "Integer-only Zero-shot Quantization for
 * Efficient Speech Recognition" (arXiv 2103.16827): every layer is an integer convolution
 * applied directly to the quantised values (Sec. 2.2), with BatchNorm folded into the
 * preceding convolution (Sec. 2.2; at run time an int32 bias), followed by a static
 * per-channel dyadic rescale back to int8 (Sec. 2.1: static quantisation, all scales are
 * inference-time constants), integer ReLU (Sec. 2.2) and an integer residual add.
 *
 * One layer, for b in [0,B), co in [0,Cout), to in [0,Tout):
 *
 *     A  = bias ? bias[co] : 0                                          (int32)
 *     A += sum_{ci, j} x[b, ci, to*stride - pad_left + j*dilation] * w[co, ci', j]
 *                      (terms whose time index falls outside [0,Tin) are 0: symmetric
 *                       quantisation has zero-point 0, Eq. 1; cross-correlation, no flip;
 *                       groups == 1: ci over [0,Cin), ci' = ci;
 *                       depthwise (groups == Cin == Cout): ci = co, ci' = 0)
 *     v  = floor((A * m[co] + 2^(s[co]-1)) / 2^s[co])                   (round half up)
 *     v += residual ? residual[b, co, to] : 0
 *     y[b, co, to] = clamp(v, (flags & QASR_FLAG_RELU) ? 0 : -128, 127)
 *
 * Conventions
 *  - Every tensor pointer is a DEVICE pointer owned by the caller (allocate through any HIP
 *    allocator, e.g. PyTorch-ROCm).  Descriptors, op lists and handles are HOST memory.
 *  - Layout: activations int8 [B, C, T] with T contiguous; weights int8 [Cout, Cin/groups, k]
 *    (PyTorch Conv1d order); bias, m, s int32 [Cout].
 *  - Forward calls only enqueue work on `stream` (a hipStream_t, NULL = default stream) and
 *    return; they never allocate device memory and never synchronise.
 *  - All argument validation happens before the first HIP call, so error paths can be
 *    exercised without a GPU.  Errors are returned as qasr_status; nothing throws or aborts.
 *  - Per-channel constants must satisfy 0 <= m < 2^31 and 1 <= s <= 62; they live in device
 *    memory and are not checked by forward calls (out-of-range values give undefined output
 *    values, never out-of-bounds accesses).
 *  - The int32 accumulator wraps on overflow; the caller guarantees
 *    fan_in * 128 * 128 + |bias| < 2^31.
 *  - y must not overlap x or residual.
 */
#ifndef QASR_H_
#define QASR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  QASR_OK = 0,
  QASR_ERR_NULL = -1,        /* a required pointer is NULL                                  */
  QASR_ERR_SHAPE = -2,       /* a size is < 1, Tout < 1, or a stride is too small           */
  QASR_ERR_PARAM = -3,       /* unknown flag bits, bad slot index, bad op wiring            */
  QASR_ERR_UNSUPPORTED = -4, /* groups not in {1, Cin==Cout}                                */
  QASR_ERR_ALIAS = -5,       /* y overlaps x or residual                                    */
  QASR_ERR_WORKSPACE = -6,   /* workspace NULL, misaligned or too small                     */
  QASR_ERR_HIP = -7          /* a HIP runtime call or kernel launch failed                  */
} qasr_status;

enum {
  QASR_FLAG_RELU = 1u,     /* clamp to [0,127] instead of [-128,127] (integer ReLU, Sec. 2.2)        */
  QASR_FLAG_W_PACKED = 2u  /* `w` was produced by qasr_pack_weights for this descriptor              */
};

typedef struct {
  int32_t B, Cin, Cout, Tin;               /* >= 1; Tout is derived (qasr_conv1d_out_len)             */
  int32_t k, stride, dilation;             /* >= 1                                                    */
  int32_t pad_left, pad_right;             /* >= 0, implicit zeros                                    */
  int32_t groups;                          /* 1 = dense / pointwise; == Cin == Cout = depthwise       */
  int64_t x_batch_stride, y_batch_stride;  /* elements between batch items; 0 => C*T.  A larger
                                              x stride lets a layer read a channel-prefix view.
                                              The residual tensor uses y_batch_stride as well.        */
  uint32_t flags;                          /* QASR_FLAG_*                                             */
} qasr_conv1d_desc;

/* Output length of the integer convolution of Sec. 2.2 under this descriptor (the usual Conv1d
 * geometry with implicit zeros, the zero-point of Eq. 1's symmetric quantiser):
 * Tout = floor((Tin + pad_left + pad_right - dilation*(k-1) - 1) / stride) + 1, or a negative
 * qasr_status if the descriptor is invalid (NULL, sizes < 1, or no output frame).  HOST only. */
int32_t qasr_conv1d_out_len(const qasr_conv1d_desc* d);

/* One integer layer as defined at the top of this file (Sec. 2.2: integer convolution, folded
 * BatchNorm bias, integer ReLU; dyadic rescale and residual as stated above).
 *   x        [B,Cin,Tin]  int8 device (batch stride x_batch_stride)
 *   w        [Cout,Cin/groups,k] int8 device; with QASR_FLAG_W_PACKED the buffer written by
 *            qasr_pack_weights for this descriptor
 *   bias     [Cout] int32 device, or NULL for 0
 *   m, s     [Cout] int32 device
 *   residual [B,Cout,Tout] int8 device or NULL
 *   y        [B,Cout,Tout] int8 device (batch stride y_batch_stride)
 * Pointwise and dense layers run fastest with packed weights; plain weights take slower loads
 * (k == 1) or the generic kernel (k > 1).  Asynchronous on `stream`. */
qasr_status qasr_conv1d_int8(const qasr_conv1d_desc* d, const int8_t* x, const int8_t* w,
                             const int32_t* bias, const int32_t* m, const int32_t* s,
                             const int8_t* residual, int8_t* y, void* stream);

/* The layer with several residual operands (the dense-residual wiring of the Jasper family named
 * in Sec. 3: a block receives the projected inputs of all earlier blocks).  Reading: every operand
 * is int8 at the output scale and shaped like y (same batch stride); all are added to the
 * unsaturated rescaled value, then the one clamp:  v = rescale(A) + sum_r residuals[r].
 * residuals: HOST array of n_res DEVICE pointers, 0 <= n_res <= QASR_MAX_RESIDUALS (else
 * QASR_ERR_PARAM); n_res <= 1 is qasr_conv1d_int8.  Otherwise as qasr_conv1d_int8. */
#define QASR_MAX_RESIDUALS 12
qasr_status qasr_conv1d_int8_multi(const qasr_conv1d_desc* d, const int8_t* x, const int8_t* w,
                                   const int32_t* bias, const int32_t* m, const int32_t* s,
                                   const int8_t* const* residuals, int32_t n_res, int8_t* y,
                                   void* stream);

/* Size in bytes of the packed form of a layer's weights (0 on an invalid descriptor).  HOST only. */
size_t qasr_packed_weight_bytes(const qasr_conv1d_desc* d);

/* Re-orders w [Cout,Cin,k] of a groups == 1 layer with Cin % 64 == 0 into the matrix-core operand
 * order [k][ceil(Cout/16)][Cin/64][64 lanes][16 bytes] (lane 16*gi + n of a block holds output
 * channel 16*co16 + n and input channels 64*kc + 8*gi + 0..7 and 64*kc + 32 + 8*gi + 0..7; rows
 * beyond Cout are zero), so that every wave-wide operand load is 1 KiB of contiguous memory.
 * For every other layer the packed form is the plain form (a copy).  Weights are fixed at
 * inference (Sec. 2.1, static quantisation), so this runs once per layer.  w_packed: device,
 * caller-owned, qasr_packed_weight_bytes(d) bytes, 16-byte aligned.  Asynchronous on `stream`. */
qasr_status qasr_pack_weights(const qasr_conv1d_desc* d, const int8_t* w, int8_t* w_packed,
                              void* stream);

/* The layer epilogue alone on int32 accumulators: what Sec. 2.2 leaves after the integer convolution
 * itself (the folded BatchNorm's bias, the return to int8 at the static output scale of Sec. 2.1 as
 * a dyadic rescale, the residual add, integer ReLU / saturation), i.e. the last four lines of the
 * layer definition at the top of this file with A = acc + bias:
 *   acc [B,C,T] int32 device; bias/m/s [C]; residual, y [B,C,T] int8 device (contiguous).
 * flags: QASR_FLAG_RELU only.  Asynchronous on `stream`. */
qasr_status qasr_requant(const int32_t* acc, int32_t B, int32_t C, int32_t T,
                         const int32_t* bias, const int32_t* m, const int32_t* s,
                         const int8_t* residual, uint32_t flags, int8_t* y, void* stream);

/* Quantiser at the entrance of the path (the paper's Eq. 1 with b = 8):
 *   q[i] = Int(clip(x[i], -alpha, alpha) / S),  S = alpha / 127,  q in [-127, 127].
 * x: n float32 features (device), q: n int8 codes (device), any alignment, same element order
 * (the [B, C, T] layout of the convolutions is just n = B*C*T here).  Single precision
 * throughout: S is computed once in float32, the division is correctly rounded, Int rounds to
 * nearest with ties to even; a NaN feature gives 0.  alpha must be finite and > 0 (and large
 * enough that alpha / 127 does not underflow), else QASR_ERR_PARAM; n == 0 is a no-op; q must
 * not overlap x.  Enqueues one kernel on `stream` and returns. */
qasr_status qasr_quantize(const float* x, size_t n, float alpha, int8_t* q, void* stream);

/* Dequantiser at the exit (the sentence after Eq. 1): x[i] = S * q[i], one float32
 * multiplication per element.  q: n int8 (device), x: n float32 (device); S finite, else
 * QASR_ERR_PARAM; n == 0 is a no-op; x must not overlap q. */
qasr_status qasr_dequantize(const int8_t* q, size_t n, float S, float* x, void* stream);

/* Offline calibration helpers: what turns a float model and calibration activations into the
 * constants the integer layers take (Sec. 2.1: S is pre-computed, static quantisation; Sec. 3.1:
 * the min/max values seen on the calibration data are the clipping range; Sec. 2.2: BatchNorm is
 * folded into the preceding convolution).  The synthetic calibration data itself (Sec. 2.3) is not
 * part of this library.
 *
 * qasr_observe_minmax: running extremes of n float32 values (device), NaNs skipped:
 *   minmax[0] = min(minmax[0], min x),  minmax[1] = max(minmax[1], max x)     (minmax: 2 floats,
 *   device; start them at +inf / -inf; zeros of either sign compare equal).  The symmetric range
 *   of Eq. 1 is then alpha = max(-minmax[0], minmax[1]).  n == 0 is a no-op.  One kernel. */
qasr_status qasr_observe_minmax(const float* x, size_t n, float* minmax, void* stream);

/* The dyadic form of a positive real multiplier M (a layer's S_w S_x / S_y): 2^30 <= m < 2^31 and
 * m 2^-s nearest to M, s = 30 - floor(log2 M).  HOST arithmetic in double precision.
 * QASR_ERR_PARAM if M is not positive and finite or s would leave [1, 62]. */
qasr_status qasr_dyadic_from_scale(double M, int32_t* m, int32_t* s);

/* BatchNorm folding and quantisation of one convolution (all pointers DEVICE).  Float model:
 *   y = gamma (conv(x, w) + conv_bias - mean) / sqrt(var + eps) + beta.        Per channel c:
 *   f = gamma / sqrt(var + eps);  w' = w f;  b' = (conv_bias - mean) f + beta    (float32, each
 *                                                        operation rounded once, nothing fused)
 *   S_w = max|w'| / 127 (1 for an all-zero channel);  q_w = Int(w' / S_w), ties to even  (Eq. 1
 *   per output channel);  bias_q = Int(b' / (S_w S_x)) int32;  (m, s) = dyadic(S_w S_x / S_y)
 *   (double precision).
 * w, q_w: [Cout][per_channel] (per_channel = Cin/groups * k), conv_bias may be NULL (zeros);
 * gamma, beta, mean, var, bias_q, m, s: [Cout]; S_w: [Cout] float32 or NULL; S_x, S_y: the input
 * and output activation scales (finite, > 0); eps finite, >= 0.  A channel whose bias leaves
 * int32 or whose multiplier has no dyadic form gets bias 0 / (m, s) = (0, 1) and adds to
 * *bad_count (device int32 the caller zeroed, or NULL).  q_w must not overlap w.  One kernel. */
qasr_status qasr_fold_bn_quantize(const float* w, const float* conv_bias, const float* gamma,
                                  const float* beta, const float* mean, const float* var, float eps,
                                  int32_t Cout, int64_t per_channel, float S_x, float S_y,
                                  int8_t* q_w, int32_t* bias_q, int32_t* m, int32_t* s, float* S_w,
                                  int32_t* bad_count, void* stream);

/* Integer-only non-linear activations (Sec. 2.2, last sentence; Sec. 3, first paragraph: Sigmoid,
 * Softmax and Swish through second-order polynomials; every result is defined and computed in
 * integers: where a kernel uses a single-precision reciprocal it is only an estimate of a quotient
 * that an exact integer remainder check then corrects).  The paper
 * refers to the integer-only Transformer work it cites for the procedure; as restated here:
 *
 *   exp(x), x <= 0:  x = -z ln2 + p, p in (-ln2, 0], exp(p) ~ 0.3585 (p + 1.353)^2 + 0.344.
 *   On integers r <= 0 at scale S' (x = S' r):
 *       z = floor(-r / q_ln2),  p = r + z q_ln2,  E = floor(((p + q_b)^2 + q_c) / 2^z)  (0 if z > 62)
 *       q_ln2 = floor(ln2 / S'),  q_b = floor(1.353 / S'),  q_c = floor(0.344 / (0.3585 S'^2)),
 *   so that exp(S' r) ~ 0.3585 S'^2 E.  An int8 code q at scale S is refined to r = q 2^u at
 *   S' = S / 2^u first (the floors above are coarse at an 8-bit step).
 *
 * qasr_iexp_init derives the three constants on the HOST in double precision.  Errors:
 * QASR_ERR_NULL; QASR_ERR_PARAM if S is not finite and positive, u is outside [0, 16],
 * q_ln2 < 1 or q_b >= 2^24. */
typedef struct {
  int32_t u;                 /* refinement shift, 0..16                                             */
  int32_t reserved;          /* 0                                                                   */
  int64_t q_ln2, q_b, q_c;   /* 1 <= q_ln2; 0 <= q_b < 2^24; 0 <= q_c < 2^48                        */
} qasr_iexp;
qasr_status qasr_iexp_init(double S, int32_t u, qasr_iexp* c);

/* Elementwise activations int8 -> int8 built on that exponential:
 *   sigmoid code, 15 fraction bits (the two-way softmax of (x, 0)):
 *       E = iexp(-|q| 2^u),  E0 = q_b^2 + q_c,  sigma_q = floor((q >= 0 ? E0 : E) 2^15 / (E0 + E))
 *   QASR_ACT_SIGMOID: v = sigma_q(q)        QASR_ACT_SWISH: v = q sigma_q(q)
 *   QASR_ACT_GLU:     v = a sigma_q(g), a = x[b, c, t], g = x[b, C + c, t]  (x has 2C channels)
 *   y = clamp(floor((v m + 2^(s-1)) / 2^s), -128, 127)   (the layer's dyadic rescale, one (m, s)
 *   per tensor: m 2^-s = S_v / S_y with S_v = 2^-15 for sigmoid, S 2^-15 for swish and GLU).
 * x: [B, C, T] ([B, 2C, T] for GLU) int8 device, batch stride x_batch_stride elements (0 => the
 * dense one); y: [B, C, T] int8 device, batch stride y_batch_stride (0 => C*T).  y may be x
 * itself (same pointer and same batch stride: in place; GLU then overwrites the value half);
 * any other overlap is QASR_ERR_ALIAS.  QASR_ERR_PARAM for an unknown kind, m outside [0, 2^31),
 * s outside [1, 62] or constants outside the ranges above; QASR_ERR_SHAPE for sizes < 1 or a
 * stride smaller than an item.  Enqueues one kernel on `stream` and returns. */
enum { QASR_ACT_SIGMOID = 1, QASR_ACT_SWISH = 2, QASR_ACT_GLU = 3 };
typedef struct {
  int32_t kind;              /* QASR_ACT_*                                                          */
  int32_t m, s;              /* dyadic rescale of the result                                        */
  int32_t reserved;          /* 0                                                                   */
  qasr_iexp e;               /* exponential at the input's scale                                    */
} qasr_act;
qasr_status qasr_act_int8(const qasr_act* a, const int8_t* x, int32_t B, int32_t C, int32_t T,
                          int64_t x_batch_stride, int64_t y_batch_stride, int8_t* y, void* stream);

/* Softmax over the last axis of int32 logits at the scale of `e` (attention scores):
 *   r_i = (q_i - max_j q_j) 2^u,  E_i = iexp(r_i),  y_i = min(127, floor(E_i 2^7 / sum_j E_j)),
 * probabilities at scale 2^-7.  x: [rows, L] int32 device, y: [rows, L] int8 device, dense;
 * 1 <= L <= 16384, rows >= 1, else QASR_ERR_SHAPE; L (q_b^2 + q_c) < 2^55 (the 64-bit row sum
 * cannot overflow), else QASR_ERR_PARAM; y must not overlap x.  Enqueues one kernel on `stream`
 * and returns. */
qasr_status qasr_softmax_int32(const qasr_iexp* e, const int32_t* x, int64_t rows, int32_t L,
                               int8_t* y, void* stream);

/* An encoder is a flat list of layers over numbered activation slots (the evaluated models of
 * Sec. 3 are such lists: QuartzNet, Jasper, Conformer-shaped linear layers).  Slot 0 is the
 * network input `x`; the last op's out_slot is the network output `y`; every other slot
 * lives in the caller's workspace. */
typedef struct {
  qasr_conv1d_desc d;        /* d.x_batch_stride / y_batch_stride as for qasr_conv1d_int8; flags
                                must not contain QASR_FLAG_W_PACKED (create packs by itself)         */
  const int8_t* w;           /* device, plain order; must stay valid while the encoder lives        */
  const int32_t* bias;       /* device or NULL                                                      */
  const int32_t* m;          /* device                                                              */
  const int32_t* s;          /* device                                                              */
  int32_t in_slot;           /* slot read                                                           */
  int32_t res_slot;          /* slot added in the epilogue, or -1                                   */
  int32_t out_slot;          /* slot written; != in_slot, != res_slot, != 0                         */
  const qasr_act* act;       /* HOST, copied by create, or NULL: activation applied in place to the
                                layer's output (after the clamp).  GLU needs an even Cout and
                                leaves its Cout/2 channels in the first half of every batch item
                                of the slot: the next layer reads them as a channel-prefix view
                                (Cin = Cout/2, x_batch_stride = Cout*Tout).                        */
  int32_t n_more_res;        /* further residual operands besides res_slot (dense-residual layers,
                                see qasr_conv1d_int8_multi): 0..QASR_MAX_RESIDUALS-1; needs
                                res_slot >= 0                                                       */
  int32_t more_res_slots[QASR_MAX_RESIDUALS - 1];   /* their slots; shaped like the output          */
} qasr_op;

typedef struct qasr_encoder qasr_encoder; /* opaque host object */

/* Validates the op list (shapes chain through the slots, no op writes a slot it reads, slot 0
 * is never written), sizes the slots, and packs the groups == 1 weights once into device memory
 * owned by the encoder (the only device allocation the library ever makes; it synchronises
 * `stream`-independent, i.e. it blocks until packing is done).  *out is set on QASR_OK. */
qasr_status qasr_encoder_create(const qasr_op* ops, int32_t n_ops, int32_t n_slots,
                                qasr_encoder** out);

/* Which memory the values of the slots live in is the library's choice (slots name values, not
 * addresses): at create time every op's output is given the workspace buffer that has been free
 * longest among those that none of the QASR_SLOT_DEPTH (environment, default 4, 0..16) ops before
 * it read or wrote, a new buffer if there is none.  On this chip a kernel that writes memory which
 * the kernel right before it read under another workgroup-to-XCD mapping runs microseconds
 * longer; the two-slot ping-pong of a plain layer chain does that in every layer (measured: the
 * QuartzNet-15x5 shape at batch 32 takes 1.77 ms per forward with the slots as buffers, 1.49 ms
 * with depth 4).  Depth 0 keeps the caller's slots as the buffers.  The workspace grows by up to
 * `depth` buffers; the depth is lowered until the buffers together take at most 192 MiB (they
 * should stay in the 256 MB memory-side cache together), down to 0.
 *   qasr_plan_slot_buffers: the same plan on bare wiring (HOST only, no device needed; for tests and
 *   diagnostics): in/res/out_slot[n_ops] as in qasr_op (res -1 for none) -> in/res/out_buf[n_ops]
 *   (buffer 0 is the network input) and the number of buffers; QASR_ERR_PARAM for wiring that
 *   qasr_encoder_create would reject or depth outside 0..16. */
qasr_status qasr_plan_slot_buffers(const int32_t* in_slot, const int32_t* res_slot, const int32_t* out_slot,
                                   int32_t n_ops, int32_t n_slots, int32_t depth, int32_t* in_buf,
                                   int32_t* res_buf, int32_t* out_buf, int32_t* n_buffers);

/* Bytes of workspace qasr_encoder_forward needs (all buffers of the plan above except the input
 * and the output, each rounded up to 256 bytes).  Known at create time because every shape and scale of the
 * integer model is static (Sec. 2.1: static quantisation, nothing is sized at inference).  HOST only. */
size_t qasr_encoder_workspace_bytes(const qasr_encoder* e);

/* Runs every op in order on `stream`.  x: [B,Cin,Tin] of the first op's descriptor; y: output
 * of the last op; workspace: device, 256-byte aligned, >= qasr_encoder_workspace_bytes(e).
 * Enqueues n_ops kernels (plus one per activation) and returns; allocates nothing; may be
 * captured into a HIP graph. */
qasr_status qasr_encoder_forward(const qasr_encoder* e, const int8_t* x, int8_t* y,
                                 void* workspace, size_t workspace_bytes, void* stream);

/* qasr_encoder_forward for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * activation slots live in a static device array inside the library, qasr_static_workspace_bytes()
 * = 32 MiB per GPU, held from the moment the library is loaded on that GPU until the process ends.
 * The call allocates nothing and frees nothing; x and y are still the caller's.  An encoder whose
 * qasr_encoder_workspace_bytes exceeds the array gives QASR_ERR_WORKSPACE (before any HIP call).
 * All calls on one GPU share that GPU's array, on every stream: two such forwards that overlap in
 * time on one GPU race (order them on one stream, or use qasr_encoder_forward with workspaces of
 * their own).  The array keeps what the last call left; no slot is read before this forward has
 * written it, so nothing needs clearing.  The device address of the array is looked up at the first
 * call on each GPU (that first call should not happen under stream capture).  Otherwise as
 * qasr_encoder_forward: same kernels, same bits. */
size_t qasr_static_workspace_bytes(void);
qasr_status qasr_encoder_forward_static(const qasr_encoder* e, const int8_t* x, int8_t* y, void* stream);

/* The forward from float features to float outputs: Eq. 1's quantiser on x (float32
 * [B,Cin,Tin], clipping range alpha, see qasr_quantize), the integer encoder, the dequantiser
 * S_out * q on its output (float32 [B,Cout,Tout], see qasr_dequantize).  The int8 copies of input
 * and output live in the workspace too: it must hold qasr_encoder_workspace_bytes_f32(e) bytes
 * (256-byte aligned).  Enqueues n_ops + 2 kernels (plus one per activation) and returns; errors
 * as for the three calls it is made of. */
size_t qasr_encoder_workspace_bytes_f32(const qasr_encoder* e);
qasr_status qasr_encoder_forward_f32(const qasr_encoder* e, const float* x, float alpha, float S_out,
                                     float* y, void* workspace, size_t workspace_bytes,
                                     void* stream);

/* The same forward as a HIP graph: one launch replays all n_ops kernels with the pointers given
 * here (x, y and workspace must stay valid and in place as long as the graph is used; their
 * contents may change between launches).  qasr_encoder_graph_create runs one ordinary forward on
 * a stream of its own (so y and the workspace are written), captures a second one, instantiates
 * it and returns the handle in *out (HOST); it synchronises and allocates, so call it at set-up.
 * qasr_encoder_graph_launch enqueues one replay on `stream` and returns.  The encoder must
 * outlive the graph.  Errors as for qasr_encoder_forward. */
typedef struct qasr_encoder_graph qasr_encoder_graph;
qasr_status qasr_encoder_graph_create(const qasr_encoder* e, const int8_t* x, int8_t* y,
                                      void* workspace, size_t workspace_bytes,
                                      qasr_encoder_graph** out);
qasr_status qasr_encoder_graph_launch(qasr_encoder_graph* g, void* stream);
void qasr_encoder_graph_destroy(qasr_encoder_graph* g);

/* Same as qasr_encoder_forward, but brackets every op with HIP events, waits for completion and
 * writes each op's device time in milliseconds to op_ms[0..n_ops) (HOST memory): the interval
 * between the events around the op minus an equal share of what the inner events cost (the
 * forward is also run once without them in the same call; the op times add up to that run's
 * duration).  For profiling only: it runs the forward twice, synchronises and creates/destroys
 * events. */
qasr_status qasr_encoder_forward_timed(const qasr_encoder* e, const int8_t* x, int8_t* y,
                                       void* workspace, size_t workspace_bytes, void* stream,
                                       float* op_ms);

/* Number of ops, and the name of the kernel family op i is dispatched to (depthwise:
 * "dw_pipe", "dw_mfma"; pointwise: "pw_pipe", "pw_tile"; dense and any other pointwise shape:
 * "conv_pipe", "gemm_mfma"; any shape: "conv_generic"; static storage, NULL if i is out of range). */
int32_t qasr_encoder_num_ops(const qasr_encoder* e);
const char* qasr_encoder_op_kernel(const qasr_encoder* e, int32_t i);
/* 1 if op i's activation (qasr_op.act) is applied inside the layer's own kernel (a unary
 * activation after a layer of the "pw_pipe" or "dw_pipe" family, through a 256-entry table of the
 * activation's int8 outputs built at create time), 0 if it runs as the separate in-place pass or
 * the op has none; -1 if i is out of range.  Same bits either way. */
int32_t qasr_encoder_op_act_fused(const qasr_encoder* e, int32_t i);

/* Runs of layers in one launch (EXPERIMENTAL: only with QASR_TEAM set in the environment when the
 * encoder is created; on encoders with more than about 85 layers in a run the kernel has given wrong
 * utterances now and then, so it is off by default and every layer is a launch of its own).  Where
 * at least 8 utterances (one per XCD) go through a stretch of
 * consecutive pointwise layers of 256 or 512 input channels and stride-1 depthwise layers (the blocks
 * of the QuartzNet family), qasr_encoder_create then plans that stretch as ONE launch of a persistent
 * kernel: every XCD takes its share of the utterances through all of the stretch's layers, with
 * barriers among that XCD's workgroups only, the activations staying in its L2 (every result bit is
 * the same: the layers are the same integer arithmetic).  qasr_encoder_forward, _forward_static,
 * _forward_f32 and the graph entry points use the plan; x and y must then be 16-byte aligned
 * (otherwise every layer is launched by itself).
 *   qasr_encoder_op_in_team: 1 if op i is inside such a run, 0 if not, -1 if i is out of range.
 *   qasr_encoder_forward_layerwise: the forward with every layer as a launch of its own, whatever
 *     the plan (same arguments and errors as qasr_encoder_forward).
 *   qasr_encoder_team_check: after the caller has synchronised the stream: *aborted = 1 if a wait
 *     inside a persistent kernel of the last forward gave up (its waits are bounded: about a second;
 *     the outputs of that forward are then invalid), else 0.  Synchronous (a small copy).
 *   qasr_encoder_forward_team_stamps: the forward with the persistent kernels' clock stamps on;
 *     synchronises and writes to op_us[0..n_ops) (HOST) the time in microseconds between the ends of
 *     consecutive layers inside a run, as seen by the first workgroup of the first XCD (0 for ops
 *     outside runs).  For profiling only. */
int32_t qasr_encoder_op_in_team(const qasr_encoder* e, int32_t i);
qasr_status qasr_encoder_forward_layerwise(const qasr_encoder* e, const int8_t* x, int8_t* y,
                                           void* workspace, size_t workspace_bytes, void* stream);
qasr_status qasr_encoder_team_check(const qasr_encoder* e, int32_t* aborted);
qasr_status qasr_encoder_forward_team_stamps(const qasr_encoder* e, const int8_t* x, int8_t* y,
                                             void* workspace, size_t workspace_bytes, void* stream,
                                             float* op_us);

void qasr_encoder_destroy(qasr_encoder* e);

/* Measured ceilings, for benchmarks that quote a kernel against what this chip sustains and not
 * only against its datasheet (no passage of the paper: measurement support, not part of the path).
 *   qasr_probe_copy: one streaming kernel that copies `bytes` (a multiple of 16; src, dst device,
 *     16-byte aligned, not overlapping; else QASR_ERR_SHAPE / QASR_ERR_ALIAS) -- time it to get the
 *     rate HBM sustains for a read plus a write.
 *   qasr_probe_mfma_i8: one kernel whose waves issue v_mfma_i32_16x16x64_i8 from registers only
 *     (8 independent accumulators per wave, `iters` rounds, 1 <= iters <= 2^24, else
 *     QASR_ERR_PARAM); writes qasr_probe_mfma_i8_outputs() int32 values to `out` (device) and the
 *     number of integer operations (2 per multiply-add) the launch performs to *ops (HOST). */
qasr_status qasr_probe_copy(const void* src, void* dst, size_t bytes, void* stream);
int32_t qasr_probe_mfma_i8_outputs(void);
qasr_status qasr_probe_mfma_i8(int32_t iters, int32_t* out, double* ops, void* stream);

/* Name of the kernel family qasr_conv1d_int8 would dispatch this descriptor to (host-only). */
const char* qasr_conv1d_kernel_name(const qasr_conv1d_desc* d);

const char* qasr_status_string(qasr_status st);

/* The library reads its tuning overrides (environment variables QASR_*: forced tile shapes, kernel
 * families switched off; for sweeps and tests, never needed for correct results) once, at first
 * use.  This reads them again.  HOST only; not to be called while another thread launches. */
void qasr_tuning_reload(void);

/* Name of the HIP error behind the calling thread's most recent QASR_ERR_HIP ("hipSuccess" if
 * there was none).  Static storage. */
const char* qasr_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* QASR_H_ */
