/*
 * libeoq -- the full-int8 training step of a Fixup residual CNN without BatchNorm
 * (EOQ framework, arXiv 2105.13890) for AMD MI355X (gfx950).
 *
 * C ABI.  No exceptions cross this boundary; every call returns an eoq_status code.
 *
 * Conventions shared by all calls
 *   - Every tensor / slot pointer is a DEVICE pointer owned by the caller, unless a
 *     parameter is explicitly marked "host".  The library never allocates or frees
 *     tensor memory and never synchronises: work is enqueued on the context's HIP
 *     stream.  The descriptor structs themselves are host memory, read during the call.
 *   - Codes.  Bit width k = 8 everywhere (Section 5.1).  A quantised value is an integer
 *     code times a power of two.  Forward tensors use fixed grids: int8 activations,
 *     int8 weights and the int32 scalar codes (bias, multiplier) have value code * 2^-7;
 *     a convolution accumulator has value acc * 2^-14.  Backward tensors (errors,
 *     gradients) carry one exponent per tensor, value = code * 2^E, with E held in a
 *     device-resident int32 "exponent slot" so that no call needs a host round trip.
 *   - R(.) of Eq.5 rounds to nearest, ties to even.
 *   - Layouts: activations / errors NHWC int8; weights KRSC int8; accumulators int32 in
 *     the layout of the tensor they become.  P, Q are the output height / width,
 *     P = (H + 2*pad - R) / stride + 1.
 *   - Statistics slots.  "absmax" slots are int32 holding max|v| (combined with atomic
 *     max), "sum" slots are int64 (combined with atomic add).  The caller zeroes them
 *     (eoq_fill_zero) before the first producer of a step.
 *   - Shapes the MFMA kernels accept: K % 16 == 0 (output channels).  Input channels
 *     C % 16 == 0 run the implicit-GEMM path directly; any other C goes through an
 *     explicit, zero-padded im2col held in the workspace.
 *   - Errors that can only be seen on the device (an accumulator leaving int32, an
 *     exponent gap too large to align) set bits in a device status word, read with
 *     eoq_status().
 */
#ifndef EOQ_H
#define EOQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum eoq_status_code {
    EOQ_OK = 0,
    EOQ_ERR_ARG = 1,       /* null pointer / bad enum / bad size */
    EOQ_ERR_SHAPE = 2,     /* shape outside what the kernels accept */
    EOQ_ERR_WORKSPACE = 3, /* workspace missing or too small */
    EOQ_ERR_RANGE = 4,     /* device status word reported a range violation */
    EOQ_ERR_HIP = 5        /* a HIP runtime call failed */
};

enum eoq_flag_bits {
    EOQ_FLAG_ACC_OVERFLOW = 1, /* a weight-gradient element does not fit int32, or a wide shortcut value is outside
                                * the range the forward epilogue computes exactly (see eoq_epilogue) */
    EOQ_FLAG_EXP_GAP = 2,      /* two exponents too far apart to align exactly */
    EOQ_FLAG_NONFINITE = 4,    /* eoq_quantize met a NaN or an infinity */
    EOQ_FLAG_SHIFT_RANGE = 8   /* an update would need a left shift beyond 24 bits */
};

typedef struct eoq_ctx eoq_ctx;

/* Create a context bound to `hip_stream` (a hipStream_t; NULL = the default stream) on the
 * current device.  Allocates device memory that the context owns until eoq_destroy: 512 bytes for the status
 * word and the call-internal statistics slots, and 8 MiB (2^20 int64) for the per-wave partial sums that
 * eoq_relu_bwd_recompute and the speculative form of eoq_conv_bwd_data_sq stage between their kernels (calls whose
 * records do not fit fall back to atomics / to the exact path).  Calls on one context are ordered by its stream;
 * two contexts share nothing. */
int eoq_create(eoq_ctx **ctx, void *hip_stream);
int eoq_destroy(eoq_ctx *ctx);
const char *eoq_strerror(int code);
/* Synchronise the stream, copy the device status word to *flags (host) and clear it.
 * Returns EOQ_ERR_RANGE when any bit was set. */
int eoq_status(eoq_ctx *ctx, uint32_t *flags);

/* Speculation statistics (see eoq_bwd_fuse::spec_state and eoq_maxpool_bwd_sq): synchronises the stream and
 * returns how many speculative calls on this context, since it was created, found their exponent right (*hits:
 * one evaluation, no intermediate) and how many had to be redone the exact way (*misses).  Either may be NULL. */
int eoq_spec_counters(eoq_ctx *ctx, int64_t *hits, int64_t *misses);

/* Convolution geometry.  Input N x H x W x C, filters K x R x S x C. */
typedef struct eoq_conv_desc {
    int32_t N, H, W, C;
    int32_t K, R, S;
    int32_t stride, pad;
} eoq_conv_desc;

enum eoq_op { EOQ_OP_CONV_FWD = 0, EOQ_OP_CONV_BWD_DATA = 1, EOQ_OP_CONV_BWD_WEIGHT = 2 };
/* Bytes of workspace the convolution call `op` needs for `desc` (0 is possible). */
size_t eoq_workspace_bytes(const eoq_conv_desc *desc, int op);

/* Set `bytes` (multiple of 4) of device memory to zero with a kernel (safe under graph capture). */
int eoq_fill_zero(eoq_ctx *ctx, void *ptr, size_t bytes);

/* ---- quantisers on real input: Section 3.2.2, Eq.5 (Q), Eq.6 (CQ), Eq.7 (SQ) ---------------
 * y = x * 2^pre_shift (exact), then
 *   EOQ_Q : q is int32[n], code = R(128 y)
 *   EOQ_CQ: q is int8[n],  code = clamp(R(128 y), -127, 127)
 *   EOQ_SQ: q is int8[n],  scale = 2^R(log2 max|y|), code = clamp(R(128 y / scale)); *exp_slot = R(..) - 7,
 *           so that value = code * 2^(*exp_slot).  An all-zero tensor gives codes 0 and exponent 0.
 *           R(log2 max) is taken from the float's exponent and mantissa, never through a log.
 * exp_slot is ignored (may be NULL) for Q and CQ.  Non-finite input sets EOQ_FLAG_NONFINITE. */
enum eoq_qmode { EOQ_Q = 0, EOQ_CQ = 1, EOQ_SQ = 2 };
int eoq_quantize(eoq_ctx *ctx, const float *x, size_t n, int mode, int pre_shift, void *q, int32_t *exp_slot);

/* ---- forward epilogue of one Fixup layer: Eq.2 lines x2..x5, Eq.9, Eq.10 ---------------------
 *   t = R(acc / 128)                               Q_a1: grid 2^-14 -> 2^-7, not clamped
 *   z = gamma * t + 128 * b_post + 128 * skip      grid 2^-14; gamma NULL = 128 (one), b_post NULL = 0
 *   relu = 1:  y = clamp(R(max(z,0) / 128), 0, 127)   Q_a2;  mask bit = [z > 0]
 *              u_next = clamp(y + b_next_pre, -127, 127)   the next layer's x1 (Eq.2 line 2)
 *   relu = 0:  only t_wide is produced (1x1 shortcut convolution)
 * skip: the residual input of the block, NPQK layout, int8 codes (skip_is_wide = 0) or wide codes on
 * the 2^-7 grid: int32 (skip_is_wide = 1; |value| < 2^22, which every Q_a1 output of a convolution with
 * R*S*C < 33000 satisfies -- a larger value sets EOQ_FLAG_ACC_OVERFLOW and the outputs of the call are
 * not valid) or int16 (skip_is_wide = 2).  t_wide receives t as int32, or as int16 when t_wide_is_16 = 1
 * (t_wide then points to int16_t[n]; the caller chooses this when 127^2 * R*S*C / 128 < 2^15, i.e. R*S*C <= 260;
 * a value that does not fit sets EOQ_FLAG_ACC_OVERFLOW).  The 16-bit forms halve the traffic of a shortcut
 * convolution's output; the values are the same.  Outputs that are NULL are not written.  relu_mask_bits holds one
 * bit per output element: bit (i % 32) of word (i / 32), i = linear NPQK index.  Scalars are read from
 * device memory at kernel time. */
typedef struct eoq_epilogue {
    const int32_t *gamma;
    const int32_t *b_post;
    const void *skip;
    int32_t skip_is_wide;
    int32_t relu;
    const int32_t *b_next_pre;
    int8_t *y;
    int8_t *u_next;
    uint32_t *relu_mask_bits;
    int32_t *t_wide;
    int32_t t_wide_is_16;
} eoq_epilogue;

/* ---- Eq.2 line x1: u = clamp(a + b_pre, -127, 127) on int8 codes (b_pre: device scalar code) -- */
int eoq_pre_bias(eoq_ctx *ctx, const int8_t *a, size_t n, const int32_t *b_pre, int8_t *u);

/* ---- forward convolution: Eq.2, conv(x1) -----------------------------------------------------
 * acc[n,p,q,k] = sum_{r,s,c} u[n, p*stride+r-pad, q*stride+s-pad, c] * w[k,r,s,c]  (zero padding).
 * When `ep` is non-NULL the epilogue above is fused and `acc` may be NULL; when `acc` is non-NULL
 * the raw int32 accumulators are stored as well.  ws: see eoq_workspace_bytes (only needed when
 * C % 16 != 0). */
int eoq_conv_fwd(eoq_ctx *ctx, const eoq_conv_desc *desc, const int8_t *u, const int8_t *w, int32_t *acc,
                 const eoq_epilogue *ep, void *ws, size_t ws_bytes);

/* ---- backward-data convolution: Eq.3 line e4 before Q_e ---------------------------------------
 * d_acc[n,h,x,c] = sum_{k,r,s} e[n,p,q,k] * w[k,r,s,c] over the (p,q) with h = p*stride+r-pad,
 * x = q*stride+s-pad.  max|d_acc| is atomically max-combined into *absmax_slot (non-NULL). */
int eoq_conv_bwd_data(eoq_ctx *ctx, const eoq_conv_desc *desc, const int8_t *e, const int8_t *w,
                      int32_t *d_acc, int32_t *absmax_slot, void *ws, size_t ws_bytes);

/* ---- backward-data convolution with Q_e fused: Eq.3 line e4 = Q_e(e3 * w) (Eq.11) ---------------
 * Same result as eoq_conv_bwd_data followed by eoq_requant_epilogue(EOQ_RQ_SQ_ACC), without the int32
 * round trip through memory and with ONE evaluation of the convolution.  The scale quantiser needs max|d|
 * before any element can be coded, so the convolution kernel max-combines max|d| into *absmax_slot (which
 * the caller zeroed) and stores every sum as a 16-bit block-scaled value in the workspace (top 14 bits
 * relative to the tile's own maximum plus a sticky bit); a second, streaming kernel rounds these to
 * e4 = clamp(R(d * 2^(7-r))), r = R(log2 max|d|) -- exactly, because the rounding position is at least 6 bits
 * above any dropped bit -- and sets *exp_out = *exp_in + exp_in_off + r - 7 (all-zero d: codes 0, exponent
 * *exp_in + exp_in_off).  When sum_out is non-NULL, *sum_out += sum of the e4 codes (the bias gradient of Eq.4).
 * `fuse` (may be NULL) adds work to the streaming kernel that would otherwise be a pass of its own:
 *  - the ReLU backward step of the layer whose output this input is (Eq.3 line e1): with e1 non-NULL,
 *    e1 = e4 where the bit of mask_bits (that layer's forward mask, one bit per element, NULL = all ones) is set
 *    and 0 elsewhere, *sum_e1 += sum(e1), *absmax_e1 max= max|e1| (each may be NULL); e4 may then be NULL;
 *  - the statistics of the block-input merge: with merge_other non-NULL (int8 codes of the other error, same
 *    shape, exponent *merge_exp_other), *merge_absmax max= max|e4 * 2^(E4-Em) + other * 2^(Eo-Em)|,
 *    Em = min(E4, Eo), what eoq_merge_absmax computes; needs e4 and excludes e1.  With merge_mask_bits (one bit per
 *    element, the forward mask of the layer that receives the merged error) *merge_absmax_masked max= the same
 *    maximum over the elements whose bit is set: what EOQ_RQ_SQ_MERGE needs to write Q_e(e1 * gamma) in its own pass.
 *  - w_transposed non-NULL: the filters in C x R x S x K order, as written by eoq_transpose_filters from the same
 *    w; the call then skips its own transposition (a caller that updates w once per step transposes it once,
 *    off the critical path).
 *  - spec_state non-NULL (one int32 per layer, owned by the caller, device memory, -1 before the first call and
 *    otherwise left alone): the exponent r of the previous call.  r rarely changes from one training step to the
 *    next, so the call first codes its sums with that exponent while taking the true max|d|; if the exponent was
 *    right the work is done (no 16-bit intermediate is written or read), if not the call falls back to the path
 *    described above.  The result is the same either way; *spec_state receives this call's r.  Ignored (left
 *    untouched) for strided 1x1 filters, for stride-2 filters larger than 1x1 and when absmax_e1 is requested.
 * Requires 127^2 * R*S*K < 2^30. */
typedef struct eoq_bwd_fuse {
    const uint32_t *mask_bits;
    int8_t *e1;
    int64_t *sum_e1;
    int32_t *absmax_e1;
    const int8_t *merge_other;
    const int32_t *merge_exp_other;
    int32_t *merge_absmax;
    const int8_t *w_transposed;
    const uint32_t *merge_mask_bits;
    int32_t *merge_absmax_masked;
    int32_t *spec_state;
} eoq_bwd_fuse;
int eoq_conv_bwd_data_sq(eoq_ctx *ctx, const eoq_conv_desc *desc, const int8_t *e, const int8_t *w, int8_t *e4,
                         int32_t *absmax_slot, const int32_t *exp_in, int32_t exp_in_off, int32_t *exp_out,
                         int64_t *sum_out, const eoq_bwd_fuse *fuse, void *ws, size_t ws_bytes);

/* Filters K x R x S x C -> C x R x S x K, the operand order of the backward-data gather (Eq.3 line e4). */
int eoq_transpose_filters(eoq_ctx *ctx, const eoq_conv_desc *desc, const int8_t *w, int8_t *wt);

/* ---- weight-gradient convolution: Eq.4 line g_w before Q_g ------------------------------------
 * g_acc[k,r,s,c] = sum_{n,p,q} e[n,p,q,k] * u[n, p*stride+r-pad, q*stride+s-pad, c], the exact integer
 * sum (partial sums of at most 131072 terms are int32, their combination is int64).  An element
 * outside int32 sets EOQ_FLAG_ACC_OVERFLOW.  max|g_acc| is max-combined into *absmax_slot. */
int eoq_conv_bwd_weight(eoq_ctx *ctx, const eoq_conv_desc *desc, const int8_t *e, const int8_t *u,
                        int32_t *g_acc, int32_t *absmax_slot, void *ws, size_t ws_bytes);

/* The same call for callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving or fine-tuning loops, harnesses that forbid hipMalloc.  It takes no workspace: the partial
 * sums (and the staged copy of an input whose C is not a multiple of 16) go to a 32 MiB array that the library holds
 * in device memory on every GPU it is loaded on, from load until the process ends; its address on the context's
 * device was looked up by eoq_create.  The call itself allocates and frees nothing.  A problem whose staged input plus
 * the partial sums of the shortest legal reduction ranges (131072 terms each) exceed 32 MiB returns
 * EOQ_ERR_WORKSPACE before anything is launched; within the limit the reduction is split into as many ranges as fit
 * (at most as many as eoq_conv_bwd_weight would use), so results are identical to eoq_conv_bwd_weight's.  Every partial
 * sum that is read was written by the same call: nothing in the array has to start at zero, and what a call leaves
 * behind is never read.  ALL calls on one GPU share that one array, whatever their context or stream: calls that overlap
 * in time on one GPU race; order them on one stream or with events. */
int eoq_conv_bwd_weight_static(eoq_ctx *ctx, const eoq_conv_desc *desc, const int8_t *e, const int8_t *u,
                               int32_t *g_acc, int32_t *absmax_slot);

/* ---- ReLU backward and the statistics of Eq.3 lines e1..e3 / Eq.4 lines g_b2, g_gamma ----------
 * e1 = e0 * [mask]; *sum_e1 += sum e1 (bias gradient); *sum_e1t += sum e1 * t (multiplier gradient,
 * t_wide and sum_e1t may be NULL); *absmax_e1 = max(*absmax_e1, max|e1|) (for Q_e of e1*gamma).
 * mask_bits NULL means no ReLU (all ones).  e1 may alias e0. */
int eoq_relu_bwd(eoq_ctx *ctx, const int8_t *e0, const uint32_t *mask_bits, const int32_t *t_wide, size_t n,
                 int8_t *e1, int64_t *sum_e1, int64_t *sum_e1t, int32_t *absmax_e1);

/* Same as eoq_relu_bwd with t_wide = R(conv(u, w) / 128) recomputed on the fly instead of read from
 * memory (the wide Q_a1 output of a multiplier layer then never has to be stored by the forward pass):
 * one more evaluation of the forward convolution (desc, u, w as in eoq_conv_fwd, C % 16 == 0) whose
 * epilogue does the masking and the three reductions.  e1 may alias e0; e1 may be NULL when only the sums
 * are wanted (e0 then already is e1 and mask_bits is NULL: the multiplier's gradient, off the critical path). */
int eoq_relu_bwd_recompute(eoq_ctx *ctx, const eoq_conv_desc *desc, const int8_t *u, const int8_t *w,
                           const int8_t *e0, const uint32_t *mask_bits, int8_t *e1, int64_t *sum_e1,
                           int64_t *sum_e1t, int32_t *absmax_e1);

/* ---- the sums of Eq.4 for a scalar parameter, on their own: *sum += sum_i e[i] (t NULL: g_b1, g_b2) or
 * *sum += sum_i e[i] * t[i] (g_gamma, t = the wide Q_a1 output x2), exact in int64.  e: int8[n], t: int32[n],
 * both 16-byte aligned; any n.  The training step takes these sums inside the kernels that produce e (ReLU backward,
 * backward-data finishing pass, merge pass); this call is the same reduction for callers that hold e already. */
int eoq_reduce_sum_i64(eoq_ctx *ctx, const int8_t *e, const int32_t *t, size_t n, int64_t *sum);

/* ---- abs-max of the exact sum of two errors with different exponents (first phase of the merge
 * of branch and shortcut errors at a block input): v = a*2^(Ea-Em) + b*2^(Eb-Em), Em = min(Ea,Eb).
 * A gap above 24 sets EOQ_FLAG_EXP_GAP. */
int eoq_merge_absmax(eoq_ctx *ctx, const int8_t *a, const int32_t *exp_a, const int8_t *b, const int32_t *exp_b,
                     size_t n, int32_t *absmax_slot);

/* ---- requantisation passes ----------------------------------------------------------------------
 * EOQ_RQ_FWD      : the forward epilogue above on a stored accumulator (acc, K, ep).
 * EOQ_RQ_SQ_ACC   : Q_e / Q_g of an int32 tensor (Eq.11, Eq.12): v = acc, E = *exp_in + exp_in_off.
 * EOQ_RQ_SQ_GAMMA : Q_e(e2 * gamma) of Eq.3: v = src_a * (*gamma), E = *exp_in + exp_in_off - 7;
 *                   *absmax is max|src_a| (the kernel multiplies it by |gamma|).
 * EOQ_RQ_SQ_MERGE : Q_e of branch + shortcut error: v as in eoq_merge_absmax, E = min(*exp_in, *exp_b).
 * For the SQ modes, with M = *absmax: r = R(log2 M) (integer test, no tie possible),
 * out = clamp(R(v * 2^(7-r)), -127, 127), *exp_out = E + r - 7; M = 0 gives zeros and *exp_out = E.
 * Optional extras: *sum_out += sum of the output codes (bias gradient of Eq.4);
 * *max_code_out = max|out| (lets eoq_update_int8 skip its own abs-max pass).
 * EOQ_RQ_SQ_MERGE can apply, in the same pass, the ReLU backward step of the layer that receives the merged
 * error (Eq.3 line e1): with mask_bits (that layer's forward mask) the output is the code where the bit is set
 * and 0 elsewhere, sum_out sums these masked codes, and *absmax_out max= max|out| (for Q_e of e1 * gamma).
 * With out_b it also writes that next step itself: out_b = what EOQ_RQ_SQ_GAMMA gives for src_a = out, *gamma,
 * *absmax = max|out|, *exp_in = the merge's *exp_out (Eq.3 line e3), and *exp_out_b = its exponent.  max|out| is
 * not known before the pass, but the quantiser is monotone: it is the code of the largest merged value under the
 * mask, *absmax_masked (from eoq_conv_bwd_data_sq's merge_absmax_masked; without mask_bits *absmax serves). */
enum eoq_rq_mode { EOQ_RQ_FWD = 0, EOQ_RQ_SQ_ACC = 1, EOQ_RQ_SQ_GAMMA = 2, EOQ_RQ_SQ_MERGE = 3 };
typedef struct eoq_requant_args {
    int32_t mode;
    int32_t K;                 /* FWD: channels (innermost extent) */
    size_t n;                  /* elements */
    const int32_t *acc;        /* FWD, SQ_ACC */
    const eoq_epilogue *ep;    /* FWD (host struct) */
    const int8_t *src_a;       /* SQ_GAMMA: e1;  SQ_MERGE: branch error, exponent *exp_in */
    const int8_t *src_b;       /* SQ_MERGE: shortcut error, exponent *exp_b */
    const int32_t *exp_b;
    const int32_t *gamma;      /* SQ_GAMMA */
    const int32_t *absmax;
    const int32_t *exp_in;
    int32_t exp_in_off;
    int8_t *out;
    int32_t *exp_out;
    int64_t *sum_out;          /* may be NULL */
    int32_t *max_code_out;     /* may be NULL */
    const uint32_t *mask_bits; /* SQ_MERGE only, may be NULL: see above (n % 16 == 0) */
    int32_t *absmax_out;       /* SQ_MERGE only, may be NULL */
    int8_t *out_b;             /* SQ_MERGE only, may be NULL: second output, see above (n % 16 == 0) */
    int32_t *exp_out_b;        /* with out_b */
    const int32_t *absmax_masked; /* with out_b and mask_bits */
} eoq_requant_args;
int eoq_requant_epilogue(eoq_ctx *ctx, const eoq_requant_args *args);

/* ---- 8-bit update: Eq.13 and Q_w (Eq.8) ----------------------------------------------------------
 * lr = m * 2^-j with integers (m, j) read from lr_slot[0], lr_slot[1] on the device, 1 <= m <= 32768.
 * u = SQ(m * g * 2^(Eg - j)) -> (u_code, Eu);  d = R(u_code * 2^(Eu + 7));  w <- clamp(w - d, -127, 127).
 * g_max_code: device slot with max|g| (from EOQ_RQ_SQ_ACC's max_code_out), or NULL to have the call
 * find it with one extra pass. */
int eoq_update_int8(eoq_ctx *ctx, int8_t *w, size_t n, const int8_t *g, const int32_t *g_exp_slot,
                    const int32_t *g_max_code, const int32_t *lr_slot);

/* ---- Q_g, Q_u and the update of one layer's filters in one pass (Eq.12, Eq.13, Eq.8) -------------
 * Same result as eoq_requant_epilogue(EOQ_RQ_SQ_ACC) on the weight-gradient sums, eoq_update_int8 with the
 * codes it wrote and (wt non-NULL) eoq_transpose_filters of the updated filters, without writing the gradient
 * codes and reading them back:  with M = *absmax_slot (max|acc|, as left by eoq_conv_bwd_weight),
 * r = R(log2 M), g = clamp(R(acc * 2^(7-r))), Eg = *exp_in + exp_in_off + r - 7, then the update of
 * eoq_update_int8 with (g, Eg, max|g|) and the learning rate in lr_slot.  acc and w are device arrays of
 * desc->K * R * S * C elements in K x R x S x C order, 16-byte aligned; w is updated in place.
 * wt (may be NULL; needs K % 16 == 0 and C % 16 == 0): receives the updated filters in C x R x S x K order.
 * g_out (may be NULL) receives the gradient codes; *exp_out = Eg and *max_code_out = max|g| when non-NULL.
 * M = 0 leaves w unchanged (wt is still written), g = 0, Eg = *exp_in + exp_in_off. */
int eoq_grad_update(eoq_ctx *ctx, const eoq_conv_desc *desc, const int32_t *acc, const int32_t *absmax_slot,
                    const int32_t *exp_in, int32_t exp_in_off, const int32_t *lr_slot, int8_t *w, int8_t *wt,
                    int8_t *g_out, int32_t *exp_out, int32_t *max_code_out);

/* ---- scalar parameters (bias, multiplier: Eq.10, Eq.4 lines g_b1, g_b2, g_gamma, Eq.13) -----------
 * The gradient of a scalar is the sum over all elements, then Q_g of that one-element tensor, then
 * the update above without the clamp.  Each descriptor names up to two terms S * 2^(E + off):
 * sums[sum_idx[t]] and exps[exp_idx[t]] + exp_off[t]  (two terms when two convolutions read the same
 * biased input).  descs is a DEVICE array.  g_code_out / g_exp_out (may be NULL) receive Q_g's result. */
typedef struct eoq_scalar_grad {
    int32_t param;      /* index into scalars[] */
    int32_t n_terms;    /* 1 or 2 */
    int32_t sum_idx[2];
    int32_t exp_idx[2];
    int32_t exp_off[2];
} eoq_scalar_grad;
int eoq_update_scalars(eoq_ctx *ctx, int32_t *scalars, const eoq_scalar_grad *descs, int32_t count,
                       const int64_t *sums, const int32_t *exps, const int32_t *lr_slot,
                       int32_t *g_code_out, int32_t *g_exp_out);

/* ---- optional stochastic rounding of the update: BEYOND the paper, never the default ---------------------------
 * Eq.13 with round-to-nearest loses every update below half a code (the paper has no stochastic rounding; its
 * deterministic rule is what eoq_update_int8 / eoq_grad_update / eoq_update_scalars implement).  The _sr forms replace
 * the last rounding, d = R(u_code * 2^(Eu + 7)), by d = floor((u_code + r) / 2^s) for s = -(Eu + 7) > 0 with r uniform in
 * [0, 2^s) -- unbiased, E[d] = u_code / 2^s; an exact left shift when s <= 0 -- and are otherwise identical.  r is the
 * low s bits (s capped at 62) of a counter-based 64-bit hash, so that both the library and any checker can regenerate
 * every element's draw:  z = seed * 0x9E3779B97F4A7C15 + tensor_id * 0xC2B2AE3D27D4EB4F + step * 0xA0761D6478BD642F
 * + index * 0xD6E8FEB86659FD93 (mod 2^64), word = the splitmix64 finaliser of z (z ^= z >> 30; z *= 0xBF58476D1CE4E5B9;
 * z ^= z >> 27; z *= 0x94D049BB133111EB; z ^= z >> 31); index = the element's linear index in K x R x S x C order (0 for a
 * scalar).  sr_slot: device uint32[2] = {seed, step}, read at kernel time; eoq_sr_next_step adds one to the step (a
 * kernel, so a captured training step advances its own counter on every replay).  tensor_id: any caller-chosen
 * constant per tensor (tensor_ids: a device array with one id per eoq_scalar_grad descriptor). */
int eoq_update_int8_sr(eoq_ctx *ctx, int8_t *w, size_t n, const int8_t *g, const int32_t *g_exp_slot,
                       const int32_t *g_max_code, const int32_t *lr_slot, const uint32_t *sr_slot, uint32_t tensor_id);
int eoq_grad_update_sr(eoq_ctx *ctx, const eoq_conv_desc *desc, const int32_t *acc, const int32_t *absmax_slot,
                       const int32_t *exp_in, int32_t exp_in_off, const int32_t *lr_slot, int8_t *w, int8_t *wt,
                       int8_t *g_out, int32_t *exp_out, int32_t *max_code_out, const uint32_t *sr_slot,
                       uint32_t tensor_id);
int eoq_update_scalars_sr(eoq_ctx *ctx, int32_t *scalars, const eoq_scalar_grad *descs, int32_t count,
                          const int64_t *sums, const int32_t *exps, const int32_t *lr_slot, int32_t *g_code_out,
                          int32_t *g_exp_out, const uint32_t *sr_slot, const uint32_t *tensor_ids);
int eoq_sr_next_step(eoq_ctx *ctx, uint32_t *sr_slot);

/* ---- pooling, head (outside the quantised arithmetic of Eq.2-13 but on the step's path) ----------
 * Max pool R x S / stride / pad on int8 codes; padding never wins; the winner of a window is its first
 * maximum in (r,s) scan order and arg[n,p,q,c] = r*S+s of the winner (arg may be NULL when no backward
 * pass follows).  y / u_next as in the epilogue (either may be NULL).
 * Backward routes each error to the recorded winner and adds overlapping windows (int32 result, |d|
 * max-combined into *absmax_slot); a requant pass (EOQ_RQ_SQ_ACC) follows.  H, W are the INPUT extents. */
int eoq_maxpool_fwd(eoq_ctx *ctx, const int8_t *a, int32_t N, int32_t H, int32_t W, int32_t C, int32_t R,
                    int32_t S, int32_t stride, int32_t pad, int8_t *y, const int32_t *b_next_pre, int8_t *u_next,
                    uint8_t *arg);
int eoq_maxpool_bwd(eoq_ctx *ctx, const uint8_t *arg, const int8_t *e, int32_t N, int32_t H, int32_t W, int32_t C,
                    int32_t R, int32_t S, int32_t stride, int32_t pad, int32_t *d, int32_t *absmax_slot);
/* The same sums followed by Q_e (Eq.11) without the int32 tensor: the sums are formed twice, first for max|d|
 * (max-combined into *absmax_slot, which must hold 0 or a valid partial maximum), then for the codes
 * e_out = SQ(d) with *exp_out = *exp_in + R(log2 max|d|) - 7 (all-zero d: codes 0, exponent passed through).
 * mask_bits (may be NULL; one bit per element of e_out, 4-byte aligned): the ReLU backward step of the layer whose
 * output was pooled (Eq.3 line e1) in the same pass -- e_out = code where the bit is set, 0 elsewhere; *sum_out
 * (may be NULL) += sum of the codes written (the bias gradient of Eq.4).
 * spec_state (may be NULL): one int32 of device memory that the caller keeps from one training step to the next
 * (-1 initially), as in eoq_bwd_fuse: the first pass then codes with the exponent it holds and takes max|d| on the
 * way; when the exponent turns out right the second pass has nothing to do, otherwise it codes again.  The results
 * are the same in both cases; the call leaves the exact exponent R(log2 max|d|) there. */
int eoq_maxpool_bwd_sq(eoq_ctx *ctx, const uint8_t *arg, const int8_t *e, int32_t N, int32_t H, int32_t W, int32_t C,
                       int32_t R, int32_t S, int32_t stride, int32_t pad, int8_t *e_out, int32_t *absmax_slot,
                       const int32_t *exp_in, int32_t *exp_out, const uint32_t *mask_bits, int64_t *sum_out,
                       int32_t *spec_state);
/* Global average pool, integer part: sum[n][c] = sum_{h,w} y[n,h,w,c]. */
int eoq_gap_sum(eoq_ctx *ctx, const int8_t *y, int32_t N, int32_t HW, int32_t C, int32_t *sum);
/* e[n,h,w,c] = codes[n][c] for all HW positions (error of the average pool, already quantised). */
int eoq_broadcast_hw(eoq_ctx *ctx, const int8_t *codes, int32_t N, int32_t HW, int32_t C, int8_t *e);
/* Float head (the last layer stays unquantised, Section 5.1), fp64 in a fixed operation order:
 * feat = sum/(128*HW); logits = b + W feat (sequential fma, ascending feature); softmax with max
 * subtraction; loss = mean cross-entropy; d = (float)((W^T dlogits) / HW) per real activation;
 * then W -= lr*dW, b -= lr*db with lr = m * 2^-j from lr_slot.  ws: at least
 * eoq_head_workspace_bytes(N, F, J) bytes; it keeps feat and dlogits of the call.
 * lr_slot == NULL leaves W and b as they are: the update (the same two kernels, the same result) is then applied by
 * eoq_head_update from the workspace the forward/backward call filled, on whatever stream that context owns -- nothing
 * else in a training step reads the classifier, so a caller may run it beside the backward pass.  The caller orders it
 * behind the eoq_head_fwd_bwd call and before the next one. */
size_t eoq_head_workspace_bytes(int32_t N, int32_t F, int32_t J);
int eoq_head_fwd_bwd(eoq_ctx *ctx, int32_t N, int32_t F, int32_t J, int32_t HW, const int32_t *gap_sum,
                     double *Wfc, double *bfc, const int32_t *labels, const int32_t *lr_slot, double *loss,
                     float *d, double *logits, void *ws, size_t ws_bytes);
int eoq_head_update(eoq_ctx *ctx, int32_t N, int32_t F, int32_t J, double *Wfc, double *bfc, const int32_t *lr_slot,
                    const void *ws, size_t ws_bytes);

#ifdef __cplusplus
}
#endif
#endif /* EOQ_H */
