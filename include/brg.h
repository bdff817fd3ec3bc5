/*
 * brg.h -- C ABI of the batch-reduce GEMM library for AMD MI355X (gfx950).
 *
 * The library implements the building block of "High-Performance Deep Learning
 * via a Single Building Block" (arXiv 1906.06440) and the primitives the paper
 * writes as loop nests around it, as hand-written HIP kernels.
 *
 * Conventions common to every entry point
 * ---------------------------------------
 *  - Return value: a brg_status_t.  Nothing throws, aborts, allocates, frees or
 *    synchronises.  All arguments are validated on the host BEFORE any GPU call,
 *    so BRG_EINVAL / BRG_EALIGN / BRG_EUNSUPPORTED can be provoked without a
 *    GPU.  brg_last_error() returns a thread-local text for the last failure.
 *  - Every data pointer is a DEVICE pointer owned by the caller (unless a
 *    comment says HOST).  The work is enqueued on `stream` (a hipStream_t passed
 *    as void*; NULL is the default stream) and is complete when the stream has
 *    drained.  Buffers must stay alive until then.
 *  - `dtype` is the element type of the multiplied inputs (activations and
 *    weights): BRG_F32 or BRG_BF16.  Accumulation is always fp32.  `out_dtype`
 *    is the element type the result is stored in (fp32, or bf16 rounded to
 *    nearest even).  bias vectors are always fp32.
 *  - Data pointers must be aligned to 16 bytes (BRG_EALIGN otherwise).
 *  - Output buffers must not overlap input buffers (undefined result).  Inputs
 *    may alias each other.
 *  - Sizes are int64_t element counts.
 */
#ifndef BRG_H
#define BRG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BRG_OK = 0,
    BRG_EINVAL = 1,       /* null pointer, negative size, blocking does not divide, bad enum */
    BRG_EALIGN = 2,       /* a data pointer is not 16-byte aligned */
    BRG_EUNSUPPORTED = 3, /* valid request this build has no kernel for */
    BRG_EHIP = 4          /* a HIP runtime call failed; see brg_last_error() */
} brg_status_t;

typedef enum { BRG_F32 = 0, BRG_BF16 = 1 } brg_dtype_t;

typedef enum { BRG_ACT_NONE = 0, BRG_ACT_RELU = 1, BRG_ACT_SIGMOID = 2, BRG_ACT_TANH = 3 } brg_act_t;

typedef void *brg_stream_t; /* a hipStream_t */

/* Text of the calling thread's last non-OK status ("" if none).  HOST pointer, owned by the library. */
const char *brg_last_error(void);

/* Library version string, HOST pointer. */
const char *brg_version(void);

/* Tuning overrides -- NOT part of the ABI contract.  A set of environment variables forces a kernel variant
 * the planner would not choose by itself; they exist so that every variant can be parity-tested and timed.
 * The environment is read once, at the first call into the library; brg_tuning_reload() reads it again
 * (not safe against calls running at the same time on other threads).  Results never depend on them
 * beyond rounding order.  A workspace size query and the call it serves must see the SAME overrides (the planner
 * that sizes the workspace is the one that uses it).  Presence alone switches the ones marked (flag); the others
 * take a number.
 *   BRG_GEMM_GENERAL (flag)   brg_gemm*: always the general tile kernel
 *   BRG_NO_RING (flag)        64-cubed fp32 blocks: the double-buffered kernel instead of the four-stage ring
 *   BRG_FC_GENERAL (flag), BRG_FC_WGT_GENERAL (flag), BRG_FC_G64 = 64|32, BRG_FC_G128 = 0|1
 *                             fully connected layers: general kernel / tile shape of the tuned ones
 *   BRG_LSTM_GENERAL (flag)   LSTM forward and backward: one general launch per time step
 *   BRG_LSTM_SPIN_LIMIT = n   resident LSTM kernel: polls of the step barrier before a workgroup gives up (0: at once;
 *                             a test's way to reach the give-up path with every wave still exiting normally)
 *   BRG_CONV_GENERAL (flag), BRG_CONV_NO1X1 (flag), BRG_CONV_WGT_GENERAL (flag)
 *                             convolutions: general kernel for all / for 1x1 layers / for the weight gradient
 *   BRG_CONV_KW = 1|2, BRG_CONV_PITCH = 0, BRG_CONV_PLANE_PAD = bytes, BRG_CONV_ZEROFILL (flag), BRG_CONV_NOFUSE (flag)
 *                             tiled kernels: feature blocks per wave, halo pitch rule, extra bytes between the LDS
 *                             planes (a multiple of 16; default 0), separate zero fill and
 *                             unfused parity classes of the strided backward pass
 *   BRG_CONV_1X1_KW = 1|2|4, BRG_CONV_1X1_PG = 2|4, BRG_CONV_1X1_WF = 1|2|4, BRG_CONV_1X1_SPLIT = 0|1,
 *   BRG_CONV_1X1_LDS = 0|1, BRG_CONV_1X1_LDS_NGW = 2|4, BRG_CONV_1X1_LDS_PM = 0|1
 *                             bf16 1x1 layers: wave tile of the streaming kernel, split-reduction and
 *                             workgroup-tiled variants
 *   BRG_CONV_SMALL = 0|1, BRG_CONV_SMALL_KW = 1|2, BRG_CONV_SMALL_PG = 1|2, BRG_CONV_SMALL_GZ = 1..16
 *                             bf16 layers on few output pixels: never / wherever the kernel applies; feature blocks
 *                             and pixel groups per workgroup; ranges of the reduction chain
 *   BRG_CONV_STEM_CLASSES (flag), BRG_CONV_STEM_GX = n
 *                             bf16 7x7 layer on a channel block of 4: per-class backward launches, grid size
 *   BRG_CONV_WGT_PS = 1|2, BRG_CONV_WGT_TARGET = n
 *                             weight gradient: slabs per step, number of workgroups aimed at */
void brg_tuning_reload(void);

/* ---------------------------------------------------------------------------
 * Batch-reduce GEMM (paper section 2, the defining equation and Algorithm 1):
 *
 *     C = act( beta * C + alpha * sum_{i<count} A_i * B_i  [+ bias] )
 *
 * A_i is m x k, B_i is k x n, C is m x n, all COLUMN-MAJOR with leading
 * dimensions lda >= m, ldb >= k, ldc >= m (in elements).  The C tile is held in
 * matrix-core accumulators across the whole reduce chain and stored once.
 *
 *  brg_gemm          address-list form: A_ptrs / B_ptrs are DEVICE arrays of
 *                    `count` DEVICE pointers (the paper's "two arrays of
 *                    pointers"); blocks may live anywhere and may alias.
 *  brg_gemm_strided  stride form: A_i = A + i*strideA, B_i = B + i*strideB
 *                    (strides in elements, may be 0).
 *
 *  beta == 0 : C is not read (NaN/Inf in C do not propagate).
 *  count == 0: C = act(beta*C [+ bias]).
 *  bias      : optional fp32 vector of length m (added per row), or NULL.
 *  m, n, k >= 0; m == 0 or n == 0 is a no-op returning BRG_OK.
 *  Block pointers need only element alignment; the pointer arrays, bias and
 *  the base pointers of the strided form need 16 bytes.
 * ------------------------------------------------------------------------ */
int brg_gemm(brg_dtype_t dtype, brg_dtype_t out_dtype, int64_t m, int64_t n, int64_t k,
             int64_t lda, int64_t ldb, int64_t ldc, const void *const *A_ptrs,
             const void *const *B_ptrs, void *C, int64_t count, float alpha, float beta,
             const float *bias, brg_act_t act, brg_stream_t stream);

int brg_gemm_strided(brg_dtype_t dtype, brg_dtype_t out_dtype, int64_t m, int64_t n, int64_t k,
                     int64_t lda, int64_t ldb, int64_t ldc, const void *A, int64_t strideA,
                     const void *B, int64_t strideB, void *C, int64_t count, float alpha,
                     float beta, const float *bias, brg_act_t act, brg_stream_t stream);

/* ---------------------------------------------------------------------------
 * Convolution on blocked layouts (paper section 3.2, Algorithms 3 and 4):
 *
 *   input   I [N][C/bc][H][W][bc]
 *   weights Wt[K/bk][C/bc][R][S][bc][bk]
 *   output  O [N][K/bk][P][Q][bk],  P = (H + 2*pad_h - R)/stride_h + 1 (floor), Q likewise
 *
 *   O[n][k][oj][oi] = act( sum_{c,r,s} Wt[k][c][r][s] * I[n][c][stride*oj + r - pad][stride*oi + s - pad] [+ bias[k]] )
 *
 * (cross-correlation, no kernel flip).  Padding is LOGICAL: buffers hold no
 * border, taps outside the image contribute zero.  Each output block is one
 * batch-reduce chain over (c-block, r, s) whose addresses are generated inside
 * the kernel; C and K must be multiples of bc and bk (a 3-channel stem is
 * stored zero-padded to one block).  This build supports bc = bk = 16, and in
 * addition ONE input channel block of 4 (bc = C = 4, bk = 16; 8 bytes per bf16
 * pixel) for the 7x7 stride-2 pad-3 layer with bf16 inputs and bf16 output,
 * width up to 224, in brg_conv_fwd, brg_conv_bwd_data and (even widths from 64,
 * K a multiple of 64, with the workspace) brg_conv_bwd_wgt; any other use of
 * bc = 4 returns BRG_EUNSUPPORTED.
 *
 *  brg_conv_fwd       O from I and Wt; optional bias[K] (fp32) and activation.
 *  brg_conv_bwd_data  dI (layout of I) from dO (layout of O) and Wt in the SAME
 *                     forward layout: the adjoint of brg_conv_fwd with respect
 *                     to I (the paper's "dual convolution"); input pixels that
 *                     no tap reads are written as 0.
 *  brg_conv_bwd_wgt   dWt (fp32, layout of Wt) = sum_{n,oj,oi} dO * I.  Tuned for bf16 layers (and fp32
 *                     ones except the bc = 4 layer) with 1x1
 *                     filters (stride 1 or 2, no padding), 3x3 filters (padding 1, stride 1 or 2) and
 *                     the bc = 4 layer (which has no other path) when given the workspace of
 *                     brg_conv_bwd_wgt_ws_bytes; general kernel otherwise.
 * Workspace: brg_conv_fwd with fp32 in and out, or bf16 in and out, uses `ws` (DEVICE memory,
 * 16-byte aligned, at least brg_conv_ws_bytes() bytes, contents undefined afterwards) for a
 * re-blocked copy of the weights that it writes on the stream before the convolution itself.  With
 * ws == NULL fp32 reads the weights as stored (a few percent slower); bf16 1x1 layers re-block the
 * weights inside the kernel and need no workspace (only the variant for C >= 1024 on at most
 * 16384 pixels is not chosen without one), other bf16 filters take a slower general kernel (the
 * bc = 4 layer: the same kernel with a slower start).  bf16 layers with few output pixels (a small
 * minibatch, paper section 4.3) run on a kernel that divides the (c-block, r, s) chain between
 * workgroups; it keeps the fp32 partial results of a long chain in `ws` and, without one, leaves the
 * chain in one piece.  brg_conv_bwd_data ignores `ws`; for brg_conv_bwd_wgt see brg_conv_bwd_wgt_ws_bytes.
 * ------------------------------------------------------------------------ */
typedef struct {
    int64_t N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, bc, bk;
} brg_conv_desc_t;

/* Bytes of workspace brg_conv_fwd can use for this layer and input type (0 = none). */
int64_t brg_conv_ws_bytes(const brg_conv_desc_t *desc, brg_dtype_t dtype);

int brg_conv_fwd(const brg_conv_desc_t *desc, brg_dtype_t dtype, brg_dtype_t out_dtype,
                 const void *I, const void *Wt, void *O, const float *bias, brg_act_t act,
                 void *ws, brg_stream_t stream);

int brg_conv_bwd_data(const brg_conv_desc_t *desc, brg_dtype_t dtype, brg_dtype_t out_dtype,
                      const void *dO, const void *Wt, void *dI, void *ws, brg_stream_t stream);

int brg_conv_bwd_wgt(const brg_conv_desc_t *desc, brg_dtype_t dtype, const void *I,
                     const void *dO, float *dWt, void *ws, brg_stream_t stream);

/* Bytes of workspace that let brg_conv_bwd_wgt run its tuned bf16 kernel for this layer (0 = none
 * needed or no tuned kernel).  The tuned kernel splits the reduction over N*P*Q (section 3.2: the
 * weight-update pass reduces over the minibatch) into ranges, writes one partial dWt per range into
 * `ws` (DEVICE memory, 16-byte aligned, contents undefined afterwards) and adds the ranges in a fixed
 * order.  With ws == NULL such a layer takes the general kernel. */
int64_t brg_conv_bwd_wgt_ws_bytes(const brg_conv_desc_t *desc, brg_dtype_t dtype);

/* brg_conv_bwd_wgt for callers that cannot allocate device memory or carry a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same planner, kernels and
 * results as brg_conv_bwd_wgt given the workspace of brg_conv_bwd_wgt_ws_bytes, but the partial sums of
 * the pixel ranges live in a device array built into the library (BRG_CONV_BWD_WGT_NOALLOC_MAX_BYTES,
 * one copy per GPU, held until the process ends).  The call allocates and frees nothing.  A layer whose
 * brg_conv_bwd_wgt_ws_bytes exceeds that size returns BRG_EUNSUPPORTED (validated on the host, before
 * any GPU call); all 53 ResNet-50 layers at minibatch 64 fit.  The array keeps the previous call's
 * contents and needs no clearing: every range is written in full before it is read.  All calls on one GPU
 * share the array, so two calls that may overlap in time on the same GPU (different streams) race;
 * calls on one stream, or on different GPUs, do not. */
#define BRG_CONV_BWD_WGT_NOALLOC_MAX_BYTES (72 * 1024 * 1024)

int brg_conv_bwd_wgt_noalloc(const brg_conv_desc_t *desc, brg_dtype_t dtype, const void *I,
                             const void *dO, float *dWt, brg_stream_t stream);

/* ---------------------------------------------------------------------------
 * Fully connected layer on blocked layouts (paper section 3.3, Algorithm 5):
 *
 *   X [N/bn][C/bc][bn][bc]   Wt[K/bk][C/bc][bc][bk]   Y [N/bn][K/bk][bn][bk]
 *
 *  brg_fc_fwd   Y[n][k] = act( sum_c Wt[k][c] * X[n][c] [+ bias[k]] ); every Y
 *               block is one batch-reduce chain of length C/bc with the
 *               bias/activation applied before the single store.
 *  brg_fc_bwd   with dZ = dY o [Y > 0] when act == BRG_ACT_RELU (Y is the STORED
 *               forward output, an input here) and dZ = dY when act == NONE:
 *                 dX [n][c] = sum_k Wt[k][c] * dZ[n][k]    (chain over K/bk; weight
 *                                                           blocks read transposed)
 *                 dWt[k][c] = sum_n dZ[n][k] * X[n][c]     (chain over N/bn), fp32
 *                 dbias[k]  = sum_n dZ[n][k]               fp32
 *               Any of dX, dWt, dbias may be NULL to skip that result.  dX has
 *               the element type `dtype`.  SIGMOID/TANH are BRG_EUNSUPPORTED in bwd.
 * N, C, K must be multiples of bn, bc, bk.
 * Tuned paths: fp32 with bn = bc = bk = 64 (forward, and backward with dX, dWt and dbias in one
 * launch); bf16 in and out with bc = bk = 16 (any bn), where the layouts above coincide with those of
 * a 1x1 convolution over N/bn images of bn pixels (Algorithm 4 with R = S = 1) and the forward pass
 * and the unmasked backward by data (act == NONE) run on the 1x1 convolution kernels, the unmasked
 * weight and bias gradient on a kernel of its own (C/16 and K/16 multiples of 4, bn of 32).  With
 * act == RELU those kernels are used when `ws` is given: DEVICE memory, 16-byte aligned, at least
 * N*K*2 bytes, contents undefined afterwards; it receives dZ = dY o [Y > 0] first (bn a multiple of
 * 16).  Every other combination takes a general, slower kernel with the same results; `ws` may be
 * NULL and is not used by any other path.
 * ------------------------------------------------------------------------ */
typedef struct {
    int64_t N, C, K, bn, bc, bk;
} brg_fc_desc_t;

int brg_fc_fwd(const brg_fc_desc_t *desc, brg_dtype_t dtype, brg_dtype_t out_dtype,
               const void *X, const void *Wt, const float *bias, brg_act_t act, void *Y,
               brg_stream_t stream);

int brg_fc_bwd(const brg_fc_desc_t *desc, brg_dtype_t dtype, const void *dY, const void *Y,
               const void *X, const void *Wt, brg_act_t act, void *dX, float *dWt,
               float *dbias, void *ws, brg_stream_t stream);

/* brg_fc_bwd with the ReLU backward of the layer that PRODUCED X fused into the dX epilogue (the
 * paper's "apply the element-wise operation while the block is hot", section 3.3, applied to the
 * backward chain of an MLP): with act_in == BRG_ACT_RELU the stored dX is dX o [X > 0], i.e. it is
 * already the dZ of the producing layer, whose own backward call then runs with act == BRG_ACT_NONE
 * (and Y == NULL).  act_in == BRG_ACT_NONE is exactly brg_fc_bwd. */
int brg_fc_bwd_chain(const brg_fc_desc_t *desc, brg_dtype_t dtype, const void *dY, const void *Y,
                     const void *X, const void *Wt, brg_act_t act, brg_act_t act_in, void *dX,
                     float *dWt, float *dbias, void *ws, brg_stream_t stream);

/* ---------------------------------------------------------------------------
 * LSTM layer forward (paper section 3.1, equations (1)-(6) and Algorithm 2),
 * gate order i, c, f, o (c is the tanh candidate, s the cell state):
 *
 *   z_g = W_g x_t + R_g h_{t-1} + b_g            one chain of C/bc + K/bk blocks per gate
 *   i, f, o = sigmoid(z);  c = tanh(z_c);  s_t = f o s_{t-1} + i o c;  h_t = o o tanh(s_t)
 *
 *   W4: four [K/bk][C/bc][bc][bk] matrices back to back;  R4: four [K/bk][K/bk][bk][bk]
 *   x: [T][N][C];  b4: fp32 [4][K] or NULL;  h0, s0: [N][K] or NULL (zeros)
 *   outputs h, s: [T][N][K];  gates: [4][T][N][K] post-activation, or NULL
 * Element types.  dtype BRG_F32: everything fp32.  dtype BRG_BF16 (the paper's kernel is "agnostic of the
 * compute precision", section 2; it gives no recipe for the recurrence, this is the one built): the tensors that
 * enter matrix products -- x, W4, R4, h0 and the result h -- are bf16, everything else (b4, s0, s, gates) is
 * fp32; accumulation is fp32; h_t is rounded to bf16 (nearest even) once, when it is stored, and that stored
 * value is what step t+1 multiplies; the cell state is carried in fp32.
 * The gate non-linearities and the state update run on the accumulators before
 * anything is stored.  `bn` is advisory (the kernel picks its own batch tile).
 *
 * Workspace: `ws` is NULL or DEVICE memory of at least 16 bytes, 16-byte aligned, whose
 * contents need no initialisation (the library clears both words on the stream, on every path).  With
 * bc = bk = 64, N <= 256, K/4 <= the number of compute units and BOTH `gates` and `ws`
 * given, the layer runs as batch-reduce GEMMs for the input projections of all time steps (T*N need not be a
 * multiple of the tile) followed by ONE resident kernel for the recurrence, whose workgroups stream the batch in
 * passes of 64 rows and meet at a counter in ws (32-bit word 0) once per time step.  The wait is bounded: if the
 * workgroups cannot all be resident for that long (another stream occupying the device), the kernel stops early
 * and sets the 32-bit word 1 of ws to a non-zero value; a kernel enqueued right behind it then overwrites h, s and
 * gates with NaN, so that such a run cannot pass for a result (a caller may also read word 1 after the stream
 * has drained).  Where the device cannot hold K/4 such workgroups at once, without `gates` or `ws`, and for other
 * shapes, every time step is a launch of its own.
 * Two calls that overlap in time must not share `ws`.
 * ------------------------------------------------------------------------ */
typedef struct {
    int64_t T, N, C, K, bn, bc, bk;
} brg_lstm_desc_t;

int brg_lstm_fwd(const brg_lstm_desc_t *desc, brg_dtype_t dtype, const void *x, const void *W4,
                 const void *R4, const float *b4, const void *h0, const void *s0, void *h,
                 void *s, void *gates, void *ws, brg_stream_t stream);

/* ---------------------------------------------------------------------------
 * LSTM layer backward (paper section 3.1 reports the backward and weight-update passes without a
 * listing; this is the chain rule on equations (1)-(6)).  Inputs: the forward inputs x, W4, R4, h0, s0
 * (h0, s0 NULL = zeros), the forward results h, s [T][N][K] and gates [4][T][N][K] (values of i, c, f, o),
 * dh [T][N][K] = gradient of the loss with respect to every output h_t, ds_last [N][K] (or NULL) =
 * gradient with respect to the final cell state.  Outputs, each may be NULL to skip it: dx [T][N][C],
 * dW4 and dR4 (fp32, blocked like W4 and R4), db4 fp32 [4][K], dh0 and ds0 [N][K].
 * Per time step, from the last to the first: the gate gradients dz_g are element-wise in the stored
 * gates and states, and dh_{t-1} += sum_g R_g^T dz_g is one batch-reduce chain of 4 K/bk weight
 * blocks per output block; dx, dW4, dR4 and db4 are sums over all time steps computed afterwards.
 * `ws`: DEVICE memory, 16-byte aligned, at least brg_lstm_bwd_ws_bytes_dtype(desc, dtype) bytes (the dz
 * of all steps and seventeen [N][K] buffers; with bf16 operands also their fp32 copies), contents undefined
 * afterwards; required.  BRG_BF16: x, W4, R4, h0 and h are bf16 (as brg_lstm_fwd takes and leaves them), every
 * other tensor and every gradient is fp32; the operands are widened exactly into the workspace and the whole
 * pass runs in fp32 arithmetic (no gradient is rounded to bf16).  Correct for every shape; with
 * bc = bk = 64 and N a multiple of 64 the GEMMs run on the kernel for 64 x 64 x 64 blocks, otherwise on the
 * general one.
 * ------------------------------------------------------------------------ */
int64_t brg_lstm_bwd_ws_bytes(const brg_lstm_desc_t *desc);   /* the fp32 layer */
int64_t brg_lstm_bwd_ws_bytes_dtype(const brg_lstm_desc_t *desc, brg_dtype_t dtype);

int brg_lstm_bwd(const brg_lstm_desc_t *desc, brg_dtype_t dtype, const void *x, const void *W4,
                 const void *R4, const void *h0, const void *s0, const void *h, const void *s,
                 const void *gates, const void *dh, const void *ds_last, void *dx, float *dW4,
                 float *dR4, float *db4, void *dh0, void *ds0, void *ws, brg_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* BRG_H */
