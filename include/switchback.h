/*
 * libswitchback -- the SwitchBack int8 linear layer (arxiv 2304.13013, Section 2.2.1, Algorithm 1) for one
 * AMD MI355X (gfx950), as a C ABI.  Declared after the five calls of Algorithm 1: the layer's variants from the same
 * paper (SwitchBackM, SwitchBackQ, float8) and its optimizer (StableAdamW), each with the passage it follows.
 *
 * Notation (Section 2.2.1 "Notation"): X [b,n] inputs, W [m,n] weights (an nn.Linear weight, out x in),
 * Y = X W^T [b,m]; dY [b,m] the gradient of the loss w.r.t. Y, dX = dY W [b,n], dW = dY^T X [m,n];
 * b = batch size x sequence length.
 *
 * Conventions shared by every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller (the binding allocates with torch).  The
 *     library never allocates, frees or synchronizes: a call only enqueues kernels on `stream` (a
 *     hipStream_t passed as void*; NULL = the default stream).  Outputs are valid once the stream reaches them.
 *   - Matrices are dense row-major without strides; callers flatten leading dimensions into b.
 *   - bf16 tensors are passed as `const void*` to 16-bit patterns.  Pointers must be 16-byte aligned.
 *   - Shapes: b >= 1 (0 is accepted and is a no-op), n % 64 == 0, m % 64 == 0, and the contraction length of
 *     the int8 products (n for forward, m for the input gradient) at most 131072 so that 127^2 * K < 2^31.
 *     The GEMM kernels use 32-bit byte offsets into an operand: (b + 256) * max(n, m) * 2 must stay below 2^32
 *     (for the int8 product alone: (M + 256) * K, (N + 256) * K and 2 * M * N below 2^32).
 *   - Inputs must be finite; NaN/Inf give unspecified values but never a fault.  There is no bias (Algorithm 1
 *     passes only the weight).
 *   - Return value: SB_OK or an error code; nothing is enqueued when an error is returned, except
 *     SB_HIP_ERROR which reports a failed launch.  No exceptions, no abort, no output to stdout/stderr.
 *   - Calls on different streams may run concurrently as long as their output / workspace buffers differ.
 */
#ifndef SWITCHBACK_H
#define SWITCHBACK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SB_OK = 0,
    SB_INVALID_ARG = 1,         /* null / negative / misaligned argument, unknown enum value */
    SB_UNSUPPORTED_SHAPE = 2,   /* shape outside the contract above */
    SB_WORKSPACE_TOO_SMALL = 3, /* ws_bytes < switchback_workspace_bytes(op, b, n, m) */
    SB_HIP_ERROR = 4            /* hipGetLastError() reported a failed launch */
} sb_status;

/* Output element type of a product.  SB_I32_RAW dumps the int32 accumulators of an int8 product and skips the
 * dequantization (verification only; not valid for the weight gradient). */
typedef enum { SB_BF16 = 0, SB_F32 = 1, SB_I32_RAW = 2 } sb_dtype;

/* Which operation a workspace is sized for. */
typedef enum {
    SB_OP_QUANTIZE_TENSORWISE = 0,
    SB_OP_FORWARD = 1,
    SB_OP_BACKWARD_INPUT = 2,
    SB_OP_BACKWARD_WEIGHT = 3,
    SB_OP_QUANTIZE_COLWISE = 4, /* also the workspace of switchback_backward_input_q; pass rows as m, cols as n */
    SB_OP_STABLE_ADAMW = 5      /* shape arguments ignored */
} sb_op;

/* What the forward pass leaves for the backward pass (Algorithm 1 saves X and W in 16 bit and re-quantizes W in
 * backward; the scale of the tensor-wise quantizer is a single scalar, so Q(W^T) = Q(W)^T and this library
 * quantizes W once and keeps both layouts).  All five buffers are caller-provided and FILLED by
 * switchback_forward; switchback_backward_input reads wq_t and state_w. */
typedef struct sb_saved {
    int8_t *xq;      /* [b,n]  Q_row(X)                                   */
    float *state_x;  /* [b]    state_row(X): the row-wise absmax values    */
    int8_t *wq;      /* [m,n]  Q_tensor(W)                                */
    int8_t *wq_t;    /* [n,m]  Q_tensor(W)^T                              */
    float *state_w;  /* [1]    state_tensor(W): the absmax of W            */
} sb_saved;

/* Row-wise quantization Q_row with its state (first quantization equation of Section 2.2.1):
 *   state[i] = max_j |x[i,j]|,  q[i,j] = round(127/state[i] * x[i,j]),  codes in [-127,127].
 * Arithmetic: binary32; scale t = 127/state formed first (one correctly rounded divide per row), each element is
 * round-half-to-even of the rounded product x*t.  A row whose absmax is 0, or so small that 127/absmax
 * overflows binary32, gets all-zero codes and state 0.
 *   x [rows,cols] bf16 in; q [rows,cols] int8 out; state [rows] f32 out.  cols % 8 == 0, cols <= 65536. */
int switchback_quantize_rowwise(const void *x_bf16, int64_t rows, int64_t cols, int8_t *q, float *state,
                                void *stream);

/* Tensor-wise quantization Q_tensor with its state (second quantization equation of Section 2.2.1): as above
 * with one absmax for the whole matrix.  Also emits the transposed code matrix (the paper's fused
 * "tensor-wise quantize transpose"), reading W from HBM once for the absmax and once for both code layouts.
 *   w [rows,cols] bf16 in; q [rows,cols] int8 out; q_t [cols,rows] int8 out or NULL; state [1] f32 out;
 *   ws: SB_OP_QUANTIZE_TENSORWISE workspace (partial maxima; contents are scratch).
 *   rows % 16 == 0, cols % 16 == 0. */
int switchback_quantize_tensorwise(const void *w_bf16, int64_t rows, int64_t cols, int8_t *q, int8_t *q_t,
                                   float *state, void *ws, size_t ws_bytes, void *stream);

/* The int8 product with fused dequantization (the dequantized forward equation of Section 2.2.1):
 *   acc[i,j] = sum_k aq[i,k] * bq[j,k]                       (int8 x int8 -> int32, exact)
 *   out[i,j] = (state_tensor/127^2 * state_row[i]) * acc[i,j]
 * evaluated in binary32 as c = state_tensor/16129, r_i = state_row[i]*c, out = (float)acc * r_i, then rounded
 * to nearest-even when out_dtype is SB_BF16.  Both operands have the contraction index contiguous.
 *   aq [M,K] int8; state_row [M] f32; bq [N,K] int8; state_tensor [1] f32 (device); out [M,N].
 *   K % 64 == 0, N % 64 == 0, K <= 131072, (M + 256) * K < 2^32, (N + 256) * K < 2^32, 2 * M * N < 2^32.  With SB_I32_RAW the states are ignored (may be NULL). */
int switchback_matmul_int8_dequant(const int8_t *aq, const float *state_row, const int8_t *bq,
                                   const float *state_tensor, int64_t M, int64_t N, int64_t K, void *out,
                                   sb_dtype out_dtype, void *stream);

/* Forward pass of Algorithm 1: Y = dequant(Q_row(X) Q_tensor(W)^T).  Fills `saved` (see sb_saved).
 *   x [b,n] bf16, w [m,n] bf16 in; y [b,m] out in y_dtype; ws: SB_OP_FORWARD workspace. */
int switchback_forward(const void *x_bf16, const void *w_bf16, int64_t b, int64_t n, int64_t m, void *y,
                       sb_dtype y_dtype, const sb_saved *saved, void *ws, size_t ws_bytes, void *stream);

/* switchback_forward for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same results bit for bit, no
 * workspace argument: the partial maxima of the tensor-wise quantizer (its only scratch, 4 KiB) live in a
 * file-scope device array of the library, one copy per GPU, held until the process ends.  The call allocates and
 * frees nothing (the address of the array on the current device is looked up on the first call made on that device).
 *   Limit: m * n <= SB_FORWARD_STATIC_MAX_WEIGHTS (2^28 weights, four times the largest layer of the paper's
 *   workloads; the array holds one partial maximum per workgroup of the first pass, at most 1024, which is sized for
 *   that); larger layers get SB_UNSUPPORTED_SHAPE and should use switchback_forward with their own workspace.
 *   All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU (different streams)
 *   race on it and may quantize W with the wrong absmax.  Serialize them, or use switchback_forward.  Nothing in the
 *   array needs clearing between calls.  Other arguments, shapes and errors as switchback_forward. */
#define SB_FORWARD_STATIC_MAX_WEIGHTS ((int64_t)1 << 28)
int switchback_forward_static(const void *x_bf16, const void *w_bf16, int64_t b, int64_t n, int64_t m, void *y,
                              sb_dtype y_dtype, const sb_saved *saved, void *stream);

/* Input gradient of Algorithm 1: dX = dequant(Q_row(dY) Q_tensor(W)), dequantized with the state of the
 * quantized dY and the state of W.  Reads saved->wq_t and saved->state_w; fills gq and state_g.
 *   dy [b,m] bf16 in; dx [b,n] out in dx_dtype; gq [b,m] int8 out; state_g [b] f32 out. */
int switchback_backward_input(const void *dy_bf16, const sb_saved *saved, int64_t b, int64_t n, int64_t m,
                              void *dx, sb_dtype dx_dtype, int8_t *gq, float *state_g, void *stream);

/* Weight gradient of Algorithm 1, the product the layer "switches back" to 16 bit for: dW = dY^T X with bf16
 * operands and binary32 accumulation (summation order unspecified but deterministic for a given shape).
 *   dy [b,m] bf16, x [b,n] bf16 in; dw [m,n] out, SB_BF16 or SB_F32; ws: SB_OP_BACKWARD_WEIGHT workspace. */
int switchback_backward_weight(const void *dy_bf16, const void *x_bf16, int64_t b, int64_t n, int64_t m,
                               void *dw, sb_dtype dw_dtype, void *ws, size_t ws_bytes, void *stream);

/* The memory-efficient variant SwitchBackM (the appendix algorithm that keeps only X_int8 and state_X of the input
 * for the backward pass instead of X in 16 bit).  Its forward pass and input gradient are those of Algorithm 1
 * (switchback_forward fills saved->xq and saved->state_x); its weight gradient first rebuilds X:
 *
 * switchback_dequantize_rowwise: x^[i,j] = q[i,j] * state[i] / 127, the row-wise quantization equation read
 * backwards, evaluated in binary32 as step_i = state[i] / 127 (correctly rounded), fl((float)q * step_i), then
 * rounded to nearest-even bf16.  q [rows,cols] int8, state [rows] f32 in; x_bf16 [rows,cols] out.  cols % 8 == 0.
 *
 * switchback_backward_weight_m: dW = dY^T X^ with X^ = dequantize_rowwise(saved->xq, saved->state_x) written to
 * x_hat_bf16 [b,n] (caller-provided scratch, may be reused once the stream has passed the call); then exactly
 * switchback_backward_weight on (dy, x_hat).  ws: SB_OP_BACKWARD_WEIGHT workspace. */
int switchback_dequantize_rowwise(const int8_t *q, const float *state, int64_t rows, int64_t cols, void *x_bf16,
                                  void *stream);
int switchback_backward_weight_m(const void *dy_bf16, const sb_saved *saved, int64_t b, int64_t n, int64_t m,
                                 void *x_hat_bf16, void *dw, sb_dtype dw_dtype, void *ws, size_t ws_bytes,
                                 void *stream);

/* The variant SwitchBackQ (the appendix algorithm with row-wise and column-wise quantization of the weights; its
 * forward pass is 1/127^2 * state_row(X) state_row(W)^T * (Q_row(X) Q_row(W)^T), the equation that follows the
 * variants paragraph of Section 2.2.1).  Both operands of a product then carry one state per row of their code
 * matrix, evaluated as c_j = state_b[j]/16129, fl(state_a[i] * c_j), fl((float)acc * that), bf16 by RNE.
 *
 * switchback_quantize_colwise_transpose ("column-wise_quantize_transpose"): one absmax per COLUMN of w [rows,cols];
 *   q_t [cols,rows] int8 (transposed codes), state [cols] f32.  Equal to switchback_quantize_rowwise of the
 *   transposed matrix.  rows % 16 == 0, cols % 16 == 0; ws: SB_OP_QUANTIZE_COLWISE workspace.
 * switchback_matmul_int8_dequant_rc: out[i,j] = state_a[i] * state_b[j] / 127^2 * sum_k aq[i,k] bq[j,k];
 *   aq [M,K], state_a [M], bq [N,K], state_b [N]; out [M,N] SB_BF16 or SB_F32; shape limits as the tensor-wise call.
 * switchback_forward_q: Y = dequant(Q_row(X) Q_row(W)^T); fills xq [b,n], state_x [b], wq [m,n], state_w_row [m].
 * switchback_backward_input_q: dX = dequant(Q_row(dY) Q_col(W)); fills gq [b,m], state_g [b], wq_t [n,m],
 *   state_w_col [n] (W is quantized again from its 16-bit values, as the algorithm does); ws as above.
 * The weight gradient of the variant is switchback_backward_weight. */
int switchback_quantize_colwise_transpose(const void *w_bf16, int64_t rows, int64_t cols, int8_t *q_t, float *state,
                                          void *ws, size_t ws_bytes, void *stream);
int switchback_matmul_int8_dequant_rc(const int8_t *aq, const float *state_a, const int8_t *bq, const float *state_b,
                                      int64_t M, int64_t N, int64_t K, void *out, sb_dtype out_dtype, void *stream);
int switchback_forward_q(const void *x_bf16, const void *w_bf16, int64_t b, int64_t n, int64_t m, void *y,
                         sb_dtype y_dtype, int8_t *xq, float *state_x, int8_t *wq, float *state_w_row, void *stream);
int switchback_backward_input_q(const void *dy_bf16, const void *w_bf16, int64_t b, int64_t n, int64_t m, void *dx,
                                sb_dtype dx_dtype, int8_t *gq, float *state_g, int8_t *wq_t, float *state_w_col,
                                void *ws, size_t ws_bytes, void *stream);

/* The linear layer's bias and the transformer block's layer-scale, fused into the epilogue of the int8 product (the
 * block equations of the section on feature magnitudes: x' = x + gamma * block(x), where block ends in a linear layer,
 * so the product's output is gamma[j] * (y[i,j] + bias[j]); the paper initialises gamma with zeros.  SwitchBackLinear
 * is an nn.Linear and has a bias; Algorithm 1 leaves it out, which is what the calls above compute).  With y the
 * dequantized product of switchback_matmul_int8_dequant, in binary32 with one rounding per operation:
 *     z = y + bias[j]   (skipped when bias is NULL),    out = gamma[j] * z   (skipped when gamma is NULL),
 * then rounded to nearest-even when out_dtype is SB_BF16.  bias, gamma: [N] f32 device vectors (16-byte aligned) or
 * NULL; out_dtype SB_BF16 or SB_F32; shapes as switchback_matmul_int8_dequant / switchback_forward.  The backward pass
 * of the two elementwise operations (dY scaled by gamma before the calls of Algorithm 1's backward, the two vector
 * gradients) is the caller's.
 *   switchback_forward_bias_layerscale: switchback_forward (fills `saved` the same way) with this epilogue. */
int switchback_matmul_int8_dequant_bias_layerscale(const int8_t *aq, const float *state_row, const int8_t *bq,
                                                   const float *state_tensor, const float *bias, const float *gamma,
                                                   int64_t M, int64_t N, int64_t K, void *out, sb_dtype out_dtype,
                                                   void *stream);
int switchback_forward_bias_layerscale(const void *x_bf16, const void *w_bf16, const float *bias, const float *gamma,
                                       int64_t b, int64_t n, int64_t m, void *y, sb_dtype y_dtype,
                                       const sb_saved *saved, void *ws, size_t ws_bytes, void *stream);

/* The float8 variant of the layer (the "float8" paragraph of Section 2.2.1: the same code path with
 * round(127 x / absmax(x)) replaced by float8cast(x / absmax(x)); the paper simulates it in 16 bit, here the codes are
 * real 8-bit floats and the product runs on the float8 matrix instructions).  Formats are those of the format paper the
 * section cites: SB_E4M3 (bias 7, no infinities, largest 448) and SB_E5M2 (bias 15, IEEE-like).  Codes are bytes with
 * the sign in bit 7; they lie in [-1, 1], so the dequantization has no 1/127^2:
 *   state = absmax (binary32), t = 1/state (one correctly rounded divide; zero or overflowing rows give zero codes and
 *   state 0), code = float8cast(fl(x * t)) with round-to-nearest-even onto the format's values, subnormals included;
 *   out[i,j] = (state_row[i] * state_tensor) * sum_k value(aq[i,k]) value(bq[j,k]), the sum accumulated in binary32
 *   by the matrix instruction (order unspecified but deterministic), r_i = fl(state_row[i] * state_tensor) formed
 *   first, output rounded to nearest-even when SB_BF16.
 * Shapes as for the int8 calls, and additionally K % 128 == 0 (n % 128 == 0 and m % 128 == 0 for the layer calls);
 * out_dtype SB_BF16 or SB_F32.  The layer calls use the int8 layer's sb_saved with its code buffers holding float8
 * bytes (same sizes).  The weight gradient of the variant is switchback_backward_weight (16 bit). */
typedef enum { SB_E4M3 = 0, SB_E5M2 = 1 } sb_f8_format;
int switchback_quantize_rowwise_f8(const void *x_bf16, int64_t rows, int64_t cols, sb_f8_format fmt, uint8_t *codes,
                                   float *state, void *stream);
int switchback_quantize_tensorwise_f8(const void *w_bf16, int64_t rows, int64_t cols, sb_f8_format fmt, uint8_t *codes,
                                      uint8_t *codes_t, float *state, void *ws, size_t ws_bytes, void *stream);
int switchback_matmul_f8_dequant(const uint8_t *aq, sb_f8_format fmt_a, const float *state_row, const uint8_t *bq,
                                 sb_f8_format fmt_b, const float *state_tensor, int64_t M, int64_t N, int64_t K,
                                 void *out, sb_dtype out_dtype, void *stream);
/* Y = dequant(f8_row(X) f8_tensor(W)^T); fills saved (xq, state_x in fmt_x; wq, wq_t, state_w in fmt_w). */
int switchback_forward_f8(const void *x_bf16, const void *w_bf16, int64_t b, int64_t n, int64_t m, void *y,
                          sb_dtype y_dtype, const sb_saved *saved, sb_f8_format fmt_x, sb_f8_format fmt_w, void *ws,
                          size_t ws_bytes, void *stream);
/* dX = dequant(f8_row(dY) f8_tensor(W)); reads saved->wq_t (fmt_w) and state_w; fills gq [b,m] (fmt_g), state_g [b]. */
int switchback_backward_input_f8(const void *dy_bf16, const sb_saved *saved, int64_t b, int64_t n, int64_t m, void *dx,
                                 sb_dtype dx_dtype, uint8_t *gq, float *state_g, sb_f8_format fmt_g,
                                 sb_f8_format fmt_w, void *stream);

/* One StableAdamW step for one parameter tensor (the optimizer algorithm of the paper's section on loss spikes: AdamW
 * with the debiasing folded into the decay rates and update clipping; the implementation note of the appendix gives
 * the guarded denominator of RMS_t).  With b1 = beta1 (1 - beta1^(t-1)) / (1 - beta1^t) and b2 likewise (formed on the
 * host in binary64, then rounded to binary32; t = 1 gives 0):
 *     v <- b1 v + (1 - b1) g,   u <- b2 u + (1 - b2) g^2,
 *     RMS_t = sqrt(mean_j(g_j^2 / max(u_j, eps^2))) over the `count` elements of this tensor,
 *     eta = alpha / max(1, RMS_t),   theta <- theta - eta lambda theta - eta v / (sqrt(u) + eps).
 * Arithmetic is binary32 per element; the mean is accumulated in binary64 in a fixed order (deterministic).
 *   theta, v, u: [count] f32 device arrays, updated in place (v, u start at zero before step 1);
 *   grad: [count] device array, SB_BF16 or SB_F32 (grad_dtype), read only; all four 16-byte aligned;
 *   t >= 1 is the step number; 0 <= beta1, beta2 < 1; eps > 0; alpha is the scheduled learning rate of this step;
 *   rms_out: optional device float that receives RMS_t (NULL to skip);
 *   ws: SB_OP_STABLE_ADAMW workspace (partial sums; scratch).  count == 0 is a no-op.
 * Tensors of one model are independent calls (the clipping is per tensor, as in the paper). */
int switchback_stable_adamw_step(float *theta, float *v, float *u, const void *grad, sb_dtype grad_dtype,
                                 int64_t count, float alpha, float beta1, float beta2, float eps, float lambda,
                                 int64_t t, float *rms_out, void *ws, size_t ws_bytes, void *stream);

/* The same step for many tensors in two launches (a model has hundreds of parameter tensors, most of them small; one
 * launch pair per tensor would be bound by launch overhead).  Each tensor is clipped by its own RMS_t exactly as in
 * switchback_stable_adamw_step, and gets the same number of workgroups as there, so the results are bit-identical
 * to per-tensor calls.
 *   switchback_stable_adamw_plan (host only, touches no GPU): fills first_block / num_blocks of a HOST table of n
 *     entries whose theta, v, u, grad, count are set, and returns the total number of workgroups (0 if n == 0,
 *     negative status code on a bad entry).  The caller then copies the table to the device once; it stays valid
 *     while the pointers do.
 *   switchback_stable_adamw_step_multi: table_dev is that device copy (16-byte aligned), total_blocks the plan's
 *     return value; all gradients share grad_dtype; rms_out: optional device array [n]; ws: at least
 *     8 * total_blocks bytes (partial sums).  Hyper-parameters as in the single-tensor call. */
typedef struct sb_adamw_tensor {
    float *theta;      /* [count] f32, updated in place        */
    float *v;          /* [count] f32 first moment             */
    float *u;          /* [count] f32 second moment            */
    const void *grad;  /* [count] SB_BF16 or SB_F32            */
    int64_t count;     /* > 0                                  */
    int32_t first_block;
    int32_t num_blocks;
} sb_adamw_tensor;
int64_t switchback_stable_adamw_plan(sb_adamw_tensor *table_host, int n);
int switchback_stable_adamw_step_multi(const sb_adamw_tensor *table_dev, int n, int64_t total_blocks,
                                       sb_dtype grad_dtype, float alpha, float beta1, float beta2, float eps,
                                       float lambda, int64_t t, float *rms_out, void *ws, size_t ws_bytes, void *stream);

/* Bytes of device workspace `op` needs for a layer of this shape (0 if none).  Shape arguments an op does not
 * use are ignored (for SB_OP_QUANTIZE_TENSORWISE pass rows as m and cols as n). */
size_t switchback_workspace_bytes(int op, int64_t b, int64_t n, int64_t m);

/* Static description of a status code. */
const char *switchback_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* SWITCHBACK_H */
