// C ABI of libswitchback: argument validation and the kernel sequence of each pass of Algorithm 1
// (arxiv 2304.13013).  Every step runs in the HIP kernels of this library; nothing here touches tensor data.
#include "sb_common.h"

#include <atomic>
#include <cmath>

// Scratch of switchback_forward_static: the partial maxima of the tensor-wise quantizer's first pass, one device copy
// per GPU, held until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; kernels get
// the per-device address that call returns.
static __device__ __align__(256) unsigned int scratch[sb::kTensorwisePartials];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<unsigned int *> g_scratch_ptr[kMaxDevices];  // zero-initialized; index = HIP device ordinal

// Device address of `scratch` on the current device, resolved once per device.  Two host threads racing to the first
// call on a device both resolve and store the same address.
int scratch_of_current_device(unsigned int **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SB_HIP_ERROR;
    unsigned int *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        void *addr = nullptr;
        if (hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)) != hipSuccess || addr == nullptr) return SB_HIP_ERROR;
        p = static_cast<unsigned int *>(addr);
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return SB_OK;
}

constexpr int64_t kMaxIntK = 131072;  // 127^2 * K < 2^31 needs K <= 133143; rounded down to a power of two

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool ok_ptr(const void *p) { return p != nullptr && aligned16(p); }
bool ok_f8(int f) { return f == SB_E4M3 || f == SB_E5M2; }
bool ok_dtype(int d) { return d == SB_BF16 || d == SB_F32 || d == SB_I32_RAW; }

int layer_shape_status(int64_t b, int64_t n, int64_t m) {
    if (b < 0 || n <= 0 || m <= 0) return SB_INVALID_ARG;
    if (n % 64 || m % 64 || b > (int64_t)1 << 30 || n > kMaxIntK || m > kMaxIntK) return SB_UNSUPPORTED_SHAPE;
    // The GEMM kernels address their operands through 32-bit buffer offsets (with a stage or tile of slack); the
    // bf16 operands of the weight gradient are the largest.
    if ((b + 256) * n * 2 >= (int64_t)1 << 32 || (b + 256) * m * 2 >= (int64_t)1 << 32) return SB_UNSUPPORTED_SHAPE;
    return SB_OK;
}

int from_hip(hipError_t e) { return e == hipSuccess ? SB_OK : SB_HIP_ERROR; }

// Corrected decay rate of StableAdamW, in binary64: beta (1 - beta^(t-1)) / (1 - beta^t); 0 at t = 1.
double corrected_decay(double beta, int64_t step) {
    if (beta == 0.0) return 0.0;
    return beta * (1.0 - std::pow(beta, (double)(step - 1))) / (1.0 - std::pow(beta, (double)step));
}

}  // namespace

extern "C" {

int switchback_quantize_rowwise(const void *x_bf16, int64_t rows, int64_t cols, int8_t *q, float *state,
                                void *stream) {
    if (rows < 0 || cols <= 0) return SB_INVALID_ARG;
    if (cols % 8 || cols > 65536 || rows > (int64_t)1 << 30) return SB_UNSUPPORTED_SHAPE;
    if (rows == 0) return SB_OK;
    if (!ok_ptr(x_bf16) || !ok_ptr(q) || state == nullptr) return SB_INVALID_ARG;
    return from_hip(sb::launch_quantize_rowwise(x_bf16, rows, cols, q, state, static_cast<hipStream_t>(stream)));
}

int switchback_dequantize_rowwise(const int8_t *q, const float *state, int64_t rows, int64_t cols, void *x_bf16,
                                  void *stream) {
    if (rows < 0 || cols <= 0) return SB_INVALID_ARG;
    if (cols % 8 || cols > 65536 || rows > (int64_t)1 << 30) return SB_UNSUPPORTED_SHAPE;
    if (rows == 0) return SB_OK;
    if (!ok_ptr(q) || !ok_ptr(x_bf16) || state == nullptr) return SB_INVALID_ARG;
    return from_hip(sb::launch_dequantize_rowwise(q, state, rows, cols, x_bf16, static_cast<hipStream_t>(stream)));
}

int switchback_quantize_tensorwise(const void *w_bf16, int64_t rows, int64_t cols, int8_t *q, int8_t *q_t,
                                   float *state, void *ws, size_t ws_bytes, void *stream) {
    if (rows <= 0 || cols <= 0) return SB_INVALID_ARG;
    if (rows % 16 || cols % 16 || rows > (int64_t)1 << 24 || cols > (int64_t)1 << 24) return SB_UNSUPPORTED_SHAPE;
    if (!ok_ptr(w_bf16) || !ok_ptr(q) || (q_t != nullptr && !aligned16(q_t)) || state == nullptr)
        return SB_INVALID_ARG;
    if (ws == nullptr || !aligned16(ws)) return SB_INVALID_ARG;
    if (ws_bytes < switchback_workspace_bytes(SB_OP_QUANTIZE_TENSORWISE, 0, cols, rows))
        return SB_WORKSPACE_TOO_SMALL;
    return from_hip(sb::launch_quantize_tensorwise(w_bf16, rows, cols, q, q_t, state,
                                                   static_cast<unsigned int *>(ws),
                                                   static_cast<hipStream_t>(stream)));
}

int switchback_matmul_int8_dequant(const int8_t *aq, const float *state_row, const int8_t *bq,
                                   const float *state_tensor, int64_t M, int64_t N, int64_t K, void *out,
                                   sb_dtype out_dtype, void *stream) {
    if (M < 0 || N <= 0 || K <= 0 || !ok_dtype(out_dtype)) return SB_INVALID_ARG;
    if (K % 64 || N % 64 || K > kMaxIntK || N > kMaxIntK || M > (int64_t)1 << 30) return SB_UNSUPPORTED_SHAPE;
    // 32-bit buffer offsets, with a tile of slack for the rows past the end that read as zero.
    if ((M + 256) * K >= (int64_t)1 << 32 || (N + 256) * K >= (int64_t)1 << 32) return SB_UNSUPPORTED_SHAPE;
    if (M * N * 2 >= (int64_t)1 << 32) return SB_UNSUPPORTED_SHAPE;  // the output too
    if (M == 0) return SB_OK;
    if (!ok_ptr(aq) || !ok_ptr(bq) || !ok_ptr(out)) return SB_INVALID_ARG;
    if (out_dtype != SB_I32_RAW && (state_row == nullptr || state_tensor == nullptr)) return SB_INVALID_ARG;
    return from_hip(sb::launch_gemm_i8_dequant(aq, state_row, bq, state_tensor, nullptr, M, N, K, out, out_dtype,
                                               static_cast<hipStream_t>(stream)));
}

int switchback_matmul_int8_dequant_bias_layerscale(const int8_t *aq, const float *state_row, const int8_t *bq,
                                                   const float *state_tensor, const float *bias, const float *gamma,
                                                   int64_t M, int64_t N, int64_t K, void *out, sb_dtype out_dtype,
                                                   void *stream) {
    if (M < 0 || N <= 0 || K <= 0 || (out_dtype != SB_BF16 && out_dtype != SB_F32)) return SB_INVALID_ARG;
    if (K % 64 || N % 64 || K > kMaxIntK || N > kMaxIntK || M > (int64_t)1 << 30) return SB_UNSUPPORTED_SHAPE;
    if ((M + 256) * K >= (int64_t)1 << 32 || (N + 256) * K >= (int64_t)1 << 32) return SB_UNSUPPORTED_SHAPE;
    if (M * N * 2 >= (int64_t)1 << 32) return SB_UNSUPPORTED_SHAPE;
    if (M == 0) return SB_OK;
    if (!ok_ptr(aq) || !ok_ptr(bq) || !ok_ptr(out) || state_row == nullptr || state_tensor == nullptr)
        return SB_INVALID_ARG;
    if ((bias != nullptr && !aligned16(bias)) || (gamma != nullptr && !aligned16(gamma))) return SB_INVALID_ARG;
    return from_hip(sb::launch_gemm_i8_dequant_post(aq, state_row, bq, state_tensor, bias, gamma, M, N, K, out,
                                                    out_dtype, static_cast<hipStream_t>(stream)));
}

int switchback_forward_bias_layerscale(const void *x_bf16, const void *w_bf16, const float *bias, const float *gamma,
                                       int64_t b, int64_t n, int64_t m, void *y, sb_dtype y_dtype,
                                       const sb_saved *saved, void *ws, size_t ws_bytes, void *stream) {
    int st = layer_shape_status(b, n, m);
    if (st != SB_OK) return st;
    if ((y_dtype != SB_BF16 && y_dtype != SB_F32) || saved == nullptr) return SB_INVALID_ARG;
    if (!ok_ptr(w_bf16) || !ok_ptr(saved->wq) || !ok_ptr(saved->wq_t) || saved->state_w == nullptr)
        return SB_INVALID_ARG;
    if (b > 0 && (!ok_ptr(x_bf16) || !ok_ptr(y) || !ok_ptr(saved->xq) || saved->state_x == nullptr))
        return SB_INVALID_ARG;
    if ((bias != nullptr && !aligned16(bias)) || (gamma != nullptr && !aligned16(gamma))) return SB_INVALID_ARG;
    if (ws == nullptr || !aligned16(ws)) return SB_INVALID_ARG;
    if (ws_bytes < switchback_workspace_bytes(SB_OP_FORWARD, b, n, m)) return SB_WORKSPACE_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Algorithm 1's forward pass; the product's epilogue continues with the layer's bias and the block's layer-scale.
    hipError_t e = sb::launch_quantize_forward_operands(x_bf16, b, n, saved->xq, saved->state_x, w_bf16, m, saved->wq,
                                                        saved->wq_t, saved->state_w, static_cast<unsigned int *>(ws), s);
    if (e != hipSuccess) return SB_HIP_ERROR;
    if (b == 0) return SB_OK;
    return from_hip(sb::launch_gemm_i8_dequant_post(saved->xq, saved->state_x, saved->wq, saved->state_w, bias, gamma,
                                                    b, m, n, y, y_dtype, s));
}

int switchback_forward(const void *x_bf16, const void *w_bf16, int64_t b, int64_t n, int64_t m, void *y,
                       sb_dtype y_dtype, const sb_saved *saved, void *ws, size_t ws_bytes, void *stream) {
    int st = layer_shape_status(b, n, m);
    if (st != SB_OK) return st;
    if (!ok_dtype(y_dtype) || saved == nullptr) return SB_INVALID_ARG;
    if (!ok_ptr(w_bf16) || !ok_ptr(saved->wq) || !ok_ptr(saved->wq_t) || saved->state_w == nullptr)
        return SB_INVALID_ARG;
    if (b > 0 && (!ok_ptr(x_bf16) || !ok_ptr(y) || !ok_ptr(saved->xq) || saved->state_x == nullptr))
        return SB_INVALID_ARG;
    if (ws == nullptr || !aligned16(ws)) return SB_INVALID_ARG;
    if (ws_bytes < switchback_workspace_bytes(SB_OP_FORWARD, b, n, m)) return SB_WORKSPACE_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Algorithm 1, forward: X_int8, state_X = row-wise quantize(X); W_int8, state_W = tensor-wise quantize(W) (its
    // absmax pass rides on the row-wise launch); Y = int8 matmul fused with the dequantization.
    hipError_t e = sb::launch_quantize_forward_operands(x_bf16, b, n, saved->xq, saved->state_x, w_bf16, m, saved->wq,
                                                        saved->wq_t, saved->state_w, static_cast<unsigned int *>(ws), s);
    if (e != hipSuccess) return SB_HIP_ERROR;
    if (b == 0) return SB_OK;
    return from_hip(sb::launch_gemm_i8_dequant(saved->xq, saved->state_x, saved->wq, saved->state_w, nullptr, b, m, n, y,
                                               y_dtype, s));
}

int switchback_forward_static(const void *x_bf16, const void *w_bf16, int64_t b, int64_t n, int64_t m, void *y,
                              sb_dtype y_dtype, const sb_saved *saved, void *stream) {
    int st = layer_shape_status(b, n, m);
    if (st != SB_OK) return st;
    if (m * n > SB_FORWARD_STATIC_MAX_WEIGHTS) return SB_UNSUPPORTED_SHAPE;
    if (!ok_dtype(y_dtype) || saved == nullptr) return SB_INVALID_ARG;
    if (!ok_ptr(w_bf16) || !ok_ptr(saved->wq) || !ok_ptr(saved->wq_t) || saved->state_w == nullptr)
        return SB_INVALID_ARG;
    if (b > 0 && (!ok_ptr(x_bf16) || !ok_ptr(y) || !ok_ptr(saved->xq) || saved->state_x == nullptr))
        return SB_INVALID_ARG;
    unsigned int *partials = nullptr;
    st = scratch_of_current_device(&partials);
    if (st != SB_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // The kernel sequence of switchback_forward.  Nothing in the scratch has to start at zero: the first pass writes
    // every partial maximum the second pass reads.
    hipError_t e = sb::launch_quantize_forward_operands(x_bf16, b, n, saved->xq, saved->state_x, w_bf16, m, saved->wq,
                                                        saved->wq_t, saved->state_w, partials, s);
    if (e != hipSuccess) return SB_HIP_ERROR;
    if (b == 0) return SB_OK;
    return from_hip(sb::launch_gemm_i8_dequant(saved->xq, saved->state_x, saved->wq, saved->state_w, nullptr, b, m, n, y,
                                               y_dtype, s));
}

int switchback_backward_input(const void *dy_bf16, const sb_saved *saved, int64_t b, int64_t n, int64_t m,
                              void *dx, sb_dtype dx_dtype, int8_t *gq, float *state_g, void *stream) {
    int st = layer_shape_status(b, n, m);
    if (st != SB_OK) return st;
    if (!ok_dtype(dx_dtype) || saved == nullptr) return SB_INVALID_ARG;
    if (b == 0) return SB_OK;
    if (!ok_ptr(dy_bf16) || !ok_ptr(dx) || !ok_ptr(gq) || state_g == nullptr || !ok_ptr(saved->wq_t) ||
        saved->state_w == nullptr)
        return SB_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Algorithm 1, backward: G_int8, state_G = row-wise quantize(dY); the tensor-wise quantized, transposed W
    // was kept by the forward pass; dX = int8 matmul over m fused with the dequantization.
    hipError_t e = sb::launch_quantize_rowwise(dy_bf16, b, m, gq, state_g, s);
    if (e != hipSuccess) return SB_HIP_ERROR;
    return from_hip(sb::launch_gemm_i8_dequant(gq, state_g, saved->wq_t, saved->state_w, nullptr, b, n, m, dx, dx_dtype, s));
}

int switchback_backward_weight(const void *dy_bf16, const void *x_bf16, int64_t b, int64_t n, int64_t m,
                               void *dw, sb_dtype dw_dtype, void *ws, size_t ws_bytes, void *stream) {
    int st = layer_shape_status(b, n, m);
    if (st != SB_OK) return st;
    if (dw_dtype != SB_BF16 && dw_dtype != SB_F32) return SB_INVALID_ARG;
    if (!ok_ptr(dw) || (b > 0 && (!ok_ptr(dy_bf16) || !ok_ptr(x_bf16)))) return SB_INVALID_ARG;
    const size_t need = switchback_workspace_bytes(SB_OP_BACKWARD_WEIGHT, b, n, m);
    if (need > 0 && (ws == nullptr || !aligned16(ws))) return SB_INVALID_ARG;
    if (ws_bytes < need) return SB_WORKSPACE_TOO_SMALL;
    // Algorithm 1, backward: W_gradient = 16-bit matmul of dY^T and X (b == 0 gives an all-zero gradient).
    return from_hip(sb::launch_gemm_bf16_tn(dy_bf16, x_bf16, b, n, m, dw, dw_dtype, ws,
                                            static_cast<hipStream_t>(stream)));
}

int switchback_backward_weight_m(const void *dy_bf16, const sb_saved *saved, int64_t b, int64_t n, int64_t m,
                                 void *x_hat_bf16, void *dw, sb_dtype dw_dtype, void *ws, size_t ws_bytes,
                                 void *stream) {
    int st = layer_shape_status(b, n, m);
    if (st != SB_OK) return st;
    if (saved == nullptr) return SB_INVALID_ARG;
    if (b > 0 && (!ok_ptr(saved->xq) || saved->state_x == nullptr || !ok_ptr(x_hat_bf16))) return SB_INVALID_ARG;
    // SwitchBackM backward: X = row-wise dequantize(X_int8, state_X), then the 16-bit matmul of Algorithm 1.  The
    // weight-gradient call validates the remaining arguments before anything is enqueued.
    if (dw_dtype != SB_BF16 && dw_dtype != SB_F32) return SB_INVALID_ARG;
    if (!ok_ptr(dw) || (b > 0 && !ok_ptr(dy_bf16))) return SB_INVALID_ARG;
    const size_t need = switchback_workspace_bytes(SB_OP_BACKWARD_WEIGHT, b, n, m);
    if (need > 0 && (ws == nullptr || !aligned16(ws))) return SB_INVALID_ARG;
    if (ws_bytes < need) return SB_WORKSPACE_TOO_SMALL;
    if (b > 0) {
        hipError_t e = sb::launch_dequantize_rowwise(saved->xq, saved->state_x, b, n, x_hat_bf16,
                                                     static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return SB_HIP_ERROR;
    }
    return switchback_backward_weight(dy_bf16, x_hat_bf16, b, n, m, dw, dw_dtype, ws, ws_bytes, stream);
}

int switchback_quantize_colwise_transpose(const void *w_bf16, int64_t rows, int64_t cols, int8_t *q_t, float *state,
                                          void *ws, size_t ws_bytes, void *stream) {
    if (rows <= 0 || cols <= 0) return SB_INVALID_ARG;
    if (rows % 16 || cols % 16 || rows > (int64_t)1 << 24 || cols > (int64_t)1 << 24) return SB_UNSUPPORTED_SHAPE;
    if (!ok_ptr(w_bf16) || !ok_ptr(q_t) || state == nullptr) return SB_INVALID_ARG;
    if (ws == nullptr || !aligned16(ws)) return SB_INVALID_ARG;
    if (ws_bytes < sb::quantize_colwise_workspace_bytes(rows, cols)) return SB_WORKSPACE_TOO_SMALL;
    return from_hip(sb::launch_quantize_colwise_transpose(w_bf16, rows, cols, q_t, state, ws,
                                                          static_cast<hipStream_t>(stream)));
}

int switchback_matmul_int8_dequant_rc(const int8_t *aq, const float *state_a, const int8_t *bq, const float *state_b,
                                      int64_t M, int64_t N, int64_t K, void *out, sb_dtype out_dtype, void *stream) {
    if (M < 0 || N <= 0 || K <= 0 || (out_dtype != SB_BF16 && out_dtype != SB_F32)) return SB_INVALID_ARG;
    if (K % 64 || N % 64 || K > kMaxIntK || N > kMaxIntK || M > (int64_t)1 << 30) return SB_UNSUPPORTED_SHAPE;
    if ((M + 256) * K >= (int64_t)1 << 32 || (N + 256) * K >= (int64_t)1 << 32) return SB_UNSUPPORTED_SHAPE;
    if (M * N * 2 >= (int64_t)1 << 32) return SB_UNSUPPORTED_SHAPE;
    if (M == 0) return SB_OK;
    if (!ok_ptr(aq) || !ok_ptr(bq) || !ok_ptr(out) || state_a == nullptr || !ok_ptr(state_b)) return SB_INVALID_ARG;
    return from_hip(sb::launch_gemm_i8_dequant(aq, state_a, bq, nullptr, state_b, M, N, K, out, out_dtype,
                                               static_cast<hipStream_t>(stream)));
}

int switchback_forward_q(const void *x_bf16, const void *w_bf16, int64_t b, int64_t n, int64_t m, void *y,
                         sb_dtype y_dtype, int8_t *xq, float *state_x, int8_t *wq, float *state_w_row, void *stream) {
    int st = layer_shape_status(b, n, m);
    if (st != SB_OK) return st;
    if (y_dtype != SB_BF16 && y_dtype != SB_F32) return SB_INVALID_ARG;
    if (!ok_ptr(w_bf16) || !ok_ptr(wq) || !ok_ptr(state_w_row)) return SB_INVALID_ARG;
    if (b > 0 && (!ok_ptr(x_bf16) || !ok_ptr(y) || !ok_ptr(xq) || state_x == nullptr)) return SB_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // SwitchBackQ forward: X_int8, state_X = row-wise quantize(X); W_int8, state_W = row-wise quantize(W); int8
    // matmul fused with the row-and-column dequantization.
    hipError_t e = sb::launch_quantize_rowwise(w_bf16, m, n, wq, state_w_row, s);
    if (e != hipSuccess) return SB_HIP_ERROR;
    if (b == 0) return SB_OK;
    e = sb::launch_quantize_rowwise(x_bf16, b, n, xq, state_x, s);
    if (e != hipSuccess) return SB_HIP_ERROR;
    return from_hip(sb::launch_gemm_i8_dequant(xq, state_x, wq, nullptr, state_w_row, b, m, n, y, y_dtype, s));
}

int switchback_backward_input_q(const void *dy_bf16, const void *w_bf16, int64_t b, int64_t n, int64_t m, void *dx,
                                sb_dtype dx_dtype, int8_t *gq, float *state_g, int8_t *wq_t, float *state_w_col,
                                void *ws, size_t ws_bytes, void *stream) {
    int st = layer_shape_status(b, n, m);
    if (st != SB_OK) return st;
    if (dx_dtype != SB_BF16 && dx_dtype != SB_F32) return SB_INVALID_ARG;
    if (!ok_ptr(w_bf16) || !ok_ptr(wq_t) || !ok_ptr(state_w_col)) return SB_INVALID_ARG;
    if (b > 0 && (!ok_ptr(dy_bf16) || !ok_ptr(dx) || !ok_ptr(gq) || state_g == nullptr)) return SB_INVALID_ARG;
    if (ws == nullptr || !aligned16(ws)) return SB_INVALID_ARG;
    if (ws_bytes < sb::quantize_colwise_workspace_bytes(m, n)) return SB_WORKSPACE_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // SwitchBackQ backward: G_int8 = row-wise quantize(dY); W_int8, state_W = column-wise quantize transpose(W); the
    // contraction runs over m, with one state per token and one per input feature.
    hipError_t e = sb::launch_quantize_colwise_transpose(w_bf16, m, n, wq_t, state_w_col, ws, s);
    if (e != hipSuccess) return SB_HIP_ERROR;
    if (b == 0) return SB_OK;
    e = sb::launch_quantize_rowwise(dy_bf16, b, m, gq, state_g, s);
    if (e != hipSuccess) return SB_HIP_ERROR;
    return from_hip(sb::launch_gemm_i8_dequant(gq, state_g, wq_t, nullptr, state_w_col, b, n, m, dx, dx_dtype, s));
}

int switchback_quantize_rowwise_f8(const void *x_bf16, int64_t rows, int64_t cols, sb_f8_format fmt, uint8_t *codes,
                                   float *state, void *stream) {
    if (rows < 0 || cols <= 0 || !ok_f8(fmt)) return SB_INVALID_ARG;
    if (cols % 8 || cols > 65536 || rows > (int64_t)1 << 30) return SB_UNSUPPORTED_SHAPE;
    if (rows == 0) return SB_OK;
    if (!ok_ptr(x_bf16) || !ok_ptr(codes) || state == nullptr) return SB_INVALID_ARG;
    return from_hip(sb::launch_quantize_rowwise_f8(x_bf16, rows, cols, fmt, codes, state,
                                                   static_cast<hipStream_t>(stream)));
}

int switchback_quantize_tensorwise_f8(const void *w_bf16, int64_t rows, int64_t cols, sb_f8_format fmt, uint8_t *codes,
                                      uint8_t *codes_t, float *state, void *ws, size_t ws_bytes, void *stream) {
    if (rows <= 0 || cols <= 0 || !ok_f8(fmt)) return SB_INVALID_ARG;
    if (rows % 16 || cols % 16 || rows > (int64_t)1 << 24 || cols > (int64_t)1 << 24) return SB_UNSUPPORTED_SHAPE;
    if (!ok_ptr(w_bf16) || !ok_ptr(codes) || (codes_t != nullptr && !aligned16(codes_t)) || state == nullptr)
        return SB_INVALID_ARG;
    if (ws == nullptr || !aligned16(ws)) return SB_INVALID_ARG;
    if (ws_bytes < switchback_workspace_bytes(SB_OP_QUANTIZE_TENSORWISE, 0, cols, rows))
        return SB_WORKSPACE_TOO_SMALL;
    return from_hip(sb::launch_quantize_tensorwise_f8(w_bf16, rows, cols, fmt, codes, codes_t, state,
                                                      static_cast<unsigned int *>(ws),
                                                      static_cast<hipStream_t>(stream)));
}

int switchback_matmul_f8_dequant(const uint8_t *aq, sb_f8_format fmt_a, const float *state_row, const uint8_t *bq,
                                 sb_f8_format fmt_b, const float *state_tensor, int64_t M, int64_t N, int64_t K,
                                 void *out, sb_dtype out_dtype, void *stream) {
    if (M < 0 || N <= 0 || K <= 0 || !ok_f8(fmt_a) || !ok_f8(fmt_b)) return SB_INVALID_ARG;
    if (out_dtype != SB_BF16 && out_dtype != SB_F32) return SB_INVALID_ARG;
    if (K % 128 || N % 64 || K > kMaxIntK || N > kMaxIntK || M > (int64_t)1 << 30) return SB_UNSUPPORTED_SHAPE;
    if ((M + 256) * K >= (int64_t)1 << 32 || (N + 256) * K >= (int64_t)1 << 32) return SB_UNSUPPORTED_SHAPE;
    if (M * N * 2 >= (int64_t)1 << 32) return SB_UNSUPPORTED_SHAPE;
    if (M == 0) return SB_OK;
    if (!ok_ptr(aq) || !ok_ptr(bq) || !ok_ptr(out) || state_row == nullptr || state_tensor == nullptr)
        return SB_INVALID_ARG;
    return from_hip(sb::launch_gemm_f8_dequant(aq, fmt_a, state_row, bq, fmt_b, state_tensor, M, N, K, out, out_dtype,
                                               static_cast<hipStream_t>(stream)));
}

int switchback_forward_f8(const void *x_bf16, const void *w_bf16, int64_t b, int64_t n, int64_t m, void *y,
                          sb_dtype y_dtype, const sb_saved *saved, sb_f8_format fmt_x, sb_f8_format fmt_w, void *ws,
                          size_t ws_bytes, void *stream) {
    int st = layer_shape_status(b, n, m);
    if (st != SB_OK) return st;
    if (n % 128 || m % 128) return SB_UNSUPPORTED_SHAPE;
    if ((y_dtype != SB_BF16 && y_dtype != SB_F32) || saved == nullptr || !ok_f8(fmt_x) || !ok_f8(fmt_w))
        return SB_INVALID_ARG;
    if (!ok_ptr(w_bf16) || !ok_ptr(saved->wq) || !ok_ptr(saved->wq_t) || saved->state_w == nullptr)
        return SB_INVALID_ARG;
    if (b > 0 && (!ok_ptr(x_bf16) || !ok_ptr(y) || !ok_ptr(saved->xq) || saved->state_x == nullptr))
        return SB_INVALID_ARG;
    if (ws == nullptr || !aligned16(ws)) return SB_INVALID_ARG;
    if (ws_bytes < switchback_workspace_bytes(SB_OP_FORWARD, b, n, m)) return SB_WORKSPACE_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t *xq = reinterpret_cast<uint8_t *>(saved->xq), *wq = reinterpret_cast<uint8_t *>(saved->wq);
    // The forward pass of Algorithm 1 with float8cast(x / absmax) as the quantizer.
    hipError_t e = sb::launch_quantize_forward_operands_f8(x_bf16, b, n, fmt_x, xq, saved->state_x, w_bf16, m, fmt_w, wq,
                                                           reinterpret_cast<uint8_t *>(saved->wq_t), saved->state_w,
                                                           static_cast<unsigned int *>(ws), s);
    if (e != hipSuccess) return SB_HIP_ERROR;
    if (b == 0) return SB_OK;
    return from_hip(sb::launch_gemm_f8_dequant(xq, fmt_x, saved->state_x, wq, fmt_w, saved->state_w, b, m, n, y,
                                               y_dtype, s));
}

int switchback_backward_input_f8(const void *dy_bf16, const sb_saved *saved, int64_t b, int64_t n, int64_t m, void *dx,
                                 sb_dtype dx_dtype, uint8_t *gq, float *state_g, sb_f8_format fmt_g,
                                 sb_f8_format fmt_w, void *stream) {
    int st = layer_shape_status(b, n, m);
    if (st != SB_OK) return st;
    if (n % 128 || m % 128) return SB_UNSUPPORTED_SHAPE;
    if ((dx_dtype != SB_BF16 && dx_dtype != SB_F32) || saved == nullptr || !ok_f8(fmt_g) || !ok_f8(fmt_w))
        return SB_INVALID_ARG;
    if (b == 0) return SB_OK;
    if (!ok_ptr(dy_bf16) || !ok_ptr(dx) || !ok_ptr(gq) || state_g == nullptr || !ok_ptr(saved->wq_t) ||
        saved->state_w == nullptr)
        return SB_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = sb::launch_quantize_rowwise_f8(dy_bf16, b, m, fmt_g, gq, state_g, s);
    if (e != hipSuccess) return SB_HIP_ERROR;
    return from_hip(sb::launch_gemm_f8_dequant(gq, fmt_g, state_g, reinterpret_cast<const uint8_t *>(saved->wq_t), fmt_w,
                                               saved->state_w, b, n, m, dx, dx_dtype, s));
}

int switchback_stable_adamw_step(float *theta, float *v, float *u, const void *grad, sb_dtype grad_dtype,
                                 int64_t count, float alpha, float beta1, float beta2, float eps, float lambda,
                                 int64_t t, float *rms_out, void *ws, size_t ws_bytes, void *stream) {
    if (count < 0 || t < 1) return SB_INVALID_ARG;
    if (grad_dtype != SB_BF16 && grad_dtype != SB_F32) return SB_INVALID_ARG;
    if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f) || !(eps > 0.0f)) return SB_INVALID_ARG;
    if (!std::isfinite(alpha) || !std::isfinite(lambda)) return SB_INVALID_ARG;
    if (count == 0) return SB_OK;
    if (!ok_ptr(theta) || !ok_ptr(v) || !ok_ptr(u) || !ok_ptr(grad) || ws == nullptr || !aligned16(ws))
        return SB_INVALID_ARG;
    if (ws_bytes < sb::stable_adamw_workspace_bytes()) return SB_WORKSPACE_TOO_SMALL;
    const double b1 = corrected_decay((double)beta1, t), b2 = corrected_decay((double)beta2, t);
    return from_hip(sb::launch_stable_adamw_step(theta, v, u, grad, grad_dtype == SB_BF16, count, alpha, (float)b1,
                                                 (float)b2, (float)(1.0 - b1), (float)(1.0 - b2), eps, lambda, rms_out,
                                                 ws, static_cast<hipStream_t>(stream)));
}

int64_t switchback_stable_adamw_plan(sb_adamw_tensor *table_host, int n) {
    if (n < 0 || (n > 0 && table_host == nullptr)) return -SB_INVALID_ARG;
    int64_t total = 0;
    for (int i = 0; i < n; ++i) {
        sb_adamw_tensor &t = table_host[i];
        if (t.count <= 0 || !ok_ptr(t.theta) || !ok_ptr(t.v) || !ok_ptr(t.u) || !ok_ptr(t.grad)) return -SB_INVALID_ARG;
        t.first_block = (int32_t)total;
        t.num_blocks = sb::stable_adamw_blocks(t.count);
        total += t.num_blocks;
        if (total > (int64_t)1 << 30) return -SB_UNSUPPORTED_SHAPE;
    }
    return total;
}

int switchback_stable_adamw_step_multi(const sb_adamw_tensor *table_dev, int n, int64_t total_blocks,
                                       sb_dtype grad_dtype, float alpha, float beta1, float beta2, float eps,
                                       float lambda, int64_t t, float *rms_out, void *ws, size_t ws_bytes, void *stream) {
    if (n < 0 || total_blocks < 0 || t < 1) return SB_INVALID_ARG;
    if (grad_dtype != SB_BF16 && grad_dtype != SB_F32) return SB_INVALID_ARG;
    if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f) || !(eps > 0.0f)) return SB_INVALID_ARG;
    if (!std::isfinite(alpha) || !std::isfinite(lambda)) return SB_INVALID_ARG;
    if (n == 0) return total_blocks == 0 ? SB_OK : SB_INVALID_ARG;
    if (total_blocks < n || total_blocks > (int64_t)1 << 30) return SB_INVALID_ARG;  // every tensor has a workgroup
    if (!ok_ptr(table_dev) || ws == nullptr || !aligned16(ws)) return SB_INVALID_ARG;
    if (ws_bytes < (size_t)total_blocks * sizeof(double)) return SB_WORKSPACE_TOO_SMALL;
    const double b1 = corrected_decay((double)beta1, t), b2 = corrected_decay((double)beta2, t);
    return from_hip(sb::launch_stable_adamw_step_multi(table_dev, n, (int)total_blocks, grad_dtype == SB_BF16, alpha,
                                                       (float)b1, (float)b2, (float)(1.0 - b1), (float)(1.0 - b2), eps,
                                                       lambda, rms_out, ws, static_cast<hipStream_t>(stream)));
}

size_t switchback_workspace_bytes(int op, int64_t b, int64_t n, int64_t m) {
    switch (op) {
        case SB_OP_QUANTIZE_TENSORWISE:
        case SB_OP_FORWARD: return sb::kTensorwisePartials * sizeof(unsigned int);
        case SB_OP_BACKWARD_INPUT: return 0;
        case SB_OP_BACKWARD_WEIGHT:
            if (b < 0 || n <= 0 || m <= 0) return 0;
            return sb::gemm_bf16_tn_workspace_bytes(b, n, m);
        case SB_OP_QUANTIZE_COLWISE:  // w is [m, n]
            if (n <= 0 || m <= 0) return 0;
            return sb::quantize_colwise_workspace_bytes(m, n);
        case SB_OP_STABLE_ADAMW: return sb::stable_adamw_workspace_bytes();
        default: return 0;
    }
}

const char *switchback_status_string(int status) {
    switch (status) {
        case SB_OK: return "ok";
        case SB_INVALID_ARG: return "invalid argument (null, negative, misaligned or unknown enum)";
        case SB_UNSUPPORTED_SHAPE: return "unsupported shape";
        case SB_WORKSPACE_TOO_SMALL: return "workspace too small";
        case SB_HIP_ERROR: return "HIP launch error";
        default: return "unknown status";
    }
}

}  // extern "C"
