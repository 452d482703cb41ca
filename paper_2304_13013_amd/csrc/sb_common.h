// Shared declarations of the SwitchBack HIP library (internal; the public C ABI is include/switchback.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/switchback.h"

namespace sb {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef __bf16 v4bf __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned short v2us __attribute__((ext_vector_type(2)));
typedef short v4s __attribute__((ext_vector_type(4)));

// s_waitcnt that waits only on the vector-memory counter (gfx9 encoding: vmcnt = simm16[15:14]:[3:0],
// expcnt [6:4] and lgkmcnt [11:8] left at their maxima).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

__device__ __forceinline__ float bf16_bits_to_float(unsigned int bits16) { return __uint_as_float(bits16 << 16); }

// Launchers (each validates nothing: the C-ABI layer has already checked shapes and pointers).
hipError_t launch_quantize_rowwise(const void *x, int64_t rows, int64_t cols, int8_t *q, float *state,
                                   hipStream_t stream);
hipError_t launch_dequantize_rowwise(const int8_t *q, const float *state, int64_t rows, int64_t cols, void *x_hat,
                                     hipStream_t stream);
size_t quantize_colwise_workspace_bytes(int64_t rows, int64_t cols);
hipError_t launch_quantize_colwise_transpose(const void *w, int64_t rows, int64_t cols, int8_t *q_t, float *state,
                                             void *partials, hipStream_t stream);
hipError_t launch_quantize_tensorwise(const void *w, int64_t rows, int64_t cols, int8_t *q, int8_t *q_t,
                                      float *state, unsigned int *partials, hipStream_t stream);
// X row-wise and W [m,n] tensor-wise (both code layouts) in two launches: the first pass of W's quantizer rides on X's
// launch.  Results are those of the separate launchers, bit for bit.
hipError_t launch_quantize_forward_operands(const void *x, int64_t b, int64_t n, int8_t *xq, float *state_x,
                                            const void *w, int64_t m, int8_t *wq, int8_t *wq_t, float *state_w,
                                            unsigned int *partials, hipStream_t stream);
hipError_t launch_quantize_forward_operands_f8(const void *x, int64_t b, int64_t n, int fmt_x, uint8_t *xq,
                                               float *state_x, const void *w, int64_t m, int fmt_w, uint8_t *wq,
                                               uint8_t *wq_t, float *state_w, unsigned int *partials,
                                               hipStream_t stream);
hipError_t launch_quantize_rowwise_f8(const void *x, int64_t rows, int64_t cols, int fmt, uint8_t *codes, float *state,
                                      hipStream_t stream);
hipError_t launch_quantize_tensorwise_f8(const void *w, int64_t rows, int64_t cols, int fmt, uint8_t *codes,
                                         uint8_t *codes_t, float *state, unsigned int *partials, hipStream_t stream);
int num_compute_units();
// state_col == nullptr: tensor-wise weight state (state_tensor[0]); else one state per output column (SwitchBackQ).
hipError_t launch_gemm_i8_dequant(const int8_t *aq, const float *state_row, const int8_t *bq,
                                  const float *state_tensor, const float *state_col, int64_t M, int64_t N,
                                  int64_t K, void *out, sb_dtype out_dtype, hipStream_t stream);
// Tensor-wise int8 product whose dequantized value continues through y + bias[j] and gamma[j] * (.) (either vector may
// be nullptr); out SB_BF16 or SB_F32.
hipError_t launch_gemm_i8_dequant_post(const int8_t *aq, const float *state_row, const int8_t *bq,
                                       const float *state_tensor, const float *bias, const float *gamma, int64_t M,
                                       int64_t N, int64_t K, void *out, sb_dtype out_dtype, hipStream_t stream);
// 8-bit float product (fmt 0: E4M3, 1: E5M2 per operand): out[i,j] = (state_row[i] * state_tensor[0]) * sum_k a b.
// K % 128 == 0; out SB_BF16 or SB_F32.
hipError_t launch_gemm_f8_dequant(const uint8_t *aq, int fmt_a, const float *state_row, const uint8_t *bq, int fmt_b,
                                  const float *state_tensor, int64_t M, int64_t N, int64_t K, void *out,
                                  sb_dtype out_dtype, hipStream_t stream);
size_t gemm_bf16_tn_workspace_bytes(int64_t b, int64_t n, int64_t m);
hipError_t launch_gemm_bf16_tn(const void *dy, const void *x, int64_t b, int64_t n, int64_t m, void *dw,
                               sb_dtype dw_dtype, void *ws, hipStream_t stream);

size_t stable_adamw_workspace_bytes();
// b1_hat / b2_hat are the corrected decay rates, omb1 / omb2 their complements to one (all formed by the caller).
hipError_t launch_stable_adamw_step(float *theta, float *v, float *u, const void *grad, bool grad_bf16, int64_t count,
                                    float alpha, float b1_hat, float b2_hat, float omb1, float omb2, float eps,
                                    float lambda, float *rms_out, void *ws, hipStream_t stream);

int stable_adamw_blocks(int64_t count);  // workgroups a tensor of this many elements gets (single and batched launch)
hipError_t launch_stable_adamw_step_multi(const sb_adamw_tensor *table, int n, int total_blocks, bool grad_bf16,
                                          float alpha, float b1_hat, float b2_hat, float omb1, float omb2, float eps,
                                          float lambda, float *rms_out, void *ws, hipStream_t stream);

constexpr int kTensorwisePartials = 1024;  // upper bound on blocks of the tensor-wise absmax pass
constexpr int kAdamwPartials = 2048;  // upper bound on the workgroups of a StableAdamW step
constexpr int kColwiseRuns = 64;  // upper bound on the row runs of the column-wise absmax pass

}  // namespace sb
