// Host-side dispatch of the 8-bit float GEMM with dequantizing epilogue (the float8 variant of SwitchBack; kernel:
// gemm_i8_kernel.h with the float8 arithmetic selected).
#include "gemm_i8_kernel.h"

#include <atomic>

namespace sb {
namespace {

// 128-byte k-steps, two stages, four loader waves, even 4/4 split of the wave column: a float8 operand fragment is
// 8 registers, so the 5-block wave tile of the int8 kernel's uneven split does not fit the register file.
typedef GemmI8Cfg<128, 2, 4, 4, 1> F8Cfg;

#define SB_GEMM_F8_ENTRY(name, OUT, FW, FX)                                      \
    __global__ __launch_bounds__(F8Cfg::THREADS) void name(GemmI8Args p) {      \
        gemm_i8_dequant_body<F8Cfg, OUT, false, MATH_F8 + 2 * FW + FX>(p);       \
    }
// name suffix: format of the token-side operand a, then of the weight-side operand b (4 = E4M3, 5 = E5M2)
SB_GEMM_F8_ENTRY(gemm_f8_a4b4_bf16, OUT_BF16, 0, 0)
SB_GEMM_F8_ENTRY(gemm_f8_a4b4_f32, OUT_F32, 0, 0)
SB_GEMM_F8_ENTRY(gemm_f8_a5b4_bf16, OUT_BF16, 0, 1)
SB_GEMM_F8_ENTRY(gemm_f8_a5b4_f32, OUT_F32, 0, 1)
SB_GEMM_F8_ENTRY(gemm_f8_a4b5_bf16, OUT_BF16, 1, 0)
SB_GEMM_F8_ENTRY(gemm_f8_a4b5_f32, OUT_F32, 1, 0)
SB_GEMM_F8_ENTRY(gemm_f8_a5b5_bf16, OUT_BF16, 1, 1)
SB_GEMM_F8_ENTRY(gemm_f8_a5b5_f32, OUT_F32, 1, 1)
#undef SB_GEMM_F8_ENTRY

}  // namespace

hipError_t launch_gemm_f8_dequant(const uint8_t *aq, int fmt_a, const float *state_row, const uint8_t *bq, int fmt_b,
                                  const float *state_tensor, int64_t M, int64_t N, int64_t K, void *out,
                                  sb_dtype out_dtype, hipStream_t stream) {
    if (M == 0 || N == 0) return hipSuccess;
    typedef void (*Kernel)(GemmI8Args);
    static const Kernel kernels[8] = {gemm_f8_a4b4_bf16, gemm_f8_a4b4_f32, gemm_f8_a5b4_bf16, gemm_f8_a5b4_f32,
                                      gemm_f8_a4b5_bf16, gemm_f8_a4b5_f32, gemm_f8_a5b5_bf16, gemm_f8_a5b5_f32};
    static std::atomic<bool> attr_set[8];  // zero-initialized; a racing second set is harmless
    const int which = (fmt_b ? 4 : 0) + (fmt_a ? 2 : 0) + (out_dtype == SB_BF16 ? 0 : 1);
    if (!attr_set[which].load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernels[which]),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, F8Cfg::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set[which].store(true, std::memory_order_release);
    }
    GemmI8Args args{reinterpret_cast<const int8_t *>(aq), reinterpret_cast<const int8_t *>(bq), state_row, state_tensor,
                    nullptr, out, (int)M, (int)N, (int)K, 0, 0, 8};
    int grid = 0;
    gemm_i8_prepare<F8Cfg>(args, num_compute_units(), &grid);
    kernels[which]<<<grid, F8Cfg::THREADS, F8Cfg::LDS_BYTES, stream>>>(args);
    return hipGetLastError();
}

}  // namespace sb
