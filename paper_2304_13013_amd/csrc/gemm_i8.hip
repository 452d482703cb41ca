// Host-side dispatch of the int8 GEMM with dequantizing epilogue (kernel: gemm_i8_kernel.h).
#include "gemm_i8_kernel.h"

namespace sb {
namespace {

int cached_num_cu() {
    static int n = 0;
    if (n == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            n = prop.multiProcessorCount;
        if (n <= 0) n = 256;
    }
    return n;
}

}  // namespace

hipError_t launch_gemm_i8_dequant(const int8_t *aq, const float *state_row, const int8_t *bq,
                                  const float *state_tensor, int64_t M, int64_t N, int64_t K, void *out,
                                  sb_dtype out_dtype, hipStream_t stream) {
    if (M == 0 || N == 0) return hipSuccess;
    GemmI8Args args{aq, bq, state_row, state_tensor, out, (int)M, (int)N, (int)K, 0, 0, 8, 0};
    // 256x256 tile.  128-byte k-steps (whole cache lines per row; two LDS stages plus the epilogue patch = 160 KiB)
    // when K allows it, else 64-byte k-steps with three stages.
    typedef GemmI8Cfg<256, 256, 128, 2, 4, 2, 1, 0, 0, 2, 1> K128;  // requests spread over two k-step groups, MFMA priority
    typedef GemmI8Cfg<256, 256, 64, 2, 4, 3, 0> K64;
    const int ncu = cached_num_cu();
    const bool wide = K % 128 == 0;
    switch (out_dtype) {
        case SB_BF16:
            return wide ? launch_gemm_i8_cfg<K128, OUT_BF16>(args, ncu, stream)
                        : launch_gemm_i8_cfg<K64, OUT_BF16>(args, ncu, stream);
        case SB_F32:
            return wide ? launch_gemm_i8_cfg<K128, OUT_F32>(args, ncu, stream)
                        : launch_gemm_i8_cfg<K64, OUT_F32>(args, ncu, stream);
        default:
            return wide ? launch_gemm_i8_cfg<K128, OUT_I32>(args, ncu, stream)
                        : launch_gemm_i8_cfg<K64, OUT_I32>(args, ncu, stream);
    }
}

}  // namespace sb
