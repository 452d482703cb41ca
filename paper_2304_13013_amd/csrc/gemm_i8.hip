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
    GemmI8Args args{aq, bq, state_row, state_tensor, out, (int)M, (int)N, (int)K, 0, 0, 8};
    typedef GemmI8Cfg<256, 256, 64, 2, 4, 4> Big;
    const int ncu = cached_num_cu();
    switch (out_dtype) {
        case SB_BF16: return launch_gemm_i8_cfg<Big, OUT_BF16>(args, ncu, stream);
        case SB_F32: return launch_gemm_i8_cfg<Big, OUT_F32>(args, ncu, stream);
        default: return launch_gemm_i8_cfg<Big, OUT_I32>(args, ncu, stream);
    }
}

}  // namespace sb
