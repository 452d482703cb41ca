// Host-side dispatch of the int8 GEMM with dequantizing epilogue (kernel: gemm_i8_kernel.h).
#include "gemm_i8_kernel.h"

#include <atomic>

namespace sb {
namespace {

// 128-byte k-steps (whole cache lines per row; two LDS stages plus the epilogue patch = 160 KiB) when K allows
// it: four loader waves with a 3-block wave tile, their SIMD partners take 5 blocks (see the kernel header).  Else
// 64-byte k-steps with four stages, every wave loading.
typedef GemmI8Cfg<128, 2, 4, 3, 1> K128;
typedef GemmI8Cfg<64, 4, 8, 4, 1> K64;
// Row-and-column scales (SwitchBackQ): the 32 column states a lane keeps need the registers of the even split.
typedef GemmI8Cfg<128, 2, 4, 4, 1> K128Q;

#define SB_GEMM_I8_ENTRY(name, CFG, OUT) \
    __global__ __launch_bounds__(CFG::THREADS) void name(GemmI8Args p) { gemm_i8_dequant_body<CFG, OUT>(p); }
SB_GEMM_I8_ENTRY(gemm_i8_k128_bf16, K128, OUT_BF16)
SB_GEMM_I8_ENTRY(gemm_i8_k128_f32, K128, OUT_F32)
SB_GEMM_I8_ENTRY(gemm_i8_k128_i32, K128, OUT_I32)
SB_GEMM_I8_ENTRY(gemm_i8_k64_bf16, K64, OUT_BF16)
SB_GEMM_I8_ENTRY(gemm_i8_k64_f32, K64, OUT_F32)
SB_GEMM_I8_ENTRY(gemm_i8_k64_i32, K64, OUT_I32)
#define SB_GEMM_I8_ENTRY_Q(name, CFG, OUT) \
    __global__ __launch_bounds__(CFG::THREADS) void name(GemmI8Args p) { gemm_i8_dequant_body<CFG, OUT, true>(p); }
SB_GEMM_I8_ENTRY_Q(gemm_i8q_k128_bf16, K128Q, OUT_BF16)
SB_GEMM_I8_ENTRY_Q(gemm_i8q_k128_f32, K128Q, OUT_F32)
SB_GEMM_I8_ENTRY_Q(gemm_i8q_k64_bf16, K64, OUT_BF16)
SB_GEMM_I8_ENTRY_Q(gemm_i8q_k64_f32, K64, OUT_F32)
#undef SB_GEMM_I8_ENTRY_Q
#undef SB_GEMM_I8_ENTRY

template <class C>
hipError_t launch(void (*kernel)(GemmI8Args), std::atomic<bool> *attr_set, GemmI8Args args, hipStream_t stream) {
    if (!attr_set->load(std::memory_order_acquire)) {  // setting it twice (two host threads racing) is harmless
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set->store(true, std::memory_order_release);
    }
    int grid = 0;
    gemm_i8_prepare<C>(args, num_compute_units(), &grid);
    kernel<<<grid, C::THREADS, C::LDS_BYTES, stream>>>(args);
    return hipGetLastError();
}

}  // namespace

// Compute units of the current device (queried once per process; the library serves one GPU).  Host threads may race
// to the first query: both store the same value.
int num_compute_units() {
    static std::atomic<int> cached{0};
    int n = cached.load(std::memory_order_relaxed);
    if (n == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            n = prop.multiProcessorCount;
        if (n <= 0) n = 256;  // no device visible (host-only callers sizing a workspace): an MI355X has 256
        cached.store(n, std::memory_order_relaxed);
    }
    return n;
}

hipError_t launch_gemm_i8_dequant(const int8_t *aq, const float *state_row, const int8_t *bq,
                                  const float *state_tensor, const float *state_col, int64_t M, int64_t N,
                                  int64_t K, void *out, sb_dtype out_dtype, hipStream_t stream) {
    if (M == 0 || N == 0) return hipSuccess;
    GemmI8Args args{aq, bq, state_row, state_tensor, state_col, out, (int)M, (int)N, (int)K, 0, 0, 8};
    if (state_col != nullptr && out_dtype != SB_I32_RAW) {
        static std::atomic<bool> q_attr_set[4];  // zero-initialized
        if (K % 128 == 0)
            return out_dtype == SB_BF16 ? launch<K128Q>(gemm_i8q_k128_bf16, &q_attr_set[0], args, stream)
                                        : launch<K128Q>(gemm_i8q_k128_f32, &q_attr_set[1], args, stream);
        return out_dtype == SB_BF16 ? launch<K64>(gemm_i8q_k64_bf16, &q_attr_set[2], args, stream)
                                    : launch<K64>(gemm_i8q_k64_f32, &q_attr_set[3], args, stream);
    }
    static std::atomic<bool> attr_set[6];  // zero-initialized
    const bool wide = K % 128 == 0;
    switch (out_dtype) {
        case SB_BF16:
            return wide ? launch<K128>(gemm_i8_k128_bf16, &attr_set[0], args, stream)
                        : launch<K64>(gemm_i8_k64_bf16, &attr_set[3], args, stream);
        case SB_F32:
            return wide ? launch<K128>(gemm_i8_k128_f32, &attr_set[1], args, stream)
                        : launch<K64>(gemm_i8_k64_f32, &attr_set[4], args, stream);
        default:
            return wide ? launch<K128>(gemm_i8_k128_i32, &attr_set[2], args, stream)
                        : launch<K64>(gemm_i8_k64_i32, &attr_set[5], args, stream);
    }
}

}  // namespace sb
