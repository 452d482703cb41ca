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
// Products with few output tiles (ViT-B/16's 768-wide outputs make 75 tiles of 256x256 for 256 compute units):
// 128x128 tiles, four waves, two workgroups per compute unit.  Twice the operand bytes per multiply-add, so it loses
// to the large tile as soon as that one fills the GPU (measured: 26 against 33 us at 75 large tiles, 26 against 24 us
// at 300).
typedef GemmI8Cfg<128, 2, 4, 2, 1, 128, 128, 2, 2> K128S;

#define SB_GEMM_I8_ENTRY(name, CFG, OUT) \
    __global__ __launch_bounds__(CFG::THREADS) void name(GemmI8Args p) { gemm_i8_dequant_body<CFG, OUT>(p); }
SB_GEMM_I8_ENTRY(gemm_i8_k128_bf16, K128, OUT_BF16)
SB_GEMM_I8_ENTRY(gemm_i8_k128_f32, K128, OUT_F32)
SB_GEMM_I8_ENTRY(gemm_i8_k128_i32, K128, OUT_I32)
SB_GEMM_I8_ENTRY(gemm_i8_k64_bf16, K64, OUT_BF16)
SB_GEMM_I8_ENTRY(gemm_i8_k64_f32, K64, OUT_F32)
SB_GEMM_I8_ENTRY(gemm_i8_k64_i32, K64, OUT_I32)
// Two waves per SIMD for the four-wave configuration (two workgroups per compute unit): at most 256 registers per lane.
#define SB_GEMM_I8_ENTRY_S(name, CFG, OUT)                                                                     \
    __global__ __launch_bounds__(CFG::THREADS) __attribute__((amdgpu_waves_per_eu(2))) void name(GemmI8Args p) { \
        gemm_i8_dequant_body<CFG, OUT>(p);                                                                     \
    }
SB_GEMM_I8_ENTRY_S(gemm_i8_k128s_bf16, K128S, OUT_BF16)
SB_GEMM_I8_ENTRY_S(gemm_i8_k128s_f32, K128S, OUT_F32)
SB_GEMM_I8_ENTRY_S(gemm_i8_k128s_i32, K128S, OUT_I32)
#undef SB_GEMM_I8_ENTRY_S
#define SB_GEMM_I8_ENTRY_Q(name, CFG, OUT) \
    __global__ __launch_bounds__(CFG::THREADS) void name(GemmI8Args p) { gemm_i8_dequant_body<CFG, OUT, true>(p); }
SB_GEMM_I8_ENTRY_Q(gemm_i8q_k128_bf16, K128Q, OUT_BF16)
SB_GEMM_I8_ENTRY_Q(gemm_i8q_k128_f32, K128Q, OUT_F32)
SB_GEMM_I8_ENTRY_Q(gemm_i8q_k64_bf16, K64, OUT_BF16)
SB_GEMM_I8_ENTRY_Q(gemm_i8q_k64_f32, K64, OUT_F32)
#undef SB_GEMM_I8_ENTRY_Q
#undef SB_GEMM_I8_ENTRY
// Bias and layer-scale after the dequantization: the even wave split (the two vectors take 64 registers in the epilogue).
#define SB_GEMM_I8_ENTRY_P(name, CFG, OUT)                                                                     \
    __global__ __launch_bounds__(CFG::THREADS) __attribute__((amdgpu_waves_per_eu(2))) void name(GemmI8Args p) { \
        gemm_i8_dequant_body<CFG, OUT, false, MATH_I8, true>(p);                                               \
    }
SB_GEMM_I8_ENTRY_P(gemm_i8p_k128_bf16, K128Q, OUT_BF16)
SB_GEMM_I8_ENTRY_P(gemm_i8p_k128_f32, K128Q, OUT_F32)
SB_GEMM_I8_ENTRY_P(gemm_i8p_k64_bf16, K64, OUT_BF16)
SB_GEMM_I8_ENTRY_P(gemm_i8p_k64_f32, K64, OUT_F32)
SB_GEMM_I8_ENTRY_P(gemm_i8p_k128s_bf16, K128S, OUT_BF16)
SB_GEMM_I8_ENTRY_P(gemm_i8p_k128s_f32, K128S, OUT_F32)
#undef SB_GEMM_I8_ENTRY_P

template <class C>
hipError_t launch(void (*kernel)(GemmI8Args), std::atomic<bool> *attr_set, GemmI8Args args, hipStream_t stream) {
    if (!attr_set->load(std::memory_order_acquire)) {  // setting it twice (two host threads racing) is harmless
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set->store(true, std::memory_order_release);
    }
    int grid = 0;
    // Workgroups that fit a compute unit at once: its 160 KiB of LDS decide (registers allow two waves per SIMD).
    constexpr int per_cu = C::LDS_BYTES * 2 <= 160 * 1024 && C::NWAVES == 4 ? 2 : 1;
    gemm_i8_prepare<C>(args, num_compute_units() * per_cu, &grid);
    kernel<<<grid, C::THREADS, C::LDS_BYTES, stream>>>(args);
    return hipGetLastError();
}

// Few large tiles: fewer than half as many 256x256 tiles as compute units.
bool few_tiles(int64_t M, int64_t N) {
    const int64_t tiles = ((M + 255) / 256) * ((N + 255) / 256);
    return tiles * 2 <= num_compute_units();
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

hipError_t launch_gemm_i8_dequant_post(const int8_t *aq, const float *state_row, const int8_t *bq,
                                       const float *state_tensor, const float *bias, const float *gamma, int64_t M,
                                       int64_t N, int64_t K, void *out, sb_dtype out_dtype, hipStream_t stream) {
    if (M == 0 || N == 0) return hipSuccess;
    GemmI8Args args{aq, bq, state_row, state_tensor, nullptr, out, (int)M, (int)N, (int)K, 0, 0, 8, bias, gamma};
    static std::atomic<bool> attr_set[6];  // zero-initialized
    const bool bf = out_dtype == SB_BF16;
    if (K % 128 != 0)
        return bf ? launch<K64>(gemm_i8p_k64_bf16, &attr_set[0], args, stream)
                  : launch<K64>(gemm_i8p_k64_f32, &attr_set[1], args, stream);
    if (few_tiles(M, N))
        return bf ? launch<K128S>(gemm_i8p_k128s_bf16, &attr_set[2], args, stream)
                  : launch<K128S>(gemm_i8p_k128s_f32, &attr_set[3], args, stream);
    return bf ? launch<K128Q>(gemm_i8p_k128_bf16, &attr_set[4], args, stream)
              : launch<K128Q>(gemm_i8p_k128_f32, &attr_set[5], args, stream);
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
    static std::atomic<bool> attr_set[9];  // zero-initialized
    const bool wide = K % 128 == 0;
    if (wide && few_tiles(M, N)) {
        switch (out_dtype) {
            case SB_BF16: return launch<K128S>(gemm_i8_k128s_bf16, &attr_set[6], args, stream);
            case SB_F32: return launch<K128S>(gemm_i8_k128s_f32, &attr_set[7], args, stream);
            default: return launch<K128S>(gemm_i8_k128s_i32, &attr_set[8], args, stream);
        }
    }
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
