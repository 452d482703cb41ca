// Measured ceilings of the GPU the library runs on: what the matrix pipes and the memory system deliver to code that
// does nothing else, so that the fraction of the published peak a product kernel reaches can be read against what the
// chip sustains.  Measurement aids only (include/switchback_ceilings.h); no step of the layer runs through them.
//
//   * matrix-instruction loops: every wave keeps a set of operand fragments in registers (as many as the product kernels
//     hold: four token-side and two weight-side fragments for each of two k-steps) and issues the sixteen
//     (fragment, fragment) products of the set over and over.  No LDS, no memory traffic inside the loop.  The
//     fragments are read once from caller-supplied code buffers, so the same loop can run on all-zero operands, on
//     uniform random codes and on the codes the quantizers of this library produce from a workload: the matrix pipes draw
//     power according to how many operand bits toggle, and the clock the GPU holds depends on it.
//   * a plain copy: 16 bytes per lane, grid-stride, read once and written once.
#include "sb_common.h"

namespace sb {
namespace {

enum { CEIL_I8 = 0, CEIL_BF16 = 1, CEIL_F8 = 2 };

constexpr int kFragsA = 4, kFragsB = 2, kBufs = 2;  // the register fragment set of the product kernels

template <int KIND>
struct CeilTraits;
template <>
struct CeilTraits<CEIL_I8> {
    typedef v4i Frag;
    typedef v16i Acc;
    static __device__ __forceinline__ Acc mma(Frag b, Frag a, Acc c) { return __builtin_amdgcn_mfma_i32_32x32x32_i8(b, a, c, 0, 0, 0); }
};
template <>
struct CeilTraits<CEIL_BF16> {
    typedef v8bf Frag;
    typedef v16f Acc;
    static __device__ __forceinline__ Acc mma(Frag b, Frag a, Acc c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, c, 0, 0, 0); }
};
template <>
struct CeilTraits<CEIL_F8> {
    typedef v8i Frag;
    typedef v16f Acc;
    static __device__ __forceinline__ Acc mma(Frag b, Frag a, Acc c) {
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b, a, c, 0, 0, 0, 0, 0, 0);  // E4M3 x E4M3
    }
};

// a, b: operand bytes; wave w of the grid takes fragment f of operand a at byte (w * frags + f) * 64 * sizeof(Frag)
// modulo the buffer length (a_bytes, b_bytes: multiples of 64 * sizeof(Frag)).  sink receives one value per lane so that
// the accumulators stay live.
template <int KIND>
__device__ __forceinline__ void mfma_loop_body(const unsigned char *a, size_t a_bytes, const unsigned char *b,
                                               size_t b_bytes, int iters, float *sink) {
    typedef CeilTraits<KIND> T;
    typedef typename T::Frag Frag;
    typedef typename T::Acc Acc;
    const int lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    constexpr size_t kWaveFrag = 64 * sizeof(Frag);
    Frag fa[kBufs][kFragsA], fb[kBufs][kFragsB];
#pragma unroll
    for (int u = 0; u < kBufs; ++u) {
#pragma unroll
        for (int i = 0; i < kFragsA; ++i) {
            const size_t off = ((wave * kBufs + u) * kFragsA + i) * kWaveFrag % a_bytes;
            fa[u][i] = *reinterpret_cast<const Frag *>(a + off + lane * sizeof(Frag));
        }
#pragma unroll
        for (int i = 0; i < kFragsB; ++i) {
            const size_t off = ((wave * kBufs + u) * kFragsB + i) * kWaveFrag % b_bytes;
            fb[u][i] = *reinterpret_cast<const Frag *>(b + off + lane * sizeof(Frag));
        }
    }
    Acc acc[kFragsA][kFragsB];
#pragma unroll
    for (int i = 0; i < kFragsA; ++i)
#pragma unroll
        for (int j = 0; j < kFragsB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kBufs; ++u)
#pragma unroll
            for (int i = 0; i < kFragsA; ++i)
#pragma unroll
                for (int j = 0; j < kFragsB; ++j) acc[i][j] = T::mma(fb[u][j], fa[u][i], acc[i][j]);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < kFragsA; ++i)
#pragma unroll
        for (int j = 0; j < kFragsB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += (float)acc[i][j][r];
    sink[wave * 64 + lane] = s;
}

__global__ __launch_bounds__(512) void ceiling_mfma_i8_kernel(const unsigned char *a, size_t a_bytes,
                                                              const unsigned char *b, size_t b_bytes, int iters,
                                                              float *sink) {
    mfma_loop_body<CEIL_I8>(a, a_bytes, b, b_bytes, iters, sink);
}
__global__ __launch_bounds__(512) void ceiling_mfma_bf16_kernel(const unsigned char *a, size_t a_bytes,
                                                                const unsigned char *b, size_t b_bytes, int iters,
                                                                float *sink) {
    mfma_loop_body<CEIL_BF16>(a, a_bytes, b, b_bytes, iters, sink);
}
__global__ __launch_bounds__(512) void ceiling_mfma_f8_kernel(const unsigned char *a, size_t a_bytes,
                                                              const unsigned char *b, size_t b_bytes, int iters,
                                                              float *sink) {
    mfma_loop_body<CEIL_F8>(a, a_bytes, b, b_bytes, iters, sink);
}

__global__ __launch_bounds__(256) void ceiling_copy_kernel(const v4u *__restrict__ src, v4u *__restrict__ dst,
                                                           size_t chunks) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < chunks; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace
}  // namespace sb

extern "C" {

int switchback_ceiling_mfma(int kind, const void *a_codes, size_t a_bytes, const void *b_codes, size_t b_bytes,
                            int workgroups, int waves_per_workgroup, int iters, float *sink, double *ops_out,
                            void *stream) {
    using namespace sb;
    if (kind < CEIL_I8 || kind > CEIL_F8 || workgroups <= 0 || iters <= 0) return SB_INVALID_ARG;
    if (waves_per_workgroup != 4 && waves_per_workgroup != 8) return SB_INVALID_ARG;
    const size_t frag = kind == CEIL_F8 ? 32 * 64 : 16 * 64;  // bytes one wave reads per fragment
    if (a_codes == nullptr || b_codes == nullptr || sink == nullptr || !aligned16(a_codes) || !aligned16(b_codes))
        return SB_INVALID_ARG;
    if (a_bytes < frag || b_bytes < frag || a_bytes % frag || b_bytes % frag) return SB_INVALID_ARG;
    const unsigned char *a = static_cast<const unsigned char *>(a_codes), *b = static_cast<const unsigned char *>(b_codes);
    const dim3 grid((unsigned)workgroups), block((unsigned)waves_per_workgroup * 64);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (kind == CEIL_I8)
        ceiling_mfma_i8_kernel<<<grid, block, 0, s>>>(a, a_bytes, b, b_bytes, iters, sink);
    else if (kind == CEIL_BF16)
        ceiling_mfma_bf16_kernel<<<grid, block, 0, s>>>(a, a_bytes, b, b_bytes, iters, sink);
    else
        ceiling_mfma_f8_kernel<<<grid, block, 0, s>>>(a, a_bytes, b, b_bytes, iters, sink);
    if (ops_out) {
        // multiply-adds count two operations: 32x32x32 (int8), 32x32x16 (bf16), 32x32x64 (float8) per instruction
        const double per_instr = 2.0 * 32 * 32 * (kind == CEIL_I8 ? 32 : kind == CEIL_BF16 ? 16 : 64);
        *ops_out = per_instr * kBufs * kFragsA * kFragsB * (double)iters * (double)workgroups * waves_per_workgroup;
    }
    return hipGetLastError() == hipSuccess ? SB_OK : SB_HIP_ERROR;
}

int switchback_ceiling_copy(const void *src, void *dst, size_t bytes, void *stream) {
    if (src == nullptr || dst == nullptr || !sb::aligned16(src) || !sb::aligned16(dst) || bytes % 16) return SB_INVALID_ARG;
    if (bytes == 0) return SB_OK;
    const size_t chunks = bytes / 16;
    size_t blocks = (chunks + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    sb::ceiling_copy_kernel<<<(unsigned)blocks, 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const sb::v4u *>(src), static_cast<sb::v4u *>(dst), chunks);
    return hipGetLastError() == hipSuccess ? SB_OK : SB_HIP_ERROR;
}

}  // extern "C"
