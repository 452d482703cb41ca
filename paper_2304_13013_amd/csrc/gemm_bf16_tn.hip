// Host-side dispatch of the bf16 weight-gradient GEMM (kernel: gemm_bf16_tn_kernel.h) and its split-K reduction.
#include "gemm_bf16_tn_kernel.h"

#include <atomic>

namespace sb {
namespace {

// Two 64-token stages, four loader waves; a loader wave computes 3 of the 8 row blocks of its wave column, its SIMD
// partner 5 (with the tile walk below this measures 0-7 % faster than the even split on all four ViT-H shapes).
typedef GemmBf16Cfg<2, 4, 3> Cfg;
constexpr int MAX_SPLITS = 16;

__global__ __launch_bounds__(Cfg::THREADS) void gemm_bf16_tn_kernel(GemmBf16Args p) { gemm_bf16_tn_body<Cfg>(p); }

// out[e] = sum over splits (ascending) of partial[s][e]; four elements per thread.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const v4f *__restrict__ partial, int64_t quads,
                                                            int splits, void *__restrict__ out, int out_bf16) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= quads) return;
    v4f s = partial[i];
    for (int k = 1; k < splits; ++k) s += partial[(int64_t)k * quads + i];
    if (out_bf16)
        static_cast<v4bf *>(out)[i] = __builtin_convertvector(s, v4bf);
    else
        static_cast<v4f *>(out)[i] = s;
}

// Splits: fill the compute units in whole rounds with as few splits as that takes.
int choose_splits(int64_t b, int tiles) {
    const int ncu = num_compute_units();
    int best = 1;
    double best_score = -1.0;
    for (int s = 1; s <= MAX_SPLITS; ++s) {
        if ((int64_t)s * Cfg::BKT * 4 > b && s > 1) break;  // keep every split at least a few stages long
        const int blocks = tiles * s;
        const int rounds = (blocks + ncu - 1) / ncu;
        const double score = (double)blocks / (rounds * ncu) - 0.015 * s;
        if (score > best_score) {
            best_score = score;
            best = s;
        }
    }
    return best;
}

int tiles_of(int64_t n, int64_t m) {
    return (int)(((m + Cfg::BM - 1) / Cfg::BM) * ((n + Cfg::BN - 1) / Cfg::BN));
}

}  // namespace

size_t gemm_bf16_tn_workspace_bytes(int64_t b, int64_t n, int64_t m) {
    const int s = choose_splits(b, tiles_of(n, m));
    return s > 1 ? (size_t)s * (size_t)m * (size_t)n * sizeof(float) : 0;
}

hipError_t launch_gemm_bf16_tn(const void *dy, const void *x, int64_t b, int64_t n, int64_t m, void *dw,
                               sb_dtype dw_dtype, void *ws, hipStream_t stream) {
    static std::atomic<bool> attr_set{false};  // a second set by a racing host thread is harmless
    void (*kernel)(GemmBf16Args) = gemm_bf16_tn_kernel;
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    GemmBf16Args a;
    a.dy = static_cast<const unsigned short *>(dy);
    a.x = static_cast<const unsigned short *>(x);
    a.b = (int)b;
    a.n = (int)n;
    a.m = (int)m;
    a.tiles_m = (int)((m + Cfg::BM - 1) / Cfg::BM);
    a.tiles_n = (int)((n + Cfg::BN - 1) / Cfg::BN);
    a.splits = choose_splits(b, a.tiles_m * a.tiles_n);
    const int64_t stages = (b + Cfg::BKT - 1) / Cfg::BKT;
    a.k_per_split = (int)((stages + a.splits - 1) / a.splits) * Cfg::BKT;
    a.partial = static_cast<float *>(ws);
    a.out = dw;
    a.out_bf16 = dw_dtype == SB_BF16;
    const int total = a.tiles_m * a.tiles_n * a.splits;
    const int per_xcd = (total + 7) / 8, cus_per_xcd = num_compute_units() / 8 > 0 ? num_compute_units() / 8 : 1;
    const int grid = 8 * (per_xcd < cus_per_xcd ? per_xcd : cus_per_xcd);  // persistent: at most one workgroup per compute unit
    gemm_bf16_tn_kernel<<<grid, Cfg::THREADS, Cfg::LDS_BYTES, stream>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.splits == 1) return e;
    const int64_t quads = m * n / 4;
    splitk_reduce_kernel<<<(unsigned int)((quads + 255) / 256), 256, 0, stream>>>(
        static_cast<const v4f *>(ws), quads, a.splits, dw, a.out_bf16);
    return hipGetLastError();
}

}  // namespace sb
