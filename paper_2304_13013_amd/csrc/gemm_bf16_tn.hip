// Host-side dispatch of the bf16 weight-gradient GEMM (kernel: gemm_bf16_tn_kernel.h) and its split-K reduction.
#include "gemm_bf16_tn_kernel.h"

#include <atomic>

namespace sb {
namespace {

// Two 64-token stages, four loader waves; a loader wave computes 3 of the 8 row blocks of its wave column, its SIMD
// partner 5 (with the tile walk below this measures 0-7 % faster than the even split on all four ViT-H shapes).
typedef GemmBf16Cfg<2, 4, 3> Big;
// 128 x 128 tiles, four waves (all load), two workgroups per compute unit: for weight gradients that the large tile
// could only spread over the GPU by cutting the token range into many short pieces, where the start and end of an item
// weigh more than the doubled operand traffic (ViT-B/16 sized layers: 10-29 % faster; within 5 % of the large tile at
// equal fill, slower on every ViT-L and ViT-H layer but ViT-L's 1024 x 1024 projection).
typedef GemmBf16Cfg<2, 4, 2, 64, 128, 2, 2> Small;
static_assert(Big::BKT == Small::BKT, "the split lengths below are in stages of either instance");
constexpr int MAX_SPLITS = 16;
constexpr int kShortItemStages = 32;  // below this many stages per work item the large tile loses to the small one

__global__ __launch_bounds__(Big::THREADS) void gemm_bf16_tn_kernel(GemmBf16Args p) { gemm_bf16_tn_body<Big>(p); }
__global__ __launch_bounds__(Small::THREADS) __attribute__((amdgpu_waves_per_eu(2))) void gemm_bf16_tn_small_kernel(
    GemmBf16Args p) {
    gemm_bf16_tn_body<Small>(p);
}

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

// Splits of the large-tile instance: fill the compute units in whole rounds with as few splits as that takes, every
// split at least four stages long.
int choose_splits_big(int64_t b, int tiles, int ncu) {
    int best = 1;
    double best_score = -1.0;
    for (int s = 1; s <= MAX_SPLITS; ++s) {
        if ((int64_t)s * Big::BKT * 4 > b && s > 1) break;
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

// Splits of the small-tile instance: its items are short, so rounds and the passes over the partial sums decide.  The
// split count minimises a time model fitted to measurements on the ViT-B/L/H layer shapes (it picks the best or
// second-best count on all of them), in units of one stage of a workgroup that shares its compute unit (1.1 us):
// every round of the persistent grid costs the stages of an item, at 0.64 of the unit while the round has at most one
// workgroup per compute unit and rising linearly to the full unit at two; the partial sums are written once and read
// once per split, plus the output pass, at 2.9 TB/s.
int choose_splits_small(int64_t b, int tiles, int ncu, int64_t m, int64_t n) {
    const int64_t stages = (b + Small::BKT - 1) / Small::BKT;
    const double pass = (double)m * (double)n * 4.0 / (2.9e12 * 1.1e-6);  // one pass over m x n floats, in stage units
    int best = 1;
    double best_cost = 0.0;
    for (int s = 1; s <= MAX_SPLITS; ++s) {
        if ((int64_t)s * Small::BKT * 4 > b && s > 1) break;
        const double per_item = (double)((stages + s - 1) / s);
        double cost = s > 1 ? (s + 0.5) * pass : 0.0;
        for (int left = tiles * s; left > 0; left -= 2 * ncu) {
            const int k = left < 2 * ncu ? left : 2 * ncu;
            cost += per_item * (k <= ncu ? 0.64 : 0.64 + 0.36 * (double)(k - ncu) / ncu);
        }
        if (s == 1 || cost < best_cost) {
            best_cost = cost;
            best = s;
        }
    }
    return best;
}

struct Plan {
    bool small;
    int tiles_m, tiles_n, splits, k_per_split;
};

// The instance and the split count are functions of the shape alone, so the workspace query and the launch agree.
Plan plan_of(int64_t b, int64_t n, int64_t m) {
    const int ncu = num_compute_units();
    const int64_t stages = (b + Big::BKT - 1) / Big::BKT;
    Plan p;
    p.small = false;
    p.tiles_m = (int)((m + Big::BM - 1) / Big::BM);
    p.tiles_n = (int)((n + Big::BN - 1) / Big::BN);
    p.splits = choose_splits_big(b, p.tiles_m * p.tiles_n, ncu);
    if (p.splits > 1 && stages / p.splits < kShortItemStages) {
        p.small = true;
        p.tiles_m = (int)((m + Small::BM - 1) / Small::BM);
        p.tiles_n = (int)((n + Small::BN - 1) / Small::BN);
        p.splits = choose_splits_small(b, p.tiles_m * p.tiles_n, ncu, m, n);
    }
    p.k_per_split = (int)((stages + p.splits - 1) / p.splits) * Big::BKT;
    return p;
}

template <class C>
hipError_t set_lds_limit_once(void (*kernel)(GemmBf16Args), std::atomic<bool> &done) {
    if (done.load(std::memory_order_acquire)) return hipSuccess;  // a second set by a racing host thread is harmless
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e == hipSuccess) done.store(true, std::memory_order_release);
    return e;
}

}  // namespace

size_t gemm_bf16_tn_workspace_bytes(int64_t b, int64_t n, int64_t m) {
    const int s = plan_of(b, n, m).splits;
    return s > 1 ? (size_t)s * (size_t)m * (size_t)n * sizeof(float) : 0;
}

hipError_t launch_gemm_bf16_tn(const void *dy, const void *x, int64_t b, int64_t n, int64_t m, void *dw,
                               sb_dtype dw_dtype, void *ws, hipStream_t stream) {
    static std::atomic<bool> big_set{false}, small_set{false};
    const Plan plan = plan_of(b, n, m);
    hipError_t e = plan.small ? set_lds_limit_once<Small>(gemm_bf16_tn_small_kernel, small_set)
                              : set_lds_limit_once<Big>(gemm_bf16_tn_kernel, big_set);
    if (e != hipSuccess) return e;
    GemmBf16Args a;
    a.dy = static_cast<const unsigned short *>(dy);
    a.x = static_cast<const unsigned short *>(x);
    a.b = (int)b;
    a.n = (int)n;
    a.m = (int)m;
    a.tiles_m = plan.tiles_m;
    a.tiles_n = plan.tiles_n;
    a.splits = plan.splits;
    a.k_per_split = plan.k_per_split;
    a.partial = static_cast<float *>(ws);
    a.out = dw;
    a.out_bf16 = dw_dtype == SB_BF16;
    // Persistent grid: at most as many workgroups as the GPU holds at once, the same number on every XCD.
    const int total = a.tiles_m * a.tiles_n * a.splits;
    const int per_xcd = (total + 7) / 8, cus_per_xcd = num_compute_units() / 8 > 0 ? num_compute_units() / 8 : 1;
    const int slots_per_xcd = cus_per_xcd * (plan.small ? 2 : 1);
    const int grid = 8 * (per_xcd < slots_per_xcd ? per_xcd : slots_per_xcd);
    if (plan.small)
        gemm_bf16_tn_small_kernel<<<grid, Small::THREADS, Small::LDS_BYTES, stream>>>(a);
    else
        gemm_bf16_tn_kernel<<<grid, Big::THREADS, Big::LDS_BYTES, stream>>>(a);
    e = hipGetLastError();
    if (e != hipSuccess || a.splits == 1) return e;
    const int64_t quads = m * n / 4;
    splitk_reduce_kernel<<<(unsigned int)((quads + 255) / 256), 256, 0, stream>>>(
        static_cast<const v4f *>(ws), quads, a.splits, dw, a.out_bf16);
    return hipGetLastError();
}

}  // namespace sb
