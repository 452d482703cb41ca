// int8 x int8 -> int32 GEMM with the dequantizing epilogue of the SwitchBack forward / input-gradient products
// (the dequantized forward equation of Section 2.2.1 of arxiv 2304.13013), hand-written for gfx950.
//
//   out[i,j] = (state_tensor/127^2 * state_row[i]) * sum_k aq[i,k] * bq[j,k]        aq [M,K], bq [N,K], K contiguous
//
// Design
//   * v_mfma_i32_32x32x32_i8.  The weight-side tile (bq rows) is the MFMA's first operand and the token-side
//     tile (aq rows) its second, so a lane ends up owning ONE output row (lane % 32) and, per accumulator quad,
//     four consecutive output columns: one row scale per lane, and packed bf16x4 leaves each quad.
//   * A persistent grid (one workgroup per compute unit) walks the output tiles in an order that keeps the 32
//     workgroups of one XCD (workgroup id % 8) on a compact patch of tiles, so its L2 sees each operand panel once.
//   * Operand tiles go HBM/L2 -> LDS with global_load_lds_dwordx4 (no VGPR staging), STAGES deep.  One wave
//     instruction fills 1 KiB of LDS linearly, so the bank-conflict-avoiding swizzle is applied on the GLOBAL side:
//     LDS slot (row, p) holds 16-byte k-chunk p ^ f(row) of that row, f(row) = (row / (256/BK)) % (BK/16).
//   * The next tile's first stages are requested BEFORE the epilogue of the current tile, whose bf16 results are
//     transposed through a wave-private LDS patch and leave as 16-byte stores covering full 128-byte row segments.
//   * Rows past M (and weight rows past N) are clamped on load and masked on store; an out-of-range row only ever
//     feeds accumulators that are never stored.
#include "sb_common.h"

namespace sb {
namespace {

enum { OUT_BF16 = 0, OUT_F32 = 1, OUT_I32 = 2 };

template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int STAGES_>
struct GemmI8Cfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, STAGES = STAGES_;
    static constexpr int NWAVES = WAVES_M * WAVES_N, THREADS = NWAVES * 64;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;  // wave tile
    static constexpr int MT = WTM / 32, NT = WTN / 32;            // 32x32 MFMA blocks per wave tile
    static constexpr int KK = BK / 32;                            // MFMA k-steps per stage
    static constexpr int CPR = BK / 16;                           // 16-byte chunks per tile row
    static constexpr int RPS = 1024 / BK;                         // tile rows per 1 KiB slab (one wave load)
    static constexpr int SWZ_DIV = 256 / BK;                      // rows that share one 256-byte bank window
    static constexpr int STAGE_BYTES = (BM + BN) * BK;
    static constexpr int NSLAB = STAGE_BYTES / 1024;
    static constexpr int LPW = NSLAB / NWAVES;                    // global->LDS loads per wave per stage
    static constexpr int EPI_STRIDE = WTN * 2 + 16;               // bytes per row of the epilogue patch
    static constexpr int EPI_WAVE_BYTES = 32 * EPI_STRIDE;
    static constexpr int EPI_STORES = MT * (32 * WTN * 2 / 1024); // 16-byte global stores per lane per tile
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES + NWAVES * EPI_WAVE_BYTES;
    static_assert(BK == 64 || BK == 128, "BK");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && NSLAB % NWAVES == 0, "tile shape");
    static_assert((32 * WTN * 2) % 1024 == 0, "epilogue patch must be whole wave reads");
    static_assert(LPW * (STAGES - 2) + EPI_STORES < 64, "vmcnt range");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

struct GemmI8Args {
    const int8_t *a;
    const int8_t *b;
    const float *state_row;
    const float *state_tensor;
    void *out;
    int M, N, K;
    int tiles_m, tiles_n;
};

// Output tile visited by workgroup `wg` in its `round`-th iteration.  Workgroups are dealt to XCDs round-robin,
// so the G/8 workgroups with equal wg % 8 share an L2; they get consecutive ids in an order that walks groups
// of GROUP_M tile-rows column by column (a patch GROUP_M tiles tall and (G/8)/GROUP_M wide per XCD per round).
__device__ __forceinline__ bool tile_of(int wg, int round, int nwg, int tiles_m, int tiles_n, int *tm, int *tn) {
    constexpr int GROUP_M = 8;
    const int per_xcd = nwg >> 3;
    const int id = (round * 8 + (wg & 7)) * per_xcd + (wg >> 3);
    if (id >= tiles_m * tiles_n) return false;
    const int per_group = GROUP_M * tiles_n;
    const int first_m = (id / per_group) * GROUP_M;
    const int group_rows = min(tiles_m - first_m, GROUP_M);
    const int r = id % per_group;
    *tm = first_m + r % group_rows;
    *tn = r / group_rows;
    return true;
}

// Workgroup barrier WITHOUT the memory fence of __syncthreads(): the fence would drain every outstanding
// global->LDS request (vmcnt(0)) and serialize the pipeline.  The explicit vmcnt waits in front of it order
// the LDS fills; LDS reads of a stage have returned before the MFMAs that consume them were issued.
__device__ __forceinline__ void block_barrier() { asm volatile("s_barrier" ::: "memory"); }

template <class C, int OUT>
__global__ __launch_bounds__(C::THREADS) void gemm_i8_dequant_kernel(GemmI8Args p) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    typedef __attribute__((address_space(3))) void lds_void;
    typedef const __attribute__((address_space(1))) void gbl_void;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / C::WAVES_N) * C::WTM, wn0 = (wave % C::WAVES_N) * C::WTN;
    const int KT = p.K / C::BK;

    // Per-lane byte offset of its MFMA operand chunk inside a 32-row block of a stage, one per k-step.
    const int frow = lane & 31;
    const int fswz = (frow / C::SWZ_DIV) % C::CPR;
    int frag_off[C::KK];
#pragma unroll
    for (int kk = 0; kk < C::KK; ++kk) frag_off[kk] = frow * C::BK + (((kk * 2 + (lane >> 5)) ^ fswz) << 4);

    // Loader role of this lane: slab s = wave*LPW + i covers stage rows [s*RPS, (s+1)*RPS).
    const int lrow_in_slab = lane / C::CPR, lpos = lane % C::CPR;

    unsigned char *epi = smem + C::STAGES * C::STAGE_BYTES + wave * C::EPI_WAVE_BYTES;

    const int8_t *gsrc[C::LPW];
    auto set_tile_sources = [&](int tm, int tn) {
#pragma unroll
        for (int i = 0; i < C::LPW; ++i) {
            const int srow = (wave * C::LPW + i) * C::RPS + lrow_in_slab;
            const int chunk = lpos ^ ((srow / C::SWZ_DIV) % C::CPR);
            if (srow < C::BM) {
                const int r = min(tm * C::BM + srow, p.M - 1);
                gsrc[i] = p.a + (int64_t)r * p.K + chunk * 16;
            } else {
                const int r = min(tn * C::BN + (srow - C::BM), p.N - 1);
                gsrc[i] = p.b + (int64_t)r * p.K + chunk * 16;
            }
        }
    };
    auto issue_stage = [&](int kt) {
        unsigned char *dst = smem + (kt % C::STAGES) * C::STAGE_BYTES + wave * C::LPW * 1024;
#pragma unroll
        for (int i = 0; i < C::LPW; ++i)
            __builtin_amdgcn_global_load_lds((gbl_void *)(gsrc[i] + (int64_t)kt * C::BK), (lds_void *)(dst + i * 1024),
                                             16, 0, 0);
    };

    int tm, tn;
    bool have = tile_of(blockIdx.x, 0, gridDim.x, p.tiles_m, p.tiles_n, &tm, &tn);
    if (have) {
        set_tile_sources(tm, tn);
#pragma unroll
        for (int s = 0; s < C::STAGES - 1; ++s)
            if (s < KT) issue_stage(s);
    }
    // Number of epilogue stores (of the previous tile) that sit between this tile's first stages and its
    // in-loop loads in the vector-memory queue; 0 when unknown/none, which only makes the waits stricter.
    int stores_in_flight = 0;

    for (int round = 0; have; ++round) {
        v16i acc[C::MT][C::NT];
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0;

        for (int kt = 0; kt < KT; ++kt) {
            // Loads are retired in order.  Behind stage kt sit the stages already requested after it (at most
            // STAGES-2) and, while kt is one of the pre-requested stages, the previous tile's output stores.
            const int later = min(KT - 1, kt + C::STAGES - 2) - kt;
            if (later == C::STAGES - 2) {
                if (kt < C::STAGES - 1 && stores_in_flight == C::EPI_STORES)
                    wait_vmcnt<C::LPW * (C::STAGES - 2) + C::EPI_STORES>();
                else
                    wait_vmcnt<C::LPW * (C::STAGES - 2)>();
            } else if (C::STAGES > 3 && later == C::STAGES - 3) {
                wait_vmcnt<C::LPW * (C::STAGES > 3 ? C::STAGES - 3 : 0)>();
            } else if (C::STAGES > 4 && later == C::STAGES - 4) {
                wait_vmcnt<C::LPW * (C::STAGES > 4 ? C::STAGES - 4 : 0)>();
            } else {
                wait_vmcnt<0>();
            }
            block_barrier();  // stage kt has landed for every wave; stage kt-1 is no longer being read
            if (kt + C::STAGES - 1 < KT) issue_stage(kt + C::STAGES - 1);

            const unsigned char *xs = smem + (kt % C::STAGES) * C::STAGE_BYTES + wm0 * C::BK;
            const unsigned char *ws = smem + (kt % C::STAGES) * C::STAGE_BYTES + (C::BM + wn0) * C::BK;
#pragma unroll
            for (int kk = 0; kk < C::KK; ++kk) {
                v4i xf[C::MT], wf[C::NT];
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt)
                    xf[mt] = *reinterpret_cast<const v4i *>(xs + mt * 32 * C::BK + frag_off[kk]);
#pragma unroll
                for (int nt = 0; nt < C::NT; ++nt)
                    wf[nt] = *reinterpret_cast<const v4i *>(ws + nt * 32 * C::BK + frag_off[kk]);
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < C::NT; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[nt], xf[mt], acc[mt][nt], 0, 0, 0);
            }
        }

        const int m_base = tm * C::BM + wm0, n_base = tn * C::BN + wn0;
        const bool interior = (tm + 1) * C::BM <= p.M && (tn + 1) * C::BN <= p.N;

        // Row scales r_i = state_row[i] * (state_tensor / 127^2), one per lane per 32-row block.
        float rscale[C::MT];
        if (OUT != OUT_I32) {
            const float c = p.state_tensor[0] / 16129.0f;
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt)
                rscale[mt] = p.state_row[min(m_base + mt * 32 + frow, p.M - 1)] * c;
            // Pin the scales (and the wait for their loads) in front of the requests issued below, so that the
            // epilogue does not have to wait for the next tile's stages.
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt) asm volatile("" : "+v"(rscale[mt]));
        }

        // Every wave is done reading the stages: request the next tile's first stages, then run the epilogue
        // while they are in flight.
        block_barrier();
        int ntm, ntn;
        have = tile_of(blockIdx.x, round + 1, gridDim.x, p.tiles_m, p.tiles_n, &ntm, &ntn);
        if (have) {
            set_tile_sources(ntm, ntn);
#pragma unroll
            for (int s = 0; s < C::STAGES - 1; ++s)
                if (s < KT) issue_stage(s);
        }
        // The wait counts of the next main loop assume these requests precede the output stores below.
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");

        if (OUT == OUT_BF16) {
            unsigned short *out = static_cast<unsigned short *>(p.out);
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt) {
#pragma unroll
                for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        v4f v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = (float)acc[mt][nt][4 * g + e] * rscale[mt];
                        *reinterpret_cast<v4bf *>(epi + frow * C::EPI_STRIDE +
                                                  (nt * 32 + 8 * g + 4 * (lane >> 5)) * 2) =
                            __builtin_convertvector(v, v4bf);
                    }
                constexpr int PIECES = C::WTN * 2 / 16;  // 16-byte pieces per patch row
#pragma unroll
                for (int j = 0; j < 32 * PIECES / 64; ++j) {
                    const int idx = j * 64 + lane;
                    const int prow = idx / PIECES, piece = idx % PIECES;
                    const v4u val = *reinterpret_cast<const v4u *>(epi + prow * C::EPI_STRIDE + piece * 16);
                    const int gr = m_base + mt * 32 + prow, gc = n_base + piece * 8;
                    if (interior || (gr < p.M && gc < p.N))
                        *reinterpret_cast<v4u *>(out + (int64_t)gr * p.N + gc) = val;
                }
            }
        } else {
            // Verification paths: binary32 results or raw accumulators, stored straight from the registers.
            const int gr0 = m_base + frow;
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int gr = gr0 + mt * 32, gc = n_base + nt * 32 + 8 * g + 4 * (lane >> 5);
                        if (gr < p.M && gc < p.N) {
                            if (OUT == OUT_F32) {
                                v4f v;
#pragma unroll
                                for (int e = 0; e < 4; ++e) v[e] = (float)acc[mt][nt][4 * g + e] * rscale[mt];
                                *reinterpret_cast<v4f *>(static_cast<float *>(p.out) + (int64_t)gr * p.N + gc) = v;
                            } else {
                                v4i v;
#pragma unroll
                                for (int e = 0; e < 4; ++e) v[e] = acc[mt][nt][4 * g + e];
                                *reinterpret_cast<v4i *>(static_cast<int *>(p.out) + (int64_t)gr * p.N + gc) = v;
                            }
                        }
                    }
        }
        stores_in_flight = (OUT == OUT_BF16 && interior) ? C::EPI_STORES : 0;
        tm = ntm;
        tn = ntn;
    }
}

template <class C, int OUT>
hipError_t launch_cfg(const GemmI8Args &args, int num_cu, hipStream_t stream) {
    static bool attr_set = false;
    auto kernel = gemm_i8_dequant_kernel<C, OUT>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    GemmI8Args a = args;
    a.tiles_m = (args.M + C::BM - 1) / C::BM;
    a.tiles_n = (args.N + C::BN - 1) / C::BN;
    int grid = num_cu - num_cu % 8;  // a multiple of the XCD count
    if (grid < 8) grid = 8;
    kernel<<<grid, C::THREADS, C::LDS_BYTES, stream>>>(a);
    return hipGetLastError();
}

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
    GemmI8Args args{aq, bq, state_row, state_tensor, out, (int)M, (int)N, (int)K, 0, 0};
    typedef GemmI8Cfg<256, 256, 64, 2, 4, 3> Big;
    const int ncu = cached_num_cu();
    switch (out_dtype) {
        case SB_BF16: return launch_cfg<Big, OUT_BF16>(args, ncu, stream);
        case SB_F32: return launch_cfg<Big, OUT_F32>(args, ncu, stream);
        default: return launch_cfg<Big, OUT_I32>(args, ncu, stream);
    }
}

}  // namespace sb
