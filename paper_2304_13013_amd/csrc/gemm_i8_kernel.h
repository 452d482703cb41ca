// int8 x int8 -> int32 GEMM kernel with the dequantizing epilogue of the SwitchBack forward / input-gradient
// products (the dequantized forward equation of Section 2.2.1 of arxiv 2304.13013), hand-written for gfx950.
//
//   out[i,j] = (state_tensor/127^2 * state_row[i]) * sum_k aq[i,k] * bq[j,k]        aq [M,K], bq [N,K], K contiguous
//
// Design
//   * v_mfma_i32_32x32x32_i8.  The weight-side tile (bq rows) is the MFMA's first operand and the token-side
//     tile (aq rows) its second, so a lane ends up owning ONE output row (lane % 32) and, per accumulator quad,
//     four consecutive output columns: one row scale per lane, and packed bf16x4 leaves each quad.
//   * A persistent grid (one workgroup per compute unit) walks the output tiles in an order that keeps the
//     workgroups of one XCD (workgroup id % 8) on a compact patch of tiles, so its L2 sees each operand panel once.
//   * Operand tiles go HBM/L2 -> LDS with global_load_lds_dwordx4 (no VGPR staging), STAGES deep.  One wave
//     instruction fills 1 KiB of LDS linearly, so the bank-conflict-avoiding swizzle is applied on the GLOBAL side:
//     LDS slot (row, p) holds 16-byte k-chunk p ^ f(row) of that row, f(row) = (row / (256/BK)) % (BK/16).
//   * MFMA operand fragments are double-buffered in registers: the ds_reads of k-step j+1 are issued before the
//     MFMAs of k-step j, also across the stage boundary (the stage hand-over barrier sits between the last
//     fragment read of a stage and its last MFMAs).
//   * The next tile's first STAGES-1 stages are requested BEFORE the epilogue of the current tile.  The epilogue
//     transposes the bf16 results through the one LDS stage those requests leave free (wave-private, XOR
//     swizzled) and stores 16 bytes per lane, covering whole 128-byte row segments.
//   * Rows past M (and weight rows past N) are clamped on load and masked on store; an out-of-range row only ever
//     feeds accumulators that are never stored.
#pragma once
#include "sb_common.h"
#include <type_traits>

namespace sb {

enum { OUT_BF16 = 0, OUT_F32 = 1, OUT_I32 = 2 };

template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int STAGES_, int EPI_OWN_ = 0, int NTS_ = 0, int DIAG_ = 0, int SPREAD_ = 0, int PRIO_ = 0, int RELAX_ = 0>
struct GemmI8Cfg {
    static constexpr int RELAX = RELAX_;      // 1: a hand-over refills the stage finished one k-tile earlier, so it need not wait
                                              // for this wave's LDS reads (needs STAGES >= 3 and an own epilogue patch)
    static constexpr int EPI_OWN = EPI_OWN_;  // 1: the epilogue patch has its own LDS region, 0: it borrows the last stage
    static constexpr int SPREAD = SPREAD_;    // >0: in-loop stage requests are issued one at a time between the MFMAs of
                                              // the first KK/SPREAD k-step groups after a stage hand-over
    static constexpr int PRIO = PRIO_;        // 1: raise the wave priority while it issues an MFMA group
    static constexpr int NTS = NTS_;          // 1: non-temporal output stores
    static constexpr int DIAG = DIAG_;  // 0 normal; timing diagnostics (bit mask): 1 no global loads, 2 no MFMA/LDS reads, 4 no epilogue,
                                        // 8 epilogue without its global stores, 16 conservative waits, 32 stores before the next requests
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
    static constexpr int EPI_PIECES = WTN * 2 / 16;               // 16-byte pieces per row of the epilogue patch
    static constexpr int EPI_WAVE_BYTES = 32 * WTN * 2;           // 32 rows of bf16 per wave
    static constexpr int EPI_STORES = MT * (EPI_WAVE_BYTES / 1024);  // 16-byte global stores per lane per tile
    static constexpr int NPRO = (EPI_OWN && !RELAX) ? STAGES : STAGES - 1;  // stages requested ahead of a tile's main loop
    static constexpr int DIST = RELAX ? STAGES - 1 : STAGES;        // hand-over of k-tile kt requests k-tile kt + DIST
    static_assert(!RELAX || (EPI_OWN && STAGES >= 3), "relaxed hand-over");
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES + (EPI_OWN ? NWAVES * EPI_WAVE_BYTES : 0);
    static_assert(BK == 64 || BK == 128, "BK");
    static_assert(STAGES >= 2 && STAGES <= 5, "STAGES");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && NSLAB % NWAVES == 0 && KK % 2 == 0, "tile shape");
    static_assert(EPI_WAVE_BYTES % 1024 == 0 && EPI_PIECES >= 8, "epilogue patch must be whole wave reads");
    static_assert(NWAVES * EPI_WAVE_BYTES <= STAGE_BYTES && NPRO >= 1 && (EPI_OWN || STAGES >= 3), "epilogue patch");
    static_assert(LPW * (NPRO - 1) + EPI_STORES < 64 && NPRO <= 4, "vmcnt range");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    static constexpr int SGROUPS = SPREAD ? KK / SPREAD : 1;        // k-step groups a stage's requests are spread over
    static constexpr int LPG = LPW / SGROUPS;                     // requests per such group
    static constexpr int LSTEP = MT * NT / LPG;                   // one request every LSTEP MFMAs
    static_assert(!SPREAD || (EPI_OWN && KK % SPREAD == 0 && LPW % SGROUPS == 0 && LPG <= MT * NT), "spread mode");
};

struct GemmI8Args {
    const int8_t *a;
    const int8_t *b;
    const float *state_row;
    const float *state_tensor;
    void *out;
    int M, N, K;
    int tiles_m, tiles_n;
    int group_m;  // tile rows per group of the tile walk
    int stagger_ticks;  // start delay per XCD index in 100 MHz ticks (0 = none)
    unsigned *dbg;      // DIAG 1024: timeline stamps
    int dbg_point;      // which code point is stamped
};

// Output tile visited by workgroup `wg` in its `round`-th iteration.  Workgroups are dealt to XCDs round-robin,
// so the nwg/8 workgroups with equal wg % 8 share an L2; they get consecutive ids in an order that walks groups
// of group_m tile-rows column by column.
__device__ __forceinline__ bool gemm_tile_of(int wg, int round, int nwg, int tiles_m, int tiles_n, int group_m,
                                             int *tm, int *tn) {
    const int per_xcd = nwg >> 3;
    const int id = (round * 8 + (wg & 7)) * per_xcd + (wg >> 3);
    if (id >= tiles_m * tiles_n) return false;
    const int per_group = group_m * tiles_n;
    const int first_m = (id / per_group) * group_m;
    const int group_rows = min(tiles_m - first_m, group_m);
    const int r = id % per_group;
    *tm = first_m + r % group_rows;
    *tn = r / group_rows;
    return true;
}

// Workgroup barrier WITHOUT the memory fence of __syncthreads(): the fence would drain every outstanding
// global->LDS request (vmcnt(0)) and serialize the pipeline.  Explicit vmcnt / lgkmcnt waits order the LDS traffic.
__device__ __forceinline__ void block_barrier() { asm volatile("s_barrier" ::: "memory"); }
__device__ __forceinline__ void wait_lds_reads() { __builtin_amdgcn_s_waitcnt(0xC07F); }  // lgkmcnt(0) only

// LDS fragment reads are written as inline asm so that the waits can be counted: the compiler's own wait insertion
// uses lgkmcnt(0) in front of every MFMA group, which also waits for the reads just issued for the NEXT group and
// exposes the LDS latency once per k-step.  LDS operations of a wave return in order, so "at most N outstanding"
// means everything but the N newest has landed.  The empty asm ties each fragment register to the wait.
template <int OFF>
__device__ __forceinline__ v4i lds_read_b128(unsigned addr) {
    v4i v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int STRIDE, int N, int I = 0>
__device__ __forceinline__ void lds_read_frags(v4i (&f)[N], unsigned addr) {
    if constexpr (I < N) {
        f[I] = lds_read_b128<I * STRIDE>(addr);
        lds_read_frags<STRIDE, N, I + 1>(f, addr);
    }
}
template <int N>
__device__ __forceinline__ void wait_lgkmcnt() {
    static_assert(N >= 0 && N < 16, "lgkmcnt is a 4-bit counter");
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void pin_frags(v4i (&f)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(f[i]));
}

// Wait until at most `later` stages (LPW loads each) plus EXTRA other vector-memory operations remain outstanding.
// Counts that do not fit the 6-bit counter are clamped, which only makes the wait stricter.
template <int LPW, int EXTRA>
__device__ __forceinline__ void wait_stage(int later) {
    constexpr int c0 = EXTRA < 63 ? EXTRA : 63, c1 = LPW + EXTRA < 63 ? LPW + EXTRA : 63;
    constexpr int c2 = 2 * LPW + EXTRA < 63 ? 2 * LPW + EXTRA : 63, c3 = 3 * LPW + EXTRA < 63 ? 3 * LPW + EXTRA : 63;
    switch (later) {
        case 0: wait_vmcnt<c0>(); break;
        case 1: wait_vmcnt<c1>(); break;
        case 2: wait_vmcnt<c2>(); break;
        default: wait_vmcnt<c3>(); break;
    }
}

template <class C, int OUT>
__global__ __launch_bounds__(C::THREADS) void gemm_i8_dequant_kernel(GemmI8Args p) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    typedef __attribute__((address_space(3))) void lds_void;
    typedef const __attribute__((address_space(1))) void gbl_void;
    constexpr int S = C::STAGES;
    constexpr int NSCALE = OUT != OUT_I32 ? C::MT : 0;  // per-lane row-scale loads per tile

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, so everything derived from it is scalar
    const int wm0 = (wave / C::WAVES_N) * C::WTM, wn0 = (wave % C::WAVES_N) * C::WTN;
    const int KT = p.K / C::BK;

    // Per-lane byte offset of its MFMA operand chunk inside a 32-row block of a stage, one per k-step.
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fswz = (frow / C::SWZ_DIV) % C::CPR;
    int frag_off[C::KK];
#pragma unroll
    for (int kk = 0; kk < C::KK; ++kk) frag_off[kk] = frow * C::BK + (((kk * 2 + fhalf) ^ fswz) << 4);

    // Loader role of this lane: slab s = wave*LPW + i covers stage rows [s*RPS, (s+1)*RPS).
    const int lrow_in_slab = lane / C::CPR, lpos = lane % C::CPR;

    const int8_t *gsrc[C::LPW];
    auto set_tile_sources = [&](int tm, int tn) {
        if (C::DIAG & 256) { tm &= 1; tn &= 1; }  // timing diagnostic: every operand panel stays L2 resident
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
        unsigned char *dst = smem + (kt % S) * C::STAGE_BYTES + wave * C::LPW * 1024;
        if (C::DIAG & 1) return;
#pragma unroll
        for (int i = 0; i < C::LPW; ++i)
            __builtin_amdgcn_global_load_lds((gbl_void *)(gsrc[i] + (int64_t)kt * C::BK), (lds_void *)(dst + i * 1024),
                                             16, 0, 0);
    };
    // One request of stage kt (spread mode): request i of this wave.
    auto issue_one = [&](int kt, int i) {
        if (C::DIAG & 1) return;
        unsigned char *dst = smem + (kt % S) * C::STAGE_BYTES + wave * C::LPW * 1024;
        __builtin_amdgcn_global_load_lds((gbl_void *)(gsrc[i] + (int64_t)kt * C::BK), (lds_void *)(dst + i * 1024), 16,
                                         0, 0);
    };
    auto issue_prologue = [&]() {
#pragma unroll
        for (int s = 0; s < C::NPRO; ++s)
            if (s < KT) issue_stage(s);
    };

    // MFMA operand fragments, double-buffered in registers.  A k-step group issues its MFMAs in the order
    // (x0,w0) (x0,w1) (x1,w0) (x1,w1) ... and reads the NEXT group's fragments in the order w0 x0 w1 x1 x2 x3, one
    // read after each of its first six MFMAs: an LDS read issued in the shadow of an MFMA costs no issue time,
    // whereas six reads in a row from all eight waves at once stall every wave until the LDS has accepted them.
    static_assert(C::MT == 4 && C::NT == 2, "fragment schedule below is written for 4x2 MFMA blocks per wave");
    constexpr int NFRAG = C::MT + C::NT;
    v4i xf[2][C::MT], wf[2][C::NT];
    if (C::DIAG & 64) {  // timing diagnostic: MFMA on constant fragments (no LDS reads)
        for (int i = 0; i < 2; ++i) {
            for (int mt = 0; mt < C::MT; ++mt) xf[i][mt] = v4i{lane, 1, 2, 3};
            for (int nt = 0; nt < C::NT; ++nt) wf[i][nt] = v4i{3, lane, 1, 0};
        }
    }
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    static_assert((C::BM + C::BN) * C::BK <= 65536, "fragment offsets must fit the 16-bit ds offset field");
    const unsigned x_off = wm0 * C::BK, w_off = (C::BM + wn0) * C::BK;
    // i-th fragment read of the group (k-tile kt, k-step kk) into register buffer buf.
    auto issue_frag_read = [&](int i, int buf, int kt, int kk) {
        if (C::DIAG & 64) return;
        const unsigned at = lds_base + (kt % S) * C::STAGE_BYTES + frag_off[kk];
        switch (i) {
            case 0: wf[buf][0] = lds_read_b128<0>(at + w_off); break;
            case 1: xf[buf][0] = lds_read_b128<0>(at + x_off); break;
            case 2: wf[buf][1] = lds_read_b128<32 * C::BK>(at + w_off); break;
            case 3: xf[buf][1] = lds_read_b128<32 * C::BK>(at + x_off); break;
            case 4: xf[buf][2] = lds_read_b128<64 * C::BK>(at + x_off); break;
            default: xf[buf][3] = lds_read_b128<96 * C::BK>(at + x_off); break;
        }
    };
    // Ties the register of the i-th fragment read to the wait that precedes this call.
    auto pin_frag = [&](int i, int buf) {
        switch (i) {
            case 0: asm volatile("" : "+v"(wf[buf][0])); break;
            case 1: asm volatile("" : "+v"(xf[buf][0])); break;
            case 2: asm volatile("" : "+v"(wf[buf][1])); break;
            case 3: asm volatile("" : "+v"(xf[buf][1])); break;
            case 4: asm volatile("" : "+v"(xf[buf][2])); break;
            default: asm volatile("" : "+v"(xf[buf][3])); break;
        }
    };
    auto wait_lgkm_at_most = [&](int n) {
        if (C::DIAG & 64) return;
        switch (n) {
            case 0: wait_lgkmcnt<0>(); break;
            case 1: wait_lgkmcnt<1>(); break;
            case 2: wait_lgkmcnt<2>(); break;
            case 3: wait_lgkmcnt<3>(); break;
            case 4: wait_lgkmcnt<4>(); break;
            case 5: wait_lgkmcnt<5>(); break;
            default: wait_lgkmcnt<6>(); break;
        }
    };

    // Phase-shift the XCDs against each other: every tile costs the same, so without this all 256 workgroups
    // reach their epilogue together and the output stores (an HBM-bound burst) never overlap the main loops.
    if (p.stagger_ticks > 0) {
        const uint64_t until = wall_clock64() + (uint64_t)((blockIdx.x & 7) * p.stagger_ticks);
        while (wall_clock64() < until) __builtin_amdgcn_s_sleep(8);
    }

    // c = state_tensor / 127^2, read once (the pointer may alias nothing the kernel writes).
    float tensor_scale = 0.0f;
    if (OUT != OUT_I32) tensor_scale = p.state_tensor[0] / 16129.0f;
    asm volatile("" : "+v"(tensor_scale));

    int tm, tn;
    bool have = gemm_tile_of(blockIdx.x, 0, gridDim.x, p.tiles_m, p.tiles_n, p.group_m, &tm, &tn);
    if (have) {
        set_tile_sources(tm, tn);
        issue_prologue();
    }
    // Whether the previous tile's EPI_STORES output stores sit right behind this tile's pre-requested stages in
    // the vector-memory queue (false when unknown, which only makes the waits stricter).
    bool stores_behind_prologue = false;

    unsigned dbg_epi_end = 0, dbg_prologue_issued = 0;
    for (int round = 0; have; ++round) {
        auto stamp = [&](int idx) {
            if ((C::DIAG & 1024) && round < 2) {
                const unsigned t = (unsigned)__builtin_readcyclecounter();
                if (lane == 0) *reinterpret_cast<unsigned *>(smem + S * C::STAGE_BYTES + wave * C::EPI_WAVE_BYTES + idx * 4) = t;
            }
        };
        v16i acc[C::MT][C::NT];
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0;

        // Stage 0 of this tile: behind it sit the other pre-requested stages (and the previous tile's stores).
        int issued_upto = min(C::NPRO - 1, KT - 1);
        if (stores_behind_prologue)
            wait_stage<C::LPW, C::EPI_STORES>(issued_upto);
        else
            wait_stage<C::LPW, 0>(issued_upto);
        block_barrier();
        stamp(200);
        if ((C::DIAG & 1024) && round < 2 && lane == 0)
            *reinterpret_cast<unsigned *>(smem + S * C::STAGE_BYTES + wave * C::EPI_WAVE_BYTES + 202 * 4) = (unsigned)wall_clock64();
        // Row absmax values of this tile, fetched now so that the epilogue finds them in registers.  They queue
        // behind the pre-requested stages (and the previous tile's stores) and ahead of every in-loop request.
        float srow[C::MT];
        if (OUT != OUT_I32) {
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt)
                srow[mt] = p.state_row[min(tm * C::BM + wm0 + mt * 32 + frow, p.M - 1)];
        }
#pragma unroll
        for (int i = 0; i < NFRAG; ++i) issue_frag_read(i, 0, 0, 0);

        // One k-tile (stage).  The tile's last k-tile is a separate instantiation, so that "another k-step group
        // follows" is known at compile time and the hot loop carries no branches for it.
        auto k_tile = [&](const int kt, auto is_last_tile) {
            constexpr bool last_tile = decltype(is_last_tile)::value;
#pragma unroll
            for (int kk = 0; kk < C::KK; ++kk) {
                const bool last_group = kk + 1 == C::KK;
                const bool has_next = !last_group || !last_tile;   // another k-step group follows in this tile
                const bool handed_over = last_group && has_next;
                if (handed_over) {
                    // Hand-over: the fragments of this last k-step of stage kt are in (or on their way to)
                    // registers.  Retire this wave's LDS reads, make sure stage kt+1 has landed, then let the
                    // freed stage be refilled.
                    if (p.dbg_point == 12) stamp(kt * 4 + 0);
                    if (kt + 1 >= C::NPRO)
                        wait_stage<C::LPW, 0>(issued_upto - (kt + 1));
                    else if (stores_behind_prologue)
                        wait_stage<C::LPW, C::EPI_STORES + NSCALE>(issued_upto - (kt + 1));
                    else
                        wait_stage<C::LPW, NSCALE>(issued_upto - (kt + 1));
                    if (p.dbg_point == 13) stamp(kt * 4 + 0);
                    if (!C::RELAX) wait_lds_reads();
                    if (p.dbg_point == 14) stamp(kt * 4 + 0);
                    block_barrier();
                    stamp(kt * 4 + 3);
                    if (!C::EPI_OWN && kt == 0 && S - 1 < KT) issue_stage(S - 1);  // the stage the last epilogue borrowed
                    if (!C::SPREAD && kt + C::DIST < KT) issue_stage(kt + C::DIST);
                    issued_upto = min(KT - 1, kt + C::DIST);
                }
                // Spread mode: the stage freed by the last hand-over (k-tile kt-1+S, or kt+S once this k-tile's own
                // hand-over has happened) is requested piecemeal between the MFMAs, so that the vector-memory
                // queue never sees a burst from all waves at once.
                const int spread_kt = last_group ? kt + C::DIST : kt - 1 + C::DIST;
                const int spread_part = last_group ? 0 : kk + 1;
                const bool spread_on = C::SPREAD && spread_part < C::SGROUPS && spread_kt < KT &&
                                       (last_group ? !last_tile : kt >= 1);
                const int cur = kk & 1, nxt = (kk + 1) & 1;
                const int next_kt = last_group ? kt + 1 : kt, next_kk = last_group ? 0 : kk + 1;
                if (p.dbg_point == kk * 3 + 0) stamp(kt * 4 + 0);
                if (C::PRIO) __builtin_amdgcn_s_setprio(2);
                int landed = 0;  // fragments of this group known to have landed
#pragma unroll
                for (int idx = 0; idx < C::MT * C::NT; ++idx) {
                    const int mt = idx / C::NT, nt = idx % C::NT;
                    // Reads of this group that MFMA idx needs: w0 x0 | w1 | x1 | - | x2 | - | x3 | -
                    const int need = idx == 0 ? 2 : idx == 1 ? 3 : idx < 4 ? 4 : idx < 6 ? 5 : 6;
                    if (need > landed) {
                        // LDS reads return in order: all but the (NFRAG - need) youngest of this group's reads, and
                        // the reads already issued for the next group, must be back.
                        if (!has_next)
                            wait_lgkm_at_most(NFRAG - need);
                        else if (!handed_over || C::RELAX)
                            wait_lgkm_at_most(NFRAG - need + min(idx, NFRAG));
                        // (a hand-over that waits for all LDS reads leaves nothing to wait for)
#pragma unroll
                        for (int i = landed; i < need; ++i) pin_frag(i, cur);
                        landed = need;
                    }
                    if (idx == 1 && p.dbg_point == kk * 3 + 1) stamp(kt * 4 + 0);
                    acc[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[cur][nt], xf[cur][mt], acc[mt][nt], 0, 0, 0);
                    if (idx < NFRAG && has_next) issue_frag_read(idx, nxt, next_kt, next_kk);
                    if (C::SPREAD && idx % C::LSTEP == C::LSTEP - 1 && idx / C::LSTEP < C::LPG && spread_on)
                        issue_one(spread_kt, spread_part * C::LPG + idx / C::LSTEP);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (C::PRIO) __builtin_amdgcn_s_setprio(0);
                if (p.dbg_point == kk * 3 + 2) stamp(kt * 4 + 0);
            }
        };
        for (int kt = 0; kt + 1 < KT; ++kt) k_tile(kt, std::false_type());
        k_tile(KT - 1, std::true_type());

        stamp(201);
        if ((C::DIAG & 1024) && round < 2 && lane == 0)
            *reinterpret_cast<unsigned *>(smem + S * C::STAGE_BYTES + wave * C::EPI_WAVE_BYTES + 203 * 4) = (unsigned)wall_clock64();
        if ((C::DIAG & 1024) && round < 2 && p.dbg && lane < 52 && (blockIdx.x == 0 || blockIdx.x == 37)) {
            const unsigned *src = reinterpret_cast<const unsigned *>(smem + S * C::STAGE_BYTES + wave * C::EPI_WAVE_BYTES);
            unsigned *dst = p.dbg + (((blockIdx.x ? 1 : 0) * 8 + wave) * 2 + round) * 208;
            for (int i = lane; i < 208; i += 52) dst[i] = i == 204 ? dbg_epi_end : i == 205 ? dbg_prologue_issued : src[i];
        }
        const int m_base = tm * C::BM + wm0, n_base = tn * C::BN + wn0;
        const bool interior = (tm + 1) * C::BM <= p.M && (tn + 1) * C::BN <= p.N;

        // Row scales r_i = state_row[i] * (state_tensor / 127^2), one per lane per 32-row block.
        float rscale[C::MT];
        if (OUT != OUT_I32) {
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt) rscale[mt] = srow[mt] * tensor_scale;
            // Pin the scales (and the wait for their loads) in front of the requests issued below, so that the
            // epilogue does not have to wait for the next tile's stages.
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt) asm volatile("" : "+v"(rscale[mt]));
        }

        // Every wave is done reading the stages: request the next tile's first stages, then run the epilogue
        // while they are in flight.
        wait_lds_reads();
        block_barrier();
        int ntm, ntn;
        have = gemm_tile_of(blockIdx.x, round + 1, gridDim.x, p.tiles_m, p.tiles_n, p.group_m, &ntm, &ntn);
        if (have && !(C::DIAG & 32)) {
            set_tile_sources(ntm, ntn);
            issue_prologue();
        }
        if (C::DIAG & 1024) dbg_prologue_issued = (unsigned)__builtin_readcyclecounter();
        // The wait counts of the next main loop assume these requests precede the output stores below.
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");

        if (C::DIAG & 4) {
        } else if (OUT == OUT_BF16) {
            unsigned short *out = static_cast<unsigned short *>(p.out);
            unsigned char *epi = smem + (C::EPI_OWN ? S : S - 1) * C::STAGE_BYTES + wave * C::EPI_WAVE_BYTES;
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt) {
#pragma unroll
                for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        v4f v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = (float)acc[mt][nt][4 * g + e] * rscale[mt];
                        const int piece = (nt * 4 + g) ^ (frow & 7);
                        *reinterpret_cast<v4bf *>(epi + frow * (C::WTN * 2) + piece * 16 + fhalf * 8) =
                            __builtin_convertvector(v, v4bf);
                    }
#pragma unroll
                for (int j = 0; j < C::EPI_WAVE_BYTES / 1024; ++j) {
                    const int idx = j * 64 + lane;
                    const int prow = idx / C::EPI_PIECES, piece = idx % C::EPI_PIECES;
                    const v4u val = *reinterpret_cast<const v4u *>(epi + prow * (C::WTN * 2) +
                                                                   ((piece ^ (prow & 7)) << 4));
                    const int gr = m_base + mt * 32 + prow, gc = n_base + piece * 8;
                    if (C::DIAG & 8) {
                        if (val.x == 0x12345678u && val.y == 0x9abcdef0u) out[0] = 1;  // keep the reads alive
                    } else if (interior || (gr < p.M && gc < p.N)) {
                        if (C::NTS)
                            __builtin_nontemporal_store(val, reinterpret_cast<v4u *>(out + (int64_t)gr * p.N + gc));
                        else
                            *reinterpret_cast<v4u *>(out + (int64_t)gr * p.N + gc) = val;
                    }
                }
            }
        } else {
            // Verification paths: binary32 results or raw accumulators, stored straight from the registers.
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int gr = m_base + mt * 32 + frow, gc = n_base + nt * 32 + 8 * g + 4 * fhalf;
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
        if (have && (C::DIAG & 32)) {
            set_tile_sources(ntm, ntn);
            issue_prologue();
        }
        if (C::DIAG & 1024) dbg_epi_end = (unsigned)__builtin_readcyclecounter();
        stores_behind_prologue = (OUT == OUT_BF16) && interior && !(C::DIAG & (8 | 16 | 32));
        tm = ntm;
        tn = ntn;
    }
}

template <class C, int OUT>
hipError_t launch_gemm_i8_cfg(GemmI8Args a, int num_cu, hipStream_t stream) {
    static bool attr_set = false;
    auto kernel = gemm_i8_dequant_kernel<C, OUT>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    a.tiles_m = (a.M + C::BM - 1) / C::BM;
    a.tiles_n = (a.N + C::BN - 1) / C::BN;
    if (a.group_m <= 0) a.group_m = 8;
    int grid = num_cu - num_cu % 8;  // a multiple of the XCD count
    if (grid < 8) grid = 8;
    kernel<<<grid, C::THREADS, C::LDS_BYTES, stream>>>(a);
    return hipGetLastError();
}

}  // namespace sb
