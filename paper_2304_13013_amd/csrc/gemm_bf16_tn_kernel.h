// Weight-gradient GEMM of the SwitchBack layer (Algorithm 1 of arxiv 2304.13013: the product the layer keeps in
// 16 bit): dW[j,k] = sum_i dY[i,j] * X[i,k], bf16 operands, binary32 accumulation, hand-written for gfx950.
//
// Both operands are stored with the contraction index (the token i) as the SLOW axis: a row of dY holds m
// consecutive outputs of one token, a row of X holds n consecutive inputs.  The tiles therefore go into LDS exactly
// as they lie in memory, [token][column], with buffer_load_dwordx4 ... lds (no VGPR staging; tokens past b read as
// zero through the buffer bounds check), and the transposition the MFMA needs happens in the LDS read:
// ds_read_b64_tr_b16 hands lane i of a 16-lane group element i%4 of the 8-byte rows addressed by lanes i/4, i/4+4,
// i/4+8 and i/4+12, so with lane r addressing token r/4 and columns 4*(r%4).. a lane receives one column at four
// consecutive tokens; two such reads make the 8-token operand of v_mfma_f32_32x32x16_bf16.
//
// Pipeline, tile walk and barriers are those of the int8 kernel (gemm_i8_kernel.h): 256x256 tile, 8 waves with
// 128x64 wave tiles, two LDS stages of 64 tokens, requests issued between MFMAs, bare s_barrier with counted waits.
// The X-side tile is the MFMA's first operand and the dY-side tile its second, so a lane owns one dW row.
//
// The contraction is long (b ~ 32k) and the output small, so work items are (split, tile) pairs (split-K); they are
// dealt to the XCDs in split-major runs so that the workgroups sharing an L2 read the same token range.  With more
// than one split the partial sums go to a binary32 workspace [split][m][n] and a second kernel adds them in split
// order (deterministic) and converts to the output type.
#pragma once
#include "gemm_i8_kernel.h"

namespace sb {

struct GemmBf16Args {
    const unsigned short *dy;  // [b,m]
    const unsigned short *x;   // [b,n]
    float *partial;            // [splits][m][n] when splits > 1
    void *out;                 // [m,n] when splits == 1
    int b, n, m;
    int tiles_m, tiles_n, splits, k_per_split;  // k_per_split is a multiple of the stage length
    int out_bf16;
};

template <int STAGES_ = 2, int SPREAD_ = 2, int PRIO_ = 1>
struct GemmBf16Cfg {
    static constexpr int BM = 256, BN = 256, BKT = 64;  // dW rows (dY columns), dW columns (X columns), tokens/stage
    static constexpr int STAGES = STAGES_, SPREAD = SPREAD_, PRIO = PRIO_;
    static constexpr int WAVES_M = 2, WAVES_N = 4, NWAVES = 8, THREADS = 512;
    static constexpr int WTM = 128, WTN = 64, MT = 4, NT = 2;
    static constexpr int KK = BKT / 16;                       // MFMA k-steps (16 tokens) per stage
    static constexpr int OP_BYTES = BKT * 512;                // one operand tile: BKT token rows of 256 bf16
    static constexpr int STAGE_BYTES = 2 * OP_BYTES;          // dY tile then X tile
    static constexpr int LPW = STAGE_BYTES / 1024 / NWAVES;   // 1 KiB requests (two token rows of one operand) per wave
    static constexpr int SGROUPS = SPREAD ? KK / SPREAD : 1;
    static constexpr int LPG = LPW / SGROUPS, LSTEP = MT * NT / LPG;
    static constexpr int EPI_WAVE_BYTES = 32 * WTN * 2, EPI_PIECES = WTN * 2 / 16;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES + NWAVES * EPI_WAVE_BYTES;
    static_assert(STAGES >= 2 && LDS_BYTES <= 160 * 1024 && LPW % SGROUPS == 0 && LPG <= MT * NT, "configuration");
};

// The kernel body; the __global__ entry that calls it lives next to the launcher (a __global__ template that uses
// device-only buffer builtins does not instantiate in the host pass).
template <class C>
__device__ __forceinline__ void gemm_bf16_tn_body(const GemmBf16Args &p) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    typedef __attribute__((address_space(3))) void lds_void;
    typedef __attribute__((address_space(3))) v4s lds_v4s;
    constexpr int S = C::STAGES;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps the buffer resources in SGPRs
    const int wm0 = (wave / C::WAVES_N) * C::WTM, wn0 = (wave % C::WAVES_N) * C::WTN;
    const int frow = lane & 31, fhalf = lane >> 5;

    // Buffer resources: the bounds check (num_records in bytes) turns token rows past b into zeros.
    const __amdgpu_buffer_rsrc_t rsrc_dy =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.dy, 0, (unsigned)((size_t)p.b * p.m * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_x =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, (unsigned)((size_t)p.b * p.n * 2), 0x00020000);

    // Loader role.  Request i of wave w fills 1 KiB = token rows (2j, 2j+1) of one operand tile, j = (w*LPW+i) % 32;
    // requests with w*LPW+i < 32 load dY, the rest X.  LDS slot (token, p) holds 16-byte column chunk
    // p ^ ((token & 3) << 2): token rows are 512 bytes apart, so without it the four token rows one transposing read
    // touches would all fall into the same 64-byte bank window.
    const int l_tok = lane >> 5, l_pos = lane & 31;
    unsigned voff[C::LPW];          // byte offset of this lane's 16 bytes for stage 0 of the current work item
    unsigned vstep_dy, vstep_x;     // bytes per stage
    vstep_dy = (unsigned)C::BKT * p.m * 2;
    vstep_x = (unsigned)C::BKT * p.n * 2;
    auto set_item_sources = [&](int tm, int tn, int k_begin) {
#pragma unroll
        for (int i = 0; i < C::LPW; ++i) {
            const int req = wave * C::LPW + i;
            const int tok = (req & 31) * 2 + l_tok;
            const int chunk = l_pos ^ ((tok & 3) << 2);
            if (req < 32) {
                const int col = min(tm * C::BM + chunk * 8, p.m - 8);
                voff[i] = ((unsigned)(k_begin + tok) * p.m + col) * 2;
            } else {
                const int col = min(tn * C::BN + chunk * 8, p.n - 8);
                voff[i] = ((unsigned)(k_begin + tok) * p.n + col) * 2;
            }
        }
    };
    auto issue_one = [&](int kt, int i) {
        const int req = wave * C::LPW + i;
        unsigned char *dst = smem + (kt % S) * C::STAGE_BYTES + req * 1024;
        if (req < 32)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_dy, (lds_void *)dst, 16, voff[i] + kt * vstep_dy, 0, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_x, (lds_void *)dst, 16, voff[i] + kt * vstep_x, 0, 0, 0);
    };
    auto issue_stage = [&](int kt) {
#pragma unroll
        for (int i = 0; i < C::LPW; ++i) issue_one(kt, i);
    };

    // Fragment reads.  Lane l: 16-lane group g = l/16 covers columns 16*(g%2).. of the 32-column block and token
    // half g/2 (8 tokens) of the 16-token k-step; within the group lane r addresses token r/4 and columns 4*(r%4)...
    const int f_r = lane & 15, f_g = lane >> 4;
    const int f_tok = (f_g >> 1) * 8 + (f_r >> 2);                  // token within the k-step for the first read
    const int f_col = (f_g & 1) * 16 + (f_r & 3) * 4;               // column within the 32-column block
    // Per-lane byte offsets (inside a stage) of the first read of k-step 0 for each 32-column block; they never change.
    // The k-step, the second read (+4 tokens) and the stage only add constants: tok = kk*16 + half*4 + f_tok keeps
    // tok & 3 == f_tok & 3, so the swizzle term is fixed per lane.
    auto frag_off = [&](int op_base, int col0) -> int {
        const int col = col0 + f_col;  // column within the 256-column operand tile
        const int chunk = (col >> 3) ^ ((f_tok & 3) << 2);
        return op_base + f_tok * 512 + chunk * 16 + (col & 7) * 2;
    };
    int goff[C::MT], xoff[C::NT];
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) goff[mt] = frag_off(0, wm0 + mt * 32);
#pragma unroll
    for (int nt = 0; nt < C::NT; ++nt) xoff[nt] = frag_off(C::OP_BYTES, wn0 + nt * 32);
    // The transposing reads are inline asm (see gemm_i8_kernel.h): the compiler would otherwise order every LDS read
    // behind ALL outstanding buffer->LDS requests (vmcnt(0)) and use lgkmcnt(0) in front of every MFMA group.
    v8bf gf[2][C::MT], xf[2][C::NT];
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    auto read_pair = [&](unsigned addr) -> v8bf {
        v2u lo, hi;
        asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(addr));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:2048" : "=v"(hi) : "v"(addr));
        return __builtin_bit_cast(v8bf, __builtin_shufflevector(lo, hi, 0, 1, 2, 3));
    };
    auto read_frags = [&](int buf, int kt, int kk) {
        const unsigned base = lds_base + (kt % S) * C::STAGE_BYTES + kk * (16 * 512);
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) gf[buf][mt] = read_pair(base + goff[mt]);
#pragma unroll
        for (int nt = 0; nt < C::NT; ++nt) xf[buf][nt] = read_pair(base + xoff[nt]);
    };
    auto frags_ready = [&](int buf, bool newer_outstanding) {
        if (newer_outstanding)
            wait_lgkmcnt<2 * (C::MT + C::NT)>();
        else
            wait_lgkmcnt<0>();
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) asm volatile("" : "+v"(gf[buf][mt]));
#pragma unroll
        for (int nt = 0; nt < C::NT; ++nt) asm volatile("" : "+v"(xf[buf][nt]));
    };

    // Work items: XCD x (workgroup id % 8) owns the contiguous run [x*per_xcd, (x+1)*per_xcd) of split-major items.
    const int tiles = p.tiles_m * p.tiles_n, total = tiles * p.splits;
    const int per_xcd = (total + 7) / 8, xcd = blockIdx.x & 7, slots = gridDim.x >> 3;
    const int run_end = min(total, (xcd + 1) * per_xcd);
    auto item_of = [&](int round, int *tm, int *tn, int *split) -> bool {
        const int item = xcd * per_xcd + (blockIdx.x >> 3) + round * slots;
        if (item >= run_end) return false;
        *split = item / tiles;
        const int tile = item % tiles;
        *tm = tile / p.tiles_n;
        *tn = tile % p.tiles_n;
        return true;
    };
    auto stages_of = [&](int split) -> int {
        const int k_begin = split * p.k_per_split, k_end = min(p.b, k_begin + p.k_per_split);
        return k_end > k_begin ? (k_end - k_begin + C::BKT - 1) / C::BKT : 0;
    };

    int tm, tn, split;
    bool have = item_of(0, &tm, &tn, &split);
    int KT = 0;
    if (have) {
        KT = stages_of(split);
        set_item_sources(tm, tn, split * p.k_per_split);
#pragma unroll
        for (int s = 0; s < S; ++s)
            if (s < KT) issue_stage(s);
    }

    for (int round = 0; have; ++round) {
        v16f acc[C::MT][C::NT];
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.0f;

        // Unlike the int8 kernel the epilogue stores here are few (the output is small), so the waits simply
        // count requests and treat everything older as retired in order.
        int issued_upto = min(S - 1, KT - 1);
        if (KT > 0) {
            wait_stage<C::LPW, 0>(issued_upto);
            block_barrier();
            read_frags(0, 0, 0);
        }
        for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
            for (int kk = 0; kk < C::KK; ++kk) {
                if (kk + 1 < C::KK) {
                    read_frags((kk + 1) & 1, kt, kk + 1);
                } else if (kt + 1 < KT) {
                    wait_stage<C::LPW, 0>(issued_upto - (kt + 1));
                    wait_lds_reads();
                    block_barrier();
                    if (!C::SPREAD && kt + S < KT) issue_stage(kt + S);
                    issued_upto = min(KT - 1, kt + S);
                    read_frags(0, kt + 1, 0);
                }
                frags_ready(kk & 1, kk + 1 < C::KK || kt + 1 < KT);
                if (C::PRIO) __builtin_amdgcn_s_setprio(2);
                const int spread_kt = (kk == C::KK - 1) ? kt + S : kt - 1 + S;
                const int spread_part = (kk == C::KK - 1) ? 0 : kk + 1;
                const bool spread_on = C::SPREAD && spread_part < C::SGROUPS && spread_kt < KT &&
                                       (kk == C::KK - 1 ? kt + 1 < KT : kt >= 1);
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < C::NT; ++nt) {
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[kk & 1][nt], gf[kk & 1][mt],
                                                                              acc[mt][nt], 0, 0, 0);
                        const int idx = mt * C::NT + nt;
                        if (C::SPREAD && idx % C::LSTEP == C::LSTEP - 1 && idx / C::LSTEP < C::LPG && spread_on)
                            issue_one(spread_kt, spread_part * C::LPG + idx / C::LSTEP);
                    }
                if (C::PRIO) __builtin_amdgcn_s_setprio(0);
            }
        }

        const int m_base = tm * C::BM + wm0, n_base = tn * C::BN + wn0;
        const int this_split = split;

        // Every wave is done reading the stages: request the next item's stages, then store this item's results.
        wait_lds_reads();
        block_barrier();
        int ntm = 0, ntn = 0, nsplit = 0;
        have = item_of(round + 1, &ntm, &ntn, &nsplit);
        int nKT = 0;
        if (have) {
            nKT = stages_of(nsplit);
            set_item_sources(ntm, ntn, nsplit * p.k_per_split);
#pragma unroll
            for (int s = 0; s < S; ++s)
                if (s < nKT) issue_stage(s);
        }

        if (p.splits == 1 && p.out_bf16) {
            // Final bf16 result: transpose through the wave-private LDS patch, 16-byte stores in 128-byte row segments.
            unsigned short *out = static_cast<unsigned short *>(p.out);
            unsigned char *epi = smem + S * C::STAGE_BYTES + wave * C::EPI_WAVE_BYTES;
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt) {
#pragma unroll
                for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        v4f v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = acc[mt][nt][4 * g + e];
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
                    if (gr < p.m && gc < p.n) *reinterpret_cast<v4u *>(out + (int64_t)gr * p.n + gc) = val;
                }
            }
        } else {
            // binary32: final result (one split) or this split's partial sums, straight from the registers.
            float *pout = p.splits > 1 ? p.partial + (int64_t)this_split * p.m * p.n : static_cast<float *>(p.out);
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int gr = m_base + mt * 32 + frow, gc = n_base + nt * 32 + 8 * g + 4 * fhalf;
                        if (gr < p.m && gc < p.n) {
                            v4f v;
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] = acc[mt][nt][4 * g + e];
                            *reinterpret_cast<v4f *>(pout + (int64_t)gr * p.n + gc) = v;
                        }
                    }
        }
        // The next item's waits count only its own requests: drain the stores (and its first stages) here.  An item
        // is ~100 stages long, so this costs well under a percent.
        wait_vmcnt<0>();
        tm = ntm;
        tn = ntn;
        split = nsplit;
        KT = nKT;
    }
}

}  // namespace sb
