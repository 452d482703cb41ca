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
// Pipeline, wave roles and barriers are those of the int8 kernel (gemm_i8_kernel.h): 256x256 tile, 8 waves with
// 128x64 wave tiles, two LDS stages of 64 tokens, four loader waves, fragment reads issued between the MFMAs of
// the preceding k-step, bare s_barrier with counted waits.  A second instance has 128x128 tiles and four waves with
// 64x64 wave tiles, two workgroups per compute unit.
// The X-side tile is the MFMA's first operand and the dY-side tile its second, so a lane owns one dW row.
//
// The contraction is long (b ~ 32k) and the output small, so work items are (split, tile) pairs (split-K); they are
// dealt to the XCDs in split-major runs of neighbouring tiles so that the workgroups sharing an L2 read the same token
// range and few distinct operand panels.  With more
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

// TILE_ x TILE_ output tile per workgroup of WAVES_M_ x WAVES_N_ waves (wave tile TILE_/WAVES_M_ rows by 64 columns).
// The default is the 256 x 256 tile of eight waves, one workgroup per compute unit.  The 128 x 128 tile of four waves
// takes 80 KiB of LDS, so two workgroups share a compute unit; it moves twice the operand bytes per multiply-add and
// serves weight gradients with too few large tiles to fill the GPU without many splits.
template <int STAGES_ = 2, int LOADERS_ = 4, int MT_LOADER_ = 4, int BKT_ = 64, int TILE_ = 256, int WAVES_M_ = 2,
          int WAVES_N_ = 4>
struct GemmBf16Cfg {
    static constexpr int BM = TILE_, BN = TILE_, BKT = BKT_;  // dW rows (dY columns), dW columns (X columns), tokens/stage
    static constexpr int PITCH = TILE_ * 2;                   // bytes of one token row of an operand tile in LDS
    static constexpr int CHUNKS = PITCH / 16;                 // 16-byte column chunks per token row
    static constexpr int ROWS_PER_REQ = 1024 / PITCH;         // token rows one 1 KiB request fills
    static constexpr int NVOFF = 4 / ROWS_PER_REQ;            // distinct (token % 4) swizzles among a wave's requests
    static constexpr int REQ_OP = BKT / ROWS_PER_REQ;         // 1 KiB requests per operand tile
    static constexpr int STAGES = STAGES_, LOADERS = LOADERS_;
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, NWAVES = WAVES_M * WAVES_N, THREADS = NWAVES * 64;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N, NT = WTN / 32;
    static constexpr int MT_EVEN = WTM / 32;                  // 32-row MFMA blocks per wave tile when all waves get the same
    static constexpr int MT_LOADER = MT_LOADER_;  // 32-row MFMA blocks of a loader wave's tile; when < MT_EVEN its SIMD partner
                                                  // (wave + 4) takes the other 2 * MT_EVEN - MT_LOADER blocks of the wave column
    static constexpr int KK = BKT / 16;                       // MFMA k-steps (16 tokens) per stage
    static constexpr int OP_BYTES = BKT * PITCH;              // one operand tile: BKT token rows
    static constexpr int STAGE_BYTES = 2 * OP_BYTES;          // dY tile then X tile
    static constexpr int LPW = STAGE_BYTES / 1024 / LOADERS;  // 1 KiB requests (of one operand) per loader wave
    static constexpr int EPI_WAVE_BYTES = 32 * WTN * 2, EPI_PIECES = WTN * 2 / 16;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES + NWAVES * EPI_WAVE_BYTES;
    static_assert(STAGES >= 2 && LDS_BYTES <= 160 * 1024 && (LOADERS == 4 || LOADERS == 8) && LOADERS <= NWAVES, "configuration");
    static_assert((TILE_ == 256 || TILE_ == 128) && NT == 2 && MT_EVEN >= 2 && MT_EVEN <= 4, "tile");
    static_assert(MT_LOADER == MT_EVEN || (LOADERS == 4 && NWAVES == 8 && WAVES_M == 2 && MT_LOADER == 3), "uneven split");
    static_assert((BKT == 64 || BKT == 32) && LPW % NVOFF == 0 && REQ_OP % LPW == 0, "stage length");
    static_assert(LPW * (STAGES - 1) < 64, "vmcnt range");
};

// What one wave does: an (MT*32) x 64 part of the workgroup's tile, rows from wm0.  Every role runs the same
// sequence of barriers.
template <class C, int MT>
__device__ __forceinline__ void gemm_bf16_tn_role(const GemmBf16Args &p, const int wave, const int wm0) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    typedef __attribute__((address_space(3))) void lds_void;
    constexpr int S = C::STAGES;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wn0 = (wave % C::WAVES_N) * C::WTN;
    const int frow = lane & 31, fhalf = lane >> 5;

    // Loader role (see the int8 kernel for why only LOADERS waves issue requests, all right after a hand-over).
    // Request i of loader wave w fills 1 KiB = ROWS_PER_REQ consecutive token rows of one operand tile, the
    // ((w*LPW + i) % REQ_OP)-th such group; the first REQ_OP requests of a stage load dY, the rest X, so a wave loads
    // one operand only.  LDS slot (token, p) holds 16-byte column chunk p ^ ((token & 3) << 2): token rows are a
    // multiple of 256 bytes apart, so without it the four token rows one transposing read touches would all fall into
    // the same 64-byte bank window.  A lane's byte offset is
    //   voff[i % NVOFF] (per lane: its token row of the group, its swizzled chunk) + i * req_step + item_soff
    //   + kt * stage_step.
    // Columns past the operand's width (partial tiles) read the next token row or, at the very end, zeros from the
    // bounds check; they only feed results that are never stored.
    const bool loader = wave < C::LOADERS;
    const bool loads_dy = wave * C::LPW < C::REQ_OP;
    const unsigned ld = loads_dy ? p.m : p.n;  // row length of the operand this wave loads
    // The bounds check of the buffer resource (num_records in bytes) turns token rows past b into zeros.
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(loads_dy ? p.dy : p.x), 0, (unsigned)((size_t)p.b * ld * 2), 0x00020000);
    const int l_tok = lane / C::CHUNKS, l_pos = lane % C::CHUNKS;  // token row of the request, 16-byte chunk of it
    const int tok0 = ((wave * C::LPW) % C::REQ_OP) * C::ROWS_PER_REQ;  // first token row of the wave's share within a stage
    unsigned voff[C::NVOFF];
#pragma unroll
    for (int v = 0; v < C::NVOFF; ++v)
        voff[v] = ((unsigned)l_tok * ld + ((l_pos ^ (((C::ROWS_PER_REQ * v + l_tok) & 3) << 2)) << 3)) * 2;
    const unsigned req_step = (unsigned)C::ROWS_PER_REQ * 2 * ld, stage_step = (unsigned)C::BKT * 2 * ld;
    unsigned item_soff = 0;
    auto set_item_sources = [&](int tm, int tn, int k_begin) {
        item_soff = ((unsigned)(k_begin + tok0) * ld + (unsigned)(loads_dy ? tm * C::BM : tn * C::BN)) * 2;
    };
    auto issue_stage = [&](int kt) {
        unsigned char *dst = smem + (kt % S) * C::STAGE_BYTES + wave * C::LPW * 1024;
        const unsigned soff = item_soff + (unsigned)kt * stage_step;
#pragma unroll
        for (int i = 0; i < C::LPW; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)(dst + i * 1024), 16, voff[i % C::NVOFF],
                                                     soff + (unsigned)i * req_step, 0, 0);
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
        const int col = col0 + f_col;  // column within the operand tile
        const int chunk = (col >> 3) ^ ((f_tok & 3) << 2);
        return op_base + f_tok * C::PITCH + chunk * 16 + (col & 7) * 2;
    };
    int goff[MT], xoff[C::NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) goff[mt] = frag_off(0, wm0 + mt * 32);
#pragma unroll
    for (int nt = 0; nt < C::NT; ++nt) xoff[nt] = frag_off(C::OP_BYTES, wn0 + nt * 32);
    // The transposing reads are inline asm (see gemm_i8_kernel.h): the compiler would otherwise order every LDS read
    // behind ALL outstanding buffer->LDS requests (vmcnt(0)) and use lgkmcnt(0) in front of every MFMA group.
    v8bf gf[2][MT], xf[2][C::NT];
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    auto read_pair = [&](unsigned addr) -> v8bf {
        v2u lo, hi;
        asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(addr));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "n"(4 * C::PITCH));
        return __builtin_bit_cast(v8bf, __builtin_shufflevector(lo, hi, 0, 1, 2, 3));
    };
    // Fragment schedule of the int8 kernel: a k-step group issues its MFMAs in the order (g0,x0) (g0,x1) (g1,x0) ...
    // and reads the next group's fragments in the order x0 g0 x1 g1 g2 g3, one fragment (two transposing reads) after
    // each of its first six MFMAs.
    static_assert(C::NT == 2, "fragment schedule below is written for MT x 2 MFMA blocks per wave");
    constexpr int NFRAG = MT + C::NT;
    auto issue_frag_read = [&](int i, int buf, int kt, int kk) {
        const unsigned base = lds_base + (kt % S) * C::STAGE_BYTES + kk * (16 * C::PITCH);
        switch (i) {
            case 0: xf[buf][0] = read_pair(base + xoff[0]); break;
            case 1: gf[buf][0] = read_pair(base + goff[0]); break;
            case 2: xf[buf][1] = read_pair(base + xoff[1]); break;
            case 3: gf[buf][1] = read_pair(base + goff[1]); break;
            case 4: gf[buf][2 % MT] = read_pair(base + goff[2 % MT]); break;
            case 5: gf[buf][3 % MT] = read_pair(base + goff[3 % MT]); break;
            default: gf[buf][4 % MT] = read_pair(base + goff[4 % MT]); break;
        }
    };
    auto pin_frag = [&](int i, int buf) {
        switch (i) {
            case 0: asm volatile("" : "+v"(xf[buf][0])); break;
            case 1: asm volatile("" : "+v"(gf[buf][0])); break;
            case 2: asm volatile("" : "+v"(xf[buf][1])); break;
            case 3: asm volatile("" : "+v"(gf[buf][1])); break;
            case 4: asm volatile("" : "+v"(gf[buf][2 % MT])); break;
            case 5: asm volatile("" : "+v"(gf[buf][3 % MT])); break;
            default: asm volatile("" : "+v"(gf[buf][4 % MT])); break;
        }
    };
    // At most n fragment reads (two LDS reads each) outstanding.
    auto wait_frags_at_most = [&](int n) {
        switch (n) {
            case 0: wait_lgkmcnt<0>(); break;
            case 1: wait_lgkmcnt<2>(); break;
            case 2: wait_lgkmcnt<4>(); break;
            case 3: wait_lgkmcnt<6>(); break;
            case 4: wait_lgkmcnt<8>(); break;
            case 5: wait_lgkmcnt<10>(); break;
            case 6: wait_lgkmcnt<12>(); break;
            default: wait_lgkmcnt<14>(); break;
        }
    };

    // Work items are (split, tile) pairs numbered split-major, the tiles of a split walked along the SHORTER side of
    // the tile grid first, so that 32 consecutive items form a compact patch (about 6 x 5 tiles: 12 operand panels for
    // 32 tiles; walking a 5 x 20 grid along its long side touches 22).  Round r of the persistent grid takes items
    // [r * grid, (r + 1) * grid), and XCD x (workgroup id % 8) the x-th run of grid / 8 consecutive items of it: the
    // workgroups sharing an L2 read one token range and neighbouring tiles, and all XCDs stream the same few token
    // ranges at the same time, so what one fetched from HBM the others find in the last-level cache.
    const int tiles = p.tiles_m * p.tiles_n, total = tiles * p.splits;
    const int xcd = blockIdx.x & 7, slots = gridDim.x >> 3;
    auto item_of = [&](int round, int *tm, int *tn, int *split) -> bool {
        const int item = round * (int)gridDim.x + xcd * slots + (blockIdx.x >> 3);
        if (item >= total) return false;
        *split = item / tiles;
        const int tile = item % tiles;
        if (p.tiles_m < p.tiles_n) {
            *tm = tile % p.tiles_m;
            *tn = tile / p.tiles_m;
        } else {
            *tm = tile / p.tiles_n;
            *tn = tile % p.tiles_n;
        }
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
        if (loader) {
#pragma unroll
            for (int s = 0; s < S; ++s)
                if (s < KT) issue_stage(s);
        }
    }

    for (int round = 0; have; ++round) {
        v16f acc[MT][C::NT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.0f;

        // Unlike the int8 kernel the epilogue stores here are few (the output is small), so the waits simply
        // count requests and treat everything older as retired in order.
        int issued_upto = min(S - 1, KT - 1);
        auto k_tile = [&](const int kt, auto is_last_tile) {
            constexpr bool last_tile = decltype(is_last_tile)::value;
#pragma unroll
            for (int kk = 0; kk < C::KK; ++kk) {
                const bool last_group = kk + 1 == C::KK;
                const bool has_next = !last_group || !last_tile;  // another k-step group follows in this item
                const bool handed_over = last_group && has_next;
                if (handed_over) {
                    // Stage hand-over (see the int8 kernel): this wave's reads of stage kt are retired, stage kt+1
                    // has landed, the freed stage may be refilled.
                    if (loader) wait_stage<C::LPW, 0>(issued_upto - (kt + 1));
                    wait_lds_reads();
                    block_barrier();
                    if (loader && kt + S < KT) issue_stage(kt + S);
                    issued_upto = min(KT - 1, kt + S);
                }
                const int cur = kk & 1, nxt = (kk + 1) & 1;
                const int next_kt = last_group ? kt + 1 : kt, next_kk = last_group ? 0 : kk + 1;
                int landed = 0;
#pragma unroll
                for (int idx = 0; idx < MT * C::NT; ++idx) {
                    const int mt = idx / C::NT, nt = idx % C::NT;
                    const int need = idx == 0 ? 2 : idx == 1 ? 3 : 3 + idx / 2;
                    if (need > landed) {
                        if (!has_next)
                            wait_frags_at_most(NFRAG - need);
                        else if (!handed_over)
                            wait_frags_at_most(NFRAG - need + min(idx, NFRAG));
#pragma unroll
                        for (int i = landed; i < need; ++i) pin_frag(i, cur);
                        landed = need;
                    }
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[cur][nt], gf[cur][mt], acc[mt][nt], 0, 0, 0);
                    if (idx < NFRAG && has_next) issue_frag_read(idx, nxt, next_kt, next_kk);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        if (KT > 0) {
            if (loader) wait_stage<C::LPW, 0>(issued_upto);
            block_barrier();
#pragma unroll
            for (int i = 0; i < NFRAG; ++i) issue_frag_read(i, 0, 0, 0);
            for (int kt = 0; kt + 1 < KT; ++kt) k_tile(kt, std::false_type());
            k_tile(KT - 1, std::true_type());
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
            if (loader) {
#pragma unroll
                for (int s = 0; s < S; ++s)
                    if (s < nKT) issue_stage(s);
            }
        }

        if (p.splits == 1 && p.out_bf16) {
            // Final bf16 result: transpose through the wave-private LDS patch, 16-byte stores in 128-byte row segments.
            unsigned short *out = static_cast<unsigned short *>(p.out);
            unsigned char *epi = smem + S * C::STAGE_BYTES + wave * C::EPI_WAVE_BYTES;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
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
            for (int mt = 0; mt < MT; ++mt)
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

// The kernel body; the __global__ entry that calls it lives next to the launcher (a __global__ template that uses
// device-only buffer builtins does not instantiate in the host pass).
template <class C>
__device__ __forceinline__ void gemm_bf16_tn_body(const GemmBf16Args &p) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform: what derives from it is scalar
    if (C::MT_LOADER == C::MT_EVEN)
        gemm_bf16_tn_role<C, C::MT_EVEN>(p, wave, (wave / C::WAVES_N) * C::WTM);
    else if (wave < C::LOADERS)
        gemm_bf16_tn_role<C, C::MT_LOADER>(p, wave, 0);
    else
        gemm_bf16_tn_role<C, 2 * C::MT_EVEN - C::MT_LOADER>(p, wave, C::MT_LOADER * 32);
}

}  // namespace sb
