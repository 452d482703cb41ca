// int8 x int8 -> int32 GEMM kernel with the dequantizing epilogue of the SwitchBack forward / input-gradient
// products (the dequantized forward equation of Section 2.2.1 of arxiv 2304.13013), hand-written for gfx950.
//
//   out[i,j] = (state_tensor/127^2 * state_row[i]) * sum_k aq[i,k] * bq[j,k]        aq [M,K], bq [N,K], K contiguous
//
// Design
//   * v_mfma_i32_32x32x32_i8.  The weight-side tile (bq rows) is the MFMA's first operand and the token-side
//     tile (aq rows) its second, so a lane ends up owning ONE output row (lane % 32) and, per accumulator quad,
//     four consecutive output columns: one row scale per lane, and packed bf16x4 leaves each quad.
//   * 256x256 output tile per workgroup of eight waves, two per SIMD; a wave tile is 64 columns wide and 128 rows
//     high (96 and 160 with the uneven split below).  A persistent grid (one workgroup per compute unit) walks the
//     tiles in an order that keeps the workgroups of one XCD (workgroup id % 8) on a compact patch of tiles, so its
//     L2 sees each operand panel once.  The tile and the wave grid are parameters of GemmI8Cfg; the other instance in
//     use is 128x128 with four waves, two workgroups per compute unit, for products with few tiles.
//   * Operand tiles go HBM/L2 -> LDS with buffer_load_dwordx4 ... lds (no VGPR staging), STAGES deep.  One wave
//     instruction fills 1 KiB of LDS linearly, so the bank-conflict-avoiding swizzle is applied on the GLOBAL side:
//     LDS slot (row, p) holds 16-byte k-chunk p ^ f(row) of that row, f(row) = (row / (256/BK)) % (BK/16).  Rows past
//     M (or N) lie beyond the buffer's num_records and read as zero; they only feed accumulators that are never
//     stored.
//   * One continuous stage pipeline: the stage ring runs across tile boundaries.  The load cursor stays STAGES
//     stages ahead of the MFMAs, so a new tile's first stages are requested during the last k-tiles of the tile
//     before it, and the epilogue needs no barrier of its own.
//   * Wave roles.  A 1 KiB request occupies the CU's address/data path for ~18 cycles and the wave that issues it
//     stalls meanwhile, MFMAs included; the 64 requests of a 64 KiB stage cost ~1200 cycles however they are dealt.
//     With LOADERS = 4 only waves 0..3 issue them, all right after the stage hand-over barrier: waves w and w+4
//     share a SIMD, so while a loader wave is stuck issuing its partner has the matrix pipe to itself, and the
//     loader runs its MFMAs afterwards.  MT_LOADER = 3 evens out the two chains: the loader computes 3 of the 8
//     32-row blocks of its wave column, its partner 5.  With LOADERS = 8 every wave issues its share at the hand-over.
//   * MFMA operand fragments are double-buffered in registers, and the LDS reads of k-step j+1 are issued one at a
//     time between the MFMAs of k-step j (also across the stage hand-over): an LDS read issued in the shadow of an
//     MFMA costs no issue time.  The reads are inline asm so that the lgkmcnt waits can be counted; the compiler's
//     own would drain the queue in front of every MFMA group.
//   * Barriers are bare s_barrier instructions with explicit vmcnt / lgkmcnt waits; __syncthreads() would drain
//     every outstanding global->LDS request.  The vector-memory counter is one in-order counter for loads and
//     stores, so every wave keeps books of what it issued after each stage's requests and waits for "at most that
//     many outstanding".
//   * The epilogue transposes the bf16 results through a wave-private, XOR-swizzled LDS patch and stores 16 bytes
//     per lane, covering whole 128-byte row segments, with non-temporal buffer stores (the output must not evict
//     the operand panels the other workgroups of the XCD are reading from L2).  It is software-pipelined over the
//     32-row blocks of the wave tile: the patch reads of one block are in flight while the next block is converted.
//   * The same pipeline serves the float8 product (MATH_F8): one v_mfma_f32_32x32x64_f8f6f4 per 64 k-values, an
//     operand fragment being the two 16-byte LDS reads that two int8 k-steps would issue.
//   * The cycle figures quoted above come from s_memtime stamps compiled into a working copy of this kernel.
#pragma once
#include "sb_common.h"
#include <type_traits>

namespace sb {

enum { OUT_BF16 = 0, OUT_F32 = 1, OUT_I32 = 2 };
// Arithmetic of the product.  MATH_I8: int8 codes, v_mfma_i32_32x32x32_i8, scale state_tensor/127^2.  MATH_F8 + 2*fw + fx:
// 8-bit float codes (f = 0: E4M3, 1: E5M2; fw for the weight-side operand b, fx for the token-side operand a),
// v_mfma_f32_32x32x64_f8f6f4 with binary32 accumulators, scale state_tensor (the codes already lie in [-1, 1]).
enum { MATH_I8 = 0, MATH_F8 = 4 };

// BM_ x BN_ output tile per workgroup of WAVES_M_ x WAVES_N_ waves; a wave tile is BM_/WAVES_M_ rows by 64 columns.
// The default is the 256x256 tile of eight waves (two per SIMD, one workgroup per compute unit).  The 128x128 tile of
// four waves needs 80 KiB of LDS and 256 registers per lane, so two workgroups share a compute unit, one wave of each
// per SIMD: they drift apart, and the epilogue of one runs under the matrix instructions of the other.  It moves twice
// the operand bytes per multiply-add, which is why it only serves products with too few 256x256 tiles to fill the GPU.
template <int BK_, int STAGES_, int LOADERS_, int MT_LOADER_ = 4, int STORE_NT_ = 0, int BM_ = 256, int BN_ = 256,
          int WAVES_M_ = 2, int WAVES_N_ = 4>
struct GemmI8Cfg {
    static constexpr int STORE_NT = STORE_NT_;  // 1: non-temporal output stores (the output should not evict operand panels from L2)
    static constexpr int BM = BM_, BN = BN_, BK = BK_, STAGES = STAGES_;
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, NWAVES = WAVES_M * WAVES_N, THREADS = NWAVES * 64;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;  // wave tile: 128 x 64 in the default configuration
    static constexpr int NT = WTN / 32;                           // 32-column MFMA blocks per wave tile
    static constexpr int MT_EVEN = WTM / 32;                      // 32-row MFMA blocks per wave tile when all waves get the same
    static constexpr int MT_LOADER = MT_LOADER_;  // 32-row MFMA blocks of a loader wave's tile; when < MT_EVEN its SIMD partner
                                                  // (wave + 4) takes the other 2 * MT_EVEN - MT_LOADER blocks of the wave column
    static constexpr int KK = BK / 32;                            // MFMA k-steps per stage
    static constexpr int CPR = BK / 16;                           // 16-byte chunks per tile row
    static constexpr int RPS = 1024 / BK;                         // tile rows per 1 KiB request
    static constexpr int SWZ_DIV = 256 / BK;                      // rows that share one 256-byte bank window
    static constexpr int STAGE_BYTES = (BM + BN) * BK;
    static constexpr int LOADERS = LOADERS_;                      // waves 0..LOADERS-1 issue the global->LDS requests
    static constexpr int RPL = (BM + BN) / LOADERS;               // stage rows per loader wave
    static constexpr int LPW = RPL / RPS;                         // requests per loader wave per stage
    static constexpr int NVAR = CPR * SWZ_DIV > RPS ? CPR * SWZ_DIV / RPS : 1;  // distinct swizzles among a wave's requests
    static constexpr int EPI_PIECES = WTN * 2 / 16;               // 16-byte pieces per row of the epilogue patch
    static constexpr int EPI_WAVE_BYTES = 32 * WTN * 2;           // 32 rows of bf16 per wave
    static constexpr int STORES_PER_BLOCK = EPI_WAVE_BYTES / 1024;  // 16-byte global stores per lane per 32-row block
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES + NWAVES * EPI_WAVE_BYTES;
    static constexpr int MT_MAX = MT_LOADER < MT_EVEN ? 2 * MT_EVEN - MT_LOADER : MT_EVEN;  // largest wave tile, in blocks
    static_assert(BK == 64 || BK == 128, "BK");
    static_assert(STAGES >= 2 && STAGES <= 4, "STAGES");
    static_assert(BM % (32 * WAVES_M) == 0 && (NWAVES == 4 || NWAVES == 8), "wave grid");
    static_assert(NT == 2 && MT_LOADER >= 2 && MT_LOADER <= MT_EVEN && MT_EVEN <= 4,
                  "the fragment schedule is written for MT x 2 MFMA blocks per wave");
    static_assert((LOADERS == 4 || LOADERS == 8) && LOADERS <= NWAVES && BM % RPL == 0 && LPW % NVAR == 0, "loader split");
    static_assert(MT_LOADER == MT_EVEN || (LOADERS == 4 && NWAVES == 8 && WAVES_M == 2),
                  "an uneven split pairs a loader wave with the non-loading wave below it in the same wave column");
    static_assert(LPW * (STAGES - 1) + MT_MAX * STORES_PER_BLOCK + MT_MAX < 64, "vmcnt range");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

struct GemmI8Args {
    const int8_t *a;
    const int8_t *b;
    const float *state_row;
    const float *state_tensor;  // [1]; unused by the row-and-column variant
    const float *state_col;     // [N], row-and-column variant only (SwitchBackQ: one weight state per output column)
    void *out;
    int M, N, K;  // M*K and N*K must stay below 2^32 (32-bit buffer offsets)
    int tiles_m, tiles_n;
    int group_m;  // tile rows per group of the tile walk
    const float *bias;   // [N] or nullptr; POST instances only: out = gamma[j] * (y + bias[j]), bias first
    const float *gamma;  // [N] or nullptr
};

// Output tile visited by workgroup `wg` in its `round`-th iteration.  Tiles are numbered along groups of group_m
// tile-rows, column by column inside a group.  Workgroups are dealt to XCDs round-robin, so the nwg/8 workgroups with
// equal wg % 8 share an L2: each XCD owns one contiguous eighth of the numbering and works through it 32 (nwg/8) tiles
// per round, so that it sweeps the columns of its own row groups and finds their token-side panels in its L2 again in
// the next round (measured: 6 % less traffic from beyond L2 than dealing the numbering to the XCDs in chunks, same
// speed; a 4 MB L2 barely holds the twelve panels of one round).
__device__ __forceinline__ bool gemm_tile_of(int wg, int round, int nwg, int tiles_m, int tiles_n, int group_m,
                                             int *tm, int *tn) {
    const int per_xcd = nwg >> 3;
    const int total = tiles_m * tiles_n;
    const int x = wg & 7;
    const int lo = (int)((long long)x * total / 8), hi = (int)((long long)(x + 1) * total / 8);
    const int id = lo + round * per_xcd + (wg >> 3);
    if (id >= hi) return false;
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

// LDS operations of a wave return in order, so "at most N outstanding" means everything but the N newest has
// landed.  An empty asm with the fragment register as in/out operand ties its uses to the wait before it.
template <int OFF>
__device__ __forceinline__ v4i lds_read_b128(unsigned addr) {
    v4i v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int N>
__device__ __forceinline__ void wait_lgkmcnt() {
    static_assert(N >= 0 && N < 16, "lgkmcnt is a 4-bit counter");
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}

// Wait until at most `later` stages (LPW requests each) plus EXTRA other vector-memory operations remain
// outstanding.  Counts that do not fit the 6-bit counter are clamped, which only makes the wait stricter.
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


// What one wave does: an (MT*32) x 64 part of the workgroup's tile, rows from wm0.  Every role runs the same
// sequence of barriers.
// COLSCALE: out[i,j] = (float)acc * fl(state_row[i] * fl(state_col[j] / 127^2)) instead of the tensor-wise scale.
// POST: the dequantized value y continues through the linear layer's bias and the block's layer-scale before it is
// stored: fl(y + bias[j]) if p.bias is given, then fl(gamma[j] * that) if p.gamma is given.  The two vectors are
// fetched at the start of the epilogue (64 more registers there, so these instances use the even wave split).
//
// The float8 product runs the same pipeline with one MFMA per 64 k-values: an operand fragment is then 32 bytes per
// lane, fetched by the two 16-byte LDS reads that two consecutive int8 k-steps would issue.  Which 64 k-values a
// lane's registers hold does not matter as long as both operands use the same assignment, which they do.
template <class C, int OUT, int MT, bool COLSCALE, int MATH = MATH_I8, bool POST = false>
__device__ __forceinline__ void gemm_i8_dequant_role(const GemmI8Args &p, const int wave, const int wm0) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    typedef __attribute__((address_space(3))) void lds_void;
    constexpr int S = C::STAGES;
    constexpr bool F8 = MATH >= MATH_F8;
    constexpr int FMT_X = MATH & 1, FMT_W = (MATH >> 1) & 1;
    constexpr int RPF = F8 ? 2 : 1;            // 16-byte LDS reads per operand fragment
    constexpr int KKG = C::KK / RPF;           // MFMA k-step groups per stage
    typedef typename std::conditional<F8, v16f, v16i>::type AccT;
    typedef typename std::conditional<F8, v8i, v4i>::type FragT;
    static_assert(!F8 || (OUT != OUT_I32 && !COLSCALE), "the float8 product has dequantized outputs and a tensor-wise weight state");
    static_assert(!POST || (OUT != OUT_I32 && !COLSCALE && !F8), "bias / layer-scale follow the tensor-wise int8 dequantization");
    static_assert(KKG >= 2 && KKG % 2 == 0, "the register double-buffering alternates per k-step group within a stage");
    constexpr int NSCALE = OUT != OUT_I32 ? MT + (COLSCALE ? C::NT * 4 : 0) : 0;  // per-lane scale loads per tile
    constexpr int NFRAG = MT + C::NT;
    constexpr int EPI_STORES = MT * C::STORES_PER_BLOCK;  // 16-byte global stores per lane per tile

    const int tid = threadIdx.x, lane = tid & 63;
    const int wn0 = (wave % C::WAVES_N) * C::WTN;
    const int KT = p.K / C::BK;
    const bool loader = wave < C::LOADERS;

    // Per-lane byte offset of its MFMA operand chunk inside a 32-row block of a stage, one per k-step.
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fswz = (frow / C::SWZ_DIV) % C::CPR;
    int frag_off[C::KK];
#pragma unroll
    for (int kk = 0; kk < C::KK; ++kk) frag_off[kk] = frow * C::BK + (((kk * 2 + fhalf) ^ fswz) << 4);

    // Loader role: wave w < LOADERS fills stage rows [w*RPL, (w+1)*RPL), request i of it the RPS rows from
    // w*RPL + i*RPS; they all belong to one operand.  A lane's byte offset into that operand is
    //   (tile row 0 + row in tile) * K + chunk * 16 + k-tile * BK
    // = voff[i % NVAR] (per lane, fixed) + i*RPS*K + tile_soff + kt*BK (scalars): the swizzled chunk depends on i
    // only through i % NVAR.
    const bool loads_a = wave * C::RPL < C::BM;
    const int lrow = lane / C::CPR, lpos = lane % C::CPR;
    const int row0_in_tile = (wave * C::RPL) % C::BM;
    unsigned voff[C::NVAR];
#pragma unroll
    for (int v = 0; v < C::NVAR; ++v) {
        const int r = v * C::RPS + lrow;  // row within the wave's share, for requests i with i % NVAR == v
        voff[v] = (unsigned)(row0_in_tile + lrow) * (unsigned)p.K + ((lpos ^ ((r / C::SWZ_DIV) % C::CPR)) << 4);
    }
    const unsigned req_step = (unsigned)C::RPS * (unsigned)p.K;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(loads_a ? p.a : p.b), 0, (unsigned)((size_t)(loads_a ? p.M : p.N) * (size_t)p.K), 0x00020000);
    unsigned tile_soff = 0;  // byte offset of the current tile's first row in the operand this wave loads
    auto set_tile_sources = [&](int tm, int tn) {
        tile_soff = (unsigned)(loads_a ? tm * C::BM : tn * C::BN) * (unsigned)p.K;
    };
    auto issue_stage = [&](int slot, int kt) {
        unsigned char *dst = smem + slot * C::STAGE_BYTES + wave * C::RPL * C::BK;
        const unsigned soff = tile_soff + (unsigned)kt * C::BK;
#pragma unroll
        for (int i = 0; i < C::LPW; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)(dst + i * 1024), 16, voff[i % C::NVAR],
                                                     soff + (unsigned)i * req_step, 0, 0);
    };

    // MFMA operand fragments, double-buffered in registers.  A k-step group issues its MFMAs in the order
    // (x0,w0) (x0,w1) (x1,w0) (x1,w1) ... and reads the NEXT group's fragments in the order w0 x0 w1 x1 x2 x3 ..., one
    // read after each of its first MT+2 MFMAs.
    FragT xf[2][MT], wf[2][C::NT];
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    static_assert((C::BM + C::BN) * C::BK <= 65536, "fragment offsets must fit the 16-bit ds offset field");
    const unsigned x_off = wm0 * C::BK, w_off = (C::BM + wn0) * C::BK;
    // i-th fragment read of the group (stage in LDS slot `slot`, k-step kk) into register buffer buf.
    auto issue_frag_read = [&](int i, int buf, int slot, int kk) {
        const unsigned at = lds_base + slot * C::STAGE_BYTES + frag_off[kk * RPF];
        const unsigned at2 = lds_base + slot * C::STAGE_BYTES + frag_off[kk * RPF + RPF - 1];  // second half (float8)
        auto read = [&](auto off, unsigned base) -> FragT {
            constexpr int OFF = decltype(off)::value;
            if constexpr (F8) {
                const v4i lo = lds_read_b128<OFF>(at + base);
                const v4i hi = lds_read_b128<OFF>(at2 + base);
                return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            } else {
                return lds_read_b128<OFF>(at + base);
            }
        };
        switch (i) {
            case 0: wf[buf][0] = read(std::integral_constant<int, 0>(), w_off); break;
            case 1: xf[buf][0] = read(std::integral_constant<int, 0>(), x_off); break;
            case 2: wf[buf][1] = read(std::integral_constant<int, 32 * C::BK>(), w_off); break;
            case 3: xf[buf][1] = read(std::integral_constant<int, 32 * C::BK>(), x_off); break;
            case 4: xf[buf][2 % MT] = read(std::integral_constant<int, 64 * C::BK>(), x_off); break;
            case 5: xf[buf][3 % MT] = read(std::integral_constant<int, 96 * C::BK>(), x_off); break;
            default: xf[buf][4 % MT] = read(std::integral_constant<int, 128 * C::BK>(), x_off); break;
        }
    };
    // Ties the register of the i-th fragment read to the wait that precedes this call.
    auto pin_frag = [&](int i, int buf) {
        switch (i) {
            case 0: asm volatile("" : "+v"(wf[buf][0])); break;
            case 1: asm volatile("" : "+v"(xf[buf][0])); break;
            case 2: asm volatile("" : "+v"(wf[buf][1])); break;
            case 3: asm volatile("" : "+v"(xf[buf][1])); break;
            case 4: asm volatile("" : "+v"(xf[buf][2 % MT])); break;
            case 5: asm volatile("" : "+v"(xf[buf][3 % MT])); break;
            default: asm volatile("" : "+v"(xf[buf][4 % MT])); break;
        }
    };
    // n counts fragments; the counter counts reads.
    static_assert(RPF * (MT + C::NT) <= 15, "lgkmcnt is a 4-bit counter");
    auto wait_lgkm_at_most = [&](int n) {
        switch (n * RPF) {
            case 0: wait_lgkmcnt<0>(); break;
            case 1: wait_lgkmcnt<1>(); break;
            case 2: wait_lgkmcnt<2>(); break;
            case 3: wait_lgkmcnt<3>(); break;
            case 4: wait_lgkmcnt<4>(); break;
            case 5: wait_lgkmcnt<5>(); break;
            case 6: wait_lgkmcnt<6>(); break;
            case 7: wait_lgkmcnt<7>(); break;
            case 8: wait_lgkmcnt<8>(); break;
            case 9: wait_lgkmcnt<9>(); break;
            case 10: wait_lgkmcnt<10>(); break;
            case 11: wait_lgkmcnt<11>(); break;
            case 12: wait_lgkmcnt<12>(); break;
            case 13: wait_lgkmcnt<13>(); break;
            default: wait_lgkmcnt<14>(); break;
        }
    };

    // Output (bf16 path) through a buffer resource: 32-bit offsets, the tile part scalar.
    const __amdgpu_buffer_rsrc_t rsrc_out =
        __builtin_amdgcn_make_buffer_rsrc(p.out, 0, (unsigned)((size_t)p.M * p.N * 2), 0x00020000);

    // c = state_tensor / 127^2, read once (the pointer may alias nothing the kernel writes).
    float tensor_scale = 0.0f;
    if (OUT != OUT_I32 && !COLSCALE) tensor_scale = F8 ? p.state_tensor[0] : p.state_tensor[0] / 16129.0f;
    asm volatile("" : "+v"(tensor_scale));

    // ---- Work list.  A segment is the k-tile range [kb, ke) of one output tile; segment i of this workgroup is the
    // tile of its i-th round of the tile walk, whole.
    struct Seg {
        int tm, tn, kb, ke;
    };
    auto segment_of = [&](int i, Seg &sg) -> bool {
        if (!gemm_tile_of(blockIdx.x, i, gridDim.x, p.tiles_m, p.tiles_n, p.group_m, &sg.tm, &sg.tn)) return false;
        sg.kb = 0;
        sg.ke = KT;
        return true;
    };

    // ---- Vector-memory bookkeeping.  younger[s] counts the vector-memory operations this wave has issued after the
    // requests of the stage now in LDS slot s (younger_scale: after the row-scale loads of the current segment).
    // The operations of a wave retire in order, so "at most younger[s] outstanding" means that stage has landed,
    // whatever else (later stages, output stores, scale loads) is still in flight behind it.
    int younger[S], younger_scale = 0;
#pragma unroll
    for (int i = 0; i < S; ++i) younger[i] = 0;
    auto note_vmem = [&](int n) {
#pragma unroll
        for (int i = 0; i < S; ++i) younger[i] += n;
        younger_scale += n;
    };
    auto wait_vmem_at_most = [&](int n) {
        switch (n < 63 ? n : 63) {
#define SB_CASE4(b) case b: wait_vmcnt<b>(); break; case b + 1: wait_vmcnt<b + 1>(); break; \
                    case b + 2: wait_vmcnt<b + 2>(); break; case b + 3: wait_vmcnt<b + 3>(); break;
            SB_CASE4(0) SB_CASE4(4) SB_CASE4(8) SB_CASE4(12) SB_CASE4(16) SB_CASE4(20) SB_CASE4(24) SB_CASE4(28)
            SB_CASE4(32) SB_CASE4(36) SB_CASE4(40) SB_CASE4(44) SB_CASE4(48) SB_CASE4(52) SB_CASE4(56) SB_CASE4(60)
#undef SB_CASE4
        }
    };
    auto wait_slot_landed = [&](int slot) {
        int n = 0;
#pragma unroll
        for (int i = 0; i < S; ++i) n = slot == i ? younger[i] : n;
        wait_vmem_at_most(n);
    };

    // ---- Load cursor: runs STAGES stages ahead of the MFMAs, across segment boundaries, so a new tile's first
    // stages are requested during the last k-tiles of the one before it.  Every wave advances the cursor; only the
    // loader waves issue.
    Seg ls;
    int l_idx = 0, l_g = 0;  // segment being loaded; global count of stages requested so far (stage g lives in slot g % S)
    bool l_have = segment_of(0, ls);
    int l_kt = l_have ? ls.kb : 0;
    if (l_have) set_tile_sources(ls.tm, ls.tn);
    auto issue_next = [&]() {
        if (!l_have) return;
        const int slot = l_g % S;
        if (loader) {
            issue_stage(slot, l_kt);
            note_vmem(C::LPW);
#pragma unroll
            for (int i = 0; i < S; ++i) younger[i] = slot == i ? 0 : younger[i];
        }
        ++l_g;
        if (++l_kt == ls.ke) {
            l_have = segment_of(++l_idx, ls);
            if (l_have) {
                l_kt = ls.kb;
                set_tile_sources(ls.tm, ls.tn);
            }
        }
    };
#pragma unroll
    for (int i = 0; i < S; ++i) issue_next();

    Seg cs;
    bool have = segment_of(0, cs);
    int g = 0;  // global index of the stage the MFMAs work on
    bool first = true;
    for (int round = 0; have; ++round) {
        AccT acc[MT][C::NT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0;

        Seg ns;
        const bool next_have = segment_of(round + 1, ns);
        const int tm = cs.tm, tn = cs.tn;

        // Row absmax values of this tile, requested now so that the epilogue finds them in registers.  Inline asm with
        // a counted wait: the compiler's own wait would drain the stages in flight.
        float srow[MT];
        v4f scol[COLSCALE ? C::NT : 1][4];
        if (OUT != OUT_I32) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const float *src = p.state_row + min(tm * C::BM + wm0 + mt * 32 + frow, p.M - 1);
                asm volatile("global_load_dword %0, %1, off" : "=v"(srow[mt]) : "v"(src) : "memory");
            }
            if (COLSCALE) {
                // The column states of this lane's accumulator quads: columns nt*32 + 8q + 4*(lane/32) .. +3.
#pragma unroll
                for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float *src = p.state_col + min(tn * C::BN + wn0 + nt * 32 + 8 * q + 4 * fhalf, p.N - 4);
                        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(scol[nt][q]) : "v"(src) : "memory");
                    }
            }
            note_vmem(NSCALE);
            younger_scale = 0;
        }
        if (first) {
            // (Re)start of the fragment pipeline: the very first stage, or the stage after a segment that ended
            // without a hand-over.  Nobody has waited for this stage yet, and the slot of the stage before it (if
            // any) has not been refilled.
            if (loader) wait_slot_landed(g % S);
            wait_lds_reads();
            block_barrier();
            if (l_g < g + S) issue_next();
#pragma unroll
            for (int i = 0; i < NFRAG; ++i) issue_frag_read(i, 0, g % S, 0);
            first = false;
        }

        // One k-tile (stage g).  Its last k-step group hands the stage over and already reads the next stage's first
        // fragments, also when that stage belongs to the next segment.  A stage that ends the fragment pipeline (the
        // workgroup's last one) is a separate instantiation, so that "another k-step group follows" is known at
        // compile time and the hot loop carries no branches for it.
        auto k_tile = [&](const int kt, auto is_last_stage) __attribute__((always_inline)) {
            constexpr bool last_stage = decltype(is_last_stage)::value;
            const int slot = g % S, next_slot = (g + 1) % S;
#pragma unroll
            for (int kk = 0; kk < KKG; ++kk) {
                const bool last_group = kk + 1 == KKG;
                const bool has_next = !last_group || !last_stage;  // another k-step group follows
                const bool handed_over = last_group && has_next;
                if (handed_over) {
                    // Hand-over: the fragments of this last k-step of the stage are in (or on their way to)
                    // registers.  Retire this wave's LDS reads, make sure the next stage has landed, then refill
                    // the freed slot.
                    if (loader) wait_slot_landed(next_slot);
                    wait_lds_reads();
                    block_barrier();
                    issue_next();
                }
                const int cur = kk & 1, nxt = (kk + 1) & 1;
                const int read_slot = last_group ? next_slot : slot, next_kk = last_group ? 0 : kk + 1;
                int landed = 0;  // fragments of this group known to have landed
#pragma unroll
                for (int idx = 0; idx < MT * C::NT; ++idx) {
                    const int mt = idx / C::NT, nt = idx % C::NT;
                    // Reads of this group that MFMA idx needs: w0 x0 | w1 | x1 | - | x2 | - | x3 | - ...
                    const int need = idx == 0 ? 2 : idx == 1 ? 3 : 3 + idx / 2;
                    if (need > landed) {
                        // All but the (NFRAG - need) youngest of this group's reads, and the reads already issued
                        // for the next group, must be back.  After a hand-over everything has landed already.
                        if (!has_next)
                            wait_lgkm_at_most(NFRAG - need);
                        else if (!handed_over)
                            wait_lgkm_at_most(NFRAG - need + min(idx, NFRAG));
#pragma unroll
                        for (int i = landed; i < need; ++i) pin_frag(i, cur);
                        landed = need;
                    }
                    if constexpr (F8)
                        acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf[cur][nt], xf[cur][mt], acc[mt][nt],
                                                                                      FMT_W, FMT_X, 0, 0, 0, 0);
                    else
                        acc[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[cur][nt], xf[cur][mt], acc[mt][nt], 0, 0, 0);
                    if (idx < NFRAG && has_next) issue_frag_read(idx, nxt, read_slot, next_kk);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            ++g;
        };
        const int nkt = cs.ke - cs.kb;
        for (int kt = 0; kt < (next_have ? nkt : nkt - 1); ++kt) k_tile(kt, std::false_type());
        if (!next_have) k_tile(nkt - 1, std::true_type());
        const int m_base = tm * C::BM + wm0, n_base = tn * C::BN + wn0;
        const bool interior = (tm + 1) * C::BM <= p.M && (tn + 1) * C::BN <= p.N;

        // Bias and layer-scale of this lane's accumulator quads (columns nt*32 + 8q + 4*(lane/32) .. +3).  Waiting for
        // them drains the vector-memory queue, the next tile's first stages included; they have mostly landed by now.
        v4f pbias[POST ? C::NT : 1][4], pgamma[POST ? C::NT : 1][4];
        const bool has_bias = POST && p.bias != nullptr, has_gamma = POST && p.gamma != nullptr;
        if (POST) {
#pragma unroll
            for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = min(tn * C::BN + wn0 + nt * 32 + 8 * q + 4 * fhalf, p.N - 4);
                    pbias[nt][q] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
                    pgamma[nt][q] = v4f{1.0f, 1.0f, 1.0f, 1.0f};
                    if (has_bias) {
                        const float *src = p.bias + col;
                        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(pbias[nt][q]) : "v"(src) : "memory");
                    }
                    if (has_gamma) {
                        const float *src = p.gamma + col;
                        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(pgamma[nt][q]) : "v"(src) : "memory");
                    }
                }
            note_vmem((has_bias ? C::NT * 4 : 0) + (has_gamma ? C::NT * 4 : 0));
            wait_vmem_at_most(0);
#pragma unroll
            for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    asm volatile("" : "+v"(pbias[nt][q]));
                    asm volatile("" : "+v"(pgamma[nt][q]));
                }
        }
        // The value stored for accumulator element e of quad (nt, q) in 32-row block mt.
        auto finish = [&](float y, int nt, int q, int e) -> float {
            if (POST) {
                if (has_bias) y = y + pbias[nt][q][e];      // -0 + 0 would lose the sign: skipped, not added, when absent
                if (has_gamma) y = pgamma[nt][q][e] * y;
            }
            return y;
        };

        // Row scales r_i = state_row[i] * (state_tensor / 127^2), one per lane per 32-row block.
        float rscale[MT];
        if (OUT != OUT_I32) {
            wait_vmem_at_most(younger_scale);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) asm volatile("" : "+v"(srow[mt]));
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) rscale[mt] = COLSCALE ? srow[mt] : srow[mt] * tensor_scale;
            if (COLSCALE) {
#pragma unroll
                for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        asm volatile("" : "+v"(scol[nt][q]));
                        scol[nt][q] = scol[nt][q] / 16129.0f;  // c_j = state_col[j] / 127^2, correctly rounded
                    }
            }
        }

        // The epilogue needs no barrier: the patch is private to the wave, and the next segment's first stages are
        // already in flight (or landed).
        {
        // The lane-dependent addresses of the epilogue are recomputed here from an opaque copy of the lane id, so that
        // the compiler does not keep them in registers through the main loop, where every register counts.
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        const int frow = lane_e & 31, fhalf = lane_e >> 5;
        if (OUT == OUT_BF16) {
            unsigned char *epi = smem + S * C::STAGE_BYTES + wave * C::EPI_WAVE_BYTES;
            const unsigned epi_voff = (unsigned)((lane_e / C::EPI_PIECES) * p.N + (lane_e % C::EPI_PIECES) * 8) * 2;
            // Software pipeline over the 32-row blocks.  The patch reads of block mt are all issued first, block mt+1
            // is converted while they travel, then the stores of block mt go out and the patch is rewritten: LDS
            // operations of one wave execute in order, so the rewrite needs no wait for the reads before it.  The
            // stores of an interior tile are branch-free; a branch per store would put a full wait after every read.
            v4bf packed[C::NT * 4];
            auto convert_block = [&](int mt) {
#pragma unroll
                for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        v4f v;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            v[e] = finish((float)(acc[mt][nt][4 * q + e]) *
                                              (COLSCALE ? rscale[mt] * scol[nt][q][e] : rscale[mt]),
                                          nt, q, e);
                        packed[nt * 4 + q] = __builtin_convertvector(v, v4bf);
                    }
            };
            auto write_patch = [&]() {
#pragma unroll
                for (int i = 0; i < C::NT * 4; ++i) {
                    const int piece = i ^ (frow & 7);
                    *reinterpret_cast<v4bf *>(epi + frow * (C::WTN * 2) + piece * 16 + fhalf * 8) = packed[i];
                }
            };
            convert_block(0);
            write_patch();
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                v4u val[C::STORES_PER_BLOCK];
#pragma unroll
                for (int j = 0; j < C::STORES_PER_BLOCK; ++j) {
                    const int idx = j * 64 + lane_e;
                    const int prow = idx / C::EPI_PIECES, piece = idx % C::EPI_PIECES;
                    val[j] = *reinterpret_cast<const v4u *>(epi + prow * (C::WTN * 2) + ((piece ^ (prow & 7)) << 4));
                }
                if (mt + 1 < MT) convert_block(mt + 1);
                // Row block j of this 32-row block starts (64 / EPI_PIECES) * j rows down; the lane's place inside it
                // is the per-lane constant epi_voff.
                if (interior) {
#pragma unroll
                    for (int j = 0; j < C::STORES_PER_BLOCK; ++j) {
                        const unsigned soff =
                            (unsigned)((m_base + mt * 32 + j * (64 / C::EPI_PIECES)) * p.N + n_base) * 2;
                        __builtin_amdgcn_raw_buffer_store_b128(val[j], rsrc_out, epi_voff, soff, C::STORE_NT ? 2 : 0);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < C::STORES_PER_BLOCK; ++j) {
                        const int idx = j * 64 + lane_e;
                        const int prow = idx / C::EPI_PIECES, piece = idx % C::EPI_PIECES;
                        const int gr = m_base + mt * 32 + prow, gc = n_base + piece * 8;
                        const unsigned soff =
                            (unsigned)((m_base + mt * 32 + j * (64 / C::EPI_PIECES)) * p.N + n_base) * 2;
                        if (gr < p.M && gc < p.N)
                            __builtin_amdgcn_raw_buffer_store_b128(val[j], rsrc_out, epi_voff, soff,
                                                                   C::STORE_NT ? 2 : 0);
                    }
                }
                if (mt + 1 < MT) write_patch();
            }
            // Count the stores only where every one of them is certain to have been issued: an overcount would
            // loosen later waits, an undercount merely makes them stricter.
            if (interior) note_vmem(EPI_STORES);
        } else {
            // Verification paths: binary32 results or raw accumulators, stored straight from the registers.
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                for (int nt = 0; nt < C::NT; ++nt) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int gr = m_base + mt * 32 + frow, gc = n_base + nt * 32 + 8 * q + 4 * fhalf;
                        if (gr < p.M && gc < p.N) {
                            if (OUT == OUT_F32) {
                                v4f v;
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    v[e] = finish((float)(acc[mt][nt][4 * q + e]) *
                                                      (COLSCALE ? rscale[mt] * scol[nt][q][e] : rscale[mt]),
                                                  nt, q, e);
                                *reinterpret_cast<v4f *>(static_cast<float *>(p.out) + (int64_t)gr * p.N + gc) = v;
                            } else {
                                v4i v;
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    v[e] = (int)acc[mt][nt][4 * q + e];
                                *reinterpret_cast<v4i *>(static_cast<int *>(p.out) + (int64_t)gr * p.N + gc) = v;
                            }
                        }
                    }
                }
            }
        }
        }
        cs = ns;
        have = next_have;
    }
}

// The kernel body.  It is a __device__ template called from non-template __global__ entry points: a __global__
// template that uses device-only buffer builtins does not instantiate in the host pass.
template <class C, int OUT, bool COLSCALE = false, int MATH = MATH_I8, bool POST = false>
__device__ __forceinline__ void gemm_i8_dequant_body(const GemmI8Args &p) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform: what derives from it is scalar
    if (C::MT_LOADER == C::MT_EVEN)
        gemm_i8_dequant_role<C, OUT, C::MT_EVEN, COLSCALE, MATH, POST>(p, wave, (wave / C::WAVES_N) * C::WTM);
    else if (wave < C::LOADERS)
        gemm_i8_dequant_role<C, OUT, C::MT_LOADER, COLSCALE, MATH, POST>(p, wave, 0);
    else
        gemm_i8_dequant_role<C, OUT, 2 * C::MT_EVEN - C::MT_LOADER, COLSCALE, MATH, POST>(p, wave, C::MT_LOADER * 32);
}

// Launch geometry shared by the entry points: a persistent grid, a multiple of the XCD count, at most one workgroup
// per compute unit.  When the tiles make only a few rounds of the full grid and do not fill the last one, the grid is
// shrunk so that every workgroup gets the same number of tiles (645 tiles: 216 workgroups x 3 instead of 256 x 2.5):
// the number of rounds is the same, and the kernel being power-bound, fewer active compute units run at a higher
// clock, which measures 4-10 % faster than a last round that leaves half the GPU idle.  With many rounds the tail is
// a small share and the full grid measures better.
template <class C>
inline void gemm_i8_prepare(GemmI8Args &a, int workgroups, int *grid, bool balance = true) {
    a.tiles_m = (a.M + C::BM - 1) / C::BM;
    a.tiles_n = (a.N + C::BN - 1) / C::BN;
    if (a.group_m <= 0) a.group_m = 8;
    int full = workgroups & ~7;
    if (full < 8) full = 8;
    int g = full;
    if (balance) {
        const long long tiles = (long long)a.tiles_m * a.tiles_n;
        const long long rounds = (tiles + full - 1) / full;
        const long long per_round = (tiles + rounds - 1) / rounds;
        if (rounds <= 4) g = (int)((per_round + 7) & ~7LL);
        if (g > full) g = full;
        if (g < 8) g = 8;
    }
    *grid = g;
}

}  // namespace sb
