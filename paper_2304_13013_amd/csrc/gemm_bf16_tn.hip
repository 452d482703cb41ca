// Weight-gradient GEMM of the SwitchBack layer (Algorithm 1 of arxiv 2304.13013: the product the layer keeps in
// 16 bit): dW[j,k] = sum_i dY[i,j] * X[i,k], bf16 operands, binary32 accumulation, hand-written for gfx950.
//
// Both operands are stored with the contraction index (the token i) as the SLOW axis: a row of dY holds m
// consecutive outputs of one token, a row of X holds n consecutive inputs.  v_mfma_f32_32x32x16_bf16 wants, per
// lane, 8 consecutive-k values of ONE output row/column, so the tiles are transposed on their way into LDS:
// a thread loads a 4(k) x 8(column) patch as four 16-byte row pieces, regroups it with v_perm_b32 into eight
// 4(k)-element column pieces and writes those into 16-byte LDS units laid out [k/8][column][k%8].  A lane's MFMA
// operand is then one ds_read_b128.  Unit index XOR ((column >> 4) & 7) spreads the transposing writes over the
// banks and keeps the reads (32 consecutive columns) conflict free.
//
// The X-side tile is the MFMA's first operand and the dY-side tile its second, so a lane owns one dW row
// (lane % 32) and four consecutive dW columns per accumulator quad.
//
// The contraction is long (b ~ 32k) and the output small, so the grid is tiles x splits (split-K); with more
// than one split the partial sums go to a binary32 workspace [split][m][n] and a second kernel adds them in
// split order (deterministic) and converts to the output type.
#include "sb_common.h"

namespace sb {
namespace {

constexpr int BM = 256;   // dW rows per tile (dY columns)
constexpr int BN = 256;   // dW columns per tile (X columns)
constexpr int BK = 32;    // tokens per stage
constexpr int WAVES_M = 2, WAVES_N = 4, THREADS = 512;
constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;  // 128 x 64 per wave
constexpr int MT = WTM / 32, NT = WTN / 32;
constexpr int KG = BK / 8;                             // 16-byte k-groups per stage
constexpr int OPERAND_BYTES = KG * 256 * 16;           // one operand tile in LDS (256 columns)
constexpr int STAGE_BYTES = 2 * OPERAND_BYTES;
constexpr int MAX_SPLITS = 16;

__device__ __forceinline__ int swizzle_col(int c) { return c ^ ((c >> 4) & 7); }

struct GemmBf16Args {
    const unsigned short *dy;  // [b,m]
    const unsigned short *x;   // [b,n]
    float *partial;            // [splits][m][n] when splits > 1
    void *out;                 // [m,n] when splits == 1
    int b, n, m;
    int tiles_m, tiles_n, splits, k_per_split;  // k_per_split is a multiple of BK
    int out_bf16;
};

__global__ __launch_bounds__(THREADS) void gemm_bf16_tn_kernel(GemmBf16Args p) {
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * STAGE_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WAVES_N) * WTM, wn0 = (wave % WAVES_N) * WTN;

    // Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous run of (split, tile) work items in
    // split-major order, so that the workgroups sharing an L2 read the same token range of dY and X.
    const int total = p.tiles_m * p.tiles_n * p.splits;
    const int per_xcd = (total + 7) / 8;
    const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (item >= total || (int)(blockIdx.x >> 3) >= per_xcd) return;  // uniform per workgroup
    const int split = item / (p.tiles_m * p.tiles_n), tile = item % (p.tiles_m * p.tiles_n);
    const int tm = tile / p.tiles_n, tn = tile % p.tiles_n;
    const int k_begin = split * p.k_per_split;
    const int k_end = min(p.b, k_begin + p.k_per_split);
    const int KT = (k_end - k_begin + BK - 1) / BK;

    // Loader role: operand (dY or X), column chunk of 8, token quad.
    const int l_op = tid >> 8, l_mc = tid & 31, l_kq = (tid >> 5) & 7;
    const unsigned short *src = l_op == 0 ? p.dy : p.x;
    const int ld = l_op == 0 ? p.m : p.n;
    const int col = (l_op == 0 ? tm * BM : tn * BN) + l_mc * 8;
    const bool col_ok = col < ld;
    unsigned char *wr_base = smem + l_op * OPERAND_BYTES + (l_kq >> 1) * 256 * 16 + (l_kq & 1) * 8;

    v4u staged[4];
    auto load_stage = [&](int kt) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int k = k_begin + kt * BK + l_kq * 4 + e;
            staged[e] = (col_ok && k < k_end)
                            ? *reinterpret_cast<const v4u *>(src + (int64_t)k * ld + col)
                            : v4u{0u, 0u, 0u, 0u};
        }
    };
    auto write_stage = [&](int stage) {
        unsigned char *base = wr_base + stage * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int d = j >> 1;
            const unsigned int sel = (j & 1) ? 0x07060302u : 0x05040100u;  // high or low halves of two dwords
            v2u piece;
            piece.x = __builtin_amdgcn_perm(staged[1][d], staged[0][d], sel);
            piece.y = __builtin_amdgcn_perm(staged[3][d], staged[2][d], sel);
            *reinterpret_cast<v2u *>(base + swizzle_col(l_mc * 8 + j) * 16) = piece;
        }
    };

    const int frow = lane & 31, fkb = lane >> 5;
    v16f acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.0f;

    if (KT > 0) load_stage(0);
    for (int kt = 0; kt < KT; ++kt) {
        write_stage(kt & 1);
        if (kt + 1 < KT) load_stage(kt + 1);
        __syncthreads();
        const unsigned char *gs = smem + (kt & 1) * STAGE_BYTES;   // dY-side tile (dW rows)
        const unsigned char *xs = gs + OPERAND_BYTES;              // X-side tile (dW columns)
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            v8bf gf[MT], xf[NT];
            const int kg = kk * 2 + fkb;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                gf[mt] = *reinterpret_cast<const v8bf *>(gs + (kg * 256 + swizzle_col(wm0 + mt * 32 + frow)) * 16);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                xf[nt] = *reinterpret_cast<const v8bf *>(xs + (kg * 256 + swizzle_col(wn0 + nt * 32 + frow)) * 16);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[nt], gf[mt], acc[mt][nt], 0, 0, 0);
        }
    }

    // Lane owns dW row (frow) of each 32-row block and columns 8g + 4*(lane/32) + e of each 32-column block.
    float *pout = p.splits > 1 ? p.partial + (int64_t)split * p.m * p.n : static_cast<float *>(p.out);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int gr = tm * BM + wm0 + mt * 32 + frow;
                const int gc = tn * BN + wn0 + nt * 32 + 8 * g + 4 * fkb;
                if (gr < p.m && gc < p.n) {
                    v4f v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[mt][nt][4 * g + e];
                    if (p.splits == 1 && p.out_bf16)
                        *reinterpret_cast<v4bf *>(static_cast<unsigned short *>(p.out) + (int64_t)gr * p.n + gc) =
                            __builtin_convertvector(v, v4bf);
                    else
                        *reinterpret_cast<v4f *>(pout + (int64_t)gr * p.n + gc) = v;
                }
            }
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

// Splits: fill the compute units in whole rounds with as few splits as that takes.
int choose_splits(int64_t b, int tiles) {
    const int ncu = 256;
    int best = 1;
    double best_score = -1.0;
    for (int s = 1; s <= MAX_SPLITS; ++s) {
        if ((int64_t)s * BK * 4 > b && s > 1) break;  // keep every split at least a few stages long
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

}  // namespace

size_t gemm_bf16_tn_workspace_bytes(int64_t b, int64_t n, int64_t m) {
    const int tiles = (int)(((m + BM - 1) / BM) * ((n + BN - 1) / BN));
    const int s = choose_splits(b, tiles);
    return s > 1 ? (size_t)s * (size_t)m * (size_t)n * sizeof(float) : 0;
}

hipError_t launch_gemm_bf16_tn(const void *dy, const void *x, int64_t b, int64_t n, int64_t m, void *dw,
                               sb_dtype dw_dtype, void *ws, hipStream_t stream) {
    GemmBf16Args a;
    a.dy = static_cast<const unsigned short *>(dy);
    a.x = static_cast<const unsigned short *>(x);
    a.b = (int)b;
    a.n = (int)n;
    a.m = (int)m;
    a.tiles_m = (int)((m + BM - 1) / BM);
    a.tiles_n = (int)((n + BN - 1) / BN);
    a.splits = choose_splits(b, a.tiles_m * a.tiles_n);
    const int64_t stages = (b + BK - 1) / BK;
    a.k_per_split = (int)((stages + a.splits - 1) / a.splits) * BK;
    a.partial = static_cast<float *>(ws);
    a.out = dw;
    a.out_bf16 = dw_dtype == SB_BF16;
    const int total = a.tiles_m * a.tiles_n * a.splits;
    gemm_bf16_tn_kernel<<<8 * ((total + 7) / 8), THREADS, 0, stream>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.splits == 1) return e;
    const int64_t quads = m * n / 4;
    splitk_reduce_kernel<<<(unsigned int)((quads + 255) / 256), 256, 0, stream>>>(
        static_cast<const v4f *>(ws), quads, a.splits, dw, a.out_bf16);
    return hipGetLastError();
}

}  // namespace sb
