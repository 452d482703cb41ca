// Fused absmax + int8 quantization kernels for gfx950 (row-wise and tensor-wise quantization equations of
// Section 2.2.1 of arxiv 2304.13013).
//
// Arithmetic (bit-exact contract): the absmax is taken on the bf16 bit patterns (|x| is monotone in the low 15
// bits), the scale is t = 127/absmax as one correctly rounded binary32 divide, each code is the
// round-half-to-even integer of the rounded binary32 product x*t.  The rounding uses the 1.5*2^23 trick: adding
// that constant to a value of magnitude <= 127.5 leaves the nearest-even integer in the low mantissa bits, whose
// low byte is the two's-complement int8 code.  The product and the addition are separate roundings (the file is
// compiled with contraction off), and binary32 subnormals are preserved (the default float mode of HIP kernels).
//
// The float8 variant of the layer (the "float8" paragraph of the same section: float8cast(x / absmax(x)) in place of
// round(127 x / absmax(x))) runs through the same kernels with CODE = CODE_E4M3 or CODE_E5M2: the scale is
// t = 1/absmax (one correctly rounded divide), each code is the hardware's round-to-nearest-even conversion
// (v_cvt_pk_fp8_f32 / v_cvt_pk_bf8_f32, OCP formats on gfx950) of the rounded binary32 product x*t.
//
// All three kernels are HBM-bound: one 16-byte load per 8 elements, the row (or tile) stays in registers between
// the absmax and the quantization, codes leave as 8- or 16-byte stores.
#include "sb_common.h"

namespace sb {
namespace {

constexpr float kRoundMagic = 12582912.0f;  // 1.5 * 2^23

enum { CODE_INT8 = 0, CODE_E4M3 = 1, CODE_E5M2 = 2 };

__device__ __forceinline__ unsigned int pk_absmax_u16(unsigned int running, unsigned int two_bf16) {
    v2us a = __builtin_bit_cast(v2us, running);
    v2us b = __builtin_bit_cast(v2us, two_bf16 & 0x7fff7fffu);
    return __builtin_bit_cast(unsigned int, __builtin_elementwise_max(a, b));
}

__device__ __forceinline__ unsigned int absmax_of_chunk(unsigned int running, v4u c) {
    running = pk_absmax_u16(running, c.x);
    running = pk_absmax_u16(running, c.y);
    running = pk_absmax_u16(running, c.z);
    return pk_absmax_u16(running, c.w);
}

__device__ __forceinline__ unsigned int wave_max_u32(unsigned int v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        unsigned int o = (unsigned int)__shfl_xor((int)v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

// absmax bit pattern (15 bits) -> (scale t, stored state).  Zero rows and rows whose scale would overflow
// binary32 quantize to zeros and store state 0.
template <int CODE = CODE_INT8>
__device__ __forceinline__ float scale_from_absmax_bits(unsigned int bits15, float *stored_state) {
    float s = bf16_bits_to_float(bits15);
    float t = (CODE == CODE_INT8 ? 127.0f : 1.0f) / s;
    if (bits15 == 0u || __builtin_isinf(t)) {
        t = 0.0f;
        s = 0.0f;
    }
    *stored_state = s;
    return t;
}

__device__ __forceinline__ unsigned int code_bits(float x, float t) {
    float p = x * t;            // one rounding
    float r = p + kRoundMagic;  // second rounding: nearest-even integer lands in the low mantissa bits
    return __float_as_uint(r);
}

// 8 bf16 (4 dwords, element 2d in the low half of dword d) -> 8 one-byte codes (2 dwords).
template <int CODE = CODE_INT8>
__device__ __forceinline__ v2u quantize_chunk(v4u c, float t) {
    if (CODE != CODE_INT8) {
        const unsigned int d[4] = {c.x, c.y, c.z, c.w};
        float p[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            p[2 * j] = __uint_as_float(d[j] << 16) * t;  // one rounding each
            p[2 * j + 1] = __uint_as_float(d[j] & 0xffff0000u) * t;
        }
        int lo = 0, hi = 0;  // the conversion writes one 16-bit half of its destination and keeps the other
        if (CODE == CODE_E4M3) {
            lo = __builtin_amdgcn_cvt_pk_fp8_f32(p[0], p[1], lo, false);
            lo = __builtin_amdgcn_cvt_pk_fp8_f32(p[2], p[3], lo, true);
            hi = __builtin_amdgcn_cvt_pk_fp8_f32(p[4], p[5], hi, false);
            hi = __builtin_amdgcn_cvt_pk_fp8_f32(p[6], p[7], hi, true);
        } else {
            lo = __builtin_amdgcn_cvt_pk_bf8_f32(p[0], p[1], lo, false);
            lo = __builtin_amdgcn_cvt_pk_bf8_f32(p[2], p[3], lo, true);
            hi = __builtin_amdgcn_cvt_pk_bf8_f32(p[4], p[5], hi, false);
            hi = __builtin_amdgcn_cvt_pk_bf8_f32(p[6], p[7], hi, true);
        }
        return v2u{(unsigned int)lo, (unsigned int)hi};
    }
    unsigned int r[8];
    r[0] = code_bits(__uint_as_float(c.x << 16), t);
    r[1] = code_bits(__uint_as_float(c.x & 0xffff0000u), t);
    r[2] = code_bits(__uint_as_float(c.y << 16), t);
    r[3] = code_bits(__uint_as_float(c.y & 0xffff0000u), t);
    r[4] = code_bits(__uint_as_float(c.z << 16), t);
    r[5] = code_bits(__uint_as_float(c.z & 0xffff0000u), t);
    r[6] = code_bits(__uint_as_float(c.w << 16), t);
    r[7] = code_bits(__uint_as_float(c.w & 0xffff0000u), t);
    // v_perm_b32: selector bytes 0-3 pick from the second operand, 4-7 from the first, 0x0c gives zero.
    unsigned int p01 = __builtin_amdgcn_perm(r[1], r[0], 0x0c0c0400u);
    unsigned int p23 = __builtin_amdgcn_perm(r[3], r[2], 0x0c0c0400u);
    unsigned int p45 = __builtin_amdgcn_perm(r[5], r[4], 0x0c0c0400u);
    unsigned int p67 = __builtin_amdgcn_perm(r[7], r[6], 0x0c0c0400u);
    v2u out;
    out.x = __builtin_amdgcn_perm(p23, p01, 0x05040100u);
    out.y = __builtin_amdgcn_perm(p67, p45, 0x05040100u);
    return out;
}

// The first pass of the tensor-wise quantizer (per-workgroup partial absmax of W) as a rider on a row-wise launch:
// workgroups [first_block, first_block + nblocks) of the grid do it instead of a row.  The forward pass quantizes X
// row-wise and W tensor-wise; the two are independent, and W's first pass is a few microseconds of work that is
// mostly launch overhead when it runs alone.  nblocks == 0: no rider.
struct TensorAbsmaxJob {
    const v4u *w;
    int64_t nchunks;
    unsigned int *partials;
    int nblocks, first_block;
};

__device__ __forceinline__ void absmax_partial_body(const v4u *__restrict__ w, int64_t nchunks,
                                                    unsigned int *__restrict__ partials, int block, int nblocks,
                                                    unsigned int *wave_max /* shared, 4 entries */) {
    unsigned int m = 0;
    const int64_t stride = (int64_t)nblocks * 256;
    for (int64_t c = (int64_t)block * 256 + threadIdx.x; c < nchunks; c += stride) m = absmax_of_chunk(m, w[c]);
    m = wave_max_u32(max(m & 0xffffu, m >> 16));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) partials[block] = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
}

// ---- row-wise: one wavefront per row (cols <= 64*8*NCH) ---------------------------------------------------
template <int NCH, int CODE>
__global__ __launch_bounds__(256) void quantize_rowwise_wave_kernel(const v4u *__restrict__ x, int64_t rows,
                                                                    int chunks, v2u *__restrict__ q,
                                                                    float *__restrict__ state, TensorAbsmaxJob job) {
    __shared__ unsigned int rider_max[4];
    if (job.nblocks > 0 && (int)blockIdx.x >= job.first_block) {  // uniform per workgroup
        absmax_partial_body(job.w, job.nchunks, job.partials, (int)blockIdx.x - job.first_block, job.nblocks, rider_max);
        return;
    }
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;  // whole wavefront leaves; the kernel has no block-level barrier
    const v4u *xr = x + row * chunks;
    v4u v[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        int c = lane + 64 * i;
        v[i] = c < chunks ? __builtin_nontemporal_load(xr + c) : v4u{0u, 0u, 0u, 0u};
    }
    unsigned int m = 0;
#pragma unroll
    for (int i = 0; i < NCH; ++i) m = absmax_of_chunk(m, v[i]);
    m = wave_max_u32(max(m & 0xffffu, m >> 16));
    float s;
    const float t = scale_from_absmax_bits<CODE>(m, &s);
    if (lane == 0) state[row] = s;
    v2u *qr = q + row * chunks;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        int c = lane + 64 * i;
        if (c < chunks) qr[c] = quantize_chunk<CODE>(v[i], t);
    }
}

// ---- row-wise: one 256-thread block per row (cols <= 256*8*NCH) ---------------------------------------------
template <int NCH, int CODE>
__global__ __launch_bounds__(256) void quantize_rowwise_block_kernel(const v4u *__restrict__ x, int chunks,
                                                                     v2u *__restrict__ q,
                                                                     float *__restrict__ state, TensorAbsmaxJob job) {
    __shared__ unsigned int wave_max[4];
    if (job.nblocks > 0 && (int)blockIdx.x >= job.first_block) {  // uniform per workgroup
        absmax_partial_body(job.w, job.nchunks, job.partials, (int)blockIdx.x - job.first_block, job.nblocks, wave_max);
        return;
    }
    const int64_t row = blockIdx.x;
    const v4u *xr = x + row * chunks;
    v4u v[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        int c = threadIdx.x + 256 * i;
        v[i] = c < chunks ? __builtin_nontemporal_load(xr + c) : v4u{0u, 0u, 0u, 0u};
    }
    unsigned int m = 0;
#pragma unroll
    for (int i = 0; i < NCH; ++i) m = absmax_of_chunk(m, v[i]);
    m = wave_max_u32(max(m & 0xffffu, m >> 16));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    m = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
    float s;
    const float t = scale_from_absmax_bits<CODE>(m, &s);
    if (threadIdx.x == 0) state[row] = s;
    v2u *qr = q + row * chunks;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        int c = threadIdx.x + 256 * i;
        if (c < chunks) qr[c] = quantize_chunk<CODE>(v[i], t);
    }
}

// ---- row-wise: very wide rows, two passes over the row (the second one hits L2) ---------------------------
template <int CODE>
__global__ __launch_bounds__(256) void quantize_rowwise_wide_kernel(const v4u *__restrict__ x, int chunks,
                                                                    v2u *__restrict__ q,
                                                                    float *__restrict__ state, TensorAbsmaxJob job) {
    __shared__ unsigned int wave_max[4];
    if (job.nblocks > 0 && (int)blockIdx.x >= job.first_block) {  // uniform per workgroup
        absmax_partial_body(job.w, job.nchunks, job.partials, (int)blockIdx.x - job.first_block, job.nblocks, wave_max);
        return;
    }
    const int64_t row = blockIdx.x;
    const v4u *xr = x + row * chunks;
    unsigned int m = 0;
    for (int c = threadIdx.x; c < chunks; c += 256) m = absmax_of_chunk(m, xr[c]);
    m = wave_max_u32(max(m & 0xffffu, m >> 16));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    m = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
    float s;
    const float t = scale_from_absmax_bits<CODE>(m, &s);
    if (threadIdx.x == 0) state[row] = s;
    v2u *qr = q + row * chunks;
    for (int c = threadIdx.x; c < chunks; c += 256) qr[c] = quantize_chunk<CODE>(xr[c], t);
}

// ---- tensor-wise pass 1: per-block partial absmax (bit patterns) --------------------------------------------
__global__ __launch_bounds__(256) void absmax_partial_kernel(const v4u *__restrict__ w, int64_t nchunks,
                                                             unsigned int *__restrict__ partials) {
    __shared__ unsigned int wave_max[4];
    absmax_partial_body(w, nchunks, partials, (int)blockIdx.x, (int)gridDim.x, wave_max);
}

// ---- tensor-wise pass 2: finish the absmax, quantize a 128x128 tile, emit it row-major and transposed ------
// The transposed copy goes through LDS so that both code matrices leave in 128-byte row segments while W is read
// once in this pass.
constexpr int kTile = 128;
// The tile's codes sit in LDS row-major as dwords (4 codes each), 33 dwords per row and the lower half of the rows
// shifted by another 8, which makes the transposing read-out below free of bank conflicts.
constexpr int kTileRowDwords = kTile / 4 + 1;
constexpr int kTileDwords = kTile * kTileRowDwords + 8;
__device__ __forceinline__ int tile_dword(int row, int dcol) { return row * kTileRowDwords + ((row >> 6) << 3) + dcol; }

// Writes the transposed tile: q_t[c0 + c, r0 + r] = tile[r, c].  Thread t takes the four columns 4*(t/8).. and the
// sixteen rows 16*(t%8)..: sixteen dword reads, 4x4 byte transposes with v_perm_b32, four 16-byte stores; eight
// consecutive lanes cover 128 contiguous bytes of one transposed row.
__device__ __forceinline__ void store_tile_transposed(const unsigned int *tile, int8_t *__restrict__ q_t, int rows,
                                                      int cols, int r0, int c0) {
    const int rb = threadIdx.x & 7, cg = threadIdx.x >> 3;
    unsigned int piece[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const unsigned int a0 = tile[tile_dword(16 * rb + 4 * g + 0, cg)], a1 = tile[tile_dword(16 * rb + 4 * g + 1, cg)];
        const unsigned int a2 = tile[tile_dword(16 * rb + 4 * g + 2, cg)], a3 = tile[tile_dword(16 * rb + 4 * g + 3, cg)];
        // v_perm_b32: selector bytes 0-3 pick from the second operand, 4-7 from the first.
        const unsigned int lo01 = __builtin_amdgcn_perm(a1, a0, 0x05010400u), hi01 = __builtin_amdgcn_perm(a1, a0, 0x07030602u);
        const unsigned int lo23 = __builtin_amdgcn_perm(a3, a2, 0x05010400u), hi23 = __builtin_amdgcn_perm(a3, a2, 0x07030602u);
        piece[0][g] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
        piece[1][g] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
        piece[2][g] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
        piece[3][g] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
    }
    const int r = r0 + 16 * rb;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int c = c0 + 4 * cg + k;
        if (c < cols && r < rows)
            *reinterpret_cast<v4u *>(q_t + (int64_t)c * rows + r) = v4u{piece[k][0], piece[k][1], piece[k][2], piece[k][3]};
    }
}

template <int CODE>
__global__ __launch_bounds__(256) void quantize_tensorwise_kernel(const v4u *__restrict__ w, int rows, int cols,
                                                                  int8_t *__restrict__ q,
                                                                  int8_t *__restrict__ q_t,
                                                                  float *__restrict__ state,
                                                                  const unsigned int *__restrict__ partials,
                                                                  int npartials) {
    __shared__ unsigned int wave_max[4];
    __shared__ unsigned int tile[kTileDwords];
    unsigned int m = 0;
    for (int i = threadIdx.x; i < npartials; i += 256) m = max(m, partials[i]);
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    m = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
    float s;
    const float t = scale_from_absmax_bits<CODE>(m, &s);
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) state[0] = s;

    const int r0 = blockIdx.y * kTile, c0 = blockIdx.x * kTile;
    const int chunks_per_row = cols >> 3;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int id = threadIdx.x + 256 * i;
        const int lr = id >> 4, lc = (id & 15) << 3;  // local row, local first column of the 8-element chunk
        const int r = r0 + lr, c = c0 + lc;
        if (r < rows && c < cols) {
            const v2u codes = quantize_chunk<CODE>(w[(int64_t)r * chunks_per_row + (c >> 3)], t);
            *reinterpret_cast<v2u *>(q + (int64_t)r * cols + c) = codes;
            if (q_t) {
                tile[tile_dword(lr, lc >> 2)] = codes.x;
                tile[tile_dword(lr, (lc >> 2) + 1)] = codes.y;
            }
        }
    }
    if (!q_t) return;  // uniform across the grid
    __syncthreads();
    store_tile_transposed(tile, q_t, rows, cols, r0, c0);
}

// ---- column-wise quantization fused with a transpose (SwitchBackQ backward) -----------------------------------
// Every column of w [rows, cols] has its own absmax; the codes leave transposed, q_t [cols, rows], with
// state [cols].  Pass 1: the rows are cut into gridDim.y runs, and each block keeps, per 8-column chunk, packed
// 16-bit maxima over its run (no atomics, deterministic).  Pass 2: a 128x128 tile; its 128 column scales are
// finished from the partial maxima first, then the tile is quantized element by element with its column's scale
// and written out through the same LDS transpose as the tensor-wise kernel.
__global__ __launch_bounds__(256) void col_absmax_partial_kernel(const v4u *__restrict__ w, int rows, int chunks,
                                                                 v4u *__restrict__ partials) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= chunks) return;
    const int per = (rows + gridDim.y - 1) / gridDim.y;
    const int r0 = blockIdx.y * per, r1 = min(rows, r0 + per);
    v4u m = {0u, 0u, 0u, 0u};
    for (int r = r0; r < r1; ++r) {
        const v4u v = w[(int64_t)r * chunks + c];
        m.x = pk_absmax_u16(m.x, v.x);
        m.y = pk_absmax_u16(m.y, v.y);
        m.z = pk_absmax_u16(m.z, v.z);
        m.w = pk_absmax_u16(m.w, v.w);
    }
    partials[(int64_t)blockIdx.y * chunks + c] = m;
}

__global__ __launch_bounds__(256) void quantize_colwise_transpose_kernel(const v4u *__restrict__ w, int rows, int cols,
                                                                         int8_t *__restrict__ q_t,
                                                                         float *__restrict__ state,
                                                                         const unsigned short *__restrict__ partials,
                                                                         int nparts) {
    __shared__ float tcol[kTile];
    __shared__ unsigned int tile[kTileDwords];
    const int r0 = blockIdx.y * kTile, c0 = blockIdx.x * kTile;
    if (threadIdx.x < kTile) {
        const int c = c0 + threadIdx.x;
        float t = 0.0f;
        if (c < cols) {
            unsigned int m = 0;  // partials: [run][column] 16-bit patterns (the packed chunks, read back per column)
            for (int i = 0; i < nparts; ++i) m = max(m, (unsigned int)partials[(int64_t)i * cols + c]);
            float s;
            t = scale_from_absmax_bits(m, &s);
            if (blockIdx.y == 0) state[c] = s;
        }
        tcol[threadIdx.x] = t;
    }
    __syncthreads();
    const int chunks_per_row = cols >> 3;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int id = threadIdx.x + 256 * i;
        const int lr = id >> 4, lc = (id & 15) << 3;  // local row, local first column of the 8-element chunk
        const int r = r0 + lr, c = c0 + lc;
        if (r < rows && c < cols) {
            const v4u v = w[(int64_t)r * chunks_per_row + (c >> 3)];
            const unsigned int d[4] = {v.x, v.y, v.z, v.w};
            unsigned int code[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                code[2 * j] = code_bits(__uint_as_float(d[j] << 16), tcol[lc + 2 * j]) & 0xffu;
                code[2 * j + 1] = code_bits(__uint_as_float(d[j] & 0xffff0000u), tcol[lc + 2 * j + 1]) & 0xffu;
            }
            tile[tile_dword(lr, lc >> 2)] = code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);
            tile[tile_dword(lr, (lc >> 2) + 1)] = code[4] | (code[5] << 8) | (code[6] << 16) | (code[7] << 24);
        }
    }
    __syncthreads();
    store_tile_transposed(tile, q_t, rows, cols, r0, c0);
}

// Row-wise dequantization of the memory-efficient variant (SwitchBackM, the appendix algorithm that saves only the
// int8 codes of X): x^[i,j] = bf16(fl((float)q[i,j] * fl(state[i] / 127))), the row-wise quantization equation read
// backwards.  One wavefront per row, 8 codes (8 bytes in, 16 bytes out) per lane and step.
__global__ __launch_bounds__(256) void dequantize_rowwise_kernel(const v2u *__restrict__ q, const float *__restrict__ state,
                                                                 int64_t rows, int chunks, v4u *__restrict__ x_hat) {
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int lane = threadIdx.x & 63;
    const float step = state[row] / 127.0f;  // correctly rounded divide
    const v2u *qr = q + row * chunks;
    v4u *xr = x_hat + row * chunks;
    for (int c = lane; c < chunks; c += 64) {
        const v2u w = __builtin_nontemporal_load(qr + c);
        v4f lo, hi;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            lo[e] = (float)(int)(signed char)(w.x >> (8 * e)) * step;
            hi[e] = (float)(int)(signed char)(w.y >> (8 * e)) * step;
        }
        const v4bf a = __builtin_convertvector(lo, v4bf), b = __builtin_convertvector(hi, v4bf);
        const v2u pa = __builtin_bit_cast(v2u, a), pb = __builtin_bit_cast(v2u, b);
        xr[c] = v4u{pa.x, pa.y, pb.x, pb.y};
    }
}

}  // namespace

hipError_t launch_dequantize_rowwise(const int8_t *q, const float *state, int64_t rows, int64_t cols, void *x_hat,
                                     hipStream_t stream) {
    if (rows == 0) return hipSuccess;
    dequantize_rowwise_kernel<<<(unsigned int)((rows + 3) / 4), 256, 0, stream>>>(
        reinterpret_cast<const v2u *>(q), state, rows, (int)(cols / 8), static_cast<v4u *>(x_hat));
    return hipGetLastError();
}

int colwise_row_runs(int64_t rows) {
    const int64_t r = (rows + 15) / 16;
    return (int)(r < 1 ? 1 : (r > kColwiseRuns ? kColwiseRuns : r));
}

size_t quantize_colwise_workspace_bytes(int64_t rows, int64_t cols) {
    return (size_t)colwise_row_runs(rows) * (size_t)cols * sizeof(unsigned short);
}

hipError_t launch_quantize_colwise_transpose(const void *w, int64_t rows, int64_t cols, int8_t *q_t, float *state,
                                             void *partials, hipStream_t stream) {
    const int chunks = (int)(cols / 8), runs = colwise_row_runs(rows);
    const v4u *wp = static_cast<const v4u *>(w);
    col_absmax_partial_kernel<<<dim3((unsigned int)((chunks + 255) / 256), (unsigned int)runs), 256, 0, stream>>>(
        wp, (int)rows, chunks, static_cast<v4u *>(partials));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 grid((unsigned int)((cols + kTile - 1) / kTile), (unsigned int)((rows + kTile - 1) / kTile));
    quantize_colwise_transpose_kernel<<<grid, 256, 0, stream>>>(wp, (int)rows, (int)cols, q_t, state,
                                                                static_cast<const unsigned short *>(partials), runs);
    return hipGetLastError();
}

// Workgroups of the tensor-wise quantizer's first pass for a matrix of this many 8-element chunks.
int tensorwise_partial_blocks(int64_t nchunks) {
    int nblocks = (int)((nchunks + 256 * 4 - 1) / (256 * 4));
    if (nblocks > kTensorwisePartials) nblocks = kTensorwisePartials;
    return nblocks < 1 ? 1 : nblocks;
}

template <int CODE>
hipError_t launch_quantize_rowwise_t(const void *x, int64_t rows, int64_t cols, void *q, float *state,
                                     hipStream_t stream, TensorAbsmaxJob job = TensorAbsmaxJob{nullptr, 0, nullptr, 0, 0}) {
    const int chunks = (int)(cols / 8);
    const v4u *xp = static_cast<const v4u *>(x);
    v2u *qp = static_cast<v2u *>(q);
    unsigned int wave_grid = (unsigned int)((rows + 3) / 4), block_grid = (unsigned int)rows;
    // The rider's workgroups follow the rows' in the grid.
    job.first_block = (int)(chunks <= 256 ? wave_grid : block_grid);
    wave_grid += (unsigned int)job.nblocks;
    block_grid += (unsigned int)job.nblocks;
#define SB_WAVE(N)                                                                                          \
    quantize_rowwise_wave_kernel<N, CODE><<<wave_grid, 256, 0, stream>>>(xp, rows, chunks, qp, state, job)
#define SB_BLOCK(N) quantize_rowwise_block_kernel<N, CODE><<<block_grid, 256, 0, stream>>>(xp, chunks, qp, state, job)
    if (chunks <= 64) SB_WAVE(1);
    else if (chunks <= 128) SB_WAVE(2);
    else if (chunks <= 192) SB_WAVE(3);
    else if (chunks <= 256) SB_WAVE(4);
    else if (chunks <= 512) SB_BLOCK(2);
    else if (chunks <= 768) SB_BLOCK(3);
    else if (chunks <= 1024) SB_BLOCK(4);
    else if (chunks <= 1536) SB_BLOCK(6);
    else if (chunks <= 2048) SB_BLOCK(8);
    else quantize_rowwise_wide_kernel<CODE><<<block_grid, 256, 0, stream>>>(xp, chunks, qp, state, job);
#undef SB_WAVE
#undef SB_BLOCK
    return hipGetLastError();
}

hipError_t launch_quantize_rowwise(const void *x, int64_t rows, int64_t cols, int8_t *q, float *state,
                                   hipStream_t stream) {
    if (rows == 0) return hipSuccess;
    return launch_quantize_rowwise_t<CODE_INT8>(x, rows, cols, q, state, stream);
}

hipError_t launch_quantize_rowwise_f8(const void *x, int64_t rows, int64_t cols, int fmt, uint8_t *codes, float *state,
                                      hipStream_t stream) {
    if (rows == 0) return hipSuccess;
    return fmt == 0 ? launch_quantize_rowwise_t<CODE_E4M3>(x, rows, cols, codes, state, stream)
                    : launch_quantize_rowwise_t<CODE_E5M2>(x, rows, cols, codes, state, stream);
}

template <int CODE>
hipError_t launch_quantize_tensorwise_t(const void *w, int64_t rows, int64_t cols, int8_t *q, int8_t *q_t,
                                        float *state, unsigned int *partials, hipStream_t stream) {
    const int64_t nchunks = rows * cols / 8;
    const v4u *wp = static_cast<const v4u *>(w);
    const int nblocks = tensorwise_partial_blocks(nchunks);
    absmax_partial_kernel<<<nblocks, 256, 0, stream>>>(wp, nchunks, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (rows == 0 || cols == 0) return hipSuccess;
    dim3 grid((unsigned int)((cols + kTile - 1) / kTile), (unsigned int)((rows + kTile - 1) / kTile));
    quantize_tensorwise_kernel<CODE><<<grid, 256, 0, stream>>>(wp, (int)rows, (int)cols, q, q_t, state, partials,
                                                               nblocks);
    return hipGetLastError();
}

// The two quantizers of a forward pass in two launches instead of three: X row-wise with the first pass of W's
// tensor-wise quantizer riding on the same launch, then W's second pass.  Same results as the separate calls, bit for
// bit (the partial maxima are formed by the same workgroup bodies over the same chunks).  CODE_X / CODE_W as above.
template <int CODE_X, int CODE_W>
hipError_t launch_quantize_forward_operands_t(const void *x, int64_t b, int64_t n, void *xq, float *state_x,
                                              const void *w, int64_t m, int8_t *wq, int8_t *wq_t, float *state_w,
                                              unsigned int *partials, hipStream_t stream) {
    if (b == 0) return launch_quantize_tensorwise_t<CODE_W>(w, m, n, wq, wq_t, state_w, partials, stream);
    const int64_t nchunks = m * n / 8;
    const v4u *wp = static_cast<const v4u *>(w);
    TensorAbsmaxJob job{wp, nchunks, partials, tensorwise_partial_blocks(nchunks), 0};
    hipError_t e = launch_quantize_rowwise_t<CODE_X>(x, b, n, xq, state_x, stream, job);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned int)((n + kTile - 1) / kTile), (unsigned int)((m + kTile - 1) / kTile));
    quantize_tensorwise_kernel<CODE_W><<<grid, 256, 0, stream>>>(wp, (int)m, (int)n, wq, wq_t, state_w, partials,
                                                                 job.nblocks);
    return hipGetLastError();
}

hipError_t launch_quantize_tensorwise(const void *w, int64_t rows, int64_t cols, int8_t *q, int8_t *q_t,
                                      float *state, unsigned int *partials, hipStream_t stream) {
    return launch_quantize_tensorwise_t<CODE_INT8>(w, rows, cols, q, q_t, state, partials, stream);
}

hipError_t launch_quantize_forward_operands(const void *x, int64_t b, int64_t n, int8_t *xq, float *state_x,
                                            const void *w, int64_t m, int8_t *wq, int8_t *wq_t, float *state_w,
                                            unsigned int *partials, hipStream_t stream) {
    return launch_quantize_forward_operands_t<CODE_INT8, CODE_INT8>(x, b, n, xq, state_x, w, m, wq, wq_t, state_w,
                                                                    partials, stream);
}

hipError_t launch_quantize_forward_operands_f8(const void *x, int64_t b, int64_t n, int fmt_x, uint8_t *xq,
                                               float *state_x, const void *w, int64_t m, int fmt_w, uint8_t *wq,
                                               uint8_t *wq_t, float *state_w, unsigned int *partials,
                                               hipStream_t stream) {
    int8_t *q = reinterpret_cast<int8_t *>(wq), *q_t = reinterpret_cast<int8_t *>(wq_t);
#define SB_F8(FX, FW) \
    launch_quantize_forward_operands_t<FX, FW>(x, b, n, xq, state_x, w, m, q, q_t, state_w, partials, stream)
    if (fmt_x == 0) return fmt_w == 0 ? SB_F8(CODE_E4M3, CODE_E4M3) : SB_F8(CODE_E4M3, CODE_E5M2);
    return fmt_w == 0 ? SB_F8(CODE_E5M2, CODE_E4M3) : SB_F8(CODE_E5M2, CODE_E5M2);
#undef SB_F8
}

hipError_t launch_quantize_tensorwise_f8(const void *w, int64_t rows, int64_t cols, int fmt, uint8_t *codes,
                                         uint8_t *codes_t, float *state, unsigned int *partials, hipStream_t stream) {
    int8_t *q = reinterpret_cast<int8_t *>(codes), *q_t = reinterpret_cast<int8_t *>(codes_t);
    return fmt == 0 ? launch_quantize_tensorwise_t<CODE_E4M3>(w, rows, cols, q, q_t, state, partials, stream)
                    : launch_quantize_tensorwise_t<CODE_E5M2>(w, rows, cols, q, q_t, state, partials, stream);
}

}  // namespace sb
