/*
 * CPU oracle for the SwitchBack int8 linear layer (arxiv 2304.13013, Section 2.2.1, Algorithm 1).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously-correct statement of
 * what the layer computes, written from the paper, and it shares no code with the GPU library.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * All matrices are dense row-major.  bf16 values travel as their 16-bit patterns (uint16_t); widening a
 * bf16 to binary32 is exact (the pattern becomes the high half of the float).  "fl" below means one IEEE
 * binary32 operation, round-to-nearest-even.  The file must be compiled without fast-math and without
 * floating-point contraction so that each "fl" is exactly one rounding.
 *
 * Paper notation: X [b,n] inputs, W [m,n] weights, Y [b,m] outputs, dY [b,m], dX [b,n], dW [m,n]
 * (Section 2.2.1 "Notation").  int8 codes lie in [-127,127] (Section 2.2.1 "Quantization").
 *
 * Readings taken where the paper is silent (each is listed in the design notes as well):
 *   - round() is round-half-to-even;
 *   - the scale is formed first, t = fl(127/absmax), then each element is fl(x*t)   (literal order of
 *     the row-wise and tensor-wise quantization equations);
 *   - an all-zero row (or tensor), or an absmax so small that 127/absmax overflows binary32, quantizes
 *     to all zeros and stores state 0;
 *   - the state is the absmax itself, kept in binary32;
 *   - dequantization order: c = fl(state_W/127^2) once, r_i = fl(state_row[i]*c) per row,
 *     y = fl((float)acc * r_i) per element                      (the forward equation with dequantization);
 *   - Algorithm 1's backward dequantizes with the state of the quantized dY (its listing reuses the
 *     forward's name for it);
 *   - the memory-efficient variant (SwitchBackM, the appendix algorithm that keeps only the int8 codes of X)
 *     names a row-wise dequantization without printing it: taken as the inverse of the row-wise quantization
 *     equation, x^_ij = fl(q_ij * fl(state_i / 127)), then rounded to bf16 (the layer's 16-bit type);
 *   - the variant with row-wise and column-wise weight quantization (SwitchBackQ) gives its forward pass as
 *     1/127^2 * state_row(X) state_row(W)^T * (int8 matmul) without an order of evaluation: taken as the order of
 *     the tensor-wise case with the weight state now per output column, c_j = fl(state_W[j]/127^2) once per
 *     column, then fl(state_row[i] * c_j), then fl((float)acc * that) per element.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- small scalar helpers -------------------------------------------------------------------------- */

static float bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* binary32 -> bf16, round-to-nearest-even on the 16 dropped bits.  NaN is out of contract (kept quiet). */
static uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* The per-row / per-tensor scale: t = fl(127/s), with the zero and overflow cases mapped to (t=0, s=0). */
static float scale_from_absmax(float s, float *stored_state) {
    float t = 127.0f / s;
    if (s == 0.0f || !isfinite(t)) {
        *stored_state = 0.0f;
        return 0.0f;
    }
    *stored_state = s;
    return t;
}

static int8_t quantize_one(float x, float t) {
    float p = x * t;        /* fl(x * t) */
    float r = rintf(p);     /* round-half-to-even under the default rounding mode */
    if (r > 127.0f) r = 127.0f;
    if (r < -127.0f) r = -127.0f;
    return (int8_t)r;
}

/* ---- quantization (row-wise and tensor-wise quantization equations) ----------------------------------- */

/* Q_row and state_row: one absmax per row. x [rows,cols] bf16 -> q [rows,cols] int8, state [rows] f32. */
void sbo_quantize_rowwise(const uint16_t *x, int64_t rows, int64_t cols, int8_t *q, float *state) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        const uint16_t *xi = x + i * cols;
        float s = 0.0f;
        for (int64_t j = 0; j < cols; ++j) {
            float a = fabsf(bf16_to_f32(xi[j]));
            if (a > s) s = a;
        }
        float t = scale_from_absmax(s, &state[i]);
        for (int64_t j = 0; j < cols; ++j) q[i * cols + j] = quantize_one(bf16_to_f32(xi[j]), t);
    }
}

/* Q_tensor and state_tensor: one absmax for the whole matrix.  w [rows,cols] -> q [rows,cols],
 * q_t [cols,rows] (the transposed copy; may be NULL), state[0].  Because the scale is a single scalar,
 * quantizing the transpose equals transposing the quantized matrix, so q_t is just q transposed. */
void sbo_quantize_tensorwise(const uint16_t *w, int64_t rows, int64_t cols, int8_t *q, int8_t *q_t,
                             float *state) {
    float s = 0.0f;
    for (int64_t e = 0; e < rows * cols; ++e) {
        float a = fabsf(bf16_to_f32(w[e]));
        if (a > s) s = a;
    }
    float t = scale_from_absmax(s, &state[0]);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            int8_t v = quantize_one(bf16_to_f32(w[i * cols + j]), t);
            q[i * cols + j] = v;
            if (q_t) q_t[j * rows + i] = v;
        }
}

/* Row-wise dequantization of the memory-efficient variant (SwitchBackM): the inverse of the row-wise quantization
 * equation.  q [rows,cols] int8, state [rows] f32 (the row absmax) -> x_hat [rows,cols] bf16 patterns. */
void sbo_dequantize_rowwise(const int8_t *q, const float *state, int64_t rows, int64_t cols, uint16_t *x_hat) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        float step = state[i] / 127.0f; /* fl(state_i / 127): what one code unit is worth in this row */
        for (int64_t j = 0; j < cols; ++j) {
            float v = (float)q[i * cols + j] * step; /* fl(q * step); (float)q is exact */
            x_hat[i * cols + j] = f32_to_bf16_rne(v);
        }
    }
}

/* ---- integer matmul ("int8 matmul" under-brace of the forward equation) -------------------------------- */

/* acc[i,j] = sum_k a[i,k] * b[j,k]; a [M,K], b [N,K] int8, acc [M,N] int32.  The sum is formed exactly in
 * int64; returns 0 when every sum fits int32 (always so while 127^2*K < 2^31), 1 otherwise. */
int sbo_matmul_int8(const int8_t *a, const int8_t *b, int64_t M, int64_t N, int64_t K, int32_t *acc) {
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int64_t s64 = 0;
            for (int64_t k = 0; k < K; ++k) s64 += (int32_t)a[i * K + k] * (int32_t)b[j * K + k];
            if (s64 > INT32_MAX || s64 < INT32_MIN) overflow = 1;
            acc[i * N + j] = (int32_t)s64;
        }
    return overflow;
}

/* ---- dequantization (forward equation with dequantization) --------------------------------------------- */

/* y32[i,j] = fl((float)acc[i,j] * fl(state_row[i] * fl(state_tensor/16129)));
 * y64[i,j] = acc * state_row[i] * state_tensor / 16129 in binary64 (may be NULL). */
void sbo_dequantize(const int32_t *acc, int64_t M, int64_t N, const float *state_row, float state_tensor,
                    float *y32, double *y64) {
    float c = state_tensor / 16129.0f;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        float r = state_row[i] * c;
        for (int64_t j = 0; j < N; ++j) {
            y32[i * N + j] = (float)acc[i * N + j] * r;
            if (y64)
                y64[i * N + j] =
                    (double)acc[i * N + j] * (double)state_row[i] * (double)state_tensor / 16129.0;
        }
    }
}

/* SwitchBackQ: both operands carry one state per row of their code matrix, so the product has a row state and a
 * column state: y32[i,j] = fl((float)acc[i,j] * fl(state_row[i] * fl(state_col[j]/16129))); y64 in binary64. */
void sbo_dequantize_rowcol(const int32_t *acc, int64_t M, int64_t N, const float *state_row, const float *state_col,
                           float *y32, double *y64) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            float c = state_col[j] / 16129.0f; /* fl(state_col[j] / 127^2) */
            float r = state_row[i] * c;        /* fl(state_row[i] * c) */
            y32[i * N + j] = (float)acc[i * N + j] * r;
            if (y64)
                y64[i * N + j] = (double)acc[i * N + j] * (double)state_row[i] * (double)state_col[j] / 16129.0;
        }
}

/* The linear layer's bias and the layer-scale of the transformer block, applied to a dequantized product (the
 * block equations of the paper's section on feature magnitudes: x' = x + gamma * block(x), where block ends in a
 * linear layer, i.e. gamma_j * (y_ij + bias_j); SwitchBackLinear is an nn.Linear and has a bias, Algorithm 1 leaves
 * it out).  One binary32 rounding per operation, in this order: z = fl(y + bias[j]) if bias is given, then
 * fl(gamma[j] * z) if gamma is given.  y [M,N] f32 in; bias, gamma [N] f32 or NULL; out [M,N] f32;
 * out64 (may be NULL): gamma[j] * (y64[i,j] + bias[j]) in binary64 from the binary64 product y64. */
void sbo_bias_layerscale(const float *y, const double *y64, int64_t M, int64_t N, const float *bias,
                         const float *gamma, float *out, double *out64) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            float z = y[i * N + j];
            if (bias) z = z + bias[j];
            if (gamma) z = gamma[j] * z;
            out[i * N + j] = z;
            if (out64) {
                double w = y64[i * N + j];
                if (bias) w = w + (double)bias[j];
                if (gamma) w = (double)gamma[j] * w;
                out64[i * N + j] = w;
            }
        }
}

void sbo_round_to_bf16(const float *y, int64_t count, uint16_t *out) {
    for (int64_t e = 0; e < count; ++e) out[e] = f32_to_bf16_rne(y[e]);
}

/* ---- weight gradient (Algorithm 1: the 16-bit matmul of dY^T and X) ------------------------------------- */

/* dw64[j,k] = sum_i dy[i,j] * x[i,k] in binary64, i ascending.  dy [b,m], x [b,n] bf16, dw64 [m,n].
 * A bf16 x bf16 product is exact in binary64 (16 significant bits), so only the additions round. */
void sbo_weight_grad(const uint16_t *dy, const uint16_t *x, int64_t b, int64_t n, int64_t m, double *dw64) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < m; ++j) {
        double *row = dw64 + j * n;
        for (int64_t k = 0; k < n; ++k) row[k] = 0.0;
        for (int64_t i = 0; i < b; ++i) {
            double g = (double)bf16_to_f32(dy[i * m + j]);
            const uint16_t *xi = x + i * n;
            for (int64_t k = 0; k < n; ++k) row[k] += g * (double)bf16_to_f32(xi[k]);
        }
    }
}

/* ---- StableAdamW (the optimizer algorithm of the paper: AdamW with the debiasing folded into the decay rates and
 * the learning rate divided by max(1, RMS_t), RMS_t^2 = mean(g^2 / u_t), taken per tensor) -------------------------
 * One step for one tensor, in binary64 throughout; the state arrays are binary32 and are read, updated and written
 * back (each stored value is the binary32 rounding of the binary64 result).  Per the implementation note of the
 * appendix the denominator of the RMS is max(u_t, eps^2).  grad may be given as bf16 patterns (g16) or binary32
 * (g32); exactly one of the two is non-NULL.  Returns RMS_t.
 *   b1 = beta1 * (1 - beta1^(t-1)) / (1 - beta1^t),  b2 likewise
 *   v = b1 v + (1 - b1) g ;  u = b2 u + (1 - b2) g^2
 *   eta = alpha / max(1, RMS_t) ;  theta = theta - eta lambda theta - eta v / (sqrt(u) + eps)            */
double sbo_stable_adamw_step(float *theta, float *v, float *u, const uint16_t *g16, const float *g32, int64_t count,
                             double alpha, double beta1, double beta2, double eps, double lambda, int64_t t) {
    const double b1 = beta1 * (1.0 - pow(beta1, (double)(t - 1))) / (1.0 - pow(beta1, (double)t));
    const double b2 = beta2 * (1.0 - pow(beta2, (double)(t - 1))) / (1.0 - pow(beta2, (double)t));
    double sum = 0.0;
    for (int64_t j = 0; j < count; ++j) { /* sequential: the sum is part of the definition, keep one order */
        const double g = g16 ? (double)bf16_to_f32(g16[j]) : (double)g32[j];
        const double vj = b1 * (double)v[j] + (1.0 - b1) * g;
        const double uj = b2 * (double)u[j] + (1.0 - b2) * g * g;
        v[j] = (float)vj;
        u[j] = (float)uj;
        const double den = uj > eps * eps ? uj : eps * eps;
        sum += g * g / den;
    }
    const double rms = count > 0 ? sqrt(sum / (double)count) : 0.0;
    const double eta = alpha / (rms > 1.0 ? rms : 1.0);
    for (int64_t j = 0; j < count; ++j) {
        const double th = (double)theta[j];
        /* the moments as stored (binary32), which is what a later step would see */
        theta[j] = (float)(th - eta * lambda * th - eta * (double)v[j] / (sqrt((double)u[j]) + eps));
    }
    return rms;
}

/* ---- float8 SwitchBack (the "float8" paragraph of Section 2.2.1: the int8 code path with
 * round(127 x / absmax(x)) replaced by float8cast(x / absmax(x)); the 8-bit float types are those of the format paper it
 * cites: E4M3 = 1 sign, 4 exponent (bias 7), 3 mantissa bits, no infinities, largest finite 448, subnormals m * 2^-9;
 * E5M2 = 1/5/2, bias 15, IEEE-like, largest finite 57344, subnormals m * 2^-16) ---------------------------------------
 * fmt: 0 = E4M3, 1 = E5M2.  Codes travel as bytes, sign in bit 7. */

static void f8_shape(int fmt, int *mbits, int *bias, double *max_finite) {
    if (fmt == 0) { *mbits = 3; *bias = 7; *max_finite = 448.0; }
    else          { *mbits = 2; *bias = 15; *max_finite = 57344.0; }
}

/* float8cast: the representable value nearest to x, ties to the even mantissa; magnitudes beyond the largest finite
 * value saturate to it (cannot happen for |x| <= 1, the only inputs the layer produces).  NaN is out of contract. */
static uint8_t f8_encode(float x, int fmt) {
    int mbits, bias;
    double maxf;
    f8_shape(fmt, &mbits, &bias, &maxf);
    const uint8_t sign = signbit(x) ? 0x80u : 0u;
    double a = fabs((double)x);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                 /* a = f * 2^e, f in [0.5, 1)  ->  a = 1.xxx * 2^(e-1) */
    int E = e - 1;
    const int emin = 1 - bias;          /* exponent of the smallest normal; subnormals share its spacing */
    if (E < emin) E = emin;
    const double step = ldexp(1.0, E - mbits);
    double r = nearbyint(a / step) * step;   /* a/step is exact; nearbyint = round-half-to-even (default mode) */
    if (r > maxf) r = maxf;
    if (r == 0.0) return sign;
    if (r < ldexp(1.0, emin)) return (uint8_t)(sign | (unsigned)(r / ldexp(1.0, emin - mbits)));
    (void)frexp(r, &e);
    E = e - 1;
    const unsigned mant = (unsigned)((r / ldexp(1.0, E) - 1.0) * (double)(1 << mbits));
    return (uint8_t)(sign | ((unsigned)(E + bias) << mbits) | mant);
}

static double f8_decode(uint8_t code, int fmt) {
    int mbits, bias;
    double maxf;
    f8_shape(fmt, &mbits, &bias, &maxf);
    const unsigned mant = code & ((1u << mbits) - 1u), ef = (code & 0x7fu) >> mbits;
    double v = ef == 0 ? ldexp((double)mant, 1 - bias - mbits)
                       : ldexp(1.0 + (double)mant / (double)(1 << mbits), (int)ef - bias);
    return (code & 0x80u) ? -v : v;     /* the NaN / infinity codes are never produced by f8_encode */
}

void sbo_float8_encode(const float *x, int64_t count, int fmt, uint8_t *codes) {
    for (int64_t i = 0; i < count; ++i) codes[i] = f8_encode(x[i], fmt);
}

void sbo_float8_decode(const uint8_t *codes, int64_t count, int fmt, double *out) {
    for (int64_t i = 0; i < count; ++i) out[i] = f8_decode(codes[i], fmt);
}

/* The scale of the float8 path: t = fl(1/s), formed first like the int8 path forms fl(127/s); zero rows and rows
 * whose 1/s overflows binary32 quantize to zeros with state 0. */
static float f8_scale_from_absmax(float s, float *stored_state) {
    float t = 1.0f / s;
    if (s == 0.0f || !isfinite(t)) {
        *stored_state = 0.0f;
        return 0.0f;
    }
    *stored_state = s;
    return t;
}

/* Row-wise: codes[i,j] = float8cast(fl(x[i,j] * fl(1/absmax_i))), state[i] = absmax_i. */
void sbo_quantize_rowwise_f8(const uint16_t *x, int64_t rows, int64_t cols, int fmt, uint8_t *codes, float *state) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        const uint16_t *xi = x + i * cols;
        float s = 0.0f;
        for (int64_t j = 0; j < cols; ++j) {
            float a = fabsf(bf16_to_f32(xi[j]));
            if (a > s) s = a;
        }
        const float t = f8_scale_from_absmax(s, &state[i]);
        for (int64_t j = 0; j < cols; ++j) {
            const float p = bf16_to_f32(xi[j]) * t;
            codes[i * cols + j] = f8_encode(p, fmt);
        }
    }
}

/* Tensor-wise: one absmax for the matrix; codes [rows,cols] and the transposed copy codes_t [cols,rows] (may be NULL). */
void sbo_quantize_tensorwise_f8(const uint16_t *w, int64_t rows, int64_t cols, int fmt, uint8_t *codes,
                                uint8_t *codes_t, float *state) {
    float s = 0.0f;
    for (int64_t e = 0; e < rows * cols; ++e) {
        float a = fabsf(bf16_to_f32(w[e]));
        if (a > s) s = a;
    }
    const float t = f8_scale_from_absmax(s, &state[0]);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            const float p = bf16_to_f32(w[i * cols + j]) * t;
            const uint8_t c = f8_encode(p, fmt);
            codes[i * cols + j] = c;
            if (codes_t) codes_t[j * rows + i] = c;
        }
}

/* acc[i,j] = sum_k value(a[i,k]) * value(b[j,k]), exactly: every product is a multiple of 2^-25 below 2^32 in
 * magnitude for |values| <= 448 x 57344, and for the layer's |values| <= 1 the partial sums stay far inside the
 * 53-bit significand, so the binary64 sum has no rounding and no order.  abs_acc (may be NULL) receives
 * sum_k |a| |b|, the quantity error bounds of a lower-precision summation are stated in. */
void sbo_matmul_f8(const uint8_t *a, int fmt_a, const uint8_t *b, int fmt_b, int64_t M, int64_t N, int64_t K,
                   double *acc, double *abs_acc) {
    double ta[256], tb[256];
    for (int c = 0; c < 256; ++c) {
        ta[c] = f8_decode((uint8_t)c, fmt_a);
        tb[c] = f8_decode((uint8_t)c, fmt_b);
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double sum = 0.0, asum = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const double pr = ta[a[i * K + k]] * tb[b[j * K + k]];
                sum += pr;
                asum += fabs(pr);
            }
            acc[i * N + j] = sum;
            if (abs_acc) abs_acc[i * N + j] = asum;
        }
}

/* Dequantization of the float8 product: the forward equation without the 1/127^2 (the codes already lie in [-1, 1]):
 * r_i = fl(state_row[i] * state_tensor) in binary32 like the int8 path, y = acc * r_i rounded once to binary32 from
 * the exact binary64 product (y64 keeps it unrounded). */
void sbo_dequantize_f8(const double *acc, int64_t M, int64_t N, const float *state_row, float state_tensor, float *y32,
                       double *y64) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        const float r = state_row[i] * state_tensor;
        for (int64_t j = 0; j < N; ++j) {
            const double y = acc[i * N + j] * (double)r;
            if (y64) y64[i * N + j] = y;
            y32[i * N + j] = (float)y;
        }
    }
}

int sbo_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
