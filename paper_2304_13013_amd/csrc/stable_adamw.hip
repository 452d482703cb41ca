// StableAdamW step for one tensor (arxiv 2304.13013, the optimizer algorithm of the section on loss spikes: AdamW whose
// debiasing is folded into the decay rates and whose learning rate is divided by max(1, RMS_t), with
// RMS_t^2 = mean(g^2 / max(u_t, eps^2)) over the tensor, per the implementation note of the appendix).
//
// The RMS over the whole tensor must be known before any parameter moves, so the step is two HBM-bound passes:
//   moments: v <- b1 v + (1-b1) g, u <- b2 u + (1-b2) g^2 in place, and one binary64 partial sum of g^2 / max(u, eps^2)
//            per workgroup (fixed grid for a given count, fixed order inside a workgroup: the result is deterministic);
//   update:  every workgroup adds the partial sums in the same order, forms eta = alpha / max(1, RMS_t) and applies
//            theta <- theta - eta lambda theta - eta v / (sqrt(u) + eps).
// Algorithmic bytes per element: g (2 or 4) + v, u read and written (16) + theta, v, u read (12) + theta written (4).
// All arithmetic is binary32 except the sum, which is binary64 so that its order does not matter at the tolerance of
// the parity tests.  Each lane handles four consecutive elements per step (16-byte accesses of the binary32 arrays);
// the count % 4 trailing elements are handled by the first lanes of workgroup 0.
#include "sb_common.h"

namespace sb {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
    return x;
}

// Sum over the workgroup, returned to every lane.  red: 5 doubles of LDS.
__device__ __forceinline__ double block_sum(double x, double *red) {
    x = wave_sum(x);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[wave] = x;
    __syncthreads();
    if (threadIdx.x == 0) red[4] = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    return red[4];
}

template <bool G_BF16>
__device__ __forceinline__ float grad_at(const void *g, int64_t j) {
    if (G_BF16) return bf16_bits_to_float(static_cast<const unsigned short *>(g)[j]);
    return static_cast<const float *>(g)[j];
}

__device__ __forceinline__ float moments_one(float g, float &v, float &u, float b1, float omb1, float b2, float omb2,
                                             float eps2) {
    v = b1 * v + omb1 * g;
    u = b2 * u + omb2 * (g * g);
    return (g * g) / fmaxf(u, eps2);
}

// Workgroup `block` of the `nblocks` that share one tensor.
template <bool G_BF16>
__device__ __forceinline__ void adamw_moments_body(const void *__restrict__ g, float *__restrict__ v,
                                                   float *__restrict__ u, int64_t count, float b1, float omb1, float b2,
                                                   float omb2, float eps2, double *__restrict__ partial, int block,
                                                   int nblocks, double *red) {
    const int64_t quads = count >> 2;
    const int64_t stride = (int64_t)nblocks * kThreads;
    double acc = 0.0;
    for (int64_t i = (int64_t)block * kThreads + threadIdx.x; i < quads; i += stride) {
        v4f vv = reinterpret_cast<const v4f *>(v)[i];
        v4f uu = reinterpret_cast<const v4f *>(u)[i];
        v4f gg;
        if (G_BF16) {
            const v2u raw = reinterpret_cast<const v2u *>(g)[i];
            gg[0] = __uint_as_float(raw[0] << 16);
            gg[1] = __uint_as_float(raw[0] & 0xffff0000u);
            gg[2] = __uint_as_float(raw[1] << 16);
            gg[3] = __uint_as_float(raw[1] & 0xffff0000u);
        } else {
            gg = reinterpret_cast<const v4f *>(g)[i];
        }
        float r[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float ve = vv[e], ue = uu[e];
            r[e] = moments_one(gg[e], ve, ue, b1, omb1, b2, omb2, eps2);
            vv[e] = ve;
            uu[e] = ue;
        }
        reinterpret_cast<v4f *>(v)[i] = vv;
        reinterpret_cast<v4f *>(u)[i] = uu;
        acc += ((double)r[0] + (double)r[1]) + ((double)r[2] + (double)r[3]);
    }
    if (block == 0 && threadIdx.x < (count & 3)) {
        const int64_t j = (quads << 2) + threadIdx.x;
        float ve = v[j], ue = u[j];
        acc += (double)moments_one(grad_at<G_BF16>(g, j), ve, ue, b1, omb1, b2, omb2, eps2);
        v[j] = ve;
        u[j] = ue;
    }
    const double total = block_sum(acc, red);
    if (threadIdx.x == 0) partial[0] = total;
}

template <bool G_BF16>
__global__ __launch_bounds__(kThreads) void adamw_moments_kernel(const void *__restrict__ g, float *__restrict__ v,
                                                                 float *__restrict__ u, int64_t count, float b1,
                                                                 float omb1, float b2, float omb2, float eps2,
                                                                 double *__restrict__ partials) {
    __shared__ double red[5];
    adamw_moments_body<G_BF16>(g, v, u, count, b1, omb1, b2, omb2, eps2, partials + blockIdx.x, blockIdx.x, gridDim.x,
                               red);
}

// The tensor that workgroup `block` of a batched launch belongs to: the table is sorted by first_block.
__device__ __forceinline__ int adamw_tensor_of(const sb_adamw_tensor *__restrict__ table, int n, int block) {
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (table[mid].first_block <= block) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

template <bool G_BF16>
__global__ __launch_bounds__(kThreads) void adamw_moments_multi_kernel(const sb_adamw_tensor *__restrict__ table, int n,
                                                                       float b1, float omb1, float b2, float omb2,
                                                                       float eps2, double *__restrict__ partials) {
    __shared__ double red[5];
    const sb_adamw_tensor t = table[adamw_tensor_of(table, n, blockIdx.x)];
    adamw_moments_body<G_BF16>(t.grad, t.v, t.u, t.count, b1, omb1, b2, omb2, eps2, partials + blockIdx.x,
                               (int)blockIdx.x - t.first_block, t.num_blocks, red);
}

__device__ __forceinline__ float update_one(float th, float v, float u, float eta, float eta_lambda, float eps) {
    return th - eta_lambda * th - eta * (v / (sqrtf(u) + eps));
}

__device__ __forceinline__ void adamw_update_body(float *__restrict__ theta, const float *__restrict__ v,
                                                  const float *__restrict__ u, int64_t count, float alpha, float lambda,
                                                  float eps, const double *__restrict__ partials, int nparts,
                                                  float *__restrict__ rms_out, int block, double *red) {
    double s = 0.0;
    for (int i = threadIdx.x; i < nparts; i += kThreads) s += partials[i];
    const double sum = block_sum(s, red);
    const float rms = (float)sqrt(sum / (double)count);
    const float eta = alpha / fmaxf(1.0f, rms);
    const float eta_lambda = eta * lambda;
    if (rms_out != nullptr && block == 0 && threadIdx.x == 0) rms_out[0] = rms;

    const int64_t quads = count >> 2;
    const int64_t stride = (int64_t)nparts * kThreads;  // one partial sum per workgroup of the tensor
    for (int64_t i = (int64_t)block * kThreads + threadIdx.x; i < quads; i += stride) {
        v4f th = reinterpret_cast<const v4f *>(theta)[i];
        const v4f vv = reinterpret_cast<const v4f *>(v)[i];
        const v4f uu = reinterpret_cast<const v4f *>(u)[i];
#pragma unroll
        for (int e = 0; e < 4; ++e) th[e] = update_one(th[e], vv[e], uu[e], eta, eta_lambda, eps);
        reinterpret_cast<v4f *>(theta)[i] = th;
    }
    if (block == 0 && threadIdx.x < (count & 3)) {
        const int64_t j = (quads << 2) + threadIdx.x;
        theta[j] = update_one(theta[j], v[j], u[j], eta, eta_lambda, eps);
    }
}

__global__ __launch_bounds__(kThreads) void adamw_update_kernel(float *__restrict__ theta, const float *__restrict__ v,
                                                                const float *__restrict__ u, int64_t count,
                                                                float alpha, float lambda, float eps,
                                                                const double *__restrict__ partials, int nparts,
                                                                float *__restrict__ rms_out) {
    __shared__ double red[5];
    adamw_update_body(theta, v, u, count, alpha, lambda, eps, partials, nparts, rms_out, blockIdx.x, red);
}

__global__ __launch_bounds__(kThreads) void adamw_update_multi_kernel(const sb_adamw_tensor *__restrict__ table, int n,
                                                                      float alpha, float lambda, float eps,
                                                                      const double *__restrict__ partials,
                                                                      float *__restrict__ rms_out) {
    __shared__ double red[5];
    const int ti = adamw_tensor_of(table, n, blockIdx.x);
    const sb_adamw_tensor t = table[ti];
    adamw_update_body(t.theta, t.v, t.u, t.count, alpha, lambda, eps, partials + t.first_block, t.num_blocks,
                      rms_out ? rms_out + ti : nullptr, (int)blockIdx.x - t.first_block, red);
}

int adamw_grid(int64_t count) {
    const int64_t per_block = (int64_t)kThreads * 4 * 4;  // four quads per lane before the grid stride matters
    int64_t blocks = (count + per_block - 1) / per_block;
    if (blocks < 1) blocks = 1;
    if (blocks > kAdamwPartials) blocks = kAdamwPartials;
    return (int)blocks;
}

}  // namespace

size_t stable_adamw_workspace_bytes() { return (size_t)kAdamwPartials * sizeof(double); }

int stable_adamw_blocks(int64_t count) { return adamw_grid(count); }

hipError_t launch_stable_adamw_step_multi(const sb_adamw_tensor *table, int n, int total_blocks, bool grad_bf16,
                                          float alpha, float b1_hat, float b2_hat, float omb1, float omb2, float eps,
                                          float lambda, float *rms_out, void *ws, hipStream_t stream) {
    double *partials = static_cast<double *>(ws);
    const float eps2 = eps * eps;
    if (grad_bf16)
        hipLaunchKernelGGL(adamw_moments_multi_kernel<true>, dim3(total_blocks), dim3(kThreads), 0, stream, table, n,
                           b1_hat, omb1, b2_hat, omb2, eps2, partials);
    else
        hipLaunchKernelGGL(adamw_moments_multi_kernel<false>, dim3(total_blocks), dim3(kThreads), 0, stream, table, n,
                           b1_hat, omb1, b2_hat, omb2, eps2, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(adamw_update_multi_kernel, dim3(total_blocks), dim3(kThreads), 0, stream, table, n, alpha, lambda,
                       eps, partials, rms_out);
    return hipGetLastError();
}

hipError_t launch_stable_adamw_step(float *theta, float *v, float *u, const void *grad, bool grad_bf16, int64_t count,
                                    float alpha, float b1_hat, float b2_hat, float omb1, float omb2, float eps,
                                    float lambda, float *rms_out, void *ws, hipStream_t stream) {
    const int grid = adamw_grid(count);
    double *partials = static_cast<double *>(ws);
    const float eps2 = eps * eps;
    if (grad_bf16)
        hipLaunchKernelGGL(adamw_moments_kernel<true>, dim3(grid), dim3(kThreads), 0, stream, grad, v, u, count, b1_hat,
                           omb1, b2_hat, omb2, eps2, partials);
    else
        hipLaunchKernelGGL(adamw_moments_kernel<false>, dim3(grid), dim3(kThreads), 0, stream, grad, v, u, count,
                           b1_hat, omb1, b2_hat, omb2, eps2, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(adamw_update_kernel, dim3(grid), dim3(kThreads), 0, stream, theta, v, u, count, alpha, lambda,
                       eps, partials, grid, rms_out);
    return hipGetLastError();
}

}  // namespace sb
