// Per-worker stochastic gradient of the linear least-squares model: for worker i with mini-batch
// A [B][d], y [B] and parameters x^{(i)}:  r = A x - y,  loss = (1/B) sum_s 0.5 r_s^2,
// g = (1/B) A^T r  (the g_i(x; xi) of Section 2, arXiv 2002.09539, for this model).
// The problem is tiny (B x d = 32 x 1024 per worker) and latency-bound; plain vector ALU code.
#include "ols_internal.h"

namespace ols {

constexpr int kThreads = 256;

// one workgroup per (sample s, worker i): r[i][s] = A[i][s][:] . x[i][:] - y[i][s]
__global__ __launch_bounds__(kThreads) void lsq_resid_kernel(const float* __restrict__ A, int64_t a_stride,
                                                             const float* __restrict__ y, int64_t y_stride,
                                                             const float* __restrict__ x, int64_t ld,
                                                             float* __restrict__ resid, float* __restrict__ loss_parts,
                                                             int B, int64_t d) {
    const int s = blockIdx.x, i = blockIdx.y;
    const float* row = A + (int64_t)i * a_stride + (int64_t)s * d;
    const float* xi = x + (int64_t)i * ld;
    float acc = 0.0f;
    for (int64_t j = threadIdx.x; j < d; j += kThreads) acc = __fmaf_rn(row[j], xi[j], acc);
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    __shared__ float part[kThreads / 64];
    if (threadIdx.x % 64 == 0) part[threadIdx.x / 64] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float r = 0.0f;
        for (int w = 0; w < kThreads / 64; ++w) r += part[w];
        r -= y[(int64_t)i * y_stride + s];
        resid[(int64_t)i * B + s] = r;
        loss_parts[(int64_t)i * B + s] = 0.5f * r * r;
    }
}

// one lane per parameter j of worker i: g[i][j] = (1/B) sum_s A[i][s][j] r[i][s]
__global__ __launch_bounds__(kThreads) void lsq_grad_kernel(const float* __restrict__ A, int64_t a_stride,
                                                            const float* __restrict__ resid, float* __restrict__ g,
                                                            int64_t ld, int B, int64_t d) {
    extern __shared__ float r_lds[];
    const int i = blockIdx.y;
    for (int s = threadIdx.x; s < B; s += kThreads) r_lds[s] = resid[(int64_t)i * B + s];
    __syncthreads();
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (j >= d) return;
    const float* col = A + (int64_t)i * a_stride + j;
    float acc = 0.0f;
    for (int s = 0; s < B; ++s) acc = __fmaf_rn(col[(int64_t)s * d], r_lds[s], acc);
    g[(int64_t)i * ld + j] = acc / (float)B;
}

// Small problems in ONE launch: residuals, loss, gradient and the local step (+ pull-back) of a worker by one
// workgroup of 1024 threads.  The three separate kernels of this model (residual, gradient, step) each cost a
// launch and a round trip for a few kFLOP of work; here a local step is one launch.  Launches this small pay for
// every instruction they fetch, so the code is two short rolled loops rather than an unrolled register tile:
// first each wavefront forms the residuals of its samples (lanes stride over the columns, one shuffle reduction
// per sample), then each thread forms the gradient entries of its columns (the mini-batch is read a second
// time, from cache) and applies the update whose operands it requested at the start.
constexpr int kStepThreads = 1024, kStepMaxB = 64, kStepMaxCols = 4;

__global__ __launch_bounds__(kStepThreads) void lsq_step_kernel(const float* __restrict__ A, int64_t a_stride,
                                                                const float* __restrict__ y, int64_t y_stride,
                                                                float* __restrict__ loss_parts, int B, int d,
                                                                FusedUpdate u) {
    constexpr int kWaves = kStepThreads / 64;
    __shared__ float s_r[kStepMaxB];
    const int i = blockIdx.x, t = threadIdx.x;
    const int wave = t / 64, lane = t % 64;
    const bool mom = u.mu != 0.0f;
    const float* Ai = A + (int64_t)i * a_stride;
    const float* xi = u.x_in + (int64_t)i * u.ld;
    float xv[kStepMaxCols], bv[kStepMaxCols], zv[kStepMaxCols];
#pragma unroll
    for (int c = 0; c < kStepMaxCols; ++c) {
        const int j = t + c * kStepThreads;
        const bool ok = j < d;
        xv[c] = ok ? xi[j] : 0.0f;
        bv[c] = (ok && mom) ? u.buf[(int64_t)i * u.ld + j] : 0.0f;
        zv[c] = (ok && u.pull) ? u.z[j] : 0.0f;
    }
    for (int s = wave; s < B; s += kWaves) {
        const float* row = Ai + (int64_t)s * d;
        float acc = 0.0f;
#pragma unroll 4
        for (int j = lane; j < d; j += 64) acc = __fmaf_rn(row[j], xi[j], acc);
        for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (lane == 0) {
            const float r = acc - y[(int64_t)i * y_stride + s];
            s_r[s] = r;
            loss_parts[(int64_t)i * B + s] = 0.5f * r * r;
        }
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kStepMaxCols; ++c) {
        const int j = t + c * kStepThreads;
        if (j >= d) break;
        const float* col = Ai + j;
        float g = 0.0f;
#pragma unroll 8
        for (int s = 0; s < B; ++s) g = __fmaf_rn(col[(int64_t)s * d], s_r[s], g);
        fused_update_store(u, (int64_t)i * u.ld + j, g / (float)B, xv[c], bv[c], zv[c]);
    }
}

bool lsq_step_fits(int B, int64_t d) { return B >= 1 && B <= kStepMaxB && d >= 1 && d <= kStepMaxCols * kStepThreads; }

hipError_t launch_lsq_step(const float* A, int64_t a_stride, const float* y, int64_t y_stride, float* loss_parts, int m,
                           int B, int64_t d, const FusedUpdate& u, hipStream_t s) {
    if (!A || !y || !loss_parts || m < 1 || !lsq_step_fits(B, d) || !u.enabled || !u.x_in || !u.x_out || u.ld < d ||
        (u.mu != 0.0f && !u.buf) || (u.pull && !u.z) || u.shadow)
        return hipErrorInvalidValue;
    lsq_step_kernel<<<(unsigned)m, kStepThreads, 0, s>>>(A, a_stride, y, y_stride, loss_parts, B, (int)d, u);
    return hipGetLastError();
}

hipError_t launch_lsq_resid(const float* A, int64_t a_stride, const float* y, int64_t y_stride, const float* x,
                            int64_t ld, float* resid, float* loss_parts, int m, int B, int64_t d, hipStream_t s) {
    if (!A || !y || !x || !resid || !loss_parts || m < 1 || m > 65535 || B < 1 || d < 1 || ld < d)
        return hipErrorInvalidValue;
    lsq_resid_kernel<<<dim3((unsigned)B, (unsigned)m), kThreads, 0, s>>>(A, a_stride, y, y_stride, x, ld, resid,
                                                                        loss_parts, B, d);
    return hipGetLastError();
}

hipError_t launch_lsq_grad(const float* A, int64_t a_stride, const float* resid, float* g, int64_t ld, int m, int B,
                           int64_t d, hipStream_t s) {
    if (!A || !resid || !g || m < 1 || m > 65535 || B < 1 || B > 8192 || d < 1 || ld < d) return hipErrorInvalidValue;
    dim3 grid((unsigned)((d + kThreads - 1) / kThreads), (unsigned)m);
    lsq_grad_kernel<<<grid, kThreads, (size_t)B * sizeof(float), s>>>(A, a_stride, resid, g, ld, B, d);
    return hipGetLastError();
}

}  // namespace ols
