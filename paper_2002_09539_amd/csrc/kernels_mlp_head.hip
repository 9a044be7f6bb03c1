// Output layer of the per-worker MLP (class count C <= 32) with softmax cross-entropy and its gradients.  The output width is far too small for matrix cores, so these run
// on the vector ALUs; they are a few MFLOP per worker and latency-bound.
//
// Per worker i with last hidden activations h [B][H], weights W [H][C], bias b [C], labels y [B]
// (the mini-batch loss whose gradient is the g_i of Section 2, arXiv 2002.09539):
//   logits = h W + b;  loss_s = logsumexp(logits_s) - logits_s[y_s];  dlogits = (softmax - onehot) / B
//   dW = h^T dlogits;  db = colsum(dlogits);  dz = (dlogits W^T) * [h > 0]
#include "ols_internal.h"

namespace ols {

constexpr int kThreads = 256;
constexpr int kWave = 64;
constexpr int kMaxC = 32;

__device__ __forceinline__ float bf16_to_f32(uint16_t v) { return __uint_as_float(((unsigned int)v) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    unsigned int u = __float_as_uint(f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
// Sum over the 64 lanes of a wavefront, result valid in every lane: four rotate-and-add steps inside
// each row of 16 lanes on the vector ALU (DPP row_ror), then two cross-row exchanges.
__device__ __forceinline__ float wave_sum(float v) {
#define OLS_ROW_ROR_ADD(n)                                                                                  \
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + (n), 0xF, 0xF, false))
    OLS_ROW_ROR_ADD(8);
    OLS_ROW_ROR_ADD(4);
    OLS_ROW_ROR_ADD(2);
    OLS_ROW_ROR_ADD(1);
#undef OLS_ROW_ROR_ADD
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
    return v;
}

template <bool BF>
__device__ __forceinline__ float load_act(const void* p, int64_t idx) {
    return BF ? bf16_to_f32(((const uint16_t*)p)[idx]) : ((const float*)p)[idx];
}

// Stages `rows` rows of the output-layer weights W [H][C] (contiguous in memory) into LDS with
// fully coalesced loads; row pitch CP = C | 1 is odd so that lanes reading different rows at the same
// column hit different banks.  Loads are issued eight at a time before any of them is consumed: a
// dependent global round trip costs of the order of a microsecond here, so they must overlap.
__device__ __forceinline__ void stage_weights(float* s_w, const float* __restrict__ W, int k0, int rows, int C, int CP) {
    const float* src = W + (int64_t)k0 * C;
    const int total = rows * C;
    for (int base = 0; base < total; base += kThreads * 8) {
        float tmp[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int t = base + u * kThreads + threadIdx.x;
            tmp[u] = t < total ? src[t] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int t = base + u * kThreads + threadIdx.x;
            if (t < total) s_w[(t / C) * CP + (t % C)] = tmp[u];
        }
    }
}

// A workgroup owns 4 * SPW samples of one worker (SPW = 64 / CMAX per wavefront); the weight matrix
// streams through LDS in chunks of kChunk rows shared by all of them.  The softmax of a wavefront's SPW
// samples runs in parallel on lane groups of CMAX lanes.  grid (ceil(B / (4 SPW)), m)
template <bool BF, int CMAX>
__global__ __launch_bounds__(kThreads) void head_fwd_kernel(const void* __restrict__ h, int64_t h_stride,
                                                            const float* __restrict__ x, int64_t ld, int64_t w_off,
                                                            int64_t b_off, const int32_t* __restrict__ labels,
                                                            int64_t label_stride, float* __restrict__ dlogits,
                                                            float* __restrict__ loss_parts, int B, int H, int C) {
    constexpr int SPW = kWave / CMAX;
    constexpr int kChunk = 256, kIters = kChunk / kWave;
    __shared__ float s_w[kChunk * (CMAX + 1)];
    __shared__ float s_logit[kThreads / kWave][SPW][CMAX];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int i = blockIdx.y;
    const int s0 = (blockIdx.x * (kThreads / kWave) + wave) * SPW;
    const float* W = x + (int64_t)i * ld + w_off;
    const int CP = C | 1;
    float acc[SPW][CMAX];
#pragma unroll
    for (int j = 0; j < SPW; ++j)
#pragma unroll
        for (int c = 0; c < CMAX; ++c) acc[j][c] = 0.0f;
    for (int k0 = 0; k0 < H; k0 += kChunk) {
        const int rows = min(kChunk, H - k0);
        // this chunk's activations first (independent of the staging), all loads in flight together
        float hv[kIters][SPW];
#pragma unroll
        for (int it = 0; it < kIters; ++it)
#pragma unroll
            for (int j = 0; j < SPW; ++j) {
                const int kk = lane + it * kWave;
                hv[it][j] = (kk < rows && s0 + j < B)
                                ? load_act<BF>(h, (int64_t)i * h_stride + (int64_t)(s0 + j) * H + k0 + kk) : 0.0f;
            }
        __syncthreads();
        stage_weights(s_w, W, k0, rows, C, CP);
        __syncthreads();
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            const int kk = lane + it * kWave;
            if (kk < rows) {
#pragma unroll
                for (int c = 0; c < CMAX; ++c) {
                    if (c < C) {
                        const float w = s_w[kk * CP + c];
#pragma unroll
                        for (int j = 0; j < SPW; ++j) acc[j][c] = __fmaf_rn(hv[it][j], w, acc[j][c]);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < SPW; ++j) {
#pragma unroll
        for (int c = 0; c < CMAX; ++c) {
            const float v = wave_sum(acc[j][c]);
            if (lane == 0) s_logit[wave][j][c] = v;
        }
    }
    __syncthreads();
    // lane group j (CMAX lanes) owns sample s0 + j; lane c of the group owns class c
    const int j = lane / CMAX, c = lane % CMAX;
    const int s = s0 + j;
    const bool live = s < B, mine = live && c < C;
    const float logit = mine ? s_logit[wave][j][c] + x[(int64_t)i * ld + b_off + c] : -INFINITY;
    float mx = logit;
#pragma unroll
    for (int off = CMAX / 2; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
    const int label = live ? labels[(int64_t)i * label_stride + s] : 0;
    const float ex = mine ? expf(logit - mx) : 0.0f;
    // Sum of the other classes' terms separately: near convergence softmax[label] is within an ulp of 1,
    // and both the loss log(1 + others / own) and the label's delta -(others / total) keep full relative
    // accuracy this way, where log(total) - logit and softmax - 1 would cancel.
    float others = c == label ? 0.0f : ex;
#pragma unroll
    for (int off = CMAX / 2; off >= 1; off >>= 1) others += __shfl_xor(others, off, kWave);
    const int src_lane = j * CMAX + (label & (CMAX - 1));
    const float own = __shfl(ex, src_lane, kWave);
    const float picked = __shfl(logit, src_lane, kWave);
    const float sum = others + own;
    if (live && c == 0)
        loss_parts[(int64_t)i * B + s] = own > 1e-30f ? log1pf(others / own) : (logf(sum) + mx) - picked;
    if (mine) {
        const float d = c == label ? -(others / sum) : ex / sum;
        dlogits[((int64_t)i * B + s) * C + c] = d / (float)B;
    }
}

// dW[k][c] = sum_s h[s][k] dlogits[s][c], db[c] = sum_s dlogits[s][c].  A workgroup owns 32 hidden units
// k; its 8 lane groups of 32 take the samples s = j, j + 8, ... and are combined by a fixed-order sum
// through LDS.  grid (ceil(H / 32), m)
template <bool BF, int CMAX>
__global__ __launch_bounds__(kThreads) void head_dw_kernel(const void* __restrict__ h, int64_t h_stride,
                                                           const float* __restrict__ dlogits, float* __restrict__ g,
                                                           int64_t ld, int64_t w_off, int64_t b_off, int B, int H,
                                                           int C, FusedUpdate upd) {
    constexpr int kCols = 32, kGroups = kThreads / kCols, kRows = 256;
    __shared__ float s_dl[kRows * kMaxC];
    __shared__ float s_part[kGroups][CMAX][kCols + 1];
    const int i = blockIdx.y;
    const int kk = threadIdx.x % kCols, grp = threadIdx.x / kCols;
    const int k = blockIdx.x * kCols + kk;
    float acc[CMAX];
#pragma unroll
    for (int c = 0; c < CMAX; ++c) acc[c] = 0.0f;
    float bias_acc = 0.0f;
    for (int s0 = 0; s0 < B; s0 += kRows) {
        const int rows = min(kRows, B - s0);
        __syncthreads();
        for (int t = threadIdx.x; t < rows * C; t += kThreads) s_dl[t] = dlogits[((int64_t)i * B + s0) * C + t];
        __syncthreads();
        if (k < H) {
            constexpr int kBatch = 8;   // activation loads in flight per lane
            for (int sb = grp; sb < rows; sb += kGroups * kBatch) {
                float hv[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int s = sb + u * kGroups;
                    hv[u] = s < rows ? load_act<BF>(h, (int64_t)i * h_stride + (int64_t)(s0 + s) * H + k) : 0.0f;
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int s = sb + u * kGroups;
                    if (s < rows) {
#pragma unroll
                        for (int c = 0; c < CMAX; ++c)
                            if (c < C) acc[c] = __fmaf_rn(hv[u], s_dl[s * C + c], acc[c]);
                    }
                }
            }
        }
        if (blockIdx.x == 0 && threadIdx.x < C)
            for (int s = 0; s < rows; ++s) bias_acc += s_dl[s * C + threadIdx.x];
    }
#pragma unroll
    for (int c = 0; c < CMAX; ++c) s_part[grp][c][kk] = acc[c];
    __syncthreads();
    // the 32 rows of this workgroup are one contiguous run of 32 C floats in g: lane t finishes
    // element t of that run (row t / C, class t % C), summing the lane groups in a fixed order
    const int k_base = blockIdx.x * kCols;
    for (int t = threadIdx.x; t < kCols * C; t += kThreads) {
        const int kl = t / C, c = t % C;
        float v = 0.0f;
#pragma unroll
        for (int j = 0; j < kGroups; ++j) v += s_part[j][c][kl];
        if (k_base + kl < H) {
            const int64_t col = w_off + (int64_t)k_base * C + t, idx = (int64_t)i * ld + col;
            if (upd.enabled) fused_update_apply(upd, idx, col, v, upd.x_in[idx], upd.mu != 0.0f ? upd.buf[idx] : 0.0f);
            else g[idx] = v;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < C) {
        const int64_t col = b_off + threadIdx.x, idx = (int64_t)i * ld + col;
        if (upd.enabled) fused_update_apply(upd, idx, col, bias_acc, upd.x_in[idx], upd.mu != 0.0f ? upd.buf[idx] : 0.0f);
        else g[idx] = bias_acc;
    }
}

// dz[s][k] = (sum_c dlogits[s][c] W[k][c]) * [h[s][k] > 0];  grid (ceil(H / 256), ceil(B / ROWS), m)
template <bool BF, int CMAX, int ROWS>
__global__ __launch_bounds__(kThreads) void head_dz_kernel(const void* __restrict__ h, int64_t h_stride,
                                                           const float* __restrict__ x, int64_t ld, int64_t w_off,
                                                           const float* __restrict__ dlogits, void* __restrict__ dz,
                                                           void* __restrict__ dz_t, int B, int H, int C) {
    __shared__ float s_dl[ROWS * kMaxC];
    __shared__ float s_w[kThreads * (CMAX + 1)];
    const int i = blockIdx.z;
    const int s0 = blockIdx.y * ROWS;
    const int rows = min(ROWS, B - s0);
    const int k0 = blockIdx.x * kThreads;
    const int CP = C | 1;
    for (int t = threadIdx.x; t < rows * C; t += kThreads) s_dl[t] = dlogits[((int64_t)i * B + s0) * C + t];
    stage_weights(s_w, x + (int64_t)i * ld + w_off, k0, min(kThreads, H - k0), C, CP);
    __syncthreads();
    const int k = k0 + threadIdx.x;
    if (k >= H) return;
    float w[CMAX];
#pragma unroll
    for (int c = 0; c < CMAX; ++c) w[c] = c < C ? s_w[threadIdx.x * CP + c] : 0.0f;
    uint16_t tr[ROWS];
#pragma unroll
    for (int s = 0; s < ROWS; ++s) {
        tr[s] = 0;
        if (s < rows) {
            const int64_t idx = (int64_t)(s0 + s) * H + k;
            float acc = 0.0f;
#pragma unroll
            for (int c = 0; c < CMAX; ++c)
                if (c < C) acc = __fmaf_rn(s_dl[s * C + c], w[c], acc);
            const float hv = load_act<BF>(h, (int64_t)i * h_stride + idx);
            const float v = hv > 0.0f ? acc : 0.0f;
            if (BF) {
                tr[s] = f32_to_bf16(v);
                ((uint16_t*)dz)[(int64_t)i * B * H + idx] = tr[s];
            } else {
                ((float*)dz)[(int64_t)i * B * H + idx] = v;
            }
        }
    }
    if (BF && dz_t) {  // transposed copy [H][B]: ROWS consecutive samples of column k
        uint16_t* o = (uint16_t*)dz_t + (int64_t)i * B * H + (int64_t)k * B + s0;
        if (rows == ROWS && ROWS == 8) {
            typedef unsigned int u4 __attribute__((ext_vector_type(4)));
            u4 pk;
            pk.x = tr[0] | ((unsigned)tr[1] << 16);
            pk.y = tr[2] | ((unsigned)tr[3] << 16);
            pk.z = tr[4] | ((unsigned)tr[5] << 16);
            pk.w = tr[6] | ((unsigned)tr[7] << 16);
            *(u4*)o = pk;
        } else {
            for (int s = 0; s < rows; ++s) o[s] = tr[s];
        }
    }
}

static bool head_args_ok(const HeadArgs& a) {
    return a.h && a.x && a.g && a.labels && a.dlogits && a.loss_parts && a.m >= 1 && a.m <= 65535 && a.B >= 1 &&
           a.H >= 1 && a.C >= 1 && a.C <= kMaxC && a.w_off >= 0 && a.b_off >= 0 &&
           a.w_off + (int64_t)a.H * a.C <= a.ld && a.b_off + a.C <= a.ld;
}

hipError_t launch_head_fwd(const HeadArgs& a, hipStream_t s) {
    if (!head_args_ok(a)) return hipErrorInvalidValue;
    const int spw = a.C <= 16 ? 4 : 2;   // samples per wavefront = 64 / CMAX
    dim3 grid((unsigned)((a.B + 4 * spw - 1) / (4 * spw)), (unsigned)a.m);
#define OLS_HEAD_FWD(BF, CM)                                                                                       \
    head_fwd_kernel<BF, CM><<<grid, kThreads, 0, s>>>(a.h, a.h_stride, a.x, a.ld, a.w_off, a.b_off, a.labels,      \
                                                      a.label_stride, a.dlogits, a.loss_parts, a.B, a.H, a.C)
    if (a.h_bf16) {
        if (a.C <= 16) OLS_HEAD_FWD(true, 16); else OLS_HEAD_FWD(true, 32);
    } else {
        if (a.C <= 16) OLS_HEAD_FWD(false, 16); else OLS_HEAD_FWD(false, 32);
    }
#undef OLS_HEAD_FWD
    return hipGetLastError();
}

hipError_t launch_head_bwd(const HeadArgs& a, hipStream_t s) {
    if (!head_args_ok(a)) return hipErrorInvalidValue;
    if (a.upd.enabled && (!a.upd.x_in || !a.upd.x_out || (a.upd.mu != 0.0f && !a.upd.buf) || (a.upd.pull && !a.upd.z) ||
                          a.upd.ld != a.ld))
        return hipErrorInvalidValue;
    // the delta for the last hidden layer first: it reads the output weights, which the gradient kernel
    // may then update in place
    if (a.dz) {
        constexpr int kRows = 8;
        const unsigned by = (unsigned)((a.B + kRows - 1) / kRows);
        if (by > 65535u || a.m > 65535) return hipErrorInvalidValue;
        dim3 grid_z((unsigned)((a.H + kThreads - 1) / kThreads), by, (unsigned)a.m);
#define OLS_HEAD_DZ(BF, CM)                                                                                        \
    head_dz_kernel<BF, CM, kRows><<<grid_z, kThreads, 0, s>>>(a.h, a.h_stride, a.x, a.ld, a.w_off, a.dlogits,      \
                                                              a.dz, a.dz_t, a.B, a.H, a.C)
        if (a.h_bf16) {
            if (a.C <= 16) OLS_HEAD_DZ(true, 16); else OLS_HEAD_DZ(true, 32);
        } else {
            if (a.C <= 16) OLS_HEAD_DZ(false, 16); else OLS_HEAD_DZ(false, 32);
        }
#undef OLS_HEAD_DZ
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    dim3 grid_w((unsigned)((a.H + 31) / 32), (unsigned)a.m);
#define OLS_HEAD_DW(BF, CM)                                                                                        \
    head_dw_kernel<BF, CM><<<grid_w, kThreads, 0, s>>>(a.h, a.h_stride, a.dlogits, a.g, a.ld, a.w_off, a.b_off,    \
                                                       a.B, a.H, a.C, a.upd)
    if (a.h_bf16) {
        if (a.C <= 16) OLS_HEAD_DW(true, 16); else OLS_HEAD_DW(true, 32);
    } else {
        if (a.C <= 16) OLS_HEAD_DW(false, 16); else OLS_HEAD_DW(false, 32);
    }
#undef OLS_HEAD_DW
    return hipGetLastError();
}

}  // namespace ols
