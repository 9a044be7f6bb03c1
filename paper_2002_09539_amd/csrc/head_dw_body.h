// Gradients of the output layer's weights and bias as a device function, so that the same code runs either as
// a kernel of its own (head_dw_kernel) or as extra "guest" workgroups at the front of the launch of a hidden
// layer's weight-gradient GEMM.  The work is a few MFLOP per worker and bound by its chain of memory round
// trips; riding in a launch that keeps every compute unit busy for a hundred microseconds hides that chain
// completely, where a kernel of its own adds its whole latency to the step.
//
//   dW[k][c] = sum_s h[s][k] dlogits[s][c],   db[c] = sum_s dlogits[s][c]
// (output-layer part of the gradient g_i of Section 2, arXiv 2002.09539), stored to g or consumed by the fused
// local step (+ pull-back).  A workgroup of 256 threads owns 32 hidden units of one worker; the activations of
// those units and the dlogits pass through LDS, kRows samples at a time; lane (k, class quad, part) sums its
// part of the samples in sample order and the parts are added in a fixed order, so the result does not depend
// on kRows.  The class dimension is padded to CMAX (16 or 32) with zeros in LDS.
#pragma once
#include "ols_internal.h"

namespace ols {

typedef float hd_f4 __attribute__((ext_vector_type(4)));
typedef unsigned int hd_u2 __attribute__((ext_vector_type(2)));

// LDS row pitch (floats) of a CMAX-wide row: a multiple of 4 so rows are read as 16-byte vectors, and an odd
// number of such vectors so that 16 lanes reading consecutive rows hit distinct banks.
__host__ __device__ constexpr int head_row_pitch(int C) { return 4 * (((C + 3) / 4) | 1); }

constexpr int kHeadDwThreads = 256;
constexpr int kHeadDwUnits = 32;   // hidden units per workgroup

__host__ __device__ constexpr int head_dw_parts(int CMAX) { return kHeadDwThreads / (kHeadDwUnits * (CMAX / 4)); }
__host__ __device__ constexpr int head_dw_lds_floats(int CMAX, int kRows) {
    return kRows * head_row_pitch(CMAX) + kRows * kHeadDwUnits + head_dw_parts(CMAX) * kHeadDwUnits * CMAX;
}
// samples per pass of a guest (64 or 32: few staging registers, so that the host kernel's register count is its
// own) whose staging fits `avail` floats; 0 if none does
__host__ __device__ constexpr int head_dw_rows_for(int CMAX, int avail) {
    for (int r = 64; r >= 32; r /= 2)
        if (head_dw_lds_floats(CMAX, r) <= avail) return r;
    return 0;
}

struct HeadDwDev {
    const void* h;          // [m][B][H] last hidden activations, fp32 or bf16
    const float* dlogits;   // [m][B][C]
    float* g;               // [m][ld] gradients (unfused route)
    int64_t h_stride, ld, w_off, b_off;
    int B, H, C;
    int bf16;               // activations are bf16
    int grid_x;             // workgroups per worker = ceil(H / 32)
    int live;               // grid_x * m workgroups do the work ...
    int blocks;             // ... out of this many reserved at the front of a host launch (a multiple of 8), 0: none
    FusedUpdate upd;
};

// host side (kernels_mlp_head.hip): argument checks and device layout; out->blocks workgroups are to be reserved
hipError_t head_dw_prepare(const HeadArgs& a, HeadDwDev* out);

__device__ __forceinline__ float head_bf16_elem(unsigned int word, int e) {
    return __uint_as_float((e & 1) ? (word & 0xFFFF0000u) : (word << 16));
}

// bx: workgroup index along the hidden units, i: worker.  lds: head_dw_lds_floats(CMAX, kRows) floats.
template <bool BF, int CMAX, int kRows>
__device__ __forceinline__ void head_dw_body(const HeadDwDev& a, float* lds, int bx, int i) {
    constexpr int kThreads = kHeadDwThreads, KW = kHeadDwUnits;
    constexpr int P = head_row_pitch(CMAX);
    constexpr int CQ = CMAX / 4;                      // class quads
    constexpr int NP = head_dw_parts(CMAX);           // parts the samples are split into (2 or 1)
    constexpr int kOut = KW * CMAX / kThreads;        // output elements per lane (class-padded)
    constexpr int kStage = kRows * CMAX / kThreads;   // staged dlogits per lane
    constexpr int kTile = kRows * KW / 4 / kThreads;  // staged 4-wide activation vectors per lane
    static_assert(kStage >= 1 && kTile >= 1 && kRows % NP == 0, "samples per pass");
    float* s_dl = lds;                  // [kRows][P]
    float* s_h = lds + kRows * P;       // [kRows][KW]
    float* s_part = s_h + kRows * KW;   // [NP][KW * CMAX]
    const FusedUpdate& upd = a.upd;
    const int B = a.B, H = a.H, C = a.C;
    const int cls = threadIdx.x % CMAX;
    const int kq = threadIdx.x % KW, cq = (threadIdx.x / KW) % CQ, part = threadIdx.x / (KW * CQ);
    const int k_base = bx * KW;
    const bool bias_lane = bx == 0 && (int)threadIdx.x < C;

    // Operands of the fused update, requested before anything else.  Output o of lane t is class t % CMAX of
    // row k_base + t / CMAX + o (256 / CMAX).
    float ux[kOut], ub[kOut], uz[kOut], bxv = 0.0f, bb = 0.0f, bz = 0.0f;
    if (upd.enabled) {
#pragma unroll
        for (int o = 0; o < kOut; ++o) {
            const int kk = k_base + threadIdx.x / CMAX + o * (kThreads / CMAX);
            ux[o] = ub[o] = uz[o] = 0.0f;
            if (cls < C && kk < H) {
                const int64_t col = a.w_off + (int64_t)kk * C + cls, idx = (int64_t)i * a.ld + col;
                ux[o] = upd.x_in[idx];
                if (upd.mu != 0.0f) ub[o] = upd.buf[idx];
                if (upd.pull) uz[o] = upd.z[col];
            }
        }
        if (bias_lane) {
            const int64_t col = a.b_off + threadIdx.x, idx = (int64_t)i * a.ld + col;
            bxv = upd.x_in[idx];
            if (upd.mu != 0.0f) bb = upd.buf[idx];
            if (upd.pull) bz = upd.z[col];
        }
    }
    hd_f4 acc = {0.f, 0.f, 0.f, 0.f};
    float bias_acc = 0.0f;
    for (int s0 = 0; s0 < B; s0 += kRows) {
        const int rows = min(kRows, B - s0);
        if (s0 > 0) __syncthreads();
        {   // dlogits rows (zero beyond C and beyond the batch) and the activation tile, one round trip
            const float* src = a.dlogits + ((int64_t)i * B + s0) * C + cls;
            float tmp[kStage];
#pragma unroll
            for (int u = 0; u < kStage; ++u) {
                const int r = threadIdx.x / CMAX + u * (kThreads / CMAX);
                tmp[u] = (cls < C && r < rows) ? src[r * C] : 0.0f;
            }
            hd_f4 th[kTile];
#pragma unroll
            for (int u = 0; u < kTile; ++u) {
                const int f = threadIdx.x + u * kThreads, r = f / (KW / 4), k = k_base + 4 * (f % (KW / 4));
                th[u] = hd_f4{0.f, 0.f, 0.f, 0.f};
                if (r < rows && k < H) {   // H is a multiple of 4
                    const int64_t idx = (int64_t)i * a.h_stride + (int64_t)(s0 + r) * H + k;
                    if constexpr (BF) {
                        const hd_u2 w = *(const hd_u2*)((const uint16_t*)a.h + idx);
                        th[u] = hd_f4{head_bf16_elem(w.x, 0), head_bf16_elem(w.x, 1), head_bf16_elem(w.y, 0),
                                      head_bf16_elem(w.y, 1)};
                    } else {
                        th[u] = *(const hd_f4*)((const float*)a.h + idx);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kStage; ++u) {
                const int r = threadIdx.x / CMAX + u * (kThreads / CMAX);
                s_dl[r * P + cls] = tmp[u];
            }
#pragma unroll
            for (int u = 0; u < kTile; ++u) *(hd_f4*)(s_h + 4 * (threadIdx.x + u * kThreads)) = th[u];
        }
        __syncthreads();
#pragma unroll 4
        for (int sidx = part; sidx < rows; sidx += NP) {
            const float hv = s_h[sidx * KW + kq];
            const hd_f4 dl = *(const hd_f4*)(s_dl + sidx * P + 4 * cq);
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = __fmaf_rn(hv, dl[q], acc[q]);
        }
        if (bias_lane)
            for (int sidx = 0; sidx < rows; ++sidx) bias_acc += s_dl[sidx * P + threadIdx.x];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) s_part[part * (KW * CMAX) + kq * CMAX + 4 * cq + q] = acc[q];
    __syncthreads();
#pragma unroll
    for (int o = 0; o < kOut; ++o) {
        const int t = threadIdx.x + o * kThreads;   // = (row inside the workgroup) * CMAX + class
        const int kk = k_base + t / CMAX;
        if (cls < C && kk < H) {
            float v = s_part[t];
#pragma unroll
            for (int q = 1; q < NP; ++q) v += s_part[q * (KW * CMAX) + t];
            const int64_t idx = (int64_t)i * a.ld + a.w_off + (int64_t)kk * C + cls;
            if (upd.enabled) fused_update_store(upd, idx, v, ux[o], ub[o], uz[o]);
            else a.g[idx] = v;
        }
    }
    if (bias_lane) {
        const int64_t idx = (int64_t)i * a.ld + a.b_off + threadIdx.x;
        if (upd.enabled) fused_update_store(upd, idx, bias_acc, bxv, bb, bz);
        else a.g[idx] = bias_acc;
    }
}

// Guest entry: workgroup `b` of the `a.blocks` reserved at the front of a host kernel whose LDS holds AVAIL floats.
template <int AVAIL>
__device__ __forceinline__ void head_dw_guest(const HeadDwDev& a, float* lds, int b) {
    constexpr int R16 = head_dw_rows_for(16, AVAIL), R32 = head_dw_rows_for(32, AVAIL);
    static_assert(R16 >= 32 && R32 >= 32, "host kernel's LDS too small for the guest");
    if (b >= a.live) return;
    const int bx = b % a.grid_x, i = b / a.grid_x;
    if (a.C <= 16) {
        if (a.bf16) head_dw_body<true, 16, R16>(a, lds, bx, i);
        else head_dw_body<false, 16, R16>(a, lds, bx, i);
    } else {
        if (a.bf16) head_dw_body<true, 32, R32>(a, lds, bx, i);
        else head_dw_body<false, 32, R32>(a, lds, bx, i);
    }
}

}  // namespace ols
