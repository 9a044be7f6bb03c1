// Epilogue of the weight-gradient GEMMs, shared by the fp32 and bf16 kernels.
//
// The accumulators hold a BM x BN tile of the gradient dW (one 32 x 32 block per (i, j), register r of a
// lane = row 8 (r / 4) + 4 (lane / 32) + r % 4, column lane % 32).  Written straight from that layout a
// wavefront touches 128-byte pieces of many rows; here the tile is first staged through the (now idle)
// operand LDS so that every lane then owns 4 consecutive columns of one row: 16-byte accesses, 512-byte
// contiguous runs per row.  Each gradient vector is then either stored to g or -- the fused route --
// consumed on the spot: parameter and momentum are read, the local step (+ pull-back) of Section 2,
// arXiv 2002.09539 is applied with the same fp32 operation sequence as the streaming kernels, and the
// results are written back, so the gradient never travels to HBM and back.
#pragma once
#include "ols_internal.h"

namespace ols {

typedef float ep_f4 __attribute__((ext_vector_type(4)));
typedef float ep_f16 __attribute__((ext_vector_type(16)));
typedef unsigned int ep_u2 __attribute__((ext_vector_type(2)));

struct DwOut {
    float* g;          // gradient destination of this group's tile origin row 0 / col 0 (unfused route)
    int ldg;           // leading dimension of g (= N)
    FusedUpdate upd;   // fused route when upd.enabled
    int64_t upd_base;  // group * ld + w_off: flat index of element (0, 0) of the layer's weight matrix
    int64_t col_base;  // w_off: position of element (0, 0) inside the replica row
};

__device__ __forceinline__ unsigned int ep_bf16(float f) { return bf16_bits_rne(f); }

#ifndef OLS_EPILOGUE_NONTEMPORAL
#define OLS_EPILOGUE_NONTEMPORAL 1
#endif
#if OLS_EPILOGUE_NONTEMPORAL
__device__ __forceinline__ ep_f4 ep_load_stream(const ep_f4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void ep_store_stream(ep_f4* p, ep_f4 v) { __builtin_nontemporal_store(v, p); }
#else
__device__ __forceinline__ ep_f4 ep_load_stream(const ep_f4* p) { return *p; }
__device__ __forceinline__ void ep_store_stream(ep_f4* p, ep_f4 v) { *p = v; }
#endif

// One vector of 4 gradient entries at (row, col .. col + 3) of the layer's weight matrix.
__device__ __forceinline__ void dw_consume(const DwOut& o, int N, int row, int col, ep_f4 g, ep_f4 x, ep_f4 b, ep_f4 z) {
    const FusedUpdate& u = o.upd;
    const int64_t off = (int64_t)row * N + col;
    ep_f4 xn, bn = b;
    const bool mom = u.mu != 0.0f, nest = u.nesterov != 0, pull = u.pull != 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float be = bn[e];
        xn[e] = local_step_elem(g[e], x[e], be, z[e], u.gamma, u.mu, u.alpha, mom, nest, pull);
        bn[e] = be;
    }
    // the state streams through once per step: non-temporal accesses keep it from displacing the operands in L2
    ep_store_stream((ep_f4*)(u.x_out + o.upd_base + off), xn);
    if (u.mu != 0.0f) ep_store_stream((ep_f4*)(u.buf + o.upd_base + off), bn);
    if (u.shadow) {
        ep_u2 pk;
        pk.x = ep_bf16(xn[0]) | (ep_bf16(xn[1]) << 16);
        pk.y = ep_bf16(xn[2]) | (ep_bf16(xn[3]) << 16);
        *(ep_u2*)(u.shadow + o.upd_base + off) = pk;
    }
}

// The state of a tile requested ahead of the contraction: lane's vector k of the epilogue (pass k / kIters, iteration
// k % kIters) is x[k] (and b[k], the momentum).  PF: 0 nothing, 1 parameters, 2 parameters and momentum.  Measured on
// the bf16 weight-gradient GEMM of the 3072-2048-2048-2048-10 model (batch 256, 16 workers; us per launch): 269.6
// without, 263.0 with the parameters (144 registers, three wavefronts per SIMD), 271.0 with parameters and momentum
// (164 registers); on the fp32 kernel at batch 64 (64 workers) 584 / 595 / 605, so only the bf16 kernel uses it.
#ifndef OLS_DW_PREFETCH
#define OLS_DW_PREFETCH 1
#endif
template <int NVEC>
struct DwState {
    ep_f4 x[NVEC], b[NVEC];
};
template <int BM, int BN, int RP, int THREADS, int PF>
__device__ __forceinline__ void dw_prefetch_state(DwState<BM * BN / 4 / THREADS>& st, const DwOut& o, int m0, int n0, int M, int N) {
    constexpr int kVecPerRow = BN / 4, kIters = RP * kVecPerRow / THREADS;
    if (PF == 0 || !o.upd.enabled) return;
    const bool mom = o.upd.mu != 0.0f;
#pragma unroll
    for (int k = 0; k < BM * BN / 4 / THREADS; ++k) {
        const int v = threadIdx.x + (k % kIters) * THREADS;
        const int row = m0 + (k / kIters) * RP + v / kVecPerRow, col = n0 + 4 * (v % kVecPerRow);
        const int64_t off = (row < M && col < N) ? (int64_t)row * N + col : 0;
        st.x[k] = ep_load_stream((const ep_f4*)(o.upd.x_in + o.upd_base + off));
        if (PF >= 2 && mom) st.b[k] = ep_load_stream((const ep_f4*)(o.upd.buf + o.upd_base + off));
    }
}

// stage: LDS scratch of at least RP * (BN + 4) floats, RP a multiple of 32 dividing BM.
// (m0, n0): tile origin; (wm0, wn0): this wavefront's origin inside the tile; M, N: matrix extents.
template <int BM, int BN, int TM, int TN, int RP, int THREADS, int PF = 0>
__device__ __forceinline__ void dw_epilogue_staged(float* stage, const ep_f16 (&acc)[TM][TN], const DwOut& o, int m0,
                                                   int n0, int wm0, int wn0, int M, int N,
                                                   const DwState<BM * BN / 4 / THREADS>* st = nullptr) {
    constexpr int kPitch = BN + 4;
    constexpr int kVecPerRow = BN / 4;
    constexpr int kVecs = RP * kVecPerRow;
    static_assert(RP % 32 == 0 && BM % RP == 0 && kVecs % THREADS == 0, "staging shape");
    constexpr int kIters = kVecs / THREADS;
    constexpr int kUnroll = kIters % 4 == 0 ? 4 : (kIters % 2 == 0 ? 2 : 1);
    const int lane = threadIdx.x % 64, lane32 = lane % 32, half = lane / 32;
    const bool fused = o.upd.enabled != 0;
    const bool mom = o.upd.mu != 0.0f, pull = o.upd.pull != 0;
#pragma unroll
    for (int p0 = 0; p0 < BM; p0 += RP) {
        __syncthreads();   // the previous pass (or the main loop) has finished with the LDS
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int br = wm0 + 32 * i - p0;   // block row inside this pass
            if (br >= 0 && br < RP) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        stage[(br + 8 * (r / 4) + 4 * half + (r % 4)) * kPitch + wn0 + 32 * j + lane32] = acc[i][j][r];
            }
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < kIters; it += kUnroll) {
            ep_f4 gv[kUnroll], xv[kUnroll], bv[kUnroll], zv[kUnroll];
            int rows[kUnroll], cols[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int v = threadIdx.x + (it + u) * THREADS;
                const int rl = v / kVecPerRow, c4 = v % kVecPerRow;
                rows[u] = m0 + p0 + rl;
                cols[u] = n0 + 4 * c4;
                gv[u] = *(const ep_f4*)(stage + rl * kPitch + 4 * c4);
                const bool ok = rows[u] < M && cols[u] < N;
                if (!ok) rows[u] = -1;
                if (fused) {   // every lane issues its loads (out-of-range lanes re-read element 0)
                    const int64_t off = ok ? (int64_t)rows[u] * N + cols[u] : 0;
                    const int k = (p0 / RP) * kIters + it + u;
                    if (PF >= 1) xv[u] = st->x[k];
                    else xv[u] = ep_load_stream((const ep_f4*)(o.upd.x_in + o.upd_base + off));
                    if (mom) {
                        if (PF >= 2) bv[u] = st->b[k];
                        else bv[u] = ep_load_stream((const ep_f4*)(o.upd.buf + o.upd_base + off));
                    }
                    if (pull) zv[u] = *(const ep_f4*)(o.upd.z + o.col_base + off);
                }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                if (rows[u] < 0) continue;
                if (fused) dw_consume(o, N, rows[u], cols[u], gv[u], xv[u], bv[u], zv[u]);
                else *(ep_f4*)(o.g + (int64_t)rows[u] * o.ldg + cols[u]) = gv[u];
            }
        }
    }
}

}  // namespace ols
