// Streaming kernels over the replica-major state [m][ld]: the local (momentum) step, the pull-back,
// their fusion into one HBM pass, and the initial broadcast.  All are bound by HBM bandwidth:
//   local step      reads g, x, buf and writes x, buf   -> 20 B per element-replica (12 B without momentum)
//   step + pull     the same plus one read of z shared by the m rows -> 20 + 4/m B
//   pull-back only  reads x, z and writes x             -> 8 + 4/m B
// Every lane moves 16-byte vectors; a workgroup covers a contiguous span of one replica row so that
// all accesses of a wavefront are to consecutive 1 KiB segments.
//
// Arithmetic (Section 2 of arXiv 2002.09539; "Momentum Variant" paragraph for the buffer):
//   buf' = mu buf + g;  dir = g + mu buf' (Nesterov) or buf' (heavy ball);  x_half = x - gamma dir
//   x'   = x_half - alpha (x_half - z)                                    on synchronisation steps
// Each line is one explicitly rounded fp32 operation (fma / sub), so the fused and the two-pass
// orders produce identical bits.
#include "ols_internal.h"

namespace ols {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));

#ifndef OLS_UPDATE_THREADS
#define OLS_UPDATE_THREADS 64
#endif
#ifndef OLS_UPDATE_UNROLL
#define OLS_UPDATE_UNROLL 1
#endif
#ifndef OLS_UPDATE_NONTEMPORAL
#define OLS_UPDATE_NONTEMPORAL 1
#endif
constexpr int kThreads = OLS_UPDATE_THREADS;
// Workgroup size and 16-byte vectors per lane per array.  Measured on the d = 11.2 M, m = 16 stream (local
// step, us): 64 threads x 1 -> 552, 128 x 1 -> 584, 256 x 1 -> 599, 256 x 2 -> 628, 256 x 4 -> 618,
// 256 x 8 -> 655, 512 x 2 -> 619, 1024 x 2 -> 654; plain instead of non-temporal accesses (256 x 1) -> 656.
// Single-wavefront workgroups stream best: 6.5 TB/s.
constexpr int kUnroll = OLS_UPDATE_UNROLL;

#if OLS_UPDATE_NONTEMPORAL
__device__ __forceinline__ f4 ld_stream(const f4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void st_stream(f4* p, f4 v) { __builtin_nontemporal_store(v, p); }
#else
__device__ __forceinline__ f4 ld_stream(const f4* p) { return *p; }
__device__ __forceinline__ void st_stream(f4* p, f4 v) { *p = v; }
#endif

__device__ __forceinline__ unsigned int bf16_rne(float f) { return bf16_bits_rne(f); }
__device__ __forceinline__ u2 pack_bf16x4(f4 v) {
    u2 r;
    r.x = bf16_rne(v.x) | (bf16_rne(v.y) << 16);
    r.y = bf16_rne(v.z) | (bf16_rne(v.w) << 16);
    return r;
}


// One workgroup per (replica, span of kThreads * kUnroll vectors); the replica is the SLOW part of the
// linear workgroup id, so consecutive workgroups stream through one row.  Measured alternatives on the
// d = 11.2 M, m = 16 stream (step + pull-back, 617 us): replica as the fast index halves the re-reads of
// the anchor z (HBM fetches 2.51 GB instead of 2.87 GB, algorithmic 2.19 GB) but takes 660 us, and one
// workgroup looping over all replicas with z in registers reaches the algorithmic traffic but takes
// 677 us -- row-wise streaming is what the memory system rewards, the extra z fetches are served by the
// last-level cache.
template <bool MOM, bool NEST, bool PULL, bool SHADOW>
__global__ __launch_bounds__(kThreads) void step_kernel(const f4* __restrict__ g, const f4* x_in, f4* x_out,
                                                        f4* buf, const f4* __restrict__ z, u2* __restrict__ shadow,
                                                        int64_t n4, int m, float gamma, float mu, float alpha) {
    const int64_t spans = (n4 + kThreads * kUnroll - 1) / (kThreads * kUnroll);
    const int64_t row = (int64_t)(blockIdx.x / spans) * n4;
    const int64_t c0 = (int64_t)(blockIdx.x % spans) * (kThreads * kUnroll) + threadIdx.x;
    f4 vg[kUnroll], vx[kUnroll], vb[kUnroll], vz[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t c = c0 + u * kThreads;
        if (c < n4) {
            vg[u] = ld_stream(g + row + c);
            vx[u] = ld_stream(x_in + row + c);
            if (MOM) vb[u] = ld_stream(buf + row + c);
            if (PULL) vz[u] = z[c];
        }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t c = c0 + u * kThreads;
        if (c < n4) {
            f4 xo, bo;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float b = MOM ? vb[u][e] : 0.0f;
                xo[e] = local_step_elem(vg[u][e], vx[u][e], b, PULL ? vz[u][e] : 0.0f, gamma, mu, alpha, MOM, NEST, PULL);
                bo[e] = b;
            }
            st_stream(x_out + row + c, xo);
            if (MOM) st_stream(buf + row + c, bo);
            if (SHADOW) shadow[row + c] = pack_bf16x4(xo);
        }
    }
}

template <bool SHADOW>
__global__ __launch_bounds__(kThreads) void pull_kernel(f4* x, const f4* __restrict__ z, u2* __restrict__ shadow,
                                                        int64_t n4, int m, float alpha) {
    const int64_t spans = (n4 + kThreads * kUnroll - 1) / (kThreads * kUnroll);
    const int64_t row = (int64_t)(blockIdx.x / spans) * n4;
    const int64_t c0 = (int64_t)(blockIdx.x % spans) * (kThreads * kUnroll) + threadIdx.x;
    f4 vx[kUnroll], vz[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t c = c0 + u * kThreads;
        if (c < n4) {
            vx[u] = ld_stream(x + row + c);
            vz[u] = z[c];
        }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t c = c0 + u * kThreads;
        if (c < n4) {
            f4 xo;
#pragma unroll
            for (int e = 0; e < 4; ++e) xo[e] = pull_back_elem(vx[u][e], vz[u][e], alpha);
            st_stream(x + row + c, xo);
            if (SHADOW) shadow[row + c] = pack_bf16x4(xo);
        }
    }
}

// Stale-average synchronisation ("Related Works": a round's local updates are applied to the average of the models
// of tau iterations before): x <- z + (x - snap), snap <- the new x; z is the average of the old snapshots.
template <bool SHADOW>
__global__ __launch_bounds__(kThreads) void stale_sync_kernel(f4* x, f4* snap, const f4* __restrict__ z,
                                                              u2* __restrict__ shadow, int64_t n4, int m) {
    const int64_t spans = (n4 + kThreads * kUnroll - 1) / (kThreads * kUnroll);
    const int64_t row = (int64_t)(blockIdx.x / spans) * n4;
    const int64_t c0 = (int64_t)(blockIdx.x % spans) * (kThreads * kUnroll) + threadIdx.x;
    f4 vx[kUnroll], vs[kUnroll], vz[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t c = c0 + u * kThreads;
        if (c < n4) {
            vx[u] = ld_stream(x + row + c);
            vs[u] = ld_stream(snap + row + c);
            vz[u] = z[c];
        }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t c = c0 + u * kThreads;
        if (c < n4) {
            f4 xo;
#pragma unroll
            for (int e = 0; e < 4; ++e) xo[e] = __fadd_rn(vz[u][e], __fsub_rn(vx[u][e], vs[u][e]));
            st_stream(x + row + c, xo);
            st_stream(snap + row + c, xo);
            if (SHADOW) shadow[row + c] = pack_bf16x4(xo);
        }
    }
}

// x rows, x_alt rows and z take x0 (zero beyond d); buf rows are cleared; grid.y = m + 1 (last = z).
__global__ __launch_bounds__(kThreads) void init_kernel(float* x, float* x_alt, float* buf, float* z,
                                                        uint16_t* shadow, const float* __restrict__ x0, int m,
                                                        int64_t d, int64_t ld) {
    const int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (c >= ld) return;
    const float v = c < d ? x0[c] : 0.0f;
    const int r = blockIdx.y;
    if (r == m) {
        z[c] = v;
        return;
    }
    const int64_t o = (int64_t)r * ld + c;
    x[o] = v;
    if (x_alt) x_alt[o] = v;
    if (buf) buf[o] = 0.0f;
    if (shadow) shadow[o] = (uint16_t)bf16_rne(v);
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <bool MOM, bool NEST, bool PULL>
static void dispatch_shadow(const UpdateArgs& a, unsigned grid, hipStream_t s) {
    const int64_t n4 = a.ld / 4;
    if (a.shadow)
        step_kernel<MOM, NEST, PULL, true><<<grid, kThreads, 0, s>>>((const f4*)a.g, (const f4*)a.x_in, (f4*)a.x_out,
                                                                    (f4*)a.buf, (const f4*)a.z, (u2*)a.shadow, n4,
                                                                    a.m, a.gamma, a.mu, a.alpha);
    else
        step_kernel<MOM, NEST, PULL, false><<<grid, kThreads, 0, s>>>((const f4*)a.g, (const f4*)a.x_in,
                                                                     (f4*)a.x_out, (f4*)a.buf, (const f4*)a.z,
                                                                     nullptr, n4, a.m, a.gamma, a.mu, a.alpha);
}

static bool grid_for(int m, int64_t ld, unsigned* grid) {
    const int64_t per_block = (int64_t)kThreads * kUnroll;
    const int64_t blocks = ((ld / 4 + per_block - 1) / per_block) * m;
    if (blocks < 1 || blocks > 0x7FFFFFFF) return false;
    *grid = (unsigned)blocks;
    return true;
}

hipError_t launch_step(const UpdateArgs& a, hipStream_t s) {
    if (a.m < 1 || a.ld < 4 || a.ld % 4 != 0) return hipErrorInvalidValue;
    if (!a.g || !a.x_in || !a.x_out || (a.mu != 0.0f && !a.buf) || (a.pull && !a.z)) return hipErrorInvalidValue;
    if (!aligned16(a.g) || !aligned16(a.x_in) || !aligned16(a.x_out) || !aligned16(a.buf) || !aligned16(a.z) ||
        !aligned16(a.shadow))
        return hipErrorInvalidValue;
    unsigned grid;
    if (!grid_for(a.m, a.ld, &grid)) return hipErrorInvalidValue;
    const bool mom = a.mu != 0.0f;
    if (mom) {
        if (a.nesterov) {
            if (a.pull) dispatch_shadow<true, true, true>(a, grid, s);
            else dispatch_shadow<true, true, false>(a, grid, s);
        } else {
            if (a.pull) dispatch_shadow<true, false, true>(a, grid, s);
            else dispatch_shadow<true, false, false>(a, grid, s);
        }
    } else {
        if (a.pull) dispatch_shadow<false, false, true>(a, grid, s);
        else dispatch_shadow<false, false, false>(a, grid, s);
    }
    return hipGetLastError();
}

hipError_t launch_pull(float* x, const float* z, uint16_t* shadow, int m, int64_t ld, float alpha, hipStream_t s) {
    if (m < 1 || ld < 4 || ld % 4 != 0 || !x || !z) return hipErrorInvalidValue;
    if (!aligned16(x) || !aligned16(z) || !aligned16(shadow)) return hipErrorInvalidValue;
    unsigned grid;
    if (!grid_for(m, ld, &grid)) return hipErrorInvalidValue;
    const int64_t n4 = ld / 4;
    if (shadow) pull_kernel<true><<<grid, kThreads, 0, s>>>((f4*)x, (const f4*)z, (u2*)shadow, n4, m, alpha);
    else pull_kernel<false><<<grid, kThreads, 0, s>>>((f4*)x, (const f4*)z, nullptr, n4, m, alpha);
    return hipGetLastError();
}

hipError_t launch_stale_sync(float* x, float* snap, const float* z, uint16_t* shadow, int m, int64_t ld,
                             hipStream_t s) {
    if (m < 1 || ld < 4 || ld % 4 != 0 || !x || !snap || !z || x == snap) return hipErrorInvalidValue;
    if (!aligned16(x) || !aligned16(snap) || !aligned16(z) || !aligned16(shadow)) return hipErrorInvalidValue;
    unsigned grid;
    if (!grid_for(m, ld, &grid)) return hipErrorInvalidValue;
    const int64_t n4 = ld / 4;
    if (shadow) stale_sync_kernel<true><<<grid, kThreads, 0, s>>>((f4*)x, (f4*)snap, (const f4*)z, (u2*)shadow, n4, m);
    else stale_sync_kernel<false><<<grid, kThreads, 0, s>>>((f4*)x, (f4*)snap, (const f4*)z, nullptr, n4, m);
    return hipGetLastError();
}

hipError_t launch_init(float* x, float* x_alt, float* buf, float* z, uint16_t* shadow, const float* x0, int m,
                       int64_t d, int64_t ld, hipStream_t s) {
    if (m < 1 || m > 65534 || d < 1 || ld < d || !x || !z || !x0) return hipErrorInvalidValue;
    dim3 grid((unsigned)((ld + kThreads - 1) / kThreads), (unsigned)(m + 1));
    init_kernel<<<grid, kThreads, 0, s>>>(x, x_alt, buf, z, shadow, x0, m, d, ld);
    return hipGetLastError();
}

}  // namespace ols
