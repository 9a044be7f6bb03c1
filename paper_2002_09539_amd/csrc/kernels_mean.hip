// Anchor refresh: z = (1/m) sum_i x^{(i)} over the replica axis of x [m][ld] (anchor update rule of
// Section 2, arXiv 2002.09539), optionally in its momentum form v <- beta v + (mean - z), z <- z + v.
//
// HBM-bound: (4 m + 4) ld bytes per refresh.  Each lane owns a 16-byte column vector so every row read
// is fully coalesced.  The replica axis can be split G ways inside a workgroup to raise the number of
// independent loads in flight when ld alone gives too few workgroups: first across lane groups of a
// wavefront (combined with wavefront shuffles), then across the wavefronts of the workgroup (combined
// by a tree through LDS).  Rows are summed in a fixed order, so the result does not depend on timing.
//
// The second kernel fuses local step + pull-back + anchor refresh for callers that prefer removing the
// separate reduction to hiding it: a lane owns its column across ALL replicas, so the new anchor costs
// only its 4-byte write on top of the 20 B per element-replica of the step.
#include "ols_internal.h"

namespace ols {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kWave = 64;

__device__ __forceinline__ f4 shfl_xor_f4(f4 v, int mask) {
    f4 r;
    r.x = __shfl_xor(v.x, mask, kWave);
    r.y = __shfl_xor(v.y, mask, kWave);
    r.z = __shfl_xor(v.z, mask, kWave);
    r.w = __shfl_xor(v.w, mask, kWave);
    return r;
}

// SW wavefront groups x SL lane groups share the replica axis; a workgroup covers
// kThreads / (SW * SL) column vectors.
// Workgroup size of the unsplit kernel and independent row loads in flight per lane.  Measured on the
// d = 11.2 M, m = 16 stream (us per refresh, nothing else running): 256 threads x 4 rows: 129, 128 x 4: 130,
// 64 x 4: 126, 64 x 8: 123, 64 x 16: 124.
#ifndef OLS_MEAN_THREADS
#define OLS_MEAN_THREADS 64
#endif
#ifndef OLS_MEAN_ROWS
#define OLS_MEAN_ROWS 8
#endif
template <int THREADS, int SW, int SL, bool ANCHOR_MOM>
__global__ __launch_bounds__(THREADS) void mean_kernel(const f4* __restrict__ x, f4* z, f4* v, int m, int64_t n4,
                                                       float beta_z) {
    constexpr int G = SW * SL;
    constexpr int kWavesPerGroup = (THREADS / kWave) / SW;   // wavefronts that form one wave group
    constexpr int kColsPerWave = kWave / SL;
    constexpr int kCols = kColsPerWave * kWavesPerGroup;      // column vectors per workgroup
    const int wave = threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    const int wgroup = wave / kWavesPerGroup;                 // 0..SW-1
    const int lgroup = lane / kColsPerWave;                   // 0..SL-1
    const int col_in_block = (wave % kWavesPerGroup) * kColsPerWave + lane % kColsPerWave;
    const int64_t c = (int64_t)blockIdx.x * kCols + col_in_block;
    const bool live = c < n4;
    const int first = wgroup * SL + lgroup;                   // rows first, first + G, ...

    f4 acc = {0.f, 0.f, 0.f, 0.f};
    if (live) {
        constexpr int R = OLS_MEAN_ROWS;
        int i = first;
        for (; i + (R - 1) * G < m; i += R * G) {             // R independent loads in flight, added in row order
            f4 a[R];
#pragma unroll
            for (int r = 0; r < R; ++r) a[r] = __builtin_nontemporal_load(x + (int64_t)(i + r * G) * n4 + c);
#pragma unroll
            for (int r = 0; r < R; ++r) acc = acc + a[r];
        }
        for (; i < m; i += G) acc = acc + __builtin_nontemporal_load(x + (int64_t)i * n4 + c);
    }
    if (SL > 1) {
#pragma unroll
        for (int off = kColsPerWave; off < kWave; off <<= 1) acc = acc + shfl_xor_f4(acc, off);
    }
    if (SW > 1) {
        __shared__ f4 part[SW][kCols];
        if (lgroup == 0) part[wgroup][col_in_block] = acc;
        __syncthreads();
#pragma unroll
        for (int stride = SW / 2; stride >= 1; stride >>= 1) {
            if (lgroup == 0 && wgroup < stride)
                part[wgroup][col_in_block] = part[wgroup][col_in_block] + part[wgroup + stride][col_in_block];
            __syncthreads();
        }
        acc = part[0][col_in_block];
    }
    if (live && wgroup == 0 && lgroup == 0) {
        const float fm = (float)m;
        f4 mean;
#pragma unroll
        for (int e = 0; e < 4; ++e) mean[e] = anchor_mean_elem(acc[e], fm);
        if (ANCHOR_MOM) {
            const f4 zo = z[c];
            f4 vn = v[c], zn;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float ve = vn[e];
                zn[e] = anchor_momentum_elem(mean[e], zo[e], ve, beta_z);
                vn[e] = ve;
            }
            v[c] = vn;
            z[c] = zn;
        } else {
            z[c] = mean;
        }
    }
}

int mean_auto_split(int m, int64_t ld) {
    // Aim for at least ~8 workgroups per compute unit (256 CUs); never split finer than the rows allow.
    const int64_t n4 = ld / 4;
    int g = 1;
    while (g < 16 && g * 2 <= m && (n4 * g + kThreads - 1) / kThreads < 2048) g *= 2;
    return g;
}

template <int THREADS, int SW, int SL>
static void mean_dispatch(const MeanArgs& a, hipStream_t s) {
    const int64_t n4 = a.ld / 4;
    const int cols = THREADS / (SW * SL);
    const unsigned grid = (unsigned)((n4 + cols - 1) / cols);
    if (a.v)
        mean_kernel<THREADS, SW, SL, true><<<grid, THREADS, 0, s>>>((const f4*)a.x, (f4*)a.z, (f4*)a.v, a.m, n4, a.beta_z);
    else
        mean_kernel<THREADS, SW, SL, false><<<grid, THREADS, 0, s>>>((const f4*)a.x, (f4*)a.z, nullptr, a.m, n4, 0.0f);
}

hipError_t launch_mean(const MeanArgs& a, hipStream_t s) {
    if (a.m < 1 || a.ld < 4 || a.ld % 4 != 0 || !a.x || !a.z) return hipErrorInvalidValue;
    if ((reinterpret_cast<uintptr_t>(a.x) | reinterpret_cast<uintptr_t>(a.z) | reinterpret_cast<uintptr_t>(a.v)) & 15u)
        return hipErrorInvalidValue;
    int g = a.split > 0 ? a.split : mean_auto_split(a.m, a.ld);
    switch (g) {
        case 1: mean_dispatch<OLS_MEAN_THREADS, 1, 1>(a, s); break;
        case 2: mean_dispatch<kThreads, 2, 1>(a, s); break;
        case 4: mean_dispatch<kThreads, 4, 1>(a, s); break;
        case 8: mean_dispatch<kThreads, 4, 2>(a, s); break;
        case 16: mean_dispatch<kThreads, 4, 4>(a, s); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// step + pull-back + anchor refresh in one pass (column owner)
// ---------------------------------------------------------------------------------------------
// Launch shape, measured on the d = 11.2 M, m = 16 stream (us per launch; threads per workgroup x rows of
// loads in flight per lane): 256 x 4: 681, 64 x 4: 652, 128 x 4: 680, 512 x 4: 698, 256 x 16: 662,
// 64 x 8: 644, 64 x 16: 634 -- single-wavefront workgroups with a whole 16-replica column in flight.
// Two or four 16-byte columns per lane (2-4 KiB contiguous per wavefront and row) with proportionally fewer rows
// in flight were slower (667-691).  Giving each XCD (workgroup id mod 8) a contiguous eighth of the columns instead of
// every eighth 1 KiB span was slower too (681 against 635 us; the local step 561 against 552): HBM serves the chip best
// when all its compute units work on neighbouring addresses.
#ifndef OLS_SPM_THREADS
#define OLS_SPM_THREADS 64
#endif
#ifndef OLS_SPM_ROWS
#define OLS_SPM_ROWS 16
#endif
constexpr int kSpmThreads = OLS_SPM_THREADS;
template <bool WITH_STEP, bool MOM, bool NEST, bool ANCHOR_MOM>
__global__ __launch_bounds__(kSpmThreads) void step_pull_mean_kernel(const f4* __restrict__ g, const f4* x_in, f4* x_out,
                                                                  f4* buf, const f4* z_in, f4* z_out, f4* v, int m,
                                                                  int64_t n4, float gamma, float mu, float alpha,
                                                                  float beta_z) {
    const int64_t c = (int64_t)blockIdx.x * kSpmThreads + threadIdx.x;
    if (c >= n4) return;
    const f4 zo = z_in[c];
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    constexpr int R = OLS_SPM_ROWS;  // rows in flight
    for (int i0 = 0; i0 < m; i0 += R) {
        f4 vg[R], vx[R], vb[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (i0 + r < m) {
                const int64_t o = (int64_t)(i0 + r) * n4 + c;
                vx[r] = __builtin_nontemporal_load(x_in + o);
                if (WITH_STEP) vg[r] = __builtin_nontemporal_load(g + o);
                if (WITH_STEP && MOM) vb[r] = __builtin_nontemporal_load(buf + o);
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (i0 + r < m) {
                const int64_t o = (int64_t)(i0 + r) * n4 + c;
                f4 xo, bo;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (WITH_STEP) {
                        float b = MOM ? vb[r][e] : 0.0f;
                        xo[e] = local_step_elem(vg[r][e], vx[r][e], b, zo[e], gamma, mu, alpha, MOM, NEST, true);
                        bo[e] = b;
                    } else {
                        xo[e] = pull_back_elem(vx[r][e], zo[e], alpha);
                    }
                }
                __builtin_nontemporal_store(xo, x_out + o);
                if (WITH_STEP && MOM) __builtin_nontemporal_store(bo, buf + o);
                acc = acc + xo;
            }
        }
    }
    const float fm = (float)m;
    f4 mean;
#pragma unroll
    for (int e = 0; e < 4; ++e) mean[e] = anchor_mean_elem(acc[e], fm);
    if (ANCHOR_MOM) {
        f4 vn = v[c], zn;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float ve = vn[e];
            zn[e] = anchor_momentum_elem(mean[e], zo[e], ve, beta_z);
            vn[e] = ve;
        }
        v[c] = vn;
        z_out[c] = zn;
    } else {
        z_out[c] = mean;
    }
}

template <bool WITH_STEP, bool MOM, bool NEST>
static void spm_dispatch(const StepPullMeanArgs& a, hipStream_t s) {
    const UpdateArgs& u = a.u;
    const int64_t n4 = u.ld / 4;
    const unsigned grid = (unsigned)((n4 + kSpmThreads - 1) / kSpmThreads);
    if (a.v)
        step_pull_mean_kernel<WITH_STEP, MOM, NEST, true><<<grid, kSpmThreads, 0, s>>>(
            (const f4*)u.g, (const f4*)u.x_in, (f4*)u.x_out, (f4*)u.buf, (const f4*)u.z, (f4*)a.z_out, (f4*)a.v, u.m, n4,
            u.gamma, u.mu, u.alpha, a.beta_z);
    else
        step_pull_mean_kernel<WITH_STEP, MOM, NEST, false><<<grid, kSpmThreads, 0, s>>>(
            (const f4*)u.g, (const f4*)u.x_in, (f4*)u.x_out, (f4*)u.buf, (const f4*)u.z, (f4*)a.z_out, nullptr, u.m, n4,
            u.gamma, u.mu, u.alpha, 0.0f);
}

// Emulated communication latency ahead of the anchor refresh (the delay that Section 2, arXiv 2002.09539 argues
// is hidden as long as it is shorter than tau local steps): one wavefront sleeps until the constant-rate wall
// clock has advanced by `ticks`.  Two exit conditions, each reached by itself: the clock, and a bound on the
// number of sleep periods (one period lasts well below a microsecond at any engine clock, so `max_spins` of
// eight per requested microsecond is never the one that ends a healthy wait by much).
__global__ __launch_bounds__(64) void delay_kernel(long long ticks, long long max_spins) {
    const long long t0 = wall_clock64();
    for (long long i = 0; i < max_spins; ++i) {
        if (wall_clock64() - t0 >= ticks) break;
        __builtin_amdgcn_s_sleep(8);
    }
}

hipError_t launch_delay(int64_t microseconds, hipStream_t s) {
    if (microseconds < 1 || microseconds > 1000000) return hipErrorInvalidValue;
    int dev = 0, khz = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev);
    if (e != hipSuccess) return e;
    if (khz < 1) return hipErrorInvalidValue;
    const long long ticks = (long long)microseconds * khz / 1000;
    // s_sleep 8 idles about 512 engine clocks: at least 0.15 us between 1 and 3.4 GHz
    delay_kernel<<<1, 64, 0, s>>>(ticks, (long long)microseconds * 8 + 64);
    return hipGetLastError();
}

hipError_t launch_step_pull_mean(const StepPullMeanArgs& a, hipStream_t s) {
    const UpdateArgs& u = a.u;
    if (u.m < 1 || u.ld < 4 || u.ld % 4 != 0 || !u.x_in || !u.x_out || !u.z || !a.z_out) return hipErrorInvalidValue;
    if (a.with_step && (!u.g || (u.mu != 0.0f && !u.buf))) return hipErrorInvalidValue;
    if (u.shadow) return hipErrorInvalidValue;  // the bf16 shadow is written by the row-wise kernels only
    if (!a.with_step) spm_dispatch<false, false, false>(a, s);
    else if (u.mu == 0.0f) spm_dispatch<true, false, false>(a, s);
    else if (u.nesterov) spm_dispatch<true, true, true>(a, s);
    else spm_dispatch<true, true, false>(a, s);
    return hipGetLastError();
}

}  // namespace ols
