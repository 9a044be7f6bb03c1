// General mixing step of the matrix-form update rule (Section 2, "Matrix-Form Update Rule", arXiv
// 2002.09539): with X = [x^(1), ..., x^(m), z] of shape d x (m + 1),
//
//     X <- X W        for a caller-given (m + 1) x (m + 1) matrix W (column j holds the weights of output j)
//
// The paper's own synchronisation step is the W printed there; the section remarks that the analysis
// extends to other column-stochastic matrices (periodic averaging, symmetric elastic mixing, ...), and this
// kernel applies any of them in ONE pass over HBM: every lane owns a parameter column across all m + 1
// rows, reads each row once into registers, and writes each output row once, so the traffic is
// 8 (m + 1) bytes per parameter (+ 2 m bytes for the bf16 shadow) against 2 (m + 1)^2 flops -- bound by
// HBM for the replica counts of interest.  Output j is the fixed-order fma chain
// sum_{i = 0..m} W[i][j] x_i.  In place: all inputs of a lane are in registers before its first store.
//
// The loop over outputs is rolled, the loop over inputs is unrolled so that the inputs stay in registers;
// the weights come from a transposed copy of W in LDS (one broadcast 16-byte read per four inputs).  MR bounds
// the rows, V is the floats per lane (16, 8 or 4 bytes: narrower lanes for more replicas keep the register
// count bounded).  The padding rows carry zero weights and zero inputs: fma(0, 0, s) = s leaves every sum as
// the chain over the real rows.  Beyond about 32 replicas the 2 (m + 1)^2 flops per parameter outweigh the
// 8 (m + 1) bytes and the kernel is bound by the vector ALUs instead.
#include "ols_internal.h"

namespace ols {


template <int V> struct Vec;
template <> struct Vec<4> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct Vec<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct Vec<1> { typedef float type; };

__device__ __forceinline__ unsigned int mix_bf16(float f) { return bf16_bits_rne(f); }
template <int V> __device__ __forceinline__ float vget(const typename Vec<V>::type& v, int e) { return v[e]; }
template <> __device__ __forceinline__ float vget<1>(const float& v, int) { return v; }
template <int V> __device__ __forceinline__ void vset(typename Vec<V>::type& v, int e, float f) { v[e] = f; }
template <> __device__ __forceinline__ void vset<1>(float& v, int, float f) { v = f; }

template <int MR, int V, int kThreads>
__global__ __launch_bounds__(kThreads) void mix_kernel(float* x, float* z, uint16_t* shadow, const float* __restrict__ W,
                                                       int rows, int64_t ld) {
    typedef typename Vec<V>::type vec;
    typedef float f4 __attribute__((ext_vector_type(4)));
    constexpr int RP = (MR + 3) / 4 * 4;   // padded row count: weights are read four inputs at a time
    // W transposed into LDS, zero beyond `rows`: s_wt[j][i] = W[i][j], so the weights of output j are
    // contiguous and every lane reads the same 16 bytes (an LDS broadcast) per four inputs.
    __shared__ __attribute__((aligned(16))) float s_wt[MR * RP];
    for (int t = threadIdx.x; t < MR * RP; t += kThreads) {
        const int j = t / RP, i = t % RP;
        s_wt[t] = (i < rows && j < rows) ? W[i * rows + j] : 0.0f;
    }
    const int64_t c = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * V;   // first column of this lane
    const bool live = c < ld;   // ld is a multiple of 64
    const int m = rows - 1;
    vec in[RP];
#pragma unroll
    for (int i = 0; i < RP; ++i) {
#pragma unroll
        for (int e = 0; e < V; ++e) vset<V>(in[i], e, 0.0f);
        if (live && i < rows) {
            const float* src = i < m ? x + (int64_t)i * ld + c : z + c;
            in[i] = __builtin_nontemporal_load((const vec*)src);
        }
    }
    __syncthreads();
    if (!live) return;
#pragma unroll 1
    for (int j = 0; j < rows; ++j) {
        vec out;
#pragma unroll
        for (int e = 0; e < V; ++e) vset<V>(out, e, 0.0f);
#pragma unroll
        for (int i4 = 0; i4 < RP / 4; ++i4) {
            const f4 w = *(const f4*)(s_wt + j * RP + 4 * i4);   // zero weights beyond the last row
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < V; ++e)
                    vset<V>(out, e, __fmaf_rn(w[q], vget<V>(in[4 * i4 + q], e), vget<V>(out, e)));
        }
        float* dst = j < m ? x + (int64_t)j * ld + c : z + c;
        __builtin_nontemporal_store(out, (vec*)dst);
        if (shadow && j < m) {
#pragma unroll
            for (int e = 0; e < V; ++e) shadow[(int64_t)j * ld + c + e] = (uint16_t)mix_bf16(vget<V>(out, e));
        }
    }
}

// Workgroup size: single-wavefront workgroups stream best while the per-workgroup staging of W is small
// (m = 16, d = 11.2 M: 266 us against 277 us with 256 threads); with 65 rows the staging dominates and 256
// threads win (462 us against 579 us).
template <int MR, int V, int kThreads>
static hipError_t mix_launch(const MixArgs& a, hipStream_t s) {
    const int64_t lanes = a.ld / V;
    const int64_t blocks = (lanes + kThreads - 1) / kThreads;
    if (blocks < 1 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    mix_kernel<MR, V, kThreads><<<(unsigned)blocks, kThreads, 0, s>>>(a.x, a.z, a.shadow, a.w, a.m + 1, a.ld);
    return hipGetLastError();
}

hipError_t launch_mix(const MixArgs& a, hipStream_t s) {
    if (!a.x || !a.z || !a.w || a.m < 1 || a.m > kMixMaxWorkers || a.ld < 64 || a.ld % 64 != 0) return hipErrorInvalidValue;
    if ((reinterpret_cast<uintptr_t>(a.x) | reinterpret_cast<uintptr_t>(a.z)) & 15u) return hipErrorInvalidValue;
    const int rows = a.m + 1;
    if (rows <= 9) return mix_launch<9, 4, 64>(a, s);
    if (rows <= 17) return mix_launch<17, 4, 64>(a, s);
    if (rows <= 33) return mix_launch<33, 4, 256>(a, s);
    if (rows <= 65) return mix_launch<65, 2, 256>(a, s);
    return mix_launch<129, 1, 256>(a, s);
}

}  // namespace ols
