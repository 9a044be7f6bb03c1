// Batch normalisation of the residual block's convolution outputs (training mode: statistics of the worker's own
// mini-batch, per channel over all samples and positions), forward and backward, grouped over the m workers.  Part of
// the model that produces the stochastic gradients g_i of Section 2, arXiv 2002.09539 (Section 4 trains a residual
// network, whose blocks normalise every convolution).
//
//   forward    mean_c, var_c over the P = B H W pixels;  inv_std_c = 1 / sqrt(var_c + eps)
//              out = act( gamma_c (z - mean_c) inv_std_c + beta_c (+ shortcut) )
//   backward   s1_c = sum_p dy,  s2_c = sum_p dy xhat   (= d beta, d gamma)
//              dz = gamma_c inv_std_c (dy - s1_c / P - xhat s2_c / P)
//
// All four passes are HBM-bound streaming kernels over [group][P][C] tensors (channel contiguous, 16-byte vectors).
// Reductions are deterministic: every workgroup reduces a contiguous pixel range in a fixed order, a second launch
// combines the ranges in range order (no atomics).  The statistics use shifted sums -- each range subtracts the value of
// its own first pixel before summing and squaring -- and the ranges are merged with the pairwise update of mean and
// second moment, so nothing cancels when a channel's mean is large against its spread.
// Options that take tensor passes out of the block: the statistics can be merged from per-wavefront parts that the
// producing convolution left (z is then read once, not twice); the second normalisation can be the block's tail (sign
// bytes and 64-pixel partial sums of the pooling instead of the stored activation); its backward pass can form the
// gradient under pooling and ReLU on the fly from the pooled gradient and those sign bytes; and a result that becomes a
// bf16 convolution's operand can be written as bf16 straight into that operand's padded layout.
// Measured and not kept: four vectors per lane in the two apply kernels (150 / 190 / 225 us either way); eight channels
// per lane with one 16-byte store of the bf16 result instead of 8-byte stores (the backward apply kernels 10 us slower
// each); the first
// normalisation's backward sums formed in the epilogue of the delta convolution that produces its gradient (the
// convolution grows by the 86 us that the saved pass over gradient and input took beyond its own share).
#include "fast_div.h"
#include "gemm_bf16_tile.h"
#include "ols_internal.h"

namespace ols {

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;

// pixel ranges per group: about 2048 pixels each, at most 256
__host__ __device__ inline int bn_ranges(int P) {
    int r = (P + 2047) / 2048;
    return r < 1 ? 1 : (r > 256 ? 256 : r);
}

// Sums over the stripes of a workgroup, in stripe order; result valid for stripe 0.
__device__ __forceinline__ f4 reduce_stripes(f4 v, f4* lds, int c4n, int stripes) {
    lds[threadIdx.x] = v;
    __syncthreads();
    f4 acc = v;
    if ((int)threadIdx.x < c4n)
        for (int s = 1; s < stripes; ++s) acc = acc + lds[s * c4n + threadIdx.x];
    __syncthreads();
    return acc;
}

// part[group][range][3][C]: shift K (the range's first pixel), sum (z - K), sum (z - K)^2
__global__ __launch_bounds__(kThreads) void bn_stats_partial_kernel(const float* __restrict__ z, int64_t s_z, float* part,
                                                                    int P, int C, int ranges) {
    __shared__ f4 lds[kThreads];
    const int c4n = C / 4, stripes = kThreads / c4n;
    const int c4 = threadIdx.x % c4n, stripe = threadIdx.x / c4n;
    const int g = blockIdx.y, r = blockIdx.x;
    const int chunk = (P + ranges - 1) / ranges;
    const int p_lo = r * chunk, p_hi = min(P, p_lo + chunk);
    const float* Z = z + (int64_t)g * s_z;
    f4 K = {0.f, 0.f, 0.f, 0.f}, s1 = K, s2 = K;
    if (p_lo < p_hi && stripe < stripes) {
        K = *(const f4*)(Z + (int64_t)p_lo * C + 4 * c4);
#pragma unroll 4
        for (int p = p_lo + stripe; p < p_hi; p += stripes) {
            const f4 v = __builtin_nontemporal_load((const f4*)(Z + (int64_t)p * C + 4 * c4)) - K;
            s1 = s1 + v;
            s2 = s2 + v * v;
        }
    }
    s1 = reduce_stripes(s1, lds, c4n, stripes);
    s2 = reduce_stripes(s2, lds, c4n, stripes);
    if ((int)threadIdx.x < c4n) {
        float* o = part + (((int64_t)g * ranges + r) * 3) * C + 4 * c4;
        *(f4*)o = K;
        *(f4*)(o + C) = s1;
        *(f4*)(o + 2 * C) = s2;
    }
}

// stats[group][2][C]: mean, 1 / sqrt(var + eps); the ranges are merged in range order
__global__ __launch_bounds__(kThreads) void bn_stats_final_kernel(const float* __restrict__ part, float* stats, int P, int C,
                                                                  int ranges, float eps) {
    const int c = blockIdx.x * kThreads + threadIdx.x;
    if (c >= C) return;
    const int g = blockIdx.y;
    const int chunk = (P + ranges - 1) / ranges;
    const int filled = (P + chunk - 1) / chunk;   // ranges that hold pixels (the last ones may be empty)
    float n = 0.0f, mean = 0.0f, m2 = 0.0f;
#pragma unroll 8
    for (int r = 0; r < filled; ++r) {   // the loads do not depend on the running merge and are issued ahead of it
        const int p_lo = r * chunk, p_hi = min(P, p_lo + chunk);
        const float nr = (float)(p_hi - p_lo);
        const float* o = part + (((int64_t)g * ranges + r) * 3) * C + c;
        const float K = o[0], s1 = o[C], s2 = o[2 * C];
        const float mean_r = K + s1 / nr;
        const float m2_r = s2 - s1 * (s1 / nr);
        const float tot = n + nr, delta = mean_r - mean;
        mean = mean + delta * (nr / tot);
        m2 = m2 + m2_r + delta * delta * (n * (nr / tot));
        n = tot;
    }
    const float var = fmaxf(m2 / n, 0.0f);
    stats[((int64_t)g * 2) * C + c] = mean;
    stats[((int64_t)g * 2 + 1) * C + c] = 1.0f / sqrtf(var + eps);
}

// The same statistics from per-wavefront parts that a convolution's epilogue left: wpart[group][w][3][C] = count, mean
// and sum of squared deviations of the image pixels among 64 consecutive padded pixels (count 0: none), merged by the
// parallel-variance rule in a fixed order.  Two levels: a workgroup takes one of up to sixteen contiguous chunks of a
// group's parts and 64 channels (a part's 64 counts, means or sums are one 256-byte run); each of its four stripes
// merges every fourth part of the chunk in order, twelve parts requested at a time (the merge is a dependent chain, the
// loads are not), and stripe 0 merges the four results in stripe order into cpart[group][chunk][3][C].  The second
// launch merges a channel's chunks in chunk order.  (One level with 8 channels x 32 stripes per workgroup took 27 us at
// the benchmark shape -- every workgroup touched all of a group's cache lines for an eighth of their bytes; with 4 x 64
// 40 us.  The two levels take 10 + 5 us; 32 or 16 channels per workgroup and 10 - 19 parts in flight change nothing.)
constexpr int kWaveStatChunks = 16, kWaveStatChannels = 64, kWaveStatStripes = kThreads / kWaveStatChannels, kWaveStatBatch = 12;
__host__ __device__ inline int wave_stat_chunks(int P) { const int r = bn_ranges(P); return r < kWaveStatChunks ? r : kWaveStatChunks; }

__device__ __forceinline__ void merge_moments(float& n, float& mean, float& m2, float nr, float mean_r, float m2_r) {
    if (nr > 0.0f) {
        const float tot = n + nr, delta = mean_r - mean;
        mean = mean + delta * (nr / tot);
        m2 = m2 + m2_r + delta * delta * (n * (nr / tot));
        n = tot;
    }
}

// grid (chunks, groups, C / 64)
__global__ __launch_bounds__(kThreads) void bn_stats_waves_kernel(const float* __restrict__ wpart, int64_t s_wpart, float* cpart,
                                                                  int C, int waves, int chunks) {
    __shared__ float lds[3][kThreads];
    const int cl = threadIdx.x % kWaveStatChannels, stripe = threadIdx.x / kWaveStatChannels;
    const int c = blockIdx.z * kWaveStatChannels + cl, g = blockIdx.y, k = blockIdx.x;
    const int per = (waves + chunks - 1) / chunks;
    const int lo = k * per, hi = min(waves, lo + per);
    float n = 0.0f, mean = 0.0f, m2 = 0.0f;
    const float* P = wpart + (int64_t)g * s_wpart + c;
    for (int w0 = lo + stripe; w0 < hi; w0 += kWaveStatStripes * kWaveStatBatch) {
        float nr[kWaveStatBatch], mr[kWaveStatBatch], qr[kWaveStatBatch];
#pragma unroll
        for (int u = 0; u < kWaveStatBatch; ++u) {
            const int w = w0 + u * kWaveStatStripes;
            const float* o = P + (int64_t)(w < hi ? w : lo) * 3 * C;   // past the chunk: an in-range part, not merged
            nr[u] = w < hi ? o[0] : 0.0f;
            mr[u] = o[C];
            qr[u] = o[2 * C];
        }
#pragma unroll
        for (int u = 0; u < kWaveStatBatch; ++u) merge_moments(n, mean, m2, nr[u], mr[u], qr[u]);
    }
    lds[0][threadIdx.x] = n;
    lds[1][threadIdx.x] = mean;
    lds[2][threadIdx.x] = m2;
    __syncthreads();
    if (stripe == 0) {
        for (int s = 1; s < kWaveStatStripes; ++s)
            merge_moments(n, mean, m2, lds[0][s * kWaveStatChannels + cl], lds[1][s * kWaveStatChannels + cl], lds[2][s * kWaveStatChannels + cl]);
        float* o = cpart + (((int64_t)g * chunks + k) * 3) * C + c;
        o[0] = n;
        o[C] = mean;
        o[2 * C] = m2;
    }
}

// grid (ceil(C / 256), groups): one lane per channel merges its chunks in chunk order
__global__ __launch_bounds__(kThreads) void bn_stats_chunks_kernel(const float* __restrict__ cpart, float* stats, int C, int chunks, float eps) {
    const int c = blockIdx.x * kThreads + threadIdx.x, g = blockIdx.y;
    if (c >= C) return;
    float n = 0.0f, mean = 0.0f, m2 = 0.0f;
    const float* P = cpart + (int64_t)g * chunks * 3 * C + c;
    float nr[kWaveStatChunks], mr[kWaveStatChunks], qr[kWaveStatChunks];
#pragma unroll
    for (int k = 0; k < kWaveStatChunks; ++k) {   // all loads first: only the merge is a dependent chain
        const float* o = P + (int64_t)(k < chunks ? k : 0) * 3 * C;
        nr[k] = k < chunks ? o[0] : 0.0f;
        mr[k] = o[C];
        qr[k] = o[2 * C];
    }
#pragma unroll
    for (int k = 0; k < kWaveStatChunks; ++k) merge_moments(n, mean, m2, nr[k], mr[k], qr[k]);
    const float var = fmaxf(m2 / n, 0.0f);
    stats[((int64_t)g * 2) * C + c] = mean;
    stats[((int64_t)g * 2 + 1) * C + c] = 1.0f / sqrtf(var + eps);
}

// Where a result becomes the operand of a bf16 convolution it is written as bf16 (to nearest even) into that operand's
// layout: [B (H + 2) (W + 2)][C] with a border that nobody writes (it is zero from the start).  Vector v = four channels
// of the unpadded pixel v / (C / 4).
struct PaddedOut {
    uint16_t* base;          // nullptr: the fp32 output is written instead
    int64_t stride;          // per group, bf16 elements
    FastDiv div_hw, div_w;
    int H, W;
};
__device__ __forceinline__ void store_padded_bf16(const PaddedOut& po, int g, unsigned pix, unsigned c4, int C, f4 o) {
    const unsigned n = fast_div(pix, po.div_hw), rem = pix - n * (unsigned)(po.H * po.W);
    const unsigned y = fast_div(rem, po.div_w), x = rem - y * (unsigned)po.W;
    const int64_t q = ((int64_t)n * (po.H + 2) + y + 1) * (po.W + 2) + x + 1;
    u2 w;   // v_cvt_pk_bf16_f32
    w.x = __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{o[0], o[1]}, bf16x2));
    w.y = __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{o[2], o[3]}, bf16x2));
    *(u2*)(po.base + (int64_t)g * po.stride + q * C + 4 * c4) = w;
}

// out = act(gamma (z - mean) inv_std + beta (+ shortcut))
__global__ __launch_bounds__(kThreads) void bn_apply_kernel(const float* __restrict__ z, int64_t s_z,
                                                            const float* __restrict__ stats, const float* __restrict__ gamma,
                                                            const float* __restrict__ beta, int64_t s_par,
                                                            const float* __restrict__ shortcut, int64_t s_sc, float* out,
                                                            int64_t s_out, unsigned vecs, int C, int relu, FastDiv div_c4,
                                                            PaddedOut po) {
    const unsigned v = blockIdx.x * kThreads + threadIdx.x;
    if (v >= vecs) return;
    const int g = blockIdx.y;
    const unsigned pixel = fast_div(v, div_c4);
    const int c = 4 * (int)(v - pixel * (unsigned)(C / 4));
    const f4 mean = *(const f4*)(stats + ((int64_t)g * 2) * C + c);
    const f4 istd = *(const f4*)(stats + ((int64_t)g * 2 + 1) * C + c);
    const f4 ga = *(const f4*)(gamma + (int64_t)g * s_par + c);
    const f4 be = *(const f4*)(beta + (int64_t)g * s_par + c);
    const f4 zv = __builtin_nontemporal_load((const f4*)(z + (int64_t)g * s_z) + v);
    f4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = __fmaf_rn(ga[e], (zv[e] - mean[e]) * istd[e], be[e]);
    if (shortcut) o = o + __builtin_nontemporal_load((const f4*)(shortcut + (int64_t)g * s_sc) + v);
    if (relu) {
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = fmaxf(o[e], 0.0f);
    }
    if (po.base) store_padded_bf16(po, g, pixel, c / 4, C, o);
    else *((f4*)(out + (int64_t)g * s_out) + v) = o;
}

// The block's tail in the normalisation: a = relu(gamma (z - mean) inv_std + beta + shortcut) is not stored -- its sign
// bytes and its channel sums per 64 consecutive pixels are (two slots per part: the sample of the part's first pixel and
// the next one; H W >= 64, so there is no third).  A workgroup owns 64 pixels: lane = (channel quad, stripe), four
// pixels per lane in flight, stripes combined in stripe order.
constexpr int kTailPixels = 64;
__global__ __launch_bounds__(kThreads) void bn_tail_kernel(const float* __restrict__ z, int64_t s_z, const float* __restrict__ stats,
                                                           const float* __restrict__ gamma, const float* __restrict__ beta,
                                                           int64_t s_par, const float* __restrict__ shortcut, int64_t s_sc,
                                                           uint8_t* sign, int64_t s_sign, float* pool_part, int P, int C, int relu,
                                                           int per, FastDiv div_per) {
    __shared__ f4 lds[kThreads];
    const int c4n = C / 4, stripes = kThreads / c4n;
    const int c4 = threadIdx.x % c4n, stripe = threadIdx.x / c4n;
    const int g = blockIdx.y, w = blockIdx.x;
    const int p0 = w * kTailPixels;
    const int next_sample = ((int)fast_div((unsigned)p0, div_per) + 1) * per;   // first pixel of the second slot's sample
    f4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0;
    if (stripe < stripes) {
        const f4 mean = *(const f4*)(stats + ((int64_t)g * 2) * C + 4 * c4);
        const f4 istd = *(const f4*)(stats + ((int64_t)g * 2 + 1) * C + 4 * c4);
        const f4 ga = *(const f4*)(gamma + (int64_t)g * s_par + 4 * c4);
        const f4 be = *(const f4*)(beta + (int64_t)g * s_par + 4 * c4);
        const float* Z = z + (int64_t)g * s_z + 4 * c4;
        const float* S = shortcut ? shortcut + (int64_t)g * s_sc + 4 * c4 : nullptr;
        uint8_t* SG = sign + (int64_t)g * s_sign + c4;
        for (int q0 = stripe; q0 < kTailPixels; q0 += 4 * stripes) {
            f4 zv[4], sv[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int p = p0 + q0 + t * stripes;
                const bool in = q0 + t * stripes < kTailPixels && p < P;
                zv[t] = in ? __builtin_nontemporal_load((const f4*)(Z + (int64_t)p * C)) : f4{0.f, 0.f, 0.f, 0.f};
                sv[t] = in && S ? __builtin_nontemporal_load((const f4*)(S + (int64_t)p * C)) : f4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int p = p0 + q0 + t * stripes;
                if (q0 + t * stripes >= kTailPixels || p >= P) continue;
                f4 o;
                unsigned bits = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    o[e] = __fmaf_rn(ga[e], (zv[t][e] - mean[e]) * istd[e], be[e]) + sv[t][e];
                    if (relu) o[e] = fmaxf(o[e], 0.0f);
                    bits |= o[e] > 0.0f ? (1u << e) : 0u;
                }
                SG[(int64_t)p * c4n] = (uint8_t)bits;
                if (p < next_sample) s0 = s0 + o; else s1 = s1 + o;
            }
        }
    }
    s0 = reduce_stripes(s0, lds, c4n, stripes);
    s1 = reduce_stripes(s1, lds, c4n, stripes);
    if ((int)threadIdx.x < c4n) {
        float* o = pool_part + (((int64_t)g * gridDim.x + w) * 2) * C + 4 * c4;
        *(f4*)o = s0;
        *(f4*)(o + C) = s1;
    }
}

// The gradient at a normalised output that sits under global average pooling and a ReLU need not be stored: it is
// dpool[sample][c] * scale where the activation is positive, else 0 -- formed here from the activation and the pooled
// gradient wherever the backward kernels would read dy.
struct PooledDelta {
    const float* gate;       // the activation, or
    const uint8_t* sign;     // one byte per pixel and four channels, bit e set iff it is positive; both nullptr: dy is read
    const float* dpool;      // [group][sample][C]
    int64_t s_gate, s_dp;
    float scale;             // 1 / positions
    FastDiv div_pos;         // pixel -> sample
};
// Where the backward kernels take the gradient at the normalised output from (a template parameter: a branch inside
// their loops would serialise the loads of one pixel behind the other's)
enum { kFromDy = 0, kFromGate = 1, kFromSign = 2 };
template <int SRC>
__device__ __forceinline__ f4 delta_at(const float* __restrict__ D, const PooledDelta& pd, int g, unsigned pixel, int C, int c4) {
    if constexpr (SRC == kFromDy) {
        return __builtin_nontemporal_load((const f4*)(D + (int64_t)pixel * C + 4 * c4));
    } else {
        const f4 d = *(const f4*)(pd.dpool + (int64_t)g * pd.s_dp + (int64_t)fast_div(pixel, pd.div_pos) * C + 4 * c4);
        f4 o;
        if constexpr (SRC == kFromSign) {
            const unsigned bits = pd.sign[(int64_t)g * pd.s_gate + (int64_t)pixel * (C / 4) + c4];
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bits >> e) & 1u ? d[e] * pd.scale : 0.0f;
        } else {
            const f4 a = __builtin_nontemporal_load((const f4*)(pd.gate + (int64_t)g * pd.s_gate + (int64_t)pixel * C + 4 * c4));
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = a[e] > 0.0f ? d[e] * pd.scale : 0.0f;
        }
        return o;
    }
}

// part[group][range][2][C]: sum dy, sum dy xhat over the range
template <int SRC>
__global__ __launch_bounds__(kThreads) void bn_bwd_partial_kernel(const float* __restrict__ dy, int64_t s_dy,
                                                                  const float* __restrict__ z, int64_t s_z,
                                                                  const float* __restrict__ stats, float* part, int P, int C,
                                                                  int ranges, PooledDelta pd) {
    __shared__ f4 lds[kThreads];
    const int c4n = C / 4, stripes = kThreads / c4n;
    const int c4 = threadIdx.x % c4n, stripe = threadIdx.x / c4n;
    const int g = blockIdx.y, r = blockIdx.x;
    const int chunk = (P + ranges - 1) / ranges;
    const int p_lo = r * chunk, p_hi = min(P, p_lo + chunk);
    const float* Z = z + (int64_t)g * s_z;
    const float* D = dy + (int64_t)g * s_dy;
    f4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = s1;
    if (stripe < stripes) {
        const f4 mean = *(const f4*)(stats + ((int64_t)g * 2) * C + 4 * c4);
        const f4 istd = *(const f4*)(stats + ((int64_t)g * 2 + 1) * C + 4 * c4);
        for (int p0 = p_lo + stripe; p0 < p_hi; p0 += 4 * stripes) {   // four pixels per lane in flight
            f4 d[4], zv[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int p = p0 + t * stripes;
                const unsigned pc = (unsigned)(p < p_hi ? p : p0);       // a lane past the range re-reads its first pixel
                d[t] = delta_at<SRC>(D, pd, g, pc, C, c4);
                zv[t] = __builtin_nontemporal_load((const f4*)(Z + (int64_t)pc * C + 4 * c4));
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (p0 + t * stripes >= p_hi) continue;
                s1 = s1 + d[t];
                s2 = s2 + d[t] * ((zv[t] - mean) * istd);
            }
        }
    }
    s1 = reduce_stripes(s1, lds, c4n, stripes);
    s2 = reduce_stripes(s2, lds, c4n, stripes);
    if ((int)threadIdx.x < c4n) {
        float* o = part + (((int64_t)g * ranges + r) * 2) * C + 4 * c4;
        *(f4*)o = s1;
        *(f4*)(o + C) = s2;
    }
}

// sums[group][2][C] = the ranges' sums added in range order; d beta = sums[0], d gamma = sums[1] go to the gradient rows
__global__ __launch_bounds__(kThreads) void bn_bwd_final_kernel(const float* __restrict__ part, float* sums, float* g_out,
                                                                int64_t ld, int64_t gamma_off, int64_t beta_off, int C,
                                                                int ranges) {
    const int c = blockIdx.x * kThreads + threadIdx.x;
    if (c >= C) return;
    const int g = blockIdx.y;
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll 8
    for (int r = 0; r < ranges; ++r) {
        const float* o = part + (((int64_t)g * ranges + r) * 2) * C + c;
        s1 += o[0];
        s2 += o[C];
    }
    sums[((int64_t)g * 2) * C + c] = s1;
    sums[((int64_t)g * 2 + 1) * C + c] = s2;
    g_out[(int64_t)g * ld + beta_off + c] = s1;
    g_out[(int64_t)g * ld + gamma_off + c] = s2;
}

// dz = gamma inv_std (dy - s1 / P - xhat s2 / P), written over dy -- or as a bf16 operand (see PaddedOut)
template <int SRC>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_kernel(float* dy, int64_t s_dy, const float* __restrict__ z,
                                                                int64_t s_z, const float* __restrict__ stats,
                                                                const float* __restrict__ sums,
                                                                const float* __restrict__ gamma, int64_t s_par, unsigned vecs,
                                                                int C, float inv_count, FastDiv div_c4, PaddedOut po, PooledDelta pd) {
    const unsigned v = blockIdx.x * kThreads + threadIdx.x;
    if (v >= vecs) return;
    const int g = blockIdx.y;
    const unsigned pixel = fast_div(v, div_c4);
    const int c = 4 * (int)(v - pixel * (unsigned)(C / 4));
    const f4 mean = *(const f4*)(stats + ((int64_t)g * 2) * C + c);
    const f4 istd = *(const f4*)(stats + ((int64_t)g * 2 + 1) * C + c);
    const f4 s1 = *(const f4*)(sums + ((int64_t)g * 2) * C + c);
    const f4 s2 = *(const f4*)(sums + ((int64_t)g * 2 + 1) * C + c);
    const f4 ga = *(const f4*)(gamma + (int64_t)g * s_par + c);
    f4* D = (f4*)(dy + (int64_t)g * s_dy) + v;
    const f4 d = delta_at<SRC>(dy + (int64_t)g * s_dy, pd, g, pixel, C, c / 4);
    const f4 xh = (__builtin_nontemporal_load((const f4*)(z + (int64_t)g * s_z) + v) - mean) * istd;
    f4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = ga[e] * istd[e] * (d[e] - s1[e] * inv_count - xh[e] * (s2[e] * inv_count));
    if (po.base) store_padded_bf16(po, g, pixel, c / 4, C, o);   // dy itself stays as it was
    else *D = o;
}

bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

bool shape_ok(int groups, int P, int C) { return groups >= 1 && groups <= 65535 && P >= 1 && C >= 4 && C % 4 == 0 && C <= 1024; }

// the optional bf16 output in the padded operand layout: P = B H W pixels, 8-byte stores, 31-bit vector indices
bool padded_out(const BnArgs& a, int64_t vecs, PaddedOut* po) {
    if (!a.out_bf16) return true;
    if (a.H < 1 || a.W < 1 || a.P % (a.H * a.W) != 0 || (reinterpret_cast<uintptr_t>(a.out_bf16) & 7u) || a.s_outb % 4 ||
        vecs >= ((int64_t)1 << 31) - kThreads)
        return false;
    po->base = a.out_bf16; po->stride = a.s_outb; po->H = a.H; po->W = a.W;
    po->div_hw = make_div((unsigned)(a.H * a.W)); po->div_w = make_div((unsigned)a.W);
    return true;
}

bool vec_grid(int64_t vecs, unsigned* blocks) {   // 31-bit vector indices (the kernels divide them by multiplication)
    const int64_t b = (vecs + kThreads - 1) / kThreads;
    if (b < 1 || vecs >= ((int64_t)1 << 31) - kThreads) return false;
    *blocks = (unsigned)b;
    return true;
}

}  // namespace

int64_t bn_partial_floats(int groups, int P, int C) { return (int64_t)groups * bn_ranges(P) * 3 * C; }

hipError_t launch_bn_forward(const BnArgs& a, hipStream_t s) {
    if (!shape_ok(a.groups, a.P, a.C) || !a.z || (!a.out && !a.out_bf16 && !a.pool_part) || !a.stats || !a.part || !a.gamma || !a.beta) return hipErrorInvalidValue;
    if (!aligned16(a.z) || !aligned16(a.out) || !aligned16(a.stats) || !aligned16(a.part) || !aligned16(a.gamma) ||
        !aligned16(a.beta) || !aligned16(a.shortcut) || a.s_z % 4 || a.s_out % 4 || a.s_par % 4 || a.s_sc % 4)
        return hipErrorInvalidValue;
    hipError_t e;
    if (a.wave_part) {   // the producer of z left per-wavefront statistics: z is not read for them
        if (a.waves < 1 || !aligned16(a.wave_part) || a.C % kWaveStatChannels) return hipErrorInvalidValue;
        const int chunks = wave_stat_chunks(a.P);   // their results fit the ranges' buffer: chunks <= bn_ranges(P)
        bn_stats_waves_kernel<<<dim3((unsigned)chunks, (unsigned)a.groups, (unsigned)(a.C / kWaveStatChannels)), kThreads, 0, s>>>(
            a.wave_part, (int64_t)a.waves * 3 * a.C, a.part, a.C, a.waves, chunks);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        bn_stats_chunks_kernel<<<dim3((unsigned)((a.C + kThreads - 1) / kThreads), (unsigned)a.groups), kThreads, 0, s>>>(a.part, a.stats, a.C, chunks, a.eps);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    } else {
        const int ranges = bn_ranges(a.P);
        bn_stats_partial_kernel<<<dim3((unsigned)ranges, (unsigned)a.groups), kThreads, 0, s>>>(a.z, a.s_z, a.part, a.P, a.C, ranges);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        bn_stats_final_kernel<<<dim3((unsigned)((a.C + kThreads - 1) / kThreads), (unsigned)a.groups), kThreads, 0, s>>>(
            a.part, a.stats, a.P, a.C, ranges, a.eps);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (a.pool_part) {   // the block's tail: sign bytes and partial sums instead of the activation
        if (!a.sign || a.positions < kTailPixels || a.P % a.positions != 0 || !aligned16(a.pool_part) || a.C > 4 * kThreads) return hipErrorInvalidValue;
        bn_tail_kernel<<<dim3((unsigned)((a.P + kTailPixels - 1) / kTailPixels), (unsigned)a.groups), kThreads, 0, s>>>(
            a.z, a.s_z, a.stats, a.gamma, a.beta, a.s_par, a.shortcut, a.s_sc, a.sign, a.s_sign, a.pool_part, a.P, a.C, a.relu, a.positions,
            make_div((unsigned)a.positions));
        return hipGetLastError();
    }
    unsigned blocks;
    const int64_t vecs = (int64_t)a.P * (a.C / 4);
    if (!vec_grid(vecs, &blocks)) return hipErrorInvalidValue;
    PaddedOut po = {};
    if (!padded_out(a, vecs, &po)) return hipErrorInvalidValue;
    bn_apply_kernel<<<dim3(blocks, (unsigned)a.groups), kThreads, 0, s>>>(a.z, a.s_z, a.stats, a.gamma, a.beta, a.s_par, a.shortcut,
                                                                          a.s_sc, a.out, a.s_out, (unsigned)vecs, a.C, a.relu, make_div((unsigned)(a.C / 4)), po);
    return hipGetLastError();
}

hipError_t launch_bn_backward(const BnArgs& a, hipStream_t s) {
    if (!shape_ok(a.groups, a.P, a.C) || !a.z || (!a.dy && !((a.gate || a.sign) && a.out_bf16)) || !a.stats || !a.part || !a.sums || !a.gamma || !a.g) return hipErrorInvalidValue;
    if (!aligned16(a.z) || !aligned16(a.dy) || !aligned16(a.stats) || !aligned16(a.part) || !aligned16(a.sums) ||
        !aligned16(a.gamma) || a.s_z % 4 || a.s_dy % 4 || a.s_par % 4)
        return hipErrorInvalidValue;
    const int ranges = bn_ranges(a.P);
    PooledDelta pd = {};
    if (a.gate || a.sign) {
        if (!a.dpool || a.positions < 1 || a.P % a.positions != 0 || !aligned16(a.gate) || !aligned16(a.dpool) || a.s_gate % 4 || a.s_dp % 4)
            return hipErrorInvalidValue;
        if (a.sign) { pd.sign = a.sign; pd.s_gate = a.s_sign; } else { pd.gate = a.gate; pd.s_gate = a.s_gate; }
        pd.dpool = a.dpool; pd.s_dp = a.s_dp;
        pd.scale = 1.0f / (float)a.positions;
        pd.div_pos = make_div((unsigned)a.positions);
    }
    const int src = a.sign ? kFromSign : a.gate ? kFromGate : kFromDy;
    auto partial = src == kFromSign ? bn_bwd_partial_kernel<kFromSign> : src == kFromGate ? bn_bwd_partial_kernel<kFromGate> : bn_bwd_partial_kernel<kFromDy>;
    auto apply = src == kFromSign ? bn_bwd_apply_kernel<kFromSign> : src == kFromGate ? bn_bwd_apply_kernel<kFromGate> : bn_bwd_apply_kernel<kFromDy>;
    partial<<<dim3((unsigned)ranges, (unsigned)a.groups), kThreads, 0, s>>>(a.dy, a.s_dy, a.z, a.s_z, a.stats, a.part, a.P, a.C, ranges, pd);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    bn_bwd_final_kernel<<<dim3((unsigned)((a.C + kThreads - 1) / kThreads), (unsigned)a.groups), kThreads, 0, s>>>(
        a.part, a.sums, a.g, a.ld, a.g_gamma_off, a.g_beta_off, a.C, ranges);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    unsigned blocks;
    const int64_t vecs = (int64_t)a.P * (a.C / 4);
    if (!vec_grid(vecs, &blocks)) return hipErrorInvalidValue;
    PaddedOut po = {};
    if (!padded_out(a, vecs, &po)) return hipErrorInvalidValue;
    apply<<<dim3(blocks, (unsigned)a.groups), kThreads, 0, s>>>(a.dy, a.s_dy, a.z, a.s_z, a.stats, a.sums, a.gamma, a.s_par, (unsigned)vecs, a.C,
                                                                1.0f / (float)a.P, make_div((unsigned)(a.C / 4)), po, pd);
    return hipGetLastError();
}

}  // namespace ols
