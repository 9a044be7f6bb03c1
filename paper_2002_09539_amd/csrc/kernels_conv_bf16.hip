// 3 x 3 convolutions (stride 1, zero padding 1) of the per-worker residual block with bf16 operands and fp32
// accumulation on the matrix cores (v_mfma_f32_32x32x16_bf16), grouped over the m workers: forward, back-propagated
// delta, kernel / bias gradient; plus the conversion of the input batch and the pooling backward that feed them.  The
// model is the first residual stage of the network of Section 4 (arXiv 2002.09539, "Experimental setting") and produces
// the stochastic gradients g_i of Section 2; every tensor is rounded to bf16 (to nearest even) where it becomes an
// operand of a convolution's products, sums and everything else stay fp32.
//
// Layout: the bf16 operand tensors are stored WITH their zero border, [group][Pp][C] with Pp = B (H + 2) (W + 2) padded
// pixels in (sample, row, column) order and the channel contiguous.  A tap (kh, kw) is then the same shift
// s = (kh - 1) (W + 2) + (kw - 1) of the pixel index for every pixel, so
//   FWD  out[q][co] = sum_{tap, ci} in[q + s_tap][ci] w[tap][ci][co]
//   DX   din[q][ci] = sum_{tap, co} dout[q - s_tap][co] w[tap][ci][co]
//   DW   dw[tap][ci][co] = sum_q in[q + s_tap][ci] dout[q][co]
// are plain GEMMs over shifted row windows with no per-pixel case analysis: interior pixels only ever reach their own
// image's border, and every producer writes zeros to the border positions (the forward epilogue explicitly, the masks of
// the backward pass by themselves, because a zero activation gates its delta).  Rows outside [0, Pp) are read as zeros.
//
// FWD / DX: one workgroup per 256 padded pixels x 64 output channels.  The input rows m0 - (W + 3) .. m0 + 256 + (W + 3)
// of a 64-channel chunk are copied to LDS ONCE (a strip, K-contiguous, pitch 64 + 8); the nine taps read their A
// fragments from it at nine row offsets, so the operand crosses the LDS write port once instead of nine times.  The
// 64 x 64 kernel slice of each tap is double-buffered through registers.  Four wavefronts of 64 x 64.
// DW: one workgroup per (pixel range, 64 x 64 block of input x output channels) holds all nine taps' accumulators
// (9 x 64 x 64 fp32 = 144 registers per lane); per 32 pixels the input strip (32 + 2 (W + 3) rows, row-contiguous,
// read with the transpose load at nine row offsets) and the delta tile pass through LDS; ranges are summed in range
// order by the finish pass shared with the fp32 kernels (no atomics).
#include <type_traits>

#include "gemm_bf16_tile.h"
#include "ols_internal.h"
#include "update_rule.h"

namespace ols {

namespace {

constexpr int kThreads = kTileThreads;
constexpr int kXcds = 8;
constexpr int kCB = 64;     // channel block: contraction chunk and output-channel tile
constexpr int kBM = 256;    // padded pixels per forward / delta tile
constexpr int kDwBK = 32;   // pixels per slice of the kernel-gradient contraction

struct ConvBDev {
    const uint16_t* in;      // FWD: layer input; DX: delta of the layer output; DW: layer input   [groups][Pp][C] bf16
    const uint16_t* w;       // FWD, DX: bf16 kernels [9][C][C]
    const uint16_t* dout;    // DW: delta of the layer output
    void* out;               // FWD, DX: [Pp][C], bf16 or fp32
    const float* bias;       // FWD
    const float* residual;   // FWD: fp32, NOT padded ([B H W][C]); added before the activation, or nullptr
    const uint16_t* mask;    // DX: padded bf16 activations whose sign gates the result
    float* partial;          // DW
    int64_t s_in, s_w, s_dout, s_out, s_bias, s_res, s_mask;
    int groups, B, H, W, C, Hp, Wp, Pp, halo;
    int relu;
    int tiles_m, tiles_n, total_tiles, chunk;
    int splits, k_chunk;
};

__device__ __forceinline__ int xcd_tile(int chunk, int total) {
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int tile = xcd * chunk + slot;
    return (slot >= chunk || tile >= total) ? -1 : tile;
}

// padded pixel q -> is it an image pixel, and which (index in the unpadded [B H W] order)
__device__ __forceinline__ bool interior(const ConvBDev& p, int q, int* unpadded) {
    const int per = p.Hp * p.Wp;
    const int n = q / per, rem = q - n * per;
    const int y = rem / p.Wp, x = rem - y * p.Wp;
    *unpadded = (n * p.H + (y - 1)) * p.W + (x - 1);
    return y >= 1 && y <= p.H && x >= 1 && x <= p.W;
}

__device__ __forceinline__ unsigned int pack2(float a, float b) { return bf16_bits_rne(a) | (bf16_bits_rne(b) << 16); }

// ---------------------------------------------------------------------------------------------
// forward (MODE 0) and back-propagated delta (MODE 1)
// ---------------------------------------------------------------------------------------------
template <int MODE, bool OUT_F32>
__global__ __launch_bounds__(kThreads, 2) void conv3x3_bf16_kernel(ConvBDev p) {
    using TB = typename std::conditional<MODE == 0, TileRC<kCB, kCB>, TileKC<kCB, kCB>>::type;   // FWD w[k = ci][n = co]; DX w[n = ci][k = co]
    constexpr int SP = kCB + 8;                  // strip pitch (bf16 elements): 144 bytes, conflict-free 16-byte reads
    constexpr int TM = 2, TN = 2;                // a wavefront owns 64 pixels x 64 channels
    extern __shared__ __attribute__((aligned(16))) uint16_t lds_all[];
    const int strip_rows = kBM + 2 * p.halo;
    uint16_t* strip = lds_all;
    uint16_t* lds_b0 = lds_all + strip_rows * SP;
    auto lds_b = [&](int buf) { return lds_b0 + buf * TB::kElems; };

    const int tile = xcd_tile(p.chunk, p.total_tiles);
    if (tile < 0) return;
    const int per_group = p.tiles_m * p.tiles_n;
    const int group = tile / per_group;
    const int tm = (tile % per_group) / p.tiles_n, tn = tile % p.tiles_n;
    const int m0 = tm * kBM, n0 = tn * kCB;
    const uint16_t* IN = p.in + (int64_t)group * p.s_in;
    const uint16_t* Wg = p.w + (int64_t)group * p.s_w;
    const int C = p.C;

    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int lane32 = lane % 32, half = lane / 32;
    const int wm0 = wave * 64;

    f16v acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // rows m0 - halo .. m0 + kBM + halo of channels c0 .. c0 + 63, zeros outside [0, Pp); four vectors in flight per lane
    auto load_strip = [&](int c0) {
        const int nvec = strip_rows * (kCB / 8);
        for (int v0 = threadIdx.x; v0 < nvec; v0 += 4 * kThreads) {
            u4 r[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int v = v0 + t * kThreads;
                const int q = m0 - p.halo + v / (kCB / 8);
                const bool ok = v < nvec && q >= 0 && q < p.Pp;
                const u4 got = *(const u4*)(IN + (ok ? (int64_t)q * C + c0 + (v % (kCB / 8)) * 8 : 0));
                const u4 zero = {0u, 0u, 0u, 0u};
                r[t] = ok ? got : zero;
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int v = v0 + t * kThreads;
                if (v < nvec) *(u4*)(strip + (v / (kCB / 8)) * SP + (v % (kCB / 8)) * 8) = r[t];
            }
        }
    };
    // the 64 x 64 kernel slice of one tap: rows k = contraction channel c0 .., columns n0 ..
    auto load_b = [&](u4 (&r)[TB::kPerThread], int tap, int c0) -> unsigned {
        // memory [ci][co].  FWD (row-contiguous tile): k = ci, rows = co; DX (K-contiguous tile): rows = ci, k = co
        return TB::load(r, Wg + (int64_t)tap * C * C, C, n0, c0, C, C);
    };

    bf16x8 fa[2][TM], fb[2][TN];
    auto load_frags = [&](int buf, const uint16_t* a_base, const uint16_t* b_tile, int s) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[buf][i] = __builtin_bit_cast(bf16x8, *(const u4*)(a_base + (wm0 + 32 * i + lane32) * SP + 16 * s + 8 * half));
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[buf][j] = TB::frag(b_tile, 32 * j, s, lane);
    };
    auto mfmas = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
    };

    u4 rb[TB::kPerThread];
    for (int c0 = 0; c0 < C; c0 += kCB) {
        // the previous chunk's last barrier has passed: nobody reads the strip or the kernel buffers any more
        unsigned okb = load_b(rb, 0, c0);
        load_strip(c0);
        TB::store(lds_b(0), rb, okb);
        __syncthreads();
        for (int tap = 0; tap < 9; ++tap) {
            if (tap + 1 < 9) okb = load_b(rb, tap + 1, c0);
            const int dy = tap / 3 - 1, dx = tap % 3 - 1;
            const int shift = (MODE == 0 ? 1 : -1) * (dy * p.Wp + dx);
            const uint16_t* a_base = strip + (p.halo + shift) * SP;
            const uint16_t* b_tile = lds_b(tap & 1);
            load_frags(0, a_base, b_tile, 0);
#pragma unroll
            for (int s = 0; s < kCB / 16; ++s) {
                if (s + 1 < kCB / 16) load_frags((s + 1) & 1, a_base, b_tile, s + 1);
                __builtin_amdgcn_sched_barrier(0);
                mfmas(s & 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (tap + 1 < 9) TB::store(lds_b((tap + 1) & 1), rb, okb);
            __syncthreads();
        }
    }

    // Epilogue.  Accumulator register r of a lane holds out[row][col] with col = lane % 32 and
    // row = 8 (r / 4) + 4 (lane / 32) + r % 4 inside its 32 x 32 block.
    if constexpr (OUT_F32) {
        // fp32 output (+ bias, shortcut, ReLU): the tile goes through LDS in two halves of 128 rows (two wavefronts each),
        // so that every lane then moves 16-byte vectors and all its shortcut loads are in flight together
        constexpr int FP = kCB + 8;                  // floats per staged row: the two half-waves hit disjoint banks
        constexpr int kVecPerRow = kCB / 4, kPer = 128 * kVecPerRow / kThreads;
        float* stage = (float*)lds_all;
        float* OUT = (float*)p.out + (int64_t)group * p.s_out;
        const float* RES = p.residual ? p.residual + (int64_t)group * p.s_res : nullptr;
        for (int h = 0; h < 2; ++h) {
            if (h) __syncthreads();                  // the first half has been read
            if (wave / 2 == h) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const int cl = 32 * j + lane32;
                        const float bias = p.bias ? p.bias[(int64_t)group * p.s_bias + n0 + cl] : 0.0f;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int rl = (wave % 2) * 64 + 32 * i + 8 * (r / 4) + 4 * half + (r % 4);
                            stage[rl * FP + cl] = acc[i][j][r] + bias;
                        }
                    }
            }
            __syncthreads();
#pragma unroll 1
            for (int t0 = 0; t0 < kPer; t0 += 4) {   // four vectors per lane at a time: their shortcut loads overlap
                f4 res[4];
                int64_t at[4];
                bool keep[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int v = threadIdx.x + (t0 + t) * kThreads;
                    const int q = m0 + 128 * h + v / kVecPerRow, cl = (v % kVecPerRow) * 4;
                    int up = 0;
                    keep[t] = q < p.Pp && interior(p, q, &up);
                    at[t] = q < p.Pp ? (int64_t)q * C + n0 + cl : -1;
                    res[t] = f4{0.f, 0.f, 0.f, 0.f};
                    if (RES && keep[t]) res[t] = __builtin_nontemporal_load((const f4*)(RES + (int64_t)up * C + n0 + cl));
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    if (at[t] < 0) continue;
                    const int v = threadIdx.x + (t0 + t) * kThreads;
                    f4 o = {0.f, 0.f, 0.f, 0.f};             // the zero border the pooling and its backward rely on
                    if (keep[t]) {
                        o = *(const f4*)(stage + (v / kVecPerRow) * FP + (v % kVecPerRow) * 4) + res[t];
                        if (p.relu) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) o[e] = fmaxf(o[e], 0.0f);
                        }
                    }
                    *(f4*)(OUT + at[t]) = o;
                }
            }
        }
    } else {
        // bf16 output: the tile goes through LDS (the strip's place) so that every lane then moves 16-byte vectors
        uint16_t* stage = lds_all;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int cl = 32 * j + lane32;
                float bias = 0.0f;
                if (MODE == 0 && p.bias) bias = p.bias[(int64_t)group * p.s_bias + n0 + cl];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rl = wm0 + 32 * i + 8 * (r / 4) + 4 * half + (r % 4);
                    float v = acc[i][j][r];
                    if (MODE == 0) {
                        v += bias;
                        if (p.relu) v = fmaxf(v, 0.0f);
                    }
                    stage[rl * SP + cl] = (uint16_t)bf16_bits_rne(v);
                }
            }
        }
        __syncthreads();
        uint16_t* OUT = (uint16_t*)p.out + (int64_t)group * p.s_out;
        const uint16_t* Mk = MODE == 1 && p.mask ? p.mask + (int64_t)group * p.s_mask : nullptr;
        constexpr int kVecPerRow = kCB / 8;
#pragma unroll 4
        for (int t = 0; t < kBM * kVecPerRow / kThreads; ++t) {
            const int v = threadIdx.x + t * kThreads;
            const int rl = v / kVecPerRow, cl = (v % kVecPerRow) * 8;
            const int q = m0 + rl;
            if (q >= p.Pp) continue;
            u4 o = *(const u4*)(stage + rl * SP + cl);
            const int64_t at = (int64_t)q * C + n0 + cl;
            if (MODE == 0) {
                int up;
                if (!interior(p, q, &up)) o = u4{0u, 0u, 0u, 0u};   // the zero border the next layer relies on
            } else if (Mk) {
                const u4 mk = *(const u4*)(Mk + at);
#pragma unroll
                for (int w = 0; w < 4; ++w) {   // a bf16 is positive iff its sign bit is clear and it is not zero
                    const unsigned int lo = mk[w] & 0xFFFFu, hi = mk[w] >> 16;
                    const unsigned int keep = ((lo != 0u && lo < 0x8000u) ? 0xFFFFu : 0u) |
                                              ((hi != 0u && hi < 0x8000u) ? 0xFFFF0000u : 0u);
                    o[w] &= keep;
                }
            }
            *(u4*)(OUT + at) = o;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// kernel / bias gradient
// ---------------------------------------------------------------------------------------------
template <int NV>   // strip vectors per lane (upper bound of (32 + 2 halo) * 8 / 256)
__global__ __launch_bounds__(kThreads) void conv3x3_dw_bf16_kernel(ConvBDev p) {
    using TD = TileRC<kCB, kDwBK>;               // delta tile: [32 pixels][64 channels + 32]
    constexpr int RP = TD::kPitch;               // the input strip uses the same pitch
    extern __shared__ __attribute__((aligned(16))) uint16_t lds_all[];
    const int strip_rows = kDwBK + 2 * p.halo;
    const int strip_elems = strip_rows * RP;
    auto lds_s = [&](int buf) { return lds_all + buf * strip_elems; };
    auto lds_d = [&](int buf) { return lds_all + 2 * strip_elems + buf * TD::kElems; };

    const int tile = xcd_tile(p.chunk, p.total_tiles);
    if (tile < 0) return;
    const int nb = p.tiles_n;                                    // 64-channel blocks
    const int per_group = p.splits * nb * nb;
    const int group = tile / per_group;
    const int rest = tile % per_group;
    const int split = rest / (nb * nb);
    const int ci0 = ((rest / nb) % nb) * kCB, co0 = (rest % nb) * kCB;
    const int lo = split * p.k_chunk, hi = min(p.Pp, lo + p.k_chunk);
    const uint16_t* IN = p.in + (int64_t)group * p.s_in;
    const uint16_t* DO = p.dout + (int64_t)group * p.s_dout;
    const int C = p.C;

    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int lane32 = lane % 32, half = lane / 32;
    const int wi = wave / 2, wj = wave % 2;      // 32 x 32 block of the 64 x 64 (ci, co) tile

    f16v acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
    const bool col_sums = ci0 == 0 && threadIdx.x < kCB;
    float col_acc = 0.0f;

    const int nvec = strip_rows * (kCB / 8);
    auto load_strip = [&](u4 (&r)[NV], int k0) -> unsigned {
        unsigned okmask = 0;
#pragma unroll
        for (int t = 0; t < NV; ++t) {
            const int v = threadIdx.x + t * kThreads;
            const int q = k0 - p.halo + v / (kCB / 8);
            const bool ok = v < nvec && q >= 0 && q < p.Pp;
            r[t] = *(const u4*)(IN + (ok ? (int64_t)q * C + ci0 + (v % (kCB / 8)) * 8 : 0));
            okmask |= ok ? (1u << t) : 0u;
        }
        return okmask;
    };
    auto store_strip = [&](uint16_t* dst, const u4 (&r)[NV], unsigned okmask) {
#pragma unroll
        for (int t = 0; t < NV; ++t) {
            const int v = threadIdx.x + t * kThreads;
            if (v < nvec) {
                const u4 zero = {0u, 0u, 0u, 0u};
                *(u4*)(dst + (v / (kCB / 8)) * RP + (v % (kCB / 8)) * 8) = (okmask >> t) & 1u ? r[t] : zero;
            }
        }
    };

    u4 rs[NV], rd[TD::kPerThread];
    unsigned oks = load_strip(rs, lo);
    unsigned okd = TD::load(rd, DO, C, co0, lo, C, hi);
    store_strip(lds_s(0), rs, oks);
    TD::store(lds_d(0), rd, okd);
    __syncthreads();
    const int nslices = (hi - lo + kDwBK - 1) / kDwBK;
    for (int t = 0; t < nslices; ++t) {
        const int cur = t & 1;
        if (t + 1 < nslices) {
            oks = load_strip(rs, lo + (t + 1) * kDwBK);
            okd = TD::load(rd, DO, C, co0, lo + (t + 1) * kDwBK, C, hi);
        }
        const uint16_t* S = lds_s(cur) + p.halo * RP;
        const uint16_t* D = lds_d(cur);
#pragma unroll
        for (int s = 0; s < kDwBK / 16; ++s) {
            const bf16x8 fd = TD::frag(D, 32 * wj, s, lane);
#pragma unroll
            for (int tap = 0; tap < 9; ++tap) {
                const int shift = (tap / 3 - 1) * p.Wp + (tap % 3 - 1);
                const bf16x8 fi = TD::frag(S + shift * RP, 32 * wi, s, lane);
                acc[tap] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fi, fd, acc[tap], 0, 0, 0);
            }
        }
        if (col_sums) {
#pragma unroll 8
            for (int k = 0; k < kDwBK; ++k) col_acc += __uint_as_float((unsigned)D[k * RP + threadIdx.x] << 16);
        }
        if (t + 1 < nslices) {
            store_strip(lds_s(cur ^ 1), rs, oks);
            TD::store(lds_d(cur ^ 1), rd, okd);
        }
        __syncthreads();
    }

    const int64_t n_w = (int64_t)9 * C * C;
    float* PART = p.partial + ((int64_t)split * p.groups + group) * (n_w + C);
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int ci = ci0 + 32 * wi + 8 * (r / 4) + 4 * half + (r % 4);
            PART[((int64_t)tap * C + ci) * C + co0 + 32 * wj + lane32] = acc[tap][r];
        }
    }
    if (col_sums) PART[n_w + co0 + threadIdx.x] = col_acc;
}

// ---------------------------------------------------------------------------------------------
// fp32 [B H W][C] -> bf16 [B (H+2) (W+2)][C] with a zero border; one lane per 8 channels of a padded pixel
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void pad_cast_bf16_kernel(const float* __restrict__ src, int64_t s_src,
                                                                 uint16_t* __restrict__ dst, int64_t s_dst, int64_t vecs, int H,
                                                                 int W, int C) {
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (v >= vecs) return;
    const int g = blockIdx.y;
    const int c8 = C / 8;
    const int q = (int)(v / c8), cv = (int)(v % c8);
    const int Wp = W + 2, per = (H + 2) * Wp;
    const int n = q / per, rem = q - n * per;
    const int y = rem / Wp, x = rem - y * Wp;
    u4 o = {0u, 0u, 0u, 0u};
    if (y >= 1 && y <= H && x >= 1 && x <= W) {
        const f4* S = (const f4*)(src + (int64_t)g * s_src + ((int64_t)(n * H + y - 1) * W + (x - 1)) * C) + 2 * cv;
        const f4 lo = __builtin_nontemporal_load(S), hi = __builtin_nontemporal_load(S + 1);
        o.x = pack2(lo.x, lo.y);
        o.y = pack2(lo.z, lo.w);
        o.z = pack2(hi.x, hi.y);
        o.w = pack2(hi.z, hi.w);
    }
    *((u4*)(dst + (int64_t)g * s_dst) + v) = o;
}

// dz[g][q][c] = bf16(dpool[g][sample][c] * scale) where a[g][q][c] > 0, else 0; a fp32 padded, dz bf16 padded
__global__ __launch_bounds__(kThreads) void pool_bwd_bf16_kernel(const float* __restrict__ dpool, int64_t s_dp,
                                                                 const float* __restrict__ a, int64_t s_a, uint16_t* dz,
                                                                 int64_t s_dz, int64_t vecs, int positions, int C, float scale) {
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (v >= vecs) return;
    const int g = blockIdx.y;
    const int c8 = C / 8;
    const int64_t q = v / c8;
    const int cv = (int)(v % c8);
    const int64_t sample = q / positions;
    const f4* A = (const f4*)(a + (int64_t)g * s_a) + 2 * v;
    const f4 a0 = __builtin_nontemporal_load(A), a1 = __builtin_nontemporal_load(A + 1);
    const f4* D = (const f4*)(dpool + (int64_t)g * s_dp + sample * C) + 2 * cv;
    const f4 d0 = D[0], d1 = D[1];
    float o[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        o[e] = a0[e] > 0.0f ? d0[e] * scale : 0.0f;
        o[4 + e] = a1[e] > 0.0f ? d1[e] * scale : 0.0f;
    }
    u4 w;
    w.x = pack2(o[0], o[1]);
    w.y = pack2(o[2], o[3]);
    w.z = pack2(o[4], o[5]);
    w.w = pack2(o[6], o[7]);
    *((u4*)(dz + (int64_t)g * s_dz) + v) = w;
}

bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

bool shape_ok(const ConvBArgs& a) {
    if (a.groups < 1 || a.groups > 65535 || a.B < 1 || a.H < 1 || a.W < 1 || a.W > kConvBf16MaxWidth || a.C < kCB || a.C % kCB != 0 ||
        a.C > 1024)
        return false;
    const int64_t Pp = (int64_t)a.B * (a.H + 2) * (a.W + 2);
    return Pp * a.C < ((int64_t)1 << 31) - ((int64_t)(kBM + 2 * (a.W + 3)) * a.C);   // 32-bit pixel indices inside one group
}

void fill(ConvBDev* p, const ConvBArgs& a) {
    p->groups = a.groups; p->B = a.B; p->H = a.H; p->W = a.W; p->C = a.C;
    p->Hp = a.H + 2; p->Wp = a.W + 2; p->Pp = a.B * p->Hp * p->Wp; p->halo = p->Wp + 1;
    p->relu = a.relu;
}

template <int MODE>
hipError_t conv_launch(const ConvBArgs& a, hipStream_t s) {
    if (!shape_ok(a) || !a.in || !a.w || !a.out || !aligned16(a.in) || !aligned16(a.w) || !aligned16(a.out)) return hipErrorInvalidValue;
    if (a.s_in % 8 || a.s_w % 8 || a.s_out % 8 || (a.mask && (!aligned16(a.mask) || a.s_mask % 8))) return hipErrorInvalidValue;
    if (MODE == 1 && a.out_f32) return hipErrorInvalidValue;   // the delta is always an operand of the next product
    ConvBDev p = {};
    fill(&p, a);
    p.in = (const uint16_t*)a.in; p.w = (const uint16_t*)a.w; p.out = a.out;
    p.bias = MODE == 0 ? a.bias : nullptr; p.residual = MODE == 0 ? a.residual : nullptr;
    p.mask = MODE == 1 ? (const uint16_t*)a.mask : nullptr;
    p.s_in = a.s_in; p.s_w = a.s_w; p.s_out = a.s_out; p.s_bias = a.s_bias; p.s_res = a.s_res; p.s_mask = a.s_mask;
    p.tiles_m = (p.Pp + kBM - 1) / kBM;
    p.tiles_n = a.C / kCB;
    const int64_t total = (int64_t)a.groups * p.tiles_m * p.tiles_n;
    if (total > (1 << 30)) return hipErrorInvalidValue;
    p.total_tiles = (int)total;
    p.chunk = (int)((total + kXcds - 1) / kXcds);
    const size_t b_elems = MODE == 0 ? TileRC<kCB, kCB>::kElems : TileKC<kCB, kCB>::kElems;
    const size_t lds = ((size_t)(kBM + 2 * p.halo) * (kCB + 8) + 2 * b_elems) * sizeof(uint16_t);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    void (*kern)(ConvBDev) = MODE == 0 ? (a.out_f32 ? conv3x3_bf16_kernel<0, true> : conv3x3_bf16_kernel<0, false>)
                                       : conv3x3_bf16_kernel<1, false>;
    if (lds > 64 * 1024) {
        hipError_t e = ensure_dynamic_lds((const void*)kern, 160 * 1024);
        if (e != hipSuccess) return e;
    }
    kern<<<(unsigned)(p.chunk * kXcds), kThreads, lds, s>>>(p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_conv3x3_bf16_fwd(const ConvBArgs& a, hipStream_t s) { return conv_launch<0>(a, s); }
hipError_t launch_conv3x3_bf16_dx(const ConvBArgs& a, hipStream_t s) { return conv_launch<1>(a, s); }

int conv3x3_bf16_dw_splits(int groups, int B, int H, int W, int C) {
    const int64_t Pp = (int64_t)B * (H + 2) * (W + 2);
    const int64_t tiles = (int64_t)groups * (C / kCB) * (C / kCB);
    int64_t s = (768 + tiles - 1) / tiles;                  // three workgroups per compute unit (their LDS allows three)
    const int64_t most = (Pp + 511) / 512;                  // a range covers at least 512 padded pixels
    if (s > most) s = most;
    if (s > 256) s = 256;
    return s < 1 ? 1 : (int)s;
}

hipError_t launch_conv3x3_bf16_dw(const ConvBArgs& a, hipStream_t s) {
    if (!shape_ok(a) || !a.in || !a.dout || !a.partial || !a.g || !aligned16(a.in) || !aligned16(a.dout)) return hipErrorInvalidValue;
    if (a.s_in % 8 || a.s_dout % 8) return hipErrorInvalidValue;
    ConvBDev p = {};
    fill(&p, a);
    p.in = (const uint16_t*)a.in; p.dout = (const uint16_t*)a.dout; p.partial = a.partial;
    p.s_in = a.s_in; p.s_dout = a.s_dout;
    p.splits = conv3x3_bf16_dw_splits(a.groups, a.B, a.H, a.W, a.C);
    p.k_chunk = (int)(((((int64_t)p.Pp + p.splits - 1) / p.splits) + kDwBK - 1) / kDwBK * kDwBK);
    p.tiles_n = a.C / kCB;
    const int64_t total = (int64_t)a.groups * p.splits * p.tiles_n * p.tiles_n;
    if (total > (1 << 30)) return hipErrorInvalidValue;
    p.total_tiles = (int)total;
    p.chunk = (int)((total + kXcds - 1) / kXcds);
    const int strip_rows = kDwBK + 2 * p.halo;
    const size_t lds = (2 * (size_t)strip_rows * TileRC<kCB, kDwBK>::kPitch + 2 * TileRC<kCB, kDwBK>::kElems) * sizeof(uint16_t);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    const int nv = (strip_rows * (kCB / 8) + kThreads - 1) / kThreads;
    void (*kern)(ConvBDev) = nullptr;
    if (nv <= 4) kern = conv3x3_dw_bf16_kernel<4>;
    else if (nv <= 10) kern = conv3x3_dw_bf16_kernel<10>;
    else return hipErrorInvalidValue;
    if (lds > 64 * 1024) {
        hipError_t e = ensure_dynamic_lds((const void*)kern, 160 * 1024);
        if (e != hipSuccess) return e;
    }
    kern<<<(unsigned)(p.chunk * kXcds), kThreads, lds, s>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_conv_dw_finish(a.partial, p.splits, a.groups, a.C, a.g, a.ld, a.g_w_off, a.g_b_off, s);
}

hipError_t launch_pad_cast_bf16(const float* src, int64_t s_src, uint16_t* dst, int64_t s_dst, int groups, int B, int H, int W,
                                int C, hipStream_t s) {
    if (!src || !dst || groups < 1 || groups > 65535 || B < 1 || H < 1 || W < 1 || C < 8 || C % 8 || !aligned16(src) ||
        !aligned16(dst) || s_src % 4 || s_dst % 8)
        return hipErrorInvalidValue;
    const int64_t vecs = (int64_t)B * (H + 2) * (W + 2) * (C / 8);
    const int64_t blocks = (vecs + kThreads - 1) / kThreads;
    if (blocks > 0x7FFFFFFF || vecs / (C / 8) > 0x7FFFFFFF) return hipErrorInvalidValue;
    pad_cast_bf16_kernel<<<dim3((unsigned)blocks, (unsigned)groups), kThreads, 0, s>>>(src, s_src, dst, s_dst, vecs, H, W, C);
    return hipGetLastError();
}

hipError_t launch_pool_bwd_bf16(const float* dpool, int64_t s_dp, const float* a, int64_t s_a, uint16_t* dz, int64_t s_dz,
                                int groups, int B, int positions, int C, float scale, hipStream_t s) {
    if (!dpool || !a || !dz || groups < 1 || groups > 65535 || B < 1 || positions < 1 || C < 8 || C % 8 || !aligned16(dpool) ||
        !aligned16(a) || !aligned16(dz) || s_dp % 4 || s_a % 4 || s_dz % 8)
        return hipErrorInvalidValue;
    const int64_t vecs = (int64_t)B * positions * (C / 8);
    const int64_t blocks = (vecs + kThreads - 1) / kThreads;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    pool_bwd_bf16_kernel<<<dim3((unsigned)blocks, (unsigned)groups), kThreads, 0, s>>>(dpool, s_dp, a, s_a, dz, s_dz, vecs, positions,
                                                                                      C, scale);
    return hipGetLastError();
}

}  // namespace ols
