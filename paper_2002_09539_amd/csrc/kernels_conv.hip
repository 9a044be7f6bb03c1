// 3 x 3 convolutions (stride 1, zero padding 1) of the per-worker residual block as implicit GEMMs on the fp32
// matrix cores (v_mfma_f32_32x32x2_f32), grouped over the m workers: forward, back-propagated delta, weight / bias
// gradient; plus the global average pooling in front of the classifier and its backward.  The model is the first
// residual stage of the network of Section 4 (arXiv 2002.09539, "Experimental setting": ResNet-18 on 32 x 32 inputs,
// mini-batch 128 per node) and produces the stochastic gradients g_i of Section 2.
//
// Layouts: activations [group][P][C] with P = B H W pixels in (sample, row, column) order and the channel contiguous
// (NHWC); kernels [group][9][C][C] as (tap = 3 kh + kw, input channel, output channel).
//
//   FWD  out[p][co] = act( sum_{tap, ci} in[p + shift(tap)][ci] w[tap][ci][co] + bias[co] (+ residual[p][co]) )
//        an M = P, N = C, K = 9 C GEMM whose A operand is gathered: K slice s lies inside one tap, and row p of the
//        slice is the contiguous channel run of the pixel shifted by (kh - 1, kw - 1), or zero outside the image
//   DX   din[p][ci] = ( sum_{tap, co} dout[p - shift(tap)][co] w[tap][ci][co] ) * [mask[p][ci] > 0]
//        the same with the opposite shifts and the kernel read with its channel indices exchanged
//   DW   dw[tap][ci][co] = sum_p in[p + shift(tap)][ci] dout[p][co];  db[co] = sum_p dout[p][co]
//        per kernel row an M = 3 C, N = C GEMM contracting over all P pixels; the pixel range is split over workgroups, the
//        parts are written raw and summed in a fixed order by a second pass (no atomics: results do not depend on
//        timing)
//
// Operand tiles go global -> registers -> LDS with 16-byte vectors and feed the MFMAs through the fragment layout of
// gemm_f32_tile.h; two slices of global loads are in flight while a third feeds the matrix cores.
//
// Measured at the benchmark shape (16 workers x 128 samples x 32 x 32 x 64 channels, 154.6 GFLOP per launch; us per
// launch).  Forward / delta, tile rows x K slice x slices in flight: 128 x 32 x 1: 1622 / 1680; 128 x 32 x 2: 1682 /
// 1713; 128 x 16 x 1: 1418 / 1404; 128 x 16 x 2: 1395 / 1386; 64 x 32 x 2: 1455 / 1461; 64 x 16 x 2: 1402 / 1450;
// 256 x 16 x 2: 1591 / 1612 -- the short slice halves the LDS of a workgroup (29 KB: five workgroups per compute unit
// instead of two), which matters more than the number of barriers.  Weight gradient: one tap per workgroup (64 x 64
// output, 32 x 32 per wavefront) 1688 with slices of 32, 1637 / 1568 with slices of 16 and one / two in flight; a kernel
// row per workgroup (192 x 64) 1626 / 1482 with one / two in flight, and 1420 with the register budget capped for three
// wavefronts per SIMD (1733 when capped for four: spills).
#include "gemm_f32_tile.h"
#include "ols_internal.h"

namespace ols {

namespace {

constexpr int kThreads = kGemmThreads;
constexpr int kXcds = 8;
constexpr int kBN = 64;   // output-channel tile

struct ConvDev {
    const float* in;        // FWD: layer input; DX: delta of the layer output; DW: layer input
    const float* w;         // FWD, DX: kernels
    const float* dout;      // DW: delta of the layer output
    float* out;             // FWD: layer output; DX: delta of the layer input
    float* partial;         // DW: [splits][groups][9 C C + C] raw partial sums
    const float* bias;      // FWD
    const float* residual;  // FWD: added before the activation, or nullptr
    const float* mask;      // DX: activations whose sign gates the result, or nullptr
    int64_t s_in, s_w, s_dout, s_out, s_bias, s_res, s_mask;   // group strides (elements)
    int groups, B, H, W, C, P;
    int relu;
    int tiles_m, tiles_n, total_tiles, chunk;
    int splits, k_chunk;
};

// XCD-aware tile id: the hardware deals workgroup b to XCD b % 8; every XCD gets a contiguous range of tiles, so the
// image rows shared by neighbouring tiles (the 3 x 3 halo) are fetched into one L2.
__device__ __forceinline__ int xcd_tile(int chunk, int total) {
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int tile = xcd * chunk + slot;
    return (slot >= chunk || tile >= total) ? -1 : tile;
}

// ---------------------------------------------------------------------------------------------
// forward (MODE 0) and back-propagated delta (MODE 1)
// ---------------------------------------------------------------------------------------------
template <int MODE, int BM, int BK, int DEPTH>
__global__ __launch_bounds__(kThreads) void conv3x3_kernel(ConvDev p) {
    constexpr bool B_KC = MODE == 1;            // DX reads w[tap][n = ci][k = co]: contraction index contiguous
    using TA = Tile<BM, BK, true>;
    using TB = Tile<kBN, BK, B_KC>;
    constexpr int WM = BM / 2, WN = kBN / 2;    // 2 x 2 wavefronts
    constexpr int TM = WM / 32, TN = WN / 32;
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 16 == 0, "tile shape");
    __shared__ __attribute__((aligned(16))) float lds_all[2 * TA::kFloats + 2 * TB::kFloats];
    auto lds_a = [&](int buf) { return lds_all + buf * TA::kFloats; };
    auto lds_b = [&](int buf) { return lds_all + 2 * TA::kFloats + buf * TB::kFloats; };

    const int tile = xcd_tile(p.chunk, p.total_tiles);
    if (tile < 0) return;
    const int per_group = p.tiles_m * p.tiles_n;
    const int group = tile / per_group;
    const int tm = (tile % per_group) / p.tiles_n, tn = tile % p.tiles_n;
    const int m0 = tm * BM, n0 = tn * kBN;
    const float* IN = p.in + (int64_t)group * p.s_in;
    const float* Wg = p.w + (int64_t)group * p.s_w;
    const int C = p.C, H = p.H, Wd = p.W;

    // Rows of the A tile are pixels.  Each lane copies the same rows in every slice: decode them once, and record
    // for which of the nine taps the shifted pixel lies inside the image.
    int pix_off[TA::kPerThread];
    unsigned tapmask[TA::kPerThread];
#pragma unroll
    for (int t = 0; t < TA::kPerThread; ++t) {
        const int v = threadIdx.x + t * kThreads;
        const int line = v / TA::kVecPerLine;
        const int pix = m0 + line;
        unsigned mask = 0;
        if ((TA::kVecs % kThreads == 0 || v < TA::kVecs) && pix < p.P) {
            const int rem = pix % (H * Wd);
            const int y = rem / Wd, x = rem % Wd;
#pragma unroll
            for (int tap = 0; tap < 9; ++tap) {
                const int dy = MODE == 0 ? tap / 3 - 1 : 1 - tap / 3;
                const int dx = MODE == 0 ? tap % 3 - 1 : 1 - tap % 3;
                const bool inside = y + dy >= 0 && y + dy < H && x + dx >= 0 && x + dx < Wd;
                mask |= inside ? (1u << tap) : 0u;
            }
        }
        tapmask[t] = mask;
        pix_off[t] = pix * C + (v % TA::kVecPerLine) * 4;
    }
    auto load_a = [&](f4 (&r)[TA::kPerThread], int s) -> unsigned {
        const int k0 = s * BK;
        const int tap = k0 / C, c0 = k0 % C;           // a slice never straddles two taps: BK divides C
        const int dy = MODE == 0 ? tap / 3 - 1 : 1 - tap / 3;
        const int dx = MODE == 0 ? tap % 3 - 1 : 1 - tap % 3;
        const int shift = (dy * Wd + dx) * C + c0;
        unsigned okmask = 0;
#pragma unroll
        for (int t = 0; t < TA::kPerThread; ++t) {
            const bool ok = tap < 9 && ((tapmask[t] >> tap) & 1u);
            r[t] = *(const f4*)(IN + (ok ? pix_off[t] + shift : 0));
            okmask |= ok ? (1u << t) : 0u;
        }
        return okmask;
    };
    auto load_b = [&](f4 (&r)[TB::kPerThread], int s) -> unsigned {
        const int k0 = s * BK;
        if (MODE == 0) return TB::load(r, Wg, C, n0, k0, C, 9 * C);             // w as a [9 C][C] matrix
        const int tap = k0 / C, c0 = k0 % C;
        if (tap >= 9) return TB::load(r, Wg, C, n0, 0, 0, 0);                   // past the end: all-zero dummy
        return TB::load(r, Wg + (int64_t)tap * C * C, C, n0, c0, C, C);         // rows = ci, contraction over co
    };

    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int lane32 = lane % 32, half = lane / 32;
    const int wm0 = (wave / 2) * WM, wn0 = (wave % 2) * WN;

    f16v acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // Fragment registers are double-buffered across k-octets and the LDS reads of octet q + 1 are issued ahead of
    // the MFMAs of octet q (a wavefront stalls at MFMA issue while the matrix pipe is busy).
    constexpr int Q = BK / 8;
    f4 fa[2][TM], fb[2][TN];
    auto load_frags = [&](int buf, int cur, int q) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[buf][i] = TA::frag(lds_a(cur), wm0 + 32 * i, q, lane32, half);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[buf][j] = TB::frag(lds_b(cur), wn0 + 32 * j, q, lane32, half);
    };
    auto mfmas = [&](int buf) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[buf][i][e], fb[buf][j][e], acc[i][j], 0, 0, 0);
    };

    // One K slice out of lds[cur]; the staged registers of the next slice are published to lds[cur ^ 1] before the
    // last octet's MFMAs, so the barrier and the first fragment reads of that slice hide behind them.
    auto slice = [&](int cur, const f4 (&na)[TA::kPerThread], unsigned oka, const f4 (&nb)[TB::kPerThread], unsigned okb) {
#pragma unroll
        for (int q = 0; q + 1 < Q; ++q) {
            load_frags((q + 1) & 1, cur, q + 1);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(q & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        TA::store(lds_a(cur ^ 1), na, oka);
        TB::store(lds_b(cur ^ 1), nb, okb);
        __syncthreads();
        load_frags(0, cur ^ 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfmas((Q - 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
    };
    // Slices past the end are zero-filled dummies (tap 9): what they publish is never consumed, or contributes zeros.
    const int nk = 9 * C / BK;
    if (DEPTH == 1) {
        f4 ra[TA::kPerThread], rb[TB::kPerThread];
        unsigned oka = load_a(ra, 0), okb = load_b(rb, 0);
        TA::store(lds_a(0), ra, oka);
        TB::store(lds_b(0), rb, okb);
        __syncthreads();
        load_frags(0, 0, 0);
        for (int kt = 0; kt < nk; ++kt) {
            oka = load_a(ra, kt + 1);
            okb = load_b(rb, kt + 1);
            slice(kt & 1, ra, oka, rb, okb);
        }
    } else {
        // Two slices of global loads in flight: while slice t feeds the matrix cores from LDS, slice t + 1 waits in
        // registers and slice t + 2 is on its way.  Slices are consumed in pairs; an odd trailing one is paired with a
        // dummy.
        f4 ra0[TA::kPerThread], rb0[TB::kPerThread], ra1[TA::kPerThread], rb1[TB::kPerThread];
        unsigned oka0 = load_a(ra0, 0), okb0 = load_b(rb0, 0);
        unsigned oka1 = load_a(ra1, 1), okb1 = load_b(rb1, 1);
        TA::store(lds_a(0), ra0, oka0);
        TB::store(lds_b(0), rb0, okb0);
        __syncthreads();
        load_frags(0, 0, 0);
        const int nk2 = (nk + 1) & ~1;
        for (int kt = 0; kt < nk2; kt += 2) {
            oka0 = load_a(ra0, kt + 2);
            okb0 = load_b(rb0, kt + 2);
            slice(0, ra1, oka1, rb1, okb1);
            oka1 = load_a(ra1, kt + 3);
            okb1 = load_b(rb1, kt + 3);
            slice(1, ra0, oka0, rb0, okb0);
        }
    }

    // Epilogue.  Accumulator register r of a lane holds out[row][col] with col = lane % 32 and
    // row = 8 (r / 4) + 4 (lane / 32) + r % 4 inside its 32 x 32 block.
    float* OUT = p.out + (int64_t)group * p.s_out;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn0 + 32 * j + lane32;
            if (col >= C) continue;
            float bias = 0.0f;
            if (MODE == 0 && p.bias) bias = p.bias[(int64_t)group * p.s_bias + col];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm0 + 32 * i + 8 * (r / 4) + 4 * half + (r % 4);
                if (row >= p.P) continue;
                const int64_t o = (int64_t)row * C + col;
                float v = acc[i][j][r];
                if (MODE == 0) {
                    v += bias;
                    if (p.residual) v += p.residual[(int64_t)group * p.s_res + o];
                    if (p.relu) v = fmaxf(v, 0.0f);
                } else if (p.mask) {
                    v = p.mask[(int64_t)group * p.s_mask + o] > 0.0f ? v : 0.0f;
                }
                OUT[o] = v;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// weight / bias gradient: one tile per (group, pixel range, kernel row kh, 64 x 64 block of input x output channels).
// A workgroup forms the gradient of the three taps of a kernel row at once: its A tile holds, side by side, the 64
// input channels of the pixel shifted by kw - 1 = -1, 0, +1 (rows 64 kw + ci of a 192 x 64 output), so one tile of dout
// serves three taps, a wavefront owns 96 x 32 (three MFMA blocks per fragment of dout), and the three shifted reads of
// the input hit the same cache lines.
// ---------------------------------------------------------------------------------------------
#ifndef OLS_CONV_DW_WAVES
#define OLS_CONV_DW_WAVES 3
#endif
template <int BK, int DEPTH>
__global__ __launch_bounds__(kThreads, OLS_CONV_DW_WAVES) void conv3x3_dw_kernel(ConvDev p) {
    constexpr int kRowTaps = 3, kBMW = 64 * kRowTaps;   // 192 rows: (kw, ci)
    using TA = Tile<kBMW, BK, false>;   // in[pixel + shift(kw)][ci]: [BK][192 + 4] in LDS
    using TB = Tile<kBN, BK, false>;    // dout[pixel][co]
    static_assert(DEPTH == 1 || DEPTH == 2, "slices of global loads in flight");
    constexpr int TM = 3;               // 2 x 2 wavefronts of 96 x 32
    __shared__ __attribute__((aligned(16))) float lds_all[2 * TA::kFloats + 2 * TB::kFloats];
    auto lds_a = [&](int buf) { return lds_all + buf * TA::kFloats; };
    auto lds_b = [&](int buf) { return lds_all + 2 * TA::kFloats + buf * TB::kFloats; };

    const int tile = xcd_tile(p.chunk, p.total_tiles);
    if (tile < 0) return;
    const int C = p.C, H = p.H, Wd = p.W;
    // tile -> (group, split, kh, tm, tn), tn fastest: the kernel rows of a pixel range are neighbours (they share dout)
    int rest = tile;
    const int tn = rest % p.tiles_n; rest /= p.tiles_n;
    const int tm = rest % p.tiles_n; rest /= p.tiles_n;
    const int kh = rest % 3; rest /= 3;
    const int split = rest % p.splits;
    const int group = rest / p.splits;
    const int m0 = tm * 64, n0 = tn * kBN;
    const int k_lo = split * p.k_chunk, k_hi = min(p.P, k_lo + p.k_chunk);
    const int dy = kh - 1;
    const float* IN = p.in + (int64_t)group * p.s_in;
    const float* DOUT = p.dout + (int64_t)group * p.s_dout;

    // Lines of the operand tiles are pixels that advance by BK per slice.  A lane copies, for ONE pixel line and one
    // group of four channels, the three shifted input vectors (kw = 0, 1, 2) and the vector of dout, so it carries a
    // single pixel position (pix, y, x) along.
    static_assert(BK == 16, "one pixel line per lane: 16 lines x 16 channel vectors = 256 lanes");
    const int line = threadIdx.x / 16, c4 = (threadIdx.x % 16) * 4;
    int pix = k_lo + line;
    int py = (pix % (H * Wd)) / Wd, px = pix % Wd;
    const bool ch_ok = m0 + c4 < C, co_ok = n0 + c4 < C;
    struct Staged {
        f4 a[kRowTaps];
        f4 b;
        unsigned ok;   // bits 0..2: the three taps, bit 3: dout
    };
    auto load_ab = [&](Staged& r) {   // loads the slice the carried pixel points at, then advances by BK pixels
        const bool in_range = pix < k_hi;
        const int y = py + dy;
        const bool row_ok = in_range && ch_ok && y >= 0 && y < H;
        const float* src = IN + (int64_t)(pix + dy * Wd) * C + m0 + c4;
        r.ok = 0;
#pragma unroll
        for (int kw = 0; kw < kRowTaps; ++kw) {
            const int x = px + kw - 1;
            const bool ok = row_ok && x >= 0 && x < Wd;
            r.a[kw] = *(const f4*)(ok ? src + (kw - 1) * C : IN);
            r.ok |= ok ? (1u << kw) : 0u;
        }
        const bool okb = in_range && co_ok;
        r.b = *(const f4*)(okb ? DOUT + (int64_t)pix * C + n0 + c4 : DOUT);
        r.ok |= okb ? 8u : 0u;
        pix += BK;
        px += BK;
        while (px >= Wd) {
            px -= Wd;
            py += 1;
        }
        while (py >= H) py -= H;
    };
    auto store_ab = [&](int buf, const Staged& r) {
        const f4 zero = {0.f, 0.f, 0.f, 0.f};
        float* qa = lds_a(buf) + line * TA::kPitch + c4;
#pragma unroll
        for (int kw = 0; kw < kRowTaps; ++kw) *(f4*)(qa + 64 * kw) = (r.ok >> kw) & 1u ? r.a[kw] : zero;
        *(f4*)(lds_b(buf) + line * TB::kPitch + c4) = (r.ok & 8u) ? r.b : zero;
    };

    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int lane32 = lane % 32, half = lane / 32;
    const int wm0 = (wave / 2) * 96, wn0 = (wave % 2) * 32;

    f16v acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    // the bias gradient is the column sum of dout over the pixel range: formed once per range (kernel row 0, first block)
    // (the rows of a slice are shared out over the four wavefronts, which add their shares in wavefront order at the end:
    // one wavefront summing alone would keep the other three at the slice's barrier)
    const bool col_sums = kh == 0 && tm == 0;
    float col_acc = 0.0f;

    constexpr int Q = BK / 8;
    f4 fa[2][TM], fb[2];
    auto load_frags = [&](int buf, int cur, int q) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[buf][i] = TA::frag(lds_a(cur), wm0 + 32 * i, q, lane32, half);
        fb[buf] = TB::frag(lds_b(cur), wn0, q, lane32, half);
    };
    auto mfmas = [&](int buf) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int i = 0; i < TM; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[buf][i][e], fb[buf][e], acc[i], 0, 0, 0);
    };
    auto slice = [&](int cur, const Staged& next) {
#pragma unroll
        for (int q = 0; q + 1 < Q; ++q) {
            load_frags((q + 1) & 1, cur, q + 1);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(q & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (col_sums) {
#pragma unroll
            for (int k = 0; k < BK / 4; ++k) col_acc += lds_b(cur)[(wave * (BK / 4) + k) * TB::kPitch + lane];
        }
        store_ab(cur ^ 1, next);
        __syncthreads();
        load_frags(0, cur ^ 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfmas((Q - 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
    };
    // Slices past the pixel range are zero-filled: they add nothing to the sums.
    const int nk = k_hi > k_lo ? (k_hi - k_lo + BK - 1) / BK : 0;
    if (nk > 0 && DEPTH == 1) {
        Staged r;
        load_ab(r);
        store_ab(0, r);
        __syncthreads();
        load_frags(0, 0, 0);
        for (int kt = 0; kt < nk; ++kt) {
            load_ab(r);          // slice kt + 1
            slice(kt & 1, r);
        }
    } else if (nk > 0) {
        // two slices of global loads in flight; slices are consumed in pairs
        Staged r0, r1;
        load_ab(r0);
        load_ab(r1);
        store_ab(0, r0);
        __syncthreads();
        load_frags(0, 0, 0);
        const int nk2 = (nk + 1) & ~1;
        for (int kt = 0; kt < nk2; kt += 2) {
            load_ab(r0);         // slice kt + 2
            slice(0, r1);
            load_ab(r1);         // slice kt + 3
            slice(1, r0);
        }
    }
    const int64_t per_group = (int64_t)9 * C * C + C;
    float* PART = p.partial + ((int64_t)split * p.groups + group) * per_group;
    if (col_sums) {
        __syncthreads();   // the operand tiles are no longer read
        float* red = lds_all;
        red[threadIdx.x] = col_acc;
        __syncthreads();
        if (threadIdx.x < kBN && n0 + (int)threadIdx.x < C)
            PART[(int64_t)9 * C * C + n0 + threadIdx.x] = ((red[threadIdx.x] + red[64 + threadIdx.x]) + red[128 + threadIdx.x]) + red[192 + threadIdx.x];
    }
    const int col = n0 + wn0 + lane32;
    if (col < C) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int trow = wm0 + 32 * i + 8 * (r / 4) + 4 * half + (r % 4);   // 0 .. 191: (kw, ci inside the block)
                const int kw = trow / 64, row = m0 + trow % 64;
                if (row < C) PART[((int64_t)(kh * 3 + kw) * C + row) * C + col] = acc[i][r];
            }
        }
    }
}

// Sums the parts of every kernel / bias entry over the pixel ranges in range order and writes the gradient.  One lane per
// four consecutive entries (the kernel's and the bias's counts are multiples of four), eight ranges' loads in flight.
__global__ __launch_bounds__(256) void conv_dw_finish_kernel(const float* __restrict__ partial, int splits, int groups,
                                                             int64_t per_group, int64_t n_w, float* g, int64_t ld,
                                                             int64_t w_off, int64_t b_off) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= per_group) return;
    const int group = blockIdx.y;
    const float* P = partial + (int64_t)group * per_group + i;
    const int64_t step = (int64_t)groups * per_group;
    f4 s = {0.f, 0.f, 0.f, 0.f};
    constexpr int kFly = 8;
    for (int sp0 = 0; sp0 < splits; sp0 += kFly) {
        f4 v[kFly];
#pragma unroll
        for (int t = 0; t < kFly; ++t)
            v[t] = sp0 + t < splits ? __builtin_nontemporal_load((const f4*)(P + (sp0 + t) * step)) : f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < kFly; ++t)
            if (sp0 + t < splits) s = s + v[t];
    }
    float* dst = i < n_w ? g + (int64_t)group * ld + w_off + i : b_off >= 0 ? g + (int64_t)group * ld + b_off + (i - n_w) : nullptr;
    if (dst) {   // a convolution without bias has b_off < 0
#pragma unroll
        for (int e = 0; e < 4; ++e) dst[e] = s[e];
    }
}

// ---------------------------------------------------------------------------------------------
// global average pooling over the H W positions of every (group, sample), and its backward
// ---------------------------------------------------------------------------------------------
// pooled[g][b][c] = (1 / HW) sum_pos a[g][b][pos][c].  One workgroup per (sample, group); thread = (channel vector,
// position stripe); stripes are combined by a fixed-order LDS tree.
__global__ __launch_bounds__(256) void pool_mean_kernel(const float* __restrict__ a, int64_t s_a, float* pooled,
                                                        int64_t s_p, int HW, int C, float inv) {
    __shared__ f4 part[256];
    const int c4n = C / 4;                       // channel vectors (<= 64)
    const int stripes = 256 / c4n;               // >= 4
    const int c4 = threadIdx.x % c4n, stripe = threadIdx.x / c4n;
    const float* A = a + (int64_t)blockIdx.y * s_a + (int64_t)blockIdx.x * HW * C;
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    if (stripe < stripes)
        for (int pos = stripe; pos < HW; pos += stripes) acc = acc + *(const f4*)(A + (int64_t)pos * C + 4 * c4);
    part[threadIdx.x] = acc;
    __syncthreads();
    if (stripe == 0) {
        for (int s = 1; s < stripes; ++s) acc = acc + part[s * c4n + c4];
        f4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = acc[e] * inv;
        *(f4*)(pooled + (int64_t)blockIdx.y * s_p + (int64_t)blockIdx.x * C + 4 * c4) = o;
    }
}

// dz[g][b][pos][c] = dpool[g][b][c] / HW where a[g][b][pos][c] > 0, else 0 (through the mean and the ReLU in front of it)
__global__ __launch_bounds__(256) void pool_bwd_kernel(const float* __restrict__ dpool, int64_t s_dp,
                                                       const float* __restrict__ a, int64_t s_a, float* dz, int64_t s_dz,
                                                       int64_t vec_per_group, int HW, int C) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= vec_per_group) return;
    const int c4n = C / 4;
    const int64_t pixel = v / c4n;
    const int c4 = (int)(v % c4n);
    const int64_t sample = pixel / HW;
    const int g = blockIdx.y;
    const f4 av = __builtin_nontemporal_load((const f4*)(a + (int64_t)g * s_a) + v);
    const f4 d = *(const f4*)(dpool + (int64_t)g * s_dp + sample * C + 4 * c4);
    const float inv = 1.0f / (float)HW;
    f4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = av[e] > 0.0f ? d[e] * inv : 0.0f;
    *((f4*)(dz + (int64_t)g * s_dz) + v) = o;
}

bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

bool shape_ok(const ConvArgs& a) {
    if (a.groups < 1 || a.groups > 65535 || a.B < 1 || a.H < 1 || a.W < 1 || a.C < 16 || a.C % 16 != 0 || a.C > 4096) return false;
    const int64_t P = (int64_t)a.B * a.H * a.W;
    return P * a.C < ((int64_t)1 << 31) - ((int64_t)(a.W + 130) * a.C);   // 32-bit element offsets inside one group
}

template <int MODE>
hipError_t conv_launch(const ConvArgs& a, hipStream_t s) {
    if (!shape_ok(a) || !a.in || !a.w || !a.out || !aligned16(a.in) || !aligned16(a.w) || !aligned16(a.out)) return hipErrorInvalidValue;
    if (a.s_in % 4 || a.s_w % 4 || a.s_out % 4) return hipErrorInvalidValue;
    ConvDev p = {};
    p.in = a.in; p.w = a.w; p.out = a.out; p.bias = a.bias; p.residual = MODE == 0 ? a.residual : nullptr;
    p.mask = MODE == 1 ? a.mask : nullptr;
    p.s_in = a.s_in; p.s_w = a.s_w; p.s_out = a.s_out; p.s_bias = a.s_bias; p.s_res = a.s_res; p.s_mask = a.s_mask;
    p.groups = a.groups; p.B = a.B; p.H = a.H; p.W = a.W; p.C = a.C; p.P = a.B * a.H * a.W;
    p.relu = a.relu;
#ifndef OLS_CONV_BM
#define OLS_CONV_BM 128
#endif
#ifndef OLS_CONV_BK
#define OLS_CONV_BK 16
#endif
#ifndef OLS_CONV_DEPTH
#define OLS_CONV_DEPTH 2
#endif
    constexpr int BM = OLS_CONV_BM;
    p.tiles_m = (p.P + BM - 1) / BM;
    p.tiles_n = (a.C + kBN - 1) / kBN;
    const int64_t total = (int64_t)a.groups * p.tiles_m * p.tiles_n;
    if (total > (1 << 30)) return hipErrorInvalidValue;
    p.total_tiles = (int)total;
    p.chunk = (int)((total + kXcds - 1) / kXcds);
    const unsigned grid = (unsigned)(p.chunk * kXcds);
    if (a.C % OLS_CONV_BK == 0) conv3x3_kernel<MODE, BM, OLS_CONV_BK, OLS_CONV_DEPTH><<<grid, kThreads, 0, s>>>(p);
    else conv3x3_kernel<MODE, BM, 16, OLS_CONV_DEPTH><<<grid, kThreads, 0, s>>>(p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_conv3x3_fwd(const ConvArgs& a, hipStream_t s) { return conv_launch<0>(a, s); }
hipError_t launch_conv3x3_dx(const ConvArgs& a, hipStream_t s) { return conv_launch<1>(a, s); }

int conv3x3_dw_splits(int groups, int B, int H, int W, int C) {
    const int64_t P = (int64_t)B * H * W;
    const int64_t tiles = (int64_t)groups * 3 * ((C + 63) / 64) * ((C + 63) / 64);   // one per kernel row and 64 x 64 block
    int64_t s = (1536 + tiles - 1) / tiles;                 // about six workgroups per compute unit
    const int64_t most = (P + 1023) / 1024;                 // a range covers at least 1024 pixels
    if (s > most) s = most;
    if (s > 32) s = 32;
    return s < 1 ? 1 : (int)s;
}

hipError_t launch_conv3x3_dw(const ConvArgs& a, hipStream_t s) {
    if (!shape_ok(a) || !a.in || !a.dout || !a.partial || !a.g || !aligned16(a.in) || !aligned16(a.dout)) return hipErrorInvalidValue;
    if (a.s_in % 4 || a.s_dout % 4) return hipErrorInvalidValue;
    ConvDev p = {};
    p.in = a.in; p.dout = a.dout; p.partial = a.partial;
    p.s_in = a.s_in; p.s_dout = a.s_dout;
    p.groups = a.groups; p.B = a.B; p.H = a.H; p.W = a.W; p.C = a.C; p.P = a.B * a.H * a.W;
    p.splits = conv3x3_dw_splits(a.groups, a.B, a.H, a.W, a.C);
#ifndef OLS_CONV_DW_BK
#define OLS_CONV_DW_BK 16
#endif
#ifndef OLS_CONV_DW_DEPTH
#define OLS_CONV_DW_DEPTH 2
#endif
    constexpr int BK = OLS_CONV_DW_BK;
    p.k_chunk = (int)(((((int64_t)p.P + p.splits - 1) / p.splits) + BK - 1) / BK * BK);
    p.tiles_n = (a.C + 63) / 64;
    p.tiles_m = p.tiles_n;
    const int64_t total = (int64_t)a.groups * p.splits * 3 * p.tiles_n * p.tiles_n;
    if (total > (1 << 30)) return hipErrorInvalidValue;
    p.total_tiles = (int)total;
    p.chunk = (int)((total + kXcds - 1) / kXcds);
    conv3x3_dw_kernel<BK, OLS_CONV_DW_DEPTH><<<(unsigned)(p.chunk * kXcds), kThreads, 0, s>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_conv_dw_finish(a.partial, p.splits, a.groups, a.C, a.g, a.ld, a.g_w_off, a.g_b_off, s);
}

hipError_t launch_conv_dw_finish(const float* partial, int splits, int groups, int C, float* g, int64_t ld, int64_t w_off,
                                 int64_t b_off, hipStream_t s) {
    if (!partial || !g || splits < 1 || groups < 1 || groups > 65535 || C < 1) return hipErrorInvalidValue;
    const int64_t n_w = (int64_t)9 * C * C, per_group = n_w + C;
    if (C % 4 || (reinterpret_cast<uintptr_t>(partial) & 15u)) return hipErrorInvalidValue;
    dim3 grid((unsigned)((per_group / 4 + 255) / 256), (unsigned)groups);
    conv_dw_finish_kernel<<<grid, 256, 0, s>>>(partial, splits, groups, per_group, n_w, g, ld, w_off, b_off);
    return hipGetLastError();
}

hipError_t launch_pool_mean(const float* a, int64_t s_a, float* pooled, int64_t s_p, int groups, int B, int HW, int C,
                            float scale, hipStream_t s) {
    if (!a || !pooled || groups < 1 || groups > 65535 || B < 1 || HW < 1 || C < 4 || C % 4 || C > 256 || !aligned16(a) ||
        !aligned16(pooled) || s_a % 4 || s_p % 4)
        return hipErrorInvalidValue;
    pool_mean_kernel<<<dim3((unsigned)B, (unsigned)groups), 256, 0, s>>>(a, s_a, pooled, s_p, HW, C, scale);
    return hipGetLastError();
}

hipError_t launch_pool_bwd(const float* dpool, int64_t s_dp, const float* a, int64_t s_a, float* dz, int64_t s_dz,
                           int groups, int B, int HW, int C, hipStream_t s) {
    if (!dpool || !a || !dz || groups < 1 || groups > 65535 || B < 1 || HW < 1 || C < 4 || C % 4 || !aligned16(dpool) ||
        !aligned16(a) || !aligned16(dz) || s_dp % 4 || s_a % 4 || s_dz % 4)
        return hipErrorInvalidValue;
    const int64_t vecs = (int64_t)B * HW * (C / 4);
    const int64_t blocks = (vecs + 255) / 256;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    pool_bwd_kernel<<<dim3((unsigned)blocks, (unsigned)groups), 256, 0, s>>>(dpool, s_dp, a, s_a, dz, s_dz, vecs, HW, C);
    return hipGetLastError();
}

}  // namespace ols
