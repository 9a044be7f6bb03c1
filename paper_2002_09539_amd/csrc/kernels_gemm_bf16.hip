// Grouped GEMMs with bf16 operands and fp32 accumulation on the matrix cores
// (v_mfma_f32_32x32x16_bf16, gfx950) for the hidden layers of the per-worker MLPs, plus the fp32 ->
// bf16 conversion of the input batch.  One group per worker, all groups in one launch.
//
//   FWD  C[M][N] = relu(A[M][K] W[K][N] + bias[N])   A: bf16 activations; W: bf16 copy of the weights; C: bf16
//   DW   C[M][N] = A[K][M]^T B[K][N]                 A: bf16 activations, B: bf16 deltas (K = batch); C: fp32
//                                                    gradient, or consumed by the fused update
//   DA   C[M][N] = (A[M][K] W[N][K]^T) * [mask > 0]  A: bf16 delta; W rows are contiguous in K; C: bf16
//
// (forward / backward of the mini-batch loss whose gradient is the g_i of Section 2, arXiv 2002.09539;
// operands are rounded to bf16 with round-to-nearest-even, products and sums are fp32.)
//
// Every operand tile is copied global -> registers -> LDS in its own memory order with 16-byte vectors;
// nothing is transposed on the way and no transposed copies of activations or deltas exist in memory.
// The MFMA takes, per lane, 8 consecutive contraction indices of one row of an operand:
//   * an operand that is K-contiguous in memory ("KC", tile [rows][BK + 8]) yields a fragment as one
//     16-byte LDS read;
//   * an operand whose rows are contiguous ("RC", memory [K][rows], tile [BK][rows + 32]) yields it as two
//     LDS transpose reads (ds_read_b64_tr_b16): within each block of 16 lanes, lane j passes the address of
//     an 8-byte piece and lane i receives element i % 4 of the pieces of lanes i / 4, 4 + i / 4, 8 + i / 4,
//     12 + i / 4 (checked with an in-bounds probe).  With lane j pointing at row k0 + j / 4, columns
//     n0 + 4 (j % 4) .., lane i therefore receives column n0 + i of rows k0 .. k0 + 3: four consecutive k.
// Row paddings keep both read patterns free of bank conflicts.
//
// The forward and delta GEMMs use 256 x 128 tiles with four wavefronts of 128 x 64: the per-wavefront
// tile sets the LDS traffic per MFMA (6 fragment reads per 8 MFMAs), and at batch 256 one tile row spans
// the whole batch so that each weight panel is fetched from HBM exactly once.  Fragment reads run one
// k-step ahead of the MFMAs, and two K slices of global loads are in flight.  The weight-gradient GEMM is
// bound by the HBM traffic of the fused update in its epilogue, not by the contraction (K = batch), and
// uses 128 x 128 tiles so that several workgroups share a compute unit and overlap their phases.
#include <type_traits>

#include "gemm_bf16_tile.h"
#include "gemm_epilogue.h"
#include "head_dw_body.h"
#include "ols_internal.h"

namespace ols {


enum GemmMode { kFwd = 0, kDw = 1, kDa = 2 };

constexpr int kThreads = kTileThreads;
constexpr int kXcds = 8;
// Lanes of the full-tile forward / delta kernel.  Eight wavefronts of 64 x 64 (two per SIMD, which cover each other's
// LDS waits, at 4/3 of the fragment bytes per MFMA) against four of 128 x 64, measured on 256 x 128 tiles at batch 256:
// delta GEMM (both operands K-contiguous, 16-byte fragment reads) 48.7 against 54.0 us, forward GEMM (weights read with
// the 8-byte transpose loads, twice as many read instructions per byte) 58.4 against 54.5 us, the same with the eight
// wavefronts laid out 2 x 4 (128 x 32 each) instead of 4 x 2.
template <int MODE, int BM>
constexpr int full_tile_threads() { return (MODE == kDa && BM == 256) ? 512 : 256; }

__device__ __forceinline__ unsigned int bf16_rne(float f) { return bf16_bits_rne(f); }
__device__ __forceinline__ float bf16_to_f32(unsigned int h) { return __uint_as_float(h << 16); }

struct GemmDevB {
    const uint16_t* a;
    const uint16_t* b;
    void* c;
    const float* bias;
    const uint16_t* mask;
    float* colsum;
    FusedUpdate upd;     // DW: update applied in the epilogue instead of storing the gradient
    int64_t upd_w_off, upd_b_off;
    int64_t sa, sb, sc, sbias, smask, scolsum;
    int M, N, K, lda, ldb, ldc;
    int tiles_m, tiles_n, total_tiles, chunk;
    HeadDwDev guest;     // DW: output-layer gradients computed by the first guest.blocks workgroups (0: none)
};

template <int MODE, int BM, int BN, int BK, int THREADS = kThreads>
struct GemmShape {
    using TA = typename std::conditional<MODE == kDw, TileRC<BM, BK, THREADS>, TileKC<BM, BK, THREADS>>::type;   // FWD, DA: A[M][K]; DW: A[K][M]
    using TB = typename std::conditional<MODE == kDa, TileKC<BN, BK, THREADS>, TileRC<BN, BK, THREADS>>::type;   // DA: W[N][K]; FWD, DW: B[K][N]
    static constexpr int kOperandElems = 2 * TA::kElems + 2 * TB::kElems;
    static constexpr int kStagePitch = BN + 8;            // bf16 output tile staged for 16-byte stores
    static constexpr int kStageElems = MODE == kDw ? 0 : BM * kStagePitch;
    static constexpr int kLdsElems = kOperandElems > kStageElems ? kOperandElems : kStageElems;
    static constexpr size_t kLdsBytes = (size_t)kLdsElems * sizeof(uint16_t);
};

template <int MODE, int BM, int BN, int BK, int DEPTH>
__global__ __launch_bounds__(kThreads) void gemm_bf16_kernel(GemmDevB p) {
    constexpr int WM = BM / 2, WN = BN / 2;     // 2 x 2 wavefronts
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int S = BK / 16;                  // MFMA steps per K slice
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 32 == 0, "tile shape");
    static_assert(DEPTH == 1 || DEPTH == 2, "global prefetch distance in K slices");
    using Shape = GemmShape<MODE, BM, BN, BK>;
    using TA = typename Shape::TA;
    using TB = typename Shape::TB;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds_all[];
    auto lds_a = [&](int buf) { return lds_all + buf * TA::kElems; };
    auto lds_b = [&](int buf) { return lds_all + 2 * TA::kElems + buf * TB::kElems; };

    // Guest workgroups come first in the launch, so they start at once and their latency-bound work runs
    // beside the tiles of the GEMM.  Their number is a multiple of 8: the tiles keep their XCD assignment.
    int bid = blockIdx.x;
    if (MODE == kDw) {
        if (bid < p.guest.blocks) {
            head_dw_guest<(int)(Shape::kLdsBytes / sizeof(float))>(p.guest, (float*)lds_all, bid);
            return;
        }
        bid -= p.guest.blocks;
    }
    // XCD-aware tile id: hardware deals workgroup b to XCD b % 8; give each XCD a contiguous tile range
    const int xcd = bid % kXcds, slot = bid / kXcds;
    const int tile = xcd * p.chunk + slot;
    if (slot >= p.chunk || tile >= p.total_tiles) return;
    const int per_group = p.tiles_m * p.tiles_n;
    const int group = tile / per_group;
    const int tm = (tile % per_group) / p.tiles_n, tn = tile % p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const uint16_t* A = p.a + (int64_t)group * p.sa;
    const uint16_t* B = p.b + (int64_t)group * p.sb;

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

    // DW with the fused update: the tile's parameters (and momentum) can be requested here, ahead of the contraction
    constexpr int kDwPf = MODE == kDw ? OLS_DW_PREFETCH : 0;
    constexpr int kDwFit = ((Shape::kLdsElems / 2) / (BN + 4)) / 32 * 32;
    constexpr int kDwRP = kDwFit >= BM ? BM : (kDwFit >= 64 ? 64 : 32);   // rows per staging pass of the epilogue
    DwState<BM * BN / 4 / kThreads> dw_state;
    DwOut dw_out;
    if constexpr (MODE == kDw) {
        dw_out.g = (float*)p.c + (int64_t)group * p.sc;
        dw_out.ldg = p.ldc;
        dw_out.upd = p.upd;
        dw_out.upd_base = (int64_t)group * p.upd.ld + p.upd_w_off;
        dw_out.col_base = p.upd_w_off;
        dw_prefetch_state<BM, BN, kDwRP, kThreads, kDwPf>(dw_state, dw_out, m0, n0, p.M, p.N);
    }

    // DW only: the tiles of the first tile row also sum each column of B (a delta column over the batch),
    // which is the bias gradient of the layer, in sample order.
    const bool col_sums = MODE == kDw && p.colsum != nullptr && tm == 0 && threadIdx.x < BN;
    float col_acc = 0.0f;

    // Fragment registers are double-buffered across k-steps, and the order "issue the LDS reads of step
    // s + 1, then the MFMAs of step s" is pinned with scheduling barriers: a wavefront stalls at the issue
    // of an MFMA while the matrix pipe is busy, so reads placed behind the MFMAs would start only when the
    // pipe is about to drain and their latency would be exposed on every step.
    static_assert(S % 2 == 0, "an even number of k-steps per slice");
    bf16x8 fa[2][TM], fb[2][TN];
    auto load_frags = [&](int buf, int cur, int s) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[buf][i] = TA::frag(lds_a(cur), wm0 + 32 * i, s, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[buf][j] = TB::frag(lds_b(cur), wn0 + 32 * j, s, lane);
    };
    auto mfmas = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
    };
    // One K slice out of lds[cur].  On entry the fragments of step 0 are already in (or on their way to)
    // buffer 0.  Before the last step's MFMAs the staged registers of the next slice are published to
    // lds[cur ^ 1], the workgroup synchronises once, and the first fragments of that slice are requested,
    // so the barrier and the LDS latency hide behind the remaining MFMAs.
    auto slice = [&](int cur, const u4 (&na)[TA::kPerThread], unsigned oka, const u4 (&nb)[TB::kPerThread],
                     unsigned okb) {
#pragma unroll
        for (int s = 0; s + 1 < S; ++s) {
            load_frags((s + 1) & 1, cur, s + 1);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(s & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (MODE == kDw && col_sums) {
#pragma unroll
            for (int k = 0; k < BK; ++k) col_acc += bf16_to_f32(lds_b(cur)[k * TB::kPitch + threadIdx.x]);
        }
        TA::store(lds_a(cur ^ 1), na, oka);
        TB::store(lds_b(cur ^ 1), nb, okb);
        __syncthreads();
        load_frags(0, cur ^ 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfmas((S - 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
    };

    // The loop bodies below are free of data-dependent branches: loads past the end of K are zero-filled
    // dummies and the tile published after the last slice is never consumed.
    const int nk = (p.K + BK - 1) / BK;
    if constexpr (MODE == kDw && DEPTH == 1) {
        // Both operands are [K][.] with K the row: the descriptor's range check zero-fills the rows from K on, and a lane
        // whose columns lie past M (N) gets an offset beyond any range once, outside the loop -- so a slice's loads are
        // one instruction per vector, with no predicates, selects or 64-bit address arithmetic (with eight slices of four
        // MFMAs per wavefront those were most of the loop's instructions).
        static_assert(TA::kVecs % kThreads == 0 && TB::kVecs % kThreads == 0, "whole vectors per lane");
        const rsrc_t a_rs = make_rsrc(A, (unsigned)p.K * (unsigned)p.lda * 2u), b_rs = make_rsrc(B, (unsigned)p.K * (unsigned)p.ldb * 2u);
        constexpr unsigned kOut = 0x80000000u;   // beyond every range the launcher admits
        unsigned a_off[TA::kPerThread], b_off[TB::kPerThread];
#pragma unroll
        for (int t = 0; t < TA::kPerThread; ++t) {
            const int v = threadIdx.x + t * kThreads, col = m0 + (v % TA::kVecPerLine) * 8;
            a_off[t] = col < p.M ? 2u * ((unsigned)(v / TA::kVecPerLine) * (unsigned)p.lda + col) : kOut;
        }
#pragma unroll
        for (int t = 0; t < TB::kPerThread; ++t) {
            const int v = threadIdx.x + t * kThreads, col = n0 + (v % TB::kVecPerLine) * 8;
            b_off[t] = col < p.N ? 2u * ((unsigned)(v / TB::kVecPerLine) * (unsigned)p.ldb + col) : kOut;
        }
        const unsigned a_step = 2u * BK * (unsigned)p.lda, b_step = 2u * BK * (unsigned)p.ldb;   // bytes per K slice
        u4 ra[TA::kPerThread], rb[TB::kPerThread];
        auto load_ab = [&](int kt) {
#pragma unroll
            for (int t = 0; t < TA::kPerThread; ++t) ra[t] = buf_load(a_rs, a_off[t] + kt * a_step, 0u);
#pragma unroll
            for (int t = 0; t < TB::kPerThread; ++t) rb[t] = buf_load(b_rs, b_off[t] + kt * b_step, 0u);
        };
        load_ab(0);
        TA::store(lds_a(0), ra, ~0u);
        TB::store(lds_b(0), rb, ~0u);
        __syncthreads();
        load_frags(0, 0, 0);
        for (int kt = 0; kt < nk; ++kt) {
            load_ab(kt + 1);   // past the last slice: zeros, published and never read
            slice(kt & 1, ra, ~0u, rb, ~0u);
        }
    } else if (DEPTH == 1) {
        u4 ra[TA::kPerThread], rb[TB::kPerThread];
        unsigned oka = TA::load(ra, A, p.lda, m0, 0, p.M, p.K);
        unsigned okb = TB::load(rb, B, p.ldb, n0, 0, p.N, p.K);
        TA::store(lds_a(0), ra, oka);
        TB::store(lds_b(0), rb, okb);
        __syncthreads();
        load_frags(0, 0, 0);
        for (int kt = 0; kt < nk; ++kt) {
            oka = TA::load(ra, A, p.lda, m0, (kt + 1) * BK, p.M, p.K);
            okb = TB::load(rb, B, p.ldb, n0, (kt + 1) * BK, p.N, p.K);
            slice(kt & 1, ra, oka, rb, okb);
        }
    } else {
        // Two K slices of global loads in flight: while slice t feeds the matrix cores from LDS, slice
        // t + 1 waits in registers and slice t + 2 is on its way from HBM.  Slices are consumed in pairs; an
        // odd trailing slice is paired with an all-zero one.
        u4 ra0[TA::kPerThread], rb0[TB::kPerThread], ra1[TA::kPerThread], rb1[TB::kPerThread];
        unsigned oka0 = TA::load(ra0, A, p.lda, m0, 0, p.M, p.K);
        unsigned okb0 = TB::load(rb0, B, p.ldb, n0, 0, p.N, p.K);
        unsigned oka1 = TA::load(ra1, A, p.lda, m0, BK, p.M, p.K);
        unsigned okb1 = TB::load(rb1, B, p.ldb, n0, BK, p.N, p.K);
        TA::store(lds_a(0), ra0, oka0);
        TB::store(lds_b(0), rb0, okb0);
        __syncthreads();
        load_frags(0, 0, 0);
        const int nk2 = (nk + 1) & ~1;
        for (int kt = 0; kt < nk2; kt += 2) {
            oka0 = TA::load(ra0, A, p.lda, m0, (kt + 2) * BK, p.M, p.K);
            okb0 = TB::load(rb0, B, p.ldb, n0, (kt + 2) * BK, p.N, p.K);
            slice(0, ra1, oka1, rb1, okb1);
            oka1 = TA::load(ra1, A, p.lda, m0, (kt + 3) * BK, p.M, p.K);
            okb1 = TB::load(rb1, B, p.ldb, n0, (kt + 3) * BK, p.N, p.K);
            slice(1, ra0, oka0, rb0, okb0);
        }
    }

    if constexpr (MODE == kDw) {
        if (col_sums && n0 + (int)threadIdx.x < p.N) {
            if (p.upd.enabled) {   // bias: gradient is the sum just formed
                const int64_t col = p.upd_b_off + n0 + threadIdx.x, idx = (int64_t)group * p.upd.ld + col;
                fused_update_apply(p.upd, idx, col, col_acc, p.upd.x_in[idx], p.upd.mu != 0.0f ? p.upd.buf[idx] : 0.0f);
            } else {
                p.colsum[(int64_t)group * p.scolsum + n0 + threadIdx.x] = col_acc;
            }
        }
        // the gradient tile is staged through the (now idle) operand LDS, as many rows per pass as it holds
        static_assert(kDwFit >= 32 && BM % kDwRP == 0, "operand LDS too small to stage the gradient tile");
        dw_epilogue_staged<BM, BN, TM, TN, kDwRP, kThreads, kDwPf>((float*)lds_all, acc, dw_out, m0, n0, wm0, wn0, p.M, p.N, &dw_state);
    } else {
        // Epilogue of FWD / DA: the bf16 tile goes through LDS so that every lane then moves 16-byte vectors
        // of 8 consecutive columns (output, and the activations whose sign gates the delta).  Accumulator
        // register r of a lane is C[row][col] with col = lane % 32 and row = 8 (r / 4) + 4 (lane / 32) + r % 4
        // inside its 32 x 32 block.
        constexpr int SP = Shape::kStagePitch;
        __syncthreads();   // the tile published after the last slice is not read; everyone is past the loop
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int cl = wn0 + 32 * j + lane32;
                float bias = 0.0f;
                if (MODE == kFwd && n0 + cl < p.N) bias = p.bias[(int64_t)group * p.sbias + n0 + cl];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rl = wm0 + 32 * i + 8 * (r / 4) + 4 * half + (r % 4);
                    float v = acc[i][j][r];
                    if (MODE == kFwd) v = fmaxf(v + bias, 0.0f);
                    lds_all[rl * SP + cl] = (uint16_t)bf16_rne(v);
                }
            }
        }
        __syncthreads();
        constexpr int kVecPerRow = BN / 8, kVecs = BM * kVecPerRow;
        static_assert(kVecs % kThreads == 0, "output tile vectors per lane");
        uint16_t* C = (uint16_t*)p.c + (int64_t)group * p.sc;
        const uint16_t* Mk = MODE == kDa ? p.mask + (int64_t)group * p.smask : nullptr;
#pragma unroll 4
        for (int t = 0; t < kVecs / kThreads; ++t) {
            const int v = threadIdx.x + t * kThreads;
            const int row = m0 + v / kVecPerRow, col = n0 + (v % kVecPerRow) * 8;
            if (row < p.M && col < p.N) {   // N is a multiple of 8
                u4 o = *(const u4*)(lds_all + (v / kVecPerRow) * SP + (v % kVecPerRow) * 8);
                if (MODE == kDa) {
                    const u4 mk = *(const u4*)(Mk + (int64_t)row * p.ldc + col);
#pragma unroll
                    for (int w = 0; w < 4; ++w) {   // a bf16 is positive iff its sign bit is clear and it is not zero
                        const unsigned int lo = mk[w] & 0xFFFFu, hi = mk[w] >> 16;
                        const unsigned int keep = ((lo != 0u && lo < 0x8000u) ? 0xFFFFu : 0u) |
                                                  ((hi != 0u && hi < 0x8000u) ? 0xFFFF0000u : 0u);
                        o[w] &= keep;
                    }
                }
                *(u4*)(C + (int64_t)row * p.ldc + col) = o;
            }
        }
    }
}


// ---------------------------------------------------------------------------------------------
// FWD / DA on full tiles: M % BM == 0, N % BN == 0, K % (NSETS BK) == 0.  One workgroup per compute unit with one
// or two wavefronts per SIMD (THREADS = 256 or 512): little else is resident to fill a stall, and a wavefront that
// has just issued an MFMA cannot issue the next one for 32 cycles, so every other instruction of the loop (fragment
// reads, the next slices' global loads, the LDS stores of the staged slice) is placed BETWEEN the MFMAs, one or
// two per MFMA, with scheduling-group barriers.  Per K slice of 64 and wavefront of 128 x 64: 32 MFMAs, 32 fragment
// reads, 12 global loads, 12 LDS stores, one workgroup barrier; addresses are one lane offset plus
// wave-uniform bases, so the loop has no vector address arithmetic.
// ---------------------------------------------------------------------------------------------
template <int MODE, int BM, int BN, int BK, int NSETS, int THREADS>
__global__ __launch_bounds__(THREADS) void gemm_bf16_full_kernel(GemmDevB p) {
    static_assert(MODE != kDw && BK == 64, "forward / delta GEMM, four k-steps per slice");
    static_assert(NSETS % 2 == 0, "the LDS buffer of a slice is its parity");
    constexpr int kWaveRows = THREADS / 128;    // wavefronts: kWaveRows x 2
    constexpr int WM = BM / kWaveRows, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    using Shape = GemmShape<MODE, BM, BN, BK, THREADS>;
    using TA = typename Shape::TA;
    using TB = typename Shape::TB;
    constexpr int NA = TA::kPerThread, NB = TB::kPerThread;
    static_assert(TA::kVecs % THREADS == 0 && TB::kVecs % THREADS == 0, "whole vectors per lane");
    extern __shared__ __attribute__((aligned(16))) uint16_t lds_all[];
    auto lds_a = [&](int buf) { return lds_all + buf * TA::kElems; };
    auto lds_b = [&](int buf) { return lds_all + 2 * TA::kElems + buf * TB::kElems; };

    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int tile = xcd * p.chunk + slot;
    if (slot >= p.chunk || tile >= p.total_tiles) return;
    const int per_group = p.tiles_m * p.tiles_n;
    const int group = tile / per_group;
    const int tm = (tile % per_group) / p.tiles_n, tn = tile % p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    // tile origins of slice 0 (wave-uniform byte pointers)
    const char* a_tile = (const char*)(p.a + (int64_t)group * p.sa + (int64_t)m0 * p.lda);
    const char* b_tile = (const char*)(p.b + (int64_t)group * p.sb + (MODE == kFwd ? (int64_t)n0 : (int64_t)n0 * p.ldb));
    const unsigned off_a = TA::lane_offset_bytes(p.lda), off_b = TB::lane_offset_bytes(p.ldb);
    const int64_t line_a = TA::line_step_bytes(p.lda), line_b = TB::line_step_bytes(p.ldb);
    const int64_t step_a = TA::slice_step_bytes(p.lda), step_b = TB::slice_step_bytes(p.ldb);

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

    bf16x8 fa[2][TM], fb[2][TN];
    auto load_frags = [&](int buf, int cur, int s) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[buf][i] = TA::frag(lds_a(cur), wm0 + 32 * i, s, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[buf][j] = TB::frag(lds_b(cur), wn0 + 32 * j, s, lane);
    };
    auto mfmas = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
    };
    auto load_a = [&](u4 (&r)[NA], const char* base) {
#pragma unroll
        for (int t = 0; t < NA; ++t) r[t] = *(const u4*)(base + t * line_a + off_a);
    };
    auto load_b = [&](u4 (&r)[NB], const char* base) {
#pragma unroll
        for (int t = 0; t < NB; ++t) r[t] = *(const u4*)(base + t * line_b + off_b);
    };
    auto store_a = [&](int buf, const u4 (&r)[NA]) {
        uint16_t* q = TA::lane_lds(lds_a(buf));
#pragma unroll
        for (int t = 0; t < NA; ++t) *(u4*)(q + t * TA::kLdsLineStep) = r[t];
    };
    auto store_b = [&](int buf, const u4 (&r)[NB]) {
        uint16_t* q = TB::lane_lds(lds_b(buf));
#pragma unroll
        for (int t = 0; t < NB; ++t) *(u4*)(q + t * TB::kLdsLineStep) = r[t];
    };
    // scheduling groups: one MFMA, then `reads` LDS reads, `writes` LDS writes, `loads` global loads
    constexpr int kMfmas = TM * TN;
#define OLS_INTERLEAVE(reads, writes, loads)                                        \
    _Pragma("unroll") for (int q = 0; q < kMfmas; ++q) {                            \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          \
        if ((reads) > 0) __builtin_amdgcn_sched_group_barrier(0x100, (reads), 0);   \
        if ((writes) > 0) __builtin_amdgcn_sched_group_barrier(0x200, (writes), 0); \
        if ((loads) > 0) __builtin_amdgcn_sched_group_barrier(0x020, (loads), 0);   \
    }
    constexpr int kReads = (TM + 2 * TN + kMfmas - 1) / kMfmas;          // LDS reads per MFMA (an RC fragment is two reads)
    constexpr int kLoads = (NA + NB + kMfmas - 1) / kMfmas;
    constexpr int kWrites = (NA + NB + kMfmas - 1) / kMfmas;
    // One K slice out of lds[cur]: fragments of step 0 are in buffer 0 on entry.  The register set `r` holds
    // the NEXT slice (requested NSETS slices ago): it is published to lds[cur ^ 1] during step 0 and the
    // same registers then request the slice NSETS further on during step 1.  lds[cur ^ 1] was last read
    // before the previous slice's barrier, so it may be overwritten from the start of this slice.
    auto slice = [&](int cur, u4 (&r_a)[NA], u4 (&r_b)[NB], const char* next_a, const char* next_b) {
        load_frags(1, cur, 1);
        store_a(cur ^ 1, r_a);
        store_b(cur ^ 1, r_b);
        mfmas(0);
        OLS_INTERLEAVE(kReads, kWrites, 0)
        __builtin_amdgcn_sched_barrier(0);
        load_frags(0, cur, 2);
        load_a(r_a, next_a);
        load_b(r_b, next_b);
        mfmas(1);
        OLS_INTERLEAVE(kReads, 0, kLoads)
        __builtin_amdgcn_sched_barrier(0);
        load_frags(1, cur, 3);
        mfmas(0);
        OLS_INTERLEAVE(kReads, 0, 0)
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        load_frags(0, cur ^ 1, 0);
        mfmas(1);
        OLS_INTERLEAVE(kReads, 0, 0)
        __builtin_amdgcn_sched_barrier(0);
    };
#undef OLS_INTERLEAVE

    // NSETS register sets form a ring: at the start of slice t they hold slices t + 1 .. t + NSETS (landed or
    // on their way), so every load has NSETS - 1 slice times to arrive.
    const int nk = p.K / BK;   // a multiple of NSETS
    u4 ra[NSETS][NA], rb[NSETS][NB];
    load_a(ra[0], a_tile);
    load_b(rb[0], b_tile);
#pragma unroll
    for (int u = 1; u < NSETS; ++u) {
        load_a(ra[u], a_tile + u * step_a);
        load_b(rb[u], b_tile + u * step_b);
    }
    store_a(0, ra[0]);
    store_b(0, rb[0]);
    {
        const int kn = NSETS < nk ? NSETS : 0;   // set 0 is free again: it takes slice NSETS
        load_a(ra[0], a_tile + kn * step_a);
        load_b(rb[0], b_tile + kn * step_b);
    }
    __syncthreads();
    load_frags(0, 0, 0);
    for (int kt = 0; kt < nk; kt += NSETS) {
#pragma unroll
        for (int u = 0; u < NSETS; ++u) {
            // this slice is t = kt + u; it publishes slice t + 1 (set (u + 1) % NSETS) and requests slice
            // t + 1 + NSETS into the same set; slices past the end re-read slice 0 (in bounds, never consumed)
            const int tn = kt + u + 1 + NSETS;
            const int kn = tn < nk ? tn : 0;
            slice(u & 1, ra[(u + 1) % NSETS], rb[(u + 1) % NSETS], a_tile + kn * step_a, b_tile + kn * step_b);
        }
    }

    // Epilogue: the bf16 tile goes through LDS so that every lane then moves 16-byte vectors of 8 consecutive
    // columns.  Accumulator register r of a lane is C[row][col] with col = lane % 32 and
    // row = 8 (r / 4) + 4 (lane / 32) + r % 4 inside its 32 x 32 block.
    constexpr int SP = Shape::kStagePitch;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int cl = wn0 + 32 * j + lane32;
            float bias = 0.0f;
            if (MODE == kFwd) bias = p.bias[(int64_t)group * p.sbias + n0 + cl];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rl = wm0 + 32 * i + 8 * (r / 4) + 4 * half + (r % 4);
                float v = acc[i][j][r];
                if (MODE == kFwd) v = fmaxf(v + bias, 0.0f);
                lds_all[rl * SP + cl] = (uint16_t)bf16_rne(v);
            }
        }
    }
    __syncthreads();
    constexpr int kVecPerRow = BN / 8, kVecs = BM * kVecPerRow;
    uint16_t* C = (uint16_t*)p.c + (int64_t)group * p.sc + (int64_t)m0 * p.ldc + n0;
    const uint16_t* Mk = MODE == kDa ? p.mask + (int64_t)group * p.smask + (int64_t)m0 * p.ldc + n0 : nullptr;
#pragma unroll 4
    for (int t = 0; t < kVecs / THREADS; ++t) {
        const int v = threadIdx.x + t * THREADS;
        const int rl = v / kVecPerRow, cl = (v % kVecPerRow) * 8;
        u4 o = *(const u4*)(lds_all + rl * SP + cl);
        if (MODE == kDa) {
            const u4 mk = *(const u4*)(Mk + (int64_t)rl * p.ldc + cl);
#pragma unroll
            for (int w = 0; w < 4; ++w) {   // a bf16 is positive iff its sign bit is clear and it is not zero
                const unsigned int lo = mk[w] & 0xFFFFu, hi = mk[w] >> 16;
                const unsigned int keep = ((lo != 0u && lo < 0x8000u) ? 0xFFFFu : 0u) |
                                          ((hi != 0u && hi < 0x8000u) ? 0xFFFF0000u : 0u);
                o[w] &= keep;
            }
        }
        *(u4*)(C + (int64_t)rl * p.ldc + cl) = o;
    }
}

static bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

template <int MODE, int BM, int BN, int BK, int DEPTH>
static hipError_t gemm_launch(const GemmArgs& g, hipStream_t s) {
    if (!g.a || !g.b || !g.c || g.groups < 1 || g.M < 1 || g.N < 1 || g.K < 1) return hipErrorInvalidValue;
    // 16-byte vectors of 8 bf16 along each operand's contiguous dimension: aligned bases, leading
    // dimensions and extents in multiples of 8
    if (!aligned16(g.a) || !aligned16(g.b) || g.lda % 8 || g.ldb % 8 || g.sa % 8 || g.sb % 8) return hipErrorInvalidValue;
    if (MODE == kDw) {   // A[K][M], B[K][N]
        if (g.M % 8 || g.N % 8 || g.lda < g.M || g.ldb < g.N) return hipErrorInvalidValue;
        // 32-bit byte offsets inside a group's operand, with room for the slice requested past the end of K
        if (((int64_t)g.K + 2 * BK) * g.lda >= ((int64_t)1 << 29) || ((int64_t)g.K + 2 * BK) * g.ldb >= ((int64_t)1 << 29)) return hipErrorInvalidValue;
    } else {
        if (g.K % 8 || g.N % 8 || g.lda < g.K) return hipErrorInvalidValue;
        if (MODE == kFwd && (g.ldb < g.N || !g.bias)) return hipErrorInvalidValue;
        if (MODE == kDa && (g.ldb < g.K || !g.mask || !aligned16(g.mask) || g.smask % 8)) return hipErrorInvalidValue;
        if (!aligned16(g.c) || g.ldc % 8 || g.sc % 8) return hipErrorInvalidValue;
    }
    if (g.ldc < g.N) return hipErrorInvalidValue;
    GemmDevB p = {};
    if (g.guest) {
        if (MODE != kDw) return hipErrorInvalidValue;
        hipError_t ge = head_dw_prepare(*g.guest, &p.guest);
        if (ge != hipSuccess) return ge;
    }
    p.a = (const uint16_t*)g.a;
    p.b = (const uint16_t*)g.b;
    p.c = g.c;
    p.bias = g.bias;
    p.mask = (const uint16_t*)g.mask;
    p.colsum = MODE == kDw ? g.colsum : nullptr;
    p.upd = g.upd;
    p.upd_w_off = g.upd_w_off;
    p.upd_b_off = g.upd_b_off;
    if (MODE != kDw) p.upd.enabled = 0;
    if (p.upd.enabled) {
        if (!p.upd.x_in || !p.upd.x_out || (p.upd.mu != 0.0f && !p.upd.buf) || (p.upd.pull && !p.upd.z) || !g.colsum ||
            g.ldc != g.N)
            return hipErrorInvalidValue;
    }
    p.sa = g.sa; p.sb = g.sb; p.sc = g.sc; p.sbias = g.sbias; p.smask = g.smask;
    p.scolsum = g.scolsum;
    p.M = g.M; p.N = g.N; p.K = g.K; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc;
    p.tiles_m = (g.M + BM - 1) / BM;
    p.tiles_n = (g.N + BN - 1) / BN;
    const int64_t total = (int64_t)g.groups * p.tiles_m * p.tiles_n;
    if (total > (1 << 30)) return hipErrorInvalidValue;
    p.total_tiles = (int)total;
    p.chunk = (int)((total + kXcds - 1) / kXcds);
    constexpr size_t lds = GemmShape<MODE, BM, BN, BK>::kLdsBytes;
    static_assert(lds <= 160 * 1024, "LDS of a compute unit");
    void (*kern)(GemmDevB) = gemm_bf16_kernel<MODE, BM, BN, BK, DEPTH>;
    unsigned threads = kThreads;
    if constexpr (MODE != kDw && BK == 64) {
        // full tiles and 32-bit lane offsets: the branch-free, interleaved kernel
        // Register sets of operand slices in flight.  Four sets (three slices of lead time) were measured equal to
        // two on configuration 3 (also with eight wavefronts: 50.9 against 49.7 us): the loop is bound by the LDS pipe
        // (fragment reads + tile stores), not by load latency.
        constexpr int kSets = 2;
        const bool full = g.M % BM == 0 && g.N % BN == 0 && g.K % (kSets * BK) == 0 &&
                          (int64_t)BM * g.lda < (1 << 29) && (int64_t)(MODE == kFwd ? BK : BN) * g.ldb < (1 << 29);
        if (full && !g.force_general) {
            constexpr int kFullThreads = full_tile_threads<MODE, BM>();
            kern = gemm_bf16_full_kernel<MODE, BM, BN, BK, kSets, kFullThreads>;
            threads = kFullThreads;
        }
    }
    if (lds > 64 * 1024) {
        hipError_t e = ensure_dynamic_lds((const void*)kern, lds);
        if (e != hipSuccess) return e;
    }
    kern<<<(unsigned)(p.guest.blocks + p.chunk * kXcds), threads, lds, s>>>(p);
    return hipGetLastError();
}

// Tile choice.  Small problems (few rows per group) take 128 x 128 tiles: a 256-row tile would be mostly padding.
hipError_t launch_gemm_bf16_fwd(const GemmArgs& g, hipStream_t s) {
    if (g.M > 128) return gemm_launch<kFwd, 256, 128, 64, 2>(g, s);
    return gemm_launch<kFwd, 128, 128, 64, 2>(g, s);
}
hipError_t launch_gemm_bf16_da(const GemmArgs& g, hipStream_t s) {
    if (g.M > 128) return gemm_launch<kDa, 256, 128, 64, 2>(g, s);
    return gemm_launch<kDa, 128, 128, 64, 2>(g, s);
}
hipError_t launch_gemm_bf16_dw(const GemmArgs& g, hipStream_t s, int variant) {
    // Measured on configuration 3 (K = batch = 256, fused update): 64 x 128 x 32 tiles leave four workgroups per
    // compute unit and take 284 us per launch; 128 x 128: 309, 128 x 64: 294, 64 x 64: 295, BK = 64: 319-341.
    switch (variant) {
        case 0:
        case 1: return gemm_launch<kDw, 64, 128, 32, 1>(g, s);
#ifdef OLS_TUNING_VARIANTS
        case 6: return gemm_launch<kDw, 128, 128, 32, 1>(g, s);
        case 2: return gemm_launch<kDw, 128, 64, 32, 1>(g, s);
        case 3: return gemm_launch<kDw, 64, 64, 32, 1>(g, s);
        case 4: return gemm_launch<kDw, 128, 128, 64, 1>(g, s);
        case 5: return gemm_launch<kDw, 64, 128, 64, 1>(g, s);
#endif
        default: return hipErrorInvalidValue;
    }
}

// ---------------------------------------------------------------------------------------------
// fp32 [groups][rows][cols] -> bf16 [groups][rows][cols]; one lane per 8 consecutive values
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void cast_bf16_kernel(const float* __restrict__ src, int64_t src_stride,
                                                             uint16_t* __restrict__ dst, int64_t per_group8) {
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (v >= per_group8) return;
    const int g = blockIdx.y;
    const f4* S = (const f4*)(src + (int64_t)g * src_stride) + 2 * v;
    const f4 lo = __builtin_nontemporal_load(S), hi = __builtin_nontemporal_load(S + 1);
    u4 o;
    o.x = bf16_rne(lo.x) | (bf16_rne(lo.y) << 16);
    o.y = bf16_rne(lo.z) | (bf16_rne(lo.w) << 16);
    o.z = bf16_rne(hi.x) | (bf16_rne(hi.y) << 16);
    o.w = bf16_rne(hi.z) | (bf16_rne(hi.w) << 16);
    *((u4*)(dst + (int64_t)g * per_group8 * 8) + v) = o;
}

hipError_t launch_cast_bf16(const float* src, int64_t src_stride, uint16_t* dst, int groups, int rows, int cols,
                            hipStream_t s) {
    if (!src || !dst || groups < 1 || groups > 65535 || rows < 1 || cols < 8 || cols % 8) return hipErrorInvalidValue;
    if (!aligned16(src) || !aligned16(dst) || src_stride % 4) return hipErrorInvalidValue;
    const int64_t per_group8 = (int64_t)rows * cols / 8;
    const int64_t blocks = (per_group8 + kThreads - 1) / kThreads;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks, (unsigned)groups);
    cast_bf16_kernel<<<grid, kThreads, 0, s>>>(src, src_stride, dst, per_group8);
    return hipGetLastError();
}

}  // namespace ols
