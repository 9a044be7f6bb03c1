// Grouped fp32 GEMMs on the matrix cores (v_mfma_f32_32x32x2_f32) for the hidden layers of the
// per-worker MLPs: one group per worker, all groups in one launch.
//
//   FWD  C[M][N] = relu(A[M][K] W[K][N] + bias[N])      activations; A rows are samples
//   DW   C[M][N] = A[K][M]^T B[K][N]                     weight gradient; contraction over the batch
//   DA   C[M][N] = (A[M][K] B[N][K]^T) * [mask > 0]      back-propagated delta through ReLU
//
// (forward / backward of the mini-batch loss whose gradient is the g_i of Section 2, arXiv 2002.09539.)
//
// Tiling: a workgroup of four wavefronts owns a BM x BN output tile; each wavefront owns TM x TN blocks
// of 32 x 32 held in accumulator registers.  K is consumed in slices of BK staged through LDS in the
// operands' own memory order with 16-byte vector copies, double-buffered so that the global loads of
// slice t+1 are in flight while slice t feeds the matrix cores.  An operand whose contraction index is
// contiguous in memory ("KC") is read from LDS as one 16-byte vector per lane that serves four
// consecutive MFMA steps; an operand whose row index is contiguous ("RC") is read one dword per step.
// Both use the same lane -> k assignment (k = 8 q + 4 (lane / 32) + e), which is all the contraction
// needs.  Row padding keeps both read patterns free of LDS bank conflicts.
//
// Workgroup ids are remapped so that consecutive tiles of one worker land on the same XCD (workgroups
// are dealt round-robin to the 8 XCDs, each with its own L2), keeping a worker's weights in one L2.
#include "gemm_epilogue.h"
#include "gemm_f32_tile.h"
#include "head_dw_body.h"
#include "ols_internal.h"

namespace ols {

enum GemmMode { kFwd = 0, kDw = 1, kDa = 2 };

constexpr int kThreads = kGemmThreads;
constexpr int kXcds = 8;

struct GemmDev {
    const float* a;
    const float* b;
    float* c;
    const float* bias;
    const float* mask;
    float* colsum;
    int64_t sa, sb, sc, sbias, smask, scolsum;
    float* partial;      // split-K: raw partial sums [split][group][M][N]
    FusedUpdate upd;     // DW: update applied in the epilogue instead of storing the gradient
    int64_t upd_w_off, upd_b_off;
    int M, N, K, lda, ldb, ldc;
    int tiles_m, tiles_n, total_tiles, chunk;
    int splits, k_chunk, groups;
    int wgs_per_xcd;     // persistent weight-gradient kernel: workgroups per XCD (each walks several tiles)
    HeadDwDev guest;     // DW: output-layer gradients computed by the first guest.blocks workgroups (0: none)
};

template <int MODE, int BM, int BN, int BK, int WAVES_M, int WAVES_N, int DEPTH, bool FULL>
__global__ __launch_bounds__(kThreads) void gemm_f32_kernel(GemmDev p) {
    constexpr bool A_KC = MODE != kDw;   // FWD, DA: A[M][K];  DW: A[K][M]
    constexpr bool B_KC = MODE == kDa;   // DA: B[N][K];  FWD, DW: B[K][N]
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    static_assert(WAVES_M * WAVES_N * 64 == kThreads, "four wavefronts");
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 8 == 0, "tile shape");
    static_assert(DEPTH == 1 || DEPTH == 2, "global prefetch distance in K slices");
    using TA = Tile<BM, BK, A_KC>;
    using TB = Tile<BN, BK, B_KC>;
    constexpr int kLdsFloats = 2 * TA::kFloats + 2 * TB::kFloats;
    __shared__ __attribute__((aligned(16))) float lds_all[kLdsFloats];
    auto lds_a = [&](int buf) { return lds_all + buf * TA::kFloats; };
    auto lds_b = [&](int buf) { return lds_all + 2 * TA::kFloats + buf * TB::kFloats; };

    // Guest workgroups come first in the launch, so they start at once and their latency-bound work runs
    // beside the tiles of the GEMM.  Their number is a multiple of 8: the tiles keep their XCD assignment.
    int bid = blockIdx.x;
    if (MODE == kDw) {
        if (bid < p.guest.blocks) {
            head_dw_guest<kLdsFloats>(p.guest, lds_all, bid);
            return;
        }
        bid -= p.guest.blocks;
    }
    // XCD-aware tile id: hardware deals workgroup b to XCD b % 8; give each XCD a contiguous tile range
    const int xcd = bid % kXcds, slot = bid / kXcds;
    const int tile = xcd * p.chunk + slot;
    if (slot >= p.chunk || tile >= p.total_tiles) return;
    const int per_split = p.tiles_m * p.tiles_n, per_group = per_split * p.splits;
    const int group = tile / per_group;
    const int split = (tile % per_group) / per_split;
    const int tm = (tile % per_split) / p.tiles_n, tn = tile % p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    // split-K: this workgroup contracts over [k_lo, k_hi) only and leaves a raw partial sum
    const int k_lo = split * p.k_chunk, k_hi = min(p.K, k_lo + p.k_chunk);

    const float* A = p.a + (int64_t)group * p.sa;
    const float* B = p.b + (int64_t)group * p.sb;

    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int lane32 = lane % 32, half = lane / 32;
    const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;

    f16v acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // DW only: the tiles of the first tile row also reduce the columns of B over the batch, which is
    // the bias gradient of the layer (sum over samples of the delta), in sample order.
    const bool col_sums = MODE == kDw && p.colsum != nullptr && tm == 0 && threadIdx.x < BN;
    float col_acc = 0.0f;

    // Fragment registers are double-buffered across k-octets, and the order "issue the LDS reads of
    // octet q+1, then the MFMAs of octet q" is pinned with scheduling barriers: a wavefront stalls at
    // the issue of an MFMA while the matrix pipe is busy, so reads placed behind the MFMAs would start
    // only when the pipe is about to drain and their latency would be exposed on every octet.
    constexpr int Q = BK / 8;
    static_assert(Q % 2 == 0, "BK must be a multiple of 16");
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
    // One K slice out of lds[cur].  On entry the fragments of octet 0 are already in (or on their way
    // to) buffer 0.  Before the last octet's MFMAs the staged registers of the next slice are published
    // to lds[cur ^ 1], the workgroup synchronises once, and the first fragments of that slice are
    // requested, so the barrier and the LDS latency hide behind the remaining MFMAs.
    auto slice = [&](int cur, const f4 (&na)[TA::kPerThread], unsigned oka, const f4 (&nb)[TB::kPerThread],
                     unsigned okb) {
        (void)oka;
        (void)okb;
#pragma unroll
        for (int q = 0; q + 1 < Q; ++q) {
            load_frags((q + 1) & 1, cur, q + 1);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(q & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (MODE == kDw && col_sums) {
#pragma unroll
            for (int k = 0; k < BK; ++k) col_acc += lds_b(cur)[k * TB::kPitch + threadIdx.x];
        }
        if (FULL) {
            TA::store_full(lds_a(cur ^ 1), na);
            TB::store_full(lds_b(cur ^ 1), nb);
        } else {
            TA::store(lds_a(cur ^ 1), na, oka);
            TB::store(lds_b(cur ^ 1), nb, okb);
        }
        __syncthreads();
        load_frags(0, cur ^ 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfmas((Q - 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
    };

    // The loop bodies below are free of data-dependent branches: loads past the end of the K range are
    // zero-filled dummies and the tile published after the last slice is never consumed.
    const int nk = (k_hi - k_lo + BK - 1) / BK;
    if constexpr (FULL) {
        // uniform bases of slice 0 and per-lane byte offsets; slices past the end re-read the last one (what
        // they publish is never consumed)
        unsigned offa[TA::kPerThread], offb[TB::kPerThread];
        TA::lane_offsets(offa, p.lda);
        TB::lane_offsets(offb, p.ldb);
        const char* a0 = (const char*)(A + (A_KC ? (int64_t)m0 * p.lda + k_lo : (int64_t)k_lo * p.lda + m0));
        const char* b0 = (const char*)(B + (B_KC ? (int64_t)n0 * p.ldb + k_lo : (int64_t)k_lo * p.ldb + n0));
        const int64_t sa = 4 * TA::slice_step(p.lda), sb = 4 * TB::slice_step(p.ldb);
        auto base_a = [&](int sl) { return a0 + (int64_t)min(sl, nk - 1) * sa; };
        auto base_b = [&](int sl) { return b0 + (int64_t)min(sl, nk - 1) * sb; };
        if (DEPTH == 1) {
            f4 ra[TA::kPerThread], rb[TB::kPerThread];
            TA::load_full(ra, base_a(0), offa);
            TB::load_full(rb, base_b(0), offb);
            TA::store_full(lds_a(0), ra);
            TB::store_full(lds_b(0), rb);
            __syncthreads();
            load_frags(0, 0, 0);
            for (int kt = 0; kt < nk; ++kt) {
                TA::load_full(ra, base_a(kt + 1), offa);
                TB::load_full(rb, base_b(kt + 1), offb);
                slice(kt & 1, ra, 0u, rb, 0u);
            }
        } else {
            // A ring of DEPTH register sets: while slice t feeds the matrix cores from LDS, slices t + 1 .. t + DEPTH - 1
            // wait in registers and slice t + DEPTH is requested into the set that slice t left.  (Four sets were
            // measured no faster than two at the same bytes in flight, and slower at twice the bytes; so was a K order
            // rotated per tile to spread concurrent workgroups over memory channels.)
            f4 ra[DEPTH][TA::kPerThread], rb[DEPTH][TB::kPerThread];
#pragma unroll
            for (int j = 0; j < DEPTH; ++j) {
                TA::load_full(ra[j], base_a(j), offa);
                TB::load_full(rb[j], base_b(j), offb);
            }
            TA::store_full(lds_a(0), ra[0]);
            TB::store_full(lds_b(0), rb[0]);
            __syncthreads();
            load_frags(0, 0, 0);
            for (int kt = 0; kt < nk; kt += DEPTH) {   // nk is a multiple of DEPTH
#pragma unroll
                for (int u = 0; u < DEPTH; ++u) {
                    TA::load_full(ra[u], base_a(kt + u + DEPTH), offa);
                    TB::load_full(rb[u], base_b(kt + u + DEPTH), offb);
                    slice(u & 1, ra[(u + 1) % DEPTH], 0u, rb[(u + 1) % DEPTH], 0u);
                }
            }
        }
    } else if (DEPTH == 1) {
        f4 ra[TA::kPerThread], rb[TB::kPerThread];
        unsigned oka = TA::load(ra, A, p.lda, m0, k_lo, p.M, k_hi);
        unsigned okb = TB::load(rb, B, p.ldb, n0, k_lo, p.N, k_hi);
        TA::store(lds_a(0), ra, oka);
        TB::store(lds_b(0), rb, okb);
        __syncthreads();
        load_frags(0, 0, 0);
        for (int kt = 0; kt < nk; ++kt) {
            oka = TA::load(ra, A, p.lda, m0, k_lo + (kt + 1) * BK, p.M, k_hi);
            okb = TB::load(rb, B, p.ldb, n0, k_lo + (kt + 1) * BK, p.N, k_hi);
            slice(kt & 1, ra, oka, rb, okb);
        }
    } else {
        // Two K slices of global loads in flight: while slice t feeds the matrix cores from LDS, slice
        // t+1 waits in registers and slice t+2 is on its way from HBM.  Slices are consumed in pairs; an
        // odd trailing slice is paired with an all-zero one.
        f4 ra0[TA::kPerThread], rb0[TB::kPerThread], ra1[TA::kPerThread], rb1[TB::kPerThread];
        unsigned oka0 = TA::load(ra0, A, p.lda, m0, k_lo, p.M, k_hi);
        unsigned okb0 = TB::load(rb0, B, p.ldb, n0, k_lo, p.N, k_hi);
        unsigned oka1 = TA::load(ra1, A, p.lda, m0, k_lo + BK, p.M, k_hi);
        unsigned okb1 = TB::load(rb1, B, p.ldb, n0, k_lo + BK, p.N, k_hi);
        TA::store(lds_a(0), ra0, oka0);
        TB::store(lds_b(0), rb0, okb0);
        __syncthreads();
        load_frags(0, 0, 0);
        const int nk2 = (nk + 1) & ~1;
        for (int kt = 0; kt < nk2; kt += 2) {
            oka0 = TA::load(ra0, A, p.lda, m0, k_lo + (kt + 2) * BK, p.M, k_hi);
            okb0 = TB::load(rb0, B, p.ldb, n0, k_lo + (kt + 2) * BK, p.N, k_hi);
            slice(0, ra1, oka1, rb1, okb1);
            oka1 = TA::load(ra1, A, p.lda, m0, k_lo + (kt + 3) * BK, p.M, k_hi);
            okb1 = TB::load(rb1, B, p.ldb, n0, k_lo + (kt + 3) * BK, p.N, k_hi);
            slice(1, ra0, oka0, rb0, okb0);
        }
    }
    if (MODE == kDw && col_sums && n0 + (int)threadIdx.x < p.N) {
        if (p.upd.enabled) {   // bias: gradient is the column sum just formed
            const int64_t col = p.upd_b_off + n0 + threadIdx.x, idx = (int64_t)group * p.upd.ld + col;
            fused_update_apply(p.upd, idx, col, col_acc, p.upd.x_in[idx], p.upd.mu != 0.0f ? p.upd.buf[idx] : 0.0f);
        } else {
            p.colsum[(int64_t)group * p.scolsum + n0 + threadIdx.x] = col_acc;
        }
    }
    if (MODE == kDw && p.upd.enabled) {
        // rows of the tile staged per pass: as many as the operand LDS holds
        constexpr int kFit = (kLdsFloats / (BN + 4)) / 32 * 32;
        constexpr int RP = kFit >= BM ? BM : kFit;
        static_assert(RP >= 32, "operand LDS too small to stage the gradient tile");
        DwOut o;
        o.g = p.c + (int64_t)group * p.sc;
        o.ldg = p.ldc;
        o.upd = p.upd;
        o.upd_base = (int64_t)group * p.upd.ld + p.upd_w_off;
        o.col_base = p.upd_w_off;
        dw_epilogue_staged<BM, BN, TM, TN, RP, kThreads>(lds_all, acc, o, m0, n0, wm0, wn0, p.M, p.N);
        return;
    }

    // Epilogue.  Accumulator register r of a lane holds C[row][col] with col = lane % 32 and
    // row = 8 (r / 4) + 4 (lane / 32) + r % 4 inside its 32 x 32 block.
    const bool raw = MODE == kFwd && p.splits > 1;
    float* C = raw ? p.partial + ((int64_t)split * p.groups + group) * p.M * p.N : p.c + (int64_t)group * p.sc;
    const int ldc = raw ? p.N : p.ldc;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn0 + 32 * j + lane32;
            if (col >= p.N) continue;
            float bias = 0.0f;
            if (MODE == kFwd && !raw) bias = p.bias[(int64_t)group * p.sbias + col];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm0 + 32 * i + 8 * (r / 4) + 4 * half + (r % 4);
                if (row >= p.M) continue;
                float v = acc[i][j][r];
                if (MODE == kFwd && !raw) v = fmaxf(v + bias, 0.0f);
                if (MODE == kDa) v = p.mask[(int64_t)group * p.smask + (int64_t)row * p.ldc + col] > 0.0f ? v : 0.0f;
                C[(int64_t)row * ldc + col] = v;
            }
        }
    }
}

// Weight gradient with the fused update as a persistent, software-pipelined kernel.
//
// In gemm_f32_kernel a workgroup first contracts (matrix cores busy, HBM idle), then streams the state of its
// tile (HBM busy, matrix cores idle); whether the two phases of different workgroups overlap is left to chance.
// Here a workgroup walks over several 64 x 64 tiles, and the update of tile t - 1 is spread over the K loop of
// tile t: the gradient tile waits transposed in its own LDS region, and every quarter of the K loop ("group")
// consumes one 16-byte vector per lane of it -- whose parameters and momenta were requested two groups earlier --
// and requests another.  Every wavefront therefore issues MFMAs and state traffic all the time.  The operand
// ring runs across tile boundaries as well, so the first slices of the next tile are on their way while the
// last ones of this tile feed the matrix cores.
//   group g of tile t:   consume vector g of tile t - 1;   request vector g + 2 of tile t - 1 (g < 2)
//                                                          or vector g - 2 of tile t     (g >= 2)
// Two register sets of state vectors alternate.  K = 64 SPG (SPG slices of 16 per group); full tiles only;
// same MFMA order and same update arithmetic as gemm_f32_kernel + dw_epilogue_staged, so identical bits.
struct DwTile {
    int group, tm, m0, n0;
    int64_t upd_base;   // group * ld + w_off + m0 * N + n0: element (m0, n0) of this worker's weight matrix
    int64_t col_base;   // w_off + m0 * N + n0: the same inside a replica row (anchor)
};

#ifndef OLS_DWP_WAVES
#define OLS_DWP_WAVES 4
#endif
template <bool V>
struct DwFlag {
    static constexpr bool value = V;
};
// The hardware counts a wavefront's outstanding vector-memory operations in issue order: waiting for an operand
// slice also waits for every state load and store issued before that slice was requested.  The number of memory
// operations between a request and its wait must therefore not depend on run-time branches (the compiler assumes
// the shortest path and would wait for operations that are still young on the longer one): momentum and pull-back
// are template parameters, and the first tile of a workgroup, which has no predecessor to update, is its own copy
// of the loop body.  Measured on 16 x (3072 x 512, K = 128): 101.6 -> 99.8 us per launch.  Measured without gain
// on top of that: four operand register sets (state traffic gets three slices of time before an operand wait
// reaches it; 98.8 us at three wavefronts per SIMD), four state register sets (a whole tile of state in flight,
// requested during the tile's own K loop; 100.6 us) and a state layout in which a tile's 4096 elements are
// contiguous (100.8 us).  Knock-out builds (wrong values on purpose, same memory touched) split the 100 us: state
// traffic alone 77 us (5.6 TB/s), + the operand loads 94 us (393 MB of L2 hits cost 17 us, half of them 9 us),
// + the MFMAs 100 us; operands + MFMAs without the state traffic take 61 us.  The three parts add up rather than
// overlap, and the matrix work hides all but 6 us.  The cost of the operand loads is not their L2 traffic: a
// generalisation of this kernel to 128 x 64 tiles (a quarter less operand traffic, two workgroups per compute unit,
// identical bits) measured 96.8 us against 96.4 us for 64 x 64 tiles and is not in the tree.
template <int SPG, bool PULL, bool MOM>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(OLS_DWP_WAVES)))
void gemm_f32_dw_pipelined_kernel(GemmDev p) {
    constexpr int RING = 2;   // register sets of the operand ring
    constexpr int BM = 64, BN = 64, BK = 16, NK = 4 * SPG;   // four 16-byte vectors per lane of a 64 x 64 tile
    static_assert(NK % RING == 0 && RING % 2 == 0, "register set and LDS buffer of a slice are static");
    using TA = Tile<BM, BK, false>;   // A[K][M]
    using TB = Tile<BN, BK, false>;   // B[K][N]
    static_assert(TA::kPerThread == 1 && TB::kPerThread == 1, "one 16-byte vector per lane and operand slice");
    constexpr int kOperand = 2 * TA::kFloats + 2 * TB::kFloats;
    constexpr int kPitch = BN + 4;
    __shared__ __attribute__((aligned(16))) float lds_all[kOperand + BM * kPitch];
    float* stage = lds_all + kOperand;
    auto lds_a = [&](int buf) { return lds_all + buf * TA::kFloats; };
    auto lds_b = [&](int buf) { return lds_all + 2 * TA::kFloats + buf * TB::kFloats; };

    int bid = blockIdx.x;
    if (bid < p.guest.blocks) {
        head_dw_guest<kOperand + BM * kPitch>(p.guest, lds_all, bid);
        return;
    }
    bid -= p.guest.blocks;
    // workgroup `slot` of XCD `xcd` walks tiles xcd * chunk + slot, + k_chunk (workgroups per XCD), ...
    const int xcd = bid % kXcds, slot = bid / kXcds, stride = p.wgs_per_xcd;
    const int tile_end = min((xcd + 1) * p.chunk, p.total_tiles);
    int tile = xcd * p.chunk + slot;
    if (tile >= tile_end) return;
    const int per_group = p.tiles_m * p.tiles_n;
    const FusedUpdate& u = p.upd;

    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, lane32 = lane % 32, half = lane / 32;
    const int wm0 = (wave / 2) * 32, wn0 = (wave % 2) * 32;

    auto decode = [&](int t) {
        DwTile d;
        d.group = t / per_group;
        d.tm = (t % per_group) / p.tiles_n;
        d.m0 = d.tm * BM;
        d.n0 = (t % p.tiles_n) * BN;
        d.col_base = p.upd_w_off + (int64_t)d.m0 * p.N + d.n0;
        d.upd_base = (int64_t)d.group * u.ld + d.col_base;
        return d;
    };
    // operand slice s of tile d: uniform base pointers; the lane's 16-byte vector sits at a fixed offset
    unsigned offa[1], offb[1];
    TA::lane_offsets(offa, p.lda);
    TB::lane_offsets(offb, p.ldb);
    auto load_slice = [&](f4 (&ra)[1], f4 (&rb)[1], const DwTile& d, int sl) {
        const char* a = (const char*)(p.a + (int64_t)d.group * p.sa + (int64_t)(sl * BK) * p.lda + d.m0);
        const char* b = (const char*)(p.b + (int64_t)d.group * p.sb + (int64_t)(sl * BK) * p.ldb + d.n0);
        TA::load_full(ra, a, offa);
        TB::load_full(rb, b, offb);
    };

    // state vector v of a tile: row v * 16 + tid / 16, columns 4 (tid % 16) .. + 3 of the tile; addresses are a
    // uniform base per tile plus a 32-bit byte offset per lane
    const int my_row = threadIdx.x / 16, my_c4 = threadIdx.x % 16;
    const unsigned my_off = 4u * (unsigned)(my_row * p.N + 4 * my_c4);   // byte offset of vector 0 inside the tile
    const unsigned vec_step = 64u * (unsigned)p.N;                        // bytes between consecutive vectors of a lane
    const float* my_stage = stage + my_row * kPitch + 4 * my_c4;
    f4 sx[2], sb[MOM ? 2 : 1], sz[PULL ? 2 : 1];
    auto issue = [&](int set, const DwTile& d, int v) {
        const unsigned o = my_off + (unsigned)v * vec_step;
        sx[set] = ep_load_stream((const ep_f4*)((const char*)(u.x_in + d.upd_base) + o));
        if (MOM) sb[MOM ? set : 0] = ep_load_stream((const ep_f4*)((const char*)(u.buf + d.upd_base) + o));
        if (PULL) sz[PULL ? set : 0] = *(const ep_f4*)((const char*)(u.z + d.col_base) + o);
    };
    auto consume = [&](int set, const DwTile& d, int v) {
        const f4 gv = *(const f4*)(my_stage + v * 16 * kPitch);
        const unsigned o = my_off + (unsigned)v * vec_step;
        f4 xn, bn;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float be = MOM ? sb[MOM ? set : 0][e] : 0.0f;
            xn[e] = local_step_elem(gv[e], sx[set][e], be, PULL ? sz[PULL ? set : 0][e] : 0.0f, u.gamma, u.mu, u.alpha, MOM,
                                    u.nesterov != 0, PULL);
            bn[e] = be;
        }
        ep_store_stream((ep_f4*)((char*)(u.x_out + d.upd_base) + o), xn);
        if (MOM) ep_store_stream((ep_f4*)((char*)(u.buf + d.upd_base) + o), bn);
    };

    f16v acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
    f4 fa[2], fb[2];
    auto load_frags = [&](int buf, int cur, int q) {
        fa[buf] = TA::frag(lds_a(cur), wm0, q, lane32, half);
        fb[buf] = TB::frag(lds_b(cur), wn0, q, lane32, half);
    };
    auto mfmas = [&](int buf) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[buf][e], fb[buf][e], acc, 0, 0, 0);
    };

    DwTile cur = decode(tile), prev = cur;
    f4 ra[RING][1], rb[RING][1];
#pragma unroll
    for (int j = 0; j < RING; ++j) load_slice(ra[j], rb[j], cur, j);
    TA::store_full(lds_a(0), ra[0]);
    TB::store_full(lds_b(0), rb[0]);
    __syncthreads();
    load_frags(0, 0, 0);

    // one tile: its K loop with the update of the previous tile (if there is one) spread over it; returns whether
    // the workgroup has another tile, in which case `cur` is that tile and its slice 0 is in LDS buffer 0
    auto run_tile = [&](auto have_prev_flag) -> bool {
        constexpr bool kHavePrev = decltype(have_prev_flag)::value;
        const int next_tile = tile + stride;
        const bool has_next = next_tile < tile_end;
        const DwTile nxt = decode(has_next ? next_tile : tile);
        const bool col_sums = p.colsum != nullptr && cur.tm == 0 && threadIdx.x < BN;
        float col_acc = 0.0f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if (kHavePrev) consume(g & 1, prev, g);
            if (g < 2) {
                if (kHavePrev) issue(g & 1, prev, g + 2);
            } else {
                issue(g & 1, cur, g - 2);
            }
#pragma unroll
            for (int ss = 0; ss < SPG; ++ss) {
                const int s = g * SPG + ss;          // static after unrolling
                const int lb = s & 1;                // LDS buffer holding slice s
                const int rs = s % RING;             // its register set is free again
                // operand slice RING jobs ahead: this tile's, the next tile's, or (at the very end) a dummy re-read
                if (s + RING < NK) load_slice(ra[rs], rb[rs], cur, s + RING);
                else load_slice(ra[rs], rb[rs], has_next ? nxt : cur, has_next ? s + RING - NK : NK - 1);
                load_frags(1, lb, 1);
                __builtin_amdgcn_sched_barrier(0);
                mfmas(0);
                __builtin_amdgcn_sched_barrier(0);
                if (col_sums) {
#pragma unroll
                    for (int k = 0; k < BK; ++k) col_acc += lds_b(lb)[k * TB::kPitch + threadIdx.x];
                }
                TA::store_full(lds_a(lb ^ 1), ra[(s + 1) % RING]);   // the next job (possibly slice 0 of the next tile)
                TB::store_full(lds_b(lb ^ 1), rb[(s + 1) % RING]);
                __syncthreads();
                if (s + 1 < NK) {
                    load_frags(0, lb ^ 1, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    mfmas(1);
                    __builtin_amdgcn_sched_barrier(0);
                } else {
                    mfmas(1);   // the tile's last MFMAs: the accumulators are complete after them
                }
            }
        }
        // bias gradient of the tiles of the first tile row: the column sums just formed, updated on the spot
        if (col_sums) {
            const int64_t col = p.upd_b_off + cur.n0 + threadIdx.x, idx = (int64_t)cur.group * u.ld + col;
            fused_update_apply(u, idx, col, col_acc, u.x_in[idx], MOM ? u.buf[idx] : 0.0f);
        }
        // Every lane has read its last vector of the previous gradient tile (group 3, at least one barrier ago):
        // the stage takes this tile's gradient, transposed so that lanes own 16-byte vectors of rows.
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            stage[(wm0 + 8 * (r / 4) + 4 * half + (r % 4)) * kPitch + wn0 + lane32] = acc[r];
            acc[r] = 0.0f;
        }
        __syncthreads();
        prev = cur;
        if (!has_next) return false;
        tile = next_tile;
        cur = nxt;
        load_frags(0, 0, 0);   // slice 0 of the new tile was published to LDS buffer 0 by the last job above
        return true;
    };
    bool more = run_tile(DwFlag<false>{});
    while (more) more = run_tile(DwFlag<true>{});
    // drain: the last tile's update (vectors 0 and 1 were requested during its last two groups)
    consume(0, prev, 0);
    issue(0, prev, 2);
    consume(1, prev, 1);
    issue(1, prev, 3);
    consume(0, prev, 2);
    consume(1, prev, 3);
}

// out[g][row][col] = relu(sum_s partial[s][g][row][col] + bias[g][col]); one lane per 4 columns
__global__ __launch_bounds__(kThreads) void splitk_finish_kernel(const f4* __restrict__ partial, int splits,
                                                                 const float* __restrict__ bias, int64_t sbias,
                                                                 float* __restrict__ out, int64_t sc, int ldc, int groups,
                                                                 int M, int N) {
    const int n4 = N / 4;
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t per_split = (int64_t)groups * M * n4;
    if (v >= per_split) return;
    const int c4 = (int)(v % n4);
    const int row = (int)((v / n4) % M);
    const int g = (int)(v / ((int64_t)n4 * M));
    f4 acc = partial[v];
    for (int s = 1; s < splits; ++s) acc = acc + partial[(int64_t)s * per_split + v];
    const f4 b = *(const f4*)(bias + (int64_t)g * sbias + 4 * c4);
    f4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = fmaxf(acc[e] + b[e], 0.0f);
    *(f4*)(out + (int64_t)g * sc + (int64_t)row * ldc + 4 * c4) = r;
}

static bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

template <int MODE, int BM, int BN, int BK, int WAVES_M, int WAVES_N, int DEPTH>
static hipError_t gemm_launch(const GemmArgs& g, hipStream_t s) {
    if (!g.a || !g.b || !g.c || g.groups < 1 || g.M < 1 || g.N < 1 || g.K < 1) return hipErrorInvalidValue;
    // 16-byte vector loads: every line start must be aligned and extents multiples of 4
    if (!aligned16(g.a) || !aligned16(g.b) || g.lda % 4 || g.ldb % 4 || g.sa % 4 || g.sb % 4) return hipErrorInvalidValue;
    const bool a_kc = MODE != kDw, b_kc = MODE == kDa;
    if ((a_kc ? g.K : g.M) % 4 || (b_kc ? g.K : g.N) % 4) return hipErrorInvalidValue;
    if (g.lda < (a_kc ? g.K : g.M) || g.ldb < (b_kc ? g.K : g.N) || g.ldc < g.N) return hipErrorInvalidValue;
    if (MODE == kFwd && !g.bias) return hipErrorInvalidValue;
    if (MODE == kDa && !g.mask) return hipErrorInvalidValue;
    GemmDev p = {};
    if (g.guest) {
        if (MODE != kDw) return hipErrorInvalidValue;
        hipError_t ge = head_dw_prepare(*g.guest, &p.guest);
        if (ge != hipSuccess) return ge;
    }
    p.a = (const float*)g.a;
    p.b = (const float*)g.b;
    p.c = (float*)g.c;
    p.bias = g.bias;
    p.mask = (const float*)g.mask;
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
    p.sa = g.sa; p.sb = g.sb; p.sc = g.sc; p.sbias = g.sbias; p.smask = g.smask; p.scolsum = g.scolsum;
    p.M = g.M; p.N = g.N; p.K = g.K; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc;
    p.tiles_m = (g.M + BM - 1) / BM;
    p.tiles_n = (g.N + BN - 1) / BN;
    p.groups = g.groups;
    p.splits = 1;
    p.k_chunk = g.K;
    p.partial = nullptr;
    if (MODE == kFwd && g.splits > 1) {
        if (!g.partial) return hipErrorInvalidValue;
        p.k_chunk = (int)round_up((g.K + g.splits - 1) / g.splits, BK);
        p.splits = (g.K + p.k_chunk - 1) / p.k_chunk;   // never an empty split
        p.partial = g.partial;
    }
    const int64_t total = (int64_t)g.groups * p.splits * p.tiles_m * p.tiles_n;
    if (total > (1 << 30)) return hipErrorInvalidValue;
    p.total_tiles = (int)total;
    p.chunk = (int)((total + kXcds - 1) / kXcds);
    // Full tiles, K ranges that are whole (for DEPTH 2: even) numbers of slices, and operands small enough for
    // 32-bit lane offsets take the kernel without bounds checks; same arithmetic, identical bits.
    constexpr bool a_kc_ = MODE != kDw, b_kc_ = MODE == kDa;
    // (measured: forward GEMM 74.5 -> 71.7 us on configuration 2, 259 -> 242 us on 5; the weight-gradient kernel, whose
    // few K slices are not where its time goes, was 1 % slower with it and keeps the bounds-checked loop)
    constexpr bool kCanFull = MODE != kDw && Tile<BM, BK, a_kc_>::kVecs % kThreads == 0 &&
                              Tile<BN, BK, b_kc_>::kVecs % kThreads == 0;
    const int q = DEPTH * BK;
    const bool full = kCanFull && !g.force_general && g.M % BM == 0 && g.N % BN == 0 && p.k_chunk % q == 0 &&
                      (g.K % p.k_chunk) % q == 0 && g.lda < (1 << 22) && g.ldb < (1 << 22);
    const unsigned grid = (unsigned)(p.guest.blocks + p.chunk * kXcds);
    if constexpr (kCanFull) {
        if (full) gemm_f32_kernel<MODE, BM, BN, BK, WAVES_M, WAVES_N, DEPTH, true><<<grid, kThreads, 0, s>>>(p);
    }
    if (!full) gemm_f32_kernel<MODE, BM, BN, BK, WAVES_M, WAVES_N, DEPTH, false><<<grid, kThreads, 0, s>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits == 1) return e;
    // second pass of a split-K forward GEMM: sum the partials, add the bias, apply the ReLU
    const int64_t vecs = (int64_t)g.groups * g.M * (g.N / 4);
    splitk_finish_kernel<<<(unsigned)((vecs + kThreads - 1) / kThreads), kThreads, 0, s>>>(
        (const f4*)p.partial, p.splits, g.bias, g.sbias, (float*)g.c, g.sc, g.ldc, g.groups, g.M, g.N);
    return hipGetLastError();
}

// persistent workgroups per compute unit: measured 16 x (3072 x 512, K = 128): one 125 us, two 97.4 us, three 98.9 us,
// four 99.7 us per launch
#ifndef OLS_DWP_WGS_PER_CU
#define OLS_DWP_WGS_PER_CU 2
#endif
// shapes the persistent pipelined weight-gradient kernel covers: fused update, full 64 x 64 tiles, K = 64, 128 or 256
static bool dw_pipelined_fits(const GemmArgs& g) {
    if (!g.upd.enabled || g.M % 64 || g.N % 64 || (g.K != 64 && g.K != 128 && g.K != 256)) return false;
    if (g.lda % 4 || g.ldb % 4 || g.sa % 4 || g.sb % 4 || g.ldc != g.N || g.lda >= (1 << 22) || g.ldb >= (1 << 22)) return false;
    if ((int64_t)g.M * g.N >= ((int64_t)1 << 30)) return false;   // 32-bit element offsets inside a weight matrix
    if (!aligned16(g.a) || !aligned16(g.b) || !aligned16(g.upd.x_in) || !aligned16(g.upd.x_out) || !aligned16(g.upd.buf) ||
        !aligned16(g.upd.z) || g.upd.shadow || g.upd_w_off % 4 || g.upd.ld % 4)   // fp32 GEMMs keep no bf16 copy
        return false;
    return true;
}
static hipError_t dw_pipelined_launch(const GemmArgs& g, hipStream_t s) {
    if (!g.a || !g.b || g.groups < 1 || !dw_pipelined_fits(g)) return hipErrorInvalidValue;
    if (!g.upd.x_in || !g.upd.x_out || (g.upd.mu != 0.0f && !g.upd.buf) || (g.upd.pull && !g.upd.z) || !g.colsum)
        return hipErrorInvalidValue;
    if (g.lda < g.M || g.ldb < g.N) return hipErrorInvalidValue;
    GemmDev p = {};
    if (g.guest) {
        hipError_t ge = head_dw_prepare(*g.guest, &p.guest);
        if (ge != hipSuccess) return ge;
    }
    p.a = (const float*)g.a;
    p.b = (const float*)g.b;
    p.colsum = g.colsum;
    p.upd = g.upd;
    p.upd_w_off = g.upd_w_off;
    p.upd_b_off = g.upd_b_off;
    p.sa = g.sa; p.sb = g.sb; p.scolsum = g.scolsum;
    p.M = g.M; p.N = g.N; p.K = g.K; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc;
    p.tiles_m = g.M / 64;
    p.tiles_n = g.N / 64;
    p.groups = g.groups;
    const int64_t total = (int64_t)g.groups * p.tiles_m * p.tiles_n;
    if (total > (1 << 30)) return hipErrorInvalidValue;
    p.total_tiles = (int)total;
    p.chunk = (int)((total + kXcds - 1) / kXcds);
    // short K loops (K = 64) hide less per tile and want twice the workgroups (648 us against 807 us on 64 x (3072 x 1024))
    const int per_cu = g.K >= 128 ? OLS_DWP_WGS_PER_CU : 2 * OLS_DWP_WGS_PER_CU;
    p.wgs_per_xcd = p.chunk < 32 * per_cu ? p.chunk : 32 * per_cu;   // 32 compute units per XCD
    const unsigned grid = (unsigned)(p.guest.blocks + p.wgs_per_xcd * kXcds);
#define OLS_DWP2(SPG, PULL, MOM) gemm_f32_dw_pipelined_kernel<SPG, PULL, MOM><<<grid, kThreads, 0, s>>>(p)
#define OLS_DWP(SPG)                                                      \
    do {                                                                  \
        const bool mom = g.upd.mu != 0.0f;                                \
        if (g.upd.pull && mom) OLS_DWP2(SPG, true, true);                 \
        else if (g.upd.pull) OLS_DWP2(SPG, true, false);                  \
        else if (mom) OLS_DWP2(SPG, false, true);                         \
        else OLS_DWP2(SPG, false, false);                                 \
    } while (0)
    if (g.K == 64) OLS_DWP(1);
    else if (g.K == 128) OLS_DWP(2);
    else OLS_DWP(4);
#undef OLS_DWP2
#undef OLS_DWP
    return hipGetLastError();
}

// Tile shapes.  Variant 0 is the default (for the forward GEMM: chosen from the shape); the others exist so
// that the choice can be re-measured (OLS_OPT_TUNING; most of them only in builds with -DOLS_TUNING_VARIANTS).  LDS per workgroup stays below 80 KiB so two workgroups fit a compute unit.
// Shape-driven choice for the forward GEMM.  Measured on configuration 2 (M = 128, N = 512, K = 3072,
// 16 groups): every tile shape lands within a few percent once there are several workgroups per compute
// unit, because the matrix pipe idles whenever a wavefront waits at the slice barrier or for its loads
// and only other resident workgroups fill those gaps; so: 64 x 64 tiles, and K ranges until the launch
// has about two workgroups per compute unit.  With the full-tile path, per launch including the pass that
// sums the parts: one K range (256 workgroups) 70.8 us, two 69.1 us, four 71.3 us, eight 82 us; the step as a
// whole 0.1808 / 0.1798 / 0.1828 / 0.194 ms (fewer parts to write and re-read, and the anchor refresh on the
// side stream finds more room beside the smaller launch).
// Where 64 x 64 tiles would give four or more workgroups per compute unit, 64 x 128 tiles (half as many, each
// A slice loaded once for twice the columns) are faster: configuration 5 (M = 64, N = 1024, 64 groups) 232 us
// against 238 us per launch, 0.8428 against 0.8504 ms per step.
void gemm_f32_fwd_plan(int groups, int M, int N, int K, int* variant, int* splits) {
    *variant = 2;
    int64_t tiles = (int64_t)groups * ((M + 63) / 64) * ((N + 63) / 64);
    if (tiles >= 1024 && N >= 128) {
        *variant = 6;
        tiles = (int64_t)groups * ((M + 63) / 64) * ((N + 127) / 128);
    }
    int s = 1;
    while (tiles * s < 512 && K / (2 * s) >= 256 && s < 8) s *= 2;
    *splits = s;
}

hipError_t launch_gemm_f32_fwd(const GemmArgs& g, hipStream_t s, int variant) {
    if (variant == 0) {
        int sp;
        gemm_f32_fwd_plan(g.groups, g.M, g.N, g.K, &variant, &sp);
    }
    switch (variant) {
        case 2: return gemm_launch<kFwd, 64, 64, 32, 2, 2, 2>(g, s);
        case 6: return gemm_launch<kFwd, 64, 128, 32, 2, 2, 2>(g, s);
#ifdef OLS_TUNING_VARIANTS
        case 1: return gemm_launch<kFwd, 64, 64, 64, 2, 2, 2>(g, s);
        case 3: return gemm_launch<kFwd, 64, 64, 32, 2, 2, 1>(g, s);
        case 4: return gemm_launch<kFwd, 64, 64, 64, 2, 2, 1>(g, s);
        case 5: return gemm_launch<kFwd, 128, 64, 32, 2, 2, 2>(g, s);
        case 7: return gemm_launch<kFwd, 128, 128, 16, 2, 2, 2>(g, s);
        case 8: return gemm_launch<kFwd, 128, 128, 32, 2, 2, 2>(g, s);
        case 9: return gemm_launch<kFwd, 128, 128, 32, 2, 2, 1>(g, s);
#endif
        default: return hipErrorInvalidValue;
    }
}
hipError_t launch_gemm_f32_dw(const GemmArgs& g, hipStream_t s, int variant) {
    if (variant == 0) {
        // Measured (configurations 2 and 5): writing the gradient out, 128 x 128 tiles are fastest; with
        // the update fused into the epilogue the kernel is bound by the HBM traffic of the state, and
        // smaller tiles (more workgroups whose compute and epilogue phases interleave) win; with the small
        // tiles a second K slice of global loads in flight costs one register and gains 3 % (configuration 2:
        // 103.3 -> 100.3 us).
        // The persistent kernel that spreads a tile's update over the next tile's K loop wins where a tile has
        // enough K slices to hide the state's latency behind (K = 128, configuration 2: 0.1853 -> 0.1826 ms per
        // step); with K = 64 (configuration 5) it loses (665 us against 585 us per launch).
        if (g.upd.enabled && g.K == 128 && dw_pipelined_fits(g)) variant = 16;
        else if (!g.upd.enabled) variant = 1;
        else variant = (int64_t)g.groups * ((g.M + 127) / 128) * ((g.N + 127) / 128) < 4096 ? 11 : 8;
    }
    switch (variant) {
        case 1: return gemm_launch<kDw, 128, 128, 16, 2, 2, 1>(g, s);
        case 8: return gemm_launch<kDw, 64, 128, 16, 2, 2, 1>(g, s);
        case 11: return gemm_launch<kDw, 64, 64, 16, 2, 2, 2>(g, s);
        case 16: return dw_pipelined_launch(g, s);
#ifdef OLS_TUNING_VARIANTS
        case 2: return gemm_launch<kDw, 128, 128, 16, 2, 2, 2>(g, s);
        case 3: return gemm_launch<kDw, 128, 128, 32, 2, 2, 2>(g, s);
        case 4: return gemm_launch<kDw, 64, 128, 32, 2, 2, 2>(g, s);
        case 5: return gemm_launch<kDw, 128, 64, 32, 2, 2, 2>(g, s);
        case 6: return gemm_launch<kDw, 64, 64, 32, 2, 2, 2>(g, s);
        case 7: return gemm_launch<kDw, 64, 64, 32, 2, 2, 1>(g, s);
        case 9: return gemm_launch<kDw, 64, 64, 16, 2, 2, 1>(g, s);
        case 10: return gemm_launch<kDw, 128, 64, 16, 2, 2, 1>(g, s);
        case 12: return gemm_launch<kDw, 64, 128, 16, 2, 2, 2>(g, s);
#endif
        default: return hipErrorInvalidValue;
    }
}
hipError_t launch_gemm_f32_da(const GemmArgs& g, hipStream_t s, int variant) {
    switch (variant) {
        case 0: return gemm_launch<kDa, 64, 64, 64, 2, 2, 2>(g, s);
#ifdef OLS_TUNING_VARIANTS
        case 1: return gemm_launch<kDa, 64, 64, 32, 2, 2, 2>(g, s);
        case 2: return gemm_launch<kDa, 64, 64, 32, 2, 2, 1>(g, s);
        case 3: return gemm_launch<kDa, 128, 64, 32, 2, 2, 2>(g, s);
#endif
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ols
