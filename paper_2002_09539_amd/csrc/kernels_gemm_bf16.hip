// Grouped GEMMs with bf16 operands and fp32 accumulation on the matrix cores
// (v_mfma_f32_32x32x16_bf16, gfx950) for the hidden layers of the per-worker MLPs, plus the fp32 ->
// bf16 conversion of the input batch.  One group per worker, all groups in one launch.
//
//   FWD  C[M][N] = relu(A[M][K] W[K][N] + bias[N])   A: bf16 activations; W: bf16 copy of the weights;
//                                                    C: bf16, stored row-major and transposed
//   DW   C[M][N] = At[M][K] Bt[N][K]^T               At, Bt: transposed bf16 copies of activations and
//                                                    deltas (K = batch, contiguous); C: fp32 gradient
//   DA   C[M][N] = (A[M][K] W[N][K]^T) * [mask > 0]  A: bf16 delta; W rows are contiguous in K;
//                                                    C: bf16, stored row-major and transposed
//
// (forward / backward of the mini-batch loss whose gradient is the g_i of Section 2, arXiv 2002.09539;
// operands are rounded to bf16 with round-to-nearest-even, products and sums are fp32.)
//
// The MFMA takes, per lane, 8 consecutive contraction indices of one row of each operand, so both
// operand tiles live in LDS as [row][BK + 8] bf16 and a fragment is one 16-byte LDS read.  Operands
// that are K-contiguous in memory are copied with 16-byte vectors.  The forward pass' weight tile is
// N-contiguous in memory: each lane fetches a 4 (k) x 8 (n) patch with four 16-byte loads, transposes
// it in registers and writes eight 8-byte column pieces, so the LDS image is K-contiguous as well.
// The epilogues that produce bf16 activations / deltas also write the transposed copy the
// weight-gradient GEMM needs (an accumulator lane holds 4 consecutive rows of one column, i.e. one
// 8-byte piece of the transposed matrix).
#include "gemm_epilogue.h"
#include "ols_internal.h"

namespace ols {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));

enum GemmMode { kFwd = 0, kDw = 1, kDa = 2 };

constexpr int kThreads = 256;
constexpr int kXcds = 8;

__device__ __forceinline__ unsigned int bf16_rne(float f) {
    unsigned int u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float bf16_to_f32(unsigned int h) { return __uint_as_float(h << 16); }

struct GemmDevB {
    const uint16_t* a;
    const uint16_t* b;
    void* c;
    uint16_t* c_t;
    const float* bias;
    const uint16_t* mask;
    float* colsum;
    FusedUpdate upd;     // DW: update applied in the epilogue instead of storing the gradient
    int64_t upd_w_off, upd_b_off;
    int64_t sa, sb, sc, sct, sbias, smask, scolsum;
    int M, N, K, lda, ldb, ldc;
    int tiles_m, tiles_n, total_tiles, chunk;
};

// K-contiguous operand tile: ROWS x BK bf16 copied with 16-byte vectors into [ROWS][BK + 8].
template <int ROWS, int BK>
struct TileKC {
    static constexpr int kPitch = BK + 8;                 // bf16 elements; 16-byte aligned rows
    static constexpr int kVecPerRow = BK / 8;
    static constexpr int kVecs = ROWS * kVecPerRow;
    static constexpr int kPerThread = (kVecs + kThreads - 1) / kThreads;
    static constexpr int kElems = ROWS * kPitch;
    __device__ static void load(u4 (&r)[kPerThread], const uint16_t* __restrict__ base, int ld, int row0, int k0,
                                int rows, int klen) {
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const int v = threadIdx.x + t * kThreads;
            u4 val = {0u, 0u, 0u, 0u};
            if (kVecs % kThreads == 0 || v < kVecs) {
                const int row = row0 + v / kVecPerRow, k = k0 + (v % kVecPerRow) * 8;
                if (row < rows && k < klen) val = *(const u4*)(base + (int64_t)row * ld + k);
            }
            r[t] = val;
        }
    }
    __device__ static void store(uint16_t* lds, const u4 (&r)[kPerThread]) {
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const int v = threadIdx.x + t * kThreads;
            if (kVecs % kThreads == 0 || v < kVecs)
                *(u4*)(lds + (v / kVecPerRow) * kPitch + (v % kVecPerRow) * 8) = r[t];
        }
    }
};

// N-contiguous operand tile (memory [K][N]) transposed into the same [ROWS = n][BK + 8] LDS image.
// A task is a 4 (k) x 8 (n) patch; consecutive lanes take consecutive n-octets of the same k-quad so
// that the four global loads of a wavefront are contiguous runs.
template <int ROWS, int BK>
struct TileNC {
    static constexpr int kPitch = BK + 8;
    static constexpr int kOctets = ROWS / 8;
    static constexpr int kTasks = kOctets * (BK / 4);
    static constexpr int kPerThread = (kTasks + kThreads - 1) / kThreads;
    static constexpr int kElems = ROWS * kPitch;
    struct Regs {
        u4 v[kPerThread][4];
    };
    __device__ static void load(Regs& r, const uint16_t* __restrict__ base, int ld, int n0, int k0, int ncols,
                                int klen) {
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const int task = threadIdx.x + t * kThreads;
            const int n = n0 + (task % kOctets) * 8, k = k0 + (task / kOctets) * 4;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                u4 val = {0u, 0u, 0u, 0u};
                if ((kTasks % kThreads == 0 || task < kTasks) && n < ncols && k + j < klen)
                    val = *(const u4*)(base + (int64_t)(k + j) * ld + n);
                r.v[t][j] = val;
            }
        }
    }
    __device__ static void store(uint16_t* lds, const Regs& r) {
#pragma unroll
        for (int t = 0; t < kPerThread; ++t) {
            const int task = threadIdx.x + t * kThreads;
            if (kTasks % kThreads == 0 || task < kTasks) {
                const int nl = (task % kOctets) * 8, kl = (task / kOctets) * 4;
#pragma unroll
                for (int p = 0; p < 4; ++p) {  // dword p of each row holds columns 2p (low) and 2p + 1 (high)
                    const unsigned int w0 = r.v[t][0][p], w1 = r.v[t][1][p], w2 = r.v[t][2][p], w3 = r.v[t][3][p];
                    u2 lo, hi;
                    lo.x = (w0 & 0xFFFFu) | (w1 << 16);
                    lo.y = (w2 & 0xFFFFu) | (w3 << 16);
                    hi.x = (w0 >> 16) | (w1 & 0xFFFF0000u);
                    hi.y = (w2 >> 16) | (w3 & 0xFFFF0000u);
                    *(u2*)(lds + (nl + 2 * p) * kPitch + kl) = lo;
                    *(u2*)(lds + (nl + 2 * p + 1) * kPitch + kl) = hi;
                }
            }
        }
    }
};

template <int MODE, int BM, int BN, int BK>
__global__ __launch_bounds__(kThreads) void gemm_bf16_kernel(GemmDevB p) {
    constexpr int WM = BM / 2, WN = BN / 2;     // 2 x 2 wavefronts
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int S = BK / 16;                  // MFMA steps per K slice
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 16 == 0, "tile shape");
    using TA = TileKC<BM, BK>;
    using TBK = TileKC<BN, BK>;
    using TBN = TileNC<BN, BK>;
    constexpr int kPitch = TA::kPitch;
    constexpr int kLdsElems = 2 * TA::kElems + 2 * TBK::kElems;
    __shared__ __attribute__((aligned(16))) uint16_t lds_all[kLdsElems];
    auto lds_a = [&](int buf) { return lds_all + buf * TA::kElems; };
    auto lds_b = [&](int buf) { return lds_all + 2 * TA::kElems + buf * TBK::kElems; };

    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
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

    // DW only: the first tile row also sums each row of Bt (a delta column over the batch), which is
    // the bias gradient of the layer, in sample order.
    const bool row_sums = MODE == kDw && p.colsum != nullptr && tm == 0 && threadIdx.x < BN;
    float row_acc = 0.0f;

    u4 ra[TA::kPerThread];
    u4 rbk[TBK::kPerThread];
    typename TBN::Regs rbn;
    auto load_tiles = [&](int k0) {
        TA::load(ra, A, p.lda, m0, k0, p.M, p.K);
        if (MODE == kFwd) TBN::load(rbn, B, p.ldb, n0, k0, p.N, p.K);
        else TBK::load(rbk, B, p.ldb, n0, k0, p.N, p.K);
    };
    auto store_tiles = [&](int buf) {
        TA::store(lds_a(buf), ra);
        if (MODE == kFwd) TBN::store(lds_b(buf), rbn);
        else TBK::store(lds_b(buf), rbk);
    };
    auto frag = [&](const uint16_t* lds, int r0, int s) {
        return *(const u4*)(lds + (r0 + lane32) * kPitch + 16 * s + 8 * half);
    };

    const int nk = (p.K + BK - 1) / BK;
    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) load_tiles((kt + 1) * BK);
#pragma unroll
        for (int s = 0; s < S; ++s) {
            u4 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = frag(lds_a(cur), wm0 + 32 * i, s);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = frag(lds_b(cur), wn0 + 32 * j, s);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i]),
                                                                        __builtin_bit_cast(bf16x8, fb[j]), acc[i][j],
                                                                        0, 0, 0);
        }
        if (MODE == kDw && row_sums) {
            const uint16_t* row = lds_b(cur) + threadIdx.x * kPitch;
#pragma unroll
            for (int k = 0; k < BK; k += 2) {
                const unsigned int pair = *(const unsigned int*)(row + k);
                row_acc += bf16_to_f32(pair & 0xFFFFu);
                row_acc += bf16_to_f32(pair >> 16);
            }
        }
        if (kt + 1 < nk) store_tiles(cur ^ 1);
        __syncthreads();
    }
    if (MODE == kDw && row_sums && n0 + (int)threadIdx.x < p.N) {
        if (p.upd.enabled) {   // bias: gradient is the sum just formed
            const int64_t col = p.upd_b_off + n0 + threadIdx.x, idx = (int64_t)group * p.upd.ld + col;
            fused_update_apply(p.upd, idx, col, row_acc, p.upd.x_in[idx], p.upd.mu != 0.0f ? p.upd.buf[idx] : 0.0f);
        } else {
            p.colsum[(int64_t)group * p.scolsum + n0 + threadIdx.x] = row_acc;
        }
    }
    if (MODE == kDw && p.upd.enabled) {
        constexpr int kFit = ((kLdsElems / 2) / (BN + 4)) / 32 * 32;   // fp32 rows the operand LDS can stage
        constexpr int RP = kFit >= BM ? BM : kFit;
        static_assert(RP >= 32, "operand LDS too small to stage the gradient tile");
        DwOut o;
        o.g = (float*)p.c + (int64_t)group * p.sc;
        o.ldg = p.ldc;
        o.upd = p.upd;
        o.upd_base = (int64_t)group * p.upd.ld + p.upd_w_off;
        o.col_base = p.upd_w_off;
        dw_epilogue_staged<BM, BN, TM, TN, RP, kThreads>((float*)lds_all, acc, o, m0, n0, wm0, wn0, p.M, p.N);
        return;
    }

    // Epilogue.  Accumulator register r of a lane is C[row][col] with col = lane % 32 and
    // row = 8 (r / 4) + 4 (lane / 32) + r % 4 inside its 32 x 32 block: four consecutive rows per r / 4.
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn0 + 32 * j + lane32;
            if (col >= p.N) continue;
            float bias = 0.0f;
            if (MODE == kFwd) bias = p.bias[(int64_t)group * p.sbias + col];
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int row = m0 + wm0 + 32 * i + 8 * rq + 4 * half;   // rows row .. row + 3 (M is a multiple of 4)
                if (row >= p.M) continue;
                if (MODE == kDw) {
                    float* C = (float*)p.c + (int64_t)group * p.sc;
#pragma unroll
                    for (int e = 0; e < 4; ++e) C[(int64_t)(row + e) * p.ldc + col] = acc[i][j][4 * rq + e];
                } else {
                    uint16_t* C = (uint16_t*)p.c + (int64_t)group * p.sc;
                    unsigned int h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float v = acc[i][j][4 * rq + e];
                        if (MODE == kFwd) v = fmaxf(v + bias, 0.0f);
                        if (MODE == kDa) {
                            const unsigned int mk = p.mask[(int64_t)group * p.smask + (int64_t)(row + e) * p.ldc + col];
                            v = bf16_to_f32(mk) > 0.0f ? v : 0.0f;
                        }
                        h[e] = bf16_rne(v);
                        C[(int64_t)(row + e) * p.ldc + col] = (uint16_t)h[e];
                    }
                    if (p.c_t) {
                        u2 pk;
                        pk.x = h[0] | (h[1] << 16);
                        pk.y = h[2] | (h[3] << 16);
                        *(u2*)(p.c_t + (int64_t)group * p.sct + (int64_t)col * p.M + row) = pk;
                    }
                }
            }
        }
    }
}

static bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

template <int MODE, int BM, int BN, int BK>
static hipError_t gemm_launch(const GemmArgs& g, hipStream_t s) {
    if (!g.a || !g.b || !g.c || g.groups < 1 || g.M < 1 || g.N < 1 || g.K < 1) return hipErrorInvalidValue;
    // 16-byte vectors of 8 bf16: aligned bases, leading dimensions and extents in multiples of 8
    if (!aligned16(g.a) || !aligned16(g.b) || g.lda % 8 || g.ldb % 8 || g.sa % 8 || g.sb % 8 || g.K % 8)
        return hipErrorInvalidValue;
    if (MODE == kFwd && (g.N % 8 || g.ldb < g.N || !g.bias)) return hipErrorInvalidValue;
    if (MODE != kFwd && g.ldb < g.K) return hipErrorInvalidValue;
    if (g.lda < g.K || g.ldc < g.N || g.M % 4) return hipErrorInvalidValue;
    if (MODE == kDa && !g.mask) return hipErrorInvalidValue;
    if (g.c_t && ((reinterpret_cast<uintptr_t>(g.c_t) & 7u) || g.sct % 4)) return hipErrorInvalidValue;
    GemmDevB p;
    p.a = (const uint16_t*)g.a;
    p.b = (const uint16_t*)g.b;
    p.c = g.c;
    p.c_t = MODE == kDw ? nullptr : (uint16_t*)g.c_t;
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
    p.sa = g.sa; p.sb = g.sb; p.sc = g.sc; p.sct = g.sct; p.sbias = g.sbias; p.smask = g.smask;
    p.scolsum = g.scolsum;
    p.M = g.M; p.N = g.N; p.K = g.K; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc;
    p.tiles_m = (g.M + BM - 1) / BM;
    p.tiles_n = (g.N + BN - 1) / BN;
    const int64_t total = (int64_t)g.groups * p.tiles_m * p.tiles_n;
    if (total > (1 << 30)) return hipErrorInvalidValue;
    p.total_tiles = (int)total;
    p.chunk = (int)((total + kXcds - 1) / kXcds);
    gemm_bf16_kernel<MODE, BM, BN, BK><<<(unsigned)(p.chunk * kXcds), kThreads, 0, s>>>(p);
    return hipGetLastError();
}

hipError_t launch_gemm_bf16_fwd(const GemmArgs& g, hipStream_t s) { return gemm_launch<kFwd, 128, 128, 64>(g, s); }
hipError_t launch_gemm_bf16_dw(const GemmArgs& g, hipStream_t s) { return gemm_launch<kDw, 128, 128, 64>(g, s); }
hipError_t launch_gemm_bf16_da(const GemmArgs& g, hipStream_t s) { return gemm_launch<kDa, 128, 128, 64>(g, s); }

// ---------------------------------------------------------------------------------------------
// fp32 [groups][rows][cols] -> bf16 row-major copy and bf16 transposed copy [groups][cols][rows]
// ---------------------------------------------------------------------------------------------
constexpr int kCastTile = 64;
__global__ __launch_bounds__(kThreads) void cast_bf16_kernel(const float* __restrict__ src, int64_t src_stride,
                                                             uint16_t* __restrict__ dst, uint16_t* __restrict__ dst_t,
                                                             int rows, int cols) {
    __shared__ uint16_t tile[kCastTile][kCastTile + 2];
    const int g = blockIdx.z;
    const int r0 = blockIdx.y * kCastTile, c0 = blockIdx.x * kCastTile;
    const float* S = src + (int64_t)g * src_stride;
    uint16_t* D = dst + (int64_t)g * rows * cols;
    uint16_t* T = dst_t + (int64_t)g * rows * cols;
    // 16 lanes x 4 floats cover a 64-column row segment; 16 rows per pass
    for (int rr = threadIdx.x / 16; rr < kCastTile; rr += kThreads / 16) {
        const int r = r0 + rr, c = c0 + (threadIdx.x % 16) * 4;
        f4 v = {0.f, 0.f, 0.f, 0.f};
        if (r < rows && c < cols) v = *(const f4*)(S + (int64_t)r * cols + c);   // cols is a multiple of 4
        unsigned int h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            h[e] = bf16_rne(v[e]);
            tile[rr][(threadIdx.x % 16) * 4 + e] = (uint16_t)h[e];
        }
        if (r < rows && c < cols) {
            u2 pk;
            pk.x = h[0] | (h[1] << 16);
            pk.y = h[2] | (h[3] << 16);
            *(u2*)(D + (int64_t)r * cols + c) = pk;
        }
    }
    __syncthreads();
    for (int cc = threadIdx.x / 16; cc < kCastTile; cc += kThreads / 16) {
        const int c = c0 + cc, r = r0 + (threadIdx.x % 16) * 4;
        if (c < cols && r < rows) {   // rows is a multiple of 4
            const int rl = (threadIdx.x % 16) * 4;
            u2 pk;
            pk.x = tile[rl][cc] | ((unsigned int)tile[rl + 1][cc] << 16);
            pk.y = tile[rl + 2][cc] | ((unsigned int)tile[rl + 3][cc] << 16);
            *(u2*)(T + (int64_t)c * rows + r) = pk;
        }
    }
}

hipError_t launch_cast_bf16(const float* src, int64_t src_stride, uint16_t* dst, uint16_t* dst_t, int groups, int rows,
                            int cols, hipStream_t s) {
    if (!src || !dst || !dst_t || groups < 1 || groups > 65535 || rows < 4 || cols < 4 || rows % 4 || cols % 4)
        return hipErrorInvalidValue;
    if (!aligned16(src) || src_stride % 4) return hipErrorInvalidValue;
    const unsigned gy = (unsigned)((rows + kCastTile - 1) / kCastTile);
    if (gy > 65535u) return hipErrorInvalidValue;
    dim3 grid((unsigned)((cols + kCastTile - 1) / kCastTile), gy, (unsigned)groups);
    cast_bf16_kernel<<<grid, kThreads, 0, s>>>(src, src_stride, dst, dst_t, rows, cols);
    return hipGetLastError();
}

}  // namespace ols
