// 3 x 3 convolutions (stride 1, zero padding 1) of the per-worker residual block with bf16 operands and fp32
// accumulation on the matrix cores (v_mfma_f32_32x32x16_bf16), grouped over the m workers: forward, back-propagated
// delta, kernel / bias gradient; plus the conversion of the input batch, the block's tail (shortcut, ReLU, pooling) and
// the pooling backward.  The model is the first residual stage of the network of Section 4 (arXiv 2002.09539,
// "Experimental setting") and produces the stochastic gradients g_i of Section 2; every tensor is rounded to bf16 (to
// nearest even) where it becomes an operand of a convolution's products, sums and everything else stay fp32.
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
// 64 x 64 kernel slice of each tap is double-buffered through registers.  Four wavefronts of 64 x 64; the MFMA takes the
// kernel fragment first, so a lane's accumulators are four consecutive channels of one pixel, packed by the hardware
// conversion and staged through LDS for 16-byte stores; every wavefront stages and stores its own 64 rows, so the
// epilogue has no workgroup barrier.  The second convolution's epilogue is the block's tail: it adds the shortcut,
// applies the ReLU, keeps the activation's sign (one bit per element) for the backward pass and the wavefront's channel
// sums for the pooling -- neither the convolution's output nor the activation is ever stored.  (Images of fewer than 64
// padded pixels take the unfused route: conv + bias in fp32, then one streaming pass.)
// DW: one workgroup per (pixel range, 64 x 64 block of input x output channels) holds all nine taps' accumulators
// (9 x 64 x 64 fp32 = 144 registers per lane); per 64 pixels the input strip (64 + 2 (W + 3) rows, row-contiguous,
// read with the transpose load at nine row offsets) and the delta tile pass through LDS; ranges are summed in range
// order by the finish pass shared with the fp32 kernels (no atomics).
// All three address global memory through buffer descriptors: the hardware's range check returns zeros for the rows a
// strip reaches past either end of the tensor and drops the stores of a last tile's missing rows, so the loads and stores
// carry no per-lane predicates, selects or 64-bit address arithmetic.
//
// Measured at the benchmark shape (16 workers x 128 samples x 32 x 32 x 64 channels, 154.6 GFLOP per launch): forward
// 200 us (bf16 out), 240 us with the fused tail (208 us for conv + bias in fp32 alone, which then needed a 224 us
// streaming pass), delta 204 us, kernel gradient 170 + 22 us, against 1390 - 1430 us for the fp32 kernels.
// Timestamps (s_memrealtime) taken inside an instrumented copy of the forward kernel showed where a tile's 11.3 us went
// before the descriptors: 2.8 us from the first instruction to the last load issued -- some 1100 instructions of
// predicates and addresses, issued by one wavefront per SIMD at a few cycles each -- 1.3 us for the loads to arrive,
// 4.6 us for the nine taps (1.9 us of MFMA issue; the other workgroup of the compute unit shares the pipe) and 2.7 us of
// epilogue.  With one workgroup per compute unit a tile takes 7.2 us, so the second one hides a third of the latencies.
// Buffer addressing took the kernel from 2150 to 1330 instructions and the tile to 9.4 us (forward 221 -> 197 us,
// fp32 out 245 -> 208, delta 252 -> 204 with the gate activations requested three taps before the end instead of after
// it).  The same treatment of the kernel gradient's slice loads: 0.70 -> 0.33 us of a slice's 2.36 us for the
// requests, 0.43 -> 0.29 for the LDS stores (186 -> 170 us); its bias column sums now come from the delta fragments the
// MFMAs use anyway instead of sixteen more LDS reads per slice.
// The fused tail's shortcut rows (fp32, 16 vectors per lane) are requested in two batches of eight, the first three
// taps before the end and the second once the tile is staged, instead of both inside the epilogue's loop: 252 -> 241 us
// (requesting the second batch before the staging as well: 248 us).
// What moved the kernel gradient from 289 us before that: fragment reads issued a kernel row ahead of the MFMAs (258),
// the bias column sums shared out over the four wavefronts instead of one wavefront summing while three wait at the
// barrier (219), and 512 workgroups -- one round at two per compute unit -- instead of 768 (185; the finish pass 46 -> 22).
// Tried and not kept: persistent workgroups that hold the whole kernel as 72 register fragments and walk the tiles of a
// worker (one wavefront per SIMD, no barrier inside a tile: 280 - 400 us; with half the fragments per wavefront and two
// workgroups per compute unit 308 - 397 us); the present forward kernel made persistent with the next tile's strip
// requested a tile ahead (the 44 extra live registers spill: 308 - 366 us); all nine kernel slices requested at the
// start of a tile (no change); in the kernel gradient two slices of loads in flight (400 registers, one wavefront per
// SIMD: 349 us), fragment reads two kernel rows ahead (259 against 258 us), and an LDS ring of input rows that fetches
// only the 64 new rows per slice three slices ahead (the wrap-around address arithmetic per fragment read costs more
// than the loads it saves: 325 us); forward / delta tiles of 128 pixels (134 registers, 53 KB of LDS, three workgroups
// per compute unit; the halo is then 1.55 x the tile: 260 / 291 / 271 us against 221 / 245 / 252); a raised wavefront
// priority (s_setprio) outside or inside the tap loop (+-1 %); the bias loaded straight into the accumulators before the
// first tap (the eight extra loads in the prologue cost what the epilogue's additions saved); a branch around the late
// requests of bias / gate activations (the compiler then makes every later wait on a kernel slice wait for them too:
// +0.8 us per tile); the first MFMAs of a tile with a zero third operand instead of cleared accumulators (200 instructions
// less, no change), and all kernel arguments fetched in one scalar round trip at the top instead of five dependent ones
// (no change either): what remains of the prologue's 2 us is the issue of its 17 vector loads per lane, about 0.1 us
// each -- with 68 KB per workgroup in flight and 7 - 8 TB/s crossing the L2 during a launch (strips, the 73 KB of
// kernel slices every tile fetches again, the outputs), the memory pipeline itself is what the loads queue for.
#include <type_traits>

#include "fast_div.h"
#include "gemm_bf16_tile.h"
#include "ols_internal.h"

namespace ols {

// Measurement builds only (-DOLS_CONV_PHASE_PROBE): lane 0 of every forward / delta workgroup leaves s_memrealtime
// readings (100 MHz) at six points of its tile, which ols_debug_conv_phases() copies out.  [kernel: 0 forward with
// bf16 output, 1 forward with another output, 2 delta][tile][point].  Without the flag nothing of this exists.
#ifdef OLS_CONV_PHASE_PROBE
constexpr int kProbeTiles = 16384;
__device__ unsigned long long conv_phase_probe[3][kProbeTiles][8];
#define OLS_TP(k)                                                                                             \
    do {                                                                                                      \
        if (threadIdx.x == 0 && tile < kProbeTiles)                                                           \
            conv_phase_probe[MODE == 1 ? 2 : (OUT == kOutBf16 ? 0 : 1)][tile][k] = wall_clock64();            \
    } while (0)
#else
#define OLS_TP(k) do { } while (0)
#endif

namespace {

constexpr int kThreads = kTileThreads;
constexpr int kXcds = 8;
constexpr int kCB = 64;     // channel block: contraction chunk and output-channel tile
constexpr int kBM = 256;    // padded pixels per forward / delta tile
constexpr int kDwBK = 64;   // pixels per slice of the kernel-gradient contraction

struct ConvBDev {
    const uint16_t* in;      // FWD: layer input; DX: delta of the layer output; DW: layer input   [groups][Pp][C] bf16
    const uint16_t* w;       // FWD, DX: bf16 kernels [9][C][C]
    const uint16_t* dout;    // DW: delta of the layer output
    void* out;               // FWD, DX: [Pp][C], bf16 or fp32
    const float* bias;       // FWD
    const uint16_t* mask;    // DX: padded bf16 activations whose sign gates the result
    float* partial;          // DW
    const float* xres;       // FWD with the fused tail: the shortcut, fp32 [B H W][C]
    uint8_t* sign;           // FWD with the fused tail: [Pp][C / 4] sign bytes
    float* pool_part;        // FWD with the fused tail: [groups][tiles_m * 4 wavefronts][2][C] partial sums of the pooling
    float* stat_part;        // FWD with the unpadded fp32 output, optional: [groups][tiles_m * 4 wavefronts][3][C] per-wavefront
                             // statistics of the output's image pixels (count, mean, sum of squared deviations)
    int64_t s_x, s_sign;
    int64_t s_in, s_w, s_dout, s_out, s_bias, s_mask;
    int groups, B, H, W, C, Hp, Wp, Pp, halo;
    int relu;
    int tiles_m, tiles_n, total_tiles, chunk;
    FastDiv div_per, div_wp; // division by (H + 2) (W + 2) and by W + 2
    FastDiv div_pg, div_tn;  // FWD, DX: division by tiles_m * tiles_n and by tiles_n
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
    const int n = (int)fast_div((unsigned)q, p.div_per), rem = q - n * per;
    const int y = (int)fast_div((unsigned)rem, p.div_wp), x = rem - y * p.Wp;
    *unpadded = (n * p.H + (y - 1)) * p.W + (x - 1);
    return y >= 1 && y <= p.H && x >= 1 && x <= p.W;
}

// ---------------------------------------------------------------------------------------------
// forward (MODE 0) and back-propagated delta (MODE 1)
// ---------------------------------------------------------------------------------------------
// LDS of the forward / delta kernel, in bf16 elements: the strip and two kernel slices -- or, if larger, the fp32 output
// staging of the four wavefronts (BM / 4 rows of 64 + 4 floats each), which takes their place after the last tap.
constexpr int kStagePitchF32 = kCB + 4;
// What the epilogue produces: bf16 in the padded operand layout; conv + bias in fp32, padded; the fused tail; or fp32 in
// the UNPADDED [B H W][C] layout (image pixels only) -- the input of a batch normalisation (forward) or of its backward
// pass (delta, gated by the sign of the bf16 activation as usual).
enum { kOutBf16 = 0, kOutF32 = 1, kOutTail = 2, kOutF32U = 3 };
template <int BM, int OUT>
__host__ __device__ constexpr int conv_main_elems(int strip_rows, int slice_elems) {
    const int work = strip_rows * (kCB + 8) + 2 * slice_elems;
    const int stage = OUT != kOutBf16 ? BM * kStagePitchF32 * 2 : 0;
    return work > stage ? work : stage;
}

// NV: strip vectors per lane (upper bound of (BM + 2 halo) * 8 / 256); BM: pixels per tile.  OUT: bf16 activations /
// deltas; the bare convolution + bias in fp32; or the residual block's tail fused into the epilogue (shortcut, ReLU,
// sign bytes and partial sums of the global average pooling -- the second convolution's output is then never stored).
template <int OUT>
constexpr bool kRowIndex = OUT == kOutTail || OUT == kOutF32U;   // the epilogue needs the rows' unpadded pixel indices

template <int MODE, int OUT, int NV, int BM>
__global__ __launch_bounds__(kThreads, BM == 128 ? 3 : 2) void conv3x3_bf16_kernel(ConvBDev p) {
    using TB = typename std::conditional<MODE == 0, TileRC<kCB, kCB>, TileKC<kCB, kCB>>::type;   // FWD w[k = ci][n = co]; DX w[n = ci][k = co]
    constexpr int SP = kCB + 8;                  // strip pitch (bf16 elements): 144 bytes, conflict-free 16-byte reads
    constexpr int TM = BM / 128, TN = 2, KS = kCB / 16; // a wavefront owns BM / 4 pixels x 64 channels
    static_assert(TB::kLineStep == 32 && TB::kPerThread == 2, "a lane's vectors are 32 rows apart in the strip and in a kernel slice");
    extern __shared__ __attribute__((aligned(16))) uint16_t lds_all[];
    constexpr int kStripRows = NV * 32;          // every lane moves NV vectors: rows past BM + 2 halo are loaded and never read
    uint16_t* strip = lds_all;
    uint16_t* lds_b0 = lds_all + kStripRows * SP;
    auto lds_b = [&](int buf) { return lds_b0 + buf * TB::kElems; };
    // the fp32 output is staged over the strip and the kernel slices together (conv_main_elems)
    uint8_t* row_flag = (uint8_t*)(lds_all + conv_main_elems<BM, OUT>(kStripRows, TB::kElems));   // [BM] 1: image pixel, 0: border
    int* row_up = (int*)row_flag;   // fused tail / unpadded output instead: [BM] the pixel's index in the unpadded [B H W] order, -1 for the border

    const int tile = xcd_tile(p.chunk, p.total_tiles);
    if (tile < 0) return;
    OLS_TP(0);   // first instruction after the tile is known
    const int per_group = p.tiles_m * p.tiles_n;
    const int group = (int)fast_div((unsigned)tile, p.div_pg);
    const int in_group = tile - group * per_group;
    const int tm = (int)fast_div((unsigned)in_group, p.div_tn), tn = in_group - tm * p.tiles_n;
    const int m0 = tm * BM, n0 = tn * kCB;
    const uint16_t* IN = p.in + (int64_t)group * p.s_in;
    const uint16_t* Wg = p.w + (int64_t)group * p.s_w;
    const int C = p.C;

    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int lane32 = lane % 32, half = lane / 32;
    const int wm0 = wave * (BM / 4);

    // Byte offsets in a [rows][C] bf16 tensor: lane t of the workgroup owns the 16-byte vector t % 8 of row t / 8, and its
    // further vectors lie 32 rows below.  The same lane offset serves the strip and the kernel slices.
    const unsigned row_bytes = 2u * (unsigned)C;
    const unsigned lane_off = (threadIdx.x / 8) * row_bytes + (threadIdx.x % 8) * 16u;
    const unsigned step32 = 32u * row_bytes;
    const rsrc_t in_rs = make_rsrc(IN, (unsigned)p.Pp * row_bytes);
    const rsrc_t w_rs = make_rsrc(Wg, 9u * (unsigned)C * row_bytes);
    // rows m0 - halo .. of channels c0 .. c0 + 63: rows before the tensor wrap to offsets beyond its end, rows after it
    // lie beyond it too -- both read as zeros.  Every lane requests all its vectors at once (one round trip), then
    // writes them to LDS.
    const unsigned strip_off = (unsigned)(m0 - p.halo) * row_bytes + lane_off;
    uint16_t* strip_lane = strip + (threadIdx.x / 8) * SP + (threadIdx.x % 8) * 8;
    auto load_strip = [&](u4 (&r)[NV], int c0) {
#pragma unroll
        for (int t = 0; t < NV; ++t) r[t] = buf_load(in_rs, strip_off + t * step32, 2u * c0);
    };
    auto store_strip = [&](const u4 (&r)[NV]) {
#pragma unroll
        for (int t = 0; t < NV; ++t) *(u4*)(strip_lane + t * 32 * SP) = r[t];
    };
    // the 64 x 64 kernel slice of one tap.  Memory [ci][co]: FWD (row-contiguous tile) k = ci, rows = co; DX
    // (K-contiguous tile) rows = ci, k = co
    auto load_b = [&](u4 (&r)[TB::kPerThread], int tap, int c0) {
        const unsigned first = 2u * (unsigned)((tap * C + (MODE == 0 ? c0 : n0)) * C + (MODE == 0 ? n0 : c0));
#pragma unroll
        for (int t = 0; t < TB::kPerThread; ++t) r[t] = buf_load(w_rs, lane_off + t * step32, first);
    };
    auto store_b = [&](int buf, const u4 (&r)[TB::kPerThread]) {
        uint16_t* dst = TB::lane_lds(lds_b(buf));
#pragma unroll
        for (int t = 0; t < TB::kPerThread; ++t) *(u4*)(dst + t * TB::kLdsLineStep) = r[t];
    };

    // The MFMA takes the KERNEL fragment first and the pixel fragment second, so the accumulator tile is out^T:
    // register r of a lane holds pixel lane % 32 and channel 8 (r / 4) + 4 (lane / 32) + r % 4 of its 32 x 32 block --
    // four consecutive channels per register quad, which the epilogue packs and stores as one piece.
    f16v acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
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
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][j], fa[buf][i], acc[i][j], 0, 0, 0);
    };

    // Kernel slices travel kAhead taps ahead of their use (a tap's 16 MFMAs per wavefront are shorter than a round trip
    // to L2): a ring of kAhead register sets, slice t in set t % kAhead.
    constexpr int kAhead = 3;
    u4 rb[kAhead][TB::kPerThread];
    // Delta: the activations whose sign gates the result -- the 16-byte vectors of the wavefront's own rows that this
    // lane will write -- are requested kMaskTap taps into a chunk, when no kernel slice is in flight any more (with the
    // long strips of wide images the registers do not allow it: there they are requested after the last tap).
    constexpr int kVecB = kCB / 8, kPerB = (BM / 4) * kVecB / 64, kMaskTap = NV <= 12 ? 6 : 9;
    u4 mk[MODE == 1 && OUT == kOutBf16 ? kPerB : 1];
    const uint16_t* Mk = MODE == 1 && p.mask ? p.mask + (int64_t)group * p.s_mask : nullptr;
    const rsrc_t mk_rs = make_rsrc(Mk ? Mk : IN, Mk ? (unsigned)p.Pp * row_bytes : 0u);
    // the wavefront's own rows of the [Pp][C] bf16 output: lane l moves the vector l % 8 of rows wm0 + l / 8 + 8 t
    const unsigned own_off = (unsigned)(m0 + wm0 + lane / kVecB) * row_bytes + 2u * (unsigned)n0 + (lane % kVecB) * 16u;
    const unsigned step8 = (64 / kVecB) * row_bytes;
    // with the fp32 output a lane moves four channels at a time (vector l % 16 of rows wm0 + l / 16 + 4 t): 8-byte pieces of
    // the gate
    constexpr int kPerF = (BM / 4) * (kCB / 4) / 64;
    u2 mkf[MODE == 1 && OUT == kOutF32U ? kPerF : 1];
    auto load_mask = [&]() {
        if constexpr (OUT == kOutF32U) {
            const unsigned first = (unsigned)(m0 + wm0 + lane / (kCB / 4)) * row_bytes + 2u * (unsigned)n0 + (lane % (kCB / 4)) * 8u;
#pragma unroll
            for (int t = 0; t < kPerF; ++t) mkf[t] = __builtin_amdgcn_raw_buffer_load_b64(mk_rs, (int)(first + t * 4u * row_bytes), 0, 0);
        } else {
#pragma unroll
            for (int t = 0; t < kPerB; ++t) mk[t] = buf_load(mk_rs, own_off + t * step8, 0u);
        }
    };
    // Forward: the lane's channels of the bias (register quad g4 of block j: channels 32 j + 8 g4 + 4 (lane / 32) ..),
    // requested at the same point and added in the epilogue.
    f4 bq[MODE == 0 ? TN : 1][4];
    // (an empty range without a bias: zeros, and no branch for the waits on the kernel slices to be merged over)
    const rsrc_t bias_rs = make_rsrc(MODE == 0 && p.bias ? (const void*)(p.bias + (int64_t)group * p.s_bias + n0) : (const void*)IN,
                                     MODE == 0 && p.bias ? kCB * 4u : 0u);
    auto load_bias = [&]() {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) bq[j][g4] = __builtin_bit_cast(f4, buf_load(bias_rs, 16u * half + 128u * j + 32u * g4, 0u));
    };
    // Fused tail: the shortcut's fp32 rows that this lane will add (vector l % 16 of the unpadded rows behind the
    // wavefront's padded rows l / 16 + 4 t) -- the first batch of eight is requested at the same point, the second in
    // the epilogue while the first is consumed.
    constexpr int kTailBatch = 8;
    f4 xpre[OUT == kOutTail ? kTailBatch : 1];
    int up_pre[OUT == kOutTail ? kTailBatch : 1];
    const rsrc_t x_rs = make_rsrc(OUT == kOutTail ? (const void*)(p.xres + (int64_t)group * p.s_x) : (const void*)IN,
                                  OUT == kOutTail ? (unsigned)(p.B * p.H * p.W) * 2u * row_bytes : 0u);
    auto load_shortcut = [&]() {
        if constexpr (OUT == kOutTail) {
#pragma unroll
            for (int t = 0; t < kTailBatch; ++t) up_pre[t] = row_up[wm0 + lane / (kCB / 4) + 4 * t];
#pragma unroll
            for (int t = 0; t < kTailBatch; ++t)   // border rows: -1 wraps to an offset beyond the tensor, zeros come back
                xpre[t] = __builtin_bit_cast(f4, buf_load(x_rs, (unsigned)up_pre[t] * 2u * row_bytes + 4u * n0 + (lane % (kCB / 4)) * 16u, 0u));
        }
    };
    for (int c0 = 0; c0 < C; c0 += kCB) {
        // the previous chunk's last barrier has passed: nobody reads the strip or the kernel buffers any more
        {
            u4 rs[NV];
            load_b(rb[0], 0, c0);   // what the first tap needs goes first
            load_strip(rs, c0);
#pragma unroll
            for (int t = 1; t < kAhead; ++t) load_b(rb[t], t, c0);
            OLS_TP(1);   // the chunk's loads are issued
            if (c0 == 0) {
                int up;   // which rows of the tile are image pixels (the others get the zero border)
                const int q = m0 + threadIdx.x;
                const bool img = q < p.Pp && interior(p, q, &up);
                if (threadIdx.x < BM) {
                    if constexpr (kRowIndex<OUT>) row_up[threadIdx.x] = img ? up : -1; else row_flag[threadIdx.x] = img ? 1 : 0;
                }
            }
            store_b(0, rb[0]);
            store_strip(rs);
        }
        __syncthreads();
        OLS_TP(2);   // the strip is in LDS
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
            if (tap + kAhead < 9) load_b(rb[tap % kAhead], tap + kAhead, c0);   // its slice is in LDS already
            if (tap == kMaskTap) {   // in every chunk: a branch here would make the waits on the kernel slices wait for these too
                if constexpr (MODE == 1) load_mask(); else load_bias();
                load_shortcut();
            }
            const int dy = tap / 3 - 1, dx = tap % 3 - 1;
            const int shift = (MODE == 0 ? 1 : -1) * (dy * p.Wp + dx);
            const uint16_t* a_base = strip + (p.halo + shift) * SP;
            const uint16_t* b_tile = lds_b(tap & 1);
            load_frags(0, a_base, b_tile, 0);
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                if (s + 1 < KS) load_frags((s + 1) & 1, a_base, b_tile, s + 1);
                __builtin_amdgcn_sched_barrier(0);
                mfmas(s & 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (tap + 1 < 9) store_b((tap + 1) & 1, rb[(tap + 1) % kAhead]);
            __syncthreads();
        }
    }

    OLS_TP(3);   // the taps are done
    if (kMaskTap >= 9) {
        if constexpr (MODE == 1) load_mask(); else load_bias();
        load_shortcut();
    }
    // Epilogue: the tile goes through LDS (the strip's place) so that every lane then moves 16-byte vectors.
    if constexpr (OUT == kOutTail) {
        // a2 = relu(convolution + bias + shortcut) on the image pixels: its sign bytes and, per wavefront (64 consecutive
        // padded pixels, which touch at most two samples because a padded image has at least 64), the channel sums of its
        // rows in the first and in the second of those samples.  A later pass adds the wavefronts' sums per sample in
        // wavefront order.  Staging as for the fp32 output; lane l then owns the channel quad l % 16 of rows l / 16 + 4 t.
        constexpr int FP = kStagePitchF32, WR = BM / 4;
        constexpr int kVecPerRow = kCB / 4, kPer = WR * kVecPerRow / 64, kBatch = kTailBatch;
        static_assert(WR == 64, "the partial sums are kept per 64 rows");
        float* stage = (float*)lds_all + wave * WR * FP;
        const int r0 = lane / kVecPerRow, cq = lane % kVecPerRow;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const f4 o = {acc[i][j][4 * g4] + bq[j][g4][0], acc[i][j][4 * g4 + 1] + bq[j][g4][1], acc[i][j][4 * g4 + 2] + bq[j][g4][2],
                                  acc[i][j][4 * g4 + 3] + bq[j][g4][3]};
                    *(f4*)(stage + (32 * i + lane32) * FP + 32 * j + 8 * g4 + 4 * half) = o;
                }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const int q0 = m0 + wm0;                                    // the wavefront's first padded pixel
        const int per = p.Hp * p.Wp;
        const int next_sample = ((int)fast_div((unsigned)q0, p.div_per) + 1) * per;   // first pixel of the second sample
        const rsrc_t sg_rs = make_rsrc(p.sign + (int64_t)group * p.s_sign, (unsigned)p.Pp * (unsigned)(C / 4));
        f4 sum0 = {0.f, 0.f, 0.f, 0.f}, sum1 = {0.f, 0.f, 0.f, 0.f};
        static_assert(kPer == 2 * kBatch, "two batches of shortcut rows per lane");
        f4 xnext[kBatch];
        int up_next[kBatch];
#pragma unroll
        for (int t = 0; t < kBatch; ++t) up_next[t] = row_up[wm0 + r0 + 4 * (kBatch + t)];
#pragma unroll
        for (int t = 0; t < kBatch; ++t)   // the second batch travels while the first is consumed
            xnext[t] = __builtin_bit_cast(f4, buf_load(x_rs, (unsigned)up_next[t] * 2u * row_bytes + 4u * n0 + cq * 16u, 0u));
#pragma unroll
        for (int t0 = 0; t0 < kPer; t0 += kBatch) {
            f4 yv[kBatch], xv[kBatch];
            int up[kBatch];
#pragma unroll
            for (int t = 0; t < kBatch; ++t) {
                up[t] = t0 == 0 ? up_pre[t] : up_next[t];
                xv[t] = t0 == 0 ? xpre[t] : xnext[t];
            }
#pragma unroll
            for (int t = 0; t < kBatch; ++t) yv[t] = *(const f4*)(stage + (r0 + 4 * (t0 + t)) * FP + cq * 4);
#pragma unroll
            for (int t = 0; t < kBatch; ++t) {
                const int q = q0 + r0 + 4 * (t0 + t);
                const bool img = up[t] >= 0;
                unsigned bits = 0;
                f4 a;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    a[e] = img ? fmaxf(yv[t][e] + xv[t][e], 0.0f) : 0.0f;
                    bits |= a[e] > 0.0f ? (1u << e) : 0u;
                }
                if (q < next_sample) sum0 = sum0 + a; else sum1 = sum1 + a;
                __builtin_amdgcn_raw_buffer_store_b8((unsigned char)bits, sg_rs, (int)((unsigned)q * (unsigned)(C / 4) + n0 / 4 + cq), 0, 0);   // rows past the tensor are dropped
            }
        }
        // the four lanes of a channel quad, in lane order, through the staging area (all its reads are done)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        f4* red = (f4*)stage;
        red[lane] = sum0;
        red[64 + lane] = sum1;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (lane < 2 * kVecPerRow) {   // lanes 0 .. 15: first sample, 16 .. 31: second
            const f4* r = red + 64 * (lane / kVecPerRow) + lane % kVecPerRow;
            const f4 o = ((r[0] + r[16]) + r[32]) + r[48];
            float* PP = p.pool_part + ((((int64_t)group * p.tiles_m + tm) * 4 + wave) * 2 + lane / kVecPerRow) * C + n0;
            *(f4*)(PP + 4 * (lane % kVecPerRow)) = o;
        }
    } else if constexpr (OUT == kOutF32 || OUT == kOutF32U) {
        // Convolution + bias only (what follows it is another kernel's).  Padded output: border rows are written as
        // computed; their consumer skips them.  Unpadded output: a row goes to its pixel's place in the [B H W] order and a
        // border row to offset -1, which the range check drops.  Every wavefront stages its own BM / 4 rows and moves them
        // itself: the LDS operations of one wavefront complete in order, so no workgroup barrier is needed after the one
        // that ended the last tap.
        constexpr int FP = kStagePitchF32, WR = BM / 4;
        constexpr int kVecPerRow = kCB / 4, kPer = WR * kVecPerRow / 64, kBatch = 8;
        static_assert(kPer == kPerF, "vectors per lane");
        float* stage = (float*)lds_all + wave * WR * FP;
        const unsigned out_rows = OUT == kOutF32U ? (unsigned)(p.B * p.H * p.W) : (unsigned)p.Pp;
        const rsrc_t out_rs = make_rsrc((const float*)p.out + (int64_t)group * p.s_out, out_rows * 2u * row_bytes);
        const unsigned col_off = 4u * (unsigned)n0 + (lane % kVecPerRow) * 16u;
        const unsigned out_off = (unsigned)(m0 + wm0 + lane / kVecPerRow) * 2u * row_bytes + col_off;
        const unsigned out_step = (64 / kVecPerRow) * 2u * row_bytes;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    f4 o = {acc[i][j][4 * g4], acc[i][j][4 * g4 + 1], acc[i][j][4 * g4 + 2], acc[i][j][4 * g4 + 3]};
                    if constexpr (MODE == 0) o = o + bq[j][g4];
                    *(f4*)(stage + (32 * i + lane32) * FP + 32 * j + 8 * g4 + 4 * half) = o;
                }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int t0 = 0; t0 < kPer; t0 += kBatch) {
            u4 val[kBatch];
            int up[kBatch];
#pragma unroll
            for (int t = 0; t < kBatch; ++t) {
                const int v = lane + (t0 + t) * 64;
                val[t] = *(const u4*)(stage + (v / kVecPerRow) * FP + (v % kVecPerRow) * 4);
                if constexpr (OUT == kOutF32U) up[t] = row_up[wm0 + v / kVecPerRow];
            }
#pragma unroll
            for (int t = 0; t < kBatch; ++t) {
                u4 o = val[t];
                if constexpr (MODE == 1 && OUT == kOutF32U) {
                    if (Mk) {   // a bf16 is positive iff its bits are in [0x0001, 0x7FFF]
                        const u2 g2 = mkf[t0 + t];
                        o[0] = ((g2.x & 0xFFFFu) - 1u) < 0x7FFFu ? o[0] : 0u;
                        o[1] = ((g2.x >> 16) - 1u) < 0x7FFFu ? o[1] : 0u;
                        o[2] = ((g2.y & 0xFFFFu) - 1u) < 0x7FFFu ? o[2] : 0u;
                        o[3] = ((g2.y >> 16) - 1u) < 0x7FFFu ? o[3] : 0u;
                    }
                }
                if constexpr (OUT == kOutF32U) buf_store(o, out_rs, (unsigned)up[t] * 2u * row_bytes + col_off);   // border rows: dropped
                else buf_store(o, out_rs, out_off + (t0 + t) * out_step);                                           // rows past the tensor are dropped
            }
        }
        if constexpr (MODE == 0 && OUT == kOutF32U) {
            // Statistics of the wavefront's image pixels for the batch normalisation that follows (which then need not
            // read the output again): count, mean, and the sum of squared deviations from that mean, per channel.  Two
            // passes over the staged rows; the four lanes of a channel quad are combined through the staging area's
            // tail in lane order.  A later pass merges the wavefronts in wavefront order (the parallel-variance rule).
            if (p.stat_part) {
                const int r0 = lane / kVecPerRow, cq = lane % kVecPerRow;
                f4* red = (f4*)(stage + WR * FP) - 64;        // the last 64 vectors of the wavefront's staging rows ...
                f4 sum = {0.f, 0.f, 0.f, 0.f};
                float cnt = 0.0f;
                f4 zv[kPer];
                bool img[kPer];
#pragma unroll
                for (int t = 0; t < kPer; ++t) {
                    zv[t] = *(const f4*)(stage + (r0 + 4 * t) * FP + cq * 4);
                    img[t] = row_up[wm0 + r0 + 4 * t] >= 0;
                    if (img[t]) { sum = sum + zv[t]; cnt += 1.0f; }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();              // ... which every lane has read by now
                red[lane] = sum;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                const f4 tot = ((red[cq] + red[16 + cq]) + red[32 + cq]) + red[48 + cq];
                const float n = ((__shfl(cnt, cq) + __shfl(cnt, 16 + cq)) + __shfl(cnt, 32 + cq)) + __shfl(cnt, 48 + cq);
                const float inv_n = n > 0.0f ? 1.0f / n : 0.0f;
                f4 mean;
#pragma unroll
                for (int e = 0; e < 4; ++e) mean[e] = tot[e] * inv_n;
                f4 dev = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t = 0; t < kPer; ++t)
                    if (img[t]) { const f4 d = zv[t] - mean; dev = dev + d * d; }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                red[lane] = dev;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                if (lane < kVecPerRow) {
                    const f4 m2 = ((red[lane] + red[16 + lane]) + red[32 + lane]) + red[48 + lane];
                    float* SP3 = p.stat_part + ((((int64_t)group * p.tiles_m + tm) * 4 + wave) * 3) * C + n0 + 4 * lane;
                    *(f4*)SP3 = f4{n, n, n, n};
                    *(f4*)(SP3 + C) = mean;
                    *(f4*)(SP3 + 2 * C) = m2;
                }
            }
        }
    } else {
        // wavefront-local like the fp32 epilogue: a wavefront stages and moves its own BM / 4 rows
        const rsrc_t out_rs = make_rsrc((const uint16_t*)p.out + (int64_t)group * p.s_out, (unsigned)p.Pp * row_bytes);
        uint16_t* stage = lds_all + wm0 * SP;
        const float floor_v = p.relu ? 0.0f : -__builtin_huge_valf();   // max(., 0) or nothing
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] = acc[i][j][4 * g4 + e];
                        if constexpr (MODE == 0) v[e] = fmaxf(v[e] + bq[j][g4][e], floor_v);
                    }
                    u2 o;   // round to nearest even (v_cvt_pk_bf16_f32)
                    o.x = __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{v[0], v[1]}, bf16x2));
                    o.y = __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{v[2], v[3]}, bf16x2));
                    *(u2*)(stage + (32 * i + lane32) * SP + 32 * j + 8 * g4 + 4 * half) = o;
                }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        u4 val[kPerB];
#pragma unroll
        for (int t = 0; t < kPerB; ++t) {
            const int v = lane + t * 64;
            val[t] = *(const u4*)(stage + (v / kVecB) * SP + (v % kVecB) * 8);
        }
#pragma unroll
        for (int t = 0; t < kPerB; ++t) {
            u4 o = val[t];
            if (MODE == 0) {
                if (!row_flag[wm0 + (lane + t * 64) / kVecB]) o = u4{0u, 0u, 0u, 0u};   // the zero border the next layer relies on
            } else if (Mk) {
#pragma unroll
                for (int w = 0; w < 4; ++w) {   // a bf16 is positive iff its bits are in [0x0001, 0x7FFF]
                    const unsigned int lo = mk[t][w] & 0xFFFFu, hi = mk[t][w] >> 16;
                    const unsigned int keep = ((lo - 1u) < 0x7FFFu ? 0xFFFFu : 0u) | ((hi - 1u) < 0x7FFFu ? 0xFFFF0000u : 0u);
                    o[w] &= keep;
                }
            }
            buf_store(o, out_rs, own_off + t * step8);   // rows past the tensor are dropped
        }
    }
    OLS_TP(4);   // the tile's stores are issued
}

// ---------------------------------------------------------------------------------------------
// kernel / bias gradient
// ---------------------------------------------------------------------------------------------
template <int NV>   // strip vectors per lane (upper bound of (32 + 2 halo) * 8 / 256)
__global__ __launch_bounds__(kThreads, 2) void conv3x3_dw_bf16_kernel(ConvBDev p) {
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
    // bias gradient: column sums of the delta, taken from the delta fragments (a lane holds 8 pixels of one channel); the
    // two wavefronts that read the same fragments share the k-steps
    const bool col_sums = ci0 == 0;
    float col_acc = 0.0f;

    // Buffer addressing as in the forward kernel: lane t of the workgroup owns the 16-byte vector t % 8 of row t / 8 of a
    // [rows][C] tensor, its further vectors lie 32 rows below.  Input rows outside the tensor read as zeros, and so do the
    // delta's rows from the end of this workgroup's pixel range on (its descriptor ends there), which removes the pixels
    // past the range from the sums.
    static_assert(TD::kLineStep == 32 && TD::kPerThread == 2, "a lane's vectors are 32 rows apart in the strip and in the delta tile");
    const unsigned row_bytes = 2u * (unsigned)C;
    const unsigned lane_off = (threadIdx.x / 8) * row_bytes + (threadIdx.x % 8) * 16u;
    const unsigned step32 = 32u * row_bytes;
    const rsrc_t in_rs = make_rsrc(IN, (unsigned)p.Pp * row_bytes);
    const rsrc_t do_rs = make_rsrc(DO, (unsigned)hi * row_bytes);
    const int nvec = strip_rows * (kCB / 8);
    auto load_slice = [&](u4 (&r)[NV], u4 (&d)[TD::kPerThread], int k0) {
        const unsigned first = (unsigned)(k0 - p.halo) * row_bytes + lane_off;
#pragma unroll
        for (int t = 0; t < NV; ++t) r[t] = buf_load(in_rs, first + t * step32, 2u * ci0);
        const unsigned dfirst = (unsigned)k0 * row_bytes + lane_off;
#pragma unroll
        for (int t = 0; t < TD::kPerThread; ++t) d[t] = buf_load(do_rs, dfirst + t * step32, 2u * co0);
    };
    auto store_slice = [&](int buf, const u4 (&r)[NV], const u4 (&d)[TD::kPerThread]) {
        uint16_t* dst = lds_s(buf) + (threadIdx.x / 8) * RP + (threadIdx.x % 8) * 8;
#pragma unroll
        for (int t = 0; t < NV; ++t)
            if ((int)threadIdx.x + t * kThreads < nvec) *(u4*)(dst + t * 32 * RP) = r[t];   // the strip ends inside one of them
        uint16_t* dd = TD::lane_lds(lds_d(buf));
#pragma unroll
        for (int t = 0; t < TD::kPerThread; ++t) *(u4*)(dd + t * TD::kLdsLineStep) = d[t];
    };

    u4 rs[NV], rd[TD::kPerThread];
    load_slice(rs, rd, lo);
    store_slice(0, rs, rd);
    __syncthreads();
    const int nslices = (hi - lo + kDwBK - 1) / kDwBK;
    for (int t = 0; t < nslices; ++t) {
        const int cur = t & 1;
        if (t + 1 < nslices) load_slice(rs, rd, lo + (t + 1) * kDwBK);
        const uint16_t* S = lds_s(cur) + p.halo * RP;
        const uint16_t* D = lds_d(cur);
        // 4 k-steps x 9 taps = 12 groups of one kernel row: the fragments of group g + 1 are requested before the MFMAs
        // of group g (a lone just-in-time read would expose the LDS latency on every MFMA)
        constexpr int kGroups = (kDwBK / 16) * 3;
        bf16x8 fi[2][3], fd[2];
        auto load_group = [&](int g) {
            const int s = g / 3, kh = g % 3;
            if (kh == 0) fd[s & 1] = TD::frag(D, 32 * wj, s, lane);
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) fi[g & 1][kw] = TD::frag(S + ((kh - 1) * p.Wp + (kw - 1)) * RP, 32 * wi, s, lane);
        };
        load_group(0);
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            if (g + 1 < kGroups) load_group(g + 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kw = 0; kw < 3; ++kw)
                acc[3 * (g % 3) + kw] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fi[g & 1][kw], fd[(g / 3) & 1], acc[3 * (g % 3) + kw], 0, 0, 0);
            if (g % 3 == 0 && col_sums && (g / 3) / 2 == wi) {
                const u4 w = __builtin_bit_cast(u4, fd[(g / 3) & 1]);
#pragma unroll
                for (int e = 0; e < 4; ++e) col_acc += __uint_as_float(w[e] << 16) + __uint_as_float(w[e] & 0xFFFF0000u);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (t + 1 < nslices) store_slice(cur ^ 1, rs, rd);
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
    if (col_sums) {   // channel c: wavefronts (wi, wj = c / 32), both halves of their lanes, added in a fixed order
        float* red = (float*)lds_all;
        red[threadIdx.x] = col_acc;
        __syncthreads();
        if (threadIdx.x < kCB) {
            const float* r0 = red + 64 * (threadIdx.x / 32) + threadIdx.x % 32;   // wi = 0; wi = 1 is 128 lanes on
            PART[n_w + co0 + threadIdx.x] = ((r0[0] + r0[32]) + r0[128]) + r0[160];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// fp32 [B H W][C] -> bf16 [B (H+2) (W+2)][C] with a zero border; one lane per 8 channels of a padded pixel
// ---------------------------------------------------------------------------------------------
constexpr int kPadCastFly = 2;   // 16-byte output vectors per lane
__global__ __launch_bounds__(kThreads) void pad_cast_bf16_kernel(const float* __restrict__ src, int64_t s_src,
                                                                 uint16_t* __restrict__ dst, int64_t s_dst, unsigned vecs, int H,
                                                                 int W, int C, FastDiv div_c8, FastDiv div_per, FastDiv div_wp) {
    const int g = blockIdx.y;
    const unsigned c8 = (unsigned)C / 8, Wp = (unsigned)W + 2, per = (unsigned)(H + 2) * Wp;
    f4 lo[kPadCastFly], hi[kPadCastFly];
    bool img[kPadCastFly];
#pragma unroll
    for (int t = 0; t < kPadCastFly; ++t) {   // the loads of all the lane's vectors before the first store
        const unsigned v = (blockIdx.x * kPadCastFly + t) * kThreads + threadIdx.x;
        const unsigned q = fast_div(v < vecs ? v : 0u, div_c8), cv = (v < vecs ? v : 0u) - q * c8;
        const unsigned n = fast_div(q, div_per), rem = q - n * per;
        const unsigned y = fast_div(rem, div_wp), x = rem - y * Wp;
        img[t] = v < vecs && y >= 1 && y <= (unsigned)H && x >= 1 && x <= (unsigned)W;
        if (img[t]) {
            const f4* S = (const f4*)(src + (int64_t)g * s_src + ((int64_t)(n * H + y - 1) * W + (x - 1)) * C) + 2 * cv;
            lo[t] = __builtin_nontemporal_load(S);
            hi[t] = __builtin_nontemporal_load(S + 1);
        }
    }
#pragma unroll
    for (int t = 0; t < kPadCastFly; ++t) {
        const unsigned v = (blockIdx.x * kPadCastFly + t) * kThreads + threadIdx.x;
        if (v >= vecs) continue;
        u4 o = {0u, 0u, 0u, 0u};
        if (img[t]) {   // round to nearest even (v_cvt_pk_bf16_f32)
            o.x = __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{lo[t][0], lo[t][1]}, bf16x2));
            o.y = __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{lo[t][2], lo[t][3]}, bf16x2));
            o.z = __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{hi[t][0], hi[t][1]}, bf16x2));
            o.w = __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{hi[t][2], hi[t][3]}, bf16x2));
        }
        *((u4*)(dst + (int64_t)g * s_dst) + v) = o;
    }
}

// The block's tail in one streaming pass: a2 = relu(y + X) for the image pixels of one (sample, worker), its mean over
// the positions (global average pooling), and the sign of a2 for the backward pass -- a2 itself is needed nowhere else,
// so it is never written.  y: convolution output + bias, fp32 [Pp][C] with border rows (skipped); X: the shortcut, fp32
// [B H W][C]; sign[q][c / 4]: one byte per padded pixel and four channels, bit e set iff a2[q][4 (c / 4) + e] > 0 (border: 0).
// One workgroup per (sample, worker); thread = (channel vector, position stripe); stripes combined in a fixed order.
__global__ __launch_bounds__(kThreads) void shortcut_relu_pool_kernel(const float* __restrict__ y, int64_t s_y,
                                                                      const float* __restrict__ X, int64_t s_x, float* pooled,
                                                                      int64_t s_p, uint8_t* sign, int64_t s_sign, int H, int W, int C,
                                                                      FastDiv div_wp, float inv) {
    __shared__ f4 part[kThreads];
    const int c4n = C / 4, stripes = kThreads / c4n;
    const int c4 = threadIdx.x % c4n, stripe = threadIdx.x / c4n;
    const int b = blockIdx.x, g = blockIdx.y;
    const int Wp = W + 2, per = (H + 2) * Wp;
    const float* Y = y + (int64_t)g * s_y + (int64_t)b * per * C + 4 * c4;
    const float* Xs = X + (int64_t)g * s_x + (int64_t)b * H * W * C + 4 * c4;
    uint8_t* S = sign + (int64_t)g * s_sign + (int64_t)b * per * c4n + c4;
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    if (stripe < stripes) {
        constexpr int kFly = 8;
        for (int p0 = stripe; p0 < per; p0 += kFly * stripes) {   // kFly positions per thread in flight
            f4 yv[kFly], xv[kFly];
            bool in[kFly];
#pragma unroll
            for (int t = 0; t < kFly; ++t) {
                const int pp = p0 + t * stripes;
                const int yy = (int)fast_div((unsigned)pp, div_wp), xx = pp - yy * Wp;
                in[t] = pp < per && yy >= 1 && yy <= H && xx >= 1 && xx <= W;
                if (in[t]) {
                    yv[t] = __builtin_nontemporal_load((const f4*)(Y + (int64_t)pp * C));
                    xv[t] = __builtin_nontemporal_load((const f4*)(Xs + (int64_t)((yy - 1) * W + (xx - 1)) * C));
                }
            }
#pragma unroll
            for (int t = 0; t < kFly; ++t) {
                const int pp = p0 + t * stripes;
                if (pp >= per) continue;
                unsigned bits = 0;
                if (in[t]) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float a = fmaxf(yv[t][e] + xv[t][e], 0.0f);
                        acc[e] += a;
                        bits |= a > 0.0f ? (1u << e) : 0u;
                    }
                }
                S[(int64_t)pp * c4n] = (uint8_t)bits;
            }
        }
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    if (stripe == 0) {
        for (int s = 1; s < stripes; ++s) acc = acc + part[s * c4n + c4];
        f4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = acc[e] * inv;
        *(f4*)(pooled + (int64_t)g * s_p + (int64_t)b * C + 4 * c4) = o;
    }
}

// dz[g][q][c] = bf16(dpool[g][sample][c] * scale) where the sign bit of (q, c) is set, else 0; dz bf16 padded
constexpr int kPoolBwdFly = 4;   // 16-byte vectors per lane
__global__ __launch_bounds__(kThreads) void pool_bwd_bf16_kernel(const float* __restrict__ dpool, int64_t s_dp,
                                                                 const uint8_t* __restrict__ sign, int64_t s_sign, uint16_t* dz,
                                                                 int64_t s_dz, unsigned vecs, FastDiv div_c8, FastDiv div_pos,
                                                                 int C, float scale) {
    const int g = blockIdx.y;
    const unsigned c8 = (unsigned)C / 8;
    const uint8_t* SG = sign + (int64_t)g * s_sign;
    const float* DP = dpool + (int64_t)g * s_dp;
    u4* DZ = (u4*)(dz + (int64_t)g * s_dz);
    unsigned bits[kPoolBwdFly];
    f4 d0[kPoolBwdFly], d1[kPoolBwdFly];
#pragma unroll
    for (int t = 0; t < kPoolBwdFly; ++t) {   // all the loads of a lane's vectors before the first store
        const unsigned v = (blockIdx.x * kPoolBwdFly + t) * kThreads + threadIdx.x;
        if (v < vecs) {
            const unsigned q = fast_div(v, div_c8);
            const unsigned cv = v - q * c8;
            const unsigned sample = fast_div(q, div_pos);
            bits[t] = *(const uint16_t*)(SG + 2 * (int64_t)v);   // two bytes: channels 8 cv .. 8 cv + 7
            const f4* D = (const f4*)(DP + (int64_t)sample * C) + 2 * cv;
            d0[t] = D[0];
            d1[t] = D[1];
        }
    }
#pragma unroll
    for (int t = 0; t < kPoolBwdFly; ++t) {
        const unsigned v = (blockIdx.x * kPoolBwdFly + t) * kThreads + threadIdx.x;
        if (v >= vecs) continue;
        float o[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o[e] = (bits[t] >> e) & 1u ? d0[t][e] * scale : 0.0f;
            o[4 + e] = (bits[t] >> (8 + e)) & 1u ? d1[t][e] * scale : 0.0f;
        }
        u4 w;   // round to nearest even (v_cvt_pk_bf16_f32)
        w.x = __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{o[0], o[1]}, bf16x2));
        w.y = __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{o[2], o[3]}, bf16x2));
        w.z = __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{o[4], o[5]}, bf16x2));
        w.w = __builtin_bit_cast(unsigned, __builtin_convertvector(f2v{o[6], o[7]}, bf16x2));
        DZ[v] = w;
    }
}

// pooled[g][n][c] = inv * sum of the partial sums that a fused tail left for sample n: part w covers the pixels
// 64 w .. 64 w + 63 (padded pixels for the convolution's tail, image pixels for the normalisation's), its first sample
// is floor(64 w / per) with per pixels per sample, and its two slots are that sample and the next.
// Added in order of w; one lane per (sample, channel quad).
__global__ __launch_bounds__(kThreads) void pool_finish_kernel(const float* __restrict__ part, int64_t s_part, float* pooled,
                                                               int64_t s_p, int B, int per, int C, float inv) {
    const int v = blockIdx.x * kThreads + threadIdx.x;
    const int c4n = C / 4;
    if (v >= B * c4n) return;
    const int n = v / c4n, c4 = v % c4n, g = blockIdx.y;
    const f4* P = (const f4*)(part + (int64_t)g * s_part) + c4;
    const int w_lo = (n * per) / 64, w_hi = ((n + 1) * per - 1) / 64;
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    constexpr int kFly = 8;   // the loads of eight parts ahead of their additions
    for (int w0 = w_lo; w0 <= w_hi; w0 += kFly) {
        f4 v[kFly];
#pragma unroll
        for (int t = 0; t < kFly; ++t) {
            const int w = w0 + t <= w_hi ? w0 + t : w_hi;
            const int slot = n - (64 * w) / per;   // 0 or 1
            v[t] = P[(int64_t)(2 * w + slot) * c4n];
        }
#pragma unroll
        for (int t = 0; t < kFly; ++t)
            if (w0 + t <= w_hi) acc = acc + v[t];
    }
    f4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = acc[e] * inv;
    *(f4*)(pooled + (int64_t)g * s_p + (int64_t)n * C + 4 * c4) = o;
}

bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

bool shape_ok(const ConvBArgs& a) {
    if (a.groups < 1 || a.groups > 65535 || a.B < 1 || a.H < 1 || a.W < 1 || a.W > kConvBf16MaxWidth || a.C < kCB || a.C % kCB != 0 ||
        a.C > 1024)
        return false;
    const int64_t Pp = (int64_t)a.B * (a.H + 2) * (a.W + 2);
    // 32-bit byte offsets inside one group's bf16 tensor, with room for the rows a tile's strip reaches past either end
    return Pp * a.C < ((int64_t)1 << 31) - (int64_t)1024 * a.C;
}

void fill(ConvBDev* p, const ConvBArgs& a) {
    p->groups = a.groups; p->B = a.B; p->H = a.H; p->W = a.W; p->C = a.C;
    p->Hp = a.H + 2; p->Wp = a.W + 2; p->Pp = a.B * p->Hp * p->Wp; p->halo = p->Wp + 1;
    p->relu = a.relu;
    p->div_per = make_div((unsigned)(p->Hp * p->Wp));
    p->div_wp = make_div((unsigned)p->Wp);
}

template <int MODE>
hipError_t conv_launch(const ConvBArgs& a, hipStream_t s) {
    const bool tail = MODE == 0 && a.tail;
    if (!shape_ok(a) || !a.in || !a.w || !aligned16(a.in) || !aligned16(a.w)) return hipErrorInvalidValue;
    if (!tail && (!a.out || !aligned16(a.out) || a.s_out % 8)) return hipErrorInvalidValue;
    if (a.s_in % 8 || a.s_w % 8 || (a.mask && (!aligned16(a.mask) || a.s_mask % 8))) return hipErrorInvalidValue;
    if (tail) {   // 16-byte vectors of the shortcut, 32-bit byte offsets in it, at most two samples per 64 padded pixels
        if (a.out_f32 || a.relu || !a.xres || !a.sign || !a.pool_part || !aligned16(a.xres) || !aligned16(a.pool_part) || a.s_x % 4 ||
            (a.H + 2) * (a.W + 2) < 64 || (int64_t)a.B * a.H * a.W * a.C >= ((int64_t)1 << 30) - 1024)
            return hipErrorInvalidValue;
    }
    if (MODE == 0 && a.bias && (!aligned16(a.bias) || a.s_bias % 4)) return hipErrorInvalidValue;   // read as 16-byte vectors
    if (MODE == 1 && a.out_f32 && !a.out_unpadded) return hipErrorInvalidValue;   // a padded fp32 delta has no consumer
    if (a.out_unpadded && (!a.out_f32 || tail || (int64_t)a.B * a.H * a.W * a.C >= ((int64_t)1 << 30) - 1024)) return hipErrorInvalidValue;
    if (a.out_f32 && a.relu) return hipErrorInvalidValue;      // the fp32 output is the bare convolution + bias
    ConvBDev p = {};
    fill(&p, a);
    p.in = (const uint16_t*)a.in; p.w = (const uint16_t*)a.w; p.out = a.out;
    p.bias = MODE == 0 ? a.bias : nullptr;
    p.mask = MODE == 1 ? (const uint16_t*)a.mask : nullptr;
    p.s_in = a.s_in; p.s_w = a.s_w; p.s_out = a.s_out; p.s_bias = a.s_bias; p.s_mask = a.s_mask;
    if (tail) { p.xres = a.xres; p.s_x = a.s_x; p.sign = a.sign; p.s_sign = a.s_sign; p.pool_part = a.pool_part; }
    if (a.stat_part) {
        if (MODE != 0 || !a.out_unpadded || !aligned16(a.stat_part)) return hipErrorInvalidValue;
        p.stat_part = a.stat_part;
    }
    constexpr int BM = kBM;   // 128 (three workgroups per compute unit, 134 registers) measured 8 - 19 % slower: halo 1.55x
    p.tiles_m = (p.Pp + BM - 1) / BM;
    p.tiles_n = a.C / kCB;
    p.div_pg = make_div((unsigned)(p.tiles_m * p.tiles_n));
    p.div_tn = make_div((unsigned)p.tiles_n);
    const int64_t total = (int64_t)a.groups * p.tiles_m * p.tiles_n;
    if (total > (1 << 30)) return hipErrorInvalidValue;
    if (a.out_f32 && (int64_t)p.Pp * a.C >= ((int64_t)1 << 30)) return hipErrorInvalidValue;   // 32-bit byte offsets in the fp32 output
    p.total_tiles = (int)total;
    p.chunk = (int)((total + kXcds - 1) / kXcds);
    const int strip_rows = BM + 2 * p.halo;
    const size_t b_elems = MODE == 0 ? TileRC<kCB, kCB>::kElems : TileKC<kCB, kCB>::kElems;
    constexpr int NV0 = ((BM + 2 * 35) * (kCB / 8) + kThreads - 1) / kThreads;                        // widths up to 32
    constexpr int NV1 = ((BM + 2 * (kConvBf16MaxWidth + 3)) * (kCB / 8) + kThreads - 1) / kThreads;    // any width
    const int nv = (strip_rows * (kCB / 8) + kThreads - 1) / kThreads;
    if (nv > NV1) return hipErrorInvalidValue;
    const int lds_rows = 32 * (nv <= NV0 ? NV0 : NV1);   // the kernel's strip holds all the vectors its lanes move
    // the bf16 output tile is staged in the strip's place (BM x 72 bf16); the fp32 one is sized by conv_main_elems
    const int out = tail ? kOutTail : a.out_unpadded ? kOutF32U : a.out_f32 ? kOutF32 : kOutBf16;
    const size_t main_elems = out != kOutBf16 ? conv_main_elems<BM, kOutF32>(lds_rows, (int)b_elems) : conv_main_elems<BM, kOutBf16>(lds_rows, (int)b_elems);
    const size_t lds = main_elems * sizeof(uint16_t) + (out == kOutTail || out == kOutF32U ? BM * sizeof(int) : BM);   // strip and kernel slices (or the fp32 staging), row flags / indices
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    void (*kern)(ConvBDev);
    if (nv <= NV0)
        kern = MODE == 1 ? (out == kOutF32U ? conv3x3_bf16_kernel<1, kOutF32U, NV0, BM> : conv3x3_bf16_kernel<1, kOutBf16, NV0, BM>)
               : out == kOutTail ? conv3x3_bf16_kernel<0, kOutTail, NV0, BM>
               : out == kOutF32U ? conv3x3_bf16_kernel<0, kOutF32U, NV0, BM>
               : out == kOutF32  ? conv3x3_bf16_kernel<0, kOutF32, NV0, BM>
                                 : conv3x3_bf16_kernel<0, kOutBf16, NV0, BM>;
    else
        kern = MODE == 1 ? (out == kOutF32U ? conv3x3_bf16_kernel<1, kOutF32U, NV1, BM> : conv3x3_bf16_kernel<1, kOutBf16, NV1, BM>)
               : out == kOutTail ? conv3x3_bf16_kernel<0, kOutTail, NV1, BM>
               : out == kOutF32U ? conv3x3_bf16_kernel<0, kOutF32U, NV1, BM>
               : out == kOutF32  ? conv3x3_bf16_kernel<0, kOutF32, NV1, BM>
                                 : conv3x3_bf16_kernel<0, kOutBf16, NV1, BM>;
    if (lds > 64 * 1024) {
        hipError_t e = ensure_dynamic_lds((const void*)kern, 160 * 1024);
        if (e != hipSuccess) return e;
    }
    kern<<<(unsigned)(p.chunk * kXcds), kThreads, lds, s>>>(p);
    return hipGetLastError();
}

}  // namespace

#ifdef OLS_CONV_PHASE_PROBE
// dst[3][tiles][8] on the host: the readings of the last launch of each of the three kernels (see conv_phase_probe)
extern "C" __attribute__((visibility("default"))) int ols_debug_conv_phases(unsigned long long* dst, int tiles) {
    if (!dst || tiles < 1 || tiles > kProbeTiles) return -1;
    if (hipDeviceSynchronize() != hipSuccess) return -2;
    for (int k = 0; k < 3; ++k)
        if (hipMemcpyFromSymbol(dst + (size_t)k * tiles * 8, HIP_SYMBOL(conv_phase_probe), (size_t)tiles * 8 * sizeof(unsigned long long),
                                (size_t)k * kProbeTiles * 8 * sizeof(unsigned long long), hipMemcpyDeviceToHost) != hipSuccess)
            return -3;
    return 0;
}
#endif

hipError_t launch_conv3x3_bf16_fwd(const ConvBArgs& a, hipStream_t s) { return conv_launch<0>(a, s); }
hipError_t launch_conv3x3_bf16_dx(const ConvBArgs& a, hipStream_t s) { return conv_launch<1>(a, s); }

int conv3x3_bf16_dw_splits(int groups, int B, int H, int W, int C) {
    const int64_t Pp = (int64_t)B * (H + 2) * (W + 2);
    const int64_t tiles = (int64_t)groups * (C / kCB) * (C / kCB);
    int64_t s = (512 + tiles - 1) / tiles;                  // two workgroups per compute unit (registers and LDS allow two)
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
    if (nv <= 5) kern = conv3x3_dw_bf16_kernel<5>;
    else if (nv <= 11) kern = conv3x3_dw_bf16_kernel<11>;
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
    if (vecs >= ((int64_t)1 << 31) - kPadCastFly * kThreads) return hipErrorInvalidValue;   // the divisions by multiplication take 31-bit dividends
    const int64_t blocks = (vecs + kPadCastFly * kThreads - 1) / (kPadCastFly * kThreads);
    pad_cast_bf16_kernel<<<dim3((unsigned)blocks, (unsigned)groups), kThreads, 0, s>>>(
        src, s_src, dst, s_dst, (unsigned)vecs, H, W, C, make_div((unsigned)(C / 8)), make_div((unsigned)((H + 2) * (W + 2))),
        make_div((unsigned)(W + 2)));
    return hipGetLastError();
}

hipError_t launch_shortcut_relu_pool(const float* y, int64_t s_y, const float* X, int64_t s_x, float* pooled, int64_t s_p,
                                     uint8_t* sign, int64_t s_sign, int groups, int B, int H, int W, int C, hipStream_t s) {
    if (!y || !X || !pooled || !sign || groups < 1 || groups > 65535 || B < 1 || H < 1 || W < 1 || C < 8 || C % 8 || C > 1024 ||
        !aligned16(y) || !aligned16(X) || !aligned16(pooled) || (reinterpret_cast<uintptr_t>(sign) & 1u) || s_y % 4 || s_x % 4 ||
        s_p % 4 || s_sign % 2)
        return hipErrorInvalidValue;
    shortcut_relu_pool_kernel<<<dim3((unsigned)B, (unsigned)groups), kThreads, 0, s>>>(
        y, s_y, X, s_x, pooled, s_p, sign, s_sign, H, W, C, make_div((unsigned)(W + 2)), 1.0f / (float)(H * W));
    return hipGetLastError();
}

int64_t conv3x3_bf16_stat_part_floats(int B, int H, int W, int C) {
    const int64_t Pp = (int64_t)B * (H + 2) * (W + 2);
    return ((Pp + kBM - 1) / kBM) * 4 * 3 * C;   // per group
}

int64_t conv3x3_bf16_pool_part_floats(int B, int H, int W, int C) {
    const int64_t Pp = (int64_t)B * (H + 2) * (W + 2);
    return ((Pp + kBM - 1) / kBM) * 4 * 2 * C;   // per group
}

hipError_t launch_pool_finish(const float* part, int64_t s_part, float* pooled, int64_t s_p, int groups, int B, int per, int C,
                              float inv, hipStream_t s) {
    if (!part || !pooled || groups < 1 || groups > 65535 || B < 1 || C < 4 || C % 4 || !aligned16(part) || !aligned16(pooled) ||
        s_part % 4 || s_p % 4 || per < 64 || (int64_t)B * per >= ((int64_t)1 << 31) - 64)
        return hipErrorInvalidValue;
    const int64_t lanes = (int64_t)B * (C / 4);
    if (lanes > 0x7FFFFFFF) return hipErrorInvalidValue;
    pool_finish_kernel<<<dim3((unsigned)((lanes + kThreads - 1) / kThreads), (unsigned)groups), kThreads, 0, s>>>(part, s_part, pooled, s_p, B,
                                                                                                             per, C, inv);
    return hipGetLastError();
}

hipError_t launch_pool_bwd_bf16(const float* dpool, int64_t s_dp, const uint8_t* sign, int64_t s_sign, uint16_t* dz, int64_t s_dz,
                                int groups, int B, int positions, int C, float scale, hipStream_t s) {
    if (!dpool || !sign || !dz || groups < 1 || groups > 65535 || B < 1 || positions < 1 || C < 8 || C % 8 || !aligned16(dpool) ||
        (reinterpret_cast<uintptr_t>(sign) & 1u) || !aligned16(dz) || s_dp % 4 || s_sign % 2 || s_dz % 8)
        return hipErrorInvalidValue;
    const int64_t vecs = (int64_t)B * positions * (C / 8);
    if (vecs >= ((int64_t)1 << 31) - kPoolBwdFly * kThreads) return hipErrorInvalidValue;   // the divisions by multiplication take 31-bit dividends
    const int64_t blocks = (vecs + kPoolBwdFly * kThreads - 1) / (kPoolBwdFly * kThreads);
    pool_bwd_bf16_kernel<<<dim3((unsigned)blocks, (unsigned)groups), kThreads, 0, s>>>(
        dpool, s_dp, sign, s_sign, dz, s_dz, (unsigned)vecs, make_div((unsigned)(C / 8)), make_div((unsigned)positions), C, scale);
    return hipGetLastError();
}

}  // namespace ols
