// Internal declarations shared by the translation units of libols (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ols.h"

namespace ols {

// ---------------------------------------------------------------------------------------------
// Launchers.  Each validates its operand shapes on the host and returns a hipError_t; kernels
// themselves live in the matching kernels_*.hip file.  All pointers are device pointers.
// ---------------------------------------------------------------------------------------------

struct UpdateArgs {
    const float* g;     // [m][ld] gradients
    const float* x_in;  // [m][ld] parameters read
    float* x_out;       // [m][ld] parameters written (may alias x_in)
    float* buf;         // [m][ld] momentum buffers, in place (nullptr iff mu == 0)
    const float* z;     // [ld] anchor, read when pull
    uint16_t* shadow;   // [m][ld] bf16 copy of x_out written in the same pass, or nullptr
    int m;
    int64_t ld;
    float gamma, mu, alpha;
    bool nesterov, pull;
};
hipError_t launch_step(const UpdateArgs& a, hipStream_t s);                      // local step (+ pull-back)
hipError_t launch_pull(float* x, const float* z, uint16_t* shadow, int m, int64_t ld, float alpha,
                       hipStream_t s);                                            // stand-alone pull-back
hipError_t launch_stale_sync(float* x, float* snap, const float* z, uint16_t* shadow, int m, int64_t ld,
                             hipStream_t s);                                      // x <- z + (x - snap); snap <- x
hipError_t launch_init(float* x, float* x_alt, float* buf, float* z, uint16_t* shadow, const float* x0, int m,
                       int64_t d, int64_t ld, hipStream_t s);

struct MeanArgs {
    const float* x;  // [m][ld]
    float* z;        // [ld] anchor (read-modify-write when v != nullptr)
    float* v;        // [ld] anchor momentum buffer or nullptr
    int m;
    int64_t ld;
    float beta_z;
    int split;  // 0 auto, else wavefronts sharing the replica axis (1, 2, 4)
};
hipError_t launch_mean(const MeanArgs& a, hipStream_t s);
int mean_auto_split(int m, int64_t ld);

// step + pull-back + anchor refresh in one pass: one thread owns a column across all replicas
struct StepPullMeanArgs {
    UpdateArgs u;   // u.pull must be true
    float* z_out;   // [ld] new anchor (may alias u.z)
    float* v;       // anchor momentum or nullptr
    float beta_z;
    bool with_step; // false: pull-back + mean only (parameters already stepped)
};
hipError_t launch_step_pull_mean(const StepPullMeanArgs& a, hipStream_t s);
// one wavefront that waits `microseconds` (1 .. 1 000 000) of wall-clock time: emulated communication latency
hipError_t launch_delay(int64_t microseconds, hipStream_t s);

// general mixing X <- X W over the m + 1 rows [x^(1..m), z]
constexpr int kMixMaxWorkers = 128;
struct MixArgs {
    float* x;          // [m][ld] replicas, updated in place
    float* z;          // [ld] anchor (row m of X), updated in place
    uint16_t* shadow;  // [m][ld] bf16 copy of the new replicas, or nullptr
    const float* w;    // [(m + 1)][(m + 1)] row-major on the device
    int m;
    int64_t ld;
};
hipError_t launch_mix(const MixArgs& a, hipStream_t s);

// linear least squares
hipError_t launch_lsq_resid(const float* A, int64_t a_stride, const float* y, int64_t y_stride, const float* x,
                            int64_t ld, float* resid, float* loss_parts, int m, int B, int64_t d, hipStream_t s);
hipError_t launch_lsq_grad(const float* A, int64_t a_stride, const float* resid, float* g, int64_t ld, int m, int B,
                           int64_t d, hipStream_t s);

// Local step (+ pull-back) applied where a gradient element is produced, instead of writing the
// gradient to HBM and streaming it back in a separate pass.  Same fp32 operation sequence as the
// streaming kernels of kernels_update.hip, so both routes give identical bits.
struct FusedUpdate {
    const float* x_in;  // [m][ld] parameters read
    float* x_out;       // [m][ld] parameters written (may alias x_in)
    float* buf;         // [m][ld] momentum buffers (nullptr iff mu == 0)
    const float* z;     // [ld] anchor (pull-back steps)
    uint16_t* shadow;   // [m][ld] bf16 copy of the new parameters, or nullptr
    int64_t ld;
    float gamma, mu, alpha;
    int nesterov, pull;
    int enabled;
};

#if defined(__HIPCC__)
}  // namespace ols
#include "update_rule.h"
namespace ols {
// One element with the anchor value passed in (all operands were fetched ahead of the gradient).
// idx = worker * ld + position inside the replica row.
__device__ __forceinline__ void fused_update_store(const FusedUpdate& u, int64_t idx, float g, float x, float b,
                                                   float z) {
    const bool mom = u.mu != 0.0f;
    const float xn = local_step_elem(g, x, b, z, u.gamma, u.mu, u.alpha, mom, u.nesterov != 0, u.pull != 0);
    if (mom) u.buf[idx] = b;
    u.x_out[idx] = xn;
    if (u.shadow) u.shadow[idx] = (uint16_t)bf16_bits_rne(xn);
}
// The same with the anchor read here (col = position inside the replica row).
__device__ __forceinline__ void fused_update_apply(const FusedUpdate& u, int64_t idx, int64_t col, float g, float x,
                                                   float b) {
    fused_update_store(u, idx, g, x, b, u.pull ? u.z[col] : 0.0f);
}
#endif

// least squares, small problems: residual, loss, gradient and the local step (+ pull-back) in one launch
bool lsq_step_fits(int B, int64_t d);
hipError_t launch_lsq_step(const float* A, int64_t a_stride, const float* y, int64_t y_stride, float* loss_parts, int m,
                           int B, int64_t d, const FusedUpdate& u, hipStream_t s);

struct HeadArgs;

// grouped GEMMs over the m workers (group strides in elements)
struct GemmArgs {
    const void* a;      // operand A, group stride sa
    const void* b;      // operand B, group stride sb
    void* c;            // output, group stride sc
    const float* bias;  // fwd: [N] per group, stride sbias
    const void* mask;   // dA: activations whose sign gates the output, same shape as c, stride smask
    float* colsum;      // dw: optional [N] per group, receives the column sums of B (the bias gradient)
    float* partial;     // fp32 fwd with splits > 1: scratch of splits * groups * M * N floats
    int splits;         // fp32 fwd: number of K ranges contracted by separate workgroups (<= 1: none)
    int force_general;  // use the bounds-checked kernel even where the full-tile kernel applies
    const HeadArgs* guest;  // dw: the output layer's weight / bias gradients (launch_head_bwd's work) are computed by
                            // extra workgroups at the front of this launch; nullptr: none
    FusedUpdate upd;    // dw: when enabled, c is NOT written; the update of W (c's position in the replica row is
    int64_t upd_w_off;  //     upd_w_off) and of the bias (upd_b_off, from the column sums) is applied instead
    int64_t upd_b_off;
    int64_t sa, sb, sc, sbias, smask, scolsum;
    int groups;
    int M, N, K;        // output M x N, contraction length K
    int lda, ldb, ldc;  // leading dimensions (elements) of the operands as stored
};
// fp32 MFMA.  fwd: C[M][N] = relu(A[M][K] W[K][N] + bias);  dw: C[M][N] = A[K][M]^T B[K][N];
// da: C[M][N] = (A[M][K] B[N][K]^T) * (mask > 0)
hipError_t launch_gemm_f32_fwd(const GemmArgs& g, hipStream_t s, int variant);
void gemm_f32_fwd_plan(int groups, int M, int N, int K, int* variant, int* splits);
hipError_t launch_gemm_f32_dw(const GemmArgs& g, hipStream_t s, int variant);
hipError_t launch_gemm_f32_da(const GemmArgs& g, hipStream_t s, int variant);
// bf16 operands, fp32 accumulate.  fwd: A[M][K], W[K][N];  dw: A[K][M], B[K][N] (K = batch);  da: A[M][K], W[N][K]
hipError_t launch_gemm_bf16_fwd(const GemmArgs& g, hipStream_t s);
hipError_t launch_gemm_bf16_dw(const GemmArgs& g, hipStream_t s, int variant);
hipError_t launch_gemm_bf16_da(const GemmArgs& g, hipStream_t s);
hipError_t launch_cast_bf16(const float* src, int64_t src_stride, uint16_t* dst, int groups, int rows, int cols,
                            hipStream_t s);

// output layer (N = classes <= 32) on plain vector ALUs
struct HeadArgs {
    const void* h;        // [m][B][H] last hidden activations (fp32, or bf16 when h_bf16)
    int64_t h_stride;     // elements between workers in h
    bool h_bf16;
    const float* x;       // [m][ld] parameters; W_L at w_off, b_L at b_off within a row
    float* g;             // [m][ld] gradients, same offsets
    int64_t ld, w_off, b_off;
    const int32_t* labels;
    int64_t label_stride;
    float* dlogits;       // [m][B][C]
    float* loss_parts;    // [m][B] per-sample losses
    void* dz;             // [m][B][H] delta for the last hidden layer (fp32 or bf16), masked by h > 0
    int m, B, H, C;
    FusedUpdate upd;      // when enabled the output layer's parameters are updated instead of writing g
};
hipError_t launch_head_fwd(const HeadArgs& a, hipStream_t s);
hipError_t launch_head_bwd(const HeadArgs& a, hipStream_t s);
// 3 x 3 convolutions (stride 1, zero padding 1) grouped over the workers; activations [group][B H W][C] (channel
// contiguous), kernels [group][9][C][C] as (tap, input channel, output channel).  C a multiple of 16.
struct ConvArgs {
    const float* in;        // fwd: layer input; dx: delta of the layer output; dw: layer input
    const float* w;         // fwd, dx: kernels
    const float* dout;      // dw: delta of the layer output
    float* out;             // fwd: layer output; dx: delta of the layer input
    const float* bias;      // fwd: [C] per group, or nullptr for a convolution without bias
    const float* residual;  // fwd: added before the activation (same shape as out), or nullptr
    const float* mask;      // dx: activations whose sign gates the result (same shape as out), or nullptr
    float* partial;         // dw: scratch of conv3x3_dw_splits(...) * groups * (9 C C + C) floats
    float* g;               // dw: gradients [groups][ld]; kernel gradient at g_w_off, bias gradient at g_b_off of a row
                            // (g_b_off < 0: no bias, nothing written for it)
    int64_t ld, g_w_off, g_b_off;
    int64_t s_in, s_w, s_dout, s_out, s_bias, s_res, s_mask;   // group strides (elements)
    int groups, B, H, W, C;
    int relu;               // fwd: apply max(., 0)
};
hipError_t launch_conv3x3_fwd(const ConvArgs& a, hipStream_t s);
hipError_t launch_conv3x3_dx(const ConvArgs& a, hipStream_t s);
hipError_t launch_conv3x3_dw(const ConvArgs& a, hipStream_t s);   // weight + bias gradient (two launches)
int conv3x3_dw_splits(int groups, int B, int H, int W, int C);   // pixel ranges the weight-gradient contraction is split into
// second pass of the kernel gradient: sums the pixel ranges' parts [splits][groups][9 C C + C] in range order into g
hipError_t launch_conv_dw_finish(const float* partial, int splits, int groups, int C, float* g, int64_t ld, int64_t w_off,
                                 int64_t b_off, hipStream_t s);
// pooled = scale * sum over the HW positions of every sample (scale = 1 / HW: global average pooling), and the backward
// of the average through the ReLU in front of it
hipError_t launch_pool_mean(const float* a, int64_t s_a, float* pooled, int64_t s_p, int groups, int B, int HW, int C,
                            float scale, hipStream_t s);
hipError_t launch_pool_bwd(const float* dpool, int64_t s_dp, const float* a, int64_t s_a, float* dz, int64_t s_dz,
                           int groups, int B, int HW, int C, hipStream_t s);

// The same convolutions with bf16 operands.  Operand tensors carry their zero border: [group][B (H+2) (W+2)][C] bf16,
// channel contiguous; kernels [group][9][C][C] bf16.  C a multiple of 64, W at most kConvBf16MaxWidth.
constexpr int kConvBf16MaxWidth = 128;
struct ConvBArgs {
    const void* in;         // fwd: layer input; dx: delta of the layer output; dw: layer input (bf16, padded)
    const void* w;          // fwd, dx: bf16 kernels
    const void* dout;       // dw: delta of the layer output (bf16, padded)
    void* out;              // fwd: layer output; dx: delta of the layer input; padded, bf16 -- or, fwd with out_f32, the
                            // bare convolution + bias in fp32 with border rows as computed (their consumer skips them)
    int out_f32;
    int out_unpadded;       // with out_f32 (fwd and dx): fp32 [B H W][C], image pixels only -- what a batch normalisation reads
    float* stat_part;       // fwd with out_unpadded, optional: conv3x3_bf16_stat_part_floats(...) floats per group; per 64
                            // padded pixels (count, mean, sum of squared deviations) [3][C] of the output's image pixels,
                            // which launch_bn_forward takes instead of reading the output for its statistics
    const float* bias;      // fwd: [C] per group, or nullptr
    const void* mask;       // dx: padded bf16 activations whose sign gates the result, or nullptr
    float* partial;         // dw: scratch of conv3x3_bf16_dw_splits(...) * groups * (9 C C + C) floats
    float* g;               // dw: gradients [groups][ld]
    int64_t ld, g_w_off, g_b_off;   // g_b_off < 0: no bias
    int64_t s_in, s_w, s_dout, s_out, s_bias, s_mask;   // group strides (elements of the tensor's own type)
    int groups, B, H, W, C;
    int relu;               // fwd with bf16 output: apply max(., 0)
    // fwd with the residual block's tail fused in (tail != 0; out unused, no relu, padded images of at least 64 pixels):
    // a2 = relu(convolution + bias + xres) is never stored -- sign[padded pixel][C / 4] gets one byte per four channels
    // with bit e set iff a2 > 0 (border: 0), and pool_part (conv3x3_bf16_pool_part_floats(...) floats per group) the
    // partial sums that launch_pool_finish turns into the mean over the positions.
    int tail;
    const float* xres;      // fp32 [B H W][C], not padded
    uint8_t* sign;
    float* pool_part;
    int64_t s_x, s_sign;    // group strides
};
hipError_t launch_conv3x3_bf16_fwd(const ConvBArgs& a, hipStream_t s);
hipError_t launch_conv3x3_bf16_dx(const ConvBArgs& a, hipStream_t s);
hipError_t launch_conv3x3_bf16_dw(const ConvBArgs& a, hipStream_t s);
int conv3x3_bf16_dw_splits(int groups, int B, int H, int W, int C);
int64_t conv3x3_bf16_pool_part_floats(int B, int H, int W, int C);   // per group
int64_t conv3x3_bf16_stat_part_floats(int B, int H, int W, int C);   // per group
// pooled[g][sample][c] = inv * the sum over the sample's positions, from partial sums [group][w][2][C] per 64 consecutive
// pixels (slot 0: the sample of pixel 64 w, slot 1: the next one) with `per` (>= 64) pixels per sample
hipError_t launch_pool_finish(const float* part, int64_t s_part, float* pooled, int64_t s_p, int groups, int B, int per, int C,
                              float inv, hipStream_t s);
// fp32 [groups][B H W][C] -> bf16 [groups][B (H+2) (W+2)][C] with a zero border
hipError_t launch_pad_cast_bf16(const float* src, int64_t s_src, uint16_t* dst, int64_t s_dst, int groups, int B, int H, int W,
                                int C, hipStream_t s);
// The block's tail: a2 = relu(y + X) on the image pixels (y fp32 padded, X fp32 not padded), pooled = its mean over the
// positions, sign[padded pixel][C / 4] = one byte per four channels with bit e set iff a2 > 0 (border: 0).  a2 is not stored.
hipError_t launch_shortcut_relu_pool(const float* y, int64_t s_y, const float* X, int64_t s_x, float* pooled, int64_t s_p,
                                     uint8_t* sign, int64_t s_sign, int groups, int B, int H, int W, int C, hipStream_t s);
// dz = bf16(dpool * scale) where the sign bit is set, else 0; dz bf16 over `positions` (padded) positions per sample
hipError_t launch_pool_bwd_bf16(const float* dpool, int64_t s_dp, const uint8_t* sign, int64_t s_sign, uint16_t* dz, int64_t s_dz,
                                int groups, int B, int positions, int C, float scale, hipStream_t s);

// Batch normalisation in training mode over [group][P][C] tensors (statistics per group and channel over the P pixels).
struct BnArgs {
    const float* z;         // convolution output
    float* out;             // fwd: act(gamma xhat + beta (+ shortcut))
    const float* shortcut;  // fwd: added before the activation, or nullptr
    float* dy;              // bwd: gradient at the normalised output on entry, gradient at z on return (in place)
    float* stats;           // [group][2][C]: mean, 1 / sqrt(var + eps); written by fwd, read by bwd
    float* sums;            // bwd: [group][2][C] scratch (sum dy, sum dy xhat)
    float* part;            // scratch of bn_partial_floats(...) floats
    const float* gamma;     // scale, [C] per group
    const float* beta;      // shift (fwd)
    float* g;               // bwd: gradients [groups][ld]; d gamma at g_gamma_off, d beta at g_beta_off of a row
    int64_t ld, g_gamma_off, g_beta_off;
    int64_t s_z, s_out, s_sc, s_dy, s_par;   // group strides (elements); s_par for gamma and beta
    int groups, P, C;
    int relu;
    float eps;
    // Optional: the result (fwd: the activation; bwd: the gradient at z) goes out as bf16, to nearest even, in the padded
    // operand layout of the bf16 convolutions, [B (H + 2) (W + 2)][C] per group with P = B H W -- only the image pixels
    // are written (the border is zero from the start and stays so); `out` / the in-place update of dy are then skipped.
    uint16_t* out_bf16;
    int64_t s_outb;
    int H, W;
    // Optional (bwd): the normalised output sits under a ReLU and global average pooling, so the gradient on entry is
    // dpool[group][sample][c] / positions where gate (the activation, [group][P][C]) is positive and 0 elsewhere; it is
    // formed on the fly and dy is only written (the gradient at z), or not touched at all with out_bf16.
    const float* gate;
    const float* dpool;
    int64_t s_gate, s_dp;
    int positions;
    // Optional (fwd): per-wavefront statistics that the producer of z left (ConvBArgs::stat_part), [group][waves][3][C]:
    // the statistics are merged from them and z is read only once, by the normalisation itself.
    const float* wave_part;
    int waves;
    // Optional (fwd, with shortcut / relu as given; H * W >= 64): the block's tail.  The activation is not stored: `sign`
    // gets one byte per pixel and four channels ([group][P][C / 4], bit e set iff the activation is positive) and
    // `pool_part` ([group][ceil(P / 64)][2][C] floats) the activation's sums per 64 pixels for launch_pool_finish.
    // (bwd) `sign` in place of `gate`: the same bytes say where the activation was positive.
    uint8_t* sign;
    float* pool_part;
    int64_t s_sign;
};
hipError_t launch_bn_forward(const BnArgs& a, hipStream_t s);    // statistics (two launches) + normalise
hipError_t launch_bn_backward(const BnArgs& a, hipStream_t s);   // sums (two launches) + gradient at z
int64_t bn_partial_floats(int groups, int P, int C);

// raises a kernel's dynamic-LDS limit once per (device, kernel)
hipError_t ensure_dynamic_lds(const void* kernel, size_t bytes);
inline int64_t round_up(int64_t v, int64_t q) { return (v + q - 1) / q * q; }

}  // namespace ols
