// The update rules of Overlap Local-SGD (arXiv 2002.09539, Section 2, "Proposed Algorithm" and the "Momentum
// Variant" paragraph) for ONE parameter element, written out once.  Every kernel that updates parameters -- the
// streaming kernels, the one-pass step + pull-back + mean kernel, the epilogues of the weight-gradient GEMMs, the
// output-layer and least-squares kernels -- calls these functions, so all routes execute the same sequence of
// explicitly rounded fp32 operations and leave identical bits.
//
//   local step   buf' = mu buf + g;  dir = g + mu buf' (Nesterov) or buf' (heavy ball);  x_half = x - gamma dir
//                (without momentum: x_half = x - gamma g)
//   pull-back    x' = x_half - alpha (x_half - z)            on the tau-th step of a round, z the OLD anchor
//   anchor       z' = (sum_i x'_i) / m;  momentum form v' = beta_z v + (mean - z), z' = z + v'
#pragma once
#include <hip/hip_runtime.h>

namespace ols {

// Pull-back of one element toward the anchor (second update rule of Section 2).
__device__ __forceinline__ float pull_back_elem(float x_half, float z, float alpha) {
    return __fmaf_rn(-alpha, __fsub_rn(x_half, z), x_half);
}

// Local (momentum) step of one element, optionally followed by the pull-back.  `b` is the momentum buffer entry,
// updated in place when mom; `z` is read only when pull.  The flags are compile-time constants at most call sites
// (the function is always inlined), run-time values of the launch elsewhere.
__device__ __forceinline__ float local_step_elem(float g, float x, float& b, float z, float gamma, float mu, float alpha,
                                                 bool mom, bool nesterov, bool pull) {
    float x_half;
    if (mom) {
        b = __fmaf_rn(mu, b, g);
        const float dir = nesterov ? __fmaf_rn(mu, b, g) : b;
        x_half = __fmaf_rn(-gamma, dir, x);
    } else {
        x_half = __fmaf_rn(-gamma, g, x);
    }
    return pull ? pull_back_elem(x_half, z, alpha) : x_half;
}

// Anchor from the sum over the m replicas (third update rule): correctly rounded division by m.
__device__ __forceinline__ float anchor_mean_elem(float sum, float m) { return __fdiv_rn(sum, m); }

// Anchor momentum ("Momentum Variant"): v' = beta_z v + (mean - z); returns z' = z + v'.
__device__ __forceinline__ float anchor_momentum_elem(float mean, float z, float& v, float beta_z) {
    v = __fmaf_rn(beta_z, v, __fsub_rn(mean, z));
    return __fadd_rn(z, v);
}

// fp32 -> bf16 bits, round to nearest even (the bf16 copy of the parameters the bf16 GEMMs read).
__device__ __forceinline__ unsigned int bf16_bits_rne(float f) {
    const unsigned int u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

}  // namespace ols
