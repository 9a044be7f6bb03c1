// Output layer of the per-worker MLP (class count C <= 32) with softmax cross-entropy, the delta it
// sends back to the last hidden layer, and its own gradients.  The output width is far too small for
// matrix cores, so these run on the vector ALUs.  They are a few MFLOP per worker: what they cost is
// (a) the chain of dependent memory round trips and (b) instruction fetch -- a launch this small runs
// every instruction a handful of times, so long unrolled code is paid for line by line from a cold
// instruction cache.  Hence the shape of both kernels: all global reads of a pass are issued together
// and land in LDS, and the arithmetic runs in short rolled loops over LDS.
//
//   head_fwd_kernel   logits, loss, dlogits AND the hidden delta dz in one launch.  Sixteen lanes (one
//                     DPP row) share a sample; the 16 partial logits are combined with DPP row
//                     rotations, every lane then evaluates the softmax redundantly, and the staged
//                     activations (ReLU mask) and weights are reused for dz.
//   head_dw_kernel    dW = h^T dlogits, db = colsum(dlogits), consumed by the fused update or stored (body in
//                     head_dw_body.h; by default it runs as guest workgroups of a weight-gradient GEMM instead).
//
// Per worker i with last hidden activations h [B][H], weights W [H][C], bias b [C], labels y [B]
// (the mini-batch loss whose gradient is the g_i of Section 2, arXiv 2002.09539):
//   logits = h W + b;  loss_s = logsumexp(logits_s) - logits_s[y_s];  dlogits = (softmax - onehot) / B
//   dW = h^T dlogits;  db = colsum(dlogits);  dz = (dlogits W^T) * [h > 0]
// The class dimension is padded to CMAX (16 or 32) with zeros in LDS so that no inner loop branches on C.
#include "head_dw_body.h"
#include "ols_internal.h"

namespace ols {

constexpr int kRow = 16;     // lanes of one DPP row
constexpr int kMaxC = 32;

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ unsigned int f32_to_bf16(float f) { return bf16_bits_rne(f); }
// Sum over the 16 lanes of a DPP row, the same bits in every lane of the row (each step adds a lane's
// value to that of its partner 8, 4, 2, 1 lanes away, which is symmetric).
__device__ __forceinline__ float row_sum(float v) {
#define OLS_ROW_ROR_ADD(n)                                                                                  \
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + (n), 0xF, 0xF, false))
    OLS_ROW_ROR_ADD(8);
    OLS_ROW_ROR_ADD(4);
    OLS_ROW_ROR_ADD(2);
    OLS_ROW_ROR_ADD(1);
#undef OLS_ROW_ROR_ADD
    return v;
}

__device__ __forceinline__ float row_max(float v) {
#define OLS_ROW_ROR_MAX(n)                                                                                  \
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + (n), 0xF, 0xF, false)))
    OLS_ROW_ROR_MAX(8);
    OLS_ROW_ROR_MAX(4);
    OLS_ROW_ROR_MAX(2);
    OLS_ROW_ROR_MAX(1);
#undef OLS_ROW_ROR_MAX
    return v;
}

struct HeadDev {
    const void* h;
    const float* x;
    const int32_t* labels;
    float* dlogits;
    float* loss_parts;
    void* dz;
    int64_t h_stride, ld, w_off, b_off, label_stride;
    int B, H, C;
};

// KC = hidden units staged per pass; THREADS / 16 samples per workgroup; activation rows are staged at pitch KC + 4
__host__ __device__ constexpr int head_fwd_lds_floats(int CMAX, int KC, int THREADS) {
    return KC * head_row_pitch(CMAX) + (THREADS / kRow) * (KC + 4) + (THREADS / kRow) * CMAX;
}

// grid (ceil(B / (THREADS / 16)), m); dynamic LDS: head_fwd_lds_floats(CMAX, KC, THREADS) floats
template <bool BF, int CMAX, int KC, int THREADS>
__global__ __launch_bounds__(THREADS) void head_fwd_kernel(HeadDev p) {
    constexpr int S = THREADS / kRow, HP = KC + 4;
    static_assert(THREADS % 64 == 0 && (KC * CMAX) % THREADS == 0 && KC % 128 == 0, "staging shape");
    constexpr int P = head_row_pitch(CMAX);         // LDS pitch of a weight row
    constexpr int NW = KC * CMAX / THREADS;    // staged weights per lane, all in flight at once
    constexpr int J = KC / (4 * kRow);         // 4-wide activation vectors per lane per pass (8)
    extern __shared__ __attribute__((aligned(16))) float s_dyn[];
    float* s_w = s_dyn;                        // [KC slots][P]
    float* s_h = s_dyn + KC * P;               // [S][HP]
    float* s_d = s_h + S * HP;                 // [S][CMAX] dlogits of the workgroup's samples

    const int C = p.C, H = p.H, B = p.B;
    const int i = blockIdx.y;
    const int row = threadIdx.x / kRow, sub = threadIdx.x % kRow;
    const int s0 = blockIdx.x * S, s = s0 + row;
    const bool live = s < B;
    const int cls = threadIdx.x % CMAX;
    const float* W = p.x + (int64_t)i * p.ld + p.w_off;

    float bias[CMAX / kRow];   // lane sub owns class sub (and sub + 16)
#pragma unroll
    for (int c0 = 0; c0 < CMAX / kRow; ++c0)
        bias[c0] = kRow * c0 + sub < C ? p.x[(int64_t)i * p.ld + p.b_off + kRow * c0 + sub] : 0.0f;
    const int label = live ? p.labels[(int64_t)i * p.label_stride + s] : 0;

    // One pass: KC rows of W from k0 (zero beyond H and beyond C) and the same KC activations of the 16
    // samples (zero beyond H and beyond the batch) into LDS; every load is issued before the first store.
    // Weight row kl goes to slot (kl % 4) * (KC / 4) + kl / 4: element e of a lane's vector j then sits at
    // slot e * (KC / 4) + sub + 16 j, consecutive across the lanes of a DPP row, and at pitch P their
    // 16-byte reads fall into distinct banks.
    auto stage = [&](int k0) {
        const float* src = W + (int64_t)k0 * C + cls;
        const int rows = H - k0;
        float tw[NW];
#pragma unroll
        for (int u = 0; u < NW; ++u) {
            const int kl = threadIdx.x / CMAX + u * (THREADS / CMAX);
            tw[u] = (cls < C && kl < rows) ? src[kl * C] : 0.0f;
        }
        if constexpr (BF) {
            constexpr int NH = S * KC / 8 / THREADS;   // 16-byte vectors of 8 bf16 per lane (4)
            u4 th[NH];
#pragma unroll
            for (int u = 0; u < NH; ++u) {
                const int f = threadIdx.x + u * THREADS, r = f / (KC / 8), kv = 8 * (f % (KC / 8));
                th[u] = u4{0u, 0u, 0u, 0u};
                if (s0 + r < B && k0 + kv < H)
                    th[u] = *(const u4*)((const uint16_t*)p.h + (int64_t)i * p.h_stride + (int64_t)(s0 + r) * H + k0 + kv);
            }
#pragma unroll
            for (int u = 0; u < NH; ++u) {
                const int f = threadIdx.x + u * THREADS, r = f / (KC / 8), kv = 8 * (f % (KC / 8));
                *(f4*)(s_h + r * HP + kv) = f4{head_bf16_elem(th[u].x, 0), head_bf16_elem(th[u].x, 1), head_bf16_elem(th[u].y, 0),
                                               head_bf16_elem(th[u].y, 1)};
                *(f4*)(s_h + r * HP + kv + 4) = f4{head_bf16_elem(th[u].z, 0), head_bf16_elem(th[u].z, 1), head_bf16_elem(th[u].w, 0),
                                                   head_bf16_elem(th[u].w, 1)};
            }
        } else {
            constexpr int NH = S * KC / 4 / THREADS;   // 16-byte vectors of 4 floats per lane (8)
            f4 th[NH];
#pragma unroll
            for (int u = 0; u < NH; ++u) {
                const int f = threadIdx.x + u * THREADS, r = f / (KC / 4), kv = 4 * (f % (KC / 4));
                th[u] = f4{0.f, 0.f, 0.f, 0.f};
                if (s0 + r < B && k0 + kv < H)
                    th[u] = *(const f4*)((const float*)p.h + (int64_t)i * p.h_stride + (int64_t)(s0 + r) * H + k0 + kv);
            }
#pragma unroll
            for (int u = 0; u < NH; ++u) {
                const int f = threadIdx.x + u * THREADS, r = f / (KC / 4), kv = 4 * (f % (KC / 4));
                *(f4*)(s_h + r * HP + kv) = th[u];
            }
        }
#pragma unroll
        for (int u = 0; u < NW; ++u) {
            const int kl = threadIdx.x / CMAX + u * (THREADS / CMAX);
            s_w[((kl % 4) * (KC / 4) + kl / 4) * P + cls] = tw[u];
        }
    };

    // Passes 0 .. n - 1 accumulate the logits over the chunks of H, the last of them ends with the softmax;
    // passes n .. 2 n - 1 (only when dz is wanted) produce dz chunk by chunk.  One loop, so that the staging
    // code exists once.  With a single chunk the weights and activations staged for the logits are still in
    // LDS for dz; otherwise they are fetched again (they hit L2).
    float acc[CMAX], d[CMAX];
#pragma unroll
    for (int c = 0; c < CMAX; ++c) acc[c] = d[c] = 0.0f;
    const int n = (H + KC - 1) / KC;
    const int passes = p.dz ? 2 * n : n;
#pragma unroll 1
    for (int pass = 0; pass < passes; ++pass) {
        const bool backward = pass >= n;
        const int k0 = (backward ? pass - n : pass) * KC;
        if (!(backward && n == 1)) {
            if (pass > 0) __syncthreads();   // the previous pass is no longer read
            stage(k0);
            __syncthreads();
        }
        if (!backward) {
#pragma unroll 1
            for (int j = 0; j < J; ++j) {
                const f4 hv = *(const f4*)(s_h + row * HP + 4 * (sub + kRow * j));
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float* wr = s_w + (e * (KC / 4) + sub + kRow * j) * P;
#pragma unroll
                    for (int c4 = 0; c4 < CMAX / 4; ++c4) {
                        const f4 w = *(const f4*)(wr + 4 * c4);
#pragma unroll
                        for (int q = 0; q < 4; ++q) acc[4 * c4 + q] = __fmaf_rn(hv[e], w[q], acc[4 * c4 + q]);
                    }
                }
            }
            if (pass != n - 1) continue;
            // Softmax with the classes spread over the 16 lanes of the row: lane sub owns class sub (and
            // sub + 16 when CMAX = 32), so each lane evaluates one or two exponentials instead of CMAX.
            // The other classes' terms are summed separately from the label's: near convergence
            // softmax[label] is within an ulp of 1, and both the loss log(1 + others / own) and the
            // label's delta -(others / total) keep full relative accuracy this way, where
            // log(total) - logit and softmax - 1 would cancel.
            float logit[CMAX / kRow], ex[CMAX / kRow];
            float mx = -INFINITY;
#pragma unroll
            for (int c0 = 0; c0 < CMAX / kRow; ++c0) {
                float v = 0.0f;
#pragma unroll
                for (int c = 0; c < kRow; ++c) {
                    const float full = row_sum(acc[kRow * c0 + c]);   // every lane takes part in every sum
                    v = c == sub ? full : v;
                }
                logit[c0] = kRow * c0 + sub < C ? v + bias[c0] : -INFINITY;
                mx = fmaxf(mx, logit[c0]);
            }
            mx = row_max(mx);
            float others = 0.0f, own = 0.0f, picked = 0.0f;
#pragma unroll
            for (int c0 = 0; c0 < CMAX / kRow; ++c0) {
                ex[c0] = expf(logit[c0] - mx);            // exp(-inf) = 0 for the padding
                const bool is_label = kRow * c0 + sub == label;
                own += is_label ? ex[c0] : 0.0f;
                picked += is_label ? logit[c0] : 0.0f;
                others += is_label ? 0.0f : ex[c0];
            }
            others = row_sum(others);
            own = row_sum(own);          // one non-zero term
            picked = row_sum(picked);    // one non-zero term
            const float sum = others + own;
            const float scale = 1.0f / (sum * (float)B);   // dlogits = (softmax - onehot) / B
            if (live && sub == 0)
                p.loss_parts[(int64_t)i * B + s] = own > 1e-30f ? log1pf(others / own) : (logf(sum) + mx) - picked;
#pragma unroll
            for (int c0 = 0; c0 < CMAX / kRow; ++c0) {
                const int c = kRow * c0 + sub;
                const float dv = (c == label ? -others : ex[c0]) * scale;   // 0 for the padding
                s_d[row * CMAX + c] = dv;
                if (live && c < C) p.dlogits[((int64_t)i * B + s) * C + c] = dv;
            }
            __syncthreads();
#pragma unroll
            for (int c4 = 0; c4 < CMAX / 4; ++c4) {
                const f4 v = *(const f4*)(s_d + row * CMAX + 4 * c4);
#pragma unroll
                for (int q = 0; q < 4; ++q) d[4 * c4 + q] = v[q];
            }
            continue;
        }
        // dz[s][k] = (sum_c dlogits[s][c] W[k][c]) * [h[s][k] > 0]
#pragma unroll 1
        for (int j = 0; j < J; ++j) {
            const int kl = 4 * (sub + kRow * j), kv = k0 + kl;
            const f4 hv = *(const f4*)(s_h + row * HP + kl);
            f4 out;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float* wr = s_w + (e * (KC / 4) + sub + kRow * j) * P;
                float a = 0.0f;
#pragma unroll
                for (int c4 = 0; c4 < CMAX / 4; ++c4) {
                    const f4 w = *(const f4*)(wr + 4 * c4);
#pragma unroll
                    for (int q = 0; q < 4; ++q) a = __fmaf_rn(d[4 * c4 + q], w[q], a);   // padding: d = 0, w = 0
                }
                out[e] = hv[e] > 0.0f ? a : 0.0f;
            }
            if constexpr (BF) {
                const unsigned int h0 = f32_to_bf16(out[0]), h1 = f32_to_bf16(out[1]), h2 = f32_to_bf16(out[2]),
                                   h3 = f32_to_bf16(out[3]);
                if (live && kv < H)
                    *(u2*)((uint16_t*)p.dz + (int64_t)i * B * H + (int64_t)s * H + kv) = u2{h0 | (h1 << 16), h2 | (h3 << 16)};
            } else {
                if (live && kv < H) *(f4*)((float*)p.dz + (int64_t)i * B * H + (int64_t)s * H + kv) = out;
            }
        }
    }
}

// Output-layer gradients as a kernel of their own (the body lives in head_dw_body.h, where it also serves as a
// guest of the weight-gradient GEMM's launch).  grid (ceil(H / 32), m)
template <bool BF, int CMAX>
__global__ __launch_bounds__(kHeadDwThreads) void head_dw_kernel(HeadDwDev a) {
    constexpr int kRows = CMAX > 16 ? 128 : 256;      // samples staged per pass (LDS stays below 64 KiB)
    __shared__ __attribute__((aligned(16))) float lds[head_dw_lds_floats(CMAX, kRows)];
    head_dw_body<BF, CMAX, kRows>(a, lds, blockIdx.x, blockIdx.y);
}

static bool head_args_ok(const HeadArgs& a) {
    return a.h && a.x && a.g && a.labels && a.dlogits && a.loss_parts && a.m >= 1 && a.m <= 65535 && a.B >= 1 &&
           a.H >= 4 && a.H % 4 == 0 && a.C >= 1 && a.C <= kMaxC && a.w_off >= 0 && a.b_off >= 0 &&
           a.w_off + (int64_t)a.H * a.C <= a.ld && a.b_off + a.C <= a.ld &&
           (reinterpret_cast<uintptr_t>(a.h) & 15u) == 0 && a.h_stride % 4 == 0;
}

template <bool BF, int CMAX, int KC, int THREADS>
static hipError_t head_fwd_launch(const HeadDev& p, int m, hipStream_t s) {
    size_t lds = (size_t)head_fwd_lds_floats(CMAX, KC, THREADS) * sizeof(float);
    auto kern = head_fwd_kernel<BF, CMAX, KC, THREADS>;
    if (lds > 64 * 1024) {
        hipError_t e = ensure_dynamic_lds((const void*)kern, lds);
        if (e != hipSuccess) return e;
    }
    constexpr int kSamples = THREADS / kRow;
    dim3 grid((unsigned)((p.B + kSamples - 1) / kSamples), (unsigned)m);
    kern<<<grid, THREADS, lds, s>>>(p);
    return hipGetLastError();
}

// logits, loss, dlogits, and (when a.dz is set) the delta of the last hidden layer
hipError_t launch_head_fwd(const HeadArgs& a, hipStream_t s) {
    if (!head_args_ok(a)) return hipErrorInvalidValue;
    // 16-byte activation vectors: 4 floats or 8 bf16
    if (a.h_bf16 && (a.H % 8 || a.h_stride % 8)) return hipErrorInvalidValue;
    if (a.dz && (reinterpret_cast<uintptr_t>(a.dz) & 15u)) return hipErrorInvalidValue;
    HeadDev p;
    p.h = a.h;
    p.x = a.x;
    p.labels = a.labels;
    p.dlogits = a.dlogits;
    p.loss_parts = a.loss_parts;
    p.dz = a.dz;
    p.h_stride = a.h_stride;
    p.ld = a.ld;
    p.w_off = a.w_off;
    p.b_off = a.b_off;
    p.label_stride = a.label_stride;
    p.B = a.B;
    p.H = a.H;
    p.C = a.C;
    // Wider layers are staged 1024 hidden units at a time (146 KiB of LDS with 16 classes): half as many
    // dependent passes, and up to H = 1024 the delta reuses what the logits staged.
    // Workgroup size.  What a workgroup pays per pass is the staging of the weights, whatever the number of its
    // samples: measured with 64 / 128 / 256 / 512 threads (4 to 32 samples) and 512 staged units, 16 workers x 128
    // samples x 512 units: 19.5 / 17.0 / 15.4 / 14.0 us; 256 samples x 2048 units: 148 / 60 / 52 / 52 us.  So:
    // 32 samples per workgroup where one pass covers the layer and the batch has them, 16 otherwise.
    const bool wide = a.H > 512 && a.C <= 16;
    const bool big = !wide && a.C <= 16 && a.B >= 32;
    if (a.h_bf16) {
        if (a.C > 16) return head_fwd_launch<true, 32, 512, 256>(p, a.m, s);
        if (big) return head_fwd_launch<true, 16, 512, 512>(p, a.m, s);
        return wide ? head_fwd_launch<true, 16, 1024, 256>(p, a.m, s) : head_fwd_launch<true, 16, 512, 256>(p, a.m, s);
    }
    if (a.C > 16) return head_fwd_launch<false, 32, 512, 256>(p, a.m, s);
    if (big) return head_fwd_launch<false, 16, 512, 512>(p, a.m, s);
    return wide ? head_fwd_launch<false, 16, 1024, 256>(p, a.m, s) : head_fwd_launch<false, 16, 512, 256>(p, a.m, s);
}

// Validates the arguments of the output layer's gradient pass and lays them out for the device.
hipError_t head_dw_prepare(const HeadArgs& a, HeadDwDev* out) {
    if (!head_args_ok(a)) return hipErrorInvalidValue;
    if (a.upd.enabled && (!a.upd.x_in || !a.upd.x_out || (a.upd.mu != 0.0f && !a.upd.buf) || (a.upd.pull && !a.upd.z) ||
                          a.upd.ld != a.ld))
        return hipErrorInvalidValue;
    HeadDwDev d = {};
    d.h = a.h;
    d.dlogits = a.dlogits;
    d.g = a.g;
    d.h_stride = a.h_stride;
    d.ld = a.ld;
    d.w_off = a.w_off;
    d.b_off = a.b_off;
    d.B = a.B;
    d.H = a.H;
    d.C = a.C;
    d.bf16 = a.h_bf16 ? 1 : 0;
    d.grid_x = (a.H + kHeadDwUnits - 1) / kHeadDwUnits;
    const int64_t live = (int64_t)d.grid_x * a.m;
    if (live > (1 << 24)) return hipErrorInvalidValue;
    d.live = (int)live;
    d.blocks = (int)round_up(live, 8);   // a host launch keeps its own workgroup -> XCD assignment
    d.upd = a.upd;
    *out = d;
    return hipSuccess;
}

// gradients of the output layer's weights and bias (stored to g, or consumed by the fused update)
hipError_t launch_head_bwd(const HeadArgs& a, hipStream_t s) {
    HeadDwDev d;
    hipError_t e = head_dw_prepare(a, &d);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)d.grid_x, (unsigned)a.m);
    if (a.h_bf16) {
        if (a.C <= 16) head_dw_kernel<true, 16><<<grid, kHeadDwThreads, 0, s>>>(d);
        else head_dw_kernel<true, 32><<<grid, kHeadDwThreads, 0, s>>>(d);
    } else {
        if (a.C <= 16) head_dw_kernel<false, 16><<<grid, kHeadDwThreads, 0, s>>>(d);
        else head_dw_kernel<false, 32><<<grid, kHeadDwThreads, 0, s>>>(d);
    }
    return hipGetLastError();
}

}  // namespace ols
