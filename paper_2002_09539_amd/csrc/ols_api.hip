// C boundary and schedule of the Overlap Local-SGD hot path (arXiv 2002.09539, Section 2).
//
// The host side here only orders kernels on two caller-owned streams and checks the call order the
// algorithm prescribes; every arithmetic step runs in the kernels of the other translation units.
//
// Overlap (the paper's timeline figure, carried out inside one GPU): after the pull-back at the end of
// round a the main stream records `ev_pulled`; the side stream waits for it, reduces the replica axis
// into the anchor and records `ev_anchor_done`; the main stream waits for that event only in front of the first
// launch that consumes the refreshed anchor: the NEXT pull-back -- on the default route, where the kernels that form
// the gradients apply step and pull-back themselves, the first updating launch of the round's tau-th step (the
// output layer's gradient kernel, or the weight-gradient launch that hosts its workgroups), after that step's
// forward and delta kernels.  The refresh must see the
// round-boundary models while the next round already updates them, so the first update after a refresh
// is written out-of-place into the second replica buffer (same HBM traffic) and the buffers swap roles;
// without a second buffer that first update waits for the refresh instead.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <string>
#include <vector>

#include "ols_internal.h"

using namespace ols;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

const char* kKernelNames[OLS_K_COUNT] = {
    "init",      "step",     "step_pull", "pull",     "mean",     "step_pull_mean", "lsq_resid", "lsq_grad",
    "gemm_fwd",  "gemm_dw",  "gemm_da",   "head_fwd", "head_bwd", "mix",            "cast_bf16", "delay",    "lsq_step",
    "stale_sync", "conv_fwd",  "conv_dx",   "conv_dw",  "pool",     "pool_bwd",      "bn_fwd",    "bn_bwd"};

enum { MODEL_NONE = 0, MODEL_LSQ = 1, MODEL_MLP = 2, MODEL_CONV = 3 };

struct TimedLaunch {
    int kind;
    hipEvent_t start, stop;
};

}  // namespace

struct ols_ctx {
    // problem
    int m = 0, tau = 1;
    int64_t d = 0, ld = 0;
    float alpha = 0, gamma = 0, mu = 0, beta_z = 0;
    // bound state
    float* x[2] = {nullptr, nullptr};
    int cur = 0;
    float *buf = nullptr, *g = nullptr, *z = nullptr, *v = nullptr;
    const float* mix_w = nullptr;   // general mixing matrix (device), or nullptr: the paper's pull-back + average
    float* snap = nullptr;          // [m][ld] models of the previous synchronisation (stale-average rule), or nullptr
    hipStream_t stream[2] = {nullptr, nullptr};
    bool bound = false, inited = false, launched = false;
    // options
    bool nesterov = true, fuse_pull = true, dry = false, timing = false, trace = false,
         fuse_mean = false, fuse_gemm_update = true;
    int serialize_mode = 2;   // 0: refresh on the side stream, 1: on the main stream, 2: chosen from the refresh's size
    int mean_split = 0;
    int64_t anchor_delay_us = 0;   // emulated communication latency ahead of every anchor refresh
    int gemm_variant[3] = {0, 0, 0};  // fwd, dw, da
    int splitk = 0;                   // 0: from the shape
    bool gemm_force_general = false;
    bool head_dw_guest = true;        // output-layer gradients ride in the last hidden layer's weight-gradient launch
    std::vector<int> fwd_splits;      // planned K ranges per hidden layer (fp32 forward GEMM)
    int64_t off_partial = 0;
    // schedule
    int64_t k = 0;
    bool pull_due = false, pending_update = false, anchor_due = false, anchor_inflight = false,
         first_after_anchor = false, anchor_precomputed = false, next_waited = false, pulled_in_step = false,
         wait_before_update = false;   // the in-flight refresh must land before the step's first updating launch
    hipEvent_t ev_pulled = nullptr, ev_anchor_done = nullptr;
    // model
    int model = MODEL_NONE, B = 0, gemm_dtype = 0;
    std::vector<int> dims;
    std::vector<int64_t> w_off, b_off;
    char* ws = nullptr;
    int64_t ws_bytes = 0, ws_need = 0;
    // workspace sub-buffers (byte offsets)
    std::vector<int64_t> off_act, off_dz;
    int64_t off_dlogits = 0, off_loss = 0, off_resid = 0, off_shadow = 0, off_x0 = 0;
    // residual convolutional block: channels, image size, classes; workspace sub-buffers
    int cv_C = 0, cv_H = 0, cv_W = 0, cv_classes = 0;
    bool cv_bn = false;     // convolutions without bias, each followed by batch normalisation
    float cv_eps = 1e-5f;
    int64_t off_a1 = 0, off_a2 = 0, off_dz1 = 0, off_dz2 = 0, off_pooled = 0, off_dpool = 0, off_cpartial = 0;
    int64_t off_z1 = 0, off_z2 = 0, off_bnstats = 0, off_bnsums = 0, off_bnpart = 0, off_dn = 0, off_wstat = 0;
    const float* X = nullptr;
    const void* y = nullptr;
    int64_t xs = 0, ys = 0;
    bool batch_set = false;
    // instrumentation
    std::vector<TimedLaunch> timed;
    std::vector<hipEvent_t> event_pool;
    int64_t stat_count[OLS_K_COUNT] = {0};
    double stat_ms[OLS_K_COUNT] = {0};
    std::vector<ols_trace_entry> trace_log;
};

namespace {

int hip_fail(hipError_t e, const char* what) {
    return fail(OLS_EHIP, "%s: %s", what, hipGetErrorString(e));
}

int ensure_events(ols_ctx* c) {
    if (c->ev_pulled || c->dry) return OLS_OK;
    // The two events order kernels of the two streams of ONE device and are never waited for by the host, so the
    // system-scope fence of an event is not needed (kernels release at device scope when they end).  Measured with a
    // probe (two 99 us kernels on the main stream, a small one on the side stream between them, fork and join by
    // events): the record costs 0.9 us instead of 2.7 us, the whole pattern 6.2 us instead of 10.2 us.
#ifndef OLS_EVENT_FLAGS
#define OLS_EVENT_FLAGS (hipEventDisableTiming | hipEventDisableSystemFence)
#endif
    hipError_t e = hipEventCreateWithFlags(&c->ev_pulled, OLS_EVENT_FLAGS);
    if (e != hipSuccess) return hip_fail(e, "hipEventCreate");
    e = hipEventCreateWithFlags(&c->ev_anchor_done, OLS_EVENT_FLAGS);
    if (e != hipSuccess) return hip_fail(e, "hipEventCreate");
    return OLS_OK;
}

int drain_timers(ols_ctx* c) {
    for (TimedLaunch& t : c->timed) {
        hipError_t e = hipEventSynchronize(t.stop);
        if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize");
        float ms = 0.0f;
        e = hipEventElapsedTime(&ms, t.start, t.stop);
        if (e != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
        c->stat_count[t.kind] += 1;
        c->stat_ms[t.kind] += ms;
        c->event_pool.push_back(t.start);
        c->event_pool.push_back(t.stop);
    }
    c->timed.clear();
    return OLS_OK;
}

int get_timer_event(ols_ctx* c, hipEvent_t* ev) {
    if (!c->event_pool.empty()) {
        *ev = c->event_pool.back();
        c->event_pool.pop_back();
        return OLS_OK;
    }
    hipError_t e = hipEventCreate(ev);
    if (e != hipSuccess) return hip_fail(e, "hipEventCreate");
    return OLS_OK;
}

// Enqueue one kernel: trace entry, optional event bracket on the kernel's own stream, launch.
template <class F>
int enqueue(ols_ctx* c, int kind, int stream_id, int src_buf, int dst_buf, F&& launch) {
    if (c->trace && c->trace_log.size() < 65536) {
        ols_trace_entry t;
        t.kind = kind;
        t.stream = stream_id;
        t.src_buf = src_buf;
        t.dst_buf = dst_buf;
        t.waited = c->next_waited ? 1 : 0;
        t.k = (int32_t)c->k;
        c->trace_log.push_back(t);
    }
    c->next_waited = false;
    if (c->dry) return OLS_OK;
    hipStream_t s = c->stream[stream_id];
    TimedLaunch t;
    if (c->timing) {
        if (c->timed.size() >= 8192) {
            int rc = drain_timers(c);
            if (rc) return rc;
        }
        t.kind = kind;
        int rc = get_timer_event(c, &t.start);
        if (rc) return rc;
        rc = get_timer_event(c, &t.stop);
        if (rc) return rc;
        hipError_t e = hipEventRecord(t.start, s);
        if (e != hipSuccess) return hip_fail(e, "hipEventRecord");
    }
    hipError_t e = launch(s);
    c->launched = true;
    if (e != hipSuccess) return fail(OLS_EHIP, "launch of %s failed: %s", kKernelNames[kind], hipGetErrorString(e));
    if (c->timing) {
        e = hipEventRecord(t.stop, s);
        if (e != hipSuccess) return hip_fail(e, "hipEventRecord");
        c->timed.push_back(t);
    }
    return OLS_OK;
}

// Whether the anchor refresh runs on the main stream.  Overlapping costs two cross-stream synchronisations per round
// (about 10 us on the main stream); a refresh that moves less than a MiB takes less than that, so by default such
// small problems run it in line -- the schedule of the paper pays once the refresh is longer than the hand-over.
bool serialized(const ols_ctx* c) {
    if (c->serialize_mode != 2) return c->serialize_mode == 1;
    return (4 * (int64_t)c->m + 4) * c->ld <= (1 << 20);
}

// The main stream must not pass this point before the in-flight anchor refresh has finished.
int main_waits_for_anchor(ols_ctx* c) {
    if (!c->anchor_inflight) return OLS_OK;
    c->anchor_inflight = false;
    c->next_waited = true;
    if (c->dry) return OLS_OK;
    hipError_t e = hipStreamWaitEvent(c->stream[0], c->ev_anchor_done, 0);
    if (e != hipSuccess) return hip_fail(e, "hipStreamWaitEvent");
    return OLS_OK;
}

// Issued immediately before the first launch of a local step that reads the anchor (pull-back) or overwrites
// parameters the refresh may still be reading: everything before it in the step only reads the models, so the
// refresh gets the whole tau steps of compute the paper's schedule allows (Section 2, the sentence after the
// anchor update rule).
int wait_if_update_must(ols_ctx* c) {
    if (!c->wait_before_update) return OLS_OK;
    c->wait_before_update = false;
    return main_waits_for_anchor(c);
}

int64_t align256(int64_t v) { return round_up(v, 256); }

// Static model workspace for callers that cannot allocate (ols_run_steps_static).  One copy per GPU, held until the
// process ends.  In host code the array's name is only a stand-in: the device address is looked up once per device
// with hipGetSymbolAddress and kept in scratch_ptr; everything below uses that pointer.
constexpr int64_t kStaticWorkspaceBytes = 64ll << 20;
constexpr int kStaticWorkspaceMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];
void* scratch_ptr[kStaticWorkspaceMaxDevices] = {nullptr};

int static_workspace(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(OLS_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kStaticWorkspaceMaxDevices) return fail(OLS_EINVAL, "device index %d is outside [0, %d)", dev,
                                                                  kStaticWorkspaceMaxDevices);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(OLS_EHIP, "hipGetSymbolAddress(static workspace): %s", hipGetErrorString(e));
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return OLS_OK;
}

}  // namespace

namespace ols {
// Kernels whose dynamic LDS exceeds 64 KiB need the limit raised once per (device, kernel), not per launch.
hipError_t ensure_dynamic_lds(const void* kernel, size_t bytes) {
    static std::mutex mu;
    static std::vector<std::pair<int, const void*>> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    for (const auto& d : done)
        if (d.first == dev && d.second == kernel) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) done.emplace_back(dev, kernel);
    return e;
}
}  // namespace ols

namespace {

// a model whose matrix products read a bf16 copy of the parameters, kept in the workspace by the update kernels
bool bf16_model(const ols_ctx* c) { return (c->model == MODEL_MLP || c->model == MODEL_CONV) && c->gemm_dtype == 1; }

uint16_t* shadow_ptr(ols_ctx* c) {
    return (bf16_model(c) && c->ws) ? (uint16_t*)(c->ws + c->off_shadow) : nullptr;
}

void plan_workspace(ols_ctx* c) {
    int64_t off = 0;
    auto take = [&](int64_t bytes) {
        int64_t o = off;
        off = align256(off + bytes);
        return o;
    };
    const int64_t m = c->m, B = c->B;
    c->off_act.clear();
    c->off_dz.clear();
    if (c->model == MODEL_LSQ) {
        c->off_resid = take(m * B * 4);
        c->off_loss = take(m * B * 4);
    } else if (c->model == MODEL_MLP) {
        const int L = (int)c->dims.size() - 1;
        const bool bf = c->gemm_dtype == 1;
        const int64_t es = bf ? 2 : 4;
        c->off_act.assign(L, 0);
        c->off_dz.assign(L, 0);
        for (int l = 1; l < L; ++l) {  // hidden activations a_l and deltas dz_l, [m][B][dims[l]]
            c->off_act[l] = take(m * B * c->dims[l] * es);
            c->off_dz[l] = take(m * B * c->dims[l] * es);
        }
        c->fwd_splits.assign(L, 1);
        if (!bf) {  // scratch for the split-K forward GEMMs: room for up to 8 K ranges where splitting is planned
            int64_t need_partial = 0;
            for (int l = 0; l < L - 1; ++l) {
                int variant, splits;
                gemm_f32_fwd_plan(c->m, c->B, c->dims[l + 1], c->dims[l], &variant, &splits);
                c->fwd_splits[l] = splits;
                if (splits > 1) need_partial = std::max<int64_t>(need_partial, 8 * m * B * c->dims[l + 1] * 4);
            }
            if (need_partial) c->off_partial = take(need_partial);
        }
        if (bf) {
            c->off_x0 = take(m * B * c->dims[0] * 2);
            c->off_shadow = take(m * c->ld * 2);
        }
        c->off_dlogits = take(m * B * c->dims[L] * 4);
        c->off_loss = take(m * B * 4);
    }
    if (c->model == MODEL_CONV && c->gemm_dtype == 1 && c->cv_bn) {
        // bf16 operand tensors with their zero border (batch, a1, both deltas); what the normalisations read and write is
        // fp32 without a border (both convolution outputs, a2, the gradients at the normalised outputs)
        const int64_t padded = m * B * (c->cv_H + 2) * (c->cv_W + 2) * c->cv_C;
        const int64_t act = m * B * c->cv_H * c->cv_W * c->cv_C * 4;
        c->off_x0 = take(padded * 2);
        c->off_a1 = take(padded * 2);
        c->off_dz2 = take(padded * 2);
        c->off_dz1 = take(padded * 2);
        c->off_z1 = take(act);
        c->off_z2 = take(act);
        c->off_a2 = take(act);
        c->off_dn = take(act);            // gradient at a normalised output (second block, then first)
        c->off_pooled = take(m * B * c->cv_C * 4);
        c->off_dpool = take(m * B * c->cv_C * 4);
        const int64_t splits = conv3x3_bf16_dw_splits(c->m, c->B, c->cv_H, c->cv_W, c->cv_C);
        c->off_cpartial = take(splits * m * ((int64_t)9 * c->cv_C * c->cv_C + c->cv_C) * 4);
        c->off_dlogits = take(m * B * c->cv_classes * 4);
        c->off_loss = take(m * B * 4);
        c->off_bnstats = take(2 * m * 2 * c->cv_C * 4);
        c->off_bnsums = take(m * 2 * c->cv_C * 4);
        c->off_bnpart = take(bn_partial_floats(c->m, c->B * c->cv_H * c->cv_W, c->cv_C) * 4);
        c->off_wstat = take(m * conv3x3_bf16_stat_part_floats(c->B, c->cv_H, c->cv_W, c->cv_C) * 4);
        c->off_shadow = take(m * c->ld * 2);
    } else if (c->model == MODEL_CONV && c->gemm_dtype == 1) {
        // operand tensors are bf16 and carry their zero border; a2's place holds the pooling's partial sums (or, for
        // images of fewer than 64 padded pixels, the second convolution's fp32 output with the border)
        const int64_t padded = m * B * (c->cv_H + 2) * (c->cv_W + 2) * c->cv_C;
        c->off_x0 = take(padded * 2);
        c->off_a1 = take(padded * 2);
        c->off_a2 = take(padded * 4);
        c->off_z1 = take(padded / 4);     // sign bytes of a2
        c->off_dz2 = take(padded * 2);
        c->off_dz1 = take(padded * 2);
        c->off_pooled = take(m * B * c->cv_C * 4);
        c->off_dpool = take(m * B * c->cv_C * 4);
        const int64_t splits = conv3x3_bf16_dw_splits(c->m, c->B, c->cv_H, c->cv_W, c->cv_C);
        c->off_cpartial = take(splits * m * ((int64_t)9 * c->cv_C * c->cv_C + c->cv_C) * 4);
        c->off_dlogits = take(m * B * c->cv_classes * 4);
        c->off_loss = take(m * B * 4);
        c->off_shadow = take(m * c->ld * 2);
    } else if (c->model == MODEL_CONV) {
        const int64_t act = m * B * c->cv_H * c->cv_W * c->cv_C * 4;   // one activation / delta tensor
        c->off_a1 = take(act);
        c->off_a2 = take(act);
        c->off_dz2 = take(act);
        c->off_dz1 = take(act);
        c->off_pooled = take(m * B * c->cv_C * 4);
        c->off_dpool = take(m * B * c->cv_C * 4);
        const int64_t splits = conv3x3_dw_splits(c->m, c->B, c->cv_H, c->cv_W, c->cv_C);
        c->off_cpartial = take(splits * m * ((int64_t)9 * c->cv_C * c->cv_C + c->cv_C) * 4);
        c->off_dlogits = take(m * B * c->cv_classes * 4);
        c->off_loss = take(m * B * 4);
        if (c->cv_bn) {   // the convolution outputs stay for the backward pass, with their statistics
            c->off_z1 = take(act);
            c->off_z2 = take(act);
            c->off_bnstats = take(2 * m * 2 * c->cv_C * 4);
            c->off_bnsums = take(m * 2 * c->cv_C * 4);
            c->off_bnpart = take(bn_partial_floats(c->m, c->B * c->cv_H * c->cv_W, c->cv_C) * 4);
        }
    }
    c->ws_need = off;
}

// The plain residual block with bf16 operands: the input batch is converted (and given its zero border) first, the
// kernels come from the bf16 copy of the parameters, a1 and both deltas are written as bf16; biases, shortcut, a2,
// pooling and classifier stay fp32.  The second convolution's epilogue adds the shortcut, applies the ReLU and keeps
// only the sign of a2 (all the backward pass needs of it) and partial sums for the pooling; images of fewer than 64
// padded pixels take conv + bias in fp32 followed by one streaming pass that does the same.
int conv_gradients_bf16(ols_ctx* c) {
    const float* xc = c->x[c->cur];
    const uint16_t* shadow = shadow_ptr(c);
    const int m = c->m, B = c->B, C = c->cv_C, H = c->cv_H, W = c->cv_W;
    const int64_t n_w = (int64_t)9 * C * C;
    const int64_t wa = 0, ba = n_w, wb = n_w + C, bb = 2 * n_w + C, wh = 2 * (n_w + C), bh = wh + (int64_t)C * c->cv_classes;
    const int positions = (H + 2) * (W + 2);
    const int64_t act = (int64_t)B * positions * C;   // elements of a padded tensor per worker
    uint16_t* xb = (uint16_t*)(c->ws + c->off_x0);
    uint16_t* a1 = (uint16_t*)(c->ws + c->off_a1);
    float* y2 = (float*)(c->ws + c->off_a2);          // second convolution + bias; a2 itself is never stored
    uint8_t* sign = (uint8_t*)(c->ws + c->off_z1);    // sign of a2, one byte per padded pixel and four channels
    uint16_t* dz1 = (uint16_t*)(c->ws + c->off_dz1);
    uint16_t* dz2 = (uint16_t*)(c->ws + c->off_dz2);
    float* pooled = (float*)(c->ws + c->off_pooled);
    float* dpool = (float*)(c->ws + c->off_dpool);
    ConvBArgs base = {};
    base.groups = m; base.B = B; base.H = H; base.W = W; base.C = C;
    base.s_w = c->ld; base.s_bias = c->ld;
    base.ld = c->ld; base.g = c->g; base.partial = (float*)(c->ws + c->off_cpartial);
    int rc;
    if ((rc = enqueue(c, OLS_K_CAST, 0, -1, -1, [&](hipStream_t s) {
             return launch_pad_cast_bf16(c->X, c->xs, xb, act, m, B, H, W, C, s);
         })))
        return rc;
    {   // a1 = bf16(relu(conv(X; Wa) + ba))
        ConvBArgs a = base;
        a.in = xb; a.s_in = act; a.w = shadow + wa; a.bias = xc + ba; a.out = a1; a.s_out = act; a.relu = 1;
        if ((rc = enqueue(c, OLS_K_CONV_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_conv3x3_bf16_fwd(a, s); }))) return rc;
    }
    if (positions >= 64) {
        // conv(a1; Wb) + bb with the block's tail in its epilogue: a2 = relu(. + X) is never stored -- its sign bytes and
        // partial sums of the pooling are (the partial sums take the place the fp32 output has without the fusion)
        ConvBArgs a = base;
        float* pool_part = y2;
        a.in = a1; a.s_in = act; a.w = shadow + wb; a.bias = xc + bb; a.tail = 1;
        a.xres = c->X; a.s_x = c->xs; a.sign = sign; a.s_sign = act / 4; a.pool_part = pool_part;
        if ((rc = enqueue(c, OLS_K_CONV_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_conv3x3_bf16_fwd(a, s); }))) return rc;
        if ((rc = enqueue(c, OLS_K_POOL, 0, -1, -1, [&](hipStream_t s) {
                 return launch_pool_finish(pool_part, conv3x3_bf16_pool_part_floats(B, H, W, C), pooled, (int64_t)B * C, m, B, positions, C,
                                           1.0f / (float)(H * W), s);
             })))
            return rc;
    } else {   // images too small for the fused tail's two-samples-per-wavefront bookkeeping
        {   // y = conv(a1; Wb) + bb, fp32
            ConvBArgs a = base;
            a.in = a1; a.s_in = act; a.w = shadow + wb; a.bias = xc + bb; a.out = y2; a.s_out = act; a.out_f32 = 1;
            if ((rc = enqueue(c, OLS_K_CONV_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_conv3x3_bf16_fwd(a, s); }))) return rc;
        }
        // a2 = relu(y + X), pooled = its mean over the positions, and the sign of a2 for the backward pass, in one pass
        if ((rc = enqueue(c, OLS_K_POOL, 0, -1, -1, [&](hipStream_t s) {
                 return launch_shortcut_relu_pool(y2, act, c->X, c->xs, pooled, (int64_t)B * C, sign, act / 4, m, B, H, W, C, s);
             })))
            return rc;
    }
    HeadArgs ha = {};
    ha.h = pooled;
    ha.h_stride = (int64_t)B * C;
    ha.h_bf16 = false;
    ha.x = xc;
    ha.g = c->g;
    ha.ld = c->ld;
    ha.w_off = wh;
    ha.b_off = bh;
    ha.labels = (const int32_t*)c->y;
    ha.label_stride = c->ys;
    ha.dlogits = (float*)(c->ws + c->off_dlogits);
    ha.loss_parts = (float*)(c->ws + c->off_loss);
    ha.dz = dpool;
    ha.m = m;
    ha.B = B;
    ha.H = C;
    ha.C = c->cv_classes;
    if ((rc = enqueue(c, OLS_K_HEAD_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_head_fwd(ha, s); }))) return rc;
    if ((rc = enqueue(c, OLS_K_HEAD_BWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_head_bwd(ha, s); }))) return rc;
    if ((rc = enqueue(c, OLS_K_POOL_BWD, 0, -1, -1, [&](hipStream_t s) {
             return launch_pool_bwd_bf16(dpool, (int64_t)B * C, sign, act / 4, dz2, act, m, B, positions, C, 1.0f / (float)(H * W), s);
         })))
        return rc;
    {   // delta at a1, gated by a1 > 0
        ConvBArgs a = base;
        a.in = dz2; a.s_in = act; a.w = shadow + wb; a.mask = a1; a.s_mask = act; a.out = dz1; a.s_out = act;
        if ((rc = enqueue(c, OLS_K_CONV_DX, 0, c->cur, -1, [&](hipStream_t s) { return launch_conv3x3_bf16_dx(a, s); }))) return rc;
    }
    {
        ConvBArgs a = base;
        a.in = a1; a.s_in = act; a.dout = dz2; a.s_dout = act; a.g_w_off = wb; a.g_b_off = bb;
        if ((rc = enqueue(c, OLS_K_CONV_DW, 0, -1, -1, [&](hipStream_t s) { return launch_conv3x3_bf16_dw(a, s); }))) return rc;
    }
    {
        ConvBArgs a = base;
        a.in = xb; a.s_in = act; a.dout = dz1; a.s_dout = act; a.g_w_off = wa; a.g_b_off = ba;
        if ((rc = enqueue(c, OLS_K_CONV_DW, 0, -1, -1, [&](hipStream_t s) { return launch_conv3x3_bf16_dw(a, s); }))) return rc;
    }
    return OLS_OK;
}

// Forward + backward of the residual convolutional block on the main stream; gradients go to g.
// The batch-normalised block with bf16 operands.  The convolutions read bf16 tensors in the padded layout and write
// fp32 without a border, which is what the normalisation kernels take; the normalisations write what becomes a
// convolution's operand (a1, the gradients at both convolution outputs) as bf16 straight into the padded layout.
// Statistics, the shortcut, a2, pooling and classifier are fp32 as in the fp32 block.
int conv_gradients_bn_bf16(ols_ctx* c) {
    const float* xc = c->x[c->cur];
    const uint16_t* shadow = shadow_ptr(c);
    const int m = c->m, B = c->B, C = c->cv_C, H = c->cv_H, W = c->cv_W;
    const int64_t n_w = (int64_t)9 * C * C, per_conv = n_w + 2 * C;   // kernels, scale, shift
    const int64_t wa = 0, ga = n_w, ba = n_w + C, wb = per_conv, gb = wb + n_w, bb = gb + C;
    const int64_t wh = 2 * per_conv, bh = wh + (int64_t)C * c->cv_classes;
    const int64_t padded = (int64_t)B * (H + 2) * (W + 2) * C;   // elements of a padded tensor per worker
    const int64_t act = (int64_t)B * H * W * C;                  // elements of an unpadded one
    uint16_t* xb = (uint16_t*)(c->ws + c->off_x0);
    uint16_t* a1 = (uint16_t*)(c->ws + c->off_a1);
    uint16_t* dz2 = (uint16_t*)(c->ws + c->off_dz2);
    uint16_t* dz1 = (uint16_t*)(c->ws + c->off_dz1);
    float* z1 = (float*)(c->ws + c->off_z1);
    float* z2 = (float*)(c->ws + c->off_z2);
    float* a2 = (float*)(c->ws + c->off_a2);
    float* dn = (float*)(c->ws + c->off_dn);
    float* pooled = (float*)(c->ws + c->off_pooled);
    float* dpool = (float*)(c->ws + c->off_dpool);
    ConvBArgs base = {};
    base.groups = m; base.B = B; base.H = H; base.W = W; base.C = C;
    base.s_w = c->ld; base.ld = c->ld; base.g = c->g; base.partial = (float*)(c->ws + c->off_cpartial);
    BnArgs nbase = {};
    nbase.groups = m; nbase.P = B * H * W; nbase.C = C; nbase.eps = c->cv_eps;
    nbase.s_z = act; nbase.s_out = act; nbase.s_dy = act; nbase.s_par = c->ld;
    nbase.ld = c->ld; nbase.g = c->g; nbase.H = H; nbase.W = W; nbase.s_outb = padded;
    nbase.part = (float*)(c->ws + c->off_bnpart);
    nbase.sums = (float*)(c->ws + c->off_bnsums);
    float* stats1 = (float*)(c->ws + c->off_bnstats);
    float* stats2 = stats1 + (int64_t)m * 2 * C;
    // the convolutions leave the statistics of their output per wavefront (64 padded pixels): the normalisations merge those
    float* wstat = (float*)(c->ws + c->off_wstat);
    const int waves = (int)(conv3x3_bf16_stat_part_floats(B, H, W, C) / (3 * C));
    // Images of at least 64 pixels: a2 is never stored -- the second normalisation leaves its sign (a byte per pixel and
    // four channels) and its sums per 64 pixels; both live in a2's place
    const bool tail = H * W >= 64;
    const int64_t tail_units = ((int64_t)B * H * W + 63) / 64;
    uint8_t* sign = (uint8_t*)a2;
    float* tail_part = a2 + ((int64_t)m * (act / 4) + 3) / 4;   // behind the sign bytes of all workers
    int rc;
    if ((rc = enqueue(c, OLS_K_CAST, 0, -1, -1, [&](hipStream_t s) {
             return launch_pad_cast_bf16(c->X, c->xs, xb, padded, m, B, H, W, C, s);
         })))
        return rc;
    {   // z1 = conv(X; Wa)
        ConvBArgs a = base;
        a.in = xb; a.s_in = padded; a.w = shadow + wa; a.out = z1; a.s_out = act; a.out_f32 = 1; a.out_unpadded = 1; a.stat_part = wstat;
        if ((rc = enqueue(c, OLS_K_CONV_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_conv3x3_bf16_fwd(a, s); }))) return rc;
    }
    {   // a1 = bf16(relu(bn(z1)))
        BnArgs a = nbase;
        a.z = z1; a.out_bf16 = a1; a.stats = stats1; a.gamma = xc + ga; a.beta = xc + ba; a.relu = 1; a.wave_part = wstat; a.waves = waves;
        if ((rc = enqueue(c, OLS_K_BN_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_bn_forward(a, s); }))) return rc;
    }
    {   // z2 = conv(a1; Wb)
        ConvBArgs a = base;
        a.in = a1; a.s_in = padded; a.w = shadow + wb; a.out = z2; a.s_out = act; a.out_f32 = 1; a.out_unpadded = 1; a.stat_part = wstat;
        if ((rc = enqueue(c, OLS_K_CONV_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_conv3x3_bf16_fwd(a, s); }))) return rc;
    }
    {   // a2 = relu(bn(z2) + X)
        BnArgs a = nbase;
        a.z = z2; a.out = a2; a.stats = stats2; a.gamma = xc + gb; a.beta = xc + bb; a.shortcut = c->X; a.s_sc = c->xs; a.relu = 1;
        a.wave_part = wstat; a.waves = waves;
        if (tail) { a.out = nullptr; a.sign = sign; a.s_sign = act / 4; a.pool_part = tail_part; a.positions = H * W; }
        if ((rc = enqueue(c, OLS_K_BN_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_bn_forward(a, s); }))) return rc;
    }
    if ((rc = enqueue(c, OLS_K_POOL, 0, -1, -1, [&](hipStream_t s) {
             return tail ? launch_pool_finish(tail_part, tail_units * 2 * C, pooled, (int64_t)B * C, m, B, H * W, C, 1.0f / (float)(H * W), s)
                         : launch_pool_mean(a2, act, pooled, (int64_t)B * C, m, B, H * W, C, 1.0f / (float)(H * W), s);
         })))
        return rc;
    HeadArgs ha = {};
    ha.h = pooled;
    ha.h_stride = (int64_t)B * C;
    ha.h_bf16 = false;
    ha.x = xc;
    ha.g = c->g;
    ha.ld = c->ld;
    ha.w_off = wh;
    ha.b_off = bh;
    ha.labels = (const int32_t*)c->y;
    ha.label_stride = c->ys;
    ha.dlogits = (float*)(c->ws + c->off_dlogits);
    ha.loss_parts = (float*)(c->ws + c->off_loss);
    ha.dz = dpool;
    ha.m = m;
    ha.B = B;
    ha.H = C;
    ha.C = c->cv_classes;
    if ((rc = enqueue(c, OLS_K_HEAD_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_head_fwd(ha, s); }))) return rc;
    if ((rc = enqueue(c, OLS_K_HEAD_BWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_head_bwd(ha, s); }))) return rc;
    {   // through the pooling, the second ReLU and the second normalisation: the gradient at the normalised output is
        // dpool / positions where a2 > 0 and is formed on the fly; scale / shift gradients; the gradient at z2 goes out as
        // the bf16 operand dz2
        BnArgs a = nbase;
        a.z = z2; a.dpool = dpool; a.s_dp = (int64_t)B * C; a.positions = H * W;
        if (tail) { a.sign = sign; a.s_sign = act / 4; } else { a.gate = a2; a.s_gate = act; }
        a.out_bf16 = dz2; a.stats = stats2; a.gamma = xc + gb; a.g_gamma_off = gb; a.g_beta_off = bb;
        if ((rc = enqueue(c, OLS_K_BN_BWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_bn_backward(a, s); }))) return rc;
    }
    {   // gradient at the first normalised output: transposed convolution of dz2 through Wb, gated by a1 > 0
        ConvBArgs a = base;
        a.in = dz2; a.s_in = padded; a.w = shadow + wb; a.mask = a1; a.s_mask = padded; a.out = dn; a.s_out = act;
        a.out_f32 = 1; a.out_unpadded = 1;
        if ((rc = enqueue(c, OLS_K_CONV_DX, 0, c->cur, -1, [&](hipStream_t s) { return launch_conv3x3_bf16_dx(a, s); }))) return rc;
    }
    {   // gradients of the second convolution
        ConvBArgs a = base;
        a.in = a1; a.s_in = padded; a.dout = dz2; a.s_dout = padded; a.g_w_off = wb; a.g_b_off = -1;
        if ((rc = enqueue(c, OLS_K_CONV_DW, 0, -1, -1, [&](hipStream_t s) { return launch_conv3x3_bf16_dw(a, s); }))) return rc;
    }
    {   // through the first normalisation
        BnArgs a = nbase;
        a.z = z1; a.dy = dn; a.out_bf16 = dz1; a.stats = stats1; a.gamma = xc + ga; a.g_gamma_off = ga; a.g_beta_off = ba;
        if ((rc = enqueue(c, OLS_K_BN_BWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_bn_backward(a, s); }))) return rc;
    }
    {   // gradients of the first convolution (its input is data: no delta beyond it)
        ConvBArgs a = base;
        a.in = xb; a.s_in = padded; a.dout = dz1; a.s_dout = padded; a.g_w_off = wa; a.g_b_off = -1;
        if ((rc = enqueue(c, OLS_K_CONV_DW, 0, -1, -1, [&](hipStream_t s) { return launch_conv3x3_bf16_dw(a, s); }))) return rc;
    }
    return OLS_OK;
}

// Plain block:       a1 = relu(conv(X; Wa) + ba);        a2 = relu(conv(a1; Wb) + bb + X)
// Batch-normalised:  a1 = relu(bn(conv(X; Wa); ga, ba)); a2 = relu(bn(conv(a1; Wb); gb, bb) + X)
int conv_gradients(ols_ctx* c) {
    if (c->gemm_dtype == 1) return c->cv_bn ? conv_gradients_bn_bf16(c) : conv_gradients_bf16(c);
    const float* xc = c->x[c->cur];
    const int m = c->m, B = c->B, C = c->cv_C, H = c->cv_H, W = c->cv_W;
    const bool bn = c->cv_bn;
    const int64_t n_w = (int64_t)9 * C * C;
    const int64_t per_conv = n_w + (bn ? 2 * C : C);   // kernels, then bias -- or scale and shift
    const int64_t wa = 0, wb = per_conv, wh = 2 * per_conv, bh = wh + (int64_t)C * c->cv_classes;
    const int64_t ba = wa + n_w + (bn ? C : 0), bb = wb + n_w + (bn ? C : 0);   // bias (plain) or shift (normalised)
    const int64_t ga = wa + n_w, gb = wb + n_w;                                  // scale (normalised only)
    const int64_t act = (int64_t)B * H * W * C;   // elements per worker
    float* a1 = (float*)(c->ws + c->off_a1);
    float* a2 = (float*)(c->ws + c->off_a2);
    float* dz1 = (float*)(c->ws + c->off_dz1);
    float* dz2 = (float*)(c->ws + c->off_dz2);
    float* z1 = (float*)(c->ws + c->off_z1);
    float* z2 = (float*)(c->ws + c->off_z2);
    float* pooled = (float*)(c->ws + c->off_pooled);
    float* dpool = (float*)(c->ws + c->off_dpool);
    ConvArgs base = {};
    base.groups = m; base.B = B; base.H = H; base.W = W; base.C = C;
    base.s_w = c->ld; base.s_bias = c->ld;
    base.ld = c->ld; base.g = c->g; base.partial = (float*)(c->ws + c->off_cpartial);
    BnArgs nbase = {};
    nbase.groups = m; nbase.P = B * H * W; nbase.C = C; nbase.eps = c->cv_eps;
    nbase.s_z = act; nbase.s_out = act; nbase.s_dy = act; nbase.s_par = c->ld;
    nbase.ld = c->ld; nbase.g = c->g;
    nbase.part = (float*)(c->ws + c->off_bnpart);
    nbase.sums = (float*)(c->ws + c->off_bnsums);
    float* stats1 = (float*)(c->ws + c->off_bnstats);
    float* stats2 = stats1 + (int64_t)m * 2 * C;
    // Normalised block on images of at least 64 pixels: a2 is never stored -- the second normalisation leaves its sign (a
    // byte per pixel and four channels) and its sums per 64 pixels; both live in a2's place
    const bool tail = bn && H * W >= 64;
    const int64_t tail_units = ((int64_t)B * H * W + 63) / 64;
    uint8_t* sign = (uint8_t*)a2;
    float* tail_part = a2 + ((int64_t)m * (act / 4) + 3) / 4;   // behind the sign bytes of all workers
    int rc;
    {   // first convolution
        ConvArgs a = base;
        a.in = c->X; a.s_in = c->xs; a.w = xc + wa;
        if (bn) { a.out = z1; a.relu = 0; } else { a.bias = xc + ba; a.out = a1; a.relu = 1; }
        a.s_out = act;
        if ((rc = enqueue(c, OLS_K_CONV_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_conv3x3_fwd(a, s); }))) return rc;
    }
    if (bn) {
        BnArgs a = nbase;
        a.z = z1; a.out = a1; a.stats = stats1; a.gamma = xc + ga; a.beta = xc + ba; a.relu = 1;
        if ((rc = enqueue(c, OLS_K_BN_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_bn_forward(a, s); }))) return rc;
    }
    {   // second convolution, with the shortcut
        ConvArgs a = base;
        a.in = a1; a.s_in = act; a.w = xc + wb; a.s_out = act;
        if (bn) { a.out = z2; a.relu = 0; }
        else { a.bias = xc + bb; a.residual = c->X; a.s_res = c->xs; a.out = a2; a.relu = 1; }
        if ((rc = enqueue(c, OLS_K_CONV_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_conv3x3_fwd(a, s); }))) return rc;
    }
    if (bn) {
        BnArgs a = nbase;
        a.z = z2; a.out = a2; a.stats = stats2; a.gamma = xc + gb; a.beta = xc + bb; a.shortcut = c->X; a.s_sc = c->xs; a.relu = 1;
        if (tail) { a.out = nullptr; a.sign = sign; a.s_sign = act / 4; a.pool_part = tail_part; a.positions = H * W; }
        if ((rc = enqueue(c, OLS_K_BN_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_bn_forward(a, s); }))) return rc;
    }
    if ((rc = enqueue(c, OLS_K_POOL, 0, -1, -1, [&](hipStream_t s) {
             return tail ? launch_pool_finish(tail_part, tail_units * 2 * C, pooled, (int64_t)B * C, m, B, H * W, C, 1.0f / (float)(H * W), s)
                         : launch_pool_mean(a2, act, pooled, (int64_t)B * C, m, B, H * W, C, 1.0f / (float)(H * W), s);
         })))
        return rc;
    HeadArgs ha = {};
    ha.h = pooled;
    ha.h_stride = (int64_t)B * C;
    ha.h_bf16 = false;
    ha.x = xc;
    ha.g = c->g;
    ha.ld = c->ld;
    ha.w_off = wh;
    ha.b_off = bh;
    ha.labels = (const int32_t*)c->y;
    ha.label_stride = c->ys;
    ha.dlogits = (float*)(c->ws + c->off_dlogits);
    ha.loss_parts = (float*)(c->ws + c->off_loss);
    ha.dz = dpool;   // dlogits Wh^T where pooled > 0 (pooled = 0 means every position is 0: no gradient either way)
    ha.m = m;
    ha.B = B;
    ha.H = C;
    ha.C = c->cv_classes;
    if ((rc = enqueue(c, OLS_K_HEAD_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_head_fwd(ha, s); }))) return rc;
    if ((rc = enqueue(c, OLS_K_HEAD_BWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_head_bwd(ha, s); }))) return rc;
    if (!bn) {
        if ((rc = enqueue(c, OLS_K_POOL_BWD, 0, -1, -1, [&](hipStream_t s) {
                 return launch_pool_bwd(dpool, (int64_t)B * C, a2, act, dz2, act, m, B, H * W, C, s);
             })))
            return rc;
    } else {   // through the pooling, the second ReLU and the second normalisation: the gradient at the normalised output
               // (dpool / positions where a2 > 0) is formed on the fly; scale / shift gradients; dz2 = the gradient at z2
        BnArgs a = nbase;
        a.z = z2; a.dy = dz2; a.dpool = dpool; a.s_dp = (int64_t)B * C; a.positions = H * W;
        if (tail) { a.sign = sign; a.s_sign = act / 4; } else { a.gate = a2; a.s_gate = act; }
        a.stats = stats2; a.gamma = xc + gb; a.g_gamma_off = gb; a.g_beta_off = bb;
        if ((rc = enqueue(c, OLS_K_BN_BWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_bn_backward(a, s); }))) return rc;
    }
    {   // delta at a1: transposed convolution of dz2 through Wb, gated by a1 > 0
        ConvArgs a = base;
        a.in = dz2; a.s_in = act; a.w = xc + wb; a.mask = a1; a.s_mask = act; a.out = dz1; a.s_out = act;
        if ((rc = enqueue(c, OLS_K_CONV_DX, 0, c->cur, -1, [&](hipStream_t s) { return launch_conv3x3_dx(a, s); }))) return rc;
    }
    {   // gradients of the second convolution
        ConvArgs a = base;
        a.in = a1; a.s_in = act; a.dout = dz2; a.s_dout = act; a.g_w_off = wb; a.g_b_off = bn ? -1 : bb;
        if ((rc = enqueue(c, OLS_K_CONV_DW, 0, -1, -1, [&](hipStream_t s) { return launch_conv3x3_dw(a, s); }))) return rc;
    }
    if (bn) {   // through the first normalisation
        BnArgs a = nbase;
        a.z = z1; a.dy = dz1; a.stats = stats1; a.gamma = xc + ga; a.g_gamma_off = ga; a.g_beta_off = ba;
        if ((rc = enqueue(c, OLS_K_BN_BWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_bn_backward(a, s); }))) return rc;
    }
    {   // gradients of the first convolution (its input is data: no delta beyond it)
        ConvArgs a = base;
        a.in = c->X; a.s_in = c->xs; a.dout = dz1; a.s_dout = act; a.g_w_off = wa; a.g_b_off = bn ? -1 : ba;
        if ((rc = enqueue(c, OLS_K_CONV_DW, 0, -1, -1, [&](hipStream_t s) { return launch_conv3x3_dw(a, s); }))) return rc;
    }
    return OLS_OK;
}

// Forward + backward of the attached model on the main stream.  Without `upd` the gradients go to g;
// with it (MLP only) every gradient element is consumed where it is produced: the kernels that form
// the weight, bias and output-layer gradients apply the local step (+ pull-back) themselves, reading
// x[src_buf] and writing x[dst_buf], and g is not written.
int compute_gradients(ols_ctx* c, const FusedUpdate* upd, int src_buf, int dst_buf) {
    const float* xc = c->x[c->cur];
    const int m = c->m, B = c->B;
    if (c->model == MODEL_LSQ) {
        float* resid = (float*)(c->ws + c->off_resid);
        float* loss = (float*)(c->ws + c->off_loss);
        if (upd) {   // small problem: one launch forms the gradient and applies the step
            const FusedUpdate u = *upd;
            if (int rc = wait_if_update_must(c)) return rc;
            return enqueue(c, OLS_K_LSQ_STEP, 0, src_buf, dst_buf, [&](hipStream_t s) {
                return launch_lsq_step(c->X, c->xs, (const float*)c->y, c->ys, loss, m, B, c->d, u, s);
            });
        }
        int rc = enqueue(c, OLS_K_LSQ_RESID, 0, c->cur, -1, [&](hipStream_t s) {
            return launch_lsq_resid(c->X, c->xs, (const float*)c->y, c->ys, xc, c->ld, resid, loss, m, B, c->d, s);
        });
        if (rc) return rc;
        return enqueue(c, OLS_K_LSQ_GRAD, 0, c->cur, -1,
                       [&](hipStream_t s) { return launch_lsq_grad(c->X, c->xs, resid, c->g, c->ld, m, B, c->d, s); });
    }
    if (c->model == MODEL_CONV) return conv_gradients(c);
    if (c->model != MODEL_MLP) return OLS_OK;

    const int L = (int)c->dims.size() - 1;
    const bool bf = c->gemm_dtype == 1;
    const int64_t es = bf ? 2 : 4;
    const uint16_t* shadow = shadow_ptr(c);
    auto act = [&](int l) -> const void* { return l == 0 ? (bf ? (const void*)(c->ws + c->off_x0) : (const void*)c->X)
                                                          : (const void*)(c->ws + c->off_act[l]); };
    auto act_stride = [&](int l) -> int64_t { return (l == 0 && !bf) ? c->xs : (int64_t)B * c->dims[l]; };
    (void)es;
    int rc;
    if (bf) {
        rc = enqueue(c, OLS_K_CAST, 0, -1, -1, [&](hipStream_t s) {
            return launch_cast_bf16(c->X, c->xs, (uint16_t*)(c->ws + c->off_x0), m, B, c->dims[0], s);
        });
        if (rc) return rc;
    }
    // hidden layers forward
    for (int l = 0; l < L - 1; ++l) {
        GemmArgs ga = {};
        ga.a = act(l);
        ga.sa = act_stride(l);
        ga.lda = c->dims[l];
        ga.b = bf ? (const void*)(shadow + c->w_off[l]) : (const void*)(xc + c->w_off[l]);
        ga.sb = c->ld;
        ga.ldb = c->dims[l + 1];
        ga.c = c->ws + c->off_act[l + 1];
        ga.sc = (int64_t)B * c->dims[l + 1];
        ga.ldc = c->dims[l + 1];
        ga.bias = xc + c->b_off[l];
        ga.sbias = c->ld;
        ga.force_general = c->gemm_force_general ? 1 : 0;
        ga.groups = m;
        ga.M = B;
        ga.N = c->dims[l + 1];
        ga.K = c->dims[l];
        if (!bf && c->fwd_splits[l] > 1) {  // a forced count applies only where scratch was planned
            ga.splits = c->splitk > 0 ? c->splitk : c->fwd_splits[l];
            ga.partial = (float*)(c->ws + c->off_partial);
        }
        rc = enqueue(c, OLS_K_GEMM_FWD, 0, c->cur, -1,
                     [&](hipStream_t s) { return bf ? launch_gemm_bf16_fwd(ga, s) : launch_gemm_f32_fwd(ga, s, c->gemm_variant[0]); });
        if (rc) return rc;
    }
    // output layer, loss, and its gradients
    HeadArgs ha = {};
    ha.h = act(L - 1);
    ha.h_stride = act_stride(L - 1);
    ha.h_bf16 = bf;
    ha.x = xc;
    ha.g = c->g;
    ha.ld = c->ld;
    ha.w_off = c->w_off[L - 1];
    ha.b_off = c->b_off[L - 1];
    ha.labels = (const int32_t*)c->y;
    ha.label_stride = c->ys;
    ha.dlogits = (float*)(c->ws + c->off_dlogits);
    ha.loss_parts = (float*)(c->ws + c->off_loss);
    ha.dz = L > 1 ? (void*)(c->ws + c->off_dz[L - 1]) : nullptr;
    ha.m = m;
    ha.B = B;
    ha.H = c->dims[L - 1];
    ha.C = c->dims[L];
    if (upd) ha.upd = *upd;
    rc = enqueue(c, OLS_K_HEAD_FWD, 0, c->cur, -1, [&](hipStream_t s) { return launch_head_fwd(ha, s); });
    if (rc) return rc;
    // The output layer's own gradients either ride along in the weight-gradient launch of layer L - 2 below
    // (nothing between here and there reads the output layer's parameters) or get a kernel of their own.
    const bool guest = c->head_dw_guest && L >= 2;
    if (!guest) {
        if (upd) {
            if ((rc = wait_if_update_must(c))) return rc;
        }
        rc = enqueue(c, OLS_K_HEAD_BWD, 0, src_buf, upd ? dst_buf : -1, [&](hipStream_t s) { return launch_head_bwd(ha, s); });
        if (rc) return rc;
    }
    // hidden layers backward.  The delta GEMM of a layer reads that layer's weights, so it runs before
    // the weight-gradient GEMM, which may update them in place.
    for (int l = L - 2; l >= 0; --l) {
        const void* dz = c->ws + c->off_dz[l + 1];
        const int64_t dz_stride = (int64_t)B * c->dims[l + 1];
        if (l > 0) {
            GemmArgs gd = {};
            gd.a = dz;
            gd.sa = dz_stride;
            gd.lda = c->dims[l + 1];
            gd.b = bf ? (const void*)(shadow + c->w_off[l]) : (const void*)(xc + c->w_off[l]);
            gd.sb = c->ld;
            gd.ldb = c->dims[l + 1];
            gd.mask = act(l);
            gd.smask = act_stride(l);
            gd.c = c->ws + c->off_dz[l];
            gd.sc = (int64_t)B * c->dims[l];
            gd.ldc = c->dims[l];
            gd.force_general = c->gemm_force_general ? 1 : 0;
            gd.groups = m;
            gd.M = B;
            gd.N = c->dims[l];
            gd.K = c->dims[l + 1];
            rc = enqueue(c, OLS_K_GEMM_DA, 0, c->cur, -1,
                         [&](hipStream_t s) { return bf ? launch_gemm_bf16_da(gd, s) : launch_gemm_f32_da(gd, s, c->gemm_variant[2]); });
            if (rc) return rc;
        }
        GemmArgs gw = {};
        gw.a = act(l);   // contraction over the batch: both operands are read as stored, [B][in] and [B][out]
        gw.sa = act_stride(l);
        gw.lda = c->dims[l];
        gw.b = dz;
        gw.sb = dz_stride;
        gw.ldb = c->dims[l + 1];
        gw.c = c->g + c->w_off[l];
        gw.sc = c->ld;
        gw.ldc = c->dims[l + 1];
        // the kernel also reduces the bias gradient while the delta streams through LDS
        gw.colsum = c->g + c->b_off[l];
        gw.scolsum = c->ld;
        if (upd) {
            gw.upd = *upd;
            gw.upd_w_off = c->w_off[l];
            gw.upd_b_off = c->b_off[l];
        }
        gw.guest = (guest && l == L - 2) ? &ha : nullptr;
        gw.force_general = c->gemm_force_general ? 1 : 0;
        gw.groups = m;
        gw.M = c->dims[l];
        gw.N = c->dims[l + 1];
        gw.K = B;
        if (upd) {   // first updating launch when the output layer's gradients ride in it
            if ((rc = wait_if_update_must(c))) return rc;
        }
        rc = enqueue(c, OLS_K_GEMM_DW, 0, upd ? src_buf : -1, upd ? dst_buf : -1,
                     [&](hipStream_t s) { return bf ? launch_gemm_bf16_dw(gw, s, c->gemm_variant[1]) : launch_gemm_f32_dw(gw, s, c->gemm_variant[1]); });
        if (rc) return rc;
    }
    return OLS_OK;
}

UpdateArgs update_args(ols_ctx* c, int src, int dst, bool pull) {
    UpdateArgs u = {};
    u.g = c->g;
    u.x_in = c->x[src];
    u.x_out = c->x[dst];
    u.buf = c->mu != 0.0f ? c->buf : nullptr;
    u.z = c->z;
    u.shadow = shadow_ptr(c);
    u.m = c->m;
    u.ld = c->ld;
    u.gamma = c->gamma;
    u.mu = c->mu;
    u.alpha = c->alpha;
    u.nesterov = c->nesterov;
    u.pull = pull;
    return u;
}

// Chooses source / destination replica buffers for an update that rewrites the parameters.  Where the write is in
// place while the refresh may still be reading, the main stream waits: at once, or (defer) in front of the step's first
// updating launch.
int pick_buffers(ols_ctx* c, int* src, int* dst, bool defer = false) {
    *src = c->cur;
    *dst = c->cur;
    if (c->first_after_anchor) {
        c->first_after_anchor = false;
        if (c->x[1] && !serialized(c)) {
            *dst = 1 - c->cur;  // the side stream may still be reading x[cur]
        } else if (defer) {
            c->wait_before_update = c->anchor_inflight;
        } else {
            int rc = main_waits_for_anchor(c);  // in-place write must not overtake the refresh
            if (rc) return rc;
        }
    }
    return OLS_OK;
}

// fp32 elements of one input sample of the attached model
int64_t sample_elems(ols_ctx* c) {
    if (c->model == MODEL_LSQ) return c->d;
    if (c->model == MODEL_CONV) return (int64_t)c->cv_H * c->cv_W * c->cv_C;
    return (int64_t)c->dims[0];
}

int need(ols_ctx* c) {
    if (!c) return fail(OLS_EINVAL, "null handle");
    return OLS_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
extern "C" {

const char* ols_last_error(void) { return g_err; }
const char* ols_version(void) { return "ols 0.1 (gfx950)"; }
const char* ols_kernel_name(int kind) { return (kind >= 0 && kind < OLS_K_COUNT) ? kKernelNames[kind] : "?"; }
int64_t ols_row_stride(int64_t d) { return d < 1 ? 0 : round_up(d, 64); }

ols_handle ols_create(int m, int64_t d, int tau, float alpha, float gamma, float beta) {
    if (m < 1 || m > 4096) return fail(OLS_EINVAL, "m must be in [1, 4096], got %d", m), nullptr;
    if (d < 1) return fail(OLS_EINVAL, "d must be >= 1"), nullptr;
    if (tau < 1) return fail(OLS_EINVAL, "tau must be >= 1, got %d", tau), nullptr;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return fail(OLS_EINVAL, "alpha must be in [0, 1]"), nullptr;
    if (!(gamma > 0.0f)) return fail(OLS_EINVAL, "gamma must be > 0"), nullptr;
    if (!(beta >= 0.0f && beta < 1.0f)) return fail(OLS_EINVAL, "beta (local momentum) must be in [0, 1)"), nullptr;
    ols_ctx* c = new ols_ctx();
    c->m = m;
    c->d = d;
    c->ld = ols_row_stride(d);
    c->tau = tau;
    c->alpha = alpha;
    c->gamma = gamma;
    c->mu = beta;
    return c;
}

int ols_destroy(ols_handle c) {
    if (!c) return OLS_OK;
    if (c->launched) {
        (void)hipStreamSynchronize(c->stream[0]);
        (void)hipStreamSynchronize(c->stream[1]);
    }
    for (TimedLaunch& t : c->timed) {
        (void)hipEventDestroy(t.start);
        (void)hipEventDestroy(t.stop);
    }
    for (hipEvent_t e : c->event_pool) (void)hipEventDestroy(e);
    if (c->ev_pulled) (void)hipEventDestroy(c->ev_pulled);
    if (c->ev_anchor_done) (void)hipEventDestroy(c->ev_anchor_done);
    delete c;
    return OLS_OK;
}

int ols_bind(ols_handle c, float* x, float* x_alt, float* buf, float* g, float* z, int64_t ld, void* main_stream,
             void* side_stream) {
    if (int rc = need(c)) return rc;
    if (!x || !g || !z) return fail(OLS_EINVAL, "x, g and z must be non-null");
    if (c->mu != 0.0f && !buf) return fail(OLS_EINVAL, "buf is required when the local momentum is non-zero");
    if (ld != c->ld) return fail(OLS_EINVAL, "ld must be ols_row_stride(d) = %lld, got %lld", (long long)c->ld,
                                 (long long)ld);
    const void* ptrs[] = {x, x_alt, buf, g, z};
    for (const void* p : ptrs)
        if (reinterpret_cast<uintptr_t>(p) & 255u) return fail(OLS_EINVAL, "device pointers must be 256-byte aligned");
    if (x_alt == x) return fail(OLS_EINVAL, "x_alt must differ from x");
    c->x[0] = x;
    c->x[1] = x_alt;
    c->cur = 0;
    c->buf = buf;
    c->g = g;
    c->z = z;
    c->stream[0] = (hipStream_t)main_stream;
    c->stream[1] = (hipStream_t)side_stream;
    c->bound = true;
    c->inited = false;
    return OLS_OK;
}

int ols_init_params(ols_handle c, const float* x0) {
    if (int rc = need(c)) return rc;
    if (!c->bound) return fail(OLS_ESTATE, "ols_bind must precede ols_init_params");
    if (!x0) return fail(OLS_EINVAL, "x0 is null");
    if (bf16_model(c) && !c->ws)
        return fail(OLS_ESTATE, "with bf16 GEMMs the workspace (it holds the bf16 weights) is bound before ols_init_params");
    if (int rc = ensure_events(c)) return rc;
    if (c->launched && !c->dry) {  // re-initialisation: nothing may still be reading the old state
        (void)hipStreamSynchronize(c->stream[0]);
        (void)hipStreamSynchronize(c->stream[1]);
    }
    c->cur = 0;
    if (c->model == MODEL_CONV && c->gemm_dtype == 1 && c->cv_bn && !c->dry) {
        // a1 and the two deltas are written by the normalisation kernels, image pixels only: their border is zeroed here, once
        const size_t bytes = (size_t)c->m * c->B * (c->cv_H + 2) * (c->cv_W + 2) * c->cv_C * 2;
        for (int64_t off : {c->off_a1, c->off_dz2, c->off_dz1}) {
            hipError_t e = hipMemsetAsync(c->ws + off, 0, bytes, c->stream[0]);
            if (e != hipSuccess) return hip_fail(e, "hipMemsetAsync(padded operands)");
        }
    }
    int rc = enqueue(c, OLS_K_INIT, 0, -1, 0, [&](hipStream_t s) {
        return launch_init(c->x[0], c->x[1], c->buf, c->z, shadow_ptr(c), x0, c->m, c->d, c->ld, s);
    });
    if (rc) return rc;
    if (c->snap && !c->dry) {  // the remembered models restart from the common point as well
        hipError_t e = hipMemcpyAsync(c->snap, c->x[0], (size_t)c->m * c->ld * sizeof(float), hipMemcpyDeviceToDevice,
                                      c->stream[0]);
        if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(snap)");
    }
    c->k = 0;
    c->pull_due = c->pending_update = c->anchor_due = c->anchor_inflight = c->first_after_anchor = false;
    c->anchor_precomputed = c->pulled_in_step = c->wait_before_update = false;
    c->inited = true;
    return OLS_OK;
}

int ols_set_anchor_momentum(ols_handle c, float beta_z, float* v) {
    if (int rc = need(c)) return rc;
    if (c->k != 0) return fail(OLS_ESTATE, "anchor momentum must be set before the first local step");
    if (!(beta_z >= 0.0f && beta_z < 1.0f)) return fail(OLS_EINVAL, "beta_z must be in [0, 1)");
    if (beta_z != 0.0f && !v) return fail(OLS_EINVAL, "v is required when beta_z is non-zero");
    if (beta_z != 0.0f && c->mix_w) return fail(OLS_EINVAL, "anchor momentum cannot be combined with general mixing");
    if (beta_z != 0.0f && c->snap) return fail(OLS_EINVAL, "anchor momentum cannot be combined with the stale-average rule");
    if (reinterpret_cast<uintptr_t>(v) & 255u) return fail(OLS_EINVAL, "v must be 256-byte aligned");
    c->beta_z = beta_z;
    c->v = beta_z != 0.0f ? v : nullptr;
    return OLS_OK;
}

int ols_set_mixing(ols_handle c, const float* w_dev) {
    if (int rc = need(c)) return rc;
    if (c->pull_due || c->anchor_due || c->pending_update)
        return fail(OLS_ESTATE, "the mixing matrix cannot change in the middle of a synchronisation");
    if (w_dev && c->m > kMixMaxWorkers) return fail(OLS_EINVAL, "general mixing supports m <= %d", kMixMaxWorkers);
    if (w_dev && c->beta_z != 0.0f) return fail(OLS_EINVAL, "general mixing cannot be combined with anchor momentum");
    if (w_dev && c->snap) return fail(OLS_EINVAL, "general mixing cannot be combined with the stale-average rule");
    if (reinterpret_cast<uintptr_t>(w_dev) & 3u) return fail(OLS_EINVAL, "w_dev must be 4-byte aligned");
    c->mix_w = w_dev;
    return OLS_OK;
}

int ols_set_stale_average(ols_handle c, float* snap) {
    if (int rc = need(c)) return rc;
    if (!c->bound || !c->inited) return fail(OLS_ESTATE, "ols_bind and ols_init_params must precede ols_set_stale_average");
    if (c->k != 0) return fail(OLS_ESTATE, "the synchronisation rule must be chosen before the first local step");
    if (snap && (c->mix_w || c->beta_z != 0.0f))
        return fail(OLS_EINVAL, "the stale-average rule cannot be combined with general mixing or anchor momentum");
    if (reinterpret_cast<uintptr_t>(snap) & 255u) return fail(OLS_EINVAL, "snap must be 256-byte aligned");
    if (snap && (snap == c->x[0] || snap == c->x[1])) return fail(OLS_EINVAL, "snap must not alias the replicas");
    if (snap && !c->dry) {  // every model starts from the common point, and so do the remembered ones
        hipError_t e = hipMemcpyAsync(snap, c->x[c->cur], (size_t)c->m * c->ld * sizeof(float), hipMemcpyDeviceToDevice,
                                      c->stream[0]);
        if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(snap)");
    }
    c->snap = snap;
    return OLS_OK;
}

int ols_set_lr(ols_handle c, float gamma) {
    if (int rc = need(c)) return rc;
    if (!(gamma > 0.0f)) return fail(OLS_EINVAL, "gamma must be > 0");
    if (c->pending_update) return fail(OLS_ESTATE, "a deferred local step is pending; call ols_sync_pull first");
    c->gamma = gamma;
    return OLS_OK;
}

int ols_attach_lsq(ols_handle c, int batch) {
    if (int rc = need(c)) return rc;
    if (batch < 1 || batch > 8192) return fail(OLS_EINVAL, "batch must be in [1, 8192]");
    if (c->k != 0) return fail(OLS_ESTATE, "models are attached before the first local step");
    c->model = MODEL_LSQ;
    c->B = batch;
    c->ws = nullptr;
    c->batch_set = false;
    plan_workspace(c);
    return OLS_OK;
}

int ols_attach_mlp(ols_handle c, int n_layers, const int* dims, int batch, int gemm_dtype) {
    if (int rc = need(c)) return rc;
    if (c->k != 0) return fail(OLS_ESTATE, "models are attached before the first local step");
    if (n_layers < 1 || n_layers > 64 || !dims) return fail(OLS_EINVAL, "n_layers must be in [1, 64]");
    if (gemm_dtype != 0 && gemm_dtype != 1) return fail(OLS_EINVAL, "gemm_dtype must be 0 (fp32) or 1 (bf16)");
    if (gemm_dtype == 1 && c->inited)
        return fail(OLS_ESTATE, "a bf16 model is attached (and its workspace bound) before ols_init_params");
    if (batch < 4 || batch % 4 != 0 || batch > 65536) return fail(OLS_EINVAL, "batch must be a multiple of 4 in [4, 65536]");
    int64_t total = 0;
    for (int l = 0; l <= n_layers; ++l) {
        if (dims[l] < 1) return fail(OLS_EINVAL, "dims[%d] must be >= 1", l);
        if (l < n_layers && dims[l] % 4 != 0) return fail(OLS_EINVAL, "dims[%d] = %d must be a multiple of 4", l, dims[l]);
        if (l < n_layers && gemm_dtype == 1 && dims[l] % 8 != 0)
            return fail(OLS_EINVAL, "bf16 GEMMs need dims[%d] = %d to be a multiple of 8", l, dims[l]);
    }
    if (gemm_dtype == 1 && batch % 8 != 0) return fail(OLS_EINVAL, "bf16 GEMMs need the batch to be a multiple of 8");
    if (dims[n_layers] > 32) return fail(OLS_EINVAL, "the class count must be <= 32, got %d", dims[n_layers]);
    std::vector<int64_t> w_off(n_layers), b_off(n_layers);
    for (int l = 0; l < n_layers; ++l) {
        w_off[l] = total;
        total += (int64_t)dims[l] * dims[l + 1];
        b_off[l] = total;
        total += dims[l + 1];
    }
    if (total != c->d) return fail(OLS_EINVAL, "layer sizes give %lld parameters but d = %lld", (long long)total,
                                   (long long)c->d);
    c->model = MODEL_MLP;
    c->B = batch;
    c->gemm_dtype = gemm_dtype;
    c->dims.assign(dims, dims + n_layers + 1);
    c->w_off = w_off;
    c->b_off = b_off;
    c->ws = nullptr;
    c->batch_set = false;
    plan_workspace(c);
    return OLS_OK;
}

namespace {
int attach_convblock(ols_ctx* c, int channels, int height, int width, int classes, int batch, bool bn, float eps, bool bf16) {
    if (int rc = need(c)) return rc;
    if (c->k != 0) return fail(OLS_ESTATE, "models are attached before the first local step");
    if (bf16) {
        if (c->inited) return fail(OLS_ESTATE, "a bf16 model is attached before ols_init_params (its bf16 weights are written there)");
        if (channels % 64 != 0) return fail(OLS_EINVAL, "bf16 convolutions need the channels to be a multiple of 64, got %d", channels);
        if (width > kConvBf16MaxWidth) return fail(OLS_EINVAL, "bf16 convolutions take widths up to %d, got %d", kConvBf16MaxWidth, width);
    }
    if (channels < 16 || channels % 16 != 0 || channels > 256) return fail(OLS_EINVAL, "channels must be a multiple of 16 in [16, 256], got %d", channels);
    if (height < 1 || width < 1 || height > 4096 || width > 4096) return fail(OLS_EINVAL, "height and width must be in [1, 4096]");
    if (classes < 1 || classes > 32) return fail(OLS_EINVAL, "the class count must be in [1, 32], got %d", classes);
    if (batch < 1 || batch > 65536) return fail(OLS_EINVAL, "batch must be in [1, 65536]");
    if (bn && !(eps > 0.0f && eps <= 1.0f)) return fail(OLS_EINVAL, "eps must be in (0, 1], got %g", (double)eps);
    const int64_t elems = (int64_t)batch * (height + (bf16 ? 2 : 0)) * (width + (bf16 ? 2 : 0)) * channels;
    if (elems >= ((int64_t)1 << 31) - ((int64_t)channels << 16))
        return fail(OLS_EINVAL, "batch * height * width * channels = %lld is too large for one worker's activation tensor", (long long)elems);
    const int64_t total =
        2 * ((int64_t)9 * channels * channels + (bn ? 2 : 1) * (int64_t)channels) + (int64_t)channels * classes + classes;
    if (total != c->d) return fail(OLS_EINVAL, "the block has %lld parameters but d = %lld", (long long)total, (long long)c->d);
    c->model = MODEL_CONV;
    c->B = batch;
    c->gemm_dtype = bf16 ? 1 : 0;
    c->cv_C = channels;
    c->cv_H = height;
    c->cv_W = width;
    c->cv_classes = classes;
    c->cv_bn = bn;
    c->cv_eps = eps;
    c->ws = nullptr;
    c->batch_set = false;
    plan_workspace(c);
    return OLS_OK;
}
}  // namespace

int ols_attach_convblock(ols_handle c, int channels, int height, int width, int classes, int batch) {
    return attach_convblock(c, channels, height, width, classes, batch, false, 0.0f, false);
}

int ols_attach_convblock_bf16(ols_handle c, int channels, int height, int width, int classes, int batch) {
    return attach_convblock(c, channels, height, width, classes, batch, false, 0.0f, true);
}

int ols_attach_convblock_bn(ols_handle c, int channels, int height, int width, int classes, int batch, float eps) {
    return attach_convblock(c, channels, height, width, classes, batch, true, eps, false);
}

int ols_attach_convblock_bn_bf16(ols_handle c, int channels, int height, int width, int classes, int batch, float eps) {
    return attach_convblock(c, channels, height, width, classes, batch, true, eps, true);
}

int64_t ols_workspace_bytes(ols_handle c) { return c ? c->ws_need : 0; }

int ols_bind_workspace(ols_handle c, void* ws, int64_t bytes) {
    if (int rc = need(c)) return rc;
    if (c->model == MODEL_NONE) return fail(OLS_ESTATE, "no model attached");
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return fail(OLS_EINVAL, "workspace must be non-null and 256-byte aligned");
    if (bytes < c->ws_need) return fail(OLS_ENOMEM, "workspace has %lld bytes, %lld needed", (long long)bytes,
                                        (long long)c->ws_need);
    if (c->inited && bf16_model(c))
        return fail(OLS_ESTATE, "with bf16 GEMMs the workspace (it holds the bf16 weights) is bound before ols_init_params");
    c->ws = (char*)ws;
    c->ws_bytes = bytes;
    return OLS_OK;
}

int ols_set_batch(ols_handle c, const float* X, int64_t x_worker_stride, const void* y, int64_t y_worker_stride) {
    if (int rc = need(c)) return rc;
    if (c->model == MODEL_NONE) return fail(OLS_ESTATE, "no model attached");
    if (!X || !y) return fail(OLS_EINVAL, "X and y must be non-null");
    if ((reinterpret_cast<uintptr_t>(X) & 15u) || (x_worker_stride % 4) != 0)
        return fail(OLS_EINVAL, "X must be 16-byte aligned with a worker stride that is a multiple of 4 elements");
    const int64_t row = sample_elems(c);
    if (x_worker_stride < (int64_t)c->B * row && c->m > 1 && x_worker_stride != 0)
        return fail(OLS_EINVAL, "x_worker_stride %lld is smaller than one batch (%lld elements)",
                    (long long)x_worker_stride, (long long)(c->B * row));
    if (y_worker_stride < c->B && c->m > 1 && y_worker_stride != 0)
        return fail(OLS_EINVAL, "y_worker_stride is smaller than one batch");
    c->X = X;
    c->xs = x_worker_stride;
    c->y = y;
    c->ys = y_worker_stride;
    c->batch_set = true;
    return OLS_OK;
}

int ols_set_gradient(ols_handle c, float* g) {
    if (int rc = need(c)) return rc;
    if (c->model != MODEL_NONE) return fail(OLS_ESTATE, "the attached model writes the gradients itself");
    if (!g || (reinterpret_cast<uintptr_t>(g) & 255u)) return fail(OLS_EINVAL, "g must be non-null and 256-byte aligned");
    if (c->pending_update) return fail(OLS_ESTATE, "a deferred local step still needs the current gradients");
    c->g = g;
    return OLS_OK;
}

int ols_local_step(ols_handle c) {
    if (int rc = need(c)) return rc;
    if (!c->bound || !c->inited) return fail(OLS_ESTATE, "ols_bind and ols_init_params must precede ols_local_step");
    if (c->pull_due) return fail(OLS_ESTATE, "k = %lld is a multiple of tau: ols_sync_pull is due", (long long)c->k);
    if (c->anchor_due) return fail(OLS_ESTATE, "ols_anchor_update_async is due after the pull");
    if (c->model != MODEL_NONE) {
        if (!c->ws) return fail(OLS_ESTATE, "the attached model needs ols_bind_workspace");
        if (!c->batch_set) return fail(OLS_ESTATE, "the attached model needs ols_set_batch");
    }
    const bool boundary = (c->k + 1) % c->tau == 0;
    // whether the synchronisation is the paper's pull-back + anchor average
    const bool paper_sync = c->mix_w == nullptr && c->snap == nullptr;
    const bool grad_kernels_update = c->model == MODEL_MLP || (c->model == MODEL_LSQ && lsq_step_fits(c->B, c->d));
    if (grad_kernels_update && c->fuse_gemm_update && !(boundary && c->fuse_mean && paper_sync)) {
        // the gradient kernels apply the update themselves; on a boundary step the pull-back as well, so the
        // anchor of the previous round must have landed before the first of them that updates starts -- not before
        // the forward pass, the output layer's forward kernel and the delta GEMMs, which only read the models
        int src, dst;
        if (int rc = pick_buffers(c, &src, &dst, true)) return rc;
        if (boundary && paper_sync && c->anchor_inflight) c->wait_before_update = true;
        FusedUpdate u = {};
        u.x_in = c->x[src];
        u.x_out = c->x[dst];
        u.buf = c->mu != 0.0f ? c->buf : nullptr;
        u.z = c->z;
        u.shadow = shadow_ptr(c);
        u.ld = c->ld;
        u.gamma = c->gamma;
        u.mu = c->mu;
        u.alpha = c->alpha;
        u.nesterov = c->nesterov ? 1 : 0;
        u.pull = (boundary && paper_sync) ? 1 : 0;
        u.enabled = 1;
        if (int rc = compute_gradients(c, &u, src, dst)) return rc;
        if (int rc = wait_if_update_must(c)) return rc;   // (a model without an updating launch: nothing to defer to)
        c->cur = dst;
        c->k += 1;
        if (boundary) {
            c->pull_due = true;
            c->pulled_in_step = paper_sync;
        }
        return OLS_OK;
    }
    if (int rc = compute_gradients(c, nullptr, c->cur, -1)) return rc;
    c->k += 1;
    if (boundary && c->fuse_pull && paper_sync) {
        c->pending_update = true;  // applied together with the pull-back in one pass
        c->pull_due = true;
        return OLS_OK;
    }
    int src, dst;
    if (int rc = pick_buffers(c, &src, &dst)) return rc;
    UpdateArgs u = update_args(c, src, dst, false);
    int rc = enqueue(c, OLS_K_STEP, 0, src, dst, [&](hipStream_t s) { return launch_step(u, s); });
    if (rc) return rc;
    c->cur = dst;
    if (boundary) c->pull_due = true;
    return OLS_OK;
}

int ols_sync_pull(ols_handle c) {
    if (int rc = need(c)) return rc;
    if (!c->pull_due) return fail(OLS_ESTATE, "no pull is due at k = %lld (tau = %d)", (long long)c->k, c->tau);
    if (c->pulled_in_step) {  // the boundary step's gradient kernels already applied step + pull-back
        c->pulled_in_step = false;
        if (!c->dry) {
            hipError_t e = hipEventRecord(c->ev_pulled, c->stream[0]);
            if (e != hipSuccess) return hip_fail(e, "hipEventRecord");
        }
        c->pull_due = false;
        c->anchor_due = true;
        return OLS_OK;
    }
    // the anchor about to be read is the one the previous round's refresh produces
    if (int rc = main_waits_for_anchor(c)) return rc;
    if (c->mix_w) {  // X <- X W over [x^(1..m), z] in one pass; the new anchor is row m of the product
        c->first_after_anchor = false;
        MixArgs a = {};
        a.x = c->x[c->cur];
        a.z = c->z;
        a.shadow = shadow_ptr(c);
        a.w = c->mix_w;
        a.m = c->m;
        a.ld = c->ld;
        int rc = enqueue(c, OLS_K_MIX, 0, c->cur, c->cur, [&](hipStream_t s) { return launch_mix(a, s); });
        if (rc) return rc;
        c->pull_due = false;
        c->anchor_due = true;
        c->anchor_precomputed = true;
        return OLS_OK;
    }
    if (c->snap) {  // x <- z + (x - snap), snap <- x; the average of the new models follows on the side stream
        c->first_after_anchor = false;
        int rc = enqueue(c, OLS_K_STALE_SYNC, 0, c->cur, c->cur, [&](hipStream_t s) {
            return launch_stale_sync(c->x[c->cur], c->snap, c->z, shadow_ptr(c), c->m, c->ld, s);
        });
        if (rc) return rc;
        if (!c->dry) {
            hipError_t e = hipEventRecord(c->ev_pulled, c->stream[0]);
            if (e != hipSuccess) return hip_fail(e, "hipEventRecord");
        }
        c->pull_due = false;
        c->anchor_due = true;
        return OLS_OK;
    }
    int src = c->cur, dst = c->cur;
    if (c->first_after_anchor) {  // only when tau == 1: nothing was written since the refresh, which has now finished
        c->first_after_anchor = false;
    }
    int rc;
    if (c->fuse_mean && !shadow_ptr(c)) {
        StepPullMeanArgs a = {};
        a.u = update_args(c, src, dst, true);
        a.z_out = c->z;
        a.v = c->v;
        a.beta_z = c->beta_z;
        a.with_step = c->pending_update;
        rc = enqueue(c, OLS_K_STEP_PULL_MEAN, 0, src, dst, [&](hipStream_t s) { return launch_step_pull_mean(a, s); });
        c->anchor_precomputed = true;
    } else if (c->pending_update) {
        UpdateArgs u = update_args(c, src, dst, true);
        rc = enqueue(c, OLS_K_STEP_PULL, 0, src, dst, [&](hipStream_t s) { return launch_step(u, s); });
    } else {
        rc = enqueue(c, OLS_K_PULL, 0, src, dst, [&](hipStream_t s) {
            return launch_pull(c->x[c->cur], c->z, shadow_ptr(c), c->m, c->ld, c->alpha, s);
        });
    }
    if (rc) return rc;
    if (!c->dry) {
        hipError_t e = hipEventRecord(c->ev_pulled, c->stream[0]);
        if (e != hipSuccess) return hip_fail(e, "hipEventRecord");
    }
    c->pending_update = false;
    c->pull_due = false;
    c->anchor_due = true;
    return OLS_OK;
}

int ols_anchor_update_async(ols_handle c) {
    if (int rc = need(c)) return rc;
    if (!c->anchor_due) return fail(OLS_ESTATE, "ols_anchor_update_async is legal only right after ols_sync_pull");
    c->anchor_due = false;
    if (c->anchor_precomputed) {  // the pull pass already produced the new anchor on the main stream
        c->anchor_precomputed = false;
        return OLS_OK;
    }
    const int sid = (serialized(c) || c->stream[1] == c->stream[0]) ? 0 : 1;
    if (sid == 1 && !c->dry) {
        hipError_t e = hipStreamWaitEvent(c->stream[1], c->ev_pulled, 0);
        if (e != hipSuccess) return hip_fail(e, "hipStreamWaitEvent");
    }
    if (sid == 1) c->next_waited = true;
    if (c->anchor_delay_us > 0) {
        const int64_t us = c->anchor_delay_us;
        int rc = enqueue(c, OLS_K_DELAY, sid, -1, -1, [&](hipStream_t s) { return launch_delay(us, s); });
        if (rc) return rc;
    }
    MeanArgs a = {};
    a.x = c->x[c->cur];
    a.z = c->z;
    a.v = c->v;
    a.m = c->m;
    a.ld = c->ld;
    a.beta_z = c->beta_z;
    a.split = c->mean_split;
    int rc = enqueue(c, OLS_K_MEAN, sid, c->cur, -1, [&](hipStream_t s) { return launch_mean(a, s); });
    if (rc) return rc;
    if (sid == 1) {
        if (!c->dry) {
            hipError_t e = hipEventRecord(c->ev_anchor_done, c->stream[1]);
            if (e != hipSuccess) return hip_fail(e, "hipEventRecord");
        }
        c->anchor_inflight = true;
        c->first_after_anchor = true;
    }
    return OLS_OK;
}

int ols_run_steps(ols_handle c, int64_t steps, const float* X, const void* y, int nb) {
    if (int rc = need(c)) return rc;
    if (c->model == MODEL_NONE) return fail(OLS_ESTATE, "ols_run_steps needs an attached model");
    if (steps < 0 || nb < 1 || !X || !y) return fail(OLS_EINVAL, "steps >= 0, nb >= 1 and non-null data are required");
    if (c->pull_due || c->anchor_due) return fail(OLS_ESTATE, "a pull or an anchor refresh is due");
    const int64_t row = sample_elems(c);
    const int64_t x_batch = (int64_t)c->B * row, y_batch = c->B;   // elements per batch
    const size_t y_elem = 4;                                          // int32 labels and fp32 targets alike
    for (int64_t it = 0; it < steps; ++it) {
        const int64_t b = c->k % nb;
        int rc = ols_set_batch(c, X + b * x_batch, (int64_t)nb * x_batch, (const char*)y + (size_t)(b * y_batch) * y_elem,
                               (int64_t)nb * y_batch);
        if (rc) return rc;
        rc = ols_local_step(c);
        if (rc) return rc;
        if (c->pull_due) {
            rc = ols_sync_pull(c);
            if (rc) return rc;
            rc = ols_anchor_update_async(c);
            if (rc) return rc;
        }
    }
    return OLS_OK;
}

int64_t ols_static_workspace_bytes(void) { return kStaticWorkspaceBytes; }

int ols_run_steps_static(ols_handle c, int64_t steps, const float* X, const void* y, int nb) {
    if (int rc = need(c)) return rc;
    if (c->model == MODEL_NONE) return fail(OLS_ESTATE, "ols_run_steps_static needs an attached model");
    if (bf16_model(c))
        return fail(OLS_EINVAL, "the bf16 model keeps its bf16 weights in the workspace, which must then outlive the call: "
                                "bind a caller-owned workspace and use ols_run_steps");
    if (c->timing) return fail(OLS_ESTATE, "per-kernel timing creates events; switch OLS_OPT_KERNEL_TIMING off first");
    if (c->ws_need > kStaticWorkspaceBytes)
        return fail(OLS_ENOMEM, "the attached model needs %lld bytes of workspace, the static workspace holds %lld",
                    (long long)c->ws_need, (long long)kStaticWorkspaceBytes);
    if (!c->dry) {
        void* p = nullptr;
        if (int rc = static_workspace(&p)) return rc;
        c->ws = (char*)p;
        c->ws_bytes = kStaticWorkspaceBytes;
    } else {
        c->ws = reinterpret_cast<char*>(uintptr_t(256));  // never dereferenced: a dry run launches nothing
        c->ws_bytes = kStaticWorkspaceBytes;
    }
    return ols_run_steps(c, steps, X, y, nb);
}

int ols_sync(ols_handle c) {
    if (int rc = need(c)) return rc;
    if (!c->bound || c->dry) return OLS_OK;
    hipError_t e = hipStreamSynchronize(c->stream[0]);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize(main)");
    e = hipStreamSynchronize(c->stream[1]);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize(side)");
    // everything has finished: no cross-stream wait is needed any more
    c->anchor_inflight = false;
    c->first_after_anchor = false;
    return OLS_OK;
}

int ols_get_params(ols_handle c, int which, float* dst, int dst_is_device) {
    if (int rc = need(c)) return rc;
    if (!c->bound || !c->inited) return fail(OLS_ESTATE, "nothing to read before ols_init_params");
    if (c->pending_update) return fail(OLS_ESTATE, "a deferred local step is pending; call ols_sync_pull first");
    if (!dst) return fail(OLS_EINVAL, "dst is null");
    if (which < -2 || which >= c->m) return fail(OLS_EINVAL, "which must be in [-2, m)");
    if (c->dry) return OLS_OK;
    if (int rc = ols_sync(c)) return rc;
    if (which == -2) {
        if (!dst_is_device) return fail(OLS_EINVAL, "the replica mean is computed into a device destination");
        if (reinterpret_cast<uintptr_t>(dst) & 255u) return fail(OLS_EINVAL, "dst must be 256-byte aligned");
        MeanArgs a = {};
        a.x = c->x[c->cur];
        a.z = dst;  // ols_row_stride(d) floats
        a.m = c->m;
        a.ld = c->ld;
        a.split = c->mean_split;
        hipError_t e = launch_mean(a, c->stream[0]);
        if (e != hipSuccess) return hip_fail(e, "replica mean");
        e = hipStreamSynchronize(c->stream[0]);
        if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
        return OLS_OK;
    }
    const float* src = which == -1 ? c->z : c->x[c->cur] + (int64_t)which * c->ld;
    hipError_t e = hipMemcpy(dst, src, (size_t)c->d * sizeof(float),
                             dst_is_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpy");
    return OLS_OK;
}

int ols_get_loss(ols_handle c, float* per_worker_host) {
    if (int rc = need(c)) return rc;
    if (c->model == MODEL_NONE || !c->ws) return fail(OLS_ESTATE, "no model with a workspace is attached");
    if (!per_worker_host) return fail(OLS_EINVAL, "null destination");
    if (c->dry) return OLS_OK;
    hipError_t e = hipStreamSynchronize(c->stream[0]);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    std::vector<float> parts((size_t)c->m * c->B);
    e = hipMemcpy(parts.data(), c->ws + c->off_loss, parts.size() * sizeof(float), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpy");
    for (int i = 0; i < c->m; ++i) {  // fixed-order mean of the per-sample losses the kernels produced
        double acc = 0.0;
        for (int s = 0; s < c->B; ++s) acc += parts[(size_t)i * c->B + s];
        per_worker_host[i] = (float)(acc / c->B);
    }
    return OLS_OK;
}

int ols_set_option(ols_handle c, int key, int64_t value) {
    if (int rc = need(c)) return rc;
    switch (key) {
        case OLS_OPT_NESTEROV: c->nesterov = value != 0; break;
        case OLS_OPT_FUSE_PULL:
            if (c->pending_update) return fail(OLS_ESTATE, "cannot change fusion while a deferred step is pending");
            c->fuse_pull = value != 0;
            break;
        case OLS_OPT_SERIALIZE:
            if (value < 0 || value > 2) return fail(OLS_EINVAL, "OLS_OPT_SERIALIZE takes 0 (overlap), 1 (serialise) or 2 (from the size)");
            c->serialize_mode = (int)value;
            break;
        case OLS_OPT_DRY_RUN:
            if (c->launched) return fail(OLS_ESTATE, "dry-run mode must be chosen before anything is launched");
            c->dry = value != 0;
            break;
        case OLS_OPT_KERNEL_TIMING:
            if (!value && c->timing) {
                if (int rc = drain_timers(c)) return rc;
            }
            c->timing = value != 0;
            break;
        case OLS_OPT_TRACE:
            c->trace = value != 0;
            if (value) c->trace_log.clear();
            break;
        case OLS_OPT_MEAN_SPLIT:
            if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8 && value != 16)
                return fail(OLS_EINVAL, "mean split must be 0, 1, 2, 4, 8 or 16");
            c->mean_split = (int)value;
            break;
        case OLS_OPT_TUNING:   // unstable: 256 * which + variant
            if (value < 0 || value / 256 > 2 || value % 256 > 31) return fail(OLS_EINVAL, "tuning value out of range");
            c->gemm_variant[value / 256] = (int)(value % 256);
            break;
        case OLS_OPT_FUSE_GEMM_UPDATE:
            if (c->pull_due || c->anchor_due) return fail(OLS_ESTATE, "cannot change fusion in the middle of a synchronisation");
            c->fuse_gemm_update = value != 0;
            break;
        case OLS_OPT_GEMM_SPLITK:
            if (value < 0 || value > 8) return fail(OLS_EINVAL, "split-K count must be in [0, 8]");
            c->splitk = (int)value;
            break;
        case OLS_OPT_GEMM_FORCE_GENERAL: c->gemm_force_general = value != 0; break;
        case OLS_OPT_HEAD_DW_GUEST: c->head_dw_guest = value != 0; break;
        case OLS_OPT_ANCHOR_DELAY_US:
            if (value < 0 || value > 1000000) return fail(OLS_EINVAL, "the anchor delay must be 0 .. 1000000 microseconds");
            c->anchor_delay_us = value;
            break;
        case OLS_OPT_FUSE_MEAN:
            if (c->pull_due || c->anchor_due) return fail(OLS_ESTATE, "cannot change fusion in the middle of a synchronisation");
            c->fuse_mean = value != 0;
            break;
        default: return fail(OLS_EINVAL, "unknown option %d", key);
    }
    return OLS_OK;
}

int64_t ols_iteration(ols_handle c) { return c ? c->k : -1; }

int ols_kernel_stats(ols_handle c, int kind, int64_t* launches, double* total_ms) {
    if (int rc = need(c)) return rc;
    if (kind < 0 || kind >= OLS_K_COUNT) return fail(OLS_EINVAL, "bad kernel kind");
    if (int rc = drain_timers(c)) return rc;
    if (launches) *launches = c->stat_count[kind];
    if (total_ms) *total_ms = c->stat_ms[kind];
    return OLS_OK;
}

int64_t ols_trace_count(ols_handle c) { return c ? (int64_t)c->trace_log.size() : 0; }

int ols_trace_get(ols_handle c, int64_t idx, ols_trace_entry* out) {
    if (int rc = need(c)) return rc;
    if (!out || idx < 0 || idx >= (int64_t)c->trace_log.size()) return fail(OLS_EINVAL, "trace index out of range");
    *out = c->trace_log[idx];
    return OLS_OK;
}

}  // extern "C"
