#!/usr/bin/env python3
"""Benchmark of the Overlap Local-SGD hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--side-configs 1,2,3,5]

A step is one iteration of the whole hot path for all m workers (the gradient of the iteration -- per-worker
forward/backward of the attached model, or the caller's gradient tensor on the update-only stream --, the local
momentum step, and on every tau-th step the pull-back and the anchor refresh) on synthetic inputs already resident in
HBM.  The headline workload is configuration 4, the update-only stream (m = 16 replicas of a ResNet-18-sized vector):
it is the one the metric's "fused update / anchor-average HBM GB/s" is defined on.  Prints ONE JSON line:
worker-iterations/s over exactly K timed steps after exactly W warm-up steps, the roofline of the dominant kernel
from HIP-event timing on the kernel's own stream, the CPU oracle timed on a bounded sample of the same workload as a
reported baseline, and under "configs" one compact record per other configuration (1, 2, 3, 5 and the convolutional
workloads 6, 7 and 8; its own run length, stated in the record): ms per step overlapped and serialised, the dominant
kernel and its roofline fraction, the oracle's rate.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=4, help="headline workload number (BASELINE configs are 1-based)")
    ap.add_argument("--side-configs", type=str, default=None,
                    help="comma-separated configurations measured after the headline and reported under \"configs\" "
                         "(default: 1,2,3,5,6,7,8,9 when the headline is configuration 4 with default options, else none)")
    ap.add_argument("--side-cpu-seconds", type=float, default=3.0,
                    help="target CPU time of the oracle baseline of each side configuration (at least one round)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle baseline; 0 skips it")
    ap.add_argument("--serialize", type=int, default=2,
                    help="0: anchor refresh on the side stream (overlapped), 1: on the main stream, 2 (default, the "
                         "library's own): overlapped unless the refresh moves at most 1 MiB")
    ap.add_argument("--fuse-mean", type=int, default=None,
                    help="1: step + pull-back + anchor refresh in one pass.  Default: 1 on the update-only stream "
                         "(configuration 4 asks for the fused step + pull-back + mean, and an HBM-bound stream gains "
                         "nothing from overlapping a second HBM-bound kernel), 0 elsewhere (side-stream refresh)")
    ap.add_argument("--mixing", choices=["none", "paper", "averaging"], default="none",
                    help="general mixing X <- X W at the synchronisation points: the paper's W or periodic averaging "
                         "applied by the one-pass mixing kernel instead of pull-back + anchor average")
    ap.add_argument("--anchor-delay-us", type=int, default=0,
                    help="emulated communication latency ahead of every anchor refresh (OLS_OPT_ANCHOR_DELAY_US); "
                         "with --serialize 1 it blocks the main stream, otherwise the side stream hides it")
    ap.add_argument("--loop", choices=["library", "python"], default="library",
                    help="who drives the iterations of a configuration with an attached model: ols_run_steps, or one "
                         "call per step from Python")
    ap.add_argument("--no-second-buffer", action="store_true")
    ap.add_argument("--fuse-gemm-update", type=int, default=1,
                    help="1 (default): gradient kernels apply the local step themselves; 0: separate streaming pass")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="before the timed region run one plain element-wise copy kernel of this size (reads and "
                         "writes that many MiB): the known-size reference the HBM traffic counters are scaled by")
    ap.add_argument("--sync-rule", choices=["paper", "stale-average"], default="paper",
                    help="synchronisation rule: the paper's pull-back + anchor average, or the stale-average "
                         "alternative of its related-work section (x <- z + (x - snapshot); the CPU baseline is then "
                         "not run, it times the paper's rule)")
    ap.add_argument("--tau", type=int, default=None,
                    help="override the configuration's tau (local steps per round), e.g. for the latency sweep at tau = 1")
    ap.add_argument("--opt", action="append", default=[], help="KEY=VALUE library option (numeric key), repeatable")
    return ap.parse_args()


def algorithmic_work(cfg, ld, fused_update=True):
    """Per-launch algorithmic bytes / flops of each kernel kind (element-replicas x bytes, 2 M N K)."""
    m = cfg.m
    er = m * ld                        # element-replicas one streaming launch touches
    mom = 8 if cfg.mu != 0.0 else 0    # read + write of the momentum buffer
    shadow = 2 if cfg.gemm_dtype == "bf16" else 0
    work = {
        "step": ("hbm", er * (12 + mom + shadow)),
        "step_pull": ("hbm", er * (12 + mom + shadow) + 4 * ld),
        "pull": ("hbm", er * (8 + shadow) + 4 * ld),
        "mean": ("hbm", (4 * m + 4) * ld),
        "step_pull_mean": ("hbm", er * (12 + mom) + 8 * ld),
        "mix": ("hbm", (8 * (m + 1) + shadow * m) * ld),     # every row of [x, z] read once and written once
        "stale_sync": ("hbm", er * (16 + shadow) + 4 * ld),  # x and snapshot read and written, z read
    }
    if cfg.kind == "mlp":
        dims, B = cfg.dims, cfg.batch
        L = len(dims) - 1
        fwd = [2.0 * m * B * dims[l] * dims[l + 1] for l in range(L - 1)]
        work["gemm_fwd"] = ("mfma", sum(fwd) / max(len(fwd), 1))
        # algorithmic bytes of the same launches (operands read once, output written once): the arithmetic intensity
        # decides whether the matrix-core peak or AI x HBM peak is the lower ceiling (batch 256 in bf16: the latter)
        es_ = 2 if cfg.gemm_dtype == "bf16" else 4
        fb = [m * es_ * (B * dims[l] + dims[l] * dims[l + 1] + B * dims[l + 1]) for l in range(L - 1)]
        work["gemm_fwd_bytes"] = sum(fb) / max(len(fb), 1)
        db = [m * es_ * (B * dims[l + 1] + dims[l] * dims[l + 1] + 2 * B * dims[l]) for l in range(1, L - 1)]
        if db:
            work["gemm_da_bytes"] = sum(db) / len(db)
        work["gemm_dw"] = ("mfma", sum(fwd) / max(len(fwd), 1))
        if fused_update and L > 1:
            # the weight-gradient kernel also applies the local step: it reads and writes the layer's
            # parameters and momentum (16 B per element-replica, 8 B without momentum, + 2 B bf16 shadow)
            # and reads its two operands; those bytes, not the flops, bound it
            es = 2 if cfg.gemm_dtype == "bf16" else 4
            per_elem = 8 + mom + shadow
            dw_bytes = [m * (dims[l] * dims[l + 1] * per_elem + B * (dims[l] + dims[l + 1]) * es) for l in range(L - 1)]
            work["gemm_dw"] = ("hbm", sum(dw_bytes) / len(dw_bytes))
            work["gemm_dw_flops"] = sum(fwd) / len(fwd)
        da = [2.0 * m * B * dims[l] * dims[l + 1] for l in range(1, L - 1)]
        if da:
            work["gemm_da"] = ("mfma", sum(da) / len(da))
    if cfg.kind == "conv":
        C, H, W, _ = cfg.dims
        flops = 2.0 * m * cfg.batch * H * W * 9 * C * C      # one 3 x 3 convolution as a GEMM, all workers
        act = 4.0 * m * cfg.batch * H * W * C                # bytes of one activation tensor
        work["conv_fwd"] = ("mfma", flops)
        work["conv_dx"] = ("mfma", flops)
        work["conv_dw"] = ("mfma", flops)
        work["pool"] = ("hbm", act)
        work["pool_bwd"] = ("hbm", 2 * act)
        if cfg.gemm_dtype == "bf16" and cfg.batch_norm:
            # convolutions: bf16 operands in, fp32 out (the normalisations' input); the delta also reads the bf16 gate
            work["cast_bf16"] = ("hbm", 1.5 * act)
            work["conv_fwd_bytes"] = 1.5 * act
            work["conv_dx_bytes"] = 2.0 * act
            work["conv_dw_bytes"] = 1.0 * act
        elif cfg.gemm_dtype == "bf16":
            # bytes of the tensors each launch has to touch once (bf16 operands are half an fp32 tensor; the border the
            # kernels store with them is overhead, not work): 288 flop per byte for a bf16-in, bf16-out convolution,
            # just below the 312 flop per byte ridge, so min(matrix peak, AI x HBM peak) is reported beside the peak
            work["cast_bf16"] = ("hbm", 1.5 * act)                      # fp32 batch in, bf16 batch out
            work["conv_dx_bytes"] = 1.5 * act                           # bf16 delta in, bf16 mask in, bf16 delta out
            work["conv_dw_bytes"] = 1.0 * act                           # bf16 input and bf16 delta
            if (H + 2) * (W + 2) >= 64:
                # the block's tail runs in the second convolution's epilogue: bf16 in, fp32 shortcut in, sign bytes out;
                # what is left of the pooling is a pass over the wavefronts' partial sums (8 C floats per 256 padded pixels)
                work["conv_fwd_bytes"] = (1.0 * act + (1.5 + 1.0 / 16) * act) / 2
                tiles = -(-(cfg.batch * (H + 2) * (W + 2)) // 256)
                work["pool"] = ("hbm", 4.0 * m * (tiles * 8 * C + cfg.batch * C))
            else:
                work["conv_fwd_bytes"] = (1.0 * act + 1.5 * act) / 2    # first: bf16 in, bf16 out; second: bf16 in, fp32 out
                work["pool"] = ("hbm", 2.0 * act + act / 16)            # shortcut + ReLU + pooling: conv output and shortcut in, sign bytes out
            work["pool_bwd"] = ("hbm", 0.5 * act + act / 16)            # sign bytes in, bf16 delta out
        if cfg.batch_norm:
            bf = cfg.gemm_dtype == "bf16"
            tail = H * W >= 64
            # Forward, first layer: the statistics read z (not with bf16 operands: the convolution's epilogue left them per
            # wavefront), the normalisation reads z and writes a1 (half a tensor as a bf16 operand).  Second layer: the
            # statistics as before; the normalisation reads z and the shortcut and writes a2 -- or, as the block's tail
            # (images of at least 64 pixels), only a2's sign bytes.  bench.py reports the mean of the two launches.
            first = (0.0 if bf else 1.0) + 1.0 + (0.5 if bf else 1.0)
            second = (0.0 if bf else 1.0) + 2.0 + (1.0 / 16 if tail else 1.0)
            work["bn_fwd"] = ("hbm", (first + second) / 2 * act)
            # Backward, second layer: the gradient under pooling and ReLU is formed from the pooled gradient and a2 (or its
            # sign bytes), so the sums read that and z, and the gradient at z reads both again and is written (half a
            # tensor as a bf16 operand).  First layer: the stored gradient instead of the gate.
            gate = 1.0 / 16 if tail else 1.0
            out = 0.5 if bf else 1.0
            work["bn_bwd"] = ("hbm", ((2 * (gate + 1.0) + out) + (4.0 + out)) / 2 * act)
            if tail:   # the pooling is a pass over the sums per 64 pixels
                work["pool"] = ("hbm", 4.0 * m * (-(-(cfg.batch * H * W) // 64) * 2 * C + cfg.batch * C))
            work.pop("pool_bwd", None)   # no such pass in the normalised blocks
    return work


def build_workload(cfg, sess, torch):
    """Uploads the configuration's synthetic inputs; returns the per-iteration input binder."""
    from ols_inputs import generate as G
    if cfg.kind == "mlp":
        X, labels = G.mlp_data(cfg)
        Xd, yd = sess.upload(X), sess.upload(labels)
        x0 = G.mlp_init(cfg)
        sess.attach_mlp(cfg.dims, cfg.batch, cfg.gemm_dtype)
        sess.init_params(x0)
        return (lambda k: sess.set_batch(Xd[:, k % cfg.nb], yd[:, k % cfg.nb])), (X, labels, x0), (Xd, yd)
    if cfg.kind == "conv":
        X, labels = G.conv_data(cfg)
        Xd, yd = sess.upload(X), sess.upload(labels)
        x0 = G.conv_init(cfg)
        sess.attach_convblock(*cfg.dims, cfg.batch, batch_norm=cfg.batch_norm, gemm_dtype=cfg.gemm_dtype)
        sess.init_params(x0)
        return (lambda k: sess.set_batch(Xd[:, k % cfg.nb], yd[:, k % cfg.nb])), (X, labels, x0), (Xd, yd)
    if cfg.kind == "lsq":
        A, y, _, x0 = G.lsq_data(cfg)
        Ad, yd = sess.upload(A), sess.upload(y)
        sess.attach_lsq(cfg.batch)
        sess.init_params(x0)
        return (lambda k: sess.set_batch(Ad[:, k % cfg.nb], yd[:, k % cfg.nb])), (A, y, x0), (Ad, yd)
    # update-only stream: a pool of gradient tensors cycled per iteration
    x0 = G.stream_x0(cfg)
    pool = []
    for j in range(cfg.grad_pool):
        t = torch.zeros(cfg.m, sess.ld, dtype=torch.float32, device=sess.device)
        t[:, : cfg.d] = torch.from_numpy(G.stream_gradient(cfg, j)).to(sess.device)
        pool.append(t)
    torch.cuda.synchronize()
    sess.bind(pool[0])
    sess.init_params(x0)
    return (lambda k: sess.set_gradient(pool[k % len(pool)])), (None, None, x0), None


def cpu_baseline(cfg, host_inputs, seconds, side=False):
    """The oracle as it stands, timed on this machine's host cores on a prefix of the same workload: one round to
    calibrate, then as many rounds as fit `seconds` (the calibration round itself where one round already takes
    longer).  As a side record the convolutional workloads, whose single round takes the oracle most of a minute, are
    timed on their first 4 workers."""
    from oracle import workloads as OW
    from ols_inputs import generate as G
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    workers_note = "all %d workers" % cfg.m
    if cfg.kind == "mlp":
        X, labels, x0 = host_inputs
        grad_fn = OW.mlp_grad_fn(cfg.dims, X, labels)
        m_eff, d_eff = cfg.m, cfg.d
    elif cfg.kind == "lsq":
        A, y, x0 = host_inputs
        grad_fn = OW.lsq_grad_fn(A, y)
        m_eff, d_eff = cfg.m, cfg.d
    elif cfg.kind == "conv":
        X, labels, x0 = host_inputs
        if side and cfg.m > 4:
            workers_note = "workers 0-3 of %d" % cfg.m
            cfg = cfg.scaled(m=4)
        grad_fn = OW.conv_grad_fn(cfg.dims, X, labels, batch_norm=cfg.batch_norm)
        m_eff, d_eff = cfg.m, cfg.d
    else:  # the update is element-wise: time the oracle on a slice of the columns
        d_eff = 1 << 20
        x0 = host_inputs[2][:d_eff]
        grads = [G.stream_gradient(cfg, j, d=d_eff) for j in range(cfg.grad_pool)]
        grad_fn = OW.stream_grad_fn(grads)
        m_eff = cfg.m
    t0 = time.perf_counter()
    OW.run_config(cfg, x0, grad_fn, K=cfg.tau)
    dt = time.perf_counter() - t0
    rounds = 1
    if dt < 0.5 * seconds:
        rounds = int(max(1, min(cfg.rounds, seconds / max(dt, 1e-6))))
        t0 = time.perf_counter()
        OW.run_config(cfg, x0, grad_fn, K=rounds * cfg.tau)
        dt = time.perf_counter() - t0
    value = m_eff * rounds * cfg.tau / dt * (d_eff / cfg.d)
    sample = "first %d iterations (%d rounds) of the workload, %s" % (rounds * cfg.tau, rounds, workers_note)
    if d_eff != cfg.d:
        sample += ", first %d of %d parameter columns (rate scaled by the column fraction)" % (d_eff, cfg.d)
    return {"value": value, "unit": "worker-iterations/s", "cores": cores, "kind": "oracle", "sample": sample,
            "seconds": dt}


def mixing_matrix_input(cfg, which):
    """The caller's W for --mixing: an INPUT of the path; only its entries are written here."""
    Wm = np.zeros((cfg.m + 1, cfg.m + 1), np.float32)
    if which == "paper":      # Section 2, matrix-form update rule
        Wm[:cfg.m, :cfg.m] = (1.0 - cfg.alpha) * np.eye(cfg.m)
        Wm[:cfg.m, cfg.m] = (1.0 - cfg.alpha) / cfg.m
        Wm[cfg.m, :] = cfg.alpha
    else:                     # Local SGD's periodic averaging (first display of Section 2)
        Wm[:cfg.m, :] = 1.0 / cfg.m
    return Wm


def measure(idx, args, K, W, cpu_seconds, side):
    """One configuration: W untimed steps, K timed steps (host clock around stream drains), a second pass of K steps
    with HIP events around every launch for the per-kernel figures, then the schedule variants (same K and W) and the
    oracle.  `side`: a record for the "configs" key -- default options, variants always measured."""
    import torch
    import ols_inputs as I
    from paper_2002_09539_amd import binding as B
    from paper_2002_09539_amd.session import Session

    cfg = I.get(idx)
    if not side and args.tau is not None:
        cfg = cfg.scaled(tau=args.tau)
    serialize = 2 if side else args.serialize
    mixing = "none" if side else args.mixing
    delay = 0 if side else args.anchor_delay_us
    sync_rule = "paper" if side else args.sync_rule
    fuse_gemm_update = 1 if side else args.fuse_gemm_update
    second_buffer = True if side else not args.no_second_buffer
    fuse_mean = None if side else args.fuse_mean
    plain = serialize == 2 and mixing == "none" and not delay and sync_rule == "paper"
    if fuse_mean is None:
        fuse_mean = 1 if (cfg.kind == "stream" and plain) else 0

    sess = Session(cfg.m, cfg.d, cfg.tau, cfg.alpha, cfg.gamma, cfg.mu,
                   overlap_buffer=second_buffer, own_gradient=cfg.kind != "stream")
    # what the library's default (2) resolves to: in line when the refresh moves at most 1 MiB
    in_line = serialize == 1 or (serialize == 2 and (4 * cfg.m + 4) * sess.ld <= (1 << 20))
    sess.set_option(B.OLS_OPT_NESTEROV, int(cfg.nesterov))
    sess.set_option(B.OLS_OPT_SERIALIZE, serialize)
    sess.set_option(B.OLS_OPT_FUSE_MEAN, fuse_mean)
    sess.set_option(B.OLS_OPT_ANCHOR_DELAY_US, delay)
    sess.set_option(B.OLS_OPT_FUSE_GEMM_UPDATE, fuse_gemm_update)
    if not side:
        for kv in args.opt:
            key, val = kv.split("=")
            sess.set_option(int(key), int(val))
    feed, host_inputs, resident = build_workload(cfg, sess, torch)
    if not side and args.loop == "python":
        resident = None
    if mixing != "none":
        sess.set_mixing(mixing_matrix_input(cfg, mixing))
    if sync_rule != "paper":
        sess.set_stale_average()

    def region(steps):
        sess.sync()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if resident is not None:      # the iteration loop runs inside the library (ols_run_steps)
            sess.run_resident(steps, *resident)
        else:
            sess.run(steps, feed)
        sess.sync()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def finish_round():
        """Untimed: completes the current round, so that options that may not change in mid-round can."""
        k = B.ols_iteration(sess.h)
        if k % cfg.tau:
            region(cfg.tau - k % cfg.tau)

    if not side and args.calibration_copy_mib > 0:
        n = args.calibration_copy_mib * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device=sess.device)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)          # one vectorised element-wise kernel: n floats in, n floats out
        torch.cuda.synchronize()
        del src, dst

    if W > 0:
        region(W)
    elapsed = region(K)
    value = cfg.m * K / elapsed

    kernels, roofline = {}, None
    if side or not args.no_kernel_timing:
        sess.set_option(B.OLS_OPT_KERNEL_TIMING, 1)
        timed_elapsed = region(K)
        stats = sess.kernel_stats()
        sess.set_option(B.OLS_OPT_KERNEL_TIMING, 0)
        work = algorithmic_work(cfg, sess.ld, fused_update=bool(fuse_gemm_update) and not fuse_mean)
        for name, (n, ms) in stats.items():
            entry = {"launches": n, "avg_us": 1e3 * ms / n, "total_ms": ms}
            if name in work:
                bound, amount = work[name]
                rate = amount / (ms / n * 1e-3)
                if bound == "hbm":
                    entry.update(bound="hbm", achieved=rate / 1e9, peak=HBM_PEAK_GBS, unit="GB/s",
                                 frac=rate / 1e9 / HBM_PEAK_GBS, per_launch=amount)
                else:
                    peak = MFMA_PEAK_TFLOPS[cfg.gemm_dtype if cfg.kind in ("mlp", "conv") else "f32"]
                    entry.update(bound="mfma", achieved=rate / 1e12, peak=peak, unit="TFLOP/s",
                                 frac=rate / 1e12 / peak, per_launch=amount)
                    if name + "_bytes" in work:   # fraction of min(matrix-core peak, arithmetic intensity x HBM peak)
                        ceiling = min(peak, amount / work[name + "_bytes"] * HBM_PEAK_GBS / 1e3)
                        entry.update(ceiling_tflops=ceiling, frac_of_ceiling=rate / 1e12 / ceiling)
            if name + "_flops" in work:
                entry["mfma_tflops"] = work[name + "_flops"] / (ms / n * 1e-3) / 1e12
            kernels[name] = entry
        ranked = sorted((e["total_ms"], n) for n, e in kernels.items() if "bound" in e)
        if ranked:
            dom = ranked[-1][1]
            e = kernels[dom]
            # HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload (counters cannot be
            # read from inside this process); null when the summary does not cover the kernel
            traffic = None
            tpath = os.path.join(ROOT, "profiles", "traffic.json")
            if os.path.exists(tpath) and plain:
                traffic = json.load(open(tpath)).get("cfg%d" % idx, {}).get(dom)
            roofline = {"kernel": dom, "bound": e["bound"], "achieved": e["achieved"], "peak": e["peak"],
                        "unit": e["unit"], "frac": e["frac"], "traffic": traffic,
                        "traffic_source": "profiles/hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)" if traffic else None,
                        "avg_launch_us": e["avg_us"], "algorithmic_per_launch": e["per_launch"]}
        kernels["_region_ms_with_event_timing"] = 1e3 * timed_elapsed

    # the other schedules of the same workload, same K and W: the refresh on the side stream beside the next round
    # (overlapped), and on the main stream (serialised)
    variants = {}
    if plain and (side or not args.no_kernel_timing):
        finish_round()
        for name, (fm, ser) in (("overlapped_side_stream", (0, 0)), ("serialized", (0, 1))):
            if fm == fuse_mean and ser == (1 if in_line else 0):
                variants[name] = 1e3 * elapsed / K
                continue
            sess.set_option(B.OLS_OPT_FUSE_MEAN, fm)
            sess.set_option(B.OLS_OPT_SERIALIZE, ser)
            if W > 0:
                region(W)
            variants[name] = 1e3 * region(K) / K
            finish_round()
        sess.set_option(B.OLS_OPT_FUSE_MEAN, fuse_mean)
        sess.set_option(B.OLS_OPT_SERIALIZE, serialize)
        if fuse_mean:
            variants["fused_step_pull_mean"] = 1e3 * elapsed / K

    base = cpu_baseline(cfg, host_inputs, cpu_seconds, side) if cpu_seconds > 0 and sync_rule == "paper" else None
    sess.close()
    del sess, feed, resident, host_inputs
    torch.cuda.empty_cache()

    config = {"workload": cfg.name, "m": cfg.m, "d": cfg.d, "tau": cfg.tau, "batch": cfg.batch,
              "dims": list(cfg.dims), "sync_rule": sync_rule,
              "overlap": ("mixing-kernel:" + mixing) if mixing != "none" else
              ("fused-mean" if fuse_mean else ("serialized" if in_line else "side-stream")),
              "second_buffer": second_buffer, "anchor_delay_us": delay,
              "loop": "library" if cfg.kind != "stream" and not (not side and args.loop == "python") else "python",
              "update": "in-gradient-kernels" if (fuse_gemm_update and cfg.kind != "stream") else "streaming"}
    return {"cfg": cfg, "value": value, "steps": K, "warmup": W, "ms_per_step": 1e3 * elapsed / K,
            "dtype": cfg.gemm_dtype if cfg.kind in ("mlp", "conv") else "f32", "config": config, "roofline": roofline,
            "cpu_baseline": base, "kernels": kernels, "ms_per_step_by_schedule": variants}


def compact(rec):
    """The record of a side configuration under "configs"."""
    r = rec["roofline"] or {}
    return {"workload": rec["config"]["workload"], "dtype": rec["dtype"], "steps": rec["steps"], "warmup": rec["warmup"],
            "ms_per_step": rec["ms_per_step"], "worker_iterations_per_s": rec["value"],
            "ms_per_step_by_schedule": rec["ms_per_step_by_schedule"], "default_schedule": rec["config"]["overlap"],
            "dominant_kernel": r.get("kernel"), "bound": r.get("bound"), "frac": r.get("frac"),
            "achieved": r.get("achieved"), "unit": r.get("unit"), "avg_launch_us": r.get("avg_launch_us"),
            "kernels_avg_us": {k: round(v["avg_us"], 2) for k, v in rec["kernels"].items() if isinstance(v, dict)},
            "kernels_frac": {k: round(v["frac"], 4) for k, v in rec["kernels"].items() if isinstance(v, dict) and "frac" in v},
            "kernels_frac_of_min_mfma_hbm_ceiling": {k: round(v["frac_of_ceiling"], 4) for k, v in rec["kernels"].items()
                                                     if isinstance(v, dict) and "frac_of_ceiling" in v},
            "oracle_worker_iterations_per_s": None if rec["cpu_baseline"] is None else rec["cpu_baseline"]["value"],
            "oracle_sample": None if rec["cpu_baseline"] is None else rec["cpu_baseline"]["sample"]}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the m workers are replicas inside one MI355X); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import ols_inputs as I

    cfg = I.get(args.config)
    # Defaults: at least the configuration's own iteration count and about a second of timed work; the warm-up covers
    # every resident batch once and lets the clocks settle.  --steps and --warmup are honoured exactly as given (a
    # region may begin and end in mid-round: K consecutive steps contain K / tau synchronisations wherever they start).
    K = args.steps if args.steps is not None else max(cfg.K, 1000)
    W = args.warmup if args.warmup is not None else max(200, 2 * max(cfg.nb, 1))
    if K < 1 or W < 0:
        print("bench.py: --steps must be >= 1 and --warmup >= 0", file=sys.stderr)
        sys.exit(2)
    default_options = (args.serialize == 2 and args.fuse_mean is None and args.mixing == "none" and not args.anchor_delay_us
                       and args.sync_rule == "paper" and args.fuse_gemm_update == 1 and not args.no_second_buffer
                       and not args.opt and args.loop == "library" and not args.no_kernel_timing and args.tau is None
                       and not args.calibration_copy_mib)
    if args.side_configs is None:
        sides = [1, 2, 3, 5, 6, 7, 8, 9] if (args.config == 4 and default_options) else []
    else:
        sides = [int(t) for t in args.side_configs.split(",") if t.strip()]

    head = measure(args.config, args, K, W, args.cpu_seconds, side=False)
    configs = {}
    for idx in sides:
        c = I.get(idx)
        # run length of a side record: the configuration's own iteration count, at least 1000 steps, after 200 warm-up
        # steps; the convolutional workload (7 ms per step) runs its own 100 iterations after 20
        k_side, w_side = (c.K, 20) if c.kind == "conv" else (max(c.K, 1000), 200)
        try:
            configs[c.name] = compact(measure(idx, args, k_side, w_side, args.side_cpu_seconds, side=True))
        except Exception as exc:   # a side record must not cost the headline
            configs[c.name] = {"workload": c.name, "error": "%s: %s" % (type(exc).__name__, exc)}

    out = {
        "metric": "worker-iterations/sec at m replicas",
        "value": head["value"],
        "unit": "worker-iterations/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic",
        "config": head["config"],
        "roofline": head["roofline"],
        "cpu_baseline": head["cpu_baseline"],
        "ms_per_step_by_schedule": head["ms_per_step_by_schedule"],
        "kernels": head["kernels"],
        "configs": configs,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
