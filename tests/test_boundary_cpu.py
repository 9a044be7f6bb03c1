"""Host-side tests of the C boundary that need no GPU: the library loads, exports every declared
symbol, validates its arguments, and enforces the call order of the algorithm (Section 2 of
arXiv 2002.09539: tau local steps, then the pull-back, then the anchor refresh).  The schedule is
exercised in dry-run mode, where nothing is launched and the launch trace is recorded."""
import os
import re

import pytest

from paper_2002_09539_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000000000  # 256-byte aligned stand-in addresses; never dereferenced in dry-run mode


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ols.h")).read()
    return sorted(set(re.findall(r"OLS_API [\w\s\*]+?\b(ols_\w+)\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = declared_symbols()
    assert len(names) >= 25
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(B._SIGNATURES), "binding and header disagree"
    assert "gfx950" in B.ols_version()


def test_row_stride():
    assert B.ols_row_stride(1) == 64 and B.ols_row_stride(64) == 64 and B.ols_row_stride(65) == 128
    assert B.ols_row_stride(1578506) == 1578560 and B.ols_row_stride(0) == 0


@pytest.mark.parametrize("args", [(0, 8, 2, .5, .1, 0.), (4, 0, 2, .5, .1, 0.), (4, 8, 0, .5, .1, 0.),
                                  (4, 8, 2, 1.5, .1, 0.), (4, 8, 2, -.1, .1, 0.), (4, 8, 2, .5, 0., 0.),
                                  (4, 8, 2, .5, .1, 1.0), (4, 8, 2, .5, .1, -0.1)])
def test_create_rejects_bad_arguments(args):
    with pytest.raises(B.OlsError) as e:
        B.ols_create(*args)
    assert e.value.code == B.OLS_EINVAL and len(str(e.value)) > 20


def dry(m=4, d=100, tau=2, alpha=0.6, gamma=0.1, mu=0.9, alt=True, trace=True):
    h = B.ols_create(m, d, tau, alpha, gamma, mu)
    B.ols_set_option(h, B.OLS_OPT_DRY_RUN, 1)
    B.ols_set_option(h, B.OLS_OPT_SERIALIZE, 0)       # the paper's overlapped schedule, also for these tiny problems
    if trace:
        B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    ld = B.ols_row_stride(d)
    B.ols_bind(h, FAKE, FAKE + (1 << 30) if alt else None, FAKE + (2 << 30) if mu else None, FAKE + (3 << 30),
               FAKE + (4 << 30), ld, None, 8)
    return h


def code_of(fn, *a):
    with pytest.raises(B.OlsError) as e:
        fn(*a)
    return e.value.code


def test_bind_validation():
    h = B.ols_create(4, 100, 2, 0.6, 0.1, 0.9)
    ld = B.ols_row_stride(100)
    assert code_of(B.ols_bind, h, FAKE, None, None, FAKE, FAKE, ld, None, None) == B.OLS_EINVAL   # buf missing
    assert code_of(B.ols_bind, h, FAKE, None, FAKE, FAKE, FAKE, 100, None, None) == B.OLS_EINVAL  # wrong ld
    assert code_of(B.ols_bind, h, FAKE + 4, None, FAKE, FAKE, FAKE, ld, None, None) == B.OLS_EINVAL  # alignment
    assert code_of(B.ols_bind, h, FAKE, FAKE, FAKE, FAKE, FAKE, ld, None, None) == B.OLS_EINVAL   # x_alt == x
    assert code_of(B.ols_local_step, h) == B.OLS_ESTATE                                           # unbound
    B.ols_destroy(h)


def test_call_order_is_enforced():
    h = dry(tau=2)
    assert code_of(B.ols_local_step, h) == B.OLS_ESTATE          # before init
    B.ols_init_params(h, FAKE)
    assert code_of(B.ols_sync_pull, h) == B.OLS_ESTATE           # k = 0
    B.ols_local_step(h)
    assert code_of(B.ols_sync_pull, h) == B.OLS_ESTATE           # k = 1, tau = 2
    assert code_of(B.ols_anchor_update_async, h) == B.OLS_ESTATE
    B.ols_local_step(h)
    assert B.ols_iteration(h) == 2
    assert code_of(B.ols_local_step, h) == B.OLS_ESTATE          # pull due
    assert code_of(B.ols_get_params, h, 0, FAKE, 1) == B.OLS_ESTATE  # deferred write pending
    assert code_of(B.ols_set_gradient, h, FAKE) == B.OLS_ESTATE
    B.ols_sync_pull(h)
    assert code_of(B.ols_sync_pull, h) == B.OLS_ESTATE           # already pulled
    assert code_of(B.ols_local_step, h) == B.OLS_ESTATE          # anchor refresh due
    B.ols_anchor_update_async(h)
    assert code_of(B.ols_anchor_update_async, h) == B.OLS_ESTATE
    B.ols_local_step(h)
    B.ols_destroy(h)


def kinds(trace):
    return [B.ols_kernel_name(t["kind"]) for t in trace]


def run_rounds(h, rounds, tau):
    B.ols_init_params(h, FAKE)
    for _ in range(rounds):
        for _ in range(tau):
            B.ols_local_step(h)
        B.ols_sync_pull(h)
        B.ols_anchor_update_async(h)


def test_overlap_schedule_with_second_buffer():
    """The first update after a refresh goes out-of-place so the side stream still sees the
    round-boundary models; the main stream waits for the refresh only at the next pull."""
    h = dry(tau=3)
    run_rounds(h, 3, 3)
    tr = B.ols_trace(h)
    assert kinds(tr) == ["init"] + ["step", "step", "step_pull", "mean"] * 3
    r1, r2, r3 = tr[1:5], tr[5:9], tr[9:13]
    # round 1: no refresh in flight yet -> in place on buffer 0, no waits
    assert [(t["src_buf"], t["dst_buf"], t["waited"]) for t in r1[:3]] == [(0, 0, 0)] * 3
    assert r1[3]["stream"] == 1 and r1[3]["src_buf"] == 0 and r1[3]["waited"] == 1   # side waits for the pull
    # round 2: first step reads 0 writes 1 without waiting; later in place on 1; pull waits for refresh 1
    assert [(t["src_buf"], t["dst_buf"], t["waited"]) for t in r2[:3]] == [(0, 1, 0), (1, 1, 0), (1, 1, 1)]
    assert r2[3]["src_buf"] == 1
    assert [(t["src_buf"], t["dst_buf"], t["waited"]) for t in r3[:3]] == [(1, 0, 0), (0, 0, 0), (0, 0, 1)]
    assert all(t["stream"] == 0 for t in tr if B.ols_kernel_name(t["kind"]) != "mean")
    B.ols_destroy(h)


def test_schedule_without_second_buffer_waits_before_first_write():
    h = dry(tau=2, alt=False)
    run_rounds(h, 2, 2)
    tr = B.ols_trace(h)
    assert kinds(tr) == ["init", "step", "step_pull", "mean", "step", "step_pull", "mean"]
    assert tr[4]["waited"] == 1 and (tr[4]["src_buf"], tr[4]["dst_buf"]) == (0, 0)   # in-place write waits
    assert tr[5]["waited"] == 0                                                     # already waited
    B.ols_destroy(h)


def test_serialized_and_unfused_schedules():
    h = dry(tau=2)
    B.ols_set_option(h, B.OLS_OPT_SERIALIZE, 1)
    B.ols_set_option(h, B.OLS_OPT_FUSE_PULL, 0)
    run_rounds(h, 2, 2)
    tr = B.ols_trace(h)
    assert kinds(tr) == ["init"] + ["step", "step", "pull", "mean"] * 2
    assert all(t["stream"] == 0 and t["waited"] == 0 for t in tr)
    assert all(t["dst_buf"] in (0, -1) for t in tr)
    B.ols_destroy(h)


def test_tau_one_and_fused_mean_schedules():
    h = dry(tau=1)
    run_rounds(h, 3, 1)
    tr = B.ols_trace(h)
    assert kinds(tr) == ["init"] + ["step_pull", "mean"] * 3
    assert [t["waited"] for t in tr[1::2]] == [0, 1, 1]          # each pull needs the previous refresh
    B.ols_destroy(h)
    h = dry(tau=2)
    B.ols_set_option(h, B.OLS_OPT_FUSE_MEAN, 1)
    run_rounds(h, 2, 2)
    assert kinds(B.ols_trace(h)) == ["init"] + ["step", "step_pull_mean"] * 2
    B.ols_destroy(h)


def test_emulated_communication_delay_precedes_every_refresh_on_its_stream():
    h = dry(tau=2)
    B.ols_set_option(h, B.OLS_OPT_ANCHOR_DELAY_US, 250)
    run_rounds(h, 2, 2)
    tr = B.ols_trace(h)
    assert kinds(tr) == ["init"] + ["step", "step_pull", "delay", "mean"] * 2
    assert [t["stream"] for t in tr if t["kind"] in (B.OLS_K_DELAY, B.OLS_K_MEAN)] == [1] * 4
    assert [t["waited"] for t in tr if t["kind"] == B.OLS_K_DELAY] == [1, 1]   # the side stream waits for the pull
    B.ols_destroy(h)
    h = dry(tau=2)   # blocking synchronisation with the same latency: everything on the main stream
    B.ols_set_option(h, B.OLS_OPT_SERIALIZE, 1)
    B.ols_set_option(h, B.OLS_OPT_ANCHOR_DELAY_US, 250)
    run_rounds(h, 1, 2)
    tr = B.ols_trace(h)
    assert kinds(tr) == ["init", "step", "step_pull", "delay", "mean"] and all(t["stream"] == 0 for t in tr)
    B.ols_destroy(h)
    h = dry(tau=2)   # no refresh kernel, nothing to delay
    B.ols_set_option(h, B.OLS_OPT_FUSE_MEAN, 1)
    B.ols_set_option(h, B.OLS_OPT_ANCHOR_DELAY_US, 250)
    run_rounds(h, 1, 2)
    assert kinds(B.ols_trace(h)) == ["init", "step", "step_pull_mean"]
    for bad in (-1, 1000001):
        with pytest.raises(B.OlsError) as e:
            B.ols_set_option(h, B.OLS_OPT_ANCHOR_DELAY_US, bad)
        assert e.value.code == B.OLS_EINVAL
    B.ols_destroy(h)


def test_trailing_steps_need_no_pull():
    h = dry(tau=4)
    B.ols_init_params(h, FAKE)
    for _ in range(3):
        B.ols_local_step(h)
    assert B.ols_iteration(h) == 3
    B.ols_get_params(h, 0, FAKE, 1)      # legal: nothing pending (dry run copies nothing)
    B.ols_destroy(h)


def test_model_attachment_validation():
    h = dry(d=3 * 8 + 8 + 8 * 4 + 4, mu=0.0)
    assert code_of(B.ols_attach_mlp, h, [3, 8, 4], 8, 0) == B.OLS_EINVAL      # dims[0] not a multiple of 4
    B.ols_destroy(h)
    d = 8 * 12 + 12 + 12 * 5 + 5
    h = dry(d=d, mu=0.0)
    assert code_of(B.ols_attach_mlp, h, [8, 12, 5], 6, 0) == B.OLS_EINVAL     # batch not a multiple of 4
    assert code_of(B.ols_attach_mlp, h, [8, 12, 40], 8, 0) == B.OLS_EINVAL    # too many classes
    assert code_of(B.ols_attach_mlp, h, [8, 16, 5], 8, 0) == B.OLS_EINVAL     # d mismatch
    assert code_of(B.ols_attach_mlp, h, [8, 12, 5], 8, 2) == B.OLS_EINVAL     # dtype
    B.ols_attach_mlp(h, [8, 12, 5], 8, 0)
    need = B.ols_workspace_bytes(h)
    assert need >= 4 * (2 * 8 * 12 + 8 * 5 + 8) * 4
    assert code_of(B.ols_bind_workspace, h, FAKE, need - 1) == B.OLS_ENOMEM
    B.ols_init_params(h, FAKE)
    assert code_of(B.ols_local_step, h) == B.OLS_ESTATE                       # no workspace
    B.ols_bind_workspace(h, FAKE, need)
    assert code_of(B.ols_local_step, h) == B.OLS_ESTATE                       # no batch
    assert code_of(B.ols_set_batch, h, FAKE, 8 * 8 - 4, FAKE, 8) == B.OLS_EINVAL  # worker stride too small
    B.ols_set_batch(h, FAKE, 8 * 8, FAKE, 8)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    B.ols_local_step(h)          # default: the gradient kernels apply the update themselves, and the output
    assert kinds(B.ols_trace(h)) == ["gemm_fwd", "head_fwd", "gemm_dw"]   # layer's gradients ride in gemm_dw's launch
    B.ols_local_step(h)          # boundary step (tau = 2): pull-back applied there as well
    B.ols_sync_pull(h)           # ... so the pull launches nothing
    B.ols_anchor_update_async(h)
    assert kinds(B.ols_trace(h)) == ["gemm_fwd", "head_fwd", "gemm_dw"] * 2 + ["mean"]
    B.ols_set_option(h, B.OLS_OPT_HEAD_DW_GUEST, 0)   # output-layer gradients in a kernel of their own
    B.ols_set_option(h, B.OLS_OPT_FUSE_GEMM_UPDATE, 0)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    B.ols_local_step(h)
    B.ols_local_step(h)
    B.ols_sync_pull(h)
    assert kinds(B.ols_trace(h)) == ["gemm_fwd", "head_fwd", "head_bwd", "gemm_dw", "step"] + \
        ["gemm_fwd", "head_fwd", "head_bwd", "gemm_dw", "step_pull"]
    assert code_of(B.ols_set_gradient, h, FAKE) == B.OLS_ESTATE               # the model owns g
    B.ols_destroy(h)


def test_least_squares_launch_plan():
    h = dry(d=100, mu=0.9, tau=2)
    B.ols_attach_lsq(h, 8)
    B.ols_bind_workspace(h, FAKE, B.ols_workspace_bytes(h))
    B.ols_init_params(h, FAKE)
    B.ols_set_batch(h, FAKE, 8 * 100, FAKE, 8)
    def one_round(tau):
        for _ in range(tau):
            B.ols_local_step(h)
        B.ols_sync_pull(h)
        B.ols_anchor_update_async(h)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    one_round(2)
    assert kinds(B.ols_trace(h)) == ["lsq_step", "lsq_step", "mean"]   # small problem: one launch per local step
    B.ols_set_option(h, B.OLS_OPT_FUSE_GEMM_UPDATE, 0)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    one_round(2)
    assert kinds(B.ols_trace(h)) == ["lsq_resid", "lsq_grad", "step", "lsq_resid", "lsq_grad", "step_pull", "mean"]
    B.ols_destroy(h)
    h = dry(d=5000, mu=0.9, tau=1)          # too wide for one workgroup: separate kernels
    B.ols_attach_lsq(h, 8)
    B.ols_bind_workspace(h, FAKE, B.ols_workspace_bytes(h))
    B.ols_init_params(h, FAKE)
    B.ols_set_batch(h, FAKE, 8 * 5000, FAKE, 8)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    one_round(1)
    assert kinds(B.ols_trace(h)) == ["lsq_resid", "lsq_grad", "step_pull", "mean"]
    B.ols_destroy(h)


def test_library_driven_loop_issues_the_launches_of_the_separate_calls():
    def attach():
        h = dry(d=100, mu=0.9, tau=3)
        B.ols_attach_lsq(h, 8)
        B.ols_bind_workspace(h, FAKE, B.ols_workspace_bytes(h))
        B.ols_init_params(h, FAKE)
        B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
        return h
    h = attach()
    B.ols_run_steps(h, 4, FAKE, FAKE, 5)
    B.ols_run_steps(h, 3, FAKE, FAKE, 5)
    assert B.ols_iteration(h) == 7
    a = [(t["kind"], t["stream"], t["src_buf"], t["dst_buf"], t["waited"], t["k"]) for t in B.ols_trace(h)]
    for bad in ((-1, FAKE, FAKE, 5), (1, None, FAKE, 5), (1, FAKE, None, 5), (1, FAKE, FAKE, 0)):
        assert code_of(B.ols_run_steps, h, *bad) == B.OLS_EINVAL
    B.ols_local_step(h)
    B.ols_local_step(h)                                   # k = 9: a pull is due
    assert code_of(B.ols_run_steps, h, 1, FAKE, FAKE, 5) == B.OLS_ESTATE
    B.ols_destroy(h)
    h = attach()
    for k in range(7):
        B.ols_set_batch(h, FAKE, 5 * 8 * 100, FAKE, 5 * 8)
        B.ols_local_step(h)
        if (k + 1) % 3 == 0:
            B.ols_sync_pull(h)
            B.ols_anchor_update_async(h)
    b = [(t["kind"], t["stream"], t["src_buf"], t["dst_buf"], t["waited"], t["k"]) for t in B.ols_trace(h)]
    assert a == b and len(a) == 7 + 2
    B.ols_destroy(h)
    h = dry(d=100)
    assert code_of(B.ols_run_steps, h, 1, FAKE, FAKE, 1) == B.OLS_ESTATE      # no model attached
    B.ols_destroy(h)


def test_deep_mlp_launch_plan():
    dims = [8, 12, 16, 20, 5]
    d = sum(dims[i] * dims[i + 1] + dims[i + 1] for i in range(4))
    h = dry(d=d, mu=0.9)
    B.ols_attach_mlp(h, dims, 8, 0)
    B.ols_bind_workspace(h, FAKE, B.ols_workspace_bytes(h))
    B.ols_init_params(h, FAKE)
    B.ols_set_batch(h, FAKE, 64, FAKE, 8)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    B.ols_local_step(h)
    # each layer's delta GEMM precedes its weight-gradient GEMM (which may update the weights in place)
    assert kinds(B.ols_trace(h)) == ["gemm_fwd"] * 3 + ["head_fwd"] + ["gemm_da", "gemm_dw"] * 2 + ["gemm_dw"]
    tr = B.ols_trace(h)
    assert all((t["src_buf"], t["dst_buf"]) == (0, 0) for t in tr if B.ols_kernel_name(t["kind"]) == "gemm_dw")
    B.ols_destroy(h)


def test_fused_update_uses_second_buffer_after_refresh():
    dims = [8, 12, 5]
    d = sum(dims[i] * dims[i + 1] + dims[i + 1] for i in range(2))
    h = dry(d=d, mu=0.9, tau=2)
    B.ols_attach_mlp(h, dims, 8, 0)
    B.ols_bind_workspace(h, FAKE, B.ols_workspace_bytes(h))
    B.ols_init_params(h, FAKE)
    B.ols_set_batch(h, FAKE, 64, FAKE, 8)
    for _ in range(2):
        B.ols_local_step(h)
        B.ols_local_step(h)
        B.ols_sync_pull(h)
        B.ols_anchor_update_async(h)
    B.ols_local_step(h)
    tr = [t for t in B.ols_trace(h) if B.ols_kernel_name(t["kind"]) in ("gemm_dw", "mean")]
    bufs = [(B.ols_kernel_name(t["kind"]), t["src_buf"], t["dst_buf"], t["waited"]) for t in tr]
    # the boundary step of round 2 pulls toward the anchor of round 1's refresh: its updating launch waits for it
    assert bufs == [("gemm_dw", 0, 0, 0), ("gemm_dw", 0, 0, 0), ("mean", 0, -1, 1),
                    ("gemm_dw", 0, 1, 0), ("gemm_dw", 1, 1, 1), ("mean", 1, -1, 1),
                    ("gemm_dw", 1, 0, 0)]
    B.ols_destroy(h)


@pytest.mark.parametrize("tau", [1, 2, 8])
@pytest.mark.parametrize("guest", [1, 0])
@pytest.mark.parametrize("alt", [True, False])
def test_refresh_is_awaited_only_by_the_first_launch_that_needs_it(tau, guest, alt):
    """Section 2, the sentence after the anchor update rule: the refreshed anchor is needed only by the NEXT pull-back,
    so the refresh may take tau steps of compute.  On the default route the kernels that form the gradients apply step
    and pull-back: the wait must sit on the boundary step's first updating launch (the output layer's gradient kernel,
    or the weight-gradient launch hosting its workgroups) and on no earlier launch of the round -- in particular not
    on that step's forward, output-layer forward and delta kernels, also when tau = 1.  Without a second replica
    buffer the first in-place write after a refresh waits instead, again not before that step's forward pass."""
    dims = [8, 12, 16, 5]
    d = sum(dims[i] * dims[i + 1] + dims[i + 1] for i in range(3))
    h = dry(d=d, mu=0.9, tau=tau, alt=alt)
    B.ols_attach_mlp(h, dims, 8, 0)
    B.ols_bind_workspace(h, FAKE, B.ols_workspace_bytes(h))
    B.ols_set_option(h, B.OLS_OPT_HEAD_DW_GUEST, guest)
    B.ols_init_params(h, FAKE)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    B.ols_run_steps(h, 3 * tau, FAKE, FAKE, 4)
    tr = B.ols_trace(h)
    step_kinds = ["gemm_fwd", "gemm_fwd", "head_fwd"] + ([] if guest else ["head_bwd"]) + ["gemm_da", "gemm_dw", "gemm_dw"]
    per_round = step_kinds * tau + ["mean"]
    assert kinds(tr) == per_round * 3
    first_update = 3                      # index within a step of head_bwd, or of the hosting weight-gradient launch
    if guest:
        first_update = step_kinds.index("gemm_dw")
    n = len(per_round)
    for r in range(3):
        rnd = tr[r * n:(r + 1) * n]
        waits = [i for i, t in enumerate(rnd[:-1]) if t["waited"]]
        if r == 0:
            assert waits == []                                   # nothing in flight yet
        elif alt:
            assert waits == [(tau - 1) * len(step_kinds) + first_update]   # the boundary step's first updating launch
        else:
            assert waits == [first_update]                       # the round's first in-place write
        assert rnd[-1]["stream"] == 1 and rnd[-1]["waited"] == 1  # the refresh itself waits for the pull
    B.ols_destroy(h)


def test_option_validation():
    h = dry()
    assert code_of(B.ols_set_option, h, 99, 1) == B.OLS_EINVAL
    assert code_of(B.ols_set_option, h, B.OLS_OPT_MEAN_SPLIT, 3) == B.OLS_EINVAL
    assert code_of(B.ols_set_lr, h, 0.0) == B.OLS_EINVAL
    assert code_of(B.ols_set_anchor_momentum, h, 0.7, None) == B.OLS_EINVAL
    B.ols_set_anchor_momentum(h, 0.7, FAKE)
    B.ols_destroy(h)


def test_general_mixing_replaces_pull_and_average_in_the_schedule():
    """With a mixing matrix set, a synchronisation point is: plain local step, one mixing pass on the
    main stream, no pull-back kernel and no anchor-mean kernel."""
    h = dry(m=4, tau=2, mu=0.9)
    B.ols_init_params(h, FAKE)
    B.ols_set_mixing(h, FAKE + (5 << 30))
    for _ in range(2):
        B.ols_local_step(h)
        B.ols_local_step(h)
        assert code_of(B.ols_local_step, h) == B.OLS_ESTATE        # the synchronisation is due
        assert code_of(B.ols_set_mixing, h, None) == B.OLS_ESTATE  # not in the middle of one
        B.ols_sync_pull(h)
        B.ols_anchor_update_async(h)
    kinds = [B.ols_kernel_name(e["kind"]) for e in B.ols_trace(h)]
    assert kinds == ["init", "step", "step", "mix", "step", "step", "mix"]
    assert all(e["stream"] == 0 for e in B.ols_trace(h))
    # back to the paper's synchronisation
    B.ols_set_mixing(h, None)
    B.ols_local_step(h)
    B.ols_local_step(h)
    B.ols_sync_pull(h)
    B.ols_anchor_update_async(h)
    kinds = [B.ols_kernel_name(e["kind"]) for e in B.ols_trace(h)][7:]
    assert kinds == ["step", "step_pull", "mean"]
    B.ols_destroy(h)


def test_general_mixing_argument_checks():
    h = B.ols_create(200, 64, 2, 0.5, 0.1, 0.0)
    assert code_of(B.ols_set_mixing, h, FAKE) == B.OLS_EINVAL          # more than 128 workers
    B.ols_destroy(h)
    h = dry(m=4, tau=2, mu=0.0)
    assert code_of(B.ols_set_mixing, h, FAKE + 2) == B.OLS_EINVAL      # alignment
    B.ols_set_anchor_momentum(h, 0.7, FAKE + (6 << 30))
    assert code_of(B.ols_set_mixing, h, FAKE) == B.OLS_EINVAL          # anchor momentum is set
    B.ols_destroy(h)


def test_stale_average_rule_in_the_schedule():
    """With the stale-average rule a synchronisation point is: plain local step, one synchronisation pass
    on the main stream, then the replica mean on the side stream (it overlaps the next round)."""
    h = dry(m=4, tau=2, mu=0.9)
    assert code_of(B.ols_set_stale_average, h, FAKE + (7 << 30)) == B.OLS_ESTATE   # before ols_init_params
    B.ols_init_params(h, FAKE)
    assert code_of(B.ols_set_stale_average, h, FAKE + (7 << 30) + 4) == B.OLS_EINVAL   # alignment
    assert code_of(B.ols_set_stale_average, h, FAKE) == B.OLS_EINVAL                   # aliases the replicas
    B.ols_set_stale_average(h, FAKE + (7 << 30))
    assert code_of(B.ols_set_mixing, h, FAKE + (5 << 30)) == B.OLS_EINVAL
    assert code_of(B.ols_set_anchor_momentum, h, 0.7, FAKE + (6 << 30)) == B.OLS_EINVAL
    for _ in range(2):
        B.ols_local_step(h)
        B.ols_local_step(h)
        assert code_of(B.ols_local_step, h) == B.OLS_ESTATE
        B.ols_sync_pull(h)
        B.ols_anchor_update_async(h)
    tr = B.ols_trace(h)
    assert [B.ols_kernel_name(e["kind"]) for e in tr] == ["init", "step", "step", "stale_sync", "mean",
                                                          "step", "step", "stale_sync", "mean"]
    assert [e["stream"] for e in tr] == [0, 0, 0, 0, 1, 0, 0, 0, 1]
    # the second synchronisation reads the average the first refresh produced: the main stream waits for it
    assert [e["waited"] for e in tr if B.ols_kernel_name(e["kind"]) == "stale_sync"] == [0, 1]
    assert code_of(B.ols_set_stale_average, h, None) == B.OLS_ESTATE   # not after the first local step
    B.ols_destroy(h)


def test_stale_average_rule_with_an_attached_mlp_uses_plain_gradient_kernels():
    dims = [8, 12, 5]
    h = dry(m=2, d=sum(dims[i] * dims[i + 1] + dims[i + 1] for i in range(2)), tau=2, mu=0.9)
    B.ols_attach_mlp(h, dims, 8, 0)
    B.ols_bind_workspace(h, FAKE + (8 << 30), B.ols_workspace_bytes(h))
    B.ols_init_params(h, FAKE)
    B.ols_set_batch(h, FAKE + (9 << 30), 64, FAKE + (10 << 30), 8)
    B.ols_set_stale_average(h, FAKE + (7 << 30))
    B.ols_local_step(h)
    B.ols_local_step(h)
    B.ols_sync_pull(h)
    B.ols_anchor_update_async(h)
    names = [B.ols_kernel_name(e["kind"]) for e in B.ols_trace(h)]
    assert names[-2:] == ["stale_sync", "mean"]
    assert "pull" not in names and "step_pull" not in names and "step_pull_mean" not in names
    B.ols_destroy(h)


def test_static_workspace_entry_point_checks_its_limits_without_a_device():
    """ols_run_steps_static in dry-run mode: the same launches as ols_run_steps, and a clear error for a model that
    does not fit the 64 MiB static array, for the bf16 model and while per-kernel timing is on."""
    assert B.ols_static_workspace_bytes() == 64 << 20

    def attach(dims, batch, dtype=0, m=4):
        d = sum(dims[i] * dims[i + 1] + dims[i + 1] for i in range(len(dims) - 1))
        h = dry(m=m, d=d, mu=0.9, tau=2)
        B.ols_attach_mlp(h, dims, batch, dtype)
        return h
    h = attach([8, 12, 5], 8)
    B.ols_init_params(h, FAKE)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    B.ols_run_steps_static(h, 4, FAKE, FAKE, 3)          # no ols_bind_workspace beforehand
    a = kinds(B.ols_trace(h))
    B.ols_set_option(h, B.OLS_OPT_KERNEL_TIMING, 1)
    assert code_of(B.ols_run_steps_static, h, 1, FAKE, FAKE, 3) == B.OLS_ESTATE
    B.ols_destroy(h)
    h = attach([8, 12, 5], 8)
    B.ols_bind_workspace(h, FAKE, B.ols_workspace_bytes(h))
    B.ols_init_params(h, FAKE)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    B.ols_run_steps(h, 4, FAKE, FAKE, 3)
    assert kinds(B.ols_trace(h)) == a and len(a) > 8
    B.ols_destroy(h)
    h = attach([64, 2048, 2048, 10], 256, m=16)          # 128 MiB of activations and deltas
    assert B.ols_workspace_bytes(h) > B.ols_static_workspace_bytes()
    B.ols_init_params(h, FAKE)
    assert code_of(B.ols_run_steps_static, h, 1, FAKE, FAKE, 1) == B.OLS_ENOMEM
    assert "static workspace" in B.last_error()
    B.ols_destroy(h)
    h = attach([64, 64, 10], 16, dtype=1)
    B.ols_bind_workspace(h, FAKE, B.ols_workspace_bytes(h))
    B.ols_init_params(h, FAKE)
    assert code_of(B.ols_run_steps_static, h, 1, FAKE, FAKE, 1) == B.OLS_EINVAL
    B.ols_destroy(h)
    h = dry(d=100)
    assert code_of(B.ols_run_steps_static, h, 1, FAKE, FAKE, 1) == B.OLS_ESTATE      # no model attached
    B.ols_destroy(h)


def test_convblock_attachment_and_launch_plan():
    C, H, W, classes, batch = 32, 8, 8, 10, 4
    d = 2 * (9 * C * C + C) + C * classes + classes
    h = dry(d=d, mu=0.9, tau=2)
    assert code_of(B.ols_attach_convblock, h, 24, H, W, classes, batch) == B.OLS_EINVAL      # channels not a multiple of 16
    assert code_of(B.ols_attach_convblock, h, C, H, W, 40, batch) == B.OLS_EINVAL            # too many classes
    assert code_of(B.ols_attach_convblock, h, C, H, W, classes + 1, batch) == B.OLS_EINVAL   # d does not match
    assert code_of(B.ols_attach_convblock, h, C, 0, W, classes, batch) == B.OLS_EINVAL
    B.ols_attach_convblock(h, C, H, W, classes, batch)
    need = B.ols_workspace_bytes(h)
    assert need >= 4 * 4 * batch * H * W * C * 4                    # four activation / delta tensors for 4 workers
    B.ols_bind_workspace(h, FAKE, need)
    B.ols_init_params(h, FAKE)
    assert code_of(B.ols_set_batch, h, FAKE, batch * H * W * C - 4, FAKE, batch) == B.OLS_EINVAL   # stride below one batch
    B.ols_set_batch(h, FAKE, batch * H * W * C, FAKE, batch)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    B.ols_local_step(h)
    B.ols_local_step(h)
    B.ols_sync_pull(h)
    B.ols_anchor_update_async(h)
    one = ["conv_fwd", "conv_fwd", "pool", "head_fwd", "head_bwd", "pool_bwd", "conv_dx", "conv_dw", "conv_dw"]
    assert kinds(B.ols_trace(h)) == one + ["step"] + one + ["step_pull", "mean"]
    B.ols_destroy(h)


def test_convblock_with_batch_norm_attachment_and_launch_plan():
    C, H, W, classes, batch = 32, 8, 8, 10, 4
    d = 2 * (9 * C * C + 2 * C) + C * classes + classes
    h = dry(d=d, mu=0.9, tau=2)
    assert code_of(B.ols_attach_convblock, h, C, H, W, classes, batch) == B.OLS_EINVAL           # d is the normalised block's
    assert code_of(B.ols_attach_convblock_bn, h, C, H, W, classes, batch, 0.0) == B.OLS_EINVAL   # eps must be positive
    assert code_of(B.ols_attach_convblock_bn, h, C, H, W, classes, batch, float("nan")) == B.OLS_EINVAL
    assert code_of(B.ols_attach_convblock_bn, h, 24, H, W, classes, batch, 1e-5) == B.OLS_EINVAL
    B.ols_attach_convblock_bn(h, C, H, W, classes, batch, 1e-5)
    need = B.ols_workspace_bytes(h)
    assert need >= 6 * 4 * batch * H * W * C * 4        # activations, deltas and both convolution outputs, 4 workers
    B.ols_bind_workspace(h, FAKE, need)
    B.ols_init_params(h, FAKE)
    B.ols_set_batch(h, FAKE, batch * H * W * C, FAKE, batch)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    B.ols_local_step(h)
    B.ols_local_step(h)
    B.ols_sync_pull(h)
    B.ols_anchor_update_async(h)
    one = ["conv_fwd", "bn_fwd", "conv_fwd", "bn_fwd", "pool", "head_fwd", "head_bwd", "bn_bwd", "conv_dx",
           "conv_dw", "bn_bwd", "conv_dw"]
    assert kinds(B.ols_trace(h)) == one + ["step"] + one + ["step_pull", "mean"]
    B.ols_destroy(h)
    h = dry(d=d - 2 * C, mu=0.9, tau=2)                # the plain block needs two tensors less
    B.ols_attach_convblock(h, C, H, W, classes, batch)
    assert B.ols_workspace_bytes(h) <= need - 2 * 4 * batch * H * W * C * 4
    B.ols_destroy(h)


def test_convblock_bf16_attachment_and_launch_plan():
    C, H, W, classes, batch = 64, 8, 8, 10, 4
    d = 2 * (9 * C * C + C) + C * classes + classes
    h = dry(d=d, mu=0.9, tau=2)
    assert code_of(B.ols_attach_convblock_bf16, h, 32, H, W, classes, batch) == B.OLS_EINVAL     # channels not a multiple of 64
    assert code_of(B.ols_attach_convblock_bf16, h, C, H, 200, classes, batch) == B.OLS_EINVAL    # too wide
    B.ols_attach_convblock_bf16(h, C, H, W, classes, batch)
    need = B.ols_workspace_bytes(h)
    padded = 4 * batch * (H + 2) * (W + 2) * C
    assert need >= padded * (4 * 2 + 4) + 4 * (d + 63) // 64 * 64 * 2    # four bf16 tensors, one fp32, the bf16 parameters
    assert code_of(B.ols_init_params, h, FAKE) == B.OLS_ESTATE           # the workspace holds the bf16 parameters
    B.ols_bind_workspace(h, FAKE, need)
    B.ols_init_params(h, FAKE)
    assert code_of(B.ols_run_steps_static, h, 1, FAKE, FAKE, 1) == B.OLS_EINVAL
    B.ols_set_batch(h, FAKE, batch * H * W * C, FAKE, batch)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    B.ols_local_step(h)
    B.ols_local_step(h)
    B.ols_sync_pull(h)
    B.ols_anchor_update_async(h)
    one = ["cast_bf16", "conv_fwd", "conv_fwd", "pool", "head_fwd", "head_bwd", "pool_bwd", "conv_dx", "conv_dw", "conv_dw"]
    assert kinds(B.ols_trace(h)) == one + ["step"] + one + ["step_pull", "mean"]
    B.ols_destroy(h)
    h = dry(d=d)
    B.ols_attach_convblock(h, C, H, W, classes, batch)
    B.ols_bind_workspace(h, FAKE, B.ols_workspace_bytes(h))
    B.ols_init_params(h, FAKE)
    assert code_of(B.ols_attach_convblock_bf16, h, C, H, W, classes, batch) == B.OLS_ESTATE      # after ols_init_params
    B.ols_destroy(h)


def test_convblock_bn_bf16_attachment_and_launch_plan():
    C, H, W, classes, batch = 64, 8, 8, 10, 4
    d = 2 * (9 * C * C + 2 * C) + C * classes + classes
    h = dry(d=d, mu=0.9, tau=2)
    assert code_of(B.ols_attach_convblock_bn_bf16, h, 32, H, W, classes, batch, 1e-5) == B.OLS_EINVAL    # channels not a multiple of 64
    assert code_of(B.ols_attach_convblock_bn_bf16, h, C, H, W, classes, batch, 0.0) == B.OLS_EINVAL      # eps must be positive
    assert code_of(B.ols_attach_convblock_bf16, h, C, H, W, classes, batch) == B.OLS_EINVAL              # d is the normalised block's
    B.ols_attach_convblock_bn_bf16(h, C, H, W, classes, batch, 1e-5)
    need = B.ols_workspace_bytes(h)
    padded, plain = 4 * batch * (H + 2) * (W + 2) * C, 4 * batch * H * W * C
    # four bf16 operand tensors with a border, four fp32 tensors without one, the bf16 parameters
    assert need >= padded * 4 * 2 + plain * 4 * 4 + 4 * (d + 63) // 64 * 64 * 2
    assert code_of(B.ols_init_params, h, FAKE) == B.OLS_ESTATE           # the workspace holds the bf16 parameters
    B.ols_bind_workspace(h, FAKE, need)
    B.ols_init_params(h, FAKE)
    B.ols_set_batch(h, FAKE, batch * H * W * C, FAKE, batch)
    B.ols_set_option(h, B.OLS_OPT_TRACE, 1)
    B.ols_local_step(h)
    B.ols_local_step(h)
    B.ols_sync_pull(h)
    B.ols_anchor_update_async(h)
    one = ["cast_bf16", "conv_fwd", "bn_fwd", "conv_fwd", "bn_fwd", "pool", "head_fwd", "head_bwd", "bn_bwd", "conv_dx",
           "conv_dw", "bn_bwd", "conv_dw"]
    assert kinds(B.ols_trace(h)) == one + ["step"] + one + ["step_pull", "mean"]
    B.ols_destroy(h)


def test_tiny_refreshes_run_in_line_by_default():
    """OLS_OPT_SERIALIZE defaults to 2: the refresh is overlapped unless it moves at most 1 MiB."""
    for d, stream in ((100, 0), (100000, 1)):
        h = dry(m=4, d=d, tau=2)
        B.ols_set_option(h, B.OLS_OPT_SERIALIZE, 2)
        run_rounds(h, 2, 2)
        means = [t for t in B.ols_trace(h) if B.ols_kernel_name(t["kind"]) == "mean"]
        assert len(means) == 2 and all(t["stream"] == stream for t in means)
        B.ols_destroy(h)
    h = dry()
    assert code_of(B.ols_set_option, h, B.OLS_OPT_SERIALIZE, 3) == B.OLS_EINVAL
    B.ols_destroy(h)
