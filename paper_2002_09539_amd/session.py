"""Device memory and streams for one Overlap Local-SGD run, handed to libols through the C boundary.

PyTorch is used here only as the allocator of HBM buffers and the owner of the two HIP streams; every
computation happens inside libols' kernels (see include/ols.h).  The class keeps the tensors alive for
as long as the handle uses them and forwards each call to the binding one-to-one.
"""
import numpy as np
import torch

from . import binding as B


def _ptr(t):
    return None if t is None else t.data_ptr()


class Session:
    def __init__(self, m, d, tau, alpha, gamma, mu, overlap_buffer=True, device="cuda:0", own_gradient=True):
        if not torch.cuda.is_available():
            raise B.OlsError(B.OLS_EHIP, "no GPU visible: the Overlap Local-SGD path has no CPU fallback")
        self.m, self.d, self.tau = m, d, tau
        self.device = torch.device(device)
        self.h = B.ols_create(m, d, tau, alpha, gamma, mu)
        self.ld = B.ols_row_stride(d)
        z = lambda *shape: torch.zeros(*shape, dtype=torch.float32, device=self.device)
        self.x = z(m, self.ld)
        self.x_alt = z(m, self.ld) if overlap_buffer else None
        self.buf = z(m, self.ld) if mu != 0.0 else None
        self.g = z(m, self.ld) if own_gradient else None
        self.z = z(self.ld)
        self.v = None
        self.ws = None
        self.main = torch.cuda.Stream(device=self.device)
        self.side = torch.cuda.Stream(device=self.device)
        self._keep = []
        torch.cuda.synchronize(self.device)   # the zero fills ran on torch's own stream
        if own_gradient:
            self.bind()

    def bind(self, g=None):
        if g is not None:
            self.g = g
        B.ols_bind(self.h, _ptr(self.x), _ptr(self.x_alt), _ptr(self.buf), _ptr(self.g), _ptr(self.z), self.ld,
                   self.main.cuda_stream, self.side.cuda_stream)

    # ---- configuration -----------------------------------------------------------------------
    def set_option(self, key, value):
        B.ols_set_option(self.h, key, int(value))

    def set_lr(self, gamma):
        """Learning rate of the local steps from now on (not while a deferred step waits for ols_sync_pull)."""
        B.ols_set_lr(self.h, float(gamma))

    def set_anchor_momentum(self, beta_z):
        self.v = torch.zeros(self.ld, dtype=torch.float32, device=self.device) if beta_z != 0.0 else None
        torch.cuda.synchronize(self.device)
        B.ols_set_anchor_momentum(self.h, beta_z, _ptr(self.v))

    def set_mixing(self, W):
        """General mixing X <- X W at every synchronisation point; W: (m+1) x (m+1) host array, or None."""
        if W is None:
            B.ols_set_mixing(self.h, None)
            self.w = None
            return
        W = np.ascontiguousarray(W, dtype=np.float32)
        assert W.shape == (self.m + 1, self.m + 1)
        self.w = self.upload(W)
        B.ols_set_mixing(self.h, _ptr(self.w))

    def set_stale_average(self, on=True):
        """Stale-average synchronisation in place of pull-back + anchor average (after init, before the first step)."""
        self.snap = torch.empty_like(self.x) if on else None
        torch.cuda.synchronize(self.device)
        B.ols_set_stale_average(self.h, _ptr(self.snap))

    def attach_lsq(self, batch):
        B.ols_attach_lsq(self.h, batch)
        self._workspace()

    def attach_mlp(self, dims, batch, gemm_dtype="f32", workspace=True):
        """workspace=False leaves the model without a bound workspace (for run_resident_static)."""
        B.ols_attach_mlp(self.h, list(dims), batch, {"f32": 0, "bf16": 1}[gemm_dtype])
        if workspace:
            self._workspace()

    def attach_convblock(self, channels, height, width, classes, batch, batch_norm=False, eps=1e-5, gemm_dtype="f32"):
        if gemm_dtype == "bf16" and batch_norm:
            B.ols_attach_convblock_bn_bf16(self.h, channels, height, width, classes, batch, eps)
        elif gemm_dtype == "bf16":
            B.ols_attach_convblock_bf16(self.h, channels, height, width, classes, batch)
        elif batch_norm:
            B.ols_attach_convblock_bn(self.h, channels, height, width, classes, batch, eps)
        else:
            B.ols_attach_convblock(self.h, channels, height, width, classes, batch)
        self._workspace()

    def _workspace(self):
        n = B.ols_workspace_bytes(self.h)
        self.ws = torch.zeros(max(n, 256), dtype=torch.uint8, device=self.device)
        torch.cuda.synchronize(self.device)
        B.ols_bind_workspace(self.h, _ptr(self.ws), self.ws.numel())

    def upload(self, array, dtype=None):
        """Host array -> device tensor (kept alive by the session)."""
        t = torch.as_tensor(np.ascontiguousarray(array))
        if dtype is not None:
            t = t.to(dtype)
        t = t.to(self.device)
        torch.cuda.synchronize(self.device)
        self._keep.append(t)
        return t

    def init_params(self, x0):
        t = x0 if torch.is_tensor(x0) else self.upload(np.asarray(x0, dtype=np.float32))
        assert t.dtype == torch.float32 and t.numel() >= self.d
        B.ols_init_params(self.h, _ptr(t))

    # ---- the iteration -----------------------------------------------------------------------
    def set_batch(self, X, y):
        """X: device [m][B][in] fp32 (worker axis may be strided), y: device [m][B] int32 / fp32."""
        assert X[0].is_contiguous() and y.stride(-1) == 1
        B.ols_set_batch(self.h, _ptr(X), X.stride(0) if self.m > 1 else X[0].numel(), _ptr(y),
                        y.stride(0) if self.m > 1 else y[0].numel())

    def set_gradient(self, g):
        assert g.is_contiguous() and tuple(g.shape) == (self.m, self.ld) and g.dtype == torch.float32
        B.ols_set_gradient(self.h, _ptr(g))

    def local_step(self):
        B.ols_local_step(self.h)

    def sync_pull(self):
        B.ols_sync_pull(self.h)

    def anchor_update_async(self):
        B.ols_anchor_update_async(self.h)

    def sync(self):
        B.ols_sync(self.h)

    def run(self, K, before_step=None, losses=None):
        """K iterations in the paper's order; before_step(k) binds that iteration's inputs."""
        for _ in range(K):
            k = B.ols_iteration(self.h)
            if before_step is not None:
                before_step(k)
            B.ols_local_step(self.h)
            if losses is not None:
                losses.append(self.losses())
            if (k + 1) % self.tau == 0:
                B.ols_sync_pull(self.h)
                B.ols_anchor_update_async(self.h)

    def run_resident(self, K, X, y):
        """K iterations over a resident data set X: device [m][nb][B][in] fp32, y: device [m][nb][B], batch
        k mod nb at iteration k; the loop runs inside the library (ols_run_steps)."""
        assert X.is_contiguous() and y.is_contiguous() and X.shape[:2] == y.shape[:2] and X.dtype == torch.float32
        B.ols_run_steps(self.h, K, _ptr(X), _ptr(y), X.shape[1])

    def run_resident_static(self, K, X, y):
        """run_resident with the model's workspace in the library's static device array (ols_run_steps_static)."""
        assert X.is_contiguous() and y.is_contiguous() and X.shape[:2] == y.shape[:2] and X.dtype == torch.float32
        B.ols_run_steps_static(self.h, K, _ptr(X), _ptr(y), X.shape[1])

    # ---- results -----------------------------------------------------------------------------
    def params(self, which):
        out = np.empty(self.d, dtype=np.float32)
        B.ols_get_params(self.h, which, out.ctypes.data, 0)
        return out

    def all_params(self):
        return np.stack([self.params(i) for i in range(self.m)])

    def replica_mean(self):
        t = torch.zeros(self.ld, dtype=torch.float32, device=self.device)
        torch.cuda.synchronize(self.device)
        B.ols_get_params(self.h, -2, _ptr(t), 1)
        return t[: self.d].cpu().numpy()

    def momentum(self):
        self.sync()
        return None if self.buf is None else self.buf[:, : self.d].cpu().numpy()

    def gradient(self):
        self.sync()
        return self.g[:, : self.d].cpu().numpy()

    def losses(self):
        return np.array(B.ols_get_loss(self.h, self.m), dtype=np.float64)

    def kernel_stats(self):
        out = {}
        for kind in range(B.OLS_K_COUNT):
            n, ms = B.ols_kernel_stats(self.h, kind)
            if n:
                out[B.ols_kernel_name(kind)] = (n, ms)
        return out

    def close(self):
        if self.h:
            B.ols_destroy(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
