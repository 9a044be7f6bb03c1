"""Workload descriptions for the five Overlap Local-SGD configurations.

Pure data: the hyper-parameters of each configuration (worker count m, model
shape, batch size, tau, alpha, gamma, local momentum mu, iteration count K) and
the recipe constants of the synthetic inputs.  Nothing of the method's
arithmetic lives here; both the CPU oracle's tests and the HIP path's tests /
benchmark read these records and then do their own computation.

Hyper-parameter names follow the paper's Section 2 notation: gamma = learning
rate, alpha = pull-back strength, tau = local steps per round, m = workers.
`mu` is the local (per-worker) momentum factor, which the paper uses but does
not name; the paper's beta is the anchor momentum factor (`beta_z` here).
"""
from dataclasses import dataclass, field, replace
from typing import Optional, Tuple

BASE_SEED = 20200209


@dataclass(frozen=True)
class Config:
    name: str
    kind: str                      # "lsq" | "mlp" | "stream" | "conv"
    m: int
    tau: int
    alpha: float
    gamma: float
    mu: float
    K: int                         # local iterations per worker
    batch: int = 0
    dims: Tuple[int, ...] = ()     # MLP layer widths, input first; conv: (channels, height, width, classes)
    d_flat: int = 0                # lsq / stream: parameter count
    nb: int = 0                    # fixed, unshuffled batches per worker (cycled)
    gemm_dtype: str = "f32"        # "f32" | "bf16"
    noniid_classes: int = 0        # >0: each worker's labels come from this many classes
    n_classes: int = 10
    grad_sigma: float = 0.1        # stream: gradients ~ N(0, sigma^2)
    grad_pool: int = 2             # stream: number of distinct gradient tensors cycled
    seed: int = BASE_SEED
    beta_z: float = 0.0            # anchor momentum (0 = plain anchor average)
    nesterov: bool = True
    batch_norm: bool = False       # conv: convolutions without bias, each followed by batch normalisation

    @property
    def d(self) -> int:
        if self.kind == "mlp":
            return sum(self.dims[l] * self.dims[l + 1] + self.dims[l + 1]
                       for l in range(len(self.dims) - 1))
        if self.kind == "conv":    # two 3x3 kernels with biases (or scale + shift), then the pooled linear classifier
            c, _, _, classes = self.dims
            return 2 * (9 * c * c + (2 * c if self.batch_norm else c)) + c * classes + classes
        return self.d_flat

    @property
    def rounds(self) -> int:
        return self.K // self.tau

    def scaled(self, **kw) -> "Config":
        """A copy with some fields replaced (used for small parity cases)."""
        return replace(self, **kw)


# Section 4 of the paper fixes batch 128 per node, 16 nodes, alpha = 0.6 for
# tau >= 2; the remaining numbers are the configurations' own.
CONFIGS = {
    1: Config(name="cfg1_lsq_m4", kind="lsq", m=4, tau=2, alpha=0.6, gamma=0.01,
              mu=0.0, K=50, batch=32, d_flat=1024, nb=50),
    2: Config(name="cfg2_mlp_f32_m16", kind="mlp", m=16, tau=2, alpha=0.6, gamma=0.05,
              mu=0.9, K=200, batch=128, dims=(3072, 512, 10), nb=24),
    3: Config(name="cfg3_mlp_bf16_m16", kind="mlp", m=16, tau=4, alpha=0.5, gamma=0.05,
              mu=0.9, K=200, batch=256, dims=(3072, 2048, 2048, 2048, 10), nb=12,
              gemm_dtype="bf16"),
    4: Config(name="cfg4_stream_m16", kind="stream", m=16, tau=2, alpha=0.6, gamma=0.1,
              mu=0.9, K=200, d_flat=11_200_000),
    5: Config(name="cfg5_mlp_noniid_m64", kind="mlp", m=64, tau=8, alpha=0.5, gamma=0.05,
              mu=0.9, K=400, batch=64, dims=(3072, 1024, 10), nb=12, noniid_classes=2),
    # Beyond the five benchmark configurations: the convolutional workload of Section 4's setting (ResNet-18 on
    # 32 x 32 inputs, 16 nodes, batch 128 per node): the network's first residual stage, 64 channels.
    6: Config(name="cfg6_convblock_m16", kind="conv", m=16, tau=2, alpha=0.6, gamma=0.05,
              mu=0.9, K=100, batch=128, dims=(64, 32, 32, 10), nb=2),
    # the same stage as the residual network has it: batch normalisation after each convolution, no biases
    7: Config(name="cfg7_convblock_bn_m16", kind="conv", m=16, tau=2, alpha=0.6, gamma=0.05,
              mu=0.9, K=100, batch=128, dims=(64, 32, 32, 10), nb=2, batch_norm=True),
    # configuration 6 with bf16 operands in the convolutions (fp32 accumulation, fp32 master parameters)
    8: Config(name="cfg8_convblock_bf16_m16", kind="conv", m=16, tau=2, alpha=0.6, gamma=0.05,
              mu=0.9, K=100, batch=128, dims=(64, 32, 32, 10), nb=2, gemm_dtype="bf16"),
    # configuration 7 with bf16 operands in the convolutions: the residual network's own stage at matrix-core speed
    9: Config(name="cfg9_convblock_bn_bf16_m16", kind="conv", m=16, tau=2, alpha=0.6, gamma=0.05,
              mu=0.9, K=100, batch=128, dims=(64, 32, 32, 10), nb=2, batch_norm=True, gemm_dtype="bf16"),
}


def get(idx: int) -> Config:
    return CONFIGS[idx]
