"""Seeded synthetic inputs shared (as DATA) by the CPU oracle and the HIP path.

Every tensor is drawn from a Philox counter-based stream keyed by
(seed, tag, worker, index), so any tensor can be regenerated on its own.  The
shapes stand in for the CIFAR-10 workload of the paper's Section 4 (3x32x32 =
3072 features, 10 classes, batch 128 per node, 16 nodes, data partitioned per
node and never shuffled); the real dataset is not used anywhere.

This module performs none of the method's arithmetic (no gradients, no
updates): it only produces random draws and the affine combinations the data
recipe itself states (y = A w* + noise; sample = noise + class mean).

Flat parameter layout of an MLP with widths dims[0..L]: for each layer l in
order, the weight matrix W_l stored row-major as [dims[l]][dims[l+1]]
(input index slow, output index fast) followed by the bias b_l [dims[l+1]].
"""
import numpy as np

from .configs import Config

TAG_W_STAR = 1
TAG_LSQ_A = 2
TAG_LSQ_NOISE = 3
TAG_CLASS_MEANS = 4
TAG_MLP_X = 5
TAG_MLP_LABELS = 6
TAG_MLP_INIT = 7
TAG_STREAM_G = 8
TAG_STREAM_X0 = 9
TAG_NONIID = 10
TAG_GENERIC = 11
TAG_CONV_X = 12
TAG_CONV_MEANS = 13
TAG_CONV_LABELS = 14
TAG_CONV_INIT = 15


def rng(seed: int, tag: int, worker: int = 0, index: int = 0) -> np.random.Generator:
    """Independent Philox stream for one tensor."""
    key = np.array([np.uint64(seed), np.uint64((tag << 48) | (worker << 24) | index)],
                   dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def normal_f32(seed, tag, worker, index, shape, sigma=1.0):
    out = rng(seed, tag, worker, index).standard_normal(shape, dtype=np.float32)
    if sigma != 1.0:
        out *= np.float32(sigma)
    return out


# ----------------------------------------------------------------------------
# configuration 1: linear least squares
# ----------------------------------------------------------------------------
def lsq_data(cfg: Config):
    """A [m][nb][B][d] fp32, y [m][nb][B] fp32, w_star [d] fp32, x0 [d] fp32 (zeros).

    w* ~ N(0, I/d); rows of A ~ N(0, I); y = A w* + 0.1 N(0,1), evaluated in
    fp64 from the fp32 A and w* and rounded once.
    """
    d, B, m, nb = cfg.d, cfg.batch, cfg.m, cfg.nb
    w_star = normal_f32(cfg.seed, TAG_W_STAR, 0, 0, (d,), sigma=1.0 / np.sqrt(d))
    A = np.empty((m, nb, B, d), dtype=np.float32)
    y = np.empty((m, nb, B), dtype=np.float32)
    for i in range(m):
        for j in range(nb):
            A[i, j] = normal_f32(cfg.seed, TAG_LSQ_A, i, j, (B, d))
            noise = normal_f32(cfg.seed, TAG_LSQ_NOISE, i, j, (B,), sigma=0.1)
            y[i, j] = (A[i, j].astype(np.float64) @ w_star.astype(np.float64)
                       + noise.astype(np.float64)).astype(np.float32)
    x0 = np.zeros(d, dtype=np.float32)
    return A, y, w_star, x0


# ----------------------------------------------------------------------------
# configurations 2, 3, 5: CIFAR-10-shaped classification
# ----------------------------------------------------------------------------
def worker_classes(cfg: Config):
    """[m][c] int: the classes worker i draws labels from (all of them when IID)."""
    if cfg.noniid_classes <= 0:
        return np.tile(np.arange(cfg.n_classes), (cfg.m, 1))
    out = np.empty((cfg.m, cfg.noniid_classes), dtype=np.int64)
    for i in range(cfg.m):
        out[i] = rng(cfg.seed, TAG_NONIID, i, 0).choice(
            cfg.n_classes, size=cfg.noniid_classes, replace=False)
    return out


def mlp_data(cfg: Config, workers=None, nb=None):
    """X [m][nb][B][in] fp32 and labels [m][nb][B] int32.

    sample = N(0, I) + mean[label]; the 10 class means are 0.5 * N(0, I), drawn
    once; labels are uniform over the worker's class set.
    """
    n_in, B = cfg.dims[0], cfg.batch
    nb = cfg.nb if nb is None else nb
    workers = range(cfg.m) if workers is None else workers
    means = normal_f32(cfg.seed, TAG_CLASS_MEANS, 0, 0, (cfg.n_classes, n_in), sigma=0.5)
    classes = worker_classes(cfg)
    X = np.empty((len(workers), nb, B, n_in), dtype=np.float32)
    labels = np.empty((len(workers), nb, B), dtype=np.int32)
    for wi, i in enumerate(workers):
        for j in range(nb):
            pick = rng(cfg.seed, TAG_MLP_LABELS, i, j).integers(0, classes.shape[1], size=B)
            lab = classes[i][pick].astype(np.int32)
            labels[wi, j] = lab
            X[wi, j] = normal_f32(cfg.seed, TAG_MLP_X, i, j, (B, n_in))
            X[wi, j] += means[lab]
    return X, labels


def mlp_init(cfg: Config):
    """Common starting point x0 [d] fp32: weights N(0, 1/fan_in), biases zero."""
    parts = []
    for l in range(len(cfg.dims) - 1):
        fan_in, fan_out = cfg.dims[l], cfg.dims[l + 1]
        parts.append(normal_f32(cfg.seed, TAG_MLP_INIT, 0, l, (fan_in * fan_out,),
                                sigma=1.0 / np.sqrt(fan_in)))
        parts.append(np.zeros(fan_out, dtype=np.float32))
    return np.concatenate(parts)


# ----------------------------------------------------------------------------
# convolutional workload: feature maps [B][H][W][C] entering the first residual stage
# ----------------------------------------------------------------------------
def conv_data(cfg: Config, workers=None, nb=None):
    """X [m][nb][B][H][W][C] fp32 and labels [m][nb][B] int32.

    Same data law as the MLP configurations at the block's input shape: sample = N(0, I) + mean[label], class means
    0.5 * N(0, I) drawn once, labels uniform over the classes; fixed batches per worker, never shuffled.
    """
    C, H, W, classes = cfg.dims
    B = cfg.batch
    nb = cfg.nb if nb is None else nb
    workers = range(cfg.m) if workers is None else workers
    means = normal_f32(cfg.seed, TAG_CONV_MEANS, 0, 0, (classes, H, W, C), sigma=0.5)
    X = np.empty((len(workers), nb, B, H, W, C), dtype=np.float32)
    labels = np.empty((len(workers), nb, B), dtype=np.int32)
    for wi, i in enumerate(workers):
        for j in range(nb):
            lab = rng(cfg.seed, TAG_CONV_LABELS, i, j).integers(0, classes, size=B).astype(np.int32)
            labels[wi, j] = lab
            X[wi, j] = normal_f32(cfg.seed, TAG_CONV_X, i, j, (B, H, W, C))
            X[wi, j] += means[lab]
    return X, labels


def conv_init(cfg: Config):
    """Common starting point x0 [d] fp32 in the block's flat layout (Wa, ba, Wb, bb, Wh, bh): kernels N(0, 1/fan_in)
    with fan_in = 9 C, classifier N(0, 1/C), biases zero.  With batch normalisation (Wa, ga, ba, Wb, gb, bb, Wh, bh)
    the scales start at one and the shifts at zero."""
    C, _, _, classes = cfg.dims
    parts = []
    for l, (count, fan_in, bias) in enumerate(((9 * C * C, 9 * C, C), (9 * C * C, 9 * C, C), (C * classes, C, classes))):
        parts.append(normal_f32(cfg.seed, TAG_CONV_INIT, 0, l, (count,), sigma=1.0 / np.sqrt(fan_in)))
        if cfg.batch_norm and l < 2:
            parts.append(np.ones(C, dtype=np.float32))
        parts.append(np.zeros(bias, dtype=np.float32))
    return np.concatenate(parts)


# ----------------------------------------------------------------------------
# configuration 4: update-only stream
# ----------------------------------------------------------------------------
def stream_x0(cfg: Config, d=None):
    d = cfg.d if d is None else d
    return normal_f32(cfg.seed, TAG_STREAM_X0, 0, 0, (d,), sigma=cfg.grad_sigma)


def stream_gradient(cfg: Config, index: int, d=None, m=None):
    """One [m][d] fp32 gradient tensor ~ N(0, sigma^2), sigma^2 = 1e-2."""
    d = cfg.d if d is None else d
    m = cfg.m if m is None else m
    out = np.empty((m, d), dtype=np.float32)
    for i in range(m):
        out[i] = normal_f32(cfg.seed, TAG_STREAM_G, i, index, (d,), sigma=cfg.grad_sigma)
    return out


def generic_normal(seed: int, index: int, shape, sigma=1.0):
    """Free-form seeded normal tensor for unit-level parity cases."""
    return normal_f32(seed, TAG_GENERIC, 0, index, shape, sigma=sigma)
