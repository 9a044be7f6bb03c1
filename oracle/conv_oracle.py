"""CPU oracle for the convolutional workload of Overlap Local-SGD.  TEST INFRASTRUCTURE ONLY.

The paper's experiments (Section 4, "Experimental setting") train ResNet-18 on CIFAR-10 with a mini-batch of 128
per node; the update rules of Section 2 are model-agnostic and live in ols_oracle.py.  This module supplies the
per-worker stochastic gradient g_i for the first residual stage of that network at CIFAR resolution, written out
from the definition of the operations, in double, with no blocking or fusion:

    a1     = relu(conv3x3(X;  Wa) + ba)
    a2     = relu(conv3x3(a1; Wb) + bb + X)           the residual ("basic") block, identity shortcut
    pooled = mean over the H x W positions of a2
    logits = pooled Wh + bh;   loss = mean over the batch of softmax cross-entropy

Readings (the paper names the architecture and nothing more): the block is the two-convolution residual block with
identity shortcut, 3 x 3 kernels, stride 1, zero padding 1, biases in place of batch normalisation (batch statistics
are not part of the data-parallel hot path this oracle serves); "convolution" is the cross-correlation every
deep-learning framework computes: out[y][x] = sum_{kh,kw} in[y + kh - 1][x + kw - 1] W[kh][kw]; the ReLU derivative
at 0 is 0; the loss is the mean over the mini-batch (as for the other models).

Layouts (an interface shared with the device path; each side computes its own offsets): activations are
[batch][height][width][channel]; the flat parameter vector holds Wa [3][3][C][C] (kh, kw, input channel, output
channel), ba [C], Wb [3][3][C][C], bb [C], Wh [C][classes], bh [classes], in that order.

Only tests/, the smoke check and the benchmark's CPU-baseline leg may import this module.
Pinned by tests/test_oracle_conv_pins.py: torch's CPU conv2d and autograd as library routines, a pure-Python
brute-force convolution, single-tap kernels that pin the tap orientation and the zero padding, central finite
differences of the whole loss, and planted mistakes that those pins must notice.
"""
import numpy as np

F64 = np.float64


def conv3x3_forward(inp, W, b):
    """out[n][y][x][co] = b[co] + sum_{kh,kw,ci} inp[n][y+kh-1][x+kw-1][ci] W[kh][kw][ci][co], zero outside the image."""
    inp, W, b = np.asarray(inp, F64), np.asarray(W, F64), np.asarray(b, F64)
    n, H, Wd, _ = inp.shape
    padded = np.zeros((n, H + 2, Wd + 2, inp.shape[3]), F64)
    padded[:, 1:H + 1, 1:Wd + 1, :] = inp
    out = np.zeros((n, H, Wd, W.shape[3]), F64) + b
    for kh in range(3):
        for kw in range(3):
            out += padded[:, kh:kh + H, kw:kw + Wd, :] @ W[kh, kw]
    return out


def conv3x3_backward(inp, W, dout):
    """Gradients of sum(out * dout) for out = conv3x3_forward(inp, W, b): (d_inp, d_W, d_b)."""
    inp, W, dout = np.asarray(inp, F64), np.asarray(W, F64), np.asarray(dout, F64)
    n, H, Wd, cin = inp.shape
    padded = np.zeros((n, H + 2, Wd + 2, cin), F64)
    padded[:, 1:H + 1, 1:Wd + 1, :] = inp
    d_padded = np.zeros_like(padded)
    dW = np.zeros_like(W)
    for kh in range(3):
        for kw in range(3):
            window = padded[:, kh:kh + H, kw:kw + Wd, :]
            dW[kh, kw] = window.reshape(-1, cin).T @ dout.reshape(-1, dout.shape[3])
            d_padded[:, kh:kh + H, kw:kw + Wd, :] += dout @ W[kh, kw].T
    return d_padded[:, 1:H + 1, 1:Wd + 1, :], dW, dout.sum(axis=(0, 1, 2))


def convblock_param_count(C, classes):
    return 2 * (9 * C * C + C) + C * classes + classes


def convblock_unpack(x, C, classes):
    """Views (Wa, ba, Wb, bb, Wh, bh) of the flat parameter vector."""
    out, off = [], 0
    for shape in ((3, 3, C, C), (C,), (3, 3, C, C), (C,), (C, classes), (classes,)):
        size = int(np.prod(shape))
        out.append(x[off:off + size].reshape(shape))
        off += size
    assert off == x.shape[0]
    return out


def convblock_loss_grad(x, C, classes, X, labels):
    """Residual block + pooled linear classifier: (mean cross-entropy over the batch, flat gradient in x's layout).
    X [B][H][W][C], labels [B]."""
    x = np.asarray(x, F64)
    X = np.asarray(X, F64)
    Wa, ba, Wb, bb, Wh, bh = convblock_unpack(x, C, classes)
    B = X.shape[0]
    a1 = np.maximum(conv3x3_forward(X, Wa, ba), 0.0)
    a2 = np.maximum(conv3x3_forward(a1, Wb, bb) + X, 0.0)
    pooled = a2.mean(axis=(1, 2))
    logits = pooled @ Wh + bh
    shifted = logits - logits.max(axis=1, keepdims=True)
    logsumexp = np.log(np.exp(shifted).sum(axis=1))
    rows = np.arange(B)
    loss = float((logsumexp - shifted[rows, labels]).mean())
    dlogits = np.exp(shifted - logsumexp[:, None])
    dlogits[rows, labels] -= 1.0
    dlogits /= B
    g = np.empty_like(x)
    gWa, gba, gWb, gbb, gWh, gbh = convblock_unpack(g, C, classes)
    gWh[...] = pooled.T @ dlogits
    gbh[...] = dlogits.sum(axis=0)
    d_pooled = dlogits @ Wh.T
    positions = X.shape[1] * X.shape[2]
    d_z2 = (d_pooled[:, None, None, :] / positions) * (a2 > 0.0)       # through the mean and the second ReLU
    d_a1, dWb, dbb = conv3x3_backward(a1, Wb, d_z2)
    gWb[...] = dWb
    gbb[...] = dbb
    d_z1 = d_a1 * (a1 > 0.0)
    _, dWa, dba = conv3x3_backward(X, Wa, d_z1)                         # the input is data: its gradient is not needed
    gWa[...] = dWa
    gba[...] = dba
    return loss, g
