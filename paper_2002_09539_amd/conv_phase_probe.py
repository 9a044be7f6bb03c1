"""Where a tile of the bf16 forward / delta convolution kernel spends its time.

Needs a measurement build of the library with the kernel's timestamp points compiled in:

    OLS_EXTRA_FLAGS=-DOLS_CONV_PHASE_PROBE OLS_BUILD_DIR=/tmp/ols_probe_build OLS_BUILD_OUTPUT=/tmp/libols_probe.so \\
        python -m paper_2002_09539_amd.build
    OLS_LIBRARY=/tmp/libols_probe.so python -m paper_2002_09539_amd.conv_phase_probe [--config 8]

Runs a few steps of the configuration, reads the s_memrealtime (100 MHz) readings that lane 0 of every workgroup of
the last launch of each kernel left, and prints the mean time between the points and how long a compute unit's two
workgroups were resident together.  The product build contains none of this.
"""
import argparse
import ctypes

import numpy as np

import ols_inputs as I
from ols_inputs import generate as G

from . import binding as B
from .session import Session

POINTS = ["tile known -> loads issued", "loads issued -> strip in LDS", "nine taps", "epilogue (taps done -> stores issued)"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=8, help="8: plain block with bf16 operands; 9: the normalised one")
    ap.add_argument("--steps", type=int, default=4)
    args = ap.parse_args()
    lib = B.load()
    if not hasattr(lib, "ols_debug_conv_phases"):
        raise SystemExit("this library was built without -DOLS_CONV_PHASE_PROBE (see the module's docstring)")
    cfg = I.get(args.config)
    X, labels = G.conv_data(cfg)
    x0 = G.conv_init(cfg)
    C, H, W, _ = cfg.dims
    tiles = cfg.m * (-(-(cfg.batch * (H + 2) * (W + 2)) // 256)) * (C // 64)
    with Session(cfg.m, cfg.d, cfg.tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
        s.attach_convblock(*cfg.dims, cfg.batch, batch_norm=cfg.batch_norm, gemm_dtype=cfg.gemm_dtype)
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        s.run_resident(args.steps, Xd, yd)
        s.sync()
        buf = np.zeros((3, tiles, 8), dtype=np.uint64)
        rc = lib.ols_debug_conv_phases(buf.ctypes.data_as(ctypes.POINTER(ctypes.c_ulonglong)), tiles)
        if rc != 0:
            raise SystemExit("ols_debug_conv_phases failed: %d" % rc)
    print("%s: %d tiles of 256 padded pixels x 64 channels per launch; times in microseconds, means over the tiles of the "
          "last launch" % (cfg.name, tiles))
    for k, name in enumerate(("forward, bf16 output", "forward, other output (fused tail / fp32)", "delta")):
        t = buf[k].astype(np.float64) / 100.0
        if not t[:, 0].any():
            continue
        d = np.diff(t[:, :5], axis=1)
        wall = t[:, 4].max() - t[:, 0].min()
        print("%s: first tile start to last tile end %.1f us" % (name, wall))
        for j, label in enumerate(POINTS):
            print("    %-40s %6.2f" % (label, d[:, j].mean()))
        print("    %-40s %6.2f   (%.1f tiles resident per compute unit on average)"
              % ("whole tile", (t[:, 4] - t[:, 0]).mean(), (t[:, 4] - t[:, 0]).sum() / wall / 256))


if __name__ == "__main__":
    main()
