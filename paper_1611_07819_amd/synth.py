"""Seeded synthetic inputs for the five benchmark configurations.

This module holds no arithmetic of the method: it only draws numbers and names shapes.  It is
the one module that both the GPU harness and the CPU oracle's tests use, so that both sides
see bit-identical inputs.

The paper trains AlexNet / GoogLeNet / Inception networks on an image data set that is not
available here (section 4).  The shapes below stand in for that workload: 9216->4096 and
4096->4096 are AlexNet's fully connected layers, batch 1024 is the paper's AlexNet batch
(section 4.1), the 256-channel 3x3 28x28 layer is a typical mid-network convolution;
uniform[0,1] stands in for post-ReLU activations and N(0, 1/fan_in) for initialised weights.

Every matrix is drawn monolithically from a Philox counter-based stream keyed by
(seed, matrix index), so its values do not depend on the block grid it is later cut into.
Values are drawn in fp64, rounded once to the storage type; those rounded host arrays are what
both sides receive.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 16110781

NP_DTYPE = {"f64": np.float64, "f32": np.float32, "f16": np.float16}


def _gen(seed: int, index: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(index)]))


def uniform(seed, index, shape, lo, hi, dtype):
    return _gen(seed, index).uniform(lo, hi, size=shape).astype(NP_DTYPE[dtype])


def normal(seed, index, shape, variance, dtype):
    return (_gen(seed, index).standard_normal(size=shape) * np.sqrt(variance)).astype(NP_DTYPE[dtype])


def small_ints(seed, index, shape, lo, hi, dtype):
    """Integers in [lo, hi]: sums of their products are exact in every precision used here,
    whatever the order of summation."""
    return _gen(seed, index).integers(lo, hi + 1, size=shape).astype(NP_DTYPE[dtype])


@dataclass
class GemmCall:
    name: str
    transA: bool
    transB: bool
    a: str            # key of the A operand in Workload.mats
    b: str
    c: str
    alpha: float = 1.0
    beta: float = 0.0

    def mnk(self, mats):
        A, B = mats[self.a], mats[self.b]
        M = A.shape[1] if self.transA else A.shape[0]
        K = A.shape[0] if self.transA else A.shape[1]
        N = B.shape[0] if self.transB else B.shape[1]
        return M, N, K


@dataclass
class Workload:
    name: str
    dtype: str                       # storage type of the inputs
    grid: tuple                      # block grid used for every matrix
    mats: dict                       # name -> host array (already rounded to its storage type)
    calls: list = field(default_factory=list)
    conv: dict | None = None         # convolution geometry for config 5
    seed: int = 0


def config1():
    """fp32 NN GEMM C = A*B + C, M=N=K=256, 2x2 grid of 128x128 blocks, uniform[-1,1]."""
    seed = BASE_SEED + 1
    mats = {n: uniform(seed, i, (256, 256), -1.0, 1.0, "f32") for i, n in enumerate("ABC")}
    return Workload("cfg1_f32_nn_256", "f32", (2, 2), mats,
                    [GemmCall("nn", False, False, "A", "B", "C", 1.0, 1.0)], seed=seed)


def config2(scale: int = 1):
    """fp32 fully connected layer forward + backward, X[1024x9216] W[9216x4096], 4x4 grid.
    ``scale`` > 1 divides every dimension (for quick parity runs)."""
    seed = BASE_SEED + 2
    b, i, o = 1024 // scale, 9216 // scale, 4096 // scale
    mats = {
        "X": uniform(seed, 0, (b, i), 0.0, 1.0, "f32"),
        "W": normal(seed, 1, (i, o), 1.0 / 9216, "f32"),
        "dY": normal(seed, 2, (b, o), 1e-2, "f32"),
        "Y": np.zeros((b, o), np.float32),
        "dW": np.zeros((i, o), np.float32),
        "dX": np.zeros((b, i), np.float32),
    }
    calls = [GemmCall("fwd_nn", False, False, "X", "W", "Y"),
             GemmCall("dW_tn", True, False, "X", "dY", "dW"),
             GemmCall("dX_nt", False, True, "dY", "W", "dX")]
    return Workload("cfg2_f32_fc_1024x9216x4096", "f32", (4, 4), mats, calls, seed=seed)


def config3(out_dtype: str = "f32", scale: int = 1):
    """fp16 inputs, fp32 accumulate, 4096x4096 layer at batch 2048, 8x8 grid."""
    seed = BASE_SEED + 3
    b, i, o = 2048 // scale, 4096 // scale, 4096 // scale
    od = NP_DTYPE[out_dtype]
    mats = {
        "X": uniform(seed, 0, (b, i), 0.0, 1.0, "f16"),
        "W": normal(seed, 1, (i, o), 1.0 / 4096, "f16"),
        "dY": normal(seed, 2, (b, o), 1e-2, "f16"),
        "Y": np.zeros((b, o), od),
        "dW": np.zeros((i, o), od),
        "dX": np.zeros((b, i), od),
    }
    calls = [GemmCall("fwd_nn", False, False, "X", "W", "Y"),
             GemmCall("dW_tn", True, False, "X", "dY", "dW"),
             GemmCall("dX_nt", False, True, "dY", "W", "dX")]
    return Workload(f"cfg3_f16_fc_2048x4096x4096_out{out_dtype}", "f16", (8, 8), mats, calls,
                    seed=seed)


def config4(scale: int = 1):
    """fp64 square GEMM 8192^3, 4x4 grid of 2048x2048 blocks, alpha=1.5 beta=-0.5."""
    seed = BASE_SEED + 4
    n = 8192 // scale
    mats = {nm: uniform(seed, i, (n, n), -1.0, 1.0, "f64") for i, nm in enumerate("ABC")}
    return Workload("cfg4_f64_nn_8192", "f64", (4, 4), mats,
                    [GemmCall("nn", False, False, "A", "B", "C", 1.5, -0.5)], seed=seed)


def config5(out_dtype: str = "f32", batch: int = 64, channels: int = 256, hw: int = 28):
    """fp16 3x3 stride-1 pad-1 convolution, NCHW batch 64, 256 -> 256 channels, 28x28,
    forward and weight gradient (dY ~ N(0,1e-2), the paper's configuration gives none)."""
    seed = BASE_SEED + 5
    od = NP_DTYPE[out_dtype]
    geom = dict(n=batch, c=channels, h=hw, w=hw, k=channels, r=3, s=3,
                pad_h=1, pad_w=1, stride_h=1, stride_w=1)
    chw = channels * hw * hw
    mats = {
        "X": uniform(seed, 0, (batch, chw), 0.0, 1.0, "f16"),
        "F": normal(seed, 1, (channels, channels * 9), 1.0 / 2304, "f16"),
        "dY": normal(seed, 2, (batch, chw), 1e-2, "f16"),
        "Y": np.zeros((batch, chw), od),
        "dF": np.zeros((channels, channels * 9), od),
    }
    return Workload(f"cfg5_f16_conv3x3_{batch}x{channels}x{hw}x{hw}_out{out_dtype}", "f16",
                    (1, 1), mats, [], conv=geom, seed=seed)
