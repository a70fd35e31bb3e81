"""Seeded synthetic inputs for the five benchmark configurations.

This module holds no arithmetic of the method itself: it only draws the input
arrays (numpy ``default_rng(seed)``, draws in the order listed, cast to FP32,
C-contiguous row-major) so that the FP64 CPU oracle and the HIP library read
identical bytes.  The shapes stand in for the workloads of the dMath paper
(arXiv 1604.01416): square local blocks of a block-distributed matrix (table
"Matrix Multiplication Performance"), the 4096-wide fully connected layers at
batch 256 of its strong-scaling experiment, and a 3x3 convolution layer.

Normal distributions are given by their standard deviation.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np


def _uniform(rng, shape):
    return rng.uniform(-1.0, 1.0, shape).astype(np.float32)


def _normal(rng, shape, sigma=1.0):
    return (sigma * rng.standard_normal(shape)).astype(np.float32)


def _relu_normal(rng, shape):
    return np.maximum(rng.standard_normal(shape), 0.0).astype(np.float32)


@dataclass
class GemmCall:
    """One dmath_gemm call: names index into ``GemmWorkload.arrays``."""
    transA: int
    transB: int
    M: int
    N: int
    K: int
    alpha: float
    A: str
    lda: int
    B: str
    ldb: int
    beta: float
    C: str
    ldc: int

    @property
    def flop(self) -> int:
        return 2 * self.M * self.N * self.K

    @property
    def algorithmic_bytes(self) -> int:
        """A and B read once, C written once (and read once when beta != 0)."""
        c_passes = 2 if self.beta != 0.0 else 1
        return 4 * (self.M * self.K + self.K * self.N + c_passes * self.M * self.N)


@dataclass
class GemmWorkload:
    name: str
    arrays: Dict[str, np.ndarray]
    calls: List[GemmCall]
    # Names of arrays that calls write (they must exist; zeros unless stated).
    outputs: List[str] = field(default_factory=list)

    @property
    def flop(self) -> int:
        return sum(c.flop for c in self.calls)


def gemm_square(n: int, seed: int, name: str) -> GemmWorkload:
    """C = A*B, NN, M=N=K=n, alpha=1, beta=0, A and B uniform[-1,1]."""
    rng = np.random.default_rng(seed)
    A = _uniform(rng, (n, n))
    B = _uniform(rng, (n, n))
    C = np.zeros((n, n), dtype=np.float32)
    call = GemmCall(0, 0, n, n, n, 1.0, "A", n, "B", n, 0.0, "C", n)
    return GemmWorkload(name, {"A": A, "B": B, "C": C}, [call], ["C"])


def config1() -> GemmWorkload:
    return gemm_square(256, 0, "gemm_nn_256")


def config2(n: int = 4096) -> GemmWorkload:
    return gemm_square(n, 1, "gemm_nn_%d" % n)


def config3(m: int = 8192, kp: int = 512, steps: int = 16, seed: int = 2) -> GemmWorkload:
    """Local update sequence of one worker: C += A_k * B_k for k = 0..steps-1.

    C is m x m drawn N(0,1); each A_k is m x kp and each B_k is kp x m, uniform[-1,1].
    """
    rng = np.random.default_rng(seed)
    arrays = {"C": _normal(rng, (m, m))}
    calls = []
    for k in range(steps):
        arrays["A%d" % k] = _uniform(rng, (m, kp))
        arrays["B%d" % k] = _uniform(rng, (kp, m))
        calls.append(GemmCall(0, 0, m, m, kp, 1.0, "A%d" % k, kp, "B%d" % k, m, 1.0, "C", m))
    return GemmWorkload("summa_update_%dx%dx%d_x%d" % (m, m, kp, steps), arrays, calls, ["C"])


def config4(batch: int = 256, width: int = 4096, seed: int = 3) -> GemmWorkload:
    """Fully connected layer: Y = X*W (NN), dX = dY*W^T (NT), dW = X^T*dY (TN)."""
    rng = np.random.default_rng(seed)
    X = _relu_normal(rng, (batch, width))
    W = _normal(rng, (width, width), 0.01)
    dY = _normal(rng, (batch, width), 1e-3)
    arrays = {
        "X": X, "W": W, "dY": dY,
        "Y": np.zeros((batch, width), dtype=np.float32),
        "dX": np.zeros((batch, width), dtype=np.float32),
        "dW": np.zeros((width, width), dtype=np.float32),
    }
    calls = [
        GemmCall(0, 0, batch, width, width, 1.0, "X", width, "W", width, 0.0, "Y", width),
        GemmCall(0, 1, batch, width, width, 1.0, "dY", width, "W", width, 0.0, "dX", width),
        GemmCall(1, 0, width, width, batch, 1.0, "X", width, "dY", width, 0.0, "dW", width),
    ]
    return GemmWorkload("fc_%d_batch%d" % (width, batch), arrays, calls, ["Y", "dX", "dW"])


@dataclass
class ConvWorkload:
    name: str
    x: np.ndarray          # N x C x H x W
    w: np.ndarray          # Kout x C x R x S
    pad: Tuple[int, int]
    stride: Tuple[int, int]
    alpha: float = 1.0
    beta: float = 0.0

    @property
    def out_shape(self) -> Tuple[int, int, int, int]:
        N, C, H, W = self.x.shape
        Kout, _, R, S = self.w.shape
        P = (H + 2 * self.pad[0] - R) // self.stride[0] + 1
        Q = (W + 2 * self.pad[1] - S) // self.stride[1] + 1
        return N, Kout, P, Q

    @property
    def gemm_view(self) -> Tuple[int, int, int]:
        """(M, N, K) of the equivalent matrix product."""
        N, Kout, P, Q = self.out_shape
        _, C, R, S = self.w.shape
        return N * P * Q, Kout, C * R * S

    @property
    def flop(self) -> int:
        M, N, K = self.gemm_view
        return 2 * M * N * K

    @property
    def algorithmic_bytes(self) -> int:
        """x, w read once and y written once; the unfolded matrix is never stored."""
        n_out = int(np.prod(self.out_shape))
        return 4 * (self.x.size + self.w.size + n_out)


def config5(batch: int = 128, channels: int = 256, kout: int = 256, hw: int = 28,
            seed: int = 4) -> ConvWorkload:
    """3x3 convolution forward, stride 1, pad 1; x = ReLU(N(0,1)), w ~ N(0, sqrt(2/fan_in))."""
    rng = np.random.default_rng(seed)
    x = _relu_normal(rng, (batch, channels, hw, hw))
    fan_in = channels * 9
    w = _normal(rng, (kout, channels, 3, 3), float(np.sqrt(2.0 / fan_in)))
    return ConvWorkload("conv3x3_n%d_c%d_k%d_%dx%d" % (batch, channels, kout, hw, hw), x, w, (1, 1), (1, 1))


def small_ints(rng, shape, lo=-4, hi=4):
    """Integer-valued FP32 entries in [lo, hi]: every FP32 summation order is exact."""
    return rng.integers(lo, hi + 1, size=shape).astype(np.float32)
