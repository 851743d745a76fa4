"""Seeded synthetic inputs for the low-bit GEMM workloads.

This module only draws random matrices; it contains none of the method's
arithmetic (no packing, no products).  Both the CPU oracle's tests and the
HIP path's tests/benchmark take their inputs from here so that the two sides
see the very same bytes.

The paper (Section IV-B) measures on a grid of matrix shapes whose contents it
does not specify and uses no dataset or trained weights; the workloads below
are conv (im2col) and fully connected shaped matrices with i.i.d. entries that
stand in for such layers.

Recipe (fixed once; changing it changes every stored expectation):
  rng = numpy.random.default_rng(seed)
  every matrix is drawn, in the order listed by the workload, as
      u = rng.integers(0, 100, size=shape, dtype=uint8)
  ternary with zero probability p0 (p0*100 an integer, (100 - p0*100) even):
      u <  100*p0                      ->  0
      100*p0 <= u < 100*p0 + h         -> +1      (h = (100 - 100*p0) / 2)
      otherwise                        -> -1
  binary:  u < 50 -> +1, else -1
All matrices are C-contiguous int8: A is M x K, B is K x N (both row-major).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np


def _lut_ternary(p0: float) -> np.ndarray:
    z = int(round(p0 * 100))
    if abs(z - p0 * 100) > 1e-9 or (100 - z) % 2:
        raise ValueError("p0*100 must be an integer with (100 - p0*100) even")
    h = (100 - z) // 2
    lut = np.empty(100, dtype=np.int8)
    lut[:z] = 0
    lut[z:z + h] = 1
    lut[z + h:] = -1
    return lut


def _lut_binary() -> np.ndarray:
    lut = np.empty(100, dtype=np.int8)
    lut[:50] = 1
    lut[50:] = -1
    return lut


def draw_ternary(rng: np.random.Generator, shape: Tuple[int, int], p0: float) -> np.ndarray:
    """int8 matrix with P(0)=p0 and P(+1)=P(-1)=(1-p0)/2."""
    u = rng.integers(0, 100, size=shape, dtype=np.uint8)
    return np.ascontiguousarray(_lut_ternary(p0)[u])


def draw_binary(rng: np.random.Generator, shape: Tuple[int, int]) -> np.ndarray:
    """int8 matrix with P(+1)=P(-1)=1/2."""
    u = rng.integers(0, 100, size=shape, dtype=np.uint8)
    return np.ascontiguousarray(_lut_binary()[u])


@dataclass(frozen=True)
class Workload:
    """One GEMM problem: kind in {"tnn","tbn","bnn"}; C = A (M x K) . B (K x N)."""
    name: str
    kind: str
    M: int
    N: int
    K: int
    seed: int
    p0_a: float  # zero probability of A when ternary (ignored when binary)
    p0_b: float  # zero probability of B when ternary (ignored when binary)
    note: str = ""

    @property
    def a_is_ternary(self) -> bool:
        return self.kind in ("tnn", "tbn")

    @property
    def b_is_ternary(self) -> bool:
        return self.kind == "tnn"

    @property
    def ops(self) -> int:
        """2*M*N*K, the count the effective-TOPS metric divides by time."""
        return 2 * self.M * self.N * self.K


# The five benchmark configurations.  cfg5 comes in three kinds that share one
# random stream (draw order: A ternary, B ternary, A binary, B binary).
WORKLOADS: Dict[str, Workload] = {
    "cfg1_tnn_conv3x3x64_16x16": Workload("cfg1_tnn_conv3x3x64_16x16", "tnn", 64, 256, 576, 0, 0.3, 0.3,
                                          "3x3x64 conv on a 16x16 map"),
    "cfg2_bnn_conv3x3x128_56x56": Workload("cfg2_bnn_conv3x3x128_56x56", "bnn", 256, 3136, 1152, 1, 0.0, 0.0,
                                           "3x3x128 conv, 56x56 output map, im2col"),
    "cfg3_tbn_conv3x3x256_28x28": Workload("cfg3_tbn_conv3x3x256_28x28", "tbn", 512, 784, 2304, 2, 0.3, 0.0,
                                           "3x3x256 conv, 28x28 map"),
    "cfg4_tnn_conv3x3x512_b16_56x56": Workload("cfg4_tnn_conv3x3x512_b16_56x56", "tnn", 1024, 50176, 4608, 3, 0.5, 0.5,
                                               "batch 16 of 56x56 im2col, 3x3x512 conv"),
    "cfg5_tnn_fc_n8": Workload("cfg5_tnn_fc_n8", "tnn", 4096, 8, 16384, 4, 0.3, 0.3, "fully connected, batch 8"),
    "cfg5_tbn_fc_n8": Workload("cfg5_tbn_fc_n8", "tbn", 4096, 8, 16384, 4, 0.3, 0.0, "fully connected, batch 8"),
    "cfg5_bnn_fc_n8": Workload("cfg5_bnn_fc_n8", "bnn", 4096, 8, 16384, 4, 0.0, 0.0, "fully connected, batch 8"),
}

HEADLINE = "cfg4_tnn_conv3x3x512_b16_56x56"


def make_inputs(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """Draw (A, B) for a workload.  Deterministic in w.seed."""
    rng = np.random.default_rng(w.seed)
    if w.name.startswith("cfg5_"):
        # one shared stream for the three skinny problems
        a_ter = draw_ternary(rng, (w.M, w.K), 0.3)
        b_ter = draw_ternary(rng, (w.K, w.N), 0.3)
        a_bin = draw_binary(rng, (w.M, w.K))
        b_bin = draw_binary(rng, (w.K, w.N))
        a = a_ter if w.a_is_ternary else a_bin
        b = b_ter if w.b_is_ternary else b_bin
        return a, b
    a = draw_ternary(rng, (w.M, w.K), w.p0_a) if w.a_is_ternary else draw_binary(rng, (w.M, w.K))
    b = draw_ternary(rng, (w.K, w.N), w.p0_b) if w.b_is_ternary else draw_binary(rng, (w.K, w.N))
    return a, b


def make_custom(kind: str, M: int, N: int, K: int, seed: int, p0: float = 0.3) -> Tuple[np.ndarray, np.ndarray]:
    """Inputs of an arbitrary shape (edge-case and sweep tests)."""
    w = Workload(f"custom_{kind}_{M}x{N}x{K}_s{seed}", kind, M, N, K, seed, p0, p0)
    return make_inputs(w)


def paper_shape_grid() -> List[Tuple[int, int, int]]:
    """The (height, width, depth) grid of the paper's timing experiment (Section IV-B)."""
    return [(h, w, d) for h in (72, 120, 240, 360) for w in (24, 48, 72, 96) for d in (128, 256, 384, 512)]
