"""Seeded synthetic inputs for the direct-convolution workloads.

This module only draws numbers and names shapes.  It holds none of the
method's arithmetic, so both the CPU oracle's tests and the HIP path's tests
may use it without sharing any code of the computation itself.

Letters follow the C ABI: batch N, channels C, image H x W, K filters of
F x F.  (The paper writes K for the filter side and F for the filter count;
see its Fig. 3 caption.)  The paper's own experiments (Sec. 5, Figs. 7 and 8)
use synthetic tensors parameterised only by size, so these stand in for them
directly.
"""
from __future__ import annotations

from dataclasses import dataclass
import numpy as np

SEED_BASE = 170510591


@dataclass(frozen=True)
class Workload:
    name: str          # short tag used in reports
    kind: str          # "single" (one input channel) or "general"
    N: int
    C: int
    H: int
    W: int
    K: int
    F: int
    in_dist: str       # "u11" = uniform[-1,1], "u01" = uniform[0,1]
    filt_dist: str     # "u11" or "he" = normal(0, sqrt(2/(C F F)))
    seed: int

    @property
    def Ho(self) -> int:
        return self.H - self.F + 1

    @property
    def Wo(self) -> int:
        return self.W - self.F + 1

    @property
    def out_elems(self) -> int:
        return self.N * self.K * self.Ho * self.Wo

    @property
    def flops(self) -> int:
        return 2 * self.out_elems * self.C * self.F * self.F

    @property
    def algorithmic_bytes(self) -> int:
        """Input + filters + output, each touched exactly once, 4 bytes each."""
        return 4 * (self.N * self.C * self.H * self.W
                    + self.K * self.C * self.F * self.F
                    + self.out_elems)

    def in_shape(self):
        return (self.H, self.W) if self.kind == "single" else (self.N, self.C, self.H, self.W)

    def filt_shape(self):
        return (self.K, self.F, self.F) if self.kind == "single" else (self.K, self.C, self.F, self.F)

    def out_shape(self):
        return (self.K, self.Ho, self.Wo) if self.kind == "single" else (self.N, self.K, self.Ho, self.Wo)


def _mk(name, kind, N, C, H, W, K, F, in_dist, filt_dist, idx):
    return Workload(name, kind, N, C, H, W, K, F, in_dist, filt_dist, SEED_BASE + idx)


# The five benchmark configurations, in the order the baseline lists them,
# plus the filter-size sweep of the large single-channel case.
S1 = _mk("S1", "single", 1, 1, 256, 256, 16, 3, "u11", "u11", 0)
S2 = _mk("S2", "single", 1, 1, 4096, 4096, 64, 5, "u11", "u11", 1)
G1 = _mk("G1", "general", 64, 3, 224, 224, 64, 11, "u11", "u11", 2)
G2 = _mk("G2", "general", 32, 64, 56, 56, 64, 3, "u01", "he", 3)
G3 = _mk("G3", "general", 32, 256, 28, 28, 512, 3, "u01", "he", 4)
S2_SWEEP = {F: _mk(f"S2_F{F}", "single", 1, 1, 4096, 4096, 64, F, "u11", "u11", 10 + F)
            for F in (3, 5, 7, 9, 11)}

CONFIGS = {w.name: w for w in (S1, S2, G1, G2, G3)}

# The other corners the paper sweeps (Sec. 5: Fig. 7 for the special case with 1x1, 3x3 and 5x5
# filters, a single filter being its stated weak spot; Fig. 8 / Table 1 for the general case
# with 3x3, 5x5 and 7x7 filters, 32 x 32 images being the one place where it lost).  The
# figures themselves did not survive, so sizes are chosen here: the image and batch sizes of
# the benchmark configurations with the paper's filter sides and corner cases.
PAPER_SWEEP = {w.name: w for w in (
    _mk("A_F1", "single", 1, 1, 4096, 4096, 64, 1, "u11", "u11", 30),     # no data sharing at all
    _mk("A_K1_F3", "single", 1, 1, 4096, 4096, 1, 3, "u11", "u11", 31),   # one filter
    _mk("A_K1_F5", "single", 1, 1, 4096, 4096, 1, 5, "u11", "u11", 32),
    _mk("A_K16_F3", "single", 1, 1, 2048, 2048, 16, 3, "u11", "u11", 33),
    _mk("B_F5", "general", 32, 64, 56, 56, 64, 5, "u01", "he", 34),
    _mk("B_F7", "general", 32, 64, 56, 56, 64, 7, "u01", "he", 35),
    _mk("B_32_F3", "general", 128, 64, 32, 32, 128, 3, "u01", "he", 36),  # very small images
    _mk("B_32_F5", "general", 128, 64, 32, 32, 128, 5, "u01", "he", 37),
    _mk("B_32_F7", "general", 128, 64, 32, 32, 128, 7, "u01", "he", 38),
    # the special case on a batch: one-channel images through dconv_general
    _mk("A_N16_512_F5", "general", 16, 1, 512, 512, 64, 5, "u11", "u11", 39),
    _mk("A_N256_28_F5", "general", 256, 1, 28, 28, 32, 5, "u11", "u11", 40),   # small images: general kernel
    # three channels, small filters: still bound by the output stream (a first layer on RGB images)
    _mk("A_C3_N16_512_F3", "general", 16, 3, 512, 512, 64, 3, "u01", "he", 41),
    _mk("A_C3_N64_224_F3", "general", 64, 3, 224, 224, 64, 3, "u01", "he", 42),
    # few filters in the general case (the weak spot of Sec. 5 carried over: a last layer to RGB, one map)
    _mk("B_K3_F3", "general", 8, 64, 224, 224, 3, 3, "u01", "he", 43),
    _mk("B_K1_F7", "general", 8, 16, 224, 224, 1, 7, "u01", "he", 44),
    # one channel where the general-case kernel is the faster one: a mid-sized image with many large
    # filters, a small image
    _mk("A_768_K192_F8", "single", 1, 1, 768, 768, 192, 8, "u11", "u11", 45),
    _mk("A_64_K128_F8", "single", 1, 1, 64, 64, 128, 8, "u11", "u11", 46),
)}


def _draw(rng: np.random.Generator, dist: str, shape, C: int, F: int) -> np.ndarray:
    if dist == "u11":
        a = rng.random(shape, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
    elif dist == "u01":
        a = rng.random(shape, dtype=np.float32)
    elif dist == "he":
        sigma = np.float32(np.sqrt(2.0 / (C * F * F)))
        a = rng.standard_normal(shape, dtype=np.float32) * sigma
    else:
        raise ValueError(dist)
    return np.ascontiguousarray(a, dtype=np.float32)


def make_inputs(w: Workload):
    """Return (input, filters) as contiguous float32 numpy arrays."""
    rng = np.random.default_rng(w.seed)
    x = _draw(rng, w.in_dist, w.in_shape(), w.C, w.F)
    f = _draw(rng, w.filt_dist, w.filt_shape(), w.C, w.F)
    return x, f


def random_case(seed: int, N: int, C: int, H: int, W: int, K: int, F: int,
                in_dist: str = "u11", filt_dist: str = "u11"):
    """Inputs for an arbitrary general-layout shape: in[N,C,H,W], filt[K,C,F,F]."""
    rng = np.random.default_rng(SEED_BASE * 7 + seed)
    x = _draw(rng, in_dist, (N, C, H, W), C, F)
    f = _draw(rng, filt_dist, (K, C, F, F), C, F)
    return x, f


def integer_case(seed: int, N: int, C: int, H: int, W: int, K: int, F: int):
    """Small-integer valued float32 inputs: pixels in [-8, 8], weights in [-4, 4].

    Every product and every partial sum is an integer far below 2**24 for the
    reduction lengths used here, so any fp32 summation order gives the same
    bits and results can be compared exactly.
    """
    rng = np.random.default_rng(SEED_BASE * 11 + seed)
    x = rng.integers(-8, 9, size=(N, C, H, W)).astype(np.float32)
    f = rng.integers(-4, 5, size=(K, C, F, F)).astype(np.float32)
    return x, f


def to_16bit(a: np.ndarray, kind: str):
    """Round float32 values to the nearest fp16 ("f16") or bf16 ("bf16") value, ties to even.

    Returns (the rounded values as float32, their 16-bit patterns as uint16): the first go to
    the oracle, the second to the device.  Values must be finite and within the type's range.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    if kind == "f16":
        h = a.astype(np.float16)
        return h.astype(np.float32), h.view(np.uint16)
    if kind == "bf16":
        u = a.view(np.uint32)
        bits = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32), bits
    raise ValueError(kind)


def sample_indices(seed: int, total: int, count: int) -> np.ndarray:
    """`count` flat output indices in [0, total): the first, the last and seeded random ones."""
    rng = np.random.default_rng(SEED_BASE * 13 + seed)
    idx = rng.integers(0, total, size=max(count - 2, 0), dtype=np.int64)
    return np.unique(np.concatenate([np.array([0, total - 1], dtype=np.int64), idx]))
