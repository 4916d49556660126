"""Seeded synthetic inputs for the mixed-precision (2/4/16-bit) weight format.

This module only draws random numbers and shapes them into the *logical*
(unpacked) arrays that both the CPU oracle and the HIP library take as
input.  It contains none of the method's arithmetic: no dequantization,
no bit packing, no matrix product.  Everything is a numpy array on the host.

Logical format of an N x K weight matrix (rows = output channels, columns =
input channels), first-order group size g1 along K, G = K/g1 groups per row,
g2 first-order groups per second-order (scale, zero) pair, S = ceil(G/g2):

    is4     uint8 [G]      1 if K-group g holds 4-bit codes for every row, else 2-bit
    codes   uint8 [N, K]   w_int, in [0, 3] (2-bit group) or [0, 15] (4-bit group)
    s_int   uint8 [N, G]   quantized first-order scale
    z1      uint8 [N, G]   first-order zero point (integer, used as is)
    s2, z2  uint16 [N, S]  fp16 bit patterns of the second-order scale / zero
                           (g2_axis = 0: one pair per g2 consecutive groups along K)
    row_ptr int32 [N+1], col uint16 [nnz], val uint16 [nnz] (fp16 bits)
                           CSR of the fp16 outliers; columns strictly increasing
                           inside a row, all of them inside 2-bit groups.

The recipes stand in for the quantized Llama checkpoints the paper measures
on (trained weights are not available offline); shapes are the real layer
shapes, value distributions are the ones the benchmark configuration names.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

BASE_SEED = 20231116


@dataclass
class MatrixSpec:
    """Shape and format parameters of one synthetic weight matrix."""

    name: str
    N: int
    K: int
    g1: int = 64
    g2: int = 16
    f4: float = 0.10      # fraction of K-groups that are 4-bit
    p_o: float = 0.005    # outlier probability per weight inside 2-bit groups
    seed: int = BASE_SEED
    g2_axis: int = 0      # 0: a second-order pair per g2 groups along K of a row; 1: per K-group of g2 rows
    meta: int = 0         # 0: byte-wide s_int / z1 and an fp16 z2; 1: the value ranges of the paper's aligned packing

    @property
    def G(self) -> int:
        return self.K // self.g1

    @property
    def S(self) -> int:
        return -(-self.G // self.g2)

    @property
    def n4(self) -> int:
        return int(np.floor(self.f4 * self.G + 0.5))


@dataclass
class Logical:
    """The logical arrays of one matrix plus its spec."""

    spec: MatrixSpec
    is4: np.ndarray
    codes: np.ndarray
    s_int: np.ndarray
    z1: np.ndarray
    s2: np.ndarray
    z2: np.ndarray
    row_ptr: np.ndarray
    col: np.ndarray
    val: np.ndarray
    extra: Dict[str, object] = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])


def matrix_seed(config: int, matrix_index: int, layer_index: int = 0) -> int:
    return BASE_SEED + 1000 * config + 10 * matrix_index + 100000 * layer_index


def f16_bits(a: np.ndarray) -> np.ndarray:
    """Round an array to fp16 (numpy's IEEE round-to-nearest-even cast) and return the bit patterns."""
    return np.asarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def draw_is4(rng: np.random.Generator, G: int, n4: int) -> np.ndarray:
    is4 = np.zeros(G, dtype=np.uint8)
    if n4 > 0:
        is4[rng.choice(G, size=n4, replace=False)] = 1
    return is4


def draw_outliers(rng: np.random.Generator, N: int, cols2: np.ndarray, p_o: float):
    """Independent Bernoulli(p_o) choice per weight over the 2-bit columns `cols2`.

    Drawn as a Bernoulli process over the flattened N x len(cols2) positions:
    gaps between successes are Geometric(p_o), which is the same distribution as
    testing every position on its own but costs O(nnz) random numbers.
    """
    K2 = int(cols2.size)
    total = N * K2
    if p_o <= 0.0 or total == 0:
        return (np.zeros(N + 1, dtype=np.int32), np.zeros(0, dtype=np.uint16),
                np.zeros(0, dtype=np.uint16))
    pos_chunks = []
    last = -1
    while True:
        want = int(max(1024, (total - last) * p_o * 1.1 + 64))
        gaps = rng.geometric(p_o, size=want).astype(np.int64)
        pos = last + np.cumsum(gaps)
        if pos[-1] >= total:
            pos_chunks.append(pos[pos < total])
            break
        pos_chunks.append(pos)
        last = int(pos[-1])
    pos = np.concatenate(pos_chunks)
    rows = pos // K2
    col = cols2[pos % K2].astype(np.uint16)
    counts = np.bincount(rows, minlength=N).astype(np.int64)
    row_ptr = np.zeros(N + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(counts)
    val = f16_bits(rng.normal(0.0, 0.5, size=pos.size))
    return row_ptr, col, val


def make_matrix(spec: MatrixSpec, z1_full_range: bool = False,
                is4: Optional[np.ndarray] = None) -> Logical:
    """Draw one matrix in the logical format from `spec.seed`."""
    if spec.K % spec.g1 != 0:
        raise ValueError("K must be a multiple of g1")
    rng = np.random.default_rng(spec.seed)
    N, K, g1, G, S = spec.N, spec.K, spec.g1, spec.G, spec.S
    if is4 is None:
        is4 = draw_is4(rng, G, spec.n4)
    else:
        is4 = np.asarray(is4, dtype=np.uint8).copy()
    hi_g = np.where(is4 != 0, 16, 4).astype(np.int64)          # exclusive upper bound per group
    hi_k = np.repeat(hi_g, g1)
    # uniform integer codes in [0, 2^b - 1]: draw a byte and reduce it (256 is a multiple of 4 and 16)
    codes = (rng.integers(0, 256, size=(N, K), dtype=np.uint8) % hi_k.astype(np.uint8)[None, :]).astype(np.uint8)
    s_int = rng.integers(0, 256, size=(N, G), dtype=np.uint8)
    if z1_full_range:
        z1 = rng.integers(0, 256, size=(N, G), dtype=np.uint8)
    else:
        z1 = (rng.integers(0, 256, size=(N, G), dtype=np.uint8) % hi_g.astype(np.uint8)[None, :]).astype(np.uint8)
    shape2 = (N, S) if spec.g2_axis == 0 else (-(-N // spec.g2), G)
    s2 = f16_bits(np.exp(rng.normal(-6.0, 0.5, size=shape2)))
    z2 = f16_bits(rng.random(size=shape2))
    if spec.meta == 1:
        # ranges of the aligned packing (Sec. 3.3): scales of Ns = 4 bits, of which the second and third of
        # every three consecutive 2-bit groups of a row have 3; an Ns-bit integer second-order zero
        pos2 = np.cumsum(is4 == 0) - 1                      # index of a 2-bit group among the 2-bit groups
        hi_s = np.where(is4 != 0, 16, np.where(pos2 % 3 == 0, 16, 8)).astype(np.uint8)
        s_int = (s_int % hi_s[None, :]).astype(np.uint8)
        z2 = f16_bits(rng.integers(0, 16, size=shape2).astype(np.float32))
        s2 = f16_bits(np.exp(rng.normal(-4.0, 0.5, size=shape2)))
    cols2 = np.nonzero(np.repeat(is4, g1) == 0)[0]
    row_ptr, col, val = draw_outliers(rng, N, cols2, spec.p_o)
    return Logical(spec, is4, codes, s_int, z1, s2, z2, row_ptr, col, val)


def make_x(seed: int, M: int, K: int) -> np.ndarray:
    """Activations X[M, K] ~ N(0, 1) rounded to fp16; returned as fp16 bit patterns (uint16)."""
    rng = np.random.default_rng(seed ^ 0x5EED)
    return f16_bits(rng.normal(0.0, 1.0, size=(M, K)))


# ---------------------------------------------------------------------------
# The benchmark configurations (shapes of the public Llama models' linear layers).
# ---------------------------------------------------------------------------

def config_specs(config: int, f4: Optional[float] = None, p_o: Optional[float] = None,
                 layer_index: int = 0) -> List[MatrixSpec]:
    """Matrix specs of benchmark configuration `config` (0..4)."""
    if config == 0:
        shapes = [("tiny", 1024, 1024)]
        g1, g2, df4, dpo = 64, 16, 0.10, 0.005
    elif config in (1, 2):
        shapes = [("qkv", 12288, 4096), ("o", 4096, 4096), ("gate_up", 22016, 4096), ("down", 4096, 11008)]
        g1, g2, df4, dpo = 64, 16, 0.10, 0.005
    elif config == 3:
        shapes = [("qkv", 6144, 4096), ("o", 4096, 4096), ("gate_up", 28672, 4096),
                  ("down", 4096, 14336), ("lm_head", 128256, 4096)]
        g1, g2, df4, dpo = 128, 16, 0.15, 0.005
    elif config == 4:
        shapes = [("qkv", 10240, 8192), ("o", 8192, 8192), ("gate_up", 57344, 8192), ("down", 8192, 28672)]
        g1, g2, df4, dpo = 64, 16, 0.10, 0.005
    else:
        raise ValueError("config must be 0..4")
    f4 = df4 if f4 is None else f4
    p_o = dpo if p_o is None else p_o
    return [MatrixSpec(name, N, K, g1, g2, f4, p_o, matrix_seed(config, i, layer_index))
            for i, (name, N, K) in enumerate(shapes)]


def stored_bytes(spec: MatrixSpec, n4: int, nnz: int) -> Dict[str, int]:
    """Bytes the format must move for one product, by section (no alignment padding)."""
    N, K, g1, G, S = spec.N, spec.K, spec.g1, spec.G, spec.S
    n2 = G - n4
    pairs = N * S if spec.g2_axis == 0 else (-(-N // spec.g2)) * G
    aligned = getattr(spec, "meta", 0) == 1   # 16 bits per three 2-bit groups, 8 per 4-bit group, 24 per pair
    out = {
        "codes": N * (n2 * g1 // 4 + n4 * g1 // 2),
        "s_int_z1": N * (2 * (-(-n2 // 3)) + n4) if aligned else 2 * N * G,
        "s2_z2": (3 if aligned else 4) * pairs,
        "outliers": 4 * nnz,
        "row_ptr": 4 * (N + 1),
    }
    out["total"] = sum(out.values())
    return out
