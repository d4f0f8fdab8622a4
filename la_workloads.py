"""Seeded synthetic inputs for the linear-attention tests and benchmark.

This module holds none of the method's arithmetic: it only draws the input
tensors and rounds them to the I/O type.  Both the CPU oracle's tests and the
HIP path's tests take their inputs from here, so the two sides see identical
values.

Recipe (the five benchmark configurations):  Q, K ~ N(0,1) i.i.d. in float64,
each row then divided by its L2 norm (the row normalisation of Sec. 3.3, done
by the caller before the attention call); V, dO ~ N(0,1).  Values are then
rounded to the I/O type (float32, or bfloat16 with round-to-nearest-even) and
handed out both in that type's bits and widened back to float64, so the oracle
consumes exactly the numbers the GPU consumes.
"""
from dataclasses import dataclass

import numpy as np

SEED_BASE = 251021956


@dataclass(frozen=True)
class Config:
    name: str
    B: int
    H: int
    N: int
    D: int
    causal: bool
    dtype: str  # "f32" or "bf16"  (I/O type; accumulation is always fp32 on the GPU)
    a: float = 1.0
    b: float = 0.5

    @property
    def token_heads(self):
        return self.B * self.H * self.N

    @property
    def tokens(self):
        return self.B * self.N


CONFIGS = [
    Config("cfg1_causal_f32_B1_H1_N256_D16", 1, 1, 256, 16, True, "f32"),
    Config("cfg2_causal_f32_B4_H16_N4096_D64", 4, 16, 4096, 64, True, "f32"),
    Config("cfg3_noncausal_f32_B8_H8_N16384_D64", 8, 8, 16384, 64, False, "f32"),
    Config("cfg4_causal_bf16_B8_H16_N2048_D128", 8, 16, 2048, 128, True, "bf16"),
    Config("cfg5_causal_bf16_B1_H16_N131072_D128", 1, 16, 131072, 128, True, "bf16"),
]


# The paper's own stand-alone layer benchmark (Sec. 5.1: B = 4, H = 16, fp32, causal; the
# sequence-length sweep at D = 128 and the head-size sweep at N = 4096).  Same value recipe;
# not part of the five benchmark configurations above.
PAPER_SHAPES = (
    [Config("paper_causal_f32_B4_H16_N%d_D128" % n, 4, 16, n, 128, True, "f32")
     for n in (1000, 10000, 100000, 300000)]
    + [Config("paper_causal_f32_B4_H16_N4096_D%d" % d, 4, 16, 4096, d, True, "f32")
       for d in (32, 64, 128, 256)]
)


def find_workload(name):
    """A configuration of CONFIGS or PAPER_SHAPES by name."""
    for c in list(CONFIGS) + list(PAPER_SHAPES):
        if c.name == name:
            return c
    raise KeyError(name)


def bf16_round_bits(x):
    """float array -> uint16 bfloat16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits):
    """uint16 bfloat16 bit patterns -> float64 values (exact)."""
    u = bits.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def round_to_dtype(x, dtype):
    """Round a float64 array to the I/O type.

    Returns (device_bits, values64): ``device_bits`` is what is uploaded
    (float32 array, or uint16 bf16 patterns) and ``values64`` the same numbers
    widened to float64 for the oracle."""
    if dtype == "f32":
        x32 = np.ascontiguousarray(x, dtype=np.float32)
        return x32, x32.astype(np.float64)
    if dtype == "bf16":
        bits = bf16_round_bits(x)
        return bits, bf16_bits_to_f64(bits)
    raise ValueError("dtype must be 'f32' or 'bf16'")


def _unit_rows(x):
    return x / np.linalg.norm(x, axis=-1, keepdims=True)


def make_slice(N, D, dtype, seed, s, normalise=True):
    """Q, K, V, dO of one (batch*head) slice ``s``: dict name -> (bits, values64),
    each [N, D].  Slice ``s`` has its own child seed, so slices can be drawn one
    at a time (large configurations) or in any subset."""
    rng = np.random.Generator(np.random.PCG64([seed, s]))
    out = {}
    for name in ("Q", "K", "V", "dO"):
        x = rng.standard_normal((N, D))
        if normalise and name in ("Q", "K"):
            x = _unit_rows(x)
        out[name] = round_to_dtype(x, dtype)
    return out


def make_inputs(B, H, N, D, dtype, seed, normalise=True, bh_subset=None):
    """Draw Q, K, V, dO of shape [B, H, N, D].

    ``bh_subset``: optional list of flat (b*H + h) indices; when given only
    those slices are generated and the result has shape [len(subset), N, D].

    Returns a dict: for each of "Q","K","V","dO" the pair
    (device_bits, values64)."""
    out = {}
    slices = list(range(B * H)) if bh_subset is None else list(bh_subset)
    bufs = {n: ([], []) for n in ("Q", "K", "V", "dO")}
    for s in slices:
        sl = make_slice(N, D, dtype, seed, s, normalise)
        for name in bufs:
            bufs[name][0].append(sl[name][0])
            bufs[name][1].append(sl[name][1])
    for name, (bl, vl) in bufs.items():
        if slices:
            bits = np.stack(bl)
            vals = np.stack(vl)
        else:
            bits = np.zeros((0, N, D), dtype=np.float32 if dtype == "f32" else np.uint16)
            vals = np.zeros((0, N, D), dtype=np.float64)
        if bh_subset is None:
            bits = bits.reshape(B, H, N, D)
            vals = vals.reshape(B, H, N, D)
        out[name] = (bits, vals)
    return out


def config_inputs(index, bh_subset=None):
    """Inputs of benchmark configuration ``index`` (0-based into CONFIGS)."""
    c = CONFIGS[index]
    return make_inputs(c.B, c.H, c.N, c.D, c.dtype, SEED_BASE + index, True, bh_subset)


def workload_seed(c):
    """Seed of a named workload: the five configurations keep theirs, the paper's shapes
    follow with 100 + their position."""
    if c in CONFIGS:
        return SEED_BASE + CONFIGS.index(c)
    return SEED_BASE + 100 + list(PAPER_SHAPES).index(c)


def workload_inputs(c, bh_subset=None):
    """Inputs of a configuration of CONFIGS or PAPER_SHAPES."""
    return make_inputs(c.B, c.H, c.N, c.D, c.dtype, workload_seed(c), True, bh_subset)
