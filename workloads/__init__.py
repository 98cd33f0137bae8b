"""Seeded synthetic inputs for the sketch-linear path.

This module only draws random numbers and names shapes.  It holds none of
the method's arithmetic (no hashing, no sketch update/query, no width
allocation, no matmul): the CPU oracle and the GPU library both receive the
arrays produced here and neither is imported here.

The shapes follow Llama-2-7B / 70B linear layers; the value distributions
follow the benchmark configurations (weights N(0, 0.02^2) in binary16 with a
small fraction of input channels scaled x20 as outliers; activations N(0,1)).
They stand in for the paper's Llama3/Qwen3 weights and Wikitext activations
(Sec. 4, experimental setup), which are not available offline.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Tuple

import numpy as np

BASE_SEED = 250617


@dataclass(frozen=True)
class Workload:
    name: str
    cfg: int                    # benchmark configuration number (1..5)
    in_features: int
    out_features: int
    tile_in: int                # group = tile_in x tile_out weights
    tile_out: int
    d: int                      # sketch rows
    bpw: float                  # target bits per weight with binary16 states
    outlier_frac: float = 0.0   # fraction of input channels scaled up
    outlier_scale: float = 20.0
    width_mult: float = 1.0     # importance of an outlier channel (others: 1)
    layer_index: int = 0
    batches: Tuple[int, ...] = (1,)
    tokens: int = 0             # > 0: prefill workload with bf16 activations

    @property
    def seed(self) -> int:
        return BASE_SEED + 1000 * self.cfg + self.layer_index

    @property
    def n_groups(self) -> int:
        return (self.in_features // self.tile_in) * (self.out_features // self.tile_out)

    @property
    def budget_states(self) -> int:
        """Total number of binary16 states the target bits/weight allows."""
        return int(self.in_features * self.out_features * self.bpw / 16)

    @property
    def n_weights(self) -> int:
        return self.in_features * self.out_features


def outlier_channels(wl: Workload) -> np.ndarray:
    """Sorted indices of the input channels that are scaled up."""
    n = int(np.ceil(wl.outlier_frac * wl.in_features)) if wl.outlier_frac > 0 else 0
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    rng = np.random.default_rng(wl.seed + 100)
    return np.sort(rng.choice(wl.in_features, size=n, replace=False))


def gen_weight(wl: Workload) -> np.ndarray:
    """W[j][o] (d_in x d_out, row major) as float16."""
    rng = np.random.default_rng(wl.seed)
    w = rng.standard_normal((wl.in_features, wl.out_features), dtype=np.float32) * np.float32(0.02)
    oc = outlier_channels(wl)
    if oc.size:
        w[oc, :] *= np.float32(wl.outlier_scale)
    return w.astype(np.float16)


def gen_hash_params(wl: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """d pairs (A_r odd, C_r), all below 2^24."""
    rng = np.random.default_rng(wl.seed + 500)
    A = (2 * rng.integers(0, 1 << 23, size=wl.d, dtype=np.int64) + 1).astype(np.uint32)
    C = rng.integers(0, 1 << 24, size=wl.d, dtype=np.int64).astype(np.uint32)
    return A, C


def gen_importance(wl: Workload) -> np.ndarray:
    """Synthetic importance per group: ``width_mult`` for groups that hold an
    outlier input channel, 1 elsewhere.  Stands in for E[a_j^2] over
    calibration activations (Sec. 3.2), which needs data not available here."""
    n_jb = wl.in_features // wl.tile_in
    n_ob = wl.out_features // wl.tile_out
    imp = np.ones((n_jb, n_ob), dtype=np.float64)
    if wl.width_mult != 1.0:
        jb = np.unique(outlier_channels(wl) // wl.tile_in)
        imp[jb, :] = wl.width_mult
    return imp.ravel()


def gen_x(wl: Workload, batch: int, salt: int = 0) -> np.ndarray:
    """Decode activations x[batch][in] ~ N(0,1) as float16."""
    rng = np.random.default_rng(wl.seed + 700 + 17 * batch + salt)
    return rng.standard_normal((batch, wl.in_features), dtype=np.float32).astype(np.float16)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even cast of float32 to bfloat16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def gen_X_bf16(wl: Workload, tokens: int, salt: int = 0) -> np.ndarray:
    """Prefill activations X[tokens][in] ~ N(0,1) as bfloat16 bit patterns."""
    rng = np.random.default_rng(wl.seed + 900 + salt)
    return f32_to_bf16_bits(rng.standard_normal((tokens, wl.in_features), dtype=np.float32))


# --------------------------------------------------------------------------
# The benchmark configurations.  1-D groups (tile_in = 1, tile_out = out) are
# the primary geometry for configurations 2-5: one sketch per input channel,
# i.e. one row of the paper's grouped weight matrix W_g and the unit of its
# row-wise importance; configuration 1 is pinned as one 256x256 group.
# --------------------------------------------------------------------------

def cfg1() -> Workload:
    return Workload("cfg1_256x256_d2", 1, 256, 256, 256, 256, 2, 0.5)


def cfg2(two_d: bool = False) -> Workload:
    if two_d:
        return Workload("cfg2_q_proj_d3_2d", 2, 4096, 4096, 256, 256, 3, 0.5, outlier_frac=0.005)
    return Workload("cfg2_q_proj_d3", 2, 4096, 4096, 1, 4096, 3, 0.5, outlier_frac=0.005)


def cfg3(which: str = "up") -> Workload:
    if which in ("up", "gate"):
        return Workload(f"cfg3_{which}_d4", 3, 4096, 11008, 1, 11008, 4, 0.5, outlier_frac=0.01,
                        width_mult=4.0, layer_index=0 if which == "up" else 1, batches=(1, 8, 16))
    if which == "down":
        return Workload("cfg3_down_d4", 3, 11008, 4096, 1, 4096, 4, 0.5, outlier_frac=0.01,
                        width_mult=4.0, layer_index=2, batches=(1, 8, 16))
    raise KeyError(which)


def cfg4(out_features: int = 4096, bpw: float = 0.5) -> Workload:
    li = (0 if out_features == 4096 else 1) * 2 + (0 if bpw == 0.5 else 1)
    return Workload(f"cfg4_prefill_{out_features}_bpw{bpw}", 4, 4096, out_features, 1, out_features,
                    4, bpw, layer_index=li, tokens=2048)


LLAMA7B_LAYER = (("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                 ("gate", 4096, 11008), ("up", 4096, 11008), ("down", 11008, 4096))


def cfg5_stack(n_layers: int = 32):
    """The 7 linear layers of each of ``n_layers`` Llama-2-7B-shaped blocks."""
    out = []
    for layer in range(n_layers):
        for i, (nm, fi, fo) in enumerate(LLAMA7B_LAYER):
            out.append(Workload(f"cfg5_L{layer}_{nm}", 5, fi, fo, 1, fo, 4, 0.5, outlier_frac=0.01,
                                width_mult=4.0, layer_index=layer * 7 + i))
    return out


def gen_layer_scales(n_layers: int, lo: float = 0.5, hi: float = 2.0) -> np.ndarray:
    """Synthetic mean squared activation per layer of a stack, log-uniform in [lo, hi]: stands in for
    the layer-wise importance statistics of a calibration set."""
    rng = np.random.default_rng(BASE_SEED + 5000 + 77)
    return np.exp(rng.uniform(np.log(lo), np.log(hi), size=n_layers))


def cfg5_70b() -> Workload:
    return Workload("cfg5_70b_8192x28672", 5, 8192, 28672, 1, 28672, 4, 0.5, outlier_frac=0.01,
                    width_mult=4.0, layer_index=900, tokens=2048)


def small(name: str, in_features: int, out_features: int, tile_in: int, tile_out: int, d: int,
          bpw: float, layer_index: int, **kw) -> Workload:
    """Small ad-hoc layers for parity tests (configuration number 0)."""
    return Workload(name, 0, in_features, out_features, tile_in, tile_out, d, bpw,
                    layer_index=layer_index, **kw)


def pack_nibbles(codes) -> np.ndarray:
    """Storage format of 4-bit codes: two's-complement nibbles, element i in byte i // 2, low nibble for
    even i (a trailing odd element leaves the high nibble of the last byte zero)."""
    c = np.asarray(codes, dtype=np.int8).astype(np.uint8) & 0xF
    if c.size % 2:
        c = np.concatenate([c, np.zeros(1, dtype=np.uint8)])
    return np.ascontiguousarray(c[0::2] | (c[1::2] << 4))
