"""Seeded synthetic inputs for the MoE expert layer (shared by the CPU oracle's
tests and the HIP path's tests/bench).

This module only draws random numbers and stores them in the dtypes the
workloads name (fp32, or bf16 kept as uint16 bit patterns).  It holds none of
the layer's arithmetic: no top-k, no softmax, no permutation, no FFN.

Recipe (every array is a pure function of (seed, stream id, shape)):
  * generator: numpy ``Generator(Philox(key=[seed, stream]))`` ->
    ``standard_normal(float32)``, scaled by the stated std;
  * stream ids: 0 = activations x, 1 = router matrix W_g, 2 = router noise z
    (Zipf-biased workloads), 10+3e+{0,1,2} = w1, w3, w2 of expert e (drawn
    from the config's weight seed, which the Mixtral-shaped single-layer
    workloads share so that one set of matrices serves all three);
  * ``N(0, 1/fan_in)``: std d^-1/2 for W_g, w1, w3 and f^-1/2 for w2;
  * bf16 = round-to-nearest-even of the fp32 draw, stored as uint16;
  * router logits are either fp32(x . W_g) accumulated in fp64 on the host
    (given identically to both sides), or fp32(z + ln p_e) with p the
    Zipf(s=1.2) pmf over experts (expert 0 hottest).

The workloads stand in for the paper's (Mixtral-8x7B on ShareGPT prompts,
Sec. 4.1), which need trained weights and a dataset that are not available:
same layer shape (Sec. 3.2: three 4096 x 14336 matrices per expert, 8 experts
per layer) and the same token counts per step (single-batch decode, beam
width 16, prefill up to 4096).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

F32 = "f32"
BF16 = "bf16"


@dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int
    d: int
    f: int
    E: int
    k: int
    w_dtype: str  # F32 or BF16
    x_dtype: str  # F32 or BF16
    seed: int
    zipf_s: Optional[float] = None  # None: logits = x.W_g ; else z + ln(zipf pmf)
    w_seed: Optional[int] = None    # seed of the expert matrices (default: seed)

    @property
    def N(self) -> int:
        return self.T * self.k

    @property
    def weight_seed(self) -> int:
        return self.seed if self.w_seed is None else self.w_seed


CONFIGS = {
    "tiny_fp32": MoEConfig("tiny_fp32", 16, 256, 512, 8, 2, F32, F32, 1001),
    "decode_t1": MoEConfig("decode_t1", 1, 4096, 14336, 8, 2, BF16, F32, 1002),
    # the three Mixtral-shaped single-layer workloads share one set of expert
    # matrices (weight seed 1002); activations and logits have their own seeds
    "beam_t16": MoEConfig("beam_t16", 16, 4096, 14336, 8, 2, BF16, F32, 1003, 1.2, 1002),
    "prefill_t4096": MoEConfig("prefill_t4096", 4096, 4096, 14336, 8, 2, BF16, BF16, 1004, 1.2,
                               1002),
    # second layer shape (paper, App. E evaluates a 16-expert top-2 model): d=4096, f=6400,
    # E=16; the layer arithmetic is the same, only the shape differs.  One weight set
    # (seed 1005) serves the three workloads.
    "e16_decode_t1": MoEConfig("e16_decode_t1", 1, 4096, 6400, 16, 2, BF16, F32, 1005),
    "e16_beam_t16": MoEConfig("e16_beam_t16", 16, 4096, 6400, 16, 2, BF16, F32, 1006, 1.2, 1005),
    "e16_prefill_t4096": MoEConfig("e16_prefill_t4096", 4096, 4096, 6400, 16, 2, BF16, BF16, 1007,
                                   1.2, 1005),
}


def stack_layer_config(layer: int, T: int) -> MoEConfig:
    """Layer `layer` of the 32-layer stack workload (independent seeds per layer)."""
    return MoEConfig(f"stack_l{layer}_t{T}", T, 4096, 14336, 8, 2, BF16, F32, 2000 + layer)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def normal_f32(seed: int, stream: int, shape, std: float = 1.0) -> np.ndarray:
    a = _rng(seed, stream).standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns.
    Inputs are finite (normal draws), so no NaN handling is needed."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of an fp32 array or a bf16-bits (uint16) array to fp64."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def zipf_log_pmf(E: int, s: float) -> np.ndarray:
    r = np.arange(1, E + 1, dtype=np.float64)
    p = r ** (-s)
    p /= p.sum()
    return np.log(p)


def expert_matrix(cfg: MoEConfig, e: int, which: int) -> np.ndarray:
    """One expert matrix in its stored dtype.  which: 0 = w1 [d,f], 1 = w3 [d,f],
    2 = w2 [f,d]."""
    if which == 2:
        shape, std = (cfg.f, cfg.d), cfg.f ** -0.5
    else:
        shape, std = (cfg.d, cfg.f), cfg.d ** -0.5
    a = normal_f32(cfg.weight_seed, 10 + 3 * e + which, shape, std)
    return f32_to_bf16_bits(a) if cfg.w_dtype == BF16 else a


@dataclass
class LayerInputs:
    cfg: MoEConfig
    x: np.ndarray        # [T,d] fp32, or uint16 bf16 bits
    logits: np.ndarray   # [T,E] fp32
    w1: np.ndarray       # [E,d,f] fp32 or uint16
    w3: np.ndarray       # [E,d,f]
    w2: np.ndarray       # [E,f,d]
    w_gate: Optional[np.ndarray] = field(default=None)  # [d,E] fp32 when logits = x.W_g


def make_activations(cfg: MoEConfig):
    """x and router logits (and W_g when the logits come from it)."""
    x32 = normal_f32(cfg.seed, 0, (cfg.T, cfg.d))
    if cfg.x_dtype == BF16:
        x = f32_to_bf16_bits(x32)
        x_val = bf16_bits_to_f32(x)
    else:
        x = x32
        x_val = x32
    if cfg.zipf_s is None:
        w_gate = normal_f32(cfg.seed, 1, (cfg.d, cfg.E), cfg.d ** -0.5)
        logits = (x_val.astype(np.float64) @ w_gate.astype(np.float64)).astype(np.float32)
    else:
        w_gate = None
        z = normal_f32(cfg.seed, 2, (cfg.T, cfg.E)).astype(np.float64)
        logits = (z + zipf_log_pmf(cfg.E, cfg.zipf_s)[None, :]).astype(np.float32)
    return x, logits, w_gate


def make_weights(cfg: MoEConfig, threads: int = 8):
    """w1, w3 [E,d,f] and w2 [E,f,d] in the stored dtype; each (expert, matrix)
    has its own Philox stream, so the result does not depend on `threads`."""
    dt = np.uint16 if cfg.w_dtype == BF16 else np.float32
    w1 = np.empty((cfg.E, cfg.d, cfg.f), dtype=dt)
    w3 = np.empty((cfg.E, cfg.d, cfg.f), dtype=dt)
    w2 = np.empty((cfg.E, cfg.f, cfg.d), dtype=dt)
    dst = (w1, w3, w2)

    def job(ew):
        e, which = ew
        dst[which][e] = expert_matrix(cfg, e, which)

    jobs = [(e, which) for e in range(cfg.E) for which in range(3)]
    if threads <= 1 or cfg.d * cfg.f < (1 << 20):
        for j in jobs:
            job(j)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(job, jobs))
    return w1, w3, w2


def make_layer(cfg: MoEConfig, threads: int = 8) -> LayerInputs:
    x, logits, w_gate = make_activations(cfg)
    w1, w3, w2 = make_weights(cfg, threads)
    return LayerInputs(cfg, x, logits, w1, w3, w2, w_gate)


def small_config(name: str, T: int, d: int, f: int, E: int, k: int, seed: int,
                 w_dtype: str = F32, x_dtype: str = F32,
                 zipf_s: Optional[float] = None) -> MoEConfig:
    return MoEConfig(name, T, d, f, E, k, w_dtype, x_dtype, seed, zipf_s)
