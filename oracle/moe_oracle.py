"""ctypes front-end of the fp64 C oracle (oracle/moe_oracle.c) -- test
infrastructure only.  Arrays in, arrays out; all arithmetic is in the C file."""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        for name in ("oracle_route", "oracle_permute", "oracle_expert_ffn", "oracle_combine",
                     "oracle_rmsnorm", "oracle_router_logits", "oracle_num_threads"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what}: oracle status {rc}")


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def route(logits: np.ndarray, k: int):
    """logits fp32 [T,E] -> idx int32 [T,k], w fp64 [T,k]."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    idx = np.zeros((T, k), dtype=np.int32)
    w = np.zeros((T, k), dtype=np.float64)
    _check(lib().oracle_route(_p(logits), C.c_long(T), C.c_int(E), C.c_int(k), _p(idx), _p(w)),
           "route")
    return idx, w


def permute(idx: np.ndarray, E: int, x: np.ndarray):
    """idx int32 [T,k], x fp64 [T,d] -> counts[E], offsets[E+1], perm[N], inv_perm[N], xg[N,d]."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    x = np.ascontiguousarray(x, dtype=np.float64)
    T, k = idx.shape
    d = x.shape[1]
    N = T * k
    counts = np.zeros(E, dtype=np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    perm = np.zeros(N, dtype=np.int32)
    inv_perm = np.zeros(N, dtype=np.int32)
    xg = np.zeros((N, d), dtype=np.float64)
    _check(lib().oracle_permute(_p(idx), C.c_long(T), C.c_int(E), C.c_int(k), _p(x), C.c_long(d),
                                _p(counts), _p(offsets), _p(perm), _p(inv_perm), _p(xg)),
           "permute")
    return counts, offsets, perm, inv_perm, xg


def expert_ffn(xg: np.ndarray, offsets: np.ndarray, w1: np.ndarray, w3: np.ndarray,
               w2: np.ndarray) -> np.ndarray:
    """xg fp64 [N,d]; w1,w3 [E,d,f], w2 [E,f,d] as fp32 or bf16 bits (uint16) -> yg fp64 [N,d]."""
    xg = np.ascontiguousarray(xg, dtype=np.float64)
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    if w1.dtype not in (np.float32, np.uint16) or w3.dtype != w1.dtype or w2.dtype != w1.dtype:
        raise ValueError("weights must all be float32 or all uint16 (bf16 bits)")
    w1 = np.ascontiguousarray(w1)
    w3 = np.ascontiguousarray(w3)
    w2 = np.ascontiguousarray(w2)
    E, d, f = w1.shape
    if w3.shape != (E, d, f) or w2.shape != (E, f, d) or xg.shape[1] != d:
        raise ValueError("shape mismatch")
    if offsets.shape != (E + 1,) or offsets[0] != 0 or offsets[E] != xg.shape[0]:
        raise ValueError("offsets do not cover xg")
    yg = np.zeros_like(xg)
    _check(lib().oracle_expert_ffn(_p(xg), _p(offsets), C.c_int(E), C.c_long(d), C.c_long(f),
                                   _p(w1), _p(w3), _p(w2), C.c_int(int(w1.dtype == np.uint16)),
                                   _p(yg)), "expert_ffn")
    return yg


def combine(yg: np.ndarray, inv_perm: np.ndarray, w: np.ndarray) -> np.ndarray:
    """yg fp64 [N,d], inv_perm int32 [N], w fp64 [T,k] -> y fp64 [T,d]."""
    yg = np.ascontiguousarray(yg, dtype=np.float64)
    inv_perm = np.ascontiguousarray(inv_perm, dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=np.float64)
    T, k = w.shape
    d = yg.shape[1]
    y = np.zeros((T, d), dtype=np.float64)
    _check(lib().oracle_combine(_p(yg), _p(inv_perm), _p(w), C.c_long(T), C.c_int(k), C.c_long(d),
                                _p(y)), "combine")
    return y


def layer(x: np.ndarray, logits: np.ndarray, w1, w3, w2, k: int) -> dict:
    """The whole layer, step by step; returns every intermediate."""
    E = w1.shape[0]
    idx, w = route(logits, k)
    counts, offsets, perm, inv_perm, xg = permute(idx, E, x)
    yg = expert_ffn(xg, offsets, w1, w3, w2)
    y = combine(yg, inv_perm, w)
    return dict(idx=idx, w=w, counts=counts, offsets=offsets, perm=perm, inv_perm=inv_perm,
                xg=xg, yg=yg, y=y)


def rmsnorm(x: np.ndarray, eps: float = 1e-5) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    h = np.zeros_like(x)
    _check(lib().oracle_rmsnorm(_p(x), C.c_long(x.shape[0]), C.c_long(x.shape[1]),
                                C.c_double(eps), _p(h)), "rmsnorm")
    return h


def router_logits(h: np.ndarray, w_gate: np.ndarray) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.float64)
    w_gate = np.ascontiguousarray(w_gate, dtype=np.float32)
    T, d = h.shape
    E = w_gate.shape[1]
    out = np.zeros((T, E), dtype=np.float32)
    _check(lib().oracle_router_logits(_p(h), _p(w_gate), C.c_long(T), C.c_long(d), C.c_int(E),
                                      _p(out)), "router_logits")
    return out


def stack(x0: np.ndarray, layers, k: int, eps: float = 1e-5, forced_logits=None) -> dict:
    """Layer stack: per layer h = rmsnorm(x); logits = fp32(h . W_g); y = layer(h, logits);
    x <- x + y.  layers: list of (w_gate fp32 [d,E], w1, w3, w2).  With forced_logits (one
    fp32 [T,E] array per layer) routing uses those logits instead of the oracle's own
    (teacher forcing, so that routing can be compared bit for bit while activations drift
    within tolerance).  Returns the final x, every layer's routing indices and the oracle's
    own logits."""
    x = np.array(x0, dtype=np.float64)
    idx_all, own_logits = [], []
    for li, (w_gate, w1, w3, w2) in enumerate(layers):
        h = rmsnorm(x, eps)
        lg_own = router_logits(h, w_gate)
        own_logits.append(lg_own)
        lg = lg_own if forced_logits is None else np.ascontiguousarray(forced_logits[li],
                                                                       dtype=np.float32)
        out = layer(h, lg, w1, w3, w2, k)
        idx_all.append(out["idx"])
        x = x + out["y"]
    return dict(x=x, idx=idx_all, logits=own_logits)
