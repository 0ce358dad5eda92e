"""Plain restatement of the paper's host-side policy (test infrastructure only): placement
by popularity (Sec. 3.4), the latency model and Algorithm 1 (Sec. 3.3).  Pure Python, in the
paper's order and notation; the library's moe_orch_* functions are checked against it."""
from __future__ import annotations

import numpy as np

SKIP, GPU_RESIDENT, GPU_TRANSFER, CPU = 0, 1, 2, 3


def place(popularity: np.ndarray, capacity: int) -> np.ndarray:
    """popularity [L,E] -> at_gpu [L,E] (0/1): as many experts as the capacity permits, in
    order of popularity (Sec. 3.4); the lower flat index first among equals."""
    pop = np.asarray(popularity, dtype=np.float64)
    flat = pop.reshape(-1)
    at_gpu = np.zeros(flat.shape, dtype=np.uint8)
    left = list(range(flat.size))
    for _ in range(min(capacity, flat.size)):
        best = left[0]
        for i in left:                      # first maximum: lower index wins ties
            if flat[i] > flat[best]:
                best = i
        at_gpu[best] = 1
        left.remove(best)
    return at_gpu.reshape(pop.shape)


def hit_rate(popularity: np.ndarray, at_gpu: np.ndarray) -> float:
    """Likelihood that a selected expert's weights are in GPU memory (App. Expert Popularity)."""
    pop = np.asarray(popularity, dtype=np.float64)
    total = pop.sum()
    return float((pop * (np.asarray(at_gpu) != 0)).sum() / total) if total > 0 else 0.0


def cpu_lat(s: int, lat: dict) -> float:
    return lat["cpu_lat_us_per_row"] * s       # proportional to the input size


def gpu_lat(s: int, lat: dict) -> float:
    return lat["gpu_lat_us"]                   # constant in the input size


def trans_lat(lat: dict) -> float:
    return lat["transfer_lat_us"]


def decide(at_gpu_layer, inp_size, lat: dict) -> np.ndarray:
    """Algorithm 1 for one layer: where each expert runs."""
    n_e = len(inp_size)
    out = np.zeros(n_e, dtype=np.int32)
    for j in range(n_e):
        s = int(inp_size[j])
        if s == 0:
            out[j] = SKIP
            continue
        if at_gpu_layer[j]:
            out[j] = GPU_RESIDENT
        elif cpu_lat(s, lat) > gpu_lat(s, lat) + trans_lat(lat):
            out[j] = GPU_TRANSFER
        else:
            out[j] = CPU
    return out
