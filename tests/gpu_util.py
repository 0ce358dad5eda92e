"""Helpers shared by the GPU parity tests: host<->device conversion of the
seeded inputs and the error metric.  No arithmetic of the layer lives here."""
import numpy as np
import torch

import moe_inputs as mi


def to_dev(a: np.ndarray) -> torch.Tensor:
    """fp32/int32 array, or bf16 bit patterns (uint16) -> device tensor."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def pack_layer(li):
    """Upload one layer's expert matrices and repack them; the device sources are
    released once the repack has run."""
    import paper_2402_07033_amd as moe
    w1, w3, w2 = to_dev(li.w1), to_dev(li.w3), to_dev(li.w2)
    W = moe.moe_weights_pack(w1, w3, w2)
    torch.cuda.synchronize()
    del w1, w3, w2
    torch.cuda.empty_cache()
    return W


def max_rel(gpu: np.ndarray, ref: np.ndarray) -> float:
    """max|gpu - ref| / max|ref| over the whole array."""
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(np.asarray(gpu, dtype=np.float64) - ref)) /
                 max(float(np.max(np.abs(ref))), 1e-300))


def skewed_logits(T: int, E: int, seed: int, zipf=1.2, empty=()):
    """N(0,1) + ln Zipf pmf logits; experts in `empty` get -30 so they stay unused."""
    z = mi.normal_f32(seed, 2, (T, E)).astype(np.float64)
    lg = z + (mi.zipf_log_pmf(E, zipf)[None, :] if zipf else 0.0)
    for e in empty:
        lg[:, e] = -30.0
    return lg.astype(np.float32)
