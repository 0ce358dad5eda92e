"""ctypes binding of include/moe.h.  Argument marshalling only: tensors become
device pointers, outputs are allocated with torch when the caller passes none,
and a non-zero status raises MoeError.  Same names as the C entry points."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

MOE_F32, MOE_BF16 = 0, 1
MOE_FFN_AUTO, MOE_FFN_STREAM, MOE_FFN_GROUPED, MOE_FFN_MID = 0, 1, 2, 3

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libmoe_hip.so")
_lib = None

# entry points of include/moe.h and of include/moe_probe.h
EXPORTS = ("moe_status_string", "moe_route", "moe_permute", "moe_weights_pack",
           "moe_weights_free", "moe_weights_bytes", "moe_expert_ffn_workspace",
           "moe_expert_ffn", "moe_expert_ffn_path", "moe_expert_ffn_plan",
           "moe_expert_ffn_parts", "moe_expert_ffn_tokens", "moe_expert_ffn_noalloc", "moe_expert_ffn_noalloc_max_bytes",
           "moe_combine", "moe_combine_parts", "moe_decode_layer", "moe_decode_block",
           "moe_rmsnorm", "moe_router_logits", "moe_residual_add", "moe_route_permute",
           "moe_norm_route_permute", "moe_combine_residual", "moe_combine_norm_route_permute",
           "moe_rmsnorm_router_logits", "moe_gate_sums", "moe_gate_sums_stride",
           "moe_decode_block_supported")
PROBE_EXPORTS = ("moe_set_ffn_mid_event", "moe_mfma_rate_probe", "moe_hbm_read_probe")
ORCH_EXPORTS = ("moe_orch_place", "moe_orch_hit_rate", "moe_orch_decide", "moe_orch_cpu_expert_ffn",
                "moe_orch_layer_create", "moe_orch_layer_free", "moe_orch_calibrate",
                "moe_orch_expert_ffn")
ORCH_SKIP, ORCH_GPU_RESIDENT, ORCH_GPU_TRANSFER, ORCH_CPU = 0, 1, 2, 3


class OrchLatency(C.Structure):
    """moe_orch_latency_t."""
    _fields_ = [("gpu_lat_us", C.c_double), ("cpu_lat_us_per_row", C.c_double),
                ("transfer_lat_us", C.c_double)]


class FfnPlan(C.Structure):
    """moe_ffn_plan_t."""
    _fields_ = [("path", C.c_int), ("n_parts", C.c_int),
                ("up_tile_rows", C.c_int), ("up_tile_features", C.c_int),
                ("down_tile_rows", C.c_int), ("down_tile_features", C.c_int)]


class MoeError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {moe_status_string(status)} (status {status})")


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2402_07033_amd.build` "
                "(there is no CPU fallback)")
        L = C.CDLL(_LIB_PATH)
        L.moe_status_string.restype = C.c_char_p
        L.moe_status_string.argtypes = [C.c_int]
        L.moe_weights_bytes.restype = C.c_size_t
        L.moe_weights_bytes.argtypes = [C.c_void_p]
        L.moe_expert_ffn_workspace.restype = C.c_size_t
        L.moe_expert_ffn_workspace.argtypes = [C.c_int] * 5
        vp, i32, f32 = C.c_void_p, C.c_int, C.c_float
        L.moe_route.argtypes = [vp, i32, i32, i32, vp, vp, vp]
        L.moe_permute.argtypes = [vp, i32, i32, i32, vp, i32, i32, vp, vp, vp, vp, vp, vp]
        L.moe_weights_pack.argtypes = [vp, vp, vp, i32, i32, i32, i32, C.POINTER(vp), vp]
        L.moe_weights_free.argtypes = [vp]
        L.moe_expert_ffn.argtypes = [vp, vp, i32, vp, i32, vp, C.c_size_t, vp, vp]
        L.moe_expert_ffn_path.argtypes = [vp, vp, i32, vp, i32, vp, C.c_size_t, vp, i32, vp]
        L.moe_combine.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
        L.moe_rmsnorm.argtypes = [vp, i32, i32, f32, vp, vp]
        L.moe_router_logits.argtypes = [vp, vp, i32, i32, i32, vp, vp]
        L.moe_residual_add.argtypes = [vp, vp, i32, i32, vp]
        L.moe_rmsnorm_router_logits.argtypes = [vp, vp, i32, i32, i32, f32, vp, vp, vp]
        L.moe_rmsnorm_router_logits.restype = C.c_int
        L.moe_set_ffn_mid_event.argtypes = [vp]
        L.moe_set_ffn_mid_event.restype = C.c_int
        L.moe_mfma_rate_probe.argtypes = [vp, i32, vp, C.POINTER(C.c_double), vp]
        L.moe_mfma_rate_probe.restype = C.c_int
        L.moe_hbm_read_probe.argtypes = [vp, C.c_size_t, vp, vp]
        L.moe_hbm_read_probe.restype = C.c_int
        L.moe_route_permute.argtypes = [vp, i32, i32, i32, vp, i32] + [vp] * 8
        L.moe_route_permute.restype = C.c_int
        L.moe_norm_route_permute.argtypes = [vp, vp, i32, i32, i32, i32, f32] + [vp] * 10
        L.moe_norm_route_permute.restype = C.c_int
        L.moe_combine_residual.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
        L.moe_combine_residual.restype = C.c_int
        L.moe_combine_norm_route_permute.argtypes = ([vp, i32, vp, vp, i32, vp, vp, vp] + [i32] * 4 +
                                                     [f32] + [vp] * 10)
        L.moe_combine_norm_route_permute.restype = C.c_int
        L.moe_expert_ffn_tokens.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, C.c_size_t, vp, vp]
        L.moe_expert_ffn_tokens.restype = C.c_int
        L.moe_expert_ffn_noalloc.argtypes = [vp, vp, i32, vp, i32, vp, vp]
        L.moe_expert_ffn_noalloc.restype = C.c_int
        L.moe_expert_ffn_noalloc_max_bytes.argtypes = []
        L.moe_expert_ffn_noalloc_max_bytes.restype = C.c_size_t
        L.moe_expert_ffn_plan.argtypes = [i32] * 6 + [C.POINTER(FfnPlan)]
        L.moe_expert_ffn_plan.restype = C.c_int
        L.moe_expert_ffn_parts.argtypes = [vp, vp, i32, vp, i32, vp, C.c_size_t, vp, i32,
                                           C.POINTER(C.c_int), vp]
        L.moe_expert_ffn_parts.restype = C.c_int
        L.moe_combine_parts.argtypes = [vp, i32, vp, vp, i32, i32, i32, vp, i32, vp, vp]
        L.moe_combine_parts.restype = C.c_int
        L.moe_decode_layer.argtypes = [vp, vp, vp, i32, i32] + [vp] * 8 + [C.c_size_t, vp, vp, vp]
        L.moe_decode_layer.restype = C.c_int
        L.moe_decode_block.argtypes = ([vp, vp, vp, i32, f32, vp, i32, i32] + [vp] * 7 +
                                       [C.c_size_t, vp, vp, vp, vp])
        L.moe_decode_block.restype = C.c_int
        L.moe_decode_block_supported.argtypes = [i32] * 6
        L.moe_decode_block_supported.restype = C.c_int
        L.moe_gate_sums.argtypes = [vp, vp, i32, i32, i32, vp, vp]
        L.moe_gate_sums.restype = C.c_int
        L.moe_gate_sums_stride.argtypes = [i32, i32]
        L.moe_gate_sums_stride.restype = C.c_size_t
        dp = C.POINTER(C.c_double)
        L.moe_orch_place.argtypes = [vp, i32, i32, i32, vp]
        L.moe_orch_hit_rate.argtypes = [vp, vp, i32, i32]
        L.moe_orch_hit_rate.restype = C.c_double
        L.moe_orch_decide.argtypes = [vp, vp, i32, C.POINTER(OrchLatency), vp]
        L.moe_orch_cpu_expert_ffn.argtypes = [vp, i32, vp, vp, vp, i32, i32, vp]
        L.moe_orch_layer_create.argtypes = [vp, vp, vp, i32, i32, i32, vp, i32, C.POINTER(vp), vp]
        L.moe_orch_layer_free.argtypes = [vp]
        L.moe_orch_calibrate.argtypes = [vp, vp, C.c_size_t, C.POINTER(OrchLatency), vp]
        L.moe_orch_expert_ffn.argtypes = [vp, C.POINTER(OrchLatency), vp, vp, i32, vp, C.c_size_t,
                                          vp, vp, vp]
        for n in ORCH_EXPORTS:
            if n != "moe_orch_hit_rate":
                getattr(L, n).restype = C.c_int
        del dp
        for n in ("moe_route", "moe_permute", "moe_weights_pack", "moe_weights_free",
                  "moe_expert_ffn", "moe_expert_ffn_path", "moe_combine", "moe_rmsnorm",
                  "moe_router_logits", "moe_residual_add", "moe_set_ffn_mid_event",
                  "moe_mfma_rate_probe", "moe_hbm_read_probe", "moe_route_permute",
                  "moe_norm_route_permute", "moe_combine_residual"):
            getattr(L, n).restype = C.c_int
        _lib = L
    return _lib


def moe_status_string(status: int) -> str:
    return lib().moe_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != 0:
        raise MoeError(status, what)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _dev(t: torch.Tensor, dtype, what: str):
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise TypeError(f"{what}: expected a contiguous device tensor of {dtype}")
    return t


def _act_dtype(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MOE_F32
    if t.dtype == torch.bfloat16:
        return MOE_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def moe_route(logits: torch.Tensor, k: int, idx=None, weights=None, stream=None):
    """logits fp32 [T,E] -> (idx int32 [T,k], weights fp32 [T,k])."""
    _dev(logits, torch.float32, "logits")
    T, E = logits.shape
    if idx is None:
        idx = torch.empty((T, k), dtype=torch.int32, device=logits.device)
    if weights is None:
        weights = torch.empty((T, k), dtype=torch.float32, device=logits.device)
    _check(lib().moe_route(_ptr(logits), T, E, k, _ptr(idx), _ptr(weights), _stream(stream)),
           "moe_route")
    return idx, weights


def moe_permute(idx: torch.Tensor, E: int, x: Optional[torch.Tensor] = None, out=None,
                stream=None):
    """idx int32 [T,k], x [T,d] -> (counts[E], offsets[E+1], perm[N], inv_perm[N], xg[N,d]).
    `out` may carry preallocated tensors in that order."""
    _dev(idx, torch.int32, "idx")
    T, k = idx.shape
    N = T * k
    dev = idx.device
    if out is None:
        i32 = dict(dtype=torch.int32, device=dev)
        out = (torch.empty(E, **i32), torch.empty(E + 1, **i32), torch.empty(N, **i32),
               torch.empty(N, **i32),
               None if x is None else torch.empty((N, x.shape[1]), dtype=x.dtype, device=dev))
    counts, offsets, perm, inv_perm, xg = out
    d, xdt = 0, MOE_F32
    if x is not None:
        if not x.is_cuda or not x.is_contiguous():
            raise TypeError("x: expected a contiguous device tensor")
        d, xdt = x.shape[1], _act_dtype(x)
    _check(lib().moe_permute(_ptr(idx), T, E, k, _ptr(x), d, xdt, _ptr(counts), _ptr(offsets),
                             _ptr(perm), _ptr(inv_perm), _ptr(xg), _stream(stream)),
           "moe_permute")
    return counts, offsets, perm, inv_perm, xg


class PackedWeights:
    """Owner of a moe_weights_t handle."""

    def __init__(self, handle: int, E: int, d: int, f: int, dtype: int):
        self.handle, self.E, self.d, self.f, self.dtype = handle, E, d, f, dtype

    @property
    def nbytes(self) -> int:
        return int(lib().moe_weights_bytes(C.c_void_p(self.handle))) if self.handle else 0

    def free(self):
        if self.handle:
            h, self.handle = self.handle, 0
            _check(lib().moe_weights_free(C.c_void_p(h)), "moe_weights_free")

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def moe_weights_pack(w1: torch.Tensor, w3: torch.Tensor, w2: torch.Tensor,
                     stream=None) -> PackedWeights:
    """w1, w3 [E,d,f], w2 [E,f,d], all fp32 or all bf16 device tensors."""
    dt = _act_dtype(w1)
    for t, n in ((w1, "w1"), (w3, "w3"), (w2, "w2")):
        _dev(t, w1.dtype, n)
    E, d, f = w1.shape
    if tuple(w3.shape) != (E, d, f) or tuple(w2.shape) != (E, f, d):
        raise ValueError("weight shapes must be w1,w3 [E,d,f] and w2 [E,f,d]")
    h = C.c_void_p()
    _check(lib().moe_weights_pack(_ptr(w1), _ptr(w3), _ptr(w2), E, d, f, dt, C.byref(h),
                                  _stream(stream)), "moe_weights_pack")
    return PackedWeights(h.value, E, d, f, dt)


def moe_weights_free(w: PackedWeights):
    w.free()


def moe_expert_ffn_workspace(N: int, E: int, d: int, f: int, act_dtype: int = MOE_F32) -> int:
    return int(lib().moe_expert_ffn_workspace(N, E, d, f, act_dtype))


def moe_expert_ffn(W: PackedWeights, xg: torch.Tensor, offsets: torch.Tensor, workspace=None,
                   yg=None, path: int = MOE_FFN_AUTO, stream=None):
    """xg [N,d] (fp32 or bf16), offsets int32 [E+1] on the device -> yg fp32 [N,d]."""
    _dev(offsets, torch.int32, "offsets")
    if not xg.is_cuda or not xg.is_contiguous():
        raise TypeError("xg: expected a contiguous device tensor")
    N = xg.shape[0]
    adt = _act_dtype(xg)
    if workspace is None:
        need = moe_expert_ffn_workspace(N, W.E, W.d, W.f, adt)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=xg.device)
    if yg is None:
        yg = torch.empty((N, W.d), dtype=torch.float32, device=xg.device)
    _check(lib().moe_expert_ffn_path(C.c_void_p(W.handle), _ptr(xg), adt, _ptr(offsets), N,
                                     _ptr(workspace), workspace.numel(), _ptr(yg), path,
                                     _stream(stream)), "moe_expert_ffn")
    return yg


def moe_expert_ffn_plan(N: int, E: int, d: int, f: int, w_dtype: int = MOE_BF16,
                        path: int = MOE_FFN_AUTO) -> dict:
    """What moe_expert_ffn would run for these sizes: kernel family, reduction parts,
    GROUPED tile shapes (host query)."""
    pl = FfnPlan()
    _check(lib().moe_expert_ffn_plan(N, E, d, f, w_dtype, path, C.byref(pl)), "moe_expert_ffn_plan")
    return {n: getattr(pl, n) for n, _ in FfnPlan._fields_}


def moe_expert_ffn_parts(W: "PackedWeights", xg: torch.Tensor, offsets: torch.Tensor, yg_parts,
                         workspace=None, stream=None) -> int:
    """moe_expert_ffn that leaves the second projection's reduction parts unsummed in
    yg_parts [max_parts, N, d]; returns the number of slabs written."""
    _dev(offsets, torch.int32, "offsets")
    _dev(yg_parts, torch.float32, "yg_parts")
    N = xg.shape[0]
    adt = _act_dtype(xg)
    if workspace is None:
        need = moe_expert_ffn_workspace(N, W.E, W.d, W.f, adt)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=xg.device)
    n = C.c_int(0)
    _check(lib().moe_expert_ffn_parts(C.c_void_p(W.handle), _ptr(xg), adt, _ptr(offsets), N,
                                      _ptr(workspace), workspace.numel(), _ptr(yg_parts),
                                      yg_parts.shape[0], C.byref(n), _stream(stream)),
           "moe_expert_ffn_parts")
    return int(n.value)


def moe_expert_ffn_tokens(W: "PackedWeights", x: torch.Tensor, k: int, perm: torch.Tensor,
                          offsets: torch.Tensor, workspace=None, yg=None, stream=None):
    """moe_expert_ffn reading row i as x[perm[i] / k]: no gathered copy.  x [T,d]."""
    _dev(perm, torch.int32, "perm")
    _dev(offsets, torch.int32, "offsets")
    if not x.is_cuda or not x.is_contiguous():
        raise TypeError("x: expected a contiguous device tensor")
    T = x.shape[0]
    N = T * k
    adt = _act_dtype(x)
    if workspace is None:
        need = moe_expert_ffn_workspace(N, W.E, W.d, W.f, adt)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    if yg is None:
        yg = torch.empty((N, W.d), dtype=torch.float32, device=x.device)
    _check(lib().moe_expert_ffn_tokens(C.c_void_p(W.handle), _ptr(x), adt, T, k, _ptr(perm),
                                       _ptr(offsets), _ptr(workspace), workspace.numel(),
                                       _ptr(yg), _stream(stream)), "moe_expert_ffn_tokens")
    return yg


def moe_expert_ffn_noalloc(W: "PackedWeights", xg: torch.Tensor, offsets: torch.Tensor,
                           yg: torch.Tensor, stream=None):
    """moe_expert_ffn on the library's static scratch: allocates nothing, so yg is the
    caller's (fp32 [N,d])."""
    _dev(offsets, torch.int32, "offsets")
    _dev(yg, torch.float32, "yg")
    if not xg.is_cuda or not xg.is_contiguous():
        raise TypeError("xg: expected a contiguous device tensor")
    _check(lib().moe_expert_ffn_noalloc(C.c_void_p(W.handle), _ptr(xg), _act_dtype(xg),
                                        _ptr(offsets), xg.shape[0], _ptr(yg), _stream(stream)),
           "moe_expert_ffn_noalloc")
    return yg


def moe_expert_ffn_noalloc_max_bytes() -> int:
    return int(lib().moe_expert_ffn_noalloc_max_bytes())


def moe_combine_parts(yg_parts: torch.Tensor, n_parts: int, inv_perm: torch.Tensor,
                      weights: torch.Tensor, y=None, residual: bool = False, yg=None, stream=None):
    """y[t] (+)= sum_j weights[t,j] * sum_p yg_parts[p, inv_perm[t*k+j]]; yg (optional)
    receives the summed rows."""
    _dev(yg_parts, torch.float32, "yg_parts")
    T, k = weights.shape
    d = yg_parts.shape[-1]
    if y is None:
        if residual:
            raise ValueError("residual=True needs y")
        y = torch.empty((T, d), dtype=torch.float32, device=yg_parts.device)
    _check(lib().moe_combine_parts(_ptr(yg_parts), n_parts, _ptr(inv_perm), _ptr(weights), T, k, d,
                                   _ptr(y), int(residual), _ptr(yg), _stream(stream)),
           "moe_combine_parts")
    return y


def moe_decode_layer(W: "PackedWeights", x: torch.Tensor, logits: torch.Tensor, k: int, idx=None,
                     weights=None, out=None, workspace=None, yg=None, y=None, want_xg=False,
                     stream=None) -> dict:
    """One decode step (T <= 16) in three launches: gate + first projection, second
    projection, combine.  `out` = (counts, offsets, perm, inv_perm, xg-or-None)."""
    _dev(x, torch.float32, "x")
    _dev(logits, torch.float32, "logits")
    T, d = x.shape
    E = logits.shape[1]
    N = T * k
    dev = x.device
    i32 = dict(dtype=torch.int32, device=dev)
    if idx is None:
        idx = torch.empty((T, k), **i32)
    if weights is None:
        weights = torch.empty((T, k), dtype=torch.float32, device=dev)
    if out is None:
        out = (torch.empty(E, **i32), torch.empty(E + 1, **i32), torch.empty(N, **i32),
               torch.empty(N, **i32),
               torch.empty((N, d), dtype=torch.float32, device=dev) if want_xg else None)
    counts, offsets, perm, inv_perm, xg = out
    if workspace is None:
        workspace = torch.empty(max(moe_expert_ffn_workspace(N, W.E, W.d, W.f, MOE_F32), 256),
                                dtype=torch.uint8, device=dev)
    if y is None:
        y = torch.empty((T, d), dtype=torch.float32, device=dev)
    _check(lib().moe_decode_layer(C.c_void_p(W.handle), _ptr(x), _ptr(logits), T, k, _ptr(idx),
                                  _ptr(weights), _ptr(counts), _ptr(offsets), _ptr(perm),
                                  _ptr(inv_perm), _ptr(xg), _ptr(workspace), workspace.numel(),
                                  _ptr(yg), _ptr(y), _stream(stream)), "moe_decode_layer")
    return dict(idx=idx, w=weights, counts=counts, offsets=offsets, perm=perm, inv_perm=inv_perm,
                xg=xg, yg=yg, y=y)


def moe_decode_block_supported(T: int, E: int, k: int, d: int, f: int, w_dtype: int = MOE_BF16) -> bool:
    """Does moe_decode_block serve these sizes on the current device (host query)?"""
    return bool(lib().moe_decode_block_supported(T, E, k, d, f, w_dtype))


def moe_gate_sums_stride(T: int, E: int) -> int:
    """Floats per share of the gating sums (host query)."""
    return int(lib().moe_gate_sums_stride(T, E))


def moe_gate_sums(x: torch.Tensor, w_gate: torch.Tensor, sums=None, stream=None):
    """x [T,d], w_gate [d,E] -> one share [stride] of the gating sums: x . w_gate[:, e] at
    t*(E+1)+e and sum(x^2) at t*(E+1)+E (the input of the first moe_decode_block of a stack)."""
    _dev(x, torch.float32, "x")
    _dev(w_gate, torch.float32, "w_gate")
    T, d = x.shape
    E = w_gate.shape[1]
    if sums is None:
        sums = torch.zeros(moe_gate_sums_stride(T, E), dtype=torch.float32, device=x.device)
    _check(lib().moe_gate_sums(_ptr(x), _ptr(w_gate), T, d, E, _ptr(sums), _stream(stream)),
           "moe_gate_sums")
    return sums


def moe_decode_block(W: "PackedWeights", x_in: torch.Tensor, k: int, gate_sums=None, n_shares: int = 0,
                     eps: float = 1e-5, logits=None, idx=None, weights=None, out=None,
                     workspace=None, x_out=None, w_gate_next=None, gate_sums_next=None,
                     stream=None) -> dict:
    """The expert layer of one block on the residual stream (T*k <= 4) in two launches:
    x_out = x_in + layer(rmsnorm(x_in)), the RMSNorm scale and the router logits derived from
    the gating sums `gate_sums` [n_shares, stride] (or, without them, layer(x_in) on the
    given logits), and with w_gate_next the d/16 shares of the next block's gating sums.
    `out` = (counts, offsets, perm, inv_perm)."""
    _dev(x_in, torch.float32, "x_in")
    T, d = x_in.shape
    E = W.E
    N = T * k
    dev = x_in.device
    i32 = dict(dtype=torch.int32, device=dev)
    f32 = dict(dtype=torch.float32, device=dev)
    if gate_sums is None:
        _dev(logits, torch.float32, "logits")
        n_shares = 0
    else:
        _dev(gate_sums, torch.float32, "gate_sums")
        if n_shares <= 0:
            n_shares = gate_sums.shape[0] if gate_sums.dim() == 2 else 1
        if logits is None:
            logits = torch.empty((T, E), **f32)
    if idx is None:
        idx = torch.empty((T, k), **i32)
    if weights is None:
        weights = torch.empty((T, k), **f32)
    if out is None:
        out = (torch.empty(E, **i32), torch.empty(E + 1, **i32), torch.empty(N, **i32),
               torch.empty(N, **i32))
    counts, offsets, perm, inv_perm = out[:4]
    if workspace is None:
        workspace = torch.empty(max(moe_expert_ffn_workspace(N, W.E, W.d, W.f, MOE_F32), 256),
                                dtype=torch.uint8, device=dev)
    if x_out is None:
        x_out = torch.empty((T, d), **f32)
    if w_gate_next is not None:
        _dev(w_gate_next, torch.float32, "w_gate_next")
        if gate_sums_next is None:
            gate_sums_next = torch.empty((d // 16, moe_gate_sums_stride(T, E)), **f32)
    _check(lib().moe_decode_block(C.c_void_p(W.handle), _ptr(x_in), _ptr(gate_sums), n_shares, eps,
                                  _ptr(logits), T, k, _ptr(idx), _ptr(weights), _ptr(counts),
                                  _ptr(offsets), _ptr(perm), _ptr(inv_perm), _ptr(workspace),
                                  workspace.numel(), _ptr(x_out), _ptr(w_gate_next),
                                  _ptr(gate_sums_next), _stream(stream)), "moe_decode_block")
    return dict(idx=idx, w=weights, counts=counts, offsets=offsets, perm=perm, inv_perm=inv_perm,
                logits=logits, x_out=x_out, gate_sums_next=gate_sums_next)


def moe_combine(yg: torch.Tensor, inv_perm: torch.Tensor, weights: torch.Tensor, y=None,
                stream=None):
    """yg fp32 [N,d], inv_perm int32 [N], weights fp32 [T,k] -> y fp32 [T,d]."""
    _dev(yg, torch.float32, "yg")
    _dev(inv_perm, torch.int32, "inv_perm")
    _dev(weights, torch.float32, "weights")
    T, k = weights.shape
    d = yg.shape[1]
    if y is None:
        y = torch.empty((T, d), dtype=torch.float32, device=yg.device)
    _check(lib().moe_combine(_ptr(yg), _ptr(inv_perm), _ptr(weights), T, k, d, _ptr(y),
                             _stream(stream)), "moe_combine")
    return y


def moe_rmsnorm(x: torch.Tensor, eps: float = 1e-5, h=None, stream=None):
    _dev(x, torch.float32, "x")
    if h is None:
        h = torch.empty_like(x)
    _check(lib().moe_rmsnorm(_ptr(x), x.shape[0], x.shape[1], eps, _ptr(h), _stream(stream)),
           "moe_rmsnorm")
    return h


def moe_router_logits(h: torch.Tensor, w_gate: torch.Tensor, logits=None, stream=None):
    _dev(h, torch.float32, "h")
    _dev(w_gate, torch.float32, "w_gate")
    T, d = h.shape
    E = w_gate.shape[1]
    if logits is None:
        logits = torch.empty((T, E), dtype=torch.float32, device=h.device)
    _check(lib().moe_router_logits(_ptr(h), _ptr(w_gate), T, d, E, _ptr(logits),
                                   _stream(stream)), "moe_router_logits")
    return logits


def moe_rmsnorm_router_logits(x: torch.Tensor, w_gate: torch.Tensor, eps: float = 1e-5, h=None,
                              logits=None, stream=None):
    """h = rmsnorm(x) and logits = h . w_gate in one launch (E <= 16)."""
    _dev(x, torch.float32, "x")
    T, d = x.shape
    E = w_gate.shape[1]
    if h is None:
        h = torch.empty_like(x)
    if logits is None:
        logits = torch.empty((T, E), dtype=torch.float32, device=x.device)
    _check(lib().moe_rmsnorm_router_logits(_ptr(x), _ptr(w_gate), T, d, E, eps, _ptr(h),
                                           _ptr(logits), _stream(stream)),
           "moe_rmsnorm_router_logits")
    return h, logits


def moe_residual_add(x: torch.Tensor, y: torch.Tensor, stream=None):
    _dev(x, torch.float32, "x")
    _dev(y, torch.float32, "y")
    _check(lib().moe_residual_add(_ptr(x), _ptr(y), x.shape[0], x.shape[1], _stream(stream)),
           "moe_residual_add")
    return x


def moe_set_ffn_mid_event(hip_event: Optional[int]):
    """hipEvent_t handle (int) recorded between the two projections, or None."""
    _check(lib().moe_set_ffn_mid_event(C.c_void_p(hip_event) if hip_event else None),
           "moe_set_ffn_mid_event")


def moe_mfma_rate_probe(operands: torch.Tensor, iters: int, out: torch.Tensor, stream=None) -> float:
    """Launch the matrix-core rate probe; returns the flop count of the launch."""
    flops = C.c_double()
    _check(lib().moe_mfma_rate_probe(_ptr(operands), iters, _ptr(out), C.byref(flops),
                                     _stream(stream)), "moe_mfma_rate_probe")
    return float(flops.value)


def moe_hbm_read_probe(data: torch.Tensor, sink: torch.Tensor, stream=None) -> int:
    """Launch the streaming-read probe over `data`; returns the number of bytes it reads."""
    nbytes = data.numel() * data.element_size()
    _check(lib().moe_hbm_read_probe(_ptr(data), C.c_size_t(nbytes), _ptr(sink), _stream(stream)),
           "moe_hbm_read_probe")
    cus = torch.cuda.get_device_properties(data.device).multi_processor_count
    per_wave = nbytes // (cus * 8 * 1024 * 16) * 16
    return per_wave * 1024 * 8 * cus


def moe_layer(W: PackedWeights, x: torch.Tensor, logits: torch.Tensor, k: int,
              path: int = MOE_FFN_AUTO, workspace=None, stream=None) -> dict:
    """The four calls of the hot path in order; returns every intermediate."""
    idx, w = moe_route(logits, k, stream=stream)
    counts, offsets, perm, inv_perm, xg = moe_permute(idx, W.E, x, stream=stream)
    yg = moe_expert_ffn(W, xg, offsets, workspace=workspace, path=path, stream=stream)
    y = moe_combine(yg, inv_perm, w, stream=stream)
    return dict(idx=idx, w=w, counts=counts, offsets=offsets, perm=perm, inv_perm=inv_perm,
                xg=xg, yg=yg, y=y)


def moe_route_permute(logits: torch.Tensor, k: int, x: torch.Tensor, idx, weights, out,
                      stream=None):
    """Fused moe_route + moe_permute for T <= 16 (fp32 x); outputs as in the two calls."""
    T, E = logits.shape
    counts, offsets, perm, inv_perm, xg = out
    _check(lib().moe_route_permute(_ptr(logits), T, E, k, _ptr(x), x.shape[1], _ptr(idx),
                                   _ptr(weights), _ptr(counts), _ptr(offsets), _ptr(perm),
                                   _ptr(inv_perm), _ptr(xg), _stream(stream)), "moe_route_permute")
    return idx, weights, out


def moe_norm_route_permute(x: torch.Tensor, w_gate: torch.Tensor, k: int, eps: float, h, logits,
                           idx, weights, out, stream=None):
    """Fused rmsnorm + router logits + route + permute for T <= 4."""
    T, d = x.shape
    E = w_gate.shape[1]
    counts, offsets, perm, inv_perm, xg = out
    _check(lib().moe_norm_route_permute(_ptr(x), _ptr(w_gate), T, d, E, k, eps, _ptr(h),
                                        _ptr(logits), _ptr(idx), _ptr(weights), _ptr(counts),
                                        _ptr(offsets), _ptr(perm), _ptr(inv_perm), _ptr(xg),
                                        _stream(stream)), "moe_norm_route_permute")
    return out


def moe_combine_residual(yg: torch.Tensor, inv_perm: torch.Tensor, weights: torch.Tensor,
                         x: torch.Tensor, stream=None):
    """x[t] += sum_j weights[t,j] * yg[inv_perm[t*k+j]] in one launch."""
    T, k = weights.shape
    _check(lib().moe_combine_residual(_ptr(yg), _ptr(inv_perm), _ptr(weights), T, k, yg.shape[1],
                                      _ptr(x), _stream(stream)), "moe_combine_residual")
    return x


def moe_combine_norm_route_permute(yg_prev, inv_perm_prev, weights_prev, x_in, x_out, w_gate,
                                   k: int, eps: float, h, logits, idx, weights, out, stream=None,
                                   n_parts_prev: int = 1):
    """Seam between two blocks in one launch: x_out = x_in + combine(yg_prev), then the
    fused front end of the next block on x_out (T <= 4).  yg_prev may hold n_parts_prev
    unsummed reduction parts.  Outputs must not alias the *_prev inputs."""
    T, d = x_in.shape
    E = w_gate.shape[1]
    counts, offsets, perm, inv_perm, xg = out
    _check(lib().moe_combine_norm_route_permute(
        _ptr(yg_prev), n_parts_prev, _ptr(inv_perm_prev), _ptr(weights_prev), weights_prev.shape[1],
        _ptr(x_in),
        _ptr(x_out), _ptr(w_gate), T, d, E, k, eps, _ptr(h), _ptr(logits), _ptr(idx),
        _ptr(weights), _ptr(counts), _ptr(offsets), _ptr(perm), _ptr(inv_perm), _ptr(xg),
        _stream(stream)), "moe_combine_norm_route_permute")
    return out


class StackBuffers:
    """Preallocated device buffers for moe_stack_forward (one layer's worth, reused).  The
    routing outputs exist twice (sets 0 and 1, used by even and odd layers) because the
    one-launch seam between two blocks reads the previous block's while writing the next
    block's; x_alt is the second residual-stream buffer of that seam."""

    def __init__(self, T: int, E: int, k: int, d: int, f: int, device="cuda"):
        N = T * k
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.h = torch.empty((T, d), **f32)
        self.logits = torch.empty((T, E), **f32)
        self.xg = torch.empty((N, d), **f32)
        self.sets = [dict(idx=torch.empty((T, k), **i32), w=torch.empty((T, k), **f32),
                          perm_out=(torch.empty(E, **i32), torch.empty(E + 1, **i32),
                                    torch.empty(N, **i32), torch.empty(N, **i32), self.xg))
                     for _ in range(2)]
        self.idx, self.w, self.perm_out = (self.sets[0][n] for n in ("idx", "w", "perm_out"))
        self.x_alt = torch.empty((T, d), **f32)
        self.ws = torch.empty(max(moe_expert_ffn_workspace(N, E, d, f, MOE_F32), 256),
                              dtype=torch.uint8, device=device)
        # the second projection's reduction parts (decode kernels; slab 0 is yg otherwise)
        try:
            plan = moe_expert_ffn_plan(N, E, d, f, MOE_BF16)
        except MoeError:   # a shape only the fp32 kernels serve
            plan = dict(n_parts=1, path=MOE_FFN_STREAM)
        self.max_parts = max(1, plan["n_parts"])
        # prefill-sized passes read the normalised rows through perm: no gathered copy
        self.rows_through_perm = plan["path"] != MOE_FFN_STREAM
        self.yg_parts = torch.empty((self.max_parts, N, d), **f32)
        self.yg = self.yg_parts[0]
        self.y = torch.empty((T, d), **f32)
        # the two-launch block step (moe_decode_block): the shares of the gating sums of the
        # current and of the next block
        stride = moe_gate_sums_stride(T, E) if E <= 16 else 0
        self.gate_sums = [torch.zeros((max(d // 16, 1), max(stride, 4)), **f32) for _ in range(2)]


def moe_stack_forward(layers, x: torch.Tensor, k: int, eps: float = 1e-5, bufs=None,
                      logits_out=None, idx_out=None, on_layer=None, fused: bool = True,
                      stream=None, seam: bool = True):
    """The layer-stack workload: for every (PackedWeights, w_gate) in `layers`
        h = rmsnorm(x); logits = h . w_gate; y = moe_layer(h, logits); x += y
    x (fp32 [T,d]) is updated in place.  logits_out / idx_out, when given, are lists
    that receive a copy of every layer's router logits / expert indices.  on_layer(l)
    is called before each layer's expert FFN is enqueued (measurement hook).  fused=True
    uses the one-launch front end (T <= 4) and combine+residual, and with seam=True also
    folds each block's combine+residual into the next block's front end -- or, with at most
    four routed rows, runs every block as the two launches of moe_decode_block; fused=False
    the separate calls.  The fused variants leave the second projection's reduction parts
    unsummed and add them inside the combine (no separate launch)."""
    _dev(x, torch.float32, "x")
    T, d = x.shape
    W0 = layers[0][0]
    if bufs is None:
        bufs = StackBuffers(T, W0.E, k, d, W0.f, x.device)
    fused_gate = fused and T <= 4 and W0.E <= 16
    seam = seam and fused_gate
    if seam and W0.dtype == MOE_BF16 and moe_decode_block_supported(T, W0.E, k, d, W0.f):
        # at most four routed rows: two launches per block, nothing between two blocks
        moe_gate_sums(x, layers[0][1], bufs.gate_sums[0], stream=stream)
        n_shares = 1
        for li, (W, _) in enumerate(layers):
            a, b = li & 1, (li + 1) & 1
            rs = bufs.sets[a]
            if on_layer is not None:
                on_layer(li)
            w_next = layers[li + 1][1] if li + 1 < len(layers) else None
            moe_decode_block(W, x, k, gate_sums=bufs.gate_sums[a], n_shares=n_shares, eps=eps,
                             logits=bufs.logits, idx=rs["idx"], weights=rs["w"], out=rs["perm_out"],
                             workspace=bufs.ws, x_out=x, w_gate_next=w_next,
                             gate_sums_next=bufs.gate_sums[b], stream=stream)
            n_shares = d // 16
            if logits_out is not None:
                logits_out.append(bufs.logits.clone())
            if idx_out is not None:
                idx_out.append(rs["idx"].clone())
        return x
    # the seam kernel adds at most 4 parts
    use_parts = fused and (not seam or bufs.max_parts <= 4)
    n_parts = 1
    cur = x  # residual stream: alternates between x and bufs.x_alt across seams
    for li, (W, w_gate) in enumerate(layers):
        rs = bufs.sets[li & 1]
        if fused_gate and seam and li > 0:
            prev = bufs.sets[(li - 1) & 1]
            nxt = bufs.x_alt if cur is x else x
            moe_combine_norm_route_permute(bufs.yg_parts, prev["perm_out"][3], prev["w"], cur, nxt,
                                           w_gate, k, eps, bufs.h, bufs.logits, rs["idx"],
                                           rs["w"], rs["perm_out"], stream=stream,
                                           n_parts_prev=n_parts)
            cur = nxt
            _, offsets, _, inv_perm, xg = rs["perm_out"]
        elif fused_gate:
            moe_norm_route_permute(cur, w_gate, k, eps, bufs.h, bufs.logits, rs["idx"], rs["w"],
                                   rs["perm_out"], stream=stream)
            _, offsets, _, inv_perm, xg = rs["perm_out"]
        else:
            if fused and W0.E <= 16:
                moe_rmsnorm_router_logits(cur, w_gate, eps, bufs.h, bufs.logits, stream=stream)
            else:
                moe_rmsnorm(cur, eps, bufs.h, stream=stream)
                moe_router_logits(bufs.h, w_gate, bufs.logits, stream=stream)
            moe_route(bufs.logits, k, rs["idx"], rs["w"], stream=stream)
            if fused and bufs.rows_through_perm and W.dtype == MOE_BF16:
                po = rs["perm_out"][:4] + (None,)
                _, offsets, perm, inv_perm, xg = moe_permute(rs["idx"], W.E, None, out=po,
                                                             stream=stream)
            else:
                _, offsets, perm, inv_perm, xg = moe_permute(rs["idx"], W.E, bufs.h,
                                                             out=rs["perm_out"], stream=stream)
        if logits_out is not None:
            logits_out.append(bufs.logits.clone())
        if idx_out is not None:
            idx_out.append(rs["idx"].clone())
        if on_layer is not None:
            on_layer(li)
        if xg is None:
            n_parts = 1
            moe_expert_ffn_tokens(W, bufs.h, k, perm, offsets, workspace=bufs.ws, yg=bufs.yg,
                                  stream=stream)
        elif use_parts:
            n_parts = moe_expert_ffn_parts(W, xg, offsets, bufs.yg_parts, workspace=bufs.ws,
                                           stream=stream)
        else:
            moe_expert_ffn(W, xg, offsets, workspace=bufs.ws, yg=bufs.yg, stream=stream)
        if seam and li + 1 < len(layers):
            continue  # folded into the next block's front end
        if fused and n_parts > 1:
            moe_combine_parts(bufs.yg_parts, n_parts, inv_perm, rs["w"], y=cur, residual=True,
                              stream=stream)
        elif fused:
            moe_combine_residual(bufs.yg, inv_perm, rs["w"], cur, stream=stream)
        else:
            moe_combine(bufs.yg, inv_perm, rs["w"], bufs.y, stream=stream)
            moe_residual_add(cur, bufs.y, stream=stream)
    if cur is not x:
        x.copy_(cur)
    return x


# ---- the paper's own method over the expert kernels (include/moe_orch.h) ----------------

def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def moe_orch_place(popularity, capacity: int):
    """popularity [L,E] (numpy, host) -> at_gpu uint8 [L,E]: the `capacity` most popular."""
    import numpy as np
    pop = np.ascontiguousarray(popularity, dtype=np.float64)
    L, E = pop.shape
    at_gpu = np.zeros((L, E), dtype=np.uint8)
    _check(lib().moe_orch_place(_np_ptr(pop), L, E, capacity, _np_ptr(at_gpu)), "moe_orch_place")
    return at_gpu


def moe_orch_hit_rate(popularity, at_gpu) -> float:
    import numpy as np
    pop = np.ascontiguousarray(popularity, dtype=np.float64)
    ag = np.ascontiguousarray(at_gpu, dtype=np.uint8)
    L, E = pop.shape
    return float(lib().moe_orch_hit_rate(_np_ptr(pop), _np_ptr(ag), L, E))


def _latency(lat) -> OrchLatency:
    if isinstance(lat, OrchLatency):
        return lat
    return OrchLatency(lat["gpu_lat_us"], lat["cpu_lat_us_per_row"], lat["transfer_lat_us"])


def moe_orch_decide(at_gpu_layer, inp_size, lat):
    """Algorithm 1 for one layer (host arrays) -> int32 [E] of ORCH_* decisions."""
    import numpy as np
    ag = np.ascontiguousarray(at_gpu_layer, dtype=np.uint8)
    sz = np.ascontiguousarray(inp_size, dtype=np.int32)
    out = np.zeros(sz.shape[0], dtype=np.int32)
    cl = _latency(lat)
    _check(lib().moe_orch_decide(_np_ptr(ag), _np_ptr(sz), sz.shape[0], C.byref(cl), _np_ptr(out)),
           "moe_orch_decide")
    return out


def moe_orch_cpu_expert_ffn(x, w1, w3, w2):
    """Host-side expert: x fp32 [s,d], w1/w3 [d,f], w2 [f,d] bf16 bits (uint16) -> y fp32 [s,d]."""
    import numpy as np
    x = np.ascontiguousarray(x, dtype=np.float32)
    w1, w3, w2 = (np.ascontiguousarray(w, dtype=np.uint16) for w in (w1, w3, w2))
    s, d = x.shape
    f = w1.shape[1]
    y = np.zeros((s, d), dtype=np.float32)
    _check(lib().moe_orch_cpu_expert_ffn(_np_ptr(x), s, _np_ptr(w1), _np_ptr(w3), _np_ptr(w2), d, f,
                                         _np_ptr(y)), "moe_orch_cpu_expert_ffn")
    return y


class OrchLayer:
    """Owner of a moe_orch_layer_t handle: a layer split between device and host memory."""

    def __init__(self, w1, w3, w2, at_gpu, max_rows: int, stream=None):
        import numpy as np
        w1, w3, w2 = (np.ascontiguousarray(w, dtype=np.uint16) for w in (w1, w3, w2))
        self.E, self.d, self.f = w1.shape
        ag = np.ascontiguousarray(at_gpu, dtype=np.uint8)
        h = C.c_void_p()
        _check(lib().moe_orch_layer_create(_np_ptr(w1), _np_ptr(w3), _np_ptr(w2), self.E, self.d,
                                           self.f, _np_ptr(ag), max_rows, C.byref(h),
                                           _stream(stream)), "moe_orch_layer_create")
        self.handle, self.max_rows = h.value, max_rows
        self.ws = torch.empty(max(moe_expert_ffn_workspace(max_rows, 1, self.d, self.f, MOE_F32), 256),
                              dtype=torch.uint8, device="cuda")

    def calibrate(self, stream=None) -> dict:
        cl = OrchLatency()
        _check(lib().moe_orch_calibrate(C.c_void_p(self.handle), _ptr(self.ws), self.ws.numel(),
                                        C.byref(cl), _stream(stream)), "moe_orch_calibrate")
        return dict(gpu_lat_us=cl.gpu_lat_us, cpu_lat_us_per_row=cl.cpu_lat_us_per_row,
                    transfer_lat_us=cl.transfer_lat_us)

    def expert_ffn(self, lat, xg: torch.Tensor, offsets: torch.Tensor, yg=None, stream=None):
        """-> (yg fp32 [N,d], decisions int32 [E] as Algorithm 1 chose them)."""
        import numpy as np
        _dev(xg, torch.float32, "xg")
        _dev(offsets, torch.int32, "offsets")
        N = xg.shape[0]
        if yg is None:
            yg = torch.empty((N, self.d), dtype=torch.float32, device=xg.device)
        dec = np.zeros(self.E, dtype=np.int32)
        cl = _latency(lat)
        _check(lib().moe_orch_expert_ffn(C.c_void_p(self.handle), C.byref(cl), _ptr(xg),
                                         _ptr(offsets), N, _ptr(self.ws), self.ws.numel(),
                                         _ptr(yg), _np_ptr(dec), _stream(stream)),
               "moe_orch_expert_ffn")
        return yg, dec

    def free(self):
        if self.handle:
            h, self.handle = self.handle, 0
            _check(lib().moe_orch_layer_free(C.c_void_p(h)), "moe_orch_layer_free")

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass
