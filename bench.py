#!/usr/bin/env python3
"""Benchmark of the MoE expert layer hot path on one MI355X.

A step = one pass of the whole hot path (gating, per-expert batching, expert
FFN, gate-weighted combine, through the C ABI) over one batch of synthetic,
Mixtral-8x7B-shaped input that is already resident in HBM.  Decode-sized
workloads (T <= 16) take the one-call step moe_decode_layer (three launches;
--four-calls times moe_route -> moe_permute -> moe_expert_ffn -> moe_combine
instead), the others the four calls.  Steps rotate over several independent
weight sets (layers) and inputs so that no step finds its expert matrices in
the last-level cache.

Prints ONE JSON line.  Headline: single-token decode (decode_t1), whole-job
tokens/s over exactly --steps steps, plus
  roofline     -- the dominant kernel (first projection of the expert FFN) timed
                  live with HIP events on the launch stream, against HBM peak
                  (decode-sized workloads) or bf16 MFMA peak (prefill), and the
                  whole step's fraction of the same peak (whole_step_frac);
  cpu_baseline -- the fp64 CPU oracle timed on this machine's host cores on a
                  bounded sample of the same workload (a baseline, not a target);
  workloads    -- the other workloads of the metric (prefill_t4096, beam_t16, the
                  32-layer stack at 1 and 512 tokens), each with its own
                  ms_per_step, roofline block and realised per-expert counts.
--workload NAME runs one workload alone (profiling, sweeps).
"""
import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published

# Where the HBM traffic of a workload's dominant kernel comes from: the committed rocprofv3
# summary of the same bench command (FETCH_SIZE / WRITE_SIZE means per dispatch, in KiB after
# the copy calibration's scale: FETCH x2, WRITE x1) and the kernels of the first projection.
# Read at run time; None when the summary or the kernel's row is missing.
TRAFFIC_SOURCES = {
    "decode_t1": ("stream_kernels_decode_t1.txt", (r"stream_kernel<16, 2,",)),
    "beam_t16": ("stream_kernels_beam_t16.txt", (r"stream_kernel<16, 2,",)),
    "e16_decode_t1": ("stream_kernels_e16_decode_t1.txt", (r"stream_kernel<16, 2,",)),
    "prefill_t4096": ("grouped_gemm_prefill_t4096.txt", (r"gg_gemm_kernel<true", r"gg_fixup_kernel<true",
                                                         r"gg_pack_kernel")),
    "e16_prefill_t4096": ("grouped_gemm_e16_prefill_t4096.txt",
                          (r"gg_gemm_kernel<true", r"gg_fixup_kernel<true", r"gg_pack_kernel")),
    # stacks: per layer; the workload multiplies by its number of layers
    "stack_t1": ("layer_stack_t1.txt", (r"stream_kernel<16, 2,",)),
    "stack_t512": ("layer_stack_t512.txt", (r"gg_gemm_kernel<true", r"gg_fixup_kernel<true",
                                            r"gg_pack_kernel")),
}


def traffic_from_profile(workload):
    """HBM bytes per launch of the workload's dominant kernel(s) from profiles/<summary>."""
    src = TRAFFIC_SOURCES.get(workload)
    if src is None:
        return None
    path = os.path.join(ROOT, "profiles", src[0])
    if not os.path.exists(path):
        return None
    section, kib = None, {"FETCH_SIZE": 0.0, "WRITE_SIZE": 0.0}
    seen = set()
    for line in open(path):
        if line.startswith("FETCH_SIZE per dispatch"):
            section = "FETCH_SIZE"
        elif line.startswith("WRITE_SIZE per dispatch"):
            section = "WRITE_SIZE"
        elif not line.strip():
            section = None
        elif section and " mean=" in line:
            name = line.strip()
            for pref in src[1]:
                if name.startswith(pref):
                    kib[section] += float(line.split("mean=")[1].split()[0])
                    seen.add((section, pref))
    if not any(sec == "FETCH_SIZE" for sec, _ in seen):
        return None
    return (2.0 * kib["FETCH_SIZE"] + 1.0 * kib["WRITE_SIZE"]) * 1024.0


WORKLOADS = {
    # name: (T, x dtype, zipf skew of the router logits, bound)
    "decode_t1": dict(T=1, x_bf16=False, zipf=None, bound="hbm"),
    "beam_t16": dict(T=16, x_bf16=False, zipf=1.2, bound="hbm"),
    "prefill_t4096": dict(T=4096, x_bf16=True, zipf=1.2, bound="mfma"),
    # 32-layer stack of MoE blocks (RMSNorm -> router -> experts -> residual), all ~90 GB of
    # expert matrices resident; a step is one pass through all layers
    # second layer shape (paper, App. E: a 16-expert top-2 model): d=4096, f=6400, E=16
    "e16_decode_t1": dict(T=1, x_bf16=False, zipf=None, bound="hbm", shape=(4096, 6400, 16, 2)),
    "e16_beam_t16": dict(T=16, x_bf16=False, zipf=1.2, bound="hbm", shape=(4096, 6400, 16, 2)),
    "e16_prefill_t4096": dict(T=4096, x_bf16=True, zipf=1.2, bound="mfma",
                              shape=(4096, 6400, 16, 2)),
    "stack_t1": dict(T=1, x_bf16=False, zipf=None, bound="hbm", layers=32),
    "stack_t512": dict(T=512, x_bf16=False, zipf=None, bound="hbm", layers=32),
}
D, F, E, K = 4096, 14336, 8, 2  # Mixtral-8x7B layer; main() replaces it by wl["shape"]


class HipEvents:
    """Minimal HIP event wrapper (torch.cuda.Event only sees torch's stream API;
    these are recorded on the raw stream handle the library launches on)."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]

    def create(self) -> int:
        ev = C.c_void_p()
        assert self.hip.hipEventCreate(C.byref(ev)) == 0
        return ev.value

    def record(self, ev: int, stream: int):
        assert self.hip.hipEventRecord(C.c_void_p(ev), C.c_void_p(stream)) == 0

    def elapsed_ms(self, a: int, b: int) -> float:
        assert self.hip.hipEventSynchronize(C.c_void_p(b)) == 0
        ms = C.c_float()
        assert self.hip.hipEventElapsedTime(C.byref(ms), C.c_void_p(a), C.c_void_p(b)) == 0
        return float(ms.value)

    def destroy(self, ev: int):
        self.hip.hipEventDestroy(C.c_void_p(ev))


def make_weight_set(torch, moe, seed):
    """Random-init bf16 expert matrices N(0, 1/fan_in), generated on the device
    (seeded torch generator), packed; returns (PackedWeights, host copy or None)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    w1 = torch.empty((E, D, F), dtype=torch.bfloat16, device="cuda")
    w3 = torch.empty((E, D, F), dtype=torch.bfloat16, device="cuda")
    w2 = torch.empty((E, F, D), dtype=torch.bfloat16, device="cuda")
    for e in range(E):
        w1[e] = (torch.randn((D, F), generator=g, device="cuda") * D ** -0.5).to(torch.bfloat16)
        w3[e] = (torch.randn((D, F), generator=g, device="cuda") * D ** -0.5).to(torch.bfloat16)
        w2[e] = (torch.randn((F, D), generator=g, device="cuda") * F ** -0.5).to(torch.bfloat16)
    W = moe.moe_weights_pack(w1, w3, w2)
    torch.cuda.synchronize()
    return W, (w1, w3, w2)


def make_inputs(torch, moe, wl, n_inputs, seed):
    import numpy as np
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    T = wl["T"]
    xs, lgs = [], []
    wg = torch.randn((D, E), generator=g, device="cuda") * D ** -0.5
    if wl["zipf"]:
        r = np.arange(1, E + 1, dtype=np.float64) ** (-wl["zipf"])
        bias = torch.tensor(np.log(r / r.sum()), dtype=torch.float32, device="cuda")
    for _ in range(n_inputs):
        x = torch.randn((T, D), generator=g, device="cuda")
        if wl["zipf"]:
            lg = torch.randn((T, E), generator=g, device="cuda") + bias[None, :]
        else:
            lg = moe.moe_router_logits(x, wg)
        if wl["x_bf16"]:
            x = x.to(torch.bfloat16)
        xs.append(x.contiguous())
        lgs.append(lg.contiguous())
    torch.cuda.synchronize()
    return xs, lgs


class Step:
    """Preallocated buffers + the C-ABI calls of one step."""

    def __init__(self, torch, moe, T, x_dtype, one_call=True, fused_gate=False,
                 gathered_copy=False):
        N = T * K
        self.one_call = (one_call and T <= 16 and N <= 64 and E <= 16 and x_dtype == torch.float32)
        self.fused_gate = fused_gate and not self.one_call and T <= 16 and x_dtype == torch.float32
        self.ffn_path = moe.MOE_FFN_AUTO
        i32 = dict(dtype=torch.int32, device="cuda")
        f32 = dict(dtype=torch.float32, device="cuda")
        self.moe = moe
        self.idx = torch.empty((T, K), **i32)
        self.w = torch.empty((T, K), **f32)
        # the one-call step and moe_expert_ffn_tokens read the token rows directly: no
        # gathered copy is asked for
        self.tokens_entry = not self.one_call and not self.fused_gate and not gathered_copy
        xg = (None if self.one_call or self.tokens_entry
              else torch.empty((N, D), dtype=x_dtype, device="cuda"))
        self.perm_out = (torch.empty(E, **i32), torch.empty(E + 1, **i32), torch.empty(N, **i32),
                         torch.empty(N, **i32), xg)
        adt = moe.MOE_BF16 if x_dtype == torch.bfloat16 else moe.MOE_F32
        self.ws = torch.empty(moe.moe_expert_ffn_workspace(N, E, D, F, adt), dtype=torch.uint8,
                              device="cuda")
        self.yg = None if self.one_call else torch.empty((N, D), **f32)
        self.y = torch.empty((T, D), **f32)

    @property
    def calls(self):
        if self.one_call:
            return "moe_decode_layer"
        if self.fused_gate:
            return "moe_route_permute, moe_expert_ffn, moe_combine"
        if self.tokens_entry:
            return "moe_route, moe_permute (indices only), moe_expert_ffn_tokens, moe_combine"
        return "moe_route, moe_permute, moe_expert_ffn, moe_combine"

    def run(self, W, x, logits, ev=None, events=None, stream=0):
        moe = self.moe
        if self.one_call:
            if ev is not None:
                events.record(ev[0], stream)
            moe.moe_decode_layer(W, x, logits, K, idx=self.idx, weights=self.w, out=self.perm_out,
                                 workspace=self.ws, y=self.y)
            if ev is not None:
                events.record(ev[2], stream)
            return
        if self.fused_gate:
            moe.moe_route_permute(logits, K, x, self.idx, self.w, self.perm_out)
            counts, offsets, perm, inv_perm, xg = self.perm_out
        else:
            moe.moe_route(logits, K, self.idx, self.w)
            counts, offsets, perm, inv_perm, xg = moe.moe_permute(
                self.idx, E, None if self.tokens_entry else x, out=self.perm_out)
        if ev is not None:
            events.record(ev[0], stream)
        if self.tokens_entry:
            moe.moe_expert_ffn_tokens(W, x, K, perm, offsets, workspace=self.ws, yg=self.yg)
        else:
            moe.moe_expert_ffn(W, xg, offsets, workspace=self.ws, yg=self.yg, path=self.ffn_path)
        if ev is not None:
            events.record(ev[2], stream)
        moe.moe_combine(self.yg, inv_perm, self.w, self.y)


def cpu_baseline(torch, wl, host_w, xs, lgs, budget_s=15.0):
    """The fp64 oracle, as it stands, on a bounded sample of this workload."""
    import numpy as np
    from oracle import moe_oracle as orc

    def host(t):
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()

    def f64(a):
        if a.dtype == np.uint16:
            return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        return a.astype(np.float64)

    w1, w3, w2 = (host(t) for t in host_w)
    T = wl["T"]
    done_tokens, t_used, i = 0, 0.0, 0
    per_call = max(1, min(T, 4))  # tokens per oracle call
    t_start = time.perf_counter()
    while True:
        x = f64(host(xs[i % len(xs)]))[:per_call]
        lg = host(lgs[i % len(lgs)])[:per_call]
        t0 = time.perf_counter()
        orc.layer(x, lg, w1, w3, w2, K)
        t_used += time.perf_counter() - t0
        done_tokens += per_call
        i += 1
        if time.perf_counter() - t_start > budget_s or done_tokens >= 512:
            break
    return dict(value=done_tokens / t_used, unit="tokens/s", cores=orc.num_threads(), kind="oracle",
                sample=f"{done_tokens} tokens of this workload, {per_call} per oracle call, "
                       f"one weight set, {t_used:.1f} s of fp64 CPU work")


PATH_NAMES = {0: "fp32", 1: "stream", 2: "grouped", 3: "mid"}


def kernel_label(moe, T, forced_path):
    """Name of the first-projection kernel that runs for T tokens, from the library's plan."""
    pl = moe.moe_expert_ffn_plan(T * K, E, D, F, moe.MOE_BF16, forced_path)
    fam = PATH_NAMES.get(pl["path"], str(pl["path"]))
    if fam == "stream":
        return "stream_kernel, first projection (x.w1, x.w3, silu*mul)", pl
    if fam == "mid":
        return "gg_pack + mid_kernel<UP> + mid_fixup (x.w1, x.w3, silu*mul)", pl
    return (f"gg_pack + gg_gemm_kernel<UP> {pl['up_tile_rows']}x{pl['up_tile_features']} tile "
            "+ fix-up (x.w1, x.w3, silu*mul)"), pl


def run_layer_workload(torch, moe, name, wl, sets, args, steps, warmup, host_w=None):
    """One single-layer workload over the given (rotated) weight sets -> result dict."""
    T = wl["T"]
    decode_like = wl["bound"] == "hbm"
    n_layers = len(sets)
    n_inputs = 16 if decode_like else 2
    xs, lgs = make_inputs(torch, moe, wl, n_inputs, 4242)
    step = Step(torch, moe, T, xs[0].dtype,
                one_call=not args.four_calls and args.ffn_path == "auto",
                fused_gate=args.fused_gate,
                gathered_copy=args.gathered_copy or args.ffn_path != "auto")
    step.ffn_path = {"auto": moe.MOE_FFN_AUTO, "stream": moe.MOE_FFN_STREAM,
                     "grouped": moe.MOE_FFN_GROUPED, "mid": moe.MOE_FFN_MID}[args.ffn_path]
    stream = torch.cuda.current_stream().cuda_stream
    events = HipEvents()

    def run_range(n, ev_list=None):
        for i in range(n):
            ev = ev_list[i] if ev_list is not None else None
            if ev is not None:
                moe.moe_set_ffn_mid_event(ev[1])
            step.run(sets[i % n_layers], xs[i % n_inputs], lgs[i % n_inputs], ev, events, stream)

    # realised per-expert counts of every input (outside any timed region)
    counts_all = []
    for i in range(n_inputs):
        step.run(sets[0], xs[i], lgs[i])
        torch.cuda.synchronize()
        counts_all.append(step.perm_out[0].cpu().tolist())

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB read + 1 GiB write
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    run_range(warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_range(steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps

    # second pass: HIP events around the two projection kernels of every step
    ev_list = [(events.create(), events.create(), events.create()) for _ in range(steps)]
    run_range(steps, ev_list)
    moe.moe_set_ffn_mid_event(None)
    torch.cuda.synchronize()
    up_ms = sum(events.elapsed_ms(a, b) for a, b, _ in ev_list) / steps
    dn_ms = sum(events.elapsed_ms(b, c) for _, b, c in ev_list) / steps
    for ev in ev_list:
        for e in ev:
            events.destroy(e)

    # algorithmic work of the dominant kernel (first projection), averaged over the steps
    act_sets = [sum(1 for c in counts_all[i % n_inputs] if c > 0) for i in range(steps)]
    n_active = sum(act_sets) / steps
    label, plan = kernel_label(moe, T, step.ffn_path)
    if step.one_call:
        label = "gating + " + label
    traffic = traffic_from_profile(name) if args.tokens is None and args.ffn_path == "auto" else None
    if decode_like:
        # bytes: w1 and w3 of every active expert, read once (2 * d * f bf16 each)
        up_bytes = n_active * 2 * D * F * 2
        achieved = up_bytes / (up_ms * 1e-3) / 1e9
        whole = n_active * 3 * D * F * 2 / (ms_per_step * 1e-3) / 1e9
        roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=achieved / HBM_PEAK_GBS, traffic=traffic, kernel=label,
                        kernel_ms=up_ms, second_projection_ms=dn_ms,
                        second_projection_GBs=n_active * D * F * 2 / (dn_ms * 1e-3) / 1e9,
                        mean_active_experts=n_active, whole_step_GBs=whole,
                        whole_step_frac=whole / HBM_PEAK_GBS)
    else:
        up_flops = T * K * 2 * 2 * D * F  # real rows only
        achieved = up_flops / (up_ms * 1e-3) / 1e12
        whole = T * K * 6 * D * F / (ms_per_step * 1e-3) / 1e12
        roofline = dict(bound="mfma", achieved=achieved, peak=MFMA_BF16_PEAK_TFLOPS,
                        unit="TFLOP/s", frac=achieved / MFMA_BF16_PEAK_TFLOPS, traffic=traffic,
                        kernel=label, kernel_ms=up_ms, second_projection_ms=dn_ms,
                        second_projection_TFLOPs=T * K * 2 * D * F / (dn_ms * 1e-3) / 1e12,
                        whole_step_TFLOPs=whole, whole_step_frac=whole / MFMA_BF16_PEAK_TFLOPS)
    if step.one_call:
        roofline["second_projection_note"] = (
            "second_projection_ms includes the combine (inside the second kernel at T*k <= 4, "
            "else its own launch)")

    result = {
        "metric": "MoE-layer tokens/s", "value": T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights x " + ("bf16" if wl["x_bf16"] else
                                      ("fp32 (bf16 hi+lo)" if plan["path"] == 1 else
                                       "fp32 (rounded to bf16)")) +
                 " activations, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": name, "T": T, "d_model": D, "d_ff": F, "experts": E,
                   "top_k": K, "weight_sets_rotated": n_layers, "inputs_rotated": n_inputs,
                   "counts_first_input": counts_all[0], "ffn_path": PATH_NAMES[plan["path"]],
                   "calls_per_step": step.calls},
        "roofline": roofline,
    }
    if host_w is not None:
        result["cpu_baseline"] = cpu_baseline(torch, wl, host_w, xs, lgs)
    return result


def make_stack_layers(torch, moe, L, keep_host_first=False):
    """L independent weight sets + router matrices (seeded), all resident."""
    g = torch.Generator(device="cuda")
    g.manual_seed(777)
    layers, host_w, host_gate = [], None, None
    for li in range(L):
        W, src = make_weight_set(torch, moe, 2000 + li)
        wg = (torch.randn((D, E), generator=g, device="cuda") * D ** -0.5).contiguous()
        if li == 0 and keep_host_first:
            host_w = tuple(t.cpu() for t in src)
            host_gate = wg.cpu()
        del src
        layers.append((W, wg))
    torch.cuda.empty_cache()
    return layers, host_w, host_gate


def run_stack_workload(torch, moe, name, wl, layers, args, steps, warmup, host_w=None,
                       host_gate=None):
    """Layer-stack workload: value = tokens/s through all layers, ms_per_step = stack time."""
    T, L = wl["T"], len(layers)
    g = torch.Generator(device="cuda")
    g.manual_seed(778)
    x0 = torch.randn((T, D), generator=g, device="cuda")
    x = torch.empty_like(x0)
    bufs = moe.StackBuffers(T, E, K, D, F)
    stream = torch.cuda.current_stream().cuda_stream
    events = HipEvents()

    def one_pass(ev=None):
        x.copy_(x0)

        def on_layer(li):
            if ev is not None:
                moe.moe_set_ffn_mid_event(ev[li][1])
                events.record(ev[li][0], stream)
        idx_out = [] if ev is not None else None
        moe.moe_stack_forward(layers, x, K, bufs=bufs, on_layer=on_layer, idx_out=idx_out)
        return idx_out

    for _ in range(warmup):
        one_pass()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        one_pass()
    t_enq = time.perf_counter()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    host_enqueue_ms = (t_enq - t0) * 1e3 / steps  # host time to issue one pass (no sync)

    # one more pass with events around each layer's first projection
    ev = [(events.create(), events.create()) for _ in range(L)]
    idx_out = one_pass(ev)
    moe.moe_set_ffn_mid_event(None)
    torch.cuda.synchronize()
    up_ms = sum(events.elapsed_ms(a, b) for a, b in ev)
    n_active = sum(len(set(t.cpu().flatten().tolist())) for t in idx_out)
    up_bytes = n_active * 2 * D * F * 2
    achieved = up_bytes / (up_ms * 1e-3) / 1e9
    all_bytes = n_active * 3 * D * F * 2
    whole_gbs = all_bytes / (ms_per_step * 1e-3) / 1e9
    whole_tf = T * K * 6 * D * F * L / (ms_per_step * 1e-3) / 1e12
    label, plan = kernel_label(moe, T, moe.MOE_FFN_AUTO)
    if moe.moe_decode_block_supported(T, E, K, D, F):
        label = "RMSNorm scale + router logits + gating + " + label   # moe_decode_block's first kernel
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=achieved / HBM_PEAK_GBS,
                    traffic=(lambda t: None if t is None else t * L)(traffic_from_profile(name)),
                    kernel=label + ", summed over the layers",
                    kernel_ms=up_ms, active_experts_all_layers=n_active,
                    whole_step_GBs=whole_gbs, whole_step_frac=whole_gbs / HBM_PEAK_GBS,
                    whole_step_TFLOPs=whole_tf,
                    whole_step_mfma_frac=whole_tf / MFMA_BF16_PEAK_TFLOPS)
    result = {
        "metric": "MoE-layer tokens/s", "value": T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights x fp32 activations" + (" (bf16 hi+lo)" if plan["path"] == 1 else
                                                      " (rounded to bf16)") + ", fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": name, "T": T, "layers": L, "d_model": D, "d_ff": F,
                   "experts": E, "top_k": K, "ffn_path": PATH_NAMES[plan["path"]],
                   "per_token_expert_time_us": ms_per_step * 1e3 / T,
                   "host_enqueue_ms": host_enqueue_ms,
                   "resident_expert_bytes": sum(W.nbytes for W, _ in layers)},
        "roofline": roofline,
    }
    if host_w is not None:
        # the oracle on a bounded sample: up to 4 tokens through ONE layer; the stack rate is
        # that per-layer rate divided by the number of layers (labelled extrapolated)
        import numpy as np
        from oracle import moe_oracle as orc
        w1, w3, w2 = (t.view(torch.int16).numpy().view(np.uint16) for t in host_w)
        n_tok = min(T, 4)
        xs = x0[:n_tok].cpu().numpy().astype(np.float64)
        reps, t_used = 0, 0.0
        while t_used < 12.0 and reps < 400:
            t0 = time.perf_counter()
            orc.stack(xs, [(host_gate.numpy(), w1, w3, w2)], K)
            t_used += time.perf_counter() - t0
            reps += 1
        per_layer_tokens_s = reps * n_tok / t_used
        result["cpu_baseline"] = dict(
            value=per_layer_tokens_s / L, unit="tokens/s", cores=orc.num_threads(), kind="oracle",
            sample=f"{reps} x {n_tok} tokens through 1 layer ({t_used:.1f} s of fp64 CPU work); "
                   f"stack rate extrapolated as the one-layer rate / {L} layers")
    return result


def nested(res):
    """The part of a workload's result that goes into the headline line's `workloads`."""
    keep = {k: res[k] for k in ("value", "unit", "steps", "warmup", "ms_per_step", "dtype")}
    keep["config"] = res["config"]
    keep["roofline"] = res["roofline"]
    return keep


def mfma_ceiling(torch, moe):
    """Sustained matrix-core rate of this board for constant and for random bf16 operands
    (register-resident MFMA loop, no memory traffic): context for the MFMA roofline."""
    events = HipEvents()
    stream = torch.cuda.current_stream().cuda_stream
    out = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
    res = {}
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    for name, ops in (("constant", torch.full((32768,), 0.5, dtype=torch.bfloat16, device="cuda")),
                      ("random_normal", torch.randn(32768, generator=g, device="cuda")
                       .to(torch.bfloat16))):
        moe.moe_mfma_rate_probe(ops, 200, out)
        torch.cuda.synchronize()
        e0, e1 = events.create(), events.create()
        events.record(e0, stream)
        flops = moe.moe_mfma_rate_probe(ops, 4000, out)
        events.record(e1, stream)
        ms = events.elapsed_ms(e0, e1)
        res[name] = flops / (ms * 1e-3) / 1e12
    return res


def hbm_ceiling(torch, moe):
    """Rate of a plain streaming read on this board (one launch per measurement over buffers
    that are rotated so that no launch finds its data in the last-level cache): context for
    the HBM roofline.  Sizes: the first and second projection's bytes at T=1, and 1 GiB."""
    events = HipEvents()
    stream = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    res = {}
    for name, nbytes in (("224MiB", 224 << 20), ("448MiB", 448 << 20), ("1GiB", 1 << 30)):
        nbuf = max(3, (3 << 30) // nbytes)
        g = torch.Generator(device="cuda")
        g.manual_seed(5)
        bufs = [torch.randint(0, 2 ** 31 - 1, (nbytes // 4,), dtype=torch.int32, device="cuda",
                              generator=g) for _ in range(nbuf)]
        for b in bufs[:2]:
            moe.moe_hbm_read_probe(b, sink)
        torch.cuda.synchronize()
        reps = 4 * nbuf
        e0, e1 = events.create(), events.create()
        events.record(e0, stream)
        read = 0
        for r in range(reps):
            read += moe.moe_hbm_read_probe(bufs[r % nbuf], sink)
        events.record(e1, stream)
        ms = events.elapsed_ms(e0, e1)
        res[name] = {"us_per_launch": ms * 1e3 / reps, "GBs": read / (ms * 1e-3) / 1e9}
        del bufs
        torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="all", choices=["all"] + sorted(WORKLOADS),
                    help="all (default): decode_t1 as the headline plus prefill_t4096, beam_t16, "
                         "stack_t1 and stack_t512 nested under `workloads`; else that one alone")
    ap.add_argument("--layers", type=int, default=None, help="independent weight sets rotated")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tokens", type=int, default=None,
                    help="override T of the workload (sweeps; the JSON names it)")
    ap.add_argument("--ffn-path", default="auto", choices=["auto", "stream", "grouped", "mid"],
                    help="force the expert-FFN kernel family (sweeps; implies --four-calls)")
    ap.add_argument("--four-calls", action="store_true",
                    help="decode-sized workloads: time moe_route, moe_permute, moe_expert_ffn, "
                         "moe_combine instead of the one-call moe_decode_layer")
    ap.add_argument("--gathered-copy", action="store_true",
                    help="four-call steps: let moe_permute write the gathered rows xg and run "
                         "moe_expert_ffn on them (default: moe_expert_ffn_tokens reads the token "
                         "rows through perm)")
    ap.add_argument("--fused-gate", action="store_true",
                    help="with --four-calls: use the one-launch moe_route_permute instead of "
                         "moe_route + moe_permute (same outputs)")
    ap.add_argument("--mfma-ceiling", action="store_true",
                    help="only measure the sustained matrix-core rate of this board")
    ap.add_argument("--hbm-ceiling", action="store_true",
                    help="only measure what a plain streaming read gets from HBM on this board")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (a known-size reference dispatch "
                         "for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
                 "use --gpus 1")

    import torch
    import paper_2402_07033_amd as moe
    moe.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.mfma_ceiling:
        print(json.dumps({"mfma_sustained_TFLOPs_bf16_16x16x32": mfma_ceiling(torch, moe),
                          "published_peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS}))
        return
    if args.hbm_ceiling:
        print(json.dumps({"hbm_streaming_read": hbm_ceiling(torch, moe),
                          "published_peak_GBs": HBM_PEAK_GBS}))
        return

    def defaults(wl):
        decode_like = wl["bound"] == "hbm"
        if "layers" in wl:
            return (20 if wl["T"] == 1 else 5), 2
        return (400 if decode_like else 30), (40 if decode_like else 5)

    global D, F, E, K
    if args.workload != "all":
        wl = dict(WORKLOADS[args.workload])
        D, F, E, K = wl.get("shape", (D, F, E, K))
        if args.tokens is not None:
            wl["T"] = args.tokens
        d_steps, d_warm = defaults(wl)
        steps = args.steps if args.steps is not None else d_steps
        warmup = args.warmup if args.warmup is not None else d_warm
        if "layers" in wl:
            L = args.layers if args.layers is not None else wl["layers"]
            layers, host_w, host_gate = make_stack_layers(torch, moe, L, not args.no_cpu_baseline)
            res = run_stack_workload(torch, moe, args.workload, wl, layers, args, steps, warmup,
                                     host_w, host_gate)
        else:
            decode_like = wl["bound"] == "hbm"
            n_layers = args.layers if args.layers is not None else (8 if decode_like else 2)
            sets, host_w = [], None
            for li in range(n_layers):
                W, src = make_weight_set(torch, moe, 2000 + li)
                if li == 0 and not args.no_cpu_baseline:
                    host_w = tuple(t.cpu() for t in src)
                del src
                sets.append(W)
            torch.cuda.empty_cache()
            res = run_layer_workload(torch, moe, args.workload, wl, sets, args, steps, warmup, host_w)
        print(json.dumps(res))
        return

    # ---- default: every workload of the metric in one line ----------------------------
    # One resident set of 32 layers (90 GB) serves all of them: the stack workloads use all,
    # the single-layer ones rotate over the first 8 (decode-sized) or 2 (prefill).
    L = args.layers if args.layers is not None else 32
    layers, host_w, _ = make_stack_layers(torch, moe, L, not args.no_cpu_baseline)
    sets = [W for W, _ in layers]
    head_wl = dict(WORKLOADS["decode_t1"])
    d_steps, d_warm = defaults(head_wl)
    steps = args.steps if args.steps is not None else d_steps
    warmup = args.warmup if args.warmup is not None else d_warm
    res = run_layer_workload(torch, moe, "decode_t1", head_wl, sets[:8], args, steps, warmup, host_w)
    others = {}
    for name in ("prefill_t4096", "beam_t16"):
        wl = dict(WORKLOADS[name])
        st, wu = defaults(wl)
        n_sets = 8 if wl["bound"] == "hbm" else 2
        others[name] = nested(run_layer_workload(torch, moe, name, wl, sets[:n_sets], args, st, wu))
    for name in ("stack_t1", "stack_t512"):
        wl = dict(WORKLOADS[name])
        st, wu = defaults(wl)
        others[name] = nested(run_stack_workload(torch, moe, name, wl, layers, args, st, wu))
    res["workloads"] = others
    print(json.dumps(res))


if __name__ == "__main__":
    main()
