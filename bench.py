#!/usr/bin/env python3
"""Benchmark of the MoE expert layer hot path on one MI355X.

A step = one pass of the whole hot path (moe_route -> moe_permute ->
moe_expert_ffn -> moe_combine, through the C ABI) over one batch of synthetic,
Mixtral-8x7B-shaped input that is already resident in HBM.  Steps rotate over
several independent weight sets (layers) and inputs so that no step finds its
expert matrices in the last-level cache.

Prints ONE JSON line: whole-job tokens/s, plus
  roofline     -- the dominant kernel (first projection of moe_expert_ffn) timed
                  live with HIP events on the launch stream, against HBM peak
                  (decode-sized workloads) or bf16 MFMA peak (prefill);
  cpu_baseline -- the fp64 CPU oracle timed on this machine's host cores on a
                  bounded sample of the same workload (a baseline, not a target).
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

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (scaled by the 1 GiB copy calibration; see the summaries under profiles/).  Static figures
# from those profile runs, not measured by this script.
TRAFFIC_BYTES = {
    "decode_t1": 470.5e6,       # profiles/stream_kernels_decode_t1.txt
    "beam_t16": 1.604e9,        # profiles/stream_kernels_beam_t16.txt (6.8 active experts)
    "prefill_t4096": 4.82e9,    # profiles/grouped_gemm_prefill_t4096.txt (fetch 4.58 GB + write 0.24 GB)
}

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
    """Preallocated buffers + the four C-ABI calls of one step."""

    def __init__(self, torch, moe, T, x_dtype, fused_gate=False):
        N = T * K
        self.fused_gate = fused_gate and T <= 16 and x_dtype == torch.float32
        self.ffn_path = moe.MOE_FFN_AUTO
        i32 = dict(dtype=torch.int32, device="cuda")
        f32 = dict(dtype=torch.float32, device="cuda")
        self.moe = moe
        self.idx = torch.empty((T, K), **i32)
        self.w = torch.empty((T, K), **f32)
        self.perm_out = (torch.empty(E, **i32), torch.empty(E + 1, **i32), torch.empty(N, **i32),
                         torch.empty(N, **i32), torch.empty((N, D), dtype=x_dtype, device="cuda"))
        adt = moe.MOE_BF16 if x_dtype == torch.bfloat16 else moe.MOE_F32
        self.ws = torch.empty(moe.moe_expert_ffn_workspace(N, E, D, F, adt), dtype=torch.uint8,
                              device="cuda")
        self.yg = torch.empty((N, D), **f32)
        self.y = torch.empty((T, D), **f32)

    def run(self, W, x, logits, ev=None, events=None, stream=0):
        moe = self.moe
        if self.fused_gate:
            moe.moe_route_permute(logits, K, x, self.idx, self.w, self.perm_out)
            counts, offsets, perm, inv_perm, xg = self.perm_out
        else:
            moe.moe_route(logits, K, self.idx, self.w)
            counts, offsets, perm, inv_perm, xg = moe.moe_permute(self.idx, E, x,
                                                                  out=self.perm_out)
        if ev is not None:
            events.record(ev[0], stream)
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


def run_stack(args, torch, moe, wl):
    """Layer-stack workload: value = tokens/s through all layers, ms_per_step = stack time."""
    T, L = wl["T"], (args.layers if args.layers is not None else wl["layers"])
    steps = args.steps if args.steps is not None else (20 if T == 1 else 5)
    warmup = args.warmup if args.warmup is not None else 2
    g = torch.Generator(device="cuda")
    g.manual_seed(777)
    layers, host_w, host_gate = [], None, None
    for li in range(L):
        W, src = make_weight_set(torch, moe, 2000 + li)
        wg = (torch.randn((D, E), generator=g, device="cuda") * D ** -0.5).contiguous()
        if li == 0 and not args.no_cpu_baseline:
            host_w = tuple(t.cpu() for t in src)
            host_gate = wg.cpu()
        del src
        layers.append((W, wg))
    torch.cuda.empty_cache()
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
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=achieved / HBM_PEAK_GBS, traffic=None,
                    kernel="first projection of moe_expert_ffn, summed over the layers",
                    kernel_ms=up_ms, active_experts_all_layers=n_active,
                    whole_stack_GBs=all_bytes / (ms_per_step * 1e-3) / 1e9,
                    whole_stack_TFLOPs=T * K * 6 * D * F * L / (ms_per_step * 1e-3) / 1e12)
    result = {
        "metric": "MoE-layer tokens/s", "value": T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights x fp32 activations" + (" (bf16 hi+lo)" if T * K <= 96 else
                                                      " (rounded to bf16)") + ", fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": args.workload, "T": T, "layers": L, "d_model": D, "d_ff": F,
                   "experts": E, "top_k": K,
                   "per_token_expert_time_us": ms_per_step * 1e3 / T,
                   "host_enqueue_ms": host_enqueue_ms,
                   "resident_expert_bytes": sum(W.nbytes for W, _ in layers)},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
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
    print(json.dumps(result))


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
    ap.add_argument("--workload", default="decode_t1", choices=sorted(WORKLOADS))
    ap.add_argument("--layers", type=int, default=None, help="independent weight sets rotated")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tokens", type=int, default=None,
                    help="override T of the workload (sweeps; the JSON names it)")
    ap.add_argument("--ffn-path", default="auto", choices=["auto", "stream", "grouped", "mid"],
                    help="force the expert-FFN kernel family (sweeps)")
    ap.add_argument("--fused-gate", action="store_true",
                    help="decode-sized workloads: use the one-launch moe_route_permute instead "
                         "of moe_route + moe_permute (same outputs)")
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
    wl = dict(WORKLOADS[args.workload])
    global D, F, E, K
    D, F, E, K = wl.get("shape", (D, F, E, K))
    if args.tokens is not None:
        wl["T"] = args.tokens
    T = wl["T"]
    if "layers" in wl:
        return run_stack(args, torch, moe, wl)
    decode_like = wl["bound"] == "hbm"
    steps = args.steps if args.steps is not None else (400 if decode_like else 30)
    warmup = args.warmup if args.warmup is not None else (40 if decode_like else 5)
    n_layers = args.layers if args.layers is not None else (8 if decode_like else 2)
    n_inputs = 16 if decode_like else 2

    sets, host_w = [], None
    for li in range(n_layers):
        W, src = make_weight_set(torch, moe, 2000 + li)
        if li == 0 and not args.no_cpu_baseline:
            host_w = tuple(t.cpu() for t in src)
        del src
        sets.append(W)
    torch.cuda.empty_cache()
    xs, lgs = make_inputs(torch, moe, wl, n_inputs, 4242)
    step = Step(torch, moe, T, xs[0].dtype, fused_gate=args.fused_gate)
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
    if decode_like:
        # bytes: w1 and w3 of every active expert, read once (2 * d * f bf16 each)
        up_bytes = n_active * 2 * D * F * 2
        achieved = up_bytes / (up_ms * 1e-3) / 1e9
        roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=achieved / HBM_PEAK_GBS, traffic=TRAFFIC_BYTES.get(args.workload),
                        kernel="stream_kernel<KSW=16,NMAT=2> (x.w1, x.w3, silu*mul)",
                        kernel_ms=up_ms, second_projection_ms=dn_ms,
                        second_projection_GBs=n_active * D * F * 2 / (dn_ms * 1e-3) / 1e9,
                        mean_active_experts=n_active)
    else:
        up_flops = T * K * 2 * 2 * D * F  # real rows only
        achieved = up_flops / (up_ms * 1e-3) / 1e12
        roofline = dict(bound="mfma", achieved=achieved, peak=MFMA_BF16_PEAK_TFLOPS,
                        unit="TFLOP/s", frac=achieved / MFMA_BF16_PEAK_TFLOPS,
                        traffic=TRAFFIC_BYTES.get(args.workload),
                        kernel="gg_pack + gg_gemm_kernel<UP> (x.w1, x.w3, silu*mul)",
                        kernel_ms=up_ms, second_projection_ms=dn_ms,
                        second_projection_TFLOPs=T * K * 2 * D * F / (dn_ms * 1e-3) / 1e12,
                        layer_TFLOPs=T * K * 6 * D * F / (ms_per_step * 1e-3) / 1e12)

    result = {
        "metric": "MoE-layer tokens/s", "value": T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights x " + ("bf16" if wl["x_bf16"] else "fp32 (bf16 hi+lo)") +
                 " activations, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": args.workload, "T": T, "d_model": D, "d_ff": F, "experts": E,
                   "top_k": K, "weight_sets_rotated": n_layers, "inputs_rotated": n_inputs,
                   "counts_first_input": counts_all[0], "ffn_path": args.ffn_path,
                   "calls_per_step": ("moe_route_permute, moe_expert_ffn, moe_combine"
                                      if step.fused_gate else
                                      "moe_route, moe_permute, moe_expert_ffn, moe_combine")},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(torch, wl, host_w, xs, lgs)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
