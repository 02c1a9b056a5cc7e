#!/usr/bin/env python3
"""Benchmark of the conv2d hot path on one MI355X.

One "step" is one pass of the whole path over one batch of a synthetic CNN layer
stack: the network input is converted NCHW -> NHWC once (layout kernel), then every
layer runs forward, backward-data and backward-weight (with its split reduction)
through the C ABI with activations resident in NHWC and filters in KRSC.  Inputs are
generated from a seed on the host and are resident in HBM before the timed region.

Prints ONE JSON line: whole-job TFLOP/s (2*N*K*P*Q*C*R*S flops per pass, three passes
per layer), the roofline figures of the dominant kernel measured with HIP events, and
the CPU oracle timed on a bounded sample of the same workload (reported baseline only).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload alexnet_b128] [--all]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_F32_TFLOPS = 157.3       # fp32 vector / matrix, published
PEAK_HBM_GBS = 8000.0         # HBM3E, published


def algorithmic_bytes(L, op, esize):
    """Bytes a pass must move: each operand read once, the result written once.  Strided
    forward/backward-weight count only the input pixels some tap touches; dw is fp32."""
    touched_h = len({p * L.stride - L.pad + r for p in range(L.P) for r in range(L.R)} & set(range(L.H)))
    touched_w = len({q * L.stride - L.pad + s for q in range(L.Q) for s in range(L.S)} & set(range(L.W)))
    x_touched = L.N * L.C * touched_h * touched_w
    x_all, w, y = L.N * L.C * L.H * L.W, L.K * L.C * L.R * L.S, L.N * L.K * L.P * L.Q
    if op == "fwd":
        return esize * (x_touched + w + y)
    if op == "bwd_data":
        return esize * (y + w + x_all)
    return esize * (x_touched + y) + 4 * w


class LayerState:
    """Device tensors of one layer, NHWC/KRSC resident, plus workspaces."""

    def __init__(self, mxc, torch, cfg, li, gen, layout="nhwc"):
        L, t = gen.layer_inputs(cfg, li)
        self.L = L
        self.dims = L.dims()
        self.dt = mxc.MXC_BF16 if cfg.dtype == "bf16" else mxc.MXC_F32
        td = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        dev = lambda a: gen.to_device(a, cfg.dtype)
        x_nchw = dev(t["x"])
        self.lay = mxc.MXC_NHWC if layout == "nhwc" else mxc.MXC_NCHW
        if layout == "nhwc":
            self.x_nchw = x_nchw if li == 0 else None        # only the network input is converted in the step
            self.x = x_nchw.view(L.N, L.C, L.H, L.W).permute(0, 2, 3, 1).contiguous().view(-1)
            self.w = dev(t["w"]).view(L.K, L.C, L.R, L.S).permute(0, 2, 3, 1).contiguous().view(-1)
            self.dy = dev(t["dy"]).view(L.N, L.K, L.P, L.Q).permute(0, 2, 3, 1).contiguous().view(-1)
        else:                                                # operands stay NCHW / KCRS; every call converts inside
            self.x_nchw = None
            self.x, self.w, self.dy = x_nchw, dev(t["w"]), dev(t["dy"])
        del t
        self.y = torch.empty(L.N * L.K * L.P * L.Q, dtype=td, device="cuda")
        self.dx = torch.empty(L.N * L.C * L.H * L.W, dtype=td, device="cuda")
        self.dw = torch.empty(L.K * L.C * L.R * L.S, dtype=torch.float32, device="cuda")
        self.bias = torch.linspace(-0.5, 0.5, L.K, dtype=torch.float32, device="cuda")
        self.w_master = self.w.float() if cfg.dtype == "bf16" else None     # fp32 master weights and velocity of the update
        self.vel = torch.zeros_like(self.w_master) if cfg.dtype == "bf16" else None
        self.db = torch.empty(L.K, dtype=torch.float32, device="cuda")
        self.ws = {}
        for op in (mxc.MXC_FWD, mxc.MXC_BWD_DATA, mxc.MXC_BWD_WEIGHT, mxc.MXC_BWD_DATA_RELU, mxc.MXC_BIAS_GRAD):
            self.ws[op] = mxc.alloc_workspace(mxc.mxc_conv2d_workspace_bytes(op, *self.dims, self.dt, self.lay))


class Network:
    def __init__(self, mxc, torch, gen, cfg, layout="nhwc"):
        self.mxc, self.torch, self.cfg, self.layout = mxc, torch, cfg, layout
        self.layers = [LayerState(mxc, torch, cfg, li, gen, layout) for li in range(len(cfg.layers))]
        self.flops_per_step = 3 * sum(s.L.flops_per_pass for s in self.layers)
        self.esize = 2 if cfg.dtype == "bf16" else 4

    def calls(self):
        """(label, op, layer, thunk) for every ABI call of one step, in order."""
        m = self.mxc
        out = []
        s0 = self.layers[0]
        L0 = s0.L
        if self.layout == "nhwc":
            out.append(("layout", "layout", s0, lambda: m.mxc_layout_convert(
                L0.N, L0.C, L0.H, L0.W, s0.dt, m.MXC_NCHW, m.MXC_NHWC, s0.x_nchw, s0.x)))
        for s in self.layers:
            out.append((s.L.name, "fwd", s, lambda s=s: m.mxc_conv2d_fwd(
                *s.dims, s.dt, s.lay, s.x, s.w, s.y, s.ws[m.MXC_FWD])))
            out.append((s.L.name, "bwd_data", s, lambda s=s: m.mxc_conv2d_bwd_data(
                *s.dims, s.dt, s.lay, s.dy, s.w, s.dx, s.ws[m.MXC_BWD_DATA])))
            out.append((s.L.name, "bwd_weight", s, lambda s=s: m.mxc_conv2d_bwd_weight(
                *s.dims, s.dt, s.lay, s.x, s.dy, s.dw, s.ws[m.MXC_BWD_WEIGHT])))
        return out

    def grouped_calls(self):
        """The same step with the grouped entry points: forward + bias + ReLU in one call, backward-data with
        the ReLU derivative of the layer below, backward-weight, and the bias gradient."""
        m = self.mxc
        out = []
        for c in self.calls():
            label, op, s, fn = c
            if op == "fwd":
                out.append((label, op, s, lambda s=s: m.mxc_conv2d_fwd_bias_act(
                    *s.dims, s.dt, s.lay, s.x, s.w, s.bias, 1, s.y, s.ws[m.MXC_FWD])))
            elif op == "bwd_data":
                out.append((label, op, s, lambda s=s: m.mxc_conv2d_bwd_data_relu(
                    *s.dims, s.dt, s.lay, s.dy, s.w, s.x, s.dx, s.ws[m.MXC_BWD_DATA_RELU])))
            else:
                out.append(c)
                if op == "bwd_weight":
                    out.append((label, "bias_grad", s, lambda s=s: m.mxc_bias_grad(
                        s.L.N, s.L.K, s.L.P, s.L.Q, s.dt, s.lay, s.dy, s.db, s.ws[m.MXC_BIAS_GRAD])))
                    if s.w_master is not None:
                        # a learning rate small enough that the synthetic gradients leave the weights where they are
                        out.append((label, "sgd_update", s, lambda s=s: m.mxc_sgd_update(
                            s.w_master, s.dw, s.vel, s.w, 1e-9, 0.9, 1e-4)))
        return out

    def step(self):
        for _, _, _, fn in self.calls():
            fn()


def time_steps(torch, net, steps, warmup, keep=lambda c: True, grouped=False):
    calls = [c[3] for c in (net.grouped_calls() if grouped else net.calls()) if keep(c)]
    for _ in range(warmup):
        for fn in calls:
            fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for fn in calls:
            fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_two_streams(torch, net, steps, warmup):
    """The same step issued the way a dependency engine (paper Section 3.2) would: backward-weight
    calls, which nothing in the step waits for, go to a second stream beside the forward /
    backward-data chain.  Reported beside the headline, which stays a single in-order stream."""
    calls = net.calls()
    main = [c[3] for c in calls if c[1] != "bwd_weight"]
    side = [c[3] for c in calls if c[1] == "bwd_weight"]
    s_main, s_side = torch.cuda.Stream(), torch.cuda.Stream()

    def step():
        fork = torch.cuda.Event()
        fork.record(s_main)
        s_side.wait_event(fork)
        with torch.cuda.stream(s_side):
            for fn in side:
                fn()
        with torch.cuda.stream(s_main):
            for fn in main:
                fn()
        join = torch.cuda.Event()
        join.record(s_side)
        s_main.wait_event(join)

    torch.cuda.synchronize()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def measure_ceilings(torch, mxc):
    """On-box ceilings beside the published ones: the matrix pipe running a register-resident bf16
    MFMA loop (two workgroups of four waves per CU) and a plain device copy of 1 GiB."""
    out = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    mxc.mxc_probe_mfma(512, 2000, out)
    torch.cuda.synchronize()
    e0.record()
    flops = mxc.mxc_probe_mfma(512, 20000, out)
    e1.record()
    torch.cuda.synchronize()
    mfma_tflops = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    n_el = 1 << 28                      # 2^28 fp32 = 1 GiB read + 1 GiB written
    src = torch.ones(n_el, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    copy = lambda: mxc.mxc_layout_convert(1, 1, 1 << 14, 1 << 14, mxc.MXC_F32, mxc.MXC_NCHW, mxc.MXC_NCHW, src, dst)
    copy()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(5):
        copy()
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2.0 * n_el * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst, out
    torch.cuda.empty_cache()
    return {"mfma_bf16_tflops_measured": round(mfma_tflops, 1), "copy_gbs_measured": round(copy_gbs, 1),
            "note": "register-resident v_mfma_f32_32x32x16_bf16 loop, 2 waves/SIMD; 1 GiB device copy, read + write bytes"}


def time_calls(torch, net, steps):
    """Per-call durations (ms, mean over `steps`) with HIP events on the stream the kernels run on
    (torch's current stream), over the same sequence of calls as the timed region.  An event pair
    with nothing between it, recorded once per step behind the same busy stream, measures what the
    two event packets themselves cost (about 5 us); that is subtracted, so that a call that is one
    launch reads as that kernel's duration.  Returns (per-call list, event-pair overhead in ms)."""
    mxc = net.mxc
    calls = net.calls()
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in calls]
          for _ in range(steps)]
    null = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    variants = []
    for i in range(steps):
        for j, (_, op, _, fn) in enumerate(calls):
            ev[i][j][0].record()
            fn()
            ev[i][j][1].record()
            if i == 0:
                variants.append(mxc.mxc_last_variant() if op != "layout" else "layout:transpose")
        null[i][0].record()
        null[i][1].record()
    torch.cuda.synchronize()
    gaps = sorted(a.elapsed_time(b) for a, b in null)
    overhead = gaps[len(gaps) // 2]
    out = []
    for j, (name, op, s, _) in enumerate(calls):
        ms = sum(ev[i][j][0].elapsed_time(ev[i][j][1]) for i in range(steps)) / steps
        out.append({"layer": name, "op": op, "variant": variants[j], "ms": max(ms - overhead, 1e-6), "state": s})
    return out, overhead


def kernel_of(variant):
    """'fwd:smallc+igemm_128x64_k64s2_w4' -> 'igemm_128x64_k64s2_w4' (the main kernel of the call)."""
    return variant.split(":")[-1].split("+")[-1]


def roofline_of(per_call, net, event_overhead_ms=0.0):
    """Roofline entry of the kernel that takes the most time in a step.  Its launches are timed with HIP
    events around the ABI call; only calls that are exactly one launch of that kernel (plain forward
    calls) enter the figure, so that the event time is the kernel's duration."""
    by_kernel = {}
    for c in per_call:
        by_kernel.setdefault(kernel_of(c["variant"]), []).append(c)
    single = lambda c: c["op"] == "fwd" and "+" not in c["variant"]      # the call is exactly one launch of the kernel
    # A call's event time includes its helper launches (packing, filter re-pack, split reduce), so kernels are
    # ranked by the time of their single-launch calls, which is kernel time proper; the committed rocprofv3
    # summary lists every kernel's total.
    ranked = {k: sum(c["ms"] for c in v if single(c)) for k, v in by_kernel.items()}
    dominant = max(ranked, key=ranked.get) if any(ranked.values()) else max(by_kernel, key=lambda v: sum(c["ms"] for c in by_kernel[v]))
    group = [c for c in by_kernel[dominant] if single(c)] or by_kernel[dominant]
    t = sum(c["ms"] for c in group) * 1e-3
    flops = sum(c["state"].L.flops_per_pass for c in group if c["op"] != "layout")
    nbytes = sum(algorithmic_bytes(c["state"].L, c["op"], net.esize) for c in group if c["op"] != "layout")
    peak_tf = PEAK_BF16_TFLOPS if net.cfg.dtype == "bf16" else PEAK_F32_TFLOPS
    t_mfma, t_hbm = flops / (peak_tf * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)
    if t_mfma >= t_hbm:
        bound = "mfma" if net.cfg.dtype == "bf16" else "alu"
        ach = flops / t / 1e12
        r = {"bound": bound, "achieved": round(ach, 2), "peak": peak_tf, "unit": "TFLOP/s", "frac": round(ach / peak_tf, 4)}
    else:
        ach = nbytes / t / 1e9
        r = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": round(ach / PEAK_HBM_GBS, 4)}
    r["kernel"] = dominant
    r["launches"] = [c["layer"] + ":" + c["op"] for c in group]
    r["avg_launch_ms"] = round(t * 1e3 / len(group), 4)
    r["event_pair_overhead_ms"] = round(event_overhead_ms, 4)      # already subtracted from avg_launch_ms
    r["algorithmic_flops_per_launch"] = flops // len(group)
    r["algorithmic_bytes_per_launch"] = nbytes // len(group)
    r["traffic"] = load_traffic(net.cfg.name, dominant)
    return r


def load_traffic(workload, variant):
    """HBM bytes per launch from the committed rocprofv3 counter summaries, if one covers this kernel."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {}).get(variant)
    except (OSError, ValueError):
        return None


def cpu_baseline(gen, cfg, sample_batch):
    """The oracle, as it stands, on the host cores: all layers, three passes, at a reduced batch."""
    from oracle import conv_oracle as orc
    flops, t = 0, 0.0
    for li in range(len(cfg.layers)):
        L, a = gen.layer_inputs(cfg, li, batch=min(sample_batch, cfg.layers[li].N))
        t0 = time.perf_counter()
        orc.conv2d_fwd(a["x"], a["w"], L.stride, L.pad)
        orc.conv2d_bwd_data(a["dy"], a["w"], a["x"].shape, L.stride, L.pad)
        orc.conv2d_bwd_weight(a["x"], a["dy"], a["w"].shape, L.stride, L.pad)
        t += time.perf_counter() - t0
        flops += 3 * L.flops_per_pass
    return {"value": round(flops / t / 1e12, 6), "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{cfg.name} all {len(cfg.layers)} layers, 3 passes, batch {sample_batch} of "
                      f"{cfg.layers[0].N} (cost is linear in batch); {t:.1f} s of fp64 7-loop oracle"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="alexnet_b128")
    ap.add_argument("--all", action="store_true", help="also time the other layer stacks (extra 'networks' field)")
    ap.add_argument("--per-layer", action="store_true", help="print a per-layer table to stderr")
    ap.add_argument("--layout", choices=["nhwc", "nchw"], default="nhwc",
                    help="nhwc: tensors resident in the working layout, network input converted once per step (headline); "
                         "nchw: every call takes NCHW/KCRS operands and converts inside (three extra HBM passes per call)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--cpu-sample-batch", type=int, default=128)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (mxc_layout_convert, same layout) so that a counter run "
                         "can scale FETCH_SIZE / WRITE_SIZE against a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU by contract (one MI355X, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1512_01274_amd import inputs as gen
    from paper_1512_01274_amd import mxc
    torch.cuda.set_device(0)

    def run_one(cfg, steps, warmup):
        net = Network(mxc, torch, gen, cfg, args.layout)
        sec = time_steps(torch, net, steps, warmup)
        per_call, ev_ms = time_calls(torch, net, steps)
        return net, sec, per_call, ev_ms

    if args.calibrate_copy:
        n_el = 1 << 28                      # 2^28 fp32 = 1 GiB read + 1 GiB written
        src = torch.ones(n_el, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        mxc.mxc_layout_convert(1, 1, 1 << 14, 1 << 14, mxc.MXC_F32, mxc.MXC_NCHW, mxc.MXC_NCHW, src, dst)
        torch.cuda.synchronize()
        del src, dst
    cfg = gen.config_by_name(args.workload)
    ceilings = measure_ceilings(torch, mxc)
    net, sec, per_call, ev_ms = run_one(cfg, args.steps, args.warmup)
    # the same step without backward-data of the first layer, which a training run never needs
    # (nothing consumes the gradient of the network input); reported beside the headline, labelled
    first = net.layers[0]
    sec_pruned = time_steps(torch, net, args.steps, args.warmup, keep=lambda c: not (c[1] == "bwd_data" and c[2] is first))
    flops_pruned = net.flops_per_step - first.L.flops_per_pass
    sec_two = time_two_streams(torch, net, args.steps, args.warmup)
    sec_grouped = time_steps(torch, net, args.steps, args.warmup, grouped=True)
    value = net.flops_per_step / sec / 1e12
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_TFLOPS
    result = {
        "metric": "conv2d fwd+bwd TFLOP/s per network on 1 MI355X", "value": round(value, 3), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "layers": len(cfg.layers), "batch": cfg.layers[0].N,
                   "layout": "nhwc-resident" if args.layout == "nhwc" else "nchw-per-call",
                   "step": ("layout(NCHW->NHWC of network input) + " if args.layout == "nhwc" else "") +
                           "per layer fwd, bwd_data, bwd_weight"},
        "frac_of_mfma_peak": round(value / peak, 4),
        "roofline": roofline_of(per_call, net, ev_ms),
        "ceilings": ceilings,
        "without_first_layer_bwd_data": {"value": round(flops_pruned / sec_pruned / 1e12, 3), "unit": "TFLOP/s",
                                         "ms_per_step": round(sec_pruned * 1e3, 4)},
        "grouped_operations": {"value": round(net.flops_per_step / sec_grouped / 1e12, 3), "unit": "TFLOP/s",
                               "ms_per_step": round(sec_grouped * 1e3, 4),
                               "note": "same convolution flops; forward + bias + ReLU, backward-data with the ReLU derivative, "
                                       "backward-weight, bias gradient, SGD update of fp32 master weights with a bf16 copy "
                                       "(the extra work is not counted as flops)"},
        "two_stream_schedule": {"value": round(net.flops_per_step / sec_two / 1e12, 3), "unit": "TFLOP/s",
                                "ms_per_step": round(sec_two * 1e3, 4),
                                "note": "backward-weight calls on a second stream; not the headline"},
    }
    if cfg.dtype == "bf16":
        result["frac_of_measured_mfma"] = round(value / ceilings["mfma_bf16_tflops_measured"], 4)
        if result["roofline"]["bound"] == "mfma":
            result["roofline"]["frac_of_measured"] = round(result["roofline"]["achieved"] / ceilings["mfma_bf16_tflops_measured"], 4)
    if result["roofline"]["bound"] == "hbm":
        result["roofline"]["frac_of_measured"] = round(result["roofline"]["achieved"] / ceilings["copy_gbs_measured"], 4)
    if args.per_layer:
        for c in per_call:
            L = c["state"].L
            if c["op"] == "layout":
                nbytes = 2 * L.N * L.C * L.H * L.W * net.esize
                print(f"{c['layer']:>24} {c['op']:>10} {c['ms']*1e3:9.1f} us {nbytes/c['ms']/1e6:8.0f} GB/s  {c['variant']}",
                      file=sys.stderr)
                continue
            tf = L.flops_per_pass / c["ms"] / 1e9
            gbs = algorithmic_bytes(L, c["op"], net.esize) / c["ms"] / 1e6
            print(f"{c['layer']:>24} {c['op']:>10} {c['ms']*1e3:9.1f} us {tf:8.1f} TFLOP/s {gbs:8.0f} GB/s  {c['variant']}",
                  file=sys.stderr)
    del net
    torch.cuda.empty_cache()
    if args.all:
        nets = {}
        for other in gen.CONFIGS:
            if other.name == cfg.name:
                continue
            n2, s2, pc2, _ = run_one(other, max(3, args.steps // 4), 2)
            pk = PEAK_BF16_TFLOPS if other.dtype == "bf16" else PEAK_F32_TFLOPS
            nbytes = sum(algorithmic_bytes(c["state"].L, c["op"], n2.esize) for c in pc2 if c["op"] != "layout")
            nets[other.name] = {"tflops": round(n2.flops_per_step / s2 / 1e12, 3), "ms_per_step": round(s2 * 1e3, 4),
                                "frac_of_mfma_peak": round(n2.flops_per_step / s2 / 1e12 / pk, 4),
                                "algorithmic_GBps": round(nbytes / s2 / 1e9, 1)}
            del n2, pc2
            torch.cuda.empty_cache()
        result["networks"] = nets
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(gen, cfg, args.cpu_sample_batch)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
