#!/usr/bin/env python3
"""Benchmark of the conv2d hot path on one MI355X.

One "step" is one pass of the whole path over one batch of a synthetic CNN layer stack: the network
input is converted NCHW -> NHWC once (layout kernel), then every layer runs forward, backward-data and
backward-weight (with its split reduction) through the C ABI with activations resident in NHWC and
filters in KRSC.  Inputs are generated from a seed on the host and are resident in HBM before the timed
region.  Backward-data reads filters prepared once per weight version (mxc_conv2d_bwd_data_prepare_filter,
outside the timed region: the weights do not change between the steps of this benchmark; the cost of
preparing them every step is reported in `filter_prepare_ms_per_step`).  A first layer (C = 3) packs its
input once per step, inside the timed region, into a buffer that its forward and its backward-weight both
read (mxc_conv2d_prepare_input); --raw-filter turns both kinds of prepared operands off.

Two schedules of the same calls are timed:
  * "single_stream": every call in program order on one stream, launched eagerly.  This is the headline
    (`value`, `ms_per_step`); per-call and per-kernel figures (the roofline entries) are measured in this
    schedule, where kernels do not overlap and their times add up to the step.
  * "engine": the order a dependency engine (paper Section 3.2) gives a training step - forward chain,
    then per layer, last to first, backward-data on the main stream and backward-weight beside it on a
    second stream (both need only that layer's output gradient), the whole step captured once into a HIP
    graph and replayed.  Reported beside the headline (`engine_schedule`); --engine makes it the headline.

Prints ONE JSON line: whole-job TFLOP/s (2*N*K*P*Q*C*R*S flops per pass, three passes per layer) of the
headline workload, the same for the other four stacks (`networks`), roofline entries of the dominant
kernels measured with HIP events, on-box ceilings, and the CPU oracle timed on a bounded sample of the
same workload (reported baseline only).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload alexnet_b128] [--groups G] [--no-all]
"""
import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_F32_TFLOPS = 157.3       # fp32 vector / matrix, published
PEAK_HBM_GBS = 8000.0         # HBM3E, published
FLOP_PER_CLK_BF16 = 256 * 4 * 1024   # CUs x SIMDs x bf16 MFMA flops per SIMD clock


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
    if op == "layout":
        return 2 * esize * x_all
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
        for op in (mxc.MXC_FWD, mxc.MXC_BWD_DATA, mxc.MXC_BWD_WEIGHT, mxc.MXC_BWD_DATA_RELU, mxc.MXC_BIAS_GRAD,
                   mxc.MXC_BWD_DATA_PREPARED, mxc.MXC_BWD_DATA_PREPARED_RELU):
            self.ws[op] = mxc.alloc_workspace(mxc.mxc_conv2d_workspace_bytes(op, *self.dims, self.dt, self.lay))
        self.w_prepared = mxc.alloc_workspace(mxc.mxc_conv2d_workspace_bytes(mxc.MXC_BWD_DATA_FILTER, *self.dims, self.dt, self.lay))
        self.prepare_filter = lambda: mxc.mxc_conv2d_bwd_data_prepare_filter(*self.dims, self.dt, self.lay, self.w, self.w_prepared)
        self.prepare_filter()
        # first layers (C = 3): forward packs x once into a buffer that backward-weight reads too
        self.x_prepared = None
        if layout == "nhwc":
            nb = mxc.mxc_conv2d_workspace_bytes(mxc.MXC_INPUT_PREPARED, *self.dims, self.dt, self.lay)
            if nb:
                self.x_prepared = mxc.alloc_workspace(nb)
                for op in (mxc.MXC_FWD_PREPARED_INPUT, mxc.MXC_BWD_WEIGHT_PREPARED_INPUT):
                    self.ws[op] = mxc.alloc_workspace(mxc.mxc_conv2d_workspace_bytes(op, *self.dims, self.dt, self.lay))


class Network:
    def __init__(self, mxc, torch, gen, cfg, layout="nhwc", prepared=True):
        self.mxc, self.torch, self.cfg, self.layout, self.prepared = mxc, torch, cfg, layout, prepared
        self.layers = [LayerState(mxc, torch, cfg, li, gen, layout) for li in range(len(cfg.layers))]
        self.flops_per_step = 3 * sum(s.L.flops_per_pass for s in self.layers)
        self.esize = 2 if cfg.dtype == "bf16" else 4
        torch.cuda.synchronize()

    def _bwd_data(self, s):
        m = self.mxc
        if self.prepared:
            return lambda: m.mxc_conv2d_bwd_data_prepared(*s.dims, s.dt, s.lay, s.dy, s.w_prepared, None, s.dx,
                                                          s.ws[m.MXC_BWD_DATA_PREPARED])
        return lambda: m.mxc_conv2d_bwd_data(*s.dims, s.dt, s.lay, s.dy, s.w, s.dx, s.ws[m.MXC_BWD_DATA])

    def fwd_thunk(self, s, x, bias=None, relu=0):
        """Forward of layer s on x; a layer with a prepared input form packs its own x here, once per step."""
        m = self.mxc
        if self.prepared and s.x_prepared is not None and x is s.x:
            def fn():
                m.mxc_conv2d_prepare_input(*s.dims, s.dt, s.lay, x, s.x_prepared)
                m.mxc_conv2d_fwd_prepared_input(*s.dims, s.dt, s.lay, s.x_prepared, s.w, bias, relu, s.y,
                                                s.ws[m.MXC_FWD_PREPARED_INPUT])
            return fn
        if bias is None and not relu:
            return lambda: m.mxc_conv2d_fwd(*s.dims, s.dt, s.lay, x, s.w, s.y, s.ws[m.MXC_FWD])
        return lambda: m.mxc_conv2d_fwd_bias_act(*s.dims, s.dt, s.lay, x, s.w, bias, relu, s.y, s.ws[m.MXC_FWD])

    def wgrad_thunk(self, s, x, dy):
        """Backward-weight of layer s; reads what fwd_thunk prepared when there is such a form."""
        m = self.mxc
        if self.prepared and s.x_prepared is not None and x is s.x:
            return lambda: m.mxc_conv2d_bwd_weight_prepared_input(*s.dims, s.dt, s.lay, s.x_prepared, dy, s.dw, m.MXC_F32,
                                                                  s.ws[m.MXC_BWD_WEIGHT_PREPARED_INPUT])
        return lambda: m.mxc_conv2d_bwd_weight(*s.dims, s.dt, s.lay, x, dy, s.dw, s.ws[m.MXC_BWD_WEIGHT])

    def calls(self):
        """(label, op, layer, thunk) for every ABI call of one step, in program order."""
        m = self.mxc
        out = []
        s0 = self.layers[0]
        L0 = s0.L
        if self.layout == "nhwc":
            out.append(("layout", "layout", s0, lambda: m.mxc_layout_convert(
                L0.N, L0.C, L0.H, L0.W, s0.dt, m.MXC_NCHW, m.MXC_NHWC, s0.x_nchw, s0.x)))
        for s in self.layers:
            out.append((s.L.name, "fwd", s, self.fwd_thunk(s, s.x)))
            out.append((s.L.name, "bwd_data", s, self._bwd_data(s)))
            out.append((s.L.name, "bwd_weight", s, self.wgrad_thunk(s, s.x, s.dy)))
        return out

    def grouped_calls(self):
        """The same step with the grouped entry points: forward + bias + ReLU in one call, backward-data with
        the ReLU derivative of the layer below, backward-weight, and the bias gradient."""
        m = self.mxc
        out = []
        for c in self.calls():
            label, op, s, fn = c
            if op == "fwd":
                out.append((label, op, s, self.fwd_thunk(s, s.x, s.bias, 1)))
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


def chained_grouped_step(net):
    """The grouped step with consecutive layers chained on the device where their shapes allow it (the output
    tensor of layer i is the input tensor of layer i+1, and backward-data of layer i+1 writes the output gradient
    that layer i reads): forward chain with bias + ReLU, then from the last layer to the first backward-weight,
    bias gradient, backward-data with the ReLU derivative, and the update.  Returns (step function, link names)."""
    m, layers = net.mxc, net.layers
    x_of = {id(s): s.x for s in layers}
    dy_of = {id(s): s.dy for s in layers}
    links = []
    for a, b in zip(layers[:-1], layers[1:]):
        if (a.L.N, a.L.K, a.L.P, a.L.Q) == (b.L.N, b.L.C, b.L.H, b.L.W):
            x_of[id(b)] = a.y
            dy_of[id(a)] = b.dx
            links.append(f"{a.L.name}->{b.L.name}")
    calls = []
    s0 = layers[0]
    if net.layout == "nhwc":
        calls.append(lambda: m.mxc_layout_convert(s0.L.N, s0.L.C, s0.L.H, s0.L.W, s0.dt, m.MXC_NCHW, m.MXC_NHWC, s0.x_nchw, s0.x))
    for s in layers:
        calls.append(net.fwd_thunk(s, x_of[id(s)], s.bias, 1))
    for s in reversed(layers):
        calls.append(net.wgrad_thunk(s, x_of[id(s)], dy_of[id(s)]))
        calls.append(lambda s=s: m.mxc_bias_grad(s.L.N, s.L.K, s.L.P, s.L.Q, s.dt, s.lay, dy_of[id(s)], s.db, s.ws[m.MXC_BIAS_GRAD]))
        calls.append(lambda s=s: m.mxc_conv2d_bwd_data_relu(*s.dims, s.dt, s.lay, dy_of[id(s)], s.w, x_of[id(s)], s.dx,
                                                            s.ws[m.MXC_BWD_DATA_RELU]))
        if s.w_master is not None:
            calls.append(lambda s=s: m.mxc_sgd_update(s.w_master, s.dw, s.vel, s.w, 1e-9, 0.9, 1e-4))

    def step():
        for fn in calls:
            fn()
    return step, links


def timed_groups(torch, run_step, steps, warmup, groups):
    """`groups` timings of exactly `steps` steps each, every group bracketed by synchronize; seconds per step."""
    for _ in range(warmup):
        run_step()
    out = []
    for _ in range(groups):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run_step()
        torch.cuda.synchronize()
        out.append((time.perf_counter() - t0) / steps)
    return out


def median(v):
    v = sorted(v)
    return v[len(v) // 2]


def single_stream_step(net, keep=lambda c: True, grouped=False):
    calls = [c[3] for c in (net.grouped_calls() if grouped else net.calls()) if keep(c)]

    def step():
        for fn in calls:
            fn()
    return step


class EngineStep:
    """One step in the order a dependency engine gives a training step (paper Section 3.2): the layout
    conversion and the forward chain, then, from the last layer to the first, backward-data on the main
    stream and backward-weight on a second stream as soon as that layer's output gradient exists (in a
    chained network that is when backward-data of the layer above has finished).  The step is captured
    into a HIP graph once and replayed; if capture is not possible it is launched eagerly on the two
    streams (`mode` says which)."""

    def __init__(self, torch, net):
        self.torch = torch
        calls = net.calls()
        self.pre = [c[3] for c in calls if c[1] in ("layout", "fwd")]
        back = {}
        for c in calls:
            if c[1] in ("bwd_data", "bwd_weight"):
                back.setdefault(id(c[2]), {})[c[1]] = c[3]
        self.back = [back[id(s)] for s in reversed(net.layers)]
        self.main, self.side = torch.cuda.Stream(), torch.cuda.Stream()
        self.graph, self.mode = None, "eager two streams"
        try:
            self._enqueue()                     # once eagerly: first-call set-up stays out of the capture
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=self.main):
                self._enqueue(capturing=True)
            self.graph, self.mode = g, "HIP graph replay, two streams"
        except Exception as ex:             # noqa: BLE001  (any capture failure: run the same schedule eagerly)
            self.capture_error = repr(ex)[:200]
            torch.cuda.synchronize()

    def _enqueue(self, capturing=False):
        torch = self.torch
        main = torch.cuda.current_stream() if capturing else self.main
        with torch.cuda.stream(main):
            for fn in self.pre:
                fn()
            for fns in self.back:
                self.side.wait_stream(main)          # this layer's output gradient is ready
                with torch.cuda.stream(self.side):
                    fns["bwd_weight"]()
                fns["bwd_data"]()
            main.wait_stream(self.side)

    def __call__(self):
        if self.graph is not None:
            self.graph.replay()
        else:
            self._enqueue()


def measure_ceilings(torch, mxc):
    """On-box ceilings beside the published ones: the matrix pipe running a register-resident bf16
    MFMA loop (two workgroups of four waves per CU), the clock that rate implies, and a plain device copy
    of 1 GiB (the copy kernel spreads 16-byte accesses over all CUs)."""
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
    return {"mfma_bf16_tflops_measured": round(mfma_tflops, 1),
            "sclk_ghz_under_mfma_load": round(mfma_tflops * 1e12 / FLOP_PER_CLK_BF16 / 1e9, 3),
            "copy_gbs_measured": round(copy_gbs, 1),
            "note": "register-resident v_mfma_f32_32x32x16_bf16 loop, 2 waves/SIMD (the clock is that rate over "
                    "256 CUs x 4 SIMDs x 1024 flop per clock); 1 GiB device copy, read + write bytes"}


def smi_clock():
    """Shader clock right now: the current level of the driver's sclk table (sysfs), else what the SMI tool prints;
    None when neither is readable.  Under a profiler no tool is spawned (its preloaded library would make the
    child a GPU process before it starts the tool)."""
    import glob
    for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
        try:
            cur = [ln.strip() for ln in open(path) if ln.strip().endswith("*")]
            if cur:
                return "pp_dpm_sclk " + cur[0]
        except OSError:
            pass
    if any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ) or "rocprof" in os.environ.get("LD_PRELOAD", ""):
        return None
    for cmd in (["rocm-smi", "--showclocks", "--json"], ["amd-smi", "metric", "--clock", "--json"]):
        try:
            r = subprocess.run(cmd, capture_output=True, text=True, timeout=10)
            if r.returncode == 0 and r.stdout.strip():
                txt = r.stdout
                i = txt.find("sclk")
                return txt[i:i + 80].replace("\n", " ") if i >= 0 else None
        except (OSError, subprocess.SubprocessError):
            pass
    return None


def time_calls(torch, net, steps):
    """Per-call durations (ms, mean over `steps`) with HIP events on the stream the kernels run on
    (torch's current stream), over the same sequence of calls as the single-stream step.  An event pair
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
    """'fwd:smallc+igemm_128x64_k64s2_w4' -> 'igemm_128x64_k64s2_w4' (the main kernel of the call);
    a two-launch plan 'igemm_A+igemm_B' keeps both names."""
    v = variant.split(":")[-1]
    for prefix in ("s2d+", "smallc+", "chanpad+"):
        if v.startswith(prefix):
            v = v[len(prefix):]
    return v


def launches_of(c, prepared):
    """What a call's event time covers besides its main kernel."""
    v = c["variant"].split(":")[-1]
    extra = []
    if any(v.startswith(p) for p in ("s2d+", "smallc+", "chanpad+")):
        extra.append("operand packing")
    if "+igemm" in kernel_of(c["variant"]):
        extra.append("second launch of the plan")
    if c["op"] == "bwd_weight":
        extra.append("split reduce")
    if c["op"] == "bwd_data" and not prepared:
        extra.append("filter re-pack")
    if c["op"] == "bwd_data" and c["state"].L.stride > 1:
        extra.append("one launch per stride residue class")
    return extra


def roofline_entry(group, net, peak_tf, event_overhead_ms):
    t = sum(c["ms"] for c in group) * 1e-3
    flops = sum(c["state"].L.flops_per_pass for c in group if c["op"] != "layout")
    nbytes = sum(algorithmic_bytes(c["state"].L, c["op"], net.esize) for c in group)
    t_mfma, t_hbm = flops / (peak_tf * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)
    if t_mfma >= t_hbm:
        bound = "mfma" if net.cfg.dtype == "bf16" else "alu"
        ach = flops / t / 1e12
        r = {"bound": bound, "achieved": round(ach, 2), "peak": peak_tf, "unit": "TFLOP/s", "frac": round(ach / peak_tf, 4)}
    else:
        ach = nbytes / t / 1e9
        r = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": round(ach / PEAK_HBM_GBS, 4)}
    r["kernel"] = kernel_of(group[0]["variant"])
    r["launches"] = [c["layer"] + ":" + c["op"] for c in group]
    r["avg_launch_ms"] = round(t * 1e3 / len(group), 4)
    r["event_pair_overhead_ms"] = round(event_overhead_ms, 4)      # already subtracted from avg_launch_ms
    r["algorithmic_flops_per_launch"] = flops // len(group)
    r["algorithmic_bytes_per_launch"] = nbytes // len(group)
    r["traffic"] = load_traffic(net.cfg.name, r["kernel"])
    return r


def rooflines(per_call, net, event_overhead_ms):
    """Roofline entries per kernel, ranked by the kernel's share of the single-stream step.  Entry 0 (also the
    line's `roofline` object) is the kernel with the most time among calls that are exactly one launch of it
    (plain forward and prepared stride-1 backward-data calls: their event time is the kernel's duration); the
    other entries follow by total call time and say what else their calls' event times cover (`also_timed`)."""
    peak_tf = PEAK_BF16_TFLOPS if net.cfg.dtype == "bf16" else PEAK_F32_TFLOPS
    by_kernel = {}
    for c in per_call:
        by_kernel.setdefault(kernel_of(c["variant"]), []).append(c)
    exact = {k: [c for c in v if not launches_of(c, net.prepared)] for k, v in by_kernel.items()}
    ranked_exact = sorted((k for k in exact if exact[k]), key=lambda k: -sum(c["ms"] for c in exact[k]))
    out = []
    if ranked_exact:
        out.append(roofline_entry(exact[ranked_exact[0]], net, peak_tf, event_overhead_ms))
        out[0]["also_timed"] = []
    seen = {out[0]["kernel"]} if out else set()
    for k in sorted(by_kernel, key=lambda k: -sum(c["ms"] for c in by_kernel[k])):
        if k in seen:
            continue
        group = exact[k] or by_kernel[k]
        e = roofline_entry(group, net, peak_tf, event_overhead_ms)
        e["also_timed"] = sorted({x for c in group for x in launches_of(c, net.prepared)})
        out.append(e)
        seen.add(k)
        if len(out) >= 6:
            break
    return out


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


def layout_entry(torch, mxc):
    """a1 on a tensor beyond the 256 MiB memory-side cache: NCHW -> NHWC and back, bf16, GB/s of read + written bytes."""
    n, c, h, w = 64, 256, 112, 112                   # 392 MiB each side
    src = torch.randn(n * c * h * w, dtype=torch.float32, device="cuda").to(torch.bfloat16)
    dst = torch.empty_like(src)
    res = {}
    for name, a, b in (("nchw_to_nhwc", mxc.MXC_NCHW, mxc.MXC_NHWC), ("nhwc_to_nchw", mxc.MXC_NHWC, mxc.MXC_NCHW)):
        f = lambda: mxc.mxc_layout_convert(n, c, h, w, mxc.MXC_BF16, a, b, src, dst)
        f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            f()
        e1.record()
        torch.cuda.synchronize()
        gbs = 10 * 2.0 * src.numel() * 2 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        res[name] = {"GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / PEAK_HBM_GBS, 4)}
    res["tensor"] = f"bf16 [{n},{c},{h},{w}], {src.numel() * 2 >> 20} MiB"
    del src, dst
    torch.cuda.empty_cache()
    return res


def transform_entry(torch, mxc, gen):
    """The other algorithm for 3x3 stride-1 layers (transform domain, 2x2 blocks from 4x4 patches) beside the direct
    implicit GEMM, forward of two VGG-style layers: microseconds per call and the workspace the transform needs."""
    cfg = gen.config_by_name("vgg_a_b64")
    out = []
    for L in cfg.layers:
        if L.name not in ("conv4_2", "conv5_2"):
            continue
        d = L.dims()
        x = torch.randn(L.N * L.C * L.H * L.W, dtype=torch.float32, device="cuda").to(torch.bfloat16)
        w = (torch.randn(L.K * L.C * L.R * L.S, dtype=torch.float32, device="cuda") * 0.05).to(torch.bfloat16)
        y = torch.empty(L.N * L.K * L.P * L.Q, dtype=torch.bfloat16, device="cuda")
        ws_d = mxc.alloc_workspace(mxc.mxc_conv2d_workspace_bytes(mxc.MXC_FWD, *d, mxc.MXC_BF16, mxc.MXC_NHWC))
        nb = mxc.mxc_conv2d_workspace_bytes(mxc.MXC_FWD_TRANSFORM, *d, mxc.MXC_BF16, mxc.MXC_NHWC)
        ws_t = mxc.alloc_workspace(nb)
        us = {}
        for name, f in (("direct_us", lambda: mxc.mxc_conv2d_fwd(*d, mxc.MXC_BF16, mxc.MXC_NHWC, x, w, y, ws_d)),
                        ("transform_us", lambda: mxc.mxc_conv2d_fwd_transform(*d, mxc.MXC_BF16, mxc.MXC_NHWC, x, w, None, 0, y, ws_t))):
            f()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                f()
            e1.record()
            torch.cuda.synchronize()
            us[name] = round(e0.elapsed_time(e1) * 100.0, 1)
        out.append({"layer": L.name, **us, "transform_workspace_MiB": nb >> 20})
        del x, w, y, ws_d, ws_t
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--groups", type=int, default=5, help="timings of exactly --steps steps each; the median is reported")
    ap.add_argument("--workload", default="alexnet_b128")
    ap.add_argument("--no-all", action="store_true", help="skip the other layer stacks (the 'networks' field)")
    ap.add_argument("--all", action="store_true", help="accepted for compatibility: the other stacks are timed by default")
    ap.add_argument("--per-layer", action="store_true", help="print a per-layer table to stderr")
    ap.add_argument("--layout", choices=["nhwc", "nchw"], default="nhwc",
                    help="nhwc: tensors resident in the working layout, network input converted once per step (headline); "
                         "nchw: every call takes NCHW/KCRS operands and converts inside (three extra HBM passes per call)")
    ap.add_argument("--raw-filter", action="store_true",
                    help="backward-data re-packs its filter inside every call (mxc_conv2d_bwd_data) instead of reading one prepared "
                         "outside the timed region")
    ap.add_argument("--engine", action="store_true", help="headline = the engine schedule (HIP graph replay, two streams)")
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

    if args.calibrate_copy:
        n_el = 1 << 28                      # 2^28 fp32 = 1 GiB read + 1 GiB written
        src = torch.ones(n_el, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        mxc.mxc_layout_convert(1, 1, 1 << 14, 1 << 14, mxc.MXC_F32, mxc.MXC_NCHW, mxc.MXC_NCHW, src, dst)
        torch.cuda.synchronize()
        del src, dst

    def measure(cfg, steps, warmup, groups, detail):
        """Both schedules of one stack.  Returns (summary dict, net, per_call, event overhead)."""
        net = Network(mxc, torch, gen, cfg, args.layout, prepared=not args.raw_filter)
        single = timed_groups(torch, single_stream_step(net), steps, warmup, groups)
        engine = EngineStep(torch, net)
        eng = timed_groups(torch, engine, steps, warmup, groups)
        head = eng if args.engine else single
        sec = median(head)
        pk = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_TFLOPS
        per_call, ev_ms = time_calls(torch, net, max(3, min(steps, 20)))
        nbytes = sum(algorithmic_bytes(c["state"].L, c["op"], net.esize) for c in per_call)
        tf = lambda s: round(net.flops_per_step / s / 1e12, 3)
        summ = {"tflops": tf(sec), "ms_per_step": round(sec * 1e3, 4), "frac_of_mfma_peak": round(tf(sec) / pk, 4),
                "algorithmic_GBps": round(nbytes / sec / 1e9, 1), "frac_of_hbm_peak": round(nbytes / sec / 1e9 / PEAK_HBM_GBS, 4),
                "schedule": engine.mode if args.engine else "single stream, eager",
                "groups_ms": [round(s * 1e3, 4) for s in head],
                "single_stream": {"tflops": tf(median(single)), "ms_per_step": round(median(single) * 1e3, 4)},
                "engine": {"tflops": tf(median(eng)), "ms_per_step": round(median(eng) * 1e3, 4), "mode": engine.mode}}
        if detail:
            return summ, net, per_call, ev_ms
        rl = rooflines(per_call, net, ev_ms)
        summ["roofline"] = rl[0] if rl else None
        if cfg.dtype == "bf16":
            chain_step, chain_links = chained_grouped_step(net)
            ch = median(timed_groups(torch, chain_step, steps, 2, 3))
            summ["chained_grouped_operations"] = {"tflops": tf(ch), "ms_per_step": round(ch * 1e3, 4), "links": chain_links}
        del net, engine
        torch.cuda.empty_cache()
        return summ, None, None, None

    cfg = gen.config_by_name(args.workload)
    ceilings = measure_ceilings(torch, mxc)
    clock_before = smi_clock()
    summ, net, per_call, ev_ms = measure(cfg, args.steps, args.warmup, args.groups, True)
    clock_after = smi_clock()
    sec = summ["ms_per_step"] * 1e-3
    # the same step without backward-data of the first layer, which a training run never needs
    # (nothing consumes the gradient of the network input); reported beside the headline, labelled
    first = net.layers[0]
    pruned = timed_groups(torch, single_stream_step(net, keep=lambda c: not (c[1] == "bwd_data" and c[2] is first)),
                          max(3, args.steps // 4), 2, 3)
    flops_pruned = net.flops_per_step - first.L.flops_per_pass
    grouped = timed_groups(torch, single_stream_step(net, grouped=True), max(3, args.steps // 4), 2, 3)
    chain_step, chain_links = chained_grouped_step(net)
    chained = timed_groups(torch, chain_step, max(3, args.steps // 4), 2, 3)
    prep_calls = [s.prepare_filter for s in net.layers]
    prep = timed_groups(torch, lambda: [f() for f in prep_calls], max(3, args.steps // 4), 2, 3)
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_TFLOPS
    rl = rooflines(per_call, net, ev_ms)
    result = {
        "metric": "conv2d fwd+bwd TFLOP/s per network on 1 MI355X", "value": summ["tflops"], "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": summ["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "layers": len(cfg.layers), "batch": cfg.layers[0].N,
                   "layout": "nhwc-resident" if args.layout == "nhwc" else "nchw-per-call",
                   "step": ("layout(NCHW->NHWC of network input) + " if args.layout == "nhwc" else "") +
                           "per layer fwd, bwd_data, bwd_weight",
                   "schedule": summ["schedule"],
                   "timing": f"median of {args.groups} groups of exactly {args.steps} steps"},
        "groups_ms_per_step": summ["groups_ms"],
        "frac_of_mfma_peak": summ["frac_of_mfma_peak"],
        "single_stream": summ["single_stream"], "engine_schedule": summ["engine"],
        "roofline": rl[0] if rl else None,
        "roofline_kernels": rl,
        "ceilings": ceilings,
        "sclk": {"smi_before": clock_before, "smi_after": clock_after,
                 "derived_under_mfma_load_ghz": ceilings["sclk_ghz_under_mfma_load"]},
        "without_first_layer_bwd_data": {"value": round(flops_pruned / median(pruned) / 1e12, 3), "unit": "TFLOP/s",
                                         "ms_per_step": round(median(pruned) * 1e3, 4), "schedule": "single stream, eager"},
        "grouped_operations": {"value": round(net.flops_per_step / median(grouped) / 1e12, 3), "unit": "TFLOP/s",
                               "ms_per_step": round(median(grouped) * 1e3, 4), "schedule": "single stream, eager",
                               "note": "same convolution flops; forward + bias + ReLU, backward-data with the ReLU derivative "
                                       "(filter re-packed inside the call), backward-weight, bias gradient, SGD update of fp32 "
                                       "master weights with a bf16 copy (the extra work is not counted as flops)"},
        "chained_grouped_operations": {"value": round(net.flops_per_step / median(chained) / 1e12, 3), "unit": "TFLOP/s",
                                       "ms_per_step": round(median(chained) * 1e3, 4), "schedule": "single stream, eager",
                                       "links": chain_links,
                                       "note": "the grouped step with the listed layers chained on the device: y of one call is "
                                               "x of the next, dx of one call is dy of the layer below"},
        "filter_prepare_ms_per_step": round(median(prep) * 1e3, 4),
    }
    if cfg.dtype == "bf16":
        result["frac_of_measured_mfma"] = round(summ["tflops"] / ceilings["mfma_bf16_tflops_measured"], 4)
    for e in rl:
        e["frac_of_measured"] = round(e["achieved"] / (ceilings["mfma_bf16_tflops_measured"] if e["bound"] == "mfma"
                                                        else ceilings["copy_gbs_measured"] if e["bound"] == "hbm" else e["peak"]), 4)
    result["layers"] = [{"layer": c["layer"], "op": c["op"], "us": round(c["ms"] * 1e3, 1), "variant": c["variant"]} for c in per_call]
    if args.per_layer:
        for c in per_call:
            L = c["state"].L
            gbs = algorithmic_bytes(L, c["op"], net.esize) / c["ms"] / 1e6
            if c["op"] == "layout":
                print(f"{c['layer']:>24} {c['op']:>10} {c['ms']*1e3:9.1f} us {'':>17} {gbs:8.0f} GB/s  {c['variant']}", file=sys.stderr)
                continue
            tf = L.flops_per_pass / c["ms"] / 1e9
            print(f"{c['layer']:>24} {c['op']:>10} {c['ms']*1e3:9.1f} us {tf:8.1f} TFLOP/s {gbs:8.0f} GB/s  {c['variant']}",
                  file=sys.stderr)
    del net, per_call
    torch.cuda.empty_cache()
    result["layout_a1"] = layout_entry(torch, mxc)
    if not args.no_all:
        result["alt_algorithm_3x3_fwd"] = transform_entry(torch, mxc, gen)
    if not args.no_all:
        nets = {}
        for other in gen.CONFIGS:
            if other.name == cfg.name:
                continue
            nets[other.name] = measure(other, max(3, args.steps // 4), 2, 3, False)[0]
        result["networks"] = nets
        # the batch size of the paper's single-GPU comparison (its Section 4: batch 32), whole stack forward + backward
        result["networks_batch32"] = {n: measure(gen.config_by_name(n), max(3, args.steps // 4), 2, 3, False)[0]
                                      for n in ("alexnet_b32", "vgg_a_b32")}
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(gen, cfg, args.cpu_sample_batch)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
