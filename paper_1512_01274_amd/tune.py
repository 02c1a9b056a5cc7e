"""Tile-plan tuning on the device: times every candidate plan of the implicit-GEMM kernels (forward and
stride-1 backward-data) and of the backward-weight kernel for the layers of the benchmark stacks and
writes the winners into csrc/tuned_igemm.inc / csrc/tuned_wgrad.inc, which the library consults
before its time model.  Run on an MI355X, then rebuild:

    python -m paper_1512_01274_amd.tune [--iters 8] [--workloads alexnet_b128,vgg_a_b64,...] [--out-dir DIR]
    python -m paper_1512_01274_amd.build

Candidates are forced through the library's own tuning hooks (MXC_FORCE_VARIANT=<main>[+<tail>],
MXC_FORCE_WGRAD=<tile>[/<splits>]), so what is timed is exactly what a table hit will run.  Between timed
calls a 512 MiB buffer is rewritten so that a layer's operands come from HBM as they do inside a network
step, not from the caches a repeated call would warm.  Inputs are random tensors of the layers' shapes.
"""
import argparse
import os
import sys

import torch

from . import inputs as gen
from . import mxc

HERE = os.path.dirname(os.path.abspath(__file__))

IGEMM_TILES = {  # name -> (bm, bn, workgroups per CU)
    "igemm_128x128_k64s2_w4": (128, 128, 2), "igemm_256x256_k64s2_w8": (256, 256, 1),
    "igemm_256x128_k64s3_w8": (256, 128, 1), "igemm_128x256_k64s3_w8": (128, 256, 1),
    "igemm_128x64_k64s2_w4": (128, 64, 3), "igemm_256x64_k32s3_w4": (256, 64, 2),
    "igemm_128x32_k64s2_w4": (128, 32, 4), "igemm_256x32_k64s2_w4": (256, 32, 2),
    "igemm_256x192_k64s2_w8": (256, 192, 1), "igemm_192x256_k64s2_w8": (192, 256, 1),
    "igemm_64x256_k64s3_w8": (64, 256, 1), "igemm_64x128_k64s3_w4": (64, 128, 2),
    "igemm_192x128_k64s3_w8": (192, 128, 1),
}
WGRAD_TILES = {  # name -> (bm, bn, bp, workgroups per CU)
    "wgrad_128x128_p64s2_w4": (128, 128, 64, 2), "wgrad_256x256_p32s4_w8": (256, 256, 32, 1),
    "wgrad_256x128_p32s4_w8": (256, 128, 32, 1), "wgrad_128x256_p32s4_w8": (128, 256, 32, 1),
    "wgrad_64x64_p64s2_w4": (64, 64, 64, 4), "wgrad_64x128_p64s2_w4": (64, 128, 64, 2),
    "wgrad_128x64_p64s2_w4": (128, 64, 64, 2), "wgrad_256x256_p64s2_w8": (256, 256, 64, 1),
    "wgrad_128x128_p32s4_w4": (128, 128, 32, 2),
}


def ceil_div(a, b):
    return (a + b - 1) // b


def igemm_candidates(M, Co):
    """Single shapes whose column tile is not mostly padding, main+tail pairs where the main shape has
    at least one whole round and leaves rows over, and the streaming and the window kernel (the library declines one where
    the filter tile does not fit on chip; such a timing is discarded)."""
    ok = [n for n, (bm, bn, _) in IGEMM_TILES.items() if bn <= 2 * max(Co, 32) and (bn <= 64 or bn * 3 <= Co * 4 or bn <= Co)]
    out = list(ok) + mxc.mxc_tile_names(2)
    for a in ok:
        bm, bn, slots = IGEMM_TILES[a]
        tiles = ceil_div(M, bm) * ceil_div(Co, bn)
        rows = (tiles // (256 * slots)) * (256 * slots) // ceil_div(Co, bn) * bm
        if bm < 128 or rows <= 0 or rows >= M:
            continue
        for b in ok:
            if b != a and IGEMM_TILES[b][0] * IGEMM_TILES[b][1] <= bm * bn:
                out.append(a + "+" + b)
    return out


def wgrad_candidates(K, RSC, M):
    out = []
    for n, (bm, bn, bp, slots) in WGRAD_TILES.items():
        if (bm > 64 and bm * 3 > K * 4) or (bn > 64 and bn * 3 > RSC * 4):
            continue
        tiles = ceil_div(K, bm) * ceil_div(RSC, bn)
        fill = max(1, (256 * slots) // tiles)
        cand = {fill, max(1, fill // 2), fill * 2, max(1, (256 * slots * 2) // tiles), max(1, (256 * slots * 3) // tiles)}
        for sp in sorted(cand):
            if sp * 2 * bp <= M:
                out.append(f"{n}/{sp}")
    return out


class Timer:
    def __init__(self, iters):
        self.iters = iters
        self.flush = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")

    def time(self, fn):
        fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(self.iters)]
        for a, b in ev:
            self.flush.add_(1)
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        t = sorted(a.elapsed_time(b) for a, b in ev)
        return t[len(t) // 2] * 1e3        # median, us


def tune_layer(L, timer, igemm_rows, wgrad_rows, log):
    dt, lay = mxc.MXC_BF16, mxc.MXC_NHWC
    dims = L.dims()
    bf = lambda n: torch.randn(n, dtype=torch.float32, device="cuda").to(torch.bfloat16)
    x, w, dy = bf(L.N * L.C * L.H * L.W), bf(L.K * L.C * L.R * L.S) * 0.05, bf(L.N * L.K * L.P * L.Q)
    y = torch.empty(L.N * L.K * L.P * L.Q, dtype=torch.bfloat16, device="cuda")
    dx = torch.empty(L.N * L.C * L.H * L.W, dtype=torch.bfloat16, device="cuda")
    dw = torch.empty(L.K * L.C * L.R * L.S, dtype=torch.float32, device="cuda")

    def run(env, val, op, fn):
        os.environ[env] = val
        try:
            ws = mxc.alloc_workspace(mxc.mxc_conv2d_workspace_bytes(op, *dims, dt, lay))
            t = timer.time(lambda: fn(ws))
            if val.split("/")[0] not in mxc.mxc_last_variant():
                t = float("inf")            # the library ran something else: this candidate cannot run the problem
        except mxc.MxcError:
            t = float("inf")
        finally:
            del os.environ[env]
        return t

    # Forward and backward-data: the table is keyed on the GEMM the library plans (for first layers, the GEMM on
    # the packed operands), which the library reports after a call.  Strided backward-data of a plain layer runs
    # one GEMM per residue class and is planned by the model.
    jobs = [("fwd", mxc.MXC_FWD, lambda ws: mxc.mxc_conv2d_fwd(*dims, dt, lay, x, w, y, ws))]
    if L.stride == 1 or L.C <= 4:
        jobs.append(("bwd_data", mxc.MXC_BWD_DATA, lambda ws: mxc.mxc_conv2d_bwd_data(*dims, dt, lay, dy, w, dx, ws)))
    for name, op, fn in jobs:
        base = timer.time(lambda: fn(mxc.alloc_workspace(mxc.mxc_conv2d_workspace_bytes(op, *dims, dt, lay))))
        if "igemm" not in mxc.mxc_last_variant():
            continue
        M, Co, Kd = mxc.mxc_last_plan_key()
        res = sorted((run("MXC_FORCE_VARIANT", c, op, fn), c) for c in igemm_candidates(M, Co))
        log(f"{L.name:>22} {name:>9} M={M} Co={Co} Kd={Kd}: library default {base:7.1f} us; best " +
            ", ".join(f"{c} {t:.1f}" for t, c in res[:4]))
        t, c = res[0]
        if t == float("inf"):
            continue
        main, _, tail = c.partition("+")
        igemm_rows[(M, Co, Kd)] = (main, tail, t)
    M, RSC = L.N * L.P * L.Q, L.R * L.S * L.C
    fn = lambda ws: mxc.mxc_conv2d_bwd_weight(*dims, dt, lay, x, dy, dw, ws)
    base = timer.time(lambda: fn(mxc.alloc_workspace(mxc.mxc_conv2d_workspace_bytes(mxc.MXC_BWD_WEIGHT, *dims, dt, lay))))
    if "wgrad" in mxc.mxc_last_variant():
        res = sorted((run("MXC_FORCE_WGRAD", c, mxc.MXC_BWD_WEIGHT, fn), c) for c in wgrad_candidates(L.K, RSC, M))
        log(f"{L.name:>22} {'wgrad':>9} K={L.K} RSC={RSC} M={M}: library default {base:7.1f} us; best " +
            ", ".join(f"{c} {t:.1f}" for t, c in res[:4]))
        t, c = res[0]
        if t != float("inf"):
            tile, _, sp = c.partition("/")
            wgrad_rows[(L.N, L.H, L.W, L.C, L.K, L.R, L.S, L.stride, L.pad)] = (tile, int(sp), t)


def write_tables(igemm_rows, wgrad_rows, out_dir):
    with open(os.path.join(out_dir, "tuned_igemm.inc"), "w") as f:
        f.write("// Measured best plans of the implicit-GEMM kernels, one line per GEMM (rows M, output columns Co, reduction\n"
                "// length Kd): the shape for the whole rounds and, where a second launch pays, the shape for the rest.\n"
                "// Written by `python -m paper_1512_01274_amd.tune` from timings on an MI355X; GEMMs not listed here are\n"
                "// planned by the time model in igemm.hip.\n"
                "struct TunedIgemm { long long M; int Co, Kd; const char *main, *tail; };\n"
                "const TunedIgemm kTunedIgemm[] = {\n    {0, 0, 0, \"\", \"\"},\n")
        for (M, Co, Kd), (main, tail, t) in sorted(igemm_rows.items()):
            f.write(f"    {{{M}, {Co}, {Kd}, \"{main}\", \"{tail}\"}},   // {t:.1f} us\n")
        f.write("};\n")
    with open(os.path.join(out_dir, "tuned_wgrad.inc"), "w") as f:
        f.write("// Measured best tile and split count of the backward-weight kernel, one line per layer geometry\n"
                "// (N, H, W, C, K, R, S, stride, pad of the caller's problem).  Written by\n"
                "// `python -m paper_1512_01274_amd.tune` from timings on an MI355X; other geometries are planned by the\n"
                "// time model in wgrad.hip.\n"
                "struct TunedWgrad { int N, H, W, C, K, R, S, stride, pad; const char *tile; int splits; };\n"
                "const TunedWgrad kTunedWgrad[] = {\n    {0, 0, 0, 0, 0, 0, 0, 0, 0, \"\", 0},\n")
        for key, (tile, sp, t) in sorted(wgrad_rows.items()):
            f.write("    {" + ", ".join(str(v) for v in key) + f", \"{tile}\", {sp}}},   // {t:.1f} us\n")
        f.write("};\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=8)
    ap.add_argument("--workloads", default="alexnet_b128,inception3a_b128,vgg_a_b64,resnet_bottleneck_b256,alexnet_b32,vgg_a_b32")
    ap.add_argument("--log", default="")
    ap.add_argument("--out-dir", default=os.path.join(HERE, "csrc"), help="where the two .inc tables are written")
    args = ap.parse_args()
    assert torch.cuda.is_available(), "tuning needs the GPU"
    assert set(IGEMM_TILES) == set(mxc.mxc_tile_names(0)) and set(WGRAD_TILES) == set(mxc.mxc_tile_names(1)), \
        "the tile tables of this script and of the library differ"
    out = open(args.log, "w") if args.log else sys.stdout

    def log(s):
        print(s, file=out, flush=True)

    timer = Timer(args.iters)
    igemm_rows, wgrad_rows = {}, {}
    for name in args.workloads.split(","):
        cfg = gen.config_by_name(name)
        for L in cfg.layers:
            tune_layer(L, timer, igemm_rows, wgrad_rows, log)
            torch.cuda.empty_cache()
    write_tables(igemm_rows, wgrad_rows, args.out_dir)
    log(f"wrote {len(igemm_rows)} igemm and {len(wgrad_rows)} wgrad entries")


if __name__ == "__main__":
    main()
