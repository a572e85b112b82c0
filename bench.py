#!/usr/bin/env python3
"""Benchmark of the per-rank tensor-parallel linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME] [--no-extra] [--no-cpu]

A step is one pass of the whole hot path of one rank's share (forward and backward, every
product and elementwise kernel) over one batch of seeded synthetic blocks that are already
resident in HBM.  The headline workload is the 3D (p = 2) share of the GPT-3-175B-shaped MLP, the
largest of the five configurations: forward 4096 x 6144 x 24576 with bias and erf-GeLU, dA, dX and dW
(3.71 TFLOP per step); the other configurations are measured after it, each for a length chosen
from its step time (>= 80 ms of warm-up, >= 250 ms timed: shorter runs sit in the power controller's
settling transient), and reported under "per_config".  Prints ONE JSON line.

value       = GEMM flops of the step / wall time of the step (bf16 TFLOP/s, fp32 accumulation)
roofline    = the dominant kernel (largest share of step time): its flops per launch / its average
              duration measured with HIP events on the launch stream, against the MI355X dense
              bf16 MFMA peak
cpu_baseline= the fp64 oracle timed on the host cores on the same share (all of it when that is a
              few seconds of BLAS-backed work, else a stated fraction of its token rows and dW rows)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0          # MI355X dense bf16 MFMA peak (published figure, 2.5 PFLOP/s)
NSETS = int(os.environ.get("TPL_BENCH_NSETS", "3"))   # buffer sets rotated through, so nothing is re-served from the 256 MB MALL

# HBM-side bytes per launch (read + written) from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# summarised in profiles/gemm4_config5_3d.md (scaled there by a copy of known size): the three products
# of the headline workload.  (Its dX is planned with K split in two: the launch is the fp32-partials
# instantiation, followed by the fix-up kernel's 252 MB.)
MEASURED_TRAFFIC_BYTES = {
    "tpl::tp_gemm4_kernel<true, false, 2, false>": 2235000000,     # forward NN + bias + GeLU: 1832 MB read, 403 MB written
    "tpl::tp_gemm4_kernel<false, false, 0, true>": 2655000000,     # dW TN: 2051 MB read, 604 MB written
    "tpl::tp_gemm4_kernel<true, true, 0, false>": 2038000000,      # dX NT (launched as <true, true, 0, true>): 1837 + 201 MB
    "tpl::tp_gemm4_kernel<true, true, 0, true>": 2038000000,
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def gemm_symbol(form: str, epi: int, f32_out: bool) -> str:
    """Name of the 256x256 GEMM instantiation a call launches (as rocprofv3 prints it, without
    'void' and the argument list).  form: NN / NT / TN; epi: 0 none, 1 bias, 2 bias+GeLU, 3 *GeLU'."""
    kc = {"NN": "true, false", "NT": "true, true", "TN": "false, false"}[form]
    return f"tpl::tp_gemm4_kernel<{kc}, {epi}, {'true' if f32_out else 'false'}>"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", default="c5_3d_p2")
    ap.add_argument("--no-extra", action="store_true", help="skip the other configurations")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--extra-steps", type=int, default=0,
                    help="timed steps of each other configuration (0 = automatic: >= 80 ms of warm-up, >= 250 ms timed)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU's share of the tensor-parallel layer; the blocks other "
              "ranks would send are pre-placed in HBM and no collective runs, so --gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2110_14883_amd as T
    import synth_inputs as S
    from paper_2110_14883_amd import workloads as WL

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    T.lib()
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    def up(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)

    def empty(shape, f32=False):
        return torch.empty(shape, dtype=torch.float32 if f32 else torch.bfloat16, device="cuda")

    def ws_for(grid, dims):
        n = max(T.tp_linear_workspace_size(grid, dims, p) for p in (0, 1, 2))
        return torch.empty(max(n, 256), dtype=torch.uint8, device="cuda")

    # ------------------------------------------------------------------ step builders
    # Each returns (calls, flops): calls = per-set lists of (label, flops, fn); fn enqueues ONE library call.
    def build_mlp1d(cfg):
        M, H, F = cfg.dims
        size, rank = cfg.grid.p, cfg.grid.ri
        inp = WL.make_mlp1d_inputs(size, rank, M, H, F)
        fb = inp["fb"]
        g1, d1 = T.Grid(T.MODE_1D_COL, p=size, ri=rank), (M, H, F)
        g2, d2 = T.Grid(T.MODE_1D_ROW, p=size, ri=rank), (M, F, H)
        one = 2.0 * M * H * fb
        sets = []
        base = {k: up(inp[k]) for k in ("X", "W1", "b1", "W2", "G")}
        for s in range(NSETS):
            b = base if s == 0 else {k: v.clone() for k, v in base.items()}
            o = dict(Z=empty((M, fb)), A=empty((M, fb)), Y=empty((M, H), True), dA=empty((M, fb)),
                     dW2=empty((fb, H), True), dX=empty((M, H), True), dW1=empty((H, fb), True),
                     ws1=ws_for(g1, d1), ws2=ws_for(g2, d2))
            calls = [
                ("fc1_fwd NN +bias+GeLU", one, gemm_symbol("NN", 2, False), lambda b=b, o=o: T.tp_linear_fwd(
                    g1, d1, 1, [b["X"]], [b["W1"]], b["b1"], T.EPI_BIAS_GELU, o["Z"], o["A"], o["ws1"])),
                ("fc2_fwd NN fp32 partial", one, gemm_symbol("NN", 0, True), lambda b=b, o=o: T.tp_linear_fwd(
                    g2, d2, 1, [o["Z"]], [b["W2"]], None, T.EPI_NONE, o["Y"], None, o["ws2"])),
                ("fc2_dX NT *GeLU'", one, gemm_symbol("NT", 3, False), lambda b=b, o=o: T.tp_linear_bwd(
                    g2, d2, 1, 0, da_row_blocks=[b["G"]], w_blocks_dx=[b["W2"]], dgelu_preact=o["A"], dx=o["dA"],
                    workspace=o["ws2"])),
                ("fc2_dW TN", one, gemm_symbol("TN", 0, True), lambda b=b, o=o: T.tp_linear_bwd(
                    g2, d2, 0, 1, x_blocks_dw=[o["Z"]], da_col_blocks=[b["G"]], dw=o["dW2"], workspace=o["ws2"])),
                ("fc1_dX NT fp32 partial", one, gemm_symbol("NT", 0, True), lambda b=b, o=o: T.tp_linear_bwd(
                    g1, d1, 1, 0, da_row_blocks=[o["dA"]], w_blocks_dx=[b["W1"]], dx=o["dX"], workspace=o["ws1"])),
                ("fc1_dW TN", one, gemm_symbol("TN", 0, True), lambda b=b, o=o: T.tp_linear_bwd(
                    g1, d1, 0, 1, x_blocks_dw=[b["X"]], da_col_blocks=[o["dA"]], dw=o["dW1"], workspace=o["ws1"])),
            ]
            sets.append(calls)
        return sets, 6 * one

    def build_share(cfg):
        grid, dims = cfg.grid, cfg.dims
        inp = WL.make_share_inputs(grid, dims, S.BASE_SEED, cfg.n_steps, cfg.backward)
        m, n, k = inp["m"], inp["n"], inp["k"]
        sf = inp["n_steps_fwd"]
        one = 2.0 * m * n * k * sf
        f32y = cfg.y_dtype == "f32"
        sets = []
        base = dict(x=[up(b) for b in inp["x_blocks"]], w=[up(b) for b in inp["w_blocks"]], bias=up(inp["bias"]))
        if cfg.backward:
            sx, sw = inp["n_steps_dx"], inp["n_steps_dw"]
            base.update(g=up(inp["g_own"]), wdx=[up(b) for b in inp["w_blocks_dx"]], xdw=[up(b) for b in inp["x_blocks_dw"]])
            # peers' dA blocks, made once by the library's own elementwise kernel from (G_peer, A_peer)
            def peer(pair):
                g, a = up(pair[0]), up(pair[1])
                out = torch.empty_like(g)
                T.tp_dgelu(g, a, out)
                return out
            memo = {}
            def peer_memo(pair):
                key = (pair[0].ctypes.data, pair[1].ctypes.data)
                if key not in memo:
                    memo[key] = peer(pair)
                return memo[key]
            if not cfg.second_linear:
                base["da_row"] = {i: peer_memo(p) for i, p in inp["peers_dx"].items()}
                base["da_col"] = {i: peer_memo(p) for i, p in inp["peers_dw"].items()}
            torch.cuda.synchronize()
        second = cfg.second_linear
        if second:
            # saved pre-activation of the previous layer for this rank's dX block: [m, k] bf16
            import math
            own = inp["dx"]["out"]
            base["a1"] = up(S.normal_block_bf16(S.BASE_SEED, S.T_PEER_A, dims[1], own[0] * m, m, own[1] * k, k,
                                                0.02 * math.sqrt(dims[1])))
            base["g_row"] = {i: up(p[0]) for i, p in inp["peers_dx"].items()}
            base["g_col"] = {i: up(p[0]) for i, p in inp["peers_dw"].items()}
        for s in range(NSETS):
            def cp(v):
                if s == 0:
                    return v
                if isinstance(v, list):
                    return [t.clone() for t in v]
                if isinstance(v, dict):
                    return {i: t.clone() for i, t in v.items()}
                return v.clone()
            b = {k_: cp(v) for k_, v in base.items()}
            o = dict(y=empty((m, n), f32y), pre=empty((m, n)), ws=ws_for(grid, dims))
            if second:
                calls = [("fwd NN +bias", one, gemm_symbol("NN", 1, f32y), lambda b=b, o=o: T.tp_linear_fwd(
                    grid, dims, sf, b["x"], b["w"], b["bias"], T.EPI_BIAS, o["y"], None, o["ws"]))]
                o.update(dx=empty((m, k)), dw=empty((k, n), True))
                rows = [b["g"] if i == inp["own_slot_dx"] else b["g_row"][i] for i in range(sx)]
                cols = [b["g"] if i == inp["own_slot_dw"] else b["g_col"][i] for i in range(sw)]
                calls += [
                    ("dX NT *GeLU'", one, gemm_symbol("NT", 3, False), lambda b=b, o=o, rows=rows: T.tp_linear_bwd(
                        grid, dims, sx, 0, da_row_blocks=rows, w_blocks_dx=b["wdx"], dgelu_preact=b["a1"], dx=o["dx"],
                        workspace=o["ws"])),
                    ("dW TN", one, gemm_symbol("TN", 0, True), lambda b=b, o=o, cols=cols: T.tp_linear_bwd(
                        grid, dims, 0, sw, x_blocks_dw=b["xdw"], da_col_blocks=cols, dw=o["dw"], workspace=o["ws"])),
                ]
                sets.append(calls)
                continue
            calls = [("fwd NN +bias+GeLU", one, gemm_symbol("NN", 2, f32y), lambda b=b, o=o: T.tp_linear_fwd(
                grid, dims, sf, b["x"], b["w"], b["bias"], T.EPI_BIAS_GELU, o["y"], o["pre"], o["ws"]))]
            if cfg.backward:
                o.update(da=empty((m, n)), dx=empty((m, k), cfg.dx_dtype == "f32"), dw=empty((k, n), True))
                rows = [o["da"] if i == inp["own_slot_dx"] else b["da_row"][i] for i in range(sx)]
                cols = [o["da"] if i == inp["own_slot_dw"] else b["da_col"][i] for i in range(sw)]
                calls += [
                    ("dA = dY*GeLU'(A)", 0.0, "tpl::tp_dgelu_kernel", lambda b=b, o=o: T.tp_linear_bwd(
                        grid, dims, 0, 0, dy_own=b["g"], preact_own=o["pre"], da_own_out=o["da"], workspace=o["ws"]), 6.0 * m * n),
                    ("dX NT", one, gemm_symbol("NT", 0, cfg.dx_dtype == "f32"), lambda b=b, o=o, rows=rows: T.tp_linear_bwd(
                        grid, dims, sx, 0, da_row_blocks=rows, w_blocks_dx=b["wdx"], dx=o["dx"], workspace=o["ws"])),
                    ("dW TN", one, gemm_symbol("TN", 0, True), lambda b=b, o=o, cols=cols: T.tp_linear_bwd(
                        grid, dims, 0, sw, x_blocks_dw=b["xdw"], da_col_blocks=cols, dw=o["dw"], workspace=o["ws"])),
                ]
            sets.append(calls)
        return sets, one * (3 if cfg.backward else 1)

    def build_partials(cfg):
        """Forward as in the owner-computes share, backward as partials for other owners."""
        grid, dims = cfg.grid, cfg.dims
        fin = WL.make_share_inputs(grid, dims, S.BASE_SEED, None, False)
        pin = WL.make_partials_inputs(grid, dims)
        m, n, k, sf, q = fin["m"], fin["n"], fin["k"], fin["n_steps_fwd"], pin["dx"]["n_steps"]
        one = 2.0 * m * n * k * sf
        wsb = max([T.tp_linear_workspace_size(grid, dims, ps) for ps in (0, 3, 4)] + [256])
        base = dict(x=[up(b) for b in fin["x_blocks"]], w=[up(b) for b in fin["w_blocks"]], bias=up(fin["bias"]),
                    g=up(pin["da_own"]), wp=[up(b) for b in pin["w_blocks"]], xp=[up(b) for b in pin["x_blocks"]])
        sets = []
        for s in range(NSETS):
            b = base if s == 0 else {k_: ([t.clone() for t in v] if isinstance(v, list) else v.clone()) for k_, v in base.items()}
            o = dict(y=empty((m, n)), pre=empty((m, n)), da=empty((m, n)), ws=torch.empty(wsb, dtype=torch.uint8, device="cuda"),
                     dxp=[empty((m, k), True) for _ in range(q)], dwp=[empty((k, n), True) for _ in range(q)])
            sets.append([
                ("fwd NN +bias+GeLU", one, gemm_symbol("NN", 2, False), lambda b=b, o=o: T.tp_linear_fwd(
                    grid, dims, sf, b["x"], b["w"], b["bias"], T.EPI_BIAS_GELU, o["y"], o["pre"], o["ws"])),
                ("dA = dY*GeLU'(A)", 0.0, "tpl::tp_dgelu_kernel", lambda b=b, o=o: T.tp_dgelu(b["g"], o["pre"], o["da"]), 6.0 * m * n),
                (f"dX partials NT x{q}", one, gemm_symbol("NT", 0, True), lambda b=b, o=o: T.tp_linear_bwd_partials(
                    grid, dims, o["da"], b["wp"], o["dxp"], None, None, o["ws"])),
                (f"dW partials TN x{q}", one, gemm_symbol("TN", 0, True), lambda b=b, o=o: T.tp_linear_bwd_partials(
                    grid, dims, o["da"], None, None, b["xp"], o["dwp"], o["ws"])),
            ])
        return sets, 3 * one

    def build_gathered(cfg):
        grid, dims = cfg.grid, cfg.dims
        inp = WL.make_gathered3d_inputs(grid, dims)
        ms, hb, fb, p, l = inp["m"], inp["h"], inp["f"], grid.p, grid.rk
        mc = ms // p
        one = 2.0 * ms * hb * fb
        base = dict(x=up(inp["x"]), w=up(inp["w"]), da=up(inp["da"]), bias=up(inp["bias"]))
        sets = []
        for s in range(NSETS):
            b = base if s == 0 else {k_: v.clone() for k_, v in base.items()}
            o = dict(c=empty((ms, fb), True), y=empty((mc, fb)), pre=empty((mc, fb)), dx=empty((ms, hb), True),
                     dw=empty((hb, fb), True), ws=ws_for(grid, dims))
            sets.append([
                ("fwd NN fp32 partial", one, gemm_symbol("NN", 0, True), lambda b=b, o=o: T.tp_linear_fwd(
                    grid, dims, 1, [b["x"]], [b["w"]], None, T.EPI_NONE, o["c"], None, o["ws"])),
                ("bias+GeLU on the rank's chunk", 0.0, "tpl::tp_bias_act_kernel", lambda b=b, o=o: T.tp_bias_act(
                    o["c"][l * mc:(l + 1) * mc], b["bias"], T.EPI_BIAS_GELU, o["y"], o["pre"]), 8.0 * mc * fb),
                ("dX NT fp32 partial", one, gemm_symbol("NT", 0, True), lambda b=b, o=o: T.tp_linear_bwd(
                    grid, dims, 1, 0, da_row_blocks=[b["da"]], w_blocks_dx=[b["w"]], dx=o["dx"], workspace=o["ws"])),
                ("dW TN fp32 partial", one, gemm_symbol("TN", 0, True), lambda b=b, o=o: T.tp_linear_bwd(
                    grid, dims, 0, 1, x_blocks_dw=[b["x"]], da_col_blocks=[b["da"]], dw=o["dw"], workspace=o["ws"])),
            ])
        return sets, 3 * one

    def run_config(cfg, steps, warmup):
        log(f"[bench] {cfg.name}: generating inputs")
        t0 = time.time()
        builder = {"partials": build_partials, "gathered": build_gathered}.get(cfg.variant) or (build_mlp1d if cfg.chain_1d else build_share)
        sets, flops = builder(cfg)
        ncall = len(sets[0])
        if steps <= 0:
            # Automatic length.  After a burst of work starts, the chip's power control first lets the clocks
            # run high, then cuts them hard and takes some tens of milliseconds to settle (seen in the kernel
            # trace: 249 us, then 376 us, then a slow return to ~255 us for the same launch).  A short workload
            # timed over 20 steps sits inside that dip, so warm up for >= 80 ms and time >= 250 ms.
            for i in range(3):
                for _, _, _, fn, *_ in sets[i % NSETS]:
                    fn()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for i in range(3):
                for _, _, _, fn, *_ in sets[i % NSETS]:
                    fn()
            torch.cuda.synchronize()
            est_ms = max((time.perf_counter() - t1) * 1e3 / 3, 1e-3)
            warmup = max(5, min(2000, int(80.0 / est_ms) + 1))
            steps = max(20, min(4000, int(250.0 / est_ms) + 1))
        log(f"[bench] {cfg.name}: inputs ready in {time.time() - t0:.1f}s; warmup {warmup}, steps {steps}")
        for i in range(warmup):
            for _, _, _, fn, *_ in sets[i % NSETS]:
                fn()
        torch.cuda.synchronize()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(ncall + 1)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            calls = sets[i % NSETS]
            ev[i][0].record(stream)
            for j, (_, _, _, fn, *_) in enumerate(calls):
                fn()
                ev[i][j + 1].record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms_step = wall * 1e3 / steps
        per_call = []
        for j, (label, fl, sym, _, *rest) in enumerate(sets[0]):
            ms = sum(ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(steps)) / steps
            row = dict(call=label, kernel=sym, ms=round(ms, 4), flops=fl, tflops=round(fl / ms / 1e9, 1) if fl else None)
            if rest:        # an HBM-bound elementwise call: algorithmic bytes (read + written) and the rate
                row.update(bytes=rest[0], tb_per_s=round(rest[0] / ms / 1e9, 2))
            per_call.append(row)
        graph = None
        if ms_step < 0.2:
            # launch-latency-bound step: also time it replayed from a HIP graph (the library only enqueues
            # kernels, so its calls can be captured); one graph per buffer set, replayed in rotation
            side = torch.cuda.Stream()
            graphs = []
            with torch.cuda.stream(side):
                for calls in sets:
                    for _, _, _, fn, *_ in calls:
                        fn()
                    side.synchronize()
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=side):
                        for _, _, _, fn, *_ in calls:
                            fn()
                    graphs.append(g)
            torch.cuda.synchronize()
            for i in range(warmup):
                graphs[i % NSETS].replay()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for i in range(steps):
                graphs[i % NSETS].replay()
            torch.cuda.synchronize()
            g_ms = (time.perf_counter() - t1) * 1e3 / steps
            graph = dict(ms_per_step=round(g_ms, 4), tflops=round(flops / g_ms / 1e9, 1))
            del graphs
        res = dict(workload=cfg.name, note=cfg.note, ms_per_step=round(ms_step, 4), gemm_flops=flops,
                   tflops=round(flops / ms_step / 1e9, 1), pct_of_peak=round(flops / ms_step / 1e9 / PEAK_BF16_TFLOPS * 100, 2),
                   steps=steps, warmup=warmup, calls=per_call)
        if graph:
            res["hip_graph_replay"] = graph
        del sets
        torch.cuda.empty_cache()
        return res

    def mfma_only_ceiling():
        """Dense bf16 MFMA rate the chip sustains with nothing else running (register-resident loop of
        libtpprobe.so, a measurement aid built beside the library, not part of it)."""
        import ctypes as C
        probe = C.CDLL(os.path.join(ROOT, "paper_2110_14883_amd", "libtpprobe.so"))
        probe.tp_mfma_probe.restype = C.c_int
        probe.tp_mfma_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.POINTER(C.c_double), C.c_void_p]
        scratch = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
        best = 0.0
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fl = C.c_double()
            st = probe.tp_mfma_probe(scratch.data_ptr(), scratch.numel() * 4, 40000, C.byref(fl), stream.cuda_stream)
            assert st == 0, f"tp_mfma_probe failed with status {st}"
            flops = fl.value
            e1.record(stream)
            torch.cuda.synchronize()
            best = max(best, flops / e0.elapsed_time(e1) / 1e9)
        return round(best, 1)

    cfg = WL.config(args.config)
    main_res = run_config(cfg, args.steps, args.warmup)
    mfma_only = mfma_only_ceiling()

    # dominant kernel = the kernel symbol with the largest share of the step
    by_sym = {}
    for c in main_res["calls"]:
        if c["tflops"] is not None:
            by_sym.setdefault(c["kernel"], []).append(c)
    kname, lst = max(by_sym.items(), key=lambda kv: sum(c["ms"] for c in kv[1]))
    flops_per_launch = sum(c["flops"] for c in lst) / len(lst)
    avg_ms = sum(c["ms"] for c in lst) / len(lst)
    achieved = flops_per_launch / avg_ms / 1e9
    roofline = dict(bound="mfma", kernel=kname, launches_per_step=len(lst), avg_launch_ms=round(avg_ms, 4),
                    flops_per_launch=flops_per_launch, achieved=round(achieved, 1), peak=PEAK_BF16_TFLOPS,
                    unit="TFLOP/s", frac=round(achieved / PEAK_BF16_TFLOPS, 4),
                    traffic=MEASURED_TRAFFIC_BYTES.get(kname),
                    measured_mfma_only_tflops=mfma_only, frac_of_measured_mfma_only=round(achieved / mfma_only, 4))

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(cfg)

    extra = []
    if not args.no_extra:
        for c in WL.CONFIGS:
            if c.name == cfg.name:
                continue
            extra.append(run_config(c, args.extra_steps, 5))

    out = {
        "metric": "bf16 TFLOP/s of per-rank TP linear fwd+bwd; % of MFMA dense peak",
        "value": main_res["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.note}", "parallelism": "one rank's share, 1 GPU",
                   "gemm_flops_per_step": main_res["gemm_flops"]},
        "pct_of_mfma_peak": main_res["pct_of_peak"],
        "roofline": roofline, "cpu_baseline": cpu, "calls": main_res["calls"], "per_config": extra,
        "hip_graph_replay": main_res.get("hip_graph_replay"),
    }
    print(json.dumps(out), flush=True)
    return 0


def cpu_baseline(cfg):
    """The fp64 oracle, as it stands, on the host cores, on the same share."""
    import numpy as np

    import synth_inputs as S
    from oracle import tp_oracle as O
    from paper_2110_14883_amd import workloads as WL

    cores = os.cpu_count() or 1
    try:
        from threadpoolctl import threadpool_info
        info = [p for p in threadpool_info() if p.get("user_api") == "blas"]
        if info:
            cores = int(info[0].get("num_threads", cores))
    except Exception:
        pass
    M, H, F = cfg.dims
    if cfg.chain_1d:
        size, rank = cfg.grid.p, cfg.grid.ri
        rows = M                                 # the whole share: a few seconds of BLAS-backed fp64 work
        inp = WL.make_mlp1d_inputs(size, rank, rows, H, F)
        X, W1, b1, W2, G = (O.bf16_bits_to_f64(inp[k]) for k in ("X", "W1", "b1", "W2", "G"))
        t0 = time.perf_counter()
        fw = O.mlp1d_fwd(X, W1, b1, W2)
        O.mlp1d_bwd(X, W1, W2, fw["A_saved"], fw["Z"], G)
        dt = time.perf_counter() - t0
        flops = 6 * 2.0 * rows * H * inp["fb"]
        sample = f"all six products of the same rank share, {rows} of {M} token rows"
    else:
        # owner-computes share: forward (+ bias, GeLU), own dA, dX over the row's dA blocks, dW over the
        # column's.  The peers' dA blocks are inputs (as on the GPU), made before the clock starts.
        # Bounded to about 6 TFLOP of fp64 work (10 - 30 s on a GPU machine's host share) by taking the first `rows` token rows of the share
        # (dW's contraction then runs over those rows only: the same arithmetic, a slab of the sum).
        inp = WL.make_share_inputs(cfg.grid, cfg.dims, S.BASE_SEED, cfg.n_steps, cfg.backward)
        m, n, k, sf = inp["m"], inp["n"], inp["k"], inp["n_steps_fwd"]
        one = 2.0 * m * n * k * sf
        nprod = 3 if cfg.backward else 1
        rows = max(1, min(m, int(m * 6.0e12 / (one * nprod))))
        rsel = slice(0, rows)
        xb = [O.bf16_bits_to_f64(b[rsel]) for b in inp["x_blocks"]]
        wb = [O.bf16_bits_to_f64(b) for b in inp["w_blocks"]]
        bias = O.bf16_bits_to_f64(inp["bias"])
        if cfg.backward:
            g_own = O.bf16_bits_to_f64(inp["g_own"][rsel])
            wdx = [O.bf16_bits_to_f64(b) for b in inp["w_blocks_dx"]]
            xdw = [O.bf16_bits_to_f64(b[rsel]) for b in inp["x_blocks_dw"]]
            peer = lambda pr: O.share_da(O.bf16_bits_to_f64(pr[0][rsel]), O.bf16_bits_to_f64(pr[1][rsel]))
            peers_dx = {i: peer(pr) for i, pr in inp["peers_dx"].items()}
            peers_dw = {i: peer(pr) for i, pr in inp["peers_dw"].items()}
        t0 = time.perf_counter()
        A, _ = O.share_fwd(xb, wb, bias, act=True)
        if cfg.backward:
            dA = O.share_da(g_own, O.round_to_bf16(A))
            O.share_dx([dA if i == inp["own_slot_dx"] else peers_dx[i] for i in range(inp["n_steps_dx"])], wdx)
            O.share_dw(xdw, [dA if i == inp["own_slot_dw"] else peers_dw[i] for i in range(inp["n_steps_dw"])])
        dt = time.perf_counter() - t0
        flops = nprod * one * rows / m
        sample = (f"the first {rows} of {m} token rows of the same rank share: forward with bias and GeLU, own dA, dX, "
                  f"and dW summed over those rows" if cfg.backward else f"the first {rows} of {m} token rows of the forward share")
    log(f"[bench] cpu oracle: {flops / dt / 1e9:.1f} GFLOP/s fp64 on {cores} threads ({dt:.1f}s)")
    return dict(value=round(flops / dt / 1e12, 4), unit="TFLOP/s", cores=cores, kind="oracle", sample=sample,
                seconds=round(dt, 2), dtype="f64")


if __name__ == "__main__":
    sys.exit(main())
