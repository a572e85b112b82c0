"""Range test of a two-linear-layer model, recast for one GPU's share.

The paper's memory-efficiency experiment (Section 4, "Memory Efficiency", the range-test figure)
builds a model of two linear layers, runs it under 1D / 2D / 2.5D tensor parallelism on 4 GPUs
and under 1D / 2.5D (depth 2) / 3D on 8 GPUs, scales it once by batch size and once by hidden
size (up to 16384), and reports the memory each GPU needs.  Here one rank of each of those grids
runs its share of the same model, forward and backward, through libtplinear, and the run reports

  * stored bytes: what the rank itself keeps of every tensor of the two layers (its chunks of the
    input, both weights and biases, the saved pre-activation, the activations, the upstream
    gradient and every gradient it produces) -- the quantity the paper's figure compares;
  * resident bytes: the device memory the step's buffers occupy in this run, i.e. stored chunks plus
    the peers' blocks the share reads (pre-placed, since no communication is performed) plus the
    split-K workspace;
  * bf16 TFLOP/s of the rank's six products.

Readings (the paper gives neither the layer widths nor the sequence length of this test): both
layers are h x h, the first with bias and GeLU, the second with bias only; 512 tokens per sample;
the batch sweep runs at h = 2048, the hidden sweep at batch 32.  Inputs are seeded random device
buffers (timing and byte counts only; the same entry points are parity-tested elsewhere).

    python -m paper_2110_14883_amd.range_test [--quick] [--iters N]

Host-side bookkeeping and timing only: every product runs in the library's kernels.
"""
from __future__ import annotations

import argparse
import json
import sys

from . import binding as B

SEQ = 512


def grids(n_gpus: int):
    """The three schemes the paper runs on 4 and on 8 GPUs, one rank each (non-zero coordinates where
    the axis exists)."""
    if n_gpus == 4:
        return [("1D", B.Grid(B.MODE_1D_COL, p=4, ri=1)), ("2D", B.Grid(B.MODE_2D, q=2, ri=1, rj=0)),
                ("2.5D d=1", B.Grid(B.MODE_2P5D, q=2, d=1, ri=1, rj=0))]
    return [("1D", B.Grid(B.MODE_1D_COL, p=8, ri=1)), ("2.5D d=2", B.Grid(B.MODE_2P5D, q=2, d=2, ri=1, rj=0, rk=1)),
            ("3D", B.Grid(B.MODE_3D, p=2, ri=1, rj=0, rk=1))]


def stored_bytes(grid: B.Grid, M: int, h: int) -> int:
    """Bytes of the chunks one rank owns for the two-layer model, forward and backward.
    bf16 = 2 bytes for inputs, weights, activations and activation gradients; fp32 = 4 for weight
    gradients and for the 1D scheme's partial sums."""
    if grid.mode in (B.MODE_1D_COL, B.MODE_1D_ROW):
        n = grid.p
        full, cut = M * h, M * h // n                      # replicated [M, h] tensors and column-cut [M, h/n] ones
        w = h * h // n
        acts = 2 * full            # X
        acts += 2 * cut * 3        # A1 saved, Z, dA1
        acts += 4 * full           # Y partial (fp32)
        acts += 2 * full           # dY
        acts += 4 * full           # dX partial (fp32)
        params = 2 * (2 * w) + 2 * (h // n) + 2 * h        # W1[:, r], W2[r, :], b1[r], b2
        grads = 4 * (2 * w)
        return acts + params + grads
    if grid.mode in (B.MODE_2D, B.MODE_2P5D):
        q, d = grid.q, (grid.d if grid.mode == B.MODE_2P5D else 1)
        blk = (M // (q * d)) * (h // q)                    # every activation chunk: [M/(q d), h/q]
        w = (h // q) * (h // q)                            # weight chunk, repeated on every depth layer
        return 2 * blk * 7 + 2 * (2 * w) + 2 * 2 * (h // q) + 4 * (2 * w)     # X, A1, Z, Y, dY, dA1, dX
    if grid.mode == B.MODE_3D:
        p = grid.p
        blk = (M // (p * p)) * (h // p)                    # [M/p^2, h/p]
        w = (h // (p * p)) * (h // p)                      # the stored weight chunk is cut twice along its first dimension too
        return 2 * blk * 7 + 2 * (2 * w) + 2 * 2 * (h // p) + 4 * (2 * w)
    raise ValueError(grid.mode)


def _rand(gen, rows, cols, std=1.0):
    import torch
    return (torch.randn((rows, cols), generator=gen, device="cuda") * std).to(torch.bfloat16)


def build_share(grid: B.Grid, M: int, h: int, gen):
    """Device buffers and the list of library calls of one rank's two-layer step.  Returns (calls, flops,
    bufs): bufs names every input block and every output of the step (what a parity check needs)."""
    import torch
    f32, bf = torch.float32, torch.bfloat16
    empty = lambda r, c, dt=bf: torch.empty((r, c), dtype=dt, device="cuda")
    dims = (M, h, h)
    if grid.mode == B.MODE_1D_COL:
        n, r = grid.p, grid.ri
        g1, g2 = grid, B.Grid(B.MODE_1D_ROW, p=n, ri=r)
        hb = h // n
        X, W1, b1 = _rand(gen, M, h), _rand(gen, h, hb, 0.02), _rand(gen, 1, hb, 0.02)[0].contiguous()
        W2, G = _rand(gen, hb, h, 0.02), _rand(gen, M, h)
        Z, A1, Y, dA1 = empty(M, hb), empty(M, hb), empty(M, h, f32), empty(M, hb)
        dW2, dX, dW1 = empty(hb, h, f32), empty(M, h, f32), empty(h, hb, f32)
        ws = torch.empty(max(256, max(B.tp_linear_workspace_size(g, dims, ps) for g in (g1, g2) for ps in (0, 1, 2))),
                         dtype=torch.uint8, device="cuda")
        calls = [
            lambda: B.tp_linear_fwd(g1, dims, 1, [X], [W1], b1, B.EPI_BIAS_GELU, Z, A1, ws),
            lambda: B.tp_linear_fwd(g2, dims, 1, [Z], [W2], None, B.EPI_NONE, Y, None, ws),
            lambda: B.tp_linear_bwd(g2, dims, 1, 1, da_row_blocks=[G], w_blocks_dx=[W2], x_blocks_dw=[Z],
                                    da_col_blocks=[G], dgelu_preact=A1, dx=dA1, dw=dW2, workspace=ws),
            lambda: B.tp_linear_bwd(g1, dims, 1, 1, da_row_blocks=[dA1], w_blocks_dx=[W1], x_blocks_dw=[X],
                                    da_col_blocks=[dA1], dx=dX, dw=dW1, workspace=ws),
        ]
        bufs = dict(X=X, W1=W1, b1=b1, W2=W2, G=G, Z=Z, A1=A1, Y=Y, dA1=dA1, dW2=dW2, dX=dX, dW1=dW1)
        return calls, 6 * 2.0 * M * h * hb, bufs
    fm = B.tp_block_map(grid, dims, B.PASS_FWD)
    xm = B.tp_block_map(grid, dims, B.PASS_DX)
    wm = B.tp_block_map(grid, dims, B.PASS_DW)
    S, m, n, k = fm["n_steps"], fm["m"], fm["n"], fm["k"]
    own = fm["out"]
    ws = torch.empty(max(256, max(B.tp_linear_workspace_size(grid, dims, ps) for ps in (0, 1, 2))), dtype=torch.uint8, device="cuda")
    # layer 1 forward: X blocks of the rank's row, W1 blocks of its column
    x1 = [_rand(gen, m, k) for _ in range(S)]
    w1 = [_rand(gen, k, n, 0.02) for _ in range(S)]
    b1, b2 = _rand(gen, 1, n, 0.02)[0].contiguous(), _rand(gen, 1, n, 0.02)[0].contiguous()
    Z, A1 = empty(m, n), empty(m, n)
    # layer 2 forward reads the Z blocks of the row: the rank's own one plus the peers' (pre-placed)
    z2 = [Z if fm["a"][s] == own else _rand(gen, m, k) for s in range(S)]
    w2 = [_rand(gen, k, n, 0.02) for _ in range(S)]
    Y = empty(m, n)
    # layer 2 backward: upstream gradient blocks of the row (dX) and of the column group (dW)
    g_row = [_rand(gen, xm["m"], xm["k"]) for _ in range(S)]
    w2x = [_rand(gen, xm["n"], xm["k"], 0.02) for _ in range(S)]
    dA1 = empty(xm["m"], xm["n"])
    z_col = [_rand(gen, wm["k"], wm["m"]) for _ in range(S)]
    g_col = [_rand(gen, wm["k"], wm["n"]) for _ in range(S)]
    dW2, dW1 = empty(wm["m"], wm["n"], f32), empty(wm["m"], wm["n"], f32)
    # layer 1 backward: dA1 blocks of the row (own one from above), X blocks of the column group
    da_row = [dA1 if xm["a"][s] == own else _rand(gen, xm["m"], xm["k"]) for s in range(S)]
    w1x = [_rand(gen, xm["n"], xm["k"], 0.02) for _ in range(S)]
    dX = empty(xm["m"], xm["n"])
    x_col = [_rand(gen, wm["k"], wm["m"]) for _ in range(S)]
    da_col = [dA1 if wm["b"][s] == own else _rand(gen, wm["k"], wm["n"]) for s in range(S)]
    calls = [
        lambda: B.tp_linear_fwd(grid, dims, S, x1, w1, b1, B.EPI_BIAS_GELU, Z, A1, ws),
        lambda: B.tp_linear_fwd(grid, dims, S, z2, w2, b2, B.EPI_BIAS, Y, None, ws),
        lambda: B.tp_linear_bwd(grid, dims, S, S, da_row_blocks=g_row, w_blocks_dx=w2x, x_blocks_dw=z_col,
                                da_col_blocks=g_col, dgelu_preact=A1, dx=dA1, dw=dW2, workspace=ws),
        lambda: B.tp_linear_bwd(grid, dims, S, S, da_row_blocks=da_row, w_blocks_dx=w1x, x_blocks_dw=x_col,
                                da_col_blocks=da_col, dx=dX, dw=dW1, workspace=ws),
    ]
    bufs = dict(steps=S, own_fwd=[fm["a"][s] == own for s in range(S)], own_dx=[xm["a"][s] == own for s in range(S)],
                own_dw=[wm["b"][s] == own for s in range(S)],
                x1=x1, w1=w1, b1=b1, b2=b2, z2=z2, w2=w2, g_row=g_row, w2x=w2x, z_col=z_col, g_col=g_col,
                da_row=da_row, w1x=w1x, x_col=x_col, da_col=da_col, Z=Z, A1=A1, Y=Y, dA1=dA1, dW2=dW2, dX=dX, dW1=dW1)
    return calls, 6 * 2.0 * m * n * k * S, bufs


def run_point(name: str, grid: B.Grid, batch: int, h: int, iters: int) -> dict:
    import torch
    M = batch * SEQ
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    base = torch.cuda.memory_allocated()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(211014883 + 131 * batch + h)
    calls, flops, _ = build_share(grid, M, h, gen)
    torch.cuda.synchronize()
    resident = torch.cuda.memory_allocated() - base           # live buffers of the step (set-up temporaries are gone)
    import time
    for _ in range(3):
        for fn in calls:
            fn()
    torch.cuda.synchronize()
    if iters <= 0:
        # length from the step time: >= 80 ms of warm-up and >= 200 ms timed, so that the point is not
        # measured inside the power controller's settling transient after the buffers were filled
        t0 = time.perf_counter()
        for _ in range(3):
            for fn in calls:
                fn()
        torch.cuda.synchronize()
        est_ms = max((time.perf_counter() - t0) * 1e3 / 3, 1e-3)
        for _ in range(min(2000, int(80.0 / est_ms) + 1)):
            for fn in calls:
                fn()
        iters = max(10, min(4000, int(200.0 / est_ms) + 1))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        for fn in calls:
            fn()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    del calls
    return dict(scheme=name, batch=batch, hidden=h, tokens=M, stored_bytes=stored_bytes(grid, M, h),
                resident_bytes=int(resident), gemm_flops=flops, ms_per_step=round(ms, 4), iters=iters,
                tflops=round(flops / ms / 1e9, 1))


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--quick", action="store_true", help="two points per sweep instead of four")
    ap.add_argument("--iters", type=int, default=0, help="timed steps per point (0 = automatic, from the step time)")
    args = ap.parse_args(argv)
    import torch
    assert torch.cuda.is_available(), "the range test needs the GPU"
    B.lib()
    batches = [64, 512] if args.quick else [64, 128, 256, 512]
    hiddens = [2048, 16384] if args.quick else [2048, 4096, 8192, 16384]
    # warm the clocks: the first launches of a process run slower
    warm = run_point("warm-up", grids(4)[1][1], 32, 2048, 200)
    print(f"# warm-up {warm['tflops']} TFLOP/s", file=sys.stderr, flush=True)
    rows = []
    for n_gpus in (4, 8):
        for sweep, points in (("batch", [(b, 2048) for b in batches]), ("hidden", [(32, hh) for hh in hiddens])):
            for batch, h in points:
                ref = None
                for name, grid in grids(n_gpus):
                    r = run_point(name, grid, batch, h, args.iters)
                    r.update(n_gpus=n_gpus, sweep=sweep)
                    if name == "1D":
                        ref = r["stored_bytes"]
                    r["stored_vs_1d_pct_lower"] = round(100.0 * (1.0 - r["stored_bytes"] / ref), 1)
                    rows.append(r)
                    print(json.dumps(r), flush=True)
    print("\n| GPUs | sweep | batch | hidden | scheme | stored MiB | lower than 1D | resident MiB | ms/step | TFLOP/s |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['n_gpus']} | {r['sweep']} | {r['batch']} | {r['hidden']} | {r['scheme']} | {r['stored_bytes'] / 2**20:.0f} | "
              f"{r['stored_vs_1d_pct_lower']} % | {r['resident_bytes'] / 2**20:.0f} | {r['ms_per_step']} | {r['tflops']} |")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
