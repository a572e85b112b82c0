"""Shared helpers of the GPU parity tests: upload seeded blocks, run the share through the C ABI
(via the thin binding), run the fp64 oracle on the same bits, compare element by element.

Tolerances (stated with the task): fp32 outputs |err| <= 1e-3 (1 + |ref|); bf16 outputs
|err| <= 8e-3 |ref| + 1e-3 (8e-3 is one bf16 step; the absolute floor is the fp32 criterion's,
needed where cancellation drives |ref| to zero).  The count of bf16 elements outside the pure
relative bound is printed with every comparison."""
from __future__ import annotations

import sys

import numpy as np
import torch

import paper_2110_14883_amd as T
import synth_inputs as S
from oracle import tp_oracle as O
from paper_2110_14883_amd import workloads as WL


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(bits: np.ndarray) -> torch.Tensor:
    """bf16 bit patterns (uint16) -> bf16 tensor on the GPU."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def host64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def f64(bits):
    return O.bf16_bits_to_f64(bits)


def compare(got: np.ndarray, ref: np.ndarray, kind: str, what: str) -> float:
    """Element-by-element comparison; prints the maxima and returns the worst err / bound."""
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - ref)
    if kind == "f32":
        bound = 1e-3 * (1.0 + np.abs(ref))
        extra = ""
    else:
        bound = 8e-3 * np.abs(ref) + 1e-3
        rel_viol = err > 8e-3 * np.abs(ref)
        extra = f" pure-relative violations {int(rel_viol.sum())}/{err.size}" + \
                (f" (largest |ref| among them {np.abs(ref)[rel_viol].max():.3g})" if rel_viol.any() else "")
    ratio = float((err / bound).max()) if err.size else 0.0
    over = int((err > bound).sum())
    say(f"    {what}: {kind} max|err| {err.max() if err.size else 0:.3g}, worst err/bound {ratio:.3f}"
        f"{'' if over == 0 else f', {over} of {err.size} elements over the bound'}{extra}")
    return ratio


def check(got: np.ndarray, ref: np.ndarray, kind: str, what: str) -> None:
    ratio = compare(got, ref, kind, what)
    assert ratio <= 1.0, f"{what}: {kind} parity violated, worst err/bound {ratio}"


def workspace_for(grid, dims) -> torch.Tensor | None:
    """Workspace for the calls made under the plan options in force (T.plan_opts): the query and the
    calls read the same options."""
    n = max(T.tp_linear_workspace_size(grid, dims, p) for p in (0, 1, 2))
    return torch.empty(max(n, 256), dtype=torch.uint8, device="cuda")


def overrides(tile=0, split=0, group=0, trim=1, rotate=1):
    """with overrides(tile=.., split=.., group=.., trim=.., rotate=..): plan options for the calls inside
    (trim / rotate: 1 on, 0 off)."""
    return T.plan_opts(tile=tile, split_k=split, group_m=group, rotate=1 if rotate else 2, trim=1 if trim else 2)


def torch_dtype(name):
    return torch.float32 if name == "f32" else torch.bfloat16


def run_share(grid, dims, n_steps=None, y_dtype="bf16", dx_dtype="bf16", backward=True, rows=None,
              w_rows=None, seed=S.BASE_SEED, synthetic_preact=False, epi=T.EPI_BIAS_GELU, want_db=False,
              use_own_slot=True, label="") -> None:
    """One rank's share on the GPU against the oracle.  rows / w_rows: sampled output rows of
    (Y, dX) / dW for big shares (None = every element).  synthetic_preact: take the own saved
    pre-activation from the generator instead of the oracle's full forward (big shares).

    Backward has two gates.  (1) Strict, always: every dA block, the rank's own included, is the
    oracle's; dX (its own dtype's tolerance) and dW, db (fp32 tolerance) against the oracle.
    (2) use_own_slot: the production path, in which the library forms its own dA block and uses
    it in dX / dW at once.  Its dA block is compared with the oracle's (bf16 tolerance); its dX,
    dW and db must equal, bit for bit, what the library computes when that same block is handed
    back as a ready-made input -- so the path is the strict path plus a dA block that differs
    from the oracle's only by bf16 rounding decisions taken in fp32 instead of fp64.  How far
    those decisions move dX / dW from the oracle's unbroken chain is printed (bf16 tolerance,
    elements over it, number of dA elements that rounded the other way), not asserted."""
    say(f"[case] {label} grid={grid} dims={dims} n_steps={n_steps} y={y_dtype} dx={dx_dtype} "
        f"rows={'all' if rows is None else len(rows)}")
    inp = WL.make_share_inputs(grid, dims, seed, n_steps, backward)
    m, n, k = inp["m"], inp["n"], inp["k"]
    ws = workspace_for(grid, dims)
    sel = slice(None) if rows is None else rows
    xs_d = [dev(b) for b in inp["x_blocks"]]
    ws_d = [dev(b) for b in inp["w_blocks"]]
    bias_d = dev(inp["bias"])
    y = torch.empty((m, n), dtype=torch_dtype(y_dtype), device="cuda")
    # an additive partial (1D row cut) takes no epilogue and saves no pre-activation
    pre = None if inp["fwd"]["partial"] else torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    say("  fwd: launching")
    T.tp_linear_fwd(grid, dims, inp["n_steps_fwd"], xs_d, ws_d, bias_d if epi != T.EPI_NONE else None, epi, y, pre, ws)
    torch.cuda.synchronize()
    x64 = [f64(b) for b in inp["x_blocks"]]
    w64 = [f64(b) for b in inp["w_blocks"]]
    A, Y = O.share_fwd(x64, w64, f64(inp["bias"]) if epi != T.EPI_NONE else None, epi == T.EPI_BIAS_GELU, rows)
    check(host64(y[sel]), Y, y_dtype, "Y")
    if pre is not None:
        check(host64(pre[sel]), A, "bf16", "A_saved")
    del xs_d, ws_d, x64, w64
    if not backward:
        return
    # ---- backward inputs: the oracle's values are what the GPU is fed
    if synthetic_preact or rows is not None:
        own = inp["fwd"]["out"]
        a_bits = S.normal_block_bf16(seed, S.T_PEER_A, dims[2], own[0] * m, m, own[1] * n, n, 0.02 * np.sqrt(dims[1]))
        A_saved = f64(a_bits)
    else:
        A_saved = O.round_to_bf16(A)
        a_bits = O.f64_to_bf16_bits(A_saved)
    g_own = f64(inp["g_own"])
    dA_own = O.share_da(g_own, A_saved)
    da_x = {inp["own_slot_dx"]: dA_own}
    da_w = {inp["own_slot_dw"]: dA_own}
    for i, (g, a) in inp["peers_dx"].items():
        da_x[i] = O.share_da(f64(g), f64(a))
    for i, (g, a) in inp["peers_dw"].items():
        da_w[i] = O.share_da(f64(g), f64(a))
    sx, sw = inp["n_steps_dx"], inp["n_steps_dw"]
    own_x, own_w = inp["own_slot_dx"], inp["own_slot_dw"]
    da_row_d = [dev(O.f64_to_bf16_bits(da_x[i])) for i in range(sx)]
    da_col_d = [da_row_d[own_x] if (i == own_w and own_x >= 0) else dev(O.f64_to_bf16_bits(da_w[i])) for i in range(sw)]
    w_dx_d = [dev(b) for b in inp["w_blocks_dx"]]
    x_dw_d = [dev(b) for b in inp["x_blocks_dw"]]
    mx = T.tp_block_map(grid, dims, T.PASS_DX)
    mw = T.tp_block_map(grid, dims, T.PASS_DW)
    g_d, a_d = dev(inp["g_own"]), dev(a_bits)

    def outputs():
        return (torch.empty((mx["m"], mx["n"]), dtype=torch_dtype(dx_dtype), device="cuda"),
                torch.empty((mw["m"], mw["n"]), dtype=torch.float32, device="cuda"),
                torch.empty((n,), dtype=torch.float32, device="cuda") if want_db else None)

    wsel = slice(None) if w_rows is None else w_rows
    w_dx64 = [f64(b) for b in inp["w_blocks_dx"]]
    x_dw64 = [f64(b) for b in inp["x_blocks_dw"]]
    dX = O.share_dx([da_x[i] for i in range(sx)], w_dx64, rows)
    dW = O.share_dw(x_dw64, [da_w[i] for i in range(sw)], w_rows)
    del w_dx64, x_dw64

    # ---- (1) strict gate: every dA block ready-made from the oracle
    say("  bwd: launching with every dA block given ready-made (the oracle's)")
    dx, dw, db = outputs()
    T.tp_linear_bwd(grid, dims, sx, sw, da_row_blocks=da_row_d, w_blocks_dx=w_dx_d, x_blocks_dw=x_dw_d,
                    da_col_blocks=da_col_d, dx=dx, dw=dw, workspace=ws)
    if want_db:
        T.tp_bias_grad(da_row_d[own_x] if own_x >= 0 else da_col_d[own_w], db, workspace=ws)
    torch.cuda.synchronize()
    check(host64(dx[sel]), dX, dx_dtype, "dX")
    check(host64(dw[wsel]), dW, "f32", "dW")
    if want_db:
        check(host64(db), dA_own.sum(axis=0), "f32", "db")
    if not use_own_slot:
        return

    # ---- (2) the library forms its own dA block and uses it at once
    say("  bwd: launching with the own dA block taken from this call")
    dx1, dw1, db1 = outputs()
    da_out = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    T.tp_linear_bwd(grid, dims, sx, sw, dy_own=g_d, preact_own=a_d,
                    da_row_blocks=[None if i == own_x else da_row_d[i] for i in range(sx)], w_blocks_dx=w_dx_d,
                    x_blocks_dw=x_dw_d, da_col_blocks=[None if i == own_w else da_col_d[i] for i in range(sw)],
                    own_slot_dx=own_x, own_slot_dw=own_w, dx=dx1, dw=dw1, da_own_out=da_out, db=db1, workspace=ws)
    torch.cuda.synchronize()
    da_gpu = host64(da_out)
    check(da_gpu, dA_own, "bf16", "dA_own")
    flips = int((da_gpu != dA_own).sum())
    say(f"    own dA: {flips} of {da_gpu.size} elements rounded the other way than the oracle's fp64 value")
    # the same products with that block handed back as a ready-made input
    dx2, dw2, db2 = outputs()
    T.tp_linear_bwd(grid, dims, sx, sw, da_row_blocks=[da_out if i == own_x else da_row_d[i] for i in range(sx)],
                    w_blocks_dx=w_dx_d, x_blocks_dw=x_dw_d,
                    da_col_blocks=[da_out if i == own_w else da_col_d[i] for i in range(sw)], dx=dx2, dw=dw2, workspace=ws)
    if want_db:
        T.tp_bias_grad(da_out, db2, workspace=ws)       # (the same workspace: the same slab sums, the same order)
    torch.cuda.synchronize()
    assert torch.equal(dx1, dx2), "dX: own-slot path differs from the ready-made path on the same dA block"
    assert torch.equal(dw1, dw2), "dW: own-slot path differs from the ready-made path on the same dA block"
    if want_db:
        assert torch.equal(db1, db2), "db: own-slot path differs from tp_bias_grad on the same dA block"
    # report only: distance of the chained results from the oracle's unbroken chain
    compare(host64(dx1[sel]), dX, "bf16", f"dX, own dA chained ({flips} flips; reported, not asserted)")
    compare(host64(dw1[wsel]), dW, "bf16", f"dW, own dA chained ({flips} flips; reported, not asserted)")
