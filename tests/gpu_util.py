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


def check(got: np.ndarray, ref: np.ndarray, kind: str, what: str, slack=None) -> None:
    """slack: an extra per-element allowance derived from oracle values only (see flip_slack)."""
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - ref)
    if slack is not None:
        err = np.maximum(err - slack, 0.0)
    if kind == "f32":
        bound = 1e-3 * (1.0 + np.abs(ref))
        extra = ""
    else:
        bound = 8e-3 * np.abs(ref) + 1e-3
        rel_viol = err > 8e-3 * np.abs(ref)
        extra = f" pure-relative violations {int(rel_viol.sum())}/{err.size}" + \
                (f" (largest |ref| among them {np.abs(ref)[rel_viol].max():.3g})" if rel_viol.any() else "")
    ratio = float((err / bound).max()) if err.size else 0.0
    say(f"    {what}: {kind} max|err| {err.max() if err.size else 0:.3g}, worst err/bound {ratio:.3f}{extra}")
    assert ratio <= 1.0, f"{what}: {kind} parity violated, worst err/bound {ratio}"


def flip_slack(exact: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """Where may a bf16 rounding taken in fp32 differ from the one taken in fp64?

    The library forms dA = bf16(g GeLU'(a)) in fp32 (|error| below 4e-6 (|g| + |value|): erf to
    1.5e-7, a handful of fp32 roundings); the oracle rounds the exact value.  The two can differ,
    by one bf16 step, only where the exact value lies that close to a rounding midpoint.  Returns
    one bf16 step at those elements and 0 elsewhere -- computed from oracle values alone.  When the
    library then USES its own dA block in dX / dW, products of this slack with |W| / |X| bound
    what those few elements can change."""
    _, e = np.frexp(exact)
    ulp = np.ldexp(1.0, e - 8)
    gap = 0.5 * ulp - np.abs(exact - O.round_to_bf16(exact))
    return np.where(gap <= 4e-6 * (np.abs(scale) + np.abs(exact)), ulp, 0.0)


def workspace_for(grid, dims) -> torch.Tensor | None:
    n = max(T.tp_linear_workspace_size(grid, dims, p) for p in (0, 1, 2))
    # overrides may ask for more planes than the automatic plan: leave room for 8
    mp = [T.tp_block_map(grid, dims, p) for p in (0, 1, 2)]
    n = max(n, max(8 * x["m"] * x["n"] * 4 for x in mp) if _overrides_active else n)
    return torch.empty(max(n, 256), dtype=torch.uint8, device="cuda")


_overrides_active = False


class overrides:
    """with overrides(tile=.., split=.., group=.., trim=..): plan overrides for the calls inside."""

    def __init__(self, tile=0, split=0, group=0, trim=1):
        self.v = (tile, split, group)
        self.trim = trim

    def __enter__(self):
        global _overrides_active
        _overrides_active = any(self.v)
        for k, v in enumerate(self.v):
            T.tp_plan_override(k, v)
        T.tp_plan_override(4, self.trim)

    def __exit__(self, *a):
        global _overrides_active
        _overrides_active = False
        for k in range(3):
            T.tp_plan_override(k, 0)
        T.tp_plan_override(4, 1)


def torch_dtype(name):
    return torch.float32 if name == "f32" else torch.bfloat16


def run_share(grid, dims, n_steps=None, y_dtype="bf16", dx_dtype="bf16", backward=True, rows=None,
              w_rows=None, seed=S.BASE_SEED, synthetic_preact=False, epi=T.EPI_BIAS_GELU, want_db=False,
              use_own_slot=True, label="") -> None:
    """One rank's share on the GPU against the oracle.  rows / w_rows: sampled output rows of
    (Y, dX) / dW for big shares (None = every element).  use_own_slot: the library uses the dA block it has just computed
    for the rank's own step (the production path; tolerance widened only at elements the oracle
    shows to sit on a bf16 rounding boundary), else every dA block is given ready-made from the
    oracle (strict tolerance everywhere).  synthetic_preact: take the own saved
    pre-activation from the generator instead of the oracle's full forward (big shares)."""
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
    pre = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    say("  fwd: launching")
    T.tp_linear_fwd(grid, dims, inp["n_steps_fwd"], xs_d, ws_d, bias_d if epi != T.EPI_NONE else None, epi, y, pre, ws)
    torch.cuda.synchronize()
    x64 = [f64(b) for b in inp["x_blocks"]]
    w64 = [f64(b) for b in inp["w_blocks"]]
    A, Y = O.share_fwd(x64, w64, f64(inp["bias"]) if epi != T.EPI_NONE else None, epi == T.EPI_BIAS_GELU, rows)
    check(host64(y[sel]), Y, y_dtype, "Y")
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
    slack = flip_slack(g_own * O.dgelu(A_saved), g_own)
    say(f"    own dA: {int((slack > 0).sum())} of {slack.size} elements lie on a bf16 rounding boundary")
    da_x = {inp["own_slot_dx"]: dA_own}
    da_w = {inp["own_slot_dw"]: dA_own}
    for i, (g, a) in inp["peers_dx"].items():
        da_x[i] = O.share_da(f64(g), f64(a))
    for i, (g, a) in inp["peers_dw"].items():
        da_w[i] = O.share_da(f64(g), f64(a))
    sx, sw = inp["n_steps_dx"], inp["n_steps_dw"]
    own_x, own_w = (inp["own_slot_dx"], inp["own_slot_dw"]) if use_own_slot else (-1, -1)
    da_row_d = [None if i == own_x else dev(O.f64_to_bf16_bits(da_x[i])) for i in range(sx)]
    da_col_d = [None if i == own_w else dev(O.f64_to_bf16_bits(da_w[i])) for i in range(sw)]
    w_dx_d = [dev(b) for b in inp["w_blocks_dx"]]
    x_dw_d = [dev(b) for b in inp["x_blocks_dw"]]
    mx = T.tp_block_map(grid, dims, T.PASS_DX)
    mw = T.tp_block_map(grid, dims, T.PASS_DW)
    dx = torch.empty((mx["m"], mx["n"]), dtype=torch_dtype(dx_dtype), device="cuda")
    dw = torch.empty((mw["m"], mw["n"]), dtype=torch.float32, device="cuda")
    da_out = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    db = torch.empty((n,), dtype=torch.float32, device="cuda") if want_db else None
    say(f"  bwd: launching (own dA block {'taken from this call' if use_own_slot else 'given ready-made'})")
    T.tp_linear_bwd(grid, dims, sx, sw, dy_own=dev(inp["g_own"]), preact_own=dev(a_bits),
                    da_row_blocks=da_row_d, w_blocks_dx=w_dx_d, x_blocks_dw=x_dw_d, da_col_blocks=da_col_d,
                    own_slot_dx=own_x, own_slot_dw=own_w,
                    dx=dx, dw=dw, da_own_out=da_out, db=db, workspace=ws)
    torch.cuda.synchronize()
    check(host64(da_out), dA_own, "bf16", "dA_own")
    if want_db:
        check(host64(db), dA_own.sum(axis=0), "f32", "db", slack.sum(axis=0))
    wsel = slice(None) if w_rows is None else w_rows
    w_dx64 = [f64(b) for b in inp["w_blocks_dx"]]
    x_dw64 = [f64(b) for b in inp["x_blocks_dw"]]
    sl_x = sl_w = None
    if use_own_slot and own_x >= 0:
        sl_x = slack[sel] @ np.abs(w_dx64[own_x]).T
    if use_own_slot and own_w >= 0:
        sl_w = np.abs(x_dw64[own_w][:, wsel]).T @ slack
    dX = O.share_dx([da_x[i] for i in range(sx)], w_dx64, rows)
    check(host64(dx[sel]), dX, dx_dtype, "dX", sl_x)
    dW = O.share_dw(x_dw64, [da_w[i] for i in range(sw)], w_rows)
    check(host64(dw[wsel]), dW, "f32", "dW", sl_w)
