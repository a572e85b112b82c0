"""tp_linear_fwd_static (the entry point for callers that cannot allocate): same result as
tp_linear_fwd with a caller workspace, on two calls in a row that share the built-in scratch array,
the second with a smaller input; both also against the fp64 oracle."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import paper_2110_14883_amd as T
import synth_inputs as S
from gpu_util import check, dev, f64, host64, say
from oracle import tp_oracle as O

pytestmark = pytest.mark.gpu


def _case(tag, m, k, n, epi, y_f32, seed):
    """One K-split forward product through both entry points."""
    grid, dims = T.Grid(T.MODE_1D_COL, p=1), (m, k, n)
    need = T.tp_linear_workspace_size(grid, dims, T.PASS_FWD)
    say(f"[no-alloc] {tag}: {m} x {k} x {n}, epi {epi}, workspace of the ordinary call {need} bytes")
    assert 0 < need <= T.tp_static_scratch_bytes(), "the case must use the scratch buffer (K split) and fit it"
    xb = S.normal_block_bf16(seed, S.T_X, k, 0, m, 0, k, 1.0)
    wb = S.normal_block_bf16(seed, S.T_W1, n, 0, k, 0, n, 0.02)
    bb = S.normal_block_bf16(seed, S.T_B1, n, 0, 1, 0, n, 0.02).reshape(-1)
    x, w, b = dev(xb), dev(wb), dev(bb)
    dt = torch.float32 if y_f32 else torch.bfloat16
    outs = []
    for static in (False, True):
        y = torch.full((m, n), float("nan"), dtype=dt, device="cuda")
        pre = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device="cuda") if epi != T.EPI_NONE else None
        bias = b if epi != T.EPI_NONE else None
        if static:
            T.tp_linear_fwd_static(grid, dims, 1, [x], [w], bias, epi, y, pre)
        else:
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            T.tp_linear_fwd(grid, dims, 1, [x], [w], bias, epi, y, pre, ws)
        torch.cuda.synchronize()
        outs.append((y, pre))
    (y0, p0), (y1, p1) = outs
    assert torch.equal(y0, y1), f"{tag}: y differs between tp_linear_fwd and tp_linear_fwd_static"
    if p0 is not None:
        assert torch.equal(p0, p1), f"{tag}: preact differs between the two entry points"
    A, Y = O.share_fwd([f64(xb)], [f64(wb)], f64(bb) if epi != T.EPI_NONE else None, act=epi == T.EPI_BIAS_GELU)
    check(host64(y1), Y, "f32" if y_f32 else "bf16", f"{tag} y (static) vs oracle")
    if p1 is not None:
        check(host64(p1), A, "bf16", f"{tag} preact (static) vs oracle")


def test_static_entry_point_matches_workspace_entry_point_twice():
    _case("first call", 520, 8192, 512, T.EPI_BIAS_GELU, False, S.BASE_SEED + 71)
    _case("second call, smaller", 296, 4096, 264, T.EPI_NONE, True, S.BASE_SEED + 72)
