"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on the same seeded bits.
Small shares are compared element by element (several tiles, ragged tails, every mode, every
macro-tile, split K); the five benchmark shares are compared at full size on sampled output rows."""
import numpy as np
import pytest
import torch

import paper_2110_14883_amd as T
import synth_inputs as S
from oracle import tp_oracle as O
from paper_2110_14883_amd import workloads as WL

from gpu_util import check, compare, dev, f64, host64, overrides, run_share, say, workspace_for

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    T.lib()                       # fails loudly if the HIP library is not built


SMALL = [
    ("2d_q2", T.Grid(T.MODE_2D, q=2, ri=1, rj=0), (2 * 300, 2 * 136, 2 * 328)),
    ("2d_q3", T.Grid(T.MODE_2D, q=3, ri=2, rj=1), (3 * 70, 3 * 64, 3 * 264)),
    ("2p5d_q2_d2", T.Grid(T.MODE_2P5D, q=2, d=2, ri=1, rj=1, rk=1), (4 * 77, 2 * 72, 2 * 264)),
    ("3d_p2", T.Grid(T.MODE_3D, p=2, ri=1, rj=0, rk=1), (4 * 130, 2 * 200, 2 * 520)),
    ("1d_col_p3", T.Grid(T.MODE_1D_COL, p=3, ri=2), (270, 96, 3 * 264)),
]


@pytest.mark.parametrize("name,grid,dims", SMALL, ids=[s[0] for s in SMALL])
def test_small_share_elementwise(name, grid, dims):
    partial_dx = T.tp_block_map(grid, dims, T.PASS_DX)["partial"]       # a summand of a reduction: fp32 only
    run_share(grid, dims, y_dtype="bf16", dx_dtype="f32" if partial_dx else "bf16", want_db=True, label=name)
    run_share(grid, dims, y_dtype="f32", dx_dtype="f32", label=name + " fp32 outputs", seed=77)
    run_share(grid, dims, y_dtype="f32", dx_dtype="f32", use_own_slot=False, label=name + " ready-made dA", seed=78)


@pytest.mark.parametrize("tile", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("split", [1, 3])
def test_every_tile_shape_and_split(tile, split):
    grid, dims = T.Grid(T.MODE_2D, q=2, ri=0, rj=1), (2 * 300, 2 * 392, 2 * 328)
    with overrides(tile=tile, split=split, group=3):
        run_share(grid, dims, y_dtype="f32", dx_dtype="bf16", label=f"tile {tile} split {split}")


def test_k_rotation_and_other_group_heights():
    """The K-tile rotation and the tile-order group only change the order of work, never the result
    beyond fp32 summation order."""
    grid, dims = T.Grid(T.MODE_2D, q=2, ri=1, rj=1), (2 * 520, 2 * 1032, 2 * 776)
    for tile in (1, 2):          # the four-wave kernel (rotation off unless asked for) and the eight-wave one (on unless asked)
        for rotate in (0, 1):
            with overrides(tile=tile, rotate=rotate):
                run_share(grid, dims, y_dtype="f32", dx_dtype="f32", use_own_slot=False, label=f"tile {tile} rotation {'on' if rotate else 'off'}")
    for group in (1, 7):
        with overrides(group=group):
            run_share(grid, dims, backward=False, label=f"group height {group}")


def test_many_tiles_per_workgroup():
    """More tiles than workgroups (128 x 128 tiles forced: 324 per product on 256 persistent
    workgroups): all three memory forms, one-step and two-step shares, ragged edges."""
    with overrides(tile=4):
        run_share(T.Grid(T.MODE_2D, q=1), (2250, 2184, 2312), use_own_slot=False, label="324 tiles per product")
        run_share(T.Grid(T.MODE_2D, q=2, ri=1, rj=0), (2 * 2250, 2 * 520, 2 * 2312), backward=False, y_dtype="f32", label="two steps")


@pytest.mark.parametrize("name,grid,ogrid,dims", [
    ("2d_q2", T.Grid(T.MODE_2D, q=2, ri=1, rj=0), O.Grid(O.MODE_2D, q=2, ri=1, rj=0), (2 * 300, 2 * 136, 2 * 328)),
    ("3d_p2", T.Grid(T.MODE_3D, p=2, ri=1, rj=0, rk=1), O.Grid(O.MODE_3D, p=2, ri=1, rj=0, rk=1), (4 * 150, 2 * 136, 2 * 264)),
])
def test_chained_forward_then_backward_end_to_end(name, grid, ogrid, dims):
    """Forward on the GPU, then backward fed with the GPU's OWN saved pre-activation, its own dA block going
    straight into dX and dW (nothing in between comes from the oracle).  Every stage is held to its own
    tolerance against the oracle run on the SAME input bits the stage had: Y and A_saved from the inputs,
    dA from the GPU's A_saved (bf16 tolerance), dX and dW from the GPU's dA block (fp32 tolerance).  How
    far the results are from the oracle's unbroken fp64 chain is printed, not asserted: one dA element
    that rounds the other way in fp32 than in fp64 moves a dW element by |x| times a bf16 step, which a
    relative bound on a near-zero dW element cannot absorb (the derivative of rounding is a spike)."""
    inp = WL.make_share_inputs(grid, dims)
    m, n, k, S_ = inp["m"], inp["n"], inp["k"], inp["n_steps_fwd"]
    ws = workspace_for(grid, dims)
    y = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    pre = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    T.tp_linear_fwd(grid, dims, S_, [dev(b) for b in inp["x_blocks"]], [dev(b) for b in inp["w_blocks"]], dev(inp["bias"]),
                    T.EPI_BIAS_GELU, y, pre, ws)
    sx, sw = inp["n_steps_dx"], inp["n_steps_dw"]
    peer = lambda pair: dev(O.f64_to_bf16_bits(O.share_da(f64(pair[0]), f64(pair[1]))))
    rows = [None if i == inp["own_slot_dx"] else peer(inp["peers_dx"][i]) for i in range(sx)]
    cols = [None if i == inp["own_slot_dw"] else peer(inp["peers_dw"][i]) for i in range(sw)]
    dx = torch.empty((m, k), dtype=torch.float32, device="cuda")
    dw = torch.empty((inp["dw"]["m"], inp["dw"]["n"]), dtype=torch.float32, device="cuda")
    da = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    T.tp_linear_bwd(grid, dims, sx, sw, dy_own=dev(inp["g_own"]), preact_own=pre, da_row_blocks=rows,
                    w_blocks_dx=[dev(b) for b in inp["w_blocks_dx"]], x_blocks_dw=[dev(b) for b in inp["x_blocks_dw"]],
                    da_col_blocks=cols, own_slot_dx=inp["own_slot_dx"], own_slot_dw=inp["own_slot_dw"],
                    dx=dx, dw=dw, da_own_out=da, workspace=ws)
    torch.cuda.synchronize()
    w_dx64 = [f64(b) for b in inp["w_blocks_dx"]]
    x_dw64 = [f64(b) for b in inp["x_blocks_dw"]]
    peers_x = {i: O.share_da(f64(p[0]), f64(p[1])) for i, p in inp["peers_dx"].items()}
    peers_w = {i: O.share_da(f64(p[0]), f64(p[1])) for i, p in inp["peers_dw"].items()}
    # stage by stage, the oracle on the bits the stage was given
    A, Y = O.share_fwd([f64(b) for b in inp["x_blocks"]], [f64(b) for b in inp["w_blocks"]], f64(inp["bias"]))
    check(host64(y), Y, "bf16", f"{name}: Y")
    check(host64(pre), A, "bf16", f"{name}: A_saved")
    pre64, da64 = host64(pre), host64(da)
    check(da64, O.share_da(f64(inp["g_own"]), pre64), "bf16", f"{name}: dA from the GPU's own A_saved")
    blocks = lambda own, peers, cnt, slot: [own if i == slot else peers[i] for i in range(cnt)]
    check(host64(dx), O.share_dx(blocks(da64, peers_x, sx, inp["own_slot_dx"]), w_dx64), "f32", f"{name}: dX from the GPU's own dA")
    check(host64(dw), O.share_dw(x_dw64, blocks(da64, peers_w, sw, inp["own_slot_dw"])), "f32", f"{name}: dW from the GPU's own dA")
    # reported only: the oracle's unbroken chain
    dA_own = O.share_da(f64(inp["g_own"]), O.round_to_bf16(A))
    say(f"    {name}: {int((pre64 != O.round_to_bf16(A)).sum())} A_saved and {int((da64 != dA_own).sum())} dA elements of {da64.size} "
        f"differ from the unbroken chain's")
    compare(host64(dx), O.share_dx(blocks(dA_own, peers_x, sx, inp["own_slot_dx"]), w_dx64), "bf16", f"{name}: dX vs the unbroken chain (reported)")
    compare(host64(dw), O.share_dw(x_dw64, blocks(dA_own, peers_w, sw, inp["own_slot_dw"])), "bf16", f"{name}: dW vs the unbroken chain (reported)")


def test_calls_can_be_captured_in_a_hip_graph():
    """The library only enqueues kernels on the caller's stream (no allocation, no synchronisation,
    no memset), so a whole forward + backward of a share can be captured once and replayed: every
    replay, with eager work and synchronisations in between, reproduces the eager results bit for bit."""
    grid, dims = T.Grid(T.MODE_2D, q=2, ri=1, rj=0), (2 * 300, 2 * 136, 2 * 328)
    inp = WL.make_share_inputs(grid, dims)
    m, n, k = inp["m"], inp["n"], inp["k"]
    xs, ws_ = [dev(b) for b in inp["x_blocks"]], [dev(b) for b in inp["w_blocks"]]
    bias, g = dev(inp["bias"]), dev(inp["g_own"])
    wdx, xdw = [dev(b) for b in inp["w_blocks_dx"]], [dev(b) for b in inp["x_blocks_dw"]]
    peers_x = {i: dev(p[0]) for i, p in inp["peers_dx"].items()}
    peers_w = {i: dev(p[0]) for i, p in inp["peers_dw"].items()}
    ws = workspace_for(grid, dims)
    with overrides(split=2):            # include the split-K fix-up kernels in the captured work
        need = 8 * 4 * max(m * n, m * k, k * n)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        outs = [dict(y=torch.zeros((m, n), dtype=torch.bfloat16, device="cuda"), pre=torch.zeros((m, n), dtype=torch.bfloat16, device="cuda"),
                     da=torch.zeros((m, n), dtype=torch.bfloat16, device="cuda"), dx=torch.zeros((m, k), dtype=torch.float32, device="cuda"),
                     dw=torch.zeros((k, n), dtype=torch.float32, device="cuda"), db=torch.zeros((n,), dtype=torch.float32, device="cuda"))
                for _ in range(2)]

        def step(o):
            T.tp_linear_fwd(grid, dims, 2, xs, ws_, bias, T.EPI_BIAS_GELU, o["y"], o["pre"], ws)
            rows = [None if i == inp["own_slot_dx"] else peers_x[i] for i in range(2)]
            cols = [None if i == inp["own_slot_dw"] else peers_w[i] for i in range(2)]
            T.tp_linear_bwd(grid, dims, 2, 2, dy_own=g, preact_own=o["pre"], da_row_blocks=rows, w_blocks_dx=wdx,
                            x_blocks_dw=xdw, da_col_blocks=cols, own_slot_dx=inp["own_slot_dx"], own_slot_dw=inp["own_slot_dw"],
                            dx=o["dx"], dw=o["dw"], da_own_out=o["da"], db=o["db"], workspace=ws)

        step(outs[0])                   # eager reference
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step(outs[1])               # warm-up on the capture stream
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step(outs[1])
        torch.cuda.synchronize()
        for replay in range(3):
            for t in outs[1].values():
                t.fill_(7.0)            # eager work between replays; also proves the replay rewrites everything
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for name in outs[0]:
                assert torch.equal(outs[0][name], outs[1][name]), (replay, name)


@pytest.mark.parametrize("trim", [1, 0])
def test_tail_rows_as_a_second_launch(trim):
    """272 tiles of 128 x 128 on 256 workgroups: with trimming the last tile row (ragged) runs as a
    launch of its own through shifted pointers -- forward with both outputs and dX (first case), dW
    (second case), the 1D chain's GeLU' epilogue (third); same results with trimming off."""
    with overrides(tile=4, trim=trim):
        run_share(T.Grid(T.MODE_2D, q=1), (2139, 2048, 2048), use_own_slot=False, want_db=True, label=f"fwd and dX trimmed ({trim})")
        run_share(T.Grid(T.MODE_2D, q=2, ri=0, rj=1), (2 * 1000, 2 * 2136, 2 * 2048), y_dtype="f32", label=f"dW trimmed, two steps ({trim})")
        _mlp1d(2, 1, 2139, 2048, 2 * 2048, rows=None)


def test_seeded_random_shapes_and_grids():
    """Forty seeded draws of (mode, grid, rank, ragged extents, output dtypes, plan overrides): every
    element of forward and backward against the oracle.  Extents span one to a few tiles with odd tails."""
    rng = np.random.default_rng(20211014)
    for case in range(40):
        mode = [T.MODE_1D_COL, T.MODE_1D_ROW, T.MODE_2D, T.MODE_2P5D, T.MODE_3D][case % 5]
        q, d, p = 1, 1, 1
        if mode in (T.MODE_1D_COL, T.MODE_1D_ROW):
            p = int(rng.integers(1, 5)); rank = (int(rng.integers(0, p)), 0, 0); rc, kc, cc = (1, 1, p) if mode == T.MODE_1D_COL else (1, p, 1)
        elif mode == T.MODE_2D:
            q = int(rng.integers(1, 4)); rank = (int(rng.integers(0, q)), int(rng.integers(0, q)), 0); rc = kc = cc = q
        elif mode == T.MODE_2P5D:
            q, d = int(rng.integers(1, 3)), int(rng.integers(1, 4))
            rank = (int(rng.integers(0, q)), int(rng.integers(0, q)), int(rng.integers(0, d))); rc, kc, cc = q * d, q, q
        else:
            p = int(rng.integers(1, 3)); rank = tuple(int(rng.integers(0, p)) for _ in range(3)); rc, kc, cc = p * p, p, p
        mb = int(rng.integers(1, 420))                       # local rows: any value
        hb = 8 * int(rng.integers(1, 50))                    # local column extents: multiples of 8
        fb = 8 * int(rng.integers(1, 50))
        grid = T.Grid(mode, q=q, d=d, p=p, ri=rank[0], rj=rank[1], rk=rank[2])
        dims = (mb * rc, hb * kc, fb * cc)
        kw = dict(y_dtype=["bf16", "f32"][int(rng.integers(0, 2))], dx_dtype=["bf16", "f32"][int(rng.integers(0, 2))],
                  want_db=bool(rng.integers(0, 2)), use_own_slot=bool(rng.integers(0, 2)))
        if mode == T.MODE_1D_ROW:
            kw.update(epi=T.EPI_NONE, backward=False, y_dtype="f32")      # the row-cut product is a partial sum: no epilogue
        if mode == T.MODE_1D_COL and p > 1:
            kw.update(dx_dtype="f32")                                     # dX is a partial sum over the ranks: fp32 only
        with overrides(tile=int(rng.integers(0, 6)), split=int(rng.integers(0, 4))):
            run_share(grid, dims, label=f"draw {case}", **kw)


def test_prefix_of_steps_and_bias_only():
    grid, dims = T.Grid(T.MODE_3D, p=2, ri=1, rj=1, rk=0), (4 * 96, 2 * 128, 2 * 256)
    run_share(grid, dims, n_steps=1, label="3d literal single step")
    run_share(grid, dims, epi=T.EPI_BIAS, backward=False, y_dtype="f32", label="bias only")
    run_share(grid, dims, epi=T.EPI_NONE, backward=False, y_dtype="f32", label="no epilogue")


def test_degenerate_extents():
    # one row, one 8-wide column block, K of one chunk
    run_share(T.Grid(T.MODE_2D, q=1), (1, 8, 8), y_dtype="f32", dx_dtype="f32", label="1x8x8")
    run_share(T.Grid(T.MODE_2D, q=2, ri=1, rj=1), (2, 16, 16), label="q2 of 2x16x16")
    run_share(T.Grid(T.MODE_1D_COL, p=1), (257, 72, 8), y_dtype="f32", label="257x72x8")


def test_largest_leading_dimension_and_many_rows():
    """Blocks that are narrow views of very wide arrays (ld = 2^21 elements, the largest the library
    takes: every in-tile byte offset still fits 31 bits) and a share with millions of ragged rows."""
    m, k, n = 300, 136, 72
    ld = 1 << 21
    x_bits = S.normal_block_bf16(21, S.T_X, k, 0, m, 0, k, 1.0)
    w_bits = S.normal_block_bf16(21, S.T_W1, n, 0, k, 0, n, 0.02)
    g_bits = S.normal_block_bf16(21, S.T_G, n, 0, m, 0, n, 1.0)
    wide_x = torch.zeros((m, ld), dtype=torch.bfloat16, device="cuda")
    wide_g = torch.zeros((m, ld), dtype=torch.bfloat16, device="cuda")
    wide_y = torch.zeros((m, ld), dtype=torch.float32, device="cuda")
    xv, gv, yv = wide_x[:, ld - k:], wide_g[:, 8:8 + n], wide_y[:, ld - n:]
    xv.copy_(dev(x_bits)); gv.copy_(dev(g_bits))
    w = dev(w_bits)
    grid, dims = T.Grid(T.MODE_2D, q=1), (m, k, n)
    T.tp_linear_fwd(grid, dims, 1, [xv], [w], None, T.EPI_NONE, yv, None, None)
    dx = torch.empty((m, k), dtype=torch.float32, device="cuda")
    dw = torch.empty((k, n), dtype=torch.float32, device="cuda")
    T.tp_linear_bwd(grid, dims, 1, 1, da_row_blocks=[gv], w_blocks_dx=[w], x_blocks_dw=[xv], da_col_blocks=[gv], dx=dx, dw=dw)
    torch.cuda.synchronize()
    x64, w64, g64 = f64(x_bits), f64(w_bits), f64(g_bits)
    check(host64(yv), x64 @ w64, "f32", "Y through ld = 2^21 views")
    check(host64(dx), O.share_dx([g64], [w64]), "f32", "dX, dA read through an ld = 2^21 view")
    check(host64(dw), O.share_dw([x64], [g64]), "f32", "dW, both operands through ld = 2^21 views")
    assert float(wide_y[:, :ld - n].abs().max()) == 0.0
    del wide_x, wide_g, wide_y
    with pytest.raises(T.TpError) as e:
        T.tp_linear_fwd(grid, dims, 1, [(xv.data_ptr(), 2 * ld)], [w], None, T.EPI_NONE, yv, None, None)
    assert e.value.status == 4
    # 3,000,003 token rows (11,719 tile rows, the last with 3 rows), narrow layer
    run_share(T.Grid(T.MODE_1D_COL, p=1), (3_000_003, 8, 16), y_dtype="f32", dx_dtype="f32", label="3M ragged rows")


def test_gelu_tails_and_strided_blocks():
    """Pre-activations far in both tails, and blocks that are views with ld > cols."""
    m, n = 64, 256
    a = np.linspace(-12.0, 12.0, m * n).reshape(m, n)
    a_bits = O.f64_to_bf16_bits(O.round_to_bf16(a))
    g_bits = S.normal_block_bf16(5, S.T_G, n, 0, m, 0, n, 1.0)
    big_a = torch.zeros((m, n + 64), dtype=torch.bfloat16, device="cuda")
    big_g = torch.zeros((m, n + 32), dtype=torch.bfloat16, device="cuda")
    big_o = torch.zeros((m, n + 8), dtype=torch.bfloat16, device="cuda")
    big_a[:, :n] = dev(a_bits)
    big_g[:, 32:] = dev(g_bits)
    T.tp_dgelu(big_g[:, 32:], big_a[:, :n], big_o[:, 8:])
    torch.cuda.synchronize()
    check(host64(big_o[:, 8:]), O.share_da(f64(g_bits), f64(a_bits)), "bf16", "dgelu over [-12, 12]")
    assert float(big_o[:, :8].abs().max()) == 0.0
    # forward with X = a (K = n), W = I block: Y = GeLU(a + b)
    eye = torch.eye(n, dtype=torch.bfloat16, device="cuda")
    bias = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    y = torch.empty((m, n), dtype=torch.float32, device="cuda")
    T.tp_linear_fwd(T.Grid(T.MODE_2D, q=1), (m, n, n), 1, [big_a[:, :n]], [eye], bias, T.EPI_BIAS_GELU, y, None, None)
    torch.cuda.synchronize()
    check(host64(y), O.gelu(f64(a_bits)), "f32", "GeLU over [-12, 12]")
    neg = f64(a_bits) < -3
    ref = O.gelu(f64(a_bits))[neg]
    ok = np.abs(ref) > 1e-30
    rel = np.abs(host64(y)[neg][ok] - ref[ok]) / np.abs(ref[ok])
    say(f"    negative-tail relative error of GeLU (fp32 out, a in [-12, -3]): max {rel.max():.3g}")


def test_mlp1d_chain_small():
    _mlp1d(2, 1, 200, 136, 2 * 264, rows=None)
    _mlp1d(3, 0, 520, 264, 3 * 72, rows=None)
    with overrides(split=2):            # the GeLU' epilogue through the split-K fix-up kernel
        _mlp1d(2, 0, 300, 264, 2 * 136, rows=None)


def _mlp1d(size, rank, M, H, F, rows=None, w_rows=None):
    """Every product of the chain is fed the oracle's (bf16-rounded) intermediate, so stage errors do
    not compound and the fp32 outputs are held to the fp32 tolerance."""
    say(f"[case] 1D chain size={size} rank={rank} M={M} H={H} F={F}")
    inp = WL.make_mlp1d_inputs(size, rank, M, H, F)
    fb = inp["fb"]
    g1, d1 = T.Grid(T.MODE_1D_COL, p=size, ri=rank), (M, H, F)
    g2, d2 = T.Grid(T.MODE_1D_ROW, p=size, ri=rank), (M, F, H)
    X, W1, b1, W2, G = (dev(inp[k]) for k in ("X", "W1", "b1", "W2", "G"))
    X64, W164, b164, W264, G64 = (f64(inp[k]) for k in ("X", "W1", "b1", "W2", "G"))
    ws = workspace_for(g1, d1)
    ws2 = workspace_for(g2, d2)
    sel = slice(None) if rows is None else rows
    wsel = slice(None) if w_rows is None else w_rows
    fw = O.mlp1d_fwd(X64, W164, b164, W264)            # full: backward needs every row of A_saved and Z
    Z = torch.empty((M, fb), dtype=torch.bfloat16, device="cuda")
    A = torch.empty((M, fb), dtype=torch.bfloat16, device="cuda")
    Y = torch.empty((M, H), dtype=torch.float32, device="cuda")
    say("  fc1 fwd")
    T.tp_linear_fwd(g1, d1, 1, [X], [W1], b1, T.EPI_BIAS_GELU, Z, A, ws)
    torch.cuda.synchronize()
    check(host64(Z[sel]), fw["Z"][sel], "bf16", "Z")
    check(host64(A[sel]), fw["A_saved"][sel], "bf16", "A_saved")
    Z_in = dev(O.f64_to_bf16_bits(fw["Z"]))
    A_in = dev(O.f64_to_bf16_bits(fw["A_saved"]))
    say("  fc2 fwd")
    T.tp_linear_fwd(g2, d2, 1, [Z_in], [W2], None, T.EPI_NONE, Y, None, ws2)
    torch.cuda.synchronize()
    check(host64(Y[sel]), fw["Y"][sel], "f32", "Y partial")
    bw = O.mlp1d_bwd(X64, W164, W264, fw["A_saved"], fw["Z"], G64, rows=rows, w_rows=w_rows)
    dA = torch.empty((M, fb), dtype=torch.bfloat16, device="cuda")
    dW2 = torch.empty((fb, H), dtype=torch.float32, device="cuda")
    say("  fc2 bwd (dZ with GeLU' epilogue, dW2)")
    T.tp_linear_bwd(g2, d2, 1, 1, da_row_blocks=[G], w_blocks_dx=[W2], x_blocks_dw=[Z_in], da_col_blocks=[G],
                    dgelu_preact=A_in, dx=dA, dw=dW2, workspace=ws2)
    torch.cuda.synchronize()
    check(host64(dA[sel]), bw["dA"], "bf16", "dA")
    check(host64(dW2[wsel]), bw["dW2"], "f32", "dW2")
    full = O.mlp1d_bwd(X64, W164, W264, fw["A_saved"], fw["Z"], G64)["dA"] if rows is not None else bw["dA"]
    dA_in = dev(O.f64_to_bf16_bits(full))
    dX = torch.empty((M, H), dtype=torch.float32, device="cuda")
    dW1 = torch.empty((H, fb), dtype=torch.float32, device="cuda")
    say("  fc1 bwd (dX partial, dW1)")
    T.tp_linear_bwd(g1, d1, 1, 1, da_row_blocks=[dA_in], w_blocks_dx=[W1], x_blocks_dw=[X], da_col_blocks=[dA_in],
                    dx=dX, dw=dW1, workspace=ws)
    torch.cuda.synchronize()
    check(host64(dX[sel]), bw["dX"], "f32", "dX partial")
    check(host64(dW1[wsel]), bw["dW1"], "f32", "dW1")


# ----------------------------------------------------------------------------- the second linear of an MLP, and projections
CHAIN = [
    ("2d_q2", T.Grid(T.MODE_2D, q=2, ri=1, rj=0), O.Grid(O.MODE_2D, q=2, ri=1, rj=0), (2 * 264, 2 * 136, 2 * 392)),
    ("2p5d_q2_d2", T.Grid(T.MODE_2P5D, q=2, d=2, ri=0, rj=1, rk=1), O.Grid(O.MODE_2P5D, q=2, d=2, ri=0, rj=1, rk=1), (4 * 72, 2 * 72, 2 * 264)),
    ("3d_p2", T.Grid(T.MODE_3D, p=2, ri=1, rj=1, rk=0), O.Grid(O.MODE_3D, p=2, ri=1, rj=1, rk=0), (4 * 130, 2 * 72, 2 * 328)),
]


@pytest.mark.parametrize("name,grid,ogrid,dims", CHAIN, ids=[c[0] for c in CHAIN])
def test_second_linear_with_fused_dgelu(name, grid, ogrid, dims):
    """The down-projection of an MLP through the same entry points: forward with a bias-only epilogue,
    backward dX with GeLU'(A1) fused as its epilogue (no separate elementwise pass) and dW2."""
    M, H, F = dims                       # layer 1: H -> F;  layer 2: F -> H
    say(f"[case] MLP second linear {name} M={M} H={H} F={F}")
    d2 = (M, F, H)
    seed = 4242
    X = f64(S.normal_block_bf16(seed, S.T_X, H, 0, M, 0, H, 1.0))
    W1 = f64(S.normal_block_bf16(seed, S.T_W1, F, 0, H, 0, F, 0.05))
    b1 = f64(S.normal_block_bf16(seed, S.T_B1, F, 0, 1, 0, F, 0.05)[0])
    W2b = S.normal_block_bf16(seed, S.T_W2, H, 0, F, 0, H, 0.05)
    b2b = S.normal_block_bf16(seed, S.T_B1 + 20, H, 0, 1, 0, H, 0.05)[0]
    G2b = S.normal_block_bf16(seed, S.T_G, H, 0, M, 0, H, 1.0)
    W2, b2, G2 = f64(W2b), f64(b2b), f64(G2b)
    A1, Zf = O.layer_fwd(X, W1, b1)                    # layer 1, unpartitioned, with its rounding points
    A1s, Z = O.round_to_bf16(A1), O.round_to_bf16(Zf)
    rc, kc, cc = O.chunk_counts(ogrid)                 # layer 2 chunk grid: Z [rc x kc], W2 [kc x cc]
    fm, xm, wm_ = (T.tp_block_map(grid, d2, p_) for p_ in (0, 1, 2))
    up = lambda a: dev(O.f64_to_bf16_bits(a))
    ws = workspace_for(grid, d2)
    # forward: Y2 = Z W2 + b2 (fp32 out)
    y2 = torch.empty((fm["m"], fm["n"]), dtype=torch.float32, device="cuda")
    T.tp_linear_fwd(grid, d2, fm["n_steps"], [up(O.chunk(Z, rc, kc, *a)) for a in fm["a"]],
                    [up(O.chunk(W2, kc, cc, *b)) for b in fm["b"]], up(O.chunk(b2, 1, cc, 0, fm["out"][1])),
                    T.EPI_BIAS, y2, None, ws)
    torch.cuda.synchronize()
    check(host64(y2), O.rank_fwd(ogrid, Z, W2, b2, act=False)[1], "f32", "Y2")
    # backward: dA1 = bf16((sum_k dY2 W2^T) * GeLU'(A1_saved)) as the dX epilogue;  dW2 = sum_k Z^T dY2
    own_a1 = O.chunk(A1s, rc, kc, *xm["out"])
    da1 = torch.empty((xm["m"], xm["n"]), dtype=torch.bfloat16, device="cuda")
    dw2 = torch.empty((wm_["m"], wm_["n"]), dtype=torch.float32, device="cuda")
    T.tp_linear_bwd(grid, d2, xm["n_steps"], wm_["n_steps"],
                    da_row_blocks=[up(O.chunk(G2, rc, cc, *a)) for a in xm["a"]],
                    w_blocks_dx=[up(O.chunk(W2, kc, cc, *b)) for b in xm["b"]],
                    x_blocks_dw=[up(O.chunk(Z, rc, kc, *a)) for a in wm_["a"]],
                    da_col_blocks=[up(O.chunk(G2, rc, cc, *b)) for b in wm_["b"]],
                    dgelu_preact=up(own_a1), dx=da1, dw=dw2, workspace=ws)
    torch.cuda.synchronize()
    dZ = O.rank_dx(ogrid, G2, W2)
    check(host64(da1), O.round_to_bf16(dZ * O.dgelu(own_a1)), "bf16", "dA1 (dX with GeLU' epilogue)")
    check(host64(dw2), O.rank_dw(ogrid, Z, G2), "f32", "dW2")


def test_attention_projection_shapes():
    """QKV (H -> 3H) and output projection (H -> H) shares: bias-only forward, backward without activation."""
    for label, grid, dims in (("qkv 2d q2", T.Grid(T.MODE_2D, q=2, ri=0, rj=1), (2 * 200, 2 * 128, 2 * 384)),
                              ("out-proj 3d p2", T.Grid(T.MODE_3D, p=2, ri=0, rj=1, rk=1), (4 * 100, 2 * 128, 2 * 128))):
        run_share(grid, dims, epi=T.EPI_BIAS, backward=False, y_dtype="bf16", label=label + " fwd")
        run_linear_backward(grid, dims, label=label + " bwd")


def run_linear_backward(grid, dims, label=""):
    """Backward of a layer without activation: the upstream gradient blocks are the 'dA' blocks."""
    say(f"[case] {label} grid={grid} dims={dims}")
    inp = WL.make_share_inputs(grid, dims, 99, None, True)
    sx, sw = inp["n_steps_dx"], inp["n_steps_dw"]
    gx = {inp["own_slot_dx"]: inp["g_own"], **{i: g for i, (g, a) in inp["peers_dx"].items()}}
    gw = {inp["own_slot_dw"]: inp["g_own"], **{i: g for i, (g, a) in inp["peers_dw"].items()}}
    mx, mw = T.tp_block_map(grid, dims, T.PASS_DX), T.tp_block_map(grid, dims, T.PASS_DW)
    dx = torch.empty((mx["m"], mx["n"]), dtype=torch.bfloat16, device="cuda")
    dw = torch.empty((mw["m"], mw["n"]), dtype=torch.float32, device="cuda")
    T.tp_linear_bwd(grid, dims, sx, sw, da_row_blocks=[dev(gx[i]) for i in range(sx)],
                    w_blocks_dx=[dev(b) for b in inp["w_blocks_dx"]], x_blocks_dw=[dev(b) for b in inp["x_blocks_dw"]],
                    da_col_blocks=[dev(gw[i]) for i in range(sw)], dx=dx, dw=dw, workspace=workspace_for(grid, dims))
    torch.cuda.synchronize()
    check(host64(dx), O.share_dx([f64(gx[i]) for i in range(sx)], [f64(b) for b in inp["w_blocks_dx"]]), "bf16", "dX")
    check(host64(dw), O.share_dw([f64(b) for b in inp["x_blocks_dw"]], [f64(gw[i]) for i in range(sw)]), "f32", "dW")


# ----------------------------------------------------------------------------- backward as partials for other owners
def _ws_bytes(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def _partials(grid, dims, rows=None, w_rows=None, ws_bytes=None, label=""):
    """tp_linear_bwd_partials against the oracle's single-step products of the same blocks."""
    say(f"[case] partials {label} grid={grid} dims={dims} rows={'all' if rows is None else len(rows)}")
    inp = WL.make_partials_inputs(grid, dims)
    m, h, f = inp["m"], inp["h"], inp["f"]
    q = inp["dx"]["n_steps"]
    assert inp["dw"]["n_steps"] == q and len(inp["w_blocks"]) == q and len(inp["x_blocks"]) == q
    da = dev(inp["da_own"])
    w_d = [dev(b) for b in inp["w_blocks"]]
    x_d = [dev(b) for b in inp["x_blocks"]]
    dxp = [torch.full((m, h), float("nan"), dtype=torch.float32, device="cuda") for _ in range(q)]
    dwp = [torch.full((h, f), float("nan"), dtype=torch.float32, device="cuda") for _ in range(q)]
    if ws_bytes is None:
        ws_bytes = max(T.tp_linear_workspace_size(grid, dims, ps) for ps in (T.PASS_DX_PARTIALS, T.PASS_DW_PARTIALS))
    say("  launching")
    T.tp_linear_bwd_partials(grid, dims, da, w_d, dxp, x_d, dwp, _ws_bytes(ws_bytes))
    torch.cuda.synchronize()
    da64 = f64(inp["da_own"])
    sel = slice(None) if rows is None else rows
    wsel = slice(None) if w_rows is None else w_rows
    for k in range(q):
        check(host64(dxp[k][sel]), O.share_dx([da64], [f64(inp["w_blocks"][k])], rows), "f32",
              f"dX partial {k} for owner {inp['dx']['out'][k]}")
        check(host64(dwp[k][wsel]), O.share_dw([f64(inp["x_blocks"][k])], [da64], w_rows), "f32",
              f"dW partial {k} for owner {inp['dw']['out'][k]}")


def test_bwd_partials_small():
    _partials(T.Grid(T.MODE_2D, q=2, ri=1, rj=0), (2 * 300, 2 * 136, 2 * 328), label="2d q2")
    _partials(T.Grid(T.MODE_2D, q=3, ri=2, rj=1), (3 * 264, 3 * 72, 3 * 200), label="2d q3")
    _partials(T.Grid(T.MODE_2P5D, q=2, d=2, ri=0, rj=1, rk=1), (4 * 130, 2 * 264, 2 * 136), label="2.5d q2 d2")
    _partials(T.Grid(T.MODE_2D, q=1), (257, 72, 8), label="q1: one product")


@pytest.mark.parametrize("tile,split", [(1, 2), (2, 1), (3, 3), (4, 1), (4, 2), (5, 2)])
def test_bwd_partials_tiles_and_split(tile, split):
    grid, dims = T.Grid(T.MODE_2D, q=3, ri=0, rj=2), (3 * 392, 3 * 264, 3 * 520)
    mx = T.tp_partials_map(grid, dims, T.PASS_DX_PARTIALS)
    mw = T.tp_partials_map(grid, dims, T.PASS_DW_PARTIALS)
    room = 8 * 3 * 4 * max(mx["m"] * mx["n"], mw["m"] * mw["n"])
    with overrides(tile=tile, split=split):
        _partials(grid, dims, ws_bytes=room, label=f"tile {tile} split {split}")


def test_bwd_partials_single_pass_and_prefix():
    """Only dX, only dW, and fewer products than the map has."""
    grid, dims = T.Grid(T.MODE_2D, q=2, ri=0, rj=1), (2 * 200, 2 * 136, 2 * 264)
    inp = WL.make_partials_inputs(grid, dims)
    m, h, f = inp["m"], inp["h"], inp["f"]
    da, da64 = dev(inp["da_own"]), f64(inp["da_own"])
    ws = _ws_bytes(8 * 2 * 4 * max(m * h, h * f))
    dxp = [torch.full((m, h), float("nan"), dtype=torch.float32, device="cuda")]
    T.tp_linear_bwd_partials(grid, dims, da, [dev(inp["w_blocks"][1])], dxp, None, None, ws)
    dwp = [torch.full((h, f), float("nan"), dtype=torch.float32, device="cuda") for _ in range(2)]
    T.tp_linear_bwd_partials(grid, dims, da, None, None, [dev(b) for b in inp["x_blocks"]], dwp, ws)
    torch.cuda.synchronize()
    check(host64(dxp[0]), O.share_dx([da64], [f64(inp["w_blocks"][1])]), "f32", "dX partial alone")
    for k in range(2):
        check(host64(dwp[k]), O.share_dw([f64(inp["x_blocks"][k])], [da64]), "f32", f"dW partial {k} alone")


# ----------------------------------------------------------------------------- 3D at its gathered local shape
def _gathered3d(grid, dims, rows=None, w_rows=None, label=""):
    say(f"[case] 3d gathered {label} grid={grid} dims={dims} rows={'all' if rows is None else len(rows)}")
    inp = WL.make_gathered3d_inputs(grid, dims)
    ms, hb, fb = inp["m"], inp["h"], inp["f"]
    x, w, da = dev(inp["x"]), dev(inp["w"]), dev(inp["da"])
    x64, w64, da64 = f64(inp["x"]), f64(inp["w"]), f64(inp["da"])
    ws = workspace_for(grid, dims)
    sel = slice(None) if rows is None else rows
    wsel = slice(None) if w_rows is None else w_rows
    y = torch.full((ms, fb), float("nan"), dtype=torch.float32, device="cuda")
    dx = torch.full((ms, hb), float("nan"), dtype=torch.float32, device="cuda")
    dw = torch.full((hb, fb), float("nan"), dtype=torch.float32, device="cuda")
    say("  launching")
    T.tp_linear_fwd(grid, dims, 1, [x], [w], None, T.EPI_NONE, y, None, ws)
    T.tp_linear_bwd(grid, dims, 1, 1, da_row_blocks=[da], w_blocks_dx=[w], x_blocks_dw=[x], da_col_blocks=[da],
                    dx=dx, dw=dw, workspace=ws)
    torch.cuda.synchronize()
    C, _ = O.share_fwd([x64], [w64], None, False, rows)
    check(host64(y[sel]), C, "f32", "forward partial")
    check(host64(dx[sel]), O.share_dx([da64], [w64], rows), "f32", "dX partial")
    check(host64(dw[wsel]), O.share_dw([x64], [da64], w_rows), "f32", "dW partial")
    # the rank's chunk of the (here: single-term) summed slab, then bias and GeLU
    p, l = grid.p, grid.rk
    mc = ms // p
    mine = y[l * mc:(l + 1) * mc]
    yb = torch.empty((mc, fb), dtype=torch.bfloat16, device="cuda")
    pre = torch.empty((mc, fb), dtype=torch.bfloat16, device="cuda")
    T.tp_bias_act(mine, dev(inp["bias"]), T.EPI_BIAS_GELU, yb, pre)
    torch.cuda.synchronize()
    if rows is None:
        A, Y = O.bias_gelu(C[l * mc:(l + 1) * mc], f64(inp["bias"]))
        check(host64(yb), Y, "bf16", "Y chunk after bias + GeLU")
        check(host64(pre), A, "bf16", "A_saved chunk")


def test_3d_gathered_small():
    _gathered3d(T.Grid(T.MODE_3D_GATHERED, p=2, ri=1, rj=0, rk=1), (4 * 150, 2 * 136, 2 * 264), label="p2")
    _gathered3d(T.Grid(T.MODE_3D_GATHERED, p=3, ri=2, rj=1, rk=0), (9 * 40, 3 * 72, 3 * 200), label="p3")
    _gathered3d(T.Grid(T.MODE_3D_GATHERED, p=1), (130, 72, 8), label="p1")


def test_bias_act_alone():
    """fp32 input with full mantissas, every epilogue kind, both output dtypes, strided views."""
    rows, cols = 70, 264
    a = f64(S.normal_block_bf16(11, S.T_X, cols, 0, rows, 0, cols, 3.0)).astype(np.float32)
    b = f64(S.normal_block_bf16(12, S.T_X, cols, 0, rows, 0, cols, 1.0)).astype(np.float32)
    c32 = (a + b * np.float32(2.0 ** -9)).astype(np.float32)
    bias_bits = S.normal_block_bf16(13, S.T_B1, cols, 0, 1, 0, cols, 0.5)[0]
    big = torch.zeros((rows, cols + 24), dtype=torch.float32, device="cuda")
    big[:, 8:8 + cols] = torch.from_numpy(c32).cuda()
    c_d = big[:, 8:8 + cols]
    c64 = c32.astype(np.float64)
    for epi, act, use_b in ((T.EPI_BIAS_GELU, True, True), (T.EPI_BIAS, False, True), (T.EPI_NONE, False, False)):
        A, Y = O.bias_gelu(c64, f64(bias_bits) if use_b else None, act)
        for dt, kind in ((torch.float32, "f32"), (torch.bfloat16, "bf16")):
            y = torch.zeros((rows, cols + 16), dtype=dt, device="cuda")
            pre = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda")
            T.tp_bias_act(c_d, dev(bias_bits) if use_b else None, epi, y[:, :cols], pre)
            torch.cuda.synchronize()
            check(host64(y[:, :cols]), Y, kind, f"bias_act epi {epi} {kind}")
            check(host64(pre), A, "bf16", f"bias_act epi {epi} saved pre-activation")
            assert float(y[:, cols:].abs().max()) == 0.0


def test_bias_grad_slab_form_and_single_pass():
    """db = 1^T dA on a tall, narrow block (config 4's shape class: many rows, few column blocks): the slab
    form (row splits + ordered second pass, given a workspace) and the single-pass form, each against
    the oracle's column sums and each bit-reproducible."""
    for rows, cols, ld in ((32896, 2560, 2560), (5000, 136, 200), (300, 64, 64), (257, 8, 8)):
        bits = S.normal_block_bf16(S.BASE_SEED + 5, S.T_G, ld, 0, rows, 0, ld, 1.0)
        da = dev(bits)
        ref = f64(bits)[:, :cols].sum(axis=0)
        need = T.tp_bias_grad_workspace_size(rows, cols)
        say(f"[case] bias grad {rows} x {cols} (ld {ld}): slab workspace {need} bytes")
        outs = []
        for ws in (torch.empty(max(need, 16), dtype=torch.uint8, device="cuda"), None):
            for rep in range(2):
                db = torch.full((cols,), float("nan"), dtype=torch.float32, device="cuda")
                T.tp_bias_grad(da, db, rows, cols, workspace=ws)
                torch.cuda.synchronize()
                outs.append(db)
            check(host64(outs[-1]), ref, "f32", f"db {'slab form' if ws is not None else 'single pass'}")
            assert torch.equal(outs[-1], outs[-2]), "bias gradient is not reproducible"


# ----------------------------------------------------------------------------- the two-layer chain of the range test
@pytest.mark.parametrize("name,grid,M,h", [
    ("1d_p4", T.Grid(T.MODE_1D_COL, p=4, ri=1), 520, 4 * 136),
    ("2d_q2", T.Grid(T.MODE_2D, q=2, ri=1, rj=0), 2 * 300, 2 * 264),
    ("2p5d_q2_d2", T.Grid(T.MODE_2P5D, q=2, d=2, ri=1, rj=0, rk=1), 4 * 150, 2 * 264),
    ("3d_p2", T.Grid(T.MODE_3D, p=2, ri=1, rj=0, rk=1), 4 * 130, 2 * 328),
], ids=["1d_p4", "2d_q2", "2p5d_q2_d2", "3d_p2"])
def test_range_test_two_layer_chain(name, grid, M, h):
    """The call chain of the range test (two linear layers, forward and backward, the rank's own
    intermediate blocks handed from call to call) at one small point per scheme: every output against
    the oracle run on the bits the producing call was given."""
    from paper_2110_14883_amd import range_test as R
    gen = torch.Generator(device="cuda")
    gen.manual_seed(14883 + M + h)
    calls, _, b = R.build_share(grid, M, h, gen)
    for fn in calls:
        fn()
    torch.cuda.synchronize()
    h64 = host64
    if grid.mode == T.MODE_1D_COL:
        A, Z = O.share_fwd([h64(b["X"])], [h64(b["W1"])], h64(b["b1"]))
        check(h64(b["A1"]), A, "bf16", f"{name}: A1 saved"); check(h64(b["Z"]), Z, "bf16", f"{name}: Z")
        _, Y = O.share_fwd([h64(b["Z"])], [h64(b["W2"])], None, act=False)
        check(h64(b["Y"]), Y, "f32", f"{name}: Y partial")
        dA1 = O.round_to_bf16(O.share_dx([h64(b["G"])], [h64(b["W2"])]) * O.dgelu(h64(b["A1"])))
        check(h64(b["dA1"]), dA1, "bf16", f"{name}: dA1")
        check(h64(b["dW2"]), O.share_dw([h64(b["Z"])], [h64(b["G"])]), "f32", f"{name}: dW2")
        check(h64(b["dX"]), O.share_dx([h64(b["dA1"])], [h64(b["W1"])]), "f32", f"{name}: dX partial")
        check(h64(b["dW1"]), O.share_dw([h64(b["X"])], [h64(b["dA1"])]), "f32", f"{name}: dW1")
        return
    L = lambda key: [h64(t) for t in b[key]]
    A, Z = O.share_fwd(L("x1"), L("w1"), h64(b["b1"]))
    check(h64(b["A1"]), A, "bf16", f"{name}: A1 saved"); check(h64(b["Z"]), Z, "bf16", f"{name}: Z")
    assert any(b["own_fwd"]) == any(t is b["Z"] for t in b["z2"])
    _, Y = O.share_fwd(L("z2"), L("w2"), h64(b["b2"]), act=False)          # (z2 holds the GPU's own Z block where the map says so)
    check(h64(b["Y"]), Y, "bf16", f"{name}: Y")
    dA1 = O.round_to_bf16(O.share_dx(L("g_row"), L("w2x")) * O.dgelu(h64(b["A1"])))
    check(h64(b["dA1"]), dA1, "bf16", f"{name}: dA1")
    check(h64(b["dW2"]), O.share_dw(L("z_col"), L("g_col")), "f32", f"{name}: dW2")
    check(h64(b["dX"]), O.share_dx(L("da_row"), L("w1x")), "bf16", f"{name}: dX")
    check(h64(b["dW1"]), O.share_dw(L("x_col"), L("da_col")), "f32", f"{name}: dW1")


# ----------------------------------------------------------------------------- the benchmark shares at full size
def test_config1_full():
    c = WL.config("c1_2d_q2_fwd")
    run_share(c.grid, c.dims, y_dtype="f32", backward=False, label=c.name)


@pytest.mark.parametrize("name", ["c3_2d_q4", "c4_2p5d_q2_d2", "c5_3d_p2"])
def test_config_full_size_every_element(name):
    """The benchmark shares at full size, every output element against the fp64 oracle (which needs a few
    seconds of BLAS per share on the host); the saved pre-activation is the oracle's own forward result."""
    c = WL.config(name)
    run_share(c.grid, c.dims, n_steps=c.n_steps, label=name)


def test_config5_exact_full_size_sampled():
    """Both steps of config 5's exact share (twice the work of c5_3d_p2): sampled rows."""
    c = WL.config("c5x_3d_p2_exact")
    mp = T.tp_block_map(c.grid, c.dims, 0)
    rows = S.sample_rows(3, mp["m"], 192)
    w_rows = S.sample_rows(4, mp["k"], 96)
    run_share(c.grid, c.dims, n_steps=c.n_steps, rows=rows, w_rows=w_rows, synthetic_preact=True, label=c.name)


def test_config2_full_size_every_element():
    c = WL.config("c2_1d_n4_mlp")
    M, H, F = c.dims
    _mlp1d(c.grid.p, c.grid.ri, M, H, F)


def test_config3_partials_full_size_sampled():
    """Config 3's backward in the partials form: four products per pass in one launch."""
    c = WL.config("c3_2d_q4")
    mx = T.tp_partials_map(c.grid, c.dims, T.PASS_DX_PARTIALS)
    _partials(c.grid, c.dims, rows=S.sample_rows(7, mx["m"], 128), w_rows=S.sample_rows(8, mx["n"], 64), label=c.name)


def test_config4_partials_full_size_sampled():
    c = WL.config("c4_2p5d_q2_d2")
    mx = T.tp_partials_map(c.grid, c.dims, T.PASS_DX_PARTIALS)
    _partials(c.grid, c.dims, rows=S.sample_rows(9, mx["m"], 128), w_rows=S.sample_rows(10, mx["n"], 64), label=c.name)


def test_config5_gathered_full_size_sampled():
    c = WL.config("c5_3d_p2")
    g = T.Grid(T.MODE_3D_GATHERED, p=c.grid.p, ri=c.grid.ri, rj=c.grid.rj, rk=c.grid.rk)
    mp = T.tp_block_map(g, c.dims, 0)
    _gathered3d(g, c.dims, rows=S.sample_rows(11, mp["m"], 128), w_rows=S.sample_rows(12, mp["k"], 64), label=c.name)
