"""The benchmark configurations and the synthetic blocks one rank needs for them.

Host-side bookkeeping only: which chunks of the full (never materialised) tensors a rank's share
reads, by the library's own partition map, generated position by position with the seeded
generator.  No arithmetic of the layer happens here.

Stand-in recipe: activations X ~ N(0,1), weights and biases ~ N(0, 0.02^2), upstream gradient
G ~ N(0,1), all rounded to bf16.  Peer ranks' dA blocks (which in a real run come from the peers'
own forward) are described by a peer gradient block G_peer ~ N(0,1) and a peer pre-activation block
A_peer ~ N(0, (0.02 sqrt(H))^2) -- the spread X W has for these inputs -- and are turned into dA by
whoever consumes the workload (the oracle in tests, tp_dgelu in the benchmark).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

import synth_inputs as S

from . import binding as B


@dataclass
class Config:
    name: str
    grid: B.Grid
    dims: tuple                    # full layer (M, H, F)
    n_steps: int | None = None     # None = the exact share's step count; an int = a prefix (literal reading)
    y_dtype: str = "bf16"          # forward output dtype
    dx_dtype: str = "bf16"
    backward: bool = True
    chain_1d: bool = False         # 1D feed-forward chain: two weights, see make_mlp1d_inputs
    second_linear: bool = False    # the down-projection of an MLP: bias-only forward, fp32 Y, and in backward
                                   # GeLU'(A1) of the previous layer fused into dX's epilogue (no separate dA pass)
    variant: str = ""              # "partials": backward as partials for other owners (tp_linear_bwd_partials);
                                   # "gathered": 3D at its gathered local shape (one product per pass)
    note: str = ""
    extra: dict = field(default_factory=dict)


# The five configurations of the benchmark, in order.  Rank choices: non-zero offsets on every
# axis that exists.
CONFIGS = [
    Config("c1_2d_q2_fwd", B.Grid(B.MODE_2D, q=2, ri=0, rj=0), (256, 1024, 4096), y_dtype="f32", backward=False,
           note="2D SUMMA q=2 rank (0,0), MLP up-projection, forward only, fp32 output"),
    Config("c2_1d_n4_mlp", B.Grid(B.MODE_1D_COL, p=4, ri=1), (16384, 4096, 16384), chain_1d=True,
           note="1D size 4 rank 1: X W1[:,r] + b1, GeLU, then Z W2[r,:] as an fp32 partial; fwd + bwd (6 products)"),
    Config("c3_2d_q4", B.Grid(B.MODE_2D, q=4, ri=1, rj=2), (8192, 8192, 32768),
           note="2D SUMMA q=4 rank (1,2): 4-step forward, dX and dW"),
    Config("c4_2p5d_q2_d2", B.Grid(B.MODE_2P5D, q=2, d=2, ri=1, rj=0, rk=1), (131584, 1280, 5120),
           note="2.5D q=2 d=2 rank (1,0,1), ViT-style MLP, ragged local M = 32896"),
    Config("c5_3d_p2", B.Grid(B.MODE_3D, p=2, ri=1, rj=0, rk=1), (16384, 12288, 49152), n_steps=1,
           note="3D p=2 rank (1,0,1), GPT-3-175B-shaped MLP, literal single local product"),
    Config("n1_2d_q4_fc2", B.Grid(B.MODE_2D, q=4, ri=1, rj=2), (8192, 32768, 8192), second_linear=True, y_dtype="f32",
           note="the second linear (F -> H) of config 3's MLP: bias-only forward, dX with fused GeLU' epilogue, dW"),
    Config("c5x_3d_p2_exact", B.Grid(B.MODE_3D, p=2, ri=1, rj=0, rk=1), (16384, 12288, 49152),
           note="as c5 with both steps of the exact share"),
    Config("r3_2d_q4_partials", B.Grid(B.MODE_2D, q=4, ri=1, rj=2), (8192, 8192, 32768), variant="partials",
           note="config 3 with the backward products as partials for other owners: 4 products per pass in one launch"),
    Config("r4_2p5d_q2_d2_partials", B.Grid(B.MODE_2P5D, q=2, d=2, ri=1, rj=0, rk=1), (131584, 1280, 5120), variant="partials",
           note="config 4 with the backward products as partials for other owners"),
    Config("g5_3d_p2_gathered", B.Grid(B.MODE_3D_GATHERED, p=2, ri=1, rj=0, rk=1), (16384, 12288, 49152), variant="gathered",
           note="config 5's layer at the gathered local shape: one 8192 x 6144 x 24576 product per pass, fp32 partials, "
                "bias + GeLU on the rank's chunk afterwards"),
]


def config(name: str) -> Config:
    for c in CONFIGS:
        if c.name == name:
            return c
    raise KeyError(name)


def _chunk_counts(grid: B.Grid):
    m = grid.mode
    if m == B.MODE_1D_COL:
        return 1, 1, grid.p
    if m == B.MODE_1D_ROW:
        return 1, grid.p, 1
    if m == B.MODE_2D:
        return grid.q, grid.q, grid.q
    if m == B.MODE_2P5D:
        return grid.q * grid.d, grid.q, grid.q
    return grid.p * grid.p, grid.p, grid.p


def make_share_inputs(grid: B.Grid, dims, seed: int = S.BASE_SEED, n_steps: int | None = None,
                      backward: bool = True) -> dict:
    """bf16 bit patterns (numpy uint16) of every block rank `grid` touches in forward and, if asked,
    backward.  Keys: maps (fwd/dx/dw), x_blocks, w_blocks, bias, and for backward g_own, w_blocks_dx,
    x_blocks_dw, peers_dx / peers_dw = {slot: (g_peer, a_peer)}, own_slot_dx / own_slot_dw."""
    M, H, F = dims
    rc, kc, cc = _chunk_counts(grid)
    mb, hb, fb = M // rc, H // kc, F // cc
    fwd = B.tp_block_map(grid, dims, B.PASS_FWD)
    s_f = fwd["n_steps"] if n_steps is None else n_steps
    sigma_a = 0.02 * math.sqrt(H)

    def X(r, c): return S.normal_block_bf16(seed, S.T_X, H, r * mb, mb, c * hb, hb, 1.0)
    def W(r, c): return S.normal_block_bf16(seed, S.T_W1, F, r * hb, hb, c * fb, fb, 0.02)
    def G(r, c): return S.normal_block_bf16(seed, S.T_G, F, r * mb, mb, c * fb, fb, 1.0)
    def PA(r, c): return S.normal_block_bf16(seed, S.T_PEER_A, F, r * mb, mb, c * fb, fb, sigma_a)

    cache: dict = {}

    def get(kind, fn, r, c):
        key = (kind, r, c)
        if key not in cache:
            cache[key] = fn(r, c)
        return cache[key]

    out = dict(grid=grid, dims=dims, fwd=fwd, n_steps_fwd=s_f, m=mb, k=hb, n=fb)
    out["x_blocks"] = [get("X", X, *fwd["a"][k]) for k in range(s_f)]
    out["w_blocks"] = [get("W", W, *fwd["b"][k]) for k in range(s_f)]
    out["bias"] = S.normal_block_bf16(seed, S.T_B1, F, 0, 1, fwd["out"][1] * fb, fb, 0.02)[0]
    if not backward:
        return out
    dxm = B.tp_block_map(grid, dims, B.PASS_DX)
    dwm = B.tp_block_map(grid, dims, B.PASS_DW)
    s_x = dxm["n_steps"] if n_steps is None else n_steps
    s_w = dwm["n_steps"] if n_steps is None else n_steps
    own = fwd["out"]
    out.update(dx=dxm, dw=dwm, n_steps_dx=s_x, n_steps_dw=s_w)
    out["g_own"] = get("G", G, *own)
    # with a prefix of the steps (literal reading) the own block is always among them: put it first
    order_x = list(range(dxm["n_steps"]))
    order_w = list(range(dwm["n_steps"]))
    if n_steps is not None:
        order_x.sort(key=lambda k: dxm["a"][k] != own)
        order_w.sort(key=lambda k: dwm["b"][k] != own)
    order_x, order_w = order_x[:s_x], order_w[:s_w]
    out["own_slot_dx"] = next((i for i, k in enumerate(order_x) if dxm["a"][k] == own), -1)
    out["own_slot_dw"] = next((i for i, k in enumerate(order_w) if dwm["b"][k] == own), -1)
    out["w_blocks_dx"] = [get("W", W, *dxm["b"][k]) for k in order_x]
    out["x_blocks_dw"] = [get("X", X, *dwm["a"][k]) for k in order_w]
    out["peers_dx"] = {i: (get("G", G, *dxm["a"][k]), get("PA", PA, *dxm["a"][k]))
                       for i, k in enumerate(order_x) if dxm["a"][k] != own}
    out["peers_dw"] = {i: (get("G", G, *dwm["b"][k]), get("PA", PA, *dwm["b"][k]))
                       for i, k in enumerate(order_w) if dwm["b"][k] != own}
    return out


def make_partials_inputs(grid: B.Grid, dims, seed: int = S.BASE_SEED) -> dict:
    """Blocks for the backward products in their partials form (2D / 2.5D): the rank's own dA block
    (taken from the upstream-gradient generator: any bf16 block serves), the W blocks of its column
    and the X blocks of its row, by the library's own map."""
    M, H, F = dims
    rc, kc, cc = _chunk_counts(grid)
    mb, hb, fb = M // rc, H // kc, F // cc
    dxm = B.tp_partials_map(grid, dims, B.PASS_DX_PARTIALS)
    dwm = B.tp_partials_map(grid, dims, B.PASS_DW_PARTIALS)
    r, c = dxm["own"]
    return dict(grid=grid, dims=dims, dx=dxm, dw=dwm, m=mb, h=hb, f=fb,
                da_own=S.normal_block_bf16(seed, S.T_G, F, r * mb, mb, c * fb, fb, 1.0),
                w_blocks=[S.normal_block_bf16(seed, S.T_W1, F, wr * hb, hb, wc * fb, fb, 0.02) for wr, wc in dxm["other"]],
                x_blocks=[S.normal_block_bf16(seed, S.T_X, H, xr * mb, mb, xc * hb, hb, 1.0) for xr, xc in dwm["other"]])


def make_gathered3d_inputs(grid: B.Grid, dims, seed: int = S.BASE_SEED) -> dict:
    """Slabs of the single gathered-shape product per pass of a 3D rank (grid.mode MODE_3D_GATHERED):
    X slab, W block, dA slab (from the upstream-gradient generator)."""
    M, H, F = dims
    p = grid.p
    ms, hb, fb = M // p, H // p, F // p
    maps = {ps: B.tp_block_map(grid, dims, ps) for ps in (B.PASS_FWD, B.PASS_DX, B.PASS_DW)}
    (xr, xc), (wr, wc) = maps[B.PASS_FWD]["a"][0], maps[B.PASS_FWD]["b"][0]
    (gr, gc) = maps[B.PASS_DX]["a"][0]
    return dict(grid=grid, dims=dims, maps=maps, m=ms, h=hb, f=fb,
                x=S.normal_block_bf16(seed, S.T_X, H, xr * ms, ms, xc * hb, hb, 1.0),
                w=S.normal_block_bf16(seed, S.T_W1, F, wr * hb, hb, wc * fb, fb, 0.02),
                da=S.normal_block_bf16(seed, S.T_G, F, gr * ms, ms, gc * fb, fb, 1.0),
                bias=S.normal_block_bf16(seed, S.T_B1, F, 0, 1, maps[B.PASS_FWD]["out"][1] * fb, fb, 0.02)[0])


def make_mlp1d_inputs(size: int, rank: int, M: int, H: int, F: int, seed: int = S.BASE_SEED) -> dict:
    """Rank `rank` of a 1D feed-forward of `size` ranks: X [M,H], W1[:, r] [H, F/size], b1[r],
    W2[r, :] [F/size, H], upstream gradient G [M, H]."""
    fb = F // size
    return dict(
        size=size, rank=rank, M=M, H=H, F=F, fb=fb,
        X=S.normal_block_bf16(seed, S.T_X, H, 0, M, 0, H, 1.0),
        W1=S.normal_block_bf16(seed, S.T_W1, F, 0, H, rank * fb, fb, 0.02),
        b1=S.normal_block_bf16(seed, S.T_B1, F, 0, 1, rank * fb, fb, 0.02)[0],
        W2=S.normal_block_bf16(seed, S.T_W2, H, rank * fb, fb, 0, H, 0.02),
        G=S.normal_block_bf16(seed, S.T_G, H, 0, M, 0, H, 1.0),
    )


def gemm_flops(cfg_or_inputs) -> dict:
    """GEMM flops (2 m n k per product) of a share: forward, backward, total."""
    if isinstance(cfg_or_inputs, Config):
        c = cfg_or_inputs
        if c.variant == "gathered":
            f = B.tp_block_map(c.grid, c.dims, B.PASS_FWD)
            one = 2.0 * f["m"] * f["n"] * f["k"]
            return dict(fwd=one, bwd=2 * one, total=3 * one)
        if c.chain_1d:
            M, H, F = c.dims
            one = 2.0 * M * H * (F // c.grid.p)
            return dict(fwd=2 * one, bwd=4 * one, total=6 * one)
        f = B.tp_block_map(c.grid, c.dims, B.PASS_FWD)
        s = f["n_steps"] if c.n_steps is None else c.n_steps
        one = 2.0 * f["m"] * f["n"] * f["k"] * s
        return dict(fwd=one, bwd=2 * one if c.backward else 0.0, total=one * (3 if c.backward else 1))
    raise TypeError
