"""Pins for the fp64 oracle: everything here checks oracle/tp_oracle.py against something
other than itself -- pure-Python brute force with math.erf, finite differences, closed forms,
special cases that reduce to a plain layer, the paper's Table 1 count and chunk shapes, and
torch's own bf16 conversion.  No GPU."""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import tp_oracle as O

RNG = np.random.default_rng(14883)


# ----------------------------------------------------------------------------- bf16 rounding
def test_bf16_roundtrip_exhaustive():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = O.bf16_bits_to_f64(bits)
    finite = np.isfinite(vals)
    back = O.f64_to_bf16_bits(O.round_to_bf16(vals[finite]))
    assert np.array_equal(back, bits[finite])
    # decode agrees with the format's definition: sign, 8-bit exponent (bias 127), 7-bit fraction
    for b in (0x3F80, 0xBF80, 0x4049, 0x0001, 0x0080, 0x7F7F, 0x3C00):
        s, e, f = b >> 15, (b >> 7) & 0xFF, b & 0x7F
        ref = (-1.0) ** s * ((f / 128.0) * 2.0 ** -126 if e == 0 else (1 + f / 128.0) * 2.0 ** (e - 127))
        assert O.bf16_bits_to_f64(np.array([b], dtype=np.uint16))[0] == ref


def test_bf16_ties_to_even_and_neighbours():
    bits = np.arange(0, 0x7F7F, dtype=np.uint32).astype(np.uint16)   # positive finite, has a successor
    lo = O.bf16_bits_to_f64(bits)
    hi = O.bf16_bits_to_f64(bits + np.uint16(1))
    mid = 0.5 * (lo + hi)                                            # exact in fp64
    even = np.where(bits % 2 == 0, lo, hi)
    assert np.array_equal(O.round_to_bf16(mid), even)
    assert np.array_equal(O.round_to_bf16(-mid), -even)
    assert np.array_equal(O.round_to_bf16(np.nextafter(mid, np.inf)), hi)
    assert np.array_equal(O.round_to_bf16(np.nextafter(mid, -np.inf)), lo)
    # a double rounding through fp32 would get this one wrong: just above a tie by less than an fp32 ulp
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert O.round_to_bf16(x) == 1.0 + 2.0 ** -7
    assert np.isinf(O.round_to_bf16(3.4e38)) and O.round_to_bf16(-3.4e38) < 0


def test_bf16_matches_torch_on_fp32_values():
    x = (RNG.standard_normal(200000) * np.exp(RNG.uniform(-20, 20, 200000))).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.round_to_bf16(x.astype(np.float64)), ref)


# ----------------------------------------------------------------------------- GeLU closed forms
def test_gelu_closed_forms():
    assert O.gelu(0.0) == 0.0
    assert O.dgelu(0.0) == 0.5
    x = np.linspace(-9, 9, 721)
    assert np.allclose(O.gelu(x) - O.gelu(-x), x, rtol=0, atol=1e-15)        # x Phi(x) + x Phi(-x)... = x
    assert np.allclose(O.dgelu(x) + O.dgelu(-x), 1.0, rtol=0, atol=1e-15)    # derivative of the line above
    assert np.allclose(O.gelu(np.array([8.0, 20.0])), [8.0, 20.0], rtol=1e-14)
    assert np.all(O.gelu(np.array([-8.0, -20.0])) <= 0) and np.all(O.gelu(np.array([-8.0, -20.0])) > -1e-13)
    # against math.erf / math.exp written out independently
    for a in (-3.7, -0.75, -1e-3, 0.3, 1.0, 2.5, 5.0):
        phi_c = 0.5 * (1 + math.erf(a / math.sqrt(2)))
        assert O.gelu(a) == pytest.approx(a * phi_c, rel=1e-14, abs=1e-300)
        assert O.dgelu(a) == pytest.approx(phi_c + a * math.exp(-a * a / 2) / math.sqrt(2 * math.pi), rel=1e-13)
    # the minimum: GeLU'(a*) = 0 near a* = -0.7518, value about -0.17
    xs = np.linspace(-1.0, -0.5, 50001)
    k = np.argmin(O.gelu(xs))
    assert abs(xs[k] + 0.75179) < 1e-4 and abs(O.gelu(xs[k]) + 0.16997) < 1e-4
    assert abs(O.dgelu(xs[k])) < 1e-4
    # dgelu is the derivative of gelu
    h = 1e-6
    xs = np.linspace(-5, 5, 101)
    assert np.allclose((O.gelu(xs + h) - O.gelu(xs - h)) / (2 * h), O.dgelu(xs), atol=1e-9)


# ----------------------------------------------------------------------------- brute force, pure Python
def _py_layer(X, W, b, act):
    M, H, F = len(X), len(W), len(W[0])
    A = [[sum(X[m][h] * W[h][f] for h in range(H)) + (b[f] if b is not None else 0.0) for f in range(F)]
         for m in range(M)]
    if not act:
        return A, A
    Y = [[0.5 * a * (1.0 + math.erf(a / math.sqrt(2.0))) for a in row] for row in A]
    return A, Y


def _py_bwd(X, W, A, G, act):
    M, H, F = len(X), len(W), len(W[0])
    def d(a):
        return 0.5 * (1 + math.erf(a / math.sqrt(2))) + a * math.exp(-a * a / 2) / math.sqrt(2 * math.pi)
    dA = [[G[m][f] * (d(A[m][f]) if act else 1.0) for f in range(F)] for m in range(M)]
    dX = [[sum(dA[m][f] * W[h][f] for f in range(F)) for h in range(H)] for m in range(M)]
    dW = [[sum(X[m][h] * dA[m][f] for m in range(M)) for f in range(F)] for h in range(H)]
    db = [sum(dA[m][f] for m in range(M)) for f in range(F)]
    return dA, dX, dW, db


def _tiny(M=12, H=12, F=24, scale_w=0.3):
    X = RNG.standard_normal((M, H))
    W = RNG.standard_normal((H, F)) * scale_w
    b = RNG.standard_normal(F) * 0.5
    G = RNG.standard_normal((M, F))
    return X, W, b, G


def test_full_layer_vs_pure_python():
    X, W, b, G = _tiny(5, 7, 6)
    A, Y = O.layer_fwd(X, W, b)
    pA, pY = _py_layer(X.tolist(), W.tolist(), b.tolist(), True)
    assert np.allclose(A, pA, rtol=1e-13, atol=1e-13) and np.allclose(Y, pY, rtol=1e-13, atol=1e-13)
    dA, dX, dW, db = O.layer_bwd(X, W, A, G)
    qA, qX, qW, qb = _py_bwd(X.tolist(), W.tolist(), pA, G.tolist(), True)
    for got, ref in ((dA, qA), (dX, qX), (dW, qW), (db, qb)):
        assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)
    # no-activation variant
    A2, Y2 = O.layer_fwd(X, W, None, act=False)
    assert np.allclose(Y2, _py_layer(X.tolist(), W.tolist(), None, False)[1], rtol=1e-13, atol=1e-13)


def _py_round_bf16(x: float) -> float:
    """Nearest 8-significant-bit float, ties to even, in plain Python: scale the mantissa of frexp to
    8 bits (exact), round() it (Python rounds exact halves to even), scale back."""
    if x == 0.0:
        return 0.0
    m, e = math.frexp(x)                  # x = m 2^e, 0.5 <= |m| < 1
    return math.ldexp(round(m * 256.0), e - 8)


def test_share_da_vs_pure_python_and_exact_midpoints():
    """share_da = bf16(G * GeLU'(A)): one rounding, after the multiply, ties to even.  Checked element by
    element against math.erf / math.exp and a hand-made rounding; the second half feeds products that
    are exact midpoints between two bf16 numbers (GeLU'(0) = 1/2 exactly, G = twice the midpoint), and
    values one fp64 ulp on either side of them."""
    G = RNG.standard_normal((9, 13)) * 3.0
    A = RNG.standard_normal((9, 13)) * 1.5
    got = O.share_da(G, A)
    for i, j in itertools.product(range(9), range(13)):
        a, g = float(A[i, j]), float(G[i, j])
        d = 0.5 * (1.0 + math.erf(a / math.sqrt(2.0))) + a * math.exp(-0.5 * a * a) / math.sqrt(2.0 * math.pi)
        assert got[i, j] == _py_round_bf16(g * d), (i, j)
        # a slip the kernel could share: rounding G * GeLU' of the ROUNDED derivative, or rounding twice
        assert abs(got[i, j] - g * d) <= abs(g * d) * 2.0 ** -8
    # exact midpoints: 1 + (2 n + 1) 2^-8 lies halfway between 1 + n 2^-7 and 1 + (n + 1) 2^-7
    mids = np.array([(1.0 + (2 * n + 1) * 2.0 ** -8) * s * 2.0 ** ex for n in (0, 1, 2, 63, 126, 127)
                     for s in (1.0, -1.0) for ex in (-3, 0, 5)])
    zeros = np.zeros_like(mids)
    r = O.share_da(2.0 * mids, zeros)
    for x, y in zip(mids.tolist(), r.tolist()):
        lo = math.ldexp(math.floor(math.frexp(abs(x))[0] * 256.0), math.frexp(abs(x))[1] - 8)
        hi = lo + math.ldexp(1.0, math.frexp(abs(x))[1] - 8)
        even = lo if (int(math.frexp(lo)[0] * 256.0) % 2 == 0) else hi
        assert abs(y) == even and math.copysign(1.0, y) == math.copysign(1.0, x), (x, y, lo, hi)
    up = O.share_da(2.0 * np.nextafter(mids, np.inf * np.sign(mids)), zeros)       # just past the midpoint: away from zero
    dn = O.share_da(2.0 * np.nextafter(mids, 0.0), zeros)                          # just short of it: towards zero
    for x, u, d_ in zip(mids.tolist(), up.tolist(), dn.tolist()):
        m, e = math.frexp(abs(x))
        lo = math.ldexp(math.floor(m * 256.0), e - 8)
        assert abs(u) == lo + math.ldexp(1.0, e - 8) and abs(d_) == lo, (x, u, d_)
    # the no-op cases: GeLU'(a) -> 1 for large a, -> 0 for very negative a
    assert O.share_da(np.array([[3.0]]), np.array([[40.0]]))[0, 0] == 3.0
    assert O.share_da(np.array([[3.0]]), np.array([[-40.0]]))[0, 0] == 0.0


def test_backward_by_finite_differences():
    X, W, b, G = _tiny(4, 5, 6)
    A, _ = O.layer_fwd(X, W, b)
    _, dX, dW, db = O.layer_bwd(X, W, A, G)
    loss = lambda X_, W_, b_: float((G * O.layer_fwd(X_, W_, b_)[1]).sum())
    h = 1e-6
    for T, dT, name in ((X, dX, "X"), (W, dW, "W"), (b, db, "b")):
        num = np.zeros_like(T)
        for idx in np.ndindex(*T.shape):
            Tp, Tm = T.copy(), T.copy()
            Tp[idx] += h
            Tm[idx] -= h
            args_p = {"X": (Tp, W, b), "W": (X, Tp, b), "b": (X, W, Tp)}[name]
            args_m = {"X": (Tm, W, b), "W": (X, Tm, b), "b": (X, W, Tm)}[name]
            num[idx] = (loss(*args_p) - loss(*args_m)) / (2 * h)
        assert np.allclose(num, dT, rtol=1e-6, atol=1e-7), name


def test_identity_and_one_hot_special_cases():
    X = RNG.standard_normal((6, 8))
    _, Y = O.layer_fwd(X, np.eye(8), np.zeros(8))
    assert np.allclose(Y, [[0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in r] for r in X], atol=1e-15)
    W = RNG.standard_normal((8, 5))
    b = RNG.standard_normal(5)
    _, Y = O.layer_fwd(np.eye(8), W, b)           # one-hot rows pick rows of W
    assert np.allclose(Y, O.gelu(W + b[None, :]), atol=1e-15)
    # a transposed operand would show here: non-square, asymmetric
    X = np.arange(6.0).reshape(2, 3)
    W = np.arange(12.0).reshape(3, 4) / 10
    A, _ = O.layer_fwd(X, W, None, act=False)
    assert np.allclose(A, [[2.0, 2.3, 2.6, 2.9], [5.6, 6.8, 8.0, 9.2]], atol=1e-14)


# ----------------------------------------------------------------------------- assembled ranks == unpartitioned layer
GRIDS = ([(O.MODE_1D_COL, dict(p=n)) for n in (1, 2, 3, 4)] +
         [(O.MODE_1D_ROW, dict(p=n)) for n in (1, 2, 3, 4)] +
         [(O.MODE_2D, dict(q=q)) for q in (1, 2, 3)] +
         [(O.MODE_2P5D, dict(q=q, d=d)) for q in (1, 2, 3) for d in (1, 2)] +
         [(O.MODE_3D, dict(p=p)) for p in (1, 2)])


@pytest.mark.parametrize("mode,kw", GRIDS, ids=[f"{m}-{k}" for m, k in GRIDS])
def test_assembled_ranks_reproduce_the_full_layer(mode, kw):
    X, W, b, G = _tiny(12, 12, 24)
    act = mode != O.MODE_1D_ROW
    bias = b if act else None
    pA, pY = _py_layer(X.tolist(), W.tolist(), None if bias is None else bias.tolist(), act)
    qA, qX, qW, _ = _py_bwd(X.tolist(), W.tolist(), pA, G.tolist(), act)
    ranks = O.all_ranks(mode, **kw)
    assert len(ranks) == ranks[0].n_ranks()
    Ys = [O.rank_fwd(g, X, W, bias, act)[1] for g in ranks]
    if mode == O.MODE_1D_ROW:
        # every rank's block is an additive partial of the whole output (the all-reduce's input)
        assert all(y.shape == (12, 24) for y in Ys)
    Y = O.assemble(ranks, O.PASS_FWD, Ys, (12, 24))
    assert np.allclose(Y, pY, rtol=0, atol=1e-12)
    dA = np.array(qA)
    dX = O.assemble(ranks, O.PASS_DX, [O.rank_dx(g, dA, W) for g in ranks], (12, 12))
    dW = O.assemble(ranks, O.PASS_DW, [O.rank_dw(g, X, dA) for g in ranks], (12, 24))
    assert np.allclose(dX, qX, rtol=0, atol=1e-12)
    assert np.allclose(dW, qW, rtol=0, atol=1e-12)
    # every output chunk is covered: exactly once when exact, by every partial-group member otherwise
    for pass_ in (O.PASS_FWD, O.PASS_DX, O.PASS_DW):
        outs = [O.block_map(g, pass_)["out"] for g in ranks]
        parts = [O.block_map(g, pass_)["partial"] for g in ranks]
        mult = {o: outs.count(o) for o in set(outs)}
        assert len(set(mult.values())) == 1
        assert all(p == (m > 1) for p, m in zip(parts, (mult[o] for o in outs)))


def test_single_rank_grids_are_the_plain_layer():
    X, W, b, G = _tiny(4, 6, 8)
    A, Y = O.layer_fwd(X, W, b)
    for g in (O.Grid(O.MODE_1D_COL), O.Grid(O.MODE_2D), O.Grid(O.MODE_2P5D), O.Grid(O.MODE_3D)):
        a, y = O.rank_fwd(g, X, W, b)
        assert np.array_equal(a, A) and np.array_equal(y, Y)
        assert np.array_equal(O.rank_dx(g, G, W), G @ W.T)
        assert np.array_equal(O.rank_dw(g, X, G), X.T @ G)


def test_depth_one_tesseract_is_2d():
    """Section 2.2: with depth 1 the 2.5D scheme coincides with 2D."""
    for q in (1, 2, 3):
        for i, j in itertools.product(range(q), range(q)):
            for pass_ in (O.PASS_FWD, O.PASS_DX, O.PASS_DW):
                assert O.block_map(O.Grid(O.MODE_2P5D, q=q, d=1, ri=i, rj=j), pass_) == \
                    O.block_map(O.Grid(O.MODE_2D, q=q, ri=i, rj=j), pass_)
            assert O.chunk_counts(O.Grid(O.MODE_2P5D, q=q, d=1)) == O.chunk_counts(O.Grid(O.MODE_2D, q=q))


def test_partial_step_counts_are_prefix_sums():
    X, W, b, _ = _tiny(8, 8, 8)
    g = O.Grid(O.MODE_3D, p=2, ri=1, rj=0, rk=1)
    A1, _ = O.rank_fwd(g, X, W, None, act=False, n_steps=1)
    r = 1 * 2 + 1
    assert np.allclose(A1, X[2 * r:2 * r + 2, 0:4] @ W[0:4, 0:4], atol=1e-14)


# ----------------------------------------------------------------------------- the paper's own numbers
def _golden(golden_dir, name):
    rows = []
    with open(os.path.join(golden_dir, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([c.strip() for c in line.split(";")])
    return rows


def test_chunk_shapes_follow_the_paper(golden_dir):
    P, Q = 720, 360
    for mode, n_expr, rows_expr, cols_expr in _golden(golden_dir, "chunk_shapes.txt"):
        for q, d, p in ((2, 1, 2), (3, 2, 1), (2, 2, 2)):
            env = dict(P=P, Q=Q, q=q, d=d, p=p)
            g = {"2D": O.Grid(O.MODE_2D, q=q), "2.5D": O.Grid(O.MODE_2P5D, q=q, d=d), "3D": O.Grid(O.MODE_3D, p=p)}[mode]
            assert g.n_ranks() == eval(n_expr, {}, env)
            rc, kc, cc = O.chunk_counts(g)
            T = np.zeros((P, Q))
            # X-like tensors are cut (rc, kc); Y-like (rc, cc): both must give the printed chunk shape
            assert O.chunk(T, rc, kc, 0, 0).shape == (eval(rows_expr, {}, env), eval(cols_expr, {}, env))
            assert O.chunk(T, rc, cc, 0, 0).shape == (eval(rows_expr, {}, env), eval(cols_expr, {}, env))


def test_2d_map_moves_table1_volume(golden_dir):
    """Table 1, 2D row: 3 (j-1)(Sx+Sw) elements for fwd + two backward products, i.e. (j-1)(Sx+Sw)
    per product: count the elements of the non-own blocks all ranks consume in the forward map."""
    expr = dict((r[0], r[1]) for r in _golden(golden_dir, "table1_comm_volume.txt"))["2D"]
    fig = dict(kv.split("=") for kv in dict((r[0], r[1]) for r in _golden(golden_dir, "table1_comm_volume.txt"))["fig"].split())
    h, s, b = int(fig["h"]), int(fig["s"]), int(fig["b"])
    Sx, Sw = b * s * h, h * h
    for j in (1, 2, 3, 4):
        if (b * s) % j or h % j:
            continue
        moved = 0
        for g in O.all_ranks(O.MODE_2D, q=j):
            mp = O.block_map(g, O.PASS_FWD)
            own_x, own_w = (g.ri, g.rj), (g.ri, g.rj)       # the chunk of X and of W stored on rank (i, j)
            moved += sum((b * s // j) * (h // j) for ab in mp["a"] if ab != own_x)
            moved += sum((h // j) * (h // j) for bb in mp["b"] if bb != own_w)
        assert 3 * moved == eval(expr, {}, dict(j=j, Sx=Sx, Sw=Sw))


def test_backward_partials_move_table1_volume(golden_dir):
    """Table 1, 2D and 2.5D rows: each of the two backward products moves as much as the forward one,
    (side-1)(Sx+Sw) (2.5D: (side-1)(Sx/d+Sw) per depth layer), when dA stays put, one block of the
    other operand arrives per step and the partial products travel to their owners.  Counted from
    the partials map: operand blocks that are not the rank's own plus partials owned by another rank."""
    rows = dict((r[0], r[1]) for r in _golden(golden_dir, "table1_comm_volume.txt"))
    fig = dict(kv.split("=") for kv in rows["fig"].split())
    h, s, b = int(fig["h"]), int(fig["s"]), int(fig["b"])
    Sx, Sw = b * s * h, h * h
    for q, d in ((1, 1), (2, 1), (4, 1), (2, 2), (4, 2), (2, 4)):
        mode = O.MODE_2D if d == 1 else O.MODE_2P5D
        ranks = O.all_ranks(mode, q=q, d=d)
        xb = (b * s // (q * d)) * (h // q)             # elements of one X / dX / dA block
        wb = (h // q) * (h // q)
        for pass_ in (O.PASS_DX, O.PASS_DW):
            moved = 0
            for g in ranks:
                mp = O.partials_map(g, pass_)
                r = mp["own"][0]
                stored_w, stored_x = (g.ri, g.rj), (r, g.rj)     # what rank (i, j[, layer]) keeps of W and of X / dX
                if pass_ == O.PASS_DX:                           # W blocks in, dX partials out
                    moved += sum(wb for k in mp["other"] if k != stored_w)
                    moved += sum(xb for o in mp["out"] if o != stored_x)
                else:                                            # X blocks in, dW partials out
                    moved += sum(xb for k in mp["other"] if k != stored_x)
                    moved += sum(wb for o in mp["out"] if o != stored_w)
            per_product = eval(rows["2D"] if d == 1 else rows["2.5D"], {}, dict(j=q, k=q, d=d, Sx=Sx, Sw=Sw)) / 3
            assert moved == (per_product if d == 1 else per_product * d)      # 2.5D row is per depth layer


def test_backward_partials_sum_to_the_plain_gradients():
    """Every partial placed on the block it belongs to and summed: dX = dA W^T, dW = X^T dA."""
    M, H, F = 24, 12, 16
    X, W, b, G = _tiny(M, H, F)
    A, Y = O.layer_fwd(X, W, b)
    dA, dX, dW, _ = O.layer_bwd(X, W, A, G)
    for mode, q, d in ((O.MODE_2D, 2, 1), (O.MODE_2P5D, 2, 3), (O.MODE_2D, 4, 1), (O.MODE_2P5D, 2, 2), (O.MODE_2D, 1, 1)):
        ranks = O.all_ranks(mode, q=q, d=d)
        gx, gw = np.zeros((M, H)), np.zeros((H, F))
        for g in ranks:
            rc, kc, cc = O.chunk_counts(g)
            for (r, c), P in O.rank_dx_partials(g, dA, W):
                hh, ww = M // rc, H // kc
                assert P.shape == (hh, ww)
                gx[r * hh:(r + 1) * hh, c * ww:(c + 1) * ww] += P
            for (r, c), P in O.rank_dw_partials(g, X, dA):
                hh, ww = H // kc, F // cc
                assert P.shape == (hh, ww)
                gw[r * hh:(r + 1) * hh, c * ww:(c + 1) * ww] += P
        assert np.allclose(gx, dX, rtol=0, atol=1e-12)
        assert np.allclose(gw, dW, rtol=0, atol=1e-12)
    # one rank, by hand: rank (1, 0) of a 2 x 2 grid, dX partial for owner (1, 1) is dA[1,0] W[1,0]^T
    g = O.Grid(O.MODE_2D, q=2, ri=1, rj=0)
    parts = dict(O.rank_dx_partials(g, dA, W))
    assert np.allclose(parts[(1, 1)], dA[12:, :8] @ W[6:, :8].T, atol=1e-13)
    parts = dict(O.rank_dw_partials(g, X, dA))
    assert np.allclose(parts[(1, 0)], X[12:, 6:].T @ dA[12:, :8], atol=1e-13)
    with pytest.raises(ValueError):
        O.partials_map(O.Grid(O.MODE_3D, p=2), O.PASS_DX)
    with pytest.raises(ValueError):
        O.partials_map(g, O.PASS_FWD)


def test_3d_gathered_products_sum_to_the_layer_and_match_the_owner_reading():
    """The single gathered-shape product per rank: partials summed over the cube axis they are
    partial over give X W, dA W^T, X^T dA; row chunk l of the summed forward slab (i, j), with
    bias and GeLU applied, is what the owner-computes 3D share of rank (i, j, l) holds."""
    p, M, H, F = 2, 16, 8, 12
    X, W, b, G = _tiny(M, H, F)
    A, Y = O.layer_fwd(X, W, b)
    dA, dX, dW, _ = O.layer_bwd(X, W, A, G)
    ranks = O.all_ranks(O.MODE_3D, p=p)
    full = {O.PASS_FWD: (np.zeros((M, F)), X @ W, M // p, F // p),
            O.PASS_DX: (np.zeros((M, H)), dX, M // p, H // p),
            O.PASS_DW: (np.zeros((H, F)), dW, H // p, F // p)}
    for g in ranks:
        for pass_, (acc, _, hh, ww) in full.items():
            (r, c), P = O.rank3d_gathered(g, pass_, X=X, W=W, dA=dA)
            assert P.shape == (hh, ww)
            acc[r * hh:(r + 1) * hh, c * ww:(c + 1) * ww] += P
    for acc, ref, _, _ in full.values():
        assert np.allclose(acc, ref, rtol=0, atol=1e-12)
    summed = full[O.PASS_FWD][0]
    for g in ranks:
        i, j, l = g.ri, g.rj, g.rk
        slab = summed[i * (M // p):(i + 1) * (M // p), j * (F // p):(j + 1) * (F // p)]
        mine = slab[l * (M // p // p):(l + 1) * (M // p // p)]
        a_ref, y_ref = O.rank_fwd(g, X, W, b)
        a, y = O.bias_gelu(mine, b[j * (F // p):(j + 1) * (F // p)])
        assert np.allclose(a, a_ref, atol=1e-12) and np.allclose(y, y_ref, atol=1e-12)
    # shapes as the paper prints them: stored chunk [P/p^2, Q/p], gathered slab [P/p, Q/p]
    g = O.Grid(O.MODE_3D, p=2, ri=1, rj=0, rk=1)
    (_, P) = O.rank3d_gathered(g, O.PASS_FWD, X=X, W=W)
    assert P.shape == (M // p, F // p) and O.rank_fwd(g, X, W, b)[0].shape == (M // p ** 2, F // p)
    with pytest.raises(ValueError):
        O.gathered3d_map(O.Grid(O.MODE_2D, q=2), O.PASS_FWD)


def test_grid_rule_rejects_bad_grids():
    with pytest.raises(ValueError):
        O.check_grid(O.Grid(O.MODE_2D, q=2, ri=2), 8, 8, 8)
    with pytest.raises(ValueError):
        O.check_grid(O.Grid(O.MODE_2P5D, q=2, d=2, rk=2), 8, 8, 8)
    with pytest.raises(ValueError):
        O.check_grid(O.Grid(O.MODE_3D, p=2), 6, 8, 8)       # M not divisible by p^2
    with pytest.raises(ValueError):
        O.check_grid(O.Grid(O.MODE_2D, q=0), 8, 8, 8)
    O.check_grid(O.Grid(O.MODE_3D, p=2, ri=1, rj=1, rk=1), 8, 8, 8)


# ----------------------------------------------------------------------------- 1D feed-forward chain with rounding points
def test_mlp1d_chain_sums_to_the_full_mlp():
    M, H, F, N = 6, 8, 12, 3
    X = O.round_to_bf16(RNG.standard_normal((M, H)))
    W1 = O.round_to_bf16(RNG.standard_normal((H, F)) * 0.3)
    b1 = O.round_to_bf16(RNG.standard_normal(F) * 0.3)
    W2 = O.round_to_bf16(RNG.standard_normal((F, H)) * 0.3)
    G = O.round_to_bf16(RNG.standard_normal((M, H)))
    tb = lambda a: torch.tensor(a, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    pA, pZ = _py_layer(X.tolist(), W1.tolist(), b1.tolist(), True)
    Zr = tb(np.array(pZ))
    Ar = tb(np.array(pA))
    fw = [O.mlp1d_fwd(X, W1[:, r * 4:(r + 1) * 4], b1[r * 4:(r + 1) * 4], W2[r * 4:(r + 1) * 4, :]) for r in range(N)]
    Zo = np.concatenate([f["Z"] for f in fw], axis=1)
    Ao = np.concatenate([f["A_saved"] for f in fw], axis=1)
    # torch rounds via fp32; allow the (measure-zero) double-rounding cases to differ by one bf16 step
    assert np.mean(Zo == Zr) > 0.98 and np.allclose(Zo, Zr, rtol=2 ** -7)
    assert np.mean(Ao == Ar) > 0.98 and np.allclose(Ao, Ar, rtol=2 ** -7)
    Yfull = np.array(_py_layer(Zo.tolist(), W2.tolist(), None, False)[1])
    assert np.allclose(sum(f["Y"] for f in fw), Yfull, atol=1e-12)
    # backward: dW2 rows and dW1 columns are exact slices, dX partials sum to the full dX
    dZ = np.array(_py_bwd(Zo.tolist(), W2.tolist(), None, G.tolist(), False)[1])
    dAf = O.round_to_bf16(dZ * np.array([[O.dgelu(a) for a in row] for row in Ao]))
    dXfull = np.array(_py_bwd(X.tolist(), W1.tolist(), None, dAf.tolist(), False)[1])
    dW1full = np.array(_py_bwd(X.tolist(), W1.tolist(), None, dAf.tolist(), False)[2])
    dW2full = np.array(_py_bwd(Zo.tolist(), W2.tolist(), None, G.tolist(), False)[2])
    bw = [O.mlp1d_bwd(X, W1[:, r * 4:(r + 1) * 4], W2[r * 4:(r + 1) * 4, :], fw[r]["A_saved"], fw[r]["Z"], G)
          for r in range(N)]
    assert np.allclose(sum(o["dX"] for o in bw), dXfull, atol=1e-12)
    assert np.allclose(np.concatenate([o["dW1"] for o in bw], axis=1), dW1full, atol=1e-12)
    assert np.allclose(np.concatenate([o["dW2"] for o in bw], axis=0), dW2full, atol=1e-12)
    # row / weight-row sampling returns the same numbers as the full computation
    o = O.mlp1d_bwd(X, W1[:, :4], W2[:4, :], fw[0]["A_saved"], fw[0]["Z"], G, rows=[1, 4], w_rows=[0, 3])
    assert np.array_equal(o["dX"], bw[0]["dX"][[1, 4]])
    assert np.allclose(o["dW1"], bw[0]["dW1"][[0, 3]], atol=1e-14) and np.allclose(o["dW2"], bw[0]["dW2"][[0, 3]], atol=1e-14)


def test_share_row_sampling_matches_full():
    xs = [RNG.standard_normal((10, 6)) for _ in range(3)]
    ws = [RNG.standard_normal((6, 8)) for _ in range(3)]
    b = RNG.standard_normal(8)
    A, Y = O.share_fwd(xs, ws, b)
    A2, Y2 = O.share_fwd(xs, ws, b, rows=[0, 9, 3])
    assert np.array_equal(A2, A[[0, 9, 3]]) and np.array_equal(Y2, Y[[0, 9, 3]])
    ds = [RNG.standard_normal((10, 8)) for _ in range(3)]
    wt = [RNG.standard_normal((6, 8)) for _ in range(3)]
    assert np.array_equal(O.share_dx(ds, wt, rows=[2, 7]), O.share_dx(ds, wt)[[2, 7]])
    assert np.allclose(O.share_dw(xs, ds, rows=[5, 1]), O.share_dw(xs, ds)[[5, 1]], atol=1e-14)
    # share_dx / share_dw against explicit loops
    ref = sum(np.einsum("mf,hf->mh", d, w) for d, w in zip(ds, wt))
    assert np.allclose(O.share_dx(ds, wt), ref, atol=1e-13)
    ref = sum(np.einsum("mh,mf->hf", x, d) for x, d in zip(xs, ds))
    assert np.allclose(O.share_dw(xs, ds), ref, atol=1e-13)
