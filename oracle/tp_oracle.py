"""fp64 CPU oracle for one rank's share of a tensor-parallel linear layer.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
GPU library is checked against.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product path never does, and
this module imports nothing from the product.

What it computes (paper Section 2.2 "Model Parallelism", tensor parallelism
paragraphs, and Section 3.1 with Table 1): a linear layer whose input, weight
and output are split over a rank grid -- 1D (Megatron: weight split by columns,
then by rows, partial outputs summed by an all-reduce), 2D (SUMMA on a q x q
square, chunks [P/q, Q/q]), 2.5D (q x q x d cuboid, N = S^2 * D) and 3D
(p x p x p cube, chunks [P/p^2, Q/p]).  The partitioned methods reach exactly
the unpartitioned layer, so the ground truth is the plain definition

    A = X W + 1 b^T          Y = GeLU(A) = A/2 (1 + erf(A / sqrt 2))
    dA = G * GeLU'(A)        GeLU'(a) = Phi(a) + a phi(a)
    dX = dA W^T              dW = X^T dA              db = 1^T dA

in fp64, and a rank's share is a block (or an additive partial) of it, picked
by the partition map below.  Conventions (the paper fixes none of them; they
are this build's readings): tokens are rows,
X:[M,H], W:[H,F] (in x out), b:[F]; the step index k runs upward; erf-GeLU.

Rounding points: where a bf16 tensor is handed from one product to the next
(the saved pre-activation, Z between the two 1D products, dA) the fp64 value is
rounded to the nearest bf16 (ties to even) straight from fp64 and the chain
continues from the rounded value.

Parity pins for every function here are in tests/test_oracle_pins.py (brute
force in pure Python, finite differences, closed forms, special cases,
Table 1's count for the forward and for both backward products in their
partials form, the two 3D readings against each other and against the plain
layer, exhaustive bf16 round trip).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
from scipy.special import erf as _erf

MODE_1D_COL = "1d_col"
MODE_1D_ROW = "1d_row"
MODE_2D = "2d"
MODE_2P5D = "2.5d"
MODE_3D = "3d"

PASS_FWD, PASS_DX, PASS_DW = 0, 1, 2


# ----------------------------------------------------------------------------- bf16
def bf16_bits_to_f64(bits) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp64."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    with np.errstate(invalid="ignore"):       # NaN patterns widen to NaN
        return b.view(np.float32).astype(np.float64)


def round_to_bf16(x) -> np.ndarray:
    """Nearest bf16 (8 significant bits, fp32's exponent range), ties to even, taken
    directly from fp64; returned as fp64.  Finite inputs; overflow goes to +-inf."""
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)                      # |x| = m 2^e, m in [0.5, 1)
    # spacing of bf16 numbers around x: 2^(e-8) for normals, 2^-133 below 2^-126
    q = np.ldexp(1.0, np.maximum(e - 8, -133))
    y = np.rint(x / q) * q                  # rint rounds halves to even
    big = np.ldexp(255.0, 120)              # largest finite bf16 = (2 - 2^-7) 2^127
    return np.where(np.abs(y) > big, np.copysign(np.inf, x), y)


def f64_to_bf16_bits(x) -> np.ndarray:
    """bf16 bit patterns of values that are already representable (e.g. round_to_bf16 output)."""
    return (np.asarray(x, dtype=np.float64).astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# ----------------------------------------------------------------------------- GeLU
def gelu(a):
    a = np.asarray(a, dtype=np.float64)
    return 0.5 * a * (1.0 + _erf(a / np.sqrt(2.0)))


def dgelu(a):
    a = np.asarray(a, dtype=np.float64)
    cdf = 0.5 * (1.0 + _erf(a / np.sqrt(2.0)))
    pdf = np.exp(-0.5 * a * a) / np.sqrt(2.0 * np.pi)
    return cdf + a * pdf


# ----------------------------------------------------------------------------- full layer
def layer_fwd(X, W, b=None, act=True):
    """Unpartitioned layer: returns (A, Y)."""
    A = X @ W
    if b is not None:
        A = A + b[None, :]
    return A, (gelu(A) if act else A)


def layer_bwd(X, W, A, G, act=True):
    """Unpartitioned backward: returns (dA, dX, dW, db)."""
    dA = G * dgelu(A) if act else G
    return dA, dA @ W.T, X.T @ dA, dA.sum(axis=0)


# ----------------------------------------------------------------------------- partition map
@dataclass(frozen=True)
class Grid:
    """Rank grid.  1D: p = size, ri = rank.  2D: q, (ri, rj).  2.5D: q, d, (ri, rj, rk = depth).
    3D: p, (ri, rj, rk)."""
    mode: str
    q: int = 1
    d: int = 1
    p: int = 1
    ri: int = 0
    rj: int = 0
    rk: int = 0

    def n_ranks(self) -> int:
        return {MODE_1D_COL: self.p, MODE_1D_ROW: self.p, MODE_2D: self.q * self.q,
                MODE_2P5D: self.q * self.q * self.d, MODE_3D: self.p ** 3}[self.mode]


def chunk_counts(g: Grid):
    """(row chunks of X/Y/dA, col chunks of X = row chunks of W, col chunks of W/Y/dA/b)."""
    if g.mode == MODE_1D_COL:
        return 1, 1, g.p
    if g.mode == MODE_1D_ROW:
        return 1, g.p, 1
    if g.mode == MODE_2D:
        return g.q, g.q, g.q
    if g.mode == MODE_2P5D:
        return g.q * g.d, g.q, g.q
    if g.mode == MODE_3D:
        return g.p * g.p, g.p, g.p
    raise ValueError(g.mode)


def check_grid(g: Grid, M: int, H: int, F: int) -> None:
    """Admissible grids (the paper's GPU-count rule: any N for 1D, n^2, a n^2, n^3) and divisibility."""
    if min(g.q, g.d, g.p) < 1:
        raise ValueError("grid sizes must be >= 1")
    lim = {MODE_1D_COL: (g.p, 1, 1), MODE_1D_ROW: (g.p, 1, 1), MODE_2D: (g.q, g.q, 1),
           MODE_2P5D: (g.q, g.q, g.d), MODE_3D: (g.p, g.p, g.p)}[g.mode]
    for c, n in zip((g.ri, g.rj, g.rk), lim):
        if not 0 <= c < n:
            raise ValueError("rank coordinate out of range")
    rc, kc, cc = chunk_counts(g)
    if M % rc or H % kc or F % cc:
        raise ValueError("layer dims not divisible by the grid")


def block_map(g: Grid, pass_: int) -> dict:
    """Which blocks one rank multiplies, step by step, and which block it produces.

    Returns dict(a=[(row_chunk, col_chunk)...], b=[...], out=(row_chunk, col_chunk), partial=bool).
    fwd:  a indexes X chunks, b indexes W chunks, out indexes Y chunks (bias chunk = out col).
    dX:   a indexes dA chunks, b indexes W chunks (used transposed), out indexes dX (= X) chunks.
    dW:   a indexes X chunks (used transposed), b indexes dA chunks, out indexes dW (= W) chunks.
    """
    m = g.mode
    if m == MODE_1D_COL:
        r = g.ri
        if pass_ == PASS_FWD:
            return dict(a=[(0, 0)], b=[(0, r)], out=(0, r), partial=False)
        if pass_ == PASS_DX:
            return dict(a=[(0, r)], b=[(0, r)], out=(0, 0), partial=g.p > 1)
        return dict(a=[(0, 0)], b=[(0, r)], out=(0, r), partial=False)
    if m == MODE_1D_ROW:
        r = g.ri
        if pass_ == PASS_FWD:
            return dict(a=[(0, r)], b=[(r, 0)], out=(0, 0), partial=g.p > 1)
        if pass_ == PASS_DX:
            return dict(a=[(0, 0)], b=[(r, 0)], out=(0, r), partial=False)
        return dict(a=[(0, r)], b=[(0, 0)], out=(r, 0), partial=False)
    if m in (MODE_2D, MODE_2P5D):
        q, i, j = g.q, g.ri, g.rj
        lay = g.rk if m == MODE_2P5D else 0
        r = lay * q + i                               # this rank's row chunk of X / Y / dA
        if pass_ == PASS_FWD:
            return dict(a=[(r, k) for k in range(q)], b=[(k, j) for k in range(q)], out=(r, j), partial=False)
        if pass_ == PASS_DX:
            return dict(a=[(r, k) for k in range(q)], b=[(j, k) for k in range(q)], out=(r, j), partial=False)
        return dict(a=[(lay * q + k, i) for k in range(q)], b=[(lay * q + k, j) for k in range(q)],
                    out=(i, j), partial=(m == MODE_2P5D and g.d > 1))
    if m == MODE_3D:
        p, i, j, l = g.p, g.ri, g.rj, g.rk
        r = i * p + l
        if pass_ == PASS_FWD:
            return dict(a=[(r, c) for c in range(p)], b=[(c, j) for c in range(p)], out=(r, j), partial=False)
        if pass_ == PASS_DX:
            return dict(a=[(r, n) for n in range(p)], b=[(j, n) for n in range(p)], out=(r, j), partial=False)
        return dict(a=[(i * p + t, l) for t in range(p)], b=[(i * p + t, j) for t in range(p)],
                    out=(l, j), partial=p > 1)
    raise ValueError(m)


def chunk(T: np.ndarray, nr: int, nc: int, r: int, c: int) -> np.ndarray:
    """Chunk (r, c) of T cut into nr x nc equal chunks (a 1-D T is cut into nc pieces, r ignored)."""
    if T.ndim == 1:
        w = T.shape[0] // nc
        return T[c * w:(c + 1) * w]
    h, w = T.shape[0] // nr, T.shape[1] // nc
    return T[r * h:(r + 1) * h, c * w:(c + 1) * w]


def stored_elements(g: Grid, M: int, h: int) -> dict:
    """What one rank keeps of a model of two h x h linear layers on M tokens (the paper's range test,
    Section 4, Memory Efficiency), counted from the chunking rules of Section 2.2: every tensor the
    scheme partitions is stored as one chunk, a tensor it replicates is stored whole.  Returns the
    element counts {"narrow": ..., "wide": ...}: narrow = inputs, weights, biases, activations and
    activation gradients, wide = weight gradients and the partial sums a scheme leaves unreduced
    (the caller prices them, e.g. 2 and 4 bytes)."""
    check_grid(g, M, h, h)
    rc, kc, cc = chunk_counts(g)
    if g.mode in (MODE_1D_COL, MODE_1D_ROW):
        n = g.p
        # the first weight is cut by columns, the second by rows; what lies between them is cut by
        # columns, everything at the layer pair's two ends is whole (and the ends' results are partial sums)
        whole, cut = M * h, M * h // n
        narrow = whole            # X
        narrow += 3 * cut         # saved pre-activation, activation, its gradient
        narrow += whole           # upstream gradient of the pair's output
        narrow += 2 * (h * h // n) + h // n + h          # W1[:, r], W2[r, :], b1[r], b2
        wide = 2 * whole          # Y and dX, each a partial sum over the ranks
        wide += 2 * (h * h // n)  # the two weight gradients
        return {"narrow": narrow, "wide": wide}
    act = (M // rc) * (h // cc)   # every [M, h] tensor is stored as one chunk of the activation grid
    if g.mode == MODE_3D:
        w = (h // (g.p * g.p)) * (h // g.p)              # both matrices of a product are stored as [P/p^2, Q/p]
    else:
        w = (h // kc) * (h // cc)                        # 2D / 2.5D: one chunk of the q x q weight grid (on every depth layer)
    narrow = 7 * act              # X, A1, Z, Y, dY, dA1, dX
    narrow += 2 * w + 2 * (h // cc)                      # two weights, two bias chunks
    wide = 2 * w                  # two weight gradients
    return {"narrow": narrow, "wide": wide}


# ----------------------------------------------------------------------------- one rank's share from its blocks
def share_fwd(x_blocks, w_blocks, bias=None, act=True, rows=None):
    """C = sum_k X_k W_k (k upward), A = C + b, Y = GeLU(A).  Returns (A, Y); ``rows`` restricts
    the output rows (each needs only the same rows of every X_k)."""
    C = 0.0
    for Xk, Wk in zip(x_blocks, w_blocks):
        C = C + (Xk if rows is None else Xk[rows]) @ Wk
    A = C if bias is None else C + bias[None, :]
    return A, (gelu(A) if act else A)


def share_da(G_own, A_saved):
    """dA = bf16(G * GeLU'(A_saved)) for the rank's own block."""
    return round_to_bf16(G_own * dgelu(A_saved))


def share_dx(da_blocks, w_blocks, rows=None):
    """dX = sum_k dA_k W_k^T."""
    C = 0.0
    for Dk, Wk in zip(da_blocks, w_blocks):
        C = C + (Dk if rows is None else Dk[rows]) @ Wk.T
    return C


def share_dw(x_blocks, da_blocks, rows=None):
    """dW = sum_k X_k^T dA_k; ``rows`` restricts the rows of dW (columns of every X_k)."""
    C = 0.0
    for Xk, Dk in zip(x_blocks, da_blocks):
        C = C + (Xk if rows is None else Xk[:, rows]).T @ Dk
    return C


# ----------------------------------------------------------------------------- one rank's share from the full tensors
def rank_fwd(g: Grid, X, W, b=None, act=True, n_steps=None):
    """Rank g's forward share, cut out of the full tensors by the partition map.  Returns (A, Y)."""
    check_grid(g, X.shape[0], X.shape[1], W.shape[1])
    rc, kc, cc = chunk_counts(g)
    mp = block_map(g, PASS_FWD)
    s = len(mp["a"]) if n_steps is None else n_steps
    xs = [chunk(X, rc, kc, *ab) for ab in mp["a"][:s]]
    ws = [chunk(W, kc, cc, *bb) for bb in mp["b"][:s]]
    bj = None if b is None else chunk(b, 1, cc, 0, mp["out"][1])
    return share_fwd(xs, ws, bj, act)


def rank_dx(g: Grid, dA, W):
    check_grid(g, dA.shape[0], W.shape[0], W.shape[1])
    rc, kc, cc = chunk_counts(g)
    mp = block_map(g, PASS_DX)
    return share_dx([chunk(dA, rc, cc, *ab) for ab in mp["a"]], [chunk(W, kc, cc, *bb) for bb in mp["b"]])


def rank_dw(g: Grid, X, dA):
    check_grid(g, X.shape[0], X.shape[1], dA.shape[1])
    rc, kc, cc = chunk_counts(g)
    mp = block_map(g, PASS_DW)
    return share_dw([chunk(X, rc, kc, *ab) for ab in mp["a"]], [chunk(dA, rc, cc, *bb) for bb in mp["b"]])


def all_ranks(mode: str, q: int = 1, d: int = 1, p: int = 1):
    if mode in (MODE_1D_COL, MODE_1D_ROW):
        return [Grid(mode, p=p, ri=r) for r in range(p)]
    if mode == MODE_2D:
        return [Grid(mode, q=q, ri=i, rj=j) for i in range(q) for j in range(q)]
    if mode == MODE_2P5D:
        return [Grid(mode, q=q, d=d, ri=i, rj=j, rk=l) for l in range(d) for i in range(q) for j in range(q)]
    if mode == MODE_3D:
        return [Grid(mode, p=p, ri=i, rj=j, rk=l) for i in range(p) for j in range(p) for l in range(p)]
    raise ValueError(mode)


def assemble(ranks, pass_, blocks, shape):
    """Put every rank's block where the map says it goes; partial blocks are summed
    (that sum is what the omitted all-reduce would do)."""
    out = np.zeros(shape, dtype=np.float64)
    for g, blk in zip(ranks, blocks):
        rc, kc, cc = chunk_counts(g)
        nr, nc = {PASS_FWD: (rc, cc), PASS_DX: (rc, kc), PASS_DW: (kc, cc)}[pass_]
        r, c = block_map(g, pass_)["out"]
        h, w = shape[0] // nr, shape[1] // nc
        out[r * h:(r + 1) * h, c * w:(c + 1) * w] += blk
    return out


# ----------------------------------------------------------------------------- backward as partials for other owners (2D, 2.5D)
def partials_map(g: Grid, pass_: int) -> dict:
    """The other SUMMA form of the two backward products on a 2D / 2.5D grid: the rank's own dA
    block stays where it is, one block of the other operand arrives per step, and every step's
    product is an additive partial of a block that some rank of the same row (dX) or column (dW)
    group owns.  This is the form whose traffic the communication-volume table of Section 3.1
    counts for 2D and 2.5D: per product, (side - 1) blocks of the moving operand in and
    (side - 1) partial blocks out.

    Returns dict(own=(row, col) of the dA block, other=[block ids of the moving operand],
    out=[block ids the partials belong to]).
    dX: partial_k = dA[r, j] W[k, j]^T   belongs to dX[r, k]   (summed over j by the row group)
    dW: partial_k = X[r, k]^T dA[r, j]   belongs to dW[k, j]   (summed over r by the column group
                                                               and, in 2.5D, over the depth layers)
    """
    if g.mode not in (MODE_2D, MODE_2P5D):
        raise ValueError("partials form exists for 2D and 2.5D grids only")
    q, j = g.q, g.rj
    r = (g.rk if g.mode == MODE_2P5D else 0) * q + g.ri
    if pass_ == PASS_DX:
        return dict(own=(r, j), other=[(k, j) for k in range(q)], out=[(r, k) for k in range(q)])
    if pass_ == PASS_DW:
        return dict(own=(r, j), other=[(r, k) for k in range(q)], out=[(k, j) for k in range(q)])
    raise ValueError(pass_)


def rank_dx_partials(g: Grid, dA, W):
    """[(block id of dX, partial)] for rank g; the partials of one block id, summed over the ranks
    that emit it, are that block of dX = dA W^T."""
    check_grid(g, dA.shape[0], W.shape[0], W.shape[1])
    rc, kc, cc = chunk_counts(g)
    mp = partials_map(g, PASS_DX)
    own = chunk(dA, rc, cc, *mp["own"])
    return [(o, own @ chunk(W, kc, cc, *wb).T) for wb, o in zip(mp["other"], mp["out"])]


def rank_dw_partials(g: Grid, X, dA):
    check_grid(g, X.shape[0], X.shape[1], dA.shape[1])
    rc, kc, cc = chunk_counts(g)
    mp = partials_map(g, PASS_DW)
    own = chunk(dA, rc, cc, *mp["own"])
    return [(o, chunk(X, rc, kc, *xb).T @ own) for xb, o in zip(mp["other"], mp["out"])]


# ----------------------------------------------------------------------------- 3D at its gathered local shape
def gathered3d_map(g: Grid, pass_: int) -> dict:
    """3D with the operands as they are after the all-gathers: ONE local product per pass on
    slabs of shape [P/p, Q/p] (Section 2.2: the stored chunk is [P/p^2, Q/p]; gathering along
    one cube axis undoes the second split of the first dimension), whose result is a partial
    that a reduce-scatter along another axis would sum and split back into [P/p^2, .] chunks.
    Block ids are in units of the gathered slabs: M in p slabs, H in p, F in p.

    fwd: P = X[i, l] W[l, j]      partial of (X W)[i, j]   over l
    dX : P = dA[i, j] W[l, j]^T   partial of dX[i, l]      over j
    dW : P = X[i, l]^T dA[i, j]   partial of dW[l, j]      over i
    Row chunk l of the summed forward slab (i, j) is the block the owner-computes reading
    gives rank (i, j, l): row chunk i p + l of p^2.
    """
    if g.mode != MODE_3D:
        raise ValueError("3D grids only")
    i, j, l = g.ri, g.rj, g.rk
    if pass_ == PASS_FWD:
        return dict(a=(i, l), b=(l, j), out=(i, j))
    if pass_ == PASS_DX:
        return dict(a=(i, j), b=(l, j), out=(i, l))
    if pass_ == PASS_DW:
        return dict(a=(i, l), b=(i, j), out=(l, j))
    raise ValueError(pass_)


def rank3d_gathered(g: Grid, pass_: int, X=None, W=None, dA=None):
    """(block id, partial) of rank g's single gathered-shape product, cut from the full tensors."""
    p = g.p
    mp = gathered3d_map(g, pass_)
    if pass_ == PASS_FWD:
        check_grid(g, X.shape[0], X.shape[1], W.shape[1])
        return mp["out"], chunk(X, p, p, *mp["a"]) @ chunk(W, p, p, *mp["b"])
    if pass_ == PASS_DX:
        check_grid(g, dA.shape[0], W.shape[0], W.shape[1])
        return mp["out"], chunk(dA, p, p, *mp["a"]) @ chunk(W, p, p, *mp["b"]).T
    check_grid(g, X.shape[0], X.shape[1], dA.shape[1])
    return mp["out"], chunk(X, p, p, *mp["a"]).T @ chunk(dA, p, p, *mp["b"])


def bias_gelu(C, bias=None, act=True):
    """What follows the summation of forward partials: A = C + b, Y = GeLU(A).  Returns (A, Y)."""
    A = C if bias is None else C + bias[None, :]
    return A, (gelu(A) if act else A)


# ----------------------------------------------------------------------------- 1D MLP chain (Megatron feed-forward)
def mlp1d_fwd(X, W1_r, b1_r, W2_r, rows=None):
    """Rank r of size N: A = X W1[:, r] + b1[r]; Z = bf16(GeLU(A)); A_saved = bf16(A);
    Y_r = Z W2[r, :] (an fp64 partial; the sum over r is the layer output).
    Returns dict(A_saved, Z, Y)."""
    A, Zf = share_fwd([X], [W1_r], b1_r, True, rows)
    Z = round_to_bf16(Zf)
    return dict(A_saved=round_to_bf16(A), Z=Z, Y=Z @ W2_r)


def mlp1d_bwd(X, W1_r, W2_r, A_saved, Z, G, rows=None, w_rows=None):
    """dW2[r,:] = Z^T G;  dZ = G W2[r,:]^T;  dA = bf16(dZ * GeLU'(A_saved));
    dW1[:, r] = X^T dA;  dX_r = dA W1[:, r]^T (partial over r).
    ``rows`` restricts token rows of dZ/dA/dX outputs, ``w_rows`` the rows of dW1 and dW2;
    dW1 needs dA for every token, so dA is always formed in full."""
    dZ = G @ W2_r.T
    dA = round_to_bf16(dZ * dgelu(A_saved))
    sel = slice(None) if rows is None else rows
    out = dict(dZ=dZ[sel], dA=dA[sel], dX=dA[sel] @ W1_r.T)
    if w_rows is None:
        out["dW2"] = Z.T @ G
        out["dW1"] = X.T @ dA
    else:
        out["dW2"] = Z[:, w_rows].T @ G
        out["dW1"] = X[:, w_rows].T @ dA
    return out
