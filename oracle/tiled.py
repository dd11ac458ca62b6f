"""The GPT-2 block operations carried out tile by tile, fp64 (test infrastructure).

A tensor is cut along every axis into a grid of tiles (section 2: tiles and
tasks; section 5: splitting across all possible axes); each operation touches a
few tiles at a time in the order the paper gives:

  linear / attention products   products and sums of elementary tiles
  layer normalisation           (1) accumulate mean and variance tile by tile,
                                (2) normalise every tile, (3) scale and add bias
  softmax                       (1) per-tile maximum and denominator, merged
                                across the tiles of a column, (2) probabilities

A tile may be absent (None): it then stands for a block of structural zeros
(for scores: a block that the causal mask removes entirely), is never computed
and contributes nothing to a product.

Exists to pin tiling invariance of definition.py; not part of the product.
"""
from __future__ import annotations

import itertools
import math

import numpy as np

from . import definition as D

F64 = np.float64


class Tiled:
    """A tensor stored as a grid of separate tile arrays."""

    def __init__(self, shape, base):
        self.shape = tuple(int(x) for x in shape)
        self.base = tuple(int(min(b, n)) for b, n in zip(base, self.shape))
        self.grid = tuple(-(-n // b) for n, b in zip(self.shape, self.base))
        self.tiles = {}

    def indices(self):
        return itertools.product(*[range(g) for g in self.grid])

    def slices(self, idx):
        return tuple(slice(i * b, min(n, (i + 1) * b)) for i, b, n in zip(idx, self.base, self.shape))

    def tile_shape(self, idx):
        return tuple(s.stop - s.start for s in self.slices(idx))

    def start(self, idx):
        return tuple(i * b for i, b in zip(idx, self.base))

    @classmethod
    def from_array(cls, a, base, absent=None):
        a = np.asarray(a, F64)
        t = cls(a.shape, base)
        for idx in t.indices():
            t.tiles[idx] = None if (absent and absent(idx)) else a[t.slices(idx)].copy()
        return t

    @classmethod
    def zeros(cls, shape, base, absent=None):
        t = cls(shape, base)
        for idx in t.indices():
            t.tiles[idx] = None if (absent and absent(idx)) else np.zeros(t.tile_shape(idx), F64)
        return t

    def to_array(self):
        a = np.zeros(self.shape, F64)
        for idx in self.indices():
            if self.tiles[idx] is not None:
                a[self.slices(idx)] = self.tiles[idx]
        return a


# --------------------------------------------------------------------------
# products and sums of elementary tiles
# --------------------------------------------------------------------------
def gemm(alpha, opA, A, opB, B, beta, C, ncontract=1, nbatch=0):
    """Tile form of definition.contract: for every tile of C, walk the tiles
    along the contracted axes; the first product applies beta, the later ones
    accumulate."""
    na, nb_ = len(A.shape) - nbatch, len(B.shape) - nbatch
    if opA == "N":
        a_free, a_con = list(range(0, na - ncontract)), list(range(na - ncontract, na))
    else:
        a_con, a_free = list(range(0, ncontract)), list(range(ncontract, na))
    if opB == "N":
        b_con, b_free = list(range(0, ncontract)), list(range(ncontract, nb_))
    else:
        b_free, b_con = list(range(0, nb_ - ncontract)), list(range(nb_ - ncontract, nb_))
    for x, y in zip(a_con, b_con):
        assert A.shape[x] == B.shape[y] and A.base[x] == B.base[y], "contracted axes tiled differently"
    con_grid = [A.grid[x] for x in a_con]
    for cidx in C.indices():
        if C.tiles[cidx] is None:
            continue
        fa = cidx[:len(a_free)]
        fb = cidx[len(a_free):len(a_free) + len(b_free)]
        bt = cidx[len(a_free) + len(b_free):]
        first = True
        for l in itertools.product(*[range(g) for g in con_grid]):
            aidx = [None] * len(A.shape)
            bidx = [None] * len(B.shape)
            for ax, v in zip(a_free, fa):
                aidx[ax] = v
            for ax, v in zip(a_con, l):
                aidx[ax] = v
            for ax, v in zip(b_free, fb):
                bidx[ax] = v
            for ax, v in zip(b_con, l):
                bidx[ax] = v
            for n_, v in enumerate(bt):
                aidx[na + n_] = v
                bidx[nb_ + n_] = v
            At, Bt = A.tiles[tuple(aidx)], B.tiles[tuple(bidx)]
            if At is None or Bt is None:
                continue
            C.tiles[cidx] = D.contract(alpha, opA, At, opB, Bt, beta if first else 1.0,
                                       C.tiles[cidx], ncontract, nbatch)
            first = False
        if first:
            C.tiles[cidx] = beta * C.tiles[cidx] if beta != 0.0 else np.zeros_like(C.tiles[cidx])
    return C


def bias_add(Y, b):
    for idx in Y.indices():
        Y.tiles[idx] = D.bias_add(Y.tiles[idx], b.tiles[(idx[0],)])
    return Y


def bias_grad(dY, db):
    """db tile = sum over every dY tile of the same row range, tile after tile."""
    seen = set()
    for idx in dY.indices():
        part = D.bias_grad(dY.tiles[idx])
        key = (idx[0],)
        db.tiles[key] = part if key not in seen else db.tiles[key] + part
        seen.add(key)
    return db


def add(alpha, X, beta, Y):
    for idx in Y.indices():
        Y.tiles[idx] = alpha * X.tiles[idx] + beta * Y.tiles[idx]
    return Y


def elementwise(fn, *tensors):
    out = Tiled(tensors[0].shape, tensors[0].base)
    for idx in out.indices():
        out.tiles[idx] = fn(*[t.tiles[idx] for t in tensors])
    return out


# --------------------------------------------------------------------------
# layer normalisation in three tile steps
# --------------------------------------------------------------------------
def layernorm_fwd(X, gamma, beta, eps):
    """X tiled [e, s, b]; gamma, beta tiled [e].  Returns Y (tiled like X) and
    stats tiled [2, s, b] = (mean, 1/sqrt(var + eps))."""
    N_e = X.shape[0]
    stats = Tiled.zeros((2,) + X.shape[1:], (2,) + X.base[1:])
    count = {}
    # step 1: every tile adds its mean and variance to the running statistics
    for idx in X.indices():
        t = X.tiles[idx]
        n_t = t.shape[0]
        mean_t = t.mean(axis=0)
        m2_t = ((t - mean_t) ** 2).sum(axis=0)
        sidx = (0,) + idx[1:]
        n_a = count.get(sidx, 0)
        st = stats.tiles[sidx]
        delta = mean_t - st[0]
        n = n_a + n_t
        st[0] = st[0] + delta * (n_t / n)
        st[1] = st[1] + m2_t + delta * delta * (n_a * n_t / n)
        count[sidx] = n
    for sidx in stats.indices():
        assert count[sidx] == N_e
        st = stats.tiles[sidx]
        st[1] = 1.0 / np.sqrt(st[1] / N_e + eps)
    Y = Tiled(X.shape, X.base)
    for idx in X.indices():
        st = stats.tiles[(0,) + idx[1:]]
        # step 2: normalise the tile
        xhat = (X.tiles[idx] - st[0]) * st[1]
        # step 3: scale and add the bias
        g = gamma.tiles[(idx[0],)].reshape(-1, 1, 1)
        bt = beta.tiles[(idx[0],)].reshape(-1, 1, 1)
        Y.tiles[idx] = g * xhat + bt
    return Y, stats


def layernorm_bwd(X, gamma, stats, dY):
    N_e = X.shape[0]
    sums = Tiled.zeros((2,) + X.shape[1:], (2,) + X.base[1:])
    dgamma = Tiled.zeros(gamma.shape, gamma.base)
    dbeta = Tiled.zeros(gamma.shape, gamma.base)
    # step 1: per-token sums of g and g*xhat over the embedding tiles,
    # per-feature sums of dy*xhat and dy over the token tiles
    for idx in X.indices():
        st = stats.tiles[(0,) + idx[1:]]
        xhat = (X.tiles[idx] - st[0]) * st[1]
        dy = dY.tiles[idx]
        g = dy * gamma.tiles[(idx[0],)].reshape(-1, 1, 1)
        sm = sums.tiles[(0,) + idx[1:]]
        sm[0] += g.sum(axis=0)
        sm[1] += (g * xhat).sum(axis=0)
        dgamma.tiles[(idx[0],)] += (dy * xhat).sum(axis=(1, 2))
        dbeta.tiles[(idx[0],)] += dy.sum(axis=(1, 2))
    # step 2: the input gradient of every tile
    dX = Tiled(X.shape, X.base)
    for idx in X.indices():
        st = stats.tiles[(0,) + idx[1:]]
        sm = sums.tiles[(0,) + idx[1:]]
        xhat = (X.tiles[idx] - st[0]) * st[1]
        g = dY.tiles[idx] * gamma.tiles[(idx[0],)].reshape(-1, 1, 1)
        dX.tiles[idx] = st[1] * (g - sm[0] / N_e - xhat * (sm[1] / N_e))
    return dX, dgamma, dbeta


# --------------------------------------------------------------------------
# softmax in two tile subroutines
# --------------------------------------------------------------------------
def softmax_fwd(A, causal):
    """A tiled [k, q, ...]; softmax over k.  In place; returns (A, stats) with
    stats tiled [2, q, ...] = (column maximum, sum of shifted exponentials)."""
    stats = Tiled((2,) + A.shape[1:], (2,) + A.base[1:])
    for sidx in stats.indices():
        st = np.zeros(stats.tile_shape(sidx), F64)
        st[0] = -np.inf
        stats.tiles[sidx] = st
    # subroutine 1: maximum and denominator per tile, merged into the column's
    for idx in A.indices():
        t = A.tiles[idx]
        if t is None:
            continue
        if causal:
            k0, q0 = A.start(idx)[0], A.start(idx)[1]
            vis = (k0 + np.arange(t.shape[0]))[:, None] <= (q0 + np.arange(t.shape[1]))[None, :]
            t = np.where(vis.reshape(vis.shape + (1,) * (t.ndim - 2)), t, -np.inf)
        m_t = t.max(axis=0)
        safe = np.where(np.isfinite(m_t), m_t, 0.0)
        d_t = np.exp(t - safe).sum(axis=0)          # 0 where the whole tile column is masked
        st = stats.tiles[(0,) + idx[1:]]
        m_new = np.maximum(st[0], m_t)
        ref = np.where(np.isfinite(m_new), m_new, 0.0)
        st[1] = st[1] * np.exp(np.where(np.isfinite(st[0]), st[0] - ref, -np.inf)) \
            + d_t * np.exp(np.where(np.isfinite(m_t), m_t - ref, -np.inf))
        st[0] = m_new
    # subroutine 2: probabilities of every tile from the merged statistics
    for idx in A.indices():
        t = A.tiles[idx]
        if t is None:
            continue
        if causal:
            k0, q0 = A.start(idx)[0], A.start(idx)[1]
            vis = (k0 + np.arange(t.shape[0]))[:, None] <= (q0 + np.arange(t.shape[1]))[None, :]
            t = np.where(vis.reshape(vis.shape + (1,) * (t.ndim - 2)), t, -np.inf)
        st = stats.tiles[(0,) + idx[1:]]
        A.tiles[idx] = np.exp(t - st[0]) / st[1]
    return A, stats


def softmax_bwd(P, dP):
    """In place on dP: dA = P o (dP - sum_k P o dP), the sum gathered tile by tile."""
    dots = Tiled.zeros((1,) + P.shape[1:], (1,) + P.base[1:])
    for idx in P.indices():
        if P.tiles[idx] is None:
            continue
        dots.tiles[(0,) + idx[1:]][0] += (P.tiles[idx] * dP.tiles[idx]).sum(axis=0)
    for idx in P.indices():
        if P.tiles[idx] is None:
            continue
        dP.tiles[idx] = P.tiles[idx] * (dP.tiles[idx] - dots.tiles[(0,) + idx[1:]][0])
    return dP


# --------------------------------------------------------------------------
# attention without the stored scores: the SoftMax subroutines' running column
# statistics carried along the key tiles (section 3, SoftMax and attention layer)
# --------------------------------------------------------------------------
def attention_fwd_online(Q, K, V, key_tile, causal=True):
    """Q, K, V: arrays [h, N_s, N_b, N_h].  Walks the keys `key_tile` at a time; after
    each tile the running maximum m, the running sum of shifted exponentials d and
    the unnormalised result are those of the keys seen so far.  Returns
    (B, m, d) with B[i, q, b, j], m and d [q, b, j]."""
    Q, K, V = (np.asarray(x, F64) for x in (Q, K, V))
    h, N_s, N_b, N_h = Q.shape
    sc = 1.0 / np.sqrt(h)
    m = np.full((N_s, N_b, N_h), -np.inf)
    d = np.zeros((N_s, N_b, N_h))
    acc = np.zeros((h, N_s, N_b, N_h))
    for k0 in range(0, N_s, key_tile):
        k1 = min(N_s, k0 + key_tile)
        A = sc * np.einsum("ikbj,iqbj->kqbj", K[:, k0:k1], Q)             # scores of this key tile
        if causal:
            vis = (k0 + np.arange(k1 - k0))[:, None] <= np.arange(N_s)[None, :]
            A = np.where(vis[:, :, None, None], A, -np.inf)
        m_t = A.max(axis=0)
        m_new = np.maximum(m, m_t)
        ref = np.where(np.isfinite(m_new), m_new, 0.0)                     # columns that have seen no key yet
        E = np.exp(A - ref)                                                # masked entries: exp(-inf) = 0
        alpha = np.exp(np.where(np.isfinite(m), m - ref, -np.inf))         # rescales what earlier tiles left
        d = d * alpha + E.sum(axis=0)
        acc = acc * alpha + np.einsum("ikbj,kqbj->iqbj", V[:, k0:k1], E)
        m = m_new
    return acc / d, m, d


def attention_bwd_recompute(Q, K, V, B, m, d, dB, query_tile, causal=True):
    """The adjoint from (Q, K, V, B, running statistics, dB), the probabilities
    recomputed query tile by query tile: P = exp(A - m) / d,
    D[q] = sum_i dB[i, q] B[i, q], dA = P o (V^T dB - D)."""
    Q, K, V, B, dB = (np.asarray(x, F64) for x in (Q, K, V, B, dB))
    h, N_s, N_b, N_h = Q.shape
    sc = 1.0 / np.sqrt(h)
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    Dq = (dB * B).sum(axis=0)
    for q0 in range(0, N_s, query_tile):
        q1 = min(N_s, q0 + query_tile)
        A = sc * np.einsum("ikbj,iqbj->kqbj", K, Q[:, q0:q1])
        if causal:
            vis = np.arange(N_s)[:, None] <= (q0 + np.arange(q1 - q0))[None, :]
            A = np.where(vis[:, :, None, None], A, -np.inf)
        P = np.exp(A - m[q0:q1]) / d[q0:q1]
        dV += np.einsum("iqbj,kqbj->ikbj", dB[:, q0:q1], P)
        dP = np.einsum("ikbj,iqbj->kqbj", V, dB[:, q0:q1])
        dA = P * (dP - Dq[q0:q1])
        dQ[:, q0:q1] = sc * np.einsum("ikbj,kqbj->iqbj", K, dA)
        dK += sc * np.einsum("iqbj,kqbj->ikbj", Q[:, q0:q1], dA)
    return dQ, dK, dV


# --------------------------------------------------------------------------
# head split / merge: pure data movement between two tilings
# --------------------------------------------------------------------------
def split_heads(Z, N_h, n_parts, base4):
    return [Tiled.from_array(p, base4) for p in D.split_heads(Z.to_array(), N_h, n_parts)]


def merge_heads(parts, base3):
    return Tiled.from_array(D.merge_heads([p.to_array() for p in parts]), base3)


# --------------------------------------------------------------------------
# optimiser: the update acts on every tile independently
# --------------------------------------------------------------------------
def adam_step(p, g, m, v, t, **kw):
    for idx in p.indices():
        p.tiles[idx], m.tiles[idx], v.tiles[idx] = D.adam_step(
            p.tiles[idx], g.tiles[idx], m.tiles[idx], v.tiles[idx], t, **kw)
    return p, m, v


# --------------------------------------------------------------------------
# the block, tile by tile
# --------------------------------------------------------------------------
def _linear_fwd(W, X, b):
    Y = Tiled.zeros((W.shape[0],) + X.shape[1:], (W.base[0],) + X.base[1:])
    gemm(1.0, "N", W, "N", X, 0.0, Y, 1, 0)
    return bias_add(Y, b)


def _linear_bwd(W, X, dY):
    dX = Tiled.zeros(X.shape, X.base)
    gemm(1.0, "T", W, "N", dY, 0.0, dX, 1, 0)
    dW = Tiled.zeros(W.shape, W.base)
    gemm(1.0, "N", dY, "T", X, 0.0, dW, 2, 0)
    db = Tiled.zeros((W.shape[0],), (W.base[0],))
    bias_grad(dY, db)
    return dX, dW, db


def block_forward(p, X, N_h, bt, eps=1e-5, gelu_variant="tanh", causal=True):
    """p: dict name -> Tiled parameter; X: Tiled [e, s, b]; bt: base tile extents
    with keys e, e3, m, s, b, j, i (embedding, 3x embedding, MLP, sequence,
    batch, head count, head size)."""
    c = {"X": X}
    h = X.shape[0] // N_h
    N_s, N_b = X.shape[1], X.shape[2]
    c["X1"], c["stats1"] = layernorm_fwd(X, p["gamma1"], p["beta1"], eps)
    QKV = _linear_fwd(p["W_qkv"], c["X1"], p["b_qkv"])
    base4 = (bt["i"], bt["s"], bt["b"], bt["j"])
    c["Q"], c["K"], c["V"] = split_heads(QKV, N_h, 3, base4)
    sbase = (bt["s"], bt["s"], bt["b"], bt["j"])
    if causal:
        def absent(idx):
            return idx[0] * sbase[0] > min(N_s, (idx[1] + 1) * sbase[1]) - 1
    else:
        absent = None
    A = Tiled.zeros((N_s, N_s, N_b, N_h), sbase, absent)
    gemm(1.0 / math.sqrt(h), "T", c["K"], "N", c["Q"], 0.0, A, 1, 2)
    c["P"], _ = softmax_fwd(A, causal)
    Bh = Tiled.zeros(c["Q"].shape, base4)
    gemm(1.0, "N", c["V"], "N", c["P"], 0.0, Bh, 1, 2)
    c["Bm"] = merge_heads([Bh], X.base)
    Y = _linear_fwd(p["W_o"], c["Bm"], p["b_o"])
    c["X2"] = add(1.0, X, 1.0, Y)
    c["X3"], c["stats2"] = layernorm_fwd(c["X2"], p["gamma2"], p["beta2"], eps)
    c["H1"] = _linear_fwd(p["W_1"], c["X3"], p["b_1"])
    c["G"] = elementwise(lambda x: D.gelu(x, gelu_variant), c["H1"])
    H2 = _linear_fwd(p["W_2"], c["G"], p["b_2"])
    Out = add(1.0, c["X2"], 1.0, H2)
    return Out, c


def block_backward(p, c, dOut, N_h, bt, gelu_variant="tanh"):
    g = {}
    h = dOut.shape[0] // N_h
    dG, g["W_2"], g["b_2"] = _linear_bwd(p["W_2"], c["G"], dOut)
    dH1 = elementwise(lambda d, x: d * D.gelu_grad(x, gelu_variant), dG, c["H1"])
    dX3, g["W_1"], g["b_1"] = _linear_bwd(p["W_1"], c["X3"], dH1)
    d2, g["gamma2"], g["beta2"] = layernorm_bwd(c["X2"], p["gamma2"], c["stats2"], dX3)
    dX2 = add(1.0, dOut, 1.0, d2)
    dBm, g["W_o"], g["b_o"] = _linear_bwd(p["W_o"], c["Bm"], dX2)
    base4 = c["Q"].base
    (dB,) = split_heads(dBm, N_h, 1, base4)
    P = c["P"]
    absent = (lambda idx: P.tiles[idx] is None)
    dV = Tiled.zeros(c["V"].shape, base4)
    gemm(1.0, "N", dB, "T", P, 0.0, dV, 1, 2)
    dP = Tiled.zeros(P.shape, P.base, absent)
    gemm(1.0, "T", c["V"], "N", dB, 0.0, dP, 1, 2)
    dA = softmax_bwd(P, dP)
    sc = 1.0 / math.sqrt(h)
    dQ = Tiled.zeros(c["Q"].shape, base4)
    gemm(sc, "N", c["K"], "N", dA, 0.0, dQ, 1, 2)
    dK = Tiled.zeros(c["K"].shape, base4)
    gemm(sc, "N", c["Q"], "T", dA, 0.0, dK, 1, 2)
    dQKV = merge_heads([dQ, dK, dV], (p["W_qkv"].base[0],) + dOut.base[1:])
    dX1, g["W_qkv"], g["b_qkv"] = _linear_bwd(p["W_qkv"], c["X1"], dQKV)
    d1, g["gamma1"], g["beta1"] = layernorm_bwd(c["X"], p["gamma1"], c["stats1"], dX1)
    dX = add(1.0, dX2, 1.0, d1)
    return dX, g
