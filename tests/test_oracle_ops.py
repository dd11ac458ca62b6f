"""Pins for oracle/definition.py that do not go through the oracle itself:
brute force on tiny inputs, closed forms, invariants, finite differences and
independent library routines (scipy, CPU torch in float64)."""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import definition as D

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(7)


# ------------------------------------------------------------------ contraction
def _brute(alpha, opA, A, opB, B, beta, C):
    """C[m,n,(b)] by explicit loops; A m x k or k x m, B k x n or n x k."""
    if A.ndim == 2:
        A, B, C = A[..., None], B[..., None], C[..., None]
        squeeze = True
    else:
        squeeze = False
    m = A.shape[0] if opA == "N" else A.shape[1]
    k = A.shape[1] if opA == "N" else A.shape[0]
    n = B.shape[1] if opB == "N" else B.shape[0]
    out = np.zeros((m, n, A.shape[2]))
    for b in range(A.shape[2]):
        for i in range(m):
            for j in range(n):
                s = 0.0
                for l in range(k):
                    a = A[i, l, b] if opA == "N" else A[l, i, b]
                    bb = B[l, j, b] if opB == "N" else B[j, l, b]
                    s += a * bb
                out[i, j, b] = alpha * s + beta * C[i, j, b]
    return out[..., 0] if squeeze else out


@pytest.mark.parametrize("opA,opB", list(itertools.product("NT", "NT")))
@pytest.mark.parametrize("batch", [0, 3])
def test_matmul2d_brute_force(opA, opB, batch):
    m, n, k = 5, 4, 7
    bs = (batch,) if batch else ()
    A = rng.standard_normal(((m, k) if opA == "N" else (k, m)) + bs)
    B = rng.standard_normal(((k, n) if opB == "N" else (n, k)) + bs)
    C = rng.standard_normal((m, n) + bs)
    got = D.matmul2d(0.7, opA, A, opB, B, -1.3, C)
    np.testing.assert_allclose(got, _brute(0.7, opA, A, opB, B, -1.3, C), rtol=1e-13, atol=1e-13)


def test_contract_two_axes_brute_force():
    # dW[d, e] = sum_{s, b} dY[d, s, b] X[e, s, b]
    dY = rng.standard_normal((3, 4, 2))
    X = rng.standard_normal((5, 4, 2))
    got = D.contract(1.0, "N", dY, "T", X, 0.0, None, 2, 0)
    ref = np.zeros((3, 5))
    for d in range(3):
        for e in range(5):
            for s in range(4):
                for b in range(2):
                    ref[d, e] += dY[d, s, b] * X[e, s, b]
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)


def test_contract_batched_attention_shapes():
    # A[k, q, b, j] = sum_i K[i, k, b, j] Q[i, q, b, j]
    K = rng.standard_normal((3, 4, 2, 2))
    Q = rng.standard_normal((3, 5, 2, 2))
    got = D.contract(1.0, "T", K, "N", Q, 0.0, None, 1, 2)
    ref = np.zeros((4, 5, 2, 2))
    for k, q, b, j, i in itertools.product(range(4), range(5), range(2), range(2), range(3)):
        ref[k, q, b, j] += K[i, k, b, j] * Q[i, q, b, j]
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)


def test_contract_identities():
    A = rng.standard_normal((6, 6))
    I = np.eye(6)
    np.testing.assert_allclose(D.matmul2d(1.0, "N", A, "N", I, 0.0, None), A)
    np.testing.assert_allclose(D.matmul2d(1.0, "T", A, "N", I, 0.0, None), A.T)
    np.testing.assert_allclose(D.matmul2d(1.0, "N", I, "T", A, 0.0, None), A.T)
    B = rng.standard_normal((6, 3))
    C0 = rng.standard_normal((6, 3))
    one = D.matmul2d(1.0, "N", A, "N", B, 0.0, None)
    acc = D.matmul2d(1.0, "N", A, "N", B, 1.0, C0)
    np.testing.assert_allclose(acc, one + C0, rtol=1e-13)


# ------------------------------------------------------------------ linear
def test_linear_fwd_brute_force_and_bwd_fd():
    W = rng.standard_normal((4, 3))
    X = rng.standard_normal((3, 5, 2))
    b = rng.standard_normal(4)
    Y = D.linear_fwd(W, X, b)
    for d, s, bb in itertools.product(range(4), range(5), range(2)):
        assert abs(Y[d, s, bb] - (sum(W[d, e] * X[e, s, bb] for e in range(3)) + b[d])) < 1e-13
    dY = rng.standard_normal(Y.shape)
    dX, dW, db = D.linear_bwd(W, X, dY)
    eps = 1e-6
    for (arr, grad) in ((W, dW), (X, dX), (b, db)):
        v = rng.standard_normal(arr.shape)
        arr += eps * v
        lp = (D.linear_fwd(W, X, b) * dY).sum()
        arr -= 2 * eps * v
        lm = (D.linear_fwd(W, X, b) * dY).sum()
        arr += eps * v
        assert abs((lp - lm) / (2 * eps) - (grad * v).sum()) < 1e-7 * (1 + abs((grad * v).sum()))
    np.testing.assert_allclose(D.bias_grad(dY), dY.sum(axis=(1, 2)))


# ------------------------------------------------------------------ GELU
@pytest.mark.parametrize("variant", ["tanh", "erf"])
def test_gelu_identities_and_library(variant):
    x = np.linspace(-6, 6, 241)
    y = D.gelu(x, variant)
    assert D.gelu(np.array([0.0]), variant)[0] == 0.0
    np.testing.assert_allclose(y - D.gelu(-x, variant), x, atol=1e-14)      # gelu(x) - gelu(-x) = x
    assert abs(D.gelu(np.array([30.0]), variant)[0] - 30.0) < 1e-12
    assert abs(D.gelu(np.array([-30.0]), variant)[0]) < 1e-12
    ref = torch.nn.functional.gelu(torch.from_numpy(x), approximate="tanh" if variant == "tanh" else "none")
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-13, atol=1e-15)
    e = 1e-6
    fd = (D.gelu(x + e, variant) - D.gelu(x - e, variant)) / (2 * e)
    np.testing.assert_allclose(D.gelu_grad(x, variant), fd, atol=1e-8)


def test_gelu_tanh_value_by_hand():
    # x = 1: 0.5 * (1 + tanh(sqrt(2/pi) * 1.044715))
    want = 0.5 * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * 1.044715))
    assert abs(D.gelu(np.array([1.0]))[0] - want) < 1e-15
    assert abs(want - 0.841191990608276) < 1e-12


# ------------------------------------------------------------------ layer norm
def test_layernorm_closed_forms():
    eps = 1e-5
    X = rng.standard_normal((16, 3, 2)) * 3 + 1.5
    ones, zeros = np.ones(16), np.zeros(16)
    Y, mean, rstd = D.layernorm_fwd(X, ones, zeros, eps)
    var = X.var(axis=0)
    np.testing.assert_allclose(Y.mean(axis=0), 0, atol=1e-14)
    np.testing.assert_allclose(Y.var(axis=0), var / (var + eps), rtol=1e-12)
    np.testing.assert_allclose(mean, X.mean(axis=0))
    np.testing.assert_allclose(rstd, 1 / np.sqrt(var + eps))
    # adding a per-token constant changes nothing
    Y2, _, _ = D.layernorm_fwd(X + rng.standard_normal((1, 3, 2)), ones, zeros, eps)
    np.testing.assert_allclose(Y2, Y, atol=1e-12)
    # N_e = 2: x = (a, b) -> +-1 / sqrt(1 + eps / sigma^2), sigma^2 = (a - b)^2 / 4
    a, b = 3.0, -1.0
    Y3, _, _ = D.layernorm_fwd(np.array([a, b]).reshape(2, 1, 1), np.ones(2), np.zeros(2), eps)
    s2 = (a - b) ** 2 / 4
    np.testing.assert_allclose(Y3.ravel(), [1 / math.sqrt(1 + eps / s2), -1 / math.sqrt(1 + eps / s2)], rtol=1e-14)


def test_layernorm_vs_torch_fwd_bwd():
    eps = 1e-5
    X = rng.standard_normal((12, 4, 3))
    g = 1 + 0.1 * rng.standard_normal(12)
    b = 0.1 * rng.standard_normal(12)
    dY = rng.standard_normal(X.shape)
    Y, mean, rstd = D.layernorm_fwd(X, g, b, eps)
    dX, dg, db = D.layernorm_bwd(X, g, mean, rstd, dY)
    xt = torch.from_numpy(X.transpose(2, 1, 0).copy()).requires_grad_()
    gt = torch.from_numpy(g).requires_grad_()
    bt = torch.from_numpy(b).requires_grad_()
    yt = torch.nn.functional.layer_norm(xt, (12,), gt, bt, eps)
    yt.backward(torch.from_numpy(dY.transpose(2, 1, 0).copy()))
    np.testing.assert_allclose(Y, yt.detach().numpy().transpose(2, 1, 0), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dX, xt.grad.numpy().transpose(2, 1, 0), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dg, gt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ softmax
def test_softmax_golden_closed_form():
    with open(os.path.join(GOLD, "softmax_closed_form.txt")) as f:
        want = [float(v) for v in [l for l in f if not l.startswith("#")][0].split()]
    t = np.log(np.arange(1.0, 5.0)).reshape(4, 1)
    P, tmax, den = D.softmax_fwd(t)
    np.testing.assert_allclose(P.ravel(), want, rtol=1e-14)
    assert abs(tmax[0] - math.log(4)) < 1e-15 and abs(den[0] - 10 / 4) < 1e-14
    # causal: 4 keys x 4 queries with the same logits in every column
    Pc, _, _ = D.softmax_fwd(np.repeat(t, 4, axis=1), causal=True)
    for q in range(4):
        tot = (q + 1) * (q + 2) / 2
        for k in range(4):
            assert abs(Pc[k, q] - ((k + 1) / tot if k <= q else 0.0)) < 1e-14


def test_softmax_invariants_and_library():
    A = rng.standard_normal((9, 9, 2, 3)) * 4
    P, _, _ = D.softmax_fwd(A)
    np.testing.assert_allclose(P.sum(axis=0), 1.0, atol=1e-12)
    np.testing.assert_allclose(P, scipy.special.softmax(A, axis=0), rtol=1e-12)
    P2, _, _ = D.softmax_fwd(A + 1000.0)        # shift invariance: no overflow, same result
    np.testing.assert_allclose(P2, P, rtol=1e-10)
    Pc, _, _ = D.softmax_fwd(np.full((5, 3), 2.5))
    np.testing.assert_allclose(Pc, 0.2)
    # causal structure
    Pm, _, _ = D.softmax_fwd(A, causal=True)
    np.testing.assert_allclose(Pm.sum(axis=0), 1.0, atol=1e-12)
    for q in range(9):
        assert np.all(Pm[q + 1:, q] == 0.0) and np.all(Pm[:q + 1, q] > 0.0)
    assert np.all(Pm[0, 0] == 1.0)
    for q in range(9):          # column q = plain softmax of its first q+1 keys
        np.testing.assert_allclose(Pm[:q + 1, q], scipy.special.softmax(A[:q + 1, q], axis=0), rtol=1e-12)


def test_softmax_bwd_fd():
    A = rng.standard_normal((6, 6, 2))
    dP = rng.standard_normal(A.shape)
    P, _, _ = D.softmax_fwd(A, causal=True)
    dA = D.softmax_bwd(P, dP)
    v = rng.standard_normal(A.shape)
    e = 1e-6
    lp = (D.softmax_fwd(A + e * v, True)[0] * dP).sum()
    lm = (D.softmax_fwd(A - e * v, True)[0] * dP).sum()
    assert abs((lp - lm) / (2 * e) - (dA * v).sum()) < 1e-8
    for q in range(6):
        assert np.all(dA[q + 1:, q] == 0.0)


# ------------------------------------------------------------------ attention
def _qkv(h=4, N_s=7, N_b=2, N_h=3):
    return [rng.standard_normal((h, N_s, N_b, N_h)) for _ in range(3)]


def test_split_merge_heads_index_map():
    N_h, h, N_s, N_b = 3, 2, 4, 2
    Z = rng.standard_normal((3 * N_h * h, N_s, N_b))
    parts = D.split_heads(Z, N_h, 3)
    for w, j, i, s, b in itertools.product(range(3), range(N_h), range(h), range(N_s), range(N_b)):
        assert parts[w][i, s, b, j] == Z[(w * N_h + j) * h + i, s, b]
    np.testing.assert_array_equal(D.merge_heads(parts), Z)


def test_attention_brute_force():
    Q, K, V = _qkv(h=3, N_s=4, N_b=1, N_h=2)
    Bo, P = D.attention_fwd(Q, K, V, causal=True)
    for j in range(2):
        for q in range(4):
            logits = [sum(K[i, k, 0, j] * Q[i, q, 0, j] for i in range(3)) / math.sqrt(3) for k in range(q + 1)]
            mx = max(logits)
            w = [math.exp(l - mx) for l in logits]
            for i in range(3):
                want = sum(w[k] * V[i, k, 0, j] for k in range(q + 1)) / sum(w)
                assert abs(Bo[i, q, 0, j] - want) < 1e-13


def test_attention_properties():
    Q, K, V = _qkv()
    Bo, P = D.attention_fwd(Q, K, V, causal=True)
    # causality: perturbing positions > s leaves outputs at <= s unchanged
    Q2, K2, V2 = Q.copy(), K.copy(), V.copy()
    for T in (Q2, K2, V2):
        T[:, 4:] += rng.standard_normal(T[:, 4:].shape)
    Bo2, _ = D.attention_fwd(Q2, K2, V2, causal=True)
    np.testing.assert_array_equal(Bo2[:, :4], Bo[:, :4])
    assert not np.allclose(Bo2[:, 4:], Bo[:, 4:])
    # batch independence and head permutation equivariance
    Bo3, _ = D.attention_fwd(Q[:, :, :1], K[:, :, :1], V[:, :, :1], causal=True)
    np.testing.assert_allclose(Bo3, Bo[:, :, :1], rtol=1e-13)
    perm = [2, 0, 1]
    Bo4, _ = D.attention_fwd(Q[..., perm], K[..., perm], V[..., perm], causal=True)
    np.testing.assert_allclose(Bo4, Bo[..., perm], rtol=1e-13)
    # one position: P = 1, B = V
    Bo5, P5 = D.attention_fwd(Q[:, :1], K[:, :1], V[:, :1], causal=True)
    np.testing.assert_array_equal(P5, np.ones_like(P5))
    np.testing.assert_allclose(Bo5, V[:, :1])


def test_attention_vs_torch_sdpa():
    Q, K, V = _qkv(h=8, N_s=6, N_b=2, N_h=2)
    Bo, _ = D.attention_fwd(Q, K, V, causal=True)
    tq, tk, tv = [torch.from_numpy(T.transpose(2, 3, 1, 0).copy()) for T in (Q, K, V)]   # [b, j, s, i]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    np.testing.assert_allclose(Bo, ref.numpy().transpose(3, 2, 0, 1), rtol=1e-11, atol=1e-13)


def test_attention_bwd_finite_differences_and_torch():
    """The attention adjoint on its own: central differences of sum(B o G), and autograd of the library routine."""
    Q, K, V = _qkv(h=5, N_s=6, N_b=2, N_h=2)
    G = rng.standard_normal(Q.shape)
    Bo, P = D.attention_fwd(Q, K, V, causal=True)
    dQ, dK, dV = D.attention_bwd(Q, K, V, P, G)
    eps = 1e-6
    for T, dT in ((Q, dQ), (K, dK), (V, dV)):
        for _ in range(6):
            idx = tuple(int(rng.integers(0, n)) for n in T.shape)
            Tp, Tm = T.copy(), T.copy()
            Tp[idx] += eps
            Tm[idx] -= eps
            args_p = [Tp if X is T else X for X in (Q, K, V)]
            args_m = [Tm if X is T else X for X in (Q, K, V)]
            fd = ((D.attention_fwd(*args_p, causal=True)[0] - D.attention_fwd(*args_m, causal=True)[0]) * G).sum() / (2 * eps)
            assert abs(fd - dT[idx]) < 1e-7 * max(1.0, abs(fd))
    tq, tk, tv = [torch.from_numpy(T.transpose(2, 3, 1, 0).copy()).requires_grad_(True) for T in (Q, K, V)]   # [b, j, s, i]
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    out.backward(torch.from_numpy(G.transpose(2, 3, 1, 0).copy()))
    for t, dT in ((tq, dQ), (tk, dK), (tv, dV)):
        np.testing.assert_allclose(dT, t.grad.numpy().transpose(3, 2, 0, 1), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("causal", [True, False])
def test_attention_online_form_equals_definition(causal):
    """Walking the key tiles with running (maximum, sum of shifted exponentials) gives the definition's
    result and statistics for any key tile, and the adjoint recomputed from those statistics is the
    definition's adjoint for any query tile."""
    from oracle import tiled as TL
    Q, K, V = _qkv(h=6, N_s=11, N_b=2, N_h=2)
    G = rng.standard_normal(Q.shape)
    Bo, P = D.attention_fwd(Q, K, V, causal=causal)
    _, tmax, den = D.softmax_fwd(D.attention_scores(K, Q), causal)
    dQ, dK, dV = D.attention_bwd(Q, K, V, P, G)
    for tile in (1, 3, 4, 11, 16):
        B2, m, d = TL.attention_fwd_online(Q, K, V, tile, causal)
        np.testing.assert_allclose(B2, Bo, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(m, tmax, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(d, den, rtol=1e-12)
        g = TL.attention_bwd_recompute(Q, K, V, B2, m, d, G, tile, causal)
        for got, want in zip(g, (dQ, dK, dV)):
            np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)
    # a large shift of all scores of one column moves the maximum, not the result (the rescaling is exact)
    K2 = K.copy()
    K2[:, 0] *= 40.0
    B3, m3, d3 = TL.attention_fwd_online(Q, K2, V, 2, causal)
    np.testing.assert_allclose(B3, D.attention_fwd(Q, K2, V, causal=causal)[0], rtol=1e-11, atol=1e-13)
    assert np.all(np.isfinite(B3)) and np.all(d3 >= 1.0 - 1e-12)


# ------------------------------------------------------------------ Adam
def test_adam_golden_two_steps():
    rows = [l.split() for l in open(os.path.join(GOLD, "adam_two_steps.txt")) if not l.startswith("#")]
    p, m, v = np.array([1.0]), np.zeros(1), np.zeros(1)
    for (step, wp, wm, wv), g in zip(rows, (2.0, -1.0)):
        p, m, v = D.adam_step(p, np.array([g]), m, v, int(step), lr=0.1, beta1=0.5, beta2=0.5, eps=0.0)
        assert abs(p[0] - float(wp)) < 1e-15 and abs(m[0] - float(wm)) < 1e-15 and abs(v[0] - float(wv)) < 1e-15


def test_adam_first_step_closed_form_and_torch():
    p0 = rng.standard_normal(50)
    g = rng.standard_normal(50)
    g[3] = 0.0
    p, m, v = D.adam_step(p0, g, np.zeros(50), np.zeros(50), 1)
    np.testing.assert_allclose(p - p0, -1e-3 * g / (np.abs(g) + 1e-8), rtol=1e-9, atol=1e-18)
    assert p[3] == p0[3]
    # three steps against torch.optim.Adam / AdamW in float64
    for wd, cls in ((0.0, torch.optim.Adam), (0.1, torch.optim.AdamW)):
        tp = torch.nn.Parameter(torch.from_numpy(p0.copy()))
        opt = cls([tp], lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=wd)
        p, m, v = p0.copy(), np.zeros(50), np.zeros(50)
        for t in range(1, 4):
            gt = rng.standard_normal(50)
            tp.grad = torch.from_numpy(gt.copy())
            opt.step()
            p, m, v = D.adam_step(p, gt, m, v, t, weight_decay=wd)
        np.testing.assert_allclose(p, tp.detach().numpy(), rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ bf16 rounding
def test_embedding_index_map_and_adjoint():
    N_e, N_v, N_s, N_b = 5, 7, 6, 2
    W = rng.standard_normal((N_e, N_v))
    tok = rng.integers(0, N_v, (N_s, N_b))
    tok[0, 0] = tok[1, 1] = 3                       # a repeated token
    Y = D.embedding_fwd(W, tok)
    for e, s, b in itertools.product(range(N_e), range(N_s), range(N_b)):
        assert Y[e, s, b] == W[e, tok[s, b]]
    G = rng.standard_normal(Y.shape)
    dW = D.embedding_bwd(G, tok, N_v)
    # adjoint identity <Y(W), G> = <W, dW>, column sums by hand, and the library's autograd
    assert abs((Y * G).sum() - (W * dW).sum()) < 1e-12
    want3 = sum(G[:, s, b] for s in range(N_s) for b in range(N_b) if tok[s, b] == 3)
    np.testing.assert_allclose(dW[:, 3], want3, rtol=1e-14)
    tw = torch.tensor(W.T.copy(), requires_grad=True)                                   # [N_v, N_e]
    out = torch.nn.functional.embedding(torch.from_numpy(tok.astype(np.int64)), tw)     # [N_s, N_b, N_e]
    out.backward(torch.from_numpy(G.transpose(1, 2, 0).copy()))
    np.testing.assert_allclose(dW, tw.grad.numpy().T, rtol=1e-13, atol=1e-15)
    unused = [v for v in range(N_v) if v not in tok]
    assert unused and np.all(dW[:, unused] == 0)


def test_cross_entropy_by_hand_library_and_differences():
    N_v, N_s, N_b = 6, 4, 3
    X = 3.0 * rng.standard_normal((N_v, N_s, N_b))
    lab = rng.integers(0, N_v, (N_s, N_b))
    L, losses, dX = D.cross_entropy(X, lab)
    for s, b in itertools.product(range(N_s), range(N_b)):
        den = sum(math.exp(X[j, s, b]) for j in range(N_v))
        assert abs(losses[s, b] + math.log(math.exp(X[lab[s, b], s, b]) / den)) < 1e-12
    assert abs(L - losses.sum()) < 1e-12
    # uniform logits: log N_v per column; a shift of a column changes nothing; gradient columns sum to zero
    L0, _, _ = D.cross_entropy(np.zeros((N_v, N_s, N_b)), lab)
    assert abs(L0 - N_s * N_b * math.log(N_v)) < 1e-12
    np.testing.assert_allclose(D.cross_entropy(X + 100.0, lab)[0], L, rtol=1e-12)
    np.testing.assert_allclose(dX.sum(axis=0), 0.0, atol=1e-14)
    # library value and autograd
    tx = torch.tensor(X.transpose(1, 2, 0).reshape(-1, N_v).copy(), requires_grad=True)
    tl = torch.nn.functional.cross_entropy(tx, torch.from_numpy(lab.reshape(-1).astype(np.int64)), reduction="sum")
    tl.backward()
    assert abs(tl.item() - L) < 1e-11
    np.testing.assert_allclose(dX, tx.grad.numpy().reshape(N_s, N_b, N_v).transpose(2, 0, 1), rtol=1e-12, atol=1e-14)
    # central differences
    for _ in range(5):
        idx = tuple(int(rng.integers(0, n)) for n in X.shape)
        Xp, Xm = X.copy(), X.copy()
        Xp[idx] += 1e-6
        Xm[idx] -= 1e-6
        fd = (D.cross_entropy(Xp, lab)[0] - D.cross_entropy(Xm, lab)[0]) / 2e-6
        assert abs(fd - dX[idx]) < 1e-8
    # over vocabulary tiles with the softmax subroutines' running statistics: the same loss
    from oracle import tiled as TL
    A = TL.Tiled.from_array(X, (4, 3, 2))
    P, stats = TL.softmax_fwd(A, causal=False)
    Pa, st = P.to_array(), stats.to_array()
    s_idx, b_idx = np.meshgrid(np.arange(N_s), np.arange(N_b), indexing="ij")
    np.testing.assert_allclose(-np.log(Pa[lab, s_idx, b_idx]), losses, rtol=1e-12)
    np.testing.assert_allclose(st[0] + np.log(st[1]) - X[lab, s_idx, b_idx], losses, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("nesterov", [False, True])
def test_sgd_momentum_closed_form_and_torch(nesterov):
    p0 = rng.standard_normal(37)
    gs = [rng.standard_normal(37) for _ in range(3)]
    lr, mu, wd = 0.05, 0.9, 0.01
    # by hand, one element, two steps from zero velocity
    g1 = gs[0][0] + wd * p0[0]
    v1 = g1
    p1 = p0[0] - lr * ((g1 + mu * v1) if nesterov else v1)
    g2 = gs[1][0] + wd * p1
    v2 = mu * v1 + g2
    p2 = p1 - lr * ((g2 + mu * v2) if nesterov else v2)
    p, v = p0.copy(), np.zeros(37)
    for k in range(2):
        p, v = D.sgd_step(p, gs[k], v, lr, mu, wd, nesterov)
    assert abs(p[0] - p2) < 1e-14 and abs(v[0] - v2) < 1e-14
    # the library optimiser, three steps
    tp = torch.tensor(p0.copy(), requires_grad=True)
    opt = torch.optim.SGD([tp], lr=lr, momentum=mu, weight_decay=wd, nesterov=nesterov)
    p, v = p0.copy(), np.zeros(37)
    for k in range(3):
        tp.grad = torch.tensor(gs[k].copy())
        opt.step()
        p, v = D.sgd_step(p, gs[k], v, lr, mu, wd, nesterov)
    np.testing.assert_allclose(p, tp.detach().numpy(), rtol=1e-13, atol=1e-15)
    # no momentum, no decay: plain gradient descent
    p, v = D.sgd_step(p0, gs[0], np.zeros(37), 0.1, 0.0, 0.0)
    np.testing.assert_allclose(p, p0 - 0.1 * gs[0], rtol=1e-15)


def test_round_to_bf16_matches_library_and_ties():
    x = np.concatenate([
        rng.standard_normal(5000).astype(np.float32) * 10,
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -1e-40, np.inf, -np.inf], np.float32),
    ])
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = D.round_to_bf16(x)
    np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1 (even); 1 + 3*2^-8 -> 1 + 2^-6
    assert D.round_to_bf16(np.array([1.00390625], np.float32))[0] == 1.0
    assert D.round_to_bf16(np.array([1.01171875], np.float32))[0] == 1.015625
    assert np.isnan(D.round_to_bf16(np.array([np.nan], np.float32))[0])
