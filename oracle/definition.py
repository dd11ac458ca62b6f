"""Untiled fp64 definition of the GPT-2 block operations (test infrastructure).

Arrays are numpy float64 indexed in the paper's axis order (section 3):
activations [e, s, b] (N_e x N_s x N_b), attention embeddings [i, s, b, j]
(h x N_s x N_b x N_h), scores [k, q, b, j] (key, query, batch, head), linear
weights [d, e] (N_d x N_e).  No tiling, blocking or fusion: each function is
the formula written out, with numpy's matmul/sum as the only library steps.

Not part of the product: only tests, the smoke check and the benchmark's
cpu_baseline leg call it.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# --------------------------------------------------------------------------
# generic contraction  C = alpha * op(A) * op(B) + beta * C   (section 2: block
# versions of matrix multiplication; section 3, linear and attention layers)
# --------------------------------------------------------------------------
def contract(alpha, opA, A, opB, B, beta, C, ncontract=1, nbatch=0):
    """C = alpha * op(A) . op(B) + beta * C over multi-axis operands.

    The last `nbatch` axes of A, B and C are batch axes.  Of the remaining
    axes, the `ncontract` contracted ones are A's last (opA = 'N') or first
    (opA = 'T') and B's first (opB = 'N') or last (opB = 'T').  C's axes are
    A's free axes, B's free axes, then the batch axes.
    """
    A = np.asarray(A, F64)
    B = np.asarray(B, F64)
    na, nb_ = A.ndim - nbatch, B.ndim - nbatch
    if opA == "N":
        a_free, a_con = list(range(0, na - ncontract)), list(range(na - ncontract, na))
    else:
        a_con, a_free = list(range(0, ncontract)), list(range(ncontract, na))
    if opB == "N":
        b_con, b_free = list(range(0, ncontract)), list(range(ncontract, nb_))
    else:
        b_free, b_con = list(range(0, nb_ - ncontract)), list(range(nb_ - ncontract, nb_))
    a_bat = list(range(na, A.ndim))
    b_bat = list(range(nb_, B.ndim))
    letters = "abcdefghijklmnopqrstuvwxyz"
    it = iter(letters)
    la = [None] * A.ndim
    lb = [None] * B.ndim
    for x, y in zip(a_con, b_con):
        assert A.shape[x] == B.shape[y], "contracted extents differ"
        la[x] = lb[y] = next(it)
    for x, y in zip(a_bat, b_bat):
        assert A.shape[x] == B.shape[y], "batch extents differ"
        la[x] = lb[y] = next(it)
    for x in a_free:
        la[x] = next(it)
    for y in b_free:
        lb[y] = next(it)
    lc = [la[x] for x in a_free] + [lb[y] for y in b_free] + [la[x] for x in a_bat]
    prod = np.einsum("".join(la) + "," + "".join(lb) + "->" + "".join(lc), A, B, optimize=True)
    out = alpha * prod
    if beta != 0.0:
        out = out + beta * np.asarray(C, F64)
    return out


def matmul2d(alpha, opA, A, opB, B, beta, C):
    """Plain matrix form: A is m x k (k x m if opA = 'T'), B is k x n (n x k if
    opB = 'T'), an optional trailing axis is a batch index."""
    nbatch = A.ndim - 2
    return contract(alpha, opA, A, opB, B, beta, C, 1, nbatch)


# --------------------------------------------------------------------------
# linear layer  Y = W X +. b   (section 3, linear layer)
# --------------------------------------------------------------------------
def bias_add(Y, b):
    """Y[d, s, b] + bias[d]: the same bias over the unchanged dimensions."""
    return Y + np.asarray(b, F64).reshape((-1,) + (1,) * (Y.ndim - 1))


def bias_grad(dY):
    return dY.reshape(dY.shape[0], -1).sum(axis=1)


def linear_fwd(W, X, b):
    W = np.asarray(W, F64)
    X = np.asarray(X, F64)
    Y = np.matmul(W, X.reshape(X.shape[0], -1)).reshape((W.shape[0],) + X.shape[1:])
    return bias_add(Y, b)


def linear_bwd(W, X, dY):
    """Adjoint of linear_fwd: dX = W^T dY, dW = sum_{s,b} dY X^T, db = sum_{s,b} dY."""
    W = np.asarray(W, F64)
    X2 = np.asarray(X, F64).reshape(X.shape[0], -1)
    dY2 = np.asarray(dY, F64).reshape(dY.shape[0], -1)
    dX = np.matmul(W.T, dY2).reshape(X.shape)
    dW = np.matmul(dY2, X2.T)
    db = dY2.sum(axis=1)
    return dX, dW, db


# --------------------------------------------------------------------------
# activation (section 3, nonlinear activations; GPT-2 uses GELU)
# --------------------------------------------------------------------------
_C0 = math.sqrt(2.0 / math.pi)
_C1 = 0.044715


def gelu(x, variant="tanh"):
    x = np.asarray(x, F64)
    if variant == "tanh":
        return 0.5 * x * (1.0 + np.tanh(_C0 * (x + _C1 * x ** 3)))
    if variant == "erf":
        return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))
    raise ValueError(variant)


def gelu_grad(x, variant="tanh"):
    x = np.asarray(x, F64)
    if variant == "tanh":
        t = np.tanh(_C0 * (x + _C1 * x ** 3))
        return 0.5 * (1.0 + t) + 0.5 * x * (1.0 - t * t) * _C0 * (1.0 + 3.0 * _C1 * x * x)
    if variant == "erf":
        return 0.5 * (1.0 + _erf(x / math.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)
    raise ValueError(variant)


# --------------------------------------------------------------------------
# layer normalisation over the embedding axis (section 3, layer normalization)
# --------------------------------------------------------------------------
def layernorm_fwd(X, gamma, beta, eps):
    """Returns Y and the per-token statistics (mean, 1/sqrt(var + eps)); the
    variance is the biased one (divided by N_e)."""
    X = np.asarray(X, F64)
    mean = X.mean(axis=0)
    var = ((X - mean) ** 2).mean(axis=0)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (X - mean) * rstd
    g = np.asarray(gamma, F64).reshape((-1,) + (1,) * (X.ndim - 1))
    bt = np.asarray(beta, F64).reshape(g.shape)
    return g * xhat + bt, mean, rstd


def layernorm_bwd(X, gamma, mean, rstd, dY):
    X = np.asarray(X, F64)
    dY = np.asarray(dY, F64)
    xhat = (X - mean) * rstd
    gm = np.asarray(gamma, F64).reshape((-1,) + (1,) * (X.ndim - 1))
    g = dY * gm
    dX = rstd * (g - g.mean(axis=0) - xhat * (g * xhat).mean(axis=0))
    red = tuple(range(1, X.ndim))
    dgamma = (dY * xhat).sum(axis=red)
    dbeta = dY.sum(axis=red)
    return dX, dgamma, dbeta


# --------------------------------------------------------------------------
# softmax over the first axis, max-shifted form (section 3, SoftMax)
# --------------------------------------------------------------------------
def causal_mask(n_k, n_q):
    """True where key index k may be seen by query index q (k <= q)."""
    return np.arange(n_k)[:, None] <= np.arange(n_q)[None, :]


def softmax_fwd(A, causal=False):
    """P[:, q, ...] = softmax over axis 0 of A[:, q, ...]; with `causal`,
    entries with key index > query index (axis 1) are excluded (probability 0).
    Returns P and the two per-column statistics (max, sum of shifted exps)."""
    A = np.asarray(A, F64)
    if causal:
        vis = causal_mask(A.shape[0], A.shape[1]).reshape(A.shape[:2] + (1,) * (A.ndim - 2))
        A = np.where(vis, A, -np.inf)
    tmax = A.max(axis=0)
    ex = np.exp(A - tmax)
    den = ex.sum(axis=0)
    return ex / den, tmax, den


def softmax_bwd(P, dP):
    """Gradient with respect to the softmax input: P o (dP - sum_k P o dP)."""
    P = np.asarray(P, F64)
    dP = np.asarray(dP, F64)
    return P * (dP - (P * dP).sum(axis=0))


# --------------------------------------------------------------------------
# attention (section 3, attention layer)
# --------------------------------------------------------------------------
def split_heads(Z, N_h, n_parts):
    """(n_parts * N_h * h) x N_s x N_b  ->  n_parts arrays h x N_s x N_b x N_h;
    row r of Z is (part, head j, component i) = ((part * N_h + j) * h + i)."""
    Z = np.asarray(Z, F64)
    rows, N_s, N_b = Z.shape
    h = rows // (n_parts * N_h)
    Z5 = Z.reshape(n_parts, N_h, h, N_s, N_b)
    return [np.ascontiguousarray(Z5[p].transpose(1, 2, 3, 0)) for p in range(n_parts)]


def merge_heads(parts):
    """Inverse of split_heads."""
    parts = [np.asarray(p, F64) for p in parts]
    h, N_s, N_b, N_h = parts[0].shape
    Z5 = np.stack([p.transpose(3, 0, 1, 2) for p in parts], axis=0)
    return Z5.reshape(len(parts) * N_h * h, N_s, N_b)


def _jb(T):   # [i, s, b, j] -> [j, b, i, s], stored contiguously so that matmul can hand each matrix to BLAS
    return np.ascontiguousarray(T.transpose(3, 2, 0, 1))


def _back(T):  # [j, b, x, y] -> [x, y, b, j]
    return T.transpose(2, 3, 1, 0)


def attention_scores(K, Q):
    """A[k, q, b, j] = (1 / sqrt(h)) sum_i K[i, k, b, j] Q[i, q, b, j]."""
    h = K.shape[0]
    return _back(np.matmul(_jb(K).transpose(0, 1, 3, 2), _jb(Q))) / math.sqrt(h)


def attention_values(V, P):
    """B[i, q, b, j] = sum_k V[i, k, b, j] P[k, q, b, j]."""
    return _back(np.matmul(_jb(V), _jb(P)))


def attention_fwd(Q, K, V, causal=True):
    A = attention_scores(K, Q)
    P, tmax, den = softmax_fwd(A, causal)
    return attention_values(V, P), P


def attention_bwd(Q, K, V, P, dB):
    h = Q.shape[0]
    sc = 1.0 / math.sqrt(h)
    Pj = _jb(P)                              # [j, b, k, q]
    dBj = _jb(dB)                            # [j, b, i, q]
    dV = _back(np.matmul(dBj, Pj.transpose(0, 1, 3, 2)))          # dV[i,k] = sum_q dB[i,q] P[k,q]
    dP = _back(np.matmul(_jb(V).transpose(0, 1, 3, 2), dBj))      # dP[k,q] = sum_i V[i,k] dB[i,q]
    dA = softmax_bwd(P, dP)
    dAj = _jb(dA)
    dQ = sc * _back(np.matmul(_jb(K), dAj))                        # dQ[i,q] = sc sum_k K[i,k] dA[k,q]
    dK = sc * _back(np.matmul(_jb(Q), dAj.transpose(0, 1, 3, 2)))  # dK[i,k] = sc sum_q Q[i,q] dA[k,q]
    return dQ, dK, dV


# --------------------------------------------------------------------------
# the GPT-2 block (pre-LN, biases on all four linear layers, no dropout)
# --------------------------------------------------------------------------
def _silent(stage):
    pass


def block_forward(p, X, N_h, eps=1e-5, gelu_variant="tanh", causal=True, progress=_silent):
    """p: dict of the 12 parameters.  Returns Out and everything the adjoint needs.
    `progress(stage)` is called after each layer (large cases take minutes; no arithmetic depends on it)."""
    c = {}
    X = np.asarray(X, F64)
    c["X"] = X
    c["X1"], c["mean1"], c["rstd1"] = layernorm_fwd(X, p["gamma1"], p["beta1"], eps)
    QKV = linear_fwd(p["W_qkv"], c["X1"], p["b_qkv"])
    c["Q"], c["K"], c["V"] = split_heads(QKV, N_h, 3)
    progress("forward: layer norm 1, QKV")
    Bh, c["P"] = attention_fwd(c["Q"], c["K"], c["V"], causal)
    c["Bm"] = merge_heads([Bh])
    progress("forward: attention")
    Y = linear_fwd(p["W_o"], c["Bm"], p["b_o"])
    c["X2"] = X + Y
    c["X3"], c["mean2"], c["rstd2"] = layernorm_fwd(c["X2"], p["gamma2"], p["beta2"], eps)
    c["H1"] = linear_fwd(p["W_1"], c["X3"], p["b_1"])
    progress("forward: output projection, layer norm 2, fc1")
    c["G"] = gelu(c["H1"], gelu_variant)
    H2 = linear_fwd(p["W_2"], c["G"], p["b_2"])
    Out = c["X2"] + H2
    progress("forward: GELU, fc2")
    return Out, c


def block_backward(p, c, dOut, N_h, gelu_variant="tanh", progress=_silent):
    """Exact adjoint of block_forward for the upstream gradient dOut.
    Returns dX and a dict with the 12 parameter gradients."""
    g = {}
    dOut = np.asarray(dOut, F64)
    dG, g["W_2"], g["b_2"] = linear_bwd(p["W_2"], c["G"], dOut)
    progress("backward: fc2")
    dH1 = dG * gelu_grad(c["H1"], gelu_variant)
    dX3, g["W_1"], g["b_1"] = linear_bwd(p["W_1"], c["X3"], dH1)
    progress("backward: GELU, fc1")
    d2, g["gamma2"], g["beta2"] = layernorm_bwd(c["X2"], p["gamma2"], c["mean2"], c["rstd2"], dX3)
    dX2 = dOut + d2
    dBm, g["W_o"], g["b_o"] = linear_bwd(p["W_o"], c["Bm"], dX2)
    progress("backward: layer norm 2, output projection")
    (dB,) = split_heads(dBm, N_h, 1)
    dQ, dK, dV = attention_bwd(c["Q"], c["K"], c["V"], c["P"], dB)
    dQKV = merge_heads([dQ, dK, dV])
    progress("backward: attention")
    dX1, g["W_qkv"], g["b_qkv"] = linear_bwd(p["W_qkv"], c["X1"], dQKV)
    progress("backward: QKV")
    d1, g["gamma1"], g["beta1"] = layernorm_bwd(c["X"], p["gamma1"], c["mean1"], c["rstd1"], dX1)
    dX = dX2 + d1
    return dX, g


# --------------------------------------------------------------------------
# optimiser (section 3, optimizers: Adam as in Kingma & Ba, with bias correction)
# --------------------------------------------------------------------------
def adam_step(p, g, m, v, t, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """One Adam step number t (t >= 1).  weight_decay > 0 gives the decoupled
    (AdamW) form p <- p - lr * wd * p before the moment update is applied."""
    p = np.asarray(p, F64)
    g = np.asarray(g, F64)
    m = beta1 * np.asarray(m, F64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, F64) + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    p = p - lr * weight_decay * p - lr * mhat / (np.sqrt(vhat) + eps)
    return p, m, v


# --------------------------------------------------------------------------
# bf16 storage rounding (round to nearest, ties to even, on the fp32 bit pattern)
# --------------------------------------------------------------------------
# --------------------------------------------------------------------------
# embedding layer and cross-entropy loss (section 3)
# --------------------------------------------------------------------------
def embedding_fwd(W, tokens):
    """W: [N_e, N_v] (one column per vocabulary item); tokens: int [N_s, N_b].
    Y[e, s, b] = W[e, tokens[s, b]]."""
    W = np.asarray(W, F64)
    return W[:, np.asarray(tokens)]


def embedding_bwd(dY, tokens, N_v):
    """dW[e, v] = sum of dY[e, s, b] over the positions (s, b) whose token is v."""
    dY = np.asarray(dY, F64)
    tokens = np.asarray(tokens)
    dW = np.zeros((dY.shape[0], N_v), F64)
    for s in range(tokens.shape[0]):
        for b in range(tokens.shape[1]):
            dW[:, tokens[s, b]] += dY[:, s, b]
    return dW


def cross_entropy(X, labels):
    """X: logits [N_v, N_s, N_b]; labels: int [N_s, N_b].
    L = - sum_{s,b} log(exp(x[c]) / sum_j exp(x[j])), c the label of the column;
    returns (L, per-column losses, dL/dX = softmax(X) - onehot(labels))."""
    X = np.asarray(X, F64)
    labels = np.asarray(labels)
    m = X.max(axis=0)
    E = np.exp(X - m)
    den = E.sum(axis=0)
    P = E / den
    s_idx, b_idx = np.meshgrid(np.arange(X.shape[1]), np.arange(X.shape[2]), indexing="ij")
    picked = X[labels, s_idx, b_idx]
    losses = m + np.log(den) - picked
    dX = P.copy()
    dX[labels, s_idx, b_idx] -= 1.0
    return losses.sum(), losses, dX


def sgd_step(p, g, v, lr=1e-2, momentum=0.9, weight_decay=0.0, nesterov=False):
    """SGD with momentum (section 3, Optimizers: a weighted sum of parameter, gradient and momentum
    term): g' = g + weight_decay p, v <- momentum v + g', p <- p - lr v; with `nesterov` the step
    direction is g' + momentum v.  Zero v before the first step gives the usual v = g'.
    Returns (p, v)."""
    p, g, v = (np.asarray(x, F64) for x in (p, g, v))
    g = g + weight_decay * p
    v = momentum * v + g
    step = g + momentum * v if nesterov else v
    return p - lr * step, v


def round_to_bf16(x):
    """Value of the nearest bf16 number to each fp32 input, returned as fp32.
    NaNs stay NaN (quiet); overflow past the largest finite bf16 gives inf."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    u = x32.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    r = r.astype(np.uint32)
    nan = np.isnan(x32)
    r = np.where(nan, (x32.view(np.uint32) | np.uint32(0x00400000)) & np.uint32(0xFFFF0000), r)
    return r.astype(np.uint32).view(np.float32).reshape(x32.shape)
