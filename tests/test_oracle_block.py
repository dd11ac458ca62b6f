"""Pins for the oracle's block forward / backward and for tiling invariance."""
import math

import numpy as np
import pytest
import torch

import workload
from oracle import definition as D
from oracle import tiled as Tl

rng = np.random.default_rng(11)


def small_cfg():
    return workload.CONFIGS[1].replace(N_e=24, N_h=3, N_m=40, N_s=10, N_b=2, tile=8)


def f64(d):
    return {k: np.asarray(v, np.float64) for k, v in d.items()}


def torch_block(p, X, N_h, eps, variant):
    """Independent library route: torch float64 layer_norm / linear / gelu and an
    explicitly masked softmax, in torch's own [b, s, e] layout, with autograd."""
    F = torch.nn.functional
    tp = {k: torch.from_numpy(np.array(v, np.float64)).requires_grad_() for k, v in p.items()}
    x = torch.from_numpy(np.array(X, np.float64).transpose(2, 1, 0).copy()).requires_grad_()   # [b, s, e]
    N_b, N_s, N_e = x.shape
    h = N_e // N_h
    x1 = F.layer_norm(x, (N_e,), tp["gamma1"], tp["beta1"], eps)
    qkv = F.linear(x1, tp["W_qkv"], tp["b_qkv"])
    q, k, v = qkv.split(N_e, dim=2)
    q, k, v = [t.view(N_b, N_s, N_h, h).transpose(1, 2) for t in (q, k, v)]                    # [b, j, s, i]
    att = (q @ k.transpose(-1, -2)) / math.sqrt(h)                                             # [b, j, q, k]
    mask = torch.tril(torch.ones(N_s, N_s, dtype=torch.bool))
    att = att.masked_fill(~mask, float("-inf")).softmax(dim=-1)
    y = (att @ v).transpose(1, 2).reshape(N_b, N_s, N_e)
    x2 = x + F.linear(y, tp["W_o"], tp["b_o"])
    x3 = F.layer_norm(x2, (N_e,), tp["gamma2"], tp["beta2"], eps)
    h1 = F.linear(x3, tp["W_1"], tp["b_1"])
    g = F.gelu(h1, approximate="tanh" if variant == "tanh" else "none")
    out = x2 + F.linear(g, tp["W_2"], tp["b_2"])
    return out, x, tp


@pytest.mark.parametrize("variant", ["tanh", "erf"])
def test_block_forward_backward_vs_torch(variant):
    cfg = small_cfg()
    inp = f64(workload.generate(cfg))
    p = {k: inp[k] for k in workload.PARAM_NAMES}
    # livelier parameters than N(0, 0.02) so that every path carries signal
    p = {k: (v * 10 if k.startswith("W") else v) for k, v in p.items()}
    Out, cache = D.block_forward(p, inp["X"], cfg.N_h, cfg.eps, variant)
    dX, grads = D.block_backward(p, cache, inp["dOut"], cfg.N_h, variant)
    out_t, x_t, tp = torch_block(p, inp["X"], cfg.N_h, cfg.eps, variant)
    np.testing.assert_allclose(Out, out_t.detach().numpy().transpose(2, 1, 0), rtol=1e-11, atol=1e-12)
    out_t.backward(torch.from_numpy(inp["dOut"].transpose(2, 1, 0).copy()))
    np.testing.assert_allclose(dX, x_t.grad.numpy().transpose(2, 1, 0), rtol=1e-9, atol=1e-11)
    for k in workload.PARAM_NAMES:
        np.testing.assert_allclose(grads[k], tp[k].grad.numpy(), rtol=1e-9, atol=1e-10, err_msg=k)


def test_block_backward_finite_differences():
    cfg = small_cfg()
    inp = f64(workload.generate(cfg))
    p = {k: (inp[k] * 10 if k.startswith("W") else inp[k]) for k in workload.PARAM_NAMES}
    X, dOut = inp["X"], inp["dOut"]
    Out, cache = D.block_forward(p, X, cfg.N_h, cfg.eps)
    dX, grads = D.block_backward(p, cache, dOut, cfg.N_h)
    grads = dict(grads, X=dX)

    def loss(pp, xx):
        return float((D.block_forward(pp, xx, cfg.N_h, cfg.eps)[0] * dOut).sum())

    e = 1e-6
    for name in list(workload.PARAM_NAMES) + ["X"]:
        base = X if name == "X" else p[name]
        v = rng.standard_normal(base.shape)
        def shifted(sign):
            if name == "X":
                return loss(p, X + sign * e * v)
            q = dict(p)
            q[name] = base + sign * e * v
            return loss(q, X)
        fd = (shifted(+1) - shifted(-1)) / (2 * e)
        an = float((grads[name] * v).sum())
        assert abs(fd - an) <= 2e-7 * max(1.0, abs(an)), (name, fd, an)


def _tile_params(p, bt):
    out = {}
    for k, v in p.items():
        if v.ndim == 1:
            base = (bt["e3"] if k == "b_qkv" else bt["m"] if k == "b_1" else bt["e"],)
        else:
            rows = bt["e3"] if k == "W_qkv" else bt["m"] if k == "W_1" else bt["e"]
            cols = bt["m"] if k == "W_2" else bt["e"]
            base = (rows, cols)
        out[k] = Tl.Tiled.from_array(v, base)
    return out


def _bt_variants(cfg):
    bt = workload.base_tiles(cfg)
    whole = dict(e=cfg.N_e, e3=3 * cfg.N_e, m=cfg.N_m, s=cfg.N_s, b=cfg.N_b, j=cfg.N_h, i=cfg.h)
    ragged = dict(e=24, e3=24, m=24, s=24, b=cfg.N_b, j=cfg.N_h, i=24)
    thin = dict(bt, b=1, j=1, i=16)
    odd = dict(e=40, e3=56, m=72, s=24, b=1, j=1, i=40)
    return {"recipe": bt, "whole": whole, "ragged24": ragged, "batch1_head1": thin, "mixed": odd}


@pytest.mark.parametrize("variant", ["recipe", "whole", "ragged24", "batch1_head1", "mixed"])
def test_tiling_invariance_block_C1(variant):
    cfg = workload.CONFIGS[1]
    inp = f64(workload.generate(cfg))
    p = {k: inp[k] for k in workload.PARAM_NAMES}
    Out, cache = D.block_forward(p, inp["X"], cfg.N_h, cfg.eps)
    dX, grads = D.block_backward(p, cache, inp["dOut"], cfg.N_h)
    bt = _bt_variants(cfg)[variant]
    tp = _tile_params(p, bt)
    xb = (bt["e"], bt["s"], bt["b"])
    Out_t, c_t = Tl.block_forward(tp, Tl.Tiled.from_array(inp["X"], xb), cfg.N_h, bt, cfg.eps)
    dX_t, g_t = Tl.block_backward(tp, c_t, Tl.Tiled.from_array(inp["dOut"], xb), cfg.N_h, bt)

    def rel(a, b):
        return np.abs(a - b).max() / np.abs(b).max()

    assert rel(Out_t.to_array(), Out) < 1e-12
    assert rel(dX_t.to_array(), dX) < 1e-12
    assert rel(c_t["P"].to_array(), cache["P"]) < 1e-12
    for k in workload.PARAM_NAMES:
        assert rel(g_t[k].to_array(), grads[k]) < 1e-12, k
    # the statistics the tile steps leave behind are the definition's
    np.testing.assert_allclose(c_t["stats1"].to_array()[0], cache["mean1"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(c_t["stats1"].to_array()[1], cache["rstd1"], rtol=1e-12)


def test_tiled_gemm_random_tilings():
    r = np.random.default_rng(5)
    for trial in range(25):
        m, n, k, nb = [int(v) for v in r.integers(1, 13, 4)]
        nb = 1 + nb % 3
        opA, opB = r.choice(["N", "T"]), r.choice(["N", "T"])
        bm, bn, bk, bb = [int(v) for v in r.integers(1, 8, 4)]
        A = r.standard_normal(((m, k) if opA == "N" else (k, m)) + (nb,))
        B = r.standard_normal(((k, n) if opB == "N" else (n, k)) + (nb,))
        C = r.standard_normal((m, n, nb))
        At = Tl.Tiled.from_array(A, ((bm, bk) if opA == "N" else (bk, bm)) + (bb,))
        Bt = Tl.Tiled.from_array(B, ((bk, bn) if opB == "N" else (bn, bk)) + (bb,))
        Ct = Tl.Tiled.from_array(C, (bm, bn, bb))
        Tl.gemm(0.5, opA, At, opB, Bt, 2.0, Ct, 1, 1)
        ref = D.contract(0.5, opA, A, opB, B, 2.0, C, 1, 1)
        np.testing.assert_allclose(Ct.to_array(), ref, rtol=1e-12, atol=1e-12)


def test_tiled_softmax_any_key_tiling_and_structural_zero_tiles():
    A = rng.standard_normal((13, 13, 2, 2)) * 3
    P, tmax, den = D.softmax_fwd(A, causal=True)
    for bk in (1, 4, 5, 13):
        base = (bk, 5, 1, 2)
        absent = lambda idx: idx[0] * base[0] > min(13, (idx[1] + 1) * base[1]) - 1
        At = Tl.Tiled.from_array(A, base, absent)
        Pt, st = Tl.softmax_fwd(At, causal=True)
        np.testing.assert_allclose(Pt.to_array(), P, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(st.to_array()[0], tmax, rtol=1e-13)
        np.testing.assert_allclose(st.to_array()[1], den, rtol=1e-12)


def test_adam_tiled_equals_untiled():
    p, g = rng.standard_normal((10, 7)), rng.standard_normal((10, 7))
    m, v = rng.standard_normal((10, 7)) * 0.1, rng.random((10, 7))
    ref = D.adam_step(p, g, m, v, 3)
    T = lambda a: Tl.Tiled.from_array(a, (4, 3))
    got = Tl.adam_step(T(p), T(g), T(m), T(v), 3)
    for a, b in zip(got, ref):
        np.testing.assert_allclose(a.to_array(), b, rtol=1e-15)


def test_workload_generator_is_seeded_and_shaped():
    cfg = workload.CONFIGS[1]
    a, b = workload.generate(cfg), workload.generate(cfg)
    for k, shape in workload.tensor_shapes(cfg).items():
        assert a[k].shape == shape and a[k].dtype == np.float32
        np.testing.assert_array_equal(a[k], b[k])
    assert abs(a["W_1"].std() - 0.02) < 2e-3 and abs(a["X"].std() - 1.0) < 0.05
    assert abs(a["gamma1"].mean() - 1.0) < 0.02
    assert workload.causal_tile_pairs(workload.CONFIGS[2]).__len__() == 10     # 4 x 4 tiles, kt <= qt
    assert abs(workload.model_flops(workload.CONFIGS[2], tile_skip=False) / 425.2e9 - 1) < 2e-3
    assert abs(workload.model_flops(workload.CONFIGS[4]) / 1619e9 - 1) < 2e-3
