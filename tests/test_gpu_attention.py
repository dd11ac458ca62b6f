"""GPU parity of the fused tile attention (forward and recomputing backward)
against the fp64 definition: softmax(scale K^T Q, masked) applied to V, and its
adjoint, per batch element and head."""
import math

import numpy as np
import pytest

from gpu_util import check, quant
from oracle import definition as D

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mods():
    from paper_2504_13236_amd import capi, tiled
    return capi, tiled


def T(tiled, ctx, a, base, dtype):
    return tiled.TiledTensor.from_numpy(ctx, np.asarray(a, np.float32), base, dtype)


def reference(Q, K, V, dB, causal):
    B, P = D.attention_fwd(Q, K, V, causal=causal)
    A = D.attention_scores(K, Q)
    _, tmax, den = D.softmax_fwd(A, causal)
    dQ, dK, dV = D.attention_bwd(Q, K, V, P, dB)
    return B, tmax, den, dQ, dK, dV


# (h, N_s, N_b, N_h), sequence tile, batch tile, head tile: whole and ragged workgroup blocks (128 rows),
# ragged streamed blocks (64 rows), ragged last tiles, tiled batch and head axes, one tile only
CASES = [
    ((64, 256, 2, 3), 128, 2, 3),
    ((64, 200, 2, 2), 96, 1, 2),
    ((64, 330, 1, 3), 400, 1, 2),
    ((64, 72, 3, 1), 40, 2, 1),
    ((128, 160, 1, 2), 160, 1, 1),
    ((64, 1, 1, 1), 1, 1, 1),              # a single position: P = 1, B = V
    ((64, 33, 2, 1), 7, 1, 1),             # tiles far smaller than a streamed block
    ((128, 200, 2, 1), 72, 2, 1),          # head size 128 on ragged tiles
]


@pytest.mark.parametrize("gran", [0, 1])
@pytest.mark.parametrize("causal", [1, 0])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", CASES, ids=lambda c: "x".join(map(str, c[0])) + "-t%d" % c[1])
def test_fused_attention(mods, case, dtype, causal, gran):
    capi, tiled = mods
    shape, ts, tb, th = case
    h, N_s, N_b, N_h = shape
    r = np.random.default_rng(hash((shape, ts, causal)) % (2 ** 31))
    Q, K, V, dB = (quant(r.standard_normal(shape), dtype) for _ in range(4))
    scale = 1.0 / math.sqrt(h)
    base = (h, ts, tb, th)
    B, tmax, den, dQ, dK, dV = reference(Q, K, V, dB, bool(causal))
    with tiled.Context(n_streams=4, granularity=gran) as ctx:
        tQ, tK, tV, tdB = (T(tiled, ctx, x, base, dtype) for x in (Q, K, V, dB))
        tB = tiled.TiledTensor(ctx, dtype, shape, base)
        tS = tiled.TiledTensor(ctx, "f32", (2, N_s, N_b, N_h), (2, ts, tb, th))
        capi.nnt_attention_fwd(ctx.h, tQ.h, tK.h, tV.h, scale, causal, tB.h, tS.h)
        check(tB.download(), B, dtype, "attention fwd")
        stats = tS.download()
        # the statistics are fp32 whatever the operands' type
        check(stats[0], tmax, "f32", "running maximum")
        check(stats[1], den, "f32", "sum of shifted exponentials")
        tdQ, tdK, tdV = (tiled.TiledTensor(ctx, dtype, shape, base) for _ in range(3))
        capi.nnt_attention_bwd(ctx.h, tQ.h, tK.h, tV.h, tB.h, tS.h, tdB.h, scale, causal, tdQ.h, tdK.h, tdV.h)
        check(tdV.download(), dV, dtype, "attention dV")
        check(tdQ.download(), dQ, dtype, "attention dQ")
        check(tdK.download(), dK, dtype, "attention dK")
        # a second call overwrites, it does not accumulate
        capi.nnt_attention_bwd(ctx.h, tQ.h, tK.h, tV.h, tB.h, tS.h, tdB.h, scale, causal, tdQ.h, tdK.h, tdV.h)
        check(tdK.download(), dK, dtype, "attention dK, second call")


# h, N_h, row tile, N_s, sequence tile, N_b, batch tile, head tile of the statistics
HEADS_CASES = [
    (64, 6, 128, 200, 96, 3, 2, 6),          # two heads per row tile, ragged sequence and batch tiles
    (64, 4, 256, 330, 400, 1, 1, 2),         # all heads of a part in one row tile, one ragged sequence tile
    (128, 4, 256, 160, 72, 2, 1, 1),         # head size 128, statistics tiled one head at a time
    (64, 3, 64, 72, 40, 2, 2, 3),            # one head per row tile
]


@pytest.mark.parametrize("gran", [0, 1])
@pytest.mark.parametrize("causal", [1, 0])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", HEADS_CASES, ids=lambda c: "h%d-Nh%d-t%d-Ns%d-ts%d" % c[:5])
def test_fused_attention_on_tensors_with_the_heads_side_by_side(mods, case, dtype, causal, gran):
    """The fused kernels read Q, K, V and dB out of, and write B, dQ, dK, dV into, the tensors of the linear layers
    ([3 N_h h, N_s, N_b] and [N_h h, N_s, N_b]): against the oracle's head split, attention and head merge."""
    capi, tiled = mods
    h, N_h, t0, N_s, ts, N_b, tb, th = case
    N_e = h * N_h
    r = np.random.default_rng(hash((case, causal)) % (2 ** 31))
    QKV = quant(r.standard_normal((3 * N_e, N_s, N_b)), dtype)
    dBm = quant(r.standard_normal((N_e, N_s, N_b)), dtype)
    Q, K, V = D.split_heads(QKV, N_h, 3)
    dB = D.split_heads(dBm, N_h, 1)[0]
    scale = 1.0 / math.sqrt(h)
    B, tmax, den, dQ, dK, dV = reference(Q, K, V, dB, bool(causal))
    with tiled.Context(n_streams=2, granularity=gran) as ctx:
        tQKV, tdBm = T(tiled, ctx, QKV, (t0, ts, tb), dtype), T(tiled, ctx, dBm, (t0, ts, tb), dtype)
        tBm = tiled.TiledTensor(ctx, dtype, (N_e, N_s, N_b), (t0, ts, tb))
        tS = tiled.TiledTensor(ctx, "f32", (2, N_s, N_b, N_h), (2, ts, tb, th))
        capi.nnt_attention_fwd_heads(ctx.h, tQKV.h, scale, causal, tBm.h, tS.h, N_h)
        check(tBm.download(), D.merge_heads([B]), dtype, "attention fwd")
        stats = tS.download()
        check(stats[0], tmax, "f32", "running maximum")
        check(stats[1], den, "f32", "sum of shifted exponentials")
        tdQKV = tiled.TiledTensor(ctx, dtype, QKV.shape, (t0, ts, tb))
        capi.nnt_attention_bwd_heads(ctx.h, tQKV.h, tBm.h, tS.h, tdBm.h, scale, causal, tdQKV.h, N_h)
        got, ref = tdQKV.download(), D.merge_heads([dQ, dK, dV])
        for part, name in enumerate(("attention dQ", "attention dK", "attention dV")):
            check(got[part * N_e:(part + 1) * N_e], ref[part * N_e:(part + 1) * N_e], dtype, name)
        # geometry that does not fit is refused
        bad = tiled.TiledTensor(ctx, dtype, (2 * N_e, N_s, N_b), (t0, ts, tb))
        with pytest.raises(capi.NntError):
            capi.nnt_attention_fwd_heads(ctx.h, bad.h, scale, causal, tBm.h, tS.h, N_h)
        with pytest.raises(capi.NntError):
            capi.nnt_attention_fwd_heads(ctx.h, tQKV.h, scale, causal, tBm.h, tS.h, N_h + 1)


def test_fused_attention_survives_large_scores(mods):
    """Scores of several hundred: the running maximum keeps every exponent at or below zero."""
    capi, tiled = mods
    r = np.random.default_rng(5)
    shape, base = (64, 96, 1, 2), (64, 48, 1, 2)
    Q, K, V = (r.standard_normal(shape) for _ in range(3))
    Q *= 30.0
    K *= 30.0
    Q, K, V = (quant(x, "f32") for x in (Q, K, V))
    B, _ = D.attention_fwd(Q, K, V, causal=True)
    with tiled.Context(n_streams=1) as ctx:
        tQ, tK, tV = (T(tiled, ctx, x, base, "f32") for x in (Q, K, V))
        tB = tiled.TiledTensor(ctx, "f32", shape, base)
        tS = tiled.TiledTensor(ctx, "f32", (2, 96, 1, 2), (2, 48, 1, 2))
        capi.nnt_attention_fwd(ctx.h, tQ.h, tK.h, tV.h, 0.125, 1, tB.h, tS.h)
        got = tB.download()
        assert np.all(np.isfinite(got))
        # exp(x) carries the rounding of its argument: a score of magnitude |x| held in fp32 is off by up to
        # |x| 2^-24, and so is the probability, relatively.  The bound scales with the largest score.
        big = float(np.abs(D.attention_scores(K, Q)).max())
        assert big > 300
        err = float(np.abs(got - B).max() / np.abs(B).max())
        assert err <= 8 * big * 2.0 ** -24, (err, big)
        with pytest.raises(capi.NntError):
            capi.nnt_attention_fwd(ctx.h, tQ.h, tK.h, tV.h, -0.125, 1, tB.h, tS.h)      # scale must be positive


def test_fused_attention_rejects_bad_operands(mods):
    capi, tiled = mods
    with tiled.Context(n_streams=1) as ctx:
        q = tiled.TiledTensor(ctx, "f32", (64, 32, 1, 1), (64, 32, 1, 1))
        s = tiled.TiledTensor(ctx, "f32", (2, 32, 1, 1), (2, 32, 1, 1))
        odd = tiled.TiledTensor(ctx, "f32", (48, 32, 1, 1), (48, 32, 1, 1))          # head size neither 64 nor 128
        s_odd = tiled.TiledTensor(ctx, "f32", (2, 32, 1, 1), (2, 16, 1, 1))          # statistics tiled differently
        split = tiled.TiledTensor(ctx, "f32", (64, 32, 1, 1), (32, 32, 1, 1))        # head axis tiled
        for args in ((odd, odd, odd, odd, s), (q, q, q, q, s_odd), (split, split, split, split, s), (q, q, q, odd, s)):
            with pytest.raises(capi.NntError):
                capi.nnt_attention_fwd(ctx.h, args[0].h, args[1].h, args[2].h, 0.125, 1, args[3].h, args[4].h)
        # argument errors leave the context usable
        out = tiled.TiledTensor(ctx, "f32", (64, 32, 1, 1), (64, 32, 1, 1))
        capi.nnt_attention_fwd(ctx.h, q.h, q.h, q.h, 0.125, 1, out.h, s.h)
        ctx.wait()
