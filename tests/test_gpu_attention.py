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
        check(stats[0], tmax, dtype, "running maximum")
        check(stats[1], den, dtype, "sum of shifted exponentials")
        tdQ, tdK, tdV = (tiled.TiledTensor(ctx, dtype, shape, base) for _ in range(3))
        capi.nnt_attention_bwd(ctx.h, tQ.h, tK.h, tV.h, tB.h, tS.h, tdB.h, scale, causal, tdQ.h, tdK.h, tdV.h)
        check(tdV.download(), dV, dtype, "attention dV")
        check(tdQ.download(), dQ, dtype, "attention dQ")
        check(tdK.download(), dK, dtype, "attention dK")
        # a second call overwrites, it does not accumulate
        capi.nnt_attention_bwd(ctx.h, tQ.h, tK.h, tV.h, tB.h, tS.h, tdB.h, scale, causal, tdQ.h, tdK.h, tdV.h)
        check(tdK.download(), dK, dtype, "attention dK, second call")


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
