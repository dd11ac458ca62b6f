"""GPU parity of the single-tile kernels against the fp64 oracle, element by
element, through the C ABI.  Sizes span several macro-tiles and ragged tails;
both vector and scalar (misaligned / odd-extent) paths are exercised."""
import itertools
import math

import numpy as np
import pytest
import torch

from gpu_util import TOL, check, code, from_dev, quant, relerr, stream_ptr, to_dev
from oracle import definition as D

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def capi():
    from paper_2504_13236_amd import capi as m
    return m


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ GEMM
GEMM_SHAPES = [(5, 4, 7), (33, 65, 17), (128, 128, 64), (200, 130, 100), (64, 300, 400), (100, 257, 33),
               (128, 520, 48), (400, 224, 400), (260, 260, 16)]


def run_gemm(capi, din, dout, opA, opB, m, n, k, batch, alpha, beta, pad=0, misalign=0, seed=0):
    r = rng(seed)
    a_shape = (m, k) if opA == "N" else (k, m)
    b_shape = (k, n) if opB == "N" else (n, k)
    lda, ldb, ldc = a_shape[0] + pad, b_shape[0] + pad, m + pad
    A = quant(r.standard_normal(a_shape + (batch,)), din)
    B = quant(r.standard_normal(b_shape + (batch,)), din)
    C0 = quant(r.standard_normal((m, n, batch)), dout)

    def padded(M, ld):
        P = np.zeros((ld,) + M.shape[1:], np.float32)
        P[:M.shape[0]] = M
        return P
    dA = to_dev(padded(A, lda), din)
    dB = to_dev(padded(B, ldb), din)
    dC = to_dev(padded(C0, ldc), dout)
    if misalign:
        # shift every operand by `misalign` elements so that no 16-byte vector access is possible
        def shift(t):
            s = torch.zeros(t.numel() + misalign, dtype=t.dtype, device=t.device)
            s[misalign:] = t
            return s
        dA, dB, dC = shift(dA), shift(dB), shift(dC)
    esz_in = 4 if din == "f32" else 2
    esz_out = 4 if dout == "f32" else 2
    capi.nnt_tile_gemm(stream_ptr(), code(din), code(dout), 0 if opA == "N" else 1, 0 if opB == "N" else 1,
                       m, n, k, batch, alpha,
                       dA.data_ptr() + misalign * esz_in, lda, lda * a_shape[1],
                       dB.data_ptr() + misalign * esz_in, ldb, ldb * b_shape[1],
                       beta, dC.data_ptr() + misalign * esz_out, ldc, ldc * n)
    torch.cuda.synchronize()
    got = from_dev(dC[misalign:], (ldc, n, batch))[:m]
    ref = D.matmul2d(alpha, opA, A, opB, B, beta, C0)
    return got, ref


@pytest.mark.parametrize("opA,opB", list(itertools.product("NT", "NT")))
@pytest.mark.parametrize("m,n,k", GEMM_SHAPES)
def test_gemm_f32(capi, opA, opB, m, n, k):
    for batch, alpha, beta, pad in ((1, 1.0, 0.0, 0), (3, 0.7, -1.3, 4)):
        got, ref = run_gemm(capi, "f32", "f32", opA, opB, m, n, k, batch, alpha, beta, pad, seed=m + n + k)
        check(got, ref, "f32", "gemm f32 %s%s %dx%dx%d b%d" % (opA, opB, m, n, k, batch))


@pytest.mark.parametrize("opA,opB", list(itertools.product("NT", "NT")))
@pytest.mark.parametrize("m,n,k", GEMM_SHAPES)
@pytest.mark.parametrize("dout", ["f32", "bf16"])
def test_gemm_bf16(capi, opA, opB, m, n, k, dout):
    for batch, alpha, beta, pad in ((1, 1.0, 0.0, 0), (3, 0.7, -1.3, 8)):
        got, ref = run_gemm(capi, "bf16", dout, opA, opB, m, n, k, batch, alpha, beta, pad, seed=m + n + k + 1)
        # fp32 output of bf16 inputs carries only accumulation error; bf16 output adds one rounding
        tol = 1e-5 if dout == "f32" else 2e-2
        e = relerr(got, ref)
        assert e <= tol, ("gemm bf16->%s %s%s %dx%dx%d" % (dout, opA, opB, m, n, k), e)


@pytest.mark.parametrize("din,dout", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32")])
@pytest.mark.parametrize("opA,opB", list(itertools.product("NT", "NT")))
def test_gemm_scalar_path_misaligned_and_odd_ld(capi, din, dout, opA, opB):
    got, ref = run_gemm(capi, din, dout, opA, opB, 70, 45, 37, 2, 1.0, 0.5, pad=3, misalign=1, seed=9)
    e = relerr(got, ref)
    assert e <= (2e-2 if dout == "bf16" else 1e-5), e


@pytest.mark.parametrize("din,dout,m,n,k", [("f32", "f32", 512, 1100, 768), ("bf16", "bf16", 768, 1100, 512),
                                            ("bf16", "f32", 512, 512, 2048), ("f32", "f32", 64, 1024, 1024),
                                            ("bf16", "bf16", 128, 1024, 1024)])
def test_gemm_multi_macro_tile(capi, din, dout, m, n, k):
    for opA, opB in (("N", "N"), ("T", "N"), ("N", "T")):
        got, ref = run_gemm(capi, din, dout, opA, opB, m, n, k, 1, 1.0, 0.0, seed=3)
        e = relerr(got, ref)
        assert e <= (2e-2 if dout == "bf16" else 1e-5), (opA, opB, e)


@pytest.mark.parametrize("dout", ["f32", "bf16"])
@pytest.mark.parametrize("opA,opB", list(itertools.product("NT", "NT")))
@pytest.mark.parametrize("m,n,k", [(256, 256, 32), (512, 768, 96), (768, 256, 416)])
def test_gemm_bf16_whole_macro_tiles_aligned(capi, opA, opB, m, n, k, dout):
    """Shapes made of whole 256 x 256 macro-tiles with k a multiple of 32 and 16-byte aligned operands:
    the kernel that loads straight into LDS (short and long k, padded leading dimensions, batch, beta)."""
    for batch, alpha, beta, pad in ((1, 1.0, 0.0, 0), (2, 0.7, -1.3, 8)):
        got, ref = run_gemm(capi, "bf16", dout, opA, opB, m, n, k, batch, alpha, beta, pad, seed=m + n + k)
        e = relerr(got, ref)
        assert e <= (2e-2 if dout == "bf16" else 1e-5), ("gemm bf16->%s %s%s %dx%dx%d b%d" % (dout, opA, opB, m, n, k, batch), e)


@pytest.mark.parametrize("opA,opB", list(itertools.product("NT", "NT")))
@pytest.mark.parametrize("m,n,k", [(128, 128, 32), (256, 384, 96), (512, 256, 416), (64, 128, 32), (64, 384, 224)])
def test_gemm_f32_whole_macro_tiles_aligned(capi, opA, opB, m, n, k):
    """fp32 shapes made of whole 128 x 128 (64 x 128 for 64 rows) macro-tiles with k a multiple of 32 and 16-byte aligned operands:
    the fp32 kernel that loads straight into LDS (short and long k, padded leading dimensions, batch, beta)."""
    for batch, alpha, beta, pad in ((1, 1.0, 0.0, 0), (2, 0.7, -1.3, 4)):
        got, ref = run_gemm(capi, "f32", "f32", opA, opB, m, n, k, batch, alpha, beta, pad, seed=m + n + k)
        check(got, ref, "f32", "gemm f32 %s%s %dx%dx%d b%d" % (opA, opB, m, n, k, batch))


@pytest.mark.parametrize("m,n", [(64, 128), (256, 256), (192, 384), (128, 200), (100, 256)])
@pytest.mark.parametrize("k", [32, 64])
def test_gemm_f32_whole_contraction_resident(capi, m, n, k):
    """fp32 products A^T B with a contraction of 32 or 64 (a head size) and both operands k-contiguous, the form of
    the scores K^T Q: whole 64 x 128 macro-tiles run in the kernel that holds the whole contraction in LDS, the last
    two shapes have ragged edges and leave it; batch, alpha / beta and padded leading dimensions."""
    for batch, alpha, beta, pad in ((1, 1.0, 0.0, 0), (5, 0.125, 0.0, 0), (3, 0.7, -1.3, 4)):
        got, ref = run_gemm(capi, "f32", "f32", "T", "N", m, n, k, batch, alpha, beta, pad, seed=7 * m + n + k)
        check(got, ref, "f32", "gemm f32 TN %dx%dx%d b%d" % (m, n, k, batch))


def test_gemm_direct_load_randomized_sweep(capi):
    """Seeded random draws over the shapes that qualify for the kernels which load straight into LDS and
    keep fragment reads in flight between the matrix instructions: m, n multiples of the macro-tile, k
    multiples of 32 (32 and 64 included), every operand orientation, batch, alpha / beta, padded leading
    dimensions; each compared element by element with the oracle's product.  Stops at the first failure."""
    r = np.random.default_rng(20250413)
    for draw in range(160):
        din = ("f32", "bf16")[draw % 2]
        dout = din if din == "f32" else ("bf16", "f32")[(draw // 2) % 2]
        unit_m, unit_n = (128, 128) if din == "f32" else (256, (256, 128)[int(r.integers(2))])
        if din == "f32" and r.integers(4) == 0:
            unit_m = 64                                     # the 64 x 128 fp32 shape
        m = unit_m * int(r.integers(1, 4 if din == "f32" else 3))
        n = unit_n * int(r.integers(1, 4))
        k = 32 * int(r.choice([1, 2, 2, 3, 4, 5, 7, 8, 12, 16]))
        opA, opB = "NT"[int(r.integers(2))], "NT"[int(r.integers(2))]
        batch = int(r.integers(1, 4))
        alpha, beta = ((1.0, 0.0), (0.7, -1.3), (-2.0, 1.0))[int(r.integers(3))]
        pad = (4 if din == "f32" else 8) * int(r.integers(0, 3))
        got, ref = run_gemm(capi, din, dout, opA, opB, m, n, k, batch, alpha, beta, pad, seed=1000 + draw)
        e = relerr(got, ref)
        assert e <= TOL[dout], ("draw %d: %s->%s %s%s %dx%dx%d batch %d alpha %g beta %g pad %d" %
                                (draw, din, dout, opA, opB, m, n, k, batch, alpha, beta, pad), e)


def test_gemm_bf16_ragged_shapes_randomized_sweep(capi):
    """bf16 products whose extents are multiples of 8 but of nothing larger (macro-tiles that end inside the
    matrix, a short last k-step, k shorter than one step): the shapes of the direct-load kernel's ragged
    variant and its neighbours, every orientation, against the oracle.  Stops at the first failure."""
    r = np.random.default_rng(4004)
    for draw in range(72):
        dout = ("bf16", "f32")[draw % 2]
        m = 8 * int(r.integers(20, 90))
        n = 8 * int(r.integers(16, 120))
        k = 8 * int(r.choice([1, 2, 3, 4, 5, 7, 13, 28, 50, 51, 64, 70]))
        opA, opB = "NT"[int(r.integers(2))], "NT"[int(r.integers(2))]
        batch = 1 if draw % 3 else 2
        alpha, beta = ((1.0, 0.0), (0.7, -1.3))[int(r.integers(2))]
        pad = 8 * int(r.integers(0, 3))
        got, ref = run_gemm(capi, "bf16", dout, opA, opB, m, n, k, batch, alpha, beta, pad, seed=5000 + draw)
        e = relerr(got, ref)
        assert e <= TOL[dout], ("draw %d: bf16->%s %s%s %dx%dx%d batch %d alpha %g beta %g pad %d" %
                                (draw, dout, opA, opB, m, n, k, batch, alpha, beta, pad), e)


def test_gemm_bf16_few_rows_randomized_sweep(capi):
    """bf16 products with at most 128 rows (m = head size in the attention layer: 64, 128, and whatever else a
    caller may bring) against long and short second operands: the 128 x 128 direct-load shape with its clamped
    loads (macro-tiles mostly empty, columns that end anywhere, a short last k-step, k shorter than a step) and
    the general kernel for what it does not take (extents that are not multiples of 8).  Every orientation,
    batches, against the oracle; stops at the first failure."""
    r = np.random.default_rng(128128)
    for draw in range(96):
        dout = ("bf16", "f32")[draw % 2]
        m = int(r.choice([8, 16, 24, 40, 64, 64, 72, 96, 120, 128, 128, 20, 100]))
        n = int(r.choice([8 * int(r.integers(1, 100)), 128 * int(r.integers(1, 6)), int(r.integers(1, 300))]))
        k = int(r.choice([8 * int(r.integers(1, 40)), 32 * int(r.integers(1, 12)), int(r.integers(1, 200))]))
        opA, opB = "NT"[int(r.integers(2))], "NT"[int(r.integers(2))]
        batch = int(r.choice([1, 1, 2, 5]))
        alpha, beta = ((1.0, 0.0), (0.7, -1.3))[int(r.integers(2))]
        pad = 8 * int(r.integers(0, 3))
        got, ref = run_gemm(capi, "bf16", dout, opA, opB, m, n, k, batch, alpha, beta, pad, seed=7000 + draw)
        e = relerr(got, ref)
        assert e <= TOL[dout], ("draw %d: bf16->%s %s%s %dx%dx%d batch %d alpha %g beta %g pad %d" %
                                (draw, dout, opA, opB, m, n, k, batch, alpha, beta, pad), e)


def test_gemm_degenerate(capi):
    # k = 0: C <- beta * C; beta = 0 must not propagate NaNs already in C
    C0 = rng(1).standard_normal((9, 5)).astype(np.float32)
    dC = to_dev(C0)
    dummy = to_dev(np.zeros((9, 1), np.float32))
    capi.nnt_tile_gemm(stream_ptr(), 0, 0, 0, 0, 9, 5, 0, 1, 1.0, dummy.data_ptr(), 9, 0, dummy.data_ptr(), 1, 0, 2.0,
                       dC.data_ptr(), 9, 45)
    torch.cuda.synchronize()
    np.testing.assert_allclose(from_dev(dC, (9, 5)), 2.0 * C0, rtol=1e-6)
    A = rng(2).standard_normal((9, 6)).astype(np.float32)
    B = rng(3).standard_normal((6, 5)).astype(np.float32)
    dC = to_dev(np.full((9, 5), np.nan, np.float32))
    dA, dB = to_dev(A), to_dev(B)
    capi.nnt_tile_gemm(stream_ptr(), 0, 0, 0, 0, 9, 5, 6, 1, 1.0, dA.data_ptr(), 9, 54, dB.data_ptr(), 6, 30, 0.0,
                       dC.data_ptr(), 9, 45)
    torch.cuda.synchronize()
    check(from_dev(dC, (9, 5)), A.astype(np.float64) @ B.astype(np.float64), "f32", "beta=0 over NaN")


# ------------------------------------------------------------------ elementwise
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,off", [(1, 0), (1000, 0), (4096 * 9 + 5, 0), (777, 1)])
def test_fill_add_gelu_cast(capi, dtype, n, off):
    r = rng(n)
    esz = 4 if dtype == "f32" else 2
    x = quant(r.standard_normal(n + off) * 3, dtype)
    y = quant(r.standard_normal(n + off), dtype)
    dx, dy = to_dev(x, dtype), to_dev(y, dtype)
    px, py = dx.data_ptr() + off * esz, dy.data_ptr() + off * esz
    st = stream_ptr()
    capi.nnt_tile_add(st, code(dtype), n, 0.5, px, -2.0, py)
    torch.cuda.synchronize()
    check(from_dev(dy, (n + off,))[off:], 0.5 * x[off:] - 2.0 * y[off:], dtype, "add")
    for variant, name in ((0, "tanh"), (1, "erf")):
        capi.nnt_tile_gelu(st, code(dtype), variant, n, px, py)
        torch.cuda.synchronize()
        check(from_dev(dy, (n + off,))[off:], D.gelu(x[off:], name), dtype, "gelu " + name)
        dg = to_dev(quant(r.standard_normal(n + off), dtype), dtype)
        g = from_dev(dg, (n + off,))
        capi.nnt_tile_gelu_bwd(st, code(dtype), variant, n, px, dg.data_ptr() + off * esz, py)
        torch.cuda.synchronize()
        check(from_dev(dy, (n + off,))[off:], g[off:] * D.gelu_grad(x[off:], name), dtype, "gelu_bwd " + name)
    capi.nnt_tile_fill(st, code(dtype), n, 1.25, py)
    torch.cuda.synchronize()
    assert np.all(from_dev(dy, (n + off,))[off:] == 1.25)
    if off:
        assert from_dev(dy, (n + off,))[0] != 1.25       # nothing written before the tile


@pytest.mark.parametrize("n", [8, 1001, 70000])
def test_cast_matches_rne(capi, n):
    x = (rng(n).standard_normal(n) * 100).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -0.0, 3.3e38][:min(4, n)]
    dx = to_dev(x)
    dy = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    capi.nnt_tile_cast(stream_ptr(), 0, 1, n, dx.data_ptr(), dy.data_ptr())
    torch.cuda.synchronize()
    got = dy.to(torch.float32).cpu().numpy()
    np.testing.assert_array_equal(got.view(np.uint32), D.round_to_bf16(x).view(np.uint32))     # bit exact
    dz = torch.empty(n, dtype=torch.float32, device="cuda")
    capi.nnt_tile_cast(stream_ptr(), 1, 0, n, dy.data_ptr(), dz.data_ptr())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(dz.cpu().numpy(), got)


def test_copy_block(capi):
    src = rng(4).standard_normal((6, 5, 4, 3)).astype(np.float32)
    d_src = to_dev(src)
    dst = np.zeros((7, 6, 5, 4), np.float32)
    d_dst = to_dev(dst)
    ext = [3, 2, 4, 2]
    s_str = [1, 6, 30, 120]
    d_str = [1, 7, 42, 210]
    s_off = 1 + 6 * 2 + 30 * 0 + 120 * 1
    d_off = 2 + 7 * 1 + 42 * 1 + 210 * 0
    capi.nnt_tile_copy_block(stream_ptr(), 0, 4, capi.i64_array(ext), d_src.data_ptr() + 4 * s_off, capi.i64_array(s_str),
                             d_dst.data_ptr() + 4 * d_off, capi.i64_array(d_str))
    torch.cuda.synchronize()
    dst[2:5, 1:3, 1:5, 0:2] = src[1:4, 2:4, 0:4, 1:3]
    np.testing.assert_array_equal(from_dev(d_dst, dst.shape), dst)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("m,n", [(256, 512), (400, 224), (33, 1000), (1024, 70)])
def test_bias_add_and_grad(capi, dtype, m, n):
    r = rng(m * n)
    Y = quant(r.standard_normal((m, n)), dtype)
    b = r.standard_normal(m).astype(np.float32)
    dY, db = to_dev(Y, dtype), to_dev(b)
    capi.nnt_tile_bias_add(stream_ptr(), code(dtype), m, n, db.data_ptr(), dY.data_ptr())
    torch.cuda.synchronize()
    check(from_dev(dY, (m, n)), D.bias_add(Y, b), dtype, "bias_add")
    dY = to_dev(Y, dtype)
    scratch = torch.empty(capi.nnt_tile_bias_grad_scratch(m, n), dtype=torch.float32, device="cuda")
    g0 = r.standard_normal(m).astype(np.float32)
    dg = to_dev(g0)
    capi.nnt_tile_bias_grad(stream_ptr(), code(dtype), m, n, dY.data_ptr(), dg.data_ptr(), 0, scratch.data_ptr())
    torch.cuda.synchronize()
    check(from_dev(dg, (m,)), D.bias_grad(Y), "f32", "bias_grad")
    capi.nnt_tile_bias_grad(stream_ptr(), code(dtype), m, n, dY.data_ptr(), dg.data_ptr(), 1, scratch.data_ptr())
    torch.cuda.synchronize()
    check(from_dev(dg, (m,)), 2 * D.bias_grad(Y), "f32", "bias_grad accumulate")


# ------------------------------------------------------------------ layer norm in tile steps
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("parts,n", [((256, 256, 256), 300), ((400, 400, 400, 400), 96), ((32, 32), 64), ((37, 91), 50)])
def test_layernorm_tile_steps(capi, dtype, parts, n):
    r = rng(sum(parts) + n)
    N = sum(parts)
    eps = 1e-5
    X = quant(r.standard_normal((N, n)) * 2 + 0.7, dtype)
    gamma = (1 + 0.1 * r.standard_normal(N)).astype(np.float32)
    beta = (0.1 * r.standard_normal(N)).astype(np.float32)
    Yref, mean, rstd = D.layernorm_fwd(X, gamma, beta, eps)
    st = stream_ptr()
    stats = torch.empty(2 * n, dtype=torch.float32, device="cuda")
    tiles, lo = [], 0
    for mpart in parts:
        tiles.append((lo, mpart, to_dev(X[lo:lo + mpart], dtype)))
        lo += mpart
    before = 0
    for i, (lo, mpart, dx) in enumerate(tiles):          # step 1, tile after tile
        fin = N if i == len(tiles) - 1 else 0
        capi.nnt_tile_ln_stats(st, code(dtype), mpart, n, dx.data_ptr(), stats.data_ptr(), before, fin, eps)
        before += mpart
    torch.cuda.synchronize()
    s = from_dev(stats, (2, n))
    check(s[0], mean, "f32", "ln mean")
    check(s[1], rstd, "f32", "ln rstd")
    dgm, dbt = to_dev(gamma), to_dev(beta)
    for lo, mpart, dx in tiles:                           # steps 2 and 3
        dy = torch.empty_like(dx)
        capi.nnt_tile_ln_apply(st, code(dtype), mpart, n, dx.data_ptr(), stats.data_ptr(), dgm.data_ptr() + 4 * lo,
                               dbt.data_ptr() + 4 * lo, dy.data_ptr())
        torch.cuda.synchronize()
        check(from_dev(dy, (mpart, n)), Yref[lo:lo + mpart], dtype, "ln apply")
    # backward
    dY = quant(r.standard_normal((N, n)), dtype)
    dRes = quant(r.standard_normal((N, n)), dtype)
    dXref, dgref, dbref = D.layernorm_bwd(X, gamma, mean, rstd, dY)
    sums = torch.empty(2 * n, dtype=torch.float32, device="cuda")
    dys = [to_dev(dY[lo:lo + mpart], dtype) for lo, mpart, _ in tiles]
    for i, (lo, mpart, dx) in enumerate(tiles):
        capi.nnt_tile_ln_bwd_sums(st, code(dtype), mpart, n, dx.data_ptr(), stats.data_ptr(), dgm.data_ptr() + 4 * lo,
                                  dys[i].data_ptr(), sums.data_ptr(), 1 if i == 0 else 0)
    for i, (lo, mpart, dx) in enumerate(tiles):
        out = torch.empty_like(dx)
        dres = to_dev(dRes[lo:lo + mpart], dtype)
        capi.nnt_tile_ln_bwd_dx(st, code(dtype), mpart, n, N, dx.data_ptr(), stats.data_ptr(), dgm.data_ptr() + 4 * lo,
                                dys[i].data_ptr(), sums.data_ptr(), dres.data_ptr(), out.data_ptr())
        torch.cuda.synchronize()
        e = relerr(from_dev(out, (mpart, n)), (dXref + dRes)[lo:lo + mpart])
        assert e <= TOL[dtype], ("ln bwd dx", e)
        capi.nnt_tile_ln_bwd_dx(st, code(dtype), mpart, n, N, dx.data_ptr(), stats.data_ptr(), dgm.data_ptr() + 4 * lo,
                                dys[i].data_ptr(), sums.data_ptr(), None, out.data_ptr())
        torch.cuda.synchronize()
        e = relerr(from_dev(out, (mpart, n)), dXref[lo:lo + mpart])
        assert e <= TOL[dtype], ("ln bwd dx no residual", e)
        scratch = torch.empty(capi.nnt_tile_ln_bwd_params_scratch(mpart, n), dtype=torch.float32, device="cuda")
        dg = torch.empty(mpart, dtype=torch.float32, device="cuda")
        dbv = torch.empty(mpart, dtype=torch.float32, device="cuda")
        capi.nnt_tile_ln_bwd_params(st, code(dtype), mpart, n, dx.data_ptr(), stats.data_ptr(), dys[i].data_ptr(),
                                    dg.data_ptr(), dbv.data_ptr(), 0, scratch.data_ptr())
        torch.cuda.synchronize()
        assert relerr(from_dev(dg, (mpart,)), dgref[lo:lo + mpart]) <= 1e-5
        assert relerr(from_dev(dbv, (mpart,)), dbref[lo:lo + mpart]) <= 1e-5


# ------------------------------------------------------------------ softmax in two subroutines
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("parts,tq,batch,q0", [((256, 256), 256, 3, 256), ((64, 64, 64), 50, 2, 140), ((33, 20), 53, 2, 0),
                                               ((128,), 128, 4, 0)])
@pytest.mark.parametrize("causal", [0, 1])
def test_softmax_tile_subroutines(capi, dtype, parts, tq, batch, q0, causal):
    r = rng(sum(parts) + tq)
    nk = sum(parts)
    scale = 0.125
    A = quant(r.standard_normal((nk, tq, batch)) * 4, dtype)
    # the reference works on global indices: embed the tile column range into a full problem
    full = np.full((nk, q0 + tq, batch), 0.0)
    full[:, q0:] = A
    Pref, tmax, den = D.softmax_fwd(scale * full, causal=bool(causal))
    Pref, tmax, den = Pref[:, q0:], tmax[q0:], den[q0:]
    st = stream_ptr()
    stats = torch.empty(2 * tq * batch, dtype=torch.float32, device="cuda")
    tiles, k0 = [], 0
    for tk in parts:
        tiles.append((k0, tk, to_dev(A[k0:k0 + tk], dtype)))
        k0 += tk
    for i, (k0, tk, da) in enumerate(tiles):
        capi.nnt_tile_softmax_stats(st, code(dtype), tk, tq, batch, k0, q0, causal, scale, da.data_ptr(), stats.data_ptr(),
                                    1 if i == 0 else 0)
    torch.cuda.synchronize()
    s = from_dev(stats, (2, tq, batch))
    check(s[0], tmax, "f32", "softmax max")
    check(s[1], den, "f32", "softmax denominator")
    for k0, tk, da in tiles:
        capi.nnt_tile_softmax_apply(st, code(dtype), tk, tq, batch, k0, q0, causal, scale, da.data_ptr(), stats.data_ptr())
        torch.cuda.synchronize()
        got = from_dev(da, (tk, tq, batch))
        check(got, Pref[k0:k0 + tk], dtype, "softmax apply")
        if causal:
            masked = (k0 + np.arange(tk))[:, None] > (q0 + np.arange(tq))[None, :]
            assert np.all(got[masked] == 0.0)
    # backward on the exact probabilities the device holds
    P = np.concatenate([from_dev(da, (tk, tq, batch)) for _, tk, da in tiles], axis=0)
    dP = quant(r.standard_normal(P.shape), dtype)
    ref = D.softmax_bwd(P, dP)
    dots = torch.empty(tq * batch, dtype=torch.float32, device="cuda")
    dps = [to_dev(dP[k0:k0 + tk], dtype) for k0, tk, _ in tiles]
    for i, (k0, tk, da) in enumerate(tiles):
        capi.nnt_tile_softmax_bwd_dot(st, code(dtype), tk, tq, batch, da.data_ptr(), dps[i].data_ptr(), dots.data_ptr(),
                                      1 if i == 0 else 0)
    for i, (k0, tk, da) in enumerate(tiles):
        capi.nnt_tile_softmax_bwd_apply(st, code(dtype), tk, tq, batch, da.data_ptr(), dps[i].data_ptr(), dots.data_ptr())
    torch.cuda.synchronize()
    got = np.concatenate([from_dev(dps[i], (tk, tq, batch)) for i, (_, tk, _) in enumerate(tiles)], axis=0)
    check(got, ref, dtype, "softmax bwd")


# ------------------------------------------------------------------ Adam
@pytest.mark.parametrize("n", [3, 1000, 100003])
@pytest.mark.parametrize("wd", [0.0, 0.1])
def test_adam_tile(capi, n, wd):
    r = rng(n)
    p = r.standard_normal(n).astype(np.float32)
    m = (0.1 * r.standard_normal(n)).astype(np.float32)
    v = (r.random(n) * 0.01).astype(np.float32)
    g = r.standard_normal(n).astype(np.float32)
    g[0] = 0.0
    dp, dm, dv, dg = to_dev(p), to_dev(m), to_dev(v), to_dev(g)
    lp = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    pr, mr, vr = p.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
    for step in (1, 2, 3):
        capi.nnt_tile_adam(stream_ptr(), n, step, 1e-3, 0.9, 0.999, 1e-8, wd, dg.data_ptr(), dp.data_ptr(), dm.data_ptr(),
                           dv.data_ptr(), lp.data_ptr())
        pr, mr, vr = D.adam_step(pr, g, mr, vr, step, weight_decay=wd)
    torch.cuda.synchronize()
    check(from_dev(dp, (n,)), pr, "f32", "adam p")
    check(from_dev(dm, (n,)), mr, "f32", "adam m")
    check(from_dev(dv, (n,)), vr, "f32", "adam v")
    # the low-precision copy is the bf16 rounding of the fp32 parameter the device holds
    got_lp = lp.to(torch.float32).cpu().numpy()
    np.testing.assert_array_equal(got_lp.view(np.uint32), D.round_to_bf16(dp.cpu().numpy()).view(np.uint32))


def test_adam_tile_with_state_beyond_the_caches(capi):
    """One tile whose optimiser state (30 bytes per parameter) exceeds 1 GiB: the kernel streams it with
    non-temporal accesses.  Two steps against the oracle, every element; a ragged tail of three."""
    n = 36 * 1024 * 1024 + 3
    r = rng(36)
    p = r.standard_normal(n).astype(np.float32)
    g = r.standard_normal(n).astype(np.float32)
    dp, dm, dv, dg = to_dev(p), to_dev(np.zeros(n, np.float32)), to_dev(np.zeros(n, np.float32)), to_dev(g)
    lp = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    pr, mr, vr = p.astype(np.float64), np.zeros(n), np.zeros(n)
    for step in (1, 2):
        capi.nnt_tile_adam(stream_ptr(), n, step, 1e-3, 0.9, 0.999, 1e-8, 0.01, dg.data_ptr(), dp.data_ptr(), dm.data_ptr(),
                           dv.data_ptr(), lp.data_ptr())
        pr, mr, vr = D.adam_step(pr, g, mr, vr, step, weight_decay=0.01)
    torch.cuda.synchronize()
    check(from_dev(dp, (n,)), pr, "f32", "adam p")
    check(from_dev(dm, (n,)), mr, "f32", "adam m")
    check(from_dev(dv, (n,)), vr, "f32", "adam v")
    got_lp = lp.to(torch.float32).cpu().numpy()
    np.testing.assert_array_equal(got_lp.view(np.uint32), D.round_to_bf16(dp.cpu().numpy()).view(np.uint32))


def test_adam_first_step_closed_form(capi):
    n = 64
    g = rng(5).standard_normal(n).astype(np.float32)
    p0 = rng(6).standard_normal(n).astype(np.float32)
    dp, dm, dv, dg = to_dev(p0), to_dev(np.zeros(n)), to_dev(np.zeros(n)), to_dev(g)
    capi.nnt_tile_adam(stream_ptr(), n, 1, 1e-3, 0.9, 0.999, 1e-8, 0.0, dg.data_ptr(), dp.data_ptr(), dm.data_ptr(),
                       dv.data_ptr(), None)
    torch.cuda.synchronize()
    want = p0.astype(np.float64) - 1e-3 * g / (np.abs(g) + 1e-8)
    check(from_dev(dp, (n,)), want, "f32", "adam closed form")


# ------------------------------------------------------------------ SGD with momentum
@pytest.mark.parametrize("n", [3, 1000, 100003])
@pytest.mark.parametrize("nesterov", [0, 1])
def test_sgd_tile(capi, n, nesterov):
    r = rng(n + nesterov)
    p = r.standard_normal(n).astype(np.float32)
    dp, dv = to_dev(p), to_dev(np.zeros(n))
    lp = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    pr, vr = p.astype(np.float64), np.zeros(n)
    for step in range(3):
        g = r.standard_normal(n).astype(np.float32)
        dg = to_dev(g)
        capi.nnt_tile_sgd(stream_ptr(), n, 0.05, 0.9, 0.01, nesterov, dg.data_ptr(), dp.data_ptr(), dv.data_ptr(), lp.data_ptr())
        torch.cuda.synchronize()
        pr, vr = D.sgd_step(pr, g, vr, 0.05, 0.9, 0.01, bool(nesterov))
    check(from_dev(dp, (n,)), pr, "f32", "sgd p")
    check(from_dev(dv, (n,)), vr, "f32", "sgd v")
    got_lp = lp.to(torch.float32).cpu().numpy()
    np.testing.assert_array_equal(got_lp.view(np.uint32), D.round_to_bf16(dp.cpu().numpy()).view(np.uint32))
    assert capi.nnt_tile_sgd.raw(stream_ptr(), n, 0.05, -0.1, 0.0, 0, dg.data_ptr(), dp.data_ptr(), dv.data_ptr(), None) == capi.NNT_EINVAL


def test_tile_calls_reject_bad_arguments(capi):
    x = torch.zeros(16, device="cuda")
    st = stream_ptr()
    assert capi.nnt_tile_add.raw(st, 3, 16, 1.0, x.data_ptr(), 0.0, x.data_ptr()) == capi.NNT_EDTYPE
    assert capi.nnt_tile_add.raw(st, 0, -1, 1.0, x.data_ptr(), 0.0, x.data_ptr()) == capi.NNT_EINVAL
    assert capi.nnt_tile_ln_stats.raw(st, 0, 4, 4, x.data_ptr(), x.data_ptr(), 4, 9, 1e-5) == capi.NNT_EINVAL
    assert capi.nnt_tile_gemm.raw(st, 0, 0, 0, 0, 4, 4, 4, 1, 1.0, x.data_ptr(), 2, 16, x.data_ptr(), 4, 16, 0.0,
                                  x.data_ptr(), 4, 16) == capi.NNT_EINVAL        # lda < m
    assert capi.nnt_tile_softmax_stats.raw(st, 0, 4, 4, 1, -1, 0, 1, 1.0, x.data_ptr(), x.data_ptr(), 1) == capi.NNT_EINVAL
