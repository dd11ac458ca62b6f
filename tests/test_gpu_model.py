"""GPU parity of the embedding layer, the cross-entropy loss over vocabulary tiles and a small
language model assembled from them (embedding -> GPT-2 block -> weight-tied head -> loss),
forward and backward, against the fp64 oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

import workload
from gpu_util import TOL, check, quant, relerr
from oracle import definition as D

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mods():
    from paper_2504_13236_amd import capi, tiled
    return capi, tiled


def T(tiled, ctx, a, base, dtype):
    return tiled.TiledTensor.from_numpy(ctx, np.asarray(a, np.float32), base, dtype)


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(np.asarray(a, np.int32).reshape(-1, order="F"))).cuda()


@pytest.mark.parametrize("wdt,ydt", [("f32", "f32"), ("f32", "bf16"), ("bf16", "bf16")])
def test_embedding_forward_backward(mods, wdt, ydt):
    capi, tiled = mods
    r = np.random.default_rng(11)
    N_e, N_v, N_s, N_b = 72, 300, 50, 3
    W = quant(r.standard_normal((N_e, N_v)), wdt)
    tok = r.integers(0, N_v, (N_s, N_b))
    tok[:5, 0] = 7                                              # several positions share a token
    G = quant(r.standard_normal((N_e, N_s, N_b)), ydt)
    with tiled.Context(n_streams=2) as ctx:
        tW = T(tiled, ctx, W, (32, 128), wdt)
        tY = tiled.TiledTensor(ctx, ydt, (N_e, N_s, N_b), (40, 16, 2))
        dtok = dev_i32(tok)
        capi.nnt_embedding_fwd(ctx.h, dtok.data_ptr(), tW.h, tY.h)
        got = tY.download()
        want = D.embedding_fwd(W, tok)
        if ydt == "bf16":
            want = quant(want, "bf16")
        np.testing.assert_array_equal(got, want.astype(np.float32))          # a copy (and one rounding): exact
        tG = T(tiled, ctx, G, (40, 16, 2), ydt)
        tdW = tiled.TiledTensor.zeros(ctx, (N_e, N_v), (32, 128))
        capi.nnt_embedding_bwd(ctx.h, dtok.data_ptr(), tG.h, tdW.h)
        check(tdW.download(), D.embedding_bwd(G, tok, N_v), "f32", "embedding dW")
        # accumulates: a second call doubles it; out-of-range tokens are ignored
        bad = tok.copy()
        bad[0, 0] = N_v + 5
        bad[1, 0] = -1
        capi.nnt_embedding_bwd(ctx.h, dev_i32(bad).data_ptr(), tG.h, tdW.h)
        ctx.wait()
        G2 = G.copy()
        G2[:, 0, 0] = 0
        G2[:, 1, 0] = 0
        check(tdW.download(), D.embedding_bwd(G, tok, N_v) + D.embedding_bwd(G2, tok, N_v), "f32", "embedding dW, second call")


@pytest.mark.parametrize("gran", [0, 1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_cross_entropy_over_vocabulary_tiles(mods, dtype, gran):
    capi, tiled = mods
    r = np.random.default_rng(12)
    N_v, N_s, N_b = 3000, 40, 3            # two vocabulary tiles of 1500: columns too long for the register-cached softmax
    X = quant(2.0 * r.standard_normal((N_v, N_s, N_b)), dtype)
    lab = r.integers(0, N_v, (N_s, N_b))
    # one column whose label is so unlikely that its probability underflows (the loss must come from the
    # logit and the column statistics, not from the stored probability)
    X[lab[0, 0], 0, 0] = -100.0
    X[(lab[0, 0] + 1) % N_v, 0, 0] = 20.0
    L, losses, dX = D.cross_entropy(X, lab)
    assert losses[0, 0] > 115
    with tiled.Context(n_streams=4, granularity=gran) as ctx:
        tX = T(tiled, ctx, X, (1500, 16, 2), dtype)
        tS = tiled.TiledTensor(ctx, "f32", (2, N_s, N_b), (2, 16, 2))
        dl = dev_i32(lab)
        col = torch.empty(N_s * N_b, device="cuda")
        tot = torch.empty(1, device="cuda")
        capi.nnt_cross_entropy(ctx.h, tX.h, dl.data_ptr(), tS.h, col.data_ptr(), tot.data_ptr())
        ctx.wait()
        check(tX.download(), dX, dtype, "dL/dlogits")
        got_col = col.cpu().numpy().reshape(N_b, N_s).T
        # losses are fp32 results of the logits and the fp32 column statistics whatever the storage type
        assert np.abs(got_col - losses).max() <= TOL["f32"] * np.abs(losses).max()
        assert abs(tot.item() - L) <= TOL["f32"] * abs(L)
        # the total is the per-column losses summed in a fixed order
        assert abs(tot.item() - float(col.double().sum())) <= 1e-6 * abs(L)


def test_small_language_model_forward_backward(mods):
    """tokens -> embedding -> one GPT-2 block -> head tied to the embedding (logits = W_emb^T Out) -> loss;
    backward to the embedding matrix, which collects the head's and the lookup's gradients."""
    capi, tiled = mods
    cfg = workload.CONFIGS[1]
    inp = workload.generate(cfg)
    r = np.random.default_rng(13)
    N_v = 200
    Wemb = (0.5 * r.standard_normal((cfg.N_e, N_v))).astype(np.float32)
    tok = r.integers(0, N_v, (cfg.N_s, cfg.N_b))
    lab = r.integers(0, N_v, (cfg.N_s, cfg.N_b))
    # oracle
    p64 = {k: np.asarray(inp[k], np.float64) for k in workload.PARAM_NAMES}
    W64 = Wemb.astype(np.float64)
    X0 = D.embedding_fwd(W64, tok)
    Out, cache = D.block_forward(p64, X0, cfg.N_h, cfg.eps, cfg.gelu)
    logits = np.einsum("ev,esb->vsb", W64, Out)
    L, _, dlogits = D.cross_entropy(logits, lab)
    dOut = np.einsum("ev,vsb->esb", W64, dlogits)
    dW_head = np.einsum("esb,vsb->ev", Out, dlogits)
    dX0, grads = D.block_backward(p64, cache, dOut, cfg.N_h, cfg.gelu)
    dW = dW_head + D.embedding_bwd(dX0, tok, N_v)
    # device
    tiles = workload.base_tiles(cfg)
    with tiled.Context(n_streams=4) as ctx:
        blk = tiled.Gpt2Block(ctx, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, tiles, dtype="f32", adam=False)
        blk.set_params({k: inp[k] for k in workload.PARAM_NAMES})
        tW = T(tiled, ctx, Wemb, (tiles["e"], 64), "f32")
        tdW = tiled.TiledTensor.zeros(ctx, Wemb.shape, (tiles["e"], 64))
        X, OutT, dOutT, dXT = blk.activation(), blk.activation(), blk.activation(), blk.activation()
        act_base = X.base
        tL = tiled.TiledTensor(ctx, "f32", (N_v, cfg.N_s, cfg.N_b), (64, act_base[1], act_base[2]))
        tS = tiled.TiledTensor(ctx, "f32", (2, cfg.N_s, cfg.N_b), (2, act_base[1], act_base[2]))
        dtok, dlab = dev_i32(tok), dev_i32(lab)
        col = torch.empty(cfg.N_s * cfg.N_b, device="cuda")
        tot = torch.empty(1, device="cuda")
        capi.nnt_embedding_fwd(ctx.h, dtok.data_ptr(), tW.h, X.h)
        blk.forward(X, OutT)
        capi.nnt_gemm(ctx.h, 1.0, 1, tW.h, 0, OutT.h, 0.0, tL.h, 1, 0, None)               # logits = W^T Out
        capi.nnt_cross_entropy(ctx.h, tL.h, dlab.data_ptr(), tS.h, col.data_ptr(), tot.data_ptr())
        capi.nnt_gemm(ctx.h, 1.0, 0, tW.h, 0, tL.h, 0.0, dOutT.h, 1, 0, None)              # dOut = W dlogits
        capi.nnt_gemm(ctx.h, 1.0, 0, OutT.h, 1, tL.h, 0.0, tdW.h, 2, 0, None)              # dW = Out dlogits^T
        blk.backward(dOutT, dXT)
        capi.nnt_embedding_bwd(ctx.h, dtok.data_ptr(), dXT.h, tdW.h)                        # + the lookup's share
        ctx.wait()
        assert abs(tot.item() - L) <= 1e-5 * abs(L)
        check(dOutT.download(), dOut, "f32", "dOut")
        check(tdW.download(), dW, "f32", "embedding matrix gradient")
        for k in workload.PARAM_NAMES:
            assert relerr(blk.grad(k).download(), grads[k]) <= 1e-5, k
        blk.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_two_block_language_model_training_step(mods, dtype):
    """tokens -> token + position embeddings -> two blocks -> final layer norm -> tied head -> loss, the
    whole backward pass and one Adam step, as one flow of tasks (tiled.Gpt2Model), against the oracle's
    composition of the same definitions."""
    capi, tiled = mods
    cfg = workload.CONFIGS[1].replace(dtype=dtype)
    tiles = workload.base_tiles(cfg)
    r = np.random.default_rng(17)
    N_v, tile_v, nblk = 200, 64, 2
    inputs = [workload.generate(cfg.replace(index=1 + 5 * i)) for i in range(nblk)]
    wte = (0.3 * r.standard_normal((cfg.N_e, N_v))).astype(np.float32)
    wpe = (0.1 * r.standard_normal((cfg.N_e, cfg.N_s))).astype(np.float32)
    gf = (1.0 + 0.05 * r.standard_normal(cfg.N_e)).astype(np.float32)
    bf = (0.05 * r.standard_normal(cfg.N_e)).astype(np.float32)
    tok = r.integers(0, N_v, (cfg.N_s, cfg.N_b))
    lab = r.integers(0, N_v, (cfg.N_s, cfg.N_b))
    # oracle
    pos = np.repeat(np.arange(cfg.N_s)[:, None], cfg.N_b, axis=1)
    p64 = [{k: np.asarray(inp[k], np.float64) for k in workload.PARAM_NAMES} for inp in inputs]
    W64, P64 = wte.astype(np.float64), wpe.astype(np.float64)
    X = D.embedding_fwd(W64, tok) + D.embedding_fwd(P64, pos)
    caches = []
    for p in p64:
        X, cache = D.block_forward(p, X, cfg.N_h, cfg.eps, cfg.gelu)
        caches.append(cache)
    Xf, mean, rstd = D.layernorm_fwd(X, gf, bf, cfg.eps)
    logits = np.einsum("ev,esb->vsb", W64, Xf)
    L, _, dlogits = D.cross_entropy(logits, lab)
    dXf = np.einsum("ev,vsb->esb", W64, dlogits)
    dW_head = np.einsum("esb,vsb->ev", Xf, dlogits)
    dX, dgf, dbf = D.layernorm_bwd(X, gf, mean, rstd, dXf)
    grads = [None] * nblk
    for i in reversed(range(nblk)):
        dX, grads[i] = D.block_backward(p64[i], caches[i], dX, cfg.N_h, cfg.gelu)
    dwte = dW_head + D.embedding_bwd(dX, tok, N_v)
    dwpe = D.embedding_bwd(dX, pos, cfg.N_s)
    # device
    with tiled.Context(n_streams=4) as ctx:
        blks = [tiled.Gpt2Block(ctx, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, tiles, dtype=dtype, adam=True) for _ in range(nblk)]
        for b, inp in zip(blks, inputs):
            b.set_params({k: inp[k] for k in workload.PARAM_NAMES})
        model = tiled.Gpt2Model(ctx, blks, N_v, tile_v)
        model.set_params(wte, wpe, gf, bf)
        model.set_batch(tok, lab)
        model.forward()
        model.backward()
        ctx.wait()
        tol = TOL[dtype]
        assert abs(model.loss.item() - L) <= tol * abs(L), (model.loss.item(), L)
        check(model.wte["g"].download(), dwte, dtype, "token embedding gradient")
        check(model.wpe["g"].download(), dwpe, dtype, "position embedding gradient")
        check(model.gamma["g"].download(), dgf, dtype, "final layer norm gain gradient")
        check(model.beta["g"].download(), dbf, dtype, "final layer norm bias gradient")
        for i, b in enumerate(blks):
            for k in workload.PARAM_NAMES:
                assert relerr(b.grad(k).download(), grads[i][k]) <= tol, (i, k)
        model.adam(1, **workload.ADAM)
        ctx.wait()
        new_wte, m_ref, v_ref = D.adam_step(W64, dwte, np.zeros_like(W64), np.zeros_like(W64), 1, **workload.ADAM)
        check(model.wte["m"].download(), m_ref, dtype, "first moment of the token embedding")
        check(model.wte["v"].download(), v_ref, dtype, "second moment of the token embedding")
        # Adam's first step moves an entry by about lr whatever the gradient's size, so the step taken is
        # compared where the gradient is well above its own error (elsewhere its sign is not determined)
        step_gpu = model.wte["p"].download().astype(np.float64) - W64
        moved = np.abs(dwte) > (1e-3 if dtype == "f32" else 0.1) * np.abs(dwte).max()
        assert moved.sum() > 10
        assert relerr(step_gpu[moved], (new_wte - W64)[moved]) <= (1e-4 if dtype == "f32" else 2e-2)
        model.close()
        for b in blks:
            b.close()
