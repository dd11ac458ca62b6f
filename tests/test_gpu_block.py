"""GPU parity of the whole GPT-2 block (forward, backward, Adam) against the fp64
oracle on the seeded workloads, in the launch configurations the benchmark times."""
import numpy as np
import pytest

import workload
from gpu_util import TOL, relerr
from oracle import definition as D

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mods():
    from paper_2504_13236_amd import capi, tiled
    return capi, tiled


def oracle_run(cfg, inp, adam, progress=None):
    say = progress or (lambda stage: None)
    p64 = {k: np.asarray(inp[k], np.float64) for k in workload.PARAM_NAMES}
    if cfg.dtype == "bf16":
        # the block multiplies with bf16 copies of the fp32 master weights
        for k in ("W_qkv", "W_o", "W_1", "W_2"):
            p64[k] = D.round_to_bf16(inp[k]).astype(np.float64)
    Out, cache = D.block_forward(p64, inp["X"], cfg.N_h, cfg.eps, cfg.gelu, progress=say)
    dX, grads = D.block_backward(p64, cache, inp["dOut"], cfg.N_h, cfg.gelu, progress=say)
    del cache
    res = {"Out": Out, "dX": dX, "grads": grads, "p0": {k: np.asarray(inp[k], np.float64) for k in workload.PARAM_NAMES}}
    if adam:
        res["adam"] = {k: D.adam_step(np.asarray(inp[k], np.float64), grads[k], 0.0, 0.0, 1, **workload.ADAM)
                       for k in workload.PARAM_NAMES}
        say("Adam")
    return res


_case_cache = {}


def full_size_case(number, adam, progress=None, **overrides):
    """(config, inputs, oracle results) of a full-size workload; the last one is kept, so that the two
    attention flows of one workload share one run of the fp64 oracle."""
    key = (number, adam, tuple(sorted(overrides.items())))
    if key not in _case_cache:
        _case_cache.clear()
        cfg = workload.CONFIGS[number].replace(**overrides) if overrides else workload.CONFIGS[number]
        inp = workload.generate(cfg)
        _case_cache[key] = (cfg, inp, oracle_run(cfg, inp, adam, progress))
    return _case_cache[key]


@pytest.fixture(scope="module", autouse=True)
def _drop_case_cache():
    yield
    _case_cache.clear()


def gpu_run(tiled, cfg, inp, tiles, adam, gran=0, n_streams=4, serial=False, fused=False):
    out = {}
    with tiled.Context(n_streams=n_streams, granularity=gran, serial=serial) as ctx:
        blk = tiled.Gpt2Block(ctx, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, tiles, dtype=cfg.dtype, eps=cfg.eps,
                              gelu=cfg.gelu, adam=adam, fused_attention=fused)
        blk.set_params({k: inp[k] for k in workload.PARAM_NAMES})
        X, dOut = blk.activation(inp["X"]), blk.activation(inp["dOut"])
        Out, dX = blk.activation(), blk.activation()
        blk.forward(X, Out)
        blk.backward(dOut, dX)
        out["Out"], out["dX"] = Out.download(), dX.download()
        out["grads"] = {k: blk.grad(k).download() for k in workload.PARAM_NAMES}
        if adam:
            blk.adam(1, **workload.ADAM)
            out["adam"] = {k: (blk.param(k).download(), blk.moment(k, "m").download(), blk.moment(k, "v").download())
                           for k in workload.PARAM_NAMES}
        out["stats"] = ctx.stats()
        blk.close()
    return out


# Adam's first step from zero moments moves a parameter by lr * g / (|g| + eps), i.e. by about lr in the
# direction of the gradient's sign whatever its size: the updated parameter is a discontinuous function
# of g at g = 0.  Where the oracle's gradient is well above the error the device's gradient may carry
# (a multiple of the gradient tolerance), the sign is determined and the parameter is compared with the
# oracle's own; on the complement (gradients that are zero or nearly so, the key bias above all: softmax
# ignores a shift of all keys, so its exact gradient is 0 and the device delivers rounding noise of
# either sign) the device's parameter is compared with the oracle's Adam formula applied to the gradient
# the device produced.
SIGN_SAFE = {"f32": 1e-3, "bf16": 5e-2}      # |g| > SIGN_SAFE * max|g|: 100x / 2.5x the gradient tolerance


def compare_adam_parameter(name, got_p, got_g, ref, dtype):
    """Max-norm relative error of an updated parameter against the oracle, masked as described above."""
    g_ref = np.asarray(ref["grads"][name], np.float64)
    p_ref = ref["adam"][name][0]
    safe = np.abs(g_ref) > SIGN_SAFE[dtype] * np.abs(g_ref).max()
    den = np.abs(p_ref).max()
    err = 0.0
    if safe.any():
        err = float(np.abs(np.asarray(got_p, np.float64) - p_ref)[safe].max() / den)
    if not safe.all():
        p_formula, _, _ = D.adam_step(ref["p0"][name], got_g, 0.0, 0.0, 1, **workload.ADAM)
        err = max(err, float(np.abs(np.asarray(got_p, np.float64) - p_formula)[~safe].max() / den))
    return err, safe


def tolerance_of(key, dtype):
    """The stated tolerance, except for Adam's second moment in bf16 configurations: v = (1 - beta2) g^2 is
    quadratic in the gradient, so a gradient within `tol` of the oracle's (in the max-norm, relative to
    max|g|) gives |v - v_ref| = (1 - beta2) |g + g_ref| |g - g_ref| <= (2 + tol) tol max|v_ref|: twice the
    gradient's tolerance is what the metric can promise for v.  (fp32 stays at the stated 1e-5.)"""
    if dtype == "bf16" and key.startswith("adam_v_"):
        return 2.0 * TOL[dtype] * (1.0 + TOL[dtype])
    return TOL[dtype]


def compare(got, ref, dtype, adam):
    tol = TOL[dtype]
    errs = {"Out": relerr(got["Out"], ref["Out"]), "dX": relerr(got["dX"], ref["dX"])}
    for k in workload.PARAM_NAMES:
        errs["d" + k] = relerr(got["grads"][k], ref["grads"][k])
    if adam:
        for k in workload.PARAM_NAMES:
            for i, nm in ((1, "m"), (2, "v")):
                errs["adam_%s_%s" % (nm, k)] = relerr(got["adam"][k][i], ref["adam"][k][i])
            errs["adam_p_%s" % k], safe = compare_adam_parameter(k, got["adam"][k][0], got["grads"][k], ref, dtype)
            if k == "b_qkv":
                # rows [N_e, 2 N_e) are the key bias: exact gradient 0, never in the sign-safe set
                n = safe.shape[0] // 3
                assert not safe[n:2 * n].any(), "key-bias entries must be compared through the device gradient"
                assert safe[2 * n:].any()
            else:
                assert safe.any(), k
    bad = {k: v for k, v in errs.items() if not v <= tolerance_of(k, dtype)}
    assert not bad, "max-norm relative errors above %.0e: %s" % (tol, bad)
    return errs


@pytest.mark.parametrize("gran", [0, 1])
def test_block_C1_forward_backward_adam(mods, gran):
    capi, tiled = mods
    cfg = workload.CONFIGS[1]
    inp = workload.generate(cfg)
    ref = oracle_run(cfg, inp, True)
    got = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), True, gran=gran)
    compare(got, ref, "f32", True)
    assert got["stats"]["tasks"] > (500 if gran else 30)      # whole-operation flow: ~40 tasks, the Adam step of all parameters is one


@pytest.mark.parametrize("tiles", [dict(e=24, m=56, s=24, b=1, j=1, i=40), dict(e=128, m=512, s=64, b=2, j=2, i=64)])
def test_block_C1_other_tilings_give_the_same_result(mods, tiles):
    """Tiling invariance on the device: ragged / whole tilings against the oracle."""
    capi, tiled = mods
    cfg = workload.CONFIGS[1]
    inp = workload.generate(cfg)
    ref = oracle_run(cfg, inp, False)
    for gran in (0, 1):
        compare(gpu_run(tiled, cfg, inp, tiles, False, gran=gran), ref, "f32", False)


def test_block_serial_and_multistream_are_bit_identical(mods):
    capi, tiled = mods
    cfg = workload.CONFIGS[1]
    inp = workload.generate(cfg)
    a = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), True, gran=1, n_streams=1, serial=True)
    b = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), True, gran=1, n_streams=8)
    c = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), True, gran=0, n_streams=8)
    assert b["stats"]["event_waits"] > 0
    for other in (b,):
        np.testing.assert_array_equal(a["Out"], other["Out"])
        np.testing.assert_array_equal(a["dX"], other["dX"])
        for k in workload.PARAM_NAMES:
            np.testing.assert_array_equal(a["grads"][k], other["grads"][k])
            np.testing.assert_array_equal(a["adam"][k][0], other["adam"][k][0])
    # one launch per operation sums in a different order: equal within fp32 tolerance only
    assert relerr(c["Out"], a["Out"]) < 1e-5 and relerr(c["dX"], a["dX"]) < 1e-5


@pytest.mark.parametrize("gran", [0, 1])
def test_block_C1_fused_attention(mods, gran):
    """The same block with scores, softmax and the product with V replaced by the fused kernels
    (whole heads per tile: tile_i = head size)."""
    capi, tiled = mods
    cfg = workload.CONFIGS[1]
    inp = workload.generate(cfg)
    ref = oracle_run(cfg, inp, True)
    tiles = dict(workload.base_tiles(cfg), i=cfg.h)
    got = gpu_run(tiled, cfg, inp, tiles, True, gran=gran, fused=True)
    compare(got, ref, "f32", True)


def test_block_fused_attention_needs_whole_heads(mods):
    capi, tiled = mods
    cfg = workload.CONFIGS[1]
    with tiled.Context(n_streams=1) as ctx:
        with pytest.raises(capi.NntError):
            tiled.Gpt2Block(ctx, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, dict(workload.base_tiles(cfg), i=32),
                            dtype="f32", fused_attention=True)


def test_block_C1_sgd_momentum_steps(mods):
    """Two forward / backward / SGD-with-momentum iterations of the block against the oracle's."""
    capi, tiled = mods
    cfg = workload.CONFIGS[1]
    inp = workload.generate(cfg)
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=0.01)
    p64 = {k: np.asarray(inp[k], np.float64) for k in workload.PARAM_NAMES}
    vel = {k: 0.0 for k in workload.PARAM_NAMES}
    with tiled.Context(n_streams=4) as ctx:
        blk = tiled.Gpt2Block(ctx, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, workload.base_tiles(cfg), dtype="f32", adam=True)
        blk.set_params({k: inp[k] for k in workload.PARAM_NAMES})
        X, dOut = blk.activation(inp["X"]), blk.activation(inp["dOut"])
        Out, dX = blk.activation(), blk.activation()
        for it in range(2):
            blk.forward(X, Out)
            blk.backward(dOut, dX)
            blk.sgd(**hyper)
            _, cache = D.block_forward(p64, inp["X"], cfg.N_h, cfg.eps, cfg.gelu)
            _, grads = D.block_backward(p64, cache, inp["dOut"], cfg.N_h, cfg.gelu)
            for k in workload.PARAM_NAMES:
                p64[k], vel[k] = D.sgd_step(p64[k], grads[k], vel[k], **hyper)
        for k in workload.PARAM_NAMES:
            assert relerr(blk.param(k).download(), p64[k]) <= 1e-5, k
            assert relerr(blk.moment(k, "m").download(), vel[k]) <= 1e-5, k
        blk.close()


def _two_block_inputs(cfg):
    a = workload.generate(cfg)
    b = workload.generate(cfg.replace(index=cfg.index + 5))      # another seed for the second block's parameters
    return a, b


def _oracle_chain(cfg, pa, pb, X, dOut):
    X1, ca = D.block_forward(pa, X, cfg.N_h, cfg.eps, cfg.gelu)
    X2, cb = D.block_forward(pb, X1, cfg.N_h, cfg.eps, cfg.gelu)
    dX1, gb = D.block_backward(pb, cb, dOut, cfg.N_h, cfg.gelu)
    dX0, ga = D.block_backward(pa, ca, dX1, cfg.N_h, cfg.gelu)
    return X2, dX0, ga, gb


@pytest.mark.parametrize("graph", [False, True], ids=["eager", "graph"])
def test_two_block_chain_forward_backward(mods, graph):
    """Two blocks chained into one flow of tasks (and, with `graph`, replayed three times from one captured
    HIP graph with eager work in between) against the oracle's composition of the two blocks."""
    import ctypes as C
    capi, tiled = mods
    cfg = workload.CONFIGS[1]
    ia, ib = _two_block_inputs(cfg)
    pa = {k: np.asarray(ia[k], np.float64) for k in workload.PARAM_NAMES}
    pb = {k: np.asarray(ib[k], np.float64) for k in workload.PARAM_NAMES}
    Out, dX0, ga, gb = _oracle_chain(cfg, pa, pb, ia["X"], ia["dOut"])
    with tiled.Context(n_streams=4) as ctx:
        blocks = [tiled.Gpt2Block(ctx, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, workload.base_tiles(cfg), dtype="f32", adam=False)
                  for _ in range(2)]
        blocks[0].set_params({k: ia[k] for k in workload.PARAM_NAMES})
        blocks[1].set_params({k: ib[k] for k in workload.PARAM_NAMES})
        st = tiled.Gpt2Stack(ctx, blocks)
        st.acts[0].upload(ia["X"])
        st.dacts[2].upload(ia["dOut"])

        def check_all(tag):
            assert relerr(st.acts[2].download(), Out) <= 1e-5, tag
            assert relerr(st.dacts[0].download(), dX0) <= 1e-5, tag
            for blk, g in ((blocks[0], ga), (blocks[1], gb)):
                for k in workload.PARAM_NAMES:
                    assert relerr(blk.grad(k).download(), g[k]) <= 1e-5, (tag, k)

        st.forward()
        st.backward()
        check_all("eager")
        if graph:
            gh = C.c_void_p()
            capi.nnt_capture_begin(ctx.h)
            st.forward()
            st.backward()
            capi.nnt_capture_end(ctx.h, C.byref(gh))
            for rep in range(3):
                # eager work between the replays: wipe the outputs so that a replay that did nothing would show
                for t in (st.acts[2], st.dacts[0]):
                    capi.nnt_fill(ctx.h, 0.0, t.h)
                ctx.wait()
                capi.nnt_graph_launch(gh)
                ctx.wait()
                check_all("replay %d" % rep)
            capi.nnt_graph_destroy(gh)
        st.close()
        for b in blocks:
            b.close()


def test_gradient_accumulation_over_micro_batches(mods):
    """Parameter gradients of two micro-batches added into accumulators equal the oracle's sum."""
    capi, tiled = mods
    cfg = workload.CONFIGS[1]
    i1 = workload.generate(cfg)
    i2 = workload.generate(cfg.replace(index=cfg.index + 7))
    p64 = {k: np.asarray(i1[k], np.float64) for k in workload.PARAM_NAMES}
    want = {k: 0.0 for k in workload.PARAM_NAMES}
    for inp in (i1, i2):
        _, cache = D.block_forward(p64, inp["X"], cfg.N_h, cfg.eps, cfg.gelu)
        _, g = D.block_backward(p64, cache, inp["dOut"], cfg.N_h, cfg.gelu)
        for k in workload.PARAM_NAMES:
            want[k] = want[k] + 0.5 * g[k]
    with tiled.Context(n_streams=4) as ctx:
        blk = tiled.Gpt2Block(ctx, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, workload.base_tiles(cfg), dtype="f32", adam=False)
        blk.set_params({k: i1[k] for k in workload.PARAM_NAMES})
        acc = [tiled.TiledTensor.zeros(ctx, blk.slots[p].shape, blk.slots[p].base) for p in range(12)]
        X, dOut, Out, dX = blk.activation(), blk.activation(), blk.activation(), blk.activation()
        for inp in (i1, i2):
            X.upload(inp["X"])
            dOut.upload(inp["dOut"])
            blk.forward(X, Out)
            blk.backward(dOut, dX)
            capi.nnt_gpt2_block_grads_axpy(blk.h, 0.5, capi.ptr_array([t.h.value for t in acc]))
            ctx.wait()
        from paper_2504_13236_amd.tiled import PARAM_SLOTS
        for k in workload.PARAM_NAMES:
            assert relerr(acc[PARAM_SLOTS[k]].download(), want[k]) <= 1e-5, k
        blk.close()


def small_bf16_cfg():
    # C3's recipe at a size the oracle finishes at once: bf16 storage, fp32 accumulate and masters, Adam
    return workload.CONFIGS[3].replace(N_e=256, N_h=4, N_m=1024, N_s=192, N_b=2, tile=128)


@pytest.mark.parametrize("gran", [0, 1])
def test_block_bf16_small(mods, gran):
    capi, tiled = mods
    cfg = small_bf16_cfg()
    inp = workload.generate(cfg)
    ref = oracle_run(cfg, inp, True)
    got = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), True, gran=gran)
    compare(got, ref, "bf16", True)


@pytest.mark.parametrize("gran", [0, 1])
def test_block_bf16_small_fused_attention(mods, gran):
    capi, tiled = mods
    cfg = small_bf16_cfg()
    inp = workload.generate(cfg)
    ref = oracle_run(cfg, inp, True)
    got = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), True, gran=gran, fused=True)
    compare(got, ref, "bf16", True)


def test_block_bf16_ragged_tiles(mods):
    # C4's recipe scaled down: tile 100 against N_e = 200 (head size 40 crosses tile edges), sequence 100 + 100 + 56
    capi, tiled = mods
    cfg = workload.CONFIGS[4].replace(N_e=200, N_h=5, N_m=800, N_s=256, N_b=2, tile=100)
    inp = workload.generate(cfg)
    ref = oracle_run(cfg, inp, False)
    got = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), False)
    compare(got, ref, "bf16", False)


def test_block_C2_full_size(mods):
    """The benchmark's workload and launch configuration, every output compared in full."""
    capi, tiled = mods
    cfg, inp, ref = full_size_case(2, False)
    got = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), False)
    errs = compare(got, ref, "f32", False)
    print("C2 max-norm relative errors:", {k: "%.2e" % v for k, v in errs.items()})


def test_block_C2_full_size_fused_attention(mods):
    capi, tiled = mods
    cfg, inp, ref = full_size_case(2, False)
    got = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), False, fused=True)
    errs = compare(got, ref, "f32", False)
    print("C2 (fused attention) max-norm relative errors:", {k: "%.2e" % v for k, v in errs.items()})


def test_block_C3_full_size_bf16(mods):
    capi, tiled = mods
    cfg, inp, ref = full_size_case(3, True)
    got = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), True)
    errs = compare(got, ref, "bf16", True)
    print("C3 max-norm relative errors:", {k: "%.2e" % v for k, v in errs.items()})


def test_block_C3_full_size_bf16_fused_attention(mods):
    capi, tiled = mods
    cfg, inp, ref = full_size_case(3, True)
    got = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), True, fused=True)
    errs = compare(got, ref, "bf16", True)
    print("C3 (fused attention) max-norm relative errors:", {k: "%.2e" % v for k, v in errs.items()})


def test_block_C4_full_size_bf16_ragged_fused_attention(mods):
    """Sequence tiles 400 + 400 + 224: workgroup blocks of 128 and streamed blocks of 64 rows end inside every tile."""
    capi, tiled = mods
    cfg, inp, ref = full_size_case(4, False)
    got = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), False, fused=True)
    errs = compare(got, ref, "bf16", False)
    print("C4 (fused attention) max-norm relative errors:", {k: "%.2e" % v for k, v in errs.items()})


def test_block_C4_full_size_bf16_ragged(mods):
    """GPT-2-XL shape: tile 400 against 1600 / 6400 / 1024 (sequence tiles 400 + 400 + 224, head size 64 crossing tile edges)."""
    capi, tiled = mods
    cfg, inp, ref = full_size_case(4, False)
    got = gpu_run(tiled, cfg, inp, workload.base_tiles(cfg), False)
    errs = compare(got, ref, "bf16", False)
    print("C4 max-norm relative errors:", {k: "%.2e" % v for k, v in errs.items()})


@pytest.mark.parametrize("fused", [False, True], ids=["tiles", "fused"])
def test_block_C5_full_batch_bf16(mods, fused, capsys):
    """The 50B-class block (N_e = 8192, head size 128, tile 1024) at its full batch of four, as the
    benchmark launches it (`bench.py --config 5`): `Out`, `dX`, all twelve parameter gradients (the
    weight-matrix gradients are the one place where batch members meet: sums over positions and batch),
    the Adam moments and the updated parameters, each compared in full with the fp64 oracle.  The oracle
    takes a few minutes on 20 TFLOP; it reports each layer it finishes, and one run serves both flows."""
    import time
    capi, tiled = mods
    t0 = time.time()

    def say(stage):
        with capsys.disabled():
            print("  [C5 oracle %4.0f s] %s" % (time.time() - t0, stage), flush=True)

    cfg, inp, ref = full_size_case(5, True, progress=say)
    assert cfg.N_b == 4
    errs = {}
    with tiled.Context(n_streams=4) as ctx:
        blk = tiled.Gpt2Block(ctx, cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, workload.base_tiles(cfg), dtype=cfg.dtype,
                              eps=cfg.eps, gelu=cfg.gelu, adam=True, fused_attention=fused)
        blk.set_params({k: inp[k] for k in workload.PARAM_NAMES})
        X, dOut = blk.activation(inp["X"]), blk.activation(inp["dOut"])
        Out, dX = blk.activation(), blk.activation()
        blk.forward(X, Out)
        blk.backward(dOut, dX)
        errs["Out"], errs["dX"] = relerr(Out.download(), ref["Out"]), relerr(dX.download(), ref["dX"])
        grads = {k: blk.grad(k).download() for k in workload.PARAM_NAMES}      # before the step: fp32, 3.2 GB
        blk.adam(1, **workload.ADAM)
        say("device forward, backward, Adam done (%s attention)" % ("fused" if fused else "tile"))
        for k in workload.PARAM_NAMES:                                          # one parameter at a time: W_1 alone is 268 M entries
            errs["d" + k] = relerr(grads[k], ref["grads"][k])
            errs["adam_m_" + k] = relerr(blk.moment(k, "m").download(), ref["adam"][k][1])
            errs["adam_v_" + k] = relerr(blk.moment(k, "v").download(), ref["adam"][k][2])
            errs["adam_p_" + k], safe = compare_adam_parameter(k, blk.param(k).download(), grads[k], ref, "bf16")
            if k == "b_qkv":
                assert not safe[cfg.N_e:2 * cfg.N_e].any()
            say("compared " + k)
        blk.close()
    with capsys.disabled():
        print("C5 (full batch%s) max-norm relative errors:" % (", fused attention" if fused else ""),
              {k: "%.2e" % v for k, v in errs.items()}, flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tolerance_of(k, "bf16")}
    assert not bad, bad
