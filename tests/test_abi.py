"""Host-only checks of the boundary: the library loads, exports every entry point
the header declares, the binding covers them all, and the host-side helpers
(tiling arithmetic, argument validation that needs no device) behave."""
import ctypes as C
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "nntile_mi.h")


def declared_symbols():
    text = open(HEADER).read()
    return sorted(set(re.findall(r"NNT_API\s+[\w\s\*]+?\b(nnt_\w+)\s*\(", text)))


@pytest.fixture(scope="module")
def capi():
    from paper_2504_13236_amd import capi as m
    return m


def test_header_declares_entry_points():
    syms = declared_symbols()
    assert len(syms) >= 60
    for must in ("nnt_tile_gemm", "nnt_gemm", "nnt_layernorm_fwd", "nnt_softmax_fwd", "nnt_adam_step",
                 "nnt_gpt2_block_forward", "nnt_gpt2_block_backward", "nnt_ctx_create", "nnt_tensor_create"):
        assert must in syms


def test_library_exports_every_declared_symbol(capi):
    out = subprocess.run(["nm", "-D", "--defined-only", capi.LIB_PATH], capture_output=True, text=True, check=True).stdout
    exported = set(re.findall(r" T (nnt_\w+)", out))
    missing = [s for s in declared_symbols() if s not in exported]
    assert not missing, missing
    # nothing but the C ABI is exported
    others = [l for l in out.splitlines() if " T " in l and " T nnt_" not in l and "_init" not in l and "_fini" not in l]
    assert not others, others[:5]


def test_binding_covers_every_declared_symbol(capi):
    syms = declared_symbols()
    assert sorted(capi.PROTOTYPES) == syms
    for s in syms:
        assert callable(getattr(capi, s))
    assert capi.nnt_version().startswith(b"nntile_mi")


def test_binding_argument_counts_match_header(capi):
    text = open(HEADER).read()
    for name, (_, argtypes) in capi.PROTOTYPES.items():
        m = re.search(r"NNT_API\s+[\w\s\*]+?\b%s\s*\(([^;]*?)\)\s*;" % name, text, re.S)
        assert m, name
        args = m.group(1).strip()
        n = 0 if args in ("", "void") else len([a for a in args.split(",") if a.strip()])
        assert n == len(argtypes), (name, n, len(argtypes))


def test_tiling_helpers_host_only(capi):
    n = C.c_int64()
    capi.nnt_tiling_ntiles(3, capi.i64_array([1600, 1024, 8]), capi.i64_array([400, 400, 8]), C.byref(n))
    assert n.value == 4 * 3 * 1
    shp = (C.c_int64 * 3)()
    # tile 11 = (3, 2, 0): ragged sequence tile 224
    capi.nnt_tiling_tile_shape(3, capi.i64_array([1600, 1024, 8]), capi.i64_array([400, 400, 8]), 11, shp)
    assert list(shp) == [400, 224, 8]
    capi.nnt_tiling_tile_shape(2, capi.i64_array([10, 7]), capi.i64_array([4, 3]), 8, shp)
    assert list(shp)[:2] == [2, 1]
    assert capi.nnt_tiling_ntiles.raw(0, capi.i64_array([1]), capi.i64_array([1]), C.byref(n)) == capi.NNT_EINVAL
    assert capi.nnt_tiling_ntiles.raw(2, capi.i64_array([4, 0]), capi.i64_array([1, 1]), C.byref(n)) == capi.NNT_EINVAL
    assert capi.nnt_tiling_tile_shape.raw(1, capi.i64_array([4]), capi.i64_array([2]), 2, shp) == capi.NNT_EINVAL


def test_argument_validation_without_device(capi):
    # these return before touching the GPU
    assert capi.nnt_tile_gemm.raw(None, 7, 0, 0, 0, 4, 4, 4, 1, 1.0, None, 4, 16, None, 4, 16, 0.0, None, 4, 16) == capi.NNT_EDTYPE
    assert capi.nnt_tile_gemm.raw(None, 0, 1, 0, 0, 4, 4, 4, 1, 1.0, None, 4, 16, None, 4, 16, 0.0, None, 4, 16) == capi.NNT_EDTYPE
    assert capi.nnt_tile_gemm.raw(None, 0, 0, 0, 0, 4, 4, 4, 1, 1.0, None, 4, 16, None, 4, 16, 0.0, None, 4, 16) == capi.NNT_EINVAL
    assert capi.nnt_tile_gemm.raw(None, 0, 0, 0, 0, 0, 4, 4, 1, 1.0, None, 4, 16, None, 4, 16, 0.0, None, 4, 16) == capi.NNT_OK
    assert capi.nnt_tile_gelu.raw(None, 0, 5, 8, None, None) == capi.NNT_EINVAL
    assert capi.nnt_tile_adam.raw(None, 8, 0, 1e-3, 0.9, 0.999, 1e-8, 0.0, None, None, None, None, None) == capi.NNT_EINVAL
    assert capi.nnt_tile_bias_grad_scratch(768, 2048) >= 768
    assert capi.nnt_tile_ln_bwd_params_scratch(768, 2048) == 2 * capi.nnt_tile_bias_grad_scratch(768, 2048)
    assert capi.nnt_wait.raw(None) == capi.NNT_EINVAL
    cfg = capi.nnt_gpt2_block_cfg()
    info = capi.nnt_slot_info()
    assert capi.nnt_gpt2_block_slot.raw(C.byref(cfg), 0, C.byref(info)) == capi.NNT_EINVAL      # all-zero config


def test_block_slot_table_host_only(capi):
    import workload
    cfg = workload.CONFIGS[4]
    bt = workload.base_tiles(cfg)
    c = capi.nnt_gpt2_block_cfg(cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, bt["e"], bt["m"], bt["s"], bt["b"], bt["j"], bt["i"],
                                capi.NNT_BF16, capi.NNT_GELU_TANH, 1e-5, 1)
    info = capi.nnt_slot_info()
    capi.nnt_gpt2_block_slot(C.byref(c), capi.NNT_BLK_P, C.byref(info))
    assert info.used and info.dtype == capi.NNT_BF16 and info.causal_tiles == 1
    assert list(info.shape) == [1024, 1024, 8, 25] and list(info.basetile) == [400, 400, 8, 25]
    capi.nnt_gpt2_block_slot(C.byref(c), capi.NNT_BLK_W_1, C.byref(info))
    assert info.dtype == capi.NNT_F32 and list(info.shape)[:2] == [6400, 1600] and list(info.basetile)[:2] == [400, 400]
    capi.nnt_gpt2_block_slot(C.byref(c), capi.NNT_BLK_LOWP + 2, C.byref(info))
    assert info.used and info.dtype == capi.NNT_BF16
    capi.nnt_gpt2_block_slot(C.byref(c), capi.NNT_BLK_Q, C.byref(info))
    assert list(info.shape) == [64, 1024, 8, 25] and list(info.basetile) == [64, 400, 8, 25]
    c.dtype = capi.NNT_F32
    capi.nnt_gpt2_block_slot(C.byref(c), capi.NNT_BLK_LOWP, C.byref(info))
    assert not info.used
    used = 0
    for s in range(capi.NNT_BLK_NSLOTS):
        capi.nnt_gpt2_block_slot(C.byref(c), s, C.byref(info))
        used += info.used
    assert used == capi.NNT_BLK_NSLOTS - 4


def test_model_slot_table_host_only(capi):
    """Type, shape and tiling of a language model's own tensors, as the library describes them."""
    import workload
    cfg = workload.CONFIGS[3]
    bt = workload.base_tiles(cfg)
    c = capi.nnt_gpt2_block_cfg(cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b, bt["e"], bt["m"], bt["s"], bt["b"], bt["j"], bt["i"],
                                capi.NNT_BF16, capi.NNT_GELU_TANH, 1e-5, 1)
    info = capi.nnt_slot_info()
    N_v, tv = 50304, 8192
    capi.nnt_gpt2_model_slot(C.byref(c), N_v, tv, capi.NNT_MDL_WTE, C.byref(info))
    assert info.used and info.dtype == capi.NNT_F32 and list(info.shape)[:2] == [1024, N_v] and list(info.basetile)[:2] == [512, tv]
    capi.nnt_gpt2_model_slot(C.byref(c), N_v, tv, capi.NNT_MDL_LOWP + capi.NNT_MDL_WPE, C.byref(info))
    assert info.used and info.dtype == capi.NNT_BF16 and list(info.shape)[:2] == [1024, 1024] and list(info.basetile)[:2] == [512, 512]
    capi.nnt_gpt2_model_slot(C.byref(c), N_v, tv, capi.NNT_MDL_GRAD + capi.NNT_MDL_GAMMA_F, C.byref(info))
    assert info.dtype == capi.NNT_F32 and info.ndim == 1 and info.shape[0] == 1024
    capi.nnt_gpt2_model_slot(C.byref(c), N_v, tv, capi.NNT_MDL_LOGITS, C.byref(info))
    assert info.dtype == capi.NNT_BF16 and list(info.shape)[:3] == [N_v, 1024, 16] and list(info.basetile)[:3] == [tv, 512, 16]
    capi.nnt_gpt2_model_slot(C.byref(c), N_v, tv, capi.NNT_MDL_LOSS_STATS, C.byref(info))
    assert info.dtype == capi.NNT_F32 and list(info.shape)[:3] == [2, 1024, 16]
    c.dtype = capi.NNT_F32
    capi.nnt_gpt2_model_slot(C.byref(c), N_v, tv, capi.NNT_MDL_LOWP, C.byref(info))
    assert not info.used                                                  # fp32 models keep no bf16 copies
    assert capi.nnt_gpt2_model_slot.raw(C.byref(c), 0, tv, 0, C.byref(info)) == capi.NNT_EINVAL
    assert capi.nnt_gpt2_model_slot.raw(C.byref(c), N_v, tv, capi.NNT_MDL_NSLOTS, C.byref(info)) == capi.NNT_EINVAL
    assert capi.nnt_gpt2_model_forward.raw(None, None, None, None, None, None) == capi.NNT_EINVAL
    assert capi.nnt_probe_mfma_rate.raw(None, 5, 0, 1, 1, None, None) == capi.NNT_EDTYPE
    assert capi.nnt_probe_mfma_rate.raw(None, 0, 0, 0, 1, None, None) == capi.NNT_EINVAL
    assert capi.nnt_tile_bias_grad_static.raw(None, 0, 1 << 20, 1 << 20, None, None, 0) == capi.NNT_EINVAL


def test_build_guard_finds_scratch_only_inside_loops():
    """The build refuses direct-load kernels that touch scratch memory inside a loop: their
    fragment registers are filled by LDS reads that are waited for later by hand."""
    from paper_2504_13236_amd.build import resource_usage, scratch_in_loops
    listing = "\n".join([
        "_Z6kernelv:                             ; @_Z6kernelv",
        "; %bb.0:",
        "\tscratch_store_dword off, v1, off",                       # prologue: allowed
        ".LBB0_1:                                ; =>This Inner Loop Header: Depth=1",
        "\tv_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], v[20:23], v[0:15]",
        "\tscratch_store_dwordx4 off, v[4:7], off offset:16 ; 16-byte Folded Spill",
        "; %bb.2:                                ;   in Loop: Header=BB0_1 Depth=1",
        "\tscratch_load_dwordx4 v[4:7], off, off offset:16 ; 16-byte Folded Reload",
        "\ts_cbranch_scc0 .LBB0_1",
        ".LBB0_3:",
        "\tscratch_store_dword off, v3, off offset:64 ; 4-byte Folded Spill",   # epilogue: allowed
        "_Z5otherv:",
        "\tscratch_store_dword off, v1, off",
    ])
    assert scratch_in_loops(listing) == [("_Z6kernelv", 6), ("_Z6kernelv", 8)]
    remarks = "\n".join([
        "a.hip:1:1: remark: Function Name: _Z6kernelv [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark:     VGPRs: 72 [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 8 [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark:     LDS Size [bytes/block]: 61440 [-Rpass-analysis=kernel-resource-usage]",
    ])
    assert resource_usage(remarks) == {"_Z6kernelv": {"VGPRs": 72, "ScratchSize": 8, "LDS Size": 61440}}


def test_build_guard_finds_registers_used_while_their_lds_read_is_in_flight():
    """The build also refuses direct-load kernels in whose assembly any instruction names a register
    between the LDS read that targets it and the next full wait (a copy the compiler schedules there
    would read stale data)."""
    from paper_2504_13236_amd.build import registers_touched_in_flight
    listing = "\n".join([
        "_Z6kernelv:                             ; @_Z6kernelv",
        "\tds_read_b128 v[4:7], v1 offset:16",
        "\tv_mfma_f32_32x32x2_f32 v[16:31], v2, v3, v[16:31]",       # other registers: fine
        "\tv_mov_b32_e32 v9, v5",                                     # copies a register of the read in flight
        "\ts_waitcnt vmcnt(0)",                                       # not a wait for LDS
        "\tds_read_b32 v10, v6",                                      # address taken from a register in flight
        "\ts_waitcnt lgkmcnt(0)",
        "\tv_mfma_f32_32x32x2_f32 v[16:31], v4, v10, v[16:31]",      # after the wait: fine
        ".LBB0_1:                                ; =>This Inner Loop Header: Depth=1",
        "\tds_read_b64_tr_b16 v[12:13], v1 offset:64",
        "\ts_waitcnt lgkmcnt(1)",                                     # a partial wait clears nothing
        "\tv_accvgpr_write_b32 a0, v13",
        "\ts_waitcnt vmcnt(0) lgkmcnt(0)",
        "\tv_accvgpr_write_b32 a0, v13",
        "\ts_endpgm",
        "_Z5otherv:",
        "\tv_mov_b32_e32 v9, v12",                                    # another kernel starts clean
    ])
    assert registers_touched_in_flight(listing) == [("_Z6kernelv", 4, "v5", 2), ("_Z6kernelv", 6, "v6", 2),
                                                    ("_Z6kernelv", 12, "v13", 10)]


def _simulate(capi, n_streams, serial, n_tiles, tasks):
    import numpy as np
    first = np.zeros(len(tasks) + 1, np.int32)
    tiles, modes = [], []
    for t, acc in enumerate(tasks):
        for tile, mode in acc:
            tiles.append(tile)
            modes.append(mode)
        first[t + 1] = len(tiles)
    tiles, modes = np.asarray(tiles, np.int32), np.asarray(modes, np.int32)
    stream = np.zeros(len(tasks), np.int32)
    seq = np.zeros(len(tasks), np.int64)
    waits = np.zeros((len(tasks), 8), np.int64)
    capi.nnt_sched_simulate(n_streams, serial, n_tiles, len(tasks), first.ctypes.data, tiles.ctypes.data, modes.ctypes.data,
                            stream.ctypes.data, seq.ctypes.data, waits.ctypes.data)
    return stream, seq, waits


@pytest.mark.parametrize("n_streams", [1, 2, 4, 8])
def test_executor_orders_every_conflicting_pair(capi, n_streams):
    """Host-side race check of the task executor's decisions: for random task sequences, every pair of
    tasks that touch a common tile, at least one of them writing, must be ordered by the happens-before
    relation that stream order and the event waits generate (read-after-write, write-after-read,
    write-after-write); tasks that only share read tiles need not be."""
    import numpy as np
    r = np.random.default_rng(100 + n_streams)
    for trial in range(20):
        n_tiles = int(r.integers(1, 9))
        n_tasks = int(r.integers(5, 120))
        tasks = []
        for _ in range(n_tasks):
            k = int(r.integers(1, min(4, n_tiles) + 1))
            chosen = r.choice(n_tiles, size=k, replace=False)
            # modes: read, write, read-write, and writes of part 0, 1 or 2 of the tile (6 + 256 * part)
            tasks.append([(int(t), int(r.choice([1, 1, 2, 3, 6, 6 + 256, 6 + 512]))) for t in chosen])
        stream, seq, waits = _simulate(capi, n_streams, 0, n_tiles, tasks)
        assert stream.min() >= 0 and stream.max() < n_streams
        at = {(int(stream[t]), int(seq[t])): t for t in range(n_tasks)}
        assert len(at) == n_tasks                                  # sequence numbers are unique per stream
        before = []                                                # before[t]: the tasks known to finish before t starts
        last_on = {}
        for t in range(n_tasks):
            s = int(stream[t])
            assert int(seq[t]) == sum(1 for u in range(t + 1) if stream[u] == s)     # streams number their tasks 1, 2, ...
            anc = set()
            preds = []
            if s in last_on:
                preds.append(last_on[s])
            for o in range(8):
                if waits[t, o]:
                    assert o != s and o < n_streams
                    preds.append(at[(o, int(waits[t, o]))])
            for p in preds:
                assert p < t
                anc.add(p)
                anc |= before[p]
            before.append(anc)
            last_on[s] = t
        for j in range(n_tasks):
            for i in range(j):
                for ti, mi in tasks[i]:
                    for tj, mj in tasks[j]:
                        # writers of different parts of a tile do not conflict; everything else with a writer does
                        parts_apart = (mi & 0xff) == 6 and (mj & 0xff) == 6 and mi != mj
                        if ti == tj and ((mi | mj) & 2) and not parts_apart:
                            assert i in before[j], (trial, i, j, tasks[i], tasks[j])
    # serial mode keeps everything on one stream
    stream, seq, waits = _simulate(capi, n_streams, 1, 3, [[(0, 2)], [(1, 2)], [(0, 1), (1, 1)], [(2, 3)]])
    assert not stream.any() and not waits.any()


def test_executor_lets_writers_of_different_parts_overlap(capi):
    """Three tasks write parts 0, 1, 2 of the same tiles (the attention products that fill the rows of Q, K and V of
    one tensor): they land on different streams and wait for nothing but the tensor's previous writer; a reader
    after them waits for all three; a second writer of part 1 waits for that reader, not for the other parts."""
    W, P0, P1, P2, R = 2, 6, 6 + 256, 6 + 512, 1
    tasks = [[(0, W), (1, W)], [(0, P0), (1, P0)], [(0, P1), (1, P1)], [(0, P2), (1, P2)], [(0, R), (1, R)], [(0, P1), (1, P1)]]
    stream, seq, waits = _simulate(capi, 4, 0, 2, tasks)
    assert len({int(stream[t]) for t in (1, 2, 3)}) == 3                       # the three part writers run side by side
    for t in (1, 2, 3):
        # (a wait names the first recorded event that covers the task asked for, so only its stream is checked)
        others = [o for o in range(8) if waits[t, o]]
        assert all(o == stream[0] for o in others) and (others or stream[t] == stream[0])
    covered = {int(stream[4])} | {o for o in range(8) if waits[4, o]}
    assert {int(stream[t]) for t in (1, 2, 3)} <= covered                      # the reader comes after every part writer
    assert stream[5] == stream[4] or waits[5, int(stream[4])] >= seq[4]         # the next writer of part 1 comes after the reader
    # a part number on a mode other than 6 is refused
    import numpy as np
    import ctypes as C
    bad = np.array([1 + 256], np.int32)
    tf, at = np.array([0, 1], np.int32), np.array([0], np.int32)
    so, sq, wo = np.zeros(1, np.int32), np.zeros(1, np.int64), np.zeros(8, np.int64)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    assert capi.nnt_sched_simulate.raw(2, 0, 1, 1, p(tf), p(at), p(bad), p(so), p(sq), p(wo)) == capi.NNT_EINVAL


def test_executor_spreads_independent_tasks_and_chains_dependent_ones(capi):
    # four independent writers land on four streams; a reader of all of them waits for the other three
    tasks = [[(t, 2)] for t in range(4)] + [[(0, 1), (1, 1), (2, 1), (3, 1)]]
    stream, seq, waits = _simulate(capi, 4, 0, 4, tasks)
    assert sorted(stream[:4].tolist()) == [0, 1, 2, 3]
    assert (waits[4] > 0).sum() == 3
    # a chain on one tile stays on the producer's stream and needs no event at all
    stream, seq, waits = _simulate(capi, 4, 0, 1, [[(0, 3)] for _ in range(6)])
    assert len(set(stream.tolist())) == 1 and not waits.any()
    # bad arguments
    import numpy as np
    z = np.zeros(8, np.int64)
    assert capi.nnt_sched_simulate.raw(0, 0, 1, 0, None, None, None, None, None, None) == capi.NNT_EINVAL
    first = np.asarray([0, 1], np.int32)
    bad_tile = np.asarray([5], np.int32)
    mode = np.asarray([1], np.int32)
    out_s = np.zeros(1, np.int32)
    assert capi.nnt_sched_simulate.raw(2, 0, 1, 1, first.ctypes.data, bad_tile.ctypes.data, mode.ctypes.data,
                                       out_s.ctypes.data, z.ctypes.data, z.ctypes.data) == capi.NNT_EINVAL


def test_executor_learns_which_tasks_need_an_event_of_their_own(capi):
    """Events are recorded on demand; a task that another stream had to wait for is remembered (by the first
    tile it writes), and its next occurrence gets an event of its own, so that the wait is exact again.
    Period: a writes t0; b writes t1; c reads t1 and writes t2 (stays behind b, so b is no longer the tail of
    its stream); d reads t0 and t1 and writes t3 (runs behind a, must wait for b on the other stream)."""
    period = [[(0, 2)], [(1, 2)], [(1, 1), (2, 2)], [(0, 1), (1, 1), (3, 2)]]
    reps = 4
    stream, seq, waits = _simulate(capi, 2, 0, 4, period * reps)
    for rep in range(reps):
        a, b, c, d = (4 * rep + i for i in range(4))
        assert stream[c] == stream[b] and seq[c] == seq[b] + 1
        sb = int(stream[b])
        assert stream[d] != sb
        w = int(waits[d, sb])
        if rep == 0:
            assert w == seq[c]          # no event of b's own yet: the wait covers the tail of that stream
        else:
            assert w == seq[b]          # b's like is known to be consumed across streams: exact wait
    # one stream, or serial mode: no waits at all
    stream, seq, waits = _simulate(capi, 1, 0, 4, period * 2)
    assert not stream.any() and not waits.any()
