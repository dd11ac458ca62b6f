"""ctypes binding of libnntile_mi.so: one Python function per C entry point, same
name, same argument order (include/nntile_mi.h).  Only argument marshalling
happens here; every status other than NNT_OK raises NntError.

The library must have been built (python -m paper_2504_13236_amd.build); there
is no fallback path: a missing library is an ImportError at load time.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libnntile_mi.so")

NNT_OK, NNT_EINVAL, NNT_EDTYPE, NNT_EHIP, NNT_ENOMEM, NNT_ESTATE = 0, -1, -2, -3, -4, -5
NNT_F32, NNT_BF16 = 0, 1
NNT_OP_N, NNT_OP_T = 0, 1
NNT_GELU_TANH, NNT_GELU_ERF = 0, 1
NNT_GRAN_OP, NNT_GRAN_TILE = 0, 1
NNT_MAX_DIM = 4

_ERR = {NNT_EINVAL: "NNT_EINVAL", NNT_EDTYPE: "NNT_EDTYPE", NNT_EHIP: "NNT_EHIP",
        NNT_ENOMEM: "NNT_ENOMEM", NNT_ESTATE: "NNT_ESTATE"}

# slots of a GPT-2 block (mirrors the enum in the header)
NNT_BLK_W_QKV, NNT_BLK_W_O, NNT_BLK_W_1, NNT_BLK_W_2 = 0, 1, 2, 3
NNT_BLK_B_QKV, NNT_BLK_B_O, NNT_BLK_B_1, NNT_BLK_B_2 = 4, 5, 6, 7
NNT_BLK_GAMMA1, NNT_BLK_BETA1, NNT_BLK_GAMMA2, NNT_BLK_BETA2 = 8, 9, 10, 11
NNT_BLK_GRAD, NNT_BLK_ADAM_M, NNT_BLK_ADAM_V, NNT_BLK_LOWP = 12, 24, 36, 48
(NNT_BLK_STATS1, NNT_BLK_X1, NNT_BLK_QKV, NNT_BLK_Q, NNT_BLK_K, NNT_BLK_V, NNT_BLK_P, NNT_BLK_SM_STATS,
 NNT_BLK_BH, NNT_BLK_BM, NNT_BLK_X2, NNT_BLK_STATS2, NNT_BLK_X3, NNT_BLK_H1, NNT_BLK_G,
 NNT_BLK_DG, NNT_BLK_DX3, NNT_BLK_DX2, NNT_BLK_DBM, NNT_BLK_DBH, NNT_BLK_DP,
 NNT_BLK_DQ, NNT_BLK_DK, NNT_BLK_DV, NNT_BLK_DQKV, NNT_BLK_DX1, NNT_BLK_NSLOTS) = range(52, 79)
# slots of a language model's own tensors
NNT_MDL_WTE, NNT_MDL_WPE, NNT_MDL_GAMMA_F, NNT_MDL_BETA_F = 0, 1, 2, 3
NNT_MDL_GRAD, NNT_MDL_ADAM_M, NNT_MDL_ADAM_V, NNT_MDL_LOWP = 4, 8, 12, 16
(NNT_MDL_XPOS, NNT_MDL_XF, NNT_MDL_DXF, NNT_MDL_STATS_F, NNT_MDL_LOGITS, NNT_MDL_LOSS_STATS, NNT_MDL_NSLOTS) = range(18, 25)


class NntError(RuntimeError):
    def __init__(self, code, where, detail=""):
        self.code = code
        super().__init__("%s returned %s%s" % (where, _ERR.get(code, code), (": " + detail) if detail else ""))


class nnt_exec_stats(C.Structure):
    _fields_ = [("tasks", C.c_int64), ("launches", C.c_int64), ("event_waits", C.c_int64), ("plans", C.c_int64),
                ("device_table_bytes", C.c_int64), ("device_workspace_bytes", C.c_int64)]


class nnt_profile_entry(C.Structure):
    _fields_ = [("label", C.c_char * 112), ("tasks", C.c_int64), ("launches", C.c_int64), ("ms", C.c_double),
                ("work", C.c_double), ("work_is_bytes", C.c_int32), ("reserved", C.c_int32)]


class nnt_adam_cfg(C.Structure):
    _fields_ = [("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("weight_decay", C.c_double)]


class nnt_gpt2_block_cfg(C.Structure):
    _fields_ = [("N_e", C.c_int64), ("N_h", C.c_int64), ("N_m", C.c_int64), ("N_s", C.c_int64), ("N_b", C.c_int64),
                ("tile_e", C.c_int64), ("tile_m", C.c_int64), ("tile_s", C.c_int64),
                ("tile_b", C.c_int64), ("tile_j", C.c_int64), ("tile_i", C.c_int64),
                ("dtype", C.c_int32), ("gelu_variant", C.c_int32), ("eps", C.c_float), ("causal", C.c_int32),
                ("fused_attention", C.c_int32)]


class nnt_sgd_cfg(C.Structure):
    _fields_ = [("lr", C.c_double), ("momentum", C.c_double), ("weight_decay", C.c_double), ("nesterov", C.c_int32)]


class nnt_slot_info(C.Structure):
    _fields_ = [("used", C.c_int32), ("dtype", C.c_int32), ("ndim", C.c_int32), ("causal_tiles", C.c_int32),
                ("shape", C.c_int64 * NNT_MAX_DIM), ("basetile", C.c_int64 * NNT_MAX_DIM)]


if not os.path.exists(LIB_PATH):
    raise ImportError("libnntile_mi.so is not built: run `python -m paper_2504_13236_amd.build` "
                      "(the HIP library is the only execution path; there is no fallback)")
lib = C.CDLL(LIB_PATH)

_p, _i32, _i64, _f, _pp = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.POINTER(C.c_void_p)
_pi64 = C.POINTER(C.c_int64)
_d = C.c_double

# name -> (restype, argtypes).  Order and types follow include/nntile_mi.h.
PROTOTYPES = {
    "nnt_ctx_create": (_i32, [_i32, _i32, _pp, _pp]),
    "nnt_ctx_destroy": (_i32, [_p]),
    "nnt_wait": (_i32, [_p]),
    "nnt_ctx_join": (_i32, [_p]),
    "nnt_ctx_stream": (_i32, [_p, _i32, _pp]),
    "nnt_last_error": (C.c_char_p, [_p]),
    "nnt_ctx_set_serial": (_i32, [_p, _i32]),
    "nnt_ctx_set_granularity": (_i32, [_p, _i32]),
    "nnt_ctx_stats": (_i32, [_p, C.POINTER(nnt_exec_stats)]),
    "nnt_profile_enable": (_i32, [_p, _i32]),
    "nnt_profile_read": (_i32, [_p, C.POINTER(nnt_profile_entry), _i32, C.POINTER(C.c_int32)]),
    "nnt_capture_begin": (_i32, [_p]),
    "nnt_capture_end": (_i32, [_p, _pp]),
    "nnt_graph_launch": (_i32, [_p]),
    "nnt_graph_destroy": (_i32, [_p]),
    "nnt_sched_simulate": (_i32, [_i32, _i32, _i32, _i32, _p, _p, _p, _p, _p, _p]),
    "nnt_tiling_ntiles": (_i32, [_i32, _pi64, _pi64, _pi64]),
    "nnt_tiling_tile_shape": (_i32, [_i32, _pi64, _pi64, _i64, _pi64]),
    "nnt_tensor_create": (_i32, [_p, _i32, _i32, _pi64, _pi64, _pp, _pp]),
    "nnt_tensor_destroy": (_i32, [_p]),
    "nnt_tensor_ntiles": (_i32, [_p, _pi64]),
    "nnt_tensor_tile_shape": (_i32, [_p, _i64, _pi64]),
    "nnt_tensor_tile_bytes": (_i32, [_p, _i64, _pi64]),
    "nnt_tile_gemm": (_i32, [_p, _i32, _i32, _i32, _i32, _i64, _i64, _i64, _i64, _f, _p, _i64, _i64, _p, _i64, _i64,
                             _f, _p, _i64, _i64]),
    "nnt_tile_fill": (_i32, [_p, _i32, _i64, _f, _p]),
    "nnt_tile_add": (_i32, [_p, _i32, _i64, _f, _p, _f, _p]),
    "nnt_tile_cast": (_i32, [_p, _i32, _i32, _i64, _p, _p]),
    "nnt_tile_copy_block": (_i32, [_p, _i32, _i32, _pi64, _p, _pi64, _p, _pi64]),
    "nnt_tile_bias_add": (_i32, [_p, _i32, _i64, _i64, _p, _p]),
    "nnt_tile_bias_grad_scratch": (_i64, [_i64, _i64]),
    "nnt_tile_bias_grad": (_i32, [_p, _i32, _i64, _i64, _p, _p, _i32, _p]),
    "nnt_gpt2_model_slot": (_i32, [C.POINTER(nnt_gpt2_block_cfg), _i64, _i64, _i32, C.POINTER(nnt_slot_info)]),
    "nnt_gpt2_model_create": (_i32, [_p, C.POINTER(nnt_gpt2_block_cfg), _i64, _i64, _p, _p, _pp]),
    "nnt_gpt2_model_destroy": (_i32, [_p]),
    "nnt_gpt2_model_sync_lowp": (_i32, [_p]),
    "nnt_gpt2_model_forward": (_i32, [_p, _p, _p, _p, _p, _p]),
    "nnt_gpt2_model_backward": (_i32, [_p]),
    "nnt_gpt2_model_adam": (_i32, [_p, _i32, C.POINTER(nnt_adam_cfg)]),
    "nnt_probe_mfma_rate": (_i32, [_p, _i32, _i32, _i32, _i32, _p, _p]),
    "nnt_tile_bias_grad_static_max": (_i64, []),
    "nnt_tile_bias_grad_static": (_i32, [_p, _i32, _i64, _i64, _p, _p, _i32]),
    "nnt_tile_gelu": (_i32, [_p, _i32, _i32, _i64, _p, _p]),
    "nnt_tile_gelu_bwd": (_i32, [_p, _i32, _i32, _i64, _p, _p, _p]),
    "nnt_tile_ln_stats": (_i32, [_p, _i32, _i64, _i64, _p, _p, _i64, _i64, _f]),
    "nnt_tile_ln_apply": (_i32, [_p, _i32, _i64, _i64, _p, _p, _p, _p, _p]),
    "nnt_tile_ln_bwd_sums": (_i32, [_p, _i32, _i64, _i64, _p, _p, _p, _p, _p, _i32]),
    "nnt_tile_ln_bwd_dx": (_i32, [_p, _i32, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _p]),
    "nnt_tile_ln_bwd_params_scratch": (_i64, [_i64, _i64]),
    "nnt_tile_ln_bwd_params": (_i32, [_p, _i32, _i64, _i64, _p, _p, _p, _p, _p, _i32, _p]),
    "nnt_tile_softmax_stats": (_i32, [_p, _i32, _i64, _i64, _i64, _i64, _i64, _i32, _f, _p, _p, _i32]),
    "nnt_tile_softmax_apply": (_i32, [_p, _i32, _i64, _i64, _i64, _i64, _i64, _i32, _f, _p, _p]),
    "nnt_tile_softmax_bwd_dot": (_i32, [_p, _i32, _i64, _i64, _i64, _p, _p, _p, _i32]),
    "nnt_tile_softmax_bwd_apply": (_i32, [_p, _i32, _i64, _i64, _i64, _p, _p, _p]),
    "nnt_tile_adam": (_i32, [_p, _i64, _i32, _d, _d, _d, _d, _d, _p, _p, _p, _p, _p]),
    "nnt_tile_sgd": (_i32, [_p, _i64, _d, _d, _d, _i32, _p, _p, _p, _p]),
    "nnt_gemm": (_i32, [_p, _f, _i32, _p, _i32, _p, _f, _p, _i32, _i32, _p]),
    "nnt_gemm_res": (_i32, [_p, _f, _i32, _p, _i32, _p, _f, _p, _i32, _i32, _p, _p]),
    "nnt_gemm_gelu": (_i32, [_p, _f, _i32, _p, _i32, _p, _p, _i32, _p, _i32, _p]),
    "nnt_gemm_gelu_bwd": (_i32, [_p, _f, _i32, _p, _i32, _p, _p, _i32, _i32, _p]),
    "nnt_gemm_heads": (_i32, [_p, _f, _i32, _p, _i32, _i32, _p, _i32, _p, _i32, _i32, _i32]),
    "nnt_fill": (_i32, [_p, _f, _p]),
    "nnt_add": (_i32, [_p, _f, _p, _f, _p]),
    "nnt_cast": (_i32, [_p, _p, _p]),
    "nnt_bias_add": (_i32, [_p, _p, _p]),
    "nnt_bias_grad": (_i32, [_p, _p, _p]),
    "nnt_gelu": (_i32, [_p, _i32, _p, _p]),
    "nnt_gelu_bwd": (_i32, [_p, _i32, _p, _p, _p]),
    "nnt_layernorm_fwd": (_i32, [_p, _p, _p, _p, _f, _p, _p]),
    "nnt_layernorm_bwd": (_i32, [_p, _p, _p, _p, _p, _p, _p, _p, _p]),
    "nnt_softmax_fwd": (_i32, [_p, _p, _p, _f, _i32]),
    "nnt_softmax_bwd": (_i32, [_p, _p, _p]),
    "nnt_head_split": (_i32, [_p, _p, _i32, _pp]),
    "nnt_head_merge": (_i32, [_p, _i32, _pp, _p]),
    "nnt_attention_fwd": (_i32, [_p, _p, _p, _p, _f, _i32, _p, _p]),
    "nnt_attention_bwd": (_i32, [_p, _p, _p, _p, _p, _p, _p, _f, _i32, _p, _p, _p]),
    "nnt_attention_fwd_heads": (_i32, [_p, _p, _f, _i32, _p, _p, _i32]),
    "nnt_attention_bwd_heads": (_i32, [_p, _p, _p, _p, _p, _f, _i32, _p, _i32]),
    "nnt_adam_step": (_i32, [_p, C.POINTER(nnt_adam_cfg), _i32, _p, _p, _p, _p, _p]),
    "nnt_embedding_fwd": (_i32, [_p, _p, _p, _p]),
    "nnt_embedding_bwd": (_i32, [_p, _p, _p, _p]),
    "nnt_cross_entropy": (_i32, [_p, _p, _p, _p, _p, _p]),
    "nnt_sgd_step": (_i32, [_p, C.POINTER(nnt_sgd_cfg), _p, _p, _p, _p]),
    "nnt_gpt2_block_slot": (_i32, [C.POINTER(nnt_gpt2_block_cfg), _i32, C.POINTER(nnt_slot_info)]),
    "nnt_gpt2_block_create": (_i32, [_p, C.POINTER(nnt_gpt2_block_cfg), _pp, _pp]),
    "nnt_gpt2_block_destroy": (_i32, [_p]),
    "nnt_gpt2_block_forward": (_i32, [_p, _p, _p]),
    "nnt_gpt2_block_backward": (_i32, [_p, _p, _p]),
    "nnt_gpt2_block_adam": (_i32, [_p, _i32, C.POINTER(nnt_adam_cfg)]),
    "nnt_gpt2_block_sgd": (_i32, [_p, C.POINTER(nnt_sgd_cfg)]),
    "nnt_gpt2_block_sync_lowp": (_i32, [_p]),
    "nnt_gpt2_block_grads_axpy": (_i32, [_p, _f, _pp]),
    "nnt_gpt2_stack_create": (_i32, [_p, _i32, _pp, _pp, _pp, _pp]),
    "nnt_gpt2_stack_destroy": (_i32, [_p]),
    "nnt_gpt2_stack_forward": (_i32, [_p]),
    "nnt_gpt2_stack_backward": (_i32, [_p]),
    "nnt_gpt2_stack_adam": (_i32, [_p, _i32, C.POINTER(nnt_adam_cfg)]),
    "nnt_version": (C.c_char_p, []),
}

# functions whose first argument is a context (their failures carry nnt_last_error text)
_CTX_FIRST = {n for n, (r, a) in PROTOTYPES.items()
              if n.startswith("nnt_") and not n.startswith("nnt_tile_") and not n.startswith("nnt_tiling_")
              and n not in ("nnt_ctx_create", "nnt_version", "nnt_gpt2_block_slot", "nnt_last_error", "nnt_sched_simulate")
              and not n.startswith("nnt_tensor_") and not n.startswith("nnt_graph_")
              and not n.startswith("nnt_gpt2_block_")
              and (not n.startswith("nnt_gpt2_stack_") or n == "nnt_gpt2_stack_create")
              and (not n.startswith("nnt_gpt2_model_") or n == "nnt_gpt2_model_create")
              and not n.startswith("nnt_probe_")}


def _wrap(name, restype, argtypes):
    fn = getattr(lib, name)
    fn.restype = restype
    fn.argtypes = argtypes
    if restype is not _i32:
        return fn

    def call(*args):
        rc = fn(*args)
        if rc != NNT_OK:
            detail = ""
            if name in _CTX_FIRST and args and args[0]:
                detail = (lib.nnt_last_error(args[0]) or b"").decode()
            raise NntError(rc, name, detail)
        return rc
    call.__name__ = name
    call.raw = fn        # unchecked form: returns the status
    return call


for _n, (_r, _a) in PROTOTYPES.items():
    globals()[_n] = _wrap(_n, _r, _a)


def i64_array(values):
    return (C.c_int64 * len(values))(*[int(v) for v in values])


def ptr_array(values):
    return (C.c_void_p * len(values))(*[C.c_void_p(v) if v else C.c_void_p(None) for v in values])
