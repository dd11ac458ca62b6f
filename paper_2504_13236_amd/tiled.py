"""Host-side helpers around the C ABI: device memory for tiles (through PyTorch),
conversion between logical numpy arrays and per-tile buffers, and the tensor set
of a GPT-2 block.  No arithmetic of the method happens here; every operation runs
in the HIP library.
"""
from __future__ import annotations

import ctypes as C
import itertools

import numpy as np
import torch

from . import capi

_ALIGN = 256


def _np_dtype_code(dtype):
    if dtype in (capi.NNT_F32, "f32"):
        return capi.NNT_F32
    if dtype in (capi.NNT_BF16, "bf16"):
        return capi.NNT_BF16
    raise ValueError(dtype)


class Context:
    """Owns an nnt_ctx.  Streams are torch streams so that torch events can time them."""

    def __init__(self, n_streams=4, device=0, serial=False, granularity=capi.NNT_GRAN_OP):
        self.device = device
        torch.cuda.set_device(device)
        self.streams = [torch.cuda.Stream(device=device) for _ in range(n_streams)]
        arr = capi.ptr_array([s.cuda_stream for s in self.streams])
        h = C.c_void_p()
        capi.nnt_ctx_create(device, n_streams, arr, C.byref(h))
        self.h = h
        if serial:
            capi.nnt_ctx_set_serial(self.h, 1)
        if granularity != capi.NNT_GRAN_OP:
            capi.nnt_ctx_set_granularity(self.h, granularity)
        self._tensors = []

    def wait(self):
        capi.nnt_wait(self.h)

    def join(self):
        capi.nnt_ctx_join(self.h)

    def stats(self):
        s = capi.nnt_exec_stats()
        capi.nnt_ctx_stats(self.h, C.byref(s))
        return dict(tasks=s.tasks, launches=s.launches, event_waits=s.event_waits, plans=s.plans,
                    device_table_bytes=s.device_table_bytes, device_workspace_bytes=s.device_workspace_bytes)

    def profile(self, on=True):
        capi.nnt_profile_enable(self.h, 1 if on else 0)

    def profile_read(self):
        """{label: dict(tasks, launches, ms, work, unit)} for the tasks run since profile(True)."""
        cap = 256
        arr = (capi.nnt_profile_entry * cap)()
        n = C.c_int32()
        capi.nnt_profile_read(self.h, arr, cap, C.byref(n))
        out = {}
        for e in arr[:min(n.value, cap)]:
            out[e.label.decode()] = dict(tasks=e.tasks, launches=e.launches, ms=e.ms, work=e.work,
                                         unit="bytes" if e.work_is_bytes else "flops")
        return out

    def set_granularity(self, g):
        capi.nnt_ctx_set_granularity(self.h, g)

    def set_serial(self, on):
        capi.nnt_ctx_set_serial(self.h, 1 if on else 0)

    def close(self):
        if self.h:
            for t in list(self._tensors):
                t.close()
            capi.nnt_ctx_destroy(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()


class TiledTensor:
    """A tiled tensor whose tiles live in one torch buffer (each tile 256-byte aligned)."""

    def __init__(self, ctx: Context, dtype, shape, base, absent=None, fill=None):
        self.ctx = ctx
        self.dtype = _np_dtype_code(dtype)
        self.shape = tuple(int(v) for v in shape)
        self.base = tuple(int(min(b, n)) for b, n in zip(base, self.shape))
        self.grid = tuple(-(-n // b) for n, b in zip(self.shape, self.base))
        self.esize = 4 if self.dtype == capi.NNT_F32 else 2
        self.tile_index = list(itertools.product(*[range(g) for g in reversed(self.grid)]))
        self.tile_index = [tuple(reversed(t)) for t in self.tile_index]      # first axis fastest
        self.offsets, self.absent = [], []
        off = 0
        for idx in self.tile_index:
            gone = bool(absent and absent(idx))
            self.absent.append(gone)
            self.offsets.append(off)
            if not gone:
                nbytes = int(np.prod(self.tile_shape(idx))) * self.esize
                off += -(-nbytes // _ALIGN) * _ALIGN
        self.nbytes = max(off, _ALIGN)
        self.buf = torch.empty(self.nbytes, dtype=torch.uint8, device="cuda:%d" % ctx.device)
        if fill is not None:
            self.buf.zero_()
            torch.cuda.synchronize()
        base_ptr = self.buf.data_ptr()
        self.ptrs = [0 if g else base_ptr + o for o, g in zip(self.offsets, self.absent)]
        h = C.c_void_p()
        capi.nnt_tensor_create(ctx.h, self.dtype, len(self.shape), capi.i64_array(self.shape), capi.i64_array(self.base),
                               capi.ptr_array(self.ptrs), C.byref(h))
        self.h = h
        ctx._tensors.append(self)

    # ---- geometry
    def slices(self, idx):
        return tuple(slice(i * b, min(n, (i + 1) * b)) for i, b, n in zip(idx, self.base, self.shape))

    def tile_shape(self, idx):
        return tuple(s.stop - s.start for s in self.slices(idx))

    def _torch_dtype(self):
        return torch.float32 if self.dtype == capi.NNT_F32 else torch.bfloat16

    def tile_view(self, k):
        """1-D torch view of tile number k in its storage type."""
        n = int(np.prod(self.tile_shape(self.tile_index[k])))
        o = self.offsets[k]
        return self.buf[o:o + n * self.esize].view(self._torch_dtype())

    # ---- host <-> device
    def upload(self, a):
        a = np.asarray(a, dtype=np.float32)
        assert a.shape == self.shape, (a.shape, self.shape)
        for k, idx in enumerate(self.tile_index):
            if self.absent[k]:
                continue
            t = np.ascontiguousarray(a[self.slices(idx)].T).reshape(-1)     # first axis fastest
            ht = torch.from_numpy(t)
            if self.dtype == capi.NNT_BF16:
                ht = ht.to(torch.bfloat16)
            self.tile_view(k).copy_(ht)
        torch.cuda.synchronize()      # the context's streams do not order after torch's current stream
        return self

    def download(self):
        """Logical fp32 array; absent tiles read as zeros.  Waits for the context first."""
        self.ctx.wait()
        torch.cuda.synchronize()
        out = np.zeros(self.shape, np.float32)
        for k, idx in enumerate(self.tile_index):
            if self.absent[k]:
                continue
            ts = self.tile_shape(idx)
            t = self.tile_view(k).to(torch.float32).cpu().numpy()
            out[self.slices(idx)] = t.reshape(tuple(reversed(ts))).T
        return out

    @classmethod
    def from_numpy(cls, ctx, a, base, dtype="f32", absent=None):
        return cls(ctx, dtype, a.shape, base, absent).upload(a)

    @classmethod
    def zeros(cls, ctx, shape, base, dtype="f32", absent=None):
        return cls(ctx, dtype, shape, base, absent, fill=0)

    def close(self):
        if self.h:
            capi.nnt_tensor_destroy(self.h)
            self.h = None
            if self in self.ctx._tensors:
                self.ctx._tensors.remove(self)
            self.buf = None


def causal_absent(base_k, base_q, n_q):
    """Predicate for score tensors [k, q, ...]: tile (kt, qt, ...) holds no visible
    score when its first key index exceeds its last query index."""
    def absent(idx):
        return idx[0] * base_k > min(n_q, (idx[1] + 1) * base_q) - 1
    return absent


PARAM_SLOTS = {"W_qkv": capi.NNT_BLK_W_QKV, "W_o": capi.NNT_BLK_W_O, "W_1": capi.NNT_BLK_W_1, "W_2": capi.NNT_BLK_W_2,
               "b_qkv": capi.NNT_BLK_B_QKV, "b_o": capi.NNT_BLK_B_O, "b_1": capi.NNT_BLK_B_1, "b_2": capi.NNT_BLK_B_2,
               "gamma1": capi.NNT_BLK_GAMMA1, "beta1": capi.NNT_BLK_BETA1,
               "gamma2": capi.NNT_BLK_GAMMA2, "beta2": capi.NNT_BLK_BETA2}


class Gpt2Block:
    """Allocates every tensor a block needs (as the library describes them slot by
    slot) and exposes forward / backward / adam."""

    def __init__(self, ctx: Context, N_e, N_h, N_m, N_s, N_b, tiles, dtype="f32", eps=1e-5, gelu="tanh",
                 causal=True, adam=True, fused_attention=False):
        self.ctx = ctx
        cfg = capi.nnt_gpt2_block_cfg()
        cfg.N_e, cfg.N_h, cfg.N_m, cfg.N_s, cfg.N_b = N_e, N_h, N_m, N_s, N_b
        cfg.tile_e, cfg.tile_m, cfg.tile_s = tiles["e"], tiles["m"], tiles["s"]
        cfg.tile_b, cfg.tile_j, cfg.tile_i = tiles["b"], tiles["j"], tiles["i"]
        cfg.dtype = _np_dtype_code(dtype)
        cfg.gelu_variant = capi.NNT_GELU_TANH if gelu == "tanh" else capi.NNT_GELU_ERF
        cfg.eps = eps
        cfg.causal = 1 if causal else 0
        cfg.fused_attention = 1 if fused_attention else 0
        self.cfg = cfg
        self.dtype = cfg.dtype
        self.slots = [None] * capi.NNT_BLK_NSLOTS
        for s in range(capi.NNT_BLK_NSLOTS):
            info = capi.nnt_slot_info()
            capi.nnt_gpt2_block_slot(C.byref(cfg), s, C.byref(info))
            if not info.used:
                continue
            if capi.NNT_BLK_ADAM_M <= s < capi.NNT_BLK_LOWP and not adam:
                continue
            shape = tuple(info.shape[:info.ndim])
            base = tuple(info.basetile[:info.ndim])
            absent = causal_absent(base[0], base[1], shape[1]) if info.causal_tiles else None
            zero = capi.NNT_BLK_GRAD <= s < capi.NNT_BLK_LOWP
            self.slots[s] = TiledTensor(ctx, info.dtype, shape, base, absent, fill=0 if zero else None)
        arr = capi.ptr_array([t.h.value if t is not None else None for t in self.slots])
        h = C.c_void_p()
        capi.nnt_gpt2_block_create(ctx.h, C.byref(cfg), arr, C.byref(h))
        self.h = h
        self.act_base = (min(tiles["e"], N_e), min(tiles["s"], N_s), min(tiles["b"], N_b))
        self.act_shape = (N_e, N_s, N_b)

    def set_params(self, params: dict):
        for name, slot in PARAM_SLOTS.items():
            self.slots[slot].upload(params[name])
        capi.nnt_gpt2_block_sync_lowp(self.h)

    def activation(self, a=None):
        t = TiledTensor(self.ctx, self.dtype, self.act_shape, self.act_base)
        if a is not None:
            t.upload(a)
        return t

    def forward(self, X, Out):
        capi.nnt_gpt2_block_forward(self.h, X.h, Out.h)

    def backward(self, dOut, dX):
        capi.nnt_gpt2_block_backward(self.h, dOut.h, dX.h)

    def adam(self, step, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
        cfg = capi.nnt_adam_cfg(lr, beta1, beta2, eps, weight_decay)
        capi.nnt_gpt2_block_adam(self.h, step, C.byref(cfg))

    def sgd(self, lr=1e-2, momentum=0.9, weight_decay=0.0, nesterov=False):
        cfg = capi.nnt_sgd_cfg(lr, momentum, weight_decay, 1 if nesterov else 0)
        capi.nnt_gpt2_block_sgd(self.h, C.byref(cfg))

    def param(self, name):
        return self.slots[PARAM_SLOTS[name]]

    def grad(self, name):
        return self.slots[capi.NNT_BLK_GRAD + PARAM_SLOTS[name]]

    def moment(self, name, which):
        return self.slots[(capi.NNT_BLK_ADAM_M if which == "m" else capi.NNT_BLK_ADAM_V) + PARAM_SLOTS[name]]

    def close(self):
        if self.h:
            self.ctx.wait()
            capi.nnt_gpt2_block_destroy(self.h)
            self.h = None


class Gpt2Stack:
    """A chain of blocks with the activations between them (allocated here) as one flow of tasks."""

    def __init__(self, ctx: Context, blocks):
        self.ctx, self.blocks = ctx, list(blocks)
        n = len(self.blocks)
        self.acts = [self.blocks[0].activation() for _ in range(n + 1)]
        self.dacts = [self.blocks[0].activation() for _ in range(n + 1)]
        h = C.c_void_p()
        capi.nnt_gpt2_stack_create(ctx.h, n, capi.ptr_array([b.h.value for b in self.blocks]),
                                   capi.ptr_array([t.h.value for t in self.acts]),
                                   capi.ptr_array([t.h.value for t in self.dacts]), C.byref(h))
        self.h = h

    def forward(self):
        capi.nnt_gpt2_stack_forward(self.h)

    def backward(self):
        capi.nnt_gpt2_stack_backward(self.h)

    def adam(self, step, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
        cfg = capi.nnt_adam_cfg(lr, beta1, beta2, eps, weight_decay)
        capi.nnt_gpt2_stack_adam(self.h, step, C.byref(cfg))

    def close(self):
        if self.h:
            self.ctx.wait()
            capi.nnt_gpt2_stack_destroy(self.h)
            self.h = None


class Gpt2Model:
    """A GPT-2-shaped language model (token + position embedding lookup, a chain of blocks, the final
    layer norm, the head tied to the token embedding, the cross-entropy loss, the whole backward pass and
    one Adam step) through the library's nnt_gpt2_model_* entry points.  This class only allocates the
    tensors the library describes slot by slot and marshals the calls.

    Tensors (paper's axis order): `wte` [N_e, N_v] and `wpe` [N_e, N_s] fp32 masters (one column per
    vocabulary item / position), their gradients and Adam moments, bf16 copies for bf16 models."""

    def __init__(self, ctx: Context, blocks, N_v, tile_v):
        self.ctx, self.blocks = ctx, list(blocks)
        b0 = self.blocks[0]
        self.N_e, self.N_s, self.N_b = b0.act_shape
        self.N_v = int(N_v)
        self.dtype = b0.dtype
        self.stack = Gpt2Stack(ctx, self.blocks)
        self.slots = [None] * capi.NNT_MDL_NSLOTS
        for s in range(capi.NNT_MDL_NSLOTS):
            info = capi.nnt_slot_info()
            capi.nnt_gpt2_model_slot(C.byref(b0.cfg), self.N_v, int(tile_v), s, C.byref(info))
            if info.used:
                zero = s < capi.NNT_MDL_LOWP            # parameters, gradients and moments start at zero
                self.slots[s] = TiledTensor(ctx, info.dtype, tuple(info.shape[:info.ndim]), tuple(info.basetile[:info.ndim]),
                                            fill=0 if zero else None)
        h = C.c_void_p()
        capi.nnt_gpt2_model_create(ctx.h, C.byref(b0.cfg), self.N_v, int(tile_v), self.stack.h,
                                   capi.ptr_array([t.h.value if t is not None else None for t in self.slots]), C.byref(h))
        self.h = h

        def group(p):
            lowp = self.slots[capi.NNT_MDL_LOWP + p] if p < 2 else None
            return dict(p=self.slots[p], g=self.slots[capi.NNT_MDL_GRAD + p], m=self.slots[capi.NNT_MDL_ADAM_M + p],
                        v=self.slots[capi.NNT_MDL_ADAM_V + p], lowp=lowp)
        self.wte, self.wpe = group(capi.NNT_MDL_WTE), group(capi.NNT_MDL_WPE)
        self.gamma, self.beta = group(capi.NNT_MDL_GAMMA_F), group(capi.NNT_MDL_BETA_F)
        self.logits = self.slots[capi.NNT_MDL_LOGITS]
        dev = "cuda:%d" % ctx.device
        self.col_loss = torch.empty(self.N_s * self.N_b, dtype=torch.float32, device=dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        pos = np.repeat(np.arange(self.N_s, dtype=np.int32)[:, None], self.N_b, axis=1)
        self.pos = torch.from_numpy(np.ascontiguousarray(pos.reshape(-1, order="F"))).to(dev)
        self.tokens = torch.zeros(self.N_s * self.N_b, dtype=torch.int32, device=dev)
        self.labels = torch.zeros(self.N_s * self.N_b, dtype=torch.int32, device=dev)
        torch.cuda.synchronize()

    def set_params(self, wte, wpe, gamma, beta):
        self.wte["p"].upload(wte)
        self.wpe["p"].upload(wpe)
        self.gamma["p"].upload(gamma)
        self.beta["p"].upload(beta)
        capi.nnt_gpt2_model_sync_lowp(self.h)
        self.ctx.wait()

    def set_batch(self, tokens, labels):
        """tokens, labels: integer arrays [N_s, N_b]."""
        for dst, a in ((self.tokens, tokens), (self.labels, labels)):
            dst.copy_(torch.from_numpy(np.ascontiguousarray(np.asarray(a, np.int32).reshape(-1, order="F"))))
        torch.cuda.synchronize()

    def forward(self):
        capi.nnt_gpt2_model_forward(self.h, self.tokens.data_ptr(), self.pos.data_ptr(), self.labels.data_ptr(),
                                    self.col_loss.data_ptr(), self.loss.data_ptr())

    def backward(self):
        capi.nnt_gpt2_model_backward(self.h)

    def adam(self, step, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
        cfg = capi.nnt_adam_cfg(lr, beta1, beta2, eps, weight_decay)
        capi.nnt_gpt2_model_adam(self.h, step, C.byref(cfg))

    def close(self):
        self.ctx.wait()
        if self.h:
            capi.nnt_gpt2_model_destroy(self.h)
            self.h = None
        self.stack.close()
