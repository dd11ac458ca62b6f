// One GPT-2 block as a flow of tile tasks (section 3: the layers of the GPT2 model
// in tile form; section 2: tasks are inserted in program order and run as soon as
// their tiles are ready).  Pre-LN block with biases on the four linear layers,
// causal attention and no dropout:
//
//   X1 = LN(X)            QKV = W_qkv X1 +. b      Q, K, V = heads(QKV)
//   P  = softmax(K^T Q / sqrt(h))  (causal)        B = V P      Bm = merge(B)
//   X2 = X + W_o Bm +. b_o
//   X3 = LN(X2)           H1 = W_1 X3 +. b_1       G = gelu(H1)
//   Out = X2 + W_2 G +. b_2
//
// The backward pass is the exact adjoint, in reverse order.
#include "internal.hpp"

#include <vector>

#include <cmath>

struct nnt_gpt2_block {
    nnt_ctx* ctx;
    nnt_gpt2_block_cfg cfg;
    nnt_tensor* s[NNT_BLK_NSLOTS];
    nnt_tensor* X;      // input of the last forward call
    nnt::AdamGroup* adam_group;   // all twelve parameters as one launch (made by the first whole-operation Adam step)
};

// A chain of blocks: acts[i] feeds block i, acts[n] is the output; dacts[i] is the gradient of acts[i].
struct nnt_gpt2_stack {
    nnt_ctx* ctx;
    std::vector<nnt_gpt2_block*> blocks;
    std::vector<nnt_tensor*> acts, dacts;
};

// A language model around a chain of blocks: the model's own tensors by slot, and what the last
// forward call was given.
struct nnt_gpt2_model {
    nnt_ctx* ctx;
    nnt_gpt2_block_cfg cfg;
    int64_t N_v;
    nnt_gpt2_stack* stack;
    nnt_tensor* s[NNT_MDL_NSLOTS];
    const int32_t* tokens;
    const int32_t* positions;
};

using namespace nnt;

namespace {

bool cfg_ok(const nnt_gpt2_block_cfg* c) {
    if (!c) return false;
    if (c->N_e < 1 || c->N_h < 1 || c->N_m < 1 || c->N_s < 1 || c->N_b < 1 || c->N_e % c->N_h != 0) return false;
    if (c->tile_e < 1 || c->tile_m < 1 || c->tile_s < 1 || c->tile_b < 1 || c->tile_j < 1 || c->tile_i < 1) return false;
    if (c->dtype != NNT_F32 && c->dtype != NNT_BF16) return false;
    if (c->gelu_variant != NNT_GELU_TANH && c->gelu_variant != NNT_GELU_ERF) return false;
    if (c->fused_attention != 0 && c->fused_attention != 1) return false;
    if (c->fused_attention && c->tile_i < c->N_e / c->N_h) return false;    // the fused kernels keep whole heads
    return true;
}

void set(nnt_slot_info* o, int dtype, int ndim, const int64_t* shape, const int64_t* base, int causal = 0) {
    o->used = 1;
    o->dtype = dtype;
    o->ndim = ndim;
    o->causal_tiles = causal;
    for (int a = 0; a < NNT_MAX_DIM; a++) {
        o->shape[a] = a < ndim ? shape[a] : 1;
        o->basetile[a] = a < ndim ? (base[a] < shape[a] ? base[a] : shape[a]) : 1;
    }
}

void param_geometry(const nnt_gpt2_block_cfg* c, int p, int* ndim, int64_t* shape, int64_t* base) {
    const int64_t e = c->N_e, m = c->N_m, te = c->tile_e, tm = c->tile_m;
    switch (p) {
        case NNT_BLK_W_QKV: *ndim = 2; shape[0] = 3 * e; shape[1] = e; base[0] = te; base[1] = te; break;
        case NNT_BLK_W_O: *ndim = 2; shape[0] = e; shape[1] = e; base[0] = te; base[1] = te; break;
        case NNT_BLK_W_1: *ndim = 2; shape[0] = m; shape[1] = e; base[0] = tm; base[1] = te; break;
        case NNT_BLK_W_2: *ndim = 2; shape[0] = e; shape[1] = m; base[0] = te; base[1] = tm; break;
        case NNT_BLK_B_QKV: *ndim = 1; shape[0] = 3 * e; base[0] = te; break;
        case NNT_BLK_B_1: *ndim = 1; shape[0] = m; base[0] = tm; break;
        default: *ndim = 1; shape[0] = e; base[0] = te; break;   // b_o, b_2, gains and biases of the layer norms
    }
}

}  // namespace

extern "C" {

int32_t nnt_gpt2_block_slot(const nnt_gpt2_block_cfg* c, int32_t slot, nnt_slot_info* o) {
    if (!cfg_ok(c) || !o || slot < 0 || slot >= NNT_BLK_NSLOTS) return NNT_EINVAL;
    *o = nnt_slot_info{};
    const int64_t e = c->N_e, m = c->N_m, s = c->N_s, b = c->N_b, j = c->N_h, h = c->N_e / c->N_h;
    const int64_t te = c->tile_e, tm = c->tile_m, ts = c->tile_s, tb = c->tile_b, tj = c->tile_j, ti = c->tile_i;
    const int act = c->dtype;
    int64_t shape[4], base[4];
    int ndim;
    if (slot < NNT_BLK_LOWP) {
        param_geometry(c, slot % 12, &ndim, shape, base);
        set(o, NNT_F32, ndim, shape, base);
        return NNT_OK;
    }
    if (slot < NNT_BLK_LOWP + 4) {
        if (act != NNT_BF16) return NNT_OK;      // unused in fp32 blocks
        param_geometry(c, slot - NNT_BLK_LOWP, &ndim, shape, base);
        set(o, NNT_BF16, ndim, shape, base);
        return NNT_OK;
    }
    const int64_t act3[3] = {e, s, b}, act3b[3] = {te, ts, tb};
    const int64_t qkv3[3] = {3 * e, s, b};
    const int64_t mlp3[3] = {m, s, b}, mlp3b[3] = {tm, ts, tb};
    const int64_t head4[4] = {h, s, b, j}, head4b[4] = {ti, ts, tb, tj};
    const int64_t sc4[4] = {s, s, b, j}, sc4b[4] = {ts, ts, tb, tj};
    const int64_t st3[3] = {2, s, b}, st3b[3] = {2, ts, tb};
    const int64_t st4[4] = {2, s, b, j}, st4b[4] = {2, ts, tb, tj};
    switch (slot) {
        case NNT_BLK_STATS1: case NNT_BLK_STATS2: set(o, NNT_F32, 3, st3, st3b); break;
        case NNT_BLK_SM_STATS: set(o, NNT_F32, 4, st4, st4b); break;
        case NNT_BLK_X1: case NNT_BLK_BM: case NNT_BLK_X2: case NNT_BLK_X3:
        case NNT_BLK_DX3: case NNT_BLK_DX2: case NNT_BLK_DBM: case NNT_BLK_DX1:
            set(o, act, 3, act3, act3b); break;
        case NNT_BLK_QKV: case NNT_BLK_DQKV: set(o, act, 3, qkv3, act3b); break;
        case NNT_BLK_Q: case NNT_BLK_K: case NNT_BLK_V: case NNT_BLK_BH:
        case NNT_BLK_DBH: case NNT_BLK_DQ: case NNT_BLK_DK: case NNT_BLK_DV:
            set(o, act, 4, head4, head4b); break;
        case NNT_BLK_P: case NNT_BLK_DP:
            if (!c->fused_attention) set(o, act, 4, sc4, sc4b, c->causal ? 1 : 0);   // never formed by the fused kernels
            break;
        case NNT_BLK_H1: case NNT_BLK_G: case NNT_BLK_DG: set(o, act, 3, mlp3, mlp3b); break;
        default: return NNT_EINVAL;
    }
    return NNT_OK;
}

int32_t nnt_gpt2_block_create(nnt_ctx* ctx, const nnt_gpt2_block_cfg* cfg, nnt_tensor* const* slots, nnt_gpt2_block** out) {
    NNT_CHECK_CTX(ctx);
    if (!out) return NNT_EINVAL;
    *out = nullptr;
    if (!cfg_ok(cfg) || !slots) return fail(ctx, NNT_EINVAL, "nnt_gpt2_block_create: bad configuration");
    nnt_gpt2_block* blk = new (std::nothrow) nnt_gpt2_block();
    if (!blk) return fail(ctx, NNT_ENOMEM, "host allocation failed");
    blk->ctx = ctx;
    blk->cfg = *cfg;
    blk->X = nullptr;
    for (int i = 0; i < NNT_BLK_NSLOTS; i++) {
        nnt_slot_info info;
        nnt_gpt2_block_slot(cfg, i, &info);
        nnt_tensor* t = slots[i];
        blk->s[i] = t;
        const bool optional = i >= NNT_BLK_ADAM_M && i < NNT_BLK_LOWP;
        if (!info.used) continue;
        if (!t) {
            if (optional) continue;
            delete blk;
            return fail(ctx, NNT_EINVAL, "nnt_gpt2_block_create: missing tensor for slot " + std::to_string(i));
        }
        bool ok = t->ctx == ctx && t->dtype == info.dtype && t->ndim == info.ndim;
        for (int a = 0; ok && a < info.ndim; a++) ok = t->shape[a] == info.shape[a] && t->base[a] == info.basetile[a];
        if (!ok) {
            delete blk;
            return fail(ctx, NNT_EINVAL, "nnt_gpt2_block_create: tensor of slot " + std::to_string(i) + " has the wrong type, shape or tiling");
        }
    }
    *out = blk;
    return NNT_OK;
}

int32_t nnt_gpt2_block_destroy(nnt_gpt2_block* blk) {
    if (!blk) return NNT_EINVAL;
    nnt::adam_group_destroy(blk->adam_group);
    delete blk;
    return NNT_OK;
}

#define TRY(x)                      \
    do {                            \
        int32_t rc__ = (x);         \
        if (rc__ != NNT_OK) return rc__; \
    } while (0)

static nnt_tensor* weight(nnt_gpt2_block* b, int p) { return b->cfg.dtype == NNT_BF16 ? b->s[NNT_BLK_LOWP + p] : b->s[p]; }

// Y = W X +. bias (+ R, the input of a residual connection): bias and residual ride in the
// product's epilogue when one launch covers the whole operation, and are tile tasks of their
// own otherwise.
static int32_t linear(nnt_gpt2_block* b, nnt_tensor* W, nnt_tensor* X, nnt_tensor* bias, nnt_tensor* Y, nnt_tensor* R = nullptr) {
    nnt_ctx* ctx = b->ctx;
    if (ctx->granularity == NNT_GRAN_OP)
        return nnt_gemm_res(ctx, 1.f, NNT_OP_N, W, NNT_OP_N, X, R ? 1.f : 0.f, Y, 1, 0, bias, R);
    TRY(nnt_gemm(ctx, 1.f, NNT_OP_N, W, NNT_OP_N, X, 0.f, Y, 1, 0, nullptr));
    TRY(nnt_bias_add(ctx, bias, Y));
    return R ? nnt_add(ctx, 1.f, R, 1.f, Y) : NNT_OK;
}

// dX = W^T dY,  dW = sum_{s,b} dY X^T,  db = sum_{s,b} dY
static int32_t linear_bwd(nnt_gpt2_block* b, nnt_tensor* W, nnt_tensor* X, nnt_tensor* dY, nnt_tensor* dX,
                          nnt_tensor* dW, nnt_tensor* db) {
    nnt_ctx* ctx = b->ctx;
    TRY(nnt_gemm(ctx, 1.f, NNT_OP_N, dY, NNT_OP_T, X, 0.f, dW, 2, 0, nullptr));
    TRY(nnt_bias_grad(ctx, dY, db));
    return nnt_gemm(ctx, 1.f, NNT_OP_T, W, NNT_OP_N, dY, 0.f, dX, 1, 0, nullptr);
}

// Whether the activation and its derivative ride on the result paths of the products next to them (nnt_gemm_gelu,
// nnt_gemm_gelu_bwd) instead of being passes of their own: whole-operation launches in fp32 (the bf16 product kernels
// have no such form).  (NNT_BLOCK_GELU_PASSES=1 keeps the passes: a measuring aid.)
static bool gelu_in_products(const nnt_gpt2_block* b) {
    static const bool passes = getenv("NNT_BLOCK_GELU_PASSES") != nullptr;
    return !passes && b->ctx->granularity == NNT_GRAN_OP && b->cfg.dtype == NNT_F32;
}

// Whether the attention products read and write the tensors of the linear layers directly (nnt_gemm_heads)
// instead of per-head copies: whole-operation launches and row tiles that hold whole heads and divide the
// embedding size.  (NNT_BLOCK_HEAD_COPIES=1 keeps the copies: a measuring aid.)
static bool head_windows(const nnt_gpt2_block* b) {
    static const bool copies = getenv("NNT_BLOCK_HEAD_COPIES") != nullptr;
    const nnt_gpt2_block_cfg& c = b->cfg;
    if (copies || b->ctx->granularity != NNT_GRAN_OP) return false;
    const int64_t h = c.N_e / c.N_h, t0 = b->s[NNT_BLK_QKV]->base[0];
    if (c.fused_attention && h != 64 && h != 128) return false;
    return t0 % h == 0 && c.N_e % t0 == 0 && b->s[NNT_BLK_BM]->base[0] == t0 && b->s[NNT_BLK_DBM]->base[0] == t0 &&
           b->s[NNT_BLK_DQKV]->base[0] == t0;
}

int32_t nnt_gpt2_block_forward(nnt_gpt2_block* b, nnt_tensor* X, nnt_tensor* Out) {
    if (!b) return NNT_EINVAL;
    nnt_ctx* ctx = b->ctx;
    NNT_CHECK_CTX(ctx);
    if (!X || !Out) return fail(ctx, NNT_EINVAL, "nnt_gpt2_block_forward: null tensor");
    nnt_tensor** s = b->s;
    const nnt_gpt2_block_cfg& c = b->cfg;
    const float sc = 1.f / std::sqrt((float)(c.N_e / c.N_h));
    if (!same_tiling(X, s[NNT_BLK_X1]) || !same_tiling(Out, s[NNT_BLK_X1]) || X->dtype != c.dtype || Out->dtype != c.dtype)
        return fail(ctx, NNT_EINVAL, "nnt_gpt2_block_forward: X / Out do not match the block's activations");
    b->X = X;
    TRY(nnt_layernorm_fwd(ctx, X, s[NNT_BLK_GAMMA1], s[NNT_BLK_BETA1], c.eps, s[NNT_BLK_X1], s[NNT_BLK_STATS1]));
    TRY(linear(b, weight(b, NNT_BLK_W_QKV), s[NNT_BLK_X1], s[NNT_BLK_B_QKV], s[NNT_BLK_QKV]));
    if (head_windows(b)) {
        // parts 0, 1, 2 of the QKV rows are Q, K, V; the heads' results go straight into Bm
        const int32_t h = (int32_t)(c.N_e / c.N_h), N_h = (int32_t)c.N_h;
        if (c.fused_attention) {
            TRY(nnt_attention_fwd_heads(ctx, s[NNT_BLK_QKV], sc, c.causal, s[NNT_BLK_BM], s[NNT_BLK_SM_STATS], N_h));
        } else {
            TRY(nnt_gemm_heads(ctx, sc, NNT_OP_T, s[NNT_BLK_QKV], 1, NNT_OP_N, s[NNT_BLK_QKV], 0, s[NNT_BLK_P], -1, h, N_h));
            TRY(nnt_softmax_fwd(ctx, s[NNT_BLK_P], s[NNT_BLK_SM_STATS], 1.f, c.causal));
            TRY(nnt_gemm_heads(ctx, 1.f, NNT_OP_N, s[NNT_BLK_QKV], 2, NNT_OP_N, s[NNT_BLK_P], -1, s[NNT_BLK_BM], 0, h, N_h));
        }
    } else {
        nnt_tensor* qkv[3] = {s[NNT_BLK_Q], s[NNT_BLK_K], s[NNT_BLK_V]};
        TRY(nnt_head_split(ctx, s[NNT_BLK_QKV], 3, qkv));
        if (c.fused_attention) {
            TRY(nnt_attention_fwd(ctx, s[NNT_BLK_Q], s[NNT_BLK_K], s[NNT_BLK_V], sc, c.causal, s[NNT_BLK_BH], s[NNT_BLK_SM_STATS]));
        } else {
            TRY(nnt_gemm(ctx, sc, NNT_OP_T, s[NNT_BLK_K], NNT_OP_N, s[NNT_BLK_Q], 0.f, s[NNT_BLK_P], 1, 2, nullptr));
            TRY(nnt_softmax_fwd(ctx, s[NNT_BLK_P], s[NNT_BLK_SM_STATS], 1.f, c.causal));
            TRY(nnt_gemm(ctx, 1.f, NNT_OP_N, s[NNT_BLK_V], NNT_OP_N, s[NNT_BLK_P], 0.f, s[NNT_BLK_BH], 1, 2, nullptr));
        }
        nnt_tensor* bh[1] = {s[NNT_BLK_BH]};
        TRY(nnt_head_merge(ctx, 1, bh, s[NNT_BLK_BM]));
    }
    TRY(linear(b, weight(b, NNT_BLK_W_O), s[NNT_BLK_BM], s[NNT_BLK_B_O], s[NNT_BLK_X2], X));      // X2 = X + W_o Bm +. b_o
    TRY(nnt_layernorm_fwd(ctx, s[NNT_BLK_X2], s[NNT_BLK_GAMMA2], s[NNT_BLK_BETA2], c.eps, s[NNT_BLK_X3], s[NNT_BLK_STATS2]));
    if (gelu_in_products(b)) {                                                                   // H1 and G = gelu(H1) from one launch
        TRY(nnt_gemm_gelu(ctx, 1.f, NNT_OP_N, weight(b, NNT_BLK_W_1), NNT_OP_N, s[NNT_BLK_X3], s[NNT_BLK_H1], 1, s[NNT_BLK_B_1],
                          c.gelu_variant, s[NNT_BLK_G]));
    } else {
        TRY(linear(b, weight(b, NNT_BLK_W_1), s[NNT_BLK_X3], s[NNT_BLK_B_1], s[NNT_BLK_H1]));
        TRY(nnt_gelu(ctx, c.gelu_variant, s[NNT_BLK_H1], s[NNT_BLK_G]));
    }
    return linear(b, weight(b, NNT_BLK_W_2), s[NNT_BLK_G], s[NNT_BLK_B_2], Out, s[NNT_BLK_X2]);   // Out = X2 + W_2 G +. b_2
}

int32_t nnt_gpt2_block_backward(nnt_gpt2_block* b, nnt_tensor* dOut, nnt_tensor* dX) {
    if (!b) return NNT_EINVAL;
    nnt_ctx* ctx = b->ctx;
    NNT_CHECK_CTX(ctx);
    if (!dOut || !dX) return fail(ctx, NNT_EINVAL, "nnt_gpt2_block_backward: null tensor");
    if (!b->X) return fail(ctx, NNT_ESTATE, "nnt_gpt2_block_backward: no forward pass to differentiate");
    nnt_tensor** s = b->s;
    const nnt_gpt2_block_cfg& c = b->cfg;
    const float sc = 1.f / std::sqrt((float)(c.N_e / c.N_h));
    if (!same_tiling(dOut, s[NNT_BLK_X1]) || !same_tiling(dX, s[NNT_BLK_X1]) || dOut->dtype != c.dtype || dX->dtype != c.dtype)
        return fail(ctx, NNT_EINVAL, "nnt_gpt2_block_backward: dOut / dX do not match the block's activations");
    nnt_tensor** g = s + NNT_BLK_GRAD;
    // MLP
    if (gelu_in_products(b)) {                                                                   // dH1 = (W_2^T dOut) * gelu'(H1) from one launch
        TRY(nnt_gemm(ctx, 1.f, NNT_OP_N, dOut, NNT_OP_T, s[NNT_BLK_G], 0.f, g[NNT_BLK_W_2], 2, 0, nullptr));
        TRY(nnt_bias_grad(ctx, dOut, g[NNT_BLK_B_2]));
        TRY(nnt_gemm_gelu_bwd(ctx, 1.f, NNT_OP_T, weight(b, NNT_BLK_W_2), NNT_OP_N, dOut, s[NNT_BLK_DG], 1, c.gelu_variant, s[NNT_BLK_H1]));
    } else {
        TRY(linear_bwd(b, weight(b, NNT_BLK_W_2), s[NNT_BLK_G], dOut, s[NNT_BLK_DG], g[NNT_BLK_W_2], g[NNT_BLK_B_2]));
        TRY(nnt_gelu_bwd(ctx, c.gelu_variant, s[NNT_BLK_H1], s[NNT_BLK_DG], s[NNT_BLK_DG]));
    }
    TRY(linear_bwd(b, weight(b, NNT_BLK_W_1), s[NNT_BLK_X3], s[NNT_BLK_DG], s[NNT_BLK_DX3], g[NNT_BLK_W_1], g[NNT_BLK_B_1]));
    // second layer norm; the residual branch adds dOut
    TRY(nnt_layernorm_bwd(ctx, s[NNT_BLK_X2], s[NNT_BLK_STATS2], s[NNT_BLK_GAMMA2], s[NNT_BLK_DX3], dOut, s[NNT_BLK_DX2],
                          g[NNT_BLK_GAMMA2], g[NNT_BLK_BETA2]));
    // attention output projection
    TRY(linear_bwd(b, weight(b, NNT_BLK_W_O), s[NNT_BLK_BM], s[NNT_BLK_DX2], s[NNT_BLK_DBM], g[NNT_BLK_W_O], g[NNT_BLK_B_O]));
    if (head_windows(b)) {
        // dV = dB P^T, dP = V^T dB, softmax adjoint, dQ = K dA / sqrt(h), dK = Q dA^T / sqrt(h): dB is read out of dBm,
        // the three results are the parts of dQKV
        const int32_t h = (int32_t)(c.N_e / c.N_h), N_h = (int32_t)c.N_h;
        if (c.fused_attention) {
            TRY(nnt_attention_bwd_heads(ctx, s[NNT_BLK_QKV], s[NNT_BLK_BM], s[NNT_BLK_SM_STATS], s[NNT_BLK_DBM], sc, c.causal,
                                        s[NNT_BLK_DQKV], N_h));
        } else {
            TRY(nnt_gemm_heads(ctx, 1.f, NNT_OP_N, s[NNT_BLK_DBM], 0, NNT_OP_T, s[NNT_BLK_P], -1, s[NNT_BLK_DQKV], 2, h, N_h));
            TRY(nnt_gemm_heads(ctx, 1.f, NNT_OP_T, s[NNT_BLK_QKV], 2, NNT_OP_N, s[NNT_BLK_DBM], 0, s[NNT_BLK_DP], -1, h, N_h));
            TRY(nnt_softmax_bwd(ctx, s[NNT_BLK_P], s[NNT_BLK_DP]));
            TRY(nnt_gemm_heads(ctx, sc, NNT_OP_N, s[NNT_BLK_QKV], 1, NNT_OP_N, s[NNT_BLK_DP], -1, s[NNT_BLK_DQKV], 0, h, N_h));
            TRY(nnt_gemm_heads(ctx, sc, NNT_OP_N, s[NNT_BLK_QKV], 0, NNT_OP_T, s[NNT_BLK_DP], -1, s[NNT_BLK_DQKV], 1, h, N_h));
        }
    } else {
        nnt_tensor* dbh[1] = {s[NNT_BLK_DBH]};
        TRY(nnt_head_split(ctx, s[NNT_BLK_DBM], 1, dbh));
        if (c.fused_attention) {
            TRY(nnt_attention_bwd(ctx, s[NNT_BLK_Q], s[NNT_BLK_K], s[NNT_BLK_V], s[NNT_BLK_BH], s[NNT_BLK_SM_STATS], s[NNT_BLK_DBH],
                                  sc, c.causal, s[NNT_BLK_DQ], s[NNT_BLK_DK], s[NNT_BLK_DV]));
        } else {
            // dV = dB P^T, dP = V^T dB, softmax adjoint, dQ = K dA / sqrt(h), dK = Q dA^T / sqrt(h)
            TRY(nnt_gemm(ctx, 1.f, NNT_OP_N, s[NNT_BLK_DBH], NNT_OP_T, s[NNT_BLK_P], 0.f, s[NNT_BLK_DV], 1, 2, nullptr));
            TRY(nnt_gemm(ctx, 1.f, NNT_OP_T, s[NNT_BLK_V], NNT_OP_N, s[NNT_BLK_DBH], 0.f, s[NNT_BLK_DP], 1, 2, nullptr));
            TRY(nnt_softmax_bwd(ctx, s[NNT_BLK_P], s[NNT_BLK_DP]));
            TRY(nnt_gemm(ctx, sc, NNT_OP_N, s[NNT_BLK_K], NNT_OP_N, s[NNT_BLK_DP], 0.f, s[NNT_BLK_DQ], 1, 2, nullptr));
            TRY(nnt_gemm(ctx, sc, NNT_OP_N, s[NNT_BLK_Q], NNT_OP_T, s[NNT_BLK_DP], 0.f, s[NNT_BLK_DK], 1, 2, nullptr));
        }
        nnt_tensor* dqkv[3] = {s[NNT_BLK_DQ], s[NNT_BLK_DK], s[NNT_BLK_DV]};
        TRY(nnt_head_merge(ctx, 3, dqkv, s[NNT_BLK_DQKV]));
    }
    TRY(linear_bwd(b, weight(b, NNT_BLK_W_QKV), s[NNT_BLK_X1], s[NNT_BLK_DQKV], s[NNT_BLK_DX1], g[NNT_BLK_W_QKV], g[NNT_BLK_B_QKV]));
    // first layer norm; the residual branch adds dX2
    return nnt_layernorm_bwd(ctx, b->X, s[NNT_BLK_STATS1], s[NNT_BLK_GAMMA1], s[NNT_BLK_DX1], s[NNT_BLK_DX2], dX,
                             g[NNT_BLK_GAMMA1], g[NNT_BLK_BETA1]);
}

int32_t nnt_gpt2_block_adam(nnt_gpt2_block* b, int32_t step, const nnt_adam_cfg* cfg) {
    if (!b) return NNT_EINVAL;
    nnt_ctx* ctx = b->ctx;
    NNT_CHECK_CTX(ctx);
    if (!cfg || step < 1) return fail(ctx, NNT_EINVAL, "nnt_gpt2_block_adam: bad argument");
    for (int p = 0; p < 12; p++)
        if (!b->s[NNT_BLK_ADAM_M + p] || !b->s[NNT_BLK_ADAM_V + p])
            return fail(ctx, NNT_ESTATE, "nnt_gpt2_block_adam: the block was created without Adam moments");
    if (ctx->granularity == NNT_GRAN_OP) {
        if (!b->adam_group) {
            if (ctx->capturing) return fail(ctx, NNT_ESTATE, "nnt_gpt2_block_adam: run the step once before capture");
            nnt_tensor* lowp[12];
            for (int p = 0; p < 12; p++) lowp[p] = (b->cfg.dtype == NNT_BF16 && p < 4) ? b->s[NNT_BLK_LOWP + p] : nullptr;
            TRY(adam_group_create(ctx, 12, b->s + NNT_BLK_GRAD, b->s, b->s + NNT_BLK_ADAM_M, b->s + NNT_BLK_ADAM_V, lowp, &b->adam_group));
        }
        return adam_group_step(ctx, b->adam_group, cfg, step);
    }
    for (int p = 0; p < 12; p++) {
        nnt_tensor* lowp = (b->cfg.dtype == NNT_BF16 && p < 4) ? b->s[NNT_BLK_LOWP + p] : nullptr;
        TRY(nnt_adam_step(ctx, cfg, step, b->s[NNT_BLK_GRAD + p], b->s[p], b->s[NNT_BLK_ADAM_M + p], b->s[NNT_BLK_ADAM_V + p], lowp));
    }
    return NNT_OK;
}

int32_t nnt_gpt2_block_sgd(nnt_gpt2_block* b, const nnt_sgd_cfg* cfg) {
    if (!b) return NNT_EINVAL;
    nnt_ctx* ctx = b->ctx;
    NNT_CHECK_CTX(ctx);
    if (!cfg) return fail(ctx, NNT_EINVAL, "nnt_gpt2_block_sgd: bad argument");
    for (int p = 0; p < 12; p++)
        if (!b->s[NNT_BLK_ADAM_M + p])
            return fail(ctx, NNT_ESTATE, "nnt_gpt2_block_sgd: the block was created without moment tensors");
    for (int p = 0; p < 12; p++) {
        nnt_tensor* lowp = (b->cfg.dtype == NNT_BF16 && p < 4) ? b->s[NNT_BLK_LOWP + p] : nullptr;
        TRY(nnt_sgd_step(ctx, cfg, b->s[NNT_BLK_GRAD + p], b->s[p], b->s[NNT_BLK_ADAM_M + p], lowp));
    }
    return NNT_OK;
}

int32_t nnt_gpt2_block_grads_axpy(nnt_gpt2_block* b, float alpha, nnt_tensor* const* acc) {
    if (!b) return NNT_EINVAL;
    nnt_ctx* ctx = b->ctx;
    NNT_CHECK_CTX(ctx);
    if (!acc) return fail(ctx, NNT_EINVAL, "nnt_gpt2_block_grads_axpy: bad argument");
    for (int p = 0; p < 12; p++)
        if (!acc[p]) return fail(ctx, NNT_EINVAL, "nnt_gpt2_block_grads_axpy: missing accumulator");
    for (int p = 0; p < 12; p++) TRY(nnt_add(ctx, alpha, b->s[NNT_BLK_GRAD + p], 1.f, acc[p]));
    return NNT_OK;
}

int32_t nnt_gpt2_stack_create(nnt_ctx* ctx, int32_t n_blocks, nnt_gpt2_block* const* blocks, nnt_tensor* const* acts,
                              nnt_tensor* const* dacts, nnt_gpt2_stack** out) {
    NNT_CHECK_CTX(ctx);
    if (!out) return NNT_EINVAL;
    *out = nullptr;
    if (n_blocks < 1 || !blocks || !acts || !dacts) return fail(ctx, NNT_EINVAL, "nnt_gpt2_stack_create: bad argument");
    for (int i = 0; i < n_blocks; i++)
        if (!blocks[i] || blocks[i]->ctx != ctx) return fail(ctx, NNT_EINVAL, "nnt_gpt2_stack_create: block of another context");
    for (int i = 0; i <= n_blocks; i++) {
        const nnt_tensor* like = blocks[0]->s[NNT_BLK_X1];
        if (!acts[i] || !dacts[i] || !same_tiling(acts[i], like) || !same_tiling(dacts[i], like) ||
            acts[i]->dtype != like->dtype || dacts[i]->dtype != like->dtype)
            return fail(ctx, NNT_EINVAL, "nnt_gpt2_stack_create: activation " + std::to_string(i) + " does not match the blocks");
    }
    nnt_gpt2_stack* st = new (std::nothrow) nnt_gpt2_stack();
    if (!st) return fail(ctx, NNT_ENOMEM, "host allocation failed");
    st->ctx = ctx;
    st->blocks.assign(blocks, blocks + n_blocks);
    st->acts.assign(acts, acts + n_blocks + 1);
    st->dacts.assign(dacts, dacts + n_blocks + 1);
    *out = st;
    return NNT_OK;
}

int32_t nnt_gpt2_stack_destroy(nnt_gpt2_stack* st) {
    if (!st) return NNT_EINVAL;
    delete st;
    return NNT_OK;
}

int32_t nnt_gpt2_stack_forward(nnt_gpt2_stack* st) {
    if (!st) return NNT_EINVAL;
    for (size_t i = 0; i < st->blocks.size(); i++) TRY(nnt_gpt2_block_forward(st->blocks[i], st->acts[i], st->acts[i + 1]));
    return NNT_OK;
}

int32_t nnt_gpt2_stack_backward(nnt_gpt2_stack* st) {
    if (!st) return NNT_EINVAL;
    for (size_t i = st->blocks.size(); i-- > 0;) TRY(nnt_gpt2_block_backward(st->blocks[i], st->dacts[i + 1], st->dacts[i]));
    return NNT_OK;
}

int32_t nnt_gpt2_stack_adam(nnt_gpt2_stack* st, int32_t step, const nnt_adam_cfg* cfg) {
    if (!st) return NNT_EINVAL;
    for (nnt_gpt2_block* b : st->blocks) TRY(nnt_gpt2_block_adam(b, step, cfg));
    return NNT_OK;
}

int32_t nnt_gpt2_block_sync_lowp(nnt_gpt2_block* b) {
    if (!b) return NNT_EINVAL;
    nnt_ctx* ctx = b->ctx;
    NNT_CHECK_CTX(ctx);
    if (b->cfg.dtype != NNT_BF16) return NNT_OK;
    for (int p = 0; p < 4; p++) TRY(nnt_cast(ctx, b->s[p], b->s[NNT_BLK_LOWP + p]));
    return NNT_OK;
}

// ---------------------------------------------------------------- language model
int32_t nnt_gpt2_model_slot(const nnt_gpt2_block_cfg* c, int64_t N_v, int64_t tile_v, int32_t slot, nnt_slot_info* o) {
    if (!cfg_ok(c) || !o || slot < 0 || slot >= NNT_MDL_NSLOTS || N_v < 1 || tile_v < 1) return NNT_EINVAL;
    *o = nnt_slot_info{};
    const int64_t e = c->N_e, sq = c->N_s, b = c->N_b, te = c->tile_e, ts = c->tile_s, tb = c->tile_b;
    const int64_t wte[2] = {e, N_v}, wteb[2] = {te, tile_v}, wpe[2] = {e, sq}, wpeb[2] = {te, ts}, vec[1] = {e}, vecb[1] = {te};
    const int64_t act3[3] = {e, sq, b}, act3b[3] = {te, ts, tb}, st3[3] = {2, sq, b}, st3b[3] = {2, ts, tb};
    const int64_t lg3[3] = {N_v, sq, b}, lg3b[3] = {tile_v, ts, tb};
    if (slot < NNT_MDL_LOWP + 2) {
        const int p = slot < NNT_MDL_LOWP ? slot % 4 : slot - NNT_MDL_LOWP;
        const int dt = slot < NNT_MDL_LOWP ? NNT_F32 : NNT_BF16;
        if (slot >= NNT_MDL_LOWP && c->dtype != NNT_BF16) return NNT_OK;      // unused in fp32 models
        if (p == NNT_MDL_WTE) set(o, dt, 2, wte, wteb);
        else if (p == NNT_MDL_WPE) set(o, dt, 2, wpe, wpeb);
        else set(o, dt, 1, vec, vecb);
        return NNT_OK;
    }
    switch (slot) {
        case NNT_MDL_XPOS: case NNT_MDL_XF: case NNT_MDL_DXF: set(o, c->dtype, 3, act3, act3b); break;
        case NNT_MDL_STATS_F: case NNT_MDL_LOSS_STATS: set(o, NNT_F32, 3, st3, st3b); break;
        case NNT_MDL_LOGITS: set(o, c->dtype, 3, lg3, lg3b); break;
        default: return NNT_EINVAL;
    }
    return NNT_OK;
}

int32_t nnt_gpt2_model_create(nnt_ctx* ctx, const nnt_gpt2_block_cfg* cfg, int64_t N_v, int64_t tile_v, nnt_gpt2_stack* stack,
                              nnt_tensor* const* slots, nnt_gpt2_model** out) {
    NNT_CHECK_CTX(ctx);
    if (!out) return NNT_EINVAL;
    *out = nullptr;
    if (!cfg_ok(cfg) || !slots || !stack || stack->ctx != ctx || N_v < 1 || tile_v < 1)
        return fail(ctx, NNT_EINVAL, "nnt_gpt2_model_create: bad argument");
    if (!same_tiling(stack->acts[0], stack->blocks[0]->s[NNT_BLK_X1]) || stack->blocks[0]->cfg.N_e != cfg->N_e ||
        stack->blocks[0]->cfg.N_s != cfg->N_s || stack->blocks[0]->cfg.N_b != cfg->N_b || stack->blocks[0]->cfg.dtype != cfg->dtype)
        return fail(ctx, NNT_EINVAL, "nnt_gpt2_model_create: the stack's blocks do not match the configuration");
    nnt_gpt2_model* m = new (std::nothrow) nnt_gpt2_model();
    if (!m) return fail(ctx, NNT_ENOMEM, "host allocation failed");
    m->ctx = ctx;
    m->cfg = *cfg;
    m->N_v = N_v;
    m->stack = stack;
    m->tokens = m->positions = nullptr;
    for (int i = 0; i < NNT_MDL_NSLOTS; i++) {
        nnt_slot_info info;
        nnt_gpt2_model_slot(cfg, N_v, tile_v, i, &info);
        nnt_tensor* t = slots[i];
        m->s[i] = t;
        if (!info.used) continue;
        const bool optional = i >= NNT_MDL_ADAM_M && i < NNT_MDL_LOWP;
        if (!t) {
            if (optional) continue;
            delete m;
            return fail(ctx, NNT_EINVAL, "nnt_gpt2_model_create: missing tensor for slot " + std::to_string(i));
        }
        bool ok = t->ctx == ctx && t->dtype == info.dtype && t->ndim == info.ndim;
        for (int a = 0; ok && a < info.ndim; a++) ok = t->shape[a] == info.shape[a] && t->base[a] == info.basetile[a];
        if (!ok) {
            delete m;
            return fail(ctx, NNT_EINVAL, "nnt_gpt2_model_create: tensor of slot " + std::to_string(i) + " has the wrong type, shape or tiling");
        }
    }
    *out = m;
    return NNT_OK;
}

int32_t nnt_gpt2_model_destroy(nnt_gpt2_model* m) {
    if (!m) return NNT_EINVAL;
    delete m;
    return NNT_OK;
}

static nnt_tensor* table_of(nnt_gpt2_model* m, int p) { return m->cfg.dtype == NNT_BF16 ? m->s[NNT_MDL_LOWP + p] : m->s[p]; }

int32_t nnt_gpt2_model_sync_lowp(nnt_gpt2_model* m) {
    if (!m) return NNT_EINVAL;
    NNT_CHECK_CTX(m->ctx);
    if (m->cfg.dtype != NNT_BF16) return NNT_OK;
    for (int p = 0; p < 2; p++) TRY(nnt_cast(m->ctx, m->s[p], m->s[NNT_MDL_LOWP + p]));
    return NNT_OK;
}

int32_t nnt_gpt2_model_forward(nnt_gpt2_model* m, const int32_t* tokens, const int32_t* positions, const int32_t* labels,
                               float* col_loss, float* loss) {
    if (!m) return NNT_EINVAL;
    nnt_ctx* ctx = m->ctx;
    NNT_CHECK_CTX(ctx);
    if (!tokens || !positions || !labels || !col_loss || !loss) return fail(ctx, NNT_EINVAL, "nnt_gpt2_model_forward: null argument");
    nnt_gpt2_stack* st = m->stack;
    nnt_tensor** s = m->s;
    m->tokens = tokens;
    m->positions = positions;
    // X_0 = W_te[:, token] + W_pe[:, position]
    TRY(nnt_embedding_fwd(ctx, tokens, table_of(m, NNT_MDL_WTE), st->acts[0]));
    TRY(nnt_embedding_fwd(ctx, positions, table_of(m, NNT_MDL_WPE), s[NNT_MDL_XPOS]));
    TRY(nnt_add(ctx, 1.f, s[NNT_MDL_XPOS], 1.f, st->acts[0]));
    TRY(nnt_gpt2_stack_forward(st));
    TRY(nnt_layernorm_fwd(ctx, st->acts.back(), s[NNT_MDL_GAMMA_F], s[NNT_MDL_BETA_F], m->cfg.eps, s[NNT_MDL_XF], s[NNT_MDL_STATS_F]));
    // logits = W_te^T X_f (the head shares the token embedding), then the loss, which leaves dL/dlogits in place
    TRY(nnt_gemm(ctx, 1.f, NNT_OP_T, table_of(m, NNT_MDL_WTE), NNT_OP_N, s[NNT_MDL_XF], 0.f, s[NNT_MDL_LOGITS], 1, 0, nullptr));
    return nnt_cross_entropy(ctx, s[NNT_MDL_LOGITS], labels, s[NNT_MDL_LOSS_STATS], col_loss, loss);
}

int32_t nnt_gpt2_model_backward(nnt_gpt2_model* m) {
    if (!m) return NNT_EINVAL;
    nnt_ctx* ctx = m->ctx;
    NNT_CHECK_CTX(ctx);
    if (!m->tokens) return fail(ctx, NNT_ESTATE, "nnt_gpt2_model_backward: no forward pass to differentiate");
    nnt_gpt2_stack* st = m->stack;
    nnt_tensor** s = m->s;
    nnt_tensor** g = s + NNT_MDL_GRAD;
    // dX_f = W_te dlogits;  dW_te = X_f dlogits^T (the head's share, summed over positions and batch)
    TRY(nnt_gemm(ctx, 1.f, NNT_OP_N, table_of(m, NNT_MDL_WTE), NNT_OP_N, s[NNT_MDL_LOGITS], 0.f, s[NNT_MDL_DXF], 1, 0, nullptr));
    TRY(nnt_gemm(ctx, 1.f, NNT_OP_N, s[NNT_MDL_XF], NNT_OP_T, s[NNT_MDL_LOGITS], 0.f, g[NNT_MDL_WTE], 2, 0, nullptr));
    TRY(nnt_layernorm_bwd(ctx, st->acts.back(), s[NNT_MDL_STATS_F], s[NNT_MDL_GAMMA_F], s[NNT_MDL_DXF], nullptr, st->dacts.back(),
                          g[NNT_MDL_GAMMA_F], g[NNT_MDL_BETA_F]));
    TRY(nnt_gpt2_stack_backward(st));
    // the lookups' share: columns of dX_0 added to the columns of their tokens / positions
    TRY(nnt_embedding_bwd(ctx, m->tokens, st->dacts[0], g[NNT_MDL_WTE]));
    TRY(nnt_fill(ctx, 0.f, g[NNT_MDL_WPE]));
    return nnt_embedding_bwd(ctx, m->positions, st->dacts[0], g[NNT_MDL_WPE]);
}

int32_t nnt_gpt2_model_adam(nnt_gpt2_model* m, int32_t step, const nnt_adam_cfg* cfg) {
    if (!m) return NNT_EINVAL;
    nnt_ctx* ctx = m->ctx;
    NNT_CHECK_CTX(ctx);
    if (!cfg || step < 1) return fail(ctx, NNT_EINVAL, "nnt_gpt2_model_adam: bad argument");
    for (int p = 0; p < 4; p++)
        if (!m->s[NNT_MDL_ADAM_M + p] || !m->s[NNT_MDL_ADAM_V + p])
            return fail(ctx, NNT_ESTATE, "nnt_gpt2_model_adam: the model was created without Adam moments");
    TRY(nnt_gpt2_stack_adam(m->stack, step, cfg));
    for (int p = 0; p < 4; p++) {
        nnt_tensor* lowp = (m->cfg.dtype == NNT_BF16 && p < 2) ? m->s[NNT_MDL_LOWP + p] : nullptr;
        TRY(nnt_adam_step(ctx, cfg, step, m->s[NNT_MDL_GRAD + p], m->s[p], m->s[NNT_MDL_ADAM_M + p], m->s[NNT_MDL_ADAM_V + p], lowp));
    }
    return NNT_OK;
}

}  // extern "C"
