// Embedding layer and cross-entropy loss (section 3, Embedding layer and
// Cross-Entropy loss) on tiled tensors.
//
//   embedding   Y[e, s, b] = W[e, token(s, b)]            W: N_e x N_v, one column per vocabulary item
//   adjoint     dW[e, v] += sum over (s, b) with token(s, b) = v of dY[e, s, b]
//   loss        L = - sum_{s, b} log( exp(x[c, s, b]) / sum_j exp(x[j, s, b]) ),  c = label(s, b)
//
// The loss is computed on logits split into vocabulary tiles with the SoftMax
// subroutines: the running (maximum, sum of shifted exponentials) of every column,
// then the probabilities in place (nnt_softmax_fwd); what is left for this file is
// one element per column: -log of the label's probability, and minus one on that
// entry, which turns the probabilities into the gradient of L with respect to x.
#include "device_util.hpp"
#include "internal.hpp"

namespace nnt {
namespace {

template <typename T> __device__ __forceinline__ float ldf(const T* p);
template <> __device__ __forceinline__ float ldf<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ldf<bf16_t>(const bf16_t* p) { return bf2f(*p); }
__device__ __forceinline__ void stf(float* p, float v) { *p = v; }
__device__ __forceinline__ void stf(bf16_t* p, float v) { *p = f2bf(v); }

// VE consecutive elements of the embedding axis as one access (VE = 4 needs every tile extent along that
// axis to be a multiple of 4 and 16-byte aligned tiles; VE = 1 otherwise)
template <int VE> __device__ __forceinline__ void ldw(const float* p, float (&f)[VE]) { ldv<VE>(p, f); }
template <int VE> __device__ __forceinline__ void ldw(const bf16_t* p, float (&f)[VE]) {
    if constexpr (VE == 4) {
        const uint2 x = *reinterpret_cast<const uint2*>(p);
        f[0] = __uint_as_float(x.x << 16); f[1] = __uint_as_float(x.x & 0xffff0000u);
        f[2] = __uint_as_float(x.y << 16); f[3] = __uint_as_float(x.y & 0xffff0000u);
    } else {
        f[0] = bf2f(p[0]);
    }
}
template <int VE> __device__ __forceinline__ void stw(float* p, const float (&f)[VE]) { stv<VE>(p, f); }
template <int VE> __device__ __forceinline__ void stw(bf16_t* p, const float (&f)[VE]) {
    if constexpr (VE == 4) {
        uint2 x;
        x.x = (uint32_t)f2bf(f[0]) | ((uint32_t)f2bf(f[1]) << 16);
        x.y = (uint32_t)f2bf(f[2]) | ((uint32_t)f2bf(f[3]) << 16);
        *reinterpret_cast<uint2*>(p) = x;
    } else {
        p[0] = f2bf(f[0]);
    }
}

// (e, s, b) of the i-th group of VE elements, first axis fastest; 32-bit arithmetic when the count allows
// (a 64-bit division costs about a hundred instructions)
template <int VE>
__device__ __forceinline__ void group_coords(int64_t i, int64_t total, int Ne, int Ns, int (&c)[kMaxDim]) {
    const int NeV = Ne / VE;
    if (total <= 0x7fffffff) {
        const unsigned u = (unsigned)i, q = u / (unsigned)NeV, q2 = q / (unsigned)Ns;
        c[0] = (int)(u - q * (unsigned)NeV) * VE; c[1] = (int)(q - q2 * (unsigned)Ns); c[2] = (int)q2;
    } else {
        c[0] = (int)(i % NeV) * VE; c[1] = (int)((i / NeV) % Ns); c[2] = (int)(i / ((int64_t)NeV * Ns));
    }
    c[3] = 0;
}

// one thread per group of VE elements of Y, first axis fastest: coalesced along the embedding axis on both sides
template <typename TW, typename TY, int VE>
__global__ void __launch_bounds__(256) embedding_fwd_kernel(const int32_t* tokens, TiledView W, TiledView Y, int64_t total) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int Ns = Y.shape[1];
    int c[kMaxDim];
    group_coords<VE>(i, total, Y.shape[0], Ns, c);
    int tile;
    int64_t off;
    locate(Y, c, tile, off);
    const int tok = tokens[c[1] + (int64_t)Ns * c[2]];
    float v[VE];
#pragma unroll
    for (int k = 0; k < VE; k++) v[k] = 0.f;
    if (tok >= 0 && tok < W.shape[1]) {
        const int cw[kMaxDim] = {c[0], tok, 0, 0};
        int tw;
        int64_t ow;
        locate(W, cw, tw, ow);
        ldw<VE>(static_cast<const TW*>(W.tiles[tw]) + ow, v);
    }
    stw<VE>(static_cast<TY*>(Y.tiles[tile]) + off, v);
}

// one thread per group of VE elements of dY; rows of dW that several positions share are summed with hardware
// floating-point atomics (the order of those additions is not fixed)
template <typename TY, int VE>
__global__ void __launch_bounds__(256) embedding_bwd_kernel(const int32_t* tokens, TiledView dY, TiledView dW, int64_t total) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int Ns = dY.shape[1];
    int c[kMaxDim];
    group_coords<VE>(i, total, dY.shape[0], Ns, c);
    const int tok = tokens[c[1] + (int64_t)Ns * c[2]];
    if (tok < 0 || tok >= dW.shape[1]) return;
    int tile;
    int64_t off;
    locate(dY, c, tile, off);
    float g[VE];
    ldw<VE>(static_cast<const TY*>(dY.tiles[tile]) + off, g);
    const int cw[kMaxDim] = {c[0], tok, 0, 0};
    int tw;
    int64_t ow;
    locate(dW, cw, tw, ow);
    float* dst = static_cast<float*>(dW.tiles[tw]) + ow;
#pragma unroll
    for (int k = 0; k < VE; k++) unsafeAtomicAdd(dst + k, g[k]);
}

// one thread per column (s, b) of the logits X[v, s, b]: keeps the label's logit (the SoftMax
// subroutines then overwrite X with the probabilities)
template <typename T>
__global__ void __launch_bounds__(256) ce_logit_kernel(const int32_t* labels, TiledView X, float* logit, int64_t ncols) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= ncols) return;
    const int Ns = X.shape[1];
    const int lab = labels[i];
    float x = 0.f;
    if (lab >= 0 && lab < X.shape[0]) {
        const int c[kMaxDim] = {lab, (int)(i % Ns), (int)(i / Ns), 0};
        int tile;
        int64_t off;
        locate(X, c, tile, off);
        x = ldf(static_cast<const T*>(X.tiles[tile]) + off);
    }
    logit[i] = x;
}

// one thread per column (s, b) of the probabilities P[v, s, b]: loss of the column from the kept logit
// and the column's fp32 statistics, -(x - max - log(sum)) (not from the stored probability, which may
// have been rounded to bf16 or have underflowed), and P[label] -= 1
template <typename T>
__global__ void __launch_bounds__(256) ce_label_kernel(const int32_t* labels, TiledView P, TiledView S, float* losses, int64_t ncols) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= ncols) return;
    const int Ns = P.shape[1];
    const int lab = labels[i];
    float loss = 0.f;
    if (lab >= 0 && lab < P.shape[0]) {
        const int c[kMaxDim] = {lab, (int)(i % Ns), (int)(i / Ns), 0};
        int tile;
        int64_t off;
        locate(P, c, tile, off);
        T* p = static_cast<T*>(P.tiles[tile]) + off;
        const int cs[kMaxDim] = {0, c[1], c[2], 0};
        int ts;
        int64_t os;
        locate(S, cs, ts, os);
        const float* st = static_cast<const float*>(S.tiles[ts]) + os;      // (maximum, sum of shifted exponentials)
        loss = -(losses[i] - st[0] - logf(st[1]));
        stf(p, ldf(p) - 1.f);
    }
    losses[i] = loss;
}

// deterministic sum of n floats by one workgroup: fixed assignment of elements to lanes, fixed tree
__global__ void __launch_bounds__(1024) sum_kernel(const float* x, int64_t n, float* out) {
    __shared__ float part[16];
    float s = 0.f;
    for (int64_t i = threadIdx.x; i < n; i += 1024) s += x[i];
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < 16; w++) t += part[w];
        out[0] = t;
    }
}

int32_t check_act(nnt_ctx* ctx, const char* who, const nnt_tensor* Y) {
    if (Y->ndim != 3) return fail(ctx, NNT_EINVAL, std::string(who) + ": the activation must be [N_e, N_s, N_b]");
    for (void* p : Y->tiles)
        if (!p) return fail(ctx, NNT_EINVAL, std::string(who) + ": structural-zero tiles not allowed");
    return NNT_OK;
}

}  // namespace
}  // namespace nnt

using namespace nnt;

int32_t nnt_embedding_fwd(nnt_ctx* ctx, const int32_t* tokens, nnt_tensor* W, nnt_tensor* Y) {
    NNT_CHECK_CTX(ctx);
    if (!tokens || !W || !Y) return fail(ctx, NNT_EINVAL, "nnt_embedding_fwd: null argument");
    int32_t rc = check_act(ctx, "nnt_embedding_fwd", Y);
    if (rc != NNT_OK) return rc;
    if (W->ndim != 2 || W->shape[0] != Y->shape[0]) return fail(ctx, NNT_EINVAL, "nnt_embedding_fwd: W must be [N_e, N_v]");
    for (void* p : W->tiles)
        if (!p) return fail(ctx, NNT_EINVAL, "nnt_embedding_fwd: structural-zero tiles not allowed");
    // four elements of the embedding axis per thread when every tile holds whole groups of four at aligned addresses
    bool vec = W->base[0] % 4 == 0 && W->shape[0] % 4 == 0 && Y->base[0] % 4 == 0;
    for (void* p : W->tiles) vec = vec && aligned16(p);
    for (void* p : Y->tiles) vec = vec && aligned16(p);
    const int64_t total = Y->shape[0] * Y->shape[1] * Y->shape[2] / (vec ? 4 : 1);
    if ((total + 255) / 256 > INT32_MAX) return fail(ctx, NNT_EINVAL, "nnt_embedding_fwd: tensor too large");
    const TiledView vw = W->view(), vy = Y->view();
    const int dw = W->dtype, dy = Y->dtype;
    OpTag tag(ctx, "embedding_fwd", (double)Y->shape[0] * Y->shape[1] * Y->shape[2] * (W->elem_size() + Y->elem_size()), true);
    return submit(ctx, {W->all(kRead), Y->all(kWrite)}, [=](hipStream_t st) {
        const dim3 grid((unsigned)((total + 255) / 256)), block(256);
#define NNT_EMB_FWD(TW, TY)                                                                                              \
    do {                                                                                                                 \
        if (vec) hipLaunchKernelGGL((embedding_fwd_kernel<TW, TY, 4>), grid, block, 0, st, tokens, vw, vy, total);       \
        else hipLaunchKernelGGL((embedding_fwd_kernel<TW, TY, 1>), grid, block, 0, st, tokens, vw, vy, total);           \
    } while (0)
        if (dw == NNT_F32 && dy == NNT_F32) NNT_EMB_FWD(float, float);
        else if (dw == NNT_F32) NNT_EMB_FWD(float, bf16_t);
        else if (dy == NNT_F32) NNT_EMB_FWD(bf16_t, float);
        else NNT_EMB_FWD(bf16_t, bf16_t);
#undef NNT_EMB_FWD
        return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
    });
}

int32_t nnt_embedding_bwd(nnt_ctx* ctx, const int32_t* tokens, nnt_tensor* dY, nnt_tensor* dW) {
    NNT_CHECK_CTX(ctx);
    if (!tokens || !dW || !dY) return fail(ctx, NNT_EINVAL, "nnt_embedding_bwd: null argument");
    int32_t rc = check_act(ctx, "nnt_embedding_bwd", dY);
    if (rc != NNT_OK) return rc;
    if (dW->ndim != 2 || dW->shape[0] != dY->shape[0] || dW->dtype != NNT_F32)
        return fail(ctx, NNT_EINVAL, "nnt_embedding_bwd: dW must be fp32 [N_e, N_v]");
    for (void* p : dW->tiles)
        if (!p) return fail(ctx, NNT_EINVAL, "nnt_embedding_bwd: structural-zero tiles not allowed");
    // one element per thread: the atomics of a wavefront then fall on consecutive words (four elements per
    // thread made the adjoint twice as slow: every atomic instruction touched every fourth word of 1 KB)
    const int64_t total = dY->shape[0] * dY->shape[1] * dY->shape[2];
    if ((total + 255) / 256 > INT32_MAX) return fail(ctx, NNT_EINVAL, "nnt_embedding_bwd: tensor too large");
    const TiledView vw = dW->view(), vy = dY->view();
    const int dy = dY->dtype;
    OpTag tag(ctx, "embedding_bwd", (double)total * (dY->elem_size() + 8), true);
    return submit(ctx, {dY->all(kRead), dW->all(kReadWrite)}, [=](hipStream_t st) {
        const dim3 grid((unsigned)((total + 255) / 256)), block(256);
        if (dy == NNT_F32) hipLaunchKernelGGL((embedding_bwd_kernel<float, 1>), grid, block, 0, st, tokens, vy, vw, total);
        else hipLaunchKernelGGL((embedding_bwd_kernel<bf16_t, 1>), grid, block, 0, st, tokens, vy, vw, total);
        return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
    });
}

int32_t nnt_cross_entropy(nnt_ctx* ctx, nnt_tensor* X, const int32_t* labels, nnt_tensor* stats, float* losses, float* loss) {
    NNT_CHECK_CTX(ctx);
    if (!X || !labels || !stats || !losses || !loss) return fail(ctx, NNT_EINVAL, "nnt_cross_entropy: null argument");
    if (X->ndim != 3) return fail(ctx, NNT_EINVAL, "nnt_cross_entropy: the logits must be [N_v, N_s, N_b]");
    for (void* p : X->tiles)
        if (!p) return fail(ctx, NNT_EINVAL, "nnt_cross_entropy: structural-zero tiles not allowed");
    const int64_t ncols = X->shape[1] * X->shape[2];
    const TiledView vx = X->view();
    const int dt = X->dtype;
    const dim3 grid((unsigned)((ncols + 255) / 256)), block(256);
    // the label's logit of every column, kept in `losses` until the last kernel turns it into the loss
    // (ordered before the in-place softmax by its read of X, and the last kernel after it by its write)
    int32_t rc;
    {
        OpTag tag(ctx, "cross_entropy_logits", (double)ncols * (X->elem_size() + 8), true);
        rc = submit(ctx, {X->all(kRead)}, [=](hipStream_t st) {
            if (dt == NNT_F32) hipLaunchKernelGGL((ce_logit_kernel<float>), grid, block, 0, st, labels, vx, losses, ncols);
            else hipLaunchKernelGGL((ce_logit_kernel<bf16_t>), grid, block, 0, st, labels, vx, losses, ncols);
            return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
        });
        if (rc != NNT_OK) return rc;
    }
    // subroutines 1 and 2 of the softmax over the vocabulary axis, in place
    rc = nnt_softmax_fwd(ctx, X, stats, 1.f, 0);
    if (rc != NNT_OK) return rc;
    const TiledView vs = stats->view();
    OpTag tag(ctx, "cross_entropy_labels", (double)ncols * (2.0 * X->elem_size() + 20), true);
    // the label entries can sit in any vocabulary tile: the task takes the whole tensor
    return submit(ctx, {X->all(kReadWrite), stats->all(kRead)}, [=](hipStream_t st) {
        if (dt == NNT_F32) hipLaunchKernelGGL((ce_label_kernel<float>), grid, block, 0, st, labels, vx, vs, losses, ncols);
        else hipLaunchKernelGGL((ce_label_kernel<bf16_t>), grid, block, 0, st, labels, vx, vs, losses, ncols);
        if (hipGetLastError() != hipSuccess) return (int32_t)NNT_EHIP;
        hipLaunchKernelGGL(sum_kernel, dim3(1), dim3(1024), 0, st, losses, ncols, loss);
        return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
    }, 2);
}
