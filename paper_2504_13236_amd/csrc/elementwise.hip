// Memory-bound elementwise tile kernels (section 3: activations apply directly to
// every tile; the optimizer update is a per-element weighted sum; the bias is
// added over the unchanged dimensions) and their tensor-level forms.
//
// One kernel template serves both forms.  In the tile form the operands are plain
// pointers; in the tensor form each operand is a table of tile pointers and
// blockIdx.y selects the tile, so a whole tiled tensor is handled by one launch.
// Every thread moves 16-byte vectors (4 fp32 or 8 bf16) when the tile extents and
// pointers allow it, single elements otherwise.
#include "device_util.hpp"
#include "ew_functors.hpp"
#include "internal.hpp"

#include <type_traits>

#include <algorithm>
#include <cmath>

namespace nnt {
namespace {

// ------------------------------------------------------------------ strided block copy
template <typename T>
__global__ void __launch_bounds__(256) copy_block_kernel(const T* src, T* dst, int e0, int e1, int e2, int e3,
                                                         int64_t s0, int64_t s1, int64_t s2, int64_t s3,
                                                         int64_t d0, int64_t d1, int64_t d2, int64_t d3) {
    const int64_t total = (int64_t)e0 * e1 * e2 * e3;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        int64_t r = i;
        const int i0 = (int)(r % e0); r /= e0;
        const int i1 = (int)(r % e1); r /= e1;
        const int i2 = (int)(r % e2); r /= e2;
        const int i3 = (int)r;
        dst[i0 * d0 + i1 * d1 + i2 * d2 + i3 * d3] = src[i0 * s0 + i1 * s1 + i2 * s2 + i3 * s3];
    }
}

// ------------------------------------------------------------------ head split / merge over tiled views
struct HeadArgs {
    TiledView z;
    TiledView part[3];
    int32_t n_parts, N_h, h, to_parts;
};

// A thread owns one vector of V rows of Z and copies it for kHeadTok consecutive tokens (s, b): the
// decomposition of its row into (part, head, component) and tiles costs integer divisions once, the
// token's share of the addresses is the same for the whole workgroup (scalar arithmetic), and
// the copies of a thread are independent loads in flight together.  Along the rows both sides are
// contiguous (whole rows of Z, runs of h elements of a part).
constexpr int kHeadTok = 8;

template <typename T, int V>
__global__ void __launch_bounds__(256) head_kernel(HeadArgs a) {
    const int rows = a.z.shape[0], N_s = a.z.shape[1], N_b = a.z.shape[2];
    const int r = (blockIdx.x * blockDim.x + threadIdx.x) * V;
    if (r >= rows) return;
    const int head = r / a.h, i = r - head * a.h;
    const int p = head / a.N_h, j = head - p * a.N_h;
    const TiledView& pv = a.part[p];
    // row part of the Z address: tile coordinate, position and pitch along axis 0
    const int zt0 = r / a.z.base[0], zr = r - zt0 * a.z.base[0];
    const int zext0 = min(a.z.base[0], rows - zt0 * a.z.base[0]);
    // row part of the part's address: axis 0 (component i) and axis 3 (head j)
    const int pt0 = i / pv.base[0], pi = i - pt0 * pv.base[0];
    const int pext0 = min(pv.base[0], a.h - pt0 * pv.base[0]);
    const int ptj = j / pv.base[3], pj = j - ptj * pv.base[3];
    const int ntok = N_s * N_b;
    const int tok0 = blockIdx.y * kHeadTok;
    using Vec = std::conditional_t<V * sizeof(T) == 16, uint4, T>;
    Vec val[kHeadTok];
    T* src[kHeadTok];
    T* dst[kHeadTok];
#pragma unroll
    for (int t = 0; t < kHeadTok; t++) {
        const int tok = min(tok0 + t, ntok - 1);           // the tail repeats the last token (same value twice)
        const int b = tok / N_s, s = tok - b * N_s;
        // all parts are tiled alike, so part 0 stands for their sequence and batch tiling
        const TiledView& q = a.part[0];
        const int zs = s / a.z.base[1], zls = zs * a.z.base[1], zes = min(a.z.base[1], N_s - zls);
        const int zb = b / a.z.base[2], zlb = zb * a.z.base[2];
        const int qs = s / q.base[1], qls = qs * q.base[1], qes = min(q.base[1], N_s - qls);
        const int qb = b / q.base[2], qlb = qb * q.base[2], qeb = min(q.base[2], N_b - qlb);
        const int ztile = zt0 + a.z.grid[0] * (zs + a.z.grid[1] * zb);
        const int64_t zoff = zr + (int64_t)zext0 * ((s - zls) + zes * (b - zlb));
        const int ptile = pt0 + q.grid[0] * (qs + q.grid[1] * (qb + q.grid[2] * ptj));
        const int64_t poff = pi + (int64_t)pext0 * ((s - qls) + (int64_t)qes * ((b - qlb) + qeb * pj));
        T* zp = static_cast<T*>(a.z.tiles[ztile]) + zoff;
        T* pp = static_cast<T*>(pv.tiles[ptile]) + poff;
        src[t] = a.to_parts ? zp : pp;
        dst[t] = a.to_parts ? pp : zp;
    }
#pragma unroll
    for (int t = 0; t < kHeadTok; t++) val[t] = *reinterpret_cast<const Vec*>(src[t]);
#pragma unroll
    for (int t = 0; t < kHeadTok; t++) *reinterpret_cast<Vec*>(dst[t]) = val[t];
}

bool all_aligned(const nnt_tensor* t) {
    for (void* p : t->tiles)
        if (p && !aligned16(p)) return false;
    return true;
}
// every tile extent along axis 0 is a multiple of v
bool axis0_multiple(const nnt_tensor* t, int v) { return t->base[0] % v == 0 && t->shape[0] % v == 0; }
int64_t max_tile_numel(const nnt_tensor* t) {
    int64_t n = 1;
    for (int a = 0; a < t->ndim; a++) n *= t->base[a];
    return n;
}
EwGeom tiled_geom(const nnt_tensor* t) {
    EwGeom g;
    g.v = t->view();
    g.n_single = 0;
    g.numel = nullptr;
    g.tiled = 1;
    return g;
}
EwGeom single_geom(int64_t n) {
    EwGeom g = {};
    g.n_single = n;
    g.tiled = 0;
    return g;
}
Operand tab(const nnt_tensor* t) { return Operand{t ? t->d_tiles : nullptr, nullptr}; }
Operand tab1(const nnt_tensor* t, int64_t tile) { return Operand{nullptr, t ? t->tiles[tile] : nullptr}; }
Operand ptr(const void* p) { return Operand{nullptr, const_cast<void*>(p)}; }

// Runs functor maker `mk(single_tile_index or -1)` either once over all tiles or tile by tile.
template <typename MakeF>
int32_t run_tensor_ew(nnt_ctx* ctx, nnt_tensor* ref, const std::vector<std::pair<nnt_tensor*, int>>& operands,
                      bool vec, MakeF mk) {
    if (ref->ntiles > 65535) return fail(ctx, NNT_EINVAL, "too many tiles for one launch");
    if (ctx->granularity == NNT_GRAN_OP) {
        std::vector<Access> acc;
        for (auto& o : operands) acc.push_back(o.first->all(o.second));
        auto f = mk((int64_t)-1);
        const EwGeom g = tiled_geom(ref);
        const int64_t mx = max_tile_numel(ref), nt = ref->ntiles;
        return submit(ctx, acc, [=](hipStream_t st) { return launch_ew(st, f, g, mx, nt, vec); });
    }
    for (int64_t t = 0; t < ref->ntiles; t++) {
        if (!ref->tiles[t]) continue;
        std::vector<Access> acc;
        for (auto& o : operands) acc.push_back(o.first->one(o.first->ntiles == ref->ntiles ? t : 0, o.second));
        auto f = mk(t);
        const int64_t n = ref->tile_numel(t);
        const EwGeom g = single_geom(n);
        int32_t rc = submit(ctx, acc, [=](hipStream_t st) { return launch_ew(st, f, g, n, 1, vec); });
        if (rc != NNT_OK) return rc;
    }
    return NNT_OK;
}

Operand opnd(const nnt_tensor* t, int64_t tile) { return tile < 0 ? tab(t) : tab1(t, tile); }

// elements held in the tiles that exist
double present_numel(const nnt_tensor* t) {
    double n = 0;
    for (int64_t i = 0; i < t->ntiles; i++)
        if (t->tiles[i]) n += (double)t->tile_numel(i);
    return n;
}

}  // namespace
}  // namespace nnt

using namespace nnt;

#define DT_OK(d) ((d) == NNT_F32 || (d) == NNT_BF16)

extern "C" {

// ------------------------------------------------------------------ tile form
int32_t nnt_tile_fill(void* stream, int32_t dtype, int64_t n, float value, void* x) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (n < 0 || (n > 0 && !x)) return NNT_EINVAL;
    const bool vec = aligned16(x);
    if (dtype == NNT_F32) return launch_ew((hipStream_t)stream, FillF<float>{ptr(x), value}, single_geom(n), n, 1, vec);
    return launch_ew((hipStream_t)stream, FillF<bf16_t>{ptr(x), value}, single_geom(n), n, 1, vec);
}

int32_t nnt_tile_add(void* stream, int32_t dtype, int64_t n, float alpha, const void* x, float beta, void* y) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (n < 0 || (n > 0 && (!x || !y))) return NNT_EINVAL;
    const bool vec = aligned16(x) && aligned16(y);
    if (dtype == NNT_F32) return launch_ew((hipStream_t)stream, AddF<float>{ptr(x), ptr(y), alpha, beta}, single_geom(n), n, 1, vec);
    return launch_ew((hipStream_t)stream, AddF<bf16_t>{ptr(x), ptr(y), alpha, beta}, single_geom(n), n, 1, vec);
}

int32_t nnt_tile_cast(void* stream, int32_t dtype_in, int32_t dtype_out, int64_t n, const void* x, void* y) {
    if (!DT_OK(dtype_in) || !DT_OK(dtype_out)) return NNT_EDTYPE;
    if (n < 0 || (n > 0 && (!x || !y))) return NNT_EINVAL;
    const bool vec = aligned16(x) && aligned16(y);
    hipStream_t st = (hipStream_t)stream;
    const EwGeom g = single_geom(n);
    if (dtype_in == NNT_F32 && dtype_out == NNT_BF16) return launch_ew(st, CastF<float, bf16_t>{ptr(x), ptr(y)}, g, n, 1, vec);
    if (dtype_in == NNT_BF16 && dtype_out == NNT_F32) return launch_ew(st, CastF<bf16_t, float>{ptr(x), ptr(y)}, g, n, 1, vec);
    if (dtype_in == NNT_F32) return launch_ew(st, CastF<float, float>{ptr(x), ptr(y)}, g, n, 1, vec);
    return launch_ew(st, CastF<bf16_t, bf16_t>{ptr(x), ptr(y)}, g, n, 1, vec);
}

int32_t nnt_tile_copy_block(void* stream, int32_t dtype, int32_t ndim, const int64_t* extent,
                            const void* src, const int64_t* ss, void* dst, const int64_t* ds) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (ndim < 1 || ndim > kMaxDim || !extent || !ss || !ds || !src || !dst) return NNT_EINVAL;
    int64_t e[4] = {1, 1, 1, 1}, s[4] = {0, 0, 0, 0}, d[4] = {0, 0, 0, 0}, total = 1;
    for (int a = 0; a < ndim; a++) {
        if (extent[a] < 0 || extent[a] > INT32_MAX) return NNT_EINVAL;
        e[a] = extent[a]; s[a] = ss[a]; d[a] = ds[a];
        total *= e[a];
    }
    if (total == 0) return NNT_OK;
    const unsigned blocks = (unsigned)std::min<int64_t>((total + 255) / 256, 1 << 16);
    hipStream_t st = (hipStream_t)stream;
    if (dtype == NNT_F32)
        hipLaunchKernelGGL((copy_block_kernel<float>), dim3(blocks), dim3(256), 0, st, (const float*)src, (float*)dst,
                           (int)e[0], (int)e[1], (int)e[2], (int)e[3], s[0], s[1], s[2], s[3], d[0], d[1], d[2], d[3]);
    else
        hipLaunchKernelGGL((copy_block_kernel<bf16_t>), dim3(blocks), dim3(256), 0, st, (const bf16_t*)src, (bf16_t*)dst,
                           (int)e[0], (int)e[1], (int)e[2], (int)e[3], s[0], s[1], s[2], s[3], d[0], d[1], d[2], d[3]);
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int32_t nnt_tile_bias_add(void* stream, int32_t dtype, int64_t m, int64_t n, const float* bias, void* Y) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (m < 0 || n < 0 || m > INT32_MAX || (m * n > 0 && (!bias || !Y))) return NNT_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const EwGeom g = single_geom(m * n);
    if (dtype == NNT_F32)
        return launch_ew(st, BiasAddF<float>{ptr(Y), ptr(bias), m}, g, m * n, 1, aligned16(Y) && aligned16(bias) && m % 4 == 0);
    return launch_ew(st, BiasAddF<bf16_t>{ptr(Y), ptr(bias), m}, g, m * n, 1, aligned16(Y) && aligned16(bias) && m % 8 == 0);
}

int32_t nnt_tile_gelu(void* stream, int32_t dtype, int32_t variant, int64_t n, const void* x, void* y) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if ((variant != NNT_GELU_TANH && variant != NNT_GELU_ERF) || n < 0 || (n > 0 && (!x || !y))) return NNT_EINVAL;
    const bool vec = aligned16(x) && aligned16(y);
    if (dtype == NNT_F32) return launch_ew((hipStream_t)stream, GeluF<float>{ptr(x), ptr(y), variant}, single_geom(n), n, 1, vec);
    return launch_ew((hipStream_t)stream, GeluF<bf16_t>{ptr(x), ptr(y), variant}, single_geom(n), n, 1, vec);
}

int32_t nnt_tile_gelu_bwd(void* stream, int32_t dtype, int32_t variant, int64_t n, const void* x, const void* dy, void* dx) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if ((variant != NNT_GELU_TANH && variant != NNT_GELU_ERF) || n < 0 || (n > 0 && (!x || !dy || !dx))) return NNT_EINVAL;
    const bool vec = aligned16(x) && aligned16(dy) && aligned16(dx);
    if (dtype == NNT_F32)
        return launch_ew((hipStream_t)stream, GeluBwdF<float>{ptr(x), ptr(dy), ptr(dx), variant}, single_geom(n), n, 1, vec);
    return launch_ew((hipStream_t)stream, GeluBwdF<bf16_t>{ptr(x), ptr(dy), ptr(dx), variant}, single_geom(n), n, 1, vec);
}

// State larger than this is streamed past the caches (four times the 256 MB last-level cache).
constexpr double kAdamStreamBytes = 1024.0 * 1024.0 * 1024.0;

static AdamF make_adam(int32_t step, double lr, double b1, double b2, double eps, double wd, double bytes) {
    AdamF f = {};
    f.stream = bytes > kAdamStreamBytes ? 1 : 0;
    f.lr = (float)lr; f.beta1 = (float)b1; f.beta2 = (float)b2; f.eps = (float)eps; f.wd = (float)wd;
    f.omb1 = (float)(1.0 - b1); f.omb2 = (float)(1.0 - b2);
    f.inv_bc1 = (float)(1.0 / (1.0 - std::pow((double)b1, (double)step)));
    f.inv_bc2 = (float)(1.0 / (1.0 - std::pow((double)b2, (double)step)));
    return f;
}

int32_t nnt_tile_adam(void* stream, int64_t n, int32_t step, double lr, double beta1, double beta2, double eps,
                      double weight_decay, const float* g, float* p, float* m, float* v, void* p_lowp) {
    if (n < 0 || step < 1 || (n > 0 && (!g || !p || !m || !v))) return NNT_EINVAL;
    AdamF f = make_adam(step, lr, beta1, beta2, eps, weight_decay, 30.0 * (double)n);
    f.g = ptr(g); f.p = ptr(p); f.m = ptr(m); f.v = ptr(v); f.lp = ptr(p_lowp);
    const bool vec = aligned16(g) && aligned16(p) && aligned16(m) && aligned16(v) && (!p_lowp || ((uintptr_t)p_lowp & 7) == 0);
    return launch_ew((hipStream_t)stream, f, single_geom(n), n, 1, vec);
}

int32_t nnt_tile_sgd(void* stream, int64_t n, double lr, double momentum, double weight_decay, int32_t nesterov,
                     const float* g, float* p, float* v, void* p_lowp) {
    if (n < 0 || momentum < 0.0 || (n > 0 && (!g || !p || !v))) return NNT_EINVAL;
    SgdF f = {};
    f.lr = (float)lr; f.mu = (float)momentum; f.wd = (float)weight_decay; f.nesterov = nesterov ? 1 : 0;
    f.g = ptr(g); f.p = ptr(p); f.v = ptr(v); f.lp = ptr(p_lowp);
    const bool vec = aligned16(g) && aligned16(p) && aligned16(v) && (!p_lowp || ((uintptr_t)p_lowp & 7) == 0);
    return launch_ew((hipStream_t)stream, f, single_geom(n), n, 1, vec);
}

// ------------------------------------------------------------------ tensor form
int32_t nnt_fill(nnt_ctx* ctx, float value, nnt_tensor* X) {
    NNT_CHECK_CTX(ctx);
    if (!X) return fail(ctx, NNT_EINVAL, "nnt_fill: null tensor");
    OpTag tag(ctx, "fill", present_numel(X) * X->elem_size(), true);
    const bool vec = all_aligned(X);
    if (X->dtype == NNT_F32)
        return run_tensor_ew(ctx, X, {{X, kWrite}}, vec, [=](int64_t t) { return FillF<float>{opnd(X, t), value}; });
    return run_tensor_ew(ctx, X, {{X, kWrite}}, vec, [=](int64_t t) { return FillF<bf16_t>{opnd(X, t), value}; });
}

int32_t nnt_add(nnt_ctx* ctx, float alpha, nnt_tensor* X, float beta, nnt_tensor* Y) {
    NNT_CHECK_CTX(ctx);
    if (!X || !Y) return fail(ctx, NNT_EINVAL, "nnt_add: null tensor");
    if (!same_tiling(X, Y) || !null_alike(X, Y)) return fail(ctx, NNT_EINVAL, "nnt_add: operands tiled differently");
    if (X->dtype != Y->dtype) return fail(ctx, NNT_EDTYPE, "nnt_add: operand types differ");
    const bool vec = all_aligned(X) && all_aligned(Y);
    OpTag tag(ctx, "add", present_numel(Y) * Y->elem_size() * (beta != 0.f ? 3 : 2), true);
    const int ymode = beta != 0.f ? kReadWrite : kWrite;
    if (X->dtype == NNT_F32)
        return run_tensor_ew(ctx, Y, {{X, kRead}, {Y, ymode}}, vec,
                             [=](int64_t t) { return AddF<float>{opnd(X, t), opnd(Y, t), alpha, beta}; });
    return run_tensor_ew(ctx, Y, {{X, kRead}, {Y, ymode}}, vec,
                         [=](int64_t t) { return AddF<bf16_t>{opnd(X, t), opnd(Y, t), alpha, beta}; });
}

int32_t nnt_cast(nnt_ctx* ctx, nnt_tensor* X, nnt_tensor* Y) {
    NNT_CHECK_CTX(ctx);
    if (!X || !Y) return fail(ctx, NNT_EINVAL, "nnt_cast: null tensor");
    if (!same_tiling(X, Y) || !null_alike(X, Y)) return fail(ctx, NNT_EINVAL, "nnt_cast: operands tiled differently");
    OpTag tag(ctx, "cast", present_numel(Y) * (X->elem_size() + Y->elem_size()), true);
    const bool vec = all_aligned(X) && all_aligned(Y);
    std::vector<std::pair<nnt_tensor*, int>> ops = {{X, kRead}, {Y, kWrite}};
    if (X->dtype == NNT_F32 && Y->dtype == NNT_BF16)
        return run_tensor_ew(ctx, Y, ops, vec, [=](int64_t t) { return CastF<float, bf16_t>{opnd(X, t), opnd(Y, t)}; });
    if (X->dtype == NNT_BF16 && Y->dtype == NNT_F32)
        return run_tensor_ew(ctx, Y, ops, vec, [=](int64_t t) { return CastF<bf16_t, float>{opnd(X, t), opnd(Y, t)}; });
    if (X->dtype == NNT_F32)
        return run_tensor_ew(ctx, Y, ops, vec, [=](int64_t t) { return CastF<float, float>{opnd(X, t), opnd(Y, t)}; });
    return run_tensor_ew(ctx, Y, ops, vec, [=](int64_t t) { return CastF<bf16_t, bf16_t>{opnd(X, t), opnd(Y, t)}; });
}

int32_t nnt_gelu(nnt_ctx* ctx, int32_t variant, nnt_tensor* X, nnt_tensor* Y) {
    NNT_CHECK_CTX(ctx);
    if (!X || !Y) return fail(ctx, NNT_EINVAL, "nnt_gelu: null tensor");
    if (variant != NNT_GELU_TANH && variant != NNT_GELU_ERF) return fail(ctx, NNT_EINVAL, "nnt_gelu: unknown variant");
    if (!same_tiling(X, Y) || !null_alike(X, Y)) return fail(ctx, NNT_EINVAL, "nnt_gelu: operands tiled differently");
    if (X->dtype != Y->dtype) return fail(ctx, NNT_EDTYPE, "nnt_gelu: operand types differ");
    OpTag tag(ctx, "gelu", present_numel(Y) * Y->elem_size() * 2, true);
    const bool vec = all_aligned(X) && all_aligned(Y);
    std::vector<std::pair<nnt_tensor*, int>> ops = {{X, kRead}, {Y, kWrite}};
    if (X->dtype == NNT_F32)
        return run_tensor_ew(ctx, Y, ops, vec, [=](int64_t t) { return GeluF<float>{opnd(X, t), opnd(Y, t), variant}; });
    return run_tensor_ew(ctx, Y, ops, vec, [=](int64_t t) { return GeluF<bf16_t>{opnd(X, t), opnd(Y, t), variant}; });
}

int32_t nnt_gelu_bwd(nnt_ctx* ctx, int32_t variant, nnt_tensor* X, nnt_tensor* dY, nnt_tensor* dX) {
    NNT_CHECK_CTX(ctx);
    if (!X || !dY || !dX) return fail(ctx, NNT_EINVAL, "nnt_gelu_bwd: null tensor");
    if (variant != NNT_GELU_TANH && variant != NNT_GELU_ERF) return fail(ctx, NNT_EINVAL, "nnt_gelu_bwd: unknown variant");
    if (!same_tiling(X, dY) || !same_tiling(X, dX) || !null_alike(X, dY) || !null_alike(X, dX))
        return fail(ctx, NNT_EINVAL, "nnt_gelu_bwd: operands tiled differently");
    if (X->dtype != dY->dtype || X->dtype != dX->dtype) return fail(ctx, NNT_EDTYPE, "nnt_gelu_bwd: operand types differ");
    const bool vec = all_aligned(X) && all_aligned(dY) && all_aligned(dX);
    OpTag tag(ctx, "gelu_bwd", present_numel(dX) * dX->elem_size() * 3, true);
    std::vector<std::pair<nnt_tensor*, int>> ops = {{X, kRead}, {dY, kRead}, {dX, dX == dY ? kReadWrite : kWrite}};
    if (dX == dY) ops.erase(ops.begin() + 1);
    if (X->dtype == NNT_F32)
        return run_tensor_ew(ctx, dX, ops, vec,
                             [=](int64_t t) { return GeluBwdF<float>{opnd(X, t), opnd(dY, t), opnd(dX, t), variant}; });
    return run_tensor_ew(ctx, dX, ops, vec,
                         [=](int64_t t) { return GeluBwdF<bf16_t>{opnd(X, t), opnd(dY, t), opnd(dX, t), variant}; });
}

int32_t nnt_bias_add(nnt_ctx* ctx, nnt_tensor* b, nnt_tensor* Y) {
    NNT_CHECK_CTX(ctx);
    if (!b || !Y) return fail(ctx, NNT_EINVAL, "nnt_bias_add: null tensor");
    if (b->dtype != NNT_F32 || b->ndim != 1 || b->shape[0] != Y->shape[0] || b->base[0] != Y->base[0])
        return fail(ctx, NNT_EINVAL, "nnt_bias_add: bias must be an fp32 vector tiled like Y's first axis");
    for (void* p : b->tiles)
        if (!p) return fail(ctx, NNT_EINVAL, "nnt_bias_add: bias tile missing");
    const int V = Y->dtype == NNT_F32 ? 4 : 8;
    const bool vec = all_aligned(Y) && axis0_multiple(Y, V);
    OpTag tag(ctx, "bias_add", present_numel(Y) * Y->elem_size() * 2, true);
    if (Y->ntiles > 65535) return fail(ctx, NNT_EINVAL, "too many tiles for one launch");
    if (ctx->granularity == NNT_GRAN_OP) {
        const EwGeom g = tiled_geom(Y);
        const int64_t mx = max_tile_numel(Y), nt = Y->ntiles;
        std::vector<Access> acc = {b->all(kRead), Y->all(kReadWrite)};
        if (Y->dtype == NNT_F32) {
            BiasAddF<float> f{tab(Y), tab(b), 0};
            return submit(ctx, acc, [=](hipStream_t st) { return launch_ew(st, f, g, mx, nt, vec); });
        }
        BiasAddF<bf16_t> f{tab(Y), tab(b), 0};
        return submit(ctx, acc, [=](hipStream_t st) { return launch_ew(st, f, g, mx, nt, vec); });
    }
    for (int64_t t = 0; t < Y->ntiles; t++) {
        if (!Y->tiles[t]) continue;
        const int64_t c0 = t % Y->grid[0];
        const int64_t m = Y->tile_extent(0, c0), n = Y->tile_numel(t) / m;
        void* yp = Y->tiles[t];
        const float* bp = static_cast<const float*>(b->tiles[c0]);
        const int32_t dt = Y->dtype;
        int32_t rc = submit(ctx, {b->one(c0, kRead), Y->one(t, kReadWrite)},
                            [=](hipStream_t st) { return nnt_tile_bias_add(st, dt, m, n, bp, yp); });
        if (rc != NNT_OK) return rc;
    }
    return NNT_OK;
}

int32_t nnt_adam_step(nnt_ctx* ctx, const nnt_adam_cfg* cfg, int32_t step, nnt_tensor* G, nnt_tensor* P,
                      nnt_tensor* M, nnt_tensor* V, nnt_tensor* LP) {
    NNT_CHECK_CTX(ctx);
    if (!cfg || !G || !P || !M || !V || step < 1) return fail(ctx, NNT_EINVAL, "nnt_adam_step: bad argument");
    if (!same_tiling(G, P) || !same_tiling(G, M) || !same_tiling(G, V) || (LP && !same_tiling(G, LP)))
        return fail(ctx, NNT_EINVAL, "nnt_adam_step: operands tiled differently");
    if (G->dtype != NNT_F32 || P->dtype != NNT_F32 || M->dtype != NNT_F32 || V->dtype != NNT_F32 || (LP && LP->dtype != NNT_BF16))
        return fail(ctx, NNT_EDTYPE, "nnt_adam_step: g, p, m, v must be fp32 and the low-precision copy bf16");
    const bool vec = all_aligned(G) && all_aligned(P) && all_aligned(M) && all_aligned(V) && (!LP || all_aligned(LP));
    OpTag tag(ctx, "adam", present_numel(P) * (28 + (LP ? 2 : 0)), true);
    AdamF base = make_adam(step, cfg->lr, cfg->beta1, cfg->beta2, cfg->eps, cfg->weight_decay, present_numel(P) * 30.0);
    std::vector<std::pair<nnt_tensor*, int>> ops = {{G, kRead}, {P, kReadWrite}, {M, kReadWrite}, {V, kReadWrite}};
    if (LP) ops.push_back({LP, kWrite});
    return run_tensor_ew(ctx, P, ops, vec, [=](int64_t t) {
        AdamF f = base;
        f.g = opnd(G, t); f.p = opnd(P, t); f.m = opnd(M, t); f.v = opnd(V, t);
        f.lp = LP ? opnd(LP, t) : Operand{nullptr, nullptr};
        return f;
    });
}

}  // extern "C"

// ------------------------------------------------------------------ Adam on a group of parameters in one launch
// The twelve parameters of a block are nine small vectors and four matrices: as twelve launches the
// step costs more in launch latency than in memory traffic.  A group keeps, in device memory, the
// tile-pointer tables of all its tensors back to back and the element count of every tile, and the
// elementwise kernel runs over that union (blockIdx.y = entry).
namespace nnt {

struct AdamGroup {
    std::vector<nnt_tensor*> G, P, M, V, LP;     // LP entries may be null
    void** tabs = nullptr;                        // 5 tables of `entries` pointers each: g, p, m, v, low-precision copy
    int64_t* numel = nullptr;
    int64_t entries = 0, max_numel = 0;
    bool vec = true;
    double bytes = 0.0;
    nnt_ctx* ctx = nullptr;
    int64_t table_bytes = 0;
};

void adam_group_destroy(AdamGroup* a) {
    if (!a) return;
    if (a->ctx) a->ctx->table_bytes -= a->table_bytes;
    if (a->tabs) (void)hipFree(a->tabs);
    if (a->numel) (void)hipFree(a->numel);
    delete a;
}

int32_t adam_group_create(nnt_ctx* ctx, int n, nnt_tensor* const* G, nnt_tensor* const* P, nnt_tensor* const* M,
                          nnt_tensor* const* V, nnt_tensor* const* LP, AdamGroup** out) {
    *out = nullptr;
    std::unique_ptr<AdamGroup, void (*)(AdamGroup*)> a(new AdamGroup(), adam_group_destroy);
    std::vector<void*> tg, tp, tm, tv, tl;
    std::vector<int64_t> ne;
    for (int i = 0; i < n; i++) {
        nnt_tensor *g = G[i], *p = P[i], *m = M[i], *v = V[i], *lp = LP ? LP[i] : nullptr;
        if (!g || !p || !m || !v) return fail(ctx, NNT_EINVAL, "adam group: null tensor");
        if (!same_tiling(g, p) || !same_tiling(g, m) || !same_tiling(g, v) || (lp && !same_tiling(g, lp)))
            return fail(ctx, NNT_EINVAL, "adam group: operands tiled differently");
        if (g->dtype != NNT_F32 || p->dtype != NNT_F32 || m->dtype != NNT_F32 || v->dtype != NNT_F32 || (lp && lp->dtype != NNT_BF16))
            return fail(ctx, NNT_EDTYPE, "adam group: g, p, m, v must be fp32 and the low-precision copy bf16");
        a->vec = a->vec && all_aligned(g) && all_aligned(p) && all_aligned(m) && all_aligned(v) && (!lp || all_aligned(lp));
        a->bytes += present_numel(p) * (28 + (lp ? 2 : 0));
        for (int64_t t = 0; t < p->ntiles; t++) {
            if (!p->tiles[t]) continue;
            if (!g->tiles[t] || !m->tiles[t] || !v->tiles[t] || (lp && !lp->tiles[t])) return fail(ctx, NNT_EINVAL, "adam group: missing tile");
            tg.push_back(g->tiles[t]); tp.push_back(p->tiles[t]); tm.push_back(m->tiles[t]); tv.push_back(v->tiles[t]);
            tl.push_back(lp ? lp->tiles[t] : nullptr);
            ne.push_back(p->tile_numel(t));
            a->max_numel = std::max(a->max_numel, p->tile_numel(t));
        }
        a->G.push_back(g); a->P.push_back(p); a->M.push_back(m); a->V.push_back(v); a->LP.push_back(lp);
    }
    a->entries = (int64_t)ne.size();
    if (a->entries == 0 || a->entries > 65535) return fail(ctx, NNT_EINVAL, "adam group: no tiles, or too many for one launch");
    const size_t E = (size_t)a->entries;
    std::vector<void*> all;
    for (auto* t : {&tg, &tp, &tm, &tv, &tl}) all.insert(all.end(), t->begin(), t->end());
    NNT_HIP(ctx, hipMalloc(&a->tabs, 5 * E * sizeof(void*)));
    NNT_HIP(ctx, hipMalloc(&a->numel, E * sizeof(int64_t)));
    NNT_HIP(ctx, hipMemcpy(a->tabs, all.data(), 5 * E * sizeof(void*), hipMemcpyHostToDevice));
    NNT_HIP(ctx, hipMemcpy(a->numel, ne.data(), E * sizeof(int64_t), hipMemcpyHostToDevice));
    a->ctx = ctx;
    a->table_bytes = (int64_t)(5 * E * sizeof(void*) + E * sizeof(int64_t));
    ctx->table_bytes += a->table_bytes;
    *out = a.release();
    return NNT_OK;
}

// One Adam step on every tensor of the group: one task, one launch (whole-operation granularity).
int32_t adam_group_step(nnt_ctx* ctx, AdamGroup* a, const nnt_adam_cfg* cfg, int32_t step) {
    OpTag tag(ctx, "adam", a->bytes, true);
    AdamF f = make_adam(step, cfg->lr, cfg->beta1, cfg->beta2, cfg->eps, cfg->weight_decay, (double)a->bytes);
    const size_t E = (size_t)a->entries;
    f.g = Operand{a->tabs, nullptr}; f.p = Operand{a->tabs + E, nullptr}; f.m = Operand{a->tabs + 2 * E, nullptr};
    f.v = Operand{a->tabs + 3 * E, nullptr}; f.lp = Operand{a->tabs + 4 * E, nullptr};
    EwGeom g = single_geom(0);
    g.numel = a->numel;
    std::vector<Access> acc;
    for (size_t i = 0; i < a->P.size(); i++) {
        acc.push_back(a->P[i]->all(kReadWrite));
        acc.push_back(a->G[i]->all(kRead));
        acc.push_back(a->M[i]->all(kReadWrite));
        acc.push_back(a->V[i]->all(kReadWrite));
        if (a->LP[i]) acc.push_back(a->LP[i]->all(kWrite));
    }
    const int64_t mx = a->max_numel, nt = a->entries;
    const bool vec = a->vec;
    return submit(ctx, acc, [=](hipStream_t st) { return launch_ew(st, f, g, mx, nt, vec); });
}

}  // namespace nnt

extern "C" {

int32_t nnt_sgd_step(nnt_ctx* ctx, const nnt_sgd_cfg* cfg, nnt_tensor* G, nnt_tensor* P, nnt_tensor* V, nnt_tensor* LP) {
    NNT_CHECK_CTX(ctx);
    if (!cfg || !G || !P || !V || cfg->momentum < 0.0) return fail(ctx, NNT_EINVAL, "nnt_sgd_step: bad argument");
    if (!same_tiling(G, P) || !same_tiling(G, V) || (LP && !same_tiling(G, LP)))
        return fail(ctx, NNT_EINVAL, "nnt_sgd_step: operands tiled differently");
    if (G->dtype != NNT_F32 || P->dtype != NNT_F32 || V->dtype != NNT_F32 || (LP && LP->dtype != NNT_BF16))
        return fail(ctx, NNT_EDTYPE, "nnt_sgd_step: g, p, v must be fp32 and the low-precision copy bf16");
    const bool vec = all_aligned(G) && all_aligned(P) && all_aligned(V) && (!LP || all_aligned(LP));
    OpTag tag(ctx, "sgd", present_numel(P) * (20 + (LP ? 2 : 0)), true);
    SgdF base = {};
    base.lr = (float)cfg->lr; base.mu = (float)cfg->momentum; base.wd = (float)cfg->weight_decay; base.nesterov = cfg->nesterov ? 1 : 0;
    std::vector<std::pair<nnt_tensor*, int>> ops = {{G, kRead}, {P, kReadWrite}, {V, kReadWrite}};
    if (LP) ops.push_back({LP, kWrite});
    return run_tensor_ew(ctx, P, ops, vec, [=](int64_t t) {
        SgdF f = base;
        f.g = opnd(G, t); f.p = opnd(P, t); f.v = opnd(V, t);
        f.lp = LP ? opnd(LP, t) : Operand{nullptr, nullptr};
        return f;
    });
}

// ------------------------------------------------------------------ head split / merge
static int32_t head_common(nnt_ctx* ctx, nnt_tensor* Z, int32_t n_parts, nnt_tensor* const* parts, int to_parts) {
    NNT_CHECK_CTX(ctx);
    if (!Z || !parts || n_parts < 1 || n_parts > 3) return fail(ctx, NNT_EINVAL, "head split/merge: bad argument");
    if (Z->ndim != 3) return fail(ctx, NNT_EINVAL, "head split/merge: Z must have 3 axes");
    for (int p = 0; p < n_parts; p++) {
        const nnt_tensor* q = parts[p];
        if (!q || q->ndim != 4 || q->dtype != Z->dtype || !same_tiling(q, parts[0]))
            return fail(ctx, NNT_EINVAL, "head split/merge: parts must be 4-axis tensors of Z's type, tiled alike");
        for (void* t : q->tiles)
            if (!t) return fail(ctx, NNT_EINVAL, "head split/merge: structural-zero tiles not allowed");
    }
    for (void* t : Z->tiles)
        if (!t) return fail(ctx, NNT_EINVAL, "head split/merge: structural-zero tiles not allowed");
    const nnt_tensor* q0 = parts[0];
    const int64_t h = q0->shape[0], N_h = q0->shape[3];
    if (Z->shape[0] != n_parts * N_h * h || Z->shape[1] != q0->shape[1] || Z->shape[2] != q0->shape[2])
        return fail(ctx, NNT_EINVAL, "head split/merge: shapes do not match");
    OpTag tag(ctx, to_parts ? "head_split" : "head_merge", present_numel(Z) * Z->elem_size() * 2, true);

    if (ctx->granularity == NNT_GRAN_OP) {
        HeadArgs a;
        a.z = Z->view();
        for (int p = 0; p < 3; p++) a.part[p] = parts[p < n_parts ? p : 0]->view();
        a.n_parts = n_parts; a.N_h = (int32_t)N_h; a.h = (int32_t)h; a.to_parts = to_parts;
        const int V = Z->dtype == NNT_F32 ? 4 : 8;
        bool vec = all_aligned(Z) && axis0_multiple(Z, V) && h % V == 0;
        for (int p = 0; p < n_parts; p++) vec = vec && all_aligned(parts[p]) && axis0_multiple(parts[p], V);
        const int v = vec ? V : 1;
        // workgroup width: the multiple of 64 lanes that wastes the fewest on the row vectors of Z
        const int64_t rowvecs = Z->shape[0] / v, ntok = Z->shape[1] * Z->shape[2];
        int bs = 256;
        int64_t waste = -1;
        for (int cand = 256; cand >= 64; cand -= 64) {
            const int64_t w = (rowvecs + cand - 1) / cand * cand - rowvecs;
            if (waste < 0 || w < waste) { waste = w; bs = cand; }
        }
        const int64_t gx = (rowvecs + bs - 1) / bs, gy = (ntok + kHeadTok - 1) / kHeadTok;
        if (gx > INT32_MAX || gy > 65535) return fail(ctx, NNT_EINVAL, "head split/merge: tensor too large");
        std::vector<Access> acc = {Z->all(to_parts ? kRead : kWrite)};
        for (int p = 0; p < n_parts; p++) acc.push_back(parts[p]->all(to_parts ? kWrite : kRead));
        const int32_t dt = Z->dtype;
        return submit(ctx, acc, [=](hipStream_t st) {
            dim3 grid((unsigned)gx, (unsigned)gy), block((unsigned)bs);
            if (dt == NNT_F32) {
                if (v == 4) hipLaunchKernelGGL((head_kernel<float, 4>), grid, block, 0, st, a);
                else hipLaunchKernelGGL((head_kernel<float, 1>), grid, block, 0, st, a);
            } else {
                if (v == 8) hipLaunchKernelGGL((head_kernel<bf16_t, 8>), grid, block, 0, st, a);
                else hipLaunchKernelGGL((head_kernel<bf16_t, 1>), grid, block, 0, st, a);
            }
            return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
        });
    }

    // tile granularity: one task per (Z tile, part tile) pair that overlaps, made of block copies
    const int32_t dt = Z->dtype;
    for (int64_t zt = 0; zt < Z->ntiles; zt++) {
        int64_t zc[kMaxDim];
        Z->tile_coords(zt, zc);
        const int64_t zr0 = zc[0] * Z->base[0], zr1 = zr0 + Z->tile_extent(0, zc[0]);
        const int64_t zs0 = zc[1] * Z->base[1], zs1 = zs0 + Z->tile_extent(1, zc[1]);
        const int64_t zb0 = zc[2] * Z->base[2], zb1 = zb0 + Z->tile_extent(2, zc[2]);
        const int64_t zm = zr1 - zr0, zsn = zs1 - zs0;
        for (int p = 0; p < n_parts; p++) {
            nnt_tensor* q = parts[p];
            for (int64_t qt = 0; qt < q->ntiles; qt++) {
                int64_t qc[kMaxDim];
                q->tile_coords(qt, qc);
                const int64_t qi0 = qc[0] * q->base[0], qi1 = qi0 + q->tile_extent(0, qc[0]);
                const int64_t qs0 = qc[1] * q->base[1], qs1 = qs0 + q->tile_extent(1, qc[1]);
                const int64_t qb0 = qc[2] * q->base[2], qb1 = qb0 + q->tile_extent(2, qc[2]);
                const int64_t qj0 = qc[3] * q->base[3], qj1 = qj0 + q->tile_extent(3, qc[3]);
                const int64_t s0 = std::max(zs0, qs0), s1 = std::min(zs1, qs1);
                const int64_t b0 = std::max(zb0, qb0), b1 = std::min(zb1, qb1);
                if (s0 >= s1 || b0 >= b1) continue;
                const int64_t qe0 = qi1 - qi0, qe1 = qs1 - qs0, qe2 = qb1 - qb0;
                struct Copy { int64_t ext[3]; int64_t zoff, qoff; };
                std::vector<Copy> copies;
                for (int64_t j = qj0; j < qj1; j++) {
                    const int64_t rbase = (p * N_h + j) * h;
                    const int64_t r0 = std::max(zr0, rbase + qi0), r1 = std::min(zr1, rbase + qi1);
                    if (r0 >= r1) continue;
                    Copy c;
                    c.ext[0] = r1 - r0; c.ext[1] = s1 - s0; c.ext[2] = b1 - b0;
                    c.zoff = (r0 - zr0) + zm * ((s0 - zs0) + zsn * (b0 - zb0));
                    c.qoff = (r0 - rbase - qi0) + qe0 * ((s0 - qs0) + qe1 * ((b0 - qb0) + qe2 * (j - qj0)));
                    copies.push_back(c);
                }
                if (copies.empty()) continue;
                const int64_t zstr[3] = {1, zm, zm * zsn};
                const int64_t qstr[3] = {1, qe0, qe0 * qe1};
                char* zbase = static_cast<char*>(Z->tiles[zt]);
                char* qbase = static_cast<char*>(q->tiles[qt]);
                const int64_t es = Z->elem_size();
                std::vector<Access> acc = {Z->one(zt, to_parts ? kRead : kReadWrite), q->one(qt, to_parts ? kReadWrite : kRead)};
                int32_t rc = submit(ctx, acc, [=](hipStream_t st) {
                    for (const Copy& c : copies) {
                        int32_t r;
                        if (to_parts) r = nnt_tile_copy_block(st, dt, 3, c.ext, zbase + c.zoff * es, zstr, qbase + c.qoff * es, qstr);
                        else r = nnt_tile_copy_block(st, dt, 3, c.ext, qbase + c.qoff * es, qstr, zbase + c.zoff * es, zstr);
                        if (r != NNT_OK) return r;
                    }
                    return (int32_t)NNT_OK;
                }, (int)copies.size());
                if (rc != NNT_OK) return rc;
            }
        }
    }
    return NNT_OK;
}

int32_t nnt_head_split(nnt_ctx* ctx, nnt_tensor* Z, int32_t n_parts, nnt_tensor* const* parts) {
    return head_common(ctx, Z, n_parts, parts, 1);
}
int32_t nnt_head_merge(nnt_ctx* ctx, int32_t n_parts, nnt_tensor* const* parts, nnt_tensor* Z) {
    return head_common(ctx, Z, n_parts, parts, 0);
}

}  // extern "C"
