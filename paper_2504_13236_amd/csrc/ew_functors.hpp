// The elementwise kernel template and its operations (section 3: activations apply
// directly to every tile; the optimizer update is a per-element weighted sum; the
// bias is added over the unchanged dimensions).
//
// One template serves the tile form (plain pointers) and the tensor form (tables
// of tile pointers, blockIdx.y = tile).  Every operation is split into a load
// phase and a compute-and-store phase: a thread first issues the loads of all its
// kUnroll vectors and only then computes and stores, so that several 16-byte loads
// per lane are in flight at once.
#pragma once
#include "device_util.hpp"
#include "gelu_math.hpp"
#include "internal.hpp"

namespace nnt {
namespace {

constexpr int kUnroll = 4;

struct EwGeom {
    TiledView v;        // tiling of the operands (tensor form)
    int64_t n_single;   // element count (tile form)
    const int64_t* numel;   // element count per entry of the pointer tables (group form: tiles of several tensors), or nullptr
    int32_t tiled;
};

struct Operand {
    void* const* table;
    void* single;
};

template <typename T>
__device__ __forceinline__ T* pick(const Operand& o, int tile) {
    return static_cast<T*>(o.table ? o.table[tile] : o.single);
}

// F provides: V (vector width), NIN (values loaded per element), Ctx, setup(),
// load<W>(ctx, i, in[NIN][W]) and store<W>(ctx, i, in[NIN][W]).
template <typename F>
__global__ void __launch_bounds__(256) ew_kernel(const F f, const EwGeom g, const int vec) {
    const int tile = blockIdx.y;
    const int64_t n = g.numel ? g.numel[tile] : (g.tiled ? tile_numel(g.v, tile) : g.n_single);
    typename F::Ctx c;
    if (!f.setup(c, g, tile)) return;
    constexpr int V = F::V, NIN = F::NIN > 0 ? F::NIN : 1;
    const int64_t base = (int64_t)blockIdx.x * kUnroll * 256 * V;
    if (base >= n) return;
    if (vec && base + (int64_t)kUnroll * 256 * V <= n) {
        // whole block inside the tile: all loads first
        float in[kUnroll][NIN][V];
#pragma unroll
        for (int u = 0; u < kUnroll; u++) f.template load<V>(c, base + ((int64_t)u * 256 + threadIdx.x) * V, in[u]);
#pragma unroll
        for (int u = 0; u < kUnroll; u++) f.template store<V>(c, base + ((int64_t)u * 256 + threadIdx.x) * V, in[u]);
    } else if (vec) {
#pragma unroll
        for (int u = 0; u < kUnroll; u++) {
            const int64_t i = base + ((int64_t)u * 256 + threadIdx.x) * V;
            if (i + V <= n) {
                float in[NIN][V];
                f.template load<V>(c, i, in);
                f.template store<V>(c, i, in);
            } else {
                for (int64_t j = i; j < n; j++) {
                    float in[NIN][1];
                    f.template load<1>(c, j, in);
                    f.template store<1>(c, j, in);
                }
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < kUnroll * V; u++) {
            const int64_t i = base + (int64_t)u * 256 + threadIdx.x;
            if (i < n) {
                float in[NIN][1];
                f.template load<1>(c, i, in);
                f.template store<1>(c, i, in);
            }
        }
    }
}

template <typename F>
int32_t launch_ew(hipStream_t st, const F& f, const EwGeom& g, int64_t max_numel, int64_t ntiles, bool vec) {
    if (max_numel <= 0 || ntiles <= 0) return NNT_OK;
    const int64_t per_block = (int64_t)256 * kUnroll * F::V;
    const int64_t gx = (max_numel + per_block - 1) / per_block;
    if (gx > INT32_MAX || ntiles > 65535) return NNT_EINVAL;
    hipLaunchKernelGGL((ew_kernel<F>), dim3((unsigned)gx, (unsigned)ntiles), dim3(256), 0, st, f, g, vec ? 1 : 0);
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

// ------------------------------------------------------------------ operations
template <typename T>
struct FillF {
    static constexpr int V = VecOf<T>::V, NIN = 0;
    Operand x;
    float value;
    struct Ctx { T* x; };
    __device__ bool setup(Ctx& c, const EwGeom&, int tile) const { c.x = pick<T>(x, tile); return c.x != nullptr; }
    template <int W> __device__ void load(const Ctx&, int64_t, float (&)[1][W]) const {}
    template <int W> __device__ void store(const Ctx& c, int64_t i, float (&)[1][W]) const {
        float f[W];
#pragma unroll
        for (int j = 0; j < W; j++) f[j] = value;
        stv<W>(c.x + i, f);
    }
};

template <typename T>
struct AddF {
    static constexpr int V = VecOf<T>::V, NIN = 2;
    Operand x, y;
    float alpha, beta;
    struct Ctx { const T* x; T* y; };
    __device__ bool setup(Ctx& c, const EwGeom&, int tile) const {
        c.x = pick<const T>(x, tile);
        c.y = pick<T>(y, tile);
        return c.y != nullptr;
    }
    template <int W> __device__ void load(const Ctx& c, int64_t i, float (&in)[2][W]) const {
        ldv<W>(c.x + i, in[0]);
        if (beta != 0.f) ldv<W>(c.y + i, in[1]);      // beta == 0 never reads y
    }
    template <int W> __device__ void store(const Ctx& c, int64_t i, float (&in)[2][W]) const {
        float r[W];
#pragma unroll
        for (int j = 0; j < W; j++) r[j] = beta != 0.f ? alpha * in[0][j] + beta * in[1][j] : alpha * in[0][j];
        stv<W>(c.y + i, r);
    }
};

template <typename TI, typename TO>
struct CastF {
    static constexpr int V = 8, NIN = 1;     // 8 elements per thread whatever the types
    Operand x, y;
    struct Ctx { const TI* x; TO* y; };
    __device__ bool setup(Ctx& c, const EwGeom&, int tile) const {
        c.x = pick<const TI>(x, tile);
        c.y = pick<TO>(y, tile);
        return c.y != nullptr;
    }
    template <int W> __device__ void load(const Ctx& c, int64_t i, float (&in)[1][W]) const {
        if constexpr (W == 8 && sizeof(TI) == 4) {
            float a[4], b[4];
            ldv<4>(c.x + i, a);
            ldv<4>(c.x + i + 4, b);
#pragma unroll
            for (int j = 0; j < 4; j++) { in[0][j] = a[j]; in[0][4 + j] = b[j]; }
        } else {
            ldv<W>(c.x + i, in[0]);
        }
    }
    template <int W> __device__ void store(const Ctx& c, int64_t i, float (&in)[1][W]) const {
        if constexpr (W == 8 && sizeof(TO) == 4) {
            float a[4], b[4];
#pragma unroll
            for (int j = 0; j < 4; j++) { a[j] = in[0][j]; b[j] = in[0][4 + j]; }
            stv<4>(c.y + i, a);
            stv<4>(c.y + i + 4, b);
        } else {
            stv<W>(c.y + i, in[0]);
        }
    }
};

template <typename T>
struct GeluF {
    static constexpr int V = VecOf<T>::V, NIN = 1;
    Operand x, y;
    int variant;
    struct Ctx { const T* x; T* y; };
    __device__ bool setup(Ctx& c, const EwGeom&, int tile) const {
        c.x = pick<const T>(x, tile);
        c.y = pick<T>(y, tile);
        return c.y != nullptr;
    }
    template <int W> __device__ void load(const Ctx& c, int64_t i, float (&in)[1][W]) const { ldv<W>(c.x + i, in[0]); }
    template <int W> __device__ void store(const Ctx& c, int64_t i, float (&in)[1][W]) const {
        float r[W];
#pragma unroll
        for (int j = 0; j < W; j++) r[j] = gelu_f(in[0][j], variant);
        stv<W>(c.y + i, r);
    }
};

template <typename T>
struct GeluBwdF {
    static constexpr int V = VecOf<T>::V, NIN = 2;
    Operand x, dy, dx;
    int variant;
    struct Ctx { const T* x; const T* dy; T* dx; };
    __device__ bool setup(Ctx& c, const EwGeom&, int tile) const {
        c.x = pick<const T>(x, tile);
        c.dy = pick<const T>(dy, tile);
        c.dx = pick<T>(dx, tile);
        return c.dx != nullptr;
    }
    template <int W> __device__ void load(const Ctx& c, int64_t i, float (&in)[2][W]) const {
        ldv<W>(c.x + i, in[0]);
        ldv<W>(c.dy + i, in[1]);
    }
    template <int W> __device__ void store(const Ctx& c, int64_t i, float (&in)[2][W]) const {
        float r[W];
#pragma unroll
        for (int j = 0; j < W; j++) r[j] = in[1][j] * gelu_grad_f(in[0][j], variant);
        stv<W>(c.dx + i, r);
    }
};

// Y (m x n, m fastest) += bias[m].  In the tensor form the bias tile is the one
// with the tile's first grid coordinate.
template <typename T>
struct BiasAddF {
    static constexpr int V = VecOf<T>::V, NIN = 2;
    Operand y, b;
    int64_t m_single;
    struct Ctx { T* y; const float* b; int m; };
    __device__ bool setup(Ctx& c, const EwGeom& g, int tile) const {
        c.y = pick<T>(y, tile);
        if (g.tiled) {
            int tc[kMaxDim], ext[kMaxDim];
            tile_geometry(g.v, tile, tc, ext);
            c.m = ext[0];
            c.b = static_cast<const float*>(b.table[tc[0]]);
        } else {
            c.m = (int)m_single;
            c.b = static_cast<const float*>(b.single);
        }
        return c.y != nullptr;
    }
    template <int W> __device__ void load(const Ctx& c, int64_t i, float (&in)[2][W]) const {
        ldv<W>(c.y + i, in[0]);
        const int r = (int)(i % c.m);       // a vector never crosses a column: m % W == 0 on the vector path
        ldv<W>(c.b + r, in[1]);
    }
    template <int W> __device__ void store(const Ctx& c, int64_t i, float (&in)[2][W]) const {
        float r[W];
#pragma unroll
        for (int j = 0; j < W; j++) r[j] = in[0][j] + in[1][j];
        stv<W>(c.y + i, r);
    }
};

struct AdamF {
    static constexpr int V = 4, NIN = 4;
    Operand g, p, m, v, lp;
    float lr, beta1, beta2, omb1, omb2, eps, wd, inv_bc1, inv_bc2;   // omb = 1 - beta, formed in double on the host
    int stream;       // non-temporal accesses: the state is far larger than the last-level cache (measured: 4 % faster
                      // at 24 GB per step, 6 % slower at 0.4 GB, where the gradients still sit in that cache)
    struct Ctx { const float* g; float* p; float* m; float* v; bf16_t* lp; };
    __device__ bool setup(Ctx& c, const EwGeom&, int tile) const {
        c.g = pick<const float>(g, tile);
        c.p = pick<float>(p, tile);
        c.m = pick<float>(m, tile);
        c.v = pick<float>(v, tile);
        c.lp = (lp.table || lp.single) ? pick<bf16_t>(lp, tile) : nullptr;
        return c.p != nullptr;
    }
    template <int W> __device__ void load(const Ctx& c, int64_t i, float (&in)[4][W]) const {
        if (stream) {
            ldv_stream<W>(c.g + i, in[0]);
            ldv_stream<W>(c.p + i, in[1]);
            ldv_stream<W>(c.m + i, in[2]);
            ldv_stream<W>(c.v + i, in[3]);
        } else {
            ldv<W>(c.g + i, in[0]);
            ldv<W>(c.p + i, in[1]);
            ldv<W>(c.m + i, in[2]);
            ldv<W>(c.v + i, in[3]);
        }
    }
    template <int W> __device__ void store(const Ctx& c, int64_t i, float (&in)[4][W]) const {
        float pp[W], mm[W], vv[W];
#pragma unroll
        for (int j = 0; j < W; j++) {
            const float gg = in[0][j];
            mm[j] = beta1 * in[2][j] + omb1 * gg;
            vv[j] = beta2 * in[3][j] + omb2 * gg * gg;
            const float mhat = mm[j] * inv_bc1;
            const float vhat = vv[j] * inv_bc2;
            pp[j] = in[1][j] - lr * wd * in[1][j] - lr * mhat / (sqrtf(vhat) + eps);
        }
        if (stream) {
            stv_stream<W>(c.p + i, pp);
            stv_stream<W>(c.m + i, mm);
            stv_stream<W>(c.v + i, vv);
        } else {
            stv<W>(c.p + i, pp);
            stv<W>(c.m + i, mm);
            stv<W>(c.v + i, vv);
        }
        if (c.lp) {
            if constexpr (W == 4) {
                uint2 x;
                x.x = (uint32_t)f2bf(pp[0]) | ((uint32_t)f2bf(pp[1]) << 16);
                x.y = (uint32_t)f2bf(pp[2]) | ((uint32_t)f2bf(pp[3]) << 16);
                *reinterpret_cast<uint2*>(c.lp + i) = x;
            } else {
                c.lp[i] = f2bf(pp[0]);
            }
        }
    }
};

// SGD with momentum (section 3, Optimizers): the update is a weighted sum of parameter, gradient and
// momentum term.  g' = g + wd p;  v <- mu v + g';  p <- p - lr v   (Nesterov: p - lr (g' + mu v)).
struct SgdF {
    static constexpr int V = 4, NIN = 3;
    Operand g, p, v, lp;
    float lr, mu, wd;
    int nesterov;
    struct Ctx { const float* g; float* p; float* v; bf16_t* lp; };
    __device__ bool setup(Ctx& c, const EwGeom&, int tile) const {
        c.g = pick<const float>(g, tile);
        c.p = pick<float>(p, tile);
        c.v = pick<float>(v, tile);
        c.lp = (lp.table || lp.single) ? pick<bf16_t>(lp, tile) : nullptr;
        return c.p != nullptr;
    }
    template <int W> __device__ void load(const Ctx& c, int64_t i, float (&in)[3][W]) const {
        ldv<W>(c.g + i, in[0]);
        ldv<W>(c.p + i, in[1]);
        ldv<W>(c.v + i, in[2]);
    }
    template <int W> __device__ void store(const Ctx& c, int64_t i, float (&in)[3][W]) const {
        float pp[W], vv[W];
#pragma unroll
        for (int j = 0; j < W; j++) {
            const float gg = in[0][j] + wd * in[1][j];
            vv[j] = mu * in[2][j] + gg;
            pp[j] = in[1][j] - lr * (nesterov ? gg + mu * vv[j] : vv[j]);
        }
        stv<W>(c.p + i, pp);
        stv<W>(c.v + i, vv);
        if (c.lp) {
            if constexpr (W == 4) {
                uint2 x;
                x.x = (uint32_t)f2bf(pp[0]) | ((uint32_t)f2bf(pp[1]) << 16);
                x.y = (uint32_t)f2bf(pp[2]) | ((uint32_t)f2bf(pp[3]) << 16);
                *reinterpret_cast<uint2*>(c.lp + i) = x;
            } else {
                c.lp[i] = f2bf(pp[0]);
            }
        }
    }
};

}  // namespace
}  // namespace nnt
