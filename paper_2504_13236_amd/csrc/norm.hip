// Layer normalisation over the embedding axis (section 3, layer normalization) and
// the column-sum reductions (bias gradient, gain / bias gradients).
//
// Tile form: the paper's steps, one kernel per step and tile -- (1) fold the
// tile's mean and variance into the running statistics, (2)+(3) normalise, scale
// and add the bias.  Tensor form: one wavefront per token walks all embedding
// tiles of that token through the tile-pointer table; the token's values stay in
// registers between the statistics pass and the output pass when they fit, so a
// whole tiled tensor costs one read and one write.  All statistics are fp32; the
// variance is the mean of the squared deviations from the mean (two passes over
// the cached token), never a difference of two large sums.
#include "colwise.hpp"
#include "internal.hpp"

#include <algorithm>
#include <mutex>

namespace nnt {
namespace {

// Visits every V-wide vector of a column: fn(slot, l, e, ext) with l the tile
// along axis 0, e the first row inside it and ext the tile's extent.  With NV > 0
// the loop is fully unrolled and `slot` is a compile-time index into a per-lane
// register cache; with NV == 0 it is a plain loop and slot is 0.
template <int V, int NV, int WPT = 1, typename Fn>
__device__ __forceinline__ void walk(const TiledView& v, int lane, Fn fn, int w = 0) {
    const int g0 = v.grid[0];
    if constexpr (NV > 0) {
        const int vpt = (v.base[0] + 64 * V - 1) / (64 * V);
        int l = 0, j = 0;                 // slot it is vector j of tile l (counted up: no division per slot)
        if constexpr (WPT > 1) {          // wave w of the WPT that share the column takes every WPT-th vector
            l = w / vpt;
            j = w - l * vpt;
        }
#pragma unroll
        for (int it = 0; it < NV; it++) {
            if (l < g0) {
                const int ext = ext0_of(v, l);
                const int e = (j * 64 + lane) * V;
                if (e < ext) fn(it, l, e, ext);
            }
            if constexpr (WPT == 1) {
                if (++j == vpt) {
                    j = 0;
                    l++;
                }
            } else {
                j += WPT;
                while (j >= vpt) {
                    j -= vpt;
                    l++;
                }
            }
        }
    } else {
        for (int l = 0; l < g0; l++) {
            const int ext = ext0_of(v, l);
            for (int e = (w * 64 + lane) * V; e < ext; e += 64 * V * WPT) fn(0, l, e, ext);
        }
    }
}

// Sum over the WPT wavefronts that share a column (all of one workgroup), in wave order.
template <int WPT>
__device__ __forceinline__ float column_sum(float x, float* red, int w, int lane) {
    x = wave_sum(x);
    if constexpr (WPT == 1) return x;
    if (lane == 0) red[w] = x;
    __syncthreads();
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < WPT; i++) s += red[i];
    __syncthreads();
    return s;
}

// WPT = 1: one wavefront per token, four tokens per workgroup.  WPT = 4: the workgroup's four wavefronts share
// one token (long tokens: a quarter of the registers per wave, four times the waves in flight).
template <typename T, int V, int NV, int WPT = 1>
__global__ void __launch_bounds__(256) ln_fwd_fused(TiledView X, TiledView Y, TiledView S, TiledView G, TiledView Bt,
                                                     float eps, int64_t ncols) {
    __shared__ float red[4];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: the index arithmetic below runs on the scalar unit
    const int64_t col = WPT == 1 ? (int64_t)blockIdx.x * 4 + wave : (int64_t)blockIdx.x;
    const int w = WPT == 1 ? 0 : wave;
    if (col >= ncols) return;
    const Column c = column_of(X, col);
    const int N = X.shape[0];
    float cache[NV > 0 ? NV : 1][V];
    // Two passes, mean first and then the squared deviations from it (the one-pass forms cancel when one
    // element of the token lies far from the rest).  The second pass runs over the register cache when
    // the token fits there and re-reads the token otherwise (it is still in the L2 of this wave's XCD).
    float s1 = 0.f;
    walk<V, NV, WPT>(X, lane, [&](int slot, int l, int e, int ext) {
        float x[V];
        ldv<V>(col_ptr<const T>(X, c, l, ext) + e, x);
#pragma unroll
        for (int k = 0; k < V; k++) {
            s1 += x[k];
            if constexpr (NV > 0) cache[slot][k] = x[k];
        }
    }, w);
    const float mean = column_sum<WPT>(s1, red, w, lane) / (float)N;
    float s2 = 0.f;
    walk<V, NV, WPT>(X, lane, [&](int slot, int l, int e, int ext) {
        float x[V];
        if constexpr (NV > 0) {
#pragma unroll
            for (int k = 0; k < V; k++) x[k] = cache[slot][k];
        } else {
            ldv<V>(col_ptr<const T>(X, c, l, ext) + e, x);
        }
#pragma unroll
        for (int k = 0; k < V; k++) s2 += (x[k] - mean) * (x[k] - mean);
    }, w);
    const float var = column_sum<WPT>(s2, red, w, lane) / (float)N;
    const float rstd = 1.f / sqrtf(var + eps);
    walk<V, NV, WPT>(X, lane, [&](int slot, int l, int e, int ext) {
        float x[V], g[V], b[V];
        if constexpr (NV > 0) {
#pragma unroll
            for (int k = 0; k < V; k++) x[k] = cache[slot][k];
        } else {
            ldv<V>(col_ptr<const T>(X, c, l, ext) + e, x);
        }
        ldv<V>(static_cast<const float*>(G.tiles[l]) + e, g);
        ldv<V>(static_cast<const float*>(Bt.tiles[l]) + e, b);
#pragma unroll
        for (int k = 0; k < V; k++) x[k] = g[k] * ((x[k] - mean) * rstd) + b[k];
        stv<V>(col_ptr<T>(Y, c, l, ext) + e, x);
    }, w);
    if (lane == 0 && w == 0) {
        float* s = static_cast<float*>(S.tiles[c.stat_tile]) + 2 * (int64_t)c.colidx;
        s[0] = mean;
        s[1] = rstd;
    }
}

template <typename T, int V, int NV, int WPT = 1>
__global__ void __launch_bounds__(256) ln_bwd_fused(TiledView X, TiledView S, TiledView G, TiledView dY, TiledView dR,
                                                     TiledView dX, int has_res, int64_t ncols) {
    __shared__ float red[4];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: the index arithmetic below runs on the scalar unit
    const int64_t col = WPT == 1 ? (int64_t)blockIdx.x * 4 + wave : (int64_t)blockIdx.x;
    const int w = WPT == 1 ? 0 : wave;
    if (col >= ncols) return;
    const Column c = column_of(X, col);
    const int N = X.shape[0];
    const float* st = static_cast<const float*>(S.tiles[c.stat_tile]) + 2 * (int64_t)c.colidx;
    const float mean = st[0], rstd = st[1];
    float cg[NV > 0 ? NV : 1][V], ch[NV > 0 ? NV : 1][V];   // g = dy * gamma, xhat
    float a = 0.f, b = 0.f;
    walk<V, NV, WPT>(X, lane, [&](int slot, int l, int e, int ext) {
        float x[V], d[V], g[V];
        ldv<V>(col_ptr<const T>(X, c, l, ext) + e, x);
        ldv<V>(col_ptr<const T>(dY, c, l, ext) + e, d);
        ldv<V>(static_cast<const float*>(G.tiles[l]) + e, g);
#pragma unroll
        for (int k = 0; k < V; k++) {
            const float gg = d[k] * g[k], xh = (x[k] - mean) * rstd;
            a += gg;
            b += gg * xh;
            if constexpr (NV > 0) { cg[slot][k] = gg; ch[slot][k] = xh; }
        }
    }, w);
    a = column_sum<WPT>(a, red, w, lane) / (float)N;
    b = column_sum<WPT>(b, red, w, lane) / (float)N;
    walk<V, NV, WPT>(X, lane, [&](int slot, int l, int e, int ext) {
        float gg[V], xh[V], r[V];
        if constexpr (NV > 0) {
#pragma unroll
            for (int k = 0; k < V; k++) { gg[k] = cg[slot][k]; xh[k] = ch[slot][k]; }
        } else {
            float x[V], d[V], g[V];
            ldv<V>(col_ptr<const T>(X, c, l, ext) + e, x);
            ldv<V>(col_ptr<const T>(dY, c, l, ext) + e, d);
            ldv<V>(static_cast<const float*>(G.tiles[l]) + e, g);
#pragma unroll
            for (int k = 0; k < V; k++) { gg[k] = d[k] * g[k]; xh[k] = (x[k] - mean) * rstd; }
        }
#pragma unroll
        for (int k = 0; k < V; k++) r[k] = rstd * (gg[k] - a - xh[k] * b);
        if (has_res) {
            float q[V];
            ldv<V>(col_ptr<const T>(dR, c, l, ext) + e, q);
#pragma unroll
            for (int k = 0; k < V; k++) r[k] += q[k];
        }
        stv<V>(col_ptr<T>(dX, c, l, ext) + e, r);
    }, w);
}

// ------------------------------------------------------------------ tile-form kernels (one wave per token of an m x n tile)
template <typename T, int V>
__global__ void __launch_bounds__(256) ln_stats_tile(const T* x, float* stats, int m, int64_t n, int64_t count_before,
                                                      int64_t finalize_total, float eps) {
    const int lane = threadIdx.x & 63;
    const int64_t col = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: the index arithmetic below runs on the scalar unit
    if (col >= n) return;
    const T* p = x + col * m;
    float s = 0.f;
    for (int e = lane * V; e < m; e += 64 * V) {
        float f[V];
        ldv<V>(p + e, f);
#pragma unroll
        for (int k = 0; k < V; k++) s += f[k];
    }
    const float mean_t = wave_sum(s) / (float)m;
    float q = 0.f;
    for (int e = lane * V; e < m; e += 64 * V) {
        float f[V];
        ldv<V>(p + e, f);
#pragma unroll
        for (int k = 0; k < V; k++) q += (f[k] - mean_t) * (f[k] - mean_t);
    }
    const float m2_t = wave_sum(q);
    if (lane == 0) {
        float mean = mean_t, m2 = m2_t;
        const float na = (float)count_before, nb = (float)m;
        if (count_before > 0) {
            // pairwise update of (count, mean, sum of squared deviations)
            const float mean_a = stats[2 * col], m2_a = stats[2 * col + 1];
            const float delta = mean_t - mean_a;
            mean = mean_a + delta * (nb / (na + nb));
            m2 = m2_a + m2_t + delta * delta * (na * nb / (na + nb));
        }
        if (finalize_total > 0) m2 = 1.f / sqrtf(m2 / (float)finalize_total + eps);
        stats[2 * col] = mean;
        stats[2 * col + 1] = m2;
    }
}

template <typename T, int V>
__global__ void __launch_bounds__(256) ln_apply_tile(const T* x, const float* stats, const float* gamma, const float* beta,
                                                      T* y, int m, int64_t n) {
    const int lane = threadIdx.x & 63;
    const int64_t col = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: the index arithmetic below runs on the scalar unit
    if (col >= n) return;
    const float mean = stats[2 * col], rstd = stats[2 * col + 1];
    for (int e = lane * V; e < m; e += 64 * V) {
        float f[V], g[V], b[V];
        ldv<V>(x + col * m + e, f);
        ldv<V>(gamma + e, g);
        ldv<V>(beta + e, b);
#pragma unroll
        for (int k = 0; k < V; k++) f[k] = g[k] * ((f[k] - mean) * rstd) + b[k];
        stv<V>(y + col * m + e, f);
    }
}

template <typename T, int V>
__global__ void __launch_bounds__(256) ln_bwd_sums_tile(const T* x, const float* stats, const float* gamma, const T* dy,
                                                         float* sums, int init, int m, int64_t n) {
    const int lane = threadIdx.x & 63;
    const int64_t col = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: the index arithmetic below runs on the scalar unit
    if (col >= n) return;
    const float mean = stats[2 * col], rstd = stats[2 * col + 1];
    float a = 0.f, b = 0.f;
    for (int e = lane * V; e < m; e += 64 * V) {
        float f[V], d[V], g[V];
        ldv<V>(x + col * m + e, f);
        ldv<V>(dy + col * m + e, d);
        ldv<V>(gamma + e, g);
#pragma unroll
        for (int k = 0; k < V; k++) {
            const float gg = d[k] * g[k];
            a += gg;
            b += gg * ((f[k] - mean) * rstd);
        }
    }
    a = wave_sum(a);
    b = wave_sum(b);
    if (lane == 0) {
        if (init) { sums[2 * col] = a; sums[2 * col + 1] = b; }
        else { sums[2 * col] += a; sums[2 * col + 1] += b; }
    }
}

template <typename T, int V>
__global__ void __launch_bounds__(256) ln_bwd_dx_tile(const T* x, const float* stats, const float* gamma, const T* dy,
                                                       const float* sums, const T* dres, T* dx, int m, int64_t n, float inv_N) {
    const int lane = threadIdx.x & 63;
    const int64_t col = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: the index arithmetic below runs on the scalar unit
    if (col >= n) return;
    const float mean = stats[2 * col], rstd = stats[2 * col + 1];
    const float a = sums[2 * col] * inv_N, b = sums[2 * col + 1] * inv_N;
    for (int e = lane * V; e < m; e += 64 * V) {
        float f[V], d[V], g[V];
        ldv<V>(x + col * m + e, f);
        ldv<V>(dy + col * m + e, d);
        ldv<V>(gamma + e, g);
#pragma unroll
        for (int k = 0; k < V; k++) f[k] = rstd * (d[k] * g[k] - a - ((f[k] - mean) * rstd) * b);
        if (dres) {
            float q[V];
            ldv<V>(dres + col * m + e, q);
#pragma unroll
            for (int k = 0; k < V; k++) f[k] += q[k];
        }
        stv<V>(dx + col * m + e, f);
    }
}

// ------------------------------------------------------------------ column sums in two stages
// Stage 1: block (bx, by, tile) sums the rows [bx * 64 V, ...) of one tile over the
// columns [by * cpb, (by + 1) * cpb) and stores a partial row; stage 2 adds the
// partials of every row.  MODE 0: sum of dy (bias gradient).  MODE 1: sums of
// dy * xhat and of dy (gain and bias gradients of the layer norm).
struct RowsumGeom {
    TiledView y;            // tiling (tensor form)
    void* const* ytab;      // tile tables (tensor form) ...
    void* const* xtab;
    void* const* stab;
    const void* y1;         // ... or single tiles
    const void* x1;
    const float* s1;
    int32_t m1;             // extents of the single tile
    int64_t n1;
    int32_t tiled;
    int32_t cpb;            // columns per block
    int32_t splits;         // column splits per tile
    int64_t rows_total;     // length of a partial row
    int64_t nslots;         // partial rows per output (the second output of MODE 1 follows the first)
};

template <typename T, int V, int MODE>
__global__ void __launch_bounds__(256) rowsum_stage1(RowsumGeom g, float* part) {
    __shared__ float red[2][4][64 * V];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tile = blockIdx.z;
    int ext0, row0;
    int64_t ncol, slot;
    const T* y;
    const T* x = nullptr;
    const float* st = nullptr;
    if (g.tiled) {
        int tc[kMaxDim], ext[kMaxDim];
        tile_geometry(g.y, tile, tc, ext);
        ext0 = ext[0];
        ncol = (int64_t)ext[1] * ext[2] * ext[3];
        row0 = tc[0] * g.y.base[0];
        y = static_cast<const T*>(g.ytab[tile]);
        const int rest = tile / g.y.grid[0];
        if (MODE == 1) {
            x = static_cast<const T*>(g.xtab[tile]);
            st = static_cast<const float*>(g.stab[rest]);
        }
        slot = (int64_t)rest * g.splits + blockIdx.y;
    } else {
        ext0 = g.m1;
        ncol = g.n1;
        row0 = 0;
        y = static_cast<const T*>(g.y1);
        if (MODE == 1) { x = static_cast<const T*>(g.x1); st = g.s1; }
        slot = blockIdx.y;
    }
    const int e = (blockIdx.x * 64 + lane) * V;
    const int64_t c0 = (int64_t)blockIdx.y * g.cpb;
    const int64_t c1 = min(ncol, c0 + g.cpb);
    float a0[V], a1[V];
#pragma unroll
    for (int k = 0; k < V; k++) a0[k] = a1[k] = 0.f;
    if (y && e < ext0) {
        // four columns per trip so that four loads per operand are in flight
        for (int64_t cb = c0 + wave; cb < c1; cb += 16) {
            float d[4][V], f[4][V];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int64_t c = cb + 4 * u;
                if (c < c1) {
                    ldv<V>(y + c * ext0 + e, d[u]);
                    if (MODE == 1) ldv<V>(x + c * ext0 + e, f[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int64_t c = cb + 4 * u;
                if (c < c1) {
                    if (MODE == 1) {
                        const float mean = st[2 * c], rstd = st[2 * c + 1];
#pragma unroll
                        for (int k = 0; k < V; k++) { a0[k] += d[u][k] * ((f[u][k] - mean) * rstd); a1[k] += d[u][k]; }
                    } else {
#pragma unroll
                        for (int k = 0; k < V; k++) a0[k] += d[u][k];
                    }
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < V; k++) {
        red[0][wave][lane * V + k] = a0[k];
        if (MODE == 1) red[1][wave][lane * V + k] = a1[k];
    }
    __syncthreads();
    if (wave == 0 && e < ext0) {
#pragma unroll
        for (int k = 0; k < V; k++) {
            const int i = lane * V + k;
            part[slot * g.rows_total + row0 + e + k] = red[0][0][i] + red[0][1][i] + red[0][2][i] + red[0][3][i];
            if (MODE == 1)
                part[(slot + g.nslots) * g.rows_total + row0 + e + k] =
                    red[1][0][i] + red[1][1][i] + red[1][2][i] + red[1][3][i];
        }
    }
}

// out[r] = (accumulate ? out[r] : 0) + sum_s part[s][r]; the output is a 1-axis tiled tensor or a plain vector.
constexpr int kStage2Rows = 16;

// gridDim.y = 2 reduces a second set of partial rows (right behind the first) into (otab_b, ob)
__global__ void __launch_bounds__(256) rowsum_stage2(const float* part, int64_t nslots, int64_t rows_total,
                                                      void* const* otab, float* o1, int base0, int accumulate,
                                                      void* const* otab_b, float* ob) {
    if (blockIdx.y) {
        part += nslots * rows_total;
        otab = otab_b;
        o1 = ob;
    }
    // 16 rows per block (64-byte runs of a partial row); 16 groups of lanes take every sixteenth partial
    // row, four loads in flight each, then combine through LDS in a fixed order.  The grid is small
    // (rows / 16 blocks), so the kernel is bound by the latency of its load chain: many short chains.
    __shared__ float red[16][17];
    const int rl = threadIdx.x & 15, kg = threadIdx.x >> 4;
    const int64_t r = (int64_t)blockIdx.x * kStage2Rows + rl;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (r < rows_total) {
        int64_t k = kg;
        for (; k + 48 < nslots; k += 64) {
            s0 += part[k * rows_total + r];
            s1 += part[(k + 16) * rows_total + r];
            s2 += part[(k + 32) * rows_total + r];
            s3 += part[(k + 48) * rows_total + r];
        }
        for (; k < nslots; k += 16) s0 += part[k * rows_total + r];
    }
    red[kg][rl] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (kg == 0 && r < rows_total) {
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < 16; q++) s += red[q][rl];
        float* o = otab ? static_cast<float*>(otab[r / base0]) + (r % base0) : o1 + r;
        *o = accumulate ? *o + s : s;
    }
}

constexpr int kColsPerBlock = 128;

int64_t scratch_elems(int64_t m, int64_t n, int mode) { return ((n + kColsPerBlock - 1) / kColsPerBlock) * m * (mode ? 2 : 1); }

template <typename T, int MODE>
int32_t launch_rowsum_t(hipStream_t st, const RowsumGeom& g, int vpt_v, int vpt_1, int64_t ntiles, bool vec, float* part) {
    constexpr int V = VecOf<T>::V;
    if (vec) hipLaunchKernelGGL((rowsum_stage1<T, V, MODE>), dim3(vpt_v, g.splits, (unsigned)ntiles), dim3(256), 0, st, g, part);
    else hipLaunchKernelGGL((rowsum_stage1<T, 1, MODE>), dim3(vpt_1, g.splits, (unsigned)ntiles), dim3(256), 0, st, g, part);
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

// single tile: dY (m x n) -> out0 (and out1 in MODE 1)
int32_t rowsum_single(hipStream_t st, int dtype, int mode, int64_t m, int64_t n, const void* dy, const void* x,
                      const float* stats, float* out0, float* out1, int accumulate, float* scratch) {
    if (m == 0) return NNT_OK;
    RowsumGeom g = {};
    g.tiled = 0;
    g.y1 = dy; g.x1 = x; g.s1 = stats;
    g.m1 = (int32_t)m; g.n1 = n;
    g.cpb = kColsPerBlock;
    g.splits = (int32_t)std::max<int64_t>(1, (n + kColsPerBlock - 1) / kColsPerBlock);
    g.rows_total = m;
    g.nslots = g.splits;
    const int V = dtype == NNT_F32 ? 4 : 8;
    const bool vec = m % V == 0 && aligned16(dy) && (!x || aligned16(x));
    const int vv = (int)((m + 64 * V - 1) / (64 * V)), v1 = (int)((m + 63) / 64);
    int32_t rc;
    if (dtype == NNT_F32) rc = mode ? launch_rowsum_t<float, 1>(st, g, vv, v1, 1, vec, scratch) : launch_rowsum_t<float, 0>(st, g, vv, v1, 1, vec, scratch);
    else rc = mode ? launch_rowsum_t<bf16_t, 1>(st, g, vv, v1, 1, vec, scratch) : launch_rowsum_t<bf16_t, 0>(st, g, vv, v1, 1, vec, scratch);
    if (rc != NNT_OK) return rc;
    const unsigned blocks = (unsigned)((m + kStage2Rows - 1) / kStage2Rows);
    hipLaunchKernelGGL(rowsum_stage2, dim3(blocks, mode ? 2 : 1), dim3(256), 0, st, scratch, (int64_t)g.splits, m, nullptr, out0, 1,
                       accumulate, nullptr, out1);
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

// whole tiled tensor dY [rows, ...] -> out0 / out1: 1-axis tensors tiled like dY's first axis
int32_t rowsum_tensor(nnt_ctx* ctx, int mode, nnt_tensor* dY, nnt_tensor* X, nnt_tensor* S, nnt_tensor* out0, nnt_tensor* out1) {
    int64_t max_cols = 1, rest_tiles = 1;
    for (int a = 1; a < dY->ndim; a++) { max_cols *= dY->base[a]; rest_tiles *= dY->grid[a]; }
    RowsumGeom g = {};
    g.tiled = 1;
    g.y = dY->view();
    g.ytab = dY->d_tiles;
    g.xtab = X ? X->d_tiles : nullptr;
    g.stab = S ? S->d_tiles : nullptr;
    // columns per block: fewer when the tensor would otherwise give the chip too few blocks
    int cpb = kColsPerBlock;
    {
        const int V0 = dY->dtype == NNT_F32 ? 4 : 8;
        const int64_t row_blocks = (dY->base[0] + 64 * V0 - 1) / (64 * V0);
        while (cpb > 32 && row_blocks * ((max_cols + cpb - 1) / cpb) * dY->ntiles < 1024) cpb /= 2;
    }
    g.cpb = cpb;
    g.splits = (int32_t)((max_cols + cpb - 1) / cpb);
    g.rows_total = dY->shape[0];
    const int64_t nslots = rest_tiles * g.splits;
    g.nslots = nslots;
    const int64_t need = nslots * g.rows_total * (mode ? 2 : 1);
    int32_t rc = ensure_scratch(ctx, need);
    if (rc != NNT_OK) return rc;
    if (dY->ntiles > 65535 || g.splits > 65535) return fail(ctx, NNT_EINVAL, "column sum: too many tiles");
    const int V = dY->dtype == NNT_F32 ? 4 : 8;
    bool vec = dY->base[0] % V == 0 && dY->shape[0] % V == 0;
    for (void* p : dY->tiles) vec = vec && aligned16(p);
    if (X) for (void* p : X->tiles) vec = vec && aligned16(p);
    const int vv = (int)((dY->base[0] + 64 * V - 1) / (64 * V)), v1 = (int)((dY->base[0] + 63) / 64);
    float* scratch = ctx->red_scratch;
    const int dtype = dY->dtype;
    const int64_t ntiles = dY->ntiles, rows = g.rows_total;
    void* const* o0 = out0->d_tiles;
    void* const* o1 = out1 ? out1->d_tiles : nullptr;
    const int base0 = (int)out0->base[0];
    std::vector<Access> acc = {dY->all(kRead), out0->all(kWrite), Access{&ctx->red_dep, 1, kReadWrite}};
    if (X) acc.push_back(X->all(kRead));
    if (S) acc.push_back(S->all(kRead));
    if (out1) acc.push_back(out1->all(kWrite));
    return submit(ctx, acc, [=](hipStream_t st) {
        int32_t r;
        if (dtype == NNT_F32) r = mode ? launch_rowsum_t<float, 1>(st, g, vv, v1, ntiles, vec, scratch) : launch_rowsum_t<float, 0>(st, g, vv, v1, ntiles, vec, scratch);
        else r = mode ? launch_rowsum_t<bf16_t, 1>(st, g, vv, v1, ntiles, vec, scratch) : launch_rowsum_t<bf16_t, 0>(st, g, vv, v1, ntiles, vec, scratch);
        if (r != NNT_OK) return r;
        const unsigned blocks = (unsigned)((rows + kStage2Rows - 1) / kStage2Rows);
        hipLaunchKernelGGL(rowsum_stage2, dim3(blocks, mode ? 2 : 1), dim3(256), 0, st, scratch, nslots, rows, o0, nullptr, base0, 0,
                           o1, nullptr);
        return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
    }, 2);
}

bool tensors_vec_ok(std::initializer_list<const nnt_tensor*> ts, int V) {
    for (const nnt_tensor* t : ts) {
        if (!t) continue;
        if (t->base[0] % V != 0 || t->shape[0] % V != 0) return false;
        for (void* p : t->tiles)
            if (p && !aligned16(p)) return false;
    }
    return true;
}

// Tokens of more vectors per lane than this are shared by the four wavefronts of a workgroup (measured: shorter
// tokens lose to the two workgroup barriers, longer ones gain from four times the loads in flight).
constexpr int kLnShareAbove = 4;

template <typename T>
int32_t launch_ln_fwd(hipStream_t st, bool vec, int nv_needed, const TiledView& X, const TiledView& Y, const TiledView& S,
                      const TiledView& G, const TiledView& B, float eps, int64_t ncols) {
    constexpr int V = VecOf<T>::V;
    // tokens of more than `kLnShareAbove` vectors per lane are shared by the four wavefronts of a workgroup
    const bool shared = vec && nv_needed > kLnShareAbove;
    const dim3 grid((unsigned)(shared ? ncols : (ncols + 3) / 4)), block(256);
    if (!vec) hipLaunchKernelGGL((ln_fwd_fused<T, 1, 0>), grid, block, 0, st, X, Y, S, G, B, eps, ncols);
    else if (!shared && nv_needed <= 4) hipLaunchKernelGGL((ln_fwd_fused<T, V, 4>), grid, block, 0, st, X, Y, S, G, B, eps, ncols);
    else if (!shared && nv_needed <= 16) hipLaunchKernelGGL((ln_fwd_fused<T, V, 16>), grid, block, 0, st, X, Y, S, G, B, eps, ncols);
    else if (!shared) hipLaunchKernelGGL((ln_fwd_fused<T, V, 0>), grid, block, 0, st, X, Y, S, G, B, eps, ncols);
    else if (nv_needed <= 16) hipLaunchKernelGGL((ln_fwd_fused<T, V, 4, 4>), grid, block, 0, st, X, Y, S, G, B, eps, ncols);
    else if (nv_needed <= 64) hipLaunchKernelGGL((ln_fwd_fused<T, V, 16, 4>), grid, block, 0, st, X, Y, S, G, B, eps, ncols);
    else hipLaunchKernelGGL((ln_fwd_fused<T, V, 0, 4>), grid, block, 0, st, X, Y, S, G, B, eps, ncols);
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

template <typename T>
int32_t launch_ln_bwd(hipStream_t st, bool vec, int nv_needed, const TiledView& X, const TiledView& S, const TiledView& G,
                      const TiledView& dY, const TiledView& dR, const TiledView& dX, int has_res, int64_t ncols) {
    constexpr int V = VecOf<T>::V;
    const bool shared = vec && nv_needed > kLnShareAbove;
    const dim3 grid((unsigned)(shared ? ncols : (ncols + 3) / 4)), block(256);
    if (!vec) hipLaunchKernelGGL((ln_bwd_fused<T, 1, 0>), grid, block, 0, st, X, S, G, dY, dR, dX, has_res, ncols);
    else if (!shared && nv_needed <= 4) hipLaunchKernelGGL((ln_bwd_fused<T, V, 4>), grid, block, 0, st, X, S, G, dY, dR, dX, has_res, ncols);
    else if (!shared && nv_needed <= 8) hipLaunchKernelGGL((ln_bwd_fused<T, V, 8>), grid, block, 0, st, X, S, G, dY, dR, dX, has_res, ncols);
    else if (!shared) hipLaunchKernelGGL((ln_bwd_fused<T, V, 0>), grid, block, 0, st, X, S, G, dY, dR, dX, has_res, ncols);
    else if (nv_needed <= 16) hipLaunchKernelGGL((ln_bwd_fused<T, V, 4, 4>), grid, block, 0, st, X, S, G, dY, dR, dX, has_res, ncols);
    else if (nv_needed <= 32) hipLaunchKernelGGL((ln_bwd_fused<T, V, 8, 4>), grid, block, 0, st, X, S, G, dY, dR, dX, has_res, ncols);
    else hipLaunchKernelGGL((ln_bwd_fused<T, V, 0, 4>), grid, block, 0, st, X, S, G, dY, dR, dX, has_res, ncols);
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int32_t check_ln_shapes(nnt_ctx* ctx, const nnt_tensor* X, const nnt_tensor* gamma, const nnt_tensor* stats, const char* who) {
    if (X->ndim < 2) return fail(ctx, NNT_EINVAL, std::string(who) + ": X needs at least 2 axes");
    if (gamma->dtype != NNT_F32 || gamma->ndim != 1 || gamma->shape[0] != X->shape[0] || gamma->base[0] != X->base[0])
        return fail(ctx, NNT_EINVAL, std::string(who) + ": gain / bias must be fp32 vectors tiled like X's first axis");
    if (stats->dtype != NNT_F32 || stats->ndim != X->ndim || stats->shape[0] != 2 || stats->base[0] != 2)
        return fail(ctx, NNT_EINVAL, std::string(who) + ": stats must be fp32 [2, ...] with an untiled first axis");
    for (int a = 1; a < X->ndim; a++)
        if (stats->shape[a] != X->shape[a] || stats->base[a] != X->base[a])
            return fail(ctx, NNT_EINVAL, std::string(who) + ": stats must be tiled like X's other axes");
    for (void* p : X->tiles) if (!p) return fail(ctx, NNT_EINVAL, std::string(who) + ": structural-zero tiles not allowed");
    for (void* p : stats->tiles) if (!p) return fail(ctx, NNT_EINVAL, std::string(who) + ": structural-zero tiles not allowed");
    for (void* p : gamma->tiles) if (!p) return fail(ctx, NNT_EINVAL, std::string(who) + ": structural-zero tiles not allowed");
    return NNT_OK;
}

}  // namespace
}  // namespace nnt

using namespace nnt;

#define DT_OK(d) ((d) == NNT_F32 || (d) == NNT_BF16)
// Runs CALL with T = element type and V = vector width (full width when `vec`, else 1).
#define DISPATCH_TV(dtype, vec, CALL)                                           \
    do {                                                                        \
        if ((dtype) == NNT_F32) {                                               \
            typedef float T;                                                    \
            if (vec) { constexpr int V = 4; CALL; } else { constexpr int V = 1; CALL; } \
        } else {                                                                \
            typedef bf16_t T;                                                   \
            if (vec) { constexpr int V = 8; CALL; } else { constexpr int V = 1; CALL; } \
        }                                                                       \
    } while (0)

static inline bool cols_ok(int64_t m, int64_t n) { return m >= 1 && n >= 0 && m <= INT32_MAX && n <= (int64_t)INT32_MAX * 4; }

// ------------------------------------------------------------------ bias gradient without any allocation
// Partial column sums of nnt_tile_bias_grad_static live in this array: one copy per GPU, held until
// the process ends.  In host code the array's name is only a stand-in for the symbol; the device
// address is looked up once per device and kept.
constexpr int64_t kStaticScratchElems = (int64_t)1 << 20;      // 4 MiB of fp32
constexpr int kStaticMaxDevices = 64;
static __device__ __align__(256) float static_scratch[kStaticScratchElems];

namespace {
std::mutex g_static_mu;
float* g_static_ptr[kStaticMaxDevices] = {};

// device address of this GPU's copy of `static_scratch` (current device), or nullptr with *rc set
float* static_scratch_of_current_device(int32_t* rc) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStaticMaxDevices) { *rc = NNT_EHIP; return nullptr; }
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        float* ptr = nullptr;
        if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(static_scratch)) != hipSuccess || !ptr) { *rc = NNT_EHIP; return nullptr; }
        g_static_ptr[dev] = ptr;
    }
    *rc = NNT_OK;
    return g_static_ptr[dev];
}
}  // namespace

namespace nnt {
int32_t static_scratch_setup() {
    int32_t rc;
    (void)static_scratch_of_current_device(&rc);
    return rc;
}
}  // namespace nnt

extern "C" {

int32_t nnt_tile_ln_stats(void* stream, int32_t dtype, int64_t m, int64_t n, const void* x, float* stats,
                          int64_t count_before, int64_t finalize_total, float eps) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (!cols_ok(m, n) || count_before < 0 || (finalize_total > 0 && finalize_total != count_before + m)) return NNT_EINVAL;
    if (n == 0) return NNT_OK;
    if (!x || !stats) return NNT_EINVAL;
    const bool vec = aligned16(x) && m % (dtype == NNT_F32 ? 4 : 8) == 0;
    const dim3 grid((unsigned)((n + 3) / 4)), block(256);
    DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((ln_stats_tile<T, V>), grid, block, 0, (hipStream_t)stream,
                                               (const T*)x, stats, (int)m, n, count_before, finalize_total, eps));
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int32_t nnt_tile_ln_apply(void* stream, int32_t dtype, int64_t m, int64_t n, const void* x, const float* stats,
                          const float* gamma, const float* beta, void* y) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (!cols_ok(m, n)) return NNT_EINVAL;
    if (n == 0) return NNT_OK;
    if (!x || !stats || !gamma || !beta || !y) return NNT_EINVAL;
    const bool vec = aligned16(x) && aligned16(y) && aligned16(gamma) && aligned16(beta) && m % (dtype == NNT_F32 ? 4 : 8) == 0;
    const dim3 grid((unsigned)((n + 3) / 4)), block(256);
    DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((ln_apply_tile<T, V>), grid, block, 0, (hipStream_t)stream,
                                               (const T*)x, stats, gamma, beta, (T*)y, (int)m, n));
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int32_t nnt_tile_ln_bwd_sums(void* stream, int32_t dtype, int64_t m, int64_t n, const void* x, const float* stats,
                             const float* gamma, const void* dy, float* sums, int32_t init) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (!cols_ok(m, n)) return NNT_EINVAL;
    if (n == 0) return NNT_OK;
    if (!x || !stats || !gamma || !dy || !sums) return NNT_EINVAL;
    const bool vec = aligned16(x) && aligned16(dy) && aligned16(gamma) && m % (dtype == NNT_F32 ? 4 : 8) == 0;
    const dim3 grid((unsigned)((n + 3) / 4)), block(256);
    DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((ln_bwd_sums_tile<T, V>), grid, block, 0, (hipStream_t)stream,
                                               (const T*)x, stats, gamma, (const T*)dy, sums, (int)init, (int)m, n));
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int32_t nnt_tile_ln_bwd_dx(void* stream, int32_t dtype, int64_t m, int64_t n, int64_t N_e, const void* x,
                           const float* stats, const float* gamma, const void* dy, const float* sums,
                           const void* dres, void* dx) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (!cols_ok(m, n) || N_e < m) return NNT_EINVAL;
    if (n == 0) return NNT_OK;
    if (!x || !stats || !gamma || !dy || !sums || !dx) return NNT_EINVAL;
    const bool vec = aligned16(x) && aligned16(dy) && aligned16(gamma) && aligned16(dx) && (!dres || aligned16(dres)) &&
                     m % (dtype == NNT_F32 ? 4 : 8) == 0;
    const dim3 grid((unsigned)((n + 3) / 4)), block(256);
    const float inv_N = 1.f / (float)N_e;
    DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((ln_bwd_dx_tile<T, V>), grid, block, 0, (hipStream_t)stream,
                                               (const T*)x, stats, gamma, (const T*)dy, sums, (const T*)dres, (T*)dx, (int)m, n, inv_N));
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int64_t nnt_tile_ln_bwd_params_scratch(int64_t m, int64_t n) { return m < 0 || n < 0 ? 0 : scratch_elems(m, std::max<int64_t>(n, 1), 1); }
int64_t nnt_tile_bias_grad_scratch(int64_t m, int64_t n) { return m < 0 || n < 0 ? 0 : scratch_elems(m, std::max<int64_t>(n, 1), 0); }

int32_t nnt_tile_ln_bwd_params(void* stream, int32_t dtype, int64_t m, int64_t n, const void* x, const float* stats,
                               const void* dy, float* dgamma, float* dbeta, int32_t accumulate, float* scratch) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (!cols_ok(m, n)) return NNT_EINVAL;
    if (!x || !stats || !dy || !dgamma || !dbeta || !scratch) return NNT_EINVAL;
    return rowsum_single((hipStream_t)stream, dtype, 1, m, n, dy, x, stats, dgamma, dbeta, accumulate, scratch);
}

int32_t nnt_tile_bias_grad(void* stream, int32_t dtype, int64_t m, int64_t n, const void* dY, float* db,
                           int32_t accumulate, float* scratch) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (!cols_ok(m, n)) return NNT_EINVAL;
    if (!dY || !db || !scratch) return NNT_EINVAL;
    return rowsum_single((hipStream_t)stream, dtype, 0, m, n, dY, nullptr, nullptr, db, nullptr, accumulate, scratch);
}

// ------------------------------------------------------------------ bias gradient without any allocation
int64_t nnt_tile_bias_grad_static_max(void) { return kStaticScratchElems; }

int32_t nnt_tile_bias_grad_static(void* stream, int32_t dtype, int64_t m, int64_t n, const void* dY, float* db,
                                  int32_t accumulate) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (!cols_ok(m, n)) return NNT_EINVAL;
    if (!dY || !db) return NNT_EINVAL;
    if (scratch_elems(m, n, 0) > kStaticScratchElems) return NNT_EINVAL;      // partial sums would not fit the static array
    int32_t rc;
    float* part = static_scratch_of_current_device(&rc);
    if (!part) return rc;
    // every partial row that stage 2 reads is written by stage 1 of this call: nothing to clear
    return rowsum_single((hipStream_t)stream, dtype, 0, m, n, dY, nullptr, nullptr, db, nullptr, accumulate, part);
}

// ------------------------------------------------------------------ tensor form
int32_t nnt_bias_grad(nnt_ctx* ctx, nnt_tensor* dY, nnt_tensor* db) {
    NNT_CHECK_CTX(ctx);
    if (!dY || !db) return fail(ctx, NNT_EINVAL, "nnt_bias_grad: null tensor");
    if (db->dtype != NNT_F32 || db->ndim != 1 || db->shape[0] != dY->shape[0] || db->base[0] != dY->base[0])
        return fail(ctx, NNT_EINVAL, "nnt_bias_grad: db must be an fp32 vector tiled like dY's first axis");
    for (void* p : dY->tiles) if (!p) return fail(ctx, NNT_EINVAL, "nnt_bias_grad: structural-zero tiles not allowed");
    for (void* p : db->tiles) if (!p) return fail(ctx, NNT_EINVAL, "nnt_bias_grad: structural-zero tiles not allowed");
    double numel = 1;
    for (int a = 0; a < dY->ndim; a++) numel *= (double)dY->shape[a];
    OpTag tag(ctx, "bias_grad", numel * dY->elem_size(), true);
    if (ctx->granularity == NNT_GRAN_OP) return rowsum_tensor(ctx, 0, dY, nullptr, nullptr, db, nullptr);
    // tile by tile: each dY tile adds its column sums to the db tile of its row range
    std::vector<char> seen(db->ntiles, 0);
    for (int64_t t = 0; t < dY->ntiles; t++) {
        const int64_t c0 = t % dY->grid[0];
        const int64_t m = dY->tile_extent(0, c0), n = dY->tile_numel(t) / m;
        int32_t rc = ensure_scratch(ctx, scratch_elems(m, n, 0));
        if (rc != NNT_OK) return rc;
        const void* yp = dY->tiles[t];
        float* op = static_cast<float*>(db->tiles[c0]);
        float* scratch = ctx->red_scratch;
        const int acc = seen[c0];
        seen[c0] = 1;
        const int dt = dY->dtype;
        rc = submit(ctx, {dY->one(t, kRead), db->one(c0, acc ? kReadWrite : kWrite), Access{&ctx->red_dep, 1, kReadWrite}},
                    [=](hipStream_t st) { return rowsum_single(st, dt, 0, m, n, yp, nullptr, nullptr, op, nullptr, acc, scratch); }, 2);
        if (rc != NNT_OK) return rc;
    }
    return NNT_OK;
}

int32_t nnt_layernorm_fwd(nnt_ctx* ctx, nnt_tensor* X, nnt_tensor* gamma, nnt_tensor* beta, float eps,
                          nnt_tensor* Y, nnt_tensor* stats) {
    NNT_CHECK_CTX(ctx);
    if (!X || !gamma || !beta || !Y || !stats) return fail(ctx, NNT_EINVAL, "nnt_layernorm_fwd: null tensor");
    int32_t rc = check_ln_shapes(ctx, X, gamma, stats, "nnt_layernorm_fwd");
    if (rc != NNT_OK) return rc;
    if (!same_tiling(gamma, beta) || beta->dtype != NNT_F32 || !same_tiling(X, Y) || X->dtype != Y->dtype)
        return fail(ctx, NNT_EINVAL, "nnt_layernorm_fwd: operands tiled or typed differently");
    for (void* p : Y->tiles) if (!p) return fail(ctx, NNT_EINVAL, "nnt_layernorm_fwd: structural-zero tiles not allowed");
    for (void* p : beta->tiles) if (!p) return fail(ctx, NNT_EINVAL, "nnt_layernorm_fwd: structural-zero tiles not allowed");
    const int dtype = X->dtype;
    double numel = 1;
    for (int a = 0; a < X->ndim; a++) numel *= (double)X->shape[a];
    // one wave per token reads x once and writes y once; tile by tile x is read twice
    OpTag tag(ctx, "layernorm_fwd", numel * X->elem_size() * (ctx->granularity == NNT_GRAN_OP ? 2 : 3), true);
    if (ctx->granularity == NNT_GRAN_OP) {
        const int V = dtype == NNT_F32 ? 4 : 8;
        const bool vec = tensors_vec_ok({X, Y, gamma, beta}, V);
        const int nv = (int)(((X->base[0] + 64 * V - 1) / (64 * V)) * X->grid[0]);
        const TiledView vx = X->view(), vy = Y->view(), vs = stats->view(), vg = gamma->view(), vb = beta->view();
        const int64_t ncols = n_columns(X);
        if (ncols > INT32_MAX) return fail(ctx, NNT_EINVAL, "nnt_layernorm_fwd: tensor too large");
        std::vector<Access> acc = {X->all(kRead), gamma->all(kRead), beta->all(kRead), Y->all(kWrite), stats->all(kWrite)};
        return submit(ctx, acc, [=](hipStream_t st) {
            return dtype == NNT_F32 ? launch_ln_fwd<float>(st, vec, nv, vx, vy, vs, vg, vb, eps, ncols)
                                    : launch_ln_fwd<bf16_t>(st, vec, nv, vx, vy, vs, vg, vb, eps, ncols);
        });
    }
    // the paper's steps, tile by tile
    const int64_t g0 = X->grid[0], rest = X->ntiles / g0, N_e = X->shape[0];
    for (int64_t r = 0; r < rest; r++) {
        float* sp = static_cast<float*>(stats->tiles[r]);
        int64_t before = 0;
        for (int64_t l = 0; l < g0; l++) {
            const int64_t t = l + g0 * r, m = X->tile_extent(0, l), n = X->tile_numel(t) / m;
            const void* xp = X->tiles[t];
            const int64_t fin = l == g0 - 1 ? N_e : 0;
            rc = submit(ctx, {X->one(t, kRead), stats->one(r, l == 0 ? kWrite : kReadWrite)},
                        [=](hipStream_t st) { return nnt_tile_ln_stats(st, dtype, m, n, xp, sp, before, fin, eps); });
            if (rc != NNT_OK) return rc;
            before += m;
        }
    }
    for (int64_t t = 0; t < X->ntiles; t++) {
        const int64_t l = t % g0, r = t / g0, m = X->tile_extent(0, l), n = X->tile_numel(t) / m;
        const void* xp = X->tiles[t];
        void* yp = Y->tiles[t];
        const float* sp = static_cast<const float*>(stats->tiles[r]);
        const float* gp = static_cast<const float*>(gamma->tiles[l]);
        const float* bp = static_cast<const float*>(beta->tiles[l]);
        rc = submit(ctx, {X->one(t, kRead), stats->one(r, kRead), gamma->one(l, kRead), beta->one(l, kRead), Y->one(t, kWrite)},
                    [=](hipStream_t st) { return nnt_tile_ln_apply(st, dtype, m, n, xp, sp, gp, bp, yp); });
        if (rc != NNT_OK) return rc;
    }
    return NNT_OK;
}

int32_t nnt_layernorm_bwd(nnt_ctx* ctx, nnt_tensor* X, nnt_tensor* stats, nnt_tensor* gamma, nnt_tensor* dY,
                          nnt_tensor* dRes, nnt_tensor* dX, nnt_tensor* dgamma, nnt_tensor* dbeta) {
    NNT_CHECK_CTX(ctx);
    if (!X || !stats || !gamma || !dY || !dX || !dgamma || !dbeta) return fail(ctx, NNT_EINVAL, "nnt_layernorm_bwd: null tensor");
    int32_t rc = check_ln_shapes(ctx, X, gamma, stats, "nnt_layernorm_bwd");
    if (rc != NNT_OK) return rc;
    if (!same_tiling(X, dY) || !same_tiling(X, dX) || (dRes && !same_tiling(X, dRes)) || X->dtype != dY->dtype ||
        X->dtype != dX->dtype || (dRes && dRes->dtype != X->dtype) || !same_tiling(gamma, dgamma) || !same_tiling(gamma, dbeta) ||
        dgamma->dtype != NNT_F32 || dbeta->dtype != NNT_F32)
        return fail(ctx, NNT_EINVAL, "nnt_layernorm_bwd: operands tiled or typed differently");
    for (nnt_tensor* t : {dY, dX, dgamma, dbeta})
        for (void* p : t->tiles) if (!p) return fail(ctx, NNT_EINVAL, "nnt_layernorm_bwd: structural-zero tiles not allowed");
    if (dRes) for (void* p : dRes->tiles) if (!p) return fail(ctx, NNT_EINVAL, "nnt_layernorm_bwd: structural-zero tiles not allowed");
    const int dtype = X->dtype;
    const int64_t g0 = X->grid[0], rest = X->ntiles / g0, N_e = X->shape[0];
    double numel = 1;
    for (int a = 0; a < X->ndim; a++) numel *= (double)X->shape[a];
    // parameter gradients read x and dy; the input gradient reads x, dy (and the residual) and writes dx
    OpTag tag(ctx, "layernorm_bwd", numel * X->elem_size() * (5 + (dRes ? 1 : 0)), true);
    if (ctx->granularity == NNT_GRAN_OP) {
        const int V = dtype == NNT_F32 ? 4 : 8;
        const bool vec = tensors_vec_ok({X, dY, dX, dRes, gamma}, V);
        const int nv = (int)(((X->base[0] + 64 * V - 1) / (64 * V)) * X->grid[0]);
        const TiledView vx = X->view(), vs = stats->view(), vg = gamma->view(), vdy = dY->view(), vdx = dX->view();
        const TiledView vr = dRes ? dRes->view() : vdy;
        const int has_res = dRes != nullptr;
        const int64_t ncols = n_columns(X);
        if (ncols > INT32_MAX) return fail(ctx, NNT_EINVAL, "nnt_layernorm_bwd: tensor too large");
        std::vector<Access> acc = {X->all(kRead), stats->all(kRead), gamma->all(kRead), dY->all(kRead), dX->all(kWrite)};
        if (dRes) acc.push_back(dRes->all(kRead));
        rc = rowsum_tensor(ctx, 1, dY, X, stats, dgamma, dbeta);
        if (rc != NNT_OK) return rc;
        return submit(ctx, acc, [=](hipStream_t st) {
            return dtype == NNT_F32 ? launch_ln_bwd<float>(st, vec, nv, vx, vs, vg, vdy, vr, vdx, has_res, ncols)
                                    : launch_ln_bwd<bf16_t>(st, vec, nv, vx, vs, vg, vdy, vr, vdx, has_res, ncols);
        });
    }
    // tile by tile.  The per-token sums live in the reduction scratch: [2][columns] per group of tiles.
    int64_t max_cols = 1;
    for (int a = 1; a < X->ndim; a++) max_cols *= X->base[a];
    int64_t pmax = 0;
    for (int64_t l = 0; l < g0; l++) pmax = std::max(pmax, scratch_elems(X->tile_extent(0, l), max_cols, 1));
    rc = ensure_scratch(ctx, 2 * max_cols + pmax);
    if (rc != NNT_OK) return rc;
    float* sums = ctx->red_scratch;
    float* pscratch = ctx->red_scratch + 2 * max_cols;
    std::vector<char> seen(gamma->ntiles, 0);
    const Access scr{&ctx->red_dep, 1, kReadWrite};
    for (int64_t r = 0; r < rest; r++) {
        const float* sp = static_cast<const float*>(stats->tiles[r]);
        for (int64_t l = 0; l < g0; l++) {
            const int64_t t = l + g0 * r, m = X->tile_extent(0, l), n = X->tile_numel(t) / m;
            const void* xp = X->tiles[t];
            const void* dyp = dY->tiles[t];
            const float* gp = static_cast<const float*>(gamma->tiles[l]);
            const int init = l == 0;
            rc = submit(ctx, {X->one(t, kRead), dY->one(t, kRead), stats->one(r, kRead), gamma->one(l, kRead), scr},
                        [=](hipStream_t st) { return nnt_tile_ln_bwd_sums(st, dtype, m, n, xp, sp, gp, dyp, sums, init); });
            if (rc != NNT_OK) return rc;
        }
        for (int64_t l = 0; l < g0; l++) {
            const int64_t t = l + g0 * r, m = X->tile_extent(0, l), n = X->tile_numel(t) / m;
            const void* xp = X->tiles[t];
            const void* dyp = dY->tiles[t];
            const void* rp = dRes ? dRes->tiles[t] : nullptr;
            void* dxp = dX->tiles[t];
            const float* gp = static_cast<const float*>(gamma->tiles[l]);
            float* dgp = static_cast<float*>(dgamma->tiles[l]);
            float* dbp = static_cast<float*>(dbeta->tiles[l]);
            const int acc = seen[l];
            seen[l] = 1;
            std::vector<Access> a1 = {X->one(t, kRead), dY->one(t, kRead), stats->one(r, kRead), gamma->one(l, kRead), scr,
                                      dgamma->one(l, acc ? kReadWrite : kWrite), dbeta->one(l, acc ? kReadWrite : kWrite)};
            rc = submit(ctx, a1, [=](hipStream_t st) {
                return rowsum_single(st, dtype, 1, m, n, dyp, xp, sp, dgp, dbp, acc, pscratch);
            }, 2);
            if (rc != NNT_OK) return rc;
            std::vector<Access> a2 = {X->one(t, kRead), dY->one(t, kRead), stats->one(r, kRead), gamma->one(l, kRead), scr,
                                      dX->one(t, kWrite)};
            if (dRes) a2.push_back(dRes->one(t, kRead));
            rc = submit(ctx, a2, [=](hipStream_t st) {
                return nnt_tile_ln_bwd_dx(st, dtype, m, n, N_e, xp, sp, gp, dyp, sums, rp, dxp);
            });
            if (rc != NNT_OK) return rc;
        }
    }
    return NNT_OK;
}

}  // extern "C"
