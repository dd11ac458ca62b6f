// Softmax over the key axis of the attention scores (section 3, SoftMax and
// attention layer), max-shifted as in the paper.
//
// Tile form: the paper's two subroutines -- (1) per tile, the maximum and the sum
// of shifted exponentials of every column, merged into the column's running
// statistics; (2) the probabilities of a tile from the merged statistics.
// Tensor form: one wavefront per column (query, batch, head) walks the key tiles
// that the causal mask leaves visible, keeps the column in registers, and writes
// the probabilities in place: one read and one write of the scores.  Tiles with
// a NULL pointer are structural zeros (entirely masked) and are skipped.
#include "colwise.hpp"
#include "internal.hpp"

#include <algorithm>

namespace nnt {
namespace {

constexpr float kNegInf = -__builtin_huge_valf();

// e^x through the hardware's 2^x (one instruction, about 1 ulp; the library routine costs some twenty
// and made the forward kernel arithmetic-bound).  -inf gives 0.
__device__ __forceinline__ float fexp(float x) { return __builtin_amdgcn_exp2f(x * 1.4426950408889634f); }

// fn(slot, l, e, ext) over the vectors of a column whose first key index is below `kmax`.
// FLAT: the vectors of all key tiles are numbered through and dealt to the lanes 64 at a time, so a lane's
// tile differs from its neighbour's (its pointer comes out of the table per lane).  For key tiles whose
// vector count is no multiple of 64 (tiles of 400 are 50 vectors of 8 bf16: three slots of 50 lanes
// otherwise, two full ones this way).
template <int V, int NV, bool FLAT = false, typename Fn>
__device__ __forceinline__ void walk_keys(const TiledView& v, int lane, int kmax, Fn fn) {
    const int g0 = v.grid[0];
    if constexpr (FLAT) {
        static_assert(NV > 0, "the flat numbering is for columns that fit in registers");
        const int vt = v.base[0] / V;                      // vectors of a whole tile
        const float inv_vt = 1.f / (float)vt;
#pragma unroll
        for (int it = 0; it < NV; it++) {
            const int f = it * 64 + lane;
            const int l = (int)(((float)f + 0.5f) * inv_vt);   // f / vt: the half keeps the product away from an integer
            if (l < g0) {
                const int ext = ext0_of(v, l);
                const int e = (f - l * vt) * V;
                if (e < ext && l * v.base[0] + e < kmax) fn(it, l, e, ext);
            }
        }
    } else if constexpr (NV > 0) {
        const int vpt = (v.base[0] + 64 * V - 1) / (64 * V);
        int l = 0, j = 0;                 // slot it is vector j of tile l (counted up: no division per slot)
#pragma unroll
        for (int it = 0; it < NV; it++) {
            if (l < g0) {
                const int ext = ext0_of(v, l);
                const int e = (j * 64 + lane) * V;
                if (e < ext && l * v.base[0] + e < kmax) fn(it, l, e, ext);
            }
            if (++j == vpt) {
                j = 0;
                l++;
            }
        }
    } else {
        for (int l = 0; l < g0 && l * v.base[0] < kmax; l++) {
            const int ext = ext0_of(v, l);
            for (int e = lane * V; e < ext && l * v.base[0] + e < kmax; e += 64 * V) fn(0, l, e, ext);
        }
    }
}

template <typename T, int V, int NV>
__global__ void __launch_bounds__(256) softmax_fwd_fused(TiledView A, TiledView S, float scale, int causal, int64_t ncols) {
    const int lane = threadIdx.x & 63;
    const int64_t col = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: the index arithmetic below runs on the scalar unit
    if (col >= ncols) return;
    const Column c = column_of(A, col);
    const int nk = A.shape[0];
    const int kmax = causal ? min(nk, c.c1 + 1) : nk;      // keys 0 .. kmax-1 are visible to query c1
    float cache[NV > 0 ? NV : 1][V];
    float mx = kNegInf;
    float sum = 0.f;
    if constexpr (NV > 0) {
        // the column fits in registers: maximum, then shifted exponentials, from one read.  The cached
        // values are the scores in units of log 2 (scale and log2(e) folded into one factor); masked
        // entries and slots the walk does not reach end up as exact zeros, so the output pass needs no mask.
#pragma unroll
        for (int i = 0; i < NV; i++)
#pragma unroll
            for (int k = 0; k < V; k++) cache[i][k] = 0.f;
        const float sc2 = scale * 1.4426950408889634f;
        walk_keys<V, NV>(A, lane, kmax, [&](int slot, int l, int e, int ext) {
            const T* p = col_ptr<const T>(A, c, l, ext);
            float x[V];
            if (p) {
                ldv<V>(p + e, x);
            } else {
#pragma unroll
                for (int k = 0; k < V; k++) x[k] = kNegInf;
            }
            const int lim = p ? kmax - (l * A.base[0] + e) : 0;      // elements [0, lim) of the vector are visible
#pragma unroll
            for (int k = 0; k < V; k++) {
                x[k] = k < lim ? x[k] * sc2 : kNegInf;
                mx = fmaxf(mx, x[k]);
                cache[slot][k] = x[k];
            }
        });
        mx = wave_max(mx);
        walk_keys<V, NV>(A, lane, kmax, [&](int slot, int l, int e, int ext) {
#pragma unroll
            for (int k = 0; k < V; k++) {
                const float x = __builtin_amdgcn_exp2f(cache[slot][k] - mx);
                sum += x;
                cache[slot][k] = x;
            }
        });
        mx *= 0.6931471805599453f;        // back to natural units for the statistics
    } else {
        // long column: one read for both statistics -- every lane keeps a running maximum and a sum
        // of exponentials shifted by it, rescaled when its maximum moves (the merge rule of the
        // tile subroutines), and the lanes are merged the same way at the end
        walk_keys<V, NV>(A, lane, kmax, [&](int slot, int l, int e, int ext) {
            const T* p = col_ptr<const T>(A, c, l, ext);
            if (!p) return;
            float x[V];
            ldv<V>(p + e, x);
            const int k0 = l * A.base[0] + e;
            float vm = kNegInf;
#pragma unroll
            for (int k = 0; k < V; k++) {
                x[k] = (k0 + k < kmax) ? x[k] * scale : kNegInf;
                vm = fmaxf(vm, x[k]);
            }
            if (vm == kNegInf) return;
            const float m_new = fmaxf(mx, vm);
            float part = 0.f;
#pragma unroll
            for (int k = 0; k < V; k++) part += fexp(x[k] - m_new);
            sum = sum * fexp(mx - m_new) + part;        // exp(-inf) = 0 the first time
            mx = m_new;
        });
        const float lane_mx = mx;
        mx = wave_max(mx);
        sum *= (lane_mx == kNegInf) ? 0.f : fexp(lane_mx - mx);
    }
    sum = wave_sum(sum);
    const float inv = 1.f / sum;
    // every vector of every present tile is written: masked entries become 0
    walk_keys<V, NV>(A, lane, nk, [&](int slot, int l, int e, int ext) {
        T* p = col_ptr<T>(A, c, l, ext);
        if (!p) return;
        const int k0 = l * A.base[0] + e;
        float x[V];
        if constexpr (NV > 0) {
#pragma unroll
            for (int k = 0; k < V; k++) x[k] = cache[slot][k] * inv;
        } else if (k0 >= kmax) {
#pragma unroll
            for (int k = 0; k < V; k++) x[k] = 0.f;
        } else {
            ldv<V>(p + e, x);
#pragma unroll
            for (int k = 0; k < V; k++) x[k] = (k0 + k < kmax) ? fexp(x[k] * scale - mx) * inv : 0.f;
        }
        stv<V>(p + e, x);
    });
    if (lane == 0) {
        float* s = static_cast<float*>(S.tiles[c.stat_tile]) + 2 * (int64_t)c.colidx;
        s[0] = mx;
        s[1] = sum;
    }
}

template <typename T, int V, int NV>
__global__ void __launch_bounds__(256) softmax_bwd_fused(TiledView P, TiledView dP, int64_t ncols) {
    const int lane = threadIdx.x & 63;
    const int64_t col = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: the index arithmetic below runs on the scalar unit
    if (col >= ncols) return;
    const Column c = column_of(P, col);
    const int nk = P.shape[0];
    float cp[NV > 0 ? NV : 1][V], cd[NV > 0 ? NV : 1][V];
    float dot = 0.f;
    walk_keys<V, NV>(P, lane, nk, [&](int slot, int l, int e, int ext) {
        const T* p = col_ptr<const T>(P, c, l, ext);
        float x[V], d[V];
        if (p) {
            ldv<V>(p + e, x);
            ldv<V>(col_ptr<const T>(dP, c, l, ext) + e, d);
        } else {
#pragma unroll
            for (int k = 0; k < V; k++) x[k] = d[k] = 0.f;
        }
#pragma unroll
        for (int k = 0; k < V; k++) {
            dot += x[k] * d[k];
            if constexpr (NV > 0) { cp[slot][k] = x[k]; cd[slot][k] = d[k]; }
        }
    });
    dot = wave_sum(dot);
    walk_keys<V, NV>(P, lane, nk, [&](int slot, int l, int e, int ext) {
        T* q = col_ptr<T>(dP, c, l, ext);
        if (!q) return;
        float x[V], d[V];
        if constexpr (NV > 0) {
#pragma unroll
            for (int k = 0; k < V; k++) { x[k] = cp[slot][k]; d[k] = cd[slot][k]; }
        } else {
            ldv<V>(col_ptr<const T>(P, c, l, ext) + e, x);
            ldv<V>(q + e, d);
        }
#pragma unroll
        for (int k = 0; k < V; k++) d[k] = x[k] * (d[k] - dot);
        stv<V>(q + e, d);
    });
}

// ------------------------------------------------------------------ several columns per wavefront
// The same two kernels for CPW consecutive columns (queries) per wavefront, for columns that fit in
// registers.  The host only picks them when groups of CPW queries never straddle a tile (extent and base
// tile of the query axis are multiples of CPW), so the columns of a wave share their tile pointers and
// differ by one column pitch: the look-up of the tiles is paid once per CPW columns, and the loads of
// all of them are in flight together.  Short columns in a narrow type (1024 bf16 keys are 2 KB) are
// otherwise bound by that look-up and by the latency of a single round of loads.
template <typename T, int V, int NV, int CPW, bool FLAT = false>
__global__ void __launch_bounds__(256) softmax_fwd_multi(TiledView A, TiledView S, float scale, int causal, int64_t ncols) {
    const int lane = threadIdx.x & 63;
    const int64_t col = ((int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6)) * CPW;
    if (col >= ncols) return;
    const Column c = column_of(A, col);
    const int nk = A.shape[0];
    const int kmax_last = causal ? min(nk, c.c1 + CPW) : nk;      // visible keys of the wave's last column
    const float sc2 = scale * 1.4426950408889634f;
    float cache[CPW][NV][V];
    float mx[CPW], sum[CPW];
#pragma unroll
    for (int q = 0; q < CPW; q++) {
        mx[q] = kNegInf;
        sum[q] = 0.f;
#pragma unroll
        for (int i = 0; i < NV; i++)
#pragma unroll
            for (int k = 0; k < V; k++) cache[q][i][k] = 0.f;
    }
    walk_keys<V, NV, FLAT>(A, lane, kmax_last, [&](int slot, int l, int e, int ext) {
        const T* p = col_ptr<const T>(A, c, l, ext);
        const int k0 = l * A.base[0] + e;
#pragma unroll
        for (int q = 0; q < CPW; q++) {
            const int kmax = causal ? min(nk, c.c1 + q + 1) : nk;
            const int lim = p ? kmax - k0 : 0;                     // elements [0, lim) of the vector are visible to column q
            float x[V];
            if (lim > 0) {
                ldv<V>(p + (int64_t)q * ext + e, x);
            } else {
#pragma unroll
                for (int k = 0; k < V; k++) x[k] = kNegInf;
            }
#pragma unroll
            for (int k = 0; k < V; k++) {
                x[k] = k < lim ? x[k] * sc2 : kNegInf;
                mx[q] = fmaxf(mx[q], x[k]);
                cache[q][slot][k] = x[k];
            }
        }
    });
#pragma unroll
    for (int q = 0; q < CPW; q++) mx[q] = wave_max(mx[q]);
    // shifted exponentials: the walk visits exactly the slots that were loaded (masked entries are -inf -> 0;
    // slots it does not reach keep their 0)
    walk_keys<V, NV, FLAT>(A, lane, kmax_last, [&](int slot, int l, int e, int ext) {
#pragma unroll
        for (int q = 0; q < CPW; q++)
#pragma unroll
            for (int k = 0; k < V; k++) {
                const float x = __builtin_amdgcn_exp2f(cache[q][slot][k] - mx[q]);
                sum[q] += x;
                cache[q][slot][k] = x;
            }
    });
    float inv[CPW];
#pragma unroll
    for (int q = 0; q < CPW; q++) {
        sum[q] = wave_sum(sum[q]);
        inv[q] = 1.f / sum[q];
    }
    // every vector of every present tile is written: masked entries (and slots never loaded) are 0
    walk_keys<V, NV, FLAT>(A, lane, nk, [&](int slot, int l, int e, int ext) {
        T* p = col_ptr<T>(A, c, l, ext);
        if (!p) return;
#pragma unroll
        for (int q = 0; q < CPW; q++) {
            float x[V];
#pragma unroll
            for (int k = 0; k < V; k++) x[k] = cache[q][slot][k] * inv[q];
            stv<V>(p + (int64_t)q * ext + e, x);
        }
    });
    if (lane < CPW) {
        float* s = static_cast<float*>(S.tiles[c.stat_tile]) + 2 * (int64_t)(c.colidx + lane);
        float m = mx[0], d = sum[0];
#pragma unroll
        for (int q = 1; q < CPW; q++)
            if (lane == q) { m = mx[q]; d = sum[q]; }
        s[0] = m * 0.6931471805599453f;       // back to natural units
        s[1] = d;
    }
}

template <typename T, int V, int NV, int CPW, bool FLAT = false>
__global__ void __launch_bounds__(256) softmax_bwd_multi(TiledView P, TiledView dP, int64_t ncols) {
    const int lane = threadIdx.x & 63;
    const int64_t col = ((int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6)) * CPW;
    if (col >= ncols) return;
    const Column c = column_of(P, col);
    const int nk = P.shape[0];
    float cp[CPW][NV][V], cd[CPW][NV][V];
    float dot[CPW];
#pragma unroll
    for (int q = 0; q < CPW; q++) dot[q] = 0.f;
    walk_keys<V, NV, FLAT>(P, lane, nk, [&](int slot, int l, int e, int ext) {
        const T* p = col_ptr<const T>(P, c, l, ext);
        const T* d = col_ptr<const T>(dP, c, l, ext);
#pragma unroll
        for (int q = 0; q < CPW; q++) {
            float x[V], y[V];
            if (p) {
                ldv<V>(p + (int64_t)q * ext + e, x);
                ldv<V>(d + (int64_t)q * ext + e, y);
            } else {
#pragma unroll
                for (int k = 0; k < V; k++) x[k] = y[k] = 0.f;
            }
#pragma unroll
            for (int k = 0; k < V; k++) {
                dot[q] += x[k] * y[k];
                cp[q][slot][k] = x[k];
                cd[q][slot][k] = y[k];
            }
        }
    });
#pragma unroll
    for (int q = 0; q < CPW; q++) dot[q] = wave_sum(dot[q]);
    walk_keys<V, NV, FLAT>(P, lane, nk, [&](int slot, int l, int e, int ext) {
        T* d = col_ptr<T>(dP, c, l, ext);
        if (!d) return;
#pragma unroll
        for (int q = 0; q < CPW; q++) {
            float y[V];
#pragma unroll
            for (int k = 0; k < V; k++) y[k] = cp[q][slot][k] * (cd[q][slot][k] - dot[q]);
            stv<V>(d + (int64_t)q * ext + e, y);
        }
    });
}

// ------------------------------------------------------------------ tile form: one wave per column of a tk x ncol tile
template <typename T, int V>
__global__ void __launch_bounds__(256) softmax_stats_tile(const T* a, float* stats, int tk, int tq, int64_t ncol, int k0, int q0,
                                                          int causal, float scale, int init) {
    const int lane = threadIdx.x & 63;
    const int64_t col = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: the index arithmetic below runs on the scalar unit
    if (col >= ncol) return;
    const int q = q0 + (int)(col % tq);
    const int kvis = causal ? min(tk, q + 1 - k0) : tk;     // rows of this tile visible to q (may be <= 0)
    const T* p = a + col * tk;
    float mx = kNegInf;
    for (int e = lane * V; e < kvis; e += 64 * V) {
        float x[V];
        ldv<V>(p + e, x);
#pragma unroll
        for (int k = 0; k < V; k++)
            if (e + k < kvis) mx = fmaxf(mx, x[k] * scale);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int e = lane * V; e < kvis; e += 64 * V) {
        float x[V];
        ldv<V>(p + e, x);
#pragma unroll
        for (int k = 0; k < V; k++)
            if (e + k < kvis) sum += fexp(x[k] * scale - mx);
    }
    sum = wave_sum(sum);
    if (lane == 0) {
        float m_old = kNegInf, s_old = 0.f;
        if (!init) { m_old = stats[2 * col]; s_old = stats[2 * col + 1]; }
        const float m_new = fmaxf(m_old, mx);
        float s_new = 0.f;
        if (m_new > kNegInf) {
            if (m_old > kNegInf) s_new += s_old * fexp(m_old - m_new);
            if (mx > kNegInf) s_new += sum * fexp(mx - m_new);
        }
        stats[2 * col] = m_new;
        stats[2 * col + 1] = s_new;
    }
}

template <typename T, int V>
__global__ void __launch_bounds__(256) softmax_apply_tile(T* a, const float* stats, int tk, int tq, int64_t ncol, int k0, int q0,
                                                          int causal, float scale) {
    const int lane = threadIdx.x & 63;
    const int64_t col = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: the index arithmetic below runs on the scalar unit
    if (col >= ncol) return;
    const int q = q0 + (int)(col % tq);
    const int kvis = causal ? min(tk, q + 1 - k0) : tk;
    const float mx = stats[2 * col], inv = 1.f / stats[2 * col + 1];
    T* p = a + col * tk;
    for (int e = lane * V; e < tk; e += 64 * V) {
        float x[V];
        ldv<V>(p + e, x);
#pragma unroll
        for (int k = 0; k < V; k++) x[k] = (e + k < kvis) ? fexp(x[k] * scale - mx) * inv : 0.f;
        stv<V>(p + e, x);
    }
}

template <typename T, int V>
__global__ void __launch_bounds__(256) softmax_bwd_dot_tile(const T* p, const T* dp, float* dots, int tk, int64_t ncol, int init) {
    const int lane = threadIdx.x & 63;
    const int64_t col = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: the index arithmetic below runs on the scalar unit
    if (col >= ncol) return;
    float dot = 0.f;
    for (int e = lane * V; e < tk; e += 64 * V) {
        float x[V], d[V];
        ldv<V>(p + col * tk + e, x);
        ldv<V>(dp + col * tk + e, d);
#pragma unroll
        for (int k = 0; k < V; k++) dot += x[k] * d[k];
    }
    dot = wave_sum(dot);
    if (lane == 0) dots[col] = init ? dot : dots[col] + dot;
}

template <typename T, int V>
__global__ void __launch_bounds__(256) softmax_bwd_apply_tile(const T* p, T* dp, const float* dots, int tk, int64_t ncol) {
    const int lane = threadIdx.x & 63;
    const int64_t col = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform: the index arithmetic below runs on the scalar unit
    if (col >= ncol) return;
    const float dot = dots[col];
    for (int e = lane * V; e < tk; e += 64 * V) {
        float x[V], d[V];
        ldv<V>(p + col * tk + e, x);
        ldv<V>(dp + col * tk + e, d);
#pragma unroll
        for (int k = 0; k < V; k++) d[k] = x[k] * (d[k] - dot);
        stv<V>(dp + col * tk + e, d);
    }
}

bool vec_ok_tensor(const nnt_tensor* t, int V) {
    if (t->base[0] % V != 0 || t->shape[0] % V != 0) return false;
    for (void* p : t->tiles)
        if (p && !aligned16(p)) return false;
    return true;
}

}  // namespace
}  // namespace nnt

using namespace nnt;

#define DT_OK(d) ((d) == NNT_F32 || (d) == NNT_BF16)
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
// fused kernels: NV is the number of cached vectors per lane
#define DISPATCH_TVN(dtype, vec, nv, KERNEL, ...)                                                      \
    do {                                                                                               \
        if ((dtype) == NNT_F32) {                                                                      \
            if (!(vec)) hipLaunchKernelGGL((KERNEL<float, 1, 0>), grid, block, 0, st, __VA_ARGS__);    \
            else if ((nv) <= 4) hipLaunchKernelGGL((KERNEL<float, 4, 4>), grid, block, 0, st, __VA_ARGS__);   \
            else if ((nv) <= 8) hipLaunchKernelGGL((KERNEL<float, 4, 8>), grid, block, 0, st, __VA_ARGS__);   \
            else hipLaunchKernelGGL((KERNEL<float, 4, 0>), grid, block, 0, st, __VA_ARGS__);           \
        } else {                                                                                       \
            if (!(vec)) hipLaunchKernelGGL((KERNEL<bf16_t, 1, 0>), grid, block, 0, st, __VA_ARGS__);   \
            else if ((nv) <= 2) hipLaunchKernelGGL((KERNEL<bf16_t, 8, 2>), grid, block, 0, st, __VA_ARGS__);  \
            else if ((nv) <= 8) hipLaunchKernelGGL((KERNEL<bf16_t, 8, 8>), grid, block, 0, st, __VA_ARGS__);  \
            else hipLaunchKernelGGL((KERNEL<bf16_t, 8, 0>), grid, block, 0, st, __VA_ARGS__);          \
        }                                                                                              \
    } while (0)

// Columns per wavefront of the tensor-level kernels: several when the column fits a small register cache
// and groups of that many queries never straddle a tile of the query axis; DISPATCH_MULTI launches the
// instance for what columns_per_wave returned.
// (The adjoint keeps two register caches per column: it takes two columns per wavefront in bf16 and stays at
// one in fp32, where more measured slower.)
static inline int columns_per_wave(const nnt_tensor* A, bool vec, int nv, bool adjoint) {
    if (!vec || nv > 4 || A->ndim < 2) return 1;
    int want;
    if (adjoint) want = A->dtype == NNT_F32 ? 1 : 2;
    else want = A->dtype == NNT_F32 ? 2 : (nv <= 2 ? 4 : 2);
    return (A->shape[1] % want == 0 && A->base[1] % want == 0) ? want : 1;
}
// Slots of the flat numbering (all vectors of a column, 64 per slot), or 0 when it saves nothing over the
// numbering by tile or the column does not fit four slots.
static inline int flat_slots(const nnt_tensor* A, bool vec, int nv_by_tile) {
    const int V = A->dtype == NNT_F32 ? 4 : 8;
    if (!vec || A->grid[0] < 2 || (A->base[0] / V) % 64 == 0) return 0;
    const int nv = (int)((A->shape[0] / V + 63) / 64);
    return (nv <= 4 && nv < nv_by_tile) ? nv : 0;
}
#define DISPATCH_MULTI(dtype, nv, cpw, KERNEL, ...)                                                        \
    do {                                                                                                   \
        if ((dtype) == NNT_F32) hipLaunchKernelGGL((KERNEL<float, 4, 4, 2>), grid, block, 0, st, __VA_ARGS__);            \
        else if ((nv) <= 2 && (cpw) == 4) hipLaunchKernelGGL((KERNEL<bf16_t, 8, 2, 4>), grid, block, 0, st, __VA_ARGS__); \
        else if ((nv) <= 2) hipLaunchKernelGGL((KERNEL<bf16_t, 8, 2, 2>), grid, block, 0, st, __VA_ARGS__);               \
        else hipLaunchKernelGGL((KERNEL<bf16_t, 8, 4, 2>), grid, block, 0, st, __VA_ARGS__);                             \
    } while (0)
// the same with the flat numbering (also for one column per wavefront: the fp32 adjoint)
#define DISPATCH_FLAT(dtype, nv, cpw, KERNEL, ...)                                                                        \
    do {                                                                                                                  \
        if ((dtype) == NNT_F32 && (cpw) == 2) hipLaunchKernelGGL((KERNEL<float, 4, 4, 2, true>), grid, block, 0, st, __VA_ARGS__);      \
        else if ((dtype) == NNT_F32) hipLaunchKernelGGL((KERNEL<float, 4, 4, 1, true>), grid, block, 0, st, __VA_ARGS__);                \
        else if ((nv) <= 2 && (cpw) == 4) hipLaunchKernelGGL((KERNEL<bf16_t, 8, 2, 4, true>), grid, block, 0, st, __VA_ARGS__);          \
        else if ((nv) <= 2 && (cpw) == 2) hipLaunchKernelGGL((KERNEL<bf16_t, 8, 2, 2, true>), grid, block, 0, st, __VA_ARGS__);          \
        else if ((cpw) == 2) hipLaunchKernelGGL((KERNEL<bf16_t, 8, 4, 2, true>), grid, block, 0, st, __VA_ARGS__);                       \
        else hipLaunchKernelGGL((KERNEL<bf16_t, 8, 4, 1, true>), grid, block, 0, st, __VA_ARGS__);                                       \
    } while (0)

static inline bool sm_ok(int64_t tk, int64_t tq, int64_t batch) {
    return tk >= 1 && tq >= 1 && batch >= 0 && tk <= INT32_MAX && tq <= INT32_MAX && tq * batch <= (int64_t)INT32_MAX * 4;
}

extern "C" {

int32_t nnt_tile_softmax_stats(void* stream, int32_t dtype, int64_t tk, int64_t tq, int64_t batch, int64_t k0, int64_t q0,
                               int32_t causal, float scale, const void* a, float* stats, int32_t init) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (!sm_ok(tk, tq, batch) || k0 < 0 || q0 < 0 || k0 > INT32_MAX || q0 > INT32_MAX) return NNT_EINVAL;
    const int64_t ncol = tq * batch;
    if (ncol == 0) return NNT_OK;
    if (!a || !stats) return NNT_EINVAL;
    const bool vec = aligned16(a) && tk % (dtype == NNT_F32 ? 4 : 8) == 0;
    const dim3 grid((unsigned)((ncol + 3) / 4)), block(256);
    DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((softmax_stats_tile<T, V>), grid, block, 0, (hipStream_t)stream, (const T*)a, stats,
                                               (int)tk, (int)tq, ncol, (int)k0, (int)q0, (int)causal, scale, (int)init));
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int32_t nnt_tile_softmax_apply(void* stream, int32_t dtype, int64_t tk, int64_t tq, int64_t batch, int64_t k0, int64_t q0,
                               int32_t causal, float scale, void* a, const float* stats) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (!sm_ok(tk, tq, batch) || k0 < 0 || q0 < 0 || k0 > INT32_MAX || q0 > INT32_MAX) return NNT_EINVAL;
    const int64_t ncol = tq * batch;
    if (ncol == 0) return NNT_OK;
    if (!a || !stats) return NNT_EINVAL;
    const bool vec = aligned16(a) && tk % (dtype == NNT_F32 ? 4 : 8) == 0;
    const dim3 grid((unsigned)((ncol + 3) / 4)), block(256);
    DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((softmax_apply_tile<T, V>), grid, block, 0, (hipStream_t)stream, (T*)a, stats,
                                               (int)tk, (int)tq, ncol, (int)k0, (int)q0, (int)causal, scale));
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int32_t nnt_tile_softmax_bwd_dot(void* stream, int32_t dtype, int64_t tk, int64_t tq, int64_t batch, const void* p,
                                 const void* dp, float* dots, int32_t init) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (!sm_ok(tk, tq, batch)) return NNT_EINVAL;
    const int64_t ncol = tq * batch;
    if (ncol == 0) return NNT_OK;
    if (!p || !dp || !dots) return NNT_EINVAL;
    const bool vec = aligned16(p) && aligned16(dp) && tk % (dtype == NNT_F32 ? 4 : 8) == 0;
    const dim3 grid((unsigned)((ncol + 3) / 4)), block(256);
    DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((softmax_bwd_dot_tile<T, V>), grid, block, 0, (hipStream_t)stream, (const T*)p,
                                               (const T*)dp, dots, (int)tk, ncol, (int)init));
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int32_t nnt_tile_softmax_bwd_apply(void* stream, int32_t dtype, int64_t tk, int64_t tq, int64_t batch, const void* p,
                                   void* dp, const float* dots) {
    if (!DT_OK(dtype)) return NNT_EDTYPE;
    if (!sm_ok(tk, tq, batch)) return NNT_EINVAL;
    const int64_t ncol = tq * batch;
    if (ncol == 0) return NNT_OK;
    if (!p || !dp || !dots) return NNT_EINVAL;
    const bool vec = aligned16(p) && aligned16(dp) && tk % (dtype == NNT_F32 ? 4 : 8) == 0;
    const dim3 grid((unsigned)((ncol + 3) / 4)), block(256);
    DISPATCH_TV(dtype, vec, hipLaunchKernelGGL((softmax_bwd_apply_tile<T, V>), grid, block, 0, (hipStream_t)stream, (const T*)p,
                                               (T*)dp, dots, (int)tk, ncol));
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

// ------------------------------------------------------------------ tensor form
static int32_t check_sm(nnt_ctx* ctx, const nnt_tensor* A, const nnt_tensor* stats, int nstat, const char* who) {
    if (A->ndim < 2) return fail(ctx, NNT_EINVAL, std::string(who) + ": scores need at least 2 axes");
    if (stats) {
        if (stats->dtype != NNT_F32 || stats->ndim != A->ndim || stats->shape[0] != nstat || stats->base[0] != nstat)
            return fail(ctx, NNT_EINVAL, std::string(who) + ": stats must be fp32 with an untiled first axis");
        for (int a = 1; a < A->ndim; a++)
            if (stats->shape[a] != A->shape[a] || stats->base[a] != A->base[a])
                return fail(ctx, NNT_EINVAL, std::string(who) + ": stats must be tiled like the scores' other axes");
        for (void* p : stats->tiles) if (!p) return fail(ctx, NNT_EINVAL, std::string(who) + ": stats tile missing");
    }
    return NNT_OK;
}

int32_t nnt_softmax_fwd(nnt_ctx* ctx, nnt_tensor* A, nnt_tensor* stats, float scale, int32_t causal) {
    NNT_CHECK_CTX(ctx);
    if (!A || !stats) return fail(ctx, NNT_EINVAL, "nnt_softmax_fwd: null tensor");
    int32_t rc = check_sm(ctx, A, stats, 2, "nnt_softmax_fwd");
    if (rc != NNT_OK) return rc;
    const int64_t g0 = A->grid[0], rest = A->ntiles / g0;
    // a NULL tile must be one that the causal mask removes entirely
    for (int64_t t = 0; t < A->ntiles; t++) {
        if (A->tiles[t]) continue;
        int64_t c[kMaxDim];
        A->tile_coords(t, c);
        const int64_t kfirst = c[0] * A->base[0];
        const int64_t qlast = c[1] * A->base[1] + A->tile_extent(1, c[1]) - 1;
        if (!causal || kfirst <= qlast) return fail(ctx, NNT_EINVAL, "nnt_softmax_fwd: a missing tile holds visible scores");
    }
    const int dtype = A->dtype;
    double present = 0;
    for (int64_t t = 0; t < A->ntiles; t++)
        if (A->tiles[t]) present += (double)A->tile_numel(t);
    // in place: the scores of every present tile are read once and written once (read twice tile by tile)
    OpTag tag(ctx, "softmax_fwd", present * A->elem_size() * (ctx->granularity == NNT_GRAN_OP ? 2 : 3), true);
    if (ctx->granularity == NNT_GRAN_OP) {
        const int V = dtype == NNT_F32 ? 4 : 8;
        const bool vec = vec_ok_tensor(A, V);
        const int nv = (int)(((A->base[0] + 64 * V - 1) / (64 * V)) * g0);
        const TiledView va = A->view(), vs = stats->view();
        const int64_t ncols = n_columns(A);
        if (ncols > INT32_MAX) return fail(ctx, NNT_EINVAL, "nnt_softmax_fwd: tensor too large");
        const int nvf = flat_slots(A, vec, nv);
        const int cpw = columns_per_wave(A, vec, nvf ? nvf : nv, false);
        return submit(ctx, {A->all(kReadWrite), stats->all(kWrite)}, [=](hipStream_t st) {
            const dim3 grid((unsigned)((ncols / cpw + 3) / 4)), block(256);
            if (nvf) DISPATCH_FLAT(dtype, nvf, cpw, softmax_fwd_multi, va, vs, scale, (int)causal, ncols);
            else if (cpw > 1) DISPATCH_MULTI(dtype, nv, cpw, softmax_fwd_multi, va, vs, scale, (int)causal, ncols);
            else DISPATCH_TVN(dtype, vec, nv, softmax_fwd_fused, va, vs, scale, (int)causal, ncols);
            return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
        });
    }
    // the paper's two subroutines, tile by tile
    for (int pass = 0; pass < 2; pass++) {
        for (int64_t r = 0; r < rest; r++) {
            bool first = true;
            for (int64_t l = 0; l < g0; l++) {
                const int64_t t = l + g0 * r;
                if (!A->tiles[t]) continue;
                int64_t c[kMaxDim];
                A->tile_coords(t, c);
                const int64_t tk = A->tile_extent(0, c[0]), tq = A->tile_extent(1, c[1]);
                const int64_t batch = A->tile_numel(t) / (tk * tq);
                const int64_t k0 = c[0] * A->base[0], q0 = c[1] * A->base[1];
                void* ap = A->tiles[t];
                float* sp = static_cast<float*>(stats->tiles[r]);
                if (pass == 0) {
                    const int init = first;
                    rc = submit(ctx, {A->one(t, kRead), stats->one(r, init ? kWrite : kReadWrite)}, [=](hipStream_t st) {
                        return nnt_tile_softmax_stats(st, dtype, tk, tq, batch, k0, q0, causal, scale, ap, sp, init);
                    });
                } else {
                    rc = submit(ctx, {A->one(t, kReadWrite), stats->one(r, kRead)}, [=](hipStream_t st) {
                        return nnt_tile_softmax_apply(st, dtype, tk, tq, batch, k0, q0, causal, scale, ap, sp);
                    });
                }
                if (rc != NNT_OK) return rc;
                first = false;
            }
        }
    }
    return NNT_OK;
}

int32_t nnt_softmax_bwd(nnt_ctx* ctx, nnt_tensor* P, nnt_tensor* dP) {
    NNT_CHECK_CTX(ctx);
    if (!P || !dP) return fail(ctx, NNT_EINVAL, "nnt_softmax_bwd: null tensor");
    int32_t rc = check_sm(ctx, P, nullptr, 0, "nnt_softmax_bwd");
    if (rc != NNT_OK) return rc;
    if (!same_tiling(P, dP) || !null_alike(P, dP) || P->dtype != dP->dtype)
        return fail(ctx, NNT_EINVAL, "nnt_softmax_bwd: operands tiled or typed differently");
    const int dtype = P->dtype;
    const int64_t g0 = P->grid[0], rest = P->ntiles / g0;
    double present = 0;
    for (int64_t t = 0; t < P->ntiles; t++)
        if (P->tiles[t]) present += (double)P->tile_numel(t);
    OpTag tag(ctx, "softmax_bwd", present * P->elem_size() * (ctx->granularity == NNT_GRAN_OP ? 3 : 5), true);
    if (ctx->granularity == NNT_GRAN_OP) {
        const int V = dtype == NNT_F32 ? 4 : 8;
        const bool vec = vec_ok_tensor(P, V) && vec_ok_tensor(dP, V);
        const int nv = (int)(((P->base[0] + 64 * V - 1) / (64 * V)) * g0);
        const TiledView vp = P->view(), vd = dP->view();
        const int64_t ncols = n_columns(P);
        if (ncols > INT32_MAX) return fail(ctx, NNT_EINVAL, "nnt_softmax_bwd: tensor too large");
        const int nvf = flat_slots(P, vec, nv);
        const int cpw = columns_per_wave(P, vec, nvf ? nvf : nv, true);
        return submit(ctx, {P->all(kRead), dP->all(kReadWrite)}, [=](hipStream_t st) {
            const dim3 grid((unsigned)((ncols / cpw + 3) / 4)), block(256);
            if (nvf) DISPATCH_FLAT(dtype, nvf, cpw, softmax_bwd_multi, vp, vd, ncols);
            else if (cpw > 1) DISPATCH_MULTI(dtype, nv, cpw, softmax_bwd_multi, vp, vd, ncols);
            else DISPATCH_TVN(dtype, vec, nv, softmax_bwd_fused, vp, vd, ncols);
            return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
        });
    }
    int64_t max_cols = 1;
    for (int a = 1; a < P->ndim; a++) max_cols *= P->base[a];
    rc = ensure_scratch(ctx, max_cols);
    if (rc != NNT_OK) return rc;
    float* dots = ctx->red_scratch;
    const Access scr{&ctx->red_dep, 1, kReadWrite};
    for (int64_t r = 0; r < rest; r++) {
        for (int pass = 0; pass < 2; pass++) {
            bool first = true;
            for (int64_t l = 0; l < g0; l++) {
                const int64_t t = l + g0 * r;
                if (!P->tiles[t]) continue;
                int64_t c[kMaxDim];
                P->tile_coords(t, c);
                const int64_t tk = P->tile_extent(0, c[0]), tq = P->tile_extent(1, c[1]);
                const int64_t batch = P->tile_numel(t) / (tk * tq);
                const void* pp = P->tiles[t];
                void* dp = dP->tiles[t];
                if (pass == 0) {
                    const int init = first;
                    rc = submit(ctx, {P->one(t, kRead), dP->one(t, kRead), scr}, [=](hipStream_t st) {
                        return nnt_tile_softmax_bwd_dot(st, dtype, tk, tq, batch, pp, dp, dots, init);
                    });
                } else {
                    rc = submit(ctx, {P->one(t, kRead), dP->one(t, kReadWrite), scr}, [=](hipStream_t st) {
                        return nnt_tile_softmax_bwd_apply(st, dtype, tk, tq, batch, pp, dp, dots);
                    });
                }
                if (rc != NNT_OK) return rc;
                first = false;
            }
        }
    }
    return NNT_OK;
}

}  // extern "C"
