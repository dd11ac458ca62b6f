// Device helpers shared by the memory-bound kernels: typed vector access with
// fp32 conversion, wavefront reductions, tile lookup in a tiled view.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "internal.hpp"

namespace nnt {

typedef uint16_t bf16_t;   // storage only; arithmetic is always fp32

template <typename T> struct VecOf;
template <> struct VecOf<float> { static constexpr int V = 4; };
template <> struct VecOf<bf16_t> { static constexpr int V = 8; };

__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {
    const __bf16 h = (__bf16)f;     // round to nearest even (v_cvt_pk_bf16_f32)
    return __builtin_bit_cast(bf16_t, h);
}

template <int V> __device__ __forceinline__ void ldv(const float* p, float (&f)[V]) {
    if constexpr (V == 4) {
        const float4 x = *reinterpret_cast<const float4*>(p);
        f[0] = x.x; f[1] = x.y; f[2] = x.z; f[3] = x.w;
    } else {
#pragma unroll
        for (int i = 0; i < V; i++) f[i] = p[i];
    }
}
template <int V> __device__ __forceinline__ void ldv(const bf16_t* p, float (&f)[V]) {
    if constexpr (V == 8) {
        const uint4 x = *reinterpret_cast<const uint4*>(p);
        f[0] = __uint_as_float(x.x << 16); f[1] = __uint_as_float(x.x & 0xffff0000u);
        f[2] = __uint_as_float(x.y << 16); f[3] = __uint_as_float(x.y & 0xffff0000u);
        f[4] = __uint_as_float(x.z << 16); f[5] = __uint_as_float(x.z & 0xffff0000u);
        f[6] = __uint_as_float(x.w << 16); f[7] = __uint_as_float(x.w & 0xffff0000u);
    } else {
#pragma unroll
        for (int i = 0; i < V; i++) f[i] = bf2f(p[i]);
    }
}
template <int V> __device__ __forceinline__ void stv(float* p, const float (&f)[V]) {
    if constexpr (V == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
    } else {
#pragma unroll
        for (int i = 0; i < V; i++) p[i] = f[i];
    }
}
template <int V> __device__ __forceinline__ void stv(bf16_t* p, const float (&f)[V]) {
    if constexpr (V == 8) {
        uint4 x;
        x.x = (uint32_t)f2bf(f[0]) | ((uint32_t)f2bf(f[1]) << 16);
        x.y = (uint32_t)f2bf(f[2]) | ((uint32_t)f2bf(f[3]) << 16);
        x.z = (uint32_t)f2bf(f[4]) | ((uint32_t)f2bf(f[5]) << 16);
        x.w = (uint32_t)f2bf(f[6]) | ((uint32_t)f2bf(f[7]) << 16);
        *reinterpret_cast<uint4*>(p) = x;
    } else {
#pragma unroll
        for (int i = 0; i < V; i++) p[i] = f2bf(f[i]);
    }
}

// Streaming forms for data that is touched once per launch and far larger than the caches (optimiser state):
// non-temporal loads and stores.
typedef float nt_f32x4 __attribute__((ext_vector_type(4)));
template <int V> __device__ __forceinline__ void ldv_stream(const float* p, float (&f)[V]) {
    if constexpr (V == 4) {
        const nt_f32x4 x = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x4*>(p));
        f[0] = x[0]; f[1] = x[1]; f[2] = x[2]; f[3] = x[3];
    } else {
#pragma unroll
        for (int i = 0; i < V; i++) f[i] = __builtin_nontemporal_load(p + i);
    }
}
template <int V> __device__ __forceinline__ void stv_stream(float* p, const float (&f)[V]) {
    if constexpr (V == 4) {
        const nt_f32x4 x = {f[0], f[1], f[2], f[3]};
        __builtin_nontemporal_store(x, reinterpret_cast<nt_f32x4*>(p));
    } else {
#pragma unroll
        for (int i = 0; i < V; i++) __builtin_nontemporal_store(f[i], p + i);
    }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Coordinates of tile number `tile` and its extents.
__device__ __forceinline__ void tile_geometry(const TiledView& v, int tile, int (&tc)[kMaxDim], int (&ext)[kMaxDim]) {
#pragma unroll
    for (int a = 0; a < kMaxDim; a++) {
        tc[a] = tile % v.grid[a];
        tile /= v.grid[a];
        const int lo = tc[a] * v.base[a];
        ext[a] = min(v.base[a], v.shape[a] - lo);
    }
}
__device__ __forceinline__ int64_t tile_numel(const TiledView& v, int tile) {
    int tc[kMaxDim], ext[kMaxDim];
    tile_geometry(v, tile, tc, ext);
    return (int64_t)ext[0] * ext[1] * ext[2] * ext[3];
}

// Address (in elements from the tile base) and tile number of logical element c.
__device__ __forceinline__ void locate(const TiledView& v, const int (&c)[kMaxDim], int& tile, int64_t& off) {
    tile = 0;
    off = 0;
    int tmul = 1;
    int64_t omul = 1;
#pragma unroll
    for (int a = 0; a < kMaxDim; a++) {
        const int t = c[a] / v.base[a];
        const int lo = t * v.base[a];
        const int ext = min(v.base[a], v.shape[a] - lo);
        tile += t * tmul;
        tmul *= v.grid[a];
        off += (int64_t)(c[a] - lo) * omul;
        omul *= ext;
    }
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace nnt
