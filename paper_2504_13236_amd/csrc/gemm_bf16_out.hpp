// Result path shared by the bf16 product kernels: a wave's block of fp32 accumulators goes
// through LDS and leaves as 16-byte vectors along m, the contiguous index of a C tile.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nnt {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// A pointer that is the same in every lane, moved to scalar registers.
template <typename T>
__device__ __forceinline__ const T* uniform_ptr(const T* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const T*>(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ void store_out(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_out(uint16_t* p, float v) {
    const __bf16 h = (__bf16)v;
    *p = __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ float load_out(const float* p) { return *p; }
__device__ __forceinline__ float load_out(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Writes one wave's (32 WMB) x (32 WNB) block of C = alpha * acc + bias + beta * C[+ cin_off].  `stage` is
// 32 rows of 32 WMB + 4 floats of LDS owned by the wave; every wave of the workgroup must call
// this (it synchronises the workgroup between the passes).  Vector stores need a 16-byte
// aligned tile and leading dimension; anything else, and the ragged edge, goes element by element.
template <typename TO, int WMB, int WNB>
__device__ __forceinline__ void write_tile(float* stage, const f32x16 (&acc)[WNB][WMB], TO* C, int64_t ldc,
                                           const float* bias, float alpha, float beta, int m_base, int n_base,
                                           int m_lim, int n_lim, int lane, int64_t cin_off = 0) {
    constexpr int MW = 32 * WMB, ROW = MW + 4;
    constexpr int V = 16 / (int)sizeof(TO);          // elements per 16-byte store
    constexpr int CH = MW / V, RPI = 64 / CH;        // vectors per row, rows per pass of the wave
    static_assert(CH <= 64 && 32 % RPI == 0, "row shape");
    const int r32 = lane & 31, half = lane >> 5;
    // (the beta term comes from C + cin_off: the tile itself, or the tile of a residual input with the same geometry)
    const bool vec_ok = (reinterpret_cast<uintptr_t>(C) % 16 == 0) && (ldc % V == 0) && (cin_off % V == 0);
#pragma unroll
    for (int bn = 0; bn < WNB; bn++) {
#pragma unroll
        for (int bm = 0; bm < WMB; bm++)
#pragma unroll
            for (int q = 0; q < 4; q++) {
                f32x4 v;
                v[0] = alpha * acc[bn][bm][4 * q];
                v[1] = alpha * acc[bn][bm][4 * q + 1];
                v[2] = alpha * acc[bn][bm][4 * q + 2];
                v[3] = alpha * acc[bn][bm][4 * q + 3];
                *reinterpret_cast<f32x4*>(&stage[r32 * ROW + bm * 32 + 8 * q + 4 * half]) = v;
            }
        __syncthreads();
        // the beta term (C itself, or a residual input's tile behind cin_off) of every row of this pass is
        // asked for before the pass's first store: a load placed after a store to what may be the same
        // tile waits for that store
        constexpr int NIT = 32 / RPI;
        uint4 cin[NIT];
        if (beta != 0.f && vec_ok) {
#pragma unroll
            for (int it = 0; it < NIT; it++) {
                const int row = it * RPI + lane / CH, mc = (lane % CH) * V;
                const int gn = n_base + bn * 32 + row, gm = m_base + mc;
                cin[it] = make_uint4(0u, 0u, 0u, 0u);
                if (gn < n_lim && gm + V <= m_lim) cin[it] = *reinterpret_cast<const uint4*>(C + gm + (int64_t)gn * ldc + cin_off);
            }
        }
#pragma unroll
        for (int it = 0; it < NIT; it++) {
            const int row = it * RPI + lane / CH, mc = (lane % CH) * V;
            float v[V];
#pragma unroll
            for (int j = 0; j < V; j += 4) {
                const f32x4 x = *reinterpret_cast<const f32x4*>(&stage[row * ROW + mc + j]);
                v[j] = x[0]; v[j + 1] = x[1]; v[j + 2] = x[2]; v[j + 3] = x[3];
            }
            const int gn = n_base + bn * 32 + row, gm = m_base + mc;
            if (gn < n_lim && gm < m_lim) {
                TO* p = C + gm + (int64_t)gn * ldc;
                if (vec_ok && gm + V <= m_lim) {
                    if (bias) {
#pragma unroll
                        for (int j = 0; j < V; j += 4) {
                            const f32x4 bv = *reinterpret_cast<const f32x4*>(bias + gm + j);
                            v[j] += bv[0]; v[j + 1] += bv[1]; v[j + 2] += bv[2]; v[j + 3] += bv[3];
                        }
                    }
                    if constexpr (sizeof(TO) == 4) {
                        if (beta != 0.f) {
                            const uint4 c = cin[it];
                            v[0] += beta * __uint_as_float(c.x); v[1] += beta * __uint_as_float(c.y);
                            v[2] += beta * __uint_as_float(c.z); v[3] += beta * __uint_as_float(c.w);
                        }
                        f32x4 o = {v[0], v[1], v[2], v[3]};
                        *reinterpret_cast<f32x4*>(p) = o;
                    } else {
                        if (beta != 0.f) {
                            const uint4 c = cin[it];
                            const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
                            for (int j = 0; j < 4; j++) {
                                v[2 * j] += beta * __uint_as_float(w[j] << 16);
                                v[2 * j + 1] += beta * __uint_as_float(w[j] & 0xffff0000u);
                            }
                        }
                        uint32_t w[4];
#pragma unroll
                        for (int j = 0; j < 4; j++) {
                            const __bf16 lo = (__bf16)v[2 * j], hi = (__bf16)v[2 * j + 1];
                            w[j] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
                        }
                        *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < V; j++) {
                        if (gm + j < m_lim) {
                            float x = v[j] + (bias ? bias[gm + j] : 0.f);
                            if (beta != 0.f) x += beta * load_out(p + cin_off + j);
                            store_out(p + j, x);
                        }
                    }
                }
            }
        }
        __syncthreads();
    }
}

}  // namespace nnt
