// fp32 tile-grid product on the gfx950 matrix cores (v_mfma_f32_32x32x2_f32):
// true fp32 inputs, fp32 accumulation.
//
// One workgroup of four wavefronts owns a BM x BN macro-tile of one C tile and
// walks the task's chunks in k-steps of 16.  Both operands are staged through
// LDS in the orientation they have in memory (no transposes): an operand whose
// contracted index is contiguous ("k-fast") is kept as [row][16 + 4 pad], one
// whose row index is contiguous as [k][rows]; the matrix-core fragments are read
// with 128-bit or 32-bit LDS loads accordingly.  Global loads for step i+1 are
// issued before the MFMAs of step i and written to the other LDS buffer after
// them, so each step costs one barrier.
//
// The matrix-core "A" operand carries the columns of C (index n) and the "B"
// operand the rows (index m): a lane then holds 16 values of one row index m =
// lane % 32, and the 32 lanes of a half-wave store 32 consecutive rows, which are
// contiguous in the column-major C tile.
#include "gemm_common.hpp"
#include "nntile_mi.h"

namespace nnt {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

// A pointer that is the same in every lane, moved to scalar registers.
template <typename T>
__device__ __forceinline__ const T* uniform_ptr(const T* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const T*>(((uint64_t)hi << 32) | lo);
}

constexpr int BK = 16;
constexpr int KP = BK + 4;   // padded k extent of a k-fast LDS row (conflict-free 128-bit reads)

template <bool KF, int ROWS>
__device__ __forceinline__ void gload(f32x4 (&v)[ROWS / 64], const float* base, int ld, int row0,
                                      int nrows, int k0, int kc, bool vec_ok, int tid) {
#pragma unroll
    for (int i = 0; i < ROWS / 64; i++) {
        const int idx = tid + 256 * i;
        int r, k;
        if (KF) { r = idx >> 2; k = (idx & 3) << 2; }
        else { k = idx / (ROWS / 4); r = (idx % (ROWS / 4)) << 2; }
        const int gr = row0 + r, gk = k0 + k;
        const float* p = KF ? base + gk + (int64_t)gr * ld : base + gr + (int64_t)gk * ld;
        const int cnt = KF ? (gr < nrows ? kc - gk : 0) : (gk < kc ? nrows - gr : 0);
        f32x4 x = {0.f, 0.f, 0.f, 0.f};
        if (cnt >= 4 && vec_ok) {
            x = *reinterpret_cast<const f32x4*>(p);
        } else {
            if (cnt > 0) x[0] = p[0];
            if (cnt > 1) x[1] = p[1];
            if (cnt > 2) x[2] = p[2];
            if (cnt > 3) x[3] = p[3];
        }
        v[i] = x;
    }
}

// Interior k-step of an aligned operand: no predicates, no branches, so the loads stay in
// flight across the matrix-core work that follows.  `base` points at (row0, k0).
template <bool KF, int ROWS>
__device__ __forceinline__ void gload_fast(f32x4 (&v)[ROWS / 64], const float* base, int ld, int tid) {
#pragma unroll
    for (int i = 0; i < ROWS / 64; i++) {
        const int idx = tid + 256 * i;
        int r, k;
        if (KF) { r = idx >> 2; k = (idx & 3) << 2; }
        else { k = idx / (ROWS / 4); r = (idx % (ROWS / 4)) << 2; }
        const float* p = KF ? base + k + (int64_t)r * ld : base + r + (int64_t)k * ld;
        v[i] = *reinterpret_cast<const f32x4*>(p);
    }
}

template <bool KF, int ROWS>
__device__ __forceinline__ void lstore(float* l, const f32x4 (&v)[ROWS / 64], int tid) {
#pragma unroll
    for (int i = 0; i < ROWS / 64; i++) {
        const int idx = tid + 256 * i;
        if (KF) {
            const int r = idx >> 2, k = (idx & 3) << 2;
            *reinterpret_cast<f32x4*>(&l[r * KP + k]) = v[i];
        } else {
            const int k = idx / (ROWS / 4), r = (idx % (ROWS / 4)) << 2;
            *reinterpret_cast<f32x4*>(&l[k * ROWS + r]) = v[i];
        }
    }
}

// The 8 k-values of this lane's half (k = 8 * half + j) for one 32-row block.
template <bool KF, int ROWS>
__device__ __forceinline__ void lfrag(float (&f)[8], const float* l, int row, int half) {
    if (KF) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(&l[row * KP + half * 8]);
        const f32x4 b = *reinterpret_cast<const f32x4*>(&l[row * KP + half * 8 + 4]);
        f[0] = a[0]; f[1] = a[1]; f[2] = a[2]; f[3] = a[3];
        f[4] = b[0]; f[5] = b[1]; f[6] = b[2]; f[7] = b[3];
    } else {
#pragma unroll
        for (int j = 0; j < 8; j++) f[j] = l[(half * 8 + j) * ROWS + row];
    }
}

template <bool AKF, bool BKF, int WAVES_M, int WAVES_N, int WMB, int WNB>
__global__ void __launch_bounds__(256) gemm_f32_kernel(const GemmArgs g) {
    constexpr int BM = 32 * WMB * WAVES_M, BN = 32 * WNB * WAVES_N;
    constexpr int A_SZ = AKF ? BM * KP : BK * BM;
    constexpr int B_SZ = BKF ? BN * KP : BK * BN;
    __shared__ __attribute__((aligned(16))) float lds[2 * (A_SZ + B_SZ)];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WAVES_M, wn = wave / WAVES_M;
    const int r32 = lane & 31, half = lane >> 5;

    GemmTask task;
    int m0, n0, bat;
    // (the chunk table is only ever addressed through g.chunks, a global pointer with a uniform
    // index, so that the descriptors arrive through scalar loads and the loop control stays scalar)
    const bool table = g.wgs != nullptr;
    if (table) {
        const GemmWg w = g.wgs[blockIdx.x];
        task = g.tasks[w.task];
        m0 = w.m0; n0 = w.n0; bat = w.batch;
    } else {
        task = g.one_task;
        const int b = blockIdx.x;
        m0 = (b % g.grid_m) * BM;
        n0 = ((b / g.grid_m) % g.grid_n) * BN;
        bat = b / (g.grid_m * g.grid_n);
    }
    // (batch members that are pairs: see GemmTask::nb1)
    int bat_lo = bat, bat_hi = 0;
    if (task.nb1 > 0) {
        bat_hi = bat / task.nb1;
        bat_lo = bat - bat_hi * task.nb1;
    }

    f32x16 acc[WNB][WMB];
#pragma unroll
    for (int bn = 0; bn < WNB; bn++)
#pragma unroll
        for (int bm = 0; bm < WMB; bm++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc[bn][bm][i] = 0.f;

    if (task.nchunk > 0) {
        // Loop state that is the same for every lane is kept in scalar registers on purpose
        // (readfirstlane): the k-loop then branches on the scalar unit and the loads address
        // memory as scalar base + per-lane offset.
        int c = 0, k0 = 0, chk = 0, chvec = 0, lda = 0, ldb = 0;
        const float* Ab = nullptr;
        const float* Bb = nullptr;
        auto set_chunk = [&](const GemmChunk& ch) {
            chk = __builtin_amdgcn_readfirstlane(ch.k);
            chvec = __builtin_amdgcn_readfirstlane(ch.vec_ok);
            lda = __builtin_amdgcn_readfirstlane((int)ch.lda);
            ldb = __builtin_amdgcn_readfirstlane((int)ch.ldb);
            Ab = uniform_ptr(static_cast<const float*>(ch.A) + (int64_t)bat_lo * ch.strideA + (int64_t)bat_hi * ch.strideA2);
            Bb = uniform_ptr(static_cast<const float*>(ch.B) + (int64_t)bat_lo * ch.strideB + (int64_t)bat_hi * ch.strideB2);
        };
        set_chunk(table ? g.chunks[task.chunk0] : g.one_chunk);
        f32x4 va[BM / 64], vb[BN / 64];
        // whole macro-tile inside the C tile: k-steps that are also whole take the branch-free loads
        const bool inside = m0 + BM <= task.m && n0 + BN <= task.n;
        auto load_step = [&]() {
            if (inside && k0 + BK <= chk && chvec == 3) {
                gload_fast<AKF, BM>(va, AKF ? Ab + k0 + (int64_t)m0 * lda : Ab + m0 + (int64_t)k0 * lda, lda, tid);
                gload_fast<BKF, BN>(vb, BKF ? Bb + k0 + (int64_t)n0 * ldb : Bb + n0 + (int64_t)k0 * ldb, ldb, tid);
            } else {
                gload<AKF, BM>(va, Ab, lda, m0, task.m, k0, chk, chvec & 1, tid);
                gload<BKF, BN>(vb, Bb, ldb, n0, task.n, k0, chk, chvec & 2, tid);
            }
        };
        load_step();
        int cur = 0;
        lstore<AKF, BM>(lds, va, tid);
        lstore<BKF, BN>(lds + A_SZ, vb, tid);
        __syncthreads();
        bool more = true;
        while (more) {
            // advance to the next k-step (possibly the next chunk) and start its loads
            k0 += BK;
            if (k0 >= chk) {
                c++;
                k0 = 0;
                if (c < task.nchunk) set_chunk(g.chunks[task.chunk0 + c]);
            }
            more = c < task.nchunk;
            if (more) load_step();
            const float* lA = lds + cur * (A_SZ + B_SZ);
            const float* lB = lA + A_SZ;
            float pf[WNB][8], qf[WMB][8];
#pragma unroll
            for (int bn = 0; bn < WNB; bn++) lfrag<BKF, BN>(pf[bn], lB, (wn * WNB + bn) * 32 + r32, half);
#pragma unroll
            for (int bm = 0; bm < WMB; bm++) lfrag<AKF, BM>(qf[bm], lA, (wm * WMB + bm) * 32 + r32, half);
#pragma unroll
            for (int j = 0; j < 8; j++)
#pragma unroll
                for (int bn = 0; bn < WNB; bn++)
#pragma unroll
                    for (int bm = 0; bm < WMB; bm++)
                        acc[bn][bm] = __builtin_amdgcn_mfma_f32_32x32x2f32(pf[bn][j], qf[bm][j], acc[bn][bm], 0, 0, 0);
            if (more) {
                float* nA = lds + (cur ^ 1) * (A_SZ + B_SZ);
                lstore<AKF, BM>(nA, va, tid);
                lstore<BKF, BN>(nA + A_SZ, vb, tid);
            }
            __syncthreads();
            cur ^= 1;
        }
    }

    // epilogue: lane holds row m = r32, columns n = 8 * (i / 4) + 4 * half + i % 4 of each 32 x 32 block
    float* C = static_cast<float*>(task.C) + (int64_t)bat_lo * task.strideC + (int64_t)bat_hi * task.strideC2;
    const float alpha = task.partial ? 1.f : g.alpha, beta = task.partial ? 0.f : g.beta;
#pragma unroll
    for (int bm = 0; bm < WMB; bm++) {
        const int gm = m0 + (wm * WMB + bm) * 32 + r32;
        if (gm >= task.m) continue;
        const float bias = task.bias ? task.bias[gm] : 0.f;
        // (the beta term of the whole row block is read before its first store: a load behind a store to
        // what may be the same tile would wait for it)
        float cin[WNB][16];
        if (beta != 0.f) {
#pragma unroll
            for (int bn = 0; bn < WNB; bn++)
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    const int gn = n0 + (wn * WNB + bn) * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
                    cin[bn][i] = gn < task.n ? C[gm + (int64_t)gn * task.ldc + task.cin_off] : 0.f;
                }
        }
#pragma unroll
        for (int bn = 0; bn < WNB; bn++) {
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const int gn = n0 + (wn * WNB + bn) * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
                if (gn < task.n) {
                    float v = alpha * acc[bn][bm][i] + bias;
                    if (beta != 0.f) v += beta * cin[bn][i];
                    C[gm + (int64_t)gn * task.ldc] = v;
                }
            }
        }
    }
}

using KernelFn = void (*)(const GemmArgs);

template <bool AKF, bool BKF>
KernelFn kernel_of(int cfg) {
    switch (cfg) {
        case kCfgSquare:
        case kCfgTall: return gemm_f32_kernel<AKF, BKF, 2, 2, 2, 2>;
        case kCfgMid:
        case kCfgResident: return gemm_f32_kernel<AKF, BKF, 2, 2, 1, 2>;
        case kCfgSkinny64: return gemm_f32_kernel<AKF, BKF, 1, 4, 2, 2>;
        case kCfgSkinny64n128: return gemm_f32_kernel<AKF, BKF, 1, 4, 2, 1>;
        case kCfgSkinny64n64: return gemm_f32_kernel<AKF, BKF, 2, 2, 1, 1>;
        default: return gemm_f32_kernel<AKF, BKF, 1, 4, 4, 2>;
    }
}

KernelFn kernel_of(int akf, int bkf, int cfg) {
    if (akf) return bkf ? kernel_of<true, true>(cfg) : kernel_of<true, false>(cfg);
    return bkf ? kernel_of<false, true>(cfg) : kernel_of<false, false>(cfg);
}

}  // namespace

int32_t launch_gemm_f32(hipStream_t st, int akf, int bkf, int cfg, const GemmArgs& g, int64_t nwg) {
    if (nwg <= 0) return NNT_OK;
    hipLaunchKernelGGL(kernel_of(akf, bkf, cfg), dim3((unsigned)nwg), dim3(256), 0, st, g);
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int gemm_f32_occupancy(int akf, int bkf, int cfg) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel_of(akf, bkf, cfg), 256, 0) != hipSuccess || n < 1) n = 1;
    return n;
}

}  // namespace nnt
