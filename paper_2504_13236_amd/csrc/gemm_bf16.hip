// bf16-input tile-grid product on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16): bf16 operands, fp32 accumulation over all chunks
// of a task, one rounding when C is written (fp32 or bf16).
//
// Four wavefronts per workgroup own a BM x BN macro-tile and walk the task's
// chunks in k-steps of BKT.  The matrix cores want 8 consecutive k per lane, so
// both operands live in LDS as [row][BKT + 8 pad] (k fastest; the pad makes the
// 128-bit fragment reads conflict-free).  An operand that is k-fast in memory is
// copied with 128-bit loads and stores; one whose row index is contiguous is read
// as 8-row vectors at 4 consecutive k and transposed in registers (16-bit packs)
// before the LDS store.
//
// Pipeline (a workgroup has the matrix cores of its CU to itself, so latency has
// to be hidden inside each wavefront):
//   * three LDS stages: while step t is multiplied, step t+1 is already complete
//     in LDS and step t+2 is being written, so one barrier per step suffices and
//     the first fragments of step t+1 can be fetched before that barrier;
//   * fragments of the next k-substep are requested from LDS before the matrix
//     instructions of the current one are issued (two fragment register sets);
//   * global loads of step t+3 are issued right after the registers of step t+2
//     have been stored to LDS and stay in flight for a whole step.
#include "gemm_bf16_out.hpp"
#include "gemm_common.hpp"
#include "nntile_mi.h"

namespace nnt {

namespace {

__device__ __forceinline__ uint4 load8_guarded(const uint16_t* p, int cnt) {
    uint16_t e[8];
#pragma unroll
    for (int j = 0; j < 8; j++) e[j] = j < cnt ? p[j] : (uint16_t)0;
    uint4 x;
    x.x = e[0] | ((uint32_t)e[1] << 16);
    x.y = e[2] | ((uint32_t)e[3] << 16);
    x.z = e[4] | ((uint32_t)e[5] << 16);
    x.w = e[6] | ((uint32_t)e[7] << 16);
    return x;
}

// ---- k-fast operand: vectors of 8 along k
template <int ROWS, int BKT>
struct LoaderK {
    static constexpr int NV = ROWS * BKT / 8 / 256 > 0 ? ROWS * BKT / 8 / 256 : 1;
    static constexpr int TOTAL = ROWS * BKT / 8;
    static constexpr int KP = BKT + 8;
    uint4 v[NV];
    __device__ __forceinline__ void load(const uint16_t* base, int ld, int row0, int nrows, int k0, int kc,
                                         bool vec_ok, int tid) {
#pragma unroll
        for (int i = 0; i < NV; i++) {
            const int idx = tid + 256 * i;
            uint4 x = {0u, 0u, 0u, 0u};
            if (TOTAL >= 256 || idx < TOTAL) {
                const int r = idx / (BKT / 8), k = (idx % (BKT / 8)) * 8;
                const int gr = row0 + r, gk = k0 + k;
                const uint16_t* p = base + gk + (int64_t)gr * ld;
                const int cnt = gr < nrows ? kc - gk : 0;
                if (cnt >= 8 && vec_ok) x = *reinterpret_cast<const uint4*>(p);
                else if (cnt > 0) x = load8_guarded(p, cnt);
            }
            v[i] = x;
        }
    }
    // interior k-step of an aligned operand; `base` points at (row0, k0)
    __device__ __forceinline__ void load_fast(const uint16_t* base, int ld, int tid) {
#pragma unroll
        for (int i = 0; i < NV; i++) {
            const int idx = tid + 256 * i;
            if (TOTAL >= 256 || idx < TOTAL) {
                const int r = idx / (BKT / 8), k = (idx % (BKT / 8)) * 8;
                v[i] = *reinterpret_cast<const uint4*>(base + k + (int64_t)r * ld);
            }
        }
    }
    __device__ __forceinline__ void store(uint16_t* l, int tid) const {
#pragma unroll
        for (int i = 0; i < NV; i++) {
            const int idx = tid + 256 * i;
            if (TOTAL >= 256 || idx < TOTAL) {
                const int r = idx / (BKT / 8), k = (idx % (BKT / 8)) * 8;
                *reinterpret_cast<uint4*>(&l[r * KP + k]) = v[i];
            }
        }
    }
};

// ---- row-fast operand: micro-blocks of 8 rows x 4 k, transposed in registers
template <int ROWS, int BKT>
struct LoaderR {
    static constexpr int TOTAL = (ROWS / 8) * (BKT / 4);
    static constexpr int NB = TOTAL / 256 > 0 ? TOTAL / 256 : 1;
    static constexpr int KP = BKT + 8;
    uint4 v[NB][4];
    __device__ __forceinline__ void load(const uint16_t* base, int ld, int row0, int nrows, int k0, int kc,
                                         bool vec_ok, int tid) {
#pragma unroll
        for (int i = 0; i < NB; i++) {
            const int idx = tid + 256 * i;
            const int kq = idx % (BKT / 4), rg = idx / (BKT / 4);
            const int gr = row0 + rg * 8;
            const int cnt = (TOTAL >= 256 || idx < TOTAL) ? nrows - gr : 0;
#pragma unroll
            for (int kk = 0; kk < 4; kk++) {
                const int gk = k0 + kq * 4 + kk;
                uint4 x = {0u, 0u, 0u, 0u};
                if (gk < kc && cnt > 0) {
                    const uint16_t* p = base + gr + (int64_t)gk * ld;
                    if (cnt >= 8 && vec_ok) x = *reinterpret_cast<const uint4*>(p);
                    else x = load8_guarded(p, cnt);
                }
                v[i][kk] = x;
            }
        }
    }
    __device__ __forceinline__ void load_fast(const uint16_t* base, int ld, int tid) {
#pragma unroll
        for (int i = 0; i < NB; i++) {
            const int idx = tid + 256 * i;
            if (TOTAL >= 256 || idx < TOTAL) {
                const int kq = idx % (BKT / 4), rg = idx / (BKT / 4);
#pragma unroll
                for (int kk = 0; kk < 4; kk++)
                    v[i][kk] = *reinterpret_cast<const uint4*>(base + rg * 8 + (int64_t)(kq * 4 + kk) * ld);
            }
        }
    }
    __device__ __forceinline__ void store(uint16_t* l, int tid) const {
#pragma unroll
        for (int i = 0; i < NB; i++) {
            const int idx = tid + 256 * i;
            if (TOTAL >= 256 || idx < TOTAL) {
                const int kq = idx % (BKT / 4), rg = idx / (BKT / 4);
                const uint32_t* w0 = reinterpret_cast<const uint32_t*>(&v[i][0]);
                const uint32_t* w1 = reinterpret_cast<const uint32_t*>(&v[i][1]);
                const uint32_t* w2 = reinterpret_cast<const uint32_t*>(&v[i][2]);
                const uint32_t* w3 = reinterpret_cast<const uint32_t*>(&v[i][3]);
#pragma unroll
                for (int d = 0; d < 4; d++) {
                    // dword d of each vector holds rows 2d (low half) and 2d + 1 (high half)
                    uint2 lo, hi;
                    lo.x = (w0[d] & 0xffffu) | (w1[d] << 16);
                    lo.y = (w2[d] & 0xffffu) | (w3[d] << 16);
                    hi.x = (w0[d] >> 16) | (w1[d] & 0xffff0000u);
                    hi.y = (w2[d] >> 16) | (w3[d] & 0xffff0000u);
                    *reinterpret_cast<uint2*>(&l[(rg * 8 + 2 * d) * KP + kq * 4]) = lo;
                    *reinterpret_cast<uint2*>(&l[(rg * 8 + 2 * d + 1) * KP + kq * 4]) = hi;
                }
            }
        }
    }
};

template <bool KF, int ROWS, int BKT>
struct LoaderSel { typedef LoaderR<ROWS, BKT> type; };
template <int ROWS, int BKT>
struct LoaderSel<true, ROWS, BKT> { typedef LoaderK<ROWS, BKT> type; };

template <typename TO, bool AKF, bool BKF, int WAVES_M, int WAVES_N, int WMB, int WNB, int BKT>
__global__ void __launch_bounds__(256) gemm_bf16_kernel(const GemmArgs g) {
    constexpr int BM = 32 * WMB * WAVES_M, BN = 32 * WNB * WAVES_N;
    constexpr int KP = BKT + 8, KS = BKT / 16;
    constexpr int A_SZ = BM * KP, B_SZ = BN * KP, ST_SZ = A_SZ + B_SZ;
    static_assert(KS % 2 == 0, "fragment buffers alternate per substep and must line up across steps");
    __shared__ __attribute__((aligned(16))) uint16_t lds[3 * ST_SZ];

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

    // number of k-steps of the whole task
    int T = 0;
    if (table) {
        for (int c = 0; c < task.nchunk; c++) T += (g.chunks[task.chunk0 + c].k + BKT - 1) / BKT;
    } else if (task.nchunk > 0) {
        T = (g.one_chunk.k + BKT - 1) / BKT;
    }
    T = __builtin_amdgcn_readfirstlane(T);

    if (T > 0) {
        // position of the next k-step to load; uniform state lives in scalar registers
        int c = 0, k0 = 0, chk = 0, chvec = 0, lda = 0, ldb = 0;
        const uint16_t* Ab = nullptr;
        const uint16_t* Bb = nullptr;
        auto set_chunk = [&](const GemmChunk& ch) {
            chk = __builtin_amdgcn_readfirstlane(ch.k);
            chvec = __builtin_amdgcn_readfirstlane(ch.vec_ok);
            lda = __builtin_amdgcn_readfirstlane((int)ch.lda);
            ldb = __builtin_amdgcn_readfirstlane((int)ch.ldb);
            Ab = uniform_ptr(static_cast<const uint16_t*>(ch.A) + (int64_t)bat_lo * ch.strideA + (int64_t)bat_hi * ch.strideA2);
            Bb = uniform_ptr(static_cast<const uint16_t*>(ch.B) + (int64_t)bat_lo * ch.strideB + (int64_t)bat_hi * ch.strideB2);
        };
        set_chunk(table ? g.chunks[task.chunk0] : g.one_chunk);
        typename LoaderSel<AKF, BM, BKT>::type la;
        typename LoaderSel<BKF, BN, BKT>::type lb;
        const bool inside = m0 + BM <= task.m && n0 + BN <= task.n;
        // loads the k-step at the current position into registers and moves the position on
        auto load_step = [&]() {
            if (inside && k0 + BKT <= chk && chvec == 3) {
                la.load_fast(AKF ? Ab + k0 + (int64_t)m0 * lda : Ab + m0 + (int64_t)k0 * lda, lda, tid);
                lb.load_fast(BKF ? Bb + k0 + (int64_t)n0 * ldb : Bb + n0 + (int64_t)k0 * ldb, ldb, tid);
            } else {
                la.load(Ab, lda, m0, task.m, k0, chk, chvec & 1, tid);
                lb.load(Bb, ldb, n0, task.n, k0, chk, chvec & 2, tid);
            }
            k0 += BKT;
            if (k0 >= chk) {
                c++;
                k0 = 0;
                if (c < task.nchunk) set_chunk(g.chunks[task.chunk0 + c]);
            }
        };
        auto store_step = [&](int stage) {
            uint16_t* s = lds + stage * ST_SZ;
            la.store(s, tid);
            lb.store(s + A_SZ, tid);
        };

        // prologue: steps 0 and 1 into LDS, step 2 into registers
        load_step();
        store_step(0);
        if (T > 1) { load_step(); store_step(1); }
        bool in_regs = false;
        if (T > 2) { load_step(); in_regs = true; }
        __syncthreads();

        bf16x8 pf[2][WNB], qf[2][WMB];
        auto frags = [&](int buf, int stage, int ks) {
            const uint16_t* lA = lds + stage * ST_SZ;
            const uint16_t* lB = lA + A_SZ;
#pragma unroll
            for (int bn = 0; bn < WNB; bn++)
                pf[buf][bn] = *reinterpret_cast<const bf16x8*>(&lB[((wn * WNB + bn) * 32 + r32) * KP + ks * 16 + half * 8]);
#pragma unroll
            for (int bm = 0; bm < WMB; bm++)
                qf[buf][bm] = *reinterpret_cast<const bf16x8*>(&lA[((wm * WMB + bm) * 32 + r32) * KP + ks * 16 + half * 8]);
        };
        frags(0, 0, 0);
        int stage = 0;                      // t % 3
        for (int t = 0; t < T; t++) {
            const int next_stage = stage == 2 ? 0 : stage + 1;
#pragma unroll
            for (int ks = 0; ks < KS; ks++) {
                // fragments of the next substep (of this step, or the first of the next step, which has
                // been complete in LDS since the previous barrier) before the matrix work of this one
                const int cur = ks & 1, nxt = cur ^ 1;
                // (after the last step this reads a stale stage, in bounds and unused: keeping the reads
                // unconditional keeps them in the same scheduling block as the matrix instructions)
                if (ks + 1 < KS) frags(nxt, stage, ks + 1);
                else frags(nxt, next_stage, 0);
#pragma unroll
                for (int bn = 0; bn < WNB; bn++)
#pragma unroll
                    for (int bm = 0; bm < WMB; bm++)
                        acc[bn][bm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[cur][bm], pf[cur][bn], acc[bn][bm], 0, 0, 0);
                // issue order: the LDS reads go out one per matrix instruction at the start of the substep,
                // so that all of them have landed when the substep ends
                constexpr int kReads = WNB + WMB, kMfma = WNB * WMB;
#pragma unroll
                for (int i = 0; i < kReads; i++) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    if (i < kMfma) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
                if (kMfma > kReads) __builtin_amdgcn_sched_group_barrier(0x008, kMfma - kReads, 0);
            }
            if (in_regs) {                  // step t + 2, loaded during the previous step
                store_step(next_stage == 2 ? 0 : next_stage + 1);
                in_regs = false;
            }
            if (t + 3 < T) { load_step(); in_regs = true; }
            __syncthreads();
            stage = next_stage;
        }
    }

    // The matrix-core "A" operand carries the rows of C (index m): a lane holds, for column
    // n = lane % 32 of each 32 x 32 block, the rows 8 * (i / 4) + 4 * half + i % 4.  Results go
    // through a per-wave LDS buffer (the pipeline stages are free by now) so that they leave as
    // 16-byte vectors along m, the contiguous index of the C tile.
    float* stage = reinterpret_cast<float*>(lds) + wave * (32 * (32 * WMB + 4));
    static_assert(4 * 32 * (32 * WMB + 4) * 4 <= 3 * ST_SZ * 2, "result staging must fit the pipeline's LDS");
    const int m_base = m0 + wm * WMB * 32, n_base = n0 + wn * WNB * 32;
    if (task.partial) {
        // one k-slice of a split product: raw fp32 sums into the scratch tile
        write_tile<float, WMB, WNB>(stage, acc, static_cast<float*>(task.C) + (int64_t)bat_lo * task.strideC + (int64_t)bat_hi * task.strideC2, task.ldc, nullptr,
                                    1.f, 0.f, m_base, n_base, task.m, task.n, lane);
    } else {
        write_tile<TO, WMB, WNB>(stage, acc, static_cast<TO*>(task.C) + (int64_t)bat_lo * task.strideC + (int64_t)bat_hi * task.strideC2, task.ldc, task.bias,
                                 g.alpha, g.beta, m_base, n_base, task.m, task.n, lane, task.cin_off);
    }
}

using KernelFn = void (*)(const GemmArgs);

template <typename TO, bool AKF, bool BKF>
KernelFn kernel_of(int cfg) {
    switch (cfg) {
        case kCfgSquare: return gemm_bf16_kernel<TO, AKF, BKF, 2, 2, 4, 4, 32>;
        case kCfgMid: return gemm_bf16_kernel<TO, AKF, BKF, 2, 2, 2, 2, 32>;
        case kCfgSkinny64: return gemm_bf16_kernel<TO, AKF, BKF, 1, 4, 2, 2, 32>;
        case kCfgSkinny64n128: return gemm_bf16_kernel<TO, AKF, BKF, 1, 4, 2, 1, 32>;
        case kCfgSkinny64n64: return gemm_bf16_kernel<TO, AKF, BKF, 2, 2, 1, 1, 32>;
        case kCfgTall: return gemm_bf16_kernel<TO, AKF, BKF, 2, 2, 4, 2, 32>;
        case kCfgWide: return gemm_bf16_kernel<TO, AKF, BKF, 2, 2, 2, 2, 32>;      // (what the direct-load kernel of the shape does not take)
        default: return gemm_bf16_kernel<TO, AKF, BKF, 1, 4, 4, 2, 32>;
    }
}

template <typename TO>
KernelFn kernel_of(int akf, int bkf, int cfg) {
    if (akf) return bkf ? kernel_of<TO, true, true>(cfg) : kernel_of<TO, true, false>(cfg);
    return bkf ? kernel_of<TO, false, true>(cfg) : kernel_of<TO, false, false>(cfg);
}

}  // namespace

int32_t launch_gemm_bf16(hipStream_t st, int out_is_f32, int akf, int bkf, int cfg, const GemmArgs& g, int64_t nwg) {
    if (nwg <= 0) return NNT_OK;
    const KernelFn fn = out_is_f32 ? kernel_of<float>(akf, bkf, cfg) : kernel_of<uint16_t>(akf, bkf, cfg);
    hipLaunchKernelGGL(fn, dim3((unsigned)nwg), dim3(256), 0, st, g);
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int gemm_bf16_occupancy(int out_is_f32, int akf, int bkf, int cfg) {
    const KernelFn fn = out_is_f32 ? kernel_of<float>(akf, bkf, cfg) : kernel_of<uint16_t>(akf, bkf, cfg);
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, fn, 256, 0) != hipSuccess || n < 1) n = 1;
    return n;
}

}  // namespace nnt
