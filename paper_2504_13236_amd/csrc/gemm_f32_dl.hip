// fp32 product kernel (v_mfma_f32_32x32x2_f32) for whole 128 x 128 macro-tiles (64 x
// 128 for products whose row count is a head size) of 16-byte aligned operands whose
// chunks are multiples of 32 long: the operands go from global memory straight into
// LDS (global_load_lds_dwordx4), five stages of one k-step of 16 each, and the loads
// of two k-steps are started together.
//
// Why: with register-staged loads a k-step's data is asked for one step ahead, in
// 64-byte pieces for an operand whose contracted index is contiguous (16 floats of a
// row).  Half-line requests issued a step apart stall the wave at issue, and one
// step of look-ahead is less than the memory latency under load.  Here the two
// halves of every 128-byte line are requested back to back, loads have two to
// three steps to land, and no registers are spent on staging, so two workgroups of
// 80 KB LDS share a compute unit.
//
// LDS layout of one step (A then B, 8 KB each; a lane's 16 bytes of a load land at
// 16 * lane of the instruction's 1 KB run, so swizzles are applied on the global
// side):
//   * k-contiguous operand: rows of 16 k = 64 bytes; the 16-byte chunk c of row r
//     sits at slot c ^ ((r >> 2) & 3).  A lane's fragment of a substep (4
//     consecutive k of one row) is one 128-bit read.
//   * row-contiguous operand: one line of all its rows (512 or 256 bytes) per k; the
//     16-byte chunk c (4 rows) of line k sits at slot c ^ (((k >> 2) & 1) << 3), which keeps
//     the two half-waves of a 32-bit fragment read (lines 4 apart) on different
//     banks.  A fragment of a substep is four 32-bit reads.
// A k-step is two substeps of 8 k: in substep s lane (row, h) holds k = 8 s + 4 h + i,
// i = 0..3, and matrix instruction i multiplies the two k that the half-waves hold.
#include "gelu_math.hpp"
#include "gemm_common.hpp"
#include "gemm_dl_common.hpp"
#include "nntile_mi.h"

namespace nnt {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kBK = 16;                                  // k-step
constexpr int kStages = 5;

// Byte offset, from (first row, first k) of an operand's ROWS x 16 block, of what this lane fetches
// in load instruction j (0 .. ROWS / 64 - 1) of its wave; the data lands in LDS at
// (wave * ROWS / 64 + j) * 1024 + 16 lane of the operand's region.
template <bool KF, int ROWS>
__device__ __forceinline__ uint32_t load_offset(int ld, int wave, int lane, int j) {
    constexpr int NI = ROWS / 64;
    if (KF) {
        // an instruction covers 16 rows; lane -> row lane / 4, slot lane % 4
        const int r = lane >> 2;
        const int c = (lane & 3) ^ ((r >> 2) & 3);
        return (uint32_t)(((16 * (NI * wave + j) + r) * ld + c * 4) * 4);
    }
    // an instruction covers 256 / ROWS k-lines; lane -> line lane / LPL, slot lane % LPL
    constexpr int LPL = ROWS / 4, LPI = 64 / LPL;            // lanes per line, lines per instruction
    const int kk = LPI * (NI * wave + j) + lane / LPL;
    const int c = (lane % LPL) ^ (((kk >> 2) & 1) << 3);
    return (uint32_t)((kk * ld + c * 4) * 4);
}

// Registers of one fragment of a substep (4 k of the lane's row) while its read is in flight.
struct Frag {
    f32x4 v;
    __device__ __forceinline__ void tie() { asm volatile("" : "+v"(v)); }
};
struct FragR {
    float v[4];
    __device__ __forceinline__ void tie() { asm volatile("" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3])); }
};
template <bool KF> struct FragSel { typedef FragR type; };
template <> struct FragSel<true> { typedef Frag type; };

__device__ __forceinline__ float frag_at(const Frag& f, int i) { return f.v[i]; }
__device__ __forceinline__ float frag_at(const FragR& f, int i) { return f.v[i]; }

// Lane- and wave-dependent parts of the fragment addresses of one operand of ROWS rows, relative to
// the stage.  k-contiguous: one value per substep (the substep flips bit 5), the block is an
// immediate.  Row-contiguous: one value per block (the block enters next to an xor), the substep is
// an immediate.
template <bool KF, int ROWS, int NB>
struct FragAddr {
    uint32_t v[KF ? 2 : NB];
    __device__ __forceinline__ void init(int lane, int first_blk) {
        const int r32 = lane & 31, h = lane >> 5;
        if constexpr (KF) {
            const uint32_t lo = (uint32_t)(r32 * 64 + ((h ^ ((r32 >> 2) & 3)) << 4));
            v[0] = lo + first_blk * 2048;
            v[1] = (lo ^ 32u) + first_blk * 2048;
        } else {
#pragma unroll
            for (int b = 0; b < NB; b++) {
                // 32-row block first_blk + b starts at byte 128 (first_blk + b) of a line; lines with
                // bit 2 of k set (h = 1) have the 128-byte halves of each 256 bytes swapped
                const uint32_t blk = (uint32_t)(first_blk + b);
                v[b] = (uint32_t)(4 * h * ROWS * 4) + ((blk * 128u + (uint32_t)r32 * 4u) ^ ((uint32_t)h * 128u));
            }
        }
    }
};

// Starts the read of fragment B (the wave's B-th 32-row block) of an operand for substep KS.
template <bool KF, int ROWS, int NB, int REGION, int B, int KS>
__device__ __forceinline__ void read_frag(typename FragSel<KF>::type& f, const FragAddr<KF, ROWS, NB>& fa, uint32_t stage_addr) {
    if constexpr (KF) {
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.v) : "v"(stage_addr + fa.v[KS]), "n"(REGION + B * 2048));
    } else {
        constexpr int LB = ROWS * 4;                            // bytes of a k-line
        const uint32_t addr = stage_addr + fa.v[B];
        asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(f.v[0]) : "v"(addr), "n"(REGION + (8 * KS + 0) * LB));
        asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(f.v[1]) : "v"(addr), "n"(REGION + (8 * KS + 1) * LB));
        asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(f.v[2]) : "v"(addr), "n"(REGION + (8 * KS + 2) * LB));
        asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(f.v[3]) : "v"(addr), "n"(REGION + (8 * KS + 3) * LB));
    }
}

// Macro-tile (64 WMB) x (64 WNB): four waves as 2 x 2, each (32 WMB) x (32 WNB).
// EPI: the activation form of the result path (GemmEpi), 0 for the plain one.
// RES: the whole contraction (two or four k-steps) is loaded by the prologue into four stages and the loop starts no
// loads (products whose contraction is a head size: their workgroups live a few microseconds, most of them waiting for
// their result stores to be acknowledged, so what counts is how many of them a compute unit holds).
template <bool AKF, bool BKF, int WMB, int WNB, int EPI, bool RES = false>
__device__ __forceinline__ void f32_dl_body(const GemmArgs& g, char* lds) {
    constexpr int kStages = RES ? 4 : nnt::kStages;
    constexpr int BM = 64 * WMB, BN = 64 * WNB;
    constexpr int kOpABytes = BM * kBK * 4, kOpBBytes = BN * kBK * 4, kStageBytes = kOpABytes + kOpBBytes;
    constexpr int NIA = BM / 64, NIB = BN / 64, kLoads = NIA + NIB;     // load instructions per wave and step
    constexpr int kFrags = WNB + WMB, kMfma = 4 * WNB * WMB;            // per substep

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int r32 = lane & 31, half = lane >> 5;

    GemmTask task;
    int m0, n0, bat;
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
    m0 = __builtin_amdgcn_readfirstlane(m0);
    n0 = __builtin_amdgcn_readfirstlane(n0);
    bat = __builtin_amdgcn_readfirstlane(bat);
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

    int T = 0;
    int chunk_i = 0;                         // index of the current chunk in g.chunks
    if (table) {
        chunk_i = __builtin_amdgcn_readfirstlane(task.chunk0);
        const int nch = __builtin_amdgcn_readfirstlane(task.nchunk);
        for (int c = 0; c < nch; c++) T += sload_chunk(g.chunks + chunk_i + c).k / kBK;
    } else if (task.nchunk > 0) {
        T = g.one_chunk.k / kBK;
    }
    T = __builtin_amdgcn_readfirstlane(T);

    if (T > 0) {
        const int chunk_end = chunk_i + __builtin_amdgcn_readfirstlane(task.nchunk);
        // Position of the next pair of k-steps to load.  A lane's loads are `base + offset` with a
        // uniform base that moves on by a fixed amount per step and per-lane byte offsets that only
        // change with the chunk.  Loads are started for every pair of the loop, needed or not, so that
        // the count of loads in flight is the same at every wait: once the last real pair has been
        // started the position stays where it is and the spare loads fetch that pair again into
        // stages nobody reads.
        int k0 = 0, chk = 0, to_issue = T;
        const char* baseA = nullptr;
        const char* baseB = nullptr;
        int64_t advA = 0, advB = 0;
        uint32_t voffA[NIA], voffB[NIB];
        auto set_chunk = [&](const ChunkS& ch) {
            chk = ch.k;
            const int lda = (int)ch.lda, ldb = (int)ch.ldb;
            const float* Ab = reinterpret_cast<const float*>(ch.A) + (int64_t)bat_lo * ch.strideA + (int64_t)bat_hi * ch.strideA2;
            const float* Bb = reinterpret_cast<const float*>(ch.B) + (int64_t)bat_lo * ch.strideB + (int64_t)bat_hi * ch.strideB2;
            baseA = reinterpret_cast<const char*>(AKF ? Ab + (int64_t)m0 * lda : Ab + m0);
            baseB = reinterpret_cast<const char*>(BKF ? Bb + (int64_t)n0 * ldb : Bb + n0);
            advA = AKF ? kBK * 4 : (int64_t)kBK * lda * 4;
            advB = BKF ? kBK * 4 : (int64_t)kBK * ldb * 4;
#pragma unroll
            for (int j = 0; j < NIA; j++) voffA[j] = load_offset<AKF, BM>(lda, wave, lane, j);
#pragma unroll
            for (int j = 0; j < NIB; j++) voffB[j] = load_offset<BKF, BN>(ldb, wave, lane, j);
        };
        if (table) {
            set_chunk(sload_chunk(g.chunks + chunk_i));
        } else {
            ChunkS one;
            one.A = reinterpret_cast<uint64_t>(g.one_chunk.A); one.B = reinterpret_cast<uint64_t>(g.one_chunk.B);
            one.lda = g.one_chunk.lda; one.ldb = g.one_chunk.ldb;
            one.strideA = g.one_chunk.strideA; one.strideB = g.one_chunk.strideB;
            one.strideA2 = g.one_chunk.strideA2; one.strideB2 = g.one_chunk.strideB2;
            one.k = g.one_chunk.k; one.vec_ok = g.one_chunk.vec_ok;
            set_chunk(one);
        }
        // load instruction i (0 .. 2 kLoads - 1) of the two k-steps at the current position: both
        // halves of a line back to back
        auto load_pair_item = [&](int stage_x, int stage_y, int i) {
            const int j = i >> 1, second = i & 1;
            char* sa = lds + (second ? stage_y : stage_x) * kStageBytes;
            if (j < NIA) {
                __builtin_amdgcn_global_load_lds((glb_void_ptr)(baseA + (second ? advA : 0) + voffA[j]),
                                                 (lds_void_ptr)(sa + (wave * NIA + j) * 1024), 16, 0, 0);
            } else {
                const int jb = j - NIA;
                __builtin_amdgcn_global_load_lds((glb_void_ptr)(baseB + (second ? advB : 0) + voffB[jb]),
                                                 (lds_void_ptr)(sa + kOpABytes + (wave * NIB + jb) * 1024), 16, 0, 0);
            }
        };
        // moves the position on by two k-steps (chunks are multiples of 32 long)
        auto advance2 = [&]() {
            to_issue -= 2;
            if (to_issue > 0) {
                k0 += 2 * kBK;
                if (k0 >= chk) {
                    chunk_i++;
                    k0 = 0;
                    if (chunk_i < chunk_end) set_chunk(sload_chunk(g.chunks + chunk_i));
                } else {
                    baseA += 2 * advA;
                    baseB += 2 * advB;
                }
            } else {
                to_issue = 2;
            }
        };
#pragma unroll
        for (int i = 0; i < 2 * kLoads; i++) load_pair_item(0, 1, i);
        advance2();
#pragma unroll
        for (int i = 0; i < 2 * kLoads; i++) load_pair_item(2, 3, i);
        advance2();

        FragAddr<AKF, BM, WMB> fa;
        FragAddr<BKF, BN, WNB> fb;
        fa.init(lane, wm * WMB);
        fb.init(lane, wn * WNB);
        typename FragSel<BKF>::type pf[2][WNB];
        typename FragSel<AKF>::type qf[2][WMB];
        const uint32_t lds0 = lds_offset(lds);
        // fragment I (first the column blocks of B, then the row blocks of A) of substep KS of a stage
        auto frag_one = [&](auto I, auto KS, int buf, uint32_t stage_addr) {
            constexpr int i = decltype(I)::value, ks = decltype(KS)::value;
            if constexpr (i < WNB) read_frag<BKF, BN, WNB, kOpABytes, i, ks>(pf[buf][i], fb, stage_addr);
            else read_frag<AKF, BM, WMB, 0, i - WNB, ks>(qf[buf][i - WNB], fa, stage_addr);
        };
        // all fragment reads issued so far have landed; the matrix instructions on set `buf` stay behind this
        auto wait_frags = [&](int buf) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < WNB; i++) pf[buf][i].tie();
#pragma unroll
            for (int i = 0; i < WMB; i++) qf[buf][i].tie();
        };
        // matrix instruction q of a substep: k pair q / 4 of block pair q % 4.  The "A" operand of
        // the matrix core carries the columns of C and "B" the rows, so that a lane owns one row of C.
        auto mfma_one = [&](int buf, int q) {
            const int i = q / (WNB * WMB), bn = (q / WMB) % WNB, bm = q % WMB;
            acc[bn][bm] = __builtin_amdgcn_mfma_f32_32x32x2f32(frag_at(pf[buf][bn], i), frag_at(qf[buf][bm], i), acc[bn][bm], 0, 0, 0);
        };
        // One substep: the matrix instructions on fragment set `buf`; under them the fragments of
        // substep F_KS of the stage at `f_addr` are fetched into the other set and NL load
        // instructions are started through `load(i)`, dealt out evenly and fenced in place.
        auto substep = [&](auto NL, auto F_KS, int buf, uint32_t f_addr, auto&& load) {
            constexpr int kItems = kFrags + decltype(NL)::value;
            wait_frags(buf);
            __builtin_amdgcn_sched_barrier(0);
            static_for<kMfma>([&](auto Q) {
                constexpr int q = decltype(Q)::value;
                mfma_one(buf, q);
                static_for<kItems>([&](auto I) {
                    constexpr int i = decltype(I)::value;
                    if constexpr (i * kMfma / kItems == q) {
                        if constexpr (i < kFrags) frag_one(I, F_KS, buf ^ 1, f_addr);
                        else load(i - kFrags);
                    }
                });
                __builtin_amdgcn_sched_barrier(0);
            });
        };
        auto no_load = [](int) {};
        using KS0 = std::integral_constant<int, 0>;
        using KS1 = std::integral_constant<int, 1>;
        using None = std::integral_constant<int, 0>;
        auto stage_addr = [&](int st) { return lds0 + (uint32_t)(st * kStageBytes); };
        auto next_of = [](int st) { return st + 1 == kStages ? 0 : st + 1; };

        // Steps come in pairs (2u, 2u + 1); the loads of a pair are started together, under the
        // second half of the odd step, four steps ahead.
        __builtin_amdgcn_s_waitcnt(wait_vm(2 * kLoads));          // pair 0 landed; pair 1 may remain
        asm volatile("s_barrier" ::: "memory");
        static_for<kFrags>([&](auto I) { frag_one(I, KS0{}, 0, lds0); });
        int st = 0;                                               // stage of step 2u
        for (int u = 0; u < T / 2; u++) {
            const int s1 = next_of(st), s2 = next_of(s1), s3 = next_of(s2), s4 = next_of(s3);
            substep(None{}, KS1{}, 0, stage_addr(st), no_load);
            // pair u complete for everybody (pair u + 1 may remain in flight)
            __builtin_amdgcn_s_waitcnt(wait_vm(2 * kLoads));
            asm volatile("s_barrier" ::: "memory");
            substep(None{}, KS0{}, 1, stage_addr(s1), no_load);
            substep(None{}, KS1{}, 0, stage_addr(s1), no_load);
            // pair u + 1 complete for everybody, and everybody done with the stages of steps 2u - 1
            // and 2u, which the next pair of loads overwrites
            __builtin_amdgcn_s_waitcnt(wait_vm(0));
            asm volatile("s_barrier" ::: "memory");
            // (after the last pair the fragment reads hit a stage that holds no new data: in bounds
            // and unused)
            if constexpr (RES) {
                substep(None{}, KS0{}, 1, stage_addr(s2), no_load);
            } else {
                substep(std::integral_constant<int, 2 * kLoads>{}, KS0{}, 1, stage_addr(s2), [&](int i) { load_pair_item(s4, st, i); });
                advance2();
            }
            st = s2;
        }
        // nothing may still be on its way into LDS or into fragment registers at the end
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    }

    // epilogue: lane holds row m = r32, columns n = 8 * (i / 4) + 4 * half + i % 4 of each 32 x 32 block
    float* C = static_cast<float*>(task.C) + (int64_t)bat_lo * task.strideC + (int64_t)bat_hi * task.strideC2;
    const float alpha = task.partial ? 1.f : g.alpha, beta = task.partial ? 0.f : g.beta;
    constexpr int emode = EPI;          // (the activation forms are never k-slices)
    const int evar = task.epi >> 4;
    // The beta term (C itself, or the tile of a residual input behind cin_off) is read for a whole row block
    // before the first store of that block: a load placed after a store to what may be the same tile has
    // to wait for it, and 32 such round trips per block cost a product with one round of workgroups a
    // quarter of its time.
#pragma unroll
    for (int bm = 0; bm < WMB; bm++) {
        const int gm = m0 + (wm * WMB + bm) * 32 + r32;
        const float bias = (task.bias && !task.partial) ? task.bias[gm] : 0.f;
        float cin[WNB][16];
        if (beta != 0.f || emode == kEpiGeluGradMul) {
#pragma unroll
            for (int bn = 0; bn < WNB; bn++)
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    const int gn = n0 + (wn * WNB + bn) * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
                    cin[bn][i] = C[gm + (int64_t)gn * task.ldc + task.cin_off];
                }
        }
#pragma unroll
        for (int bn = 0; bn < WNB; bn++) {
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const int gn = n0 + (wn * WNB + bn) * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
                float v = alpha * acc[bn][bm][i] + bias;
                if (emode == kEpiGeluGradMul) v *= gelu_grad_f(cin[bn][i], evar);
                else if (beta != 0.f) v += beta * cin[bn][i];
                C[gm + (int64_t)gn * task.ldc] = v;
                if (emode == kEpiGeluOut) C[gm + (int64_t)gn * task.ldc + task.cin_off] = gelu_f(v, evar);
            }
        }
    }
}

template <bool AKF, bool BKF, int WMB, int WNB>
__global__ void __launch_bounds__(256, 2) gemm_f32_dl_kernel(const GemmArgs g) {
    __shared__ __attribute__((aligned(16))) char lds[kStages * (64 * WMB + 64 * WNB) * kBK * 4];
    f32_dl_body<AKF, BKF, WMB, WNB, 0>(g, lds);
}

// The same product with an activation on its result path (nnt_gemm_gelu: EPI = kEpiGeluOut, B as [k, n];
// nnt_gemm_gelu_bwd: kEpiGeluGradMul, A read transposed): kernels of their own, so that the plain ones carry
// none of that code.
template <bool AKF, int WMB, int WNB, int EPI>
__global__ void __launch_bounds__(256, 2) gemm_f32_dl_act_kernel(const GemmArgs g) {
    __shared__ __attribute__((aligned(16))) char lds[kStages * (64 * WMB + 64 * WNB) * kBK * 4];
    f32_dl_body<AKF, true, WMB, WNB, EPI>(g, lds);
}

// 64 x 128 macro-tiles of products with a contraction of 32 or 64, both operands k-contiguous (the scores K^T Q and
// their like): 48 KB of LDS and at most 168 registers, so that a compute unit holds three workgroups.
__global__ void __launch_bounds__(256, 3) gemm_f32_dl_rk_kernel(const GemmArgs g) {
    __shared__ __attribute__((aligned(16))) char lds[4 * (64 + 128) * kBK * 4];
    f32_dl_body<true, true, 1, 2, 0, true>(g, lds);
}

using KernelFn = void (*)(const GemmArgs);

template <int WMB, int WNB>
KernelFn act_kernel_of(int epi_mode) {
    return epi_mode == kEpiGeluOut ? gemm_f32_dl_act_kernel<false, WMB, WNB, kEpiGeluOut> : gemm_f32_dl_act_kernel<true, WMB, WNB, kEpiGeluGradMul>;
}

template <int WMB, int WNB>
KernelFn kernel_of(int akf, int bkf) {
    if (akf) return bkf ? gemm_f32_dl_kernel<true, true, WMB, WNB> : gemm_f32_dl_kernel<true, false, WMB, WNB>;
    return bkf ? gemm_f32_dl_kernel<false, true, WMB, WNB> : gemm_f32_dl_kernel<false, false, WMB, WNB>;
}

KernelFn kernel_of(int akf, int bkf, int cfg) {
    if (cfg == kCfgResident) return (akf && bkf) ? gemm_f32_dl_rk_kernel : nullptr;
    return (cfg == kCfgSkinny64n128 || cfg == kCfgMid) ? kernel_of<1, 2>(akf, bkf) : kernel_of<2, 2>(akf, bkf);
}

}  // namespace

bool gemm_f32_dl_has_act(int akf, int bkf, int epi_mode) {
    return bkf && ((epi_mode == kEpiGeluOut && !akf) || (epi_mode == kEpiGeluGradMul && akf));
}

int32_t launch_gemm_f32_dl(hipStream_t st, int akf, int bkf, int cfg, const GemmArgs& g, int64_t nwg, int epi_mode) {
    if (nwg <= 0) return NNT_OK;
    if (epi_mode) {
        if (!gemm_f32_dl_has_act(akf, bkf, epi_mode)) return NNT_EINVAL;
        const bool mid = cfg == kCfgSkinny64n128 || cfg == kCfgMid;
        const KernelFn fn = mid ? act_kernel_of<1, 2>(epi_mode) : act_kernel_of<2, 2>(epi_mode);
        hipLaunchKernelGGL(fn, dim3((unsigned)nwg), dim3(256), 0, st, g);
        return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
    }
    if (!kernel_of(akf, bkf, cfg)) return NNT_EINVAL;
    hipLaunchKernelGGL(kernel_of(akf, bkf, cfg), dim3((unsigned)nwg), dim3(256), 0, st, g);
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int gemm_f32_dl_occupancy(int akf, int bkf, int cfg) {
    int n = 0;
    if (!kernel_of(akf, bkf, cfg)) return 1;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel_of(akf, bkf, cfg), 256, 0) != hipSuccess || n < 1) n = 1;
    return n;
}

}  // namespace nnt
