// bf16 product kernel for whole 256 x 256 or 256 x 128 macro-tiles of 16-byte
// aligned operands whose chunks are multiples of 32 long: the operands go from
// global memory straight into LDS (global_load_lds_dwordx4), three or four k-steps
// of 32 deep, so that loads stay in flight across whole steps and no registers are
// spent on staging.
//
// LDS layout of one step (A then B, 64 bytes per row), chosen so that both the
// 1 KB runs a wave's load instruction fills (lane i -> bytes 16 i .. 16 i + 15)
// and the fragment reads of the matrix cores are free of bank conflicts (64 banks
// of 4 bytes):
//   * operand with the contracted index contiguous in memory ("k-fast"): rows of
//     32 k = 64 bytes; the 16-byte chunk c of row r sits at slot c ^ ((r >> 2) & 3).
//     A lane's fragment (8 consecutive k of one row) is one 128-bit read.
//   * operand with the row index contiguous: one line of all its rows per k;
//     the 16-byte chunk c (8 rows) of line k sits at slot c ^ ((k & 3) << 2).
//     Fragments are fetched with ds_read_b64_tr_b16, which hands each lane four
//     consecutive k of its row from four lines (two reads per fragment).
// The swizzles are applied on the global side: a lane picks the global address
// whose data belongs in its LDS slot.
//
// Synchronisation per k-step, between its two substeps of 16: every wave waits
// until its own loads of the next step have landed (vmcnt, leaving the younger
// steps in flight), one barrier makes all waves' parts visible and at the same
// time proves that everybody is done with the stage of the previous step, which
// the loads started right after the barrier overwrite.  The first fragments of the
// next step are then fetched under the matrix instructions of the second substep.
#include "gemm_bf16_out.hpp"
#include "gemm_common.hpp"
#include "nntile_mi.h"

#include <type_traits>

namespace nnt {

namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* glb_void_ptr;

constexpr int kBK = 32;                 // k-step

// s_waitcnt immediate (gfx9 encoding) that constrains only vmcnt
constexpr int wait_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }

// A chunk descriptor in scalar registers.  The descriptor tables are constant for the lifetime of
// a launch, but the compiler cannot know that next to the loads that write LDS, so the scalar
// loads are spelled out.
struct ChunkS {
    uint64_t A, B;
    int64_t lda, ldb, strideA, strideB;
    int32_t k, vec_ok;
};
static_assert(sizeof(ChunkS) == sizeof(GemmChunk) && sizeof(GemmChunk) == 56, "descriptor layout");

__device__ __forceinline__ ChunkS sload_chunk(const GemmChunk* p) {
    typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    u32x8 a;
    u32x4 b;
    u32x2 c;
    asm volatile("s_load_dwordx8 %0, %3, 0x0\n\ts_load_dwordx4 %1, %3, 0x20\n\ts_load_dwordx2 %2, %3, 0x30\n\ts_waitcnt lgkmcnt(0)"
                 : "=&s"(a), "=&s"(b), "=&s"(c)
                 : "s"(p)
                 : "memory");
    ChunkS r;
    r.A = a[0] | ((uint64_t)a[1] << 32);
    r.B = a[2] | ((uint64_t)a[3] << 32);
    r.lda = (int64_t)(a[4] | ((uint64_t)a[5] << 32));
    r.ldb = (int64_t)(a[6] | ((uint64_t)a[7] << 32));
    r.strideA = (int64_t)(b[0] | ((uint64_t)b[1] << 32));
    r.strideB = (int64_t)(b[2] | ((uint64_t)b[3] << 32));
    r.k = (int32_t)c[0];
    r.vec_ok = (int32_t)c[1];
    return r;
}

// Starts load instruction j (0 .. ROWS / 64 - 1) of this wave for one operand of one k-step.  `tile`
// points at (first row, first k) of the ROWS x 32 block, `dst` at its LDS region; both are the same
// for all lanes.
template <bool KF, int ROWS>
__device__ __forceinline__ void issue_one(const uint16_t* tile, int ld, char* dst, int wave, int lane, int j) {
    constexpr int NI = ROWS / 64;                            // instructions per wave and step
    const uint16_t* gp;
    if (KF) {
        // an instruction covers 16 rows; lane -> row lane / 4, slot lane % 4
        const int r = lane >> 2;
        const int c = (lane & 3) ^ ((r >> 2) & 3);
        gp = tile + (int64_t)(16 * (NI * wave + j)) * ld + (uint32_t)(r * ld + c * 8);
    } else {
        // an instruction covers 1024 / (2 ROWS) k-lines; lane -> line lane / LPL, slot lane % LPL
        constexpr int LPL = ROWS / 8, LPI = 64 / LPL;        // lanes per line, lines per instruction
        const int kk = LPI * j + lane / LPL;                 // line within the wave's 8; 8 * wave is 0 mod 4
        const int c = (lane % LPL) ^ ((kk & 3) << 2);
        gp = tile + (int64_t)(8 * wave + LPI * j) * ld + (uint32_t)((lane / LPL) * ld + c * 8);
    }
    __builtin_amdgcn_global_load_lds((glb_void_ptr)gp, (lds_void_ptr)(dst + (wave * NI + j) * 1024), 16, 0, 0);
}

// Per-lane part of the fragment address of an operand region of ROWS rows.
template <bool KF, int ROWS>
__device__ __forceinline__ uint32_t frag_lane_offset(int lane) {
    if (KF) {
        const int r32 = lane & 31, half = lane >> 5;
        return (uint32_t)(r32 * 64 + ((half ^ ((r32 >> 2) & 3)) << 4));
    }
    const int j = lane & 15, gq = lane >> 4, half = gq >> 1;
    const int x = (j >> 2) & 3;                                 // k & 3 of the line this lane addresses
    const int low2 = 2 * (gq & 1) + ((j & 3) >> 1);             // 16-byte chunk within the 32-row block
    return (uint32_t)((8 * half + (j >> 2)) * (2 * ROWS) + x * 64 + low2 * 16 + (j & 1) * 8);
}

// LDS reads of the pipeline are spelled as inline assembly: the compiler treats every LDS read
// it knows of as possibly touching what the in-flight global->LDS loads write and would wait for
// all of them (vmcnt 0) first, which is exactly what the stages are there to avoid.  The price is
// that the waits for these reads are ours too (wait_frags).
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}

// Registers of one fragment (8 consecutive k of the lane's row) while its read is in flight.
template <bool KF>
struct Frag {
    bf16x8 v;
    __device__ __forceinline__ void tie() { asm volatile("" : "+v"(v)); }
    __device__ __forceinline__ bf16x8 value() const { return v; }
};
template <>
struct Frag<false> {
    s16x4 lo, hi;
    __device__ __forceinline__ void tie() { asm volatile("" : "+v"(lo), "+v"(hi)); }
    __device__ __forceinline__ bf16x8 value() const {
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        const s16x8 x = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, x);
    }
};

// Starts the read of the fragment of 32-row block `blk` of an operand region of ROWS rows (LDS
// byte offset `region`) for substep ks (16 k each).
template <bool KF, int ROWS>
__device__ __forceinline__ void read_frag(Frag<KF>& f, uint32_t region, uint32_t lane_off, int blk, int ks) {
    if constexpr (KF) {
        const uint32_t addr = region + blk * 2048 + (lane_off ^ (uint32_t)(ks * 32));
        asm volatile("ds_read_b128 %0, %1" : "=v"(f.v) : "v"(addr));
    } else {
        constexpr int LB = 2 * ROWS;                            // bytes of a k-line
        const uint32_t addr = region + ks * 16 * LB + (blk >> 2) * 256 + (lane_off ^ (uint32_t)((blk & 3) * 64));
        asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(f.lo) : "v"(addr));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.hi) : "v"(addr), "n"(4 * LB));
    }
}

// Macro-tile 256 x 64 WNB: WNB = 4 has a CU to itself (four stages), WNB = 2 leaves room for two
// workgroups per CU (three stages each), which cover each other's first loads and result stores.
template <int WNB>
struct DlShape {
    static constexpr int kStages = WNB == 4 ? 4 : 3;
    static constexpr int kStageBytes = (256 + 64 * WNB) * kBK * 2;
    static constexpr int kLdsBytes = kStages * kStageBytes;
};

template <typename TO, bool AKF, bool BKF, int WNB>
__device__ __forceinline__ void dl_body(const GemmArgs& g, char* lds) {
    constexpr int WMB = 4, BM = 256, BN = 64 * WNB;
    constexpr int kStages = DlShape<WNB>::kStages;
    constexpr int kOpABytes = BM * kBK * 2, kStageBytes = DlShape<WNB>::kStageBytes;
    constexpr int NIA = BM / 64, NIB = BN / 64, kLoads = NIA + NIB;     // load instructions per wave and step
    constexpr int kFrags = WNB + WMB, kMfma = WNB * WMB;
    static_assert(4 * 32 * (32 * WMB + 4) * 4 <= kStages * kStageBytes, "result staging must fit the pipeline's LDS");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;

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
        // Position of the next k-step to load (all uniform).  Loads are started for every step of
        // the loop, needed or not, so that the count of loads in flight is the same at every wait:
        // once the last real step has been started the position stays where it is and the spare
        // loads fetch that step again into a stage nobody reads.
        int k0 = 0, chk = 0, lda = 0, ldb = 0, to_issue = T;
        const uint16_t* Ab = nullptr;
        const uint16_t* Bb = nullptr;
        const uint16_t* At = nullptr;
        const uint16_t* Bt = nullptr;
        auto set_chunk = [&](const ChunkS& ch) {
            chk = ch.k;
            lda = (int)ch.lda;
            ldb = (int)ch.ldb;
            Ab = reinterpret_cast<const uint16_t*>(ch.A) + (int64_t)bat * ch.strideA;
            Bb = reinterpret_cast<const uint16_t*>(ch.B) + (int64_t)bat * ch.strideB;
        };
        auto set_step = [&]() {
            At = AKF ? Ab + (int64_t)m0 * lda + k0 : Ab + m0 + (int64_t)k0 * lda;
            Bt = BKF ? Bb + (int64_t)n0 * ldb + k0 : Bb + n0 + (int64_t)k0 * ldb;
        };
        if (table) {
            set_chunk(sload_chunk(g.chunks + chunk_i));
        } else {
            ChunkS one;
            one.A = reinterpret_cast<uint64_t>(g.one_chunk.A); one.B = reinterpret_cast<uint64_t>(g.one_chunk.B);
            one.lda = g.one_chunk.lda; one.ldb = g.one_chunk.ldb;
            one.strideA = g.one_chunk.strideA; one.strideB = g.one_chunk.strideB;
            one.k = g.one_chunk.k; one.vec_ok = g.one_chunk.vec_ok;
            set_chunk(one);
        }
        set_step();
        // load instruction i (first those of A, then those of B) of the k-step at the current position
        auto load_one = [&](int stage, int i) {
            char* sa = lds + stage * kStageBytes;
            if (i < NIA) issue_one<AKF, BM>(At, lda, sa, wave, lane, i);
            else issue_one<BKF, BN>(Bt, ldb, sa + kOpABytes, wave, lane, i - NIA);
        };
        auto advance = [&]() {
            if (--to_issue > 0) {
                k0 += kBK;
                if (k0 >= chk) {
                    chunk_i++;
                    k0 = 0;
                    if (chunk_i < chunk_end) set_chunk(sload_chunk(g.chunks + chunk_i));
                }
                set_step();
            } else {
                to_issue = 1;
            }
        };
        for (int s = 0; s < kStages - 1; s++) {
#pragma unroll
            for (int i = 0; i < kLoads; i++) load_one(s, i);
            advance();
        }

        const uint32_t offA = frag_lane_offset<AKF, BM>(lane), offB = frag_lane_offset<BKF, BN>(lane);
        Frag<BKF> pf[2][WNB];
        Frag<AKF> qf[2][WMB];
        const uint32_t lds0 = lds_offset(lds);
        // fragment i (first the column blocks of B, then the row blocks of A) of a substep
        auto frag_one = [&](int buf, int stage, int ks, int i) {
            const uint32_t sa = lds0 + stage * kStageBytes;
            if (i < WNB) read_frag<BKF, BN>(pf[buf][i], sa + kOpABytes, offB, wn * WNB + i, ks);
            else read_frag<AKF, BM>(qf[buf][i - WNB], sa, offA, wm * WMB + i - WNB, ks);
        };
        // all fragment reads issued so far have landed; the matrix instructions on set `buf` stay behind this
        auto wait_frags = [&](int buf) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < WNB; i++) pf[buf][i].tie();
#pragma unroll
            for (int i = 0; i < WMB; i++) qf[buf][i].tie();
        };
        auto mfma_one = [&](int buf, int i) {
            const int bn = i / WMB, bm = i % WMB;
            acc[bn][bm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[buf][bm].value(), pf[buf][bn].value(), acc[bn][bm], 0, 0, 0);
        };
        // One substep: the matrix instructions on fragment set `buf`; under them the fragments of
        // the next substep are fetched into the other set and, with `with_loads`, the load
        // instructions of a k-step are started.  The pieces are dealt out evenly over the matrix
        // instructions and fenced so that they stay there.
        auto substep = [&](auto with_loads, int buf, int f_stage, int f_ks, int load_stage) {
            constexpr int kItems = kFrags + (decltype(with_loads)::value ? kLoads : 0);
            wait_frags(buf);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < kMfma; q++) {
                mfma_one(buf, q);
#pragma unroll
                for (int i = 0; i < kItems; i++) {
                    if (i * kMfma / kItems != q) continue;
                    if (i < kFrags) frag_one(buf ^ 1, f_stage, f_ks, i);
                    else load_one(load_stage, i - kFrags);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // step 0 has landed in this wave's part once only the loads of steps 1 .. kStages - 2 remain
        __builtin_amdgcn_s_waitcnt(wait_vm((kStages - 2) * kLoads));
        asm volatile("s_barrier" ::: "memory");
#pragma unroll
        for (int i = 0; i < kFrags; i++) frag_one(0, 0, 0, i);
        int stage = 0, next_stage = kStages - 1;
        for (int t = 0; t < T; t++) {
            const int stage1 = stage + 1 == kStages ? 0 : stage + 1;
            substep(std::false_type{}, 0, stage, 1, 0);
            // step t + 1 complete for everybody (loads of steps t + 2 .. t + kStages - 2 may remain),
            // and everybody done with the stage of step t - 1, which the next loads overwrite
            __builtin_amdgcn_s_waitcnt(wait_vm((kStages - 3) * kLoads));
            asm volatile("s_barrier" ::: "memory");
            // (after the last step the fragment reads hit a stage that holds no new data: in bounds
            // and unused)
            substep(std::true_type{}, 1, stage1, 0, next_stage);
            advance();
            next_stage = next_stage + 1 == kStages ? 0 : next_stage + 1;
            stage = stage1;
        }
        // nothing may still be on its way into LDS or into fragment registers when the results are staged
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");
    }

    float* stage = reinterpret_cast<float*>(lds) + wave * (32 * (32 * WMB + 4));
    const int m_base = m0 + wm * WMB * 32, n_base = n0 + wn * WNB * 32;
    if (task.partial) {
        write_tile<float, WMB, WNB>(stage, acc, static_cast<float*>(task.C) + (int64_t)bat * task.strideC, task.ldc, nullptr,
                                    1.f, 0.f, m_base, n_base, task.m, task.n, lane);
    } else {
        write_tile<TO, WMB, WNB>(stage, acc, static_cast<TO*>(task.C) + (int64_t)bat * task.strideC, task.ldc, task.bias,
                                 g.alpha, g.beta, m_base, n_base, task.m, task.n, lane);
    }
}

template <typename TO, bool AKF, bool BKF>
__global__ void __launch_bounds__(256) gemm_bf16_dl_kernel(const GemmArgs g) {
    __shared__ __attribute__((aligned(16))) char lds[DlShape<4>::kLdsBytes];
    dl_body<TO, AKF, BKF, 4>(g, lds);
}

// two workgroups per compute unit: at most 256 registers per lane
template <typename TO, bool AKF, bool BKF>
__global__ void __launch_bounds__(256, 2) gemm_bf16_dl_tall_kernel(const GemmArgs g) {
    __shared__ __attribute__((aligned(16))) char lds[DlShape<2>::kLdsBytes];
    dl_body<TO, AKF, BKF, 2>(g, lds);
}

using KernelFn = void (*)(const GemmArgs);

template <typename TO>
KernelFn kernel_of(int akf, int bkf, bool tall) {
    if (tall) {
        if (akf) return bkf ? gemm_bf16_dl_tall_kernel<TO, true, true> : gemm_bf16_dl_tall_kernel<TO, true, false>;
        return bkf ? gemm_bf16_dl_tall_kernel<TO, false, true> : gemm_bf16_dl_tall_kernel<TO, false, false>;
    }
    if (akf) return bkf ? gemm_bf16_dl_kernel<TO, true, true> : gemm_bf16_dl_kernel<TO, true, false>;
    return bkf ? gemm_bf16_dl_kernel<TO, false, true> : gemm_bf16_dl_kernel<TO, false, false>;
}

KernelFn kernel_of(int out_is_f32, int akf, int bkf, int cfg) {
    return out_is_f32 ? kernel_of<float>(akf, bkf, cfg == kCfgTall) : kernel_of<uint16_t>(akf, bkf, cfg == kCfgTall);
}

}  // namespace

int32_t launch_gemm_bf16_dl(hipStream_t st, int out_is_f32, int akf, int bkf, int cfg, const GemmArgs& g, int64_t nwg) {
    if (nwg <= 0) return NNT_OK;
    hipLaunchKernelGGL(kernel_of(out_is_f32, akf, bkf, cfg), dim3((unsigned)nwg), dim3(256), 0, st, g);
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int gemm_bf16_dl_occupancy(int out_is_f32, int akf, int bkf, int cfg) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel_of(out_is_f32, akf, bkf, cfg), 256, 0) != hipSuccess || n < 1) n = 1;
    return n;
}

}  // namespace nnt
