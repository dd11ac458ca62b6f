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
#include "gemm_dl_common.hpp"
#include "nntile_mi.h"

#include <type_traits>
#include <utility>

namespace nnt {

namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 32;                 // k-step

// Byte offset, from (first row, first k) of an operand's ROWS x 32 block, of what this lane
// fetches in load instruction j (0 .. ROWS / 64 - 1) of its wave; the data lands in LDS at
// (wave * ROWS / 64 + j) * 1024 + 16 * lane of the operand's region.
template <bool KF, int ROWS>
__device__ __forceinline__ uint32_t load_offset(int ld, int wave, int lane, int j) {
    constexpr int NI = ROWS / 64;                            // instructions per wave and step
    if (KF) {
        // an instruction covers 16 rows; lane -> row lane / 4, slot lane % 4
        const int r = lane >> 2;
        const int c = (lane & 3) ^ ((r >> 2) & 3);
        return (uint32_t)(((16 * (NI * wave + j) + r) * ld + c * 8) * 2);
    }
    // an instruction covers 1024 / (2 ROWS) k-lines; lane -> line lane / LPL, slot lane % LPL
    constexpr int LPL = ROWS / 8, LPI = 64 / LPL;            // lanes per line, lines per instruction
    const int kk = LPI * j + lane / LPL;                     // line within the wave's 8; 8 * wave is 0 mod 4
    const int c = (lane % LPL) ^ ((kk & 3) << 2);
    return (uint32_t)(((8 * wave + kk) * ld + c * 8) * 2);
}

// The same for a block of which only `rows` rows (a multiple of 8 when the row index is the
// contiguous one) and `kv` of the 32 k (a multiple of 8) exist: a lane whose 16 bytes lie outside
// fetches an existing vector of the block instead (row clamped to the last one, k or row group set
// back to the first), so that no address leaves the operand.  What lands in LDS for the missing
// rows only reaches results that are never stored; what lands for the missing k is multiplied by
// fragments that the kernel sets to zero.
template <bool KF, int ROWS>
__device__ __forceinline__ uint32_t load_offset_clamped(int ld, int wave, int lane, int j, int rows, int kv) {
    constexpr int NI = ROWS / 64;
    if (KF) {
        const int r = lane >> 2;
        int c = (lane & 3) ^ ((r >> 2) & 3);
        if (c * 8 >= kv) c = 0;
        const int row = min(16 * (NI * wave + j) + r, rows - 1);
        return (uint32_t)((row * ld + c * 8) * 2);
    }
    constexpr int LPL = ROWS / 8, LPI = 64 / LPL;
    const int kk = LPI * j + lane / LPL;
    int c = (lane % LPL) ^ ((kk & 3) << 2);
    if (c * 8 >= rows) c = 0;
    int line = 8 * wave + kk;
    if (line >= kv) line = 0;
    return (uint32_t)((line * ld + c * 8) * 2);
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

// Registers of one fragment (8 consecutive k of the lane's row) while its read is in flight.
template <bool KF>
struct Frag {
    bf16x8 v;
    __device__ __forceinline__ void tie() { asm volatile("" : "+v"(v)); }
    __device__ __forceinline__ bf16x8 value() const { return v; }
    // keeps the fragment (mask = ~0) or sets it to zero (mask = 0); only after its read has been waited for
    __device__ __forceinline__ void mask(uint32_t m) {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        u32x4 x = __builtin_bit_cast(u32x4, v);
        x &= m;
        v = __builtin_bit_cast(bf16x8, x);
    }
};
template <>
struct Frag<false> {
    s16x4 lo, hi;
    __device__ __forceinline__ void tie() { asm volatile("" : "+v"(lo), "+v"(hi)); }
    __device__ __forceinline__ void mask(uint32_t m) {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        u32x2 a = __builtin_bit_cast(u32x2, lo), b = __builtin_bit_cast(u32x2, hi);
        a &= m;
        b &= m;
        lo = __builtin_bit_cast(s16x4, a);
        hi = __builtin_bit_cast(s16x4, b);
    }
    __device__ __forceinline__ bf16x8 value() const {
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        const s16x8 x = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, x);
    }
};

// Starts the read of fragment B (the wave's B-th 32-row block) of an operand for substep KS (16 k
// each).  `addr` is the LDS byte address of the stage plus everything that depends on the lane
// and the wave (see FragAddr); the rest is an immediate, REGION being the operand's offset inside
// the stage.
template <bool KF, int ROWS, int REGION, int B, int KS>
__device__ __forceinline__ void read_frag(Frag<KF>& f, uint32_t addr) {
    if constexpr (KF) {
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.v) : "v"(addr), "n"(REGION + B * 2048));
    } else {
        constexpr int LB = 2 * ROWS;                            // bytes of a k-line
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.lo) : "v"(addr), "n"(REGION + KS * 16 * LB));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.hi) : "v"(addr), "n"(REGION + KS * 16 * LB + 4 * LB));
    }
}

// Lane- and wave-dependent parts of the fragment addresses of one operand, relative to the stage.
// k-contiguous operand: one value per substep (the substep flips bit 5 of the lane's offset), the
// block index is an immediate.  Row-contiguous operand: one value per block (the block index
// enters through an xor), the substep is an immediate.
template <bool KF, int ROWS, int NB>
struct FragAddr {
    static constexpr int N = KF ? 2 : NB;
    uint32_t v[N];
    __device__ __forceinline__ void init(int lane, int first_blk) {
        const uint32_t lo = frag_lane_offset<KF, ROWS>(lane);
        if constexpr (KF) {
            v[0] = lo + first_blk * 2048;
            v[1] = (lo ^ 32u) + first_blk * 2048;
        } else {
#pragma unroll
            for (int b = 0; b < NB; b++) v[b] = (lo ^ (uint32_t)(((first_blk + b) & 3) * 64)) + ((first_blk + b) >> 2) * 256;
        }
    }
    template <int B, int KS>
    __device__ __forceinline__ uint32_t at(uint32_t stage_addr) const { return stage_addr + v[KF ? KS : B]; }
};

// WM waves along m (2: the four waves as 2 x 2, 256 rows; 1: side by side, 128 rows), each 128 rows x 32 WNB columns.
template <int WNB, int WM = 2>
struct DlShape {
    static constexpr int BM = 128 * WM, BN = 32 * WNB * (4 / WM);
    static constexpr int kStages = (WNB == 4 || WM == 1) ? 5 : 3;
    static constexpr int kStageBytes = (BM + BN) * kBK * 2;
    static constexpr int kLdsBytes = kStages * kStageBytes;
};

// RAG: the macro-tile may end inside its C tile (rows of the operands beyond the tile's edge are
// not loaded, see load_offset_clamped; the epilogue stores nothing for them) and chunk lengths are
// multiples of 8 instead of 32 (the last k-step of such a chunk is short: the fragments of the A
// operand that stand for k beyond it are set to zero before the matrix instructions).
template <typename TO, bool AKF, bool BKF, int WNB, bool RAG = false, int WM = 2>
__device__ __forceinline__ void dl_body(const GemmArgs& g, char* lds) {
    constexpr int WMB = 4, BM = DlShape<WNB, WM>::BM, BN = DlShape<WNB, WM>::BN;
    constexpr int kStages = DlShape<WNB, WM>::kStages;
    constexpr int kOpABytes = BM * kBK * 2, kStageBytes = DlShape<WNB, WM>::kStageBytes;
    constexpr int NIA = BM / 64, NIB = BN / 64, kLoads = NIA + NIB;     // load instructions per wave and step
    constexpr int kFrags = WNB + WMB, kMfma = WNB * WMB;
#ifndef NNT_FRAG_SPAN_NUM
#define NNT_FRAG_SPAN_NUM 2
#endif
    constexpr int kFragSpan = kMfma * NNT_FRAG_SPAN_NUM / 4;
    // The 256 x 256 shape starts its loads two k-steps at a time (see the loop below); its chunks
    // must be multiples of 64 long.
    constexpr bool kPaired = WNB == 4 && WM == 2;
    static_assert(!kPaired || kStages == 5, "the paired schedule needs five stages");
    static_assert(!(kPaired && RAG), "short k-steps need the schedule that starts its loads one step at a time");
    static_assert(4 * 32 * (32 * WMB + 4) * 4 <= kStages * kStageBytes, "result staging must fit the pipeline's LDS");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = WM == 2 ? wave & 1 : 0, wn = WM == 2 ? wave >> 1 : wave;

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
        for (int c = 0; c < nch; c++) T += (sload_chunk(g.chunks + chunk_i + c).k + (RAG ? kBK - 1 : 0)) / kBK;
    } else if (task.nchunk > 0) {
        T = (g.one_chunk.k + (RAG ? kBK - 1 : 0)) / kBK;
    }
    T = __builtin_amdgcn_readfirstlane(T);

    if (T > 0) {
        const int chunk_first = chunk_i;
        const int chunk_end = chunk_i + __builtin_amdgcn_readfirstlane(task.nchunk);
        // Position of the next k-step to load.  A lane's loads of a step are `base + offset` with a
        // uniform base that moves on by a fixed amount per step and per-lane byte offsets that only
        // change with the chunk (they depend on the leading dimension).  Loads are started for every
        // step of the loop, needed or not, so that the count of loads in flight is the same at every
        // wait: once the last real step has been started the position stays where it is and the spare
        // loads fetch that step again into a stage nobody reads.
        int k0 = 0, chk = 0, to_issue = T;
        const char* baseA = nullptr;
        const char* baseB = nullptr;
        int64_t advA = 0, advB = 0;
        uint32_t voffA[NIA], voffB[NIB];
        uint32_t toffA[RAG ? NIA : 1], toffB[RAG ? NIB : 1];      // offsets for the short last step of the chunk
        const int rowsA = RAG ? min(BM, task.m - m0) : BM, rowsB = RAG ? min(BN, task.n - n0) : BN;
        auto set_chunk = [&](const ChunkS& ch) {
            chk = ch.k;
            const int lda = (int)ch.lda, ldb = (int)ch.ldb;
            const uint16_t* Ab = reinterpret_cast<const uint16_t*>(ch.A) + (int64_t)bat_lo * ch.strideA + (int64_t)bat_hi * ch.strideA2;
            const uint16_t* Bb = reinterpret_cast<const uint16_t*>(ch.B) + (int64_t)bat_lo * ch.strideB + (int64_t)bat_hi * ch.strideB2;
            baseA = reinterpret_cast<const char*>(AKF ? Ab + (int64_t)m0 * lda : Ab + m0);
            baseB = reinterpret_cast<const char*>(BKF ? Bb + (int64_t)n0 * ldb : Bb + n0);
            advA = AKF ? kBK * 2 : (int64_t)kBK * lda * 2;
            advB = BKF ? kBK * 2 : (int64_t)kBK * ldb * 2;
            if constexpr (RAG) {
                const int kt = chk % kBK ? chk % kBK : kBK;
#pragma unroll
                for (int j = 0; j < NIA; j++) {
                    voffA[j] = load_offset_clamped<AKF, BM>(lda, wave, lane, j, rowsA, kBK);
                    toffA[j] = load_offset_clamped<AKF, BM>(lda, wave, lane, j, rowsA, kt);
                }
#pragma unroll
                for (int j = 0; j < NIB; j++) {
                    voffB[j] = load_offset_clamped<BKF, BN>(ldb, wave, lane, j, rowsB, kBK);
                    toffB[j] = load_offset_clamped<BKF, BN>(ldb, wave, lane, j, rowsB, kt);
                }
            } else {
#pragma unroll
                for (int j = 0; j < NIA; j++) voffA[j] = load_offset<AKF, BM>(lda, wave, lane, j);
#pragma unroll
                for (int j = 0; j < NIB; j++) voffB[j] = load_offset<BKF, BN>(ldb, wave, lane, j);
            }
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
        // load instruction i (first those of A, then those of B) of the k-step at the current position
        auto load_one = [&](int stage, int i) {
            char* sa = lds + stage * kStageBytes;
            const bool short_step = RAG && chk - k0 < kBK;       // uniform: the step at the current position is the chunk's short last one
            if (i < NIA) {
                const uint32_t off = short_step ? toffA[RAG ? i : 0] : voffA[i];
                __builtin_amdgcn_global_load_lds((glb_void_ptr)(baseA + off), (lds_void_ptr)(sa + (wave * NIA + i) * 1024), 16, 0, 0);
            } else {
                const int j = i - NIA;
                const uint32_t off = short_step ? toffB[RAG ? j : 0] : voffB[j];
                __builtin_amdgcn_global_load_lds((glb_void_ptr)(baseB + off), (lds_void_ptr)(sa + kOpABytes + (wave * NIB + j) * 1024), 16, 0, 0);
            }
        };
        auto advance = [&]() {
            if (--to_issue > 0) {
                k0 += kBK;
                if (k0 >= chk) {
                    chunk_i++;
                    k0 = 0;
                    if (chunk_i < chunk_end) set_chunk(sload_chunk(g.chunks + chunk_i));
                } else {
                    baseA += advA;
                    baseB += advB;
                }
            } else {
                to_issue = 1;
            }
        };
        // Paired schedule: load instruction i (0 .. 2 kLoads - 1) of the two k-steps at the current
        // position.  The two steps take the two 64-byte halves of the same 128-byte lines of a
        // k-contiguous operand; asking for both halves back to back lets the second request ride on
        // the first one's miss (measured: half-line requests issued a step apart stall the wave
        // at issue and cost about a fifth of the matrix rate, paired ones cost nothing).
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
        // moves the position on by two k-steps (chunks are multiples of 64 long)
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
        if constexpr (kPaired) {
#pragma unroll
            for (int i = 0; i < 2 * kLoads; i++) load_pair_item(0, 1, i);
            advance2();
#pragma unroll
            for (int i = 0; i < 2 * kLoads; i++) load_pair_item(2, 3, i);
            advance2();
        } else {
            for (int s = 0; s < kStages - 1; s++) {
#pragma unroll
                for (int i = 0; i < kLoads; i++) load_one(s, i);
                advance();
            }
        }

        FragAddr<AKF, BM, WMB> fa;
        FragAddr<BKF, BN, WNB> fb;
        fa.init(lane, wm * WMB);
        fb.init(lane, wn * WNB);
        Frag<BKF> pf[2][WNB];
        Frag<AKF> qf[2][WMB];
        const uint32_t lds0 = lds_offset(lds);
        // fragment I (first the column blocks of B, then the row blocks of A) of substep KS of a stage
        auto frag_one = [&](auto I, auto KS, int buf, uint32_t stage_addr) {
            constexpr int i = decltype(I)::value, ks = decltype(KS)::value;
            if constexpr (i < WNB) read_frag<BKF, BN, kOpABytes, i, ks>(pf[buf][i], fb.template at<i, ks>(stage_addr));
            else read_frag<AKF, BM, 0, i - WNB, ks>(qf[buf][i - WNB], fa.template at<i - WNB, ks>(stage_addr));
        };
        // all fragment reads issued so far have landed; the matrix instructions on set `buf` stay behind this
        auto wait_frags = [&](int buf) {
#ifndef NNT_PROBE_NO_LGKM
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#endif
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
        // substep F_KS of the stage at `f_addr` are fetched into the other set and NL load
        // instructions are started through `load(i)`.  The pieces are dealt out evenly over the
        // matrix instructions and fenced so that they stay there.
        // RAG: k that the step under the matrix instructions really has (32 except in the short last
        // step of a chunk), and a cursor over the chunk lengths on the computing side
        // (it starts at the task's first chunk: the loading side has already moved on, past that chunk
        // when it is no longer than the steps the prologue starts)
        int kv_now = kBK, c_rem = 0, c_chunk = chunk_first;
        if constexpr (RAG) {
            c_rem = table ? sload_chunk(g.chunks + c_chunk).k : g.one_chunk.k;
            kv_now = min(kBK, c_rem);
        }
        auto next_step_k = [&]() {
            c_rem -= kv_now;
            if (c_rem <= 0 && ++c_chunk < chunk_end) c_rem = sload_chunk(g.chunks + c_chunk).k;
            kv_now = c_rem > 0 ? min(kBK, c_rem) : kBK;       // (past the last step: nothing is multiplied any more)
        };
        const int lane_k8 = (lane >> 5) * 8;                  // first k, within a substep of 16, of the lane's fragments
        auto substep = [&](auto NL, auto F_KS, int buf, uint32_t f_addr, auto&& load, int ks_now = 0) {
            constexpr int kItems = kFrags + decltype(NL)::value;
            wait_frags(buf);
            if constexpr (RAG) {
                if (kv_now < kBK) {
                    // short step: the A fragments that stand for k >= kv_now become zero
                    const uint32_t keep = 16 * ks_now + lane_k8 < kv_now ? 0xffffffffu : 0u;
#pragma unroll
                    for (int i = 0; i < WMB; i++) qf[buf][i].mask(keep);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            static_for<kMfma>([&](auto Q) {
                constexpr int q = decltype(Q)::value;
                mfma_one(buf, q);
                static_for<kItems>([&](auto I) {
                    constexpr int i = decltype(I)::value;
                    // fragment reads go under the first kFragSpan matrix instructions (their latency
                    // has the rest of the substep to pass), load instructions are spread over all of them
                    constexpr int slot = i < kFrags ? i * kFragSpan / kFrags : (i - kFrags) * kMfma / (kItems > kFrags ? kItems - kFrags : 1);
                    if constexpr (slot == q) {
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
        if constexpr (kPaired) {
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
#ifndef NNT_PROBE_NO_VM
                __builtin_amdgcn_s_waitcnt(wait_vm(2 * kLoads));
#endif
#ifndef NNT_PROBE_NO_BAR
                asm volatile("s_barrier" ::: "memory");
#endif
                substep(None{}, KS0{}, 1, stage_addr(s1), no_load);
                substep(None{}, KS1{}, 0, stage_addr(s1), no_load);
                // pair u + 1 complete for everybody, and everybody done with the stages of steps
                // 2u - 1 and 2u, which the next pair of loads overwrites
#ifndef NNT_PROBE_NO_VM
                __builtin_amdgcn_s_waitcnt(wait_vm(0));
#endif
#ifndef NNT_PROBE_NO_BAR
                asm volatile("s_barrier" ::: "memory");
#endif
                // (after the last pair the fragment reads hit a stage that holds no new data: in
                // bounds and unused)
                substep(std::integral_constant<int, 2 * kLoads>{}, KS0{}, 1, stage_addr(s2), [&](int i) { load_pair_item(s4, st, i); });
                advance2();
                st = s2;
            }
        } else {
            // step 0 has landed in this wave's part once only the loads of steps 1 .. kStages - 2 remain
            __builtin_amdgcn_s_waitcnt(wait_vm((kStages - 2) * kLoads));
            asm volatile("s_barrier" ::: "memory");
            static_for<kFrags>([&](auto I) { frag_one(I, KS0{}, 0, lds0); });
            int stage = 0, next_stage = kStages - 1;
            for (int t = 0; t < T; t++) {
                const int stage1 = next_of(stage);
                substep(None{}, KS1{}, 0, stage_addr(stage), no_load, 0);
                // step t + 1 complete for everybody (loads of steps t + 2 .. t + kStages - 2 may
                // remain), and everybody done with the stage of step t - 1, which the next loads overwrite
                __builtin_amdgcn_s_waitcnt(wait_vm((kStages - 3) * kLoads));
                asm volatile("s_barrier" ::: "memory");
                // (after the last step the fragment reads hit a stage that holds no new data: in
                // bounds and unused)
                substep(std::integral_constant<int, kLoads>{}, KS0{}, 1, stage_addr(stage1), [&](int i) { load_one(next_stage, i); }, 1);
                if constexpr (RAG) next_step_k();
                advance();
                next_stage = next_of(next_stage);
                stage = stage1;
            }
        }
        // nothing may still be on its way into LDS or into fragment registers when the results are staged
        // (the fragment registers are named once more behind the wait, so that none of them is handed to
        // another value while the last, unused reads are still filling them)
        wait_frags(0);
        wait_frags(1);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");
    }

    float* stage = reinterpret_cast<float*>(lds) + wave * (32 * (32 * WMB + 4));
    const int m_base = m0 + wm * WMB * 32, n_base = n0 + wn * WNB * 32;
    if (task.partial) {
        write_tile<float, WMB, WNB>(stage, acc, static_cast<float*>(task.C) + (int64_t)bat_lo * task.strideC + (int64_t)bat_hi * task.strideC2, task.ldc, nullptr,
                                    1.f, 0.f, m_base, n_base, task.m, task.n, lane);
    } else {
        write_tile<TO, WMB, WNB>(stage, acc, static_cast<TO*>(task.C) + (int64_t)bat_lo * task.strideC + (int64_t)bat_hi * task.strideC2, task.ldc, task.bias,
                                 g.alpha, g.beta, m_base, n_base, task.m, task.n, lane, task.cin_off);
    }
}

template <typename TO, bool AKF, bool BKF>
__global__ void __launch_bounds__(256) gemm_bf16_dl_kernel(const GemmArgs g) {
    __shared__ __attribute__((aligned(16))) char lds[DlShape<4>::kLdsBytes];
    dl_body<TO, AKF, BKF, 4>(g, lds);
}

// two workgroups per compute unit: at most 256 registers per lane
template <typename TO, bool AKF, bool BKF, bool RAG>
__global__ void __launch_bounds__(256, 2) gemm_bf16_dl_tall_kernel(const GemmArgs g) {
    __shared__ __attribute__((aligned(16))) char lds[DlShape<2>::kLdsBytes];
    dl_body<TO, AKF, BKF, 2, RAG>(g, lds);
}

// 128 x 128 macro-tiles for products with few rows (m = head size: the other operand is the score-shaped one and
// the kernel streams it): the four waves side by side, 128 rows x 32 columns each, five stages of 16 KB so that
// the loads of four k-steps are in flight, two workgroups per compute unit.  Always the ragged variant (m = 64
// is half a macro-tile; sequence tiles need not be multiples of 128).
template <typename TO, bool AKF, bool BKF>
__global__ void __launch_bounds__(256, 2) gemm_bf16_dl_wide_kernel(const GemmArgs g) {
    __shared__ __attribute__((aligned(16))) char lds[DlShape<1, 1>::kLdsBytes];
    dl_body<TO, AKF, BKF, 1, true, 1>(g, lds);
}

using KernelFn = void (*)(const GemmArgs);

template <typename TO>
KernelFn wide_kernel_of(int akf, int bkf) {
    if (akf) return bkf ? gemm_bf16_dl_wide_kernel<TO, true, true> : gemm_bf16_dl_wide_kernel<TO, true, false>;
    return bkf ? gemm_bf16_dl_wide_kernel<TO, false, true> : gemm_bf16_dl_wide_kernel<TO, false, false>;
}

template <typename TO, bool RAG>
KernelFn tall_kernel_of(int akf, int bkf) {
    if (akf) return bkf ? gemm_bf16_dl_tall_kernel<TO, true, true, RAG> : gemm_bf16_dl_tall_kernel<TO, true, false, RAG>;
    return bkf ? gemm_bf16_dl_tall_kernel<TO, false, true, RAG> : gemm_bf16_dl_tall_kernel<TO, false, false, RAG>;
}

template <typename TO>
KernelFn kernel_of(int akf, int bkf, bool tall, bool ragged) {
    if (tall) return ragged ? tall_kernel_of<TO, true>(akf, bkf) : tall_kernel_of<TO, false>(akf, bkf);
    if (akf) return bkf ? gemm_bf16_dl_kernel<TO, true, true> : gemm_bf16_dl_kernel<TO, true, false>;
    return bkf ? gemm_bf16_dl_kernel<TO, false, true> : gemm_bf16_dl_kernel<TO, false, false>;
}

KernelFn kernel_of(int out_is_f32, int akf, int bkf, int cfg, bool ragged) {
    if (cfg == kCfgWide) return out_is_f32 ? wide_kernel_of<float>(akf, bkf) : wide_kernel_of<uint16_t>(akf, bkf);
    return out_is_f32 ? kernel_of<float>(akf, bkf, cfg == kCfgTall, ragged) : kernel_of<uint16_t>(akf, bkf, cfg == kCfgTall, ragged);
}

}  // namespace

int32_t launch_gemm_bf16_dl(hipStream_t st, int out_is_f32, int akf, int bkf, int cfg, bool ragged, const GemmArgs& g, int64_t nwg) {
    if (nwg <= 0) return NNT_OK;
    if (ragged && cfg != kCfgTall && cfg != kCfgWide) return NNT_EINVAL;
    hipLaunchKernelGGL(kernel_of(out_is_f32, akf, bkf, cfg, ragged), dim3((unsigned)nwg), dim3(256), 0, st, g);
    return hipGetLastError() == hipSuccess ? NNT_OK : NNT_EHIP;
}

int gemm_bf16_dl_occupancy(int out_is_f32, int akf, int bkf, int cfg) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel_of(out_is_f32, akf, bkf, cfg, false), 256, 0) != hipSuccess || n < 1) n = 1;
    return n;
}

}  // namespace nnt
