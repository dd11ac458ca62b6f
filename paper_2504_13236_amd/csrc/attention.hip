// Fused tile attention (section 3, attention layer and SoftMax): scores, causal
// mask, softmax over the keys and the product with the values in one kernel per
// direction, without ever forming the N_s x N_s tensor.
//
//   forward   B[i,q] = sum_k V[i,k] P[k,q],  P = softmax_k(scale * sum_i K[i,k] Q[i,q])
//   backward  dV[i,k] = sum_q dB[i,q] P[k,q]
//             dA[k,q] = P[k,q] (sum_i V[i,k] dB[i,q] - D[q]),  D[q] = sum_i dB[i,q] B[i,q]
//             dQ[i,q] = scale sum_k K[i,k] dA[k,q],  dK[i,k] = scale sum_q Q[i,q] dA[k,q]
//
// for every (batch, head) pair.  The forward pass walks the key tiles of a query
// block and carries the paper's running column statistics (maximum, sum of shifted
// exponentials) from tile to tile, rescaling the partial result whenever the maximum
// moves; it leaves the final statistics for the backward pass, which recomputes the
// probabilities from them instead of reading them from memory.
//
// Work split.  A workgroup owns 128 rows of one sequence tile (queries in the
// forward and dQ kernels, keys in the dK/dV kernel), 32 per wavefront, and streams
// blocks of 64 rows of the other kind through LDS, double-buffered, one barrier per
// block.  Every product is a chain of 32x32 matrix instructions whose B operand sits
// in registers (the wavefront's own rows, or the probabilities it has just computed:
// the accumulator layout of a 32x32 result, lane = column, is the B layout of the
// next product) and whose A operand is read from LDS.  Rows beyond a tile's extent
// are loaded as zeros and masked, so ragged tiles need no separate path.
#include "device_util.hpp"
#include "internal.hpp"

#include <cmath>
#include <type_traits>

namespace nnt {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWgRows = 128;   // rows owned by a workgroup
constexpr int kBlk = 64;       // rows streamed per iteration
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegInf = -__builtin_huge_valf();

// The tensors of one call: all are (H, N_s, N_b, N_h), tiled alike along the last three axes.
struct AttnGeom {
    int H, Ns, Nb, Nh;
    int bs, bb, bh;      // base tile along sequence, batch, head
    int gs, gb, gh;      // tiles along them
    int nblk;            // workgroup row blocks per sequence tile
    int nstep;           // streamed blocks per sequence tile
    int tile0;           // first sequence tile this launch covers
    int causal;
    float scale;
    // Operands that are windows on tensors [parts * N_h * H, N_s, N_b] with the heads side by side along the first
    // axis (win = 1; the statistics stay an ordinary tensor, to which bh and gh then belong): `pitch` elements
    // between the rows of consecutive positions (H otherwise), `hp` heads per row tile.
    int win, pitch, hp;
};

// Where a windowed operand starts in its tensor: first row tile of its part, row tiles of the tensor.
struct Win { int im0, g0; };

struct Slab {
    int64_t off;   // where (0, 0, b, j) sits in its tile, counted in rows (a row = the first-axis elements of one position)
    int tile;      // tile number
    int ext;       // extent of the tile along the sequence axis
};

// The part of a slab lookup that depends on (batch b, head j) only.
struct Pair {
    int tile;      // tile number of sequence tile 0 for this pair
    int rows;      // (b, j)'s position among the pairs of its tile: its slab starts rows * ext rows into the tile
};
__device__ __forceinline__ Pair pair_of(const AttnGeom& g, int b, int j) {
    const int tb = b / g.bb, tj = j / g.bh;
    const int eb = min(g.bb, g.Nb - tb * g.bb);
    Pair p;
    p.tile = g.gs * (tb + g.gb * tj);
    p.rows = (b - tb * g.bb) + eb * (j - tj * g.bh);
    return p;
}
// where the rows of that pair in sequence tile l live; `off` counts rows of the slab's first axis
__device__ __forceinline__ Slab slab_of(const AttnGeom& g, const Pair& p, int l) {
    Slab s;
    s.ext = min(g.bs, g.Ns - l * g.bs);
    s.tile = l + p.tile;
    s.off = (int64_t)s.ext * p.rows;
    return s;
}

template <typename T>
__device__ __forceinline__ T* rows_of(void* const* tiles, const Slab& s, int width) {
    return static_cast<T*>(tiles[s.tile]) + s.off * width;
}
// Row 0 of (batch b, head j) in sequence tile `s` of a data operand; its rows are g.pitch elements apart.
template <typename T>
__device__ __forceinline__ T* rows_win(void* const* tiles, const AttnGeom& g, const Win& w, const Pair& pr, const Slab& s, int b, int j) {
    if (!g.win) return static_cast<T*>(tiles[s.tile]) + s.off * g.H;
    const int tb = b / g.bb, l = s.tile - pr.tile, hl = j / g.hp;
    const int tile = (w.im0 + hl) + w.g0 * (l + g.gs * tb);
    return static_cast<T*>(tiles[tile]) + (j - hl * g.hp) * g.H + (int64_t)g.pitch * ((int64_t)s.ext * (b - tb * g.bb));
}

// ---------------------------------------------------------------- element-type traits
// What differs between the two storage types: how a block of 64 streamed rows sits in LDS, how a
// lane keeps its own row, and the two kinds of products.
//
//   rows_times_own   acc[r][c] += sum_i block[32 sub + r][i] * own[c][i]      (32 x 32, contraction over
//                    the first axis; A operand read row-wise from LDS, B operand = the lane's own row)
//   cols_times_acc   out[rb][i][c] += sum_r block[32 sub + r][32 rb + i] * p[r][c]   (contraction over the
//                    block's rows; p comes from accumulator registers: register r of lane half hh holds
//                    row acc_row(r, hh), and the A operand is read from LDS in that same order)

__device__ __forceinline__ int acc_row(int r, int hh) { return 8 * (r / 4) + 4 * hh + (r % 4); }
// the part of acc_row that is known at compile time: a bound `row < lim` on acc_row(r, hh) is the
// per-lane bound `acc_row0(r) < lim - 4 hh`, one comparison with a constant per register
__device__ __forceinline__ constexpr int acc_row0(int r) { return 8 * (r / 4) + (r % 4); }

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; i++) z[i] = 0.f;
    return z;
}

template <int H_> struct F32Traits {
    static constexpr int H = H_;
    using T = float;
    using Vec = float4;                               // 16 bytes of a row
    static constexpr int kPer = 4;                    // elements per Vec
    static constexpr int kVec = H / 16;               // Vec per thread per block (64 rows x H / 4 over 256 threads)
    // v_mfma_f32_32x32x2_f32: a lane supplies one element per instruction, half hh the k index hh.
    // Row pitch H + 4: rows stay 16-byte aligned, so a lane fetches four k-steps of its row with one
    // 128-bit read, and 16 lanes (rows r .. r+15, 4 r + c modulo 64) cover all 64 banks.
    static constexpr int LD = H + 4;
    // pitch for a block that is only read column-wise: puts the two lane halves 32 banks apart
    static constexpr int LD_COLS = H + 8;
    static constexpr int kDkvBlocks = 2;
    struct Own { float v[H / 2]; };                   // elements s + (H/2) hh of the lane's row
    struct Packed { f32x16 v; };

    static __device__ __forceinline__ Vec zero_vec() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    template <int LDX>
    static __device__ __forceinline__ void put(T* lds, int row, int c, const Vec& x) {
        T* d = lds + row * LDX + c * kPer;
        if constexpr (LDX % 4 == 0) {
            *reinterpret_cast<Vec*>(d) = x;
        } else {
            d[0] = x.x; d[1] = x.y; d[2] = x.z; d[3] = x.w;
        }
    }
    static __device__ __forceinline__ void load_own(const T* slab, int pitch, int row, int hh, bool valid, Own& o) {
        const float4* p = reinterpret_cast<const float4*>(slab + (int64_t)row * pitch + (H / 2) * hh);
#pragma unroll
        for (int s4 = 0; s4 < H / 8; s4++) {
            const float4 x = valid ? p[s4] : make_float4(0.f, 0.f, 0.f, 0.f);
            o.v[4 * s4 + 0] = x.x; o.v[4 * s4 + 1] = x.y; o.v[4 * s4 + 2] = x.z; o.v[4 * s4 + 3] = x.w;
        }
    }
    // sum over the first axis of a[i] * b[i] restricted to this lane's half of the row
    static __device__ __forceinline__ float dot_own(const Own& a, const Own& b) {
        float d = 0.f;
#pragma unroll
        for (int k = 0; k < H / 2; k++) d += a.v[k] * b.v[k];
        return d;
    }
    template <int LDX>
    static __device__ __forceinline__ f32x16 rows_times_own(const T* lds, int sub, int ln, int hh, const Own& o) {
        static_assert(LDX % 4 == 0, "128-bit fragment reads need 16-byte aligned rows");
        const float4* p = reinterpret_cast<const float4*>(lds + (32 * sub + ln) * LDX + (H / 2) * hh);
        f32x16 acc = zero16();
#pragma unroll
        for (int k4 = 0; k4 < H / 8; k4++) {
            const float4 a = p[k4];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, o.v[4 * k4], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, o.v[4 * k4 + 1], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, o.v[4 * k4 + 2], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, o.v[4 * k4 + 3], acc, 0, 0, 0);
        }
        return acc;
    }
    static __device__ __forceinline__ void pack(const f32x16& x, Packed& pk) { pk.v = x; }
    static __device__ __forceinline__ void set(Packed& pk, int r, float x) { pk.v[r] = x; }
    template <int LDX>
    static __device__ __forceinline__ void cols_times_acc(f32x16 (&out)[H / 32], const T* lds, int sub, int lane, const Packed& pk) {
        const int ln = lane & 31, hh = lane >> 5;
#pragma unroll
        for (int r = 0; r < 16; r++)
#pragma unroll
            for (int rb = 0; rb < H / 32; rb++)
                out[rb] = __builtin_amdgcn_mfma_f32_32x32x2f32(lds[(32 * sub + acc_row(r, hh)) * LDX + 32 * rb + ln], pk.v[r], out[rb], 0, 0, 0);
    }
    static __device__ __forceinline__ void store4(T* p, float a, float b, float c, float d) {
        *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
    }
};

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

template <int H_> struct Bf16Traits {
    static constexpr int H = H_;
    using T = bf16_t;
    using Vec = uint4;
    static constexpr int kPer = 8;
    static constexpr int kVec = H / 32;               // 64 rows x H / 8 vectors over 256 threads
    // v_mfma_f32_32x32x16_bf16: a lane supplies 8 consecutive k per instruction, half hh the k indices 8 hh ..
    // Row-wise fragments are 16-byte reads of rows 144 (272) bytes apart: 16 lanes cover all 64 banks.
    static constexpr int LD = H + 8;
    // Column-wise fragments are transposing reads (ds_read_b64_tr_b16) of 4 rows x 64 bytes per half
    // wave: rows 64 bytes apart modulo 256 keep the four rows on different banks.
    static constexpr int LD_COLS = H + 32;
    static constexpr int kDkvBlocks = H == 64 ? 2 : 1;
    struct Own { bf16x8 v[H / 16]; };                 // elements 16 s + 8 hh .. + 7 of the lane's row
    struct Packed { bf16x8 v[2]; };                   // registers 8 m .. 8 m + 7 of an accumulator, rounded

    static __device__ __forceinline__ Vec zero_vec() { return make_uint4(0u, 0u, 0u, 0u); }
    template <int LDX>
    static __device__ __forceinline__ void put(T* lds, int row, int c, const Vec& x) {
        *reinterpret_cast<Vec*>(lds + row * LDX + c * kPer) = x;
    }
    static __device__ __forceinline__ void load_own(const T* slab, int pitch, int row, int hh, bool valid, Own& o) {
        const uint4* p = reinterpret_cast<const uint4*>(slab + (int64_t)row * pitch + 8 * hh);
#pragma unroll
        for (int s = 0; s < H / 16; s++) {
            const uint4 x = valid ? p[2 * s] : make_uint4(0u, 0u, 0u, 0u);
            o.v[s] = __builtin_bit_cast(bf16x8, x);
        }
    }
    static __device__ __forceinline__ float dot_own(const Own& a, const Own& b) {
        float d = 0.f;
#pragma unroll
        for (int s = 0; s < H / 16; s++)
#pragma unroll
            for (int e = 0; e < 8; e++) d += (float)a.v[s][e] * (float)b.v[s][e];
        return d;
    }
    template <int LDX>
    static __device__ __forceinline__ f32x16 rows_times_own(const T* lds, int sub, int ln, int hh, const Own& o) {
        const T* p = lds + (32 * sub + ln) * LDX + 8 * hh;
        f32x16 acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(p), o.v[0], zero16(), 0, 0, 0);
#pragma unroll
        for (int s = 1; s < H / 16; s++)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(p + 16 * s), o.v[s], acc, 0, 0, 0);
        return acc;
    }
    static __device__ __forceinline__ void pack(const f32x16& x, Packed& pk) {
#pragma unroll
        for (int m = 0; m < 2; m++)
#pragma unroll
            for (int e = 0; e < 8; e++) pk.v[m][e] = (__bf16)x[8 * m + e];
    }
    static __device__ __forceinline__ void set(Packed& pk, int r, float x) { pk.v[r / 8][r % 8] = (__bf16)x; }
    template <int LDX>
    static __device__ __forceinline__ void cols_times_acc(f32x16 (&out)[H / 32], const T* lds, int sub, int lane, const Packed& pk) {
        // Accumulator registers 8 m + e of half hh are the rows 16 m + 8 (e / 4) + 4 hh + e % 4: two runs of
        // four consecutive rows, one transposing read each.  In such a read the 16 lanes of a group fetch
        // 8 bytes each -- lane j the columns 4 (j % 4) .. + 3 of row j / 4 of a 4 x 16 patch -- and lane j
        // receives the four rows of column j.
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        const int j = lane & 15, grp = lane >> 4, hh = grp >> 1;
        const T* base = lds + (32 * sub + 4 * hh + (j >> 2)) * LDX + 16 * (grp & 1) + 4 * (j & 3);
#pragma unroll
        for (int m = 0; m < 2; m++)
#pragma unroll
            for (int rb = 0; rb < H / 32; rb++) {
                const T* p = base + (16 * m) * LDX + 32 * rb;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * LDX));
                const s16x8 x = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                out[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, x), pk.v[m], out[rb], 0, 0, 0);
            }
    }
    static __device__ __forceinline__ void store4(T* p, float a, float b, float c, float d) {
        uint2 x;
        x.x = (uint32_t)f2bf(a) | ((uint32_t)f2bf(b) << 16);
        x.y = (uint32_t)f2bf(c) | ((uint32_t)f2bf(d) << 16);
        *reinterpret_cast<uint2*>(p) = x;
    }
};

// rows r0 .. r0+63 of a slab (rows of H contiguous elements, `pitch` apart) into registers, zeros beyond `ext`
template <class X>
__device__ __forceinline__ void load_block(const typename X::T* slab, int pitch, int r0, int ext, int tid, typename X::Vec (&reg)[X::kVec]) {
    constexpr int kRowVecs = X::H / X::kPer;
#pragma unroll
    for (int c = 0; c < X::kVec; c++) {
        const int idx = tid + 256 * c;
        const int row = idx / kRowVecs, cv = idx % kRowVecs;
        reg[c] = (r0 + row < ext) ? *reinterpret_cast<const typename X::Vec*>(slab + (int64_t)(r0 + row) * pitch + cv * X::kPer)
                                  : X::zero_vec();
    }
}
template <class X, int LDX>
__device__ __forceinline__ void store_block(typename X::T* lds, int tid, const typename X::Vec (&reg)[X::kVec]) {
    constexpr int kRowVecs = X::H / X::kPer;
#pragma unroll
    for (int c = 0; c < X::kVec; c++) {
        const int idx = tid + 256 * c;
        X::template put<LDX>(lds, idx / kRowVecs, idx % kRowVecs, reg[c]);
    }
}

// accumulators (lane = this lane's row of the slab, register r = first-axis element 32 rb + acc_row(r)) to memory
template <class X>
__device__ __forceinline__ void store_own_row(typename X::T* slab, int pitch, int row, int hh, bool valid, float mul, const f32x16 (&acc)[X::H / 32]) {
    if (!valid) return;
    typename X::T* p = slab + (int64_t)row * pitch;
#pragma unroll
    for (int rb = 0; rb < X::H / 32; rb++)
#pragma unroll
        for (int g = 0; g < 4; g++)
            X::store4(p + 32 * rb + 8 * g + 4 * hh, acc[rb][4 * g] * mul, acc[rb][4 * g + 1] * mul, acc[rb][4 * g + 2] * mul,
                      acc[rb][4 * g + 3] * mul);
}

struct FwdArgs {
    AttnGeom g;
    void* const* Q; void* const* K; void* const* V; void* const* O; void* const* stats;
    Win wQ, wK, wV, wO;
};

// ---------------------------------------------------------------- forward
template <class X>
__global__ void __launch_bounds__(256, 2) attn_fwd(const FwdArgs a) {
    using T = typename X::T;
    constexpr int H = X::H, LDK = X::LD, LDV = X::LD_COLS;
    constexpr int kBufElems = kBlk * LDK + kBlk * LDV;
    __shared__ __attribute__((aligned(16))) T lds[2][kBufElems];
    const AttnGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, hh = lane >> 5, ln = lane & 31;
    // under the causal mask the later a query block, the more key blocks it walks: the longest go first
    const int rblk = g.causal ? gridDim.y - 1 - blockIdx.y : blockIdx.y;
    const int l = g.tile0 + rblk / g.nblk, e0 = (rblk % g.nblk) * kWgRows;
    const int b = blockIdx.x % g.Nb, j = blockIdx.x / g.Nb;
    const Pair pr = pair_of(g, b, j);
    const Slab sq = slab_of(g, pr, l);
    if (e0 >= sq.ext) return;
    const int eq = e0 + 32 * w + ln;
    const bool qvalid = eq < sq.ext;
    const int qglob = l * g.bs + eq;
    const int wave_qfirst = l * g.bs + e0 + 32 * w;
    const int wave_qlast = l * g.bs + min(e0 + 32 * w + 31, sq.ext - 1);
    const int wg_qlast = l * g.bs + min(e0 + kWgRows - 1, sq.ext - 1);
    const float sc2 = g.scale * kLog2e;        // scores are kept in units of log 2

    typename X::Own qf;
    X::load_own(rows_win<const T>(a.Q, g, a.wQ, pr, sq, b, j), g.pitch, eq, hh, qvalid, qf);

    int nit;
    if (g.causal) nit = (wg_qlast / g.bs) * g.nstep + (wg_qlast % g.bs) / kBlk + 1;
    else nit = (g.gs - 1) * g.nstep + (g.Ns - (g.gs - 1) * g.bs + kBlk - 1) / kBlk;

    f32x16 O[H / 32];
#pragma unroll
    for (int rb = 0; rb < H / 32; rb++) O[rb] = zero16();
    float m = kNegInf, lsum = 0.f;

    typename X::Vec kr[X::kVec], vr[X::kVec];
    auto fetch = [&](int it) {
        const int lk = it / g.nstep, k0 = (it % g.nstep) * kBlk;
        const Slab sk = slab_of(g, pr, lk);
        load_block<X>(rows_win<const T>(a.K, g, a.wK, pr, sk, b, j), g.pitch, k0, sk.ext, tid, kr);
        load_block<X>(rows_win<const T>(a.V, g, a.wV, pr, sk, b, j), g.pitch, k0, sk.ext, tid, vr);
    };
    auto stash = [&](int buf) {
        store_block<X, LDK>(lds[buf], tid, kr);
        store_block<X, LDV>(lds[buf] + kBlk * LDK, tid, vr);
    };
    fetch(0);
    stash(0);
    __syncthreads();
    for (int it = 0; it < nit; it++) {
        if (it + 1 < nit) fetch(it + 1);
        const int lk = it / g.nstep, kloc0 = (it % g.nstep) * kBlk;
        const int ext_k = min(g.bs, g.Ns - lk * g.bs);
        const int kglob0 = lk * g.bs + kloc0;
        if (!(g.causal && kglob0 > wave_qlast)) {
            const T* Ks = lds[it & 1];
            const T* Vs = Ks + kBlk * LDK;
            // the second half of the block may be hidden from all of this wave's queries
            const bool two = !(g.causal && kglob0 + 32 > wave_qlast) && kloc0 + 32 < ext_k;
            const bool plain = kloc0 + kBlk <= ext_k && (!g.causal || kglob0 + kBlk - 1 <= wave_qfirst);
            f32x16 s[2];
            s[0] = X::template rows_times_own<LDK>(Ks, 0, ln, hh, qf);
            if (two) s[1] = X::template rows_times_own<LDK>(Ks, 1, ln, hh, qf);
            else s[1] = s[0];                       // masked below
            // the running maximum is kept in units of the raw scores (scale > 0 keeps the order)
            float mx = kNegInf;
            if (plain) {
#pragma unroll
                for (int sub = 0; sub < 2; sub++)
#pragma unroll
                    for (int r = 0; r < 16; r++) mx = fmaxf(mx, s[sub][r]);
            } else {
                // keys [0, lim) of the block are inside the tile, visible to this lane's query and computed
                int lim = min(ext_k - kloc0, two ? kBlk : 32);
                if (g.causal) lim = min(lim, qglob - kglob0 + 1);
                const int lim_h = lim - 4 * hh;
#pragma unroll
                for (int sub = 0; sub < 2; sub++)
#pragma unroll
                    for (int r = 0; r < 16; r++) {
                        s[sub][r] = 32 * sub + acc_row0(r) < lim_h ? s[sub][r] : kNegInf;
                        mx = fmaxf(mx, s[sub][r]);
                    }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m, mx);
            const float shift = m_new == kNegInf ? 0.f : m_new * sc2;
            const float alpha = m == m_new ? 1.f : __builtin_amdgcn_exp2f(m * sc2 - shift);
            m = m_new;
            float rowsum = 0.f;
#pragma unroll
            for (int sub = 0; sub < 2; sub++)
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    s[sub][r] = __builtin_amdgcn_exp2f(fmaf(s[sub][r], sc2, -shift));
                    rowsum += s[sub][r];
                }
            lsum = lsum * alpha + rowsum;
            if (__any(alpha != 1.f)) {              // after the first blocks the maxima seldom move
#pragma unroll
                for (int rb = 0; rb < H / 32; rb++)
#pragma unroll
                    for (int r = 0; r < 16; r++) O[rb][r] *= alpha;
            }
            typename X::Packed pk;
            X::pack(s[0], pk);
            X::template cols_times_acc<LDV>(O, Vs, 0, lane, pk);
            if (two) {
                X::pack(s[1], pk);
                X::template cols_times_acc<LDV>(O, Vs, 1, lane, pk);
            }
        }
        if (it + 1 < nit) stash((it + 1) & 1);
        __syncthreads();
    }
    lsum += __shfl_xor(lsum, 32, 64);
    store_own_row<X>(rows_win<T>(a.O, g, a.wO, pr, sq, b, j), g.pitch, eq, hh, qvalid, 1.f / lsum, O);
    if (qvalid && hh == 0) {
        float* st = rows_of<float>(a.stats, sq, 2) + 2 * (int64_t)eq;
        st[0] = m * g.scale;
        st[1] = lsum;
    }
}

struct BwdArgs {
    AttnGeom g;
    void* const* Q; void* const* K; void* const* V; void* const* O; void* const* stats; void* const* dO;
    void* const* dQ; void* const* dK; void* const* dV;
    float* aux;     // per (query, batch, head): log2 of (softmax denominator times 2^maximum), and D
    Win wQ, wK, wV, wO, wdO, wdQ, wdK, wdV;
};

// ---------------------------------------------------------------- dQ (also writes aux)
template <class X>
__global__ void __launch_bounds__(256, 2) attn_dq(const BwdArgs a) {
    using T = typename X::T;
    constexpr int H = X::H, LD = X::LD;
    __shared__ __attribute__((aligned(16))) T lds[2][2 * kBlk * LD];
    const AttnGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, hh = lane >> 5, ln = lane & 31;
    const int rblk = g.causal ? gridDim.y - 1 - blockIdx.y : blockIdx.y;
    const int l = g.tile0 + rblk / g.nblk, e0 = (rblk % g.nblk) * kWgRows;
    const int b = blockIdx.x % g.Nb, j = blockIdx.x / g.Nb;
    const Pair pr = pair_of(g, b, j);
    const Slab sq = slab_of(g, pr, l);
    if (e0 >= sq.ext) return;
    const int eq = e0 + 32 * w + ln;
    const bool qvalid = eq < sq.ext;
    const int qglob = l * g.bs + eq;
    const int wave_qfirst = l * g.bs + e0 + 32 * w;
    const int wave_qlast = l * g.bs + min(e0 + 32 * w + 31, sq.ext - 1);
    const int wg_qlast = l * g.bs + min(e0 + kWgRows - 1, sq.ext - 1);
    const float sc2 = g.scale * kLog2e;

    typename X::Own qf, dof;
    X::load_own(rows_win<const T>(a.Q, g, a.wQ, pr, sq, b, j), g.pitch, eq, hh, qvalid, qf);
    X::load_own(rows_win<const T>(a.dO, g, a.wdO, pr, sq, b, j), g.pitch, eq, hh, qvalid, dof);
    float lse = 0.f, D = 0.f;
    {
        typename X::Own of;
        X::load_own(rows_win<const T>(a.O, g, a.wO, pr, sq, b, j), g.pitch, eq, hh, qvalid, of);
        D = X::dot_own(of, dof);
        D += __shfl_xor(D, 32, 64);
        if (qvalid) {
            const float* st = rows_of<const float>(a.stats, sq, 2) + 2 * (int64_t)eq;
            lse = st[0] * kLog2e + log2f(st[1]);
            if (hh == 0) {
                float* ax = a.aux + 2 * ((int64_t)qglob + (int64_t)g.Ns * (b + (int64_t)g.Nb * j));
                ax[0] = lse;
                ax[1] = D;
            }
        }
    }

    int nit;
    if (g.causal) nit = (wg_qlast / g.bs) * g.nstep + (wg_qlast % g.bs) / kBlk + 1;
    else nit = (g.gs - 1) * g.nstep + (g.Ns - (g.gs - 1) * g.bs + kBlk - 1) / kBlk;

    f32x16 dQ[H / 32];
#pragma unroll
    for (int rb = 0; rb < H / 32; rb++) dQ[rb] = zero16();

    typename X::Vec kr[X::kVec], vr[X::kVec];
    auto fetch = [&](int it) {
        const int lk = it / g.nstep, k0 = (it % g.nstep) * kBlk;
        const Slab sk = slab_of(g, pr, lk);
        load_block<X>(rows_win<const T>(a.K, g, a.wK, pr, sk, b, j), g.pitch, k0, sk.ext, tid, kr);
        load_block<X>(rows_win<const T>(a.V, g, a.wV, pr, sk, b, j), g.pitch, k0, sk.ext, tid, vr);
    };
    auto stash = [&](int buf) {
        store_block<X, LD>(lds[buf], tid, kr);
        store_block<X, LD>(lds[buf] + kBlk * LD, tid, vr);
    };
    fetch(0);
    stash(0);
    __syncthreads();
    for (int it = 0; it < nit; it++) {
        if (it + 1 < nit) fetch(it + 1);
        const int lk = it / g.nstep, kloc0 = (it % g.nstep) * kBlk;
        const int ext_k = min(g.bs, g.Ns - lk * g.bs);
        const int kglob0 = lk * g.bs + kloc0;
        if (!(g.causal && kglob0 > wave_qlast)) {
            const T* Ks = lds[it & 1];
            const T* Vs = Ks + kBlk * LD;
            const int nsub = (!(g.causal && kglob0 + 32 > wave_qlast) && kloc0 + 32 < ext_k) ? 2 : 1;
            const bool plain = kloc0 + kBlk <= ext_k && (!g.causal || kglob0 + kBlk - 1 <= wave_qfirst);
            // keys [0, lim) of the block are inside the tile and visible to this lane's query
            int lim = ext_k - kloc0;
            if (g.causal) lim = min(lim, qglob - kglob0 + 1);
            const int lim_h = lim - 4 * hh;
            // (two copies of the body: blocks that are visible as a whole skip the mask arithmetic)
            auto body = [&](auto masked) {
                for (int sub = 0; sub < nsub; sub++) {
                    f32x16 s = X::template rows_times_own<LD>(Ks, sub, ln, hh, qf);
                    const f32x16 dp = X::template rows_times_own<LD>(Vs, sub, ln, hh, dof);
#pragma unroll
                    for (int r = 0; r < 16; r++) {
                        float p = __builtin_amdgcn_exp2f(s[r] * sc2 - lse);
                        if (decltype(masked)::value) p = 32 * sub + acc_row0(r) < lim_h ? p : 0.f;
                        s[r] = p * (dp[r] - D);
                    }
                    typename X::Packed pk;
                    X::pack(s, pk);
                    X::template cols_times_acc<LD>(dQ, Ks, sub, lane, pk);
                }
            };
            if (plain) body(std::false_type{});
            else body(std::true_type{});
        }
        if (it + 1 < nit) stash((it + 1) & 1);
        __syncthreads();
    }
    store_own_row<X>(rows_win<T>(a.dQ, g, a.wdQ, pr, sq, b, j), g.pitch, eq, hh, qvalid, g.scale, dQ);
}

// ---------------------------------------------------------------- dK and dV (reads aux)
// (bf16 with head size 128 needs more than 256 registers per lane for its four accumulator sets and two
// fragment sets: compiled for one workgroup per CU it keeps them all, for two it spills and runs 3x slower)
template <class X>
__global__ void __launch_bounds__(256, X::kDkvBlocks) attn_dkv(const BwdArgs a) {
    using T = typename X::T;
    constexpr int H = X::H, LD = X::LD;
    constexpr int kAuxElems = 2 * kBlk * (int)(sizeof(float) / sizeof(T));   // 2 x 64 floats, in units of T
    __shared__ __attribute__((aligned(16))) T lds[2][2 * kBlk * LD + kAuxElems];
    const AttnGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, hh = lane >> 5, ln = lane & 31;
    // (under the causal mask the earliest key blocks meet the most query blocks: already first)
    const int l = g.tile0 + blockIdx.y / g.nblk, e0 = (blockIdx.y % g.nblk) * kWgRows;
    const int b = blockIdx.x % g.Nb, j = blockIdx.x / g.Nb;
    const Pair pr = pair_of(g, b, j);
    const Slab sk = slab_of(g, pr, l);
    if (e0 >= sk.ext) return;
    const int ek = e0 + 32 * w + ln;
    const bool kvalid = ek < sk.ext;
    const int kglob = l * g.bs + ek;
    const int wave_kfirst = l * g.bs + e0 + 32 * w;
    const int wave_klast = wave_kfirst + 31;
    const float sc2 = g.scale * kLog2e;

    typename X::Own kf, vf;
    X::load_own(rows_win<const T>(a.K, g, a.wK, pr, sk, b, j), g.pitch, ek, hh, kvalid, kf);
    X::load_own(rows_win<const T>(a.V, g, a.wV, pr, sk, b, j), g.pitch, ek, hh, kvalid, vf);

    const int nit = (g.gs - 1) * g.nstep + (g.Ns - (g.gs - 1) * g.bs + kBlk - 1) / kBlk;
    // with the causal mask the first query block that sees any of these keys is the one that holds key e0
    const int it0 = g.causal ? l * g.nstep + e0 / kBlk : 0;

    f32x16 dK[H / 32], dV[H / 32];
#pragma unroll
    for (int rb = 0; rb < H / 32; rb++) { dK[rb] = zero16(); dV[rb] = zero16(); }

    typename X::Vec qr[X::kVec], dr[X::kVec];
    float2 ar = make_float2(0.f, 0.f);
    const float* aux_pair = a.aux + 2 * (int64_t)g.Ns * (b + (int64_t)g.Nb * j);
    auto fetch = [&](int it) {
        const int lq = it / g.nstep, q0 = (it % g.nstep) * kBlk;
        const Slab sq = slab_of(g, pr, lq);
        load_block<X>(rows_win<const T>(a.Q, g, a.wQ, pr, sq, b, j), g.pitch, q0, sq.ext, tid, qr);
        load_block<X>(rows_win<const T>(a.dO, g, a.wdO, pr, sq, b, j), g.pitch, q0, sq.ext, tid, dr);
        if (tid < kBlk) {
            const bool ok = q0 + tid < sq.ext;
            ar = ok ? *reinterpret_cast<const float2*>(aux_pair + 2 * (lq * g.bs + q0 + tid)) : make_float2(0.f, 0.f);
        }
    };
    auto stash = [&](int buf) {
        store_block<X, LD>(lds[buf], tid, qr);
        store_block<X, LD>(lds[buf] + kBlk * LD, tid, dr);
        if (tid < kBlk) {
            float* ax = reinterpret_cast<float*>(lds[buf] + 2 * kBlk * LD);
            ax[tid] = ar.x;
            ax[kBlk + tid] = ar.y;
        }
    };
    if (it0 < nit) {
        fetch(it0);
        stash(it0 & 1);
    }
    __syncthreads();
    for (int it = it0; it < nit; it++) {
        if (it + 1 < nit) fetch(it + 1);
        const int lq = it / g.nstep, qloc0 = (it % g.nstep) * kBlk;
        const int ext_q = min(g.bs, g.Ns - lq * g.bs);
        const int qglob0 = lq * g.bs + qloc0;
        if (!(g.causal && qglob0 + kBlk - 1 < wave_kfirst)) {
            const T* Qs = lds[it & 1];
            const T* Ds = Qs + kBlk * LD;
            const float* lses = reinterpret_cast<const float*>(Ds + kBlk * LD);
            const float* dsum = lses + kBlk;
            // the first half of the block may hold only queries that precede all of this wave's keys
            const int sub0 = (g.causal && qglob0 + 31 < wave_kfirst) ? 1 : 0;
            const int nsub = qloc0 + 32 < ext_q ? 2 : 1;
            const bool plain = qloc0 + kBlk <= ext_q && (!g.causal || wave_klast <= qglob0);
            const int lo = g.causal ? max(kglob - qglob0, 0) : 0, hi = ext_q - qloc0;
            const int lo_h = lo - 4 * hh;
            const unsigned width = (unsigned)max(hi - lo, 0);
            // (not unrolled: the second pass would keep a second set of temporaries alive and spill)
#pragma unroll 1
            for (int sub = sub0; sub < nsub; sub++) {
                f32x16 s = X::template rows_times_own<LD>(Qs, sub, ln, hh, kf);
                const f32x16 dp = X::template rows_times_own<LD>(Ds, sub, ln, hh, vf);
                // log-sum-exp and D of the 16 queries this lane's accumulator registers stand for: four runs of four
                float lse_r[16], d_r[16];
#pragma unroll
                for (int q4 = 0; q4 < 4; q4++) {
                    const float4 a4 = *reinterpret_cast<const float4*>(lses + 32 * sub + 8 * q4 + 4 * hh);
                    const float4 b4 = *reinterpret_cast<const float4*>(dsum + 32 * sub + 8 * q4 + 4 * hh);
                    lse_r[4 * q4] = a4.x; lse_r[4 * q4 + 1] = a4.y; lse_r[4 * q4 + 2] = a4.z; lse_r[4 * q4 + 3] = a4.w;
                    d_r[4 * q4] = b4.x; d_r[4 * q4 + 1] = b4.y; d_r[4 * q4 + 2] = b4.z; d_r[4 * q4 + 3] = b4.w;
                }
                typename X::Packed pk;
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    // queries [lo, hi) of the block are inside the tile and see this lane's key: one unsigned
                    // comparison of the register's row, shifted by the lane half, against the width of that range
                    const bool ok = plain || (unsigned)(32 * sub + acc_row0(r) - lo_h) < width;
                    const float p = ok ? __builtin_amdgcn_exp2f(s[r] * sc2 - lse_r[r]) : 0.f;
                    X::set(pk, r, p);
                    s[r] = p * (dp[r] - d_r[r]);
                }
                X::template cols_times_acc<LD>(dV, Ds, sub, lane, pk);
                X::pack(s, pk);
                X::template cols_times_acc<LD>(dK, Qs, sub, lane, pk);
            }
        }
        if (it + 1 < nit) stash((it + 1) & 1);
        __syncthreads();
    }
    store_own_row<X>(rows_win<T>(a.dK, g, a.wdK, pr, sk, b, j), g.pitch, ek, hh, kvalid, g.scale, dK);
    store_own_row<X>(rows_win<T>(a.dV, g, a.wdV, pr, sk, b, j), g.pitch, ek, hh, kvalid, 1.f, dV);
}

using FwdKernel = void (*)(const FwdArgs);
using BwdKernel = void (*)(const BwdArgs);

FwdKernel fwd_kernel(int dtype, int H) {
    if (dtype == NNT_F32) return H == 64 ? attn_fwd<F32Traits<64>> : attn_fwd<F32Traits<128>>;
    return H == 64 ? attn_fwd<Bf16Traits<64>> : attn_fwd<Bf16Traits<128>>;
}
BwdKernel dq_kernel(int dtype, int H) {
    if (dtype == NNT_F32) return H == 64 ? attn_dq<F32Traits<64>> : attn_dq<F32Traits<128>>;
    return H == 64 ? attn_dq<Bf16Traits<64>> : attn_dq<Bf16Traits<128>>;
}
BwdKernel dkv_kernel(int dtype, int H) {
    if (dtype == NNT_F32) return H == 64 ? attn_dkv<F32Traits<64>> : attn_dkv<F32Traits<128>>;
    return H == 64 ? attn_dkv<Bf16Traits<64>> : attn_dkv<Bf16Traits<128>>;
}

}  // namespace
}  // namespace nnt

using namespace nnt;

// ------------------------------------------------------------------ host side
namespace {

int32_t check_attn(nnt_ctx* ctx, const char* who, std::initializer_list<const nnt_tensor*> ts, const nnt_tensor* stats, float scale) {
    const nnt_tensor* first = *ts.begin();
    for (const nnt_tensor* t : ts) {
        if (!t) return fail(ctx, NNT_EINVAL, std::string(who) + ": null tensor");
        if (t->ndim != 4) return fail(ctx, NNT_EINVAL, std::string(who) + ": operands are (h, N_s, N_b, N_h) tensors");
        if (t->dtype != first->dtype || !same_tiling(t, first))
            return fail(ctx, NNT_EINVAL, std::string(who) + ": operands differ in type, extents or tiling");
        if (t->base[0] != t->shape[0]) return fail(ctx, NNT_EINVAL, std::string(who) + ": the head axis must not be tiled");
        for (void* p : t->tiles)
            if (!p || !aligned16(p)) return fail(ctx, NNT_EINVAL, std::string(who) + ": missing or unaligned tile");
    }
    if (first->dtype != NNT_F32 && first->dtype != NNT_BF16) return fail(ctx, NNT_EDTYPE, std::string(who) + ": fp32 or bf16 operands");
    if (first->shape[0] != 64 && first->shape[0] != 128)
        return fail(ctx, NNT_EINVAL, std::string(who) + ": head size must be 64 or 128");
    if (!stats) return fail(ctx, NNT_EINVAL, std::string(who) + ": null tensor");
    if (!(scale > 0.f)) return fail(ctx, NNT_EINVAL, std::string(who) + ": scale must be positive");
    if (stats->dtype != NNT_F32 || stats->ndim != 4 || stats->shape[0] != 2 || stats->base[0] != 2)
        return fail(ctx, NNT_EINVAL, std::string(who) + ": stats must be fp32 (2, N_s, N_b, N_h) with an untiled first axis");
    for (int a = 1; a < 4; a++)
        if (stats->shape[a] != first->shape[a] || stats->base[a] != first->base[a])
            return fail(ctx, NNT_EINVAL, std::string(who) + ": stats must be tiled like the operands' other axes");
    for (void* p : stats->tiles)
        if (!p) return fail(ctx, NNT_EINVAL, std::string(who) + ": stats tile missing");
    if (first->grid[1] * ((first->base[1] + kWgRows - 1) / kWgRows) > 65535 || first->shape[2] * first->shape[3] > INT32_MAX)
        return fail(ctx, NNT_EINVAL, std::string(who) + ": sequence too long for one launch");
    return NNT_OK;
}

AttnGeom geom_of(const nnt_tensor* q, float scale, int causal) {
    AttnGeom g;
    g.H = (int)q->shape[0]; g.Ns = (int)q->shape[1]; g.Nb = (int)q->shape[2]; g.Nh = (int)q->shape[3];
    g.bs = (int)q->base[1]; g.bb = (int)q->base[2]; g.bh = (int)q->base[3];
    g.gs = (int)q->grid[1]; g.gb = (int)q->grid[2]; g.gh = (int)q->grid[3];
    g.nblk = (g.bs + kWgRows - 1) / kWgRows;
    g.nstep = (g.bs + kBlk - 1) / kBlk;
    g.tile0 = 0;
    g.causal = causal;
    g.scale = scale;
    g.win = 0;
    g.pitch = g.H;
    g.hp = 1;
    return g;
}

// Geometry for operands that are windows on tensors [parts * N_h * H, N_s, N_b] (`ts`: the tensors with their
// part counts); the statistics are an ordinary tensor (2, N_s, N_b, N_h).
int32_t geom_of_windows(nnt_ctx* ctx, const char* who, std::initializer_list<std::pair<const nnt_tensor*, int>> ts, const nnt_tensor* stats,
                        int32_t N_h, float scale, int causal, AttnGeom* out) {
    const nnt_tensor* first = ts.begin()->first;
    if (!first || !stats || N_h < 1) return fail(ctx, NNT_EINVAL, std::string(who) + ": null tensor or bad head count");
    const int64_t N_e = first->ndim == 3 ? first->shape[0] / ts.begin()->second : 0;
    if (N_e < 1 || N_e % N_h != 0) return fail(ctx, NNT_EINVAL, std::string(who) + ": rows are not whole parts of N_h heads");
    const int64_t H = N_e / N_h, t0 = first->base[0];
    if (H != 64 && H != 128) return fail(ctx, NNT_EINVAL, std::string(who) + ": head size must be 64 or 128");
    if (t0 % H != 0 || N_e % t0 != 0) return fail(ctx, NNT_EINVAL, std::string(who) + ": row tiles must hold whole heads and a part whole row tiles");
    for (const auto& tp : ts) {
        const nnt_tensor* t = tp.first;
        if (!t) return fail(ctx, NNT_EINVAL, std::string(who) + ": null tensor");
        if (t->ndim != 3 || t->dtype != first->dtype || t->shape[0] != tp.second * N_e || t->base[0] != t0 || t->shape[1] != first->shape[1] ||
            t->shape[2] != first->shape[2] || t->base[1] != first->base[1] || t->base[2] != first->base[2])
            return fail(ctx, NNT_EINVAL, std::string(who) + ": operands differ in type, extents or tiling");
        for (void* p : t->tiles)
            if (!p || !aligned16(p)) return fail(ctx, NNT_EINVAL, std::string(who) + ": missing or unaligned tile");
    }
    if (first->dtype != NNT_F32 && first->dtype != NNT_BF16) return fail(ctx, NNT_EDTYPE, std::string(who) + ": fp32 or bf16 operands");
    if (!(scale > 0.f)) return fail(ctx, NNT_EINVAL, std::string(who) + ": scale must be positive");
    if (stats->dtype != NNT_F32 || stats->ndim != 4 || stats->shape[0] != 2 || stats->base[0] != 2 || stats->shape[3] != N_h ||
        stats->shape[1] != first->shape[1] || stats->shape[2] != first->shape[2] || stats->base[1] != first->base[1] || stats->base[2] != first->base[2])
        return fail(ctx, NNT_EINVAL, std::string(who) + ": stats must be fp32 (2, N_s, N_b, N_h), tiled like the operands along N_s and N_b");
    for (void* p : stats->tiles)
        if (!p) return fail(ctx, NNT_EINVAL, std::string(who) + ": stats tile missing");
    if (first->grid[1] * ((first->base[1] + kWgRows - 1) / kWgRows) > 65535 || first->shape[2] * (int64_t)N_h > INT32_MAX)
        return fail(ctx, NNT_EINVAL, std::string(who) + ": sequence too long for one launch");
    AttnGeom g;
    g.H = (int)H; g.Ns = (int)first->shape[1]; g.Nb = (int)first->shape[2]; g.Nh = N_h;
    g.bs = (int)first->base[1]; g.bb = (int)first->base[2]; g.bh = (int)stats->base[3];
    g.gs = (int)first->grid[1]; g.gb = (int)first->grid[2]; g.gh = (int)stats->grid[3];
    g.nblk = (g.bs + kWgRows - 1) / kWgRows;
    g.nstep = (g.bs + kBlk - 1) / kBlk;
    g.tile0 = 0;
    g.causal = causal;
    g.scale = scale;
    g.win = 1;
    g.pitch = (int)t0;
    g.hp = (int)(t0 / H);
    *out = g;
    return NNT_OK;
}
Win window_at(const nnt_tensor* t, int part, int64_t N_e) { return Win{(int)(part * (N_e / t->base[0])), (int)t->grid[0]}; }

// visible (key, query) pairs of one (batch, head) pair for queries q0 .. q1-1
double visible_pairs(int64_t Ns, int64_t q0, int64_t q1, int causal) {
    if (!causal) return (double)Ns * (double)(q1 - q0);
    return 0.5 * ((double)q1 * (q1 + 1) - (double)q0 * (q0 + 1));
}

// the tiles of `t` whose sequence-tile coordinate is l, any batch / head tile
std::vector<Access> seq_tile(nnt_tensor* t, int64_t l, int mode) {
    std::vector<Access> v;
    for (int64_t x = l; x < t->ntiles; x += t->grid[1]) v.push_back(t->one(x, mode));
    return v;
}

}  // namespace

int32_t nnt_attention_fwd(nnt_ctx* ctx, nnt_tensor* Q, nnt_tensor* K, nnt_tensor* V, float scale, int32_t causal,
                          nnt_tensor* B, nnt_tensor* stats) {
    NNT_CHECK_CTX(ctx);
    int32_t rc = check_attn(ctx, "nnt_attention_fwd", {Q, K, V, B}, stats, scale);
    if (rc != NNT_OK) return rc;
    AttnGeom g = geom_of(Q, scale, causal);
    FwdArgs a{g, Q->d_tiles, K->d_tiles, V->d_tiles, B->d_tiles, stats->d_tiles};
    const double pair_flops = 4.0 * g.H * g.Nb * g.Nh;   // two products, 2 flops per multiply-add
    const FwdKernel kernel = fwd_kernel(Q->dtype, g.H);
    auto launch = [kernel](hipStream_t st, const FwdArgs& fa, int ntile) {
        const dim3 grid((unsigned)(fa.g.Nb * fa.g.Nh), (unsigned)(ntile * fa.g.nblk)), block(256);
        hipLaunchKernelGGL(kernel, grid, block, 0, st, fa);
        return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
    };
    OpTag tag(ctx, "attention_fwd", pair_flops * visible_pairs(g.Ns, 0, g.Ns, causal), false);
    if (ctx->granularity == NNT_GRAN_OP) {
        const int ntile = g.gs;
        return submit(ctx, {Q->all(kRead), K->all(kRead), V->all(kRead), B->all(kWrite), stats->all(kWrite)},
                      [=](hipStream_t st) { return launch(st, a, ntile); });
    }
    // one task per query tile
    for (int64_t l = 0; l < g.gs; l++) {
        std::vector<Access> acc = seq_tile(Q, l, kRead);
        for (int64_t lk = 0; lk < (causal ? l + 1 : (int64_t)g.gs); lk++) {
            for (const Access& x : seq_tile(K, lk, kRead)) acc.push_back(x);
            for (const Access& x : seq_tile(V, lk, kRead)) acc.push_back(x);
        }
        for (const Access& x : seq_tile(B, l, kWrite)) acc.push_back(x);
        for (const Access& x : seq_tile(stats, l, kWrite)) acc.push_back(x);
        FwdArgs al = a;
        al.g.tile0 = (int)l;
        rc = submit(ctx, acc, [=](hipStream_t st) { return launch(st, al, 1); });
        if (rc != NNT_OK) return rc;
    }
    return NNT_OK;
}

int32_t nnt_attention_bwd(nnt_ctx* ctx, nnt_tensor* Q, nnt_tensor* K, nnt_tensor* V, nnt_tensor* B, nnt_tensor* stats,
                          nnt_tensor* dB, float scale, int32_t causal, nnt_tensor* dQ, nnt_tensor* dK, nnt_tensor* dV) {
    NNT_CHECK_CTX(ctx);
    int32_t rc = check_attn(ctx, "nnt_attention_bwd", {Q, K, V, B, dB, dQ, dK, dV}, stats, scale);
    if (rc != NNT_OK) return rc;
    AttnGeom g = geom_of(Q, scale, causal);
    rc = ensure_scratch(ctx, 2 * (int64_t)g.Ns * g.Nb * g.Nh);
    if (rc != NNT_OK) return rc;
    BwdArgs a{g, Q->d_tiles, K->d_tiles, V->d_tiles, B->d_tiles, stats->d_tiles, dB->d_tiles,
              dQ->d_tiles, dK->d_tiles, dV->d_tiles, ctx->red_scratch};
    const double pair_flops = 2.0 * g.H * g.Nb * g.Nh;   // per product
    const double pairs = visible_pairs(g.Ns, 0, g.Ns, causal);
    const Access scr{&ctx->red_dep, 1, kReadWrite};
    const BwdKernel k_dq = dq_kernel(Q->dtype, g.H), k_dkv = dkv_kernel(Q->dtype, g.H);
    // one task, two launches: the dQ kernel leaves log-sum-exp and D per query for the dK/dV kernel
    OpTag tag(ctx, "attention_bwd_dq", 3.0 * pair_flops * pairs, false);
    return submit(ctx, {Q->all(kRead), K->all(kRead), V->all(kRead), B->all(kRead), stats->all(kRead), dB->all(kRead),
                        dQ->all(kWrite), dK->all(kWrite), dV->all(kWrite), scr},
                  [=](hipStream_t st) {
                      const dim3 grid((unsigned)(a.g.Nb * a.g.Nh), (unsigned)(a.g.gs * a.g.nblk)), block(256);
                      hipLaunchKernelGGL(k_dq, grid, block, 0, st, a);
                      if (hipGetLastError() != hipSuccess) return (int32_t)NNT_EHIP;
                      profile_mark(ctx, st, "attention_bwd_dkv", 4.0 * pair_flops * pairs, false);
                      hipLaunchKernelGGL(k_dkv, grid, block, 0, st, a);
                      return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
                  }, 2);
}

int32_t nnt_attention_fwd_heads(nnt_ctx* ctx, nnt_tensor* QKV, float scale, int32_t causal, nnt_tensor* Bm, nnt_tensor* stats, int32_t N_h) {
    NNT_CHECK_CTX(ctx);
    AttnGeom g;
    int32_t rc = geom_of_windows(ctx, "nnt_attention_fwd_heads", {{QKV, 3}, {Bm, 1}}, stats, N_h, scale, causal, &g);
    if (rc != NNT_OK) return rc;
    const int64_t N_e = (int64_t)g.H * g.Nh;
    FwdArgs a{g, QKV->d_tiles, QKV->d_tiles, QKV->d_tiles, Bm->d_tiles, stats->d_tiles,
              window_at(QKV, 0, N_e), window_at(QKV, 1, N_e), window_at(QKV, 2, N_e), window_at(Bm, 0, N_e)};
    const double pair_flops = 4.0 * g.H * g.Nb * g.Nh;
    const FwdKernel kernel = fwd_kernel(QKV->dtype, g.H);
    OpTag tag(ctx, "attention_fwd", pair_flops * visible_pairs(g.Ns, 0, g.Ns, causal), false);
    return submit(ctx, {QKV->all(kRead), Bm->all(kWrite), stats->all(kWrite)}, [=](hipStream_t st) {
        const dim3 grid((unsigned)(a.g.Nb * a.g.Nh), (unsigned)(a.g.gs * a.g.nblk)), block(256);
        hipLaunchKernelGGL(kernel, grid, block, 0, st, a);
        return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
    });
}

int32_t nnt_attention_bwd_heads(nnt_ctx* ctx, nnt_tensor* QKV, nnt_tensor* Bm, nnt_tensor* stats, nnt_tensor* dBm, float scale,
                                int32_t causal, nnt_tensor* dQKV, int32_t N_h) {
    NNT_CHECK_CTX(ctx);
    AttnGeom g;
    int32_t rc = geom_of_windows(ctx, "nnt_attention_bwd_heads", {{QKV, 3}, {Bm, 1}, {dBm, 1}, {dQKV, 3}}, stats, N_h, scale, causal, &g);
    if (rc != NNT_OK) return rc;
    rc = ensure_scratch(ctx, 2 * (int64_t)g.Ns * g.Nb * g.Nh);
    if (rc != NNT_OK) return rc;
    const int64_t N_e = (int64_t)g.H * g.Nh;
    BwdArgs a{g, QKV->d_tiles, QKV->d_tiles, QKV->d_tiles, Bm->d_tiles, stats->d_tiles, dBm->d_tiles,
              dQKV->d_tiles, dQKV->d_tiles, dQKV->d_tiles, ctx->red_scratch,
              window_at(QKV, 0, N_e), window_at(QKV, 1, N_e), window_at(QKV, 2, N_e), window_at(Bm, 0, N_e), window_at(dBm, 0, N_e),
              window_at(dQKV, 0, N_e), window_at(dQKV, 1, N_e), window_at(dQKV, 2, N_e)};
    const double pair_flops = 2.0 * g.H * g.Nb * g.Nh;
    const double pairs = visible_pairs(g.Ns, 0, g.Ns, causal);
    const Access scr{&ctx->red_dep, 1, kReadWrite};
    const BwdKernel k_dq = dq_kernel(QKV->dtype, g.H), k_dkv = dkv_kernel(QKV->dtype, g.H);
    OpTag tag(ctx, "attention_bwd_dq", 3.0 * pair_flops * pairs, false);
    return submit(ctx, {QKV->all(kRead), Bm->all(kRead), stats->all(kRead), dBm->all(kRead), dQKV->all(kWrite), scr},
                  [=](hipStream_t st) {
                      const dim3 grid((unsigned)(a.g.Nb * a.g.Nh), (unsigned)(a.g.gs * a.g.nblk)), block(256);
                      hipLaunchKernelGGL(k_dq, grid, block, 0, st, a);
                      if (hipGetLastError() != hipSuccess) return (int32_t)NNT_EHIP;
                      profile_mark(ctx, st, "attention_bwd_dkv", 4.0 * pair_flops * pairs, false);
                      hipLaunchKernelGGL(k_dkv, grid, block, 0, st, a);
                      return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
                  }, 2);
}
