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

namespace nnt {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWgRows = 128;   // rows owned by a workgroup
constexpr int kBlk = 64;       // rows streamed per iteration
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
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
};

struct Slab {
    int64_t off;   // element offset of (0, 0, b, j) in its tile, in units of one first-axis element
    int tile;      // tile number
    int ext;       // extent of the tile along the sequence axis
};

// where the rows of (batch b, head j) of sequence tile l live; `off` counts rows of the slab's first axis
__device__ __forceinline__ Slab slab_of(const AttnGeom& g, int l, int b, int j) {
    const int tb = b / g.bb, tj = j / g.bh;
    Slab s;
    s.ext = min(g.bs, g.Ns - l * g.bs);
    const int eb = min(g.bb, g.Nb - tb * g.bb);
    s.tile = l + g.gs * (tb + g.gb * tj);
    s.off = (int64_t)s.ext * ((b - tb * g.bb) + (int64_t)eb * (j - tj * g.bh));
    return s;
}

template <typename T>
__device__ __forceinline__ T* rows_of(void* const* tiles, const Slab& s, int width) {
    return static_cast<T*>(tiles[s.tile]) + s.off * width;
}

// ---------------------------------------------------------------- fp32 building blocks
template <int H> struct F32Block {
    static constexpr int LD = H + 1;                 // odd row pitch: row-wise and column-wise fragment reads both spread over the banks
    static constexpr int kFloats = kBlk * LD;
    static constexpr int kVec = H / 16;              // float4 per thread per block (64 rows x H / 4 vectors over 256 threads)

    // rows r0 .. r0+63 of a slab (rows of H contiguous floats), zeros beyond `ext`
    static __device__ __forceinline__ void load(const float* slab, int r0, int ext, int tid, float4 (&reg)[kVec]) {
#pragma unroll
        for (int c = 0; c < kVec; c++) {
            const int idx = tid + 256 * c;
            const int row = idx / (H / 4), c4 = idx % (H / 4);
            reg[c] = (r0 + row < ext) ? *reinterpret_cast<const float4*>(slab + (int64_t)(r0 + row) * H + c4 * 4)
                                      : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    static __device__ __forceinline__ void store(float* lds, int tid, const float4 (&reg)[kVec]) {
#pragma unroll
        for (int c = 0; c < kVec; c++) {
            const int idx = tid + 256 * c;
            const int row = idx / (H / 4), c4 = idx % (H / 4);
            float* d = lds + row * LD + c4 * 4;
            d[0] = reg[c].x; d[1] = reg[c].y; d[2] = reg[c].z; d[3] = reg[c].w;
        }
    }
    // A operand of a product whose rows are the block's rows and whose contraction runs over the
    // first axis: lane (row ln, half hh) of k-step s takes element s + (H/2) hh of row 32 sub + ln
    static __device__ __forceinline__ float by_row(const float* lds, int sub, int ln, int hh, int s) {
        return lds[(32 * sub + ln) * LD + s + (H / 2) * hh];
    }
    // A operand of a product whose rows are first-axis elements 32 rb + ln and whose contraction
    // runs over the block's rows: k-step r of half hh is row 32 sub + 8 (r/4) + 4 hh + r%4, the row
    // that accumulator register r of that half belongs to
    static __device__ __forceinline__ float by_col(const float* lds, int sub, int rb, int ln, int hh, int r) {
        return lds[(32 * sub + 8 * (r / 4) + 4 * hh + (r % 4)) * LD + 32 * rb + ln];
    }
};

__device__ __forceinline__ int acc_row(int r, int hh) { return 8 * (r / 4) + 4 * hh + (r % 4); }

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; i++) z[i] = 0.f;
    return z;
}

// this lane's half (elements (H/2) hh ..) of row `row` of a slab, times `mul`; zeros if !valid
template <int H>
__device__ __forceinline__ void load_own_row(const float* slab, int row, int hh, bool valid, float mul, float (&f)[H / 2]) {
    const float4* p = reinterpret_cast<const float4*>(slab + (int64_t)row * H + (H / 2) * hh);
#pragma unroll
    for (int s4 = 0; s4 < H / 8; s4++) {
        const float4 v = valid ? p[s4] : make_float4(0.f, 0.f, 0.f, 0.f);
        f[4 * s4 + 0] = v.x * mul; f[4 * s4 + 1] = v.y * mul; f[4 * s4 + 2] = v.z * mul; f[4 * s4 + 3] = v.w * mul;
    }
}

// accumulators (lane = this lane's row of the slab, register r = first-axis element 32 rb + acc_row(r)) to memory
template <int H>
__device__ __forceinline__ void store_own_row(float* slab, int row, int hh, bool valid, float mul, const f32x16 (&acc)[H / 32]) {
    if (!valid) return;
    float* p = slab + (int64_t)row * H;
#pragma unroll
    for (int rb = 0; rb < H / 32; rb++)
#pragma unroll
        for (int g = 0; g < 4; g++)
            *reinterpret_cast<float4*>(p + 32 * rb + 8 * g + 4 * hh) =
                make_float4(acc[rb][4 * g] * mul, acc[rb][4 * g + 1] * mul, acc[rb][4 * g + 2] * mul, acc[rb][4 * g + 3] * mul);
}

struct FwdArgs {
    AttnGeom g;
    void* const* Q; void* const* K; void* const* V; void* const* O; void* const* stats;
};

// ---------------------------------------------------------------- forward, fp32
template <int H>
__global__ void __launch_bounds__(256, 2) attn_fwd_f32(const FwdArgs a) {
    using Blk = F32Block<H>;
    constexpr int LDV = H + 8;   // values are only read column-wise: this pitch puts the two lane halves 32 banks apart
    __shared__ float lds[2][Blk::kFloats + kBlk * LDV];
    const AttnGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, hh = lane >> 5, ln = lane & 31;
    // under the causal mask the later a query block, the more key blocks it walks: the longest go first
    const int rblk = g.causal ? gridDim.y - 1 - blockIdx.y : blockIdx.y;
    const int l = g.tile0 + rblk / g.nblk, e0 = (rblk % g.nblk) * kWgRows;
    const int b = blockIdx.x % g.Nb, j = blockIdx.x / g.Nb;
    const Slab sq = slab_of(g, l, b, j);
    if (e0 >= sq.ext) return;
    const int eq = e0 + 32 * w + ln;
    const bool qvalid = eq < sq.ext;
    const int qglob = l * g.bs + eq;
    const int wave_qlast = l * g.bs + min(e0 + 32 * w + 31, sq.ext - 1);
    const int wg_qlast = l * g.bs + min(e0 + kWgRows - 1, sq.ext - 1);

    // queries pre-multiplied so that the scores come out in units of log 2
    float qf[H / 2];
    load_own_row<H>(rows_of<const float>(a.Q, sq, H), eq, hh, qvalid, g.scale * kLog2e, qf);

    int nit;
    if (g.causal) nit = (wg_qlast / g.bs) * g.nstep + (wg_qlast % g.bs) / kBlk + 1;
    else nit = (g.gs - 1) * g.nstep + (g.Ns - (g.gs - 1) * g.bs + kBlk - 1) / kBlk;

    f32x16 O[H / 32];
#pragma unroll
    for (int rb = 0; rb < H / 32; rb++) O[rb] = zero16();
    float m = kNegInf, lsum = 0.f;

    float4 kr[Blk::kVec], vr[Blk::kVec];
    auto fetch = [&](int it) {
        const int lk = it / g.nstep, k0 = (it % g.nstep) * kBlk;
        const Slab sk = slab_of(g, lk, b, j);
        Blk::load(rows_of<const float>(a.K, sk, H), k0, sk.ext, tid, kr);
        Blk::load(rows_of<const float>(a.V, sk, H), k0, sk.ext, tid, vr);
    };
    auto stash = [&](int buf) {
        Blk::store(lds[buf], tid, kr);
        float* vs = lds[buf] + Blk::kFloats;
#pragma unroll
        for (int c = 0; c < Blk::kVec; c++) {
            const int idx = tid + 256 * c;
            const int row = idx / (H / 4), c4 = idx % (H / 4);
            *reinterpret_cast<float4*>(vs + row * LDV + c4 * 4) = vr[c];
        }
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
            const float* Ks = lds[it & 1];
            const float* Vs = Ks + Blk::kFloats;
            f32x16 s[2] = {zero16(), zero16()};
#pragma unroll
            for (int k = 0; k < H / 2; k++) {
                s[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(Blk::by_row(Ks, 0, ln, hh, k), qf[k], s[0], 0, 0, 0);
                s[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(Blk::by_row(Ks, 1, ln, hh, k), qf[k], s[1], 0, 0, 0);
            }
            float mx = kNegInf;
#pragma unroll
            for (int sub = 0; sub < 2; sub++)
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int kl = 32 * sub + acc_row(r, hh);
                    const bool ok = kloc0 + kl < ext_k && (!g.causal || kglob0 + kl <= qglob);
                    s[sub][r] = ok ? s[sub][r] : kNegInf;
                    mx = fmaxf(mx, s[sub][r]);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m, mx);
            const float shift = m_new == kNegInf ? 0.f : m_new;
            const float alpha = m == m_new ? 1.f : __builtin_amdgcn_exp2f(m - shift);
            m = m_new;
            float rowsum = 0.f;
#pragma unroll
            for (int sub = 0; sub < 2; sub++)
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    s[sub][r] = __builtin_amdgcn_exp2f(s[sub][r] - shift);
                    rowsum += s[sub][r];
                }
            lsum = lsum * alpha + rowsum;
#pragma unroll
            for (int rb = 0; rb < H / 32; rb++)
#pragma unroll
                for (int r = 0; r < 16; r++) O[rb][r] *= alpha;
#pragma unroll
            for (int sub = 0; sub < 2; sub++)
#pragma unroll
                for (int r = 0; r < 16; r++)
#pragma unroll
                    for (int rb = 0; rb < H / 32; rb++)
                        O[rb] = __builtin_amdgcn_mfma_f32_32x32x2f32(Vs[(32 * sub + acc_row(r, hh)) * LDV + 32 * rb + ln], s[sub][r], O[rb], 0, 0, 0);
        }
        if (it + 1 < nit) stash((it + 1) & 1);
        __syncthreads();
    }
    lsum += __shfl_xor(lsum, 32, 64);
    store_own_row<H>(rows_of<float>(a.O, sq, H), eq, hh, qvalid, 1.f / lsum, O);
    if (qvalid && hh == 0) {
        float* st = rows_of<float>(a.stats, sq, 2) + 2 * (int64_t)eq;
        st[0] = m * kLn2;
        st[1] = lsum;
    }
}

struct BwdArgs {
    AttnGeom g;
    void* const* Q; void* const* K; void* const* V; void* const* O; void* const* stats; void* const* dO;
    void* const* dQ; void* const* dK; void* const* dV;
    float* aux;     // per (query, batch, head): log2 of the softmax denominator times 2^maximum, and D
};

// ---------------------------------------------------------------- dQ, fp32 (also writes aux)
template <int H>
__global__ void __launch_bounds__(256, 2) attn_dq_f32(const BwdArgs a) {
    using Blk = F32Block<H>;
    __shared__ float lds[2][2 * Blk::kFloats];
    const AttnGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, hh = lane >> 5, ln = lane & 31;
    // under the causal mask the later a query block, the more key blocks it walks: the longest go first
    const int rblk = g.causal ? gridDim.y - 1 - blockIdx.y : blockIdx.y;
    const int l = g.tile0 + rblk / g.nblk, e0 = (rblk % g.nblk) * kWgRows;
    const int b = blockIdx.x % g.Nb, j = blockIdx.x / g.Nb;
    const Slab sq = slab_of(g, l, b, j);
    if (e0 >= sq.ext) return;
    const int eq = e0 + 32 * w + ln;
    const bool qvalid = eq < sq.ext;
    const int qglob = l * g.bs + eq;
    const int wave_qlast = l * g.bs + min(e0 + 32 * w + 31, sq.ext - 1);
    const int wg_qlast = l * g.bs + min(e0 + kWgRows - 1, sq.ext - 1);

    float qf[H / 2], dof[H / 2];
    load_own_row<H>(rows_of<const float>(a.Q, sq, H), eq, hh, qvalid, g.scale * kLog2e, qf);
    load_own_row<H>(rows_of<const float>(a.dO, sq, H), eq, hh, qvalid, 1.f, dof);
    float lse = 0.f, D = 0.f;
    {
        float of[H / 2];
        load_own_row<H>(rows_of<const float>(a.O, sq, H), eq, hh, qvalid, 1.f, of);
#pragma unroll
        for (int k = 0; k < H / 2; k++) D += of[k] * dof[k];
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

    float4 kr[Blk::kVec], vr[Blk::kVec];
    auto fetch = [&](int it) {
        const int lk = it / g.nstep, k0 = (it % g.nstep) * kBlk;
        const Slab sk = slab_of(g, lk, b, j);
        Blk::load(rows_of<const float>(a.K, sk, H), k0, sk.ext, tid, kr);
        Blk::load(rows_of<const float>(a.V, sk, H), k0, sk.ext, tid, vr);
    };
    auto stash = [&](int buf) {
        Blk::store(lds[buf], tid, kr);
        Blk::store(lds[buf] + Blk::kFloats, tid, vr);
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
            const float* Ks = lds[it & 1];
            const float* Vs = Ks + Blk::kFloats;
#pragma unroll
            for (int sub = 0; sub < 2; sub++) {
                f32x16 s = zero16(), dp = zero16();
#pragma unroll
                for (int k = 0; k < H / 2; k++) {
                    s = __builtin_amdgcn_mfma_f32_32x32x2f32(Blk::by_row(Ks, sub, ln, hh, k), qf[k], s, 0, 0, 0);
                    dp = __builtin_amdgcn_mfma_f32_32x32x2f32(Blk::by_row(Vs, sub, ln, hh, k), dof[k], dp, 0, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int kl = 32 * sub + acc_row(r, hh);
                    const bool ok = kloc0 + kl < ext_k && (!g.causal || kglob0 + kl <= qglob);
                    const float p = ok ? __builtin_amdgcn_exp2f(s[r] - lse) : 0.f;
                    s[r] = p * (dp[r] - D);
                }
#pragma unroll
                for (int r = 0; r < 16; r++)
#pragma unroll
                    for (int rb = 0; rb < H / 32; rb++)
                        dQ[rb] = __builtin_amdgcn_mfma_f32_32x32x2f32(Blk::by_col(Ks, sub, rb, ln, hh, r), s[r], dQ[rb], 0, 0, 0);
            }
        }
        if (it + 1 < nit) stash((it + 1) & 1);
        __syncthreads();
    }
    store_own_row<H>(rows_of<float>(a.dQ, sq, H), eq, hh, qvalid, g.scale, dQ);
}

// ---------------------------------------------------------------- dK and dV, fp32 (reads aux)
template <int H>
__global__ void __launch_bounds__(256, 2) attn_dkv_f32(const BwdArgs a) {
    using Blk = F32Block<H>;
    __shared__ float lds[2][2 * Blk::kFloats + 2 * kBlk];
    const AttnGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, hh = lane >> 5, ln = lane & 31;
    // (under the causal mask the earliest key blocks meet the most query blocks: already first)
    const int l = g.tile0 + blockIdx.y / g.nblk, e0 = (blockIdx.y % g.nblk) * kWgRows;
    const int b = blockIdx.x % g.Nb, j = blockIdx.x / g.Nb;
    const Slab sk = slab_of(g, l, b, j);
    if (e0 >= sk.ext) return;
    const int ek = e0 + 32 * w + ln;
    const bool kvalid = ek < sk.ext;
    const int kglob = l * g.bs + ek;
    const int wave_kfirst = l * g.bs + e0 + 32 * w;

    float kf[H / 2], vf[H / 2];
    load_own_row<H>(rows_of<const float>(a.K, sk, H), ek, hh, kvalid, g.scale * kLog2e, kf);
    load_own_row<H>(rows_of<const float>(a.V, sk, H), ek, hh, kvalid, 1.f, vf);

    const int nit = (g.gs - 1) * g.nstep + (g.Ns - (g.gs - 1) * g.bs + kBlk - 1) / kBlk;
    // with the causal mask the first query block that sees any of these keys is the one that holds key e0
    const int it0 = g.causal ? l * g.nstep + e0 / kBlk : 0;

    f32x16 dK[H / 32], dV[H / 32];
#pragma unroll
    for (int rb = 0; rb < H / 32; rb++) { dK[rb] = zero16(); dV[rb] = zero16(); }

    float4 qr[Blk::kVec], dr[Blk::kVec];
    float2 ar = make_float2(0.f, 0.f);
    auto fetch = [&](int it) {
        const int lq = it / g.nstep, q0 = (it % g.nstep) * kBlk;
        const Slab sq = slab_of(g, lq, b, j);
        Blk::load(rows_of<const float>(a.Q, sq, H), q0, sq.ext, tid, qr);
        Blk::load(rows_of<const float>(a.dO, sq, H), q0, sq.ext, tid, dr);
        if (tid < kBlk) {
            const bool ok = q0 + tid < sq.ext;
            const int64_t qg = (int64_t)lq * g.bs + q0 + tid;
            ar = ok ? *reinterpret_cast<const float2*>(a.aux + 2 * (qg + (int64_t)g.Ns * (b + (int64_t)g.Nb * j))) : make_float2(0.f, 0.f);
        }
    };
    auto stash = [&](int buf) {
        Blk::store(lds[buf], tid, qr);
        Blk::store(lds[buf] + Blk::kFloats, tid, dr);
        if (tid < kBlk) {
            lds[buf][2 * Blk::kFloats + tid] = ar.x;
            lds[buf][2 * Blk::kFloats + kBlk + tid] = ar.y;
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
            const float* Qs = lds[it & 1];
            const float* Ds = Qs + Blk::kFloats;
            const float* lses = Ds + Blk::kFloats;
            const float* dsum = lses + kBlk;
#pragma unroll
            for (int sub = 0; sub < 2; sub++) {
                f32x16 s = zero16(), dp = zero16();
#pragma unroll
                for (int k = 0; k < H / 2; k++) {
                    s = __builtin_amdgcn_mfma_f32_32x32x2f32(Blk::by_row(Qs, sub, ln, hh, k), kf[k], s, 0, 0, 0);
                    dp = __builtin_amdgcn_mfma_f32_32x32x2f32(Blk::by_row(Ds, sub, ln, hh, k), vf[k], dp, 0, 0, 0);
                }
                f32x16 p;
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int ql = 32 * sub + acc_row(r, hh);
                    const bool ok = qloc0 + ql < ext_q && (!g.causal || kglob <= qglob0 + ql);
                    p[r] = ok ? __builtin_amdgcn_exp2f(s[r] - lses[ql]) : 0.f;
                    s[r] = p[r] * (dp[r] - dsum[ql]);
                }
#pragma unroll
                for (int r = 0; r < 16; r++)
#pragma unroll
                    for (int rb = 0; rb < H / 32; rb++) {
                        dV[rb] = __builtin_amdgcn_mfma_f32_32x32x2f32(Blk::by_col(Ds, sub, rb, ln, hh, r), p[r], dV[rb], 0, 0, 0);
                        dK[rb] = __builtin_amdgcn_mfma_f32_32x32x2f32(Blk::by_col(Qs, sub, rb, ln, hh, r), s[r], dK[rb], 0, 0, 0);
                    }
            }
        }
        if (it + 1 < nit) stash((it + 1) & 1);
        __syncthreads();
    }
    store_own_row<H>(rows_of<float>(a.dK, sk, H), ek, hh, kvalid, g.scale, dK);
    store_own_row<H>(rows_of<float>(a.dV, sk, H), ek, hh, kvalid, 1.f, dV);
}

}  // namespace
}  // namespace nnt

using namespace nnt;

// ------------------------------------------------------------------ host side
namespace {

int32_t check_attn(nnt_ctx* ctx, const char* who, std::initializer_list<const nnt_tensor*> ts, const nnt_tensor* stats) {
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
    if (first->dtype != NNT_F32) return fail(ctx, NNT_EDTYPE, std::string(who) + ": fp32 only");
    if (first->shape[0] != 64 && first->shape[0] != 128)
        return fail(ctx, NNT_EINVAL, std::string(who) + ": head size must be 64 or 128");
    if (!stats) return fail(ctx, NNT_EINVAL, std::string(who) + ": null tensor");
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
    return g;
}

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
    int32_t rc = check_attn(ctx, "nnt_attention_fwd", {Q, K, V, B}, stats);
    if (rc != NNT_OK) return rc;
    AttnGeom g = geom_of(Q, scale, causal);
    FwdArgs a{g, Q->d_tiles, K->d_tiles, V->d_tiles, B->d_tiles, stats->d_tiles};
    const double pair_flops = 4.0 * g.H * g.Nb * g.Nh;   // two products, 2 flops per multiply-add
    auto launch = [](hipStream_t st, const FwdArgs& fa, int ntile) {
        const dim3 grid((unsigned)(fa.g.Nb * fa.g.Nh), (unsigned)(ntile * fa.g.nblk)), block(256);
        if (fa.g.H == 64) hipLaunchKernelGGL(attn_fwd_f32<64>, grid, block, 0, st, fa);
        else hipLaunchKernelGGL(attn_fwd_f32<128>, grid, block, 0, st, fa);
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
    int32_t rc = check_attn(ctx, "nnt_attention_bwd", {Q, K, V, B, dB, dQ, dK, dV}, stats);
    if (rc != NNT_OK) return rc;
    AttnGeom g = geom_of(Q, scale, causal);
    rc = ensure_scratch(ctx, 2 * (int64_t)g.Ns * g.Nb * g.Nh);
    if (rc != NNT_OK) return rc;
    BwdArgs a{g, Q->d_tiles, K->d_tiles, V->d_tiles, B->d_tiles, stats->d_tiles, dB->d_tiles,
              dQ->d_tiles, dK->d_tiles, dV->d_tiles, ctx->red_scratch};
    const double pair_flops = 2.0 * g.H * g.Nb * g.Nh;   // per product
    const double pairs = visible_pairs(g.Ns, 0, g.Ns, causal);
    const Access scr{&ctx->red_dep, 1, kReadWrite};
    // one task, two launches: the dQ kernel leaves log-sum-exp and D per query for the dK/dV kernel
    OpTag tag(ctx, "attention_bwd_dq", 3.0 * pair_flops * pairs, false);
    return submit(ctx, {Q->all(kRead), K->all(kRead), V->all(kRead), B->all(kRead), stats->all(kRead), dB->all(kRead),
                        dQ->all(kWrite), dK->all(kWrite), dV->all(kWrite), scr},
                  [=](hipStream_t st) {
                      const dim3 grid((unsigned)(a.g.Nb * a.g.Nh), (unsigned)(a.g.gs * a.g.nblk)), block(256);
                      if (a.g.H == 64) hipLaunchKernelGGL(attn_dq_f32<64>, grid, block, 0, st, a);
                      else hipLaunchKernelGGL(attn_dq_f32<128>, grid, block, 0, st, a);
                      if (hipGetLastError() != hipSuccess) return (int32_t)NNT_EHIP;
                      profile_mark(ctx, st, "attention_bwd_dkv", 4.0 * pair_flops * pairs, false);
                      if (a.g.H == 64) hipLaunchKernelGGL(attn_dkv_f32<64>, grid, block, 0, st, a);
                      else hipLaunchKernelGGL(attn_dkv_f32<128>, grid, block, 0, st, a);
                      return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
                  }, 2);
}
