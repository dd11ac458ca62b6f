// Tile-grid products: the single-tile entry point and the tensor-level nnt_gemm,
// which turns a contraction of tiled tensors into a cached plan (tables of tasks,
// chunks and workgroups in device memory) and submits it to the executor.
#include "gemm_common.hpp"
#include "internal.hpp"

#include <algorithm>
#include <cstdlib>
#include <sstream>

namespace nnt {

// One macro-tile of C whose contraction was cut into k-slices: where the slices lie and where
// the sum goes.
struct SplitReduce {
    void* C;                // base of the C tile
    const float* bias;      // bias of the C tile (length m of the tile), or nullptr
    const float* ws;        // slice s of element (i, j) of the macro-tile at ws[s * slice + j * ldw + i]
    int64_t ldc, slice;
    int32_t m0, n0, rows, cols, ldw, nsplit;
    int64_t cin_off;        // the beta term is read at C + cin_off elements (0: C itself; else a residual input's tile)
};

template <typename TO>
__global__ void __launch_bounds__(256) splitk_reduce(const SplitReduce* tab, float alpha, float beta) {
    const SplitReduce t = tab[blockIdx.y];
    const int q = t.ldw >> 2;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int i = (idx % q) << 2, j = idx / q;
    if (j >= t.cols || i >= t.rows) return;
    const int n = t.rows - i < 4 ? t.rows - i : 4;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const float* p = t.ws + (int64_t)j * t.ldw + i;       // 16-byte aligned: ldw is a multiple of 4
    // slices are added in their fixed order; four loads are started before the first of them is used
    int sl = 0;
    for (; sl + 4 <= t.nsplit; sl += 4) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; u++) v[u] = *reinterpret_cast<const float4*>(p + (int64_t)(sl + u) * t.slice);
#pragma unroll
        for (int u = 0; u < 4; u++) {
            acc[0] += v[u].x; acc[1] += v[u].y; acc[2] += v[u].z; acc[3] += v[u].w;
        }
    }
    for (; sl < t.nsplit; sl++) {
        const float4 v = *reinterpret_cast<const float4*>(p + (int64_t)sl * t.slice);
        acc[0] += v.x; acc[1] += v.y; acc[2] += v.z; acc[3] += v.w;
    }
    TO* c = static_cast<TO*>(t.C) + (t.m0 + i) + (int64_t)(t.n0 + j) * t.ldc;
    if constexpr (sizeof(TO) == 4) {
        // four whole rows at a 16-byte aligned address: one vector access instead of four
        if (n == 4 && (reinterpret_cast<uintptr_t>(c) & 15) == 0 && (t.cin_off & 3) == 0) {
            float4 o = make_float4(alpha * acc[0], alpha * acc[1], alpha * acc[2], alpha * acc[3]);
            if (t.bias) {
                const float* bp = t.bias + t.m0 + i;
                o.x += bp[0]; o.y += bp[1]; o.z += bp[2]; o.w += bp[3];
            }
            float4* c4 = reinterpret_cast<float4*>(c);
            if (beta != 0.f) {
                const float4 old = *reinterpret_cast<const float4*>(c + t.cin_off);
                o.x += beta * old.x; o.y += beta * old.y; o.z += beta * old.z; o.w += beta * old.w;
            }
            *c4 = o;
            return;
        }
    } else {
        if (n == 4 && (reinterpret_cast<uintptr_t>(c) & 7) == 0 && (t.cin_off & 3) == 0) {
            float o[4];
            uint2* c2 = reinterpret_cast<uint2*>(c);
            uint2 old = make_uint2(0u, 0u);
            if (beta != 0.f) old = *reinterpret_cast<const uint2*>(c + t.cin_off);
            const uint32_t ow[2] = {old.x, old.y};
#pragma unroll
            for (int jj = 0; jj < 4; jj++) {
                o[jj] = alpha * acc[jj];
                if (t.bias) o[jj] += t.bias[t.m0 + i + jj];
                if (beta != 0.f) o[jj] += beta * __uint_as_float((jj & 1) ? (ow[jj >> 1] & 0xffff0000u) : (ow[jj >> 1] << 16));
            }
            uint32_t h[4];
#pragma unroll
            for (int jj = 0; jj < 4; jj++) {
                const __bf16 b = (__bf16)o[jj];
                h[jj] = (uint32_t)__builtin_bit_cast(uint16_t, b);
            }
            *c2 = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
            return;
        }
    }
    for (int jj = 0; jj < n; jj++) {
        float v = alpha * acc[jj];
        if (t.bias) v += t.bias[t.m0 + i + jj];
        if (beta != 0.f) {
            if constexpr (sizeof(TO) == 4) v += beta * (float)c[t.cin_off + jj];
            else v += beta * __uint_as_float((uint32_t)c[t.cin_off + jj] << 16);
        }
        if constexpr (sizeof(TO) == 4) c[jj] = v;
        else { const __bf16 h = (__bf16)v; c[jj] = __builtin_bit_cast(uint16_t, h); }
    }
}

struct GemmPlan {
    nnt_ctx* ctx = nullptr;
    uint64_t ids[5] = {0, 0, 0, 0, 0};         // tensors the tables point into (A, B, C, bias, residual input)
    int dtype_in = NNT_F32, dtype_out = NNT_F32;
    int akf = 0, bkf = 0, cfg = kCfgSquare;
    double flops = 0.0;                        // 2 m n k summed over tasks, chunks and batch members
    std::string label;                         // the kernel instance that runs the plan
    std::vector<GemmTask> tasks;
    std::vector<GemmChunk> chunks;
    std::vector<GemmWg> wgs, wgs_op;
    std::vector<int64_t> task_wg0;             // first workgroup of each task (+ total at the end)
    std::vector<int64_t> task_nfast;           // leading workgroups of each task that qualify for the direct-load kernel
    int64_t op_nfast = 0;                      // the same for the whole-operation order
    int64_t table_bytes = 0, ws_bytes = 0;     // device memory of the descriptor tables / the k-slice workspaces
    int epi_mode = 0;                          // GemmEpi mode of a product with an activation on its result path
    bool epi_ok = false;                       // every workgroup runs in a direct-load kernel that has that form
    bool dl_ragged = false;                    // they need the direct-load kernel's variant for ragged macro-tiles and short k-steps
    std::vector<int64_t> task_ctile;           // C tile index per task
    std::vector<std::vector<int64_t>> task_atiles, task_btiles;   // operand tiles per task (dependencies)
    std::vector<int64_t> task_bias_tile;
    GemmTask* d_tasks = nullptr;
    GemmChunk* d_chunks = nullptr;
    GemmWg* d_wgs = nullptr;
    GemmWg* d_wgs_op = nullptr;
    // Whole-operation launches may cut the contraction of some macro-tiles (the last `n_split`
    // of the launch order) into `splits` k-slices: each slice is a workgroup of its own that
    // writes raw fp32 sums to scratch memory, and a second kernel adds the slices in a fixed
    // order and applies alpha, beta and the bias.  The extra tasks and chunks of the slices
    // follow the regular ones in the same device tables.
    int splits = 1;
    int64_t n_split = 0, op_nwg = 0;
    int red_blocks = 0;
    int64_t slice_elems = 0;                   // elements of one slice of one cut macro-tile
    SplitReduce* d_red = nullptr;
    float* d_ws = nullptr;
    TileDep ws_dep;
    // Per-tile launches: a task that has only a few macro-tiles but a long contraction (a tile of a
    // weight gradient: 256 x 256 over all tokens) would leave the chip idle, so its contraction is cut
    // the same way, into its own scratch block (tasks of one operation run concurrently on several
    // streams), followed by the slice sum over just that task's macro-tiles.
    struct TileSplit { int64_t wg0 = 0, nwg = 0, nfast = 0, red0 = 0, nred = 0; };
    std::vector<TileSplit> tile_split;         // per task; nwg == 0: launched whole
    std::vector<GemmWg> wgs_ts;
    int64_t slice_elems_ts = 0;
    GemmWg* d_wgs_ts = nullptr;
    SplitReduce* d_red_ts = nullptr;
    float* d_ws_ts = nullptr;
    ~GemmPlan() {
        for (void* p : {(void*)d_tasks, (void*)d_chunks, (void*)d_wgs, (void*)d_wgs_op, (void*)d_red, (void*)d_ws, (void*)d_wgs_ts,
                        (void*)d_red_ts, (void*)d_ws_ts})
            if (p) (void)hipFree(p);
    }
};

void plan_device_bytes(nnt_ctx* ctx, int64_t* tables, int64_t* workspaces) {
    for (const auto& kv : ctx->gemm_plans) {
        *tables += kv.second->table_bytes;
        *workspaces += kv.second->ws_bytes;
    }
}

void drop_plans_of(nnt_ctx* ctx, uint64_t id) {
    for (auto it = ctx->gemm_plans.begin(); it != ctx->gemm_plans.end();) {
        const uint64_t* ids = it->second->ids;
        if (ids[0] == id || ids[1] == id || ids[2] == id || ids[3] == id || ids[4] == id) it = ctx->gemm_plans.erase(it);
        else ++it;
    }
}

// The first `nfast` workgroups of the table qualify for the direct-load kernel of the type.
static int32_t launch_any(hipStream_t st, int dtype_in, int dtype_out, int akf, int bkf, int cfg,
                          const GemmArgs& g, int64_t nwg, int64_t nfast = 0, bool ragged = false, int epi_mode = 0) {
    const bool f32 = dtype_in == NNT_F32;
    if (epi_mode) {     // (plans with an activation form are only run when all their workgroups qualify: GemmPlan::epi_ok)
        if (nfast != nwg) return NNT_EINVAL;
        return f32 ? launch_gemm_f32_dl(st, akf, bkf, cfg, g, nwg, epi_mode) : NNT_EINVAL;
    }
    auto general = [&](const GemmArgs& ga, int64_t n) {
        return f32 ? launch_gemm_f32(st, akf, bkf, cfg, ga, n) : launch_gemm_bf16(st, dtype_out == NNT_F32, akf, bkf, cfg, ga, n);
    };
    // debugging aid: NNT_GEMM_NO_DL=1 sends every workgroup to the general kernels
    static const bool no_dl = getenv("NNT_GEMM_NO_DL") != nullptr;
    if (nfast <= 0 || no_dl) return general(g, nwg);
    int32_t rc = f32 ? launch_gemm_f32_dl(st, akf, bkf, cfg, g, nfast) : launch_gemm_bf16_dl(st, dtype_out == NNT_F32, akf, bkf, cfg, ragged, g, nfast);
    if (rc != NNT_OK || nfast == nwg) return rc;
    GemmArgs rest = g;
    if (rest.wgs) rest.wgs += nfast;
    return general(rest, nwg - nfast);
}

static int vec_flag(const void* p, int64_t ld, int64_t stride, int elem) {
    const int per = 16 / elem;
    return ((uintptr_t)p % 16 == 0) && (ld % per == 0) && (stride % per == 0);
}

// Workgroups are handed to the 8 XCDs (each with its own L2) in turn by their linear id, so the
// workgroups with id = x (mod 8) run on XCD x, about one per CU at a time.  The list arrives in
// tile order (rows fastest, then columns, batch members, tasks).  Each macro-tile grid is cut into
// blocks of 16 x 16 tiles; inside a block XCD x owns a sub-block of 8 x 4 tiles, so the workgroups
// that an XCD runs together need 8 + 4 operand panels instead of up to 33, and the eight XCDs
// together work on one compact 16 x 16 region whose panels meet in the last-level cache.  Small
// grids (batched attention products) go to one XCD each.  The per-XCD queues are then dealt out
// in turn; a queue that runs dry takes work from the longest one.
static void xcd_interleave(std::vector<GemmWg>& wgs, int bm, int bn) {
    const size_t n = wgs.size();
    if (n < 64) return;
    std::vector<GemmWg> q[8];
    int small_turn = 0;
    size_t a = 0;
    while (a < n) {
        size_t b = a;
        int gm = 0, gn = 0;
        while (b < n && wgs[b].task == wgs[a].task && wgs[b].batch == wgs[a].batch) {
            gm = std::max(gm, wgs[b].m0 / bm + 1);
            gn = std::max(gn, wgs[b].n0 / bn + 1);
            b++;
        }
        if ((size_t)gm * gn != b - a || gm * gn < 64) {
            // small or irregular grid: keep it together on one XCD
            std::vector<GemmWg>& dst = q[small_turn++ & 7];
            dst.insert(dst.end(), wgs.begin() + a, wgs.begin() + b);
        } else {
            for (int J = 0; J < gn; J += 16)
                for (int I = 0; I < gm; I += 16)
                    for (int x = 0; x < 8; x++)
                        for (int j = 0; j < 4; j++)
                            for (int i = 0; i < 8; i++) {
                                const int ii = I + (x & 1) * 8 + i, jj = J + (x >> 1) * 4 + j;
                                if (ii < gm && jj < gn) q[x].push_back(wgs[a + (size_t)jj * gm + ii]);
                            }
        }
        a = b;
    }
    std::vector<GemmWg> out;
    out.reserve(n);
    size_t head[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    while (out.size() < n) {
        for (int x = 0; x < 8 && out.size() < n; x++) {
            if (head[x] < q[x].size()) {
                out.push_back(q[x][head[x]++]);
            } else {
                int longest = 0;
                for (int y = 1; y < 8; y++)
                    if (q[y].size() - head[y] > q[longest].size() - head[longest]) longest = y;
                out.push_back(q[longest].back());
                q[longest].pop_back();
            }
        }
    }
    wgs.swap(out);
}

// Cost model for a product of whole matrices (no batch axes): picks the macro-tile shape, how
// many macro-tiles get their contraction cut into k-slices, and into how many.  The matrix cores
// bound these kernels, so a compute unit that holds two workgroups needs twice as long as one
// that holds one: a launch of W equal workgroups takes ceil(W / 256) workgroup times, plus the
// start-up of a workgroup (first loads, result stores), which overlaps only with other
// workgroups on the same unit.  A launch whose W is not a multiple of 256 leaves units idle in
// its last round; cutting the W mod 256 macro-tiles of that round into s slices turns it into
// 1/s of a round.  A launch with few macro-tiles cuts all of them.  Slices cost a second pass
// over the fp32 partial results.  The rates are measured ones (large products of each shape);
// the model only has to rank the candidates.
constexpr int kSplitStep = 64;
struct ShapeChoice { int cfg; int64_t n_split; int s; };
// `ragged`: tile extents or chunk lengths that only the 256 x 128 bf16 direct-load kernel takes (the 256 x 256
// shape would run on the general kernel, at about a third of the rate).
static ShapeChoice choose_shape(bool bf16, bool out_f32, int akf, int bkf, const std::vector<int64_t>& tm,
                                const std::vector<int64_t>& tn, const std::vector<int64_t>& ktot, bool may_split, bool ragged = false) {
    // rate of a compute unit with its full set of workgroups; start-up time of a workgroup; factor by
    // which a workgroup that is alone on its unit is slower than its share of that rate
    struct Cand { int cfg; double flops_per_s_cu; double t0; double solo; };
    static const Cand f32c[] = {{kCfgSquare, 0.56e12, 2.5e-6, 1.7}, {kCfgMid, 0.45e12, 2.0e-6, 1.3}};
    static const Cand bf16c[] = {{kCfgSquare, 4.4e12, 8.0e-6, 1.0}, {kCfgTall, 4.2e12, 3.0e-6, 1.6}, {kCfgMid, 1.6e12, 3.0e-6, 1.5}};
    static const Cand bf16r[] = {{kCfgSquare, 1.5e12, 8.0e-6, 1.0}, {kCfgTall, 4.0e12, 3.0e-6, 1.6}, {kCfgMid, 1.6e12, 3.0e-6, 1.5}};
    const Cand* cands = bf16 ? (ragged ? bf16r : bf16c) : f32c;
    const int ncand = bf16 ? 3 : 2;
    ShapeChoice best = {kCfgSquare, 0, 1};
    double best_t = 1e30;
    int64_t kmax = 0, kmin = INT64_MAX;
    for (int64_t kq : ktot) { kmax = std::max(kmax, kq); kmin = std::min(kmin, kq); }
    for (int ci = 0; ci < ncand; ci++) {
        const Cand& cd = cands[ci];
        int bm, bn;
        gemm_cfg_tile(bf16, cd.cfg, &bm, &bn);
        const int occ = !bf16 ? gemm_f32_dl_occupancy(akf, bkf, cd.cfg)
                        : (cd.cfg == kCfgMid ? gemm_bf16_occupancy(out_f32, akf, bkf, cd.cfg) : gemm_bf16_dl_occupancy(out_f32, akf, bkf, cd.cfg));
        const int64_t G = 256 * (int64_t)occ;      // workgroups resident at a time
        int64_t W = 0;
        for (size_t i = 0; i < tm.size(); i++) W += ((tm[i] + bm - 1) / bm) * ((tn[i] + bn - 1) / bn);
        auto tile_time = [&](int64_t k) { return 2.0 * bm * bn * (double)k / cd.flops_per_s_cu; };
        // X equal workgroups: whole resident sets, each as slow as `occ` workgroups in a row on
        // every unit, then a last set spread over the units
        auto group_time = [&](int64_t X, int64_t k) {
            const int64_t last = (X % G + 255) / 256;          // workgroups per unit in the last, partial set
            const double last_t = (last == 1 && occ > 1) ? cd.solo : (double)last;
            return ((double)(X / G) * occ + last_t) * tile_time(k) + (double)((X + G - 1) / G) * cd.t0;
        };
        const double t_plain = group_time(W, kmax);
        if (t_plain < best_t) { best_t = t_plain; best = {cd.cfg, 0, 1}; }
        if (!may_split) continue;
        const int64_t R = W % G;
        const int64_t ns_cands[2] = {W, (W > G && R > 0) ? R : 0};
        for (int64_t ns : ns_cands) {
            if (ns <= 0) continue;
            for (int sp = 2; sp <= 32; sp++) {
                const int64_t part = ((kmax + sp - 1) / sp + kSplitStep - 1) / kSplitStep * kSplitStep;
                if (part < 256 || part * (sp - 1) >= kmin) break;
                const double t = (ns < W ? group_time(W - ns, kmax) : 0.0) + group_time(ns * sp, part) + 6e-6 +
                                 (double)ns * bm * bn * 4.0 * (sp + 1) / 3.5e12;
                if (t < best_t) { best_t = t; best = {cd.cfg, ns, sp}; }
            }
        }
    }
    return best;
}

// `kk`: both operands are k-contiguous (A read transposed, B as [k, n]).
static int pick_cfg(int bf16, int64_t m_max, int64_t n_max, int64_t n_tiles_big, int64_t k_max, bool kk = false) {
    // fp32 products whose whole contraction is a head size and whose result is score-shaped: bound by their result
    // stores, which a workgroup waits out before it ends, so the shape of which a compute unit holds three
    if (!bf16 && kk && k_max <= 64 && m_max >= 64 && n_max >= 128) return kCfgResident;
    // bf16 products with few rows (m = head size) read a score-shaped operand and are bound by that traffic: the
    // 128-row direct-load shape streams it four k-steps ahead
    if (bf16 && m_max <= 128) return kCfgWide;
    if (m_max <= 64) return kCfgSkinny64n128;                         // (fp32 from here to the next line) the shape its direct-load kernel has
    if (m_max <= 128 && n_max > 128) return kCfgSkinny128;
    if (bf16 && (m_max <= 128 || n_max <= 128 || n_tiles_big < 256)) return kCfgMid;
    // short contractions are bound by the result stores: several small workgroups per compute
    // unit overlap one's stores with another's loads, one large workgroup cannot
    // (tiles that are not whole macro-tiles go to the ragged variant of that kernel: C4's tiles of 400 are 256 + 144 by 3 x 128 + 16)
    if (bf16 && k_max <= 128) return (m_max >= 256 && n_max >= 128) ? kCfgTall : kCfgMid;
    return kCfgSquare;
}

}  // namespace nnt

using namespace nnt;

extern "C" int32_t nnt_tile_gemm(void* stream, int32_t dtype_in, int32_t dtype_out, int32_t opA, int32_t opB,
                                 int64_t m, int64_t n, int64_t k, int64_t batch, float alpha,
                                 const void* A, int64_t lda, int64_t strideA,
                                 const void* B, int64_t ldb, int64_t strideB,
                                 float beta, void* C, int64_t ldc, int64_t strideC) {
    if (dtype_in != NNT_F32 && dtype_in != NNT_BF16) return NNT_EDTYPE;
    if (dtype_out != NNT_F32 && dtype_out != NNT_BF16) return NNT_EDTYPE;
    if (dtype_in == NNT_F32 && dtype_out != NNT_F32) return NNT_EDTYPE;
    if ((opA != NNT_OP_N && opA != NNT_OP_T) || (opB != NNT_OP_N && opB != NNT_OP_T)) return NNT_EINVAL;
    if (m < 0 || n < 0 || k < 0 || batch < 0 || m > INT32_MAX || n > INT32_MAX || k > INT32_MAX) return NNT_EINVAL;
    if (m == 0 || n == 0 || batch == 0) return NNT_OK;
    if (!C || (k > 0 && (!A || !B))) return NNT_EINVAL;
    const int64_t a_rows = opA == NNT_OP_N ? m : k, b_rows = opB == NNT_OP_N ? k : n;
    if (ldc < m || (k > 0 && (lda < a_rows || ldb < b_rows))) return NNT_EINVAL;
    const int bf = dtype_in == NNT_BF16;
    const int elem = bf ? 2 : 4;
    GemmArgs g = {};
    g.wgs = nullptr;
    g.one_task = GemmTask{};
    g.one_task.C = C;
    g.one_task.bias = nullptr;
    g.one_task.ldc = ldc;
    g.one_task.strideC = strideC;
    g.one_task.m = (int32_t)m;
    g.one_task.n = (int32_t)n;
    g.one_task.chunk0 = 0;
    g.one_task.nchunk = k > 0 ? 1 : 0;
    g.one_chunk.A = A;
    g.one_chunk.B = B;
    g.one_chunk.lda = lda;
    g.one_chunk.ldb = ldb;
    g.one_chunk.strideA = strideA;
    g.one_chunk.strideB = strideB;
    g.one_chunk.k = (int32_t)k;
    g.one_chunk.vec_ok = vec_flag(A, lda, strideA, elem) | (vec_flag(B, ldb, strideB, elem) << 1);
    g.alpha = alpha;
    g.beta = beta;
    int bm, bn;
    int cfg = pick_cfg(bf, m, n, ((m + 255) / 256) * ((n + 255) / 256) * batch, k, opA == NNT_OP_T && opB == NNT_OP_N);
    const bool odd_shape = bf && (m % 256 != 0 || n % 256 != 0 || k % 64 != 0);
    if (batch == 1 && (cfg == kCfgSquare || cfg == kCfgMid || cfg == kCfgTall))
        cfg = choose_shape(bf, dtype_out == NNT_F32, opA == NNT_OP_T, opB == NNT_OP_N, {m}, {n}, {k}, false, odd_shape).cfg;
    // debugging aid: NNT_TILE_GEMM_CFG=<number of a macro-tile configuration> overrides the choice for this entry point
    static const char* const force = getenv("NNT_TILE_GEMM_CFG");
    if (force && atoi(force) >= kCfgSquare && atoi(force) <= kCfgWide) cfg = atoi(force);      // (not kCfgResident: it exists for one operand form)
    gemm_cfg_tile(bf, cfg, &bm, &bn);
    g.grid_m = (int32_t)((m + bm - 1) / bm);
    g.grid_n = (int32_t)((n + bn - 1) / bn);
    const int64_t nwg = (int64_t)g.grid_m * g.grid_n * batch;
    if (nwg > INT32_MAX) return NNT_EINVAL;
    bool fast = (bf ? (cfg == kCfgSquare || cfg == kCfgTall || cfg == kCfgWide) : (cfg == kCfgSquare || cfg == kCfgSkinny64n128 || cfg == kCfgMid || cfg == kCfgResident)) &&
                m % bm == 0 && n % bn == 0 && k > 0 && k % ((bf && cfg == kCfgSquare) ? 64 : 32) == 0 && g.one_chunk.vec_ok == 3;
    bool ragged = false;
    if (!fast && bf && (cfg == kCfgTall || cfg == kCfgWide) && k > 0 && k % 8 == 0 && g.one_chunk.vec_ok == 3) {
        // the variant for macro-tiles that end inside the tile and for a short last k-step
        const bool akf = opA == NNT_OP_T, bkf = opB == NNT_OP_N;
        fast = ragged = (akf || (m % bm) % 8 == 0) && (bkf || (n % bn) % 8 == 0);
    }
    return launch_any((hipStream_t)stream, dtype_in, dtype_out, opA == NNT_OP_T, opB == NNT_OP_N, cfg, g, nwg, fast ? nwg : 0, ragged);
}

// ---------------------------------------------------------------- tensor-level product
namespace {

struct AxisMap {
    std::vector<int> a_free, a_con, b_con, b_free, a_bat, b_bat;
};

int64_t prod_extent(const nnt_tensor* t, const int64_t* tc, const std::vector<int>& axes) {
    int64_t p = 1;
    for (int a : axes) p *= t->tile_extent(a, tc[a]);
    return p;
}

// Appends to P->chunks the chunks of `S` consecutive k-slices of task `t0` (slice lengths in multiples
// of the step the kernels want) and returns (first chunk, chunk count) per slice.
std::vector<std::pair<int32_t, int32_t>> cut_into_slices(GemmPlan* P, const GemmTask& t0, int64_t ktot, int S, int elem) {
    std::vector<std::pair<int32_t, int32_t>> ranges;
    const int64_t part = ((ktot + S - 1) / S + kSplitStep - 1) / kSplitStep * kSplitStep;
    int32_t q = t0.chunk0;
    int64_t used = 0;                       // k already consumed of chunk q
    for (int sidx = 0; sidx < S; sidx++) {
        const int32_t c0i = (int32_t)P->chunks.size();
        int64_t want = part;
        while (want > 0 && q < t0.chunk0 + t0.nchunk) {
            const GemmChunk c0 = P->chunks[q];
            const int64_t take = std::min<int64_t>(want, c0.k - used);
            GemmChunk c = c0;
            c.A = static_cast<const char*>(c0.A) + used * (P->akf ? 1 : c0.lda) * elem;
            c.B = static_cast<const char*>(c0.B) + used * (P->bkf ? 1 : c0.ldb) * elem;
            c.k = (int32_t)take;
            c.vec_ok = vec_flag(c.A, c.lda, c.strideA, elem) | (vec_flag(c.B, c.ldb, c.strideB, elem) << 1);
            P->chunks.push_back(c);
            want -= take;
            used += take;
            if (used == c0.k) { q++; used = 0; }
        }
        ranges.push_back({c0i, (int32_t)P->chunks.size() - c0i});
    }
    return ranges;
}

// The slices of macro-tile `mw` of task `t0`: one partial task per slice, writing raw fp32 sums into
// `block` (slice after slice, bm x bn each), appended to P->tasks; their workgroups go to `by_slice`.
// Returns the record from which the slice-sum kernel finishes the macro-tile.
SplitReduce add_slice_tasks(GemmPlan* P, const GemmTask& t0, const GemmWg& mw, const std::vector<std::pair<int32_t, int32_t>>& ranges,
                            float* block, int bm, int bn, std::vector<std::vector<GemmWg>>& by_slice) {
    const int S = (int)ranges.size();
    const int64_t slice = (int64_t)bm * bn;
    SplitReduce r;
    r.C = t0.C; r.bias = t0.bias; r.ws = block; r.ldc = t0.ldc; r.slice = slice; r.cin_off = t0.cin_off;
    r.m0 = mw.m0; r.n0 = mw.n0;
    r.rows = std::min<int32_t>(bm, t0.m - mw.m0);
    r.cols = std::min<int32_t>(bn, t0.n - mw.n0);
    r.ldw = bm; r.nsplit = S;
    for (int sidx = 0; sidx < S; sidx++) {
        GemmTask t = t0;
        // element (m0 + i, n0 + j) of the "tile" lands on block[i + j * bm] of this slice
        t.C = block + (int64_t)sidx * slice - (mw.m0 + (int64_t)mw.n0 * bm);
        t.ldc = bm;
        t.strideC = 0;
        t.bias = nullptr;
        t.cin_off = 0;
        t.epi = 0;
        t.partial = 1;
        t.chunk0 = ranges[sidx].first;
        t.nchunk = ranges[sidx].second;
        by_slice[sidx].push_back(GemmWg{(int32_t)P->tasks.size(), mw.m0, mw.n0, 0});
        P->tasks.push_back(t);
    }
    return r;
}

// `view_ld` (or nullptr): per operand (A, B, C) the leading dimension of a tensor that is a window on a tensor
// with the heads side by side along its first axis (see nnt_gemm_heads), or 0 for an ordinary tensor.  With it
// the two batch axes stay apart (batch member, head): GemmTask::nb1 and the second strides.
int32_t build_plan(nnt_ctx* ctx, int opA, nnt_tensor* A, int opB, nnt_tensor* B, nnt_tensor* C, int ncon, int nbat,
                   nnt_tensor* bias, nnt_tensor* R, GemmPlan* P, const int64_t* view_ld = nullptr, int epi = 0) {
    const bool pairs = view_ld != nullptr;
    if (epi && (nbat != 0 || !R || pairs)) return fail(ctx, NNT_EINVAL, "nnt_gemm_gelu: unsupported form");
    if (pairs && (nbat != 2 || ncon != 1 || bias || R)) return fail(ctx, NNT_EINVAL, "nnt_gemm_heads: unsupported form");
    const int na = A->ndim - nbat, nb = B->ndim - nbat;
    if (ncon < 1 || nbat < 0 || na < ncon || nb < ncon)
        return fail(ctx, NNT_EINVAL, "nnt_gemm: axis counts do not fit the operands");
    AxisMap ax;
    if (opA == NNT_OP_N) { for (int i = 0; i < na - ncon; i++) ax.a_free.push_back(i); for (int i = na - ncon; i < na; i++) ax.a_con.push_back(i); }
    else { for (int i = 0; i < ncon; i++) ax.a_con.push_back(i); for (int i = ncon; i < na; i++) ax.a_free.push_back(i); }
    if (opB == NNT_OP_N) { for (int i = 0; i < ncon; i++) ax.b_con.push_back(i); for (int i = ncon; i < nb; i++) ax.b_free.push_back(i); }
    else { for (int i = 0; i < nb - ncon; i++) ax.b_free.push_back(i); for (int i = nb - ncon; i < nb; i++) ax.b_con.push_back(i); }
    for (int i = 0; i < nbat; i++) { ax.a_bat.push_back(na + i); ax.b_bat.push_back(nb + i); }
    const int nfa = (int)ax.a_free.size(), nfb = (int)ax.b_free.size();
    if (C->ndim != nfa + nfb + nbat) return fail(ctx, NNT_EINVAL, "nnt_gemm: C has the wrong number of axes");
    for (int i = 0; i < ncon; i++)
        if (A->shape[ax.a_con[i]] != B->shape[ax.b_con[i]] || A->base[ax.a_con[i]] != B->base[ax.b_con[i]])
            return fail(ctx, NNT_EINVAL, "nnt_gemm: contracted axes differ in extent or tiling");
    for (int i = 0; i < nfa; i++)
        if (A->shape[ax.a_free[i]] != C->shape[i] || A->base[ax.a_free[i]] != C->base[i])
            return fail(ctx, NNT_EINVAL, "nnt_gemm: free axes of A and C differ in extent or tiling");
    for (int i = 0; i < nfb; i++)
        if (B->shape[ax.b_free[i]] != C->shape[nfa + i] || B->base[ax.b_free[i]] != C->base[nfa + i])
            return fail(ctx, NNT_EINVAL, "nnt_gemm: free axes of B and C differ in extent or tiling");
    for (int i = 0; i < nbat; i++) {
        const int ca = nfa + nfb + i;
        if (A->shape[ax.a_bat[i]] != C->shape[ca] || A->base[ax.a_bat[i]] != C->base[ca] ||
            B->shape[ax.b_bat[i]] != C->shape[ca] || B->base[ax.b_bat[i]] != C->base[ca])
            return fail(ctx, NNT_EINVAL, "nnt_gemm: batch axes differ in extent or tiling");
    }
    if (A->dtype != B->dtype) return fail(ctx, NNT_EDTYPE, "nnt_gemm: A and B must have one element type");
    if (A->dtype == NNT_F32 && C->dtype != NNT_F32) return fail(ctx, NNT_EDTYPE, "nnt_gemm: fp32 operands need an fp32 result");
    if (bias) {
        if (bias->dtype != NNT_F32 || bias->ndim != 1 || nfa != 1 || bias->shape[0] != C->shape[0] || bias->base[0] != C->base[0])
            return fail(ctx, NNT_EINVAL, "nnt_gemm: bias must be an fp32 vector tiled like C's first axis");
    }

    P->ctx = ctx;
    P->ids[0] = A->id; P->ids[1] = B->id; P->ids[2] = C->id; P->ids[3] = bias ? bias->id : 0; P->ids[4] = R ? R->id : 0;
    P->dtype_in = A->dtype;
    P->dtype_out = C->dtype;
    P->akf = opA == NNT_OP_T;
    P->bkf = opB == NNT_OP_N;
    const int elem = A->dtype == NNT_BF16 ? 2 : 4;

    // contracted tile grid
    int64_t ncon_tiles = 1;
    for (int i = 0; i < ncon; i++) ncon_tiles *= A->grid[ax.a_con[i]];
    int64_t m_max = 0, n_max = 0, big = 0;

    struct TaskGeom { int64_t m, n, batch; };
    std::vector<TaskGeom> geom;
    for (int64_t ci = 0; ci < C->ntiles; ci++) {
        if (!C->tiles[ci]) continue;
        int64_t cc[kMaxDim], ac[kMaxDim] = {0, 0, 0, 0}, bc[kMaxDim] = {0, 0, 0, 0};
        C->tile_coords(ci, cc);
        for (int i = 0; i < nfa; i++) ac[ax.a_free[i]] = cc[i];
        for (int i = 0; i < nfb; i++) bc[ax.b_free[i]] = cc[nfa + i];
        for (int i = 0; i < nbat; i++) { ac[ax.a_bat[i]] = cc[nfa + nfb + i]; bc[ax.b_bat[i]] = cc[nfa + nfb + i]; }
        const int64_t m = prod_extent(A, ac, ax.a_free), n = prod_extent(B, bc, ax.b_free);
        const int64_t batch = prod_extent(A, ac, ax.a_bat);
        if (m > INT32_MAX || n > INT32_MAX) return fail(ctx, NNT_EINVAL, "nnt_gemm: tile too large");
        GemmTask t = {};
        t.C = C->tiles[ci];
        t.bias = bias ? static_cast<const float*>(bias->tiles[cc[0]]) : nullptr;
        if (bias && !t.bias) return fail(ctx, NNT_EINVAL, "nnt_gemm: bias tile missing");
        if (R) {
            // the beta term of this tile comes from the residual input's tile: same geometry, so one offset does
            const ptrdiff_t delta = static_cast<const char*>(R->tiles[ci]) - static_cast<const char*>(C->tiles[ci]);
            if (delta % (ptrdiff_t)C->elem_size() != 0) return fail(ctx, NNT_EINVAL, "nnt_gemm_res: residual tile not aligned to the element size");
            t.cin_off = delta / (ptrdiff_t)C->elem_size();
            t.epi = epi;
        }
        t.ldc = (pairs && view_ld[2]) ? view_ld[2] : m;
        t.strideC = t.ldc * n;
        int64_t nb1 = 0;
        if (pairs) {
            nb1 = C->tile_extent(nfa + nfb, cc[nfa + nfb]);         // batch members of the tile; the heads follow
            t.nb1 = (int32_t)nb1;
            t.strideC2 = view_ld[2] ? m : t.strideC * nb1;           // a window keeps head hl at rows hl * h .. of its tile
        }
        t.m = (int32_t)m;
        t.n = (int32_t)n;
        t.chunk0 = (int32_t)P->chunks.size();
        std::vector<int64_t> atl, btl;
        for (int64_t l = 0; l < ncon_tiles; l++) {
            int64_t rem = l;
            for (int i = 0; i < ncon; i++) {
                const int64_t gi = A->grid[ax.a_con[i]];
                ac[ax.a_con[i]] = rem % gi;
                bc[ax.b_con[i]] = rem % gi;
                rem /= gi;
            }
            const int64_t ai = A->tile_index(ac), bi = B->tile_index(bc);
            if (!A->tiles[ai] || !B->tiles[bi]) continue;      // structural zeros: no contribution
            const int64_t k = prod_extent(A, ac, ax.a_con);
            GemmChunk ch = {};
            ch.A = A->tiles[ai];
            ch.B = B->tiles[bi];
            ch.lda = (pairs && view_ld[0]) ? view_ld[0] : (P->akf ? k : m);
            ch.ldb = (pairs && view_ld[1]) ? view_ld[1] : (P->bkf ? k : n);
            ch.strideA = ch.lda * (P->akf ? m : k);
            ch.strideB = ch.ldb * (P->bkf ? n : k);
            ch.k = (int32_t)k;
            if (pairs) {
                // the first axis of a window is the head size: m of A (k when A is read transposed), k of B (n when transposed)
                ch.strideA2 = view_ld[0] ? (P->akf ? k : m) : ch.strideA * nb1;
                ch.strideB2 = view_ld[1] ? (P->bkf ? k : n) : ch.strideB * nb1;
            }
            ch.vec_ok = (vec_flag(ch.A, ch.lda, ch.strideA, elem) && ch.strideA2 % (16 / elem) == 0 ? 1 : 0) |
                        (vec_flag(ch.B, ch.ldb, ch.strideB, elem) && ch.strideB2 % (16 / elem) == 0 ? 2 : 0);
            P->chunks.push_back(ch);
            atl.push_back(ai);
            btl.push_back(bi);
        }
        t.nchunk = (int32_t)P->chunks.size() - t.chunk0;
        for (int32_t q = t.chunk0; q < t.chunk0 + t.nchunk; q++) P->flops += 2.0 * m * n * P->chunks[q].k * batch;
        P->tasks.push_back(t);
        P->task_ctile.push_back(ci);
        P->task_atiles.push_back(atl);
        P->task_btiles.push_back(btl);
        P->task_bias_tile.push_back(bias ? cc[0] : -1);
        geom.push_back({m, n, batch});
        m_max = std::max(m_max, m);
        n_max = std::max(n_max, n);
        big += ((m + 255) / 256) * ((n + 255) / 256) * batch;
    }
    const bool bf = A->dtype == NNT_BF16;
    std::vector<int64_t> ktot(P->tasks.size(), 0);
    for (size_t ti = 0; ti < P->tasks.size(); ti++)
        for (int32_t q = P->tasks[ti].chunk0; q < P->tasks[ti].chunk0 + P->tasks[ti].nchunk; q++) ktot[ti] += P->chunks[q].k;
    int64_t k_max = 0;
    for (int64_t kq : ktot) k_max = std::max(k_max, kq);
    P->cfg = pick_cfg(bf, m_max, n_max, big, k_max, P->akf && P->bkf);
    int S = 1;
    int64_t n_split = 0;
    if (nbat == 0 && !P->tasks.empty() && (P->cfg == kCfgSquare || P->cfg == kCfgMid || P->cfg == kCfgTall)) {
        // products of whole matrices: macro-tile shape and k-slices by the cost model
        std::vector<int64_t> tm, tn;
        for (const TaskGeom& gq : geom) { tm.push_back(gq.m); tn.push_back(gq.n); }
        bool ragged = false;
        for (const TaskGeom& gq : geom) ragged = ragged || gq.m % 256 != 0 || gq.n % 256 != 0;
        for (const GemmChunk& c : P->chunks) ragged = ragged || c.k % 64 != 0;
        // (the activation forms keep the whole contraction in one workgroup: the slice sum does not know them)
        const ShapeChoice sc = choose_shape(bf, C->dtype == NNT_F32, P->akf, P->bkf, tm, tn, ktot, epi == 0, bf && ragged);
        P->cfg = sc.cfg;
        S = sc.s;
        n_split = sc.n_split;
    }
    int bm, bn;
    gemm_cfg_tile(bf, P->cfg, &bm, &bn);
    {
        // spelled like the demangled kernel name, so that profiler output can be matched against it
        static const char* const shape[9] = {"2, 2, 4, 4", "2, 2, 2, 2", "1, 4, 2, 2", "1, 4, 4, 2", "1, 4, 2, 1", "2, 2, 1, 1", "2, 2, 4, 2", "2, 2, 2, 2", "2, 2, 1, 2"};
        std::ostringstream l;
        const char* tf[2] = {"false", "true"};
        if (A->dtype == NNT_F32) l << "gemm_f32_kernel<" << tf[P->akf] << ", " << tf[P->bkf] << ", " << (P->cfg == kCfgSquare ? "2, 2, 2, 2" : P->cfg == kCfgMid ? "2, 2, 1, 2" : shape[P->cfg]) << ">";
        else l << "gemm_bf16_kernel<" << (C->dtype == NNT_F32 ? "float" : "unsigned short") << ", " << tf[P->akf] << ", " << tf[P->bkf]
               << ", " << shape[P->cfg] << ", 32>";
        if (nbat > 0) l << " batched";     // per-head attention products: short contractions, memory-leaning
        if (getenv("NNT_LABEL_SHAPES")) {  // one profile line per product shape instead of per kernel instance
            int64_t kmax = 0;
            for (int64_t kq : ktot) kmax = std::max(kmax, kq);
            int64_t rows = 1, cols = 1;
            for (int i = 0; i < nfa; i++) rows *= C->shape[i];
            for (int i = nfa; i < nfa + nfb; i++) cols *= C->shape[i];
            l << " [" << rows << " x " << cols << ", k/tile " << kmax << ", " << n_split << " macro-tiles in " << S << " slices]";
        }
        P->label = l.str();
    }
    // Workgroup order inside a task: m index fastest, so that workgroups in flight
    // together share a column panel of B.
    for (size_t ti = 0; ti < P->tasks.size(); ti++) {
        P->task_wg0.push_back((int64_t)P->wgs.size());
        const int64_t gm = (geom[ti].m + bm - 1) / bm, gn = (geom[ti].n + bn - 1) / bn;
        for (int64_t b = 0; b < geom[ti].batch; b++)
            for (int64_t j = 0; j < gn; j++)
                for (int64_t i = 0; i < gm; i++)
                    P->wgs.push_back(GemmWg{(int32_t)ti, (int32_t)(i * bm), (int32_t)(j * bn), (int32_t)b});
    }
    P->task_wg0.push_back((int64_t)P->wgs.size());
    if (P->wgs.size() > (size_t)INT32_MAX) return fail(ctx, NNT_EINVAL, "nnt_gemm: too many workgroups");
    // whole-operation launches use the XCD-aware order; per-task launches keep the order by task
    P->wgs_op = P->wgs;
    {
        // tasks of unequal length (causal attention: one to N_s / tile chunks): longest first, so that
        // the short ones fill the end of the launch instead of the long ones making its tail
        int64_t kmx = 0, kmn = INT64_MAX;
        for (int64_t kq : ktot) { kmx = std::max(kmx, kq); kmn = std::min(kmn, kq); }
        if (kmx > kmn)
            std::stable_sort(P->wgs_op.begin(), P->wgs_op.end(),
                             [&](const GemmWg& a, const GemmWg& b) { return ktot[a.task] > ktot[b.task]; });
    }
    xcd_interleave(P->wgs_op, bm, bn);

    // ---- k-slices for the last n_split macro-tiles of the whole-operation order
    // (a workspace above 2 GiB is not worth its memory: such a product runs without slices)
    if (S > 1 && (int64_t)std::min<int64_t>(n_split, (int64_t)P->wgs_op.size()) * S * bm * bn * (int64_t)sizeof(float) > ((int64_t)2 << 30)) {
        S = 1;
        n_split = 0;
    }
    P->splits = S;
    P->n_split = n_split = std::min<int64_t>(n_split, (int64_t)P->wgs_op.size());
    if (S > 1 && n_split > 0) {
        const size_t keep = P->wgs_op.size() - (size_t)n_split;
        const std::vector<GemmWg> cut(P->wgs_op.begin() + keep, P->wgs_op.end());
        P->wgs_op.resize(keep);
        const int64_t slice = (int64_t)bm * bn;
        NNT_HIP(ctx, hipMalloc((void**)&P->d_ws, (size_t)n_split * S * slice * sizeof(float)));
        P->ws_bytes += (int64_t)n_split * S * slice * (int64_t)sizeof(float);
        // chunk ranges of the slices, built once per C tile
        std::vector<std::vector<std::pair<int32_t, int32_t>>> ranges(P->tasks.size());
        std::vector<SplitReduce> red;
        std::vector<std::vector<GemmWg>> by_slice(S);
        for (size_t w = 0; w < cut.size(); w++) {
            const GemmWg& mw = cut[w];
            const GemmTask t0 = P->tasks[mw.task];
            if (ranges[mw.task].empty()) ranges[mw.task] = cut_into_slices(P, t0, ktot[mw.task], S, elem);
            red.push_back(add_slice_tasks(P, t0, mw, ranges[mw.task], P->d_ws + (int64_t)w * S * slice, bm, bn, by_slice));
        }
        // Launch order of the slices: workgroup p runs on XCD p mod 8, and the workgroups of one k-slice read
        // one k-range of both operands, so each slice is dealt to one XCD (slice s to XCD s mod 8): that XCD's
        // L2 then fetches the range once for all macro-tiles.  An XCD whose queue runs dry takes from the
        // longest one.
        {
            std::vector<GemmWg> q[8];
            for (int sidx = 0; sidx < S; sidx++) q[sidx & 7].insert(q[sidx & 7].end(), by_slice[sidx].begin(), by_slice[sidx].end());
            size_t head[8] = {0, 0, 0, 0, 0, 0, 0, 0}, left = 0;
            for (int x = 0; x < 8; x++) left += q[x].size();
            while (left > 0) {
                const int x = (int)(P->wgs_op.size() & 7);
                if (head[x] < q[x].size()) {
                    P->wgs_op.push_back(q[x][head[x]++]);
                } else {
                    int longest = 0;
                    for (int y = 1; y < 8; y++)
                        if (q[y].size() - head[y] > q[longest].size() - head[longest]) longest = y;
                    P->wgs_op.push_back(q[longest].back());
                    q[longest].pop_back();
                }
                left--;
            }
        }
        P->red_blocks = (int)((slice / 4 + 255) / 256);
        P->slice_elems = slice;
        NNT_HIP(ctx, hipMalloc((void**)&P->d_red, red.size() * sizeof(SplitReduce)));
        P->table_bytes += (int64_t)(red.size() * sizeof(SplitReduce));
        NNT_HIP(ctx, hipMemcpy(P->d_red, red.data(), red.size() * sizeof(SplitReduce), hipMemcpyHostToDevice));
    } else {
        P->splits = 1;
        P->n_split = 0;
    }
    P->op_nwg = (int64_t)P->wgs_op.size();

    // ---- k-slices per task for tile-granular launches
    const size_t n_tile_tasks = P->task_ctile.size();
    P->tile_split.assign(n_tile_tasks, GemmPlan::TileSplit{});
    std::vector<SplitReduce> red_ts;
    if (nbat == 0 && epi == 0 && ctx->granularity == NNT_GRAN_TILE) {      // (a plan first built for whole-operation launches has none)
        constexpr int64_t kTargetWgs = 64, kMinSlice = 512;
        constexpr int64_t kScratchCap = (int64_t)2 << 30;      // bytes of slice scratch per plan
        const int64_t slice = (int64_t)bm * bn;
        int64_t ws_blocks = 0;
        std::vector<int> st(n_tile_tasks, 1);
        for (int64_t max_slices = 8; max_slices >= 2; max_slices /= 2) {
            ws_blocks = 0;
            for (size_t ti = 0; ti < n_tile_tasks; ti++) {
                st[ti] = 1;
                const int64_t nwg = P->task_wg0[ti + 1] - P->task_wg0[ti];
                if (nwg == 0 || nwg >= kTargetWgs) continue;
                const int64_t want = std::min<int64_t>({max_slices, (kTargetWgs + nwg - 1) / nwg, ktot[ti] / kMinSlice});
                if (want < 2) continue;
                st[ti] = (int)want;
                ws_blocks += nwg * want;
            }
            if (ws_blocks * slice * (int64_t)sizeof(float) <= kScratchCap) break;
            ws_blocks = 0;
            std::fill(st.begin(), st.end(), 1);
        }
        if (ws_blocks > 0) {
            NNT_HIP(ctx, hipMalloc((void**)&P->d_ws_ts, (size_t)ws_blocks * slice * sizeof(float)));
            P->ws_bytes += (int64_t)ws_blocks * slice * (int64_t)sizeof(float);
            float* next_block = P->d_ws_ts;
            for (size_t ti = 0; ti < n_tile_tasks; ti++) {
                const int St = st[ti];
                if (St < 2) continue;
                const GemmTask t0 = P->tasks[ti];
                const std::vector<std::pair<int32_t, int32_t>> ranges = cut_into_slices(P, t0, ktot[ti], St, elem);
                GemmPlan::TileSplit& ts = P->tile_split[ti];
                ts.wg0 = (int64_t)P->wgs_ts.size();
                ts.red0 = (int64_t)red_ts.size();
                std::vector<std::vector<GemmWg>> by_slice(St);
                for (int64_t w = P->task_wg0[ti]; w < P->task_wg0[ti + 1]; w++) {
                    red_ts.push_back(add_slice_tasks(P, t0, P->wgs[w], ranges, next_block, bm, bn, by_slice));
                    next_block += (int64_t)St * slice;
                }
                for (int sidx = 0; sidx < St; sidx++) P->wgs_ts.insert(P->wgs_ts.end(), by_slice[sidx].begin(), by_slice[sidx].end());
                ts.nwg = (int64_t)P->wgs_ts.size() - ts.wg0;
                ts.nred = (int64_t)red_ts.size() - ts.red0;
            }
            P->red_blocks = (int)((slice / 4 + 255) / 256);    // (the same value the whole-operation slices set)
            P->slice_elems_ts = slice;
            NNT_HIP(ctx, hipMalloc((void**)&P->d_red_ts, red_ts.size() * sizeof(SplitReduce)));
            P->table_bytes += (int64_t)(red_ts.size() * sizeof(SplitReduce));
            NNT_HIP(ctx, hipMemcpy(P->d_red_ts, red_ts.data(), red_ts.size() * sizeof(SplitReduce), hipMemcpyHostToDevice));
        }
    }

    // workgroups that qualify for the direct-load kernel go first in every launch range
    P->task_nfast.assign(P->task_ctile.size(), 0);
    if (bf ? (P->cfg == kCfgSquare || P->cfg == kCfgTall || P->cfg == kCfgWide) : (P->cfg == kCfgSquare || P->cfg == kCfgSkinny64n128 || P->cfg == kCfgMid || P->cfg == kCfgResident)) {
        const int kmul = (bf && P->cfg == kCfgSquare) ? 64 : 32;   // loads are started two k-steps at a time
        // the 256 x 128 bf16 kernel has a variant for chunk lengths that are multiples of 8 and macro-tiles that end
        // inside their C tile (at a multiple of 8 rows of an operand whose row index is the contiguous one)
        const bool rag_ok = bf && (P->cfg == kCfgTall || P->cfg == kCfgWide);
        std::vector<char> task_ok(P->tasks.size(), 1), task_rag(P->tasks.size(), 0);
        if (P->cfg == kCfgResident)      // the whole contraction, one chunk of at most 64, sits in LDS at once
            for (size_t ti = 0; ti < P->tasks.size(); ti++)
                if (P->tasks[ti].nchunk != 1 || P->chunks[P->tasks[ti].chunk0].k > 64) task_ok[ti] = 0;
        for (size_t ti = 0; ti < P->tasks.size(); ti++)
            for (int32_t q = P->tasks[ti].chunk0; q < P->tasks[ti].chunk0 + P->tasks[ti].nchunk; q++) {
                const GemmChunk& c = P->chunks[q];
                if (c.vec_ok != 3 || c.k <= 0 || c.k % (rag_ok ? 8 : kmul) != 0) task_ok[ti] = 0;
                else if (c.k % kmul != 0) task_rag[ti] = 1;
            }
        auto edge_ok = [&](const GemmWg& w) {
            const GemmTask& t = P->tasks[w.task];
            const int mv = std::min(bm, t.m - w.m0), nv = std::min(bn, t.n - w.n0);
            return rag_ok && (P->akf || mv % 8 == 0) && (P->bkf || nv % 8 == 0);
        };
        auto whole = [&](const GemmWg& w) {
            const GemmTask& t = P->tasks[w.task];
            return w.m0 + bm <= t.m && w.n0 + bn <= t.n;
        };
        auto qualifies = [&](const GemmWg& w) { return task_ok[w.task] && (whole(w) || edge_ok(w)); };
        for (const std::vector<GemmWg>* list : {&P->wgs, &P->wgs_op, &P->wgs_ts})
            for (const GemmWg& w : *list)
                if (qualifies(w) && (task_rag[w.task] || !whole(w))) P->dl_ragged = true;
        P->op_nfast = std::stable_partition(P->wgs_op.begin(), P->wgs_op.end(), qualifies) - P->wgs_op.begin();
        for (size_t ti = 0; ti + 1 < P->task_wg0.size(); ti++)
            P->task_nfast[ti] = std::stable_partition(P->wgs.begin() + P->task_wg0[ti], P->wgs.begin() + P->task_wg0[ti + 1], qualifies) -
                                (P->wgs.begin() + P->task_wg0[ti]);
        for (GemmPlan::TileSplit& ts : P->tile_split)
            if (ts.nwg > 0)
                ts.nfast = std::stable_partition(P->wgs_ts.begin() + ts.wg0, P->wgs_ts.begin() + ts.wg0 + ts.nwg, qualifies) -
                           (P->wgs_ts.begin() + ts.wg0);
        if (2 * P->op_nfast >= P->op_nwg && P->op_nwg > 0) {
            // most of the work runs in the direct-load kernel: profile lines carry its name
            const std::string old_name = P->label.substr(0, P->label.find('>') + 1);
            const char* tf[2] = {"false", "true"};
            std::ostringstream l;
            if (bf)
                l << (P->cfg == kCfgTall ? "gemm_bf16_dl_tall_kernel<" : P->cfg == kCfgWide ? "gemm_bf16_dl_wide_kernel<" : "gemm_bf16_dl_kernel<")
                  << (C->dtype == NNT_F32 ? "float" : "unsigned short")
                  << ", " << tf[P->akf] << ", " << tf[P->bkf] << (P->cfg == kCfgTall ? (P->dl_ragged ? ", true>" : ", false>") : ">");
            else if (P->cfg == kCfgResident)
                l << "gemm_f32_dl_rk_kernel";
            else
                l << "gemm_f32_dl_kernel<" << tf[P->akf] << ", " << tf[P->bkf] << (P->cfg == kCfgSquare ? ", 2, 2>" : ", 1, 2>");
            P->label = l.str() + P->label.substr(old_name.size());
        }
    }

    if (epi) {
        P->epi_mode = epi & 15;
        bool all_fast = P->op_nwg > 0 && P->op_nfast == P->op_nwg && getenv("NNT_GEMM_NO_DL") == nullptr;
        for (size_t ti = 0; ti + 1 < P->task_wg0.size(); ti++) all_fast = all_fast && P->task_nfast[ti] == P->task_wg0[ti + 1] - P->task_wg0[ti];
        P->epi_ok = all_fast && !bf && gemm_f32_dl_has_act(P->akf, P->bkf, P->epi_mode);
        if (P->epi_ok) {
            const std::string old_name = P->label.substr(0, P->label.find('>') + 1);
            const char* tf[2] = {"false", "true"};
            std::ostringstream l;
            l << "gemm_f32_dl_act_kernel<" << tf[P->akf] << (P->cfg == kCfgSquare ? ", 2, 2, " : ", 1, 2, ") << P->epi_mode << ">";
            P->label = l.str() + P->label.substr(old_name.size());
        }
    }

    auto up = [&](void** d, const void* h, size_t bytes) -> hipError_t {
        if (bytes == 0) return hipSuccess;
        hipError_t e = hipMalloc(d, bytes);
        if (e != hipSuccess) return e;
        P->table_bytes += (int64_t)bytes;
        return hipMemcpy(*d, h, bytes, hipMemcpyHostToDevice);
    };
    NNT_HIP(ctx, up((void**)&P->d_tasks, P->tasks.data(), P->tasks.size() * sizeof(GemmTask)));
    NNT_HIP(ctx, up((void**)&P->d_chunks, P->chunks.data(), P->chunks.size() * sizeof(GemmChunk)));
    NNT_HIP(ctx, up((void**)&P->d_wgs, P->wgs.data(), P->wgs.size() * sizeof(GemmWg)));
    NNT_HIP(ctx, up((void**)&P->d_wgs_op, P->wgs_op.data(), P->wgs_op.size() * sizeof(GemmWg)));
    NNT_HIP(ctx, up((void**)&P->d_wgs_ts, P->wgs_ts.data(), P->wgs_ts.size() * sizeof(GemmWg)));
    return NNT_OK;
}

}  // namespace

extern "C" int32_t nnt_gemm(nnt_ctx* ctx, float alpha, int32_t opA, nnt_tensor* A, int32_t opB, nnt_tensor* B,
                            float beta, nnt_tensor* C, int32_t ncon, int32_t nbat, nnt_tensor* bias) {
    return nnt_gemm_res(ctx, alpha, opA, A, opB, B, beta, C, ncon, nbat, bias, nullptr);
}

namespace {

// what gemm_core answers when the plan of a product with an activation form has workgroups that no kernel with that
// form takes (never leaves the library: the callers then run the product and the activation as two passes)
constexpr int32_t kNoActKernel = 1 << 20;

// The product proper.  A, B, C give the geometry (ordinary tensors, or the windows of nnt_gemm_heads: then `view_ld`
// and `key_extra` are set); `dep` are the tensors whose tiles order the tasks (the operands themselves, or what
// the windows look at).
int32_t gemm_core(nnt_ctx* ctx, float alpha, int32_t opA, nnt_tensor* A, int32_t opB, nnt_tensor* B, float beta, nnt_tensor* C,
                  int32_t ncon, int32_t nbat, nnt_tensor* bias, nnt_tensor* R, nnt_tensor* const* dep, const int64_t* view_ld,
                  const std::string& key_extra, int32_t part_c = 0, int epi = 0) {
    std::ostringstream key;
    key << opA << opB << ':' << A->id << ':' << B->id << ':' << C->id << ':' << (bias ? bias->id : 0) << ':' << ncon << ':' << nbat
        << ':' << (R ? R->id : 0) << key_extra;
    GemmPlan* P;
    auto it = ctx->gemm_plans.find(key.str());
    if (it == ctx->gemm_plans.end()) {
        if (ctx->capturing) return fail(ctx, NNT_ESTATE, "nnt_gemm: plan must exist before capture (run the call once first)");
        std::shared_ptr<GemmPlan> np(new GemmPlan());
        int32_t rc = build_plan(ctx, opA, A, opB, B, C, ncon, nbat, bias, R, np.get(), view_ld, epi);
        if (rc != NNT_OK) return rc;
        P = np.get();
        ctx->gemm_plans[key.str()] = np;
    } else {
        P = it->second.get();
    }
    if (epi && !P->epi_ok) return kNoActKernel;
    const int epi_mode = P->epi_mode;
    nnt_tensor* const dA = dep[0];
    nnt_tensor* const dB = dep[1];
    nnt_tensor* const dC = dep[2];
    OpTag tag(ctx, P->label.c_str(), P->flops, false);
    GemmArgs g = {};
    g.tasks = P->d_tasks;
    g.chunks = P->d_chunks;
    g.alpha = alpha;
    g.beta = beta;
    const int cmode = beta != 0.f ? kReadWrite : kWrite;
    if (ctx->granularity == NNT_GRAN_OP || view_ld) {
        // (a window writes the rows of its part in every tile it touches and leaves the others)
        std::vector<Access> acc = {dA->all(kRead), dB->all(kRead), dC->all((view_ld && view_ld[2]) ? kWritePart : (R ? kWrite : cmode))};
        acc[2].part = part_c;
        if (bias) acc.push_back(bias->all(kRead));
        if (R && (beta != 0.f || epi)) acc.push_back(R->all((epi & 15) == kEpiGeluOut ? kWrite : kRead));
        g.wgs = P->d_wgs_op;
        const int64_t nwg = P->op_nwg;
        if (nwg == 0) return NNT_OK;
        if (P->n_split > 0) {
            acc.push_back(Access{&P->ws_dep, 1, kReadWrite});
            const double red_bytes = (double)P->n_split * P->slice_elems * 4.0 * (P->splits + 1);
            return submit(ctx, acc, [=](hipStream_t st) {
                int32_t rc = launch_any(st, P->dtype_in, P->dtype_out, P->akf, P->bkf, P->cfg, g, nwg, P->op_nfast, P->dl_ragged);
                if (rc != NNT_OK) return rc;
                profile_mark(ctx, st, "splitk_reduce", red_bytes, true);
                const dim3 grid((unsigned)P->red_blocks, (unsigned)P->n_split), block(256);
                if (P->dtype_out == NNT_F32) hipLaunchKernelGGL((splitk_reduce<float>), grid, block, 0, st, P->d_red, alpha, beta);
                else hipLaunchKernelGGL((splitk_reduce<uint16_t>), grid, block, 0, st, P->d_red, alpha, beta);
                return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
            }, 2);
        }
        return submit(ctx, acc, [=](hipStream_t st) {
            return launch_any(st, P->dtype_in, P->dtype_out, P->akf, P->bkf, P->cfg, g, nwg, P->op_nfast, P->dl_ragged, epi_mode);
        });
    }
    const size_t n_tile_tasks = P->task_ctile.size();
    for (size_t ti = 0; ti < n_tile_tasks; ti++) {
        std::vector<Access> acc;
        acc.push_back(C->one(P->task_ctile[ti], R ? kWrite : cmode));
        if (R && (beta != 0.f || epi)) acc.push_back(R->one(P->task_ctile[ti], (epi & 15) == kEpiGeluOut ? kWrite : kRead));
        for (int64_t a : P->task_atiles[ti]) acc.push_back(A->one(a, kRead));
        for (int64_t b : P->task_btiles[ti]) acc.push_back(B->one(b, kRead));
        if (bias) acc.push_back(bias->one(P->task_bias_tile[ti], kRead));
        GemmArgs gt = g;
        const GemmPlan::TileSplit ts = P->tile_split[ti];
        int32_t rc;
        if (ts.nwg > 0) {
            // few macro-tiles, long contraction: k-slices into this task's scratch block, then their sum
            gt.wgs = P->d_wgs_ts + ts.wg0;
            const double red_bytes = (double)ts.nred * P->slice_elems_ts * 4.0 * (ts.nwg / ts.nred + 1);
            rc = submit(ctx, acc, [=](hipStream_t st) {
                int32_t r = launch_any(st, P->dtype_in, P->dtype_out, P->akf, P->bkf, P->cfg, gt, ts.nwg, ts.nfast, P->dl_ragged);
                if (r != NNT_OK) return r;
                profile_mark(ctx, st, "splitk_reduce", red_bytes, true);
                const dim3 grid((unsigned)P->red_blocks, (unsigned)ts.nred), block(256);
                if (P->dtype_out == NNT_F32) hipLaunchKernelGGL((splitk_reduce<float>), grid, block, 0, st, P->d_red_ts + ts.red0, alpha, beta);
                else hipLaunchKernelGGL((splitk_reduce<uint16_t>), grid, block, 0, st, P->d_red_ts + ts.red0, alpha, beta);
                return hipGetLastError() == hipSuccess ? (int32_t)NNT_OK : (int32_t)NNT_EHIP;
            }, 2);
        } else {
            gt.wgs = P->d_wgs + P->task_wg0[ti];
            const int64_t nwg = P->task_wg0[ti + 1] - P->task_wg0[ti];
            const int64_t nfast = P->task_nfast[ti];
            rc = submit(ctx, acc, [=](hipStream_t st) {
                return launch_any(st, P->dtype_in, P->dtype_out, P->akf, P->bkf, P->cfg, gt, nwg, nfast, P->dl_ragged, epi_mode);
            });
        }

        if (rc != NNT_OK) return rc;
    }
    return NNT_OK;
}

// A window on `T` ([n_parts * N_h * h, N_s, N_b], the heads side by side along the first axis): rows
// [part * N_h * h, (part + 1) * N_h * h) seen as [h, N_s, N_b, N_h].  Its tiles are T's own (one per group of
// base[0] / h heads), addressed with T's leading dimension; nothing is copied.  Parts and groups of heads must
// coincide with T's row tiles.
int32_t make_window(nnt_ctx* ctx, nnt_tensor* T, int32_t part, int64_t h, int64_t N_h, nnt_tensor* W, int64_t* ld) {
    const int64_t N_e = h * N_h, t0 = T->base[0];
    if (T->ndim != 3 || part < 0 || T->shape[0] % N_e != 0 || (int64_t)(part + 1) * N_e > T->shape[0])
        return fail(ctx, NNT_EINVAL, "nnt_gemm_heads: a window needs a 3-axis tensor of whole parts of N_h * h rows and a part inside it");
    if (t0 % h != 0 || N_e % t0 != 0)
        return fail(ctx, NNT_EINVAL, "nnt_gemm_heads: row tiles must hold whole heads and a part whole row tiles");
    const int64_t hp = t0 / h;
    W->ctx = ctx;
    W->dtype = T->dtype;
    W->ndim = 4;
    const int64_t shape[4] = {h, T->shape[1], T->shape[2], N_h}, base[4] = {h, T->base[1], T->base[2], hp};
    W->ntiles = 1;
    for (int a = 0; a < 4; a++) {
        W->shape[a] = shape[a];
        W->base[a] = base[a];
        W->grid[a] = (shape[a] + base[a] - 1) / base[a];
        W->ntiles *= W->grid[a];
    }
    W->tiles.assign((size_t)W->ntiles, nullptr);
    W->d_tiles = nullptr;
    W->id = T->id;
    for (int64_t i = 0; i < W->ntiles; i++) {
        int64_t wc[kMaxDim], tc[kMaxDim] = {0, 0, 0, 0};
        W->tile_coords(i, wc);
        tc[0] = (int64_t)part * (N_e / t0) + wc[3];
        tc[1] = wc[1];
        tc[2] = wc[2];
        W->tiles[(size_t)i] = T->tiles[(size_t)T->tile_index(tc)];
        if (!W->tiles[(size_t)i]) return fail(ctx, NNT_EINVAL, "nnt_gemm_heads: a tensor with the heads side by side must hold all its tiles");
    }
    *ld = t0;
    return NNT_OK;
}

// An ordinary tensor [., ., N_b, N_h] seen with `hp` heads per tile along its last axis (what the windows on the
// other operands have): a tile of the coarser tiling is cut along its slowest axis, so the pieces are contiguous
// and keep its strides.  Absent tiles stay absent.
int32_t make_retiled(nnt_ctx* ctx, nnt_tensor* T, int64_t hp, nnt_tensor* W) {
    if (T->ndim != 4 || T->base[3] % hp != 0)
        return fail(ctx, NNT_EINVAL, "nnt_gemm_heads: the head axis of an ordinary operand must be tiled in multiples of the heads per row tile");
    *W = *T;                           // geometry, type, id
    W->deps.clear();
    W->d_tiles = nullptr;
    W->base[3] = hp;
    W->grid[3] = (T->shape[3] + hp - 1) / hp;
    W->ntiles = W->grid[0] * W->grid[1] * W->grid[2] * W->grid[3];
    W->tiles.assign((size_t)W->ntiles, nullptr);
    for (int64_t i = 0; i < W->ntiles; i++) {
        int64_t wc[kMaxDim], tc[kMaxDim];
        W->tile_coords(i, wc);
        for (int a = 0; a < 3; a++) tc[a] = wc[a];
        tc[3] = wc[3] * hp / T->base[3];
        char* basep = static_cast<char*>(T->tiles[(size_t)T->tile_index(tc)]);
        if (!basep) continue;
        const int64_t first = wc[3] * hp - tc[3] * T->base[3];           // heads of the coarse tile before this piece
        const int64_t per_head = T->tile_extent(0, tc[0]) * T->tile_extent(1, tc[1]) * T->tile_extent(2, tc[2]);
        W->tiles[(size_t)i] = basep + first * per_head * T->elem_size();
    }
    return NNT_OK;
}

}  // namespace

extern "C" int32_t nnt_gemm_res(nnt_ctx* ctx, float alpha, int32_t opA, nnt_tensor* A, int32_t opB, nnt_tensor* B,
                                float beta, nnt_tensor* C, int32_t ncon, int32_t nbat, nnt_tensor* bias, nnt_tensor* R) {
    NNT_CHECK_CTX(ctx);
    if (!A || !B || !C) return fail(ctx, NNT_EINVAL, "nnt_gemm: null tensor");
    if ((opA != NNT_OP_N && opA != NNT_OP_T) || (opB != NNT_OP_N && opB != NNT_OP_T))
        return fail(ctx, NNT_EINVAL, "nnt_gemm: bad op");
    if (R == C) R = nullptr;
    if (R) {
        if (R->dtype != C->dtype || !same_tiling(R, C)) return fail(ctx, NNT_EINVAL, "nnt_gemm_res: the residual input must have C's type, shape and tiling");
        for (int64_t t = 0; t < C->ntiles; t++)
            if (C->tiles[t] && !R->tiles[t]) return fail(ctx, NNT_EINVAL, "nnt_gemm_res: the residual input lacks a tile that C has");
        if (R == A || R == B) return fail(ctx, NNT_EINVAL, "nnt_gemm_res: the residual input must not be an operand");
    }
    nnt_tensor* const dep[3] = {A, B, C};
    return gemm_core(ctx, alpha, opA, A, opB, B, beta, C, ncon, nbat, bias, R, dep, nullptr, std::string());
}

namespace {

int32_t gemm_gelu(nnt_ctx* ctx, const char* who, int mode, float alpha, int32_t opA, nnt_tensor* A, int32_t opB, nnt_tensor* B, nnt_tensor* C,
                  int32_t ncon, nnt_tensor* bias, int32_t variant, nnt_tensor* X) {
    NNT_CHECK_CTX(ctx);
    if (!A || !B || !C || !X) return fail(ctx, NNT_EINVAL, std::string(who) + ": null tensor");
    if ((opA != NNT_OP_N && opA != NNT_OP_T) || (opB != NNT_OP_N && opB != NNT_OP_T) || (variant != NNT_GELU_TANH && variant != NNT_GELU_ERF))
        return fail(ctx, NNT_EINVAL, std::string(who) + ": bad op or GELU variant");
    if (X == C || X == A || X == B || X->dtype != C->dtype || !same_tiling(X, C))
        return fail(ctx, NNT_EINVAL, std::string(who) + ": the second tensor must be distinct from A, B and C and have C's type, shape and tiling");
    for (int64_t t = 0; t < C->ntiles; t++)
        if (C->tiles[t] && !X->tiles[t]) return fail(ctx, NNT_EINVAL, std::string(who) + ": the second tensor lacks a tile that C has");
    nnt_tensor* const dep[3] = {A, B, C};
    std::ostringstream extra;
    extra << ":gelu" << mode << variant;
    if (A->dtype == NNT_F32 && gemm_f32_dl_has_act(opA == NNT_OP_T, opB == NNT_OP_N, mode)) {
        const int32_t rc = gemm_core(ctx, alpha, opA, A, opB, B, 0.f, C, ncon, 0, bias, X, dep, nullptr, extra.str(), 0, mode | (variant << 4));
        if (rc != kNoActKernel) return rc;
    }
    // bf16, or ragged macro-tiles, operand forms or alignments that only the general kernels take: product, then activation
    int32_t r2 = gemm_core(ctx, alpha, opA, A, opB, B, 0.f, C, ncon, 0, bias, nullptr, dep, nullptr, std::string());
    if (r2 != NNT_OK) return r2;
    return mode == kEpiGeluOut ? nnt_gelu(ctx, variant, C, X) : nnt_gelu_bwd(ctx, variant, X, C, C);
}

}  // namespace

extern "C" int32_t nnt_gemm_gelu(nnt_ctx* ctx, float alpha, int32_t opA, nnt_tensor* A, int32_t opB, nnt_tensor* B, nnt_tensor* C,
                                 int32_t ncon, nnt_tensor* bias, int32_t variant, nnt_tensor* G) {
    return gemm_gelu(ctx, "nnt_gemm_gelu", kEpiGeluOut, alpha, opA, A, opB, B, C, ncon, bias, variant, G);
}

extern "C" int32_t nnt_gemm_gelu_bwd(nnt_ctx* ctx, float alpha, int32_t opA, nnt_tensor* A, int32_t opB, nnt_tensor* B, nnt_tensor* C,
                                     int32_t ncon, int32_t variant, nnt_tensor* X) {
    return gemm_gelu(ctx, "nnt_gemm_gelu_bwd", kEpiGeluGradMul, alpha, opA, A, opB, B, C, ncon, nullptr, variant, X);
}

extern "C" int32_t nnt_gemm_heads(nnt_ctx* ctx, float alpha, int32_t opA, nnt_tensor* A, int32_t partA, int32_t opB, nnt_tensor* B,
                                  int32_t partB, nnt_tensor* C, int32_t partC, int32_t h, int32_t N_h) {
    NNT_CHECK_CTX(ctx);
    if (!A || !B || !C) return fail(ctx, NNT_EINVAL, "nnt_gemm_heads: null tensor");
    if ((opA != NNT_OP_N && opA != NNT_OP_T) || (opB != NNT_OP_N && opB != NNT_OP_T) || h < 1 || N_h < 1)
        return fail(ctx, NNT_EINVAL, "nnt_gemm_heads: bad argument");
    nnt_tensor win[3];
    nnt_tensor* geo[3] = {A, B, C};
    nnt_tensor* const dep[3] = {A, B, C};
    const int32_t part[3] = {partA, partB, partC};
    int64_t view_ld[3] = {0, 0, 0};
    std::ostringstream extra;
    extra << ":heads" << h << 'x' << N_h;
    int64_t hp = 0;
    for (int i = 0; i < 3; i++) {
        extra << ':' << part[i];
        if (part[i] < 0) continue;
        int32_t rc = make_window(ctx, dep[i], part[i], h, N_h, &win[i], &view_ld[i]);
        if (rc != NNT_OK) return rc;
        geo[i] = &win[i];
        if (hp && hp != win[i].base[3]) return fail(ctx, NNT_EINVAL, "nnt_gemm_heads: the tensors with parts must have one row tiling");
        hp = win[i].base[3];
    }
    if (!hp) return fail(ctx, NNT_EINVAL, "nnt_gemm_heads: no operand has a part (use nnt_gemm)");
    for (int i = 0; i < 3; i++) {
        if (part[i] >= 0) continue;
        if (dep[i]->ndim != 4 || dep[i]->shape[3] != N_h)
            return fail(ctx, NNT_EINVAL, "nnt_gemm_heads: tensors without a part must have the axes [., ., N_b, N_h]");
        if (dep[i]->base[3] == hp) continue;
        int32_t rc = make_retiled(ctx, dep[i], hp, &win[i]);
        if (rc != NNT_OK) return rc;
        geo[i] = &win[i];
    }
    return gemm_core(ctx, alpha, opA, geo[0], opB, geo[1], 0.f, geo[2], 1, 2, nullptr, nullptr, dep, view_ld, extra.str(), partC > 0 ? partC : 0);
}
