// Internal declarations shared by the translation units of libnntile_mi.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <functional>
#include <map>
#include <memory>
#include <string>
#include <unordered_set>
#include <vector>

#include "nntile_mi.h"

namespace nnt {

constexpr int kMaxStreams = 8;
constexpr int kMaxDim = NNT_MAX_DIM;

// ---------------------------------------------------------------- device-side views
// A tiled tensor as kernels see it: extents, base tile, grid and the table of
// tile pointers (device memory, grid order, first axis fastest).
struct TiledView {
    void* const* tiles;
    int32_t ndim;
    int32_t shape[kMaxDim];
    int32_t base[kMaxDim];
    int32_t grid[kMaxDim];
};

// ---------------------------------------------------------------- dependency tracking
// What the executor remembers per tile: who wrote it last and who has read it
// since (one sequence number per stream is enough: streams run in order).
struct TileDep {
    int32_t w_stream = -1;
    uint64_t w_seq = 0;
    uint64_t r_seq[kMaxStreams] = {0, 0, 0, 0, 0, 0, 0, 0};
    // writers of parts of the tile (kWritePart) since the last writer of all of it: per stream the last one's
    // sequence number and part, and whether that stream has had writers of different parts
    uint64_t p_seq[kMaxStreams] = {0, 0, 0, 0, 0, 0, 0, 0};
    int32_t p_part[kMaxStreams] = {0, 0, 0, 0, 0, 0, 0, 0};
    uint8_t p_mixed[kMaxStreams] = {0, 0, 0, 0, 0, 0, 0, 0};
};

// kWritePart: the task writes the part `Access::part` of every tile it names and leaves the rest of the tile as
// it is (the attention products that write the rows of Q, K or V inside one tensor).  Writers of different parts
// are not ordered among themselves; towards everything else each of them is a writer.
enum AccessMode { kRead = 1, kWrite = 2, kReadWrite = 3, kWritePart = 6 };

struct Access {
    TileDep* first;
    int64_t count;
    int mode;
    int32_t part = 0;
};

struct GemmPlan;

}  // namespace nnt

struct nnt_tensor {
    nnt_ctx* ctx;
    int32_t dtype;
    int32_t ndim;
    int64_t shape[nnt::kMaxDim];
    int64_t base[nnt::kMaxDim];
    int64_t grid[nnt::kMaxDim];
    int64_t ntiles;
    std::vector<void*> tiles;        // host copy of the tile pointers
    void** d_tiles;                  // device copy
    std::vector<nnt::TileDep> deps;  // one per tile
    uint64_t id;

    int64_t elem_size() const { return dtype == NNT_F32 ? 4 : 2; }
    void tile_coords(int64_t idx, int64_t* c) const {
        for (int a = 0; a < ndim; a++) { c[a] = idx % grid[a]; idx /= grid[a]; }
    }
    int64_t tile_index(const int64_t* c) const {
        int64_t idx = 0;
        for (int a = ndim - 1; a >= 0; a--) idx = idx * grid[a] + c[a];
        return idx;
    }
    int64_t tile_extent(int a, int64_t c) const {
        int64_t lo = c * base[a];
        int64_t hi = lo + base[a];
        return (hi > shape[a] ? shape[a] : hi) - lo;
    }
    int64_t tile_numel(int64_t idx) const {
        int64_t c[nnt::kMaxDim];
        tile_coords(idx, c);
        int64_t n = 1;
        for (int a = 0; a < ndim; a++) n *= tile_extent(a, c[a]);
        return n;
    }
    nnt::TiledView view() const {
        nnt::TiledView v;
        v.tiles = d_tiles;
        v.ndim = ndim;
        for (int a = 0; a < nnt::kMaxDim; a++) {
            v.shape[a] = a < ndim ? (int32_t)shape[a] : 1;
            v.base[a] = a < ndim ? (int32_t)base[a] : 1;
            v.grid[a] = a < ndim ? (int32_t)grid[a] : 1;
        }
        return v;
    }
    nnt::Access all(int mode) { return nnt::Access{deps.data(), ntiles, mode}; }
    nnt::Access one(int64_t idx, int mode) { return nnt::Access{&deps[idx], 1, mode}; }
};

struct nnt_ctx {
    int device = 0;
    int n_streams = 1;
    bool own_streams = true;
    bool serial = false;
    int granularity = NNT_GRAN_OP;
    int status = NNT_OK;             // sticky
    std::string error;
    hipStream_t streams[nnt::kMaxStreams];
    uint64_t tail_seq[nnt::kMaxStreams];     // last sequence number issued per stream
    uint64_t synced_seq[nnt::kMaxStreams];   // everything up to here is known complete
    uint64_t waited[nnt::kMaxStreams][nnt::kMaxStreams];  // waited[s][d]: s already waits for d up to this seq
    std::vector<hipEvent_t> events[nnt::kMaxStreams];     // events recorded on stream s since the last sync ...
    std::vector<uint64_t> event_seq[nnt::kMaxStreams];    // ... and the sequence number each of them covers (ascending)
    // Which tasks get an event of their own: those whose result (identified by the first tile the task
    // writes) a task on another stream has waited for before.  A flow that repeats every step settles on
    // the few producers that are consumed across streams; everything else is covered on demand.
    std::unordered_set<const void*> hot_producers;
    std::vector<const void*> task_key[nnt::kMaxStreams];  // key of the task with sequence number synced_seq + 1 + i
    std::vector<hipEvent_t> event_pool;
    std::vector<hipEvent_t> capture_events;               // fork / join events of the open capture
    int rr = 0;                      // round-robin cursor
    bool capturing = false;
    nnt_exec_stats stats = {0, 0, 0, 0, 0, 0};
    int64_t table_bytes = 0;         // device bytes of tensor tile tables and optimiser group tables (plans count their own)
    uint64_t next_tensor_id = 1;
    std::map<std::string, std::shared_ptr<nnt::GemmPlan>> gemm_plans;
    int64_t live_tensors = 0;
    // fp32 scratch for two-stage reductions (bias gradient, layer-norm parameter
    // gradients); grows on demand, guarded by its own dependency record.
    float* red_scratch = nullptr;
    int64_t red_scratch_elems = 0;
    nnt::TileDep red_dep;
    // per-task timing (nnt_profile_*): what the operation being submitted is called and
    // how much algorithmic work it stands for; the first task of the operation carries it
    bool profiling = false;
    const char* cur_label = nullptr;
    double cur_work = 0.0;
    bool cur_work_is_bytes = false;
    struct ProfileRec { std::string label; hipEvent_t start, stop; double work; bool bytes; int launches; };
    std::vector<ProfileRec> profile;
    std::vector<hipEvent_t> timing_pool;
    ProfileRec* cur_prof = nullptr;   // record of the task whose launches are being issued, if timed
};

namespace nnt {
// Names the tensor-level operation whose tasks are submitted while it is alive.
struct OpTag {
    nnt_ctx* c;
    OpTag(nnt_ctx* ctx, const char* label, double work, bool bytes) : c(ctx) {
        c->cur_label = label;
        c->cur_work = work;
        c->cur_work_is_bytes = bytes;
    }
    ~OpTag() { c->cur_label = nullptr; c->cur_work = 0.0; }
};
}  // namespace nnt

namespace nnt {

int32_t fail(nnt_ctx* ctx, int32_t code, const std::string& msg);
// Inside a task's launch function, between two of its kernels: when tasks are being timed, what was
// launched so far is closed as one profile record and the rest of the task gets a record of its own.
void profile_mark(nnt_ctx* ctx, hipStream_t st, const char* label, double work, bool bytes);
#define NNT_CHECK_CTX(ctx)                                         \
    do {                                                           \
        if (!(ctx)) return NNT_EINVAL;                             \
        if ((ctx)->status != NNT_OK) return NNT_ESTATE;            \
    } while (0)
#define NNT_HIP(ctx, expr)                                                                   \
    do {                                                                                     \
        hipError_t e__ = (expr);                                                             \
        if (e__ != hipSuccess)                                                               \
            return nnt::fail((ctx), NNT_EHIP, std::string(#expr) + ": " + hipGetErrorString(e__)); \
    } while (0)

// Submits one task: waits for the tiles' pending users, runs `launch` on the
// chosen stream, records the task's completion.  `launch` returns a status.
int32_t submit(nnt_ctx* ctx, const std::vector<Access>& acc,
               const std::function<int32_t(hipStream_t)>& launch, int n_launches = 1);
int32_t ensure_scratch(nnt_ctx* ctx, int64_t elems);
int32_t static_scratch_setup();      // looks up the current device's address of the static scratch array (norm.hip)

// Adam on several parameter tensors in one launch (elementwise.hip); the group owns small device tables.
struct AdamGroup;
int32_t adam_group_create(nnt_ctx* ctx, int n, nnt_tensor* const* G, nnt_tensor* const* P, nnt_tensor* const* M,
                          nnt_tensor* const* V, nnt_tensor* const* LP, AdamGroup** out);
int32_t adam_group_step(nnt_ctx* ctx, AdamGroup* a, const nnt_adam_cfg* cfg, int32_t step);
void adam_group_destroy(AdamGroup* a);
void drop_plans_of(nnt_ctx* ctx, uint64_t tensor_id);
void plan_device_bytes(nnt_ctx* ctx, int64_t* tables, int64_t* workspaces);      // adds what the cached product plans hold

inline bool same_tiling(const nnt_tensor* a, const nnt_tensor* b) {
    if (a->ndim != b->ndim) return false;
    for (int i = 0; i < a->ndim; i++)
        if (a->shape[i] != b->shape[i] || a->base[i] != b->base[i]) return false;
    return true;
}
inline bool null_alike(const nnt_tensor* a, const nnt_tensor* b) {
    for (int64_t i = 0; i < a->ntiles; i++)
        if ((a->tiles[i] == nullptr) != (b->tiles[i] == nullptr)) return false;
    return true;
}

// ---- stream-level launchers used both by the tile API and by the tensor ops
int32_t launch_status(const char* what);

}  // namespace nnt
