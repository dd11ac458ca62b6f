// Sequential-task-flow executor on the HIP streams of one GPU (section 2, task
// submission): tasks arrive in program order with the tiles they read and write;
// read-after-write, write-after-read and write-after-write order per tile is kept
// with events between streams, everything else may overlap.
#include "internal.hpp"

#include <algorithm>
#include <cstring>

namespace nnt {

int32_t fail(nnt_ctx* ctx, int32_t code, const std::string& msg) {
    if (ctx) {
        ctx->error = msg;
        // argument errors are the caller's to fix and leave the context usable;
        // runtime failures stick
        if (code == NNT_EHIP) ctx->status = code;
    }
    return code;
}

int32_t launch_status(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        fprintf(stderr, "nntile_mi: launch of %s failed: %s\n", what, hipGetErrorString(e));
        return NNT_EHIP;
    }
    return NNT_OK;
}

static int32_t get_event(nnt_ctx* ctx, hipEvent_t* ev) {
    if (!ctx->event_pool.empty()) {
        *ev = ctx->event_pool.back();
        ctx->event_pool.pop_back();
        return NNT_OK;
    }
    NNT_HIP(ctx, hipEventCreateWithFlags(ev, hipEventDisableTiming));
    return NNT_OK;
}

// Everything recorded so far is complete: forget the events.
static void mark_all_synced(nnt_ctx* ctx) {
    for (int s = 0; s < ctx->n_streams; s++) {
        for (hipEvent_t e : ctx->events[s]) ctx->event_pool.push_back(e);
        ctx->events[s].clear();
        ctx->event_seq[s].clear();
        ctx->task_key[s].clear();
        ctx->synced_seq[s] = ctx->tail_seq[s];
    }
}

static int32_t sync_all(nnt_ctx* ctx) {
    for (int s = 0; s < ctx->n_streams; s++) NNT_HIP(ctx, hipStreamSynchronize(ctx->streams[s]));
    mark_all_synced(ctx);
    return NNT_OK;
}

// Which recorded sequence number of a stream covers `need`: the first one at or after it, or, if
// there is none, the stream's tail (which then gets an event).  Pure bookkeeping, shared with the
// host-side simulation.
static uint64_t covering_seq(const std::vector<uint64_t>& recorded, uint64_t need, uint64_t tail, bool* fresh) {
    auto it = std::lower_bound(recorded.begin(), recorded.end(), need);
    *fresh = it == recorded.end();
    return *fresh ? tail : *it;
}

// An event of stream `s` that completes no earlier than its task number `need`: the task's own event
// when it has one, else one recorded now at the tail of the stream.
static int32_t event_covering(nnt_ctx* ctx, int s, uint64_t need, hipEvent_t* ev, uint64_t* got) {
    bool fresh;
    *got = covering_seq(ctx->event_seq[s], need, ctx->tail_seq[s], &fresh);
    if (!fresh) {
        const size_t i = std::lower_bound(ctx->event_seq[s].begin(), ctx->event_seq[s].end(), need) - ctx->event_seq[s].begin();
        *ev = ctx->events[s][i];
        return NNT_OK;
    }
    int32_t rc = get_event(ctx, ev);
    if (rc != NNT_OK) return rc;
    NNT_HIP(ctx, hipEventRecord(*ev, ctx->streams[s]));
    ctx->events[s].push_back(*ev);
    ctx->event_seq[s].push_back(*got);
    return NNT_OK;
}

void profile_mark(nnt_ctx* ctx, hipStream_t st, const char* label, double work, bool bytes) {
    nnt_ctx::ProfileRec* p = ctx->cur_prof;
    if (!p) return;
    hipEvent_t ev[2];
    for (hipEvent_t& e : ev) {
        if (!ctx->timing_pool.empty()) { e = ctx->timing_pool.back(); ctx->timing_pool.pop_back(); }
        else if (hipEventCreate(&e) != hipSuccess) return;
    }
    nnt_ctx::ProfileRec done = *p;
    done.launches = p->launches > 1 ? p->launches - 1 : 1;
    (void)hipEventRecord(ev[0], st);
    (void)hipEventRecord(ev[1], st);
    // the events of the running record: its start goes with the closed part, its stop stays for the rest
    done.stop = ev[0];
    ctx->profile.push_back(done);
    p->start = ev[1];
    p->label = label;
    p->work = work;
    p->bytes = bytes;
    p->launches = 1;
}

// What identifies a task when the flow repeats: the first tile it writes (else the first it touches).
static const void* task_key_of(const std::vector<Access>& acc) {
    for (const Access& a : acc)
        if ((a.mode & kWrite) && a.count > 0) return a.first;
    return acc.empty() ? nullptr : static_cast<const void*>(acc[0].first);
}

// Where a task goes and what it has to wait for: pure bookkeeping, no device calls (the host-side
// simulation below runs the same two functions).
struct TaskPlan {
    int chosen;                          // stream of the task
    uint64_t wait_seq[kMaxStreams];      // per other stream: sequence number to wait for, 0 = none
};

// A task must run after the last writer of every tile it touches (read-after-write, write-after-write)
// and, if it writes, after every reader since that write (write-after-read).  One sequence number
// per stream is enough because a stream runs its tasks in order.
// `ns` streams may take the task; dependencies are looked for on all `ns_all` streams of the context (while a
// capture is open fewer streams take tasks than exist).
static TaskPlan plan_task(const std::vector<Access>& acc, int ns, int ns_all, bool serial, const uint64_t* tail_seq,
                          const uint64_t* synced_seq, uint64_t (*waited)[kMaxStreams], int* rr) {
    uint64_t need[kMaxStreams] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (const Access& a : acc) {
        for (int64_t i = 0; i < a.count; i++) {
            const TileDep& d = a.first[i];
            if (d.w_stream >= 0) need[d.w_stream] = std::max(need[d.w_stream], d.w_seq);
            // writers of parts: everybody comes after them, except a writer of another part
            for (int s = 0; s < ns_all; s++)
                if (d.p_seq[s] && !(a.mode == kWritePart && d.p_part[s] != a.part && !d.p_mixed[s])) need[s] = std::max(need[s], d.p_seq[s]);
            if (a.mode & kWrite)
                for (int s = 0; s < ns_all; s++) need[s] = std::max(need[s], d.r_seq[s]);
        }
    }
    for (int s = 0; s < ns_all; s++)
        if (need[s] <= synced_seq[s]) need[s] = 0;

    // Stream choice: stay behind a producer whose task is the tail of its stream
    // (no wait needed at all); otherwise take the next stream in turn, so that
    // independent consumers of one result spread over the streams.
    TaskPlan plan = {};
    int chosen = -1;
    if (serial || ns == 1) {
        chosen = 0;
    } else {
        uint64_t best = 0;
        for (int s = 0; s < ns; s++)
            if (need[s] && need[s] == tail_seq[s] && need[s] >= best) { best = need[s]; chosen = s; }
        if (chosen < 0) {
            *rr = (*rr + 1) % ns;
            chosen = *rr;
        }
    }
    plan.chosen = chosen;
    for (int s = 0; s < ns_all; s++) {
        if (s == chosen || !need[s]) continue;
        if (waited[chosen][s] >= need[s]) continue;      // an earlier task of this stream already waited that far
        plan.wait_seq[s] = need[s];
        waited[chosen][s] = need[s];
    }
    return plan;
}

// The task with sequence number `seq` on stream `chosen` becomes the last user of its tiles.
static void commit_task(const std::vector<Access>& acc, int chosen, uint64_t seq) {
    for (const Access& a : acc) {
        for (int64_t i = 0; i < a.count; i++) {
            TileDep& d = a.first[i];
            if (a.mode == kWritePart) {
                // (the readers it has waited for stay on record: a later writer waits for them once more)
                if (d.p_seq[chosen] && d.p_part[chosen] != a.part) d.p_mixed[chosen] = 1;
                d.p_seq[chosen] = seq;
                d.p_part[chosen] = a.part;
            } else if (a.mode & kWrite) {
                d.w_stream = chosen;
                d.w_seq = seq;
                std::memset(d.r_seq, 0, sizeof(d.r_seq));
                std::memset(d.p_seq, 0, sizeof(d.p_seq));
                std::memset(d.p_part, 0, sizeof(d.p_part));
                std::memset(d.p_mixed, 0, sizeof(d.p_mixed));
            } else {
                d.r_seq[chosen] = seq;
            }
        }
    }
}

int32_t submit(nnt_ctx* ctx, const std::vector<Access>& acc,
               const std::function<int32_t(hipStream_t)>& launch, int n_launches) {
    NNT_CHECK_CTX(ctx);
    // While a capture is open only streams 0 and 1 take tasks: ending a capture in which two forked
    // streams wait on each other's events has crashed inside the HIP runtime on this ROCm release.
    const int ns = ctx->capturing ? std::min(ctx->n_streams, 2) : ctx->n_streams;
    const TaskPlan plan = plan_task(acc, ns, ctx->n_streams, ctx->serial, ctx->tail_seq, ctx->synced_seq, ctx->waited, &ctx->rr);
    const int chosen = plan.chosen;
    hipStream_t st = ctx->streams[chosen];
    for (int s = 0; s < ctx->n_streams; s++) {
        if (!plan.wait_seq[s]) continue;
        // the task waited for is consumed across streams: from now on its like gets an event of its own
        const uint64_t rel = plan.wait_seq[s] - ctx->synced_seq[s] - 1;
        if (rel < ctx->task_key[s].size() && ctx->task_key[s][rel]) {
            if (ctx->hot_producers.size() > (1u << 16)) ctx->hot_producers.clear();      // stale keys of destroyed tensors: learn afresh
            ctx->hot_producers.insert(ctx->task_key[s][rel]);
        }
        hipEvent_t ev;
        uint64_t got;
        int32_t wrc = event_covering(ctx, s, plan.wait_seq[s], &ev, &got);
        if (wrc != NNT_OK) return wrc;
        NNT_HIP(ctx, hipStreamWaitEvent(st, ev, 0));
        ctx->waited[chosen][s] = std::max(ctx->waited[chosen][s], got);
        ctx->stats.event_waits++;
    }
    nnt_ctx::ProfileRec prof;
    const bool timed = ctx->profiling && !ctx->capturing;
    if (timed) {
        for (hipEvent_t* e : {&prof.start, &prof.stop}) {
            if (!ctx->timing_pool.empty()) { *e = ctx->timing_pool.back(); ctx->timing_pool.pop_back(); }
            else NNT_HIP(ctx, hipEventCreate(e));
        }
        prof.label = ctx->cur_label ? ctx->cur_label : "task";
        prof.work = ctx->cur_work;
        prof.bytes = ctx->cur_work_is_bytes;
        prof.launches = n_launches;
        ctx->cur_work = 0.0;     // the operation's work is counted once, on its first task
        NNT_HIP(ctx, hipEventRecord(prof.start, st));
    }
    ctx->cur_prof = timed ? &prof : nullptr;
    int32_t rc = launch(st);
    ctx->cur_prof = nullptr;
    if (timed) {
        NNT_HIP(ctx, hipEventRecord(prof.stop, st));
        ctx->profile.push_back(prof);
    }
    if (rc != NNT_OK) {
        if (rc == NNT_EHIP) return fail(ctx, rc, "kernel launch failed");
        return rc;
    }
    ctx->stats.tasks++;
    ctx->stats.launches += n_launches;
    uint64_t seq = ++ctx->tail_seq[chosen];
    commit_task(acc, chosen, seq);
    // A marker between two kernels costs the device more than a microsecond, and most tasks are only
    // ever waited for by their successor on the same stream, so only the tasks known to be consumed
    // across streams get an event of their own; a wait for any other task records one at the tail of
    // that stream at that moment (and so may wait for later tasks of that stream as well: a branch
    // that should overlap is serialised once, then its producer is known).  With one stream nothing
    // is ever waited for.
    const void* key = task_key_of(acc);
    ctx->task_key[chosen].push_back(key);
    if (ns > 1 && !ctx->serial && key && ctx->hot_producers.count(key)) {
        hipEvent_t ev;
        int32_t erc = get_event(ctx, &ev);
        if (erc != NNT_OK) return erc;
        NNT_HIP(ctx, hipEventRecord(ev, st));
        ctx->events[chosen].push_back(ev);
        ctx->event_seq[chosen].push_back(seq);
    }
    // bound the bookkeeping of long runs without nnt_wait
    if (!ctx->capturing && (ctx->events[chosen].size() > (1u << 16) || ctx->task_key[chosen].size() > (1u << 20))) return sync_all(ctx);
    return NNT_OK;
}

int32_t ensure_scratch(nnt_ctx* ctx, int64_t elems) {
    if (elems <= ctx->red_scratch_elems) return NNT_OK;
    if (ctx->capturing) return fail(ctx, NNT_ESTATE, "reduction scratch must exist before capture: run the operation once first");
    int32_t rc = sync_all(ctx);
    if (rc != NNT_OK) return rc;
    if (ctx->red_scratch) NNT_HIP(ctx, hipFree(ctx->red_scratch));
    ctx->red_scratch = nullptr;
    ctx->red_scratch_elems = 0;
    int64_t want = std::max<int64_t>(elems, 1 << 20);
    NNT_HIP(ctx, hipMalloc((void**)&ctx->red_scratch, want * sizeof(float)));
    ctx->red_scratch_elems = want;
    return NNT_OK;
}

}  // namespace nnt

using namespace nnt;

struct nnt_graph {
    nnt_ctx* ctx;
    hipGraph_t graph;
    hipGraphExec_t exec;
};

extern "C" {

const char* nnt_version(void) { return "nntile_mi 0.1 (gfx950)"; }

int32_t nnt_sched_simulate(int32_t n_streams, int32_t serial, int32_t n_tiles, int32_t n_tasks, const int32_t* task_first,
                           const int32_t* acc_tile, const int32_t* acc_mode, int32_t* stream_out, int64_t* seq_out,
                           int64_t* wait_seq_out) {
    if (n_streams < 1 || n_streams > kMaxStreams || n_tiles < 0 || n_tasks < 0) return NNT_EINVAL;
    if (n_tasks > 0 && (!task_first || !acc_tile || !acc_mode || !stream_out || !seq_out || !wait_seq_out)) return NNT_EINVAL;
    std::vector<TileDep> tiles((size_t)n_tiles);
    uint64_t tail[kMaxStreams] = {0}, synced[kMaxStreams] = {0}, waited[kMaxStreams][kMaxStreams] = {{0}};
    std::vector<uint64_t> recorded[kMaxStreams];
    std::vector<const void*> keys[kMaxStreams];
    std::unordered_set<const void*> hot;
    int rr = 0;
    for (int t = 0; t < n_tasks; t++) {
        std::vector<Access> acc;
        for (int i = task_first[t]; i < task_first[t + 1]; i++) {
            const int mode = acc_mode[i] & 0xff, part = acc_mode[i] >> 8;
            if (acc_tile[i] < 0 || acc_tile[i] >= n_tiles || acc_mode[i] < 0 || !((mode >= kRead && mode <= kReadWrite) || mode == kWritePart) ||
                (mode != kWritePart && part != 0))
                return NNT_EINVAL;
            acc.push_back(Access{&tiles[(size_t)acc_tile[i]], 1, mode, part});
        }
        const TaskPlan plan = plan_task(acc, n_streams, n_streams, serial != 0, tail, synced, waited, &rr);
        // the waits as the executor would issue them: on the first recorded event that covers the
        // task asked for, else on a new one at the tail of that stream
        for (int s = 0; s < kMaxStreams; s++) {
            uint64_t got = 0;
            if (plan.wait_seq[s]) {
                if (keys[s][plan.wait_seq[s] - 1]) hot.insert(keys[s][plan.wait_seq[s] - 1]);
                bool fresh;
                got = covering_seq(recorded[s], plan.wait_seq[s], tail[s], &fresh);
                if (fresh) recorded[s].push_back(got);
                waited[plan.chosen][s] = std::max(waited[plan.chosen][s], got);
            }
            wait_seq_out[(size_t)t * kMaxStreams + s] = (int64_t)got;
        }
        const uint64_t seq = ++tail[plan.chosen];
        commit_task(acc, plan.chosen, seq);
        const void* key = task_key_of(acc);
        keys[plan.chosen].push_back(key);
        if (n_streams > 1 && !serial && key && hot.count(key)) recorded[plan.chosen].push_back(seq);
        stream_out[t] = plan.chosen;
        seq_out[t] = (int64_t)seq;
    }
    return NNT_OK;
}

int32_t nnt_ctx_create(int32_t device, int32_t n_streams, void* const* caller_streams, nnt_ctx** out) {
    if (!out || n_streams < 1 || n_streams > kMaxStreams) return NNT_EINVAL;
    *out = nullptr;
    if (hipSetDevice(device) != hipSuccess) return NNT_EHIP;
    if (static_scratch_setup() != NNT_OK) return NNT_EHIP;      // this device's address of the static scratch array
    nnt_ctx* ctx = new (std::nothrow) nnt_ctx();
    if (!ctx) return NNT_ENOMEM;
    ctx->device = device;
    ctx->n_streams = n_streams;
    ctx->own_streams = caller_streams == nullptr;
    for (int s = 0; s < kMaxStreams; s++) {
        ctx->streams[s] = nullptr;
        ctx->tail_seq[s] = ctx->synced_seq[s] = 0;
        for (int d = 0; d < kMaxStreams; d++) ctx->waited[s][d] = 0;
    }
    for (int s = 0; s < n_streams; s++) {
        if (caller_streams) {
            ctx->streams[s] = (hipStream_t)caller_streams[s];
        } else if (hipStreamCreateWithFlags(&ctx->streams[s], hipStreamNonBlocking) != hipSuccess) {
            delete ctx;
            return NNT_EHIP;
        }
    }
    *out = ctx;
    return NNT_OK;
}

int32_t nnt_ctx_destroy(nnt_ctx* ctx) {
    if (!ctx) return NNT_EINVAL;
    if (ctx->live_tensors != 0) return fail(ctx, NNT_ESTATE, "tensors still alive on this context");
    for (int s = 0; s < ctx->n_streams; s++) (void)hipStreamSynchronize(ctx->streams[s]);
    mark_all_synced(ctx);
    for (hipEvent_t e : ctx->event_pool) (void)hipEventDestroy(e);
    for (auto& r : ctx->profile) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    for (hipEvent_t e : ctx->timing_pool) (void)hipEventDestroy(e);
    ctx->gemm_plans.clear();
    if (ctx->red_scratch) (void)hipFree(ctx->red_scratch);
    if (ctx->own_streams)
        for (int s = 0; s < ctx->n_streams; s++) (void)hipStreamDestroy(ctx->streams[s]);
    delete ctx;
    return NNT_OK;
}

int32_t nnt_wait(nnt_ctx* ctx) {
    if (!ctx) return NNT_EINVAL;
    if (ctx->capturing) return fail(ctx, NNT_ESTATE, "nnt_wait during capture");
    for (int s = 0; s < ctx->n_streams; s++) {
        hipError_t e = hipStreamSynchronize(ctx->streams[s]);
        if (e != hipSuccess) return fail(ctx, NNT_EHIP, std::string("hipStreamSynchronize: ") + hipGetErrorString(e));
    }
    mark_all_synced(ctx);
    return ctx->status;
}

int32_t nnt_ctx_join(nnt_ctx* ctx) {
    NNT_CHECK_CTX(ctx);
    hipStream_t s0 = ctx->streams[0];
    for (int s = 1; s < ctx->n_streams; s++) {
        uint64_t tail = ctx->tail_seq[s];
        if (tail <= ctx->synced_seq[s] || ctx->waited[0][s] >= tail) continue;
        hipEvent_t ev;
        uint64_t got;
        int32_t rc = event_covering(ctx, s, tail, &ev, &got);
        if (rc != NNT_OK) return rc;
        NNT_HIP(ctx, hipStreamWaitEvent(s0, ev, 0));
        ctx->waited[0][s] = tail;
    }
    return NNT_OK;
}

int32_t nnt_ctx_stream(nnt_ctx* ctx, int32_t i, void** out) {
    if (!ctx || !out || i < 0 || i >= ctx->n_streams) return NNT_EINVAL;
    *out = (void*)ctx->streams[i];
    return NNT_OK;
}

const char* nnt_last_error(nnt_ctx* ctx) { return ctx ? ctx->error.c_str() : "null context"; }

int32_t nnt_ctx_set_serial(nnt_ctx* ctx, int32_t serial) {
    NNT_CHECK_CTX(ctx);
    ctx->serial = serial != 0;
    return NNT_OK;
}

int32_t nnt_ctx_set_granularity(nnt_ctx* ctx, int32_t g) {
    NNT_CHECK_CTX(ctx);
    if (g != NNT_GRAN_OP && g != NNT_GRAN_TILE) return fail(ctx, NNT_EINVAL, "unknown granularity");
    ctx->granularity = g;
    return NNT_OK;
}

int32_t nnt_ctx_stats(nnt_ctx* ctx, nnt_exec_stats* out) {
    if (!ctx || !out) return NNT_EINVAL;
    *out = ctx->stats;
    out->plans = (int64_t)ctx->gemm_plans.size();
    out->device_table_bytes = ctx->table_bytes;
    out->device_workspace_bytes = ctx->red_scratch_elems * (int64_t)sizeof(float);
    plan_device_bytes(ctx, &out->device_table_bytes, &out->device_workspace_bytes);
    return NNT_OK;
}

// ---------------------------------------------------------------- per-task timing
int32_t nnt_profile_enable(nnt_ctx* ctx, int32_t on) {
    NNT_CHECK_CTX(ctx);
    if (ctx->capturing) return fail(ctx, NNT_ESTATE, "nnt_profile_enable during capture");
    int32_t rc = sync_all(ctx);
    if (rc != NNT_OK) return rc;
    for (auto& r : ctx->profile) { ctx->timing_pool.push_back(r.start); ctx->timing_pool.push_back(r.stop); }
    ctx->profile.clear();
    ctx->profiling = on != 0;
    return NNT_OK;
}

int32_t nnt_profile_read(nnt_ctx* ctx, nnt_profile_entry* out, int32_t capacity, int32_t* n_out) {
    NNT_CHECK_CTX(ctx);
    if (!n_out || capacity < 0 || (capacity > 0 && !out)) return fail(ctx, NNT_EINVAL, "nnt_profile_read: bad argument");
    int32_t rc = sync_all(ctx);
    if (rc != NNT_OK) return rc;
    std::map<std::string, nnt_profile_entry> agg;
    for (auto& r : ctx->profile) {
        float ms = 0.f;
        NNT_HIP(ctx, hipEventElapsedTime(&ms, r.start, r.stop));
        auto it = agg.find(r.label);
        if (it == agg.end()) {
            nnt_profile_entry e = {};
            snprintf(e.label, sizeof(e.label), "%s", r.label.c_str());
            e.work_is_bytes = r.bytes ? 1 : 0;
            it = agg.insert({r.label, e}).first;
        }
        it->second.tasks += 1;
        it->second.launches += r.launches;
        it->second.ms += ms;
        it->second.work += r.work;
    }
    int32_t n = 0;
    for (auto& kv : agg) {
        if (n < capacity) out[n] = kv.second;
        n++;
    }
    *n_out = n;
    return NNT_OK;
}

// ---------------------------------------------------------------- graph capture
int32_t nnt_capture_begin(nnt_ctx* ctx) {
    NNT_CHECK_CTX(ctx);
    if (ctx->capturing) return fail(ctx, NNT_ESTATE, "capture already open");
    int32_t rc = sync_all(ctx);
    if (rc != NNT_OK) return rc;
    NNT_HIP(ctx, hipStreamBeginCapture(ctx->streams[0], hipStreamCaptureModeRelaxed));
    ctx->capturing = true;
    // fork: every other stream joins the capture by waiting for a node of stream 0
    if (ctx->n_streams > 1) {
        hipEvent_t ev;
        rc = get_event(ctx, &ev);
        if (rc != NNT_OK) return rc;
        NNT_HIP(ctx, hipEventRecord(ev, ctx->streams[0]));
        for (int s = 1; s < std::min(ctx->n_streams, 2); s++) NNT_HIP(ctx, hipStreamWaitEvent(ctx->streams[s], ev, 0));
        ctx->capture_events.push_back(ev);      // no event is recorded twice inside one capture
    }
    return NNT_OK;
}

int32_t nnt_capture_end(nnt_ctx* ctx, nnt_graph** out) {
    if (!ctx || !out) return NNT_EINVAL;
    if (!ctx->capturing) return fail(ctx, NNT_ESTATE, "no capture open");
    *out = nullptr;
    // join: stream 0 waits for the tail of the other capturing stream
    for (int s = 1; s < std::min(ctx->n_streams, 2); s++) {
        hipEvent_t ev;
        int32_t rc = get_event(ctx, &ev);
        if (rc != NNT_OK) return rc;
        NNT_HIP(ctx, hipEventRecord(ev, ctx->streams[s]));
        NNT_HIP(ctx, hipStreamWaitEvent(ctx->streams[0], ev, 0));
        ctx->capture_events.push_back(ev);
    }
    hipGraph_t graph;
    ctx->capturing = false;
    const bool trace = getenv("NNT_TRACE") != nullptr;
    if (trace) fprintf(stderr, "nnt: capture_end: joined, ending capture\n");
    NNT_HIP(ctx, hipStreamEndCapture(ctx->streams[0], &graph));
    if (trace) fprintf(stderr, "nnt: capture_end: capture ended, instantiating\n");
    // the recorded tasks have not run: their events mean nothing outside the graph
    mark_all_synced(ctx);
    for (hipEvent_t e : ctx->capture_events) ctx->event_pool.push_back(e);
    ctx->capture_events.clear();
    hipGraphExec_t exec;
    NNT_HIP(ctx, hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));
    if (trace) fprintf(stderr, "nnt: capture_end: instantiated\n");
    nnt_graph* g = new (std::nothrow) nnt_graph{ctx, graph, exec};
    if (!g) return NNT_ENOMEM;
    *out = g;
    return NNT_OK;
}

int32_t nnt_graph_launch(nnt_graph* g) {
    if (!g) return NNT_EINVAL;
    nnt_ctx* ctx = g->ctx;
    NNT_CHECK_CTX(ctx);
    // everything submitted earlier on other streams must be done before the replay starts
    int32_t rc = nnt_ctx_join(ctx);
    if (rc != NNT_OK) return rc;
    NNT_HIP(ctx, hipGraphLaunch(g->exec, ctx->streams[0]));
    // later tasks on any stream must see the replay's results: they order after stream 0
    if (ctx->n_streams > 1) {
        hipEvent_t ev;
        rc = get_event(ctx, &ev);
        if (rc != NNT_OK) return rc;
        NNT_HIP(ctx, hipEventRecord(ev, ctx->streams[0]));
        for (int s = 1; s < ctx->n_streams; s++) NNT_HIP(ctx, hipStreamWaitEvent(ctx->streams[s], ev, 0));
        ctx->event_pool.push_back(ev);   // safe to reuse: a re-record does not disturb waits already enqueued
    }
    ctx->stats.launches++;
    return NNT_OK;
}

int32_t nnt_graph_destroy(nnt_graph* g) {
    if (!g) return NNT_EINVAL;
    (void)hipGraphExecDestroy(g->exec);
    (void)hipGraphDestroy(g->graph);
    delete g;
    return NNT_OK;
}

}  // extern "C"
