// The C ABI of include/p2.h: argument checks, planning, table upload, kernel launches and
// copy-back.  All arithmetic of the method runs in the kernels; this file only moves data.
#include <algorithm>
#include <chrono>
#include <cstddef>
#include <cstring>
#include <atomic>
#include <functional>
#include <thread>
#include <limits>
#include <string>
#include <vector>

#include "p2_device.h"
#include "p2_plan.h"

namespace p2 {
hipError_t launch_cost_literal(const DevQuery* q, int R, int k, const unsigned long long* sorted, uint32_t n,
                               p2_program* out_prog, double* out_cost, int only_missing, void* gscratch,
                               hipStream_t stream);
}

namespace {

thread_local std::string g_err;

struct DevBuf {
    void* p = nullptr;
    size_t cap = 0;
    hipError_t ensure(size_t bytes) {
        if (bytes <= cap) return hipSuccess;
        if (p) (void)hipFree(p);
        p = nullptr; cap = 0;
        size_t want = std::max(bytes, (size_t)4096);
        want = (want + 4095) & ~(size_t)4095;
        hipError_t e = hipMalloc(&p, want);
        if (e == hipSuccess) cap = want;
        return e;
    }
};
// grow a device buffer to `bytes`, keeping its first `keep` bytes
hipError_t grow_keep(DevBuf& b, size_t bytes, size_t keep, hipStream_t stream) {
    if (bytes <= b.cap) return hipSuccess;
    size_t want = std::max(bytes, b.cap * 2);
    want = (want + 4095) & ~(size_t)4095;
    void* np = nullptr;
    hipError_t e = hipMalloc(&np, want);
    if (e != hipSuccess) return e;
    if (b.p && keep) {
        e = hipMemcpyAsync(np, b.p, keep, hipMemcpyDeviceToDevice, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e != hipSuccess) { (void)hipFree(np); return e; }
    }
    if (b.p) (void)hipFree(b.p);
    b.p = np; b.cap = want;
    return hipSuccess;
}

struct HostBuf {
    void* p = nullptr;
    size_t cap = 0;
    hipError_t ensure(size_t bytes) {
        if (bytes <= cap) return hipSuccess;
        if (p) (void)hipHostFree(p);
        p = nullptr; cap = 0;
        size_t want = std::max(bytes, (size_t)4096);
        want = (want + 4095) & ~(size_t)4095;
        hipError_t e = hipHostMalloc(&p, want, hipHostMallocDefault);
        if (e == hipSuccess) cap = want;
        return e;
    }
};

// Event pairs around single launches: a pool that grows on demand and is kept.
struct SpanRec {
    enum Kind { kClassify = 0, kLiteral = 1, kMaterialize = 2, kGroup = 3, kKinds = 4 };
    struct Span { int kind; size_t first; int dispatches; };
    bool on = false;
    bool kernels_only = false;         // only the classification and the building of children are timed
    bool open = false;                 // the span begun last is being recorded
    std::vector<hipEvent_t> pool;
    std::vector<Span> spans;
    size_t used = 0;
    hipError_t begin(int kind, hipStream_t stream, int dispatches = 1) {
        open = on && !(kernels_only && kind != kClassify && kind != kMaterialize);
        if (!open) return hipSuccess;
        while (pool.size() < used + 2) {
            hipEvent_t e = nullptr;
            const hipError_t rc = hipEventCreate(&e);
            if (rc != hipSuccess) return rc;
            pool.push_back(e);
        }
        spans.push_back(Span{kind, used, dispatches});
        used += 2;
        return hipEventRecord(pool[used - 2], stream);
    }
    hipError_t end(hipStream_t stream) { return open ? hipEventRecord(pool[used - 1], stream) : hipSuccess; }
    void reset() { spans.clear(); used = 0; }
    // after the stream has been waited for: time and launches per kind, added to what is there
    hipError_t collect(float ms[kKinds], int32_t launches[kKinds]) {
        for (const Span& sp : spans) {
            float t = 0.f;
            const hipError_t rc = hipEventElapsedTime(&t, pool[sp.first], pool[sp.first + 1]);
            if (rc != hipSuccess) return rc;
            ms[sp.kind] += t;
            launches[sp.kind] += sp.dispatches;
        }
        reset();
        return hipSuccess;
    }
    void release() {
        for (auto& e : pool) (void)hipEventDestroy(e);
        pool.clear(); reset();
    }
};

// What one enumeration of the frontier engine works in: its own stream (and a second one for the literal prefixes
// of a level), its lists, its counters.  A call runs as many enumerations side by side as there are slots, a host
// thread each: an enumeration is a chain of small launches with one host wait per level, and several chains fill
// the chip where one does not.
constexpr int kFrontSlots = 4;
struct FrontSlot {
    hipStream_t stream = nullptr;         // (created by Ctx::open_slot_streams, together with those of the other slots)
    DevBuf f_entries[2], f_states[2], f_sums[2], f_entries2[2], f_states2[2], f_sums2[2], f_literal[2];
    DevBuf f_surv, f_surv_literal, f_unknown, f_ctr, lit_scratch;
    DevBuf f_hash[2], f_hash2[2], f_table, f_rep[2], f_replist[2], f_codes[2], f_unk[2];     // search for equal states
    DevBuf f_sid[2], f_sid2[2], f_delta[3], f_childof[2], f_ssurv;                           // prefixes -> states -> children
    DevBuf f_rowcnt[2];                                                                      // per row of codes: how many survivors by kind
    DevBuf f_walk[2];                                                                        // the last level: states worth a walk
    HostBuf h_fctr;
    SpanRec spans;
    // what the slot's launches of this call worked on (the figures of p2_profile)
    double prof_prefixes = 0.0, prof_state_bytes = 0.0, prof_lane_ops = 0.0, prof_children = 0.0, prof_mat_bytes = 0.0, prof_entries = 0.0;
    int32_t rc = 0;
    std::string err;
    void release() {
        DevBuf* dev[] = {&f_entries[0], &f_entries[1], &f_states[0], &f_states[1], &f_sums[0], &f_sums[1], &f_entries2[0], &f_entries2[1],
                         &f_states2[0], &f_states2[1], &f_sums2[0], &f_sums2[1], &f_literal[0], &f_literal[1], &f_surv, &f_surv_literal,
                         &f_unknown, &f_ctr, &lit_scratch, &f_hash[0], &f_hash[1], &f_hash2[0], &f_hash2[1], &f_table, &f_rep[0], &f_rep[1],
                         &f_replist[0], &f_replist[1], &f_codes[0], &f_codes[1], &f_unk[0], &f_unk[1], &f_sid[0], &f_sid[1], &f_sid2[0],
                         &f_sid2[1], &f_delta[0], &f_delta[1], &f_delta[2], &f_childof[0], &f_childof[1], &f_ssurv, &f_walk[0], &f_walk[1], &f_rowcnt[0], &f_rowcnt[1]};
        for (DevBuf* b : dev) { if (b->p) (void)hipFree(b->p); b->p = nullptr; b->cap = 0; }
        if (h_fctr.p) (void)hipHostFree(h_fctr.p);
        h_fctr.p = nullptr; h_fctr.cap = 0;
        spans.release();
        if (stream) { (void)hipStreamDestroy(stream); stream = nullptr; }
    }
};

// Device scratch owned by the library, one set per host thread, reused between calls.
struct Ctx {
    ~Ctx();
    void release();
    DevBuf rows, rows_hdr;
    DevBuf blob, valid, rerun, sorted, progs, costs, counters, topk_scratch, topk_pos, topk_in, topk_jobs, lit_scratch, post;
    DevBuf sel_progs, sel_costs, gather;                    // the rows that shortlists picked, and whose they are
    HostBuf h_gather;
    DevBuf f_finish;                                        // frontier engine: what every query's rows are written from
    HostBuf h_finish;
    DevBuf f_rank, f_share;                                 // frontier engine: ranks of the valid programs, queries of the enumerations
    std::vector<DevBuf> f_evalid, f_egsums;                 // ... per enumeration: valid candidate indices, their cost sums
    FrontSlot slots[kFrontSlots];
    static constexpr int kSpareStreams = 6;
    hipStream_t spare_streams[kSpareStreams] = {};          // created beside the slots' streams and found to share a queue with one: never used
    DevBuf probe_sink;
    hipError_t open_slot_streams();
    hipEvent_t front_go = nullptr;                          // the call's stream has reached the enumerations
    HostBuf h_rows, h_rows_hdr;
    hipStream_t copy_stream = nullptr;      // uploads that overlap with the kernels of the call's stream
    hipEvent_t copy_done = nullptr;
    HostBuf h_blob, h_counters, h_progs, h_costs, h_pos, h_post, h_topk_jobs, h_fshare;
};
thread_local Ctx g_ctx;

// The streams of the slots.  The runtime deals a process's streams out to its hardware queues (four unless the
// caller's environment says otherwise) as they are created, streams that share a queue take turns, and which queue a
// new stream lands on depends on every stream the process has created before.  So the library looks: it creates a
// handful of streams, runs a short one-block kernel on pairs of them (side by side: the time of one; taking turns:
// of two) and gives the slots streams that do not take turns with each other; the other streams stay unused.  With
// fewer independent queues than slots the remaining slots share.  Only the overlap depends on this, never a result;
// a pair that is wrongly taken to share (the host thread lost its turn while timing) costs overlap and nothing else.
__global__ __launch_bounds__(64) void k_queue_probe(uint32_t* sink, int n) {
    uint32_t x = threadIdx.x + 1u;
    for (int i = 0; i < n; ++i) x = x * 1664525u + 1013904223u;
    if (x == 0x9e3779b9u) sink[0] = x;               // (keeps the loop; the sink is the library's own word)
}
hipError_t Ctx::open_slot_streams() {
    if (slots[0].stream) return hipSuccess;
    constexpr int kCandidates = kFrontSlots + kSpareStreams;
    constexpr int kProbeSteps = 8000;                 // some 0.1 ms: several times what a launch and a wait take
    hipStream_t made[kCandidates] = {};
    hipError_t e = probe_sink.ensure(256);
    for (int i = 0; i < kCandidates && e == hipSuccess; ++i) e = hipStreamCreateWithFlags(&made[i], hipStreamNonBlocking);
    auto timed = [&](hipStream_t a, hipStream_t b, double& ms) -> hipError_t {
        const auto t0 = std::chrono::steady_clock::now();
        hipLaunchKernelGGL(k_queue_probe, dim3(1), dim3(64), 0, a, static_cast<uint32_t*>(probe_sink.p), kProbeSteps);
        if (b) hipLaunchKernelGGL(k_queue_probe, dim3(1), dim3(64), 0, b, static_cast<uint32_t*>(probe_sink.p), kProbeSteps);
        hipError_t r = hipGetLastError();
        const hipError_t ra = hipStreamSynchronize(a);
        const hipError_t rb = b ? hipStreamSynchronize(b) : hipSuccess;
        ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
        return r != hipSuccess ? r : ra != hipSuccess ? ra : rb;
    };
    int chosen[kFrontSlots], n_chosen = 0;
    bool taken[kCandidates] = {};
    if (e == hipSuccess) {
        double one = 1e30, t = 0.0;
        for (int rep = 0; rep < 4 && e == hipSuccess; ++rep) {        // (the first launch also loads the kernel)
            e = timed(made[0], nullptr, t);
            if (rep > 0) one = std::min(one, t);
        }
        for (int c = 0; c < kCandidates && n_chosen < kFrontSlots && e == hipSuccess; ++c) {
            bool apart = true;
            for (int k = 0; k < n_chosen && apart && e == hipSuccess; ++k) {
                double best = 1e30;
                for (int rep = 0; rep < 2 && e == hipSuccess; ++rep) { e = timed(made[chosen[k]], made[c], t); best = std::min(best, t); }
                apart = best < 1.5 * one;
            }
            if (apart && e == hipSuccess) { chosen[n_chosen++] = c; taken[c] = true; }
        }
        for (int c = 0; c < kCandidates && n_chosen < kFrontSlots; ++c)
            if (!taken[c]) { chosen[n_chosen++] = c; taken[c] = true; }
    }
    if (e != hipSuccess) {
        for (hipStream_t st : made) if (st) (void)hipStreamDestroy(st);
        return e;
    }
    for (int t = 0; t < kFrontSlots; ++t) slots[t].stream = made[chosen[t]];
    int n_spare = 0;
    for (int c = 0; c < kCandidates; ++c) if (!taken[c]) spare_streams[n_spare++] = made[c];
    return hipSuccess;
}

// Frontier lists shorter than this are judged entry by entry: grouping them by state would cost more than it saves.
constexpr uint32_t kGroupMin = 256;

struct Prof {
    ~Prof();
    void release();
    bool on = false;
    bool kernels_only = false;      // p2_set_profiling(2): of the frontier engine's launches, only classification and children
    hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};     // evaluation begin / end, post end, frontier begin / end
    p2_profile last = {};
};
thread_local Prof g_prof;

// What a host thread's calls have cached on the device is given back when the thread ends, or on request
// (p2_release_thread).  The thread that loaded the library is left alone at process exit: by then the HIP
// runtime may be shutting down, and the process's memory goes with it anyway.
const std::thread::id g_loader_thread = std::this_thread::get_id();

void Ctx::release() {
    DevBuf* dev[] = {&rows, &rows_hdr, &blob, &valid, &rerun, &sorted, &progs, &costs, &counters, &topk_scratch, &topk_pos,
                     &topk_in, &topk_jobs, &lit_scratch, &post, &f_rank, &f_share, &sel_progs, &sel_costs, &gather, &f_finish, &probe_sink};
    for (DevBuf* b : dev) { if (b->p) (void)hipFree(b->p); b->p = nullptr; b->cap = 0; }
    for (auto* v : {&f_evalid, &f_egsums}) {
        for (DevBuf& b : *v) if (b.p) (void)hipFree(b.p);
        v->clear();
    }
    for (FrontSlot& sl : slots) sl.release();
    for (hipStream_t& sp : spare_streams) { if (sp) (void)hipStreamDestroy(sp); sp = nullptr; }
    HostBuf* host[] = {&h_rows, &h_rows_hdr, &h_blob, &h_counters, &h_progs, &h_costs, &h_pos, &h_post, &h_topk_jobs, &h_fshare, &h_gather, &h_finish};
    for (HostBuf* b : host) { if (b->p) (void)hipHostFree(b->p); b->p = nullptr; b->cap = 0; }
    if (front_go) { (void)hipEventDestroy(front_go); front_go = nullptr; }
    if (copy_done) { (void)hipEventDestroy(copy_done); copy_done = nullptr; }
    if (copy_stream) { (void)hipStreamDestroy(copy_stream); copy_stream = nullptr; }
}
Ctx::~Ctx() { if (std::this_thread::get_id() != g_loader_thread) release(); }
void Prof::release() {
    for (auto& e : ev) { if (e) (void)hipEventDestroy(e); e = nullptr; }
    on = false;
}
Prof::~Prof() { if (std::this_thread::get_id() != g_loader_thread) release(); }

int32_t fail(int32_t code, const std::string& msg) {
    g_err = msg;
    return code;
}
// Stream of the call in progress on this thread.  When a HIP call fails, what the call has queued so far
// (kernels and copies that use the cached pinned and device buffers) is waited for before the error goes
// back to the caller, so that the next call does not reuse buffers that are still in flight.
thread_local hipStream_t g_call_stream = nullptr;
thread_local bool g_call_active = false;
int32_t hip_fail(hipError_t e, const char* what) {
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    (void)hipGetLastError();
    if (g_call_active) {
        (void)hipStreamSynchronize(g_call_stream);
        if (g_ctx.copy_stream) (void)hipStreamSynchronize(g_ctx.copy_stream);
        (void)hipGetLastError();
    }
    return P2_EDEVICE;
}
struct CallScope {
    explicit CallScope(hipStream_t s) { g_call_stream = s; g_call_active = true; }
    ~CallScope() { g_call_active = false; g_call_stream = nullptr; }
};
#define P2_HIP(call)                                      \
    do {                                                  \
        hipError_t e_ = (call);                           \
        if (e_ != hipSuccess) return hip_fail(e_, #call); \
    } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Selections over at most this many valid programs go into one launch for the whole batch
// (one wavefront each); longer lists take the two-stage selection, one query at a time.
constexpr size_t kTopkJobMax = 8192;

struct QueryRun {
    p2::Plan plan;
    int engine = P2_ENGINE_LITERAL;       // engine evaluating the bulk (LITERAL or COMPACT)
    bool frontier = false;                // enumeration by size with pruning instead of index by index
    bool regs = false;                    // per-candidate small-group engine (steps computed in registers)
    bool shared = false;                  // shared-prefix engine (the common instructions of a group applied once)
    bool auto_groups = false;             // its handed-over groups are picked up by the device-driven literal launch
    bool wave_cost = false;               // valid programs costed by the wavefront-per-program kernel
    int enum_id = -1, share_pos = 0;      // frontier: its enumeration, and its place among the enumeration's queries
    int topk = 0;
    size_t off_query = 0, off_rowptr = 0, off_rowlevel = 0, off_entries = 0;
    size_t off_goal = 0, off_rank = 0;    // hierarchies other than the collapsed one: goal masks, ranks of members
    int same_as = -1;                     // an earlier query of the batch with the same reduction group, chunks, patterns,
                                          // alphabet and size limit: its valid programs are this query's too
    uint32_t valid_cap = 0, rerun_cap = 0;
    size_t off_valid = 0, off_rerun = 0;  // element offsets into the valid / rerun buffers
    uint32_t n_valid = 0, n_rerun = 0, n_rerun_groups = 0;
    unsigned long long steps = 0, members = 0;
    unsigned long long evaluated = 0, evaluated_members = 0;   // instruction applications carried out where they differ from steps
    size_t out_first = 0;                 // first row of this query in the sorted/prog/cost buffers
};

int32_t run_batch(const p2_query* queries, int32_t n_queries, const double* msg_bytes, int32_t n_msg,
                  p2_program* out_prog, double* out_cost, int64_t cap, int64_t* out_offset, p2_stats* stats) {
    using namespace p2;
    if (!queries || n_queries < 1 || !out_offset) return fail(P2_EINVAL, "null or empty query list");
    if (n_msg < 0 || (n_msg > 0 && !msg_bytes)) return fail(P2_EINVAL, "bad message size list");
    if (n_msg > kMaxMsg) return fail(P2_EUNSUPPORTED, "more than 64 message sizes");
    if (cap < 0 || (cap > 0 && (!out_prog || (n_msg > 0 && !out_cost)))) return fail(P2_EINVAL, "bad output buffers");
    for (int m = 0; m < n_msg; ++m)
        if (!(msg_bytes[m] >= 0.0)) return fail(P2_EINVAL, "message size must be >= 0");
    hipStream_t stream = (queries[0].opt) ? (hipStream_t)queries[0].opt->hip_stream : nullptr;
    Ctx& C = g_ctx;
    CallScope scope(stream);

    // ---- plan every query on the host
    const auto t_begin = std::chrono::steady_clock::now();
    std::vector<QueryRun> runs(n_queries);
    {
        // (the bandwidth rows of the cost model are built later, while the GPU evaluates; large batches: the
        //  queries' plans are independent, a few host threads share them)
        std::vector<int32_t> plan_st((size_t)n_queries, P2_OK);
        std::vector<std::string> plan_err((size_t)n_queries);
        auto plan_one = [&](int i) {
            const p2_query& Q = queries[i];
            plan_st[i] = make_plan(Q.h, Q.axes, Q.n_axes, Q.placement, Q.reduce_axes, Q.n_reduce, Q.max_len, Q.opt, n_msg > 0,
                                   runs[i].plan, plan_err[i], false);
        };
        const unsigned hw = std::thread::hardware_concurrency();
        const int n_threads = n_queries >= 64 ? (int)std::min<unsigned>(std::max(hw, 1u), 8u) : 1;
        if (n_threads <= 1) {
            for (int i = 0; i < n_queries; ++i) plan_one(i);
        } else {
            std::atomic<int> next{0};
            auto work = [&]() { for (int i = next.fetch_add(1); i < n_queries; i = next.fetch_add(1)) plan_one(i); };
            std::vector<std::thread> pool;
            for (int t = 1; t < n_threads; ++t) pool.emplace_back(work);
            work();
            for (auto& th : pool) th.join();
        }
        for (int i = 0; i < n_queries; ++i)
            if (plan_st[i] != P2_OK) return fail(plan_st[i], "query " + std::to_string(i) + ": " + plan_err[i]);
    }
    for (int i = 0; i < n_queries; ++i) {
        const p2_query& Q = queries[i];
        runs[i].topk = Q.opt ? Q.opt->topk : 0;
        if (runs[i].topk < 0) return fail(P2_EINVAL, "topk < 0");
        if (runs[i].topk > kMaxTopK) return fail(P2_EUNSUPPORTED, "topk > 1024");
        if (runs[i].topk > 0 && n_msg == 0) return fail(P2_EINVAL, "topk needs at least one message size");
        const int want = Q.opt ? Q.opt->engine : P2_ENGINE_AUTO;
        const Plan& pl = runs[i].plan;
        const bool lit_ok = true;        // the literal engine falls back to a global state buffer
        const bool cmp_ok = compact_lanes(pl.R, pl.k) != 0;
        if (pl.hierarchy != P2_HIERARCHY_COLLAPSED) {
            // ranks inside a group and per-device goals are known to the literal engine only
            if (want != P2_ENGINE_LITERAL && want != P2_ENGINE_AUTO)
                return fail(P2_EUNSUPPORTED, "query " + std::to_string(i) + ": this synthesis hierarchy runs on the literal engine only");
            if (pl.n_candidates > (1ull << 30))
                return fail(P2_EUNSUPPORTED, "query " + std::to_string(i) + ": more than 2^30 candidates under this synthesis hierarchy");
            runs[i].engine = P2_ENGINE_LITERAL;
        } else if (want == P2_ENGINE_LITERAL) {
            if (!lit_ok) return fail(P2_EUNSUPPORTED, "state too large for the literal engine");
            runs[i].engine = P2_ENGINE_LITERAL;
        } else if (want == P2_ENGINE_FRONTIER || (want == P2_ENGINE_AUTO && pl.n_candidates > (1ull << 30))) {
            runs[i].engine = P2_ENGINE_COMPACT;      // its programs are costed like the compact engine's
            runs[i].frontier = true;
        } else if (want == P2_ENGINE_COMPACT || want == P2_ENGINE_AUTO || want == P2_ENGINE_SMALL || want == P2_ENGINE_SHARED) {
            // power-of-two patterns: the shared-prefix engine holds up to 64 devices, the per-candidate
            // small-group engine up to 32 devices and 32 chunks
            bool shared_ok = pl.R <= 64, regs_ok = pl.R <= 32 && pl.k <= 32;
            for (const Pattern& p : pl.patterns) {
                shared_ok = shared_ok && reg_shape_of(p.g, p.s, p.master, 6) >= 0;
                regs_ok = regs_ok && reg_shape_of(p.g, p.s, p.master, 5) >= 0;
            }
            if (want == P2_ENGINE_SMALL && !regs_ok)
                return fail(P2_EUNSUPPORTED, "the small-group engine needs R <= 32, k <= 32 and power-of-two patterns");
            if (want == P2_ENGINE_SHARED && !shared_ok)
                return fail(P2_EUNSUPPORTED, "the shared-prefix engine needs R <= 64 and power-of-two patterns");
            runs[i].regs = want == P2_ENGINE_SMALL;
            runs[i].shared = shared_ok && (want == P2_ENGINE_SHARED || want == P2_ENGINE_AUTO);
            if (cmp_ok) runs[i].engine = P2_ENGINE_COMPACT;
            else if (lit_ok && want == P2_ENGINE_AUTO) runs[i].engine = P2_ENGINE_LITERAL;
            else return fail(P2_EUNSUPPORTED, "state too large for the available engines");
        } else return fail(P2_EINVAL, "unknown engine");
        if ((size_t)pl.patterns.size() > (size_t)kMaxPatterns) return fail(P2_EUNSUPPORTED, "more than 64 patterns");
        // valid programs of these queries are costed one per wavefront, lanes as devices
        runs[i].wave_cost = runs[i].engine == P2_ENGINE_COMPACT && pl.R <= 64;
        for (const Pattern& p : pl.patterns) runs[i].wave_cost = runs[i].wave_cost && reg_shape_of(p.g, p.s, p.master, 6) >= 0;
    }

    // Validity depends on the reduction group, the chunks, the patterns and the alphabet only (not on the
    // links, nor on where the placement puts the group in the system): a query that equals an earlier one of
    // the batch in these is not evaluated again; it takes over the list of valid programs and the counts, and
    // only its costs are worked out, from its own bandwidth rows.  (The frontier engine does the same further
    // down.)  P2_FLAG_EVALUATE_EVERY_QUERY in any query's options switches this off for the batch.
    bool share_validity = true;
    for (int i = 0; i < n_queries; ++i)
        if (queries[i].opt && (queries[i].opt->flags & P2_FLAG_EVALUATE_EVERY_QUERY)) share_validity = false;
    {
        for (int i = 0; i < n_queries && share_validity; ++i) {
            QueryRun& r = runs[i];
            const Plan& pl = r.plan;
            if (r.frontier || pl.hierarchy != P2_HIERARCHY_COLLAPSED || pl.n_candidates == 0) continue;
            for (int j = 0; j < i && r.same_as < 0; ++j) {
                const QueryRun& c = runs[j];
                const Plan& o = c.plan;
                if (c.same_as >= 0 || c.frontier || o.hierarchy != P2_HIERARCHY_COLLAPSED || c.engine != r.engine || c.shared != r.shared ||
                    c.regs != r.regs || o.R != pl.R || o.k != pl.k || o.max_len != pl.max_len || o.alphabet != pl.alphabet ||
                    o.n_ops != pl.n_ops || o.patterns.size() != pl.patterns.size() || o.n_candidates != pl.n_candidates)
                    continue;
                bool eq = true;
                for (int t = 0; t < pl.n_ops && eq; ++t) eq = o.ops[t] == pl.ops[t];
                for (size_t t = 0; t < pl.patterns.size() && eq; ++t)
                    eq = o.patterns[t].g == pl.patterns[t].g && o.patterns[t].s == pl.patterns[t].s &&
                         o.patterns[t].master == pl.patterns[t].master && o.patterns[t].n_groups == pl.patterns[t].n_groups;
                if (eq) r.same_as = j;
            }
        }
    }
    g_prof.last.host_plan_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t_begin).count();
    // ---- lay out the table blob: queries, message sizes, bandwidth rows
    size_t off = 0;
    for (auto& r : runs) { r.off_query = off; off += sizeof(DevQuery); }      // one contiguous DevQuery array
    off = align_up(off, 256);
    // compact-engine queries are launched together, one launch per (chunk words, mask words) class
    struct Launch {
        int kind;                                   // 0 compact engine (state in LDS), 1 per-candidate small-group, 2 shared-prefix
        int kw, mw, max_R, max_k; std::vector<DevSegment> segs; unsigned blocks; size_t off_segs;
        std::vector<DevShare> shares; unsigned grid = 0; size_t off_shares = 0;     // shared-prefix kernel only
    };
    std::vector<Launch> launches;
    auto word_class = [](int bits) { int w = (bits + 31) / 32; return w <= 1 ? 1 : w <= 2 ? 2 : w <= 4 ? 4 : w <= 8 ? 8 : 16; };
    for (int i = 0; i < n_queries; ++i) {
        if (runs[i].engine != P2_ENGINE_COMPACT || runs[i].frontier || runs[i].same_as >= 0 || runs[i].plan.n_candidates == 0) continue;
        const Plan& pl = runs[i].plan;
        const int kind = runs[i].shared ? 2 : runs[i].regs ? 1 : 0;
        const int kw = kind == 1 ? 1 : word_class(pl.k), mw = kind == 1 ? 1 : word_class(pl.R);
        Launch* L = nullptr;
        for (auto& c : launches) if (c.kind == kind && c.kw == kw && c.mw == mw) L = &c;
        if (!L) { launches.push_back(Launch{kind, kw, mw, 0, 0, {}, 0u, 0, {}, 0u, 0}); L = &launches.back(); }
        L->max_R = std::max(L->max_R, pl.R);
        L->max_k = std::max(L->max_k, pl.k);
    }
    // stems (prefixes of len-2 instructions) of all shared-prefix queries of the batch
    unsigned long long shared_stems = 0;
    for (int i = 0; i < n_queries; ++i) {
        const Plan& pl = runs[i].plan;
        if (!runs[i].shared || runs[i].frontier || runs[i].same_as >= 0 || pl.n_candidates == 0 || pl.alphabet == 0) continue;
        for (int len = 2; len <= pl.max_len; ++len)
            shared_stems += (pl.base[len + 1] - pl.base[len]) / ((unsigned long long)pl.alphabet * (unsigned long long)pl.alphabet);
    }
    const unsigned long long shared_cut = shared_stems >= (1ull << 17) ? 1 : shared_stems >= (1ull << 15) ? 2 : 4;
    for (auto& L : launches) {
        const int lanes = L.kind != 0 ? 64 : compact_lanes(L.max_R, L.max_k);
        if (lanes == 0) return fail(P2_EUNSUPPORTED, "state too large for the compact engine");
        unsigned long long blocks = 0;
        for (int i = 0; i < n_queries; ++i) {
            const Plan& pl = runs[i].plan;
            if (runs[i].engine != P2_ENGINE_COMPACT || runs[i].frontier || runs[i].same_as >= 0 || pl.n_candidates == 0) continue;
            const int kind = runs[i].shared ? 2 : runs[i].regs ? 1 : 0;
            if (kind != L.kind || (kind == 1 ? 1 : word_class(pl.k)) != L.kw || (kind == 1 ? 1 : word_class(pl.R)) != L.mw) continue;
            for (int len = 1; len <= pl.max_len; ++len) {
                const unsigned long long count = pl.base[len + 1] - pl.base[len];
                DevSegment sg;
                sg.first_block = (uint32_t)blocks; sg.query = i; sg.len = len;
                sg.first_index = pl.base[len]; sg.count = count;
                if (L.kind == 2) {
                    // shared-prefix kernel: an item is a run of groups under one stem (the first len-2
                    // instructions).  With few stems a stem is cut into four items, which balances the load
                    // of the fixed grid; with many stems a whole stem is one item, so its state is worked out once
                    const unsigned long long I = (unsigned long long)pl.alphabet;
                    const unsigned long long per_item = len >= 2 ? (I + shared_cut - 1) / shared_cut : 1;
                    sg.iters = (int)per_item;
                    blocks += len >= 2 ? (count / (I * I)) * shared_cut : 1;     // (items past a short stem's groups are empty)
                } else {
                    const unsigned long long chunks = (count + lanes - 1) / lanes;
                    unsigned long long iters = (chunks + 4095) / 4096;
                    iters = std::min<unsigned long long>(std::max<unsigned long long>(iters, 1), 64);
                    sg.iters = (int)iters;
                    blocks += (chunks + iters - 1) / iters;
                }
                L.segs.push_back(sg);
                if (blocks > 0x7fffffffull) return fail(P2_EUNSUPPORTED, "too many candidates for one launch");
            }
        }
        L.blocks = (unsigned)blocks;
        L.off_segs = off;
        off += align_up(sizeof(DevSegment) * L.segs.size(), 256);
        if (L.kind == 2) {
            // divide a grid of about 8192 blocks (32 wavefronts per compute unit) among the queries by their items
            const unsigned long long target = 8192;
            for (size_t a = 0; a < L.segs.size();) {
                size_t b = a;
                while (b < L.segs.size() && L.segs[b].query == L.segs[a].query) ++b;
                DevShare shq;
                shq.first_item = L.segs[a].first_block;
                shq.n_items = (b < L.segs.size() ? L.segs[b].first_block : L.blocks) - shq.first_item;
                unsigned long long nb = (target * shq.n_items + L.blocks / 2) / std::max(1u, L.blocks);
                nb = std::min<unsigned long long>(std::max<unsigned long long>(nb, 1), std::max(1u, shq.n_items));
                shq.first_block = L.grid; shq.n_blocks = (uint32_t)nb;
                shq.query = L.segs[a].query; shq.first_seg = (int32_t)a; shq.n_segs = (int32_t)(b - a);
                shq.cut_log = shared_cut == 4 ? 2 : shared_cut == 2 ? 1 : 0;
                L.grid += (unsigned)nb;
                L.shares.push_back(shq);
                a = b;
            }
            L.off_shares = off;
            off += align_up(sizeof(DevShare) * L.shares.size(), 256);
        }
    }
    // Groups that the shared-prefix engine hands to the literal engine are found on the device, so that kernel
    // is queued right behind the evaluation: one launch per mask width, each with the list of its queries.
    struct AutoGroups { int cls = 0, max_R = 0, max_k = 0, class_cap = 64; std::vector<int32_t> qlist; size_t off = 0; };
    std::vector<AutoGroups> autos;
    for (int i = 0; i < n_queries; ++i) {
        QueryRun& r = runs[i];
        if (!r.shared || r.frontier || r.same_as >= 0 || r.plan.n_candidates == 0) continue;
        const int mw = r.plan.R <= 32 ? 1 : 2;
        const int cls = mw;
        AutoGroups* A = nullptr;
        for (auto& a : autos) if (a.cls == cls) A = &a;
        if (!A) { autos.emplace_back(); A = &autos.back(); A->cls = cls; }
        A->max_R = std::max(A->max_R, r.plan.R); A->max_k = std::max(A->max_k, r.plan.k);
        A->class_cap = std::min(A->class_cap, r.plan.max_row_classes);
        A->qlist.push_back(i);
        r.auto_groups = true;
    }
    for (auto& A : autos) { A.off = off; off += align_up(sizeof(int32_t) * A.qlist.size(), 256); }
    for (auto& r : runs) {
        if (r.plan.hierarchy == P2_HIERARCHY_COLLAPSED) continue;
        r.off_goal = off;
        off += align_up(sizeof(uint32_t) * (r.plan.goal.empty() ? 0 : (size_t)r.plan.R * literal_mask_words(r.plan.R)), 256);
        r.off_rank = off;
        size_t n_rank = 0;
        for (const Pattern& p : r.plan.patterns) n_rank += p.rank.size();
        off += align_up(sizeof(int32_t) * n_rank, 256);
    }
    const size_t off_msg = off;
    off += align_up(sizeof(double) * (size_t)std::max(n_msg, 1), 256);
    const size_t blob_bytes = off;
    // The bandwidth rows (cost model) live in buffers of their own: the rows, and per query a header (DevRows)
    // that the query descriptor points at.  They are built on the host after the evaluation kernels have been
    // queued and uploaded on a second stream, so both overlap with the evaluation; the call's stream waits
    // for the upload before its first cost kernel.
    bool rows_ready = false;
    P2_HIP(C.rows_hdr.ensure(sizeof(DevRows) * (size_t)std::max(n_queries, 1)));
    P2_HIP(C.h_rows_hdr.ensure(sizeof(DevRows) * (size_t)std::max(n_queries, 1)));
    if (!C.copy_stream) {
        P2_HIP(hipStreamCreateWithFlags(&C.copy_stream, hipStreamNonBlocking));
        P2_HIP(hipEventCreateWithFlags(&C.copy_done, hipEventDisableTiming));
        P2_HIP(hipEventCreateWithFlags(&C.front_go, hipEventDisableTiming));
    }
    auto build_and_upload_rows = [&]() -> int32_t {
        if (rows_ready) return P2_OK;
        size_t bytes = 0;
        // (large batches: the queries' tables are independent, a few host threads share them, for building and for packing)
        const unsigned hw = std::thread::hardware_concurrency();
        const int n_threads = n_queries >= 256 ? (int)std::min<unsigned>(std::max(hw, 1u), 16u) : n_queries >= 32 ? (int)std::min<unsigned>(std::max(hw, 1u), 8u) : 1;
        auto for_every_query = [&](const std::function<void(int)>& f) {
            if (n_threads <= 1) { for (int i = 0; i < n_queries; ++i) f(i); return; }
            std::atomic<int> next{0};
            auto work = [&]() { for (int i = next.fetch_add(1); i < n_queries; i = next.fetch_add(1)) f(i); };
            std::vector<std::thread> pool;
            for (int t = 1; t < n_threads; ++t) pool.emplace_back(work);
            work();
            for (auto& th : pool) th.join();
        };
        if (n_msg > 0) for_every_query([&](int i) { build_cost_tables(runs[i].plan); });    // without message sizes the tables stay empty
        for (auto& r : runs) {
            size_t n_rows = 0, n_ent = 0;
            for (const Pattern& p : r.plan.patterns) { n_rows += p.row_level.size(); n_ent += p.entries.size(); }
            r.off_rowptr = bytes; bytes += align_up(sizeof(int32_t) * (n_rows + 1), 16);
            r.off_rowlevel = bytes; bytes += align_up(sizeof(int32_t) * std::max<size_t>(n_rows, 1), 16);
            r.off_entries = bytes; bytes += align_up(sizeof(uint32_t) * std::max<size_t>(n_ent, 1), 256);
        }
        P2_HIP(C.rows.ensure(bytes));
        P2_HIP(C.h_rows.ensure(bytes));
        char* hr = static_cast<char*>(C.h_rows.p);
        char* dr = static_cast<char*>(C.rows.p);
        DevRows* hdr = static_cast<DevRows*>(C.h_rows_hdr.p);
        for_every_query([&](int i) {
            const QueryRun& r = runs[i];
            const Plan& pl = r.plan;
            int32_t* rp = reinterpret_cast<int32_t*>(hr + r.off_rowptr);
            int32_t* rl = reinterpret_cast<int32_t*>(hr + r.off_rowlevel);
            uint32_t* en = reinterpret_cast<uint32_t*>(hr + r.off_entries);
            DevRows& H = hdr[i];
            std::memset(&H, 0, sizeof H);
            int row = 0, ent = 0;
            rp[0] = 0;
            for (size_t pi = 0; pi < pl.patterns.size(); ++pi) {
                const Pattern& p = pl.patterns[pi];
                H.pat_begin[pi] = row;
                for (size_t t = 0; t < p.row_level.size(); ++t) {
                    uint32_t sum = 0;
                    for (int e = p.row_ptr[t]; e < p.row_ptr[t + 1]; ++e) { en[ent++] = p.entries[e]; sum += entry_cnt(p.entries[e]); }
                    rl[row] = p.row_level[t];
                    rp[++row] = ent;
                    H.level_max[pi][p.row_level[t]] = std::max(H.level_max[pi][p.row_level[t]], sum);
                }
            }
            for (size_t pi = pl.patterns.size(); pi <= (size_t)kMaxPatterns; ++pi) H.pat_begin[pi] = row;
            H.row_ptr = reinterpret_cast<const int32_t*>(dr + r.off_rowptr);
            H.row_level = reinterpret_cast<const int32_t*>(dr + r.off_rowlevel);
            H.entries = reinterpret_cast<const uint32_t*>(dr + r.off_entries);
        });
        rows_ready = true;
        P2_HIP(hipMemcpyAsync(C.rows.p, C.h_rows.p, bytes, hipMemcpyHostToDevice, C.copy_stream));
        P2_HIP(hipMemcpyAsync(C.rows_hdr.p, C.h_rows_hdr.p, sizeof(DevRows) * (size_t)n_queries, hipMemcpyHostToDevice, C.copy_stream));
        P2_HIP(hipEventRecord(C.copy_done, C.copy_stream));
        P2_HIP(hipStreamWaitEvent(stream, C.copy_done, 0));
        return P2_OK;
    };
    P2_HIP(C.blob.ensure(blob_bytes));
    P2_HIP(C.h_blob.ensure(blob_bytes));
    P2_HIP(C.counters.ensure(sizeof(DevCounters) * (size_t)n_queries));
    P2_HIP(C.h_counters.ensure(sizeof(DevCounters) * (size_t)n_queries));

    // valid / rerun list capacities (grown and retried if a query overflows them)
    auto layout_lists = [&]() {
        size_t v = 0, rr = 0;
        for (auto& r : runs) { r.off_valid = v; v += r.valid_cap; r.off_rerun = rr; rr += r.rerun_cap; }
        return std::make_pair(v, rr);
    };
    for (auto& r : runs) {
        const unsigned long long N = r.plan.n_candidates;
        r.valid_cap = (r.frontier || r.same_as >= 0) ? 0u : (uint32_t)std::min<unsigned long long>(N, 1u << 15);
        r.rerun_cap = (r.engine == P2_ENGINE_COMPACT && !r.frontier && r.same_as < 0) ? (uint32_t)std::min<unsigned long long>(N, 1u << 10) : 0u;
    }

    // global state buffer for literal evaluations whose state does not fit in LDS
    auto lit_scratch = [&](const Plan& pl, void** out) -> hipError_t {
        *out = nullptr;
        if (literal_lds_bytes(pl.R, pl.k) != 0) return hipSuccess;
        unsigned nb = 0;
        hipError_t e = C.lit_scratch.ensure(literal_scratch_bytes(pl.R, pl.k, &nb));
        *out = C.lit_scratch.p;
        return e;
    };
    // Segment tables for the kernels that serve many queries per launch.  Tables of one phase are
    // packed into C.post and uploaded with one copy; `PostLaunch` remembers where each one starts.
    struct PostLaunch { int cls = 0; int max_R = 0, max_k = 0; size_t lit_lds = 0; std::vector<DevPostSeg> segs; unsigned blocks = 0; size_t off = 0; };
    auto add_seg = [](std::vector<PostLaunch>& v, int cls, const Plan& pl, int query, uint32_t count, uint32_t per_block,
                      size_t in_off, size_t out_off) {
        PostLaunch* L = nullptr;
        for (auto& c : v) if (c.cls == cls) L = &c;
        if (!L) { v.emplace_back(); L = &v.back(); L->cls = cls; }
        L->max_R = std::max(L->max_R, pl.R); L->max_k = std::max(L->max_k, pl.k);
        L->lit_lds = std::max(L->lit_lds, literal_lds_bytes(pl.R, pl.k));     // what the literal kernels would need
        DevPostSeg sg;
        sg.first_block = L->blocks; sg.query = query; sg.count = count; sg.per_block = per_block;
        sg.in_off = in_off; sg.out_off = out_off;
        L->segs.push_back(sg);
        L->blocks += (count + per_block - 1) / per_block;
    };
    auto upload_segs = [&](std::vector<std::vector<PostLaunch>*> groups) -> hipError_t {
        size_t bytes = 0;
        for (auto* g : groups) for (auto& L : *g) { L.off = bytes; bytes += align_up(sizeof(DevPostSeg) * L.segs.size(), 256); }
        if (bytes == 0) return hipSuccess;
        hipError_t e = C.post.ensure(bytes);
        if (e != hipSuccess) return e;
        e = C.h_post.ensure(bytes);
        if (e != hipSuccess) return e;
        for (auto* g : groups) for (auto& L : *g)
            std::memcpy(static_cast<char*>(C.h_post.p) + L.off, L.segs.data(), sizeof(DevPostSeg) * L.segs.size());
        return hipMemcpyAsync(C.post.p, C.h_post.p, bytes, hipMemcpyHostToDevice, stream);
    };
    auto segs_of = [&](const PostLaunch& L) { return reinterpret_cast<const DevPostSeg*>(static_cast<char*>(C.post.p) + L.off); };
    auto mask_class = [](int R) { return R <= 32 ? 1 : R <= 64 ? 2 : R <= 128 ? 4 : R <= 256 ? 8 : 16; };
    char* hb = static_cast<char*>(C.h_blob.p);
    char* db = static_cast<char*>(C.blob.p);
    std::vector<char> done(n_queries, 0);
    for (int attempt = 0; attempt < 4; ++attempt) {
        auto tot = layout_lists();
        P2_HIP(C.valid.ensure(sizeof(unsigned long long) * std::max<size_t>(tot.first, 1)));
        P2_HIP(C.rerun.ensure(sizeof(unsigned long long) * std::max<size_t>(tot.second, 1)));
        std::memset(hb, 0, blob_bytes);
        for (int m = 0; m < n_msg; ++m) reinterpret_cast<double*>(hb + off_msg)[m] = msg_bytes[m];
        for (int i = 0; i < n_queries; ++i) {
            QueryRun& r = runs[i];
            const Plan& pl = r.plan;
            DevQuery* dq = reinterpret_cast<DevQuery*>(hb + r.off_query);
            dq->R = pl.R; dq->k = pl.k;
            dq->MW = (pl.R + 31) / 32; dq->KW = (pl.k + 31) / 32;
            dq->n_patterns = (int)pl.patterns.size(); dq->n_ops = pl.n_ops; dq->alphabet = pl.alphabet; dq->algo = pl.algo;
            dq->max_len = pl.max_len; dq->n_levels = pl.n; dq->n_msg = n_msg;
            dq->n_candidates = pl.n_candidates;
            for (int l = 0; l <= P2_MAX_LEN + 1; ++l) dq->base[l] = pl.base[l];
            for (int o = 0; o < pl.n_ops; ++o) dq->ops[o] = (uint8_t)pl.ops[o];
            dq->magic_alphabet = pl.alphabet <= 1 ? 0xffffffffu : (uint32_t)((1ull << 32) / (unsigned)pl.alphabet + 1ull);
            for (int d = 0; d < pl.alphabet; ++d)
                dq->instr_of_digit[d] = (uint16_t)(((d / pl.n_ops) << 3) | pl.ops[d % pl.n_ops]);
            for (int j = 0; j < pl.n; ++j) { dq->alpha[j] = pl.alpha[j]; dq->inv_bw[j] = 1.0 / pl.bw[j]; }
            for (size_t pi = 0; pi < pl.patterns.size(); ++pi) {
                const Pattern& p = pl.patterns[pi];
                DevPattern& dp = dq->pat[pi];
                dp.g = p.g; dp.s = p.s; dp.master = p.master; dp.n_groups = p.n_groups; dp.span_level = p.span;
                dp.reg_shape = reg_shape_of(p.g, p.s, p.master, 5);
                dp.rank_off = 0; dp.pad1 = 0;
            }
            dq->goal_mask = nullptr; dq->rank_tbl = nullptr;
            if (pl.hierarchy != P2_HIERARCHY_COLLAPSED) {
                if (!pl.goal.empty()) {
                    // the plan's rows are ceil(R/32) words long, the kernels' a power of two
                    const int mw = (pl.R + 31) / 32, mwd = literal_mask_words(pl.R);
                    uint32_t* goal = reinterpret_cast<uint32_t*>(hb + r.off_goal);
                    for (int d = 0; d < pl.R; ++d)
                        for (int w = 0; w < mwd; ++w) goal[(size_t)d * mwd + w] = w < mw ? pl.goal[(size_t)d * mw + w] : 0u;
                    dq->goal_mask = reinterpret_cast<const uint32_t*>(db + r.off_goal);
                }
                int32_t* ranks = reinterpret_cast<int32_t*>(hb + r.off_rank);
                int32_t at = 0;
                for (size_t pi = 0; pi < pl.patterns.size(); ++pi) {
                    const Pattern& p = pl.patterns[pi];
                    if (p.rank.empty()) continue;
                    std::memcpy(ranks + at, p.rank.data(), sizeof(int32_t) * p.rank.size());
                    dq->pat[pi].rank_off = at + 1;
                    at += (int32_t)p.rank.size();
                }
                dq->rank_tbl = reinterpret_cast<const int32_t*>(db + r.off_rank);
            }
            dq->rows = static_cast<const DevRows*>(C.rows_hdr.p) + i;
            dq->reg_sum_part = 0;
            for (size_t pi = 0; pi < pl.patterns.size(); ++pi) {
                const Pattern& p = pl.patterns[pi];
                const int shape = reg_shape_of(p.g, p.s, p.master, 6);
                unsigned long long part = pl.R >= 64 ? ~0ull : ((1ull << pl.R) - 1ull);
                if (p.master) {
                    unsigned long long every = 0;             // bit d set iff d % s == 0
                    for (int d = 0; d < 64; d += p.s) every |= 1ull << d;
                    part &= every;
                }
                dq->reg_shape[pi] = (shape < 0 ? 0u : (uint32_t)shape) | ((uint32_t)(p.n_groups * p.g) << 16);
                dq->reg_part[pi] = part;
                dq->reg_sum_part += (uint32_t)(p.n_groups * p.g) * (uint32_t)pl.n_ops;
            }
            dq->msg_bytes = reinterpret_cast<const double*>(db + off_msg);
            dq->valid_idx = static_cast<unsigned long long*>(C.valid.p) + r.off_valid;
            dq->rerun_idx = static_cast<unsigned long long*>(C.rerun.p) + r.off_rerun;
            dq->valid_cap = r.valid_cap; dq->rerun_cap = r.rerun_cap;
            dq->counters = static_cast<DevCounters*>(C.counters.p) + i;
        }
        for (auto& L : launches)
        {
            std::memcpy(hb + L.off_segs, L.segs.data(), sizeof(DevSegment) * L.segs.size());
            if (!L.shares.empty()) std::memcpy(hb + L.off_shares, L.shares.data(), sizeof(DevShare) * L.shares.size());
        }
        for (auto& A : autos) std::memcpy(hb + A.off, A.qlist.data(), sizeof(int32_t) * A.qlist.size());
        P2_HIP(hipMemcpyAsync(db, hb, blob_bytes, hipMemcpyHostToDevice, stream));
        P2_HIP(hipMemsetAsync(C.counters.p, 0, sizeof(DevCounters) * (size_t)n_queries, stream));
        // ---- evaluate every candidate of every query
        int eval_launches = 0;
        if (g_prof.on) P2_HIP(hipEventRecord(g_prof.ev[0], stream));
        for (auto& L : launches) {
            ++eval_launches;
            if (L.kind == 2)
                P2_HIP(launch_eval_shared(reinterpret_cast<const DevQuery*>(db), reinterpret_cast<const DevSegment*>(db + L.off_segs),
                                          (int)L.segs.size(), reinterpret_cast<const DevShare*>(db + L.off_shares),
                                          (int)L.shares.size(), L.grid, L.max_R, L.max_k, stream));
            else if (L.kind == 1)
                P2_HIP(launch_eval_regs(reinterpret_cast<const DevQuery*>(db), reinterpret_cast<const DevSegment*>(db + L.off_segs),
                                        (int)L.segs.size(), L.blocks, stream));
            else
                P2_HIP(launch_eval_compact(reinterpret_cast<const DevQuery*>(db), reinterpret_cast<const DevSegment*>(db + L.off_segs),
                                           (int)L.segs.size(), L.blocks, L.max_R, L.max_k, stream));
        }
        for (int i = 0; i < n_queries; ++i) {
            QueryRun& r = runs[i];
            const DevQuery* dq = reinterpret_cast<const DevQuery*>(db + r.off_query);
            if (r.engine == P2_ENGINE_LITERAL && r.same_as < 0 && r.plan.n_candidates > 0) {
                ++eval_launches;
                void* gs = nullptr;
                P2_HIP(lit_scratch(r.plan, &gs));
                P2_HIP(launch_eval_literal(dq, r.plan.R, r.plan.k, 0ull, r.plan.n_candidates, nullptr, nullptr, gs, stream));
            }
        }
        if (g_prof.on) { P2_HIP(hipEventRecord(g_prof.ev[1], stream)); g_prof.last.eval_launches = eval_launches; }
        for (auto& A : autos) {
            unsigned nb = 0;
            P2_HIP(C.lit_scratch.ensure(literal_group_scratch_bytes(A.max_R, A.max_k, &nb)));
            P2_HIP(launch_eval_literal_groups_auto(reinterpret_cast<const DevQuery*>(db), reinterpret_cast<const int32_t*>(db + A.off),
                                                   (int)A.qlist.size(), A.max_R, A.max_k, C.lit_scratch.p, A.class_cap, stream));
        }
        // while the GPU evaluates: the cost model's tables (first attempt only)
        {
            const int32_t rc = build_and_upload_rows();
            if (rc != P2_OK) return rc;
        }
        P2_HIP(launch_copy_out(C.h_counters.p, C.counters.p, sizeof(DevCounters) * (size_t)n_queries, stream));
        P2_HIP(hipStreamSynchronize(stream));
        bool again = false;
        const DevCounters* hc = static_cast<const DevCounters*>(C.h_counters.p);
        // candidates whose state the compact engine could not hold go through the literal engine:
        // one launch per mask-width class for the states that fit in LDS, one per query otherwise
        bool reran = false;
        std::vector<PostLaunch> rerun_launches;
        for (int i = 0; i < n_queries; ++i) {
            QueryRun& r = runs[i];
            if (hc[i].n_rerun == 0 || hc[i].n_rerun > r.rerun_cap || r.auto_groups) continue;
            reran = true;
            if (literal_lds_bytes(r.plan.R, r.plan.k) != 0) {
                add_seg(rerun_launches, mask_class(r.plan.R), r.plan, i, hc[i].n_rerun, 1, r.off_rerun, 0);
            } else {
                void* gs = nullptr;
                P2_HIP(lit_scratch(r.plan, &gs));
                P2_HIP(launch_eval_literal(reinterpret_cast<const DevQuery*>(db + r.off_query), r.plan.R, r.plan.k, 0ull,
                                           hc[i].n_rerun, static_cast<unsigned long long*>(C.rerun.p) + r.off_rerun, nullptr, gs, stream));
            }
        }
        if (!rerun_launches.empty()) {
            P2_HIP(upload_segs({&rerun_launches}));
            for (auto& L : rerun_launches)
                P2_HIP(launch_eval_literal_list(reinterpret_cast<const DevQuery*>(db), segs_of(L), (int)L.segs.size(), L.blocks,
                                                L.max_R, L.lit_lds, static_cast<unsigned long long*>(C.rerun.p), stream));
        }
        if (reran) {
            P2_HIP(launch_copy_out(C.h_counters.p, C.counters.p, sizeof(DevCounters) * (size_t)n_queries, stream));
            P2_HIP(hipStreamSynchronize(stream));
        }
        for (int i = 0; i < n_queries; ++i) {
            QueryRun& r = runs[i];
            r.n_valid = hc[i].n_valid; r.n_rerun = hc[i].n_rerun; r.n_rerun_groups = hc[i].n_rerun_groups;
            r.steps = 0; r.members = 0;
            for (int t = 0; t < kCounterStripes; ++t) { r.steps += hc[i].steps[t]; r.members += hc[i].members[t]; }
            r.evaluated = 0; r.evaluated_members = 0;
            for (int t = 0; t < kCounterStripes; ++t) { r.evaluated += hc[i].evaluated[t]; r.evaluated_members += hc[i].evaluated_members[t]; }
            if (r.same_as >= 0) {                       // (the earlier query's figures; nothing was carried out for this one)
                const QueryRun& o = runs[r.same_as];
                r.n_valid = o.n_valid; r.n_rerun = o.n_rerun; r.n_rerun_groups = o.n_rerun_groups;
                r.steps = o.steps; r.members = o.members; r.off_valid = o.off_valid;
                continue;
            }
            if (r.n_valid > r.valid_cap || r.n_rerun > r.rerun_cap) {
                again = true;
                r.valid_cap = std::max(r.valid_cap, r.n_valid);
                r.rerun_cap = std::max(r.rerun_cap, r.n_rerun);
            }
        }
        if (!again) break;
        if (attempt == 3) return fail(P2_EDEVICE, "result lists kept overflowing");
    }

    // ---- frontier queries: enumeration by program size (Sec. 3.5).  Queries that agree in everything validity
    //      depends on form one enumeration; its prefixes carry the running cost sums of every member query.
    struct Enum {
        int leader = -1, id = 0;
        std::vector<int32_t> members;
        size_t off_valid = 0, off_share = 0;     // element offsets into f_rank, f_share
        uint32_t n_valid = 0, n_goal_literal = 0;
    };
    std::vector<Enum> enums;
    for (int i = 0; i < n_queries; ++i) {
        QueryRun& r = runs[i];
        if (!r.frontier) continue;
        const Plan& pl = r.plan;
        r.n_valid = 0; r.n_rerun = 0; r.steps = 0; r.members = 0;
        if (pl.n_candidates == 0) continue;
        int found = -1;
        for (size_t e = 0; e < enums.size() && found < 0 && share_validity; ++e) {
            const Plan& o = runs[enums[e].leader].plan;
            if (o.R != pl.R || o.k != pl.k || o.max_len != pl.max_len || o.alphabet != pl.alphabet || o.n_ops != pl.n_ops ||
                o.patterns.size() != pl.patterns.size() || o.n_candidates != pl.n_candidates ||
                o.max_row_classes != pl.max_row_classes || o.frontier_pairs != pl.frontier_pairs)
                continue;
            bool eq = true;
            for (int t = 0; t < pl.n_ops && eq; ++t) eq = o.ops[t] == pl.ops[t];
            for (size_t t = 0; t < pl.patterns.size() && eq; ++t)
                eq = o.patterns[t].g == pl.patterns[t].g && o.patterns[t].s == pl.patterns[t].s &&
                     o.patterns[t].master == pl.patterns[t].master && o.patterns[t].n_groups == pl.patterns[t].n_groups;
            if (eq) found = (int)e;
        }
        if (found < 0) { enums.emplace_back(); found = (int)enums.size() - 1; enums[found].leader = i; }
        r.enum_id = found;
        r.share_pos = (int)enums[found].members.size();
        enums[found].members.push_back(i);
    }
    if (!enums.empty()) {
        size_t n_share_all = 0;
        for (auto& E : enums) { E.off_share = n_share_all; n_share_all += E.members.size(); }
        P2_HIP(C.f_share.ensure(sizeof(int32_t) * n_share_all));
        P2_HIP(C.h_fshare.ensure(sizeof(int32_t) * n_share_all));
        for (auto& E : enums) std::memcpy(static_cast<int32_t*>(C.h_fshare.p) + E.off_share, E.members.data(), sizeof(int32_t) * E.members.size());
        P2_HIP(hipMemcpyAsync(C.f_share.p, C.h_fshare.p, sizeof(int32_t) * n_share_all, hipMemcpyHostToDevice, stream));
    }
    // ---- the enumerations, up to kFrontSlots of them side by side (a host thread and a stream each); they start
    //      once the call's stream has got here, and the call's stream goes on when they are all through
    auto run_enum = [&](Enum& E, FrontSlot& S) -> int32_t {
        const int i = E.leader;
        DevBuf& EV = C.f_evalid[E.id];
        DevBuf& EG = C.f_egsums[E.id];
        QueryRun& r = runs[i];
        const Plan& pl = r.plan;
        const int n_share = (int)E.members.size();
        const size_t sum_doubles = n_msg > 0 ? (size_t)2 * n_share : 0;      // per prefix / per goal
        const DevQuery* dq = reinterpret_cast<const DevQuery*>(db + r.off_query);
        const size_t sw = frontier_state_words(pl.R, pl.k);
        // words of a device's (chunk set, mask) pair, and the devices that the alphabet's patterns visit per prefix
        const double pair_words = (double)((pl.k + 31) / 32 + (pl.R + 31) / 32);
        double pattern_members = 0.0;
        for (const auto& pt : pl.patterns) pattern_members += (double)pt.g * pt.n_groups;
        // state pairs per device: 2 where two planes fit in LDS; the option can lower it (1: as the compact form;
        // 4: no pair states at all, every prefix on the literal list) or, with 3, have every two-pair prefix
        // classified by the literal kernels (the path of prefixes whose groups are not aligned)
        const int fp = pl.frontier_pairs;
        const int max_pairs = fp == P2_FRONTIER_PAIRS_NONE ? 0 : fp == P2_FRONTIER_PAIRS_ONE ? 1 : frontier_max_pairs(pl.R, pl.k);
        P2_HIP(S.f_ctr.ensure(sizeof(FrontCounters)));
        P2_HIP(S.h_fctr.ensure(sizeof(FrontCounters)));
        FrontCounters* dctr = static_cast<FrontCounters*>(S.f_ctr.p);
        const FrontCounters* hctr = static_cast<const FrontCounters*>(S.h_fctr.p);
        P2_HIP(hipMemsetAsync(dctr, 0, sizeof(FrontCounters), S.stream));
        int cur = 0;
        P2_HIP(S.f_entries[cur].ensure(sizeof(FrontEntry)));
        P2_HIP(S.f_states[cur].ensure(sw * 4));
        P2_HIP(S.f_sums[cur].ensure(std::max<size_t>(sum_doubles, 1) * 8));
        P2_HIP(S.f_sid[cur].ensure(sizeof(uint32_t)));
        P2_HIP(S.f_literal[cur].ensure(sizeof(FrontEntry)));
        // A level: two lists of states (one pair per device; up to two) with n_s entries, of which the distinct ones
        // are judged; two lists of prefixes (n_c, n_c2 entries), each prefix with the index of its state; the
        // literal list (n_l prefixes that are judged from their instructions).
        uint32_t n_s[2] = {0, 0}, n_c = 0, n_c2 = 0, n_l = 0;
        bool grouped[2] = {false, false};            // the state list has been searched for equal states
        if (max_pairs >= 1) {
            P2_HIP(launch_front_init(dq, (uint32_t)i, pl.R, pl.k, static_cast<FrontEntry*>(S.f_entries[cur].p),
                                     static_cast<uint32_t*>(S.f_states[cur].p), static_cast<double*>(S.f_sums[cur].p),
                                     static_cast<uint32_t*>(S.f_sid[cur].p), (int)sum_doubles / 2, S.stream));
            n_c = 1; n_s[0] = 1;
        } else {
            const FrontEntry root{(uint32_t)i, 0u, 0ull};
            P2_HIP(hipMemcpyAsync(S.f_literal[cur].p, &root, sizeof root, hipMemcpyHostToDevice, S.stream));
            P2_HIP(hipStreamSynchronize(S.stream));
            n_l = 1;
        }
        void* gs = nullptr;
        const int handover = fp == P2_FRONTIER_PAIRS_TWO_HANDOVER ? 1 : 0;
        bool ctr_clean = true;                       // (all of the counters were cleared above)
        for (int len = 0; len < pl.max_len && (n_c > 0 || n_c2 > 0 || n_l > 0); ++len) {
            const int keep = len + 1 < pl.max_len ? 1 : 0;
            size_t cap_c = std::max<size_t>(1024, ((size_t)n_c + n_c2) * pl.alphabet / 8);
            size_t cap_l = std::max<size_t>(1024, ((size_t)n_l + n_c2 / 8) * pl.alphabet / 2);
            uint32_t n_surv_l_first = 0;
            P2_HIP(S.f_unknown.ensure(std::max<size_t>(n_c2, 1) * sizeof(FrontEntry)));
            const DevBuf* list_states[2] = {&S.f_states[cur], &S.f_states2[cur]};
            // ---- one state of every group of equal states is judged against the alphabet, into a row of codes
            for (int li = 0; li < 2; ++li) {
                if (n_s[li] == 0) continue;
                P2_HIP(S.f_codes[li].ensure((size_t)n_s[li] * front_code_stride(pl.alphabet)));
                P2_HIP(S.f_unk[li].ensure(n_s[li]));
                P2_HIP(S.f_rowcnt[li].ensure((size_t)n_s[li] * sizeof(unsigned long long)));
            }
            // The literal prefixes of the level.  (On a second stream of the slot they would overlap with the pair states'
            // kernels only if that stream had a hardware queue to itself, which it would take from another slot.)
            auto literal_prefixes = [&]() -> int32_t {
                if (n_l == 0) return P2_OK;
                P2_HIP(S.f_surv_literal.ensure(cap_l * sizeof(FrontSurvivor)));
                P2_HIP(S.lit_scratch.ensure(front_literal_scratch_bytes(pl.R, pl.k, std::max(n_l, n_c2))));
                gs = S.lit_scratch.p;
                P2_HIP(S.spans.begin(SpanRec::kLiteral, S.stream));
                P2_HIP(launch_front_classify_literal(dq, pl.R, pl.k, static_cast<const FrontEntry*>(S.f_literal[cur].p), n_l, len, keep ? 0 : 1,
                                                     static_cast<FrontSurvivor*>(S.f_surv_literal.p), (uint32_t)cap_l, dctr, gs,
                                                     pl.max_row_classes, S.stream));
                P2_HIP(S.spans.end(S.stream));
                return P2_OK;
            };
            // (the kernel that built the last level's children has cleared the counters of a level's first half; the
            //  kernel that brings them to the host clears those of its second half)
            if (!ctr_clean) P2_HIP(hipMemsetAsync(dctr, 0, offsetof(FrontCounters, steps), S.stream));
            ctr_clean = false;
            { const int32_t rc = literal_prefixes(); if (rc != P2_OK) return rc; }
            // At the last level only goals count: a filter first leaves the classification the few states from which an
            // instruction can still end at the goal.
            const uint32_t* cls_list[2]; const uint32_t* cls_n[2];
            for (int li = 0; li < 2; ++li) {
                cls_list[li] = grouped[li] ? static_cast<const uint32_t*>(S.f_replist[li].p) : nullptr;
                cls_n[li] = grouped[li] ? &dctr->n_reps[li] : nullptr;
            }
            if (!keep && n_s[0] + n_s[1] > 0) {
                P2_HIP(S.spans.begin(SpanRec::kGroup, S.stream));
                for (int li = 0; li < 2; ++li) {
                    if (n_s[li] == 0) continue;
                    P2_HIP(S.f_walk[li].ensure((size_t)n_s[li] * sizeof(uint32_t)));
                    P2_HIP(launch_front_goal_filter(dq, pl.R, pl.k, static_cast<const uint32_t*>(list_states[li]->p), n_s[li], cls_list[li],
                                                    cls_n[li], li + 1, static_cast<uint8_t*>(S.f_codes[li].p), static_cast<unsigned long long*>(S.f_rowcnt[li].p),
                                                    static_cast<uint8_t*>(S.f_unk[li].p), static_cast<uint32_t*>(S.f_walk[li].p),
                                                    &dctr->n_walk[li], S.stream));
                    cls_list[li] = static_cast<const uint32_t*>(S.f_walk[li].p);
                    cls_n[li] = &dctr->n_walk[li];
                }
                P2_HIP(S.spans.end(S.stream));
            }
            if (n_s[0] + n_s[1] > 0) P2_HIP(S.spans.begin(SpanRec::kClassify, S.stream, (n_s[0] > 0) + (n_s[1] > 0)));
            for (int li = 0; li < 2; ++li)
                P2_HIP(launch_front_classify(dq, pl.R, pl.k, static_cast<const uint32_t*>(list_states[li]->p), n_s[li], cls_list[li],
                                             cls_n[li], li + 1, max_pairs, keep ? 0 : 1, (li == 1 && handover) ? 0 : 1,
                                             static_cast<uint8_t*>(S.f_codes[li].p), static_cast<unsigned long long*>(S.f_rowcnt[li].p),
                                             static_cast<uint8_t*>(S.f_unk[li].p), dctr, S.stream));
            if (n_s[0] + n_s[1] > 0) P2_HIP(S.spans.end(S.stream));
            uint32_t walked_planes = 0, kids[3] = {0u, 0u, 0u};
            for (int attempt = 0;; ++attempt) {     // list the survivors of the prefixes; repeat with larger lists if they overflow
                P2_HIP(S.f_surv.ensure(cap_c * sizeof(FrontSurvivor)));
                if (attempt > 0) {
                    P2_HIP(hipMemsetAsync(dctr, 0, offsetof(FrontCounters, steps), S.stream));
                    // (the classification is not repeated: what it counted goes back in)
                    P2_HIP(hipMemcpyAsync(&dctr->t_count[0], kids, sizeof kids, hipMemcpyHostToDevice, S.stream));
                    const int32_t rc = literal_prefixes();
                    if (rc != P2_OK) return rc;
                }
                if (n_c + n_c2 > 0) P2_HIP(S.spans.begin(SpanRec::kGroup, S.stream));
                P2_HIP(launch_front_expand(dq, static_cast<const FrontEntry*>(S.f_entries[cur].p), n_c,
                                           static_cast<const uint32_t*>(S.f_sid[cur].p),
                                           static_cast<const uint8_t*>(S.f_codes[0].p), static_cast<const unsigned long long*>(S.f_rowcnt[0].p),
                                           static_cast<const uint8_t*>(S.f_unk[0].p), 1, 0,
                                           static_cast<FrontSurvivor*>(S.f_surv.p), (uint32_t)cap_c, nullptr, dctr, S.stream));
                P2_HIP(launch_front_expand(dq, static_cast<const FrontEntry*>(S.f_entries2[cur].p), n_c2,
                                           static_cast<const uint32_t*>(S.f_sid2[cur].p),
                                           static_cast<const uint8_t*>(S.f_codes[1].p), static_cast<const unsigned long long*>(S.f_rowcnt[1].p),
                                           static_cast<const uint8_t*>(S.f_unk[1].p), 2, handover,
                                           static_cast<FrontSurvivor*>(S.f_surv.p), (uint32_t)cap_c,
                                           static_cast<FrontEntry*>(S.f_unknown.p), dctr, S.stream));
                // (how many children the judged states have, by kind, the classification has counted)
                if (n_c + n_c2 > 0) P2_HIP(S.spans.end(S.stream));
                P2_HIP(launch_front_counters_out(static_cast<FrontCounters*>(S.h_fctr.p), dctr, S.stream));
                P2_HIP(hipStreamSynchronize(S.stream));
                if (attempt == 0) {                  // (a repeat clears the level's counters)
                    walked_planes = hctr->n_walked_planes;
                    for (int kd = 0; kd < 3; ++kd) kids[kd] = hctr->t_count[kd];
                }
                n_surv_l_first = hctr->n_surv_literal;
                if (hctr->n_unknown > 0 && hctr->n_surv_literal <= cap_l) {
                    // two-pair prefixes that this form could not judge: the literal kernels classify them from their
                    // instructions; their survivors follow those of the literal list
                    const uint32_t n_u = hctr->n_unknown;
                    P2_HIP(hipMemsetAsync(&dctr->n_overflow, 0, sizeof(uint32_t), S.stream));
                    P2_HIP(S.lit_scratch.ensure(front_literal_scratch_bytes(pl.R, pl.k, std::max(std::max(n_l, n_c2), n_u))));
                    gs = S.lit_scratch.p;
                    P2_HIP(S.spans.begin(SpanRec::kLiteral, S.stream));
                    P2_HIP(launch_front_classify_literal(dq, pl.R, pl.k, static_cast<const FrontEntry*>(S.f_unknown.p), n_u, len, keep ? 0 : 1,
                                                         static_cast<FrontSurvivor*>(S.f_surv_literal.p), (uint32_t)cap_l, dctr, gs,
                                                         pl.max_row_classes, S.stream));
                    P2_HIP(S.spans.end(S.stream));
                    P2_HIP(launch_front_counters_out(static_cast<FrontCounters*>(S.h_fctr.p), dctr, S.stream));
                    P2_HIP(hipStreamSynchronize(S.stream));
                }
                if ((uint32_t)hctr->surv_goal <= cap_c && hctr->n_surv_literal <= cap_l) break;
                // the repeated listing counts its steps again: take them back
                cap_c = std::max<size_t>(cap_c, (uint32_t)hctr->surv_goal); cap_l = std::max<size_t>(cap_l, (size_t)hctr->n_surv_literal * 2);
                FrontCounters fix = *hctr;
                fix.steps = r.steps; fix.members = r.members;
                P2_HIP(hipMemcpyAsync(dctr, &fix, sizeof(FrontCounters), hipMemcpyHostToDevice, S.stream));
                P2_HIP(hipStreamSynchronize(S.stream));
            }
            {   // what the classification launches of this level worked on
                const double j1 = grouped[0] ? (double)hctr->n_reps[0] : (double)n_s[0], j2 = grouped[1] ? (double)hctr->n_reps[1] : (double)n_s[1];
                // (at the last level only the states from which an instruction can still end at the goal are walked)
                const double planes = keep ? j1 + 2.0 * j2 : (double)walked_planes;
                S.prof_entries += (double)n_c + n_c2;
                S.prof_prefixes += j1 + j2;
                S.prof_state_bytes += planes * pl.R * pair_words * 4.0;
                S.prof_lane_ops += planes * pattern_members * pair_words * 4.0;
            }
            const uint32_t n_surv = (uint32_t)hctr->surv_goal, n_surv_l = hctr->n_surv_literal;
            const uint32_t n_goal_pair = (uint32_t)(hctr->surv_goal >> 32), n_goal_lit = hctr->n_goal, n_goal = n_goal_pair + n_goal_lit;
            const uint32_t n_prefix = (uint32_t)hctr->pref_pref2, n_prefix2 = (uint32_t)(hctr->pref_pref2 >> 32), n_plit = hctr->n_prefix_literal;
            const uint32_t t1 = hctr->t_count[0], t2 = hctr->t_count[1], tg = hctr->t_count[2], n_ss = t1 + t2 + tg;
            r.steps = hctr->steps; r.members = hctr->members;
            r.n_rerun += n_plit + hctr->n_unknown;
            E.n_goal_literal += n_goal_lit;
            P2_HIP(grow_keep(EV, ((size_t)E.n_valid + n_goal + 1) * sizeof(unsigned long long), (size_t)E.n_valid * sizeof(unsigned long long), S.stream));
            P2_HIP(grow_keep(EG, (((size_t)E.n_valid + n_goal) * sum_doubles + 1) * sizeof(double), (size_t)E.n_valid * sum_doubles * sizeof(double), S.stream));
            const int nxt = cur ^ 1;
            // the next level's prefixes ...
            P2_HIP(S.f_entries[nxt].ensure(std::max<size_t>(n_prefix, 1) * sizeof(FrontEntry)));
            P2_HIP(S.f_sums[nxt].ensure(std::max<size_t>((size_t)n_prefix * sum_doubles, 1) * 8));
            P2_HIP(S.f_sid[nxt].ensure(std::max<size_t>(n_prefix, 1) * sizeof(uint32_t)));
            P2_HIP(S.f_entries2[nxt].ensure(std::max<size_t>(n_prefix2, 1) * sizeof(FrontEntry)));
            P2_HIP(S.f_sums2[nxt].ensure(std::max<size_t>((size_t)n_prefix2 * sum_doubles, 1) * 8));
            P2_HIP(S.f_sid2[nxt].ensure(std::max<size_t>(n_prefix2, 1) * sizeof(uint32_t)));
            P2_HIP(S.f_literal[nxt].ensure(std::max<size_t>(n_plit, 1) * sizeof(FrontEntry)));
            // ... and states: a child per (judged state, valid instruction), its hash, what the step
            // adds to the cost sums; where a state's children are
            P2_HIP(S.f_states[nxt].ensure(std::max<size_t>(t1, 1) * sw * 4));
            P2_HIP(S.f_states2[nxt].ensure(std::max<size_t>(t2, 1) * sw * 8));
            P2_HIP(S.f_hash[nxt].ensure(std::max<size_t>(t1, 1) * sizeof(unsigned long long)));
            P2_HIP(S.f_hash2[nxt].ensure(std::max<size_t>(t2, 1) * sizeof(unsigned long long)));
            P2_HIP(S.f_delta[0].ensure(std::max<size_t>((size_t)t1 * sum_doubles, 1) * 8));
            P2_HIP(S.f_delta[1].ensure(std::max<size_t>((size_t)t2 * sum_doubles, 1) * 8));
            P2_HIP(S.f_delta[2].ensure(std::max<size_t>((size_t)tg * sum_doubles, 1) * 8));
            P2_HIP(S.f_ssurv.ensure(std::max<size_t>(n_ss, 1) * sizeof(FrontSurvivor)));
            for (int li = 0; li < 2; ++li) P2_HIP(S.f_childof[li].ensure(std::max<size_t>((size_t)n_s[li] * pl.alphabet, 1) * sizeof(uint32_t)));
            if (n_ss > 0) P2_HIP(S.spans.begin(SpanRec::kGroup, S.stream));
            for (int li = 0; li < 2; ++li) {
                if (li == 1 && handover) continue;
                P2_HIP(launch_front_children(dq, n_s[li], grouped[li] ? static_cast<const uint32_t*>(S.f_replist[li].p) : nullptr,
                                             grouped[li] ? &dctr->n_reps[li] : nullptr, static_cast<const uint8_t*>(S.f_codes[li].p),
                                             static_cast<const uint8_t*>(S.f_unk[li].p), li + 1, keep, 1, static_cast<uint32_t*>(S.f_childof[li].p),
                                             static_cast<FrontSurvivor*>(S.f_ssurv.p), dctr, S.stream));
            }
            if (n_ss > 0) P2_HIP(S.spans.end(S.stream));
            FrontLevel lv;
            std::memset(&lv, 0, sizeof lv);
            lv.query = (uint32_t)i;
            lv.share = static_cast<const int32_t*>(C.f_share.p) + E.off_share;
            lv.n_share = n_share; lv.n_msg = n_msg;
            lv.states1 = static_cast<const uint32_t*>(S.f_states[cur].p); lv.states2 = static_cast<const uint32_t*>(S.f_states2[cur].p);
            lv.surv = static_cast<const FrontSurvivor*>(S.f_ssurv.p); lv.n_surv = n_ss;
            lv.lds_planes = (n_s[1] > 0 || t2 > 0) ? 2 : 1;
            lv.n_reps = &dctr->n_reps[0];
            lv.ctr = dctr;
            ctr_clean = n_ss > 0;                    // (the kernel is launched only if there are children)
            lv.next_states1 = static_cast<uint32_t*>(S.f_states[nxt].p); lv.next_states2 = static_cast<uint32_t*>(S.f_states2[nxt].p);
            lv.next_hash1 = static_cast<unsigned long long*>(S.f_hash[nxt].p); lv.next_hash2 = static_cast<unsigned long long*>(S.f_hash2[nxt].p);
            lv.delta1 = static_cast<double*>(S.f_delta[0].p); lv.delta2 = static_cast<double*>(S.f_delta[1].p);
            lv.delta_goal = static_cast<double*>(S.f_delta[2].p);
            if (n_ss > 0) P2_HIP(S.spans.begin(SpanRec::kMaterialize, S.stream));
            P2_HIP(launch_front_materialize(reinterpret_cast<const DevQuery*>(db), pl.R, pl.k, lv, S.stream));
            if (n_ss > 0) {
                P2_HIP(S.spans.end(S.stream));
                // every child reads its parent (one plane at least) and is written: state and what the step costs
                S.prof_children += (double)n_ss;
                S.prof_mat_bytes += ((double)n_ss + (double)t1 + 2.0 * t2) * pl.R * pair_words * 4.0 + (double)n_ss * (double)sum_doubles * 8.0;
            }
            // ---- the next state lists searched for equal states (hashes propose, a word-by-word comparison decides)
            const uint32_t n_next[2] = {t1, t2};
            const DevBuf* next_states[2] = {&S.f_states[nxt], &S.f_states2[nxt]};
            const DevBuf* next_hash[2] = {&S.f_hash[nxt], &S.f_hash2[nxt]};
            bool grouped_next[2] = {false, false};
            for (int li = 0; li < 2; ++li) grouped_next[li] = n_next[li] >= kGroupMin && n_next[li] < (1u << 24);
            for (int li = 0; li < 2; ++li) {
                const uint32_t n = n_next[li];
                if (!grouped_next[li]) continue;
                size_t table = 1024;
                while (table < (size_t)n * 2) table *= 2;
                P2_HIP(S.f_table.ensure(table * sizeof(unsigned long long)));
                P2_HIP(S.f_rep[li].ensure((size_t)n * sizeof(uint32_t)));
                P2_HIP(S.f_replist[li].ensure((size_t)n * sizeof(uint32_t)));
                P2_HIP(S.spans.begin(SpanRec::kGroup, S.stream));
                P2_HIP(hipMemsetAsync(S.f_table.p, 0xff, table * sizeof(unsigned long long), S.stream));
                P2_HIP(launch_front_dedup(static_cast<const uint32_t*>(next_states[li]->p), sw * (li + 1),
                                          static_cast<const unsigned long long*>(next_hash[li]->p), n,
                                          static_cast<unsigned long long*>(S.f_table.p), (uint32_t)table,
                                          static_cast<uint32_t*>(S.f_rep[li].p), static_cast<uint32_t*>(S.f_replist[li].p),
                                          &dctr->n_reps[li], S.stream));
                P2_HIP(S.spans.end(S.stream));
            }
            // ---- the next level's prefixes and this level's goals: those of the pair kernels at the places the listing
            //      gave them, then those of literal prefixes
            unsigned long long* vout = static_cast<unsigned long long*>(EV.p) + E.n_valid;
            double* gsums = static_cast<double*>(EG.p) + (size_t)E.n_valid * sum_doubles;
            unsigned long long* vout_lit = vout + n_goal_pair;
            double* gsums_lit = gsums + (size_t)n_goal_pair * sum_doubles;
            FrontPrefixes px;
            std::memset(&px, 0, sizeof px);
            px.query = (uint32_t)i; px.n_share = n_share; px.n_msg = n_msg;
            px.surv = static_cast<const FrontSurvivor*>(S.f_surv.p); px.n_surv = n_surv;
            px.parent_len = len; px.keep_prefixes = keep;
            px.entries1 = static_cast<const FrontEntry*>(S.f_entries[cur].p); px.sid1 = static_cast<const uint32_t*>(S.f_sid[cur].p);
            px.sums1 = static_cast<const double*>(S.f_sums[cur].p);
            px.entries2 = static_cast<const FrontEntry*>(S.f_entries2[cur].p); px.sid2 = static_cast<const uint32_t*>(S.f_sid2[cur].p);
            px.sums2 = static_cast<const double*>(S.f_sums2[cur].p);
            px.child_of1 = static_cast<const uint32_t*>(S.f_childof[0].p); px.child_of2 = static_cast<const uint32_t*>(S.f_childof[1].p);
            px.rep1 = grouped_next[0] ? static_cast<const uint32_t*>(S.f_rep[0].p) : nullptr;
            px.rep2 = grouped_next[1] ? static_cast<const uint32_t*>(S.f_rep[1].p) : nullptr;
            px.delta1 = lv.delta1; px.delta2 = lv.delta2; px.delta_goal = lv.delta_goal;
            px.next_entries1 = static_cast<FrontEntry*>(S.f_entries[nxt].p); px.next_sid1 = static_cast<uint32_t*>(S.f_sid[nxt].p);
            px.next_sums1 = static_cast<double*>(S.f_sums[nxt].p);
            px.next_entries2 = static_cast<FrontEntry*>(S.f_entries2[nxt].p); px.next_sid2 = static_cast<uint32_t*>(S.f_sid2[nxt].p);
            px.next_sums2 = static_cast<double*>(S.f_sums2[nxt].p);
            px.next_literal = static_cast<FrontEntry*>(S.f_literal[nxt].p);
            px.valid_out = vout; px.goal_sums = gsums; px.ctr = dctr;
            if (n_surv > 0) P2_HIP(S.spans.begin(SpanRec::kGroup, S.stream));
            P2_HIP(launch_front_prefixes(reinterpret_cast<const DevQuery*>(db), px, S.stream));
            if (n_surv > 0) P2_HIP(S.spans.end(S.stream));
            P2_HIP(launch_front_emit(dq, (uint32_t)i, static_cast<const FrontEntry*>(S.f_literal[cur].p),
                                     static_cast<const FrontSurvivor*>(S.f_surv_literal.p), n_surv_l_first, len, keep,
                                     static_cast<FrontEntry*>(S.f_literal[nxt].p), vout_lit, gsums_lit, (int)sum_doubles / 2, dctr, S.stream));
            P2_HIP(launch_front_emit(dq, (uint32_t)i, static_cast<const FrontEntry*>(S.f_unknown.p),
                                     static_cast<const FrontSurvivor*>(S.f_surv_literal.p) + n_surv_l_first, n_surv_l - n_surv_l_first, len, keep,
                                     static_cast<FrontEntry*>(S.f_literal[nxt].p), vout_lit, gsums_lit, (int)sum_doubles / 2, dctr, S.stream));
            E.n_valid += n_goal;
            n_c = keep ? n_prefix : 0;
            n_c2 = keep ? n_prefix2 : 0;
            n_l = keep ? n_plit : 0;
            n_s[0] = keep ? t1 : 0; n_s[1] = keep ? t2 : 0;
            grouped[0] = grouped_next[0]; grouped[1] = grouped_next[1];
            cur = nxt;
        }
        // steps of the last level
        P2_HIP(launch_copy_out(S.h_fctr.p, dctr, sizeof(FrontCounters), S.stream));
        P2_HIP(hipStreamSynchronize(S.stream));
        r.steps = hctr->steps; r.members = hctr->members;
        for (int32_t m : E.members) {        // every query of the enumeration reports its counts
            QueryRun& o = runs[m];
            o.n_valid = E.n_valid; o.n_rerun = r.n_rerun; o.steps = r.steps; o.members = r.members;
        }
        return P2_OK;
    };
    if (g_prof.on) P2_HIP(hipEventRecord(g_prof.ev[3], stream));
    for (FrontSlot& S : C.slots) {       // (also the slots that this call leaves idle: their figures are summed below)
        S.prof_prefixes = S.prof_state_bytes = S.prof_lane_ops = S.prof_children = S.prof_mat_bytes = S.prof_entries = 0.0;
        S.spans.reset();
    }
    if (!enums.empty()) {
        for (size_t e = 0; e < enums.size(); ++e) enums[e].id = (int)e;
        if (C.f_evalid.size() < enums.size()) { C.f_evalid.resize(enums.size()); C.f_egsums.resize(enums.size()); }
        bool one_at_a_time = false;
        for (int i = 0; i < n_queries; ++i)
            one_at_a_time |= queries[i].opt && (queries[i].opt->flags & P2_FLAG_ONE_ENUMERATION_AT_A_TIME) != 0u;
        const int n_slots = one_at_a_time ? 1 : (int)std::min<size_t>(kFrontSlots, enums.size());
        P2_HIP(hipEventRecord(C.front_go, stream));
        if (!C.slots[0].stream) {            // (first time: the streams are chosen by timing, on a quiet device)
            P2_HIP(hipStreamSynchronize(stream));
            P2_HIP(hipStreamSynchronize(C.copy_stream));
        }
        P2_HIP(C.open_slot_streams());
        for (int t = 0; t < n_slots; ++t) {
            FrontSlot& S = C.slots[t];
            P2_HIP(hipStreamWaitEvent(S.stream, C.front_go, 0));
            S.spans.on = g_prof.on; S.spans.kernels_only = g_prof.kernels_only; S.spans.reset();
            S.rc = P2_OK; S.err.clear();
        }
        // the long chains first: large reduction groups, large alphabets
        std::vector<int> order(enums.size());
        for (size_t e = 0; e < enums.size(); ++e) order[e] = (int)e;
        std::stable_sort(order.begin(), order.end(), [&](int x, int y) {
            const Plan& px = runs[enums[x].leader].plan; const Plan& py = runs[enums[y].leader].plan;
            if (px.R != py.R) return px.R > py.R;
            return px.alphabet > py.alphabet;
        });
        std::atomic<size_t> next{0};
        int device = 0;
        P2_HIP(hipGetDevice(&device));
        auto work = [&](int t, bool own_thread) {
            FrontSlot& S = C.slots[t];
            if (own_thread && hipSetDevice(device) != hipSuccess) { S.rc = P2_EDEVICE; S.err = "hipSetDevice failed in a worker thread"; return; }
            for (size_t at = next.fetch_add(1); at < order.size(); at = next.fetch_add(1)) {
                const int32_t rc = run_enum(enums[order[at]], S);
                if (rc != P2_OK) { S.rc = rc; S.err = g_err; break; }
            }
            // (whatever the slot has queued is waited for, also after a failure: its buffers are reused)
            (void)hipStreamSynchronize(S.stream);
        };
        if (n_slots == 1) {
            work(0, false);
        } else {
            std::vector<std::thread> pool;
            for (int t = 1; t < n_slots; ++t) pool.emplace_back(work, t, true);
            work(0, false);
            for (auto& th : pool) th.join();
        }
        for (int t = 0; t < n_slots; ++t)
            if (C.slots[t].rc != P2_OK) return fail(C.slots[t].rc, C.slots[t].err);
    }

    if (g_prof.on) {
        P2_HIP(hipEventRecord(g_prof.ev[4], stream));
        p2_profile& L = g_prof.last;
        L.front_prefixes = L.front_classify_state_bytes = L.front_classify_lane_ops = L.front_survivors = 0.0;
        L.front_materialize_bytes = L.front_entries = 0.0;
        for (const FrontSlot& S : C.slots) {
            L.front_prefixes += S.prof_prefixes; L.front_classify_state_bytes += S.prof_state_bytes;
            L.front_classify_lane_ops += S.prof_lane_ops; L.front_survivors += S.prof_children;
            L.front_materialize_bytes += S.prof_mat_bytes; L.front_entries += S.prof_entries;
        }
    }

    // ---- order, cost, select
    size_t total_valid = 0;
    for (auto& r : runs) { r.out_first = total_valid; total_valid += r.n_valid; }
    const size_t nm = (size_t)std::max(n_msg, 1);
    // rows the caller gets; without room for them (the sizing call with cap = 0) only the counts are returned,
    // and nothing is ordered, costed or selected
    int64_t need = 0;
    for (auto& r : runs) need += r.topk > 0 ? (int64_t)n_msg * (int64_t)std::min<size_t>(r.topk, r.n_valid) : (int64_t)r.n_valid;
    const bool store = cap >= need && cap > 0;
    // (every query with valid programs asks for a shortlist: only the rows that are picked go back to the host)
    bool only_shortlists = n_msg > 0;
    for (const auto& r : runs) only_shortlists = only_shortlists && (r.n_valid == 0 || r.topk > 0);
    size_t pos_off = 0;
    if (store) {
    P2_HIP(C.sorted.ensure(sizeof(unsigned long long) * std::max<size_t>(total_valid, 1)));
    P2_HIP(C.progs.ensure(sizeof(p2_program) * std::max<size_t>(total_valid, 1)));
    P2_HIP(C.costs.ensure(sizeof(double) * std::max<size_t>(total_valid, 1) * nm));
    size_t topk_rows = 0, topk_scratch = 0;
    for (auto& r : runs)
        if (r.topk > 0 && r.n_valid > 0) {
            topk_rows += (size_t)n_msg * std::min<size_t>(r.topk, r.n_valid);
            topk_scratch = std::max(topk_scratch, topk_scratch_bytes(r.n_valid, r.topk));
        }
    P2_HIP(C.topk_pos.ensure(sizeof(long long) * std::max<size_t>(topk_rows, 1)));
    P2_HIP(C.topk_scratch.ensure(std::max<size_t>(topk_scratch, 256)));
    int post_launches = 0;
    std::vector<DevTopkJob> topk_jobs, topk_big;          // short lists (a block each); long lists (cut into shares)
    int topk_jobs_k = 0, topk_big_k = 0;
    // ordering and costing: one launch per kernel and state-size class
    std::vector<PostLaunch> sort_launches, ccost_launches, scost_launches, lcost_launches;
    for (int i = 0; i < n_queries; ++i) {
        QueryRun& r = runs[i];
        if (r.n_valid == 0) continue;
        if (r.frontier) {
            // ordered and costed from the enumeration's sums (below); programs that came from literal prefixes
            // have no sums and are costed by the literal kernel
            const bool lit_cost = enums[r.enum_id].n_goal_literal > 0 && n_msg > 0;
            if (lit_cost && literal_lds_bytes(r.plan.R, r.plan.k) != 0)
                add_seg(lcost_launches, mask_class(r.plan.R) * 2 + 1, r.plan, i, r.n_valid, 1, 0, r.out_first);
            continue;
        }
        const size_t list_at = r.off_valid;
        if (r.wave_cost) {
            // one wavefront per program; it also finds the program's place in the ascending order
            add_seg(scost_launches, word_class(r.plan.k) * 100 + word_class(r.plan.R), r.plan, i, r.n_valid, 1, list_at,
                    r.out_first);
        } else {
            add_seg(sort_launches, 0, r.plan, i, r.n_valid, 256, list_at, r.out_first);
        }
        if (r.wave_cost) {
        } else if (r.engine == P2_ENGINE_COMPACT) {
            const int cls = word_class(r.plan.k) * 100 + word_class(r.plan.R);
            add_seg(ccost_launches, cls, r.plan, i, r.n_valid, 1, 0, r.out_first);     // per_block set below
        }
        const bool lit_cost = r.engine == P2_ENGINE_LITERAL || (r.n_rerun > 0 && n_msg > 0);
        if (lit_cost && literal_lds_bytes(r.plan.R, r.plan.k) != 0)
            add_seg(lcost_launches, mask_class(r.plan.R) * 2 + (r.engine == P2_ENGINE_COMPACT ? 1 : 0), r.plan, i, r.n_valid, 1, 0,
                    r.out_first);
    }
    for (auto& L : ccost_launches) {      // a block of the compact cost kernel takes as many entries as it has lanes
        // (one, with the lanes sharing the work, where only a few states fit in LDS)
        const uint32_t lanes = cost_wide_applies(L.max_R, L.max_k) ? 1u : (uint32_t)compact_lanes(L.max_R, L.max_k);
        L.blocks = 0;
        for (auto& sg : L.segs) { sg.per_block = lanes; sg.first_block = L.blocks; L.blocks += (sg.count + lanes - 1) / lanes; }
    }
    P2_HIP(upload_segs({&sort_launches, &ccost_launches, &scost_launches, &lcost_launches}));
    unsigned long long* sorted_base = static_cast<unsigned long long*>(C.sorted.p);
    p2_program* progs_base = static_cast<p2_program*>(C.progs.p);
    double* costs_base = static_cast<double*>(C.costs.p);
    for (auto& L : sort_launches) {
        ++post_launches;
        P2_HIP(launch_rank_sort(static_cast<unsigned long long*>(C.valid.p), nullptr, sorted_base,
                                segs_of(L), (int)L.segs.size(), L.blocks, stream));
    }
    // the compact engine costs what it can hold and marks the rest with NaN for the literal engine
    for (auto& L : ccost_launches) {
        ++post_launches;
        if (cost_wide_applies(L.max_R, L.max_k))
            P2_HIP(launch_cost_wide_list(reinterpret_cast<const DevQuery*>(db), segs_of(L), (int)L.segs.size(), L.blocks, L.max_R,
                                         L.max_k, sorted_base, progs_base, costs_base, stream));
        else
            P2_HIP(launch_cost_compact_list(reinterpret_cast<const DevQuery*>(db), segs_of(L), (int)L.segs.size(), L.blocks, L.max_R,
                                            L.max_k, sorted_base, progs_base, costs_base, stream));
    }
    for (auto& L : scost_launches) {
        ++post_launches;
        P2_HIP(launch_cost_shared(reinterpret_cast<const DevQuery*>(db), segs_of(L), (int)L.segs.size(), L.blocks, L.max_R,
                                  L.max_k, static_cast<unsigned long long*>(C.valid.p), nullptr,
                                  sorted_base, progs_base, costs_base, stream));
    }
    // frontier enumerations: the place of every program in ascending index order, once per enumeration; then
    // every query of the enumeration writes its rows (programs, and costs from its own sums)
    if (!enums.empty()) {
        size_t ranked = 0;
        for (auto& E : enums) { E.off_valid = ranked; ranked += E.n_valid; }
        P2_HIP(C.f_rank.ensure(sizeof(uint32_t) * std::max<size_t>(ranked, 1)));
        std::vector<FrontFinish> jobs;
        uint32_t max_valid = 0;
        for (auto& E : enums) {
            if (E.n_valid == 0) continue;
            const unsigned long long* list = static_cast<const unsigned long long*>(C.f_evalid[E.id].p);
            uint32_t* rank = static_cast<uint32_t*>(C.f_rank.p) + E.off_valid;
            // (a query that asks for the cheapest programs only has them selected by (cost, index): its rows need no order)
            bool ordered = false;
            for (int32_t m : E.members) ordered |= runs[m].topk == 0;
            if (ordered) {
                ++post_launches;
                P2_HIP(launch_front_rank(list, E.n_valid, rank, stream));
            }
            for (size_t m = 0; m < E.members.size(); ++m) {
                FrontFinish F;
                std::memset(&F, 0, sizeof F);
                F.query = (uint32_t)E.members[m]; F.n_share = (int32_t)E.members.size(); F.share_pos = (int32_t)m;
                F.n_valid = E.n_valid; F.valid = list; F.rank = runs[E.members[m]].topk == 0 ? rank : nullptr;
                F.goal_sums = static_cast<const double*>(C.f_egsums[E.id].p);
                F.out_first = runs[E.members[m]].out_first;
                F.sorted = sorted_base; F.progs = progs_base; F.costs = costs_base;
                jobs.push_back(F);
                max_valid = std::max(max_valid, E.n_valid);
            }
        }
        if (!jobs.empty()) {                        // the rows of all of them in one launch
            P2_HIP(C.f_finish.ensure(sizeof(FrontFinish) * jobs.size()));
            P2_HIP(C.h_finish.ensure(sizeof(FrontFinish) * jobs.size()));
            std::memcpy(C.h_finish.p, jobs.data(), sizeof(FrontFinish) * jobs.size());
            P2_HIP(hipMemcpyAsync(C.f_finish.p, C.h_finish.p, sizeof(FrontFinish) * jobs.size(), hipMemcpyHostToDevice, stream));
            ++post_launches;
            P2_HIP(launch_front_finish(reinterpret_cast<const DevQuery*>(db), static_cast<const FrontFinish*>(C.f_finish.p),
                                       (uint32_t)jobs.size(), max_valid, stream));
        }
    }
    for (auto& L : lcost_launches) {
        ++post_launches;
        P2_HIP(launch_cost_literal_list(reinterpret_cast<const DevQuery*>(db), segs_of(L), (int)L.segs.size(), L.blocks, L.max_R,
                                        L.lit_lds, sorted_base, progs_base, costs_base, L.cls & 1, stream));
    }
    for (int i = 0; i < n_queries; ++i) {
        QueryRun& r = runs[i];
        if (r.n_valid == 0) continue;
        const DevQuery* dq = reinterpret_cast<const DevQuery*>(db + r.off_query);
        unsigned long long* sorted = sorted_base + r.out_first;
        p2_program* progs = progs_base + r.out_first;
        double* costs = costs_base + r.out_first * nm;
        const bool lit_cost = r.frontier ? (enums[r.enum_id].n_goal_literal > 0 && n_msg > 0)
                                         : (r.engine == P2_ENGINE_LITERAL || (r.n_rerun > 0 && n_msg > 0));
        if (lit_cost && literal_lds_bytes(r.plan.R, r.plan.k) == 0) {      // literal state too large for LDS
            void* gs = nullptr;
            P2_HIP(lit_scratch(r.plan, &gs));
            ++post_launches;
            P2_HIP(launch_cost_literal(dq, r.plan.R, r.plan.k, sorted, r.n_valid, progs, costs,
                                       r.engine == P2_ENGINE_COMPACT ? 1 : 0, gs, stream));
        }
        if (r.topk > 0) {
            const size_t kk = std::min<size_t>(r.topk, r.n_valid);
            for (int m = 0; m < n_msg; ++m) {
                long long* out_pos = static_cast<long long*>(C.topk_pos.p) + pos_off;
                uint32_t* nan_flag = &static_cast<DevCounters*>(C.counters.p)[i].nan_seen;
                if (r.n_valid <= kTopkJobMax) {            // short lists: one launch for all of them, below
                    DevTopkJob J;
                    J.cost = costs + m; J.index = sorted; J.out_pos = out_pos; J.nan_flag = nan_flag;
                    J.n = (long long)r.n_valid; J.stride = n_msg; J.k = r.topk; J.pad = 0;
                    topk_jobs.push_back(J);
                    topk_jobs_k = std::max(topk_jobs_k, r.topk);
                } else {
                    DevTopkJob J;
                    J.cost = costs + m; J.index = sorted; J.out_pos = out_pos; J.nan_flag = nan_flag;
                    J.n = (long long)r.n_valid; J.stride = n_msg; J.k = r.topk; J.pad = 0;
                    topk_big.push_back(J);
                    topk_big_k = std::max(topk_big_k, r.topk);
                }
                pos_off += kk;
            }
        }
    }
    if (!topk_jobs.empty() || !topk_big.empty()) {
        const size_t n_small = topk_jobs.size(), n_big = topk_big.size();
        const size_t bytes = sizeof(DevTopkJob) * (n_small + n_big);
        P2_HIP(C.topk_jobs.ensure(bytes));
        P2_HIP(C.h_topk_jobs.ensure(bytes));
        DevTopkJob* hj = static_cast<DevTopkJob*>(C.h_topk_jobs.p);
        if (n_small) std::memcpy(hj, topk_jobs.data(), sizeof(DevTopkJob) * n_small);
        if (n_big) std::memcpy(hj + n_small, topk_big.data(), sizeof(DevTopkJob) * n_big);
        P2_HIP(hipMemcpyAsync(C.topk_jobs.p, C.h_topk_jobs.p, bytes, hipMemcpyHostToDevice, stream));
        const DevTopkJob* dj = static_cast<const DevTopkJob*>(C.topk_jobs.p);
        if (n_small) {
            ++post_launches;
            P2_HIP(launch_topk_jobs(dj, (unsigned)n_small, topk_jobs_k, stream));
        }
        // long lists: two launches per 16384 of them
        for (size_t at = 0; at < n_big; at += 16384) {
            const unsigned n = (unsigned)std::min<size_t>(16384, n_big - at);
            P2_HIP(C.topk_scratch.ensure(topk_big_scratch_bytes(n, topk_big_k)));
            post_launches += 2;
            P2_HIP(launch_topk_big(dj + n_small + at, n, topk_big_k, C.topk_scratch.p, stream));
        }
    }
    if (g_prof.on) { P2_HIP(hipEventRecord(g_prof.ev[2], stream)); g_prof.last.post_launches = post_launches; }
    P2_HIP(C.h_pos.ensure(sizeof(long long) * std::max<size_t>(topk_rows, 1)));
    if (only_shortlists) {
        // every query asks for a shortlist: the rows that were picked are gathered on the device, and only they go back
        std::vector<DevGatherSeg> segs;
        size_t at = 0;
        for (int i = 0; i < n_queries; ++i) {
            const QueryRun& r = runs[i];
            if (r.n_valid == 0) continue;
            const size_t rows = (size_t)n_msg * std::min<size_t>(r.topk, r.n_valid);
            segs.push_back(DevGatherSeg{(unsigned long long)r.out_first, (unsigned long long)at, (uint32_t)rows, 0u});
            at += rows;
        }
        P2_HIP(C.gather.ensure(sizeof(DevGatherSeg) * std::max<size_t>(segs.size(), 1)));
        P2_HIP(C.h_gather.ensure(sizeof(DevGatherSeg) * std::max<size_t>(segs.size(), 1)));
        P2_HIP(C.sel_progs.ensure(sizeof(p2_program) * std::max<size_t>(topk_rows, 1)));
        P2_HIP(C.sel_costs.ensure(sizeof(double) * std::max<size_t>(topk_rows, 1) * nm));
        P2_HIP(C.h_progs.ensure(sizeof(p2_program) * std::max<size_t>(topk_rows, 1)));
        P2_HIP(C.h_costs.ensure(sizeof(double) * std::max<size_t>(topk_rows, 1) * nm));
        if (!segs.empty()) {
            std::memcpy(C.h_gather.p, segs.data(), sizeof(DevGatherSeg) * segs.size());
            P2_HIP(hipMemcpyAsync(C.gather.p, C.h_gather.p, sizeof(DevGatherSeg) * segs.size(), hipMemcpyHostToDevice, stream));
            P2_HIP(launch_gather_rows(static_cast<const DevGatherSeg*>(C.gather.p), (unsigned)segs.size(), progs_base, costs_base, n_msg,
                                      static_cast<const long long*>(C.topk_pos.p), static_cast<p2_program*>(C.sel_progs.p),
                                      static_cast<double*>(C.sel_costs.p), stream));
        }
        P2_HIP(launch_copy_out3(C.h_progs.p, C.sel_progs.p, sizeof(p2_program) * topk_rows,
                                C.h_costs.p, C.sel_costs.p, sizeof(double) * topk_rows * nm,
                                C.h_pos.p, C.topk_pos.p, sizeof(long long) * topk_rows, stream));
    } else {
        P2_HIP(C.h_progs.ensure(sizeof(p2_program) * std::max<size_t>(total_valid, 1)));
        P2_HIP(C.h_costs.ensure(sizeof(double) * std::max<size_t>(total_valid, 1) * nm));
        P2_HIP(launch_copy_out3(C.h_progs.p, C.progs.p, sizeof(p2_program) * total_valid,
                                C.h_costs.p, C.costs.p, n_msg > 0 ? sizeof(double) * total_valid * nm : 0,
                                C.h_pos.p, C.topk_pos.p, sizeof(long long) * topk_rows, stream));
    }
    if (topk_rows > 0)      // the selections flag a NaN cost in their query's counters
        P2_HIP(launch_copy_out(C.h_counters.p, C.counters.p, sizeof(DevCounters) * (size_t)n_queries, stream));
    P2_HIP(hipStreamSynchronize(stream));
    if (topk_rows > 0) {
        const DevCounters* hc = static_cast<const DevCounters*>(C.h_counters.p);
        for (int i = 0; i < n_queries; ++i)
            if (runs[i].topk > 0 && hc[i].nan_seen)
                return fail(P2_EINVAL, "query " + std::to_string(i) + ": NaN cost (a message size that is not finite?)");
    }
    }  // store

    if (g_prof.on) {
        P2_HIP(hipEventElapsedTime(&g_prof.last.eval_ms, g_prof.ev[0], g_prof.ev[1]));
        g_prof.last.post_ms = 0.0f;
        if (store) P2_HIP(hipEventElapsedTime(&g_prof.last.post_ms, g_prof.ev[4], g_prof.ev[2]));
        P2_HIP(hipEventSynchronize(g_prof.ev[4]));      // (a call that only sizes its result has not waited since)
        P2_HIP(hipEventElapsedTime(&g_prof.last.front_ms, g_prof.ev[3], g_prof.ev[4]));
        float ms[SpanRec::kKinds] = {0.f, 0.f, 0.f, 0.f};
        int32_t launches[SpanRec::kKinds] = {0, 0, 0, 0};
        for (FrontSlot& S : C.slots) P2_HIP(S.spans.collect(ms, launches));
        g_prof.last.front_classify_ms = ms[SpanRec::kClassify]; g_prof.last.front_classify_launches = launches[SpanRec::kClassify];
        g_prof.last.front_literal_ms = ms[SpanRec::kLiteral]; g_prof.last.front_literal_launches = launches[SpanRec::kLiteral];
        g_prof.last.front_materialize_ms = ms[SpanRec::kMaterialize]; g_prof.last.front_materialize_launches = launches[SpanRec::kMaterialize];
        g_prof.last.front_group_ms = ms[SpanRec::kGroup];
    }
    // ---- hand the results over
    const p2_program* hp = static_cast<const p2_program*>(C.h_progs.p);
    const double* hcst = static_cast<const double*>(C.h_costs.p);
    const long long* hpos = static_cast<const long long*>(C.h_pos.p);
    int64_t w = 0;
    pos_off = 0;
    for (int i = 0; i < n_queries; ++i) {
        QueryRun& r = runs[i];
        out_offset[i] = w;
        if (r.topk > 0) {
            const size_t kk = std::min<size_t>(r.topk, r.n_valid);
            if (!store) w += (int64_t)n_msg * (int64_t)kk;
            for (int m = 0; m < n_msg && store; ++m)
                for (size_t t = 0; t < kk; ++t, ++w) {
                    const size_t sel = pos_off;
                    const long long pos = hpos[pos_off++];
                    if (pos < 0 || pos >= (long long)r.n_valid) return fail(P2_EDEVICE, "top-k returned a bad position");
                    const size_t row = only_shortlists ? sel : r.out_first + (size_t)pos;
                    out_prog[w] = hp[row];
                    for (int c = 0; c < n_msg; ++c) out_cost[w * n_msg + c] = hcst[row * nm + c];
                }
        } else {
            if (store) {
                std::memcpy(out_prog + w, hp + r.out_first, sizeof(p2_program) * r.n_valid);
                if (n_msg > 0) std::memcpy(out_cost + w * n_msg, hcst + r.out_first * nm, sizeof(double) * r.n_valid * nm);
            }
            w += r.n_valid;
        }
        if (stats) {
            p2_stats& s = stats[i];
            s.candidates = r.plan.n_candidates; s.steps_executed = r.steps; s.member_visits = r.members;
            s.literal_reruns = r.shared ? (uint64_t)r.n_rerun_groups * (uint64_t)r.plan.alphabet : r.n_rerun;
            s.steps_evaluated = r.shared ? r.evaluated : r.steps;
            s.members_evaluated = r.shared ? r.evaluated_members : r.members;
            s.valid = r.n_valid; s.group_size = r.plan.R; s.n_patterns = (int32_t)r.plan.patterns.size();
            s.evaluated_with = r.frontier ? (r.enum_id >= 0 && enums[r.enum_id].leader != i ? enums[r.enum_id].leader : -1) : r.same_as;
            s.reserved0 = 0;
            s.alphabet = r.plan.alphabet; s.engine = r.frontier ? P2_ENGINE_FRONTIER : r.shared ? P2_ENGINE_SHARED : r.regs ? P2_ENGINE_SMALL : r.engine;
        }
    }
    out_offset[n_queries] = w;
    g_prof.last.host_total_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t_begin).count();
    if (!store && need > 0) return fail(P2_ENOSPC, "output buffer too small: " + std::to_string(need) + " rows needed");
    return P2_OK;
}

}  // namespace

extern "C" {

const char* p2_last_error(void) { return g_err.c_str(); }

int32_t p2_set_profiling(int32_t on) {
    if (on && !g_prof.ev[0])
        for (auto& e : g_prof.ev) P2_HIP(hipEventCreate(&e));
    g_prof.on = on != 0;
    g_prof.kernels_only = on == 2;
    return P2_OK;
}
int32_t p2_get_profile(p2_profile* out) {
    if (!out) return fail(P2_EINVAL, "null argument");
    *out = g_prof.last;
    return P2_OK;
}

int32_t p2_release_thread(void) {
    g_ctx.release();
    g_prof.release();
    return P2_OK;
}

int32_t p2_measure_alu_peak(int32_t reps, double* out_lane_ops_per_s, void* hip_stream) {
    if (!out_lane_ops_per_s || reps < 1 || reps > 100) return fail(P2_EINVAL, "bad arguments");
    P2_HIP(p2::measure_alu_peak(reps, out_lane_ops_per_s, (hipStream_t)hip_stream));
    return P2_OK;
}

int32_t p2_measure_lds_peak(int32_t reps, double* out_bytes_per_s, void* hip_stream) {
    if (!out_bytes_per_s || reps < 1 || reps > 100) return fail(P2_EINVAL, "bad arguments");
    P2_HIP(p2::measure_lds_peak(reps, out_bytes_per_s, (hipStream_t)hip_stream));
    return P2_OK;
}

int32_t p2_enumerate_placements(const p2_hierarchy* h, const int32_t* axes, int32_t n_axes, int32_t* out, int64_t cap,
                                int64_t* out_count) {
    std::string err;
    int32_t st = p2::enumerate_placements(h, axes, n_axes, out, cap, out_count, err);
    if (st != P2_OK) g_err = err;
    return st;
}

int32_t p2_synthesize_batch(const p2_query* queries, int32_t n_queries, const double* msg_bytes, int32_t n_msg,
                            p2_program* out_prog, double* out_cost, int64_t cap, int64_t* out_offset, p2_stats* stats) {
    try {
        return run_batch(queries, n_queries, msg_bytes, n_msg, out_prog, out_cost, cap, out_offset, stats);
    } catch (const std::exception& e) {
        return fail(P2_EDEVICE, std::string("host failure: ") + e.what());
    }
}

int32_t p2_synthesize(const p2_hierarchy* h, const int32_t* axes, int32_t n_axes, const int32_t* placement,
                      const int32_t* reduce_axes, int32_t n_reduce, int32_t max_len, const double* msg_bytes, int32_t n_msg,
                      const p2_options* opt, p2_program* out_prog, double* out_cost, int64_t cap, int64_t* out_count,
                      uint64_t* out_candidates_evaluated, p2_stats* stats) {
    if (!out_count) return fail(P2_EINVAL, "out_count is null");
    p2_query q{h, axes, n_axes, placement, reduce_axes, n_reduce, max_len, opt};
    int64_t offs[2] = {0, 0};
    p2_stats st;
    std::memset(&st, 0, sizeof st);
    int32_t rc = p2_synthesize_batch(&q, 1, msg_bytes, n_msg, out_prog, out_cost, cap, offs, &st);
    if (rc == P2_OK || rc == P2_ENOSPC) {
        *out_count = offs[1];
        if (out_candidates_evaluated) *out_candidates_evaluated = st.candidates;
        if (stats) *stats = st;
    }
    return rc;
}

int32_t p2_search_placements(const p2_hierarchy* h, const int32_t* axes, int32_t n_axes, const int32_t* reduce_sets,
                             const int32_t* reduce_set_len, int32_t n_sets, const double* weights, int32_t max_len,
                             double msg_bytes, const p2_options* opt, int32_t* out_placements, p2_search_row* out_rows,
                             double* out_total, int32_t* out_order, int64_t cap, int64_t* out_count) {
    try {
        if (!h || !axes || !reduce_sets || !reduce_set_len || !out_count) return fail(P2_EINVAL, "null argument");
        if (n_sets < 1) return fail(P2_EINVAL, "no reduction requested");
        if (cap < 0 || (cap > 0 && (!out_placements || !out_rows || !out_total || !out_order)))
            return fail(P2_EINVAL, "bad output buffer");
        if (!(msg_bytes >= 0.0)) return fail(P2_EINVAL, "msg_bytes is negative or NaN");
        if (opt && opt->hierarchy != P2_HIERARCHY_COLLAPSED)
            return fail(P2_EUNSUPPORTED, "the placement search synthesizes on the collapsed hierarchy");
        std::vector<const int32_t*> set_ptr((size_t)n_sets);
        {
            const int32_t* at = reduce_sets;
            for (int s = 0; s < n_sets; ++s) {
                if (reduce_set_len[s] < 1) return fail(P2_EINVAL, "empty set of reduce axes");
                set_ptr[(size_t)s] = at;
                at += reduce_set_len[s];
            }
        }
        int64_t n_pl = 0;
        std::string err;
        int32_t st = p2::enumerate_placements(h, axes, n_axes, nullptr, 0, &n_pl, err);
        if (st != P2_OK) return fail(st, err);
        *out_count = n_pl;
        if (cap == 0) return P2_OK;
        if (cap < n_pl) return fail(P2_ENOSPC, "output buffers too small: " + std::to_string(n_pl) + " placements");
        const size_t per = (size_t)n_axes * (size_t)h->n_levels;
        st = p2::enumerate_placements(h, axes, n_axes, out_placements, n_pl, &n_pl, err);
        if (st != P2_OK) return fail(st, err);
        if (n_pl * (int64_t)n_sets * 2 > 0x7fffffff) return fail(P2_EUNSUPPORTED, "too many (placement, reduction) pairs");

        // two queries per (placement, reduction): the search itself, keeping its cheapest program,
        // and the one-instruction AllReduce over the whole reduction group
        p2_options main_opt;
        std::memset(&main_opt, 0, sizeof main_opt);
        if (opt) main_opt = *opt;
        main_opt.topk = 1;
        p2_options base_opt = main_opt;
        base_opt.form_mask = 1; base_opt.op_mask = 1; base_opt.topk = 0; base_opt.engine = P2_ENGINE_AUTO;
        const int n_q = (int)(n_pl * n_sets * 2);
        std::vector<p2_query> qs((size_t)n_q);
        for (int64_t p = 0; p < n_pl; ++p)
            for (int s = 0; s < n_sets; ++s) {
                const size_t at = ((size_t)p * (size_t)n_sets + (size_t)s) * 2;
                qs[at] = p2_query{h, axes, n_axes, out_placements + (size_t)p * per, set_ptr[(size_t)s], reduce_set_len[s], max_len, &main_opt};
                qs[at + 1] = p2_query{h, axes, n_axes, out_placements + (size_t)p * per, set_ptr[(size_t)s], reduce_set_len[s], 1, &base_opt};
            }
        std::vector<p2_program> progs((size_t)n_q);
        std::vector<double> costs((size_t)n_q);
        std::vector<int64_t> offs((size_t)n_q + 1);
        std::vector<p2_stats> stats((size_t)n_q);
        int32_t rc = run_batch(qs.data(), n_q, &msg_bytes, 1, progs.data(), costs.data(), n_q, offs.data(), stats.data());
        if (rc != P2_OK) return rc;
        const double inf = std::numeric_limits<double>::infinity();
        for (int64_t p = 0; p < n_pl; ++p) {
            double total = 0.0;
            for (int s = 0; s < n_sets; ++s) {
                const size_t at = ((size_t)p * (size_t)n_sets + (size_t)s) * 2;
                p2_search_row& row = out_rows[(size_t)p * (size_t)n_sets + (size_t)s];
                std::memset(&row, 0, sizeof row);
                row.candidates = stats[at].candidates;
                row.valid = stats[at].valid;
                if (stats[at].alphabet == 0) {                  // a reduction over one device: nothing to do
                    row.best_cost = 0.0; row.allreduce_cost = 0.0;
                } else {
                    if (offs[at + 1] > offs[at]) { row.best = progs[(size_t)offs[at]]; row.best_cost = costs[(size_t)offs[at]]; }
                    else row.best_cost = inf;
                    if (offs[at + 2] - offs[at + 1] != 1) return fail(P2_EDEVICE, "the AllReduce baseline did not evaluate to one program");
                    row.allreduce_cost = costs[(size_t)offs[at + 1]];
                }
                total += (weights ? weights[s] : 1.0) * row.best_cost;
            }
            out_total[p] = total;
        }
        for (int64_t p = 0; p < n_pl; ++p) out_order[p] = (int32_t)p;
        std::stable_sort(out_order, out_order + n_pl, [&](int32_t a, int32_t b) { return out_total[a] < out_total[b]; });
        return P2_OK;
    } catch (const std::exception& e) {
        return fail(P2_EDEVICE, std::string("host failure: ") + e.what());
    }
}

int32_t p2_describe_pattern(const p2_hierarchy* h, const int32_t* axes, int32_t n_axes, const int32_t* placement,
                            const int32_t* reduce_axes, int32_t n_reduce, const p2_options* opt, int32_t pattern_id,
                            int32_t* slice_level, int32_t* form, int32_t* form_level, int32_t* group_of_device,
                            int32_t* rank_in_group, int32_t* out_n_patterns) {
    try {
        p2::Plan pl;
        std::string err;
        int32_t st = p2::make_plan(h, axes, n_axes, placement, reduce_axes, n_reduce, 1, opt, false, pl, err);
        if (st != P2_OK) return fail(st, err);
        if (out_n_patterns) *out_n_patterns = (int32_t)pl.patterns.size();
        if (pattern_id < 0 || pattern_id >= (int32_t)pl.patterns.size()) return fail(P2_EINVAL, "pattern id out of range");
        const p2::Pattern& p = pl.patterns[pattern_id];
        if (slice_level) *slice_level = p.slice;
        if (form) *form = p.form;
        if (form_level) *form_level = p.form_level;
        if (group_of_device && rank_in_group) p2::describe_pattern(pl, pattern_id, group_of_device, rank_in_group);
        return P2_OK;
    } catch (const std::exception& e) {
        return fail(P2_EDEVICE, std::string("host failure: ") + e.what());
    }
}

int32_t p2_topk_device(const double* cost, int64_t cost_stride, const uint64_t* index, int64_t n, int32_t k,
                       int64_t* out_pos, void* stream_) {
    using namespace p2;
    if (n < 0 || k < 0 || cost_stride < 1) return fail(P2_EINVAL, "bad n, k or stride");
    if (k > kMaxTopK) return fail(P2_EUNSUPPORTED, "topk > 1024");
    if (n == 0 || k == 0) return P2_OK;
    if (!cost || !index || !out_pos) return fail(P2_EINVAL, "null argument");
    hipStream_t stream = (hipStream_t)stream_;
    Ctx& C = g_ctx;
    P2_HIP(C.topk_scratch.ensure(topk_scratch_bytes(n, k)));
    P2_HIP(C.counters.ensure(sizeof(DevCounters)));
    P2_HIP(C.h_counters.ensure(sizeof(DevCounters)));
    P2_HIP(hipMemsetAsync(C.counters.p, 0, sizeof(DevCounters), stream));
    DevCounters* dc = static_cast<DevCounters*>(C.counters.p);
    P2_HIP(launch_topk(cost, cost_stride, reinterpret_cast<const unsigned long long*>(index), n, k,
                       reinterpret_cast<long long*>(out_pos), C.topk_scratch.p, &dc->nan_seen, stream));
    P2_HIP(launch_copy_out(C.h_counters.p, C.counters.p, sizeof(DevCounters), stream));
    P2_HIP(hipStreamSynchronize(stream));
    if (static_cast<const DevCounters*>(C.h_counters.p)->nan_seen) return fail(P2_EINVAL, "NaN cost");
    return P2_OK;
}

int32_t p2_topk_device_noalloc(const double* cost, int64_t cost_stride, const uint64_t* index, int64_t n, int32_t k,
                               int64_t* out_pos, uint32_t* out_nan, void* stream_) {
    using namespace p2;
    if (n < 0 || k < 0 || cost_stride < 1) return fail(P2_EINVAL, "bad n, k or stride");
    if (k > topk_fixed_max_k()) return fail(P2_EUNSUPPORTED, "topk > 64 without allocation: the fixed scratch holds lists of at most 64 entries");
    if (n == 0 || k == 0) return P2_OK;
    if (!cost || !index || !out_pos) return fail(P2_EINVAL, "null argument");
    P2_HIP(launch_topk_fixed(cost, cost_stride, reinterpret_cast<const unsigned long long*>(index), n, k,
                             reinterpret_cast<long long*>(out_pos), out_nan, (hipStream_t)stream_));
    return P2_OK;
}

int32_t p2_topk(const double* cost, const uint64_t* index, int64_t n, int32_t k, int64_t* out_pos) {
    using namespace p2;
    if (n < 0 || k < 0) return fail(P2_EINVAL, "bad n or k");
    if (k > kMaxTopK) return fail(P2_EUNSUPPORTED, "topk > 1024");
    if (n == 0 || k == 0) return P2_OK;
    if (!cost || !index || !out_pos) return fail(P2_EINVAL, "null argument");
    Ctx& C = g_ctx;
    const size_t kk = (size_t)std::min<int64_t>(k, n);
    P2_HIP(C.topk_in.ensure((size_t)n * 16));
    P2_HIP(C.topk_pos.ensure(kk * sizeof(long long)));
    double* dcost = static_cast<double*>(C.topk_in.p);
    uint64_t* didx = reinterpret_cast<uint64_t*>(dcost + n);
    P2_HIP(hipMemcpy(dcost, cost, (size_t)n * 8, hipMemcpyHostToDevice));
    P2_HIP(hipMemcpy(didx, index, (size_t)n * 8, hipMemcpyHostToDevice));
    int32_t rc = p2_topk_device(dcost, 1, didx, n, k, static_cast<int64_t*>(C.topk_pos.p), nullptr);
    if (rc != P2_OK) return rc;
    P2_HIP(hipMemcpy(out_pos, C.topk_pos.p, kk * sizeof(long long), hipMemcpyDeviceToHost));
    return P2_OK;
}

}  // extern "C"
