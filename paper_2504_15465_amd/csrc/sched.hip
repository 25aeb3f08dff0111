// Tenants, the dispatcher/tracker machinery around the policy core, and the
// native load generators (LithOS Sections 4.2, 4.3; clients of Section 7.1).
//
// One tracker thread per context polls completion events, feeds measured atom
// latencies back into the core (sync queues / predictor) and dispatches the
// atoms that become eligible.  A submitting thread also dispatches inline, so
// an arriving high-priority kernel does not wait for a thread hand-off.
//
// "Handing CUs to another tenant at an atom boundary" is done by choosing
// which pre-created CU-masked queue receives the next atom: a tenant owns one
// queue per CU set it has ever used (its quota, quota + stolen sets).  When a
// tenant's consecutive atoms go to different queues an event keeps them in
// order.
#include "runtime.hpp"
#include "sched_core.hpp"

#include <chrono>
#include <condition_variable>
#include <deque>
#include <map>
#include <mutex>
#include <thread>
#include <vector>
#include <cstring>

namespace lithos {

static inline double now_us()
{
    using namespace std::chrono;
    return duration<double, std::micro>(steady_clock::now().time_since_epoch()).count();
}

struct PendingOp {
    lithos_op_t op;
    OpPlan plan;
    uint64_t kernel_id;
};

struct Fly {
    uint64_t atom_id;       // 0 for pass-through kernels
    hipEvent_t ev;
    double t_launch;
    uint64_t kernel_done;   // kernel id completed by this atom, or 0
};

} // namespace lithos

struct lithos_tenant {
    lithos_ctx* ctx = nullptr;
    int cls = LITHOS_CLASS_BE;
    const lithos_partition* quota = nullptr;
    bool passthrough = false;
    int core_idx = -1;
    int group = -1;
    hipStream_t own_stream = nullptr;                 // pass-through only
    std::deque<lithos::PendingOp> ops;                // submitted, not fully launched
    std::deque<lithos::Fly> fly;                      // launched, completion not yet seen
    std::map<uint32_t, hipStream_t> streams;          // group mask -> CU-masked queue
    hipStream_t last_stream = nullptr;
    hipEvent_t switch_ev = nullptr;
    double last_done_us = 0.0;
    std::atomic<uint64_t> submitted{0};               // kernels submitted
    std::atomic<uint64_t> completed{0};               // kernels completed (in order)
    uint64_t pt_kernel_seq = 0;                       // pass-through ticket counter
    std::mutex pt_mu;                                 // pass-through: guards fly
    lithos_stats_t pt_stats{};
};

namespace lithos {

// ---- queue coupling ---------------------------------------------------------------
// Hardware queues that the driver placed on the same command-processor pipe are
// not independent: while one of them holds a grid that is only partly dispatched
// (more workgroups than its CUs have room for), packets of the other queues on
// that pipe wait.  A high-priority queue that shares a pipe with a best-effort
// queue would therefore wait for whole best-effort atoms.  Which pipe a queue
// gets is decided at creation and cannot be asked for, so it is measured: a
// four-wave spin grid is started on queue `busy`, then a one-block kernel on
// queue `probe`; if the latter takes as long as the grid, the two are coupled.
static int queues_coupled(lithos_ctx* ctx, hipStream_t busy, int busy_cus, hipStream_t probe, bool* coupled)
{
    lithos_op_t big{}, tiny{};
    big.kind = tiny.kind = LITHOS_OP_SPIN;
    big.dim[0] = 8 * (int64_t)busy_cus;     // two blocks fit on a CU: four waves of blocks
    big.dim[1] = 10000;                      // 100 us each
    tiny.dim[0] = 1;
    tiny.dim[1] = 1;
    OpPlan pb, pt;
    int rc = op_plan(big, &pb);
    if (rc == LITHOS_OK) rc = op_plan(tiny, &pt);
    if (rc != LITHOS_OK) return rc;
    AtomArgs ab{0, pb.total, pb.grid.x, pb.grid.y, 1, 0, nullptr}, at{0, 1, 1, 1, 1, 0, nullptr};
    LITHOS_HIP(hipStreamSynchronize(busy));
    LITHOS_HIP(hipStreamSynchronize(probe));
    rc = op_launch(big, pb, ab, busy);
    if (rc != LITHOS_OK) return rc;
    const double t0 = now_us();
    rc = op_launch(tiny, pt, at, probe);
    if (rc != LITHOS_OK) return rc;
    LITHOS_HIP(hipStreamSynchronize(probe));
    const double dt = now_us() - t0;
    LITHOS_HIP(hipStreamSynchronize(busy));
    *coupled = dt > 200.0;                   // uncoupled: tens of microseconds; coupled: ~300
    return LITHOS_OK;
}

struct OtherQueue { hipStream_t stream; int cus; };

// A CU-masked queue that is coupled with none of `others`.  The pipe of a queue
// follows from its position among the process's live queues (measured: position
// modulo the pipe count; destroying a queue moves all later ones up).  Queues are
// therefore only ever appended here: a rejected candidate is parked, not destroyed,
// so that the next candidate lands one position, and one pipe, further on.
static int make_decoupled_stream(lithos_ctx* ctx, const uint32_t* mask, const std::vector<OtherQueue>& others, hipStream_t* out)
{
    const uint32_t words = (ctx->n_cu + 31) / 32;
    for (int attempt = 0; attempt < 8; ++attempt) {
        hipStream_t s = nullptr;
        hipError_t e = hipExtStreamCreateWithCUMask(&s, words, mask);
        if (e != hipSuccess) return fail(LITHOS_EHIP, "hipExtStreamCreateWithCUMask: %s", hipGetErrorString(e));
        bool bad = false;
        int rc = LITHOS_OK;
        for (const OtherQueue& o : others) {
            bool c = false;
            rc = queues_coupled(ctx, o.stream, o.cus, s, &c);
            if (rc != LITHOS_OK || c) { bad = true; break; }
        }
        if (!bad) { *out = s; return LITHOS_OK; }
        { std::lock_guard<std::mutex> lk(ctx->park_mu); ctx->parked.push_back(s); }
        if (rc != LITHOS_OK) return rc;
    }
    return fail(LITHOS_EHIP, "no CU-masked queue independent of the other tenants' queues after 8 attempts");
}

struct Scheduler {
    lithos_ctx* ctx;
    std::mutex mu;
    std::condition_variable cv_done;     // a kernel completed
    std::condition_variable cv_work;     // something was submitted
    Core core;
    std::vector<lithos_tenant*> tenants; // index = core tenant index; nullptr once destroyed
    std::vector<hipEvent_t> free_events;
    std::thread tracker;
    bool stop = false;
    int error = LITHOS_OK;               // sticky first launch failure
    char error_text[256] = "";

    explicit Scheduler(lithos_ctx* c) : ctx(c), core(c->cfg, {}) {}

    hipEvent_t get_event()
    {
        if (!free_events.empty()) { hipEvent_t e = free_events.back(); free_events.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return nullptr;
        return e;
    }

    void record_error(int code)
    {
        if (error == LITHOS_OK) { error = code; snprintf(error_text, sizeof error_text, "%s", lithos_last_error()); }
    }

    // queue of tenant t for a set of groups (created on first use)
    hipStream_t stream_for(lithos_tenant* t, uint32_t group_mask)
    {
        if (group_mask == (1u << t->group)) return t->quota->stream;
        auto it = t->streams.find(group_mask);
        if (it != t->streams.end()) return it->second;
        uint32_t mask[LITHOS_MASK_WORDS] = {0};
        for (size_t i = 0; i < tenants.size(); ++i)
            if (tenants[i] && (group_mask >> tenants[i]->group & 1u))
                for (int w = 0; w < LITHOS_MASK_WORDS; ++w) mask[w] |= tenants[i]->quota->mask[w];
        hipStream_t s = nullptr;
        uint32_t words = (ctx->n_cu + 31) / 32;
        if (hipExtStreamCreateWithCUMask(&s, words, mask) != hipSuccess) {
            fail(LITHOS_EHIP, "hipExtStreamCreateWithCUMask failed for a stolen-CU queue");
            return nullptr;
        }
        t->streams[group_mask] = s;
        return s;
    }

    // Launch every atom the core allows for tenant t.  Caller holds mu.
    void pump(lithos_tenant* t)
    {
        lithos_core_atom_t a;
        while (error == LITHOS_OK && core.next_atom(t->core_idx, now_us(), &a)) {
            PendingOp& p = t->ops.front();
            hipStream_t s = stream_for(t, a.group_mask);
            if (!s) { record_error(LITHOS_EHIP); return; }
            if (t->last_stream && t->last_stream != s) {
                // atoms of one tenant stay ordered across its queues
                if (hipEventRecord(t->switch_ev, t->last_stream) != hipSuccess ||
                    hipStreamWaitEvent(s, t->switch_ev, 0) != hipSuccess) {
                    fail(LITHOS_EHIP, "queue switch: event record/wait failed");
                    record_error(LITHOS_EHIP);
                    return;
                }
            }
            t->last_stream = s;
            int dies = ctx->n_xcd;
            AtomArgs args = make_atom(ctx, p.plan, a.lo, a.hi, dies);
            int rc = op_launch(p.op, p.plan, args, s);
            if (rc != LITHOS_OK) { record_error(rc); return; }
            Fly f;
            f.atom_id = a.atom_id;
            f.ev = get_event();
            f.t_launch = now_us();
            f.kernel_done = (a.hi >= p.plan.total) ? p.kernel_id : 0;
            if (!f.ev || hipEventRecord(f.ev, s) != hipSuccess) {
                fail(LITHOS_EHIP, "completion event record failed");
                record_error(LITHOS_EHIP);
                return;
            }
            t->fly.push_back(f);
            if (a.hi >= p.plan.total) t->ops.pop_front();
        }
    }

    // Collect finished atoms of every tenant; returns true if any finished.
    bool reap()
    {
        bool any = false;
        for (lithos_tenant* t : tenants) {
            if (!t) continue;
            while (!t->fly.empty()) {
                Fly& f = t->fly.front();
                hipError_t e = hipEventQuery(f.ev);
                if (e == hipErrorNotReady) break;
                if (e != hipSuccess) { fail(LITHOS_EHIP, "hipEventQuery: %s", hipGetErrorString(e)); record_error(LITHOS_EHIP); }
                double t_now = now_us();
                double measured = t_now - std::max(f.t_launch, t->last_done_us);
                t->last_done_us = t_now;
                uint64_t done = 0;
                core.complete(f.atom_id, t_now, measured, &done);
                if (done) t->completed.fetch_add(1);
                free_events.push_back(f.ev);
                t->fly.pop_front();
                any = true;
            }
        }
        return any;
    }

    void pump_all()
    {
        for (int pass = 0; pass < 2; ++pass)            // high-priority tenants first
            for (lithos_tenant* t : tenants)
                if (t && (t->cls == LITHOS_CLASS_HP) == (pass == 0)) pump(t);
    }

    void run()
    {
        (void)hipSetDevice(ctx->device);
        std::unique_lock<std::mutex> lk(mu);
        int idle_spins = 0;
        while (!stop) {
            bool any = reap();
            if (any) { pump_all(); cv_done.notify_all(); }
            bool inflight = false;
            for (lithos_tenant* t : tenants) if (t && !t->fly.empty()) inflight = true;
            if (inflight || any) {
                idle_spins = 0;
                lk.unlock();                 // let submitters in between polls
                __builtin_ia32_pause();
                lk.lock();
            } else if (++idle_spins < 2000) {
                lk.unlock();
                __builtin_ia32_pause();
                lk.lock();
            } else {
                cv_work.wait_for(lk, std::chrono::milliseconds(2));
            }
        }
    }
};

void sched_shutdown(lithos_ctx* ctx)
{
    Scheduler* s = ctx->sched;
    if (!s) return;
    {
        std::lock_guard<std::mutex> lk(s->mu);
        s->stop = true;
    }
    s->cv_work.notify_all();
    if (s->tracker.joinable()) s->tracker.join();
    for (hipEvent_t e : s->free_events) (void)hipEventDestroy(e);
    delete s;
    ctx->sched = nullptr;
}

static std::mutex g_sched_create_mu;

static Scheduler* get_sched(lithos_ctx* ctx)
{
    std::lock_guard<std::mutex> lk(g_sched_create_mu);
    if (!ctx->sched) {
        ctx->sched = new Scheduler(ctx);
        ctx->sched->tracker = std::thread([s = ctx->sched] { s->run(); });
    }
    return ctx->sched;
}

} // namespace lithos

using namespace lithos;

extern "C" {

int lithos_tenant_create(lithos_ctx_t* ctx, int cls, const lithos_partition_t* quota, lithos_tenant_t** out)
{
    if (!ctx || !out) return fail(LITHOS_EINVAL, "lithos_tenant_create: null argument");
    if (cls != LITHOS_CLASS_HP && cls != LITHOS_CLASS_BE) return fail(LITHOS_EINVAL, "lithos_tenant_create: unknown class %d", cls);
    (void)hipSetDevice(ctx->device);
    auto* t = new lithos_tenant();
    t->ctx = ctx;
    t->cls = cls;
    t->quota = quota;
    if (!quota) {
        t->passthrough = true;
        hipError_t e = hipStreamCreateWithFlags(&t->own_stream, hipStreamNonBlocking);
        if (e != hipSuccess) { delete t; return fail(LITHOS_EHIP, "hipStreamCreateWithFlags: %s", hipGetErrorString(e)); }
    } else {
        if (quota->ctx != ctx) { delete t; return fail(LITHOS_EINVAL, "lithos_tenant_create: quota belongs to another context"); }
        Scheduler* s = get_sched(ctx);
        std::lock_guard<std::mutex> lk(s->mu);
        for (lithos_tenant* o : s->tenants)
            if (o)
                for (int w = 0; w < LITHOS_MASK_WORDS; ++w)
                    if (o->quota->mask[w] & quota->mask[w]) { delete t; return fail(LITHOS_EMASK, "lithos_tenant_create: quota overlaps another tenant's"); }
        hipError_t e = hipEventCreateWithFlags(&t->switch_ev, hipEventDisableTiming);
        if (e != hipSuccess) { delete t; return fail(LITHOS_EHIP, "hipEventCreateWithFlags: %s", hipGetErrorString(e)); }
        t->group = s->core.add_group(quota->n_cus);
        if (t->group < 0) { (void)hipEventDestroy(t->switch_ev); delete t; return fail(LITHOS_ELIMIT, "lithos_tenant_create: at most 32 tenants per context"); }
        t->core_idx = s->core.add_tenant(cls, 1u << t->group);
        s->tenants.resize(t->core_idx + 1, nullptr);
        // Queues of different tenants must not share a command-processor pipe: give this
        // tenant a quota queue, and each pair of tenants their quota-plus-stolen queues,
        // that are independent of every queue of the other tenants.
        std::vector<OtherQueue> others;
        for (lithos_tenant* o : s->tenants)
            if (o) {
                others.push_back({o->quota->stream, o->quota->n_cus});
                for (auto& kv : o->streams) others.push_back({kv.second, s->core.cus_of(kv.first)});
            }
        if (!others.empty()) {
            lithos_partition* q = const_cast<lithos_partition*>(quota);
            bool coupled = false;
            int rc = LITHOS_OK;
            for (const OtherQueue& o : others) {
                bool c = false;
                rc = queues_coupled(ctx, o.stream, o.cus, q->stream, &c);
                if (rc != LITHOS_OK) break;
                coupled = coupled || c;
            }
            if (rc == LITHOS_OK && coupled) {
                hipStream_t fresh = nullptr;
                rc = make_decoupled_stream(ctx, q->mask, others, &fresh);
                if (rc == LITHOS_OK) {
                    std::lock_guard<std::mutex> pk(ctx->park_mu);
                    ctx->parked.push_back(q->stream);           // parked, not destroyed: positions stay
                    q->stream = fresh;
                }
            }
            // quota + stolen queues, both directions, for every pair with an existing tenant
            for (size_t i = 0; i < s->tenants.size() && rc == LITHOS_OK; ++i) {
                lithos_tenant* o = s->tenants[i];
                if (!o) continue;
                const uint32_t gm = (1u << t->group) | (1u << o->group);
                uint32_t mask[LITHOS_MASK_WORDS];
                for (int w = 0; w < LITHOS_MASK_WORDS; ++w) mask[w] = q->mask[w] | o->quota->mask[w];
                const int cus = q->n_cus + o->quota->n_cus;
                // the new tenant's union queue: independent of all queues of all other tenants
                hipStream_t mine = nullptr;
                rc = make_decoupled_stream(ctx, mask, others, &mine);
                if (rc != LITHOS_OK) break;
                t->streams[gm] = mine;
                // the existing tenant's union queue: independent of this tenant's queues (and third parties')
                std::vector<OtherQueue> foes;
                foes.push_back({q->stream, q->n_cus});
                for (auto& kv : t->streams) foes.push_back({kv.second, cus});
                for (lithos_tenant* x : s->tenants)
                    if (x && x != o) {
                        foes.push_back({x->quota->stream, x->quota->n_cus});
                        for (auto& kv : x->streams) foes.push_back({kv.second, s->core.cus_of(kv.first)});
                    }
                hipStream_t theirs = nullptr;
                rc = make_decoupled_stream(ctx, mask, foes, &theirs);
                if (rc != LITHOS_OK) break;
                o->streams[gm] = theirs;
                others.push_back({theirs, cus});
            }
            if (rc != LITHOS_OK) {
                for (auto& kv : t->streams) retire_stream(ctx, kv.second);
                (void)hipEventDestroy(t->switch_ev);
                delete t;
                return rc;
            }
        }
        s->tenants[t->core_idx] = t;
    }
    ctx->live_tenants.fetch_add(1);
    *out = t;
    return LITHOS_OK;
}

int lithos_submit(lithos_tenant_t* t, const lithos_op_t* op, uint64_t* ticket_out)
{
    if (!t || !op) return fail(LITHOS_EINVAL, "lithos_submit: null argument");
    (void)hipSetDevice(t->ctx->device);
    PendingOp p;
    p.op = *op;
    int rc = op_plan(p.op, &p.plan);
    if (rc != LITHOS_OK) return rc;
    if ((rc = check_counters(t->ctx, p.plan)) != LITHOS_OK) return rc;
    if (t->passthrough) {
        std::lock_guard<std::mutex> lk(t->pt_mu);
        rc = op_launch(p.op, p.plan, make_atom(t->ctx, p.plan, 0, p.plan.total, t->ctx->n_xcd), t->own_stream);
        if (rc != LITHOS_OK) return rc;
        Fly f;
        f.atom_id = 0;
        f.t_launch = now_us();
        f.kernel_done = ++t->pt_kernel_seq;
        hipError_t e = hipEventCreateWithFlags(&f.ev, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventRecord(f.ev, t->own_stream);
        if (e != hipSuccess) return fail(LITHOS_EHIP, "pass-through completion event: %s", hipGetErrorString(e));
        t->fly.push_back(f);
        t->submitted.fetch_add(1);
        t->ctx->pt_kernels.fetch_add(1);
        t->pt_stats.kernels++;
        t->pt_stats.atoms++;
        if (ticket_out) *ticket_out = f.kernel_done;
        return LITHOS_OK;
    }
    Scheduler* s = t->ctx->sched;
    std::lock_guard<std::mutex> lk(s->mu);
    if (s->error != LITHOS_OK) return fail(s->error, "scheduler stopped after an error: %s", s->error_text);
    p.kernel_id = s->core.submit(t->core_idx, p.plan.total, p.plan.wg_per_cu);
    t->ops.push_back(p);
    uint64_t seq = t->submitted.fetch_add(1) + 1;
    if (ticket_out) *ticket_out = seq;
    s->pump(t);
    if (s->error != LITHOS_OK) return fail(s->error, "%s", s->error_text);
    s->cv_work.notify_one();
    return LITHOS_OK;
}

int lithos_sync_mark(lithos_tenant_t* t)
{
    if (!t) return fail(LITHOS_EINVAL, "lithos_sync_mark: null tenant");
    if (t->passthrough) return LITHOS_OK;
    Scheduler* s = t->ctx->sched;
    std::lock_guard<std::mutex> lk(s->mu);
    s->core.sync_mark(t->core_idx);
    return LITHOS_OK;
}

static void pt_reap(lithos_tenant_t* t, bool block)
{
    std::lock_guard<std::mutex> lk(t->pt_mu);
    while (!t->fly.empty()) {
        Fly& f = t->fly.front();
        hipError_t e = block ? hipEventSynchronize(f.ev) : hipEventQuery(f.ev);
        if (e == hipErrorNotReady) break;
        (void)hipEventDestroy(f.ev);
        t->completed.fetch_add(1);
        t->fly.pop_front();
    }
}

int lithos_sync(lithos_tenant_t* t)
{
    if (!t) return fail(LITHOS_EINVAL, "lithos_sync: null tenant");
    (void)hipSetDevice(t->ctx->device);
    if (t->passthrough) { pt_reap(t, true); return LITHOS_OK; }
    Scheduler* s = t->ctx->sched;
    std::unique_lock<std::mutex> lk(s->mu);
    s->core.sync_mark(t->core_idx);
    const uint64_t target = t->submitted.load();
    s->cv_done.wait(lk, [&] { return t->completed.load() >= target || s->error != LITHOS_OK; });
    if (s->error != LITHOS_OK) return fail(s->error, "%s", s->error_text);
    return LITHOS_OK;
}

int lithos_poll(lithos_tenant_t* t, uint64_t ticket, int* done_out)
{
    if (!t || !done_out) return fail(LITHOS_EINVAL, "lithos_poll: null argument");
    if (t->passthrough) { (void)hipSetDevice(t->ctx->device); pt_reap(t, false); }
    *done_out = t->completed.load() >= ticket ? 1 : 0;
    return LITHOS_OK;
}

int lithos_tenant_stats(lithos_tenant_t* t, lithos_stats_t* out)
{
    if (!t || !out) return fail(LITHOS_EINVAL, "lithos_tenant_stats: null argument");
    if (t->passthrough) { *out = t->pt_stats; return LITHOS_OK; }
    Scheduler* s = t->ctx->sched;
    std::lock_guard<std::mutex> lk(s->mu);
    *out = s->core.stats(t->core_idx);
    return LITHOS_OK;
}

int lithos_stats(lithos_ctx_t* ctx, lithos_stats_t* out)
{
    if (!ctx || !out) return fail(LITHOS_EINVAL, "lithos_stats: null argument");
    memset(out, 0, sizeof *out);
    if (Scheduler* s = ctx->sched) {
        std::lock_guard<std::mutex> lk(s->mu);
        *out = s->core.totals();
    }
    const uint64_t pt = ctx->pt_kernels.load();     // pass-through kernels: one whole launch each
    out->kernels += pt;
    out->atoms += pt;
    return LITHOS_OK;
}

int lithos_tenant_destroy(lithos_tenant_t* t)
{
    if (!t) return fail(LITHOS_EINVAL, "lithos_tenant_destroy: null tenant");
    int rc = lithos_sync(t);
    (void)rc;
    if (t->passthrough) {
        (void)hipStreamDestroy(t->own_stream);
    } else {
        Scheduler* s = t->ctx->sched;
        std::lock_guard<std::mutex> lk(s->mu);
        for (auto& kv : t->streams) { (void)hipStreamSynchronize(kv.second); retire_stream(t->ctx, kv.second); }
        (void)hipEventDestroy(t->switch_ev);
        s->tenants[t->core_idx] = nullptr;   // its core slot stays (idle for ever): others may steal its CUs
    }
    if (t->ctx->live_tenants.fetch_sub(1) == 1) drain_parked(t->ctx);
    delete t;
    return LITHOS_OK;
}

// ---- load generators ----------------------------------------------------------------

int lithos_drive_open_loop(lithos_tenant_t* t, const lithos_op_t* ops, int ops_per_request, int n_variants,
                           const double* arrivals_s, int n_requests, double* latency_us_out)
{
    if (!t || !ops || !arrivals_s || !latency_us_out || ops_per_request <= 0 || n_variants <= 0 || n_requests < 0)
        return fail(LITHOS_EINVAL, "lithos_drive_open_loop: bad argument");
    std::deque<std::pair<int, uint64_t>> pending;      // (request, ticket of its last kernel)
    const double t0 = now_us();
    int next = 0;
    while (next < n_requests || !pending.empty()) {
        // completions first: their time stamp is the latency's end
        while (!pending.empty()) {
            int done = 0;
            int rc = lithos_poll(t, pending.front().second, &done);
            if (rc != LITHOS_OK) return rc;
            if (!done) break;
            int r = pending.front().first;
            latency_us_out[r] = now_us() - (t0 + arrivals_s[r] * 1e6);
            pending.pop_front();
        }
        if (next < n_requests) {
            double due = t0 + arrivals_s[next] * 1e6;
            double wait = due - now_us();
            if (wait <= 0) {
                const lithos_op_t* req = ops + (size_t)(next % n_variants) * ops_per_request;
                uint64_t ticket = 0;
                for (int i = 0; i < ops_per_request; ++i) {
                    int rc = lithos_submit(t, &req[i], &ticket);
                    if (rc != LITHOS_OK) return rc;
                }
                int rc = lithos_sync_mark(t);
                if (rc != LITHOS_OK) return rc;
                pending.emplace_back(next, ticket);
                ++next;
                continue;
            }
            if (pending.empty() && wait > 300.0)
                std::this_thread::sleep_for(std::chrono::microseconds((long)(wait - 200.0)));
        }
        __builtin_ia32_pause();
    }
    return LITHOS_OK;
}

} // extern "C"

struct lithos_driver {
    lithos_tenant* tenant;
    std::vector<lithos_op_t> ops;
    int depth;
    std::thread th;
    std::atomic<bool> stop{false};
    uint64_t iterations = 0;
    double seconds = 0.0;
    int rc = LITHOS_OK;
};

extern "C" {

int lithos_drive_closed_loop_start(lithos_tenant_t* t, const lithos_op_t* ops, int ops_per_iter, int depth, lithos_driver_t** out)
{
    if (!t || !ops || !out || ops_per_iter <= 0 || depth <= 0) return fail(LITHOS_EINVAL, "lithos_drive_closed_loop_start: bad argument");
    auto* d = new lithos_driver();
    d->tenant = t;
    d->ops.assign(ops, ops + ops_per_iter);
    d->depth = depth;
    d->th = std::thread([d] {
        std::deque<uint64_t> tickets;
        const double t0 = now_us();
        double t_last = t0;
        while (true) {
            while (!d->stop.load() && (int)tickets.size() < d->depth) {
                uint64_t ticket = 0;
                for (const lithos_op_t& op : d->ops)
                    if ((d->rc = lithos_submit(d->tenant, &op, &ticket)) != LITHOS_OK) return;
                if ((d->rc = lithos_sync_mark(d->tenant)) != LITHOS_OK) return;
                tickets.push_back(ticket);
            }
            if (tickets.empty()) break;
            int done = 0;
            if ((d->rc = lithos_poll(d->tenant, tickets.front(), &done)) != LITHOS_OK) return;
            if (done) {
                tickets.pop_front();
                d->iterations++;
                t_last = now_us();
                d->seconds = (t_last - t0) * 1e-6;
            } else {
                std::this_thread::sleep_for(std::chrono::microseconds(20));
            }
        }
    });
    *out = d;
    return LITHOS_OK;
}

int lithos_drive_closed_loop_stop(lithos_driver_t* d, uint64_t* iterations_out, double* seconds_out)
{
    if (!d) return fail(LITHOS_EINVAL, "lithos_drive_closed_loop_stop: null driver");
    d->stop.store(true);
    if (d->th.joinable()) d->th.join();
    if (iterations_out) *iterations_out = d->iterations;
    if (seconds_out) *seconds_out = d->seconds;
    int rc = d->rc;
    delete d;
    return rc;
}

} // extern "C"

extern "C" int lithos_partitions_coupled(lithos_ctx_t* ctx, const lithos_partition_t* busy, const lithos_partition_t* probe, int* coupled_out)
{
    if (!ctx || !busy || !probe || !coupled_out || busy == probe) return fail(LITHOS_EINVAL, "lithos_partitions_coupled: bad argument");
    (void)hipSetDevice(ctx->device);
    bool c = false;
    int rc = queues_coupled(ctx, busy->stream, busy->n_cus, probe->stream, &c);
    if (rc != LITHOS_OK) return rc;
    *coupled_out = c ? 1 : 0;
    return LITHOS_OK;
}
