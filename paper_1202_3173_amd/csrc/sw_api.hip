// Host side of the library: the C ABI of include/sw_gemm.h, the BFS/DFS schedule planner and the executor
// that walks the recursion tree and enqueues kernels on one HIP stream.  No device memory is allocated here.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <string>
#include <vector>

#include "sw_internal.h"

namespace sw {

// ---- error text ---------------------------------------------------------------------------------------------

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

int hip_fail(hipError_t e, const char* what)
{
    set_error("%s: %s", what, hipGetErrorString(e));
    return SW_EHIP;
}

// ---- library state --------------------------------------------------------------------------------------------

// Process-wide settings.  Every entry point reads them ONCE, on entry (current_opts, library_state); nothing
// below the entry points looks at them, so a setter called from another thread affects later calls only.
static void* g_ws = nullptr;
static int64_t g_ws_bytes = 0;
static hipStream_t g_stream = nullptr;
static std::atomic<int> g_odd_mode{SW_ODD_PAD};   // what to do when 2^levels does not divide n
static std::atomic<int> g_overlap{1};             // 0: one stream.  > 0: additions and leaf products on separate streams (when
                                                  // the step order has a DFS step); the addition kernels beside the leaf
                                                  // products then run with a limited number of workgroups: 1 = sized to the
                                                  // work, k > 1 = k
static std::atomic<bool> g_prof_on{false};

CallOpts current_opts() { return CallOpts{g_overlap.load(), g_odd_mode.load(), g_prof_on.load(), false}; }

void library_state(void** ws, int64_t* ws_bytes, hipStream_t* stream)
{
    *ws = g_ws;
    *ws_bytes = g_ws_bytes;
    *stream = g_stream;
}

// ---- record-only runs ---------------------------------------------------------------------------------------------

static thread_local Tracer* t_tracer = nullptr;
static thread_local int64_t t_withhold = -1;   // see Exec::withhold; set by sw_trace_gemm only
Tracer* tracer() { return t_tracer; }
void set_tracer(Tracer* t) { t_tracer = t; }

// ---- profiling ------------------------------------------------------------------------------------------------

struct Profiler {
    struct Rec { hipEvent_t e0, e1; int cls; double work; };
    std::mutex mu;              // records may come from several host threads
    std::vector<Rec> recs;
    std::vector<hipEvent_t> pool;
    hipEvent_t take()
    {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
};

static Profiler g_prof;

Profiler* profiler() { return g_prof_on.load() ? &g_prof : nullptr; }

// Brackets one launch (or a short run of launches on one stream) with two events.  The record is appended
// only when both events have been recorded, so records of concurrent callers never interleave.
void prof_begin(Profiler* p, hipStream_t s, int cls, double work, ProfMark* m)
{
    m->e0 = m->e1 = nullptr;
    m->cls = cls;
    m->work = work;
    if (!p) return;
    {
        std::lock_guard<std::mutex> g(p->mu);
        m->e0 = p->take();
        m->e1 = p->take();
    }
    if (m->e0) (void)hipEventRecord(m->e0, s);
}

void prof_end(Profiler* p, hipStream_t s, const ProfMark* m)
{
    if (!p) return;
    if (m->e1) (void)hipEventRecord(m->e1, s);
    std::lock_guard<std::mutex> g(p->mu);
    p->recs.push_back(Profiler::Rec{m->e0, m->e1, m->cls, m->work});
}

// ---- schedule checks and the planner ------------------------------------------------------------------------------

bool schedule_ok(const char* s, int levels)
{
    if ((int)strlen(s) != levels) return false;
    for (int i = 0; i < levels; ++i)
        if (s[i] != 'B' && s[i] != 'D') return false;
    return true;
}

int check_shape(int64_t n, int levels)
{
    if (n < 0 || levels < 0 || levels > SW_MAX_LEVELS) {
        set_error("bad shape: n = %lld, levels = %d (0 <= levels <= %d)", (long long)n, levels, SW_MAX_LEVELS);
        return SW_EINVAL;
    }
    if (n > 0 && ((int64_t)1 << levels) > n) {
        set_error("2^levels = %lld exceeds n = %lld", (long long)((int64_t)1 << levels), (long long)n);
        return SW_EINVAL;
    }
    if (n > 200000) {
        set_error("n = %lld is above the supported maximum of 200000", (long long)n);
        return SW_EINVAL;
    }
    return SW_OK;
}

// Total workspace bytes for (n, schedule): with padding the recursion runs on the next multiple of 2^levels
// and needs padded copies of A, B, C; with peeling it runs in place on the previous multiple.
static Dims padded_dims(Dims d, int levels) { return Dims{padded_n(d.m, levels), padded_n(d.n, levels), padded_n(d.k, levels)}; }
static Dims floor_dims(Dims d, int levels)
{
    const int64_t q = (int64_t)1 << levels;
    return Dims{d.m - d.m % q, d.n - d.n % q, d.k - d.k % q};
}

int64_t total_need(Dims d, int levels, const char* sched) { return total_need(d, levels, sched, g_odd_mode.load()); }
int plan(Dims d, int levels, int64_t budget, char* out) { return plan(d, levels, budget, out, g_odd_mode.load(), g_overlap.load() != 0); }

int64_t total_need(Dims d, int levels, const char* sched, int odd_mode)
{
    if (d.m == 0 || d.n == 0 || d.k == 0) return 0;
    // peeling: the recursion runs in place on the previous multiples of 2^levels, no copies
    if (odd_mode == SW_ODD_PEEL) return ws_need_bytes(floor_dims(d, levels), sched, 1);
    // peeling level by level: in place on the extents as they are (every step halves them, rounding down)
    if (odd_mode == SW_ODD_PEEL_LEVELS) return ws_need_bytes(d, sched, 1);
    const Dims p = padded_dims(d, levels);
    int64_t bytes = ws_need_bytes(p, sched, 1);
    if (p.m != d.m || p.n != d.n || p.k != d.k)
        bytes += (ws_mat_elems(p.m, p.k) + ws_mat_elems(p.k, p.n) + ws_mat_elems(p.m, p.n)) * (int64_t)sizeof(double);
    return bytes;
}

int plan(Dims d, int levels, int64_t budget, char* out, int odd_mode, bool overlap)
{
    // The candidates are the Limited-Memory shapes of Section 3.4: l DFS steps followed by k = levels - l BFS
    // steps.  Each one that fits is scored with the cost model (leaf products at the kernel's measured rate for
    // the leaf shape and the fill of its launches, additions at their measured HBM rate, the additions next to
    // the leaves beside the products when they overlap).  The model is good to about 5 %, and the best orders
    // lie closer together than that, so among the candidates within 6 % of the best score the structure decides:
    // an even k with a DFS step above (the BFS steps then run as fused pairs and their additions beside the leaf
    // products of the neighbouring launches) before the rest; then the score.  An order whose leaf launches
    // would not fill the workgroup slots of the machine three times over is left out while another one remains.
    // On the measured sweeps of all step orders at n = 4096 ... 47040 this picks an order within 0.3 % of the best.
    struct Cand { char s[SW_MAX_LEVELS + 1]; double t; bool paired, full; };
    Cand cand[SW_MAX_LEVELS + 1];
    int nc = 0;
    const Dims p = odd_mode == SW_ODD_PEEL ? floor_dims(d, levels) : (odd_mode == SW_ODD_PEEL_LEVELS ? d : padded_dims(d, levels));
    for (int l = 0; l <= levels; ++l) {
        Cand c;
        for (int i = 0; i < levels; ++i) c.s[i] = i < l ? 'D' : 'B';
        c.s[levels] = '\0';
        if (total_need(d, levels, c.s, odd_mode) > budget) continue;
        c.t = modelled_order(d, levels, c.s, budget, overlap, odd_mode);
        const int k = levels - l;
        c.paired = overlap && l >= 1 && k >= 2 && k % 2 == 0;
        double tiles = (double)(((p.m >> levels) + 127) / 128) * (double)(((p.n >> levels) + 127) / 128);
        for (int i = 0; i < k; ++i) tiles *= 7.0;
        c.full = tiles >= 3.0 * 512.0 || levels == 0;
        cand[nc++] = c;
    }
    if (nc == 0) {
        set_error("no step order for %lld x %lld x %lld, levels = %d fits a workspace of %lld bytes (all-DFS needs %lld)",
                  (long long)d.m, (long long)d.n, (long long)d.k, levels, (long long)budget,
                  (long long)total_need(d, levels, std::string((size_t)levels, 'D').c_str(), odd_mode));
        return SW_ENOMEM;
    }
    bool any_full = false;
    for (int i = 0; i < nc; ++i) any_full = any_full || cand[i].full;
    double best_t = -1.0;
    for (int i = 0; i < nc; ++i)
        if ((cand[i].full || !any_full) && (best_t < 0.0 || cand[i].t < best_t)) best_t = cand[i].t;
    int pick = -1;
    for (int i = 0; i < nc; ++i) {
        if ((!cand[i].full && any_full) || cand[i].t > 1.06 * best_t) continue;
        if (pick < 0 || (cand[i].paired && !cand[pick].paired) || (cand[i].paired == cand[pick].paired && cand[i].t < cand[pick].t)) pick = i;
    }
    memcpy(out, cand[pick].s, (size_t)levels + 1);
    return SW_OK;
}

// ---- three in-order streams with tracked dependencies ----------------------------------------------------------
//
// The additions are bound by HBM and the leaf products by the matrix cores, so they are run side by side:
// kernels that FORM operands (pre-additions) go to one stream, leaf products to a second, kernels that FOLD
// products into C (post-additions) stay on the caller's stream.  Every kernel declares the address ranges it
// reads and writes; before a launch the stream is made to wait (hipStreamWaitEvent) for every earlier kernel of
// ANOTHER stream that conflicts with it (read-after-write, write-after-read, write-after-write).  Order inside
// a stream needs nothing.  Correctness therefore never rests on how the executor happens to interleave its
// calls: a buffer used too early is a declared conflict and becomes a wait.  All waits point to kernels
// submitted earlier, so they cannot form a cycle.

enum { S_POST = 0, S_PRE = 1, S_MM = 2, NSTREAM = 3 };

struct Range { uintptr_t lo, hi; };

// bounding byte range of `count` matrices of rows x cols
static Range rng(const Mat& m, int64_t rows, int64_t cols, int64_t count = 1)
{
    const uintptr_t lo = (uintptr_t)m.p;
    return Range{lo, lo + (uintptr_t)(((count - 1) * m.stride + (rows - 1) * m.ld + cols) * (int64_t)sizeof(double))};
}

struct Sched {
    static constexpr int RING = 256;
    hipStream_t st[NSTREAM] = {nullptr, nullptr, nullptr};
    bool multi = false;
    uint64_t seq[NSTREAM] = {0, 0, 0};              // kernels issued per stream
    uint64_t waited[NSTREAM][NSTREAM] = {};         // waited[c][s]: stream c is ordered after kernel number .. of s
    struct Acc { uintptr_t lo, hi; uint64_t seq; uint8_t stream; bool write; };
    std::vector<Acc> live;
    hipError_t err = hipSuccess;
    Tracer* tr = nullptr;                           // record-only run: events and waits are written down, not issued

    // Two internal streams and the events of one product in flight on the host side.  A call takes a lane for
    // its duration (from entry to return; the GPU work it enqueued may still run) and hands it back, so two
    // host threads inside the library at once never share events, while consecutive calls of one thread reuse
    // the same streams.  Lanes are created on demand and live until the process ends.
    struct Lane { hipStream_t pre = nullptr, mm = nullptr; hipEvent_t ring[NSTREAM][RING]; hipEvent_t entry = nullptr; bool busy = false; };
    Lane* lane = nullptr;

    static std::mutex& lanes_mutex() { static std::mutex m; return m; }
    static std::vector<Lane*>& lanes() { static std::vector<Lane*> v; return v; }

    static Lane* take_lane()
    {
        std::lock_guard<std::mutex> g(lanes_mutex());
        for (Lane* l : lanes())
            if (!l->busy) { l->busy = true; return l; }
        Lane* l = new Lane;
        bool good = hipStreamCreateWithFlags(&l->pre, hipStreamNonBlocking) == hipSuccess &&
                    hipStreamCreateWithFlags(&l->mm, hipStreamNonBlocking) == hipSuccess &&
                    hipEventCreateWithFlags(&l->entry, hipEventDisableTiming) == hipSuccess;
        for (int s = 0; s < NSTREAM && good; ++s)
            for (int i = 0; i < RING && good; ++i)
                good = hipEventCreateWithFlags(&l->ring[s][i], hipEventDisableTiming) == hipSuccess;
        if (!good) { (void)hipGetLastError(); delete l; return nullptr; }   // no streams or events to be had (what was created stays)
        l->busy = true;
        lanes().push_back(l);
        return l;
    }
    static void give_lane(Lane* l)
    {
        std::lock_guard<std::mutex> g(lanes_mutex());
        l->busy = false;
    }

    void note(hipError_t e) { if (err == hipSuccess && e != hipSuccess) err = e; }

    // slot -1 is the entry event (recorded on the caller's stream), slot i >= 0 is ring[s][i]
    void ev_record(int s, int slot)
    {
        if (tr) { tr->record(s, slot); return; }
        note(hipEventRecord(slot < 0 ? lane->entry : lane->ring[s][slot], st[s]));
    }
    void ev_wait(int c, int s, int slot)
    {
        if (tr) { tr->wait(c, s, slot); return; }
        note(hipStreamWaitEvent(st[c], slot < 0 ? lane->entry : lane->ring[s][slot], 0));
    }

    // the caller's stream carries the post-additions; the two others first wait for what the caller queued
    void start(hipStream_t caller, bool want_multi)
    {
        tr = tracer();
        if (tr) caller = (hipStream_t)(uintptr_t)1;
        st[S_POST] = st[S_PRE] = st[S_MM] = caller;
        multi = false;
        if (!want_multi) return;
        if (tr) {
            st[S_PRE] = (hipStream_t)(uintptr_t)2;
            st[S_MM] = (hipStream_t)(uintptr_t)3;
        } else {
            // under stream capture everything stays on the capturing stream: the graph then holds the kernels in
            // program order (forking a capture over the library's own streams is not attempted)
            hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
            if (hipStreamIsCapturing(caller, &cap) != hipSuccess) { (void)hipGetLastError(); cap = hipStreamCaptureStatusNone; }
            if (cap != hipStreamCaptureStatusNone) return;
            lane = take_lane();
            if (!lane) return;                          // stay on one stream
            st[S_PRE] = lane->pre;
            st[S_MM] = lane->mm;
        }
        multi = true;
        ev_record(S_POST, -1);
        ev_wait(S_PRE, S_POST, -1);
        ev_wait(S_MM, S_POST, -1);
    }

    void wait_for(int c, int s, uint64_t n)          // stream c waits for kernel number n (1-based) of stream s
    {
        if (c == s || waited[c][s] >= n) return;
        const uint64_t use = (seq[s] - n < (uint64_t)RING) ? n : seq[s];   // its own event, or a later one
        ev_wait(c, s, (int)((use - 1) % RING));
        waited[c][s] = use;
    }

    static bool hit(const Range& r, const Acc& a) { return r.lo < a.hi && a.lo < r.hi; }

    void acquire(int c, const Range* reads, int nr, const Range* writes, int nw)
    {
        if (!multi) return;
        for (const Acc& a : live) {
            if (a.stream == c || waited[c][a.stream] >= a.seq) continue;
            bool conflict = false;
            for (int i = 0; i < nw && !conflict; ++i) conflict = hit(writes[i], a);
            if (a.write)
                for (int i = 0; i < nr && !conflict; ++i) conflict = hit(reads[i], a);
            if (conflict) wait_for(c, a.stream, a.seq);
        }
    }

    void release(int c, const Range* reads, int nr, const Range* writes, int nw)
    {
        if (!multi) return;
        ++seq[c];
        ev_record(c, (int)((seq[c] - 1) % RING));
        for (int i = 0; i < nr; ++i) live.push_back(Acc{reads[i].lo, reads[i].hi, seq[c], (uint8_t)c, false});
        for (int i = 0; i < nw; ++i) live.push_back(Acc{writes[i].lo, writes[i].hi, seq[c], (uint8_t)c, true});
        if (live.size() >= 512) prune();
    }

    void join_all()
    {
        for (int c = 0; c < NSTREAM; ++c)
            for (int s = 0; s < NSTREAM; ++s)
                if (seq[s] > 0) wait_for(c, s, seq[s]);
    }

    void prune()
    {
        // forget what every other stream is already ordered after; if that does not help, order everything
        auto settled = [&](const Acc& a) {
            for (int c = 0; c < NSTREAM; ++c)
                if (c != a.stream && waited[c][a.stream] < a.seq) return false;
            return true;
        };
        size_t k = 0;
        for (size_t i = 0; i < live.size(); ++i)
            if (!settled(live[i])) live[k++] = live[i];
        live.resize(k);
        if (live.size() >= 384) {
            if (tr) tr->joined((int64_t)live.size());
            join_all();
            live.clear();
        }
    }

    // the caller's stream ends up ordered after everything
    void finish()
    {
        if (multi)
            for (int s = 1; s < NSTREAM; ++s)
                if (seq[s] > 0) wait_for(S_POST, s, seq[s]);
        if (lane) { give_lane(lane); lane = nullptr; }
    }
    ~Sched() { if (lane) give_lane(lane); }
};

// ---- the executor ----------------------------------------------------------------------------------------------

struct Exec {
    Sched sc;
    char* ws;
    int64_t ws_bytes;
    int64_t used = 0;
    const char* sched;
    int levels;
    uint32_t rich = 0;      // DFS levels that keep BFS-style storage (choose_options)
    bool dbl = false;       // the buffers next to the leaves exist twice and alternate between launches
    uint64_t flip = 0;
    int cap_bg = 0;               // workgroup cap of the addition kernels that run beside leaf products (0: none)
    int cap_fixed = 0;            // > 1: the caller's cap for the kernels beside the leaf products; else sized per step
    bool bg = false;              // the operations being issued are the leaf-side ones of a double-buffered step
    Profiler* prof;
    hipError_t err = hipSuccess;
    bool peel_levels = false;     // SW_ODD_PEEL_LEVELS: peel the odd row / column / inner index at every level
    int64_t declared = 0;         // ranges declared to the dependency tracker so far
    int64_t withhold = -1;        // record-only runs: the number of ONE declared range to keep from the tracker (a
                                  // planted mistake, which the checker of the record must then find); -1: none

    double* take(int64_t elems)
    {
        double* p = reinterpret_cast<double*>(ws + used);
        if (sc.tr) sc.tr->take(used, elems * (int64_t)sizeof(double));
        used += elems * (int64_t)sizeof(double);
        return p;
    }
    void pop_to(int64_t mark)
    {
        used = mark;
        if (sc.tr) sc.tr->pop(mark);
    }

    void note(hipError_t e) { if (err == hipSuccess && e != hipSuccess) err = e; }

    // Workgroups for the addition kernels that run beside a leaf launch: enough to move their bytes (`units`
    // elements per parent, three kernels) in about two thirds of the time the launch takes (`per` products of
    // size m per parent at about 70 TFLOP/s), at the 20 GB/s a resident streaming workgroup sustains beside the
    // products; more than 256 would mean they cannot keep up anyway, then they run uncapped and the two simply
    // take turns.  n = 94080, leaves of 2940: 0.4 TB/s needed, 32 workgroups.
    static int leaf_side_cap(double units, int64_t live, int per, Dims leaf)
    {
        const double bytes = 8.0 * units * (double)live;
        const double seconds = (double)per * (double)live * 2.0 * (double)leaf.m * (double)leaf.n * (double)leaf.k / 70e12;
        const double need = bytes / (0.65 * seconds);            // bytes per second
        const double groups = need / 20e9;
        if (groups > 256.0) return 0;
        return groups < 32.0 ? 32 : (int)(groups + 0.5);
    }

    // bytes moved by a kernel with `nin` input and `nout` output matrices of r x c per parent
    static double bytes(int64_t live, int64_t r, int64_t c, int nin, int nout) { return 8.0 * live * (double)r * (double)c * (nin + nout); }

    // One kernel: on stream `s`, after everything of the other streams it conflicts with.
    template <class F>
    void op(int s, int cls, double work, std::initializer_list<Range> reads, std::initializer_list<Range> writes, F&& launch)
    {
        if (err != hipSuccess) return;
        if (reads.size() > 8 || writes.size() > 8) { err = hipErrorInvalidValue; return; }
        Range rd[8], wr[8];
        int nr = 0, nw = 0;
        for (const Range& r : reads) if (declared++ != withhold) rd[nr++] = r;
        for (const Range& r : writes) if (declared++ != withhold) wr[nw++] = r;
        sc.acquire(s, rd, nr, wr, nw);
        if (sc.multi) set_add_block_cap(bg ? cap_bg : 0);   // kernels on the critical path get the whole machine
        ProfMark pm_;
        prof_begin(prof, sc.st[s], cls, work, &pm_);
        note(launch(sc.st[s]));
        prof_end(prof, sc.st[s], &pm_);
        sc.release(s, rd, nr, wr, nw);
        note(sc.err);
    }

    // Z = X + sign * Y on r x c matrices (stream s: S_PRE when Z is an operand of a product, S_POST when it is part of C)
    void ew(int s, Mat z, Mat x, Mat y, int sign, int64_t live, int64_t r, int64_t c)
    {
        op(s, SW_CLASS_DFS_ADD, bytes(live, r, c, 2, 1), {rng(x, r, c, live), rng(y, r, c, live)}, {rng(z, r, c, live)},
           [&](hipStream_t st) { return launch_ew(z, x, y, sign, live, r, c, st); });
    }

    // the A-side operation (on hm x hk matrices) and the B-side operation (hk x hn) of a DFS step: one launch
    // when the two shapes coincide, else two
    void ew2(int s, Mat z0, Mat x0, Mat y0, int s0, Mat z1, Mat x1, Mat y1, int s1, int64_t live, Dims h)
    {
        if (h.m != h.k || h.k != h.n) {
            ew(s, z0, x0, y0, s0, live, h.m, h.k);
            ew(s, z1, x1, y1, s1, live, h.k, h.n);
            return;
        }
        const int64_t e = h.m;
        op(s, SW_CLASS_DFS_ADD, bytes(live, e, e, 4, 2),
           {rng(x0, e, e, live), rng(y0, e, e, live), rng(x1, e, e, live), rng(y1, e, e, live)},
           {rng(z0, e, e, live), rng(z1, e, e, live)},
           [&](hipStream_t st) { return launch_ew2(z0, x0, y0, s0, z1, x1, y1, s1, live, e, e, st); });
    }

    // C = A * B for `live` independent problems of shape d, steps sched[level..] (Algorithm 2: procedures DFS
    // and BFS).  With h = d / 2: operands T are h.m x h.k, S are h.k x h.n, products Q are h.m x h.n.
    void mul(Mat A, Mat B, Mat C, Dims d, int level, int64_t live)
    {
        if (err != hipSuccess) return;
        if (level == levels) {
            op(S_MM, SW_CLASS_LEAF, 2.0 * live * (double)d.m * (double)d.n * (double)d.k,
               {rng(A, d.m, d.k, live), rng(B, d.k, d.n, live)}, {rng(C, d.m, d.n, live)},
               [&](hipStream_t st) { return launch_gemm(d.m, d.n, d.k, live, A, B, C, false, st); });
            return;
        }
        if (peel_levels && ((d.m | d.n | d.k) & 1)) {
            // Peeling at this level (Section 3.1, "dynamic peeling"): the step runs on the leading even extents, in
            // place; the last row, column and inner index of all `live` problems are finished by thin classical
            // products on the MFMA kernel.  Behind every row of the even part lies the peeled element.
            //   before the step:  c12 = [A11 a12] * [b12; b22],  [c21 c22] = [a21 a22] * B,  copies of a12 and b21
            //   after it:         C11 += a12 * b21  from the copies
            // so that A and B are read for the last time before the step's own kernels: were the strips read from A
            // and B after it, whatever forms the operands of the NEXT problem in the same buffers would have to wait
            // for this problem's products, and the leaf products would stand still meanwhile.
            const Dims e{d.m & ~(int64_t)1, d.n & ~(int64_t)1, d.k & ~(int64_t)1};
            const int64_t rm = d.m - e.m, rn = d.n - e.n, rk = d.k - e.k;
            Mat Ae = A, Be = B, Ce = C;
            Ae.padded = A.padded || rk;
            Be.padded = B.padded || rn;
            Ce.padded = C.padded || rn;
            const bool thin = thin_grid_ok(d.m > d.n ? d.m : d.n, live);   // the streaming one-wide kernels, else the MFMA kernel
            const int64_t mark = used;
            const int64_t sa = (e.m + 31) / 32 * 32, sb = (e.n + 31) / 32 * 32;
            const Mat a12c{rk ? take(live * sa) : nullptr, 1, sa, false}, b21c{rk ? take(live * sb) : nullptr, e.n, sb, false};
            const Mat a12{A.p + e.k, A.ld, A.stride, A.padded}, b21{B.p + e.k * B.ld, B.ld, B.stride, B.padded};
            const Mat bright{B.p + e.n, B.ld, B.stride, B.padded}, c12{C.p + e.n, C.ld, C.stride, C.padded};
            const Mat abot{A.p + e.m * A.ld, A.ld, A.stride, A.padded}, cbot{C.p + e.m * C.ld, C.ld, C.stride, C.padded};
            if (rk && e.m && e.n)
                op(S_POST, SW_CLASS_PEEL, 0.0, {rng(A, d.m, d.k, live), rng(B, d.k, d.n, live)},
                   {rng(a12c, e.m, 1, live), rng(b21c, 1, e.n, live)}, [&](hipStream_t st) {
                       hipError_t e1 = launch_strip_copy(a12, e.m, 1, a12c, live, st);
                       hipError_t e2 = launch_strip_copy(b21, 1, e.n, b21c, live, st);
                       return e1 != hipSuccess ? e1 : e2;
                   });
            if (rn || rm)
                op(S_POST, SW_CLASS_PEEL, 2.0 * live * ((double)e.m * rn * d.k + (double)rm * d.n * d.k),
                   {rng(A, d.m, d.k, live), rng(B, d.k, d.n, live)}, {rng(C, d.m, d.n, live)}, [&](hipStream_t st) {
                       // c12 = [A11 a12] * [b12; b22] and [c21 c22] = [a21 a22] * B
                       hipError_t e2 = !rn ? hipSuccess : (thin ? launch_matvec(e.m, d.k, live, A, bright, c12, st) : launch_gemm(e.m, rn, d.k, live, A, bright, c12, false, st));
                       hipError_t e3 = !rm ? hipSuccess : (thin ? launch_vecmat(d.n, d.k, live, abot, B, cbot, st) : launch_gemm(rm, d.n, d.k, live, abot, B, cbot, false, st));
                       return e2 != hipSuccess ? e2 : e3;
                   });
            mul(Ae, Be, Ce, e, level, live);                             // C11  = A11 * B11
            if (rk && e.m && e.n)
                op(S_POST, SW_CLASS_PEEL, 2.0 * live * (double)e.m * e.n * rk, {rng(a12c, e.m, 1, live), rng(b21c, 1, e.n, live), rng(C, d.m, d.n, live)},
                   {rng(C, d.m, d.n, live)},
                   [&](hipStream_t st) {                                                                  // C11 += a12 * b21
                       return thin ? launch_rank1(e.m, e.n, live, a12c, b21c, Ce, st) : launch_gemm(e.m, e.n, rk, live, a12c, b21c, Ce, true, st);
                   });
            pop_to(mark);
            return;
        }
        const Dims h = d.half();
        const int64_t eT = ws_mat_elems(h.m, h.k), eS = ws_mat_elems(h.k, h.n), eQ = ws_mat_elems(h.m, h.n);
        const int64_t mark = used;
        const bool fused = fuse_here(d, sched + level);
        const Dims q = h.half();
        const int64_t e4T = ws_mat_elems(q.m, q.k), e4S = ws_mat_elems(q.k, q.n), e4Q = ws_mat_elems(q.m, q.n);
        // the step whose children are the leaves: with two sets of buffers, consecutive launches alternate
        if (dbl && sched[level] == 'B' && level + (fused ? 2 : 1) == levels && (flip++ & 1))
            used += (fused ? 49 * live * (e4T + e4S + e4Q) : 7 * live * (eT + eS + eQ)) * (int64_t)sizeof(double);   // skip the first set
        const bool was_bg = bg;
        bg = dbl && sched[level] == 'B' && level + (fused ? 2 : 1) == levels;
        if (bg)
            cap_bg = cap_fixed > 1 ? cap_fixed
                                   : (fused ? leaf_side_cap(65.0 * ((double)q.m * q.k + (double)q.k * q.n + (double)q.m * q.n), live, 49, q)
                                            : leaf_side_cap(11.0 * ((double)h.m * h.k + (double)h.k * h.n + (double)h.m * h.n), live, 7, h));
        if (fused) {
            // two BFS steps in one pass: the 49 grandchildren's operands come straight from the parents and
            // their products go straight back; the level in between exists in registers only
            Mat T = ws_mat(take(49 * live * e4T), q.m, q.k), S = ws_mat(take(49 * live * e4S), q.k, q.n),
                Q = ws_mat(take(49 * live * e4Q), q.m, q.n);
            op(S_PRE, SW_CLASS_PRE_ADD, bytes(live, q.m, q.k, 16, 49), {rng(A, d.m, d.k, live)}, {rng(T, q.m, q.k, 49 * live)},
               [&](hipStream_t st) { return launch_pre_add2(0, A, live, q.m, q.k, T, st); });
            op(S_PRE, SW_CLASS_PRE_ADD, bytes(live, q.k, q.n, 16, 49), {rng(B, d.k, d.n, live)}, {rng(S, q.k, q.n, 49 * live)},
               [&](hipStream_t st) { return launch_pre_add2(1, B, live, q.k, q.n, S, st); });
            mul(T, S, Q, q, level + 2, 49 * live);
            op(S_POST, SW_CLASS_POST_ADD, bytes(live, q.m, q.n, 49, 16), {rng(Q, q.m, q.n, 49 * live)}, {rng(C, d.m, d.n, live)},
               [&](hipStream_t st) { return launch_post_add2(Q, live, q.m, q.n, C, st); });
        } else if (sched[level] == 'B') {
            // BFS step: all seven (T, S, Q) triples of every parent exist at once (Section 3.3.1)
            Mat T = ws_mat(take(7 * live * eT), h.m, h.k), S = ws_mat(take(7 * live * eS), h.k, h.n),
                Q = ws_mat(take(7 * live * eQ), h.m, h.n);
            op(S_PRE, SW_CLASS_PRE_ADD, bytes(live, h.m, h.k, 4, 7), {rng(A, d.m, d.k, live)}, {rng(T, h.m, h.k, 7 * live)},
               [&](hipStream_t st) { return launch_pre_add(0, A, live, h.m, h.k, T, true, st); });
            op(S_PRE, SW_CLASS_PRE_ADD, bytes(live, h.k, h.n, 4, 7), {rng(B, d.k, d.n, live)}, {rng(S, h.k, h.n, 7 * live)},
               [&](hipStream_t st) { return launch_pre_add(1, B, live, h.k, h.n, S, true, st); });
            mul(T, S, Q, h, level + 1, 7 * live);
            op(S_POST, SW_CLASS_POST_ADD, bytes(live, h.m, h.n, 7, 4), {rng(Q, h.m, h.n, 7 * live)}, {rng(C, d.m, d.n, live)},
               [&](hipStream_t st) { return launch_post_add(Q, live, h.m, h.n, C, st); });
        } else if (rich & (1u << level)) {
            // DFS step with the storage of a BFS step: the four non-trivial T, four S and seven Q of every
            // parent are kept, so the additions are the one-pass BFS kernels (27 instead of 38 half-size
            // matrices moved per parent), but the seven subproblems are still solved in sequence.
            Mat Tn = ws_mat(take(4 * live * eT), h.m, h.k), Sn = ws_mat(take(4 * live * eS), h.k, h.n),
                Q = ws_mat(take(7 * live * eQ), h.m, h.n);
            op(S_PRE, SW_CLASS_PRE_ADD, bytes(live, h.m, h.k, 4, 4), {rng(A, d.m, d.k, live)}, {rng(Tn, h.m, h.k, 4 * live)},
               [&](hipStream_t st) { return launch_pre_add(0, A, live, h.m, h.k, Tn, false, st); });
            op(S_PRE, SW_CLASS_PRE_ADD, bytes(live, h.k, h.n, 4, 4), {rng(B, d.k, d.n, live)}, {rng(Sn, h.k, h.n, 4 * live)},
               [&](hipStream_t st) { return launch_pre_add(1, B, live, h.k, h.n, Sn, false, st); });
            auto slot = [&](const Mat& base, int k, int per, int64_t e) { return Mat{base.p + k * e, base.ld, per * e, base.padded}; };
            const Mat Ta[7] = {quad(A, h.m, h.k, 0, 0), quad(A, h.m, h.k, 0, 1), slot(Tn, 0, 4, eT), slot(Tn, 1, 4, eT),
                               slot(Tn, 2, 4, eT), slot(Tn, 3, 4, eT), quad(A, h.m, h.k, 1, 1)};
            const Mat Sb[7] = {quad(B, h.k, h.n, 0, 0), quad(B, h.k, h.n, 1, 0), slot(Sn, 0, 4, eS), slot(Sn, 1, 4, eS),
                               slot(Sn, 2, 4, eS), quad(B, h.k, h.n, 1, 1), slot(Sn, 3, 4, eS)};
            for (int j = 0; j < 7; ++j) mul(Ta[j], Sb[j], slot(Q, j, 7, eQ), h, level + 1, live);
            op(S_POST, SW_CLASS_POST_ADD, bytes(live, h.m, h.n, 7, 4), {rng(Q, h.m, h.n, 7 * live)}, {rng(C, d.m, d.n, live)},
               [&](hipStream_t st) { return launch_post_add(Q, live, h.m, h.n, C, st); });
        } else {
            // DFS step: the seven products one after the other (Section 3.4), written straight into the
            // quadrants of C, with two temporaries per parent: X holds the T operands and later the product Q0
            // (two views of one buffer large enough for either), Y holds the S operands.  The additions are
            // those of Appendix A in the printed association, so the result is bit-identical to the BFS form.
            const int64_t eX = eT > eQ ? eT : eQ;
            double* const xp = take(live * eX);
            const Mat X{xp, ws_ld(h.k), eX, ws_ld(h.k) > h.k};      // as a T operand, h.m x h.k
            const Mat XQ{xp, ws_ld(h.n), eX, ws_ld(h.n) > h.n};     // as the product Q0, h.m x h.n
            const Mat Y = ws_mat(take(live * eS), h.k, h.n);
            const Mat A11 = quad(A, h.m, h.k, 0, 0), A12 = quad(A, h.m, h.k, 0, 1), A21 = quad(A, h.m, h.k, 1, 0), A22 = quad(A, h.m, h.k, 1, 1);
            const Mat B11 = quad(B, h.k, h.n, 0, 0), B12 = quad(B, h.k, h.n, 0, 1), B21 = quad(B, h.k, h.n, 1, 0), B22 = quad(B, h.k, h.n, 1, 1);
            const Mat C11 = quad(C, h.m, h.n, 0, 0), C12 = quad(C, h.m, h.n, 0, 1), C21 = quad(C, h.m, h.n, 1, 0), C22 = quad(C, h.m, h.n, 1, 1);
            ew2(S_PRE, X, A11, A21, -1, Y, B22, B12, -1, live, h);     // T4 = A11 - A21, S4 = B22 - B12
            mul(X, Y, C21, h, level + 1, live);                        // C21 <- Q4
            ew2(S_PRE, X, A21, A22, +1, Y, B12, B11, -1, live, h);     // T2 = A21 + A22, S2 = B12 - B11
            mul(X, Y, C22, h, level + 1, live);                        // C22 <- Q2
            ew2(S_PRE, X, X, A11, -1, Y, B22, Y, -1, live, h);         // T3 = T2 - A11,  S3 = B22 - S2
            mul(X, Y, C12, h, level + 1, live);                        // C12 <- Q3
            ew(S_PRE, X, A12, X, -1, live, h.m, h.k);                  // T5 = A12 - T3
            mul(X, B22, C11, h, level + 1, live);                      // C11 <- Q5 = T5 * B22
            mul(A11, B11, XQ, h, level + 1, live);                     // X   <- Q0 = A11 * B11
            op(S_POST, SW_CLASS_DFS_ADD, bytes(live, h.m, h.n, 5, 3),
               {rng(XQ, h.m, h.n, live), rng(C11, h.m, h.n, live), rng(C12, h.m, h.n, live), rng(C21, h.m, h.n, live),
                rng(C22, h.m, h.n, live)},
               {rng(C12, h.m, h.n, live), rng(C21, h.m, h.n, live), rng(C22, h.m, h.n, live)},
               [&](hipStream_t st) { return launch_dfs_post(XQ, C11, C12, C21, C22, live, h.m, h.n, st); });  // C12, C22 final; C21 = U2
            ew(S_PRE, Y, Y, B21, -1, live, h.k, h.n);                  // S6 = S3 - B21
            mul(A22, Y, C11, h, level + 1, live);                      // C11 <- Q6 = A22 * S6
            ew(S_POST, C21, C21, C11, -1, live, h.m, h.n);             // C21 = U2 - Q6
            mul(A12, B21, C11, h, level + 1, live);                    // C11 <- Q1 = A12 * B21
            ew(S_POST, C11, XQ, C11, +1, live, h.m, h.n);              // C11 = Q0 + Q1
        }
        bg = was_bg;
        pop_to(mark);
    }
};

bool overlaps(const double* p, int64_t pn, const double* q, int64_t qn)
{
    const uintptr_t a0 = (uintptr_t)p, a1 = a0 + (uintptr_t)pn * sizeof(double);
    const uintptr_t b0 = (uintptr_t)q, b1 = b0 + (uintptr_t)qn * sizeof(double);
    return a0 < b1 && b0 < a1;
}

int gemm_rect_impl(Dims d, const double* A, int64_t lda, const double* B, int64_t ldb, double* C, int64_t ldc,
                   int levels, const char* schedule, void* ws, int64_t ws_bytes, hipStream_t stream)
{
    return gemm_rect_impl(d, A, lda, B, ldb, C, ldc, levels, schedule, ws, ws_bytes, stream, current_opts());
}

int gemm_rect_impl(Dims d, const double* A, int64_t lda, const double* B, int64_t ldb, double* C, int64_t ldc,
                   int levels, const char* schedule, void* ws, int64_t ws_bytes, hipStream_t stream, const CallOpts& opts)
{
    const int64_t dmin = d.m < d.n ? (d.m < d.k ? d.m : d.k) : (d.n < d.k ? d.n : d.k);
    const int64_t dmax = d.m > d.n ? (d.m > d.k ? d.m : d.k) : (d.n > d.k ? d.n : d.k);
    if (levels < 0) {
        // depth left open: the cost model's choice for this workspace, step order by the planner
        if (dmin < 0 || dmax > 200000) { set_error("bad shape: %lld x %lld x %lld", (long long)d.m, (long long)d.n, (long long)d.k); return SW_EINVAL; }
        levels = plan_levels(dmin, (ws || opts.check_only) ? ws_bytes : 0);
        schedule = nullptr;
    }
    int rc = check_shape(dmin, levels);
    if (rc == SW_OK) rc = check_shape(dmax, 0);
    if (rc != SW_OK) return rc;
    if (d.m == 0 || d.n == 0) return SW_OK;
    if (d.k == 0) { set_error("empty inner dimension"); return SW_EINVAL; }
    if (!A || !B || !C) { set_error("NULL matrix pointer"); return SW_EINVAL; }
    if (lda < d.k || ldb < d.n || ldc < d.n) { set_error("leading dimension smaller than the row length"); return SW_EINVAL; }
    if (!gemm_pitches_ok(lda, ldb)) {
        set_error("leading dimension too large for the product kernel's 32-bit offsets (lda <= 4227329, ldb <= 35791385)");
        return SW_EINVAL;
    }
    const int64_t spanA = (d.m - 1) * lda + d.k, spanB = (d.k - 1) * ldb + d.n, spanC = (d.m - 1) * ldc + d.n;
    if (overlaps(C, spanC, A, spanA) || overlaps(C, spanC, B, spanB)) {
        set_error("C overlaps A or B");
        return SW_EINVAL;
    }
    char chosen[SW_MAX_LEVELS + 1];
    if (!schedule || !*schedule) {
        rc = plan(d, levels, (ws || opts.check_only) ? ws_bytes : 0, chosen, opts.odd_mode, opts.overlap != 0);
        if (rc != SW_OK) return rc;
        schedule = chosen;
    } else if (!schedule_ok(schedule, levels)) {
        set_error("schedule \"%s\" must be %d characters of B or D", schedule, levels);
        return SW_EINVAL;
    }
    const int64_t need = total_need(d, levels, schedule, opts.odd_mode);
    if (need > 0 && opts.check_only) {
        if (ws_bytes < need) {
            set_error("workspace of %lld bytes is too small: %lld x %lld x %lld, schedule %s needs %lld", (long long)ws_bytes,
                      (long long)d.m, (long long)d.n, (long long)d.k, schedule, (long long)need);
            return SW_ENOMEM;
        }
    } else if (need > 0) {
        if (!ws || ws_bytes < need) {
            set_error("workspace of %lld bytes is too small: %lld x %lld x %lld, schedule %s needs %lld", (long long)(ws ? ws_bytes : 0),
                      (long long)d.m, (long long)d.n, (long long)d.k, schedule, (long long)need);
            return SW_ENOMEM;
        }
        if ((uintptr_t)ws & 255u) { set_error("workspace must be 256-byte aligned"); return SW_EINVAL; }
        if (overlaps((const double*)ws, need / 8, A, spanA) || overlaps((const double*)ws, need / 8, B, spanB) ||
            overlaps((const double*)ws, need / 8, C, spanC)) {
            set_error("workspace overlaps A, B or C");
            return SW_EINVAL;
        }
    }
    if (opts.check_only) return SW_OK;

    Exec ex;
    ex.ws = (char*)ws;
    ex.ws_bytes = ws_bytes;
    ex.sched = schedule;
    ex.levels = levels;
    const Dims lead = floor_dims(d, levels);
    const bool peel = opts.odd_mode == SW_ODD_PEEL && (lead.m != d.m || lead.n != d.n || lead.k != d.k);
    const bool peel_levels = opts.odd_mode == SW_ODD_PEEL_LEVELS;
    const Dims rec = peel ? lead : (peel_levels ? d : padded_dims(d, levels));
    ex.peel_levels = peel_levels;
    {
        // spend what the workspace has beyond the minimum: first on a second set of the buffers next to the
        // leaves (so that additions and leaf products of consecutive launches overlap), then on the rich form
        // of the deepest DFS steps
        const int64_t fixed = need - ws_need_bytes(rec, schedule, 1);
        choose_options(rec, levels, schedule, ws_bytes - fixed, opts.overlap != 0, &ex.rich, &ex.dbl);
    }
    ex.prof = (opts.profile && !tracer()) ? profiler() : nullptr;
    ex.withhold = t_withhold;
    // with BFS steps only the kernels form one chain: nothing could overlap, so one stream it is
    ex.sc.start(stream, opts.overlap != 0 && levels > 0 && strchr(schedule, 'D') != nullptr);
    set_add_block_cap(0);
    ex.cap_fixed = opts.overlap;

    Mat a{const_cast<double*>(A), lda, 0}, b{const_cast<double*>(B), ldb, 0}, c{C, ldc, 0};
    if (peel) {
        // Peeling (Section 3.1 names it beside padding): the leading blocks, whose extents are the previous
        // multiples of 2^levels, go through the recursion in place; the fewer than 2^levels peeled rows, columns
        // and inner indices are finished by up to three thin classical products on the same MFMA kernel.
        const int64_t rm = d.m - rec.m, rn = d.n - rec.n, rk = d.k - rec.k;
        ex.mul(a, b, c, rec, 0, 1);                                  // C11  = A11 * B11
        const Mat a12{a.p + rec.k, lda, 0}, b21{b.p + rec.k * ldb, ldb, 0};
        const Mat bright{b.p + rec.n, ldb, 0}, c12{c.p + rec.n, ldc, 0};
        const Mat abot{a.p + rec.m * lda, lda, 0}, cbot{c.p + rec.m * ldc, ldc, 0};
        ex.op(S_POST, SW_CLASS_PEEL,
              2.0 * ((double)rec.m * rec.n * rk + (double)rec.m * rn * d.k + (double)rm * d.n * d.k),
              {rng(a, d.m, d.k), rng(b, d.k, d.n)}, {rng(c, d.m, d.n)}, [&](hipStream_t st) {
                  hipError_t e1 = rk ? launch_gemm(rec.m, rec.n, rk, 1, a12, b21, c, true, st) : hipSuccess;      // C11 += A12 * B21
                  hipError_t e2 = rn ? launch_gemm(rec.m, rn, d.k, 1, a, bright, c12, false, st) : hipSuccess;    // C12  = [A11 A12] * [B12; B22]
                  hipError_t e3 = rm ? launch_gemm(rm, d.n, d.k, 1, abot, b, cbot, false, st) : hipSuccess;       // [C21 C22] = [A21 A22] * B
                  return e1 != hipSuccess ? e1 : (e2 != hipSuccess ? e2 : e3);
              });
    } else {
        const Dims p = rec;
        const bool padded = p.m != d.m || p.n != d.n || p.k != d.k;
        if (padded) {
            // zero-pad into workspace copies of the next multiples of 2^levels (Section 3.1)
            a = ws_mat(ex.take(ws_mat_elems(p.m, p.k)), p.m, p.k);
            b = ws_mat(ex.take(ws_mat_elems(p.k, p.n)), p.k, p.n);
            c = ws_mat(ex.take(ws_mat_elems(p.m, p.n)), p.m, p.n);
            a.stride = b.stride = c.stride = 0;
            const Mat ua{const_cast<double*>(A), lda, 0}, ub{const_cast<double*>(B), ldb, 0};
            ex.op(S_PRE, SW_CLASS_PAD, 8.0 * ((double)d.m * d.k + (double)d.k * d.n + (double)p.m * p.k + (double)p.k * p.n),
                  {rng(ua, d.m, d.k), rng(ub, d.k, d.n)}, {rng(a, p.m, p.k), rng(b, p.k, p.n)}, [&](hipStream_t st) {
                      hipError_t e1 = launch_pad_copy(A, lda, d.m, d.k, a.p, a.ld, p.m, p.k, st);
                      hipError_t e2 = launch_pad_copy(B, ldb, d.k, d.n, b.p, b.ld, p.k, p.n, st);
                      return e1 != hipSuccess ? e1 : e2;
                  });
        }
        ex.mul(a, b, c, p, 0, 1);
        if (padded) {
            const Mat uc{C, ldc, 0};
            ex.op(S_POST, SW_CLASS_PAD, 8.0 * 2.0 * (double)d.m * d.n, {rng(c, p.m, p.n)}, {rng(uc, d.m, d.n)},
                  [&](hipStream_t st) { return launch_pad_copy(c.p, c.ld, p.m, p.n, C, ldc, d.m, d.n, st); });
        }
    }
    ex.sc.finish();
    set_add_block_cap(0);
    ex.note(ex.sc.err);
    if (ex.err != hipSuccess) return hip_fail(ex.err, "kernel launch");
    return SW_OK;
}

int gemm_impl(int64_t n, const double* A, int64_t lda, const double* B, int64_t ldb, double* C, int64_t ldc,
              int levels, const char* schedule, void* ws, int64_t ws_bytes, hipStream_t stream)
{
    return gemm_rect_impl(Dims{n, n, n}, A, lda, B, ldb, C, ldc, levels, schedule, ws, ws_bytes, stream);
}

}  // namespace sw

using namespace sw;

// ================================================ C ABI ==========================================================

extern "C" {

int sw_gemm(int64_t n, const double* A, const double* B, double* C, int levels, const char* schedule)
{
    return gemm_impl(n, A, n, B, n, C, n, levels, schedule, g_ws, g_ws_bytes, g_stream);
}

int sw_gemm_ex(int64_t n, const double* A, int64_t lda, const double* B, int64_t ldb, double* C, int64_t ldc,
               int levels, const char* schedule, void* workspace, int64_t workspace_bytes, void* hip_stream)
{
    if (workspace_bytes < 0) { set_error("negative workspace size"); return SW_EINVAL; }
    return gemm_impl(n, A, lda, B, ldb, C, ldc, levels, schedule, workspace, workspace_bytes, (hipStream_t)hip_stream);
}

int sw_gemm_rect(int64_t M, int64_t N, int64_t K, const double* A, int64_t lda, const double* B, int64_t ldb, double* C,
                 int64_t ldc, int levels, const char* schedule, void* workspace, int64_t workspace_bytes, void* hip_stream)
{
    if (workspace_bytes < 0) { set_error("negative workspace size"); return SW_EINVAL; }
    if (M < 0 || N < 0 || K < 0) { set_error("negative dimension"); return SW_EINVAL; }
    return gemm_rect_impl(Dims{M, N, K}, A, lda, B, ldb, C, ldc, levels, schedule, workspace, workspace_bytes, (hipStream_t)hip_stream);
}

int64_t sw_trace_gemm(int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb, int64_t ldc, int levels, const char* schedule,
                      int64_t workspace_bytes, int overlap, int odd_mode, int64_t withhold, int64_t* log, int64_t log_words)
{
    if (workspace_bytes < 0 || M < 0 || N < 0 || K < 0 || log_words < 0 || overlap < 0) { set_error("negative argument"); return SW_EINVAL; }
    if (odd_mode != SW_ODD_PAD && odd_mode != SW_ODD_PEEL && odd_mode != SW_ODD_PEEL_LEVELS) { set_error("unknown mode %d", odd_mode); return SW_EINVAL; }
    // synthetic operand addresses, 2^40 bytes apart (no matrix the library accepts is that large)
    const uintptr_t T = (uintptr_t)1 << 40;
    Tracer t;
    t.out = log;
    t.cap = log ? log_words : 0;
    set_tracer(&t);
    t_withhold = withhold;
    const int rc = gemm_rect_impl(Dims{M, N, K}, (const double*)(1 * T), lda, (const double*)(2 * T), ldb, (double*)(3 * T), ldc, levels,
                                  schedule, (void*)(4 * T), workspace_bytes, nullptr, CallOpts{overlap, odd_mode, false, false});
    set_tracer(nullptr);
    t_withhold = -1;
    return rc != SW_OK ? rc : t.words;
}

int64_t sw_plan_memory_rect(int64_t M, int64_t N, int64_t K, int levels, const char* schedule)
{
    if (M < 0 || N < 0 || K < 0) { set_error("negative dimension"); return SW_EINVAL; }
    const int64_t dmin = M < N ? (M < K ? M : K) : (N < K ? N : K), dmax = M > N ? (M > K ? M : K) : (N > K ? N : K);
    int rc = check_shape(dmin, levels);
    if (rc == SW_OK) rc = check_shape(dmax, 0);
    if (rc != SW_OK) return rc;
    std::string s = (schedule && *schedule) ? std::string(schedule) : std::string((size_t)levels, 'D');
    if (!schedule_ok(s.c_str(), levels)) {
        set_error("schedule \"%s\" must be %d characters of B or D", s.c_str(), levels);
        return SW_EINVAL;
    }
    return total_need(Dims{M, N, K}, levels, s.c_str());
}

// ---- diagonal scaling around the product (Section 6.1) ------------------------------------------------------

static int64_t scaled_extra_bytes(int64_t n)
{
    // scaled copies of A and B, and seven vectors (row/column maxima and D1, D2, 1/D2, D3)
    return 2 * ws_mat_elems(n) * (int64_t)sizeof(double) + 7 * ((n + 31) / 32 * 32) * (int64_t)sizeof(double);
}

int64_t sw_plan_memory_scaled(int64_t n, int levels, const char* schedule)
{
    const int64_t base = sw_plan_memory(n, levels, schedule);
    return base < 0 ? base : base + scaled_extra_bytes(n);
}

int sw_gemm_scaled(int64_t n, const double* A, const double* B, double* C, int levels, const char* schedule,
                   int scaling)
{
    if (scaling < 0 || scaling > (SW_SCALE_OUTSIDE | SW_SCALE_INSIDE)) { set_error("unknown scaling %d", scaling); return SW_EINVAL; }
    if (scaling == 0) return sw_gemm(n, A, B, C, levels, schedule);
    int rc = check_shape(n, levels);
    if (rc != SW_OK) return rc;
    if (n == 0) return SW_OK;
    if (!A || !B || !C) { set_error("NULL matrix pointer"); return SW_EINVAL; }
    if (overlaps(C, n * n, A, n * n) || overlaps(C, n * n, B, n * n)) { set_error("C overlaps A or B"); return SW_EINVAL; }
    const int64_t extra = scaled_extra_bytes(n);
    if (!g_ws || g_ws_bytes < extra) {
        set_error("workspace of %lld bytes is too small for the scaled copies (%lld)", (long long)g_ws_bytes, (long long)extra);
        return SW_ENOMEM;
    }
    if (overlaps((const double*)g_ws, extra / 8, A, n * n) || overlaps((const double*)g_ws, extra / 8, B, n * n) ||
        overlaps((const double*)g_ws, extra / 8, C, n * n)) {
        set_error("workspace overlaps A, B or C");
        return SW_EINVAL;
    }
    hipStream_t st = g_stream;
    char* w = (char*)g_ws;
    const int64_t ld = ws_ld(n), e = ws_mat_elems(n), nv = (n + 31) / 32 * 32;
    double* As = (double*)w;
    double* Bs = As + e;
    double* vec = Bs + e;
    double *ma = vec, *mb = vec + nv, *d1 = vec + 2 * nv, *d3 = vec + 3 * nv, *d2 = vec + 4 * nv, *d2i = vec + 5 * nv,
           *tmp = vec + 6 * nv;
    hipError_t err = hipSuccess;
    auto note = [&](hipError_t x) { if (err == hipSuccess && x != hipSuccess) err = x; };
    const bool outside = scaling & SW_SCALE_OUTSIDE, inside = scaling & SW_SCALE_INSIDE;
    Profiler* prof = profiler();
    ProfMark pm_;
    prof_begin(prof, st, SW_CLASS_SCALE, 8.0 * n * n * (outside ? 2.0 : 0.0) + 8.0 * n * n * (inside ? 2.0 : 0.0) + 8.0 * n * n * 4.0, &pm_);
    if (outside) {
        note(launch_absmax_rows(A, n, n, nullptr, ma, st));            // max_j |A_ij|
        note(launch_outside_scale(ma, n, d1, st));
        note(launch_absmax_cols(B, n, n, nullptr, mb, st));            // max_i |B_ij|
        note(launch_outside_scale(mb, n, d3, st));
    }
    if (inside) {
        note(launch_absmax_cols(A, n, n, outside ? d1 : nullptr, ma, st));   // max_i D1_ii |A_ik|
        note(launch_absmax_rows(B, n, n, outside ? d3 : nullptr, tmp, st));  // max_j |B_kj| D3_jj
        note(launch_inside_scale(ma, tmp, n, d2, d2i, st));
    }
    note(launch_scale_copy(A, n, n, outside ? d1 : nullptr, inside ? d2 : nullptr, As, ld, st));    // D1 A D2
    note(launch_scale_copy(B, n, n, inside ? d2i : nullptr, outside ? d3 : nullptr, Bs, ld, st));   // D2^-1 B D3
    prof_end(prof, st, &pm_);
    if (err != hipSuccess) return hip_fail(err, "scaling kernels");
    rc = gemm_impl(n, As, ld, Bs, ld, C, n, levels, schedule, w + extra, g_ws_bytes - extra, st);
    if (rc != SW_OK) return rc;
    if (outside) {
        // C = D1^-1 C' D3^-1: the reciprocals of powers of two are formed exactly
        ProfMark pm_;
        prof_begin(prof, st, SW_CLASS_SCALE, 8.0 * n * n * 2.0, &pm_);
        note(launch_outside_scale(d1, n, ma, st));     // 2^-e(2^-k) = 2^k: reuses the exponent kernel to invert
        note(launch_outside_scale(d3, n, mb, st));
        note(launch_scale_copy(C, n, n, ma, mb, C, n, st));
        prof_end(prof, st, &pm_);
        if (err != hipSuccess) return hip_fail(err, "unscaling kernels");
    }
    return SW_OK;
}

int64_t sw_plan_memory(int64_t n, int levels, const char* schedule)
{
    int rc = check_shape(n, levels);
    if (rc != SW_OK) return rc;
    std::string s = (schedule && *schedule) ? std::string(schedule) : std::string((size_t)levels, 'D');
    if (!schedule_ok(s.c_str(), levels)) {
        set_error("schedule \"%s\" must be %d characters of B or D", s.c_str(), levels);
        return SW_EINVAL;
    }
    return total_need(n, levels, s.c_str());
}

int64_t sw_plan_workspace(int64_t n, int levels, const char* schedule, int64_t budget_bytes)
{
    int rc = check_shape(n, levels);
    if (rc != SW_OK) return rc;
    if (!schedule || !schedule_ok(schedule, levels)) { set_error("bad schedule"); return SW_EINVAL; }
    const int64_t need = total_need(n, levels, schedule);
    if (need > budget_bytes) {
        set_error("schedule %s needs %lld bytes, budget is %lld", schedule, (long long)need, (long long)budget_bytes);
        return SW_ENOMEM;
    }
    if (n == 0) return 0;
    const int64_t q = (int64_t)1 << levels;
    const int mode = g_odd_mode.load();
    const int64_t nrec = mode == SW_ODD_PEEL_LEVELS ? n : ((n % q && mode == SW_ODD_PEEL) ? n - n % q : padded_n(n, levels));
    const int64_t fixed = need - ws_need_bytes(nrec, schedule, 1);
    uint32_t rich = 0;
    bool dbl = false;
    choose_options(nrec, levels, schedule, budget_bytes - fixed, g_overlap != 0, &rich, &dbl);
    return fixed + ws_need_bytes(nrec, schedule, 1, rich, dbl);
}

int sw_plan_schedule(int64_t n, int levels, int64_t budget_bytes, char* out)
{
    int rc = check_shape(n, levels);
    if (rc != SW_OK) return rc;
    if (!out) { set_error("NULL output buffer"); return SW_EINVAL; }
    if (budget_bytes < 0) { set_error("negative budget"); return SW_EINVAL; }
    return plan(n, levels, budget_bytes, out);
}

int64_t sw_model_words(int64_t n, int levels, const char* schedule)
{
    int rc = check_shape(n, levels);
    if (rc != SW_OK) return rc;
    if (!schedule || !schedule_ok(schedule, levels)) { set_error("bad schedule"); return SW_EINVAL; }
    if (n % ((int64_t)1 << levels)) { set_error("n is not a multiple of 2^levels"); return SW_EINVAL; }
    int64_t words = 3 * n * n, live = 1, size = n;
    for (int i = 0; i < levels; ++i) {
        if (schedule[i] == 'B') live *= 7;
        size /= 2;
        words += 3 * live * size * size;
    }
    return words;
}

int sw_lm_dfs_steps(double n, double P, double M_words)
{
    if (!(n > 0) || !(P >= 1) || !(M_words > 0)) { set_error("bad argument"); return SW_EINVAL; }
    const double w0 = log2(7.0);
    const double l = ceil(log2(4.0 * n / (pow(P, 1.0 / w0) * sqrt(M_words))));
    return l > 0 ? (int)l : 0;
}

double sw_flop_count(int64_t n, int levels)
{
    if (check_shape(n, levels) != SW_OK || n % ((int64_t)1 << levels)) return -1.0;
    const double m = (double)(n >> levels);
    double leaves = 1.0, adds = 0.0, size = (double)n;
    for (int i = 0; i < levels; ++i) {
        adds += 15.0 * leaves * (size / 2) * (size / 2);
        leaves *= 7.0;
        size /= 2;
    }
    return leaves * (2.0 * m * m * m - m * m) + adds;
}

int sw_set_workspace(void* dev_ptr, int64_t bytes)
{
    if (bytes < 0 || (!dev_ptr && bytes != 0)) { set_error("bad workspace"); return SW_EINVAL; }
    if ((uintptr_t)dev_ptr & 255u) { set_error("workspace must be 256-byte aligned"); return SW_EINVAL; }
    g_ws = dev_ptr;
    g_ws_bytes = bytes;
    return SW_OK;
}

int sw_set_overlap(int on)
{
    if (on < 0) { set_error("negative argument"); return SW_EINVAL; }
    g_overlap = on;
    return SW_OK;
}

int sw_set_odd_mode(int mode)
{
    if (mode != SW_ODD_PAD && mode != SW_ODD_PEEL && mode != SW_ODD_PEEL_LEVELS) { set_error("unknown mode %d", mode); return SW_EINVAL; }
    g_odd_mode = mode;
    return SW_OK;
}

int sw_set_stream(void* hip_stream)
{
    g_stream = (hipStream_t)hip_stream;
    return SW_OK;
}

const char* sw_last_error(void) { return g_err; }

// ---- single steps -------------------------------------------------------------------------------------------------

static bool bad_dims(int64_t live, int64_t h) { return live < 0 || h < 0 || h > 131070 || live > 65535; }

int sw_pre_add(int side, const double* parent, int64_t parent_ld, int64_t parent_stride, int64_t live,
               int64_t h, double* child, int64_t child_ld, int64_t child_stride, void* hip_stream)
{
    if ((side != 0 && side != 1) || bad_dims(live, h) || !parent || !child || parent_ld < 2 * h || child_ld < h) {
        set_error("sw_pre_add: bad argument");
        return SW_EINVAL;
    }
    hipError_t e = launch_pre_add(side, Mat{const_cast<double*>(parent), parent_ld, parent_stride}, live, h,
                                  Mat{child, child_ld, child_stride}, true, (hipStream_t)hip_stream);
    return e == hipSuccess ? SW_OK : hip_fail(e, "sw_pre_add");
}

int sw_post_add(const double* Q, int64_t q_ld, int64_t q_stride, int64_t live, int64_t h, double* parent,
                int64_t parent_ld, int64_t parent_stride, void* hip_stream)
{
    if (bad_dims(live, h) || !Q || !parent || parent_ld < 2 * h || q_ld < h) {
        set_error("sw_post_add: bad argument");
        return SW_EINVAL;
    }
    hipError_t e = launch_post_add(Mat{const_cast<double*>(Q), q_ld, q_stride}, live, h,
                                   Mat{parent, parent_ld, parent_stride}, (hipStream_t)hip_stream);
    return e == hipSuccess ? SW_OK : hip_fail(e, "sw_post_add");
}

int sw_pre_add2(int side, const double* parent, int64_t parent_ld, int64_t parent_stride, int64_t live,
                int64_t m, double* child, int64_t child_ld, int64_t child_stride, void* hip_stream)
{
    if ((side != 0 && side != 1) || bad_dims(live, m) || m > 65535 || !parent || !child || parent_ld < 4 * m || child_ld < m) {
        set_error("sw_pre_add2: bad argument");
        return SW_EINVAL;
    }
    hipError_t e = launch_pre_add2(side, Mat{const_cast<double*>(parent), parent_ld, parent_stride}, live, m,
                                   Mat{child, child_ld, child_stride}, (hipStream_t)hip_stream);
    return e == hipSuccess ? SW_OK : hip_fail(e, "sw_pre_add2");
}

int sw_post_add2(const double* Q, int64_t q_ld, int64_t q_stride, int64_t live, int64_t m, double* parent,
                 int64_t parent_ld, int64_t parent_stride, void* hip_stream)
{
    if (bad_dims(live, m) || m > 65535 || !Q || !parent || parent_ld < 4 * m || q_ld < m) {
        set_error("sw_post_add2: bad argument");
        return SW_EINVAL;
    }
    hipError_t e = launch_post_add2(Mat{const_cast<double*>(Q), q_ld, q_stride}, live, m,
                                    Mat{parent, parent_ld, parent_stride}, (hipStream_t)hip_stream);
    return e == hipSuccess ? SW_OK : hip_fail(e, "sw_post_add2");
}

int sw_leaf_gemm(int64_t m, int64_t batch, const double* A, int64_t lda, int64_t stride_a, const double* B,
                 int64_t ldb, int64_t stride_b, double* C, int64_t ldc, int64_t stride_c, void* hip_stream)
{
    if (m < 0 || batch < 0 || m > 200000 || !A || !B || !C || lda < m || ldb < m || ldc < m) {
        set_error("sw_leaf_gemm: bad argument");
        return SW_EINVAL;
    }
    if (!gemm_pitches_ok(lda, ldb)) {
        set_error("sw_leaf_gemm: leading dimension too large for the kernel's 32-bit offsets (lda <= 4227329, ldb <= 35791385)");
        return SW_EINVAL;
    }
    hipError_t e = launch_leaf_gemm(m, batch, Mat{const_cast<double*>(A), lda, stride_a},
                                    Mat{const_cast<double*>(B), ldb, stride_b}, Mat{C, ldc, stride_c},
                                    (hipStream_t)hip_stream);
    return e == hipSuccess ? SW_OK : hip_fail(e, "sw_leaf_gemm");
}

int sw_gemm_classical(int64_t M, int64_t N, int64_t K, const double* A, int64_t lda, const double* B, int64_t ldb,
                      double* C, int64_t ldc, int accumulate, void* hip_stream)
{
    if (M < 0 || N < 0 || K < 0 || M > 200000 || N > 200000 || K > 200000 || lda < K || ldb < N || ldc < N ||
        ((M > 0 && N > 0) && (!C || (K > 0 && (!A || !B))))) {
        set_error("sw_gemm_classical: bad argument");
        return SW_EINVAL;
    }
    if (!gemm_pitches_ok(lda, ldb)) {
        set_error("sw_gemm_classical: leading dimension too large for the kernel's 32-bit offsets (lda <= 4227329, ldb <= 35791385)");
        return SW_EINVAL;
    }
    if (M == 0 || N == 0) return SW_OK;
    if (K == 0) {
        if (accumulate) return SW_OK;
        hipError_t e = launch_pad_copy(C, ldc, 0, 0, C, ldc, M, N, (hipStream_t)hip_stream);   // an empty sum: zeros
        return e == hipSuccess ? SW_OK : hip_fail(e, "sw_gemm_classical");
    }
    hipError_t e = launch_gemm(M, N, K, 1, Mat{const_cast<double*>(A), lda, 0}, Mat{const_cast<double*>(B), ldb, 0},
                               Mat{C, ldc, 0}, accumulate != 0, (hipStream_t)hip_stream);
    return e == hipSuccess ? SW_OK : hip_fail(e, "sw_gemm_classical");
}

int sw_pad_copy(const double* src, int64_t src_ld, int64_t rows, int64_t cols, double* dst, int64_t dst_ld,
                int64_t prows, int64_t pcols, void* hip_stream)
{
    if (!src || !dst || rows < 0 || cols < 0 || prows < 0 || pcols < 0 || src_ld < cols || dst_ld < pcols ||
        prows > 262140 || pcols > 0x7fffffff) {
        set_error("sw_pad_copy: bad argument");
        return SW_EINVAL;
    }
    hipError_t e = launch_pad_copy(src, src_ld, rows, cols, dst, dst_ld, prows, pcols, (hipStream_t)hip_stream);
    return e == hipSuccess ? SW_OK : hip_fail(e, "sw_pad_copy");
}

// ---- measurement ----------------------------------------------------------------------------------------------------

int sw_profile_enable(int on)
{
    g_prof_on = on != 0;
    return SW_OK;
}

int sw_profile_read(double* ms, int64_t* launches, double* work)
{
    if (!ms || !launches || !work) { set_error("NULL output"); return SW_EINVAL; }
    for (int i = 0; i < SW_NUM_CLASSES; ++i) { ms[i] = 0.0; launches[i] = 0; work[i] = 0.0; }
    hipError_t bad = hipSuccess;
    std::lock_guard<std::mutex> guard(g_prof.mu);
    for (auto& r : g_prof.recs) {
        if (r.e0 && r.e1) {
            float t = 0.f;
            hipError_t e = hipEventSynchronize(r.e1);
            if (e == hipSuccess) e = hipEventElapsedTime(&t, r.e0, r.e1);
            if (e == hipSuccess) {
                ms[r.cls] += (double)t;
                launches[r.cls] += 1;
                work[r.cls] += r.work;
            } else if (bad == hipSuccess) {
                bad = e;
            }
        }
        if (r.e0) g_prof.pool.push_back(r.e0);
        if (r.e1) g_prof.pool.push_back(r.e1);
    }
    g_prof.recs.clear();
    return bad == hipSuccess ? SW_OK : hip_fail(bad, "sw_profile_read");
}

}  // extern "C"
