// Host side of the batched Estimator: the C ABI of include/estimator.h, input validation, the
// per-run plan (which streams feed which stage) and the tiling of candidates over device scratch.
// Every step of the simulation itself runs in the kernels of est_device.h.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/estimator.h"
#include "est_backend.h"
#include "est_types.h"

static_assert(sizeof(EstStageCfg) == sizeof(est_stage_cfg_t), "configuration entry layout");

#include "est_handle.h"

namespace {

int fail(estimator *h, int code, const char *fmt, ...) {
    if (h) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        h->err = buf;
    }
    return code;
}

int dev_fail(estimator *h, const char *what) { return fail(h, EST_EDEVICE, "%s: %s", what, estbe::last_error()); }

uint64_t pow2ceil(uint64_t x) {
    uint64_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

// Sizes of one candidate's scratch, in units of each area.
struct Sizes {
    uint64_t state_words = 0, ring_elems = 0, rep_words = 0, slot_words = 0, tab_bytes = 0;
    uint64_t per_cfg_bytes(uint64_t n, bool with_lat) const {
        return state_words * 4 + ring_elems * 8 + rep_words * 4 + slot_words * 4 + tab_bytes + (with_lat ? n * 4 : 0);
    }
};

struct PlanOut {
    EstPlan plan;
    Sizes sz;
    uint32_t n_acc = 0;
    uint32_t lds_bytes = 0;
    uint32_t acc_stage[EST_MAX_STAGES + 1];
    uint8_t acc_slot_of_src[EST_MAX_STAGES + 1][EST_TRACE_BIT + 1];
};

// Build the operation list for one run from the DAG and what the trace scan found.
//
// For stage c (and for the virtual sink, index S) the trace scan gives the union over visiting
// queries of the query's nearest visited ancestors.  Those are the streams the stage's input has to
// be merged from.  A stage fed by exactly one stream, every element of which visits the stage, reads
// that stream directly.
int build_plan(estimator *h, const EstStatus &st, uint64_t n, PlanOut &po, bool small_rings = false) {
    const uint32_t S = h->dag.S;
    EstPlan &P = po.plan;
    memset(&P, 0, sizeof P);
    memset(po.acc_slot_of_src, 0xFF, sizeof po.acc_slot_of_src);

    auto count_of = [&](uint32_t src) -> uint64_t { return src == EST_TRACE_BIT ? n : st.n_visit[src]; };

    uint32_t max_rb = 1;
    for (uint32_t s = 0; s < S; ++s) max_rb = std::max(max_rb, st.r_max[s] * st.b_max[s]);
    // A bounded ring must take a whole group of batches that complete together (<= R*B members)
    // while its consumer still holds back a look-ahead window, and a merge wants 64 x sources free.
    // Beyond that need, longer rings let an operation run longer before it has to hand over to its neighbour:
    // 8,192 elements (64 KB) instead of the 1,024 the need alone gives take 4 % off a sweep of the ten-stage
    // pipeline (11.0 -> 10.5 s; 32,768 and more: 10.5 s).  A run inside a fixed scratch keeps the short ones (more
    // candidates in flight matter more there), and so does a call that gives each candidate several wavefronts.  EST_RING_ELEMS sets another floor (tests use a small one, so that
    // short traces wrap the rings).
    uint64_t ring_floor = small_rings ? 1024 : 8192;
    if (const char *e = getenv("EST_RING_ELEMS"))
        if (atol(e) >= 64 && atol(e) <= (1l << 24)) ring_floor = (uint64_t)atol(e);
    const uint64_t cap_bounded = pow2ceil(std::max<uint64_t>(ring_floor, (uint64_t)max_rb + 64 * EST_KMAX + 65));

    std::vector<int32_t> out_ring(S, -1), in_ring(S, -1);
    struct Src { uint32_t n; int32_t ring_src[EST_KMAX]; };  // ring_src: stage index or EST_TRACE_BIT
    std::vector<Src> srcs(S + 1);
    std::vector<bool> direct(S + 1, false), filtered(S + 1, false), live(S + 1, false);

    for (uint32_t c = 0; c <= S; ++c) {
        live[c] = c == S ? true : st.n_visit[c] > 0;
        srcs[c].n = 0;
        if (!live[c]) continue;
        uint64_t u = st.src_union[c];
        if (u == 0) return fail(h, EST_EINTERNAL, "stage %u is visited but has no input stream", c);
        for (uint32_t b = 0; b <= EST_TRACE_BIT; ++b) {
            if (!((u >> b) & 1ull)) continue;
            if (srcs[c].n == EST_KMAX)
                return fail(h, EST_EUNSUPPORTED, "stage %u draws from more than %d input streams", c, EST_KMAX);
            if (b != EST_TRACE_BIT && (b >= S || !live[b]))
                return fail(h, EST_EINTERNAL, "stage %u fed by dead stage %u", c, b);
            po.acc_slot_of_src[c][b] = (uint8_t)srcs[c].n;
            srcs[c].ring_src[srcs[c].n++] = (int32_t)b;
        }
        direct[c] = c < S && srcs[c].n == 1 && count_of((uint32_t)srcs[c].ring_src[0]) == st.n_visit[c];
        // one source, but only some of its elements visit the stage: the scan filters while it reads
        filtered[c] = c < S && srcs[c].n == 1 && !direct[c];
    }

    // rings
    uint32_t nr = 0;
    for (uint32_t s = 0; s < S; ++s) {
        if (!live[s]) continue;
        out_ring[s] = (int32_t)nr++;
        if (!direct[s] && !filtered[s]) in_ring[s] = (int32_t)nr++;
    }
    P.n_rings = nr;

    // operations in topological order, consumers registered on the rings they read
    uint32_t no = 0, ne = 0;
    auto add_consumer = [&](int32_t ring, uint32_t edge) -> bool {
        if (ring < 0) return true;
        EstRing &R = P.rings[ring];
        if (R.n_cons == EST_MAX_CONS) return false;
        R.cons_edge[R.n_cons++] = (uint16_t)edge;
        return true;
    };
    auto ring_of_src = [&](int32_t src) -> int32_t { return src == EST_TRACE_BIT ? EST_SRC_TRACE : out_ring[src]; };

    for (uint32_t c = 0; c <= S; ++c) {
        if (!live[c]) continue;
        if (c == S || (!direct[c] && !filtered[c])) {
            EstOp &op = P.ops[no++];
            op.type = c == S ? EST_OP_LAT : EST_OP_MERGE;
            op.stage = c;
            op.n_src = srcs[c].n;
            for (uint32_t j = 0; j < srcs[c].n; ++j) {
                op.src_ring[j] = ring_of_src(srcs[c].ring_src[j]);
                op.src_edge[j] = ne;
                if (!add_consumer(op.src_ring[j], ne)) return fail(h, EST_EUNSUPPORTED, "too many consumers of one stream");
                ++ne;
            }
            op.out_ring = c == S ? -1 : in_ring[c];
            op.acc_idx = po.n_acc;
            po.acc_stage[po.n_acc++] = c;
            op.has_cnt = st.multi[c] ? 1 : 0;
            if (op.has_cnt) {
                // every stream that feeds some query together with another stream gets a table of times by query
                op.tab_off = po.sz.tab_bytes;
                op.tab_len = (uint32_t)align_up(n, 64);
                for (uint32_t j = 0; j < srcs[c].n; ++j)
                    if ((st.multi_union[c] >> srcs[c].ring_src[j]) & 1ull) op.tab_mask |= 1u << j;
                po.sz.tab_bytes += (uint64_t)__builtin_popcount(op.tab_mask) * op.tab_len * 4;
            }
        }
        if (c < S) {
            EstOp &op = P.ops[no++];
            op.type = EST_OP_SCAN;
            op.stage = c;
            op.n_src = 1;
            op.src_ring[0] = (direct[c] || filtered[c]) ? ring_of_src(srcs[c].ring_src[0]) : in_ring[c];
            op.filtered = filtered[c] ? 1 : 0;
            if (filtered[c]) {
                op.acc_idx = po.n_acc;
                po.acc_stage[po.n_acc++] = c;
            }
            op.src_edge[0] = ne;
            if (!add_consumer(op.src_ring[0], ne)) return fail(h, EST_EUNSUPPORTED, "too many consumers of one stream");
            ++ne;
            op.out_ring = out_ring[c];
            op.r_max = st.r_max[c];
            op.b_max = st.b_max[c];
            op.rep_off = (uint32_t)po.sz.rep_words;
            po.sz.rep_words += 3ull * op.r_max;
            op.slot_off = po.sz.slot_words;
            po.sz.slot_words += (uint64_t)op.r_max * op.b_max;
        }
    }
    P.n_ops = no;
    P.n_edges = ne;
    {
        // several wavefronts per candidate: the operations, in pipeline order, are cut into EST_MW_WAVES runs of
        // about equal work (elements an operation reads), so that neighbouring wavefronts are neighbouring pipeline sections
        std::vector<uint64_t> work(no);
        uint64_t total = 0;
        for (uint32_t i = 0; i < no; ++i) {
            const EstOp &op = P.ops[i];
            uint64_t wk = 0;
            for (uint32_t j = 0; j < op.n_src; ++j)
                wk += op.src_ring[j] == EST_SRC_TRACE ? n : (op.type == EST_OP_SCAN && !op.filtered ? st.n_visit[op.stage] : n);
            work[i] = std::max<uint64_t>(wk, 1);
            total += work[i];
        }
        uint64_t acc = 0;
        for (uint32_t i = 0; i < no; ++i) {
            P.ops[i].owner = (uint32_t)std::min<uint64_t>(EST_MW_WAVES - 1, acc * EST_MW_WAVES / total);
            acc += work[i];
        }
    }
    P.max_src = 1;
    for (uint32_t i = 0; i < no; ++i) P.max_src = std::max(P.max_src, P.ops[i].n_src);
    // the scans' in-ring: 256 keys, or 128 where that lets one more wavefront share a SIMD (the smaller ring is
    // refilled twice as often, which costs less than the extra wavefront brings)
    const uint32_t lds256 = (uint32_t)align_up(std::max<uint64_t>(EST_LDS_MERGE_BYTES(P.max_src), EST_LDS_SCAN_BYTES(max_rb, 256u)), 256);
    const uint32_t lds128 = (uint32_t)align_up(std::max<uint64_t>(EST_LDS_MERGE_BYTES(P.max_src), EST_LDS_SCAN_BYTES(max_rb, 128u)), 256);
    P.scan_ring = estbe::waves_per_simd(lds128) > estbe::waves_per_simd(lds256) ? 128u : 256u;
    if (const char *e = getenv("EST_SCAN_RING"))  // for tests: 128 or 256
        if (atoi(e) == 128 || atoi(e) == 256) P.scan_ring = (uint32_t)atoi(e);
    po.lds_bytes = P.scan_ring == 128u ? lds128 : lds256;

    // ring capacities: a stream read by several operations may have to hold the whole skew between
    // them (one branch of a fork can lag another by the length of its simulated queue), so it gets
    // room for every element; a stream with one reader is a bounded ring
    uint64_t off = 0;
    for (uint32_t s = 0; s < S; ++s) {
        if (!live[s]) continue;
        {
            EstRing &R = P.rings[out_ring[s]];
            uint64_t cap = R.n_cons >= 2 ? std::max<uint64_t>(cap_bounded, pow2ceil(st.n_visit[s])) : cap_bounded;
            R.off = off;
            R.cap_mask = (uint32_t)(cap - 1);
            off += cap;
        }
        if (in_ring[s] >= 0) {
            EstRing &R = P.rings[in_ring[s]];
            R.off = off;
            R.cap_mask = (uint32_t)(cap_bounded - 1);
            off += cap_bounded;
        }
    }
    po.sz.ring_elems = off;

    P.wr_off = 0;
    P.fin_off = P.n_rings;
    P.rd_off = 2 * P.n_rings;
    P.done_off = P.rd_off + P.n_edges;
    P.miss_off = P.done_off + P.n_ops;
    P.pub_off = P.miss_off + 2;
    P.state_words = (uint32_t)align_up(P.pub_off + P.n_rings, 4);
    po.sz.state_words = P.state_words;
    po.sz.rep_words = align_up(po.sz.rep_words, 4);
    po.sz.slot_words = align_up(po.sz.slot_words, 4);
    return EST_OK;
}

struct EventSet {
    std::vector<void *> ev;
    ~EventSet() {
        for (void *e : ev) estbe::event_destroy(e);
    }
    void *make() {
        void *e = estbe::event_create();
        if (e) ev.push_back(e);
        return e;
    }
};

enum { MODE_P99 = 0, MODE_LAT = 1 };

struct DevBuf {
    void *p = nullptr;
    ~DevBuf() {
        if (p) estbe::dfree(p);
    }
    bool alloc(size_t bytes) {
        p = estbe::dmalloc(bytes ? bytes : 4);
        return p != nullptr;
    }
};



int run_core(estimator *h, uint64_t n, const uint32_t *d_arrival, const uint32_t *d_mask,
             const est_stage_cfg_t *d_cfg, uint64_t n_cfg, uint32_t slo_us, int mode, uint32_t *d_p99,
             uint32_t *d_miss, uint64_t *d_cost, uint32_t *d_lat_out, void *workspace, uint64_t workspace_bytes,
             void *stream, bool no_alloc = false) {
    if (n >= (1ull << 31)) return fail(h, EST_EINVAL, "trace too long (%llu queries)", (unsigned long long)n);
    if (n_cfg >= (1ull << 31)) return fail(h, EST_EINVAL, "too many configurations");
    if (n_cfg == 0) return EST_OK;
    const uint32_t S = h->dag.S;
    // (a run that must not allocate uses the handle's events and page-locked staging, and no diagnostics buffer)
    EventSet evs;
    void *ev_p0 = no_alloc ? h->ev[0] : evs.make(), *ev_p1 = no_alloc ? h->ev[1] : evs.make(), *ev_p2 = no_alloc ? h->ev[2] : evs.make(),
         *ev_p3 = no_alloc ? h->ev[3] : evs.make();
    if (!ev_p0 || !ev_p1 || !ev_p2 || !ev_p3) return dev_fail(h, "event create");
    if (no_alloc && !workspace) return fail(h, EST_EINTERNAL, "no scratch");

    // ---- scan the configurations and the trace
    if (estbe::zero(h->d_status, sizeof(EstStatus), stream)) return dev_fail(h, "clear status");
    estbe::event_record(ev_p0, stream);
    EstCfgArgs ca;
    ca.dag = h->d_dag;
    ca.cfg = (const EstStageCfg *)d_cfg;
    ca.n_cfg = n_cfg;
    ca.status = h->d_status;
    if (estbe::launch_cfg(ca, stream)) return dev_fail(h, "configuration scan");
    EstPrepArgs pa;
    memset(&pa, 0, sizeof pa);
    pa.dag = h->d_dag;
    pa.arrival = d_arrival;
    pa.mask = d_mask;
    pa.n = (uint32_t)n;
    pa.status = h->d_status;
    if (n > 0 && estbe::launch_prep1(pa, stream)) return dev_fail(h, "trace scan");
    estbe::event_record(ev_p1, stream);
    EstStatus st_local;
    EstStatus &st = no_alloc ? h->pin->st[0] : st_local;
    if (estbe::d2h(&st, h->d_status, sizeof st, stream) || estbe::sync(stream)) return dev_fail(h, "read status");
    if (st.bad_cfg) return fail(h, EST_EINVAL, "a configuration entry is out of range (hw < %u, 1 <= batch <= %u, 1 <= replicas <= %d)",
                                h->dag.H, h->dag.Bmax, EST_MAX_REPLICAS);
    if (st.bad_trace) return fail(h, EST_EINVAL, "arrival times decrease");
    if (n > 0 && (uint64_t)st.last_arrival + h->sum_max_lat + slo_us >= EST_HORIZON_US)
        return fail(h, EST_EINVAL, "trace too close to the horizon: last arrival %u + worst service %llu + slo %u >= 2^32-1",
                    st.last_arrival, (unsigned long long)h->sum_max_lat, slo_us);
    st.n_visit[S] = (uint32_t)n;

    PlanOut po;
    po.sz = Sizes();
    po.n_acc = 0;
    if (n > 0) {
        // Calls whose candidates will get several wavefronts each (below) keep the short rings: there the operations of
        // a candidate run side by side, and a consumer starts when its producer first hands over, so long rings delay
        // the pipeline instead of saving hand-overs (the planner on a five-stage pipeline: 0.67 s with short rings,
        // 0.72 s with long ones).
        bool small_rings = no_alloc;
        const char *e = getenv("EST_WAVES_PER_CANDIDATE");
        if (e ? (atoi(e) == 2 || atoi(e) == EST_MW_WAVES) : n_cfg * 2 <= (uint64_t)estbe::max_resident_groups(1024, EST_MW_WAVES) * 3)
            small_rings = true;
        int rc = build_plan(h, st, n, po, small_rings);
        if (rc != EST_OK) return rc;
    } else {
        memset(&po.plan, 0, sizeof po.plan);
        po.plan.state_words = 4;
        po.sz.state_words = 4;
    }
    const bool with_lat = mode == MODE_P99 && n > 0;

    // ---- lay out the scratch
    const uint64_t n_pad = align_up(std::max<uint64_t>(n, 1), 256);
    uint64_t fixed = 0;
    auto take = [&](uint64_t bytes) {
        uint64_t at = fixed;
        fixed = align_up(fixed + bytes, 256);
        return at;
    };
    const uint64_t o_keys = take(n_pad * 8);
    const uint64_t o_acc = take((uint64_t)std::max<uint32_t>(po.n_acc, 1) * n_pad);
    const uint64_t o_p99 = take(n_cfg * 4);
    const uint64_t o_miss = take(n_cfg * 4);
    const uint64_t o_cost = take(n_cfg * 8);
    const uint64_t per_cfg = po.sz.per_cfg_bytes(n, with_lat) + 64;  // + alignment slack per area

    uint8_t *ws = (uint8_t *)workspace;
    uint64_t ws_bytes = workspace_bytes;
    if (!ws) {
        const uint64_t max_slots = std::min<uint64_t>(n_cfg, std::max<uint32_t>(estbe::max_resident_waves(po.lds_bytes), 1));
        uint64_t want = fixed + per_cfg * max_slots + 8 * 256;
        uint64_t avail = (uint64_t)estbe::mem_free() + h->ws_bytes;
        uint64_t budget = std::min<uint64_t>(want, avail / 100 * 92);  // (an allocation that fails is tried again smaller, below)
        // (when the free memory is what limits the scratch, the budget moves a little from call to call with whatever
        // else the process allocates: a cached workspace within a sixteenth of it is kept, since freeing and
        // allocating a few hundred GB costs seconds)
        const bool too_small = budget < want ? h->ws_bytes < budget - budget / 16 : h->ws_bytes < budget;
        if (too_small || h->ws_bytes > 2 * budget + (64u << 20)) {
            if (h->ws) estbe::dfree(h->ws);
            h->ws = nullptr;
            h->ws_bytes = 0;
            // (a little more than this call needs, when there is room: a later call with some more candidates, whose
            // result staging is a few bytes each, then finds the cached scratch large enough)
            if (budget == want) budget = std::min<uint64_t>(want + std::min<uint64_t>(64ull << 20, want / 64 + (1ull << 20)), std::max<uint64_t>(want, avail / 100 * 92));
            h->ws = estbe::dmalloc(budget);
            if (!h->ws && budget > want) {
                budget = want;
                h->ws = estbe::dmalloc(budget);
            }
            for (int shrink = 0; !h->ws && shrink < 3 && budget < want; ++shrink) {  // the free memory was less than reported: fewer slots
                budget = budget / 8 * 7;
                h->ws = estbe::dmalloc(budget);
            }
            if (!h->ws) return fail(h, EST_ENOMEM, "cannot allocate %llu bytes of device scratch", (unsigned long long)budget);
            h->ws_bytes = budget;
        }
        ws = (uint8_t *)h->ws;
        ws_bytes = h->ws_bytes;
    }
    if (((uintptr_t)ws & 255) != 0) return fail(h, EST_EINVAL, "workspace must be 256-byte aligned");
    if (ws_bytes < fixed + per_cfg + 8 * 256)
        return fail(h, EST_ENOMEM, "workspace of %llu bytes cannot hold one candidate (%llu + %llu bytes needed)",
                    (unsigned long long)ws_bytes, (unsigned long long)fixed, (unsigned long long)per_cfg);
    // scratch slots: one per wavefront that works on this launch; more than the device can hold at once
    // would only wait
    uint64_t n_slots = std::min<uint64_t>((ws_bytes - fixed - 8 * 256) / per_cfg, n_cfg);
    n_slots = std::min<uint64_t>(n_slots, std::max<uint32_t>(estbe::max_resident_waves(po.lds_bytes), 1));
    // A call with so few candidates that most of the device would stay empty gives every candidate a workgroup of
    // EST_MW_WAVES wavefronts instead of one wavefront, up to one and a half times the workgroups the device holds at
    // once (EST_WAVES_PER_CANDIDATE = 1, 2 or 4 overrides the choice).  Measured on a ten-stage pipeline, 10^6 queries,
    // 1,536 resident workgroups of four, kernel seconds with 1 / 2 / 4 wavefronts per candidate: 1,024 candidates
    // 0.87 / 0.65 / 0.41; 1,536: 1.17 / 0.91 / 0.65; 2,304: 1.28 / 1.06 / 0.92; 3,072: 1.27 / 1.18 / 1.04; on a
    // five-stage pipeline four stop paying at 2,048 candidates (104 / 104 / 102 ms; 3,072: 117 / 127 / 136).
    // Workgroups of two are never better than both alternatives by much, so they are not chosen automatically.
    uint32_t nw = 1;  // wavefronts per candidate
    if (n > 0 && po.plan.n_ops >= 2 && n_cfg <= n_slots && n_cfg * 2 <= (uint64_t)estbe::max_resident_groups(po.lds_bytes, EST_MW_WAVES) * 3)
        nw = EST_MW_WAVES;
    if (const char *e = getenv("EST_WAVES_PER_CANDIDATE")) nw = n > 0 && (atoi(e) == 2 || atoi(e) == EST_MW_WAVES) ? (uint32_t)atoi(e) : 1;
    if (getenv("EST_DEBUG_TICKS") && !no_alloc) nw = 1;  // (the step counters are per wavefront)
    const bool several = nw > 1;
    if (several) {
        n_slots = std::min<uint64_t>(n_slots, std::max<uint32_t>(estbe::max_resident_groups(po.lds_bytes, nw), 1));
        // (build_plan cut the operations into EST_MW_WAVES runs; a smaller workgroup takes neighbouring runs together)
        for (uint32_t i = 0; i < po.plan.n_ops; ++i) po.plan.ops[i].owner = po.plan.ops[i].owner * nw / EST_MW_WAVES;
    }
    uint64_t at = fixed;
    auto area = [&](uint64_t bytes_per_cfg) {
        uint64_t a0 = at;
        at = align_up(at + bytes_per_cfg * n_slots, 256);
        return a0;
    };
    const uint64_t o_state = area(po.sz.state_words * 4);
    const uint64_t o_rings = area(po.sz.ring_elems * 8);
    const uint64_t o_rep = area(po.sz.rep_words * 4);
    const uint64_t o_slots = area(po.sz.slot_words * 4);
    const uint64_t o_tab = area(po.sz.tab_bytes);
    const uint64_t o_lat = area(with_lat ? n * 4 : 0);
    if (at > ws_bytes) return fail(h, EST_EINTERNAL, "scratch layout overflow");

    // ---- per-query tables
    estbe::event_record(ev_p2, stream);
    if (n > 0) {
        const EstPlan *plan_src = &po.plan;
        if (no_alloc) {
            h->pin->plan = po.plan;
            plan_src = &h->pin->plan;
        }
        if (estbe::h2d(h->d_plan, plan_src, sizeof(EstPlan), stream)) return dev_fail(h, "upload plan");
        pa.trace_keys = (uint64_t *)(ws + o_keys);
        pa.acc = ws + o_acc;
        pa.acc_stride = n_pad;
        pa.n_acc = po.n_acc;
        memcpy(pa.acc_stage, po.acc_stage, sizeof(uint32_t) * po.n_acc);
        memcpy(pa.acc_slot_of_src, po.acc_slot_of_src, sizeof pa.acc_slot_of_src);
        if (estbe::launch_prep2(pa, stream)) return dev_fail(h, "trace tables");
    }
    estbe::event_record(ev_p3, stream);

    // ---- the simulation launch
    uint32_t *s_p99 = (uint32_t *)(ws + o_p99);
    uint32_t *s_miss = (uint32_t *)(ws + o_miss);
    uint64_t *s_cost = (uint64_t *)(ws + o_cost);
    if (n == 0 && mode == MODE_P99) {
        if (estbe::zero(s_p99, n_cfg * 4, stream) || estbe::zero(s_miss, n_cfg * 4, stream)) return dev_fail(h, "clear results");
    }
    // diagnostics: EST_DEBUG_TICKS=<file> dumps how long each candidate's wavefront ran (100 MHz ticks)
    const char *dbg_path = getenv("EST_DEBUG_TICKS");
    DevBuf dbg_buf;
    uint64_t *dbg_ticks = nullptr;
    const uint64_t dbg_words = n_cfg * (1 + (uint64_t)EST_DBG_WORDS * EST_MAX_STAGES);  // per candidate: ticks, then the counters per stage
    if (dbg_path && !no_alloc && n > 0 && dbg_buf.alloc(dbg_words * 8) && !estbe::zero(dbg_buf.p, dbg_words * 8, stream)) dbg_ticks = (uint64_t *)dbg_buf.p;
    void *e0 = no_alloc ? h->ev[4] : evs.make(), *e1 = no_alloc ? h->ev[5] : evs.make();
    if (!e0 || !e1) return dev_fail(h, "event create");
    estbe::event_record(e0, stream);
    {
        EstSimArgs sa;
        memset(&sa, 0, sizeof sa);
        sa.plan = h->d_plan;
        sa.dag = h->d_dag;
        sa.lat_us = h->d_lat;
        sa.cost_uusd_hr = h->d_cost;
        sa.arrival = d_arrival;
        sa.trace_keys = (const uint64_t *)(ws + o_keys);
        sa.acc = ws + o_acc;
        sa.acc_stride = n_pad;
        sa.cfg = (const EstStageCfg *)d_cfg;
        sa.n = (uint32_t)n;
        sa.n_cfg = (uint32_t)n_cfg;
        sa.slo_us = slo_us;
        sa.lat_by_qid = mode == MODE_LAT;
        sa.max_src = po.plan.max_src;
        sa.lds_bytes = n > 0 ? po.lds_bytes : 1024;
        sa.n_slots = (uint32_t)n_slots;
        sa.have_lat = with_lat ? 1 : 0;
        sa.state = (uint32_t *)(ws + o_state);  sa.state_stride = po.sz.state_words;
        sa.rings = (uint64_t *)(ws + o_rings);  sa.ring_stride = po.sz.ring_elems;
        sa.rep = (uint32_t *)(ws + o_rep);      sa.rep_stride = po.sz.rep_words;
        sa.slots = (uint32_t *)(ws + o_slots);  sa.slot_stride = po.sz.slot_words;
        sa.tabs = ws + o_tab;               sa.tab_stride = po.sz.tab_bytes;
        if (mode == MODE_LAT) {
            sa.lat = d_lat_out;
            sa.lat_stride = n;
        } else {
            sa.lat = (uint32_t *)(ws + o_lat);
            sa.lat_stride = n;
        }
        sa.status = h->d_status;
        sa.dbg_ticks = dbg_ticks;
        sa.p99 = s_p99; sa.miss = s_miss; sa.cost = s_cost;
        if (mode == MODE_P99 || n > 0)
            if (several ? estbe::launch_sim_mw(sa, nw, stream) : estbe::launch_sim(sa, stream)) return dev_fail(h, "simulation kernel");
    }
    estbe::event_record(e1, stream);
    EstStatus st2_local;
    EstStatus &st2 = no_alloc ? h->pin->st[1] : st2_local;
    if (estbe::d2h(&st2, h->d_status, sizeof st2, stream) || estbe::sync(stream)) return dev_fail(h, "run");
    if (st2.sim_error) return fail(h, EST_EINTERNAL, "the simulation kernel stopped without finishing a candidate");
    if (dbg_ticks) {
        std::vector<uint64_t> ticks(dbg_words);
        if (!estbe::d2h(ticks.data(), dbg_ticks, dbg_words * 8, stream) && !estbe::sync(stream)) {
            if (FILE *f = fopen(dbg_path, "wb")) {
                fwrite(ticks.data(), 8, dbg_words, f);
                fclose(f);
            }
        }
    }
    if (mode == MODE_P99) {
        if (estbe::d2d(d_p99, s_p99, n_cfg * 4, stream) || estbe::d2d(d_miss, s_miss, n_cfg * 4, stream) ||
            estbe::d2d(d_cost, s_cost, n_cfg * 8, stream) || estbe::sync(stream))
            return dev_fail(h, "copy results");
    }
    est_stats_t &ss = h->stats;
    memset(&ss, 0, sizeof ss);
    ss.n_launches = 1;
    ss.n_slots = (uint32_t)n_slots;
    ss.waves_per_candidate = nw;
    ss.sim_ms = estbe::event_ms(e0, e1);
    ss.prep_ms = estbe::event_ms(ev_p0, ev_p1) + estbe::event_ms(ev_p2, ev_p3);
    for (uint32_t s = 0; s < S; ++s) ss.stage_visits += st.n_visit[s];
    ss.workspace_bytes = at;
    h->have_stats = true;
    return EST_OK;
}

// Candidates that share upstream stages with a base configuration (Section 4.3: the candidates of a
// planner step differ from the current configuration in one model).  A stage's output depends only on
// the configurations of the stage and of its ancestors, so for every candidate the operations whose
// stage and ancestors are configured as in the candidate's base are not run: their output streams are
// read from one captured run of the base.  Two launches: the bases, leaving the streams some candidate
// will read in full-length buffers (and running only what those streams need); then the candidates.
int run_shared_core(estimator *h, uint64_t n, const uint32_t *d_arrival, const uint32_t *d_mask, const est_stage_cfg_t *d_bases,
                    uint64_t n_bases, const est_stage_cfg_t *d_cfg, const uint32_t *d_base_of, uint64_t n_cfg, uint32_t slo_us,
                    uint32_t *d_p99, uint32_t *d_miss, uint64_t *d_cost, void *stream) {
    if (n >= (1ull << 31)) return fail(h, EST_EINVAL, "trace too long (%llu queries)", (unsigned long long)n);
    if (n_cfg >= (1ull << 31) || n_bases >= (1ull << 31)) return fail(h, EST_EINVAL, "too many configurations");
    if (n_cfg == 0) return EST_OK;
    if (n == 0 || n_bases == 0)  // nothing to share
        return run_core(h, n, d_arrival, d_mask, d_cfg, n_cfg, slo_us, MODE_P99, d_p99, d_miss, d_cost, nullptr, nullptr, 0, stream);
    const uint32_t S = h->dag.S;
    EventSet evs;
    void *ev_p0 = evs.make(), *ev_p1 = evs.make(), *ev_p2 = evs.make(), *ev_p3 = evs.make();
    void *e0 = evs.make(), *e2 = evs.make();
    if (!ev_p0 || !ev_p1 || !ev_p2 || !ev_p3 || !e0 || !e2) return dev_fail(h, "event create");

    // ---- scan the configurations (bases and candidates) and the trace
    if (estbe::zero(h->d_status, sizeof(EstStatus), stream)) return dev_fail(h, "clear status");
    estbe::event_record(ev_p0, stream);
    EstCfgArgs ca;
    ca.dag = h->d_dag;
    ca.status = h->d_status;
    ca.cfg = (const EstStageCfg *)d_bases;
    ca.n_cfg = n_bases;
    if (estbe::launch_cfg(ca, stream)) return dev_fail(h, "configuration scan");
    ca.cfg = (const EstStageCfg *)d_cfg;
    ca.n_cfg = n_cfg;
    if (estbe::launch_cfg(ca, stream)) return dev_fail(h, "configuration scan");
    EstPrepArgs pa;
    memset(&pa, 0, sizeof pa);
    pa.dag = h->d_dag;
    pa.arrival = d_arrival;
    pa.mask = d_mask;
    pa.n = (uint32_t)n;
    pa.status = h->d_status;
    if (estbe::launch_prep1(pa, stream)) return dev_fail(h, "trace scan");
    estbe::event_record(ev_p1, stream);
    EstStatus st;
    std::vector<est_stage_cfg_t> cfg(n_cfg * S), bases(n_bases * S);
    std::vector<uint32_t> base_of(n_cfg);
    if (estbe::d2h(&st, h->d_status, sizeof st, stream) || estbe::d2h(cfg.data(), d_cfg, cfg.size() * sizeof(est_stage_cfg_t), stream) ||
        estbe::d2h(bases.data(), d_bases, bases.size() * sizeof(est_stage_cfg_t), stream) ||
        estbe::d2h(base_of.data(), d_base_of, n_cfg * 4, stream) || estbe::sync(stream))
        return dev_fail(h, "read status and configurations");
    if (st.bad_cfg) return fail(h, EST_EINVAL, "a configuration entry is out of range (hw < %u, 1 <= batch <= %u, 1 <= replicas <= %d)",
                                h->dag.H, h->dag.Bmax, EST_MAX_REPLICAS);
    if (st.bad_trace) return fail(h, EST_EINVAL, "arrival times decrease");
    if ((uint64_t)st.last_arrival + h->sum_max_lat + slo_us >= EST_HORIZON_US)
        return fail(h, EST_EINVAL, "trace too close to the horizon: last arrival %u + worst service %llu + slo %u >= 2^32-1",
                    st.last_arrival, (unsigned long long)h->sum_max_lat, slo_us);
    for (uint64_t t = 0; t < n_cfg; ++t)
        if (base_of[t] >= n_bases) return fail(h, EST_EINVAL, "base_of[%llu] = %u is not a base (%llu bases)", (unsigned long long)t, base_of[t], (unsigned long long)n_bases);
    st.n_visit[S] = (uint32_t)n;

    PlanOut po;
    po.sz = Sizes();
    po.n_acc = 0;
    int rc = build_plan(h, st, n, po);
    if (rc != EST_OK) return rc;
    const EstPlan &P = po.plan;
    if (P.n_ops > 64 || P.n_rings > 64) return fail(h, EST_EUNSUPPORTED, "shared runs handle at most 64 operations and 64 streams");

    // ---- which operations each candidate skips, which streams must be captured, what the capture has to run
    std::vector<int32_t> producer(P.n_rings, -1);
    for (uint32_t i = 0; i < P.n_ops; ++i)
        if (P.ops[i].out_ring >= 0) producer[P.ops[i].out_ring] = (int32_t)i;
    std::vector<uint64_t> skip(n_cfg);
    uint64_t captured_rings = 0;
    for (uint64_t t = 0; t < n_cfg; ++t) {
        const est_stage_cfg_t *c = &cfg[t * S], *b = &bases[(uint64_t)base_of[t] * S];
        uint64_t same = 0;  // operations whose output equals the base's
        for (uint32_t i = 0; i < P.n_ops; ++i) {
            const EstOp &op = P.ops[i];
            if (op.type == EST_OP_LAT) continue;
            bool eq = true;
            for (uint32_t j = 0; j < op.n_src; ++j)
                if (op.src_ring[j] >= 0 && !((same >> producer[op.src_ring[j]]) & 1ull)) eq = false;
            if (op.type == EST_OP_SCAN && memcmp(&c[op.stage], &b[op.stage], sizeof(est_stage_cfg_t)) != 0) eq = false;
            if (eq) same |= 1ull << i;
        }
        skip[t] = same;
        for (uint32_t i = 0; i < P.n_ops; ++i) {  // streams a skipped operation hands to one that runs
            if ((same >> i) & 1ull) continue;
            const EstOp &op = P.ops[i];
            for (uint32_t j = 0; j < op.n_src; ++j)
                if (op.src_ring[j] >= 0 && ((same >> producer[op.src_ring[j]]) & 1ull)) captured_rings |= 1ull << op.src_ring[j];
        }
    }
    uint64_t needed = 0;  // the producers of the captured streams and everything upstream of them
    for (int32_t i = (int32_t)P.n_ops - 1; i >= 0; --i) {
        const EstOp &op = P.ops[i];
        if (op.out_ring >= 0 && ((captured_rings >> op.out_ring) & 1ull)) needed |= 1ull << i;
        if ((needed >> i) & 1ull)
            for (uint32_t j = 0; j < op.n_src; ++j)
                if (op.src_ring[j] >= 0) needed |= 1ull << producer[op.src_ring[j]];
    }
    const uint64_t all_ops = P.n_ops == 64 ? ~0ull : ((1ull << P.n_ops) - 1ull);

    // the capture's layout: the same operations and streams; captured streams, and streams one of whose
    // readers the capture does not run, with room for every element
    // (nobody consumes during the capture, and a producer only writes while it sees the free room a
    // bounded ring offers when its reader has caught up: so that much room on top of the stream itself)
    EstPlan PC = P;
    uint64_t cap_elems = 0, room = ~0ull;
    for (uint32_t r = 0; r < P.n_rings; ++r) room = std::min<uint64_t>(room, (uint64_t)P.rings[r].cap_mask + 1);
    for (uint32_t r = 0; r < P.n_rings; ++r) {
        uint64_t cap = (uint64_t)P.rings[r].cap_mask + 1;
        bool idle_reader = false;  // a reader the capture does not run never frees anything
        for (uint32_t i = 0; i < P.n_ops; ++i)
            for (uint32_t j = 0; j < P.ops[i].n_src; ++j)
                if (P.ops[i].src_ring[j] == (int32_t)r && !((needed >> i) & 1ull)) idle_reader = true;
        if (((captured_rings >> r) & 1ull) || (idle_reader && ((needed >> producer[r]) & 1ull)))
            cap = std::max<uint64_t>(cap, pow2ceil(st.n_visit[P.ops[producer[r]].stage] + room));
        PC.rings[r].off = cap_elems;
        PC.rings[r].cap_mask = (uint32_t)(cap - 1);
        cap_elems += cap;
    }

    // ---- rounds: when the captured streams of all bases do not fit beside the candidates' scratch, the bases
    //      are taken a group at a time, with two capture areas: while the candidates of one group run on the
    //      caller's stream, the next group's bases run on a second stream and fill the wavefront slots the
    //      candidates leave (a launch of a few hundred bases alone would leave most of the device idle for as
    //      long as one simulation takes)
    const uint64_t n_pad = align_up(std::max<uint64_t>(n, 1), 256);
    // (the bases need the joins' time tables only when their launch runs a join)
    uint64_t cap_tab_bytes = 0;
    for (uint32_t i = 0; i < P.n_ops; ++i)
        if (((needed >> i) & 1ull) && P.ops[i].tab_mask) cap_tab_bytes = po.sz.tab_bytes;
    const uint64_t cap_bytes = po.sz.state_words * 4 + cap_elems * 8 + po.sz.rep_words * 4 + po.sz.slot_words * 4 + cap_tab_bytes + 8 + 8;
    const uint64_t per_cfg = po.sz.per_cfg_bytes(n, true) + 64;
    const uint32_t resident = std::max<uint32_t>(estbe::max_resident_waves(po.lds_bytes), 1);
    const uint64_t avail = ((uint64_t)estbe::mem_free() + h->ws_bytes) / 100 * 85;
    const uint64_t fixed_est = n_pad * 8 + (uint64_t)std::max<uint32_t>(po.n_acc, 1) * n_pad + n_cfg * 32 + sizeof(EstPlan) + 2 * sizeof(EstStatus) + 64 * 256;
    uint64_t n_slots = std::min<uint64_t>(n_cfg, resident);
    uint64_t nb = n_bases;  // bases per round
    uint32_t n_areas = 1;
    // what a base brings in candidate work, in units of one full simulation: its candidates x the share of the
    // plan's elements they still move
    double all_work = 0, run_work = 0;
    for (uint32_t i = 0; i < P.n_ops; ++i) all_work += (double)st.n_visit[P.ops[i].stage];
    for (uint64_t t = 0; t < n_cfg; ++t)
        for (uint32_t i = 0; i < P.n_ops; ++i)
            if (!((skip[t] >> i) & 1ull)) run_work += (double)st.n_visit[P.ops[i].stage];
    const double work_per_base = std::max(run_work / std::max(all_work, 1.0) / (double)n_bases, 1e-3);
    if (fixed_est + n_bases * cap_bytes + per_cfg * n_slots > avail) {
        n_areas = 2;
        // A round's bases run beside the previous round's candidates and last as long as the slowest full simulation
        // among them; they stay hidden when the candidates of a round keep their wavefronts busy for at least that long.
        // In units of an average full simulation a base brings work_per_base of candidate work (its candidates x the
        // share of the plan's elements they still move), and the slowest of a round takes about two: so a round
        // wants at least n_slots / (work_per_base / 2) bases, and the memory is split between candidate slots and
        // the two capture areas in that proportion.
        const double room = avail > fixed_est ? (double)(avail - fixed_est) : 0.0;
        const double balanced = room / ((double)per_cfg + 2.0 * (double)cap_bytes * 2.0 / work_per_base);
        n_slots = std::min<uint64_t>(n_slots, std::max<uint64_t>(64, (uint64_t)balanced));
        for (;;) {
            const uint64_t rest = avail > fixed_est + per_cfg * n_slots ? avail - fixed_est - per_cfg * n_slots : 0;
            nb = rest / (2 * cap_bytes);
            if (nb >= 1 || n_slots <= 64) break;
            n_slots = std::max<uint64_t>(64, n_slots / 2);  // fewer candidates in flight to make room for one base per area
        }
        if (nb < 1)
            return fail(h, EST_ENOMEM, "one base's captured streams (%llu bytes) and one candidate's scratch (%llu) do not fit in %llu free bytes",
                        (unsigned long long)cap_bytes, (unsigned long long)per_cfg, (unsigned long long)avail);
        nb = std::min<uint64_t>(nb, n_bases);
    }
    if (const char *e = getenv("EST_SHARED_BASES_PER_ROUND")) {  // for tests: force small rounds
        const long v = atol(e);
        if (v >= 1 && (uint64_t)v < nb) {
            nb = (uint64_t)v;
            n_areas = 2;
        }
    }
    const uint64_t n_rounds = (n_bases + nb - 1) / nb;
    if (n_rounds == 1) n_areas = 1;
    if (n_rounds > 1 && !getenv("EST_SHARED_BASES_PER_ROUND") && !getenv("EST_SHARED_ALWAYS")) {
        // Sharing is an optimisation, not a semantics: when the rounds the memory forces are estimated to take longer
        // than simulating every candidate on its own, do that.  Times in units of one average full simulation on a
        // full device: a round lasts as long as its bases (about two, the slowest of them) or its candidates, the
        // launches of a round end on their own tails (x 1.3, measured), the first round's bases run alone.
        const double per_round = std::max(2.0, (double)nb * work_per_base / (double)n_slots);
        const double est_shared = 1.3 * (double)n_rounds * per_round + 2.0;
        const double est_plain = (double)n_cfg / (double)std::min<uint64_t>(n_cfg, resident);
        if (est_shared >= est_plain) {
            const int rc = run_core(h, n, d_arrival, d_mask, d_cfg, n_cfg, slo_us, MODE_P99, d_p99, d_miss, d_cost, nullptr, nullptr, 0, stream);
            if (rc == EST_OK) h->stats.ops_run_fraction = 1.0f;
            return rc;
        }
    }

    // candidates grouped by round; inside a round those that run the most operations are handed out first,
    // so that a launch ends on short ones
    std::vector<uint32_t> order(n_cfg), base_local(n_cfg);
    for (uint64_t t = 0; t < n_cfg; ++t) {
        order[t] = (uint32_t)t;
        base_local[t] = (uint32_t)(base_of[t] % nb);
    }
    std::vector<uint64_t> work(n_cfg, 0);  // elements the candidate's operations will move: what its run time goes with
    for (uint64_t t = 0; t < n_cfg; ++t)
        for (uint32_t i = 0; i < P.n_ops; ++i)
            if (!((skip[t] >> i) & 1ull)) work[t] += st.n_visit[P.ops[i].stage];
    std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) {
        const uint64_t rx = base_of[x] / nb, ry = base_of[y] / nb;
        if (rx != ry) return rx < ry;
        return work[x] > work[y];
    });
    std::vector<uint64_t> round_lo(n_rounds + 1, n_cfg);
    for (uint64_t i = n_cfg; i-- > 0;) round_lo[base_of[order[i]] / nb] = i;
    for (uint64_t k = n_rounds; k-- > 0;) round_lo[k] = std::min(round_lo[k], round_lo[k + 1]);  // rounds without candidates

    // ---- lay out the scratch (in the handle's cached workspace, grown when it is too small)
    uint64_t at = 0;
    auto take = [&](uint64_t bytes) {
        uint64_t a0 = at;
        at = align_up(at + bytes, 256);
        return a0;
    };
    const uint64_t o_keys = take(n_pad * 8);
    const uint64_t o_acc = take((uint64_t)std::max<uint32_t>(po.n_acc, 1) * n_pad);
    const uint64_t o_p99 = take(n_cfg * 4), o_miss = take(n_cfg * 4), o_cost = take(n_cfg * 8);
    const uint64_t o_skip = take(n_cfg * 8), o_skip_cap = take(nb * 8), o_order = take(n_cfg * 4), o_base_local = take(n_cfg * 4);
    const uint64_t o_res_cap = take(nb * 8);  // results of the bases' launches (only the cost is written; unused)
    const uint64_t o_plan_cap = take(sizeof(EstPlan));
    const uint64_t o_status = take(2 * sizeof(EstStatus));  // work counters of the two kinds of launch
    uint64_t o_cstate[2], o_crings[2], o_crep[2], o_cslots[2], o_ctab[2];
    for (uint32_t i = 0; i < n_areas; ++i) {
        o_cstate[i] = take(nb * po.sz.state_words * 4);
        o_crings[i] = take(nb * cap_elems * 8);
        o_crep[i] = take(nb * po.sz.rep_words * 4);
        o_cslots[i] = take(nb * po.sz.slot_words * 4);
        o_ctab[i] = take(nb * cap_tab_bytes);
    }
    auto area = [&](uint64_t bytes_per_cfg) {
        uint64_t a0 = at;
        at = align_up(at + bytes_per_cfg * n_slots, 256);
        return a0;
    };
    const uint64_t o_state = area(po.sz.state_words * 4);
    const uint64_t o_rings = area(po.sz.ring_elems * 8);
    const uint64_t o_rep = area(po.sz.rep_words * 4);
    const uint64_t o_slots = area(po.sz.slot_words * 4);
    const uint64_t o_tab = area(po.sz.tab_bytes);
    const uint64_t o_lat = area(n * 4);
    if (h->ws_bytes < at) {
        if (h->ws) estbe::dfree(h->ws);
        h->ws = nullptr;
        h->ws_bytes = 0;
        h->ws = estbe::dmalloc(at);
        if (!h->ws) return fail(h, EST_ENOMEM, "cannot allocate %llu bytes of device scratch", (unsigned long long)at);
        h->ws_bytes = at;
    }
    uint8_t *ws = (uint8_t *)h->ws;
    EstStatus *st_cap = (EstStatus *)(ws + o_status), *st_rep = st_cap + 1;

    // ---- per-query tables, plans, masks
    const std::vector<uint64_t> skip_cap(nb, all_ops & ~needed);
    estbe::event_record(ev_p2, stream);
    if (estbe::h2d(h->d_plan, &po.plan, sizeof(EstPlan), stream) || estbe::h2d(ws + o_plan_cap, &PC, sizeof(EstPlan), stream) ||
        estbe::h2d(ws + o_skip, skip.data(), n_cfg * 8, stream) || estbe::h2d(ws + o_order, order.data(), n_cfg * 4, stream) ||
        estbe::h2d(ws + o_base_local, base_local.data(), n_cfg * 4, stream) || estbe::h2d(ws + o_skip_cap, skip_cap.data(), nb * 8, stream) ||
        estbe::zero(ws + o_status, 2 * sizeof(EstStatus), stream))
        return dev_fail(h, "upload plan");
    pa.trace_keys = (uint64_t *)(ws + o_keys);
    pa.acc = ws + o_acc;
    pa.acc_stride = n_pad;
    pa.n_acc = po.n_acc;
    memcpy(pa.acc_stage, po.acc_stage, sizeof(uint32_t) * po.n_acc);
    memcpy(pa.acc_slot_of_src, po.acc_slot_of_src, sizeof pa.acc_slot_of_src);
    if (estbe::launch_prep2(pa, stream)) return dev_fail(h, "trace tables");
    estbe::event_record(ev_p3, stream);

    EstSimArgs sa;
    memset(&sa, 0, sizeof sa);
    sa.dag = h->d_dag;
    sa.lat_us = h->d_lat;
    sa.cost_uusd_hr = h->d_cost;
    sa.arrival = d_arrival;
    sa.trace_keys = (const uint64_t *)(ws + o_keys);
    sa.acc = ws + o_acc;
    sa.acc_stride = n_pad;
    sa.n = (uint32_t)n;
    sa.slo_us = slo_us;
    sa.max_src = po.plan.max_src;
    sa.lds_bytes = po.lds_bytes;

    const bool capture = needed != 0;
    struct SideStream {  // the second stream, drained and destroyed on every path out
        void *s = nullptr;
        ~SideStream() {
            if (s) {
                estbe::sync(s);
                estbe::stream_destroy(s);
            }
        }
    } side;
    void *cap_stream = stream;
    if (capture && n_rounds > 1) {
        side.s = estbe::stream_create();
        if (!side.s) return dev_fail(h, "stream create");
        cap_stream = side.s;
        if (estbe::stream_wait_event(cap_stream, ev_p3)) return dev_fail(h, "stream wait");  // tables and plans are in place
    }
    std::vector<void *> cap_begin(n_rounds, nullptr), cap_done(n_rounds, nullptr), rep_done(n_rounds, nullptr);
    for (uint64_t k = 0; k < n_rounds; ++k) {
        cap_begin[k] = evs.make(); cap_done[k] = evs.make(); rep_done[k] = evs.make();
        if (!cap_begin[k] || !cap_done[k] || !rep_done[k]) return dev_fail(h, "event create");
    }
    // the bases of round k, candidate t in slot t of capture area k mod 2, streams left in place
    auto launch_bases = [&](uint64_t k) -> int {
        const uint64_t b0 = k * nb, nbk = std::min<uint64_t>(nb, n_bases - b0);
        const uint32_t ar = (uint32_t)(k % n_areas);
        EstSimArgs c2 = sa;
        c2.status = st_cap;
        c2.plan = (const EstPlan *)(ws + o_plan_cap);
        c2.cfg = (const EstStageCfg *)d_bases + b0 * S;
        c2.n_cfg = (uint32_t)nbk;
        c2.n_slots = (uint32_t)std::min<uint64_t>(nbk, resident);
        c2.have_lat = 0;
        c2.state = (uint32_t *)(ws + o_cstate[ar]);  c2.state_stride = po.sz.state_words;
        c2.rings = (uint64_t *)(ws + o_crings[ar]);  c2.ring_stride = cap_elems;
        c2.rep = (uint32_t *)(ws + o_crep[ar]);      c2.rep_stride = po.sz.rep_words;
        c2.slots = (uint32_t *)(ws + o_cslots[ar]);  c2.slot_stride = po.sz.slot_words;
        c2.tabs = ws + o_ctab[ar];               c2.tab_stride = cap_tab_bytes;
        c2.lat = nullptr;
        c2.p99 = (uint32_t *)(ws + o_res_cap); c2.miss = (uint32_t *)(ws + o_res_cap); c2.cost = (uint64_t *)(ws + o_res_cap);
        c2.skip_ops = (const uint64_t *)(ws + o_skip_cap);
        c2.slot_by_cfg = 1;
        if (nbk == 0 || nbk > nb || ar >= n_areas) return 1;  // a launch must stay inside the scratch laid out above
        if (k >= 2 && estbe::stream_wait_event(cap_stream, rep_done[k - 2])) return 1;  // the area's previous readers are done
        estbe::event_record(cap_begin[k], cap_stream);
        if (estbe::zero(&st_cap->next_cfg, 4, cap_stream) || estbe::launch_sim(c2, cap_stream)) return 1;
        estbe::event_record(cap_done[k], cap_stream);
        return 0;
    };
    auto launch_candidates = [&](uint64_t k) -> int {
        const uint64_t lo = round_lo[k], hi = round_lo[k + 1];
        const uint32_t ar = (uint32_t)(k % n_areas);
        if (capture && cap_stream != stream && estbe::stream_wait_event(stream, cap_done[k])) return 1;
        if (hi > lo) {
            EstSimArgs cb = sa;
            cb.status = st_rep;
            cb.plan = h->d_plan;
            cb.cfg = (const EstStageCfg *)d_cfg;
            cb.n_cfg = (uint32_t)(hi - lo);
            // the next round's bases become runnable when this launch starts: leave them their wavefront slots,
            // or they would wait for this launch's wavefronts to finish
            uint64_t mine = n_slots;
            if (capture && k + 1 < n_rounds) {
                const uint64_t next = std::min<uint64_t>(nb, n_bases - (k + 1) * nb);
                mine = std::max<uint64_t>(n_slots > next ? n_slots - next : 0, std::min<uint64_t>(n_slots, 64));  // never more than exist
            }
            cb.n_slots = (uint32_t)std::min<uint64_t>(mine, hi - lo);
            cb.have_lat = 1;
            cb.state = (uint32_t *)(ws + o_state);  cb.state_stride = po.sz.state_words;
            cb.rings = (uint64_t *)(ws + o_rings);  cb.ring_stride = po.sz.ring_elems;
            cb.rep = (uint32_t *)(ws + o_rep);      cb.rep_stride = po.sz.rep_words;
            cb.slots = (uint32_t *)(ws + o_slots);  cb.slot_stride = po.sz.slot_words;
            cb.tabs = ws + o_tab;               cb.tab_stride = po.sz.tab_bytes;
            cb.lat = (uint32_t *)(ws + o_lat);      cb.lat_stride = n;
            cb.p99 = (uint32_t *)(ws + o_p99); cb.miss = (uint32_t *)(ws + o_miss); cb.cost = (uint64_t *)(ws + o_cost);
            cb.skip_ops = (const uint64_t *)(ws + o_skip);
            cb.base_of = (const uint32_t *)(ws + o_base_local);
            cb.order = (const uint32_t *)(ws + o_order) + lo;
            cb.cap_plan = (const EstPlan *)(ws + o_plan_cap);
            if (capture) {
                cb.cap_rings = (const uint64_t *)(ws + o_crings[ar]);  cb.cap_ring_stride = cap_elems;
                cb.cap_state = (const uint32_t *)(ws + o_cstate[ar]);  cb.cap_state_stride = po.sz.state_words;
            }
            if (cb.n_slots > n_slots || cb.n_slots == 0) return 1;  // a launch must stay inside the scratch laid out above
            if (estbe::zero(&st_rep->next_cfg, 4, stream) || estbe::launch_sim(cb, stream)) return 1;
        }
        estbe::event_record(rep_done[k], stream);
        return 0;
    };
    estbe::event_record(e0, stream);
    if (capture && launch_bases(0)) return dev_fail(h, "simulation kernel (bases)");
    for (uint64_t k = 0; k < n_rounds; ++k) {
        if (capture && k + 1 < n_rounds && launch_bases(k + 1)) return dev_fail(h, "simulation kernel (bases)");
        if (launch_candidates(k)) return dev_fail(h, "simulation kernel");
    }
    estbe::event_record(e2, stream);
    EstStatus st2, st3;
    if (estbe::d2h(&st2, st_cap, sizeof st2, stream) || estbe::d2h(&st3, st_rep, sizeof st3, stream) || estbe::sync(stream))
        return dev_fail(h, "run");
    if (st2.sim_error || st3.sim_error) return fail(h, EST_EINTERNAL, "the simulation kernel stopped without finishing a candidate");
    if (estbe::d2d(d_p99, ws + o_p99, n_cfg * 4, stream) || estbe::d2d(d_miss, ws + o_miss, n_cfg * 4, stream) ||
        estbe::d2d(d_cost, ws + o_cost, n_cfg * 8, stream) || estbe::sync(stream))
        return dev_fail(h, "copy results");
    float capture_ms = 0.f;
    if (capture)
        for (uint64_t k = 0; k < n_rounds; ++k) capture_ms += estbe::event_ms(cap_begin[k], cap_done[k]);
    est_stats_t &ss = h->stats;
    memset(&ss, 0, sizeof ss);
    ss.n_launches = (uint32_t)((capture ? 2 : 1) * n_rounds);
    ss.waves_per_candidate = 1;
    ss.n_slots = (uint32_t)n_slots;
    ss.capture_ms = capture_ms;
    ss.sim_ms = estbe::event_ms(e0, e2);
    ss.prep_ms = estbe::event_ms(ev_p0, ev_p1) + estbe::event_ms(ev_p2, ev_p3);
    for (uint32_t s = 0; s < S; ++s) ss.stage_visits += st.n_visit[s];
    ss.workspace_bytes = at;
    // operations actually run, in units of one candidate's whole operation list (1.0 = nothing shared)
    {
        double ran = (double)n_bases * __builtin_popcountll(needed);
        for (uint64_t t = 0; t < n_cfg; ++t) ran += P.n_ops - __builtin_popcountll(skip[t]);
        ss.ops_run_fraction = (float)(ran / ((double)n_cfg * P.n_ops));
    }
    h->have_stats = true;
    return EST_OK;
}

int check_run_args(estimator *h, const est_trace_t *trace, const est_stage_cfg_t *configs, uint64_t n_cfg) {
    if (!h) return EST_EINVAL;
    h->err.clear();
    if (!trace) return fail(h, EST_EINVAL, "trace is NULL");
    if (trace->n > 0 && (!trace->arrival_us || !trace->visit_mask)) return fail(h, EST_EINVAL, "trace arrays are NULL");
    if (n_cfg > 0 && !configs) return fail(h, EST_EINVAL, "configs is NULL");
    return EST_OK;
}

}  // namespace

extern "C" {

int estimator_create(const est_dag_t *dag, const est_profiles_t *prof, estimator_t **out) {
    if (!out) return EST_EINVAL;
    *out = nullptr;
    if (!dag || !prof || !dag->parent_off || !prof->lat_us || !prof->cost_uusd_hr) return EST_EINVAL;
    const uint32_t S = dag->n_stages;
    if (S < 1 || S > EST_MAX_STAGES) return EST_EINVAL;
    if (prof->n_hw < 1 || prof->n_hw > 255 || prof->max_batch < 1 || prof->max_batch > EST_MAX_BATCH) return EST_EINVAL;
    if (dag->parent_off[0] != 0) return EST_EINVAL;
    for (uint32_t c = 0; c < S; ++c) {
        if (dag->parent_off[c + 1] < dag->parent_off[c] || dag->parent_off[c + 1] - dag->parent_off[c] > c) return EST_EINVAL;
        if (dag->parent_off[c + 1] > dag->parent_off[c] && !dag->parent_idx) return EST_EINVAL;
        for (uint32_t e = dag->parent_off[c]; e < dag->parent_off[c + 1]; ++e) {
            if (dag->parent_idx[e] >= c) return EST_EINVAL;
            for (uint32_t f = dag->parent_off[c]; f < e; ++f)
                if (dag->parent_idx[f] == dag->parent_idx[e]) return EST_EINVAL;
        }
    }
    const size_t nl = (size_t)S * prof->n_hw * prof->max_batch;
    for (size_t i = 0; i < nl; ++i)
        if (prof->lat_us[i] == 0) return EST_EINVAL;

    estimator *h = new (std::nothrow) estimator;
    if (!h) return EST_ENOMEM;
    try {
        h->lat.assign(prof->lat_us, prof->lat_us + nl);
        h->cost.assign(prof->cost_uusd_hr, prof->cost_uusd_hr + (size_t)S * prof->n_hw);
    } catch (...) {
        delete h;
        return EST_ENOMEM;
    }
    memset(&h->dag, 0, sizeof h->dag);
    memset(&h->stats, 0, sizeof h->stats);
    h->dag.S = S;
    h->dag.H = prof->n_hw;
    h->dag.Bmax = prof->max_batch;
    bool has_child[EST_MAX_STAGES] = {false};
    const uint32_t E = dag->parent_off[S];
    for (uint32_t c = 0; c <= S; ++c) h->dag.parent_off[c] = dag->parent_off[c];
    for (uint32_t e = 0; e < E; ++e) {
        h->dag.parent_idx[e] = dag->parent_idx[e];
        has_child[dag->parent_idx[e]] = true;
    }
    uint32_t e2 = E;  // the virtual sink's parents: every stage without children
    for (uint32_t s = 0; s < S; ++s)
        if (!has_child[s]) h->dag.parent_idx[e2++] = s;
    h->dag.parent_off[S + 1] = e2;
    for (uint32_t s = 0; s < S; ++s) {
        uint32_t m = 0;
        for (size_t i = 0; i < (size_t)prof->n_hw * prof->max_batch; ++i)
            m = std::max(m, h->lat[(size_t)s * prof->n_hw * prof->max_batch + i]);
        h->sum_max_lat += m;
    }
    if (estbe::init()) {
        delete h;
        return EST_EDEVICE;
    }
    h->d_dag = (EstDag *)estbe::dmalloc(sizeof(EstDag));
    h->d_lat = (uint32_t *)estbe::dmalloc(nl * 4);
    h->d_cost = (uint64_t *)estbe::dmalloc(h->cost.size() * 8);
    h->d_plan = (EstPlan *)estbe::dmalloc(sizeof(EstPlan));
    h->d_status = (EstStatus *)estbe::dmalloc(sizeof(EstStatus));
    h->pin = (estimator::Staging *)estbe::host_pinned_alloc(sizeof(estimator::Staging));
    bool have_ev = true;
    for (void *&e : h->ev) {
        e = estbe::event_create();
        have_ev = have_ev && e != nullptr;
    }
    if (!h->d_dag || !h->d_lat || !h->d_cost || !h->d_plan || !h->d_status || !h->pin || !have_ev) {
        estimator_destroy(h);
        return EST_ENOMEM;
    }
    (void)estbe::static_scratch(nullptr);  // resolve the fixed scratch's address on this device now (a run asks again for its own device)
    if (estbe::h2d(h->d_dag, &h->dag, sizeof(EstDag), nullptr) || estbe::h2d(h->d_lat, h->lat.data(), nl * 4, nullptr) ||
        estbe::h2d(h->d_cost, h->cost.data(), h->cost.size() * 8, nullptr) || estbe::sync(nullptr)) {
        estimator_destroy(h);
        return EST_EDEVICE;
    }
    *out = h;
    return EST_OK;
}

int estimator_run_dev(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *configs, uint64_t n_cfg,
                      uint32_t slo_us, est_result_t *out, void *workspace, uint64_t workspace_bytes, void *hip_stream) {
    int rc = check_run_args(h, trace, configs, n_cfg);
    if (rc != EST_OK) return rc;
    if (n_cfg > 0 && (!out || !out->p99_us || !out->miss_count || !out->cost_uusd_hr)) return fail(h, EST_EINVAL, "result arrays are NULL");
    try {
        return run_core(h, trace->n, trace->arrival_us, trace->visit_mask, configs, n_cfg, slo_us, MODE_P99, out ? out->p99_us : nullptr,
                        out ? out->miss_count : nullptr, out ? out->cost_uusd_hr : nullptr, nullptr, workspace, workspace_bytes, hip_stream);
    } catch (const std::bad_alloc &) {
        return fail(h, EST_ENOMEM, "host allocation failed");
    } catch (...) {
        return fail(h, EST_EINTERNAL, "unexpected exception");
    }
}

int estimator_run_static_dev(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *configs, uint64_t n_cfg,
                             uint32_t slo_us, est_result_t *out, void *hip_stream) {
    int rc = check_run_args(h, trace, configs, n_cfg);
    if (rc != EST_OK) return rc;
    if (n_cfg > 0 && (!out || !out->p99_us || !out->miss_count || !out->cost_uusd_hr)) return fail(h, EST_EINVAL, "result arrays are NULL");
    uint64_t bytes = 0;
    void *scratch = estbe::static_scratch(&bytes);  // this device's copy of the fixed array (resolved on first use, no allocation)
    if (!scratch) return dev_fail(h, "fixed scratch");
    try {
        return run_core(h, trace->n, trace->arrival_us, trace->visit_mask, configs, n_cfg, slo_us, MODE_P99, out ? out->p99_us : nullptr,
                        out ? out->miss_count : nullptr, out ? out->cost_uusd_hr : nullptr, nullptr, scratch, bytes, hip_stream, true);
    } catch (const std::bad_alloc &) {
        return fail(h, EST_ENOMEM, "host allocation failed");
    } catch (...) {
        return fail(h, EST_EINTERNAL, "unexpected exception");
    }
}

int estimator_run_shared_dev(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *bases, uint64_t n_bases,
                             const est_stage_cfg_t *configs, const uint32_t *base_of, uint64_t n_cfg, uint32_t slo_us,
                             est_result_t *out, void *hip_stream) {
    int rc = check_run_args(h, trace, configs, n_cfg);
    if (rc != EST_OK) return rc;
    if (n_cfg > 0 && (!out || !out->p99_us || !out->miss_count || !out->cost_uusd_hr)) return fail(h, EST_EINVAL, "result arrays are NULL");
    if (n_cfg > 0 && n_bases > 0 && (!bases || !base_of)) return fail(h, EST_EINVAL, "bases or base_of is NULL");
    try {
        return run_shared_core(h, trace->n, trace->arrival_us, trace->visit_mask, bases, n_bases, configs, base_of, n_cfg, slo_us,
                               out ? out->p99_us : nullptr, out ? out->miss_count : nullptr, out ? out->cost_uusd_hr : nullptr, hip_stream);
    } catch (const std::bad_alloc &) {
        return fail(h, EST_ENOMEM, "host allocation failed");
    } catch (...) {
        return fail(h, EST_EINTERNAL, "unexpected exception");
    }
}

int estimator_run_latencies_dev(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *configs, uint64_t n_cfg,
                                uint32_t *lat_us_out, void *workspace, uint64_t workspace_bytes, void *hip_stream) {
    int rc = check_run_args(h, trace, configs, n_cfg);
    if (rc != EST_OK) return rc;
    if (n_cfg > 0 && trace->n > 0 && !lat_us_out) return fail(h, EST_EINVAL, "lat_us_out is NULL");
    try {
        return run_core(h, trace->n, trace->arrival_us, trace->visit_mask, configs, n_cfg, 0, MODE_LAT, nullptr, nullptr, nullptr,
                        lat_us_out, workspace, workspace_bytes, hip_stream);
    } catch (const std::bad_alloc &) {
        return fail(h, EST_ENOMEM, "host allocation failed");
    } catch (...) {
        return fail(h, EST_EINTERNAL, "unexpected exception");
    }
}

static int run_host(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *configs, uint64_t n_cfg, uint32_t slo_us,
                    est_result_t *out, uint32_t *lat_out) {
    const uint64_t n = trace->n;
    const uint32_t S = h->dag.S;
    if (n >= (1ull << 31) || n_cfg >= (1ull << 31)) return fail(h, EST_EINVAL, "trace or configuration set too large");
    if (n_cfg == 0) return EST_OK;
    // validate on the host first, so that a bad input never reaches the GPU
    for (uint64_t q = 1; q < n; ++q)
        if (trace->arrival_us[q] < trace->arrival_us[q - 1]) return fail(h, EST_EINVAL, "arrival times decrease at query %llu", (unsigned long long)q);
    for (uint64_t i = 0; i < n_cfg * S; ++i) {
        const est_stage_cfg_t &e = configs[i];
        if (e.hw >= h->dag.H || e.batch < 1 || e.batch > h->dag.Bmax || e.replicas < 1 || e.replicas > EST_MAX_REPLICAS)
            return fail(h, EST_EINVAL, "configuration %llu stage %llu out of range", (unsigned long long)(i / S), (unsigned long long)(i % S));
    }
    DevBuf d_arr, d_mask, d_cfg, d_p99, d_miss, d_cost, d_lat;
    if (!d_arr.alloc(n * 4) || !d_mask.alloc(n * 4) || !d_cfg.alloc(n_cfg * S * sizeof(est_stage_cfg_t)))
        return fail(h, EST_ENOMEM, "device allocation of the inputs failed");
    if (estbe::h2d(d_arr.p, trace->arrival_us, n * 4, nullptr) || estbe::h2d(d_mask.p, trace->visit_mask, n * 4, nullptr) ||
        estbe::h2d(d_cfg.p, configs, n_cfg * S * sizeof(est_stage_cfg_t), nullptr))
        return dev_fail(h, "upload inputs");
    int rc;
    if (lat_out) {
        if (!d_lat.alloc(n_cfg * n * 4)) return fail(h, EST_ENOMEM, "device allocation of the latency matrix failed");
        rc = run_core(h, n, (const uint32_t *)d_arr.p, (const uint32_t *)d_mask.p, (const est_stage_cfg_t *)d_cfg.p, n_cfg, 0, MODE_LAT,
                      nullptr, nullptr, nullptr, (uint32_t *)d_lat.p, nullptr, 0, nullptr);
        if (rc != EST_OK) return rc;
        if (n > 0 && (estbe::d2h(lat_out, d_lat.p, n_cfg * n * 4, nullptr) || estbe::sync(nullptr))) return dev_fail(h, "download latencies");
        return EST_OK;
    }
    if (!d_p99.alloc(n_cfg * 4) || !d_miss.alloc(n_cfg * 4) || !d_cost.alloc(n_cfg * 8)) return fail(h, EST_ENOMEM, "device allocation of the results failed");
    rc = run_core(h, n, (const uint32_t *)d_arr.p, (const uint32_t *)d_mask.p, (const est_stage_cfg_t *)d_cfg.p, n_cfg, slo_us, MODE_P99,
                  (uint32_t *)d_p99.p, (uint32_t *)d_miss.p, (uint64_t *)d_cost.p, nullptr, nullptr, 0, nullptr);
    if (rc != EST_OK) return rc;
    std::vector<uint32_t> p99(n_cfg), miss(n_cfg);
    std::vector<uint64_t> cost(n_cfg);
    if (estbe::d2h(p99.data(), d_p99.p, n_cfg * 4, nullptr) || estbe::d2h(miss.data(), d_miss.p, n_cfg * 4, nullptr) ||
        estbe::d2h(cost.data(), d_cost.p, n_cfg * 8, nullptr) || estbe::sync(nullptr))
        return dev_fail(h, "download results");
    memcpy(out->p99_us, p99.data(), n_cfg * 4);
    memcpy(out->miss_count, miss.data(), n_cfg * 4);
    memcpy(out->cost_uusd_hr, cost.data(), n_cfg * 8);
    return EST_OK;
}

int estimator_run(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *configs, uint64_t n_cfg, uint32_t slo_us,
                  est_result_t *out) {
    int rc = check_run_args(h, trace, configs, n_cfg);
    if (rc != EST_OK) return rc;
    if (n_cfg > 0 && (!out || !out->p99_us || !out->miss_count || !out->cost_uusd_hr)) return fail(h, EST_EINVAL, "result arrays are NULL");
    try {
        return run_host(h, trace, configs, n_cfg, slo_us, out, nullptr);
    } catch (const std::bad_alloc &) {
        return fail(h, EST_ENOMEM, "host allocation failed");
    } catch (...) {
        return fail(h, EST_EINTERNAL, "unexpected exception");
    }
}

int estimator_run_latencies(estimator_t *h, const est_trace_t *trace, const est_stage_cfg_t *configs, uint64_t n_cfg,
                            uint32_t *lat_us_out) {
    int rc = check_run_args(h, trace, configs, n_cfg);
    if (rc != EST_OK) return rc;
    if (n_cfg > 0 && trace->n > 0 && !lat_us_out) return fail(h, EST_EINVAL, "lat_us_out is NULL");
    static uint32_t dummy;
    try {
        return run_host(h, trace, configs, n_cfg, 0, nullptr, lat_us_out ? lat_us_out : &dummy);
    } catch (const std::bad_alloc &) {
        return fail(h, EST_ENOMEM, "host allocation failed");
    } catch (...) {
        return fail(h, EST_EINTERNAL, "unexpected exception");
    }
}

uint64_t estimator_workspace_bytes(const estimator_t *h, uint64_t n, uint64_t n_cfg) {
    if (!h) return 0;
    const uint32_t S = h->dag.S;
    const uint64_t n_pad = align_up(std::max<uint64_t>(n, 1), 256);
    // every stage forking: an unbounded out ring, a bounded in ring, full slots
    const uint64_t cap_b = pow2ceil(EST_MAX_REPLICAS * EST_MAX_BATCH + 64 * EST_KMAX + 65);
    uint64_t per_cfg = (4ull * EST_MAX_RINGS + EST_MAX_EDGES + EST_MAX_OPS) * 4;
    per_cfg += (uint64_t)S * (std::max(cap_b, pow2ceil(std::max<uint64_t>(n, 1))) + cap_b) * 8;
    per_cfg += (uint64_t)S * (2 * EST_MAX_REPLICAS + EST_MAX_REPLICAS * EST_MAX_BATCH) * 4;
    // time tables of joins: a stage (or the sink) can be fed by several streams at once when it has several
    // parents, or a parent that has (a query that skips that parent takes its ready time from further up);
    // one table per stream, at most EST_KMAX and at most one per ancestor plus the arrivals
    {
        bool joins[EST_MAX_STAGES + 1];
        for (uint32_t c = 0; c <= S; ++c) {
            const uint32_t b = h->dag.parent_off[c], e = h->dag.parent_off[c + 1];
            joins[c] = e - b >= 2;
            for (uint32_t i = b; i < e; ++i) joins[c] = joins[c] || joins[h->dag.parent_idx[i]];
            if (joins[c]) per_cfg += (uint64_t)std::min<uint32_t>(EST_KMAX, c + 1) * align_up(n, 64) * 4;
        }
    }
    per_cfg += n * 4 + 64;
    uint64_t fixed = n_pad * 8 + (uint64_t)(S + 1) * n_pad + n_cfg * 16 + 16 * 256;
    return fixed + per_cfg * std::max<uint64_t>(n_cfg, 1);
}

int estimator_last_stats(const estimator_t *h, est_stats_t *out) {
    if (!h || !out) return EST_EINVAL;
    if (!h->have_stats) return EST_EINVAL;
    *out = h->stats;
    return EST_OK;
}

const char *estimator_last_error(const estimator_t *h) { return h ? h->err.c_str() : "invalid handle"; }

void estimator_destroy(estimator_t *h) {
    if (!h) return;
    if (h->d_dag) estbe::dfree(h->d_dag);
    if (h->d_lat) estbe::dfree(h->d_lat);
    if (h->d_cost) estbe::dfree(h->d_cost);
    if (h->d_plan) estbe::dfree(h->d_plan);
    if (h->d_status) estbe::dfree(h->d_status);
    if (h->ws) estbe::dfree(h->ws);
    if (h->pin) estbe::host_pinned_free(h->pin);
    for (void *e : h->ev)
        if (e) estbe::event_destroy(e);
    delete h;
}

}  // extern "C"
