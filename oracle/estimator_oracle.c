/*
 * CPU oracle for the InferLine Estimator (arXiv 1812.01776, Section 4.2).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU
 * library is checked against.  It shares no code with the GPU path and must never be
 * called from it; only tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * What it computes: the paper's Estimator is a continuous-time discrete-event simulator
 * with one global logical clock that is advanced from event to event, events being
 * processed in temporal order (Section 4.2).  It replays a query arrival trace through a
 * pipeline DAG (Section 2) whose stages are fed by a centralized batched queue that hands
 * batches of at most the configured maximum batch size to the stage's replicas
 * (Section 3, serving-system requirements; Section 2.1 on maximum batch size: a whole
 * batch returns together).  The time a batch takes is read from the model profile for
 * the stage's hardware type and the batch's actual size (Section 4.2, last paragraph).
 * Conditional control flow is modelled with a per-query visit mask drawn from the scale
 * factors of Section 4.1.  Outputs: the latency of every query (Section 4.2), from which
 * the P99 (Section 2: 99% of query latencies must be below the constraint), the number of
 * SLO misses and the cost of the configuration (Section 6, cost model) follow.
 *
 * Readings of points the paper leaves open (the same list is in the design notes):
 *   - no batching timeout: an idle replica takes whatever is queued (>= 1 query) at once;
 *   - all deliveries at a timestamp happen before any dispatch at that timestamp;
 *   - queue order is (time the query became ready at the stage, query id);
 *   - replicas are identical, so only the number of idle ones is tracked;
 *   - a partial batch costs the profile entry of its actual size;
 *   - a query that does not visit a stage passes through it in zero time;
 *   - a stage with several parents becomes ready at the max of the parents' completions;
 *   - end-to-end completion is the max over sink stages;
 *   - P99 is the nearest-rank order statistic k = ceil(0.99 N);
 *   - a miss is latency > slo;
 *   - every computed time saturates at a horizon (2^32-1 us in production use).
 *
 * Parity pins (tests/test_oracle_*.py): three hand-traced examples, the Lindley recursion,
 * the burst closed form, the no-contention service time, the M/D/1 mean wait, a 1-us tick
 * simulator on tiny inputs, a per-stage sorted-scan formulation and structural invariants.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)
#define ORACLE_ENOMEM (-2)

/* ------------------------------------------------------------------ event heap */

enum { EV_ARRIVAL = 0, EV_BATCH_DONE = 1 };

typedef struct {
    uint64_t time;
    uint32_t kind;  /* EV_ARRIVAL or EV_BATCH_DONE */
    uint32_t stage; /* EV_BATCH_DONE: the stage */
    uint64_t id;    /* EV_ARRIVAL: query id; EV_BATCH_DONE: batch index */
} event_t;

typedef struct {
    event_t *a;
    size_t n, cap;
} evheap_t;

static int ev_less(const event_t *x, const event_t *y)
{
    if (x->time != y->time) return x->time < y->time;
    if (x->kind != y->kind) return x->kind < y->kind;
    if (x->stage != y->stage) return x->stage < y->stage;
    return x->id < y->id;
}

static int evheap_push(evheap_t *h, event_t e)
{
    if (h->n == h->cap) {
        size_t nc = h->cap ? h->cap * 2 : 1024;
        event_t *na = (event_t *)realloc(h->a, nc * sizeof(event_t));
        if (!na) return ORACLE_ENOMEM;
        h->a = na;
        h->cap = nc;
    }
    size_t i = h->n++;
    h->a[i] = e;
    while (i > 0) {
        size_t p = (i - 1) / 2;
        if (!ev_less(&h->a[i], &h->a[p])) break;
        event_t t = h->a[i]; h->a[i] = h->a[p]; h->a[p] = t;
        i = p;
    }
    return ORACLE_OK;
}

static event_t evheap_pop(evheap_t *h)
{
    event_t top = h->a[0];
    h->a[0] = h->a[--h->n];
    size_t i = 0;
    for (;;) {
        size_t l = 2 * i + 1, r = l + 1, m = i;
        if (l < h->n && ev_less(&h->a[l], &h->a[m])) m = l;
        if (r < h->n && ev_less(&h->a[r], &h->a[m])) m = r;
        if (m == i) break;
        event_t t = h->a[i]; h->a[i] = h->a[m]; h->a[m] = t;
        i = m;
    }
    return top;
}

/* ------------------------------------------------------------------ per-stage queue:
 * a min-heap of (ready_time, query id) pairs, i.e. FIFO by time of arrival at the stage,
 * ties by query id. */

typedef struct {
    uint64_t ready;
    uint64_t qid;
} qent_t;

typedef struct {
    qent_t *a;
    size_t n, cap;
} qheap_t;

static int q_less(const qent_t *x, const qent_t *y)
{
    if (x->ready != y->ready) return x->ready < y->ready;
    return x->qid < y->qid;
}

static int qheap_push(qheap_t *h, qent_t e)
{
    if (h->n == h->cap) {
        size_t nc = h->cap ? h->cap * 2 : 256;
        qent_t *na = (qent_t *)realloc(h->a, nc * sizeof(qent_t));
        if (!na) return ORACLE_ENOMEM;
        h->a = na;
        h->cap = nc;
    }
    size_t i = h->n++;
    h->a[i] = e;
    while (i > 0) {
        size_t p = (i - 1) / 2;
        if (!q_less(&h->a[i], &h->a[p])) break;
        qent_t t = h->a[i]; h->a[i] = h->a[p]; h->a[p] = t;
        i = p;
    }
    return ORACLE_OK;
}

static qent_t qheap_pop(qheap_t *h)
{
    qent_t top = h->a[0];
    h->a[0] = h->a[--h->n];
    size_t i = 0;
    for (;;) {
        size_t l = 2 * i + 1, r = l + 1, m = i;
        if (l < h->n && q_less(&h->a[l], &h->a[m])) m = l;
        if (r < h->n && q_less(&h->a[r], &h->a[m])) m = r;
        if (m == i) break;
        qent_t t = h->a[i]; h->a[i] = h->a[m]; h->a[m] = t;
        i = m;
    }
    return top;
}

/* ------------------------------------------------------------------ simulator state */

typedef struct {
    uint32_t stage;
    uint64_t start_time, end_time;
    uint64_t first; /* index of the first member in sim->members */
    uint32_t count;
} batch_t;

typedef struct {
    /* inputs */
    uint32_t S;
    const uint32_t *parent_off, *parent_idx;
    uint32_t H, Bmax;
    const uint32_t *lat_us; /* [S][H][Bmax] */
    uint64_t n;
    const uint32_t *arrival, *mask;
    const uint8_t *hw, *batch;
    const uint16_t *replicas;
    uint64_t horizon;
    /* derived DAG */
    uint32_t *child_off, *child_idx;
    uint32_t *n_parents;
    /* dynamic */
    evheap_t ev;
    qheap_t *queue;     /* [S] */
    uint32_t *idle;     /* [S] idle replicas */
    uint8_t *reported;  /* [S][n] parents that have reported */
    uint64_t *ready;    /* [S][n] max over reported parents; final = ready time */
    uint64_t *done;     /* [S][n] completion time at the stage */
    batch_t *batches;
    size_t n_batches, cap_batches;
    uint64_t *members;
    size_t n_members, cap_members;
    int err;
} sim_t;

static void deliver(sim_t *s, uint64_t q, uint32_t c, uint64_t time);

/* query q has completed stage c at `time`: record it and tell every child. */
static void complete(sim_t *s, uint64_t q, uint32_t c, uint64_t time)
{
    s->done[(size_t)c * s->n + q] = time;
    for (uint32_t e = s->child_off[c]; e < s->child_off[c + 1]; ++e)
        deliver(s, q, s->child_idx[e], time);
}

/* one parent of stage c (or the source, for a root) reports query q at `time`. */
static void deliver(sim_t *s, uint64_t q, uint32_t c, uint64_t time)
{
    size_t at = (size_t)c * s->n + q;
    if (time > s->ready[at]) s->ready[at] = time;
    s->reported[at]++;
    uint32_t need = s->n_parents[c] ? s->n_parents[c] : 1; /* a root hears once, from the source */
    if (s->reported[at] < need) return;
    uint64_t ready = s->ready[at]; /* join: max over the parents' completions */
    if (!((s->mask[q] >> c) & 1u)) {
        /* conditional control flow: the query skips this stage in zero time */
        complete(s, q, c, ready);
    } else {
        qent_t e = { ready, q };
        if (qheap_push(&s->queue[c], e) != ORACLE_OK) s->err = ORACLE_ENOMEM;
    }
}

static int dispatch(sim_t *s, uint32_t c, uint64_t T)
{
    /* centralized queue: while a replica is idle and queries wait, hand it a batch */
    while (s->idle[c] > 0 && s->queue[c].n > 0) {
        uint32_t B = s->batch[c];
        uint32_t b = (s->queue[c].n < B) ? (uint32_t)s->queue[c].n : B;
        if (s->n_batches == s->cap_batches) {
            size_t nc = s->cap_batches ? s->cap_batches * 2 : 1024;
            batch_t *nb = (batch_t *)realloc(s->batches, nc * sizeof(batch_t));
            if (!nb) return ORACLE_ENOMEM;
            s->batches = nb;
            s->cap_batches = nc;
        }
        if (s->n_members + b > s->cap_members) {
            size_t nc = s->cap_members ? s->cap_members * 2 : 4096;
            while (nc < s->n_members + b) nc *= 2;
            uint64_t *nm = (uint64_t *)realloc(s->members, nc * sizeof(uint64_t));
            if (!nm) return ORACLE_ENOMEM;
            s->members = nm;
            s->cap_members = nc;
        }
        batch_t *bt = &s->batches[s->n_batches];
        bt->stage = c;
        bt->start_time = T;
        bt->first = s->n_members;
        bt->count = b;
        for (uint32_t i = 0; i < b; ++i) s->members[s->n_members++] = qheap_pop(&s->queue[c]).qid;
        uint64_t L = s->lat_us[((size_t)c * s->H + s->hw[c]) * s->Bmax + (b - 1)];
        uint64_t end = T + L;
        if (end > s->horizon) end = s->horizon; /* saturating clock */
        bt->end_time = end;
        s->idle[c]--;
        event_t e = { end, EV_BATCH_DONE, c, (uint64_t)s->n_batches };
        s->n_batches++;
        int rc = evheap_push(&s->ev, e);
        if (rc != ORACLE_OK) return rc;
    }
    return ORACLE_OK;
}

static void sim_free(sim_t *s)
{
    free(s->child_off); free(s->child_idx); free(s->n_parents);
    free(s->ev.a);
    if (s->queue) for (uint32_t c = 0; c < s->S; ++c) free(s->queue[c].a);
    free(s->queue); free(s->idle); free(s->reported); free(s->ready); free(s->done);
    free(s->batches); free(s->members);
}

static int validate(uint32_t S, const uint32_t *parent_off, const uint32_t *parent_idx, uint32_t H,
                    uint32_t Bmax, const uint32_t *lat_us, uint64_t n, const uint32_t *arrival,
                    const uint32_t *mask)
{
    if (S < 1 || S > 32 || !parent_off || H < 1 || Bmax < 1 || Bmax > 64 || !lat_us) return ORACLE_EINVAL;
    if (parent_off[0] != 0) return ORACLE_EINVAL;
    for (uint32_t c = 0; c < S; ++c) {
        if (parent_off[c + 1] < parent_off[c]) return ORACLE_EINVAL;
        for (uint32_t e = parent_off[c]; e < parent_off[c + 1]; ++e) {
            if (!parent_idx || parent_idx[e] >= c) return ORACLE_EINVAL;
            for (uint32_t f = parent_off[c]; f < e; ++f)
                if (parent_idx[f] == parent_idx[e]) return ORACLE_EINVAL;
        }
    }
    for (size_t i = 0; i < (size_t)S * H * Bmax; ++i)
        if (lat_us[i] == 0) return ORACLE_EINVAL;
    if (n > 0 && (!arrival || !mask)) return ORACLE_EINVAL;
    for (uint64_t q = 1; q < n; ++q)
        if (arrival[q] < arrival[q - 1]) return ORACLE_EINVAL;
    return ORACLE_OK;
}

/*
 * Simulate one configuration.
 *   parent_off[S+1], parent_idx[]  CSR list of each stage's parents; parents precede children.
 *   lat_us[S][H][Bmax]             profile: entry b-1 is the latency of a batch of b queries, in us.
 *   arrival[n]                     non-decreasing arrival times, us.
 *   mask[n]                        bit s set = the query visits stage s.
 *   hw[S], batch[S], replicas[S]   the configuration.
 *   horizon                        every computed time is min(true time, horizon).
 *   latency_out[n]                 required.  end-to-end latency of each query, us.
 *   ready_out[S*n], done_out[S*n]  optional; per stage, when each query became ready / finished.
 *   batch_log[4*batch_cap]         optional; (stage, start, end, size) of every dispatched batch in
 *                                  dispatch order; *n_batches_out gets the total number dispatched.
 */
int oracle_simulate(uint32_t S, const uint32_t *parent_off, const uint32_t *parent_idx, uint32_t H,
                    uint32_t Bmax, const uint32_t *lat_us, uint64_t n, const uint32_t *arrival,
                    const uint32_t *mask, const uint8_t *hw, const uint8_t *batch,
                    const uint16_t *replicas, uint64_t horizon, uint64_t *latency_out,
                    uint64_t *ready_out, uint64_t *done_out, uint64_t *batch_log, uint64_t batch_cap,
                    uint64_t *n_batches_out)
{
    int rc = validate(S, parent_off, parent_idx, H, Bmax, lat_us, n, arrival, mask);
    if (rc != ORACLE_OK) return rc;
    if (!hw || !batch || !replicas || (n > 0 && !latency_out)) return ORACLE_EINVAL;
    for (uint32_t c = 0; c < S; ++c)
        if (hw[c] >= H || batch[c] < 1 || batch[c] > Bmax || replicas[c] < 1) return ORACLE_EINVAL;
    if (n_batches_out) *n_batches_out = 0;
    if (n == 0) return ORACLE_OK;

    sim_t s;
    memset(&s, 0, sizeof s);
    s.S = S; s.parent_off = parent_off; s.parent_idx = parent_idx; s.H = H; s.Bmax = Bmax;
    s.lat_us = lat_us; s.n = n; s.arrival = arrival; s.mask = mask;
    s.hw = hw; s.batch = batch; s.replicas = replicas; s.horizon = horizon;

    uint32_t E = parent_off[S];
    s.child_off = (uint32_t *)calloc(S + 1, sizeof(uint32_t));
    s.child_idx = (uint32_t *)calloc(E ? E : 1, sizeof(uint32_t));
    s.n_parents = (uint32_t *)calloc(S, sizeof(uint32_t));
    s.queue = (qheap_t *)calloc(S, sizeof(qheap_t));
    s.idle = (uint32_t *)calloc(S, sizeof(uint32_t));
    s.reported = (uint8_t *)calloc((size_t)S * n, 1);
    s.ready = (uint64_t *)calloc((size_t)S * n, sizeof(uint64_t));
    s.done = (uint64_t *)calloc((size_t)S * n, sizeof(uint64_t));
    if (!s.child_off || !s.child_idx || !s.n_parents || !s.queue || !s.idle || !s.reported ||
        !s.ready || !s.done) {
        sim_free(&s);
        return ORACLE_ENOMEM;
    }
    /* children lists from parent lists */
    for (uint32_t c = 0; c < S; ++c) {
        s.n_parents[c] = parent_off[c + 1] - parent_off[c];
        for (uint32_t e = parent_off[c]; e < parent_off[c + 1]; ++e) s.child_off[parent_idx[e] + 1]++;
    }
    for (uint32_t c = 0; c < S; ++c) s.child_off[c + 1] += s.child_off[c];
    {
        uint32_t *fill = (uint32_t *)calloc(S, sizeof(uint32_t));
        if (!fill) { sim_free(&s); return ORACLE_ENOMEM; }
        for (uint32_t c = 0; c < S; ++c)
            for (uint32_t e = parent_off[c]; e < parent_off[c + 1]; ++e) {
                uint32_t p = parent_idx[e];
                s.child_idx[s.child_off[p] + fill[p]++] = c;
            }
        free(fill);
    }
    for (uint32_t c = 0; c < S; ++c) s.idle[c] = replicas[c]; /* all replicas idle at t=0 */

    /* every query arrives at the source at its trace time */
    for (uint64_t q = 0; q < n && rc == ORACLE_OK; ++q) {
        event_t e = { arrival[q], EV_ARRIVAL, 0, q };
        rc = evheap_push(&s.ev, e);
    }

    while (rc == ORACLE_OK && s.ev.n > 0) {
        uint64_t T = s.ev.a[0].time; /* advance the global clock to the next event time */
        while (s.ev.n > 0 && s.ev.a[0].time == T) {
            event_t e = evheap_pop(&s.ev);
            if (e.kind == EV_ARRIVAL) {
                for (uint32_t c = 0; c < S; ++c)
                    if (s.n_parents[c] == 0) deliver(&s, e.id, c, T);
            } else {
                batch_t bt = s.batches[e.id];
                s.idle[bt.stage]++;
                /* the whole batch returns together */
                for (uint32_t i = 0; i < bt.count; ++i) complete(&s, s.members[bt.first + i], bt.stage, T);
            }
        }
        if (s.err) { rc = s.err; break; }
        /* only now, with every delivery at T made, form batches */
        for (uint32_t c = 0; c < S && rc == ORACLE_OK; ++c) rc = dispatch(&s, c, T);
    }

    if (rc == ORACLE_OK) {
        for (uint64_t q = 0; q < n; ++q) {
            uint64_t fin = 0;
            for (uint32_t c = 0; c < S; ++c)
                if (s.child_off[c + 1] == s.child_off[c]) { /* sink */
                    uint64_t d = s.done[(size_t)c * n + q];
                    if (d > fin) fin = d;
                }
            latency_out[q] = fin - arrival[q];
        }
        if (ready_out) memcpy(ready_out, s.ready, (size_t)S * n * sizeof(uint64_t));
        if (done_out) memcpy(done_out, s.done, (size_t)S * n * sizeof(uint64_t));
        if (n_batches_out) *n_batches_out = s.n_batches;
        if (batch_log)
            for (size_t i = 0; i < s.n_batches && i < batch_cap; ++i) {
                batch_log[4 * i + 0] = s.batches[i].stage;
                batch_log[4 * i + 1] = s.batches[i].start_time;
                batch_log[4 * i + 2] = s.batches[i].end_time;
                batch_log[4 * i + 3] = s.batches[i].count;
            }
    }
    sim_free(&s);
    return rc;
}

static int cmp_u64(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return (x > y) - (x < y);
}

/* nearest-rank P99: the k-th smallest with k = ceil(99 n / 100); 0 for an empty trace. */
uint64_t oracle_p99(const uint64_t *latency, uint64_t n)
{
    if (n == 0) return 0;
    uint64_t *tmp = (uint64_t *)malloc(n * sizeof(uint64_t));
    if (!tmp) return UINT64_MAX;
    memcpy(tmp, latency, n * sizeof(uint64_t));
    qsort(tmp, n, sizeof(uint64_t), cmp_u64);
    uint64_t k = (99 * n + 99) / 100;
    uint64_t v = tmp[k - 1];
    free(tmp);
    return v;
}

/*
 * Simulate n_cfg configurations one after the other (single thread).
 *   configs hw/batch/replicas are [n_cfg][S].
 *   cost_uusd_hr[S][H]: micro-dollars per replica-hour.
 *   outputs p99_us[n_cfg], miss_count[n_cfg] (latency > slo), cost_out[n_cfg]
 *   lat_all (optional): [n_cfg][n] every per-query latency.
 */
int oracle_run(uint32_t S, const uint32_t *parent_off, const uint32_t *parent_idx, uint32_t H,
               uint32_t Bmax, const uint32_t *lat_us, const uint64_t *cost_uusd_hr, uint64_t n,
               const uint32_t *arrival, const uint32_t *mask, uint64_t n_cfg, const uint8_t *hw,
               const uint8_t *batch, const uint16_t *replicas, uint64_t slo_us, uint64_t horizon,
               uint64_t *p99_us, uint64_t *miss_count, uint64_t *cost_out, uint64_t *lat_all)
{
    if (n_cfg == 0) return ORACLE_OK;
    if (!p99_us || !miss_count || !cost_out || !cost_uusd_hr) return ORACLE_EINVAL;
    uint64_t *lat = (uint64_t *)malloc((n ? n : 1) * sizeof(uint64_t));
    if (!lat) return ORACLE_ENOMEM;
    int rc = ORACLE_OK;
    for (uint64_t c = 0; c < n_cfg && rc == ORACLE_OK; ++c) {
        const uint8_t *chw = hw + c * S, *cb = batch + c * S;
        const uint16_t *cr = replicas + c * S;
        rc = oracle_simulate(S, parent_off, parent_idx, H, Bmax, lat_us, n, arrival, mask, chw, cb, cr,
                             horizon, lat, NULL, NULL, NULL, 0, NULL);
        if (rc != ORACLE_OK) break;
        uint64_t miss = 0;
        for (uint64_t q = 0; q < n; ++q) miss += lat[q] > slo_us;
        uint64_t cost = 0;
        for (uint32_t s = 0; s < S; ++s) cost += (uint64_t)cr[s] * cost_uusd_hr[(size_t)s * H + chw[s]];
        p99_us[c] = oracle_p99(lat, n);
        miss_count[c] = miss;
        cost_out[c] = cost;
        if (lat_all) memcpy(lat_all + c * n, lat, n * sizeof(uint64_t));
    }
    free(lat);
    return rc;
}
