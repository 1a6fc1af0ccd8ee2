// Device code of the batched Estimator: one 64-lane wavefront simulates one candidate
// configuration end to end.  Written against the wv:: primitives only, so that the same text
// also compiles for a lock-step CPU emulation used by the host-side checks of the kernel logic.
//
// The simulated system is the centralized batched queue of arXiv 1812.01776 (Section 3, serving
// system requirements; Section 2.1, maximum batch size; Section 4.2, event order).  Because
// queues are unbounded and the DAG is feed-forward, a stage depends only on its own input
// stream ordered by (ready time, query index); the global event order of Section 4.2 is
// reproduced by running every stage over its ordered stream:
//
//   SCAN   one stage.  Walk the stage's input stream; a batch starts at T = max(earliest replica
//          free time, ready time of the first waiting query), takes every waiting query with
//          ready <= T up to the maximum batch size, and completes at T + L(actual size)
//          (Section 4.2: latency from the profile for a batch of the given size; Section 2.1: the
//          whole batch returns together).  Completed batches are emitted to the output stream in
//          (completion time, query index) order.
//   MERGE  builds a stage's input stream from the output streams of the query's nearest visited
//          ancestors: a query that skips a stage passes through it in zero time (Section 4.1,
//          scale factor / conditional control flow) and a stage with several parents is ready at
//          the maximum of their completions.
//   LAT    a MERGE into the virtual sink: latency = completion - arrival (Section 4.2), and the
//          SLO miss count (Section 2: latencies must be below the constraint).
//
// Streams are per-candidate rings of 64-bit keys (time << 32 | query index) in global memory,
// so that comparing keys compares (time, query index).  All operations of a candidate are run
// round-robin by its wavefront until every stream is drained; an operation stops when it needs
// input that is not there yet or output space that is not free yet.
#pragma once
#include "est_types.h"

namespace estdev {

EST_DEV uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }
EST_DEV uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
EST_DEV uint32_t popc64(uint64_t x) { return (uint32_t)__builtin_popcountll(x); }
EST_DEV uint32_t ctz64(uint64_t x) { return (uint32_t)__builtin_ctzll(x); }
EST_DEV uint64_t lanes_below(uint32_t l) { return l >= 64 ? ~0ull : ((1ull << l) - 1ull); }

// Saturating clock: every computed time is min(true time, horizon = 2^32 - 1).
EST_DEV uint32_t sat_add(uint32_t t, uint32_t d) {
    uint32_t e = t + d;
    return e < t ? 0xFFFFFFFFu : e;
}

// LDS of one wavefront while it merges, for a plan whose widest merge has k sources: see merge_run.
// Size: EST_LDS_MERGE_BYTES(k).

struct Ctx {
    const EstSimArgs *a;
    const EstPlan *P;
    uint32_t *st;
    uint64_t *rings;
    uint32_t *rep;
    uint32_t *slots;
    uint8_t *tab;  // time tables of the merges that join several streams
    uint32_t *lat;
    const EstStageCfg *cfg;
    uint64_t *lds;
    uint32_t t;  // candidate index
    // streams taken from another candidate's captured run instead of this one's scratch (bit per ring)
    uint64_t memo_rings;
    const uint64_t *cap_rings;
};

// Diagnostics record of candidate t and stage s: EST_DBG_WORDS words (general steps, ticks in the stage's scan,
// shortcut steps, queries in shortcut steps, of which: lean light-load, light-load, one-per-batch, block of batches;
// then ticks spent in steps that ended as: lean light-load, light-load, one-per-batch, block, backlog or horizon, general;
// then ticks in the recurrence of the block steps and the batches those ran ahead).
// The record of stage EST_MAX_STAGES-1 holds what belongs to no stage: ticks in merges, in the sink, in the
// selection, merge rounds, merge output elements, merge calls, scan calls, queries in general steps.
EST_DEV uint64_t *est_dbg_rec(const EstSimArgs *a, uint32_t t, uint32_t s) {
    return a->dbg_ticks + a->n_cfg + ((uint64_t)t * EST_MAX_STAGES + s) * EST_DBG_WORDS;
}

// Ring cursors and the other state words of a candidate are written by the operation that owns them and read
// by its neighbours, which may run in another wavefront of the workgroup (several wavefronts per candidate):
// they are read and written through these (the value is the same in every lane).
EST_DEV uint32_t ld_st(const uint32_t *p) { return wv::load_shared(p); }
EST_DEV void st_st(uint32_t *p, uint32_t v) { wv::store_shared(p, v); }

struct View {
    const uint64_t *base;
    uint32_t mask, wr, fin;
};

template <bool MEMO>
EST_DEV View view_of(const Ctx &c, int32_t ring) {
    View v;
    if (ring == EST_SRC_TRACE) {
        v.base = c.a->trace_keys;
        v.mask = 0xFFFFFFFFu;
        v.wr = c.a->n;
        v.fin = 1;
    } else if (MEMO && ((c.memo_rings >> ring) & 1ull)) {  // a whole stream somebody else produced; cursors were preset
        const EstRing &R = c.a->cap_plan->rings[ring];
        v.base = c.cap_rings + R.off;
        v.mask = R.cap_mask;
        v.wr = c.st[c.P->wr_off + ring];
        v.fin = 1;
    } else {
        const EstRing &R = c.P->rings[ring];
        v.base = c.rings + R.off;
        v.mask = R.cap_mask;
        v.fin = ld_st(&c.st[c.P->fin_off + ring]);  // (before the cursor: a stream seen as ended is seen whole)
        v.wr = ld_st(&c.st[c.P->wr_off + ring]);
    }
    return v;
}

// The same with the scalars marked as identical in every lane (they are: one address, one value), which
// keeps everything computed from them in scalar registers.
template <bool MEMO>
EST_DEV View uniform_view_of(const Ctx &c, int32_t ring) {
    View v = view_of<MEMO>(c, ring);
    v.mask = wv::uniform(v.mask);
    v.wr = wv::uniform(v.wr);
    v.fin = wv::uniform(v.fin);
    return v;
}

// Free elements of a ring: capacity minus the distance to its slowest consumer.
EST_DEV uint32_t ring_space(const Ctx &c, int32_t ring, uint32_t wr) {
    const EstRing &R = c.P->rings[ring];
    uint32_t used = 0;
    for (uint32_t i = 0; i < R.n_cons; ++i) used = umax(used, wr - ld_st(&c.st[c.P->rd_off + R.cons_edge[i]]));
    EST_CHECK(used <= R.cap_mask + 1u);
    return R.cap_mask + 1u - used;
}

// Lanes that keep the smaller value in the compare-exchange step (k, j) of a bitonic network:
// those whose bit j and bit k are both clear or both set.
constexpr uint64_t keep_min_mask(uint32_t k, uint32_t j) {
    uint64_t m = 0;
    for (uint32_t l = 0; l < 64; ++l)
        if (((l & j) == 0) == ((l & k) == 0)) m |= 1ull << l;
    return m;
}

// Ascending bitonic sort of the values of lanes 0 .. width-1 (width a power of two, the same in
// every lane; lanes beyond it take part but their result is not used).
template <uint32_t K, uint32_t J>
EST_DEV uint32_t cmpx(uint32_t v, uint32_t o) {
    constexpr uint64_t M = keep_min_mask(K, J);
    return wv::lane_in(M) ? umin(v, o) : umax(v, o);
}
EST_DEV uint32_t sort_lanes(uint32_t v, uint32_t width) {
    const uint32_t ln = wv::lane();
    v = cmpx<2, 1>(v, wv::xor1(v));
    if (width <= 2) return v;
    v = cmpx<4, 2>(v, wv::xor2(v));
    v = cmpx<4, 1>(v, wv::xor1(v));
    if (width <= 4) return v;
    v = cmpx<8, 4>(v, wv::xor4(v));
    v = cmpx<8, 2>(v, wv::xor2(v));
    v = cmpx<8, 1>(v, wv::xor1(v));
    if (width <= 8) return v;
    v = cmpx<16, 8>(v, wv::xor8(v));
    v = cmpx<16, 4>(v, wv::xor4(v));
    v = cmpx<16, 2>(v, wv::xor2(v));
    v = cmpx<16, 1>(v, wv::xor1(v));
    if (width <= 16) return v;
    v = cmpx<32, 16>(v, wv::shfl(v, ln ^ 16));
    v = cmpx<32, 8>(v, wv::xor8(v));
    v = cmpx<32, 4>(v, wv::xor4(v));
    v = cmpx<32, 2>(v, wv::xor2(v));
    v = cmpx<32, 1>(v, wv::xor1(v));
    if (width <= 32) return v;
    v = cmpx<64, 32>(v, wv::shfl(v, ln ^ 32));
    v = cmpx<64, 16>(v, wv::shfl(v, ln ^ 16));
    v = cmpx<64, 8>(v, wv::xor8(v));
    v = cmpx<64, 4>(v, wv::xor4(v));
    v = cmpx<64, 2>(v, wv::xor2(v));
    v = cmpx<64, 1>(v, wv::xor1(v));
    return v;
}

// Ascending bitonic sort of one 64-bit key per lane over all 64 lanes.
template <uint32_t K, uint32_t J>
EST_DEV uint64_t cmpx64(uint64_t v, uint32_t ohi, uint32_t olo) {
    constexpr uint64_t M = keep_min_mask(K, J);
    const uint64_t o = ((uint64_t)ohi << 32) | olo;
    return ((o < v) == wv::lane_in(M)) ? o : v;
}
template <uint32_t K>
EST_DEV uint64_t sort_merge64(uint64_t v) {  // the compare-exchange steps (K, K/2), ..., (K, 1)
    const uint32_t ln = wv::lane();
    if (K >= 64) v = cmpx64<K, 32>(v, wv::shfl((uint32_t)(v >> 32), ln ^ 32), wv::shfl((uint32_t)v, ln ^ 32));
    if (K >= 32) v = cmpx64<K, 16>(v, wv::shfl((uint32_t)(v >> 32), ln ^ 16), wv::shfl((uint32_t)v, ln ^ 16));
    if (K >= 16) v = cmpx64<K, 8>(v, wv::xor8((uint32_t)(v >> 32)), wv::xor8((uint32_t)v));
    if (K >= 8) v = cmpx64<K, 4>(v, wv::xor4((uint32_t)(v >> 32)), wv::xor4((uint32_t)v));
    if (K >= 4) v = cmpx64<K, 2>(v, wv::xor2((uint32_t)(v >> 32)), wv::xor2((uint32_t)v));
    return cmpx64<K, 1>(v, wv::xor1((uint32_t)(v >> 32)), wv::xor1((uint32_t)v));
}
EST_DEV uint64_t sort_lanes64(uint64_t v) {
    v = sort_merge64<2>(v);
    v = sort_merge64<4>(v);
    v = sort_merge64<8>(v);
    v = sort_merge64<16>(v);
    v = sort_merge64<32>(v);
    return sort_merge64<64>(v);
}

// Keys (e << 32 | q) of the lanes in VM, ascending, in lanes 0 .. popcount(VM)-1 (2^64-1 elsewhere).
// Every e is at least base.  While the times span less than 2^26 the sort runs on 32-bit
// (time - base, lane) pairs; equal times keep their lane order, and if that is not the order of the
// query indices the full 64-bit sort is used after all.
EST_DEV uint64_t sort_time_query(uint32_t e, uint32_t q, uint64_t VM, uint32_t base) {
    const uint32_t ln = wv::lane();
    const bool valid = wv::lane_in(VM);
    const uint32_t d = e - base;
    if ((VM & wv::ballot(d >= (1u << 26))) == 0) {
        const uint32_t k = sort_lanes(valid ? ((d << 6) | ln) : 0xFFFFFFFFu, 64);
        const uint32_t qs = wv::shfl(q, k & 63u);
        const uint32_t ds = k >> 6;
        const uint32_t dp = wv::shr1(ds), qp = wv::shr1(qs);
        const uint32_t n = popc64(VM);
        if ((lanes_below(n) & ~1ull & wv::ballot(dp == ds) & wv::ballot(qp > qs)) == 0)
            return ln < n ? (((uint64_t)(base + ds) << 32) | qs) : ~0ull;
    }
    return sort_lanes64(valid ? (((uint64_t)e << 32) | q) : ~0ull);
}

// ------------------------------------------------------------------------------------------ SCAN
//
// Per-wavefront working set of a scan, in LDS:
//   in-ring   128 or 256 keys (EstPlan::scan_ring: the smaller one where it lets one more wavefront share a SIMD):
//             the next elements of the stage's input stream,
//             refilled from the source ring in chunks (and filtered on the way, when only some
//             elements of the source visit the stage);
//   slots     one per replica: the members of the replica's last batch, sorted by query index,
//             waiting to be emitted when the batch completes.
// The replica table lives in registers, lane r holding the r-th replica in order of the time it is
// free again, so the earliest free replica is lane 0 and batches complete in lane order.


// Number of lanes whose value is below x (<= x with incl), for values that ascend with the lane: a binary search
// over the lanes, the same for every lane's own x.  Only the first width lanes are searched (a power of two, the
// same in every lane): no lane from there on may pass the test.
EST_DEV uint32_t lanes_less(uint32_t v, uint32_t x, bool incl, uint32_t width = 64u) {
    uint32_t pos = 0;
    for (uint32_t step = width >> 1; step >= 1; step >>= 1) {
        const uint32_t y = wv::shfl(v, pos + step - 1u);
        if (incl ? y <= x : y < x) pos += step;
    }
    const uint32_t y = wv::shfl(v, width - 1u);  // (pos is width-1 only when the lanes before that one all pass)
    if (pos == width - 1u && (incl ? y <= x : y < x)) pos = width;
    return pos;
}

// The smallest power of two that is at least n (n from 1 to 64), at least 2
EST_DEV uint32_t pow2_at_least(uint32_t n) { return n <= 2u ? 2u : 1u << (32u - (uint32_t)__builtin_clz(n - 1u)); }

// Write the members of the batches in the table lanes of tie, which all complete at time mv, merged by
// query index, to out[base ...]; returns their number.  (Times clamped at the horizon need no order:
// everything downstream of a clamped time is clamped too, so those are concatenated.)  tw: lanes of the table.
EST_DEV uint32_t emit_tied(const EstOp &op, const uint32_t *lslots, uint64_t tie, uint32_t mv, uint32_t rcnt, uint32_t rslot,
                           uint64_t *out, uint32_t omask, uint32_t base, uint32_t tw) {
    const uint32_t ln = wv::lane();
    const uint32_t bm = wv::uniform(op.b_max);
    const uint64_t tkey = (uint64_t)mv << 32;
    uint32_t total = 0;
    if (mv == 0xFFFFFFFFu) {
        for (uint64_t m = tie; m; m &= m - 1) {
            const uint32_t r = ctz64(m);
            const uint32_t cr = wv::bcast(rcnt, r), sl = wv::bcast(rslot, r);
            if (ln < cr) out[(base + total + ln) & omask] = tkey | lslots[sl * bm + ln];
            total += cr;
        }
        return total;
    }
    for (uint64_t m = tie; m; m &= m - 1) total += wv::bcast(rcnt, ctz64(m));
    if (total <= 64u) {
        // all members fit one per lane (a group that arrived together and was cut into many small batches, say): lane i
        // takes the i-th member in table order, and one sorting network over the query indices does the merge
        const uint32_t c = wv::lane_in(tie) ? rcnt : 0u;
        const uint32_t off = wv::prefix_excl_u32(c);
        const uint32_t l = lanes_less(off, ln, true, tw) - 1u;  // the last table lane whose batch starts at or before position ln
        const uint32_t o = wv::shfl(off, l), sl = wv::shfl(rslot, l);
        const uint32_t x = ln < total ? lslots[sl * bm + (ln - o)] : 0xFFFFFFFFu;  // (query indices stay below 2^31)
        const uint32_t sorted = sort_lanes(x, pow2_at_least(total));
        if (ln < total) out[(base + ln) & omask] = tkey | sorted;
        return total;
    }
    // rank every member among all of them
    total = 0;
    for (uint64_t m = tie; m; m &= m - 1) {
        const uint32_t r = ctz64(m);
        const uint32_t cr = wv::bcast(rcnt, r), sl = wv::bcast(rslot, r);
        const uint32_t x = ln < cr ? lslots[sl * bm + ln] : 0u;
        uint32_t rank = ln;
        for (uint64_t m2 = tie; m2; m2 &= m2 - 1) {
            const uint32_t r2 = ctz64(m2);
            const uint32_t c2 = wv::bcast(rcnt, r2), sl2 = wv::bcast(rslot, r2);
            if (r2 == r || ln >= cr) continue;
            const uint32_t *s2 = lslots + sl2 * bm;
            uint32_t lo = 0, hi = c2;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (s2[mid] < x) lo = mid + 1; else hi = mid;
            }
            rank += lo;
        }
        if (ln < cr) out[(base + rank) & omask] = tkey | x;
        total += cr;
    }
    return total;
}

// The batches in the table lanes of E (ascending completion times, no two of them equal) written out in table
// order in one sweep: off (the members of the lanes of E before mine, e.g. from emit_offsets) turns an output
// position into a batch and a member.  Every member goes to out[base + its position + extra of its batch], where
// extra is a per-batch displacement (lane = table lane; 0 to write them back to back).
EST_DEV void emit_many(const EstOp &op, const uint32_t *lslots, uint32_t total, uint32_t off, uint32_t extra, uint32_t rend,
                       uint32_t rslot, uint64_t *out, uint32_t omask, uint32_t base, uint32_t tw) {
    const uint32_t ln = wv::lane();
    const uint32_t bm = wv::uniform(op.b_max);
    for (uint32_t i0 = 0; i0 < total; i0 += 64) {
        const uint32_t i = i0 + ln;
        const uint32_t l = lanes_less(off, i, true, tw) - 1u;  // the last lane whose batch starts at or before position i
        const uint32_t o = wv::shfl(off, l), e = wv::shfl(rend, l), sl = wv::shfl(rslot, l), x = wv::shfl(extra, l);
        if (i < total) out[(base + i + x) & omask] = ((uint64_t)e << 32) | lslots[sl * bm + (i - o)];
    }
}

// Older waiting batches (table lanes in woven, ascending completion times, all different from the new
// ones) leave together with new queries: the new ones, whose completion times are ke in the lanes of emitm,
// have been placed already, each shifted by the members of the older batches that finish before it; here the
// older batches are written into the gaps, those that complete together merged by query index.
EST_DEV void weave_out(const EstOp &op, const uint32_t *lslots, uint64_t woven, uint64_t emitm, uint32_t ke, uint32_t rend,
                       uint32_t rcnt, uint32_t rslot, uint64_t *out, uint32_t omask, uint32_t wr, uint32_t tw) {
    const uint32_t ln = wv::lane();
    const uint32_t bm = wv::uniform(op.b_max);
    uint32_t before = 0;
    for (uint64_t pm = woven; pm;) {
        const uint32_t j = ctz64(pm);
        const uint32_t ej = wv::bcast(rend, j);
        const uint64_t tie = pm & wv::ballot(rend == ej);
        const uint32_t pos = wr + before + popc64(emitm & wv::ballot(ke < ej));
        if ((tie & (tie - 1)) == 0) {
            const uint32_t cj = wv::bcast(rcnt, j), sj = wv::bcast(rslot, j);
            if (ln < cj) out[(pos + ln) & omask] = ((uint64_t)ej << 32) | lslots[sj * bm + ln];
            before += cj;
        } else {
            before += emit_tied(op, lslots, tie, ej, rcnt, rslot, out, omask, pos, tw);
        }
        pm &= ~tie;
    }
}

// New queries (their keys in the lanes of emit_me, rank orank among them, ns in all, ascending by rank) leave
// together with the older waiting batches in the table lanes of woven (extra members in all, completion times
// different from every new one): everything is written to out[wr ...] in (time, query) order.  With many older
// batches and no two of them completing together, both sides find their places by binary searches over the
// other side (lscr: 64 words of LDS scratch); otherwise batch by batch.
EST_DEV void weave_all(const EstOp &op, const uint32_t *lslots, uint32_t *lscr, uint64_t woven, uint32_t extra, bool emit_me, uint64_t emitm,
                       uint32_t orank, uint32_t ns, uint64_t key, uint32_t rend, uint32_t rcnt, uint32_t rslot, uint64_t *out,
                       uint32_t omask, uint32_t wr, uint32_t tw) {
    const uint32_t ln = wv::lane();
    const uint32_t ke = (uint32_t)(key >> 32);
    const uint64_t tied = woven & ~1ull & wv::ballot(rend == wv::shr1(rend));
    if (popc64(woven) >= 6 && tied == 0) {
        const uint32_t c = wv::lane_in(woven) ? rcnt : 0u;
        const uint32_t off = wv::prefix_excl_u32(c);
        const uint32_t pos = lanes_less(rend, ke, false, tw);        // table lanes that are free before my completion time
        const uint32_t before = wv::shfl(off, pos);                  // members of the woven batches among them
        if (emit_me) out[(wr + orank + (pos < 64u ? before : extra)) & omask] = key;
        wv::sync_lds();
        if (emit_me) lscr[orank] = ke;
        wv::sync_lds();
        const uint32_t kc = ln < ns ? lscr[ln] : 0xFFFFFFFFu;        // the new completion times in rank order
        const uint32_t nb = lanes_less(kc, rend, false, pow2_at_least(ns));  // new queries that leave before my batch
        emit_many(op, lslots, extra, off, nb, rend, rslot, out, omask, wr, tw);
        wv::sync_lds();
        return;
    }
    uint32_t shift = 0;
    for (uint64_t pm = woven; pm; pm &= pm - 1) {
        const uint32_t j = ctz64(pm);
        const uint32_t ej = wv::bcast(rend, j), cj = wv::bcast(rcnt, j);
        if (ej < ke) shift += cj;
    }
    if (emit_me) out[(wr + orank + shift) & omask] = key;
    weave_out(op, lslots, woven, emitm, ke, rend, rcnt, rslot, out, omask, wr, tw);
}

// Emit, in (completion time, query index) order, the batches whose replica-table lanes are in E
// (ascending lanes = ascending completion time).  Batches that complete at the same time are
// merged by query index.  Stops early (returns false) when the output ring cannot take the next
// group.
EST_DEV bool scan_emit(const EstOp &op, const uint32_t *lslots, uint64_t E, uint32_t rend, uint32_t &rcnt,
                       uint32_t rslot, uint64_t *out, uint32_t omask, uint32_t &wr, uint32_t &space, bool &progress, uint32_t tw) {
    const uint32_t ln = wv::lane();
    const uint32_t bm = wv::uniform(op.b_max);
    if (popc64(E) >= 3) {
        // several batches, no two completing together, and room for all of them: one sweep.  (The table is in
        // order of time, so two batches of E with the same time have only lanes of that time between them: a lane
        // of E whose time equals its left neighbour's is taken as a tie, whatever that neighbour holds.)
        const uint64_t tied = E & ~1ull & wv::ballot(rend == wv::shr1(rend));
        const uint32_t c = wv::lane_in(E) ? rcnt : 0u;
        const uint32_t off = wv::prefix_excl_u32(c);
        const uint32_t total = wv::bcast(off, 63) + wv::bcast(c, 63);
        if (tied == 0 && total <= space) {
            emit_many(op, lslots, total, off, 0u, rend, rslot, out, omask, wr, tw);
            wr += total;
            space -= total;
            if (wv::lane_in(E)) rcnt = 0;
            progress = true;
            return true;
        }
    }
    while (E) {
        const uint32_t l0 = ctz64(E);
        const uint32_t mv = wv::bcast(rend, l0);
        const uint64_t tie = E & wv::ballot(rend == mv);
        const uint64_t tkey = (uint64_t)mv << 32;
        if ((tie & (tie - 1)) == 0) {  // the common case: one batch
            const uint32_t cr = wv::bcast(rcnt, l0), sl = wv::bcast(rslot, l0);
            EST_CHECK(cr >= 1 && cr <= bm);
            if (cr > space) return false;
            if (ln < cr) out[(wr + ln) & omask] = tkey | lslots[sl * bm + ln];
            wr += cr;
            space -= cr;
        } else {
            uint32_t total = 0;
            for (uint64_t m = tie; m; m &= m - 1) total += wv::bcast(rcnt, ctz64(m));
            if (total > space) return false;
            emit_tied(op, lslots, tie, mv, rcnt, rslot, out, omask, wr, tw);
            wr += total;
            space -= total;
        }
        if ((tie >> ln) & 1ull) rcnt = 0;
        E &= ~tie;
        progress = true;
    }
    return true;
}

template <bool DIAG, bool MEMO>
EST_DEV bool scan_run(const Ctx &c, const EstOp &op, uint32_t opi) {
    const uint32_t ln = wv::lane();
    const EstPlan &P = *c.P;
    const uint32_t s = op.stage;
    const EstStageCfg sc = c.cfg[s];
    // (values read from memory are the same in every lane; saying so keeps what is computed from them in
    // scalar registers, off the vector unit)
    const uint32_t B = wv::uniform(sc.batch), R = wv::uniform(sc.replicas), bm = wv::uniform(op.b_max);
    EST_CHECK(B >= 1 && B <= op.b_max && R >= 1 && R <= op.r_max);
    const uint32_t *Ltab = c.a->lat_us + ((uint64_t)s * c.a->dag->H + sc.hw) * c.a->dag->Bmax;
    const uint32_t Lmine = ln < B ? Ltab[ln] : 0u;  // lane l holds L(l+1)
    const uint32_t L1 = wv::bcast(Lmine, 0);
    // the light-load shortcut below needs: no batch is faster than a single query
    const bool mono = (lanes_below(B) & wv::ballot(Lmine < L1)) == 0;
    uint32_t *g_end = c.rep + op.rep_off, *g_cnt = g_end + op.r_max, *g_slot = g_cnt + op.r_max;
    uint32_t *g_slots = c.slots + op.slot_off;
    uint64_t *lkey = c.lds;
    const uint32_t RING = wv::uniform(P.scan_ring), rmask = RING - 1u;
    uint32_t *ltab = (uint32_t *)(c.lds + RING);  // 4 x 64 words of per-group values (reused as staging by the rare table re-sort)
    uint32_t *lstart = ltab + 256;         // 65 (of 72): first lane of each group of a window (+ the end)
    uint16_t *linv = (uint16_t *)(ltab + 328);  // 64 half words: linv[d-1] = ceil(65536 / d) - 1, so that floor(x / d) = x * (linv[d-1] + 1) >> 16 for x <= 64
    uint32_t *lslots = ltab + 360;
    const uint8_t *acc = c.a->acc + (uint64_t)op.acc_idx * c.a->acc_stride;
    linv[ln] = (uint16_t)((65536u + ln) / (ln + 1u) - 1u);
    const uint32_t inv_b = (65536u + B - 1u) / B, inv_r = (65536u + R - 1u) / R;

    // replica table, sorted by the time the replica is free again
    const bool isrep = ln < R;
    const uint64_t REP = lanes_below(R);  // (lanes beyond the table hold end = 2^32-1, count 0)
    const uint32_t tw = pow2_at_least(R);  // searches over the table look at this many lanes
    uint32_t rend = isrep ? g_end[ln] : 0xFFFFFFFFu;
    uint32_t rcnt = isrep ? g_cnt[ln] : 0u;
    uint32_t rslot = isrep ? g_slot[ln] : 0u;
    for (uint64_t m = wv::ballot(rcnt > 0); m; m &= m - 1) {  // members still waiting: back into LDS
        const uint32_t l = ctz64(m);
        const uint32_t cn = wv::bcast(rcnt, l), sl = wv::bcast(rslot, l);
        if (ln < cn) lslots[sl * bm + ln] = g_slots[sl * bm + ln];
    }
    wv::sync_lds();

    View in = view_of<MEMO>(c, op.src_ring[0]);
    in.mask = wv::uniform(in.mask);
    in.wr = wv::uniform(in.wr);
    in.fin = wv::uniform(in.fin);
    uint32_t rraw = wv::uniform(c.st[P.rd_off + op.src_edge[0]]);  // next source position to read
    const uint32_t rd_entry = rraw;
    uint32_t lhead = 0, ltail = 0;                     // in-ring: consumed / filled
    const EstRing &OR = P.rings[op.out_ring];
    uint64_t *out = c.rings + OR.off;
    const uint32_t omask = wv::uniform(OR.cap_mask);
    uint32_t wr = wv::uniform(c.st[P.wr_off + op.out_ring]);
    uint32_t space = wv::uniform(ring_space(c, op.out_ring, wr));
    bool progress = false, finished = false;
    EST_CHK_ORDER_INIT();  // (host-side emulation only: everything written from here on is verified to be in order, step by step)
    uint32_t fp_skip = 0;   // general batches still to do before the light-load shortcut is tried again
    uint32_t sat_skip = 0;  // the same for the backlog shortcut
    uint32_t single_skip = 0;  // and for the one-query-per-batch shortcut
    uint32_t blk_skip = 0;     // and for the block of batches
    uint32_t lean_skip = 0;    // and for the light-load step on large groups
    uint32_t cf_skip = 0;      // and for the closed forms of one query per batch
    uint64_t d_blkl = 0, d_blkk = 0;  // diagnostics: ticks in the recurrence of the block step, batches it ran ahead
    uint64_t d_tk[6] = {0, 0, 0, 0, 0, 0}, tk0 = 0;  // diagnostics: ticks by the kind of step that ended the iteration
    uint32_t d_gen = 0, d_gene = 0, d_fp = 0, d_fpe = 0, d_b1 = 0, d_b1e = 0, d_sat = 0, d_sate = 0, d_hz = 0, d_blk = 0, d_blke = 0, d_lean = 0, d_leane = 0;  // diagnostics

    for (;;) {
        uint32_t staged = ltail - lhead;
        if (staged < 64 && rraw != in.wr) {
            // refill: as much of the source as the ring has room for beside what is staged (up to three loads of 64
            // elements, issued together)
            const uint32_t left = umin(umin(in.wr - rraw, RING - staged), 192u);
            const uint32_t w0 = umin(left, 64u), w1 = left > 64 ? umin(left - 64, 64u) : 0u,
                           w2 = left > 128 ? umin(left - 128, 64u) : 0u;
            const uint64_t k0 = ln < w0 ? in.base[(rraw + ln) & in.mask] : 0ull;
            const uint64_t k1 = ln < w1 ? in.base[(rraw + 64 + ln) & in.mask] : 0ull;
            const uint64_t k2 = ln < w2 ? in.base[(rraw + 128 + ln) & in.mask] : 0ull;
            // (lane masks are combined as scalars: one vector compare per term)
            uint64_t A0 = lanes_below(w0), A1 = lanes_below(w1), A2 = lanes_below(w2);
            bool a0 = ln < w0, a1 = ln < w1, a2 = ln < w2;
            if (op.filtered) {  // (lanes beyond a window hold key 0: query 0 exists)
                const bool f0 = (acc[(uint32_t)k0] & 1u) != 0u, f1 = (acc[(uint32_t)k1] & 1u) != 0u, f2 = (acc[(uint32_t)k2] & 1u) != 0u;
                A0 &= wv::ballot(f0); A1 &= wv::ballot(f1); A2 &= wv::ballot(f2);
                a0 = a0 && f0; a1 = a1 && f1; a2 = a2 && f2;
            }
            const uint32_t i0 = (ltail + wv::rank_below(A0)) & rmask;
            ltail += popc64(A0);
            const uint32_t i1 = (ltail + wv::rank_below(A1)) & rmask;
            ltail += popc64(A1);
            const uint32_t i2 = (ltail + wv::rank_below(A2)) & rmask;
            ltail += popc64(A2);
            if (a0) lkey[i0] = k0;
            if (a1) lkey[i1] = k1;
            if (a2) lkey[i2] = k2;
            rraw += w0 + w1 + w2;
            EST_CHECK(ltail - lhead <= RING);
            wv::sync_lds();
            continue;
        }
        if (staged == 0) {
            if (in.fin) {  // input exhausted for good: flush what is still in flight
                const uint64_t E = wv::ballot(rcnt > 0);
                if (!E || scan_emit(op, lslots, E, rend, rcnt, rslot, out, omask, wr, space, progress, tw)) finished = true;
            }
            break;
        }
        // every step below works on a window of up to 64 queries and may emit as many: with less room
        // than that in the output ring, let the reader run first rather than squeeze batches through
        if (space < 64u) break;
        if (DIAG) tk0 = wv::ticks();
        const uint32_t w = umin(staged, 64u);
        const uint64_t key = ln < w ? lkey[(lhead + ln) & rmask] : ~0ull;
        const uint32_t rdy = (uint32_t)(key >> 32);
        uint32_t q = (uint32_t)key;
        EST_CHECK(ln == 0 || ln >= w || rdy == 0xFFFFFFFFu || key > lkey[(lhead + ln - 1) & rmask]);  // input is ordered
        const uint32_t f0 = wv::uniform(rend);  // earliest free replica = lane 0
        if (f0 == 0xFFFFFFFFu) {
            // Every replica is busy up to the horizon: whatever is still queued starts and ends at the
            // horizon, where order no longer matters.  Waiting batches leave first, then the window.
            const uint64_t E = wv::ballot(rcnt > 0);
            if (E && !scan_emit(op, lslots, E, rend, rcnt, rslot, out, omask, wr, space, progress, tw)) break;
            const uint32_t m = umin(w, space);
            if (m == 0) break;
            if (ln < m) out[(wr + ln) & omask] = 0xFFFFFFFF00000000ull | q;
            wr += m;
            space -= m;
            lhead += m;
            d_hz += m;
            if (DIAG) d_tk[4] += wv::ticks() - tk0;
            progress = true;
            continue;
        }
        if (B >= 2) {
            if (sat_skip == 0 && B <= 32 && w >= 2 * B && wv::bcast(rdy, B - 1) <= f0) {
                // Backlog: while the queue holds a full batch whenever a replica frees, the replicas take
                // full batches in rotation.  With the free times f_0 <= ... <= f_{R-1} < f_0 + L(B), batch k
                // (queries kB .. kB+B-1 of the window) starts at f_k, where f_k = f_{k-R} + L(B) for k >= R,
                // provided its last member is ready by then.  The leading batches that satisfy this are all
                // dispatched at once; as in the general step, everything that completes by the last of
                // these dispatch times leaves, the rest waits in the slots of the replicas.
                const uint32_t LB = wv::bcast(Lmine, B - 1);
                const uint32_t tl = wv::bcast(rend, R - 1);
                uint32_t nacc = 0;
                if (tl < wv::sat_add_uniform(f0, LB)) {
                    const uint32_t lo = wv::opaque(ln);
                    const uint32_t kb = (lo * inv_b) >> 16;        // my batch
                    const uint32_t kd = (kb * inv_r) >> 16, km = kb - kd * R;
                    const uint64_t ft = (uint64_t)wv::shfl(rend, km) + (uint64_t)kd * LB;
                    const uint32_t fk = ft >= 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)ft;
                    const uint32_t e = sat_add(fk, LB);
                    const uint32_t nfull = (w * inv_b) >> 16;
                    const uint32_t lastr = wv::shfl(rdy, kb * B + B - 1u);
                    const uint64_t okm = lanes_below(nfull * B) & wv::ballot(lastr <= fk) & wv::ballot(e != 0xFFFFFFFFu);
                    const uint32_t nl = okm == ~0ull ? 64u : ctz64(~okm);  // a multiple of B: the test is per batch
                    nacc = (nl * inv_b) >> 16;
                    if (nacc >= 2) {
                        const uint32_t na = nacc * B;
                        const uint32_t Tlast = wv::bcast(fk, na - 1u);
                        const uint64_t E = wv::ballot(rcnt > 0) & wv::ballot(rend <= Tlast);
                        const uint64_t D = lanes_below(na) & wv::ballot(e <= Tlast);  // replaced again inside this step: never wait
                        const bool direct = ln < na && e <= Tlast;
                        const uint32_t nd = popc64(D);
                        if (popc64(E) * B + nd > space) {
                            nacc = 0;  // tight output ring: batch by batch
                        } else {
                            scan_emit(op, lslots, E, rend, rcnt, rslot, out, omask, wr, space, progress, tw);
                            const uint32_t eprev = wv::shr1(e), qprev = wv::shr1(q), kprev = wv::shr1(kb);
                            uint64_t okey = direct ? (((uint64_t)e << 32) | q) : ~0ull;
                            if (D & ~1ull & wv::ballot(eprev == e) & wv::ballot(qprev > q)) okey = sort_lanes64(okey);
                            if (ln < nd) out[(wr + ln) & omask] = okey;  // (times ascend with the batch: a prefix)
                            wr += nd;
                            space -= nd;
                            EST_CHK_ORDER(6);
                            // members wait sorted by query index
                            uint32_t qs = q;
                            if (lanes_below(na) & ~lanes_below(umax(nd, 1u)) & wv::ballot(kprev == kb) & wv::ballot(qprev > q))
                                qs = (uint32_t)sort_lanes64(ln < na ? (((uint64_t)kb << 32) | q) : ~0ull);
                            const uint32_t myslot = wv::shfl(rslot, km);
                            if (ln >= nd && ln < na) lslots[myslot * bm + (ln - kb * B)] = qs;
                            // new table: the entries not replaced, then the last min(nacc, R) batches
                            const uint32_t nn = umin(nacc, R);
                            const uint32_t src = (nacc - R + ln) * B;  // first lane of the batch that lands in table lane ln
                            const uint32_t oe = wv::shfl(rend, ln + nn), oc = wv::shfl(rcnt, ln + nn), os = wv::shfl(rslot, ln + nn);
                            const uint32_t ne = wv::shfl(e, src), ns = wv::shfl(myslot, src);
                            if (isrep) {
                                if (ln + nn < R) {
                                    rend = oe; rcnt = oc; rslot = os;
                                } else {
                                    rend = ne; rcnt = ne > Tlast ? B : 0u; rslot = ns;
                                }
                            }
                            wv::sync_lds();
                            lhead += na;
                            ++d_sat; d_sate += na;
                            if (DIAG) d_tk[4] += wv::ticks() - tk0;
                            progress = true;
                            continue;
                        }
                    }
                }
                if (nacc < 2) sat_skip = 4;
            }
        }
        if (cf_skip == 0 && L1 > 0 && (B == 1 || mono) && w >= 32 && R <= 31 && wv::ballot(rcnt > 0) == 0) {
            // Closed forms for a whole window of queries that are each a batch of their own, checked with one
            // vote and left to the steps below when they do not hold.  Query i runs on the replica that served
            // query i-R (the table's entry i for the first R).
            //   Nobody waits: every query finds that replica free again by the time it is ready, ready[i] >=
            //   ready[i-R] + L(1) (for B > 1 no two queries may become ready together): end[i] = ready[i] + L(1).
            //   Everybody waits (B = 1): ready[i] <= end[i-R], so end[i] = free[i mod R] + (i div R + 1) L(1), as
            //   long as these ascend strictly (they do while the free times lie within one L(1) of each other;
            //   equal completion times would have to be put in query order).
            const bool final = staged <= 64 && rraw == in.wr && in.fin;
            const uint64_t WM = lanes_below(w);
            const uint32_t back = ln >= R && ln < w ? (uint32_t)(lkey[(lhead + ln - R) & rmask] >> 32) : 0u;
            const uint32_t prev1 = ln < R ? rend : sat_add(back, L1);
            uint64_t ok1 = WM & wv::ballot(prev1 <= rdy);
            if (B > 1) ok1 &= wv::ballot(rdy != wv::shl1(rdy)) | ~lanes_below(w - 1u);
            uint32_t m = 0, x = 0;
            if (ok1 == WM) {
                m = (B > 1 && !final) ? w - 1u : w;  // (for B > 1 the last query may yet be joined by the next)
                x = sat_add(rdy, L1);
            } else if (B == 1) {
                const uint32_t lo = wv::opaque(ln);
                const uint32_t kd = (lo * inv_r) >> 16, km = lo - kd * R;
                const uint64_t st = (uint64_t)wv::shfl(rend, km) + (uint64_t)kd * L1;  // when my replica is free for me
                const uint64_t en = st + L1;
                x = en >= 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)en;
                const uint32_t xp = wv::shr1(x);
                if ((WM & ~(wv::ballot((uint64_t)rdy <= st) & wv::ballot(x != 0xFFFFFFFFu) & (wv::ballot(x > xp) | 1ull))) == 0) m = w;
            }
            if (m >= R && wv::bcast(x, m - 1u) != 0xFFFFFFFFu) {
                if (ln < m) out[(wr + ln) & omask] = ((uint64_t)x << 32) | q;
                wr += m;
                space -= m;
                EST_CHK_ORDER(9);
                const uint32_t tnew = wv::shfl(x, ln + m - R);  // the table becomes the last R completion times
                if (isrep) rend = tnew;
                lhead += m;
                ++d_b1; d_b1e += m;
                if (DIAG) d_tk[2] += wv::ticks() - tk0;
                progress = true;
                continue;
            }
            cf_skip = 6;
        } else if (cf_skip) {
            --cf_skip;
        }
        const bool b1 = B == 1 && L1 > 0;
        // With larger batch sizes the same evaluation holds as long as no query waits and no two become
        // ready together: then every query is a batch of its own, started on arrival.
        const bool single = !b1 && B > 1 && mono && L1 > 0 && single_skip == 0 && w >= 16 && wv::ballot(rcnt > 0) == 0;
        if (b1 || single) {
            // Maximum batch size 1: every query is its own batch and the service time is the constant
            // L(1), so completions keep the input order and query i runs on the replica that served
            // query i-R:  end_i = max(ready_i, end_{i-R}) + L(1).  The sorted replica table is exactly
            // (end_{i-R}, ..., end_{i-1}), so a whole window is evaluated at once with a max-plus
            // scan of stride R.  Nothing waits in slots: results are written out immediately.
            EST_CHECK(wv::ballot(rcnt > 0) == 0);
            uint32_t x = sat_add(umax(rdy, isrep ? rend : 0u), L1);
            for (uint32_t d = R, mul = 1; d < 64; d <<= 1, mul <<= 1) {
                const uint32_t y = wv::shfl(x, ln - d);
                const uint32_t inc = (uint64_t)mul * L1 > 0xFFFFFFFFull ? 0xFFFFFFFFu : mul * L1;
                if (ln >= d) x = umax(x, sat_add(y, inc));
            }
            const bool last = staged <= 64 && rraw == in.wr && in.fin;
            uint32_t m = umin(w, space);
            bool sorted = true;
            if (single) {
                // the leading queries that start on arrival, each alone at its ready time (the one after
                // it must be seen to become ready later); completion times then ascend strictly, and
                // whatever is dispatched later finishes later still
                const uint32_t rnext = wv::shl1(rdy);
                const uint64_t gm = lanes_below(w) & wv::ballot(x == sat_add(rdy, L1)) & wv::ballot(x != 0xFFFFFFFFu) &
                                    ((wv::ballot(rdy != rnext) & lanes_below(w - 1u)) | (last ? 1ull << (w - 1u) : 0ull));
                const uint32_t m1 = gm == ~0ull ? 64u : ctz64(~gm);
                if (m1 < 12) {
                    single_skip = 6;  // not the regime: leave it alone for a few steps
                    m = 0;
                } else {
                    m = umin(m1, space);
                    if (m == 0) break;  // wait for the consumer
                }
            } else {
                // Queries that complete at the same time leave ordered by query index.  Since
                // end_i > end_{i-R}, such a run has at most R members; a shorter run at the end of what
                // can be written now may continue with the next query, and is kept back until that is
                // known (times clamped at the horizon need no order).
                const uint32_t xp = wv::shr1(x);
                const uint32_t qp = wv::shr1(q);
                const uint64_t bnd = (lanes_below(w) & wv::ballot(x != xp)) | 1ull;  // starts of runs
                if (m > 0) {
                    const uint32_t s0 = 63u - (uint32_t)__builtin_clzll(bnd & lanes_below(m));  // start of the run of lane m-1
                    const uint32_t xl = wv::bcast(x, m - 1u);
                    const bool complete = m < w ? wv::bcast(x, m) != xl : (last || xl == 0xFFFFFFFFu || m - s0 >= R);
                    if (!complete) m = s0;
                }
                if (m == 0) break;  // wait for the consumer, or for the rest of the run
                sorted = (lanes_below(m) & ~1ull & wv::ballot(x == xp) & wv::ballot(q < qp) & wv::ballot(x != 0xFFFFFFFFu)) == 0;
            }
            if (m > 0) {
                uint64_t okey = ln < m ? (((uint64_t)x << 32) | q) : ~0ull;
                if (!sorted) okey = sort_lanes64(okey);
                if (ln < m) out[(wr + ln) & omask] = okey;
                wr += m;
                space -= m;
                ++d_b1; d_b1e += m;
                if (DIAG) d_tk[2] += wv::ticks() - tk0;
                EST_CHK_ORDER(1);
                // the table becomes the last R completion times
                const uint32_t keep = R > m ? R - m : 0u;  // old entries that stay
                const uint32_t told = wv::shfl(rend, ln + m);
                const uint32_t tnew = wv::shfl(x, ln + m - R);
                if (isrep) rend = ln < keep ? told : tnew;
                // (old entries that stay hold no members, so they ended by some earlier start + L(1): no later than the new ends)
                const uint32_t rbefore = wv::shr1(rend);
                EST_CHECK(ln == 0 || !isrep || rend >= rbefore);
                (void)rbefore;
                lhead += m;
                progress = true;
                continue;
            }
        }
        if (single_skip) --single_skip;
        if (mono && L1 > 0 && lean_skip == 0 && w >= 16) {
            // Light load, large groups: the queries of a run (same ready time, at most B of them) are one batch,
            // started at that time on a replica that is idle when the window's first query becomes ready.  When
            // the new completion times ascend from run to run and all lie after every completion time already in
            // the table, the table stays sorted by appending them, and the output order is settled by the table
            // alone: the members of the new batches wait in their replicas' slots, and what leaves now are the older
            // batches that finish before tau = (ready time of the first query after the accepted runs) + L(1),
            // before which nothing dispatched later can finish.  Work per run, not per query, apart from moving
            // the query indices.
            const uint32_t r0 = wv::uniform(rdy);
            const uint64_t WM = lanes_below(w);
            const uint32_t rprev = wv::shr1(rdy);
            const uint64_t heads = WM & (wv::ballot(rdy != rprev) | 1ull);
            const bool final = staged <= 64 && rraw == in.wr && in.fin;
            const uint32_t p = popc64(REP & wv::ballot(rend <= r0));  // idle now: a prefix of the sorted table
            const uint32_t gid = wv::rank_below(heads >> 1);           // my run (lane 0 starts run 0)
            uint32_t m = final ? w : 63u - (uint32_t)__builtin_clzll(heads);  // the last run may go on beyond the window
            {
                const uint64_t fits = WM & wv::ballot(gid < p);               // one idle replica per run
                m = umin(m, fits == ~0ull ? 64u : ctz64(~fits));
            }
            const uint64_t AM = lanes_below(m);
            const uint64_t hA = heads & AM;
            const uint32_t G = popc64(hA);
            bool done = false;
            if (m >= 16 && 4u * G <= m) {
                // my run: lanes [start, nh)
                const uint64_t upto = lanes_below(wv::opaque(ln) + 1u);
                const uint32_t start = 63u - (uint32_t)__builtin_clzll((hA & upto) | 1ull);
                const uint64_t later = ln == 63 ? 0ull : (hA >> (ln + 1));
                const uint32_t nh = later ? ln + 1u + ctz64(later) : m;
                const uint32_t g = nh - start;
                const uint32_t e = sat_add(rdy, wv::shfl(Lmine, (g - 1u) & 63u));  // (L is 0 beyond B: rejected below)
                const uint32_t eprev = wv::shr1(e);
                const uint64_t bad = AM & (wv::ballot(g > B) | wv::ballot(e == 0xFFFFFFFFu) | (hA & ~1ull & wv::ballot(eprev >= e)));
                const uint32_t e0 = wv::uniform(e), last_old = wv::bcast(rend, R - 1u);
                if (bad == 0 && (G == R || e0 > last_old)) {
                    const bool tau_inf = final && m >= w;
                    const uint32_t tau = tau_inf ? 0xFFFFFFFFu : wv::sat_add_uniform(wv::bcast(rdy, umin(m, w - 1u)), L1);
                    const uint64_t E = wv::ballot(rcnt > 0) & (tau_inf ? ~0ull : wv::ballot(rend < tau));
                    if (E && !scan_emit(op, lslots, E, rend, rcnt, rslot, out, omask, wr, space, progress, tw)) break;  // wait for the consumer
                    EST_CHK_ORDER(8);
                    wv::sync_lds();  // the slots of batches just written out may be taken again
                    const uint32_t myslot = wv::shfl(rslot, gid);
                    if (ln < m) lslots[myslot * bm + (ln - start)] = q;
                    if (ln < m && ln == start) { ltab[gid] = e; ltab[64 + gid] = g; }
                    wv::sync_lds();
                    // new table: the entries not taken move down, the new batches follow in run order
                    const uint32_t keep = R - G;
                    const uint32_t oe = wv::shfl(rend, ln + G), oc = wv::shfl(rcnt, ln + G), os = wv::shfl(rslot, ln + G);
                    const uint32_t k = ln >= keep && ln < R ? ln - keep : 0u;
                    const uint32_t ns = wv::shfl(rslot, k);
                    const uint32_t ne = ltab[k], nc = ltab[64 + k];
                    if (isrep) {
                        if (ln < keep) {
                            rend = oe; rcnt = oc; rslot = os;
                        } else {
                            rend = ne; rcnt = nc; rslot = ns;
                        }
                    }
                    wv::sync_lds();
                    lhead += m;
                    ++d_lean; d_leane += m;
                    if (DIAG) d_tk[0] += wv::ticks() - tk0;
                    progress = true;
                    done = true;
                }
            }
            if (done) continue;
            lean_skip = 4;
        } else if (lean_skip) {
            --lean_skip;
        }
        if (mono && fp_skip == 0) {
            // Light load: as long as every group of queries that become ready at the same instant
            // finds an idle replica at that instant and fits one batch, each group is one batch started
            // at its ready time r and finished at r + L(group size).  A whole run of groups is
            // evaluated at once.  Let tau = (ready time of the first query after the run) + L(1): no
            // later batch can finish before tau.  Batches of the run that finish before tau are
            // written out right away, ordered by (completion time, query index), together with older
            // waiting batches that finish before tau; the others wait in their replica's slot like any
            // dispatched batch.  The p replicas idle at the first ready time serve the groups in turn
            // (group k takes the replica of group k-p, which must be free again by then); replicas
            // still busy are left alone.
            const uint32_t r0 = wv::uniform(rdy);
            const uint64_t idle0 = REP & wv::ballot(rend <= r0);
            const uint64_t E0 = idle0 & wv::ballot(rcnt > 0);
            if (E0 && !scan_emit(op, lslots, E0, rend, rcnt, rslot, out, omask, wr, space, progress, tw)) break;
            EST_CHK_ORDER(5);
            const uint32_t pidle = popc64(idle0);  // idle now: a prefix of the sorted table
            uint32_t m = 0;
            if (pidle > 0) {
                uint32_t *lend = ltab, *lg = ltab + 64, *luns = ltab + 128;  // per group: end, size, waits
                // groups: queries with the same ready time, cut into pieces of B (a piece of B queries is
                // a full batch; the queries of a run are in query-index order, so piece j holds its
                // members j*B .. j*B+B-1, as the queue would hand them out)
                const uint32_t rprev = wv::shr1(rdy);
                const uint64_t WM = lanes_below(w);
                const uint64_t runs = WM & (wv::ballot(rdy != rprev) | 1ull);
                // first lane of every run through LDS (run r starts at lstart[r]; lstart[number of runs] = w)
                const uint32_t nruns = popc64(runs);
                const uint32_t rid = wv::rank_below(runs >> 1);  // my run (lane 0 always starts one)
                if (ln < w && (ln == 0 || rdy != rprev)) lstart[rid] = ln;
                if (ln == 0) lstart[nruns] = w;
                wv::sync_lds();
                uint64_t heads = runs;
                uint32_t bid = rid, start = lstart[rid], nh = lstart[rid + 1u];
                const uint32_t rlen = ln < nruns ? lstart[ln + 1u] - lstart[ln] : 0u;
                if (wv::ballot(rlen > B)) {
                    // some run is longer than a batch: cut the runs into pieces of B
                    const uint64_t upto = lanes_below(wv::opaque(ln) + 1u);
                    const uint32_t off = ln - start;
                    heads = WM & wv::ballot(off == B * ((off * inv_b) >> 16));  // first query of each group
                    bid = popc64(heads & upto) - 1u;                               // group index of this lane
                    start = 63u - (uint32_t)__builtin_clzll(heads & upto);
                    const uint64_t later = ln == 63 ? 0ull : (heads >> (ln + 1));
                    nh = later ? ln + 1 + ctz64(later) : w;                        // where the next group starts
                }
                const uint32_t g = nh - start;
                const bool final = staged <= 64 && rraw == in.wr && in.fin;
                const uint32_t e = sat_add(rdy, wv::shfl(Lmine, g - 1));       // (L is 0 beyond B: rejected below)
                uint32_t *lrdy = ltab + 192;                                   // per group: ready time
                if (ln < w && ln == start) { lend[bid] = e; lg[bid] = g; lrdy[bid] = rdy; }
                wv::sync_lds();
                // replicas that serve the run: the table's first p entries, each free by the time its turn
                // comes (group l takes entry l); later groups take the replica of the group p before them
                const uint32_t ngroups = popc64(heads);
                const uint64_t usable = REP & lanes_below(ngroups) & wv::ballot(rend <= lrdy[ln < ngroups ? ln : 0]);
                const uint32_t p = usable == ~0ull ? 64u : ctz64(~usable);     // >= 1: entry 0 is idle now
                // no new completion time may equal an older waiting one (older ones that tie with each other are
                // merged by query index when they leave)
                const uint64_t busyp = wv::ballot(rcnt > 0);  // all of these end after r0
                uint64_t okm = WM & wv::ballot(e != 0xFFFFFFFFu) & wv::ballot(g <= B);  // (a clamped time never passes)
                if (busyp) {
                    // (one search over the table per lane; an entry that no longer holds members counts as well, which
                    // only ends the run early)
                    const uint32_t pos = lanes_less(rend, e, false, tw);  // the first table lane that is free no earlier than e
                    okm &= ~wv::ballot(wv::shfl(rend, pos & 63u) == e && pos < 64u);
                }
                okm &= final ? ~0ull : (wv::ballot(nh < w) | wv::ballot(g == B));                    // the whole group is in view (or it is full)
                okm &= wv::ballot(bid < p) | wv::ballot(lend[bid >= p ? bid - p : 0u] <= rdy);     // its replica is free again
                m = okm == ~0ull ? 64u : ctz64(~okm);                    // (a group is accepted or rejected as a whole)
                if (m > 0) {
                    // the next batch starts no earlier than the next query's ready time; if the run took
                    // the whole window, that is at least the window's last ready time
                    bool tau_inf = m >= w && final;                      // nothing follows at all
                    uint32_t tau = tau_inf ? 0xFFFFFFFFu : wv::sat_add_uniform(wv::bcast(rdy, umin(m, w - 1u)), L1);
                    uint64_t safem = lanes_below(m) & (tau_inf ? ~0ull : wv::ballot(e < tau));
                    if (safem != lanes_below(m)) {
                        // Some batch of the run would have to wait.  Waiting batches cost slot traffic and
                        // weaving in the steps that follow; if the run up to the first of them is long and
                        // nothing in it has to wait once the run ends there, stop the run there: the rest is
                        // looked at again with more of the input in view.
                        const uint32_t m2 = ctz64(~safem);               // (the first query of its group)
                        if (m2 >= 16) {
                            const uint32_t tau2 = wv::sat_add_uniform(wv::bcast(rdy, m2), L1);
                            if ((lanes_below(m2) & ~wv::ballot(e < tau2)) == 0) {
                                m = m2;
                                tau = tau2;
                                tau_inf = false;
                                safem = lanes_below(m2);
                            }
                        }
                    }
                    const bool safe = ln < m && (tau_inf || e < tau);
                    const uint32_t ns = popc64(safem);
                    // older waiting batches that finish before tau go out with the run (the table is in order of
                    // time: the rest finish later and keep waiting)
                    const uint64_t woven = tau_inf ? busyp : busyp & wv::ballot(rend < tau);
                    const uint32_t extra = woven ? wv::sum_u32(wv::lane_in(woven) ? rcnt : 0u) : 0u;
                    if (ns + extra > space) {
                        m = 0;  // leave it to the general path (or to the consumer)
                    } else {
                        // order the run's own output: usually already ordered
                        uint64_t key = safe ? (((uint64_t)e << 32) | q) : ~0ull;
                        // completion times that never decrease along the run, with query indices ascending where they are
                        // equal: already in output order.  (Measured: where this test fails, an exact test over the safe
                        // queries alone fails as well, so none is made.)
                        const uint32_t eprev1 = wv::shr1(e);
                        const uint32_t qprev = wv::shr1(q);
                        const uint64_t inv = lanes_below(m) & ~1ull & (wv::ballot(eprev1 > e) | (wv::ballot(eprev1 == e) & wv::ballot(qprev > q)));
                        uint32_t orank = wv::rank_below(safem);
                        if (inv) {
                            key = sort_time_query(e, q, safem, r0);
                            orank = ln;
                        }
                        const bool emit_me = inv ? ln < ns : safe;
                        const uint64_t emitm = inv ? lanes_below(ns) : safem;
                        weave_all(op, lslots, lrdy, woven, extra, emit_me, emitm, orank, ns, key, rend, rcnt, rslot, out, omask, wr, tw);
                        if ((woven >> ln) & 1ull) rcnt = 0;
                        wr += ns + extra;
                        space -= ns + extra;
                        EST_CHK_ORDER(inv ? 3 : 2);
                        // the run's batches that finish at or after tau wait in the slot of their replica
                        const uint32_t inv_p = wv::uniform((uint32_t)linv[p - 1u]) + 1u;                      // floor(x / p) = x * inv_p >> 16 for x < 64
                        const uint32_t kmod = bid - p * ((bid * inv_p) >> 16);   // the replica (idle-table lane) of my group
                        const uint32_t myslot = wv::shfl(rslot, kmod);
                        const bool waits = ln < m && !safe;
                        if (waits) lslots[myslot * bm + (ln - start)] = q;
                        if (ln < m && ln == start) luns[bid] = waits ? 1u : 0u;
                        wv::sync_lds();
                        // new table: every idle replica that served a group holds its last group's completion
                        // time (and its members, if they wait); then everything is put back in order of time
                        const uint32_t nb = popc64(heads & lanes_below(m));      // groups accepted
                        uint32_t cend = rend, ccnt = rcnt, cslot = rslot;
                        if (ln < p && ln < nb) {
                            const uint32_t x = nb - 1u - ln;
                            const uint32_t klast = ln + p * ((x * inv_p) >> 16);
                            cend = lend[klast];
                            ccnt = luns[klast] ? lg[klast] : 0u;
                        }
                        // back in order of time: sort (time since r0, lane) pairs -- entries idle at r0 count
                        // as 0 and keep their order -- and fetch each entry from the lane it was in
                        const uint32_t dl = cend > r0 ? cend - r0 : 0u;
                        if ((REP & wv::ballot(dl >= (1u << 26))) == 0) {
                            uint32_t width = 2;
                            while (width < R) width <<= 1;
                            const uint32_t from = sort_lanes(isrep ? ((dl << 6) | ln) : 0xFFFFFFFFu, width) & 63u;
                            const uint32_t se = wv::shfl(cend, from), sc = wv::shfl(ccnt, from), ss = wv::shfl(cslot, from);
                            if (isrep) { rend = se; rcnt = sc; rslot = ss; }
                        } else {
                            uint32_t trank = 0;
                            for (uint32_t j = 0; j < R; ++j) {
                                const uint32_t ej = wv::bcast(cend, j);
                                if (ej < cend || (ej == cend && j < ln)) ++trank;
                            }
                            wv::sync_lds();  // (the per-group values in this area have been read)
                            if (isrep) { ltab[trank] = cend; ltab[64 + trank] = ccnt; ltab[128 + trank] = cslot; }
                            wv::sync_lds();
                            if (isrep) { rend = ltab[ln]; rcnt = ltab[64 + ln]; rslot = ltab[128 + ln]; }
                            wv::sync_lds();
                        }
                        lhead += m;
                        progress = true;
                    }
                }
            }
            ++d_fp; d_fpe += m;
            if (DIAG && m > 0) d_tk[1] += wv::ticks() - tk0;
            if (m < 3) fp_skip = 6;  // not the regime for this shortcut: leave it alone for a few batches
            if (m > 0) continue;
            if (space == 0) break;
        }
        if (fp_skip) --fp_skip;
        if (sat_skip) --sat_skip;
        if (B >= 2 && mono && L1 > 0 && blk_skip == 0 && w >= 4) {
            // A block of batches: the batch-by-batch recurrence (start = max(earliest free replica,
            // first ready time), members = those ready by then, up to B) needs only scalars and one
            // vector compare per batch, so it is run ahead for as many batches as the window decides,
            // on a copy of the table; emission, slots and the new table are then done once for the
            // whole block, with the same rule as the light-load step: whatever finishes before
            // tau = (earliest possible next start) + L(1) is written out now in (completion, query)
            // order, older waiting batches that finish before tau are woven in, the rest waits.  A
            // batch replaced on its replica inside the block finished by that later start, hence before tau.
            const uint64_t WM = lanes_below(w);
            const bool final = staged <= 64 && rraw == in.wr && in.fin;
            const uint64_t busyp = wv::ballot(rcnt > 0);
            // working table: free time, and packed (members waiting << 16 | batch of this block on the entry, 0xFF = none, << 8 | slot)
            uint32_t trend = rend, tinfo = (rcnt << 16) | 0xFF00u | rslot;
            uint32_t vE = 0, vP = 0;                                          // per batch (lane k): end, and slot << 16 | first lane << 8 | size
            uint64_t heads = 0;
            uint32_t a = 0, K = 0;
            uint32_t cap = 0xFFFFFFFFu;  // a new batch completes together with an older waiting one at this time: nothing from there on leaves in this step
            const uint64_t tkl = DIAG ? wv::ticks() : 0;
            const uint32_t wf = final ? 65u : w;  // a batch that is not full is decided once a query ready later is in view (or none can follow)
            // (one exit and one branch per batch: the tests are combined as integers, which keeps them on the scalar unit)
            for (uint32_t go = 1u; go;) {
                const uint32_t f = wv::uniform(trend);
                const uint32_t ti0 = wv::uniform(tinfo);
                const uint32_t T = umax(f, wv::bcast(rdy, a));
                // (lanes beyond the window hold 2^32-1: they count only when T is the horizon, and then the step ends here)
                const uint32_t ready = popc64(wv::ballot(rdy <= T));
                const uint32_t b = umin(B, ready - a);
                const uint32_t e = wv::sat_add_uniform(T, wv::bcast(Lmine, b - 1u));
                // stop: more members may still arrive | a clamped time never passes
                const uint32_t stop = wv::flag_ne_and_ge(b, B, ready, wf) | wv::flag_ge(e, 0xFFFFFFFFu);
                go = 0u;
                if (stop == 0u) {
                    // the earliest entry leaves the table, the new one goes in behind everything that ends no later (the
                    // entry that leaves is free by T < e, so it is counted; lanes beyond the table hold 2^32-1 > e)
                    const uint32_t p = popc64(wv::ballot(trend <= e)) - 1u;
                    const uint32_t slot0 = ti0 & 0xFFu;
                    uint32_t more = 1u;
                    if (wv::bcast(trend, p) == e) {
                        // completes together with an entry of the table; if that is an older batch still waiting, the pair is
                        // merged by query index when it leaves, later: nothing from this time on leaves in this step, and the
                        // block ends here (an entry taken after this would lose its slot and have to leave)
                        const uint32_t e2 = wv::opaque_uniform(e);
                        const uint64_t tiem = wv::ballot(tinfo >= 0x10000u) & wv::ballot(trend == e2);
                        const uint32_t hit = wv::flag_ne((uint32_t)tiem | (uint32_t)(tiem >> 32), 0u);
                        cap = hit ? e2 : cap;
                        more = hit ^ 1u;
                    }
                    vE = wv::set_lane(vE, e, K);
                    vP = wv::set_lane(vP, (slot0 << 16) | (a << 8) | b, K);
                    const uint32_t ne = wv::shl1_any(trend), ni = wv::shl1_any(tinfo);  // (p < 64: lane 63 is never among the lanes below p)
                    if (ln < p) {
                        trend = ne; tinfo = ni;
                    }
                    trend = wv::set_lane(trend, e, p);
                    tinfo = wv::set_lane(tinfo, (K << 8) | slot0, p);
                    heads |= 1ull << a;
                    a += b;
                    ++K;
                    go = more & wv::flag_lt(a, w);
                }
                go = wv::opaque_uniform(go);
            }
            bool done = false;
            if (DIAG) { d_blkl += wv::ticks() - tkl; d_blkk += K; }
            if (K >= 2) {
                const uint32_t f_next = wv::uniform(trend);
                bool tau_inf = final && a >= w;
                const uint32_t r_next = wv::bcast(rdy, a < w ? a : w - 1u);  // what follows is ready no earlier
                uint32_t tau = tau_inf ? 0xFFFFFFFFu : wv::sat_add_uniform(umax(f_next, r_next), L1);
                const uint32_t kb = wv::rank_below(heads >> 1);             // my batch (lane 0 starts batch 0)
                const uint32_t e = wv::shfl(vE, kb), pk = wv::shfl(vP, kb), st = (pk >> 8) & 0xFFu, myslot = pk >> 16;
                const uint64_t AM = lanes_below(a);
                if (cap != 0xFFFFFFFFu && (tau_inf || cap < tau)) {
                    tau = cap;
                    tau_inf = false;
                }
                const uint64_t safem = AM & (tau_inf ? ~0ull : wv::ballot(e < tau));
                const uint32_t nsafe = popc64(safem);
                // older waiting batches that finish before tau leave with the block (the table is in order of time).  None of
                // them completes together with a new batch that leaves now: such a pair would have set the cap.
                const uint64_t woven = tau_inf ? busyp : busyp & wv::ballot(rend < tau);
                const uint32_t extra = woven ? wv::sum_u32(wv::lane_in(woven) ? rcnt : 0u) : 0u;
                const bool safe = ln < a && (tau_inf || e < tau);
                if (nsafe + extra <= space) {
                    const uint32_t eprev = wv::shr1(e), qprev = wv::shr1(q), kprev = wv::shr1(kb);
                    uint64_t key = safe ? (((uint64_t)e << 32) | q) : ~0ull;
                    // in output order already?  (only checked when the safe queries are the leading ones)
                    const bool ordered = safem == lanes_below(nsafe) &&
                                         (safem & ~1ull & (wv::ballot(eprev > e) | (wv::ballot(eprev == e) & wv::ballot(qprev > q)))) == 0;
                    if (!ordered) key = sort_time_query(e, q, safem, wv::uniform(rdy));
                    const bool emit_me = ln < nsafe;
                    weave_all(op, lslots, ltab + 192, woven, extra, emit_me, lanes_below(nsafe), ln, nsafe, key, rend, rcnt, rslot, out, omask, wr, tw);
                    wr += nsafe + extra;
                    space -= nsafe + extra;
                    EST_CHK_ORDER(7);
                    wv::sync_lds();  // the slots of woven batches have been read: they may be written again
                    // members of batches that wait go to their replica's slot, sorted by query index
                    const uint64_t waitm = AM & ~safem;
                    uint32_t qs = q;
                    if (waitm & ~1ull & wv::ballot(kprev == kb) & wv::ballot(qprev > q))
                        qs = (uint32_t)sort_lanes64(ln < a ? (((uint64_t)kb << 32) | q) : ~0ull);
                    if (ln < a && !safe) lslots[myslot * bm + (ln - st)] = qs;
                    // the working table becomes the table: older entries written out lose their members,
                    // entries of this block keep theirs if they wait
                    const uint32_t tk = (tinfo >> 8) & 0xFFu;
                    const uint32_t bsz = wv::shfl(vP, tk) & 0xFFu;
                    const bool late = !tau_inf && trend >= tau;
                    if (isrep) {
                        rend = trend;
                        rslot = tinfo & 0xFFu;
                        rcnt = tk == 0xFFu ? (late ? tinfo >> 16 : 0u) : (late ? bsz : 0u);
                    }
                    wv::sync_lds();
                    lhead += a;
                    ++d_blk; d_blke += a;
                    if (DIAG) d_tk[3] += wv::ticks() - tk0;
                    progress = true;
                    done = true;
                }
            }
            if (done) continue;
            blk_skip = 4;
        } else if (blk_skip) {
            --blk_skip;
        }
        ++d_gen;
        const uint32_t f = wv::uniform(rend);  // earliest free replica = lane 0
        const uint32_t r0 = wv::uniform(rdy);
        const uint32_t T = umax(f, r0);  // dispatch time of the next batch
        const uint64_t mm = lanes_below(umin(w, B)) & wv::ballot(rdy <= T);
        const uint32_t b = popc64(mm);
        EST_CHECK(b >= 1 && mm == lanes_below(b));
        // The batch is known once it is full, or a later query is seen to be ready only after T,
        // or no further input can come.  (Fewer than 64 staged means the source is drained.)
        const bool decidable = (b == B) || (b < w) || in.fin;
        if (!decidable) break;
        // everything that completes by T leaves before this batch is dispatched
        const uint64_t E = wv::ballot(rcnt > 0) & wv::ballot(rend <= T);
        if (E && !scan_emit(op, lslots, E, rend, rcnt, rslot, out, omask, wr, space, progress, tw)) break;
        EST_CHK_ORDER(4);
        // members wait in the replica's slot sorted by query index
        if (b > 1) {
            const uint32_t prev = wv::shr1(q);
            if (lanes_below(b) & ~1ull & wv::ballot(q < prev)) {
                uint32_t width = 2;
                while (width < b) width <<= 1;
                q = sort_lanes(ln < b ? q : 0xFFFFFFFFu, width);
            }
        }
        const uint32_t slot = wv::uniform(rslot);  // the earliest free replica takes the batch
        EST_CHECK(wv::uniform(rcnt) == 0 && slot < op.r_max);
        if (ln < b) lslots[slot * bm + ln] = q;
        const uint32_t end = wv::sat_add_uniform(T, wv::bcast(Lmine, b - 1));
        // drop lane 0 from the table and insert the new entry so that the table stays sorted
        const uint32_t p = popc64(REP & ~1ull & wv::ballot(rend <= end));
        const uint32_t nend = wv::shl1(rend), ncnt = wv::shl1(rcnt), nslot = wv::shl1(rslot);
        if (ln < p) {
            rend = nend; rcnt = ncnt; rslot = nslot;
        } else if (ln == p) {
            rend = end; rcnt = b; rslot = slot;
        }
        lhead += b;
        d_gene += b;
        if (DIAG) d_tk[5] += wv::ticks() - tk0;
        progress = true;
    }

    if (DIAG && c.a->dbg_ticks && ln == 0) {
        uint64_t *pc = est_dbg_rec(c.a, c.t, s);  // per candidate and stage (one writer: no atomics)
        pc[0] += d_gen; pc[2] += d_fp + d_b1 + d_sat + d_blk + d_lean; pc[3] += d_fpe + d_b1e + d_sate + d_hz + d_blke + d_leane;
        pc[4] += d_leane; pc[5] += d_fpe; pc[6] += d_b1e; pc[7] += d_blke;
        for (uint32_t i = 0; i < 6; ++i) pc[8 + i] += d_tk[i];
        pc[14] += d_blkl; pc[15] += d_blkk;
        uint64_t *po = est_dbg_rec(c.a, c.t, EST_MAX_STAGES - 1);
        po[6] += 1; po[7] += d_gene;
    }
    // back to memory: the table, the members still waiting, the cursors
    if (isrep) {
        g_end[ln] = rend;
        g_cnt[ln] = rcnt;
        g_slot[ln] = rslot;
    }
    for (uint64_t m = wv::ballot(rcnt > 0); m; m &= m - 1) {
        const uint32_t l = ctz64(m);
        const uint32_t cn = wv::bcast(rcnt, l), sl = wv::bcast(rslot, l);
        if (ln < cn) g_slots[sl * bm + ln] = lslots[sl * bm + ln];
    }
    // Staged but unconsumed queries are read again next time: the read cursor goes back to the first of
    // them.  Without a filter that is simply their number of places back; with one, the source is walked
    // backwards, a window at a time, until that many accepted queries have been passed.
    uint32_t cursor = rraw;
    {
        uint32_t need = ltail - lhead;
        if (!op.filtered) {
            cursor = rraw - need;
        } else {
            while (need > 0) {
                const uint32_t wb = umin(64u, cursor - rd_entry);  // (never back beyond where this call started)
                EST_CHECK(wb > 0);
                const uint32_t from = cursor - wb;
                const uint64_t kb = ln < wb ? in.base[(from + ln) & in.mask] : 0ull;
                const uint64_t Ab = lanes_below(wb) & wv::ballot((acc[(uint32_t)kb] & 1u) != 0u);
                const uint32_t have = popc64(Ab);
                if (have < need) {
                    need -= have;
                    cursor = from;
                    continue;
                }
                // the need-th accepted query from the top of this window
                uint64_t rest = Ab;
                for (uint32_t i = have; i > need; --i) rest &= rest - 1;  // drop the accepted ones below it
                cursor = from + ctz64(rest);
                need = 0;
            }
        }
    }
    wv::sync();  // what was written to the output ring is in place before its cursor moves
    if (ln == 0) {
        st_st(&c.st[P.rd_off + op.src_edge[0]], cursor);
        st_st(&c.st[P.wr_off + op.out_ring], wr);
        if (finished) {
            st_st(&c.st[P.fin_off + op.out_ring], 1);
            c.st[P.done_off + opi] = 1;
        }
    }
    wv::sync();
    return progress;
}

// ------------------------------------------------------------------------------------------ MERGE

// Keys clamped at the horizon may appear in any order inside a stream (see scan_emit); for merging
// they are ordered by (source, staging index) instead of by query index.
EST_DEV uint64_t eff_key(uint64_t key, uint32_t j, uint32_t l) {
    return (uint32_t)(key >> 32) == 0xFFFFFFFFu ? (0xFFFFFFFF00000000ull | (uint64_t)(j << 8) | l) : key;
}

enum { MERGE_RING = 128, MERGE_GROUP = 4 };  // staged elements per source of a merge (LDS ring); sources whose loads are issued together

template <bool DIAG, bool MEMO>
EST_DEV bool merge_run(const Ctx &c, const EstOp &op, uint32_t opi) {
    const uint32_t ln = wv::lane();
    const EstPlan &P = *c.P;
    const uint32_t K = wv::uniform(op.n_src);
    const bool is_lat = wv::uniform(op.type) == EST_OP_LAT;
    const uint8_t *acc = c.a->acc + (uint64_t)op.acc_idx * c.a->acc_stride;
    uint64_t *out = nullptr;
    uint32_t omask = 0, wr, space = 0xFFFFFFFFu;
    if (is_lat) {
        wr = wv::uniform(c.st[P.miss_off + 1]);
    } else {
        const EstRing &OR = P.rings[op.out_ring];
        out = c.rings + OR.off;
        omask = wv::uniform(OR.cap_mask);
        wr = wv::uniform(c.st[P.wr_off + op.out_ring]);
        space = wv::uniform(ring_space(c, op.out_ring, wr));
    }
    uint32_t miss = 0;
    uint32_t d_rounds = 0, d_elems = 0;  // diagnostics
    bool progress = false, finished = false;

    if (K == 1 && !op.has_cnt) {
        // one source, every query fed by it alone: filter and copy, four windows of 64 at a time (their
        // loads are issued together)
        const View sv = uniform_view_of<MEMO>(c, op.src_ring[0]);
        uint32_t rc = wv::uniform(c.st[P.rd_off + op.src_edge[0]]);
        const uint32_t slo = wv::uniform(c.a->slo_us);
        for (;;) {
            if (!is_lat && space < 256u) break;  // wait for the consumer
            if (rc == sv.wr) {
                finished = sv.fin != 0;
                break;
            }
            const uint32_t left = sv.wr - rc;
            uint64_t key[4];
            uint32_t av[4], arr[4];
EST_UNROLL
            for (uint32_t u = 0; u < 4; ++u) key[u] = u * 64u + ln < left ? sv.base[(rc + u * 64u + ln) & sv.mask] : 0ull;
EST_UNROLL
            for (uint32_t u = 0; u < 4; ++u) av[u] = acc[(uint32_t)key[u]];  // (idle lanes look at query 0)
            if (is_lat) {
EST_UNROLL
                for (uint32_t u = 0; u < 4; ++u) arr[u] = c.a->arrival[(uint32_t)key[u]];
            }
EST_UNROLL
            for (uint32_t u = 0; u < 4; ++u) {
                const bool a = u * 64u + ln < left && (av[u] & 1u) != 0u;
                const uint64_t A = wv::ballot(a);
                const uint32_t pos = wr + wv::rank_below(A);
                if (a) {
                    if (is_lat) {
                        const uint32_t l = (uint32_t)(key[u] >> 32) - arr[u];
                        c.lat[c.a->lat_by_qid ? (uint32_t)key[u] : pos] = l;
                        miss += l > slo;
                    } else {
                        out[pos & omask] = key[u];
                    }
                }
                const uint32_t na = popc64(A);
                wr += na;
                if (!is_lat) space -= na;
            }
            rc += umin(left, 256u);
            progress = true;
        }
        if (ln == 0) st_st(&c.st[P.rd_off + op.src_edge[0]], rc);
    } else {
        // Several sources.  A query fed by several of them is ready at the largest of its times: of its
        // elements only the one with the largest key (time, query; equal times: the higher source) is passed
        // on.  Every accepted element leaves its time in its source's table when it is staged; an entry
        // still unset reads as the horizon.  Sources are consumed in key order, so when an element is
        // consumed every element of the same query with a smaller key has been staged already, and an
        // element whose partner is unset or larger is not the last.  No counting, no read-modify-write.
        //
        // LDS: per source a ring of MERGE_RING staged keys (uint64) | per source 64 passed-on keys (uint64) |
        // per source MERGE_RING accept masks (uint8).  The per-source scalars live in two vector registers, one
        // lane per (field, source): reading one is a lane read into a scalar register, not a trip to LDS.
        const uint32_t KS = P.max_src;
        uint64_t *rkey = c.lds;
        uint64_t *lst = c.lds + KS * MERGE_RING;
        uint8_t *racc = (uint8_t *)(lst + KS * 64);
        enum { F_RD = 0, F_WR = 8, F_FIN = 16, F_HEAD = 24, F_TAIL = 32, F_MASK = 40, F_BLO = 48, F_BHI = 56,  // va: lane = field + source
               F_NFIN = 0, F_CONS = 8 };                                                                    // vb: passed on / consumed this round
        uint32_t va = 0, vb = 0;
        const uint32_t tab_mask = wv::uniform(op.tab_mask), tab_len = wv::uniform(op.tab_len);
        uint32_t *tab0 = (uint32_t *)(c.tab + op.tab_off);
        for (uint32_t j = 0; j < K; ++j) {
            const View sv = uniform_view_of<MEMO>(c, op.src_ring[j]);
            const uint64_t bp = (uint64_t)(uintptr_t)sv.base;
            va = wv::set_lane(va, wv::uniform(c.st[P.rd_off + op.src_edge[j]]), F_RD + j);
            va = wv::set_lane(va, sv.wr, F_WR + j);
            va = wv::set_lane(va, sv.fin, F_FIN + j);
            va = wv::set_lane(va, sv.mask, F_MASK + j);
            va = wv::set_lane(va, wv::uniform((uint32_t)bp), F_BLO + j);
            va = wv::set_lane(va, wv::uniform((uint32_t)(bp >> 32)), F_BHI + j);
        }
        for (;;) {
            if (!is_lat && space < 64u * K) break;  // wait for the consumer
            // ---- refill: every source with no more than a window staged takes up to 64 further elements; the
            //      loads of all sources are issued before any is used
            bool any = false;
            for (uint32_t j0 = 0; j0 < K; j0 += MERGE_GROUP) {
                uint64_t kx[MERGE_GROUP];
                uint32_t wx[MERGE_GROUP], ax[MERGE_GROUP];
                bool some = false;
EST_UNROLL
                for (uint32_t u = 0; u < MERGE_GROUP; ++u) {
                    const uint32_t j = j0 + u;
                    wx[u] = 0;
                    kx[u] = 0;
                    if (j < K) {
                        const uint32_t staged = wv::bcast(va, F_TAIL + j) - wv::bcast(va, F_HEAD + j);
                        const uint32_t rd = wv::bcast(va, F_RD + j), left = wv::bcast(va, F_WR + j) - rd;
                        if (staged <= 64u && left > 0u) {
                            const uint64_t *base = (const uint64_t *)(uintptr_t)(((uint64_t)wv::bcast(va, F_BHI + j) << 32) | wv::bcast(va, F_BLO + j));
                            const uint32_t smask = wv::bcast(va, F_MASK + j);
                            wx[u] = umin(64u, left);
                            if (ln < wx[u]) kx[u] = base[(rd + ln) & smask];
                            some = true;
                        }
                    }
                }
                if (!some) continue;
                any = true;
EST_UNROLL
                for (uint32_t u = 0; u < MERGE_GROUP; ++u) ax[u] = (wx[u] && ln < wx[u]) ? acc[(uint32_t)kx[u]] : 0u;
EST_UNROLL
                for (uint32_t u = 0; u < MERGE_GROUP; ++u) {
                    const uint32_t j = j0 + u;
                    if (!wx[u]) continue;
                    uint32_t am = ax[u];
                    if (!((am >> j) & 1u)) am = 0;  // not for this stage, or superseded by a nearer ancestor
                    if (((tab_mask >> j) & 1u) && (am & (am - 1u)))
                        tab0[(uint64_t)__builtin_popcount(tab_mask & ((1u << j) - 1u)) * tab_len + (uint32_t)kx[u]] = (uint32_t)(kx[u] >> 32);
                    const uint32_t tl = wv::bcast(va, F_TAIL + j);
                    const uint32_t at = j * MERGE_RING + ((tl + ln) & (MERGE_RING - 1u));
                    if (ln < wx[u]) {
                        rkey[at] = kx[u];
                        racc[at] = (uint8_t)am;
                    }
                    va = wv::set_lane(va, tl + wx[u], F_TAIL + j);
                    va = wv::set_lane(va, wv::bcast(va, F_RD + j) + wx[u], F_RD + j);
                }
            }
            if (any) wv::sync();  // (tables and staged elements: written above, read below by other lanes)
            // ---- the window of every source: its first 64 staged elements
            uint32_t more = 0, total = 0;  // more, bit j: source j may hold elements beyond its window
            bool blocked = false, clamped = false;
            uint64_t bound = ~0ull;  // everything up to the smallest last key of a source that may hold more is final
            for (uint32_t j = 0; j < K; ++j) {
                const uint32_t h = wv::bcast(va, F_HEAD + j), staged = wv::bcast(va, F_TAIL + j) - h;
                const uint32_t w = umin(64u, staged);
                const bool has_more = staged > 64u || wv::bcast(va, F_RD + j) != wv::bcast(va, F_WR + j) || !wv::bcast(va, F_FIN + j);
                if (has_more) more |= 1u << j;
                total += w;
                if (w == 0) {
                    blocked = blocked || has_more;
                } else {
                    const uint64_t lk = rkey[j * MERGE_RING + ((h + w - 1u) & (MERGE_RING - 1u))];
                    const uint32_t tl = wv::uniform((uint32_t)(lk >> 32)), ql = wv::uniform((uint32_t)lk);
                    clamped = clamped || tl == 0xFFFFFFFFu;
                    if (has_more) {
                        const uint64_t last = eff_key(((uint64_t)tl << 32) | ql, j, w - 1u);
                        bound = last < bound ? last : bound;
                    }
                }
            }
            if (blocked || total == 0) {
                if (!blocked) finished = more == 0;
                break;
            }
            // ---- which of the consumed elements are passed on (the table look-ups of all sources are issued together)
            uint32_t n_out = 0;
            for (uint32_t j0 = 0; j0 < K; j0 += MERGE_GROUP) {
                uint64_t kx[MERGE_GROUP];
                uint32_t amx[MERGE_GROUP], t2x[MERGE_GROUP];
                bool px[MERGE_GROUP];
                uint32_t hard = 0;  // bit u: some element of the source has more than one partner
EST_UNROLL
                for (uint32_t u = 0; u < MERGE_GROUP; ++u) {
                    const uint32_t j = j0 + u;
                    kx[u] = 0; amx[u] = 0; t2x[u] = 0; px[u] = false;
                    if (j < K) {
                        const uint32_t h = wv::bcast(va, F_HEAD + j);
                        const uint32_t w = umin(64u, wv::bcast(va, F_TAIL + j) - h);
                        const uint32_t at = j * MERGE_RING + ((h + ln) & (MERGE_RING - 1u));
                        if (ln < w) { kx[u] = rkey[at]; amx[u] = racc[at]; }
                        const uint64_t x = clamped ? eff_key(kx[u], j, ln) : kx[u];
                        const bool consumed = ln < w && x <= bound;  // a prefix of the window: a source's keys ascend
                        const uint32_t mj = popc64(wv::ballot(consumed));
                        vb = wv::set_lane(vb, mj, F_CONS + j);
                        px[u] = consumed && amx[u] != 0u;
                        const uint32_t others = amx[u] & ~(1u << j);
                        if (px[u] && others != 0u) {
                            const uint32_t j2 = (uint32_t)__builtin_ctz(others);
                            t2x[u] = tab0[(uint64_t)__builtin_popcount(tab_mask & ((1u << j2) - 1u)) * tab_len + (uint32_t)kx[u]];
                        }
                        if (wv::ballot(px[u] && (others & (others - 1u)) != 0u)) hard |= 1u << u;
                    }
                }
EST_UNROLL
                for (uint32_t u = 0; u < MERGE_GROUP; ++u) {
                    const uint32_t j = j0 + u;
                    if (j < K) {
                        const uint32_t t = (uint32_t)(kx[u] >> 32);
                        const uint32_t others = amx[u] & ~(1u << j);
                        bool pass = px[u];
                        if (pass && others != 0u) {
                            const uint32_t j2 = (uint32_t)__builtin_ctz(others);
                            if (!(t2x[u] < t || (t2x[u] == t && j2 < j))) pass = false;
                        }
                        if ((hard >> u) & 1u) {  // more than two parents: the remaining partners one by one
                            for (uint32_t j2 = 0; j2 < K; ++j2) {
                                const bool need = pass && j2 != j && ((others >> j2) & 1u);
                                if (!wv::ballot(need)) continue;
                                const uint32_t t2 = need ? tab0[(uint64_t)__builtin_popcount(tab_mask & ((1u << j2) - 1u)) * tab_len + (uint32_t)kx[u]] : 0u;
                                if (need && !(t2 < t || (t2 == t && j2 < j))) pass = false;
                            }
                        }
                        const uint64_t F = wv::ballot(pass);
                        const uint32_t fr = wv::rank_below(F);
                        if (pass) lst[j * 64 + fr] = kx[u];
                        vb = wv::set_lane(vb, popc64(F), F_NFIN + j);
                        n_out += popc64(F);
                    }
                }
            }
            ++d_rounds; d_elems += n_out;
            wv::sync_lds();
            // ---- place every passed-on element: its rank in its own list plus the smaller elements of the others
            for (uint32_t j = 0; j < K; ++j) {
                const uint32_t nf = wv::bcast(vb, F_NFIN + j);
                if (nf == 0) continue;
                const bool have = ln < nf;
                const uint64_t rk = have ? lst[j * 64 + ln] : 0ull;
                uint32_t rank = ln;
                for (uint32_t j2 = 0; j2 < K; ++j2) {
                    const uint32_t n2 = wv::bcast(vb, F_NFIN + j2);
                    if (j2 == j || n2 == 0) continue;
                    const uint64_t *l2 = lst + j2 * 64;
                    const uint32_t top = 1u << (31u - (uint32_t)__builtin_clz(n2));  // the largest power of two within the list
                    uint32_t lo = 0;  // elements of list j2 below rk (no two lists hold the same key: one element per query is passed on)
                    if (!clamped) {
                        for (uint32_t step = top; step >= 1; step >>= 1) {
                            const uint32_t i = lo + step;
                            const bool in = i <= n2;
                            const uint64_t y = l2[in ? i - 1u : 0u];
                            if (in && y < rk) lo = i;
                        }
                    } else {
                        const uint64_t x = eff_key(rk, j, ln);
                        for (uint32_t step = top; step >= 1; step >>= 1) {
                            const uint32_t i = lo + step;
                            const bool in = i <= n2;
                            const uint64_t y = eff_key(l2[in ? i - 1u : 0u], j2, in ? i - 1u : 0u);
                            if (in && y < x) lo = i;
                        }
                    }
                    rank += lo;
                }
                if (have) {
                    const uint32_t pos = wr + rank;
                    if (is_lat) {
                        const uint32_t q = (uint32_t)rk;
                        const uint32_t l = (uint32_t)(rk >> 32) - c.a->arrival[q];
                        c.lat[c.a->lat_by_qid ? q : pos] = l;
                        miss += l > c.a->slo_us;
                    } else {
                        out[pos & omask] = rk;
                    }
                }
            }
            wr += n_out;
            if (!is_lat) space -= n_out;  // (nobody consumes while this operation runs)
            for (uint32_t j = 0; j < K; ++j) va = wv::set_lane(va, wv::bcast(va, F_HEAD + j) + wv::bcast(vb, F_CONS + j), F_HEAD + j);
            progress = true;
            wv::sync_lds();
        }
        // staged but not consumed: read again next time
        for (uint32_t j = 0; j < K; ++j) {
            const uint32_t back = wv::bcast(va, F_RD + j) - (wv::bcast(va, F_TAIL + j) - wv::bcast(va, F_HEAD + j));
            if (ln == 0) st_st(&c.st[P.rd_off + op.src_edge[j]], back);
        }
    }

    if (DIAG && c.a->dbg_ticks && ln == 0) { uint64_t *po = est_dbg_rec(c.a, c.t, EST_MAX_STAGES - 1); po[3] += d_rounds; po[4] += d_elems; po[5] += 1; }
    const uint32_t miss_all = is_lat ? wv::sum_u32(miss) : 0u;
    wv::sync();  // what was written to the output ring is in place before its cursor moves
    if (ln == 0) {
        if (is_lat) {
            c.st[P.miss_off + 1] = wr;
            c.st[P.miss_off] += miss_all;
        } else {
            st_st(&c.st[P.wr_off + op.out_ring], wr);
        }
        if (finished) {
            if (!is_lat) st_st(&c.st[P.fin_off + op.out_ring], 1);
            c.st[P.done_off + opi] = 1;
        }
    }
    wv::sync();
    return progress;
}

// ------------------------------------------------------------------------------------------ driver

// One wavefront = one candidate.  Every loop ends: an operation that consumes or emits nothing
// reports no progress, and a full pass over the operations without progress stops the candidate with
// an error flag.
EST_DEV Ctx make_ctx(const EstSimArgs &a, uint32_t t, uint32_t slot, uint64_t *lds) {
    Ctx c;
    c.a = &a;
    c.P = a.plan;
    c.st = a.state + (uint64_t)slot * a.state_stride;
    c.rings = a.rings + (uint64_t)slot * a.ring_stride;
    c.rep = a.rep + (uint64_t)slot * a.rep_stride;
    c.slots = a.slots + (uint64_t)slot * a.slot_stride;
    c.tab = a.tabs + (uint64_t)slot * a.tab_stride;
    c.lat = a.lat + (uint64_t)(a.lat_by_qid ? t : slot) * a.lat_stride;
    c.cfg = a.cfg + (uint64_t)t * a.dag->S;
    c.lds = lds;
    c.t = t;
    c.memo_rings = 0;
    c.cap_rings = nullptr;
    return c;
}

// A candidate's scratch before its first operation: cursors and flags zero, every replica idle at t = 0 and
// owning one slot, no element of any joined stream looked at yet.
EST_DEV void sim_init(const EstSimArgs &a, const Ctx &c) {
    const uint32_t ln = wv::lane();
    const EstPlan &P = *c.P;
    for (uint32_t i = ln; i < P.state_words; i += 64) c.st[i] = 0;
    for (uint64_t i = ln; i < a.rep_stride; i += 64) c.rep[i] = 0;
    wv::sync();
    for (uint32_t opi = 0; opi < P.n_ops; ++opi) {
        const EstOp &op = P.ops[opi];
        if (op.type == EST_OP_SCAN && ln < op.r_max) c.rep[op.rep_off + 2 * op.r_max + ln] = ln;
    }
    {
        uint32_t *tw = (uint32_t *)c.tab;
        for (uint64_t i = ln; i < a.tab_stride / 4; i += 64) tw[i] = 0xFFFFFFFFu;
    }
    wv::sync();
}

// One wavefront = one candidate.  Every loop ends: an operation that consumes or emits nothing
// reports no progress, and a full pass over the operations without progress stops the candidate with
// an error flag.
template <bool DIAG, bool MEMO>
EST_DEV void sim_wave(const EstSimArgs &a, uint32_t t, uint32_t slot, uint64_t *lds) {
    const uint32_t ln = wv::lane();
    const EstPlan &P = *a.plan;
    Ctx c = make_ctx(a, t, slot, lds);
    sim_init(a, c);
    c.memo_rings = 0;
    c.cap_rings = nullptr;
    if (MEMO) {
        // Operations this candidate does not run count as done.  In a replay the streams they would have
        // produced are complete already in the captured run of the candidate's base: point the readers
        // there and preset the write cursors to the captured lengths.
        const uint64_t skip = a.skip_ops[t];
        const bool replay = a.cap_rings != nullptr;
        const uint32_t b = replay ? a.base_of[t] : 0u;
        const uint32_t *cs = replay ? a.cap_state + (uint64_t)b * a.cap_state_stride : nullptr;
        if (replay) c.cap_rings = a.cap_rings + (uint64_t)b * a.cap_ring_stride;
        uint64_t mr = 0;
        for (uint32_t opi = 0; opi < P.n_ops; ++opi) {
            if (!((skip >> opi) & 1ull)) continue;
            const int32_t r = P.ops[opi].out_ring;
            if (ln == 0) c.st[P.done_off + opi] = 1;
            if (replay && r >= 0) {
                mr |= 1ull << r;
                if (ln == 0) {
                    c.st[P.wr_off + r] = cs[P.wr_off + r];
                    c.st[P.fin_off + r] = 1;
                }
            }
        }
        c.memo_rings = mr;
        wv::sync();
    }

    for (;;) {
        bool progress = false, alldone = true;
        for (uint32_t opi = 0; opi < P.n_ops; ++opi) {
            if (wv::uniform(c.st[P.done_off + opi])) continue;
            const EstOp &op = P.ops[opi];
            const uint64_t k0 = (DIAG && a.dbg_ticks) ? wv::ticks() : 0;
            bool p = op.type == EST_OP_SCAN ? scan_run<DIAG, MEMO>(c, op, opi) : merge_run<DIAG, MEMO>(c, op, opi);
            if (DIAG && a.dbg_ticks && ln == 0) {
                const uint64_t dt = wv::ticks() - k0;
                if (op.type == EST_OP_SCAN) est_dbg_rec(&a, t, op.stage)[1] += dt;
                else est_dbg_rec(&a, t, EST_MAX_STAGES - 1)[op.type == EST_OP_LAT ? 1 : 0] += dt;
            }
            progress = progress || p;
            alldone = alldone && wv::uniform(c.st[P.done_off + opi]) != 0;
        }
        if (alldone) break;
        if (!progress) {
            if (ln == 0) a.status->sim_error = 1;
            break;
        }
    }
}

// Several wavefronts per candidate (for calls with fewer candidates than the device has room for: the time
// of such a call is the time of one simulation, Section 4.2).  The operations of the candidate are dealt out
// to the wavefronts of a workgroup (EstOp::owner), which then run as a pipeline: streams between operations of
// different wavefronts are the same rings, their cursors read and written through ld_st / st_st.  One call =
// one pass of wavefront `wave` over its own operations.  Returns bit 0: progress, bit 1: all of them are done.
EST_DEV void mw_init(const EstSimArgs &a, uint32_t t, uint32_t slot) {
    const Ctx c = make_ctx(a, t, slot, nullptr);
    sim_init(a, c);
}

EST_DEV uint32_t mw_pass(const EstSimArgs &a, uint32_t t, uint32_t slot, uint64_t *lds, uint32_t wave) {
    const EstPlan &P = *a.plan;
    const Ctx c = make_ctx(a, t, slot, lds);
    bool progress = false, alldone = true;
    for (uint32_t opi = 0; opi < P.n_ops; ++opi) {
        const EstOp &op = P.ops[opi];
        if (wv::uniform(op.owner) != wave) continue;
        if (wv::uniform(c.st[P.done_off + opi])) continue;  // (written by this wavefront only)
        const bool p = op.type == EST_OP_SCAN ? scan_run<false, false>(c, op, opi) : merge_run<false, false>(c, op, opi);
        progress = progress || p;
        alldone = alldone && wv::uniform(c.st[P.done_off + opi]) != 0;
    }
    return (progress ? 1u : 0u) | (alldone ? 2u : 0u);
}

// ------------------------------------------------------------------------------------------ P99

// Nearest-rank P99 of one candidate's latencies by a 4-pass radix select (8 bits per pass), one
// wavefront per candidate, plus the candidate's cost = sum over stages of replicas x price
// (Section 6, cost model).
EST_DEV void select_wave(const EstSimArgs &a, uint32_t t, uint32_t slot, uint64_t *lds) {
    const uint32_t ln = wv::lane();
    const EstStageCfg *cfg = a.cfg + (uint64_t)t * a.dag->S;
    if (ln == 0) {
        uint64_t cost = 0;
        for (uint32_t s = 0; s < a.dag->S; ++s)
            cost += (uint64_t)cfg[s].replicas * a.cost_uusd_hr[(uint64_t)s * a.dag->H + cfg[s].hw];
        a.cost[t] = cost;
    }
    if (!a.have_lat) return;
    const uint32_t *lat = a.lat + (uint64_t)slot * a.lat_stride;
    uint32_t *hist = (uint32_t *)lds;  // 256 bins
    const uint32_t n = a.n;
    uint32_t k = (uint32_t)(((uint64_t)99 * n + 99) / 100);  // 1-based rank, ceil(0.99 n)
    uint32_t prefix = 0;
    for (int pass = 3; pass >= 0; --pass) {
        const uint32_t shift = (uint32_t)pass * 8;
        for (uint32_t i = ln; i < 256; i += 64) hist[i] = 0;
        wv::sync_lds();
        for (uint32_t i0 = 0; i0 < n; i0 += 512) {  // eight loads in flight per lane
            uint32_t v[8];
EST_UNROLL
            for (uint32_t u = 0; u < 8; ++u) {
                const uint32_t i = i0 + u * 64u + ln;
                v[u] = i < n ? lat[i] : 0u;
            }
EST_UNROLL
            for (uint32_t u = 0; u < 8; ++u) {
                const bool match = i0 + u * 64u + ln < n && (pass == 3 || (v[u] >> (shift + 8)) == (prefix >> (shift + 8)));
                if (match) wv::lds_add(&hist[(v[u] >> shift) & 255u], 1u);
            }
        }
        wv::sync_lds();
        // lane l owns bins 4l .. 4l+3
        const uint32_t h0 = hist[4 * ln], h1 = hist[4 * ln + 1], h2 = hist[4 * ln + 2], h3 = hist[4 * ln + 3];
        const uint32_t mine = h0 + h1 + h2 + h3;
        const uint32_t before = wv::prefix_excl_u32(mine);
        const uint64_t hit = wv::ballot(before < k && k <= before + mine);
        EST_CHECK(popc64(hit) == 1);
        const uint32_t hl = ctz64(hit);
        uint32_t digit = 0, kk = 0;
        if (ln == hl) {
            uint32_t r = k - before;  // rank inside my four bins
            if (r <= h0) { digit = 4 * ln; kk = r; }
            else if (r <= h0 + h1) { digit = 4 * ln + 1; kk = r - h0; }
            else if (r <= h0 + h1 + h2) { digit = 4 * ln + 2; kk = r - h0 - h1; }
            else { digit = 4 * ln + 3; kk = r - h0 - h1 - h2; }
        }
        digit = wv::bcast(digit, hl);
        k = wv::bcast(kk, hl);
        prefix |= digit << shift;
        wv::sync_lds();
    }
    if (ln == 0) {
        a.p99[t] = prefix;
        a.miss[t] = a.state[(uint64_t)slot * a.state_stride + a.plan->miss_off];
    }
}

// A wavefront takes candidates from the launch's work counter until none is left, simulating each
// in its own scratch slot and, unless per-query latencies were asked for, selecting the P99 right
// away from the slot's latency array.
template <bool DIAG, bool MEMO>
EST_DEV void slot_loop(const EstSimArgs &a, uint32_t wave_slot, uint64_t *lds) {
    for (;;) {
        uint32_t t = 0;
        if (wv::lane() == 0) t = wv::fetch_add_u32(&a.status->next_cfg, 1u);
        t = wv::bcast(t, 0);
        if (t >= a.n_cfg) break;
        if (MEMO && a.order) t = a.order[t];
        const uint32_t slot = (MEMO && a.slot_by_cfg) ? t : wave_slot;
        const uint64_t t0 = (DIAG && a.dbg_ticks) ? wv::ticks() : 0;
        if (a.n > 0) sim_wave<DIAG, MEMO>(a, t, slot, lds);
        wv::sync();
        const uint64_t k1 = (DIAG && a.dbg_ticks) ? wv::ticks() : 0;
        if (!a.lat_by_qid) select_wave(a, t, slot, lds);
        wv::sync();
        if (DIAG && a.dbg_ticks && wv::lane() == 0) est_dbg_rec(&a, t, EST_MAX_STAGES - 1)[2] += wv::ticks() - k1;
        if (DIAG && a.dbg_ticks && wv::lane() == 0) a.dbg_ticks[t] = wv::ticks() - t0;
    }
}

// ------------------------------------------------------------------------------------------ preprocessing

// Nearest visited ancestors of every stage (and of the virtual sink, index S) for one query:
// bit p = the completion of stage p feeds the stage directly, bit EST_TRACE_BIT = the arrival does.
// A member that is an ancestor of another member is left out: times never decrease along a path of the
// pipeline (a skipped stage passes its ready time on), so its completion is no later than the other's and never
// decides the maximum (Section 4.1, conditional control flow: a query that takes one branch of a fork and skips
// the other is fed by that branch alone, not also by the stage before the fork).
EST_DEV void nearest_sets(const EstDag &d, uint32_t mask, uint64_t *nv) {
    uint64_t anc[EST_MAX_STAGES + 1];  // every ancestor of the stage, and the arrival
    for (uint32_t c = 0; c <= d.S; ++c) {
        uint64_t s = 0, a = 1ull << EST_TRACE_BIT;
        const uint32_t b = d.parent_off[c], e = d.parent_off[c + 1];
        if (b == e) s = 1ull << EST_TRACE_BIT;
        for (uint32_t i = b; i < e; ++i) {
            const uint32_t p = d.parent_idx[i];
            s |= ((mask >> p) & 1u) ? (1ull << p) : nv[p];
            a |= (1ull << p) | anc[p];
        }
        uint64_t dominated = 0;
        for (uint64_t t = s & ~(1ull << EST_TRACE_BIT); t; t &= t - 1) dominated |= anc[__builtin_ctzll(t)];
        nv[c] = s & ~dominated;
        anc[c] = a;
    }
}

// Pass 1 over the trace (thread tid of nthreads, strided): monotonicity, per-stage source unions,
// visit counts.
EST_DEV void prep1_thread(const EstPrepArgs &a, uint32_t tid, uint32_t nthreads) {
    const EstDag &d = *a.dag;
    uint64_t uni[EST_MAX_STAGES + 1], muni[EST_MAX_STAGES + 1];
    uint32_t cntv[EST_MAX_STAGES + 1];
    uint64_t multi = 0;  // bit c: some visiting query of stage c has more than one nearest visited ancestor
    bool bad = false;
    for (uint32_t c = 0; c <= d.S; ++c) { uni[c] = 0; muni[c] = 0; cntv[c] = 0; }
    for (uint64_t q = tid; q < a.n; q += nthreads) {
        const uint32_t m = a.mask[q];
        if (q > 0 && a.arrival[q] < a.arrival[q - 1]) bad = true;
        uint64_t nv[EST_MAX_STAGES + 1];
        nearest_sets(d, m, nv);
        for (uint32_t c = 0; c <= d.S; ++c) {
            if (c < d.S && !((m >> c) & 1u)) continue;
            uni[c] |= nv[c];
            cntv[c]++;
            if (__builtin_popcountll(nv[c]) > 1) {
                multi |= 1ull << c;
                muni[c] |= nv[c];
            }
        }
    }
    for (uint32_t c = 0; c <= d.S; ++c) {
        if (cntv[c]) {
            wv::atomic_or_u64(&a.status->src_union[c], uni[c]);
            wv::atomic_add_u32(&a.status->n_visit[c], cntv[c]);
            if ((multi >> c) & 1ull) {
                wv::atomic_or_u32(&a.status->multi[c], 1u);
                wv::atomic_or_u64(&a.status->multi_union[c], muni[c]);
            }
        }
    }
    if (bad) wv::atomic_or_u32(&a.status->bad_trace, 1u);
    if (tid == 0 && a.n > 0) a.status->last_arrival = a.arrival[a.n - 1];
}

// Pass 2: the key stream of the trace, and for every merge operation the per-query accept mask:
// bit j set = source j of the operation is one of the query's nearest visited ancestors.
EST_DEV void prep2_thread(const EstPrepArgs &a, uint32_t tid, uint32_t nthreads) {
    const EstDag &d = *a.dag;
    for (uint64_t q = tid; q < a.n; q += nthreads) {
        const uint32_t m = a.mask[q];
        a.trace_keys[q] = ((uint64_t)a.arrival[q] << 32) | q;
        uint64_t nv[EST_MAX_STAGES + 1];
        nearest_sets(d, m, nv);
        for (uint32_t i = 0; i < a.n_acc; ++i) {
            const uint32_t c = a.acc_stage[i];
            uint8_t bits = 0;
            if (c == d.S || ((m >> c) & 1u)) {
                for (uint64_t s = nv[c]; s; s &= s - 1) {
                    const uint32_t src = (uint32_t)__builtin_ctzll(s);
                    bits |= (uint8_t)(1u << a.acc_slot_of_src[c][src]);
                }
            }
            a.acc[(uint64_t)i * a.acc_stride + q] = bits;
        }
    }
}

// Range check of every configuration entry and the per-stage maxima that size the scratch.
EST_DEV void cfg_thread(const EstCfgArgs &a, uint32_t tid, uint32_t nthreads) {
    const EstDag &d = *a.dag;
    uint32_t rmax[EST_MAX_STAGES], bmax[EST_MAX_STAGES];
    bool bad = false;
    for (uint32_t s = 0; s < d.S; ++s) { rmax[s] = 0; bmax[s] = 0; }
    for (uint64_t i = tid; i < a.n_cfg; i += nthreads) {
        for (uint32_t s = 0; s < d.S; ++s) {
            const EstStageCfg e = a.cfg[i * d.S + s];
            if (e.hw >= d.H || e.batch < 1 || e.batch > d.Bmax || e.replicas < 1 || e.replicas > EST_MAX_REPLICAS) bad = true;
            rmax[s] = umax(rmax[s], e.replicas);
            bmax[s] = umax(bmax[s], e.batch);
        }
    }
    for (uint32_t s = 0; s < d.S; ++s) {
        if (rmax[s]) wv::atomic_max_u32(&a.status->r_max[s], rmax[s]);
        if (bmax[s]) wv::atomic_max_u32(&a.status->b_max[s], bmax[s]);
    }
    if (bad) wv::atomic_or_u32(&a.status->bad_cfg, 1u);
}

// Traffic envelope of the trace (Section 5, "traffic envelopes"): for every window width the largest
// number of arrivals in any half-open window [t, t + width).  The maximum is attained by a window
// that starts at an arrival.  Thread tid (of nthreads) takes a run of consecutive queries; for the
// first it finds, per width, the first arrival at or after arrival[j] + width (the widths ascend, so
// each search starts where the previous one ended: gallop, then bisect); for the following queries
// the window ends only move forward, a step at a time.
EST_DEV void envelope_thread(const EstEnvArgs &a, uint32_t tid, uint32_t nthreads) {
    const uint64_t chunk = (a.n + nthreads - 1) / nthreads;
    const uint64_t j0 = (uint64_t)tid * chunk, j1 = j0 + chunk < a.n ? j0 + chunk : a.n;
    if (j0 >= j1) return;
    uint32_t best[EST_MAX_WINDOWS], end[EST_MAX_WINDOWS];  // arrivals [j, end[i]) lie inside window i of query j
EST_UNROLL
    for (uint32_t i = 0; i < EST_MAX_WINDOWS; ++i) best[i] = end[i] = 0;
    const uint32_t n = (uint32_t)a.n;
    {
        const uint64_t t0 = a.arrival[j0];
        uint32_t e = (uint32_t)j0 + 1;
EST_UNROLL
        for (uint32_t i = 0; i < EST_MAX_WINDOWS; ++i) {
            if (i < a.n_win) {
                const uint64_t limit = t0 + a.win_us[i];
                // invariant: arrival[e - 1] < limit
                uint32_t step = 1;
                while (e + step <= n && (uint64_t)a.arrival[e + step - 1] < limit) {
                    e += step;
                    step <<= 1;
                }
                uint32_t lo = e, hi = e + step - 1 < n ? e + step - 1 : n;  // the answer is in [lo, hi]
                while (lo < hi) {
                    const uint32_t mid = lo + ((hi - lo) >> 1);
                    if ((uint64_t)a.arrival[mid] < limit) lo = mid + 1; else hi = mid;
                }
                e = lo;
                end[i] = e;
                best[i] = e - (uint32_t)j0;
            }
        }
    }
    for (uint64_t j = j0 + 1; j < j1; ++j) {
        const uint64_t t0 = a.arrival[j];
EST_UNROLL
        for (uint32_t i = 0; i < EST_MAX_WINDOWS; ++i) {
            if (i < a.n_win) {
                const uint64_t limit = t0 + a.win_us[i];
                uint32_t e = end[i];  // (> j: the window of the query before already held that query and this one's predecessor)
                if (e <= (uint32_t)j) e = (uint32_t)j + 1;
                while (e < n && (uint64_t)a.arrival[e] < limit) ++e;
                end[i] = e;
                const uint32_t cnt = e - (uint32_t)j;
                best[i] = cnt > best[i] ? cnt : best[i];
            }
        }
    }
EST_UNROLL
    for (uint32_t i = 0; i < EST_MAX_WINDOWS; ++i)
        if (i < a.n_win && best[i] > a.max_queries[i]) wv::atomic_max_u32(&a.max_queries[i], best[i]);
}

}  // namespace estdev
