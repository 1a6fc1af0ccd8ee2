// Lock-step CPU emulation of the 64-lane wavefront primitives (test infrastructure).
//
// The device code of the Estimator is written against the wv:: primitives only.  Here every lane is
// a fiber; a primitive is a rendezvous of all 64 fibers, so lanes advance in lock step between
// primitives exactly as far as the device code may rely on.  It exists to run the kernel logic on
// the host with consistency checks (EST_CHECK) enabled; it is never part of the GPU library and
// the Python binding cannot load it.
#pragma once
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#define EST_DEV static inline
#define EST_DEV_NOINLINE static
#define EST_UNROLL
#define EST_CHECK(cond)                                                                       \
    do {                                                                                      \
        if (!(cond)) {                                                                        \
            fprintf(stderr, "EST_CHECK failed: %s at %s:%d (lane %u)\n", #cond, __FILE__, __LINE__, wv::lane()); \
            abort();                                                                          \
        }                                                                                     \
    } while (0)

// Order check of a scan's output (used inside scan_run, where out, omask, wr, ln and s are in scope): after
// every step, what the step wrote must ascend by (time, query), except at the horizon.
#define EST_CHK_ORDER_INIT() uint32_t chk_wr = wr
#define EST_CHK_ORDER(tag)                                                                             \
    do {                                                                                               \
        wv::sync();                                                                                    \
        if (ln == 0)                                                                                   \
            for (uint32_t i_ = chk_wr > 0 ? chk_wr : 1; i_ < wr; ++i_) {                               \
                const uint64_t a_ = out[(i_ - 1) & omask], b_ = out[i_ & omask];                       \
                if ((uint32_t)(b_ >> 32) != 0xFFFFFFFFu && !(a_ < b_)) {                               \
                    fprintf(stderr, "order violated by path %d at out[%u]: %llx then %llx (stage %u)\n", tag, i_, (unsigned long long)a_, (unsigned long long)b_, s); \
                    abort();                                                                           \
                }                                                                                      \
            }                                                                                          \
        chk_wr = wr;                                                                                   \
    } while (0)

namespace emu {
uint32_t lane();
// all 64 lanes deposit v, then every lane may read any lane's value through the returned array
const uint64_t *exchange(uint64_t v, uint32_t tag);
}  // namespace emu

namespace wv {

EST_DEV uint32_t lane() { return emu::lane(); }

EST_DEV uint64_t ballot(bool p) {
    const uint64_t *x = emu::exchange(p ? 1 : 0, 1);
    uint64_t m = 0;
    for (int l = 0; l < 64; ++l) m |= (x[l] & 1ull) << l;
    return m;
}

EST_DEV uint32_t shfl(uint32_t v, uint32_t src) { return (uint32_t)emu::exchange(v, 2)[src & 63u]; }

EST_DEV uint32_t bcast(uint32_t v, uint32_t l) {
    const uint64_t *x = emu::exchange(((uint64_t)l << 32) | v, 3);
    for (int i = 0; i < 64; ++i)
        if ((uint32_t)(x[i] >> 32) != l) {
            fprintf(stderr, "bcast: lane index not uniform (%u vs %u)\n", (uint32_t)(x[i] >> 32), l);
            abort();
        }
    if (l >= 64) {
        fprintf(stderr, "bcast: lane %u out of range\n", l);
        abort();
    }
    return (uint32_t)x[l];
}

EST_DEV uint32_t shr1(uint32_t v) { const uint64_t *x = emu::exchange(v, 9); uint32_t l = emu::lane(); return l == 0 ? v : (uint32_t)x[l - 1]; }
// (lane 63: unspecified on the device; a value here that a wrong use would trip over)
EST_DEV uint32_t shl1_any(uint32_t v) { const uint64_t *x = emu::exchange(v, 18); uint32_t l = emu::lane(); return l == 63 ? 0xDEADBEEFu : (uint32_t)x[l + 1]; }
EST_DEV uint32_t shl1(uint32_t v) { const uint64_t *x = emu::exchange(v, 10); uint32_t l = emu::lane(); return l == 63 ? v : (uint32_t)x[l + 1]; }
EST_DEV uint32_t xor1(uint32_t v) { return (uint32_t)emu::exchange(v, 11)[emu::lane() ^ 1u]; }
EST_DEV uint32_t xor2(uint32_t v) { return (uint32_t)emu::exchange(v, 12)[emu::lane() ^ 2u]; }
EST_DEV uint32_t xor4(uint32_t v) { return (uint32_t)emu::exchange(v, 13)[emu::lane() ^ 4u]; }
EST_DEV uint32_t xor8(uint32_t v) { return (uint32_t)emu::exchange(v, 14)[emu::lane() ^ 8u]; }

EST_DEV bool lane_in(uint64_t m) { return (m >> emu::lane()) & 1ull; }

// (every lane must pass the same mask: checked like any other wave-uniform argument)
EST_DEV uint32_t rank_below(uint64_t m) {
    const uint64_t *x = emu::exchange(m, 15);
    EST_CHECK(x[0] == m);
    const uint32_t l = emu::lane();
    return (uint32_t)__builtin_popcountll(m & (l >= 64 ? ~0ull : ((1ull << l) - 1ull)));
}

EST_DEV uint32_t opaque(uint32_t v) { return v; }
EST_DEV uint32_t opaque_uniform(uint32_t v) { return v; }
EST_DEV void check_uniform2(uint32_t a, uint32_t b, const char *what) {
    const uint64_t mine = ((uint64_t)a << 32) | b;
    const uint64_t *x = emu::exchange(mine, 17);
    for (int i = 0; i < 64; ++i)
        if (x[i] != mine) {
            fprintf(stderr, "%s: operands not uniform\n", what);
            abort();
        }
}
EST_DEV uint32_t set_lane(uint32_t v, uint32_t x, uint32_t l) {
    check_uniform2(x, l, "set_lane");
    if (l >= 64) {
        fprintf(stderr, "set_lane: lane %u out of range\n", l);
        abort();
    }
    return emu::lane() == l ? x : v;
}
EST_DEV uint32_t flag_ge(uint32_t a, uint32_t b) { check_uniform2(a, b, "flag_ge"); return a >= b ? 1u : 0u; }
EST_DEV uint32_t flag_lt(uint32_t a, uint32_t b) { check_uniform2(a, b, "flag_lt"); return a < b ? 1u : 0u; }
EST_DEV uint32_t flag_ne_and_ge(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    check_uniform2(a, b, "flag_ne_and_ge");
    check_uniform2(c, d, "flag_ne_and_ge");
    EST_CHECK(d >= 1u);
    return (a != b && c >= d) ? 1u : 0u;
}
EST_DEV uint32_t flag_ne(uint32_t a, uint32_t b) { check_uniform2(a, b, "flag_ne"); return a != b ? 1u : 0u; }
// (both operands must be the same in every lane: checked)
EST_DEV uint32_t sat_add_uniform(uint32_t t, uint32_t d) {
    check_uniform2(t, d, "sat_add_uniform");
    const uint32_t r = t + d;
    return r < t ? 0xFFFFFFFFu : r;
}

EST_DEV uint32_t uniform(uint32_t v) { return (uint32_t)emu::exchange(v, 4)[0]; }

EST_DEV uint32_t min_u32(uint32_t v) {
    const uint64_t *x = emu::exchange(v, 5);
    uint32_t m = 0xFFFFFFFFu;
    for (int l = 0; l < 64; ++l) m = (uint32_t)x[l] < m ? (uint32_t)x[l] : m;
    return m;
}

EST_DEV uint32_t sum_u32(uint32_t v) {
    const uint64_t *x = emu::exchange(v, 6);
    uint32_t s = 0;
    for (int l = 0; l < 64; ++l) s += (uint32_t)x[l];
    return s;
}

EST_DEV uint32_t prefix_excl_u32(uint32_t v) {
    const uint64_t *x = emu::exchange(v, 7);
    uint32_t s = 0;
    for (uint32_t l = 0; l < emu::lane(); ++l) s += (uint32_t)x[l];
    return s;
}

EST_DEV uint32_t load_shared(const uint32_t *p) { return *(const volatile uint32_t *)p; }
EST_DEV void store_shared(uint32_t *p, uint32_t v) { *(volatile uint32_t *)p = v; }
EST_DEV void sync() { (void)emu::exchange(0, 8); }
EST_DEV void sync_lds() { (void)emu::exchange(0, 16); }  // (memory here is host memory either way)

EST_DEV void lds_add(uint32_t *p, uint32_t v) { *p += v; }
EST_DEV void atomic_or_u64(uint64_t *p, uint64_t v) { *p |= v; }
EST_DEV void atomic_or_u32(uint32_t *p, uint32_t v) { *p |= v; }
EST_DEV void atomic_add_u32(uint32_t *p, uint32_t v) { *p += v; }
EST_DEV void atomic_max_u32(uint32_t *p, uint32_t v) { if (v > *p) *p = v; }
EST_DEV uint32_t fetch_add_u32(uint32_t *p, uint32_t v) { uint32_t o = *p; *p += v; return o; }
EST_DEV uint64_t ticks() { return 0; }
EST_DEV void atomic_add_u64(uint64_t *p, uint64_t v) { *p += v; }

}  // namespace wv
