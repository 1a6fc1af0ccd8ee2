// Wavefront-level primitives for gfx950 (64 lanes).  They act inside one wavefront; a workgroup may hold several.
// Every function here must be called by all 64 lanes in wave-uniform control flow.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define EST_DEV __device__ __forceinline__
#define EST_DEV_NOINLINE __device__ __attribute__((noinline))
#define EST_UNROLL _Pragma("unroll")
#define EST_CHECK(cond) ((void)0)
#define EST_CHK_ORDER_INIT() ((void)0)
#define EST_CHK_ORDER(tag) ((void)0)

namespace wv {

EST_DEV uint32_t lane() { return threadIdx.x & 63u; }

EST_DEV uint64_t ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// value of v in lane src (src may differ per lane)
EST_DEV uint32_t shfl(uint32_t v, uint32_t src) {
    return (uint32_t)__builtin_amdgcn_ds_bpermute((int)(src << 2), (int)v);
}

// value of v in lane l; l must be the same in every lane
EST_DEV uint32_t bcast(uint32_t v, uint32_t l) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)__builtin_amdgcn_readfirstlane((int)l));
}

// value of lane-1 (lane 0 keeps its own) / of lane+1 (lane 63 keeps its own: shl1)
EST_DEV uint32_t shr1(uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x138, 0xF, 0xF, false); }
// the same, except that lane 63 gets an unspecified value (no copy of the old value is needed first)
EST_DEV uint32_t shl1_any(uint32_t v) { return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x130, 0xF, 0xF, true); }
EST_DEV uint32_t shl1(uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x130, 0xF, 0xF, false); }
// value of lane ^ 1, ^ 2, ^ 4, ^ 8 (data-parallel-primitive moves inside a row of 16 lanes; every
// lane has a source, so no previous value is carried)
EST_DEV uint32_t xor1(uint32_t v) { return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true); }
EST_DEV uint32_t xor2(uint32_t v) { return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true); }
EST_DEV uint32_t xor8(uint32_t v) { return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x128, 0xF, 0xF, true); }
EST_DEV uint32_t xor4(uint32_t v) {
    const uint32_t down = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x124, 0xF, 0xF, true);  // from lane-4 (mod 16)
    const uint32_t up = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x12C, 0xF, 0xF, true);    // from lane+4 (mod 16)
    return __builtin_amdgcn_inverse_ballot_w64(0xF0F0F0F0F0F0F0F0ull) ? down : up;
}

// is this lane's bit set in m?  (m must be the same in every lane; the mask is used as the lane
// predicate directly, no vector instruction is spent on it)
EST_DEV bool lane_in(uint64_t m) { return __builtin_amdgcn_inverse_ballot_w64(m); }

// number of set bits of m below this lane's position (m must be the same in every lane)
EST_DEV uint32_t rank_below(uint64_t m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// v, hidden from the optimiser: what is computed from the result inside a loop is not moved out of the loop
// (where it would hold registers for the whole loop)
EST_DEV uint32_t opaque(uint32_t v) {
    asm volatile("" : "+v"(v));
    return v;
}

// the value of the first lane, in a scalar register (for a value the compiler already knows to be the same in every
// lane this costs nothing)
EST_DEV uint32_t uniform(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }

// The helpers below take operands that are the same in every lane and work on the scalar unit.  Their operands go
// through uniform() first: where the compiler keeps such a value in a vector register (it does when it cannot
// prove the value uniform), the scalar-register operand of the instruction text would otherwise not assemble.

// v (the same in every lane), hidden from the optimiser and kept in a scalar register: a test of the result stays a
// scalar compare and branch of its own instead of being merged with its neighbours into lane-mask arithmetic
EST_DEV uint32_t opaque_uniform(uint32_t v) {
    v = uniform(v);
    asm volatile("" : "+s"(v));
    return v;
}

// 1 when a >= b (a != b), else 0, for operands that are the same in every lane: a scalar compare whose result is an
// integer in a scalar register (several tests combined with & and | then cost one branch, and no lane masks)
EST_DEV uint32_t flag_ge(uint32_t a, uint32_t b) {
    uint32_t r;
    a = uniform(a); b = uniform(b);
    asm("s_cmp_ge_u32 %1, %2\n\ts_cselect_b32 %0, 1, 0" : "=s"(r) : "s"(a), "s"(b) : "scc");
    return r;
}
EST_DEV uint32_t flag_lt(uint32_t a, uint32_t b) {
    uint32_t r;
    a = uniform(a); b = uniform(b);
    asm("s_cmp_lt_u32 %1, %2\n\ts_cselect_b32 %0, 1, 0" : "=s"(r) : "s"(a), "s"(b) : "scc");
    return r;
}
// 1 when a != b and c >= d (d at least 1), else 0
EST_DEV uint32_t flag_ne_and_ge(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    uint32_t r;
    a = uniform(a); b = uniform(b); c = uniform(c); d = uniform(d);
    asm("s_cmp_lg_u32 %1, %2\n\ts_cselect_b32 %0, %3, 0\n\ts_cmp_ge_u32 %0, %4\n\ts_cselect_b32 %0, 1, 0"
        : "=&s"(r) : "s"(a), "s"(b), "s"(c), "s"(d) : "scc");
    return r;
}
EST_DEV uint32_t flag_ne(uint32_t a, uint32_t b) {
    uint32_t r;
    a = uniform(a); b = uniform(b);
    asm("s_cmp_lg_u32 %1, %2\n\ts_cselect_b32 %0, 1, 0" : "=s"(r) : "s"(a), "s"(b) : "scc");
    return r;
}

// v with lane l replaced by x (l and x the same in every lane, l < 64): v_writelane_b32, reached through its
// compiler intrinsic (this compiler declares no builtin for it), so wait states and m0 are the compiler's business.
extern "C" __device__ uint32_t est_llvm_writelane(uint32_t x, uint32_t l, uint32_t v) __asm("llvm.amdgcn.writelane");
EST_DEV uint32_t set_lane(uint32_t v, uint32_t x, uint32_t l) { return est_llvm_writelane(x, l, v); }

// min(t + d, 2^32 - 1) for operands that are the same in every lane, on the scalar unit (the compiler's own
// saturating add exists on the vector unit only, with a trip there and back)
EST_DEV uint32_t sat_add_uniform(uint32_t t, uint32_t d) {
    uint32_t r;
    t = uniform(t); d = uniform(d);
    asm("s_add_u32 %0, %1, %2\n\ts_cselect_b32 %0, -1, %0" : "=s"(r) : "s"(t), "s"(d) : "scc");
    return r;
}

EST_DEV uint32_t min_u32(uint32_t v) {
#pragma unroll
    for (uint32_t d = 32; d >= 1; d >>= 1) {
        uint32_t o = shfl(v, lane() ^ d);
        v = o < v ? o : v;
    }
    return uniform(v);
}

// (moves inside the rows of 16 lanes, then one scalar read per row: no trip through the LDS crossbar)
EST_DEV uint32_t sum_u32(uint32_t v) {
    v += xor1(v);
    v += xor2(v);
    v += (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x124, 0xF, 0xF, true);  // + lane-4 (mod 16)
    v += xor8(v);
    return bcast(v, 0) + bcast(v, 16) + bcast(v, 32) + bcast(v, 48);
}

// exclusive prefix sum over lanes: shifts by 1, 2, 4, 8 inside the rows of 16 lanes (zeros come in at the row's
// start), then the totals of the rows before a lane's own are added from scalar registers.  (Carrying the row
// totals across with row broadcasts instead measured 5 % slower on the whole sweep.)
EST_DEV uint32_t prefix_excl_u32(uint32_t v) {
    uint32_t x = v;
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xF, 0xF, true);  // row_shr:1
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xF, 0xF, true);  // row_shr:2
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xF, 0xF, true);  // row_shr:4
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xF, 0xF, true);  // row_shr:8
    const uint32_t t0 = bcast(x, 15), t1 = t0 + bcast(x, 31), t2 = t1 + bcast(x, 47);
    const uint32_t row = lane() >> 4;
    const uint32_t before = row == 0u ? 0u : row == 1u ? t0 : row == 2u ? t1 : t2;
    return x + before - v;
}

// Make earlier memory writes (global and LDS) of any lane visible to later reads of any lane
// of this wavefront.
EST_DEV void sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// The same for LDS only: earlier LDS writes of any lane are visible to later LDS reads of any lane of
// this wavefront.  Does not wait for outstanding global loads or stores.
EST_DEV void sync_lds() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// A word that another wavefront of the workgroup may write or read (the same address and value in every lane)
EST_DEV uint32_t load_shared(const uint32_t *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
EST_DEV void store_shared(uint32_t *p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }

EST_DEV void lds_add(uint32_t *p, uint32_t v) { atomicAdd(p, v); }
EST_DEV void atomic_or_u64(uint64_t *p, uint64_t v) { atomicOr((unsigned long long *)p, (unsigned long long)v); }
EST_DEV void atomic_or_u32(uint32_t *p, uint32_t v) { atomicOr(p, v); }
EST_DEV void atomic_add_u32(uint32_t *p, uint32_t v) { atomicAdd(p, v); }
EST_DEV void atomic_max_u32(uint32_t *p, uint32_t v) { atomicMax(p, v); }
EST_DEV uint32_t fetch_add_u32(uint32_t *p, uint32_t v) { return atomicAdd(p, v); }
EST_DEV uint64_t ticks() { return wall_clock64(); }
EST_DEV void atomic_add_u64(uint64_t *p, uint64_t v) { atomicAdd((unsigned long long *)p, (unsigned long long)v); }

}  // namespace wv
