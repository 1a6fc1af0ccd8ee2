// Test-only library (never part of libestimator.so): runs the wavefront primitives of
// paper_1812_01776_amd/csrc/wave_gfx950.h and the bitonic network built from them on one wavefront and
// hands the lane-by-lane results to the GPU tests.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../paper_1812_01776_amd/csrc/wave_gfx950.h"
#include "../../paper_1812_01776_amd/csrc/est_device.h"

// Lane-layout check of the wavefront primitives: out[i][lane] for the input v = 7 * lane + 3
// (i = 0..5: shr1, shl1, xor1, xor2, xor4, xor8) and for sort_lanes of a scrambled input at widths
// 2..64 (i = 6..11), rank_below of a fixed mask (12), and the scalar-unit helpers: shl1_any (13; lane 63
// unspecified), set_lane twice (14), sat_add_uniform without and with overflow (15, 16), the flags (17: bit 0
// flag_ge(5,5), bit 1 flag_ge(4,5), bit 2 flag_lt(4,5), bit 3 flag_lt(5,5), bit 4 flag_ne(4,5), bit 5 flag_ne(5,5),
// bit 6 flag_ne_and_ge(1,2,7,7), bit 7 flag_ne_and_ge(2,2,7,7), bit 8 flag_ne_and_ge(1,2,6,7)), opaque_uniform (18),
// prefix_excl_u32 and sum_u32 of scr^2 + 1 (19, 20).
// (The operands are read from memory so that nothing is folded at compile time.)
static __global__ __launch_bounds__(64) void est_wave_selftest_kernel(uint32_t *out, const uint32_t *in) {
    const uint32_t ln = threadIdx.x;
    const uint32_t v = 7u * ln + 3u;
    out[0 * 64 + ln] = wv::shr1(v);
    out[1 * 64 + ln] = wv::shl1(v);
    out[2 * 64 + ln] = wv::xor1(v);
    out[3 * 64 + ln] = wv::xor2(v);
    out[4 * 64 + ln] = wv::xor4(v);
    out[5 * 64 + ln] = wv::xor8(v);
    const uint32_t scr = (ln * 37u + 11u) & 63u;  // a permutation of 0..63
    uint32_t i = 6;
    for (uint32_t width = 2; width <= 64; width <<= 1, ++i)
        out[i * 64 + ln] = estdev::sort_lanes(ln < width ? scr : 0xFFFFFFFFu, width);
    out[12 * 64 + ln] = wv::rank_below(0xF0F0A5A5C3C3FF01ull);
    // in[] = {1, 2, 4, 5, 6, 7, 17, 41, 1000, 0xFFFFFF00, 0x200}
    const uint32_t c1 = wv::uniform(in[0]), c2 = wv::uniform(in[1]), c4 = wv::uniform(in[2]), c5 = wv::uniform(in[3]), c6 = wv::uniform(in[4]),
                   c7 = wv::uniform(in[5]), l17 = wv::uniform(in[6]), l41 = wv::uniform(in[7]), k = wv::uniform(in[8]),
                   big = wv::uniform(in[9]), d = wv::uniform(in[10]);
    out[13 * 64 + ln] = wv::shl1_any(v);
    out[14 * 64 + ln] = wv::set_lane(wv::set_lane(v, k, l17), k + c1, l41);
    out[15 * 64 + ln] = wv::sat_add_uniform(k, d);
    out[16 * 64 + ln] = wv::sat_add_uniform(big, d);
    out[17 * 64 + ln] = wv::flag_ge(c5, c5) | (wv::flag_ge(c4, c5) << 1) | (wv::flag_lt(c4, c5) << 2) | (wv::flag_lt(c5, c5) << 3) |
                        (wv::flag_ne(c4, c5) << 4) | (wv::flag_ne(c5, c5) << 5) | (wv::flag_ne_and_ge(c1, c2, c7, c7) << 6) |
                        (wv::flag_ne_and_ge(c2, c2, c7, c7) << 7) | (wv::flag_ne_and_ge(c1, c2, c6, c7) << 8);
    out[18 * 64 + ln] = wv::opaque_uniform(k) + ln;
    out[19 * 64 + ln] = wv::prefix_excl_u32(scr * scr + 1u);
    out[20 * 64 + ln] = wv::sum_u32(scr * scr + 1u);
}


// Runs the lane-layout check kernel and copies its 21 x 64 results to host memory.  Returns 0 on success.
extern "C" int est_selftest_wave(uint32_t *host_out) {
    static const uint32_t operands[11] = {1, 2, 4, 5, 6, 7, 17, 41, 1000, 0xFFFFFF00u, 0x200};
    uint32_t *d = nullptr, *in = nullptr;
    if (hipMalloc((void **)&d, 21 * 64 * 4) != hipSuccess) return 1;
    if (hipMalloc((void **)&in, sizeof operands) != hipSuccess) {
        (void)hipFree(d);
        return 1;
    }
    int rc = hipMemcpy(in, operands, sizeof operands, hipMemcpyHostToDevice) != hipSuccess;
    if (!rc) {
        est_wave_selftest_kernel<<<1, 64>>>(d, in);
        rc = hipGetLastError() != hipSuccess;
        rc = rc || hipMemcpy(host_out, d, 21 * 64 * 4, hipMemcpyDeviceToHost) != hipSuccess;
    }
    (void)hipFree(d);
    (void)hipFree(in);
    return rc;
}
