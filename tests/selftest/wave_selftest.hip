// Test-only library (never part of libestimator.so): runs the wavefront primitives of
// paper_1812_01776_amd/csrc/wave_gfx950.h and the bitonic network built from them on one wavefront and
// hands the lane-by-lane results to the GPU tests.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../paper_1812_01776_amd/csrc/wave_gfx950.h"
#include "../../paper_1812_01776_amd/csrc/est_device.h"

// Lane-layout check of the wavefront primitives: out[i][lane] for the input v = 7 * lane + 3
// (i = 0..5: shr1, shl1, xor1, xor2, xor4, xor8) and for sort_lanes of a scrambled input at widths
// 2..64 (i = 6..11).
static __global__ __launch_bounds__(64) void est_wave_selftest_kernel(uint32_t *out) {
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
}


// Runs the lane-layout check kernel and copies its 13 x 64 results to host memory.  Returns 0 on success.
extern "C" int est_selftest_wave(uint32_t *host_out) {
    uint32_t *d = nullptr;
    if (hipMalloc((void **)&d, 13 * 64 * 4) != hipSuccess) return 1;
    est_wave_selftest_kernel<<<1, 64>>>(d);
    int rc = hipGetLastError() != hipSuccess;
    rc = rc || hipMemcpy(host_out, d, 13 * 64 * 4, hipMemcpyDeviceToHost) != hipSuccess;
    (void)hipFree(d);
    return rc;
}
