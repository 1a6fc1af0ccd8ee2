// Device-side services the host planner needs: memory, copies, kernel launches, events.
// Implemented for the GPU in est_kernels.hip.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "est_types.h"

namespace estbe {

int init();                       // 0, or non-zero with last_error() set when no usable GPU is present
const char *last_error();
void *dmalloc(size_t bytes);      // nullptr on failure
void dfree(void *p);
size_t mem_free();                // free device memory in bytes
int h2d(void *dst, const void *src, size_t bytes, void *stream);
int d2h(void *dst, const void *src, size_t bytes, void *stream);
int d2d(void *dst, const void *src, size_t bytes, void *stream);
int zero(void *dst, size_t bytes, void *stream);
int sync(void *stream);

int launch_cfg(const EstCfgArgs &a, void *stream);
int launch_prep1(const EstPrepArgs &a, void *stream);
int launch_prep2(const EstPrepArgs &a, void *stream);
int launch_sim(const EstSimArgs &a, void *stream);
int launch_sim_mw(const EstSimArgs &a, uint32_t waves, void *stream);  // one workgroup of `waves` (2 or EST_MW_WAVES) wavefronts per scratch slot (a.n_slots workgroups)
int launch_envelope(const EstEnvArgs &a, void *stream);
uint32_t max_resident_waves(uint32_t lds_bytes_per_wave);  // wavefronts of the simulation kernel the device holds at once
uint32_t waves_per_simd(uint32_t lds_bytes_per_wave);      // which build of the simulation kernel runs at this LDS need: 4, 5 or 6 wavefronts per SIMD
uint32_t max_resident_groups(uint32_t lds_bytes_per_wave, uint32_t waves);  // workgroups of launch_sim_mw the device holds at once

void *stream_create();            // a second stream at the default priority; nullptr on failure
void stream_destroy(void *stream);
int stream_wait_event(void *stream, void *ev);  // later work on stream starts after ev has completed

// The library's own fixed scratch on the current device (a file-scope device array, resolved once per
// device): its address and size, or nullptr with last_error() set.  Nothing is allocated.
void *static_scratch(uint64_t *bytes);
void *host_pinned_alloc(size_t bytes);  // page-locked host memory; nullptr on failure
void host_pinned_free(void *p);

void *event_create();
void event_destroy(void *ev);
int event_record(void *ev, void *stream);
float event_ms(void *start, void *stop);  // both must have completed

}  // namespace estbe
