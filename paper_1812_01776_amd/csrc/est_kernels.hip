// GPU back end: kernel entry points (one 64-lane wavefront per workgroup) and the HIP runtime
// calls the host planner needs.  gfx950 only.
#include <hip/hip_runtime.h>

#include <stdlib.h>

#include <string>

#include "est_backend.h"
#include "wave_gfx950.h"
#include "est_device.h"

namespace {

thread_local std::string g_err;

int check(hipError_t e, const char *what) {
    if (e == hipSuccess) return 0;
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    return 1;
}

// Four wavefronts per workgroup; each wavefront owns one scratch slot and its own part of the LDS
// and works through candidates until the launch's work counter runs out.  The register budget is
// pinned per build (WAVES_PER_SIMD resident wavefronts per SIMD: 128, 96 or 80 registers per lane).
#define EST_WAVES_PER_BLOCK 4
template <bool DIAG, int WAVES_PER_SIMD, bool MEMO = false>
__global__ __launch_bounds__(64 * EST_WAVES_PER_BLOCK) __attribute__((amdgpu_waves_per_eu(WAVES_PER_SIMD, WAVES_PER_SIMD)))
void est_sim_kernel(EstSimArgs a) {
    extern __shared__ uint64_t lds[];  // EST_WAVES_PER_BLOCK x a.lds_bytes
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t slot = blockIdx.x * EST_WAVES_PER_BLOCK + wave;
    if (slot < a.n_slots) estdev::slot_loop<DIAG, MEMO>(a, slot, lds + (size_t)wave * (a.lds_bytes / 8));
}

// Several wavefronts per candidate: a workgroup of 2 to EST_MW_WAVES wavefronts (the launch's block size) owns one scratch slot and takes
// candidates from the work counter; the candidate's operations are dealt out to the wavefronts (EstOp::owner),
// which run them as a pipeline through the rings.  A wavefront that finds nothing to do waits a little and looks
// again; every wait is bounded (a stuck candidate sets the error flag and every wavefront leaves).
constexpr uint32_t MW_IDLE_LIMIT = 1u << 24;
template <int WAVES_PER_SIMD>
__global__ __launch_bounds__(64 * EST_MW_WAVES) __attribute__((amdgpu_waves_per_eu(WAVES_PER_SIMD, WAVES_PER_SIMD)))
void est_sim_mw_kernel(EstSimArgs a) {
    extern __shared__ uint64_t lds[];  // wavefronts of the workgroup x a.lds_bytes
    __shared__ uint32_t next_t;
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t slot = blockIdx.x;
    uint64_t *my_lds = lds + (size_t)wave * (a.lds_bytes / 8);
    for (;;) {
        if (threadIdx.x == 0) next_t = atomicAdd(&a.status->next_cfg, 1u);
        __syncthreads();
        const uint32_t t = next_t;
        __syncthreads();
        if (t >= a.n_cfg) break;
        if (a.n > 0) {
            if (wave == 0) estdev::mw_init(a, t, slot);
            __syncthreads();
            for (uint32_t idle = 0;;) {
                const uint32_t r = estdev::mw_pass(a, t, slot, my_lds, wave);
                if (r & 2u) break;
                if (r & 1u) {
                    idle = 0;
                    continue;
                }
                // waiting for a neighbour: give the other wavefronts the issue slots, give up if it never comes
                if (++idle > MW_IDLE_LIMIT || wv::load_shared(&a.status->sim_error)) {
                    if (wv::lane() == 0) a.status->sim_error = 1;
                    break;
                }
                __builtin_amdgcn_s_sleep(4);
            }
        }
        __syncthreads();
        if (wave == 0 && !a.lat_by_qid) estdev::select_wave(a, t, slot, my_lds);
        __syncthreads();
    }
}

// The kernel is built for four wavefronts per SIMD (128 registers per lane, no spills), for five (96, a few
// spills) and for six (80, about twenty): the build with the most wavefronts that the LDS need of the launch
// allows is used, because each extra wavefront hides more latency than its spills cost.
constexpr uint32_t LDS_PER_CU = 160u * 1024u;
int waves_fit(uint32_t lds_bytes_per_wave) {
    static const char *cap = getenv("EST_WAVES_PER_SIMD");  // tuning aid: no more than this many (4, 5 or 6)
    const int most = cap ? atoi(cap) : 6;
    for (int w = 6; w > 4; --w)
        if (w <= most && (uint64_t)lds_bytes_per_wave * EST_WAVES_PER_BLOCK * (uint32_t)w <= LDS_PER_CU) return w;
    return 4;
}

__global__ __launch_bounds__(256) void est_prep1_kernel(EstPrepArgs a) {
    estdev::prep1_thread(a, blockIdx.x * blockDim.x + threadIdx.x, gridDim.x * blockDim.x);
}

__global__ __launch_bounds__(256) void est_prep2_kernel(EstPrepArgs a) {
    estdev::prep2_thread(a, blockIdx.x * blockDim.x + threadIdx.x, gridDim.x * blockDim.x);
}

__global__ __launch_bounds__(256) void est_envelope_kernel(EstEnvArgs a) {
    estdev::envelope_thread(a, blockIdx.x * blockDim.x + threadIdx.x, gridDim.x * blockDim.x);
}

__global__ __launch_bounds__(256) void est_cfg_kernel(EstCfgArgs a) {
    estdev::cfg_thread(a, blockIdx.x * blockDim.x + threadIdx.x, gridDim.x * blockDim.x);
}

// Scratch of estimator_run_static_dev, the entry point for callers that cannot allocate: every GPU the
// library runs on holds this array until the process ends.  In host code the array's name is only a
// symbol: its device address is asked for once per device (static_scratch below) and used from then on.
static __device__ __align__(256) unsigned char scratch[EST_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES];

uint32_t blocks_for(uint64_t items, uint32_t per_block, uint32_t max_blocks) {
    uint64_t b = (items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    return (uint32_t)(b > max_blocks ? max_blocks : b);
}

}  // namespace

namespace estbe {

const char *last_error() { return g_err.c_str(); }

int init() {
    int n = 0;
    if (check(hipGetDeviceCount(&n), "hipGetDeviceCount")) return 1;
    if (n < 1) {
        g_err = "no HIP device";
        return 1;
    }
    return 0;
}

void *dmalloc(size_t bytes) {
    void *p = nullptr;
    if (check(hipMalloc(&p, bytes), "hipMalloc")) {
        (void)hipGetLastError();  // (the caller may try again smaller: no stale error for the next launch check to find)
        return nullptr;
    }
    return p;
}

void dfree(void *p) { (void)hipFree(p); }

size_t mem_free() {
    size_t f = 0, t = 0;
    if (hipMemGetInfo(&f, &t) != hipSuccess) return 0;
    return f;
}

int h2d(void *dst, const void *src, size_t bytes, void *stream) {
    if (bytes == 0) return 0;
    return check(hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, (hipStream_t)stream), "hipMemcpyAsync H2D");
}
int d2h(void *dst, const void *src, size_t bytes, void *stream) {
    if (bytes == 0) return 0;
    return check(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, (hipStream_t)stream), "hipMemcpyAsync D2H");
}
int d2d(void *dst, const void *src, size_t bytes, void *stream) {
    if (bytes == 0) return 0;
    return check(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, (hipStream_t)stream), "hipMemcpyAsync D2D");
}
int zero(void *dst, size_t bytes, void *stream) {
    if (bytes == 0) return 0;
    return check(hipMemsetAsync(dst, 0, bytes, (hipStream_t)stream), "hipMemsetAsync");
}
int sync(void *stream) { return check(hipStreamSynchronize((hipStream_t)stream), "hipStreamSynchronize"); }

int launch_cfg(const EstCfgArgs &a, void *stream) {
    est_cfg_kernel<<<blocks_for(a.n_cfg, 256, 1024), 256, 0, (hipStream_t)stream>>>(a);
    return check(hipGetLastError(), "est_cfg_kernel");
}
int launch_prep1(const EstPrepArgs &a, void *stream) {
    est_prep1_kernel<<<blocks_for(a.n, 256 * 8, 1024), 256, 0, (hipStream_t)stream>>>(a);
    return check(hipGetLastError(), "est_prep1_kernel");
}
int launch_prep2(const EstPrepArgs &a, void *stream) {
    est_prep2_kernel<<<blocks_for(a.n, 256, 4096), 256, 0, (hipStream_t)stream>>>(a);
    return check(hipGetLastError(), "est_prep2_kernel");
}
int launch_envelope(const EstEnvArgs &a, void *stream) {
    est_envelope_kernel<<<blocks_for(a.n, 256 * 16, 8192), 256, 0, (hipStream_t)stream>>>(a);  // 16 queries in a row per thread
    return check(hipGetLastError(), "est_envelope_kernel");
}
uint32_t waves_per_simd(uint32_t lds_bytes_per_wave) { return (uint32_t)waves_fit(lds_bytes_per_wave); }
int launch_sim_mw(const EstSimArgs &a, uint32_t waves, void *stream) {
    if (waves < 2 || waves > EST_MW_WAVES) {
        g_err = "est_sim_mw_kernel: a workgroup has 2 to 4 wavefronts";
        return 1;
    }
    const size_t lds = (size_t)a.lds_bytes * waves;
    if (waves_fit(a.lds_bytes) == 6)  // (the builds for four and for six wavefronts per SIMD, as for est_sim_kernel)
        est_sim_mw_kernel<6><<<dim3(a.n_slots), dim3(64 * waves), lds, (hipStream_t)stream>>>(a);
    else
        est_sim_mw_kernel<4><<<dim3(a.n_slots), dim3(64 * waves), lds, (hipStream_t)stream>>>(a);
    return check(hipGetLastError(), "est_sim_mw_kernel");
}
uint32_t max_resident_groups(uint32_t lds_bytes_per_wave, uint32_t waves) {
    int dev = 0, cus = 0, blocks = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    const hipError_t e = waves_fit(lds_bytes_per_wave) == 6
                             ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, est_sim_mw_kernel<6>, 64 * (int)waves, (size_t)lds_bytes_per_wave * waves)
                             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, est_sim_mw_kernel<4>, 64 * (int)waves, (size_t)lds_bytes_per_wave * waves);
    if (e != hipSuccess || blocks < 1)
        blocks = 1;
    return (uint32_t)cus * (uint32_t)blocks;
}
int launch_sim(const EstSimArgs &a, void *stream) {
    const uint32_t blocks = (a.n_slots + EST_WAVES_PER_BLOCK - 1) / EST_WAVES_PER_BLOCK;
    // (the variant that keeps diagnostic counters is launched only when they are asked for)
    const size_t lds = (size_t)a.lds_bytes * EST_WAVES_PER_BLOCK;
    const dim3 grid(blocks), block(64 * EST_WAVES_PER_BLOCK);
    if (a.skip_ops) {  // candidates that skip operations (shared upstream stages): the variant that reads the extra arguments
        const int w = waves_fit(a.lds_bytes);
        if (w == 6)
            est_sim_kernel<false, 6, true><<<grid, block, lds, (hipStream_t)stream>>>(a);
        else if (w == 5)
            est_sim_kernel<false, 5, true><<<grid, block, lds, (hipStream_t)stream>>>(a);
        else
            est_sim_kernel<false, 4, true><<<grid, block, lds, (hipStream_t)stream>>>(a);
    } else if (a.dbg_ticks)
        est_sim_kernel<true, 4><<<grid, block, lds, (hipStream_t)stream>>>(a);
    else if (waves_fit(a.lds_bytes) == 6)
        est_sim_kernel<false, 6><<<grid, block, lds, (hipStream_t)stream>>>(a);
    else if (waves_fit(a.lds_bytes) == 5)
        est_sim_kernel<false, 5><<<grid, block, lds, (hipStream_t)stream>>>(a);
    else
        est_sim_kernel<false, 4><<<grid, block, lds, (hipStream_t)stream>>>(a);
    return check(hipGetLastError(), "est_sim_kernel");
}

// Wavefronts of the simulation kernel the device holds at once for a given LDS size per wavefront
// (registers allow four per SIMD; LDS may allow fewer).  More scratch slots than that would only
// hold memory: a wavefront that starts after the others have finished finds no candidates left.
uint32_t max_resident_waves(uint32_t lds_bytes_per_wave) {
    int dev = 0, cus = 0, blocks = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    const int w = waves_fit(lds_bytes_per_wave);
    const size_t lds = (size_t)lds_bytes_per_wave * EST_WAVES_PER_BLOCK;
    const hipError_t e = w == 6   ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, est_sim_kernel<false, 6>, 64 * EST_WAVES_PER_BLOCK, lds)
                         : w == 5 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, est_sim_kernel<false, 5>, 64 * EST_WAVES_PER_BLOCK, lds)
                                  : hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, est_sim_kernel<false, 4>, 64 * EST_WAVES_PER_BLOCK, lds);
    if (e != hipSuccess || blocks < 1) blocks = 8;  // unknown: assume the most a compute unit can hold
    return (uint32_t)cus * (uint32_t)blocks * EST_WAVES_PER_BLOCK;
}

void *stream_create() {
    hipStream_t st = nullptr;
    if (check(hipStreamCreateWithFlags(&st, hipStreamNonBlocking), "hipStreamCreate")) return nullptr;
    return (void *)st;
}
void stream_destroy(void *stream) { (void)hipStreamDestroy((hipStream_t)stream); }
int stream_wait_event(void *stream, void *ev) { return check(hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)ev, 0), "hipStreamWaitEvent"); }

void *static_scratch(uint64_t *bytes) {
    int dev = 0;
    if (check(hipGetDevice(&dev), "hipGetDevice")) return nullptr;
    if (dev < 0 || dev >= MAX_DEVICES) {
        g_err = "device index out of range for the static scratch";
        return nullptr;
    }
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (check(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)")) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    if (bytes) *bytes = EST_STATIC_SCRATCH_BYTES;
    return g_scratch_ptr[dev];
}

void *host_pinned_alloc(size_t bytes) {
    void *p = nullptr;
    if (check(hipHostMalloc(&p, bytes, hipHostMallocDefault), "hipHostMalloc")) return nullptr;
    return p;
}
void host_pinned_free(void *p) { (void)hipHostFree(p); }

void *event_create() {
    hipEvent_t e = nullptr;
    if (check(hipEventCreate(&e), "hipEventCreate")) return nullptr;
    return (void *)e;
}
void event_destroy(void *ev) { (void)hipEventDestroy((hipEvent_t)ev); }
int event_record(void *ev, void *stream) { return check(hipEventRecord((hipEvent_t)ev, (hipStream_t)stream), "hipEventRecord"); }
float event_ms(void *start, void *stop) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, (hipEvent_t)start, (hipEvent_t)stop) != hipSuccess) return 0.f;
    return ms;
}

}  // namespace estbe
