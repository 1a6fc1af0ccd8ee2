// Host back end for the lock-step wavefront emulation (test infrastructure): "device" memory is
// host memory, a kernel launch runs every wavefront as 64 fibers, one wavefront after the other.
#include <string.h>
#include <ucontext.h>

#include <functional>
#include <string>
#include <vector>

#include "wave_emu.h"
#include "../../paper_1812_01776_amd/csrc/est_backend.h"
#include "../../paper_1812_01776_amd/csrc/est_device.h"

namespace emu {

namespace {
const size_t STACK = 256 * 1024;
ucontext_t g_sched, g_ctx[64];
std::vector<char> g_stacks;
bool g_done[64];
uint32_t g_cur;
uint64_t g_x[2][64];
uint32_t g_tag[64];
uint32_t g_nb[64];
const std::function<void()> *g_body;

void trampoline() {
    (*g_body)();
    g_done[g_cur] = true;
    swapcontext(&g_ctx[g_cur], &g_sched);
}
}  // namespace

uint32_t lane() { return g_cur; }

const uint64_t *exchange(uint64_t v, uint32_t tag) {
    const uint32_t me = g_cur;
    const uint32_t ph = g_nb[me] & 1u;
    g_x[ph][me] = v;
    g_tag[me] = tag;
    g_nb[me]++;
    swapcontext(&g_ctx[me], &g_sched);  // wait for the other lanes
    g_cur = me;
    return g_x[ph];
}

void run_wave(const std::function<void()> &body) {
    if (g_stacks.empty()) g_stacks.resize(64 * STACK);
    g_body = &body;
    for (int l = 0; l < 64; ++l) {
        g_done[l] = false;
        g_nb[l] = 0;
        getcontext(&g_ctx[l]);
        g_ctx[l].uc_stack.ss_sp = g_stacks.data() + (size_t)l * STACK;
        g_ctx[l].uc_stack.ss_size = STACK;
        g_ctx[l].uc_link = &g_sched;
        makecontext(&g_ctx[l], trampoline, 0);
    }
    for (;;) {
        int ndone = 0;
        for (int l = 0; l < 64; ++l) {
            if (g_done[l]) { ++ndone; continue; }
            g_cur = (uint32_t)l;
            swapcontext(&g_sched, &g_ctx[l]);
            if (g_done[l]) ++ndone;
        }
        if (ndone == 64) break;
        if (ndone != 0) {
            fprintf(stderr, "emu: %d lanes left the kernel while others wait in a primitive\n", ndone);
            abort();
        }
        for (int l = 1; l < 64; ++l)
            if (g_tag[l] != g_tag[0] || g_nb[l] != g_nb[0]) {
                fprintf(stderr, "emu: lanes diverged at a primitive (lane %d tag %u vs lane 0 tag %u)\n", l, g_tag[l], g_tag[0]);
                abort();
            }
    }
}

}  // namespace emu

namespace estbe {

static std::string g_err;
const char *last_error() { return g_err.c_str(); }
int init() { return 0; }
void *dmalloc(size_t bytes) {
    void *p = nullptr;
    if (posix_memalign(&p, 256, bytes ? bytes : 256)) return nullptr;
    memset(p, 0xA5, bytes);  // uninitialised device memory is not zero
    return p;
}
void dfree(void *p) { free(p); }
size_t mem_free() { return (size_t)2 << 30; }
int h2d(void *d, const void *s, size_t n, void *) { if (n) memcpy(d, s, n); return 0; }
int d2h(void *d, const void *s, size_t n, void *) { if (n) memcpy(d, s, n); return 0; }
int d2d(void *d, const void *s, size_t n, void *) { if (n) memcpy(d, s, n); return 0; }
int zero(void *d, size_t n, void *) { if (n) memset(d, 0, n); return 0; }
int sync(void *) { return 0; }

int launch_cfg(const EstCfgArgs &a, void *) {
    for (uint32_t t = 0; t < 7; ++t) estdev::cfg_thread(a, t, 7);
    return 0;
}
int launch_prep1(const EstPrepArgs &a, void *) {
    for (uint32_t t = 0; t < 7; ++t) estdev::prep1_thread(a, t, 7);
    return 0;
}
int launch_prep2(const EstPrepArgs &a, void *) {
    for (uint32_t t = 0; t < 7; ++t) estdev::prep2_thread(a, t, 7);
    return 0;
}
int launch_envelope(const EstEnvArgs &a, void *) {
    for (uint32_t t = 0; t < 7; ++t) estdev::envelope_thread(a, t, 7);
    return 0;
}
int launch_sim(const EstSimArgs &a, void *) {
    static uint64_t lds[(64 * 1024) / 8];
    if (a.lds_bytes > sizeof lds) abort();
    // the slots run one after the other; the first takes candidates until the counter runs out, so to
    // exercise every slot's scratch the counter is handed out in turns: slot k gets candidates k, k+n_slots, ...
    EstSimArgs b = a;
    for (uint32_t slot = 0; slot < a.n_slots; ++slot) {
        for (uint32_t t = slot; t < a.n_cfg; t += a.n_slots) {
            EstStatus *st = a.status;
            st->next_cfg = t;
            b.n_cfg = t + 1;  // this slot stops after candidate t
            memset(lds, 0x5A, sizeof lds);
            emu::run_wave([&] {
                if (b.skip_ops)
                    estdev::slot_loop<false, true>(b, slot, lds);
                else if (b.dbg_ticks)
                    estdev::slot_loop<true, false>(b, slot, lds);
                else
                    estdev::slot_loop<false, false>(b, slot, lds);
            });
        }
    }
    return 0;
}
// Several wavefronts per candidate: the wavefronts of a workgroup take turns, one pass over their own operations
// each, until all are done (a full turn without progress is a stuck candidate).
int launch_sim_mw(const EstSimArgs &a, uint32_t waves, void *) {
    static uint64_t lds[EST_MW_WAVES][(64 * 1024) / 8];
    if (a.lds_bytes > sizeof lds[0]) abort();
    for (uint32_t t = 0; t < a.n_cfg; ++t) {
        const uint32_t slot = t % a.n_slots;
        memset(lds, 0x5A, sizeof lds);
        if (a.n > 0) {
            emu::run_wave([&] { estdev::mw_init(a, t, slot); });
            uint32_t done = 0;
            while (done != (1u << waves) - 1u) {
                bool progress = false;
                for (uint32_t wv_ = 0; wv_ < waves; ++wv_) {
                    if ((done >> wv_) & 1u) continue;
                    uint32_t r = 0;
                    emu::run_wave([&] { uint32_t x = estdev::mw_pass(a, t, slot, lds[wv_], wv_); if (wv::lane() == 0) r = x; });
                    if (r & 2u) done |= 1u << wv_;
                    progress = progress || (r & 3u);
                }
                if (!progress) {
                    a.status->sim_error = 1;
                    break;
                }
            }
        }
        if (!a.lat_by_qid) emu::run_wave([&] { estdev::select_wave(a, t, slot, lds[0]); });
    }
    return 0;
}
uint32_t max_resident_groups(uint32_t, uint32_t) { return 2; }
uint32_t max_resident_waves(uint32_t) { return 3; }
uint32_t waves_per_simd(uint32_t) { return 4; }

void *stream_create() { return malloc(1); }  // everything runs in program order here
void stream_destroy(void *s) { free(s); }
int stream_wait_event(void *, void *) { return 0; }

void *static_scratch(uint64_t *bytes) {
    static std::vector<unsigned char> buf(EST_STATIC_SCRATCH_BYTES + 256);
    if (bytes) *bytes = EST_STATIC_SCRATCH_BYTES;
    return (void *)(((uintptr_t)buf.data() + 255) & ~(uintptr_t)255);
}
void *host_pinned_alloc(size_t bytes) { return malloc(bytes ? bytes : 1); }
void host_pinned_free(void *p) { free(p); }

void *event_create() { return malloc(1); }
void event_destroy(void *e) { free(e); }
int event_record(void *, void *) { return 0; }
float event_ms(void *, void *) { return 0.f; }

}  // namespace estbe
