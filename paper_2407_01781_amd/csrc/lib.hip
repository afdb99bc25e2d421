// Library-wide plumbing: error text, device allocation, pinned staging, version.
#include "common.h"

#include <stdarg.h>
#include <stdlib.h>

#include <mutex>
#include <vector>

namespace fx {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

// Stream-ordered allocation from the device's default memory pool; the pool keeps freed
// blocks (release threshold = max) so steady-state builds do not reach the driver.
// FVDB_HOTPATH_SYNC_ALLOC=1 switches to plain hipMalloc / hipFree.
static int use_sync_alloc() {
    static int v = -1;
    if (v < 0) {
        const char* e = getenv("FVDB_HOTPATH_SYNC_ALLOC");
        v = (e && e[0] == '1') ? 1 : 0;
    }
    return v;
}

static void ensure_pool_configured() {
    static thread_local int done_for_device = -1;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return;
    if (done_for_device == dev) return;
    hipMemPool_t pool;
    if (hipDeviceGetDefaultMemPool(&pool, dev) == hipSuccess) {
        uint64_t thr = UINT64_MAX;
        (void)hipMemPoolSetAttribute(pool, hipMemPoolAttrReleaseThreshold, &thr);
    }
    done_for_device = dev;
}

fx_status dev_alloc(void** p, size_t bytes, hipStream_t s) {
    if (bytes == 0) bytes = 256;
    hipError_t e;
    if (use_sync_alloc()) {
        e = hipMalloc(p, bytes);
    } else {
        ensure_pool_configured();
        e = hipMallocAsync(p, bytes, s);
    }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        set_error("device allocation of %zu bytes failed: %s", bytes, hipGetErrorString(e));
        *p = nullptr;
        return e == hipErrorOutOfMemory ? FX_ENOMEM : FX_EDEVICE;
    }
    return FX_OK;
}

void dev_free(void* p, hipStream_t s) {
    if (!p) return;
    if (use_sync_alloc()) {
        (void)hipFree(p);
    } else if (hipFreeAsync(p, s) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(p);
    }
}

struct Staging {
    void* p = nullptr;
    size_t bytes = 0;
    ~Staging() { if (p) (void)hipHostFree(p); }
};

fx_status host_staging(void** p, size_t bytes) {
    static thread_local Staging st;
    if (st.bytes < bytes) {
        if (st.p) (void)hipHostFree(st.p);
        st.p = nullptr;
        size_t want = bytes < 65536 ? 65536 : bytes;
        hipError_t e = hipHostMalloc(&st.p, want, hipHostMallocDefault);
        if (e != hipSuccess) {
            st.bytes = 0;
            set_error("pinned host allocation of %zu bytes failed: %s", want, hipGetErrorString(e));
            return FX_ENOMEM;
        }
        st.bytes = want;
    }
    *p = st.p;
    return FX_OK;
}

// ---------------------------------------------------------------------------------- profiler
struct ProfRec { int slot; hipEvent_t a, b; };
static std::atomic<bool> g_prof_on{false};
static std::mutex g_prof_mu;
static std::vector<ProfRec> g_prof_open;     // begun, not yet ended
static std::vector<ProfRec> g_prof_done;
static double g_prof_ms[kProfSlotCount];
static long long g_prof_count[kProfSlotCount];

bool prof_enabled() { return g_prof_on.load(std::memory_order_relaxed); }

void prof_begin(int slot, hipStream_t s) {
    ProfRec r{slot, nullptr, nullptr};
    if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
    (void)hipEventRecord(r.a, s);
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_open.push_back(r);
}

void prof_end(int slot, hipStream_t s) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (size_t i = g_prof_open.size(); i-- > 0;) {
        if (g_prof_open[i].slot == slot) {
            ProfRec r = g_prof_open[i];
            g_prof_open.erase(g_prof_open.begin() + (long)i);
            (void)hipEventRecord(r.b, s);
            g_prof_done.push_back(r);
            return;
        }
    }
}

static void prof_drain() {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (ProfRec& r : g_prof_done) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
            g_prof_ms[r.slot] += ms;
            g_prof_count[r.slot] += 1;
        }
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_prof_done.clear();
}

static const char* kProfNames[kProfSlotCount] = {
    "k_find_tiles", "k_rank_tiles", "k_insert<0>", "scan_upper", "k_insert<1>", "scan_lower", "k_insert<2>",
    "scan_leaves", "k_vox_base", "k_grid_ijk", "k_nbmap", "k_leaf_neighbors", "k_build_tiles", "k_pack_weights",
    "k_conv_mfma",
    "k_conv_scalar", "memset"};

}  // namespace fx

extern "C" void fx_profile_enable(int on) { fx::g_prof_on.store(on != 0); }

extern "C" void fx_profile_reset(void) {
    fx::prof_drain();
    for (int i = 0; i < fx::kProfSlotCount; ++i) { fx::g_prof_ms[i] = 0; fx::g_prof_count[i] = 0; }
}

extern "C" int fx_profile_slot_count(void) { return fx::kProfSlotCount; }

extern "C" const char* fx_profile_slot_name(int slot) {
    return (slot >= 0 && slot < fx::kProfSlotCount) ? fx::kProfNames[slot] : "";
}

extern "C" fx_status fx_profile_read(int slot, double* total_ms, int64_t* count) {
    if (slot < 0 || slot >= fx::kProfSlotCount) { fx::set_error("fx_profile_read: bad slot"); return FX_EINVAL; }
    fx::prof_drain();
    if (total_ms) *total_ms = fx::g_prof_ms[slot];
    if (count) *count = fx::g_prof_count[slot];
    return FX_OK;
}

extern "C" const char* fx_version(void) { return "fvdb-hotpath-gfx950 0.1"; }

extern "C" const char* fx_last_error(void) { return fx::g_err; }

extern "C" fx_status fx_init(void) {
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || n <= 0) {
        fx::set_error("no HIP device: %s", e == hipSuccess ? "device count is 0" : hipGetErrorString(e));
        return FX_EDEVICE;
    }
    return FX_OK;
}
