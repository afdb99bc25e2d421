// Library-wide plumbing: error text, device allocation, pinned staging, version.
#include "conv_common.h"

#include <stdarg.h>
#include <stdlib.h>
#include <string.h>

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

// ---------------------------------------------------------------------------------- options
static std::atomic<int> g_options[kOptCount] = {};          // stored as value + 1, so that zero-initialised = automatic
static const char* const kOptionNames[kOptCount] = {"force_scalar", "leaf_dispatch", "fp32_tiles", "conv_gather", "gather_lds",
                                                    "scalar_lds",   "grid_direct",   "leaf_links", "cache_mb",   "sync_alloc"};
int option(Option o) { return g_options[o].load(std::memory_order_relaxed) - 1; }

// Device memory.  With a caller's allocator set (fx_set_allocator) every block comes from it and goes back to it.
// Otherwise blocks come from a cache owned by the library: a freed block is kept and handed to the next request
// of a similar size, so steady-state calls (same shapes every step) never reach the driver -- hipMallocAsync /
// hipFreeAsync cost 70-300 us per call here.  All work of this library is stream-ordered, so a block released on
// stream S can be reused at once by later work on S; reuse from another stream first waits for the device.
// Option sync_alloc = 1 switches to plain hipMalloc / hipFree; option cache_mb bounds the bytes kept (2048 by
// default).
static fx_alloc_fn g_user_alloc = nullptr;
static fx_free_fn g_user_free = nullptr;
static void* g_user_ctx = nullptr;

static int use_sync_alloc() { return option(kOptSyncAlloc) == 1; }

struct Block { void* p; size_t bytes; hipStream_t stream; int device; };
static std::mutex g_mem_mu;
static std::vector<Block> g_mem_free;              // cached, oldest first
static std::vector<Block> g_mem_live;
static size_t g_mem_cached = 0;

static size_t cache_limit() {
    const int mb = option(kOptCacheMb);
    return (size_t)(mb >= 0 ? mb : 2048) << 20;
}

static size_t round_size(size_t bytes) {   // at most 12.5 % above the request, few distinct sizes
    if (bytes < 4096) return 4096;
    size_t p2 = (size_t)1 << (63 - __builtin_clzll((unsigned long long)bytes));
    const size_t step = p2 >> 3;
    return (bytes + step - 1) / step * step;
}

static void release_cached_locked() {
    for (auto& b : g_mem_free) (void)hipFree(b.p);
    g_mem_free.clear();
    g_mem_cached = 0;
}

fx_status dev_alloc(void** p, size_t bytes, hipStream_t s) {
    *p = nullptr;
    if (g_user_alloc) {
        *p = g_user_alloc(bytes ? bytes : 256, (void*)s, g_user_ctx);
        if (!*p) { set_error("the caller's allocator returned no memory for %zu bytes", bytes); return FX_ENOMEM; }
        return FX_OK;
    }
    if (use_sync_alloc()) {
        hipError_t e = hipMalloc(p, bytes ? bytes : 256);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            set_error("device allocation of %zu bytes failed: %s", bytes, hipGetErrorString(e));
            return e == hipErrorOutOfMemory ? FX_ENOMEM : FX_EDEVICE;
        }
        return FX_OK;
    }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { set_error("hipGetDevice failed"); return FX_EDEVICE; }
    const size_t need = round_size(bytes);
    std::lock_guard<std::mutex> lock(g_mem_mu);
    int best = -1;
    for (int i = 0; i < (int)g_mem_free.size(); ++i) {
        const Block& b = g_mem_free[i];
        if (b.device != dev || b.bytes < need || b.bytes > 2 * need) continue;
        if (best < 0 || b.bytes < g_mem_free[best].bytes || (b.bytes == g_mem_free[best].bytes && b.stream == s)) best = i;
    }
    Block blk;
    if (best >= 0) {
        blk = g_mem_free[best];
        g_mem_free.erase(g_mem_free.begin() + best);
        g_mem_cached -= blk.bytes;
        if (blk.stream != s && hipDeviceSynchronize() != hipSuccess) {
            (void)hipFree(blk.p);
            set_error("hipDeviceSynchronize failed while reusing a cached block");
            return FX_EDEVICE;
        }
        blk.stream = s;
    } else {
        hipError_t e = hipMalloc(&blk.p, need);
        if (e == hipErrorOutOfMemory) {       // give the cache back and try once more
            (void)hipGetLastError();
            release_cached_locked();
            e = hipMalloc(&blk.p, need);
        }
        if (e != hipSuccess) {
            (void)hipGetLastError();
            set_error("device allocation of %zu bytes failed: %s", need, hipGetErrorString(e));
            return e == hipErrorOutOfMemory ? FX_ENOMEM : FX_EDEVICE;
        }
        blk.bytes = need; blk.stream = s; blk.device = dev;
    }
    g_mem_live.push_back(blk);
    *p = blk.p;
    return FX_OK;
}

void dev_free(void* p, hipStream_t s) {
    if (!p) return;
    std::lock_guard<std::mutex> lock(g_mem_mu);
    for (int i = (int)g_mem_live.size() - 1; i >= 0; --i) {
        if (g_mem_live[i].p != p) continue;
        Block blk = g_mem_live[i];
        g_mem_live[i] = g_mem_live.back();
        g_mem_live.pop_back();
        blk.stream = s;
        g_mem_free.push_back(blk);
        g_mem_cached += blk.bytes;
        while (g_mem_cached > cache_limit() && !g_mem_free.empty()) {   // hipFree waits for the device
            g_mem_cached -= g_mem_free.front().bytes;
            (void)hipFree(g_mem_free.front().p);
            g_mem_free.erase(g_mem_free.begin());
        }
        return;
    }
    // not a block of the cache: the caller's allocator's, or a plain hipMalloc (sync_alloc)
    if (g_user_free) g_user_free(p, (void*)s, g_user_ctx);
    else (void)hipFree(p);
}

}  // namespace fx
extern "C" void fx_release_cached_memory(void) {
    std::lock_guard<std::mutex> lock(fx::g_mem_mu);
    (void)hipDeviceSynchronize();
    fx::release_cached_locked();
}
namespace fx {

struct Staging {
    void* p = nullptr;
    size_t bytes = 0;
    ~Staging() { if (p) (void)hipHostFree(p); }
};

fx_status host_staging(void** p, size_t bytes, int area) {
    static thread_local Staging areas[2];
    Staging& st = areas[area & 1];
    if (st.bytes < bytes) {
        if (st.p) {
            (void)hipDeviceSynchronize();   // an upload from the old area may still be in flight
            (void)hipHostFree(st.p);
        }
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


int compute_units() {
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n_cu = prop.multiProcessorCount;
        if (n_cu <= 0) n_cu = 256;
    }
    return n_cu;
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
    "k_bucket_count", "k_bucket_scan", "k_bucket_scatter", "k_bucket_leaves", "k_voxels_to_leaves", "k_find_tiles", "k_rank_tiles", "k_insert<0>", "scan_upper", "k_insert<1>", "scan_lower", "k_insert<2>",
    "scan_leaves", "k_grid_ijk", "k_nbmap", "k_leaf_neighbors", "k_build_tiles", "k_pack_weights",
    "k_conv_mfma", "k_conv_gather",
    "k_conv_scalar", "memset", "k_dgrad_strided", "k_wgrad", "k_wgrad_reduce", "k_pool2", "k_upsample2", "k_conv_leaf", "k_points_to_ijk"};

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

extern "C" fx_status fx_set_allocator(fx_alloc_fn alloc, fx_free_fn release, void* ctx) {
    if ((alloc == nullptr) != (release == nullptr)) { fx::set_error("fx_set_allocator: both functions or neither"); return FX_EINVAL; }
    std::lock_guard<std::mutex> lock(fx::g_mem_mu);
    fx::g_user_alloc = alloc; fx::g_user_free = release; fx::g_user_ctx = ctx;
    return FX_OK;
}

extern "C" fx_status fx_set_option(const char* name, int32_t value) {
    if (!name || value < -1) { fx::set_error("fx_set_option: null name or value below -1"); return FX_EINVAL; }
    for (int o = 0; o < fx::kOptCount; ++o)
        if (!strcmp(name, fx::kOptionNames[o])) { fx::g_options[o].store(value + 1); return FX_OK; }
    fx::set_error("fx_set_option: unknown option '%s'", name);
    return FX_EINVAL;
}

extern "C" fx_status fx_get_option(const char* name, int32_t* value) {
    if (!name || !value) { fx::set_error("fx_get_option: null pointer"); return FX_EINVAL; }
    for (int o = 0; o < fx::kOptCount; ++o)
        if (!strcmp(name, fx::kOptionNames[o])) { *value = fx::option((fx::Option)o); return FX_OK; }
    fx::set_error("fx_get_option: unknown option '%s'", name);
    return FX_EINVAL;
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
    return fx::conv_noalloc_setup(nullptr);     // the static scratch buffer's address on the current device
}
