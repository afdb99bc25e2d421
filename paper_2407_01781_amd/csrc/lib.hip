// Library-wide plumbing: error text, device allocation, pinned staging, version.
#include "common.h"

#include <stdarg.h>
#include <stdlib.h>

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

}  // namespace fx

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
