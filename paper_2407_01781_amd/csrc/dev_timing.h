// Development-only cycle stamps for the kernels of this library.  Everything here compiles to nothing unless
// the translation unit is built with -DFX_DEV_TIMING; product builds carry no instrumentation.
//
//   FX_STAMP(slot)            thread 0 of a workgroup records the cycle counter in slot 0..15 of its row
//   FX_STAMP_HWID(slot)       ... the hardware id register (compute unit, shader engine) and, in slot + 1, the XCC id
//   FX_CYCLES_BEGIN()         start of a timed stretch (declares a local)
//   FX_CYCLES_ADD(var)        adds the cycles since FX_CYCLES_BEGIN() to var
//   FX_DEV_TIMING_EXPORT(fn)  defines  extern "C" int fn(unsigned long long* h_out, size_t bytes)  that copies the
//                             translation unit's stamp buffer to the host
#pragma once

#ifdef FX_DEV_TIMING
#include <hip/hip_runtime.h>
namespace fx { namespace devt {
constexpr int kRows = 4096, kSlots = 16;
static __device__ unsigned long long g_stamps[kRows * kSlots];
} }
#define FX_STAMP(slot)                                                                                 \
    do {                                                                                               \
        if (threadIdx.x == 0 && blockIdx.x < fx::devt::kRows)                                          \
            fx::devt::g_stamps[blockIdx.x * fx::devt::kSlots + (slot)] = __builtin_readcyclecounter(); \
    } while (0)
#define FX_STAMP_HWID(slot)                                                                            \
    do {                                                                                               \
        if (threadIdx.x == 0 && blockIdx.x < fx::devt::kRows) {                                        \
            fx::devt::g_stamps[blockIdx.x * fx::devt::kSlots + (slot)] = __builtin_amdgcn_s_getreg((31 << 11) | 4);      \
            fx::devt::g_stamps[blockIdx.x * fx::devt::kSlots + (slot) + 1] = __builtin_amdgcn_s_getreg((31 << 11) | 20); \
        }                                                                                              \
    } while (0)
#define FX_STAMP_VALUE(row, slot, v)                                                                   \
    do { if ((row) < fx::devt::kRows) fx::devt::g_stamps[(row) * fx::devt::kSlots + (slot)] = (v); } while (0)
#define FX_CYCLES_BEGIN() const unsigned long long _fx_t0 = __builtin_readcyclecounter()
#define FX_CYCLES_ADD(var) var += __builtin_readcyclecounter() - _fx_t0
#define FX_CYCLES_NOW() __builtin_readcyclecounter()
#define FX_DEV_TIMING_EXPORT(fn)                                                                       \
    extern "C" int fn(unsigned long long* h_out, size_t bytes) {                                       \
        return (int)hipMemcpyFromSymbol(h_out, HIP_SYMBOL(fx::devt::g_stamps), bytes);                 \
    }
#else
#define FX_STAMP(slot) do { } while (0)
#define FX_STAMP_HWID(slot) do { } while (0)
#define FX_STAMP_VALUE(row, slot, v) do { } while (0)
#define FX_CYCLES_BEGIN() do { } while (0)
#define FX_CYCLES_ADD(var) do { } while (0)
#define FX_CYCLES_NOW() 0ull
#define FX_DEV_TIMING_EXPORT(fn)
#endif
