// Optional phase timestamps for kernel tuning.  Compiled out unless the library is built with
// -DRA_DEBUG_TS.  Each translation unit that uses RA_TS gets its own buffer and exports a reader
// through RA_TS_DEFINE_READER(name): int name(long long* host, int n).
#pragma once

#include <hip/hip_runtime.h>

#ifdef RA_DEBUG_TS
namespace ra {
constexpr int kDbgWorkgroups = 8192, kDbgSlots = 16;
static __device__ long long dbg_ts[kDbgWorkgroups * kDbgSlots];
}  // namespace ra
#define RA_TS(k)                                                                                        \
    do {                                                                                                \
        const int wg_ = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;                 \
        if (threadIdx.x == 0 && wg_ < ::ra::kDbgWorkgroups)                                             \
            ::ra::dbg_ts[wg_ * ::ra::kDbgSlots + (k)] = wall_clock64();                                 \
    } while (0)
#define RA_TS_DEFINE_READER(name)                                                                       \
    extern "C" int name(long long* host, int n) {                                                       \
        return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(::ra::dbg_ts), (size_t)n * sizeof(long long)); \
    }
// Lap accumulators (thread 0's view): RA_LAP(i) adds the clock ticks since the previous lap to lap i.
#define RA_LAP_DECL long long lap_[8] = {0, 0, 0, 0, 0, 0, 0, 0}, lap_t_ = 0
#define RA_LAP_START lap_t_ = clock64()
#define RA_LAP(i)                          \
    do {                                   \
        const long long now_ = clock64();  \
        lap_[i] += now_ - lap_t_;          \
        lap_t_ = now_;                     \
    } while (0)
#define RA_LAP_COUNT(i, v) lap_[i] += (v)
#define RA_LAP_FLUSH(first)                                                              \
    do {                                                                                 \
        const int wg_ = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;  \
        if (threadIdx.x == 0 && wg_ < ::ra::kDbgWorkgroups)                              \
            for (int i_ = 0; i_ < 8; ++i_) ::ra::dbg_ts[wg_ * ::ra::kDbgSlots + (first) + i_] = lap_[i_]; \
    } while (0)
#else
#define RA_TS(k)
#define RA_TS_DEFINE_READER(name)
#define RA_LAP_DECL
#define RA_LAP_START
#define RA_LAP(i)
#define RA_LAP_COUNT(i, v)
#define RA_LAP_FLUSH(first)
#endif
