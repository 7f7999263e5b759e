// Internal declarations shared by the translation units of libround_attention (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>

#include "round_attention.h"

namespace ra {

// ---- error reporting ------------------------------------------------------------------------
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
#define RA_HIP_CHECK(expr)                                                                      \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess) return ::ra::fail(RA_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)
#define RA_REQUIRE(cond, code, ...)                      \
    do {                                                 \
        if (!(cond)) return ::ra::fail(code, __VA_ARGS__); \
    } while (0)

// ---- context ---------------------------------------------------------------------------------
struct Workspace {
    char* base = nullptr;
    size_t bytes = 0;
};

}  // namespace ra

struct ra_ctx {
    int device = 0;
    int num_cu = 256;
    ra::Workspace ws;
    int prefill_p_half = 0;  // ra_set_prefill_precision
    // kernel timing on request (ra_profile_kernels)
    bool profile = false, timed = false;
    hipEvent_t ev_start = nullptr, ev_stop = nullptr;
};

namespace ra {
// While a KernelTimer is alive on a profiling context, RA_LAUNCH_TIMED hands the context's two events to the
// launch itself, so that they carry the kernel's own start and end time stamps (no extra packets on the stream).
extern thread_local ra_ctx* g_timed_ctx;
struct KernelTimer {
    ra_ctx* prev;
    KernelTimer(ra_ctx* ctx, hipStream_t) : prev(g_timed_ctx) { g_timed_ctx = ctx->profile ? ctx : nullptr; }
    ~KernelTimer() { g_timed_ctx = prev; }
};
}  // namespace ra

// Launch of a streaming kernel (the one ra_profile_last_ms reports).
#define RA_LAUNCH_TIMED(kernel, grid, block, smem, st, ...)                                                      \
    do {                                                                                                         \
        if (::ra::g_timed_ctx) {                                                                                 \
            hipExtLaunchKernelGGL(kernel, grid, block, (std::uint32_t)(smem), st, ::ra::g_timed_ctx->ev_start,    \
                                  ::ra::g_timed_ctx->ev_stop, 0, __VA_ARGS__);                                   \
            ::ra::g_timed_ctx->timed = true;                                                                     \
        } else {                                                                                                 \
            hipLaunchKernelGGL(kernel, grid, block, smem, st, __VA_ARGS__);                                      \
        }                                                                                                        \
    } while (0)

namespace ra {

// View as the kernels see it (passed by value).
struct DevView {
    const void* k;
    const void* v;
    const int64_t* seg_off;
    const int64_t* seg_off_v;
    const int32_t* seg_len;
    const int32_t* n_rounds;
    const int32_t* block_table;
    int32_t block_size, max_blocks, B, R_max, Hkv, d;
};

int check_view(const ra_kv_view* v, bool need_v, const char* who);
int static_scratch_init(int device);  // decode.hip: device address of the built-in scratch of the no-allocation entry point
DevView to_dev(const ra_kv_view* v);

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Number of KV splits the decode / prefill launchers use for a given shape.
int decode_splits(int num_cu, int B, int Hkv, int64_t max_tokens);

constexpr int kUnitTokens = 16;   // tokens per work unit of the streaming kernels (= one paged block)
constexpr int kMaxRounds = 1024;  // largest R_max any entry point accepts
constexpr int kMaxBatch = 1024;   // largest batch of the matrix-core attention kernels (their schedule lives in LDS)
// Head of the workspace kept for small integer state (ra_set_workspace clears it once; nothing relies on that):
//   [0, 16384)       pieces every sequence was cut into by the last generic / many-row attention call
//   [16384, 24576)   first record and number of records of every sequence, matrix-core decode kernel
//   last 64 bytes    a spare word for the bandwidth probe
constexpr size_t kWsSmallState = 16384;
constexpr size_t kWsSeqRecOff = 16384;
constexpr size_t kWsReserved = 32768;

// ---- device helpers --------------------------------------------------------------------------
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;  // finite stand-in for "no score yet" (keeps max/exp free of inf - inf)

}  // namespace ra
