// Context, workspace and argument checking of libround_attention.
#include "common.hpp"
#include "stream_kv.hpp"

#include <stdarg.h>
#include <stdio.h>
#include <new>

namespace ra {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_view(const ra_kv_view* v, bool need_v, const char* who) {
    RA_REQUIRE(v != nullptr, RA_ERR_INVALID_ARG, "%s: view is NULL", who);
    RA_REQUIRE(v->B > 0 && v->R_max >= 0 && v->Hkv > 0 && v->d > 0, RA_ERR_INVALID_ARG,
               "%s: view needs B > 0, R_max >= 0, Hkv > 0, d > 0 (got %d, %d, %d, %d)", who, v->B, v->R_max, v->Hkv,
               v->d);
    RA_REQUIRE(v->R_max <= kMaxRounds, RA_ERR_UNSUPPORTED, "%s: R_max %d exceeds %d", who, v->R_max, kMaxRounds);
    RA_REQUIRE(v->dtype == RA_F32 || v->dtype == RA_BF16, RA_ERR_UNSUPPORTED, "%s: unknown dtype %d", who, v->dtype);
    RA_REQUIRE(v->n_rounds != nullptr, RA_ERR_INVALID_ARG, "%s: view.n_rounds is NULL", who);
    if (v->R_max > 0) {
        RA_REQUIRE(v->k != nullptr, RA_ERR_INVALID_ARG, "%s: view.k is NULL", who);
        RA_REQUIRE(!need_v || v->v != nullptr, RA_ERR_INVALID_ARG, "%s: view.v is NULL", who);
        RA_REQUIRE(v->seg_off != nullptr && v->seg_len != nullptr, RA_ERR_INVALID_ARG,
                   "%s: view.seg_off / seg_len is NULL", who);
    }
    RA_REQUIRE(v->block_size == 0 || v->block_size == kUnitTokens, RA_ERR_UNSUPPORTED,
               "%s: block_size must be 0 or %d (got %d)", who, kUnitTokens, v->block_size);
    if (v->block_size != 0 && v->R_max > 0) {
        RA_REQUIRE(v->block_table != nullptr && v->max_blocks > 0, RA_ERR_INVALID_ARG,
                   "%s: paged view needs block_table and max_blocks > 0", who);
    }
    RA_REQUIRE(v->max_tokens >= 0, RA_ERR_INVALID_ARG, "%s: view.max_tokens is negative", who);
    return RA_OK;
}

DevView to_dev(const ra_kv_view* v) {
    DevView d;
    d.k = v->k;
    d.v = v->v;
    d.seg_off = v->seg_off;
    d.seg_off_v = v->seg_off_v ? v->seg_off_v : v->seg_off;
    d.seg_len = v->seg_len;
    d.n_rounds = v->n_rounds;
    d.block_table = v->block_table;
    d.block_size = v->block_size;
    d.max_blocks = v->max_blocks;
    d.B = v->B;
    d.R_max = v->R_max;
    d.Hkv = v->Hkv;
    d.d = v->d;
    return d;
}

int decode_splits(int num_cu, int B, int Hkv, int64_t max_tokens) {
    // Aim for about 8 workgroups per compute unit so that uneven selections even out, but never
    // cut a sequence into pieces of fewer than 128 tokens (two 16-token units per wave).
    const int64_t target = (int64_t)num_cu * 8;
    int64_t s = (target + (int64_t)B * Hkv - 1) / ((int64_t)B * Hkv);
    int64_t cap = max_tokens / 128;
    if (cap < 1) cap = 1;
    if (s > cap) s = cap;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    return (int)s;
}

thread_local ra_ctx* g_timed_ctx = nullptr;

}  // namespace ra

using namespace ra;

extern "C" {

const char* ra_last_error(void) { return g_err; }

int ra_create(ra_ctx** out, int device) {
    RA_REQUIRE(out != nullptr, RA_ERR_INVALID_ARG, "ra_create: out is NULL");
    *out = nullptr;
    int n = 0;
    RA_HIP_CHECK(hipGetDeviceCount(&n));
    RA_REQUIRE(device >= 0 && device < n, RA_ERR_INVALID_ARG, "ra_create: device %d out of range (%d devices)", device,
               n);
    hipDeviceProp_t prop;
    RA_HIP_CHECK(hipGetDeviceProperties(&prop, device));
    if (int rc = static_scratch_init(device)) return rc;
    ra_ctx* c = new (std::nothrow) ra_ctx();
    RA_REQUIRE(c != nullptr, RA_ERR_OOM, "ra_create: out of host memory");
    c->device = device;
    c->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    *out = c;
    return RA_OK;
}

int ra_destroy(ra_ctx* ctx) {
    if (ctx) {
        if (ctx->ev_start) (void)hipEventDestroy(ctx->ev_start);
        if (ctx->ev_stop) (void)hipEventDestroy(ctx->ev_stop);
    }
    delete ctx;
    return RA_OK;
}

int ra_profile_kernels(ra_ctx* ctx, int enable) {
    RA_REQUIRE(ctx != nullptr, RA_ERR_INVALID_ARG, "ra_profile_kernels: ctx is NULL");
    if (enable && !ctx->ev_start) {
        RA_HIP_CHECK(hipEventCreate(&ctx->ev_start));
        RA_HIP_CHECK(hipEventCreate(&ctx->ev_stop));
    }
    ctx->profile = enable != 0;
    ctx->timed = false;
    return RA_OK;
}

int ra_profile_last_ms(ra_ctx* ctx, float* ms_out) {
    RA_REQUIRE(ctx != nullptr && ms_out != nullptr, RA_ERR_INVALID_ARG, "ra_profile_last_ms: NULL argument");
    RA_REQUIRE(ctx->profile && ctx->timed, RA_ERR_STATE,
               "ra_profile_last_ms: no profiled call since ra_profile_kernels(ctx, 1)");
    RA_HIP_CHECK(hipEventSynchronize(ctx->ev_stop));
    RA_HIP_CHECK(hipEventElapsedTime(ms_out, ctx->ev_start, ctx->ev_stop));
    return RA_OK;
}

namespace ra {
// Plain streaming read: every wave streams its own contiguous span with non-temporal 16-byte loads (1 KB per load
// instruction, sixteen in flight), everything folded into one word per wave so that the loads cannot be dropped.  What
// this reaches is the practical ceiling the streaming kernels are compared with.  Measured on one MI355X over 4 GiB:
// this form 7.0-7.15 TB/s with one to eight workgroups per compute unit (eight loads in flight: 6.9-7.05); the same
// with ordinary loads 6.0-6.2; grid-stride with ordinary loads 5.5-5.9, with non-temporal loads 5.9-6.5.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ p, size_t n, unsigned* __restrict__ sink) {
    constexpr int kInFlight = 16;
    const size_t waves = (size_t)gridDim.x * 4, w = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const size_t per = (n / waves) & ~(size_t)63;  // 16-byte words per wave, whole kilobytes
    const int lane = threadIdx.x & 63;
    const uint4* q = p + w * per + lane;
    unsigned acc = 0;
    size_t i = 0;
    for (; i + (size_t)kInFlight * 64 <= per; i += (size_t)kInFlight * 64) {
        uint4 v[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) v[u] = ra::load_once(q + i + u * 64);
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < per; i += 64) {
        const uint4 a = ra::load_once(q + i);
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    // what the equal spans leave over at the end of the buffer, by the whole grid
    for (size_t r = waves * per + (size_t)blockIdx.x * 256 + threadIdx.x; r < n; r += (size_t)gridDim.x * 256) {
        const uint4 a = p[r];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o, 64);
    if (lane == 0 && acc == 0x9e3779b9u) atomicAdd(sink, 1u);  // (practically never taken)
}
}  // namespace ra

int ra_measure_read_bandwidth(ra_ctx* ctx, void* stream, const void* device_buf, size_t bytes, int iters,
                              float* gb_per_s) {
    RA_REQUIRE(ctx != nullptr && device_buf != nullptr && gb_per_s != nullptr, RA_ERR_INVALID_ARG,
               "ra_measure_read_bandwidth: NULL argument");
    RA_REQUIRE(bytes >= 16 && bytes % 16 == 0 && ((uintptr_t)device_buf & 15) == 0 && iters > 0, RA_ERR_INVALID_ARG,
               "ra_measure_read_bandwidth: needs a 16-byte aligned buffer of a multiple of 16 bytes and iters > 0");
    RA_REQUIRE(ctx->ws.base != nullptr && ctx->ws.bytes >= kWsReserved, RA_ERR_WORKSPACE,
               "ra_measure_read_bandwidth: no workspace set");
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    hipEvent_t e0, e1;
    RA_HIP_CHECK(hipEventCreate(&e0));
    RA_HIP_CHECK(hipEventCreate(&e1));
    unsigned* sink = reinterpret_cast<unsigned*>(ctx->ws.base + kWsReserved - 64);  // a spare word of the reserved head
    const dim3 grid(ctx->num_cu * 2), block(256);  // two workgroups per compute unit (1, 2, 3, 4 and 8 measured alike)
    hipLaunchKernelGGL(ra::stream_read_kernel, grid, block, 0, st, static_cast<const uint4*>(device_buf), bytes / 16, sink);
    hipError_t e = hipEventRecord(e0, st);
    for (int i = 0; i < iters && e == hipSuccess; ++i)
        hipLaunchKernelGGL(ra::stream_read_kernel, grid, block, 0, st, static_cast<const uint4*>(device_buf), bytes / 16,
                           sink);
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return fail(RA_ERR_HIP, "ra_measure_read_bandwidth: %s", hipGetErrorString(e));
    *gb_per_s = ms > 0.f ? (float)((double)bytes * iters / (ms * 1e-3) / 1e9) : 0.f;
    return RA_OK;
}

int ra_workspace_bytes(const ra_problem* p, size_t* bytes_out) {
    RA_REQUIRE(p != nullptr && bytes_out != nullptr, RA_ERR_INVALID_ARG, "ra_workspace_bytes: NULL argument");
    RA_REQUIRE(p->B > 0 && p->R_max >= 0 && p->Hq > 0 && p->Hkv > 0 && p->d > 0 && p->q_len_max > 0 &&
                   p->max_tokens >= 0,
               RA_ERR_INVALID_ARG, "ra_workspace_bytes: non-positive dimension");
    RA_REQUIRE(p->Hq % p->Hkv == 0, RA_ERR_INVALID_ARG, "ra_workspace_bytes: Hq %% Hkv != 0");
    const size_t rows = (size_t)p->B * p->q_len_max * p->Hq;
    // attention partials: up to 64 splits of (d accumulators + running max + running sum) per output row
    size_t attn = rows * 64 * ((size_t)p->d + 2) * sizeof(float);
    // ... or, in the matrix-core kernel for few query rows, one partial result of 16 rows per (range, KV head, row
    // block) and per (sequence, KV head, row block): at most 4096 wavefronts with a range each, and never more
    // ranges than half the batch's 32-token key tiles
    const size_t inner2 = (size_t)p->Hkv * 2;
    size_t slots = ((size_t)p->B * ((size_t)(p->max_tokens / 32) + p->R_max + 2) / 2 + 1) * inner2;
    if (slots > 4096) slots = 4096;
    const size_t few = (slots + (size_t)p->B * inner2) * 16 * ((size_t)p->d + 2) * sizeof(float) + 512;
    if (few > attn) attn = few;
    // score intermediates: one log-sum-exp per (row, 256-token chunk), plus up to eight partial per-head score rows
    const size_t chunks = (size_t)(p->max_tokens / 256) + p->R_max + 2;
    // and a 16-byte descriptor per (sequence, chunk)
    const size_t sc = rows * chunks * sizeof(float) + (size_t)8 * p->B * p->Hq * p->R_max * sizeof(float) + 256 +
                      (size_t)p->B * chunks * 16 + 256;
    // decode at the watershed layer keeps, besides the attention partials, one log-sum-exp per (row, 32-token tile)
    const size_t tiles = (size_t)(p->max_tokens / 32) + p->R_max + 2;
    const size_t fused = align_up(attn, 256) + align_up(rows * tiles * sizeof(float), 256) +
                         (size_t)8 * p->B * p->Hq * p->R_max * sizeof(float) + 512;
    size_t both = align_up(attn, 256) > align_up(sc, 256) + 256 ? align_up(attn, 256) : align_up(sc, 256) + 256;
    if (fused > both) both = fused;
    const size_t plan = (size_t)p->B * (((size_t)(p->R_max + 1) * 24 + 4 + 16 + 15) & ~(size_t)15);
    *bytes_out = kWsReserved + align_up(plan, 256) + both + 3 * 256;
    return RA_OK;
}

int ra_set_workspace(ra_ctx* ctx, void* device_ptr, size_t bytes) {
    RA_REQUIRE(ctx != nullptr, RA_ERR_INVALID_ARG, "ra_set_workspace: ctx is NULL");
    RA_REQUIRE(device_ptr != nullptr || bytes == 0, RA_ERR_INVALID_ARG, "ra_set_workspace: NULL pointer with bytes > 0");
    RA_REQUIRE(((uintptr_t)device_ptr & 255u) == 0, RA_ERR_INVALID_ARG, "ra_set_workspace: pointer not 256-byte aligned");
    RA_REQUIRE(bytes == 0 || bytes >= kWsReserved, RA_ERR_WORKSPACE,
               "ra_set_workspace: a workspace must have at least %zu bytes", kWsReserved);
    if (bytes) RA_HIP_CHECK(hipMemset(device_ptr, 0, kWsReserved));
    ctx->ws.base = (char*)device_ptr;
    ctx->ws.bytes = bytes;
    return RA_OK;
}

}  // extern "C"
