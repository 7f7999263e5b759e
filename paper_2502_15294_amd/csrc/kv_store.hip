// Round-indexed KV store for the post-watershed layers (paper Sec. 3.2 and Fig. 1: the "upper half"
// u_m of every round stays in host memory as one tensor; the tensors of the selected rounds are
// moved to the GPU, each in one transfer, once the selection is known).
//
// Mostly host side: a registry of pinned per-round tensors, a bump-allocated device pool, the index
// tables of the compact per-layer views, and the hipMemcpyAsync / event choreography on a side
// stream.  The copied bytes keep the host layout: per layer the keys [Hkv][len][d] followed by the
// values in transposed 16-token tiles [Hkv][ceil(len/16)][d][16].  Every slice is therefore already a
// round block in the device layout and staging needs no repacking kernel.
//
// The one kernel here runs at the end of a turn (Sec. 3.2, last step; Alg. 1, last line): it gathers
// the new round's token-major keys and values of every post-watershed layer into that round layout
// behind the staged rounds in the pool, from where each sequence's new round leaves for host memory
// in one copy.  The registry also counts how often each round was staged, which is what KV-cache
// dropping (Sec. 3.4) decides on.
#include "common.hpp"

#include <new>
#include <vector>

struct ra_kv_store {
    ra_store_cfg cfg;
    size_t token_bytes = 0;  // bytes of one token of one layer of K (or V): Hkv * d * elem
    struct Round {
        const char* host = nullptr;
        int len = -1;  // -1 = never registered
        uint32_t turns = 0, hits = 0;  // stage calls since registration / of those, the ones that selected it
        bool dropped = false;
    };
    std::vector<Round> rounds;  // [B][R_max]
    char* pool = nullptr;
    // index tables: host pinned mirror and device copy
    int64_t* h_off = nullptr;  // [n_layers][2][B][R_max]
    int32_t* h_len = nullptr;  // [B][R_max]
    int32_t* h_n = nullptr;    // [B]
    int64_t* d_off = nullptr;
    int32_t* d_len = nullptr;
    int32_t* d_n = nullptr;
    std::vector<hipEvent_t> ready;
    bool staged = false;
    int64_t max_tokens = 0;
    size_t staged_tok = 0;  // pool cursor behind the staged rounds, in units of token_bytes
    // turn-end write-back of the new round: placement table (pinned mirror + device copy) and events
    int64_t* h_wb_off = nullptr;  // [B] start of the round's tensor in the pool, in tokens; -1 = skip
    int32_t* h_wb_len = nullptr;  // [B]
    int64_t* d_wb_off = nullptr;
    int32_t* d_wb_len = nullptr;
    hipEvent_t wb_packed = nullptr, wb_done = nullptr;
    bool wb_pending = false;
    uint64_t saved_bytes = 0;
    uint64_t staged_bytes = 0, n_copies = 0;
};

using namespace ra;

// Tokens' worth of storage of one layer of one round: len rows of keys plus the values padded to
// whole 16-token tiles.
static inline size_t layer_tokens(int len) { return (size_t)len + (size_t)((len + 15) / 16) * 16; }

// Layers in group gi of the grouped staging order for L layers: first max(1, L / 8); last 1; the layers in
// between in three groups as equal as possible (fewer when there are fewer layers).
static int grouped_stage_size(int L, int gi) {
    const int first = L / 8 > 1 ? L / 8 : 1;
    if (gi == 0) return first < L ? first : L;
    const int middle = L - first - 1;                 // layers between the first group and the last layer
    const int n_mid = middle < 3 ? (middle > 0 ? middle : 0) : 3;
    if (gi <= n_mid) return middle / n_mid + (gi <= middle % n_mid ? 1 : 0);
    return 1;
}

static bool is_pinned_host(const void* p) {
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();  // ordinary pageable memory: not an error of ours, clear the sticky code
        return false;
    }
    return attr.type == hipMemoryTypeHost;
}

namespace {
constexpr int kRepackThreads = 256;

template <typename T>
union Vec16 {
    uint4 u;
    T e[16 / sizeof(T)];
};

// Turn-end gather of one layer of the new round (Sec. 3.2, last step).  A workgroup moves one
// 16-token tile of one kv head of one sequence: the key rows go out unchanged to row t of head g,
// the value rows are turned through LDS into the [d][16] tile of the round layout, rows past the
// round's length as zeros.  Pure data movement in 16-byte pieces; T only fixes the element width.
template <typename T>
__global__ __launch_bounds__(kRepackThreads) void repack_round_kernel(const T* __restrict__ cur_k,
                                                                      const T* __restrict__ cur_v, int cur_cap,
                                                                      int Hkv, int d, int layer,
                                                                      const int64_t* __restrict__ wb_off,
                                                                      const int32_t* __restrict__ wb_len,
                                                                      T* __restrict__ pool) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int V = 16 / sizeof(T);  // elements per 16-byte piece; also the row padding in LDS
    T* tile = reinterpret_cast<T*>(smem);  // [16][d + V]
    const int b = blockIdx.z, g = blockIdx.y, t0 = blockIdx.x * 16;
    const int64_t off = wb_off[b];
    const int n = wb_len[b];
    if (off < 0 || t0 >= n) return;
    const int tiles = (n + 15) / 16;
    const size_t layer_tok = (size_t)off + (size_t)layer * ((size_t)n + (size_t)tiles * 16);
    T* kdst = pool + (layer_tok * Hkv + (size_t)g * n) * d;
    T* vdst = pool + (layer_tok + n) * Hkv * d + ((size_t)g * tiles + blockIdx.x) * d * 16;
    const int pieces = d / V, pitch = d + V;
    for (int i = threadIdx.x; i < 16 * pieces; i += kRepackThreads) {
        const int j = i / pieces, c = (i % pieces) * V, t = t0 + j;
        uint4 vv = make_uint4(0, 0, 0, 0);
        if (t < n) {
            const size_t src = (((size_t)b * cur_cap + t) * Hkv + g) * d + c;
            *reinterpret_cast<uint4*>(kdst + (size_t)t * d + c) = *reinterpret_cast<const uint4*>(cur_k + src);
            vv = *reinterpret_cast<const uint4*>(cur_v + src);
        }
        *reinterpret_cast<uint4*>(tile + j * pitch + c) = vv;
    }
    __syncthreads();
    constexpr int per_channel = 16 / V;  // 16-byte pieces of one channel's 16 tokens
    for (int i = threadIdx.x; i < d * per_channel; i += kRepackThreads) {
        const int c = i / per_channel, j0 = (i % per_channel) * V;
        Vec16<T> x;
#pragma unroll
        for (int e = 0; e < V; ++e) x.e[e] = tile[(j0 + e) * pitch + c];
        *reinterpret_cast<uint4*>(vdst + c * 16 + j0) = x.u;
    }
}
}  // namespace

extern "C" {

int ra_kv_store_create(ra_kv_store** out, const ra_store_cfg* cfg) {
    RA_REQUIRE(out != nullptr && cfg != nullptr, RA_ERR_INVALID_ARG, "kv_store_create: NULL argument");
    *out = nullptr;
    RA_REQUIRE(cfg->n_layers > 0 && cfg->B > 0 && cfg->R_max > 0 && cfg->Hkv > 0 && cfg->d > 0, RA_ERR_INVALID_ARG,
               "kv_store_create: non-positive dimension");
    RA_REQUIRE(cfg->R_max <= kMaxRounds, RA_ERR_UNSUPPORTED, "kv_store_create: R_max %d exceeds %d", cfg->R_max,
               kMaxRounds);
    RA_REQUIRE(cfg->dtype == RA_F32 || cfg->dtype == RA_BF16, RA_ERR_UNSUPPORTED, "kv_store_create: unknown dtype");
    RA_REQUIRE(cfg->device_pool_bytes > 0, RA_ERR_INVALID_ARG, "kv_store_create: device_pool_bytes is 0");
    int ndev = 0, prev = 0;
    RA_HIP_CHECK(hipGetDeviceCount(&ndev));
    RA_REQUIRE(cfg->device >= 0 && cfg->device < ndev, RA_ERR_INVALID_ARG, "kv_store_create: device out of range");
    RA_HIP_CHECK(hipGetDevice(&prev));
    RA_HIP_CHECK(hipSetDevice(cfg->device));

    ra_kv_store* s = new (std::nothrow) ra_kv_store();
    RA_REQUIRE(s != nullptr, RA_ERR_OOM, "kv_store_create: out of host memory");
    s->cfg = *cfg;
    s->token_bytes = (size_t)cfg->Hkv * cfg->d * (cfg->dtype == RA_BF16 ? 2 : 4);
    s->rounds.resize((size_t)cfg->B * cfg->R_max);
    const size_t n_off = (size_t)cfg->n_layers * 2 * cfg->B * cfg->R_max;
    const size_t n_len = (size_t)cfg->B * cfg->R_max;
    hipError_t e = hipMalloc((void**)&s->pool, cfg->device_pool_bytes);
    if (e == hipSuccess) e = hipMalloc((void**)&s->d_off, n_off * sizeof(int64_t));
    if (e == hipSuccess) e = hipMalloc((void**)&s->d_len, n_len * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void**)&s->d_n, (size_t)cfg->B * sizeof(int32_t));
    if (e == hipSuccess) e = hipHostMalloc((void**)&s->h_off, n_off * sizeof(int64_t), hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc((void**)&s->h_len, n_len * sizeof(int32_t), hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc((void**)&s->h_n, (size_t)cfg->B * sizeof(int32_t), hipHostMallocDefault);
    if (e == hipSuccess) e = hipMalloc((void**)&s->d_wb_off, (size_t)cfg->B * sizeof(int64_t));
    if (e == hipSuccess) e = hipMalloc((void**)&s->d_wb_len, (size_t)cfg->B * sizeof(int32_t));
    if (e == hipSuccess) e = hipHostMalloc((void**)&s->h_wb_off, (size_t)cfg->B * sizeof(int64_t), hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc((void**)&s->h_wb_len, (size_t)cfg->B * sizeof(int32_t), hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->wb_packed, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->wb_done, hipEventDisableTiming);
    if (e == hipSuccess) {
        s->ready.resize(cfg->n_layers, nullptr);
        for (int l = 0; l < cfg->n_layers && e == hipSuccess; ++l)
            e = hipEventCreateWithFlags(&s->ready[l], hipEventDisableTiming);
    }
    (void)hipSetDevice(prev);
    if (e != hipSuccess) {
        const bool oom = e == hipErrorOutOfMemory;
        (void)hipGetLastError();
        ra_kv_store_destroy(s);
        return fail(oom ? RA_ERR_OOM : RA_ERR_HIP, "kv_store_create: %s", hipGetErrorString(e));
    }
    *out = s;
    return RA_OK;
}

int ra_kv_store_destroy(ra_kv_store* s) {
    if (!s) return RA_OK;
    for (hipEvent_t ev : s->ready)
        if (ev) (void)hipEventDestroy(ev);
    if (s->pool) (void)hipFree(s->pool);
    if (s->d_off) (void)hipFree(s->d_off);
    if (s->d_len) (void)hipFree(s->d_len);
    if (s->d_n) (void)hipFree(s->d_n);
    if (s->h_off) (void)hipHostFree(s->h_off);
    if (s->h_len) (void)hipHostFree(s->h_len);
    if (s->h_n) (void)hipHostFree(s->h_n);
    if (s->wb_pending) (void)hipEventSynchronize(s->wb_done);  // host tensors may be freed right after this call
    if (s->d_wb_off) (void)hipFree(s->d_wb_off);
    if (s->d_wb_len) (void)hipFree(s->d_wb_len);
    if (s->h_wb_off) (void)hipHostFree(s->h_wb_off);
    if (s->h_wb_len) (void)hipHostFree(s->h_wb_len);
    if (s->wb_packed) (void)hipEventDestroy(s->wb_packed);
    if (s->wb_done) (void)hipEventDestroy(s->wb_done);
    delete s;
    return RA_OK;
}

size_t ra_kv_store_round_bytes(const ra_kv_store* s, int len) {
    if (!s || len < 0) return 0;
    return (size_t)s->cfg.n_layers * layer_tokens(len) * s->token_bytes;
}

int ra_kv_store_register_round(ra_kv_store* s, int seq, int round, const void* host_kv, int len) {
    RA_REQUIRE(s != nullptr, RA_ERR_INVALID_ARG, "kv_store_register_round: store is NULL");
    RA_REQUIRE(seq >= 0 && seq < s->cfg.B && round >= 0 && round < s->cfg.R_max, RA_ERR_INVALID_ARG,
               "kv_store_register_round: (seq %d, round %d) outside [0,%d) x [0,%d)", seq, round, s->cfg.B,
               s->cfg.R_max);
    RA_REQUIRE(len >= 0, RA_ERR_INVALID_ARG, "kv_store_register_round: negative length");
    RA_REQUIRE(len == 0 || host_kv != nullptr, RA_ERR_INVALID_ARG, "kv_store_register_round: host_kv is NULL");
    RA_REQUIRE(!s->staged, RA_ERR_STATE, "kv_store_register_round: rounds are staged; call ra_kv_store_release first");
    if (len > 0)
        RA_REQUIRE(is_pinned_host(host_kv), RA_ERR_INVALID_ARG,
                   "kv_store_register_round: host_kv is not pinned host memory (use hipHostMalloc / pin_memory)");
    ra_kv_store::Round& r = s->rounds[(size_t)seq * s->cfg.R_max + round];
    r.host = static_cast<const char*>(host_kv);
    r.len = len;
    r.turns = r.hits = 0;
    r.dropped = false;
    return RA_OK;
}

int ra_kv_store_stage(ra_kv_store* s, const int32_t* sel_idx_host, const int32_t* n_sel_host, int order,
                      void* side_stream) {
    RA_REQUIRE(s != nullptr && sel_idx_host != nullptr && n_sel_host != nullptr, RA_ERR_INVALID_ARG,
               "kv_store_stage: NULL argument");
    RA_REQUIRE(order == RA_STAGE_ROUND_MAJOR || order == RA_STAGE_LAYER_MAJOR || order == RA_STAGE_GROUPED,
               RA_ERR_INVALID_ARG, "kv_store_stage: unknown order %d", order);
    RA_REQUIRE(!s->staged, RA_ERR_STATE, "kv_store_stage: already staged; call ra_kv_store_release first");
    const int B = s->cfg.B, R = s->cfg.R_max, L = s->cfg.n_layers;
    // ---- validate the selection and place every selected round in the pool ----------------------
    struct Job { const char* src; size_t dst_tok; int len; };
    std::vector<Job> jobs;
    size_t tok = 0;  // pool cursor in units of token_bytes
    int64_t max_tokens = 0;
    for (int b = 0; b < B; ++b) {
        const int n = n_sel_host[b];
        RA_REQUIRE(n >= 0 && n <= R, RA_ERR_INVALID_ARG, "kv_store_stage: n_sel[%d] = %d outside [0, %d]", b, n, R);
        int64_t seq_tokens = 0;
        int prev = -1;
        for (int i = 0; i < n; ++i) {
            const int r = sel_idx_host[(size_t)b * R + i];
            RA_REQUIRE(r > prev && r < R, RA_ERR_INVALID_ARG,
                       "kv_store_stage: sel_idx[%d][%d] = %d is not an ascending round index below %d", b, i, r, R);
            prev = r;
            const ra_kv_store::Round& rd = s->rounds[(size_t)b * R + r];
            RA_REQUIRE(rd.len >= 0, RA_ERR_STATE, "kv_store_stage: round %d of sequence %d was never registered", r, b);
            jobs.push_back({rd.host, tok, rd.len});
            tok += (size_t)L * layer_tokens(rd.len);
            seq_tokens += rd.len;
        }
        if (seq_tokens > max_tokens) max_tokens = seq_tokens;
    }
    RA_REQUIRE(tok * s->token_bytes <= s->cfg.device_pool_bytes, RA_ERR_OOM,
               "kv_store_stage: selected rounds need %zu bytes, the device pool has %zu", tok * s->token_bytes,
               s->cfg.device_pool_bytes);
    // ---- index tables of the compact views (round i of the view = i-th selected round) ----------
    const size_t plane = (size_t)B * R;
    for (size_t i = 0; i < (size_t)L * 2 * plane; ++i) s->h_off[i] = 0;
    for (size_t i = 0; i < plane; ++i) s->h_len[i] = 0;
    size_t j = 0;
    for (int b = 0; b < B; ++b) {
        s->h_n[b] = n_sel_host[b];
        for (int i = 0; i < n_sel_host[b]; ++i, ++j) {
            const Job& jb = jobs[j];
            s->h_len[(size_t)b * R + i] = jb.len;
            for (int l = 0; l < L; ++l) {
                s->h_off[((size_t)l * 2 + 0) * plane + (size_t)b * R + i] = (int64_t)(jb.dst_tok + (size_t)l * layer_tokens(jb.len));
                s->h_off[((size_t)l * 2 + 1) * plane + (size_t)b * R + i] =
                    (int64_t)(jb.dst_tok + (size_t)l * layer_tokens(jb.len) + jb.len);
            }
        }
    }
    // ---- activity counters (Sec. 3.4): every kept round was a candidate, the selected ones were hit --
    for (int b = 0; b < B; ++b) {
        for (int r = 0; r < R; ++r) {
            ra_kv_store::Round& rd = s->rounds[(size_t)b * R + r];
            if (rd.len >= 0 && !rd.dropped) ++rd.turns;
        }
        for (int i = 0; i < n_sel_host[b]; ++i) {
            ra_kv_store::Round& rd = s->rounds[(size_t)b * R + sel_idx_host[(size_t)b * R + i]];
            if (!rd.dropped) ++rd.hits;
        }
    }
    // ---- enqueue the copies ------------------------------------------------------------------------
    hipStream_t st = reinterpret_cast<hipStream_t>(side_stream);
    // a round saved at the end of the last turn may be selected now, and its packed copy may still
    // sit where this selection is about to land: both wait for the write-back
    if (s->wb_pending) RA_HIP_CHECK(hipStreamWaitEvent(st, s->wb_done, 0));
    RA_HIP_CHECK(hipMemcpyAsync(s->d_off, s->h_off, (size_t)L * 2 * plane * sizeof(int64_t), hipMemcpyHostToDevice, st));
    RA_HIP_CHECK(hipMemcpyAsync(s->d_len, s->h_len, plane * sizeof(int32_t), hipMemcpyHostToDevice, st));
    RA_HIP_CHECK(hipMemcpyAsync(s->d_n, s->h_n, (size_t)B * sizeof(int32_t), hipMemcpyHostToDevice, st));
    s->staged_bytes = 0;
    s->n_copies = 0;
    if (order == RA_STAGE_ROUND_MAJOR) {
        for (const Job& jb : jobs) {
            if (jb.len == 0) continue;
            const size_t bytes = (size_t)L * layer_tokens(jb.len) * s->token_bytes;
            RA_HIP_CHECK(hipMemcpyAsync(s->pool + jb.dst_tok * s->token_bytes, jb.src, bytes, hipMemcpyHostToDevice, st));
            s->staged_bytes += bytes;
            ++s->n_copies;
        }
        for (int l = 0; l < L; ++l) RA_HIP_CHECK(hipEventRecord(s->ready[l], st));
    } else if (order == RA_STAGE_GROUPED) {
        // Groups of consecutive layers, one copy per (group, round): a round's layers are contiguous in its host
        // tensor, so a group is one slice.  A small first group lets the first post-watershed layer start early, a
        // last group of one layer leaves a single layer's attention to run after the last byte has arrived, and
        // up to three larger groups in between keep the number of copies (and their fixed cost on the link) down.
        for (int l0 = 0, gi = 0; l0 < L; ++gi) {
            const int l1 = l0 + grouped_stage_size(L, gi);
            for (const Job& jb : jobs) {
                if (jb.len == 0) continue;
                const size_t bytes = (size_t)(l1 - l0) * layer_tokens(jb.len) * s->token_bytes;
                const size_t o = (size_t)l0 * layer_tokens(jb.len) * s->token_bytes;
                RA_HIP_CHECK(hipMemcpyAsync(s->pool + jb.dst_tok * s->token_bytes + o, jb.src + o, bytes,
                                            hipMemcpyHostToDevice, st));
                s->staged_bytes += bytes;
                ++s->n_copies;
            }
            for (int l = l0; l < l1; ++l) RA_HIP_CHECK(hipEventRecord(s->ready[l], st));
            l0 = l1;
        }
    } else {
        for (int l = 0; l < L; ++l) {
            for (const Job& jb : jobs) {
                if (jb.len == 0) continue;
                const size_t bytes = layer_tokens(jb.len) * s->token_bytes;
                const size_t o = (size_t)l * layer_tokens(jb.len) * s->token_bytes;
                RA_HIP_CHECK(hipMemcpyAsync(s->pool + jb.dst_tok * s->token_bytes + o, jb.src + o, bytes,
                                            hipMemcpyHostToDevice, st));
                s->staged_bytes += bytes;
                ++s->n_copies;
            }
            RA_HIP_CHECK(hipEventRecord(s->ready[l], st));
        }
    }
    s->max_tokens = max_tokens;
    s->staged_tok = tok;
    s->staged = true;
    return RA_OK;
}

int ra_kv_store_wait_layer(ra_kv_store* s, int layer, void* compute_stream) {
    RA_REQUIRE(s != nullptr, RA_ERR_INVALID_ARG, "kv_store_wait_layer: store is NULL");
    RA_REQUIRE(layer >= 0 && layer < s->cfg.n_layers, RA_ERR_INVALID_ARG, "kv_store_wait_layer: layer out of range");
    RA_REQUIRE(s->staged, RA_ERR_STATE, "kv_store_wait_layer: nothing is staged");
    RA_HIP_CHECK(hipStreamWaitEvent(reinterpret_cast<hipStream_t>(compute_stream), s->ready[layer], 0));
    return RA_OK;
}

int ra_kv_store_layer_view(ra_kv_store* s, int layer, ra_kv_view* out) {
    RA_REQUIRE(s != nullptr && out != nullptr, RA_ERR_INVALID_ARG, "kv_store_layer_view: NULL argument");
    RA_REQUIRE(layer >= 0 && layer < s->cfg.n_layers, RA_ERR_INVALID_ARG, "kv_store_layer_view: layer out of range");
    RA_REQUIRE(s->staged, RA_ERR_STATE, "kv_store_layer_view: nothing is staged");
    const size_t plane = (size_t)s->cfg.B * s->cfg.R_max;
    out->k = s->pool;
    out->v = s->pool;
    out->seg_off = s->d_off + ((size_t)layer * 2 + 0) * plane;
    out->seg_off_v = s->d_off + ((size_t)layer * 2 + 1) * plane;
    out->seg_len = s->d_len;
    out->n_rounds = s->d_n;
    out->block_table = nullptr;
    out->block_size = 0;
    out->max_blocks = 0;
    out->B = s->cfg.B;
    out->R_max = s->cfg.R_max;
    out->Hkv = s->cfg.Hkv;
    out->d = s->cfg.d;
    out->dtype = s->cfg.dtype;
    out->reserved = 0;
    out->max_tokens = s->max_tokens;
    return RA_OK;
}

int ra_kv_store_stats(const ra_kv_store* s, uint64_t* staged_bytes, uint64_t* registered_bytes, uint64_t* n_copies) {
    RA_REQUIRE(s != nullptr, RA_ERR_INVALID_ARG, "kv_store_stats: store is NULL");
    if (staged_bytes) *staged_bytes = s->staged_bytes;
    if (n_copies) *n_copies = s->n_copies;
    if (registered_bytes) {
        uint64_t t = 0;
        for (const auto& r : s->rounds)
            if (r.len > 0) t += (uint64_t)s->cfg.n_layers * layer_tokens(r.len) * s->token_bytes;
        *registered_bytes = t;
    }
    return RA_OK;
}

int ra_kv_store_save_round(ra_kv_store* s, const int32_t* round_host, const int32_t* len_host,
                           const void* const* cur_k_layers, const void* const* cur_v_layers, int cur_cap,
                           void* const* host_kv, void* compute_stream, void* side_stream) {
    RA_REQUIRE(s != nullptr && round_host != nullptr && len_host != nullptr && cur_k_layers != nullptr &&
                   cur_v_layers != nullptr && host_kv != nullptr,
               RA_ERR_INVALID_ARG, "kv_store_save_round: NULL argument");
    RA_REQUIRE(cur_cap > 0, RA_ERR_INVALID_ARG, "kv_store_save_round: cur_cap must be positive");
    const int B = s->cfg.B, R = s->cfg.R_max, L = s->cfg.n_layers;
    const size_t elem = s->cfg.dtype == RA_BF16 ? 2 : 4;
    RA_REQUIRE(((size_t)s->cfg.d * elem) % 16 == 0, RA_ERR_UNSUPPORTED,
               "kv_store_save_round: a row of d = %d elements is not a whole number of 16-byte pieces", s->cfg.d);
    size_t tok = s->staged ? s->staged_tok : 0;
    int max_len = 0;
    std::vector<int64_t> off(B, -1);
    for (int b = 0; b < B; ++b) {
        const int r = round_host[b];
        if (r == -1) continue;
        const int n = len_host[b];
        RA_REQUIRE(r >= 0 && r < R, RA_ERR_INVALID_ARG, "kv_store_save_round: round[%d] = %d outside [0, %d)", b, r, R);
        RA_REQUIRE(n >= 0 && n <= cur_cap, RA_ERR_INVALID_ARG, "kv_store_save_round: len[%d] = %d outside [0, %d]", b,
                   n, cur_cap);
        if (n > 0)
            RA_REQUIRE(host_kv[b] != nullptr && is_pinned_host(host_kv[b]), RA_ERR_INVALID_ARG,
                       "kv_store_save_round: host_kv[%d] is not pinned host memory", b);
        off[b] = (int64_t)tok;
        tok += (size_t)L * layer_tokens(n);
        if (n > max_len) max_len = n;
    }
    RA_REQUIRE(tok * s->token_bytes <= s->cfg.device_pool_bytes, RA_ERR_OOM,
               "kv_store_save_round: staged rounds plus the new round need %zu bytes, the device pool has %zu",
               tok * s->token_bytes, s->cfg.device_pool_bytes);
    if (max_len > 0)
        for (int l = 0; l < L; ++l) {
            RA_REQUIRE(cur_k_layers[l] != nullptr && cur_v_layers[l] != nullptr, RA_ERR_INVALID_ARG,
                       "kv_store_save_round: layer %d has a NULL key or value pointer", l);
            RA_REQUIRE(((uintptr_t)cur_k_layers[l] | (uintptr_t)cur_v_layers[l]) % 16 == 0, RA_ERR_INVALID_ARG,
                       "kv_store_save_round: layer %d pointers are not 16-byte aligned", l);
        }
    // the placement table's pinned mirror and the pool area behind the staged rounds are reused from
    // call to call: the previous write-back must have left them
    if (s->wb_pending) {
        RA_HIP_CHECK(hipEventSynchronize(s->wb_done));
        s->wb_pending = false;
    }
    hipStream_t cs = reinterpret_cast<hipStream_t>(compute_stream);
    hipStream_t ss = reinterpret_cast<hipStream_t>(side_stream);
    s->saved_bytes = 0;
    if (max_len > 0) {
        for (int b = 0; b < B; ++b) {
            s->h_wb_off[b] = off[b];
            s->h_wb_len[b] = off[b] < 0 ? 0 : len_host[b];
        }
        RA_HIP_CHECK(hipMemcpyAsync(s->d_wb_off, s->h_wb_off, (size_t)B * sizeof(int64_t), hipMemcpyHostToDevice, cs));
        RA_HIP_CHECK(hipMemcpyAsync(s->d_wb_len, s->h_wb_len, (size_t)B * sizeof(int32_t), hipMemcpyHostToDevice, cs));
        const dim3 grid((max_len + 15) / 16, s->cfg.Hkv, B), block(kRepackThreads);
        for (int l = 0; l < L; ++l) {
            if (elem == 2) {
                const size_t smem = 16 * (size_t)(s->cfg.d + 8) * 2;
                hipLaunchKernelGGL(repack_round_kernel<uint16_t>, grid, block, smem, cs,
                                   static_cast<const uint16_t*>(cur_k_layers[l]),
                                   static_cast<const uint16_t*>(cur_v_layers[l]), cur_cap, s->cfg.Hkv, s->cfg.d, l,
                                   s->d_wb_off, s->d_wb_len, reinterpret_cast<uint16_t*>(s->pool));
            } else {
                const size_t smem = 16 * (size_t)(s->cfg.d + 4) * 4;
                hipLaunchKernelGGL(repack_round_kernel<uint32_t>, grid, block, smem, cs,
                                   static_cast<const uint32_t*>(cur_k_layers[l]),
                                   static_cast<const uint32_t*>(cur_v_layers[l]), cur_cap, s->cfg.Hkv, s->cfg.d, l,
                                   s->d_wb_off, s->d_wb_len, reinterpret_cast<uint32_t*>(s->pool));
            }
            RA_HIP_CHECK(hipGetLastError());
        }
        RA_HIP_CHECK(hipEventRecord(s->wb_packed, cs));
        RA_HIP_CHECK(hipStreamWaitEvent(ss, s->wb_packed, 0));
        for (int b = 0; b < B; ++b) {
            if (off[b] < 0 || len_host[b] == 0) continue;
            const size_t bytes = (size_t)L * layer_tokens(len_host[b]) * s->token_bytes;
            RA_HIP_CHECK(hipMemcpyAsync(host_kv[b], s->pool + (size_t)off[b] * s->token_bytes, bytes,
                                        hipMemcpyDeviceToHost, ss));
            s->saved_bytes += bytes;
        }
        RA_HIP_CHECK(hipEventRecord(s->wb_done, ss));
        s->wb_pending = true;
    }
    for (int b = 0; b < B; ++b) {
        if (off[b] < 0) continue;
        ra_kv_store::Round& r = s->rounds[(size_t)b * R + round_host[b]];
        r.host = len_host[b] > 0 ? static_cast<const char*>(host_kv[b]) : nullptr;
        r.len = len_host[b];
        r.turns = r.hits = 0;
        r.dropped = false;
    }
    return RA_OK;
}

int ra_kv_store_save_wait(ra_kv_store* s, uint64_t* saved_bytes) {
    RA_REQUIRE(s != nullptr, RA_ERR_INVALID_ARG, "kv_store_save_wait: store is NULL");
    if (s->wb_pending) {
        RA_HIP_CHECK(hipEventSynchronize(s->wb_done));
        s->wb_pending = false;
    }
    if (saved_bytes) *saved_bytes = s->saved_bytes;
    return RA_OK;
}

int ra_kv_store_round_activity(const ra_kv_store* s, int seq, int round, uint32_t* turns, uint32_t* hits) {
    RA_REQUIRE(s != nullptr, RA_ERR_INVALID_ARG, "kv_store_round_activity: store is NULL");
    RA_REQUIRE(seq >= 0 && seq < s->cfg.B && round >= 0 && round < s->cfg.R_max, RA_ERR_INVALID_ARG,
               "kv_store_round_activity: (seq %d, round %d) outside [0,%d) x [0,%d)", seq, round, s->cfg.B,
               s->cfg.R_max);
    const ra_kv_store::Round& r = s->rounds[(size_t)seq * s->cfg.R_max + round];
    RA_REQUIRE(r.len >= 0, RA_ERR_STATE, "kv_store_round_activity: round %d of sequence %d was never registered", round,
               seq);
    if (turns) *turns = r.turns;
    if (hits) *hits = r.hits;
    return RA_OK;
}

// A dropped round keeps its index as an empty round: selecting it stages nothing.
static void drop_one(ra_kv_store::Round& r) {
    r.host = nullptr;
    r.len = 0;
    r.dropped = true;
}

int ra_kv_store_drop_round(ra_kv_store* s, int seq, int round) {
    RA_REQUIRE(s != nullptr, RA_ERR_INVALID_ARG, "kv_store_drop_round: store is NULL");
    RA_REQUIRE(seq >= 0 && seq < s->cfg.B && round >= 0 && round < s->cfg.R_max, RA_ERR_INVALID_ARG,
               "kv_store_drop_round: (seq %d, round %d) outside [0,%d) x [0,%d)", seq, round, s->cfg.B, s->cfg.R_max);
    RA_REQUIRE(!s->staged, RA_ERR_STATE, "kv_store_drop_round: rounds are staged; call ra_kv_store_release first");
    ra_kv_store::Round& r = s->rounds[(size_t)seq * s->cfg.R_max + round];
    RA_REQUIRE(r.len >= 0, RA_ERR_STATE, "kv_store_drop_round: round %d of sequence %d was never registered", round, seq);
    if (s->wb_pending) {  // the caller frees the host tensor next: no copy may still be writing it
        RA_HIP_CHECK(hipEventSynchronize(s->wb_done));
        s->wb_pending = false;
    }
    drop_one(r);
    return RA_OK;
}

int ra_kv_store_drop_inactive(ra_kv_store* s, uint32_t min_turns, int32_t* dropped_idx, int32_t* n_dropped) {
    RA_REQUIRE(s != nullptr && dropped_idx != nullptr && n_dropped != nullptr, RA_ERR_INVALID_ARG,
               "kv_store_drop_inactive: NULL argument");
    RA_REQUIRE(!s->staged, RA_ERR_STATE, "kv_store_drop_inactive: rounds are staged; call ra_kv_store_release first");
    if (s->wb_pending) {
        RA_HIP_CHECK(hipEventSynchronize(s->wb_done));
        s->wb_pending = false;
    }
    const int B = s->cfg.B, R = s->cfg.R_max;
    for (int b = 0; b < B; ++b) {
        int n = 0;
        for (int r = 0; r < R; ++r) {
            dropped_idx[(size_t)b * R + r] = -1;
            ra_kv_store::Round& rd = s->rounds[(size_t)b * R + r];
            if (rd.len < 0 || rd.dropped || rd.hits != 0 || rd.turns < min_turns) continue;
            drop_one(rd);
            dropped_idx[(size_t)b * R + n++] = r;
        }
        n_dropped[b] = n;
    }
    return RA_OK;
}

int ra_kv_store_release(ra_kv_store* s) {
    RA_REQUIRE(s != nullptr, RA_ERR_INVALID_ARG, "kv_store_release: store is NULL");
    if (s->staged) {
        // the pinned mirrors of the index tables are rewritten by the next stage call: make sure the
        // copies that read them have finished
        RA_HIP_CHECK(hipEventSynchronize(s->ready[s->cfg.n_layers - 1]));
        s->staged = false;
        s->staged_tok = 0;
    }
    return RA_OK;
}

}  // extern "C"
