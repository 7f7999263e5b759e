// Round scores at the watershed layer (paper Sec. 3.1, Eq. 1 and the normalisation after it).
//
// Two kernels.  (1) A streaming pass over the watershed layer's keys, bandwidth bound like decode
// attention but without values: workgroup (r, g, b*q_len+i) reduces the logits of query token i
// against the tokens of round r (or of the visible part of the current round) to one log-sum-exp
// per query head.  (2) A small finishing kernel turns the log-sum-exps into Eq. 1: per query token
// the softmax normaliser over all rounds and the current round, the probability mass of every
// history round summed over query tokens, normalisation over history rounds, mean over heads.
#include "stream_kv.hpp"

namespace ra {

struct ScoreArgs {
    DevView view;
    const void* q;      // [B][q_len][Hq][D]
    const void* cur_k;  // [B][cur_len][Hkv][D] or null
    int cur_len, q_len, Hq;
    float c;            // scale * log2(e)
    float* lse;         // [B][Hq][q_len][R_max + 1] natural-log sum-exp of the scaled logits; last = current round
};

template <typename T, int D, int G, bool PAGED>
__global__ __launch_bounds__(256) void scores_stream_kernel(ScoreArgs a) {
    constexpr int EPL = D / 16;
    using Ops = RowOps<T, EPL>;
    constexpr int WORDS = Ops::WORDS;
    constexpr int EB = Ops::ELEM_BYTES;
    __shared__ float sm[4][G], sl[4][G];

    const DevView& vw = a.view;
    const int r = blockIdx.x, g = blockIdx.y;
    const int b = blockIdx.z / a.q_len, i = blockIdx.z - b * a.q_len;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, grp = lane >> 4, sub = lane & 15;
    const int Hkv = vw.Hkv;
    const bool is_cur = r >= vw.R_max;

    int len = 0;
    long long off = 0;
    if (is_cur) {
        len = min(max(a.cur_len - a.q_len + i + 1, 0), a.cur_len);  // causal: tokens 0 .. cur_len - q_len + i
    } else {
        const int n_rounds = min(max(vw.n_rounds[b], 0), vw.R_max);
        if (r < n_rounds) {
            len = max(vw.seg_len[(size_t)b * vw.R_max + r], 0);
            off = vw.seg_off[(size_t)b * vw.R_max + r];
        }
    }
    const int units = (len + kUnitTokens - 1) / kUnitTokens;

    uint32_t qw[G][WORDS];
    {
        const char* qp = reinterpret_cast<const char*>(a.q) +
                         ((((size_t)b * a.q_len + i) * a.Hq) + (size_t)g * G) * D * EB;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            Frag<WORDS> f = load_frag<WORDS>(qp + ((size_t)h * D + sub * EPL) * EB);
#pragma unroll
            for (int e = 0; e < WORDS; ++e) qw[h][e] = f.w[e];
        }
    }
    float m[G], l[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = kNegBig;
        l[h] = 0.f;
    }

    const char* kbase = reinterpret_cast<const char*>(vw.k);
    auto issue = [&](int u, Frag<WORDS>* kf, int& ntok) {
        const int tok0 = u * kUnitTokens;
        ntok = min(kUnitTokens, len - tok0);
        const char* kp;
        size_t stride;
        if (is_cur) {
            kp = reinterpret_cast<const char*>(a.cur_k) + ((((size_t)b * a.cur_len + tok0) * Hkv + g) * D) * EB;
            stride = (size_t)Hkv * D * EB;
        } else if (PAGED) {
            long long si = off + u;
            si = si < 0 ? 0 : (si >= vw.max_blocks ? vw.max_blocks - 1 : si);
            int blk = vw.block_table[(size_t)b * vw.max_blocks + si];
            if (blk < 0) { blk = 0; ntok = 0; }
            kp = kbase + ((((size_t)blk * Hkv + g) * kUnitTokens) * D) * EB;
            stride = (size_t)D * EB;
        } else {
            kp = kbase + (((size_t)off * Hkv + (size_t)g * len + tok0) * D) * EB;
            stride = (size_t)D * EB;
        }
        const int last = max(ntok - 1, 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = min(j * 4 + grp, last);
            kf[j] = load_frag<WORDS>(kp + (size_t)t * stride + (size_t)sub * EPL * EB);
        }
    };
    auto consume = [&](const Frag<WORDS>* kf, int ntok) {
        float sc[4][G];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool valid = (j * 4 + grp) < ntok;
#pragma unroll
            for (int h = 0; h < G; ++h) {
                float d = row16_sum(Ops::dot(kf[j].w, qw[h]));
                sc[j][h] = valid ? d : -__builtin_inff();
            }
        }
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float mx = fmaxf(fmaxf(sc[0][h], sc[1][h]), fmaxf(sc[2][h], sc[3][h]));
            const float m_new = fmaxf(m[h], mx);
            const float mc = m_new * a.c;
            float ps = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) ps += fast_exp2(__builtin_fmaf(sc[j][h], a.c, -mc));
            l[h] = __builtin_fmaf(l[h], fast_exp2(__builtin_fmaf(m[h], a.c, -mc)), ps);
            m[h] = m_new;
        }
    };

    {
        int u = wave;
        Frag<WORDS> kf[4];
        int ntok = 0;
        bool have = u < units;
        if (have) issue(u, kf, ntok);
        while (have) {
            const int un = u + 4;
            const bool have_n = un < units;
            Frag<WORDS> kn[4];
            int ntok_n = 0;
            if (have_n) issue(un, kn, ntok_n);
            consume(kf, ntok);
#pragma unroll
            for (int j = 0; j < 4; ++j) kf[j] = kn[j];
            ntok = ntok_n;
            u = un;
            have = have_n;
        }
    }

#pragma unroll
    for (int h = 0; h < G; ++h) {
        float M = fmaxf(m[h], xrow_get(m[h], 16));
        M = fmaxf(M, xrow_get(M, 32));
        float lv = l[h] * fast_exp2((m[h] - M) * a.c);
        lv += xrow_get(lv, 16);
        lv += xrow_get(lv, 32);
        if (lane == 0) {
            sm[wave][h] = M;
            sl[wave][h] = lv;
        }
    }
    __syncthreads();
    if (tid < G) {
        const int h = tid;
        const float M = fmaxf(fmaxf(sm[0][h], sm[1][h]), fmaxf(sm[2][h], sm[3][h]));
        float den = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) den = __builtin_fmaf(sl[w][h], fast_exp2((sm[w][h] - M) * a.c), den);
        const size_t idx = ((((size_t)b * a.Hq + (size_t)g * G + h) * a.q_len) + i) * (vw.R_max + 1) + r;
        // natural log of sum_j exp(scale * logit_j) = ln2 * (M * c + log2(den))
        a.lse[idx] = den > 0.f ? kLn2 * __builtin_fmaf(M, a.c, fast_log2(den)) : -__builtin_inff();
    }
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// grid (B), block 256.  Wave w finishes heads w, w + 4, ...; lane j owns rounds j, j + 64, ...
// P is written to p_out [B][Hq][R_max]; afterwards the whole workgroup averages over heads.
constexpr int kRoundsPerLane = kMaxRounds / 64;
__global__ __launch_bounds__(256) void scores_finish_kernel(const float* lse, const int32_t* n_rounds_arr, int R_max,
                                                           int Hq, int q_len, bool has_cur, float* p_out,
                                                           float* s_out) {
    const int b = blockIdx.x;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int R = min(max(n_rounds_arr[b], 0), R_max);
    const int W = R_max + 1;
    for (int h = wave; h < Hq; h += 4) {
        float qatt[kRoundsPerLane];
#pragma unroll
        for (int k = 0; k < kRoundsPerLane; ++k) qatt[k] = 0.f;
        for (int i = 0; i < q_len; ++i) {
            const float* row = lse + (((size_t)b * Hq + h) * q_len + i) * W;
            float lv[kRoundsPerLane];
            float mx = -__builtin_inff();
#pragma unroll
            for (int k = 0; k < kRoundsPerLane; ++k) {
                const int r = lane + 64 * k;
                lv[k] = r < R ? row[r] : -__builtin_inff();
                mx = fmaxf(mx, lv[k]);
            }
            const float lc = has_cur ? row[R_max] : -__builtin_inff();
            mx = fmaxf(wave_max(mx), lc);
            if (mx == -__builtin_inff()) continue;  // this query token sees no key at all
            float e[kRoundsPerLane], sum = 0.f;
#pragma unroll
            for (int k = 0; k < kRoundsPerLane; ++k) {
                e[k] = __expf(lv[k] - mx);
                sum += e[k];
            }
            const float z = wave_sum(sum) + __expf(lc - mx);
            const float inv = 1.f / z;
#pragma unroll
            for (int k = 0; k < kRoundsPerLane; ++k) qatt[k] = __builtin_fmaf(e[k], inv, qatt[k]);
        }
        float tot = 0.f;
#pragma unroll
        for (int k = 0; k < kRoundsPerLane; ++k) tot += qatt[k];
        tot = wave_sum(tot);
        const float inv = tot > 0.f ? 1.f / tot : 0.f;
#pragma unroll
        for (int k = 0; k < kRoundsPerLane; ++k) {
            const int r = lane + 64 * k;
            if (r < R_max) p_out[((size_t)b * Hq + h) * R_max + r] = r < R ? qatt[k] * inv : 0.f;
        }
    }
    __threadfence_block();
    __syncthreads();
    const float inv_h = 1.f / (float)Hq;
    for (int r = tid; r < R_max; r += 256) {
        float s = 0.f;
        for (int h = 0; h < Hq; ++h) s += p_out[((size_t)b * Hq + h) * R_max + r];
        s_out[(size_t)b * R_max + r] = s * inv_h;
    }
}

template <typename T, int D, int G>
static void launch_scores(bool paged, dim3 grid, hipStream_t st, const ScoreArgs& a) {
    if (paged)
        hipLaunchKernelGGL((scores_stream_kernel<T, D, G, true>), grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((scores_stream_kernel<T, D, G, false>), grid, dim3(256), 0, st, a);
}

template <typename T, int D>
static int dispatch_scores(int G, bool paged, dim3 grid, hipStream_t st, const ScoreArgs& a) {
    switch (G) {
        case 1: launch_scores<T, D, 1>(paged, grid, st, a); return RA_OK;
        case 2: launch_scores<T, D, 2>(paged, grid, st, a); return RA_OK;
        case 4: launch_scores<T, D, 4>(paged, grid, st, a); return RA_OK;
        case 8: launch_scores<T, D, 8>(paged, grid, st, a); return RA_OK;
        default: return fail(RA_ERR_UNSUPPORTED, "round_scores: Hq / Hkv = %d not in {1, 2, 4, 8}", G);
    }
}

}  // namespace ra

using namespace ra;

extern "C" int ra_round_scores(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq,
                               const ra_kv_view* watershed, const void* cur_k, int cur_len, float scale,
                               float* scores_head, float* scores) {
    RA_REQUIRE(ctx != nullptr, RA_ERR_INVALID_ARG, "round_scores: ctx is NULL");
    RA_REQUIRE(q != nullptr && scores != nullptr, RA_ERR_INVALID_ARG, "round_scores: q or scores is NULL");
    if (int rc = check_view(watershed, false, "round_scores")) return rc;
    RA_REQUIRE(q_len > 0, RA_ERR_INVALID_ARG, "round_scores: q_len must be positive");
    RA_REQUIRE(Hq > 0 && Hq % watershed->Hkv == 0, RA_ERR_INVALID_ARG,
               "round_scores: Hq %d is not a multiple of Hkv %d", Hq, watershed->Hkv);
    RA_REQUIRE(cur_len >= 0 && (cur_k != nullptr) == (cur_len > 0), RA_ERR_INVALID_ARG,
               "round_scores: cur_k and cur_len > 0 must be given together");
    RA_REQUIRE(cur_k == nullptr || cur_len >= q_len, RA_ERR_INVALID_ARG,
               "round_scores: the q_len query tokens are the tail of the current round, so cur_len >= q_len");
    RA_REQUIRE(scale > 0.f && scale == scale, RA_ERR_INVALID_ARG, "round_scores: scale must be positive");
    RA_REQUIRE(watershed->R_max > 0, RA_ERR_INVALID_ARG, "round_scores: R_max is 0, there is nothing to score");
    const int G = Hq / watershed->Hkv, D = watershed->d, B = watershed->B, R_max = watershed->R_max;
    RA_REQUIRE(D == 64 || D == 128, RA_ERR_UNSUPPORTED, "round_scores: head_dim %d not in {64, 128}", D);
    RA_REQUIRE((int64_t)B * q_len <= 65535, RA_ERR_UNSUPPORTED, "round_scores: B * q_len exceeds 65535");

    // With a single query token the current round's share of the softmax cancels in the
    // normalisation over history rounds, so its keys need not be read at all.
    const bool use_cur = cur_k != nullptr && q_len > 1;
    const size_t rows = (size_t)B * Hq * q_len;
    const size_t lse_bytes = align_up(rows * (R_max + 1) * sizeof(float), 256);
    const size_t p_bytes = scores_head ? 0 : align_up((size_t)B * Hq * R_max * sizeof(float), 256);
    RA_REQUIRE(ctx->ws.base != nullptr && ctx->ws.bytes >= lse_bytes + p_bytes, RA_ERR_WORKSPACE,
               "round_scores: workspace has %zu bytes, this call needs %zu", ctx->ws.bytes, lse_bytes + p_bytes);

    ScoreArgs a;
    a.view = to_dev(watershed);
    a.q = q;
    a.cur_k = use_cur ? cur_k : nullptr;
    a.cur_len = use_cur ? cur_len : 0;
    a.q_len = q_len;
    a.Hq = Hq;
    a.c = scale * kLog2e;
    a.lse = reinterpret_cast<float*>(ctx->ws.base);
    float* p_out = scores_head ? scores_head : reinterpret_cast<float*>(ctx->ws.base + lse_bytes);

    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const dim3 grid(R_max + (use_cur ? 1 : 0), watershed->Hkv, B * q_len);
    const bool paged = watershed->block_size != 0;
    int rc;
    if (watershed->dtype == RA_BF16)
        rc = D == 128 ? dispatch_scores<BF16, 128>(G, paged, grid, st, a) : dispatch_scores<BF16, 64>(G, paged, grid, st, a);
    else
        rc = D == 128 ? dispatch_scores<F32, 128>(G, paged, grid, st, a) : dispatch_scores<F32, 64>(G, paged, grid, st, a);
    if (rc) return rc;
    hipLaunchKernelGGL(scores_finish_kernel, dim3(B), dim3(256), 0, st, a.lse, watershed->n_rounds, R_max, Hq, q_len,
                       use_cur, p_out, scores);
    RA_HIP_CHECK(hipGetLastError());
    return RA_OK;
}
