// Round scores at the watershed layer (paper Sec. 3.1, Eq. 1 and the normalisation after it): the generic
// streaming kernel, the finishing kernels and the entry point.
//
// (1) A streaming pass over the watershed layer's keys, HBM-bandwidth bound like decode attention but
//     without values, leaves one log-sum-exp per (query row, 256-token chunk of a round).  For bf16 / d = 128
//     it runs on the matrix cores (scores_mfma.hip, scores_prefill_mfma.hip); the kernel below serves fp32 and
//     d = 64: workgroup (c, g, b*q_len+i) owns chunk c of sequence b for KV head g and query token i, each of
//     its four waves issues the loads of its four 16-token units up front (16 KB in flight per workgroup), then
//     reduces the logits of the chunk to one log-sum-exp per query head.  Equal-sized work items keep long
//     rounds from becoming the tail of the launch.
// (2) Finishing kernels turn the per-chunk log-sum-exps into Eq. 1: per round the log-sum-exp over its chunks,
//     per query token the softmax normaliser over all rounds and the visible part of the current round, the
//     probability mass of every history round summed over the query tokens, normalisation over history
//     rounds, mean over query heads.  One kernel does all of it for a single query token; for several query
//     tokens the work of a head is split over several workgroups and a second small kernel normalises.
#include "scores_common.hpp"
#include "select_common.hpp"
#include "stream_kv.hpp"

namespace ra {

template <typename T, int D, int G, bool PAGED>
__global__ __launch_bounds__(256) void scores_stream_kernel(ScoreArgs a) {
    constexpr int EPL = D / 16;
    using Ops = RowOps<T, EPL>;
    constexpr int WORDS = Ops::WORDS;
    constexpr int EB = Ops::ELEM_BYTES;
    __shared__ float sm[4][G], sl[4][G];
    extern __shared__ __align__(16) char smem[];

    const DevView& vw = a.view;
    const int c = blockIdx.x, g = blockIdx.y;
    const int b = blockIdx.z / a.q_len, i = blockIdx.z - b * a.q_len;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, grp = lane >> 4, sub = lane & 15;
    const int Hkv = vw.Hkv;

    // ---- which round does chunk c belong to? -------------------------------------------------------
    const int n_hist = min(max(vw.n_rounds[b], 0), vw.R_max);
    const int cur_vis = a.cur_k ? cur_visible(a.cur_len, a.q_len, i) : 0;
    // the current round is chunked by its full length (the same for every query token); what a query
    // token may see of it is applied as a mask
    const int n_slots = n_hist + (a.cur_k && a.cur_len > 0 ? 1 : 0);
    const int cap = vw.R_max + 1;
    long long* t_off = reinterpret_cast<long long*>(smem);
    int* t_len = reinterpret_cast<int*>(t_off + cap);
    int* t_cum = t_len + cap;
    for (int s = tid; s < n_slots; s += 256) {
        int len = a.cur_len;
        long long off = 0;
        if (s < n_hist) {
            len = max(vw.seg_len[(size_t)b * vw.R_max + s], 0);
            off = vw.seg_off[(size_t)b * vw.R_max + s];
        }
        t_len[s] = len;
        t_off[s] = off;
        t_cum[s] = chunks_of(len);
    }
    exclusive_scan_units(t_cum, n_slots);
    const int total = n_slots > 0 ? t_cum[n_slots] : 0;
    if (c >= total) return;
    const int slot = find_slot(t_cum, n_slots, c);
    const int len = t_len[slot];
    const long long off = t_off[slot];
    const bool is_cur = slot >= n_hist;
    const int vis = is_cur ? cur_vis : len;  // tokens of this segment the query token may see
    const int chunk_tok0 = (c - t_cum[slot]) * kChunkTokens;

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

    // ---- issue every load of this wave's four units, then do the arithmetic ---------------------------
    const char* kbase = reinterpret_cast<const char*>(vw.k);
    Frag<WORDS> kf[4][4];
    int ntok[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int tok0 = chunk_tok0 + (j * 4 + wave) * kUnitTokens;  // the four waves read adjacent units
        ntok[j] = min(kUnitTokens, vis - tok0);
        if (ntok[j] > 0) {
            const char* kp;
            size_t stride;
            if (is_cur) {
                kp = reinterpret_cast<const char*>(a.cur_k) + ((((size_t)b * a.cur_len + tok0) * Hkv + g) * D) * EB;
                stride = (size_t)Hkv * D * EB;
            } else if (PAGED) {
                long long si = off + tok0 / kUnitTokens;
                si = si < 0 ? 0 : (si >= vw.max_blocks ? vw.max_blocks - 1 : si);
                int blk = vw.block_table[(size_t)b * vw.max_blocks + si];
                if (blk < 0) { blk = 0; ntok[j] = 0; }
                kp = kbase + ((((size_t)blk * Hkv + g) * kUnitTokens) * D) * EB;
                stride = (size_t)D * EB;
            } else {
                kp = kbase + (((size_t)off * Hkv + (size_t)g * len + tok0) * D) * EB;
                stride = (size_t)D * EB;
            }
            const int last = max(ntok[j] - 1, 0);
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                const int t = min(t4 * 4 + grp, last);  // rows past the round's end re-read its last row
                kf[j][t4] = load_frag<WORDS>(kp + (size_t)t * stride + (size_t)sub * EPL * EB);
            }
        }
    }

    float m[G], l[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = kNegBig;
        l[h] = 0.f;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (ntok[j] > 0) {
            float sc[4][G];
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                const bool valid = (t4 * 4 + grp) < ntok[j];
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    float d = row16_sum(Ops::dot(kf[j][t4].w, qw[h]));
                    sc[t4][h] = valid ? d : -__builtin_inff();
                }
            }
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const float mx = fmaxf(fmaxf(sc[0][h], sc[1][h]), fmaxf(sc[2][h], sc[3][h]));
                const float m_new = fmaxf(m[h], mx);
                const float mc = m_new * a.c;
                float ps = 0.f;
#pragma unroll
                for (int t4 = 0; t4 < 4; ++t4) ps += fast_exp2(__builtin_fmaf(sc[t4][h], a.c, -mc));
                // (m - m_new) * c, not fma(m, c, -mc): a lane row that has seen no token yet keeps m = m_new = the
                // finite stand-in, and the fused form would leave the rounding residue of its huge product in the exponent
                l[h] = __builtin_fmaf(l[h], fast_exp2((m[h] - m_new) * a.c), ps);
                m[h] = m_new;
            }
        }
    }

    // ---- merge the four 16-lane rows of the wave, then the four waves ------------------------------------
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float M = xrow_max4(m[h]);
        float lv = l[h] * fast_exp2((m[h] - M) * a.c);
        lv = xrow_sum4(lv);
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
        const size_t idx = ((((size_t)b * a.Hq + (size_t)g * G + h) * a.q_len) + i) * a.n_chunks_max + c;
        // natural log of sum_j exp(scale * logit_j) = ln2 * (M * c + log2(den))
        a.part[idx] = den > 0.f ? kLn2 * __builtin_fmaf(M, a.c, fast_log2(den)) : -__builtin_inff();
    }
}

// Reductions over the 64 lanes of a wavefront, every lane ends with the result: DPP inside the 16-lane rows,
// then lane-permute swaps across the rows; no LDS traffic.
__device__ __forceinline__ float wave_max(float v) {
    v = vmax(v, dpp_mov<0xB1>(v));   // quad_perm [1,0,3,2]
    v = vmax(v, dpp_mov<0x4E>(v));   // quad_perm [2,3,0,1]
    v = vmax(v, dpp_mov<0x141>(v));  // row_half_mirror
    v = vmax(v, dpp_mov<0x140>(v));  // row_mirror
    return xrow_max4(v);
}
__device__ __forceinline__ float wave_sum(float v) { return xrow_sum4(row16_sum(v)); }
// log-sum-exp of x[lo .. hi)
__device__ __forceinline__ float lse_range(const float* x, int lo, int hi) {
    float mx = -__builtin_inff();
    for (int k = lo; k < hi; ++k) mx = fmaxf(mx, x[k]);
    if (hi - lo <= 1 || mx == -__builtin_inff()) return mx;
    float s = 0.f;
    for (int k = lo; k < hi; ++k) s += __expf(x[k] - mx);
    return mx + __logf(s);
}

// grid (B), block 512.  Wave w finishes heads w, w + 8, ...; lane j owns rounds j, j + 64, ...
// (KPL rounds per lane).  P goes to p_out [B][Hq][R_max] if wanted; the head mean is accumulated per
// wave in registers and reduced over the eight waves through LDS in a fixed order.
constexpr int kFinishWaves = 8;
constexpr int kRowBufMax = 2048;  // chunk values a wave can stage in LDS (8 waves x 8 KB)

template <int KPL, int W>
__global__ __launch_bounds__(W * 64) void scores_finish_kernel(FinishArgs a, bool stage_rows) {
    extern __shared__ __align__(16) char smem[];
    int* cum = reinterpret_cast<int*>(smem);                       // [R_max + 2] chunk prefix of the history rounds
    float* hs = reinterpret_cast<float*>(smem) + (a.R_max + 2);    // [W][R_max] per-wave head sums
    float* rowbuf = hs + W * a.R_max;                   // [W][n_chunks_max] if staged
    const int b = blockIdx.x;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    // The first row this wave needs is fetched (whole, whatever the number of chunks turns out to be) while the
    // round lengths are on their way: one memory round trip less on the path of this latency-bound kernel.
    const bool prefetched = stage_rows && wave < a.Hq;
    if (prefetched) {
        const float* row = a.part + ((size_t)b * a.Hq + wave) * a.q_len * a.n_chunks_max;
        float* mybuf = rowbuf + (size_t)wave * a.n_chunks_max;
        for (int c = lane; c < a.n_chunks_max; c += 64) mybuf[c] = row[c];
    }
    const int R = min(max(a.n_rounds[b], 0), a.R_max);
    for (int r = tid; r < a.R_max; r += W * 64) {
        const int len = a.seg_len[(size_t)b * a.R_max + r];  // (loaded whether or not r < R: no wait for R)
        if (r < R) cum[r] = chunks_of(max(len, 0), a.chunk_tokens);
    }
    exclusive_scan_units(cum, R);
    const int hist_chunks = R > 0 ? cum[R] : 0;
    const bool overflow = hist_chunks + (a.has_cur ? chunks_of(a.cur_len, a.chunk_tokens) : 0) > a.n_chunks_max;

    float hsum[KPL];
#pragma unroll
    for (int k = 0; k < KPL; ++k) hsum[k] = 0.f;
    for (int h = wave; h < a.Hq; h += W) {
        float qatt[KPL];
#pragma unroll
        for (int k = 0; k < KPL; ++k) qatt[k] = 0.f;
        for (int i = 0; i < a.q_len && !overflow; ++i) {
            const float* row = a.part + (((size_t)b * a.Hq + h) * a.q_len + i) * a.n_chunks_max;
            if (stage_rows) {  // one coalesced pass over the row instead of dependent loads per round
                float* mybuf = rowbuf + (size_t)(tid >> 6) * a.n_chunks_max;
                __builtin_amdgcn_wave_barrier();
                if (!(prefetched && h == wave && i == 0))
                    for (int c = lane; c < hist_chunks + (a.has_cur ? chunks_of(a.cur_len, a.chunk_tokens) : 0); c += 64)
                        mybuf[c] = row[c];
                __builtin_amdgcn_wave_barrier();  // same wave: LDS operations complete in program order
                row = mybuf;
            }
            float lv[KPL];
            float mx = -__builtin_inff();
#pragma unroll
            for (int k = 0; k < KPL; ++k) {
                const int r = lane + 64 * k;
                lv[k] = r < R ? lse_range(row, cum[r], cum[r + 1]) : -__builtin_inff();
                mx = fmaxf(mx, lv[k]);
            }
            float lc = -__builtin_inff();
            if (a.has_cur) lc = lse_range(row, hist_chunks, hist_chunks + chunks_of(a.cur_len, a.chunk_tokens));
            mx = fmaxf(wave_max(mx), lc);
            if (mx == -__builtin_inff()) continue;  // this query token sees no key at all
            float e[KPL], sum = 0.f;
#pragma unroll
            for (int k = 0; k < KPL; ++k) {
                e[k] = __expf(lv[k] - mx);
                sum += e[k];
            }
            const float z = wave_sum(sum) + __expf(lc - mx);
            const float inv = 1.f / z;
#pragma unroll
            for (int k = 0; k < KPL; ++k) qatt[k] = __builtin_fmaf(e[k], inv, qatt[k]);
        }
        if (a.acc && !overflow) {
#pragma unroll
            for (int k = 0; k < KPL; ++k) {
                const int r = lane + 64 * k;
                if (r < R) {
                    float* slot = a.acc + ((size_t)b * a.Hq + h) * a.R_max + r;
                    qatt[k] += *slot;
                    *slot = qatt[k];
                }
            }
        }
        float tot = 0.f;
#pragma unroll
        for (int k = 0; k < KPL; ++k) tot += qatt[k];
        tot = wave_sum(tot);
        const float inv = tot > 0.f ? 1.f / tot : 0.f;
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const int r = lane + 64 * k;
            // a max_tokens that understates the cache would leave chunks unscored: make that loud
            const float val = overflow ? __builtin_nanf("") : (r < R ? qatt[k] * inv : 0.f);
            hsum[k] += val;
            if (a.p_out && r < a.R_max) a.p_out[((size_t)b * a.Hq + h) * a.R_max + r] = val;
        }
    }
#pragma unroll
    for (int k = 0; k < KPL; ++k) {
        const int r = lane + 64 * k;
        if (r < a.R_max) hs[wave * a.R_max + r] = hsum[k];
    }
    __syncthreads();
    const float inv_h = 1.f / (float)a.Hq;
    float* svec = reinterpret_cast<float*>(cum);  // the sequence's scores, for the selection (cum is no longer read)
    for (int r = tid; r < a.R_max; r += W * 64) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < W; ++w) s += hs[w * a.R_max + r];
        const float val = s * inv_h;
        a.s_out[(size_t)b * a.R_max + r] = val;
        if (a.with_select) svec[r] = val;
    }
    if (a.with_select) {  // Sec. 3.3 on the scores just written, same bits
        __shared__ SelectShared<W> sh;
        __syncthreads();
        select_rounds_block<W>(svec, R, a.R_max, a.sel, a.sel_idx + (size_t)b * a.R_max, a.n_sel + b, sh);
    }
}

// Finishing kernel for several query tokens: grid (B, Hq, Z), block 512.  Z workgroups per (sequence, head);
// the eight waves of workgroup z take the query tokens i = 8*z + wave, + 8*Z, ...  A wave first copies token
// i's row of chunk log-sum-exps into its own LDS strip with coalesced loads (when it fits), then every lane
// folds the chunks of its rounds.  The per-wave round masses are summed over the waves in LDS in a fixed
// order and written, not yet normalised, to p_part [B][Hq][Z][R_max]; scores_heads_kernel finishes.

template <int KPL>
__global__ __launch_bounds__(kFinishWaves * 64) void scores_finish_rows_kernel(FinishArgs a, float* p_part,
                                                                                bool stage_rows) {
    extern __shared__ __align__(16) char smem[];
    int* cum = reinterpret_cast<int*>(smem);                        // [R_max + 2]
    float* hs = reinterpret_cast<float*>(smem) + (a.R_max + 2);     // [kFinishWaves][R_max]
    float* rowbuf = hs + kFinishWaves * a.R_max;                    // [kFinishWaves][n_chunks_max] if staged
    const int b = blockIdx.x, h = blockIdx.y;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int R = min(max(a.n_rounds[b], 0), a.R_max);
    for (int r = tid; r < R; r += kFinishWaves * 64) cum[r] = chunks_of(max(a.seg_len[(size_t)b * a.R_max + r], 0), a.chunk_tokens);
    exclusive_scan_units(cum, R);
    const int hist_chunks = R > 0 ? cum[R] : 0;
    const int all_chunks = hist_chunks + (a.has_cur ? chunks_of(a.cur_len, a.chunk_tokens) : 0);
    const bool overflow = all_chunks > a.n_chunks_max;

    float qatt[KPL];
#pragma unroll
    for (int k = 0; k < KPL; ++k) qatt[k] = 0.f;
    float* mybuf = rowbuf + (size_t)wave * a.n_chunks_max;
    // One query token (then gridDim.z is 1): instead of leaving seven waves idle and one lane per round walking its
    // values one after the other, the eight waves share the rounds, and a wave folds a round's values with all its
    // lanes (coalesced reads; the second pass over the same values comes from cache).  The round's log-sum-exps meet
    // in LDS and wave 0 normalises them as below.
    const bool one_token = a.q_len == 1 && !a.has_cur;
    if (one_token && !overflow) {
        const float* row = a.part + ((size_t)b * a.Hq + h) * a.n_chunks_max;
        if (stage_rows) {  // the whole row into LDS with one round trip (the launch made room for it)
            for (int c = tid; c < hist_chunks; c += kFinishWaves * 64) rowbuf[c] = row[c];
            __syncthreads();
            row = rowbuf;
        }
        float* round_lse = hs;  // [R_max] of the [kFinishWaves][R_max] floats; rewritten below after a barrier
        for (int r = wave; r < R; r += kFinishWaves) {
            const int lo = cum[r], hi = cum[r + 1];
            float mx = -__builtin_inff();
            for (int k = lo + lane; k < hi; k += 64) mx = fmaxf(mx, row[k]);
            mx = wave_max(mx);
            float sum = 0.f;
            if (mx != -__builtin_inff())
                for (int k = lo + lane; k < hi; k += 64) sum += __expf(row[k] - mx);
            sum = wave_sum(sum);
            if (lane == 0) round_lse[r] = mx == -__builtin_inff() ? mx : mx + __logf(sum);
        }
        __syncthreads();
        if (wave == 0) {
            float lv[KPL];
            float mx = -__builtin_inff();
#pragma unroll
            for (int k = 0; k < KPL; ++k) {
                const int r = lane + 64 * k;
                lv[k] = r < R ? round_lse[r] : -__builtin_inff();
                mx = fmaxf(mx, lv[k]);
            }
            mx = wave_max(mx);
            if (mx != -__builtin_inff()) {
                float e[KPL], sum = 0.f;
#pragma unroll
                for (int k = 0; k < KPL; ++k) {
                    e[k] = __expf(lv[k] - mx);
                    sum += e[k];
                }
                const float inv = 1.f / wave_sum(sum);
#pragma unroll
                for (int k = 0; k < KPL; ++k) qatt[k] = e[k] * inv;
            }
        }
        __syncthreads();  // round_lse is part of hs, which every wave writes next
    }
    for (int i = blockIdx.z * kFinishWaves + wave; i < a.q_len && !overflow && !one_token; i += kFinishWaves * gridDim.z) {
        const float* row = a.part + (((size_t)b * a.Hq + h) * a.q_len + i) * a.n_chunks_max;
        if (stage_rows) {
            for (int c = lane; c < all_chunks; c += 64) mybuf[c] = row[c];
            __builtin_amdgcn_wave_barrier();  // same wave: LDS operations complete in program order
            row = mybuf;
        }
        float lv[KPL];
        float mx = -__builtin_inff();
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const int r = lane + 64 * k;
            lv[k] = r < R ? lse_range(row, cum[r], cum[r + 1]) : -__builtin_inff();
            mx = fmaxf(mx, lv[k]);
        }
        float lc = -__builtin_inff();
        if (a.has_cur) lc = lse_range(row, hist_chunks, all_chunks);
        __builtin_amdgcn_wave_barrier();
        mx = fmaxf(wave_max(mx), lc);
        if (mx == -__builtin_inff()) continue;  // this query token sees no key at all
        float e[KPL], sum = 0.f;
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            e[k] = __expf(lv[k] - mx);
            sum += e[k];
        }
        const float inv = 1.f / (wave_sum(sum) + __expf(lc - mx));
#pragma unroll
        for (int k = 0; k < KPL; ++k) qatt[k] = __builtin_fmaf(e[k], inv, qatt[k]);
    }
#pragma unroll
    for (int k = 0; k < KPL; ++k) {
        const int r = lane + 64 * k;
        if (r < a.R_max) hs[wave * a.R_max + r] = qatt[k];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const int r = lane + 64 * k;
            float tot = 0.f;
            if (r < R)
                for (int w = 0; w < kFinishWaves; ++w) tot += hs[w * a.R_max + r];
            if (r < a.R_max)
                p_part[(((size_t)b * a.Hq + h) * gridDim.z + blockIdx.z) * a.R_max + r] = overflow ? __builtin_nanf("") : tot;
        }
    }
}

// grid (B), block 1024: per head, the Z partial round masses are added in order and normalised over the rounds
// (Eq. 1; written to p_out [B][Hq][R_max] if given); scores[b][r] is the mean over heads.  A wave takes heads
// wave, wave + 16, ... and a lane the rounds lane, lane + 64, ..., so all sums run in a fixed order.
constexpr int kHeadsWaves = 16;
struct HeadsSelect {
    bool with_select;
    ra_select_params sel;
    const int32_t* n_rounds;
    int32_t* sel_idx;
    int32_t* n_sel;
};
__global__ __launch_bounds__(kHeadsWaves * 64) void scores_heads_kernel(const float* p_part, int Z, int R_max, int Hq,
                                                                        float* p_out, float* s_out, float* acc,
                                                                        HeadsSelect hsel) {
    extern __shared__ __align__(16) char smem[];
    float* sacc = reinterpret_cast<float*>(smem);  // [kHeadsWaves][R_max]
    constexpr int KPL = kMaxRounds / 64;
    const int b = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float mine[KPL];  // this wave's sum over its heads of the normalised masses of rounds lane + 64 k
#pragma unroll
    for (int k = 0; k < KPL; ++k) mine[k] = 0.f;
    for (int h = wave; h < Hq; h += kHeadsWaves) {
        const float* ph = p_part + ((size_t)b * Hq + h) * Z * R_max;
        float tot[KPL], all = 0.f;
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const int r = lane + 64 * k;
            tot[k] = 0.f;
            if (r < R_max)
                for (int z = 0; z < Z; ++z) tot[k] += ph[(size_t)z * R_max + r];
            if (acc && r < R_max && tot[k] == tot[k]) {  // (an undersized pass leaves the running masses alone)
                float* slot = acc + ((size_t)b * Hq + h) * R_max + r;
                tot[k] += *slot;
                *slot = tot[k];
            }
            all += tot[k];
        }
        all = wave_sum(all);
        const float inv = all > 0.f ? 1.f / all : (all == all ? 0.f : all);  // (NaN marks an undersized pass)
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const int r = lane + 64 * k;
            const float p = tot[k] * inv;
            if (p_out && r < R_max) p_out[((size_t)b * Hq + h) * R_max + r] = p;
            mine[k] += p;
        }
    }
#pragma unroll
    for (int k = 0; k < KPL; ++k)
        if (lane + 64 * k < R_max) sacc[wave * R_max + lane + 64 * k] = mine[k];
    __syncthreads();
    const float inv_h = 1.f / (float)Hq;
    for (int r = threadIdx.x; r < R_max; r += kHeadsWaves * 64) {
        float s = 0.f;
        for (int w = 0; w < kHeadsWaves; ++w) s += sacc[w * R_max + r];
        const float val = s * inv_h;
        s_out[(size_t)b * R_max + r] = val;
        if (hsel.with_select) sacc[r] = val;  // (a thread only ever touches its own column r of sacc)
    }
    if (hsel.with_select) {  // Sec. 3.3 on the scores just written, same bits
        __shared__ SelectShared<kHeadsWaves> sh;
        __syncthreads();
        const int R = min(max(hsel.n_rounds[b], 0), R_max);
        select_rounds_block<kHeadsWaves>(sacc, R, R_max, hsel.sel, hsel.sel_idx + (size_t)b * R_max, hsel.n_sel + b, sh);
    }
}

template <typename T, int D, int G>
static void launch_scores(bool paged, dim3 grid, size_t smem, hipStream_t st, const ScoreArgs& a) {
    if (paged)
        RA_LAUNCH_TIMED((scores_stream_kernel<T, D, G, true>), grid, dim3(256), smem, st, a);
    else
        RA_LAUNCH_TIMED((scores_stream_kernel<T, D, G, false>), grid, dim3(256), smem, st, a);
}

template <typename T, int D>
static int dispatch_scores(int G, bool paged, dim3 grid, size_t smem, hipStream_t st, const ScoreArgs& a) {
    switch (G) {
        case 1: launch_scores<T, D, 1>(paged, grid, smem, st, a); return RA_OK;
        case 2: launch_scores<T, D, 2>(paged, grid, smem, st, a); return RA_OK;
        case 4: launch_scores<T, D, 4>(paged, grid, smem, st, a); return RA_OK;
        case 8: launch_scores<T, D, 8>(paged, grid, smem, st, a); return RA_OK;
        default: return fail(RA_ERR_UNSUPPORTED, "round_scores: Hq / Hkv = %d not in {1, 2, 4, 8}", G);
    }
}

}  // namespace ra

using namespace ra;

namespace ra {
// Several query tokens: Z workgroups per (sequence, head) leave partial round masses in p_part
// [B][Hq][Z][R_max], a second kernel adds, normalises and averages them.
int scores_finish_splits(int q_len, int B, int Hq) {
    int Z = q_len / 32 < 1 ? 1 : (q_len / 32 > 8 ? 8 : q_len / 32);
    while (Z > 1 && (int64_t)B * Hq * Z > 2048) --Z;
    return Z;
}
void launch_scores_finish_rows(const FinishArgs& f, int B, float* p_part, int Z, hipStream_t st) {
    const int R_max = f.R_max, Hq = f.Hq, n_chunks_max = f.n_chunks_max;
    const size_t fin_smem = (size_t)(R_max + 2) * sizeof(int) + (size_t)kFinishWaves * R_max * sizeof(float);
    const dim3 fin_block(kFinishWaves * 64);
    bool stage_rows =
        n_chunks_max <= kRowBufMax && fin_smem + (size_t)kFinishWaves * n_chunks_max * sizeof(float) <= 60 * 1024;
    size_t smem = fin_smem + (stage_rows ? (size_t)kFinishWaves * n_chunks_max * sizeof(float) : 0);
    if (f.q_len == 1 && !f.has_cur) {  // one row per workgroup, shared by its waves: staged whole if it fits
        stage_rows = fin_smem + (size_t)n_chunks_max * sizeof(float) <= 60 * 1024;
        smem = fin_smem + (stage_rows ? (size_t)n_chunks_max * sizeof(float) : 0);
    }
    const dim3 fgrid(B, Hq, Z);
    if (R_max <= 64)
        hipLaunchKernelGGL((scores_finish_rows_kernel<1>), fgrid, fin_block, smem, st, f, p_part, stage_rows);
    else if (R_max <= 256)
        hipLaunchKernelGGL((scores_finish_rows_kernel<4>), fgrid, fin_block, smem, st, f, p_part, stage_rows);
    else
        hipLaunchKernelGGL((scores_finish_rows_kernel<kMaxRounds / 64>), fgrid, fin_block, smem, st, f, p_part,
                           stage_rows);
    HeadsSelect hsel;
    hsel.with_select = f.with_select;
    hsel.sel = f.sel;
    hsel.n_rounds = f.n_rounds;
    hsel.sel_idx = f.sel_idx;
    hsel.n_sel = f.n_sel;
    hipLaunchKernelGGL(scores_heads_kernel, dim3(B), dim3(kHeadsWaves * 64), (size_t)kHeadsWaves * R_max * sizeof(float),
                       st, p_part, Z, R_max, Hq, f.p_out, f.s_out, f.acc, hsel);
}

// One query token: the finishing kernel for B sequences (a.q_len must be 1).
void launch_scores_finish_single(const FinishArgs& f, int B, hipStream_t st) {
    const int R_max = f.R_max, Hq = f.Hq, n_chunks_max = f.n_chunks_max;
    const size_t fin_smem = (size_t)(R_max + 2) * sizeof(int) + (size_t)kFinishWaves * R_max * sizeof(float);
    const dim3 fin_block(kFinishWaves * 64);
    const bool stage_rows =
        n_chunks_max <= kRowBufMax && fin_smem + (size_t)kFinishWaves * n_chunks_max * sizeof(float) <= 60 * 1024;
    const size_t smem = fin_smem + (stage_rows ? (size_t)kFinishWaves * n_chunks_max * sizeof(float) : 0);
    // sixteen waves (two heads each at Hq = 32) when the per-wave LDS strips still fit
    const size_t smem16 = (size_t)(R_max + 2) * sizeof(int) + (size_t)16 * R_max * sizeof(float) +
                          (stage_rows ? (size_t)16 * n_chunks_max * sizeof(float) : 0);
    if (R_max <= 64 && Hq > 8 && smem16 <= 60 * 1024)
        hipLaunchKernelGGL((scores_finish_kernel<1, 16>), dim3(B), dim3(1024), smem16, st, f, stage_rows);
    else if (R_max <= 64)
        hipLaunchKernelGGL((scores_finish_kernel<1, kFinishWaves>), dim3(B), fin_block, smem, st, f, stage_rows);
    else if (R_max <= 256 && Hq > 8 && smem16 <= 60 * 1024)
        hipLaunchKernelGGL((scores_finish_kernel<4, 16>), dim3(B), dim3(1024), smem16, st, f, stage_rows);
    else if (R_max <= 256)
        hipLaunchKernelGGL((scores_finish_kernel<4, kFinishWaves>), dim3(B), fin_block, smem, st, f, stage_rows);
    else
        hipLaunchKernelGGL((scores_finish_kernel<kMaxRounds / 64, kFinishWaves>), dim3(B), fin_block, smem, st, f,
                           stage_rows);
}
void launch_scores_finish(const FinishArgs& f, int B, float* p_part, hipStream_t st) {
    if (scores_finish_by_rows(f.q_len, f.Hq, f.n_chunks_max))
        launch_scores_finish_rows(f, B, p_part, scores_finish_splits(f.q_len, B, f.Hq), st);
    else
        launch_scores_finish_single(f, B, st);
}
}  // namespace ra

static int scores_impl(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq, const ra_kv_view* watershed,
                       const void* cur_k, int cur_len, float scale, float* acc, float* scores_head, float* scores,
                       const ra_select_params* sel = nullptr, int32_t* sel_idx = nullptr, int32_t* n_sel = nullptr) {
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
    if (sel) {
        RA_REQUIRE(sel_idx != nullptr && n_sel != nullptr, RA_ERR_INVALID_ARG, "round_scores_select: sel_idx or n_sel is NULL");
        if (int rc = check_select_params(sel, "round_scores_select")) return rc;
    }
    const int G = Hq / watershed->Hkv, D = watershed->d, B = watershed->B, R_max = watershed->R_max;
    RA_REQUIRE(D == 64 || D == 128, RA_ERR_UNSUPPORTED, "round_scores: head_dim %d not in {64, 128}", D);
    RA_REQUIRE((int64_t)B * q_len <= 65535, RA_ERR_UNSUPPORTED, "round_scores: B * q_len exceeds 65535");

    // With a single query token the current round's share of the softmax cancels in the
    // normalisation over history rounds, so its keys need not be read at all -- unless the masses are
    // added to those of other tokens, each with its own share.
    const bool use_cur = cur_k != nullptr && (q_len > 1 || acc != nullptr);
    const bool mfma = watershed->dtype == RA_BF16 && D == 128;
    const int chunk_tokens = kChunkTokens;
    const int64_t nc64 = watershed->max_tokens / chunk_tokens + R_max + (use_cur ? (cur_len + chunk_tokens - 1) / chunk_tokens : 0);
    RA_REQUIRE(nc64 <= (int64_t)1 << 24, RA_ERR_UNSUPPORTED, "round_scores: max_tokens too large");
    const int n_chunks_max = (int)(nc64 < 1 ? 1 : nc64);
    const size_t rows = (size_t)B * Hq * q_len;
    const size_t part_bytes = align_up(rows * n_chunks_max * sizeof(float), 256);
    // several query tokens (or many chunks): Z workgroups per head leave partial round masses in a buffer
    const size_t p_bytes = scores_finish_part_bytes(q_len, B, Hq, R_max, n_chunks_max);
    // more than 16 query rows per KV head on the matrix cores: persistent kernel driven by segment tables
    const bool many_rows = mfma && q_len * G > 16;
    if (mfma) RA_REQUIRE(G <= 16, RA_ERR_UNSUPPORTED, "round_scores: Hq / Hkv = %d exceeds 16", G);
    if (many_rows) RA_REQUIRE(B <= kMaxBatch, RA_ERR_UNSUPPORTED, "round_scores: batch %d exceeds %d", B, kMaxBatch);
    const size_t plan_bytes = many_rows ? align_up((size_t)B * plan_stride(R_max + 1), 256) : 0;
    // few rows on the matrix cores: one 16-byte descriptor per (sequence, chunk)
    const size_t desc_bytes = mfma && !many_rows ? align_up((size_t)B * n_chunks_max * 16, 256) : 0;
    RA_REQUIRE(ctx->ws.base != nullptr && ctx->ws.bytes >= kWsReserved + part_bytes + p_bytes + plan_bytes + desc_bytes,
               RA_ERR_WORKSPACE, "round_scores: workspace has %zu bytes, this call needs %zu", ctx->ws.bytes,
               kWsReserved + part_bytes + p_bytes + plan_bytes + desc_bytes);

    ScoreArgs a;
    a.view = to_dev(watershed);
    a.q = q;
    a.cur_k = use_cur ? cur_k : nullptr;
    a.cur_len = use_cur ? cur_len : 0;
    a.q_len = q_len;
    a.Hq = Hq;
    a.n_chunks_max = n_chunks_max;
    a.chunk_tokens = chunk_tokens;
    a.c = scale * kLog2e;
    a.part = reinterpret_cast<float*>(ctx->ws.base + kWsReserved);
    a.plan = ctx->ws.base + kWsReserved + part_bytes + p_bytes;
    a.chunks = desc_bytes ? ctx->ws.base + kWsReserved + part_bytes + p_bytes + plan_bytes : nullptr;
    a.S = 1 << 20;
    a.min_units = 16;

    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const dim3 grid(n_chunks_max, watershed->Hkv, B * q_len);
    const size_t tab_bytes = (size_t)(R_max + 1) * 16 + 16;
    const bool paged = watershed->block_size != 0;
    int rc;
    if (many_rows) launch_scores_plan(a, st);
    {
        KernelTimer timer(ctx, st);
        if (many_rows)
            rc = launch_scores_prefill_mfma(a, paged, ctx->num_cu, st);
        else if (mfma)
            rc = launch_scores_mfma(a, paged, ctx->num_cu, st);
        else if (watershed->dtype == RA_BF16)
            rc = dispatch_scores<BF16, 64>(G, paged, grid, tab_bytes, st, a);
        else
            rc = D == 128 ? dispatch_scores<F32, 128>(G, paged, grid, tab_bytes, st, a)
                          : dispatch_scores<F32, 64>(G, paged, grid, tab_bytes, st, a);
    }
    if (rc) return rc;

    FinishArgs f;
    f.part = a.part;
    f.n_rounds = watershed->n_rounds;
    f.seg_len = watershed->seg_len;
    f.R_max = R_max;
    f.Hq = Hq;
    f.q_len = q_len;
    f.cur_len = a.cur_len;
    f.n_chunks_max = n_chunks_max;
    f.chunk_tokens = chunk_tokens;
    f.has_cur = use_cur;
    f.p_out = scores_head;
    f.s_out = scores;
    f.acc = acc;
    if (sel) {
        f.with_select = true;
        f.sel = *sel;
        f.sel_idx = sel_idx;
        f.n_sel = n_sel;
    }
    launch_scores_finish(f, B, reinterpret_cast<float*>(ctx->ws.base + kWsReserved + part_bytes), st);
    RA_HIP_CHECK(hipGetLastError());
    return RA_OK;
}

extern "C" int ra_round_scores(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq,
                               const ra_kv_view* watershed, const void* cur_k, int cur_len, float scale,
                               float* scores_head, float* scores) {
    return scores_impl(ctx, stream, q, q_len, Hq, watershed, cur_k, cur_len, scale, nullptr, scores_head, scores);
}

extern "C" int ra_round_scores_accumulate(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq,
                                          const ra_kv_view* watershed, const void* cur_k, int cur_len, float scale,
                                          float* acc, float* scores_head, float* scores) {
    RA_REQUIRE(acc != nullptr, RA_ERR_INVALID_ARG, "round_scores_accumulate: acc is NULL");
    return scores_impl(ctx, stream, q, q_len, Hq, watershed, cur_k, cur_len, scale, acc, scores_head, scores);
}

extern "C" int ra_round_scores_select(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq,
                                      const ra_kv_view* watershed, const void* cur_k, int cur_len, float scale,
                                      const ra_select_params* params, float* scores_head, float* scores,
                                      int32_t* sel_idx, int32_t* n_sel) {
    RA_REQUIRE(params != nullptr, RA_ERR_INVALID_ARG, "round_scores_select: params is NULL");
    return scores_impl(ctx, stream, q, q_len, Hq, watershed, cur_k, cur_len, scale, nullptr, scores_head, scores, params,
                       sel_idx, n_sel);
}
