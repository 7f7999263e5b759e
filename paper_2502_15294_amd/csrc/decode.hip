// Round-sparse decode attention (paper Sec. 3.2 step 5): one query token per sequence attends over
// the KV segments of the selected rounds, gathered through the round-offset index, plus the
// current round.  HBM-bandwidth bound: K and V of every selected token are read exactly once and
// serve all Hq/Hkv query heads of their KV head.
//
// This file holds the entry points, the planning kernel, and the generic vector-ALU kernel with its merge kernel,
// used for fp32 caches and head_dim 64; bf16 with head_dim 128 goes to the matrix-core kernel (attn_mfma.hip),
// which has a schedule of its own (one wavefront per equal range of the batch's key tiles).
//
// Work decomposition of the generic kernel: grid (S, Hkv, B).  A workgroup (4 wavefronts) owns KV head g of
// sequence b and the s-th of S_eff equal shares of that sequence's work units, S_eff <= S being chosen
// on the device from the number of selected tokens.  Its waves take units round-robin, keep an
// online-softmax state in registers and are merged through LDS into one piece (max, sum, d
// accumulators) per query head.  A sequence with a short selection is not split and its output is
// written directly; otherwise a second small kernel merges the pieces.
#include "attn_common.hpp"
#include "scores_common.hpp"
#include "stream_kv.hpp"

namespace ra {

// Smallest piece a sequence's key set is cut into, in 32-token tiles (pieces of 4 and of 16 tiles measured slower).
int attn_min_units() { return 8; }

size_t attn_plan_bytes(int B, int R_max) { return (size_t)B * plan_stride(R_max + 1); }

// Planning kernel, grid (B): resolves the selection of sequence b into the table of segments its
// attention runs over (selected history rounds in list order, then the current round), with the
// prefix sum of their work-unit counts, and decides into how many pieces the sequence is cut.
__global__ __launch_bounds__(256) void plan_kernel(AttnArgs a, int unit_tokens) {
    extern __shared__ __align__(16) char smem[];
    const DevView& vw = a.view;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int cap = vw.R_max + 1;
    int* cum = reinterpret_cast<int*>(smem);
    char* plan_b = a.plan + (size_t)b * plan_stride(cap);
    long long* g_off_k = reinterpret_cast<long long*>(plan_b + sizeof(PlanHeader));
    long long* g_off_v = g_off_k + cap;
    int* g_len = reinterpret_cast<int*>(g_off_v + cap);
    int* g_cum = g_len + cap;

    const int n_rounds = min(max(vw.n_rounds[b], 0), vw.R_max);
    const int n_hist = a.sel_idx ? min(max(a.n_sel[b], 0), vw.R_max) : n_rounds;
    int cur_len = 0;
    if (a.cur_k) cur_len = min(max(a.cur_len_dev ? a.cur_len_dev[b] : a.cur_len_host, 0), a.cur_cap);
    const int n_slots = n_hist + (cur_len > 0 ? 1 : 0);
    for (int i = tid; i < cap; i += 256) {
        int len = 0;
        long long ok = 0, ov = 0;
        // the list entry is asked for before the counts have arrived (one memory round trip less)
        const int listed = (a.sel_idx && i < vw.R_max) ? a.sel_idx[(size_t)b * vw.R_max + i] : i;
        if (i < n_hist) {
            const int r = listed;
            if (r >= 0 && r < n_rounds) {  // entries that are not rounds of this sequence are ignored
                len = max(vw.seg_len[(size_t)b * vw.R_max + r], 0);
                ok = vw.seg_off[(size_t)b * vw.R_max + r];
                ov = vw.seg_off_v[(size_t)b * vw.R_max + r];
            }
        } else if (i < n_slots) {
            len = cur_len;
        }
        g_len[i] = len;
        g_off_k[i] = ok;
        g_off_v[i] = ov;
        cum[i] = (len + unit_tokens - 1) / unit_tokens;
    }
    exclusive_scan_units(cum, cap);
    for (int i = tid; i <= cap; i += 256) g_cum[i] = cum[i];
    if (tid == 0) {
        const int U = cum[n_slots];
        const int S_eff = min(a.S, max(1, U / a.min_units));
        PlanHeader h;
        h.n_slots = n_slots;
        h.n_hist = n_hist;
        h.U = U;
        h.S_eff = S_eff;
        *reinterpret_cast<PlanHeader*>(plan_b) = h;
        a.n_parts[b] = S_eff;
    }
}

void launch_plan(const AttnArgs& a, int unit_tokens, hipStream_t st) {
    const size_t smem = (size_t)(a.view.R_max + 3) * sizeof(int);
    hipLaunchKernelGGL(plan_kernel, dim3(a.view.B), dim3(256), smem, st, a, unit_tokens);
}

// Generic kernel.  A unit is 16 tokens.  Scores: the wave is four rows of 16 lanes, row `grp` takes one
// token at a time and lane `sub` owns D/16 channels of the key; four DPP adds finish a dot product.
// Values are stored transposed in 16-token tiles ([D][16]), so for P.V lane `lane` owns channels
// lane, lane + 64, ... and reads the 16 tokens of each with contiguous loads; the 16 x G probabilities
// of the unit reach it as scalars (v_readlane), so P.V needs no cross-lane reduction.
template <typename T, int D, int G, bool PAGED>
__global__ __launch_bounds__(256) void decode_generic_kernel(AttnArgs a) {
    constexpr int EPL = D / 16;
    using Ops = RowOps<T, EPL>;
    constexpr int WORDS = Ops::WORDS;
    constexpr int EB = Ops::ELEM_BYTES;
    constexpr int DPL = D / 64;                 // channels per lane in the P.V phase
    constexpr int VW = kUnitTokens * EB / 4;    // 32-bit words of one channel's 16 tokens

    extern __shared__ __align__(16) char smem[];
    const int b = blockIdx.z, g = blockIdx.y, s = blockIdx.x;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, grp = lane >> 4, sub = lane & 15;
    const DevView& vw = a.view;
    const int Hkv = vw.Hkv;

    const int cap = vw.R_max + 1;
    SlotTable tab;
    tab.carve(smem, cap);
    float* red = reinterpret_cast<float*>(smem + ((SlotTable::bytes(cap) + 15) & ~(size_t)15));
    const PlanHeader hdr = load_plan(a.plan + (size_t)b * plan_stride(cap), cap, tab);
    const int n_slots = hdr.n_slots, n_hist = hdr.n_hist, U = hdr.U, S_eff = hdr.S_eff;
    if (s >= S_eff) return;
    __syncthreads();
    const int u_lo = (int)(((long long)U * s) / S_eff);
    const int u_hi = (int)(((long long)U * (s + 1)) / S_eff);

    uint32_t qw[G][WORDS];
    {
        const char* qp = reinterpret_cast<const char*>(a.q) + ((size_t)b * a.Hq + (size_t)g * G) * D * EB;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            Frag<WORDS> f = load_frag<WORDS>(qp + ((size_t)h * D + sub * EPL) * EB);
#pragma unroll
            for (int e = 0; e < WORDS; ++e) qw[h][e] = f.w[e];
        }
    }
    float m[G], l[G], acc[G][DPL];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = kNegBig;
        l[h] = 0.f;
#pragma unroll
        for (int k = 0; k < DPL; ++k) acc[h][k] = 0.f;
    }
    const char* kbase = reinterpret_cast<const char*>(vw.k);
    const char* vbase = reinterpret_cast<const char*>(vw.v);

    for (int u = u_lo + wave, slot = -1; u < u_hi; u += 4) {
        if (slot < 0) slot = find_slot(tab.cum, n_slots, u);
        while (u >= tab.cum[slot + 1]) ++slot;
        const int len = tab.len[slot];
        const int uin = u - tab.cum[slot];
        const int tok0 = uin * kUnitTokens;
        const int ntok = min(kUnitTokens, len - tok0);
        const bool is_cur = slot >= n_hist;
        // ---- keys: four steps of four tokens -----------------------------------------------------
        const char* kp;
        size_t kstride;
        if (is_cur) {
            kp = reinterpret_cast<const char*>(a.cur_k) + ((((size_t)b * a.cur_cap + tok0) * Hkv + g) * D) * EB;
            kstride = (size_t)Hkv * D * EB;
        } else if (PAGED) {
            long long si = tab.off_k[slot] + uin;
            si = si < 0 ? 0 : (si >= vw.max_blocks ? vw.max_blocks - 1 : si);
            const int pb = max(vw.block_table[(size_t)b * vw.max_blocks + si], 0);
            kp = kbase + ((((size_t)pb * Hkv + g) * kUnitTokens) * D) * EB;
            kstride = (size_t)D * EB;
        } else {
            kp = kbase + (((size_t)tab.off_k[slot] * Hkv + (size_t)g * len + tok0) * D) * EB;
            kstride = (size_t)D * EB;
        }
        Frag<WORDS> kf[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = min(j * 4 + grp, ntok - 1);  // rows past the segment's end re-read its last row
            kf[j] = load_frag<WORDS>(kp + (size_t)t * kstride + (size_t)sub * EPL * EB);
        }
        // ---- values: 16 tokens of each of this lane's channels ---------------------------------------
        float vf[DPL][kUnitTokens];
        if (is_cur) {  // token-major: strided gather (the current round is short)
#pragma unroll
            for (int k = 0; k < DPL; ++k)
#pragma unroll
                for (int t = 0; t < kUnitTokens; ++t) {
                    const int tt = min(tok0 + t, len - 1);
                    const char* p = reinterpret_cast<const char*>(a.cur_v) +
                                    ((((size_t)b * a.cur_cap + tt) * Hkv + g) * D + lane + 64 * k) * EB;
                    if constexpr (EB == 4) vf[k][t] = *reinterpret_cast<const float*>(p);
                    else vf[k][t] = as_f32((uint32_t)*reinterpret_cast<const unsigned short*>(p) << 16);
                }
        } else {
            const char* vp;
            if (PAGED) {
                long long si = tab.off_k[slot] + uin;
                si = si < 0 ? 0 : (si >= vw.max_blocks ? vw.max_blocks - 1 : si);
                const int pb = max(vw.block_table[(size_t)b * vw.max_blocks + si], 0);
                vp = vbase + (((size_t)pb * Hkv + g) * D * kUnitTokens) * EB;
            } else {
                const size_t L16 = (size_t)((len + 15) >> 4) * 16;
                vp = vbase + (((size_t)tab.off_v[slot] * Hkv + (size_t)g * L16 + tok0) * D) * EB;
            }
#pragma unroll
            for (int k = 0; k < DPL; ++k) {
                Frag<VW> f = load_frag<VW>(vp + (size_t)(lane + 64 * k) * kUnitTokens * EB);
                if constexpr (EB == 4) {
#pragma unroll
                    for (int t = 0; t < kUnitTokens; ++t) vf[k][t] = as_f32(f.w[t]);
                } else {
#pragma unroll
                    for (int t = 0; t < kUnitTokens / 2; ++t) {
                        vf[k][2 * t] = as_f32(f.w[t] << 16);
                        vf[k][2 * t + 1] = as_f32(f.w[t] & 0xffff0000u);
                    }
                }
            }
        }
        // ---- scores and online softmax with one running max per head for the whole wave ------------------
        float p[4][G];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float sc[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float d = row16_sum(Ops::dot(kf[j].w, qw[h]));
                sc[j] = (j * 4 + grp) < ntok ? d : -__builtin_inff();
            }
            float mx = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
            mx = xrow_max4(mx);
            const float m_new = fmaxf(m[h], mx);
            const float mc = m_new * a.c;
            const float alpha = fast_exp2((m[h] - m_new) * a.c);  // exactly 1 when the maximum did not move
            m[h] = m_new;
            float ps = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                p[j][h] = fast_exp2(__builtin_fmaf(sc[j], a.c, -mc));
                ps += p[j][h];
            }
            l[h] = __builtin_fmaf(l[h], alpha, ps);  // partial sum of this lane row; rows are added at the end
#pragma unroll
            for (int k = 0; k < DPL; ++k) acc[h][k] *= alpha;
        }
        // ---- P.V: token (j, grp) lives in lane row grp; broadcast its probability as a scalar ---------------
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int gr = 0; gr < 4; ++gr)
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const float pv = as_f32((uint32_t)__builtin_amdgcn_readlane((int)as_u32(p[j][h]), gr * 16));
#pragma unroll
                    for (int k = 0; k < DPL; ++k) acc[h][k] = __builtin_fmaf(pv, vf[k][j * 4 + gr], acc[h][k]);
                }
    }

    // ---- merge: lane rows (sum only; max is already wave-wide), then the four waves through LDS ---------------
    float* sm = red;             // [4][G]
    float* sl = red + 4 * G;     // [4][G]
    float* sacc = red + 8 * G;   // [4][G][D]
#pragma unroll
    for (int h = 0; h < G; ++h) {
        float lv = l[h];
        lv = xrow_sum4(lv);
        if (lane == 0) {
            sm[wave * G + h] = m[h];
            sl[wave * G + h] = lv;
        }
#pragma unroll
        for (int k = 0; k < DPL; ++k) sacc[(wave * G + h) * D + lane + 64 * k] = acc[h][k];
    }
    __syncthreads();
    const size_t row0 = (size_t)b * a.Hq + (size_t)g * G;
    for (int idx = tid; idx < G * D; idx += 256) {
        const int h = idx / D, dim = idx - h * D;
        const float M = fmaxf(fmaxf(sm[h], sm[G + h]), fmaxf(sm[2 * G + h], sm[3 * G + h]));
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float f = fast_exp2((sm[w * G + h] - M) * a.c);
            num = __builtin_fmaf(sacc[(w * G + h) * D + dim], f, num);
            den = __builtin_fmaf(sl[w * G + h], f, den);
        }
        if (S_eff > 1) {
            const size_t pr = (row0 + h) * a.S + s;
            a.part_acc[pr * D + dim] = num;
            if (dim == 0) {
                a.part_m[pr] = M;
                a.part_l[pr] = den;
            }
        } else {
            a.out[(row0 + h) * D + dim] = den > 0.f ? num / den : 0.f;
            if (a.lse && dim == 0)
                a.lse[row0 + h] = den > 0.f ? __builtin_fmaf(M, a.scale, __builtin_logf(den)) : -__builtin_inff();
        }
    }
}

// Merge the pieces of every (sequence, query token, query head) row that was split; grid (rows), block D.
template <int D>
__global__ __launch_bounds__(D) void combine_kernel(const float* part_acc, const float* part_m, const float* part_l,
                                                   const int* n_parts, int S, int rows_per_seq, float c, float scale,
                                                   float* out, float* lse) {
    const size_t row = blockIdx.x;
    const int n = n_parts[row / rows_per_seq];
    if (n <= 1) return;  // written directly by the streaming kernel
    const int dim = threadIdx.x;
    const float* pm = part_m + row * S;
    const float* pl = part_l + row * S;
    const float* pa = part_acc + row * S * D + dim;
    float M = kNegBig;
    for (int p = 0; p < n; ++p) M = fmaxf(M, pm[p]);
    float num = 0.f, den = 0.f;
    int p = 0;
    for (; p + 4 <= n; p += 4) {
        const float a0 = pa[(size_t)p * D], a1 = pa[(size_t)(p + 1) * D];
        const float a2 = pa[(size_t)(p + 2) * D], a3 = pa[(size_t)(p + 3) * D];
        const float f0 = fast_exp2((pm[p] - M) * c), f1 = fast_exp2((pm[p + 1] - M) * c);
        const float f2 = fast_exp2((pm[p + 2] - M) * c), f3 = fast_exp2((pm[p + 3] - M) * c);
        num = __builtin_fmaf(a0, f0, num); den = __builtin_fmaf(pl[p], f0, den);
        num = __builtin_fmaf(a1, f1, num); den = __builtin_fmaf(pl[p + 1], f1, den);
        num = __builtin_fmaf(a2, f2, num); den = __builtin_fmaf(pl[p + 2], f2, den);
        num = __builtin_fmaf(a3, f3, num); den = __builtin_fmaf(pl[p + 3], f3, den);
    }
    for (; p < n; ++p) {
        const float f = fast_exp2((pm[p] - M) * c);
        num = __builtin_fmaf(pa[(size_t)p * D], f, num);
        den = __builtin_fmaf(pl[p], f, den);
    }
    out[row * D + dim] = den > 0.f ? num / den : 0.f;
    if (lse && dim == 0) lse[row] = den > 0.f ? __builtin_fmaf(M, scale, __builtin_logf(den)) : -__builtin_inff();
}

void launch_combine(const AttnArgs& a, int D, size_t rows, hipStream_t st) {
    const int rows_per_seq = a.q_len * a.Hq;
    if (D == 128)
        hipLaunchKernelGGL((combine_kernel<128>), dim3((unsigned)rows), dim3(128), 0, st, a.part_acc, a.part_m, a.part_l,
                           a.n_parts, a.S, rows_per_seq, a.c, a.scale, a.out, a.lse);
    else
        hipLaunchKernelGGL((combine_kernel<64>), dim3((unsigned)rows), dim3(64), 0, st, a.part_acc, a.part_m, a.part_l,
                           a.n_parts, a.S, rows_per_seq, a.c, a.scale, a.out, a.lse);
}

template <typename T, int D, int G>
static void launch_generic(bool paged, dim3 grid, size_t smem, hipStream_t st, const AttnArgs& a) {
    if (paged)
        RA_LAUNCH_TIMED((decode_generic_kernel<T, D, G, true>), grid, dim3(256), smem, st, a);
    else
        RA_LAUNCH_TIMED((decode_generic_kernel<T, D, G, false>), grid, dim3(256), smem, st, a);
}

template <typename T, int D>
static int dispatch_generic(bool paged, dim3 grid, hipStream_t st, const AttnArgs& a, size_t tab_bytes) {
    auto smem = [&](int g) { return tab_bytes + (size_t)(8 * g + 4 * g * D) * sizeof(float); };
    switch (a.G) {
        case 1: launch_generic<T, D, 1>(paged, grid, smem(1), st, a); return RA_OK;
        case 2: launch_generic<T, D, 2>(paged, grid, smem(2), st, a); return RA_OK;
        case 4: launch_generic<T, D, 4>(paged, grid, smem(4), st, a); return RA_OK;
        case 8: launch_generic<T, D, 8>(paged, grid, smem(8), st, a); return RA_OK;
        default: return fail(RA_ERR_UNSUPPORTED, "decode: Hq / Hkv = %d not in {1, 2, 4, 8}", a.G);
    }
}

}  // namespace ra

using namespace ra;

// Shared by the two decode entry points.  With `scores` given (watershed layer) the attention runs over every
// history round and the kernel also leaves one log-sum-exp per 32-token key tile, which the finishing kernel of
// the score pass turns into Eq. 1.
static int decode_impl(ra_ctx* ctx, const Workspace* scratch, void* stream, const void* q, int Hq, const ra_kv_view* layer,
                       const int32_t* sel_idx, const int32_t* n_sel, const void* cur_k, const void* cur_v,
                       const int32_t* cur_len, int cur_cap, float scale, float* out, float* lse, float* scores_head,
                       float* scores) {
    RA_REQUIRE(ctx != nullptr, RA_ERR_INVALID_ARG, "decode: ctx is NULL");
    const Workspace ws = scratch ? *scratch : ctx->ws;  // the context's workspace, or the built-in scratch
    RA_REQUIRE(q != nullptr && out != nullptr, RA_ERR_INVALID_ARG, "decode: q or out is NULL");
    if (int rc = check_view(layer, true, "decode")) return rc;
    RA_REQUIRE(Hq > 0 && Hq % layer->Hkv == 0, RA_ERR_INVALID_ARG, "decode: Hq %d is not a multiple of Hkv %d", Hq,
               layer->Hkv);
    RA_REQUIRE((sel_idx == nullptr) == (n_sel == nullptr), RA_ERR_INVALID_ARG,
               "decode: sel_idx and n_sel must both be given or both be NULL");
    const bool has_cur = cur_k != nullptr || cur_v != nullptr || cur_len != nullptr;
    if (has_cur) {
        RA_REQUIRE(cur_k && cur_v && cur_len && cur_cap > 0, RA_ERR_INVALID_ARG,
                   "decode: cur_k, cur_v, cur_len and cur_cap > 0 must be given together");
    }
    RA_REQUIRE(layer->R_max > 0 || has_cur, RA_ERR_INVALID_ARG,
               "decode: no history rounds and no current round: the key set is empty");
    RA_REQUIRE(scale > 0.f && scale == scale, RA_ERR_INVALID_ARG, "decode: scale must be positive");
    const int G = Hq / layer->Hkv, D = layer->d, B = layer->B;
    RA_REQUIRE(D == 64 || D == 128, RA_ERR_UNSUPPORTED, "decode: head_dim %d not in {64, 128}", D);
    const bool mfma = layer->dtype == RA_BF16 && D == 128;
    if (mfma)
        RA_REQUIRE(G <= 16, RA_ERR_UNSUPPORTED, "decode: Hq / Hkv = %d exceeds 16", G);
    else
        RA_REQUIRE(G == 1 || G == 2 || G == 4 || G == 8, RA_ERR_UNSUPPORTED,
                   "decode: Hq / Hkv = %d not in {1, 2, 4, 8} for this dtype / head_dim", G);
    RA_REQUIRE((size_t)B * sizeof(int) <= kWsSmallState, RA_ERR_UNSUPPORTED, "decode: B = %d exceeds %zu", B,
               kWsSmallState / sizeof(int));

    const bool with_scores = scores != nullptr;
    if (with_scores) {
        RA_REQUIRE(mfma, RA_ERR_UNSUPPORTED, "watershed decode: only bf16 with head_dim 128 is implemented");
        RA_REQUIRE(layer->R_max > 0, RA_ERR_INVALID_ARG, "watershed decode: R_max is 0, there is nothing to score");
    }

    const int64_t max_tok = layer->max_tokens + (has_cur ? cur_cap : 0);
    const size_t rows = (size_t)B * Hq;
    // scratch: the matrix-core kernel keeps one partial result per (range, sequence) it cuts; the generic kernel
    // one per (sequence, split)
    MfmaDecodeShape shape = {};
    size_t plan_off, scratch_total;
    int S = 1;
    AttnWorkspace w = {};
    MfmaDecodeWorkspace mw = {};
    if (mfma) {
        RA_REQUIRE(B <= kMaxBatch, RA_ERR_UNSUPPORTED, "decode: batch %d exceeds %d", B, kMaxBatch);
        const long long max_tiles = mfma_max_tiles(B, layer->max_tokens, layer->R_max, has_cur ? cur_cap : 0);
        RA_REQUIRE(max_tiles < ((long long)1 << 30), RA_ERR_UNSUPPORTED, "decode: max_tokens too large for this batch");
        shape = mfma_decode_shape(ctx->num_cu, B, layer->R_max, layer->Hkv, G, max_tiles);
        mw = mfma_decode_workspace(shape, B, layer->R_max);
        plan_off = mw.plan_off;
        scratch_total = mw.total;
    } else {
        S = decode_splits(ctx->num_cu, B, layer->Hkv, max_tok);
        w = attn_workspace(rows, S, D, B, layer->R_max);
        plan_off = w.plan_off;
        scratch_total = w.total;
    }
    // one entry per 32-token tile of a sequence's table: history rounds (each rounded up), then the current round
    const int64_t n_tiles64 = layer->max_tokens / 32 + layer->R_max + (has_cur ? cur_cap / 32 + 1 : 0);
    RA_REQUIRE(!with_scores || n_tiles64 <= (int64_t)1 << 24, RA_ERR_UNSUPPORTED, "watershed decode: max_tokens too large");
    const int n_tiles_max = (int)n_tiles64;
    const size_t tile_bytes = with_scores ? align_up(rows * n_tiles_max * sizeof(float), 256) : 0;
    const size_t p_bytes = with_scores ? scores_finish_part_bytes(1, B, Hq, layer->R_max, n_tiles_max) : 0;
    RA_REQUIRE(ws.base != nullptr && ws.bytes >= scratch_total + tile_bytes + p_bytes, RA_ERR_WORKSPACE,
               "decode: %s has %zu bytes, this call needs %zu", scratch ? "the built-in scratch" : "the workspace", ws.bytes,
               scratch_total + tile_bytes + p_bytes);

    AttnArgs a = {};
    a.view = to_dev(layer);
    a.q = q;
    a.sel_idx = sel_idx;
    a.n_sel = n_sel;
    a.cur_k = has_cur ? cur_k : nullptr;
    a.cur_v = has_cur ? cur_v : nullptr;
    a.cur_len_dev = has_cur ? cur_len : nullptr;
    a.cur_len_host = 0;
    a.cur_cap = has_cur ? cur_cap : 0;
    a.max_tokens = layer->max_tokens;
    a.q_len = 1;
    a.Hq = Hq;
    a.G = G;
    a.S = S;
    a.min_units = mfma ? kMfmaMinUnits : attn_min_units();
    a.c = scale * kLog2e;
    a.scale = scale;
    a.part_acc = mfma ? nullptr : reinterpret_cast<float*>(ws.base + w.acc_off);
    a.part_m = mfma ? nullptr : reinterpret_cast<float*>(ws.base + w.m_off);
    a.part_l = mfma ? nullptr : reinterpret_cast<float*>(ws.base + w.l_off);
    a.n_parts = reinterpret_cast<int*>(ws.base);
    a.plan = ws.base + plan_off;
    a.out = out;
    a.lse = lse;
    a.tile_lse = with_scores ? reinterpret_cast<float*>(ws.base + scratch_total) : nullptr;
    a.n_tiles_max = with_scores ? n_tiles_max : 0;
    a.rec_acc = mfma ? reinterpret_cast<float*>(ws.base + mw.rec_off) : nullptr;
    a.rec_ml = mfma ? reinterpret_cast<float*>(ws.base + mw.ml_off) : nullptr;
    a.seq_rec = reinterpret_cast<int*>(ws.base + kWsSeqRecOff);
    a.max_ranges = shape.max_ranges;
    a.range_skew = kRangeSkew;

    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const bool paged = layer->block_size != 0;
    int rc;
    if (!(mfma && attn_mfma_plans_inline(B, layer->R_max))) launch_plan(a, mfma ? 32 : kUnitTokens, st);
    {
        KernelTimer timer(ctx, st);
        if (mfma) {
            rc = launch_attn_mfma(a, paged, ctx->num_cu, st);
        } else {
            const dim3 grid(S, layer->Hkv, B);
            const size_t tab_bytes = align_up(SlotTable::bytes(layer->R_max + 1), 16);
            if (layer->dtype == RA_BF16)
                rc = dispatch_generic<BF16, 64>(paged, grid, st, a, tab_bytes);
            else
                rc = D == 128 ? dispatch_generic<F32, 128>(paged, grid, st, a, tab_bytes)
                              : dispatch_generic<F32, 64>(paged, grid, st, a, tab_bytes);
        }
    }
    if (rc) return rc;
    if (mfma) launch_merge_records(a, ctx->num_cu, st);
    else if (S > 1) launch_combine(a, D, rows, st);
    if (with_scores) {
        // With a single query token the current round cancels in the normalisation over history rounds: the
        // finishing kernel reads the history tiles only.
        FinishArgs f;
        f.part = a.tile_lse;
        f.n_rounds = layer->n_rounds;
        f.seg_len = layer->seg_len;
        f.R_max = layer->R_max;
        f.Hq = Hq;
        f.q_len = 1;
        f.cur_len = 0;
        f.n_chunks_max = n_tiles_max;
        f.chunk_tokens = 32;
        f.has_cur = false;
        f.p_out = scores_head;
        f.s_out = scores;
        launch_scores_finish(f, B, reinterpret_cast<float*>(ws.base + scratch_total + tile_bytes), st);
    }
    RA_HIP_CHECK(hipGetLastError());
    return RA_OK;
}

extern "C" int ra_round_sparse_attn_decode(ra_ctx* ctx, void* stream, const void* q, int Hq, const ra_kv_view* layer,
                                           const int32_t* sel_idx, const int32_t* n_sel, const void* cur_k,
                                           const void* cur_v, const int32_t* cur_len, int cur_cap, float scale,
                                           float* out, float* lse) {
    return decode_impl(ctx, nullptr, stream, q, Hq, layer, sel_idx, n_sel, cur_k, cur_v, cur_len, cur_cap, scale, out, lse,
                       nullptr, nullptr);
}

// ---- the same call for callers that cannot allocate ------------------------------------------------------------
// Scratch in a file-scope device array instead of a caller-provided workspace.  In host code the array's name only
// stands for the symbol: its device address is asked for once per device (every GPU holds its own copy) and that
// pointer is what kernels and entry points get.
namespace ra {
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static char* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, null until asked for

// Called by ra_create with the context's device: looks the address up the first time a device is seen.
int static_scratch_init(int device) {
    RA_REQUIRE(device >= 0 && device < kMaxDevices, RA_ERR_UNSUPPORTED, "device %d: at most %d devices", device, kMaxDevices);
    if (g_scratch_ptr[device]) return RA_OK;
    int prev = 0;
    RA_HIP_CHECK(hipGetDevice(&prev));
    RA_HIP_CHECK(hipSetDevice(device));
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    (void)hipSetDevice(prev);
    if (e != hipSuccess || ptr == nullptr)
        return fail(RA_ERR_HIP, "hipGetSymbolAddress(built-in scratch) on device %d: %s", device, hipGetErrorString(e));
    g_scratch_ptr[device] = static_cast<char*>(ptr);
    return RA_OK;
}
}  // namespace ra

extern "C" int ra_round_sparse_attn_decode_noalloc(ra_ctx* ctx, void* stream, const void* q, int Hq,
                                                   const ra_kv_view* layer, const int32_t* sel_idx, const int32_t* n_sel,
                                                   const void* cur_k, const void* cur_v, const int32_t* cur_len,
                                                   int cur_cap, float scale, float* out, float* lse) {
    RA_REQUIRE(ctx != nullptr, RA_ERR_INVALID_ARG, "decode: ctx is NULL");
    RA_REQUIRE(ctx->device >= 0 && ctx->device < kMaxDevices && g_scratch_ptr[ctx->device] != nullptr, RA_ERR_STATE,
               "decode: the built-in scratch of device %d was not set up by ra_create", ctx->device);
    const Workspace builtin = {g_scratch_ptr[ctx->device], kStaticScratchBytes};
    return decode_impl(ctx, &builtin, stream, q, Hq, layer, sel_idx, n_sel, cur_k, cur_v, cur_len, cur_cap, scale, out, lse,
                       nullptr, nullptr);
}

extern "C" int ra_watershed_attn_decode(ra_ctx* ctx, void* stream, const void* q, int Hq, const ra_kv_view* watershed,
                                        const void* cur_k, const void* cur_v, const int32_t* cur_len, int cur_cap,
                                        float scale, float* out, float* lse, float* scores_head, float* scores) {
    RA_REQUIRE(scores != nullptr, RA_ERR_INVALID_ARG, "watershed decode: scores is NULL");
    return decode_impl(ctx, nullptr, stream, q, Hq, watershed, nullptr, nullptr, cur_k, cur_v, cur_len, cur_cap, scale, out,
                       lse, scores_head, scores);
}
