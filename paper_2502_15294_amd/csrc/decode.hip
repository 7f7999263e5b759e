// Round-sparse decode attention (paper Sec. 3.2 step 5): one query token per sequence attends over
// the KV segments of the selected rounds, gathered through the round-offset index, plus the
// current round.  HBM-bandwidth bound: K and V of every selected token are read exactly once and
// serve all Hq/Hkv query heads of their KV head.
//
// Work decomposition: grid (S, Hkv, B).  A workgroup (4 wavefronts) owns KV head g of sequence b and
// the s-th of S equal shares of that sequence's 16-token units; its waves take units round-robin,
// keep an online-softmax state per 16-lane row in registers, and merge rows, then waves (LDS), into
// one partial (max, sum, d accumulators) per query head.  A sequence with a short selection is not
// split and its output is written directly; otherwise a second small kernel merges the pieces.
#include "stream_kv.hpp"

#include <stdlib.h>

namespace ra {

struct DecodeArgs {
    DevView view;
    const void* q;
    const int32_t* sel_idx;
    const int32_t* n_sel;
    const void* cur_k;
    const void* cur_v;
    const int32_t* cur_len;
    int cur_cap;
    int Hq;
    int S;
    int min_units;  // a sequence is never cut into pieces of fewer 16-token units than this
    float c;      // scale * log2(e)
    float scale;
    float* part_acc;  // [B][Hq][S][D]
    float* part_m;    // [B][Hq][S]  running max of the raw (unscaled) logits
    float* part_l;    // [B][Hq][S]  sum of 2^((logit - max) * c)
    int* n_parts;     // [B]         number of pieces sequence b was really cut into
    float* out;       // [B][Hq][D]
    float* lse;       // [B][Hq] or null
};

// A sequence is cut into at most S pieces, but never into pieces of fewer units than this: short
// selections would otherwise pay the per-workgroup set-up for a handful of tokens.
constexpr int kMinUnitsPerWorkgroup = 8;
static int min_units_per_workgroup() {
    static const int v = [] {
        const char* e = getenv("RA_DECODE_MIN_UNITS");  // tuning knob for experiments
        const int x = e ? atoi(e) : kMinUnitsPerWorkgroup;
        return x > 0 ? x : kMinUnitsPerWorkgroup;
    }();
    return v;
}

template <typename T, int D, int G, bool PAGED>
__global__ __launch_bounds__(256) void decode_kernel(DecodeArgs a) {
    constexpr int EPL = D / 16;
    using Ops = RowOps<T, EPL>;
    constexpr int WORDS = Ops::WORDS;
    constexpr int EB = Ops::ELEM_BYTES;

    extern __shared__ __align__(16) char smem[];
    const int b = blockIdx.z, g = blockIdx.y, s = blockIdx.x;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, grp = lane >> 4, sub = lane & 15;
    const DevView& vw = a.view;
    const int Hkv = vw.Hkv;

    // ---- table of segments this sequence attends over -------------------------------------
    int n_rounds = vw.n_rounds[b];
    n_rounds = min(max(n_rounds, 0), vw.R_max);
    int n_hist = a.sel_idx ? min(max(a.n_sel[b], 0), vw.R_max) : n_rounds;
    int cur_len = (a.cur_k && a.cur_len) ? min(max(a.cur_len[b], 0), a.cur_cap) : 0;
    const int n_slots = n_hist + (cur_len > 0 ? 1 : 0);
    const int cap = vw.R_max + 1;
    SlotTable tab;
    tab.carve(smem, cap);
    float* red = reinterpret_cast<float*>(smem + ((SlotTable::bytes(cap) + 15) & ~(size_t)15));

    for (int i = tid; i < n_slots; i += 256) {
        int len = 0;
        long long ok = 0, ov = 0;
        if (i < n_hist) {
            int r = a.sel_idx ? a.sel_idx[(size_t)b * vw.R_max + i] : i;
            if (r >= 0 && r < n_rounds) {
                len = max(vw.seg_len[(size_t)b * vw.R_max + r], 0);
                ok = vw.seg_off[(size_t)b * vw.R_max + r];
                ov = vw.seg_off_v[(size_t)b * vw.R_max + r];
            }
        } else {
            len = cur_len;
        }
        tab.len[i] = len;
        tab.off_k[i] = ok;
        tab.off_v[i] = ov;
        tab.cum[i] = (len + kUnitTokens - 1) / kUnitTokens;
    }
    exclusive_scan_units(tab.cum, n_slots);
    const int U = n_slots > 0 ? tab.cum[n_slots] : 0;
    const int S_eff = min(a.S, max(1, U / a.min_units));  // pieces this sequence is really cut into
    if (s >= S_eff) return;
    const int u_lo = (int)(((long long)U * s) / S_eff);
    const int u_hi = (int)(((long long)U * (s + 1)) / S_eff);

    // ---- this lane's share of the G queries ----------------------------------------------------
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

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = kNegBig;
        l[h] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[h][e] = 0.f;
    }

    const char* kbase = reinterpret_cast<const char*>(vw.k);
    const char* vbase = reinterpret_cast<const char*>(vw.v);
    const char* ck = reinterpret_cast<const char*>(a.cur_k);
    const char* cv = reinterpret_cast<const char*>(a.cur_v);

    // Addresses of the four rows (j = 0..3) this lane reads in unit u of segment `slot`.
    auto issue = [&](int u, int slot, Frag<WORDS>* kf, Frag<WORDS>* vf, int& ntok) {
        const int len = tab.len[slot];
        const int uin = u - tab.cum[slot];
        const int tok0 = uin * kUnitTokens;
        ntok = min(kUnitTokens, len - tok0);
        const char *kp, *vp;
        size_t stride;
        if (slot >= n_hist) {  // current round, token-major
            size_t e0 = (((size_t)b * a.cur_cap + tok0) * Hkv + g) * D;
            kp = ck + e0 * EB;
            vp = cv + e0 * EB;
            stride = (size_t)Hkv * D * EB;
        } else if (PAGED) {
            long long slot_idx = tab.off_k[slot] + uin;
            slot_idx = slot_idx < 0 ? 0 : (slot_idx >= vw.max_blocks ? vw.max_blocks - 1 : slot_idx);
            int blk = vw.block_table[(size_t)b * vw.max_blocks + slot_idx];
            if (blk < 0) { blk = 0; ntok = 0; }
            size_t e0 = (((size_t)blk * Hkv + g) * kUnitTokens) * D;
            kp = kbase + e0 * EB;
            vp = vbase + e0 * EB;
            stride = (size_t)D * EB;
        } else {
            kp = kbase + (((size_t)tab.off_k[slot] * Hkv + (size_t)g * len + tok0) * D) * EB;
            vp = vbase + (((size_t)tab.off_v[slot] * Hkv + (size_t)g * len + tok0) * D) * EB;
            stride = (size_t)D * EB;
        }
        const int last = max(ntok - 1, 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = min(j * 4 + grp, last);  // rows past the segment's end re-read its last row
            const size_t o = (size_t)t * stride + (size_t)sub * EPL * EB;
            kf[j] = load_frag<WORDS>(kp + o);
            vf[j] = load_frag<WORDS>(vp + o);
        }
    };

    auto consume = [&](const Frag<WORDS>* kf, const Frag<WORDS>* vf, int ntok) {
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
        float p[4][G];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float mx = fmaxf(fmaxf(sc[0][h], sc[1][h]), fmaxf(sc[2][h], sc[3][h]));
            const float m_new = fmaxf(m[h], mx);
            const float mc = m_new * a.c;
            const float alpha = fast_exp2(__builtin_fmaf(m[h], a.c, -mc));
            m[h] = m_new;
            float ps = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                p[j][h] = fast_exp2(__builtin_fmaf(sc[j][h], a.c, -mc));
                ps += p[j][h];
            }
            l[h] = __builtin_fmaf(l[h], alpha, ps);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[h][e] *= alpha;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float vfl[EPL];
            Ops::widen(vf[j].w, vfl);
#pragma unroll
            for (int h = 0; h < G; ++h)
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[h][e] = __builtin_fmaf(p[j][h], vfl[e], acc[h][e]);
        }
    };

    // ---- stream this wave's units, one unit of loads in flight ahead of the arithmetic ---------
    {
        int u = u_lo + wave;
        Frag<WORDS> kf[4], vf[4];
        int ntok = 0, slot = 0;
        bool have = u < u_hi;
        if (have) {
            slot = find_slot(tab.cum, n_slots, u);
            issue(u, slot, kf, vf, ntok);
        }
        while (have) {
            const int un = u + 4;
            const bool have_n = un < u_hi;
            Frag<WORDS> kn[4], vn[4];
            int ntok_n = 0;
            if (have_n) {
                while (un >= tab.cum[slot + 1]) ++slot;
                issue(un, slot, kn, vn, ntok_n);
            }
            consume(kf, vf, ntok);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                kf[j] = kn[j];
                vf[j] = vn[j];
            }
            ntok = ntok_n;
            u = un;
            have = have_n;
        }
    }

    // ---- merge the four 16-lane rows of the wave ------------------------------------------------
#pragma unroll
    for (int h = 0; h < G; ++h) {
        float M = fmaxf(m[h], xrow_get(m[h], 16));
        M = fmaxf(M, xrow_get(M, 32));
        const float f = fast_exp2((m[h] - M) * a.c);
        float lv = l[h] * f;
        lv += xrow_get(lv, 16);
        lv += xrow_get(lv, 32);
        l[h] = lv;
        m[h] = M;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            float x = acc[h][e] * f;
            x += xrow_get(x, 16);
            x += xrow_get(x, 32);
            acc[h][e] = x;
        }
    }
    // ---- merge the four waves through LDS ---------------------------------------------------------
    float* sm = red;               // [4][G]
    float* sl = red + 4 * G;       // [4][G]
    float* sacc = red + 8 * G;     // [4][G][D]
    if (grp == 0) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
            if (sub == 0) {
                sm[wave * G + h] = m[h];
                sl[wave * G + h] = l[h];
            }
#pragma unroll
            for (int e = 0; e < EPL; ++e) sacc[(wave * G + h) * D + sub * EPL + e] = acc[h][e];
        }
    }
    __syncthreads();
    if (s == 0 && g == 0 && tid == 0) a.n_parts[b] = S_eff;
    const size_t row0 = (size_t)b * a.Hq + (size_t)g * G;
    if (S_eff > 1) {
        for (int idx = tid; idx < G * D; idx += 256) {
            const int h = idx / D, dim = idx - h * D;
            float M = fmaxf(fmaxf(sm[h], sm[G + h]), fmaxf(sm[2 * G + h], sm[3 * G + h]));
            float num = 0.f, den = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float f = fast_exp2((sm[w * G + h] - M) * a.c);
                num = __builtin_fmaf(sacc[(w * G + h) * D + dim], f, num);
                den = __builtin_fmaf(sl[w * G + h], f, den);
            }
            const size_t slot_row = (row0 + h) * a.S + s;
            a.part_acc[slot_row * D + dim] = num;
            if (dim == 0) {
                a.part_m[slot_row] = M;
                a.part_l[slot_row] = den;
            }
        }
    } else {
        for (int idx = tid; idx < G * D; idx += 256) {
            const int h = idx / D, dim = idx - h * D;
            float M = fmaxf(fmaxf(sm[h], sm[G + h]), fmaxf(sm[2 * G + h], sm[3 * G + h]));
            float num = 0.f, den = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float f = fast_exp2((sm[w * G + h] - M) * a.c);
                num = __builtin_fmaf(sacc[(w * G + h) * D + dim], f, num);
                den = __builtin_fmaf(sl[w * G + h], f, den);
            }
            a.out[(row0 + h) * D + dim] = den > 0.f ? num / den : 0.f;
            if (a.lse && dim == 0)
                a.lse[row0 + h] = den > 0.f ? __builtin_fmaf(M, a.scale, __builtin_logf(den)) : -__builtin_inff();
        }
    }
}

// Merge the pieces of every (sequence, query head) row that was split; grid (B * Hq), block D.
template <int D>
__global__ __launch_bounds__(D) void combine_kernel(const float* part_acc, const float* part_m, const float* part_l,
                                                   const int* n_parts, int S, int Hq, float c, float scale,
                                                   float* out, float* lse) {
    const size_t row = blockIdx.x;
    const int n = n_parts[row / Hq];
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
        float a0 = pa[(size_t)p * D], a1 = pa[(size_t)(p + 1) * D], a2 = pa[(size_t)(p + 2) * D], a3 = pa[(size_t)(p + 3) * D];
        float f0 = fast_exp2((pm[p] - M) * c), f1 = fast_exp2((pm[p + 1] - M) * c);
        float f2 = fast_exp2((pm[p + 2] - M) * c), f3 = fast_exp2((pm[p + 3] - M) * c);
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

template <typename T, int D, int G>
static int launch_decode(bool paged, dim3 grid, size_t smem, hipStream_t st, const DecodeArgs& a) {
    if (paged)
        hipLaunchKernelGGL((decode_kernel<T, D, G, true>), grid, dim3(256), smem, st, a);
    else
        hipLaunchKernelGGL((decode_kernel<T, D, G, false>), grid, dim3(256), smem, st, a);
    return RA_OK;
}

template <typename T, int D>
static int dispatch_g(int G, bool paged, dim3 grid, size_t smem_of_g_times_d, hipStream_t st, const DecodeArgs& a,
                      size_t tab_bytes) {
    auto smem = [&](int g) { return tab_bytes + (size_t)(8 * g + 4 * g * D) * sizeof(float); };
    (void)smem_of_g_times_d;
    switch (G) {
        case 1: return launch_decode<T, D, 1>(paged, grid, smem(1), st, a);
        case 2: return launch_decode<T, D, 2>(paged, grid, smem(2), st, a);
        case 4: return launch_decode<T, D, 4>(paged, grid, smem(4), st, a);
        case 8: return launch_decode<T, D, 8>(paged, grid, smem(8), st, a);
        default: return fail(RA_ERR_UNSUPPORTED, "decode: Hq / Hkv = %d not in {1, 2, 4, 8}", G);
    }
}

}  // namespace ra

using namespace ra;

extern "C" int ra_round_sparse_attn_decode(ra_ctx* ctx, void* stream, const void* q, int Hq, const ra_kv_view* layer,
                                           const int32_t* sel_idx, const int32_t* n_sel, const void* cur_k,
                                           const void* cur_v, const int32_t* cur_len, int cur_cap, float scale,
                                           float* out, float* lse) {
    RA_REQUIRE(ctx != nullptr, RA_ERR_INVALID_ARG, "decode: ctx is NULL");
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

    int64_t max_tok = layer->max_tokens + (has_cur ? cur_cap : 0);
    const int S = decode_splits(ctx->num_cu, B, layer->Hkv, max_tok);
    const size_t rows = (size_t)B * Hq;
    RA_REQUIRE((size_t)B * sizeof(int) <= kWsReserved, RA_ERR_UNSUPPORTED, "decode: B = %d exceeds %zu", B,
               kWsReserved / sizeof(int));
    const size_t need = kWsReserved + align_up(rows * S * D * sizeof(float), 256) +
                        2 * align_up(rows * S * sizeof(float), 256);
    RA_REQUIRE(ctx->ws.base != nullptr && ctx->ws.bytes >= need, RA_ERR_WORKSPACE,
               "decode: workspace has %zu bytes, this call needs %zu", ctx->ws.bytes, need);

    DecodeArgs a;
    a.view = to_dev(layer);
    a.q = q;
    a.sel_idx = sel_idx;
    a.n_sel = n_sel;
    a.cur_k = has_cur ? cur_k : nullptr;
    a.cur_v = has_cur ? cur_v : nullptr;
    a.cur_len = has_cur ? cur_len : nullptr;
    a.cur_cap = has_cur ? cur_cap : 0;
    a.Hq = Hq;
    a.S = S;
    a.min_units = min_units_per_workgroup();
    a.c = scale * kLog2e;
    a.scale = scale;
    a.out = out;
    a.lse = lse;
    a.n_parts = reinterpret_cast<int*>(ctx->ws.base);
    a.part_acc = reinterpret_cast<float*>(ctx->ws.base + kWsReserved);
    a.part_m = reinterpret_cast<float*>(ctx->ws.base + kWsReserved + align_up(rows * S * D * sizeof(float), 256));
    a.part_l = reinterpret_cast<float*>(reinterpret_cast<char*>(a.part_m) + align_up(rows * S * sizeof(float), 256));

    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const dim3 grid(S, layer->Hkv, B);
    const size_t tab_bytes = align_up(SlotTable::bytes(layer->R_max + 1), 16);
    const bool paged = layer->block_size != 0;
    int rc;
    if (layer->dtype == RA_BF16) {
        rc = D == 128 ? dispatch_g<BF16, 128>(G, paged, grid, 0, st, a, tab_bytes)
                      : dispatch_g<BF16, 64>(G, paged, grid, 0, st, a, tab_bytes);
    } else {
        rc = D == 128 ? dispatch_g<F32, 128>(G, paged, grid, 0, st, a, tab_bytes)
                      : dispatch_g<F32, 64>(G, paged, grid, 0, st, a, tab_bytes);
    }
    if (rc) return rc;
    if (S > 1) {
        if (D == 128)
            hipLaunchKernelGGL((combine_kernel<128>), dim3((unsigned)rows), dim3(128), 0, st, a.part_acc, a.part_m,
                               a.part_l, a.n_parts, S, Hq, a.c, scale, out, lse);
        else
            hipLaunchKernelGGL((combine_kernel<64>), dim3((unsigned)rows), dim3(64), 0, st, a.part_acc, a.part_m,
                               a.part_l, a.n_parts, S, Hq, a.c, scale, out, lse);
    }
    RA_HIP_CHECK(hipGetLastError());
    return RA_OK;
}
