// Round-sparse question-prefill attention (paper Sec. 3.2 step 4): the q_len tokens of the current
// question attend over the selected rounds' KV (fully visible) and, causally, over the question's own
// KV.  Entry point only; the arithmetic is in the matrix-core kernels.
#include "attn_common.hpp"
#include "scores_common.hpp"

using namespace ra;

// Shared by the two prefill entry points.  With `scores` given (watershed layer) the attention runs over every
// history round and the kernel also leaves one log-sum-exp per (query row, score unit: a 32-token key tile in the
// 16-row kernel, a 256-token chunk of a round in the many-row kernel), which the finishing kernels of the score
// pass turn into Eq. 1.
static int prefill_impl(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq, const ra_kv_view* layer,
                        const int32_t* sel_idx, const int32_t* n_sel, const void* cur_k, const void* cur_v, int cur_len,
                        float scale, float* out, float* lse, float* scores_head, float* scores) {
    RA_REQUIRE(ctx != nullptr, RA_ERR_INVALID_ARG, "prefill: ctx is NULL");
    RA_REQUIRE(q != nullptr && out != nullptr, RA_ERR_INVALID_ARG, "prefill: q or out is NULL");
    if (int rc = check_view(layer, true, "prefill")) return rc;
    RA_REQUIRE(q_len > 0, RA_ERR_INVALID_ARG, "prefill: q_len must be positive");
    RA_REQUIRE(Hq > 0 && Hq % layer->Hkv == 0, RA_ERR_INVALID_ARG, "prefill: Hq %d is not a multiple of Hkv %d", Hq,
               layer->Hkv);
    RA_REQUIRE((sel_idx == nullptr) == (n_sel == nullptr), RA_ERR_INVALID_ARG,
               "prefill: sel_idx and n_sel must both be given or both be NULL");
    RA_REQUIRE(cur_len >= 0 && (cur_k != nullptr) == (cur_len > 0) && (cur_v != nullptr) == (cur_len > 0),
               RA_ERR_INVALID_ARG, "prefill: cur_k, cur_v and cur_len > 0 must be given together");
    RA_REQUIRE(cur_len == 0 || cur_len >= q_len, RA_ERR_INVALID_ARG,
               "prefill: the q_len query tokens are the tail of the current round, so cur_len >= q_len");
    RA_REQUIRE(layer->R_max > 0 || cur_len > 0, RA_ERR_INVALID_ARG,
               "prefill: no history rounds and no current round: the key set is empty");
    RA_REQUIRE(scale > 0.f && scale == scale, RA_ERR_INVALID_ARG, "prefill: scale must be positive");
    RA_REQUIRE(layer->dtype == RA_BF16 && layer->d == 128, RA_ERR_UNSUPPORTED,
               "prefill: only bf16 with head_dim 128 is implemented");
    const int G = Hq / layer->Hkv, B = layer->B, D = 128;
    RA_REQUIRE(G <= 16, RA_ERR_UNSUPPORTED, "prefill: Hq / Hkv = %d exceeds 16", G);
    RA_REQUIRE(B <= kMaxBatch, RA_ERR_UNSUPPORTED, "prefill: batch %d exceeds %d", B, kMaxBatch);

    // Few query rows per KV head: the decode kernel (one wave per range of key tiles and block of 16 rows);
    // otherwise the kernel whose waves own different rows and share each key tile through LDS.
    const bool few_rows = q_len * G <= 32;
    const size_t rows = (size_t)B * q_len * Hq;
    MfmaDecodeShape shape = {};
    MfmaDecodeWorkspace mw = {};
    AttnWorkspace w = {};
    int S = 1;
    size_t plan_off, scratch_total;
    if (few_rows) {
        const long long max_tiles = mfma_max_tiles(B, layer->max_tokens, layer->R_max, cur_len);
        RA_REQUIRE(max_tiles < ((long long)1 << 30), RA_ERR_UNSUPPORTED, "prefill: max_tokens too large for this batch");
        shape = mfma_decode_shape(ctx->num_cu, B, layer->R_max, layer->Hkv, q_len * G, max_tiles);
        mw = mfma_decode_workspace(shape, B, layer->R_max);
        plan_off = mw.plan_off;
        scratch_total = mw.total;
    } else {
        S = mfma_max_pieces(layer->max_tokens + cur_len, attn_min_units(), 8);
        w = attn_workspace(rows, S, D, B, layer->R_max);
        plan_off = w.plan_off;
        scratch_total = w.total;
    }
    const bool with_scores = scores != nullptr;
    RA_REQUIRE(!with_scores || layer->R_max > 0, RA_ERR_INVALID_ARG, "watershed prefill: R_max is 0, there is nothing to score");
    // score output: one entry per 32-token tile (decode kernel) or per 256-token chunk (many-row kernel) of a
    // sequence's table: history rounds (each rounded up), then the current round
    const int score_unit = few_rows ? 32 : 256;
    const int64_t n_tiles64 = layer->max_tokens / score_unit + layer->R_max + cur_len / score_unit + 1;
    RA_REQUIRE(!with_scores || n_tiles64 <= (int64_t)1 << 24, RA_ERR_UNSUPPORTED, "watershed prefill: max_tokens too large");
    const int n_tiles_max = (int)n_tiles64;
    const size_t tile_bytes = with_scores ? align_up(rows * n_tiles_max * sizeof(float), 256) : 0;
    const size_t p_bytes = with_scores ? scores_finish_part_bytes(q_len, B, Hq, layer->R_max, n_tiles_max) : 0;
    RA_REQUIRE(ctx->ws.base != nullptr && ctx->ws.bytes >= scratch_total + tile_bytes + p_bytes, RA_ERR_WORKSPACE,
               "prefill: workspace has %zu bytes, this call needs %zu", ctx->ws.bytes, scratch_total + tile_bytes + p_bytes);

    AttnArgs a = {};
    a.view = to_dev(layer);
    a.q = q;
    a.sel_idx = sel_idx;
    a.n_sel = n_sel;
    a.cur_k = cur_len ? cur_k : nullptr;
    a.cur_v = cur_len ? cur_v : nullptr;
    a.cur_len_dev = nullptr;
    a.cur_len_host = cur_len;
    a.cur_cap = cur_len;
    a.max_tokens = layer->max_tokens;
    a.q_len = q_len;
    a.Hq = Hq;
    a.G = G;
    a.S = S;
    a.min_units = few_rows ? kMfmaMinUnits : attn_min_units();
    a.c = scale * kLog2e;
    a.scale = scale;
    a.part_acc = few_rows ? nullptr : reinterpret_cast<float*>(ctx->ws.base + w.acc_off);
    a.part_m = few_rows ? nullptr : reinterpret_cast<float*>(ctx->ws.base + w.m_off);
    a.part_l = few_rows ? nullptr : reinterpret_cast<float*>(ctx->ws.base + w.l_off);
    a.n_parts = reinterpret_cast<int*>(ctx->ws.base);
    a.plan = ctx->ws.base + plan_off;
    a.out = out;
    a.lse = lse;
    a.tile_lse = with_scores ? reinterpret_cast<float*>(ctx->ws.base + scratch_total) : nullptr;
    a.n_tiles_max = with_scores ? n_tiles_max : 0;
    a.rec_acc = few_rows ? reinterpret_cast<float*>(ctx->ws.base + mw.rec_off) : nullptr;
    a.rec_ml = few_rows ? reinterpret_cast<float*>(ctx->ws.base + mw.ml_off) : nullptr;
    a.seq_rec = reinterpret_cast<int*>(ctx->ws.base + kWsSeqRecOff);
    a.max_ranges = shape.max_ranges;
    a.range_skew = kRangeSkew;
    a.p_half = with_scores ? 0 : ctx->prefill_p_half;  // the watershed call's scores decide the selection: full precision
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!(few_rows && attn_mfma_plans_inline(B, layer->R_max))) launch_plan(a, 32, st);
    {
        KernelTimer timer(ctx, st);
        if (int rc = few_rows ? launch_attn_mfma(a, layer->block_size != 0, ctx->num_cu, st)
                              : launch_attn_prefill_mfma(a, layer->block_size != 0, ctx->num_cu, st))
            return rc;
    }
    if (few_rows) launch_merge_records(a, ctx->num_cu, st);
    else if (S > 1) launch_combine(a, D, rows, st);
    if (with_scores) {
        // Eq. 1 over history rounds and, for several query tokens, the visible part of the question itself
        // (with one query token the current round cancels in the normalisation over history rounds).
        FinishArgs f;
        f.part = a.tile_lse;
        f.n_rounds = layer->n_rounds;
        f.seg_len = layer->seg_len;
        f.R_max = layer->R_max;
        f.Hq = Hq;
        f.q_len = q_len;
        f.has_cur = cur_len > 0 && q_len > 1;
        f.cur_len = f.has_cur ? cur_len : 0;
        f.n_chunks_max = n_tiles_max;
        f.chunk_tokens = score_unit;
        f.p_out = scores_head;
        f.s_out = scores;
        launch_scores_finish(f, B, reinterpret_cast<float*>(ctx->ws.base + scratch_total + tile_bytes), st);
    }
    RA_HIP_CHECK(hipGetLastError());
    return RA_OK;
}

extern "C" int ra_round_sparse_attn_prefill(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq,
                                            const ra_kv_view* layer, const int32_t* sel_idx, const int32_t* n_sel,
                                            const void* cur_k, const void* cur_v, int cur_len, float scale, float* out,
                                            float* lse) {
    return prefill_impl(ctx, stream, q, q_len, Hq, layer, sel_idx, n_sel, cur_k, cur_v, cur_len, scale, out, lse, nullptr,
                        nullptr);
}

extern "C" int ra_watershed_attn_prefill(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq,
                                         const ra_kv_view* watershed, const void* cur_k, const void* cur_v, int cur_len,
                                         float scale, float* out, float* lse, float* scores_head, float* scores) {
    RA_REQUIRE(scores != nullptr, RA_ERR_INVALID_ARG, "watershed prefill: scores is NULL");
    return prefill_impl(ctx, stream, q, q_len, Hq, watershed, nullptr, nullptr, cur_k, cur_v, cur_len, scale, out, lse,
                        scores_head, scores);
}

extern "C" int ra_set_prefill_precision(ra_ctx* ctx, int mode) {
    RA_REQUIRE(ctx != nullptr, RA_ERR_INVALID_ARG, "ra_set_prefill_precision: ctx is NULL");
    RA_REQUIRE(mode == RA_PREFILL_P_BF16X2 || mode == RA_PREFILL_P_F16, RA_ERR_INVALID_ARG,
               "ra_set_prefill_precision: unknown mode %d", mode);
    ctx->prefill_p_half = mode == RA_PREFILL_P_F16;
    return RA_OK;
}
