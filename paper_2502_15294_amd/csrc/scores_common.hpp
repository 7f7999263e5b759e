// Argument block shared by the round-score streaming kernels.
#pragma once

#include "common.hpp"

namespace ra {

constexpr int kChunkUnits = 16;                          // units per chunk
constexpr int kChunkTokens = kChunkUnits * kUnitTokens;  // 256: chunk of the workgroup-per-chunk kernels

struct ScoreArgs {
    DevView view;
    const void* q;      // [B][q_len][Hq][D]
    const void* cur_k;  // [B][cur_len][Hkv][D] or null
    int cur_len, q_len, Hq;
    int n_chunks_max;   // row length of `part`
    int chunk_tokens;   // tokens per chunk (a chunk never crosses a round)
    float c;            // scale * log2(e)
    float* part;        // [B][Hq][q_len][n_chunks_max] natural-log sum-exp of the scaled logits of one chunk
    void* chunks = nullptr;  // few-row kernel only: room for [B][n_chunks_max] 16-byte chunk descriptors, or null
    // many-row kernel only: room for its segment tables and the bounds of its schedule
    const char* plan;   // [B][plan_stride(R_max + 1)]
    int S, min_units;   // a sequence is cut into at most S pieces of at least min_units key tiles
};

// Input of the finishing kernels: per-chunk log-sum-exps -> Eq. 1.
struct FinishArgs {
    const float* part;         // [B][Hq][q_len][n_chunks_max]
    const int32_t* n_rounds;
    const int32_t* seg_len;
    int R_max, Hq, q_len, cur_len, n_chunks_max, chunk_tokens;
    bool has_cur;
    float* p_out;  // may be null
    float* s_out;
    float* acc = nullptr;  // [B][Hq][R_max] running round masses of earlier calls (Eq. 1 over a growing set of
                           // query tokens): added to this call's masses before normalising, then updated
    // Sec. 3.3 in the same kernel: the workgroup that has a sequence's scores in LDS also selects its rounds
    bool with_select = false;
    ra_select_params sel = {};
    int32_t* sel_idx = nullptr;  // [B][R_max]
    int32_t* n_sel = nullptr;    // [B]
};
void launch_scores_finish_single(const FinishArgs& f, int B, hipStream_t st);
int scores_finish_splits(int q_len, int B, int Hq);  // Z of launch_scores_finish_rows
void launch_scores_finish_rows(const FinishArgs& f, int B, float* p_part, int Z, hipStream_t st);
// Whether the finishing pass runs as one workgroup per (sequence, head, split) plus a head-mean kernel (several
// query tokens, or one token whose heads have many partial values to fold) rather than one workgroup per sequence.
inline bool scores_finish_by_rows(int q_len, int Hq, int n_chunks_max) {
    return q_len > 1 || (int64_t)Hq * n_chunks_max >= 16384;
}
// Bytes of the partial round masses the by-rows pass needs ([B][Hq][Z][R_max] floats), 0 for the other pass.
inline size_t scores_finish_part_bytes(int q_len, int B, int Hq, int R_max, int n_chunks_max) {
    if (!scores_finish_by_rows(q_len, Hq, n_chunks_max)) return 0;
    return ((size_t)B * Hq * scores_finish_splits(q_len, B, Hq) * R_max * sizeof(float) + 255) & ~(size_t)255;
}
// Picks the pass; p_part must hold scores_finish_part_bytes() bytes when that is not 0.
void launch_scores_finish(const FinishArgs& f, int B, float* p_part, hipStream_t st);

__device__ __forceinline__ int chunks_of(int len, int chunk_tokens = kChunkTokens) {
    return (len + chunk_tokens - 1) / chunk_tokens;
}
// Tokens of the current round visible to query token i (causal, aligned to the round's end).
__device__ __forceinline__ int cur_visible(int cur_len, int q_len, int i) {
    return min(max(cur_len - q_len + i + 1, 0), cur_len);
}

// bf16, d = 128, Hq/Hkv <= 16: matrix-core streaming kernels, for up to 16 query rows per KV head and for more.
void launch_scores_plan(const ScoreArgs& a, hipStream_t st);  // segment tables of the many-row kernel; run it first
int launch_scores_prefill_mfma(const ScoreArgs& a, bool paged, int num_cu, hipStream_t st);
int launch_scores_mfma(const ScoreArgs& a, bool paged, int num_cu, hipStream_t st);

}  // namespace ra
