// Argument block and launch interface shared by the round-sparse attention kernels
// (decode and question prefill; generic vector-ALU path and bf16 matrix-core path).
#pragma once

#include "common.hpp"

namespace ra {

struct AttnArgs {
    DevView view;
    const void* q;             // [B][q_len][Hq][D]
    const int32_t* sel_idx;    // [B][R_max] or null (= every round of the view)
    const int32_t* n_sel;      // [B] or null
    const void* cur_k;         // [B][cur_cap][Hkv][D] token-major, or null
    const void* cur_v;
    const int32_t* cur_len_dev;  // [B] per-sequence length of the current round, or null
    int cur_len_host;            // used when cur_len_dev is null
    int cur_cap;
    long long max_tokens;        // host-known bound on a sequence's history tokens (sizes the launch only)
    int q_len, Hq, G;
    int S;          // upper bound of the pieces a sequence's key set is cut into
    int min_units;  // a sequence is never cut into pieces of fewer work units than this
    float c;        // scale * log2(e)
    float scale;
    float* part_acc;  // [rows][S][D]   rows = B * q_len * Hq, row = (b * q_len + i) * Hq + h
    float* part_m;    // [rows][S]      running max of the raw (unscaled) logits
    float* part_l;    // [rows][S]      sum of 2^((logit - max) * c)
    int* n_parts;     // [B]            pieces sequence b was really cut into
    char* plan;       // [B][plan_stride(R_max + 1)] per-sequence segment tables (see stream_kv.hpp)
    float* out;       // [rows][D]
    float* lse;       // [rows] or null
    // at the watershed layer only: natural-log sum-exp of the scaled logits of every score unit of a sequence's
    // table (history rounds in order, then the current round), [rows][n_tiles_max]; the unit is a 32-token key
    // tile in the 16-row kernel and a 256-token chunk of a round in the many-row kernel; null otherwise
    float* tile_lse;
    int n_tiles_max;
};

// Workspace layout of one attention call; returns the bytes needed past the reserved head.
struct AttnWorkspace {
    size_t plan_off, acc_off, m_off, l_off, total;
};
size_t attn_plan_bytes(int B, int R_max);
inline AttnWorkspace attn_workspace(size_t rows, int S, int D, int B, int R_max) {
    AttnWorkspace w;
    w.plan_off = kWsReserved;
    w.acc_off = w.plan_off + align_up(attn_plan_bytes(B, R_max), 256);
    w.m_off = w.acc_off + align_up(rows * S * D * sizeof(float), 256);
    w.l_off = w.m_off + align_up(rows * S * sizeof(float), 256);
    w.total = w.l_off + align_up(rows * S * sizeof(float), 256);
    return w;
}

// Builds the per-sequence segment tables for work units of `unit_tokens` tokens (grid B).
void launch_plan(const AttnArgs& a, int unit_tokens, hipStream_t st);
int attn_min_units();  // smallest piece of a sequence's key set, in 32-token tiles

// bf16, d = 128, Hq/Hkv <= 16: matrix-core streaming kernel, the waves of a workgroup split the key tiles
// of 16 query rows (decode, short questions).
int launch_attn_mfma(const AttnArgs& a, bool paged, int num_cu, hipStream_t st);
// Same operands, many query rows per KV head: the waves own different rows and share key tiles through LDS.
int launch_attn_prefill_mfma(const AttnArgs& a, bool paged, int num_cu, hipStream_t st);
// Small batches: the 16-row matrix-core kernel resolves the selection itself (every workgroup reads the whole
// batch's segment lists in one memory round trip and builds its sequences' tables in LDS), so that no planning
// kernel runs before it.
inline size_t attn_mfma_inline_bytes(int B, int R_max) { return (size_t)B * R_max * 24 + (size_t)B * 12 + 16; }
inline bool attn_mfma_plans_inline(int B, int R_max) {
    // ... as long as the lists, the workgroup's own table (24 bytes per segment) and the 33 KB merge buffer stay
    // within 64 KB of LDS, so that two workgroups still fit a compute unit
    return B <= 64 && (long long)B * R_max <= 1024 &&
           attn_mfma_inline_bytes(B, R_max) + (size_t)(R_max + 1) * 24 + 64 + 33280 <= 64 * 1024;
}
// Most pieces one sequence can be cut into by the matrix-core kernel (row length of the piece buffers).
inline int mfma_max_pieces(int64_t max_tokens, int min_units, int cap) {
    int64_t s = max_tokens / (32 * (int64_t)min_units);
    return (int)(s < 1 ? 1 : (s > cap ? cap : s));
}
// Merge of the split pieces; launched by the entry points when S > 1.
void launch_combine(const AttnArgs& a, int D, size_t rows, hipStream_t st);

}  // namespace ra
