// Argument block and launch interface shared by the round-sparse attention kernels
// (decode and question prefill; generic vector-ALU path and bf16 matrix-core path).
#pragma once

#include "common.hpp"

namespace ra {

// Share of the batch's key tiles that the first half of the decode kernel's ranges gets beyond one half, in
// 1/1000 (RangeCut in range_schedule.hpp).  It is 0: the launch puts one workgroup on every compute unit, one wave on
// every SIMD, and all waves stream at the same rate.  The two-class cut dates from the launch with two workgroups per
// unit, whose second workgroup's waves shared their SIMD with an older wave that the hardware served first (0.27
// against 0.20 tiles per microsecond for the whole kernel): while all loads were ordinary ones a skew of 90 took the
// kernel from 217 to 212 microseconds on the large paged workload at 13.9 % kept (0: 217.0-217.9, 20: 215.7,
// 40: 215.4-216.0, 60: 213.2, 80: 211.4, 100: 212.4, 140: 216.6, 180: 217.7, 220: 220.6); behind the non-temporal
// value loads it no longer mattered (0: 199.1, 50: 199.8, 90: 198.6-201.0, 130: 200.7), since the first wave of a
// SIMD got its 0.27 whatever the other one got, and a skew only moved time between the two phases.  The cut stays
// available for a part or a launch shape that serves its waves unevenly.
constexpr int kRangeSkew = 0;

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
    // matrix-core kernel for up to 32 query rows per KV head (range schedule, see range_schedule.hpp): partial
    // results of the sequences that lie in several ranges
    float* rec_acc;   // [records][inner][16][D]   inner = Hkv * row blocks
    float* rec_ml;    // [records][inner][16][2]   running max of the raw logits, sum of 2^((logit - max) * c)
    int* seq_rec;     // [B][2] first record and number of records of every sequence (written by the kernel)
    int max_ranges;   // most ranges the batch's key tiles are cut into
    int range_skew;   // in 1/1000: how much more than half of the tiles the first half of the ranges gets (see RangeCut)
    int p_half;       // many-row kernel: probabilities as one fp16 operand instead of two bf16 (ra_set_prefill_precision)
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

// bf16, d = 128, Hq/Hkv <= 16, up to 32 query rows per KV head (decode, short questions): matrix-core streaming
// kernel, one wavefront per (range of the batch's key tiles, KV head, block of 16 query rows).
int launch_attn_mfma(const AttnArgs& a, bool paged, int num_cu, hipStream_t st);
void launch_merge_records(const AttnArgs& a, int num_cu, hipStream_t st);  // ... and its second step
// Same operands, many query rows per KV head: the waves own different rows and share key tiles through LDS.
int launch_attn_prefill_mfma(const AttnArgs& a, bool paged, int num_cu, hipStream_t st);
// Small batches: the first kernel resolves the selection itself (every workgroup reads the whole batch's segment
// lists in one memory round trip and keeps them in LDS), so that no planning kernel runs before it.
inline size_t attn_mfma_inline_bytes(int B, int R_max) {
    return (size_t)B * R_max * 24 + (size_t)B * (R_max + 2) * 4 + (size_t)B * 16 + 16;
}
inline bool attn_mfma_plans_inline(int B, int R_max) {
    return B <= 64 && (long long)B * R_max <= 1024;  // at most 29 KB of LDS beside the 17 KB of score staging
}
// Launch shape and scratch of that kernel.  `max_tiles` bounds the 32-token key tiles of the whole batch.
constexpr int kMfmaMinUnits = 4;  // shortest range in key tiles (two tiles are in flight per wave; ranges of 2 and of 8 measured no better)
struct MfmaDecodeShape {
    int n_rowblocks, inner, grid, max_ranges, records;
    size_t rec_bytes, ml_bytes;
};
inline MfmaDecodeShape mfma_decode_shape(int num_cu, int B, int R_max, int Hkv, int rows_total, long long max_tiles) {
    MfmaDecodeShape s;
    s.n_rowblocks = (rows_total + 15) / 16;
    s.inner = Hkv * s.n_rowblocks;
    long long want = max_tiles / kMfmaMinUnits;  // ranges the batch can have at most
    if (want < 1) want = 1;
    long long grid = (want * s.inner + 3) / 4;   // four waves per workgroup, at least one work item per wave
    // One workgroup per compute unit, i.e. one wave per SIMD.  With two, the hardware serves the older wave of a
    // SIMD first: the second workgroup's waves stream at three quarters of the first's rate for the whole kernel
    // and finish a quarter later, while the sum stays what the memory system gives.  Alone on its SIMD every wave
    // runs at the same rate, and there are half as many records to merge (headline decode kernel 198.7 -> 194.6
    // microseconds, 85.1 -> 82.8 at 6 % of the tokens kept, 415.8 -> 410.4 per layer of the long-context workload).
    const long long full = num_cu > 512 ? 512 : num_cu;
    if (grid > full) grid = full;
    if (grid < 1) grid = 1;
    s.grid = (int)grid;
    long long ranges = grid * 4 / s.inner;  // one range per wave
    if (ranges > want) ranges = want;
    s.max_ranges = (int)(ranges < 1 ? 1 : ranges);
    s.records = s.max_ranges + B;
    s.rec_bytes = align_up((size_t)s.records * s.inner * 16 * 128 * sizeof(float), 256);
    s.ml_bytes = align_up((size_t)s.records * s.inner * 16 * 2 * sizeof(float), 256);
    return s;
}
// Bound of the 32-token tiles of a batch: every round and the current round may end with a partial tile.
inline long long mfma_max_tiles(int B, long long max_tokens, int R_max, int cur_cap) {
    return (long long)B * (max_tokens / 32 + R_max + cur_cap / 32 + 1);
}
struct MfmaDecodeWorkspace {
    size_t plan_off, rec_off, ml_off, total;
};
inline MfmaDecodeWorkspace mfma_decode_workspace(const MfmaDecodeShape& s, int B, int R_max) {
    MfmaDecodeWorkspace w;
    w.plan_off = kWsReserved;
    w.rec_off = w.plan_off + align_up(attn_plan_bytes(B, R_max), 256);
    w.ml_off = w.rec_off + s.rec_bytes;
    w.total = w.ml_off + s.ml_bytes;
    return w;
}
// Most pieces one sequence can be cut into by the many-row kernel (row length of its piece buffers).
inline int mfma_max_pieces(int64_t max_tokens, int min_units, int cap) {
    int64_t s = max_tokens / (32 * (int64_t)min_units);
    return (int)(s < 1 ? 1 : (s > cap ? cap : s));
}
// Merge of the split pieces; launched by the entry points when S > 1.
void launch_combine(const AttnArgs& a, int D, size_t rows, hipStream_t st);

}  // namespace ra
