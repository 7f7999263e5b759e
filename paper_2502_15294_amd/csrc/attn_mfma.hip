// Round-sparse attention over the selected rounds, bf16 / head_dim 128, on the matrix cores
// (paper Sec. 3.2 steps 4 and 5: question prefill and decode after the watershed layer).
//
// This kernel serves decode and short questions; long questions use the kernel that shares key tiles
// through LDS.  The "query rows" of a KV head g are the pairs (query token i, head h of the group),
// row = i * G + h: G rows for decode, q_len * G in general; they are handled in blocks of 16 rows.
// Keys/values are streamed in tiles of 32 tokens that never cross a round:
//
//   S^T tile  [16 tokens x 16 rows]  = K[16 x 128] . Q^T[128 x 16]        4 x mfma 16x16x32 per 16 tokens
//   O^T tile  [16 channels x 16 rows] += V^T[16 x 32 tokens] . P[32 x 16]  8 x mfma 16x16x32 (x2: P = hi + lo)
//
// With D = A.B the instruction puts D[4*(lane/16)+i][lane%16] in lane's register i, and takes from
// lane the 8 contraction entries k = 8*(lane/16) .. +7 of row/column lane%16.  Choosing the roles
// as above, lane%16 is the query row everywhere: a lane's S registers are 4+4 tokens of its row, they
// become its P operand as they are (the V^T operand is loaded with the matching token order), and its
// O^T registers are channels of the same row, so the running max / sum / rescale of the online softmax
// never leave the lane except for one max over the four lane groups.  Values are stored transposed in
// 16-token tiles so that the V^T operand is a plain 8-byte load per lane.
//
// P is rounded to bf16 twice (P = hi + lo, both bf16) so that the product carries ~16 bits of P.
//
// Work decomposition (range_schedule.hpp): the key tiles of the whole batch are cut into equal ranges, and ONE
// WAVEFRONT streams one range for one (KV head, block of 16 query rows), two tiles in flight, everything it
// needs in its own registers.  After the prologue, in which a workgroup derives the batch's tile prefix (and,
// for small batches, resolves the selections itself), the waves never meet again: there is no barrier and no
// shared buffer in the streaming loop, and no wave ever waits for another.  A sequence that lies in one range is
// written out directly; otherwise each of its segments leaves a partial result ("record") and a second, small
// kernel merges the records of every sequence that was cut.
#include "attn_common.hpp"
#include "mfma_util.hpp"
#include "range_schedule.hpp"

namespace ra {

constexpr int kTile = 32;  // tokens per key tile (two 16-token halves)
constexpr int D128 = 128;
constexpr int kLsePitch = 65;  // floats per row of a wave's strip of staged tile log-sum-exps

struct KVTile {
    uint4 k[2][4];  // [half][kk]: 8 channels kk*32 + 8*(lane/16) .. of token half*16 + lane%16
    uint2 v[8][2];  // [dt][half]: tokens 4*(lane/16) .. +3 of that half, channel dt*16 + lane%16
};

// Where a key tile lies; every field is the same in all lanes of the wave.
struct TileRef {
    int len;           // tokens of the segment (round) the tile belongs to
    int uin;           // index of the tile inside its segment
    int u_seq;         // index of the tile inside the sequence's table
    bool is_cur;       // the segment is the current round (token-major keys and values)
    long long ok, ov;  // start of the segment's keys / values (tokens, or block-table slots when paged)
    int pb0, pb1;      // paged history: physical blocks of the tile's two 16-token halves
};

__device__ __forceinline__ int lane_get(int v, int l) { return __builtin_amdgcn_readlane(v, l); }
__device__ __forceinline__ long long lane_get64(long long v, int l) {
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(unsigned long long)v, l);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)((unsigned long long)v >> 32), l);
    return (long long)(((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Exclusive prefix sum over the 64 lanes of a wave; `total` receives the sum of all lanes.
__device__ __forceinline__ int wave_exclusive_scan(int v, int lane, int& total) {
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off, 64);
        if (lane >= off) incl += t;
    }
    total = __builtin_amdgcn_readlane(incl, 63);
    return incl - v;
}

// Merge of the records (a record: the accumulators of the 16 rows of a block, row-major [16][128], and (max, sum)
// per row) of every (sequence, KV head, row block) that was cut; grid (B * inner), block 256.
// Thread = (group, row, four channels): the rows of the block (at most eight per pass) times 32 channel quads fill
// 32 .. 256 threads, and when they fill fewer the remaining threads form further groups that take every NG-th
// record; the groups are then merged through LDS.  Four records per thread are in flight at a time.
__global__ __launch_bounds__(256) void merge_records_kernel(AttnArgs a, int n_rowblocks) {
    __shared__ float sh_num[8][8][D128];  // [group][row][channel]
    __shared__ float sh_ml[8][8][2];
    const int Hkv = a.view.Hkv, inner = Hkv * n_rowblocks;
    const int b = blockIdx.x / inner, gi = blockIdx.x - b * inner;
    const int g = gi % Hkv, rowblock = gi / Hkv;
    const int rec0 = a.seq_rec[2 * b], n_parts = a.seq_rec[2 * b + 1];
    if (n_parts <= 1) return;  // written directly by the streaming kernel (or no key at all)
    const int rows_here = min(16, a.q_len * a.G - rowblock * 16);
    const int t = threadIdx.x;
    for (int row0 = 0; row0 < rows_here; row0 += 8) {
        const int R = min(8, rows_here - row0);
        const int rp_log2 = R <= 1 ? 0 : (R <= 2 ? 1 : (R <= 4 ? 2 : 3));
        const int group_threads = 32 << rp_log2, NG = 256 >> (5 + rp_log2);
        const int grp = t >> (5 + rp_log2), tt = t & (group_threads - 1);
        const int r = tt >> 5, c4 = tt & 31;
        const bool active = r < R;
        const int row = row0 + (active ? r : 0);
        float M = kNegBig, den = 0.f;
        floatx4_t num = floatx4_t{0.f, 0.f, 0.f, 0.f};
        for (int p0 = grp; p0 < n_parts; p0 += 4 * NG) {
            floatx4_t v[4];
            float2 ml[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int p = p0 + j * NG;
                v[j] = floatx4_t{0.f, 0.f, 0.f, 0.f};
                ml[j] = make_float2(kNegBig, 0.f);
                if (p < n_parts && active) {
                    const size_t rrow = ((size_t)(rec0 + p) * inner + gi) * 16 + row;
                    v[j] = *reinterpret_cast<const floatx4_t*>(a.rec_acc + rrow * D128 + c4 * 4);
                    ml[j] = *reinterpret_cast<const float2*>(a.rec_ml + rrow * 2);
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float m_new = fmaxf(M, ml[j].x);
                const float f_old = fast_exp2((M - m_new) * a.c), f_new = fast_exp2((ml[j].x - m_new) * a.c);
                den = __builtin_fmaf(ml[j].y, f_new, den * f_old);
                num = v[j] * f_new + num * f_old;
                M = m_new;
            }
        }
        if (active) {
            *reinterpret_cast<floatx4_t*>(&sh_num[grp][r][c4 * 4]) = num;
            if (c4 == 0) {
                sh_ml[grp][r][0] = M;
                sh_ml[grp][r][1] = den;
            }
        }
        __syncthreads();
        if (grp == 0 && active) {
            float Mx = kNegBig;
            for (int k = 0; k < NG; ++k) Mx = fmaxf(Mx, sh_ml[k][r][0]);
            float d = 0.f;
            floatx4_t o = floatx4_t{0.f, 0.f, 0.f, 0.f};
            for (int k = 0; k < NG; ++k) {
                const float f = fast_exp2((sh_ml[k][r][0] - Mx) * a.c);
                d = __builtin_fmaf(sh_ml[k][r][1], f, d);
                o += *reinterpret_cast<const floatx4_t*>(&sh_num[k][r][c4 * 4]) * f;
            }
            const int rw = rowblock * 16 + row, qi = rw / a.G;
            const size_t rid = ((size_t)b * a.q_len + qi) * a.Hq + (size_t)g * a.G + (rw - qi * a.G);
            const float inv = d > 0.f ? 1.f / d : 0.f;
            *reinterpret_cast<floatx4_t*>(a.out + rid * D128 + c4 * 4) = o * inv;
            if (a.lse && c4 == 0) a.lse[rid] = d > 0.f ? __builtin_fmaf(Mx, a.scale, __builtin_logf(d)) : -__builtin_inff();
        }
        __syncthreads();  // the next pass reuses the buffers
    }
}

// TILE_LSE: also one log-sum-exp per (query row, key tile), the raw material of the round scores at the watershed
// layer; staged per wave in LDS and written out in runs of up to 64 tiles per row.
// INLINE_PLAN: the workgroup resolves the batch's selections itself instead of reading the planning kernel's tables.
template <bool PAGED, bool TILE_LSE, bool INLINE_PLAN>
__global__ __launch_bounds__(256, 2) void attn_mfma_kernel(AttnArgs a, int n_rowblocks) {
    extern __shared__ __align__(16) char smem[];
    __shared__ int sU[kMaxBatch], sps[kMaxBatch + 1];
    const DevView& vw = a.view;
    const int Hkv = vw.Hkv, B = vw.B;
    const int tid = threadIdx.x;
    const int wave = uni(tid >> 6);
    const int lane = tid & 63, n = lane & 15, q4 = lane >> 4;
    const int G = a.G, q_len = a.q_len;
    const int rows_total = q_len * G;
    const int cap = vw.R_max + 1;
    const int inner = Hkv * n_rowblocks;

    // ---- LDS: this wave's strip of staged tile log-sum-exps; the batch's raw segment lists ---------------------
    float* lse_buf = reinterpret_cast<float*>(smem) + (TILE_LSE ? wave * 16 * kLsePitch : 0);  // [16][kLsePitch]
    char* lists = smem + (TILE_LSE ? 4 * 16 * kLsePitch * sizeof(float) : 0);
    const int BR = B * vw.R_max;
    long long* raw_ok = reinterpret_cast<long long*>(lists);  // [B][R_max], by round index
    long long* raw_ov = raw_ok + BR;
    int* raw_len = reinterpret_cast<int*>(raw_ov + BR);
    int* raw_sel = raw_len + BR;
    int* meta = raw_sel + BR;   // [B][4]: rounds of the sequence, listed rounds, length of the current round, segments
    int* cum_l = meta + 4 * B;  // [B][cap + 1] tile prefix of every sequence's table
    // Segment i of sequence b's table, as the planning kernel defines it: the i-th listed round (entries that are
    // not rounds of the sequence count as empty), then the current round.
    auto plan_entry = [&](int b, int i, int& len, long long& ok, long long& ov) {
        const int n_rounds = meta[4 * b], n_hist = meta[4 * b + 1], cur_len = meta[4 * b + 2];
        len = 0;
        ok = ov = 0;
        if (i < n_hist) {
            const int r = raw_sel[b * vw.R_max + i];
            if (r >= 0 && r < n_rounds) {
                len = max(raw_len[b * vw.R_max + r], 0);
                ok = raw_ok[b * vw.R_max + r];
                ov = raw_ov[b * vw.R_max + r];
            }
        } else if (i == n_hist && cur_len > 0) {
            len = cur_len;
        }
    };
    const size_t pstride = plan_stride(cap);

    // ---- prologue (the only part with barriers): tiles of every sequence, their prefix over the batch ----------
    if constexpr (INLINE_PLAN) {
        for (int idx = tid; idx < BR; idx += 256) {
            raw_len[idx] = vw.seg_len[idx];
            raw_ok[idx] = vw.seg_off[idx];
            raw_ov[idx] = vw.seg_off_v[idx];
            raw_sel[idx] = a.sel_idx ? a.sel_idx[idx] : idx % vw.R_max;
        }
        for (int b = tid; b < B; b += 256) {
            const int n_rounds = min(max(vw.n_rounds[b], 0), vw.R_max);
            const int n_hist = a.sel_idx ? min(max(a.n_sel[b], 0), vw.R_max) : n_rounds;
            const int cur_len = a.cur_k ? min(max(a.cur_len_dev ? a.cur_len_dev[b] : a.cur_len_host, 0), a.cur_cap) : 0;
            meta[4 * b] = n_rounds;
            meta[4 * b + 1] = n_hist;
            meta[4 * b + 2] = cur_len;
            meta[4 * b + 3] = n_hist + (cur_len > 0 ? 1 : 0);
        }
        __syncthreads();
        if (cap <= 128) {
            // short tables (the usual case): the tile count of every entry by its own thread, then one thread per
            // sequence turns its row into the exclusive prefix with a few dozen LDS operations
            for (int idx = tid; idx < B * cap; idx += 256) {
                const int b = idx / cap, i = idx - b * cap;
                int len;
                long long ok, ov;
                plan_entry(b, i, len, ok, ov);
                cum_l[b * (cap + 1) + i] = (len + kTile - 1) / kTile;
            }
            __syncthreads();
            for (int b = tid; b < B; b += 256) {
                int run = 0;
                for (int i = 0; i < cap; ++i) {
                    const int u = cum_l[b * (cap + 1) + i];
                    cum_l[b * (cap + 1) + i] = run;
                    run += u;
                }
                cum_l[b * (cap + 1) + cap] = run;
                sU[b] = run;
            }
        } else {
            for (int b = wave; b < B; b += 4) {  // one wave per sequence: prefix of its segments' tile counts
                int carry = 0;
                for (int i0 = 0; i0 < cap; i0 += 64) {
                    const int i = i0 + lane;
                    int units = 0;
                    if (i < cap) {
                        int len;
                        long long ok, ov;
                        plan_entry(b, i, len, ok, ov);
                        units = (len + kTile - 1) / kTile;
                    }
                    int total;
                    const int excl = wave_exclusive_scan(units, lane, total);
                    if (i < cap) cum_l[b * (cap + 1) + i] = carry + excl;
                    carry += total;
                }
                if (lane == 0) {
                    cum_l[b * (cap + 1) + cap] = carry;
                    sU[b] = carry;
                }
            }
        }
        __syncthreads();
        if (tid == 0) {  // at most 64 sequences here: their prefix by one thread
            int run = 0;
            for (int b = 0; b < B; ++b) {
                sps[b] = run;
                run += sU[b];
            }
            sps[B] = run;
        }
        __syncthreads();
    } else {
        for (int b = tid; b < B; b += 256) sU[b] = reinterpret_cast<const PlanHeader*>(a.plan + (size_t)b * pstride)->U;
        __syncthreads();
        for (int b = tid; b < B; b += 256) sps[b] = sU[b];
        exclusive_scan_units(sps, B);
    }
    // sps[b] = first tile of sequence b in the batch's list, sps[B] = all tiles
    const int total = sps[B];

    // A sequence with an empty key set has no tile and therefore no wave: its rows are written here.
    if (blockIdx.x == 0) {
        const int rows_seq = q_len * a.Hq;
        for (int b = wave; b < B; b += 4) {
            if (sU[b] != 0) continue;
            for (int i = lane; i < rows_seq * D128; i += 64) a.out[(size_t)b * rows_seq * D128 + i] = 0.f;
            if (a.lse)
                for (int i = lane; i < rows_seq; i += 64) a.lse[(size_t)b * rows_seq + i] = -__builtin_inff();
        }
    }
    if (total == 0) {
        if (blockIdx.x == 0)
            for (int b = tid; b < B; b += 256) a.seq_rec[2 * b] = a.seq_rec[2 * b + 1] = 0;
        return;
    }

    const RangeCut cut = range_cut((unsigned)total, a.min_units, a.max_ranges, a.range_skew);
    const int n_items = (int)cut.n_ranges * inner;
    if (blockIdx.x == 0)  // for the merge kernel: first record and number of records of every sequence
        for (int b = tid; b < B; b += 256) {
            SeqParts sp = {0, 0};
            if (sU[b] > 0) sp = seq_parts(cut, sps[b], sps[b + 1]);
            a.seq_rec[2 * b] = record_index(sp.first_range, b);
            a.seq_rec[2 * b + 1] = sp.n_parts;
        }
    const int n_waves = gridDim.x * 4;
    const char* kbase = reinterpret_cast<const char*>(vw.k);
    const char* vbase = reinterpret_cast<const char*>(vw.v);
    const char* ck = reinterpret_cast<const char*>(a.cur_k);
    const char* cv = reinterpret_cast<const char*>(a.cur_v);

    // One work item per wave (a second one only when there are more items than waves).  Handing the items out
    // dynamically in smaller ranges was measured and lost: under load every dependent memory round trip at the
    // start of an item waits for the compute unit's whole queue of tile loads, 5 to 10 microseconds.
    for (int item = blockIdx.x * 4 + wave; item < n_items; item += n_waves) {
        const int range = item / inner, gi = item - range * inner;  // the (KV head, row block) items of a range are neighbours
        const int g = gi % Hkv, rowblock = gi / Hkv;
        int t_lo = (int)range_begin(cut, range);
        const int t_hi = (int)range_begin(cut, range + 1);
        int b;  // the sequence that holds tile t_lo: the last one with sps[b] <= t_lo
        if (B <= 64) b = __popcll(__ballot(lane < B && sps[lane < B ? lane : 0] <= t_lo)) - 1;
        else b = upper_slot(sps, B, t_lo);

        // ---- the segments of this range: one per sequence it touches --------------------------------------
        for (; t_lo < t_hi; ++b) {
            const int seq_lo = sps[b], seq_hi = sps[b + 1];
            const int seg_hi = min(t_hi, seq_hi);
            if (seg_hi <= t_lo) continue;  // a sequence without tiles
            const int u_lo = t_lo - seq_lo, u_hi = seg_hi - seq_lo;  // tiles of the sequence's own table
            t_lo = seg_hi;
            const SeqParts parts = seq_parts(cut, seq_lo, seq_hi);
            const int rec = record_index(range, b);

            // ---- this wave's query rows ---------------------------------------------------------------
            const int row = rowblock * 16 + n;
            const bool row_ok = row < rows_total;
            const int rr = row_ok ? row : 0;
            const int qtok = rr / G;
            const size_t rowid = ((size_t)b * q_len + qtok) * a.Hq + (size_t)g * G + (rr - qtok * G);
            uint4 qf[4];
            {
                const uint4* qp = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.q) + rowid * D128 * 2);
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) qf[kk] = row_ok ? qp[kk * 4 + q4] : make_uint4(0, 0, 0, 0);
            }

            // ---- the sequence's segment table: a window of 64 entries in this wave's registers -------------
            int n_hist;  // segments before the current round's
            const char* plan_b = a.plan + (size_t)b * pstride;
            if constexpr (INLINE_PLAN) n_hist = meta[4 * b + 1];
            else n_hist = uni(reinterpret_cast<const PlanHeader*>(plan_b)->n_hist);
            const long long* g_ok = reinterpret_cast<const long long*>(plan_b + sizeof(PlanHeader));
            const long long* g_ov = g_ok + cap;
            const int* g_len = reinterpret_cast<const int*>(g_ov + cap);
            const int* g_cum = g_len + cap;
            auto cum_at = [&](int i) { return INLINE_PLAN ? cum_l[b * (cap + 1) + i] : g_cum[i]; };  // i <= cap
            int win_lo = 0, w_len = 0, w_cum = 0;
            long long w_ok = 0, w_ov = 0;
            auto fill_window = [&](int lo) {  // entries lo .. lo + 63 (those past the table read as empty)
                win_lo = lo;
                const int i = lo + lane;
                w_len = 0;
                w_ok = w_ov = 0;
                w_cum = cum_at(min(i, cap));
                if (i < cap) {
                    if constexpr (INLINE_PLAN) {
                        plan_entry(b, i, w_len, w_ok, w_ov);
                    } else {
                        w_len = g_len[i];
                        w_ok = g_ok[i];
                        w_ov = g_ov[i];
                    }
                }
            };
            // The first 64 entries are fetched together with the table's header and the queries (one memory round
            // trip for a sequence of up to 63 segments).  Slot of tile u_lo: the last entry with cum[i] <= u_lo;
            // entries past the sequence's segments hold the total, which is larger.
            fill_window(0);
            int slot = __popcll(__ballot(lane < cap && w_cum <= u_lo)) - 1;
            for (int i0 = 64; i0 < cap; i0 += 64) {
                const int i = i0 + lane;
                slot += __popcll(__ballot(i < cap && cum_at(min(i, cap)) <= u_lo));
            }
            int s_len, s_first, s_end;  // the slot the walk stands in: tokens, first tile, tile after the last
            long long s_ok, s_ov;
            auto open_slot = [&]() {
                if (slot - win_lo >= 63) {  // entry slot + 1 must be in the window too
                    fill_window(slot);
                    wait_for_loads_so_far();  // here, once per window, not after the join on every segment
                }
                const int j = slot - win_lo;
                s_len = lane_get(w_len, j);
                s_first = lane_get(w_cum, j);
                s_end = lane_get(w_cum, j + 1);
                s_ok = lane_get64(w_ok, j);
                s_ov = lane_get64(w_ov, j);
            };
            open_slot();
            // Paged layout: the physical blocks of the tiles ahead, 64 block-table entries at a time in this wave's
            // registers.  A look-up per tile would be a load that the tile's own loads depend on, and loads return in
            // order: it would come back only after everything still in flight, so no tile could be requested before
            // the one before it had arrived.  With the window the walk waits once per 32 tiles (or segment).
            long long bt_lo = 0;  // block-table slot of lane 0's entry
            int bt_val = 0, bt_n = 0;
            auto block_of = [&](long long sl) {  // sl clamped to the table
                if (sl < bt_lo || sl >= bt_lo + bt_n) {
                    bt_lo = sl;
                    bt_n = 64;
                    const long long mine = min(sl + lane, (long long)vw.max_blocks - 1);
                    bt_val = vw.block_table[(size_t)b * vw.max_blocks + mine];
                    wait_for_loads_so_far();  // here, once per window, not after the join on every tile
                }
                return max(lane_get(bt_val, (int)(sl - bt_lo)), 0);
            };
            auto tile_at = [&](int u) {  // u >= the tile of the last call
                while (u >= s_end) {
                    ++slot;
                    open_slot();
                }
                TileRef t;
                t.len = s_len;
                t.uin = u - s_first;
                t.u_seq = u;
                t.is_cur = slot >= n_hist;
                t.ok = s_ok;
                t.ov = s_ov;
                t.pb0 = t.pb1 = 0;
                if (PAGED && !t.is_cur) {
                    const int nblk = (s_len + 15) >> 4;
                    const long long last = (long long)vw.max_blocks - 1;
                    const long long sl0 = min(max(s_ok + min(t.uin * 2, nblk - 1), 0ll), last);
                    const long long sl1 = min(max(s_ok + min(t.uin * 2 + 1, nblk - 1), 0ll), last);
                    t.pb0 = block_of(sl0);
                    t.pb1 = block_of(sl1);
                }
                return t;
            };

            floatx4_t acc[8];
            float m = kNegBig, l = 0.f;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) acc[dt] = floatx4_t{0.f, 0.f, 0.f, 0.f};

            // Loads of a tile.  Halves that lie past the segment's end re-read its last 16-token block (their
            // scores are masked), so every address stays inside the segment.
            auto issue = [&](const TileRef& r, KVTile& t) {
                const int len = r.len;
                const int nblk = (len + 15) >> 4;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int blk = min(r.uin * 2 + h, nblk - 1);  // uniform
                    const int rin = min(n, len - 1 - blk * 16);    // row inside the block, clamped
                    if (r.is_cur) {
                        const size_t e0 = (((size_t)b * a.cur_cap + blk * 16 + rin) * Hkv + g) * D128;
                        const uint4* kp = reinterpret_cast<const uint4*>(ck + e0 * 2);
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk) t.k[h][kk] = kp[kk * 4 + q4];
                        // token-major values: gather 4 tokens of one channel with 2-byte loads
                        const unsigned short* vp = reinterpret_cast<const unsigned short*>(cv);
#pragma unroll
                        for (int dt = 0; dt < 8; ++dt) {
                            uint32_t e[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int tok = min(blk * 16 + q4 * 4 + j, len - 1);
                                e[j] = vp[(((size_t)b * a.cur_cap + tok) * Hkv + g) * D128 + dt * 16 + n];
                            }
                            t.v[dt][h] = make_uint2(e[0] | (e[1] << 16), e[2] | (e[3] << 16));
                        }
                    } else {
                        const char *kp, *vp;
                        if (PAGED) {
                            const int pb = h ? r.pb1 : r.pb0;
                            kp = kbase + ((((size_t)pb * Hkv + g) * 16 + rin) * D128) * 2;
                            vp = vbase + (((size_t)pb * Hkv + g) * D128 * 16) * 2;
                        } else {
                            const size_t L16 = (size_t)nblk * 16;
                            kp = kbase + ((((size_t)r.ok * Hkv + (size_t)g * len + blk * 16 + rin) * D128)) * 2;
                            vp = vbase + ((((size_t)r.ov * Hkv + (size_t)g * L16 + (size_t)blk * 16) * D128)) * 2;
                        }
                        const uint4* kq = reinterpret_cast<const uint4*>(kp);
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk) t.k[h][kk] = kq[kk * 4 + q4];
                        const uint2* vq = reinterpret_cast<const uint2*>(vp);
#pragma unroll
                        // 4 x 8 bytes per channel: an instruction reads 512 contiguous bytes, whole cache lines, which is
                        // what the non-temporal hint needs to pay (see load_once).  The variant for small batches keeps
                        // ordinary loads: it is bound by latency, not bandwidth, and was 6 % slower with the hint
                        // (16.4 -> 17.4 microseconds on the small-batch workload).
                        for (int dt = 0; dt < 8; ++dt) {
                            if constexpr (INLINE_PLAN) t.v[dt][h] = vq[(dt * 16 + n) * 4 + q4];
                            else t.v[dt][h] = load_once(vq + (dt * 16 + n) * 4 + q4);
                        }
                    }
                }
            };

            // Row r of the strip, tiles of this segment from index `first` on, to tile_lse in the score pass's
            // row order [B][Hq][q_len]: 64 consecutive lanes write 64 consecutive tiles of one row.
            auto flush_tile_lse = [&](int first, int count) {
                __builtin_amdgcn_wave_barrier();  // same wave: LDS operations complete in program order
                const int rows_here = min(16, rows_total - rowblock * 16);
                for (int r = 0; r < rows_here; ++r) {
                    const int rw = rowblock * 16 + r, qt = rw / G;
                    const size_t head = (size_t)g * G + (rw - qt * G);
                    float* dst = a.tile_lse + (((size_t)b * a.Hq + head) * q_len + qt) * a.n_tiles_max;
                    const int ut = u_lo + first + lane;
                    if (lane < count && ut < a.n_tiles_max) dst[ut] = lse_buf[r * kLsePitch + lane];
                }
                __builtin_amdgcn_wave_barrier();
            };

            auto consume = [&](const KVTile& t, const TileRef& r) {
                const int tok0 = r.uin * kTile, len = r.len;
                const bool full = !r.is_cur && (len - tok0 >= kTile);
                floatx4_t sc[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    sc[h] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) sc[h] = mfma16(t.k[h][kk], qf[kk], sc[h]);
                }
                if (!full) {
                    // tokens this row may see: the segment's length, or inside the current round the causal limit
                    int lim = len;
                    if (r.is_cur) lim = min(len, max(len - q_len + qtok + 1, 0));
                    if (!row_ok) lim = 0;
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (tok0 + h * 16 + q4 * 4 + i >= lim) sc[h][i] = -__builtin_inff();
                }
                float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                                 fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
                mx = xrow_max4(mx);
                const float m_new = fmaxf(m, mx);
                if (__any(m_new > m)) {
                    const float alpha = fast_exp2((m - m_new) * a.c);
                    l *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt) acc[dt] *= alpha;
                    m = m_new;
                }
                const float mc = m * a.c;
                float p[8];
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i) p[h * 4 + i] = fast_exp2(__builtin_fmaf(sc[h][i], a.c, -mc));
                const float ps = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
                l += ps;
                if constexpr (TILE_LSE) {  // the tile's share of the softmax normaliser: the round scores' raw material
                    const float pt = xrow_sum4(ps);
                    const int ut = r.u_seq - u_lo;
                    if (q4 == 0)
                        lse_buf[n * kLsePitch + (ut & 63)] =
                            pt > 0.f ? kLn2 * __builtin_fmaf(m, a.c, fast_log2(pt)) : -__builtin_inff();
                    if ((ut & 63) == 63) flush_tile_lse(ut - 63, 64);
                }
                uint4 phi, plo;
                phi.x = pack_trunc(p[0], p[1]);
                phi.y = pack_trunc(p[2], p[3]);
                phi.z = pack_trunc(p[4], p[5]);
                phi.w = pack_trunc(p[6], p[7]);
                plo.x = pack_trunc(p[0] - trunc_bf16(p[0]), p[1] - trunc_bf16(p[1]));
                plo.y = pack_trunc(p[2] - trunc_bf16(p[2]), p[3] - trunc_bf16(p[3]));
                plo.z = pack_trunc(p[4] - trunc_bf16(p[4]), p[5] - trunc_bf16(p[5]));
                plo.w = pack_trunc(p[6] - trunc_bf16(p[6]), p[7] - trunc_bf16(p[7]));
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) {
                    const uint4 vf = make_uint4(t.v[dt][0].x, t.v[dt][0].y, t.v[dt][1].x, t.v[dt][1].y);
                    acc[dt] = mfma16(vf, phi, acc[dt]);
                    acc[dt] = mfma16(vf, plo, acc[dt]);
                }
            };

            // ---- stream the tiles u_lo .. u_hi - 1 --------------------------------------------------------
            // Two tile buffers used alternately, and no register that is still being loaded is ever copied.  The
            // next request sits under a condition, so the compiler waits for all outstanding loads before a tile's
            // first product: both tiles are requested back to back and arrive together.  A form of this loop whose
            // waits leave the other tile's loads outstanding was measured and is no faster: the memory system is
            // full either way.
            {
                KVTile ta, tb;
                TileRef ref_a, ref_b;
                int u = u_lo;
                ref_a = tile_at(u);
                issue(ref_a, ta);
                while (true) {
                    ++u;
                    const bool have_b = u < u_hi;
                    if (have_b) {
                        ref_b = tile_at(u);
                        issue(ref_b, tb);
                    }
                    consume(ta, ref_a);
                    if (!have_b) break;
                    ++u;
                    const bool have_a = u < u_hi;
                    if (have_a) {
                        ref_a = tile_at(u);
                        issue(ref_a, ta);
                    }
                    consume(tb, ref_b);
                    if (!have_a) break;
                }
                if constexpr (TILE_LSE) {
                    const int done = u_hi - u_lo;
                    if (done & 63) flush_tile_lse(done & ~63, done & 63);
                }
            }

            // ---- the four lane groups hold partial sums of the same rows -------------------------------------
            l = xrow_sum4(l);
            if (parts.n_parts == 1) {
                if (row_ok) {
                    const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt)
                        *reinterpret_cast<floatx4_t*>(a.out + rowid * D128 + dt * 16 + q4 * 4) = acc[dt] * inv;
                    if (a.lse && q4 == 0)
                        a.lse[rowid] = l > 0.f ? __builtin_fmaf(m, a.scale, __builtin_logf(l)) : -__builtin_inff();
                }
                continue;
            }

            // ---- the sequence lies in several ranges: leave this segment's partial result ---------------------
            if (row_ok) {
                const size_t rrow = ((size_t)rec * inner + gi) * 16 + n;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt)
                    *reinterpret_cast<floatx4_t*>(a.rec_acc + rrow * D128 + dt * 16 + q4 * 4) = acc[dt];
                if (q4 == 0) *reinterpret_cast<float2*>(a.rec_ml + rrow * 2) = make_float2(m, l);
            }
        }
    }
}

int launch_attn_mfma(const AttnArgs& a, bool paged, int num_cu, hipStream_t st) {
    const int rows_total = a.q_len * a.G;
    const int B = a.view.B, Hkv = a.view.Hkv;
    if (a.G > 16) return fail(RA_ERR_UNSUPPORTED, "attention: Hq / Hkv = %d exceeds 16", a.G);
    if (B > kMaxBatch) return fail(RA_ERR_UNSUPPORTED, "attention: batch %d exceeds %d", B, kMaxBatch);
    const MfmaDecodeShape s =
        mfma_decode_shape(num_cu, B, a.view.R_max, Hkv, rows_total, mfma_max_tiles(B, a.max_tokens, a.view.R_max, a.cur_cap));
    if (a.max_ranges != s.max_ranges) return fail(RA_ERR_INVALID_ARG, "attention: launch shape mismatch");
    const bool inline_plan = attn_mfma_plans_inline(B, a.view.R_max);
    const bool tile_lse = a.tile_lse != nullptr;
    const size_t smem = (tile_lse ? (size_t)4 * 16 * kLsePitch * sizeof(float) : 0) +
                        (inline_plan ? attn_mfma_inline_bytes(B, a.view.R_max) : 0);
    const dim3 g((unsigned)s.grid), blk(256);
#define RA_ATTN_CASE(P_, L_, I_)                                                                          \
    if (paged == P_ && tile_lse == L_ && inline_plan == I_) {                                             \
        RA_LAUNCH_TIMED((attn_mfma_kernel<P_, L_, I_>), g, blk, smem, st, a, s.n_rowblocks);              \
        return RA_OK;                                                                                     \
    }
    RA_ATTN_CASE(false, false, false) RA_ATTN_CASE(false, false, true) RA_ATTN_CASE(true, false, false)
    RA_ATTN_CASE(true, false, true) RA_ATTN_CASE(false, true, false) RA_ATTN_CASE(false, true, true)
    RA_ATTN_CASE(true, true, false) RA_ATTN_CASE(true, true, true)
#undef RA_ATTN_CASE
    return RA_OK;
}

// Second step of the matrix-core kernel above: merges the records of the sequences that were cut.
void launch_merge_records(const AttnArgs& a, int num_cu, hipStream_t st) {
    const MfmaDecodeShape s = mfma_decode_shape(num_cu, a.view.B, a.view.R_max, a.view.Hkv, a.q_len * a.G,
                                                mfma_max_tiles(a.view.B, a.max_tokens, a.view.R_max, a.cur_cap));
    if (s.max_ranges <= 1) return;  // a single range never cuts a sequence
    hipLaunchKernelGGL(merge_records_kernel, dim3((unsigned)(a.view.B * s.inner)), dim3(256), 0, st, a, s.n_rowblocks);
}

}  // namespace ra
