// Round-sparse attention over the selected rounds, bf16 / head_dim 128, on the matrix cores
// (paper Sec. 3.2 steps 4 and 5: question prefill and decode after the watershed layer).
//
// This kernel serves decode and short questions; long questions use the kernel that shares key tiles
// through LDS.  The "query rows" of a KV head g are the pairs (query token i, head h of the group),
// row = i * G + h: G rows for decode, q_len * G in general; they are handled in tiles of 16 rows.
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
// Launch: persistent workgroups, about two per compute unit.  Every workgroup derives the same
// balanced schedule of the batch (see build_schedule) and walks the work items
// (piece of a sequence, KV head, row block) with stride gridDim.x.
// The four waves of a workgroup take different key tiles of the same 16 rows and are merged through LDS.
#include "attn_common.hpp"
#include "mfma_util.hpp"
#include "debug_ts.hpp"

namespace ra {

constexpr int kTile = 32;  // tokens per key tile (two 16-token halves)
constexpr int D128 = 128;
constexpr int kPiecesPerWorkgroup = 4;  // pieces a persistent workgroup aims to get when work is plentiful

struct KVTile {
    uint4 k[2][4];  // [half][kk]: 8 channels kk*32 + 8*(lane/16) .. of token half*16 + lane%16
    uint2 v[8][2];  // [dt][half]: tokens 4*(lane/16) .. +3 of that half, channel dt*16 + lane%16
};

// TILE_LSE: 0 = attention only; 1 = also one log-sum-exp per (query row, key tile), stored as it is produced;
// 2 = the same, staged in LDS and written out in blocks of 64 tiles (pays when a piece has many tiles).
// INLINE_PLAN: the workgroup resolves the batch's selections itself instead of reading the planning kernel's tables.
template <bool PAGED, int TILE_LSE, bool INLINE_PLAN>
__global__ __launch_bounds__(256, 2) void attn_mfma_kernel(AttnArgs a, int n_rowblocks) {
    extern __shared__ __align__(16) char smem[];
    __shared__ int sU[kMaxBatch], sps[kMaxBatch + 1];
    RA_TS(0);
    const DevView& vw = a.view;
    const int Hkv = vw.Hkv;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, n = lane & 15, q4 = lane >> 4;
    const int G = a.G, q_len = a.q_len;
    const int rows_total = q_len * G;
    constexpr int NT = 1, RB = 16;  // one tile of 16 rows per work item

    const int cap = vw.R_max + 1;
    SlotTable tab;
    tab.carve(smem, cap);
    float* red = reinterpret_cast<float*>(smem + ((SlotTable::bytes(cap) + 15) & ~(size_t)15));
    constexpr int kLsePitch = 65, kLseBlock = 16 * kLsePitch;
    float* lse_buf = red + 128;  // [2][16][65] tile log-sum-exps on their way out; reused by the merge afterwards

    // ---- the batch's schedule, identical in every workgroup --------------------------------------------
    const int inner = Hkv * n_rowblocks;  // work items per piece
    const long long slots = ((long long)gridDim.x * kPiecesPerWorkgroup + inner - 1) / inner;
    // Without a planning kernel: the raw segment lists of the whole batch, by round index, in LDS.
    const int BR = vw.B * vw.R_max;
    long long* raw_ok = reinterpret_cast<long long*>(red + 128 + 4 * 16 * 128);  // [B][R_max]
    long long* raw_ov = raw_ok + BR;
    int* raw_len = reinterpret_cast<int*>(raw_ov + BR);
    int* raw_sel = raw_len + BR;
    int* meta = raw_sel + BR;  // [B][3]: rounds of the sequence, listed rounds, length of the current round
    // Segment i of sequence b's table, as the planning kernel defines it: the i-th listed round (entries that are
    // not rounds of the sequence count as empty), then the current round.
    auto plan_entry = [&](int b, int i, int& len, long long& ok, long long& ov) {
        const int n_rounds = meta[3 * b], n_hist = meta[3 * b + 1], cur_len = meta[3 * b + 2];
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
    int P;
    if constexpr (INLINE_PLAN) {
        for (int idx = tid; idx < BR; idx += 256) {
            raw_len[idx] = vw.seg_len[idx];
            raw_ok[idx] = vw.seg_off[idx];
            raw_ov[idx] = vw.seg_off_v[idx];
            raw_sel[idx] = a.sel_idx ? a.sel_idx[idx] : idx % vw.R_max;
        }
        for (int b = tid; b < vw.B; b += 256) {
            const int n_rounds = min(max(vw.n_rounds[b], 0), vw.R_max);
            meta[3 * b] = n_rounds;
            meta[3 * b + 1] = a.sel_idx ? min(max(a.n_sel[b], 0), vw.R_max) : n_rounds;
            meta[3 * b + 2] = a.cur_k ? min(max(a.cur_len_dev ? a.cur_len_dev[b] : a.cur_len_host, 0), a.cur_cap) : 0;
            sU[b] = 0;
        }
        __syncthreads();
        // work units of every sequence: one table entry per thread, integer adds in LDS (order does not matter)
        for (int idx = tid; idx < vw.B * cap; idx += 256) {
            const int b = idx / cap, i = idx - b * cap;
            int len;
            long long ok, ov;
            plan_entry(b, i, len, ok, ov);
            if (len > 0) atomicAdd(&sU[b], (len + kTile - 1) / kTile);
        }
        P = schedule_from_counts(vw.B, a.S, a.min_units, slots, sU, sps);
    } else {
        P = build_schedule(a.plan, cap, vw.B, a.S, a.min_units, slots, sU, sps);
    }
    if (blockIdx.x == 0)
        for (int b = tid; b < vw.B; b += 256) a.n_parts[b] = sps[b + 1] - sps[b];

    const char* kbase = reinterpret_cast<const char*>(vw.k);
    const char* vbase = reinterpret_cast<const char*>(vw.v);
    const char* ck = reinterpret_cast<const char*>(a.cur_k);
    const char* cv = reinterpret_cast<const char*>(a.cur_v);
    const long long n_items = (long long)P * inner;
    RA_TS(1);

    for (long long item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int piece = (int)(item / inner);
        const int rest = (int)(item - (long long)piece * inner);
        const int g = rest % Hkv, rowblock = rest / Hkv;
        const int b = find_slot(sps, vw.B, piece);  // sps[b] <= piece < sps[b + 1]
        const int s = piece - sps[b];
        const int S_eff = sps[b + 1] - sps[b];
        const int U = sU[b];
        const int u_lo = (int)(((long long)U * s) / S_eff);
        const int u_hi = (int)(((long long)U * (s + 1)) / S_eff);

        __syncthreads();  // the previous item's readers of tab / red are done
        int n_slots, n_hist;
        if constexpr (INLINE_PLAN) {
            n_hist = meta[3 * b + 1];
            n_slots = n_hist + (meta[3 * b + 2] > 0 ? 1 : 0);
            for (int i = tid; i < cap; i += 256) {
                int len;
                long long ok, ov;
                plan_entry(b, i, len, ok, ov);
                tab.len[i] = len;
                tab.off_k[i] = ok;
                tab.off_v[i] = ov;
                tab.cum[i] = (len + kTile - 1) / kTile;
            }
            exclusive_scan_units(tab.cum, cap);
        } else {
            const PlanHeader hdr = load_plan(a.plan + (size_t)b * plan_stride(cap), cap, tab);
            n_slots = hdr.n_slots;
            n_hist = hdr.n_hist;
            __syncthreads();
        }

        RA_TS(2);
        // ---- this wave's query rows -------------------------------------------------------------------
        int qtok[NT];
        bool row_ok[NT];
        size_t rowid[NT];
        uint4 qf[NT][4];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int row = rowblock * RB + nt * 16 + n;
            row_ok[nt] = row < rows_total;
            const int rr = row_ok[nt] ? row : 0;
            qtok[nt] = rr / G;
            rowid[nt] = ((size_t)b * q_len + qtok[nt]) * a.Hq + (size_t)g * G + (rr - qtok[nt] * G);
            const uint4* qp = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.q) + rowid[nt] * D128 * 2);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) qf[nt][kk] = row_ok[nt] ? qp[kk * 4 + q4] : make_uint4(0, 0, 0, 0);
        }

        floatx4_t acc[NT][8];
        float m[NT], l[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            m[nt] = kNegBig;
            l[nt] = 0.f;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) acc[nt][dt] = floatx4_t{0.f, 0.f, 0.f, 0.f};
        }

        // Loads of tile `uin` of segment `slot`.  Halves that lie past the segment's end re-read its
        // last 16-token block (their scores are masked), so every address stays inside the segment.
        auto issue = [&](int uin, int slot, KVTile& t, int& len_out, bool& is_cur_out) {
            const int len = tab.len[slot];
            const bool is_cur = slot >= n_hist;
            len_out = len;
            is_cur_out = is_cur;
            const int nblk = (len + 15) >> 4;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int blk = min(uin * 2 + h, nblk - 1);  // uniform
                const int rin = min(n, len - 1 - blk * 16);  // row inside the block, clamped
                if (is_cur) {
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
                        long long si = tab.off_k[slot] + blk;
                        si = si < 0 ? 0 : (si >= vw.max_blocks ? vw.max_blocks - 1 : si);
                        int pb = vw.block_table[(size_t)b * vw.max_blocks + si];
                        pb = pb < 0 ? 0 : pb;
                        kp = kbase + ((((size_t)pb * Hkv + g) * 16 + rin) * D128) * 2;
                        vp = vbase + (((size_t)pb * Hkv + g) * D128 * 16) * 2;
                    } else {
                        const size_t L16 = (size_t)nblk * 16;
                        kp = kbase + ((((size_t)tab.off_k[slot] * Hkv + (size_t)g * len + blk * 16 + rin) * D128)) * 2;
                        vp = vbase + ((((size_t)tab.off_v[slot] * Hkv + (size_t)g * L16 + (size_t)blk * 16) * D128)) * 2;
                    }
                    const uint4* kq = reinterpret_cast<const uint4*>(kp);
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) t.k[h][kk] = kq[kk * 4 + q4];
                    const uint2* vq = reinterpret_cast<const uint2*>(vp);
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt) t.v[dt][h] = vq[(dt * 16 + n) * 4 + q4];  // 4 x 8 bytes per channel
                }
            }
        };

        auto consume = [&](const KVTile& t, int uin, int len, bool is_cur, int u_seq) {
            const int tok0 = uin * kTile;
            const bool full = !is_cur && (len - tok0 >= kTile);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                floatx4_t sc[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    sc[h] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) sc[h] = mfma16(t.k[h][kk], qf[nt][kk], sc[h]);
                }
                if (!full) {
                    // tokens this row may see: the segment's length, or inside the current round the causal limit
                    int lim = len;
                    if (is_cur) lim = min(len, max(len - q_len + qtok[nt] + 1, 0));
                    if (!row_ok[nt]) lim = 0;
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (tok0 + h * 16 + q4 * 4 + i >= lim) sc[h][i] = -__builtin_inff();
                }
                float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                                 fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
                mx = xrow_max4(mx);
                const float m_new = fmaxf(m[nt], mx);
                if (__any(m_new > m[nt])) {
                    const float alpha = fast_exp2((m[nt] - m_new) * a.c);
                    l[nt] *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt) acc[nt][dt] *= alpha;
                    m[nt] = m_new;
                }
                const float mc = m[nt] * a.c;
                float p[8];
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i) p[h * 4 + i] = fast_exp2(__builtin_fmaf(sc[h][i], a.c, -mc));
                const float ps = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
                l[nt] += ps;
                if constexpr (TILE_LSE == 1) {  // the tile's share of the softmax normaliser: the round scores' raw material
                    const float pt = xrow_sum4(ps);
                    if (q4 == 0 && row_ok[nt] && u_seq < a.n_tiles_max) {
                        // row order of the score pass: [B][Hq][q_len]
                        const size_t head = rowid[nt] - ((size_t)b * q_len + qtok[nt]) * a.Hq;
                        const size_t srow = ((size_t)b * a.Hq + head) * q_len + qtok[nt];
                        a.tile_lse[srow * a.n_tiles_max + u_seq] =
                            pt > 0.f ? kLn2 * __builtin_fmaf(m[nt], a.c, fast_log2(pt)) : -__builtin_inff();
                    }
                } else if constexpr (TILE_LSE == 2) {
                    // Staged in LDS, [2 blocks of 64 tiles][16 rows][64 + 1]; flush_tile_lse writes a block out in
                    // whole runs per row (one scattered 4-byte store per row and tile costs 14 % of a long pass).
                    const float pt = xrow_sum4(ps);
                    const int ut = u_seq - u_lo;
                    if (q4 == 0)
                        lse_buf[((ut >> 6) & 1) * kLseBlock + n * kLsePitch + (ut & 63)] =
                            pt > 0.f ? kLn2 * __builtin_fmaf(m[nt], a.c, fast_log2(pt)) : -__builtin_inff();
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
                    acc[nt][dt] = mfma16(vf, phi, acc[nt][dt]);
                    acc[nt][dt] = mfma16(vf, plo, acc[nt][dt]);
                }
            }
        };

        // Block k of the staged tile log-sum-exps (tiles u_lo + 64 k ...) to tile_lse, rows in the score pass's
        // order [B][Hq][q_len]: 16 consecutive lanes write 16 consecutive tiles of one row.
        auto flush_tile_lse = [&](int k) {
            const int r = tid >> 4, rr = rowblock * RB + r;
            if (rr >= rows_total) return;
            const int qt = rr / G;
            const size_t head = (size_t)g * G + (rr - qt * G);
            float* dst = a.tile_lse + (((size_t)b * a.Hq + head) * q_len + qt) * a.n_tiles_max;
            const float* src = lse_buf + (k & 1) * kLseBlock + r * kLsePitch;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int col = (tid & 15) + 16 * i;
                const int ut = u_lo + 64 * k + col;
                if (ut < u_hi && ut < a.n_tiles_max) dst[ut] = src[col];
            }
        };

        // ---- stream the key tiles --------------------------------------------------------------------
        {
            const int step = 4;
            int u = u_lo + wave;
            bool have = u < u_hi;
            int slot = 0;
            // Two tile buffers used alternately: the loads of one tile are in flight while the other
            // is consumed, and no register that is still being loaded is ever copied.
            KVTile ta, tb;
            int len_a = 0, uin_a = 0, len_b = 0, uin_b = 0, us_a = 0, us_b = 0;
            bool cur_a = false, cur_b = false;
            if (have) {
                slot = find_slot(tab.cum, n_slots, u);
                uin_a = u - tab.cum[slot];
                us_a = u;
                issue(uin_a, slot, ta, len_a, cur_a);
            }
            if constexpr (TILE_LSE == 2) {
                // Same walk, but with a trip count every wave shares (a pair of tiles per wave and trip, eight
                // tiles per workgroup), so that the workgroup can meet at a barrier after each block of 64 tiles
                // and write that block out while the next one is computed into the other half of the buffer.
                const int n_trips = (u_hi - u_lo + 7) >> 3;
                for (int trip = 0; trip < n_trips; ++trip) {
                    if (have) {
                        u += step;
                        const bool have_b = u < u_hi;
                        if (have_b) {
                            while (u >= tab.cum[slot + 1]) ++slot;
                            uin_b = u - tab.cum[slot];
                            us_b = u;
                            issue(uin_b, slot, tb, len_b, cur_b);
                        }
                        consume(ta, uin_a, len_a, cur_a, us_a);
                        have = false;
                        if (have_b) {
                            u += step;
                            have = u < u_hi;
                            if (have) {
                                while (u >= tab.cum[slot + 1]) ++slot;
                                uin_a = u - tab.cum[slot];
                                us_a = u;
                                issue(uin_a, slot, ta, len_a, cur_a);
                            }
                            consume(tb, uin_b, len_b, cur_b, us_b);
                        }
                    }
                    if ((trip & 7) == 7 || trip == n_trips - 1) {
                        __syncthreads();  // every wave's values of this block are in LDS
                        flush_tile_lse(trip >> 3);
                    }
                }
                __syncthreads();  // the staging buffer shares its memory with the merge below
            } else
            while (have) {
                u += step;
                const bool have_b = u < u_hi;
                if (have_b) {
                    while (u >= tab.cum[slot + 1]) ++slot;
                    uin_b = u - tab.cum[slot];
                    us_b = u;
                    issue(uin_b, slot, tb, len_b, cur_b);
                }
                consume(ta, uin_a, len_a, cur_a, us_a);
                if (!have_b) break;
                u += step;
                have = u < u_hi;
                if (have) {
                    while (u >= tab.cum[slot + 1]) ++slot;
                    uin_a = u - tab.cum[slot];
                    us_a = u;
                    issue(uin_a, slot, ta, len_a, cur_a);
                }
                consume(tb, uin_b, len_b, cur_b, us_b);
            }
        }

        RA_TS(3);
        // ---- the four lane groups hold partial sums of the same rows ---------------------------------------
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            l[nt] = xrow_sum4(l[nt]);
        }

        {
            // ---- merge the four waves (different tokens, same rows) through LDS ----------------------------
            float* sm = red;          // [4][16]
            float* sl = red + 64;     // [4][16]
            float* sacc = red + 128;  // [4][16][128]
            if (q4 == 0) {
                sm[wave * 16 + n] = m[0];
                sl[wave * 16 + n] = l[0];
            }
#pragma unroll
            for (int dt = 0; dt < 8; ++dt)
                *reinterpret_cast<floatx4_t*>(sacc + ((wave * 16 + n) * D128) + dt * 16 + q4 * 4) = acc[0][dt];
            __syncthreads();
            const int rows_here = min(16, rows_total - rowblock * RB);
            for (int idx = tid; idx < rows_here * D128; idx += 256) {
                const int r = idx >> 7, dim = idx & 127;
                const float M = fmaxf(fmaxf(sm[r], sm[16 + r]), fmaxf(sm[32 + r], sm[48 + r]));
                float num = 0.f, den = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float f = fast_exp2((sm[w * 16 + r] - M) * a.c);
                    num = __builtin_fmaf(sacc[(w * 16 + r) * D128 + dim], f, num);
                    den = __builtin_fmaf(sl[w * 16 + r], f, den);
                }
                const int rr = rowblock * RB + r;
                const int qi = rr / G;
                const size_t rid = ((size_t)b * q_len + qi) * a.Hq + (size_t)g * G + (rr - qi * G);
                if (S_eff > 1) {
                    const size_t pr = rid * a.S + s;
                    a.part_acc[pr * D128 + dim] = num;
                    if (dim == 0) {
                        a.part_m[pr] = M;
                        a.part_l[pr] = den;
                    }
                } else {
                    a.out[rid * D128 + dim] = den > 0.f ? num / den : 0.f;
                    if (a.lse && dim == 0)
                        a.lse[rid] = den > 0.f ? __builtin_fmaf(M, a.scale, __builtin_logf(den)) : -__builtin_inff();
                }
            }
        }
        RA_TS(4);
    }
    RA_TS(5);
}

RA_TS_DEFINE_READER(ra_debug_read_ts_attn)

int launch_attn_mfma(const AttnArgs& a, bool paged, int num_cu, hipStream_t st) {
    const int rows_total = a.q_len * a.G;
    const int B = a.view.B, Hkv = a.view.Hkv;
    if (a.G > 16) return fail(RA_ERR_UNSUPPORTED, "attention: Hq / Hkv = %d exceeds 16", a.G);
    if (B > kMaxBatch) return fail(RA_ERR_UNSUPPORTED, "attention: batch %d exceeds %d", B, kMaxBatch);
    const size_t tab_bytes = align_up(SlotTable::bytes(a.view.R_max + 1), 16);
    const int n_rowblocks = (rows_total + 15) / 16;
    // Persistent launch: two workgroups per compute unit, but never more than the work items the batch
    // can have at most (every sequence has at least one piece and at most S).
    const long long max_tiles = (long long)B * (a.max_tokens / kTile + a.view.R_max + 1 + a.cur_cap / kTile + 1);
    long long max_pieces = (long long)B + max_tiles / a.min_units;
    if (max_pieces > (long long)B * a.S) max_pieces = (long long)B * a.S;
    long long grid = (long long)2 * num_cu;
    if (grid > max_pieces * Hkv * n_rowblocks) grid = max_pieces * Hkv * n_rowblocks;
    if (grid < 1) grid = 1;
    const bool inline_plan = attn_mfma_plans_inline(B, a.view.R_max);
    // tiles a piece is expected to hold: a sequence's tiles over the pieces it gets when the work is spread
    // over the grid (at most S)
    const long long tiles_seq = a.max_tokens / kTile + 1;
    long long pieces_seq = grid * kPiecesPerWorkgroup / ((long long)B * Hkv * n_rowblocks);
    pieces_seq = pieces_seq < 1 ? 1 : (pieces_seq > a.S ? a.S : pieces_seq);
    const int lse_mode = !a.tile_lse ? 0 : (tiles_seq / pieces_seq >= 128 ? 2 : 1);
    const size_t smem = tab_bytes + (128 + 4 * 16 * 128) * sizeof(float) +
                        (inline_plan ? attn_mfma_inline_bytes(B, a.view.R_max) : 0);
    const dim3 g((unsigned)grid), blk(256);
#define RA_ATTN_CASE(P_, L_, I_)                                                                          \
    if (paged == P_ && lse_mode == L_ && inline_plan == I_) {                                             \
        RA_LAUNCH_TIMED((attn_mfma_kernel<P_, L_, I_>), g, blk, smem, st, a, n_rowblocks);                \
        return RA_OK;                                                                                     \
    }
    RA_ATTN_CASE(false, 0, false) RA_ATTN_CASE(false, 0, true) RA_ATTN_CASE(true, 0, false) RA_ATTN_CASE(true, 0, true)
    RA_ATTN_CASE(false, 1, false) RA_ATTN_CASE(false, 1, true) RA_ATTN_CASE(true, 1, false) RA_ATTN_CASE(true, 1, true)
    RA_ATTN_CASE(false, 2, false) RA_ATTN_CASE(false, 2, true) RA_ATTN_CASE(true, 2, false) RA_ATTN_CASE(true, 2, true)
#undef RA_ATTN_CASE
    return RA_OK;
}

}  // namespace ra
