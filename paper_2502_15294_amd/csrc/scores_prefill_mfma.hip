// Round scores (paper Sec. 3.1, Eq. 1) for a question of many tokens: streaming pass over the watershed
// layer's keys for bf16 / head_dim 128 on the matrix cores, many query rows per KV head.
//
// Same roles as in the attention kernels: S^T[16 tokens x 16 rows] = K . Q^T, lane%16 is the query row, so a
// row's running (reference logit, sum of exponentials) stays in its lane.  What is produced is one
// log-sum-exp per (query row, 256-token chunk of a round); the finishing kernels turn those into round masses.
//
//   * a work item is (piece of the sequence's chunks, KV head, block of 256 query rows): four waves with
//     four 16-row tiles each walk the key tiles of the piece's chunks in lockstep;
//   * every 32-token key tile (8 KB) is fetched from global memory once per workgroup, one tile ahead, with
//     whole-row coalesced loads that go straight into one of two LDS buffers (no registers, no LDS stores): the
//     tile's image there is row-major with the 16-byte chunks of row r rotated by r, so that the operand reads
//     (16 lanes = 16 rows, one chunk) touch every bank once; all four waves read it; one barrier per tile;
//   * the reference logit of a lane is only raised when one of its logits exceeds it by 2^16 after scaling,
//     so the common tile costs one multiply-add, one exponential and one add per logit;
//   * persistent launch with the batch-wide balanced schedule used by the attention kernels.  The schedule
//     is made in units of key tiles (chunks at the end of a round are short, so chunk counts would balance
//     badly) and each piece boundary is then moved to the start of the chunk it falls in.
#include "scores_common.hpp"
#include "mfma_util.hpp"
#include "stream_kv.hpp"

namespace ra {

constexpr int kTileSP = 32;                      // tokens per key tile
constexpr int kNTS = 4;                          // 16-row tiles per wave
constexpr int kRowsPerItemS = 4 * kNTS * 16;     // 256
constexpr int kTilesPerChunk = kChunkTokens / kTileSP;
constexpr int kKTileBytes = 8192;
constexpr int kPiecesPerWorkgroupS = 1;  // measured on the 4 x 32 K-token question-prefill workload: 1: 167-172 us, 2: 174-180, 3: 176
constexpr int kWorkgroupsPerCuS = 3;

// Planning kernel, grid (B): the table of segments of sequence b (all history rounds, then the current round)
// in the layout the attention kernels use, with cum = prefix sum of the segments' chunk counts, the unused
// value-offset column holding the prefix sum of their key-tile counts, and U = total key tiles.
__global__ __launch_bounds__(256) void scores_plan_kernel(ScoreArgs a, char* plan) {
    extern __shared__ __align__(16) char smem[];
    const DevView& vw = a.view;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int cap = vw.R_max + 1;
    int* cum = reinterpret_cast<int*>(smem);  // [cap + 1] chunks
    int* tcum = cum + cap + 1;                // [cap + 1] tiles
    char* plan_b = plan + (size_t)b * plan_stride(cap);
    long long* g_off_k = reinterpret_cast<long long*>(plan_b + sizeof(PlanHeader));
    long long* g_tcum = g_off_k + cap;
    int* g_len = reinterpret_cast<int*>(g_tcum + cap);
    int* g_cum = g_len + cap;
    const int n_hist = min(max(vw.n_rounds[b], 0), vw.R_max);
    const int n_slots = n_hist + (a.cur_k && a.cur_len > 0 ? 1 : 0);
    for (int i = tid; i < cap; i += 256) {
        int len = 0;
        long long ok = 0;
        if (i < n_hist) {
            len = max(vw.seg_len[(size_t)b * vw.R_max + i], 0);
            ok = vw.seg_off[(size_t)b * vw.R_max + i];
        } else if (i < n_slots) {
            len = a.cur_len;
        }
        g_len[i] = len;
        g_off_k[i] = ok;
        cum[i] = chunks_of(len);
        tcum[i] = (len + kTileSP - 1) / kTileSP;
    }
    exclusive_scan_units(cum, cap);
    exclusive_scan_units(tcum, cap);
    for (int i = tid; i <= cap; i += 256) g_cum[i] = cum[i];
    for (int i = tid; i < cap; i += 256) g_tcum[i] = tcum[i];
    if (tid == 0) {
        PlanHeader h;
        h.n_slots = n_slots;
        h.n_hist = n_hist;
        h.U = tcum[n_slots];
        h.S_eff = 1;
        *reinterpret_cast<PlanHeader*>(plan_b) = h;
    }
}

template <bool PAGED>
__global__ __launch_bounds__(256, kWorkgroupsPerCuS) void scores_prefill_mfma_kernel(ScoreArgs a, int n_rowblocks) {
    extern __shared__ __align__(16) char smem[];
    __shared__ int sU[kMaxBatch], sps[kMaxBatch + 1];
    const DevView& vw = a.view;
    const int Hkv = vw.Hkv;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, n = lane & 15, q4 = lane >> 4;
    const int G = a.Hq / Hkv, q_len = a.q_len;
    const int rows_total = q_len * G;

    const int cap = vw.R_max + 1;
    SlotTable tab;
    tab.carve(smem, cap);
    char* tiles = smem + ((SlotTable::bytes(cap) + 15) & ~(size_t)15);  // two key-tile buffers
    const unsigned tiles_lds = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lptr_t)tiles);

    const int inner = Hkv * n_rowblocks;
    const long long slots = ((long long)gridDim.x * kPiecesPerWorkgroupS + inner - 1) / inner;
    const int P = build_schedule(a.plan, cap, vw.B, a.S, a.min_units, slots, sU, sps);

    const char* kbase = reinterpret_cast<const char*>(vw.k);
    const char* ck = reinterpret_cast<const char*>(a.cur_k);
    const long long n_items = (long long)P * inner;
    const float slack = 16.f / a.c;
    auto uni = [](int x) { return __builtin_amdgcn_readfirstlane(x); };
    auto uni64 = [&](long long x) { return ((long long)uni((int)(x >> 32)) << 32) | (unsigned)uni((int)x); };

    for (long long item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int piece = (int)(item / inner);
        const int rest = (int)(item - (long long)piece * inner);
        const int g = rest % Hkv, rowblock = rest / Hkv;
        const int b = find_slot(sps, vw.B, piece);
        const int s = piece - sps[b];
        const int S_eff = sps[b + 1] - sps[b];
        const int T = sU[b];  // key tiles of sequence b; the piece is tiles [t_lo, t_hi) moved to chunk starts
        const int t_lo = (int)(((long long)T * s) / S_eff), t_hi = (int)(((long long)T * (s + 1)) / S_eff);

        __syncthreads();  // the previous item's readers of the table and the tile buffers are done
        const PlanHeader hdr = load_plan(a.plan + (size_t)b * plan_stride(cap), cap, tab);
        const int n_slots = uni(hdr.n_slots), n_hist = uni(hdr.n_hist);
        __syncthreads();
        auto chunk_of_tile = [&](int t) {  // index of the chunk that holds tile t (the chunk count for t == T)
            if (t >= T) return uni(tab.cum[n_slots]);
            const int sl = find_slot(tab.off_v, n_slots, (long long)t);
            return uni(tab.cum[sl] + (t - (int)tab.off_v[sl]) / kTilesPerChunk);
        };
        const int u_lo = chunk_of_tile(t_lo), u_hi = chunk_of_tile(t_hi);  // chunks [u_lo, u_hi) of sequence b
        if (u_lo >= u_hi) continue;

        // ---- this wave's query rows -------------------------------------------------------------------
        // (row nt of this lane is row0 + 16*nt; whatever else is needed of it is recomputed where it is used)
        const int row0 = rowblock * kRowsPerItemS + wave * kNTS * 16 + n;
        uint4 qf[kNTS][4];
#pragma unroll
        for (int nt = 0; nt < kNTS; ++nt) {
            const int row = row0 + nt * 16;
            const int rr = row < rows_total ? row : 0;
            const int qtok = rr / G;
            const size_t qrow = ((size_t)b * q_len + qtok) * a.Hq + (size_t)g * G + (rr - qtok * G);
            const uint4* qp = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.q) + qrow * 256);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) qf[nt][kk] = row < rows_total ? qp[kk * 4 + q4] : make_uint4(0, 0, 0, 0);
        }
        float m[kNTS], l[kNTS];
#pragma unroll
        for (int nt = 0; nt < kNTS; ++nt) {
            m[nt] = kNegBig;
            l[nt] = 0.f;
        }

        // Uniform state of the loader: the segment it stands in (the table in LDS is read on entry only), and
        // inside it the next tile: the address of its first token's keys (head g) and the tokens left from there.
        int seg_len = 0, seg_first = 0, seg_end = 0, rows_left = 0;
        bool seg_cur = false;
        const char *seg_k = nullptr, *tile_k = nullptr;  // contiguous history / current round
        long long seg_tab = 0;                           // paged history: first block-table slot
        unsigned kstride = 256;                          // bytes from one token's keys to the next
        // This wave fills rows 8 wave .. + 7 of the tile's LDS image (row = token of the tile, 256 bytes) with two
        // loads of four whole rows each, 16 lanes per row; lane L's 16 bytes land at position L % 16 of its row,
        // where chunk (L % 16 - row) mod 16 belongs.
        const int row_a = 8 * wave + q4;                 // this lane helps to load tile rows row_a and row_a + 4
        const unsigned chunk_a = (unsigned)((n - row_a) & 15) * 16u, chunk_b = (unsigned)((n - row_a - 4) & 15) * 16u;
        unsigned off_a = 0, off_b = 0;                   // byte offsets from tile_k for a full tile
        auto open_seg = [&](int slot) {
            seg_len = uni(tab.len[slot]);
            seg_first = uni(tab.cum[slot]);
            seg_end = uni(tab.cum[slot + 1]);
            seg_cur = slot >= n_hist;
            kstride = seg_cur ? (unsigned)Hkv * 256u : 256u;
            if (seg_cur)
                seg_k = ck + ((size_t)b * a.cur_len * Hkv + g) * 256;
            else if (PAGED)
                seg_tab = uni64(tab.off_k[slot]);
            else
                seg_k = kbase + ((size_t)uni64(tab.off_k[slot]) * Hkv + (size_t)g * seg_len) * 256;
            off_a = (unsigned)row_a * kstride + chunk_a;
            off_b = (unsigned)(row_a + 4) * kstride + chunk_b;
        };
        auto open_chunk = [&](int u) {  // of the open segment
            const int tok0 = (u - seg_first) * kChunkTokens;
            rows_left = seg_len - tok0;
            tile_k = seg_k + (size_t)tok0 * kstride;
        };
        // This wave's quarter (rows 8*wave .. +7) of the next key tile goes to the buffer at LDS address `buf_lds`;
        // afterwards the loader stands at the tile that follows.  Rows past the segment's end re-read its last row
        // (their scores are masked).
        auto load_tile = [&](unsigned buf_lds) {
            const unsigned kd = buf_lds + 8 * wave * 256;
            if (!seg_cur && PAGED) {
                const int tok0 = seg_len - rows_left;
                const int blk = min((tok0 >> 4) + (wave >> 1), (seg_len - 1) >> 4);
                const long long si = min(max(seg_tab + blk, 0ll), (long long)vw.max_blocks - 1);
                const int pb = max(uni(vw.block_table[(size_t)b * vw.max_blocks + si]), 0);
                const char* kb = kbase + ((size_t)pb * Hkv + g) * 4096;
                const int last_row = seg_len - 1 - blk * 16;
                const int r0 = min(8 * (wave & 1) + q4, last_row), r1 = min(8 * (wave & 1) + 4 + q4, last_row);
                load_to_lds(kb, (unsigned)r0 * 256u + chunk_a, kd);
                load_to_lds(kb, (unsigned)r1 * 256u + chunk_b, kd + 1024);
            } else if (rows_left >= kTileSP) {
                load_to_lds(tile_k, off_a, kd);
                load_to_lds(tile_k, off_b, kd + 1024);
            } else {
                load_to_lds(tile_k, (unsigned)min(row_a, rows_left - 1) * kstride + chunk_a, kd);
                load_to_lds(tile_k, (unsigned)min(row_a + 4, rows_left - 1) * kstride + chunk_b, kd + 1024);
            }
            rows_left -= kTileSP;
            tile_k += (size_t)kTileSP * kstride;
        };
        auto consume = [&](const char* buf, int tok0, int len, bool is_cur) {
            const bool full = !is_cur && (len - tok0 >= kTileSP);
            const uint4* kb = reinterpret_cast<const uint4*>(buf);
            floatx4_t sc[kNTS][2];
            uint4 kf[2][4];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) kf[h][kk] = kb[(h * 16 + n) * 16 + ((kk * 4 + q4 + n) & 15)];
            asm volatile("" ::: "memory");  // all eight fragment reads are in flight before the first product is issued
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)  // the four row tiles' chains interleaved: no instruction waits for the one before
#pragma unroll
                    for (int nt = 0; nt < kNTS; ++nt)
                        sc[nt][h] = mfma16(kf[h][kk], qf[nt][kk], kk ? sc[nt][h] : floatx4_t{0.f, 0.f, 0.f, 0.f});
            if (!full) {
#pragma unroll
                for (int nt = 0; nt < kNTS; ++nt) {
                    // tokens of this segment the row may see (causal inside the current round)
                    const int lim = is_cur ? cur_visible(len, q_len, min(row0 + nt * 16, rows_total - 1) / G) : len;
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (tok0 + h * 16 + q4 * 4 + i >= lim) sc[nt][h][i] = -__builtin_inff();
                }
            }
            float mx[kNTS];
            bool raise = false;
#pragma unroll
            for (int nt = 0; nt < kNTS; ++nt) {
                mx[nt] = max8(sc[nt][0], sc[nt][1]);
                raise |= mx[nt] > m[nt] + slack;
            }
            if (__any(raise)) {  // each lane keeps its own reference: the four lane groups of a row are merged per chunk
#pragma unroll
                for (int nt = 0; nt < kNTS; ++nt) {
                    const float m_new = vmax(m[nt], mx[nt]);
                    l[nt] *= fast_exp2((m[nt] - m_new) * a.c);
                    m[nt] = m_new;
                }
            }
#pragma unroll
            for (int nt = 0; nt < kNTS; ++nt) {
                const float mc = m[nt] * a.c;
                float p[8];
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i) p[h * 4 + i] = fast_exp2(__builtin_fmaf(sc[nt][h][i], a.c, -mc));
                l[nt] += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
            }
        };
        // End of chunk u: merge the four lane groups of every row, write the chunk's log-sum-exp, start afresh.
        auto finish_chunk = [&](int u) {
#pragma unroll
            for (int nt = 0; nt < kNTS; ++nt) {
                const float M = xrow_max4(m[nt]);
                float lv = l[nt] * fast_exp2((m[nt] - M) * a.c);
                lv = xrow_sum4(lv);
                const int row = row0 + nt * 16;
                if (row < rows_total && q4 == 0 && u < a.n_chunks_max) {  // (a caller that understated max_tokens loses chunks)
                    const int qtok = row / G;
                    const size_t rowid = ((size_t)b * a.Hq + (size_t)g * G + (row - qtok * G)) * q_len + qtok;  // [B][Hq][q_len]
                    a.part[rowid * a.n_chunks_max + u] =
                        lv > 0.f ? kLn2 * __builtin_fmaf(M, a.c, fast_log2(lv)) : -__builtin_inff();
                }
                m[nt] = kNegBig;
                l[nt] = 0.f;
            }
        };
        // ---- walk the key tiles of chunks [u_lo, u_hi): the whole workgroup in lockstep ------------------------
        int slot = find_slot(tab.cum, n_slots, u_lo);
        open_seg(slot);
        open_chunk(u_lo);
        int lu = u_lo, lj = 0;  // the tile the loader fetches next: tile lj of chunk lu
        int c_tok0 = seg_len - rows_left;
        load_tile(tiles_lds);
        int bufsel = 0;
        while (true) {
            char* buf = tiles + bufsel * kKTileBytes;
            wait_for_direct_loads();  // this wave's quarter of the tile has landed in LDS
            // the tile just stored, as the consumer needs it; it ends its chunk if the chunk or the segment ends
            const int c_len = seg_len, c_u = lu, c_t = c_tok0;
            const bool c_cur = seg_cur, c_last = lj + 1 == kTilesPerChunk || rows_left <= 0;
            __syncthreads();
            bool more = true;
            if (!c_last) {
                ++lj;
            } else {
                ++lu;
                lj = 0;
                more = lu < u_hi;
                if (more && lu >= seg_end) {
                    do ++slot; while (lu >= uni(tab.cum[slot + 1]));
                    open_seg(slot);
                    open_chunk(lu);
                }
            }
            if (more) {
                c_tok0 = seg_len - rows_left;
                load_tile(tiles_lds + (bufsel ^ 1) * kKTileBytes);
            }
            consume(buf, c_t, c_len, c_cur);
            if (c_last) finish_chunk(c_u);
            if (!more) break;
            bufsel ^= 1;
        }
    }
}


void launch_scores_plan(const ScoreArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(scores_plan_kernel, dim3(a.view.B), dim3(256), (size_t)(a.view.R_max + 2) * 2 * sizeof(int), st, a,
                       const_cast<char*>(a.plan));
}

int launch_scores_prefill_mfma(const ScoreArgs& a, bool paged, int num_cu, hipStream_t st) {
    const int G = a.Hq / a.view.Hkv;
    if (G > 16) return fail(RA_ERR_UNSUPPORTED, "round_scores: Hq / Hkv = %d exceeds 16", G);
    const int B = a.view.B, Hkv = a.view.Hkv;
    if (B > kMaxBatch) return fail(RA_ERR_UNSUPPORTED, "round_scores: batch %d exceeds %d", B, kMaxBatch);
    const int rows_total = a.q_len * G;
    const int n_rowblocks = (rows_total + kRowsPerItemS - 1) / kRowsPerItemS;
    const size_t smem = align_up(SlotTable::bytes(a.view.R_max + 1), 16) + 2 * kKTileBytes;
    long long max_pieces = (long long)B + (long long)B * a.n_chunks_max * kTilesPerChunk / a.min_units;
    if (max_pieces > (long long)B * a.S) max_pieces = (long long)B * a.S;
    long long grid = (long long)kWorkgroupsPerCuS * num_cu;
    if (grid > max_pieces * Hkv * n_rowblocks) grid = max_pieces * Hkv * n_rowblocks;
    if (grid < 1) grid = 1;
    if (paged)
        RA_LAUNCH_TIMED((scores_prefill_mfma_kernel<true>), dim3((unsigned)grid), dim3(256), smem, st, a, n_rowblocks);
    else
        RA_LAUNCH_TIMED((scores_prefill_mfma_kernel<false>), dim3((unsigned)grid), dim3(256), smem, st, a, n_rowblocks);
    return RA_OK;
}

}  // namespace ra
