// Round scores (paper Sec. 3.1, Eq. 1), streaming pass over the watershed layer's keys for bf16 /
// head_dim 128 on the matrix cores.  Same roles as in the attention kernel: the query rows of a KV
// head (query token i, head h of the group; row = i * G + h) are handled in tiles of 16, keys in
// tiles of 32 tokens, S^T[16 tokens x 16 rows] = K . Q^T with four mfma 16x16x32 per 16 tokens, and
// lane%16 is the query row, so the running (max, sum-exp) of a row stays in its lane.
//
// This kernel serves up to 16 query rows per KV head (decode, very short questions); more rows use the
// kernel that shares key tiles through LDS.
// Work item: (chunk c of 256 tokens, KV head g, sequence b) -> one log-sum-exp per row.  The four waves
// take two key tiles each, all loads issued up front, and are merged through LDS.  The keys come in as whole rows
// with non-temporal loads (this pass reads the whole layer once and should leave the caches alone) and reach the
// operand layout through an 8 KB strip of LDS per wave.
// Which round a chunk belongs to: a workgroup starts while the compute unit's vector memory queue is full of other
// workgroups' key tiles, so what it needs to find its round should not come through that queue.  In large launches
// it is a descriptor that a small kernel wrote beforehand and that arrives by one scalar load; for sequences of up
// to 32 rounds the rounds' lengths by scalar loads and a prefix sum over the lanes, with no kernel before; otherwise
// the sequence's table built in LDS from vector loads.
#include "scores_common.hpp"
#include "mfma_util.hpp"

namespace ra {

constexpr int kTileS = 32;
// Launches of at least this many workgroups (twice what the chip holds at once) read chunk descriptors: 732 -> 668
// microseconds on 4.3 GB of keys, 38.7 -> 33.8 on 199 MB; below it the descriptor kernel costs more than it saves.
constexpr long long kDescMinWorkgroups = 2048;
// ... and with few rounds, where a workgroup can find its round from scalar loads alone (about 0.1 microseconds of
// scalar work at every start, against 4 microseconds once for the descriptor kernel), only from here on
constexpr long long kDescMinWorkgroupsFewRounds = 32768;
// LDS that the large launches ask for and do not use: with it three workgroups fit a compute unit instead of four
// (34 + 12 KB each of 160 KB), which streams 1 % faster there (664-665 -> 657-660 microseconds on 4.3 GB of keys;
// two workgroups: 736, one: 1151).  The small launches, a few workgroups per slot in all, lose with it (34.6 -> 35.3).
constexpr size_t kDescLdsPad = 12 * 1024;
constexpr long long kDescPadMinWorkgroups = 16384;  // launches of at least this many workgroups get the padding

// A 32-token key tile on its way from memory: load j holds 16 bytes (chunk lane%16) of the row of token
// 4 j + lane/16, so that one load instruction reads four whole rows (eight whole cache lines).
struct KTile {
    uint4 r[8];
};

// Where chunk c of a sequence lies: written once per call by scores_chunks_kernel for the large launches, whose
// workgroups then start with one scalar load instead of building the sequence's table themselves.
struct ChunkDesc {
    long long off;  // the segment's offset in the store (tokens, or blocks when paged)
    int len;        // tokens of the segment
    int tok0_bits;  // first token of the chunk within the segment (a multiple of 256) | 1 current round | 2 exists
};
static_assert(sizeof(ChunkDesc) == 16, "one 16-byte scalar load");

// A load whose address is the same in every lane and whose memory no kernel of this launch writes: through the
// constant address space, so that it is a scalar load.  Scalar loads do not queue behind the compute unit's vector
// loads, which is where a workgroup of a saturated launch otherwise waits for its first table entry.
typedef const __attribute__((address_space(4))) u32x4_t* scalar_u32x4_ptr;
typedef const __attribute__((address_space(4))) int* scalar_int_ptr;
__device__ __forceinline__ uint4 load_uniform(const uint4* p) {
    const u32x4_t v = *(scalar_u32x4_ptr)(uintptr_t)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ int load_uniform(const int* p) { return *(scalar_int_ptr)(uintptr_t)p; }
typedef const __attribute__((address_space(4))) u32x2_t* scalar_u32x2_ptr;
__device__ __forceinline__ uint2 load_uniform(const uint2* p) {
    const u32x2_t v = *(scalar_u32x2_ptr)(uintptr_t)p;
    return make_uint2(v.x, v.y);
}

// The chunk table of sequence b in LDS (t_off, t_len, t_cum[n_slots + 1]); all threads of the workgroup call it.
__device__ __forceinline__ void build_chunk_table(const ScoreArgs& a, int b, int tid, long long* t_off, int* t_len,
                                                  int* t_cum, int& n_hist, int& n_slots) {
    const DevView& vw = a.view;
    // The first 256 table entries are asked for before the round count has arrived (entries past it are
    // dropped): one memory round trip instead of two at the start of every workgroup.
    int len0 = 0;
    long long off0 = 0;
    if (tid < vw.R_max) {
        len0 = vw.seg_len[(size_t)b * vw.R_max + tid];
        off0 = vw.seg_off[(size_t)b * vw.R_max + tid];
    }
    n_hist = min(max(vw.n_rounds[b], 0), vw.R_max);
    n_slots = n_hist + (a.cur_k && a.cur_len > 0 ? 1 : 0);
    for (int s = tid; s < n_slots; s += 256) {
        int len = a.cur_len;
        long long off = 0;
        if (s < n_hist) {
            len = max(s < 256 ? len0 : vw.seg_len[(size_t)b * vw.R_max + s], 0);
            off = s < 256 ? off0 : vw.seg_off[(size_t)b * vw.R_max + s];
        }
        t_len[s] = len;
        t_off[s] = off;
        t_cum[s] = chunks_of(len);
    }
    exclusive_scan_units(t_cum, n_slots);
}

// One workgroup per sequence: the descriptor of every chunk the launch has a workgroup for.
__global__ __launch_bounds__(256) void scores_chunks_kernel(ScoreArgs a, ChunkDesc* desc) {
    extern __shared__ __align__(16) char smem[];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int cap = a.view.R_max + 1;
    long long* t_off = reinterpret_cast<long long*>(smem);
    int* t_len = reinterpret_cast<int*>(t_off + cap);
    int* t_cum = t_len + cap;
    int n_hist, n_slots;
    build_chunk_table(a, b, tid, t_off, t_len, t_cum, n_hist, n_slots);
    const int total = n_slots > 0 ? t_cum[n_slots] : 0;
    for (int c = tid; c < a.n_chunks_max; c += 256) {
        ChunkDesc d = {0, 0, 0};
        if (c < total) {
            const int slot = find_slot(t_cum, n_slots, c);
            d.off = t_off[slot];
            d.len = t_len[slot];
            d.tok0_bits = (c - t_cum[slot]) * kChunkTokens | (slot >= n_hist ? 1 : 0) | 2;
        }
        desc[(size_t)b * a.n_chunks_max + c] = d;
    }
}

// How a workgroup finds its chunk's round
constexpr int kTableInLds = 0;    // the sequence's table built in LDS from vector loads (any number of rounds)
constexpr int kDescriptors = 1;   // one scalar load of what scores_chunks_kernel wrote (large launches)
constexpr int kTableScalar = 2;   // at most kScalarRounds rounds: their lengths by scalar loads, the prefix in
constexpr int kScalarRounds = 32; // scalar registers: no LDS, no barrier, no vector load, and no kernel before

template <bool PAGED, int TAB>
__global__ __launch_bounds__(256) void scores_mfma_kernel(ScoreArgs a) {
    constexpr bool DESC = TAB != kTableInLds;  // the table's loads go the scalar way
    extern __shared__ __align__(16) char smem[];
    __shared__ float sm[4][16], sl[4][16];
    __shared__ uint4 strip[4][512];  // per wave: one key tile, row-major, the 16-byte chunks of row r rotated by r
    const DevView& vw = a.view;
    const int Hkv = vw.Hkv;
    const int c = blockIdx.x, b = blockIdx.z;
    const int g = blockIdx.y % Hkv, rowblock = blockIdx.y / Hkv;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, n = lane & 15, q4 = lane >> 4;
    const int G = a.Hq / Hkv, q_len = a.q_len;
    const int rows_total = q_len * G;
    constexpr int NT = 1, RB = 16;

    // ---- which round does chunk c belong to? -------------------------------------------------------
    int len, chunk_tok0;
    long long off;
    bool is_cur;
    if constexpr (TAB == kTableScalar) {
        // Every length is asked for at once (the index clamped to the table, so nothing outside it is read) and
        // lands in lane s of one register; the current round's length goes to the lane after the history's.  A
        // prefix sum over the lanes' chunk counts then tells which lane's segment holds chunk c.
        const int n_hist = min(max(load_uniform(vw.n_rounds + b), 0), vw.R_max);
        int lens = 0;
#pragma unroll
        for (int s = 0; s < kScalarRounds; ++s) {
            const int v = load_uniform(vw.seg_len + (size_t)b * vw.R_max + min(s, vw.R_max - 1));
            lens = lane == s ? v : lens;
        }
        const bool use_cur = a.cur_k && a.cur_len > 0;
        const int mine = lane < n_hist ? max(lens, 0) : (lane == n_hist && use_cur ? a.cur_len : 0);
        const int nc = chunks_of(mine);
        // inclusive prefix over the lanes: shifts inside the rows of 16 lanes (zeros come in at a row's start), then
        // the totals of the rows before added from scalar registers -- no trip through LDS
        int incl = nc;
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x111, 0xf, 0xf, false);  // row_shr:1
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x112, 0xf, 0xf, false);  // row_shr:2
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x114, 0xf, 0xf, false);  // row_shr:4
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x118, 0xf, 0xf, false);  // row_shr:8
        {
            const int t0 = __builtin_amdgcn_readlane(incl, 15), t1 = __builtin_amdgcn_readlane(incl, 31),
                      t2 = __builtin_amdgcn_readlane(incl, 47);
            incl += lane < 16 ? 0 : (lane < 32 ? t0 : (lane < 48 ? t0 + t1 : t0 + t1 + t2));
        }
        const unsigned long long hit = __ballot(c >= incl - nc && c < incl);  // at most one lane
        if (hit == 0) return;
        const int slot = __ffsll((long long)hit) - 1;
        len = __builtin_amdgcn_readlane(mine, slot);
        chunk_tok0 = (c - __builtin_amdgcn_readlane(incl - nc, slot)) * kChunkTokens;
        is_cur = slot >= n_hist;
        off = 0;
        if (!is_cur) {
            const uint2 o = load_uniform(reinterpret_cast<const uint2*>(vw.seg_off + (size_t)b * vw.R_max + slot));
            off = (long long)(((unsigned long long)o.y << 32) | o.x);
        }
    } else if constexpr (TAB == kDescriptors) {
        const uint4 raw = load_uniform(reinterpret_cast<const uint4*>(a.chunks) + (size_t)b * a.n_chunks_max + c);
        if (!(raw.w & 2)) return;
        off = (long long)(((unsigned long long)raw.y << 32) | raw.x);
        len = (int)raw.z;
        is_cur = raw.w & 1;
        chunk_tok0 = (int)(raw.w & ~255u);
    } else {
        const int cap = vw.R_max + 1;
        long long* t_off = reinterpret_cast<long long*>(smem);
        int* t_len = reinterpret_cast<int*>(t_off + cap);
        int* t_cum = t_len + cap;
        int n_hist, n_slots;
        build_chunk_table(a, b, tid, t_off, t_len, t_cum, n_hist, n_slots);
        const int total = n_slots > 0 ? t_cum[n_slots] : 0;
        if (c >= total) return;
        const int slot = find_slot(t_cum, n_slots, c);
        len = t_len[slot];
        off = t_off[slot];
        is_cur = slot >= n_hist;
        chunk_tok0 = (c - t_cum[slot]) * kChunkTokens;
    }

    // ---- this wave's query rows -----------------------------------------------------------------------
    int lim[NT];
    bool row_ok[NT];
    size_t rowid[NT];
    uint4 qf[NT][4];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int row = rowblock * RB + nt * 16 + n;
        row_ok[nt] = row < rows_total;
        const int rr = row_ok[nt] ? row : 0;
        const int qtok = rr / G;
        rowid[nt] = ((size_t)b * a.Hq + (size_t)g * G + (rr - qtok * G)) * q_len + qtok;  // [B][Hq][q_len]
        const size_t qrow = ((size_t)b * q_len + qtok) * a.Hq + (size_t)g * G + (rr - qtok * G);
        const uint4* qp = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.q) + qrow * 256);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) qf[nt][kk] = row_ok[nt] ? qp[kk * 4 + q4] : make_uint4(0, 0, 0, 0);
        // tokens of this segment the row may see (causal inside the current round)
        lim[nt] = is_cur ? cur_visible(len, q_len, qtok) : len;
        if (!row_ok[nt]) lim[nt] = 0;
    }
    float m[NT], l[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m[nt] = kNegBig;
        l[nt] = 0.f;
    }

    const char* kbase = reinterpret_cast<const char*>(vw.k);
    // Whole rows per load instruction, non-temporal: every key is read once, and this pass, which streams the whole
    // watershed layer, then leaves the caches to what the next kernels need (segment tables, block tables).  Rows
    // past the segment's end re-read its last row (their scores are masked), so every address stays inside it.
    // Row t of a tile's half hh is at base[hh] + (t & mask) * pitch: one form for the current round, a contiguous
    // segment and the two blocks of a paged tile (the second one clamped to the segment's last block, as the rows
    // are), so that the load loop has no branches.  The block look-ups of both of the wave's tiles are made, for any
    // kind of segment and with clamped indices, before its first key load: they are in flight together, where a
    // look-up between the key loads would be waited for right there, one round trip per load instruction.
    struct TileBase {
        const char* base[2];
    };
    const long long pitch = is_cur ? (long long)Hkv * 256 : 256;
    const int mask = (PAGED && !is_cur) ? 15 : -1;
    auto bases_of = [&](const int (&tok0)[2], TileBase (&tb)[2]) {
        if constexpr (PAGED) {
            const int* bt[2][2];
            int pb[2][2];
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    long long si = off + (min(tok0[j] + 16 * hh, len - 1) >> 4);
                    si = si < 0 ? 0 : (si >= vw.max_blocks ? vw.max_blocks - 1 : si);
                    bt[j][hh] = vw.block_table + (size_t)b * vw.max_blocks + si;  // the same in all lanes
                }
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) pb[j][hh] = DESC ? load_uniform(bt[j][hh]) : *bt[j][hh];
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh)
                    tb[j].base[hh] = kbase + ((size_t)max(pb[j][hh], 0) * Hkv + g) * 16 * 256;
        } else {
#pragma unroll
            for (int j = 0; j < 2; ++j) tb[j].base[0] = tb[j].base[1] = kbase + ((size_t)off * Hkv + (size_t)g * len) * 256;
        }
        if (is_cur) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
                tb[j].base[0] = tb[j].base[1] =
                    reinterpret_cast<const char*>(a.cur_k) + ((size_t)b * a.cur_len * Hkv + g) * 256;
        }
    };
    auto issue = [&](int tok0, const TileBase& tb, KTile& t) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int tok = min(tok0 + 4 * j + q4, len - 1);
            const char* kp = tb.base[j >> 2] + (long long)(tok & mask) * pitch;
            t.r[j] = load_once(reinterpret_cast<const uint4*>(kp) + n);
        }
    };
    auto consume = [&](const KTile& t, int tok0) {
        const bool full = !is_cur && (len - tok0 >= kTileS);
        // through the wave's LDS strip into the operand layout: lane (n, q4) needs chunk kk*4 + q4 of row h*16 + n.
        // (Same wave: LDS operations complete in program order, so the next tile's writes follow these reads.)
        uint4* st = strip[wave];
#pragma unroll
        for (int j = 0; j < 8; ++j) st[(4 * j + q4) * 16 + ((n + 4 * j + q4) & 15)] = t.r[j];
        uint4 kf[2][4];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) kf[h][kk] = st[(h * 16 + n) * 16 + ((kk * 4 + q4 + n) & 15)];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            floatx4_t sc[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                sc[h] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) sc[h] = mfma16(kf[h][kk], qf[nt][kk], sc[h]);
            }
            if (!full) {
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (tok0 + h * 16 + q4 * 4 + i >= lim[nt]) sc[h][i] = -__builtin_inff();
            }
            const float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                                   fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
            // each lane keeps its own running max: the four lane groups of a row are merged at the end
            const float m_new = fmaxf(m[nt], mx);
            const float mc = m_new * a.c;
            float ps = 0.f;
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < 4; ++i) ps += fast_exp2(__builtin_fmaf(sc[h][i], a.c, -mc));
            // (m - m_new) * c, not fma(m, c, -mc): a lane that has seen no token yet keeps m = m_new = the finite
            // stand-in, and the fused form would then leave the rounding residue of its huge product in the exponent
            l[nt] = __builtin_fmaf(l[nt], fast_exp2((m[nt] - m_new) * a.c), ps);
            m[nt] = m_new;
        }
    };

    {
        KTile t[2];
        int tok0[2];
        TileBase tb[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) tok0[j] = chunk_tok0 + (j * 4 + wave) * kTileS;  // the four waves read adjacent tiles
        bases_of(tok0, tb);
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (tok0[j] < len) issue(tok0[j], tb[j], t[j]);
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (tok0[j] < len) consume(t[j], tok0[j]);
    }

    // ---- merge the four lane groups of every row
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const float M = xrow_max4(m[nt]);
        float lv = l[nt] * fast_exp2((m[nt] - M) * a.c);
        lv = xrow_sum4(lv);
        m[nt] = M;
        l[nt] = lv;
    }
    {
        if (q4 == 0) {
            sm[wave][n] = m[0];
            sl[wave][n] = l[0];
        }
        __syncthreads();
        if (tid < 16 && rowblock * RB + tid < rows_total) {
            const int r = tid;
            const float M = fmaxf(fmaxf(sm[0][r], sm[1][r]), fmaxf(sm[2][r], sm[3][r]));
            float den = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) den = __builtin_fmaf(sl[w][r], fast_exp2((sm[w][r] - M) * a.c), den);
            // wave 0's lanes 0..15 have q4 == 0 and n == tid, so rowid[0] is this row's index
            a.part[rowid[0] * a.n_chunks_max + c] =
                den > 0.f ? kLn2 * __builtin_fmaf(M, a.c, fast_log2(den)) : -__builtin_inff();
        }
    }
}


int launch_scores_mfma(const ScoreArgs& a, bool paged, int /*num_cu*/, hipStream_t st) {
    const int G = a.Hq / a.view.Hkv;
    if (G > 16) return fail(RA_ERR_UNSUPPORTED, "round_scores: Hq / Hkv = %d exceeds 16", G);
    const int rows_total = a.q_len * G;
    const size_t tab_bytes = (size_t)(a.view.R_max + 1) * 16 + 16;
    if (rows_total > 16) return fail(RA_ERR_UNSUPPORTED, "round_scores: %d query rows per KV head in the 16-row kernel", rows_total);
    const dim3 grid(a.n_chunks_max, a.view.Hkv, a.view.B);
    // From a few workgroups per slot of the chip on, a small kernel writes every chunk's descriptor first
    const long long n_wg = (long long)a.n_chunks_max * a.view.Hkv * a.view.B;
    if (a.chunks && n_wg >= (a.view.R_max <= kScalarRounds ? kDescMinWorkgroupsFewRounds : kDescMinWorkgroups)) {
        hipLaunchKernelGGL(scores_chunks_kernel, dim3(a.view.B), dim3(256), tab_bytes, st, a,
                           reinterpret_cast<ChunkDesc*>(a.chunks));
        const size_t pad = n_wg >= kDescPadMinWorkgroups ? kDescLdsPad : 0;
        if (paged)
            RA_LAUNCH_TIMED((scores_mfma_kernel<true, kDescriptors>), grid, dim3(256), pad, st, a);
        else
            RA_LAUNCH_TIMED((scores_mfma_kernel<false, kDescriptors>), grid, dim3(256), pad, st, a);
        return RA_OK;
    }
    if (a.view.R_max <= kScalarRounds) {
        if (paged)
            RA_LAUNCH_TIMED((scores_mfma_kernel<true, kTableScalar>), grid, dim3(256), 0, st, a);
        else
            RA_LAUNCH_TIMED((scores_mfma_kernel<false, kTableScalar>), grid, dim3(256), 0, st, a);
        return RA_OK;
    }
    if (paged)
        RA_LAUNCH_TIMED((scores_mfma_kernel<true, kTableInLds>), grid, dim3(256), tab_bytes, st, a);
    else
        RA_LAUNCH_TIMED((scores_mfma_kernel<false, kTableInLds>), grid, dim3(256), tab_bytes, st, a);
    return RA_OK;
}

}  // namespace ra
