// Round-sparse question-prefill attention on the matrix cores (paper Sec. 3.2 step 4), bf16 / head_dim 128.
//
// Same operand roles as the decode kernel (S^T = K.Q^T, O^T += V^T.P, query row = lane%16, P = hi + lo), but
// here a KV head has many query rows (q_len * G), so the key/value tiles are shared:
//   * a work item is (piece of the sequence's key tiles, KV head, block of 128 query rows); its four
//     waves own two 16-row tiles each and walk the key tiles in lockstep;
//   * every 32-token tile (8 KB of keys, 8 KB of transposed values) is fetched from global memory ONCE per
//     workgroup: while the previous tile is being consumed each wave requests a quarter of the next one with
//     loads that go from global memory straight into one of two LDS buffers (no registers, no LDS store
//     instructions; only the values of the current round, which are gathered token by token, and the values of
//     the fp16 mode, which are converted, pass through registers), and after one barrier all waves read the
//     operand fragments they need, 16 bytes per lane, conflict-free;
//   * with two buffers a single barrier per tile is enough: a wave can only write buffer X again after
//     the barrier that every wave passes once it has finished reading X.
// The launch is persistent with the balanced schedule of the decode kernel; pieces are merged by the same
// merge kernel.
//
// At the watershed layer the same pass also yields the round scores' raw material (TILE_LSE): one log-sum-exp
// per (query row, 256-token chunk of a round), the unit of the stand-alone score pass.  A row's running sum is
// never restarted for that: the chunk's share is the difference of the running sum between the chunk's ends (a
// mark that is rescaled together with the sum), exact to a few ulp of the sum, i.e. far below the 1e-5 the
// normalised scores are held to.  Pieces then begin and end on chunk boundaries, so that one piece owns a chunk.
//
// P_HALF (ra_set_prefill_precision, not the default): P goes to the matrix cores once, as fp16, instead of twice
// as hi + lo bf16.  The values are converted to fp16 on their way into LDS (a bf16 number is an fp16 number as
// long as its magnitude lies in [2^-14, 65504]; larger ones saturate, smaller ones lose low bits), P is kept in
// [2^-24, 2^15] by a softmax reference that lags the running maximum by at most 2^8 and a fixed scale of 2^7, it
// is rounded to fp16 (nearest even) and the SAME rounded values are summed for the normaliser (dot2 against ones,
// fp32 accumulate), so the rounding acts as a perturbation of the weights of at most 2^-12 each, of either sign,
// that averages out over the keys.  One third fewer matrix-core instructions per tile; the output error grows
// from about 2e-5 to about 4e-4 of the row's largest magnitude (contract: 2e-3).
#include "attn_common.hpp"
#include "mfma_util.hpp"
#include "stream_kv.hpp"

namespace ra {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ floatx4_t mfma16h(uint4 a, uint4 b, floatx4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
}
// Two floats -> packed fp16 pair (low half = a): by truncation, exact for numbers that fp16 holds ...
__device__ __forceinline__ uint32_t pack_half_rtz(float a, float b) {
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a, b));
}
// ... and rounded to nearest even (one v_cvt_pk_f16_f32): relative error <= 2^-12 in fp16's normal range.
__device__ __forceinline__ uint32_t pack_half_rne(float a, float b) {
    typedef float float2_t __attribute__((ext_vector_type(2)));
    const float2_t f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, half2_t));
}
// Four bf16 numbers -> the same four numbers as fp16 (exact inside fp16's normal range).
__device__ __forceinline__ uint2 bf16x4_to_half(uint2 x) {
    return make_uint2(pack_half_rtz(as_f32(x.x << 16), as_f32(x.x & 0xffff0000u)),
                      pack_half_rtz(as_f32(x.y << 16), as_f32(x.y & 0xffff0000u)));
}
constexpr int kHalfScaleLog2 = 7;  // P is carried as 2^7 x its value in the fp16 mode (see above)

constexpr int kTileP = 32;                      // tokens per key tile
constexpr int kNTP = 2;                         // 16-row tiles per wave
constexpr int kRowsPerItem = 4 * kNTP * 16;     // 128
constexpr int kTileBytes = 16384;               // 8 K fragments of 1 KB + 16 V fragments of 512 B
constexpr int kPiecesPerWorkgroupP = 4;

// A wave's quarter of a key/value tile on its way from global memory to LDS.
struct Share {
    uint4 v0, v1;  // V^T fragments dt = 2*wave, 2*wave + 1: tokens 8*(lane/16) .. +7 of channel dt*16 + lane%16
    bool pending;  // the values are in these registers (current round, or fp16 mode) and still have to go to LDS
};

template <bool PAGED, bool TILE_LSE, bool P_HALF>
__global__ __launch_bounds__(256, 2) void attn_prefill_mfma_kernel(AttnArgs a, int n_rowblocks) {
    extern __shared__ __align__(16) char smem[];
    __shared__ int sU[kMaxBatch], sps[kMaxBatch + 1];
    const DevView& vw = a.view;
    const int Hkv = vw.Hkv;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, n = lane & 15, q4 = lane >> 4;
    const int G = a.G, q_len = a.q_len;
    const int rows_total = q_len * G;

    const int cap = vw.R_max + 1;
    SlotTable tab;
    tab.carve(smem, cap);
    char* tiles = smem + ((SlotTable::bytes(cap) + 15) & ~(size_t)15);  // two tile buffers
    const unsigned tiles_lds = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lptr_t)tiles);
    int* ccum = reinterpret_cast<int*>(tiles + 2 * kTileBytes);        // [cap + 1] chunk prefix (score output only)

    const int inner = Hkv * n_rowblocks;
    const long long slots = ((long long)gridDim.x * kPiecesPerWorkgroupP + inner - 1) / inner;
    const int P = build_schedule(a.plan, cap, vw.B, a.S, a.min_units, slots, sU, sps);
    if (blockIdx.x == 0)
        for (int b = tid; b < vw.B; b += 256) a.n_parts[b] = sps[b + 1] - sps[b];

    const char* kbase = reinterpret_cast<const char*>(vw.k);
    const char* vbase = reinterpret_cast<const char*>(vw.v);
    const char* ck = reinterpret_cast<const char*>(a.cur_k);
    const char* cv = reinterpret_cast<const char*>(a.cur_v);
    const long long n_items = (long long)P * inner;

    for (long long item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int piece = (int)(item / inner);
        const int rest = (int)(item - (long long)piece * inner);
        const int g = rest % Hkv, rowblock = rest / Hkv;
        const int b = find_slot(sps, vw.B, piece);
        const int s = piece - sps[b];
        const int S_eff = sps[b + 1] - sps[b];
        const int U = sU[b];
        int u_lo = (int)(((long long)U * s) / S_eff);
        int u_hi = (int)(((long long)U * (s + 1)) / S_eff);

        __syncthreads();  // the previous item's readers of the table and the tile buffers are done
        const PlanHeader hdr = load_plan(a.plan + (size_t)b * plan_stride(cap), cap, tab);
        const int n_slots = __builtin_amdgcn_readfirstlane(hdr.n_slots), n_hist = __builtin_amdgcn_readfirstlane(hdr.n_hist);
        __syncthreads();
        if constexpr (TILE_LSE) {
            // chunk prefix of the sequence's segments (a chunk = 256 tokens = 8 tiles, never crossing a segment)
            for (int i = tid; i < cap; i += 256) ccum[i] = i < n_slots ? (tab.len[i] + 255) >> 8 : 0;
            exclusive_scan_units(ccum, cap);
            // a piece owns whole chunks: its ends move down to the chunk start at or before them
            auto snap = [&](int u) {
                if (u <= 0 || u >= U) return u <= 0 ? 0 : U;
                const int sl = find_slot(tab.cum, n_slots, u);
                return tab.cum[sl] + ((u - tab.cum[sl]) & ~7);
            };
            u_lo = __builtin_amdgcn_readfirstlane(snap(u_lo));
            u_hi = __builtin_amdgcn_readfirstlane(snap(u_hi));
        }

        // ---- this wave's query rows -------------------------------------------------------------------
        int qtok[kNTP];
        bool row_ok[kNTP];
        size_t rowid[kNTP];
        uint4 qf[kNTP][4];
#pragma unroll
        for (int nt = 0; nt < kNTP; ++nt) {
            const int row = rowblock * kRowsPerItem + wave * kNTP * 16 + nt * 16 + n;
            row_ok[nt] = row < rows_total;
            const int rr = row_ok[nt] ? row : 0;
            qtok[nt] = rr / G;
            rowid[nt] = ((size_t)b * q_len + qtok[nt]) * a.Hq + (size_t)g * G + (rr - qtok[nt] * G);
            const uint4* qp = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(a.q) + rowid[nt] * 256);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) qf[nt][kk] = row_ok[nt] ? qp[kk * 4 + q4] : make_uint4(0, 0, 0, 0);
        }
        floatx4_t acc[kNTP][8];
        float m[kNTP], l[kNTP];
        float l_mark[kNTP];  // the running sum as it stood at the start of the current chunk (score output only)
        const float slack = (P_HALF ? 8.f : 16.f) / a.c;
#pragma unroll
        for (int nt = 0; nt < kNTP; ++nt) {
            m[nt] = kNegBig;
            l[nt] = 0.f;
            l_mark[nt] = 0.f;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) acc[nt][dt] = floatx4_t{0.f, 0.f, 0.f, 0.f};
        }

        // Uniform state of the loader: the segment it stands in (the table in LDS is only read on entry) and,
        // inside it, the next tile: the addresses of its first token's keys and of its first V^T block (head g)
        // and the tokens left from there.  A tile's addresses then cost a handful of scalar operations.
        int seg_len = 0, seg_first = 0, seg_end = 0, rows_left = 0;
        bool seg_cur = false;
        const char *seg_k = nullptr, *seg_v = nullptr;  // contiguous history / current round: token 0 of head g
        const char *tile_k = nullptr, *tile_v = nullptr;
        long long seg_tab = 0;                          // paged history: first block-table slot
        unsigned kstride = 256;                         // bytes from one token's keys to the next
        // Direct loads: 16 bytes per lane, lane L's piece landing at (destination + 16 L).  Keys: the tile's LDS
        // image is row-major, 256 bytes per row, row rho = 16 h + r being row r of the operand of half h, i.e. token
        // 8 (r / 4) + 4 h + r % 4 of the tile (which makes a lane's eight probabilities eight consecutive tokens),
        // and inside a row the 16-byte chunk x sits at position (x + r) mod 16: the rotation lets the operand reads
        // (16 lanes = 16 rows, one chunk) touch every bank once.  This wave fills rows 8 wave .. + 7 with two loads
        // of four whole rows each: 16 lanes per row, so the global side is as coalesced as a plain row copy.
        int k_tok[2];       // token (inside the tile) of the row this lane helps to load, for the two loads
        unsigned k_chunk[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int rho = 8 * wave + 4 * j + q4, h = rho >> 4, r = rho & 15;
            k_tok[j] = 8 * (r >> 2) + 4 * h + (r & 3);
            k_chunk[j] = (unsigned)((n - r) & 15) * 16u;
        }
        unsigned off_k[2] = {0, 0};                     // byte offsets from tile_k for a full tile
        // V^T: tokens 8 * q4 .. + 7 of channel dt * 16 + n: block q4 / 2 of the tile, 16 contiguous bytes
        const unsigned off_v = (unsigned)((2 * wave * 16 + n) * 32 + (q4 & 1) * 16);
        auto uni = [](int x) { return __builtin_amdgcn_readfirstlane(x); };
        auto uni64 = [&](long long x) { return ((long long)uni((int)(x >> 32)) << 32) | (unsigned)uni((int)x); };
        auto open_seg = [&](int slot, int u) {  // ... and stand at its tile u - first
            seg_len = uni(tab.len[slot]);
            seg_first = uni(tab.cum[slot]);
            seg_end = uni(tab.cum[slot + 1]);
            seg_cur = slot >= n_hist;
            kstride = seg_cur ? (unsigned)Hkv * 256u : 256u;
            if (seg_cur) {
                seg_k = ck + ((size_t)b * a.cur_cap * Hkv + g) * 256;
                seg_v = cv + ((size_t)b * a.cur_cap * Hkv + g) * 256;
            } else if (PAGED) {
                seg_tab = uni64(tab.off_k[slot]);
            } else {
                seg_k = kbase + ((size_t)uni64(tab.off_k[slot]) * Hkv + (size_t)g * seg_len) * 256;
                seg_v = vbase + ((size_t)uni64(tab.off_v[slot]) * Hkv + (size_t)g * ((seg_len + 15) & ~15)) * 256;
            }
            off_k[0] = (unsigned)k_tok[0] * kstride + k_chunk[0];
            off_k[1] = (unsigned)k_tok[1] * kstride + k_chunk[1];
            const int uin = u - seg_first;
            rows_left = seg_len - uin * kTileP;
            tile_k = seg_k + (size_t)uin * kTileP * kstride;
            tile_v = seg_v + (size_t)uin * 8192;
        };
        // This wave's quarter of the next tile goes to `buf`: two K fragments and two V^T fragments.  Keys and the
        // values of history rounds travel from global memory straight into LDS; the values of the current round
        // (token-major: gathered with 2-byte loads) and, in the fp16 mode, all values (converted on the way) pass
        // through registers and are written by store_share at the top of the next iteration.  Rows and blocks past
        // the segment's end re-read its last ones (their scores are masked).  Afterwards the loader stands at the
        // tile that follows.
        auto load_tile = [&](unsigned buf_lds) -> Share {
            Share sh;
            sh.pending = false;
            sh.v0 = sh.v1 = make_uint4(0, 0, 0, 0);
            const int tok0 = seg_len - rows_left;
            const unsigned kd = buf_lds + 8 * wave * 256, vd = buf_lds + 8192 + 2 * wave * 1024;
            if (!seg_cur && PAGED) {
                const int blk0 = tok0 >> 4, blk1 = min(blk0 + 1, (seg_len - 1) >> 4);
                const long long last = vw.max_blocks - 1;
                const long long s0 = min(max(seg_tab + blk0, 0ll), last), s1 = min(max(seg_tab + blk1, 0ll), last);
                const int p0 = max(uni(vw.block_table[(size_t)b * vw.max_blocks + s0]), 0);
                const int p1 = max(uni(vw.block_table[(size_t)b * vw.max_blocks + s1]), 0);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const bool upper = k_tok[j] >> 4;
                    const int last_row = seg_len - 1 - (upper ? blk1 : blk0) * 16;
                    const char* kb = kbase + ((size_t)(upper ? p1 : p0) * Hkv + g) * 4096;
                    load_to_lds(kb + min(k_tok[j] & 15, last_row) * 256 + k_chunk[j], kd + j * 1024);
                }
                const char* vb = vbase + ((size_t)((q4 >> 1) ? p1 : p0) * Hkv + g) * 4096;
                if constexpr (P_HALF) {
                    sh.v0 = *reinterpret_cast<const uint4*>(vb + off_v);
                    sh.v1 = *reinterpret_cast<const uint4*>(vb + off_v + 512);
                    sh.pending = true;
                } else {
                    load_to_lds(vb + off_v, vd);
                    load_to_lds(vb + off_v + 512, vd + 1024);
                }
            } else {
                if (rows_left >= kTileP) {
                    load_to_lds(tile_k, off_k[0], kd);
                    load_to_lds(tile_k, off_k[1], kd + 1024);
                } else {
                    load_to_lds(tile_k, (unsigned)min(k_tok[0], rows_left - 1) * kstride + k_chunk[0], kd);
                    load_to_lds(tile_k, (unsigned)min(k_tok[1], rows_left - 1) * kstride + k_chunk[1], kd + 1024);
                }
                if (seg_cur) {  // token-major values: gather 8 tokens of one channel with 2-byte loads
                    auto gather = [&](int dt) {
                        uint32_t e[8];
#pragma unroll
                        for (int t = 0; t < 8; ++t) {
                            const int tok = min(tok0 + q4 * 8 + t, seg_len - 1);
                            e[t] = *reinterpret_cast<const unsigned short*>(seg_v + (size_t)tok * kstride + (dt * 16 + n) * 2);
                        }
                        return make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
                    };
                    sh.v0 = gather(2 * wave);
                    sh.v1 = gather(2 * wave + 1);
                    sh.pending = true;
                } else {
                    const unsigned second = (q4 >> 1) && rows_left > 16 ? 4096u : 0u;  // the tile's second 16-token block, if any
                    if constexpr (P_HALF) {
                        sh.v0 = *reinterpret_cast<const uint4*>(tile_v + (off_v + second));
                        sh.v1 = *reinterpret_cast<const uint4*>(tile_v + (off_v + second + 512));
                        sh.pending = true;
                    } else {
                        load_to_lds(tile_v, off_v + second, vd);
                        load_to_lds(tile_v, off_v + second + 512, vd + 1024);
                    }
                }
            }
            rows_left -= kTileP;
            tile_k += (size_t)kTileP * kstride;
            tile_v += 8192;
            return sh;
        };
        // V^T fragment dt holds lane L's 16 bytes at (8192 + dt*1024 + 16*L).
        auto store_share = [&](char* buf, const Share& sh) {  // the values that came through registers
            if (!sh.pending) return;
            uint4* vd = reinterpret_cast<uint4*>(buf + 8192) + 2 * wave * 64 + lane;
            if constexpr (P_HALF) {
                const uint2 a0 = bf16x4_to_half(make_uint2(sh.v0.x, sh.v0.y)), a1 = bf16x4_to_half(make_uint2(sh.v0.z, sh.v0.w));
                const uint2 b0 = bf16x4_to_half(make_uint2(sh.v1.x, sh.v1.y)), b1 = bf16x4_to_half(make_uint2(sh.v1.z, sh.v1.w));
                vd[0] = make_uint4(a0.x, a0.y, a1.x, a1.y);
                vd[64] = make_uint4(b0.x, b0.y, b1.x, b1.y);
            } else {
                vd[0] = sh.v0;
                vd[64] = sh.v1;
            }
        };
        auto consume = [&](const char* buf, int tok0, int len, bool is_cur) {
            const bool full = !is_cur && (len - tok0 >= kTileP);
            const uint4* kb = reinterpret_cast<const uint4*>(buf);
            const uint4* vb = reinterpret_cast<const uint4*>(buf + 8192);
            uint4 kf[2][4];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) kf[h][kk] = kb[(h * 16 + n) * 16 + ((kk * 4 + q4 + n) & 15)];
            floatx4_t sc[kNTP][2];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)  // four independent chains interleaved: no instruction waits for the one before
#pragma unroll
                for (int nt = 0; nt < kNTP; ++nt)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        sc[nt][h] = mfma16(kf[h][kk], qf[nt][kk], kk ? sc[nt][h] : floatx4_t{0.f, 0.f, 0.f, 0.f});
            if (!full) {
#pragma unroll
                for (int nt = 0; nt < kNTP; ++nt) {
                    // tokens this row may see: the segment's length, or inside the current round the causal limit
                    int lim = len;
                    if (is_cur) lim = min(len, max(len - q_len + qtok[nt] + 1, 0));
                    if (!row_ok[nt]) lim = 0;
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (tok0 + q4 * 8 + h * 4 + i >= lim) sc[nt][h][i] = -__builtin_inff();
                }
            }
            // The reference logit m of a row is only raised when some logit exceeds it by more than `slack`
            // (2^16 after scaling), which a lane can tell from its own eight logits: the common tile has no
            // cross-lane traffic and no rescale, and P stays far inside the fp32 / bf16 range.
            float mx[kNTP];
            bool raise = false;
#pragma unroll
            for (int nt = 0; nt < kNTP; ++nt) {
                mx[nt] = max8(sc[nt][0], sc[nt][1]);
                raise |= mx[nt] > m[nt] + slack;
            }
            if (__any(raise)) {
#pragma unroll
                for (int nt = 0; nt < kNTP; ++nt) {
                    const float r = xrow_max4(mx[nt]);
                    const float m_new = vmax(m[nt], r);
                    const float alpha = fast_exp2((m[nt] - m_new) * a.c);
                    l[nt] *= alpha;
                    if constexpr (TILE_LSE) l_mark[nt] *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt) acc[nt][dt] *= alpha;
                    m[nt] = m_new;
                }
            }
            uint4 vf[8];  // V^T operand fragments of the tile, shared by both row tiles
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) vf[dt] = vb[dt * 64 + lane];
            auto probabilities = [&](int nt, uint4& phi, uint4& plo) {  // P (hi + lo, or fp16) of row tile nt, and its row sums
                const float mc = m[nt] * a.c - (P_HALF ? (float)kHalfScaleLog2 : 0.f);
                float p[8];
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i) p[h * 4 + i] = fast_exp2(__builtin_fmaf(sc[nt][h][i], a.c, -mc));
                if constexpr (P_HALF) {
                    phi.x = pack_half_rne(p[0], p[1]);
                    phi.y = pack_half_rne(p[2], p[3]);
                    phi.z = pack_half_rne(p[4], p[5]);
                    phi.w = pack_half_rne(p[6], p[7]);
                    const half2_t ones = {(_Float16)1.0f, (_Float16)1.0f};
                    float ps = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, phi.x), ones, 0.f, false);
                    ps = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, phi.y), ones, ps, false);
                    ps = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, phi.z), ones, ps, false);
                    ps = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, phi.w), ones, ps, false);
                    l[nt] += ps;  // the rounded values, the ones the products use
                    plo = phi;
                } else {
                    const float ps = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
                    l[nt] += ps;
                    phi.x = pack_hi16(p[0], p[1]);
                    phi.y = pack_hi16(p[2], p[3]);
                    phi.z = pack_hi16(p[4], p[5]);
                    phi.w = pack_hi16(p[6], p[7]);
                    plo.x = pack_hi16(p[0] - trunc_bf16(p[0]), p[1] - trunc_bf16(p[1]));
                    plo.y = pack_hi16(p[2] - trunc_bf16(p[2]), p[3] - trunc_bf16(p[3]));
                    plo.z = pack_hi16(p[4] - trunc_bf16(p[4]), p[5] - trunc_bf16(p[5]));
                    plo.w = pack_hi16(p[6] - trunc_bf16(p[6]), p[7] - trunc_bf16(p[7]));
                }
            };
            auto accumulate = [&](int nt, const uint4& phi, const uint4& plo) {
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) {
                    if constexpr (P_HALF) {
                        acc[nt][dt] = mfma16h(vf[dt], phi, acc[nt][dt]);
                    } else {
                        acc[nt][dt] = mfma16(vf[dt], phi, acc[nt][dt]);
                        acc[nt][dt] = mfma16(vf[dt], plo, acc[nt][dt]);
                    }
                }
            };
            // Row tile by row tile: the first tile's products can run on the matrix cores while the vector ALU
            // turns the second tile's logits into probabilities.
            uint4 phi0, plo0, phi1, plo1;
            probabilities(0, phi0, plo0);
            accumulate(0, phi0, plo0);
            probabilities(1, phi1, plo1);
            accumulate(1, phi1, plo1);
        };

        // ---- walk the key tiles: the whole workgroup in lockstep -----------------------------------------
        if (u_lo < u_hi) {
            int slot = find_slot(tab.cum, n_slots, u_lo);
            open_seg(slot, u_lo);
            int c_tok0 = seg_len - rows_left;
            Share sh = load_tile(tiles_lds);
            int bufsel = 0;
            for (int u = u_lo; u < u_hi; ++u) {
                char* buf = tiles + bufsel * kTileBytes;
                store_share(buf, sh);
                wait_for_direct_loads();  // this wave's quarter of the tile has landed in LDS
                const int len = seg_len, tok0 = c_tok0;  // of the tile just stored
                const bool is_cur = seg_cur;
                const int t_slot = slot, t_first = seg_first, t_end = seg_end;
                __syncthreads();
                if (u + 1 < u_hi) {
                    if (u + 1 >= seg_end) {
                        do ++slot; while (u + 1 >= uni(tab.cum[slot + 1]));
                        open_seg(slot, u + 1);
                    }
                    c_tok0 = seg_len - rows_left;
                    sh = load_tile(tiles_lds + (bufsel ^ 1) * kTileBytes);
                }
                consume(buf, tok0, len, is_cur);
                if constexpr (TILE_LSE) {
                    const int uin = u - t_first;
                    if ((uin & 7) == 7 || u + 1 == t_end || u + 1 == u_hi) {  // the chunk ends with this tile
                        const int chunk = ccum[t_slot] + (uin >> 3);
#pragma unroll
                        for (int nt = 0; nt < kNTP; ++nt) {
                            const float share = xrow_sum4(l[nt] - l_mark[nt]);
                            l_mark[nt] = l[nt];
                            if (q4 == 0 && row_ok[nt] && chunk < a.n_tiles_max) {
                                // row order of the score pass: [B][Hq][q_len]
                                const size_t head = rowid[nt] - ((size_t)b * q_len + qtok[nt]) * a.Hq;
                                const size_t srow = ((size_t)b * a.Hq + head) * q_len + qtok[nt];
                                a.tile_lse[srow * a.n_tiles_max + chunk] =
                                    share > 0.f ? kLn2 * (__builtin_fmaf(m[nt], a.c, fast_log2(share)) -
                                                          (P_HALF ? (float)kHalfScaleLog2 : 0.f))
                                                : -__builtin_inff();
                            }
                        }
                    }
                }
                bufsel ^= 1;
            }
        }

        // ---- the four lane groups hold partial sums of the same rows; each wave owns its rows ------------------
#pragma unroll
        for (int nt = 0; nt < kNTP; ++nt) {
            l[nt] = xrow_sum4(l[nt]);
            if constexpr (P_HALF) {  // take the fixed scale of P out again (a power of two: exact)
                constexpr float unscale = 1.f / (float)(1 << kHalfScaleLog2);
                l[nt] *= unscale;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) acc[nt][dt] *= unscale;
            }
            if (!row_ok[nt]) continue;
            if (S_eff > 1) {
                const size_t pr = rowid[nt] * a.S + s;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt)
                    *reinterpret_cast<floatx4_t*>(a.part_acc + pr * 128 + dt * 16 + q4 * 4) = acc[nt][dt];
                if (q4 == 0) {
                    a.part_m[pr] = m[nt];
                    a.part_l[pr] = l[nt];
                }
            } else {
                const float inv = l[nt] > 0.f ? 1.f / l[nt] : 0.f;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt)
                    *reinterpret_cast<floatx4_t*>(a.out + rowid[nt] * 128 + dt * 16 + q4 * 4) = acc[nt][dt] * inv;
                if (a.lse && q4 == 0)
                    a.lse[rowid[nt]] =
                        l[nt] > 0.f ? __builtin_fmaf(m[nt], a.scale, __builtin_logf(l[nt])) : -__builtin_inff();
            }
        }
    }
}


int launch_attn_prefill_mfma(const AttnArgs& a, bool paged, int num_cu, hipStream_t st) {
    const int rows_total = a.q_len * a.G;
    const int B = a.view.B, Hkv = a.view.Hkv;
    if (a.G > 16) return fail(RA_ERR_UNSUPPORTED, "prefill: Hq / Hkv = %d exceeds 16", a.G);
    if (B > kMaxBatch) return fail(RA_ERR_UNSUPPORTED, "prefill: batch %d exceeds %d", B, kMaxBatch);
    const int n_rowblocks = (rows_total + kRowsPerItem - 1) / kRowsPerItem;
    const size_t smem = align_up(SlotTable::bytes(a.view.R_max + 1), 16) + 2 * kTileBytes +
                        (a.tile_lse ? (size_t)(a.view.R_max + 3) * sizeof(int) : 0);
    const long long max_tiles = (long long)B * (a.max_tokens / kTileP + a.view.R_max + 1 + a.cur_cap / kTileP + 1);
    long long max_pieces = (long long)B + max_tiles / a.min_units;
    if (max_pieces > (long long)B * a.S) max_pieces = (long long)B * a.S;
    long long grid = (long long)2 * num_cu;
    if (grid > max_pieces * Hkv * n_rowblocks) grid = max_pieces * Hkv * n_rowblocks;
    if (grid < 1) grid = 1;
    const bool lse = a.tile_lse != nullptr, half = a.p_half != 0;
#define RA_PREFILL_CASE(P_, L_, H_)                                                                                  \
    if (paged == P_ && lse == L_ && half == H_) {                                                                    \
        RA_LAUNCH_TIMED((attn_prefill_mfma_kernel<P_, L_, H_>), dim3((unsigned)grid), dim3(256), smem, st, a, n_rowblocks); \
        return RA_OK;                                                                                                \
    }
    RA_PREFILL_CASE(false, false, false) RA_PREFILL_CASE(false, true, false) RA_PREFILL_CASE(true, false, false)
    RA_PREFILL_CASE(true, true, false) RA_PREFILL_CASE(false, false, true) RA_PREFILL_CASE(false, true, true)
    RA_PREFILL_CASE(true, false, true) RA_PREFILL_CASE(true, true, true)
#undef RA_PREFILL_CASE
    return RA_OK;
}

}  // namespace ra
