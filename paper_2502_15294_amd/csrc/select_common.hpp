// Round selection (paper Sec. 3.3) for one sequence by one workgroup, on a score vector that already lies in LDS.
// Shared by the stand-alone selection kernel and by the score pass's finishing kernel when a call asks for the
// scores and the selection together.
//
// Every strategy reduces to "keep the n best rounds" (higher score first, then lower index):
//   ADAPTIVE / THRESHOLD  n = number of scores above the cut (those are exactly the n best)
//   TOP_FRACTION          n = ceil(fraction * R)
// then n is clamped by min_rounds / max_rounds.  Ranks are found by counting in LDS, the kept rounds are
// compacted in ascending order with wavefront ballots and a prefix over the waves.
// keep_first / keep_last (an optional policy, not the paper's) add the first and the most recent rounds to
// whatever the rule kept; the rule itself is evaluated as without them.
#pragma once

#include "common.hpp"

namespace ra {

// The cut of the adaptive rule in IEEE double, sums taken sequentially in round order with separate
// multiply and add (no contraction), so that a host reference doing the same steps gets the same bits.
#pragma clang fp contract(off)
__device__ static double adaptive_cut(const float* s, int R, double lambda, int ddof) {
    double total = 0.0;
    for (int r = 0; r < R; ++r) total = total + (double)s[r];
    const double mean = total / (double)R;
    double ss = 0.0;
    for (int r = 0; r < R; ++r) {
        const double dev = (double)s[r] - mean;
        ss = ss + dev * dev;
    }
    const int den = R - ddof;
    const double sd = den > 0 ? __builtin_sqrt(ss / (double)den) : 0.0;
    return mean + lambda * sd;
}

// LDS a workgroup of NW waves needs for the selection, beside the score vector itself.
template <int NW>
struct SelectShared {
    double cut;
    int wave_cnt[NW];
    int n_pass;
};

// s[0..R): the sequence's scores in LDS (complete: a barrier lies between their last write and this call).
// out[0..R_max): the sequence's row of sel_idx; *n_sel_out: its count.  Must be called by all NW * 64 threads.
template <int NW>
__device__ void select_rounds_block(const float* s, int R, int R_max, const ra_select_params& p, int32_t* out,
                                    int32_t* n_sel_out, SelectShared<NW>& sh) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    constexpr int NT = NW * 64;
    for (int r = tid; r < R_max; r += NT) out[r] = -1;
    if (tid == 0) sh.n_pass = 0;
    __syncthreads();
    if (R == 0) {
        if (tid == 0) *n_sel_out = 0;
        return;
    }
    int n_keep;
    if (p.strategy == RA_SEL_TOP_FRACTION) {
        const double want = __builtin_ceil(p.fraction * (double)R);
        n_keep = want < 1.0 ? 1 : (want > (double)R ? R : (int)want);
    } else {
        if (tid == 0) sh.cut = p.strategy == RA_SEL_ADAPTIVE ? adaptive_cut(s, R, p.lambda, p.ddof) : p.threshold;
        __syncthreads();
        const double cut = sh.cut;
        int cnt = 0;
        for (int r = tid; r < R; r += NT) cnt += ((double)s[r] > cut) ? 1 : 0;
        for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
        if (lane == 0) atomicAdd(&sh.n_pass, cnt);  // integer sum: order does not matter
        __syncthreads();
        n_keep = sh.n_pass;
    }
    if (n_keep < p.min_rounds) n_keep = p.min_rounds;
    if (p.max_rounds > 0 && n_keep > p.max_rounds) n_keep = p.max_rounds;
    if (n_keep > R) n_keep = R;

    // keep[r] <=> rank(r) < n_keep, rank = number of rounds preferred over r
    int base = 0;
    for (int r0 = 0; r0 < R; r0 += NT) {
        const int r = r0 + tid;
        bool keep = false;
        if (r < R) {
            const float x = s[r];
            int rank = 0;
            for (int j = 0; j < R; ++j) {
                const float y = s[j];
                rank += (y > x || (y == x && j < r)) ? 1 : 0;
            }
            keep = rank < n_keep || r < p.keep_first || r >= R - p.keep_last;
        }
        const unsigned long long mask = __ballot(keep);
        if (lane == 0) sh.wave_cnt[wave] = __popcll(mask);
        __syncthreads();
        int before = base, all = 0;
        for (int w = 0; w < NW; ++w) {
            if (w < wave) before += sh.wave_cnt[w];
            all += sh.wave_cnt[w];
        }
        if (keep) out[before + __popcll(mask & ((1ull << lane) - 1ull))] = r;
        base += all;
        __syncthreads();
    }
    if (tid == 0) *n_sel_out = base;
}

// Host-side check of the selection parameters shared by the entry points; `who` prefixes the error text.
int check_select_params(const ra_select_params* params, const char* who);

}  // namespace ra
