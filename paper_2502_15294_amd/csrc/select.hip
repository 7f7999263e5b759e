// Round selection (paper Sec. 3.3): from the per-sequence round scores choose the rounds whose KV
// the post-watershed layers will attend over.  One workgroup per sequence; the score vector lives in
// LDS.  Every strategy reduces to "keep the n best rounds" (higher score first, then lower index):
//   ADAPTIVE / THRESHOLD  n = number of scores above the cut (those are exactly the n best)
//   TOP_FRACTION          n = ceil(fraction * R)
// then n is clamped by min_rounds / max_rounds.  Ranks are found by counting in LDS, the kept rounds
// are compacted in ascending order with wavefront ballots and a prefix over the four waves.
// keep_first / keep_last (an optional policy, not the paper's) add the first and the most recent
// rounds to whatever the rule kept; the rule itself is evaluated as without them.
#include "common.hpp"

namespace ra {

struct SelectArgs {
    const float* scores;
    const int32_t* n_rounds;
    int R_max;
    ra_select_params p;
    int32_t* sel_idx;
    int32_t* n_sel;
};

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

__global__ __launch_bounds__(256) void select_kernel(SelectArgs a) {
    __shared__ float s[kMaxRounds];
    __shared__ double cut_sh;
    __shared__ int wave_cnt[4];
    __shared__ int n_pass_sh;
    const int b = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int R = min(max(a.n_rounds[b], 0), a.R_max);
    int32_t* out = a.sel_idx + (size_t)b * a.R_max;
    for (int r = tid; r < a.R_max; r += 256) {
        const float v = a.scores[(size_t)b * a.R_max + r];  // asked for before the round count has arrived
        if (r < R) s[r] = v;
        out[r] = -1;
    }
    if (tid == 0) n_pass_sh = 0;
    __syncthreads();
    if (R == 0) {
        if (tid == 0) a.n_sel[b] = 0;
        return;
    }

    int n_keep;
    if (a.p.strategy == RA_SEL_TOP_FRACTION) {
        const double want = __builtin_ceil(a.p.fraction * (double)R);
        n_keep = want < 1.0 ? 1 : (want > (double)R ? R : (int)want);
    } else {
        if (tid == 0) cut_sh = a.p.strategy == RA_SEL_ADAPTIVE ? adaptive_cut(s, R, a.p.lambda, a.p.ddof) : a.p.threshold;
        __syncthreads();
        const double cut = cut_sh;
        int cnt = 0;
        for (int r = tid; r < R; r += 256) cnt += ((double)s[r] > cut) ? 1 : 0;
        for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
        if (lane == 0) atomicAdd(&n_pass_sh, cnt);  // integer sum: order does not matter
        __syncthreads();
        n_keep = n_pass_sh;
    }
    if (n_keep < a.p.min_rounds) n_keep = a.p.min_rounds;
    if (a.p.max_rounds > 0 && n_keep > a.p.max_rounds) n_keep = a.p.max_rounds;
    if (n_keep > R) n_keep = R;

    // keep[r] <=> rank(r) < n_keep, rank = number of rounds preferred over r
    int base = 0;
    for (int r0 = 0; r0 < R; r0 += 256) {
        const int r = r0 + tid;
        bool keep = false;
        if (r < R) {
            const float x = s[r];
            int rank = 0;
            for (int j = 0; j < R; ++j) {
                const float y = s[j];
                rank += (y > x || (y == x && j < r)) ? 1 : 0;
            }
            keep = rank < n_keep || r < a.p.keep_first || r >= R - a.p.keep_last;
        }
        const unsigned long long mask = __ballot(keep);
        if (lane == 0) wave_cnt[wave] = __popcll(mask);
        __syncthreads();
        int before = base;
        for (int w = 0; w < wave; ++w) before += wave_cnt[w];
        if (keep) out[before + __popcll(mask & ((1ull << lane) - 1ull))] = r;
        base += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
        __syncthreads();
    }
    if (tid == 0) a.n_sel[b] = base;
}

}  // namespace ra

using namespace ra;

extern "C" int ra_select_rounds(ra_ctx* ctx, void* stream, const float* scores, const int32_t* n_rounds, int B,
                                int R_max, const ra_select_params* params, int32_t* sel_idx, int32_t* n_sel) {
    RA_REQUIRE(ctx != nullptr, RA_ERR_INVALID_ARG, "select_rounds: ctx is NULL");
    RA_REQUIRE(scores && n_rounds && params && sel_idx && n_sel, RA_ERR_INVALID_ARG, "select_rounds: NULL argument");
    RA_REQUIRE(B > 0 && R_max > 0, RA_ERR_INVALID_ARG, "select_rounds: B and R_max must be positive");
    RA_REQUIRE(R_max <= kMaxRounds, RA_ERR_UNSUPPORTED, "select_rounds: R_max %d exceeds %d", R_max, kMaxRounds);
    RA_REQUIRE(params->strategy >= RA_SEL_ADAPTIVE && params->strategy <= RA_SEL_THRESHOLD, RA_ERR_INVALID_ARG,
               "select_rounds: unknown strategy %d", params->strategy);
    RA_REQUIRE(params->min_rounds >= 0 && params->max_rounds >= 0 && params->ddof >= 0, RA_ERR_INVALID_ARG,
               "select_rounds: min_rounds, max_rounds and ddof must be non-negative");
    RA_REQUIRE(params->keep_first >= 0 && params->keep_last >= 0, RA_ERR_INVALID_ARG,
               "select_rounds: keep_first and keep_last must be non-negative");
    RA_REQUIRE(params->lambda == params->lambda && params->fraction == params->fraction &&
                   params->threshold == params->threshold,
               RA_ERR_INVALID_ARG, "select_rounds: NaN parameter");
    if (params->strategy == RA_SEL_TOP_FRACTION)
        RA_REQUIRE(params->fraction > 0.0 && params->fraction <= 1.0, RA_ERR_INVALID_ARG,
                   "select_rounds: fraction must be in (0, 1]");
    SelectArgs a;
    a.scores = scores;
    a.n_rounds = n_rounds;
    a.R_max = R_max;
    a.p = *params;
    a.sel_idx = sel_idx;
    a.n_sel = n_sel;
    hipLaunchKernelGGL(select_kernel, dim3(B), dim3(256), 0, reinterpret_cast<hipStream_t>(stream), a);
    RA_HIP_CHECK(hipGetLastError());
    return RA_OK;
}
