// Round selection (paper Sec. 3.3): from the per-sequence round scores choose the rounds whose KV
// the post-watershed layers will attend over.  One workgroup per sequence; the score vector lives in
// LDS and select_common.hpp does the work.  This file holds the stand-alone kernel and entry point.
#include "select_common.hpp"

namespace ra {

struct SelectArgs {
    const float* scores;
    const int32_t* n_rounds;
    int R_max;
    ra_select_params p;
    int32_t* sel_idx;
    int32_t* n_sel;
};

__global__ __launch_bounds__(256) void select_kernel(SelectArgs a) {
    __shared__ float s[kMaxRounds];
    __shared__ SelectShared<4> sh;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int R = min(max(a.n_rounds[b], 0), a.R_max);
    for (int r = tid; r < a.R_max; r += 256) {
        const float v = a.scores[(size_t)b * a.R_max + r];  // asked for before the round count has arrived
        if (r < R) s[r] = v;
    }
    __syncthreads();
    select_rounds_block<4>(s, R, a.R_max, a.p, a.sel_idx + (size_t)b * a.R_max, a.n_sel + b, sh);
}

int check_select_params(const ra_select_params* params, const char* who) {
    RA_REQUIRE(params != nullptr, RA_ERR_INVALID_ARG, "%s: params is NULL", who);
    RA_REQUIRE(params->strategy >= RA_SEL_ADAPTIVE && params->strategy <= RA_SEL_THRESHOLD, RA_ERR_INVALID_ARG,
               "%s: unknown strategy %d", who, params->strategy);
    RA_REQUIRE(params->min_rounds >= 0 && params->max_rounds >= 0 && params->ddof >= 0, RA_ERR_INVALID_ARG,
               "%s: min_rounds, max_rounds and ddof must be non-negative", who);
    RA_REQUIRE(params->keep_first >= 0 && params->keep_last >= 0, RA_ERR_INVALID_ARG,
               "%s: keep_first and keep_last must be non-negative", who);
    RA_REQUIRE(params->lambda == params->lambda && params->fraction == params->fraction &&
                   params->threshold == params->threshold,
               RA_ERR_INVALID_ARG, "%s: NaN parameter", who);
    if (params->strategy == RA_SEL_TOP_FRACTION)
        RA_REQUIRE(params->fraction > 0.0 && params->fraction <= 1.0, RA_ERR_INVALID_ARG,
                   "%s: fraction must be in (0, 1]", who);
    return RA_OK;
}

// Stand-alone launch, also used by the score entry point when its finishing pass cannot take the selection along.
void launch_select(const float* scores, const int32_t* n_rounds, int B, int R_max, const ra_select_params& p,
                   int32_t* sel_idx, int32_t* n_sel, hipStream_t st) {
    SelectArgs a;
    a.scores = scores;
    a.n_rounds = n_rounds;
    a.R_max = R_max;
    a.p = p;
    a.sel_idx = sel_idx;
    a.n_sel = n_sel;
    hipLaunchKernelGGL(select_kernel, dim3(B), dim3(256), 0, st, a);
}

}  // namespace ra

using namespace ra;

extern "C" int ra_select_rounds(ra_ctx* ctx, void* stream, const float* scores, const int32_t* n_rounds, int B,
                                int R_max, const ra_select_params* params, int32_t* sel_idx, int32_t* n_sel) {
    RA_REQUIRE(ctx != nullptr, RA_ERR_INVALID_ARG, "select_rounds: ctx is NULL");
    RA_REQUIRE(scores && n_rounds && params && sel_idx && n_sel, RA_ERR_INVALID_ARG, "select_rounds: NULL argument");
    RA_REQUIRE(B > 0 && R_max > 0, RA_ERR_INVALID_ARG, "select_rounds: B and R_max must be positive");
    RA_REQUIRE(R_max <= kMaxRounds, RA_ERR_UNSUPPORTED, "select_rounds: R_max %d exceeds %d", R_max, kMaxRounds);
    if (int rc = check_select_params(params, "select_rounds")) return rc;
    launch_select(scores, n_rounds, B, R_max, *params, sel_idx, n_sel, reinterpret_cast<hipStream_t>(stream));
    RA_HIP_CHECK(hipGetLastError());
    return RA_OK;
}
