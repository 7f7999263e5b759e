// Statistics over round distributions that sit beside the hot path:
//   * the curve that locates the watershed layer (paper Sec. 3.1, Observation 2 and Fig. 2b): for every
//     layer the mean Kullback-Leibler divergence of its round distribution to those of the later layers;
//   * the share of a round distribution that a selection covers, used with the running distribution of the
//     answer tokens (Eq. 1, right-hand form) to watch a selection drift during a long answer.
// Both are small reductions in IEEE double; they take the [.][B][R_max] score tensors of ra_round_scores.
#include "common.hpp"

namespace ra {

constexpr int kKlThreads = 256;
constexpr int kKlPerThread = kMaxRounds / kKlThreads;

// grid (L - 1, B), block 256.  Thread t owns rounds t, t + 256, ...: it keeps P^l_r and ln P^l_r in
// registers and walks the later layers, adding P^l_r (ln P^l_r - ln P^l'_r); rounds with P^l_r = 0 add
// nothing, a later layer with P^l'_r = 0 < P^l_r gives +inf.  The 256 partial sums are added in a fixed
// tree order through LDS.
__global__ __launch_bounds__(kKlThreads) void layer_divergence_kernel(const float* __restrict__ p,
                                                                      const int32_t* __restrict__ n_rounds, int L, int B,
                                                                      int R_max, double* __restrict__ kl) {
    __shared__ double red[kKlThreads];
    const int l = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int R = min(max(n_rounds[b], 0), R_max);
    const size_t plane = (size_t)B * R_max;
    const float* mine = p + (size_t)l * plane + (size_t)b * R_max;
    double pl[kKlPerThread], lg[kKlPerThread];
#pragma unroll
    for (int k = 0; k < kKlPerThread; ++k) {
        const int r = tid + kKlThreads * k;
        pl[k] = r < R ? (double)mine[r] : 0.0;
        lg[k] = pl[k] > 0.0 ? log(pl[k]) : 0.0;
    }
    double sum = 0.0;
    for (int l2 = l + 1; l2 < L; ++l2) {
        const float* other = p + (size_t)l2 * plane + (size_t)b * R_max;
#pragma unroll
        for (int k = 0; k < kKlPerThread; ++k) {
            const int r = tid + kKlThreads * k;
            if (r < R && pl[k] > 0.0) {
                const double q = (double)other[r];
                sum += q > 0.0 ? pl[k] * (lg[k] - log(q)) : (double)__builtin_inff();
            }
        }
    }
    red[tid] = sum;
    __syncthreads();
    for (int s = kKlThreads / 2; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) kl[(size_t)b * (L - 1) + l] = red[0] / (double)(L - 1 - l);
}

// grid (1), block 256: mean over the sequences, added in sequence order.
__global__ __launch_bounds__(kKlThreads) void divergence_mean_kernel(const double* __restrict__ kl, int B, int n,
                                                                     double* __restrict__ kl_mean) {
    for (int l = threadIdx.x; l < n; l += kKlThreads) {
        double s = 0.0;
        for (int b = 0; b < B; ++b) s += kl[(size_t)b * n + l];
        kl_mean[l] = s / (double)B;
    }
}

// grid (B), block 64: lane j adds the scores of the selected rounds j, j + 64, ... of its sequence.
__global__ __launch_bounds__(64) void coverage_kernel(const float* __restrict__ scores, const int32_t* __restrict__ sel_idx,
                                                      const int32_t* __restrict__ n_sel, int R_max,
                                                      float* __restrict__ coverage) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int n = min(max(n_sel[b], 0), R_max);
    double s = 0.0;
    for (int i = lane; i < n; i += 64) {
        const int r = sel_idx[(size_t)b * R_max + i];
        if (r >= 0 && r < R_max) s += (double)scores[(size_t)b * R_max + r];
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) coverage[b] = (float)s;
}

}  // namespace ra

using namespace ra;

extern "C" int ra_layer_divergence(ra_ctx* ctx, void* stream, const float* p, const int32_t* n_rounds, int L, int B,
                                   int R_max, double* kl, double* kl_mean) {
    RA_REQUIRE(ctx != nullptr, RA_ERR_INVALID_ARG, "layer_divergence: ctx is NULL");
    RA_REQUIRE(p != nullptr && n_rounds != nullptr && kl != nullptr, RA_ERR_INVALID_ARG,
               "layer_divergence: NULL argument");
    RA_REQUIRE(L >= 2 && B > 0 && R_max > 0, RA_ERR_INVALID_ARG,
               "layer_divergence: needs at least two layers and positive B and R_max");
    RA_REQUIRE(R_max <= kMaxRounds, RA_ERR_UNSUPPORTED, "layer_divergence: R_max %d exceeds %d", R_max, kMaxRounds);
    RA_REQUIRE(L - 1 <= 65535 && B <= 65535, RA_ERR_UNSUPPORTED, "layer_divergence: L or B exceeds 65535");
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(layer_divergence_kernel, dim3(L - 1, B), dim3(kKlThreads), 0, st, p, n_rounds, L, B, R_max, kl);
    if (kl_mean) hipLaunchKernelGGL(divergence_mean_kernel, dim3(1), dim3(kKlThreads), 0, st, kl, B, L - 1, kl_mean);
    RA_HIP_CHECK(hipGetLastError());
    return RA_OK;
}

extern "C" int ra_selection_coverage(ra_ctx* ctx, void* stream, const float* scores, const int32_t* sel_idx,
                                     const int32_t* n_sel, int B, int R_max, float* coverage) {
    RA_REQUIRE(ctx != nullptr, RA_ERR_INVALID_ARG, "selection_coverage: ctx is NULL");
    RA_REQUIRE(scores && sel_idx && n_sel && coverage, RA_ERR_INVALID_ARG, "selection_coverage: NULL argument");
    RA_REQUIRE(B > 0 && R_max > 0, RA_ERR_INVALID_ARG, "selection_coverage: B and R_max must be positive");
    hipLaunchKernelGGL(coverage_kernel, dim3(B), dim3(64), 0, reinterpret_cast<hipStream_t>(stream), scores, sel_idx,
                       n_sel, R_max, coverage);
    RA_HIP_CHECK(hipGetLastError());
    return RA_OK;
}
