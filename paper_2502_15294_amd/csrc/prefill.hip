// Round-sparse question-prefill attention (paper Sec. 3.2 step 4).
#include "common.hpp"

using namespace ra;

extern "C" int ra_round_sparse_attn_prefill(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq,
                                            const ra_kv_view* layer, const int32_t* sel_idx, const int32_t* n_sel,
                                            const void* cur_k, const void* cur_v, int cur_len, float scale, float* out,
                                            float* lse) {
    (void)ctx; (void)stream; (void)q; (void)q_len; (void)Hq; (void)layer; (void)sel_idx; (void)n_sel;
    (void)cur_k; (void)cur_v; (void)cur_len; (void)scale; (void)out; (void)lse;
    return fail(RA_ERR_UNSUPPORTED, "prefill: not implemented yet");
}
