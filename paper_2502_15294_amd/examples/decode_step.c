/*
 * The hot path driven from plain C through the C boundary alone (no Python, no PyTorch): round scores at the
 * watershed layer -> dynamic selection -> round-sparse decode attention on one post-watershed layer
 * (paper Sec. 3.2 steps 3 and 5, Sec. 3.3).  Device memory comes from hipMalloc, everything runs on the
 * null stream.
 *
 *   decode_step <input file> <output file>
 *
 * Input (little endian): int32 B, R_max, Hq, Hkv, d, lambda * 1000, history tokens, padded value tokens;
 * int64 max_tokens; int32 n_rounds[B]; int32 seg_len[B][R_max]; int64 seg_off[B][R_max];
 * int64 seg_off_v[B][R_max]; then bf16 bit patterns: q of the watershed layer [B][Hq][d], q of the attention
 * layer [B][Hq][d], keys of the watershed layer, keys and values of the attention layer in the contiguous
 * round layout of round_attention.h.
 * Output: float scores[B][R_max]; int32 sel_idx[B][R_max]; int32 n_sel[B]; float out[B][Hq][d]; float lse[B][Hq].
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "round_attention.h"

#define CHECK_HIP(x)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                       \
            return 2;                                                                     \
        }                                                                                 \
    } while (0)
#define CHECK_RA(x)                                                                       \
    do {                                                                                  \
        int rc_ = (x);                                                                    \
        if (rc_ != RA_OK) {                                                               \
            fprintf(stderr, "%s -> %d: %s\n", #x, rc_, ra_last_error());                  \
            return 3;                                                                     \
        }                                                                                 \
    } while (0)

static void* read_block(FILE* f, size_t bytes) {
    void* p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, f) != bytes) {
        fprintf(stderr, "short read (%zu bytes wanted)\n", bytes);
        exit(4);
    }
    return p;
}

static int to_device(void** dptr, const void* host, size_t bytes) {
    CHECK_HIP(hipMalloc(dptr, bytes ? bytes : 16));
    if (bytes) CHECK_HIP(hipMemcpy(*dptr, host, bytes, hipMemcpyHostToDevice));
    return 0;
}

int main(int argc, char** argv) {
    if (argc != 3) {
        fprintf(stderr, "usage: %s <input> <output>\n", argv[0]);
        return 1;
    }
    FILE* f = fopen(argv[1], "rb");
    if (!f) {
        perror(argv[1]);
        return 1;
    }
    int32_t* hdr = (int32_t*)read_block(f, 8 * sizeof(int32_t));
    const int B = hdr[0], R = hdr[1], Hq = hdr[2], Hkv = hdr[3], d = hdr[4];
    const double lambda = hdr[5] / 1000.0;
    const size_t n_tok = (size_t)hdr[6], n_tok_v = (size_t)hdr[7];
    int64_t* max_tokens = (int64_t*)read_block(f, sizeof(int64_t));
    const size_t BR = (size_t)B * R, q_elems = (size_t)B * Hq * d;
    int32_t* n_rounds = (int32_t*)read_block(f, B * sizeof(int32_t));
    int32_t* seg_len = (int32_t*)read_block(f, BR * sizeof(int32_t));
    int64_t* seg_off = (int64_t*)read_block(f, BR * sizeof(int64_t));
    int64_t* seg_off_v = (int64_t*)read_block(f, BR * sizeof(int64_t));
    uint16_t* q0 = (uint16_t*)read_block(f, q_elems * 2);
    uint16_t* q1 = (uint16_t*)read_block(f, q_elems * 2);
    const size_t k_bytes = n_tok * Hkv * d * 2, v_bytes = n_tok_v * Hkv * d * 2;
    void* k0 = read_block(f, k_bytes);
    void* k1 = read_block(f, k_bytes);
    void* v1 = read_block(f, v_bytes);
    fclose(f);

    CHECK_HIP(hipSetDevice(0));
    void *d_n_rounds, *d_seg_len, *d_seg_off, *d_seg_off_v, *d_q0, *d_q1, *d_k0, *d_k1, *d_v1;
    if (to_device(&d_n_rounds, n_rounds, B * sizeof(int32_t)) || to_device(&d_seg_len, seg_len, BR * sizeof(int32_t)) ||
        to_device(&d_seg_off, seg_off, BR * sizeof(int64_t)) || to_device(&d_seg_off_v, seg_off_v, BR * sizeof(int64_t)) ||
        to_device(&d_q0, q0, q_elems * 2) || to_device(&d_q1, q1, q_elems * 2) || to_device(&d_k0, k0, k_bytes) ||
        to_device(&d_k1, k1, k_bytes) || to_device(&d_v1, v1, v_bytes))
        return 2;

    ra_ctx* ctx = NULL;
    CHECK_RA(ra_create(&ctx, 0));
    ra_problem prob = {B, R, Hq, Hkv, d, 1, RA_BF16, 0, *max_tokens};
    size_t ws_bytes = 0;
    CHECK_RA(ra_workspace_bytes(&prob, &ws_bytes));
    void* ws = NULL;
    CHECK_HIP(hipMalloc(&ws, ws_bytes));
    CHECK_RA(ra_set_workspace(ctx, ws, ws_bytes));

    ra_kv_view watershed = {0}, layer = {0};
    watershed.k = d_k0;
    watershed.v = NULL; /* the score pass reads keys only */
    watershed.seg_off = (const int64_t*)d_seg_off;
    watershed.seg_off_v = NULL;
    watershed.seg_len = (const int32_t*)d_seg_len;
    watershed.n_rounds = (const int32_t*)d_n_rounds;
    watershed.B = B;
    watershed.R_max = R;
    watershed.Hkv = Hkv;
    watershed.d = d;
    watershed.dtype = RA_BF16;
    watershed.max_tokens = *max_tokens;
    layer = watershed;
    layer.k = d_k1;
    layer.v = d_v1;
    layer.seg_off_v = (const int64_t*)d_seg_off_v;

    float *d_scores, *d_out, *d_lse;
    int32_t *d_sel, *d_nsel;
    CHECK_HIP(hipMalloc((void**)&d_scores, BR * sizeof(float)));
    CHECK_HIP(hipMalloc((void**)&d_sel, BR * sizeof(int32_t)));
    CHECK_HIP(hipMalloc((void**)&d_nsel, B * sizeof(int32_t)));
    CHECK_HIP(hipMalloc((void**)&d_out, q_elems * sizeof(float)));
    CHECK_HIP(hipMalloc((void**)&d_lse, (size_t)B * Hq * sizeof(float)));

    const float scale = 1.0f / sqrtf((float)d);
    ra_select_params params = {RA_SEL_ADAPTIVE, 0, 1, 0, lambda, 0.10, 0.10, 0, 0};
    CHECK_RA(ra_round_scores(ctx, NULL, d_q0, 1, Hq, &watershed, NULL, 0, scale, NULL, d_scores));
    CHECK_RA(ra_select_rounds(ctx, NULL, d_scores, (const int32_t*)d_n_rounds, B, R, &params, d_sel, d_nsel));
    CHECK_RA(ra_round_sparse_attn_decode(ctx, NULL, d_q1, Hq, &layer, d_sel, d_nsel, NULL, NULL, NULL, 0, scale, d_out,
                                         d_lse));
    CHECK_HIP(hipDeviceSynchronize());

    float* scores = (float*)malloc(BR * sizeof(float));
    int32_t* sel = (int32_t*)malloc(BR * sizeof(int32_t));
    int32_t* nsel = (int32_t*)malloc(B * sizeof(int32_t));
    float* out = (float*)malloc(q_elems * sizeof(float));
    float* lse = (float*)malloc((size_t)B * Hq * sizeof(float));
    CHECK_HIP(hipMemcpy(scores, d_scores, BR * sizeof(float), hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(sel, d_sel, BR * sizeof(int32_t), hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(nsel, d_nsel, B * sizeof(int32_t), hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(out, d_out, q_elems * sizeof(float), hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(lse, d_lse, (size_t)B * Hq * sizeof(float), hipMemcpyDeviceToHost));
    FILE* o = fopen(argv[2], "wb");
    if (!o) {
        perror(argv[2]);
        return 1;
    }
    fwrite(scores, sizeof(float), BR, o);
    fwrite(sel, sizeof(int32_t), BR, o);
    fwrite(nsel, sizeof(int32_t), B, o);
    fwrite(out, sizeof(float), q_elems, o);
    fwrite(lse, sizeof(float), (size_t)B * Hq, o);
    fclose(o);
    CHECK_RA(ra_destroy(ctx));
    printf("decode_step: B=%d rounds<=%d Hq=%d Hkv=%d d=%d, kept rounds of sequence 0: %d\n", B, R, Hq, Hkv, d, nsel[0]);
    return 0;
}
