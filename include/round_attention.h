/*
 * round_attention.h -- C ABI of the Round Attention hot path for AMD MI355X (gfx950).
 *
 * The library implements the part of the Round Attention inference pipeline (paper Sec. 3.2,
 * steps 3-5, and Sec. 3.3) that runs on the GPU once the watershed layer L_w has been reached:
 *
 *   ra_round_scores               round-level attention distribution of the current question over
 *                                 the history rounds at the watershed layer (Sec. 3.1, Eq. 1)
 *   ra_select_rounds              choice of the relevant rounds from that distribution (Sec. 3.3)
 *   ra_kv_store_*                 round-indexed store of the post-watershed KV ("u_m", Sec. 3.2):
 *                                 host-resident per round, selected rounds copied to the GPU
 *   ra_round_sparse_attn_decode   attention of one new token over the selected rounds (step 5)
 *   ra_watershed_attn_decode,     decode / question prefill at the watershed layer: dense attention and, from
 *   ra_watershed_attn_prefill     the same pass over the keys, the round scores (steps 2-3 fused)
 *   ra_round_sparse_attn_prefill  attention of the question's tokens over the selected rounds
 *                                 and, causally, over the question itself (step 4)
 *
 * Conventions
 * -----------
 * - Plain C, no exceptions.  Every call returns RA_OK (0) or a negative ra_status; the text of the
 *   last failure on the calling thread is available from ra_last_error().
 * - "device" pointers are HIP device memory on the context's GPU; "host" pointers are ordinary or
 *   pinned host memory as stated.  The caller owns every buffer it passes in.  The library owns its
 *   context, and the store owns its device pool and its small index tables.
 * - Compute calls validate their arguments on the host, enqueue kernels on the caller's stream
 *   (a hipStream_t passed as void*; NULL is the default stream), do not synchronise, and do not
 *   allocate: scratch memory comes from the workspace given to ra_set_workspace().  Outputs are
 *   fully overwritten.  Identical inputs give bitwise identical outputs.
 * - Arguments are checked before anything is launched; on error nothing has been enqueued.
 * - Head mapping under grouped-query attention: query head h reads KV head h / (Hq / Hkv).
 *
 * KV layout (one layer), round-indexed
 * ------------------------------------
 * Keys are stored token-major (one row of d channels per token).  Values are stored TRANSPOSED in
 * tiles of 16 tokens, [d][16] per tile, the last tile of a round padded (the padding must hold finite
 * numbers, e.g. zeros), so that the matrix-core kernels read several consecutive tokens of a channel
 * with one load.
 * contiguous (block_size == 0): the keys of round r of sequence b are a block of Hkv * len * d
 *   elements, [Hkv][len][d]; seg_off[b][r] is its start in units of tokens:
 *     K(g, t, c) = (seg_off * Hkv + g * len + t) * d + c                         relative to `k`.
 *   The values are a block of Hkv * L16 * d elements, [Hkv][L16 / 16][d][16], L16 = 16 * ceil(len / 16);
 *   seg_off_v[b][r] (seg_off if seg_off_v is NULL) is its start in units of tokens:
 *     V(g, t, c) = (seg_off_v * Hkv + g * L16 + (t / 16) * 16) * d + c * 16 + t % 16   relative to `v`.
 * paged (block_size == 16): storage is an array of physical blocks, [n_blocks][Hkv][16][d] for keys and
 *   [n_blocks][Hkv][d][16] for values; a round owns ceil(len / 16) consecutive slots of row b of
 *   block_table starting at slot seg_off[b][r].  With blk = block_table[b][seg_off + t / 16]:
 *     K(g, t, c) = ((blk * Hkv + g) * 16 + t % 16) * d + c,   V(g, t, c) = ((blk * Hkv + g) * d + c) * 16 + t % 16.
 * The current round's own K/V ("cur", the question so far / the tokens generated so far) is passed
 * separately, token-major for both keys and values: [B][cur_cap][Hkv][d].
 */
#ifndef ROUND_ATTENTION_H
#define ROUND_ATTENTION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ra_status {
    RA_OK = 0,
    RA_ERR_INVALID_ARG = -1, /* null pointer, negative size, inconsistent shapes               */
    RA_ERR_UNSUPPORTED = -2, /* dtype / head_dim / group size / block size not implemented      */
    RA_ERR_WORKSPACE = -3,   /* no workspace set, or it is too small for this call              */
    RA_ERR_STATE = -4,       /* call made in the wrong order (e.g. view requested before stage) */
    RA_ERR_OOM = -5,         /* the store's device pool cannot hold the selected rounds         */
    RA_ERR_HIP = -6          /* a HIP runtime call failed; see ra_last_error()                  */
} ra_status;

typedef enum ra_dtype { RA_F32 = 0, RA_BF16 = 1 } ra_dtype;

/* Sec. 3.3: strategy 3 (adaptive), strategy 2 (top fraction), strategy 1 (fixed threshold). */
typedef enum ra_strategy { RA_SEL_ADAPTIVE = 0, RA_SEL_TOP_FRACTION = 1, RA_SEL_THRESHOLD = 2 } ra_strategy;

typedef struct ra_select_params {
    int32_t strategy;   /* ra_strategy                                                          */
    int32_t ddof;       /* ADAPTIVE: variance divisor is R - ddof (0 = population, the default)  */
    int32_t min_rounds; /* keep at least this many rounds, best score first (default 1)          */
    int32_t max_rounds; /* keep at most this many rounds; 0 = no cap                             */
    double lambda;      /* ADAPTIVE: keep score > mean + lambda * std (Sec. 3.3; default 1.0,
                           0.0 gives the "greater than the average" rule of Sec. 4.4)            */
    double fraction;    /* TOP_FRACTION: keep the ceil(fraction * R) best rounds (paper: 0.10)   */
    double threshold;   /* THRESHOLD: keep score > threshold (paper: v = 0.1)                    */
    int32_t keep_first; /* optional policy, not the paper's: the first keep_first rounds and ...  */
    int32_t keep_last;  /* ... the most recent keep_last rounds are added to what the rule kept;
                           the rule (statistics, min_rounds, max_rounds) is applied to all rounds
                           as without them.  0 = off.                                            */
} ra_select_params;

/* One layer's round-indexed KV cache.  All pointers are device pointers. */
typedef struct ra_kv_view {
    const void* k;              /* keys                                                          */
    const void* v;              /* values; may be NULL for ra_round_scores                       */
    const int64_t* seg_off;     /* [B][R_max] round start: tokens (contiguous) or slots (paged)  */
    const int64_t* seg_off_v;   /* [B][R_max] same for values, or NULL to use seg_off            */
    const int32_t* seg_len;     /* [B][R_max] tokens in each round (0 is legal)                  */
    const int32_t* n_rounds;    /* [B] number of history rounds of each sequence, 0..R_max       */
    const int32_t* block_table; /* [B][max_blocks] physical block ids (paged) or NULL            */
    int32_t block_size;         /* 0 (contiguous) or 16 (paged)                                  */
    int32_t max_blocks;         /* row length of block_table                                     */
    int32_t B, R_max, Hkv, d;   /* R_max <= 1024; d is 64 or 128                                 */
    int32_t dtype;              /* ra_dtype of k, v, q and cur                                   */
    int32_t reserved;
    int64_t max_tokens;         /* host-known upper bound on one sequence's history tokens.  It sizes
                                   launches and scratch, never indexes memory; if it understates the
                                   cache, ra_round_scores returns NaN scores for that sequence      */
} ra_kv_view;

/* Shape envelope used to size the workspace. */
typedef struct ra_problem {
    int32_t B, R_max, Hq, Hkv, d, q_len_max;
    int32_t dtype;
    int32_t reserved;
    int64_t max_tokens; /* per sequence, history + current round */
} ra_problem;

typedef struct ra_ctx ra_ctx;

const char* ra_last_error(void);

/* Create / destroy a context bound to HIP device `device`.  Creation queries the device once. */
int ra_create(ra_ctx** out, int device);
int ra_destroy(ra_ctx* ctx);

/* Upper bound of the scratch bytes any compute call needs for problems inside `p`. */
int ra_workspace_bytes(const ra_problem* p, size_t* bytes_out);
/* Hand the context a device buffer (256-byte aligned, at least 32 KB) to use as scratch.  The caller keeps
 * ownership and must keep it alive, and must not run two calls that use it concurrently. */
int ra_set_workspace(ra_ctx* ctx, void* device_ptr, size_t bytes);

/*
 * Measurement aid (Sec. 4.3 and App. C break the latency down into the selection and attention steps; this is
 * how a benchmark gets the duration of the kernel that dominates a call, without the small kernels around it).
 * While enabled, ra_round_scores, ra_round_sparse_attn_decode and ra_round_sparse_attn_prefill attach two HIP
 * events to the launch of their streaming kernel (the pass over the keys, or over the selected keys and
 * values), which then carry that kernel's own start and end time stamps.  ra_profile_last_ms waits for the end
 * event of the most recent such call and returns the milliseconds between the two; RA_ERR_STATE if no call was
 * made since enabling.  Leave this off when timing whole steps.  The first enable creates the two events (the
 * only allocation); not for use under stream capture.
 */
int ra_profile_kernels(ra_ctx* ctx, int enable);
int ra_profile_last_ms(ra_ctx* ctx, float* ms_out);
/*
 * Second measurement aid: the bandwidth a plain read kernel (non-temporal 16-byte loads, every wave streaming its
 * own contiguous span, nothing else) reaches on this GPU over the caller's device buffer, the practical ceiling
 * the streaming kernels are compared with beside the published peak.  One untimed pass, then `iters` timed passes between two HIP events on `stream`.
 * Unlike the compute calls this one WAITS for its kernels and creates (and destroys) two events; the buffer
 * should be much larger than the 256 MB of last-level cache.  Needs a workspace (it keeps one word there).
 *   device_buf  device memory, 16-byte aligned; bytes a multiple of 16;  gb_per_s  host, 1e9 bytes per second
 */
int ra_measure_read_bandwidth(ra_ctx* ctx, void* stream, const void* device_buf, size_t bytes, int iters,
                              float* gb_per_s);

/*
 * Round scores at the watershed layer (Sec. 3.1, Eq. 1 and the normalisation after it).
 * For every sequence b and query head h: softmax of scale * q . k over all history tokens and,
 * if cur_k is given, over the current round's keys visible to each query token (query token i
 * sees cur token j iff j <= cur_len - q_len + i); the probabilities are summed per history
 * round and over the q_len query tokens, then normalised over the history rounds.
 *   q            device [B][q_len][Hq][d], dtype of the view
 *   watershed    the watershed layer's view; only keys are read
 *   cur_k        device [B][cur_len][Hkv][d] or NULL (cur_len = 0)
 *   scores_head  device float [B][Hq][R_max]: per-head distribution, rows sum to 1 over r < n_rounds[b],
 *                entries r >= n_rounds[b] are 0; may be NULL
 *   scores       device float [B][R_max]: arithmetic mean of scores_head over the query heads
 * Zero-length rounds score 0; a sequence with no history tokens gets all zeros.
 */
int ra_round_scores(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq, const ra_kv_view* watershed,
                    const void* cur_k, int cur_len, float scale, float* scores_head, float* scores);

/*
 * Eq. 1, right-hand form (aAtt): the round masses of the answer tokens, added up as the answer is
 * generated.  Same computation and arguments as ra_round_scores, except that the query tokens'
 * un-normalised round masses (each token's softmax taken over the history and the keys of the
 * current round it sees) are first added to `acc`, and scores_head / scores are the normalised
 * running totals.  Called once per decode step with q_len = 1 and the grown cur_k / cur_len, after
 * T steps acc holds sum_i sum_{j in round k} Att(a_i, K_j) over the T answer tokens, exactly what one
 * ra_round_scores call with q_len = T would normalise.  With a single query token the current
 * round's keys ARE read here (their share no longer cancels).
 *   acc   device float [B][Hq][R_max], in/out; the caller zeroes it at the start of the answer
 */
int ra_round_scores_accumulate(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq,
                               const ra_kv_view* watershed, const void* cur_k, int cur_len, float scale,
                               float* acc, float* scores_head, float* scores);

/*
 * Round selection (Sec. 3.3).  Per sequence, from scores[b][0 .. n_rounds[b]):
 *   ADAPTIVE      keep r with score > mean + lambda * std   (mean/std in double, summed in round order)
 *   TOP_FRACTION  keep the ceil(fraction * R) highest
 *   THRESHOLD     keep r with score > threshold
 * then at least min_rounds and at most max_rounds are kept, preferring higher score, then lower
 * round index.  Output is ascending.
 *   scores   device float [B][R_max]      n_rounds  device int32 [B]
 *   sel_idx  device int32 [B][R_max], unused tail entries set to -1
 *   n_sel    device int32 [B]
 * Scores must not be NaN.
 */
int ra_select_rounds(ra_ctx* ctx, void* stream, const float* scores, const int32_t* n_rounds, int B, int R_max,
                     const ra_select_params* params, int32_t* sel_idx, int32_t* n_sel);

/*
 * Round scores and round selection in one call (Sec. 3.2 step 3: "identify the top-k relevant rounds" with the
 * watershed layer's attention; Sec. 3.1 Eq. 1 followed by Sec. 3.3).  Same arguments and outputs as
 * ra_round_scores followed by ra_select_rounds on its `scores`; the workgroup that finishes a sequence's scores
 * selects its rounds while they are still on chip, which saves a kernel launch on the path of every question.
 * scores_head, scores, sel_idx and n_sel are bitwise what the two separate calls give.
 *   params   as for ra_select_rounds;  sel_idx device int32 [B][R_max];  n_sel device int32 [B]
 */
int ra_round_scores_select(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq, const ra_kv_view* watershed,
                           const void* cur_k, int cur_len, float scale, const ra_select_params* params,
                           float* scores_head, float* scores, int32_t* sel_idx, int32_t* n_sel);

/*
 * Round-sparse decode attention (Sec. 3.2 step 5): one query token per sequence attends over the
 * tokens of the selected rounds of `layer` plus the first cur_len[b] tokens of the current round.
 *   q        device [B][Hq][d]
 *   sel_idx  device int32 [B][R_max] and n_sel device int32 [B]; both NULL = every round of the view
 *            (entries outside 0..n_rounds[b]-1 are ignored)
 *   cur_k/v  device [B][cur_cap][Hkv][d] or NULL;  cur_len device int32 [B] (values clamped to cur_cap)
 *   out      device float [B][Hq][d];  lse device float [B][Hq] or NULL: natural log of the
 *            softmax normaliser of the scaled logits
 * A sequence whose key set is empty (nothing selected and no current tokens) gets out = 0, lse = -inf.
 */
int ra_round_sparse_attn_decode(ra_ctx* ctx, void* stream, const void* q, int Hq, const ra_kv_view* layer,
                                const int32_t* sel_idx, const int32_t* n_sel, const void* cur_k,
                                const void* cur_v, const int32_t* cur_len, int cur_cap, float scale, float* out,
                                float* lse);

/*
 * ra_round_sparse_attn_decode for callers that cannot allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, bitwise the same
 * results; the scratch is a 32 MiB array inside the library's device code (every GPU the library runs on holds it
 * until the process ends), whose address ra_create looks up once per device.  The context's workspace is neither
 * needed nor touched.  The call allocates nothing, synchronises nothing and records no memset.
 * RA_ERR_WORKSPACE if the call would need more than 32 MiB of scratch (about 4000 partial results: every
 * benchmark configuration of this repository fits); RA_ERR_UNSUPPORTED etc. as for the other call.
 * All calls on one GPU share the array: two calls that overlap in time (different streams, different contexts)
 * race; consecutive calls on one stream do not.  Nothing in the array has to be cleared between calls.
 */
int ra_round_sparse_attn_decode_noalloc(ra_ctx* ctx, void* stream, const void* q, int Hq, const ra_kv_view* layer,
                                        const int32_t* sel_idx, const int32_t* n_sel, const void* cur_k,
                                        const void* cur_v, const int32_t* cur_len, int cur_cap, float scale,
                                        float* out, float* lse);

/*
 * Decode at the watershed layer itself (Sec. 3.2 steps 2-3: the round scores are taken with the watershed
 * layer's own attention, qAtt^{L_w}; Eq. 1 in its one-query-token form): dense attention of one query token per
 * sequence over every history round of `watershed` (which must carry values) plus the current round, and, from
 * the same pass over the keys, the round scores that ra_round_scores would return for this q and this layer
 * (no current round in the scores: with one query token it cancels in the normalisation over history rounds).
 * One read of K and V instead of a read of K for the scores and another of K and V for the attention.
 *   q, cur_k, cur_v, cur_len, cur_cap, out, lse   as for ra_round_sparse_attn_decode with sel_idx = NULL
 *   scores_head  device float [B][Hq][R_max] or NULL;  scores  device float [B][R_max] (required)
 * bf16 with d = 128 only (RA_ERR_UNSUPPORTED otherwise).  As in ra_round_scores, a view whose max_tokens
 * understates the history gives NaN scores.
 */
int ra_watershed_attn_decode(ra_ctx* ctx, void* stream, const void* q, int Hq, const ra_kv_view* watershed,
                             const void* cur_k, const void* cur_v, const int32_t* cur_len, int cur_cap, float scale,
                             float* out, float* lse, float* scores_head, float* scores);

/*
 * Question prefill at the watershed layer itself (Sec. 3.2 steps 2-3, Eq. 1 in its q_len-token form): dense
 * attention of the question's q_len tokens over every history round of `watershed` and, causally, over the
 * question itself, and from the same pass the round scores that ra_round_scores would return for this q, this
 * layer and this cur_k.
 *   q, q_len, cur_k, cur_v, cur_len, out, lse   as for ra_round_sparse_attn_prefill with sel_idx = NULL
 *   scores_head  device float [B][Hq][R_max] or NULL;  scores  device float [B][R_max] (required)
 */
int ra_watershed_attn_prefill(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq, const ra_kv_view* watershed,
                              const void* cur_k, const void* cur_v, int cur_len, float scale, float* out, float* lse,
                              float* scores_head, float* scores);

/*
 * Round-sparse question-prefill attention (Sec. 3.2 step 4): q_len query tokens per sequence, the
 * last q_len tokens of the current round.  History rounds are fully visible; inside the current
 * round query i sees token j iff j <= cur_len - q_len + i.
 *   q        device [B][q_len][Hq][d]
 *   cur_k/v  device [B][cur_len][Hkv][d] or NULL (then cur_len must be 0); if given, cur_len >= q_len
 *   out      device float [B][q_len][Hq][d];  lse device float [B][q_len][Hq] or NULL
 * Only bf16 with d = 128 is implemented (matrix-core path).
 */
int ra_round_sparse_attn_prefill(ra_ctx* ctx, void* stream, const void* q, int q_len, int Hq,
                                 const ra_kv_view* layer, const int32_t* sel_idx, const int32_t* n_sel,
                                 const void* cur_k, const void* cur_v, int cur_len, float scale, float* out,
                                 float* lse);

/*
 * How ra_round_sparse_attn_prefill with many query rows (q_len * Hq / Hkv > 32; Sec. 3.2 step 4) feeds the softmax
 * probabilities P to the matrix cores for P.V.  A setting of the context; it changes no other call (not
 * ra_watershed_attn_prefill either, whose scores decide the selection).
 *   RA_PREFILL_P_BF16X2  (default) P as the sum of two bf16 numbers, two passes over V: about 16 bits of P,
 *                        output error about 2e-5 of a row's largest magnitude
 *   RA_PREFILL_P_F16     P rounded to fp16, V converted to fp16 on chip, one pass: a third fewer matrix-core
 *                        instructions; output error about 4e-4 of a row's largest magnitude, 20 times the
 *                        default's (the contract of every attention call is 2e-3).
 *                        Values beyond fp16's range (|v| > 65504) saturate: use the default for such caches.
 */
typedef enum ra_prefill_precision { RA_PREFILL_P_BF16X2 = 0, RA_PREFILL_P_F16 = 1 } ra_prefill_precision;
int ra_set_prefill_precision(ra_ctx* ctx, int mode);

/*
 * Sec. 3.1, Observation 2 and Fig. 2b: the curve whose drop marks the watershed layer.  For each
 * layer l = 0 .. L-2 and each sequence, the mean over the later layers l' > l of
 * KL(P^l || P^l') = sum_r P^l_r ln(P^l_r / P^l'_r) (natural logarithm; a round with P^l_r = 0 adds
 * nothing, P^l'_r = 0 < P^l_r gives +inf), computed in double.
 *   p         device float [L][B][R_max]: per layer the `scores` output of ra_round_scores
 *   n_rounds  device int32 [B]
 *   kl        device double [B][L-1]
 *   kl_mean   device double [L-1] or NULL: mean of kl over the sequences (the plotted curve)
 * The paper reads L_w off the plot; no rule is given, so none is applied here.
 */
int ra_layer_divergence(ra_ctx* ctx, void* stream, const float* p, const int32_t* n_rounds, int L, int B,
                        int R_max, double* kl, double* kl_mean);

/*
 * Share of a round distribution that falls on a selection: coverage[b] = sum over the selected
 * rounds of scores[b][r].  With the running answer distribution of ra_round_scores_accumulate it
 * tells how much of the answer's attention the rounds chosen from the question still cover
 * (Sec. 3.1, Observation 1 is the claim that this stays high).
 *   scores device float [B][R_max]; sel_idx device int32 [B][R_max]; n_sel device int32 [B];
 *   coverage device float [B]
 */
int ra_selection_coverage(ra_ctx* ctx, void* stream, const float* scores, const int32_t* sel_idx,
                          const int32_t* n_sel, int B, int R_max, float* coverage);

/* ------------------------------------------------------------------------------------------
 * Round-indexed KV store for the post-watershed layers (Sec. 3.2: "u_m" lives in host memory as
 * one tensor per round and is moved to the GPU in one transfer when the round is selected).
 *
 * Host layout of one round's tensor: for each of the n_layers layers in turn, the keys [Hkv][len][d]
 * followed by the values in transposed 16-token tiles [Hkv][ceil(len/16)][d][16] (padding zeroed);
 * ra_kv_store_round_bytes() gives the size.  It lives in PINNED host memory (hipHostMalloc or torch
 * pin_memory); the caller keeps it alive and unchanged while registered.  Staging copies it as is into
 * the device pool, so each slice already is a round block of the contiguous layout described above;
 * the per-layer views index it through seg_off / seg_off_v.
 * ------------------------------------------------------------------------------------------ */
typedef struct ra_kv_store ra_kv_store;

typedef struct ra_store_cfg {
    int32_t device;
    int32_t n_layers; /* number of post-watershed layers held per round */
    int32_t B, R_max, Hkv, d;
    int32_t dtype;
    int32_t reserved;
    size_t device_pool_bytes; /* capacity of the device pool the selected rounds are staged into */
} ra_store_cfg;

typedef enum ra_stage_order {
    RA_STAGE_ROUND_MAJOR = 0, /* one copy per selected round (the paper's monolithic transfer).  Every layer
                                 becomes ready only when the last round has arrived: no overlap with compute   */
    RA_STAGE_LAYER_MAJOR = 1, /* one copy per (layer, round), layer by layer: the first post-watershed layer can
                                 start after 1 / n_layers of the transfer, at the price of n_layers times the copies */
    RA_STAGE_GROUPED = 2      /* one copy per (group of consecutive layers, round): a first group of n_layers / 8
                                 layers, up to three larger groups, a last group of one layer.  Overlaps like
                                 LAYER_MAJOR with a fifth of its copies (24 layers: groups of 3, 7, 7, 6, 1); the order
                                 to use when compute should overlap the transfer (Sec. 3.2)                    */
} ra_stage_order;

int ra_kv_store_create(ra_kv_store** out, const ra_store_cfg* cfg);
int ra_kv_store_destroy(ra_kv_store* store);
/* Register (or replace) the host tensor of round `round` of sequence `seq`; len >= 0 tokens.
 * Returns RA_ERR_INVALID_ARG if host_kv is not pinned host memory. */
int ra_kv_store_register_round(ra_kv_store* store, int seq, int round, const void* host_kv, int len);
/* Bytes of one registered round's host tensor for a given length. */
size_t ra_kv_store_round_bytes(const ra_kv_store* store, int len);
/*
 * Enqueue on `side_stream` the host-to-device copies of every selected round and of the index
 * tables of the compact per-layer views, and record one "ready" event per layer.
 *   sel_idx_host int32 [B][R_max], n_sel_host int32 [B]  (host memory; read before returning)
 * Returns RA_ERR_STATE if a selected round was never registered, RA_ERR_OOM if the pool is too
 * small (nothing is enqueued in either case).
 */
int ra_kv_store_stage(ra_kv_store* store, const int32_t* sel_idx_host, const int32_t* n_sel_host, int order,
                      void* side_stream);
/* Make `compute_stream` wait until `layer` (0-based) has fully arrived. */
int ra_kv_store_wait_layer(ra_kv_store* store, int layer, void* compute_stream);
/* Compact view of one staged layer: its rounds are the selected rounds in ascending order, so the
 * attention calls take it with sel_idx = n_sel = NULL. */
int ra_kv_store_layer_view(ra_kv_store* store, int layer, ra_kv_view* out);
/* Byte accounting of the last stage call: bytes copied to the device and bytes of all registered rounds. */
int ra_kv_store_stats(const ra_kv_store* store, uint64_t* staged_bytes, uint64_t* registered_bytes,
                      uint64_t* n_copies);
/* Forget the staged rounds (the pool is reused by the next stage call); registrations are kept.
 * The caller must have finished all work that reads the staged views. */
int ra_kv_store_release(ra_kv_store* store);

/*
 * End of a turn (Sec. 3.2, last step of the pipeline; Alg. 1, last line): the keys and values that the
 * post-watershed layers produced for the new round go to host memory, one tensor per sequence in
 * the host layout above, and are registered as round round_host[b] of sequence b.  (The selected
 * rounds need no copy back: their host tensors are never modified.)
 *   round_host   host int32 [B]: the index the new round gets; -1 = nothing to save for this sequence
 *   len_host     host int32 [B]: tokens of the new round, 0 <= len <= cur_cap
 *   cur_k_layers, cur_v_layers   host arrays of n_layers DEVICE pointers, one per post-watershed
 *                layer, each [B][cur_cap][Hkv][d] token-major (the cur_k / cur_v of the attention
 *                calls), 16-byte aligned
 *   host_kv      host array of B pointers to PINNED host memory of ra_kv_store_round_bytes(len[b])
 *                bytes each; written asynchronously, owned by the caller, kept alive while registered
 * On `compute_stream` (after the work that wrote cur_k / cur_v) a gather kernel per layer packs the
 * rounds into the device pool behind the staged rounds; `side_stream` waits for it and carries one
 * device-to-host copy per sequence.  The call returns without waiting; a later ra_kv_store_stage
 * that selects the new round is ordered behind the copy.  Needs d * element size to be a multiple
 * of 16 bytes (RA_ERR_UNSUPPORTED otherwise).  RA_ERR_OOM if staged rounds plus the new rounds
 * exceed the pool; nothing is enqueued or registered on any error found before the first launch.
 * A second call first waits (on the host) for the previous call's copies.
 */
int ra_kv_store_save_round(ra_kv_store* store, const int32_t* round_host, const int32_t* len_host,
                           const void* const* cur_k_layers, const void* const* cur_v_layers, int cur_cap,
                           void* const* host_kv, void* compute_stream, void* side_stream);
/* Block the host until the tensors of the last ra_kv_store_save_round are complete in host memory;
 * saved_bytes (may be NULL) receives the bytes that call moved. */
int ra_kv_store_save_wait(ra_kv_store* store, uint64_t* saved_bytes);

/*
 * KV-cache dropping (Sec. 3.4): rounds that are never selected are deleted rather than kept.
 * Every ra_kv_store_stage call counts one turn for each registered round of each sequence and one
 * hit for each round it selects; registering or saving a round resets its two counters.
 * A dropped round keeps its index as an empty round (length 0, no host tensor): a later selection
 * that names it stages nothing for it, and the caller may free its host tensor once the drop call
 * has returned.  Both drop calls return RA_ERR_STATE while rounds are staged.
 */
int ra_kv_store_round_activity(const ra_kv_store* store, int seq, int round, uint32_t* turns, uint32_t* hits);
int ra_kv_store_drop_round(ra_kv_store* store, int seq, int round);
/* Drops every round with no hit in at least min_turns turns.  dropped_idx host int32 [B][R_max]
 * receives the dropped rounds of each sequence in ascending order (-1 beyond), n_dropped host int32 [B]
 * their count.  The paper gives no such threshold; it is the caller's. */
int ra_kv_store_drop_inactive(ra_kv_store* store, uint32_t min_turns, int32_t* dropped_idx, int32_t* n_dropped);

#ifdef __cplusplus
}
#endif
#endif /* ROUND_ATTENTION_H */
