/*
 * eesd.h - C ABI of the MI355X (gfx950) library for the hot path of
 * Early-exiting Speculative Decoding (EESD).
 *
 * One context decodes one sequence (batch 1).  A decoding round is
 *
 *     eesd_draft_step x K  ->  eesd_verify  ->  eesd_accept  ->  eesd_rollback
 *
 * and eesd_generate runs the paper's whole loop (Algorithm 1) on top of those
 * calls, with the draft length K of every round chosen on the host by the
 * Beta-posterior Thompson-sampling controller (Section 3.3, Algorithm 2).
 *
 * Conventions that hold for every call:
 *   - returns EESD_OK (0) or a negative eesd_status; never throws, never aborts;
 *   - out-parameters are written only on success;
 *   - "device" pointers are HIP device memory of the current device, "host"
 *     pointers are ordinary host memory;
 *   - all work is enqueued on the HIP stream given to eesd_create; calls that
 *     return a value to the host synchronise that stream, the others do not;
 *   - a context is not thread-safe.
 *
 * Model: a LLaMA-style pre-norm decoder (RMSNorm, rotary embedding on
 * half-split pairs (j, j + head_dim/2), grouped-query causal attention,
 * SwiGLU feed-forward).  The draft model of Section 3.1, Eq. 1 is the first
 * n_draft_layers decoder layers of the target (same weights, same KV cache)
 * followed by one extra decoder layer, an RMSNorm and an own LM head.
 */
#ifndef EESD_H
#define EESD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct eesd_ctx eesd_ctx; /* opaque; created by eesd_create, freed by eesd_destroy */

typedef enum eesd_status {
    EESD_OK = 0,
    EESD_EINVAL = -1,  /* null pointer, bad shape, token id outside [0, vocab) */
    EESD_ENOMEM = -2,  /* device or host allocation failed */
    EESD_ESTATE = -3,  /* call out of order (see the state machine below) */
    EESD_ERANGE = -4,  /* sequence, draft count or schedule exceeds a configured limit */
    EESD_EDEVICE = -5  /* a HIP call failed; eesd_last_error has the text */
} eesd_status;

enum { EESD_DTYPE_F32 = 0, EESD_DTYPE_BF16 = 1 };
enum { EESD_WEIGHTS_ROW_MAJOR = 0, EESD_WEIGHTS_TILED = 1 };
enum { EESD_PACK_PLAIN = 0, EESD_PACK_GATE_UP = 1, EESD_PACK_QKV = 2 };
enum { EESD_TS_BETA = 0, EESD_TS_FIXED = 1, EESD_TS_SCHEDULE = 2, EESD_TS_CALI = 3 };
enum { EESD_GEMM_AUTO = 0, EESD_GEMM_VALU = 1, EESD_GEMM_MFMA = 2 };

typedef struct eesd_config {
    int32_t n_layers;        /* L: decoder layers of the target model */
    int32_t n_draft_layers;  /* N: leading layers the draft model shares with it (1 <= N < L) */
    int32_t d_model;
    int32_t n_heads;         /* query heads */
    int32_t n_kv_heads;      /* key/value heads; n_heads % n_kv_heads == 0 */
    int32_t head_dim;        /* even; 64 or 128 for the bf16 path */
    int32_t d_ff;            /* SwiGLU width */
    int32_t vocab;
    float rms_eps;
    float rope_base;
    int32_t dtype;           /* EESD_DTYPE_*: storage type of the weights and of the KV cache;
                                accumulation, residual stream, logits and probabilities are fp32 */
    int32_t max_seq;         /* most tokens the KV cache can hold */
    int32_t kv_page;         /* tokens per KV page (power of two, >= 16); bf16 caches with pages of 32 tokens or more are kept in
                                the order of the attention's MFMA operands (contiguous reads), smaller pages row by row */
    int32_t k_cap;           /* most draft tokens per round, 1..15 */
    float temperature;       /* 0 => greedy (Section 4.1 footnote); > 0 => sampling at that temperature */
    uint64_t seed;           /* seed of the counter-based uniforms (draft, accept, resample, controller) */
    double ts_alpha0;        /* prior Beta(alpha0, beta0) of the controller (Algorithm 2, step 1) */
    double ts_beta0;
    int32_t ts_mode;         /* EESD_TS_BETA: Algorithm 2; EESD_TS_FIXED: always k_cap drafts
                                (the "w/o TS" ablation); EESD_TS_SCHEDULE: eesd_set_draft_schedule;
                                EESD_TS_CALI: Algorithm 3 (needs eesd_set_calibration) */
    int32_t ts_update;       /* reading of Eq. 3-4: 0: r = a, n = min(a+1, K) (drafts the target judged);
                                1: |Q_v| = a+1 taken literally, r = a, n = min(a+2, K) */
    int32_t gemm_path;       /* EESD_GEMM_*: AUTO picks per pass; the others force one kernel family */
    int32_t tree_width;      /* 0 or 1: one draft token per step (Algorithm 1).  2..4: candidate tree (Section 4.3,
                                tree-attention table): every draft step proposes its tree_width most likely tokens,
                                the first is drafted on from, the others are leaves; one verify pass judges all
                                1 + K * tree_width rows under a tree mask and keeps only candidates that are the
                                target's top-1 token.  Needs temperature == 0 and 1 + k_cap * tree_width <= 16 */
    int32_t verify_reuse;    /* 1: eesd_verify takes the layer-N hidden states of rows 0..K-1 from the draft steps that
                                computed them (Section 3.1: the draft model IS the target's first N layers) and runs
                                layers 1..N for the last draft token only; 0: all L layers on all K+1 rows.  Same
                                result up to rounding; ignored in tree mode */
    int32_t weight_layout;   /* EESD_WEIGHTS_ROW_MAJOR, or EESD_WEIGHTS_TILED: every matrix except tok_emb and the norm gains
                                was rearranged by eesd_pack_weight (bf16 models, MFMA kernel family only) */
    int32_t logits_bf16;     /* 1: both LM heads store their logits as bf16 (rounded to nearest even from the fp32 sums) and the
                                softmax / sampling / accept kernels read those; probabilities stay fp32.  bf16 models, MFMA
                                kernel family only.  0: fp32 logits */
} eesd_config;

/* One decoder layer.  Every matrix is row-major [out][in] in the configured dtype. */
typedef struct eesd_layer_weights {
    const void* attn_norm;  /* [d_model] */
    const void* wqkv;       /* [(n_heads + 2 n_kv_heads) head_dim][d_model]: q heads, k heads, v heads */
    const void* wo;         /* [d_model][n_heads head_dim] */
    const void* ffn_norm;   /* [d_model] */
    const void* w_gate_up;  /* [2 d_ff][d_model]: gate rows, then up rows */
    const void* w_down;     /* [d_model][d_ff] */
} eesd_layer_weights;

/* DEVICE pointers, BORROWED: the caller owns the memory and keeps it alive and
 * unchanged until eesd_destroy.  `layers` itself is a host array of n_layers entries
 * (copied by eesd_create). */
typedef struct eesd_weights {
    const void* tok_emb;                /* [vocab][d_model] */
    const eesd_layer_weights* layers;   /* host array, n_layers entries */
    const void* final_norm;             /* [d_model] */
    const void* lm_head;                /* [vocab][d_model], target head */
    eesd_layer_weights ee_layer;        /* the early-exit decoder layer (Eq. 1, Transformer^e) */
    const void* ee_norm;                /* [d_model] */
    const void* ee_head;                /* [vocab][d_model], draft head W of Eq. 1 */
} eesd_weights;

/* Counters of Section 4.1 "Metrics" / Appendix D and the time buckets of the
 * paper's breakdown table (drafting, verification, sampling, others). */
typedef struct eesd_stats {
    int64_t rounds;
    int64_t drafted;     /* N_all_draft */
    int64_t accepted;    /* N_right */
    int64_t generated;   /* L: tokens returned by eesd_generate (0 outside it) */
    double v_d, r_d, hm; /* acceptance rate, draft proportion, their harmonic mean in percent */
    double alpha, beta;  /* current posterior of the controller */
    double ms_draft, ms_verify, ms_accept, ms_other; /* filled by eesd_generate */
} eesd_stats;

/*
 * State machine:  created --prefill--> ready --draft_step (0..k_cap times)--> ready
 *                 ready --verify--> verified --accept--> accepted --rollback--> ready
 * Any other order returns EESD_ESTATE.  eesd_prefill may be called in any state
 * and starts a new sequence.
 */

/* Algorithm 1, REQUIRE line: the target model, the draft model (the same weights' first N layers, the early-exit
 * layer and its head: Section 3.1), the hyper-parameters of the controller and the decoding limits, as one context.
 * Allocates the paged KV cache (L target layers, the first N shared with the draft
 * model, plus the early-exit layer's own cache) and all scratch memory on the current
 * device.  hip_stream is a hipStream_t (NULL = the default stream).  Weights are
 * borrowed.  Errors: EESD_EINVAL (null pointer, unsupported shape), EESD_ENOMEM. */
int eesd_create(const eesd_config* cfg, const eesd_weights* w, void* hip_stream, eesd_ctx** out);
void eesd_destroy(eesd_ctx* ctx);

/* Runs the n prompt tokens (HOST array) through all L target layers, fills the KV
 * cache of every layer and of the early-exit layer, and draws the first generated
 * token from the target (argmax when greedy).  That token becomes the pending token
 * of the first round (Algorithm 1 starts from Q_g = prompt).  Synchronises.
 * Errors: EESD_EINVAL (n < 1, token out of range), EESD_ERANGE (n + k_cap + 1 > max_seq). */
int eesd_prefill(eesd_ctx* ctx, const int32_t* prompt, int32_t n, int32_t* first_token);

/* Algorithm 1 step 6: one draft token from the draft model (Eq. 1) given everything
 * committed and drafted so far.  The token and its probability row stay on the device;
 * if tok_or_null is not NULL the call synchronises and returns the token.
 * Errors: EESD_ESTATE, EESD_ERANGE (k_cap drafts already made, or cache full). */
int eesd_draft_step(eesd_ctx* ctx, int32_t* tok_or_null);

/* Algorithm 1 step 15: ONE target forward over [pending, d_1..d_K] (K = drafts since
 * the last rollback, K = 0 allowed: a plain auto-regressive step), against the paged
 * KV cache.  Leaves K+1 rows of target logits on the device.  Does not synchronise. */
int eesd_verify(eesd_ctx* ctx);
/* Tree mode (tree_width = w >= 2): the block has 1 + K*w rows - row 0 the pending token, rows
 * 1 + (i-1)*w + j the j-th candidate of depth i (j = 0: the one drafted on from).  A row is
 * written to cache slot base + row, rotated for position base + depth, and attends to the cache,
 * row 0, the j = 0 rows of the depths above it, and itself. */

/* Algorithm 1, steps 15-17, on the logits eesd_verify left: which drafts the target keeps, and the token it
 * contributes after them.  Greedy (Section 4.1, footnote: one top-1 candidate per step, kept while consistent with
 * the target's top-1 token): drafts are kept while equal to the target's top-1; the
 * next token is the top-1 after them.  Sampling (the speculative-sampling rule of the works the paper builds on,
 * which keeps the output distributed as auto-regressive decoding, Section 1): draft i is accepted iff
 * u_i * q_i(d_i) < p_i(d_i); the first rejected position is resampled from
 * norm(max(0, p - q)); if all K pass, a bonus token is drawn from p_{K+1}.
 * uniforms_or_null: HOST array of K+1 doubles in [0,1) (K accept tests, then the
 * resample/bonus draw); NULL uses the context's counter-based uniforms.
 * Synchronises; returns a = *n_accepted and y = *next_token. */
int eesd_accept(eesd_ctx* ctx, const double* uniforms_or_null, int32_t* n_accepted, int32_t* next_token);

/* The tokens the last eesd_accept kept, in order (without the next token): the first a drafts,
 * or, in tree mode (Section 4.3), the tokens of the accepted root path, whose last node may be
 * a leaf candidate.  In tree mode eesd_accept has already moved the accepted nodes' keys and
 * values to their final positions in every cache, uniforms are ignored, and eesd_rollback takes
 * at most the a it returned.  toks: HOST array of at least `cap` entries; *n receives a.
 * Valid between eesd_accept and the next eesd_accept. */
int eesd_accepted_tokens(eesd_ctx* ctx, int32_t* toks, int32_t cap, int32_t* n);

/* Keeps the accepted prefix (Algorithm 1, steps 16-18; the rejected and the unjudged drafts are
 * discarded, Appendix F): the valid length of every layer's KV cache (and of the early-exit layer's)
 * becomes base + n_accepted + 1, whole pages past it return to the pool, the token eesd_accept
 * returned becomes the pending token, and the controller's posterior is updated (Eq. 3-4).
 * n_accepted must be the a that eesd_accept returned - any other count would commit drafts the
 * accept rule rejected, or drop ones it kept, and the output would no longer be distributed as
 * auto-regressive decoding - else EESD_ERANGE. */
int eesd_rollback(eesd_ctx* ctx, int32_t n_accepted);

/* Algorithm 1 end to end: prefill, then rounds until max_new tokens exist.  prompt: HOST,
 * n_prompt tokens; out: HOST buffer of at least max_new entries; *n_out = tokens written
 * (= max_new).  stats_or_null receives the counters and time buckets of this call.
 * Errors: as the calls above; EESD_ERANGE if n_prompt + max_new + k_cap + 1 > max_seq. */
int eesd_generate(eesd_ctx* ctx, const int32_t* prompt, int32_t n_prompt, int32_t max_new,
                  int32_t* out, int32_t* n_out, eesd_stats* stats_or_null);

int eesd_get_stats(const eesd_ctx* ctx, eesd_stats* out);
/* Text of the last error of this context (never NULL; static text if ctx is NULL). */
const char* eesd_last_error(const eesd_ctx* ctx);

/* ---- controller input -------------------------------------------------------------- */
/* EESD_TS_SCHEDULE: K of round r (r = 0, 1, ...) is k_per_round[r] (HOST, copied),
 * clipped to [1, min(k_cap, tokens still wanted)]; rounds past the end use the last entry. */
int eesd_set_draft_schedule(eesd_ctx* ctx, const int32_t* k_per_round, int32_t n_rounds);
/* K the controller would choose for the coming round given k_max (consumes its random draws
 * exactly as eesd_generate does). */
int eesd_next_draft_len(eesd_ctx* ctx, int32_t k_max, int32_t* k_out);

/* ---- host-only pieces (no device needed) ------------------------------------------------- */
/* The counter-based uniform of (seed, stream, round, slot, sub): top 53 bits of the splitmix64
 * output function of the packed key, times 2^-53.  Streams: 1 draft, 2 accept, 3 resample,
 * 4 controller theta, 5 controller chi. */
double eesd_host_uniform(uint64_t seed, int32_t stream, int64_t round, int32_t slot, int32_t sub);
/* K that Algorithm 2 (steps 5-14) draws for `round` from the posterior Beta(alpha, beta), at most
 * k_max.  Returns K >= 1, or EESD_EINVAL. */
int eesd_host_draw_k(double alpha, double beta, uint64_t seed, int64_t round, int32_t k_max);
/* Posterior update of Eq. 3-4 in place (reading as eesd_config.ts_update). */
int eesd_host_ts_update(double* alpha, double* beta, int32_t n_accepted, int32_t n_drafted, int32_t reading);
/* Where the operand-order layouts keep an element, as the kernels compute it (for tests of the layouts; -1 on bad
 * arguments).  what = 0: key of slot a (position inside its KV page), channel b, head_dim n -> element offset inside one
 * KV head's block of the page; 1: the same for a value; 2: activation row a, column b of a prefill block with 32 n
 * columns -> element offset inside the block's buffer; 3 / 4: first row / number of rows of row group a of a tile-major
 * matrix of b rows (a multiple of 16) on a device of n compute units; 5: the number of row groups of that matrix. */
int64_t eesd_host_layout_offset(int32_t what, int32_t a, int32_t b, int32_t n);

/* ---- Thompson sampling with calibration (Section 3.3 Eq. 5-8, Algorithm 3) ------------ */
/* The predictor of Eq. 5 and the hyper-parameters of the Gaussian posterior.  w and wp are DEVICE
 * pointers, BORROWED until eesd_destroy, row-major [out][in] in the model's storage type. */
typedef struct eesd_calibration {
    const void* w;       /* W^1..W^n_mats: [n_mats][d_model][d_model]; draft step i uses W^min(i, n_mats).  Each matrix
                            in the context's weight_layout (EESD_PACK_PLAIN) */
    const void* wp;      /* W_p: [2][2 d_model]; its input is (W^i H_t^(T), H_{t+i}^(D)) */
    int32_t n_mats;      /* 1..10 */
    int32_t update;      /* reading of Eq. 8: 0: theta_hat is the mean of the chi the target judged (a successes out of
                            min(a+1, K)); 1: as printed (a successes out of a) */
    double sigma_m;      /* > 0: standard deviation of the predictor's error */
    double sigma_s;      /* > 0: standard deviation of a round's sample mean */
    double theta_hat0;   /* initial observed mean; counts as one observation */
} eesd_calibration;

/* Installs the predictor; required before the first round when ts_mode == EESD_TS_CALI (any
 * ts_mode may install it to use eesd_cali_score).  Resets the controller's observations. */
int eesd_set_calibration(eesd_ctx* ctx, const eesd_calibration* cal);

/* Eq. 5 for the draft step just made (i = drafts since the last rollback >= 1):
 * theta_M = logistic(z_1 - z_0), z = W_p (W^min(i,n_mats) H_t^(T), H^(D)), where H_t^(T) is the target's
 * last-layer hidden state at the last verified position (the one whose output is the pending
 * token) and H^(D) the draft model's last-layer hidden state of this step.  Synchronises. */
int eesd_cali_score(eesd_ctx* ctx, float* theta_m);

/* Host-only parts of Algorithm 3 (no GPU needed).
 * decide: mu, sigma^2 by Eq. 6-7 from (theta_m, theta_hat, n verifications), theta = mu + sigma z with z
 * a Box-Muller normal of the context's counter-based uniforms (stream TS_THETA, subs 0 and 1),
 * chi = u < theta with u of stream TS_CHI.  update: Eq. 8 in the chosen reading, n += 1. */
int eesd_host_cali_decide(double sigma_m, double sigma_s, double theta_hat, int64_t n, double theta_m, uint64_t seed,
                          int64_t round, int32_t slot, double* theta, int32_t* chi);
int eesd_host_cali_update(double* theta_hat, double* weight, int64_t* n, int32_t n_accepted, int32_t n_drafted, int32_t reading);

/* =====================================================================================================
 * TEST AND BENCHMARK HOOKS - not part of decoding.  Everything from here to the stand-alone kernels reads internal
 * state, forces tokens, times launches or turns launch-shape knobs; no product code path needs any of it.
 * ===================================================================================================== */
enum {
    EESD_READ_DRAFT_LOGITS = 0,  /* index = draft slot i (0-based): vocab floats */
    EESD_READ_DRAFT_PROBS = 1,   /* index = draft slot: vocab floats (sampling mode only) */
    EESD_READ_VERIFY_LOGITS = 2, /* index = verify row i (0..K): vocab floats */
    EESD_READ_KV_K = 3,          /* index = layer (n_layers = the early-exit layer): kv_len x n_kv_heads x head_dim floats */
    EESD_READ_KV_V = 4,
    EESD_READ_TOKENS = 5,        /* the block [pending, d_1..d_K] as int32 */
    EESD_READ_KV_LEN = 6,        /* one int32 */
    EESD_READ_PAGE_TABLE = 7,    /* ceil(max_seq / kv_page) int32 (-1 = unmapped) */
    EESD_READ_TREE_TOKENS = 8,   /* tree mode: the tokens of the block's 1 + K * tree_width rows as int32 */
    EESD_READ_CALI_STATE = 9,    /* three doubles: theta_hat, the observations behind it, verifications n */
    EESD_READ_VERIFY_PROBS = 10, /* index = verify row i: vocab floats, the probability row the last eesd_accept judged draft i on
                                    (sampling mode; rows 0..a: the one-workgroup accept kernel stops at the first rejection, the kernels that take all
                                    rows at once - "smp_spread" under eesd_set_tunable - fill the rows past a as well) */
    EESD_READ_LAUNCH_COUNTS = 11 /* 20 int32: weight-streaming product launches since eesd_create, [kernel][epilogue] with kernel
                                    0 = VALU family, 1 = one workgroup per 16-row tile, 2 = one workgroup per row group,
                                    3 = tiles sharing the activations through LDS, 4 = prefill GEMM on tile-major weights;
                                    epilogue 0 LM head, 1 residual, 2 SwiGLU, 3 QKV */
};
/* Copies internal state to HOST memory as fp32 / int32.  Synchronises.  n_tokens limits KV reads. */
int eesd_debug_read(eesd_ctx* ctx, int what, int index, int32_t n_tokens, void* host_dst, size_t bytes);
/* Teacher forcing: the next n draft steps emit toks[i] instead of the token they sample
 * (their logits and probability rows are still those of the draft model). */
int eesd_debug_force_drafts(eesd_ctx* ctx, const int32_t* toks, int32_t n);
/* Teacher forcing: replaces the pending token (state must be ready). */
int eesd_debug_force_pending(eesd_ctx* ctx, int32_t tok);
/* Teacher forcing: eesd_rollback with ANY 0 <= n_accepted <= K (tree mode: <= the accepted depth) and a pending
 * token of the caller's choice, so that a test can keep the library on another implementation's token stream.
 * NOT lossless: never part of decoding. */
int eesd_debug_rollback(eesd_ctx* ctx, int32_t n_accepted, int32_t pending_tok);
/* Fills KV rows [0, n_tokens) of every cache with a cheap deterministic pattern and sets
 * kv_len = n_tokens, pending = tok: a stand-in for a prefilled cache in micro-benchmarks. */
int eesd_debug_fill_cache(eesd_ctx* ctx, int32_t n_tokens, int32_t pending_tok);

/* Times one class of weight-streaming product launches with HIP events on the context's
 * stream: family 0 = VALU (M = 1 / fp32), 1 = MFMA (bf16, M >= 2); epilogue_kind 0 = LM head,
 * 1 = residual (attention output and FFN down), 2 = SwiGLU (gate/up), 3 = QKV; in_dim filters
 * on the reduction length (0 = any).  _end synchronises and returns launches seen and their
 * summed duration (at most 8192 launches are timed). */
int eesd_debug_profile_begin(eesd_ctx* ctx, int32_t family, int32_t epilogue_kind, int32_t in_dim);
int eesd_debug_profile_end(eesd_ctx* ctx, int32_t* n_launches, double* total_ms);

/* Copies `bytes` (a multiple of 16) DEVICE to DEVICE with a plain streaming kernel named
 * eesd_calibration_copy_kernel: hardware-counter runs are scaled by what the same counters read
 * for this kernel, whose traffic is known (bytes read + bytes written).  Does not synchronise. */
int eesd_debug_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/* Launch-shape knobs for benchmark sweeps.  PROCESS-WIDE: they change the launch heuristics of every context of the
 * process, are not synchronised with running calls and are meant for single-threaded sweeps only (0, or -1 for
 * "fuse_norm", restores the built-in heuristic):
 * "valu_nw", "valu_tpw", "valu_rp", "mfma_nw", "mfma_ksplit", "fuse_norm", "mfma_tile", "tile_kc", "tile_nwt", "pf_kc",
 * "pf_rows" (rows of a prefill block on tile-major weights, 128 / 256 / 512; read by eesd_create), "grp_minsteps" (row-group residual products take 4 waves below this many steps per wave), "pf_ts", "pf_nbw" (tile slots per
 * workgroup and 16-token blocks per wave of the prefill GEMM), "pf_merge" (0: the 4-row tails of 20-row groups take a tile slot each instead of sharing one), "attn_split", "mfma_min_m", "nw_plain", "nw_resid", "nw_swiglu", "nw_qkv" (waves per workgroup of the per-tile
 * product by epilogue), "smp_spread" (the sampling tails of the draft step and of the accept at temperature > 0: 1 = three
 * kernels over 64 workgroups per row, 0 = one workgroup, -1 = built-in: spread for vocabularies of 4096 to 65536 entries). */
int eesd_set_tunable(const char* name, int value);

/* ---- stand-alone kernels (device buffers in, host results out) ----------------------- */
/* The accept/resample decision on given probability rows (sampling) or logit rows (greedy).
 * p_rows: DEVICE fp32 [K+1][vocab]; q_rows: DEVICE fp32 [K][vocab] (ignored when greedy);
 * drafts: DEVICE int32 [K]; uniforms: HOST double [K+1]; result: HOST int32[2] = {a, y}. */
int eesd_op_accept(const float* p_rows, const float* q_rows, const int32_t* drafts, const double* uniforms,
                   int32_t K, int32_t vocab, int32_t greedy, void* hip_stream, int32_t* result);
/* The verification tail as eesd_accept runs it, on given logit rows: p_logits DEVICE [K+1][vocab], fp32 or (logits_bf16 = 1)
 * bf16; row i becomes softmax(p_logits[i] / temperature) in p_rows[i] (DEVICE fp32 [K+1][vocab]; rows 0..a are always written, rows
 * past the first rejection only by the kernels that handle all rows at once, see "smp_spread"), draft i is accepted iff u_i q_i(d_i) < p_i(d_i), the first rejected position is resampled
 * from norm(max(0, p - q)), K acceptances draw the bonus token from row K.  temperature 0: greedy on the logits, p_rows,
 * q_rows and uniforms unused.  q_rows, drafts, uniforms, result as eesd_op_accept. */
int eesd_op_accept_logits(const void* p_logits, int32_t logits_bf16, float* p_rows, const float* q_rows, const int32_t* drafts,
                          const double* uniforms, int32_t K, int32_t vocab, float temperature, void* hip_stream, int32_t* result);
/* softmax(logits / temperature) of one DEVICE fp32 row into probs (DEVICE fp32), then an
 * inverse-CDF draw with u (temperature 0: argmax, probs untouched).  *token: HOST. */
int eesd_op_softmax_sample(const float* logits, float* probs, int32_t vocab, float temperature, double u,
                           void* hip_stream, int32_t* token);
/* Y[m][r] = sum_k X[m][k] W[r][k]: the weight-streaming product of the draft (M = 1), verify
 * (M = K+1 <= 16) and prefill (bf16 MFMA family, in % 256 == 0: M <= 128 with out % 64 == 0 on row-major weights,
 * M <= 512 with out % 16 == 0 on tile-major weights) passes without prologue or epilogue.  W: DEVICE [out][in] in dtype (weight_layout EESD_WEIGHTS_TILED:
 * packed with kind EESD_PACK_PLAIN); X: DEVICE fp32 [M][in]; Y: DEVICE fp32 [M][out]; path: EESD_GEMM_*.
 * The bf16 path stages the activation rows in one buffer per process: calls that overlap on the GPU race. */
int eesd_op_gemm(const void* W, const float* X, float* Y, int32_t M, int32_t out, int32_t in,
                 int32_t dtype, int32_t path, int32_t weight_layout, void* hip_stream);

/* eesd_op_gemm for callers that cannot allocate (code under HIP graph capture, serving loops and harnesses that
 * forbid hipMalloc): the same product on bf16 weights (MFMA kernel family; W, X, Y, weight_layout as above), but
 * the bf16 staging rows of the activations live in a fixed 1 MiB device array of this library (per GPU, held until
 * the process ends) instead of a buffer that eesd_op_gemm grows with hipMalloc.  No allocation of any kind is made.
 * Limits: 1 <= M <= 16, 128 <= in <= 32768, else EESD_ERANGE; out % 16 == 0, in % 128 == 0 else EESD_EINVAL.
 * All calls on one GPU share that array, which keeps the last call's contents (nothing in it has to start at zero:
 * rows >= M are never used): calls that overlap on one GPU - different streams, different threads - race.
 * Does not synchronise. */
int eesd_op_gemm_noalloc(const void* W, const float* X, float* Y, int32_t M, int32_t out, int32_t in,
                         int32_t weight_layout, void* hip_stream);

/* Rearranges one bf16 weight matrix (DEVICE, row-major [out_rows][in_dim]) into the tile-major layout
 * the MFMA kernel family streams with contiguous reads (EESD_WEIGHTS_TILED).  The rows are dealt to row
 * groups in units of 4 rows; a group is stored contiguously as blocks of 32 columns, each block holding
 * the group's tiles of 16 rows (the last one possibly shorter) in the lane order of the MFMA operand.
 * Matrices with at most one 16-row tile per compute unit of the CURRENT DEVICE, or with at least four,
 * keep one tile per group; those in between are dealt to exactly one group per compute unit, so that
 * every CU streams the same number of bytes (the layout therefore depends on the device's CU count:
 * pack on the device that will run the model).  Which rows form a tile follows the epilogue the matrix
 * feeds: kind EESD_PACK_PLAIN (LM heads, attention output, FFN down, the calibration matrices):
 * consecutive rows; EESD_PACK_GATE_UP (fused gate|up, out_rows = 2 d_ff): 8 gate rows and their 8 up
 * rows; EESD_PACK_QKV (fused q|k|v; head_dim given): 8 rows of a head and their rotary partners
 * head_dim/2 further.  dst: DEVICE, out_rows * in_dim elements, must not overlap src.
 * out_rows % 16 == 0 (QKV: % head_dim), in_dim % 128 == 0.  Does not synchronise. */
int eesd_pack_weight(const void* src, void* dst, int32_t out_rows, int32_t in_dim, int32_t kind, int32_t head_dim,
                     void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* EESD_H */
