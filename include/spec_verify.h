/*
 * spec_verify.h - C ABI of the batched speculative-verification step for
 * AMD Instinct MI355X (gfx950).
 *
 * The step is the data-parallel hot path behind goodput-driven speculation
 * control (arXiv 2406.14066): for B requests, request b having k_b draft
 * tokens and a paged KV cache of kv_len[b] tokens,
 *   (a) "score": lookahead attention of the k_b+1 query positions against the
 *       request's KV cache, causal inside the draft (Section 2.2: position
 *       n+i is conditioned on x_1..x_{n+i-1}; Section 4: all k+1 positions are
 *       scored in one forward pass; Eq. 3 attributes the context-dependent
 *       part of that pass to loading the KV cache), and
 *   (b) "accept": rejection sampling over the vocabulary (Section 4's
 *       acceptance phase), giving the number m_b of accepted draft tokens and
 *       the bonus token that corrects the first wrong draft token or extends a
 *       fully accepted draft, so the step emits m_b+1 tokens (Section 2.2),
 *       plus the counters behind goodput (Eq. 1) and the acceptance-rate
 *       estimate that feeds Eq. 4.
 *
 * Conventions
 *   - Pointers are DEVICE pointers unless the name starts with host_.
 *   - Ownership: the library allocates and frees nothing.  The caller owns all
 *     buffers and the workspace, and keeps them valid until the stream has
 *     finished the call.
 *   - Calls enqueue work on `hip_stream` (a hipStream_t; NULL = the default
 *     stream) and return without synchronising.
 *   - Arguments are validated on the host before anything is launched; a
 *     failed validation launches nothing.  A launch failure is SPEC_EHIP.
 *     What only the device can see (lengths, block-table entries and draft
 *     tokens in device memory) is checked again by the kernels: an entry out of
 *     range is never used as an address, the request or test it belongs to is
 *     skipped or rejected, and the count of such findings is reported (see
 *     error_count and counters[6]).
 *   - Same inputs and same (philox_seed, philox_step) give the same outputs.
 *   - Limits: k_b <= SPEC_K_MAX, block_size == 16, d in {64, 128},
 *     Hq % Hkv == 0, Hq/Hkv <= 16, kv_len[b] >= q_len[b] >= 1.
 *   - Speed: bf16 runs on the matrix-instruction kernel, the whole step in one
 *     launch, for every draft length and group width within the limits (up to
 *     9 * 16 fused rows per KV head) and both head dims: fastest with pages in
 *     the SPEC_KV_MFMA layout; token-major pages take the same kernel, 3 to 8%
 *     slower up to 48 fused rows and about 20% slower beyond (V is transposed
 *     through LDS inside the kernel).  fp32 runs on plain, untuned kernels (two
 *     or three launches).  spec_verify_plan tells which path a call takes.
 */
#ifndef SPEC_VERIFY_H
#define SPEC_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPEC_K_MAX 8
#define SPEC_BLOCK_SIZE 16
#define SPEC_NUM_COUNTERS 8

typedef enum {
    SPEC_OK = 0,
    SPEC_EINVAL = -1,       /* malformed argument (null pointer, bad size, k_b > SPEC_K_MAX, ...) */
    SPEC_EUNSUPPORTED = -2, /* well-formed but outside the supported shapes/dtypes/layouts */
    SPEC_EWORKSPACE = -3,   /* workspace missing, misaligned or too small */
    SPEC_EHIP = -4          /* a HIP call failed */
} spec_status;

typedef enum { SPEC_F32 = 0, SPEC_BF16 = 1 } spec_dtype;

/*
 * Page layouts of the KV cache (the paper leaves the layout to the serving
 * engine's memory manager).  A page holds SPEC_BLOCK_SIZE consecutive tokens
 * of one request for all KV heads; logical token t of request b is in page
 * block_table[b][t / 16], slot t % 16.
 *   SPEC_KV_TOKEN_MAJOR: K and V are [num_blocks][Hkv][16][d].
 *   SPEC_KV_MFMA: bf16 only; both pools are tiled in the operand order of the
 *     gfx950 matrix instructions, so that each 16-byte-per-lane load of a
 *     wavefront is one contiguous 1 KB burst.
 *     K is [num_blocks][Hkv][d/8][16 tokens][8 dims]: element (token s, dim c)
 *       of a (page, head) is at (c/8)*128 + s*8 + c%8.
 *     V is [num_blocks][Hkv][d/32][4 token groups][16 dims][2 dim halves][4 tokens]:
 *       element (token s, dim c) is at
 *       ((((c/32)*4 + s/4)*16 + c%16)*2 + (c/16)%2)*4 + s%4.
 *     spec_kv_repack_mfma converts a token-major pool.
 */
typedef enum { SPEC_KV_TOKEN_MAJOR = 0, SPEC_KV_MFMA = 1 } spec_kv_layout;

/* Lookahead attention of the k_b+1 query positions (Section 2.2, Section 4). */
typedef struct {
    int32_t B;                  /* requests */
    int32_t Hq, Hkv;            /* query heads, KV heads (query head h reads KV head h / (Hq/Hkv)) */
    int32_t d;                  /* head dim: 64 or 128 */
    int32_t block_size;         /* must be SPEC_BLOCK_SIZE */
    int32_t num_blocks;         /* pages in the pool */
    int32_t max_blocks_per_req; /* row length of block_table */
    int32_t T;                  /* sum_b q_len[b], q_len[b] = k_b + 1 */
    int32_t qkv_dtype;          /* spec_dtype of q, k_cache, v_cache; out is fp32 */
    int32_t kv_layout;          /* spec_kv_layout */
    const void *q;              /* [T][Hq][d], rows packed by request: rows cu_q_len[b]..cu_q_len[b+1]-1
                                   (q, k_cache, v_cache and out must be 32-byte aligned: SPEC_EINVAL otherwise) */
    const void *k_cache;        /* page pool, see spec_kv_layout */
    const void *v_cache;
    const int32_t *block_table; /* [B][max_blocks_per_req]; entries past ceil(kv_len/16) are not read */
    const int32_t *kv_len;      /* [B] valid KV tokens, INCLUDING this step's q_len[b] new tokens:
                                   query j sits at position kv_len[b]-q_len[b]+j and sees keys 0..that */
    const int32_t *cu_q_len;    /* [B+1] exclusive prefix sum of q_len */
    float softmax_scale;        /* 0 means 1/sqrt(d) */
    float *out;                 /* [T][Hq][d] fp32 */
    const int32_t *host_kv_len;   /* HOST copy of kv_len, used to plan the split over the KV length
                                     (may be NULL if max_kv_len > 0) */
    const int32_t *host_cu_q_len; /* HOST copy of cu_q_len */
    /* Everything below may be zero / NULL. */
    int32_t max_kv_len;         /* Length bucket.  0: the launch is planned from host_kv_len and is valid for
                                   exactly those lengths.  > 0: the plan (split of the KV length, grid,
                                   workspace size) depends on the shapes, host_cu_q_len and this bound only;
                                   the kernels take the actual lengths from the device-side kv_len, so one
                                   captured launch (HIP graph) stays valid while the lengths change from
                                   step to step, as long as q_len[b] <= kv_len[b] <= max_kv_len.  host_kv_len,
                                   if given, is then only a hint (order of the work items) and is checked
                                   against the bound. */
    int32_t validate;           /* 1: also check host_block_table (if given) on the host: every entry of a
                                   page in use must be in [0, num_blocks), else SPEC_EINVAL */
    const int32_t *host_block_table; /* optional HOST copy of block_table, read only when validate == 1 */
    int64_t *error_count;       /* optional DEVICE counter [1], ADDED to: findings of the device-side checks
                                   (a request whose kv_len is below its q_len, above the planned bound or
                                   beyond its block-table row; a block-table entry outside [0, num_blocks)).
                                   Such a request's output rows are not written; a bad page reads as zeros.
                                   In spec_verify_step a NULL here means &reject->counters[6]. */
} spec_attn_args;

/*
 * Rejection sampling with bonus token (Section 4's acceptance phase; the
 * accept rule is the cited speculative-sampling method's: accept draft token
 * x_i iff u_i < p_i(x_i)/q_i(x_i), p = softmax(target row), q = softmax(draft
 * row); at the first rejection draw the next token from the normalised
 * positive part of p - q, after k_b acceptances draw it from the last target
 * row).
 *
 * Random numbers: Philox4x32-10, key = (seed low 32, seed high 32), counter =
 * (index, b, step low 32, (step bits 32..55) << 8 | stream).  Stream 0, index
 * i, word 0 gives the accept uniform u = (word >> 8) * 2^-24 in [0,1).  Stream
 * 1, index v >> 2, word v & 3 gives U' = ((word >> 8) + 1) * 2^-24 in (0,1];
 * the next token is argmax_v r_v / (-log U'_v) (an exponential race, i.e. a
 * draw with probability proportional to the weights r_v; weights 0 never win,
 * equal scores go to the lowest v).
 *
 * accept_mode selects the acceptance rule (Section 2.2 describes the greedy
 * one; Section 7 evaluates proposers that give tokens without a distribution):
 *   SPEC_ACCEPT_SAMPLE       the rule above; needs draft_logits.
 *   SPEC_ACCEPT_GREEDY       x_i is accepted iff it is the arg-max of target row
 *                            i (lowest id among equal maxima); the next token is
 *                            the arg-max of the row after the last accepted one.
 *                            No random numbers; draft_logits is ignored (may be
 *                            NULL); debug_u_ratio is not written.
 *   SPEC_ACCEPT_POINT_DRAFT  the rule above with q_i the point mass on x_i:
 *                            accept iff u_i < p_i(x_i); at the first rejection
 *                            draw from p with the rejected token removed.
 *                            draft_logits is ignored (may be NULL); debug_u_ratio
 *                            holds u and p_i(x_i).
 * Logits must not be NaN.
 */
typedef enum {
    SPEC_ACCEPT_SAMPLE = 0,
    SPEC_ACCEPT_GREEDY = 1,
    SPEC_ACCEPT_POINT_DRAFT = 2
} spec_accept_mode;

typedef struct {
    int32_t B, V, T;
    const float *target_logits;   /* [T][V]; request b owns rows cu_q_len[b] .. cu_q_len[b]+k_b */
    const float *draft_logits;    /* [T-B][V]; request b owns rows cu_q_len[b]-b .. +k_b-1; row i produced x_i.
                                     The rows of positions after a request's first rejection decide nothing
                                     (Section 4: the accept chain stops there) and may be left unread. */
    const int32_t *draft_tokens;  /* [T-B] */
    const int32_t *cu_q_len;      /* [B+1] */
    const int32_t *host_cu_q_len; /* HOST copy (validation and launch planning) */
    uint64_t philox_seed;
    uint64_t philox_step;
    int32_t *accepted_len;        /* [B] out: m_b in [0, k_b] (draft tokens only, bonus not counted);
                                     -1 for a request counted in counters[7] */
    int32_t *next_token;          /* [B] out: correction or bonus token; -1 for a request counted in counters[7] */
    int32_t *out_tokens;          /* optional [B][SPEC_K_MAX+1]: accepted tokens, next token, -1 padding */
    int64_t *counters;            /* [SPEC_NUM_COUNTERS], ADDED to (caller zeroes):
                                     [0] proposed  sum k_b
                                     [1] accepted  sum m_b
                                     [2] attempted sum min(m_b+1, k_b)  (accept tests evaluated)
                                     [3] emitted   sum (m_b+1)          (goodput numerator, Eq. 1)
                                     [4] near ties: evaluated accept tests with |u - p/q| < 1e-6
                                     [5] requests
                                     [6] findings of the device-side input checks: draft tokens outside
                                         [0, V) (such a token is rejected, never used as an index) and, in
                                         spec_verify_step, the attention half's findings (see error_count)
                                     [7] requests abandoned because a bounded wait inside the launch ran out
                                         (never in a healthy launch): all their outputs are -1 and they are
                                         not counted in [0]..[5] */
    double *debug_u_ratio;        /* optional [T-B][2]: u and p/q of each evaluated accept test, NaN otherwise */
    int32_t accept_mode;          /* spec_accept_mode */
    /* Cache bookkeeping after acceptance (Section 5.1, "KV Cache of Bonus Tokens"); all three
     * optional (NULL), kv_len is needed if either output is given: */
    const int32_t *kv_len;        /* [B] the attention's kv_len (includes this step's q_len positions) */
    int32_t *new_kv_len;          /* [B] out: kv_len - (k_b - m_b): the rejected tail is dropped; the next
                                     token is not in the cache yet (it is the next step's first query) */
    int32_t *draft_next_len;      /* [B] out: tokens the draft model's cache is behind by: 2 after full
                                     acceptance of k_b > 0 tokens (last draft token + bonus), else 1 */
    /* Everything below may be zero / NULL. */
    const uint64_t *philox_step_device; /* DEVICE [1]: if not NULL the step counter is read from here when the
                                     kernels run and philox_step is ignored, so that a captured launch draws
                                     fresh random numbers on every replay (the caller advances the word) */
    int32_t validate;             /* 1: also check host_draft_tokens (if given) on the host: SPEC_EINVAL if a
                                     token is outside [0, V) */
    const int32_t *host_draft_tokens; /* optional HOST copy of draft_tokens, read only when validate == 1 */
} spec_reject_args;

/* Host-only: bytes of workspace the three calls below need for these shapes
 * (either argument may be NULL).  Returns 0 if the arguments are malformed.
 * The workspace must be 256-byte aligned device memory; its contents need no
 * initialisation and are undefined afterwards. */
size_t spec_verify_workspace_bytes(const spec_attn_args *attn, const spec_reject_args *reject);

/* (a) only: writes attn->out. */
spec_status spec_verify_attn(const spec_attn_args *attn, void *workspace, size_t workspace_bytes,
                             void *hip_stream);

/* (b) only: writes accepted_len, next_token, out_tokens, debug_u_ratio; adds to counters. */
spec_status spec_reject_sample(const spec_reject_args *reject, void *workspace, size_t workspace_bytes,
                               void *hip_stream);

/* The whole step: (a) then (b) on one stream.  The logits do not depend on
 * attn->out inside this library (the layers between them belong to the model). */
spec_status spec_verify_step(const spec_attn_args *attn, const spec_reject_args *reject, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/*
 * The whole step for callers that cannot allocate or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments,
 * results and errors as spec_verify_step, but the workspace is a device array inside the
 * library (SPEC_STATIC_SCRATCH_BYTES per GPU, held by every GPU the library runs on until the
 * process ends).  The call allocates and frees nothing.
 *   - A step whose workspace (spec_verify_workspace_bytes) exceeds SPEC_STATIC_SCRATCH_BYTES is
 *     refused with SPEC_EWORKSPACE before anything is launched; use spec_verify_step then.
 *   - The first call on a GPU resolves the array's device address (one runtime query, no
 *     allocation); make that call outside stream capture.
 *   - All calls on one GPU share that GPU's array, which keeps the previous call's contents
 *     (nothing in it has to start at zero: every record carries its call's tag).  Calls that
 *     overlap in time on one GPU (two streams, two threads) race on it; calls on one stream
 *     do not.
 */
#define SPEC_STATIC_SCRATCH_BYTES (16u << 20)
spec_status spec_verify_step_static(const spec_attn_args *attn, const spec_reject_args *reject, void *hip_stream);

/*
 * Host-only: how the library would run this step (either argument may be NULL), for
 * callers and tests that want to know which kernel a shape takes.
 */
#define SPEC_PATH_NONE 0
#define SPEC_PATH_MFMA 1     /* matrix-instruction attention inside the one-launch step kernel */
#define SPEC_PATH_GENERIC 2  /* scalar attention kernel, plus a merge kernel when a request is split (fp32) */
typedef struct {
    int32_t attn_path;       /* SPEC_PATH_* */
    int32_t row_tiles;       /* 16-row tiles of query rows per wavefront (matrix path, 1..3) */
    int32_t row_groups;      /* groups of wavefronts inside an attention block (1, 2 or 4): with more than
                                48 fused rows per KV head the block's wavefronts split the rows instead of
                                the pages and read every page side by side, so K and V still cross the
                                memory interface once */
    int32_t chunk_tokens;    /* bound of the tokens per chunk of the split over the KV length */
    int32_t max_chunks;      /* chunks of the longest request the plan allows for */
    int32_t launches;        /* kernel launches of the step */
    int32_t early_stop;      /* 1: statistics in position order, rows after a first rejection unread */
    int32_t stat_segments, race_segments;
    int32_t attn_blocks, reject_blocks;
    int32_t reserved;
    uint64_t workspace_bytes;
} spec_plan_info;
spec_status spec_verify_plan(const spec_attn_args *attn, const spec_reject_args *reject, spec_plan_info *info);

/* The tuning switches of the planner (environment variables SPEC_VERIFY_*) are read once, at
 * the first call; this re-reads them (for sweeps and tests that change them in-process). */
void spec_verify_reload_env(void);

/* Host-only validation, exactly what the calls above run first. */
spec_status spec_validate_attn(const spec_attn_args *attn);
spec_status spec_validate_reject(const spec_reject_args *reject);

/*
 * The step before the path (Section 5.1): the K and V rows of this step's query
 * positions enter the paged cache.  Row cu_q_len[b] + j of new_k / new_v
 * ([T][Hkv][d], same dtype as the cache) is written to token position
 * kv_len[b] - q_len[b] + j of request b, through the block table, in the given
 * page layout.  Everything else in the pools is left as it is.  Device pointers;
 * host_kv_len / host_cu_q_len are HOST copies used for validation only.
 * SPEC_EINVAL if a position falls outside the request's block-table row, or if new_k, new_v or
 * a pool is not 32-byte aligned (rows move as vectors of 8 elements).
 */
typedef struct {
    int32_t B, Hkv, d, num_blocks, max_blocks_per_req, T;
    int32_t dtype;                /* spec_dtype */
    int32_t kv_layout;            /* spec_kv_layout (SPEC_KV_MFMA: bf16, d % 32 == 0) */
    const void *new_k, *new_v;    /* [T][Hkv][d] */
    void *k_cache, *v_cache;      /* the pools, written in place */
    const int32_t *block_table;   /* [B][max_blocks_per_req] */
    const int32_t *kv_len;        /* [B], INCLUDING the rows being appended */
    const int32_t *cu_q_len;      /* [B+1] */
    const int32_t *host_kv_len, *host_cu_q_len;
    int64_t *error_count;         /* optional DEVICE counter [1], ADDED to: rows not written because the
                                     device-side position fell outside the block-table row or its page
                                     index outside [0, num_blocks) */
} spec_kv_append_args;
spec_status spec_kv_append(const spec_kv_append_args *args, void *hip_stream);

/* Re-tile a token-major bf16 page pool [num_blocks][Hkv][16][d] into the
 * SPEC_KV_MFMA layout (dst_k, dst_v; same byte sizes; must not alias the sources). */
spec_status spec_kv_repack_mfma(const void *src_k, const void *src_v, void *dst_k, void *dst_v,
                                int32_t num_blocks, int32_t Hkv, int32_t d, void *hip_stream);

/*
 * Host-side speculation control (Section 4.1, "Using Goodput for Speculation"; no GPU
 * work, no device pointers; all pointers are HOST pointers owned by the caller).
 *
 *   goodput (Eq. 1)     generated tokens of a step / time of the step
 *   time (Eq. 2, 3)     T_draft + T_target, each forward pass modelled as
 *                       c_context * N_context + c_batched * N_batched + c_fixed
 *                       (N_context: tokens whose KV is cached, summed over the batch;
 *                        N_batched: tokens scored in the pass)
 *   generated (Eq. 4)   per request (1 - a^(k+1)) / (1 - a), a = token acceptance rate,
 *                       bonus token included
 */
typedef struct {
    double c_context;   /* seconds per context token  (Eq. 3's first coefficient)  */
    double c_batched;   /* seconds per batched token  (Eq. 3's second coefficient) */
    double c_fixed;     /* seconds per pass           (Eq. 3's constant)           */
} spec_latency_model;

/* Eq. 4.  alpha in [0,1], k >= 0; alpha == 1 gives k + 1.  NaN on bad arguments. */
double spec_expected_generated_len(double alpha, int32_t k);

/* Eq. 3 evaluated. */
double spec_predict_latency(const spec_latency_model *model, double n_context, double n_batched);

/* Ordinary least squares fit of Eq. 3 to n >= 3 measured passes (seconds[i] at
 * n_context[i], n_batched[i]).  SPEC_EINVAL if the three columns are linearly
 * dependent (e.g. every pass has the same N_batched) or an argument is NULL. */
spec_status spec_fit_latency(const double *n_context, const double *n_batched, const double *seconds, int32_t n,
                             spec_latency_model *model);

/* Running estimate of the token acceptance rate (Section 4.1, "Accepted Length": a
 * weighted average over past steps).  Feed it the step's counters: accepted =
 * counters[1], attempted = counters[2] (accept tests actually evaluated; positions after
 * the first rejection carry no information).  rate = sum_j w^(age_j) accepted_j /
 * sum_j w^(age_j) attempted_j with decay w in (0,1]; steps with attempted == 0 leave it
 * unchanged.  Zero-initialise the struct; rate is `prior` until something was observed. */
typedef struct {
    double accepted_weighted;
    double attempted_weighted;
} spec_acceptance_tracker;
void spec_acceptance_update(spec_acceptance_tracker *tracker, int64_t accepted, int64_t attempted, double decay);
double spec_acceptance_rate(const spec_acceptance_tracker *tracker, double prior);

/* The search for the proposed length (Section 4.2, the listing "Finding k to maximize
 * goodput").  For k = 0 .. max_k: skip k if the batch would need more than free_kv_tokens
 * new KV slots (B * (k + 1)); generated(k) = sum_b Eq. 4(alpha_b, k);
 * time(k) = target(N_context, B * (k + 1)) + T_draft(k), where T_draft(k) =
 * k * draft(N_context, B) for a draft model (k sequential passes over the batch) or
 * draft_fixed_seconds for a proposer whose cost does not depend on k (k > 0 only; a
 * step with k = 0 runs no proposer).  Returns the k with the largest
 * generated(k) / time(k) (the smallest such k on ties), or -1 on bad arguments or if no
 * k fits.  k = 0 is ordinary decoding: the search can switch speculation off.
 * goodput_per_k (optional, max_k + 1 entries) receives every candidate's value in
 * tokens/s (NaN for a skipped k). */
typedef struct {
    int32_t B;
    int32_t max_k;                  /* <= SPEC_K_MAX */
    const int32_t *context_len;     /* [B] cached tokens per request */
    const double *alpha;            /* [B], or [1] if alpha_per_request == 0 */
    int32_t alpha_per_request;
    spec_latency_model target;
    int32_t draft_is_model;         /* 1: T_draft = k * draft(N_context, B); 0: draft_fixed_seconds */
    spec_latency_model draft;
    double draft_fixed_seconds;
    int64_t free_kv_tokens;         /* < 0: unlimited */
} spec_goodput_args;
int32_t spec_argmax_goodput(const spec_goodput_args *args, double *goodput_per_k);

/*
 * Measurement aid (not part of the step): per-kernel GPU time from HIP events.
 * Between spec_profile_begin and spec_profile_end every kernel the library
 * launches (up to max_launches of them) gets a pair of events: the step kernel
 * carries them itself (they receive the time stamps of the launch's own begin
 * and end), the other kernels are bracketed by two event records on the launch
 * stream.  spec_profile_end waits for those events and returns, per kernel id,
 * the summed duration in milliseconds and the number of launches (both arrays
 * have SPEC_NUM_KERNELS entries).  begin creates the events, so it must not be
 * called during stream capture; the pair is not thread safe.
 */
#define SPEC_NUM_KERNELS 5
#define SPEC_KERNEL_STEP 0          /* the whole step in one launch (attention + rejection sampling) */
#define SPEC_KERNEL_ATTN 1          /* attention-only launch of the matrix-instruction kernel */
#define SPEC_KERNEL_ATTN_GENERIC 2  /* generic attention over one KV chunk (fp32 / token-major path) */
#define SPEC_KERNEL_ATTN_COMBINE 3  /* merge of the generic kernel's chunk partials */
#define SPEC_KERNEL_REJECT 4        /* rejection-sampling-only launch */
spec_status spec_profile_begin(int32_t max_launches);
spec_status spec_profile_end(float *total_ms, int32_t *launches);

const char *spec_status_string(spec_status status);

/* Library version: major * 10000 + minor * 100 + patch. */
int32_t spec_verify_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_VERIFY_H */
