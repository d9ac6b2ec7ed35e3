// Shared declarations of the HIP library's translation units (host planning
// structs and kernel launchers).  Nothing here is used by the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spec_verify.h"

namespace specv {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr double kLog2eD = 1.4426950408889634074;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kEmptyMax = -1.0e30f;  // running maximum of a row that has seen no key yet

// ---------------------------------------------------------------- attention
// Split of the KV length.  A request of L tokens is cut into
// nch = ceil(L / chunk_tokens) chunks.  The generic kernel uses chunks of exactly
// chunk_tokens; the matrix-instruction kernel evens them out per request
// (chunk = ceil(L / nch) rounded up to 64 tokens).  Each (query row, query head,
// chunk) owns one partial result in the workspace:
//   acc  [T*Hq][max_chunks][d]  un-normalised sum_t 2^(s_t - m) V_t
//   ml   [T*Hq][max_chunks][2]  running maximum m (base-2 units) and sum l of 2^(s_t - m)
// tickets [B*Hkv] count the chunks of a (request, KV head) that have finished;
// the block that finishes last merges the partials (matrix-instruction kernel).
constexpr int kMaxFusedChunks = 64;   // beyond this many chunks per request a separate launch merges the partials

struct AttnPlan {
    int32_t chunk_tokens;
    int32_t max_chunks;
    int32_t max_q_len;
    int32_t use_mfma;      // 1: bf16 matrix-instruction kernel, 0: generic kernel
    int32_t row_tiles;     // 16-row tiles of query rows per wave group (mfma kernel, 1..3)
    int32_t row_groups;    // wave groups per attention block (1, 2 or 4): row_groups * row_tiles tiles cover max_q_len * (Hq/Hkv) rows
    int32_t capacity_tokens;  // longest kv_len the plan allows for (chunk_tokens * max_chunks, capped by the bucket)
    int32_t fused_combine; // mfma kernel merges the chunk partials itself (few chunks) or leaves it to the combine kernel
    int32_t short_attn;    // the attention half streams for less time than the rejection stages' chain takes
    size_t acc_bytes;
    size_t ml_bytes;
    size_t ticket_bytes;
    size_t total_bytes;
};

struct AttnParams {
    // (scalars first and in pairs of 4-byte fields, so that the struct has no padding holes:
    // a hole next to a pointer made the compiler keep a private-memory copy of that slice)
    int32_t B, Hq, Hkv, d, num_blocks, max_blocks_per_req, T;
    int32_t kv_layout;
    int32_t chunk_tokens, max_chunks;
    float scale_log2;  // softmax scale times log2(e): scores are kept in base-2 units
    uint32_t generation;  // tags this call's ticket values, never 0
    int32_t fused_combine;        // matrix kernel: the last chunk's block merges the partials (needs max_chunks <= kMaxFusedChunks)
    int32_t attn_first_limit;     // attention blocks go first in the grid when there are at most this many
    float reject_span;            // fraction of the attention items among which the rejection items are spread in the grid
    int32_t split_p;              // feed the softmax weights to the PV product as bf16 high + low parts
    int32_t reserved;
    int32_t reject_even_xcds;     // fused step: rejection blocks only at even positions of the grid's rows of 8 (see GridSplit)
    int32_t reject_even_limit;    // ... when there are at most this many attention blocks (the number of compute units)
    int32_t capacity_tokens;      // a request whose device-side kv_len exceeds this is skipped and counted in *errors
    int32_t row_groups;           // see AttnPlan
    int32_t reject_first_limit;   // fused step: up to this many rejection items go first in the grid (0: never)
    const void *q, *k_cache, *v_cache;
    const int32_t *block_table, *kv_len, *cu_q_len;
    float *out;
    float *ws_acc;
    float *ws_ml;
    unsigned long long *tickets;  // [B * Hkv]
    unsigned long long *errors;   // findings of the device-side input checks are added here (may be null)
};
static_assert(sizeof(AttnParams) == 22 * 4 + 11 * 8, "AttnParams has padding");

// What the kernels check of a request before they use its lengths as loop bounds and indices.
__host__ __device__ inline bool request_lengths_ok(int kv_len, int q_len, int capacity_tokens, int max_blocks_per_req)
{
    return q_len >= 1 && q_len <= SPEC_K_MAX + 1 && kv_len >= q_len && kv_len <= capacity_tokens &&
           (kv_len + SPEC_BLOCK_SIZE - 1) / SPEC_BLOCK_SIZE <= max_blocks_per_req;
}

// ---------------------------------------------------------------- rejection
// Records handed between the rejection stages are arrays of 8-byte words, each a
// 32-bit payload with the call's generation tag in the high half:
//   statistics of one (row, vocabulary segment): 3 words: low and high half of
//     sum_v 2^(x_v*log2(e) - off2) as fp64, and off2 (integer-valued base-2 offset) as fp32
//     (greedy mode: the segment's largest logit as fp32 and its lowest id, third word unused)
//   race partial of one (request, segment): 2 words: best score (fp32), its id
//   race info of one request: m | k << 8 | near ties << 16
constexpr int kStatWords = 3;

struct RejectPlan {
    int32_t stat_segments, stat_seg_len;   // vocabulary segments per row in the statistics pass
    int32_t race_segments, race_seg_len;   // vocabulary segments per request in the race
    size_t stats_off, stats_bytes;         // [rows][stat_segments][3] words
    size_t partial_off, partial_bytes;     // race partials [B][race_segments][2], then race info [B]
    size_t total_bytes;
    int32_t early_stop, uniform_k;         // see RejectParams
};

struct RejectParams {
    // (4-byte scalars first, an even number of them: no padding holes, see AttnParams)
    int32_t B, V, T;
    int32_t mode;   // spec_accept_mode
    uint32_t seed_lo, seed_hi, step_lo, step_hi24;
    int32_t stat_segments, stat_seg_len;
    int32_t race_segments, race_seg_len;
    int32_t spin_limit;                  // polls a consumer block spends waiting for its producers
    uint32_t generation;
    int32_t early_stop;                  // statistics in position order, rows after a request's first rejection are not read (see stats_role)
    int32_t uniform_k;                   // with early_stop: every request's draft length
    int32_t short_naps;                  // a small launch: the bounded waits poll at short intervals at first
    int32_t reserved;
    const float *target_logits, *draft_logits;
    const int32_t *draft_tokens, *cu_q_len;
    int32_t *accepted_len, *next_token, *out_tokens;
    unsigned long long *counters;
    double *debug_u_ratio;
    const int32_t *kv_len;               // cache bookkeeping after acceptance (optional)
    int32_t *new_kv_len, *draft_next_len;
    unsigned long long *stats;           // [rows][stat_segments][3]
    unsigned long long *race_partial;    // [B][race_segments][2]
    unsigned long long *race_info;       // [B]
    const unsigned long long *step_device;   // if not null: the Philox step counter, read when the kernel runs
};
static_assert(sizeof(RejectParams) == 18 * 4 + 16 * 8, "RejectParams has padding");

// Order in which the attention items take the requests (longest first), passed as a
// kernel argument.  n == 0: the given order.
constexpr int kMaxOrdered = 1024;
struct UnitOrder {
    int32_t n;
    alignas(4) uint16_t request[kMaxOrdered];
};

// Events that receive the begin and end time stamps of a kernel launch itself (both null:
// none).  Unlike event records placed before and after the launch on the stream they do
// not include the time the stream spends on the records.
struct LaunchEvents {
    hipEvent_t start, stop;
};

// One launch for the whole step (either half may be absent).  `attn` needs the
// matrix-instruction path (bf16, either page layout, d = 128 or 64; row_tiles tiles per wave
// group, ap.row_groups wave groups per block).  `order` may be null.
int step_attn_items(const AttnParams &ap);   // attention blocks of the launch
// attention items per chunk index: one per (request, KV head), padded to whole rows of 8 blocks (one per XCD) when requests are split
__host__ __device__ inline int attn_row_items(const AttnParams &ap)
{
    const int units = ap.B * ap.Hkv;
    return ap.max_chunks > 1 ? (units + 7) / 8 * 8 : units;
}
hipError_t launch_step_fused(const AttnParams *attn, int row_tiles, const RejectParams *reject, const UnitOrder *order,
                             LaunchEvents events, hipStream_t stream);

// Generic attention path: partial kernel + combine kernel.
hipError_t launch_attn_generic(const AttnParams &p, int dtype, hipStream_t stream);
hipError_t launch_attn_combine(const AttnParams &p, hipStream_t stream);
struct KvAppendParams {
    int32_t B, Hkv, d, max_blocks_per_req, T, kv_layout, elem_bytes, num_blocks;
    const void *new_k, *new_v;
    void *k_cache, *v_cache;
    const int32_t *block_table, *kv_len, *cu_q_len;
    unsigned long long *errors;   // rows skipped by the device-side checks are counted here (may be null)
};
hipError_t launch_kv_append(const KvAppendParams &p, hipStream_t stream);
hipError_t launch_kv_repack(const void *src_k, const void *src_v, void *dst_k, void *dst_v, int32_t num_blocks,
                            int32_t Hkv, int32_t d, hipStream_t stream);

}  // namespace specv
