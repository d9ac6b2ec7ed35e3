// C ABI of the speculative-verification library: host-side validation, launch
// planning and the exported entry points declared in spec_verify.h.
//
// A call costs the host: scalar checks of the argument structs, one hash over the host
// copies of the lengths, a look-up of the launch plan under that hash (the per-request
// checks, the split of the KV length, the order table and the grid layout are computed when a
// shape is seen for the first time), and the launch.  The tuning switches are read from the
// environment once.
#include "common.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <vector>

// ---------------------------------------------------------------------------
// Scratch memory for callers that cannot allocate (spec_verify_step_static): one file-scope
// device array per GPU, held until the process ends.  In host code the array's name is only
// a stand-in for the symbol; its device address is resolved once per device, with that device
// current, and kept.  Each GPU has its own copy of the array at its own address.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[SPEC_STATIC_SCRATCH_BYTES];

namespace specv {

namespace {

constexpr size_t kAlign = 256;

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

void *static_scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        // (two threads may both resolve it: they get the same address)
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return nullptr;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    return ptr;
}

// ---------------------------------------------------------------------------
// Optional per-kernel timing with HIP events (spec_profile_begin / spec_profile_end).
// Off by default; when on, every kernel launch is bracketed by two event records on
// the launch stream.  Not thread safe; meant for the benchmark.
// ---------------------------------------------------------------------------
struct KernelProfiler {
    bool on = false;
    std::vector<hipEvent_t> events;   // pairs: start, stop
    std::vector<int> kernel_of_pair;
    size_t capacity_pairs = 0;
};
KernelProfiler g_prof;

template <typename F>
hipError_t timed(int kernel_id, hipStream_t stream, F launch)
{
    const bool rec = g_prof.on && g_prof.kernel_of_pair.size() < g_prof.capacity_pairs;
    size_t pair = 0;
    if (rec) {
        pair = g_prof.kernel_of_pair.size();
        g_prof.kernel_of_pair.push_back(kernel_id);
        (void)hipEventRecord(g_prof.events[2 * pair], stream);
    }
    const hipError_t err = launch();
    if (rec) (void)hipEventRecord(g_prof.events[2 * pair + 1], stream);
    return err;
}
// The same for a launch that can carry its events itself.
template <typename F>
hipError_t timed_launch(int kernel_id, F launch)
{
    LaunchEvents ev = {nullptr, nullptr};
    if (g_prof.on && g_prof.kernel_of_pair.size() < g_prof.capacity_pairs) {
        const size_t pair = g_prof.kernel_of_pair.size();
        g_prof.kernel_of_pair.push_back(kernel_id);
        ev.start = g_prof.events[2 * pair];
        ev.stop = g_prof.events[2 * pair + 1];
    }
    return launch(ev);
}
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// ---------------------------------------------------------------------------
// Tuning switches (environment variables, for sweeps; none is needed in normal use).
// Read once; spec_verify_reload_env re-reads them.
// ---------------------------------------------------------------------------
struct Tuning {
    int force_generic = 0;        // SPEC_VERIFY_FORCE_GENERIC=1: every shape through the generic attention kernels
    long target_blocks = 0;       // SPEC_VERIFY_TARGET_BLOCKS: attention blocks to aim for when splitting requests (0: automatic)
    long chunk = 0;               // SPEC_VERIFY_CHUNK: tokens per chunk, multiple of 16 (0: automatic)
    int race_blocks = 512;        // SPEC_VERIFY_RACE_BLOCKS: race blocks to aim for
    int early_stop = -1;          // SPEC_VERIFY_EARLY_STOP=0/1: statistics in position order (-1: automatic)
    float reject_span = 0.5f;     // SPEC_VERIFY_REJECT_SPAN: fraction of the attention items among which the rejection items are spread
    long attn_first_limit = -1;   // SPEC_VERIFY_ATTN_FIRST_LIMIT: attention blocks up to which they all precede the rejection blocks (-1: automatic)
    int reject_first_limit = 1024; // SPEC_VERIFY_REJECT_FIRST_LIMIT: rejection blocks up to which they precede the blocks of a short attention half
    int split_p = 1;              // SPEC_VERIFY_SPLIT_P=0: softmax weights as one bf16 instead of high + low parts
    int reject_even = 1;          // SPEC_VERIFY_REJECT_EVEN=0: rejection blocks on all XCDs
    int spin_limit = 1 << 20;     // SPEC_VERIFY_SPIN_LIMIT: polls of a bounded wait (about a second at the default)
    uint32_t epoch = 1;           // changes with every reload: part of the plan cache's key
};
Tuning g_tuning;
std::once_flag g_tuning_once;
std::atomic<uint32_t> g_tuning_epoch{1};

void read_tuning()
{
    Tuning t;
    if (const char *e = getenv("SPEC_VERIFY_FORCE_GENERIC")) t.force_generic = e[0] == '1';
    if (const char *e = getenv("SPEC_VERIFY_TARGET_BLOCKS")) {
        const long v = strtol(e, nullptr, 10);
        if (v >= 1 && v <= (1 << 20)) t.target_blocks = v;
    }
    if (const char *e = getenv("SPEC_VERIFY_CHUNK")) {
        const long v = strtol(e, nullptr, 10);
        if (v >= 16 && v <= 4096 && v % SPEC_BLOCK_SIZE == 0) t.chunk = v;
    }
    if (const char *e = getenv("SPEC_VERIFY_RACE_BLOCKS")) {
        const int v = atoi(e);
        if (v >= 1 && v <= 65536) t.race_blocks = v;
    }
    if (const char *e = getenv("SPEC_VERIFY_EARLY_STOP")) t.early_stop = e[0] != '0';
    if (const char *e = getenv("SPEC_VERIFY_REJECT_SPAN")) {
        const double v = strtod(e, nullptr);
        if (v > 0.0 && v <= 1.0) t.reject_span = (float)v;
    }
    if (const char *e = getenv("SPEC_VERIFY_ATTN_FIRST_LIMIT")) {
        const long v = strtol(e, nullptr, 10);
        if (v >= 0 && v <= (1 << 20)) t.attn_first_limit = v;
    }
    if (const char *e = getenv("SPEC_VERIFY_REJECT_FIRST_LIMIT")) {
        const long v = strtol(e, nullptr, 10);
        if (v >= 0 && v <= (1 << 20)) t.reject_first_limit = (int)v;
    }
    if (const char *e = getenv("SPEC_VERIFY_SPLIT_P")) t.split_p = e[0] != '0';
    if (const char *e = getenv("SPEC_VERIFY_REJECT_EVEN")) t.reject_even = e[0] != '0';
    if (const char *e = getenv("SPEC_VERIFY_SPIN_LIMIT")) {
        const long v = strtol(e, nullptr, 10);
        if (v >= 1 && v <= (1 << 30)) t.spin_limit = (int)v;
    }
    t.epoch = g_tuning_epoch.fetch_add(1) + 1;
    g_tuning = t;
}

const Tuning &tuning()
{
    std::call_once(g_tuning_once, read_tuning);
    return g_tuning;
}

// Number of compute units of the current device (cached per process; one GPU).
int compute_units()
{
    static int cached = 0;
    if (cached == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;   // MI355X
        cached = n;
    }
    return cached;
}

// ---------------------------------------------------------------------------
// Validation.  The scalar part runs on every call; the per-request part (one pass over the
// host copies of the lengths) is what a cached plan vouches for.
// ---------------------------------------------------------------------------
spec_status validate_attn_scalars(const spec_attn_args *a)
{
    if (a == nullptr) return SPEC_EINVAL;
    if (a->B < 1 || a->Hq < 1 || a->Hkv < 1 || a->num_blocks < 1 || a->max_blocks_per_req < 1 || a->T < a->B)
        return SPEC_EINVAL;
    if (a->q == nullptr || a->k_cache == nullptr || a->v_cache == nullptr || a->block_table == nullptr ||
        a->kv_len == nullptr || a->cu_q_len == nullptr || a->out == nullptr || a->host_cu_q_len == nullptr)
        return SPEC_EINVAL;
    // (rows and pages move as vectors of up to 32 bytes)
    if (((reinterpret_cast<uintptr_t>(a->q) | reinterpret_cast<uintptr_t>(a->k_cache) | reinterpret_cast<uintptr_t>(a->v_cache) |
          reinterpret_cast<uintptr_t>(a->out)) & 31) != 0)
        return SPEC_EINVAL;
    if (a->max_kv_len < 0 || (a->max_kv_len == 0 && a->host_kv_len == nullptr)) return SPEC_EINVAL;
    if (a->Hq % a->Hkv != 0) return SPEC_EINVAL;
    if (!(a->softmax_scale >= 0.0f) || isinf(a->softmax_scale)) return SPEC_EINVAL;
    if (a->qkv_dtype != SPEC_F32 && a->qkv_dtype != SPEC_BF16) return SPEC_EINVAL;
    if (a->kv_layout != SPEC_KV_TOKEN_MAJOR && a->kv_layout != SPEC_KV_MFMA) return SPEC_EINVAL;
    if (a->validate != 0 && a->validate != 1) return SPEC_EINVAL;
    if (a->host_cu_q_len[0] != 0 || a->host_cu_q_len[a->B] != a->T) return SPEC_EINVAL;
    if (a->max_kv_len > 0 && (a->max_kv_len + SPEC_BLOCK_SIZE - 1) / SPEC_BLOCK_SIZE > a->max_blocks_per_req)
        return SPEC_EINVAL;
    return SPEC_OK;
}

spec_status validate_attn_requests(const spec_attn_args *a)
{
    for (int b = 0; b < a->B; ++b) {
        const int q_len = a->host_cu_q_len[b + 1] - a->host_cu_q_len[b];
        if (q_len < 1 || q_len > SPEC_K_MAX + 1) return SPEC_EINVAL;
        if (a->host_kv_len == nullptr) continue;
        const int len = a->host_kv_len[b];
        if (len < q_len) return SPEC_EINVAL;
        if ((len + SPEC_BLOCK_SIZE - 1) / SPEC_BLOCK_SIZE > a->max_blocks_per_req) return SPEC_EINVAL;
        if (a->max_kv_len > 0 && len > a->max_kv_len) return SPEC_EINVAL;
    }
    return SPEC_OK;
}

spec_status validate_attn_unsupported(const spec_attn_args *a)
{
    if (a->block_size != SPEC_BLOCK_SIZE) return SPEC_EUNSUPPORTED;
    if (a->d != 64 && a->d != 128) return SPEC_EUNSUPPORTED;
    if (a->Hq / a->Hkv > 16) return SPEC_EUNSUPPORTED;
    if (a->kv_layout == SPEC_KV_MFMA && a->qkv_dtype != SPEC_BF16) return SPEC_EUNSUPPORTED;
    if (a->T > 65535 || a->Hq > 65535) return SPEC_EUNSUPPORTED;
    return SPEC_OK;
}

// validate == 1: the host copy of the block table, every entry of a page in use
spec_status validate_attn_table(const spec_attn_args *a)
{
    if (a->validate != 1 || a->host_block_table == nullptr || a->host_kv_len == nullptr) return SPEC_OK;
    for (int b = 0; b < a->B; ++b) {
        const int pages = (a->host_kv_len[b] + SPEC_BLOCK_SIZE - 1) / SPEC_BLOCK_SIZE;
        const int32_t *row = a->host_block_table + (size_t)b * a->max_blocks_per_req;
        for (int i = 0; i < pages; ++i)
            if (row[i] < 0 || row[i] >= a->num_blocks) return SPEC_EINVAL;
    }
    return SPEC_OK;
}

spec_status validate_attn(const spec_attn_args *a)
{
    spec_status st = validate_attn_scalars(a);
    if (st != SPEC_OK) return st;
    st = validate_attn_requests(a);
    if (st != SPEC_OK) return st;
    st = validate_attn_unsupported(a);
    if (st != SPEC_OK) return st;
    return validate_attn_table(a);
}

spec_status validate_reject_scalars(const spec_reject_args *r)
{
    if (r == nullptr) return SPEC_EINVAL;
    if (r->B < 1 || r->V < 1 || r->T < r->B) return SPEC_EINVAL;
    if (r->target_logits == nullptr || r->cu_q_len == nullptr || r->host_cu_q_len == nullptr ||
        r->accepted_len == nullptr || r->next_token == nullptr || r->counters == nullptr)
        return SPEC_EINVAL;
    if (r->accept_mode != SPEC_ACCEPT_SAMPLE && r->accept_mode != SPEC_ACCEPT_GREEDY &&
        r->accept_mode != SPEC_ACCEPT_POINT_DRAFT)
        return SPEC_EINVAL;
    if (r->validate != 0 && r->validate != 1) return SPEC_EINVAL;
    if (r->T > r->B && r->draft_tokens == nullptr) return SPEC_EINVAL;
    if (r->T > r->B && r->accept_mode == SPEC_ACCEPT_SAMPLE && r->draft_logits == nullptr) return SPEC_EINVAL;
    if (r->host_cu_q_len[0] != 0 || r->host_cu_q_len[r->B] != r->T) return SPEC_EINVAL;
    if ((r->new_kv_len != nullptr || r->draft_next_len != nullptr) && r->kv_len == nullptr) return SPEC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(r->target_logits) & 15) != 0 ||
        (r->accept_mode == SPEC_ACCEPT_SAMPLE && (reinterpret_cast<uintptr_t>(r->draft_logits) & 15) != 0) ||
        (reinterpret_cast<uintptr_t>(r->philox_step_device) & 7) != 0)
        return SPEC_EINVAL;
    return SPEC_OK;
}

spec_status validate_reject_requests(const spec_reject_args *r)
{
    for (int b = 0; b < r->B; ++b) {
        const int q_len = r->host_cu_q_len[b + 1] - r->host_cu_q_len[b];
        if (q_len < 1 || q_len > SPEC_K_MAX + 1) return SPEC_EINVAL;
    }
    return SPEC_OK;
}

spec_status validate_reject_unsupported(const spec_reject_args *r)
{
    if (r->V % 4 != 0) return SPEC_EUNSUPPORTED;  // rows are read as 16-byte vectors
    if (r->B > 65535 || 2 * (int64_t)r->T - r->B > 65535) return SPEC_EUNSUPPORTED;
    return SPEC_OK;
}

// validate == 1: the host copy of the draft tokens
spec_status validate_reject_tokens(const spec_reject_args *r)
{
    if (r->validate != 1 || r->host_draft_tokens == nullptr) return SPEC_OK;
    for (int i = 0; i < r->T - r->B; ++i)
        if (r->host_draft_tokens[i] < 0 || r->host_draft_tokens[i] >= r->V) return SPEC_EINVAL;
    return SPEC_OK;
}

spec_status validate_reject(const spec_reject_args *r)
{
    spec_status st = validate_reject_scalars(r);
    if (st != SPEC_OK) return st;
    st = validate_reject_requests(r);
    if (st != SPEC_OK) return st;
    st = validate_reject_unsupported(r);
    if (st != SPEC_OK) return st;
    return validate_reject_tokens(r);
}

// ---------------------------------------------------------------------------
// Planning.
// ---------------------------------------------------------------------------
// Split of the KV length.  The matrix-instruction kernel runs one block per (request, KV head,
// chunk); the chunk is sized so that the launch has about one block per compute unit
// (two with three row tiles), in multiples of the 16 tokens of a page.  The longest length the
// plan allows for is the caller's bucket (max_kv_len) or, without one, the longest host length.
AttnPlan plan_attn(const spec_attn_args *a, const Tuning &tu)
{
    AttnPlan pl;
    memset(&pl, 0, sizeof pl);
    int max_len = a->max_kv_len, max_q = 0;
    for (int b = 0; b < a->B; ++b) {
        if (a->max_kv_len == 0 && a->host_kv_len[b] > max_len) max_len = a->host_kv_len[b];
        const int q_len = a->host_cu_q_len[b + 1] - a->host_cu_q_len[b];
        if (q_len > max_q) max_q = q_len;
    }
    pl.max_q_len = max_q;
    const int group = a->Hq / a->Hkv;
    const int tiles = (max_q * group + 15) / 16;
    // bf16 runs on the matrix-instruction kernel, in either page layout (token-major pages have
    // their V transposed through LDS)
    pl.use_mfma = (a->qkv_dtype == SPEC_BF16 && !tu.force_generic) ? 1 : 0;
    pl.row_groups = 1;
    pl.row_tiles = tiles;
    if (pl.use_mfma) {
        // A wavefront holds up to three 16-row tiles of query rows in registers.  With up to 48 rows
        // per KV head the block's four wavefronts share the pages between them; with more (long
        // drafts on wide query groups) they form 2 or 4 groups that each own a share of the rows and
        // walk all pages, reading them side by side.
        pl.row_groups = tiles <= 3 ? 1 : (tiles <= 6 ? 2 : 4);
        pl.row_tiles = (tiles + pl.row_groups - 1) / pl.row_groups;
        if (pl.row_groups > 1 && pl.row_tiles < 2) pl.row_tiles = 2;
        // Splitting costs (partials, a merge, more block start-ups), so the longest request is split
        // only as far as needed to give every compute unit a block.  With three row tiles the
        // wavefronts spend a larger share of their time on arithmetic and need a second block beside
        // them to keep loads in flight: then the target is two blocks per compute unit, less an
        // eighth of the slots, which the rejection items flow through while the attention blocks
        // (all resident from the start) stream (with a sixteenth the rejection items of the ragged
        // long-context workload ended after the attention: 90.0 against 88.2 us).
        const long cus = compute_units();
        long target_blocks = pl.row_tiles >= 3 ? 2 * cus - cus / 4 : cus;
        if (tu.target_blocks > 0) target_blocks = tu.target_blocks;
        const int64_t units = (int64_t)a->B * a->Hkv;
        int64_t nsplit = (target_blocks + units - 1) / units;
        if (nsplit < 1) nsplit = 1;
        // Few, short requests are bound by latencies, not by bytes: every further chunk adds block
        // start-ups and partials to merge (eight chunks per pass of the merge), and a chunk of
        // less than a few pages per wavefront does not repay its fixed cost.  So such requests get
        // at most 8 chunks (beyond that only chunks of 1024 tokens or more), of 256 tokens or more.
        // One request with 64/8 heads and 2749 tokens: 29 chunks 24.9 us, 8 chunks 15.8 us; four
        // of 204 tokens: 4 chunks 11.1 us, unsplit 7.9 us; 32/32 heads, 2048 tokens: 8 chunks
        // 13.6 us, 16 chunks 19.3 us, 2 chunks 17.2 us.
        int64_t min_chunk = 64;
        if (tu.target_blocks == 0) {
            const int64_t most = std::max<int64_t>(8, (max_len + 1023) / 1024);
            if (nsplit > most) nsplit = most;
            min_chunk = 256;
        }
        int64_t chunk = (max_len + nsplit - 1) / nsplit;
        chunk = (chunk + SPEC_BLOCK_SIZE - 1) / SPEC_BLOCK_SIZE * SPEC_BLOCK_SIZE;
        if (chunk < min_chunk) chunk = min_chunk;
        // a wavefront holds its pages' block-table entries one per lane, and takes every
        // (4 / row_groups)-th page of the chunk
        const int64_t chunk_cap = 4096 / pl.row_groups;
        if (chunk > chunk_cap) chunk = chunk_cap;
        if (tu.chunk > 0 && tu.chunk <= chunk_cap) chunk = tu.chunk;
        pl.chunk_tokens = (int32_t)chunk;
    } else {
        pl.chunk_tokens = 256;  // one key per thread of the generic kernel
    }
    pl.max_chunks = (max_len + pl.chunk_tokens - 1) / pl.chunk_tokens;
    pl.capacity_tokens = pl.chunk_tokens * pl.max_chunks;
    pl.fused_combine = (pl.use_mfma && pl.max_chunks <= kMaxFusedChunks) ? 1 : 0;
    // (a request that is not split writes its output directly: the matrix kernel needs no partial
    // slots when no request can have a second chunk)
    const size_t slots = (pl.use_mfma && pl.max_chunks == 1) ? 0 : (size_t)a->T * a->Hq * pl.max_chunks;
    pl.acc_bytes = align_up(slots * a->d * sizeof(float));
    pl.ml_bytes = align_up(slots * 2 * sizeof(float));
    pl.ticket_bytes = align_up((size_t)a->B * a->Hkv * sizeof(unsigned long long));
    pl.total_bytes = pl.acc_bytes + pl.ml_bytes + pl.ticket_bytes;
    return pl;
}

// Rough duration of the attention half in microseconds (the KV bytes at 5.5 TB/s: what it takes
// when it streams well); from the host lengths, or from the bucket bound where there are none.
double attn_estimate_us(const spec_attn_args *a)
{
    double tokens = 0.0;
    for (int b = 0; b < a->B; ++b) tokens += a->host_kv_len != nullptr ? (double)a->host_kv_len[b] : 0.75 * a->max_kv_len;
    return tokens * 2.0 * a->Hkv * a->d * (a->qkv_dtype == SPEC_BF16 ? 2 : 4) / 5.5e6;
}

// attn_us: rough duration of the attention half that runs in the same launch (microseconds), or
// negative if the rejection half runs alone.
RejectPlan plan_reject(const spec_reject_args *r, size_t base, const Tuning &tu, double attn_us = -1.0)
{
    RejectPlan pl;
    memset(&pl, 0, sizeof pl);
    // logit rows that get a statistics pass: the draft rows only when there is a draft distribution
    const int rows = r->accept_mode == SPEC_ACCEPT_SAMPLE ? 2 * r->T - r->B : r->T;
    // statistics: about 256 blocks in all, segments of >= 8192 logits, at most 32 per row
    int segs = (256 + rows - 1) / rows;
    const int max_by_len = (r->V + 8191) / 8192;
    if (segs > max_by_len) segs = max_by_len;
    if (segs > 32) segs = 32;
    if (segs < 1) segs = 1;
    int seg_len = (r->V + segs - 1) / segs;
    seg_len = (seg_len + 3) / 4 * 4;
    pl.stat_seg_len = seg_len;
    pl.stat_segments = (r->V + seg_len - 1) / seg_len;
    // race: about 512 blocks in all, segments of >= 2048 vocabulary ids, at most 64 per request
    int rsegs = (tu.race_blocks + r->B - 1) / r->B;
    const int rmax_by_len = (r->V + 2047) / 2048;
    if (rsegs > rmax_by_len) rsegs = rmax_by_len;
    if (rsegs > 64) rsegs = 64;
    if (rsegs < 1) rsegs = 1;
    int rlen = (r->V + rsegs - 1) / rsegs;
    rlen = (rlen + 3) / 4 * 4;
    pl.race_seg_len = rlen;
    pl.race_segments = (r->V + rlen - 1) / rlen;

    // Early stop: with one draft length for all requests the statistics items can be taken in
    // position order and the rows after a request's first rejection left unread.  That turns the
    // pass into a chain of k+1 dependent stages (about 12 us each, then the race), which must stay
    // hidden: under a launch that streams (KV and logit bytes at 5.5 TB/s) for clearly longer than
    // the chain takes, or, when the rejection half runs alone, behind several rounds of blocks per
    // position.  Measured (step with / without): B=256 k=2 (64/8 heads) -4%, the same at k=7 -15%,
    // B=64 k=8 (32/32 heads, L=1024) -8%, B=64 k=4 -3%, B=32 k=1..3 -2%, B=32 k=4 +2%, B=32 k=8 +16%,
    // B=16 k=2 (L=2048) +2%, B=8 k=4 +32%.
    pl.early_stop = 0;
    pl.uniform_k = 0;
    if (r->T > r->B && r->T % r->B == 0) {
        const int q = r->T / r->B;
        bool uniform = true;
        for (int b = 0; b < r->B && uniform; ++b) uniform = r->host_cu_q_len[b + 1] - r->host_cu_q_len[b] == q;
        bool wanted;
        if (attn_us >= 0.0) {
            const double logits_us = (double)rows * r->V * 4.0 / 5.5e6;
            wanted = r->B >= 32 && 12.0 * q + 30.0 <= 0.85 * (attn_us + logits_us);
        } else {
            const int64_t per_position = (int64_t)(r->accept_mode == SPEC_ACCEPT_SAMPLE ? 2 : 1) * r->B * pl.stat_segments;
            wanted = (int64_t)rows * pl.stat_segments >= 3ll * compute_units() && per_position >= compute_units();
        }
        if (tu.early_stop >= 0) wanted = tu.early_stop != 0;
        if (uniform && wanted) { pl.early_stop = 1; pl.uniform_k = q - 1; }
    }
    pl.stats_off = base;
    pl.stats_bytes = align_up((size_t)rows * pl.stat_segments * kStatWords * sizeof(unsigned long long));
    pl.partial_off = pl.stats_off + pl.stats_bytes;
    pl.partial_bytes = align_up(((size_t)r->B * pl.race_segments * 2 + r->B) * sizeof(unsigned long long));
    pl.total_bytes = pl.stats_bytes + pl.partial_bytes;
    return pl;
}

// Requests by falling KV length (stable; from the host copy of kv_len).  The grid takes the
// attention items in this order: blocks that run at the same time then take about
// equally long, which the in-order hardware dispatcher needs to keep its block slots
// filled, and the short items even out the end of the launch.  Any order gives the same
// results, so under a length bucket the table made from the lengths at planning time stays
// valid (lengths that grow by a few tokens per step keep their ranks, more or less).  No table
// (given order) when all lengths are equal, unknown, or there are too many requests.
void make_order(const spec_attn_args *a, UnitOrder &order)
{
    order.n = 0;
    if (a->B > kMaxOrdered || a->host_kv_len == nullptr) return;
    bool equal = true;
    for (int b = 1; b < a->B; ++b)
        if (a->host_kv_len[b] != a->host_kv_len[0]) equal = false;
    if (equal) return;
    std::vector<int> idx(a->B);
    for (int b = 0; b < a->B; ++b) idx[b] = b;
    std::stable_sort(idx.begin(), idx.end(), [&](int x, int y) { return a->host_kv_len[x] > a->host_kv_len[y]; });
    for (int b = 0; b < a->B; ++b) order.request[b] = (uint16_t)idx[b];
    order.n = a->B;
}

// ---------------------------------------------------------------------------
// Plan cache: what one shape needs beyond the scalar checks, keyed by a hash of everything the
// plan depends on.  Per thread, sixteen entries (one per draft length and then some), replaced in turn.
// ---------------------------------------------------------------------------
struct StepPlan {
    uint64_t key = 0;
    bool used = false;
    spec_status status = SPEC_OK;   // of the per-request validation
    bool has_attn = false, has_reject = false;
    AttnPlan apl;
    RejectPlan rpl;
    UnitOrder order;
    // (for telling a hash collision from a hit)
    int32_t B = 0, T = 0, V = 0;
};

inline uint64_t mix(uint64_t h, uint64_t x)
{
    h ^= x;
    h *= 0x9E3779B97F4A7C15ull;
    return h ^ (h >> 29);
}

uint64_t hash_i32(uint64_t h, const int32_t *v, int n)
{
    int i = 0;
    for (; i + 1 < n; i += 2) h = mix(h, (uint64_t)(uint32_t)v[i] | ((uint64_t)(uint32_t)v[i + 1] << 32));
    if (i < n) h = mix(h, (uint64_t)(uint32_t)v[i]);
    return h;
}

uint64_t plan_key(const spec_attn_args *a, const spec_reject_args *r, const Tuning &tu)
{
    uint64_t h = mix(0x5EC0DEull, tu.epoch);
    if (a != nullptr) {
        h = mix(h, (uint64_t)(uint32_t)a->B | ((uint64_t)(uint32_t)a->Hq << 32));
        h = mix(h, (uint64_t)(uint32_t)a->Hkv | ((uint64_t)(uint32_t)a->d << 32));
        h = mix(h, (uint64_t)(uint32_t)a->T | ((uint64_t)(uint32_t)a->max_blocks_per_req << 32));
        h = mix(h, (uint64_t)(uint32_t)a->qkv_dtype | ((uint64_t)(uint32_t)a->kv_layout << 8) |
                       ((uint64_t)(uint32_t)a->block_size << 16) | ((uint64_t)(uint32_t)a->max_kv_len << 32));
        h = hash_i32(h, a->host_cu_q_len, a->B + 1);
        if (a->host_kv_len != nullptr) h = hash_i32(mix(h, 1), a->host_kv_len, a->B);
    }
    if (r != nullptr) {
        h = mix(h, 0xACCE97ull);
        h = mix(h, (uint64_t)(uint32_t)r->B | ((uint64_t)(uint32_t)r->V << 32));
        h = mix(h, (uint64_t)(uint32_t)r->T | ((uint64_t)(uint32_t)r->accept_mode << 32));
        if (a == nullptr || a->host_cu_q_len != r->host_cu_q_len) h = hash_i32(h, r->host_cu_q_len, r->B + 1);
    }
    return h | 1ull;
}

constexpr int kPlanCacheEntries = 16;
struct PlanCache {
    StepPlan entry[kPlanCacheEntries];
    int next = 0;
};

// The plan of (attn, reject); either may be null.  Scalar validation has passed.
const StepPlan &plan_for(const spec_attn_args *a, const spec_reject_args *r)
{
    thread_local PlanCache cache;
    const Tuning &tu = tuning();
    const uint64_t key = plan_key(a, r, tu);
    for (StepPlan &e : cache.entry)
        if (e.used && e.key == key && e.has_attn == (a != nullptr) && e.has_reject == (r != nullptr) &&
            e.B == (a != nullptr ? a->B : r->B) && e.T == (a != nullptr ? a->T : r->T) && e.V == (r != nullptr ? r->V : 0))
            return e;
    StepPlan &e = cache.entry[cache.next];
    cache.next = (cache.next + 1) % kPlanCacheEntries;
    e.key = key;
    e.used = true;
    e.has_attn = a != nullptr;
    e.has_reject = r != nullptr;
    e.B = a != nullptr ? a->B : r->B;
    e.T = a != nullptr ? a->T : r->T;
    e.V = r != nullptr ? r->V : 0;
    e.order.n = 0;
    e.status = SPEC_OK;
    if (a != nullptr) {
        e.status = validate_attn_requests(a);
        if (e.status == SPEC_OK) e.status = validate_attn_unsupported(a);
    }
    if (e.status == SPEC_OK && r != nullptr) {
        e.status = validate_reject_requests(r);
        if (e.status == SPEC_OK) e.status = validate_reject_unsupported(r);
    }
    if (e.status != SPEC_OK) return e;
    size_t base = 0;
    if (a != nullptr) {
        e.apl = plan_attn(a, tu);
        e.apl.short_attn = attn_estimate_us(a) <= 20.0 ? 1 : 0;
        if (e.apl.use_mfma) make_order(a, e.order);
        base = e.apl.total_bytes;
    }
    if (r != nullptr)
        e.rpl = plan_reject(r, base, tu, (a != nullptr && e.apl.use_mfma) ? attn_estimate_us(a) : -1.0);
    return e;
}

// Tag of a call's tickets (see step_kernel.hip); unique per call within the process, never 0.
uint32_t next_generation()
{
    static std::atomic<uint32_t> counter{0x5EC0u};
    uint32_t g = ++counter;
    if (g == 0) g = ++counter;
    return g;
}

spec_status check_workspace(void *ws, size_t have, size_t need)
{
    if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & (kAlign - 1)) != 0 || have < need) return SPEC_EWORKSPACE;
    return SPEC_OK;
}

AttnParams attn_params(const spec_attn_args *a, const AttnPlan &pl, char *ws, int64_t *errors)
{
    const Tuning &tu = tuning();
    AttnParams p;
    memset(&p, 0, sizeof p);
    p.B = a->B; p.Hq = a->Hq; p.Hkv = a->Hkv; p.d = a->d;
    p.num_blocks = a->num_blocks; p.max_blocks_per_req = a->max_blocks_per_req; p.T = a->T;
    p.kv_layout = a->kv_layout;
    p.chunk_tokens = pl.chunk_tokens; p.max_chunks = pl.max_chunks;
    p.capacity_tokens = pl.capacity_tokens;
    p.row_groups = pl.row_groups;
    const double scale = a->softmax_scale > 0.0f ? (double)a->softmax_scale : 1.0 / sqrt((double)a->d);
    p.scale_log2 = (float)(scale * kLog2eD);
    p.q = a->q; p.k_cache = a->k_cache; p.v_cache = a->v_cache;
    p.block_table = a->block_table; p.kv_len = a->kv_len; p.cu_q_len = a->cu_q_len;
    p.out = a->out;
    p.ws_acc = reinterpret_cast<float *>(ws);
    p.ws_ml = reinterpret_cast<float *>(ws + pl.acc_bytes);
    p.tickets = reinterpret_cast<unsigned long long *>(ws + pl.acc_bytes + pl.ml_bytes);
    p.errors = reinterpret_cast<unsigned long long *>(a->error_count != nullptr ? a->error_count : errors);
    p.generation = next_generation();
    p.fused_combine = pl.fused_combine;
    p.split_p = tu.split_p;
    p.reject_span = tu.reject_span;
    // as many attention blocks as there are block slots: all start at once
    p.attn_first_limit = tu.attn_first_limit >= 0 ? (int32_t)tu.attn_first_limit : 2 * compute_units();
    p.reject_even_xcds = tu.reject_even;
    p.reject_even_limit = compute_units();
    p.reject_first_limit = pl.short_attn ? tu.reject_first_limit : 0;
    return p;
}

RejectParams reject_params(const spec_reject_args *r, const RejectPlan &pl, char *ws)
{
    RejectParams p;
    memset(&p, 0, sizeof p);
    p.B = r->B; p.V = r->V; p.T = r->T;
    p.mode = r->accept_mode;
    p.target_logits = r->target_logits; p.draft_logits = r->draft_logits;
    p.draft_tokens = r->draft_tokens; p.cu_q_len = r->cu_q_len;
    p.seed_lo = (uint32_t)(r->philox_seed & 0xFFFFFFFFull);
    p.seed_hi = (uint32_t)(r->philox_seed >> 32);
    p.step_lo = (uint32_t)(r->philox_step & 0xFFFFFFFFull);
    p.step_hi24 = (uint32_t)((r->philox_step >> 32) & 0xFFFFFFull);
    p.step_device = reinterpret_cast<const unsigned long long *>(r->philox_step_device);
    p.accepted_len = r->accepted_len; p.next_token = r->next_token; p.out_tokens = r->out_tokens;
    p.counters = reinterpret_cast<unsigned long long *>(r->counters);
    p.debug_u_ratio = r->debug_u_ratio;
    p.kv_len = r->kv_len; p.new_kv_len = r->new_kv_len; p.draft_next_len = r->draft_next_len;
    p.stat_segments = pl.stat_segments; p.stat_seg_len = pl.stat_seg_len;
    p.race_segments = pl.race_segments; p.race_seg_len = pl.race_seg_len;
    p.early_stop = pl.early_stop; p.uniform_k = pl.uniform_k;
    p.spin_limit = tuning().spin_limit;
    {
        // (a launch of at most one rejection block per compute unit counts as small)
        const int64_t rows = r->accept_mode == SPEC_ACCEPT_SAMPLE ? 2 * (int64_t)r->T - r->B : r->T;
        p.short_naps = rows * pl.stat_segments + (int64_t)r->B * (pl.race_segments + 1) <= compute_units() ? 1 : 0;
    }
    p.stats = reinterpret_cast<unsigned long long *>(ws + pl.stats_off);
    p.race_partial = reinterpret_cast<unsigned long long *>(ws + pl.partial_off);
    p.race_info = p.race_partial + (size_t)r->B * pl.race_segments * 2;
    p.generation = next_generation();
    return p;
}

spec_status run_attn_generic(const AttnParams &p, int dtype, hipStream_t stream)
{
    hipError_t err = timed(SPEC_KERNEL_ATTN_GENERIC, stream, [&] { return launch_attn_generic(p, dtype, stream); });
    if (err != hipSuccess) return SPEC_EHIP;
    if (p.max_chunks == 1) return SPEC_OK;   // no request is split: every row was written directly
    err = timed(SPEC_KERNEL_ATTN_COMBINE, stream, [&] { return launch_attn_combine(p, stream); });
    return err == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

// Checks shared by the entry points that take both halves; leaves the plan in `plan`.
spec_status prepare_step(const spec_attn_args *attn, const spec_reject_args *reject, const StepPlan *&plan)
{
    spec_status st = validate_attn_scalars(attn);
    if (st != SPEC_OK) return st;
    st = validate_reject_scalars(reject);
    if (st != SPEC_OK) return st;
    if (attn->B != reject->B || attn->T != reject->T) return SPEC_EINVAL;
    plan = &plan_for(attn, reject);
    if (plan->status != SPEC_OK) return plan->status;
    st = validate_attn_table(attn);
    if (st != SPEC_OK) return st;
    return validate_reject_tokens(reject);
}

// The whole step on a given workspace (shared by spec_verify_step and spec_verify_step_static).
spec_status step_on_workspace(const spec_attn_args *attn, const spec_reject_args *reject, const StepPlan &plan,
                              void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const AttnPlan &apl = plan.apl;
    const RejectPlan &rpl = plan.rpl;
    const spec_status st = check_workspace(workspace, workspace_bytes, apl.total_bytes + rpl.total_bytes);
    if (st != SPEC_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const AttnParams ap = attn_params(attn, apl, static_cast<char *>(workspace), reject->counters + 6);
    const RejectParams rp = reject_params(reject, rpl, static_cast<char *>(workspace));
    if (apl.use_mfma) {
        // the whole step in one launch
        hipError_t err = timed_launch(SPEC_KERNEL_STEP, [&](LaunchEvents ev) {
            return launch_step_fused(&ap, apl.row_tiles, &rp, &plan.order, ev, stream);
        });
        if (err == hipSuccess && !apl.fused_combine && apl.max_chunks > 1)
            err = timed(SPEC_KERNEL_ATTN_COMBINE, stream, [&] { return launch_attn_combine(ap, stream); });
        return err == hipSuccess ? SPEC_OK : SPEC_EHIP;
    }
    const spec_status sa = run_attn_generic(ap, attn->qkv_dtype, stream);
    if (sa != SPEC_OK) return sa;
    const hipError_t err =
        timed_launch(SPEC_KERNEL_REJECT, [&](LaunchEvents ev) { return launch_step_fused(nullptr, 0, &rp, nullptr, ev, stream); });
    return err == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

}  // namespace

}  // namespace specv

using namespace specv;

extern "C" {

spec_status spec_validate_attn(const spec_attn_args *attn) { return validate_attn(attn); }

spec_status spec_validate_reject(const spec_reject_args *reject) { return validate_reject(reject); }

void spec_verify_reload_env(void)
{
    (void)tuning();   // the first read, if it has not happened yet
    read_tuning();
}

size_t spec_verify_workspace_bytes(const spec_attn_args *attn, const spec_reject_args *reject)
{
    if (attn == nullptr && reject == nullptr) return 0;
    if (attn != nullptr && validate_attn_scalars(attn) != SPEC_OK) return 0;
    if (reject != nullptr && validate_reject_scalars(reject) != SPEC_OK) return 0;
    if (attn != nullptr && reject != nullptr && (attn->B != reject->B || attn->T != reject->T)) return 0;
    const StepPlan &plan = plan_for(attn, reject);
    if (plan.status != SPEC_OK) return 0;
    return (attn != nullptr ? plan.apl.total_bytes : 0) + (reject != nullptr ? plan.rpl.total_bytes : 0);
}

spec_status spec_verify_plan(const spec_attn_args *attn, const spec_reject_args *reject, spec_plan_info *info)
{
    if (info == nullptr || (attn == nullptr && reject == nullptr)) return SPEC_EINVAL;
    memset(info, 0, sizeof *info);
    spec_status st = attn != nullptr ? validate_attn_scalars(attn) : SPEC_OK;
    if (st != SPEC_OK) return st;
    st = reject != nullptr ? validate_reject_scalars(reject) : SPEC_OK;
    if (st != SPEC_OK) return st;
    if (attn != nullptr && reject != nullptr && (attn->B != reject->B || attn->T != reject->T)) return SPEC_EINVAL;
    const StepPlan &plan = plan_for(attn, reject);
    if (plan.status != SPEC_OK) return plan.status;
    if (attn != nullptr) {
        const AttnPlan &pl = plan.apl;
        info->attn_path = pl.use_mfma ? SPEC_PATH_MFMA : SPEC_PATH_GENERIC;
        info->row_tiles = pl.row_tiles;
        info->row_groups = pl.row_groups;
        info->chunk_tokens = pl.chunk_tokens;
        info->max_chunks = pl.max_chunks;
        if (pl.use_mfma) {
            AttnParams ap;
            memset(&ap, 0, sizeof ap);
            ap.B = attn->B; ap.Hkv = attn->Hkv; ap.max_chunks = pl.max_chunks; ap.row_groups = pl.row_groups;
            info->attn_blocks = step_attn_items(ap);
            info->launches = 1 + ((!pl.fused_combine && pl.max_chunks > 1) ? 1 : 0);
        } else {
            info->attn_blocks = pl.max_chunks * attn->Hq * attn->T;
            info->launches = pl.max_chunks > 1 ? 2 : 1;
        }
        info->workspace_bytes += pl.total_bytes;
    }
    if (reject != nullptr) {
        const RejectPlan &pl = plan.rpl;
        info->early_stop = pl.early_stop;
        info->stat_segments = pl.stat_segments;
        info->race_segments = reject->accept_mode == SPEC_ACCEPT_GREEDY ? 0 : pl.race_segments;
        const int rows = reject->accept_mode == SPEC_ACCEPT_SAMPLE ? 2 * reject->T - reject->B : reject->T;
        info->reject_blocks = rows * pl.stat_segments + reject->B * info->race_segments + reject->B;
        if (attn == nullptr || info->attn_path != SPEC_PATH_MFMA) info->launches += 1;
        info->workspace_bytes += pl.total_bytes;
    }
    return SPEC_OK;
}

spec_status spec_verify_attn(const spec_attn_args *attn, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    spec_status st = validate_attn_scalars(attn);
    if (st != SPEC_OK) return st;
    const StepPlan &plan = plan_for(attn, nullptr);
    if (plan.status != SPEC_OK) return plan.status;
    st = validate_attn_table(attn);
    if (st != SPEC_OK) return st;
    const AttnPlan &pl = plan.apl;
    st = check_workspace(workspace, workspace_bytes, pl.total_bytes);
    if (st != SPEC_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const AttnParams ap = attn_params(attn, pl, static_cast<char *>(workspace), nullptr);
    if (!pl.use_mfma) return run_attn_generic(ap, attn->qkv_dtype, stream);
    hipError_t err = timed_launch(SPEC_KERNEL_ATTN, [&](LaunchEvents ev) {
        return launch_step_fused(&ap, pl.row_tiles, nullptr, &plan.order, ev, stream);
    });
    if (err == hipSuccess && !pl.fused_combine && pl.max_chunks > 1)
        err = timed(SPEC_KERNEL_ATTN_COMBINE, stream, [&] { return launch_attn_combine(ap, stream); });
    return err == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

spec_status spec_reject_sample(const spec_reject_args *reject, void *workspace, size_t workspace_bytes,
                               void *hip_stream)
{
    spec_status st = validate_reject_scalars(reject);
    if (st != SPEC_OK) return st;
    const StepPlan &plan = plan_for(nullptr, reject);
    if (plan.status != SPEC_OK) return plan.status;
    st = validate_reject_tokens(reject);
    if (st != SPEC_OK) return st;
    const RejectPlan &pl = plan.rpl;
    st = check_workspace(workspace, workspace_bytes, pl.total_bytes);
    if (st != SPEC_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const RejectParams rp = reject_params(reject, pl, static_cast<char *>(workspace));
    const hipError_t err =
        timed_launch(SPEC_KERNEL_REJECT, [&](LaunchEvents ev) { return launch_step_fused(nullptr, 0, &rp, nullptr, ev, stream); });
    return err == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

spec_status spec_verify_step(const spec_attn_args *attn, const spec_reject_args *reject, void *workspace,
                             size_t workspace_bytes, void *hip_stream)
{
    const StepPlan *plan = nullptr;
    const spec_status st = prepare_step(attn, reject, plan);
    if (st != SPEC_OK) return st;
    return step_on_workspace(attn, reject, *plan, workspace, workspace_bytes, hip_stream);
}

spec_status spec_verify_step_static(const spec_attn_args *attn, const spec_reject_args *reject, void *hip_stream)
{
    // sizes first, on the host: a step that does not fit is refused before anything touches the GPU
    const StepPlan *plan = nullptr;
    const spec_status st = prepare_step(attn, reject, plan);
    if (st != SPEC_OK) return st;
    if (plan->apl.total_bytes + plan->rpl.total_bytes > SPEC_STATIC_SCRATCH_BYTES) return SPEC_EWORKSPACE;
    void *ws = static_scratch_of_current_device();
    if (ws == nullptr) return SPEC_EHIP;
    return step_on_workspace(attn, reject, *plan, ws, SPEC_STATIC_SCRATCH_BYTES, hip_stream);
}

spec_status spec_kv_append(const spec_kv_append_args *a, void *hip_stream)
{
    if (a == nullptr || a->B < 1 || a->Hkv < 1 || a->T < a->B || a->num_blocks < 1 || a->max_blocks_per_req < 1)
        return SPEC_EINVAL;
    if (a->new_k == nullptr || a->new_v == nullptr || a->k_cache == nullptr || a->v_cache == nullptr ||
        a->block_table == nullptr || a->kv_len == nullptr || a->cu_q_len == nullptr || a->host_kv_len == nullptr ||
        a->host_cu_q_len == nullptr)
        return SPEC_EINVAL;
    if (a->dtype != SPEC_F32 && a->dtype != SPEC_BF16) return SPEC_EINVAL;
    if (a->kv_layout != SPEC_KV_TOKEN_MAJOR && a->kv_layout != SPEC_KV_MFMA) return SPEC_EINVAL;
    // (rows and pools are moved as vectors of 8 elements)
    if (((reinterpret_cast<uintptr_t>(a->new_k) | reinterpret_cast<uintptr_t>(a->new_v) |
          reinterpret_cast<uintptr_t>(a->k_cache) | reinterpret_cast<uintptr_t>(a->v_cache)) & 31) != 0)
        return SPEC_EINVAL;
    if (a->d != 64 && a->d != 128) return SPEC_EUNSUPPORTED;
    if (a->kv_layout == SPEC_KV_MFMA && a->dtype != SPEC_BF16) return SPEC_EUNSUPPORTED;
    if (a->host_cu_q_len[0] != 0 || a->host_cu_q_len[a->B] != a->T) return SPEC_EINVAL;
    for (int b = 0; b < a->B; ++b) {
        const int q_len = a->host_cu_q_len[b + 1] - a->host_cu_q_len[b];
        if (q_len < 1 || q_len > SPEC_K_MAX + 1 || a->host_kv_len[b] < q_len) return SPEC_EINVAL;
        if ((a->host_kv_len[b] + SPEC_BLOCK_SIZE - 1) / SPEC_BLOCK_SIZE > a->max_blocks_per_req) return SPEC_EINVAL;
    }
    KvAppendParams p;
    memset(&p, 0, sizeof p);
    p.B = a->B; p.Hkv = a->Hkv; p.d = a->d; p.max_blocks_per_req = a->max_blocks_per_req; p.T = a->T;
    p.kv_layout = a->kv_layout;
    p.elem_bytes = a->dtype == SPEC_BF16 ? 2 : 4;
    p.num_blocks = a->num_blocks;
    p.new_k = a->new_k; p.new_v = a->new_v; p.k_cache = a->k_cache; p.v_cache = a->v_cache;
    p.block_table = a->block_table; p.kv_len = a->kv_len; p.cu_q_len = a->cu_q_len;
    p.errors = reinterpret_cast<unsigned long long *>(a->error_count);
    return launch_kv_append(p, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

spec_status spec_kv_repack_mfma(const void *src_k, const void *src_v, void *dst_k, void *dst_v, int32_t num_blocks,
                                int32_t Hkv, int32_t d, void *hip_stream)
{
    if (src_k == nullptr || src_v == nullptr || dst_k == nullptr || dst_v == nullptr || num_blocks < 1 || Hkv < 1)
        return SPEC_EINVAL;
    if (src_k == dst_k || src_v == dst_v || src_k == dst_v || src_v == dst_k) return SPEC_EINVAL;
    if (d != 64 && d != 128) return SPEC_EUNSUPPORTED;
    const hipError_t err = launch_kv_repack(src_k, src_v, dst_k, dst_v, num_blocks, Hkv, d,
                                            static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

spec_status spec_profile_begin(int32_t max_launches)
{
    if (max_launches < 1 || max_launches > (1 << 20)) return SPEC_EINVAL;
    if (g_prof.on) return SPEC_EINVAL;
    g_prof.events.assign(2 * (size_t)max_launches, nullptr);
    for (auto &e : g_prof.events)
        if (hipEventCreate(&e) != hipSuccess) return SPEC_EHIP;
    g_prof.kernel_of_pair.clear();
    g_prof.kernel_of_pair.reserve(max_launches);
    g_prof.capacity_pairs = (size_t)max_launches;
    g_prof.on = true;
    return SPEC_OK;
}

spec_status spec_profile_end(float *total_ms, int32_t *launches)
{
    if (!g_prof.on || total_ms == nullptr || launches == nullptr) return SPEC_EINVAL;
    g_prof.on = false;
    for (int i = 0; i < SPEC_NUM_KERNELS; ++i) { total_ms[i] = 0.0f; launches[i] = 0; }
    spec_status st = SPEC_OK;
    for (size_t pair = 0; pair < g_prof.kernel_of_pair.size(); ++pair) {
        float ms = 0.0f;
        if (hipEventSynchronize(g_prof.events[2 * pair + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_prof.events[2 * pair], g_prof.events[2 * pair + 1]) != hipSuccess) {
            st = SPEC_EHIP;
            break;
        }
        total_ms[g_prof.kernel_of_pair[pair]] += ms;
        launches[g_prof.kernel_of_pair[pair]] += 1;
    }
    for (auto &e : g_prof.events) (void)hipEventDestroy(e);
    g_prof.events.clear();
    g_prof.kernel_of_pair.clear();
    g_prof.capacity_pairs = 0;
    return st;
}

const char *spec_status_string(spec_status status)
{
    switch (status) {
        case SPEC_OK: return "ok";
        case SPEC_EINVAL: return "invalid argument";
        case SPEC_EUNSUPPORTED: return "unsupported shape, dtype or layout";
        case SPEC_EWORKSPACE: return "workspace missing, misaligned or too small";
        case SPEC_EHIP: return "HIP call failed";
    }
    return "unknown status";
}

int32_t spec_verify_version(void) { return 200; }

}  // extern "C"
