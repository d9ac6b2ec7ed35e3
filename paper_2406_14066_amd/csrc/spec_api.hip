// C ABI of the speculative-verification library: host-side validation, launch
// planning and the exported entry points declared in spec_verify.h.
#include "common.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <vector>

namespace specv {

namespace {

constexpr size_t kAlign = 256;

// Optional per-kernel timing with HIP events (spec_profile_begin / spec_profile_end).
// Off by default; when on, every kernel launch is bracketed by two event records on
// the launch stream.  Not thread safe; meant for the benchmark.
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

spec_status validate_attn(const spec_attn_args *a)
{
    if (a == nullptr) return SPEC_EINVAL;
    if (a->B < 1 || a->Hq < 1 || a->Hkv < 1 || a->num_blocks < 1 || a->max_blocks_per_req < 1 || a->T < a->B)
        return SPEC_EINVAL;
    if (a->q == nullptr || a->k_cache == nullptr || a->v_cache == nullptr || a->block_table == nullptr ||
        a->kv_len == nullptr || a->cu_q_len == nullptr || a->out == nullptr || a->host_kv_len == nullptr ||
        a->host_cu_q_len == nullptr)
        return SPEC_EINVAL;
    if (a->Hq % a->Hkv != 0) return SPEC_EINVAL;
    if (!(a->softmax_scale >= 0.0f) || isinf(a->softmax_scale)) return SPEC_EINVAL;
    if (a->qkv_dtype != SPEC_F32 && a->qkv_dtype != SPEC_BF16) return SPEC_EINVAL;
    if (a->kv_layout != SPEC_KV_TOKEN_MAJOR && a->kv_layout != SPEC_KV_MFMA) return SPEC_EINVAL;
    if (a->host_cu_q_len[0] != 0 || a->host_cu_q_len[a->B] != a->T) return SPEC_EINVAL;
    for (int b = 0; b < a->B; ++b) {
        const int q_len = a->host_cu_q_len[b + 1] - a->host_cu_q_len[b];
        const int len = a->host_kv_len[b];
        if (q_len < 1 || q_len > SPEC_K_MAX + 1) return SPEC_EINVAL;
        if (len < q_len) return SPEC_EINVAL;
        if ((len + SPEC_BLOCK_SIZE - 1) / SPEC_BLOCK_SIZE > a->max_blocks_per_req) return SPEC_EINVAL;
    }
    if (a->block_size != SPEC_BLOCK_SIZE) return SPEC_EUNSUPPORTED;
    if (a->d != 64 && a->d != 128) return SPEC_EUNSUPPORTED;
    if (a->Hq / a->Hkv > 16) return SPEC_EUNSUPPORTED;
    if (a->kv_layout == SPEC_KV_MFMA && a->qkv_dtype != SPEC_BF16) return SPEC_EUNSUPPORTED;
    if (a->T > 65535 || a->Hq > 65535) return SPEC_EUNSUPPORTED;
    return SPEC_OK;
}

spec_status validate_reject(const spec_reject_args *r)
{
    if (r == nullptr) return SPEC_EINVAL;
    if (r->B < 1 || r->V < 1 || r->T < r->B) return SPEC_EINVAL;
    if (r->target_logits == nullptr || r->cu_q_len == nullptr || r->host_cu_q_len == nullptr ||
        r->accepted_len == nullptr || r->next_token == nullptr || r->counters == nullptr)
        return SPEC_EINVAL;
    if (r->accept_mode != SPEC_ACCEPT_SAMPLE && r->accept_mode != SPEC_ACCEPT_GREEDY &&
        r->accept_mode != SPEC_ACCEPT_POINT_DRAFT)
        return SPEC_EINVAL;
    if (r->T > r->B && r->draft_tokens == nullptr) return SPEC_EINVAL;
    if (r->T > r->B && r->accept_mode == SPEC_ACCEPT_SAMPLE && r->draft_logits == nullptr) return SPEC_EINVAL;
    if (r->host_cu_q_len[0] != 0 || r->host_cu_q_len[r->B] != r->T) return SPEC_EINVAL;
    for (int b = 0; b < r->B; ++b) {
        const int q_len = r->host_cu_q_len[b + 1] - r->host_cu_q_len[b];
        if (q_len < 1 || q_len > SPEC_K_MAX + 1) return SPEC_EINVAL;
    }
    if ((r->new_kv_len != nullptr || r->draft_next_len != nullptr) && r->kv_len == nullptr) return SPEC_EINVAL;
    if (r->V % 4 != 0) return SPEC_EUNSUPPORTED;  // rows are read as 16-byte vectors
    if (r->B > 65535 || 2 * (int64_t)r->T - r->B > 65535) return SPEC_EUNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(r->target_logits) & 15) != 0 ||
        (r->accept_mode == SPEC_ACCEPT_SAMPLE && (reinterpret_cast<uintptr_t>(r->draft_logits) & 15) != 0))
        return SPEC_EINVAL;
    return SPEC_OK;
}

// Split of the KV length.  The matrix-instruction kernel runs one block per
// (request, KV head, chunk); the chunk is sized so that the launch has about
// eight blocks per compute unit, in multiples of the 64 tokens a block's four
// wavefronts take per round.
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

AttnPlan plan_attn(const spec_attn_args *a)
{
    AttnPlan pl;
    memset(&pl, 0, sizeof pl);
    int max_len = 0, max_q = 0;
    for (int b = 0; b < a->B; ++b) {
        if (a->host_kv_len[b] > max_len) max_len = a->host_kv_len[b];
        const int q_len = a->host_cu_q_len[b + 1] - a->host_cu_q_len[b];
        if (q_len > max_q) max_q = q_len;
    }
    pl.max_q_len = max_q;
    const int group = a->Hq / a->Hkv;
    const int rows = max_q * group;
    pl.row_tiles = (rows + 15) / 16;
    pl.use_mfma = (a->qkv_dtype == SPEC_BF16 && a->kv_layout == SPEC_KV_MFMA && a->d == 128 && pl.row_tiles <= 3) ? 1 : 0;
    // diagnostic switch: SPEC_VERIFY_FORCE_GENERIC=1 routes every shape through the generic kernel
    const char *force = getenv("SPEC_VERIFY_FORCE_GENERIC");
    if (force != nullptr && force[0] == '1') pl.use_mfma = 0;
    if (pl.use_mfma) {
        // One block per (request, KV head, chunk).  Splitting costs (partials, a merge, more
        // block start-ups), so the longest request is split only as far as needed to give every
        // compute unit a block.  With three row tiles the wavefronts spend a larger share of their
        // time on arithmetic and need a second block beside them to keep loads in flight: then
        // the target is two blocks per compute unit, less a sixteenth of the slots, which the
        // rejection items flow through while the attention blocks (all resident from the start)
        // stream.
        const long cus = compute_units();
        long target_blocks = pl.row_tiles >= 3 ? 2 * cus - cus / 8 : cus;
        if (const char *t = getenv("SPEC_VERIFY_TARGET_BLOCKS")) {   // tuning switch
            const long v = strtol(t, nullptr, 10);
            if (v >= 1 && v <= (1 << 20)) target_blocks = v;
        }
        const int64_t units = (int64_t)a->B * a->Hkv;
        int64_t nsplit = (target_blocks + units - 1) / units;
        if (nsplit < 1) nsplit = 1;
        int64_t chunk = (max_len + nsplit - 1) / nsplit;
        chunk = (chunk + SPEC_BLOCK_SIZE - 1) / SPEC_BLOCK_SIZE * SPEC_BLOCK_SIZE;
        if (chunk < 64) chunk = 64;
        if (chunk > 4096) chunk = 4096;  // a wavefront holds its pages' block-table entries one per lane
        if (const char *forced = getenv("SPEC_VERIFY_CHUNK")) {      // tuning switch: tokens, multiple of 16
            const long v = strtol(forced, nullptr, 10);
            if (v >= 16 && v <= 4096 && v % SPEC_BLOCK_SIZE == 0) chunk = v;
        }
        pl.chunk_tokens = (int32_t)chunk;
    } else {
        pl.chunk_tokens = 256;  // one key per thread of the generic kernel
    }
    pl.max_chunks = (max_len + pl.chunk_tokens - 1) / pl.chunk_tokens;
    pl.fused_combine = (pl.use_mfma && pl.max_chunks <= kMaxFusedChunks) ? 1 : 0;
    // (a request that is not split writes its output directly: the matrix kernel needs no partial
    // slots when no request has a second chunk)
    const size_t slots = (pl.use_mfma && pl.max_chunks == 1) ? 0 : (size_t)a->T * a->Hq * pl.max_chunks;
    pl.acc_bytes = align_up(slots * a->d * sizeof(float));
    pl.ml_bytes = align_up(slots * 2 * sizeof(float));
    pl.ticket_bytes = align_up((size_t)a->B * a->Hkv * sizeof(unsigned long long));
    pl.total_bytes = pl.acc_bytes + pl.ml_bytes + pl.ticket_bytes;
    return pl;
}

// attn_us: rough duration of the attention half that runs in the same launch (microseconds), or
// negative if the rejection half runs alone.
RejectPlan plan_reject(const spec_reject_args *r, size_t base, double attn_us = -1.0)
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
    int race_blocks = 512;
    if (const char *e = getenv("SPEC_VERIFY_RACE_BLOCKS")) {   // tuning switch
        const int v = atoi(e);
        if (v >= 1 && v <= 65536) race_blocks = v;
    }
    int rsegs = (race_blocks + r->B - 1) / r->B;
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
    // hidden: under an attention half that takes clearly longer than the chain, or, when the
    // rejection half runs alone, behind several rounds of blocks per position.  Measured (step
    // with / without): B=256 k=2 (64/8 heads) -4%, B=64 k=8 (32/32 heads, L=1024) -8%, B=64 k=4 -3%,
    // B=32 k=1..3 -2%, B=32 k=4 +2%, B=32 k=8 +16%, B=16 k=2 (L=2048) +2%, B=8 k=4 +32%.
    pl.early_stop = 0;
    pl.uniform_k = 0;
    if (r->T > r->B && r->T % r->B == 0) {
        const int q = r->T / r->B;
        bool uniform = true;
        for (int b = 0; b < r->B && uniform; ++b) uniform = r->host_cu_q_len[b + 1] - r->host_cu_q_len[b] == q;
        bool wanted;
        if (attn_us >= 0.0) {
            wanted = r->B >= 32 && 12.0 * q + 30.0 <= 0.85 * attn_us;
        } else {
            const int64_t per_position = (int64_t)(r->accept_mode == SPEC_ACCEPT_SAMPLE ? 2 : 1) * r->B * pl.stat_segments;
            wanted = (int64_t)rows * pl.stat_segments >= 3ll * compute_units() && per_position >= compute_units();
        }
        if (const char *e = getenv("SPEC_VERIFY_EARLY_STOP")) wanted = e[0] != '0';   // tuning switch
        if (uniform && wanted) { pl.early_stop = 1; pl.uniform_k = q - 1; }
    }
    pl.stats_off = base;
    pl.stats_bytes = align_up((size_t)rows * pl.stat_segments * kStatWords * sizeof(unsigned long long));
    pl.partial_off = pl.stats_off + pl.stats_bytes;
    pl.partial_bytes = align_up(((size_t)r->B * pl.race_segments * 2 + r->B) * sizeof(unsigned long long));
    pl.total_bytes = pl.stats_bytes + pl.partial_bytes;
    return pl;
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

AttnParams attn_params(const spec_attn_args *a, const AttnPlan &pl, char *ws)
{
    AttnParams p;
    memset(&p, 0, sizeof p);
    p.B = a->B; p.Hq = a->Hq; p.Hkv = a->Hkv; p.d = a->d;
    p.num_blocks = a->num_blocks; p.max_blocks_per_req = a->max_blocks_per_req; p.T = a->T;
    p.kv_layout = a->kv_layout;
    p.chunk_tokens = pl.chunk_tokens; p.max_chunks = pl.max_chunks;
    const double scale = a->softmax_scale > 0.0f ? (double)a->softmax_scale : 1.0 / sqrt((double)a->d);
    p.scale_log2 = (float)(scale * kLog2eD);
    p.q = a->q; p.k_cache = a->k_cache; p.v_cache = a->v_cache;
    p.block_table = a->block_table; p.kv_len = a->kv_len; p.cu_q_len = a->cu_q_len;
    p.out = a->out;
    p.ws_acc = reinterpret_cast<float *>(ws);
    p.ws_ml = reinterpret_cast<float *>(ws + pl.acc_bytes);
    p.tickets = reinterpret_cast<unsigned long long *>(ws + pl.acc_bytes + pl.ml_bytes);
    p.generation = next_generation();
    p.fused_combine = pl.fused_combine;
    p.single_chunk_direct = pl.use_mfma;
    p.split_p = 1;
    p.reject_span = 0.5f;
    if (const char *e = getenv("SPEC_VERIFY_REJECT_SPAN")) {   // tuning switch
        const double v = strtod(e, nullptr);
        if (v > 0.0 && v <= 1.0) p.reject_span = (float)v;
    }
    p.attn_first_limit = 2 * compute_units();   // as many attention blocks as there are block slots: all start at once
    if (const char *e = getenv("SPEC_VERIFY_ATTN_FIRST_LIMIT")) {   // tuning switch
        const long v = strtol(e, nullptr, 10);
        if (v >= 0 && v <= (1 << 20)) p.attn_first_limit = (int32_t)v;
    }
    if (const char *e = getenv("SPEC_VERIFY_SPLIT_P")) p.split_p = (e[0] != '0');   // experiment switch
    p.reject_even_xcds = 1;
    p.reject_even_limit = compute_units();
    if (const char *e = getenv("SPEC_VERIFY_REJECT_EVEN")) p.reject_even_xcds = (e[0] != '0');   // tuning switch
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
    p.accepted_len = r->accepted_len; p.next_token = r->next_token; p.out_tokens = r->out_tokens;
    p.counters = reinterpret_cast<unsigned long long *>(r->counters);
    p.debug_u_ratio = r->debug_u_ratio;
    p.kv_len = r->kv_len; p.new_kv_len = r->new_kv_len; p.draft_next_len = r->draft_next_len;
    p.stat_segments = pl.stat_segments; p.stat_seg_len = pl.stat_seg_len;
    p.race_segments = pl.race_segments; p.race_seg_len = pl.race_seg_len;
    p.early_stop = pl.early_stop; p.uniform_k = pl.uniform_k;
    p.spin_limit = 1 << 20;   // about a second of polling; never reached in a healthy launch
    p.stats = reinterpret_cast<unsigned long long *>(ws + pl.stats_off);
    p.race_partial = reinterpret_cast<unsigned long long *>(ws + pl.partial_off);
    p.race_info = p.race_partial + (size_t)r->B * pl.race_segments * 2;
    p.generation = next_generation();
    return p;
}

// Requests by falling KV length (stable; from the host copy of kv_len).  The grid takes the
// attention items in this order: blocks that run at the same time then take about
// equally long, which the in-order hardware dispatcher needs to keep its block slots
// filled, and the short items even out the end of the launch.  Returns null (given order)
// when all lengths are equal or there are too many requests for the table.
const UnitOrder *make_order(const spec_attn_args *a, UnitOrder &order)
{
    order.n = 0;
    if (a->B > kMaxOrdered) return nullptr;
    bool equal = true;
    for (int b = 1; b < a->B; ++b)
        if (a->host_kv_len[b] != a->host_kv_len[0]) equal = false;
    if (equal) return nullptr;
    std::vector<int> idx(a->B);
    for (int b = 0; b < a->B; ++b) idx[b] = b;
    std::stable_sort(idx.begin(), idx.end(), [&](int x, int y) { return a->host_kv_len[x] > a->host_kv_len[y]; });
    for (int b = 0; b < a->B; ++b) order.request[b] = (uint16_t)idx[b];
    order.n = a->B;
    return &order;
}

spec_status run_attn_generic(const AttnParams &p, int dtype, hipStream_t stream)
{
    hipError_t err = timed(SPEC_KERNEL_ATTN_GENERIC, stream, [&] { return launch_attn_generic(p, dtype, stream); });
    if (err != hipSuccess) return SPEC_EHIP;
    err = timed(SPEC_KERNEL_ATTN_COMBINE, stream, [&] { return launch_attn_combine(p, stream); });
    return err == hipSuccess ? SPEC_OK : SPEC_EHIP;
}


// ---------------------------------------------------------------------------
// Scratch memory for callers that cannot allocate (spec_verify_step_static): one file-scope
// device array per GPU, held until the process ends.  In host code the array's name is only
// a stand-in for the symbol; its device address is resolved once per device, with that device
// current, and kept.  Each GPU has its own copy of the array at its own address.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[SPEC_STATIC_SCRATCH_BYTES];

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

// The whole step on a given workspace (shared by spec_verify_step and spec_verify_step_static).
spec_status step_on_workspace(const spec_attn_args *attn, const spec_reject_args *reject, void *workspace,
                              size_t workspace_bytes, void *hip_stream)
{
    spec_status st = validate_attn(attn);
    if (st != SPEC_OK) return st;
    st = validate_reject(reject);
    if (st != SPEC_OK) return st;
    if (attn->B != reject->B || attn->T != reject->T) return SPEC_EINVAL;
    const AttnPlan apl = plan_attn(attn);
    // (the KV bytes at 5.5 TB/s: what the attention half takes when it streams well)
    double kv_bytes = 0.0;
    for (int b = 0; b < attn->B; ++b) kv_bytes += (double)attn->host_kv_len[b];
    kv_bytes *= 2.0 * attn->Hkv * attn->d * (attn->qkv_dtype == SPEC_BF16 ? 2 : 4);
    const RejectPlan rpl = plan_reject(reject, apl.total_bytes, apl.use_mfma ? kv_bytes / 5.5e6 : -1.0);
    st = check_workspace(workspace, workspace_bytes, apl.total_bytes + rpl.total_bytes);
    if (st != SPEC_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const AttnParams ap = attn_params(attn, apl, static_cast<char *>(workspace));
    const RejectParams rp = reject_params(reject, rpl, static_cast<char *>(workspace));
    if (apl.use_mfma) {
        // the whole step in one launch
        UnitOrder order_table;
        const UnitOrder *order = make_order(attn, order_table);
        hipError_t err = timed_launch(SPEC_KERNEL_STEP, [&](LaunchEvents ev) {
            return launch_step_fused(&ap, apl.row_tiles, &rp, order, ev, stream);
        });
        if (err == hipSuccess && !apl.fused_combine && apl.max_chunks > 1)
            err = timed(SPEC_KERNEL_ATTN_COMBINE, stream, [&] { return launch_attn_combine(ap, stream); });
        return err == hipSuccess ? SPEC_OK : SPEC_EHIP;
    }
    st = run_attn_generic(ap, attn->qkv_dtype, stream);
    if (st != SPEC_OK) return st;
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

size_t spec_verify_workspace_bytes(const spec_attn_args *attn, const spec_reject_args *reject)
{
    size_t total = 0;
    if (attn != nullptr) {
        if (validate_attn(attn) != SPEC_OK) return 0;
        total += plan_attn(attn).total_bytes;
    }
    if (reject != nullptr) {
        if (validate_reject(reject) != SPEC_OK) return 0;
        total += plan_reject(reject, total).total_bytes;
    }
    return total;
}

spec_status spec_verify_attn(const spec_attn_args *attn, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    spec_status st = validate_attn(attn);
    if (st != SPEC_OK) return st;
    const AttnPlan pl = plan_attn(attn);
    st = check_workspace(workspace, workspace_bytes, pl.total_bytes);
    if (st != SPEC_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const AttnParams ap = attn_params(attn, pl, static_cast<char *>(workspace));
    if (!pl.use_mfma) return run_attn_generic(ap, attn->qkv_dtype, stream);
    UnitOrder order_table;
    const UnitOrder *order = make_order(attn, order_table);
    hipError_t err = timed_launch(SPEC_KERNEL_ATTN, [&](LaunchEvents ev) {
        return launch_step_fused(&ap, pl.row_tiles, nullptr, order, ev, stream);
    });
    if (err == hipSuccess && !pl.fused_combine && pl.max_chunks > 1)
        err = timed(SPEC_KERNEL_ATTN_COMBINE, stream, [&] { return launch_attn_combine(ap, stream); });
    return err == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

spec_status spec_reject_sample(const spec_reject_args *reject, void *workspace, size_t workspace_bytes,
                               void *hip_stream)
{
    spec_status st = validate_reject(reject);
    if (st != SPEC_OK) return st;
    const RejectPlan pl = plan_reject(reject, 0);
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
    return step_on_workspace(attn, reject, workspace, workspace_bytes, hip_stream);
}

spec_status spec_verify_step_static(const spec_attn_args *attn, const spec_reject_args *reject, void *hip_stream)
{
    // sizes first, on the host: a step that does not fit is refused before anything touches the GPU
    spec_status st = validate_attn(attn);
    if (st != SPEC_OK) return st;
    st = validate_reject(reject);
    if (st != SPEC_OK) return st;
    if (attn->B != reject->B || attn->T != reject->T) return SPEC_EINVAL;
    const size_t need = spec_verify_workspace_bytes(attn, reject);
    if (need == 0) return SPEC_EINVAL;
    if (need > SPEC_STATIC_SCRATCH_BYTES) return SPEC_EWORKSPACE;
    void *ws = static_scratch_of_current_device();
    if (ws == nullptr) return SPEC_EHIP;
    return step_on_workspace(attn, reject, ws, SPEC_STATIC_SCRATCH_BYTES, hip_stream);
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
    p.new_k = a->new_k; p.new_v = a->new_v; p.k_cache = a->k_cache; p.v_cache = a->v_cache;
    p.block_table = a->block_table; p.kv_len = a->kv_len; p.cu_q_len = a->cu_q_len;
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

int32_t spec_verify_version(void) { return 100; }

}  // extern "C"
