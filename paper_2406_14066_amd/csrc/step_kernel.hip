// The speculative-verification step as ONE kernel launch (arXiv 2406.14066:
// "score" = lookahead attention of the k+1 query positions against the paged KV
// cache, Section 2.2 / Section 4; "accept" = rejection sampling with bonus token,
// Section 4; the accept rule is the cited speculative-sampling method's).
//
// The grid is a list of work items; a block's index selects its role:
//
//   statistics   one (logit row, vocabulary segment) each: offset and sum of
//                exponentials, published with the call's generation tag.
//   race         one (request, vocabulary segment) each: recomputes the request's
//                (cheap) accept chain from the published statistics, then races
//                its segment for the next token.
//   final        one per request: picks the race winner, writes the request's
//                outputs and counters.
//   attention    one (request, KV head, KV chunk) each; the block that completes
//                the LAST chunk of a (request, KV head) merges the chunk partials
//                and writes the output.
// Other acceptance rules reuse the stages: greedy acceptance computes (largest logit,
// lowest id) per (target row, segment) in the statistics stage and has no race; a
// point-mass draft needs statistics of the target rows only and leaves the rejected
// token out of the race.
// Large batches with one draft length take the statistics items in position order and skip
// the rows after a request's first rejection (stats_role): the accept chain of a request
// stops there (Section 4), so those rows decide nothing.
// The rejection items keep that order among themselves and are mixed into the first part
// of the attention items (see GridSplit), so that the rejection half, whose stages depend
// on each other, runs underneath the attention stream and is done before it.
//
// Attention blocks never wait: "last one out merges" is decided with one atomic
// ticket per (request, KV head).  Race and final items consume what earlier items
// of the grid published (tagged with the call's generation).  The producers precede
// the consumers in the grid, so they were dispatched before them, and they wait for
// nothing: the bounded wait that checks for the data always ends.  (Same-address atomic
// tickets cost about 0.3 us per arrival here, so they are kept for the attention chunks,
// which arrive spread out in time, and avoided for the hundreds of statistics blocks of a
// request, which arrive together.)  Tickets and records carry the call's generation tag
// in their high half, so a workspace needs no zero-initialisation and a call that never
// finished cannot poison the next; the last user also resets them, so a replayed HIP
// graph (same tag) works too.
//
// Attention arithmetic, per 16-token page and 16-row tile (lane = 16*g + n):
//   S^T[token][row] = K[token][:] . Q[row][:]        4 x v_mfma_f32_16x16x32_bf16
//   base-2 online softmax on the lane's tokens 4g..4g+3 of query row n
//   O^T[dim][row] += V^T[dim][token] . P^T[token][row]   8 x v_mfma_f32_16x16x16_bf16,
//   P^T being S^T's own accumulator layout; P is fed as bf16 high + low parts so
//   that its rounding does not limit the result.  All q_len * (Hq/Hkv) query rows
//   sharing a KV head are fused into the N dimension: K and V are read once.
//
// Rejection arithmetic: the streaming part is fp32; what happens once per row or
// per decision (segment sums, log-sum-exp, p/q of the draft token, the comparison
// with u) is fp64.
#include "common.h"

#include <hip/hip_ext.h>

#include <float.h>
#include <math.h>
#include <stddef.h>
#include <string.h>

#include <type_traits>

namespace specv {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kD = 128;   // head dim of the main variants (those for 64: see head_dim_of)
constexpr int kBufferFlags = 0x00020000;   // raw 32-bit buffer descriptor, word 3
// Cache policy of the loads that stream data read once (KV pages, the race's logit rows):
// non-temporal, i.e. the lines are first in line for replacement in the L2.  Without it the
// stream pushes out what the blocks do come back to (code, block tables, queries, hand-off
// words); measured on the four large workloads the hint alone takes 8-10% off the step.
constexpr int kStreamPolicy = 2;           // "nt" bit of a raw buffer load
constexpr float kRescaleSlack = 8.0f;      // see the online softmax of the attention role
constexpr int kXcds = 8;                   // the hardware deals consecutive blocks of a grid to the 8 XCDs in turn

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Exchanges between the four 16-lane rows of a wavefront with the gfx950 row-swap instructions
// (vector ALU, a few cycles) instead of a round trip through the LDS crossbar, which is what a
// generic lane shuffle by 16 or 32 compiles to: v_permlane16_swap trades the odd rows of its
// first operand with the even rows of its second, v_permlane32_swap the upper half of the first
// with the lower half of the second.  Fed the same value twice, the two results hold, in every
// lane l, the values of lanes l and l ^ 16 (l ^ 32).
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float max_across_xor16(float v)
{
    const u32x2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float max_across_xor32(float v)
{
    const u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_rows(float v)   // over lanes l, l ^ 16, l ^ 32, l ^ 48
{
    u32x2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 16 bytes of logits that this launch will not read again (see kStreamPolicy).
__device__ __forceinline__ float4 load_streaming(const float *p)
{
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
    return make_float4(v[0], v[1], v[2], v[3]);
}

// ---------------------------------------------------------------------------
// Tickets.  Word = generation << 32 | arrivals.  Returns how many blocks arrived
// before this one.  The common case is one atomic add: the word carries this call's
// generation already.  The first arrivals of a call find something else (garbage, the
// zero its last user left, or either plus what other early arrivals added) and replace
// it; the last arrival, which is the one the merge waits for, is never among them.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t ticket_arrive(unsigned long long *ticket, uint32_t generation)
{
    const unsigned long long got = atomicAdd(ticket, 1ull);
    if ((uint32_t)(got >> 32) == generation) return (uint32_t)got;
    unsigned long long cur = got + 1ull;
    for (;;) {
        const unsigned long long first = ((unsigned long long)generation << 32) | 1ull;
        const unsigned long long seen = atomicCAS(ticket, cur, first);
        if (seen == cur) return 0u;
        if ((uint32_t)(seen >> 32) == generation) return (uint32_t)atomicAdd(ticket, 1ull);
        cur = seen;
    }
}

__device__ __forceinline__ void ticket_reset(unsigned long long *ticket)
{
    __hip_atomic_store(ticket, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Data handed from one block to another inside the launch (chunk partials, row
// statistics) is written and read with relaxed agent-scope atomic accesses, which
// go past the non-coherent cache levels, and published by waiting for the
// writes to complete before the ticket is taken.  A full agent-scope fence would
// also write back and invalidate the whole L2 of the XCD on every block; that is
// far too slow for thousands of blocks.
__device__ __forceinline__ void publish_u64(unsigned long long *dst, unsigned long long v)
{
    __hip_atomic_store(dst, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ unsigned long long fetch_u64(const unsigned long long *src)
{
    return __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ unsigned long long pack_f32x2(float a, float b)
{
    return (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
}

// A 32-bit payload and the call's generation tag in one 8-byte word: written and read
// atomically, so a reader that finds this call's tag also has the payload, with no
// ordering needed between the words of a record.
__device__ __forceinline__ void publish_tagged(unsigned long long *dst, uint32_t payload, uint32_t generation)
{
    publish_u64(dst, (unsigned long long)payload | ((unsigned long long)generation << 32));
}

__device__ __forceinline__ bool tagged_ok(unsigned long long word, uint32_t generation)
{
    return (uint32_t)(word >> 32) == generation;
}

__device__ __forceinline__ void writes_complete()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);  // every outstanding store of this wavefront has been acknowledged
}

__device__ __forceinline__ void order_after_ticket()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// Read-only inputs indexed by a block-uniform value (lengths, row offsets) are read through
// the constant address space, which makes them scalar loads: they are served by the scalar
// cache (these arrays are small and every block reads them) instead of a round trip to
// the L2 under load, and they have a wait counter of their own.
typedef const int32_t __attribute__((address_space(4))) *uniform_i32_ptr;
__device__ __forceinline__ int uniform_load(const int32_t *base, int index)
{
    return ((uniform_i32_ptr)(uintptr_t)base)[__builtin_amdgcn_readfirstlane(index)];
}

// ===========================================================================
// Rejection half
// ===========================================================================

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies,
// a word permutation with key xor, and a Weyl sequence on the key.
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // full 64-bit products: one multiply instruction each instead of a high and a low one
        const unsigned long long pa = (unsigned long long)0xD2511F53u * (unsigned long long)c.x;
        const unsigned long long pb = (unsigned long long)0xCD9E8D57u * (unsigned long long)c.z;
        c = make_uint4((uint32_t)(pb >> 32) ^ c.y ^ k0, (uint32_t)pb, (uint32_t)(pa >> 32) ^ c.w ^ k1, (uint32_t)pa);
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c;
}

// The step counter of the random numbers: the launch's own, or, if the caller gave a device word
// (a captured launch that draws fresh numbers on every replay), what that word holds now.
struct StepWords {
    uint32_t lo, hi24;
};
typedef const unsigned long long __attribute__((address_space(4))) *uniform_u64_ptr;
__device__ __forceinline__ StepWords philox_step_words(const RejectParams &p)
{
    StepWords w = {p.step_lo, p.step_hi24};
    if (p.step_device != nullptr) {
        const unsigned long long s = *((uniform_u64_ptr)(uintptr_t)p.step_device);
        w.lo = (uint32_t)s;
        w.hi24 = (uint32_t)(s >> 32) & 0xFFFFFFu;
    }
    return w;
}

constexpr int kMaxStatSegments = 32;
constexpr float kLog2eHi = 1.4426950216293335f;     // fp32(log2 e)
constexpr float kLog2eLo = 1.9259629911266175e-8f;  // log2 e - kLog2eHi

struct RejectShared {
    float red_f[kWaves];
    double red_d[kWaves];
    double lse2[2 * SPEC_K_MAX + 1];  // log2-sum-exp: target rows 0..k, then draft rows 0..k-1
    double u[SPEC_K_MAX], ratio[SPEC_K_MAX];
    int accept[SPEC_K_MAX];
    int m, near, last;
    float best_score[kWaves];
    int best_id[kWaves];
    double seg_sum[2 * SPEC_K_MAX + 1][kMaxStatSegments];
    float seg_off[2 * SPEC_K_MAX + 1][kMaxStatSegments];
};

// One (row, segment): offset and sum of 2^(x*log2e - offset) over the segment.
// The running offset is integer-valued in base-2 units, so every rescale is an
// exact power of two and x*log2(e) - offset is rounded once (log2 e enters as an
// fp32 hi/lo pair inside fused multiply-adds).
template <int UNROLL>   // vectors of 16 bytes in flight per thread (these blocks share the attention role's register budget)
__device__ __forceinline__ void stats_block(const RejectParams &p, int row, int seg, RejectShared &sh)
{
    const int tid = threadIdx.x;
    const float *base = row < p.T ? p.target_logits + (size_t)row * p.V
                                  : p.draft_logits + (size_t)(row - p.T) * p.V;
    const int v0 = seg * p.stat_seg_len;
    const int v1 = min(p.V, v0 + p.stat_seg_len);
    const float4 *vec = reinterpret_cast<const float4 *>(base + v0);
    const int nvec = (v1 - v0) >> 2;

    float m = -FLT_MAX;   // largest logit seen
    float off = kEmptyMax;
    float s = 0.0f;
    for (int i = tid; i < nvec; i += kThreads * UNROLL) {
        float4 x[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int idx = i + u * kThreads;
            x[u] = idx < nvec ? vec[idx] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        }
        float cm = m;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) cm = fmaxf(cm, fmaxf(fmaxf(x[u].x, x[u].y), fmaxf(x[u].z, x[u].w)));
        if (cm > m) {
            const float new_off = ceilf(cm * kLog2eHi);
            s *= fast_exp2(off - new_off);
            off = new_off;
            m = cm;
        }
        const float noff = -off;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            s += fast_exp2(fmaf(x[u].x, kLog2eHi, fmaf(x[u].x, kLog2eLo, noff)));
            s += fast_exp2(fmaf(x[u].y, kLog2eHi, fmaf(x[u].y, kLog2eLo, noff)));
            s += fast_exp2(fmaf(x[u].z, kLog2eHi, fmaf(x[u].z, kLog2eLo, noff)));
            s += fast_exp2(fmaf(x[u].w, kLog2eHi, fmaf(x[u].w, kLog2eLo, noff)));
        }
    }

    const int wave = tid / kWave, lane = tid % kWave;
    float wm = off;
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) wm = fmaxf(wm, __shfl_xor(wm, o));
    if (lane == 0) sh.red_f[wave] = wm;
    __syncthreads();
    float boff = sh.red_f[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) boff = fmaxf(boff, sh.red_f[w]);
    // one exact power-of-two rescale per thread, then the cross-thread sum in fp64
    double sd = (double)s * (double)fast_exp2(off - boff);
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) sd += __shfl_xor(sd, o);
    if (lane == 0) sh.red_d[wave] = sd;
    __syncthreads();
    if (tid == 0) {
        double total = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) total += sh.red_d[w];
        // three tagged words: low and high half of the fp64 sum, and the offset
        unsigned long long *dst = p.stats + 3 * ((size_t)row * p.stat_segments + seg);
        const unsigned long long bits = (unsigned long long)__double_as_longlong(total);
        publish_tagged(dst + 0, (uint32_t)bits, p.generation);
        publish_tagged(dst + 1, (uint32_t)(bits >> 32), p.generation);
        publish_tagged(dst + 2, __float_as_uint(boff), p.generation);
    }
}

// Greedy mode: one (target row, segment): the largest logit and the lowest id that has it.
__device__ __forceinline__ void argmax_block(const RejectParams &p, int row, int seg, RejectShared &sh)
{
    constexpr int UNROLL = 16;
    const int tid = threadIdx.x;
    const float *base = p.target_logits + (size_t)row * p.V;
    const int v0 = seg * p.stat_seg_len;
    const int v1 = min(p.V, v0 + p.stat_seg_len);
    const float4 *vec = reinterpret_cast<const float4 *>(base + v0);
    const int nvec = (v1 - v0) >> 2;
    float best = -INFINITY;
    int best_id = 0x7FFFFFFF;
    for (int i = tid; i < nvec; i += kThreads * UNROLL) {
        float4 x[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int idx = i + u * kThreads;
            x[u] = idx < nvec ? vec[idx] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            // vectors past the end were filled with -inf and ids that only grow: they change
            // nothing unless the whole row is -inf, and then the lowest id still wins
            const int id0 = v0 + 4 * (i + u * kThreads);
            if (x[u].x > best || (x[u].x == best && id0 + 0 < best_id)) { best = x[u].x; best_id = id0 + 0; }
            if (x[u].y > best || (x[u].y == best && id0 + 1 < best_id)) { best = x[u].y; best_id = id0 + 1; }
            if (x[u].z > best || (x[u].z == best && id0 + 2 < best_id)) { best = x[u].z; best_id = id0 + 2; }
            if (x[u].w > best || (x[u].w == best && id0 + 3 < best_id)) { best = x[u].w; best_id = id0 + 3; }
        }
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        const float ov = __shfl_xor(best, o);
        const int oi = __shfl_xor(best_id, o);
        if (ov > best || (ov == best && oi < best_id)) { best = ov; best_id = oi; }
    }
    const int wave = tid / kWave, lane = tid % kWave;
    if (lane == 0) { sh.best_score[wave] = best; sh.best_id[wave] = best_id; }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < kWaves; ++w) {
            const float ov = sh.best_score[w];
            const int oi = sh.best_id[w];
            if (ov > best || (ov == best && oi < best_id)) { best = ov; best_id = oi; }
        }
        unsigned long long *dst = p.stats + 3 * ((size_t)row * p.stat_segments + seg);
        publish_tagged(dst + 0, __float_as_uint(best), p.generation);
        publish_tagged(dst + 1, (uint32_t)best_id, p.generation);
    }
}

__device__ __forceinline__ float race_exponential(uint32_t word)
{
    // U' = n * 2^-24 with n = (word >> 8) + 1 in [1, 2^24]; e = -log(U').
    const uint32_t n = (word >> 8) + 1u;
    const uint32_t j = 16777216u - n;  // U' = 1 - j * 2^-24
    if (j < 4096u) {
        // -log(1 - x) = x + x^2/2 + x^3/3 + ..., x < 2^-12: three terms are exact to fp32
        const float x = (float)j * 5.9604644775390625e-8f;
        return x * fmaf(x, fmaf(x, 0.33333334f, 0.5f), 1.0f);
    }
    const float u = (float)n * 5.9604644775390625e-8f;
    return -__builtin_amdgcn_logf(u) * kLn2;   // v_log_f32 is log2
}

// The race over vocabulary ids [v0, v1) of one request: best r_v / e_v, e_v = -log(U'_v).
// draft_row == nullptr: weights are the target probabilities (bonus token), with
// exclude_id left out (point-mass draft: the rejected token; -1: none);
// otherwise the positive part of p - q.
//   p_v = corr_t * 2^(x_v * log2e + off_t), off_t = fp32(-log2-sum-exp), corr_t the
//   factor lost by rounding off_t.  Ties keep the lowest id; weights <= 0 never win.
// Returns the block's best (score, id) to every thread.
__device__ __forceinline__ void race_segment(const RejectParams &p, const float *target_row, const float *draft_row, int exclude_id,
                             int b, int v0, int v1, float off_t, float corr_t, float off_d, float corr_d,
                             RejectShared &sh, float &win_score, int &win_id)
{
    float best_score = -1.0f;
    int best_id = 0x7FFFFFFF;
    const int g_begin = v0 >> 2, g_end = v1 >> 2;
    const StepWords step = philox_step_words(p);
    const uint32_t c3 = (step.hi24 << 8) | 1u;
    constexpr int U = 8;  // row vectors in flight per thread
    for (int g0 = g_begin + threadIdx.x; g0 < g_end; g0 += kThreads * U) {
        float4 xt[U], xd[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = g0 + u * kThreads;
            const float4 ninf = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            xt[u] = g < g_end ? load_streaming(target_row + 4 * g) : ninf;
            xd[u] = (draft_row != nullptr && g < g_end) ? load_streaming(draft_row + 4 * g) : ninf;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = g0 + u * kThreads;
            if (g >= g_end) break;
            const int v = 4 * g;
            float r[4];
            {
                const float x[4] = {xt[u].x, xt[u].y, xt[u].z, xt[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    r[e] = corr_t * fast_exp2(fmaf(x[e], kLog2eHi, fmaf(x[e], kLog2eLo, off_t)));
            }
            if (draft_row != nullptr) {
                const float x[4] = {xd[u].x, xd[u].y, xd[u].z, xd[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    r[e] -= corr_d * fast_exp2(fmaf(x[e], kLog2eHi, fmaf(x[e], kLog2eLo, off_d)));
            }
            const uint4 w = philox4x32_10(make_uint4((uint32_t)g, (uint32_t)b, step.lo, c3), p.seed_lo, p.seed_hi);
            const uint32_t word[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (r[e] > 0.0f && v + e != exclude_id) {
                    const float ex = race_exponential(word[e]);
                    const float score = r[e] * __builtin_amdgcn_rcpf(ex);  // ex == 0 -> +inf
                    if (score > best_score) {  // ids rise within a thread: strict > keeps the lowest
                        best_score = score;
                        best_id = v + e;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        const float os = __shfl_xor(best_score, o);
        const int oi = __shfl_xor(best_id, o);
        if (os > best_score || (os == best_score && oi < best_id)) { best_score = os; best_id = oi; }
    }
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    __syncthreads();
    if (lane == 0) { sh.best_score[wave] = best_score; sh.best_id[wave] = best_id; }
    __syncthreads();
    win_score = sh.best_score[0];
    win_id = sh.best_id[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
        const float os = sh.best_score[w];
        const int oi = sh.best_id[w];
        if (os > win_score || (os == win_score && oi < win_id)) { win_score = os; win_id = oi; }
    }
    __syncthreads();
}

// Bounded wait until `ready` holds for every thread of the block (block-wide AND).
// `probe` re-evaluates the condition; returns false if the limit ran out.
template <typename F>
__device__ __forceinline__ bool wait_all(const RejectParams &p, F probe)
{
    for (int spin = 0; spin < p.spin_limit; ++spin) {
        if (__syncthreads_and(probe() ? 1 : 0)) return true;
        // In a small launch the data is a poll or two away and a long nap would be most of the wait:
        // short naps first.  In a large one many blocks wait at once and their polls compete with the
        // streams (short naps there: the 7B- and 70B-shaped steps 0.5 to 0.8% slower).
        if (p.short_naps && spin < 4) __builtin_amdgcn_s_sleep(2);
        else if (p.short_naps && spin < 8) __builtin_amdgcn_s_sleep(8);
        else __builtin_amdgcn_s_sleep(32);
    }
    return false;
}

// Accept chain of request b from the published row statistics.  Cheap (a few
// hundred loads and fp64 operations), so every block that needs its result just
// recomputes it.  Waits (bounded) until all of the request's statistics carry this
// call's tag.  Leaves log2-sum-exp per row in sh.lse2, m in sh.m, the near-tie count
// in sh.near.  Returns false if the statistics never arrived.
__device__ __forceinline__ bool accept_phase(const RejectParams &p, int b, RejectShared &sh, bool write_debug, int npos = -1)
{
    const int tid = threadIdx.x;
    const int row_t0 = uniform_load(p.cu_q_len, b);
    const int k = uniform_load(p.cu_q_len, b + 1) - row_t0 - 1;
    const int row_d0 = row_t0 - b;
    const bool has_draft_rows = p.mode == SPEC_ACCEPT_SAMPLE;
    const int nrows = has_draft_rows ? 2 * k + 1 : k + 1;
    const int nstat = nrows * p.stat_segments;
    // npos >= 0: only the first npos positions (their target and draft rows) are looked at, and
    // sh.m counts the leading accepts among them
    const int npos_eval = npos < 0 ? k : npos;

    // the draft tokens' logits do not depend on the statistics: fetch them first
    // (a token outside the vocabulary is never used as an index: it has probability 0 under the
    // target, so its test rejects; the final stage counts it among the input errors)
    float tx = -INFINITY, dx = 0.0f;
    if (tid < npos_eval) {
        const int x = p.draft_tokens[row_d0 + tid];
        if ((unsigned)x < (unsigned)p.V) {
            tx = p.target_logits[(size_t)(row_t0 + tid) * p.V + x];
            if (has_draft_rows) dx = p.draft_logits[(size_t)(row_d0 + tid) * p.V + x];
        }
    }

    // poll and fetch in one: every word carries its own tag
    const bool ok = wait_all(p, [&] {
        bool mine = true;
        for (int i = tid; i < nstat; i += kThreads) {
            const int ri = i / p.stat_segments;
            const int sg = i - ri * p.stat_segments;
            if (npos >= 0 && (ri <= k ? ri : ri - k - 1) >= npos) continue;   // a row of a later position
            const int row = ri <= k ? row_t0 + ri : p.T + row_d0 + (ri - k - 1);
            const unsigned long long *st = p.stats + 3 * ((size_t)row * p.stat_segments + sg);
            const unsigned long long w0 = fetch_u64(st), w1 = fetch_u64(st + 1), w2 = fetch_u64(st + 2);
            mine = mine && tagged_ok(w0, p.generation) && tagged_ok(w1, p.generation) && tagged_ok(w2, p.generation);
            sh.seg_sum[ri][sg] = __longlong_as_double((long long)((w0 & 0xFFFFFFFFull) | (w1 << 32)));
            sh.seg_off[ri][sg] = __uint_as_float((uint32_t)w2);
        }
        return mine;
    });
    if (!ok) return false;
    if (tid < nrows && (npos < 0 || (tid <= k ? tid : tid - k - 1) < npos)) {
        float mx = kEmptyMax;
        for (int sg = 0; sg < p.stat_segments; ++sg) mx = fmaxf(mx, sh.seg_off[tid][sg]);
        double total = 0.0;
        for (int sg = 0; sg < p.stat_segments; ++sg)
            total += sh.seg_sum[tid][sg] * exp2((double)(sh.seg_off[tid][sg] - mx));   // exact power of two
        sh.lse2[tid] = (double)mx + log2(total);
    }
    __syncthreads();

    // accept tests, all evaluated in parallel; the chain is resolved below
    if (tid < npos_eval) {
        const double log2_p = (double)tx * kLog2eD - sh.lse2[tid];
        const double log2_q = has_draft_rows ? (double)dx * kLog2eD - sh.lse2[k + 1 + tid] : 0.0;   // point mass: q(x) = 1
        const double ratio = exp2(log2_p - log2_q);  // p = 0 -> 0, q = 0 < p -> inf, both 0 -> NaN (rejects)
        const StepWords step = philox_step_words(p);
        const uint4 w = philox4x32_10(make_uint4((uint32_t)tid, (uint32_t)b, step.lo, (step.hi24 << 8) | 0u),
                                      p.seed_lo, p.seed_hi);
        const double u = (double)(w.x >> 8) * (1.0 / 16777216.0);
        sh.u[tid] = u;
        sh.ratio[tid] = ratio;
        sh.accept[tid] = (u < ratio) ? 1 : 0;
    }
    __syncthreads();
    if (tid == 0) {
        int m = 0;
        while (m < npos_eval && sh.accept[m]) ++m;
        int near = 0;
        const int evaluated = m + 1 < npos_eval ? m + 1 : npos_eval;
        for (int i = 0; i < evaluated; ++i)
            if (fabs(sh.u[i] - sh.ratio[i]) < 1e-6) ++near;
        sh.m = m;
        sh.near = near;
    }
    __syncthreads();
    if (write_debug && p.debug_u_ratio != nullptr && tid < k) {
        const bool evaluated = tid <= sh.m;
        p.debug_u_ratio[2 * (size_t)(row_d0 + tid) + 0] = evaluated ? sh.u[tid] : (double)NAN;
        p.debug_u_ratio[2 * (size_t)(row_d0 + tid) + 1] = evaluated ? sh.ratio[tid] : (double)NAN;
    }
    return true;
}

// Greedy mode: how many of the first npos draft tokens of request b equal their row's arg-max
// (a leading run), from the arg-max records of the target rows 0 .. npos-1.  Waits (bounded)
// for those records; the result is left in sh.m.  Returns false if they never arrived.
__device__ __forceinline__ bool greedy_prefix(const RejectParams &p, int b, int npos, RejectShared &sh)
{
    const int tid = threadIdx.x;
    const int row_t0 = uniform_load(p.cu_q_len, b);
    const int row_d0 = row_t0 - b;
    const int nstat = npos * p.stat_segments;
    const bool ok = wait_all(p, [&] {
        bool mine = true;
        for (int i = tid; i < nstat; i += kThreads) {
            const int ri = i / p.stat_segments;
            const int sg = i - ri * p.stat_segments;
            const unsigned long long *st = p.stats + 3 * ((size_t)(row_t0 + ri) * p.stat_segments + sg);
            const unsigned long long w0 = fetch_u64(st), w1 = fetch_u64(st + 1);
            mine = mine && tagged_ok(w0, p.generation) && tagged_ok(w1, p.generation);
            sh.seg_off[ri][sg] = __uint_as_float((uint32_t)w0);
            sh.seg_sum[ri][sg] = (double)(uint32_t)w1;   // the id, exactly
        }
        return mine;
    });
    if (!ok) return false;
    if (tid < npos) {
        float best = -INFINITY;
        int best_id = 0x7FFFFFFF;
        for (int sg = 0; sg < p.stat_segments; ++sg) {
            const float v = sh.seg_off[tid][sg];
            const int id = (int)sh.seg_sum[tid][sg];
            if (v > best || (v == best && id < best_id)) { best = v; best_id = id; }
        }
        sh.accept[tid] = p.draft_tokens[row_d0 + tid] == (best_id == 0x7FFFFFFF ? 0 : best_id) ? 1 : 0;
    }
    __syncthreads();
    if (tid == 0) {
        int m = 0;
        while (m < npos && sh.accept[m]) ++m;
        sh.m = m;
    }
    __syncthreads();
    return true;
}

// Statistics items are ordered by request (its target rows, then its draft rows), so that
// the first requests' statistics are complete early and their races can start while
// later requests' rows are still being read.
template <int UNROLL>
__device__ __forceinline__ void stats_role(const RejectParams &p, int item, RejectShared &sh)
{
    const int rec = item / p.stat_segments;          // (request, row of the request)
    const int seg = item - rec * p.stat_segments;
    if (p.early_stop) {
        // Position order (every request has uniform_k draft tokens): the target and draft rows (the
        // target rows, if the draft is a point mass) of position 0 of all requests, then those of
        // position 1, ..., then the bonus rows.  The rows
        // of a position are only needed if the request's earlier positions were all accepted; by
        // the time a block of position j starts, the statistics of positions < j were dispatched
        // long before (two items per request and position), so the check costs a round trip, not a
        // wait.  A row that is not needed gets a placeholder record, so that later stages, which
        // poll all of a request's records and use those up to the first rejection, find it.
        const int k = p.uniform_k;
        const bool has_draft_rows = p.mode == SPEC_ACCEPT_SAMPLE;
        const int per_position = has_draft_rows ? 2 * p.B : p.B;
        int j, b;
        bool is_draft = false;
        if (rec < per_position * k) {
            j = rec / per_position;
            const int w = rec - j * per_position;
            b = has_draft_rows ? w >> 1 : w;
            is_draft = has_draft_rows && (w & 1) != 0;
        } else {
            j = k;
            b = rec - per_position * k;
        }
        const int row_t0 = b * (k + 1);
        const int row = is_draft ? p.T + (row_t0 - b) + j : row_t0 + j;
        const bool greedy = p.mode == SPEC_ACCEPT_GREEDY;
        if (j > 0 && (greedy ? greedy_prefix(p, b, j, sh) : accept_phase(p, b, sh, false, j)) && sh.m < j) {
            if (threadIdx.x == 0) {
                unsigned long long *dst = p.stats + 3 * ((size_t)row * p.stat_segments + seg);
                if (greedy) {   // (largest logit, id) of nothing
                    publish_tagged(dst + 0, __float_as_uint(-INFINITY), p.generation);
                    publish_tagged(dst + 1, 0x7FFFFFFFu, p.generation);
                } else {        // sum 1, offset 0
                    const unsigned long long bits = (unsigned long long)__double_as_longlong(1.0);
                    publish_tagged(dst + 0, (uint32_t)bits, p.generation);
                    publish_tagged(dst + 1, (uint32_t)(bits >> 32), p.generation);
                    publish_tagged(dst + 2, __float_as_uint(0.0f), p.generation);
                }
            }
            return;
        }
        if (greedy) argmax_block(p, row, seg, sh);
        else stats_block<UNROLL>(p, row, seg, sh);
        return;
    }
    if (p.mode != SPEC_ACCEPT_SAMPLE) {   // target rows only: rec is the row
        if (p.mode == SPEC_ACCEPT_GREEDY) argmax_block(p, rec, seg, sh);
        else stats_block<UNROLL>(p, rec, seg, sh);
        return;
    }
    // largest b with 2 * cu_q_len[b] - b <= rec (rows of the requests before b).  Start from
    // where b would be if all requests had equally many rows, and walk: with equal draft
    // lengths that is one round of loads instead of the log2(B) dependent ones of a bisection.
    const int nrec = 2 * p.T - p.B;
    int lo = (int)(((long long)rec * p.B) / nrec);
    if (lo > p.B - 1) lo = p.B - 1;
    while (lo > 0 && 2 * uniform_load(p.cu_q_len, lo) - lo > rec) --lo;
    while (lo < p.B - 1 && 2 * uniform_load(p.cu_q_len, lo + 1) - (lo + 1) <= rec) ++lo;
    const int b = lo;
    const int row_t0 = uniform_load(p.cu_q_len, b);
    const int k = uniform_load(p.cu_q_len, b + 1) - row_t0 - 1;
    const int ri = rec - (2 * row_t0 - b);
    const int row = ri <= k ? row_t0 + ri : p.T + (row_t0 - b) + (ri - k - 1);
    stats_block<UNROLL>(p, row, seg, sh);
}

// A request whose bounded wait ran out (never in a healthy launch): every output gets its
// sentinel and the request is counted in counters[7] only.
__device__ __forceinline__ void abandon_request(const RejectParams &p, int b)
{
    const int tid = threadIdx.x;
    if (p.out_tokens != nullptr && tid <= SPEC_K_MAX) p.out_tokens[(size_t)b * (SPEC_K_MAX + 1) + tid] = -1;
    if (tid != 0) return;
    p.accepted_len[b] = -1;
    p.next_token[b] = -1;
    if (p.new_kv_len != nullptr) p.new_kv_len[b] = -1;
    if (p.draft_next_len != nullptr) p.draft_next_len[b] = -1;
    atomicAdd(&p.counters[7], 1ull);
}

// Draft tokens of request b outside [0, V): counted among the input errors (counters[6]).
__device__ __forceinline__ void count_bad_draft_tokens(const RejectParams &p, int row_d0, int k)
{
    int bad = 0;
    for (int i = 0; i < k; ++i)
        if ((unsigned)p.draft_tokens[row_d0 + i] >= (unsigned)p.V) ++bad;
    if (bad) atomicAdd(&p.counters[6], (unsigned long long)bad);
}

// Offsets of the race rows of request b after accept_phase.
struct RaceRows {
    const float *trow, *drow;
    float off_t, corr_t, off_d, corr_d;
    int m, k, row_d0;
    int exclude;   // point-mass draft: the rejected token takes no part in the race
};

__device__ __forceinline__ RaceRows race_rows(const RejectParams &p, int b, const RejectShared &sh)
{
    RaceRows rr;
    const int row_t0 = uniform_load(p.cu_q_len, b);
    rr.k = uniform_load(p.cu_q_len, b + 1) - row_t0 - 1;
    rr.row_d0 = row_t0 - b;
    rr.m = sh.m;
    const double off_t_exact = -sh.lse2[rr.m];
    rr.off_t = (float)off_t_exact;
    rr.corr_t = (float)exp2(off_t_exact - (double)rr.off_t);
    rr.off_d = 0.0f;
    rr.corr_d = 0.0f;
    rr.trow = p.target_logits + (size_t)(row_t0 + rr.m) * p.V;
    rr.drow = nullptr;
    rr.exclude = -1;
    if (rr.m < rr.k && p.mode == SPEC_ACCEPT_POINT_DRAFT) rr.exclude = p.draft_tokens[rr.row_d0 + rr.m];
    if (rr.m < rr.k && p.mode == SPEC_ACCEPT_SAMPLE) {
        const double off_d_exact = -sh.lse2[rr.k + 1 + rr.m];
        rr.off_d = (float)off_d_exact;
        rr.corr_d = (float)exp2(off_d_exact - (double)rr.off_d);
        rr.drow = p.draft_logits + (size_t)(rr.row_d0 + rr.m) * p.V;
    }
    return rr;
}

// One (request, vocabulary segment) of the race.  Race items follow all statistics
// items in the grid, so the statistics blocks they wait for (inside accept_phase, with
// a bound) were scheduled before them and never wait themselves: the wait ends.
// Should the bound ever run out, the block publishes nothing and the request's final stage,
// whose own wait then runs out too, abandons the request.
__device__ __forceinline__ void race_role(const RejectParams &p, int item, RejectShared &sh)
{
    const int tid = threadIdx.x;
    const int b = item / p.race_segments;
    const int seg = item - b * p.race_segments;
    if (!accept_phase(p, b, sh, seg == 0)) return;
    const RaceRows rr = race_rows(p, b, sh);
    const int v0 = seg * p.race_seg_len;
    const int v1 = min(p.V, v0 + p.race_seg_len);
    float win_score;
    int win_id;
    race_segment(p, rr.trow, rr.drow, rr.exclude, b, v0, v1, rr.off_t, rr.corr_t, rr.off_d, rr.corr_d, sh, win_score,
                 win_id);
    if (tid == 0) {
        unsigned long long *dst = p.race_partial + 2 * ((size_t)b * p.race_segments + seg);
        publish_tagged(dst + 0, __float_as_uint(win_score), p.generation);
        publish_tagged(dst + 1, (uint32_t)win_id, p.generation);
        if (seg == 0)   // the accept chain's result, for the final stage
            publish_tagged(p.race_info + b, (uint32_t)rr.m | ((uint32_t)rr.k << 8) | ((uint32_t)sh.near << 16),
                           p.generation);
    }
}

// Greedy mode, last stage of request b (there is no race): waits (bounded) for the
// arg-max records of the request's k+1 target rows, accepts the leading run of draft
// tokens that equal their row's arg-max, and emits the arg-max of the row after it.
__device__ __forceinline__ void greedy_final(const RejectParams &p, int b, RejectShared &sh)
{
    const int tid = threadIdx.x;
    const int row_t0 = uniform_load(p.cu_q_len, b);
    const int k = uniform_load(p.cu_q_len, b + 1) - row_t0 - 1;
    const int row_d0 = row_t0 - b;
    const int nstat = (k + 1) * p.stat_segments;
    const bool ok = wait_all(p, [&] {
        bool mine = true;
        for (int i = tid; i < nstat; i += kThreads) {
            const int ri = i / p.stat_segments;
            const int sg = i - ri * p.stat_segments;
            const unsigned long long *st = p.stats + 3 * ((size_t)(row_t0 + ri) * p.stat_segments + sg);
            const unsigned long long w0 = fetch_u64(st), w1 = fetch_u64(st + 1);
            mine = mine && tagged_ok(w0, p.generation) && tagged_ok(w1, p.generation);
            sh.seg_off[ri][sg] = __uint_as_float((uint32_t)w0);
            sh.seg_sum[ri][sg] = (double)(uint32_t)w1;   // the id, exactly
        }
        return mine;
    });
    if (!ok) {
        abandon_request(p, b);
        return;
    }
    if (tid <= k) {
        float best = -INFINITY;
        int best_id = 0x7FFFFFFF;
        for (int sg = 0; sg < p.stat_segments; ++sg) {   // segments in rising id order: > keeps the lowest id
            const float v = sh.seg_off[tid][sg];
            const int id = (int)sh.seg_sum[tid][sg];
            if (v > best || (v == best && id < best_id)) { best = v; best_id = id; }
        }
        sh.lse2[tid] = (double)(best_id == 0x7FFFFFFF ? 0 : best_id);
    }
    __syncthreads();
    if (tid == 0) {
        int m = 0;
        while (m < k && p.draft_tokens[row_d0 + m] == (int)sh.lse2[m]) ++m;
        const int next = (int)sh.lse2[m];
        p.accepted_len[b] = m;
        p.next_token[b] = next;
        if (p.new_kv_len != nullptr) p.new_kv_len[b] = p.kv_len[b] - (k - m);
        if (p.draft_next_len != nullptr) p.draft_next_len[b] = (k > 0 && m == k) ? 2 : 1;
        if (p.out_tokens != nullptr) {
            int32_t *row = p.out_tokens + (size_t)b * (SPEC_K_MAX + 1);
            for (int i = 0; i <= SPEC_K_MAX; ++i)
                row[i] = i < m ? p.draft_tokens[row_d0 + i] : (i == m ? next : -1);
        }
        atomicAdd(&p.counters[0], (unsigned long long)k);
        atomicAdd(&p.counters[1], (unsigned long long)m);
        atomicAdd(&p.counters[2], (unsigned long long)(m + 1 < k ? m + 1 : k));
        atomicAdd(&p.counters[3], (unsigned long long)(m + 1));
        atomicAdd(&p.counters[5], 1ull);
        count_bad_draft_tokens(p, row_d0, k);
    }
    // clear this request's tags
    for (int i = tid; i < 2 * nstat; i += kThreads) {
        const int rec = i >> 1;
        publish_u64(p.stats + 3 * ((size_t)row_t0 * p.stat_segments + rec) + (i & 1), 0ull);
    }
}

// Last stage of request b (one item per request, after all race items):
// waits (bounded) for the request's race segments, picks the winner, writes the
// outputs and counters, and clears the request's tags so that a replay of the
// same launch (HIP graph) starts clean.
__device__ __forceinline__ void final_role(const RejectParams &p, int b, RejectShared &sh)
{
    if (p.mode == SPEC_ACCEPT_GREEDY) {
        greedy_final(p, b, sh);
        return;
    }
    const int tid = threadIdx.x;
    unsigned long long *part = p.race_partial + 2 * (size_t)b * p.race_segments;
    // poll and fetch in one: the race partials (race_segments <= 64: wavefront 0 holds
    // them all) and the accept chain's result
    float best_score = -1.0f;
    int best_id = 0x7FFFFFFF;
    uint32_t info = 0;
    const bool ok = wait_all(p, [&] {
        bool mine = true;
        if (tid < p.race_segments) {
            const unsigned long long w0 = fetch_u64(part + 2 * tid), w1 = fetch_u64(part + 2 * tid + 1);
            mine = tagged_ok(w0, p.generation) && tagged_ok(w1, p.generation);
            best_score = __uint_as_float((uint32_t)w0);
            best_id = (int)(uint32_t)w1;
        }
        if (tid == 0) {
            const unsigned long long wi = fetch_u64(p.race_info + b);
            mine = mine && tagged_ok(wi, p.generation);
            info = (uint32_t)wi;
        }
        return mine;
    });
    if (!ok) {
        abandon_request(p, b);
        return;
    }
    if (tid == 0) sh.m = (int)info;
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        const float os = __shfl_xor(best_score, o);
        const int oi = __shfl_xor(best_id, o);
        if (os > best_score || (os == best_score && oi < best_id)) { best_score = os; best_id = oi; }
    }
    if (tid == 0) { sh.best_score[0] = best_score; sh.best_id[0] = best_id; }
    __syncthreads();
    float win_score = sh.best_score[0];
    int win_id = sh.best_id[0];
    info = (uint32_t)sh.m;
    __syncthreads();
    const int m = (int)(info & 0xFFu), k = (int)((info >> 8) & 0xFFu), near = (int)(info >> 16);
    const int row_t0 = uniform_load(p.cu_q_len, b);
    const int row_d0 = row_t0 - b;
    if (!(win_score > 0.0f)) {
        // p - q has no positive entry (p == q to rounding): draw from p instead
        if (!accept_phase(p, b, sh, false)) {
            abandon_request(p, b);
            return;
        }
        const RaceRows rr = race_rows(p, b, sh);
        race_segment(p, rr.trow, nullptr, -1, b, 0, p.V, rr.off_t, rr.corr_t, 0.0f, 0.0f, sh, win_score, win_id);
    }
    if (tid == 0) {
        p.accepted_len[b] = m;
        p.next_token[b] = win_id;
        if (p.new_kv_len != nullptr) p.new_kv_len[b] = p.kv_len[b] - (k - m);
        if (p.draft_next_len != nullptr) p.draft_next_len[b] = (k > 0 && m == k) ? 2 : 1;
        if (p.out_tokens != nullptr) {
            int32_t *row = p.out_tokens + (size_t)b * (SPEC_K_MAX + 1);
            for (int i = 0; i <= SPEC_K_MAX; ++i)
                row[i] = i < m ? p.draft_tokens[row_d0 + i] : (i == m ? win_id : -1);
        }
        atomicAdd(&p.counters[0], (unsigned long long)k);
        atomicAdd(&p.counters[1], (unsigned long long)m);
        atomicAdd(&p.counters[2], (unsigned long long)(m + 1 < k ? m + 1 : k));
        atomicAdd(&p.counters[3], (unsigned long long)(m + 1));
        atomicAdd(&p.counters[4], (unsigned long long)near);
        atomicAdd(&p.counters[5], 1ull);
        count_bad_draft_tokens(p, row_d0, k);
    }
    // clear this request's tags
    const int nstat = (p.mode == SPEC_ACCEPT_SAMPLE ? 2 * k + 1 : k + 1) * p.stat_segments;
    for (int i = tid; i < 3 * nstat; i += kThreads) {
        const int rec = i / 3;
        const int ri = rec / p.stat_segments;
        const int sg = rec - ri * p.stat_segments;
        const int row = ri <= k ? row_t0 + ri : p.T + row_d0 + (ri - k - 1);
        publish_u64(p.stats + 3 * ((size_t)row * p.stat_segments + sg) + (i - 3 * rec), 0ull);
    }
    if (tid < 2 * p.race_segments) publish_u64(part + tid, 0ull);
    if (tid == 0) publish_u64(p.race_info + b, 0ull);
}

// ===========================================================================
// Attention half
// ===========================================================================
template <int D>
struct PageRegs {
    u32x4 k[D / 32];  // k[kk]: token n, dims 32*kk + 8g .. +7
    u32x4 v[D / 32];  // v[pp]: dims 32*pp + n (low half) and 32*pp + 16 + n (high half), tokens 4g .. 4g+3
};

// The query rows and the output tile pass through LDS so that global memory sees them as
// whole rows (full cache lines, each once per block) instead of the 64-byte pieces of the
// matrix-operand layout, once per wavefront: with 32 to 48 query rows per KV head (grouped
// heads) these requests were a fifth of all the block's memory requests, and the launch is
// bound by requests as much as by bytes.  Rows are padded against bank conflicts.
constexpr int q_stride(int D) { return D * 2 + 16; }   // bytes per bf16 query row in LDS
constexpr int o_stride(int D) { return D * 4 + 16; }   // bytes per fp32 output row in LDS

// Wave groups.  A block's four wavefronts form WG groups of PW = 4 / WG wavefronts.  Each group
// owns NT 16-row tiles of the query rows of one (request, KV head) and walks ALL pages of the
// block's chunk, its PW wavefronts taking them in turn.  WG = 1 is the common case (up to 48
// fused rows).  With more rows per KV head (long drafts on wide query groups: up to 9 x 16 = 144
// rows) the groups of one block read the same pages at the same time, so the pages cross the
// memory interface once and the groups find each other's loads in the compute unit's cache or
// in flight.
// Token-major pages ([16 tokens][D dims] per page and KV head).  K is loaded straight into the
// matrix operand order from that layout too (a lane's 16 bytes are 8 consecutive dims of one
// token); V has to be transposed (the PV product wants, per lane, four consecutive tokens of one
// dim): each wavefront loads its V page as whole rows (coalesced 16-byte loads), stages it in a
// region of its own in LDS and reads it back two bytes at a time in operand order.  Token rows
// are padded by 16 bytes (272 at D = 128): the 16 lanes of a row group then read 8 banks, and the
// four row groups of a wavefront, 4 tokens apart, land 16 banks apart: no conflicts.
constexpr int vt_row_bytes(int D) { return D * 2 + 16; }
constexpr int vt_wave_bytes(int D) { return SPEC_BLOCK_SIZE * vt_row_bytes(D); }

template <int NT, int WG, bool TM = false, int D = kD>
struct AttnShared {
    static constexpr int kRowsMax = WG * NT * 16;
    union {
        f32x4 acc[2][NT][D / 16][kWave];          // epilogue: partial results of the wavefronts being merged
        unsigned char q[kRowsMax * q_stride(D)];  // prologue: the block's query rows
        unsigned char o[WG == 1 ? NT * 16 * o_stride(D) : 16];   // epilogue of an unsplit request (one group): the output tile
    };
    float m[2][NT][kWave];
    float l[2][NT][kWave];
    int last;
    alignas(16) unsigned char vt[TM ? kWaves * vt_wave_bytes(D) : 16];   // token-major pages: V staged per wavefront
};

// The order in which the attention items take the requests (longest first), as the kernel
// sees it: a pointer into the kernel-argument segment, read with scalar loads (taking the
// address of the by-value argument instead would make the compiler copy the table to
// private memory).  Two 16-bit entries per word; n == 0: the given order.
typedef const uint32_t __attribute__((address_space(4))) *uniform_u32_ptr;
struct OrderTable {
    int n;
    uniform_u32_ptr pairs;
};

// VAR: 0 = pages in the matrix-operand layout, softmax weights fed as bf16 high + low parts;
//      1 = the same with the weights as one bf16 (an experiment switch);
//      2 = token-major pages (V transposed through LDS), weights as high + low parts;
//      3 = as 0 with a head dim of 64, 4 = as 2 with a head dim of 64 (all others: 128).
constexpr int head_dim_of(int VAR) { return (VAR == 3 || VAR == 4) ? 64 : kD; }
constexpr bool token_major_of(int VAR) { return VAR == 2 || VAR == 4; }

template <int NT, int WG, int VAR>
__device__ __forceinline__ void attn_role(const AttnParams &p, OrderTable order, int item,
                                          AttnShared<NT, WG, token_major_of(VAR), head_dim_of(VAR)> &sh)
{
    constexpr bool SPLIT_P = VAR != 1;
    constexpr bool TM = token_major_of(VAR);
    constexpr int D = head_dim_of(VAR);
    constexpr int KK = D / 32;                        // 32-dim steps of the score product = 1 KB loads per K or V page
    constexpr int MT = D / 16;                        // 16-dim slices of the output
    constexpr int kQStride = q_stride(D), kOStride = o_stride(D);
    constexpr int kPageHeadBytes = SPEC_BLOCK_SIZE * D * 2;   // one (page, KV head) of K or of V: 4096 at D = 128
    constexpr int QP = D / 8;                         // 16-byte pieces of a bf16 query row
    constexpr int QI = (NT * WG * 16 * QP + kThreads - 1) / kThreads;   // ... of all the block's rows, per thread
    constexpr int kVtRowBytes = vt_row_bytes(D), kVtWaveBytes = vt_wave_bytes(D);
    constexpr int PW = kWaves / WG;   // wavefronts that share the pages of a group between them
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave / PW;        // this wavefront's row group
    const int pw = wave % PW;         // ... and its place in the page walk of the group
    const int lane = tid & 63;
    const int n16 = lane & 15;
    const int g = lane >> 4;
    // Items are chunk-major: all first chunks (requests longest first, KV heads innermost),
    // then all second chunks, ...  Consecutive blocks go to different XCDs, so every XCD
    // gets the same mix of chunk indices; the chunk indices that only the longest requests
    // have come last (blocks of the others for these indices exit at once), instead of
    // always falling on the same XCDs.
    // With split requests a row of items (one chunk index) is padded to whole rows of kXcds blocks, so
    // that all chunks of a (request, KV head) run on one XCD and find its query rows, table entries,
    // partial results and ticket in that XCD's L2 (spread over the XCDs the ragged long-context
    // workload takes 4% longer).
    const int n_units = p.B * p.Hkv;
    const int row_items = attn_row_items(p);
    const int chunk = item / row_items;
    const int place = item - chunk * row_items;
    if (place >= n_units) return;   // padding
    const int kvh = place % p.Hkv;
    int b = place / p.Hkv;   // rank in the order of the attention items
    if (order.n > 0) {
        const uint32_t pair = order.pairs[b >> 1];
        b = (int)((b & 1) ? pair >> 16 : pair & 0xFFFFu);
    }
    const int unit = b * p.Hkv + kvh;

    // When no request is split, a wavefront's block-table entries do not depend on kv_len:
    // fetch them alongside it (entries past the request's pages are never used).
    int bt = 0;
    if (p.max_chunks == 1 && pw + PW * lane < p.max_blocks_per_req)
        bt = p.block_table[(size_t)b * p.max_blocks_per_req + pw + PW * lane];
    const int L = uniform_load(p.kv_len, b);
    const int row0 = uniform_load(p.cu_q_len, b);
    const int q_len = uniform_load(p.cu_q_len, b + 1) - row0;
    // The lengths come from device memory and bound every loop and index below: a request
    // whose lengths do not fit the launch (longer than planned for, beyond its block-table row,
    // shorter than its own query rows) is left out and reported.
    if (!request_lengths_ok(L, q_len, p.capacity_tokens, p.max_blocks_per_req)) {
        if (chunk == 0 && kvh == 0 && tid == 0 && p.errors != nullptr) atomicAdd(p.errors, 1ull);
        return;
    }
    const int nchunks = (L + p.chunk_tokens - 1) / p.chunk_tokens;   // <= max_chunks, since L <= capacity_tokens
    if (chunk >= nchunks) return;
    // even chunks per request, page aligned (never longer than chunk_tokens)
    const int C = ((L + nchunks - 1) / nchunks + SPEC_BLOCK_SIZE - 1) & ~(SPEC_BLOCK_SIZE - 1);
    const int group = p.Hq / p.Hkv;
    // (the plan sized WG and NT for the longest draft of the host copy of cu_q_len; should the device
    // copy disagree, the rows beyond that are left out rather than staged out of bounds)
    const int rows = min(q_len * group, WG * NT * 16);
    const int row_lo = grp * (NT * 16);          // first row of this wavefront's group
    const int grp_rows = min(max(rows - row_lo, 0), NT * 16);
    const int tok0 = chunk * C;
    const int tok1 = min(L, tok0 + C);
    const int npages = (tok1 - tok0 + SPEC_BLOCK_SIZE - 1) / SPEC_BLOCK_SIZE;  // <= 64 * PW
    const int page0 = tok0 / SPEC_BLOCK_SIZE;

    // block-table entries of this wavefront's pages (pw, pw + PW, ...), one per lane
    if (p.max_chunks != 1 && pw + PW * lane < npages)
        bt = p.block_table[(size_t)b * p.max_blocks_per_req + page0 + pw + PW * lane];
    {
        // an entry outside the pool is never turned into an address: the page reads as zeros
        const bool bad = pw + PW * lane < npages && (unsigned)bt >= (unsigned)p.num_blocks;
        if (bad) bt = -1;
        const unsigned long long bad_lanes = __builtin_amdgcn_ballot_w64(bad);
        if (bad_lanes != 0 && kvh == 0 && grp == 0 && p.errors != nullptr && lane == 0)
            atomicAdd(p.errors, (unsigned long long)__builtin_popcountll(bad_lanes));
    }

    // Q: the block fetches its query rows once, 16 bytes per thread and consecutive threads
    // along a row (the heads of a group are adjacent in memory), and leaves them in LDS
    u32x4 qpiece[QI];
#pragma unroll
    for (int i = 0; i < QI; ++i) {
        const int piece = tid + i * kThreads;   // QP pieces per row
        const int r = piece / QP, c = piece % QP;
        qpiece[i] = (u32x4){0u, 0u, 0u, 0u};
        if (r < rows) {
            const size_t rh = (size_t)(row0 + r / group) * p.Hq + kvh * group + r % group;
            qpiece[i] = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(p.q) + rh * (D * 2) + c * 16);
        }
    }
    bf16x8 qreg[NT][KK];   // filled from LDS below
    int limit[NT];     // each lane's last visible key
    int out_row[NT];   // packed (token row * Hq + head) of this lane's query row, -1 if padding
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int r = row_lo + nt * 16 + n16;
        const bool valid = r < rows;
        const int j = valid ? r / group : 0;
        const int gq = valid ? r % group : 0;
        limit[nt] = valid ? L - q_len + j : -1;
        out_row[nt] = valid ? (int)((size_t)(row0 + j) * p.Hq + kvh * group + gq) : -1;
    }

    // Pages are read with buffer loads through a descriptor that covers exactly one
    // (page, KV head): 4 KB of K or V.  A page index past the end gets a descriptor of
    // length 0, for which the hardware returns zeros without touching memory.  That
    // keeps every load unconditional, so the loads of later pages stay in flight across
    // the arithmetic of the current one (a branch around them would make the compiler
    // wait for all outstanding loads at every use).
    const char *khead = static_cast<const char *>(p.k_cache) + (size_t)kvh * kPageHeadBytes;
    const char *vhead = static_cast<const char *>(p.v_cache) + (size_t)kvh * kPageHeadBytes;
    const size_t page_stride = (size_t)p.Hkv * kPageHeadBytes;
    // pages pw, pw + PW, ... (none for a group that has no rows of this request)
    const int my_pages = (npages > pw && grp_rows > 0) ? (npages - pw + PW - 1) / PW : 0;
    const int lane_off = lane * 16;

    auto load_page = [&](int it, PageRegs<D> &r) {   // it-th page of this wavefront
        const int entry = __builtin_amdgcn_readlane(bt, it < my_pages ? it : 0);
        const bool valid = it < my_pages && entry >= 0;
        const int page = valid ? entry : 0;
        const int bytes = valid ? kPageHeadBytes : 0;
        const __amdgpu_buffer_rsrc_t kd = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char *>(khead + (size_t)page * page_stride), 0, bytes, kBufferFlags);
        const __amdgpu_buffer_rsrc_t vd = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char *>(vhead + (size_t)page * page_stride), 0, bytes, kBufferFlags);
        if constexpr (TM) {
            // K: token n16, dims 32 i + 8 g .. + 7 sit at n16 * 2 D + 64 i + 16 g
#pragma unroll
            for (int i = 0; i < KK; ++i)
                r.k[i] = __builtin_amdgcn_raw_buffer_load_b128(kd, n16 * (D * 2) + g * 16, i * 64, kStreamPolicy);
        } else {
#pragma unroll
            for (int i = 0; i < KK; ++i) r.k[i] = __builtin_amdgcn_raw_buffer_load_b128(kd, lane_off, i * 1024, kStreamPolicy);
        }
        // V: in operand order already, or (token-major) as whole rows: with D / 8 lanes per row, lane L of load i holds
        // token (512 / D) i + 8 L / D, dims 8 (L % (D / 8)) .. + 7
#pragma unroll
        for (int i = 0; i < KK; ++i) r.v[i] = __builtin_amdgcn_raw_buffer_load_b128(vd, lane_off, i * 1024, kStreamPolicy);
    };

    f32x4 acc[NT][MT];
    float m_run[NT], l_run[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m_run[nt] = kEmptyMax;
        l_run[nt] = 0.0f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = (f32x4){0.0f, 0.0f, 0.0f, 0.0f};
    }

    const int first_masked_token = L - q_len + 1;  // keys from here on are hidden from some row (or past the end)

    // Software pipeline: the loads of the next DEPTH pages are in flight while a page is
    // consumed.  The ring is indexed statically (the loop is unrolled by its length).
    auto consume = [&](PageRegs<D> &cur, int pi) {
        const int page_tok = tok0 + pi * SPEC_BLOCK_SIZE;
        const bool need_mask = page_tok + SPEC_BLOCK_SIZE > first_masked_token;
        const int tbase = page_tok + 4 * g;

        if constexpr (TM) {
            // V through this wavefront's LDS region: rows in, operand order out (LDS executes a
            // wavefront's accesses in order, so the reads see the writes without a barrier)
            unsigned char *vl = sh.vt + wave * kVtWaveBytes;
            constexpr int LR = D / 8;   // lanes per token row of a 1 KB load (16 bytes each)
#pragma unroll
            for (int i = 0; i < KK; ++i)
                *reinterpret_cast<u32x4 *>(vl + ((kWave / LR) * i + lane / LR) * kVtRowBytes + (lane % LR) * 16) = cur.v[i];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const unsigned char *src = vl + (4 * g) * kVtRowBytes + n16 * 2;
#pragma unroll
            for (int pp = 0; pp < KK; ++pp) {
                uint32_t w[4];
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    const unsigned char *e = src + (32 * pp + 16 * hf) * 2;
                    const uint32_t t0 = *reinterpret_cast<const uint16_t *>(e);
                    const uint32_t t1 = *reinterpret_cast<const uint16_t *>(e + kVtRowBytes);
                    const uint32_t t2 = *reinterpret_cast<const uint16_t *>(e + 2 * kVtRowBytes);
                    const uint32_t t3 = *reinterpret_cast<const uint16_t *>(e + 3 * kVtRowBytes);
                    w[2 * hf + 0] = t0 | (t1 << 16);
                    w[2 * hf + 1] = t2 | (t3 << 16);
                }
                cur.v[pp] = (u32x4){w[0], w[1], w[2], w[3]};
            }
        }

        if (page_tok + SPEC_BLOCK_SIZE > L) {
            // slots past kv_len in the request's last page may hold anything: clear their V
            // (the branch is the same for the whole wavefront and holds no loads)
            const int nvalid = min(max(L - tbase, 0), 4);
            const uint32_t lo = nvalid >= 2 ? 0xFFFFFFFFu : (nvalid == 1 ? 0x0000FFFFu : 0u);
            const uint32_t hi = nvalid >= 4 ? 0xFFFFFFFFu : (nvalid == 3 ? 0x0000FFFFu : 0u);
#pragma unroll
            for (int i = 0; i < KK; ++i) {
                cur.v[i].x &= lo; cur.v[i].y &= hi;
                cur.v[i].z &= lo; cur.v[i].w &= hi;
            }
        }

#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (nt > 0 && nt * 16 >= grp_rows) continue;   // a tile this request has no rows for (the same for the whole wavefront)
            f32x4 s = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, cur.k[kk]), qreg[nt][kk], s, 0, 0, 0);
            // (the softmax scale, folded with log2 e, is applied inside the exponent's fused
            // multiply-add below; the maximum commutes with it, the scale being positive)
            if (need_mask) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (tbase + r > limit[nt]) s[r] = -INFINITY;
            }
            float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
            mx = max_across_xor32(max_across_xor16(mx)) * p.scale_log2;
            // The reference of the running sums follows the maximum lazily: it is raised only when
            // a score exceeds it by more than 8 (base-2 units), so weights reach at most 2^8 and
            // the accumulators are rescaled on few pages instead of on most early ones (the
            // result is the same up to rounding: numerator and denominator share the reference).
            const float m_new = mx > m_run[nt] + kRescaleSlack ? mx : m_run[nt];
            f32x4 pr;
#pragma unroll
            for (int r = 0; r < 4; ++r) pr[r] = fast_exp2(fmaf(s[r], p.scale_log2, -m_new));
            if (__builtin_amdgcn_ballot_w64(m_new != m_run[nt]) != 0) {   // some row's reference moved: rescale
                const float alpha = fast_exp2(m_run[nt] - m_new);
                l_run[nt] *= alpha;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[nt][mt] *= alpha;
                m_run[nt] = m_new;
            }
            l_run[nt] += (pr[0] + pr[1]) + (pr[2] + pr[3]);
            const bf16x4 p_hi = __builtin_convertvector(pr, bf16x4);
            bf16x4 p_lo;
            if (SPLIT_P) p_lo = __builtin_convertvector(pr - __builtin_convertvector(p_hi, f32x4), bf16x4);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const u32x4 vv = cur.v[mt >> 1];
                const u32x2 half = (mt & 1) ? (u32x2){vv.z, vv.w} : (u32x2){vv.x, vv.y};
                const bf16x4 va = __builtin_bit_cast(bf16x4, half);
                acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, p_hi, acc[nt][mt], 0, 0, 0);
                if (SPLIT_P) acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, p_lo, acc[nt][mt], 0, 0, 0);
            }
        }
    };

    // Two register batches of P pages each.  While one batch is consumed the loads of the
    // other are in flight.  The order inside a half-step matters: first wait for the batch
    // about to be consumed (at that point it is the only one outstanding, so the full
    // wait the compiler emits waits for nothing else), then issue the other batch's loads,
    // then do the arithmetic, which needs no further wait.
    // pages per batch: two bring nothing once the launch keeps the memory system busy, except with the
    // half-size pages of a head dim of 64 (the same bytes in flight per wavefront as at 128)
    constexpr int P = D == 64 ? 2 : 1;
    PageRegs<D> batch_a[P], batch_b[P];
    auto load_batch = [&](int it, PageRegs<D>(&r)[P]) {
#pragma unroll
        for (int j = 0; j < P; ++j) load_page(it + j, r[j]);
    };
    auto arrived = [&](PageRegs<D>(&r)[P]) {
#pragma unroll
        for (int j = 0; j < P; ++j) {
            if constexpr (KK == 4)
                asm volatile("" ::"v"(r[j].k[0]), "v"(r[j].k[1]), "v"(r[j].k[2]), "v"(r[j].k[3]), "v"(r[j].v[0]),
                             "v"(r[j].v[1]), "v"(r[j].v[2]), "v"(r[j].v[3])
                             : "memory");
            else
                asm volatile("" ::"v"(r[j].k[0]), "v"(r[j].k[1]), "v"(r[j].v[0]), "v"(r[j].v[1]) : "memory");
        }
    };
    auto consume_batch = [&](PageRegs<D>(&r)[P], int it) {
#pragma unroll
        for (int j = 0; j < P; ++j)
            if (it + j < my_pages) consume(r[j], pw + PW * (it + j));
    };
    load_batch(0, batch_a);

    // Q as the B operand of S^T = K Q^T, out of LDS (the first pages are on their way)
#pragma unroll
    for (int i = 0; i < QI; ++i) {
        const int piece = tid + i * kThreads;
        if (QI * kThreads == NT * WG * 16 * QP || piece < NT * WG * 16 * QP)
            *reinterpret_cast<u32x4 *>(sh.q + (piece / QP) * kQStride + (piece % QP) * 16) = qpiece[i];
    }
    __syncthreads();
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            qreg[nt][kk] = *reinterpret_cast<const bf16x8 *>(sh.q + (row_lo + nt * 16 + n16) * kQStride + kk * 64 + g * 16);
    }
    __syncthreads();   // the epilogue reuses this memory

    for (int it0 = 0; it0 < my_pages; it0 += 2 * P) {
        arrived(batch_a);
        load_batch(it0 + P, batch_b);
        consume_batch(batch_a, it0);
        arrived(batch_b);
        load_batch(it0 + 2 * P, batch_a);
        consume_batch(batch_b, it0 + P);
    }

    // each lane summed its own four tokens per page: finish the row sums
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        l_run[nt] = sum_across_rows(l_run[nt]);
    }

    // merge the wavefronts of each group into the group's first one
    auto put = [&](int buf) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) sh.acc[buf][nt][mt][lane] = acc[nt][mt];
            sh.m[buf][nt][lane] = m_run[nt];
            sh.l[buf][nt][lane] = l_run[nt];
        }
    };
    auto merge = [&](int buf) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const float mo = sh.m[buf][nt][lane];
            const float lo = sh.l[buf][nt][lane];
            const float mn = fmaxf(m_run[nt], mo);
            const float wa = fast_exp2(m_run[nt] - mn);
            const float wb = fast_exp2(mo - mn);
            l_run[nt] = l_run[nt] * wa + lo * wb;
            m_run[nt] = mn;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = acc[nt][mt] * wa + sh.acc[buf][nt][mt][lane] * wb;
        }
    };
    if constexpr (WG == 1) {          // 2,3 -> 0,1 then 1 -> 0 (the last step below, by wavefront 0)
        if (wave >= 2) put(wave - 2);
        __syncthreads();
        if (wave < 2) merge(wave);
        __syncthreads();
        if (wave == 1) put(0);
        __syncthreads();
    } else if constexpr (WG == 2) {   // 1 -> 0 and 3 -> 2
        if (pw == 1) put(grp);
        __syncthreads();
        if (pw == 0) merge(grp);
        __syncthreads();
    }
    const bool lead = pw == 0 && grp_rows > 0;   // this wavefront holds its group's result

    if (nchunks == 1) {
        if constexpr (WG == 1) {
            // the only chunk of this (request, KV head): normalise, lay the tile out by rows in
            // LDS, and let the whole block write the rows (16 bytes per thread, consecutive
            // threads along a row)
            if (wave == 0) {
                merge(0);   // (its reads of the shared partials precede the writes below in program order)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const float inv = 1.0f / l_run[nt];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        *reinterpret_cast<f32x4 *>(sh.o + (nt * 16 + n16) * kOStride + mt * 64 + g * 16) = acc[nt][mt] * inv;
                }
            }
            __syncthreads();
            constexpr int OP = D / 4;   // 16-byte pieces of an fp32 output row
            for (int piece = tid; piece < rows * OP; piece += kThreads) {
                const int r = piece / OP, c = piece % OP;
                const size_t rh = (size_t)(row0 + r / group) * p.Hq + kvh * group + r % group;
                __builtin_nontemporal_store(*reinterpret_cast<const f32x4 *>(sh.o + r * kOStride + c * 16),
                                            reinterpret_cast<f32x4 *>(p.out + rh * D + c * 4));
            }
        } else if (lead) {
            // several groups: each group's first wavefront writes its rows itself (a lane holds four
            // consecutive head dims of one row per 16-dim slice)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                if (out_row[nt] < 0) continue;
                const float inv = 1.0f / l_run[nt];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    __builtin_nontemporal_store(acc[nt][mt] * inv,
                                                reinterpret_cast<f32x4 *>(p.out + (size_t)out_row[nt] * D + mt * 16 + 4 * g));
            }
        }
        return;
    }

    if (WG == 1 ? wave == 0 : lead) {
        if constexpr (WG == 1) merge(0);
        // one partial per query row: acc[dim], running max, running sum
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (out_row[nt] < 0) continue;
            const size_t slot = (size_t)out_row[nt] * p.max_chunks + chunk;
            unsigned long long *dst = reinterpret_cast<unsigned long long *>(p.ws_acc + slot * D + 4 * g);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                publish_u64(dst + 8 * mt + 0, pack_f32x2(acc[nt][mt][0], acc[nt][mt][1]));
                publish_u64(dst + 8 * mt + 1, pack_f32x2(acc[nt][mt][2], acc[nt][mt][3]));
            }
            if (g == 0)
                publish_u64(reinterpret_cast<unsigned long long *>(p.ws_ml + slot * 2), pack_f32x2(m_run[nt], l_run[nt]));
        }
        writes_complete();  // the partials are in memory before the ticket is taken
    }
    if (!p.fused_combine) return;   // a separate combine launch merges the partials
    if constexpr (WG > 1) __syncthreads();   // ... those of every group
    if (tid == 0) {
        unsigned long long *ticket = &p.tickets[unit];
        const uint32_t before = ticket_arrive(ticket, p.generation);
        const int last = (before + 1u == (uint32_t)nchunks) ? 1 : 0;
        if (last) ticket_reset(ticket);
        sh.last = last;
    }
    __syncthreads();
    if (!sh.last) return;
    order_after_ticket();

    // Last chunk of this (request, KV head) to finish: merge all chunks in chunk order.
    // Half a wavefront takes two query rows at a time (four head dims per lane) and eight
    // chunks of each per pass; every load of a pass is issued before the first is used, so
    // a pass costs one memory round trip.
    constexpr int GROUP = 8;   // chunks merged per pass (16 per pass spill 200 to 340 bytes per lane)
    constexpr int RB = NT >= 2 ? 2 : 1;   // rows in flight per half wavefront (one row tile: at most two passes anyway, and registers are tight)
    const int half = lane >> 5, l32 = lane & 31;
    const bool dims_on = 4 * l32 < D;   // (a head dim of 64 keeps half of the lanes busy)
    for (int r0 = 2 * wave + half; r0 < rows; r0 += 2 * kWaves * RB) {
        bool rv[RB];
        size_t rh[RB];
        const unsigned long long *ml[RB], *pa[RB];
        float mx[RB], denom[RB];
        f32x4 o[RB];
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            const int r = r0 + 2 * kWaves * j;
            rv[j] = r < rows;
            const int rr = rv[j] ? r : 0;
            rh[j] = (size_t)(row0 + rr / group) * p.Hq + kvh * group + rr % group;
            const size_t base = rh[j] * p.max_chunks;
            ml[j] = reinterpret_cast<const unsigned long long *>(p.ws_ml) + base;
            pa[j] = reinterpret_cast<const unsigned long long *>(p.ws_acc) + base * (D / 2) + 2 * l32;
            mx[j] = kEmptyMax;
            denom[j] = 0.0f;
            o[j] = (f32x4){0.0f, 0.0f, 0.0f, 0.0f};
        }
        for (int c0 = 0; c0 < nchunks; c0 += GROUP) {
            unsigned long long mlv[RB][GROUP], a0[RB][GROUP], a1[RB][GROUP];
#pragma unroll
            for (int j = 0; j < RB; ++j) {
#pragma unroll
                for (int c = 0; c < GROUP; ++c) {
                    const bool on = rv[j] && c0 + c < nchunks;
                    mlv[j][c] = on ? fetch_u64(ml[j] + c0 + c) : pack_f32x2(kEmptyMax, 0.0f);
                    a0[j][c] = on && dims_on ? fetch_u64(pa[j] + (size_t)(c0 + c) * (D / 2)) : 0ull;
                    a1[j][c] = on && dims_on ? fetch_u64(pa[j] + (size_t)(c0 + c) * (D / 2) + 1) : 0ull;
                }
            }
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                float gmx = mx[j];
#pragma unroll
                for (int c = 0; c < GROUP; ++c) gmx = fmaxf(gmx, __uint_as_float((uint32_t)mlv[j][c]));
                const float keep = fast_exp2(mx[j] - gmx);   // rescale of what earlier passes summed
                denom[j] *= keep;
                o[j] *= keep;
                mx[j] = gmx;
#pragma unroll
                for (int c = 0; c < GROUP; ++c) {
                    const float w = fast_exp2(__uint_as_float((uint32_t)mlv[j][c]) - gmx);
                    denom[j] = fmaf(w, __uint_as_float((uint32_t)(mlv[j][c] >> 32)), denom[j]);
                    o[j][0] = fmaf(w, __uint_as_float((uint32_t)a0[j][c]), o[j][0]);
                    o[j][1] = fmaf(w, __uint_as_float((uint32_t)(a0[j][c] >> 32)), o[j][1]);
                    o[j][2] = fmaf(w, __uint_as_float((uint32_t)a1[j][c]), o[j][2]);
                    o[j][3] = fmaf(w, __uint_as_float((uint32_t)(a1[j][c] >> 32)), o[j][3]);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < RB; ++j)
            if (rv[j] && dims_on) *reinterpret_cast<f32x4 *>(p.out + rh[j] * D + 4 * l32) = o[j] * (1.0f / denom[j]);
    }
}

// ===========================================================================
// The kernel
// ===========================================================================
// Grid order.  The hardware dispatcher places blocks strictly in grid order and waits for
// the slot it has chosen, so block slots sit idle when neighbouring blocks run for very
// different times.  The order keeps neighbours alike and ends on independent work.
// The rejection items always keep their own order (statistics, race, final).
//  - No more attention blocks than block slots: attention first.  All of them are
//    resident from the start (one per compute unit if there are few: two on one unit
//    would take twice as long as the rest), and the rejection items flow through the
//    slots that are left.
//  - More attention blocks: they take the requests longest first (so blocks that run at
//    the same time take about equally long), and the rejection items are mixed into the
//    first part of them (reject_span of the attention rows), so that the dependent
//    rejection stages are done before the attention items are and the tail of the launch
//    is short attention blocks.  The mixing is done per row of 8 consecutive blocks: the
//    hardware deals consecutive blocks to the 8 XCDs in turn, and a finer pattern would
//    alias with that (with equal counts, "every other block" would put all attention on
//    four XCDs and all rejection on the other four).  Within the mixed part, row r is an
//    attention row iff floor((r+1) * rows_attn / rows) > floor(r * rows_attn / rows).
struct GridSplit {
    int n_stat, n_reject, n_attn;
    int attn_first;        // 1: attention items first, 0: mixed (with no attention rows in the mixed part: rejection items first)
    int rows_attn_mixed;   // attention rows among which the rejection rows are spread; the other attention rows follow
    int reject_cols;       // positions of a row of 8 blocks that carry rejection items: all 8, or the 4 even ones
};

// All kernel arguments in one struct, so that the place of the order table inside the
// kernel-argument segment is known.
struct StepArgs {
    AttnParams ap;
    RejectParams rp;
    GridSplit gs;
    UnitOrder order;
};

template <int NT, int WG, bool HAS_ATTN, bool HAS_REJECT, int VAR>
__global__ __launch_bounds__(kThreads, 2) void spec_step_kernel(StepArgs args)
{
    const AttnParams &ap = args.ap;
    const RejectParams &rp = args.rp;
    const GridSplit &gs = args.gs;
    int item = blockIdx.x;
    bool is_attn = HAS_ATTN;
    if constexpr (HAS_ATTN && HAS_REJECT) {
        if (gs.attn_first) {
            const int n_attn_rows8 = (gs.n_attn + kXcds - 1) / kXcds * kXcds;   // whole rows: positions keep their XCD
            is_attn = item < n_attn_rows8;
            if (is_attn) {
                if (item >= gs.n_attn) return;   // padding of the last attention row
            } else {
                item -= n_attn_rows8;
                if (gs.reject_cols != kXcds) {
                    if (item & 1) return;
                    item >>= 1;
                }
                if (item >= gs.n_reject) return;
            }
        } else {
            // rows of kXcds consecutive blocks (one per XCD, the hardware deals blocks to the
            // XCDs round-robin) share a role, so every XCD sees the same mix
            const int row = item / kXcds, col = item % kXcds;
            const long long rows_attn = gs.rows_attn_mixed;
            const long long rows_all = rows_attn + (gs.n_reject + gs.reject_cols - 1) / gs.reject_cols;
            if (row < rows_all) {
                const int before = (int)((row * rows_attn) / rows_all);
                const int upto = (int)(((row + 1) * rows_attn) / rows_all);
                is_attn = upto > before;
                if (is_attn) {
                    item = before * kXcds + col;
                } else if (gs.reject_cols == kXcds) {
                    item = (row - before) * kXcds + col;
                } else {
                    if (col & 1) return;
                    item = (row - before) * (kXcds / 2) + (col >> 1);
                }
            } else {   // the attention rows after the last rejection row
                is_attn = true;
                item = (int)(rows_attn + (row - rows_all)) * kXcds + col;
            }
            if (item >= (is_attn ? gs.n_attn : gs.n_reject)) return;   // padding of the last row
        }
    }
    if constexpr (HAS_REJECT) {
        if (!is_attn) {
            __shared__ RejectShared rsh;
            if (item < gs.n_stat) {
                // a whole 32000-entry row per round trip where the registers allow it
                stats_role<(HAS_ATTN && NT >= 2) ? 32 : 16>(rp, item, rsh);
            } else {
                const int after = item - gs.n_stat;
                const int n_race = rp.B * rp.race_segments;
                if (after < n_race) race_role(rp, after, rsh);
                else final_role(rp, after - n_race, rsh);
            }
            return;
        }
    }
    if constexpr (HAS_ATTN) {
        __shared__ AttnShared<NT, WG, token_major_of(VAR), head_dim_of(VAR)> ash;
        OrderTable order;
        order.n = args.order.n;
        order.pairs = (uniform_u32_ptr)((const char __attribute__((address_space(4))) *)__builtin_amdgcn_kernarg_segment_ptr() +
                                        offsetof(StepArgs, order) + offsetof(UnitOrder, request));
        attn_role<NT, WG, VAR>(ap, order, item, ash);
    }
}

template <int NT, int WG, bool HAS_ATTN, bool HAS_REJECT>
hipError_t launch(const AttnParams &ap, const RejectParams &rp, int n_stat, int n_attn, int n_race,
                  const UnitOrder *order, LaunchEvents ev, hipStream_t stream)
{
    StepArgs args;
    args.ap = ap;
    args.rp = rp;
    args.order.n = 0;
    if (HAS_ATTN && order != nullptr && order->n > 0) {
        args.order.n = order->n;
        memcpy(args.order.request, order->request, sizeof(uint16_t) * (size_t)order->n);
    }
    GridSplit &gs = args.gs;
    gs.n_stat = n_stat;
    gs.n_reject = n_stat + n_race;
    gs.n_attn = n_attn;
    gs.attn_first = (n_attn <= ap.attn_first_limit) ? 1 : 0;
    const int n_reject = n_stat + n_race;
    // The rejection items are a chain of dependent stages that takes some 15 us whatever its size.
    // Beside an attention half that streams for no longer than that (the planner's estimate), the
    // chain is what the launch waits for: its items go first, ahead of the attention blocks, which
    // lose a few microseconds of dispatch to them.  (Four requests of 512 tokens: 21.2 -> 18.0 us;
    // sixteen with 64/8 heads: 28.3 -> 24.6 us; two of 2048 tokens: 22.4 -> 19.2 us.)
    // (In terms of the mixed order: no attention rows among the rejection rows.)
    const bool reject_first = HAS_ATTN && HAS_REJECT && n_reject <= ap.reject_first_limit;
    if (reject_first) gs.attn_first = 0;
    const bool mixed = HAS_ATTN && HAS_REJECT && !gs.attn_first;
    // The rejection stages of a request wait for each other, so the last rejection item sits
    // well before the end of the grid: the tail of the launch is attention only.
    const int rows_attn_all = (n_attn + kXcds - 1) / kXcds;
    gs.rows_attn_mixed = (int)(rows_attn_all * (double)ap.reject_span);
    if (gs.rows_attn_mixed < 1) gs.rows_attn_mixed = 1;
    if (gs.rows_attn_mixed > rows_attn_all) gs.rows_attn_mixed = rows_attn_all;
    if (reject_first) gs.rows_attn_mixed = 0;
    // XCDs 1, 3, 5, 7 of this device stream from memory some 6% slower than XCDs 0, 2, 4, 6 (block
    // traces of equal attention blocks), and a launch ends with its slowest XCD.  When there is at
    // most one attention block per compute unit (all resident from the start, the rejection blocks
    // beside them), the rejection blocks, which slow down the attention block they share a compute
    // unit with, go to the even XCDs only: even positions of a row of 8 blocks; the odd positions
    // of such rows exit at once.  (With more attention blocks it does not pay: measured 1% slower
    // with two per compute unit, 15% slower where the rejection half is a fifth of the step.)
    gs.reject_cols = (HAS_ATTN && HAS_REJECT && ap.reject_even_xcds && n_attn <= ap.reject_even_limit && !reject_first) ? kXcds / 2 : kXcds;
    const int rows_reject = (n_reject + gs.reject_cols - 1) / gs.reject_cols;
    const dim3 grid(mixed ? (rows_attn_all + rows_reject) * kXcds
                          : (HAS_ATTN && HAS_REJECT ? (rows_attn_all + rows_reject) * kXcds : n_reject + n_attn));
    // (with events the extended launch attaches them to the kernel's own begin and end)
    auto go = [&](auto var) {
        constexpr int VAR = decltype(var)::value;
        if (ev.start != nullptr)
            hipExtLaunchKernelGGL((spec_step_kernel<NT, WG, HAS_ATTN, HAS_REJECT, VAR>), grid, dim3(kThreads), 0, stream, ev.start,
                                  ev.stop, 0, args);
        else
            hipLaunchKernelGGL((spec_step_kernel<NT, WG, HAS_ATTN, HAS_REJECT, VAR>), grid, dim3(kThreads), 0, stream, args);
        return hipGetLastError();
    };
    if constexpr (HAS_ATTN) {
        if (ap.kv_layout == SPEC_KV_TOKEN_MAJOR)
            return ap.d == 64 ? go(std::integral_constant<int, 4>()) : go(std::integral_constant<int, 2>());
        if (ap.d == 64) return go(std::integral_constant<int, 3>());
        // (the single-bf16 experiment exists for one wave group only)
        if constexpr (WG == 1)
            if (!ap.split_p) return go(std::integral_constant<int, 1>());
    }
    return go(std::integral_constant<int, 0>());
}

}  // namespace

// The kernel variants of this file take over a minute to compile in one piece, so the build
// compiles the file several times, each time with SPEC_STEP_PART set to the part whose
// launchers it should hold (everything else of the file is shared, file-local code):
//   0: the dispatcher below, the rejection-only kernel, one row tile    1: two row tiles
//   2: three row tiles    3: two wave groups    4: four wave groups      (unset: all of it)
#ifndef SPEC_STEP_PART
#define SPEC_STEP_PART -1
#endif
#define SPEC_STEP_HAS_PART(k) (SPEC_STEP_PART < 0 || SPEC_STEP_PART == (k))

// launchers of the (row tiles, wave groups) variants, one function each
#define SPEC_STEP_LAUNCHER(NAME) \
    hipError_t NAME(const AttnParams &ap, const RejectParams &rp, bool with_reject, int n_stat, int n_attn, int n_race, \
                    const UnitOrder *order, LaunchEvents ev, hipStream_t stream)
SPEC_STEP_LAUNCHER(launch_step_tiles1);
SPEC_STEP_LAUNCHER(launch_step_tiles2);
SPEC_STEP_LAUNCHER(launch_step_tiles3);
SPEC_STEP_LAUNCHER(launch_step_tiles2_groups2);
SPEC_STEP_LAUNCHER(launch_step_tiles3_groups2);
SPEC_STEP_LAUNCHER(launch_step_tiles2_groups4);
SPEC_STEP_LAUNCHER(launch_step_tiles3_groups4);
#define SPEC_STEP_DEFINE(NAME, NT_, WG_)                                                                     \
    SPEC_STEP_LAUNCHER(NAME)                                                                                 \
    {                                                                                                        \
        return with_reject ? launch<NT_, WG_, true, true>(ap, rp, n_stat, n_attn, n_race, order, ev, stream) \
                           : launch<NT_, WG_, true, false>(ap, rp, 0, n_attn, 0, order, ev, stream);         \
    }
#if SPEC_STEP_HAS_PART(0)
SPEC_STEP_DEFINE(launch_step_tiles1, 1, 1)
#endif
#if SPEC_STEP_HAS_PART(1)
SPEC_STEP_DEFINE(launch_step_tiles2, 2, 1)
#endif
#if SPEC_STEP_HAS_PART(2)
SPEC_STEP_DEFINE(launch_step_tiles3, 3, 1)
#endif
#if SPEC_STEP_HAS_PART(3)
SPEC_STEP_DEFINE(launch_step_tiles2_groups2, 2, 2)
SPEC_STEP_DEFINE(launch_step_tiles3_groups2, 3, 2)
#endif
#if SPEC_STEP_HAS_PART(4)
SPEC_STEP_DEFINE(launch_step_tiles2_groups4, 2, 4)
SPEC_STEP_DEFINE(launch_step_tiles3_groups4, 3, 4)
#endif
#undef SPEC_STEP_DEFINE
#undef SPEC_STEP_LAUNCHER

#if SPEC_STEP_HAS_PART(0)
int step_attn_items(const AttnParams &ap)
{
    return attn_row_items(ap) * ap.max_chunks;
}

hipError_t launch_step_fused(const AttnParams *attn, int row_tiles, const RejectParams *reject, const UnitOrder *order,
                             LaunchEvents ev, hipStream_t stream)
{
    AttnParams ap = {};
    RejectParams rp = {};
    int n_stat = 0, n_attn = 0, n_race = 0;
    if (reject != nullptr) {
        rp = *reject;
        if (rp.stat_segments > kMaxStatSegments || rp.race_segments > kWave || rp.spin_limit < 1)
            return hipErrorInvalidValue;
        if (rp.mode == SPEC_ACCEPT_GREEDY) rp.race_segments = 0;   // no race stage
        n_stat = (rp.mode == SPEC_ACCEPT_SAMPLE ? 2 * rp.T - rp.B : rp.T) * rp.stat_segments;
        n_race = rp.B * rp.race_segments + rp.B;   // race segments, then one final item per request
    }
    if (attn != nullptr) {
        ap = *attn;
        // tiles per wave group and wave groups per block that the kernel is built for
        const bool shape_ok = (ap.row_groups == 1 && row_tiles >= 1 && row_tiles <= 3) ||
                              ((ap.row_groups == 2 || ap.row_groups == 4) && (row_tiles == 2 || row_tiles == 3));
        // (a wavefront keeps the block-table entries of its pages one per lane)
        const bool dim_ok = ap.d == kD || ap.d == 64;
        if (!dim_ok || !shape_ok || ap.chunk_tokens > 4096 / ap.row_groups || ap.chunk_tokens % SPEC_BLOCK_SIZE != 0 ||
            ap.capacity_tokens > ap.chunk_tokens * ap.max_chunks ||
            (ap.fused_combine && ap.max_chunks > kMaxFusedChunks) || (order != nullptr && order->n != 0 && order->n != ap.B))
            return hipErrorInvalidValue;
        n_attn = step_attn_items(ap);
    }
    if (attn == nullptr) return launch<1, 1, false, true>(ap, rp, n_stat, 0, n_race, nullptr, ev, stream);
    const bool with_reject = reject != nullptr;
    switch (ap.row_groups * 10 + row_tiles) {
        case 11: return launch_step_tiles1(ap, rp, with_reject, n_stat, n_attn, n_race, order, ev, stream);
        case 12: return launch_step_tiles2(ap, rp, with_reject, n_stat, n_attn, n_race, order, ev, stream);
        case 13: return launch_step_tiles3(ap, rp, with_reject, n_stat, n_attn, n_race, order, ev, stream);
        case 22: return launch_step_tiles2_groups2(ap, rp, with_reject, n_stat, n_attn, n_race, order, ev, stream);
        case 23: return launch_step_tiles3_groups2(ap, rp, with_reject, n_stat, n_attn, n_race, order, ev, stream);
        case 42: return launch_step_tiles2_groups4(ap, rp, with_reject, n_stat, n_attn, n_race, order, ev, stream);
        default: return launch_step_tiles3_groups4(ap, rp, with_reject, n_stat, n_attn, n_race, order, ev, stream);
    }
}
#endif   // part 0

}  // namespace specv
