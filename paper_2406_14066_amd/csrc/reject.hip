// Rejection sampling with bonus token over the vocabulary (the acceptance
// phase of Section 4 of arXiv 2406.14066; accept rule of the cited
// speculative-sampling method), as two HBM-streaming kernels:
//
//   logit_stats_kernel   one pass over every target and draft logit row:
//                        per (row, vocabulary segment) the maximum and the
//                        sum of exp(x - max).
//   accept_race_kernel   per request: log-sum-exp of its rows, the accept
//                        chain over its draft tokens, then an exponential race
//                        over the one row pair that decides the next token,
//                        split over several blocks; the last block to finish
//                        picks the winner and writes the outputs.
//
// Precision: the streaming arithmetic is fp32 (the kernels are bound by HBM
// bandwidth and an fp64 exp per logit would not be); everything that happens
// once per row or per decision (combining segment sums, log-sum-exp, p/q of
// the draft token, the comparison with u) is fp64.
#include "common.h"

#include <float.h>
#include <math.h>

namespace specv {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies,
// a word permutation with key xor, and a Weyl sequence on the key.
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi_a = __umulhi(0xD2511F53u, c.x), lo_a = 0xD2511F53u * c.x;
        const uint32_t hi_b = __umulhi(0xCD9E8D57u, c.z), lo_b = 0xCD9E8D57u * c.z;
        c = make_uint4(hi_b ^ c.y ^ k0, lo_b, hi_a ^ c.w ^ k1, lo_a);
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// ---------------------------------------------------------------------------
// Pass 1: row statistics.  grid = (segments, rows); rows 0..T-1 are target rows,
// rows T..2T-B-1 are draft rows.
// ---------------------------------------------------------------------------
template <int UNROLL>
__global__ __launch_bounds__(kThreads) void logit_stats_kernel(RejectParams p)
{
    const int tid = threadIdx.x;
    const int row = blockIdx.y;
    const int seg = blockIdx.x;
    if (row == 0 && seg == 0)
        for (int i = tid; i < p.B; i += kThreads) p.tickets[i] = 0;  // used by the race pass

    const float *base = row < p.T ? p.target_logits + (size_t)row * p.V
                                  : p.draft_logits + (size_t)(row - p.T) * p.V;
    const int v0 = seg * p.stat_seg_len;
    const int v1 = min(p.V, v0 + p.stat_seg_len);
    const float4 *vec = reinterpret_cast<const float4 *>(base + v0);
    const int nvec = (v1 - v0) >> 2;

    // Running offset `off` in base-2 units, kept integer-valued so that every
    // rescale is an exact power of two and x*log2(e) - off is rounded once
    // (log2(e) is applied as an fp32 hi/lo pair inside fused multiply-adds).
    constexpr float kLog2eHi = 1.4426950216293335f;
    constexpr float kLog2eLo = 1.9259629911266175e-8f;
    float m = -FLT_MAX;   // largest logit seen
    float off = kEmptyMax;
    float s = 0.0f;       // sum of 2^(x*log2e - off)
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

    __shared__ float sh_max[kWaves];
    __shared__ double sh_sum[kWaves];
    const int wave = tid / kWave, lane = tid % kWave;
    float wm = wave_max(off);
    if (lane == 0) sh_max[wave] = wm;
    __syncthreads();
    float boff = sh_max[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) boff = fmaxf(boff, sh_max[w]);
    // one exact power-of-two rescale per thread, then the cross-thread sum in fp64
    double sd = (double)s * (double)fast_exp2(off - boff);
    sd = wave_sum(sd);
    if (lane == 0) sh_sum[wave] = sd;
    __syncthreads();
    if (tid == 0) {
        double total = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) total += sh_sum[w];
        RowStat st;
        st.sum = total;
        st.off2 = boff;
        st.pad = 0.0f;
        p.stats[(size_t)row * p.stat_segments + seg] = st;
    }
}

// ---------------------------------------------------------------------------
// The race over vocabulary ids [v0, v1) of one request: best r_v / e_v with
// e_v = -log(U'_v).  `draft_row` == nullptr means the weights are the target
// probabilities (bonus token); otherwise the positive part of p - q.
//   p_v = corr_t * 2^(x_v * log2e + off_t), off_t = fp32(-log2-sum-exp), corr_t
//   the factor lost by rounding off_t; log2e is applied as a hi/lo pair so that
//   the exponent carries one rounding only.
// Returns this thread's best (score, id); ties keep the lowest id.
// ---------------------------------------------------------------------------
struct Best {
    float score;
    int32_t id;
};

__device__ __forceinline__ void take_better(Best &a, float score, int32_t id)
{
    if (score > a.score || (score == a.score && id < a.id)) {
        a.score = score;
        a.id = id;
    }
}

__device__ __forceinline__ float race_exponential(uint32_t word)
{
    // U' = (n) * 2^-24 with n = (word >> 8) + 1 in [1, 2^24]; e = -log(U').
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

__device__ Best race_segment(const float *target_row, const float *draft_row, int v0, int v1, int b,
                             const RejectParams &p, float off_t, float corr_t, float off_d, float corr_d)
{
    constexpr float kLog2eHi = 1.4426950216293335f;   // fp32(log2 e)
    constexpr float kLog2eLo = 1.9259629911266175e-8f;  // log2 e - kLog2eHi
    Best best;
    best.score = -1.0f;
    best.id = 0x7FFFFFFF;
    const int ngroups = (v1 - v0) >> 2;
    const uint32_t c3 = (p.step_hi24 << 8) | 1u;
    for (int g = threadIdx.x; g < ngroups; g += kThreads) {
        const int v = v0 + 4 * g;
        const float4 xt = *reinterpret_cast<const float4 *>(target_row + v);
        float r[4];
        {
            const float x[4] = {xt.x, xt.y, xt.z, xt.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                r[e] = corr_t * fast_exp2(fmaf(x[e], kLog2eHi, fmaf(x[e], kLog2eLo, off_t)));
        }
        if (draft_row != nullptr) {
            const float4 xd = *reinterpret_cast<const float4 *>(draft_row + v);
            const float x[4] = {xd.x, xd.y, xd.z, xd.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                r[e] -= corr_d * fast_exp2(fmaf(x[e], kLog2eHi, fmaf(x[e], kLog2eLo, off_d)));
        }
        const uint4 w = philox4x32_10(make_uint4((uint32_t)v >> 2, (uint32_t)b, p.step_lo, c3), p.seed_lo, p.seed_hi);
        const uint32_t word[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (r[e] > 0.0f) {
                const float ex = race_exponential(word[e]);
                const float score = r[e] * __builtin_amdgcn_rcpf(ex);  // ex == 0 -> +inf
                if (score > best.score) {  // ids rise within a thread: strict > keeps the lowest
                    best.score = score;
                    best.id = v + e;
                }
            }
        }
    }
    return best;
}

__device__ Best block_best(Best mine, Best *sh)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        const float os = __shfl_xor(mine.score, off);
        const int32_t oi = __shfl_xor(mine.id, off);
        take_better(mine, os, oi);
    }
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    __syncthreads();  // sh may still be read from an earlier call
    if (lane == 0) sh[wave] = mine;
    __syncthreads();
    Best out = sh[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) take_better(out, sh[w].score, sh[w].id);
    return out;
}

__device__ __forceinline__ unsigned long long pack_best(Best b)
{
    return ((unsigned long long)__float_as_uint(b.score) << 32) | (unsigned long long)(uint32_t)b.id;
}

__device__ __forceinline__ Best unpack_best(unsigned long long v)
{
    Best b;
    b.score = __uint_as_float((uint32_t)(v >> 32));
    b.id = (int32_t)(uint32_t)(v & 0xFFFFFFFFull);
    return b;
}

// ---------------------------------------------------------------------------
// Pass 2: accept chain + race.  grid = (race_segments, B).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void accept_race_kernel(RejectParams p)
{
    const int tid = threadIdx.x;
    const int b = blockIdx.y;
    const int seg = blockIdx.x;

    __shared__ double sh_lse2[2 * SPEC_K_MAX + 1];  // log2-sum-exp: target rows 0..k, then draft rows 0..k-1
    __shared__ double sh_u[SPEC_K_MAX], sh_ratio[SPEC_K_MAX];
    __shared__ int sh_accept[SPEC_K_MAX];
    __shared__ int sh_m, sh_near, sh_last;
    __shared__ Best sh_best[kWaves];

    const int row_t0 = p.cu_q_len[b];
    const int k = p.cu_q_len[b + 1] - row_t0 - 1;
    const int row_d0 = row_t0 - b;

    // log-sum-exp of the request's rows from the segment statistics (fp64)
    if (tid < 2 * k + 1) {
        const int row = tid <= k ? row_t0 + tid : p.T + row_d0 + (tid - k - 1);
        const RowStat *st = p.stats + (size_t)row * p.stat_segments;
        float mx = st[0].off2;
        for (int s = 1; s < p.stat_segments; ++s) mx = fmaxf(mx, st[s].off2);
        double total = 0.0;
        for (int s = 0; s < p.stat_segments; ++s) total += st[s].sum * exp2((double)(st[s].off2 - mx));
        sh_lse2[tid] = (double)mx + log2(total);
    }
    __syncthreads();

    // accept tests (all evaluated in parallel, the chain is resolved below)
    if (tid < k) {
        const int x = p.draft_tokens[row_d0 + tid];
        const float tx = p.target_logits[(size_t)(row_t0 + tid) * p.V + x];
        const float dx = p.draft_logits[(size_t)(row_d0 + tid) * p.V + x];
        const double log2_p = (double)tx * kLog2eD - sh_lse2[tid];
        const double log2_q = (double)dx * kLog2eD - sh_lse2[k + 1 + tid];
        const double ratio = exp2(log2_p - log2_q);  // p = 0 -> 0, q = 0 < p -> inf, both 0 -> NaN (rejects)
        const uint4 w = philox4x32_10(make_uint4((uint32_t)tid, (uint32_t)b, p.step_lo, (p.step_hi24 << 8) | 0u),
                                      p.seed_lo, p.seed_hi);
        const double u = (double)(w.x >> 8) * (1.0 / 16777216.0);
        sh_u[tid] = u;
        sh_ratio[tid] = ratio;
        sh_accept[tid] = (u < ratio) ? 1 : 0;
    }
    __syncthreads();
    if (tid == 0) {
        int m = 0;
        while (m < k && sh_accept[m]) ++m;
        int near = 0;
        const int evaluated = m + 1 < k ? m + 1 : k;
        for (int i = 0; i < evaluated; ++i)
            if (fabs(sh_u[i] - sh_ratio[i]) < 1e-6) ++near;
        sh_m = m;
        sh_near = near;
    }
    __syncthreads();
    const int m = sh_m;
    const bool correction = m < k;

    if (seg == 0 && p.debug_u_ratio != nullptr && tid < k) {
        const bool evaluated = tid <= m;
        p.debug_u_ratio[2 * (size_t)(row_d0 + tid) + 0] = evaluated ? sh_u[tid] : (double)NAN;
        p.debug_u_ratio[2 * (size_t)(row_d0 + tid) + 1] = evaluated ? sh_ratio[tid] : (double)NAN;
    }

    // race over this block's vocabulary segment
    const float *trow = p.target_logits + (size_t)(row_t0 + m) * p.V;
    const float *drow = correction ? p.draft_logits + (size_t)(row_d0 + m) * p.V : nullptr;
    const double off_t_exact = -sh_lse2[m];
    const float off_t = (float)off_t_exact;
    const float corr_t = (float)exp2(off_t_exact - (double)off_t);
    float off_d = 0.0f, corr_d = 0.0f;
    if (correction) {
        const double off_d_exact = -sh_lse2[k + 1 + m];
        off_d = (float)off_d_exact;
        corr_d = (float)exp2(off_d_exact - (double)off_d);
    }
    const int v0 = seg * p.race_seg_len;
    const int v1 = min(p.V, v0 + p.race_seg_len);
    Best mine = race_segment(trow, drow, v0, v1, b, p, off_t, corr_t, off_d, corr_d);
    Best blk = block_best(mine, sh_best);

    if (tid == 0) {
        __hip_atomic_store(&p.race_partial[(size_t)b * p.race_segments + seg], pack_best(blk), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();
        const int ticket = atomicAdd(&p.tickets[b], 1);
        sh_last = (ticket == p.race_segments - 1) ? 1 : 0;
    }
    __syncthreads();
    if (!sh_last) return;

    // last block of this request: pick the winner
    __threadfence();
    Best win;
    win.score = -1.0f;
    win.id = 0x7FFFFFFF;
    if (tid == 0) {
        for (int s = 0; s < p.race_segments; ++s) {
            const Best o = unpack_best(__hip_atomic_load(&p.race_partial[(size_t)b * p.race_segments + s],
                                                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            take_better(win, o.score, o.id);
        }
        sh_best[0] = win;
    }
    __syncthreads();
    win = sh_best[0];
    __syncthreads();
    if (!(win.score > 0.0f)) {
        // p - q has no positive entry (p == q to rounding): draw from p instead
        Best again = race_segment(trow, nullptr, 0, p.V, b, p, off_t, corr_t, 0.0f, 0.0f);
        win = block_best(again, sh_best);
    }
    if (tid == 0) {
        p.accepted_len[b] = m;
        p.next_token[b] = win.id;
        if (p.out_tokens != nullptr) {
            int32_t *row = p.out_tokens + (size_t)b * (SPEC_K_MAX + 1);
            for (int i = 0; i <= SPEC_K_MAX; ++i)
                row[i] = i < m ? p.draft_tokens[row_d0 + i] : (i == m ? win.id : -1);
        }
        atomicAdd(&p.counters[0], (unsigned long long)k);
        atomicAdd(&p.counters[1], (unsigned long long)m);
        atomicAdd(&p.counters[2], (unsigned long long)(m + 1 < k ? m + 1 : k));
        atomicAdd(&p.counters[3], (unsigned long long)(m + 1));
        atomicAdd(&p.counters[4], (unsigned long long)sh_near);
        atomicAdd(&p.counters[5], 1ull);
        p.tickets[b] = 0;
    }
}

}  // namespace

hipError_t launch_logit_stats(const RejectParams &p, hipStream_t stream)
{
    const int rows = 2 * p.T - p.B;
    dim3 grid(p.stat_segments, rows);
    hipLaunchKernelGGL(logit_stats_kernel<4>, grid, dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_accept_race(const RejectParams &p, hipStream_t stream)
{
    dim3 grid(p.race_segments, p.B);
    hipLaunchKernelGGL(accept_race_kernel, grid, dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace specv
