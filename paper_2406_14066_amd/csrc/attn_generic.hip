// Lookahead attention, generic kernels (Section 2.2 / Section 4 of arXiv
// 2406.14066: the k+1 query positions of a request are scored against its
// cached keys and values, query j seeing keys 0 .. kv_len - q_len + j).
//
//   attn_generic_kernel   any dtype (fp32, bf16) and page layout, scalar fp32
//                         arithmetic: one block per (KV chunk, query head,
//                         query row), one thread per key of the chunk.  This is
//                         the fp32 path and the fallback for shapes the
//                         matrix-instruction kernel does not take.
//   attn_combine_kernel   merges the per-chunk partial results of either
//                         attention kernel: out = sum_c w_c acc_c / sum_c w_c l_c,
//                         w_c = 2^(m_c - max_c m_c).  Requests with one chunk are
//                         written by the kernel that holds their only partial.
//   kv_repack_kernel      token-major pages -> matrix-instruction page layout.
//
// Scores are kept in base-2 units (the softmax scale is folded with log2 e).
#include "common.h"

#include <math.h>

namespace specv {

namespace {

constexpr int kChunkThreads = 256;

__device__ __forceinline__ float load_as_float(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_as_float(const uint16_t *p, size_t i)
{
    return __uint_as_float((uint32_t)p[i] << 16);
}

// index of K/V element (page, kv head, slot, dim) in the two page layouts
__device__ __forceinline__ size_t k_index(int layout, int page, int Hkv, int kvh, int slot, int c, int d)
{
    const size_t head = (size_t)page * Hkv + kvh;
    if (layout == SPEC_KV_TOKEN_MAJOR) return (head * SPEC_BLOCK_SIZE + slot) * d + c;
    return ((head * (d >> 3) + (c >> 3)) * SPEC_BLOCK_SIZE + slot) * 8 + (c & 7);
}

// SPEC_KV_MFMA value layout inside one (page, kv head): [d/32][4 token groups][16 dims][2 dim halves][4 tokens]
__device__ __forceinline__ size_t v_tiled_offset(int c, int slot)
{
    const int pair = c >> 5, half = (c >> 4) & 1, m = c & 15, g = slot >> 2, r = slot & 3;
    return (size_t)((((pair * 4 + g) * 16 + m) * 2 + half) * 4 + r);
}

__device__ __forceinline__ size_t v_index(int layout, int page, int Hkv, int kvh, int slot, int c, int d)
{
    const size_t head = (size_t)page * Hkv + kvh;
    if (layout == SPEC_KV_TOKEN_MAJOR) return (head * SPEC_BLOCK_SIZE + slot) * d + c;
    return head * d * SPEC_BLOCK_SIZE + v_tiled_offset(c, slot);
}

// request that owns packed query row `row`: largest b with cu_q_len[b] <= row
// (T = cu_q_len[B]; with one draft length for all requests the first guess is right, and its two
// loads replace a chain of log2 B dependent ones)
__device__ __forceinline__ int find_request(const int32_t *cu_q_len, int B, int T, int row)
{
    const int guess = min((int)(((long long)row * B) / T), B - 1);
    if (cu_q_len[guess] <= row && row < cu_q_len[guess + 1]) return guess;
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (cu_q_len[mid] <= row) lo = mid; else hi = mid - 1;
    }
    return lo;
}

template <typename KV_T>
__global__ __launch_bounds__(kChunkThreads) void attn_generic_kernel(AttnParams p)
{
    const int tid = threadIdx.x;
    const int chunk = blockIdx.x;
    const int h = blockIdx.y;
    const int row = blockIdx.z;
    const int b = find_request(p.cu_q_len, p.B, p.T, row);
    const int q_len = p.cu_q_len[b + 1] - p.cu_q_len[b];
    const int j = row - p.cu_q_len[b];
    const int L = p.kv_len[b];
    // (lengths from device memory bound the loops and indices below: a request that does not fit
    // the launch is left out and reported once)
    if (!request_lengths_ok(L, q_len, p.capacity_tokens, p.max_blocks_per_req)) {
        if (chunk == 0 && h == 0 && j == 0 && tid == 0 && p.errors != nullptr) atomicAdd(p.errors, 1ull);
        return;
    }
    const int nchunks = (L + p.chunk_tokens - 1) / p.chunk_tokens;
    if (chunk >= nchunks) return;
    const int last_visible = L - q_len + j;
    const int kvh = h / (p.Hq / p.Hkv);
    const int d = p.d;

    __shared__ float sh_q[128];
    __shared__ float sh_p[kChunkThreads];
    __shared__ int sh_page[kChunkThreads];
    __shared__ float sh_red[kChunkThreads / kWave];

    const KV_T *q = static_cast<const KV_T *>(p.q);
    const KV_T *kc = static_cast<const KV_T *>(p.k_cache);
    const KV_T *vc = static_cast<const KV_T *>(p.v_cache);
    if (tid < d) sh_q[tid] = load_as_float(q, ((size_t)row * p.Hq + h) * d + tid);
    __syncthreads();

    // one key per thread (chunk_tokens == blockDim.x)
    const int token = chunk * p.chunk_tokens + tid;
    const bool visible = tid < p.chunk_tokens && token <= last_visible;
    float score = -INFINITY;
    int page = -1;
    if (visible) {
        page = p.block_table[(size_t)b * p.max_blocks_per_req + token / SPEC_BLOCK_SIZE];
        const int slot = token % SPEC_BLOCK_SIZE;
        if ((unsigned)page < (unsigned)p.num_blocks) {
            // eight consecutive head dims are contiguous in both page layouts: one vector load per
            // group, several groups in flight (element by element the loop is a chain of load
            // latencies: 37 us for 128 keys of 64 dims)
            struct alignas(8 * sizeof(KV_T)) Vec8 { KV_T e[8]; };
            float dot = 0.0f;
#pragma unroll 8
            for (int c = 0; c < d; c += 8) {
                const Vec8 kv = *reinterpret_cast<const Vec8 *>(kc + k_index(p.kv_layout, page, p.Hkv, kvh, slot, c, d));
#pragma unroll
                for (int e = 0; e < 8; ++e) dot = fmaf(sh_q[c + e], load_as_float(kv.e, e), dot);
            }
            score = dot * p.scale_log2;
        } else {
            // an entry outside the pool is never turned into an address: the page reads as zeros
            page = -1;
            score = 0.0f;
            if (slot == 0 && h == 0 && j == 0 && p.errors != nullptr) atomicAdd(p.errors, 1ull);
        }
    }
    sh_page[tid] = page;

    // block maximum
    float mx = score;
    for (int off = kWave / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if (tid % kWave == 0) sh_red[tid / kWave] = mx;
    __syncthreads();
    mx = kEmptyMax;
    for (int w = 0; w < kChunkThreads / kWave; ++w) mx = fmaxf(mx, sh_red[w]);
    __syncthreads();

    const float prob = visible ? __builtin_amdgcn_exp2f(score - mx) : 0.0f;
    sh_p[tid] = prob;
    float sum = prob;
    for (int off = kWave / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if (tid % kWave == 0) sh_red[tid / kWave] = sum;
    __syncthreads();
    sum = 0.0f;
    for (int w = 0; w < kChunkThreads / kWave; ++w) sum += sh_red[w];

    // weighted sum of values: the block's 256 / d thread groups take the keys in turn, one head
    // dim per thread, and the groups' sums are added through shared memory (d is 64 or 128)
    const size_t slot_index = ((size_t)row * p.Hq + h) * p.max_chunks + chunk;
    const int ngrp = kChunkThreads / d;
    const int grp = tid / d, c = tid % d;
    {
        const int ntok = min(p.chunk_tokens, last_visible - chunk * p.chunk_tokens + 1);
        float acc = 0.0f;
        // (no branch in the loop, so that the loads of several keys are in flight together: a page
        // that is not there is read as page 0 with weight 0)
#pragma unroll 8
        for (int t = grp; t < ntok; t += ngrp) {
            const int slot = (chunk * p.chunk_tokens + t) % SPEC_BLOCK_SIZE;
            const int pg = sh_page[t];
            const float v = load_as_float(vc, v_index(p.kv_layout, max(pg, 0), p.Hkv, kvh, slot, c, d));
            acc = fmaf(pg >= 0 ? sh_p[t] : 0.0f, pg >= 0 ? v : 0.0f, acc);
        }
        __syncthreads();     // every thread has read its probabilities: the buffer now carries the groups' sums
        sh_p[tid] = acc;
        __syncthreads();
    }
    if (tid < d) {
        float acc = 0.0f;
        for (int gi = 0; gi < ngrp; ++gi) acc += sh_p[gi * d + tid];
        // the only chunk of its request: the row is complete, no merge needed
        if (nchunks == 1) p.out[((size_t)row * p.Hq + h) * d + tid] = acc / sum;
        else p.ws_acc[slot_index * d + tid] = acc;
    }
    if (tid == 0 && nchunks > 1) {
        p.ws_ml[slot_index * 2 + 0] = mx;
        p.ws_ml[slot_index * 2 + 1] = sum;
    }
}

// grid = T*Hq blocks of d threads
__global__ void attn_combine_kernel(AttnParams p)
{
    const int row = blockIdx.x / p.Hq;
    const int h = blockIdx.x % p.Hq;
    const int tid = threadIdx.x;
    const int b = find_request(p.cu_q_len, p.B, p.T, row);
    if (!request_lengths_ok(p.kv_len[b], p.cu_q_len[b + 1] - p.cu_q_len[b], p.capacity_tokens, p.max_blocks_per_req))
        return;   // left out by the partial kernel too
    const int nchunks = (p.kv_len[b] + p.chunk_tokens - 1) / p.chunk_tokens;
    if (nchunks == 1) return;   // written by the kernel that made the partial results
    const size_t base = ((size_t)row * p.Hq + h) * p.max_chunks;
    float mx = kEmptyMax;
#pragma unroll 8
    for (int c = 0; c < nchunks; ++c) mx = fmaxf(mx, p.ws_ml[(base + c) * 2]);
    float denom = 0.0f, acc = 0.0f;
#pragma unroll 8
    for (int c = 0; c < nchunks; ++c) {
        const float w = __builtin_amdgcn_exp2f(p.ws_ml[(base + c) * 2] - mx);
        denom = fmaf(w, p.ws_ml[(base + c) * 2 + 1], denom);
        acc = fmaf(w, p.ws_acc[(base + c) * p.d + tid], acc);
    }
    p.out[((size_t)row * p.Hq + h) * p.d + tid] = acc / denom;
}

// one thread per (page, kv head, slot, group of 8 dims)
__global__ void kv_repack_kernel(const uint16_t *src_k, const uint16_t *src_v, uint16_t *dst_k, uint16_t *dst_v,
                                 size_t heads, int d)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int groups = d >> 3;
    const size_t total = heads * SPEC_BLOCK_SIZE * groups;
    if (idx >= total) return;
    const int g = (int)(idx % groups);
    const int slot = (int)((idx / groups) % SPEC_BLOCK_SIZE);
    const size_t head = idx / ((size_t)groups * SPEC_BLOCK_SIZE);
    const size_t src = (head * SPEC_BLOCK_SIZE + slot) * d + (size_t)g * 8;
    const uint4 kk = *reinterpret_cast<const uint4 *>(src_k + src);
    *reinterpret_cast<uint4 *>(dst_k + ((head * groups + g) * SPEC_BLOCK_SIZE + slot) * 8) = kk;
    for (int e = 0; e < 8; ++e) dst_v[head * d * SPEC_BLOCK_SIZE + v_tiled_offset(g * 8 + e, slot)] = src_v[src + e];
}

// KV append: one thread per (packed row, kv head, group of 8 elements).
template <typename T>
__global__ void kv_append_kernel(KvAppendParams p)
{
    const int groups = p.d >> 3;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t total = (size_t)p.T * p.Hkv * groups;
    if (idx >= total) return;
    const int g = (int)(idx % groups);
    const int kvh = (int)((idx / groups) % p.Hkv);
    const int row = (int)(idx / ((size_t)groups * p.Hkv));
    const int b = find_request(p.cu_q_len, p.B, p.T, row);
    const int q_len = p.cu_q_len[b + 1] - p.cu_q_len[b];
    const int pos = p.kv_len[b] - q_len + (row - p.cu_q_len[b]);
    // position and page index come from device memory: a row that would land outside the
    // request's block-table row or outside the pool is not written, and counted
    int page = -1;
    if (pos >= 0 && pos / SPEC_BLOCK_SIZE < p.max_blocks_per_req)
        page = p.block_table[(size_t)b * p.max_blocks_per_req + pos / SPEC_BLOCK_SIZE];
    if ((unsigned)page >= (unsigned)p.num_blocks) {
        if (g == 0 && kvh == 0 && p.errors != nullptr) atomicAdd(p.errors, 1ull);
        return;
    }
    const int slot = pos % SPEC_BLOCK_SIZE;
    const T *sk = static_cast<const T *>(p.new_k) + ((size_t)row * p.Hkv + kvh) * p.d + g * 8;
    const T *sv = static_cast<const T *>(p.new_v) + ((size_t)row * p.Hkv + kvh) * p.d + g * 8;
    T *dk = static_cast<T *>(p.k_cache);
    T *dv = static_cast<T *>(p.v_cache);
    // the 8 elements of a thread are contiguous in the cache in every case but one (V in the tiled
    // layout, where consecutive dims of a token are 16 bytes apart): whole-vector stores where they are
    struct alignas(8 * sizeof(T)) Vec8 { T e[8]; };
    *reinterpret_cast<Vec8 *>(dk + k_index(p.kv_layout, page, p.Hkv, kvh, slot, g * 8, p.d)) = *reinterpret_cast<const Vec8 *>(sk);
    if (p.kv_layout == SPEC_KV_TOKEN_MAJOR) {
        *reinterpret_cast<Vec8 *>(dv + v_index(p.kv_layout, page, p.Hkv, kvh, slot, g * 8, p.d)) = *reinterpret_cast<const Vec8 *>(sv);
    } else {
        const Vec8 v = *reinterpret_cast<const Vec8 *>(sv);
#pragma unroll
        for (int e = 0; e < 8; ++e) dv[v_index(p.kv_layout, page, p.Hkv, kvh, slot, g * 8 + e, p.d)] = v.e[e];
    }
}

}  // namespace

hipError_t launch_kv_append(const KvAppendParams &p, hipStream_t stream)
{
    const size_t total = (size_t)p.T * p.Hkv * (p.d >> 3);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (p.elem_bytes == 4)
        hipLaunchKernelGGL(kv_append_kernel<float>, dim3(blocks), dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL(kv_append_kernel<uint16_t>, dim3(blocks), dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_attn_generic(const AttnParams &p, int dtype, hipStream_t stream)
{
    dim3 grid(p.max_chunks, p.Hq, p.T);
    if (dtype == SPEC_F32)
        hipLaunchKernelGGL(attn_generic_kernel<float>, grid, dim3(kChunkThreads), 0, stream, p);
    else
        hipLaunchKernelGGL(attn_generic_kernel<uint16_t>, grid, dim3(kChunkThreads), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_attn_combine(const AttnParams &p, hipStream_t stream)
{
    hipLaunchKernelGGL(attn_combine_kernel, dim3(p.T * p.Hq), dim3(p.d), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_kv_repack(const void *src_k, const void *src_v, void *dst_k, void *dst_v, int32_t num_blocks,
                            int32_t Hkv, int32_t d, hipStream_t stream)
{
    const size_t heads = (size_t)num_blocks * Hkv;
    const size_t total = heads * SPEC_BLOCK_SIZE * (d >> 3);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(kv_repack_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<const uint16_t *>(src_k),
                       static_cast<const uint16_t *>(src_v), static_cast<uint16_t *>(dst_k),
                       static_cast<uint16_t *>(dst_v), heads, d);
    return hipGetLastError();
}

}  // namespace specv
