// Lookahead attention over a bf16 paged KV cache with gfx950 matrix
// instructions (Section 2.2 / Section 4 of arXiv 2406.14066: the k+1 query
// positions of a request are scored in one pass against its cached keys and
// values; Eq. 3 names the KV-cache read as the context-dependent cost, and this
// kernel is built to be bound by exactly that read).
//
// One block = (request b, KV head, chunk of the KV length); its four wavefronts
// take the chunk's 16-token pages round-robin.  All q_len * (Hq/Hkv) query rows
// that share the KV head are fused into the N dimension of the matrix
// instructions, so every K and V byte of the request is read from HBM once.
//
// Per page and per 16-row tile (lane = 16*g + n, n = query row, g = 0..3):
//   S^T[token][row] = K[token][:] . Q[row][:]      4 x v_mfma_f32_16x16x32_bf16
//        (A = K page, lane holds token n, dims 8g..8g+7 of each 32-dim step;
//         the SPEC_KV_MFMA page layout makes that one contiguous 1 KB load)
//   online softmax in base 2 on the lane's four tokens 4g..4g+3 of its row
//   O^T[dim][row] += V^T[dim][token] . P^T[token][row]   8 x v_mfma_f32_16x16x16_bf16
//        (B = P^T is S^T's own accumulator layout, no shuffle; P is fed as a
//         bf16 high part plus a bf16 low part so its rounding does not limit the
//         result; A = V page, again one contiguous 1 KB load per two dim tiles)
// Next page's loads are issued before the current page's arithmetic.
// The four wavefronts' states are merged through LDS and the block writes one
// partial (acc, m, l) per query row, merged across chunks by the combine kernel.
#include "common.h"

#include <math.h>

namespace specv {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kD = 128;
constexpr int kPageHeadBytes = SPEC_BLOCK_SIZE * kD * 2;  // 4096

struct PageRegs {
    u32x4 k[4];  // k[kk]: token n, dims 32*kk + 8g .. +7
    u32x4 v[4];  // v[pp]: dims 32*pp + n (low half) and 32*pp + 16 + n (high half), tokens 4g .. 4g+3
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float group_max(float v)
{
    v = fmaxf(v, __shfl_xor(v, 16));
    v = fmaxf(v, __shfl_xor(v, 32));
    return v;
}

template <int NT, bool SPLIT_P>
__global__ __launch_bounds__(kThreads, 2) void attn_mfma_kernel(AttnParams p)
{
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int n16 = lane & 15;
    const int g = lane >> 4;
    const int chunk = blockIdx.x;
    const int kvh = blockIdx.y;
    const int b = blockIdx.z;

    const int L = p.kv_len[b];
    const int C = p.chunk_tokens;
    const int nchunks = (L + C - 1) / C;
    if (chunk >= nchunks) return;
    const int row0 = p.cu_q_len[b];
    const int q_len = p.cu_q_len[b + 1] - row0;
    const int group = p.Hq / p.Hkv;
    const int rows = q_len * group;
    const int tok0 = chunk * C;
    const int tok1 = min(L, tok0 + C);
    const int npages = (tok1 - tok0 + SPEC_BLOCK_SIZE - 1) / SPEC_BLOCK_SIZE;  // <= 64
    const int page0 = tok0 / SPEC_BLOCK_SIZE;

    // this chunk's slice of the block table, one entry per lane
    int bt = 0;
    if (lane < npages) bt = p.block_table[(size_t)b * p.max_blocks_per_req + page0 + lane];

    // Q as the B operand of S^T = K Q^T, and each lane's last visible key
    bf16x8 qreg[NT][4];
    int limit[NT];
    int out_row[NT];   // packed (token row * Hq + head) of this lane's query row, -1 if padding
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int r = nt * 16 + n16;
        const bool valid = r < rows;
        const int j = valid ? r / group : 0;
        const int gq = valid ? r % group : 0;
        const size_t rh = (size_t)(row0 + j) * p.Hq + kvh * group + gq;
        const __bf16 *qp = static_cast<const __bf16 *>(p.q) + rh * kD + g * 8;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
            qreg[nt][kk] = valid ? *reinterpret_cast<const bf16x8 *>(qp + kk * 32) : z;
        }
        limit[nt] = valid ? L - q_len + j : -1;
        out_row[nt] = valid ? (int)rh : -1;
    }

    const char *kbase = static_cast<const char *>(p.k_cache) + (size_t)kvh * kPageHeadBytes + lane * 16;
    const char *vbase = static_cast<const char *>(p.v_cache) + (size_t)kvh * kPageHeadBytes + lane * 16;
    const size_t page_stride = (size_t)p.Hkv * kPageHeadBytes;

    auto load_page = [&](int pi, PageRegs &r) {
        if (pi < npages) {
            const int page = __builtin_amdgcn_readlane(bt, pi);
            const char *kp = kbase + (size_t)page * page_stride;
            const char *vp = vbase + (size_t)page * page_stride;
#pragma unroll
            for (int i = 0; i < 4; ++i) r.k[i] = *reinterpret_cast<const u32x4 *>(kp + i * 1024);
#pragma unroll
            for (int i = 0; i < 4; ++i) r.v[i] = *reinterpret_cast<const u32x4 *>(vp + i * 1024);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                r.k[i] = (u32x4){0, 0, 0, 0};
                r.v[i] = (u32x4){0, 0, 0, 0};
            }
        }
    };

    f32x4 acc[NT][8];
    float m_run[NT], l_run[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m_run[nt] = kEmptyMax;
        l_run[nt] = 0.0f;
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) acc[nt][mt] = (f32x4){0.0f, 0.0f, 0.0f, 0.0f};
    }

    const int first_masked_token = L - q_len + 1;  // keys from here on are hidden from some row (or past the end)

    PageRegs cur;
    load_page(wave, cur);
    for (int pi = wave; pi < npages; pi += 4) {
        PageRegs nxt;
        load_page(pi + 4, nxt);

        const int page_tok = tok0 + pi * SPEC_BLOCK_SIZE;
        const bool need_mask = page_tok + SPEC_BLOCK_SIZE > first_masked_token;
        const int tbase = page_tok + 4 * g;

        if (page_tok + SPEC_BLOCK_SIZE > L) {
            // last page of the request: slots past kv_len may hold anything; clear their V
            const int nvalid = min(max(L - tbase, 0), 4);
            const uint32_t lo = nvalid >= 2 ? 0xFFFFFFFFu : (nvalid == 1 ? 0x0000FFFFu : 0u);
            const uint32_t hi = nvalid >= 4 ? 0xFFFFFFFFu : (nvalid == 3 ? 0x0000FFFFu : 0u);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                cur.v[i].x &= lo; cur.v[i].y &= hi;
                cur.v[i].z &= lo; cur.v[i].w &= hi;
            }
        }

#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            f32x4 s = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, cur.k[kk]), qreg[nt][kk], s, 0, 0, 0);
            s *= p.scale_log2;
            if (need_mask) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (tbase + r > limit[nt]) s[r] = -INFINITY;
            }
            const float mx = group_max(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])));
            const float m_new = fmaxf(m_run[nt], mx);
            const float alpha = fast_exp2(m_run[nt] - m_new);
            f32x4 pr;
#pragma unroll
            for (int r = 0; r < 4; ++r) pr[r] = fast_exp2(s[r] - m_new);
            l_run[nt] = l_run[nt] * alpha + ((pr[0] + pr[1]) + (pr[2] + pr[3]));
            m_run[nt] = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int mt = 0; mt < 8; ++mt) acc[nt][mt] *= alpha;
            }
            const bf16x4 p_hi = __builtin_convertvector(pr, bf16x4);
            bf16x4 p_lo;
            if (SPLIT_P) p_lo = __builtin_convertvector(pr - __builtin_convertvector(p_hi, f32x4), bf16x4);
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) {
                const u32x4 vv = cur.v[mt >> 1];
                const u32x2 half = (mt & 1) ? (u32x2){vv.z, vv.w} : (u32x2){vv.x, vv.y};
                const bf16x4 va = __builtin_bit_cast(bf16x4, half);
                acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, p_hi, acc[nt][mt], 0, 0, 0);
                if (SPLIT_P) acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, p_lo, acc[nt][mt], 0, 0, 0);
            }
        }
        cur = nxt;
    }

    // each lane summed its own four tokens per page: finish the row sums
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        l_run[nt] += __shfl_xor(l_run[nt], 16);
        l_run[nt] += __shfl_xor(l_run[nt], 32);
    }

    // merge the four wavefronts: 2,3 -> 0,1 then 1 -> 0
    __shared__ f32x4 sh_acc[2][NT][8][kWave];
    __shared__ float sh_m[2][NT][kWave];
    __shared__ float sh_l[2][NT][kWave];
    auto put = [&](int buf) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) sh_acc[buf][nt][mt][lane] = acc[nt][mt];
            sh_m[buf][nt][lane] = m_run[nt];
            sh_l[buf][nt][lane] = l_run[nt];
        }
    };
    auto merge = [&](int buf) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const float mo = sh_m[buf][nt][lane];
            const float lo = sh_l[buf][nt][lane];
            const float mn = fmaxf(m_run[nt], mo);
            const float wa = fast_exp2(m_run[nt] - mn);
            const float wb = fast_exp2(mo - mn);
            l_run[nt] = l_run[nt] * wa + lo * wb;
            m_run[nt] = mn;
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) acc[nt][mt] = acc[nt][mt] * wa + sh_acc[buf][nt][mt][lane] * wb;
        }
    };
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) merge(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave != 0) return;
    merge(0);

    // one partial per query row: acc[dim], running max, running sum
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        if (out_row[nt] < 0) continue;
        const size_t slot = (size_t)out_row[nt] * p.max_chunks + chunk;
        float *dst = p.ws_acc + slot * kD + 4 * g;
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) *reinterpret_cast<f32x4 *>(dst + 16 * mt) = acc[nt][mt];
        if (g == 0) {
            p.ws_ml[slot * 2 + 0] = m_run[nt];
            p.ws_ml[slot * 2 + 1] = l_run[nt];
        }
    }
}

}  // namespace

hipError_t launch_attn_mfma(const AttnParams &p, int row_tiles, hipStream_t stream)
{
    if (p.d != kD || p.chunk_tokens > 1024 || p.chunk_tokens % SPEC_BLOCK_SIZE != 0) return hipErrorInvalidValue;
    dim3 grid(p.max_chunks, p.Hkv, p.B);
    switch (row_tiles) {
        case 1: hipLaunchKernelGGL((attn_mfma_kernel<1, true>), grid, dim3(kThreads), 0, stream, p); break;
        case 2: hipLaunchKernelGGL((attn_mfma_kernel<2, true>), grid, dim3(kThreads), 0, stream, p); break;
        case 3: hipLaunchKernelGGL((attn_mfma_kernel<3, true>), grid, dim3(kThreads), 0, stream, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace specv
