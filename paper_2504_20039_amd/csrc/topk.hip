// Top-K lossy baseline (Section 4, "Our baselines": a mismatching draft token is accepted when it is
// within the top-K most likely tokens of the target model).  Two small kernels around the LM-head pass:
//   before: the logit of each slot's draft token (one dot product per verify row), which the LM-head
//           kernels then compare every logit of the row against while it is still in registers;
//   after : per window, reduce the per-block maxima (greedy token) and the per-block counts (rank of
//           the draft token), find the first slot whose rank is not below top_k, emit.
#include "aj_internal.h"

namespace aj {

namespace {

constexpr int TK_WAVES = 16;
constexpr int MAXK = 1023;

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// thr[r] = hidden_t[r] . W_lm[draft token of row r], fp32 accumulation; +inf and token -1 for the bonus
// row of a window and for a token outside the vocabulary.  One wave per verify row.
template <bool BF16>
__global__ __launch_bounds__(256) void k_draft_logit(TopkArgs a)
{
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= a.B * (a.K + 1)) return;
    const int b = r / (a.K + 1), j = r - b * (a.K + 1);
    int32_t tok = j < a.K ? a.draft_tok[(size_t)b * a.K + j] : -1;
    if (tok < 0 || tok >= a.V) tok = -1;
    float acc = 0.f;
    if (tok >= 0) {
        const size_t es = BF16 ? 2 : 4;
        const u32x4 *x = (const u32x4 *)((const char *)a.hidden_t + (size_t)r * a.d_t * es);
        const u32x4 *w = (const u32x4 *)((const char *)a.W_lm + (size_t)tok * a.d_t * es);
        const int nchunks = a.d_t / (BF16 ? 8 : 4);
        for (int c = lane; c < nchunks; c += 64) {
            const u32x4 xv = x[c], wv = w[c];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (BF16) {
                    acc = fmaf(bf16_lo(xv[q]), bf16_lo(wv[q]), acc);
                    acc = fmaf(bf16_hi(xv[q]), bf16_hi(wv[q]), acc);
                } else {
                    acc = fmaf(__uint_as_float(xv[q]), __uint_as_float(wv[q]), acc);
                }
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    }
    if (lane == 0) {
        a.thr[r] = tok >= 0 ? acc : INFINITY;
        a.thr_tok[r] = tok;
    }
}

// One workgroup per window.  Phase 1: a wave per verify row reduces the row's block maxima (lowest
// index among equals) and sums its block counts.  Phase 2: wave 0 finds the first rejected slot.
__global__ __launch_bounds__(TK_WAVES * 64) void k_topk_tail(TopkArgs a)
{
    __shared__ int32_t s_t[MAXK + 1];
    __shared__ uint8_t s_rej[MAXK + 1];
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int K = a.K, R = K + 1;

    for (int j = wave; j < R; j += TK_WAVES) {
        const size_t row = (size_t)b * R + j;
        const Best *p = a.part + row * a.nblocks;
        const int32_t *c = a.cnt + row * a.nblocks;
        float bv = -INFINITY;
        int32_t bi = 0x7fffffff, cn = 0;
        for (int nb0 = lane; nb0 < a.nblocks; nb0 += 256) {       // 4 loads in flight per lane
            Best x[4];
            int32_t y[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int nb = nb0 + 64 * u;
                x[u] = nb < a.nblocks ? p[nb] : Best{-INFINITY, 0x7fffffff};
                y[u] = nb < a.nblocks ? c[nb] : 0;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (better(x[u].v, x[u].i, bv, bi)) {
                    bv = x[u].v;
                    bi = x[u].i;
                }
                cn += y[u];
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const float ov = __shfl_xor(bv, off);
            const int32_t oi = __shfl_xor(bi, off);
            if (better(ov, oi, bv, bi)) {
                bv = ov;
                bi = oi;
            }
            cn += __shfl_xor(cn, off);
        }
        if (lane == 0) {
            // a token outside the vocabulary is in no top-k: rank V.  The greedy token itself has rank 0 by
            // definition (top_k = 1 is greedy verification): its threshold logit comes from a separate dot product
            // whose rounding differs from the MFMA accumulation, so a runner-up within that rounding could otherwise
            // be counted before it.
            const int32_t tk = j < K ? a.thr_tok[row] : -1;
            const int32_t rank = j < K ? (tk < 0 ? a.V : (tk == bi ? 0 : cn)) : 0;
            s_t[j] = bi;
            s_rej[j] = j < K && !(rank < a.top_k);
            a.t_star[row] = bi;
            a.maxlogit[row] = bv;
            a.rank[row] = rank;
        }
    }
    __syncthreads();

    if (wave == 0) {
        int n = K;
        for (int base = 0; base < K; base += 64) {
            const int j = base + lane;
            const bool r = j < K && s_rej[j];
            const unsigned long long m = __ballot(r);
            if (m) {
                n = base + __builtin_ctzll(m);
                break;
            }
        }
        if (lane == 0) {
            a.out_len[b] = n;
            a.out_tok[b] = s_t[n];
        }
    }
}

}  // namespace

hipError_t topk_draft_logit(const TopkArgs &a, hipStream_t s)
{
    const int M = a.B * (a.K + 1);
    if (M <= 0) return hipSuccess;
    if (a.dtype == 1) hipLaunchKernelGGL(k_draft_logit<true>, dim3((M + 3) / 4), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(k_draft_logit<false>, dim3((M + 3) / 4), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t topk_tail(const TopkArgs &a, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_topk_tail, dim3(a.B), dim3(TK_WAVES * 64), 0, s, a);
    return hipGetLastError();
}

}  // namespace aj
