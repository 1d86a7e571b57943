// Steps 2 (second half) to 4: cross-block greedy maximum, mismatch test + judge, first-reject scan.
#include "aj_internal.h"

namespace aj {

namespace {

// ---------------------------------------------------------------- step 2: reduce the block partials
// 64 verify rows per workgroup, 4 threads per row each scanning every 4th vocabulary block;
// reads are coalesced over rows (partials are stored [block][row]).
__global__ __launch_bounds__(256) void k_argmax_reduce(const float *pval, const int32_t *pidx, int nblocks,
                                                       int M, int32_t *t_star, float *maxlogit)
{
    __shared__ float sv[4][64];
    __shared__ int32_t si[4][64];
    const int rl = threadIdx.x & 63, sl = threadIdx.x >> 6;
    const int row = blockIdx.x * 64 + rl;
    float bv = -INFINITY;
    int32_t bi = 0x7fffffff;
    if (row < M) {
        for (int nb = sl; nb < nblocks; nb += 4) {
            float v = pval[(size_t)nb * M + row];
            int32_t i = pidx[(size_t)nb * M + row];
            if (better(v, i, bv, bi)) {
                bv = v;
                bi = i;
            }
        }
    }
    sv[sl][rl] = bv;
    si[sl][rl] = bi;
    __syncthreads();
    if (sl == 0 && row < M) {
#pragma unroll
        for (int s = 1; s < 4; ++s)
            if (better(sv[s][rl], si[s][rl], bv, bi)) {
                bv = sv[s][rl];
                bi = si[s][rl];
            }
        t_star[row] = bi;
        maxlogit[row] = bv;
    }
}

// ---------------------------------------------------------------- steps 3-4
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// wave-wide partial dot of n elements (n % 8 == 0 for bf16, % 4 for f32), fp32 accumulation
template <bool BF16>
__device__ __forceinline__ float dot_part(const void *x, const void *w, int n, int lane)
{
    float acc = 0.f;
    if (BF16) {
        const u32x4 *xp = (const u32x4 *)x, *wp = (const u32x4 *)w;
        for (int c = lane; c < n / 8; c += 64) {
            u32x4 xv = xp[c], wv = wp[c];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                acc = fmaf(bf16_lo(xv[q]), bf16_lo(wv[q]), acc);
                acc = fmaf(bf16_hi(xv[q]), bf16_hi(wv[q]), acc);
            }
        }
    } else {
        const f32x4 *xp = (const f32x4 *)x, *wp = (const f32x4 *)w;
        for (int c = lane; c < n / 4; c += 64) {
            f32x4 xv = xp[c], wv = wp[c];
#pragma unroll
            for (int q = 0; q < 4; ++q) acc = fmaf(xv[q], wv[q], acc);
        }
    }
    return acc;
}

// One workgroup per window.  Each wave takes every 4th slot; at a mismatching slot (a
// wave-uniform condition) its 64 lanes share the judge dot product and reduce it with
// cross-lane shuffles.  Wave 0 then finds the first rejected slot with ballots.
template <bool BF16>
__global__ __launch_bounds__(256) void k_judge_scan(TailArgs a)
{
    __shared__ uint8_t rej[1024];
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int K = a.K, R = K + 1;
    const size_t es = BF16 ? 2 : 4;
    const int32_t *t = a.t_star + (size_t)b * R;
    for (int j = wave; j < K; j += 4) {
        const bool mis = t[j] != a.draft_tok[(size_t)b * K + j];
        float z = __builtin_nanf("");
        bool r = false;
        if (mis) {
            const size_t row = (size_t)b * R + j + a.feat_offset;
            float acc = dot_part<BF16>((const char *)a.hidden_t + row * a.d_t * es, a.clf_w, a.d_t, lane);
            if (a.d_d > 0)
                acc += dot_part<BF16>((const char *)a.hidden_d + row * a.d_d * es,
                                      (const char *)a.clf_w + (size_t)a.d_t * es, a.d_d, lane);
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
            z = acc + a.clf_b;
            r = !(z < a.zthr);
        }
        if (lane == 0) {
            rej[j] = r;
            if (a.score) {
                a.score[(size_t)b * K + j] = z;
                a.score[(size_t)a.B * K + (size_t)b * K + j] = 1.f / (1.f + __expf(-z));
            }
        }
    }
    __syncthreads();
    if (wave == 0) {
        int n = K;
        for (int base = 0; base < K; base += 64) {
            const int j = base + lane;
            const bool r = j < K && rej[j];
            const unsigned long long m = __ballot(r);
            if (m) {
                n = base + __builtin_ctzll(m);
                break;
            }
        }
        if (lane == 0) {
            a.out_len[b] = n;
            a.out_tok[b] = t[n];
        }
    }
}

}  // namespace

hipError_t argmax_reduce(const TailArgs &a, hipStream_t s)
{
    const int M = a.B * (a.K + 1);
    if (M <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_argmax_reduce, dim3((M + 63) / 64), dim3(256), 0, s, a.pval, a.pidx, a.nblocks, M,
                       a.t_star, a.maxlogit);
    return hipGetLastError();
}

hipError_t judge_scan(const TailArgs &a, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    if (a.dtype == 1)
        hipLaunchKernelGGL(k_judge_scan<true>, dim3(a.B), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(k_judge_scan<false>, dim3(a.B), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace aj
