// LM head + per-block greedy maximum for fp32 storage: plain FMA tiles (the fp32 workload is a
// tiny latency-bound case; the matrix cores are used by the bf16 kernels).
// One workgroup: 64 vocabulary rows x 16 verify rows; a wave owns 4 verify rows, its 64 lanes the
// 64 vocabulary rows, so the per-row maximum is one wave reduction.
#include "aj_internal.h"

namespace aj {

namespace {

constexpr int FBN = 64, FBM = 16, FBK = 32;

template <bool DUMP>
__global__ __launch_bounds__(256) void k_lm_head_f32(LmHeadArgs a)
{
    __shared__ float sW[FBN][FBK + 1];
    __shared__ float sH[FBM][FBK + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.x * FBM, v0 = blockIdx.y * FBN;
    const float *W = (const float *)a.W, *H = (const float *)a.H;
    const int d = a.d;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < d; k0 += FBK) {
        __syncthreads();
        for (int c = tid; c < FBN * FBK; c += 256) {
            int r = c / FBK, k = c % FBK;
            sW[r][k] = (v0 + r < a.V && k0 + k < d) ? W[(size_t)(v0 + r) * d + k0 + k] : 0.f;
        }
        for (int c = tid; c < FBM * FBK; c += 256) {
            int r = c / FBK, k = c % FBK;
            sH[r][k] = (m0 + r < a.M && k0 + k < d) ? H[(size_t)(m0 + r) * d + k0 + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < FBK; ++k) {
            float w = sW[lane][k];
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = fmaf(w, sH[wave * 4 + i][k], acc[i]);
        }
    }
    const int v = v0 + lane;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = m0 + wave * 4 + i;
        if (DUMP && v < a.V && row < a.M) a.dump[(size_t)row * a.V + v] = acc[i];
        if (a.key && row < a.M && v < a.V) {     // sampling mode: logit / T + Gumbel noise(row key, v)
            const uint64_t key = a.key[row];
            acc[i] = fmaf(acc[i], a.inv_temp, gumbel_noise((uint32_t)key, (uint32_t)(key >> 32), (uint32_t)v));
        }
        float bv = v < a.V ? acc[i] : -INFINITY;
        int32_t bi = v < a.V ? v : 0x7fffffff;
        // top-K baseline: is this lane's entry ordered before the row's draft token?
        int32_t cn = 0;
        if (a.thr && row < a.M && v < a.V) cn = ranks_before(acc[i], v, a.thr[row], a.thr_tok[row]);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            float ov = __shfl_xor(bv, off);
            int32_t oi = __shfl_xor(bi, off);
            if (better(ov, oi, bv, bi)) {
                bv = ov;
                bi = oi;
            }
            cn += __shfl_xor(cn, off);
        }
        if (lane == 0 && row < a.M) {
            a.part[(size_t)row * a.nblocks + blockIdx.y] = Best{bv, bi};
            if (a.cnt) a.cnt[(size_t)row * a.nblocks + blockIdx.y] = cn;
        }
    }
}

}  // namespace

int lm_head_f32_blocks(int V) { return (V + FBN - 1) / FBN; }

hipError_t lm_head_f32(const LmHeadArgs &a, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    dim3 grid((a.M + FBM - 1) / FBM, lm_head_f32_blocks(a.V));
    if (a.dump)
        hipLaunchKernelGGL(k_lm_head_f32<true>, grid, dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(k_lm_head_f32<false>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace aj
