// LM head (step 1) fused with the per-vocabulary-block greedy maximum (first half of step 2):
// general-shape bf16 MFMA kernel.  One workgroup owns a 128 (vocabulary) x 128 (verify rows)
// tile of logits, accumulates it over d_t with v_mfma_f32_32x32x16_bf16 from LDS-staged
// operand tiles, and reduces it to one (max, lowest index) pair per verify row.  The logits
// themselves stay in registers.
//
// MFMA roles: A = W_lm tile (row i = vocabulary index), B = hidden_t tile (column j = verify
// row), so D[i][j] = logit[verify row j][vocabulary i].  A lane then owns ONE verify row
// (j = lane % 32) and 16 vocabulary entries per 32x32 block, which makes the running
// (max, index) of a row a purely in-lane scan in ascending vocabulary order; only the two
// lane halves and the two vocabulary halves of the tile are combined at the very end.
#include "aj_internal.h"

namespace aj {

namespace {

constexpr int BN = 128;      // vocabulary rows per workgroup
constexpr int BM = 128;      // verify rows per workgroup
constexpr int BK = 32;       // k elements per LDS stage
constexpr int LSTR = BK + 8; // LDS row stride in elements (80 B: conflict-free 16-byte fragment reads)

template <bool DUMP>
__global__ __launch_bounds__(256) void k_lm_head_tile(LmHeadArgs a)
{
    __shared__ __attribute__((aligned(16))) uint16_t sW[BN * LSTR];
    __shared__ __attribute__((aligned(16))) uint16_t sH[BM * LSTR];
    __shared__ float red_v[BM];
    __shared__ int32_t red_i[BM];
    __shared__ int32_t red_c[BM];     // top-K baseline: counts of the second wave column

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wv = wave & 1, wh = wave >> 1;     // wave's vocabulary half / verify-row half
    const int i32 = lane & 31, kh = lane >> 5;
    const int m0 = blockIdx.x * BM, v0 = blockIdx.y * BN;
    const int d = a.d;
    const uint16_t *W = (const uint16_t *)a.W, *H = (const uint16_t *)a.H;

    // global -> LDS loader: the tile is 128 rows x 4 chunks of 8 elements; 2 chunks per thread
    const uint16_t *wp[2], *hp[2];
    int lds_off[2], kc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        int c = tid + i * 256, row = c >> 2;
        kc[i] = (c & 3) * 8;
        int vr = min(v0 + row, a.V - 1), mr = min(m0 + row, a.M - 1);   // clamped: stays in bounds
        wp[i] = W + (size_t)vr * d + kc[i];
        hp[i] = H + (size_t)mr * d + kc[i];
        lds_off[i] = row * LSTR + kc[i];
    }
    u32x4 rw[2], rh[2];
    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (k0 + kc[i] < d) {               // d % 8 == 0: a chunk is wholly inside or outside
                rw[i] = *(const u32x4 *)(wp[i] + k0);
                rh[i] = *(const u32x4 *)(hp[i] + k0);
            } else {
                rw[i] = u32x4{0, 0, 0, 0};
                rh[i] = u32x4{0, 0, 0, 0};
            }
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

    gload(0);
    for (int k0 = 0; k0 < d; k0 += BK) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            *(u32x4 *)(sW + lds_off[i]) = rw[i];
            *(u32x4 *)(sH + lds_off[i]) = rh[i];
        }
        __syncthreads();
        if (k0 + BK < d) gload(k0 + BK);
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                fa[x] = *(const bf16x8 *)(sW + (wv * 64 + x * 32 + i32) * LSTR + s * 16 + kh * 8);
                fb[x] = *(const bf16x8 *)(sH + (wh * 64 + x * 32 + i32) * LSTR + s * 16 + kh * 8);
            }
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y)
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[x], fb[y], acc[x][y], 0, 0, 0);
        }
    }

    // epilogue: D register r of a lane is vocabulary row 8*(r/4) + 4*(lane/32) + r%4 of the block
#pragma unroll
    for (int y = 0; y < 2; ++y) {
        const int row = m0 + wh * 64 + y * 32 + i32;
        float bv = -INFINITY;
        int32_t bi = 0x7fffffff;
        // top-K baseline: the row's draft token and the number of this block's entries ordered before it
        float th = INFINITY;
        int32_t tk = -1, cn = 0;
        if (a.thr && row < a.M) {
            th = a.thr[row];
            tk = a.thr_tok[row];
        }
        uint32_t klo = 0, khi = 0;      // sampling mode: the row's noise key
        const bool sample = a.key != nullptr;
        if (sample && row < a.M) {
            klo = (uint32_t)a.key[row];
            khi = (uint32_t)(a.key[row] >> 32);
        }
#pragma unroll
        for (int x = 0; x < 2; ++x) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int v = v0 + wv * 64 + x * 32 + (r >> 2) * 8 + kh * 4 + (r & 3);
                float val = acc[x][y][r];
                if (v < a.V) {
                    if (DUMP && row < a.M) a.dump[(size_t)row * a.V + v] = val;
                    if (sample) val = fmaf(val, a.inv_temp, gumbel_noise(klo, khi, (uint32_t)v));
                    if (val > bv) {          // ascending v inside a lane: strict keeps the lowest
                        bv = val;
                        bi = v;
                    }
                    cn += ranks_before(val, v, th, tk);
                }
            }
        }
        float ov = __shfl_xor(bv, 32);
        int32_t oi = __shfl_xor(bi, 32);
        if (better(ov, oi, bv, bi)) {
            bv = ov;
            bi = oi;
        }
        const int lr = wh * 64 + y * 32 + i32;
        cn += __shfl_xor(cn, 32);
        if (wv == 1 && kh == 0) {
            red_v[lr] = bv;
            red_i[lr] = bi;
            red_c[lr] = cn;
        }
        __syncthreads();
        if (wv == 0 && kh == 0 && row < a.M) {
            if (better(red_v[lr], red_i[lr], bv, bi)) {
                bv = red_v[lr];
                bi = red_i[lr];
            }
            a.part[(size_t)row * a.nblocks + blockIdx.y] = Best{bv, bi};
            if (a.cnt) a.cnt[(size_t)row * a.nblocks + blockIdx.y] = cn + red_c[lr];
        }
        __syncthreads();
    }
}

}  // namespace

int lm_head_tile_blocks(int V) { return (V + BN - 1) / BN; }

hipError_t lm_head_tile_bf16(const LmHeadArgs &a, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    dim3 grid((a.M + BM - 1) / BM, lm_head_tile_blocks(a.V));
    if (a.dump)
        hipLaunchKernelGGL(k_lm_head_tile<true>, grid, dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(k_lm_head_tile<false>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace aj
