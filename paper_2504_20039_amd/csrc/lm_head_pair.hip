// LM head (step 1) + per-vocabulary-block greedy maximum (first half of step 2), MFMA-bound regime:
// 256 vocabulary x 256 verify rows per workgroup, 4 waves of 128 x 128 (4 x 4 blocks of
// v_mfma_f32_32x32x16_bf16, 256 accumulator registers), hand-scheduled like the BIG variant of
// lm_head_mfma.hip, with a different operand pipeline.
//
// What bounds the 256 x 256 tile on this chip is the L2 -> CU path, and that path moves whole 128-byte
// lines: a 64-byte row piece (32 k elements) costs a full line, and asking for the other half one
// pipeline stage later misses the 32 KB L1 again (a stage touches 64 KB of lines).  128-byte pieces
// with the usual "both operands per stage" ring would need 64 KB stages, i.e. only two of them in
// LDS.  Here a TIME STEP still computes 32 k elements (two k steps of 16) of both operands, but the
// loads issued during a time step fetch ONE operand for 64 k elements: both 64-byte halves of each
// line, in adjacent instructions, so that the second half is an L1 hit.  W_lm slabs are issued at odd
// time steps, hidden_t slabs at even ones:
//
//     time step 2j-3 : W slab j   (halves W_j.0, W_j.1)        needed at steps 2j, 2j+1
//     time step 2j-2 : H slab j   (halves H_j.0, H_j.1)        needed at steps 2j, 2j+1
//     time step 2j+h : MFMAs on (W_j.h, H_j.h); its two 16 KB half-buffers are free afterwards
//
// Exactly 8 half-buffers of 16 KB (256 rows x 64 B) are live at any time, the same 128 KB as four
// ordinary stages.  The two buffers freed after step t are the ones the loads of step t+1 (at the
// latest) go to, which makes W_j.1 and H_j.0 trade places every other slab; the assignment repeats
// every 8 time steps (see buf_w / buf_h), so the step body is instantiated for t mod 8 = 0..7 with
// every LDS address a compile-time constant, and d_t must be a multiple of 256.
#include "../../include/aj.h"
#include "aj_internal.h"
#include "lds_pipeline.h"
#include <type_traits>

namespace aj {

namespace {

constexpr int PT = 256;              // tile edge (vocabulary rows and verify rows)
constexpr int HB = PT * 64;          // bytes of a half-buffer: 256 rows x 64 B (32 k elements)
constexpr int LBB = 5;               // loads of a time step that precede its barrier (slots 0..4)

// half-buffer of W_lm / hidden_t read at time step u (mod 8): u = 2*(slab mod 4) + half
constexpr int buf_w(int u)
{
    const int p = (u >> 1) & 1, q = (u >> 2) & 1, h = u & 1;
    return h == 0 ? p : (q ? 5 + 2 * p : 4 + 2 * p);
}
constexpr int buf_h(int u)
{
    const int p = (u >> 1) & 1, q = (u >> 2) & 1, h = u & 1;
    return h == 1 ? 2 + p : (q ? 4 + 2 * p : 5 + 2 * p);
}

template <int U>
using step_c = std::integral_constant<int, U>;

template <bool DUMP, bool TOPK, bool SAMPLE>
__global__ __launch_bounds__(256) void k_lm_head_pair(LmHeadArgs a, Sched sc)
{
    constexpr int TN = 4, TM = 4, NG = 4, GS = 4;
    __shared__ __attribute__((aligned(1024))) char lds[8 * HB];
    __shared__ Best red[PT];
    __shared__ int32_t redc[PT];      // top-K baseline: counts of the second wave column

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wn = wave & 1, wm = wave >> 1;
    const int l32 = lane & 31, kh = lane >> 5;
    const int d = a.d, NBLK = d / 256;     // blocks of 8 time steps per tile (host guarantees d % 256 == 0)
    const char *W = (const char *)a.W, *H = (const char *)a.H;
    const uint32_t rowbytes = (uint32_t)d * 2u;

    const int G = gridDim.x, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, SL = G >> 3;
    auto tile_at = [&](int step) { return (step * 8 + xcd) * SL + slot; };

    // loader: an instruction covers 16 tile rows x 64 B; lane i fills slot (row i/4, chunk i%4) and
    // fetches global chunk (i%4) ^ ((row/4)%4) of its half (conflict-free 16-byte fragment reads)
    const int rl = lane >> 2;
    const uint32_t cg16 = (uint32_t)(((lane & 3) ^ ((rl >> 2) & 3)) * 16);
    const uint32_t lds_w = lds_offset_of(lds) + wave * 1024;      // this wave's 1 KB inside a 4 KB load round
    // fragment reads: lane (row l32, k half kh) of block x reads chunk (2*s + kh) ^ swizzle(row)
    const int swz = (l32 >> 2) & 3;
    const int a_row = (wn * 128 + l32) * 64, b_row = (wm * 128 + l32) * 64;
    const int pos0 = ((0 + kh) ^ swz) * 16, pos1 = ((2 + kh) ^ swz) * 16;

    f32x16 acc[TN][TM];
    bf16x8 fa[2][TN], fb[2][TM];
    uint32_t vw[4], vh[4], vw2[4], vh2[4];   // lane offsets of this wave's 4 row groups: this tile, next tile
    auto tile_offsets = [&](int mt_, int nt_, uint32_t(&ow)[4], uint32_t(&oh)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = (i * 4 + wave) * 16 + rl;
            ow[i] = __umul24(min(nt_ * PT + row, a.V - 1), rowbytes) + cg16;    // clamped: ragged tiles stay in bounds
            oh[i] = __umul24(min(mt_ * PT + row, a.M - 1), rowbytes) + cg16;
        }
    };
    // the 8 loads of one operand slab (k bytes kb .. kb+128 of every tile row) into half-buffers b0, b1
    auto issue_slab = [&](const char *base, const uint32_t(&vo)[4], int kb, int b0, int b1) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            lds_dma_16(base + kb + (i & 1) * 64, vo[i >> 1], lds_w + ((i & 1) ? b1 : b0) * HB + (i >> 1) * 4096);
    };
    // fragments i0..i1 of k step s of half-buffers (bw, bh) into set `to`, in the order fa0, fb0.., fa1..
    auto R = [&](int bw, int bh, int s, int to, int i0, int i1) {
        const int pos = s ? pos1 : pos0;
#pragma unroll
        for (int i = i0; i < i1; ++i) {
            if (i == 0) fa[to][0] = *(const bf16x8 *)(lds + bw * HB + a_row + pos);
            else if (i <= TM) fb[to][i - 1] = *(const bf16x8 *)(lds + bh * HB + b_row + (i - 1) * 2048 + pos);
            else fa[to][i - TM] = *(const bf16x8 *)(lds + bw * HB + a_row + (i - TM) * 2048 + pos);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // One time step.  With one wave per SIMD every instruction that is not an MFMA must sit in the
    // shadow of a running one: the 16 MFMAs of a k step go out in 4 groups of 4, each followed by one
    // load and, after groups 0 and 1 (1 and 2 in the second k step, where the wait + barrier for the
    // next time step comes right after group 1), by half of the next k step's 8 fragment reads.
    // gb: operand base + k offset of the slab this step loads (W at odd steps, hidden_t at even).
    auto time_step = [&](auto uc, const char *gb, const uint32_t(&vo)[4], bool issuing, bool next_step) {
        constexpr int U = decltype(uc)::value, UN = (U + 1) & 7;
        constexpr bool load_w = (U & 1) != 0;
        constexpr int js = load_w ? ((U + 3) >> 1) & 3 : ((U + 2) >> 1) & 3;          // slab (mod 4) being loaded
        constexpr int d0 = load_w ? buf_w(2 * js) : buf_h(2 * js), d1 = load_w ? buf_w(2 * js + 1) : buf_h(2 * js + 1);
        // loads still allowed in flight at the barrier that opens step U+1: its operands are older than
        // this step's loads, and when U+1 is odd also older than the previous step's 8
        constexpr int VM = (UN & 1) ? 8 + LBB : LBB;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int g = 0; g < NG; ++g) {
#pragma unroll
                for (int m = g * GS; m < (g + 1) * GS; ++m)
                    acc[m / TM][m % TM] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[t][m / TM], fb[t][m % TM],
                                                                                  acc[m / TM][m % TM], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (t == 1 && g == 1 && next_step) {
                    if (issuing) wait_vm_lgkm_and_barrier<VM>();
                    else wait_vm_lgkm_and_barrier<0>();      // fewer loads in flight than the constant assumes
                }
                const int rg = t == 1 ? g - 1 : g;
                if (rg == 0 || rg == 1) {
                    if (t == 0) R(buf_w(U), buf_h(U), 1, 1, rg * 4, rg * 4 + 4);
                    else if (next_step) R(buf_w(UN), buf_h(UN), 0, 0, rg * 4, rg * 4 + 4);
                }
                if (issuing) {
                    const int i = t * NG + g;
                    lds_dma_16(gb + (i & 1) * 64, vo[i >> 1], lds_w + ((i & 1) ? d1 : d0) * HB + (i >> 1) * 4096);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    int T = tile_at(0);
    int mt = 0, nt = 0;
    if (T < sc.total) {
        tile_of(sc, T, mt, nt);
        tile_offsets(mt, nt, vw, vh);
        issue_slab(W, vw, 0, buf_w(0), buf_w(1));
        issue_slab(H, vh, 0, buf_h(0), buf_h(1));
        issue_slab(W, vw, 128, buf_w(2), buf_w(3));
        wait_vm_lgkm_and_barrier<8>();                // slab 0 of both operands has landed
        R(buf_w(0), buf_h(0), 0, 0, 0, 8);
    }

    for (int step = 0; T < sc.total; ++step) {
        const int T2 = tile_at(step + 1);
        const bool have_next = T2 < sc.total;
        int mt2 = 0, nt2 = 0;
        if (have_next) {
            tile_of(sc, T2, mt2, nt2);
            tile_offsets(mt2, nt2, vw2, vh2);
        }
#pragma unroll
        for (int x = 0; x < TN; ++x)
#pragma unroll
            for (int y = 0; y < TM; ++y)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

        // blocks of 8 time steps = 4 slabs = 512 bytes of k; all but the last load within this tile
        for (int blk = 0; blk < NBLK - 1; ++blk) {
            const char *Wb = W + blk * 512, *Hb = H + blk * 512;
            time_step(step_c<0>{}, Hb + 128, vh, true, true);
            time_step(step_c<1>{}, Wb + 256, vw, true, true);
            time_step(step_c<2>{}, Hb + 256, vh, true, true);
            time_step(step_c<3>{}, Wb + 384, vw, true, true);
            time_step(step_c<4>{}, Hb + 384, vh, true, true);
            time_step(step_c<5>{}, Wb + 512, vw, true, true);
            time_step(step_c<6>{}, Hb + 512, vh, true, true);
            time_step(step_c<7>{}, Wb + 640, vw, true, true);
        }
        {   // last block: its steps 5..7 load slabs 0, 0, 1 of the next tile, if there is one
            const char *Wb = W + (NBLK - 1) * 512, *Hb = H + (NBLK - 1) * 512;
            time_step(step_c<0>{}, Hb + 128, vh, true, true);
            time_step(step_c<1>{}, Wb + 256, vw, true, true);
            time_step(step_c<2>{}, Hb + 256, vh, true, true);
            time_step(step_c<3>{}, Wb + 384, vw, true, true);
            time_step(step_c<4>{}, Hb + 384, vh, true, true);
            time_step(step_c<5>{}, W, vw2, have_next, true);
            time_step(step_c<6>{}, H, vh2, have_next, true);
            time_step(step_c<7>{}, W + 128, vw2, have_next, have_next);
        }

        // ---- greedy maximum: D register r of a lane = vocabulary row 8*(r/4) + 4*(lane/32) + r%4 of its block
        const int v_base = nt * PT + wn * 128 + kh * 4;
        float pv[TM];
        int32_t pi[TM], pc[TM];
#pragma unroll
        for (int y = 0; y < TM; ++y) {
            const int lr = wm * 128 + y * 32 + l32;          // verify row inside the tile
            const int row = mt * PT + lr;
            float bv = -INFINITY;
            int32_t bi = 0x7fffffff;
            // top-K baseline: the row's draft token and the number of this block's entries ordered before it
            float th = INFINITY;
            int32_t tk = -1, cn = 0;
            if (TOPK && row < a.M) {
                th = a.thr[row];
                tk = a.thr_tok[row];
            }
            uint32_t klo = 0, khi = 0;      // sampling mode: the row's noise key
            if (SAMPLE && row < a.M) {
                klo = (uint32_t)a.key[row];
                khi = (uint32_t)(a.key[row] >> 32);
            }
#pragma unroll
            for (int x = 0; x < TN; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int v = v_base + x * 32 + (r >> 2) * 8 + (r & 3);
                    float val = acc[x][y][r];
                    if (v < a.V) {
                        if (DUMP && row < a.M) a.dump[(size_t)row * a.V + v] = val;
                        if (SAMPLE) val = fmaf(val, a.inv_temp, gumbel_noise(klo, khi, (uint32_t)v));
                        if (val > bv) {      // ascending v inside a lane: strict > keeps the lowest index
                            bv = val;
                            bi = v;
                        }
                        if (TOPK) cn += ranks_before(val, v, th, tk);
                    }
                }
            if (TOPK) cn += __shfl_xor(cn, 32);
            const float ov = __shfl_xor(bv, 32);
            const int32_t oi = __shfl_xor(bi, 32);
            if (better(ov, oi, bv, bi)) {
                bv = ov;
                bi = oi;
            }
            if (wn > 0 && kh == 0) {
                red[lr] = Best{bv, bi};
                if (TOPK) redc[lr] = cn;
            }
            pv[y] = bv;
            pi[y] = bi;
            pc[y] = cn;
        }
        // LDS writes of `red` done and visible; do not wait for the prefetch loads in flight
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (wn == 0 && kh == 0) {
#pragma unroll
            for (int y = 0; y < TM; ++y) {
                const int lr = wm * 128 + y * 32 + l32;
                const int row = mt * PT + lr;
                float bv = pv[y];
                int32_t bi = pi[y];
                const Best o = red[lr];
                if (better(o.v, o.i, bv, bi)) {
                    bv = o.v;
                    bi = o.i;
                }
                if (row < a.M) a.part[(size_t)row * a.nblocks + nt] = Best{bv, bi};
                if (TOPK && row < a.M) a.cnt[(size_t)row * a.nblocks + nt] = pc[y] + redc[lr];
            }
        }
        // `red` is next written after the barriers of the following tile's time steps: no extra barrier
        if (have_next) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                vw[i] = vw2[i];
                vh[i] = vh2[i];
            }
        }
        T = T2;
        mt = mt2;
        nt = nt2;
    }
}

}  // namespace

int lm_head_pair_blocks(int V) { return (V + PT - 1) / PT; }

int lm_head_pair_padded_rows(int M) { return (M + PT - 1) / PT * PT; }

bool lm_head_pair_supports(int M, int V, int d)
{
    if (M <= 0 || V <= 0 || d < 256 || d % 256 != 0) return false;
    // lane offsets are 32-bit and row indices go through a 24-bit multiply
    if ((uint64_t)V * d * 2 >= (1ull << 32) || (uint64_t)M * d * 2 >= (1ull << 32)) return false;
    return V < (1 << 24) && M < (1 << 24) && d * 2 < (1 << 24);
}

hipError_t lm_head_pair_bf16(const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    Sched sc;
    sc.tiles_m = (a.M + PT - 1) / PT;
    sc.tiles_n = (a.V + PT - 1) / PT;
    sc.gm = sc.tiles_m < 8 ? sc.tiles_m : 8;
    sc.total = sc.tiles_m * sc.tiles_n;
    const int grid = persistent_grid(num_cus, sc.total);
    // the top-K baseline's counting and the sampling noise are separate instantiations: the greedy judge path
    // pays nothing for them
    // (non-temporal W_lm loads for a single row tile were tried here as in the streaming kernel: no measurable change)
    if (a.dump) hipLaunchKernelGGL((k_lm_head_pair<true, false, false>), dim3(grid), dim3(256), 0, s, a, sc);
    else if (a.thr) hipLaunchKernelGGL((k_lm_head_pair<false, true, false>), dim3(grid), dim3(256), 0, s, a, sc);
    else if (a.key) hipLaunchKernelGGL((k_lm_head_pair<false, false, true>), dim3(grid), dim3(256), 0, s, a, sc);
    else hipLaunchKernelGGL((k_lm_head_pair<false, false, false>), dim3(grid), dim3(256), 0, s, a, sc);
    return hipGetLastError();
}

}  // namespace aj
