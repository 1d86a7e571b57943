// LM head (step 1) + per-vocabulary-block greedy maximum (first half of step 2) for 257..288 verify rows
// per row tile: 256 vocabulary x 288 verify rows per workgroup, the operand pipeline of lm_head_pair.hip
// (one operand per time step, both 64-byte halves of every 128-byte line in adjacent loads, 8 rotating
// half-buffers) with another wave layout: 4 waves side by side along the vocabulary, each 64 vocabulary
// rows x all 288 verify rows = 2 x 9 blocks of v_mfma_f32_32x32x16_bf16, 288 accumulator registers out of
// the 512 a wave has at one wave per SIMD.  One row tile then holds a batch such as 8 windows x 33 rows, so
// W_lm is streamed from HBM once and 8 % of the MFMA work is padding instead of 48 %.
//
// Time steps, slabs and the buffer rotation are those of lm_head_pair.hip (see there); what differs:
//   * a half-buffer slot is 18 KB (288 rows x 64 B; a W_lm half uses 16 KB of it), 8 slots = 144 KB;
//   * a W_lm slab is 8 loads per wave (16 row groups of 16 rows over 4 waves, 2 halves), a hidden_t slab
//     10 (18 row groups: waves 0 and 1 own five, waves 2 and 3 repeat their fourth - same rows to the same
//     place - so that every wave counts the same number of loads);
//   * a k step is 18 MFMAs in 6 groups of 3, 11 fragment reads (fa0, fb0..fb8, fa1 - the order the groups
//     need them) spread 4, 3, 3, 1 over the first groups of the step before.
#include "../../include/aj.h"
#include "aj_internal.h"
#include "lds_pipeline.h"
#include <type_traits>

namespace aj {

namespace {

constexpr int P9N = 256, P9M = 288;   // tile: vocabulary rows, verify rows
constexpr int SLOT = P9M * 64;        // bytes of a half-buffer slot
constexpr int WLOADS = 8, HLOADS = 10;
constexpr int LBB9 = 7;               // loads of a time step that precede its barrier (slots 0..6)

// half-buffer slot of W_lm / hidden_t read at time step u (mod 8): u = 2*(slab mod 4) + half
constexpr int slot_w(int u)
{
    const int p = (u >> 1) & 1, q = (u >> 2) & 1, h = u & 1;
    return h == 0 ? p : (q ? 5 + 2 * p : 4 + 2 * p);
}
constexpr int slot_h(int u)
{
    const int p = (u >> 1) & 1, q = (u >> 2) & 1, h = u & 1;
    return h == 1 ? 2 + p : (q ? 4 + 2 * p : 5 + 2 * p);
}

template <int U>
using step9_c = std::integral_constant<int, U>;

template <bool DUMP, bool TOPK, bool SAMPLE>
__global__ __launch_bounds__(256) void k_lm_head_pair9(LmHeadArgs a, Sched sc)
{
    constexpr int TN = 2, TM = 9, NG = 6, GS = 3, NR = TN + TM;
    __shared__ __attribute__((aligned(1024))) char lds[8 * SLOT];
    __shared__ Best red[3 * P9M];
    __shared__ int32_t redc[3 * P9M];     // top-K baseline: counts of the other wave columns

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wn = wave;
    const int l32 = lane & 31, kh = lane >> 5;
    const int d = a.d, NBLK = d / 256;     // blocks of 8 time steps per tile (host guarantees d % 256 == 0)
    const char *W = (const char *)a.W, *H = (const char *)a.H;
    const uint32_t rowbytes = (uint32_t)d * 2u;

    const int G = gridDim.x, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, SL = G >> 3;
    auto tile_at = [&](int step) { return (step * 8 + xcd) * SL + slot; };

    // loader: an instruction covers 16 tile rows x 64 B; lane i fills slot (row i/4, chunk i%4) and
    // fetches global chunk (i%4) ^ ((row/4)%4) of its half (conflict-free 16-byte fragment reads).
    // Row group of load pair g of this wave: 4g + wave; the fifth hidden_t group is 16 + wave for waves
    // 0 and 1 and a repeat of the fourth for the others.
    const int rl = lane >> 2;
    const uint32_t cg16 = (uint32_t)(((lane & 3) ^ ((rl >> 2) & 3)) * 16);
    const uint32_t lds_w = lds_offset_of(lds) + wave * 1024;
    const int g4 = wave < 2 ? 16 + wave : 12 + wave;                  // fifth hidden_t row group
    const uint32_t lds_g4 = lds_offset_of(lds) + g4 * 1024;
    // fragment reads: lane (row l32, k half kh) of a block reads chunk (2*s + kh) ^ swizzle(row)
    const int swz = (l32 >> 2) & 3;
    const int a_row = (wn * 64 + l32) * 64, b_row = l32 * 64;
    const int pos0 = ((0 + kh) ^ swz) * 16, pos1 = ((2 + kh) ^ swz) * 16;

    f32x16 acc[TN][TM - 1], acc9[TN];     // acc9: row block 8, kept in VGPRs (see time_step)
    bf16x8 fa[2][TN], fb[2][TM];
    uint32_t vw[4], vh[5], vw2[4], vh2[5];   // lane offsets of this wave's row groups: this tile, next tile
    auto tile_offsets = [&](int mt_, int nt_, uint32_t(&ow)[4], uint32_t(&oh)[5]) {
#pragma unroll
        for (int i = 0; i < 5; ++i) {
            const int row = (i < 4 ? i * 4 + wave : g4) * 16 + rl;
            if (i < 4) ow[i] = __umul24(min(nt_ * P9N + row, a.V - 1), rowbytes) + cg16;   // clamped: stays in bounds
            oh[i] = __umul24(min(mt_ * P9M + row, a.M - 1), rowbytes) + cg16;
        }
    };
    // load i of a slab: row group i/2, half i%2, into slots (s0, s1)
    auto load_w = [&](const char *gb, const uint32_t(&vo)[4], int i, int s0, int s1) {
        lds_dma_16(gb + (i & 1) * 64, vo[i >> 1], lds_w + ((i & 1) ? s1 : s0) * SLOT + (i >> 1) * 4096);
    };
    auto load_h = [&](const char *gb, const uint32_t(&vo)[5], int i, int s0, int s1) {
        const uint32_t dst = (i >> 1) < 4 ? lds_w + (i >> 1) * 4096 : lds_g4;
        lds_dma_16(gb + (i & 1) * 64, vo[i >> 1], dst + ((i & 1) ? s1 : s0) * SLOT);
    };
    // fragments i0..i1 of k step s of slots (sw, sh) into set `to`, in the order fa0, fb0..fb8, fa1
    auto R = [&](int sw, int sh, int s, int to, int i0, int i1) {
        const int pos = s ? pos1 : pos0;
#pragma unroll
        for (int i = i0; i < i1; ++i) {
            if (i == 0) fa[to][0] = *(const bf16x8 *)(lds + sw * SLOT + a_row + pos);
            else if (i <= TM) fb[to][i - 1] = *(const bf16x8 *)(lds + sh * SLOT + b_row + (i - 1) * 2048 + pos);
            else fa[to][1] = *(const bf16x8 *)(lds + sw * SLOT + a_row + 2048 + pos);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // reads that follow group rg (0..3) of the step before: 4, 3, 3, 1
    constexpr int RB[5] = {0, 4, 7, 10, NR};

    // One time step = two k steps of 18 MFMAs in 6 groups of 3.  After each group: part of the next k step's
    // fragment reads (groups 0..3; in the second k step groups 1..4, after the wait + barrier that opens the
    // next time step, which follows group 1) and at most one load of the slab this step fetches.
    auto time_step = [&](auto uc, const char *gb, const uint32_t(&vow)[4], const uint32_t(&voh)[5], bool issuing,
                         bool next_step) {
        constexpr int U = decltype(uc)::value, UN = (U + 1) & 7;
        constexpr bool ld_w = (U & 1) != 0;
        constexpr int js = ld_w ? ((U + 3) >> 1) & 3 : ((U + 2) >> 1) & 3;          // slab (mod 4) being loaded
        constexpr int d0 = ld_w ? slot_w(2 * js) : slot_h(2 * js), d1 = ld_w ? slot_w(2 * js + 1) : slot_h(2 * js + 1);
        constexpr int NL = ld_w ? WLOADS : HLOADS;
        // loads still allowed in flight at the barrier that opens step U+1: its operands are older than
        // this step's loads, and when U+1 is odd (this step fetches hidden_t) also older than the W_lm slab
        // of the step before
        constexpr int VM = (UN & 1) ? WLOADS + LBB9 : LBB9;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int g = 0; g < NG; ++g) {
#pragma unroll
                for (int m = g * GS; m < (g + 1) * GS; ++m) {
                    if (m % TM == TM - 1) {
                        // the ninth row block accumulates in VGPRs, stated explicitly: 16 of the 18 blocks fill the
                        // 256 AGPRs, and left to itself the compiler shuffles accumulators between the two files
                        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
                                     : "+v"(acc9[m / TM])
                                     : "v"(fa[t][m / TM]), "v"(fb[t][TM - 1]));
                    } else {
                        acc[m / TM][m % TM] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            fa[t][m / TM], fb[t][m % TM], acc[m / TM][m % TM], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                if (t == 1 && g == 1 && next_step) {
                    if (issuing) wait_vm_lgkm_and_barrier<VM>();
                    else wait_vm_lgkm_and_barrier<0>();      // fewer loads in flight than the constant assumes
                }
                const int rg = t == 1 ? g - 1 : g;
                if (rg >= 0 && rg < 4) {
                    if (t == 0) R(slot_w(U), slot_h(U), 1, 1, RB[rg], RB[rg + 1]);
                    else if (next_step) R(slot_w(UN), slot_h(UN), 0, 0, RB[rg], RB[rg + 1]);
                }
                const int i = t * NG + g;
                if (issuing && i < NL) {
                    if (ld_w) load_w(gb, vow, i, d0, d1);
                    else load_h(gb, voh, i, d0, d1);
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
#pragma unroll
        for (int i = 0; i < WLOADS; ++i) load_w(W, vw, i, slot_w(0), slot_w(1));
#pragma unroll
        for (int i = 0; i < HLOADS; ++i) load_h(H, vh, i, slot_h(0), slot_h(1));
#pragma unroll
        for (int i = 0; i < WLOADS; ++i) load_w(W + 128, vw, i, slot_w(2), slot_w(3));
        wait_vm_lgkm_and_barrier<WLOADS>();           // slab 0 of both operands has landed
        R(slot_w(0), slot_h(0), 0, 0, 0, NR);
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
                for (int r = 0; r < 16; ++r) {
                    if (y < TM - 1) acc[x][y][r] = 0.f;
                    else acc9[x][r] = 0.f;
                }

        // blocks of 8 time steps = 4 slabs = 512 bytes of k; all but the last load within this tile
        for (int blk = 0; blk < NBLK - 1; ++blk) {
            const char *Wb = W + blk * 512, *Hb = H + blk * 512;
            time_step(step9_c<0>{}, Hb + 128, vw, vh, true, true);
            time_step(step9_c<1>{}, Wb + 256, vw, vh, true, true);
            time_step(step9_c<2>{}, Hb + 256, vw, vh, true, true);
            time_step(step9_c<3>{}, Wb + 384, vw, vh, true, true);
            time_step(step9_c<4>{}, Hb + 384, vw, vh, true, true);
            time_step(step9_c<5>{}, Wb + 512, vw, vh, true, true);
            time_step(step9_c<6>{}, Hb + 512, vw, vh, true, true);
            time_step(step9_c<7>{}, Wb + 640, vw, vh, true, true);
        }
        {   // last block: its steps 5..7 load slabs 0, 0, 1 of the next tile, if there is one
            const char *Wb = W + (NBLK - 1) * 512, *Hb = H + (NBLK - 1) * 512;
            time_step(step9_c<0>{}, Hb + 128, vw, vh, true, true);
            time_step(step9_c<1>{}, Wb + 256, vw, vh, true, true);
            time_step(step9_c<2>{}, Hb + 256, vw, vh, true, true);
            time_step(step9_c<3>{}, Wb + 384, vw, vh, true, true);
            time_step(step9_c<4>{}, Hb + 384, vw, vh, true, true);
            time_step(step9_c<5>{}, W, vw2, vh2, have_next, true);
            time_step(step9_c<6>{}, H, vw2, vh2, have_next, true);
            time_step(step9_c<7>{}, W + 128, vw2, vh2, have_next, have_next);
        }

        // the hand-written MFMAs are invisible to the compiler's hazard handling: let the last of them retire
        // before their accumulators are read
        asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
        // ---- greedy maximum: D register r of a lane = vocabulary row 8*(r/4) + 4*(lane/32) + r%4 of its block
        const int v_base = nt * P9N + wn * 64 + kh * 4;
        float pv[TM];
        int32_t pi[TM], pc[TM];
#pragma unroll
        for (int y = 0; y < TM; ++y) {
            const int lr = y * 32 + l32;                     // verify row inside the tile
            const int row = mt * P9M + lr;
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
                    float val = y < TM - 1 ? acc[x][y][r] : acc9[x][r];
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
                red[(wn - 1) * P9M + lr] = Best{bv, bi};
                if (TOPK) redc[(wn - 1) * P9M + lr] = cn;
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
                const int lr = y * 32 + l32;
                const int row = mt * P9M + lr;
                float bv = pv[y];
                int32_t bi = pi[y], cn = pc[y];
#pragma unroll
                for (int w = 0; w < 3; ++w) {
                    const Best o = red[w * P9M + lr];
                    if (better(o.v, o.i, bv, bi)) {
                        bv = o.v;
                        bi = o.i;
                    }
                    if (TOPK) cn += redc[w * P9M + lr];
                }
                if (row < a.M) a.part[(size_t)row * a.nblocks + nt] = Best{bv, bi};
                if (TOPK && row < a.M) a.cnt[(size_t)row * a.nblocks + nt] = cn;
            }
        }
        // `red` is next written after the barriers of the following tile's time steps: no extra barrier
        if (have_next) {
#pragma unroll
            for (int i = 0; i < 5; ++i) {
                if (i < 4) vw[i] = vw2[i];
                vh[i] = vh2[i];
            }
        }
        T = T2;
        mt = mt2;
        nt = nt2;
    }
}

}  // namespace

int lm_head_pair9_blocks(int V) { return (V + P9N - 1) / P9N; }

int lm_head_pair9_padded_rows(int M) { return (M + P9M - 1) / P9M * P9M; }

bool lm_head_pair9_supports(int M, int V, int d) { return lm_head_pair_supports(M, V, d); }

hipError_t lm_head_pair9_bf16(const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    Sched sc;
    sc.tiles_m = (a.M + P9M - 1) / P9M;
    sc.tiles_n = (a.V + P9N - 1) / P9N;
    sc.gm = sc.tiles_m < 8 ? sc.tiles_m : 8;
    sc.total = sc.tiles_m * sc.tiles_n;
    const int grid = persistent_grid(num_cus, sc.total);
    // the top-K baseline's counting and the sampling noise are separate instantiations: the greedy judge path
    // pays nothing for them
    if (a.dump) hipLaunchKernelGGL((k_lm_head_pair9<true, false, false>), dim3(grid), dim3(256), 0, s, a, sc);
    else if (a.thr) hipLaunchKernelGGL((k_lm_head_pair9<false, true, false>), dim3(grid), dim3(256), 0, s, a, sc);
    else if (a.key) hipLaunchKernelGGL((k_lm_head_pair9<false, false, true>), dim3(grid), dim3(256), 0, s, a, sc);
    else hipLaunchKernelGGL((k_lm_head_pair9<false, false, false>), dim3(grid), dim3(256), 0, s, a, sc);
    return hipGetLastError();
}

}  // namespace aj
