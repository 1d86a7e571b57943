// LM head (step 1) fused with the per-vocabulary-block greedy maximum (first half of step 2):
// the general template of the large-tile and streaming-tile kernels.
//
//   * persistent workgroups (one per compute unit) walk a list of logit tiles; the k-loop of
//     all their tiles is ONE software pipeline, so the HBM stream never drains at a tile edge;
//   * operand tiles go global -> LDS with asynchronous direct-to-LDS loads (no register
//     staging), NS stages deep; every load instruction covers whole 64..256-byte row segments;
//   * LDS rows are XOR-swizzled in 16-byte chunks so that the 16-byte MFMA fragment reads are
//     bank-conflict free; the swizzle costs nothing because each lane picks its global chunk;
//   * v_mfma_f32_32x32x16_bf16 with A = W_lm (row = vocabulary) and B = hidden_t (column =
//     verify row): a lane owns one verify row and 16 vocabulary entries per block, so the
//     greedy maximum is an in-lane scan in ascending vocabulary order (strict > keeps the lowest
//     index), then one cross-half shuffle and one cross-wave exchange per tile;
//   * tiles are ordered in groups of GM row-tiles x all column-tiles, and consecutive runs of
//     tiles go to the workgroups of one XCD (workgroup id mod 8), so that the 32 compute units
//     behind one L2 work on a compact block of tiles that share operand panels.
//
// Instantiations:
//   STREAM  128 vocabulary x 32 verify rows, BK = 128, 3 stages, one running partial per workgroup and
//           wave column: W_lm-streaming regime (M <= 32) at hidden sizes the register-resident
//           16-row-tile kernel (lm_head_stream16.hip) does not take; the same with 128 x 64 tiles for
//           33..64 rows and 128 x 128 tiles (BK = 64, 4 stages) for 65..128 rows.
//   BIG     256 x 256, 4 waves of 128 x 128, BK = 32, 4 stages, hand-scheduled stage: MFMA-bound regime at
//           hidden sizes lm_head_pair.hip does not take (not a multiple of 256).
//   TALL    256 x 320 or 256 x 288 (wave rows of 5 + 4 blocks), 8 waves, BK = 64, 2 stages: 289..320 verify
//           rows in ONE row tile (and 257..288 at hidden sizes lm_head_pair9.hip does not take), so that
//           W_lm is read once and no nearly empty second row tile is computed.
#include "../../include/aj.h"
#include "aj_internal.h"
#include "lds_pipeline.h"

namespace aj {

namespace {

template <int TN_, int TM_, int WN_, int WM_, int WK_, int BK_, int NS_, bool RUNNING_, bool PIPE_ = false, int MCUT_ = 0>
struct Shape {
    static constexpr int TN = TN_, TM = TM_, WN = WN_, WM = WM_, WK = WK_, BK = BK_, NS = NS_;
    static constexpr bool RUNNING = RUNNING_;     // one running partial per workgroup (needs a single row tile)
    // PIPE: MFMA-bound schedule.  Fragments of k step s+1 are read while the MFMAs of step s run, the
    // stage's loads are issued in KSTEPS parts between them, and the wait + barrier for the NEXT
    // stage sits before the MFMAs of a stage's last k step, so the matrix pipe never waits for it.
    static constexpr bool PIPE = PIPE_;
    static constexpr int NW = WN * WM * WK;       // waves per workgroup
    static constexpr int BN = 32 * TN * WN;       // vocabulary rows per tile
    // MCUT: the LAST wave row computes MCUT fewer 32-row blocks than the others (a tile of 9 blocks =
    // 5 + 4), so that the tile height fits the row count more tightly
    static constexpr int MCUT = MCUT_;
    static constexpr int BM = 32 * (TM * WM - MCUT);   // verify rows per tile
    static constexpr int CH = BK / 8;             // 16-byte chunks per tile row
    static constexpr int RPI = 64 / CH;           // tile rows covered by one wave-wide load
    static constexpr int RPW = CH >= 16 ? 1 : 16 / CH;   // tile rows per 256-byte bank wrap
    static constexpr int SWM = CH >= 16 ? 16 : CH;       // swizzle modulus: XOR acts on the low bits of the chunk index
    static constexpr int KSTEPS = BK / 16 / WK;   // k16 steps per wave per stage
    static constexpr int WI = BN / RPI, HI = BM / RPI;   // wave-wide loads per stage: W tile, H tile
    static constexpr int HLW = (HI + NW - 1) / NW;   // H loads per wave (when HI % NW != 0 the last waves repeat a load)
    static constexpr int LPW = WI / NW + HLW;     // loads per wave per stage
    static constexpr int W_BYTES = BN * BK * 2, H_BYTES = BM * BK * 2;
    static constexpr int STAGE_BYTES = W_BYTES + H_BYTES;
    static constexpr int RED_BYTES = (WK - 1) * WN * WM * TN * TM * 16 * 64 * 4;   // k-split partial sums
    static_assert(CH == 4 || CH == 8 || CH == 16 || CH == 32, "BK must be 32, 64, 128 or 256");
    static_assert(WI % NW == 0, "W loads must split evenly over the waves");
    static_assert(MCUT == 0 || (!PIPE_ && MCUT < TM && WM > 1), "short last wave row: compiler-scheduled path only");
    static_assert((BK / 16) % WK == 0, "k steps must split evenly over the k-split waves");
    static_assert((NW * RPI) % 16 == 0, "the chunk a lane fetches must not depend on the load index");
    static_assert((NS - 2) * LPW <= 63, "vmcnt range");
    static_assert(NS * STAGE_BYTES + BM * WN * 12 + RED_BYTES <= 160 * 1024, "LDS budget");
    static constexpr int LPP = LPW / KSTEPS;      // PIPE: loads per wave per k step
    // PIPE schedule.  The TN*TM MFMAs of a k step go out in NG groups (x-major order); a "slot" is the
    // shadow of one group.  Fragment reads of the next step (TN + TM of them, in the order fa0, fb0..,
    // fa1.. that the first groups need) follow groups 0 and 1, or groups 1 and 2 in a stage's last
    // step, where the wait + barrier for the next stage comes right after group 1.  The stage's LPW
    // loads are spread evenly over all KSTEPS*NG slots.
    static constexpr int NG = (TN * TM) % 4 == 0 ? 4 : 5;          // 4x4 blocks: 4 groups of 4; 2x5: 5 groups of 2
    static constexpr int GS = TN * TM / NG;
    static constexpr int SLOTS = KSTEPS * NG;
    static constexpr int NR = TN + TM, NR0 = (NR + 1) / 2;          // reads: first chunk, then the rest
    static constexpr int loads_begin(int slot) { return (slot * LPW + SLOTS - 1) / SLOTS; }   // ceil(slot*LPW/SLOTS)
    static constexpr int loads_end(int slot) { return ((slot + 1) * LPW + SLOTS - 1) / SLOTS; }
    // loads of the stage being issued that precede the barrier (those in slots up to the last step's group 0)
    static constexpr int LOADS_BEFORE_BARRIER = loads_end((KSTEPS - 1) * NG);
    static constexpr int PIPE_VMCNT = NS == 2 ? 0 : (NS - 3) * LPW + LOADS_BEFORE_BARRIER;
    static_assert(!PIPE || (WK == 1 && NS >= 2 && KSTEPS >= 2 && KSTEPS % 2 == 0 && (TN * TM) % NG == 0 && NG >= 3),
                  "hand-scheduled stage: even number of k steps (two fragment sets alternate), at least 3 groups");
    static_assert(!PIPE || NS > 2 || LOADS_BEFORE_BARRIER == LPW, "two stages: the whole next stage precedes the barrier");
    static_assert(!PIPE || PIPE_VMCNT <= 63, "vmcnt range");
};

using StreamShape = Shape<1, 1, 4, 1, 1, 128, 3, true>;            // up to 32 verify rows; any d_t % 128 == 0
using Stream64Shape = Shape<1, 2, 4, 1, 1, 128, 3, true>;          // 33..64 rows: 128 x 64 tile, same pipeline
using Stream128Shape = Shape<1, 4, 4, 1, 1, 64, 4, true>;          // 65..128 rows: 128 x 128 tile, BK = 64, 4 stages
using BigShape = Shape<4, 4, 2, 2, 1, 32, 4, false, true>;
using TallShape = Shape<2, 5, 4, 2, 1, 64, 2, false>;                 // 256 x 320, 8 waves: 289..320 verify rows in ONE row tile
using Tall288Shape = Shape<2, 5, 4, 2, 1, 64, 2, false, false, 1>;   // 256 x 288 (wave rows of 5 + 4 blocks)

template <class S, bool DUMP, bool TOPK, bool SAMPLE>
__global__ __launch_bounds__(S::NW * 64) void k_lm_head_mfma(LmHeadArgs a, Sched sc)
{
    constexpr int TN = S::TN, TM = S::TM, WN = S::WN, WM = S::WM, WK = S::WK, NW = S::NW, BK = S::BK, NS = S::NS;
    constexpr int CH = S::CH, RPI = S::RPI, RPW = S::RPW, SWM = S::SWM, LPW = S::LPW;
    constexpr int AHEAD = NS - 1;                  // stages in flight ahead of the one being computed
    __shared__ __attribute__((aligned(1024))) char lds[NS * S::STAGE_BYTES];
    __shared__ Best red[S::BM * (WN > 1 ? WN - 1 : 1)];
    __shared__ int32_t redc[S::BM * (WN > 1 ? WN - 1 : 1)];     // top-K baseline: counts of the other wave columns
    __shared__ float redk[WK > 1 ? S::RED_BYTES / 4 : 1];

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wn = wave % WN, wm = (wave / WN) % WM, wk = wave / (WN * WM);
    const int l32 = lane & 31, kh = lane >> 5;
    const int d = a.d, KS = d / BK;       // host guarantees KS >= AHEAD
    const char *W = (const char *)a.W, *H = (const char *)a.H;

    // ---- persistent tile list of this workgroup: runs of (gridDim/8) consecutive tiles per XCD
    const int G = gridDim.x, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, SL = G >> 3;
    auto tile_at = [&](int step) { return (step * 8 + xcd) * SL + slot; };

    // ---- loader constants
    // A wave-wide load covers 1 KB of LDS = RPI whole tile rows; lane i fills slot (row i / CH,
    // chunk i % CH) and must therefore fetch global chunk (i % CH) ^ swizzle(row).  Load j of wave w
    // covers tile rows (j*NW + w)*RPI ..; NW*RPI is a multiple of the swizzle period (16 rows), so
    // the chunk a lane fetches does not depend on j.
    const int rl = lane / CH;
    const uint32_t cg16 = (uint32_t)(((lane % CH) ^ (((wave * RPI + rl) / RPW) % SWM)) * 16);
    const uint32_t rowbytes = (uint32_t)d * 2u;
    const uint32_t lds_base = lds_offset_of(lds);
    // ---- fragment-read constants
    const int swz = (l32 / RPW) % SWM;
    const int a_row = (wn * TN * 32 + l32) * BK * 2;              // byte offset of the lane's row in the W tile
    const int b_row = S::W_BYTES + (wm * TM * 32 + l32) * BK * 2; // ... in the H tile

    // One pipeline stage: the W tile [BN][BK] and the H tile [BM][BK] of tile (mt, nt) at k = ks*BK, into
    // ring buffer `buf`.  Each load is "uniform 64-bit base + 32-bit lane offset"; the lane offsets are
    // recomputed at every stage (a few VALU ops beside hundreds of MFMA cycles) rather than kept in
    // registers across the k loop - the laundered `rl_now` stops the compiler from hoisting them.
    const bool w_once = sc.tiles_m == 1;
    auto issue = [&](int mt, int nt, int ks, int buf, int part = -1) {   // part >= 0: only that share of the loads
        int rl_now = rl;
        asm volatile("" : "+v"(rl_now));
        const int n_first = nt * S::BN + wave * RPI + rl_now;     // the lane's row in load j = 0
        const int m_first = mt * S::BM + wave * RPI + rl_now;
        const uint32_t koff = (uint32_t)(ks * BK * 2) + cg16;
        const uint32_t stage = lds_base + buf * S::STAGE_BYTES + wave * 1024;
#pragma unroll
        for (int j = 0; j < LPW; ++j) {
            if (part >= 0 && j / S::LPP != part) continue;
            if (j < S::WI / NW) {
                const int row = min(n_first + j * NW * RPI, a.V - 1);       // clamped: ragged tiles stay in bounds
                // with a single row tile W_lm is streamed from HBM exactly once: non-temporal
                if (w_once) load_to_lds_16_nt(W, __umul24(row, rowbytes) + koff, stage + j * NW * 1024);
                else load_to_lds_16(W, __umul24(row, rowbytes) + koff, stage + j * NW * 1024);
            } else {
                // H load jj of this wave is tile load jj*NW + wave; a wave that has none left (HI is not a
                // multiple of NW) repeats its previous one: same rows to the same place, harmless
                int jj = j - S::WI / NW;
                if (jj * NW + wave >= S::HI) jj -= 1;
                const int row = min(m_first + jj * NW * RPI, a.M - 1);
                load_to_lds_16(H, __umul24(row, rowbytes) + koff,
                               __builtin_amdgcn_readfirstlane(stage + S::W_BYTES + jj * NW * 1024));
            }
        }
    };

    f32x16 acc[TN][TM];
    float run_v[TM];
    int32_t run_i[TM], run_c[TM];
#pragma unroll
    for (int y = 0; y < TM; ++y) {
        run_v[y] = -INFINITY;
        run_i[y] = 0x7fffffff;
        run_c[y] = 0;
    }

    // MFMAs of one landed stage (ring buffer `buf`); this wave's share of the k steps
    const int ty = (S::MCUT > 0 && wm == WM - 1) ? TM - S::MCUT : TM;   // 32-row blocks this wave computes (wave-uniform)
    auto compute = [&](int ks, int buf) {
        const char *stage = lds + buf * S::STAGE_BYTES;
#pragma unroll
        for (int s0 = 0; s0 < S::KSTEPS; ++s0) {
            const int s = wk * S::KSTEPS + s0;
            const int pos = ((2 * s + kh) ^ swz) * 16;
            bf16x8 fa[TN], fb[TM];
#pragma unroll
            for (int x = 0; x < TN; ++x) fa[x] = *(const bf16x8 *)(stage + a_row + x * 32 * BK * 2 + pos);
#pragma unroll
            for (int y = 0; y < TM; ++y) {
                if (y < ty) fb[y] = *(const bf16x8 *)(stage + b_row + y * 32 * BK * 2 + pos);
            }
#pragma unroll
            for (int x = 0; x < TN; ++x)
#pragma unroll
                for (int y = 0; y < TM; ++y)
                    if (y < ty) acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[x], fb[y], acc[x][y], 0, 0, 0);
        }
    };

    // PIPE: two fragment sets
    bf16x8 fa[2][TN], fb[2][TM];
    auto read_frags = [&](int buf, int s, bf16x8(&ra)[TN], bf16x8(&rb)[TM]) {
        const char *stage = lds + buf * S::STAGE_BYTES;
        const int pos = ((2 * s + kh) ^ swz) * 16;
#pragma unroll
        for (int x = 0; x < TN; ++x) ra[x] = *(const bf16x8 *)(stage + a_row + x * 32 * BK * 2 + pos);
#pragma unroll
        for (int y = 0; y < TM; ++y) rb[y] = *(const bf16x8 *)(stage + b_row + y * 32 * BK * 2 + pos);
    };
    // PIPE: lane offsets of the loads of a stage, fixed per tile
    constexpr int WL = S::WI / NW;     // loads 0..WL-1 fetch W_lm rows, the rest hidden_t rows
    uint32_t voff[LPW];
    auto tile_offsets = [&](int mt_, int nt_, uint32_t(&vo)[LPW]) {
        const int n_first = nt_ * S::BN + wave * RPI + rl, m_first = mt_ * S::BM + wave * RPI + rl;
#pragma unroll
        for (int j = 0; j < LPW; ++j) {
            if (j < WL) vo[j] = __umul24(min(n_first + j * NW * RPI, a.V - 1), rowbytes) + cg16;
            else {
                static_assert(!S::PIPE || S::HI % NW == 0, "hand-scheduled path: H loads split evenly");
                vo[j] = __umul24(min(m_first + (j - WL) * NW * RPI, a.M - 1), rowbytes) + cg16;
            }
        }
    };

    int T = tile_at(0);
    int mt = 0, nt = 0, buf = 0;       // buf: ring buffer of the stage computed next
    if (T < sc.total) {
        tile_of(sc, T, mt, nt);
        if constexpr (S::PIPE) tile_offsets(mt, nt, voff);
#pragma unroll
        for (int p = 0; p < AHEAD; ++p) issue(mt, nt, p, p);
        if constexpr (S::PIPE) {
            wait_vm_lgkm_and_barrier<(AHEAD - 1) * LPW>();
            read_frags(0, 0, fa[0], fb[0]);
        }
    }

    for (int step = 0; T < sc.total; ++step) {
        const int T2 = tile_at(step + 1);
        const bool have_next = T2 < sc.total;
        int mt2 = 0, nt2 = 0;
        if (have_next) tile_of(sc, T2, mt2, nt2);
#pragma unroll
        for (int x = 0; x < TN; ++x)
#pragma unroll
            for (int y = 0; y < TM; ++y)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

        if constexpr (S::PIPE) {
            // Hand-scheduled stage for the MFMA-bound shapes (4x4 blocks per wave).  With one wave per
            // SIMD every instruction that is not an MFMA must sit in the shadow of a running MFMA, so
            // the 16 MFMAs of a k step go out in 4 groups of 4 (128 cycles each) and a few LDS reads
            // or loads follow each group; sched_barrier pins that order.  Fragments of (stage ks,
            // step 0) are already in set 0 (read after the previous stage's early barrier).  Per k step
            // t: groups 0 and 1 are followed by the 8 fragment reads of step t+1; in the LAST step
            // group 1 is followed by the wait + barrier for stage ks+1, and the reads (that stage's
            // step 0) follow groups 1 and 2.  Loads of the stage being issued follow the groups given by S::loads_after.
            // At the barrier the loads younger than stage ks+1 are AHEAD-2 whole stages plus those of
            // the stage being issued that precede the barrier (AHEAD = 1: it IS stage ks+1, and all
            // of it precedes the barrier).  Without a next tile fewer loads are in flight: wait for all.
            uint32_t voff2[LPW];
            if (have_next) tile_offsets(mt2, nt2, voff2);
            auto pipe_stage = [&](int ks, bool hot) {
                const int nbuf = buf + 1 == NS ? 0 : buf + 1;                       // next stage's buffer
                const int ibuf = buf + AHEAD >= NS ? buf + AHEAD - NS : buf + AHEAD; // buffer being refilled
                const bool next_stage = hot || ks + 1 < KS || have_next;
                const bool same_tile = hot || ks + AHEAD < KS;
                const bool issuing = same_tile || have_next;
                const int iks = same_tile ? ks + AHEAD : ks + AHEAD - KS;           // stage being issued
                const char *Wk = W + iks * BK * 2, *Hk = H + iks * BK * 2;
                const uint32_t dst = lds_base + ibuf * S::STAGE_BYTES + wave * 1024;
                auto L = [&](int j0, int j1) {
                    if (issuing) {
#pragma unroll
                        for (int j = j0; j < j1; ++j) {
                            const uint32_t vo = same_tile ? voff[j] : voff2[j];
                            if (j < WL) lds_dma_16(Wk, vo, dst + j * NW * 1024);
                            else lds_dma_16(Hk, vo, dst + S::W_BYTES + (j - WL) * NW * 1024);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                };
                auto Gx = [&](int cur, int g) {                   // MFMAs g*GS .. of the step, x-major
#pragma unroll
                    for (int m = g * S::GS; m < (g + 1) * S::GS; ++m)
                        acc[m / TM][m % TM] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][m / TM], fb[cur][m % TM],
                                                                                      acc[m / TM][m % TM], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                };
                // fragments i0..i1 of (buffer b, step st) into set `to`, in the order fa0, fb0.., fa1..
                auto R = [&](int b, int st, int to, int i0, int i1) {
                    const char *stage = lds + b * S::STAGE_BYTES;
                    const int pos = ((2 * st + kh) ^ swz) * 16;
#pragma unroll
                    for (int i = i0; i < i1; ++i) {
                        if (i == 0) fa[to][0] = *(const bf16x8 *)(stage + a_row + pos);
                        else if (i <= TM) fb[to][i - 1] = *(const bf16x8 *)(stage + b_row + (i - 1) * 32 * BK * 2 + pos);
                        else fa[to][i - TM] = *(const bf16x8 *)(stage + a_row + (i - TM) * 32 * BK * 2 + pos);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                };
#pragma unroll
                for (int t = 0; t < S::KSTEPS; ++t) {
                    const int cur = t & 1;
                    const bool last = t == S::KSTEPS - 1;
#pragma unroll
                    for (int g = 0; g < S::NG; ++g) {
                        Gx(cur, g);
                        if (last && g == 1 && next_stage) {
                            if (issuing) wait_vm_lgkm_and_barrier<S::PIPE_VMCNT>();
                            else wait_vm_lgkm_and_barrier<0>();
                        }
                        const int rg = last ? g - 1 : g;          // 0: first chunk of reads, 1: second
                        if (rg == 0 || rg == 1) {
                            if (!last) R(buf, t + 1, cur ^ 1, rg ? S::NR0 : 0, rg ? S::NR : S::NR0);
                            else if (next_stage) R(nbuf, 0, cur ^ 1, rg ? S::NR0 : 0, rg ? S::NR : S::NR0);
                        }
                        L(S::loads_begin(t * S::NG + g), S::loads_end(t * S::NG + g));
                    }
                }
                buf = nbuf;
            };
            for (int ks = 0; ks < KS - AHEAD; ++ks) pipe_stage(ks, true);
#pragma unroll
            for (int p = 0; p < AHEAD; ++p) pipe_stage(KS - AHEAD + p, false);
            if (have_next) {
#pragma unroll
                for (int j = 0; j < LPW; ++j) voff[j] = voff2[j];
            }
        } else {
        // Stage ks has landed once at most the NS-2 younger stages are outstanding (loads complete in
        // order).  The barrier also frees the buffer computed in the previous iteration, which is the
        // one the new loads go to.  Hot part: the stage issued belongs to the same tile - no branches.
        for (int ks = 0; ks < KS - AHEAD; ++ks) {
            wait_vm_and_barrier<(NS - 2) * LPW>();
            issue(mt, nt, ks + AHEAD, buf + AHEAD >= NS ? buf + AHEAD - NS : buf + AHEAD);
            compute(ks, buf);
            buf = buf + 1 == NS ? 0 : buf + 1;
        }
        // Last AHEAD stages of the tile: prefetch the first stages of the next tile, if there is one;
        // otherwise fewer loads are in flight than the constant assumes, so wait for all of them.
#pragma unroll
        for (int p = 0; p < AHEAD; ++p) {
            if (have_next) {
                wait_vm_and_barrier<(NS - 2) * LPW>();
                issue(mt2, nt2, p, buf + AHEAD >= NS ? buf + AHEAD - NS : buf + AHEAD);
            } else {
                wait_vm_and_barrier<0>();
            }
            compute(KS - AHEAD + p, buf);
            buf = buf + 1 == NS ? 0 : buf + 1;
        }
        }

        // ---- k-split waves: add the partial sums of waves wk > 0 into wave wk == 0 (through LDS)
        if (WK > 1) {
            const int blk = (wm * WN + wn) * TN * TM;
            if (wk > 0) {
#pragma unroll
                for (int x = 0; x < TN; ++x)
#pragma unroll
                    for (int y = 0; y < TM; ++y)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            redk[((((wk - 1) * WN * WM * TN * TM + blk + x * TM + y) * 16) + r) * 64 + lane] = acc[x][y][r];
            }
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            if (wk == 0) {
#pragma unroll
                for (int w = 1; w < WK; ++w)
#pragma unroll
                    for (int x = 0; x < TN; ++x)
#pragma unroll
                        for (int y = 0; y < TM; ++y)
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                acc[x][y][r] += redk[((((w - 1) * WN * WM * TN * TM + blk + x * TM + y) * 16) + r) * 64 + lane];
            }
            // redk is rewritten only after the k-loop barriers of the next tile
        }

        // ---- greedy maximum: D register r of a lane = vocabulary row 8*(r/4) + 4*(lane/32) + r%4 of its block
        const int v_base = nt * S::BN + wn * TN * 32 + kh * 4;
        float pv[TM];
        int32_t pi[TM], pc[TM];
#pragma unroll
        for (int y = 0; y < TM; ++y) {
            const int lr = wm * TM * 32 + y * 32 + l32;          // verify row inside the tile
            const int row = (y < ty) ? mt * S::BM + lr : a.M;    // a block this wave does not compute: no row
            float bv = S::RUNNING ? run_v[y] : -INFINITY;
            int32_t bi = S::RUNNING ? run_i[y] : 0x7fffffff;
            // top-K baseline: the row's draft token and the number of this block's entries ordered before it
            float th = INFINITY;
            int32_t tk = -1, cn = S::RUNNING ? run_c[y] : 0;
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
                        if (DUMP && row < a.M && wk == 0) a.dump[(size_t)row * a.V + v] = val;
                        if (SAMPLE) val = fmaf(val, a.inv_temp, gumbel_noise(klo, khi, (uint32_t)v));
                        // ascending v inside a lane and over a workgroup's tiles: strict > keeps the lowest
                        if (val > bv) {
                            bv = val;
                            bi = v;
                        }
                        if (TOPK) cn += ranks_before(val, v, th, tk);
                    }
                }
            if (S::RUNNING) {
                run_v[y] = bv;
                run_i[y] = bi;
                run_c[y] = cn;
                continue;
            }
            if (TOPK) cn += __shfl_xor(cn, 32);
            const float ov = __shfl_xor(bv, 32);
            const int32_t oi = __shfl_xor(bi, 32);
            if (better(ov, oi, bv, bi)) {
                bv = ov;
                bi = oi;
            }
            if (WN > 1 && wn > 0 && kh == 0 && y < ty) {
                red[(wn - 1) * S::BM + lr] = Best{bv, bi};
                if (TOPK) redc[(wn - 1) * S::BM + lr] = cn;
            }
            pv[y] = bv;
            pi[y] = bi;
            pc[y] = cn;
        }
        if (!S::RUNNING) {
            // LDS writes of `red` done and visible; do not wait for the prefetch loads in flight
            if (WN > 1) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            if (wn == 0 && kh == 0 && wk == 0) {
#pragma unroll
                for (int y = 0; y < TM; ++y) {
                    const int lr = wm * TM * 32 + y * 32 + l32;
                    const int row = (y < ty) ? mt * S::BM + lr : a.M;
                    float bv = pv[y];
                    int32_t bi = pi[y], cn = pc[y];
#pragma unroll
                    for (int w = 1; w < WN && y < ty; ++w) {
                        const Best o = red[(w - 1) * S::BM + lr];
                        if (better(o.v, o.i, bv, bi)) {
                            bv = o.v;
                            bi = o.i;
                        }
                        if (TOPK) cn += redc[(w - 1) * S::BM + lr];
                    }
                    if (row < a.M) a.part[(size_t)row * a.nblocks + nt] = Best{bv, bi};
                    if (TOPK && row < a.M) a.cnt[(size_t)row * a.nblocks + nt] = cn;
                }
            }
            // `red` is next written after the k-loop barriers of the following tile: no extra barrier
        }
        T = T2;
        mt = mt2;
        nt = nt2;
    }

    if (S::RUNNING) {
        // one partial per verify row, workgroup and wave column (a neutral one if there was no tile)
        static_assert(!S::RUNNING || WM == 1, "running partials: a single row tile");
#pragma unroll
        for (int y = 0; y < TM; ++y) {
            float bv = run_v[y];
            int32_t bi = run_i[y];
            const float ov = __shfl_xor(bv, 32);
            const int32_t oi = __shfl_xor(bi, 32);
            if (better(ov, oi, bv, bi)) {
                bv = ov;
                bi = oi;
            }
            const int row = y * 32 + l32;
            if (wk == 0 && kh == 0 && row < a.M)
                a.part[(size_t)row * a.nblocks + blockIdx.x * WN + wn] = Best{bv, bi};
            if (TOPK) {
                const int32_t cn = run_c[y] + __shfl_xor(run_c[y], 32);
                if (wk == 0 && kh == 0 && row < a.M) a.cnt[(size_t)row * a.nblocks + blockIdx.x * WN + wn] = cn;
            }
        }
    }
}

template <class S>
hipError_t launch(const LmHeadArgs &a, int num_cus, int gm, hipStream_t s)
{
    Sched sc;
    sc.tiles_m = (a.M + S::BM - 1) / S::BM;
    sc.tiles_n = (a.V + S::BN - 1) / S::BN;
    sc.gm = gm < 1 ? 1 : (gm > sc.tiles_m ? sc.tiles_m : gm);
    sc.total = sc.tiles_m * sc.tiles_n;
    const int grid = persistent_grid(num_cus, sc.total);
    // the top-K baseline's counting and the sampling noise are separate instantiations: the greedy judge path
    // pays nothing for them
    if (a.dump)
        hipLaunchKernelGGL((k_lm_head_mfma<S, true, false, false>), dim3(grid), dim3(S::NW * 64), 0, s, a, sc);
    else if (a.thr)
        hipLaunchKernelGGL((k_lm_head_mfma<S, false, true, false>), dim3(grid), dim3(S::NW * 64), 0, s, a, sc);
    else if (a.key)
        hipLaunchKernelGGL((k_lm_head_mfma<S, false, false, true>), dim3(grid), dim3(S::NW * 64), 0, s, a, sc);
    else
        hipLaunchKernelGGL((k_lm_head_mfma<S, false, false, false>), dim3(grid), dim3(S::NW * 64), 0, s, a, sc);
    return hipGetLastError();
}

}  // namespace

int lm_head_mfma_blocks(int variant, int V, int d, int num_cus)
{
    if (variant == AJ_KERNEL_STREAM) {  // one running partial per workgroup
        return persistent_grid(num_cus, (V + StreamShape::BN - 1) / StreamShape::BN) * StreamShape::WN;
    }
    if (variant == AJ_KERNEL_TALL) return (V + TallShape::BN - 1) / TallShape::BN;
    return (V + BigShape::BN - 1) / BigShape::BN;
}

bool lm_head_mfma_supports(int variant, int M, int V, int d)
{
    if (M <= 0 || V <= 0) return false;
    // lane offsets are 32-bit and row indices go through a 24-bit multiply
    if ((uint64_t)V * d * 2 >= (1ull << 32) || (uint64_t)M * d * 2 >= (1ull << 32)) return false;
    if (V >= (1 << 24) || M >= (1 << 24) || d * 2 >= (1 << 24)) return false;
    // whole k stages only, and at least as many as the pipeline runs ahead
    if (variant == AJ_KERNEL_STREAM)
        return d % StreamShape::BK == 0 && d / StreamShape::BK >= Stream128Shape::NS - 1 && M <= Stream128Shape::BM;
    if (variant == AJ_KERNEL_BIG) return d % BigShape::BK == 0 && d / BigShape::BK >= BigShape::NS - 1;
    if (variant == AJ_KERNEL_TALL)
        return d % TallShape::BK == 0 && d / TallShape::BK >= TallShape::NS - 1;
    return false;
}

// verify rows the variant computes for M rows (M rounded up to whole row tiles)
int lm_head_mfma_padded_rows(int variant, int M)
{
    auto pad = [M](int bm) { return (M + bm - 1) / bm * bm; };
    if (variant == AJ_KERNEL_TALL) return pad(Tall288Shape::BM) < pad(TallShape::BM) ? pad(Tall288Shape::BM) : pad(TallShape::BM);
    if (variant == AJ_KERNEL_BIG) return pad(BigShape::BM);
    return M <= StreamShape::BM ? StreamShape::BM : M <= Stream64Shape::BM ? Stream64Shape::BM : pad(Stream128Shape::BM);
}

hipError_t lm_head_mfma_bf16(int variant, const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    if (variant == AJ_KERNEL_STREAM)
        return a.M <= StreamShape::BM     ? launch<StreamShape>(a, num_cus, 1, s)
               : a.M <= Stream64Shape::BM ? launch<Stream64Shape>(a, num_cus, 1, s)
                                          : launch<Stream128Shape>(a, num_cus, 1, s);
    if (variant == AJ_KERNEL_TALL) {
        // 288- or 320-row tiles, whichever pads the row count less (ties: the taller one, fewer tiles)
        const int pad288 = (a.M + Tall288Shape::BM - 1) / Tall288Shape::BM * Tall288Shape::BM;
        const int pad320 = (a.M + TallShape::BM - 1) / TallShape::BM * TallShape::BM;
        return pad288 < pad320 ? launch<Tall288Shape>(a, num_cus, 8, s) : launch<TallShape>(a, num_cus, 8, s);
    }
    return launch<BigShape>(a, num_cus, 8, s);
}

}  // namespace aj
