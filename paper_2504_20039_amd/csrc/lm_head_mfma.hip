// LM head (step 1) fused with the per-vocabulary-block greedy maximum (first half of step 2):
// the two performance kernels, one template.
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
// Two instantiations:
//   STREAM  128 vocabulary x 32 verify rows, BK = 128, 3 stages: W_lm-streaming (HBM-bound) regime
//   BIG     256 x 256, BK = 64, 2 stages: MFMA-bound regime
#include "../../include/aj.h"
#include "aj_internal.h"

namespace aj {

namespace {

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void gbl_void;

template <int N>
__device__ __forceinline__ void wait_vm_and_barrier()
{
    // wait until at most N of this wave's global loads are outstanding, then workgroup barrier.
    // The memory clobber keeps the compiler from moving LDS accesses across it.
    static_assert(N >= 0 && N <= 63, "vmcnt field");
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

template <int TN_, int TM_, int WN_, int WM_, int BK_, int NS_>
struct Shape {
    static constexpr int TN = TN_, TM = TM_, WN = WN_, WM = WM_, BK = BK_, NS = NS_;
    static constexpr int NW = WN * WM;            // waves per workgroup
    static constexpr int BN = 32 * TN * WN;       // vocabulary rows per tile
    static constexpr int BM = 32 * TM * WM;       // verify rows per tile
    static constexpr int CH = BK / 8;             // 16-byte chunks per tile row
    static constexpr int RPI = 64 / CH;           // tile rows covered by one wave-wide load
    static constexpr int RPW = CH >= 16 ? 1 : 16 / CH;   // tile rows per 256-byte bank wrap
    static constexpr int WI = BN / RPI, HI = BM / RPI;   // wave-wide loads per stage: W tile, H tile
    static constexpr int LPW = (WI + HI) / NW;    // loads per wave per stage
    static constexpr int W_BYTES = BN * BK * 2, H_BYTES = BM * BK * 2;
    static constexpr int STAGE_BYTES = W_BYTES + H_BYTES;
    static_assert(CH == 4 || CH == 8 || CH == 16, "BK must be 32, 64 or 128");
    static_assert(WI % NW == 0 && HI % NW == 0, "loads must split evenly over the waves");
    static_assert((NW * RPI) % 16 == 0, "per-lane swizzle must not depend on the load index");
    static_assert((NS - 2) * LPW <= 63, "vmcnt range");
    static_assert(NS * STAGE_BYTES + BM * WN * 8 <= 160 * 1024, "LDS budget");
};

using StreamShape = Shape<1, 1, 4, 1, 128, 3>;
using BigShape = Shape<4, 4, 2, 2, 64, 2>;

struct Sched {
    int tiles_m, tiles_n, gm, total;
};

__device__ __forceinline__ void tile_of(const Sched &sc, int T, int &mt, int &nt)
{
    const int per_group = sc.gm * sc.tiles_n;
    const int ngroups = (sc.tiles_m + sc.gm - 1) / sc.gm;
    int grp = T / per_group;
    if (grp > ngroups - 1) grp = ngroups - 1;
    const int within = T - grp * per_group;
    const int g = (grp == ngroups - 1) ? sc.tiles_m - grp * sc.gm : sc.gm;
    mt = grp * sc.gm + within % g;
    nt = within / g;
}

template <class S, bool DUMP>
__global__ __launch_bounds__(S::NW * 64) void k_lm_head_mfma(LmHeadArgs a, Sched sc)
{
    constexpr int TN = S::TN, TM = S::TM, WN = S::WN, NW = S::NW, BK = S::BK, NS = S::NS;
    constexpr int CH = S::CH, RPI = S::RPI, RPW = S::RPW, LPW = S::LPW;
    __shared__ __attribute__((aligned(1024))) char lds[NS * S::STAGE_BYTES];
    __shared__ Best red[S::BM * (WN > 1 ? WN - 1 : 1)];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wn = wave % WN, wm = wave / WN;
    const int l32 = lane & 31, kh = lane >> 5;
    const int d = a.d, KS = d / BK;
    const char *W = (const char *)a.W, *H = (const char *)a.H;

    // ---- persistent tile list of this workgroup: runs of (gridDim/8) consecutive tiles per XCD
    const int G = gridDim.x, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, SL = G >> 3;
    auto tile_at = [&](int step) { return (step * 8 + xcd) * SL + slot; };

    // ---- loader constants
    const int rl = lane / CH;                                     // row inside one wave-wide load
    const int cg = (lane % CH) ^ (((wave * RPI + rl) / RPW) % CH);  // global chunk landing at this lane's LDS slot
    // ---- fragment-read constants
    const int swz = (l32 / RPW) % CH;
    const int a_row = (wn * TN * 32 + l32) * BK * 2;              // byte offset of the lane's row in the W tile
    const int b_row = S::W_BYTES + (wm * TM * 32 + l32) * BK * 2; // ... in the H tile

    // issue cursor (tile, k-stage) runs NS-1 stages ahead of the compute cursor
    int i_step = 0, i_ks = 0, i_buf = 0;
    int i_T = tile_at(0), i_mt = 0, i_nt = 0;
    if (i_T < sc.total) tile_of(sc, i_T, i_mt, i_nt);

    auto issue = [&]() {
        // one pipeline stage: the W tile [BN][BK] and the H tile [BM][BK] of (i_mt, i_nt) at k = i_ks*BK
        const int n0 = i_nt * S::BN, m0 = i_mt * S::BM, kbyte = i_ks * BK * 2 + cg * 16;
        char *stage = lds + i_buf * S::STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < LPW; ++j) {
            const int q = j * NW + wave;                          // load index inside the stage (wave-uniform)
            if (j < S::WI / NW) {
                const int row = min(n0 + q * RPI + rl, a.V - 1);  // clamped: ragged tiles stay in bounds
                const char *g = W + (size_t)row * (size_t)(d * 2) + kbyte;
                __builtin_amdgcn_global_load_lds((gbl_void *)g, (lds_void *)(stage + q * 1024), 16, 0, 0);
            } else {
                const int qh = q - S::WI;
                const int row = min(m0 + qh * RPI + rl, a.M - 1);
                const char *g = H + (size_t)row * (size_t)(d * 2) + kbyte;
                __builtin_amdgcn_global_load_lds((gbl_void *)g, (lds_void *)(stage + S::W_BYTES + qh * 1024), 16, 0, 0);
            }
        }
        i_buf = (i_buf + 1 == NS) ? 0 : i_buf + 1;
        if (++i_ks == KS) {
            i_ks = 0;
            i_T = tile_at(++i_step);
            if (i_T < sc.total) tile_of(sc, i_T, i_mt, i_nt);
        }
    };

#pragma unroll
    for (int p = 0; p < NS - 1; ++p)
        if (i_T < sc.total) issue();

    f32x16 acc[TN][TM];
    int c_buf = 0;
    for (int step = 0;; ++step) {
        const int T = tile_at(step);
        if (T >= sc.total) break;
        int mt, nt;
        tile_of(sc, T, mt, nt);
#pragma unroll
        for (int x = 0; x < TN; ++x)
#pragma unroll
            for (int y = 0; y < TM; ++y)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

        for (int ks = 0; ks < KS; ++ks) {
            // stage (T, ks) has landed once at most the NS-2 younger stages are outstanding;
            // when the issue cursor is exhausted fewer are in flight, so wait for everything.
            if (i_T < sc.total) {
                wait_vm_and_barrier<(NS - 2) * LPW>();
                issue();                                  // into the buffer freed by the barrier
            } else {
                wait_vm_and_barrier<0>();
            }
            const char *stage = lds + c_buf * S::STAGE_BYTES;
#pragma unroll
            for (int s = 0; s < BK / 16; ++s) {
                const int pos = ((2 * s + kh) ^ swz) * 16;
                bf16x8 fa[TN], fb[TM];
#pragma unroll
                for (int x = 0; x < TN; ++x) fa[x] = *(const bf16x8 *)(stage + a_row + x * 32 * BK * 2 + pos);
#pragma unroll
                for (int y = 0; y < TM; ++y) fb[y] = *(const bf16x8 *)(stage + b_row + y * 32 * BK * 2 + pos);
#pragma unroll
                for (int x = 0; x < TN; ++x)
#pragma unroll
                    for (int y = 0; y < TM; ++y)
                        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[x], fb[y], acc[x][y], 0, 0, 0);
            }
            c_buf = (c_buf + 1 == NS) ? 0 : c_buf + 1;
        }

        // ---- epilogue: D register r of a lane = vocabulary row 8*(r/4) + 4*(lane/32) + r%4 of its block
        const int v_base = nt * S::BN + wn * TN * 32 + kh * 4;
        float pv[TM];
        int32_t pi[TM];
#pragma unroll
        for (int y = 0; y < TM; ++y) {
            const int lr = wm * TM * 32 + y * 32 + l32;          // verify row inside the tile
            const int row = mt * S::BM + lr;
            float bv = -INFINITY;
            int32_t bi = 0x7fffffff;
#pragma unroll
            for (int x = 0; x < TN; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int v = v_base + x * 32 + (r >> 2) * 8 + (r & 3);
                    const float val = acc[x][y][r];
                    if (v < a.V) {
                        if (DUMP && row < a.M) a.dump[(size_t)row * a.V + v] = val;
                        if (val > bv) {
                            bv = val;
                            bi = v;
                        }
                    }
                }
            const float ov = __shfl_xor(bv, 32);
            const int32_t oi = __shfl_xor(bi, 32);
            if (better(ov, oi, bv, bi)) {
                bv = ov;
                bi = oi;
            }
            if (WN > 1 && wn > 0 && kh == 0) red[(wn - 1) * S::BM + lr] = Best{bv, bi};
            pv[y] = bv;
            pi[y] = bi;
        }
        // LDS writes of `red` done and visible; do not wait for the prefetch loads in flight
        if (WN > 1) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (wn == 0 && kh == 0) {
#pragma unroll
            for (int y = 0; y < TM; ++y) {
                const int lr = wm * TM * 32 + y * 32 + l32;
                const int row = mt * S::BM + lr;
                float bv = pv[y];
                int32_t bi = pi[y];
#pragma unroll
                for (int w = 1; w < WN; ++w) {
                    const Best o = red[(w - 1) * S::BM + lr];
                    if (better(o.v, o.i, bv, bi)) {
                        bv = o.v;
                        bi = o.i;
                    }
                }
                if (row < a.M) a.part[(size_t)row * a.nblocks + nt] = Best{bv, bi};
            }
        }
        // `red` is next written after the k-loop barriers of the following tile: no extra barrier
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
    int grid = (num_cus / 8) * 8;
    if (grid < 8) grid = 8;
    // no more workgroups than tiles (rounded up to the XCD count so that the run mapping holds)
    const int need = ((sc.total + 7) / 8) * 8;
    if (grid > need) grid = need;
    if (a.dump)
        hipLaunchKernelGGL((k_lm_head_mfma<S, true>), dim3(grid), dim3(S::NW * 64), 0, s, a, sc);
    else
        hipLaunchKernelGGL((k_lm_head_mfma<S, false>), dim3(grid), dim3(S::NW * 64), 0, s, a, sc);
    return hipGetLastError();
}

}  // namespace

int lm_head_mfma_blocks(int variant, int V)
{
    const int bn = variant == AJ_KERNEL_STREAM ? StreamShape::BN : BigShape::BN;
    return (V + bn - 1) / bn;
}

bool lm_head_mfma_supports(int variant, int M, int V, int d)
{
    if (M <= 0 || V <= 0) return false;
    if (variant == AJ_KERNEL_STREAM) return d % StreamShape::BK == 0 && M <= StreamShape::BM;
    if (variant == AJ_KERNEL_BIG) return d % BigShape::BK == 0;
    return false;
}

hipError_t lm_head_mfma_bf16(int variant, const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    if (variant == AJ_KERNEL_STREAM) return launch<StreamShape>(a, num_cus, 1, s);
    return launch<BigShape>(a, num_cus, 8, s);
}

}  // namespace aj
