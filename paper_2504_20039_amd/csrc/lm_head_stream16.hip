// LM head (step 1) + running greedy maximum (first half of step 2) for the W_lm-streaming regime:
// at most 32 verify rows, d_t = 2048 or 4096.  HBM-bound: the only operand that moves is W_lm.
//
//   * hidden_t lives in REGISTERS for the whole kernel.  The 8 waves of a workgroup split the k range:
//     wave w owns k in [w*d_t/8, (w+1)*d_t/8) and keeps the v_mfma_f32_16x16x32_bf16 B-fragments
//     (column = verify row) of that range: d_t/256 k steps x 2 row blocks x 4 VGPRs = 128 VGPRs at
//     d_t = 4096.
//   * tiles of 16 vocabulary rows.  Every wave streams ITS OWN k slice of the tile - 16 rows x 512 B per
//     stage, eight 1 KB direct-to-LDS loads of two whole 512-byte row segments each - through a private
//     two-buffer ring, so the load pipeline needs no workgroup barrier: a wave issues its next stage,
//     waits for its own loads of the current one (s_waitcnt vmcnt), and computes it (8 fragment reads,
//     16 MFMAs).  One stage per wave, 64 KB per compute unit, is always in flight.  Few rows with long
//     contiguous runs is what the HBM likes best: load-only kernels with this pattern read 6.9 TB/s on
//     this chip, with 32-row tiles 6.7, with 128 rows x 256 B 5.0.
//   * W_lm is read exactly once, so its loads carry the non-temporal hint (6.2 -> 6.5 TB/s).
//   * per tile the 8 partial 16x32 logit blocks meet in LDS and every wave adds up one eighth of the block
//     (one accumulator register index: verify rows 16b..16b+15 x vocabulary rows 4q+r for its (b, r)),
//     keeping a running (max, lowest index) per lane: no wave does more than the others, and the one
//     barrier of this exchange (its area is double-buffered) is the only one of a tile.  Lane l holds verify row l % 16 and
//     vocabulary row 4*(l/16) + r of the tile: ascending over a workgroup's tiles, so strict > keeps the
//     lowest index; the 4 waves of a row block are merged once, at the end.
//   * FP8W: W_lm stored as OCP FP8 E4M3 (one byte per element, d_t = 4096): half the bytes to stream.  A
//     stage is still 16 rows x 512 B, now 512 k elements = 16 k steps; a lane reads its 8 k elements as 8
//     bytes and widens them exactly to bf16 (v_cvt_pk_f32_fp8, then the upper halves of the floats: E4M3 has
//     4 significant bits), so the MFMAs and every value they see are those of the bf16 path.
#include "../../include/aj.h"
#include "aj_internal.h"
#include "lds_pipeline.h"

namespace aj {

namespace {

constexpr int S16_WAVES = 8;
constexpr int S16_ROWS = 16;                    // vocabulary rows per tile
constexpr int S16_SEG = 512;                    // bytes of each row per stage (256 k elements = 8 k steps)
constexpr int S16_STAGE = S16_ROWS * S16_SEG;   // 8 KB = eight 1 KB loads
constexpr int S16_LOADS = S16_STAGE / 1024;

template <int NST, bool DUMP, bool TOPK, bool SAMPLE, bool FP8W>   // NST stages per tile and wave: d_t = NST * 2048 (4096 with FP8W)
__global__ __launch_bounds__(S16_WAVES * 64) void k_lm_head_stream16(LmHeadArgs a, int ntiles)
{
    constexpr int KSTEPS = FP8W ? 16 : 8;       // k steps of 32 per stage (512 B of a row)
    static_assert(!FP8W || NST == 1, "FP8 W_lm: one 512-byte stage per wave and tile");
    __shared__ __attribute__((aligned(1024))) char lds[S16_WAVES * 2 * S16_STAGE];   // per wave: 2 stage buffers
    __shared__ float redk[2 * S16_WAVES * 7 * 64];   // partial logit blocks: [tile parity][share][source slot][lane]
    __shared__ Best fin[32 * 4];                // final merge of the 4 waves of a row block
    __shared__ int32_t finc[32 * 4];

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, q4 = lane >> 4;
    const char *W = (const char *)a.W, *H = (const char *)a.H;
    const uint32_t rowbytes = (uint32_t)a.d * (FP8W ? 1u : 2u);    // of W_lm
    const uint32_t kslice = (uint32_t)wave * (NST * S16_SEG);      // byte offset of this wave's k range in a W_lm row
    const uint32_t hslice = kslice * (FP8W ? 2u : 1u);             // ... in a hidden_t row (always bf16)
    const uint32_t lds_mine = lds_offset_of(lds) + wave * (2 * S16_STAGE);
    const char *lds_rd = lds + wave * (2 * S16_STAGE);

    // persistent tile list: runs of (gridDim/8) consecutive tiles per XCD
    const int G = gridDim.x, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, SL = G >> 3;
    auto tile_at = [&](int step) { return (step * 8 + xcd) * SL + slot; };

    // loader: load j of a stage covers tile rows 2j, 2j+1; lane i fills slot (row i/32, chunk i%32) and
    // fetches global chunk (i%32) ^ row (XOR on the low 4 bits: conflict-free fragment reads)
    const int rsub = lane >> 5;
    auto issue = [&](int tile, int st, int buf) {    // stage st of `tile` (this wave's k slice) into buffer buf
        const uint32_t dst = lds_mine + buf * S16_STAGE;
        const uint32_t koff = kslice + (uint32_t)(st * S16_SEG);
#pragma unroll
        for (int j = 0; j < S16_LOADS; ++j) {
            const int tr = 2 * j + rsub;
            const int row = min(tile * S16_ROWS + tr, a.V - 1);    // clamped: a ragged last tile stays in bounds
            lds_dma_16_nt(W, __umul24(row, rowbytes) + koff + (uint32_t)(((lane & 31) ^ tr) * 16), dst + j * 1024);
        }
    };
    // A fragment (16 vocabulary rows x 32 k) of k step t: lane (row l16, k group q4) reads chunk 4t + q4
    const int a_base = l16 * S16_SEG;

    // hidden_t fragments of this wave's k range: block b = verify rows 16b..16b+15 (clamped)
    bf16x8 hf[NST * KSTEPS][2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const char *hrow = H + (size_t)min(b * 16 + l16, a.M - 1) * ((size_t)a.d * 2) + hslice;
#pragma unroll
        for (int t = 0; t < NST * KSTEPS; ++t) hf[t][b] = *(const bf16x8 *)(hrow + (t * 32 + q4 * 8) * 2);
    }
    // this wave's share of every tile: accumulator register (bsel, rsel); its verify row and, for the
    // top-K baseline, that row's draft token
    const int bsel = wave >> 2, rsel = wave & 3;
    const int myrow = bsel * 16 + l16;
    float th = INFINITY;
    int32_t tk = -1, run_c = 0;
    if (TOPK) {
        th = a.thr[min(myrow, a.M - 1)];
        tk = a.thr_tok[min(myrow, a.M - 1)];
    }
    uint32_t klo = 0, khi = 0;          // sampling mode: the row's noise key
    if (SAMPLE) {
        const uint64_t key = a.key[min(myrow, a.M - 1)];
        klo = (uint32_t)key;
        khi = (uint32_t)(key >> 32);
    }
    // make the compiler retire these loads here: its waits must not land inside the pipelined loop,
    // where they would drain the kernel's own asynchronous loads
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int t = 0; t < NST * KSTEPS; ++t) asm volatile("" : "+v"(hf[t][b]));
    asm volatile("" : "+v"(th), "+v"(tk), "+v"(klo), "+v"(khi));

    float run_v = -INFINITY;
    int32_t run_i = 0x7fffffff;

    // Stages of this wave are numbered f = step * NST + st and use buffer f & 1.  At stage f the wave first
    // issues stage f+1 into the other buffer (its fragments went to registers during stage f-1), then
    // waits until only those loads are outstanding - loads complete in order - and computes stage f.
    int T = tile_at(0);
    if (T < ntiles) issue(T, 0, 0);
    for (int step = 0; T < ntiles; ++step) {
        const int T2 = tile_at(step + 1);
        const bool have_next = T2 < ntiles;
        f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int st = 0; st < NST; ++st) {
            const int cur = NST == 2 ? st : (step & 1);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // the other buffer's fragment reads are done
            if (st + 1 < NST) {
                issue(T, st + 1, cur ^ 1);
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(S16_LOADS) : "memory");
            } else if (have_next) {
                issue(T2, 0, cur ^ 1);
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(S16_LOADS) : "memory");
            } else {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            const char *buf = lds_rd + cur * S16_STAGE;
#pragma unroll
            for (int t = 0; t < KSTEPS; ++t) {
                bf16x8 fa;
                if (FP8W) {
                    // 8 k elements = 8 bytes: 16-byte chunk 2t + q4/2 of the row (swizzled), its half q4 % 2
                    const uint2 raw = *(const uint2 *)(buf + a_base + (((2 * t + (q4 >> 1)) ^ l16) * 16) + (q4 & 1) * 8);
                    fa = fp8x8_to_bf16x8(raw);
                } else {
                    fa = *(const bf16x8 *)(buf + a_base + (((4 * t + q4) ^ l16) * 16));
                }
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, hf[st * KSTEPS + t][0], acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, hf[st * KSTEPS + t][1], acc[1], 0, 0, 0);
            }
        }

        // ---- the 8 partial blocks meet in LDS; wave w adds up register (bsel, rsel) = share w of all of them.
        // A wave keeps its own share in registers and writes the 7 others; the exchange area is double-buffered
        // by tile parity, so ONE barrier per tile suffices: a wave that writes buffer p again (two tiles later) has
        // passed the barrier in between, which every wave reaches only after its reads of buffer p.
        float *rk = redk + (step & 1) * (S16_WAVES * 7 * 64);
        float own = 0.f;
#pragma unroll
        for (int s = 0; s < S16_WAVES; ++s) {
            const float val = acc[s >> 2][s & 3];
            if (s == wave) own = val;
            else rk[(s * 7 + (wave < s ? wave : wave - 1)) * 64 + lane] = val;     // share s, slot of source wave
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < S16_WAVES; ++w)      // ascending source wave, whichever wave adds
            sum += w == wave ? own : rk[(wave * 7 + (w < wave ? w : w - 1)) * 64 + lane];
        const int v = T * S16_ROWS + q4 * 4 + rsel;
        if (v < a.V) {
            if (DUMP && myrow < a.M) a.dump[(size_t)myrow * a.V + v] = sum;
            if (SAMPLE) sum = fmaf(sum, a.inv_temp, gumbel_noise(klo, khi, (uint32_t)v));
            if (sum > run_v) {
                run_v = sum;
                run_i = v;
            }
            if (TOPK) run_c += ranks_before(sum, v, th, tk);
        }
        T = T2;
    }

    // ---- merge: the 4 vocabulary sub-rows of a lane group, then the 4 waves of a row block
    float bv = run_v;
    int32_t bi = run_i, cn = run_c;
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const float ov = __shfl_xor(bv, off);
        const int32_t oi = __shfl_xor(bi, off);
        if (better(ov, oi, bv, bi)) {
            bv = ov;
            bi = oi;
        }
        cn += __shfl_xor(cn, off);
    }
    if (q4 == 0) {
        fin[myrow * 4 + rsel] = Best{bv, bi};
        finc[myrow * 4 + rsel] = cn;
    }
    __syncthreads();
    if (rsel == 0 && q4 == 0 && myrow < a.M) {
        cn = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const Best o = fin[myrow * 4 + r];
            if (r == 0 || better(o.v, o.i, bv, bi)) {
                bv = o.v;
                bi = o.i;
            }
            cn += finc[myrow * 4 + r];
        }
        a.part[(size_t)myrow * a.nblocks + blockIdx.x] = Best{bv, bi};
        if (TOPK) a.cnt[(size_t)myrow * a.nblocks + blockIdx.x] = cn;
    }
}

template <int NST, bool FP8W>
hipError_t launch16(const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    const int ntiles = (a.V + S16_ROWS - 1) / S16_ROWS;
    const int grid = persistent_grid(num_cus, ntiles);
    // the top-K baseline's counting and the sampling noise are separate instantiations: the greedy judge path
    // pays nothing for them
    if (a.dump)
        hipLaunchKernelGGL((k_lm_head_stream16<NST, true, false, false, FP8W>), dim3(grid), dim3(S16_WAVES * 64), 0, s, a, ntiles);
    else if (a.thr)
        hipLaunchKernelGGL((k_lm_head_stream16<NST, false, true, false, FP8W>), dim3(grid), dim3(S16_WAVES * 64), 0, s, a, ntiles);
    else if (a.key)
        hipLaunchKernelGGL((k_lm_head_stream16<NST, false, false, true, FP8W>), dim3(grid), dim3(S16_WAVES * 64), 0, s, a, ntiles);
    else
        hipLaunchKernelGGL((k_lm_head_stream16<NST, false, false, false, FP8W>), dim3(grid), dim3(S16_WAVES * 64), 0, s, a, ntiles);
    return hipGetLastError();
}

}  // namespace

bool lm_head_stream16_supports(int M, int V, int d)
{
    if (M <= 0 || M > 32 || V <= 0) return false;
    if (d != 4096 && d != 2048) return false;
    return (uint64_t)V * d * 2 < (1ull << 32) && V < (1 << 24);   // 32-bit lane offsets, 24-bit multiply
}

int lm_head_stream16_blocks(int V, int num_cus) { return persistent_grid(num_cus, (V + S16_ROWS - 1) / S16_ROWS); }

hipError_t lm_head_stream16_bf16(const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    return a.d == 4096 ? launch16<2, false>(a, num_cus, s) : launch16<1, false>(a, num_cus, s);
}

// W_lm in OCP FP8 E4M3, hidden_t in bf16: M <= 32 and d_t = 4096 only
bool lm_head_stream16_fp8w_supports(int M, int V, int d)
{
    return M > 0 && M <= 32 && V > 0 && d == 4096 && (uint64_t)V * d < (1ull << 32) && V < (1 << 24);
}

hipError_t lm_head_stream16_fp8w(const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    return launch16<1, true>(a, num_cus, s);
}

}  // namespace aj
