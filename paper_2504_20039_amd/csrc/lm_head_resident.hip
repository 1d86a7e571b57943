// LM head (step 1) + greedy maximum (first half of step 2) for the W_lm-streaming regime at up to 128 verify
// rows and any hidden size that is a multiple of 256: the logits stay in registers for the WHOLE kernel.
//
// hidden_t of 33..128 rows at d_t = 8192 fits neither the registers nor the LDS of a compute unit, so a kernel
// that walks vocabulary tiles has to stream the hidden_t tile again for every W_lm tile (as much L2 -> CU
// traffic as W_lm itself at 128 x 128).  What does fit is the OUTPUT: a compute unit's share of the vocabulary
// (V / 256 = 501 rows) x 128 verify rows x 4 bytes = 256 KB of its 512 KB of registers.  So the loops are turned
// inside out:
//
//   * every wave owns 64 vocabulary rows (4 blocks of 16; 8 waves = 512 rows per workgroup, one workgroup per
//     compute unit) and keeps their logits against all verify rows in accumulators - 4 x MB blocks of
//     v_mfma_f32_16x16x32_bf16, MB = ceil(M / 16) <= 8 - from the first k element to the last; the greedy
//     maximum is taken once, at the end.  A vocabulary larger than grid x 512 rows takes several such passes;
//   * k advances in slabs of 256 elements.  The hidden_t slab (M rows x 512 B) is staged in LDS, double
//     buffered, by asynchronous direct-to-LDS loads shared among the 8 waves: ONE workgroup barrier per slab,
//     and every compute unit reads hidden_t exactly once per pass;
//   * W_lm goes global -> registers, never through LDS, by non-temporal buffer loads that the compiler's own
//     s_waitcnt accounting tracks.  A wave visits its 4 blocks one after the other within a slab; the 8 loads of
//     a visit (16 rows x 512 contiguous bytes) go out in one burst, one visit before their use, so 8 KB per wave
//     (64 KB per compute unit) are always in flight.  Every load instruction asks for WHOLE 128-byte lines (8 rows
//     x 128 B): with the non-temporal bit, half lines per instruction (the MFMA's own 16 rows x 64 B) stream at
//     5.9 TB/s in a load-only kernel, whole lines at 6.6.  The halves reach the MFMA layout by one DPP rotation
//     per register (see w_load / half_of).  Measured on the 70B shapes: 16 x 64 B loads refilled one by one 5.5
//     TB/s, the same in bursts per block 5.9, whole lines 6.7; a deeper ring changed nothing;
//   * FP8W: W_lm stored as OCP FP8 E4M3.  A 16-byte load then holds 16 k elements = the lane's share of TWO k
//     steps; the bytes are widened exactly to bf16 in registers, so the MFMAs see the values of the bf16 path.
#include "../../include/aj.h"
#include "aj_internal.h"
#include "lds_pipeline.h"

namespace aj {

namespace {

constexpr int RS_WAVES = 8;
constexpr int RS_NBW = 4;                       // 16-row vocabulary blocks per wave and pass
constexpr int RS_KS = 256;                      // k elements per slab
constexpr int RS_HROW = RS_KS * 2;              // bytes of a hidden_t row per slab

template <int MB, bool FP8W, bool DUMP, bool TOPK, bool SAMPLE, bool JUDGE = false>
__global__ __launch_bounds__(RS_WAVES * 64) void k_lm_head_resident(LmHeadArgs a, int passes, int rot_step)
{
    constexpr int HSLAB = MB * 16 * RS_HROW;                 // bytes of a hidden_t slab in LDS
    constexpr int WSEG = FP8W ? RS_KS : RS_KS * 2;           // bytes of a W_lm row per slab
    constexpr int USES = WSEG / 64 * RS_NBW;                 // fragment loads per wave and slab: 32 (bf16), 16 (FP8)
    // hidden_t fragment sets: two (the next pair's k step is read during this one's MFMAs) while registers allow
    constexpr int HFB = MB * (FP8W ? 2 : 1) <= 6 ? 2 : 1;
    // A wave visits its 4 vocabulary blocks one after the other within a slab.  The fragments of a visit (UPV
    // loads of 1 KB: 16 rows x 64 * UPV contiguous bytes) are requested in one burst, AHEAD visits before their use,
    // into one of NG register groups.
    constexpr int UPV = USES / RS_NBW;                       // 8 (bf16), 4 (FP8)
    // PV: a visit covers a PAIR of blocks over half of the slab (32 rows x 64 * UPV / 2 bytes) instead of one block over
    // all of it, and the two blocks share the hidden_t fragments of each k step: half the LDS reads, which is what
    // bounds the kernel from 6 row blocks on and with FP8 weights (twice the MFMAs and fragment reads per streamed byte)
    constexpr bool PV = FP8W || MB <= 7;
    constexpr int LPB = UPV / 2, PPV = UPV / 2;              // PV: loads per block and pieces per visit
    constexpr int NG = FP8W && MB <= 5 ? 4 : 2, AHEAD = NG - 1;
    __shared__ __attribute__((aligned(1024))) char lds[2 * HSLAB];
    __shared__ Best fin[RS_WAVES][MB * 16];
    __shared__ int32_t finc[TOPK ? RS_WAVES : 1][MB * 16];

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, q4 = lane >> 4;
    const char *W = (const char *)a.W, *H = (const char *)a.H;
    const uint32_t wrow = (uint32_t)a.d * (FP8W ? 1u : 2u);     // bytes of a W_lm row
    const uint32_t hrow = (uint32_t)a.d * 2u;                   // bytes of a hidden_t row
    const int NS = a.d / RS_KS;                                 // slabs per pass
    const int nwaves = gridDim.x * RS_WAVES, gw = blockIdx.x * RS_WAVES + wave;
    const int rot = (int)((blockIdx.x * (unsigned)rot_step) % (unsigned)NS);   // this workgroup's first slab
    const int total = passes * NS;

    // ---- hidden_t slab loader: load i of wave w fills LDS rows 2*(8i + w) and the next; lane (row half lane/32,
    // chunk slot lane%32) fetches global chunk slot ^ (row % 16), so that fragment reads are conflict free
    const uint32_t lds_base = lds_offset_of(lds);
    const int tr0 = 2 * wave + (lane >> 5);             // the lane's LDS row in load 0; load i: + 16 * i
    const uint32_t hchunk = (uint32_t)(((lane & 31) ^ (tr0 & 15)) * 16);
    auto load_h = [&](int slab, int buf) {
        const char *hb = H + (size_t)slab * RS_HROW;
#pragma unroll
        for (int i = 0; i < MB; ++i)    // rows beyond M repeat the last one (their logits are never looked at)
            lds_dma_16(hb, __umul24(min(tr0 + 16 * i, a.M - 1), hrow) + hchunk,
                       lds_base + buf * HSLAB + (i * RS_WAVES + wave) * 1024);
    };
    // slab of iteration `it` (k rotation per workgroup)
    auto slab_of = [&](int it) {
        int s = it % NS + rot;
        return s >= NS ? s - NS : s;
    };
    // W_lm fragment loads are buffer loads (lane offset + uniform offset + immediate) with the non-temporal bit -
    // W_lm is read exactly once - as an operand of the instruction, which no compiler pass can drop.  With that
    // bit a load instruction has to ask for WHOLE 128-byte lines: 16 rows x 64 B per instruction (the MFMA's own
    // layout) streams at 5.9 TB/s in a load-only kernel, 8 rows x 128 B at 6.6.  So load 2*pr + h of a block
    // visit covers rows 8h .. 8h+7 of the block x line pr of the slab segment: lane (l16, q4) asks for row
    // l16 % 8 and the 16 bytes at (q4 + 4 * (l16 / 8)) * 16 of the line.  The two loads of a line pair then hold,
    // for 64-byte half c of the line, rows 0..7 in lanes l16 / 8 == c of the first and rows 8..15 in the same
    // lanes of the second: one rotation by 8 lanes within each group of 16 (a DPP move) per register gives the
    // MFMA layout (lane l16 <-> row l16) of both halves.
    const __amdgpu_buffer_rsrc_t wres =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.W, 0, (int)((uint32_t)a.V * wrow), 0x00020000);
    // first vocabulary row of this wave in the pass of iteration `it`
    auto w_first = [&](int it) { return ((it / NS) * nwaves + gw) * (RS_NBW * 16); };
    const int r8 = l16 & 7;
    const uint32_t cbyte = (uint32_t)(q4 + 4 * (l16 >> 3)) * 16u;
    // load j = 2*pr + h of the visit to block blk of the wave whose first row is v0; slab_off: byte offset of the
    // slab in a row (uniform).  Rows are clamped into the vocabulary (their logits are never looked at).
    // JUDGE: the judge's target weights clf_w[0:d] are one more vocabulary row, the first of the 16-row block that
    // follows the vocabulary's last one (Section 3.2: the regression fused with the LM head); all 16 lanes rows of that
    // block read the same row, whose logits go to a.zt instead of the maximum.
    const int vj = (a.V + 15) / 16 * 16;
    const __amdgpu_buffer_rsrc_t jres =
        __builtin_amdgcn_make_buffer_rsrc((void *)(JUDGE ? a.judge_w : a.W), 0, (int)wrow, 0x00020000);
    auto w_load = [&](int v0, int slab_off, int blk, int j) {
        if (JUDGE && v0 + blk * 16 == vj)       // wave-uniform
            return __builtin_amdgcn_raw_buffer_load_b128(jres, (int)cbyte + (j >> 1) * 128, slab_off, 0);
        const int row = min(v0 + blk * 16 + (j & 1) * 8 + r8, a.V - 1);
        return __builtin_amdgcn_raw_buffer_load_b128(wres, (int)(__umul24(row, wrow) + cbyte) + (j >> 1) * 128,
                                                     slab_off, 2 /* nt */);
    };
    // 64-byte half c of a line pair (x: rows 0..7, y: rows 8..15) in MFMA layout
    auto half_of = [&](const u32x4 &x, const u32x4 &y, int c) {
        u32x4 r;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            r[k] = c == 0 ? (uint32_t)__builtin_amdgcn_update_dpp((int)x[k], (int)y[k], 0x128 /* row_ror:8 */, 0xF, 0xC, false)
                          : (uint32_t)__builtin_amdgcn_update_dpp((int)y[k], (int)x[k], 0x128, 0xF, 0x3, false);
        return r;
    };

    f32x4 acc[RS_NBW][MB];
#pragma unroll
    for (int y = 0; y < MB; ++y) {
#pragma unroll
        for (int b = 0; b < RS_NBW; ++b) acc[b][y] = f32x4{0.f, 0.f, 0.f, 0.f};
        // the wave's running (maximum, lowest index) and top-K count per verify row live in its own row of
        // `fin` between passes, not in registers; only this wave touches them until the final merge
        if (q4 == 0) {
            fin[wave][y * 16 + l16] = Best{-INFINITY, 0x7fffffff};
            if (TOPK) finc[wave][y * 16 + l16] = 0;
        }
    }

    // a wave whose first row lies beyond the vocabulary in pass 0 never computes: it only helps to stage hidden_t
    const bool active = gw * (RS_NBW * 16) < (JUDGE ? vj + 16 : a.V);

    int wcur, wnxt;
    int scur = slab_of(0) * WSEG, snxt = 0;          // byte offset of the slab in a W_lm row
    u32x4 ring[NG][UPV];
    load_h(slab_of(0), 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    wcur = w_first(0);
    if (active) {
#pragma unroll
        for (int v = 0; v < AHEAD; ++v)
#pragma unroll
            for (int p = 0; p < UPV; ++p)
                ring[v][p] = PV ? w_load(wcur, scur, 2 * (v >> 1) + p / (UPV / 2), (v & 1) * (UPV / 2) + p % (UPV / 2))
                                : w_load(wcur, scur, v, p);
    }

    for (int it = 0; it < total; ++it) {
        const int buf = it & 1;
        // slab `it` has landed: its loads are older than the USES fragment loads this wave has issued since
        if (it > 0) {
            if (active) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(USES) : "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        // every wave's part of the slab is in LDS, and every wave has finished reading the other buffer
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        const bool more = it + 1 < total;
        if (more) load_h(slab_of(it + 1), buf ^ 1);
        // after the last slab the ring refills with data nobody uses
        wnxt = w_first(more ? it + 1 : it);
        snxt = slab_of(more ? it + 1 : it) * WSEG;

        if (active) {
            const char *hs = lds + buf * HSLAB + l16 * RS_HROW;
            constexpr int NK = FP8W ? 2 : 1;      // k steps per fragment load
            // hidden_t fragments of the k step(s) of piece p of the slab (the same for every vocabulary block)
            auto read_h = [&](int p, bf16x8(&hf)[NK][MB]) {
#pragma unroll
                for (int y = 0; y < MB; ++y)
#pragma unroll
                    for (int k = 0; k < NK; ++k) {
                        // FP8W: the lane's 16 bytes are k elements 64*p + 16*q4 .. + 15, two k steps of 8 each
                        const int chunk = FP8W ? 8 * p + 2 * q4 + k : 4 * p + q4;
                        hf[k][y] = *(const bf16x8 *)(hs + y * 16 * RS_HROW + ((chunk ^ l16) * 16));
                    }
            };
            // The order below is the order of execution (sched_barrier): left to itself the compiler sinks every
            // load to just before its use, which empties the ring.
            bf16x8 hf[HFB][NK][MB];
            read_h(0, hf[0]);
#pragma unroll
            for (int v = 0; v < RS_NBW; ++v) {
                // a burst of UPV loads: the 16 rows of the block visited AHEAD visits from now, 64 * UPV contiguous
                // bytes of each, into the registers of the visit that has just ended
                {
                    const int vv = v + AHEAD;
#pragma unroll
                    for (int p = 0; p < UPV; ++p) {
                        const int vs = vv < RS_NBW ? vv : vv - RS_NBW;           // visit within its slab
                        // block and load index (2 * line + rows half) within the slab of load p of visit vs
                        const int blk = PV ? 2 * (vs >> 1) + p / LPB : vs;
                        const int j = PV ? (vs & 1) * LPB + p % LPB : p;
                        ring[vv % NG][p] = vv < RS_NBW ? w_load(wcur, scur, blk, j) : w_load(wnxt, snxt, blk, j);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                // steps of the visit: a step is one 64-byte piece of the slab (k step(s) P) for the visit's block(s)
                constexpr int NSTEP = PV ? PPV : UPV, NBS = PV ? 2 : 1;
                // piece of the slab of step u (counted over the slab's 4 visits)
                auto piece_of = [&](int u) { return PV ? ((u / NSTEP) & 1) * PPV + u % NSTEP : u % NSTEP; };
#pragma unroll
                for (int q = 0; q < NSTEP; ++q) {
                    const int u = v * NSTEP + q, cur = HFB == 2 ? u & 1 : 0;
                    if (HFB == 2 && u + 1 < 4 * NSTEP) read_h(piece_of(u + 1), hf[cur ^ 1]);
#pragma unroll
                    for (int bb = 0; bb < NBS; ++bb) {
                        const int base = PV ? bb * LPB + (q >> 1) * 2 : (q & ~1), blk = PV ? 2 * (v >> 1) + bb : v;
                        const u32x4 raw = half_of(ring[v % NG][base], ring[v % NG][base + 1], q & 1);
                        if (FP8W) {
                            const bf16x8 f0 = fp8x8_to_bf16x8(uint2{raw[0], raw[1]}), f1 = fp8x8_to_bf16x8(uint2{raw[2], raw[3]});
#pragma unroll
                            for (int y = 0; y < MB; ++y) {
                                acc[blk][y] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0, hf[cur][0][y], acc[blk][y], 0, 0, 0);
                                acc[blk][y] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f1, hf[cur][NK - 1][y], acc[blk][y], 0, 0, 0);
                            }
                        } else {
                            const bf16x8 f0 = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
                            for (int y = 0; y < MB; ++y)
                                acc[blk][y] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0, hf[cur][0][y], acc[blk][y], 0, 0, 0);
                        }
                    }
                    if (HFB == 1 && u + 1 < 4 * NSTEP) read_h(piece_of(u + 1), hf[0]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        wcur = wnxt;
        scur = snxt;

        if ((it + 1) % NS == 0 && active) {
            // ---- end of a pass: lane (l16, q4) holds verify row 16y + l16 against vocabulary rows
            // v0 + 16b + 4*q4 + r of its wave, ascending in (b, r): strict > keeps the lowest
            const int v0 = ((it / NS) * nwaves + gw) * (RS_NBW * 16);
#pragma unroll
            for (int y = 0; y < MB; ++y) {
                const int row = y * 16 + l16, rowc = min(row, a.M - 1);
                float th = INFINITY;
                int32_t tk = -1;
                if (TOPK) {
                    th = a.thr[rowc];
                    tk = a.thr_tok[rowc];
                }
                uint32_t klo = 0, khi = 0;
                if (SAMPLE) {
                    const uint64_t key = a.key[rowc];
                    klo = (uint32_t)key;
                    khi = (uint32_t)(key >> 32);
                }
                float bv = -INFINITY;
                int32_t bi = 0x7fffffff, cn = 0;
#pragma unroll
                for (int b = 0; b < RS_NBW; ++b) {
                    if (JUDGE && v0 + b * 16 == vj && q4 == 0 && row < a.M) a.zt[row] = acc[b][y][0];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int v = v0 + b * 16 + q4 * 4 + r;
                        float val = acc[b][y][r];
                        if (v < a.V) {
                            if (DUMP && row < a.M) a.dump[(size_t)row * a.V + v] = val;
                            if (SAMPLE) val = fmaf(val, a.inv_temp, gumbel_noise(klo, khi, (uint32_t)v));
                            if (val > bv) {
                                bv = val;
                                bi = v;
                            }
                            if (TOPK) cn += ranks_before(val, v, th, tk);
                        }
                    }
                    acc[b][y] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
                // the 4 vocabulary sub-rows of a lane group, then what earlier passes left
#pragma unroll
                for (int off = 16; off <= 32; off <<= 1) {
                    const float ov = __shfl_xor(bv, off);
                    const int32_t oi = __shfl_xor(bi, off);
                    if (better(ov, oi, bv, bi)) {
                        bv = ov;
                        bi = oi;
                    }
                    if (TOPK) cn += __shfl_xor(cn, off);
                }
                if (q4 == 0) {
                    const Best o = fin[wave][row];
                    if (better(bv, bi, o.v, o.i)) fin[wave][row] = Best{bv, bi};
                    if (TOPK) finc[wave][row] += cn;
                }
            }
            // the slab wait above counts this wave's loads: let the logit dump's stores retire here
            if (DUMP) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
    }

    // ---- merge the 8 waves
    __syncthreads();
    if ((int)threadIdx.x < MB * 16 && (int)threadIdx.x < a.M) {
        const int row = threadIdx.x;
        Best best = fin[0][row];
        int32_t cn = TOPK ? finc[0][row] : 0;
#pragma unroll
        for (int w = 1; w < RS_WAVES; ++w) {
            const Best o = fin[w][row];
            if (better(o.v, o.i, best.v, best.i)) best = o;
            if (TOPK) cn += finc[w][row];
        }
        a.part[(size_t)row * a.nblocks + blockIdx.x] = best;
        if (TOPK) a.cnt[(size_t)row * a.nblocks + blockIdx.x] = cn;
    }
}

int resident_grid(int V, int num_cus)
{
    const int nb = (V + 15) / 16;                                        // 16-row vocabulary blocks
    return persistent_grid(num_cus, (nb + RS_WAVES * RS_NBW - 1) / (RS_WAVES * RS_NBW));
}

template <int MB, bool FP8W>
hipError_t launch_resident(const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    const bool judge = a.judge_w != nullptr;
    const int grid = resident_grid(a.V + 16, num_cus);      // = lm_head_resident_blocks: one partial per workgroup
    const int nb = (a.V + 15) / 16 + (judge ? 1 : 0), per_pass = grid * RS_WAVES * RS_NBW;
    const int passes = (nb + per_pass - 1) / per_pass;
    // workgroups start at different slabs (5 apart): at any moment the chip reads many k offsets of W_lm, not the
    // same column of every row
    const int rot_step = 5;
    const dim3 g(grid), b(RS_WAVES * 64);
    if (a.dump) hipLaunchKernelGGL((k_lm_head_resident<MB, FP8W, true, false, false>), g, b, 0, s, a, passes, rot_step);
    else if (a.thr) hipLaunchKernelGGL((k_lm_head_resident<MB, FP8W, false, true, false>), g, b, 0, s, a, passes, rot_step);
    else if (a.key) hipLaunchKernelGGL((k_lm_head_resident<MB, FP8W, false, false, true>), g, b, 0, s, a, passes, rot_step);
    else if (judge && !FP8W) hipLaunchKernelGGL((k_lm_head_resident<MB, false, false, false, false, true>), g, b, 0, s, a, passes, rot_step);
    else hipLaunchKernelGGL((k_lm_head_resident<MB, FP8W, false, false, false>), g, b, 0, s, a, passes, rot_step);
    return hipGetLastError();
}

template <bool FP8W>
hipError_t dispatch_resident(const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    switch ((a.M + 15) / 16) {
        case 1: return launch_resident<1, FP8W>(a, num_cus, s);
        case 2: return launch_resident<2, FP8W>(a, num_cus, s);
        case 3: return launch_resident<3, FP8W>(a, num_cus, s);
        case 4: return launch_resident<4, FP8W>(a, num_cus, s);
        case 5: return launch_resident<5, FP8W>(a, num_cus, s);
        case 6: return launch_resident<6, FP8W>(a, num_cus, s);
        case 7: return launch_resident<7, FP8W>(a, num_cus, s);
        case 8: return launch_resident<8, FP8W>(a, num_cus, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool lm_head_resident_supports(int M, int V, int d, bool fp8w)
{
    if (M <= 0 || M > 128 || V <= 0 || d <= 0 || d % RS_KS != 0) return false;
    // 32-bit lane offsets, 24-bit multiplies
    if ((uint64_t)V * d * (fp8w ? 1 : 2) >= (1ull << 32) || (uint64_t)M * d * 2 >= (1ull << 32)) return false;
    return V < (1 << 24) && d * 2 < (1 << 24);
}

// V + 16: room for the fused judge row's block, whether it is used or not (a neutral partial costs nothing)
int lm_head_resident_blocks(int V, int num_cus) { return resident_grid(V + 16, num_cus); }

hipError_t lm_head_resident_bf16(const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    return dispatch_resident<false>(a, num_cus, s);
}

hipError_t lm_head_resident_fp8w(const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    return dispatch_resident<true>(a, num_cus, s);
}

}  // namespace aj
