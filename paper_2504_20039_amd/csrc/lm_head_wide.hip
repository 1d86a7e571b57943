// LM head (step 1) + per-vocabulary-block greedy maximum (first half of step 2) for 113..272 verify rows in ONE
// row tile (e.g. 8 windows x 33 rows = 264): 256 vocabulary rows x 16*MB verify rows per workgroup, MB <= 17 blocks
// of v_mfma_f32_16x16x32_bf16, so that 264 rows pad to 272 (3 %) and W_lm is streamed from HBM exactly once.
//
// 4 waves side by side along the vocabulary (one per SIMD, 512 registers each): a wave owns 64 vocabulary rows
// (4 blocks of 16) against all verify rows = 4 x MB accumulator blocks of 4 registers (272 at MB = 17).
//   * W_lm rows are private to a wave, so they never touch LDS: non-temporal buffer loads of whole 128-byte lines
//     (8 rows x 128 B per instruction) straight into registers, brought to the MFMA layout by one DPP rotation per
//     register, in place - the load path of lm_head_resident.hip.  A ring of 4 groups of 8 loads (64 rows x one line); a group
//     is refilled as its registers fall free, three lines (3.3 us of MFMA work) ahead, ONE load after a row block's
//     MFMAs at a time.  The loads are hand-written with the kernel's own s_waitcnt accounting, and all of a load's address but
//     one lane offset travels in scalar registers: with one wave per SIMD, whatever the wave does that is not an MFMA
//     leaves the matrix pipe idle.
//   * hidden_t is shared by the 4 waves: slabs of 64 k elements (16*MB rows x one 128-byte line) staged in LDS, four
//     buffers (three slabs ahead), by asynchronous direct-to-LDS loads; one workgroup barrier per slab.  A slab is 2 pieces of 32 k; a
//     piece is 4 x MB MFMAs ordered row block by row block.  The hidden_t fragments are a rolling window of 8: the
//     fragment used 8 row blocks from now (in this piece or the next) is read from LDS right after the 4 MFMAs that
//     used the slot's previous content, so the LDS latency hides behind two row blocks' MFMAs and the window costs 32
//     registers instead of 4 * MB.  The wait + barrier for the next slab sits before the LAST piece of a slab, during
//     which the first fragments of the new buffer are read.
//   * 272 accumulator registers do not fit the 256 AGPRs, and left to choose the compiler moves accumulators between
//     the two register files inside the hot loop.  So every MFMA is a hand-written statement that names the file:
//     row blocks 0..15 in AGPRs, row block 16 (MB = 17 only) in VGPRs.
#include "../../include/aj.h"
#include "aj_internal.h"
#include "lds_pipeline.h"

namespace aj {

namespace {

constexpr int WD_WAVES = 4;
constexpr int WD_N = 256;                       // vocabulary rows per tile
constexpr int WD_KS = 64;                       // k elements per hidden_t slab: one 128-byte line of a row
constexpr int WD_HROW = WD_KS * 2;              // bytes of a hidden_t row per slab
constexpr int WD_MAXB = 17;

template <int MB, bool FP8W, bool DUMP, bool TOPK, bool SAMPLE>
__global__ __launch_bounds__(WD_WAVES * 64) void k_lm_head_wide(LmHeadArgs a, int ntiles)
{
    // FP8 weights: a 128-byte line of a W_lm row holds 128 k elements = TWO hidden_t slabs; everything else (ring,
    // loads, layout moves, slab pipeline) is the same, and a lane's 16 bytes of a line half - 16 k elements, its share of
    // the slab's two pieces - are widened to bf16 (exactly) one piece ahead of their use
    constexpr int SPG = FP8W ? 2 : 1;                           // hidden_t slabs per W_lm line
    constexpr int HSLAB = MB * 16 * WD_HROW;                    // bytes of a hidden_t slab in LDS
    constexpr int MBA = MB > 16 ? 16 : MB;                      // row blocks accumulated through the builtin
    constexpr int NHB = 4;                                      // hidden_t slab buffers
    __shared__ __attribute__((aligned(1024))) char lds[NHB * HSLAB];
    __shared__ Best red[WD_WAVES][MB * 16];
    __shared__ int32_t redc[TOPK ? WD_WAVES : 1][MB * 16];

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, q4 = lane >> 4;
    // The lane index once more, for the rarely taken paths (rows beyond M or V, the epilogue): derived on the spot from an
    // opaque zero, so that neither it nor anything computed from it occupies a register across the slab loop
    auto lane_now = [] {
        int zz = 0;
        asm volatile("" : "+v"(zz));
        return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, (uint32_t)zz));
    };
    const char *H = (const char *)a.H;
    const uint32_t wrow = (uint32_t)a.d * (FP8W ? 1u : 2u);     // bytes of a W_lm row
    const uint32_t hrow = (uint32_t)a.d * 2u;                   // bytes of a hidden_t row
    const int NS = a.d / WD_KS;                                 // slabs per tile: a multiple of 4 * SPG (host)

    // ---- hidden_t slab loader: a load covers 8 LDS rows x 128 B (1 KB); load i of wave w covers row group 4i + w
    // (beyond the slab: its last group once more - same data to the same place); lane (row lane/8, chunk slot lane%8)
    // fetches global chunk slot ^ ((row / 2) % 8), so that the fragment reads are conflict free.  The group index
    // depends on an opaque scalar, so that each lane offset is computed here (a few VALU operations) instead of living in a
    // register, and in scratch memory, across the kernel.
    // A group that lies inside the M rows (all but the last one or two of a slab) is loaded with ONE lane offset, that of
    // the wave's first group (the swizzle term does not depend on i: rows 32 apart), the group's distance travelling in the
    // scalar base address - scalar instructions only.  One wave per SIMD: nothing covers vector work that is not an MFMA.
    constexpr int HG = 2 * MB, HL = (HG + WD_WAVES - 1) / WD_WAVES;     // row groups per slab, loads per wave
    const uint32_t lds_base = lds_offset_of(lds);
    const uint32_t hoff0 = __umul24(8 * wave + (lane >> 3), hrow) + (uint32_t)(((lane & 7) ^ ((4 * wave + (lane >> 4)) & 7)) * 16);
    auto load_h1 = [&](int slab, int bufoff, int i) {        // load i (0 .. HL - 1) of a slab
        const char *hb = H + (size_t)slab * WD_HROW;
        // M > 16 * (MB - 1): groups 0 .. HG - 3 lie inside the M rows whatever M is
        constexpr int IF = (HG - 6) / WD_WAVES + 1;      // loads i < IF touch those groups only
        const int gq = i * WD_WAVES + wave;
        if (i < IF) {
            lds_dma_16(hb + (size_t)i * (32 * hrow), hoff0, lds_base + bufoff + gq * 1024);
        } else {
            int z = 0;
            asm volatile("" : "+s"(z));                  // an opaque zero
            const int gg = min(gq + z, HG - 1), ln = lane_now();
            const int hr = 8 * gg + (ln >> 3);           // rows beyond M repeat the last one (their logits are never looked at)
            lds_dma_16(hb, __umul24(min(hr, a.M - 1), hrow) + (uint32_t)(((ln & 7) ^ ((hr >> 1) & 7)) * 16),
                       lds_base + bufoff + gg * 1024);
        }
    };
    auto load_h = [&](int slab, int bufoff) {
#pragma unroll
        for (int i = 0; i < HL; ++i) load_h1(slab, bufoff, i);
    };

    // ---- W_lm loads (see lm_head_resident.hip): load 2*blk + h of a line covers rows 8h .. 8h+7 of block blk
    // The loads are hand-written, with the kernel's own s_waitcnt accounting (W_WAIT, H_WAIT below): the compiler
    // does not count the direct-to-LDS loads, so its own waits for buffer loads issued between them come out stricter
    // than needed and let only one line of W_lm be in flight.
    const uint64_t wbase = (uint64_t)a.W;
    const u32x4 wres = {(uint32_t)wbase, (uint32_t)(wbase >> 32), (uint32_t)a.V * wrow, 0x00020000u};   // raw buffer
    // lane (l16, q4): row l16 % 8 of a group of 8, bytes (q4 + 4 * (l16 / 8)) * 16 .. + 15 of the line
    const uint32_t woff0 = __umul24(l16 & 7, wrow) + (uint32_t)(q4 + 4 * (l16 >> 3)) * 16u;
    // vb: first of the wave's 64 rows; load j of a burst covers rows vb + 8j .. + 7 of line `line` (the index of the 128-byte
    // line in the row).  One lane offset serves every load, the rest of the address travels in the scalar offset - scalar
    // instructions only.  A wave whose 64 rows would reach beyond the vocabulary (in the last tile) starts at V - 64
    // instead, so that every row it reads exists; the epilogue drops the logits of the rows below its own range.
    auto w_load1 = [&](u32x4 &dst, int vb, int line, int j) {
        asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen nt"
                     : "=v"(dst)
                     : "v"(woff0), "s"(wres), "s"((uint32_t)(vb + 8 * j) * wrow + (uint32_t)line * 128u)
                     : "memory");
    };
    auto w_burst = [&](u32x4(&dst)[8], int vb, int line) {
#pragma unroll
        for (int j = 0; j < 8; ++j) w_load1(dst[j], vb, line, j);
    };
    // The two loads of a block's line (x: rows 0..7, y: rows 8..15; lanes l16 < 8 hold the first 64 bytes, the others
    // the second) become, in place, the block's two k steps in MFMA layout (lane l16 <-> row l16): x keeps its lower
    // lanes and takes y's lower lanes into its upper ones, y keeps its upper lanes and takes x's upper lanes.
    auto to_mfma_layout = [&](u32x4 &x, u32x4 &y) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int xk = (int)x[k], yk = (int)y[k];
            x[k] = (uint32_t)__builtin_amdgcn_update_dpp(xk, yk, 0x128 /* row_ror:8 */, 0xF, 0xC, false);
            y[k] = (uint32_t)__builtin_amdgcn_update_dpp(yk, xk, 0x128, 0xF, 0x3, false);
        }
    };

    f32x4 acc[4][MBA], accv[4];       // accv: row block 16, in VGPRs
    u32x4 ring[4][8];                 // 4 lines x (4 blocks x 2 halves of the block's rows)
    bf16x8 wf[2][4];                  // FP8 weights: the widened W_lm fragments of this piece and of the next
    auto widen = [&](const u32x4 &x, int half) { return fp8x8_to_bf16x8(uint2{x[2 * half], x[2 * half + 1]}); };
    constexpr int HW = MB >= 15 ? 4 : 8;   // hidden_t fragment window (registers are scarce at 15+ row blocks)
    static_assert(MB >= HW, "the window reaches into the next piece only");
    bf16x8 hf[HW];
    // fragment of row block y, piece p (0, 1) of a slab: lds + buffer offset + hs[p] + y * 16 rows; the row-block part
    // travels in the instruction's offset field.  k elements of lane group q4 in piece p: 32p + 8*q4 .. + 7 (bf16 weights),
    // 16*q4 + 8p .. + 7 (FP8 weights: the two halves of the lane's 16 bytes) - chunk 4p + q4 or 2*q4 + p of the row's 8
    const int hsw = (l16 >> 1) & 7;
    const int hc0 = FP8W ? 2 * q4 : q4, hc1 = FP8W ? 2 * q4 + 1 : 4 + q4;
    const int hs[2] = {l16 * WD_HROW + ((hc0 ^ hsw) * 16), l16 * WD_HROW + ((hc1 ^ hsw) * 16)};
    auto read_h = [&](const char *base, int y) { return *(const bf16x8 *)(base + y * 16 * WD_HROW); };

    // one piece (p = 0, 1) of a slab: 4 x MB MFMAs with half p of ring group g (FP8 weights: with piece p of half hh of
    // the group, widened during the piece before).  n0 = index of the piece's first row
    // block in the fragment sequence (mod HW); after row block y the window slot is refilled with the fragment HW
    // positions on: this piece's (buffer cb), or the next piece's (piece np of buffer nb)
    // `after(y)` runs after the MFMAs of row block y: the loads of the step, one at a time - a burst of them fills the
    // address queue of the vector-memory path and the wave, the only one of its SIMD, stands at the load instead of
    // issuing MFMAs
    auto piece = [&](int g, int hh, int p, int n0, int cb, int nb, int np, auto after) {
        // the buffer offsets stay opaque run-time values: folded into constants (they cycle with the 4 slabs of a trip)
        // the compiler keeps dozens of precomputed LDS addresses in registers
        asm volatile("" : "+s"(cb), "+s"(nb));
        const char *bc = lds + (cb + hs[p]), *bn = lds + (nb + hs[np]);
        // In the last piece of a line the NEXT line's registers are brought to the MFMA layout, one block after
        // every FS row blocks, in the shadow of the MFMAs (with one wave per SIMD nothing else covers VALU work; as a
        // block of 48 moves before the first piece it left the matrix pipe idle for a tenth of the slab).  FP8 weights:
        // one row block later the next piece's fragments of that block are widened.
        constexpr int FS = MB / 4;
        const int gn = (g + 1) & 3;
        const bool last = hh == SPG - 1 && p == 1;
#pragma unroll
        for (int y = 0; y < MB; ++y) {
            const int slot = (n0 + y) % HW;
            if (last && y % FS == 0 && y / FS < 4) to_mfma_layout(ring[gn][2 * (y / FS)], ring[gn][2 * (y / FS) + 1]);
            if (FP8W && y % FS == 1 && y / FS < 4) {
                const int bb = y / FS;
                if (p == 0) wf[1][bb] = widen(ring[g][2 * bb + hh], 1);
                else if (!last) wf[0][bb] = widen(ring[g][2 * bb + 1], 0);
                else wf[0][bb] = widen(ring[gn][2 * bb], 0);
            }
            // Every MFMA is written out with its accumulator's register file stated: row blocks 0..15 in AGPRs (all
            // 256 of them), row block 16 in VGPRs.  Left to choose, the compiler moves accumulators between the two
            // files inside this loop.
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (FP8W) {
                    if (y < MBA) {
                        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0"
                                     : "+a"(acc[b][y < MBA ? y : 0])
                                     : "v"(wf[p][b]), "v"(hf[slot]));
                    } else {
                        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(accv[b]) : "v"(wf[p][b]), "v"(hf[slot]));
                    }
                } else if (y < MBA) {
                    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0"
                                 : "+a"(acc[b][y < MBA ? y : 0])
                                 : "v"(ring[g][2 * b + p]), "v"(hf[slot]));
                } else {
                    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(accv[b]) : "v"(ring[g][2 * b + p]), "v"(hf[slot]));
                }
            }
            hf[slot] = y + HW < MB ? read_h(bc, y + HW) : read_h(bn, y + HW - MB);
            after(y);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // The (tile, slab) sequence of a workgroup is ONE pipeline: hidden_t slabs are the same for every tile (a single
    // row tile), so slab loads simply wrap around, and ring refills past a tile's last line fetch the first lines of
    // the workgroup's next tile.  After the last tile both run on into data nobody uses.
    const int lines = NS / SPG;                      // 128-byte lines per W_lm row
    int T = blockIdx.x;
    if (T >= ntiles) return;
    {
        // lines 0..2 whole and the even registers of line 3: its odd ones are loaded in the first piece of slab 0, like those of
        // every later line.  (No hand-written load may go into a register that is overwritten before it is read: the
        // compiler gives such an output a register it also uses for other values, and the data arrives later.)
        const int vb = min(T * WD_N + wave * 64, a.V - 64);
#pragma unroll
        for (int g = 0; g < 3; ++g) w_burst(ring[g], vb, g);
#pragma unroll
        for (int j = 0; j < 8; j += 2) w_load1(ring[3][j], vb, 3, j);
    }
    load_h(0, 0);
    load_h(1, HSLAB);
    load_h(2, 2 * HSLAB);
    // (the first line's registers are operands of the wait: the moves below must not be scheduled before it)
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier"
                 : "+v"(ring[0][0]), "+v"(ring[0][1]), "+v"(ring[0][2]), "+v"(ring[0][3]), "+v"(ring[0][4]), "+v"(ring[0][5]),
                   "+v"(ring[0][6]), "+v"(ring[0][7])
                 :
                 : "memory");
#pragma unroll
    for (int b = 0; b < 4; ++b) to_mfma_layout(ring[0][2 * b], ring[0][2 * b + 1]);
    if (FP8W) {
#pragma unroll
        for (int b = 0; b < 4; ++b) wf[0][b] = widen(ring[0][2 * b], 0);
    }
#pragma unroll
    for (int y = 0; y < HW; ++y) hf[y] = read_h(lds + hs[0], y);
    int cb = 0;                                       // byte offset of the LDS buffer of the slab being computed

    for (; T < ntiles; T += gridDim.x) {
        // v0: first vocabulary row of the wave's own range; vb, vbn: first row it reads in this tile and in its next one
        const int v0 = T * WD_N + wave * 64, vb = min(v0, a.V - 64), vbn = min(v0 + (int)gridDim.x * WD_N, a.V - 64);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
#pragma unroll
            for (int y = 0; y < MBA; ++y) acc[b][y] = f32x4{0.f, 0.f, 0.f, 0.f};
            accv[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        // The hand-written MFMAs are invisible to the compiler's hazard handling, and it may sink the zeroing above
        // to just before an accumulator's first use: make every zeroed register an operand here, then wait.
#pragma unroll
        for (int b = 0; b < 4; ++b) {
#pragma unroll
            for (int y = 0; y < MBA; ++y) asm volatile("" : "+a"(acc[b][y]));
            asm volatile("" : "+v"(accv[b]));
        }
        asm volatile("s_nop 7" ::: "memory");
        // load j of the refill of ring group g with line `line` (past the tile's last line: of the workgroup's next tile)
        auto refill1 = [&](int g, int line, int j) {
            const bool wrap = line >= lines;
            w_load1(ring[g][j], wrap ? vbn : vb, wrap ? line - lines : line, j);
        };

        // Whatever the compiler itself has loaded up to here (spilled values) has landed after this wait, which it
        // knows about: otherwise its own count-down waits for those loads end up inside the loop below, where from
        // the second trip on they would wait for the kernel's hand-written loads.
        __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
        // Four lines per trip: line L = s / SPG + g uses ring group g; the fragment sequence advances by 2 * MB per slab.
        // Loads of slab sl, one after a row block's MFMAs each, in this order:
        //   first piece:  Ro - in a line's first slab, the 4 loads of the odd registers of the group before (its line L + 3)
        //   second piece: D  - the HL loads of hidden_t slab sl + 3 (its buffer is free after the barrier between the pieces)
        //                 Re - in a line's last slab, the 4 loads of the even registers of this group (line L + 4): a group's
        //                      even registers were last read in the first piece of its last slab, the odd ones in the second
        // and they complete in that order.
        for (int s = 0; s < NS; s += 4 * SPG) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
#pragma unroll
                for (int hh = 0; hh < SPG; ++hh) {
                    const int sl = s + g * SPG + hh, pi = 2 * (g * SPG + hh), L = s / SPG + g;
                    const int nb = cb + HSLAB >= NHB * HSLAB ? 0 : cb + HSLAB;     // buffer of slab sl + 1
                    const int fb = cb == 0 ? (NHB - 1) * HSLAB : cb - HSLAB;         // ... of slab sl - 1 = of slab sl + 3
                    piece(g, hh, 0, pi * MB, cb, cb, 1, [&](int y) {
                        if (hh == 0 && y < 4) refill1((g + 3) & 3, L + 3, 2 * y + 1);
                    });
                    // Slab sl + 1 has landed once at most what was issued after its loads is outstanding: Re Ro D(sl+2) Re
                    // Ro (FP8 weights: D(sl+2) and one Re Ro pair).  Every wave has finished slab sl - 1, so its buffer
                    // can take slab sl + 3 (wrapping into the next tile: hidden_t slabs are the same for every tile).
                    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(HL + (FP8W ? 8 : 16)) : "memory");
                    // The next line, whose registers the piece below rearranges, has landed once at most the loads after
                    // its last one - D(sl+1) Re Ro D(sl+2) Re Ro - are outstanding (FP8 weights: it was issued five
                    // slabs ago, before everything the wait above let through).  The registers are operands of
                    // the wait, so nothing that reads them can be scheduled before it.
                    if (hh == SPG - 1) {
                        u32x4(&rn)[8] = ring[(g + 1) & 3];
                        asm volatile("s_waitcnt vmcnt(%8)"
                                     : "+v"(rn[0]), "+v"(rn[1]), "+v"(rn[2]), "+v"(rn[3]), "+v"(rn[4]), "+v"(rn[5]), "+v"(rn[6]),
                                       "+v"(rn[7])
                                     : "n"(FP8W ? HL + 8 : 2 * HL + 16));
                    }
                    piece(g, hh, 1, (pi + 1) * MB, cb, nb, 0, [&](int y) {
                        if (y < HL) load_h1(sl + 3 < NS ? sl + 3 : sl + 3 - NS, fb, y);
                        else if (hh == SPG - 1 && y < HL + 4) refill1(g, L + 4, 2 * (y - HL));
                    });
                    cb = nb;
                }
            }
        }

        // the hand-written MFMAs are invisible to the compiler's hazard handling: let the last of them retire
        // before their accumulators are read
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        // (the lane's coordinates are derived again from an opaque copy of its index: values computed from them once, before
        // the tile loop, would have to live - in scratch memory - across the slab loop, and their reloads bring the
        // compiler's own waits for them into it)
        const int lane_e = lane_now();
        const int le16 = lane_e & 15, qe4 = lane_e >> 4;
        // ---- lane (l16, q4) holds verify row 16y + l16 against vocabulary rows vb + 16b + 4*q4 + r, ascending in (b, r);
        // those below v0 (a wave that starts early so as to stay inside the vocabulary) belong to another wave
#pragma unroll
        for (int y = 0; y < MB; ++y) {
            const int row = y * 16 + le16, rowc = min(row, a.M - 1);
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
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int v = vb + b * 16 + qe4 * 4 + r;
                    float val = y < MBA ? acc[b][y < MBA ? y : 0][r] : accv[b][r];
                    if (v >= v0 && v < a.V) {
                        if (DUMP && row < a.M) a.dump[(size_t)row * a.V + v] = val;
                        if (SAMPLE) val = fmaf(val, a.inv_temp, gumbel_noise(klo, khi, (uint32_t)v));
                        if (val > bv) {      // strict >: the lowest index of the maximum
                            bv = val;
                            bi = v;
                        }
                        if (TOPK) cn += ranks_before(val, v, th, tk);
                    }
                }
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
            if (qe4 == 0) {
                red[wave][row] = Best{bv, bi};
                if (TOPK) redc[wave][row] = cn;
            }
            // one row block's accumulators at a time: read all at once they need more registers than there are
            __builtin_amdgcn_sched_barrier(0);
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        for (int row = wave * 64 + lane_e; row < MB * 16 && row < a.M; row += WD_WAVES * 64) {
            Best best = red[0][row];
            int32_t cn = TOPK ? redc[0][row] : 0;
#pragma unroll
            for (int w = 1; w < WD_WAVES; ++w) {
                const Best o = red[w][row];
                if (better(o.v, o.i, best.v, best.i)) best = o;
                if (TOPK) cn += redc[w][row];
            }
            a.part[(size_t)row * a.nblocks + T] = best;
            if (TOPK) a.cnt[(size_t)row * a.nblocks + T] = cn;
        }
        // `red` is rewritten only after the barriers of the next tile.  The slab waits count this wave's loads in
        // issue order, and stores need not retire in that order: let the stores above retire here.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
}

template <int MB, bool FP8W>
hipError_t launch_wide(const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    const int ntiles = (a.V + WD_N - 1) / WD_N;
    const int grid = ntiles < num_cus ? ntiles : num_cus;
    const dim3 g(grid), b(WD_WAVES * 64);
    if (a.dump) hipLaunchKernelGGL((k_lm_head_wide<MB, FP8W, true, false, false>), g, b, 0, s, a, ntiles);
    else if (a.thr) {
        if (FP8W) return hipErrorInvalidValue;       // no top-K baseline on FP8 weights (refused at create time)
        hipLaunchKernelGGL((k_lm_head_wide<MB, false, false, true, false>), g, b, 0, s, a, ntiles);
    } else if (a.key) hipLaunchKernelGGL((k_lm_head_wide<MB, FP8W, false, false, true>), g, b, 0, s, a, ntiles);
    else hipLaunchKernelGGL((k_lm_head_wide<MB, FP8W, false, false, false>), g, b, 0, s, a, ntiles);
    return hipGetLastError();
}

template <bool FP8W>
hipError_t dispatch_wide(const LmHeadArgs &a, int num_cus, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    switch ((a.M + 15) / 16) {
        case 8: return launch_wide<8, FP8W>(a, num_cus, s);
        case 9: return launch_wide<9, FP8W>(a, num_cus, s);
        case 10: return launch_wide<10, FP8W>(a, num_cus, s);
        case 11: return launch_wide<11, FP8W>(a, num_cus, s);
        case 12: return launch_wide<12, FP8W>(a, num_cus, s);
        case 13: return launch_wide<13, FP8W>(a, num_cus, s);
        case 14: return launch_wide<14, FP8W>(a, num_cus, s);
        case 15: return launch_wide<15, FP8W>(a, num_cus, s);
        case 16: return launch_wide<16, FP8W>(a, num_cus, s);
        case 17: return launch_wide<17, FP8W>(a, num_cus, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool lm_head_wide_supports(int M, int V, int d, bool fp8w)
{
    // a trip of the slab loop covers 4 lines of a W_lm row: 256 k elements, 512 with FP8 weights
    const int trip = fp8w ? 512 : 256, wb = fp8w ? 1 : 2;
    if (M <= 112 || M > WD_MAXB * 16 || V < WD_N || d < trip || d % trip != 0) return false;
    if ((uint64_t)V * d * wb >= (1ull << 32) || (uint64_t)M * d * 2 >= (1ull << 32)) return false;
    return V < (1 << 24) && d * 2 < (1 << 24);
}

int lm_head_wide_blocks(int V) { return (V + WD_N - 1) / WD_N; }

hipError_t lm_head_wide_bf16(const LmHeadArgs &a, int num_cus, hipStream_t s) { return dispatch_wide<false>(a, num_cus, s); }

hipError_t lm_head_wide_fp8w(const LmHeadArgs &a, int num_cus, hipStream_t s) { return dispatch_wide<true>(a, num_cus, s); }

}  // namespace aj
