// Steps 2 (second half) to 4: cross-block greedy maximum, mismatch test + judge, first-reject scan.
// Two forms.  k_verify_tail does everything in one launch with one workgroup per speculation window: right for
// many short windows and for draft trees (a node is checked against its PARENT's row, which the same workgroup
// has just reduced).  For chains with few windows of many rows (batch 1 with 33 or 65 verify rows has ONE
// workgroup walk 65 rows x 1024 partials in five dependent rounds) the work is split by verify row instead:
// k_tail_rows gives every row a wave of its own (maximum of the row's partials, mismatch test of the row's slot,
// judge dot product at a mismatch), k_tail_scan then finds each window's first rejected slot.
#include <stdlib.h>

#include "aj_internal.h"

namespace aj {

namespace {

constexpr int TAIL_WAVES = 16;
constexpr int MAXK = 1023;

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// wave-wide partial dot of n elements (n % 8 == 0 for bf16, % 4 for f32), fp32 accumulation.
// Four 16-byte chunks per operand are requested before any is used: this kernel is a chain of
// memory round trips, so what counts is how many loads are in flight, not the arithmetic.
template <bool BF16, int U = 4>
__device__ __forceinline__ float dot_part(const void *x, const void *w, int n, int lane)
{
    float acc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) acc[u] = 0.f;
    const int nchunks = n / (BF16 ? 8 : 4);
    const u32x4 *xp = (const u32x4 *)x, *wp = (const u32x4 *)w;
    for (int c0 = lane; c0 < nchunks; c0 += 64 * U) {
        u32x4 xv[U], wv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + 64 * u;
            const bool in = c < nchunks;
            xv[u] = in ? xp[c] : u32x4{0, 0, 0, 0};
            wv[u] = in ? wp[c] : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (BF16) {
                    acc[u] = fmaf(bf16_lo(xv[u][q]), bf16_lo(wv[u][q]), acc[u]);
                    acc[u] = fmaf(bf16_hi(xv[u][q]), bf16_hi(wv[u][q]), acc[u]);
                } else {
                    acc[u] = fmaf(__uint_as_float(xv[u][q]), __uint_as_float(wv[u][q]), acc[u]);
                }
            }
        }
    }
    float sum = 0.f;
#pragma unroll
    for (int u = 0; u < U; u += 4) sum += (acc[u] + acc[u + 1]) + (acc[u + 2] + acc[u + 3]);
    return sum;
}

// Phase 1: a wave per verify row reduces the row's block partials (coalesced: they are stored
//          [row][block]) with lowest-index tie-break.
// Phase 2: a wave per slot; at a mismatching slot (wave-uniform) its lanes share the judge dot
//          product and reduce it with cross-lane shuffles.
// Phase 3: wave 0 finds the first rejected slot with ballots and emits.
// TREE: the K slots are nodes of a draft tree (a.parent[b][j] in [-1, j)): node j is checked against the
//          greedy token of its parent's row, phase 3 finds the accepted node of greatest depth.
template <bool BF16, bool TREE>
__global__ __launch_bounds__(TAIL_WAVES * 64) void k_verify_tail(TailArgs a)
{
    __shared__ int32_t s_t[MAXK + 1];
    __shared__ uint8_t s_rej[MAXK + 1];
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int K = a.K, R = K + 1;
    const size_t es = BF16 ? 2 : 4;

    for (int j = wave; j < R; j += TAIL_WAVES) {
        const size_t row = (size_t)b * R + j;
        const Best *p = a.part + row * a.nblocks;
        float bv = -INFINITY;
        int32_t bi = 0x7fffffff;
        for (int nb0 = lane; nb0 < a.nblocks; nb0 += 256) {       // 4 loads in flight per lane
            Best x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int nb = nb0 + 64 * u;
                x[u] = nb < a.nblocks ? p[nb] : Best{-INFINITY, 0x7fffffff};
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (better(x[u].v, x[u].i, bv, bi)) {
                    bv = x[u].v;
                    bi = x[u].i;
                }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            float ov = __shfl_xor(bv, off);
            int32_t oi = __shfl_xor(bi, off);
            if (better(ov, oi, bv, bi)) {
                bv = ov;
                bi = oi;
            }
        }
        if (lane == 0) {
            s_t[j] = bi;
            a.t_star[row] = bi;
            a.maxlogit[row] = bv;
        }
    }
    __syncthreads();

    for (int j = wave; j < K; j += TAIL_WAVES) {
        // row whose prediction slot j is checked against: j in a chain, the parent's row in a tree
        // (a parent outside [-1, j) is clamped into it: malformed input stays inside the window's rows)
        const int prow = TREE ? min(max(a.parent[(size_t)b * K + j], -1), j - 1) + 1 : j;
        const bool mis = s_t[prow] != a.draft_tok[(size_t)b * K + j];
        float z = __builtin_nanf("");
        bool r = false;
        if (mis) {
            const size_t row = (size_t)b * R + (TREE ? (a.feat_offset ? j + 1 : prow) : j + a.feat_offset);
            // target half: from the LM-head pass (fused judge row), else a dot product here
            float acc = a.zt ? (lane == 0 ? a.zt[row] : 0.f)
                             : dot_part<BF16>((const char *)a.hidden_t + row * a.d_t * es, a.clf_w, a.d_t, lane);
            if (a.d_d > 0)
                acc += dot_part<BF16>((const char *)a.hidden_d + row * a.d_d * es,
                                      (const char *)a.clf_w + (size_t)a.d_t * es, a.d_d, lane);
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
            z = acc + a.clf_b;
            r = !(z < a.zthr);
        }
        if (lane == 0) {
            s_rej[j] = r;
            if (a.score) {
                a.score[(size_t)b * K + j] = z;
                a.score[(size_t)a.B * K + (size_t)b * K + j] = 1.f / (1.f + expf(-z));
            }
        }
    }
    __syncthreads();

    if (TREE) {
        // depth of every accepted node, in topological order (parents come first); K is small, so one lane
        // walks the nodes; then the deepest accepted node, lowest index among equals
        __shared__ int32_t s_depth[MAXK + 1];
        if (threadIdx.x == 0) {
            int best = -1, best_depth = 0;
            for (int j = 0; j < K; ++j) {
                const int p = min(max(a.parent[(size_t)b * K + j], -1), j - 1);
                const int pd = p < 0 ? 0 : s_depth[p];
                const int dj = (!s_rej[j] && (p < 0 || pd > 0)) ? pd + 1 : 0;
                s_depth[j] = dj;
                if (dj > best_depth) {
                    best_depth = dj;
                    best = j;
                }
            }
            a.out_len[b] = best_depth;
            a.out_tok[b] = s_t[best + 1];
            a.out_node[b] = best;
        }
        return;
    }
    if (wave == 0) {
        int n = K;
        for (int base = 0; base < K; base += 64) {
            const int j = base + lane;
            const bool r = j < K && s_rej[j];
            const unsigned long long m = __ballot(r);
            if (m) {
                n = base + __builtin_ctzll(m);
                break;
            }
        }
        if (lane == 0) {
            a.out_len[b] = n;
            a.out_tok[b] = s_t[n];
        }
    }
}

// Split form, first kernel: a wave per verify row (4 rows per workgroup).  All of a row's partials are requested
// before any is used (8 loads per lane in flight), so the row costs one memory round trip, the mismatch test a
// second (the draft token is requested with the partials) and a judge dot product two more.
constexpr int ROWS_PER_WG = 4;
template <bool BF16>
__global__ __launch_bounds__(ROWS_PER_WG * 64) void k_tail_rows(TailArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int K = a.K, R = K + 1;
    const int row = blockIdx.x * ROWS_PER_WG + wave;
    if (row >= a.B * R) return;
    const int b = row / R, j = row - b * R;
    const size_t es = BF16 ? 2 : 4;
    const int32_t dtok = j < K ? a.draft_tok[(size_t)b * K + j] : 0;

    const Best *p = a.part + (size_t)row * a.nblocks;
    float bv = -INFINITY;
    int32_t bi = 0x7fffffff;
    constexpr int U = 8;
    for (int nb0 = lane; nb0 < a.nblocks; nb0 += 64 * U) {
        Best x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int nb = nb0 + 64 * u;
            x[u] = nb < a.nblocks ? p[nb] : Best{-INFINITY, 0x7fffffff};
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (better(x[u].v, x[u].i, bv, bi)) {
                bv = x[u].v;
                bi = x[u].i;
            }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        float ov = __shfl_xor(bv, off);
        int32_t oi = __shfl_xor(bi, off);
        if (better(ov, oi, bv, bi)) {
            bv = ov;
            bi = oi;
        }
    }
    if (lane == 0) {
        a.t_star[row] = bi;
        a.maxlogit[row] = bv;
    }
    if (j >= K) return;                     // the bonus row has no slot to check

    const bool mis = bi != dtok;            // wave-uniform: every lane holds the reduced maximum
    float z = __builtin_nanf("");
    bool r = false;
    if (mis) {
        const size_t frow = (size_t)row + a.feat_offset;     // same window: j + feat_offset <= K
        float acc = a.zt ? (lane == 0 ? a.zt[frow] : 0.f)
                         : dot_part<BF16, 8>((const char *)a.hidden_t + frow * a.d_t * es, a.clf_w, a.d_t, lane);
        if (a.d_d > 0)
            acc += dot_part<BF16, 8>((const char *)a.hidden_d + frow * a.d_d * es,
                                     (const char *)a.clf_w + (size_t)a.d_t * es, a.d_d, lane);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
        z = acc + a.clf_b;
        r = !(z < a.zthr);
    }
    if (lane == 0) {
        a.rej[(size_t)b * K + j] = r;
        if (a.score) {
            a.score[(size_t)b * K + j] = z;
            a.score[(size_t)a.B * K + (size_t)b * K + j] = 1.f / (1.f + expf(-z));
        }
    }
}

// Split form, second kernel: a wave per window finds the first rejected slot with ballots and emits.
__global__ __launch_bounds__(64) void k_tail_scan(TailArgs a)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const int K = a.K;
    int n = K;
    for (int base = 0; base < K; base += 64) {
        const int j = base + lane;
        const bool r = j < K && a.rej[(size_t)b * K + j];
        const unsigned long long m = __ballot(r);
        if (m) {
            n = base + __builtin_ctzll(m);
            break;
        }
    }
    if (lane == 0) {
        a.out_len[b] = n;
        a.out_tok[b] = a.t_star[(size_t)b * (K + 1) + n];
    }
}

// 1: split form, 0: one launch; AJ_TAIL=split|fused in the environment overrides the choice (for measurements)
bool use_split_tail(const TailArgs &a)
{
    static const int forced = [] {
        const char *e = getenv("AJ_TAIL");
        return !e ? -1 : (e[0] == 's' ? 1 : (e[0] == 'f' ? 0 : -1));
    }();
    if (a.parent || !a.rej) return false;
    if (forced >= 0) return forced == 1;
    // measured on the six benchmark workloads: the split form wins from 33 rows on (6 against 16 us at 1 x 33
    // rows, 11 against 27 at 1 x 65, 13 against 26 at 8 x 33, 15 against 51 at 128 x 65); at 17 rows the one
    // launch is a microsecond cheaper
    return a.B * (a.K + 1) > 32;
}

}  // namespace

hipError_t verify_tail(const TailArgs &a, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    if (use_split_tail(a)) {
        const int rows = a.B * (a.K + 1);
        const int grid = (rows + ROWS_PER_WG - 1) / ROWS_PER_WG;
        if (a.dtype == 1) hipLaunchKernelGGL((k_tail_rows<true>), dim3(grid), dim3(ROWS_PER_WG * 64), 0, s, a);
        else hipLaunchKernelGGL((k_tail_rows<false>), dim3(grid), dim3(ROWS_PER_WG * 64), 0, s, a);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k_tail_scan, dim3(a.B), dim3(64), 0, s, a);
        return hipGetLastError();
    }
    if (a.parent) {
        if (a.dtype == 1) hipLaunchKernelGGL((k_verify_tail<true, true>), dim3(a.B), dim3(TAIL_WAVES * 64), 0, s, a);
        else hipLaunchKernelGGL((k_verify_tail<false, true>), dim3(a.B), dim3(TAIL_WAVES * 64), 0, s, a);
    } else {
        if (a.dtype == 1) hipLaunchKernelGGL((k_verify_tail<true, false>), dim3(a.B), dim3(TAIL_WAVES * 64), 0, s, a);
        else hipLaunchKernelGGL((k_verify_tail<false, false>), dim3(a.B), dim3(TAIL_WAVES * 64), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace aj
