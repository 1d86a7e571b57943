// C ABI of libaj (declared in include/aj.h): argument checks, workspace, kernel dispatch.
#include <math.h>
#include <mutex>
#include <new>

#include "../../include/aj.h"
#include "aj_internal.h"

using namespace aj;

struct aj_handle {
    aj_config cfg;
    int M;
    int variant;   // AJ_KERNEL_* actually used (for bf16), or -1 for the fp32 kernel
    bool stream16; // AJ_KERNEL_STREAM served by the 16-row-tile kernel
    bool fp8w;     // W_lm stored as FP8 E4M3 (16-row-tile kernel only)
    int nblocks;   // partials per verify row
    int device;
    int num_cus;
    Best *part;    // [M][nblocks]
    int32_t *t_star;
    float *maxlogit;
    float *score;  // [2][B][K] or nullptr
    uint8_t *rej;  // [B][K] rejected-slot flags (tail kernels' split form)
    float *zt;     // [M] fused judge row's logits (AJ_FLAG_FUSED_JUDGE)
    // top-K baseline workspace (AJ_FLAG_TOPK)
    int32_t *cnt;      // [M][nblocks]
    float *thr;        // [M]
    int32_t *thr_tok;  // [M]
    int32_t *rank;     // [M]
    hipEvent_t ev[64][2];
    bool ev_ok;
    uint64_t calls;
};

static thread_local int g_last_hip = 0;

static int hip_fail(hipError_t e)
{
    g_last_hip = (int)e;
    return AJ_EHIP;
}

extern "C" int aj_last_hip_error(void) { return g_last_hip; }

extern "C" const char *aj_strerror(int status)
{
    switch (status) {
        case AJ_OK: return "ok";
        case AJ_EINVAL: return "invalid argument (null/misaligned pointer, bad shape, or tau outside [0,1])";
        case AJ_ENOMEM: return "device workspace allocation failed";
        case AJ_EHIP: return "a HIP call failed (see aj_last_hip_error)";
        case AJ_ESTATE: return "call not valid for this handle";
        case AJ_ELIMIT: return "the shape needs more workspace than the static buffer of aj_verify_static holds";
        default: return "unknown status";
    }
}

static bool aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }

static void free_all(aj_handle *h)
{
    if (h->part) (void)hipFree(h->part);
    if (h->t_star) (void)hipFree(h->t_star);
    if (h->maxlogit) (void)hipFree(h->maxlogit);
    if (h->score) (void)hipFree(h->score);
    if (h->rej) (void)hipFree(h->rej);
    if (h->zt) (void)hipFree(h->zt);
    if (h->cnt) (void)hipFree(h->cnt);
    if (h->thr) (void)hipFree(h->thr);
    if (h->thr_tok) (void)hipFree(h->thr_tok);
    if (h->rank) (void)hipFree(h->rank);
    if (h->ev_ok)
        for (int i = 0; i < 64; ++i) {
            (void)hipEventDestroy(h->ev[i][0]);
            (void)hipEventDestroy(h->ev[i][1]);
        }
}

// Validate a configuration and choose the LM-head kernel for it on the current device: fills everything of *h
// that is not a device allocation.  Allocates nothing.
static int plan_handle(const aj_config &c, aj_handle *h)
{
    if (c.dtype != AJ_F32 && c.dtype != AJ_BF16) return AJ_EINVAL;
    const int mult = c.dtype == AJ_BF16 ? 8 : 4;
    if (c.B < 0 || c.K < 1 || c.K > 1023 || c.V < 1 || c.d_t < mult || c.d_d < 0) return AJ_EINVAL;
    if (c.d_t % mult || c.d_d % mult) return AJ_EINVAL;
    if (c.feat_offset != 0 && c.feat_offset != 1) return AJ_EINVAL;
    if (c.kernel < AJ_KERNEL_AUTO || c.kernel > AJ_KERNEL_WIDE) return AJ_EINVAL;
    if ((int64_t)c.B * (c.K + 1) > (int64_t)1 << 24) return AJ_EINVAL;
    // vocabulary indices go through 24-bit multiplies (tile offsets, the sampling generator's first step)
    if (c.V >= (1 << 24)) return AJ_EINVAL;

    if (c.flags & ~(AJ_FLAG_DEBUG | AJ_FLAG_PROFILE | AJ_FLAG_TOPK | AJ_FLAG_FUSED_JUDGE)) return AJ_EINVAL;
    h->cfg = c;
    h->M = c.B * (c.K + 1);
    hipError_t e = hipGetDevice(&h->device);
    if (e != hipSuccess) return hip_fail(e);
    e = hipDeviceGetAttribute(&h->num_cus, hipDeviceAttributeMultiprocessorCount, h->device);
    if (e != hipSuccess) return hip_fail(e);
    if (c.w_dtype != AJ_W_SAME && c.w_dtype != AJ_W_FP8_E4M3) {
        return AJ_EINVAL;
    }
    if (c.w_dtype == AJ_W_FP8_E4M3) {
        // FP8 weights: the kernels that stream W_lm straight into registers (up to 272 verify rows; beyond that the path
        // is bound by the matrix pipe and the bytes of W_lm cost no time), and no top-K baseline (its pre-pass reads
        // W_lm rows)
        if (c.dtype != AJ_BF16 || (c.flags & (AJ_FLAG_TOPK | AJ_FLAG_FUSED_JUDGE))) return AJ_EINVAL;
        const bool s16 = (c.kernel == AJ_KERNEL_AUTO || c.kernel == AJ_KERNEL_STREAM) &&
                         lm_head_stream16_fp8w_supports(h->M, c.V, c.d_t);
        const bool res = (c.kernel == AJ_KERNEL_AUTO || c.kernel == AJ_KERNEL_RESIDENT) &&
                         lm_head_resident_supports(h->M, c.V, c.d_t, true);
        const bool wide = (c.kernel == AJ_KERNEL_AUTO || c.kernel == AJ_KERNEL_WIDE) &&
                          lm_head_wide_supports(h->M, c.V, c.d_t, true);
        if (h->M > 0 && !s16 && !res && !wide) return AJ_EINVAL;
        h->fp8w = true;
        if (s16 || h->M == 0) {
            h->variant = AJ_KERNEL_STREAM;
            h->stream16 = true;
            h->nblocks = lm_head_stream16_blocks(c.V, h->num_cus);
        } else if (res && !(wide && h->M > 112 && c.kernel == AJ_KERNEL_AUTO)) {     // (113..128 rows: see the bf16 rule below)
            h->variant = AJ_KERNEL_RESIDENT;
            h->nblocks = lm_head_resident_blocks(c.V, h->num_cus);
        } else {
            h->variant = AJ_KERNEL_WIDE;
            h->nblocks = lm_head_wide_blocks(c.V);
        }
    } else if (c.dtype == AJ_F32) {
        if (c.kernel != AJ_KERNEL_AUTO || (c.flags & AJ_FLAG_FUSED_JUDGE)) {
            return AJ_EINVAL;
        }
        h->variant = -1;
        h->nblocks = lm_head_f32_blocks(c.V);
        if (h->nblocks > 65535) return AJ_EINVAL;   // one vocabulary block per gridDim.y entry
    } else {
        int v = c.kernel;
        if (v == AJ_KERNEL_AUTO) {
            // W_lm-streaming kernels up to 128 verify rows: the 16-row-tile kernel with hidden_t in registers
            // (<= 32 rows, d_t = 2048 or 4096), else the kernel that keeps the logits in registers (d_t % 256 == 0, <= 112 rows), else
            // 128-vocabulary tiles of 32, 64 or 128 rows with a running maximum.  113..272 rows: the wide kernel.
            // Above that, the large-tile kernel with the lowest cost = padded row count x a per-row factor against the
            // 256-row whole-line kernel (PAIR = 1).  Measured on 1056 rows at d_t = 4096 / 8192 and 8320 rows at 8192
            // (one device; devices differ by about 5 %): the 288-row variant 1.09 / 1.05 / 1.03, the 256-row kernel
            // with 64-byte pieces 1.11 / 1.09 / 1.10, the 8-wave 288/320-row kernel 1.24 / 1.26 / 1.19; constants
            // 1.06, 1.10, 1.20.  Padded rows are wasted MFMA work, and a batch of 257..320 rows in ONE row tile reads
            // W_lm from HBM only once.  The general kernel serves what is left: hidden sizes that are not a multiple
            // of 32.
            if (lm_head_stream16_supports(h->M, c.V, c.d_t)) {
                v = AJ_KERNEL_STREAM;
            } else if (h->M <= 112 && lm_head_resident_supports(h->M, c.V, c.d_t, false)) {
                v = AJ_KERNEL_RESIDENT;     // up to 112 rows at any hidden size that is a multiple of 256
            } else if (lm_head_wide_supports(h->M, c.V, c.d_t, false)) {
                // 113..272 rows: W_lm straight into registers, 16-row blocks, one row tile (0.37 ms against 0.46 of a padded
                // 256-row tile at 144 rows of the 70B shape, 0.51 against 0.55 of the 288-row tile at 264; at 8 row blocks 0.36
                // against the 0.40 of the accumulator-resident kernel, which is short of registers there)
                v = AJ_KERNEL_WIDE;
            } else if (lm_head_resident_supports(h->M, c.V, c.d_t, false)) {
                v = AJ_KERNEL_RESIDENT;     // 113..128 rows where the wide kernel does not apply (a vocabulary under 256)
            } else if (lm_head_mfma_supports(AJ_KERNEL_STREAM, h->M, c.V, c.d_t)) {
                v = AJ_KERNEL_STREAM;
            } else {
                const bool pair = lm_head_pair_supports(h->M, c.V, c.d_t);
                struct { int kernel; bool ok; double cost; } cand[4] = {
                    {AJ_KERNEL_PAIR, pair, 1.00 * lm_head_pair_padded_rows(h->M)},
                    {AJ_KERNEL_PAIR9, pair, 1.06 * lm_head_pair9_padded_rows(h->M)},
                    {AJ_KERNEL_BIG, lm_head_mfma_supports(AJ_KERNEL_BIG, h->M, c.V, c.d_t),
                     1.10 * lm_head_mfma_padded_rows(AJ_KERNEL_BIG, h->M)},
                    {AJ_KERNEL_TALL, lm_head_mfma_supports(AJ_KERNEL_TALL, h->M, c.V, c.d_t),
                     1.20 * lm_head_mfma_padded_rows(AJ_KERNEL_TALL, h->M)},
                };
                v = AJ_KERNEL_TILE;
                double best = 0.0;
                for (const auto &k : cand)
                    if (k.ok && (v == AJ_KERNEL_TILE || k.cost < best)) {
                        v = k.kernel;
                        best = k.cost;
                    }
            }
        } else if (v == AJ_KERNEL_RESIDENT) {
            if (h->M > 0 && !lm_head_resident_supports(h->M, c.V, c.d_t, false)) return AJ_EINVAL;
        } else if (v == AJ_KERNEL_WIDE) {
            if (h->M > 0 && !lm_head_wide_supports(h->M, c.V, c.d_t, false)) return AJ_EINVAL;
        } else if (v == AJ_KERNEL_PAIR || v == AJ_KERNEL_PAIR9 ? (h->M > 0 && !lm_head_pair_supports(h->M, c.V, c.d_t))
                   : v != AJ_KERNEL_TILE && h->M > 0 && !lm_head_mfma_supports(v, h->M, c.V, c.d_t) &&
                         !(v == AJ_KERNEL_STREAM && lm_head_stream16_supports(h->M, c.V, c.d_t))) {
            return AJ_EINVAL;   // a forced variant that cannot run this shape
        }
        if (v == AJ_KERNEL_TILE && lm_head_tile_blocks(c.V) > 65535) return AJ_EINVAL;   // gridDim.y
        if ((c.flags & AJ_FLAG_FUSED_JUDGE) && h->M > 0) {
            // the fused judge row lives in the accumulator-resident kernel
            if (c.kernel != AJ_KERNEL_AUTO && c.kernel != AJ_KERNEL_RESIDENT) return AJ_EINVAL;
            if (!lm_head_resident_supports(h->M, c.V, c.d_t, false)) return AJ_EINVAL;
            v = AJ_KERNEL_RESIDENT;
        }
        h->variant = v;
        h->stream16 = v == AJ_KERNEL_STREAM && lm_head_stream16_supports(h->M, c.V, c.d_t);
        h->nblocks = v == AJ_KERNEL_TILE ? lm_head_tile_blocks(c.V)
                     : v == AJ_KERNEL_PAIR ? lm_head_pair_blocks(c.V)
                     : v == AJ_KERNEL_PAIR9 ? lm_head_pair9_blocks(c.V)
                     : v == AJ_KERNEL_RESIDENT ? lm_head_resident_blocks(c.V, h->num_cus)
                     : v == AJ_KERNEL_WIDE ? lm_head_wide_blocks(c.V)
                     : h->stream16     ? lm_head_stream16_blocks(c.V, h->num_cus)
                                       : lm_head_mfma_blocks(v, c.V, c.d_t, h->num_cus);
    }
    return AJ_OK;
}

extern "C" int aj_create(const aj_config *cfg, aj_handle **out)
{
    if (out) *out = nullptr;
    if (!cfg || !out) return AJ_EINVAL;
    const aj_config &c = *cfg;
    aj_handle *h = new (std::nothrow) aj_handle();
    if (!h) return AJ_ENOMEM;
    const int rc = plan_handle(c, h);
    if (rc != AJ_OK) {
        delete h;
        return rc;
    }
    if (h->M > 0) {
        const size_t np = (size_t)h->nblocks * h->M;
        bool ok = hipMalloc(&h->part, np * sizeof(Best)) == hipSuccess &&
                  hipMalloc(&h->t_star, (size_t)h->M * sizeof(int32_t)) == hipSuccess &&
                  hipMalloc(&h->maxlogit, (size_t)h->M * sizeof(float)) == hipSuccess &&
                  hipMalloc(&h->rej, (size_t)h->M) == hipSuccess;
        if (ok && (c.flags & AJ_FLAG_DEBUG))
            ok = hipMalloc(&h->score, (size_t)2 * c.B * c.K * sizeof(float)) == hipSuccess;
        if (ok && (c.flags & AJ_FLAG_FUSED_JUDGE))
            ok = hipMalloc(&h->zt, (size_t)h->M * sizeof(float)) == hipSuccess;
        if (ok && (c.flags & AJ_FLAG_TOPK))
            ok = hipMalloc(&h->cnt, np * sizeof(int32_t)) == hipSuccess &&
                 hipMalloc(&h->thr, (size_t)h->M * sizeof(float)) == hipSuccess &&
                 hipMalloc(&h->thr_tok, (size_t)h->M * sizeof(int32_t)) == hipSuccess &&
                 hipMalloc(&h->rank, (size_t)h->M * sizeof(int32_t)) == hipSuccess;
        if (!ok) {
            (void)hipGetLastError();
            free_all(h);
            delete h;
            return AJ_ENOMEM;
        }
    }
    if (c.flags & AJ_FLAG_PROFILE) {
        h->ev_ok = true;
        for (int i = 0; i < 64; ++i)
            for (int j = 0; j < 2; ++j) {
                const hipError_t e = hipEventCreate(&h->ev[i][j]);
                if (e != hipSuccess) {   // destroy what exists, then fail
                    for (int ii = 0; ii <= i; ++ii)
                        for (int jj = 0; jj < (ii == i ? j : 2); ++jj) (void)hipEventDestroy(h->ev[ii][jj]);
                    h->ev_ok = false;
                    free_all(h);
                    delete h;
                    return hip_fail(e);
                }
            }
    }
    *out = h;
    return AJ_OK;
}

extern "C" int aj_destroy(aj_handle *h)
{
    if (!h) return AJ_EINVAL;
    free_all(h);
    delete h;
    return AJ_OK;
}

static hipError_t launch_lm_head(aj_handle *h, const void *hidden_t, const void *W_lm, float *dump, hipStream_t s,
                                 bool topk = false, const uint64_t *key = nullptr, float inv_temp = 1.f,
                                 const void *judge_w = nullptr)
{
    LmHeadArgs a;
    a.H = hidden_t;
    a.W = W_lm;
    a.M = h->M;
    a.V = h->cfg.V;
    a.d = h->cfg.d_t;
    a.part = h->part;
    a.nblocks = h->nblocks;
    a.dump = dump;
    a.thr = topk ? h->thr : nullptr;
    a.thr_tok = topk ? h->thr_tok : nullptr;
    a.cnt = topk ? h->cnt : nullptr;
    a.key = key;
    a.inv_temp = inv_temp;
    a.judge_w = judge_w;
    a.zt = judge_w ? h->zt : nullptr;
    if (h->variant < 0) return lm_head_f32(a, s);
    if (h->variant == AJ_KERNEL_TILE) return lm_head_tile_bf16(a, s);
    if (h->variant == AJ_KERNEL_RESIDENT)
        return h->fp8w ? lm_head_resident_fp8w(a, h->num_cus, s) : lm_head_resident_bf16(a, h->num_cus, s);
    if (h->variant == AJ_KERNEL_WIDE) return h->fp8w ? lm_head_wide_fp8w(a, h->num_cus, s) : lm_head_wide_bf16(a, h->num_cus, s);
    if (h->fp8w) return lm_head_stream16_fp8w(a, h->num_cus, s);
    if (h->stream16) return lm_head_stream16_bf16(a, h->num_cus, s);
    if (h->variant == AJ_KERNEL_PAIR) return lm_head_pair_bf16(a, h->num_cus, s);
    if (h->variant == AJ_KERNEL_PAIR9) return lm_head_pair9_bf16(a, h->num_cus, s);
    return lm_head_mfma_bf16(h->variant, a, h->num_cus, s);
}

// aj_verify, aj_verify_sampled and aj_verify_tree: the same steps; key == nullptr selects the greedy token,
// parent == nullptr a chain of draft tokens
static int verify_common(aj_handle *h, const void *hidden_t, const void *hidden_d, const void *W_lm,
                         const int32_t *draft_tok, const void *clf_w, float clf_b, float tau,
                         const uint64_t *key, float inv_temp, const int32_t *parent, int32_t *out_node,
                         int32_t *out_len, int32_t *out_tok, void *stream)
{
    if (!h) return AJ_EINVAL;
    if (!(tau >= 0.f && tau <= 1.f)) return AJ_EINVAL;   // also refuses NaN
    if (!isfinite(clf_b)) return AJ_EINVAL;
    if (h->M == 0) return AJ_OK;
    const aj_config &c = h->cfg;
    if (!hidden_t || !W_lm || !draft_tok || !clf_w || !out_len || !out_tok) return AJ_EINVAL;
    if (c.d_d > 0 && !hidden_d) return AJ_EINVAL;
    if (!aligned16(hidden_t) || !aligned16(W_lm) || !aligned16(clf_w) || (c.d_d > 0 && !aligned16(hidden_d)))
        return AJ_EINVAL;
    hipStream_t s = (hipStream_t)stream;

    const bool prof = h->ev_ok;
    const int slot = (int)(h->calls % 64);
    hipError_t e;
    if (prof && (e = hipEventRecord(h->ev[slot][0], s)) != hipSuccess) return hip_fail(e);
    // fused judge row: greedy chains and trees on a handle created for it (the sampling variant computes the judge
    // in the tail, as usual)
    const bool fused = h->zt && !key && h->variant == AJ_KERNEL_RESIDENT && !h->fp8w;
    if ((e = launch_lm_head(h, hidden_t, W_lm, nullptr, s, false, key, inv_temp, fused ? clf_w : nullptr)) != hipSuccess)
        return hip_fail(e);
    if (prof && (e = hipEventRecord(h->ev[slot][1], s)) != hipSuccess) return hip_fail(e);
    if (prof) h->calls++;

    TailArgs t;
    t.hidden_t = hidden_t;
    t.hidden_d = hidden_d;
    t.clf_w = clf_w;
    t.draft_tok = draft_tok;
    t.part = h->part;
    t.nblocks = h->nblocks;
    t.B = c.B;
    t.K = c.K;
    t.d_t = c.d_t;
    t.d_d = c.d_d;
    t.V = c.V;
    t.dtype = c.dtype;
    t.feat_offset = c.feat_offset;
    t.clf_b = clf_b;
    // threshold in logit space, computed in double from the float tau, rounded once to float
    t.zthr = tau <= 0.f ? -INFINITY : (tau >= 1.f ? INFINITY : (float)log((double)tau / (1.0 - (double)tau)));
    t.t_star = h->t_star;
    t.maxlogit = h->maxlogit;
    t.zt = fused ? h->zt : nullptr;
    t.score = h->score;
    t.rej = h->rej;
    t.out_len = out_len;
    t.out_tok = out_tok;
    t.parent = parent;
    t.out_node = out_node;
    if ((e = verify_tail(t, s)) != hipSuccess) return hip_fail(e);
    return AJ_OK;
}

extern "C" int aj_verify(aj_handle *h, const void *hidden_t, const void *hidden_d, const void *W_lm,
                         const int32_t *draft_tok, const void *clf_w, float clf_b, float tau,
                         int32_t *out_len, int32_t *out_tok, void *stream)
{
    return verify_common(h, hidden_t, hidden_d, W_lm, draft_tok, clf_w, clf_b, tau, nullptr, 1.f, nullptr, nullptr,
                         out_len, out_tok, stream);
}

// ---- aj_verify without any allocation: the workspace is a static device array -----------------------------
// Every GPU the library runs on holds its own copy of `scratch` at its own address until the process ends.  In
// host code the array's NAME is only a stand-in: the device address comes from hipGetSymbolAddress, once per
// device with that device current, and that pointer is what kernels get.
static __device__ __align__(256) unsigned char scratch[AJ_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[MAX_DEVICES];   // device address of `scratch` per device, nullptr until first use

static int scratch_of_current_device(int device, unsigned char **out)
{
    if (device < 0 || device >= MAX_DEVICES) return AJ_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!p) return hip_fail(hipErrorInvalidSymbol);
        g_scratch_ptr[device] = p;
    }
    *out = (unsigned char *)g_scratch_ptr[device];
    return AJ_OK;
}

static size_t round256(size_t n) { return (n + 255) & ~(size_t)255; }

extern "C" int aj_verify_static(const aj_config *cfg, const void *hidden_t, const void *hidden_d, const void *W_lm,
                                const int32_t *draft_tok, const void *clf_w, float clf_b, float tau,
                                int32_t *out_len, int32_t *out_tok, void *stream)
{
    if (!cfg) return AJ_EINVAL;
    if (cfg->flags != 0) return AJ_EINVAL;        // debug scores, profiling events and top-K counts need a handle
    aj_handle h = {};
    const int rc = plan_handle(*cfg, &h);          // validates, chooses the kernel; allocates nothing
    if (rc != AJ_OK) return rc;
    if (h.M == 0) return AJ_OK;
    // workspace of this shape: [M][nblocks] partials, then t_star[M], maxlogit[M] and the rejected-slot flags
    // (M bytes), each 256-byte aligned
    const size_t part_bytes = round256((size_t)h.M * h.nblocks * sizeof(Best));
    const size_t row_bytes = round256((size_t)h.M * sizeof(int32_t));
    if (part_bytes + 3 * row_bytes > AJ_STATIC_SCRATCH_BYTES) return AJ_ELIMIT;
    unsigned char *base = nullptr;
    const int rs = scratch_of_current_device(h.device, &base);
    if (rs != AJ_OK) return rs;
    // every word the tail kernel reads is written by the LM-head kernel of the same call (one partial per row and
    // block, empty blocks included), so nothing has to start at zero and the last call's contents do not matter
    h.part = (Best *)base;
    h.t_star = (int32_t *)(base + part_bytes);
    h.maxlogit = (float *)(base + part_bytes + row_bytes);
    h.rej = base + part_bytes + 2 * row_bytes;
    return verify_common(&h, hidden_t, hidden_d, W_lm, draft_tok, clf_w, clf_b, tau, nullptr, 1.f, nullptr, nullptr,
                         out_len, out_tok, stream);
}

extern "C" int aj_verify_tree(aj_handle *h, const void *hidden_t, const void *hidden_d, const void *W_lm,
                              const int32_t *draft_tok, const int32_t *parent, const void *clf_w, float clf_b,
                              float tau, int32_t *out_len, int32_t *out_tok, int32_t *out_node, void *stream)
{
    if (!h) return AJ_EINVAL;
    if (h->M > 0 && (!parent || !out_node)) return AJ_EINVAL;
    return verify_common(h, hidden_t, hidden_d, W_lm, draft_tok, clf_w, clf_b, tau, nullptr, 1.f, parent, out_node,
                         out_len, out_tok, stream);
}

extern "C" int aj_verify_sampled(aj_handle *h, const void *hidden_t, const void *hidden_d, const void *W_lm,
                                 const int32_t *draft_tok, const void *clf_w, float clf_b, float tau,
                                 float inv_temperature, const uint64_t *row_key,
                                 int32_t *out_len, int32_t *out_tok, void *stream)
{
    if (!h) return AJ_EINVAL;
    if (!(inv_temperature >= 0.f) || !isfinite(inv_temperature)) return AJ_EINVAL;
    if (h->M > 0 && (!row_key || (((uintptr_t)row_key) & 7u))) return AJ_EINVAL;
    return verify_common(h, hidden_t, hidden_d, W_lm, draft_tok, clf_w, clf_b, tau, row_key, inv_temperature, nullptr,
                         nullptr, out_len, out_tok, stream);
}

extern "C" int aj_verify_topk(aj_handle *h, const void *hidden_t, const void *W_lm, const int32_t *draft_tok,
                              int32_t top_k, int32_t *out_len, int32_t *out_tok, void *stream)
{
    if (!h) return AJ_EINVAL;
    if (top_k < 1) return AJ_EINVAL;
    if (!(h->cfg.flags & AJ_FLAG_TOPK)) return AJ_ESTATE;
    if (h->M == 0) return AJ_OK;
    const aj_config &c = h->cfg;
    if (!hidden_t || !W_lm || !draft_tok || !out_len || !out_tok) return AJ_EINVAL;
    if (!aligned16(hidden_t) || !aligned16(W_lm)) return AJ_EINVAL;
    hipStream_t s = (hipStream_t)stream;

    TopkArgs t;
    t.hidden_t = hidden_t;
    t.W_lm = W_lm;
    t.draft_tok = draft_tok;
    t.B = c.B;
    t.K = c.K;
    t.d_t = c.d_t;
    t.V = c.V;
    t.dtype = c.dtype;
    t.top_k = top_k;
    t.thr = h->thr;
    t.thr_tok = h->thr_tok;
    t.part = h->part;
    t.cnt = h->cnt;
    t.nblocks = h->nblocks;
    t.t_star = h->t_star;
    t.maxlogit = h->maxlogit;
    t.rank = h->rank;
    t.out_len = out_len;
    t.out_tok = out_tok;

    hipError_t e;
    if ((e = topk_draft_logit(t, s)) != hipSuccess) return hip_fail(e);
    const bool prof = h->ev_ok;
    const int slot = (int)(h->calls % 64);
    if (prof && (e = hipEventRecord(h->ev[slot][0], s)) != hipSuccess) return hip_fail(e);
    if ((e = launch_lm_head(h, hidden_t, W_lm, nullptr, s, true)) != hipSuccess) return hip_fail(e);
    if (prof && (e = hipEventRecord(h->ev[slot][1], s)) != hipSuccess) return hip_fail(e);
    if (prof) h->calls++;
    if ((e = topk_tail(t, s)) != hipSuccess) return hip_fail(e);
    return AJ_OK;
}

extern "C" int aj_debug_copy_rank(aj_handle *h, int32_t *rank_host, void *stream)
{
    if (!h || !rank_host) return AJ_EINVAL;
    if (!(h->cfg.flags & AJ_FLAG_TOPK)) return AJ_ESTATE;
    if (h->M == 0) return AJ_OK;
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e == hipSuccess) e = hipMemcpy(rank_host, h->rank, (size_t)h->M * sizeof(int32_t), hipMemcpyDeviceToHost);
    return e == hipSuccess ? AJ_OK : hip_fail(e);
}

extern "C" int aj_debug_ptrs(aj_handle *h, const int32_t **t_star, const float **maxlogit, const float **score)
{
    if (!h) return AJ_EINVAL;
    if (score && !h->score && h->M > 0) return AJ_ESTATE;
    if (t_star) *t_star = h->t_star;
    if (maxlogit) *maxlogit = h->maxlogit;
    if (score) *score = h->score;
    return AJ_OK;
}

extern "C" int aj_debug_copy(aj_handle *h, int32_t *t_star_host, float *maxlogit_host, float *score_host,
                             void *stream)
{
    if (!h) return AJ_EINVAL;
    if (score_host && !h->score && h->M > 0) return AJ_ESTATE;
    if (h->M == 0) return AJ_OK;
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e == hipSuccess && t_star_host)
        e = hipMemcpy(t_star_host, h->t_star, (size_t)h->M * sizeof(int32_t), hipMemcpyDeviceToHost);
    if (e == hipSuccess && maxlogit_host)
        e = hipMemcpy(maxlogit_host, h->maxlogit, (size_t)h->M * sizeof(float), hipMemcpyDeviceToHost);
    if (e == hipSuccess && score_host)
        e = hipMemcpy(score_host, h->score, (size_t)2 * h->cfg.B * h->cfg.K * sizeof(float), hipMemcpyDeviceToHost);
    return e == hipSuccess ? AJ_OK : hip_fail(e);
}

extern "C" int aj_debug_logits(aj_handle *h, const void *hidden_t, const void *W_lm, float *logits, void *stream)
{
    if (!h) return AJ_EINVAL;
    if (h->M == 0) return AJ_OK;
    if (!hidden_t || !W_lm || !logits || !aligned16(hidden_t) || !aligned16(W_lm)) return AJ_EINVAL;
    hipError_t e = launch_lm_head(h, hidden_t, W_lm, logits, (hipStream_t)stream);
    return e == hipSuccess ? AJ_OK : hip_fail(e);
}

extern "C" int aj_profile_read(aj_handle *h, float *ms, int32_t *n)
{
    if (!h || !ms || !n || *n < 0) return AJ_EINVAL;
    if (!h->ev_ok) return AJ_ESTATE;
    const uint64_t have = h->calls < 64 ? h->calls : 64;
    const int want = (int)((uint64_t)*n < have ? (uint64_t)*n : have);
    for (int i = 0; i < want; ++i) {
        const int slot = (int)((h->calls - want + i) % 64);
        hipError_t e = hipEventSynchronize(h->ev[slot][1]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms[i], h->ev[slot][0], h->ev[slot][1]);
        if (e != hipSuccess) return hip_fail(e);
    }
    *n = want;
    return AJ_OK;
}

extern "C" const char *aj_kernel_name(const aj_handle *h)
{
    if (!h) return "none";
    switch (h->variant) {
        case -1: return "lm_head_f32";
        case AJ_KERNEL_TILE: return "lm_head_tile_bf16";
        case AJ_KERNEL_STREAM:
            return h->fp8w ? "lm_head_stream16_fp8w" : h->stream16 ? "lm_head_stream16_bf16" : "lm_head_stream_bf16";
        case AJ_KERNEL_BIG: return "lm_head_big_bf16";
        case AJ_KERNEL_TALL: return "lm_head_tall_bf16";
        case AJ_KERNEL_PAIR: return "lm_head_pair_bf16";
        case AJ_KERNEL_PAIR9: return "lm_head_pair9_bf16";
        case AJ_KERNEL_WIDE: return h->fp8w ? "lm_head_wide_fp8w" : "lm_head_wide_bf16";
        case AJ_KERNEL_RESIDENT: return h->fp8w ? "lm_head_resident_fp8w" : "lm_head_resident_bf16";
        default: return "unknown";
    }
}
