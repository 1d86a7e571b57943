// Internal declarations shared by the HIP translation units of libaj (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aj {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// (value, index) pair ordered by larger value, then lower index.
struct __attribute__((aligned(8))) Best {
    float v;
    int32_t i;
};

// One LM-head launch: logits of M verify rows against V vocabulary rows, reduced per
// (row, vocabulary block) to the block's maximum and its lowest index.
struct LmHeadArgs {
    const void *H;      // [M][d] hidden_t
    const void *W;      // [V][d] W_lm
    int M, V, d;
    Best *part;         // [M][nblocks] block maximum and the lowest vocabulary index attaining it
    int nblocks;        // partials per verify row (fixed by the kernel variant and V)
    float *dump;        // debug: all logits [M][V], or nullptr
    // top-K baseline (all three nullptr otherwise): per verify row the logit and index of its draft
    // token (+inf and -1 for a row without one), and per (row, block) the number of the block's
    // vocabulary entries that are ordered before that token
    const float *thr;       // [M]
    const int32_t *thr_tok; // [M]
    int32_t *cnt;           // [M][nblocks]
    // sampling mode (nullptr otherwise): one 64-bit key per verify row; the kernels maximise
    // logit * inv_temp + Gumbel noise(key, vocabulary index) instead of the logit
    const uint64_t *key;    // [M]
    float inv_temp;
    // fused judge row (nullptr otherwise; accumulator-resident kernel only): judge_w = clf_w[0:d], one more row of
    // the LM-head operand that takes no part in the maximum; its logits go to zt [M]
    const void *judge_w;
    float *zt;
};

__device__ __forceinline__ bool better(float v, int32_t i, float bv, int32_t bi)
{
    return v > bv || (v == bv && i < bi);
}

// top-K baseline: 1 when vocabulary entry v with logit val is ordered before the row's draft token
// (logit th, index tk): larger logit first, lower index first among equals; the token itself never.
__device__ __forceinline__ int32_t ranks_before(float val, int32_t v, float th, int32_t tk)
{
    return (int32_t)((v != tk) & ((val > th) | ((val == th) & (v < tk))));
}

// Sampling mode (Appendix A, "Generalization to sampling": argmax of log-probabilities plus Gumbel noise
// from a generator seeded by the random state and the context).  Counter-based generator, one 64-bit key
// per verify row:  h = v * 0x9E3779 + lo32(key); h ^= h >> 16; h *= 0x85EBCA6B; h ^= hi32(key); h ^= h >> 13;
// h *= 0xC2B2AE35; h ^= h >> 16; h *= 0x27D4EB2F; h ^= h >> 15;  u = ((h >> 9) + 0.5) * 2^-23 (exact in fp32);
// noise = -log(-log(u)).  The largest noise values, which decide the maximum over the vocabulary, come from u
// within 1e-4 of 1, where a hardware log2 has no relative accuracy: there -log(u) = -log(1 - x), x = 1 - u
// (exact), is taken from its series; elsewhere, and for the outer logarithm, the fast log2 is accurate to ~1e-7
// of the result.  
__device__ __forceinline__ float gumbel_noise(uint32_t klo, uint32_t khi, uint32_t v)
{
    uint32_t h = __umul24(v, 0x9E3779u) + klo;       // v < 2^24 and a 24-bit constant: a full-rate multiply-add
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= khi;
    h ^= h >> 13;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    h *= 0x27D4EB2Fu;
    h ^= h >> 15;
    const float u = ((float)(h >> 9) + 0.5f) * (1.0f / 8388608.0f);
    const float x = 1.0f - u;
    // -log(1 - x) = x + x^2/2 + x^3/3 + x^4/4 + x^5/5 + ...: below x = 1/16 the omitted terms are < 2e-8 of the sum
    const float series = x * fmaf(x, fmaf(x, fmaf(x, fmaf(x, 0.2f, 0.25f), 1.0f / 3.0f), 0.5f), 1.0f);
    // v_log_f32 is log2; its arguments here are never subnormal (u >= 2^-24, -log u >= 5.9e-8)
    const float e = x < 0.0625f ? series : -0.69314718f * __builtin_amdgcn_logf(u);
    return -0.69314718f * __builtin_amdgcn_logf(e);
}

// 8 OCP FP8 E4M3 values -> 8 bf16, exactly (E4M3 has 4 significant bits and a narrower exponent range):
// v_cvt_scalef32_pk_bf16_fp8 with scale 1 widens two bytes per instruction
__device__ __forceinline__ bf16x8 fp8x8_to_bf16x8(uint2 raw)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw.x, 1.0f, false);
    const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw.x, 1.0f, true);
    const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw.y, 1.0f, false);
    const bf16x2 e = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw.y, 1.0f, true);
    return bf16x8{a[0], a[1], b[0], b[1], c[0], c[1], e[0], e[1]};
}

// Number of vocabulary blocks (partials per row) each variant produces for V.
int lm_head_tile_blocks(int V);
int lm_head_f32_blocks(int V);
int lm_head_mfma_blocks(int variant, int V, int d, int num_cus);  // variant: AJ_KERNEL_STREAM, _BIG or _TALL
bool lm_head_mfma_supports(int variant, int M, int V, int d);
int lm_head_mfma_padded_rows(int variant, int M);

// Launchers return hipSuccess or the launch error.
hipError_t lm_head_tile_bf16(const LmHeadArgs &a, hipStream_t s);
hipError_t lm_head_f32(const LmHeadArgs &a, hipStream_t s);
hipError_t lm_head_mfma_bf16(int variant, const LmHeadArgs &a, int num_cus, hipStream_t s);

// W_lm-streaming kernel with 16-row tiles and hidden_t in registers (M <= 32, d_t = 2048 or 4096)
bool lm_head_stream16_supports(int M, int V, int d);
int lm_head_stream16_blocks(int V, int num_cus);
hipError_t lm_head_stream16_bf16(const LmHeadArgs &a, int num_cus, hipStream_t s);
// the same kernel with W_lm stored as OCP FP8 E4M3 (hidden_t stays bf16): M <= 32, d_t = 4096
bool lm_head_stream16_fp8w_supports(int M, int V, int d);
hipError_t lm_head_stream16_fp8w(const LmHeadArgs &a, int num_cus, hipStream_t s);

// W_lm-streaming kernel with the logits resident in registers for the whole kernel (M <= 128, d_t % 256 == 0);
// W_lm in bf16 or as OCP FP8 E4M3 bytes (hidden_t stays bf16)
bool lm_head_resident_supports(int M, int V, int d, bool fp8w);
int lm_head_resident_blocks(int V, int num_cus);
hipError_t lm_head_resident_bf16(const LmHeadArgs &a, int num_cus, hipStream_t s);
hipError_t lm_head_resident_fp8w(const LmHeadArgs &a, int num_cus, hipStream_t s);

// 129..272 verify rows in one row tile: 256 vocabulary rows x 16-row blocks, W_lm global -> registers (d_t % 256 == 0)
bool lm_head_wide_supports(int M, int V, int d, bool fp8w);
int lm_head_wide_blocks(int V);
hipError_t lm_head_wide_bf16(const LmHeadArgs &a, int num_cus, hipStream_t s);
hipError_t lm_head_wide_fp8w(const LmHeadArgs &a, int num_cus, hipStream_t s);

// 256 x 256 tiles with paired 64-byte half loads (whole 128-byte lines per request pair); d_t % 256 == 0
bool lm_head_pair_supports(int M, int V, int d);
int lm_head_pair_blocks(int V);
int lm_head_pair_padded_rows(int M);
hipError_t lm_head_pair_bf16(const LmHeadArgs &a, int num_cus, hipStream_t s);

// 256 x 288 tiles, same operand pipeline, 4 waves of 64 x 288 (257..288 verify rows in one row tile)
bool lm_head_pair9_supports(int M, int V, int d);
int lm_head_pair9_blocks(int V);
int lm_head_pair9_padded_rows(int M);
hipError_t lm_head_pair9_bf16(const LmHeadArgs &a, int num_cus, hipStream_t s);

struct TailArgs {
    const void *hidden_t, *hidden_d, *clf_w;
    const int32_t *draft_tok;
    const Best *part;       // [M][nblocks]
    int nblocks;
    int B, K, d_t, d_d, V, dtype, feat_offset;
    float clf_b, zthr;      // zthr = log(tau/(1-tau)), -inf/+inf at the ends
    int32_t *t_star;        // [M] out
    float *maxlogit;        // [M] out
    const float *zt;        // [M] target half of the judge logit of every verify row (fused judge row), or nullptr
    float *score;           // [B][K] out or nullptr
    uint8_t *rej;           // [B][K] workspace of the split form: 1 = slot rejected (nullptr: one-launch form only)
    int32_t *out_len, *out_tok;
    // draft trees (nullptr for chains): parent[B][K] in [-1, j), and the accepted node per window
    const int32_t *parent;
    int32_t *out_node;
};
hipError_t verify_tail(const TailArgs &a, hipStream_t s);     // partials -> t_star; steps 3-4


// Top-K baseline: kernels before and after the LM-head pass
struct TopkArgs {
    const void *hidden_t, *W_lm;
    const int32_t *draft_tok;
    int B, K, d_t, V, dtype, top_k;
    float *thr;             // [M] out of topk_draft_logit, in of the LM head
    int32_t *thr_tok;       // [M]
    const Best *part;       // [M][nblocks]
    const int32_t *cnt;     // [M][nblocks]
    int nblocks;
    int32_t *t_star;        // [M] out
    float *maxlogit;        // [M] out
    int32_t *rank;          // [M] out: rank of the slot's draft token (V: not in the vocabulary; 0 for the bonus row)
    int32_t *out_len, *out_tok;
};
hipError_t topk_draft_logit(const TopkArgs &a, hipStream_t s);
hipError_t topk_tail(const TopkArgs &a, hipStream_t s);

}  // namespace aj
