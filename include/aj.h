/*
 * libaj - judge-augmented verification of speculation windows on AMD MI355X (gfx950).
 *
 * One call verifies a batch of B speculation windows, each holding K draft
 * tokens plus one bonus position (K+1 "verify rows" per window):
 *
 *   1. LM head     logit[r][v] = sum_k hidden_t[r][k] * W_lm[v][k]
 *   2. greedy      t*[r] = lowest v attaining max_v logit[r][v]
 *                  (greedy verification compares the draft tokens with the
 *                   target's own next-token predictions: Section 2, footnote)
 *   3. judge       slot j mismatches when t*[b][j] != draft_tok[b][j]; at a
 *                  mismatch z = clf_w . [hidden_t[b][j+o] ; hidden_d[b][j+o]] + clf_b
 *                  with o = feat_offset (1: the states that encode the draft
 *                  token, Section 3.2 item 1 and Appendix B); the mismatch is
 *                  accepted when sigmoid(z) < tau (Section 3.3: the classifier is
 *                  called where the base algorithm would reject; an unimportant
 *                  token is accepted and verification goes on)
 *   4. scan        out_len[b] = first slot that mismatches and is not accepted
 *                  (K if none); out_tok[b] = t*[b][out_len[b]]: the target's
 *                  correction token, or the bonus token when out_len == K
 *                  (Section 2: the first mismatching token and all after it are
 *                  rejected).
 *
 * The B*(K+1) x V logits are never written to memory.  The threshold test is
 * evaluated as z < log(tau/(1-tau)) (-inf / +inf at tau = 0 / 1), which equals
 * sigmoid(z) < tau in real arithmetic and makes tau = 0 plain greedy
 * speculative decoding and tau = 1 accept every draft token.
 *
 * aj_verify is that path.  On the same LM-head pass: aj_verify_sampled (step 2 samples the target's
 * token with the Gumbel-max trick instead of taking the maximum), aj_verify_tree (the K slots form a
 * draft tree), aj_verify_topk (the paper's top-K lossy baseline in place of the judge).
 *
 * Conventions
 *   - All tensor arguments are DEVICE pointers owned by the caller, row-major,
 *     16-byte aligned; clf_b and tau are host scalars.  The library keeps none
 *     of them past the call.  Inputs must be finite.
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream); outputs are valid once the stream has been
 *     synchronised.  No host<->device copies, no host synchronisation.
 *   - A handle owns a device workspace sized at aj_create; one handle = one
 *     call in flight.  Different handles are independent.
 *   - Every function returns AJ_OK (0) or a negative aj_status; nothing throws.
 *     Draft tokens outside [0, V) are legal and simply never match.
 */
#ifndef AJ_H
#define AJ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct aj_handle aj_handle; /* opaque */

typedef enum { AJ_F32 = 0, AJ_BF16 = 1 } aj_dtype;

typedef enum {
    AJ_OK = 0,
    AJ_EINVAL = -1,  /* null pointer, bad shape, tau outside [0,1] or NaN, misaligned pointer */
    AJ_ENOMEM = -2,  /* workspace allocation failed */
    AJ_EHIP = -3,    /* a HIP call failed; aj_last_hip_error() has the hipError_t */
    AJ_ESTATE = -4,  /* call not valid for this handle (e.g. debug data not enabled) */
    AJ_ELIMIT = -5   /* aj_verify_static: the shape needs more workspace than the static buffer holds */
} aj_status;

enum {
    AJ_FLAG_DEBUG = 1,   /* keep per-slot judge scores for aj_debug_ptrs */
    AJ_FLAG_PROFILE = 2, /* record HIP events around the LM-head kernel (aj_profile_read) */
    AJ_FLAG_TOPK = 4,    /* also allocate the workspace of aj_verify_topk */
    AJ_FLAG_FUSED_JUDGE = 8 /* the judge's target half, clf_w[0:d_t] . hidden_t[r], is computed for EVERY verify row
                               inside the LM-head pass, as one more row of the LM-head operand (Section 3.2, "Classifier
                               model": the regression can be fused with the LM head layer); at a mismatch the tail then adds
                               only the draft half and the bias.  Same results within the score tolerance.  Served by the
                               kernel for up to 128 verify rows at d_t % 256 == 0 with bf16 weights (AJ_EINVAL otherwise);
                               aj_verify_sampled and aj_verify_topk calls on such a handle compute the judge as usual. */
};

enum { AJ_W_SAME = 0, AJ_W_FP8_E4M3 = 1 };

/* LM-head kernel choice; AJ_KERNEL_AUTO picks by shape. The others force one for tests/benchmarks. */
enum { AJ_KERNEL_AUTO = 0, AJ_KERNEL_TILE = 1, AJ_KERNEL_STREAM = 2, AJ_KERNEL_BIG = 3, AJ_KERNEL_TALL = 4,
       AJ_KERNEL_PAIR = 5, AJ_KERNEL_PAIR9 = 6, AJ_KERNEL_RESIDENT = 7, AJ_KERNEL_WIDE = 8 };

typedef struct {
    int32_t B;           /* windows per call, >= 0 (0: the call does nothing) */
    int32_t K;           /* draft tokens per window, 1 <= K <= 1023 */
    int32_t d_t;         /* target hidden size; multiple of 8 (bf16) or 4 (f32) */
    int32_t d_d;         /* draft hidden size; 0 = judge on target states only; same multiples */
    int32_t V;           /* vocabulary size, 1 <= V < 2^24 */
    int32_t dtype;       /* aj_dtype of hidden_t, hidden_d, W_lm, clf_w */
    int32_t feat_offset; /* 1 (default) or 0: the judge reads verify row j + feat_offset */
    int32_t flags;       /* AJ_FLAG_* */
    int32_t kernel;      /* AJ_KERNEL_* */
    int32_t w_dtype;     /* storage of W_lm: AJ_W_SAME (0) = `dtype`; AJ_W_FP8_E4M3 = OCP FP8 E4M3 bytes [V][d_t],
                            widened exactly to bf16 in registers (the 405B run of Section 4 serves the LM head in
                            FP8); needs dtype = AJ_BF16 and either B*(K+1) <= 128 with d_t a multiple of 256 or
                            B*(K+1) <= 272 with d_t a multiple of 512 (AJ_EINVAL otherwise: beyond that the path is
                            bound by the matrix pipe, not by the bytes of W_lm) and is not available to aj_verify_topk.  A per-tensor scale of the FP8 weights is the caller's
                            business: no step of the path depends on the scale of the logits except the
                            temperature of aj_verify_sampled, into which it can be folded. */
} aj_config;

/* Validate cfg, allocate the workspace on the current device. *out is NULL on failure. */
int aj_create(const aj_config *cfg, aj_handle **out);

/*
 * Steps 1-4 (see the top of this file).
 *   hidden_t  [B][K+1][d_t]   target final hidden states
 *   hidden_d  [B][K+1][d_d]   draft final hidden states (may be NULL when d_d == 0)
 *   W_lm      [V][d_t]        LM-head weight
 *   draft_tok [B][K] int32
 *   clf_w     [d_t + d_d]     judge weight, target part first
 *   out_len   [B] int32       accepted draft tokens, in [0, K]
 *   out_tok   [B] int32       emitted token, in [0, V)
 * AJ_EINVAL on null / misaligned pointers, tau outside [0,1] or NaN, or a non-finite clf_b; AJ_EHIP on a
 * launch failure.
 */
int aj_verify(aj_handle *h, const void *hidden_t, const void *hidden_d, const void *W_lm,
              const int32_t *draft_tok, const void *clf_w, float clf_b, float tau,
              int32_t *out_len, int32_t *out_tok, void *stream);

/*
 * aj_verify for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  No handle: the call takes the configuration itself (flags must be 0) and keeps its
 * workspace (per-block maxima, greedy tokens) in a static device array of AJ_STATIC_SCRATCH_BYTES that every GPU
 * the library runs on holds until the process ends.  It calls no hipMalloc / hipFree or any other allocating
 * routine; the first call on a device looks the array's address up once.  Same kernels, same results and same
 * errors as aj_create + aj_verify, plus
 *   AJ_ELIMIT when B*(K+1) * (partials per row) * 8 + 3 * B*(K+1) * 4 bytes (each part rounded up to 256)
 *             exceed AJ_STATIC_SCRATCH_BYTES: e.g. 70B-shaped, 8 windows x 33 rows needs 1.1 MB and fits,
 *             128 windows x 65 rows needs 33 MB and does not; use a handle for those;
 *   AJ_EINVAL when cfg->flags != 0 (debug scores, profiling and the top-K workspace live in handles).
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (different streams or
 * threads) race; calls on one stream are ordered and safe.  Nothing in the array has to start at zero - every
 * word a call reads it has written itself - so a call is not affected by what the previous one left.
 */
#define AJ_STATIC_SCRATCH_BYTES (8u << 20)
int aj_verify_static(const aj_config *cfg, const void *hidden_t, const void *hidden_d, const void *W_lm,
                     const int32_t *draft_tok, const void *clf_w, float clf_b, float tau,
                     int32_t *out_len, int32_t *out_tok, void *stream);

/*
 * The same steps on draft TREES (Section 3.3, "Generality": the judge applies to tree-based verification
 * stages as well; the rule of aj_verify is applied edge by edge).  The K slots of a window are tree nodes:
 *   parent    [B][K] int32   device; parent[b][j] in [-1, j) is node j's parent (-1 = the root, i.e. the
 *                            context); parents come before their children.  Values outside that range are
 *                            clamped into it.
 *   hidden_t / hidden_d      row 0 of a window = the root's state, row j+1 = the state that has consumed node
 *                            j's token
 * Node j is checked against the greedy token of its parent's row; at a mismatch the judge reads row j+1
 * (feat_offset = 1; the parent's row with feat_offset = 0).  A node is accepted when its edge matches or is
 * judged unimportant AND its parent is accepted.  Outputs per window:
 *   out_node [B] int32       the accepted node of greatest depth, lowest index among equals; -1 if none
 *   out_len  [B] int32       its depth (tokens on the accepted path, which parent[] spells out)
 *   out_tok  [B] int32       greedy token of that node's row (of row 0 when out_node = -1)
 * With parent[b][j] = j - 1 this is aj_verify; with tau = 0 it is greedy tree verification.
 * Errors as aj_verify, plus AJ_EINVAL for a null parent or out_node.
 */
int aj_verify_tree(aj_handle *h, const void *hidden_t, const void *hidden_d, const void *W_lm,
                   const int32_t *draft_tok, const int32_t *parent, const void *clf_w, float clf_b, float tau,
                   int32_t *out_len, int32_t *out_tok, int32_t *out_node, void *stream);

/*
 * The same steps for stochastic decoding, made a deterministic function of a random state with the
 * Gumbel-max trick (Appendix A, "Generalization to sampling"): the target's token of a verify row is
 *     y[r] = lowest v attaining max_v ( logit[r][v] * inv_temperature + G(row_key[r], v) )
 * with G standard Gumbel noise, so that y[r] is distributed as softmax(logit[r] / T); the mismatch test,
 * the judge and the scan then run on y as they do on the greedy token in aj_verify.
 *   row_key [B][K+1] uint64  device; one key per verify row - what the caller's random state joined with
 *                            the row's context hashes to (the same key gives the same noise)
 *   inv_temperature          1/T >= 0, finite (0: uniformly random tokens; large: greedy decoding)
 * Noise generator (counter-based, any (row, v) on its own), all arithmetic mod 2^32:
 *     h = v * 0x9E3779 + lo32(key); h ^= h >> 16; h *= 0x85EBCA6B; h ^= hi32(key);
 *     h ^= h >> 13; h *= 0xC2B2AE35; h ^= h >> 16; h *= 0x27D4EB2F; h ^= h >> 15;
 *     u = ((h >> 9) + 0.5) * 2^-23;   G = -log(-log(u))
 * aj_debug_* then report y and the perturbed maximum in place of the greedy token and its logit.
 * Errors as aj_verify, plus AJ_EINVAL for a null or misaligned row_key or a bad inv_temperature.
 */
int aj_verify_sampled(aj_handle *h, const void *hidden_t, const void *hidden_d, const void *W_lm,
                      const int32_t *draft_tok, const void *clf_w, float clf_b, float tau,
                      float inv_temperature, const uint64_t *row_key,
                      int32_t *out_len, int32_t *out_tok, void *stream);

/*
 * The top-K lossy baseline the paper compares against (Section 4, "Our baselines"): a mismatching
 * draft token is accepted when it is within the top_k most likely tokens of the target model.  Same
 * LM-head pass as aj_verify; instead of the judge, every logit of a verify row is compared, while still
 * in registers, with the logit of the row's draft token:
 *   rank[b][j] = number of vocabulary entries ordered before draft_tok[b][j] in row (b, j)
 *                (larger logit first, lower index first among equal logits; rank 0 = greedy token);
 *                V for a token outside [0, V).  The token's own logit is computed by a separate dot product,
 *                so entries within fp32 rounding of it (~1e-6 relative) may fall on either side; the greedy
 *                token is given rank 0 outright
 *   out_len[b] = first slot with rank >= top_k (K if none), out_tok[b] = greedy token of that row.
 * top_k = 1 is plain greedy verification, top_k >= V accepts every valid token.
 * Needs AJ_FLAG_TOPK at aj_create (AJ_ESTATE otherwise); AJ_EINVAL on null / misaligned pointers or
 * top_k < 1.  Arguments as in aj_verify.
 */
int aj_verify_topk(aj_handle *h, const void *hidden_t, const void *W_lm, const int32_t *draft_tok,
                   int32_t top_k, int32_t *out_len, int32_t *out_tok, void *stream);

/*
 * After aj_verify_topk: rank [B*(K+1)] int32 (0 at the bonus row of each window) copied to a HOST
 * array; synchronises `stream` first.  t_star / maxlogit of that call are read with aj_debug_copy.
 */
int aj_debug_copy_rank(aj_handle *h, int32_t *rank_host, void *stream);

/* Frees the workspace. The caller must have synchronised any stream still using the handle. */
int aj_destroy(aj_handle *h);

/*
 * Device pointers into the handle's workspace, valid after the stream of the last
 * aj_verify has been synchronised and until the next call / aj_destroy:
 *   t_star   [B*(K+1)] int32  greedy token of every verify row           (always kept)
 *   maxlogit [B*(K+1)] float  its logit                                   (always kept)
 *   score    [2][B][K] float  plane 0: judge logit z, plane 1: sigmoid(z) = P(important), at
 *                             mismatching slots; NaN at matching ones
 *                             (AJ_FLAG_DEBUG only, else AJ_ESTATE if requested)
 * Any of the three out-pointers may be NULL.
 */
int aj_debug_ptrs(aj_handle *h, const int32_t **t_star, const float **maxlogit, const float **score);

/*
 * Same data copied to HOST arrays of the sizes above (NULL to skip one). Synchronises `stream`
 * (the one of the last aj_verify) first, then copies synchronously.
 */
int aj_debug_copy(aj_handle *h, int32_t *t_star_host, float *maxlogit_host, float *score_host, void *stream);

/*
 * Debug: step 1 alone, writing all logits [B*(K+1)][V] as float to device memory
 * `logits` (the product path never does this). Uses the same kernels as aj_verify.
 */
int aj_debug_logits(aj_handle *h, const void *hidden_t, const void *W_lm, float *logits, void *stream);

/*
 * AJ_FLAG_PROFILE: synchronises the events of the most recent calls (at most 64 are
 * kept) and writes the LM-head kernel's duration of each, oldest first, in
 * milliseconds; *n in: capacity of ms, out: count written.
 */
int aj_profile_read(aj_handle *h, float *ms, int32_t *n);

/* Name of the LM-head kernel variant this handle dispatches to (static string). */
const char *aj_kernel_name(const aj_handle *h);

const char *aj_strerror(int status);
int aj_last_hip_error(void); /* hipError_t of the last AJ_EHIP on this thread */

#ifdef __cplusplus
}
#endif
#endif /* AJ_H */
