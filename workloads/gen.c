/*
 * Seeded synthetic tensors for the judge-augmented verification workloads.
 *
 * This file holds NO arithmetic of the verification method itself: it only
 * draws random numbers and lays them out.  Every element is a pure function
 * of (seed, tensor_id, flat index), so any row range can be produced on its
 * own, in any order, by any number of threads, and always gives the same
 * bytes.
 *
 *   counter hash : two rounds of the splitmix64 finaliser over
 *                  seed, tensor_id and a 64-bit counter
 *   uniform      : top 53 bits, centred, strictly inside (0,1)
 *   normal       : Box-Muller, cosine branch, one value per flat index
 *   bf16         : round-to-nearest-even of the fp32 rounding of the fp64 draw
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { WL_F32 = 0, WL_BF16 = 1 };

static inline uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

static inline uint64_t ctr_hash(uint64_t seed, uint64_t tensor_id, uint64_t ctr)
{
    uint64_t k = mix64(seed + 0x9E3779B97F4A7C15ULL * (tensor_id + 1));
    return mix64(k ^ mix64(ctr + 0xD1B54A32D192ED03ULL));
}

static inline double u01(uint64_t h)
{
    return ((double)(h >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}

static inline double normal_at(uint64_t seed, uint64_t tensor_id, uint64_t idx)
{
    double u1 = u01(ctr_hash(seed, tensor_id, 2 * idx));
    double u2 = u01(ctr_hash(seed, tensor_id, 2 * idx + 1));
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
}

static inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;            /* inputs are finite and far from overflow */
    return (uint16_t)(u >> 16);
}

/* out[i] = uniform(0,1) at counters idx0 .. idx0+n-1 */
void wl_uniform(uint64_t seed, uint64_t tensor_id, uint64_t idx0, uint64_t n, double *out)
{
    for (uint64_t i = 0; i < n; ++i)
        out[i] = u01(ctr_hash(seed, tensor_id, idx0 + i));
}

/*
 * Rows row0 .. row0+rows-1 of a [*, cols] tensor of N(0, std^2) draws.
 * rms_norm != 0: each row is divided by sqrt(mean of squares) (in fp64, before
 * the cast), i.e. a unit-gain RMSNorm output; std is then irrelevant.
 * dtype selects the storage type of `out` (fp32 or bf16 as uint16).
 * Returns 0, or -1 on a bad argument / allocation failure.
 */
int wl_normal_rows(uint64_t seed, uint64_t tensor_id, uint64_t row0, uint64_t rows,
                   uint64_t cols, double std, int rms_norm, int dtype, void *out)
{
    if (!out || (dtype != WL_F32 && dtype != WL_BF16) || cols == 0)
        return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *tmp = (double *)malloc(sizeof(double) * cols);
        if (!tmp) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (int64_t r = 0; r < (int64_t)rows; ++r) {
            if (!tmp)
                continue;
            uint64_t base = (row0 + (uint64_t)r) * cols;
            double ss = 0.0;
            for (uint64_t c = 0; c < cols; ++c) {
                tmp[c] = std * normal_at(seed, tensor_id, base + c);
                ss += tmp[c] * tmp[c];
            }
            double scale = 1.0;
            if (rms_norm)
                scale = 1.0 / sqrt(ss / (double)cols);
            if (dtype == WL_F32) {
                float *o = (float *)out + (uint64_t)r * cols;
                for (uint64_t c = 0; c < cols; ++c)
                    o[c] = (float)(tmp[c] * scale);
            } else {
                uint16_t *o = (uint16_t *)out + (uint64_t)r * cols;
                for (uint64_t c = 0; c < cols; ++c)
                    o[c] = f32_to_bf16_rne((float)(tmp[c] * scale));
            }
        }
        free(tmp);
    }
    return fail ? -1 : 0;
}
