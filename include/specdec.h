/*
 * specdec.h -- C ABI of the verification step of speculative decoding
 * (Algorithm 1: "determine the accepted token length n_t" and "verify and update
 * the draft sequence") on batches of synthetic draft / target distributions.
 *
 * A batch holds B independent steps.  Step b has k draft positions over a
 * vocabulary of V tokens:
 *   q[b][j][.]  draft distribution at position j (j < k),
 *   p[b][j][.]  target distribution at position j (j <= k; row k is used when
 *               every draft token is accepted),
 *   tok[b][j]   the draft token x_j (drawn from q[b][j] by the caller),
 *   r[b][j]     the uniform r_j in [0, 1) of the acceptance test,
 *   u[b]        a uniform 32-bit integer for the resampling draw.
 * All arrays are DEVICE pointers, row-major float32 / int32 / uint32, owned by the
 * caller and read-only; outputs are device pointers owned by the caller.  Calls
 * are asynchronous on `hip_stream` (a hipStream_t; NULL = default stream).  The
 * library allocates nothing.
 *
 * Every function returns 0 or a negative sd_status.
 */
#ifndef SPECDEC_H
#define SPECDEC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SD_OK = 0,
    SD_EINVAL = -1,        /* null / misaligned pointer, non-positive size */
    SD_EUNSUPPORTED = -2,  /* k > SD_MAX_K or V > SD_MAX_V */
    SD_EHIP = -3           /* HIP runtime error */
} sd_status;

#define SD_MAX_K 64         /* candidate length */
#define SD_MAX_V 262144     /* vocabulary size */
#define SD_FIXED_BITS 40    /* probabilities are summed as integers in units of 2^-40 */

/*
 * Accepted length and next token of every step (Algorithm 1):
 *   n[b]    = min({ j : r_j > p_j(x_j) / q_j(x_j) } U { k })   (0-based j: the number of
 *             accepted draft tokens); the test is evaluated as NOT(r_j * q_j(x_j) <= p_j(x_j))
 *             in float32, so q_j(x_j) = 0 accepts;
 *   next[b] ~ p' with p'(x) proportional to max(0, p_n(x) - q_n(x)) if n < k, and p' = p_k
 *             otherwise.
 * The draw is the inverse CDF in exact integer arithmetic, so it does not depend on
 * summation order: m(x) = trunc(2^40 * max(0, p_n(x) - q_n(x))) (float32 subtraction),
 * Z = sum_x m(x), target = floor(Z * u / 2^32), next = the smallest x whose inclusive prefix
 * sum exceeds target.  If Z == 0 (the residual vanishes at this resolution) p' = p_n.
 * tok values outside [0, V) are clamped.  n_dev, next_dev: device [B] int32.
 */
int sd_verify(const float *p_dev, const float *q_dev, const int32_t *tok_dev, const float *r_dev,
              const uint32_t *u_dev, int64_t B, int64_t k, int64_t V, int32_t *n_dev,
              int32_t *next_dev, void *hip_stream);

/*
 * Acceptance rate of every draft position, Eq. (1):
 *   acc[b][j] = E_{x ~ q_j} min{1, p_j(x) / q_j(x)} = sum_x min(p_j(x), q_j(x)) = 1 - TV(p_j, q_j),
 * summed in float64 in a fixed order.  acc_dev: device [B][k] float64.  p_dev has k+1 rows
 * per step as in sd_verify (row k is not read).
 */
int sd_acceptance(const float *p_dev, const float *q_dev, int64_t B, int64_t k, int64_t V,
                  double *acc_dev, void *hip_stream);

/* Static, human-readable text for a status code. */
const char *sd_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SPECDEC_H */
