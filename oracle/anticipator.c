/* CPU oracle for the instance load anticipator (paper Sec. 3.4.1 "Instance Load
 * Anticipator"): fold per-request predicted response lengths into per-instance
 * future-load curves.
 *
 * TEST INFRASTRUCTURE ONLY: the plain definition the GPU library is checked against.
 * It shares no code with the GPU path; only tests, the smoke check and the benchmark's
 * CPU-baseline leg may call it.
 *
 * The paper's look-ahead map holds, per instance, the load expected at each future step,
 * and is updated per request once its response length D has been predicted (Sec. 3.4.1).
 * Here a step is a one-second bucket and what is recorded is the number of tokens the
 * instance is expected to decode in that second: a request that arrives in bucket a on
 * instance k decodes its D predicted tokens over `dur` consecutive buckets a, a+1, ...,
 * spread as evenly as integers allow, the earlier buckets taking the remainder.
 *   rate == NULL : dur = horizon - a            (spread to the end of the horizon)
 *   otherwise    : dur = ceil(D / rate[k])      (the instance decodes rate[k] tokens/s)
 * Tokens that fall at or after `horizon` are counted in overflow[k], so that for every
 * instance  sum_b load[k][b] + overflow[k]  grows by exactly the sum of its requests' D.
 *
 * Records with D < 0, k outside [0, n_inst), a outside [0, horizon) or rate[k] < 1 are
 * skipped; the index of the first such record is reported.  A bucket whose final value
 * does not fit int32 is reported too (its stored value is then the low 32 bits).
 */
#include <stdint.h>
#include <stdlib.h>

/* return: 0 ok, 1 some record skipped, 2 a bucket left int32 range, 3 both, -1 no memory */
int pso_anticipate(const int32_t *pred_tokens, const int32_t *instance_id,
                   const int32_t *arrival_bucket, const int32_t *rate, int64_t n_req,
                   int32_t n_inst, int32_t horizon, int32_t *load, int64_t *overflow,
                   int64_t *first_bad)
{
    int status = 0;
    int64_t cells = (int64_t)n_inst * horizon;
    int64_t *acc = (int64_t *)malloc(sizeof(int64_t) * (size_t)(cells > 0 ? cells : 1));
    if (!acc) return -1;
    for (int64_t i = 0; i < cells; ++i) acc[i] = load[i];
    *first_bad = -1;

    for (int64_t r = 0; r < n_req; ++r) {
        int64_t D = pred_tokens[r];
        int64_t k = instance_id[r];
        int64_t a = arrival_bucket[r];
        if (D < 0 || k < 0 || k >= n_inst || a < 0 || a >= horizon || (rate && rate[k] < 1)) {
            if (*first_bad < 0) *first_bad = r;
            status |= 1;
            continue;
        }
        if (D == 0) continue;
        int64_t dur = rate ? (D + rate[k] - 1) / rate[k] : (int64_t)horizon - a;
        int64_t q = D / dur, rem = D % dur;
        for (int64_t j = 0; j < dur; ++j) {
            int64_t c = q + (j < rem ? 1 : 0);
            int64_t b = a + j;
            if (b < horizon) acc[k * horizon + b] += c;
            else             overflow[k] += c;
        }
    }
    for (int64_t i = 0; i < cells; ++i) {
        if (acc[i] > INT32_MAX || acc[i] < INT32_MIN) status |= 2;
        load[i] = (int32_t)(uint32_t)(uint64_t)acc[i];
    }
    free(acc);
    return status;
}
