/* CPU oracle for the load-look-ahead map in the paper's own units (Sec. 3.4.1 "Instance Load
 * Anticipator"): per instance, the number of KV-cache tokens expected to be resident at each of
 * the next map_len decoding iterations.  The paper records the fraction U_i of the token capacity
 * M; this file keeps the token counts N_i = U_i * M as integers (exact), the fraction is N_i / M.
 *
 * TEST INFRASTRUCTURE ONLY: the plain definition the GPU library is checked against.  It shares
 * no code with the GPU path; only tests, the smoke check and the benchmark's CPU-baseline leg may
 * call it.
 *
 * Update rule (Sec. 3.4.1): a request with P prompt tokens and D predicted response tokens whose
 * first decoding iteration is map slot s holds P + i tokens at its i-th iteration, so
 *     N[s + i] += P + i   for i in [0, D).
 * The corrections of the same section are the same ramp over a sub-range of i, added or
 * subtracted: a request that finishes after D' < D iterations has the rest taken out,
 *     N[s + i] -= P + i   for i in [D', D),
 * and one that is still running after D iterations gets a virtual extension [D, D + ext) added,
 * whose unused part is taken out again when it finishes.  One record therefore is
 *     (instance k, slot s, prompt P, i_begin, i_end, sign)  ->  N[k][s + i] += sign * (P + i),
 *     i in [i_begin, i_end).
 * Iterations that fall at or after map_len are counted (signed) in overflow[k].
 *
 * Records with k outside [0, n_inst), s outside [0, map_len), P outside [0, 2^20),
 * i_begin < 0, i_end < i_begin, i_end > 65535 or sign not +1 / -1 are skipped; the index of the
 * first such record is reported.  A slot whose final value does not fit int32 is reported too
 * (its stored value is then the low 32 bits).
 */
#include <stdint.h>
#include <stdlib.h>

/* return: 0 ok, 1 some record skipped, 2 a slot left int32 range, 3 both, -1 no memory */
int pso_lookahead_update(const int32_t *instance_id, const int32_t *start_iter,
                         const int32_t *prompt_tokens, const int32_t *i_begin, const int32_t *i_end,
                         const int32_t *sign, int64_t n_rec, int32_t n_inst, int32_t map_len,
                         int32_t *kv_tokens, int64_t *overflow, int64_t *first_bad)
{
    int status = 0;
    int64_t cells = (int64_t)n_inst * map_len;
    int64_t *acc = (int64_t *)malloc(sizeof(int64_t) * (size_t)(cells > 0 ? cells : 1));
    if (!acc) return -1;
    for (int64_t c = 0; c < cells; ++c) acc[c] = kv_tokens[c];
    *first_bad = -1;

    for (int64_t r = 0; r < n_rec; ++r) {
        int64_t k = instance_id[r], s = start_iter[r], P = prompt_tokens[r];
        int64_t b = i_begin[r], e = i_end[r], sg = sign[r];
        if (k < 0 || k >= n_inst || s < 0 || s >= map_len || P < 0 || P >= (1 << 20) ||
            b < 0 || e < b || e > 65535 || (sg != 1 && sg != -1)) {
            if (*first_bad < 0) *first_bad = r;
            status |= 1;
            continue;
        }
        for (int64_t i = b; i < e; ++i) {
            int64_t t = s + i;
            if (t < map_len) acc[k * map_len + t] += sg * (P + i);
            else             overflow[k] += sg * (P + i);
        }
    }
    for (int64_t c = 0; c < cells; ++c) {
        if (acc[c] > INT32_MAX || acc[c] < INT32_MIN) status |= 2;
        kv_tokens[c] = (int32_t)(uint32_t)(uint64_t)acc[c];
    }
    free(acc);
    return status;
}
