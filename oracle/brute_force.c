/*
 * Exhaustive check of the strategy-search problem on tiny instances (test
 * infrastructure only; used to pin the dynamic-programming oracle, never by the
 * product).  It knows nothing about the recurrence: it walks every plan in
 * {0..S-1}^L like an odometer, drops the plans whose memory exceeds the budget and
 * keeps the smallest fp32 chain cost, the chain being summed left to right as
 * acc = (acc + R) + T  (paper section 2, "Search Engine": the most effective
 * combination of per-layer strategies that fits the device memory).
 */
#include <math.h>
#include <stdint.h>

/* Returns the number of feasible plans (or -1 on bad arguments / too many plans).
 *   min_cost  out: smallest chain cost over feasible plans, +inf when there is none
 *   n_optimal out: how many feasible plans attain it (0 when there is none)        */
int64_t oracle_brute_force(int32_t L, int32_t S, int32_t E, int32_t K,
                           const float *T, const int32_t *O, const float *R,
                           const int32_t *r_index, float *min_cost, int64_t *n_optimal)
{
    if (L < 1 || L > 16 || S < 1 || E < 0 || K < 1) return -1;
    double total = 1.0;
    for (int32_t l = 0; l < L; ++l) total *= (double)S;
    if (total > 5.0e7) return -1;

    int32_t digit[16];
    for (int32_t l = 0; l < L; ++l) digit[l] = 0;
    float best = INFINITY;
    int64_t feasible = 0, ties = 0;
    for (;;) {
        int64_t mem = 0;
        for (int32_t l = 0; l < L; ++l) mem += O[(int64_t)l * S + digit[l]];
        if (mem <= (int64_t)E) {
            float acc = T[digit[0]];
            for (int32_t l = 1; l < L; ++l) {
                const float *Rl = R + (int64_t)r_index[l] * S * S;
                acc = acc + Rl[(int64_t)digit[l - 1] * S + digit[l]];
                acc = acc + T[(int64_t)l * S + digit[l]];
            }
            ++feasible;
            if (acc < best) { best = acc; ties = 1; }
            else if (acc == best) ++ties;
        }
        int32_t pos = L - 1;
        while (pos >= 0 && ++digit[pos] == S) { digit[pos] = 0; --pos; }
        if (pos < 0) break;
    }
    *min_cost = best;
    *n_optimal = (feasible > 0) ? ties : 0;
    return feasible;
}
