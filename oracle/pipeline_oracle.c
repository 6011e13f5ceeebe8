/*
 * CPU oracle for the pipeline-aware outer reduction (test infrastructure only; the product
 * never links or calls it).
 *
 * The paper lists pipeline parallelism among the searched dimensions (abstract; section 2,
 * "Search Engine") but prints no formula for combining the stages of one pipeline
 * candidate.  Reading used by this build ("parity unpinned" against the paper): a
 * candidate (pipeline degree, stage split, micro-batch count m) owns one solved
 * instance per stage, whose optimum t_stage is the per-micro-batch time of that stage.
 * With the stages run as a synchronous pipeline over m micro-batches the iteration time is
 *     cost = ( t_0 + t_1 + ... + t_{pp-1} ) + (m - 1) * max_stage t_stage
 * evaluated in fp32: the sum left to right over the members in the order given, then the
 * product fl((float)(m-1) * max), then one add.  A candidate is infeasible (+inf) as soon as
 * one member is infeasible (+inf) or its id is outside [0, B).  The winner is the
 * candidate of smallest cost, lowest index on ties, -1 if none is feasible.
 *
 *   stage_cost     [B]        best_cost of every solved instance
 *   group_offsets  [G+1]      CSR offsets into group_members
 *   group_members  [offsets[G]] instance ids
 *   group_micro    [G]        micro-batch count m >= 1
 *   group_cost     out [G]
 *   best_group     out [1]
 */
#include <math.h>
#include <stdint.h>

int oracle_pipeline_reduce(int32_t B, int32_t G, const float *stage_cost,
                           const int32_t *group_offsets, const int32_t *group_members,
                           const int32_t *group_micro, float *group_cost, int32_t *best_group)
{
    if (B < 1 || G < 1 || !stage_cost || !group_offsets || !group_members || !group_micro ||
        !group_cost || !best_group)
        return -1;
    float best = INFINITY;
    int32_t arg = -1;
    for (int32_t g = 0; g < G; ++g) {
        float sum = 0.0f, mx = 0.0f, cost;
        int ok = group_offsets[g + 1] > group_offsets[g] && group_micro[g] >= 1;
        for (int32_t x = group_offsets[g]; ok && x < group_offsets[g + 1]; ++x) {
            const int32_t b = group_members[x];
            if (b < 0 || b >= B || isinf(stage_cost[b])) { ok = 0; break; }
            const float t = stage_cost[b];
            sum = (x == group_offsets[g]) ? t : sum + t;
            if (t > mx) mx = t;
        }
        if (ok) {
            const float bubble = (float)(group_micro[g] - 1) * mx;
            cost = sum + bubble;
        } else {
            cost = INFINITY;
        }
        group_cost[g] = cost;
        if (cost < best) { best = cost; arg = g; }
    }
    *best_group = arg;
    return 0;
}
