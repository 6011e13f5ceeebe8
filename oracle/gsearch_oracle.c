/*
 * CPU oracle for the layer-wise strategy-search dynamic program of the Galvatron
 * search engine (paper section 2, "Search Engine": a strategy is chosen for every
 * model layer by dynamic programming under the device-memory constraint; section 1,
 * feature 2: the choice balances memory against computation and communication time).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded reference
 * that the tests, the smoke check and the benchmark's cpu_baseline leg call.  The
 * product (the HIP library) never links, loads or calls it, and it shares no code,
 * header, table or helper with the HIP sources.
 *
 * Problem statement (one instance):
 *   L layers, S candidate strategies per layer, a memory budget of E bins.
 *   T[l][s]  time of layer l under strategy s            (fp32, >= 0, finite)
 *   O[l][s]  memory of layer l under strategy s in bins  (int32, >= 0)
 *   R[k][si][sj] cost of switching from strategy si (previous layer) to sj (this
 *                layer); layer l >= 1 uses matrix k = r_index[l]
 *   Over all plans p in {0..S-1}^L with sum_l O[l][p_l] <= E minimise
 *       cost(p) = T[0][p_0] (+) sum_{l>=1} ( R[r_index[l]][p_{l-1}][p_l] (+) T[l][p_l] )
 *   evaluated in fp32 left to right as acc = (acc + R) + T.
 *
 * The optimum is reached exactly by the recurrence
 *   C[0][e][s]  = T[0][s]                          if e >= O[0][s], else +inf
 *   C[l][e][sj] = ( min_si ( C[l-1][e-O[l][sj]][si] + R[si][sj] ) ) + T[l][sj]
 *                                                  if e >= O[l][sj], else +inf
 *   bp[l][e][sj] = the lowest si attaining the min (0 when every candidate is +inf
 *                  or the state does not fit)
 * where e means "at most e bins are used".  Because fp32 addition is monotone the
 * recurrence value equals the minimum of the fp32 chain costs bit for bit; the scan
 * order below (si ascending, strict <) only fixes which optimal plan is reported.
 *
 * Cost-table model and strategy enumeration: the paper names them (decision-tree
 * enumeration of data / tensor / sharded-data / sequence degrees and recomputation
 * with infeasible combinations discarded; time and memory cost models per strategy)
 * but prints no formula.  The alpha-beta form used here is this build's own reading
 * and is therefore "parity unpinned" against the paper; its arithmetic is pinned
 * only by closed-form special cases in the tests.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_BAD_ARG (-1)
#define ORACLE_NO_MEM (-2)

/* ------------------------------------------------------------------------------------------
 * Forward recurrence + final minimum + backtrace for ONE instance.
 *
 *   T, O        [L][S]
 *   R           [K][S][S], R[k][si][sj]
 *   r_index     [L]  (entry 0 is ignored: layer 0 has no predecessor)
 *   best_cost   out: min_s C[L-1][E][s]  (+inf when no plan fits)
 *   best_s      out: lowest s attaining it, -1 when infeasible
 *   final_row   out [S] or NULL: C[L-1][E][.]
 *   plan        out [L] or NULL: chosen strategy per layer, all -1 when infeasible
 *   mem_used    out or NULL: sum of O along the plan, -1 when infeasible
 *   curve       out [E+1] or NULL: min_s C[L-1][e][s] for every e in 0..E
 *   C_all       out [L][E+1][S] or NULL: every plane of the recurrence
 *   bp_all      out [L][E+1][S] or NULL: every backpointer (plane 0 is all 0)
 * ---------------------------------------------------------------------------------------- */
int oracle_solve(int32_t L, int32_t S, int32_t E, int32_t K,
                 const float *T, const int32_t *O, const float *R, const int32_t *r_index,
                 float *best_cost, int32_t *best_s, float *final_row,
                 int32_t *plan, int32_t *mem_used, float *curve,
                 float *C_all, uint16_t *bp_all)
{
    if (L < 1 || S < 1 || S > 65535 || E < 0 || K < 1 || !T || !O || !R || !r_index ||
        !best_cost || !best_s)
        return ORACLE_BAD_ARG;
    for (int32_t l = 1; l < L; ++l)
        if (r_index[l] < 0 || r_index[l] >= K) return ORACLE_BAD_ARG;
    for (int64_t x = 0; x < (int64_t)L * S; ++x)
        if (O[x] < 0) return ORACLE_BAD_ARG;

    const size_t plane = (size_t)(E + 1) * (size_t)S;
    float *C = (float *)malloc(sizeof(float) * plane * (size_t)L);
    uint16_t *bp = (uint16_t *)malloc(sizeof(uint16_t) * plane * (size_t)L);
    if (!C || !bp) { free(C); free(bp); return ORACLE_NO_MEM; }

    /* layer 0: no transition term */
    for (int32_t e = 0; e <= E; ++e)
        for (int32_t s = 0; s < S; ++s) {
            C[(size_t)e * S + s] = (e >= O[s]) ? T[s] : INFINITY;
            bp[(size_t)e * S + s] = 0;
        }

    for (int32_t l = 1; l < L; ++l) {
        const float *Cp = C + plane * (size_t)(l - 1);
        float *Cl = C + plane * (size_t)l;
        uint16_t *bl = bp + plane * (size_t)l;
        const float *Rl = R + (size_t)r_index[l] * S * S;
        for (int32_t e = 0; e <= E; ++e)
            for (int32_t j = 0; j < S; ++j) {
                const int32_t o = O[(size_t)l * S + j];
                if (e < o) {
                    Cl[(size_t)e * S + j] = INFINITY;
                    bl[(size_t)e * S + j] = 0;
                    continue;
                }
                const float *src = Cp + (size_t)(e - o) * S;
                float best = INFINITY;
                int32_t arg = 0;
                for (int32_t i = 0; i < S; ++i) {
                    const float v = src[i] + Rl[(size_t)i * S + j];
                    if (v < best) { best = v; arg = i; }
                }
                Cl[(size_t)e * S + j] = best + T[(size_t)l * S + j];
                bl[(size_t)e * S + j] = (uint16_t)arg;
            }
    }

    /* final minimum at the full budget, lowest index on ties */
    const float *last = C + plane * (size_t)(L - 1);
    float bc = INFINITY;
    int32_t bs = -1;
    for (int32_t s = 0; s < S; ++s) {
        const float v = last[(size_t)E * S + s];
        if (v < bc) { bc = v; bs = s; }
    }
    *best_cost = bc;
    *best_s = bs;
    if (final_row)
        for (int32_t s = 0; s < S; ++s) final_row[s] = last[(size_t)E * S + s];
    if (curve)
        for (int32_t e = 0; e <= E; ++e) {
            float m = INFINITY;
            for (int32_t s = 0; s < S; ++s) {
                const float v = last[(size_t)e * S + s];
                if (v < m) m = v;
            }
            curve[e] = m;
        }

    /* backtrace from (L-1, E, best_s) */
    if (plan || mem_used) {
        if (bs < 0) {
            if (plan) for (int32_t l = 0; l < L; ++l) plan[l] = -1;
            if (mem_used) *mem_used = -1;
        } else {
            int32_t s = bs, e = E, used = 0;
            for (int32_t l = L - 1; l >= 1; --l) {
                if (plan) plan[l] = s;
                const int32_t prev = bp[plane * (size_t)l + (size_t)e * S + s];
                const int32_t o = O[(size_t)l * S + s];
                used += o;
                e -= o;
                s = prev;
            }
            if (plan) plan[0] = s;
            used += O[s];
            if (mem_used) *mem_used = used;
        }
    }

    if (C_all) memcpy(C_all, C, sizeof(float) * plane * (size_t)L);
    if (bp_all) memcpy(bp_all, bp, sizeof(uint16_t) * plane * (size_t)L);
    free(C);
    free(bp);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------
 * Re-evaluate one plan: fp32 chain cost in the defining order and its memory use.
 * ---------------------------------------------------------------------------------------- */
int oracle_plan_cost(int32_t L, int32_t S, int32_t K,
                     const float *T, const int32_t *O, const float *R, const int32_t *r_index,
                     const int32_t *plan, float *cost, int32_t *mem)
{
    if (L < 1 || S < 1 || K < 1 || !plan || !cost || !mem) return ORACLE_BAD_ARG;
    for (int32_t l = 0; l < L; ++l)
        if (plan[l] < 0 || plan[l] >= S) return ORACLE_BAD_ARG;
    float acc = T[plan[0]];
    int32_t used = O[plan[0]];
    for (int32_t l = 1; l < L; ++l) {
        const float *Rl = R + (size_t)r_index[l] * S * S;
        acc = acc + Rl[(size_t)plan[l - 1] * S + plan[l]];
        acc = acc + T[(size_t)l * S + plan[l]];
        used += O[(size_t)l * S + plan[l]];
    }
    *cost = acc;
    *mem = used;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------
 * Batch wrapper: every instance solved in turn, then the minimum over instances
 * (lowest instance index on ties; -1 when every instance is infeasible).
 *   T, O [B][L][S]; R [K][S][S]; r_index [B][L]; budget [B]
 *   best_cost [B], best_s [B], final_row [B][S] or NULL, plan [B][L] or NULL,
 *   mem_used [B] or NULL, best_instance [1]
 * ---------------------------------------------------------------------------------------- */
int oracle_solve_batch(int32_t B, int32_t L, int32_t S, int32_t K,
                       const float *T, const int32_t *O, const float *R,
                       const int32_t *r_index, const int32_t *budget,
                       float *best_cost, int32_t *best_s, float *final_row,
                       int32_t *plan, int32_t *mem_used, int32_t *best_instance)
{
    if (B < 1 || !budget || !best_instance) return ORACLE_BAD_ARG;
    float gbest = INFINITY;
    int32_t garg = -1;
    for (int32_t b = 0; b < B; ++b) {
        const size_t off = (size_t)b * L * S;
        int rc = oracle_solve(L, S, budget[b], K, T + off, O + off, R, r_index + (size_t)b * L,
                              best_cost + b, best_s + b,
                              final_row ? final_row + (size_t)b * S : NULL,
                              plan ? plan + (size_t)b * L : NULL,
                              mem_used ? mem_used + b : NULL, NULL, NULL, NULL);
        if (rc != ORACLE_OK) return rc;
        if (best_cost[b] < gbest) { gbest = best_cost[b]; garg = b; }
    }
    *best_instance = garg;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------
 * Strategy enumeration (paper section 2: the configuration space is modelled as a
 * decision tree and infeasible configurations are discarded).
 *
 * Tree levels, in order: sequence degree sp, tensor degree tp, (data degree dp is
 * what is left of the devices), sharded-data flag sdp, recomputation flag ckpt.
 * A branch is discarded when the degrees do not multiply to N, when a cap is
 * exceeded, or when sdp is asked for with dp == 1 (nothing to shard over).
 * Leaves are emitted in tree order: ascending (sp, tp, sdp, ckpt), ckpt fastest.
 * Each descriptor is 5 int32: tp, sp, dp, sdp, ckpt.
 * Returns the number of leaves; writes at most cap of them when desc != NULL.
 * ---------------------------------------------------------------------------------------- */
int32_t oracle_enumerate(int32_t N, int32_t tp_max, int32_t sp_max, int32_t tpsp_max,
                         int32_t *desc, int32_t cap)
{
    if (N < 1 || (N & (N - 1)) != 0) return ORACLE_BAD_ARG;
    int32_t n = 0;
    for (int32_t sp = 1; sp <= N; sp *= 2) {
        if (sp_max > 0 && sp > sp_max) continue;
        for (int32_t tp = 1; tp * sp <= N; tp *= 2) {
            if (tp_max > 0 && tp > tp_max) continue;
            if (tpsp_max > 0 && tp * sp > tpsp_max) continue;
            const int32_t dp = N / (tp * sp);
            for (int32_t sdp = 0; sdp <= 1; ++sdp) {
                if (sdp == 1 && dp == 1) continue;
                for (int32_t ckpt = 0; ckpt <= 1; ++ckpt) {
                    if (desc && n < cap) {
                        int32_t *d = desc + (size_t)n * 5;
                        d[0] = tp; d[1] = sp; d[2] = dp; d[3] = sdp; d[4] = ckpt;
                    }
                    ++n;
                }
            }
        }
    }
    return n;
}

/* ------------------------------------------------------------------------------------------
 * Cost tables from an alpha-beta model (this build's reading; see the file header).
 * All arithmetic is fp64, one operation at a time in the order written, no fused
 * multiply-add; each table entry is rounded once at the end.
 *
 * layer[b][l] = { hidden h, sequence length q, tokens per step n, time_scale,
 *                 state_scale, act_scale }                      (6 doubles)
 * hw          = { flops_per_s, bytes_per_s, bin_bytes, ckpt_keep } (4 doubles)
 * rmodel[k]   = { hidden h, tokens n }                           (2 doubles)
 *
 * With t = n / (dp*sp) tokens per replica and P = 12 h^2 parameters:
 *   flops = 3 (24 t h^2 + 4 t q h), times 4/3 when ckpt
 *   comm  = [tp>1] 16 t h (tp-1)/tp  +  [dp>1] 4 (P/tp) (dp-1)/dp (x1.5 if sdp)
 *           +  [sp>1] 8 t h (sp-1)/sp                                  bytes
 *   T     = fp32( time_scale * 1000 * ( flops/(tp*flops_per_s) + comm/bytes_per_s ) )
 *   mem   = state_scale * 16 P / (tp * (sdp ? dp : 1))
 *           + act_scale * (68 t h / tp) * (ckpt ? ckpt_keep : 1)       bytes
 *   O     = min( max(1, ceil(mem / bin_bytes)), M + 1 )
 *   R[k][si][sj] = 0 when (tp, sp, dp) agree, else
 *           fp32( 1000 * 2 h (n/(dp_j sp_j)) (1 - w * lo/hi) / bytes_per_s ),
 *           lo/hi = min/max of dp_i sp_i and dp_j sp_j, w = 1 if tp_i == tp_j else 0.5
 * ---------------------------------------------------------------------------------------- */
int oracle_build_tables(int32_t B, int32_t L, int32_t S, int32_t M, int32_t K,
                        const int32_t *desc, const double *layer, const double *hw,
                        const double *rmodel, float *T, int32_t *O, float *R)
{
    if (B < 1 || L < 1 || S < 1 || M < 1 || K < 1 || !desc || !layer || !hw || !rmodel ||
        !T || !O || !R)
        return ORACLE_BAD_ARG;
    const double F = hw[0], BW = hw[1], bin = hw[2], keep = hw[3];
    for (int32_t b = 0; b < B; ++b)
        for (int32_t l = 0; l < L; ++l) {
            const double *p = layer + ((size_t)b * L + l) * 6;
            const double h = p[0], q = p[1], n = p[2];
            const double tscale = p[3], sscale = p[4], ascale = p[5];
            for (int32_t s = 0; s < S; ++s) {
                const int32_t *d = desc + (size_t)s * 5;
                const double tp = d[0], sp = d[1], dp = d[2];
                const int sdp = d[3], ckpt = d[4];
                const double t = n / (dp * sp);
                const double hh = h * h;
                const double P = 12.0 * hh;
                double flops = 24.0 * t;
                flops = flops * hh;
                double attn = 4.0 * t;
                attn = attn * q;
                attn = attn * h;
                flops = flops + attn;
                flops = 3.0 * flops;
                if (ckpt) { flops = flops * 4.0; flops = flops / 3.0; }
                double comm = 0.0;
                if (d[0] > 1) {
                    double x = 16.0 * t;
                    x = x * h;
                    x = x * (tp - 1.0);
                    x = x / tp;
                    comm = comm + x;
                }
                if (d[2] > 1) {
                    double x = P / tp;
                    x = 4.0 * x;
                    x = x * (dp - 1.0);
                    x = x / dp;
                    if (sdp) x = x * 1.5;
                    comm = comm + x;
                }
                if (d[1] > 1) {
                    double x = 8.0 * t;
                    x = x * h;
                    x = x * (sp - 1.0);
                    x = x / sp;
                    comm = comm + x;
                }
                double sec = flops / (tp * F);
                sec = sec + comm / BW;
                double ms = tscale * 1000.0;
                ms = ms * sec;
                T[((size_t)b * L + l) * S + s] = (float)ms;

                const double shard = sdp ? dp : 1.0;
                double state = 16.0 * P;
                state = state / (tp * shard);
                state = sscale * state;
                double act = 68.0 * t;
                act = act * h;
                act = act / tp;
                if (ckpt) act = act * keep;
                act = ascale * act;
                const double bins = ceil((state + act) / bin);
                int32_t o;
                if (!(bins >= 1.0)) o = 1;
                else if (bins > (double)M + 1.0) o = M + 1;
                else o = (int32_t)bins;
                O[((size_t)b * L + l) * S + s] = o;
            }
        }
    for (int32_t k = 0; k < K; ++k) {
        const double h = rmodel[(size_t)k * 2], n = rmodel[(size_t)k * 2 + 1];
        for (int32_t i = 0; i < S; ++i)
            for (int32_t j = 0; j < S; ++j) {
                const int32_t *a = desc + (size_t)i * 5, *c = desc + (size_t)j * 5;
                float r = 0.0f;
                if (!(a[0] == c[0] && a[1] == c[1] && a[2] == c[2])) {
                    const double gi = (double)a[2] * (double)a[1];
                    const double gj = (double)c[2] * (double)c[1];
                    const double lo = gi < gj ? gi : gj, hi = gi < gj ? gj : gi;
                    const double w = (a[0] == c[0]) ? 1.0 : 0.5;
                    double x = 2.0 * h;
                    x = x * (n / gj);
                    double keepfrac = w * lo;
                    keepfrac = keepfrac / hi;
                    x = x * (1.0 - keepfrac);
                    x = x / BW;
                    x = 1000.0 * x;
                    r = (float)x;
                }
                R[((size_t)k * S + i) * S + j] = r;
            }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------
 * Profile-driven cost tables (paper section 2, "Profiler" and "Search Engine": measured
 * per-layer compute time and memory and measured inter-device bandwidth at different
 * group sizes feed the cost models; section 3 step 3).  The paper prints no formula; this
 * reading is this build's own ("parity unpinned" against the paper).  fp64, one rounding
 * per operation in the order written, one final rounding.
 *
 *   layer_type [B][L]      index into profile
 *   profile    [Y][3]      { fwd_ms_per_1000_tokens at tp = 1, param_bytes, act_bytes_per_token }
 *   bw         [NB]        measured collective bandwidth in bytes/s for a group of 2^g devices
 *                          (entry g; entry 0 unused)
 *   par        [5]         { tokens, overlap in [0,1], bin_bytes, ckpt_keep, state_factor }
 * With t = tokens / (dp * sp):
 *   comp    = 3 * fwd_ms * (t / 1000) / tp, times 4/3 under recomputation
 *   tp_comm = [tp>1] 1000 * (4 * act * t * (tp-1)/tp) / bw[log2 tp]
 *   dp_comm = [dp>1] 1000 * (2 * (param/tp) * (dp-1)/dp * (sdp ? 1.5 : 1)) / bw[log2 dp]
 *   sp_comm = [sp>1] 1000 * (2 * act * t * (sp-1)/sp) / bw[log2 sp]
 *   T = fp32( ((comp + tp_comm) + (1 - overlap) * dp_comm) + sp_comm )
 *   mem = state_factor * param / (tp * (sdp ? dp : 1)) + (act * t / tp) * (ckpt ? ckpt_keep : 1)
 *   O = min(max(1, ceil(mem / bin_bytes)), M + 1)
 * ---------------------------------------------------------------------------------------- */
static int ilog2_i32(int32_t v) { int g = 0; while ((1 << g) < v) ++g; return g; }

int oracle_build_tables_profiled(int32_t B, int32_t L, int32_t S, int32_t M, int32_t Y,
                                 int32_t NB, const int32_t *desc, const int32_t *layer_type,
                                 const double *profile, const double *bw, const double *par,
                                 float *T, int32_t *O)
{
    if (B < 1 || L < 1 || S < 1 || M < 1 || Y < 1 || NB < 1 || !desc || !layer_type ||
        !profile || !bw || !par || !T || !O)
        return ORACLE_BAD_ARG;
    const double tokens = par[0], overlap = par[1], bin = par[2], keep = par[3], sf = par[4];
    for (int64_t x = 0; x < (int64_t)B * L; ++x) {
        const int32_t y = layer_type[x];
        if (y < 0 || y >= Y) return ORACLE_BAD_ARG;
        const double fwd = profile[(size_t)y * 3], param = profile[(size_t)y * 3 + 1];
        const double act = profile[(size_t)y * 3 + 2];
        for (int32_t s = 0; s < S; ++s) {
            const int32_t *d = desc + (size_t)s * 5;
            const double tp = d[0], sp = d[1], dp = d[2];
            const int gt = ilog2_i32(d[0]), gs = ilog2_i32(d[1]), gd = ilog2_i32(d[2]);
            if (gt >= NB || gs >= NB || gd >= NB) return ORACLE_BAD_ARG;
            const double t = tokens / (dp * sp);
            double comp = t / 1000.0;
            comp = fwd * comp;
            comp = 3.0 * comp;
            comp = comp / tp;
            if (d[4]) { comp = comp * 4.0; comp = comp / 3.0; }
            double tpc = 0.0, dpc = 0.0, spc = 0.0;
            if (d[0] > 1) {
                double v = 4.0 * act;
                v = v * t;
                v = v * (tp - 1.0);
                v = v / tp;
                v = 1000.0 * v;
                tpc = v / bw[gt];
            }
            if (d[2] > 1) {
                double v = param / tp;
                v = 2.0 * v;
                v = v * (dp - 1.0);
                v = v / dp;
                if (d[3]) v = v * 1.5;
                v = 1000.0 * v;
                dpc = v / bw[gd];
            }
            if (d[1] > 1) {
                double v = 2.0 * act;
                v = v * t;
                v = v * (sp - 1.0);
                v = v / sp;
                v = 1000.0 * v;
                spc = v / bw[gs];
            }
            double ms = comp + tpc;
            ms = ms + (1.0 - overlap) * dpc;
            ms = ms + spc;
            T[(size_t)x * S + s] = (float)ms;

            const double shard = d[3] ? dp : 1.0;
            double state = sf * param;
            state = state / (tp * shard);
            double a = act * t;
            a = a / tp;
            if (d[4]) a = a * keep;
            const double bins = ceil((state + a) / bin);
            int32_t o;
            if (!(bins >= 1.0)) o = 1;
            else if (bins > (double)M + 1.0) o = M + 1;
            else o = (int32_t)bins;
            O[(size_t)x * S + s] = o;
        }
    }
    return ORACLE_OK;
}
