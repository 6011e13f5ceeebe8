/*
 * gsearch — batched per-layer parallel-strategy search on one MI355X (gfx950).
 *
 * The library solves, for a batch of independent instances, the problem the Galvatron
 * search engine solves for every candidate (pipeline degree, stage split, micro-batch
 * count): choose one hybrid-parallel strategy per Transformer layer so that the summed
 * layer time plus strategy-switch time is smallest while the summed layer memory stays
 * within the device budget (paper section 2, "Search Engine"; section 1, feature 2).
 *
 * One instance:  L layers, S strategies, budget of E bins (E <= M), tables
 *   T[l][s]        time of layer l under strategy s         fp32, finite, >= +0
 *   O[l][s]        memory of layer l under s, in bins       int32, >= 0 (> M: never fits)
 *   R[k][si][sj]   cost of going from si (layer l-1) to sj (layer l), fp32 >= +0,
 *                  +inf = forbidden; layer l uses matrix k = r_index[l]
 * State C[l][e][s] = cheapest fp32 chain cost of layers 0..l that ends in strategy s and
 * uses AT MOST e bins:
 *   C[0][e][s]  = T[0][s] if e >= O[0][s] else +inf
 *   C[l][e][sj] = ( min_si ( C[l-1][e-O[l][sj]][si] + R[k][si][sj] ) ) + T[l][sj]
 *                 if e >= O[l][sj] else +inf            (two fp32 adds, in that order)
 *   bp[l][e][sj] = lowest si attaining the min (0 if all candidates are +inf)
 * Result per instance: min_s C[L-1][E][s] (lowest s on ties), the plan obtained by
 * walking bp back from there, and over the batch the instance with the smallest cost
 * (lowest instance index on ties).  An instance that fits no plan is a RESULT
 * (cost +inf, indices -1), not an error.
 *
 * Conventions
 *   - Every function returns GSEARCH_OK (0) or a negative gsearch_status code.  Nothing
 *     throws or aborts across this boundary.
 *   - Pointers named "device" are HIP device pointers owned by the caller (for example
 *     torch tensors); pointers named "host" are ordinary host pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Kernels
 *     are enqueued on it and the call returns without waiting; outputs are valid once
 *     the caller has synchronised that stream.
 *   - A context is not thread-safe, and two solves on one context overlap in its
 *     workspace: serialise them on one stream.
 *   - Table contents live on the device, so they are checked there: a NaN, negative,
 *     -0 or (for T) infinite entry, a negative O, a budget outside [0, M] or an r_index
 *     outside [0, K) sets bits in the data-status word; the solve then still runs on
 *     sanitised copies (memory-safe), reports every instance as infeasible, and
 *     gsearch_data_status returns the bits.
 */
#ifndef GSEARCH_H
#define GSEARCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GSEARCH_OK = 0,
  GSEARCH_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, bad flag            */
  GSEARCH_ERR_CAPACITY = -2,    /* shape exceeds what the context was created for       */
  GSEARCH_ERR_NO_DEVICE = -3,   /* no usable GPU / bad device index                     */
  GSEARCH_ERR_HIP = -4,         /* a HIP runtime call failed                            */
  GSEARCH_ERR_NOT_SOLVED = -5,  /* backtrace / export asked before any solve            */
  GSEARCH_ERR_NO_MEMORY = -6,   /* workspace allocation failed                          */
  GSEARCH_ERR_UNSUPPORTED = -7  /* option needs a flag the context was not created with */
} gsearch_status;

/* gsearch_config.flags */
#define GSEARCH_FLAG_KEEP_PLANES 0x1u    /* keep every C plane (needed by export / curve of
                                            any layer); default keeps two plane slots that
                                            take turns (four where the class kernel's
                                            several-fronts form can run).
                                            (With r_class the planes are kept in a compact
                                            form, one row per class, from which C is rebuilt
                                            wherever it is read.)                          */
#define GSEARCH_FLAG_FORCE_GENERIC 0x2u  /* always use the shape-agnostic forward kernel    */
#define GSEARCH_FLAG_NO_BACKPOINTERS 0x4u /* min-only forward pass: no bp stream is written,
                                            every C plane is kept instead and the backtrace
                                            re-derives each argmin from the planes (same
                                            plans, bit for bit)                             */

#define GSEARCH_FLAG_FORCE_PUSH 0x8u      /* testing/tuning: always the register-tiled push
                                            kernel (flat four-instruction argmin)          */
#define GSEARCH_FLAG_FORCE_TILE 0x10u     /* testing/tuning: always the LDS-staged kernel
                                            with the two-level argmin                      */
#define GSEARCH_FLAG_NO_BIN_UNIT 0x20u    /* testing: do not rescale an instance whose memories
                                            share a divisor.  By default an instance is solved
                                            in its own bin unit g = gcd of the O[l][s] that fit
                                            its budget at all (rows e .. e + g - 1 of a plane
                                            are equal, so only one is computed): same costs
                                            and plans bit for bit, mem_used, budget curve and
                                            export still in the caller's bins               */

/* bits of the data-status word */
#define GSEARCH_DATA_BAD_T 0x1
#define GSEARCH_DATA_BAD_R 0x2
#define GSEARCH_DATA_BAD_O 0x4
#define GSEARCH_DATA_BAD_BUDGET 0x8
#define GSEARCH_DATA_BAD_RINDEX 0x10
#define GSEARCH_DATA_BAD_RCLASS 0x20 /* r_class is not a valid partition, has more classes
                                        than announced (r_class_bound) or than
                                        GSEARCH_MAX_CLASSES, or R differs inside one */

#define GSEARCH_DATA_INTERNAL 0x40   /* not about the data: a bounded wait inside the class
                                        kernel's several-fronts-per-launch form gave up, or a
                                        tile found rows written on another XCD; the forward
                                        pass is incomplete (every instance is reported as
                                        infeasible) */

#define GSEARCH_MAX_CLASSES 64 /* transition classes a solve can exploit (see r_class) */
#define GSEARCH_DEFAULT_CLASSES 32 /* ... unless r_class_bound announces more (a bound of 16 or
                                      less selects a leaner form of the same kernel) */

#define GSEARCH_MAX_S 1024 /* strategies per layer (bp is uint8 up to 256, uint16 above) */

typedef struct gsearch_ctx gsearch_ctx; /* opaque, owned by the library */

/* Capacity of a context.  The workspace (C planes, backpointer streams, sanitised
 * tables) is allocated once at create time for these maxima; see
 * gsearch_workspace_bytes. */
typedef struct {
  int32_t device; /* HIP device index                          */
  int32_t max_B;  /* instances per solve                       */
  int32_t max_L;  /* layers                                    */
  int32_t max_S;  /* strategies, <= GSEARCH_MAX_S              */
  int32_t max_M;  /* memory bins (budgets are 0..M)            */
  int32_t max_K;  /* transition matrices in the pool           */
  uint32_t flags; /* GSEARCH_FLAG_*                            */
} gsearch_config;

/* One batch.  All pointers are DEVICE pointers, row-major, densely packed. */
typedef struct {
  int32_t B, L, S, M, K;  /* uniform shape of the batch                            */
  const float *T;         /* [B][L][S]                                             */
  const int32_t *O;       /* [B][L][S]                                             */
  const float *R;         /* [K][S][S]   R[k][si][sj], row = previous layer        */
  const int32_t *r_index; /* [B][L]      matrix used INTO layer l; entry l=0 unused */
  const int32_t *budget;  /* [B]         E_b, 0 <= E_b <= M                        */
  const int32_t *r_class; /* [S] or NULL.  Optional promise about R that lets the solve do
                             less work for bit-identical results: strategies are grouped
                             into contiguous classes (r_class[0] = 0, each entry equal to
                             its predecessor or one more, at most GSEARCH_MAX_CLASSES
                             classes, see r_class_bound), and R depends on the strategies only through their
                             classes, i.e. rows si, si' of one class are equal in every
                             matrix of the pool and so are columns sj, sj' of one class.
                             That is the case when the transition cost is a resharding
                             cost between parallel layouts and several strategies share a
                             layout (they differ in recomputation or parameter sharding
                             only); gsearch_layout_classes derives it from descriptors.
                             The promise is checked on the device: a violation sets
                             GSEARCH_DATA_BAD_RCLASS and the solve reports every instance
                             as infeasible.  NULL: no assumption.                        */
  int32_t r_class_bound;  /* HOST value: upper bound on the number of classes in r_class
                             (gsearch_layout_classes reports the count).  0 or anything up
                             to GSEARCH_DEFAULT_CLASSES: at most 32 classes, the narrow
                             and faster form of the class kernel; up to GSEARCH_MAX_CLASSES:
                             the wide form.  More classes than announced (or than 64) are
                             flagged like any other broken promise.  Ignored without
                             r_class.                                                    */
} gsearch_problem;

/* Caller-allocated DEVICE outputs of a solve; any pointer may be NULL to skip it. */
typedef struct {
  float *best_cost;       /* [B]    min_s C[L-1][E_b][s]; +inf if infeasible        */
  int32_t *best_s;        /* [B]    lowest s attaining it; -1 if infeasible         */
  float *final_row;       /* [B][S] C[L-1][E_b][.]                                  */
  int32_t *best_instance; /* [1]    argmin_b best_cost, lowest b; -1 if none        */
} gsearch_result;

/* Size in bytes of the device workspace gsearch_create would allocate for `cfg`
 * (0 if cfg is NULL or invalid).  Pure host arithmetic; needs no GPU. */
size_t gsearch_workspace_bytes(const gsearch_config *cfg);

/* Create a context on cfg->device and allocate its workspace.
 * Errors: INVALID_ARG (null, sizes < 1, max_S > GSEARCH_MAX_S, unknown flag bits), NO_DEVICE,
 * NO_MEMORY, HIP. */
int gsearch_create(const gsearch_config *cfg, gsearch_ctx **out);

/* Free the workspace and the context.  NULL is accepted.  The caller must have
 * synchronised every stream that still runs work of this context. */
int gsearch_destroy(gsearch_ctx *ctx);

/* Forward dynamic program for the whole batch (recurrence above), per-instance final
 * minimum and the minimum over instances.  Asynchronous on `stream`.
 * Errors: INVALID_ARG (null problem/tables, shape < 1), CAPACITY, HIP. */
int gsearch_solve_batch(gsearch_ctx *ctx, const gsearch_problem *problem,
                        const gsearch_result *result, void *stream);

/* Plans of the most recent solve on this context.
 *   instances  device [n] instance ids, or NULL for instances 0..n-1.  An id outside
 *              [0, B) (for example best_instance == -1) yields plan = -1, mem_used = -1.
 *   plan       device [n][L]: strategy per layer, all -1 for an infeasible instance
 *   mem_used   device [n] or NULL: sum of O along the plan, -1 if infeasible
 * The tables of the solved problem are read from the context's own copies, so the
 * caller may already have released them.  Asynchronous on `stream`.
 * Errors: INVALID_ARG, NOT_SOLVED, HIP. */
int gsearch_backtrace(gsearch_ctx *ctx, const int32_t *instances, int32_t n, int32_t *plan,
                      int32_t *mem_used, void *stream);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  gsearch_solve_batch followed by gsearch_backtrace of
 * every instance, with the workspace in a fixed array inside the library's device image
 * (GSEARCH_NOALLOC_SCRATCH_BYTES per GPU, held until the process ends) instead of a context:
 * no hipMalloc, hipFree, stream or event creation in this call.  Default mode only (with
 * backpointers, no flags); one chain of launches on `stream`.
 *   device       HIP device index whose copy of the array is used (made current for the call)
 *   problem, result   as for gsearch_solve_batch (device pointers, caller-owned)
 *   plan         device [B][L] or NULL: plans of all instances (as gsearch_backtrace, NULL ids)
 *   mem_used     device [B] or NULL
 *   data_status  device [1] or NULL: the data-status word of this solve (GSEARCH_DATA_* bits)
 * A shape fits when gsearch_workspace_bytes of a config with exactly its sizes and flags 0 is
 * at most GSEARCH_NOALLOC_SCRATCH_BYTES; anything larger returns GSEARCH_ERR_CAPACITY and
 * launches nothing.  All calls on one GPU share the one array, which keeps the last call's
 * contents (the call clears what it needs cleared): calls that overlap on a GPU, on any
 * streams, race; order them on one stream or with events.
 * Errors: INVALID_ARG, CAPACITY, NO_DEVICE, HIP. */
#define GSEARCH_NOALLOC_SCRATCH_BYTES 16777216u /* 16 MiB */
int gsearch_solve_batch_noalloc(int32_t device, const gsearch_problem *problem,
                                const gsearch_result *result, int32_t *plan, int32_t *mem_used,
                                int32_t *data_status, void *stream);

/* Waits for `stream`, then copies the data-status word of the most recent solve to
 * *host_bits (0 = tables were valid; else GSEARCH_DATA_* bits).  Errors: NOT_SOLVED, HIP. */
int gsearch_data_status(gsearch_ctx *ctx, void *stream, int32_t *host_bits);

/* Tuning.  The instances of a batch are independent, so a solve may cut the batch into
 * `groups` contiguous groups whose chains of layer-front launches run side by side: the
 * first on the caller's stream, the others on streams the context owns (default priority,
 * created on first use), forked from and joined back into the caller's stream with events,
 * so that work queued on the caller's stream after the solve still sees every result.
 * Results do not depend on the number of groups.  groups = 0 restores the default (chosen
 * from the batch shape); values above 8 or above B are clamped.  Applies to later solves.
 * Errors: INVALID_ARG (null context, negative count). */
int gsearch_set_instance_groups(gsearch_ctx *ctx, int groups);
/* Number of groups the most recent solve ran side by side (1 for the one-launch path of
 * small instances; 0 before any solve or for a null context). */
int gsearch_instance_groups(gsearch_ctx *ctx);

/* Tuning knobs: overrides of the launch heuristics, for sweeps and tests; results never depend
 * on them.  A context takes their initial values from the environment variables
 * GSEARCH_<NAME IN CAPITALS> when it is created (the library reads the environment nowhere
 * else) and keeps them per context.  Names: "kernel" (1 push, 2 tile, 3 wide: general forward
 * kernel), "small" (0/1: one-launch kernel for small instances never / wherever it fits),
 * "jsplit" (waves per tile), "waves_per_block", "row_groups", "streams" (instance groups),
 * "fronts" (class kernel: layer fronts per launch, 2..64; 0 or 1: one launch per front; -1, the
 * default: 64 wherever that form can run, i.e. a batch that is a multiple of 8 or has 64 instances
 * or more, three layers or more, no forced instance groups, a GPU whose eight XCDs take workgroups in turn),
 * "front_tiles" (that form: workgroups per instance and layer front, in eights; 0, the default: as
 * many as the fronts of earlier solves of the context had 64-row tiles with work, one per tile of
 * the budget at first.  Whatever the number, the results are the same: a solve whose fronts need
 * more is redone by a slow launch of k_dp_class_fronts_plain behind the fast ones),
 * "spin_limit" and "hold_flags" (that form, tests of its error path: polls before a wait between
 * dependent tiles gives up, default 2^18; 1 = finished tiles publish no flags, so that every wait
 * gives up, every kernel still ends normally and the solve reports GSEARCH_DATA_INTERNAL).  0 (or -1
 * for "small" and "fronts") restores the heuristic.  gsearch_knob_name lists the names (NULL beyond the last;
 * host only, needs no GPU).  Errors: INVALID_ARG (null context, unknown name, value outside
 * [-1, 64], null output). */
const char *gsearch_knob_name(int index);
/* The value a context created now would start the knob with: its default, or what the
 * environment variable GSEARCH_<NAME IN CAPITALS> says (a decimal integer in [-1, 64]; anything
 * else is ignored).  Host only, needs no GPU.  Errors: INVALID_ARG (unknown name, null output). */
int gsearch_knob_initial(const char *name, int *value);
int gsearch_set_knob(gsearch_ctx *ctx, const char *name, int value);
int gsearch_get_knob(gsearch_ctx *ctx, const char *name, int *value);

/* Measurement aid.  With profiling enabled, every later solve records one HIP event on
 * its stream just before the first forward-DP launch (layer 1) and one just after the
 * last (layer L-1; with instance groups: after the other groups' streams have joined).
 * gsearch_forward_ms waits for the second event of the most recent solve and returns the
 * elapsed milliseconds between the two in *host_ms, i.e. the time of the L-1 layer fronts
 * of every group including the gaps between launches.
 * Errors: NOT_SOLVED (no profiled solve yet, or L == 1), HIP. */
int gsearch_set_profiling(gsearch_ctx *ctx, int enable);
int gsearch_forward_ms(gsearch_ctx *ctx, float *host_ms);
/* Name of the forward kernel the most recent solve launched for its layer fronts
 * ("k_dp_class_fronts", "k_dp_class", "k_dp_tile", "k_dp_wide", "k_dp_push", "k_dp_generic" or
 * "k_dp_small"; "" before any
 * solve; "k_dp_class_fronts" also when its slow stand-in did the work, which only the device
 * knows).  Static string. */
const char *gsearch_forward_kernel(gsearch_ctx *ctx);

/* Test aid for the class kernel's several-fronts form, whose completion flags are stamped
 * with the number of the solve (a counter in the workspace that every solve advances on the
 * device and that wraps at 2^29): sets that counter, on `stream`, so that a test can walk a
 * context across the wrap.  Errors: INVALID_ARG (null context, value >= 2^29), UNSUPPORTED (the
 * context has no such flags: see the knob "fronts"), HIP. */
int gsearch_set_solve_counter(gsearch_ctx *ctx, uint32_t value, void *stream);

/* Measurement aid: LDS traffic of exactly known size, by which the profiler's LDS counters are
 * scaled (as its HBM counters are by a plain copy).  One launch of 1024 x 256 threads, each
 * doing `iters` (1 .. 2^20) operations of one kind on a 16 KB table without bank conflicts:
 * mode 0 four-byte loads, 1 sixteen-byte loads, 2 four-byte stores, 3 float-minimum atomics,
 * i.e. 262144 x iters x (4 | 16 | 4 | 4) bytes.  sink: device [262144] floats (scratch output).
 * Asynchronous on `stream`.  Errors: INVALID_ARG, HIP. */
int gsearch_lds_calibration(int32_t mode, int32_t iters, float *sink, void *stream);

/* Best cost for EVERY budget of the most recent solve (the last plane already holds
 * it): curve[b][e] = min_s C[L-1][e][s] for e <= E_b, +inf for E_b < e <= M.
 * curve is device [B][M+1].  Paper section 1, feature 2 (adapting to hardware
 * constraints): one solve answers every smaller device memory as well. */
int gsearch_budget_curve(gsearch_ctx *ctx, float *curve, void *stream);

/* Pipeline-aware outer reduction over the most recent solve (paper abstract and section 2:
 * pipeline parallelism is one of the searched dimensions; the paper gives no formula, this
 * is the synchronous-pipeline reading).  A candidate g = (pipeline degree, stage split,
 * micro-batch count m) owns the solved instances group_members[group_offsets[g] ..
 * group_offsets[g+1]), one per stage; their optima t are per-micro-batch stage times and
 *     group_cost[g] = (t_0 + t_1 + ...) + (m - 1) * max t          (fp32, in that order)
 * +inf if any member is infeasible or not a valid instance id.  best_group = argmin,
 * lowest g on ties, -1 if none is feasible (NULL to skip).
 *   group_offsets device [G+1], group_members device [n_members], group_micro device [G],
 *   group_cost device [G], best_group device [1].  Asynchronous on `stream`.
 * Errors: INVALID_ARG, NOT_SOLVED, HIP. */
int gsearch_pipeline_reduce(gsearch_ctx *ctx, int32_t G, const int32_t *group_offsets,
                            const int32_t *group_members, int32_t n_members,
                            const int32_t *group_micro, float *group_cost, int32_t *best_group,
                            void *stream);

/* Debug export of the most recent solve in canonical layout (needs KEEP_PLANES):
 *   C  device [B][L][M+1][S] fp32, rows e > E_b are filled with +inf
 *   bp device [B][L][M+1][S] int32, plane 0 and rows e > E_b are 0; NULL to skip (must be
 *      NULL for a NO_BACKPOINTERS context).
 * Errors: UNSUPPORTED without the flag, NOT_SOLVED, INVALID_ARG. */
int gsearch_export_planes(gsearch_ctx *ctx, float *C, int32_t *bp, void *stream);

/* ---- strategy enumeration (paper section 2: decision-tree model of the parallel
 * configuration space with infeasible configurations discarded) -------------------
 * Descriptor = 5 int32 (tp, sp, dp, sdp, ckpt): tensor, sequence and data degree
 * (powers of two with tp*sp*dp == N), sharded-data flag (only when dp > 1) and
 * recomputation flag.  Tree order: ascending (sp, tp, sdp, ckpt), ckpt fastest.
 * Caps: tp <= tp_max, sp <= sp_max, tp*sp <= tpsp_max; a cap <= 0 means "none". */

/* Transition classes of an enumerated strategy set (paper sections 1 and 2: a strategy
 * combines the data / tensor / sequence degrees with sharded data parallelism and with
 * recomputation as dimensions of their own; only the degrees fix how activations are laid
 * out between layers).  r_class[s] (device [S]) counts the
 * changes of the layout (tp, sp, dp) along desc[0..s], so strategies that follow each other
 * with the same layout share a class; count_out (device [1], may be NULL) receives the
 * number of classes.  Feed r_class to gsearch_problem when R was built from the same
 * descriptors by gsearch_build_tables (its R depends on the layouts only).
 * Asynchronous on `stream`.  Errors: INVALID_ARG (null pointers, S outside 1..GSEARCH_MAX_S). */
int gsearch_layout_classes(const int32_t *desc, int32_t S, int32_t *r_class, int32_t *count_out,
                           void *stream);

/* Number of strategies (host arithmetic, no GPU).  Negative status if N is not a power
 * of two in [1, 2^30]. */
int32_t gsearch_enumerate_count(int32_t N, int32_t tp_max, int32_t sp_max, int32_t tpsp_max);

/* Device enumeration: writes min(count, cap) descriptors to desc (device [cap][5]) and
 * the full count to count_out (device [1], may be NULL).  Asynchronous on `stream`. */
int gsearch_enumerate(int32_t N, int32_t tp_max, int32_t sp_max, int32_t tpsp_max,
                      int32_t *desc, int32_t cap, int32_t *count_out, void *stream);

/* ---- cost tables (paper section 2: time and memory cost models per strategy) ------
 * The paper prints no formula; this is an alpha-beta model evaluated in fp64, one
 * rounding per operation, no fused multiply-add, rounded once to the output type.
 *   layer  device [B][L] of gsearch_layer_model
 *   hw     host pointer
 *   rmodel device [K] of gsearch_reshard_model
 * With t = tokens/(dp*sp), P = 12 hidden^2:
 *   flops = 3 (24 t h^2 + 4 t seq h), x 4/3 under recomputation
 *   comm  = [tp>1] 16 t h (tp-1)/tp + [dp>1] 4 (P/tp)(dp-1)/dp (x1.5 if sdp)
 *           + [sp>1] 8 t h (sp-1)/sp
 *   T     = fp32( time_scale * 1000 * (flops/(tp*flops_per_s) + comm/bytes_per_s) )
 *   mem   = state_scale * 16 P/(tp*(sdp?dp:1)) + act_scale * (68 t h/tp) * (ckpt?ckpt_keep:1)
 *   O     = min(max(1, ceil(mem/bin_bytes)), M+1)
 *   R[k][si][sj] = 0 if (tp,sp,dp) agree, else
 *           fp32( 1000 * 2 h (tokens/(dp_j sp_j)) (1 - w lo/hi) / bytes_per_s ),
 *           lo/hi = min/max(dp_i sp_i, dp_j sp_j), w = 1 if tp_i == tp_j else 0.5
 * Outputs T [B][L][S], O [B][L][S], R [K][S][S] are device buffers. */
typedef struct {
  double hidden, seq, tokens, time_scale, state_scale, act_scale;
} gsearch_layer_model;
typedef struct {
  double flops_per_s, bytes_per_s, bin_bytes, ckpt_keep;
} gsearch_hw_model;
typedef struct {
  double hidden, tokens;
} gsearch_reshard_model;

int gsearch_build_tables(int32_t B, int32_t L, int32_t S, int32_t M, int32_t K,
                         const int32_t *desc, const gsearch_layer_model *layer,
                         const gsearch_hw_model *hw, const gsearch_reshard_model *rmodel,
                         float *T, int32_t *O, float *R, void *stream);

/* ---- profile-driven cost tables (paper section 2, "Profiler": measured per-layer compute
 * time and memory and measured inter-device bandwidth at different group sizes are what
 * the cost models are built from; the paper prints no formula, this is this library's
 * reading).  Same conventions as gsearch_build_tables; R is not touched.
 *   layer_type device [B][L]   index into profile
 *   profile    device [Y]      per layer type: forward ms per 1000 tokens at tp = 1,
 *                              parameter bytes, activation bytes per token
 *   bandwidth  device [NB]     measured collective bandwidth (bytes/s) of a group of 2^g
 *                              devices, entry g (entry 0 unused)
 *   par        host
 * With t = tokens/(dp*sp):
 *   comp    = 3 * fwd_ms * (t/1000) / tp, x 4/3 under recomputation
 *   tp_comm = [tp>1] 1000 * (4 act t (tp-1)/tp) / bandwidth[log2 tp]
 *   dp_comm = [dp>1] 1000 * (2 (param/tp) (dp-1)/dp (x1.5 if sdp)) / bandwidth[log2 dp]
 *   sp_comm = [sp>1] 1000 * (2 act t (sp-1)/sp) / bandwidth[log2 sp]
 *   T = fp32( ((comp + tp_comm) + (1 - overlap) * dp_comm) + sp_comm )
 *   mem = state_factor * param / (tp*(sdp?dp:1)) + (act t / tp) * (ckpt ? ckpt_keep : 1)
 *   O = min(max(1, ceil(mem/bin_bytes)), M+1)
 * A layer type outside [0, Y) or a degree beyond the bandwidth table gives T = +inf and
 * O = M+1 (the solve then flags the table as invalid). */
typedef struct {
  double fwd_ms_per_ktoken, param_bytes, act_bytes_per_token;
} gsearch_layer_profile;
typedef struct {
  double tokens, overlap, bin_bytes, ckpt_keep, state_factor;
} gsearch_profile_params;

int gsearch_build_tables_profiled(int32_t B, int32_t L, int32_t S, int32_t M, int32_t Y,
                                  int32_t NB, const int32_t *desc, const int32_t *layer_type,
                                  const gsearch_layer_profile *profile, const double *bandwidth,
                                  const gsearch_profile_params *par, float *T, int32_t *O,
                                  void *stream);

/* Static description of an error code. */
const char *gsearch_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* GSEARCH_H */
