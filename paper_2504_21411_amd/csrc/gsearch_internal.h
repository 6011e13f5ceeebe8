// Internal declarations shared by the HIP translation units of libgsearch (gfx950 only).
// Nothing here is part of the C ABI; see include/gsearch.h for that.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace gs {

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kRowsPerBlock = 256; // budget rows handled by one workgroup (4 waves)
constexpr int kMaxClasses = 64;    // most transition classes a solve can exploit (capacity of the
                                   // class kernel's wide variant; the narrow one holds 32)

// Launch-heuristic overrides of one context (sweeps and tests; 0 or -1 = use the heuristic).
// A context reads them once from the environment when it is created (GSEARCH_<NAME>) and
// gsearch_set_knob changes them afterwards; nothing in the library reads the environment later.
struct Tuning {
  int kernel = 0;          // 1 push, 2 tile, 3 wide: force that general forward kernel
  int small = -1;          // 0 / 1: the one-launch kernel for small instances never / wherever it fits
  int jsplit = 0;          // waves per tile
  int waves_per_block = 0; // push kernel: waves per workgroup (1..4)
  int row_groups = 0;      // push kernel: 64-row groups per wave
  int streams = 0;         // instance groups on parallel streams
  int fronts = -1;         // class kernel: layer fronts per launch, 2..64 (0, 1: one launch per
                           // front; -1: 64 wherever that form can run)
  int front_tiles = 0;     // that form: workgroups per instance and front, in eights (0: what
                           // earlier solves of the context needed, all tiles at first)
  int spin_limit = 0;      // that form: polls before a wait gives up (0: the default, 2^18)
  int hold_flags = 0;      // that form, tests only: 1 = finished tiles publish no flags, so that
                           // every wait runs into its limit (the error path, with no fault)
};

// More than 64 KB of dynamic LDS per workgroup has to be asked for once per kernel (and
// device; a context lives on one device): the largest size already asked for, per kernel.
struct LdsGrants {
  static constexpr int kMax = 48;
  const void *fn[kMax] = {};
  size_t bytes[kMax] = {};
  int n = 0;
};

// Shape of the batch being solved plus the padded pitches of the workspace copies.
struct Shape {
  int B, L, S, M, K;
  int SP;    // pitch of one (b,l) row of Tq/Oq and of both dimensions of Rt
  int pitch; // pitch (in elements) of one strategy row of a C plane / bp plane
  int bp16;  // backpointers are uint16 (S > 256) instead of uint8
  int Bc;    // instances in flight at the same time (>= B when this shape is one group of
             // a batch whose groups run on parallel streams); launch heuristics only
  int NC;    // class capacity of this solve (32, or 64 when the caller announces more than 32
             // classes): row stride of Rc, columns of the per-class backpointers, cap of the
             // compact planes' rows
  Tuning tune;       // the context's launch overrides
  LdsGrants *grants; // the context's record of LDS sizes asked for (never null in a solve)
};

// Device pointers into the context's workspace.
struct Workspace {
  float *planes;     // [nplanes][B][S][pitch]  C planes, budget index contiguous; after a
                     // class-kernel solve every slot holds the compact plane
                     // [B][class_rows][pitch] of its layer at its head instead
  void *bp;          // [L-1][B][S][pitch]       uint8 or uint16 backpointers (may be null);
                     // after a class-kernel solve [L-1][B][NC][pitch] uint8 indexed by
                     // (target class, SOURCE row), see by_class
  const float *zero_row; // [pitch of max_M] zeros, written once when the context is created:
                     // source of the class kernel's first front when Q[0] = 0 is not stored
  int by_class;      // 1: the class kernel ran.  Planes are compact, C[l][e][s] =
                     // Q[l][class s][e - O[l][s]] + T[l][s] with Q[0] = 0, and bp[l][e][sj] =
                     // bpc[l][class sj][e - O[l][sj]] when that row is >= lowsum[l-1], else 0
                     // (every strategy of a class shares the argmin)
  float *Tq;         // [B][L][SP]   sanitised copy of T
  int32_t *Oq;       // [B][L][SP]   sanitised copy of O, clamped to [0, M+1], divided by unit
  float *Rt;         // [K][SP][SP]  transposed copy: Rt[k][sj][si] = R[k][si][sj]
  int32_t *ridx;     // [B][L]       clamped r_index (entry l=0 is 0)
  int32_t *budget;   // [B]          clamped budgets, in the instance's own bin unit
  int32_t *budget0;  // [B]          clamped budgets in the caller's bins
  int32_t *unit;     // [B]          bin unit g of the instance (see k_bin_unit): Oq, minO,
                     //              lowsum, budget and every plane row count multiples of g
  int32_t *minO;     // [B][L]       min_s Oq
  int32_t *topsum;   // [B][L]       sum over layers l..L-1 of minO, clamped to M+1: a source row
                     //              r of front l above E - topsum[l] leads to no result and is
                     //              skipped (the layer's own minO when every row is wanted)
  int32_t *lowsum;   // [B][L]       sum over layers 0..l of minO, clamped to M+1: budget rows
                     //              below it cannot hold any plan of layers 0..l (all +inf)
  int32_t *best_s;   // [B]          result of the final reduction (kept for backtrace)
  float *best_cost;  // [B]
  int32_t *status;   // [1]          data-status bits
  int32_t *status_acc; // [1]        where k_prepare collects its bits; zero between solves
                     //              (k_bin_unit moves them to `status` and clears it again)
  // Transition classes (only meaningful when the caller gave r_class):
  int32_t *cmeta;    // [2]          number of classes, longest class
  int32_t *cstart;   // [NC+1]  first strategy of class c; S for c >= number of classes
  int32_t *cls;      // [SP]         class of strategy s (0 for the padding)
  float *Rc;         // [K][NC][NC]  Rc[k][cj][ci] = R between the classes'
                     //              first strategies, +inf for padding classes
  // Several layer fronts per launch of the class kernel (see k_dp_class_fronts):
  int32_t *maxfit;   // [B][L]       largest O[b][l][s] that fits the budget at all (0: none)
  unsigned *stop;    // one word: a bounded wait gave up somewhere in this solve
  size_t front_flag_words; // words the context has room for
  unsigned *front_flags; // [L][B][tiles] completion flags; a flag set by solve number n holds n.
                     // At a fixed place of the context's allocation, cleared when it is created.
  unsigned *epoch;   // [3] at a fixed place of the allocation: number of the current solve
                     // (1 .. 2^29 - 1, advanced on the device by the prepare step, so that a
                     // replayed graph advances it too), "wrapped, clear the flags", "cleared"
};

inline size_t plane_elems(const Shape &s) { return (size_t)s.B * s.S * s.pitch; }
// Compact planes of the class kernel: one row per transition class instead of per strategy.
inline int class_rows(const Shape &s) { return s.S < s.NC ? s.S : s.NC; }

// ---- launchers (all asynchronous on `st`) -------------------------------------------
// Sanitised tables, data-status bits, bin units and least-memory sums.  With r_class (may be
// null) the same two launches also validate r_class and R against each other (status bit on
// violation) and fill cmeta / cstart / cls / Rc; an invalid partition is replaced by the
// one-class partition, so that the class kernel stays memory-safe.
void launch_prepare(const Shape &s, const float *T, const int32_t *O, const float *R,
                    const int32_t *r_index, const int32_t *budget, const int32_t *r_class,
                    const Workspace &w, bool compress_bins, bool all_rows, hipStream_t st);
bool class_path_applies(const Shape &s);
// One layer front with the class kernel: src and dst are compact planes
// [B][class_rows][pitch] holding Q[l-1] and Q[l], where
// C[l][e][s] = Q[l][class s][e - O[l][s]] + T[l][s] and Q[0] = 0: a plane filled by
// launch_class_zero when the planes are kept, else src = w.zero_row, one row of zeros that
// every class of every instance reads.
const char *launch_dp_class(const Shape &s, const Workspace &w, int l, const float *src,
                            float *dst, void *bp_l, hipStream_t st);
void launch_class_zero(const Shape &s, float *q0, hipStream_t st);
// The forward pass of the class kernel with `fronts` layer fronts per launch, the tiles of a
// launch waiting for each other through flags (batch a multiple of 8, 3 layers or more).
// Unless the planes are kept, Q[l] goes to plane slot l % ring (ring = 2 or 4 slots are there).
// y0: workgroups per instance and front (0: one per tile of the budget); a solve in which a
// front has more tiles with work than that is redone by a slow launch behind the fast ones.
// hint (host memory that the device can write, or null): receives the most tiles with work of
// any front.  resident_wgs: workgroups of 512 threads the GPU surely holds at once.
const char *launch_dp_class_fronts(const Shape &s, const Workspace &w, bool keep, bool with_bp,
                                   size_t plane_elems_all, size_t bp_layer_bytes, int fronts,
                                   int ring, int y0, unsigned *hint, int resident_wgs,
                                   hipStream_t st);
bool fronts_shape_ok(const Shape &s);              // that form can take this shape
// out[i] = id of the XCD that workgroup i of a grid of kXccProbeGrid workgroups ran on
constexpr int kXccProbeGrid = 512;
void launch_xcc_probe(unsigned *out, hipStream_t st);
void launch_layout_classes(const int32_t *desc, int S, int32_t *r_class, int32_t *count_out,
                           hipStream_t st);
void launch_init_layer0(const Shape &s, const Workspace &w, float *plane0, hipStream_t st);
// Forward-kernel choice: Auto picks by shape; the others force one implementation.
enum class ForwardKernel { Auto, Generic, Push, Tile };
// One layer front of the recurrence: plane l-1 -> plane l (+ backpointers of layer l).
// Returns the name of the kernel it launched.
const char *launch_dp_layer(const Shape &s, const Workspace &w, int l, const float *src,
                            float *dst, void *bp_l, ForwardKernel which, hipStream_t st);
// Single-launch forward pass for small instances (includes layer 0); see dp_kernels.hip.
bool small_path_applies(const Shape &s, bool with_bp);
void launch_dp_small(const Shape &s, const Workspace &w, bool keep_all, int last_plane,
                     hipStream_t st);
void launch_final(const Shape &s, const Workspace &w, const float *last_plane,
                  float *best_cost, int32_t *best_s, float *final_row, int32_t *best_instance,
                  hipStream_t st);
void launch_backtrace_bp(const Shape &s, const Workspace &w, const int32_t *instances, int n,
                         int32_t *plan, int32_t *mem_used, hipStream_t st);
void launch_backtrace_planes(const Shape &s, const Workspace &w, const int32_t *instances, int n,
                             int32_t *plan, int32_t *mem_used, hipStream_t st);
void launch_pipeline_reduce(const Shape &s, const Workspace &w, int G, const int32_t *offsets,
                            const int32_t *members, int n_members, const int32_t *micro,
                            float *group_cost, int32_t *best_group, hipStream_t st);
void launch_budget_curve(const Shape &s, const Workspace &w, const float *last_plane,
                         float *curve, hipStream_t st);
void launch_export(const Shape &s, const Workspace &w, float *C, int32_t *bp, hipStream_t st);
// LDS traffic of known size (see k_lds_calibration); sink: 1024 * 256 floats
void launch_lds_calibration(int mode, int iters, float *sink, hipStream_t st);
void launch_enumerate(int N, int tp_max, int sp_max, int tpsp_max, int32_t *desc, int cap,
                      int32_t *count_out, hipStream_t st);
void launch_build_tables_profiled(int B, int L, int S, int M, int Y, int NB, const int32_t *desc,
                                  const int32_t *layer_type, const double *profile,
                                  const double *bw, double tokens, double overlap, double bin,
                                  double keep, double sf, float *T, int32_t *O, hipStream_t st);
void launch_build_tables(int B, int L, int S, int M, int K, const int32_t *desc,
                         const double *layer, double flops_per_s, double bytes_per_s,
                         double bin_bytes, double ckpt_keep, const double *rmodel, float *T,
                         int32_t *O, float *R, hipStream_t st);

// Register-tiled forward kernels exist for these padded strategy counts.
int tuned_sp_for(int S); // smallest supported SP >= S, or 0 if S is too large
int class_sp_for(int S); // the same for the class kernel, which also has 192 and 256

} // namespace gs
