// C ABI of libgsearch (see include/gsearch.h): argument checking, workspace layout and the
// sequence of kernel launches.  No arithmetic of the method happens on the host.
#include "../../include/gsearch.h"

#include <cctype>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>
#include <new>

#include "gsearch_internal.h"

namespace {

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Names of the tuning knobs, in the order gsearch_knob_name lists them, and where each lives.
struct KnobDesc {
  const char *name;
  int gs::Tuning::*field;
};
const KnobDesc kKnobs[] = {
    {"kernel", &gs::Tuning::kernel},   {"small", &gs::Tuning::small},
    {"jsplit", &gs::Tuning::jsplit},   {"waves_per_block", &gs::Tuning::waves_per_block},
    {"row_groups", &gs::Tuning::row_groups}, {"streams", &gs::Tuning::streams},
    {"fronts", &gs::Tuning::fronts},   {"spin_limit", &gs::Tuning::spin_limit},
    {"hold_flags", &gs::Tuning::hold_flags}, {"front_tiles", &gs::Tuning::front_tiles},
};
constexpr int kKnobCount = (int)(sizeof(kKnobs) / sizeof(kKnobs[0]));

int knob_index(const char *name) {
  if (!name) return -1;
  for (int i = 0; i < kKnobCount; ++i)
    if (strcmp(name, kKnobs[i].name) == 0) return i;
  return -1;
}

// Initial knob values of a new context: GSEARCH_<NAME IN CAPITALS> in the environment, read
// here and nowhere else (an unset or non-numeric variable leaves the default).
gs::Tuning tuning_from_env() {
  gs::Tuning t;
  for (int i = 0; i < kKnobCount; ++i) {
    char var[64] = "GSEARCH_";
    size_t n = strlen(var);
    for (const char *c = kKnobs[i].name; *c && n + 1 < sizeof(var); ++c)
      var[n++] = (char)toupper((unsigned char)*c);
    var[n] = 0;
    const char *e = getenv(var);
    if (!e || !*e) continue;
    char *end = nullptr;
    const long v = strtol(e, &end, 10);
    if (end && *end == 0 && v >= -1 && v <= 64) t.*(kKnobs[i].field) = (int)v;
  }
  return t;
}

struct Layout {
  size_t planes, bp, Tq, Oq, Rt, ridx, budget, budget0, unit, minO, lowsum, topsum, best_s, best_cost,
      status, cmeta, cstart, cls, Rc, maxfit, stop, total;
  int nplanes;
};

gs::Shape make_shape(int B, int L, int S, int M, int K) {
  gs::Shape s;
  s.B = B; s.L = L; s.S = S; s.M = M; s.K = K;
  const int tsp = gs::class_sp_for(S);
  s.SP = tsp ? tsp : (int)align_up((size_t)S, 16); // (16: k_dp_wide takes two chunks per request)
  s.pitch = (int)align_up((size_t)M + 1, 64);
  s.bp16 = S > 256;
  s.Bc = B;
  s.NC = 32;
  s.grants = nullptr;
  return s;
}

bool keeps_all_planes(uint32_t flags) {
  return (flags & (GSEARCH_FLAG_KEEP_PLANES | GSEARCH_FLAG_NO_BACKPOINTERS)) != 0;
}

// ring: the several-fronts form of the class kernel may run, which rotates kFrontRing plane
// slots instead of two (the other kernels use the first two).
constexpr int kFrontRing = 4;
Layout make_layout(const gs::Shape &s, uint32_t flags, bool ring) {
  Layout y;
  size_t off = 0;
  auto take = [&off](size_t bytes) {
    const size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  };
  const int slots = ring ? kFrontRing : 2;
  y.nplanes = keeps_all_planes(flags) ? s.L : (s.L < slots ? s.L : slots);
  // The class kernel keeps compact planes (one row per class) at the head of the slots.
  // Behind the last slot, slack of one padded instance row block: the tile kernel reads
  // (and discards) the strategy rows S..SP-1 of an instance without clamping the address.
  y.planes = take(sizeof(float) * (gs::plane_elems(s) * (size_t)y.nplanes +
                                   (size_t)s.SP * s.pitch));
  const bool want_bp = !(flags & GSEARCH_FLAG_NO_BACKPOINTERS) && s.L > 1;
  // (the class kernel stores one column per class, 32 or 64 per instance, instead of S)
  const size_t bp_cols = s.S > gs::kMaxClasses ? s.S : (s.S > 32 ? gs::kMaxClasses : 32);
  y.bp = take(want_bp ? (size_t)s.B * bp_cols * s.pitch * (size_t)(s.L - 1) * (s.bp16 ? 2 : 1) : 0);
  y.Tq = take(sizeof(float) * (size_t)s.B * s.L * s.SP);
  y.Oq = take(sizeof(int32_t) * (size_t)s.B * s.L * s.SP);
  y.Rt = take(sizeof(float) * ((size_t)s.K * s.SP * s.SP + s.SP));
  y.ridx = take(sizeof(int32_t) * (size_t)s.B * s.L);
  y.budget = take(sizeof(int32_t) * (size_t)s.B);
  y.budget0 = take(sizeof(int32_t) * (size_t)s.B);
  y.unit = take(sizeof(int32_t) * (size_t)s.B);
  y.minO = take(sizeof(int32_t) * (size_t)s.B * s.L);
  y.lowsum = take(sizeof(int32_t) * (size_t)s.B * s.L);
  y.topsum = take(sizeof(int32_t) * (size_t)s.B * s.L);
  y.best_s = take(sizeof(int32_t) * (size_t)s.B);
  y.best_cost = take(sizeof(float) * (size_t)s.B);
  y.status = take(sizeof(int32_t));
  y.cmeta = take(sizeof(int32_t) * 2);
  y.cstart = take(sizeof(int32_t) * (gs::kMaxClasses + 1));
  y.cls = take(sizeof(int32_t) * (size_t)s.SP);
  // (more than 32 classes need more than 32 strategies)
  const size_t ncap = s.S > 32 ? gs::kMaxClasses : 32;
  y.Rc = take(sizeof(float) * (size_t)s.K * ncap * ncap);
  // queues of the one-launch form of the class kernel
  y.maxfit = take(sizeof(int32_t) * (size_t)s.B * s.L);
  y.stop = take(sizeof(uint32_t));
  y.total = off;
  return y;
}

// Behind the per-solve layout: one plane row of zeros, cleared when the context is created and
// never written afterwards (it stands for Q[0] = 0 in the class kernel's first front).
// Its last 256 bytes hold the word in which k_prepare collects data-status bits (zero between solves).
size_t zero_row_bytes(int max_M) {
  return align_up(((size_t)max_M + 1 + 63) / 64 * 64 * sizeof(float), 256) + 256;
}

// Before the zero row: the completion flags of the class kernel's several-fronts-per-launch
// form, one word per
// (layer, instance, 64-row tile) of the largest batch, cleared when the context is created
// (a flag holds the number of the solve that set it, so solves need not clear them).  A batch
// shape that would need more than 64 M flags gets none and runs one launch per layer front.
size_t front_flag_bytes(const gsearch_config *c) {
  const size_t n = (size_t)c->max_L * (size_t)c->max_B * (((size_t)c->max_M + 64) / 64);
  // (256 bytes in front of them hold the solve counter, see Workspace::epoch)
  return n > ((size_t)64 << 20) ? 0 : align_up(n * sizeof(uint32_t), 256) + 256;
}

bool config_ok(const gsearch_config *c) {
  return c && c->max_B >= 1 && c->max_L >= 1 && c->max_S >= 1 && c->max_S <= GSEARCH_MAX_S &&
         c->max_M >= 1 && c->max_K >= 1 && c->device >= 0 && c->max_B <= (1 << 20) &&
         c->max_L <= (1 << 16) && c->max_M <= (1 << 24) && c->max_K <= (1 << 16) &&
         (c->flags & ~(GSEARCH_FLAG_KEEP_PLANES | GSEARCH_FLAG_FORCE_GENERIC |
                       GSEARCH_FLAG_NO_BACKPOINTERS | GSEARCH_FLAG_FORCE_PUSH |
                       GSEARCH_FLAG_FORCE_TILE | GSEARCH_FLAG_NO_BIN_UNIT)) == 0;
}

// Makes the context's device current for the duration of a call.
struct DeviceScope {
  int prev = -1;
  bool ok = false;
  explicit DeviceScope(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) return;
    ok = (prev == dev) || hipSetDevice(dev) == hipSuccess;
    if (prev == dev) prev = -1;
  }
  ~DeviceScope() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

} // namespace

struct gsearch_ctx {
  gsearch_config cfg;
  char *base = nullptr;
  size_t bytes = 0;
  bool solved = false;
  gs::Shape shape{};
  gs::Workspace ws{};
  int last_plane = 0; // index of the plane that holds layer L-1
  bool profiling = false;
  bool timed = false; // the most recent solve recorded both events
  hipEvent_t ev_begin = nullptr, ev_end = nullptr;
  const char *forward_kernel = ""; // kernel used by the most recent solve's layer fronts
  // Instances are independent, so the batch is cut into groups whose chains of layer
  // fronts run side by side: group 0 on the caller's stream, the others on these streams
  // (default priority), forked and joined with events.  While one group's launch drains,
  // the workgroups of another fill the compute units, and launch gaps overlap.
  static constexpr int kMaxSide = 7;
  hipStream_t side[kMaxSide] = {};
  hipEvent_t ev_fork = nullptr, ev_join[kMaxSide] = {};
  int n_side = 0;
  int groups = 0; // 0 = choose from the shape
  int groups_used = 0; // by the most recent solve
  // One-launch form of the class kernel: needs the chip's XCDs to be numbered 0..7 (looked at
  // once, when the context is created) and the flag words at the end of the workspace.
  bool fronts_ok = false; // the XCDs take workgroups in turn and the flags have room
  // That form sizes its grid by the most tiles with work that a front of an earlier solve of
  // this context had: the device writes that count here when a solve ends (host memory that
  // it can reach), and the next call reads whatever has arrived, without waiting.  A count
  // that is out of date costs time, never results (see k_dp_class_fronts_plain).
  unsigned *front_hint = nullptr;
  int resident_wgs = 0; // workgroups of 512 threads the GPU surely holds at once
  gs::Tuning tune;      // launch overrides (from the environment at create, gsearch_set_knob)
  gs::LdsGrants grants; // LDS sizes already asked for, per kernel
};

namespace {

// Number of instance groups for a batch (the knob "streams" overrides).  Measured on MI355X
// over S = 24..128 and fronts of 6e7..2.4e9 relaxations: two groups pay as soon as a layer
// front is worth about 3e8 relaxations (8 to 35 % on the large batches:
// a front there is a few rounds of long workgroups, and the second chain fills the tail of
// each round and the gap between launches) and cost 10 to 40 % below 1.5e8 (fronts of a
// few microseconds lose to the fork and join); more than two add little.
int group_count(const gs::Shape &s, int requested, bool class_kernel) {
  const int env = s.tune.streams;
  const double front = (double)s.B * (s.M + 1) * s.S * s.S;
  // (the class kernel's launches are one round of short workgroups; a second chain was
  // measured to add its own launch overhead without filling anything)
  int g = requested >= 1 ? requested : env >= 1 ? env : (front >= 3.0e8 && !class_kernel ? 2 : 1);
  if (g > gsearch_ctx::kMaxSide + 1) g = gsearch_ctx::kMaxSide + 1;
  return g < s.B ? g : s.B;
}

// Side streams and events are made on first use and live as long as the context.
bool ensure_side_streams(gsearch_ctx *ctx, int n) {
  if (!ctx->ev_fork &&
      hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming) != hipSuccess)
    return false;
  while (ctx->n_side < n) {
    const int i = ctx->n_side;
    if (hipStreamCreateWithFlags(&ctx->side[i], hipStreamNonBlocking) != hipSuccess) return false;
    if (hipEventCreateWithFlags(&ctx->ev_join[i], hipEventDisableTiming) != hipSuccess) {
      (void)hipStreamDestroy(ctx->side[i]);
      ctx->side[i] = nullptr;
      return false;
    }
    ctx->n_side = i + 1;
  }
  return true;
}

// View of instances [b0, b0 + nb) of a workspace: the same kernels run on it as a batch
// of nb instances.  Plane and backpointer bases are offset by the caller.
gs::Workspace group_view(const gs::Shape &s, const gs::Workspace &w, int b0) {
  gs::Workspace g = w;
  g.Tq = w.Tq + (size_t)b0 * s.L * s.SP;
  g.Oq = w.Oq + (size_t)b0 * s.L * s.SP;
  g.ridx = w.ridx + (size_t)b0 * s.L;
  g.budget = w.budget + b0;
  g.budget0 = w.budget0 + b0;
  g.unit = w.unit + b0;
  g.minO = w.minO + (size_t)b0 * s.L;
  g.lowsum = w.lowsum + (size_t)b0 * s.L;
  g.topsum = w.topsum + (size_t)b0 * s.L;
  return g;
}

// (a kernel, not hipMemsetAsync: the caller may be capturing the stream into a graph)
__global__ __launch_bounds__(256) void k_clear_words(uint32_t *__restrict__ p, size_t n) {
  for (size_t x = (size_t)blockIdx.x * 256 + threadIdx.x; x < n; x += (size_t)gridDim.x * 256)
    p[x] = 0u;
}

__global__ void k_set_word(uint32_t *__restrict__ p, uint32_t v) {
  if (blockIdx.x == 0 && threadIdx.x == 0) *p = v;
}

// Layer fronts per launch of the class kernel (0: one launch per front).  The several-fronts
// form needs the eight XCDs to take workgroups in turn and a batch that is a multiple of 8.
int fronts_per_launch(const gsearch_ctx *ctx, const gs::Shape &s) {
  if (!ctx->fronts_ok || !gs::fronts_shape_ok(s) || ctx->groups > 1) return 0;
  if (ctx->tune.fronts < 0) return 64;
  return ctx->tune.fronts >= 2 ? ctx->tune.fronts : 0;
}

// The solve behind gsearch_solve_batch and gsearch_solve_batch_noalloc.
int solve_impl(gsearch_ctx *ctx, const gsearch_problem *p, const gsearch_result *r, void *stream) {
  if (!ctx || !p || !r) return GSEARCH_ERR_INVALID_ARG;
  if (p->B < 1 || p->L < 1 || p->S < 1 || p->M < 1 || p->K < 1 || !p->T || !p->O || !p->R ||
      !p->r_index || !p->budget)
    return GSEARCH_ERR_INVALID_ARG;
  const gsearch_config &c = ctx->cfg;
  if (p->B > c.max_B || p->L > c.max_L || p->S > c.max_S || p->M > c.max_M || p->K > c.max_K)
    return GSEARCH_ERR_CAPACITY;
  DeviceScope scope(c.device);
  if (!scope.ok) return GSEARCH_ERR_HIP;
  hipStream_t st = static_cast<hipStream_t>(stream);

  gs::Shape s = make_shape(p->B, p->L, p->S, p->M, p->K);
  s.tune = ctx->tune;
  s.grants = &ctx->grants;
  // class capacity of this solve: the wide form only when the caller announces it, the
  // narrow one (half the LDS and registers for the class minima, so more workgroups per
  // compute unit) when it announces sixteen classes at most
  if (p->r_class && p->r_class_bound > 32 && p->S > 32) s.NC = gs::kMaxClasses;
  else if (p->r_class && p->r_class_bound >= 1 && p->r_class_bound <= 16) s.NC = 16;
  const Layout y = make_layout(s, c.flags, ctx->fronts_ok);
  const size_t zb = zero_row_bytes(c.max_M);
  if (y.total > ctx->bytes - zb - front_flag_bytes(&c)) return GSEARCH_ERR_CAPACITY;
  gs::Workspace w;
  w.by_class = 0;
  char *base = ctx->base;
  w.zero_row = reinterpret_cast<const float *>(base + (ctx->bytes - zb));
  w.status_acc = reinterpret_cast<int32_t *>(base + (ctx->bytes - 256));
  w.planes = reinterpret_cast<float *>(base + y.planes);
  const bool with_bp = !(c.flags & GSEARCH_FLAG_NO_BACKPOINTERS) && s.L > 1;
  w.bp = with_bp ? static_cast<void *>(base + y.bp) : nullptr;
  w.Tq = reinterpret_cast<float *>(base + y.Tq);
  w.Oq = reinterpret_cast<int32_t *>(base + y.Oq);
  w.Rt = reinterpret_cast<float *>(base + y.Rt);
  w.ridx = reinterpret_cast<int32_t *>(base + y.ridx);
  w.budget = reinterpret_cast<int32_t *>(base + y.budget);
  w.budget0 = reinterpret_cast<int32_t *>(base + y.budget0);
  w.unit = reinterpret_cast<int32_t *>(base + y.unit);
  w.minO = reinterpret_cast<int32_t *>(base + y.minO);
  w.lowsum = reinterpret_cast<int32_t *>(base + y.lowsum);
  w.topsum = reinterpret_cast<int32_t *>(base + y.topsum);
  w.best_s = reinterpret_cast<int32_t *>(base + y.best_s);
  w.best_cost = reinterpret_cast<float *>(base + y.best_cost);
  w.status = reinterpret_cast<int32_t *>(base + y.status);
  w.cmeta = reinterpret_cast<int32_t *>(base + y.cmeta);
  w.cstart = reinterpret_cast<int32_t *>(base + y.cstart);
  w.cls = reinterpret_cast<int32_t *>(base + y.cls);
  w.Rc = reinterpret_cast<float *>(base + y.Rc);
  w.maxfit = reinterpret_cast<int32_t *>(base + y.maxfit);
  w.stop = reinterpret_cast<unsigned *>(base + y.stop);
  w.epoch = nullptr;
  w.front_flags = nullptr;
  w.front_flag_words = 0;
  if (ctx->fronts_ok && front_flag_bytes(&c) > 0) {
    char *fb = base + (ctx->bytes - zb - front_flag_bytes(&c));
    w.epoch = reinterpret_cast<unsigned *>(fb);
    w.front_flags = reinterpret_cast<unsigned *>(fb + 256);
    w.front_flag_words = (front_flag_bytes(&c) - 256) / sizeof(uint32_t);
  }
  ctx->solved = false;
  ctx->forward_kernel = ""; // (a solve of one layer launches no forward kernel)
  ctx->shape = s;
  ctx->ws = w;

  const size_t pe = gs::plane_elems(s);
  const bool keep = keeps_all_planes(c.flags);
  size_t bp_layer_bytes = pe * (s.bp16 ? 2 : 1);
  gs::ForwardKernel which = gs::ForwardKernel::Auto;
  if (c.flags & GSEARCH_FLAG_FORCE_GENERIC) which = gs::ForwardKernel::Generic;
  else if (c.flags & GSEARCH_FLAG_FORCE_PUSH) which = gs::ForwardKernel::Push;
  else if (c.flags & GSEARCH_FLAG_FORCE_TILE) which = gs::ForwardKernel::Tile;

  // Transition classes: checked whenever the caller states them, exploited by the class
  // kernel when no particular kernel is forced and the shape has a register-tiled size.
  gs::launch_prepare(s, p->T, p->O, p->R, p->r_index, p->budget,
                     s.L > 1 ? p->r_class : nullptr, w, !(c.flags & GSEARCH_FLAG_NO_BIN_UNIT),
                     // kept planes are exported whole: no skipping of rows that lead nowhere
                     (c.flags & GSEARCH_FLAG_KEEP_PLANES) != 0, st);
  const bool use_classes =
      p->r_class && s.L > 1 && which == gs::ForwardKernel::Auto && gs::class_path_applies(s);
  // The class kernel works on compact planes (one row per class, at the head of each plane
  // slot) and stores one backpointer per (target class, source row).
  w.by_class = use_classes;
  size_t bp_inst_bytes = (size_t)s.S * s.pitch * (s.bp16 ? 2 : 1); // one instance, one layer
  if (use_classes) {
    bp_inst_bytes = (size_t)s.NC * s.pitch;
    bp_layer_bytes = (size_t)s.B * bp_inst_bytes;
  }
  ctx->ws = w;
  int cur = 0;
  ctx->timed = false;
  const bool timing = ctx->profiling && s.L > 1;
  if (which == gs::ForwardKernel::Auto && !use_classes && gs::small_path_applies(s, with_bp)) {
    // latency path: layer 0 and every layer front in one launch, planes in LDS
    cur = keep ? s.L - 1 : ((s.L - 1) & 1);
    if (timing && hipEventRecord(ctx->ev_begin, st) != hipSuccess) return GSEARCH_ERR_HIP;
    gs::launch_dp_small(s, w, keep, cur, st);
    ctx->forward_kernel = "k_dp_small";
    ctx->groups_used = 1;
  } else if (use_classes && fronts_per_launch(ctx, s) > 0) {
    // several layer fronts per launch, the instances bound to XCDs (see k_dp_class_fronts)
    if (keep) gs::launch_class_zero(s, w.planes, st);
    if (timing && hipEventRecord(ctx->ev_begin, st) != hipSuccess) return GSEARCH_ERR_HIP;
    // (a power of two; not used when the planes are kept)
    const int ring = y.nplanes < kFrontRing ? 2 : kFrontRing;
    // workgroups per instance and front: what the fronts of earlier solves needed and a
    // sixteenth more (four at least); all tiles while nothing is known, after a solve that
    // did not fit, and where no row is left out
    int y0 = 0;
    if (ctx->front_hint && !(c.flags & GSEARCH_FLAG_KEEP_PLANES)) {
      const unsigned seen = *static_cast<volatile unsigned *>(ctx->front_hint);
      if (seen >= 1u && seen < (1u << 22))
        y0 = (int)seen + ((int)seen / 16 > 4 ? (int)seen / 16 : 4);
    }
    ctx->forward_kernel = gs::launch_dp_class_fronts(s, w, keep, with_bp, pe, bp_layer_bytes,
                                                     fronts_per_launch(ctx, s), ring, y0,
                                                     ctx->front_hint, ctx->resident_wgs, st);
    ctx->groups_used = 1;
    cur = keep ? s.L - 1 : ((s.L - 1) & (ring - 1));
  } else {
    // Q[0] = 0: stored only when the planes are kept (the readers of kept planes read it);
    // otherwise the first front reads the context's row of zeros for every class
    if (use_classes && keep) gs::launch_class_zero(s, w.planes, st);
    else if (!use_classes) gs::launch_init_layer0(s, w, w.planes, st);
    if (timing && hipEventRecord(ctx->ev_begin, st) != hipSuccess) return GSEARCH_ERR_HIP;
    const int groups = s.L > 1 ? group_count(s, ctx->groups, use_classes) : 1;
    ctx->groups_used = groups;
    if (groups > 1) {
      if (!ensure_side_streams(ctx, groups - 1)) return GSEARCH_ERR_HIP;
      if (hipEventRecord(ctx->ev_fork, st) != hipSuccess) return GSEARCH_ERR_HIP;
    }
    // one instance's share of a plane slot
    const size_t inst_elems = (size_t)(use_classes ? gs::class_rows(s) : s.S) * s.pitch;
    int last = 0;
    bool failed = false;
    bool fed[gsearch_ctx::kMaxSide] = {};    // side stream i may have been given work
    for (int g = groups - 1; g >= 0 && !failed; --g) { // the caller's stream (group 0) is fed last
      const int b0 = (int)((long long)s.B * g / groups);
      const int b1 = (int)((long long)s.B * (g + 1) / groups);
      gs::Shape sg = s;
      sg.B = b1 - b0;
      const gs::Workspace wg = group_view(s, w, b0);
      hipStream_t sst = g == 0 ? st : ctx->side[g - 1];
      if (g > 0) {
        if (hipStreamWaitEvent(sst, ctx->ev_fork, 0) != hipSuccess) {
          failed = true;
          break;
        }
        fed[g - 1] = true;
      }
      int c2 = 0;
      for (int l = 1; l < s.L; ++l) {
        const int nxt = keep ? l : (c2 ^ 1);
        void *bp_l = with_bp ? static_cast<char *>(w.bp) + (size_t)(l - 1) * bp_layer_bytes +
                                   (size_t)b0 * bp_inst_bytes
                             : nullptr;
        const float *src_l = w.planes + (size_t)c2 * pe + (size_t)b0 * inst_elems;
        if (use_classes && !keep && l == 1) src_l = w.zero_row; // Q[0] = 0 is not stored
        float *dst_l = w.planes + (size_t)nxt * pe + (size_t)b0 * inst_elems;
        ctx->forward_kernel = use_classes
                                  ? gs::launch_dp_class(sg, wg, l, src_l, dst_l, bp_l, sst)
                                  : gs::launch_dp_layer(sg, wg, l, src_l, dst_l, bp_l, which, sst);
        c2 = nxt;
      }
      last = c2;
    }
    // Join: the caller's stream waits for every side stream that was given work, also when a
    // call above failed (whatever those streams still run must be over before the caller's
    // next call on this context touches the workspace).  Where even the join cannot be
    // recorded, the call waits for that stream itself.
    for (int i = 0; i < groups - 1; ++i) {
      if (!fed[i]) continue;
      if (hipEventRecord(ctx->ev_join[i], ctx->side[i]) == hipSuccess &&
          hipStreamWaitEvent(st, ctx->ev_join[i], 0) == hipSuccess)
        continue;
      {
        failed = true;
        (void)hipGetLastError();
        (void)hipStreamSynchronize(ctx->side[i]);
      }
    }
    if (failed) {
      (void)hipGetLastError();
      return GSEARCH_ERR_HIP;
    }
    cur = last;
  }
  if (timing) {
    if (hipEventRecord(ctx->ev_end, st) != hipSuccess) return GSEARCH_ERR_HIP;
    ctx->timed = true;
  }
  ctx->last_plane = cur;
  gs::launch_final(s, w, w.planes + (size_t)cur * pe, r->best_cost, r->best_s, r->final_row,
                   r->best_instance, st);
  if (hipGetLastError() != hipSuccess) return GSEARCH_ERR_HIP;
  ctx->solved = true;
  return GSEARCH_OK;
}

// ---- the entry point that allocates nothing ---------------------------------------------
// Workspace of gsearch_solve_batch_noalloc: a fixed array in the library's device image
// instead of a hipMalloc'ed block.  Every GPU holds its own copy at its own address; in host
// code the name only stands for the symbol, so the address is asked for once per device
// (static_scratch_base) and only that pointer is ever handed to kernels or copies.
__device__ __align__(256) unsigned char scratch[GSEARCH_NOALLOC_SCRATCH_BYTES];

struct StaticSlot {
  unsigned char *ptr = nullptr; // device address of `scratch` on this device
  gsearch_ctx ctx;              // context whose workspace is that array (no streams, no events)
};
constexpr int kMaxStaticDevices = 64;
StaticSlot g_static[kMaxStaticDevices];
std::mutex g_static_mutex;

// Device address of this device's copy of `scratch` (the device must be current).
unsigned char *static_scratch_base(int device) {
  std::lock_guard<std::mutex> lock(g_static_mutex);
  StaticSlot &slot = g_static[device];
  if (!slot.ptr) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    slot.ptr = static_cast<unsigned char *>(ptr);
  }
  return slot.ptr;
}

} // namespace

extern "C" {

const char *gsearch_strerror(int status) {
  switch (status) {
    case GSEARCH_OK: return "ok";
    case GSEARCH_ERR_INVALID_ARG: return "invalid argument";
    case GSEARCH_ERR_CAPACITY: return "problem exceeds the capacity of the context (or of the fixed scratch array)";
    case GSEARCH_ERR_NO_DEVICE: return "no usable GPU device";
    case GSEARCH_ERR_HIP: return "HIP runtime error";
    case GSEARCH_ERR_NOT_SOLVED: return "no solve has been issued on this context";
    case GSEARCH_ERR_NO_MEMORY: return "out of device or host memory";
    case GSEARCH_ERR_UNSUPPORTED: return "operation needs a flag the context was not created with";
    default: return "unknown status";
  }
}

size_t gsearch_workspace_bytes(const gsearch_config *cfg) {
  if (!config_ok(cfg)) return 0;
  return make_layout(make_shape(cfg->max_B, cfg->max_L, cfg->max_S, cfg->max_M, cfg->max_K),
                     cfg->flags, front_flag_bytes(cfg) > 0)
             .total +
         front_flag_bytes(cfg) + zero_row_bytes(cfg->max_M);
}

int gsearch_create(const gsearch_config *cfg, gsearch_ctx **out) {
  if (!out) return GSEARCH_ERR_INVALID_ARG;
  *out = nullptr;
  if (!config_ok(cfg)) return GSEARCH_ERR_INVALID_ARG;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1 || cfg->device >= ndev) {
    (void)hipGetLastError();
    return GSEARCH_ERR_NO_DEVICE;
  }
  DeviceScope scope(cfg->device);
  if (!scope.ok) return GSEARCH_ERR_NO_DEVICE;
  gsearch_ctx *ctx = new (std::nothrow) gsearch_ctx;
  if (!ctx) return GSEARCH_ERR_NO_MEMORY;
  ctx->cfg = *cfg;
  ctx->tune = tuning_from_env();
  ctx->bytes = gsearch_workspace_bytes(cfg);
  void *p = nullptr;
  if (hipMalloc(&p, ctx->bytes) != hipSuccess) {
    (void)hipGetLastError();
    delete ctx;
    return GSEARCH_ERR_NO_MEMORY;
  }
  ctx->base = static_cast<char *>(p);
  const size_t zb = zero_row_bytes(cfg->max_M) + front_flag_bytes(cfg);
  // (waited for here: solves may run on streams that do not order themselves after it)
  bool ok = hipMemset(ctx->base + (ctx->bytes - zb), 0, zb) == hipSuccess;
  // Do workgroups whose indices agree mod 8 run on the same XCD?  (The class kernel's
  // several-fronts form keeps an instance in one L2 that way; asked once, on a small grid,
  // written into the head of the workspace, which every workspace has room for.)
  std::vector<unsigned> where(gs::kXccProbeGrid, 0xFFu);
  bool turns = ok && ctx->bytes >= sizeof(unsigned) * gs::kXccProbeGrid;
  if (turns) {
    gs::launch_xcc_probe(reinterpret_cast<unsigned *>(ctx->base), nullptr);
    ok = hipGetLastError() == hipSuccess && hipStreamSynchronize(nullptr) == hipSuccess &&
         hipMemcpy(where.data(), ctx->base, sizeof(unsigned) * gs::kXccProbeGrid,
                   hipMemcpyDeviceToHost) == hipSuccess;
    for (int i = 0; i < gs::kXccProbeGrid; ++i) turns = turns && where[i] == where[i & 7];
  }
  if (!ok) {
    (void)hipGetLastError();
    (void)hipFree(p);
    delete ctx;
    return GSEARCH_ERR_HIP;
  }
  ctx->fronts_ok = turns && front_flag_bytes(cfg) > 0;
  if (ctx->fronts_ok) {
    hipDeviceProp_t prop;
    void *hp = nullptr;
    if (hipGetDeviceProperties(&prop, cfg->device) == hipSuccess)
      ctx->resident_wgs = prop.multiProcessorCount; // (one per compute unit, whatever else runs)
    if (hipHostMalloc(&hp, 64, hipHostMallocMapped) == hipSuccess && hp) {
      ctx->front_hint = static_cast<unsigned *>(hp);
      *ctx->front_hint = 0u;
    } else {
      (void)hipGetLastError(); // (without it the grid keeps one workgroup per tile)
    }
  }
  *out = ctx;
  return GSEARCH_OK;
}

int gsearch_destroy(gsearch_ctx *ctx) {
  if (!ctx) return GSEARCH_OK;
  int rc = GSEARCH_OK;
  {
    DeviceScope scope(ctx->cfg.device);
    if (ctx->ev_begin) (void)hipEventDestroy(ctx->ev_begin);
    if (ctx->ev_end) (void)hipEventDestroy(ctx->ev_end);
    if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
    for (int i = 0; i < ctx->n_side; ++i) {
      (void)hipStreamSynchronize(ctx->side[i]);
      (void)hipEventDestroy(ctx->ev_join[i]);
      (void)hipStreamDestroy(ctx->side[i]);
    }
    if (ctx->base && hipFree(ctx->base) != hipSuccess) rc = GSEARCH_ERR_HIP;
    // (after the free above, which waits for whatever may still write the word)
    if (ctx->front_hint && hipHostFree(ctx->front_hint) != hipSuccess) rc = GSEARCH_ERR_HIP;
  }
  delete ctx;
  return rc;
}

int gsearch_solve_batch(gsearch_ctx *ctx, const gsearch_problem *p, const gsearch_result *r,
                        void *stream) {
  return solve_impl(ctx, p, r, stream);
}

int gsearch_solve_batch_noalloc(int32_t device, const gsearch_problem *p, const gsearch_result *r,
                                int32_t *plan, int32_t *mem_used, int32_t *data_status,
                                void *stream) {
  if (!p || !r || device < 0 || device >= kMaxStaticDevices) return GSEARCH_ERR_INVALID_ARG;
  if (p->B < 1 || p->L < 1 || p->S < 1 || p->M < 1 || p->K < 1) return GSEARCH_ERR_INVALID_ARG;
  gsearch_config cfg;
  cfg.device = device;
  cfg.max_B = p->B; cfg.max_L = p->L; cfg.max_S = p->S; cfg.max_M = p->M; cfg.max_K = p->K;
  cfg.flags = 0;
  if (!config_ok(&cfg)) return GSEARCH_ERR_INVALID_ARG;
  // the workspace a context of exactly this shape would allocate has to fit the fixed array
  if (gsearch_workspace_bytes(&cfg) > (size_t)GSEARCH_NOALLOC_SCRATCH_BYTES)
    return GSEARCH_ERR_CAPACITY;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) {
    (void)hipGetLastError();
    return GSEARCH_ERR_NO_DEVICE;
  }
  DeviceScope scope(device);
  if (!scope.ok) return GSEARCH_ERR_NO_DEVICE;
  unsigned char *base = static_scratch_base(device);
  if (!base) return GSEARCH_ERR_HIP;
  hipStream_t st = static_cast<hipStream_t>(stream);
  gsearch_ctx *ctx = &g_static[device].ctx;
  ctx->cfg = cfg;
  ctx->base = reinterpret_cast<char *>(base);
  ctx->bytes = (size_t)GSEARCH_NOALLOC_SCRATCH_BYTES;
  ctx->profiling = false;
  ctx->groups = 1; // one chain of launches on the caller's stream: no streams or events to create
  ctx->fronts_ok = false; // (that form of the class kernel keeps flags across solves: not on this array)
  // The array keeps whatever the last call left.  What a solve expects to find cleared sits at
  // the end of the workspace: the row of zeros that stands for Q[0] and the word in which the
  // data-status bits are collected.  Its place depends on M, so it is cleared on every call.
  const size_t zb = zero_row_bytes(cfg.max_M);
  // (solve_impl places the zero row at the very end of the workspace)
  hipLaunchKernelGGL(k_clear_words, dim3((unsigned)((zb / 4 + 255) / 256)), dim3(256), 0, st,
                     reinterpret_cast<uint32_t *>(base + (ctx->bytes - zb)), zb / 4);
  const int rc = solve_impl(ctx, p, r, stream);
  if (rc != GSEARCH_OK) return rc;
  if (plan) gs::launch_backtrace_bp(ctx->shape, ctx->ws, nullptr, p->B, plan, mem_used, st);
  if (data_status &&
      hipMemcpyAsync(data_status, ctx->ws.status, sizeof(int32_t), hipMemcpyDeviceToDevice, st) !=
          hipSuccess)
    return GSEARCH_ERR_HIP;
  return hipGetLastError() == hipSuccess ? GSEARCH_OK : GSEARCH_ERR_HIP;
}

int gsearch_backtrace(gsearch_ctx *ctx, const int32_t *instances, int32_t n, int32_t *plan,
                      int32_t *mem_used, void *stream) {
  if (!ctx || !plan || n < 1) return GSEARCH_ERR_INVALID_ARG;
  if (!ctx->solved) return GSEARCH_ERR_NOT_SOLVED;
  if (!instances && n > ctx->shape.B) return GSEARCH_ERR_INVALID_ARG;
  DeviceScope scope(ctx->cfg.device);
  if (!scope.ok) return GSEARCH_ERR_HIP;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (ctx->cfg.flags & GSEARCH_FLAG_NO_BACKPOINTERS)
    gs::launch_backtrace_planes(ctx->shape, ctx->ws, instances, n, plan, mem_used, st);
  else
    gs::launch_backtrace_bp(ctx->shape, ctx->ws, instances, n, plan, mem_used, st);
  return hipGetLastError() == hipSuccess ? GSEARCH_OK : GSEARCH_ERR_HIP;
}

int gsearch_data_status(gsearch_ctx *ctx, void *stream, int32_t *host_bits) {
  if (!ctx || !host_bits) return GSEARCH_ERR_INVALID_ARG;
  if (!ctx->solved) return GSEARCH_ERR_NOT_SOLVED;
  DeviceScope scope(ctx->cfg.device);
  if (!scope.ok) return GSEARCH_ERR_HIP;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hipStreamSynchronize(st) != hipSuccess) return GSEARCH_ERR_HIP;
  if (hipMemcpy(host_bits, ctx->ws.status, sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess)
    return GSEARCH_ERR_HIP;
  return GSEARCH_OK;
}

const char *gsearch_forward_kernel(gsearch_ctx *ctx) {
  return (ctx && ctx->solved) ? ctx->forward_kernel : "";
}

int gsearch_set_instance_groups(gsearch_ctx *ctx, int groups) {
  if (!ctx || groups < 0) return GSEARCH_ERR_INVALID_ARG;
  ctx->groups = groups;
  return GSEARCH_OK;
}

const char *gsearch_knob_name(int index) {
  return (index >= 0 && index < kKnobCount) ? kKnobs[index].name : nullptr;
}

int gsearch_knob_initial(const char *name, int *value) {
  const int i = knob_index(name);
  if (i < 0 || !value) return GSEARCH_ERR_INVALID_ARG;
  const gs::Tuning t = tuning_from_env();
  *value = t.*(kKnobs[i].field);
  return GSEARCH_OK;
}

int gsearch_set_knob(gsearch_ctx *ctx, const char *name, int value) {
  const int i = knob_index(name);
  if (!ctx || i < 0 || value < -1 || value > 64) return GSEARCH_ERR_INVALID_ARG;
  ctx->tune.*(kKnobs[i].field) = value;
  return GSEARCH_OK;
}

int gsearch_get_knob(gsearch_ctx *ctx, const char *name, int *value) {
  const int i = knob_index(name);
  if (!ctx || i < 0 || !value) return GSEARCH_ERR_INVALID_ARG;
  *value = ctx->tune.*(kKnobs[i].field);
  return GSEARCH_OK;
}

int gsearch_instance_groups(gsearch_ctx *ctx) { return (ctx && ctx->solved) ? ctx->groups_used : 0; }

int gsearch_set_profiling(gsearch_ctx *ctx, int enable) {
  if (!ctx) return GSEARCH_ERR_INVALID_ARG;
  DeviceScope scope(ctx->cfg.device);
  if (!scope.ok) return GSEARCH_ERR_HIP;
  if (enable && !ctx->ev_begin) {
    if (hipEventCreate(&ctx->ev_begin) != hipSuccess) return GSEARCH_ERR_HIP;
    if (hipEventCreate(&ctx->ev_end) != hipSuccess) {
      (void)hipEventDestroy(ctx->ev_begin);
      ctx->ev_begin = nullptr;
      return GSEARCH_ERR_HIP;
    }
  }
  ctx->profiling = enable != 0;
  if (!enable) ctx->timed = false;
  return GSEARCH_OK;
}

int gsearch_forward_ms(gsearch_ctx *ctx, float *host_ms) {
  if (!ctx || !host_ms) return GSEARCH_ERR_INVALID_ARG;
  if (!ctx->solved || !ctx->timed) return GSEARCH_ERR_NOT_SOLVED;
  DeviceScope scope(ctx->cfg.device);
  if (!scope.ok) return GSEARCH_ERR_HIP;
  if (hipEventSynchronize(ctx->ev_end) != hipSuccess) return GSEARCH_ERR_HIP;
  if (hipEventElapsedTime(host_ms, ctx->ev_begin, ctx->ev_end) != hipSuccess)
    return GSEARCH_ERR_HIP;
  return GSEARCH_OK;
}

int gsearch_set_solve_counter(gsearch_ctx *ctx, uint32_t value, void *stream) {
  if (!ctx || value >= (1u << 29)) return GSEARCH_ERR_INVALID_ARG;
  const size_t fb = front_flag_bytes(&ctx->cfg);
  if (!ctx->fronts_ok || fb == 0) return GSEARCH_ERR_UNSUPPORTED;
  DeviceScope scope(ctx->cfg.device);
  if (!scope.ok) return GSEARCH_ERR_NO_DEVICE;
  char *at = ctx->base + (ctx->bytes - zero_row_bytes(ctx->cfg.max_M) - fb);
  hipLaunchKernelGGL(k_set_word, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                     reinterpret_cast<uint32_t *>(at), value);
  return hipGetLastError() == hipSuccess ? GSEARCH_OK : GSEARCH_ERR_HIP;
}

int gsearch_lds_calibration(int32_t mode, int32_t iters, float *sink, void *stream) {
  if (mode < 0 || mode > 3 || iters < 1 || iters > (1 << 20) || !sink) return GSEARCH_ERR_INVALID_ARG;
  gs::launch_lds_calibration(mode, iters, sink, static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? GSEARCH_OK : GSEARCH_ERR_HIP;
}

int gsearch_budget_curve(gsearch_ctx *ctx, float *curve, void *stream) {
  if (!ctx || !curve) return GSEARCH_ERR_INVALID_ARG;
  if (!ctx->solved) return GSEARCH_ERR_NOT_SOLVED;
  DeviceScope scope(ctx->cfg.device);
  if (!scope.ok) return GSEARCH_ERR_HIP;
  const float *last = ctx->ws.planes + (size_t)ctx->last_plane * gs::plane_elems(ctx->shape);
  gs::launch_budget_curve(ctx->shape, ctx->ws, last, curve, static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? GSEARCH_OK : GSEARCH_ERR_HIP;
}

int gsearch_pipeline_reduce(gsearch_ctx *ctx, int32_t G, const int32_t *group_offsets,
                            const int32_t *group_members, int32_t n_members,
                            const int32_t *group_micro, float *group_cost, int32_t *best_group,
                            void *stream) {
  if (!ctx || G < 1 || n_members < 1 || !group_offsets || !group_members || !group_micro ||
      !group_cost)
    return GSEARCH_ERR_INVALID_ARG;
  if (!ctx->solved) return GSEARCH_ERR_NOT_SOLVED;
  DeviceScope scope(ctx->cfg.device);
  if (!scope.ok) return GSEARCH_ERR_HIP;
  gs::launch_pipeline_reduce(ctx->shape, ctx->ws, G, group_offsets, group_members, n_members,
                             group_micro, group_cost, best_group,
                             static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? GSEARCH_OK : GSEARCH_ERR_HIP;
}

int gsearch_export_planes(gsearch_ctx *ctx, float *C, int32_t *bp, void *stream) {
  if (!ctx || (!C && !bp)) return GSEARCH_ERR_INVALID_ARG;
  if (!(ctx->cfg.flags & GSEARCH_FLAG_KEEP_PLANES)) return GSEARCH_ERR_UNSUPPORTED;
  if (bp && (ctx->cfg.flags & GSEARCH_FLAG_NO_BACKPOINTERS)) return GSEARCH_ERR_INVALID_ARG;
  if (!ctx->solved) return GSEARCH_ERR_NOT_SOLVED;
  DeviceScope scope(ctx->cfg.device);
  if (!scope.ok) return GSEARCH_ERR_HIP;
  gs::launch_export(ctx->shape, ctx->ws, C, bp, static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? GSEARCH_OK : GSEARCH_ERR_HIP;
}

int32_t gsearch_enumerate_count(int32_t N, int32_t tp_max, int32_t sp_max, int32_t tpsp_max) {
  if (N < 1 || N > (1 << 30) || (N & (N - 1)) != 0) return GSEARCH_ERR_INVALID_ARG;
  int32_t n = 0;
  for (int64_t sp = 1; sp <= N; sp *= 2)
    for (int64_t tp = 1; tp * sp <= N; tp *= 2) {
      if ((sp_max > 0 && sp > sp_max) || (tp_max > 0 && tp > tp_max) ||
          (tpsp_max > 0 && tp * sp > tpsp_max))
        continue;
      n += (N / (tp * sp) > 1) ? 4 : 2; // sdp needs dp > 1; ckpt doubles both
    }
  return n;
}

int gsearch_layout_classes(const int32_t *desc, int32_t S, int32_t *r_class, int32_t *count_out,
                           void *stream) {
  if (!desc || !r_class || S < 1 || S > GSEARCH_MAX_S) return GSEARCH_ERR_INVALID_ARG;
  gs::launch_layout_classes(desc, S, r_class, count_out, static_cast<hipStream_t>(stream));
  if (hipGetLastError() != hipSuccess) return GSEARCH_ERR_HIP;
  return GSEARCH_OK;
}

int gsearch_enumerate(int32_t N, int32_t tp_max, int32_t sp_max, int32_t tpsp_max, int32_t *desc,
                      int32_t cap, int32_t *count_out, void *stream) {
  if (N < 1 || N > (1 << 30) || (N & (N - 1)) != 0 || cap < 0 || (cap > 0 && !desc))
    return GSEARCH_ERR_INVALID_ARG;
  gs::launch_enumerate(N, tp_max, sp_max, tpsp_max, desc, cap, count_out,
                       static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? GSEARCH_OK : GSEARCH_ERR_HIP;
}

int gsearch_build_tables(int32_t B, int32_t L, int32_t S, int32_t M, int32_t K,
                         const int32_t *desc, const gsearch_layer_model *layer,
                         const gsearch_hw_model *hw, const gsearch_reshard_model *rmodel, float *T,
                         int32_t *O, float *R, void *stream) {
  if (B < 1 || L < 1 || S < 1 || M < 1 || K < 1 || !desc || !layer || !hw || !rmodel || !T ||
      !O || !R)
    return GSEARCH_ERR_INVALID_ARG;
  if (!(hw->flops_per_s > 0.0) || !(hw->bytes_per_s > 0.0) || !(hw->bin_bytes > 0.0))
    return GSEARCH_ERR_INVALID_ARG;
  gs::launch_build_tables(B, L, S, M, K, desc, reinterpret_cast<const double *>(layer),
                          hw->flops_per_s, hw->bytes_per_s, hw->bin_bytes, hw->ckpt_keep,
                          reinterpret_cast<const double *>(rmodel), T, O, R,
                          static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? GSEARCH_OK : GSEARCH_ERR_HIP;
}

int gsearch_build_tables_profiled(int32_t B, int32_t L, int32_t S, int32_t M, int32_t Y,
                                  int32_t NB, const int32_t *desc, const int32_t *layer_type,
                                  const gsearch_layer_profile *profile, const double *bandwidth,
                                  const gsearch_profile_params *par, float *T, int32_t *O,
                                  void *stream) {
  if (B < 1 || L < 1 || S < 1 || M < 1 || Y < 1 || NB < 1 || !desc || !layer_type || !profile ||
      !bandwidth || !par || !T || !O)
    return GSEARCH_ERR_INVALID_ARG;
  if (!(par->tokens > 0.0) || !(par->bin_bytes > 0.0) || !(par->overlap >= 0.0) ||
      !(par->overlap <= 1.0))
    return GSEARCH_ERR_INVALID_ARG;
  gs::launch_build_tables_profiled(B, L, S, M, Y, NB, desc, layer_type,
                                   reinterpret_cast<const double *>(profile), bandwidth,
                                   par->tokens, par->overlap, par->bin_bytes, par->ckpt_keep,
                                   par->state_factor, T, O, static_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? GSEARCH_OK : GSEARCH_ERR_HIP;
}

} // extern "C"
