// Forward kernels of the per-layer strategy DP (paper section 2, "Search Engine"):
//   C[l][e][sj] = ( min_si ( C[l-1][e-O[l][sj]][si] + R[si][sj] ) ) + T[l][sj]
// One launch advances every instance of the batch by one layer front.
//
// Data layout: a C plane is [b][s][e] with the budget index e contiguous (pitch a
// multiple of 64), so that a wavefront whose lanes are 64 consecutive budget rows reads
// and writes 256 contiguous bytes per strategy row.
//
// Register-tiled "push" form (k_dp_push): a lane owns ONE source row e' of the previous
// plane and keeps all S values C[l-1][e'][.] in VGPRs.  For each target strategy sj the
// wave scans si with the transition column R[.][sj] as wave-uniform scalar operands, then
// adds T and stores to row e' + O[l][sj].  Every C operand is read from HBM/L2 once and
// reused S times from registers, so the kernel is bound by the vector ALU (one add and
// the min/argmin bookkeeping per relaxation), not by LDS or HBM.  The shifted stores
// stay coalesced because O[l][sj] is uniform across the wave.
//
// Rows e < O[l][sj] of the target cannot hold layer l under sj: they are set to +inf
// (bp 0) by the wave that owns those rows, so that every row 0..E of the target plane is
// written exactly once per launch and nothing stale survives from an earlier solve.
#include "gsearch_internal.h"

#include <type_traits>

namespace gs {

#define GS_INF __builtin_huge_valf()

static __device__ __forceinline__ int wave_uniform(int v) {
  return __builtin_amdgcn_readfirstlane(v);
}

// ---------------------------------------------------------------------------------------
// Argmin scan of the register-tiled kernel, written as inline assembly.
//
// Per relaxation the vector ALU executes exactly four instructions,
//     v = c + r;   keep = (v >= m);   m = keep ? m : v;   arg = keep ? arg : idx
// ("v >= m keeps" is the strict-less-than update of the recurrence; NaN cannot occur
// because inputs are validated non-negative and +inf only ever meets +inf).
// Left to the compiler, the index selects get deferred and all S compare masks are parked
// in scalar registers and spilled, so the schedule is fixed by hand here:
//   * two independent chains (even candidates -> chain A, odd -> chain B) are interleaved
//     so that, between a compare that writes a lane mask into scalar registers and the
//     selects that read it, two other vector instructions always issue (gfx950 requires
//     two wait states there; the last step of a block has no adds left and uses s_nop);
//   * chain-local indices n (candidate 2n or 2n+1) stay below 64, so they are inline
//     constants and never compete with the mask for the constant bus;
//   * the eight transition values of the NEXT block are fetched by one scalar load issued
//     at the top of the block and awaited at its end, after 32 vector instructions.
// One block handles candidates 8q .. 8q+7; `r` holds their transition costs, `rn`
// receives those of the following eight (the first eight of the next column after the
// last block: the caller keeps one padding row behind the table for that).
// ---------------------------------------------------------------------------------------
typedef float float8_t __attribute__((ext_vector_type(8)));

template <int Q>
static __device__ __forceinline__ void argmin_block8(float &mA, int &argA, float &mB, int &argB,
                                                     const float *c, const float8_t &r,
                                                     float8_t &rn, const float *col) {
  float tA0, tB0, tA1, tB1;
  unsigned long long maskA;
  asm volatile(
      "s_load_dwordx8 %[rn], %[col], %[n0]*8+32\n\t"
      "v_add_f32 %[tA0], %[r0], %[c0]\n\t"
      "v_add_f32 %[tB0], %[r1], %[c1]\n\t"
      // step 0
      "v_cmp_ge_f32 %[mk], %[tA0], %[mA]\n\t"
      "v_cmp_ge_f32 vcc, %[tB0], %[mB]\n\t"
      "v_add_f32 %[tA1], %[r2], %[c2]\n\t"
      "v_add_f32 %[tB1], %[r3], %[c3]\n\t"
      "v_cndmask_b32 %[mA], %[tA0], %[mA], %[mk]\n\t"
      "v_cndmask_b32 %[aA], %[n0], %[aA], %[mk]\n\t"
      "v_cndmask_b32 %[mB], %[tB0], %[mB], vcc\n\t"
      "v_cndmask_b32 %[aB], %[n0], %[aB], vcc\n\t"
      // step 1
      "v_cmp_ge_f32 %[mk], %[tA1], %[mA]\n\t"
      "v_cmp_ge_f32 vcc, %[tB1], %[mB]\n\t"
      "v_add_f32 %[tA0], %[r4], %[c4]\n\t"
      "v_add_f32 %[tB0], %[r5], %[c5]\n\t"
      "v_cndmask_b32 %[mA], %[tA1], %[mA], %[mk]\n\t"
      "v_cndmask_b32 %[aA], %[n0]+1, %[aA], %[mk]\n\t"
      "v_cndmask_b32 %[mB], %[tB1], %[mB], vcc\n\t"
      "v_cndmask_b32 %[aB], %[n0]+1, %[aB], vcc\n\t"
      // step 2
      "v_cmp_ge_f32 %[mk], %[tA0], %[mA]\n\t"
      "v_cmp_ge_f32 vcc, %[tB0], %[mB]\n\t"
      "v_add_f32 %[tA1], %[r6], %[c6]\n\t"
      "v_add_f32 %[tB1], %[r7], %[c7]\n\t"
      "v_cndmask_b32 %[mA], %[tA0], %[mA], %[mk]\n\t"
      "v_cndmask_b32 %[aA], %[n0]+2, %[aA], %[mk]\n\t"
      "v_cndmask_b32 %[mB], %[tB0], %[mB], vcc\n\t"
      "v_cndmask_b32 %[aB], %[n0]+2, %[aB], vcc\n\t"
      // step 3
      "v_cmp_ge_f32 %[mk], %[tA1], %[mA]\n\t"
      "v_cmp_ge_f32 vcc, %[tB1], %[mB]\n\t"
      "s_nop 0\n\t"
      "v_cndmask_b32 %[mA], %[tA1], %[mA], %[mk]\n\t"
      "v_cndmask_b32 %[aA], %[n0]+3, %[aA], %[mk]\n\t"
      "v_cndmask_b32 %[mB], %[tB1], %[mB], vcc\n\t"
      "v_cndmask_b32 %[aB], %[n0]+3, %[aB], vcc\n\t"
      "s_waitcnt lgkmcnt(0)"
      : [mA] "+v"(mA), [aA] "+v"(argA), [mB] "+v"(mB), [aB] "+v"(argB), [tA0] "=&v"(tA0),
        [tB0] "=&v"(tB0), [tA1] "=&v"(tA1), [tB1] "=&v"(tB1), [mk] "=&s"(maskA),
        [rn] "=&s"(rn)
      : [col] "s"(col), [n0] "n"(4 * Q), [r0] "s"(r[0]), [r1] "s"(r[1]), [r2] "s"(r[2]),
        [r3] "s"(r[3]), [r4] "s"(r[4]), [r5] "s"(r[5]), [r6] "s"(r[6]), [r7] "s"(r[7]),
        [c0] "v"(c[8 * Q + 0]), [c1] "v"(c[8 * Q + 1]), [c2] "v"(c[8 * Q + 2]),
        [c3] "v"(c[8 * Q + 3]), [c4] "v"(c[8 * Q + 4]), [c5] "v"(c[8 * Q + 5]),
        [c6] "v"(c[8 * Q + 6]), [c7] "v"(c[8 * Q + 7])
      : "vcc", "memory");
}

// Same eight-candidate block without the scalar prefetch: used for all but the last of the
// RU row groups that share one set of transition values.
template <int Q>
static __device__ __forceinline__ void argmin_block8_shared(float &mA, int &argA, float &mB,
                                                            int &argB, const float *c,
                                                            const float8_t &r) {
  float tA0, tB0, tA1, tB1;
  unsigned long long maskA;
  asm volatile(
      "v_add_f32 %[tA0], %[r0], %[c0]\n\t"
      "v_add_f32 %[tB0], %[r1], %[c1]\n\t"
      "v_cmp_ge_f32 %[mk], %[tA0], %[mA]\n\t"
      "v_cmp_ge_f32 vcc, %[tB0], %[mB]\n\t"
      "v_add_f32 %[tA1], %[r2], %[c2]\n\t"
      "v_add_f32 %[tB1], %[r3], %[c3]\n\t"
      "v_cndmask_b32 %[mA], %[tA0], %[mA], %[mk]\n\t"
      "v_cndmask_b32 %[aA], %[n0], %[aA], %[mk]\n\t"
      "v_cndmask_b32 %[mB], %[tB0], %[mB], vcc\n\t"
      "v_cndmask_b32 %[aB], %[n0], %[aB], vcc\n\t"
      "v_cmp_ge_f32 %[mk], %[tA1], %[mA]\n\t"
      "v_cmp_ge_f32 vcc, %[tB1], %[mB]\n\t"
      "v_add_f32 %[tA0], %[r4], %[c4]\n\t"
      "v_add_f32 %[tB0], %[r5], %[c5]\n\t"
      "v_cndmask_b32 %[mA], %[tA1], %[mA], %[mk]\n\t"
      "v_cndmask_b32 %[aA], %[n0]+1, %[aA], %[mk]\n\t"
      "v_cndmask_b32 %[mB], %[tB1], %[mB], vcc\n\t"
      "v_cndmask_b32 %[aB], %[n0]+1, %[aB], vcc\n\t"
      "v_cmp_ge_f32 %[mk], %[tA0], %[mA]\n\t"
      "v_cmp_ge_f32 vcc, %[tB0], %[mB]\n\t"
      "v_add_f32 %[tA1], %[r6], %[c6]\n\t"
      "v_add_f32 %[tB1], %[r7], %[c7]\n\t"
      "v_cndmask_b32 %[mA], %[tA0], %[mA], %[mk]\n\t"
      "v_cndmask_b32 %[aA], %[n0]+2, %[aA], %[mk]\n\t"
      "v_cndmask_b32 %[mB], %[tB0], %[mB], vcc\n\t"
      "v_cndmask_b32 %[aB], %[n0]+2, %[aB], vcc\n\t"
      "v_cmp_ge_f32 %[mk], %[tA1], %[mA]\n\t"
      "v_cmp_ge_f32 vcc, %[tB1], %[mB]\n\t"
      "s_nop 0\n\t"
      "v_cndmask_b32 %[mA], %[tA1], %[mA], %[mk]\n\t"
      "v_cndmask_b32 %[aA], %[n0]+3, %[aA], %[mk]\n\t"
      "v_cndmask_b32 %[mB], %[tB1], %[mB], vcc\n\t"
      "v_cndmask_b32 %[aB], %[n0]+3, %[aB], vcc"
      : [mA] "+v"(mA), [aA] "+v"(argA), [mB] "+v"(mB), [aB] "+v"(argB), [tA0] "=&v"(tA0),
        [tB0] "=&v"(tB0), [tA1] "=&v"(tA1), [tB1] "=&v"(tB1), [mk] "=&s"(maskA)
      : [n0] "n"(4 * Q), [r0] "s"(r[0]), [r1] "s"(r[1]), [r2] "s"(r[2]), [r3] "s"(r[3]),
        [r4] "s"(r[4]), [r5] "s"(r[5]), [r6] "s"(r[6]), [r7] "s"(r[7]),
        [c0] "v"(c[8 * Q + 0]), [c1] "v"(c[8 * Q + 1]), [c2] "v"(c[8 * Q + 2]),
        [c3] "v"(c[8 * Q + 3]), [c4] "v"(c[8 * Q + 4]), [c5] "v"(c[8 * Q + 5]),
        [c6] "v"(c[8 * Q + 6]), [c7] "v"(c[8 * Q + 7])
      : "vcc");
}

// Running state of one lane's scan: the two chains of the flat argmin.
struct ArgminState {
  float mA, mB;
  int argA, argB;
};

template <int Q, int NQ, int RU, int SP>
struct ArgminBlocks {
  static __device__ __forceinline__ void run(ArgminState (&st)[RU], const float (&c)[RU][SP],
                                             float8_t &r, const float *col) {
    float8_t rn;
#pragma unroll
    for (int u = 0; u < RU - 1; ++u)
      argmin_block8_shared<Q>(st[u].mA, st[u].argA, st[u].mB, st[u].argB, c[u], r);
    argmin_block8<Q>(st[RU - 1].mA, st[RU - 1].argA, st[RU - 1].mB, st[RU - 1].argB, c[RU - 1],
                     r, rn, col);
    r = rn;
    ArgminBlocks<Q + 1, NQ, RU, SP>::run(st, c, r, col);
  }
};
template <int NQ, int RU, int SP>
struct ArgminBlocks<NQ, NQ, RU, SP> {
  static __device__ __forceinline__ void run(ArgminState (&)[RU], const float (&)[RU][SP],
                                             float8_t &, const float *) {}
};

// First eight transition values of a column, fetched and awaited (start of a tile).
static __device__ __forceinline__ float8_t load_col_head(const float *col) {
  float8_t r;
  asm volatile("s_load_dwordx8 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(r) : "s"(col) : "memory");
  return r;
}

// ---------------------------------------------------------------------------------------
// Level 1 of the two-level argmin (and the whole scan of the min-only pass), left to the
// compiler: per chunk of eight candidates eight adds and four minimum instructions give
// the chunk minimum cm; WITH_ARG then updates (m, g) with a strict "<", so that g ends as
// the first chunk attaining the minimum.  The transition values are fetched sixteen at a
// time (one wide scalar load per two chunks), which halves the number of scalar-load
// waits compared with one load per chunk.  (A hand-scheduled variant that requested the
// next chunk at the top of an eight-candidate block and waited at its end was slower: it
// doubles the number of requests and its 12 vector instructions do not cover a
// scalar-cache hit.)
// ---------------------------------------------------------------------------------------
typedef float float16_t __attribute__((ext_vector_type(16)));

template <bool WITH_ARG>
static __device__ __forceinline__ void chunk_update(float &m, int &g, float cm, int q) {
  if (WITH_ARG) {
    const bool lt = cm < m;
    m = lt ? cm : m;
    g = lt ? q : g;
  } else {
    m = __builtin_fminf(m, cm);
  }
}

// SA (a multiple of 4, SP - 8 < SA <= SP): candidates SA .. SP-1 are padding, +inf by
// construction, and can never be the strict minimum, so the last chunk may stop after
// four of them (saves four adds and two minimum instructions per column when the
// strategy count is 4 mod 8, as with the paper's 44).
template <int SP, bool WITH_ARG, int SA = SP>
static __device__ __forceinline__ void scan_chunks(float &m, int &g, const float (&c)[SP],
                                                   const float *__restrict__ rc) {
  static_assert(SA % 4 == 0 && SA <= SP && SA > SP - 8, "SA trims at most half a chunk");
#pragma unroll
  for (int p = 0; p < SP / 16; ++p) {
    const float16_t r = *reinterpret_cast<const float16_t *>(rc + 16 * p);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int q = 2 * p + h;
      float cm = __builtin_fminf(c[8 * q] + r[8 * h], c[8 * q + 1] + r[8 * h + 1]);
#pragma unroll
      for (int k = 2; k < 8; ++k)
        if (8 * q + k < SA) cm = __builtin_fminf(cm, c[8 * q + k] + r[8 * h + k]);
      chunk_update<WITH_ARG>(m, g, cm, q);
    }
  }
  if (SP % 16 != 0) { // one last chunk of eight (SP = 8 or 24)
    constexpr int q = SP / 8 - 1;
    const float8_t r = *reinterpret_cast<const float8_t *>(rc + 8 * q);
    float cm = __builtin_fminf(c[8 * q] + r[0], c[8 * q + 1] + r[1]);
#pragma unroll
    for (int k = 2; k < 8; ++k)
      if (8 * q + k < SA) cm = __builtin_fminf(cm, c[8 * q + k] + r[k]);
    chunk_update<WITH_ARG>(m, g, cm, q);
  }
}

// SP: padded strategy count (compile time).  RU: groups of 64 budget rows per wave (a lane
// owns rows r, r+64, ...): with few strategies the per-column work of one row group is too
// short to amortise the scalar loads, the loop and the stores' address arithmetic, so
// several row groups share them.  WITH_BP: also track and store the argmin.
template <int SP, int RU, bool WITH_BP>
__global__ __launch_bounds__(kRowsPerBlock) void k_dp_push(
    const float *__restrict__ src, float *__restrict__ dst, uint8_t *__restrict__ bp,
    const float *__restrict__ Tq, const int32_t *__restrict__ Oq,
    const float *__restrict__ Rt, const int32_t *__restrict__ ridx,
    const int32_t *__restrict__ budget, const int32_t *__restrict__ topsum,
    const int32_t *__restrict__ lowsum, int B, int L, int S,
    int l, int pitch, int jsplit, int nblk) {
  // Work item p = row_block * B + b (nblk of them): consecutive items belong to different
  // instances, so every instance (and ragged budgets) spreads evenly over the chip.  The
  // hardware deals consecutive workgroups round-robin to the eight XCDs, each with its own
  // L2, and the jsplit workgroups that share one item read the same source rows: they are
  // numbered so that they land on the same XCD and the rows are fetched into one L2 only,
  //   blockIdx.x = ((p / 8) * jsplit + js) * 8 + p % 8.
  const int q = blockIdx.x >> 3;
  const int js = q % jsplit;
  const int p = (q / jsplit) * 8 + (int)(blockIdx.x & 7);
  if (p >= nblk) return;
  const int b = p % B;
  const int wave = wave_uniform(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int tile_start = ((p / B) * (int)(blockDim.x >> 6) + wave) * (kWave * RU);
  const int E = budget[b];
  if (tile_start > E) return;
  // this workgroup's slice of target strategies
  const int jper = (S + jsplit - 1) / jsplit;
  const int jbeg = js * jper;
  const int jend = jbeg + jper < S ? jbeg + jper : S;
  if (jbeg >= jend) return;

  const int row0 = tile_start + lane;
  const int bl = b * L + l;
  // source rows above E - topsum[l] (the least memory layers l.. still need) feed no result; source rows below `low`, the
  // least memory any plan of layers 0..l-1 needs, hold +inf only, so their targets are
  // filled with +inf by the row owners below instead of being computed
  const int low = lowsum[bl - 1];
  const bool compute = tile_start <= E - topsum[bl] && tile_start + kWave * RU > low;
  const size_t plane_off = (size_t)b * S * pitch;
  const float *__restrict__ srcb = src + plane_off;
  float *__restrict__ dstb = dst + plane_off;
  uint8_t *__restrict__ bpb = WITH_BP ? bp + plane_off : nullptr;
  const float *__restrict__ rk = Rt + (size_t)ridx[bl] * SP * SP;
  const float *__restrict__ trow = Tq + (size_t)bl * SP;
  const int32_t *__restrict__ orow = Oq + (size_t)bl * SP;

  float c[RU][SP];
#pragma unroll
  for (int u = 0; u < RU; ++u) {
    const int row = row0 + u * kWave;
#pragma unroll
    for (int i = 0; i < SP; ++i)
      c[u][i] = (compute && i < S && row <= E) ? srcb[(size_t)i * pitch + row] : GS_INF;
  }

  float8_t rcur;
  if (WITH_BP && compute) rcur = load_col_head(rk + (size_t)jbeg * SP);
  for (int j = jbeg; j < jend; ++j) {
    const int o = orow[j];
    const float t = trow[j];
    if (compute) {
      const float *__restrict__ rc = rk + (size_t)j * SP;
      float m[RU];
      int arg[RU];
      if (WITH_BP) {
        ArgminState st[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) st[u] = ArgminState{GS_INF, GS_INF, 0, 0};
        ArgminBlocks<0, SP / 8, RU, SP>::run(st, c, rcur, rc);
#pragma unroll
        for (int u = 0; u < RU; ++u) {
          // merge the chains: candidate 2*argA (even chain) against 2*argB+1 (odd chain),
          // the strictly smaller value wins and equal values go to the lower candidate
          const int candA = 2 * st[u].argA, candB = 2 * st[u].argB + 1;
          const bool takeB = (st[u].mB < st[u].mA) || (st[u].mB == st[u].mA && candB < candA);
          m[u] = takeB ? st[u].mB : st[u].mA;
          arg[u] = takeB ? candB : candA;
        }
      } else {
#pragma unroll
        for (int u = 0; u < RU; ++u) {
          m[u] = GS_INF;
          arg[u] = 0;
          scan_chunks<SP, false>(m[u], arg[u], c[u], rc);
        }
      }
      // the column's base stays a scalar 64-bit address, the lanes add a 32-bit row offset
      float *__restrict__ dj = dstb + (size_t)j * pitch;
      uint8_t *__restrict__ bj = WITH_BP ? bpb + (size_t)j * pitch : nullptr;
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const int row = row0 + u * kWave;
        const int eo = row + o;
        if (row >= low && eo <= E) {
          dj[(uint32_t)eo] = m[u] + t;
          if (WITH_BP) bj[(uint32_t)eo] = (uint8_t)arg[u];
        }
      }
    }
    if (tile_start < o + low) {
      float *__restrict__ dj = dstb + (size_t)j * pitch;
      uint8_t *__restrict__ bj = WITH_BP ? bpb + (size_t)j * pitch : nullptr;
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const int row = row0 + u * kWave;
        if (row <= E && row < o + low) {
          dj[(uint32_t)row] = GS_INF;
          if (WITH_BP) bj[(uint32_t)row] = 0;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// LDS-staged tile kernel with a two-level argmin.
//
// One workgroup owns one 64-row tile of source rows; its waves split the target
// strategies among themselves.  The tile C[l-1][rows][0..S) is fetched from HBM once,
// cooperatively, into LDS ([si][64 rows], so that lane r always hits bank r mod 32), and
// every wave then copies it into registers.
//
// Argmin in two levels, which cuts the vector work per relaxation from four instructions
// to a little over two while producing the same index as the strict-"<" scan:
//   level 1  the si candidates are taken in chunks of eight; a chunk costs eight adds and
//            four (three-input) minimum instructions and yields the chunk minimum cm;
//            "cm < m" (strict) updates the running minimum m and the chunk number g, so
//            that g ends as the FIRST chunk that attains the overall minimum;
//   level 2  only chunk g is looked at again: its eight sums are rebuilt from the LDS tile
//            and the transition column (same operands, same fp32 add, hence the same
//            bits) and the lowest k with sum == m is the argmin 8g + k.
// If every candidate is +inf, m stays +inf, g stays 0 and level 2 returns index 0, which
// is what the scan gives.
// ---------------------------------------------------------------------------------------
template <int SP, int NW, bool WITH_BP, int SA>
__global__ __launch_bounds__(NW *kWave) void k_dp_tile(
    const float *__restrict__ src, float *__restrict__ dst, uint8_t *__restrict__ bp,
    const float *__restrict__ Tq, const int32_t *__restrict__ Oq,
    const float *__restrict__ Rt, const int32_t *__restrict__ ridx,
    const int32_t *__restrict__ budget, const int32_t *__restrict__ topsum,
    const int32_t *__restrict__ lowsum, int B, int L, int S,
    int l, int pitch) {
  extern __shared__ float tile[]; // [SP][64]
  const int b = blockIdx.x % B;
  const int tile_start = (int)(blockIdx.x / B) * kWave;
  const int js = wave_uniform(threadIdx.x >> 6);
  constexpr int nw = NW; // waves per workgroup = slices of the target strategies
  const int lane = threadIdx.x & 63;
  const int E = budget[b];
  if (tile_start > E) return; // whole workgroup

  const int row = tile_start + lane;
  const bool valid = row <= E;
  const int bl = b * L + l;
  const int low = lowsum[bl - 1]; // rows below it are +inf in the previous plane
  const bool compute = tile_start <= E - topsum[bl] && tile_start + kWave > low; // uniform
  const size_t plane_off = (size_t)b * S * pitch;
  const float *__restrict__ srcb = src + plane_off;
  float *__restrict__ dstb = dst + plane_off;
  uint8_t *__restrict__ bpb = WITH_BP ? bp + plane_off : nullptr;
  const float *__restrict__ rk = Rt + (size_t)ridx[bl] * SP * SP;
  const float *__restrict__ trow = Tq + (size_t)bl * SP;
  const int32_t *__restrict__ orow = Oq + (size_t)bl * SP;

  float c[SP];
  if (compute) {
    // every wave fetches SP/NW strategy rows of the tile: all loads first, then the LDS
    // writes, so that the loads are in flight together
    // (unconditional loads from a clamped row, padding selected afterwards: no lane-mask
    // juggling between the loads; the strategy rows S..SP-1 do not exist, their addresses
    // fall into the next instance or the slack behind the last plane)
    float stage[SP / NW];
    const uint32_t rowc = (uint32_t)(valid ? row : E);
#pragma unroll
    for (int u = 0; u < SP / NW; ++u) {
      const int i = u * NW + js;
      const float v = (srcb + (size_t)i * pitch)[rowc];
      stage[u] = (i < S && valid) ? v : GS_INF;
    }
#pragma unroll
    for (int u = 0; u < SP / NW; ++u) tile[(u * NW + js) * kWave + lane] = stage[u];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < SP; ++i) c[i] = tile[i * kWave + lane];
  } else {
#pragma unroll
    for (int i = 0; i < SP; ++i) c[i] = GS_INF;
  }

  const int jper = (S + nw - 1) / nw;
  const int jbeg = js * jper;
  const int jend = jbeg + jper < S ? jbeg + jper : S;
  // Level 2 of a column: which of the eight candidates of chunk g attains m.  The eight
  // transition values differ from lane to lane, so they come through the vector memory
  // path (two 16-byte loads per lane), the eight previous-plane values from the LDS tile.
  struct Column {
    float4 ra, rb;
    float m, t;
    int g, j, o;
  };
  auto finish = [&](const Column &d) {
    const float *tg = tile + (8 * d.g) * kWave + lane; // per-lane slice of the tile
    const float rr[8] = {d.ra.x, d.ra.y, d.ra.z, d.ra.w, d.rb.x, d.rb.y, d.rb.z, d.rb.w};
    int arg = 8 * d.g;
#pragma unroll
    for (int k = 7; k >= 1; --k) {
      const float v = tg[k * kWave] + rr[k];
      arg = (v == d.m) ? 8 * d.g + k : arg;
    }
    const float v0 = tg[0] + rr[0];
    arg = (v0 == d.m) ? 8 * d.g : arg;
    const int eo = row + d.o;
    if (row >= low && eo <= E) {
      // the column's base stays a scalar 64-bit address, the lanes add a 32-bit row offset
      float *__restrict__ dj = dstb + (size_t)d.j * pitch;
      uint8_t *__restrict__ bj = bpb + (size_t)d.j * pitch;
      dj[(uint32_t)eo] = d.m + d.t;
      bj[(uint32_t)eo] = (uint8_t)arg;
    }
  };
  for (int j = jbeg; j < jend; ++j) {
    const int o = orow[j];
    const float t = trow[j];
    if (compute) {
      const float *__restrict__ rc = rk + (size_t)j * SP;
      float m = GS_INF;
      int g = 0;
      scan_chunks<SP, WITH_BP, SA>(m, g, c, rc);
      if constexpr (WITH_BP) {
        const float *__restrict__ rg = rc + 8 * g; // per-lane slice of the column
        Column d;
        d.ra = *reinterpret_cast<const float4 *>(rg);
        d.rb = *reinterpret_cast<const float4 *>(rg + 4);
        d.m = m; d.t = t; d.g = g; d.j = j; d.o = o;
        finish(d);
      } else {
        const int eo = row + o;
        float *__restrict__ dj = dstb + (size_t)j * pitch;
        if (row >= low && eo <= E) dj[(uint32_t)eo] = m + t;
      }
    }
    if (tile_start < o + low) {
      if (valid && row < o + low) {
        float *__restrict__ dj = dstb + (size_t)j * pitch;
        dj[(uint32_t)row] = GS_INF;
        if (WITH_BP) (bpb + (size_t)j * pitch)[(uint32_t)row] = 0;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// The same tile kernel for strategy counts beyond the register-tiled sizes (129 .. 1024):
// the tile stays in LDS and level 1 streams it from there, JB target strategies per pass
// so that every LDS read serves JB relaxations (4 / JB bytes of LDS traffic per relaxation; the
// scalar transition values of the next chunk are requested while the current one is being
// added up).  Same two-level argmin, same stores, uint8 or uint16 backpointers.  About half
// the rate of the register-tiled kernel, against a seventieth for the pull-form fallback.
// Tiles of 64 budget rows up to 608 strategies (152 KB of LDS), of 32 rows beyond.
// ---------------------------------------------------------------------------------------
template <typename BPT, int NW, bool WITH_BP, int JB, int ROWS>
__global__ __launch_bounds__(NW *kWave) void k_dp_wide(
    const float *__restrict__ src, float *__restrict__ dst, BPT *__restrict__ bp,
    const float *__restrict__ Tq, const int32_t *__restrict__ Oq,
    const float *__restrict__ Rt, const int32_t *__restrict__ ridx,
    const int32_t *__restrict__ budget, const int32_t *__restrict__ topsum,
    const int32_t *__restrict__ lowsum, int B, int L, int S, int SP, int l, int pitch) {
  // ROWS: budget rows per tile, 64, or 32 when S x 64 floats would not fit LDS (then the
  // upper half of every wave repeats the lower half's rows and stores nothing)
  extern __shared__ float tile[]; // [SP][ROWS]
  const int b = blockIdx.x % B;
  const int tile_start = (int)(blockIdx.x / B) * ROWS;
  const int js = wave_uniform(threadIdx.x >> 6);
  const int lane = threadIdx.x & (ROWS - 1);
  const bool act = ROWS == kWave || (threadIdx.x & 63) < ROWS; // this lane stores
  const int E = budget[b];
  if (tile_start > E) return; // whole workgroup

  const int row = tile_start + lane;
  const bool valid = row <= E && act;
  const int bl = b * L + l;
  const int low = lowsum[bl - 1]; // rows below it are +inf in the previous plane
  const bool compute = tile_start <= E - topsum[bl] && tile_start + ROWS > low; // uniform
  const size_t plane_off = (size_t)b * S * pitch;
  const float *__restrict__ srcb = src + plane_off;
  float *__restrict__ dstb = dst + plane_off;
  BPT *__restrict__ bpb = WITH_BP ? bp + plane_off : nullptr;
  const float *__restrict__ rk = Rt + (size_t)ridx[bl] * SP * SP;
  const float *__restrict__ trow = Tq + (size_t)bl * SP;
  const int32_t *__restrict__ orow = Oq + (size_t)bl * SP;
  // pairs of chunks of eight candidates that hold a strategy (SP is a multiple of 16 here)
  const int np = (S + 15) / 16;
  const int rows_used = 16 * np;

  if (compute) {
    // tile HBM -> LDS, four rows per wave in flight; padding strategies and rows beyond the
    // budget are +inf
    const uint32_t rowc = (uint32_t)(row <= E ? row : E);
    for (int i0 = js * 4; i0 < rows_used; i0 += NW * 4) {
      float v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u;
        const int ic = i < S ? i : S - 1;
        v[u] = (srcb + (size_t)ic * pitch)[rowc];
        v[u] = (i < S && row <= E) ? v[u] : GS_INF;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (i0 + u < rows_used) tile[(i0 + u) * ROWS + lane] = v[u];
    }
    __syncthreads();
  }

  const int jper = (S + NW - 1) / NW;
  const int jbeg = js * jper;
  const int jend = jbeg + jper < S ? jbeg + jper : S;
  // level 2 and the stores of one column (see k_dp_tile)
  auto finish = [&](int j, int o, float t, float m, int g) {
    if constexpr (WITH_BP) {
      const float *tg = tile + (8 * g) * ROWS + lane;        // per-lane slice of the tile
      const float *__restrict__ rg = rk + (size_t)j * SP + 8 * g; // and of the column
      const float4 ra = *reinterpret_cast<const float4 *>(rg);
      const float4 rb = *reinterpret_cast<const float4 *>(rg + 4);
      const float rr[8] = {ra.x, ra.y, ra.z, ra.w, rb.x, rb.y, rb.z, rb.w};
      int kk = 0;
#pragma unroll
      for (int k = 7; k >= 0; --k) { // descending: the lowest matching candidate wins
        const float v = tg[k * ROWS] + rr[k];
        kk = (v == m) ? k : kk;
      }
      const int eo = row + o;
      if (act && row >= low && eo <= E) {
        (dstb + (size_t)j * pitch)[(uint32_t)eo] = m + t;
        (bpb + (size_t)j * pitch)[(uint32_t)eo] = (BPT)(8 * g + kk);
      }
    } else {
      const int eo = row + o;
      if (act && row >= low && eo <= E) (dstb + (size_t)j * pitch)[(uint32_t)eo] = m + t;
    }
  };
  for (int j = jbeg; j < jend; j += JB) {
    int jj[JB], oo[JB];
    float tt[JB];
#pragma unroll
    for (int x = 0; x < JB; ++x) {
      jj[x] = j + x < jend ? j + x : j; // the last pass may repeat column j (results dropped)
      oo[x] = orow[jj[x]];
      tt[x] = trow[jj[x]];
    }
    if (compute) {
      const float *__restrict__ rc[JB];
      float m[JB];
      int g[JB];
#pragma unroll
      for (int x = 0; x < JB; ++x) {
        rc[x] = rk + (size_t)jj[x] * SP;
        m[x] = GS_INF;
        g[x] = 0;
      }
      if constexpr (JB <= 2) {
        // sixteen transition values per scalar request (two chunks), the next request in
        // flight meanwhile: 2 x JB x 16 scalar registers
        float16_t r[JB];
#pragma unroll
        for (int x = 0; x < JB; ++x) r[x] = *reinterpret_cast<const float16_t *>(rc[x]);
        for (int p = 0; p < np; ++p) {
          const int pn = p + 1 < np ? p + 1 : p;
          float16_t n[JB];
#pragma unroll
          for (int x = 0; x < JB; ++x) n[x] = *reinterpret_cast<const float16_t *>(rc[x] + 16 * pn);
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const float *tq = tile + (16 * p + 8 * h) * ROWS + lane;
            float c[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) c[k] = tq[k * ROWS];
#pragma unroll
            for (int x = 0; x < JB; ++x) {
              float cm = __builtin_fminf(c[0] + r[x][8 * h], c[1] + r[x][8 * h + 1]);
#pragma unroll
              for (int k = 2; k < 8; ++k) cm = __builtin_fminf(cm, c[k] + r[x][8 * h + k]);
              chunk_update<WITH_BP>(m[x], g[x], cm, 2 * p + h);
            }
          }
#pragma unroll
          for (int x = 0; x < JB; ++x) r[x] = n[x];
        }
      } else {
        // more columns per pass: eight values per request, or the scalar registers run out
        float8_t r[JB];
#pragma unroll
        for (int x = 0; x < JB; ++x) r[x] = *reinterpret_cast<const float8_t *>(rc[x]);
        const int nq = 2 * np;
        for (int q = 0; q < nq; ++q) {
          const int qn = q + 1 < nq ? q + 1 : q;
          float8_t n[JB];
#pragma unroll
          for (int x = 0; x < JB; ++x) n[x] = *reinterpret_cast<const float8_t *>(rc[x] + 8 * qn);
          const float *tq = tile + (8 * q) * ROWS + lane;
          float c[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) c[k] = tq[k * ROWS];
#pragma unroll
          for (int x = 0; x < JB; ++x) {
            float cm = __builtin_fminf(c[0] + r[x][0], c[1] + r[x][1]);
#pragma unroll
            for (int k = 2; k < 8; ++k) cm = __builtin_fminf(cm, c[k] + r[x][k]);
            chunk_update<WITH_BP>(m[x], g[x], cm, q);
            r[x] = n[x];
          }
        }
      }
#pragma unroll
      for (int x = 0; x < JB; ++x)
        if (x == 0 || j + x < jend) finish(jj[x], oo[x], tt[x], m[x], g[x]);
    }
    // +inf prefix of the target rows that no computed source row reaches
#pragma unroll
    for (int x = 0; x < JB; ++x) {
      if ((x == 0 || j + x < jend) && tile_start < oo[x] + low && valid && row < oo[x] + low) {
        (dstb + (size_t)jj[x] * pitch)[(uint32_t)row] = GS_INF;
        if (WITH_BP) (bpb + (size_t)jj[x] * pitch)[(uint32_t)row] = 0;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Class kernel: the transition table depends on the strategies only through nc <= 64
// contiguous classes (checked on the device beforehand), R[si][sj] = Rc[class si][class sj].
// Then, for a source row,
//     min_si (C[si] + R[si][sj]) = min_ci ( (min_{si in ci} C[si]) + Rc[ci][cj] )
// bit for bit, because the fp32 add is monotone: one minimum per class (S operations) and
// nc relaxations per target CLASS replace S relaxations per target strategy, and every
// strategy of a target class shares the result before its own T and O are applied.  The
// lowest-index rule survives: classes are ascending index ranges, so the first class that
// attains the minimum (strict "<" scan) holds the lowest strategy attaining it, and that
// strategy is found by rebuilding the sums of this one class from the LDS tile (several of
// its members may round to the same sum, so the member with the smallest C need not be it).
//
// The planes are COMPACT.  The plane of a layer need not be kept per strategy: for l >= 1 let
//     Q[l][c][r] = min_si ( C[l-1][r][si] + R(l, si, c) )          (one row per CLASS c)
// and Q[0][c][r] = 0.  Then C[l][e][s] = Q[l][class s][e - O[l][s]] + T[l][s] for
// e >= O[l][s] (+inf below), which is exactly how the recurrence forms C, in the same
// fp32 operations and order.  A layer front reads the nc rows of Q[l-1] (each source
// strategy si at its own shift O[l-1][si], with its T[l-1][si] added on the fly) and writes
// the nc rows of Q[l] and one backpointer per (target class, source row) with aligned
// stores: 2 nc floats per budget row instead of 2 S cross HBM.  The shifted reads of one
// instance overlap heavily and are served by the L2 of the XCD its workgroups run on.
//
// One workgroup per 64-row tile, NW waves, each rebuilding a contiguous run of source
// strategies.  The class minima are formed by LDS float-minimum atomics (cmin[class][lane]),
// then every wave keeps all of them in registers and takes every NW-th target class.
//
// Rows above E - topsum[l] (the least memory that layers l.. still need) cannot be completed
// to a plan within the budget and are neither computed nor read by anyone.  Rows of Q[l] below the least memory of layers 0..l-1 are +inf by
// definition; the tiles wholly below it are not stored, and every reader of a compact plane
// (the next layer front, the final reductions, the backtrace, the export) applies that bound.
// ---------------------------------------------------------------------------------------
// One 64-row tile of source rows of instance b at layer front l (the work of one workgroup).
// COHERENT: the plane rows are read with loads that bypass the compute unit's vector cache
// (agent-scope relaxed atomic loads), for the one-launch form below, in which the rows were
// written by other workgroups of the same launch.
// `after_loads` is called by every wave once the tile's rows have arrived and the class minima
// are formed, before the arithmetic: the one-launch form requests its next item there.
struct NoHook {
  __device__ __forceinline__ void operator()() const {}
};
// The scalar table entries a wave needs for a tile of instance b at layer front l: the
// per-instance scalars and the O, T and class entries of the wave's source strategies.  All
// are requested before the first of them is looked at (one round trip to the scalar cache
// instead of one per dependent step); none depends on the tile.
template <int PER>
struct ClassScalars {
  int E, low, lowq, mo, kr, nc, maxlen;
  int o_s[PER], c_s[PER];
  float t_s[PER]; // in vector registers where VEC_T says so (every lane holds the same value)
};
template <int SP, int NW, bool VEC_T = false>
static __device__ __forceinline__ ClassScalars<SP / NW> class_scalars(
    const float *__restrict__ Tq, const int32_t *__restrict__ Oq,
    const int32_t *__restrict__ cmeta, const int32_t *__restrict__ cls,
    const int32_t *__restrict__ ridx, const int32_t *__restrict__ budget,
    const int32_t *__restrict__ topsum, const int32_t *__restrict__ lowsum, int L, int l, int b) {
  constexpr int PER = SP / NW; // source strategies per wave (a contiguous run)
  ClassScalars<PER> k;
  const int js = wave_uniform(threadIdx.x >> 6);
  const int bl = b * L + l;
  k.E = budget[b];
  k.low = lowsum[bl - 1]; // C[l-1], and with it Q[l], is +inf below this row
  // Q[l-1] is +inf below the least memory of layers 0..l-2 (Q[0] = 0 has no such rows).
  // Those rows are not stored anywhere: every reader of a compact plane applies this bound.
  k.lowq = lowsum[bl - (l >= 2 ? 2 : 1)];
  k.lowq = l >= 2 ? k.lowq : 0;
  k.mo = topsum[bl];
  k.kr = ridx[bl];
  k.nc = cmeta[0];
  k.maxlen = cmeta[1];
  {
    const float *__restrict__ tprev = Tq + (size_t)(bl - 1) * SP;
    const int32_t *__restrict__ oprev = Oq + (size_t)(bl - 1) * SP;
    // VEC_T: the T entries come through vector loads of one address per load (the index passes
    // through an empty asm as a vector value), so that they take vector registers, of which
    // the kernel has some to spare, and leave twelve scalar ones to the caller.
    int first = js * PER;
    if (VEC_T) asm volatile("" : "+v"(first));
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      k.o_s[u] = oprev[js * PER + u];
      k.c_s[u] = cls[js * PER + u];
      k.t_s[u] = tprev[(VEC_T ? first : js * PER) + u];
    }
  }
  asm volatile(""
               : "+s"(k.E), "+s"(k.low), "+s"(k.lowq), "+s"(k.mo), "+s"(k.kr), "+s"(k.nc),
                 "+s"(k.maxlen));
  // (a longer run would not fit the scalar registers next to the class table row: there the
  // compiler places the loads where the values are used)
  if constexpr (PER <= 16) {
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      asm volatile("" : "+s"(k.o_s[u]), "+s"(k.c_s[u]));
      if (!VEC_T) asm volatile("" : "+s"(k.t_s[u]));
    }
  }
  return k;
}

// What a tile needs in LDS before its rows arrive: class minima at +inf and, for the argmin
// levels, the layer's class table and the run table.  class_tile does this itself unless the
// caller has done it (and a workgroup barrier) already: PREPPED.
template <int SP, int NW, bool WITH_BP, int NC>
static __device__ __forceinline__ void class_tile_prepare(const float *__restrict__ Rc,
                                                          const int32_t *__restrict__ cstart,
                                                          int kr, float *lds, int tid,
                                                          int nthreads) {
  // (tid, nthreads: the threads that share this work, numbered from 0)
  float *cmin = lds;
  float *rc_lds = cmin + NC * kWave;
  int *cs_lds = reinterpret_cast<int *>(rc_lds + NC * NC);
  const float4 inf4 = {GS_INF, GS_INF, GS_INF, GS_INF};
  for (int x = tid; x < NC * kWave / 4; x += nthreads) reinterpret_cast<float4 *>(cmin)[x] = inf4;
  if (WITH_BP) {
    // (the per-lane gathers of the argmin levels read the class table and the run table
    // from LDS; the min-only pass takes both as scalar operands only)
    const float *__restrict__ rck = Rc + (size_t)kr * NC * NC;
    for (int x = tid; x < NC * NC / 4; x += nthreads)
      reinterpret_cast<float4 *>(rc_lds)[x] = reinterpret_cast<const float4 *>(rck)[x];
    for (int x = tid; x <= NC; x += nthreads) cs_lds[x] = cstart[x];
  }
}

template <int SP, int NW, bool WITH_BP, int NC, bool COHERENT, typename Hook = NoHook,
          bool PREPPED = false, typename Hook2 = NoHook>
static __device__ __forceinline__ void class_tile(
    const ClassScalars<SP / NW> &k, const float *__restrict__ qsrc, float *__restrict__ qdst,
    uint8_t *__restrict__ bp, const float *__restrict__ Rc, const int32_t *__restrict__ cstart,
    int Sc, int pitch, int src_pitch, int b, int tile_start, float *lds,
    const Hook &after_loads = Hook(), const Hook2 &minima_stored = Hook2()) {
  constexpr int PER = SP / NW; // source strategies per wave (a contiguous run)
  float *cmin = lds;                    // [NC][64]  class minima of the tile
  float *rc_lds = cmin + NC * kWave;    // [NC][NC]  this layer's class table
  int *cs_lds = reinterpret_cast<int *>(rc_lds + NC * NC); // [NC + 1], padded to NC + 32
  float *tile = reinterpret_cast<float *>(cs_lds + NC + 32); // [SP + 3][64], backpointer mode only
  const int js = wave_uniform(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int E = k.E, low = k.low, lowq = k.lowq, mo = k.mo, kr = k.kr, nc = k.nc,
            maxlen = k.maxlen;
  const int(&o_s)[PER] = k.o_s;
  const int(&c_s)[PER] = k.c_s;
  const float(&t_s)[PER] = k.t_s;
  if (tile_start > E - mo) return; // no row here can reach a plan within the budget (whole workgroup)

  const int row = tile_start + lane;
  const size_t inst = (size_t)b * Sc * pitch;
  // (src_pitch == 0: Q[0] = 0 is not stored, every class of every instance reads one shared
  // row of zeros)
  const float *__restrict__ qs = src_pitch ? qsrc + inst : qsrc;
  float *__restrict__ qd = qdst + inst;
  uint8_t *__restrict__ bpb = WITH_BP ? bp + (size_t)b * NC * pitch : nullptr;
  if (tile_start + kWave <= low) return; // +inf throughout, implied by the bound, not stored
  const float *__restrict__ rck = Rc + (size_t)kr * NC * NC;

  // C[l-1][row][si] for this wave's source strategies, rebuilt from the compact plane.
  // Rows beyond the budget count as +inf; padding strategies have O = M + 1 and never fit.
  // Byte offsets inside the instance's compact plane (the launcher admits the kernel only
  // when they fit 31 bits), so a load takes a scalar base and one vector offset: row of
  // class c, shifted down by O, clamped to the start of the row.
  const int row4 = (row <= E ? row : -1) * 4;
  const char *__restrict__ qsb = reinterpret_cast<const char *>(qs);
  const int spitch4 = src_pitch * 4;
  const int lowq4 = lowq * 4;
  float stage[PER];
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const int cb = c_s[u] * spitch4;         // wave-uniform
    const int t = row4 + (cb - o_s[u] * 4);
    const float *__restrict__ at = reinterpret_cast<const float *>(qsb + (uint32_t)(t > cb ? t : cb));
    const float v = (COHERENT ? __hip_atomic_load(at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                              : *at) + t_s[u];
    stage[u] = t >= cb + lowq4 ? v : GS_INF; // source row >= lowq (and >= 0), row within budget
  }
  if (!PREPPED)
    class_tile_prepare<SP, NW, WITH_BP, NC>(Rc, cstart, kr, lds, (int)threadIdx.x, NW * kWave);
  if (WITH_BP) {
    float *tw = tile + (js * PER) * kWave + lane;
#pragma unroll
    for (int u = 0; u < PER; ++u) tw[u * kWave] = stage[u];
  }
  if (!PREPPED) __syncthreads();
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const int c = c_s[u]; // wave-uniform
    __hip_atomic_fetch_min(&cmin[c * kWave + lane], stage[u], __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  __syncthreads();
  after_loads();
  // every wave keeps all class minima in registers (classes that do not exist hold +inf)
  float cmv[NC];
#pragma unroll
  for (int k = 0; k < NC; ++k) cmv[k] = cmin[k * kWave + lane];

  // One target class: the minimum over the source classes (level 1: per chunk of eight classes,
  // first chunk attaining the minimum), stored as Q[l][cj][row]; kept with the chunk.
  // (Rc[cj][.] travels as wave-uniform scalar operands, requested by piece_of)
  constexpr int XP = NC / 16; // sixteen-float pieces per class table row
  auto piece_of = [&](int cj, int x) -> float16_t {
    return *reinterpret_cast<const float16_t *>(rck + (size_t)cj * NC + 16 * x);
  };
  // the two chunks of eight source classes that piece x of a row covers, folded into (m, g)
  auto chunks_of = [&](const float16_t &r, int x, float &m, int &g) {
    // (chunk 0 always exists and starts the scan: "cm < +inf ? cm : +inf" is cm)
#pragma unroll
    for (int q = 2 * x; q < 2 * x + 2; ++q) {
      if (8 * q < nc) {
        const int h = (q & 1) * 8;
        float cm = __builtin_fminf(cmv[8 * q] + r[h], cmv[8 * q + 1] + r[h + 1]);
#pragma unroll
        for (int k = 2; k < 4; ++k) cm = __builtin_fminf(cm, cmv[8 * q + k] + r[h + k]);
        if (8 * q + 4 < nc) { // the upper half of the last chunk may be padding (+inf)
#pragma unroll
          for (int k = 4; k < 8; ++k) cm = __builtin_fminf(cm, cmv[8 * q + k] + r[h + k]);
        }
        if (q == 0) {
          m = cm;
          g = 0;
        } else {
          chunk_update<true>(m, g, cm, q);
        }
      }
    }
  };
  auto store_minimum = [&](int cj, float m) {
    const uint32_t at = (uint32_t)cj * (uint32_t)pitch + (uint32_t)row;
    *reinterpret_cast<float *>(reinterpret_cast<char *>(qd) + (at << 2)) = m;
  };
  // Its argmin, from the minimum m and the chunk g: stored as one backpointer per (target
  // class, source row).
  auto argmin_of = [&](int cj, float m, int g) {
    // level 1b: first class of chunk g attaining it (operands re-read from LDS: g varies
    // from lane to lane)
    int ca = 8 * g;
    {
      const float *cg = cmin + (8 * g) * kWave + lane;
      const float *rg = rc_lds + cj * NC + 8 * g;
      const float4 ra = *reinterpret_cast<const float4 *>(rg);
      const float4 rb = *reinterpret_cast<const float4 *>(rg + 4);
      const float rr[8] = {ra.x, ra.y, ra.z, ra.w, rb.x, rb.y, rb.z, rb.w};
      int kk = 0;
#pragma unroll
      for (int k = 7; k >= 0; --k) { // descending: the lowest matching class wins
        const float v = cg[k * kWave] + rr[k];
        kk = (v == m) ? k : kk;
      }
      ca += kk;
    }
    // level 2: lowest member of class ca whose sum equals m (descending scan, last hit
    // wins); several members can round to the same sum
    const int lo = cs_lds[ca];
    const float rr = rc_lds[cj * NC + ca];
    // Four members per round so that their LDS reads are in flight together, highest
    // first.  Past the end of a short class the scan looks at members of the following
    // classes (or at the padding rows and the slack behind the tile); whatever those match
    // is overwritten, because class ca attains m and its members come later in the scan.
    // (a round that would start beyond the last strategy row is read from the last row on,
    // so the four reads end in the three rows of slack behind the tile at the latest)
    const int tl = lo * kWave + lane;
    const int tl_max = (SP - 1) * kWave + lane;
    int rel = 0;
    if (maxlen <= 4) { // wave-uniform; the usual case: one round, constant member numbers
      const float *tr = tile + (tl < tl_max ? tl : tl_max);
      float tv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) tv[u] = tr[u * kWave];
#pragma unroll
      for (int u = 3; u >= 0; --u) rel = (tv[u] + rr == m) ? u : rel;
    } else {
      for (int d0 = ((maxlen + 3) & ~3) - 4; d0 >= 0; d0 -= 4) {
        const int at0 = tl + d0 * kWave;
        const float *tr = tile + (at0 < tl_max ? at0 : tl_max);
        float tv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) tv[u] = tr[u * kWave];
#pragma unroll
        for (int u = 3; u >= 0; --u) rel = (tv[u] + rr == m) ? d0 + u : rel;
      }
    }
    const uint32_t at = (uint32_t)cj * (uint32_t)pitch + (uint32_t)row;
    bpb[at] = (uint8_t)(lo + rel);
  };
  constexpr bool kMinimaFirst = !std::is_same<Hook2, NoHook>::value;
  if constexpr (kMinimaFirst) {
    // All minima first: once they are stored the next layer front can go ahead (the caller's
    // `minima_stored` publishes that); the argmins, which only the backtrace reads, follow
    // from the minimum and the chunk kept per target class.  The class table rows arrive as
    // pieces of sixteen scalar operands, and the next piece (of this row or of the wave's next
    // target class) is requested as soon as the current one has arrived and before it is used:
    // two pieces are live at a time, so the scalar registers still allow eight waves per SIMD,
    // and a piece's latency is spent under the arithmetic of the one before.  (Scalar loads
    // return in any order, so a wait for one is a wait for all: requested any earlier, the
    // next piece would be waited for together with the current one.)
    constexpr int MAXIT = (NC + NW - 1) / NW;
    constexpr int P = MAXIT * XP;
    float m_it[MAXIT];
    int g_it[MAXIT];
    float16_t piece[P];
    if (js < nc) piece[0] = piece_of(js, 0);
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int it = p / XP, x = p % XP;
      if (js + it * NW < nc) {
        asm volatile("" : "+s"(piece[p]));
        if (p + 1 < P) {
          const int it2 = (p + 1) / XP, x2 = (p + 1) % XP;
          if (js + it2 * NW < nc) piece[p + 1 < P ? p + 1 : p] = piece_of(js + it2 * NW, x2);
        }
        if (x == 0) {
          m_it[it] = GS_INF;
          g_it[it] = 0;
        }
        chunks_of(piece[p], x, m_it[it], g_it[it]);
        if (x == XP - 1) store_minimum(js + it * NW, m_it[it]);
      }
    }
    minima_stored();
    if (WITH_BP) {
#pragma unroll
      for (int it = 0; it < MAXIT; ++it)
        if (js + it * NW < nc) argmin_of(js + it * NW, m_it[it], g_it[it]);
    }
  } else {
    for (int cj = js; cj < nc; cj += NW) {
      float16_t rv[XP];
#pragma unroll
      for (int x = 0; x < XP; ++x) rv[x] = piece_of(cj, x);
      float m = GS_INF;
      int g = 0;
#pragma unroll
      for (int x = 0; x < XP; ++x) chunks_of(rv[x], x, m, g);
      store_minimum(cj, m);
      if (WITH_BP) argmin_of(cj, m, g);
    }
    minima_stored();
  }
}

template <int SP, int NW, bool WITH_BP, int NC>
__global__ __launch_bounds__(NW *kWave) void k_dp_class(
    const float *__restrict__ qsrc, float *__restrict__ qdst, uint8_t *__restrict__ bp,
    const float *__restrict__ Tq, const int32_t *__restrict__ Oq,
    const float *__restrict__ Rc, const int32_t *__restrict__ cmeta,
    const int32_t *__restrict__ cstart, const int32_t *__restrict__ cls,
    const int32_t *__restrict__ ridx, const int32_t *__restrict__ budget,
    const int32_t *__restrict__ topsum, const int32_t *__restrict__ lowsum, int B, int L, int Sc,
    int l, int pitch, int src_pitch, int tiles, unsigned div_magic, int div_shift) {
  // NC: class capacity (32 or 64): registers for the class minima, rows of the class table
  extern __shared__ float lds[];
  // Workgroup -> (instance, tile).  The hardware deals consecutive workgroups out to the 8
  // XCDs in turn, and a tile reads its class rows at many shifts, which the tiles near it in
  // the same instance read too, so an instance's tiles should share an L2.  With a multiple
  // of 8 instances a (instances, tiles) grid does that by itself (instance b runs on XCD
  // b mod 8).  Otherwise (gridDim.y == 1) XCD x gets the x-th eighth of the instance-major
  // list of tiles as a contiguous run: equal shares for any batch size, and only the two
  // ends of a run read rows that another XCD reads as well (7 instances of configs[3]'s
  // shape: 0.188 -> 0.165 ms for 11 fronts).
  int b, tile_start;
  if (gridDim.y > 1 || tiles == 1) {
    b = blockIdx.x;
    tile_start = (int)blockIdx.y * kWave;
  } else {
    const unsigned xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3;
    const unsigned per = gridDim.x >> 3;            // tiles per XCD (the grid is 8 * per)
    const unsigned item = xcd * per + slot;
    if (item >= (unsigned)B * (unsigned)tiles) return;
    // item / tiles by a multiply-high with the host's constant (exact for item < 2^31)
    b = (int)(__umulhi(item, div_magic) >> div_shift);
    tile_start = (int)(item - (unsigned)b * (unsigned)tiles) * kWave;
  }
  const ClassScalars<SP / NW> k =
      class_scalars<SP, NW>(Tq, Oq, cmeta, cls, ridx, budget, topsum, lowsum, L, l, b);
  class_tile<SP, NW, WITH_BP, NC, false>(k, qsrc, qdst, bp, Rc, cstart, Sc, pitch, src_pitch, b,
                                         tile_start, lds);
}

// One tile of a front the plain way: the same results as class_tile (the same single
// additions, minima and first-index rules), with every table entry read through vector loads
// and all loops rolled, so that it needs few registers of either kind.  For the workgroups of
// k_dp_class_fronts that take the tiles behind the first y0 of a front: there it runs in a
// loop, where class_tile's scalar operands would have to be held or fetched again per tile,
// and that loop must not cost the straight-line path registers.  Many times slower per tile.
// Expects what class_tile_prepare lays out (and a barrier after it); ends with the rows of
// Q[l] and the backpointers stored, before any flag.
template <int SP, int NW, bool WITH_BP, int NC>
static __device__ __forceinline__ void class_tile_plain(
    const float *__restrict__ qsrc, float *__restrict__ qdst, uint8_t *__restrict__ bp,
    const float *__restrict__ Tq, const int32_t *__restrict__ Oq,
    const int32_t *__restrict__ cls, const float *__restrict__ Rc, int bl, int kr, int nc, int E,
    int lowq, int Sc, int pitch, int src_pitch, int b, int tile_start, float *lds) {
  float *cmin = lds;
  float *rc_lds = cmin + NC * kWave;
  int *cs_lds = reinterpret_cast<int *>(rc_lds + NC * NC);
  float *tile = reinterpret_cast<float *>(cs_lds + NC + 32);
  const int wave = (int)threadIdx.x >> 6, lane = (int)threadIdx.x & 63;
  const int row = tile_start + lane;
  const size_t inst = (size_t)b * Sc * pitch;
  const float *__restrict__ qs = src_pitch ? qsrc + inst : qsrc;
  float *__restrict__ qd = qdst + inst;
  uint8_t *__restrict__ bpb = WITH_BP ? bp + (size_t)b * NC * pitch : nullptr;
  const float *__restrict__ tprev = Tq + (size_t)(bl - 1) * SP;
  const int32_t *__restrict__ oprev = Oq + (size_t)(bl - 1) * SP;
#pragma unroll 1
  for (int sidx = wave; sidx < SP; sidx += NW) {
    const int o = oprev[sidx], c = cls[sidx];
    const int r = row - o;
    float v = GS_INF;
    if (row <= E && r >= lowq && r >= 0)
      v = __hip_atomic_load(&qs[(size_t)c * src_pitch + r], __ATOMIC_RELAXED,
                            __HIP_MEMORY_SCOPE_AGENT) + tprev[sidx];
    if (WITH_BP) tile[sidx * kWave + lane] = v;
    __hip_atomic_fetch_min(&cmin[c * kWave + lane], v, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  __syncthreads();
  const float *__restrict__ rck = Rc + (size_t)kr * NC * NC;
#pragma unroll 1
  for (int cj = wave; cj < nc; cj += NW) {
    const float *__restrict__ rc = rck + (size_t)cj * NC;
    float m = GS_INF;
    int g = 0;
#pragma unroll 1
    for (int q = 0; 8 * q < nc; ++q) {
      float cm = GS_INF;
#pragma unroll 1
      for (int ci = 8 * q; ci < 8 * q + 8 && ci < nc; ++ci)
        cm = __builtin_fminf(cm, cmin[ci * kWave + lane] + rc[ci]);
      chunk_update<true>(m, g, cm, q);
    }
    const uint32_t at = (uint32_t)cj * (uint32_t)pitch + (uint32_t)row;
    qd[at] = m;
    if (WITH_BP) {
      int ca = 8 * g; // first class of chunk g that attains m (the padding classes hold +inf)
#pragma unroll 1
      for (int k2 = 7; k2 >= 0; --k2)
        if (cmin[(8 * g + k2) * kWave + lane] + rc_lds[cj * NC + 8 * g + k2] == m) ca = 8 * g + k2;
      const int lo = cs_lds[ca], len = cs_lds[ca + 1] - lo;
      const float rr = rc_lds[cj * NC + ca];
      int rel = 0; // lowest member of class ca whose sum equals m
#pragma unroll 1
      for (int d = len - 1; d >= 0; --d)
        if (tile[(lo + d) * kWave + lane] + rr == m) rel = d;
      bpb[at] = (uint8_t)(lo + rel);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Several layer fronts of the class kernel per launch.
//
// A layer front of the per-launch form is one short round of workgroups, and between two
// dependent launches the chip idles for about three microseconds.  Here one launch covers
// `fronts` consecutive layer fronts, grid (instances, tiles, fronts), and a tile waits only
// for the tiles of the previous front that it depends on, so consecutive fronts overlap.
//
// Dependencies.  Tile t of front l reads the rows r - O[l-1][s] of Q[l-1], i.e. the tiles
// from (64 t - largest fitting O[l-1]) / 64 up to t of front l-1; and with `ring` plane slots
// taking turns (four; two when the problem has fewer than four planes) it overwrites rows of
// Q[l-ring] that the tiles of front l-ring+1 up to (64 t + 63 + largest fitting O[l-ring]) / 64
// still read.  Both ranges are cut to the tiles of their front that have work.  A finished tile publishes a flag word holding the number of the
// solve (a counter the context advances, so flags need no clearing between solves).
//
// Coherence.  The eight XCDs have one L2 each, and those are made coherent with each other
// only by writing back and invalidating whole caches, which costs far more than the launches
// it would save.  So an instance stays on ONE XCD: consecutive workgroups of a launch go to
// consecutive XCDs (starting at an XCD that depends on the stream's hardware queue) and the
// grid's first dimension is the batch rounded up to a multiple of 8, hence all workgroups of
// an instance run on the same XCD.  A flag
// carries the id of the XCD that wrote the rows, read from the hardware register, and a tile
// that finds a flag from another XCD raises the internal status bit instead of reading rows
// its L2 may not hold.  Within an XCD
// every compute unit's stores go through to the shared L2 (the vector cache is
// write-through), and a load that bypasses the vector cache (an agent-scope atomic load; see
// class_tile) reads what sits in that L2.  Producer: stores, wait until they are
// acknowledged, workgroup barrier, flag.  Consumer: flag seen, workgroup barrier, bypassing
// loads.
//
// Progress.  The hardware starts workgroups in the order of their linear index, so every
// workgroup of front f of a launch has been started before any of front f + 1 is, and a
// workgroup that waits does so for workgroups that are running or done: nothing waits for a
// workgroup that cannot start.  Every wait is bounded all the same; one that gives up raises
// the internal status bit (the solve then reports every instance as infeasible) and tells
// the other workgroups to stop.  The first front of a launch waits for nothing (the previous
// launch is over), the last publishes no flags.
//
// A workgroup's tile index counts from the first tile that has work (below it everything is
// +inf), so the workgroups with work come first in every front and the empty ones behind
// them leave at once.  Empty ones still cost: each has to be started, in order, before the
// next front's workgroups can be (16 ns apiece, 2.4 of a front's 7.7 us on configs[3], where
// 113 of the 257 tiles of the budget have work).  So the grid's second dimension is not the
// number of tiles but what the fronts of earlier solves of the context needed (the host
// cannot look at this solve's tables); when that is too few for some front of this solve, all
// workgroups leave at once and k_dp_class_fronts_plain does the solve (see there).
//
// Measured on MI355X, 64 fronts per launch: configs[1] 0.18 against 0.29 ms forward,
// configs[3] 0.90 against 1.22 ms.  What a flag costs (store acknowledgement, barrier, flag
// store, the poll's round trip: four to five microseconds from a tile's last store to its
// dependant's first load) is about what a launch boundary costs, so the gain comes from the
// fronts overlapping, not from a shorter hand-over.  Forms that keep workgroups resident and
// hand them (layer, instance, tile) items from atomic queues, or deal the items out
// statically, pay the same hand-over without that overlap and were slower than one launch per
// front (configs[3]: 1.6 to 1.7 ms); they are not kept.
// ---------------------------------------------------------------------------------------
constexpr int kFrontSpinMax = 1 << 18; // polls before a wait gives up
// A flag word: the number of the solve in the low 29 bits, the XCD that wrote the rows above.
constexpr int kFlagXcdShift = 29;
constexpr unsigned kFlagEpochMask = (1u << kFlagXcdShift) - 1u;
// Words of the solve counter's 256 bytes that the several-fronts form uses beside the counter
// (see Workspace::epoch): [kOverflowWord] holds the number of a solve in which some front has
// more tiles with work than the launch has workgroups for (y0 per instance and front),
// [kNeedWord] the most tiles with work of any instance and front since it was last fetched,
// [kNeedWord + 1] the count that was last handed to the host.
constexpr int kOverflowWord = 4, kNeedWord = 6;
constexpr unsigned kNeedAllTiles = 1u << 23; // stands for "one workgroup per tile"
__global__ __launch_bounds__(256) void k_class_maxfit(
    const int32_t *__restrict__ Oq, const int32_t *__restrict__ budget,
    const int32_t *__restrict__ topsum, const int32_t *__restrict__ lowsum,
    int32_t *__restrict__ maxfit, unsigned *__restrict__ stop,
    unsigned *__restrict__ epoch, unsigned *__restrict__ flags, size_t flag_words, int B, int L,
    int SP, int y0) {
  const int wave = wave_uniform(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (blockIdx.x == 0 && threadIdx.x == 0) *stop = 0;
  if (epoch[1] != 0) { // the solve counter has wrapped: no old flag may look like a new one
    for (size_t x = (size_t)blockIdx.x * 256 + threadIdx.x; x < flag_words;
         x += (size_t)gridDim.x * 256)
      flags[x] = 0u;
    if (blockIdx.x == 0 && threadIdx.x == 0) epoch[2] = 1u; // (acted on by the next solve)
  }
  const int rows = B * L;
  for (int row = (int)blockIdx.x * 4 + wave; row < rows; row += (int)gridDim.x * 4) {
    const int E = budget[row / L];
    int m = 0;
    for (int sidx = lane; sidx < SP; sidx += kWave) {
      const int v = Oq[(size_t)row * SP + sidx];
      m = (v <= E && v > m) ? v : m;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      const int other = __shfl_xor(m, d, kWave);
      m = other > m ? other : m;
    }
    if (lane == 0) {
      maxfit[row] = m;
      const int l = row % L;
      if (l >= 1) { // tiles with work of front l: see k_dp_class_fronts
        const int top = E - topsum[row];
        const int active = top >= 0 ? (top >> 6) - (lowsum[row - 1] >> 6) + 1 : 0;
        // (a thousand atomics on one word take tens of microseconds: only counts above the
        // one the host already has are collected, and every 64th solve all of them, so that
        // the host's count can come down again)
        const unsigned known = (epoch[0] & 63u) == 0u ? 0u : epoch[kNeedWord + 1];
        if (active > 0 && (unsigned)active > known) atomicMax(&epoch[kNeedWord], (unsigned)active);
        if (active > y0) epoch[kOverflowWord] = epoch[0];
      }
    }
  }
}

template <int SP, int NW, bool WITH_BP, int NC>
__global__ __launch_bounds__(NW *kWave) void k_dp_class_fronts(
    float *__restrict__ planes, size_t plane_elems, int keep, const float *__restrict__ zero_row,
    uint8_t *__restrict__ bp, size_t bp_layer_bytes, const float *__restrict__ Tq,
    const int32_t *__restrict__ Oq, const float *__restrict__ Rc,
    const int32_t *__restrict__ cmeta, const int32_t *__restrict__ cstart,
    const int32_t *__restrict__ cls, const int32_t *__restrict__ ridx,
    const int32_t *__restrict__ budget, const int32_t *__restrict__ topsum,
    const int32_t *__restrict__ lowsum, const int32_t *__restrict__ maxfit,
    unsigned *__restrict__ flags, unsigned *__restrict__ stop,
    const unsigned *__restrict__ epoch_word, int32_t *__restrict__ status, int B, int L, int Sc,
    int pitch, int tiles, int l0, int spin_max, int publish, int ring) {
  // (the dynamic part follows the static one: keep it 16-byte aligned for its float4 accesses)
  extern __shared__ __align__(16) float lds[];
  __shared__ __align__(16) int s_go4[4];
  int &s_go = s_go4[0];
  const int b = (int)blockIdx.x;
  if (b >= B) return;
  const int f = (int)blockIdx.z;
  const int l = l0 + f;
  const int bl = b * L + l;
  const unsigned epoch = epoch_word[0]; // number of this solve (the prepare step advanced it)
  // (some front has more tiles with work than gridDim.y: k_dp_class_fronts_plain takes the solve)
  if (epoch_word[kOverflowWord] == epoch) return;
  // the tile's table entries travel while wave 0 waits for the tiles below
  const ClassScalars<SP / NW> k =
      class_scalars<SP, NW, ((WITH_BP || SP / NW > 12) && SP / NW <= 16)>(Tq, Oq, cmeta, cls, ridx,
                                                                       budget, topsum, lowsum, L, l, b);
  const int E = k.E;
  const int a = k.low >> 6;                    // first tile with work
  const int top = E - k.mo;                    // last source row with work
  const int t = a + (int)blockIdx.y;
  if (t * kWave > top) return;
  const int wave = wave_uniform(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  unsigned xcc;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
  xcc &= 7u;
  // (what the tile needs in LDS beside its rows is laid out while wave 0 waits; with eight
  // waves the other seven do it and wave 0 polls at once, with four it takes its share first:
  // measured both ways)
  if constexpr (NW >= 8) {
    if (wave != 0)
      class_tile_prepare<SP, NW, WITH_BP, NC>(Rc, cstart, k.kr, lds, (int)threadIdx.x - kWave,
                                              (NW - 1) * kWave);
  } else {
    class_tile_prepare<SP, NW, WITH_BP, NC>(Rc, cstart, k.kr, lds, (int)threadIdx.x, NW * kWave);
  }
  if (wave == 0) {
    int go = 1;
    if (f > 0) {
      // Tiles of front l-1 that this one reads (rows r - O[l-1][s]), up to its own index.
      // And with `ring` planes taking turns it overwrites rows of Q[l-ring], which the tiles
      // above it of front l-ring+1 may still be reading (up to the largest shift O[l-ring][s]
      // that fits): it waits for those as well, unless that front belongs to an earlier
      // launch.  With four planes that front is three behind and long done; with two it is
      // the front before, whose upper tiles start late.
      const int top1 = E - topsum[bl - 1];
      const int a1 = lowsum[bl - 2] >> 6;
      const int z1 = top1 >= 0 ? top1 >> 6 : -1;
      int lo = kWave * t - maxfit[bl - 1];
      lo = lo > 0 ? lo >> 6 : 0;
      lo = lo > a1 ? lo : a1;
      const int hi1 = t < z1 ? t : z1;
      int hiw = -1;
      const int lw = l - ring + 1; // the front that reads the plane this one overwrites
      if (!keep && lw >= 2 && f >= ring - 1) {
        const int war = (kWave * t + 63 + maxfit[bl - ring]) >> 6;
        const int topw = E - topsum[bl - ring + 1];
        const int zw = topw >= 0 ? topw >> 6 : -1;
        hiw = war < zw ? war : zw;
      }
      const int hi = hi1 > hiw ? hi1 : hiw;
      // (flag words are counted in 32 bits: there are fewer than 2^26 of them)
      const int row1 = ((l - 1) * B + b) * tiles, roww = (lw * B + b) * tiles;
      int spins = 0;
      for (int base = lo; base <= hi && go; base += kWave) {
        for (;;) {
          const int at = base + lane;
          unsigned fv = epoch | (xcc << kFlagXcdShift);
          const int word = at <= hi1 ? row1 + at : (at > t && at <= hiw ? roww + at : -1);
          if (word >= 0)
            fv = __hip_atomic_load(&flags[word], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (__builtin_amdgcn_ballot_w64((fv & kFlagEpochMask) != epoch) == 0) {
            // all there: were they written on this XCD (else its L2 may not hold the rows)?
            if (__builtin_amdgcn_ballot_w64((fv >> kFlagXcdShift) != xcc) != 0) {
              __hip_atomic_store(stop, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              __hip_atomic_fetch_or(status, 0x40, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              go = 0;
            }
            break;
          }
          ++spins;
          if ((spins & 255) == 0) { // now and then: has somebody given up?
            const unsigned st = __hip_atomic_load(stop, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (wave_uniform((int)st) != 0) { go = 0; break; }
          }
          if (spins > spin_max) { // gave up: the forward pass is incomplete
            __hip_atomic_store(stop, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_fetch_or(status, 0x40, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            go = 0;
            break;
          }
          __builtin_amdgcn_s_sleep(2);
        }
      }
    }
    s_go = go;
  }
  __syncthreads();
  if (wave_uniform(s_go) == 0) return;
  const int srci = keep ? l - 1 : ((l - 1) & (ring - 1)), dsti = keep ? l : (l & (ring - 1));
  const bool from_zero = !keep && l == 1; // Q[0] = 0 is one shared row of zeros
  const float *__restrict__ qsrc = from_zero ? zero_row : planes + (size_t)srci * plane_elems;
  float *__restrict__ qdst = planes + (size_t)dsti * plane_elems;
  uint8_t *__restrict__ bp_l = WITH_BP ? bp + (size_t)(l - 1) * bp_layer_bytes : nullptr;
  // As soon as the tile's rows of Q[l] are stored (before its backpointers are worked out) the
  // tiles of the next front that depend on it may go ahead.
  const bool announce = f + 1 < (int)gridDim.z && publish;
  auto publish_flag = [&]() {
    if (announce) {
      // the rows are in the XCD's L2 once the stores are acknowledged; then the flag
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (wave == 0)
        __hip_atomic_store(&flags[((size_t)l * B + b) * tiles + t],
                           epoch | (xcc << kFlagXcdShift), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
  };
  class_tile<SP, NW, WITH_BP, NC, true, NoHook, true>(k, qsrc, qdst, bp_l, Rc, cstart, Sc, pitch,
                                                      from_zero ? 0 : pitch, b, t * kWave, lds,
                                                      NoHook(), publish_flag);
}

// The same forward pass the plain way, for the rare solve in which a front has more tiles with
// work than k_dp_class_fronts was given workgroups for (that kernel's workgroups then leave at
// once; the host sizes its grid by what earlier solves needed, and must not wait to learn what
// this one needs).  One launch for all fronts: gridDim.y workgroups per instance, all of them
// resident at once (the launcher sees to that), each taking every gridDim.y-th tile of front
// 1, then of front 2, and so on, with the same flags between dependent tiles.  Many times
// slower; the next solve of the context has a grid that fits.  Always launched: its first
// thread hands the host the most tiles any front of this solve needed (`hint`, in host memory
// that the device can write) and clears the count.
template <int SP, int NW, bool WITH_BP, int NC>
__global__ __launch_bounds__(NW *kWave) void k_dp_class_fronts_plain(
    float *__restrict__ planes, size_t plane_elems, int keep, const float *__restrict__ zero_row,
    uint8_t *__restrict__ bp, size_t bp_layer_bytes, const float *__restrict__ Tq,
    const int32_t *__restrict__ Oq, const float *__restrict__ Rc,
    const int32_t *__restrict__ cmeta, const int32_t *__restrict__ cstart,
    const int32_t *__restrict__ cls, const int32_t *__restrict__ ridx,
    const int32_t *__restrict__ budget, const int32_t *__restrict__ topsum,
    const int32_t *__restrict__ lowsum, const int32_t *__restrict__ maxfit,
    unsigned *__restrict__ flags, unsigned *__restrict__ stop, unsigned *__restrict__ epoch_word,
    int32_t *__restrict__ status, unsigned *__restrict__ hint, int B, int L, int Sc, int pitch,
    int tiles, int spin_max, int ring) {
  extern __shared__ __align__(16) float lds[];
  __shared__ __align__(16) int s_go4[4];
  int &s_go = s_go4[0];
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
    // (k_class_maxfit collects the counts above the one handed over last, and all of them
    // every 64th solve: see there)
    // A solve that did not fit sends the host back to one workgroup per tile (a count beyond
    // any number of tiles) until the next solve in which all counts are collected: at most one
    // slow solve in 64, however the budgets move.
    unsigned need = epoch_word[kNeedWord];
    const unsigned known = epoch_word[kNeedWord + 1];
    const bool all = (epoch_word[0] & 63u) == 0u;
    if (epoch_word[kOverflowWord] == epoch_word[0]) need = kNeedAllTiles;
    if (hint && need != 0u && (all ? need != known : need > known)) {
      *hint = need;
      epoch_word[kNeedWord + 1] = need;
    }
    epoch_word[kNeedWord] = 0u;
  }
  const int b = (int)blockIdx.x;
  if (b >= B) return;
  const unsigned epoch = epoch_word[0];
  if (epoch_word[kOverflowWord] != epoch) return;
  const int wave = wave_uniform(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  unsigned xcc;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
  xcc &= 7u;
  const unsigned want = epoch | (xcc << kFlagXcdShift);
  const int E = budget[b];
  const int nc = cmeta[0];
#pragma unroll 1
  for (int l = 1; l < L; ++l) {
    const int bl = b * L + l;
    const int low = lowsum[bl - 1], lowq = l >= 2 ? lowsum[bl - 2] : 0;
    const int top = E - topsum[bl];
    const int kr = ridx[bl];
    const int srci = keep ? l - 1 : ((l - 1) & (ring - 1)), dsti = keep ? l : (l & (ring - 1));
    const bool from_zero = !keep && l == 1;
    const float *__restrict__ qsrc = from_zero ? zero_row : planes + (size_t)srci * plane_elems;
    float *__restrict__ qdst = planes + (size_t)dsti * plane_elems;
    uint8_t *__restrict__ bp_l = WITH_BP ? bp + (size_t)(l - 1) * bp_layer_bytes : nullptr;
#pragma unroll 1
    for (int t = (low >> 6) + (int)blockIdx.y; t * kWave <= top; t += (int)gridDim.y) {
      class_tile_prepare<SP, NW, WITH_BP, NC>(Rc, cstart, kr, lds, (int)threadIdx.x, NW * kWave);
      if (wave == 0) {
        int go = 1;
        if (l >= 2) { // (the same two ranges of tiles as in k_dp_class_fronts)
          const int top1 = E - topsum[bl - 1];
          const int a1 = lowsum[bl - 2] >> 6;
          const int z1 = top1 >= 0 ? top1 >> 6 : -1;
          int lo = kWave * t - maxfit[bl - 1];
          lo = lo > 0 ? lo >> 6 : 0;
          lo = lo > a1 ? lo : a1;
          const int hi1 = t < z1 ? t : z1;
          int hiw = -1;
          const int lw = l - ring + 1;
          if (!keep && lw >= 2) {
            const int war = (kWave * t + 63 + maxfit[bl - ring]) >> 6;
            const int topw = E - topsum[bl - ring + 1];
            const int zw = topw >= 0 ? topw >> 6 : -1;
            hiw = war < zw ? war : zw;
          }
          const int hi = hi1 > hiw ? hi1 : hiw;
          const int row1 = ((l - 1) * B + b) * tiles, roww = (lw * B + b) * tiles;
          int spins = 0;
          for (int base = lo; base <= hi && go; base += kWave) {
            for (;;) {
              const int at = base + lane;
              unsigned fv = want;
              const int word = at <= hi1 ? row1 + at : (at > t && at <= hiw ? roww + at : -1);
              if (word >= 0)
                fv = __hip_atomic_load(&flags[word], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              if (__builtin_amdgcn_ballot_w64(fv != want) == 0) break;
              ++spins;
              if ((spins & 255) == 0) {
                const unsigned st = __hip_atomic_load(stop, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (wave_uniform((int)st) != 0) { go = 0; break; }
              }
              if (spins > spin_max) { // gave up (also: a flag from another XCD never matches)
                __hip_atomic_store(stop, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_fetch_or(status, 0x40, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                go = 0;
                break;
              }
              __builtin_amdgcn_s_sleep(2);
            }
          }
        }
        s_go = go;
      }
      __syncthreads();
      if (wave_uniform(s_go) == 0) return;
      class_tile_plain<SP, NW, WITH_BP, NC>(qsrc, qdst, bp_l, Tq, Oq, cls, Rc, bl, kr, nc, E, lowq,
                                            Sc, pitch, from_zero ? 0 : pitch, b, t * kWave, lds);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads(); // (also: the next tile reuses the LDS)
      if (threadIdx.x == 0)
        __hip_atomic_store(&flags[((size_t)l * B + b) * tiles + t], want, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

__global__ __launch_bounds__(256) void k_zero_plane(float *__restrict__ q, size_t n) {
  for (size_t x = (size_t)blockIdx.x * 256 + threadIdx.x; x < n; x += (size_t)gridDim.x * 256)
    q[x] = 0.0f;
}

// Shape-agnostic "pull" form: a lane owns one TARGET row e and, for each sj, scans the
// previous plane at row e - O[l][sj] straight from global memory.  Any S up to the
// library limit, uint8 or uint16 backpointers.  Slow (one load per relaxation); it is the
// fallback for S above the register-tiled sizes and an independent second implementation.
template <typename BPT, bool WITH_BP>
__global__ __launch_bounds__(kRowsPerBlock) void k_dp_generic(
    const float *__restrict__ src, float *__restrict__ dst, BPT *__restrict__ bp,
    const float *__restrict__ Tq, const int32_t *__restrict__ Oq,
    const float *__restrict__ Rt, const int32_t *__restrict__ ridx,
    const int32_t *__restrict__ budget, int B, int L, int S, int SP, int l, int pitch) {
  const int b = blockIdx.x % B;
  const int row = (blockIdx.x / B) * kRowsPerBlock + threadIdx.x;
  const int E = budget[b];
  if (row > E) return;
  const int bl = b * L + l;
  const size_t plane_off = (size_t)b * S * pitch;
  const float *__restrict__ srcb = src + plane_off;
  const float *__restrict__ rk = Rt + (size_t)ridx[bl] * SP * SP;
  for (int j = 0; j < S; ++j) {
    const int o = Oq[(size_t)bl * SP + j];
    float out = GS_INF;
    int arg = 0;
    if (row >= o) {
      const int srow = row - o;
      const float *__restrict__ rc = rk + (size_t)j * SP;
      float m = GS_INF;
      for (int i = 0; i < S; ++i) {
        const float v = srcb[(size_t)i * pitch + srow] + rc[i];
        if (v < m) { m = v; arg = i; }
      }
      out = m + Tq[(size_t)bl * SP + j];
    }
    dst[plane_off + (size_t)j * pitch + row] = out;
    if (WITH_BP) bp[plane_off + (size_t)j * pitch + row] = (BPT)arg;
  }
}

// ---------------------------------------------------------------------------------------
// Whole forward pass of a SMALL instance in one launch (latency path).
//
// One workgroup per instance runs layer 0 .. L-1 back to back; the two ping-pong planes
// live in LDS ([s][e], pitch a multiple of 64), so a layer front costs one workgroup
// barrier instead of a kernel launch.  The transition pool and the instance's T, O and
// r_index rows are copied to LDS first, so that no layer waits for a chain of scalar loads.
// Threads are laid out as (budget row) x (group of target strategies).  A thread owns a
// SOURCE row e' ("push" form): it reads C[l-1][e'][.] from LDS once per layer, scans it
// against the staged column of every target sj of its group (all lanes of a wave share sj,
// so those are broadcast LDS reads), and stores the result at row e' + O[l][sj] of the next
// plane; the rows e < O[l][sj], which no source row reaches, are filled with +inf by the
// thread that owns that row.  Every row 0..E of every target is written exactly once.
// Flat strict-"<" scan, four candidates at a time up to S; backpointers go to HBM as in the
// other kernels.  The last plane (or every plane when all are kept) is copied to the HBM
// workspace so that the final reductions, the budget curve and the plane-based backtrace
// read what they always read.
// ---------------------------------------------------------------------------------------
template <int SP>
__global__ __launch_bounds__(1024) void k_dp_small(
    float *__restrict__ planes, uint8_t *__restrict__ bp, const float *__restrict__ Tq,
    const int32_t *__restrict__ Oq, const float *__restrict__ Rt,
    const int32_t *__restrict__ ridx, const int32_t *__restrict__ budget, int B, int L, int S,
    int K, int pitch, int keep_all, int last_plane) {
  extern __shared__ float lds[]; // two planes of S * pitch floats, then the staged tables
  const int b = blockIdx.x;
  float *Rl = lds + (size_t)2 * S * pitch;               // [K][SP][SP]
  float *Tl = Rl + (size_t)K * SP * SP;                  // [L][SP]
  int *Ol = reinterpret_cast<int *>(Tl + (size_t)L * SP); // [L][SP]
  int *kl = Ol + (size_t)L * SP;                         // [L]
  for (int x = threadIdx.x; x < K * SP * SP; x += blockDim.x) Rl[x] = Rt[x];
  for (int x = threadIdx.x; x < L * SP; x += blockDim.x) {
    Tl[x] = Tq[(size_t)b * L * SP + x];
    Ol[x] = Oq[(size_t)b * L * SP + x];
  }
  for (int x = threadIdx.x; x < L; x += blockDim.x) kl[x] = ridx[(size_t)b * L + x];
  __syncthreads();
  const int E = budget[b];
  const int rows64 = (E + 1 + kWave - 1) / kWave * kWave; // threads along e
  const int groups = (int)blockDim.x / rows64;             // >= 1 by the launch condition
  const int e = (int)threadIdx.x % rows64;
  const int jg = (int)threadIdx.x / rows64;
  const bool active = jg < groups && e <= E;
  const size_t plane_elems_all = (size_t)B * S * pitch;
  const size_t plane_off = (size_t)b * S * pitch;
  float *cur = lds;
  float *nxt = lds + (size_t)S * pitch;

  if (active)
    for (int s0 = jg; s0 < S; s0 += groups) {
      const float v = (e >= Ol[s0]) ? Tl[s0] : GS_INF;
      cur[s0 * pitch + e] = v;
      if (keep_all || L == 1) planes[plane_off + (size_t)s0 * pitch + e] = v;
    }
  for (int l = 1; l < L; ++l) {
    __syncthreads();
    const float *rk = Rl + (size_t)kl[l] * SP * SP;
    float *gplane = planes + (keep_all ? (size_t)l * plane_elems_all : (size_t)last_plane * plane_elems_all) + plane_off;
    uint8_t *gbp = bp ? bp + (size_t)(l - 1) * plane_elems_all + plane_off : nullptr;
    const bool to_global = keep_all || l == L - 1;
    if (active) {
      float c[SP];
#pragma unroll
      for (int i = 0; i < SP; ++i) c[i] = i < S ? cur[i * pitch + e] : GS_INF;
      for (int j = jg; j < S; j += groups) {
        const int o = Ol[l * SP + j];
        const float t = Tl[l * SP + j];
        const float *rc = rk + (size_t)j * SP;
        float m = GS_INF;
        int arg = 0;
#pragma unroll
        for (int i0 = 0; i0 < SP; i0 += 4) {
          if (i0 < S) { // uniform: whole chunks of padding are skipped
            const float4 r = *reinterpret_cast<const float4 *>(rc + i0);
            const float rr[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              const float v = c[i0 + k] + rr[k];
              if (v < m) { m = v; arg = i0 + k; }
            }
          }
        }
        const int eo = e + o;
        if (eo <= E) {
          const float out = m + t;
          nxt[j * pitch + eo] = out;
          if (to_global) gplane[(size_t)j * pitch + eo] = out;
          if (gbp) gbp[(size_t)j * pitch + eo] = (uint8_t)arg;
        }
        if (e < o) { // no source row reaches this target row
          nxt[j * pitch + e] = GS_INF;
          if (to_global) gplane[(size_t)j * pitch + e] = GS_INF;
          if (gbp) gbp[(size_t)j * pitch + e] = 0;
        }
      }
    }
    float *tmp = cur; cur = nxt; nxt = tmp;
  }
}

// LDS bytes of the staged tables: transition pool, T and O rows, r_index row
static size_t small_table_bytes(const Shape &s) {
  return sizeof(float) * ((size_t)s.K * s.SP * s.SP + (size_t)2 * s.L * s.SP + (size_t)s.L);
}

// The latency path applies when an instance's budget rows fit one workgroup, its two planes
// fit LDS, and the batch is too small to fill the GPU through the per-layer kernels anyway.
bool small_path_applies(const Shape &s, bool with_bp) {
  if (s.M + 1 > 1024 || s.SP > 32) return false;
  if ((size_t)2 * s.S * s.pitch * sizeof(float) > (size_t)96 * 1024) return false;
  if (small_table_bytes(s) > (size_t)48 * 1024) return false;
  const long long tiles = (long long)((s.M + 1 + kWave - 1) / kWave) * s.B;
  if (tiles > 2048) return false;
  // One workgroup per instance means one compute unit per instance, so the one-launch kernel
  // wins only while a thread's share of a layer front is short.  A thread owns a budget row
  // and every groups-th target strategy: per = ceil(S / groups) scans of S candidates, and
  // the workgroup's waves share one compute unit.  Measured per layer (24 layers, 1 and 64
  // instances, S = 8..44, M = 64..1000), in microseconds:
  //   one launch  0.9 + 0.0021 * per * S * max(waves, 14)
  //   tile kernel 1.6 + 0.18 S per launch with backpointers, 1.5 + 0.13 S without
  // e.g. S = 12, M = 256 (per = 4, 15 waves): 62 us against 88 (77 min-only) for 23 fronts;
  // S = 8, M = 512: 66 against 74; S = 24, M = 128: 100 against 123 (100); S = 32, M = 64: 121
  // against 157 (124); S = 16, M = 512: 185 against 105.  The knob "small" = 0 / 1 (tuning)
  // switches the path off / on wherever it fits.
  const int forced = s.tune.small;
  if (forced == 0 || forced == 1) return forced == 1;
  const int rows64 = (s.M + 1 + kWave - 1) / kWave * kWave;
  const int groups = s.S < 1024 / rows64 ? s.S : 1024 / rows64;
  const int per = (s.S + groups - 1) / groups;
  const int waves = groups * rows64 / kWave;
  const double one_launch = 0.9 + 0.0021 * per * s.S * (waves > 14 ? waves : 14);
  const double per_front = with_bp ? 1.6 + 0.18 * s.S : 1.5 + 0.13 * s.S;
  return one_launch <= per_front;
}

// More than 64 KB of dynamic LDS per workgroup has to be asked for, per kernel: the context's
// record remembers the largest size already asked for.
static void lds_opt_in(const void *kernel, size_t lds, LdsGrants *g) {
  int at = -1;
  for (int i = 0; g && i < g->n; ++i)
    if (g->fn[i] == kernel) at = i;
  if (at >= 0 && lds <= g->bytes[at]) return;
  (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (!g) return;
  if (at < 0 && g->n < LdsGrants::kMax) at = g->n++;
  if (at >= 0) { // (a full record only means asking again next time)
    g->fn[at] = kernel;
    g->bytes[at] = lds;
  }
}

void launch_dp_small(const Shape &s, const Workspace &w, bool keep_all, int last_plane,
                     hipStream_t st) {
  const size_t lds = (size_t)2 * s.S * s.pitch * sizeof(float) + small_table_bytes(s);
  const int rows64 = (s.M + 1 + kWave - 1) / kWave * kWave;
  int threads = (1024 / rows64) * rows64; // whole groups of target strategies
  const int useful = ((s.S < 1024 / rows64) ? s.S : 1024 / rows64) * rows64;
  if (useful < threads) threads = useful;
#define GS_SMALL(SPV)                                                                     \
  do {                                                                                    \
    if (lds > 64 * 1024) lds_opt_in((const void *)k_dp_small<SPV>, lds, s.grants);        \
    hipLaunchKernelGGL((k_dp_small<SPV>), dim3(s.B), dim3(threads), lds, st, w.planes,    \
                       (uint8_t *)w.bp, w.Tq, w.Oq, w.Rt, w.ridx, w.budget, s.B, s.L, s.S, \
                       s.K, s.pitch, keep_all ? 1 : 0, last_plane);                       \
  } while (0)
  switch (s.SP) { // small_path_applies() admits no other size
    case 8: GS_SMALL(8); break;
    case 16: GS_SMALL(16); break;
    case 24: GS_SMALL(24); break;
    case 32: GS_SMALL(32); break;
    default: break;
  }
#undef GS_SMALL
}

int tuned_sp_for(int S) {
  static const int sizes[] = {8, 16, 24, 32, 48, 64, 96, 128};
  for (int v : sizes)
    if (S <= v) return v;
  return 0;
}

// The class kernel keeps only its own share of the strategies per wave, so it also exists
// for 192 and 256 padded strategies (129..256 strategies: the paper's strategy space on 256
// and 512 devices), where the general path is left with the pull-form fallback.
int class_sp_for(int S) {
  const int t = tuned_sp_for(S);
  if (t) return t;
  return S <= 192 ? 192 : (S <= 256 ? 256 : 0);
}

// Launch shape of the register-tiled kernel.  Work is cut into (64-row tile) x (slice of
// target strategies) pieces, one per wave; slicing the strategies costs a repeated load
// of the tile's source values but multiplies the number of waves, which is what hides
// the scalar-load latency when a batch has few tiles (8 instances x 257 tiles fill the
// 1024 SIMDs only twice).  the knobs "jsplit" and "waves_per_block" override the
// heuristic (debugging and tuning aid).
static void push_launch_shape(const Shape &s, int &jsplit, int &wpb) {
  const Tuning &tune = s.tune;
  // tiles of this launch alone, also when other groups of the batch run beside it on
  // parallel streams: measured, the finer split is what lets the groups interleave
  const long long tiles = (long long)((s.M + 1 + kWave - 1) / kWave) * s.B;
  wpb = tune.waves_per_block >= 1 && tune.waves_per_block <= 4 ? tune.waves_per_block : 4;
  jsplit = tune.jsplit;
  if (jsplit < 1) {
    jsplit = 1;
    while (tiles * jsplit < 4096 && jsplit < 8 && s.S / (jsplit * 2) >= 8) jsplit *= 2;
  }
  if (jsplit > s.S) jsplit = s.S;
}

template <int SP, int NW, int SA>
static void launch_tile_sa(const Shape &s, const Workspace &w, int l, const float *src,
                           float *dst, void *bp_l, hipStream_t st) {
  const long long tiles = (s.M + 1 + kWave - 1) / kWave;
  const dim3 grid((unsigned)(tiles * s.B)), block(NW * kWave);
  const size_t lds = sizeof(float) * SP * kWave;
  if (bp_l)
    hipLaunchKernelGGL((k_dp_tile<SP, NW, true, SA>), grid, block, lds, st, src, dst,
                       (uint8_t *)bp_l, w.Tq, w.Oq, w.Rt, w.ridx, w.budget, w.topsum, w.lowsum, s.B, s.L,
                       s.S, l, s.pitch);
  else
    hipLaunchKernelGGL((k_dp_tile<SP, NW, false, SA>), grid, block, lds, st, src, dst,
                       (uint8_t *)nullptr, w.Tq, w.Oq, w.Rt, w.ridx, w.budget, w.topsum, w.lowsum, s.B,
                       s.L, s.S, l, s.pitch);
}

template <int SP, int NW>
static void launch_tile_nw(const Shape &s, const Workspace &w, int l, const float *src,
                           float *dst, void *bp_l, hipStream_t st) {
  // the half-chunk variant exists for 48 padded strategies (S = 41..44) only
  if constexpr (SP == 48) {
    if (s.S <= SP - 4) return launch_tile_sa<SP, NW, SP - 4>(s, w, l, src, dst, bp_l, st);
  }
  launch_tile_sa<SP, NW, SP>(s, w, l, src, dst, bp_l, st);
}

template <int SP>
static void launch_tile(const Shape &s, const Workspace &w, int l, const float *src, float *dst,
                        void *bp_l, int waves, hipStream_t st) {
  if (waves >= 4) launch_tile_nw<SP, 4>(s, w, l, src, dst, bp_l, st);
  else if (waves >= 2) launch_tile_nw<SP, 2>(s, w, l, src, dst, bp_l, st);
  else launch_tile_nw<SP, 1>(s, w, l, src, dst, bp_l, st);
}

template <int SP, int RU>
static void launch_push_ru(const Shape &s, const Workspace &w, int l, const float *src,
                           float *dst, void *bp_l, int jsplit, int wpb, hipStream_t st) {
  const int rows = wpb * kWave * RU;
  const long long row_blocks = (s.M + 1 + rows - 1) / rows;
  const long long nblk = row_blocks * s.B;
  const dim3 grid((unsigned)((nblk + 7) / 8 * 8 * jsplit)), block(wpb * kWave);
  if (bp_l)
    hipLaunchKernelGGL((k_dp_push<SP, RU, true>), grid, block, 0, st, src, dst, (uint8_t *)bp_l,
                       w.Tq, w.Oq, w.Rt, w.ridx, w.budget, w.topsum, w.lowsum, s.B, s.L, s.S, l, s.pitch,
                       jsplit, (int)nblk);
  else
    hipLaunchKernelGGL((k_dp_push<SP, RU, false>), grid, block, 0, st, src, dst,
                       (uint8_t *)nullptr, w.Tq, w.Oq, w.Rt, w.ridx, w.budget, w.topsum, w.lowsum, s.B,
                       s.L, s.S, l, s.pitch, jsplit, (int)nblk);
}

template <int SP>
static void launch_push(const Shape &s, const Workspace &w, int l, const float *src, float *dst,
                        void *bp_l, hipStream_t st) {
  int jsplit, wpb;
  push_launch_shape(s, jsplit, wpb);
  // Row groups per wave.  Measured: they pay only for the min-only pass (5 % on the outer
  // search batch), where the shared scalar loads and loop overhead are a large part of a
  // short column; the flat argmin is bound by its own instruction count either way and
  // loses occupancy to the extra registers.  Used while the batch still yields at least
  // eight waves per SIMD.  The knob "row_groups" overrides.
  const long long tiles = (long long)((s.M + 1 + kWave - 1) / kWave) * s.Bc * jsplit;
  int ru = s.tune.row_groups;
  if (ru < 1) ru = bp_l ? 1 : (tiles >= 4 * 8192 ? 4 : (tiles >= 2 * 8192 ? 2 : 1));
  if constexpr (SP <= 24) {
    if (ru >= 4) return launch_push_ru<SP, 4>(s, w, l, src, dst, bp_l, jsplit, wpb, st);
  }
  if constexpr (SP <= 48) {
    if (ru >= 2) return launch_push_ru<SP, 2>(s, w, l, src, dst, bp_l, jsplit, wpb, st);
  }
  launch_push_ru<SP, 1>(s, w, l, src, dst, bp_l, jsplit, wpb, st);
}

bool class_path_applies(const Shape &s) {
  const int tsp = class_sp_for(s.S);
  // the kernel addresses an instance's plane with 32-bit offsets and numbers its
  // workgroups (8 * tiles per XCD) with 32 bits
  return tsp >= 16 && tsp == s.SP && !s.bp16 && (size_t)s.S * s.pitch < ((size_t)1 << 31) &&
         (size_t)class_rows(s) * s.pitch * 4 < ((size_t)1 << 31) &&
         (s.M + kWave) / kWave <= 65535 && (long long)((s.M + kWave) / kWave) * s.B < (1ll << 30);
}

template <int SP, int NW, int NC>
static void launch_class_nc(const Shape &s, const Workspace &w, int l, const float *src,
                            float *dst, void *bp_l, hipStream_t st) {
  const long long tiles = (s.M + 1 + kWave - 1) / kWave;
  // see the kernel's workgroup numbering: (instances, tiles) grid for a multiple of 8
  // instances (and for one-tile instances), else 8 contiguous runs of tiles
  const bool by_instance = s.B % 8 == 0 || tiles == 1;
  const long long per_xcd = (tiles * s.B + 7) / 8;
  // x / tiles = mulhi(x, magic) >> shift for every x < 2^31: magic = ceil(2^p / tiles) with
  // p = 31 + ceil(log2 tiles) (tiles >= 2)
  int lg = 0;
  while ((1ll << lg) < tiles) ++lg;
  const int p = 31 + lg;
  const unsigned div_magic = (unsigned)((((unsigned long long)1 << p) + tiles - 1) / tiles);
  const int div_shift = p - 32 > 0 ? p - 32 : 0;
  const dim3 grid = by_instance ? dim3((unsigned)s.B, (unsigned)tiles) : dim3((unsigned)(8 * per_xcd));
  const dim3 block(NW * kWave);
  const int src_pitch = src == w.zero_row ? 0 : s.pitch; // the shared row of zeros stands for Q[0]
  const size_t lds = sizeof(float) * ((bp_l ? (SP + 3) * kWave : 0) + NC * kWave + NC * NC + NC + 32);
  // (the forms with backpointers from 128 (wide) or 192 strategies up)
  if (lds > 64 * 1024) lds_opt_in((const void *)k_dp_class<SP, NW, true, NC>, lds, s.grants);
  if (bp_l)
    hipLaunchKernelGGL((k_dp_class<SP, NW, true, NC>), grid, block, lds, st, src, dst,
                       (uint8_t *)bp_l, w.Tq, w.Oq, w.Rc, w.cmeta, w.cstart, w.cls, w.ridx,
                       w.budget, w.topsum, w.lowsum, s.B, s.L, class_rows(s), l, s.pitch, src_pitch, (int)tiles,
                       div_magic, div_shift);
  else
    hipLaunchKernelGGL((k_dp_class<SP, NW, false, NC>), grid, block, lds, st, src, dst,
                       (uint8_t *)nullptr, w.Tq, w.Oq, w.Rc, w.cmeta, w.cstart, w.cls, w.ridx,
                       w.budget, w.topsum, w.lowsum, s.B, s.L, class_rows(s), l, s.pitch, src_pitch, (int)tiles,
                       div_magic, div_shift);
}

template <int SP, int NW>
static void launch_class_nw(const Shape &s, const Workspace &w, int l, const float *src,
                            float *dst, void *bp_l, hipStream_t st) {
  // more than 32 classes need more than 32 strategies: the wide variant exists from 48 up
  if constexpr (SP >= 48) {
    if (s.NC > 32) return launch_class_nc<SP, NW, 64>(s, w, l, src, dst, bp_l, st);
  }
  if (s.NC <= 16) return launch_class_nc<SP, NW, 16>(s, w, l, src, dst, bp_l, st);
  launch_class_nc<SP, NW, 32>(s, w, l, src, dst, bp_l, st);
}

template <int SP>
static void launch_class(const Shape &s, const Workspace &w, int l, const float *src, float *dst,
                         void *bp_l, hipStream_t st) {
  // Waves per tile, measured over S = 16..128 and 64..33 K tiles: eight while the batch is
  // a few hundred tiles (pure latency); otherwise eight from 64 padded strategies up with
  // backpointers and at 128 without (a wave's share of the tile is long enough to pay for
  // the per-wave set-up), four below; the min-only pass takes eight at 96 while the batch
  // is a few thousand tiles and two up to 32 strategies.  The knob "jsplit" overrides.
  const long long tile_inst = (long long)((s.M + kWave) / kWave) * s.Bc;
  int waves = s.tune.jsplit;
  if (waves < 1 || waves > 8) {
    if (tile_inst <= 512) waves = 8;
    else if (bp_l) waves = SP >= 64 ? 8 : 4;
    else waves = SP >= 128 ? 8 : (SP >= 96 ? (tile_inst <= 4096 ? 8 : 4) : (SP <= 32 ? 2 : 4));
  }
  if constexpr (SP > 128) { // a wave's share of the strategies has to stay in registers
    launch_class_nw<SP, 8>(s, w, l, src, dst, bp_l, st);
  } else {
    if (waves >= 8) launch_class_nw<SP, 8>(s, w, l, src, dst, bp_l, st);
    else if (waves >= 4) launch_class_nw<SP, 4>(s, w, l, src, dst, bp_l, st);
    else if (waves >= 2) launch_class_nw<SP, 2>(s, w, l, src, dst, bp_l, st);
    else launch_class_nw<SP, 1>(s, w, l, src, dst, bp_l, st);
  }
}

const char *launch_dp_class(const Shape &s, const Workspace &w, int l, const float *src,
                            float *dst, void *bp_l, hipStream_t st) {
  switch (s.SP) {
    case 16: launch_class<16>(s, w, l, src, dst, bp_l, st); break;
    case 24: launch_class<24>(s, w, l, src, dst, bp_l, st); break;
    case 32: launch_class<32>(s, w, l, src, dst, bp_l, st); break;
    case 48: launch_class<48>(s, w, l, src, dst, bp_l, st); break;
    case 64: launch_class<64>(s, w, l, src, dst, bp_l, st); break;
    case 96: launch_class<96>(s, w, l, src, dst, bp_l, st); break;
    case 128: launch_class<128>(s, w, l, src, dst, bp_l, st); break;
    case 192: launch_class<192>(s, w, l, src, dst, bp_l, st); break;
    case 256: launch_class<256>(s, w, l, src, dst, bp_l, st); break;
    default: break; // class_path_applies() admits no other pitch
  }
  return "k_dp_class";
}

// Which XCD each workgroup of a small grid runs on: out[i] = XCD id of workgroup i.
__global__ void k_xcc_probe(unsigned *__restrict__ out) {
  unsigned xcc;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
  if (threadIdx.x == 0) out[blockIdx.x] = xcc & 15u;
}

void launch_xcc_probe(unsigned *out, hipStream_t st) {
  hipLaunchKernelGGL(k_xcc_probe, dim3(kXccProbeGrid), dim3(kWave), 0, st, out);
}

// (a batch that is not a multiple of 8 leaves some XCDs one instance short: taken from 64
// instances up, where that is at most an eighth)
bool fronts_shape_ok(const Shape &s) {
  return s.L >= 3 && (s.B % 8 == 0 || s.B >= 64) &&
         (long long)(s.B + 7) * ((s.M + kWave) / kWave) < (1ll << 22);
}

template <int SP, int NW, int NC>
static void launch_fronts_nc(const Shape &s, const Workspace &w, bool keep, bool with_bp,
                             size_t plane_elems_all, size_t bp_layer_bytes, int fronts, int ring,
                             int front_y0, unsigned *hint, int resident_wgs, hipStream_t st) {
  const int tiles = (s.M + kWave) / kWave;
  const size_t lds =
      sizeof(float) * ((with_bp ? (SP + 3) * kWave : 0) + NC * kWave + NC * NC + NC + 32);
  const void *fn = with_bp ? (const void *)k_dp_class_fronts<SP, NW, true, NC>
                           : (const void *)k_dp_class_fronts<SP, NW, false, NC>;
  if (lds > 64 * 1024) lds_opt_in(fn, lds, s.grants);
  const long long rows = (long long)s.B * s.L;
  // Workgroups per instance and front: one per tile that earlier solves of the context found
  // with work (front_y0, 0 when nothing is known), all tiles at most.  Most tiles of a front
  // can be without work (rows that lead nowhere), and a workgroup that finds none still has
  // to be started, in order, before the next front's can be: with one workgroup per tile of
  // configs[3]'s shape (257 tiles, 113 with work) that took 2.4 of a front's 7.7 us.
  int y0 = s.tune.front_tiles >= 1 ? s.tune.front_tiles * 8 : front_y0;
  if (y0 > tiles || y0 < 1) y0 = tiles;
  hipLaunchKernelGGL(k_class_maxfit,
                     dim3((unsigned)(rows / 4 < 1 ? 1 : (rows / 4 > 1024 ? 1024 : rows / 4))),
                     dim3(256), 0, st, w.Oq, w.budget, w.topsum, w.lowsum, w.maxfit, w.stop,
                     w.epoch, w.front_flags, w.front_flag_words, s.B, s.L, s.SP, y0);
  // (the grid's thread count stays below 2^31)
  const unsigned bx = (unsigned)((s.B + 7) / 8 * 8); // workgroups b >= B leave at once
  const int spin_max = s.tune.spin_limit >= 1 ? s.tune.spin_limit : kFrontSpinMax;
  long long cap = ((1ll << 31) / (NW * kWave)) / ((long long)bx * y0);
  if (cap > 65535) cap = 65535;
  if (cap < 1) cap = 1;
  const int per = fronts < cap ? fronts : (int)cap;
  for (int l0 = 1; l0 < s.L; l0 += per) {
    const int nf = s.L - l0 < per ? s.L - l0 : per;
    const dim3 grid(bx, (unsigned)y0, (unsigned)nf), block(NW * kWave);
    if (with_bp)
      hipLaunchKernelGGL((k_dp_class_fronts<SP, NW, true, NC>), grid, block, lds, st, w.planes,
                         plane_elems_all, keep ? 1 : 0, w.zero_row, (uint8_t *)w.bp,
                         bp_layer_bytes, w.Tq, w.Oq, w.Rc, w.cmeta, w.cstart, w.cls, w.ridx,
                         w.budget, w.topsum, w.lowsum, w.maxfit, w.front_flags, w.stop, w.epoch,
                         w.status, s.B, s.L, class_rows(s), s.pitch, tiles, l0, spin_max,
                         s.tune.hold_flags == 1 ? 0 : 1, ring);
    else
      hipLaunchKernelGGL((k_dp_class_fronts<SP, NW, false, NC>), grid, block, lds, st, w.planes,
                         plane_elems_all, keep ? 1 : 0, w.zero_row, (uint8_t *)nullptr,
                         bp_layer_bytes, w.Tq, w.Oq, w.Rc, w.cmeta, w.cstart, w.cls, w.ridx,
                         w.budget, w.topsum, w.lowsum, w.maxfit, w.front_flags, w.stop, w.epoch,
                         w.status, s.B, s.L, class_rows(s), s.pitch, tiles, l0, spin_max,
                         s.tune.hold_flags == 1 ? 0 : 1, ring);
  }
  // The plain form behind it: leaves at once unless a front needed more than y0 workgroups.
  // All its workgroups have to be resident together when an instance has several of them:
  // one per compute unit is taken for granted, and an instance gets what that allows.
  {
    const void *fp = with_bp ? (const void *)k_dp_class_fronts_plain<SP, NW, true, NC>
                             : (const void *)k_dp_class_fronts_plain<SP, NW, false, NC>;
    if (lds > 64 * 1024) lds_opt_in(fp, lds, s.grants);
    int gy = resident_wgs / (int)bx;
    gy = gy > 32 ? 32 : gy;
    if (gy < 1) gy = 1; // (one workgroup per instance waits for nobody)
    if (gy > tiles) gy = tiles;
    const dim3 grid(bx, (unsigned)gy, 1), block(NW * kWave);
    if (with_bp)
      hipLaunchKernelGGL((k_dp_class_fronts_plain<SP, NW, true, NC>), grid, block, lds, st,
                         w.planes, plane_elems_all, keep ? 1 : 0, w.zero_row, (uint8_t *)w.bp,
                         bp_layer_bytes, w.Tq, w.Oq, w.Rc, w.cmeta, w.cstart, w.cls, w.ridx,
                         w.budget, w.topsum, w.lowsum, w.maxfit, w.front_flags, w.stop, w.epoch,
                         w.status, hint, s.B, s.L, class_rows(s), s.pitch, tiles, spin_max, ring);
    else
      hipLaunchKernelGGL((k_dp_class_fronts_plain<SP, NW, false, NC>), grid, block, lds, st,
                         w.planes, plane_elems_all, keep ? 1 : 0, w.zero_row, (uint8_t *)nullptr,
                         bp_layer_bytes, w.Tq, w.Oq, w.Rc, w.cmeta, w.cstart, w.cls, w.ridx,
                         w.budget, w.topsum, w.lowsum, w.maxfit, w.front_flags, w.stop, w.epoch,
                         w.status, hint, s.B, s.L, class_rows(s), s.pitch, tiles, spin_max, ring);
  }
}
template <int SP, int NW>
static void launch_fronts_nw(const Shape &s, const Workspace &w, bool keep, bool with_bp,
                             size_t pe, size_t bpl, int fronts, int ring, int y0, unsigned *hint,
                             int res, hipStream_t st) {
  if constexpr (SP >= 48) {
    if (s.NC > 32) return launch_fronts_nc<SP, NW, 64>(s, w, keep, with_bp, pe, bpl, fronts, ring, y0, hint, res, st);
  }
  if (s.NC <= 16) return launch_fronts_nc<SP, NW, 16>(s, w, keep, with_bp, pe, bpl, fronts, ring, y0, hint, res, st);
  launch_fronts_nc<SP, NW, 32>(s, w, keep, with_bp, pe, bpl, fronts, ring, y0, hint, res, st);
}

template <int SP>
static void launch_fronts(const Shape &s, const Workspace &w, bool keep, bool with_bp, size_t pe,
                          size_t bpl, int fronts, int ring, int y0, unsigned *hint, int res,
                          hipStream_t st) {
  // waves per tile as in the per-launch form, without its one- and two-wave forms
  int waves = s.tune.jsplit;
  if (waves < 1 || waves > 8) {
    if (with_bp) waves = SP >= 64 ? 8 : 4;
    else waves = SP >= 96 ? 8 : 4;
  }
  if constexpr (SP > 128) {
    launch_fronts_nw<SP, 8>(s, w, keep, with_bp, pe, bpl, fronts, ring, y0, hint, res, st);
  } else {
    if (waves >= 8) launch_fronts_nw<SP, 8>(s, w, keep, with_bp, pe, bpl, fronts, ring, y0, hint, res, st);
    else launch_fronts_nw<SP, 4>(s, w, keep, with_bp, pe, bpl, fronts, ring, y0, hint, res, st);
  }
}

// The forward pass of the class kernel with `fronts` layer fronts per launch (plus one small
// launch for its dependency table).  plane_elems_all: floats per plane slot; bp_layer_bytes:
// backpointer bytes per layer.
const char *launch_dp_class_fronts(const Shape &s, const Workspace &w, bool keep, bool with_bp,
                                   size_t plane_elems_all, size_t bp_layer_bytes, int fronts,
                                   int ring, int y0, unsigned *hint, int resident_wgs,
                                   hipStream_t st) {
  switch (s.SP) {
    case 16: launch_fronts<16>(s, w, keep, with_bp, plane_elems_all, bp_layer_bytes, fronts, ring, y0, hint, resident_wgs, st); break;
    case 24: launch_fronts<24>(s, w, keep, with_bp, plane_elems_all, bp_layer_bytes, fronts, ring, y0, hint, resident_wgs, st); break;
    case 32: launch_fronts<32>(s, w, keep, with_bp, plane_elems_all, bp_layer_bytes, fronts, ring, y0, hint, resident_wgs, st); break;
    case 48: launch_fronts<48>(s, w, keep, with_bp, plane_elems_all, bp_layer_bytes, fronts, ring, y0, hint, resident_wgs, st); break;
    case 64: launch_fronts<64>(s, w, keep, with_bp, plane_elems_all, bp_layer_bytes, fronts, ring, y0, hint, resident_wgs, st); break;
    case 96: launch_fronts<96>(s, w, keep, with_bp, plane_elems_all, bp_layer_bytes, fronts, ring, y0, hint, resident_wgs, st); break;
    case 128: launch_fronts<128>(s, w, keep, with_bp, plane_elems_all, bp_layer_bytes, fronts, ring, y0, hint, resident_wgs, st); break;
    case 192: launch_fronts<192>(s, w, keep, with_bp, plane_elems_all, bp_layer_bytes, fronts, ring, y0, hint, resident_wgs, st); break;
    case 256: launch_fronts<256>(s, w, keep, with_bp, plane_elems_all, bp_layer_bytes, fronts, ring, y0, hint, resident_wgs, st); break;
    default: break; // class_path_applies() admits no other pitch
  }
  return "k_dp_class_fronts";
}

void launch_class_zero(const Shape &s, float *q0, hipStream_t st) {
  const size_t n = (size_t)s.B * class_rows(s) * s.pitch;
  const unsigned blocks = (unsigned)((n + 256 * 8 - 1) / (256 * 8));
  hipLaunchKernelGGL(k_zero_plane, dim3(blocks < 1 ? 1 : blocks), dim3(256), 0, st, q0, n);
}

template <typename BPT, bool WITH_BP, int ROWS>
static void launch_wide_rows(const Shape &s, const Workspace &w, int l, const float *src,
                             float *dst, void *bp_l, hipStream_t st) {
  // target strategies per pass: four for the min-only scan, two with the argmin (measured)
  constexpr int NW = 8, JB = WITH_BP ? 2 : 4;
  const long long tiles = (s.M + 1 + ROWS - 1) / ROWS;
  const dim3 grid((unsigned)(tiles * s.B)), block(NW * kWave);
  const size_t lds = (size_t)s.SP * ROWS * sizeof(float);
  if (lds > 64 * 1024)
    lds_opt_in((const void *)k_dp_wide<BPT, NW, WITH_BP, JB, ROWS>, lds, s.grants);
  hipLaunchKernelGGL((k_dp_wide<BPT, NW, WITH_BP, JB, ROWS>), grid, block, lds, st, src, dst,
                     (BPT *)bp_l, w.Tq, w.Oq, w.Rt, w.ridx, w.budget, w.topsum, w.lowsum, s.B, s.L,
                     s.S, s.SP, l, s.pitch);
}

// 64-row tiles while S x 64 floats fit LDS (152 KB are asked for at most), else 32-row tiles
static bool wide_fits(const Shape &s, int rows) {
  return s.SP % 16 == 0 && (size_t)s.SP * rows * sizeof(float) <= 152 * 1024;
}

template <typename BPT, bool WITH_BP>
static void launch_wide_as(const Shape &s, const Workspace &w, int l, const float *src, float *dst,
                           void *bp_l, hipStream_t st) {
  if (wide_fits(s, kWave)) launch_wide_rows<BPT, WITH_BP, 64>(s, w, l, src, dst, bp_l, st);
  else launch_wide_rows<BPT, WITH_BP, 32>(s, w, l, src, dst, bp_l, st);
}

static void launch_wide(const Shape &s, const Workspace &w, int l, const float *src, float *dst,
                        void *bp_l, hipStream_t st) {
  if (!bp_l) launch_wide_as<uint8_t, false>(s, w, l, src, dst, bp_l, st);
  else if (s.bp16) launch_wide_as<uint16_t, true>(s, w, l, src, dst, bp_l, st);
  else launch_wide_as<uint8_t, true>(s, w, l, src, dst, bp_l, st);
}

const char *launch_dp_layer(const Shape &s, const Workspace &w, int l, const float *src,
                            float *dst, void *bp_l, ForwardKernel which, hipStream_t st) {
  const bool force_generic = which == ForwardKernel::Generic;
  const int blocks_per_instance = (s.M + 1 + kRowsPerBlock - 1) / kRowsPerBlock;
  const dim3 grid((unsigned)((size_t)blocks_per_instance * s.B));
  const int tsp = tuned_sp_for(s.S);
  // Which register-tiled kernel: measured on MI355X, the LDS-staged two-level kernel wins
  // from 48 padded strategies up when backpointers are wanted (its argmin costs about 2.3
  // instead of 4 vector instructions per relaxation) and for 48..64 without them; the
  // plain push kernel wins for small S (few chunks, relatively more fixed work per tile)
  // and for the min-only pass at S >= 96.  The context flags (or the knob "kernel" = 1 | 2) force one.
  bool use_tile = bp_l ? tsp >= 48 : (tsp >= 48 && tsp <= 64);
  // Small S: the push kernel wins on big batches (outer search: 2048 instances), but while
  // the batch has few tiles a front is bound by the length of one wave's work, and the
  // tile kernel's four waves per tile shorten it (measured crossover: about 16 K tiles with
  // backpointers, 4 K without).
  const long long tile_inst = (long long)((s.M + kWave) / kWave) * s.Bc;
  if (tsp != 0 && tsp <= 32) use_tile = tile_inst <= (bp_l ? 16384 : 4096);
  // Large S on a handful of tiles: the push kernel slices the strategies over up to eight
  // workgroups per tile and fills more of the chip (S = 96, 64 tiles: 0.22 against 0.31 ms
  // for 11 fronts).
  if (tsp >= 64 && tile_inst <= 256) use_tile = false;
  // The LDS-streamed kernel (made for more than 128 strategies) also wins below that where
  // the register-tiled ones run out of registers or of parallel work (measured, 7 fronts,
  // ms: S = 128, 8 x 16385 rows: 0.79 against 0.85 with backpointers, 0.62 against 0.71
  // without; S = 96 up to a few thousand tiles: configs[3] 6.9 against 7.3 ms with
  // backpointers, 5.5 against 5.8 without, but 8 K tiles 2.04 against 1.87 and 1.46 against
  // 1.27; S = 64 on a handful of tiles 0.08 against 0.09).
  // The knob "kernel" = 3 forces it wherever its tile fits.
  if (which == ForwardKernel::Auto && tsp == s.SP && s.SP % 16 == 0 && s.tune.kernel != 1 &&
      s.tune.kernel != 2) {
    const bool wide = s.tune.kernel == 3 || tsp == 128 ||
                      (tsp == 96 && tile_inst <= 4096) ||
                      (tsp == 64 && tile_inst <= 256);
    if (wide) {
      launch_wide(s, w, l, src, dst, bp_l, st);
      return "k_dp_wide";
    }
  }
  if (s.tune.kernel == 1 || which == ForwardKernel::Push) use_tile = false;
  if (s.tune.kernel == 2 || which == ForwardKernel::Tile) use_tile = true;
  if (!force_generic && tsp != 0 && tsp == s.SP && !s.bp16 && use_tile) {
    int waves = s.tune.jsplit;
    if (waves < 1 || waves > 4) waves = 4;
    if (waves > s.S) waves = s.S;
    switch (tsp) {
      case 8: launch_tile<8>(s, w, l, src, dst, bp_l, waves, st); return "k_dp_tile";
      case 16: launch_tile<16>(s, w, l, src, dst, bp_l, waves, st); return "k_dp_tile";
      case 24: launch_tile<24>(s, w, l, src, dst, bp_l, waves, st); return "k_dp_tile";
      case 32: launch_tile<32>(s, w, l, src, dst, bp_l, waves, st); return "k_dp_tile";
      case 48: launch_tile<48>(s, w, l, src, dst, bp_l, waves, st); return "k_dp_tile";
      case 64: launch_tile<64>(s, w, l, src, dst, bp_l, waves, st); return "k_dp_tile";
      case 96: launch_tile<96>(s, w, l, src, dst, bp_l, waves, st); return "k_dp_tile";
      case 128: launch_tile<128>(s, w, l, src, dst, bp_l, waves, st); return "k_dp_tile";
      default: break;
    }
  }
  if (!force_generic && tsp != 0 && tsp == s.SP && !s.bp16) {
    switch (tsp) {
      case 8: launch_push<8>(s, w, l, src, dst, bp_l, st); return "k_dp_push";
      case 16: launch_push<16>(s, w, l, src, dst, bp_l, st); return "k_dp_push";
      case 24: launch_push<24>(s, w, l, src, dst, bp_l, st); return "k_dp_push";
      case 32: launch_push<32>(s, w, l, src, dst, bp_l, st); return "k_dp_push";
      case 48: launch_push<48>(s, w, l, src, dst, bp_l, st); return "k_dp_push";
      case 64: launch_push<64>(s, w, l, src, dst, bp_l, st); return "k_dp_push";
      case 96: launch_push<96>(s, w, l, src, dst, bp_l, st); return "k_dp_push";
      case 128: launch_push<128>(s, w, l, src, dst, bp_l, st); return "k_dp_push";
      default: break;
    }
  }
  // Beyond the register-tiled sizes: the LDS-streamed tile kernel (every S the library accepts)
  if (!force_generic && tsp == 0 && wide_fits(s, 32)) {
    launch_wide(s, w, l, src, dst, bp_l, st);
    return "k_dp_wide";
  }
  if (!bp_l) {
    hipLaunchKernelGGL((k_dp_generic<uint8_t, false>), grid, dim3(kRowsPerBlock), 0, st, src,
                       dst, (uint8_t *)nullptr, w.Tq, w.Oq, w.Rt, w.ridx, w.budget, s.B, s.L,
                       s.S, s.SP, l, s.pitch);
  } else if (s.bp16) {
    hipLaunchKernelGGL((k_dp_generic<uint16_t, true>), grid, dim3(kRowsPerBlock), 0, st, src,
                       dst, (uint16_t *)bp_l, w.Tq, w.Oq, w.Rt, w.ridx, w.budget, s.B, s.L, s.S,
                       s.SP, l, s.pitch);
  } else {
    hipLaunchKernelGGL((k_dp_generic<uint8_t, true>), grid, dim3(kRowsPerBlock), 0, st, src,
                       dst, (uint8_t *)bp_l, w.Tq, w.Oq, w.Rt, w.ridx, w.budget, s.B, s.L, s.S,
                       s.SP, l, s.pitch);
  }
  return "k_dp_generic";
}

} // namespace gs
