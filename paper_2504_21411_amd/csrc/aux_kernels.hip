// Kernels around the forward DP: input sanitising, layer-0 initialisation, final
// reductions, backtrace, budget curve, debug export, strategy enumeration and the
// alpha-beta cost-table builder.  All of them are small next to the forward pass.
#include "gsearch_internal.h"

namespace gs {

#define GS_INF __builtin_huge_valf()

// ----------------------------------------------------------------------------------------
// Sanitised copies of the caller's tables (so that the hot kernels are memory-safe for
// any input) and the data-status word.  One wave per work item group:
//   wave < B*L            : one (b,l) row of T and O (lanes = strategies), r_index[b][l],
//                           min_s O by a wave reduction
//   remaining waves       : 64 consecutive entries each of the transposed transition pool
//                           (incl. the padding row behind it, which the push kernel's
//                           prefetch reads but never uses), then the budgets
// ----------------------------------------------------------------------------------------
static __device__ void prepare_part(
    int block, const float *__restrict__ T, const int32_t *__restrict__ O,
    const float *__restrict__ R,
    const int32_t *__restrict__ r_index, const int32_t *__restrict__ budget,
    float *__restrict__ Tq, int32_t *__restrict__ Oq, float *__restrict__ Rt,
    int32_t *__restrict__ ridx, int32_t *__restrict__ budq, int32_t *__restrict__ minO,
    int32_t *__restrict__ status, int B, int L, int S, int M, int K, int SP) {
  const long long nrow = (long long)B * L;
  const long long nr = (long long)K * SP * SP + SP;
  const long long nr_waves = (nr + kWave - 1) / kWave;
  const long long nb_waves = ((long long)B + kWave - 1) / kWave;
  const long long wave = ((long long)block * blockDim.x + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  int bad = 0;
  if (wave < nrow) {
    const int l = (int)(wave % L);
    int mo = M + 1;
    for (int s = lane; s < SP; s += kWave) {
      float t = 0.0f;
      int o = M + 1; // padding strategies never fit
      if (s < S) {
        t = T[wave * S + s];
        if (!(t >= 0.0f) || t == GS_INF || __builtin_signbit(t)) bad |= 0x1;
        o = O[wave * S + s];
        if (o < 0) { bad |= 0x4; o = M + 1; }
        if (o > M + 1) o = M + 1;
        mo = o < mo ? o : mo;
      }
      Tq[wave * SP + s] = t;
      Oq[wave * SP + s] = o;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      const int other = __shfl_xor(mo, d, 64);
      mo = other < mo ? other : mo;
    }
    if (lane == 0) {
      minO[wave] = mo;
      int k = 0;
      if (l > 0) {
        k = r_index[wave];
        if (k < 0 || k >= K) { bad |= 0x10; k = 0; }
      }
      ridx[wave] = k;
    }
  } else if (wave < nrow + nr_waves) {
    const long long x = (wave - nrow) * kWave + lane;
    if (x < nr) {
      float r = 0.0f;
      if (x < (long long)K * SP * SP) {
        const int i = (int)(x % SP);
        const int j = (int)((x / SP) % SP);
        const int k = (int)(x / ((long long)SP * SP));
        if (i < S && j < S) {
          r = R[((long long)k * S + i) * S + j];
          if (!(r >= 0.0f) || __builtin_signbit(r)) bad |= 0x2;
        }
      }
      Rt[x] = r;
    }
  } else if (wave < nrow + nr_waves + nb_waves) {
    const long long b = (wave - nrow - nr_waves) * kWave + lane;
    if (b < B) {
      int e = budget[b];
      if (e < 0 || e > M) { bad |= 0x8; e = e < 0 ? 0 : M; }
      budq[b] = e;
    }
  }
  if (bad) atomicOr(status, bad);
}

// ----------------------------------------------------------------------------------------
// Bin unit of an instance.  Let g be the greatest common divisor of the memories O[l][s]
// that can fit at all (O <= E; the others never fit whatever the unit).  Every reachable
// memory sum is a multiple of g, so C[l][e][s] depends on e only through floor(e / g), and
// the instance can be solved with O / g under the budget floor(E / g): the same plans are
// feasible, their costs are the same sums, every argmin sees the same candidates, and the
// planes have g times fewer rows.  This kernel (one workgroup per instance) finds g,
// rewrites the sanitised O table, its per-layer minima and the budget in that unit and
// keeps g and the budget in the caller's bins for the readers that report in the caller's
// bins (memory of a plan, budget curve, export).  g = 1 when nothing fits, when everything
// that fits needs no memory, or when the compression is switched off.
// Each wave stops scanning as soon as its running divisor is 1, the usual case.
//
// Last, in the same unit: lowsum[b][l] = min(M+1, sum_{l' <= l} min_s O[l'][s]).  A plan of
// layers 0..l needs at least that many bins, so C[l][e][.] is +inf for every e below it, and
// the forward kernels fill those rows without computing them.  Wave 0 scans 64 layers per
// round, inclusive scan across the lanes, carry from round to round (every term is at most
// M + 1 <= 2^24 + 1 and the running sum is clamped each round, so int32 cannot overflow).
// ----------------------------------------------------------------------------------------
static __device__ __forceinline__ int gcd_i32(int a, int b) { // a, b >= 0; gcd(0, x) = x
  while (b != 0) {
    const int t = a % b;
    a = b;
    b = t;
  }
  return a;
}

static __device__ __forceinline__ int wave_gcd(int g) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) g = gcd_i32(g, __shfl_xor(g, d, kWave));
  return g;
}

static __device__ void bin_unit_part(int b, int32_t *__restrict__ Oq,
                                     int32_t *__restrict__ budget,
                                     int32_t *__restrict__ budget0, int32_t *__restrict__ unit,
                                     int32_t *__restrict__ minO, int32_t *__restrict__ lowsum,
                                     int32_t *__restrict__ topsum, int32_t *__restrict__ status,
                                     int32_t *__restrict__ status_acc, int L, int SP, int M,
                                     int enable, int all_rows) {
  __shared__ int red[4];
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int lane = threadIdx.x & 63;
  const int E0 = budget[b];
  const int n = L * SP;
  int32_t *__restrict__ o = Oq + (size_t)b * n;
  int g = 0; // divisor of what this wave has seen so far (0: nothing yet)
  if (enable) {
    for (int x0 = wave * 4 * kWave; x0 < n; x0 += 16 * kWave) { // four loads in flight per lane
      int v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int x = x0 + u * kWave + lane;
        v[u] = x < n ? o[x] : 0;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) g = gcd_i32(g, v[u] <= E0 ? v[u] : 0);
      // (a lane that has reached 1 settles it for the wave without the reduction)
      g = __builtin_amdgcn_ballot_w64(g == 1) != 0 ? 1 : wave_gcd(g);
      if (g == 1) break; // wave-uniform
    }
  } else {
    g = 1;
  }
  if (lane == 0) red[wave] = g;
  __syncthreads(); // also: every thread has read the budget before thread 0 rewrites it
  g = gcd_i32(gcd_i32(red[0], red[1]), gcd_i32(red[2], red[3]));
  g = g < 1 ? 1 : g;
  if (g > 1) {
    for (int x = threadIdx.x; x < n; x += 256) {
      const int v = o[x];
      if (v <= E0) o[x] = v / g;
    }
    __syncthreads();
    for (int l = wave; l < L; l += 4) {
      int mo = M + 1;
      for (int s = lane; s < SP; s += kWave) {
        const int v = o[l * SP + s];
        mo = v < mo ? v : mo;
      }
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) {
        const int other = __shfl_xor(mo, d, kWave);
        mo = other < mo ? other : mo;
      }
      if (lane == 0) minO[(size_t)b * L + l] = mo;
    }
  }
  if (threadIdx.x == 0) {
    budget0[b] = E0;
    budget[b] = E0 / g;
    unit[b] = g;
    if (b == 0) { // the data-status word of this solve: what k_prepare found; cleared for the next
      *status = *status_acc;
      *status_acc = 0;
    }
  }
  __syncthreads(); // the minima rewritten above are visible to wave 0
  if (wave != 0) return;
  int carry = 0;
  for (int l0 = 0; l0 < L; l0 += kWave) {
    const int l = l0 + lane;
    int v = l < L ? minO[(size_t)b * L + l] : 0;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      const int up = __shfl_up(v, d, kWave);
      if (lane >= d) v = (v + up > M + 1) ? M + 1 : v + up;
    }
    v = (v + carry > M + 1) ? M + 1 : v + carry;
    if (l < L) lowsum[(size_t)b * L + l] = v;
    carry = __shfl(v, kWave - 1, kWave);
  }
  // The same from the other end: topsum[b][l] = min(M+1, sum_{l' >= l} min_s O[l'][s]), the
  // least memory layers l..L-1 still need.  A state (l-1, r) with r > E - topsum[l] cannot be
  // completed within the budget, so no result reads it (final row, budget curve and every
  // plan pass through states below that bound only): the forward kernels skip the tiles of
  // source rows above it.  With all_rows (kept planes are exported whole) the bound is the
  // layer's own least memory, beyond which a source row has no target row at all.
  carry = 0;
  for (int k0 = 0; k0 < L; k0 += kWave) {
    const int l = L - 1 - (k0 + lane);
    int v = l >= 0 ? minO[(size_t)b * L + l] : 0;
    const int own = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      const int up = __shfl_up(v, d, kWave);
      if (lane >= d) v = (v + up > M + 1) ? M + 1 : v + up;
    }
    v = (v + carry > M + 1) ? M + 1 : v + carry;
    if (l >= 0) topsum[(size_t)b * L + l] = all_rows ? own : v;
    carry = __shfl(v, kWave - 1, kWave);
  }
}

// ----------------------------------------------------------------------------------------
// Transition classes.  The caller's r_class[S] promises that R depends on the strategies
// only through contiguous classes.  Block 0 checks the partition itself (starts at 0, steps
// of 0 or 1, at most NC classes) and writes its run table; every block checks a
// share of the table entries against their left and upper neighbours of the same class,
// which together imply that R is constant on every (class, class) block.  A bad partition
// is replaced by the single class {0..S-1} so that whatever reads the run table stays in
// bounds; the status bit makes the solve report every instance as infeasible anyway.
// ----------------------------------------------------------------------------------------
static __device__ void prepare_classes_part(
    int block, int nblocks, const int32_t *__restrict__ r_class, const float *__restrict__ R,
    int32_t *__restrict__ cmeta, int32_t *__restrict__ cstart, int32_t *__restrict__ cls,
    int32_t *__restrict__ status, int S, int SP, int K, int NC) {
  __shared__ int s_bad, s_maxlen;
  int bad = 0;
  if (block == 0) {
    if (threadIdx.x == 0) { s_bad = 0; s_maxlen = 0; }
    __syncthreads();
    int pbad = 0;
    for (int i = threadIdx.x; i < S; i += blockDim.x) {
      const int c = r_class[i];
      const int prev = i ? r_class[i - 1] : 0;
      if (i == 0 ? c != 0 : (c != prev && c != prev + 1)) pbad = 1;
      if (c < 0 || c >= NC) pbad = 1;
    }
    if (pbad) atomicOr(&s_bad, 1);
    __syncthreads();
    const bool ok = s_bad == 0;
    const int nc = ok ? r_class[S - 1] + 1 : 1;
    for (int c = threadIdx.x; c <= NC; c += blockDim.x) cstart[c] = c == 0 ? 0 : S;
    __syncthreads();
    for (int i = threadIdx.x; i < SP; i += blockDim.x) {
      const int c = (ok && i < S) ? r_class[i] : 0;
      cls[i] = c;
      if (ok && i > 0 && i < S && c != r_class[i - 1]) cstart[c] = i;
    }
    __syncthreads();
    // longest class: thread c looks at its own run
    for (int c = threadIdx.x; c < nc; c += blockDim.x)
      atomicMax(&s_maxlen, (c + 1 < nc ? cstart[c + 1] : S) - cstart[c]);
    __syncthreads();
    if (threadIdx.x == 0) { cmeta[0] = nc; cmeta[1] = s_maxlen; }
    if (!ok) bad = 0x20;
  }
  // R constant inside classes: compare with the left (sj-1) and upper (si-1) neighbour, in
  // the caller's table (the sanitised copy holds the same values, transposed)
  const long long total = (long long)K * S * S;
  for (long long x = (long long)block * blockDim.x + threadIdx.x; x < total;
       x += (long long)nblocks * blockDim.x) {
    const int j = (int)(x % S);
    const int i = (int)((x / S) % S);
    const long long k = x / ((long long)S * S);
    const float *m = R + k * S * S;
    const uint32_t v = __float_as_uint(m[(size_t)i * S + j]);
    if (j > 0 && r_class[j] == r_class[j - 1] && v != __float_as_uint(m[(size_t)i * S + j - 1]))
      bad = 0x20;
    if (i > 0 && r_class[i] == r_class[i - 1] && v != __float_as_uint(m[(size_t)(i - 1) * S + j]))
      bad = 0x20;
  }
  if (bad) atomicOr(status, bad);
  (void)SP;
}

// Rc[k][cj][ci] = Rt[k][first strategy of cj][first strategy of ci], +inf for padding classes.
static __device__ void build_Rc_part(int block, int nblocks, const float *__restrict__ Rt,
                                     const int32_t *__restrict__ cmeta,
                                     const int32_t *__restrict__ cstart,
                                     float *__restrict__ Rc, int SP, int K, int NC) {
  const int nc = cmeta[0];
  const long long total = (long long)K * NC * NC;
  for (long long x = (long long)block * blockDim.x + threadIdx.x; x < total;
       x += (long long)nblocks * blockDim.x) {
    const int ci = (int)(x % NC);
    const int cj = (int)((x / NC) % NC);
    const long long k = x / (NC * NC);
    float r = GS_INF;
    if (ci < nc && cj < nc) r = Rt[k * SP * SP + (size_t)cstart[cj] * SP + cstart[ci]];
    Rc[x] = r;
  }
}

// r_class[s] = number of layout changes along desc[0..s] (one block, serial prefix over S
// <= 1024 entries by a scan in shared memory).
__global__ __launch_bounds__(1024) void k_layout_classes(const int32_t *__restrict__ desc, int S,
                                                         int32_t *__restrict__ r_class,
                                                         int32_t *__restrict__ count_out) {
  __shared__ int flag[1024];
  const int s = threadIdx.x;
  int f = 0;
  if (s > 0 && s < S)
    f = desc[5 * s] != desc[5 * (s - 1)] || desc[5 * s + 1] != desc[5 * (s - 1) + 1] ||
        desc[5 * s + 2] != desc[5 * (s - 1) + 2];
  flag[s] = f;
  __syncthreads();
  for (int d = 1; d < 1024; d <<= 1) { // inclusive scan
    const int add = s >= d ? flag[s - d] : 0;
    __syncthreads();
    flag[s] += add;
    __syncthreads();
  }
  if (s < S) r_class[s] = flag[s];
  if (s == S - 1 && count_out) *count_out = flag[s] + 1;
}

// Layer 0 has no predecessor: C[0][e][s] = T[0][s] if e >= O[0][s] else +inf.
__global__ void k_init_layer0(float *__restrict__ plane, const float *__restrict__ Tq,
                              const int32_t *__restrict__ Oq, const int32_t *__restrict__ budget,
                              int B, int L, int S, int SP, int pitch) {
  const int b = blockIdx.x % B;
  const int e = (blockIdx.x / B) * blockDim.x + threadIdx.x;
  if (e > budget[b]) return;
  for (int s = 0; s < S; ++s) {
    const float t = Tq[(size_t)b * L * SP + s];
    const int o = Oq[(size_t)b * L * SP + s];
    plane[((size_t)b * S + s) * pitch + e] = (e >= o) ? t : GS_INF;
  }
}

// Lexicographic (value, index) minimum across the 64 lanes of a wave, left in every lane.
// Inside a row of 16 lanes the partners come from DPP moves (two quad permutations, then
// rotations by 4 and 8: the minimum is idempotent, so a rotation serves as well as an
// exchange); the four row results are read out as scalars and combined.  About a quarter
// of the latency of six rounds of cross-lane permutes through the LDS crossbar, which
// matters to the backtrace from planes, where one such reduction sits in every layer's
// dependent chain.
static __device__ __forceinline__ void lexmin(float &v, int &idx, float ov, int oi) {
  const bool take = (ov < v) | ((ov == v) & (oi < idx)); // no short circuit: no branches
  v = take ? ov : v;
  idx = take ? oi : idx;
}
template <int CTRL>
static __device__ __forceinline__ void lexmin_dpp(float &v, int &idx) {
  const int vb = __float_as_int(v);
  const float ov = __int_as_float(__builtin_amdgcn_update_dpp(vb, vb, CTRL, 0xF, 0xF, false));
  const int oi = __builtin_amdgcn_update_dpp(idx, idx, CTRL, 0xF, 0xF, false);
  lexmin(v, idx, ov, oi);
}
static __device__ __forceinline__ void wave_argmin(float &v, int &idx) {
  lexmin_dpp<0xB1>(v, idx);  // quad_perm [1,0,3,2]
  lexmin_dpp<0x4E>(v, idx);  // quad_perm [2,3,0,1]
  lexmin_dpp<0x124>(v, idx); // row_ror 4
  lexmin_dpp<0x128>(v, idx); // row_ror 8
  float rv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  int ri = __builtin_amdgcn_readlane(idx, 0);
#pragma unroll
  for (int row = 1; row < 4; ++row)
    lexmin(rv, ri, __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16 * row)),
           __builtin_amdgcn_readlane(idx, 16 * row));
  v = rv;
  idx = ri;
}

// One wave per instance: min_s C[L-1][E_b][s] with the lowest s on ties.
// BY_CLASS: `last` is the class kernel's compact plane of layer L-1 and
// C[L-1][E][s] = Q[class s][E - O[L-1][s]] + T[L-1][s] (+inf when the strategy does not fit).
template <bool BY_CLASS>
static __device__ __forceinline__ float final_of_instance(
    int b, int lane, const float *__restrict__ last, const int32_t *__restrict__ budget,
    const int32_t *__restrict__ status, const float *__restrict__ Tq,
    const int32_t *__restrict__ Oq, const int32_t *__restrict__ cls,
    const int32_t *__restrict__ lowsum, float *__restrict__ ws_cost, int32_t *__restrict__ ws_s,
    float *__restrict__ best_cost, int32_t *__restrict__ best_s, float *__restrict__ final_row,
    int L, int S, int SP, int Sc, int pitch) {
  const int E = budget[b];
  const bool poisoned = *status != 0;
  const size_t tab = ((size_t)b * L + L - 1) * SP;
  // rows of the compact plane below the least memory of the earlier layers are +inf and not stored
  const int ql = (BY_CLASS && L > 1) ? lowsum[(size_t)b * L + L - 2] : 0;
  float m = GS_INF;
  int arg = 0x7fffffff;
  for (int s = lane; s < S; s += kWave) {
    float v;
    if (BY_CLASS) {
      const int d = E - Oq[tab + s];
      v = GS_INF;
      if (d >= ql) v = last[((size_t)b * Sc + cls[s]) * pitch + d] + Tq[tab + s];
    } else {
      v = last[((size_t)b * S + s) * pitch + E];
    }
    if (poisoned) v = GS_INF;
    if (final_row) final_row[(size_t)b * S + s] = v;
    if (v < m || arg == 0x7fffffff) { m = v; arg = s; }
  }
  wave_argmin(m, arg);
  if (lane == 0) {
    const int s = (m < GS_INF) ? arg : -1;
    ws_cost[b] = m;
    ws_s[b] = s;
    if (best_cost) best_cost[b] = m;
    if (best_s) best_s[b] = s;
  }
  return m; // the same in every lane
}

template <bool BY_CLASS>
__global__ void k_final_instance(const float *__restrict__ last,
                                 const int32_t *__restrict__ budget,
                                 const int32_t *__restrict__ status, const float *__restrict__ Tq,
                                 const int32_t *__restrict__ Oq, const int32_t *__restrict__ cls,
                                 const int32_t *__restrict__ lowsum,
                                 float *__restrict__ ws_cost, int32_t *__restrict__ ws_s,
                                 float *__restrict__ best_cost, int32_t *__restrict__ best_s,
                                 float *__restrict__ final_row, int B, int L, int S, int SP, int Sc,
                                 int pitch) {
  (void)final_of_instance<BY_CLASS>((int)blockIdx.x, (int)threadIdx.x, last, budget, status, Tq,
                                    Oq, cls, lowsum, ws_cost, ws_s, best_cost, best_s, final_row,
                                    L, S, SP, Sc, pitch);
  (void)B;
}

// Both final reductions in one launch for a batch of at most 16 instances: one workgroup, a
// wave per instance, then the minimum over instances, lowest instance on ties.
template <bool BY_CLASS>
__global__ __launch_bounds__(1024) void k_final_few(
    const float *__restrict__ last, const int32_t *__restrict__ budget,
    const int32_t *__restrict__ status, const float *__restrict__ Tq,
    const int32_t *__restrict__ Oq, const int32_t *__restrict__ cls,
    const int32_t *__restrict__ lowsum, float *__restrict__ ws_cost, int32_t *__restrict__ ws_s,
    float *__restrict__ best_cost, int32_t *__restrict__ best_s, float *__restrict__ final_row,
    int32_t *__restrict__ best_instance, int B, int L, int S, int SP, int Sc, int pitch) {
  __shared__ float sv[1024 / kWave];
  __shared__ int si[1024 / kWave];
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int lane = threadIdx.x & 63;
  const int nw = (int)(blockDim.x >> 6);
  float m = GS_INF;
  int arg = 0x7fffffff;
  for (int b = wave; b < B; b += nw) { // ascending: a strict "<" keeps the lowest instance
    const float v = final_of_instance<BY_CLASS>(b, lane, last, budget, status, Tq, Oq, cls, lowsum,
                                                ws_cost, ws_s, best_cost, best_s, final_row, L,
                                                S, SP, Sc, pitch);
    if (v < m) { m = v; arg = b; }
  }
  if (lane == 0) { sv[wave] = m; si[wave] = arg; }
  __syncthreads();
  if (threadIdx.x == 0 && best_instance) {
    for (int w = 1; w < nw; ++w)
      if (sv[w] < m || (sv[w] == m && si[w] < arg)) { m = sv[w]; arg = si[w]; }
    *best_instance = (m < GS_INF) ? arg : -1;
  }
}

// One block: argmin over instances, lowest instance on ties, -1 if none is feasible.
__global__ void k_final_global(const float *__restrict__ ws_cost, int32_t *__restrict__ out,
                               int B) {
  __shared__ float sv[256 / kWave];
  __shared__ int si[256 / kWave];
  float m = GS_INF;
  int arg = 0x7fffffff;
  for (int b = threadIdx.x; b < B; b += blockDim.x) {
    const float v = ws_cost[b];
    if (v < m) { m = v; arg = b; }
  }
  wave_argmin(m, arg);
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = m; si[threadIdx.x >> 6] = arg; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < (int)(blockDim.x >> 6); ++w)
      if (sv[w] < m || (sv[w] == m && si[w] < arg)) { m = sv[w]; arg = si[w]; }
    *out = (m < GS_INF) ? arg : -1;
  }
}

// Backtrace over stored backpointers: one thread per requested instance walks
//   s <- best_s; e <- E_b; for l = L-1 .. 1: plan[l] = s; s' = bp[l][e][s]; e -= O[l][s]; s = s'
// (the form for more than 256 strategies, uint16 backpointers).
template <typename BPT>
__global__ void k_backtrace_bp(const BPT *__restrict__ bp, const int32_t *__restrict__ Oq,
                               const int32_t *__restrict__ budget,
                               const int32_t *__restrict__ unit,
                               const int32_t *__restrict__ ws_s,
                               const int32_t *__restrict__ instances, int n,
                               int32_t *__restrict__ plan, int32_t *__restrict__ mem_used, int B,
                               int L, int S, int SP, int pitch) {
  const int q = blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= n) return;
  const int b = instances ? instances[q] : q;
  int s = (b >= 0 && b < B) ? ws_s[b] : -1;
  if (s < 0) {
    for (int l = 0; l < L; ++l) plan[(size_t)q * L + l] = -1;
    if (mem_used) mem_used[q] = -1;
    return;
  }
  int e = budget[b];
  int used = 0;
  const size_t layer_stride = (size_t)B * S * pitch;
  for (int l = L - 1; l >= 1; --l) {
    plan[(size_t)q * L + l] = s;
    const int o = Oq[((size_t)b * L + l) * SP + s];
    const int prev = (int)bp[(size_t)(l - 1) * layer_stride + ((size_t)b * S + s) * pitch + e];
    used += o;
    e -= o;
    s = prev;
  }
  plan[(size_t)q * L] = s;
  used += Oq[(size_t)b * L * SP + s];
  if (mem_used) mem_used[q] = used * unit[b]; // back to the caller's bins
}

// The same walk by one WAVE per requested instance (S <= 64 PL, uint8 backpointers): the O
// row of the current layer sits in registers, O[l][s] and the class of s are lane reads, and
// the O row of the layer below is fetched while the backpointer load is in flight - one
// memory round trip per layer instead of two.
// BY_CLASS: the class kernel stores one backpointer per (target class, SOURCE row), NC
// columns per instance: bp[l][e][s] = bpc[l][class s][e - O[l][s]].  A state on an optimal
// path is finite, so its source row exists and lies above the rows that hold +inf only.
template <bool BY_CLASS, int PL>
__global__ __launch_bounds__(kWave) void k_backtrace_bp_rows(
    const uint8_t *__restrict__ bp, const int32_t *__restrict__ Oq,
    const int32_t *__restrict__ cls, const int32_t *__restrict__ budget,
    const int32_t *__restrict__ unit, const int32_t *__restrict__ ws_s,
    const int32_t *__restrict__ instances, int n, int32_t *__restrict__ plan,
    int32_t *__restrict__ mem_used, int B, int L, int S, int SP, int NC, int pitch) {
  const int q = blockIdx.x;
  if (q >= n) return; // (the grid is n workgroups)
  const int lane = threadIdx.x;
  const int b = instances ? instances[q] : q;
  int s = (b >= 0 && b < B) ? ws_s[b] : -1;
  if (s < 0) {
    for (int l = lane; l < L; l += kWave) plan[(size_t)q * L + l] = -1;
    if (mem_used && lane == 0) mem_used[q] = -1;
    return;
  }
  int e = budget[b];
  int used = 0;
  const int cols = BY_CLASS ? NC : S;
  const size_t layer_stride = (size_t)B * cols * pitch;
  const size_t tab = (size_t)b * L * SP;
  // Two layers per memory round trip: while the backpointer of layer l is in flight, every
  // lane requests the backpointer of layer l-1 that would be needed if ITS strategy were the
  // answer (the row e - O[l][s] is already known, only the strategy is not); the answer then
  // picks its successor out of the lanes.
  int ic[PL], cl[PL], o_cur[PL], o_low[PL];
  const int lb = L > 1 ? L - 2 : 0;
#pragma unroll
  for (int u = 0; u < PL; ++u) {
    const int i = lane + kWave * u;
    ic[u] = i < S ? i : 0;
    cl[u] = BY_CLASS ? cls[ic[u]] : 0;
    o_cur[u] = Oq[tab + (size_t)(L - 1) * SP + ic[u]];
    o_low[u] = Oq[tab + (size_t)lb * SP + ic[u]];
  }
  auto pick = [&](const int (&row)[PL], int idx) {
    int r = 0;
#pragma unroll
    for (int u = 0; u < PL; ++u) {
      const int v = __shfl(row[u], idx & 63, kWave);
      r = (idx >> 6) == u ? v : r;
    }
    return r;
  };
  int l = L - 1;
  for (; l >= 2; l -= 2) {
    const int o = pick(o_cur, s);
    const int col = BY_CLASS ? pick(cl, s) : s;
    const int at = BY_CLASS ? e - o : e;
    const int e1 = e - o; // budget row of layer l-1
    int p1 = (int)bp[(size_t)(l - 1) * layer_stride + ((size_t)b * cols + col) * pitch + at];
    int spec[PL];
#pragma unroll
    for (int u = 0; u < PL; ++u) {
      const int cc = BY_CLASS ? cl[u] : ic[u];
      int a2 = BY_CLASS ? e1 - o_low[u] : e1;
      a2 = a2 > 0 ? a2 : 0; // a strategy that does not fit is never the answer
      spec[u] = (int)bp[(size_t)(l - 2) * layer_stride + ((size_t)b * cols + cc) * pitch + a2];
    }
    int n0[PL], n1[PL]; // O rows of layers l-2 and l-3 for the next round
    const int l3 = l >= 3 ? l - 3 : 0;
#pragma unroll
    for (int u = 0; u < PL; ++u) {
      n0[u] = Oq[tab + (size_t)(l - 2) * SP + ic[u]];
      n1[u] = Oq[tab + (size_t)l3 * SP + ic[u]];
    }
    asm volatile("" : "+v"(p1));
#pragma unroll
    for (int u = 0; u < PL; ++u) asm volatile("" : "+v"(spec[u]));
    const int s1 = p1;
    const int o1 = pick(o_low, s1);
    const int s2 = pick(spec, s1);
    if (lane == 0) {
      plan[(size_t)q * L + l] = s;
      plan[(size_t)q * L + l - 1] = s1;
    }
    used += o + o1;
    e = e1 - o1;
    s = s2;
#pragma unroll
    for (int u = 0; u < PL; ++u) { o_cur[u] = n0[u]; o_low[u] = n1[u]; }
  }
  if (l == 1) { // an odd layer left over: the plain step
    const int o = pick(o_cur, s);
    const int col = BY_CLASS ? pick(cl, s) : s;
    const int at = BY_CLASS ? e - o : e;
    const int prev = (int)bp[((size_t)b * cols + col) * pitch + at];
    if (lane == 0) plan[(size_t)q * L + 1] = s;
    used += o;
    e -= o;
    s = prev;
#pragma unroll
    for (int u = 0; u < PL; ++u) o_cur[u] = o_low[u];
  }
  const int o = pick(o_cur, s); // O[0][s]: the loops leave the row of layer 0 in o_cur
  if (lane == 0) {
    plan[(size_t)q * L] = s;
    if (mem_used) mem_used[q] = (used + o) * unit[b]; // back to the caller's bins
  }
}

// Backtrace without stored backpointers: one wave per requested instance re-derives every
// argmin from the kept planes, argmin_si ( C[l-1][e-O][si] + R[si][s] ), lowest si on ties
// (all +inf gives 0) - the same value the forward pass would have stored.
// BY_CLASS: the kept planes are the class kernel's compact ones, and
// C[l-1][r][si] = Q[l-1][class si][r - O[l-1][si]] + T[l-1][si] (+inf when r < O[l-1][si]),
// the very additions the forward pass made.
template <bool BY_CLASS>
__global__ void k_backtrace_planes(const float *__restrict__ planes,
                                   const float *__restrict__ Rt, const float *__restrict__ Tq,
                                   const int32_t *__restrict__ Oq,
                                   const int32_t *__restrict__ cls,
                                   const int32_t *__restrict__ lowsum,
                                   const int32_t *__restrict__ ridx,
                                   const int32_t *__restrict__ budget,
                                   const int32_t *__restrict__ unit,
                                   const int32_t *__restrict__ ws_s,
                                   const int32_t *__restrict__ instances, int n,
                                   int32_t *__restrict__ plan, int32_t *__restrict__ mem_used,
                                   int B, int L, int S, int SP, int Sc, int pitch) {
  const int q = blockIdx.x;
  if (q >= n) return; // (the grid is n workgroups)
  const int lane = threadIdx.x;
  const int b = instances ? instances[q] : q;
  int s = (b >= 0 && b < B) ? ws_s[b] : -1;
  if (s < 0) {
    for (int l = lane; l < L; l += kWave) plan[(size_t)q * L + l] = -1;
    if (mem_used && lane == 0) mem_used[q] = -1;
    return;
  }
  int e = budget[b];
  int used = 0;
  const size_t layer_stride = (size_t)B * S * pitch;
  const size_t inst = (size_t)b * (BY_CLASS ? Sc : S) * pitch;
  for (int l = L - 1; l >= 1; --l) {
    if (lane == 0) plan[(size_t)q * L + l] = s;
    const int o = Oq[((size_t)b * L + l) * SP + s];
    used += o;
    e -= o;
    const float *prevp = planes + (size_t)(l - 1) * layer_stride + inst;
    const float *rc = Rt + ((size_t)ridx[(size_t)b * L + l] * SP + s) * SP;
    const size_t prow = ((size_t)b * L + l - 1) * SP; // the previous layer's O and T rows
    // rows of the compact plane of layer l-1 below the least memory of layers 0..l-2 are
    // +inf and not stored
    const int ql = (BY_CLASS && l >= 2) ? lowsum[(size_t)b * L + l - 2] : 0;
    float m = GS_INF;
    int arg = 0x7fffffff;
    for (int i = lane; i < S; i += kWave) {
      float c;
      if (BY_CLASS) {
        const int d = e - Oq[prow + i];
        c = GS_INF;
        if (d >= ql) c = prevp[(size_t)cls[i] * pitch + d] + Tq[prow + i];
      } else {
        c = prevp[(size_t)i * pitch + e];
      }
      const float v = c + rc[i];
      if (v < m || arg == 0x7fffffff) { m = v; arg = i; }
    }
    wave_argmin(m, arg);
    s = arg;
  }
  if (lane == 0) {
    plan[(size_t)q * L] = s;
    used += Oq[(size_t)b * L * SP + s];
    if (mem_used) mem_used[q] = used * unit[b]; // back to the caller's bins
  }
}

// The same walk with one memory round trip per layer instead of four or five: the wave
// keeps the O row of the current layer and the O and T rows of the layer below in registers
// (PL strategies per lane, S <= 64 PL), fetches the rows two layers down and the next
// r_index while the plane values it depends on are in flight, and picks O[l][s] out of the
// registers with a lane read.  What still depends on the argmin just found - the plane
// values at row e and the transition column of s - is requested together.
template <bool BY_CLASS, int PL>
__global__ __launch_bounds__(kWave) void k_backtrace_planes_rows(
    const float *__restrict__ planes, const float *__restrict__ Rt, const float *__restrict__ Tq,
    const int32_t *__restrict__ Oq, const int32_t *__restrict__ cls,
    const int32_t *__restrict__ lowsum, const int32_t *__restrict__ ridx,
    const int32_t *__restrict__ budget, const int32_t *__restrict__ unit,
    const int32_t *__restrict__ ws_s, const int32_t *__restrict__ instances, int n,
    int32_t *__restrict__ plan, int32_t *__restrict__ mem_used, int B, int L, int S, int SP,
    int Sc, int M, int pitch) {
  const int q = blockIdx.x;
  if (q >= n) return; // (the grid is n workgroups)
  const int lane = threadIdx.x;
  const int b = instances ? instances[q] : q;
  int s = (b >= 0 && b < B) ? ws_s[b] : -1;
  if (s < 0) {
    for (int l = lane; l < L; l += kWave) plan[(size_t)q * L + l] = -1;
    if (mem_used && lane == 0) mem_used[q] = -1;
    return;
  }
  int e = budget[b];
  int used = 0;
  const size_t layer_stride = (size_t)B * S * pitch;
  const size_t inst = (size_t)b * (BY_CLASS ? Sc : S) * pitch;
  const size_t tab = (size_t)b * L * SP;
  // Every load below is unconditional (index clamped, value selected afterwards), so that
  // the loads of a step are in flight together and are awaited once.
  int ic[PL];      // lane + 64 u, or 0 for the lanes past the last strategy
  int cl[PL];      // class of that strategy
  int o_cur[PL];   // O[l][.]
  int o_low[PL];   // O[l-1][.]  (padding strategies: M + 1, they never fit)
  float t_low[PL]; // T[l-1][.]
  const int lb = L > 1 ? L - 2 : 0;
#pragma unroll
  for (int u = 0; u < PL; ++u) {
    const int i = lane + kWave * u;
    ic[u] = i < S ? i : 0;
    cl[u] = BY_CLASS ? cls[ic[u]] : 0;
    const int oc = Oq[tab + (size_t)(L - 1) * SP + ic[u]];
    const int ol = Oq[tab + (size_t)lb * SP + ic[u]];
    o_cur[u] = i < S ? oc : M + 1;
    o_low[u] = i < S ? ol : M + 1;
    t_low[u] = Tq[tab + (size_t)lb * SP + ic[u]];
  }
  int k = L > 1 ? ridx[(size_t)b * L + L - 1] : 0;
  // rows of the compact plane of layer l-1 below the least memory of layers 0..l-2 are +inf
  // and not stored: ql for the current step, fetched a step ahead like the other rows
  int ql = (BY_CLASS && L > 2) ? lowsum[(size_t)b * L + L - 3] : 0;
  for (int l = L - 1; l >= 1; --l) {
    if (lane == 0) plan[(size_t)q * L + l] = s;
    int o = 0;
#pragma unroll
    for (int u = 0; u < PL; ++u) {
      const int v = __shfl(o_cur[u], s & 63, kWave);
      o = (s >> 6) == u ? v : o;
    }
    used += o;
    e -= o;
    // rows two layers down and the next matrix index: independent of (s, e)
    int o_nxt[PL];
    float t_nxt[PL];
    const int l2 = l >= 2 ? l - 2 : 0;
    int ql_nxt = BY_CLASS ? lowsum[(size_t)b * L + (l >= 3 ? l - 3 : 0)] : 0;
    ql_nxt = l >= 3 ? ql_nxt : 0;
#pragma unroll
    for (int u = 0; u < PL; ++u) {
      o_nxt[u] = Oq[tab + (size_t)l2 * SP + ic[u]];
      t_nxt[u] = Tq[tab + (size_t)l2 * SP + ic[u]];
    }
    const int k_nxt = ridx[(size_t)b * L + (l >= 2 ? l - 1 : 1)];
    // what depends on (s, e): the plane values and the transition column of s
    const float *prevp = planes + (size_t)(l - 1) * layer_stride + inst;
    const float *rcol = Rt + ((size_t)k * SP + s) * SP;
    float craw[PL], rraw[PL];
    int dd[PL];
#pragma unroll
    for (int u = 0; u < PL; ++u) {
      if (BY_CLASS) {
        dd[u] = e - o_low[u];
        craw[u] = prevp[(size_t)cl[u] * pitch + (dd[u] > 0 ? dd[u] : 0)];
      } else {
        dd[u] = 0;
        craw[u] = prevp[(size_t)ic[u] * pitch + (e > 0 ? e : 0)];
      }
      rraw[u] = rcol[ic[u]];
    }
    // (keeps the compiler from sinking a load into the branch that selects its value,
    // where it would be awaited on its own)
#pragma unroll
    for (int u = 0; u < PL; ++u) asm volatile("" : "+v"(craw[u]), "+v"(rraw[u]));
    float m = GS_INF;
    int arg = lane;
#pragma unroll
    for (int u = 0; u < PL; ++u) {
      const int i = lane + kWave * u;
      float c = BY_CLASS ? craw[u] + t_low[u] : craw[u];
      c = (i < S && dd[u] >= ql) ? c : GS_INF;
      const float v = c + rraw[u];
      if (u == 0 || v < m) { m = v; arg = i; }
    }
    wave_argmin(m, arg);
    s = arg;
    k = k_nxt;
    ql = ql_nxt;
#pragma unroll
    for (int u = 0; u < PL; ++u) {
      const int i = lane + kWave * u;
      o_cur[u] = o_low[u];
      o_low[u] = i < S ? o_nxt[u] : M + 1;
      t_low[u] = t_nxt[u];
    }
  }
  if (lane == 0) plan[(size_t)q * L] = s;
  // O[0][s] sits in o_cur (the loop left the row of layer 0 there)
  int o = 0;
#pragma unroll
  for (int u = 0; u < PL; ++u) {
    const int v = __shfl(o_cur[u], s & 63, kWave);
    o = (s >> 6) == u ? v : o;
  }
  if (lane == 0 && mem_used) mem_used[q] = (used + o) * unit[b]; // back to the caller's bins
}

// Pipeline-aware outer reduction: one thread per candidate (pipeline degree, stage split,
// micro-batch count).  cost = (t_0 + ... + t_{pp-1}) + (m - 1) * max t, in fp32: the sum
// left to right over the members as listed, the product rounded, then one add; +inf as
// soon as a member is infeasible or not a valid instance id.  Offsets are clamped to the
// member list so that a corrupt offset table cannot read outside it.
__global__ void k_pipeline_groups(const float *__restrict__ stage_cost, int B, int G,
                                  const int32_t *__restrict__ offsets,
                                  const int32_t *__restrict__ members, int n_members,
                                  const int32_t *__restrict__ micro, float *__restrict__ cost) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= G) return;
  int lo = offsets[g], hi = offsets[g + 1];
  const int m = micro[g];
  bool ok = lo >= 0 && hi <= n_members && hi > lo && m >= 1;
  float sum = 0.0f, mx = 0.0f;
  for (int x = lo; ok && x < hi; ++x) {
    const int b = members[x];
    if (b < 0 || b >= B) { ok = false; break; }
    const float t = stage_cost[b];
    if (t == GS_INF) { ok = false; break; }
    sum = (x == lo) ? t : sum + t;
    mx = t > mx ? t : mx;
  }
  float out = GS_INF;
  if (ok) {
    const float bubble = (float)(m - 1) * mx;
    out = sum + bubble;
  }
  cost[g] = out;
}

// curve[b][e] = min_s C[L-1][e][s] for e <= E_b, +inf above.  BY_CLASS: from the compact
// plane, C[L-1][e][s] = Q[class s][e - O[L-1][s]] + T[L-1][s].  The plane is indexed in the
// instance's own bin unit g (row e / g holds the caller's rows e .. e + g - 1); budget0 is the
// budget in the caller's bins.
template <bool BY_CLASS>
__global__ void k_budget_curve(const float *__restrict__ last, const int32_t *__restrict__ budget0,
                               const int32_t *__restrict__ unit,
                               const int32_t *__restrict__ status, const float *__restrict__ Tq,
                               const int32_t *__restrict__ Oq, const int32_t *__restrict__ cls,
                               const int32_t *__restrict__ lowsum, float *__restrict__ curve,
                               int B, int L, int S, int SP, int Sc, int M, int pitch) {
  const int b = blockIdx.x % B;
  const int e0 = (blockIdx.x / B) * blockDim.x + threadIdx.x; // row in the caller's bins
  if (e0 > M) return;
  const int e = e0 / unit[b];
  const size_t tab = ((size_t)b * L + L - 1) * SP;
  const int ql = (BY_CLASS && L > 1) ? lowsum[(size_t)b * L + L - 2] : 0; // as in k_final_instance
  float m = GS_INF;
  if (e0 <= budget0[b] && *status == 0)
    for (int s = 0; s < S; ++s) {
      float v;
      if (BY_CLASS) {
        const int d = e - Oq[tab + s];
        v = GS_INF;
        if (d >= ql) v = last[((size_t)b * Sc + cls[s]) * pitch + d] + Tq[tab + s];
      } else {
        v = last[((size_t)b * S + s) * pitch + e];
      }
      m = v < m ? v : m;
    }
  curve[(size_t)b * (M + 1) + e0] = m;
}

// Canonical [b][l][e][s] export of the kept planes and backpointers (debug).  BY_CLASS: the
// planes are compact (one row per class) and the backpointers are stored per (target
// class, source row); both are expanded here.
template <typename BPT, bool BY_CLASS>
__global__ void k_export(const float *__restrict__ planes, const BPT *__restrict__ bp,
                         const int32_t *__restrict__ budget0,
                         const int32_t *__restrict__ unit, const float *__restrict__ Tq,
                         const int32_t *__restrict__ Oq, const int32_t *__restrict__ cls,
                         const int32_t *__restrict__ lowsum, float *__restrict__ C,
                         int32_t *__restrict__ bpo, int B, int L, int S, int SP, int Sc, int NC,
                         int M, int pitch) {
  const long long total = (long long)B * L * (M + 1) * S;
  const size_t layer_stride = (size_t)B * S * pitch;
  for (long long x = (long long)blockIdx.x * blockDim.x + threadIdx.x; x < total;
       x += (long long)gridDim.x * blockDim.x) {
    const int s = (int)(x % S);
    const int e0 = (int)((x / S) % (M + 1)); // row in the caller's bins
    const int l = (int)((x / ((long long)S * (M + 1))) % L);
    const int b = (int)(x / ((long long)S * (M + 1) * L));
    const bool in = e0 <= budget0[b];
    const int e = e0 / unit[b]; // the planes are indexed in the instance's own bin unit
    const size_t off = ((size_t)b * S + s) * pitch + e;
    const size_t tab = ((size_t)b * L + l) * SP + s;
    const int src = e - Oq[tab]; // source row of this state
    if (C) {
      float v = GS_INF;
      if (in) {
        if (BY_CLASS) {
          // (rows of a compact plane below the least memory of the earlier layers: +inf, not stored)
          const int ql = l > 0 ? lowsum[(size_t)b * L + l - 1] : 0;
          if (src >= ql)
            v = planes[(size_t)l * layer_stride + ((size_t)b * Sc + cls[s]) * pitch + src] + Tq[tab];
        } else {
          v = planes[(size_t)l * layer_stride + off];
        }
      }
      C[x] = v;
    }
    if (bpo) {
      int32_t v = 0;
      if (in && l > 0 && bp) {
        if (BY_CLASS) {
          // rows below the least memory of the earlier layers hold +inf only, their
          // targets' backpointer is 0
          if (src >= 0 && src >= lowsum[(size_t)b * L + l - 1])
            v = (int32_t)bp[(size_t)(l - 1) * B * NC * pitch +
                            ((size_t)b * NC + cls[s]) * pitch + src];
        } else {
          v = (int32_t)bp[(size_t)(l - 1) * layer_stride + off];
        }
      }
      bpo[x] = v;
    }
  }
}

// ----------------------------------------------------------------------------------------
// Strategy enumeration (paper section 2: decision tree over the parallel dimensions,
// infeasible branches discarded).  Tree levels: sp, tp, (dp = N / (tp*sp)), sdp, ckpt.
// One thread per leaf of the unpruned tree decides whether its leaf survives and, if so,
// finds its position by counting the surviving leaves before it in tree order.
// ----------------------------------------------------------------------------------------
static __device__ __forceinline__ bool leaf_alive(int leaf, int k, int N, int tp_max, int sp_max,
                                                  int tpsp_max, int *d) {
  const int ckpt = leaf & 1, sdp = (leaf >> 1) & 1;
  const int a = (leaf >> 2) % (k + 1); // log2 tp
  const int c = (leaf >> 2) / (k + 1); // log2 sp
  if (a + c > k) return false;
  const int tp = 1 << a, sp = 1 << c, dp = N >> (a + c);
  if (tp_max > 0 && tp > tp_max) return false;
  if (sp_max > 0 && sp > sp_max) return false;
  if (tpsp_max > 0 && tp * sp > tpsp_max) return false;
  if (sdp && dp == 1) return false;
  d[0] = tp; d[1] = sp; d[2] = dp; d[3] = sdp; d[4] = ckpt;
  return true;
}

// Single workgroup of 1024 threads; the unpruned tree has at most 31*31*4 = 3844 leaves, so
// every thread owns up to four consecutive leaves and the ranks come from one block-wide
// exclusive scan of the survivor counts.
__global__ __launch_bounds__(1024) void k_enumerate(int N, int k, int tp_max, int sp_max,
                                                    int tpsp_max, int32_t *__restrict__ desc,
                                                    int cap, int32_t *__restrict__ count_out) {
  __shared__ int wave_sum[16];
  const int leaves = (k + 1) * (k + 1) * 4;
  const int first = threadIdx.x * 4;
  int d[4][5];
  bool alive[4];
  int mine = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    alive[u] = first + u < leaves && leaf_alive(first + u, k, N, tp_max, sp_max, tpsp_max, d[u]);
    mine += alive[u] ? 1 : 0;
  }
  // inclusive scan inside the wave, then across the 16 waves
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  int incl = mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int v = __shfl_up(incl, off, 64);
    if (lane >= off) incl += v;
  }
  if (lane == 63) wave_sum[wv] = incl;
  __syncthreads();
  int base = 0, total = 0;
  for (int x = 0; x < 16; ++x) {
    if (x < wv) base += wave_sum[x];
    total += wave_sum[x];
  }
  int rank = base + incl - mine;
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (alive[u]) {
      if (rank < cap)
        for (int x = 0; x < 5; ++x) desc[(size_t)rank * 5 + x] = d[u][x];
      ++rank;
    }
  if (threadIdx.x == 0 && count_out) *count_out = total;
}

// ----------------------------------------------------------------------------------------
// Alpha-beta cost tables (paper section 2: time and memory cost models per strategy).
// fp64, one rounding per operation in the order written (the file is compiled without
// floating-point contraction), one final rounding to the output type.
// ----------------------------------------------------------------------------------------
static __device__ void build_TO(long long first, long long stride, int B, int L, int S, int M,
                                const int32_t *__restrict__ desc,
                                const double *__restrict__ layer, double F, double BW,
                                double bin, double keep, float *__restrict__ T,
                                int32_t *__restrict__ O) {
  const long long total = (long long)B * L * S;
  for (long long x = first; x < total; x += stride) {
    const int s = (int)(x % S);
    const long long row = x / S;
    const double *p = layer + row * 6;
    const double h = p[0], q = p[1], n = p[2], tscale = p[3], sscale = p[4], ascale = p[5];
    const int itp = desc[s * 5 + 0], isp = desc[s * 5 + 1], idp = desc[s * 5 + 2];
    const int sdp = desc[s * 5 + 3], ckpt = desc[s * 5 + 4];
    const double tp = itp, sp = isp, dp = idp;
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
    if (ckpt) {
      flops = flops * 4.0;
      flops = flops / 3.0;
    }
    double comm = 0.0;
    if (itp > 1) {
      double y = 16.0 * t;
      y = y * h;
      y = y * (tp - 1.0);
      y = y / tp;
      comm = comm + y;
    }
    if (idp > 1) {
      double y = P / tp;
      y = 4.0 * y;
      y = y * (dp - 1.0);
      y = y / dp;
      if (sdp) y = y * 1.5;
      comm = comm + y;
    }
    if (isp > 1) {
      double y = 8.0 * t;
      y = y * h;
      y = y * (sp - 1.0);
      y = y / sp;
      comm = comm + y;
    }
    double sec = flops / (tp * F);
    sec = sec + comm / BW;
    double ms = tscale * 1000.0;
    ms = ms * sec;
    T[x] = (float)ms;

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
    int o;
    if (!(bins >= 1.0)) o = 1;
    else if (bins > (double)M + 1.0) o = M + 1;
    else o = (int)bins;
    O[x] = o;
  }
}

// Profile-driven tables: measured per-layer-type compute time and memory plus measured
// collective bandwidth per group size (see include/gsearch.h for the formula).  fp64, one
// rounding per operation in the order written.  A layer type outside [0, Y) or a degree
// whose log2 is not covered by the bandwidth table yields T = +inf, O = M+1 (never fits).
__global__ void k_build_TO_profiled(int B, int L, int S, int M, int Y, int NB,
                                    const int32_t *__restrict__ desc,
                                    const int32_t *__restrict__ layer_type,
                                    const double *__restrict__ profile,
                                    const double *__restrict__ bw, double tokens, double overlap,
                                    double bin, double keep, double sf, float *__restrict__ T,
                                    int32_t *__restrict__ O) {
  const long long total = (long long)B * L * S;
  for (long long x = (long long)blockIdx.x * blockDim.x + threadIdx.x; x < total;
       x += (long long)gridDim.x * blockDim.x) {
    const int s = (int)(x % S);
    const long long row = x / S;
    const int y = layer_type[row];
    const int itp = desc[s * 5 + 0], isp = desc[s * 5 + 1], idp = desc[s * 5 + 2];
    const int sdp = desc[s * 5 + 3], ckpt = desc[s * 5 + 4];
    int gt = 0, gs = 0, gd = 0;
    while ((1 << gt) < itp) ++gt;
    while ((1 << gs) < isp) ++gs;
    while ((1 << gd) < idp) ++gd;
    if (y < 0 || y >= Y || gt >= NB || gs >= NB || gd >= NB) {
      T[x] = GS_INF;
      O[x] = M + 1;
      continue;
    }
    const double fwd = profile[y * 3], param = profile[y * 3 + 1], act = profile[y * 3 + 2];
    const double tp = itp, sp = isp, dp = idp;
    const double t = tokens / (dp * sp);
    double comp = t / 1000.0;
    comp = fwd * comp;
    comp = 3.0 * comp;
    comp = comp / tp;
    if (ckpt) {
      comp = comp * 4.0;
      comp = comp / 3.0;
    }
    double tpc = 0.0, dpc = 0.0, spc = 0.0;
    if (itp > 1) {
      double v = 4.0 * act;
      v = v * t;
      v = v * (tp - 1.0);
      v = v / tp;
      v = 1000.0 * v;
      tpc = v / bw[gt];
    }
    if (idp > 1) {
      double v = param / tp;
      v = 2.0 * v;
      v = v * (dp - 1.0);
      v = v / dp;
      if (sdp) v = v * 1.5;
      v = 1000.0 * v;
      dpc = v / bw[gd];
    }
    if (isp > 1) {
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
    T[x] = (float)ms;

    const double shard = sdp ? dp : 1.0;
    double state = sf * param;
    state = state / (tp * shard);
    double a = act * t;
    a = a / tp;
    if (ckpt) a = a * keep;
    const double bins = ceil((state + a) / bin);
    int o;
    if (!(bins >= 1.0)) o = 1;
    else if (bins > (double)M + 1.0) o = M + 1;
    else o = (int)bins;
    O[x] = o;
  }
}

static __device__ void build_R(long long first, long long stride, int S, int K,
                               const int32_t *__restrict__ desc,
                               const double *__restrict__ rmodel, double BW,
                               float *__restrict__ R) {
  const long long total = (long long)K * S * S;
  for (long long x = first; x < total; x += stride) {
    const int j = (int)(x % S), i = (int)((x / S) % S), k = (int)(x / ((long long)S * S));
    const int32_t *a = desc + i * 5, *c = desc + j * 5;
    float r = 0.0f;
    if (!(a[0] == c[0] && a[1] == c[1] && a[2] == c[2])) {
      const double h = rmodel[k * 2], n = rmodel[k * 2 + 1];
      const double gi = (double)a[2] * (double)a[1];
      const double gj = (double)c[2] * (double)c[1];
      const double lo = gi < gj ? gi : gj, hi = gi < gj ? gj : gi;
      const double w = (a[0] == c[0]) ? 1.0 : 0.5;
      double y = 2.0 * h;
      y = y * (n / gj);
      double keepfrac = w * lo;
      keepfrac = keepfrac / hi;
      y = y * (1.0 - keepfrac);
      y = y / BW;
      y = 1000.0 * y;
      r = (float)y;
    }
    R[x] = r;
  }
}

// ---- launchers -------------------------------------------------------------------------
static unsigned blocks_for(long long items, int threads, long long cap = 65535) {
  long long b = (items + threads - 1) / threads;
  if (b < 1) b = 1;
  if (b > cap) b = cap;
  return (unsigned)b;
}

// Both tables of the alpha-beta model in one launch: the first nb_to workgroups fill T and O,
// the others R.
__global__ __launch_bounds__(256) void k_build_tables(
    int nb_to, int B, int L, int S, int M, int K, const int32_t *__restrict__ desc,
    const double *__restrict__ layer, double F, double BW, double bin, double keep,
    const double *__restrict__ rmodel, float *__restrict__ T, int32_t *__restrict__ O,
    float *__restrict__ R) {
  const int nb = (int)blockIdx.x;
  if (nb < nb_to)
    build_TO((long long)nb * 256 + threadIdx.x, (long long)nb_to * 256, B, L, S, M, desc, layer, F,
             BW, bin, keep, T, O);
  else
    build_R((long long)(nb - nb_to) * 256 + threadIdx.x, (long long)((int)gridDim.x - nb_to) * 256,
            S, K, desc, rmodel, BW, R);
}

// The two launches that open a solve.  k_prepare: sanitised copies of the tables in its
// first nb_tables workgroups and, when the caller states transition classes, the check of
// that promise (against the caller's R) in the others.  k_bin_unit: one workgroup per
// instance for the bin unit and the least-memory scan, and behind them the workgroups that
// fill the class table (which needs the run table k_prepare's class part has written).
__global__ __launch_bounds__(256) void k_prepare(
    int nb_tables, const float *__restrict__ T, const int32_t *__restrict__ O,
    const float *__restrict__ R, const int32_t *__restrict__ r_index,
    const int32_t *__restrict__ budget, float *__restrict__ Tq, int32_t *__restrict__ Oq,
    float *__restrict__ Rt, int32_t *__restrict__ ridx, int32_t *__restrict__ budq,
    int32_t *__restrict__ minO, int32_t *__restrict__ status_acc, int B, int L, int S, int M,
    int K, int SP, const int32_t *__restrict__ r_class, int32_t *__restrict__ cmeta,
    int32_t *__restrict__ cstart, int32_t *__restrict__ cls, int NC) {
  const int block = (int)blockIdx.x;
  if (block < nb_tables)
    prepare_part(block, T, O, R, r_index, budget, Tq, Oq, Rt, ridx, budq, minO, status_acc, B, L,
                 S, M, K, SP);
  else
    prepare_classes_part(block - nb_tables, (int)gridDim.x - nb_tables, r_class, R, cmeta, cstart,
                         cls, status_acc, S, SP, K, NC);
}

__global__ __launch_bounds__(256) void k_bin_unit(
    int B, int32_t *__restrict__ Oq, int32_t *__restrict__ budget,
    int32_t *__restrict__ budget0, int32_t *__restrict__ unit, int32_t *__restrict__ minO,
    int32_t *__restrict__ lowsum, int32_t *__restrict__ topsum, int32_t *__restrict__ status,
    int32_t *__restrict__ status_acc, int L, int SP, int M, int enable, int all_rows,
    const float *__restrict__ Rt, const int32_t *__restrict__ cmeta,
    const int32_t *__restrict__ cstart, float *__restrict__ Rc, int K, int NC,
    unsigned *__restrict__ epoch) {
  const int block = (int)blockIdx.x;
  // The solve counter the class kernel's flags are stamped with (see k_dp_class_fronts):
  // advanced here, on the device, so that a captured and replayed solve advances it as well.
  // epoch[1]: the counter has wrapped and the flags still have to be cleared, which the next
  // solve that uses them does, setting epoch[2].
  if (epoch && block == 0 && threadIdx.x == 0) {
    if (epoch[2] != 0) epoch[1] = epoch[2] = 0;
    unsigned next = epoch[0] + 1u;
    if (next >= (1u << 29)) {
      next = 1u;
      epoch[1] = 1u;
    }
    epoch[0] = next;
  }
  if (block < B)
    bin_unit_part(block, Oq, budget, budget0, unit, minO, lowsum, topsum, status, status_acc, L,
                  SP, M, enable, all_rows);
  else
    build_Rc_part(block - B, (int)gridDim.x - B, Rt, cmeta, cstart, Rc, SP, K, NC);
}

void launch_prepare(const Shape &s, const float *T, const int32_t *O, const float *R,
                    const int32_t *r_index, const int32_t *budget, const int32_t *r_class,
                    const Workspace &w, bool compress_bins, bool all_rows, hipStream_t st) {
  const long long nr = (long long)s.K * s.SP * s.SP + s.SP;
  const long long waves = (long long)s.B * s.L + (nr + kWave - 1) / kWave + (s.B + kWave - 1) / kWave;
  const unsigned nb_tables = (unsigned)((waves + 3) / 4);
  // r_class: the class promise is checked, and the class table built, in the same launches
  const unsigned nb_classes = r_class ? blocks_for((long long)s.K * s.S * s.S, 256, 4096) : 0;
  const unsigned nb_rc = r_class ? blocks_for((long long)s.K * s.NC * s.NC, 256, 4096) : 0;
  hipLaunchKernelGGL(k_prepare, dim3(nb_tables + nb_classes), dim3(256), 0, st, (int)nb_tables, T,
                     O, R, r_index, budget, w.Tq, w.Oq, w.Rt, w.ridx, w.budget, w.minO,
                     w.status_acc, s.B, s.L, s.S, s.M, s.K, s.SP, r_class, w.cmeta, w.cstart,
                     w.cls, s.NC);
  hipLaunchKernelGGL(k_bin_unit, dim3((unsigned)s.B + nb_rc), dim3(256), 0, st, s.B, w.Oq,
                     w.budget, w.budget0, w.unit, w.minO, w.lowsum, w.topsum, w.status,
                     w.status_acc, s.L, s.SP, s.M, compress_bins ? 1 : 0, all_rows ? 1 : 0, w.Rt,
                     w.cmeta, w.cstart, w.Rc, s.K, s.NC, w.epoch);
}

void launch_layout_classes(const int32_t *desc, int S, int32_t *r_class, int32_t *count_out,
                           hipStream_t st) {
  hipLaunchKernelGGL(k_layout_classes, dim3(1), dim3(1024), 0, st, desc, S, r_class, count_out);
}

void launch_init_layer0(const Shape &s, const Workspace &w, float *plane0, hipStream_t st) {
  const int per = (s.M + 1 + 255) / 256;
  hipLaunchKernelGGL(k_init_layer0, dim3((unsigned)((size_t)per * s.B)), dim3(256), 0, st, plane0,
                     w.Tq, w.Oq, w.budget, s.B, s.L, s.S, s.SP, s.pitch);
}

void launch_final(const Shape &s, const Workspace &w, const float *last_plane, float *best_cost,
                  int32_t *best_s, float *final_row, int32_t *best_instance, hipStream_t st) {
  if (s.B <= 16) { // one launch, a wave per instance (64 instances in four turns measured
                   // 10.2 us against 8.6 us for the two launches)
    const dim3 block(kWave * s.B);
    if (w.by_class)
      hipLaunchKernelGGL((k_final_few<true>), dim3(1), block, 0, st, last_plane, w.budget,
                         w.status, w.Tq, w.Oq, w.cls, w.lowsum, w.best_cost, w.best_s, best_cost,
                         best_s, final_row, best_instance, s.B, s.L, s.S, s.SP, class_rows(s),
                         s.pitch);
    else
      hipLaunchKernelGGL((k_final_few<false>), dim3(1), block, 0, st, last_plane, w.budget,
                         w.status, w.Tq, w.Oq, w.cls, w.lowsum, w.best_cost, w.best_s, best_cost,
                         best_s, final_row, best_instance, s.B, s.L, s.S, s.SP, class_rows(s),
                         s.pitch);
    return;
  }
  if (w.by_class)
    hipLaunchKernelGGL((k_final_instance<true>), dim3(s.B), dim3(kWave), 0, st, last_plane,
                       w.budget, w.status, w.Tq, w.Oq, w.cls, w.lowsum, w.best_cost, w.best_s, best_cost,
                       best_s, final_row, s.B, s.L, s.S, s.SP, class_rows(s), s.pitch);
  else
    hipLaunchKernelGGL((k_final_instance<false>), dim3(s.B), dim3(kWave), 0, st, last_plane,
                       w.budget, w.status, w.Tq, w.Oq, w.cls, w.lowsum, w.best_cost, w.best_s, best_cost,
                       best_s, final_row, s.B, s.L, s.S, s.SP, class_rows(s), s.pitch);
  if (best_instance)
    hipLaunchKernelGGL(k_final_global, dim3(1), dim3(256), 0, st, w.best_cost, best_instance,
                       s.B);
}

template <bool BY_CLASS>
static void launch_backtrace_bp_rows(const Shape &s, const Workspace &w, const int32_t *instances,
                                     int n, int32_t *plan, int32_t *mem_used, hipStream_t st) {
  const dim3 grid(n), block(kWave);
#define GS_ROWS(PL)                                                                          \
  hipLaunchKernelGGL((k_backtrace_bp_rows<BY_CLASS, PL>), grid, block, 0, st,               \
                     (const uint8_t *)w.bp, w.Oq, w.cls, w.budget, w.unit, w.best_s, instances, n, \
                     plan, mem_used, s.B, s.L, s.S, s.SP, s.NC, s.pitch)
  if (s.S <= 64) GS_ROWS(1);
  else if (s.S <= 128) GS_ROWS(2);
  else GS_ROWS(4);
#undef GS_ROWS
}

void launch_backtrace_bp(const Shape &s, const Workspace &w, const int32_t *instances, int n,
                         int32_t *plan, int32_t *mem_used, hipStream_t st) {
  if (!s.bp16) { // S <= 256: one wave per instance, table rows in registers
    if (w.by_class) launch_backtrace_bp_rows<true>(s, w, instances, n, plan, mem_used, st);
    else launch_backtrace_bp_rows<false>(s, w, instances, n, plan, mem_used, st);
    return;
  }
  hipLaunchKernelGGL((k_backtrace_bp<uint16_t>), dim3((n + 63) / 64), dim3(64), 0, st,
                     (const uint16_t *)w.bp, w.Oq, w.budget, w.unit, w.best_s, instances, n, plan, mem_used,
                     s.B, s.L, s.S, s.SP, s.pitch);
}

template <bool BY_CLASS>
static void launch_backtrace_planes_of(const Shape &s, const Workspace &w, const int32_t *instances,
                                       int n, int32_t *plan, int32_t *mem_used, hipStream_t st) {
  const dim3 grid(n), block(kWave);
#define GS_ROWS(PL)                                                                              \
  hipLaunchKernelGGL((k_backtrace_planes_rows<BY_CLASS, PL>), grid, block, 0, st, w.planes, w.Rt, \
                     w.Tq, w.Oq, w.cls, w.lowsum, w.ridx, w.budget, w.unit, w.best_s, instances, n, plan, \
                     mem_used, s.B, s.L, s.S, s.SP, class_rows(s), s.M, s.pitch)
  if (s.S <= 64) GS_ROWS(1);
  else if (s.S <= 128) GS_ROWS(2);
  else if (s.S <= 256) GS_ROWS(4);
  else
    hipLaunchKernelGGL((k_backtrace_planes<BY_CLASS>), grid, block, 0, st, w.planes, w.Rt, w.Tq,
                       w.Oq, w.cls, w.lowsum, w.ridx, w.budget, w.unit, w.best_s, instances, n, plan,
                       mem_used, s.B, s.L, s.S, s.SP, class_rows(s), s.pitch);
#undef GS_ROWS
}

void launch_backtrace_planes(const Shape &s, const Workspace &w, const int32_t *instances, int n,
                             int32_t *plan, int32_t *mem_used, hipStream_t st) {
  if (w.by_class) launch_backtrace_planes_of<true>(s, w, instances, n, plan, mem_used, st);
  else launch_backtrace_planes_of<false>(s, w, instances, n, plan, mem_used, st);
}

void launch_pipeline_reduce(const Shape &s, const Workspace &w, int G, const int32_t *offsets,
                            const int32_t *members, int n_members, const int32_t *micro,
                            float *group_cost, int32_t *best_group, hipStream_t st) {
  hipLaunchKernelGGL(k_pipeline_groups, dim3((G + 255) / 256), dim3(256), 0, st, w.best_cost,
                     s.B, G, offsets, members, n_members, micro, group_cost);
  if (best_group)
    hipLaunchKernelGGL(k_final_global, dim3(1), dim3(256), 0, st, group_cost, best_group, G);
}

void launch_budget_curve(const Shape &s, const Workspace &w, const float *last_plane,
                         float *curve, hipStream_t st) {
  const int per = (s.M + 1 + 255) / 256;
  const dim3 grid((unsigned)((size_t)per * s.B)), block(256);
  if (w.by_class)
    hipLaunchKernelGGL((k_budget_curve<true>), grid, block, 0, st, last_plane, w.budget0, w.unit, w.status,
                       w.Tq, w.Oq, w.cls, w.lowsum, curve, s.B, s.L, s.S, s.SP, class_rows(s), s.M,
                       s.pitch);
  else
    hipLaunchKernelGGL((k_budget_curve<false>), grid, block, 0, st, last_plane, w.budget0, w.unit,
                       w.status, w.Tq, w.Oq, w.cls, w.lowsum, curve, s.B, s.L, s.S, s.SP,
                       class_rows(s), s.M, s.pitch);
}

void launch_export(const Shape &s, const Workspace &w, float *C, int32_t *bp, hipStream_t st) {
  const long long total = (long long)s.B * s.L * (s.M + 1) * s.S;
  const dim3 grid(blocks_for(total, 256, 1 << 20)), block(256);
  if (w.by_class)
    hipLaunchKernelGGL((k_export<uint8_t, true>), grid, block, 0, st, w.planes,
                       (const uint8_t *)w.bp, w.budget0, w.unit, w.Tq, w.Oq, w.cls, w.lowsum, C, bp, s.B,
                       s.L, s.S, s.SP, class_rows(s), s.NC, s.M, s.pitch);
  else if (s.bp16)
    hipLaunchKernelGGL((k_export<uint16_t, false>), grid, block, 0, st, w.planes,
                       (const uint16_t *)w.bp, w.budget0, w.unit, w.Tq, w.Oq, w.cls, w.lowsum, C, bp,
                       s.B, s.L, s.S, s.SP, class_rows(s), s.NC, s.M, s.pitch);
  else
    hipLaunchKernelGGL((k_export<uint8_t, false>), grid, block, 0, st, w.planes,
                       (const uint8_t *)w.bp, w.budget0, w.unit, w.Tq, w.Oq, w.cls, w.lowsum, C, bp, s.B,
                       s.L, s.S, s.SP, class_rows(s), s.NC, s.M, s.pitch);
}

// ----------------------------------------------------------------------------------------
// Measurement aid: a kernel whose LDS traffic is known exactly, to scale the profiler's LDS
// counters by (what a plain copy is to the HBM counters).  Every lane of 1024 x 256 threads
// performs `iters` operations of one kind on a 16 KB table, conflict-free (consecutive lanes,
// consecutive words or 16-byte vectors): 0 four-byte loads, 1 sixteen-byte loads, 2 four-byte
// stores, 3 float-minimum atomics.  The sum that keeps the loads alive goes to `sink`.
// ----------------------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void k_lds_calibration(float *__restrict__ sink, int iters) {
  __shared__ float4 tab[1024]; // 16 KB
  float *f = reinterpret_cast<float *>(tab);
  for (int i = threadIdx.x; i < 1024; i += 256) tab[i] = make_float4(1.0f, 2.0f, 3.0f, 4.0f);
  __syncthreads();
  float acc = 0.0f;
  unsigned idx = threadIdx.x;
  for (int i = 0; i < iters; ++i) {
    if (MODE == 0) {
      acc += f[idx & 4095];
    } else if (MODE == 1) {
      const float4 r = tab[idx & 1023];
      acc += r.x + r.w;
    } else if (MODE == 2) {
      f[idx & 4095] = acc + (float)i;
    } else {
      __hip_atomic_fetch_min(&f[idx & 4095], acc - (float)i, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    idx += 256;
    asm volatile("" : "+v"(acc)); // one LDS instruction per iteration, none merged or hoisted
  }
  __syncthreads();
  sink[blockIdx.x * 256 + threadIdx.x] = acc + f[threadIdx.x];
}

void launch_lds_calibration(int mode, int iters, float *sink, hipStream_t st) {
  const dim3 grid(1024), block(256);
  switch (mode) {
    case 0: hipLaunchKernelGGL(k_lds_calibration<0>, grid, block, 0, st, sink, iters); break;
    case 1: hipLaunchKernelGGL(k_lds_calibration<1>, grid, block, 0, st, sink, iters); break;
    case 2: hipLaunchKernelGGL(k_lds_calibration<2>, grid, block, 0, st, sink, iters); break;
    default: hipLaunchKernelGGL(k_lds_calibration<3>, grid, block, 0, st, sink, iters); break;
  }
}

void launch_enumerate(int N, int tp_max, int sp_max, int tpsp_max, int32_t *desc, int cap,
                      int32_t *count_out, hipStream_t st) {
  int k = 0;
  while ((1 << k) < N) ++k;
  hipLaunchKernelGGL(k_enumerate, dim3(1), dim3(1024), 0, st, N, k, tp_max, sp_max, tpsp_max,
                     desc, cap, count_out);
}

void launch_build_tables_profiled(int B, int L, int S, int M, int Y, int NB, const int32_t *desc,
                                  const int32_t *layer_type, const double *profile,
                                  const double *bw, double tokens, double overlap, double bin,
                                  double keep, double sf, float *T, int32_t *O, hipStream_t st) {
  hipLaunchKernelGGL(k_build_TO_profiled, dim3(blocks_for((long long)B * L * S, 256)), dim3(256),
                     0, st, B, L, S, M, Y, NB, desc, layer_type, profile, bw, tokens, overlap, bin,
                     keep, sf, T, O);
}

void launch_build_tables(int B, int L, int S, int M, int K, const int32_t *desc,
                         const double *layer, double flops_per_s, double bytes_per_s,
                         double bin_bytes, double ckpt_keep, const double *rmodel, float *T,
                         int32_t *O, float *R, hipStream_t st) {
  const unsigned nb_to = blocks_for((long long)B * L * S, 256);
  const unsigned nb_r = blocks_for((long long)K * S * S, 256);
  hipLaunchKernelGGL(k_build_tables, dim3(nb_to + nb_r), dim3(256), 0, st, (int)nb_to, B, L, S, M,
                     K, desc, layer, flops_per_s, bytes_per_s, bin_bytes, ckpt_keep, rmodel, T, O,
                     R);
}

} // namespace gs
