// Score tables of LFPS (Sec. 4.2: Eq. 4 initialisation, Eq. 7-8 thresholds, Eq. 10 update; App. B.2).
//
// Per query head two tables over positions, vertical and slash.  Eq. 10 decays every entry by gamma each
// step, moves slash history from i-1 to i, and adds (w_i - 1/(2|C_2|)) on the selected positions only.
// Stored so that a step touches the selected entries and nothing else:
//   * scale: a table entry is  Phi(i) = g * A(i)  with one factor g per head.  The decay is g <- gamma g;
//     a selected entry becomes A(i) += delta_i / (gamma g).  (When g gets small a dense pass
//     folds it back into A, at the end of the update that made it small; each head decides for itself.)
//   * slash frame: A_sla is stored at index  i - cnt + Lcap  (cnt = updates applied so far), so the move
//     of history from i-1 to i is the increment of cnt.  The entry of a new position is the slot its
//     predecessor had; position 0 moves onto a slot that was never written (zero).
//   * statistics: Eq. 8 needs the mean, sum (x-mean)^2 and sum (x-mean)^4 of each table.  The raw
//     moments M_p = sum x^p (p = 1..4, fp64) follow the update exactly: M_p <- gamma^p M_p +
//     sum over selected of ((gamma x + delta)^p - (gamma x)^p); a new position adds a zero.
//     The thresholds of a step are derived from them when its scan starts.
// Sink positions (< n_sink) are outside the tables: never flagged, counted or updated.
//
// The only dense work of a step is the scan (k_table_flags): both tables are read once and two bits
// per position and head are written (initial candidate; above the mean).
#include "lfps_internal.h"

#include <type_traits>

namespace lfps {

constexpr int kTabThreads = 256;
constexpr int kFlagIters = 8;      // 64-position tests per wave of the scan kernel
constexpr double kFoldBelow = 1e-20;   // gamma = 0.95 gets here after ~900 updates; stored values stay < 1e20 * Phi

// head state (doubles): scale, update count, raw moments of both tables, and "the table was flat (every
// entry equal) when it was imported with N entries" marks.  The thresholds of Eq. 8 are derived from the
// moments at the start of every scan for the number of rows that scan sees, so a head whose update was
// skipped (a bypassed head) or a cache that grew by several rows needs no special case: new positions are zeros.
enum {
  TS_G = 0, TS_CNT = 1,
  TS_MV = 2,            // M1..M4 of the vertical table: [2..5]
  TS_MS = 6,            // M1..M4 of the slash table:    [6..9]
  TS_FLAT_V = 10, TS_FLAT_S = 11, TS_FLAT_N = 12,
};

// The update count as stored (a double) brought into [0, Lcap - 1]: every slash-frame index formed with
// it stays inside the table's 2 * Lcap slots (the host refuses updates beyond that count).
__device__ __forceinline__ int clamp_count(double c, int Lcap) {
  const int v = (int)c;
  return v < 0 ? 0 : (v > Lcap - 1 ? Lcap - 1 : v);
}

__device__ __forceinline__ double block_sum(double v, double* red, int tid) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) v += __shfl_xor(v, d);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < (int)blockDim.x / 64; ++w) t += red[w];
  return t;
}

__device__ __forceinline__ float block_min(float v, float* red, int tid) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) v = fminf(v, __shfl_xor(v, d));
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  float t = red[0];
  for (int w = 1; w < (int)blockDim.x / 64; ++w) t = fminf(t, red[w]);
  return t;
}

// Eq. 8 from raw moments over N entries: thresholds and means in true units.
__device__ __forceinline__ void thresholds_from_moments(const double* M, double N, double a, bool flat, double* tau,
                                                        double* mean) {
  if (N <= 0.0) {
    *tau = INFINITY;
    *mean = 0.0;
    return;
  }
  const double m = M[0] / N;
  *mean = m;
  const double c2 = M[1] - N * m * m;
  const double c4 = M[3] - 4.0 * m * M[2] + 6.0 * m * m * M[1] - 3.0 * N * m * m * m * m;
  if (flat || !(c2 > 0.0) || !(c4 > 0.0)) {
    *tau = INFINITY;                        // no pattern: nothing exceeds the threshold
    return;
  }
  const double kappa = c4 / (c2 * c2);
  *tau = a * m / kappa;
}

// ----------------------------------------------------------------------------- scan (Eq. 7, Eq. 9 predicates)
// Largest float <= t (t finite or +inf; NaN gives +inf: nothing passes).  For a float x and a double
// threshold t:  x > t  <=>  x > float_below(t), so the scan can compare in fp32 without changing a decision.
__device__ __forceinline__ float float_below(double t) {
  if (!(t == t)) return INFINITY;
  float f = (float)t;                                   // round to nearest
  if ((double)f > t) f = nextafterf(f, -INFINITY);
  return f;
}

// grid (chunks, B*Hq).  Each wave tests 64 consecutive positions per iteration; the ballots are the
// flag words.  A table entry is g * A(i); the comparison  g * A > threshold  is made as  A > threshold / g
// with the quotient (fp64) rounded down to fp32 once per head.
__global__ __launch_bounds__(kTabThreads) void k_table_flags(Shape s, const float* __restrict__ tab_ver,
                                                             const float* __restrict__ tab_sla,
                                                             const double* __restrict__ state,
                                                             const int32_t* __restrict__ seq_lens,
                                                             uint32_t* __restrict__ f0, uint32_t* __restrict__ fm,
                                                             int flag_words, int rows_per_block, double a,
                                                             const int32_t* __restrict__ gate) {
  __shared__ uint32_t w0[kFlagIters * kTabThreads / 32], wm[kFlagIters * kTabThreads / 32];
  const int bh = blockIdx.y, b = bh / s.Hq;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  const int n_round = (n + 63) & ~63;                     // whole flag words up to the end of the sequence
  if (gate && gate[bh] != 0) {                            // bypassed head: it proposes no candidates
    const int w_begin = (blockIdx.x * rows_per_block) >> 5;
    const int w_end = ((blockIdx.x + 1) * rows_per_block < n_round ? (blockIdx.x + 1) * rows_per_block : n_round) >> 5;
    for (int w = w_begin + tid; w < w_end; w += kTabThreads) {
      f0[(int64_t)bh * flag_words + w] = 0u;
      fm[(int64_t)bh * flag_words + w] = 0u;
    }
    return;
  }
  const double* st = state + (int64_t)bh * kTableStateDoubles;
  const double g = st[TS_G];
  const int cnt = clamp_count(st[TS_CNT], s.Lcap);
  float tau_v, tau_s, mean_v, mean_s;
  {
    const double N = (double)(n - s.n_sink > 0 ? n - s.n_sink : 0);
    double Mv[4], Ms[4], t, m;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      Mv[p] = st[TS_MV + p];
      Ms[p] = st[TS_MS + p];
    }
    const bool same_n = st[TS_FLAT_N] == N;
    thresholds_from_moments(Mv, N, a, st[TS_FLAT_V] != 0.0 && (same_n || Mv[1] == 0.0), &t, &m);
    tau_v = float_below(t / g);
    mean_v = float_below(m / g);
    thresholds_from_moments(Ms, N, a, st[TS_FLAT_S] != 0.0 && (same_n || Ms[1] == 0.0), &t, &m);
    tau_s = float_below(t / g);
    mean_s = float_below(m / g);
  }
  const float* ver = tab_ver + (int64_t)bh * s.Lcap;
  const float* sla = tab_sla + (int64_t)bh * 2 * s.Lcap + (s.Lcap - cnt);
  uint32_t* o0 = f0 + (int64_t)bh * flag_words;
  uint32_t* om = fm + (int64_t)bh * flag_words;
  // A workgroup covers rows_per_block consecutive positions in passes of kFlagIters * 256; in a pass wave w
  // takes every fourth 64-position word pair, and all its loads are issued before the first comparison
  // (fixed trip count, fully unrolled).  The flag words of a pass meet in LDS and leave as two coalesced stores.
  constexpr int kPassRows = kFlagIters * kTabThreads, kPassWords = kPassRows / 32;
  const int block_begin = blockIdx.x * rows_per_block;
  const int block_end = block_begin + rows_per_block < n_round ? block_begin + rows_per_block : n_round;
  for (int pass = block_begin; pass < block_end; pass += kPassRows) {
    const int begin = pass + wave * 64;
    float av[kFlagIters], as[kFlagIters];
#pragma unroll
    for (int it = 0; it < kFlagIters; ++it) {
      const int i = begin + it * kTabThreads + lane;
      const bool in = i >= s.n_sink && i < n;
      av[it] = in ? ver[i] : 0.f;
      as[it] = in ? sla[i] : 0.f;
    }
#pragma unroll
    for (int it = 0; it < kFlagIters; ++it) {
      const int i = begin + it * kTabThreads + lane;
      const bool in = i >= s.n_sink && i < n;
      const uint64_t m0 = __ballot(in && (av[it] > tau_v || as[it] > tau_s));
      const uint64_t mm = __ballot(in && (av[it] > mean_v || as[it] > mean_s));
      if (lane == 0) {
        const int w = (it * kTabThreads + wave * 64) >> 5;
        w0[w] = (uint32_t)m0;
        w0[w + 1] = (uint32_t)(m0 >> 32);
        wm[w] = (uint32_t)mm;
        wm[w + 1] = (uint32_t)(mm >> 32);
      }
    }
    __syncthreads();
    {
      const int w = tid & (kPassWords - 1);
      const int gw = (pass >> 5) + w;
      if (gw < (n_round >> 5)) {
        if (tid < kPassWords) o0[gw] = w0[w];
        else if (tid < 2 * kPassWords) om[gw] = wm[w];
      }
    }
    __syncthreads();
  }
}

// ----------------------------------------------------------------------------- update (Eq. 10)
// grid B*Hq.  The step saw n rows and selected idx[bh, 0:k_b] with scaled scores sc; entries outside
// [n_sink, n) are padding.  w = softmax over the valid entries; delta = w - 1/(2 * valid).
// kDistinct: the positions of a head's list are known to be distinct (the library's own Top-k), so an entry's old
// value can be read beside the addition; otherwise (a caller's list, where a position may appear twice) every
// addition returns the value it found, which keeps the moments exact for a repeated position too.
template <bool kDistinct>
__global__ __launch_bounds__(kTabThreads) void k_table_update(Shape s, float* __restrict__ tab_ver,
                                                              float* __restrict__ tab_sla, double* __restrict__ state,
                                                              const int32_t* __restrict__ seq_lens,
                                                              const int32_t* __restrict__ idx,
                                                              const float* __restrict__ sc,
                                                              const int32_t* __restrict__ kk, double gamma,
                                                              const int32_t* __restrict__ gate,
                                                              int32_t* __restrict__ flags) {
  __shared__ double red[kTabThreads / 64];
  __shared__ float redf[kTabThreads / 64];
  const int bh = blockIdx.x, b = bh / s.Hq, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (gate && gate[bh] != 0) return;                        // bypassed head: Eq. 10 is skipped for it
  // The slash frame has room for Lcap - 1 moves since the tables were last written whole: past that the
  // update is refused here (the host refuses it too, but counts only the calls it sees, not graph replays).
  if (state[(int64_t)bh * kTableStateDoubles + TS_CNT] >= (double)(s.Lcap - 1)) {   // workgroup-uniform
    if (tid == 0) atomicOr(flags, LFPS_FLAG_TABLE_FULL);
    return;
  }
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  double* st = state + (int64_t)bh * kTableStateDoubles;
  const double g = st[TS_G];
  const int cnt = clamp_count(st[TS_CNT], s.Lcap);
  const int32_t* ih = idx + (int64_t)bh * s.kmax;
  const float* sh = sc + (int64_t)bh * s.kmax;
  float* ver = tab_ver + (int64_t)bh * s.Lcap;
  float* sla = tab_sla + (int64_t)bh * 2 * s.Lcap + (s.Lcap - cnt);   // indexed by position in the frame of this step

  // softmax over the valid selected entries
  float m = -INFINITY;
  int nvalid = 0;
  for (int e = tid; e < kb; e += kTabThreads) {
    const int p = ih[e];
    if (p >= s.n_sink && p < n) {
      m = fmaxf(m, sh[e]);
      ++nvalid;
    }
  }
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) m = fmaxf(m, __shfl_xor(m, d));
  if (lane == 0) redf[wave] = m;
  __syncthreads();
  m = redf[0];
  for (int w = 1; w < kTabThreads / 64; ++w) m = fmaxf(m, redf[w]);
  double zsum = 0.0;
  for (int e = tid; e < kb; e += kTabThreads) {
    const int p = ih[e];
    if (p >= s.n_sink && p < n) zsum += (double)expf(sh[e] - m);
  }
  zsum = block_sum(zsum, red, tid);
  const double nv = block_sum((double)nvalid, red, tid);
  const double half = nv > 0.0 ? 0.5 / nv : 0.0;
  const double g1 = gamma * g;                               // scale after this step

  // selected entries: moments' change and the new unscaled values
  double dv[4] = {0, 0, 0, 0}, ds[4] = {0, 0, 0, 0};
  for (int e = tid; e < kb; e += kTabThreads) {
    const int p = ih[e];
    if (p >= s.n_sink && p < n) {
      const double delta = (double)expf(sh[e] - m) / zsum - half;
      const float inc = (float)(delta / g1);
      // (hardware fp32 adds in L2.)  Position p in the next frame (cnt + 1) is the slot of p - 1 in this one (for
      // p = 0 the never-written slot just below the frame).
      float old_v, old_s = 0.f;
      if constexpr (kDistinct) {
        old_v = ver[p];
        if (p - 1 >= s.n_sink) old_s = sla[p - 1];
        unsafeAtomicAdd(&ver[p], inc);
        unsafeAtomicAdd(&sla[p - 1], inc);
      } else {
        old_v = unsafeAtomicAdd(&ver[p], inc);
        old_s = unsafeAtomicAdd(&sla[p - 1], inc);
      }
      const double xv = gamma * g * (double)old_v;           // decayed old value
      const double xs = p - 1 >= s.n_sink ? gamma * g * (double)old_s : 0.0;   // decayed value moving in from p-1
      const double yv = xv + delta, ys = xs + delta;
      dv[0] += yv - xv;
      dv[1] += yv * yv - xv * xv;
      dv[2] += yv * yv * yv - xv * xv * xv;
      dv[3] += yv * yv * yv * yv - xv * xv * xv * xv;
      ds[0] += ys - xs;
      ds[1] += ys * ys - xs * xs;
      ds[2] += ys * ys * ys - xs * xs * xs;
      ds[3] += ys * ys * ys * ys - xs * xs * xs * xs;
    }
  }
  double tv[4], ts[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    tv[p] = block_sum(dv[p], red, tid);
    ts[p] = block_sum(ds[p], red, tid);
  }
  if (tid == 0) {
    double gp = 1.0;
    double Mv[4], Ms[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      gp *= gamma;
      Mv[p] = gp * st[TS_MV + p] + tv[p];
      Ms[p] = gp * st[TS_MS + p] + ts[p];
      st[TS_MV + p] = Mv[p];
      st[TS_MS + p] = Ms[p];
    }
    st[TS_G] = g1;
    st[TS_CNT] = (double)(cnt + 1);
    if (nv > 0.0) {                                          // entries were changed: no longer a flat table
      st[TS_FLAT_V] = 0.0;
      st[TS_FLAT_S] = 0.0;
    }
  }
  // Once the scale has become small it is folded into the stored values (A <- g A, g <- 1; the values g A
  // do not change).  The head decides for itself from its own state, here at the end of the update that
  // made the scale small, so no host-side count is involved and a recorded graph folds when an eager run would.
  // This step's additions were made in L2 (atomics): they are waited for, and the entries are then read
  // with device-scope loads, which do not look at this CU's vector cache (it may hold the old values).
  if (g1 < kFoldBelow) {                                     // workgroup-uniform
    __threadfence();
    __syncthreads();
    float* sla_all = tab_sla + (int64_t)bh * 2 * s.Lcap;
    for (int i = tid; i < s.Lcap; i += kTabThreads) {
      const float x = __hip_atomic_load(&ver[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ver[i] = (float)(g1 * (double)x);
    }
    for (int i = tid; i < 2 * s.Lcap; i += kTabThreads) {
      const float x = __hip_atomic_load(&sla_all[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      sla_all[i] = (float)(g1 * (double)x);
    }
    __syncthreads();
    if (tid == 0) st[TS_G] = 1.0;
  }
}

// ----------------------------------------------------------------------------- import / export / renormalise
// Import true table values phi_*[bh, 0:n_b] (fp32, position frame): scale 1, count 0, dense moments.
__global__ __launch_bounds__(kTabThreads) void k_table_import(Shape s, float* __restrict__ tab_ver,
                                                              float* __restrict__ tab_sla, double* __restrict__ state,
                                                              const int32_t* __restrict__ seq_lens,
                                                              const float* __restrict__ phi_ver,
                                                              const float* __restrict__ phi_sla) {
  __shared__ double red[kTabThreads / 64];
  __shared__ float redf[kTabThreads / 64];
  const int bh = blockIdx.x, b = bh / s.Hq, tid = threadIdx.x;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  float* ver = tab_ver + (int64_t)bh * s.Lcap;
  float* sla = tab_sla + (int64_t)bh * 2 * s.Lcap;
  const float* pv = phi_ver + (int64_t)bh * s.Lcap;
  const float* ps = phi_sla + (int64_t)bh * s.Lcap;
  double mv[4] = {0, 0, 0, 0}, ms[4] = {0, 0, 0, 0};
  float lo_v = INFINITY, hi_v = -INFINITY, lo_s = INFINITY, hi_s = -INFINITY;
  for (int i = tid; i < 2 * s.Lcap; i += kTabThreads) sla[i] = 0.f;
  __syncthreads();
  for (int i = tid; i < s.Lcap; i += kTabThreads) {
    const bool in = i >= s.n_sink && i < n;
    const float xv = in ? pv[i] : 0.f, xs = in ? ps[i] : 0.f;
    ver[i] = xv;
    sla[i + s.Lcap] = xs;
    if (in) {
      const double a1 = xv, b1 = xs;
      mv[0] += a1; mv[1] += a1 * a1; mv[2] += a1 * a1 * a1; mv[3] += a1 * a1 * a1 * a1;
      ms[0] += b1; ms[1] += b1 * b1; ms[2] += b1 * b1 * b1; ms[3] += b1 * b1 * b1 * b1;
      lo_v = fminf(lo_v, xv); hi_v = fmaxf(hi_v, xv);
      lo_s = fminf(lo_s, xs); hi_s = fmaxf(hi_s, xs);
    }
  }
  double Mv[4], Ms[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    Mv[p] = block_sum(mv[p], red, tid);
    Ms[p] = block_sum(ms[p], red, tid);
  }
  // a flat table (every entry equal) has no pattern: block minimum == block maximum
  lo_v = block_min(lo_v, redf, tid);
  hi_v = -block_min(-hi_v, redf, tid);
  lo_s = block_min(lo_s, redf, tid);
  hi_s = -block_min(-hi_s, redf, tid);
  const double N = (double)(n - s.n_sink > 0 ? n - s.n_sink : 0);
  if (tid == 0) {
    double* st = state + (int64_t)bh * kTableStateDoubles;
    st[TS_G] = 1.0;
    st[TS_CNT] = 0.0;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      st[TS_MV + p] = Mv[p];
      st[TS_MS + p] = Ms[p];
    }
    st[TS_FLAT_V] = hi_v > lo_v ? 0.0 : 1.0;
    st[TS_FLAT_S] = hi_s > lo_s ? 0.0 : 1.0;
    st[TS_FLAT_N] = N;
  }
}

// True table values of positions [0, n_b) as fp64 (zeros elsewhere up to Lcap).
__global__ __launch_bounds__(kTabThreads) void k_table_export(Shape s, const float* __restrict__ tab_ver,
                                                              const float* __restrict__ tab_sla,
                                                              const double* __restrict__ state,
                                                              const int32_t* __restrict__ seq_lens,
                                                              double* __restrict__ phi_ver,
                                                              double* __restrict__ phi_sla) {
  const int bh = blockIdx.y, b = bh / s.Hq;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  const double* st = state + (int64_t)bh * kTableStateDoubles;
  const double g = st[TS_G];
  const int cnt = clamp_count(st[TS_CNT], s.Lcap);
  const int i = blockIdx.x * kTabThreads + threadIdx.x;
  if (i >= s.Lcap) return;
  const bool in = i >= s.n_sink && i < n;
  phi_ver[(int64_t)bh * s.Lcap + i] = in ? g * (double)tab_ver[(int64_t)bh * s.Lcap + i] : 0.0;
  phi_sla[(int64_t)bh * s.Lcap + i] = in ? g * (double)tab_sla[(int64_t)bh * 2 * s.Lcap + (s.Lcap - cnt) + i] : 0.0;
}

// ----------------------------------------------------------------------------- Eq. 4
// Tables from the attention weights of the last s prefill queries.  One launch per query: the j-th most
// recent query (j = 1..s) sees rows [0, n_b - j + 1); its weights w (softmax over the offloaded rows it
// sees) are added to the vertical table at i and to the slash table at i + j - 1 (Eq. 4's w_{i-j+1}),
// times 1/(2 s (1 - gamma)).  j = 1 overwrites, later launches accumulate.  score[bh, 0:n_b] holds the
// scaled scores of query j.  grid B*Hq.  k_table_finish then derives the statistics.
__global__ __launch_bounds__(1024) void k_table_init(Shape s, float* __restrict__ tab_ver, float* __restrict__ tab_sla,
                                                     const int32_t* __restrict__ seq_lens,
                                                     const float* __restrict__ score, int64_t score_stride, double gamma,
                                                     int j, int n_queries) {
  __shared__ double red[16];
  __shared__ float redf[16];
  const int bh = blockIdx.x, b = bh / s.Hq, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  const int seen = n - j + 1 > 0 ? n - j + 1 : 0;           // rows query j sees
  const float* sc = score + (int64_t)bh * score_stride;
  float* ver = tab_ver + (int64_t)bh * s.Lcap;
  float* sla = tab_sla + (int64_t)bh * 2 * s.Lcap + s.Lcap;  // position frame (update count 0)
  float m = -INFINITY;
  for (int i = s.n_sink + tid; i < seen; i += 1024) m = fmaxf(m, sc[i]);
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) m = fmaxf(m, __shfl_xor(m, d));
  if (lane == 0) redf[wave] = m;
  __syncthreads();
  m = redf[0];
  for (int w = 1; w < 16; ++w) m = fmaxf(m, redf[w]);
  double z = 0.0;
  for (int i = s.n_sink + tid; i < seen; i += 1024) z += (double)expf(sc[i] - m);
  z = block_sum(z, red, tid);
  const double norm = z > 0.0 ? 1.0 / (2.0 * (double)n_queries * (1.0 - gamma) * z) : 0.0;
  if (j == 1) {
    for (int i = tid; i < s.Lcap; i += 1024) {
      ver[i] = 0.f;
      sla[i - s.Lcap] = 0.f;
      sla[i] = 0.f;
    }
    __syncthreads();
  }
  // a position receives at most one vertical and one slash contribution per launch: plain read-modify-write
  for (int i = s.n_sink + tid; i < seen; i += 1024) {
    const float x = (float)((double)expf(sc[i] - m) * norm);
    ver[i] += x;
    sla[i + j - 1] += x;                                     // i + j - 1 <= n - 1
  }
}

// Scale 1, update count 0, raw moments and flat marks of the tables as they stand in the position frame.
__global__ __launch_bounds__(kTabThreads) void k_table_finish(Shape s, const float* __restrict__ tab_ver,
                                                              const float* __restrict__ tab_sla,
                                                              double* __restrict__ state,
                                                              const int32_t* __restrict__ seq_lens) {
  __shared__ double red[kTabThreads / 64];
  __shared__ float redf[kTabThreads / 64];
  const int bh = blockIdx.x, b = bh / s.Hq, tid = threadIdx.x;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  const float* ver = tab_ver + (int64_t)bh * s.Lcap;
  const float* sla = tab_sla + (int64_t)bh * 2 * s.Lcap + s.Lcap;
  double mv[4] = {0, 0, 0, 0}, ms[4] = {0, 0, 0, 0};
  float lo_v = INFINITY, hi_v = -INFINITY, lo_s = INFINITY, hi_s = -INFINITY;
  for (int i = s.n_sink + tid; i < n; i += kTabThreads) {
    const float xv = ver[i], xs = sla[i];
    const double a1 = xv, b1 = xs;
    mv[0] += a1; mv[1] += a1 * a1; mv[2] += a1 * a1 * a1; mv[3] += a1 * a1 * a1 * a1;
    ms[0] += b1; ms[1] += b1 * b1; ms[2] += b1 * b1 * b1; ms[3] += b1 * b1 * b1 * b1;
    lo_v = fminf(lo_v, xv); hi_v = fmaxf(hi_v, xv);
    lo_s = fminf(lo_s, xs); hi_s = fmaxf(hi_s, xs);
  }
  double Mv[4], Ms[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    Mv[p] = block_sum(mv[p], red, tid);
    Ms[p] = block_sum(ms[p], red, tid);
  }
  lo_v = block_min(lo_v, redf, tid);
  hi_v = -block_min(-hi_v, redf, tid);
  lo_s = block_min(lo_s, redf, tid);
  hi_s = -block_min(-hi_s, redf, tid);
  if (tid == 0) {
    double* st = state + (int64_t)bh * kTableStateDoubles;
    st[TS_G] = 1.0;
    st[TS_CNT] = 0.0;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      st[TS_MV + p] = Mv[p];
      st[TS_MS + p] = Ms[p];
    }
    st[TS_FLAT_V] = hi_v > lo_v ? 0.0 : 1.0;
    st[TS_FLAT_S] = hi_s > lo_s ? 0.0 : 1.0;
    st[TS_FLAT_N] = (double)(n - s.n_sink > 0 ? n - s.n_sink : 0);
  }
}

// ----------------------------------------------------------------------------- head sparsity (Eq. 5, Eq. 6)
// One wave per (b, h).  rho = w_sink / (w_sink + w_global + w_local):
//   w_sink   = sum over rows [0, n_sink) of exp(q.K_i/sqrt(D)),
//   w_global = n * exp(q.kbar/sqrt(D) + |q|^2 sigma2_hat / 2)        (log-normal mean of the weights, App. B.1),
//   w_local  = sum over the newest n_local rows of exp(q.K_i/sqrt(D)).
// A head with rho > eps is bypassed: its output row is vbar, its index row -1 (Alg. 1 lines 1-4); the later
// kernels of the step skip it.  The three terms are kept as exponent + log-sum so that a dominant sink
// (logit in the hundreds) cannot overflow.
template <typename T, bool kPaged>
__global__ __launch_bounds__(64) void k_head_sparsity(Shape s, const float* __restrict__ q, const T* __restrict__ K,
                                                      int64_t stride_b, int64_t stride_h, int64_t stride_n, KvPage pg,
                                                      const int32_t* __restrict__ seq_lens,
                                                      const float* __restrict__ kbar,
                                                      const float* __restrict__ sigma2_hat, int n_local, float eps,
                                                      float* __restrict__ rho_out, int32_t* __restrict__ gate_out,
                                                      const float* __restrict__ vbar, int32_t* __restrict__ topk_idx,
                                                      float* __restrict__ topk_score, float* __restrict__ out,
                                                      float* __restrict__ thr_state) {
  const int bh = blockIdx.x, b = bh / s.Hq, h = bh % s.Hq, g = h / s.G, lane = threadIdx.x;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  const float scale = 0.08838834764831845f;
  const float q0 = q[(int64_t)bh * kD + 2 * lane], q1 = q[(int64_t)bh * kD + 2 * lane + 1];
  using Rows = RowMap<kPaged>;
  const T* Kbg = K + Rows::base(b, g, stride_b, stride_h);
  auto logit_of_row = [&](int row) {
    float k0, k1;
    const T* kr = Kbg + Rows::offset(pg, Rows::phys(pg, b, row), stride_b, stride_n) + 2 * lane;
    if constexpr (sizeof(T) == 1) {                 // two E4M3 bytes
      const uint32_t w = *reinterpret_cast<const uint16_t*>(kr);
      float x[4];
      fp8x4_to_f32(w, x);
      k0 = x[0];
      k1 = x[1];
    } else if constexpr (sizeof(T) == 2 && !std::is_same<T, _Float16>::value) {   // two bf16
      const uint32_t w = *reinterpret_cast<const uint32_t*>(kr);
      k0 = bf16_lo(w);
      k1 = bf16_hi(w);
    } else {
      k0 = (float)kr[0];
      k1 = (float)kr[1];
    }
    float d = fmaf(q1, k1, q0 * k0);
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) d += __shfl_xor(d, o);
    return (double)(d * scale);
  };
  // log-sum-exp accumulators (double: a handful of terms per head)
  auto lse_add = [](double& m, double& z, double x) {
    if (x > m) {
      z = z * exp(m - x) + 1.0;
      m = x;
    } else {
      z += exp(x - m);
    }
  };
  double m_sink = -INFINITY, z_sink = 0.0, m_loc = -INFINITY, z_loc = 0.0;
  const int ns = s.n_sink < n ? s.n_sink : n;
  for (int i = 0; i < ns; ++i) lse_add(m_sink, z_sink, logit_of_row(i));
  const int lo = n - n_local > 0 ? n - n_local : 0;
  for (int i = lo; i < n; ++i) lse_add(m_loc, z_loc, logit_of_row(i));
  float dk = fmaf(q1, kbar[((int64_t)b * s.Hkv + g) * kD + 2 * lane + 1], q0 * kbar[((int64_t)b * s.Hkv + g) * kD + 2 * lane]);
  float qq = fmaf(q1, q1, q0 * q0);
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    dk += __shfl_xor(dk, o);
    qq += __shfl_xor(qq, o);
  }
  const double l_glob = n > 0 ? log((double)n) + (double)(dk * scale) + (double)qq * (double)sigma2_hat[bh] * 0.5 : -INFINITY;
  const double l_sink = z_sink > 0.0 ? m_sink + log(z_sink) : -INFINITY;
  const double l_loc = z_loc > 0.0 ? m_loc + log(z_loc) : -INFINITY;
  // rho = exp(l_sink) / (exp(l_sink) + exp(l_glob) + exp(l_loc))
  double rho = 0.0;
  if (l_sink > -INFINITY) rho = 1.0 / (1.0 + exp(l_glob - l_sink) + exp(l_loc - l_sink));
  const bool bypass = rho > (double)eps;
  if (lane == 0) {
    if (rho_out) rho_out[bh] = (float)rho;
    gate_out[bh] = bypass ? 1 : 0;
  }
  if (bypass && out) {
    out[(int64_t)bh * kD + 2 * lane] = vbar[((int64_t)b * s.Hkv + g) * kD + 2 * lane];
    out[(int64_t)bh * kD + 2 * lane + 1] = vbar[((int64_t)b * s.Hkv + g) * kD + 2 * lane + 1];
    for (int i = lane; i < s.kmax; i += 64) {
      topk_idx[(int64_t)bh * s.kmax + i] = -1;
      if (topk_score) topk_score[(int64_t)bh * s.kmax + i] = 0.f;
    }
    // A head bypassed since the history was reset has no k-th score to remember, and a group with such a
    // head would be taken as "no previous step" by the filtered scoring pass at every step.  +inf keeps
    // nothing for this head there (its select is skipped anyway) and lets the group's other heads be
    // filtered; when the head is no longer bypassed its first select falls back to the unfiltered pass.
    if (thr_state && lane == 0 && isnan(thr_state[bh])) thr_state[bh] = INFINITY;
  }
}

// ----------------------------------------------------------------------------- prefill priors (Sec. 4.2 "Prefilling")
// Mean K row and mean V row over rows [n_sink, n_b) of one (b, g).  1024 threads: 64 row slots x 16 lanes
// of 8 channels; fp32 partial sums per thread, fp64 across the row slots.
template <typename TK, typename T, bool kPaged>
__global__ __launch_bounds__(1024) void k_prior_means(Shape s, const TK* __restrict__ K, const T* __restrict__ V,
                                                      int64_t stride_b, int64_t stride_h, int64_t stride_n, KvPage pg,
                                                      const int32_t* __restrict__ seq_lens, float* __restrict__ kbar,
                                                      float* __restrict__ vbar) {
  __shared__ float red[64][16][8];
  const int bg = blockIdx.x, b = bg / s.Hkv, g = bg % s.Hkv, tid = threadIdx.x;
  const int slot = tid >> 4, j = tid & 15;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  using Rows = RowMap<kPaged>;
  const int64_t base = Rows::base(b, g, stride_b, stride_h) + 8 * j;
  for (int which = 0; which < 2; ++which) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int r = s.n_sink + slot; r < n; r += 64) {
      float x[8];
      const int64_t off = base + Rows::offset(pg, Rows::phys(pg, b, r), stride_b, stride_n);
      if (which == 0)
        load8(K + off, x);
      else
        load8(V + off, x);
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] += x[c];
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 8; ++c) red[slot][j][c] = acc[c];
    __syncthreads();
    if (tid < kD) {
      double t = 0.0;
      for (int sl = 0; sl < 64; ++sl) t += (double)red[sl][tid >> 3][tid & 7];
      const int cnt = n - s.n_sink;
      (which == 0 ? kbar : vbar)[(int64_t)bg * kD + tid] = cnt > 0 ? (float)(t / (double)cnt) : 0.f;
    }
  }
}

// sigma2_hat[b, h] = (variance over rows [n_sink, n_b) of score[bh, i]) / |q[b, h]|^2.  grid B*Hq.
__global__ __launch_bounds__(1024) void k_prior_variance(Shape s, const float* __restrict__ q,
                                                         const int32_t* __restrict__ seq_lens,
                                                         const float* __restrict__ score, int64_t score_stride,
                                                         float* __restrict__ sigma2_hat) {
  __shared__ double red[16];
  const int bh = blockIdx.x, b = bh / s.Hq, tid = threadIdx.x;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  const float* sc = score + (int64_t)bh * score_stride;
  const int cnt = n - s.n_sink;
  double sum = 0.0;
  for (int i = s.n_sink + tid; i < n; i += 1024) sum += (double)sc[i];
  sum = block_sum(sum, red, tid);
  const double mean = cnt > 0 ? sum / (double)cnt : 0.0;
  double ss = 0.0;
  for (int i = s.n_sink + tid; i < n; i += 1024) {
    const double d = (double)sc[i] - mean;
    ss += d * d;
  }
  ss = block_sum(ss, red, tid);
  double qq = 0.0;
  for (int c = tid; c < kD; c += 1024) qq += (double)q[(int64_t)bh * kD + c] * (double)q[(int64_t)bh * kD + c];
  qq = block_sum(qq, red, tid);
  if (tid == 0) sigma2_hat[bh] = (cnt > 0 && qq > 0.0) ? (float)(ss / (double)cnt / qq) : 0.f;
}

// ----------------------------------------------------------------------------- launchers
hipError_t launch_table_flags(const Shape& s, const float* tab_ver, const float* tab_sla, const double* state,
                              const int32_t* seq_lens, uint32_t* f0, uint32_t* fm, int flag_words, double a,
                              const int32_t* gate, hipStream_t st) {
  // about 4096 workgroups in all, each a whole number of passes
  const int pass_rows = kTabThreads * kFlagIters;
  int per_head = 4096 / (s.B * s.Hq);
  per_head = per_head < 1 ? 1 : per_head;
  int rows_per_block = ((s.Lcap + per_head - 1) / per_head + pass_rows - 1) / pass_rows * pass_rows;
  if (rows_per_block < pass_rows) rows_per_block = pass_rows;
  const int chunks = (s.Lcap + rows_per_block - 1) / rows_per_block;
  hipLaunchKernelGGL(k_table_flags, dim3(chunks, s.B * s.Hq), dim3(kTabThreads), 0, st, s, tab_ver, tab_sla, state,
                     seq_lens, f0, fm, flag_words, rows_per_block, a, gate);
  return hipGetLastError();
}

hipError_t launch_table_update(const Shape& s, float* tab_ver, float* tab_sla, double* state, const int32_t* seq_lens,
                               const int32_t* idx, const float* sc, const int32_t* k, double gamma, const int32_t* gate,
                               int32_t* flags, bool distinct, hipStream_t st) {
  if (distinct)
    hipLaunchKernelGGL(k_table_update<true>, dim3(s.B * s.Hq), dim3(kTabThreads), 0, st, s, tab_ver, tab_sla, state,
                       seq_lens, idx, sc, k, gamma, gate, flags);
  else
    hipLaunchKernelGGL(k_table_update<false>, dim3(s.B * s.Hq), dim3(kTabThreads), 0, st, s, tab_ver, tab_sla, state,
                       seq_lens, idx, sc, k, gamma, gate, flags);
  return hipGetLastError();
}

hipError_t launch_table_import(const Shape& s, float* tab_ver, float* tab_sla, double* state, const int32_t* seq_lens,
                               const float* phi_ver, const float* phi_sla, hipStream_t st) {
  hipLaunchKernelGGL(k_table_import, dim3(s.B * s.Hq), dim3(kTabThreads), 0, st, s, tab_ver, tab_sla, state, seq_lens,
                     phi_ver, phi_sla);
  return hipGetLastError();
}

hipError_t launch_table_export(const Shape& s, const float* tab_ver, const float* tab_sla, const double* state,
                               const int32_t* seq_lens, double* phi_ver, double* phi_sla, hipStream_t st) {
  hipLaunchKernelGGL(k_table_export, dim3((s.Lcap + kTabThreads - 1) / kTabThreads, s.B * s.Hq), dim3(kTabThreads), 0,
                     st, s, tab_ver, tab_sla, state, seq_lens, phi_ver, phi_sla);
  return hipGetLastError();
}

hipError_t launch_table_init(const Shape& s, float* tab_ver, float* tab_sla, const int32_t* seq_lens,
                             const float* score, int64_t score_stride, double gamma, int j, int n_queries,
                             hipStream_t st) {
  hipLaunchKernelGGL(k_table_init, dim3(s.B * s.Hq), dim3(1024), 0, st, s, tab_ver, tab_sla, seq_lens, score,
                     score_stride, gamma, j, n_queries);
  return hipGetLastError();
}

hipError_t launch_table_finish(const Shape& s, const float* tab_ver, const float* tab_sla, double* state,
                               const int32_t* seq_lens, hipStream_t st) {
  hipLaunchKernelGGL(k_table_finish, dim3(s.B * s.Hq), dim3(kTabThreads), 0, st, s, tab_ver, tab_sla, state, seq_lens);
  return hipGetLastError();
}

hipError_t launch_head_sparsity(const Shape& s, int dtype, const float* q, const KvView& kv, const float* kbar,
                                const float* sigma2_hat, int n_local, float eps, float* rho, int32_t* gate,
                                const float* vbar, int32_t* topk_idx, float* topk_score, float* out, float* thr_state,
                                hipStream_t st) {
#define LFPS_LAUNCH_HSP(TYPE, PAGED)                                                                             \
  hipLaunchKernelGGL((k_head_sparsity<TYPE, PAGED>), dim3(s.B * s.Hq), dim3(64), 0, st, s, q, (const TYPE*)kv.k,     \
                     kv.stride_b, kv.stride_h, kv.stride_n, kv.page, kv.seq_lens, kbar, sigma2_hat, n_local, eps, rho, \
                     gate, vbar, topk_idx, topk_score, out, thr_state)
  const bool paged = kv.page.table != nullptr;
  if (dtype == LFPS_BF16 && kv.k_fp8) {
    if (paged) LFPS_LAUNCH_HSP(uint8_t, true);
    else LFPS_LAUNCH_HSP(uint8_t, false);
  } else if (dtype == LFPS_BF16) {
    if (paged) LFPS_LAUNCH_HSP(uint16_t, true);
    else LFPS_LAUNCH_HSP(uint16_t, false);
  } else if (dtype == LFPS_F16) {
    if (paged) LFPS_LAUNCH_HSP(_Float16, true);
    else LFPS_LAUNCH_HSP(_Float16, false);
  } else {
    if (paged) LFPS_LAUNCH_HSP(float, true);
    else LFPS_LAUNCH_HSP(float, false);
  }
#undef LFPS_LAUNCH_HSP
  return hipGetLastError();
}

hipError_t launch_prior_means(const Shape& s, int dtype, const KvView& kv, float* kbar, float* vbar, hipStream_t st) {
#define LFPS_LAUNCH_PM(KTYPE, TYPE, PAGED)                                                                        \
  hipLaunchKernelGGL((k_prior_means<KTYPE, TYPE, PAGED>), dim3(s.B * s.Hkv), dim3(1024), 0, st, s,                  \
                     (const KTYPE*)kv.k, (const TYPE*)kv.v, kv.stride_b, kv.stride_h, kv.stride_n, kv.page,         \
                     kv.seq_lens, kbar, vbar)
  const bool paged = kv.page.table != nullptr;
  if (dtype == LFPS_BF16 && kv.k_fp8 && kv.v_fp8) {
    if (paged) LFPS_LAUNCH_PM(uint8_t, uint8_t, true);
    else LFPS_LAUNCH_PM(uint8_t, uint8_t, false);
  } else if (dtype == LFPS_BF16 && kv.k_fp8) {
    if (paged) LFPS_LAUNCH_PM(uint8_t, uint16_t, true);
    else LFPS_LAUNCH_PM(uint8_t, uint16_t, false);
  } else if (dtype == LFPS_BF16 && kv.v_fp8) {
    if (paged) LFPS_LAUNCH_PM(uint16_t, uint8_t, true);
    else LFPS_LAUNCH_PM(uint16_t, uint8_t, false);
  } else if (dtype == LFPS_BF16) {
    if (paged) LFPS_LAUNCH_PM(uint16_t, uint16_t, true);
    else LFPS_LAUNCH_PM(uint16_t, uint16_t, false);
  } else if (dtype == LFPS_F16) {
    if (paged) LFPS_LAUNCH_PM(_Float16, _Float16, true);
    else LFPS_LAUNCH_PM(_Float16, _Float16, false);
  } else {
    if (paged) LFPS_LAUNCH_PM(float, float, true);
    else LFPS_LAUNCH_PM(float, float, false);
  }
#undef LFPS_LAUNCH_PM
  return hipGetLastError();
}

hipError_t launch_prior_variance(const Shape& s, const float* q, const int32_t* seq_lens, const float* score,
                                 int64_t score_stride, float* sigma2_hat, hipStream_t st) {
  hipLaunchKernelGGL(k_prior_variance, dim3(s.B * s.Hq), dim3(1024), 0, st, s, q, seq_lens, score, score_stride,
                     sigma2_hat);
  return hipGetLastError();
}

}  // namespace lfps
