// S3 — per query head, the k best of the scored rows (Alg. 1 line 8 / Sec. 1 Step 2).
//
// One workgroup (16 waves) per (b, h); wave w owns the contiguous slice w of the head's scores.
// When the head has at most 32768 scores they are read from global memory once and kept in LDS
// (128 KB) for every later pass; otherwise each pass streams them again (L2).
//
//  1. block min/max of the scores;
//  2. one LDS histogram of 2048 bins that are *linear in the score* between min and max.  (Bins
//     taken from the raw float bits would put a bell-shaped score distribution into a few dozen
//     bins and serialise the LDS atomics; linear bins spread it and leave only a handful of
//     scores in the bin that holds the k-th largest.)
//  3. the bin of the k-th largest score, by a suffix scan over the histogram;
//  4. the exact k-th largest inside that bin: its members go to a small LDS list and each is
//     ranked against the others; if the bin is too full for the list (degenerate inputs: all
//     scores equal, one huge outlier) an exact most-significant-digit radix descent over the
//     order-preserving 32-bit keys of the bin's members finds it instead;
//  5. ordered compaction (per-thread contiguous runs of the LDS copy + one block scan; ballots and
//     prefix counts when streaming; no atomics): every row above the k-th value plus as many rows
//     equal to it as still needed, lowest position first.  The output is ascending in position
//     and identical from run to run.
// The second kernel applies the same steps to the short (score, position) lists that the filtered
// scoring pass leaves per head.
#include <float.h>

#include "lfps_internal.h"

namespace lfps {

constexpr int kSelThreads = 1024;       // workgroup of the general kernel
constexpr int kFilterSelThreads = 512;  // workgroup of the kernel that selects from the short survivor lists
constexpr int kCacheElems = 32768;      // scores of one head kept in LDS (dynamic, 128 KB)

// NT threads: 2*NT histogram bins (two per thread), up to NT members of the threshold bin ranked directly.
template <int NT>
struct SelectShared {
  uint32_t hist[2 * NT];
  uint32_t list[NT];
  uint32_t wsum[NT / 64];
  float wlo[NT / 64], whi[NT / 64];
  uint32_t cnt_gt[NT / 64], cnt_eq[NT / 64];
  uint32_t need, bin, list_n, thr, need_eq;
};

__device__ __forceinline__ int lanes_below(uint64_t m) {   // set bits of m at lanes lower than mine
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}

// Scores are made finite and -0 becomes +0, so that float comparisons order them exactly like
// their 32-bit keys and the linear bins are monotone.
__device__ __forceinline__ float sanitize(float x) { return fmaxf(fminf(x, FLT_MAX), -FLT_MAX) + 0.0f; }

__device__ __forceinline__ float key2f(uint32_t k) {       // inverse of f2key
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// Largest digit d (bins 2t, 2t+1 owned by thread t) whose suffix count reaches `need`.
// Writes sm.bin = d and sm.need = need - (count in bins above d).  All threads must call.
template <int NT>
__device__ __forceinline__ void find_bin(SelectShared<NT>& sm, uint32_t need, int tid, int lane, int wv) {
  constexpr int kSelWaves = NT / 64;
  const uint32_t lo = sm.hist[2 * tid], hi = sm.hist[2 * tid + 1];
  const uint32_t mine = lo + hi;
  uint32_t inc = mine;                       // inclusive suffix sum within the wave
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t o = __shfl_down(inc, d);
    if (lane + d < 64) inc += o;
  }
  if (lane == 0) sm.wsum[wv] = inc;
  __syncthreads();
  uint32_t above_waves = 0;
  for (int w = wv + 1; w < kSelWaves; ++w) above_waves += sm.wsum[w];
  const uint32_t suffix_incl = above_waves + inc;    // count in bins >= 2t
  const uint32_t suffix_excl = suffix_incl - mine;   // count in bins >  2t+1
  if (suffix_incl >= need && suffix_excl < need) {   // exactly one thread
    if (suffix_excl + hi >= need) {
      sm.bin = 2 * tid + 1;
      sm.need = need - suffix_excl;
    } else {
      sm.bin = 2 * tid;
      sm.need = need - (suffix_excl + hi);
    }
  }
  __syncthreads();
}

// Visits the wave's slice: `i` = row slot, `in` = slot valid, `x` = its sanitised score (from the
// LDS copy when CACHED, else from global memory).  Eight 64-slot rows are loaded before the first is
// used, so a streaming pass keeps eight loads in flight per lane; the trip counts are wave-uniform,
// so ballots inside see the whole wave.
#define LFPS_FOR_EACH(...)                                                            \
  for (int it0 = 0; it0 < nit; it0 += 8) {                                            \
    float xb_[8];                                                                     \
    _Pragma("unroll") for (int u_ = 0; u_ < 8; ++u_) {                                \
      const int i_ = r0 + 64 * (it0 + u_) + lane;                                     \
      xb_[u_] = CACHED ? cache[i_ < r1 ? i_ : r0] : sanitize(sc[i_ < r1 ? i_ : r0]);  \
    }                                                                                 \
    _Pragma("unroll") for (int u_ = 0; u_ < 8; ++u_) {                                \
      if (it0 + u_ < nit) {                                                           \
        const int i = r0 + 64 * (it0 + u_) + lane;                                    \
        const bool in = i < r1;                                                       \
        const float x = xb_[u_];                                                      \
        __VA_ARGS__                                                                   \
      }                                                                               \
    }                                                                                 \
  }

// `slot_of` (LDS, or NULL for identity) maps an element of the scored list to its candidate slot;
// `cbg` (or NULL for identity) maps a candidate slot to its position; a position outside [0, n_valid)
// (a bad entry of a caller's candidate list: its score is -inf, so it is taken only when fewer than k
// valid candidates exist) is written as -1 with score 0.  `thr_out` receives the k-th largest score.
// kHaveRange: the caller has already seen every element (it filled the cache) and passes its own
// thread's smallest and largest in pre_lo / pre_hi, which saves the first pass over the data.
template <bool CACHED, int NT, bool kHaveRange = false>
__device__ __forceinline__ void select_body(SelectShared<NT>& sm, float* __restrict__ cache,
                                            const float* __restrict__ sc, int c, int ksel,
                                            const int32_t* __restrict__ slot_of, const int32_t* __restrict__ cbg,
                                            int32_t* __restrict__ oi, float* __restrict__ os,
                                            float* __restrict__ thr_out, float pre_lo = FLT_MAX,
                                            float pre_hi = -FLT_MAX, int n_valid = 0x7FFFFFFF) {
  constexpr int kSelWaves = NT / 64, kBins = 2 * NT, kListCap = NT;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int chunk = (((c + kSelWaves - 1) / kSelWaves) + 63) & ~63;
  const int r0 = wv * chunk, r1 = (r0 + chunk < c) ? r0 + chunk : c;
  const int nit = r1 > r0 ? (r1 - r0 + 63) >> 6 : 0;

  // ---- 1. load (once, into LDS, if the head fits) and block min / max
  if (CACHED && sc) {                      // sc == NULL: the caller has already filled the cache
#pragma unroll 8
    for (int it = 0; it < nit; ++it) {
      const int i = r0 + 64 * it + lane;
      if (i < r1) cache[i] = sanitize(sc[i]);
    }
  }
  float lo = pre_lo, hi = pre_hi;
  if constexpr (!kHaveRange) {
    LFPS_FOR_EACH(lo = in ? fminf(lo, x) : lo; hi = in ? fmaxf(hi, x) : hi;)
  }
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    lo = fminf(lo, __shfl_xor(lo, d));
    hi = fmaxf(hi, __shfl_xor(hi, d));
  }
  if (lane == 0) {
    sm.wlo[wv] = lo;
    sm.whi[wv] = hi;
  }
  for (int i = tid; i < kBins; i += NT) sm.hist[i] = 0u;
  if (tid == 0) sm.list_n = 0u;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    lo = fminf(lo, sm.wlo[w]);
    hi = fmaxf(hi, sm.whi[w]);
  }
  const float range = hi - lo;
  const float scale = (range > 0.f && range < FLT_MAX) ? (float)kBins / range : 0.f;
  // monotone in x; the unsigned min also catches a NaN-poisoned or negative conversion
#define LFPS_BIN(x) ((int)min((uint32_t)(int)(((x)-lo) * scale), (uint32_t)(kBins - 1)))

  // ---- 2. histogram over linear bins
  LFPS_FOR_EACH(if (in) atomicAdd(&sm.hist[LFPS_BIN(x)], 1u);)
  __syncthreads();
  // ---- 3. bin of the ksel-th largest
  find_bin(sm, (uint32_t)ksel, tid, lane, wv);
  const int tb = (int)sm.bin;
  uint32_t need = sm.need;                 // rows still to take from bin tb (>= 1)
  const uint32_t m = sm.hist[tb];          // members of bin tb (>= need)
  __syncthreads();

  // ---- 4. exact threshold inside bin tb
  if (m <= (uint32_t)kListCap) {
    // members of bin tb lie within one bin width of its lower edge: a cheap float test first
    const float inv = scale > 0.f ? 1.0f / scale : 0.f;
    const float e_lo = lo + ((float)tb - 1.0f) * inv, e_hi = lo + ((float)tb + 2.0f) * inv;
    LFPS_FOR_EACH({
      const bool near = in && (scale == 0.f || (x >= e_lo && x <= e_hi));
      if (__ballot(near)) {
        const bool hit = near && LFPS_BIN(x) == tb;
        const uint64_t mh = __ballot(hit);
        if (mh) {
          uint32_t base = 0;
          if (lane == 0) base = atomicAdd(&sm.list_n, (uint32_t)__popcll(mh));
          base = __shfl(base, 0);
          if (hit) sm.list[base + lanes_below(mh)] = f2key(x);
        }
      }
    })
    __syncthreads();
    if (tid < (int)m) {
      const uint32_t u = sm.list[tid];
      uint32_t gt = 0, ge = 0;
      for (uint32_t jj = 0; jj < m; ++jj) {
        const uint32_t o = sm.list[jj];
        gt += o > u;
        ge += o >= u;
      }
      if (gt < need && need <= ge) {       // u is the need-th largest (equal keys write equal values)
        sm.thr = u;
        sm.need_eq = need - gt;
      }
    }
    __syncthreads();
  } else {
    uint32_t prefix = 0, mask = 0;
#pragma unroll 1
    for (int pass = 0; pass < 4; ++pass) {
      // digits of log2(kBins) bits from the top; the last pass takes what is left
      constexpr int kDigit = NT == 1024 ? 11 : 9;
      constexpr int kPasses = (32 + kDigit - 1) / kDigit;
      if (pass >= kPasses) break;
      const int shift = 32 - kDigit * (pass + 1) > 0 ? 32 - kDigit * (pass + 1) : 0;
      const uint32_t dmask = (pass == kPasses - 1) ? ((1u << (32 - kDigit * (kPasses - 1))) - 1u) : ((1u << kDigit) - 1u);
      for (int i = tid; i < kBins; i += NT) sm.hist[i] = 0u;
      __syncthreads();
      LFPS_FOR_EACH(if (in && LFPS_BIN(x) == tb) {
        const uint32_t key = f2key(x);
        if (((key ^ prefix) & mask) == 0u) atomicAdd(&sm.hist[(key >> shift) & dmask], 1u);
      })
      __syncthreads();
      find_bin(sm, need, tid, lane, wv);
      prefix |= sm.bin << shift;
      need = sm.need;
      mask |= dmask << shift;
      __syncthreads();
    }
    if (tid == 0) {
      sm.thr = prefix;
      sm.need_eq = need;
    }
    __syncthreads();
  }
  const float thr = key2f(sm.thr);          // the ksel-th largest score
  if (thr_out && tid == 0) *thr_out = thr;
  const uint32_t need_eq = sm.need_eq;      // rows equal to it that are taken

  // ---- 5. ordered compaction: every row above the threshold, plus the first need_eq rows equal to it
  if (CACHED) {
    // Thread t owns the contiguous elements [t*E, (t+1)*E) of the LDS copy (E odd: no bank conflicts).
    // Count, one block scan, write: no cross-lane traffic inside the loops.
    const int E = ((c + NT - 1) / NT) | 1;
    const int e0 = tid * E < c ? tid * E : c, e1 = e0 + E < c ? e0 + E : c;
    uint32_t mine = 0;                                  // (rows > thr) << 16 | (rows == thr)
    for (int i = e0; i < e1; ++i) {
      const float x = cache[i];
      mine += (x > thr ? 0x10000u : 0u) + (x == thr ? 1u : 0u);
    }
    const uint32_t inc = (uint32_t)wave_inclusive_sum((int)mine);
    if (lane == 63) sm.cnt_gt[wv] = inc;
    __syncthreads();
    uint32_t before = inc - mine;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) before += w < wv ? sm.cnt_gt[w] : 0u;
    uint32_t eq_run = before & 0xFFFFu;
    uint32_t pos = (before >> 16) + (eq_run < need_eq ? eq_run : need_eq);
    for (int i = e0; i < e1; ++i) {
      const float x = cache[i];
      const bool eq = x == thr;
      const bool take = x > thr || (eq && eq_run < need_eq);
      eq_run += eq ? 1u : 0u;
      if (take) {
        if (pos < (uint32_t)ksel) {
          const int sl = slot_of ? slot_of[i] : i;
          const int p = cbg ? cbg[sl] : sl;
          const bool okp = (uint32_t)p < (uint32_t)n_valid;
          oi[pos] = okp ? p : -1;
          if (os) os[pos] = okp ? x : 0.f;
        }
        ++pos;
      }
    }
  } else {
    uint32_t ngt = 0, neq = 0;
    LFPS_FOR_EACH(ngt += __popcll(__ballot(in && x > thr)); neq += __popcll(__ballot(in && x == thr));)
    if (lane == 0) {
      sm.cnt_gt[wv] = ngt;
      sm.cnt_eq[wv] = neq;
    }
    __syncthreads();
    uint32_t gt_before = 0, eq_before = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
      gt_before += w < wv ? sm.cnt_gt[w] : 0u;
      eq_before += w < wv ? sm.cnt_eq[w] : 0u;
    }
    uint32_t eq_run = eq_before;
    uint32_t out_run = gt_before + (eq_before < need_eq ? eq_before : need_eq);
    LFPS_FOR_EACH({
      const bool gt = in && x > thr;
      const bool eq = in && x == thr;
      const uint64_t m_eq = __ballot(eq);
      const bool take = gt || (eq && eq_run + lanes_below(m_eq) < need_eq);
      const uint64_t m_take = __ballot(take);
      if (take) {
        const uint32_t pos = out_run + lanes_below(m_take);
        if (pos < (uint32_t)ksel) {
          const int sl = slot_of ? slot_of[i] : i;
          const int p = cbg ? cbg[sl] : sl;
          const bool okp = (uint32_t)p < (uint32_t)n_valid;
          oi[pos] = okp ? p : -1;
          if (os) os[pos] = okp ? x : 0.f;
        }
      }
      eq_run += __popcll(m_eq);
      out_run += __popcll(m_take);
    })
  }
#undef LFPS_BIN
}
#undef LFPS_FOR_EACH

// The streaming variant is a real call, so that its code does not compete for registers with
// the register-resident variant.
__device__ __noinline__ void select_stream(SelectShared<kSelThreads>& sm, const float* __restrict__ sc, int c, int ksel,
                                           const int32_t* __restrict__ cbg, int32_t* __restrict__ oi,
                                           float* __restrict__ os, float* __restrict__ thr_out, int n_valid) {
  select_body<false, kSelThreads>(sm, nullptr, sc, c, ksel, nullptr, cbg, oi, os, thr_out, FLT_MAX, -FLT_MAX, n_valid);
}

__global__ __launch_bounds__(kSelThreads) void k_select(Shape s, const float* __restrict__ score,
                                                        int64_t score_stride, const int32_t* __restrict__ cand,
                                                        const int32_t* __restrict__ count_arr,
                                                        const int32_t* __restrict__ kk, int32_t* __restrict__ topk_idx,
                                                        float* __restrict__ topk_score, int cache_elems,
                                                        const int32_t* __restrict__ only_if,
                                                        float* __restrict__ thr_state,
                                                        const int32_t* __restrict__ skip_if,
                                                        const int32_t* __restrict__ seq_lens) {
  __shared__ SelectShared<kSelThreads> sm;
  extern __shared__ float cache[];
  const int bh = blockIdx.x, b = bh / s.Hq, h = bh % s.Hq, g = h / s.G;
  const int tid = threadIdx.x;
  if (only_if && only_if[bh] == 0) return;          // this head was already settled by the filtered pass
  if (skip_if && skip_if[bh] != 0) return;          // bypassed head: its rows were written by the gate
  const bool gather = cand != nullptr;
  int c = gather ? count_arr[b * s.Hkv + g] : count_arr[b];
  const int c_max = gather ? s.cand_cap : s.Lcap;
  c = c < 0 ? 0 : (c > c_max ? c_max : c);
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  const int ksel = kb < c ? kb : c;

  int32_t* oi = topk_idx + (int64_t)bh * s.kmax;
  float* os = topk_score ? topk_score + (int64_t)bh * s.kmax : nullptr;
  for (int i = ksel + tid; i < s.kmax; i += kSelThreads) {   // padding
    oi[i] = -1;
    if (os) os[i] = 0.f;
  }
  float* thr_out = thr_state ? thr_state + bh : nullptr;
  if (ksel == 0) {
    if (thr_out && tid == 0) *thr_out = -INFINITY;
    return;
  }

  const float* sc = score + (int64_t)bh * score_stride;
  const int32_t* cbg = gather ? cand + ((int64_t)b * s.Hkv + g) * s.cand_cap : nullptr;
  int n_valid = 0x7FFFFFFF;
  if (gather && seq_lens) {
    n_valid = seq_lens[b];
    n_valid = n_valid < 0 ? 0 : (n_valid > s.Lcap ? s.Lcap : n_valid);
  }
  if (c <= cache_elems)
    select_body<true, kSelThreads>(sm, cache, sc, c, ksel, nullptr, cbg, oi, os, thr_out, FLT_MAX, -FLT_MAX, n_valid);
  else
    select_stream(sm, sc, c, ksel, cbg, oi, os, thr_out, n_valid);
}

// ----------------------------------------------------------------------------- filtered input
// Select from the survivor lists written by the filtered score kernel.  That kernel cuts the
// line of all groups' candidate slots into parts of S slots (S = *seg_rows_in), one per wave; my
// group starts at slot pg = group_start[b, g] of the line, and its piece `sgm` is what wave
// w_first + sgm took of it, w_first = pg / S: the group's slots [lo, hi).  The piece holds
// seg_count[bh, sgm] (score, row position) pairs at offset lo of the head's score / position rows,
// ascending in position within and across pieces.  If the survivors are fewer than k (the filter
// threshold was too high) or more than the LDS list holds, the head is flagged for the unfiltered
// pass instead and nothing is written.  Workgroup 0 leaves *line_total at zero for the next step.
__global__ __launch_bounds__(kFilterSelThreads) void k_filter_select(Shape s, const float* __restrict__ score,
                                                               const int32_t* __restrict__ slot_in,
                                                               int64_t score_stride,
                                                               const int32_t* __restrict__ seg_count,
                                                               const int32_t* __restrict__ seg_rows_in, int nseg,
                                                               const int32_t* __restrict__ cand_count,
                                                               const int64_t* __restrict__ group_start,
                                                               int64_t* __restrict__ line_total,
                                                               const int32_t* __restrict__ kk,
                                                               int32_t* __restrict__ topk_idx,
                                                               float* __restrict__ topk_score,
                                                               float* __restrict__ thr_state,
                                                               int32_t* __restrict__ redo_g,
                                                               int32_t* __restrict__ redo_h, int cap,
                                                               const int32_t* __restrict__ skip_if,
                                                               int32_t* __restrict__ rescored) {
  constexpr int NT = kFilterSelThreads, kSelWaves = NT / 64;
  constexpr int kPiecesPerThread = 1024 / NT;      // nseg <= 1024
  __shared__ SelectShared<NT> sm;
  __shared__ int seg_off[kPiecesPerThread * NT];
  __shared__ int wtot[kSelWaves];
  extern __shared__ float cache[];                 // cap scores, then cap row positions
  int32_t* lslot = reinterpret_cast<int32_t*>(cache + cap);
  const int bh = blockIdx.x, b = bh / s.Hq, h = bh % s.Hq, g = h / s.G;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int bg = b * s.Hkv + g;
  if (bh == 0 && tid == 0) *line_total = 0;          // the scoring pass that read it has finished
  if (skip_if && skip_if[bh] != 0) return;           // bypassed head: its rows were written by the gate
  int raw[kPiecesPerThread];                         // piece counts of this head, masked once the geometry is known
#pragma unroll
  for (int u = 0; u < kPiecesPerThread; ++u) {
    const int sgm = kPiecesPerThread * tid + u;
    raw[u] = sgm < nseg ? seg_count[(int64_t)bh * nseg + sgm] : 0;
  }
  int c = cand_count[bg];
  c = c < 0 ? 0 : (c > s.cand_cap ? s.cand_cap : c);
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  const int ksel = kb < c ? kb : c;
  int64_t S = *seg_rows_in;                          // chosen by the scoring pass of this step
  S = S < 64 ? 64 : S;
  const int64_t pg = group_start[bg];
  const int64_t w_first = pg / S;
  auto piece_lo = [&](int sgm) {                     // first slot of piece sgm within my group
    const int64_t lo = (w_first + sgm) * S - pg;
    return lo < 0 ? (int64_t)0 : lo;
  };
  auto piece_hi = [&](int sgm) {
    const int64_t hi = (w_first + sgm + 1) * S - pg;
    return hi > c ? (int64_t)c : hi;
  };

  // exclusive prefix of the piece counts (kPiecesPerThread consecutive pieces per thread); the counts
  // were loaded above, before the group's geometry was known: entries of pieces that do not exist
  // hold stale values and are masked here
  int cntp[kPiecesPerThread];
  int cnt = 0;
#pragma unroll
  for (int u = 0; u < kPiecesPerThread; ++u) {
    const int sgm = kPiecesPerThread * tid + u;
    cntp[u] = 0;
    if (sgm < nseg) {
      const int64_t room = piece_hi(sgm) - piece_lo(sgm);   // rows the piece covers
      if (room > 0) {
        const int v = raw[u] < 0 ? 0 : raw[u];
        cntp[u] = v > room ? (int)room : v;
      }
    }
    cnt += cntp[u];
  }
  const int inc = wave_inclusive_sum(cnt);
  if (lane == 63) wtot[wv] = inc;
  __syncthreads();
  int base = 0, n = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const int t = wtot[w];
    base += w < wv ? t : 0;
    n += t;
  }
  {
    int off = base + inc - cnt;
#pragma unroll
    for (int u = 0; u < kPiecesPerThread; ++u) {
      seg_off[kPiecesPerThread * tid + u] = off;
      off += cntp[u];
    }
  }
  if (n < ksel || n > cap) {                        // block-uniform
    if (tid == 0) {
      redo_g[bg] = 1;
      redo_h[bh] = 1;
      if (rescored) atomicAdd(rescored, 1);          // heads sent to the unfiltered pass since the last poll
    }
    return;
  }
  int32_t* oi = topk_idx + (int64_t)bh * s.kmax;
  float* os = topk_score ? topk_score + (int64_t)bh * s.kmax : nullptr;
  for (int i = ksel + tid; i < s.kmax; i += NT) {   // padding
    oi[i] = -1;
    if (os) os[i] = 0.f;
  }
  if (ksel == 0) {
    if (tid == 0) thr_state[bh] = -INFINITY;
    return;
  }
  __syncthreads();
  const float* sc = score + (int64_t)bh * score_stride;
  const int32_t* sl = slot_in + (int64_t)bh * score_stride;
  // Flat copy of the survivors into LDS: element e lies in the piece found by a binary search over
  // the offsets.  kGatherBatch elements per thread are searched together (fixed trip count, no
  // branches) and all their loads are issued before the first is used, so the copy costs a few
  // memory round trips instead of one per element.
  int np = (int)((pg + c - 1) / S - w_first) + 1;   // pieces my group was cut into
  np = np < 1 ? 1 : (np > nseg ? nseg : np);
  np = np < kPiecesPerThread * NT ? np : kPiecesPerThread * NT;
  int top = 1;
  while (top < np) top <<= 1;
  constexpr int kGatherBatch = 12;
  float my_lo = FLT_MAX, my_hi = -FLT_MAX;             // range of the elements this thread copies
  for (int e0 = tid; e0 < n; e0 += kGatherBatch * NT) {
    int pc[kGatherBatch];
#pragma unroll
    for (int u = 0; u < kGatherBatch; ++u) pc[u] = 0;
    for (int half = top >> 1; half >= 1; half >>= 1) {   // last piece with seg_off <= e (seg_off[0] = 0)
#pragma unroll
      for (int u = 0; u < kGatherBatch; ++u) {
        const int mid = pc[u] + half;
        const int e = e0 + u * NT;
        if (mid < np && seg_off[mid] <= e) pc[u] = mid;
      }
    }
    float v[kGatherBatch];
    int32_t ps[kGatherBatch];
#pragma unroll
    for (int u = 0; u < kGatherBatch; ++u) {
      const int e = e0 + u * NT;
      v[u] = 0.f;
      ps[u] = 0;
      if (e < n) {
        const int64_t src = piece_lo(pc[u]) + (e - seg_off[pc[u]]);
        v[u] = sc[src];
        ps[u] = sl[src];                              // the row position, written by the scoring pass
      }
    }
#pragma unroll
    for (int u = 0; u < kGatherBatch; ++u) {
      const int e = e0 + u * NT;
      if (e < n) {
        const float x = sanitize(v[u]);
        cache[e] = x;
        lslot[e] = ps[u];
        my_lo = fminf(my_lo, x);
        my_hi = fmaxf(my_hi, x);
      }
    }
  }
  __syncthreads();
  select_body<true, NT, true>(sm, cache, nullptr, n, ksel, lslot, nullptr, oi, os, thr_state + bh, my_lo, my_hi);
}


static int select_cache_elems(const Shape& s, bool gather) {
  const int rows_max = gather ? s.cand_cap : s.Lcap;
  const int e = rows_max < kCacheElems ? rows_max : kCacheElems;
  return (e + 63) & ~63;
}

int filter_list_cap(const Shape& s) {
  int cap = 4 * s.kmax;
  if (cap < 1024) cap = 1024;
  if (cap > 7680) {             // 60 KB of LDS: two workgroups per CU ...
    cap = 7680;
    // ... unless the budget itself needs more room: twice the budget, up to 128 KB (one workgroup per CU)
    if (2 * s.kmax > cap) cap = 2 * s.kmax < 16384 ? 2 * s.kmax : 16384;
  }
  return cap;
}

// Called once per context at creation: the score cache needs more dynamic LDS than the default limit.
hipError_t configure_select(const Shape& s) {
  hipError_t e = hipFuncSetAttribute((const void*)k_select, hipFuncAttributeMaxDynamicSharedMemorySize, kCacheElems * 4);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute((const void*)k_filter_select, hipFuncAttributeMaxDynamicSharedMemorySize,
                             filter_list_cap(s) * 8);
}

hipError_t launch_select(const Shape& s, const float* score, int64_t score_stride, const int32_t* cand,
                         const int32_t* count, const int32_t* k, int32_t* topk_idx, float* topk_score,
                         const int32_t* only_if, float* thr_state, const int32_t* skip_if, const int32_t* seq_lens,
                         hipStream_t st) {
  // A conditional launch (only_if) is expected to find nothing to do: it streams from global memory
  // instead of reserving the LDS cache, so that its workgroups are cheap to place and retire.
  const int ce = only_if ? 0 : select_cache_elems(s, cand != nullptr);
  hipLaunchKernelGGL(k_select, dim3(s.B * s.Hq), dim3(kSelThreads), (size_t)ce * 4, st, s, score, score_stride, cand,
                     count, k, topk_idx, topk_score, ce, only_if, thr_state, skip_if, seq_lens);
  return hipGetLastError();
}

hipError_t launch_filter_select(const Shape& s, const float* score, const int32_t* slot_in, int64_t score_stride,
                                const int32_t* seg_count, const int32_t* seg_rows, int nseg,
                                const int32_t* cand_count, const int64_t* group_start, int64_t* line_total,
                                const int32_t* k, int32_t* topk_idx, float* topk_score,
                                float* thr_state, int32_t* redo_g, int32_t* redo_h, const int32_t* skip_if,
                                int32_t* rescored, hipStream_t st) {
  const int cap = filter_list_cap(s);
  hipLaunchKernelGGL(k_filter_select, dim3(s.B * s.Hq), dim3(kFilterSelThreads), (size_t)cap * 8, st, s, score, slot_in,
                     score_stride, seg_count, seg_rows, nseg, cand_count, group_start, line_total, k, topk_idx, topk_score, thr_state, redo_g,
                     redo_h, cap, skip_if, rescored);
  return hipGetLastError();
}

}  // namespace lfps
