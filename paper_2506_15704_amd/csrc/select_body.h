// The select shared by the kernels that end in "the k best of a head's scored rows" (S3; Alg. 1 line 8 /
// Sec. 1 Step 2): LDS state, the histogram select itself and the streaming variant.  See select.hip for the
// description of the five passes.
#pragma once
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
                                            float pre_hi = -FLT_MAX, int n_valid = 0x7FFFFFFF,
                                            float* top_out = nullptr) {
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
  if (top_out) *top_out = hi;               // the largest score of the head: it is always among the selected
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
// Returns the head's largest score.
template <int NT>
static __device__ __noinline__ float select_stream(SelectShared<NT>& sm, const float* __restrict__ sc, int c, int ksel,
                                                   const int32_t* __restrict__ cbg, int32_t* __restrict__ oi,
                                                   float* __restrict__ os, float* __restrict__ thr_out, int n_valid) {
  float top = 0.f;
  select_body<false, NT>(sm, nullptr, sc, c, ksel, nullptr, cbg, oi, os, thr_out, FLT_MAX, -FLT_MAX, n_valid, &top);
  return top;
}

}  // namespace lfps
