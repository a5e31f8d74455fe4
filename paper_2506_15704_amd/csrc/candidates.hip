// S1 — candidate set of one (request, KV group) from the previous step's per-head Top-k
// (Alg. 1 lines 6-7 in the memoryless form: vertical = same position, slash = position + 1,
// both widened by the expansion radius; Sec. 4.2 stages 2-3).
//
// One workgroup per (b, g).  The set is built as a bitmap over positions in LDS: every valid
// previous index ORs the (2r+2)-bit window [i-r, i+r+1] (clipped to [0, n)) into the words it
// spans, which also dedupes within a head and across the G heads of the group.  A popcount +
// block scan then assigns each word its output offset and the set bits are emitted in ascending
// order, so the output is sorted and identical from run to run.  (The G <= 4 heads per group
// that the library supports are unrolled.)  Capacity: 64 * 1024 rounds of words is far above what
// the LDS bitmap can hold, so the bitmap size is the limit.
#include "lfps_internal.h"

namespace lfps {

constexpr int kCandThreads = 1024;

__device__ __forceinline__ void set_bit_range(uint32_t* bm, int lo, int hi) {  // inclusive, lo <= hi
  int w0 = lo >> 5, w1 = hi >> 5;
  for (int w = w0; w <= w1; ++w) {
    int a = (w == w0) ? (lo & 31) : 0;
    int b = (w == w1) ? (hi & 31) : 31;
    uint32_t m = (b == 31 ? 0xFFFFFFFFu : ((1u << (b + 1)) - 1u)) & ~((1u << a) - 1u);
    atomicOr(&bm[w], m);
  }
}

// Emits the set bits of the LDS bitmap bm[0:W] as ascending positions into cand[bg, :] and leaves the
// count in cand_count[bg] (truncated to cand_cap with the overflow flag raised).  All threads of the
// workgroup call it after a barrier that follows the last write to the bitmap.  Emission goes in rounds
// of 64 consecutive words, one round per wave at a time: (a) set bits per round, (b) exclusive offsets
// of the rounds by a block scan, (c) per round every lane expands its word into a wave-private LDS
// stage at the lane's offset within the round, then the wave copies the stage out with consecutive
// lanes writing consecutive entries.  `part` of `nparts` workgroups that share the group emit every
// nparts-th round.  group_start / line_total (or NULL): the group's place on the line of all candidate slots that
// the filtered scoring pass cuts into equal parts: the group adds its (truncated) count to *line_total (the caller
// has left it at zero) and keeps the value before the addition.  The addition is issued as soon as the count is
// known and its result stored after the emission, so its round trip hides behind the emission.
__device__ __forceinline__ void emit_bitmap(const Shape& s, const uint32_t* bm, int W, uint32_t* rcnt, uint16_t* stage,
                                            int* wave_tot, int bg, int part, int nparts, int32_t* __restrict__ cand,
                                            int32_t* __restrict__ cand_count, int32_t* __restrict__ flags,
                                            int64_t* __restrict__ group_start,
                                            unsigned long long* __restrict__ line_total) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = tid >> 6;
  const int nr = (W + 63) >> 6;                                  // rounds (<= kCandThreads, checked at creation)
  for (int r_ = wv; r_ < nr; r_ += kCandThreads / 64) {
    const int w = r_ * 64 + lane;
    const int c_ = wave_inclusive_sum(w < W ? __popc(bm[w]) : 0);
    if (lane == 63) rcnt[r_] = (uint32_t)c_;                      // the round's total
  }
  __syncthreads();
  int cnt = tid < nr ? (int)rcnt[tid] : 0;
  const int inc = wave_inclusive_sum(cnt);
  if (lane == 63) wave_tot[wv] = inc;
  __syncthreads();
  int base = 0, total = 0;
#pragma unroll
  for (int i = 0; i < kCandThreads / 64; ++i) {
    int t = wave_tot[i];
    if (i < wv) base += t;
    total += t;
  }
  if (tid < nr) rcnt[tid] = (uint32_t)(base + inc - cnt);        // now the exclusive offset of round tid
  const bool places = tid == 0 && part == 0 && group_start != nullptr;
  unsigned long long place = 0;
  if (places) place = atomicAdd(line_total, (unsigned long long)(total > s.cand_cap ? s.cand_cap : total));
  __syncthreads();

  int32_t* out = cand + (int64_t)bg * s.cand_cap;
  uint16_t* st = stage + wv * 2048;
  for (int r_ = wv * nparts + part; r_ < nr; r_ += (kCandThreads / 64) * nparts) {
    const int w = r_ * 64 + lane;
    uint32_t bits = w < W ? bm[w] : 0u;
    const int c_ = __popc(bits);
    const int incl = wave_inclusive_sum(c_);
    const int tot = __shfl(incl, 63);
    int o_ = incl - c_;
    while (bits) {
      const int p = __ffs(bits) - 1;
      bits &= bits - 1;
      st[o_++] = (uint16_t)((lane << 5) | p);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int ro = (int)rcnt[r_];
    for (int e = lane; e < tot; e += 64) {
      const uint32_t v = st[e];
      if (ro + e < s.cand_cap) out[ro + e] = (((r_ << 6) + (int)(v >> 5)) << 5) + (int)(v & 31u);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  if (tid == 0 && part == 0) {
    int kept = total;
    if (kept > s.cand_cap) {
      atomicOr(flags, LFPS_FLAG_CAND_OVERFLOW);
      kept = s.cand_cap;
    }
    cand_count[bg] = kept;
  }
  if (places) group_start[bg] = (int64_t)place;
}

// Dynamic LDS: bitmap words [ceil(Lcap/32)], round counts/offsets [ceil(words/64)], then a
// 4 KB stage per wave (64 words x 32 bits as 16-bit (word-in-round, bit) codes).
__global__ __launch_bounds__(kCandThreads) void k_candidates(Shape s, const int32_t* __restrict__ prev_topk,
                                                             const int32_t* __restrict__ kk,
                                                             const int32_t* __restrict__ seq_lens,
                                                             int32_t* __restrict__ cand,
                                                             int32_t* __restrict__ cand_count,
                                                             int32_t* __restrict__ flags,
                                                             int64_t* __restrict__ group_start,
                                                             unsigned long long* __restrict__ line_total) {
  extern __shared__ uint32_t lds[];
  __shared__ int wave_tot[kCandThreads / 64];
  // gridDim.x workgroups share one (b, g): each builds the whole bitmap (cheap) and emits every
  // gridDim.x-th round of words, so that small batches still spread over the chip.
  const int bg = blockIdx.y, b = bg / s.Hkv, g = bg % s.Hkv;
  const int part = blockIdx.x, nparts = gridDim.x;
  const int tid = threadIdx.x;
  uint32_t* bm = lds;
  const int words_cap = (s.Lcap + 31) >> 5;
  uint32_t* rcnt = lds + words_cap;
  uint16_t* stage = reinterpret_cast<uint16_t*>(rcnt + ((words_cap + 63) >> 6));

  // The previous Top-k of the group's heads: issue every load of a round before touching LDS, so
  // their latencies overlap (4 heads x 2 entries per thread and round).  The first round is fetched
  // up to the row length kmax, not the request's budget, and masked when used: its loads then wait
  // for nothing (neither the budget nor the length), and the three fetches share one round trip.
  constexpr int kU = 2;
  const int r = s.radius;
  const int32_t* pt = prev_topk + ((int64_t)b * s.Hq + (int64_t)g * s.G) * s.kmax;
  int first_ids[4 * kU];
#pragma unroll
  for (int h = 0; h < 4; ++h)
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int j = tid + u * kCandThreads;
      first_ids[h * kU + u] = (h < s.G && j < s.kmax) ? pt[(int64_t)h * s.kmax + j] : -1;
    }
  for (int w = tid; w < words_cap; w += kCandThreads) bm[w] = 0u;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  const int W = (n + 31) >> 5;
  __syncthreads();

#pragma unroll
  for (int e = 0; e < 4 * kU; ++e) {
    const int i = (tid + (e % kU) * kCandThreads < kb) ? first_ids[e] : -1;
    if (i >= 0 && i < n) {
      const int lo = i - r < 0 ? 0 : i - r;
      const int64_t hi64 = (int64_t)i + r + 1;
      set_bit_range(bm, lo, hi64 > n - 1 ? n - 1 : (int)hi64);
    }
  }
  for (int j0 = kU * kCandThreads; j0 < kb; j0 += kU * kCandThreads) {   // budgets beyond kU * kCandThreads per head
    int ids[4 * kU];
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const int j = j0 + tid + u * kCandThreads;
        ids[h * kU + u] = (h < s.G && j < kb) ? pt[(int64_t)h * s.kmax + j] : -1;
      }
#pragma unroll
    for (int e = 0; e < 4 * kU; ++e) {
      const int i = ids[e];
      if (i >= 0 && i < n) {
        const int lo = i - r < 0 ? 0 : i - r;
        const int64_t hi64 = (int64_t)i + r + 1;
        set_bit_range(bm, lo, hi64 > n - 1 ? n - 1 : (int)hi64);
      }
    }
  }
  if (tid == 0 && n > 0) {
    if (s.n_recent > 0) set_bit_range(bm, n - s.n_recent < 0 ? 0 : n - s.n_recent, n - 1);
    if (s.n_sink > 0) set_bit_range(bm, 0, (s.n_sink > n ? n : s.n_sink) - 1);
  }
  __syncthreads();

  emit_bitmap(s, bm, W, rcnt, stage, wave_tot, bg, part, nparts, cand, cand_count, flags, group_start, line_total);
}

// ----------------------------------------------------------------------------- score-table form
// Candidate set of one (request, KV group) from the per-head flag bitmaps that the table scan left
// (Eq. 7 and Eq. 9): f0 marks the initial candidates of a head (a table entry above its kurtosis
// threshold), fm the positions whose vertical or slash score exceeds the table mean.  For every
// head the initial candidates are widened by the offsets -r ... r+1 (bit shifts across word
// boundaries) and masked with fm; the heads are OR-ed; the newest and the sink rows are added.
__global__ __launch_bounds__(kCandThreads) void k_table_candidates(Shape s, const uint32_t* __restrict__ f0,
                                                                   const uint32_t* __restrict__ fm, int flag_words,
                                                                   const int32_t* __restrict__ seq_lens,
                                                                   int32_t* __restrict__ cand,
                                                                   int32_t* __restrict__ cand_count,
                                                                   int32_t* __restrict__ flags,
                                                                   int64_t* __restrict__ group_start,
                                                                   unsigned long long* __restrict__ line_total) {
  extern __shared__ uint32_t lds[];
  __shared__ int wave_tot[kCandThreads / 64];
  const int bg = blockIdx.y, b = bg / s.Hkv, g = bg % s.Hkv;
  const int part = blockIdx.x, nparts = gridDim.x;
  const int tid = threadIdx.x;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  const int W = (n + 31) >> 5;
  uint32_t* bm = lds;
  const int words_cap = (s.Lcap + 31) >> 5;
  uint32_t* rcnt = lds + words_cap;
  uint16_t* stage = reinterpret_cast<uint16_t*>(rcnt + ((words_cap + 63) >> 6));
  const int r = s.radius;
  for (int w = tid; w < W; w += kCandThreads) {
    // the words of all heads (G <= 4) are fetched before any is used: sixteen loads in flight per thread
    uint32_t lo[4], mid[4], hi[4], mean[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const bool live = h < s.G;
      const int64_t row = ((int64_t)b * s.Hq + (int64_t)g * s.G + (live ? h : 0)) * flag_words;
      lo[h] = (live && w > 0) ? f0[row + w - 1] : 0u;
      mid[h] = live ? f0[row + w] : 0u;
      hi[h] = (live && w + 1 < W) ? f0[row + w + 1] : 0u;
      mean[h] = live ? fm[row + w] : 0u;
    }
    uint32_t acc = 0u;
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      uint32_t d = mid[h];
      for (int e = 1; e <= r + 1; ++e) d |= (mid[h] << e) | (lo[h] >> (32 - e));      // j = i + e
      for (int e = 1; e <= r; ++e) d |= (mid[h] >> e) | (hi[h] << (32 - e));           // j = i - e
      acc |= d & mean[h];
    }
    bm[w] = acc;
  }
  __syncthreads();
  if (tid == 0 && n > 0) {
    if (s.n_recent > 0) set_bit_range(bm, n - s.n_recent < 0 ? 0 : n - s.n_recent, n - 1);
    if (s.n_sink > 0) set_bit_range(bm, 0, (s.n_sink > n ? n : s.n_sink) - 1);
  }
  __syncthreads();
  emit_bitmap(s, bm, W, rcnt, stage, wave_tot, bg, part, nparts, cand, cand_count, flags, group_start, line_total);
}

static size_t candidates_lds_bytes(const Shape& s) {
  const size_t words = ((size_t)s.Lcap + 31) / 32;
  return words * 4 + ((words + 63) / 64) * 4 + (kCandThreads / 64) * 4096;   // bitmap + round offsets + stages
}

// Called once per context at creation: raises the kernel's dynamic-LDS limit when the bitmap of
// the longest sequence needs more than the default 64 KB.
hipError_t configure_candidates(const Shape& s) {
  const size_t lds_bytes = candidates_lds_bytes(s);
  if (lds_bytes > 32 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)k_candidates, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void*)k_table_candidates, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  }
  return hipSuccess;
}

hipError_t launch_candidates(const Shape& s, const int32_t* prev_topk, const int32_t* k, const int32_t* seq_lens,
                             int32_t* cand, int32_t* cand_count, int32_t* flags, int64_t* group_start,
                             int64_t* line_total, hipStream_t st) {
  int nparts = 256 / (s.B * s.Hkv);                    // one workgroup per CU in total (82 KB of LDS each)
  nparts = nparts < 1 ? 1 : (nparts > 8 ? 8 : nparts);
  hipLaunchKernelGGL(k_candidates, dim3(nparts, s.B * s.Hkv), dim3(kCandThreads), candidates_lds_bytes(s), st, s,
                     prev_topk, k, seq_lens, cand, cand_count, flags, group_start,
                     reinterpret_cast<unsigned long long*>(line_total));
  return hipGetLastError();
}

hipError_t launch_table_candidates(const Shape& s, const uint32_t* f0, const uint32_t* fm, int flag_words,
                                   const int32_t* seq_lens, int32_t* cand, int32_t* cand_count, int32_t* flags,
                                   int64_t* group_start, int64_t* line_total, hipStream_t st) {
  int nparts = 256 / (s.B * s.Hkv);
  nparts = nparts < 1 ? 1 : (nparts > 8 ? 8 : nparts);
  hipLaunchKernelGGL(k_table_candidates, dim3(nparts, s.B * s.Hkv), dim3(kCandThreads), candidates_lds_bytes(s), st, s,
                     f0, fm, flag_words, seq_lens, cand, cand_count, flags, group_start,
                     reinterpret_cast<unsigned long long*>(line_total));
  return hipGetLastError();
}

}  // namespace lfps
