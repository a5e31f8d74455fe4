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
#include "candidates.h"

namespace lfps {

constexpr int kCandThreads = 1024;

// gridDim.x workgroups share one (b, g), so that small batches still spread over the chip.
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
  const int bg = blockIdx.y, b = bg / s.Hkv, g = bg % s.Hkv;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  const int32_t* pt = prev_topk + ((int64_t)b * s.Hq + (int64_t)g * s.G) * s.kmax;
  candidates_from_topk<kCandThreads>(s, lds, wave_tot, pt, n, kb, bg, blockIdx.x, gridDim.x, cand, cand_count, flags,
                                     group_start, line_total);
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
  emit_bitmap<kCandThreads>(s, bm, W, rcnt, stage, wave_tot, bg, part, nparts, cand, cand_count, flags, group_start,
                            line_total);
}

// Called once per context at creation: raises the kernel's dynamic-LDS limit when the bitmap of
// the longest sequence needs more than the default 64 KB.
hipError_t configure_candidates(const Shape& s) {
  const size_t lds_bytes = candidates_lds_bytes(s, kCandThreads);
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
  hipLaunchKernelGGL(k_candidates, dim3(nparts, s.B * s.Hkv), dim3(kCandThreads), candidates_lds_bytes(s, kCandThreads), st, s,
                     prev_topk, k, seq_lens, cand, cand_count, flags, group_start,
                     reinterpret_cast<unsigned long long*>(line_total));
  return hipGetLastError();
}

hipError_t launch_table_candidates(const Shape& s, const uint32_t* f0, const uint32_t* fm, int flag_words,
                                   const int32_t* seq_lens, int32_t* cand, int32_t* cand_count, int32_t* flags,
                                   int64_t* group_start, int64_t* line_total, hipStream_t st) {
  int nparts = 256 / (s.B * s.Hkv);
  nparts = nparts < 1 ? 1 : (nparts > 8 ? 8 : nparts);
  hipLaunchKernelGGL(k_table_candidates, dim3(nparts, s.B * s.Hkv), dim3(kCandThreads), candidates_lds_bytes(s, kCandThreads), st, s,
                     f0, fm, flag_words, seq_lens, cand, cand_count, flags, group_start,
                     reinterpret_cast<unsigned long long*>(line_total));
  return hipGetLastError();
}

}  // namespace lfps
