// S1 — candidate set of one (request, KV group) from the previous step's per-head Top-k
// (Alg. 1 lines 6-7 in the memoryless form: vertical = same position, slash = position + 1,
// both widened by the expansion radius; Sec. 4.2 stages 2-3).
//
// One workgroup per (b, g).  The set is built as a bitmap over positions in LDS: every valid
// previous index ORs the (2r+2)-bit window [i-r, i+r+1] (clipped to [0, n)) into the words it
// spans, which also dedupes within a head and across the G heads of the group.  A popcount +
// block scan then assigns each word its output offset and the set bits are emitted in ascending
// order, so the output is sorted and identical from run to run.  (The G <= 4 heads per group
// that the library supports are unrolled.)
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

// Dynamic LDS: bitmap words [W] followed by the exclusive output offset of every word [W].
__global__ __launch_bounds__(kCandThreads) void k_candidates(Shape s, const int32_t* __restrict__ prev_topk,
                                                             const int32_t* __restrict__ kk,
                                                             const int32_t* __restrict__ seq_lens,
                                                             int32_t* __restrict__ cand,
                                                             int32_t* __restrict__ cand_count,
                                                             int32_t* __restrict__ flags,
                                                             int32_t* __restrict__ redo_g,
                                                             int32_t* __restrict__ redo_h) {
  extern __shared__ uint32_t lds[];
  __shared__ int wave_tot[kCandThreads / 64];
  const int bg = blockIdx.x, b = bg / s.Hkv, g = bg % s.Hkv;
  const int tid = threadIdx.x;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  // first kernel of a step: clear the group's "needs the unfiltered pass" marks
  if (redo_g && tid == 0) redo_g[bg] = 0;
  if (redo_h && tid < s.G) redo_h[(int64_t)b * s.Hq + (int64_t)g * s.G + tid] = 0;
  const int W = (n + 31) >> 5;
  uint32_t* bm = lds;
  uint32_t* woff = lds + ((s.Lcap + 31) >> 5);

  // The previous Top-k of the group's heads: issue every load of a round before touching LDS, so
  // their latencies overlap (4 heads x 2 entries per thread and round).
  constexpr int kU = 2;
  const int r = s.radius;
  const int32_t* pt = prev_topk + ((int64_t)b * s.Hq + (int64_t)g * s.G) * s.kmax;
  int first_ids[4 * kU];
#pragma unroll
  for (int h = 0; h < 4; ++h)
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int j = tid + u * kCandThreads;
      first_ids[h * kU + u] = (h < s.G && j < kb) ? pt[(int64_t)h * s.kmax + j] : -1;
    }

  for (int w = tid; w < W; w += kCandThreads) bm[w] = 0u;
  __syncthreads();

#pragma unroll
  for (int e = 0; e < 4 * kU; ++e) {
    const int i = first_ids[e];
    if (i >= 0 && i < n) {
      const int lo = i - r < 0 ? 0 : i - r;
      const int64_t hi64 = (int64_t)i + r + 1;
      set_bit_range(bm, lo, hi64 > n - 1 ? n - 1 : (int)hi64);
    }
  }
  for (int j0 = kU * kCandThreads; j0 < kb; j0 += kU * kCandThreads) {   // budgets beyond 2048 per head
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

  // exclusive output offset of every word: each thread scans a contiguous slice of words,
  // then a block scan of the slice totals
  const int wpt = (W + kCandThreads - 1) / kCandThreads;
  const int w_lo = tid * wpt, w_hi = (w_lo + wpt < W) ? w_lo + wpt : W;
  int cnt = 0;
  for (int w = w_lo; w < w_hi; ++w) {
    woff[w] = (uint32_t)cnt;
    cnt += __popc(bm[w]);
  }
  const int lane = tid & 63, wv = tid >> 6;
  int inc = cnt;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    int o = __shfl_up(inc, d);
    if (lane >= d) inc += o;
  }
  if (lane == 63) wave_tot[wv] = inc;
  __syncthreads();
  int base = 0, total = 0;
#pragma unroll
  for (int i = 0; i < kCandThreads / 64; ++i) {
    int t = wave_tot[i];
    if (i < wv) base += t;
    total += t;
  }
  const int slice_off = base + inc - cnt;
  for (int w = w_lo; w < w_hi; ++w) woff[w] += (uint32_t)slice_off;
  __syncthreads();

  // emit: consecutive threads expand consecutive words, so a wave writes one contiguous stretch
  int32_t* out = cand + (int64_t)bg * s.cand_cap;
  for (int w = tid; w < W; w += kCandThreads) {
    uint32_t bits = bm[w];
    int off = (int)woff[w];
    while (bits) {
      const int p = __ffs(bits) - 1;
      bits &= bits - 1;
      if (off < s.cand_cap) out[off] = (w << 5) + p;
      ++off;
    }
  }
  if (tid == 0) {
    if (total > s.cand_cap) {
      atomicOr(flags, LFPS_FLAG_CAND_OVERFLOW);
      total = s.cand_cap;
    }
    cand_count[bg] = total;
  }
}

static size_t candidates_lds_bytes(const Shape& s) {
  size_t b = ((size_t)(s.Lcap + 31) / 32) * 8;     // bitmap + per-word offsets
  return b < 8 ? 8 : b;
}

// Called once per context at creation: raises the kernel's dynamic-LDS limit when the bitmap of
// the longest sequence needs more than the default 64 KB.
hipError_t configure_candidates(const Shape& s) {
  const size_t lds_bytes = candidates_lds_bytes(s);
  if (lds_bytes > 32 * 1024)
    return hipFuncSetAttribute((const void*)k_candidates, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  return hipSuccess;
}

hipError_t launch_candidates(const Shape& s, const int32_t* prev_topk, const int32_t* k, const int32_t* seq_lens,
                             int32_t* cand, int32_t* cand_count, int32_t* flags, int32_t* redo_g, int32_t* redo_h,
                             hipStream_t st) {
  hipLaunchKernelGGL(k_candidates, dim3(s.B * s.Hkv), dim3(kCandThreads), candidates_lds_bytes(s), st, s, prev_topk, k,
                     seq_lens, cand, cand_count, flags, redo_g, redo_h);
  return hipGetLastError();
}

}  // namespace lfps
