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
// select_attend.hip applies the same steps to the short (score, position) lists that the filtered scoring
// pass leaves per head, and runs the attention over the selected rows in the same kernel.
#include "select_body.h"

namespace lfps {

__global__ __launch_bounds__(kSelThreads) void k_select(Shape s, const float* __restrict__ score,
                                                        int64_t score_stride, const int32_t* __restrict__ cand,
                                                        const int32_t* __restrict__ count_arr,
                                                        const int32_t* __restrict__ kk, int32_t* __restrict__ topk_idx,
                                                        float* __restrict__ topk_score, int cache_elems,
                                                        float* __restrict__ thr_state,
                                                        const int32_t* __restrict__ skip_if,
                                                        const int32_t* __restrict__ seq_lens) {
  __shared__ SelectShared<kSelThreads> sm;
  extern __shared__ float cache[];
  const int bh = blockIdx.x, b = bh / s.Hq, h = bh % s.Hq, g = h / s.G;
  const int tid = threadIdx.x;
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
  return configure_select_attend(s);
}

hipError_t launch_select(const Shape& s, const float* score, int64_t score_stride, const int32_t* cand,
                         const int32_t* count, const int32_t* k, int32_t* topk_idx, float* topk_score,
                         float* thr_state, const int32_t* skip_if, const int32_t* seq_lens, hipStream_t st) {
  const int ce = select_cache_elems(s, cand != nullptr);
  hipLaunchKernelGGL(k_select, dim3(s.B * s.Hq), dim3(kSelThreads), (size_t)ce * 4, st, s, score, score_stride, cand,
                     count, k, topk_idx, topk_score, ce, thr_state, skip_if, seq_lens);
  return hipGetLastError();
}

}  // namespace lfps
