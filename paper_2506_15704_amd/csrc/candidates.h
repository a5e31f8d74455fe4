// Building blocks of the candidate kernels (S1), for a workgroup of NT threads: the LDS bitmap over positions, its
// emission as an ascending list, and the memoryless rule itself (Alg. 1 lines 6-7: the previous Top-k of the
// group's heads, each position widened to [i - r, i + r + 1]).
#pragma once
#include "lfps_internal.h"

namespace lfps {

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
// of 64 consecutive words, one round per wave at a time (NT = threads of the workgroup): (a) set bits per round, (b) exclusive offsets
// of the rounds by a block scan, (c) per round every lane expands its word into a wave-private LDS
// stage at the lane's offset within the round, then the wave copies the stage out with consecutive
// lanes writing consecutive entries.  `part` of `nparts` workgroups that share the group emit every
// nparts-th round.  group_start / line_total (or NULL): the group's place on the line of all candidate slots that
// the filtered scoring pass cuts into equal parts: the group adds its (truncated) count to *line_total (the caller
// has left it at zero) and keeps the value before the addition.  The addition is issued as soon as the count is
// known and its result stored after the emission, so its round trip hides behind the emission.
template <int NT>
__device__ __forceinline__ void emit_bitmap(const Shape& s, const uint32_t* bm, int W, uint32_t* rcnt, uint16_t* stage,
                                            int* wave_tot, int bg, int part, int nparts, int32_t* __restrict__ cand,
                                            int32_t* __restrict__ cand_count, int32_t* __restrict__ flags,
                                            int64_t* __restrict__ group_start,
                                            unsigned long long* __restrict__ line_total) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = tid >> 6;
  const int nr = (W + 63) >> 6;                                  // rounds (<= NT, checked at creation)
  for (int r_ = wv; r_ < nr; r_ += NT / 64) {
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
  for (int i = 0; i < NT / 64; ++i) {
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
  for (int r_ = wv * nparts + part; r_ < nr; r_ += (NT / 64) * nparts) {
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

// Dynamic LDS the functions below need for NT threads: bitmap words [ceil(Lcap/32)], round counts/offsets
// [ceil(words/64)], then a 4 KB stage per wave (64 words x 32 bits as 16-bit (word-in-round, bit) codes).
inline size_t candidates_lds_bytes(const Shape& s, int nt) {
  const size_t words = ((size_t)s.Lcap + 31) / 32;
  return words * 4 + ((words + 63) / 64) * 4 + (size_t)(nt / 64) * 4096;
}

// The candidate set of group bg = (b, g) from pt = the Top-k rows [G, kmax] of its heads (entries < 0 and >= n are
// skipped), for a request of n rows and budget kb: vertical = same position, slash = position + 1, both widened by
// the radius; the newest n_recent and the first n_sink rows are always in.  Written as an ascending list to
// cand[bg, :] with its length in cand_count[bg]; `part` of `nparts` workgroups that share the group each build the
// whole bitmap (cheap) and emit every nparts-th round of words.  All NT threads call; lds as sized above; wave_tot:
// NT / 64 ints of LDS.  See emit_bitmap for group_start / line_total.
template <int NT>
__device__ __forceinline__ void candidates_from_topk(const Shape& s, uint32_t* lds, int* wave_tot,
                                                     const int32_t* pt, int n, int kb, int bg, int part, int nparts,
                                                     int32_t* __restrict__ cand, int32_t* __restrict__ cand_count,
                                                     int32_t* __restrict__ flags, int64_t* __restrict__ group_start,
                                                     unsigned long long* __restrict__ line_total) {
  const int tid = threadIdx.x;
  uint32_t* bm = lds;
  const int words_cap = (s.Lcap + 31) >> 5;
  uint32_t* rcnt = lds + words_cap;
  uint16_t* stage = reinterpret_cast<uint16_t*>(rcnt + ((words_cap + 63) >> 6));
  const int W = (n + 31) >> 5;
  const int r = s.radius;
  // Every load of a round is issued before LDS is touched, so their latencies overlap (4 heads x kU entries per
  // thread and round).  A round is fetched up to the row length kmax, not the budget, and masked when used, and the
  // first round is unconditional and precedes the clearing of the bitmap: its loads wait neither for the budget nor
  // for the length, should the caller's fetches of those still be on their way.
  constexpr int kU = 2048 / NT;
  int ids[4 * kU];
  auto fetch = [&](int j0) {
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const int j = j0 + tid + u * NT;
        ids[h * kU + u] = (h < s.G && j < s.kmax) ? pt[(int64_t)h * s.kmax + j] : -1;
      }
  };
  fetch(0);
  for (int w = tid; w < words_cap; w += NT) bm[w] = 0u;
  __syncthreads();
  for (int j0 = 0;;) {
#pragma unroll
    for (int e = 0; e < 4 * kU; ++e) {
      const int i = (j0 + tid + (e % kU) * NT < kb) ? ids[e] : -1;
      if (i >= 0 && i < n) {
        const int lo = i - r < 0 ? 0 : i - r;
        const int64_t hi64 = (int64_t)i + r + 1;
        set_bit_range(bm, lo, hi64 > n - 1 ? n - 1 : (int)hi64);
      }
    }
    j0 += kU * NT;
    if (j0 >= kb) break;
    fetch(j0);
  }
  if (tid == 0 && n > 0) {
    if (s.n_recent > 0) set_bit_range(bm, n - s.n_recent < 0 ? 0 : n - s.n_recent, n - 1);
    if (s.n_sink > 0) set_bit_range(bm, 0, (s.n_sink > n ? n : s.n_sink) - 1);
  }
  __syncthreads();
  emit_bitmap<NT>(s, bm, W, rcnt, stage, wave_tot, bg, part, nparts, cand, cand_count, flags, group_start, line_total);
}

}  // namespace lfps
