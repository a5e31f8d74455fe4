// S3 — per query head, the k best of the scored rows (Alg. 1 line 8 / Sec. 1 Step 2).
//
// One workgroup per (b, h).  Scores are mapped to order-preserving 32-bit keys and the k-th
// largest key is found exactly by a most-significant-digit radix descent (11 + 11 + 10 bits)
// with LDS histograms; the scores are streamed from global memory/L2 on every pass because a
// head can have more scores than LDS holds.  The final pass writes every row above the k-th
// key, plus as many rows equal to it as are still needed, lowest position first.  Output is
// compacted in row order (ballot + prefix counts, no atomics), so it is ascending in position
// and identical from run to run.
#include "lfps_internal.h"

namespace lfps {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kBins = 2048;

__device__ __forceinline__ int lanes_below(uint64_t m) {   // set bits of m at lanes lower than mine
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}

__global__ __launch_bounds__(kSelThreads) void k_select(Shape s, const float* __restrict__ score,
                                                        int64_t score_stride, const int32_t* __restrict__ cand,
                                                        const int32_t* __restrict__ count_arr,
                                                        const int32_t* __restrict__ kk, int32_t* __restrict__ topk_idx,
                                                        float* __restrict__ topk_score) {
  __shared__ uint32_t hist[kBins];
  __shared__ uint32_t wsum[kSelWaves];
  __shared__ uint32_t sh_prefix, sh_need;
  __shared__ uint32_t cnt_gt[kSelWaves], cnt_eq[kSelWaves];

  const int bh = blockIdx.x, b = bh / s.Hq, h = bh % s.Hq, g = h / s.G;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
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
  if (ksel == 0) return;

  const float* sc = score + (int64_t)bh * score_stride;
  const int32_t* cbg = gather ? cand + ((int64_t)b * s.Hkv + g) * s.cand_cap : nullptr;

  // ---- radix descent for the ksel-th largest key
  uint32_t prefix = 0, mask = 0, need = (uint32_t)ksel;
  const int shifts[3] = {21, 10, 0};
  const int widths[3] = {11, 11, 10};
#pragma unroll 1
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = shifts[pass];
    const uint32_t dmask = (1u << widths[pass]) - 1u;
    for (int i = tid; i < kBins; i += kSelThreads) hist[i] = 0u;
    __syncthreads();
    for (int i = tid; i < c; i += kSelThreads) {
      uint32_t key = f2key(sc[i]);
      if (((key ^ prefix) & mask) == 0u) atomicAdd(&hist[(key >> shift) & dmask], 1u);
    }
    __syncthreads();
    // thread t owns bins 2t (low) and 2t+1 (high); suffix sums from the top bin down
    const uint32_t lo = hist[2 * tid], hi = hist[2 * tid + 1];
    const uint32_t mine = lo + hi;
    uint32_t inc = mine;   // inclusive suffix sum over lanes >= mine within the wave
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      uint32_t o = __shfl_down(inc, d);
      if (lane + d < 64) inc += o;
    }
    if (lane == 0) wsum[wv] = inc;
    __syncthreads();
    uint32_t above_waves = 0;
    for (int w = wv + 1; w < kSelWaves; ++w) above_waves += wsum[w];
    const uint32_t suffix_incl = above_waves + inc;      // keys in bins >= 2t
    const uint32_t suffix_excl = suffix_incl - mine;     // keys in bins >  2t+1
    if (suffix_incl >= need && suffix_excl < need) {     // exactly one thread
      uint32_t digit, above;
      if (suffix_excl + hi >= need) {
        digit = 2 * tid + 1;
        above = suffix_excl;
      } else {
        digit = 2 * tid;
        above = suffix_excl + hi;
      }
      sh_prefix = prefix | (digit << shift);
      sh_need = need - above;
    }
    __syncthreads();
    prefix = sh_prefix;
    need = sh_need;
    mask |= dmask << shift;
    __syncthreads();
  }
  const uint32_t thr = prefix;   // the ksel-th largest key; `need` rows equal to it are taken

  // ---- ordered compaction: wave w owns rows [w*chunk, (w+1)*chunk)
  const int chunk = (((c + kSelWaves - 1) / kSelWaves) + 63) & ~63;
  const int r0 = wv * chunk, r1 = (r0 + chunk < c) ? r0 + chunk : c;
  uint32_t ngt = 0, neq = 0;
  for (int base = r0; base < r1; base += 64) {          // wave-uniform trip count
    const int i = base + lane;
    const bool in = i < r1;
    const uint32_t key = in ? f2key(sc[i]) : 0u;
    ngt += __popcll(__ballot(in && key > thr));
    neq += __popcll(__ballot(in && key == thr));
  }
  if (lane == 0) {
    cnt_gt[wv] = ngt;
    cnt_eq[wv] = neq;
  }
  __syncthreads();
  uint32_t gt_before = 0, eq_before = 0;
  for (int w = 0; w < wv; ++w) {
    gt_before += cnt_gt[w];
    eq_before += cnt_eq[w];
  }
  uint32_t eq_run = eq_before;
  uint32_t out_run = gt_before + (eq_before < need ? eq_before : need);
  for (int base = r0; base < r1; base += 64) {
    const int i = base + lane;
    const bool in = i < r1;
    const float v = in ? sc[i] : 0.f;
    const uint32_t key = in ? f2key(v) : 0u;
    const bool gt = in && key > thr, eq = in && key == thr;
    const uint64_t m_eq = __ballot(eq);
    const bool take = gt || (eq && eq_run + lanes_below(m_eq) < need);
    const uint64_t m_take = __ballot(take);
    if (take) {
      uint32_t pos = out_run + lanes_below(m_take);
      if (pos < (uint32_t)ksel) {
        oi[pos] = gather ? cbg[i] : i;
        if (os) os[pos] = v;
      }
    }
    eq_run += __popcll(m_eq);
    out_run += __popcll(m_take);
  }
}

hipError_t launch_select(const Shape& s, const float* score, int64_t score_stride, const int32_t* cand,
                         const int32_t* count, const int32_t* k, int32_t* topk_idx, float* topk_score,
                         hipStream_t st) {
  hipLaunchKernelGGL(k_select, dim3(s.B * s.Hq), dim3(kSelThreads), 0, st, s, score, score_stride, cand, count, k,
                     topk_idx, topk_score);
  return hipGetLastError();
}

}  // namespace lfps
