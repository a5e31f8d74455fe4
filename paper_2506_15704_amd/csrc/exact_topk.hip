// Exact Top-k baseline (Sec. 1 Steps 1-2 over all keys; the "exact Top-k" upper bound of Sec. 5), set-up of its
// fast form.  Writing a score for every row and selecting from that array costs a second and further passes over
// 4 bytes per row and head; instead the baseline takes the machinery of the chained steps:
//   1. a strided sample of each group's rows is scored (the gather kernel) and, per head, the sample score of a
//      rank chosen so that, with near certainty, between k rows and the select's list capacity reach it becomes a
//      threshold;
//   2. the filtered scoring kernel streams all rows once and keeps only those that reach the threshold;
//   3. the select picks the exact k best from the survivors; a head whose survivors are fewer than k (or too many
//      for the on-chip list) is rescored the plain way, so the result is always the exact Top-k.
#include "lfps_internal.h"

namespace lfps {

// grid B*Hkv, 256 threads.
__global__ __launch_bounds__(256) void k_dense_prep(Shape s, const int32_t* __restrict__ seq_lens,
                                                    const int32_t* __restrict__ kk, int ns_max, int list_cap,
                                                    int32_t* __restrict__ x_cnt, int64_t* __restrict__ x_start,
                                                    int32_t* __restrict__ x_nsg, int32_t* __restrict__ x_ns,
                                                    int32_t* __restrict__ x_rank, int32_t* __restrict__ sample) {
  __shared__ long long part[256];
  const int bg = blockIdx.x, b = bg / s.Hkv, g = bg % s.Hkv, tid = threadIdx.x;
  const int n_groups = s.B * s.Hkv;
  auto len = [&](int bb) {
    int n = seq_lens[bb];
    return n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  };
  // my place on the line: rows of the groups before mine (and, for the last group, the line's length)
  long long before = 0, all = 0;
  for (int i = tid; i < n_groups; i += 256) {
    const long long n_i = len(i / s.Hkv);
    before += i < bg ? n_i : 0;
    all += n_i;
  }
  part[tid] = before;
  __syncthreads();
  for (int d = 128; d >= 1; d >>= 1) {
    if (tid < d) part[tid] += part[tid + d];
    __syncthreads();
  }
  const long long my_start = part[0];
  __syncthreads();
  part[tid] = all;
  __syncthreads();
  for (int d = 128; d >= 1; d >>= 1) {
    if (tid < d) part[tid] += part[tid + d];
    __syncthreads();
  }
  const long long total = part[0];
  const int n = len(b);
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  kb = kb < n ? kb : n;
  // The sample and the rank r of the sample score that becomes the threshold.  With p = k / n the rows of the whole
  // context above the r-th best of ns sampled scores number about n r / ns, with a relative spread of 1 / sqrt(r).
  // That count must land between k (else too few survive) and the select's list capacity: it is aimed at t k with
  // t = min(2, (1 + cap / k) / 2), the middle of the two limits, and r is made large enough for both to lie
  // z = 4.5 standard deviations away (a miss costs a rescoring of that head, never a wrong result); the sample
  // size follows as ns = (r / t) n / k.  A context no larger than that is sampled whole, with r = k.
  int ns = n, r = kb;
  if (kb > 0 && n > kb) {
    const float c = (float)list_cap / (float)kb;
    const float t = fminf(2.f, 0.5f * (1.f + c));
    if (t > 1.05f) {
      const float sr = 4.5f * t / (t - 1.f);
      r = (int)ceilf(sr * sr);
      const float want = ((float)r / t) * ((float)n / (float)kb);
      int cap_ns = ns_max < s.cand_cap ? ns_max : s.cand_cap;
      cap_ns = cap_ns < n ? cap_ns : n;
      if (want < (float)cap_ns) {
        ns = (int)ceilf(want);
      } else {                                   // no room for the wanted sample: what fits, with the rank that aims at t k
        ns = cap_ns;
        r = ns < n ? (int)(t * (float)ns * (float)kb / (float)n) : kb;
      }
      if (ns >= n) {
        ns = n;
        r = kb;
      }
    } else {                                     // the list barely holds the budget: no room to aim, sample everything
      ns = n < s.cand_cap ? n : s.cand_cap;
      r = ns == n ? kb : 1;
    }
  }
  r = r < 1 ? 1 : r;
  r = r > s.kmax ? s.kmax : r;
  r = r > ns ? ns : r;
  if (tid == 0) {
    x_cnt[bg] = n;
    x_start[bg] = my_start;
    if (bg == n_groups - 1) x_start[n_groups] = total;
    x_nsg[bg] = ns;
    if (g == 0) {
      x_ns[b] = ns;
      x_rank[b] = r;
    }
  }
  int32_t* out = sample + (int64_t)bg * s.cand_cap;
  for (int i = tid; i < ns; i += 256) out[i] = (int)(((long long)i * n) / ns);
}

hipError_t launch_dense_prep(const Shape& s, const int32_t* seq_lens, const int32_t* k, int ns_max, int list_cap, int32_t* x_cnt,
                             int64_t* x_start, int32_t* x_nsg, int32_t* x_ns, int32_t* x_rank, int32_t* sample,
                             hipStream_t st) {
  hipLaunchKernelGGL(k_dense_prep, dim3(s.B * s.Hkv), dim3(256), 0, st, s, seq_lens, k, ns_max, list_cap, x_cnt, x_start, x_nsg,
                     x_ns, x_rank, sample);
  return hipGetLastError();
}

}  // namespace lfps
