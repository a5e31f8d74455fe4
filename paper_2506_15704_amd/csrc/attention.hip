// S4 — sparse attention over the selected rows (Eq. 1), and the full-attention baseline
// (Sec. 1 with idx = every row; the "full attention" upper bound of Sec. 5).
//
// Sparse: the scores of the selected rows are already known (from S3, or recomputed by the
// per-head score kernel), so the softmax maximum is known before any V row is read and every
// split of a head uses the same reference; partial sums then merge by plain addition.
// Split s of head (b, h) gathers rows idx[256 s, 256 s + 256): 16 lanes per V row, 16-byte loads,
// sixteen independent row loads in flight per wave.
//
// Full: split-K over contiguous row ranges with the G heads of a group sharing every K and V
// row; running (max, sum, acc) per lane group, merged with the online-softmax rule.
#include "lfps_internal.h"

namespace lfps {

constexpr int kAttnThreads = 256;
constexpr int kRowsPerSplit = 256;   // sparse attention: rows per workgroup

template <typename T>
__device__ __forceinline__ void load8(const T* p, float x[8]) {
  if constexpr (sizeof(T) == 2) {
    u32x4 w = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      x[2 * c] = bf16_lo(w[c]);
      x[2 * c + 1] = bf16_hi(w[c]);
    }
  } else {
    float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
}

int sparse_attn_splits(const Shape& s) { return (s.kmax + kRowsPerSplit - 1) / kRowsPerSplit; }

// grid (n_split, B*Hq); part [B*Hq, n_split, D+1]
template <typename T>
__global__ __launch_bounds__(kAttnThreads) void k_sparse_attn(Shape s, const T* __restrict__ V, int64_t stride_b,
                                                              int64_t stride_h, int64_t stride_n,
                                                              const int32_t* __restrict__ seq_lens,
                                                              const int32_t* __restrict__ idx,
                                                              const float* __restrict__ idx_score,
                                                              const int32_t* __restrict__ kk, float* __restrict__ part,
                                                              int n_split) {
  __shared__ float red[4][kD];
  __shared__ float redm[4], redl[4];
  const int bh = blockIdx.y, b = bh / s.Hq, h = bh % s.Hq, g = h / s.G;
  const int split = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, rs = lane >> 4;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  if (split * kRowsPerSplit >= kb) return;
  const int32_t* ih = idx + (int64_t)bh * s.kmax;
  const float* sh = idx_score + (int64_t)bh * s.kmax;

  // softmax reference: the largest score among the head's valid rows
  float m = -INFINITY;
  for (int i = tid; i < kb; i += kAttnThreads) {
    int r = ih[i];
    if (r >= 0 && r < n) m = fmaxf(m, sh[i]);
  }
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) m = fmaxf(m, __shfl_xor(m, d));
  if (lane == 0) redm[wave] = m;
  __syncthreads();
  m = fmaxf(fmaxf(redm[0], redm[1]), fmaxf(redm[2], redm[3]));

  const int my_i = split * kRowsPerSplit + wave * 64 + lane;
  int my_row = -1;
  float my_p = 0.f;
  if (my_i < kb) {
    int r = ih[my_i];
    if (r >= 0 && r < n) {
      my_row = r;
      my_p = __expf(sh[my_i] - m);
    }
  }
  const T* Vbg = V + (int64_t)b * stride_b + (int64_t)g * stride_h + 8 * j;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    int row = __shfl(my_row, 4 * t + rs);
    float p = __shfl(my_p, 4 * t + rs);
    float x[8];
    load8(Vbg + (int64_t)(row < 0 ? 0 : row) * stride_n, x);
    p = row < 0 ? 0.f : p;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = fmaf(p, x[c], acc[c]);
  }
  float l = my_p;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) l += __shfl_xor(l, d);
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    acc[c] += __shfl_xor(acc[c], 16);
    acc[c] += __shfl_xor(acc[c], 32);
  }
  if (rs == 0) {
#pragma unroll
    for (int c = 0; c < 8; ++c) red[wave][8 * j + c] = acc[c];
  }
  if (lane == 0) redl[wave] = l;
  __syncthreads();
  float* po = part + ((int64_t)bh * n_split + split) * (kD + 1);
  if (tid < kD) po[tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
  if (tid == kD) po[kD] = (redl[0] + redl[1]) + (redl[2] + redl[3]);
}

// grid B*Hq, 128 threads
__global__ __launch_bounds__(kD) void k_attn_merge(Shape s, const int32_t* __restrict__ kk,
                                                   const float* __restrict__ part, int n_split,
                                                   float* __restrict__ out) {
  const int bh = blockIdx.x, b = bh / s.Hq, c = threadIdx.x;
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  const int nv = (kb + kRowsPerSplit - 1) / kRowsPerSplit;
  float a = 0.f, l = 0.f;
  for (int sp = 0; sp < nv; ++sp) {
    const float* p = part + ((int64_t)bh * n_split + sp) * (kD + 1);
    a += p[c];
    l += p[kD];
  }
  out[(int64_t)bh * kD + c] = l > 0.f ? a / l : 0.f;
}

hipError_t launch_sparse_attn(const Shape& s, int dtype, const KvView& kv, const int32_t* idx, const float* idx_score,
                              const int32_t* k, float* part, hipStream_t st) {
  const int ns = sparse_attn_splits(s);
  dim3 grid(ns, s.B * s.Hq), block(kAttnThreads);
  if (dtype == LFPS_BF16)
    hipLaunchKernelGGL((k_sparse_attn<uint16_t>), grid, block, 0, st, s, (const uint16_t*)kv.v, kv.stride_b,
                       kv.stride_h, kv.stride_n, kv.seq_lens, idx, idx_score, k, part, ns);
  else
    hipLaunchKernelGGL((k_sparse_attn<float>), grid, block, 0, st, s, (const float*)kv.v, kv.stride_b, kv.stride_h,
                       kv.stride_n, kv.seq_lens, idx, idx_score, k, part, ns);
  return hipGetLastError();
}

hipError_t launch_attn_merge(const Shape& s, const int32_t* k, const float* part, float* out, hipStream_t st) {
  hipLaunchKernelGGL(k_attn_merge, dim3(s.B * s.Hq), dim3(kD), 0, st, s, k, part, sparse_attn_splits(s), out);
  return hipGetLastError();
}

// ============================================================================ full attention
int full_attn_splits(const Shape& s) {
  int ns = (2048 + s.B * s.Hkv - 1) / (s.B * s.Hkv);
  int by_len = (s.Lcap + 255) / 256;       // at least 256 rows per split
  if (ns > by_len) ns = by_len;
  if (ns > kMaxSplits) ns = kMaxSplits;
  return ns < 1 ? 1 : ns;
}

__device__ __forceinline__ int rows_per_split(int n, int n_split) { return (((n + n_split - 1) / n_split) + 15) & ~15; }

// grid (n_split, B*Hkv); part [B*Hkv, n_split, G, D+2]: acc[D], m, l
template <typename T, int G>
__global__ __launch_bounds__(kAttnThreads) void k_full_attn(Shape s, const float* __restrict__ q,
                                                            const T* __restrict__ K, const T* __restrict__ V,
                                                            int64_t stride_b, int64_t stride_h, int64_t stride_n,
                                                            const int32_t* __restrict__ seq_lens,
                                                            float* __restrict__ part, int n_split, float scale) {
  __shared__ float red_acc[4][G][kD];
  __shared__ float red_m[4][G], red_l[4][G];
  const int bg = blockIdx.y, b = bg / s.Hkv, g = bg % s.Hkv, split = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, rs = lane >> 4;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  const int rps = rows_per_split(n, n_split);
  const int r_begin = split * rps;
  const int r_end = (r_begin + rps < n) ? r_begin + rps : n;
  if (r_begin >= n) return;

  float qr[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const float* qh = q + ((int64_t)b * s.Hq + (int64_t)g * G + h) * kD + 8 * j;
#pragma unroll
    for (int c = 0; c < 8; ++c) qr[h][c] = qh[c] * scale;
  }
  const T* Kbg = K + (int64_t)b * stride_b + (int64_t)g * stride_h + 8 * j;
  const T* Vbg = V + (int64_t)b * stride_b + (int64_t)g * stride_h + 8 * j;

  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m[h] = -INFINITY;
    l[h] = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[h][c] = 0.f;
  }

  constexpr int U = 4;                       // rows in flight per lane group
  // wave w takes rows r_begin + 16*(4*i + w) + 4*u + rs
  for (int r0 = r_begin + 16 * wave; r0 < r_end; r0 += 64) {
    float kx[U][8], vx[U][8];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int r = r0 + 4 * u + rs;
      ok[u] = r < r_end;
      r = ok[u] ? r : r_end - 1;
      load8(Kbg + (int64_t)r * stride_n, kx[u]);
      load8(Vbg + (int64_t)r * stride_n, vx[u]);
    }
    float sc[U][G];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float a = qr[h][0] * kx[u][0];
#pragma unroll
        for (int c = 1; c < 8; ++c) a = fmaf(qr[h][c], kx[u][c], a);
        sc[u][h] = a;
      }
#pragma unroll
    for (int d = 1; d < 16; d <<= 1)
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int h = 0; h < G; ++h) sc[u][h] += __shfl_xor(sc[u][h], d);
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float mx = m[h];
#pragma unroll
      for (int u = 0; u < U; ++u) mx = ok[u] ? fmaxf(mx, sc[u][h]) : mx;
      // a lane group whose rows all lie past the end still has mx = -inf: keep its empty state
      const float alpha = (mx == -INFINITY) ? 1.f : __expf(m[h] - mx);   // exp(-inf) = 0 on the first tile
      float p[U];
#pragma unroll
      for (int u = 0; u < U; ++u) p[u] = ok[u] ? __expf(sc[u][h] - mx) : 0.f;
      float ls = l[h] * alpha;
#pragma unroll
      for (int u = 0; u < U; ++u) ls += p[u];
      l[h] = ls;
      m[h] = mx;
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        float a = acc[h][c] * alpha;
#pragma unroll
        for (int u = 0; u < U; ++u) a = fmaf(p[u], vx[u][c], a);
        acc[h][c] = a;
      }
    }
  }

  // merge the 4 lane groups of the wave, then the 4 waves
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float mx = fmaxf(m[h], __shfl_xor(m[h], 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float a = (m[h] == -INFINITY) ? 0.f : __expf(m[h] - mx);   // lane groups that saw no row
    float ls = l[h] * a;
    ls += __shfl_xor(ls, 16);
    ls += __shfl_xor(ls, 32);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      float v = acc[h][c] * a;
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      acc[h][c] = v;
    }
    m[h] = mx;
    l[h] = ls;
  }
  if (rs == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
#pragma unroll
      for (int c = 0; c < 8; ++c) red_acc[wave][h][8 * j + c] = acc[h][c];
      if (j == 0) {
        red_m[wave][h] = m[h];
        red_l[wave][h] = l[h];
      }
    }
  }
  __syncthreads();
  float* po = part + ((int64_t)bg * n_split + split) * G * (kD + 2);
  for (int e = tid; e < G * kD; e += kAttnThreads) {
    const int h = e / kD, c = e % kD;
    float mx = fmaxf(fmaxf(red_m[0][h], red_m[1][h]), fmaxf(red_m[2][h], red_m[3][h]));
    float a = 0.f, ls = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = (red_m[w][h] == -INFINITY) ? 0.f : __expf(red_m[w][h] - mx);
      a = fmaf(red_acc[w][h][c], f, a);
      ls = fmaf(red_l[w][h], f, ls);
    }
    po[h * (kD + 2) + c] = a;
    if (c == 0) {
      po[h * (kD + 2) + kD] = mx;
      po[h * (kD + 2) + kD + 1] = ls;
    }
  }
}

// grid B*Hq, 128 threads
__global__ __launch_bounds__(kD) void k_full_merge(Shape s, const int32_t* __restrict__ seq_lens,
                                                   const float* __restrict__ part, int n_split,
                                                   float* __restrict__ out) {
  const int bh = blockIdx.x, b = bh / s.Hq, h = bh % s.Hq, g = h / s.G, hg = h % s.G, c = threadIdx.x;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  if (n == 0) {
    out[(int64_t)bh * kD + c] = 0.f;
    return;
  }
  const int rps = rows_per_split(n, n_split);
  const int nv = (n + rps - 1) / rps;
  const float* pb = part + ((int64_t)(b * s.Hkv + g) * n_split) * s.G * (kD + 2) + (int64_t)hg * (kD + 2);
  float mx = -INFINITY;
  for (int sp = 0; sp < nv; ++sp) mx = fmaxf(mx, pb[(int64_t)sp * s.G * (kD + 2) + kD]);
  float a = 0.f, l = 0.f;
  for (int sp = 0; sp < nv; ++sp) {
    const float* p = pb + (int64_t)sp * s.G * (kD + 2);
    const float f = __expf(p[kD] - mx);
    a = fmaf(p[c], f, a);
    l = fmaf(p[kD + 1], f, l);
  }
  out[(int64_t)bh * kD + c] = a / l;
}

template <typename T>
static hipError_t launch_full_t(const Shape& s, const float* q, const KvView& kv, float* part, int n_split,
                                hipStream_t st) {
  dim3 grid(n_split, s.B * s.Hkv), block(kAttnThreads);
  const float scale = 0.08838834764831845f;
  const T* K = (const T*)kv.k;
  const T* V = (const T*)kv.v;
  switch (s.G) {
    case 1:
      hipLaunchKernelGGL((k_full_attn<T, 1>), grid, block, 0, st, s, q, K, V, kv.stride_b, kv.stride_h, kv.stride_n,
                         kv.seq_lens, part, n_split, scale);
      break;
    case 2:
      hipLaunchKernelGGL((k_full_attn<T, 2>), grid, block, 0, st, s, q, K, V, kv.stride_b, kv.stride_h, kv.stride_n,
                         kv.seq_lens, part, n_split, scale);
      break;
    case 4:
      hipLaunchKernelGGL((k_full_attn<T, 4>), grid, block, 0, st, s, q, K, V, kv.stride_b, kv.stride_h, kv.stride_n,
                         kv.seq_lens, part, n_split, scale);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_full_attn(const Shape& s, int dtype, const float* q, const KvView& kv, float* part, int n_split,
                            hipStream_t st) {
  return dtype == LFPS_BF16 ? launch_full_t<uint16_t>(s, q, kv, part, n_split, st)
                            : launch_full_t<float>(s, q, kv, part, n_split, st);
}

hipError_t launch_full_merge(const Shape& s, const int32_t* seq_lens, const float* part, int n_split, float* out,
                             hipStream_t st) {
  hipLaunchKernelGGL(k_full_merge, dim3(s.B * s.Hq), dim3(kD), 0, st, s, seq_lens, part, n_split, out);
  return hipGetLastError();
}

}  // namespace lfps
