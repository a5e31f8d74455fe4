// S4 — sparse attention over the selected rows (Eq. 1), and the full-attention baseline
// (Sec. 1 with idx = every row; the "full attention" upper bound of Sec. 5).
//
// Sparse: the scores of the selected rows are already known (from S3, or recomputed by the
// per-head score kernel), so the softmax maximum is known before any V row is read and the
// partial sums of the waves merge by plain addition.  One workgroup of 4, 8 or 16 waves per
// (b, h): wave w gathers its share of the head's rows, 16 lanes per V row, 16-byte loads, sixteen
// independent row loads in flight per wave; the partial sums meet in LDS and the output row is
// written once (no partials in global memory, no second kernel).
//
// Full: split-K over contiguous row ranges with the G heads of a group sharing every K and V
// row; running (max, sum, acc) per lane group, merged with the online-softmax rule.
#include "attend.h"

namespace lfps {

constexpr int kAttnThreads = 256;       // full attention

// grid B*Hq, kSparseWaves waves per workgroup
template <typename T, int kSparseWaves, bool kPaged>
__global__ __launch_bounds__(kSparseWaves * 64) void k_sparse_attn(Shape s, const T* __restrict__ V, int64_t stride_b,
                                                                int64_t stride_h, int64_t stride_n, KvPage pg,
                                                                const int32_t* __restrict__ seq_lens,
                                                                const int32_t* __restrict__ idx,
                                                                const float* __restrict__ idx_score,
                                                                const int32_t* __restrict__ kk,
                                                                float* __restrict__ out,
                                                                const int32_t* __restrict__ skip_if) {
  __shared__ AttendShared sm;
  const int bh = head_of_block(s, blockIdx.x);
  if (skip_if && skip_if[bh] != 0) return;            // bypassed head: the gate wrote its output row
  const int b = bh / s.Hq, h = bh % s.Hq, g = h / s.G;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  attend_rows<T, kSparseWaves, kPaged>(sm, V, stride_b, stride_h, stride_n, pg, b, g, n, kb,
                                       idx + (int64_t)bh * s.kmax, idx_score + (int64_t)bh * s.kmax, false, 0.f,
                                       out + (int64_t)bh * kD);
}

template <typename T>
static hipError_t launch_sparse_t(const Shape& s, const KvView& kv, const int32_t* idx, const float* idx_score,
                                  const int32_t* k, float* out, const int32_t* skip_if, hipStream_t st) {
  // as many waves per head as keep every head's workgroup resident at once (256 CUs x 32 waves)
  const int heads = s.B * s.Hq;
  const T* V = (const T*)kv.v;
#define LFPS_LAUNCH_SPARSE_P(NW, PAGED)                                                                        \
  hipLaunchKernelGGL((k_sparse_attn<T, NW, PAGED>), dim3(heads), dim3(NW * 64), 0, st, s, V, kv.stride_b,      \
                     kv.stride_h, kv.stride_n, kv.page, kv.seq_lens, idx, idx_score, k, out, skip_if)
#define LFPS_LAUNCH_SPARSE(NW)          \
  if (kv.page.table) {                  \
    LFPS_LAUNCH_SPARSE_P(NW, true);     \
  } else {                              \
    LFPS_LAUNCH_SPARSE_P(NW, false);    \
  }
  if (heads * 16 <= 4096) {
    LFPS_LAUNCH_SPARSE(16)
  } else if (heads * 8 <= 4096) {
    LFPS_LAUNCH_SPARSE(8)
  } else {
    LFPS_LAUNCH_SPARSE(4)
  }
#undef LFPS_LAUNCH_SPARSE
#undef LFPS_LAUNCH_SPARSE_P
  return hipGetLastError();
}

hipError_t launch_sparse_attn(const Shape& s, int dtype, const KvView& kv, const int32_t* idx, const float* idx_score,
                              const int32_t* k, float* out, const int32_t* skip_if, hipStream_t st) {
  if (dtype == LFPS_BF16 && kv.v_fp8) return launch_sparse_t<uint8_t>(s, kv, idx, idx_score, k, out, skip_if, st);
  if (dtype == LFPS_F16) return launch_sparse_t<_Float16>(s, kv, idx, idx_score, k, out, skip_if, st);
  return dtype == LFPS_BF16 ? launch_sparse_t<uint16_t>(s, kv, idx, idx_score, k, out, skip_if, st)
                            : launch_sparse_t<float>(s, kv, idx, idx_score, k, out, skip_if, st);
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
template <typename TK, typename T, int G, bool kPaged>
__global__ __launch_bounds__(kAttnThreads) void k_full_attn(Shape s, const float* __restrict__ q,
                                                            const TK* __restrict__ K, const T* __restrict__ V,
                                                            int64_t stride_b, int64_t stride_h, int64_t stride_n,
                                                            KvPage pg, const int32_t* __restrict__ seq_lens,
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
  using Rows = RowMap<kPaged>;
  const TK* Kbg = K + Rows::base(b, g, stride_b, stride_h) + 8 * j;
  const T* Vbg = V + Rows::base(b, g, stride_b, stride_h) + 8 * j;

  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m[h] = -INFINITY;
    l[h] = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[h][c] = 0.f;
  }

  constexpr int U = 4;                       // rows per lane group and tile
  // Wave w takes rows r_begin + 16*(4*i + w) + 4*u + rs of tile i.  Two tiles are kept in flight: the loads of
  // the next one are issued before the current one is used, as raw cache elements (half or a quarter of the
  // registers of their fp32 form).  Rows past the end are read from the last row and weigh nothing, so no
  // load sits behind a branch.
  struct Tile {
    Raw8<TK> k[U];
    Raw8<T> v[U];
    bool ok[U];
  };
  auto issue = [&](Tile& t, int r0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int r = r0 + 4 * u + rs;
      t.ok[u] = r < r_end;
      r = t.ok[u] ? r : r_end - 1;
      const int64_t off = Rows::offset(pg, Rows::phys(pg, b, r), stride_b, stride_n);
      t.k[u].load(Kbg + off);
      t.v[u].load(Vbg + off);
    }
  };
  auto consume = [&](const Tile& t) {
    float kx[U][8], vx[U][8];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      t.k[u].get(kx[u]);
      t.v[u].get(vx[u]);
      ok[u] = t.ok[u];
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
  };
  Tile ta, tb;
  issue(ta, r_begin + 16 * wave);
  for (int r0 = r_begin + 16 * wave; r0 < r_end; r0 += 128) {
    issue(tb, r0 + 64);
    consume(ta);
    issue(ta, r0 + 128);
    consume(tb);
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

template <typename TK, typename T>
static hipError_t launch_full_t(const Shape& s, const float* q, const KvView& kv, float* part, int n_split,
                                hipStream_t st) {
  dim3 grid(n_split, s.B * s.Hkv), block(kAttnThreads);
  const float scale = 0.08838834764831845f;
  const TK* K = (const TK*)kv.k;
  const T* V = (const T*)kv.v;
#define LFPS_LAUNCH_FULL_P(GG, PAGED)                                                                           \
  hipLaunchKernelGGL((k_full_attn<TK, T, GG, PAGED>), grid, block, 0, st, s, q, K, V, kv.stride_b, kv.stride_h, \
                     kv.stride_n, kv.page, kv.seq_lens, part, n_split, scale)
#define LFPS_LAUNCH_FULL(GG)          \
  if (kv.page.table) {                \
    LFPS_LAUNCH_FULL_P(GG, true);     \
  } else {                            \
    LFPS_LAUNCH_FULL_P(GG, false);    \
  }
  switch (s.G) {
    case 1: LFPS_LAUNCH_FULL(1); break;
    case 2: LFPS_LAUNCH_FULL(2); break;
    case 4: LFPS_LAUNCH_FULL(4); break;
    default: return hipErrorInvalidValue;
  }
#undef LFPS_LAUNCH_FULL
#undef LFPS_LAUNCH_FULL_P
  return hipGetLastError();
}

hipError_t launch_full_attn(const Shape& s, int dtype, const float* q, const KvView& kv, float* part, int n_split,
                            hipStream_t st) {
  if (dtype == LFPS_BF16 && kv.k_fp8 && kv.v_fp8) return launch_full_t<uint8_t, uint8_t>(s, q, kv, part, n_split, st);
  if (dtype == LFPS_BF16 && kv.k_fp8) return launch_full_t<uint8_t, uint16_t>(s, q, kv, part, n_split, st);
  if (dtype == LFPS_BF16 && kv.v_fp8) return launch_full_t<uint16_t, uint8_t>(s, q, kv, part, n_split, st);
  if (dtype == LFPS_F16) return launch_full_t<_Float16, _Float16>(s, q, kv, part, n_split, st);
  return dtype == LFPS_BF16 ? launch_full_t<uint16_t, uint16_t>(s, q, kv, part, n_split, st)
                            : launch_full_t<float, float>(s, q, kv, part, n_split, st);
}

hipError_t launch_full_merge(const Shape& s, const int32_t* seq_lens, const float* part, int n_split, float* out,
                             hipStream_t st) {
  hipLaunchKernelGGL(k_full_merge, dim3(s.B * s.Hq), dim3(kD), 0, st, s, seq_lens, part, n_split, out);
  return hipGetLastError();
}

}  // namespace lfps
