// Device code shared by the kernels that end in sparse attention (Eq. 1 over a head's selected rows).
#pragma once
#include "lfps_internal.h"

namespace lfps {

// Workgroups are dealt to the 8 XCDs round-robin (workgroup i runs on XCD i % 8) and every XCD has
// its own L2.  The heads of a KV group select largely the same rows, so the G workgroups of a group
// are given ids that differ by multiples of 8: they run on one XCD at about the same time and a V
// row fetched for one head is an L2 hit for the others.  Returns the head (b * Hq + h) of a workgroup.
__device__ __forceinline__ int head_of_block(const Shape& s, int block) {
  const int n_kvg = s.B * s.Hkv;                   // KV groups in the launch
  if (n_kvg % 8 != 0) return block;
  const int xcd = block & 7, slot = block >> 3;
  return ((slot / s.G) * 8 + xcd) * s.G + slot % s.G;
}

// The list of a head is cut into kAttendChunks equal chunks (a multiple of 64 entries each); every chunk's partial
// sum is formed by one wave in list order and the chunks are added in chunk order, whatever the number of waves
// (a wave takes kAttendChunks / NW consecutive chunks): the output row does not depend on the launch shape.
constexpr int kAttendChunks = 16;

struct AttendShared {
  float red[kAttendChunks][kD];
  float redl[kAttendChunks];
  float redm[kAttendChunks];
};

// out_row[0:D] = sum_i softmax_i(sh[i]) V[b, g, ih[i]] over the entries i < kb with 0 <= ih[i] < n, computed by the
// NW waves of the workgroup (every thread calls; ends with the row written by the first D threads; zeros when
// no entry is valid).  The scores are known, so the softmax reference (their maximum over the valid entries) is
// fixed before any V row is read and the partial sums add; a caller that already knows it passes it
// (have_m, m_known) and saves the pass over the scores.  16 lanes per V row, 16-byte loads.
template <typename T, int NW, bool kPaged>
__device__ __forceinline__ void attend_rows(AttendShared& sm, const T* __restrict__ V, int64_t stride_b,
                                            int64_t stride_h, int64_t stride_n, const KvPage& pg, int b, int g, int n,
                                            int kb, const int32_t* ih, const float* sh, bool have_m, float m_known,
                                            float* __restrict__ out_row) {
  static_assert(kAttendChunks % NW == 0, "a wave takes a whole number of chunks");
  constexpr int kPerWave = kAttendChunks / NW;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, rs = lane >> 4;

  // wave w takes entries [r0, r1) of the head's index list: its kPerWave chunks
  const int chunk = (((kb + kAttendChunks - 1) / kAttendChunks) + 63) & ~63;
  const int r0 = wave * kPerWave * chunk, r1 = r0 + kPerWave * chunk < kb ? r0 + kPerWave * chunk : kb;

  using Rows = RowMap<kPaged>;
  auto entry = [&](int i, int& row, float& sv) {          // list entry i of my lane: physical row or -1, score
    row = -1;
    sv = 0.f;
    if (i < r1) {
      const int r = ih[i];
      sv = sh[i];
      if (r >= 0 && r < n) row = Rows::phys(pg, b, r);
    }
  };
  int first_row = -1;                 // as a physical row (never negative), or -1 for "no row"
  float first_s = -INFINITY;
  float m = m_known;
  if (have_m) {
    entry(r0 + lane, first_row, first_s);
  } else {
    // softmax reference: the largest score among the head's valid rows.  Each lane looks at the
    // entries it will own in the loop below (first 64-entry tile kept in registers).
    m = -INFINITY;
    for (int i = r0 + lane; i < r1; i += 64) {
      const int r = ih[i];
      const float sv = sh[i];
      const bool ok = r >= 0 && r < n;
      if (i < r0 + 64) {
        first_row = ok ? Rows::phys(pg, b, r) : -1;
        first_s = sv;
      }
      if (ok) m = fmaxf(m, sv);
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) m = fmaxf(m, __shfl_xor(m, d));
    if (lane == 0) sm.redm[wave] = m;
    __syncthreads();
    m = sm.redm[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) m = fmaxf(m, sm.redm[w]);
  }

  const T* Vbg = V + Rows::base(b, g, stride_b, stride_h) + 8 * j;
  // A tile = 64 entries of the list, one per lane (row, weight); the entries of the next tile are fetched
  // before the rows of the current one.  The rows of a tile are read in two batches of eight loads per lane
  // (32 rows per wave), every load of a batch issued before the first is used: the compiler, left alone,
  // orders one load ahead of its use and the loop becomes a chain of single memory round trips.
  constexpr int kBatch = 8;
  int next_row = -1;
  float next_s = 0.f;
  if (r0 + 64 < r1) entry(r0 + 64 + lane, next_row, next_s);
  int my_row = first_row;
  float my_p = my_row >= 0 ? __expf(first_s - m) : 0.f;
#pragma unroll 1
  for (int cc = 0; cc < kPerWave; ++cc) {
    const int ck = wave * kPerWave + cc;
    const int c0 = ck * chunk, c1 = c0 + chunk < kb ? c0 + chunk : kb;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
    for (int base = c0; base < c1; base += 64) {          // the prefetched entries run on across chunk boundaries
      l += my_p;
      const int cur_row = my_row;
      const float cur_p = my_p;
      my_row = next_row;                                      // becomes current at the next trip
      my_p = my_row >= 0 ? __expf(next_s - m) : 0.f;
      if (base + 128 < r1) entry(base + 128 + lane, next_row, next_s);
      else next_row = -1;
#pragma unroll
      for (int half = 0; half < 16 / kBatch; ++half) {
        Raw8<T> rw[kBatch];
        float pw[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const int t = half * kBatch + u;
          const int row = __shfl(cur_row, 4 * t + rs);
          const float p = __shfl(cur_p, 4 * t + rs);
          rw[u].load(Vbg + Rows::offset(pg, row < 0 ? 0 : row, stride_b, stride_n));
          pw[u] = row < 0 ? 0.f : p;
        }
        __builtin_amdgcn_sched_barrier(0);                    // keep the batch's loads ahead of its arithmetic
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          float x[8];
          rw[u].get(x);
#pragma unroll
          for (int c = 0; c < 8; ++c) acc[c] = fmaf(pw[u], x[c], acc[c]);
        }
      }
    }
    // the chunk's partial sums (zeros for a chunk past the end of the list)
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) l += __shfl_xor(l, d);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      acc[c] += __shfl_xor(acc[c], 16);
      acc[c] += __shfl_xor(acc[c], 32);
    }
    if (rs == 0) {
#pragma unroll
      for (int c = 0; c < 8; ++c) sm.red[ck][8 * j + c] = acc[c];
    }
    if (lane == 0) sm.redl[ck] = l;
  }
  __syncthreads();
  if (tid < kD) {
    float a = 0.f, ls = 0.f;
#pragma unroll
    for (int w = 0; w < kAttendChunks; ++w) {
      a += sm.red[w][tid];
      ls += sm.redl[w];
    }
    out_row[tid] = ls > 0.f ? a / ls : 0.f;
  }
}

}  // namespace lfps
