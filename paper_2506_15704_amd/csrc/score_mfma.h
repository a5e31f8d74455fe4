// The MFMA scoring arithmetic shared by the kernels that score K rows against the G query heads of a KV group
// (Alg. 1 line 8; Sec. 1 Step 1): the three-term split of the fp32 query, the register tile of K rows, and the loop
// that scores a strided set of a group's candidate slots.  One definition, so that a row's score is the same bits
// whichever kernel computes it.
#pragma once
#include "lfps_internal.h"

namespace lfps {

constexpr int kScoreThreads = 256;           // 4 waves
constexpr int kRowsPerWaveIter = 64;         // rows a wave scores per loop iteration

// Storage format of the K rows a scoring kernel reads.
enum { kKindBf16 = 0, kKindFp8 = 1, kKindF16 = 2 };

// Round-to-nearest-even bf16 bits of x (the building block of the three-term split q = q0 + q1 + q2).
__device__ __forceinline__ uint16_t bf16_rne_bits(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Term t (0, 1, 2) of the three-way split of an fp32 query element into the operand's 16-bit format, as bits,
// and the sum of the three MFMA results that undoes the split.
template <typename Op>
struct Split3;
template <>
struct Split3<bf16x8> {
  using Elem = uint16_t;
  static constexpr bool kHalf = false;
  __device__ static __forceinline__ uint16_t term(float f, int t) {
    const uint16_t t0 = bf16_rne_bits(f);
    const float r1 = f - __uint_as_float((uint32_t)t0 << 16);
    const uint16_t t1 = bf16_rne_bits(r1);
    const float r2 = r1 - __uint_as_float((uint32_t)t1 << 16);
    const uint16_t t2 = bf16_rne_bits(r2);
    return t == 0 ? t0 : (t == 1 ? t1 : t2);            // selected without branching
  }
  __device__ static __forceinline__ float sum(const f32x4& acc) { return (acc[0] + acc[1]) + acc[2]; }
};
template <>
struct Split3<f16x8> {
  using Elem = _Float16;
  static constexpr bool kHalf = true;
  // q = t0 + t1 / 2^11 + t2 / 2^22 (11 significant bits per term; the scaling keeps t1, t2 normal)
  __device__ static __forceinline__ uint16_t term(float f, int t) {
    const _Float16 t0 = (_Float16)f;
    const float r1 = f - (float)t0;
    const _Float16 t1 = (_Float16)(r1 * 2048.0f);
    const float r2 = r1 - (float)t1 * (1.0f / 2048.0f);
    const _Float16 t2 = (_Float16)(r2 * 4194304.0f);
    const _Float16 sel = t == 0 ? t0 : (t == 1 ? t1 : t2);
    return __builtin_bit_cast(uint16_t, sel);
  }
  __device__ static __forceinline__ float sum(const f32x4& acc) {
    return (acc[0] + acc[1] * (1.0f / 2048.0f)) + acc[2] * (1.0f / 4194304.0f);
  }
};

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma16(f16x8 a, f16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// The MFMA A operand of lane (j, kb): row m = j of the 16x32 A tile of step kk holds term (m & 3)
// of head (m >> 2), channels of the 16-byte chunk kk + 4*kb of the row (the chunk that lane group kb
// loads from K at step kk).  Heads >= G contribute zeros.  The query is fetched with eight 16-byte
// loads issued together; a lane-dependent branch here would serialise 32 single loads.
// Returns true if this lane met a query element beyond the fp16 range (fp16 operands only): the element is
// clamped to +-65504 so that the scores stay finite, and the caller raises LFPS_FLAG_Q_RANGE.
template <int G, typename Op>
__device__ __forceinline__ bool load_query_operand(Op (&A)[4], const float* __restrict__ q, int64_t head0, int j,
                                                   int kb) {
  const int h = j >> 2, t = j & 3;
  const float4* qh = reinterpret_cast<const float4*>(q + (head0 + (h < G ? h : 0)) * kD);
  float4 x[4][2];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    x[kk][0] = qh[2 * (kk + 4 * kb)];
    x[kk][1] = qh[2 * (kk + 4 * kb) + 1];
  }
  const bool live = h < G && t < 3;
  bool clipped = false;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    float f[8] = {x[kk][0].x, x[kk][0].y, x[kk][0].z, x[kk][0].w, x[kk][1].x, x[kk][1].y, x[kk][1].z, x[kk][1].w};
    if constexpr (sizeof(typename Split3<Op>::Elem) == sizeof(_Float16) && Split3<Op>::kHalf) {
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        if (fabsf(f[c]) > 65504.0f) {               // also +-inf; a NaN goes through as in the other formats
          clipped |= live;
          f[c] = copysignf(65504.0f, f[c]);
        }
      }
    }
    union {
      Op v;
      uint16_t h[8];
    } a;
#pragma unroll
    for (int c = 0; c < 8; ++c) a.h[c] = live ? Split3<Op>::term(f[c], t) : (uint16_t)0;
    A[kk] = a.v;
  }
  return clipped;
}

// One lane of the wave reports a clamped query element (fp16 caches only; compiled out otherwise).
__device__ __forceinline__ void report_q_range(bool clipped, int32_t* __restrict__ flags) {
  if (__ballot(clipped) != 0 && (threadIdx.x & 63) == 0) atomicOr(flags, LFPS_FLAG_Q_RANGE);
}

// The registers a lane (j, kb) holds of one 64-row K tile: its 32 channels [32 kb, 32 kb + 32) of the
// four rows 16 t + j, in the storage format of K.  operand(t, kk) is the MFMA B operand of step kk, the
// channels 32 kb + 8 kk .. + 7 as bf16: the value as stored for a bf16 cache, converted (exactly: every
// E4M3 value is a bf16 value) when it is multiplied for an FP8 cache, so that a tile in flight costs half
// the registers and half the loads.
template <int kKind>
struct KTile;
template <>
struct KTile<kKindBf16> {
  using Operand = bf16x8;
  static constexpr int kElemBytes = 2;
  bf16x8 v[4][4];
  __device__ __forceinline__ void load_row(int t, const char* row, int kb) {
    const bf16x8* p = reinterpret_cast<const bf16x8*>(row) + 4 * kb;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) v[t][kk] = p[kk];
  }
  __device__ __forceinline__ bf16x8 operand(int t, int kk) const { return v[t][kk]; }
};
template <>
struct KTile<kKindF16> {
  using Operand = f16x8;
  static constexpr int kElemBytes = 2;
  f16x8 v[4][4];
  __device__ __forceinline__ void load_row(int t, const char* row, int kb) {
    const f16x8* p = reinterpret_cast<const f16x8*>(row) + 4 * kb;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) v[t][kk] = p[kk];
  }
  __device__ __forceinline__ f16x8 operand(int t, int kk) const { return v[t][kk]; }
};
template <>
struct KTile<kKindFp8> {
  using Operand = bf16x8;
  static constexpr int kElemBytes = 1;
  u32x4 v[4][2];
  __device__ __forceinline__ void load_row(int t, const char* row, int kb) {
    const u32x4* p = reinterpret_cast<const u32x4*>(row) + 2 * kb;
    v[t][0] = p[0];
    v[t][1] = p[1];
  }
  __device__ __forceinline__ bf16x8 operand(int t, int kk) const {
    const u32x4 w = v[t][kk >> 1];
    return (kk & 1) ? fp8x8_to_bf16x8(w[2], w[3]) : fp8x8_to_bf16x8(w[0], w[1]);
  }
};

// Scores of the slots first .. first+63, first+step .. first+step+63, ... (below count) of one KV group, by one wave:
// lane (j, kb) = (lane & 15, lane >> 4) loads the chunks of K that lane group kb owns and ends up holding head kb's
// score of slot base + 16 t + j.  cbg: the group's candidate list (slot -> row position), or NULL when slot = row
// position.  A slot whose position lies outside [0, n) reads row 0 and scores -inf: it ranks below every row.
// The row ids of the next visit are fetched, and the scores of the previous visit stored, right after this visit's
// loads are issued.  sc: the score row of head kb (ignored by lanes with store == false).
template <int G, bool kPaged, int kKind>
__device__ __forceinline__ void score_slots_mfma(const typename KTile<kKind>::Operand (&A)[4], const char* Kbg,
                                                 const KvPage& pg, int b, int64_t stride_b, int64_t stride_n,
                                                 const int32_t* __restrict__ cbg, int n, int count, int first, int step,
                                                 float* __restrict__ sc, bool store, float scale) {
  using Rows = RowMap<kPaged>;
  using Op = typename KTile<kKind>::Operand;
  constexpr int ES = KTile<kKind>::kElemBytes;
  const int lane = threadIdx.x & 63;
  const int j = lane & 15, kb = lane >> 4;
  auto valid = [&](int row) { return row >= 0 && row < n; };
  auto physical = [&](int row) { return Rows::phys(pg, b, valid(row) ? row : 0); };

  float pv[4] = {0.f, 0.f, 0.f, 0.f};   // scores of the previous visit, not yet stored
  int pbase = -1;
  int my_row = -1;
  if (first + lane < count) my_row = cbg ? cbg[first + lane] : first + lane;
  int my_ok = valid(my_row);
  my_row = physical(my_row);
  for (int base = first; base < count; base += step) {
    KTile<kKind> Bt;
    bool ok_t[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int row = __shfl(my_row, 16 * t + j);
      ok_t[t] = __shfl(my_ok, 16 * t + j) != 0;
      Bt.load_row(t, Kbg + Rows::offset(pg, row, stride_b, stride_n) * ES, kb);
    }
    const int nb = base + step;
    int next_row = -1;
    if (nb + lane < count) next_row = cbg ? cbg[nb + lane] : nb + lane;
    const int next_ok = valid(next_row);
    next_row = physical(next_row);
    if (pbase >= 0) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int slot = pbase + 16 * t + j;
        if (store && slot < count) sc[slot] = pv[t];
      }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        acc = mfma16(A[kk], Bt.operand(t, kk), acc);
      // lane (j, kb): D rows 4*kb .. 4*kb+3 = the three terms (and a zero row) of head kb, column j
      pv[t] = ok_t[t] ? Split3<Op>::sum(acc) * scale : -INFINITY;
    }
    pbase = base;
    my_row = next_row;
    my_ok = next_ok;
  }
  if (pbase >= 0) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int slot = pbase + 16 * t + j;
      if (store && slot < count) sc[slot] = pv[t];
    }
  }
}

}  // namespace lfps
