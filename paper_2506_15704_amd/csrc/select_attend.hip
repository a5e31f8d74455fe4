// S3 + S4 in one kernel inside the chained steps: per query head the k best of its scored rows
// (Alg. 1 line 8 / Sec. 1 Step 2), then the attention output over exactly those rows (Eq. 1 / Sec. 1 Step 3).
// Both stages have one workgroup per (b, h); fused, the selected (position, score) pairs are consumed by the
// workgroup that has just produced them (the largest score, the softmax reference, is known from the select),
// heads that finish selecting early start gathering V rows while others still select, and a step has one kernel
// boundary less.
//
//   k_filter_select_attend   selects from the survivor lists that the filtered scoring pass leaves per head.
//                            A head whose survivors are fewer than k (or more than its on-chip list holds) takes
//                            the unfiltered pass on the spot: its workgroup scores every candidate of the group
//                            for this head (the same MFMA arithmetic as the group scoring kernel, hence the same
//                            bits) into the head's score row and selects from that.  This is rare once a history
//                            exists (the threshold sits a margin below the previous k-th best score) and costs
//                            that workgroup the bytes of all candidate rows; in exchange a step has no conditional
//                            launches behind this kernel.
//   k_select_attend          selects from a head's full score row (all candidates): contexts without the filter.
#include "attend.h"
#include "score_mfma.h"
#include "select_body.h"

#include <type_traits>

namespace lfps {

// ----------------------------------------------------------------------------- from the survivor lists
// The filtered score kernel cuts the line of all groups' candidate slots into parts of S slots
// (S = *seg_rows_in), one per wave; my group starts at slot pg = group_start[b, g] of the line, and its piece
// `sgm` is what wave w_first + sgm took of it, w_first = pg / S: the group's slots [lo, hi).  The piece holds
// seg_count[bh, sgm] (score, row position) pairs at offset lo of the head's score / position rows, ascending in
// position within and across pieces.  Workgroup 0 leaves *line_total at zero for the next step.
// The unfiltered pass needs the query, the K rows (format kKind, G heads per group) and the group's candidate list
// (cand; NULL when the candidates are all rows 0 .. count-1, the exact Top-k baseline's dense pass).
template <typename T, bool kPaged, int G, int kKind>
__global__ __launch_bounds__(kFilterSelThreads) void k_filter_select_attend(
    Shape s, float* score, const int32_t* __restrict__ slot_in, int64_t score_stride,
    const int32_t* __restrict__ seg_count, const int32_t* __restrict__ seg_rows_in, int nseg,
    const int32_t* __restrict__ cand, const int32_t* __restrict__ cand_count, const int64_t* __restrict__ group_start,
    int64_t* __restrict__ line_total, const int32_t* __restrict__ kk, int32_t* topk_idx, float* topk_score,
    float* __restrict__ thr_state, int cap, const int32_t* __restrict__ skip_if, int32_t* __restrict__ rescored,
    const float* __restrict__ q, const void* __restrict__ K, float scale, int32_t* __restrict__ flags,
    const T* __restrict__ V, int64_t stride_b, int64_t stride_h, int64_t stride_n, KvPage page,
    const int32_t* __restrict__ seq_lens, float* __restrict__ out) {
  constexpr int NT = kFilterSelThreads, kSelWaves = NT / 64;
  constexpr int kPiecesPerThread = 1024 / NT;      // nseg <= 1024
  __shared__ SelectShared<NT> sm;
  __shared__ int seg_off[kPiecesPerThread * NT];
  __shared__ int wtot[kSelWaves];
  extern __shared__ float cache[];                 // cap scores, then cap row positions; the attention's partial sums later
  int32_t* lslot = reinterpret_cast<int32_t*>(cache + cap);
  if (blockIdx.x == 0 && threadIdx.x == 0) *line_total = 0;   // the scoring pass that read it has finished
  const int bh = head_of_block(s, blockIdx.x);     // the heads of a KV group on one XCD: they share V rows in its L2
  const int b = bh / s.Hq, h = bh % s.Hq, g = h / s.G;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int bg = b * s.Hkv + g;
  if (skip_if && skip_if[bh] != 0) return;           // bypassed head: its rows were written by the gate
  int raw[kPiecesPerThread];                         // piece counts of this head, masked once the geometry is known
#pragma unroll
  for (int u = 0; u < kPiecesPerThread; ++u) {
    const int sgm = kPiecesPerThread * tid + u;
    raw[u] = sgm < nseg ? seg_count[(int64_t)bh * nseg + sgm] : 0;
  }
  int c = cand_count[bg];
  c = c < 0 ? 0 : (c > s.cand_cap ? s.cand_cap : c);
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  const int ksel = kb < c ? kb : c;
  int64_t S = *seg_rows_in;                          // chosen by the scoring pass of this step
  S = S < 64 ? 64 : S;
  const int64_t pg = group_start[bg];
  const int64_t w_first = pg / S;
  auto piece_lo = [&](int sgm) {                     // first slot of piece sgm within my group
    const int64_t lo = (w_first + sgm) * S - pg;
    return lo < 0 ? (int64_t)0 : lo;
  };
  auto piece_hi = [&](int sgm) {
    const int64_t hi = (w_first + sgm + 1) * S - pg;
    return hi > c ? (int64_t)c : hi;
  };

  // exclusive prefix of the piece counts (kPiecesPerThread consecutive pieces per thread); the counts
  // were loaded above, before the group's geometry was known: entries of pieces that do not exist
  // hold stale values and are masked here
  int cntp[kPiecesPerThread];
  int cnt = 0;
#pragma unroll
  for (int u = 0; u < kPiecesPerThread; ++u) {
    const int sgm = kPiecesPerThread * tid + u;
    cntp[u] = 0;
    if (sgm < nseg) {
      const int64_t room = piece_hi(sgm) - piece_lo(sgm);   // rows the piece covers
      if (room > 0) {
        const int v = raw[u] < 0 ? 0 : raw[u];
        cntp[u] = v > room ? (int)room : v;
      }
    }
    cnt += cntp[u];
  }
  const int inc = wave_inclusive_sum(cnt);
  if (lane == 63) wtot[wv] = inc;
  __syncthreads();
  int base = 0, n_surv = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const int t = wtot[w];
    base += w < wv ? t : 0;
    n_surv += t;
  }
  {
    int off = base + inc - cnt;
#pragma unroll
    for (int u = 0; u < kPiecesPerThread; ++u) {
      seg_off[kPiecesPerThread * tid + u] = off;
      off += cntp[u];
    }
  }
  const bool unfiltered = n_surv < ksel || n_surv > cap;   // block-uniform: the list cannot give the k best
  if (unfiltered && tid == 0 && rescored) atomicAdd(rescored, 1);   // heads that took the unfiltered pass since the last poll
  int32_t* oi = topk_idx + (int64_t)bh * s.kmax;
  float* os = topk_score + (int64_t)bh * s.kmax;
  for (int i = ksel + tid; i < s.kmax; i += NT) {   // padding
    oi[i] = -1;
    os[i] = 0.f;
  }
  float top = 0.f;
  if (ksel == 0) {
    if (tid == 0) thr_state[bh] = -INFINITY;
  } else if (unfiltered) {
    // every candidate slot of the group, 64 per wave and visit, scored for the G heads; my head's lane group stores
    using Rows = RowMap<kPaged>;
    using Op = typename KTile<kKind>::Operand;
    Op A[4];
    report_q_range(load_query_operand<G>(A, q, (int64_t)b * s.Hq + (int64_t)g * G, lane & 15, lane >> 4), flags);
    const char* Kbg = static_cast<const char*>(K) + Rows::base(b, g, stride_b, stride_h) * KTile<kKind>::kElemBytes;
    const int32_t* cbg = cand ? cand + (int64_t)bg * s.cand_cap : nullptr;
    float* sc = score + (int64_t)bh * score_stride;   // the survivor list there is given up
    score_slots_mfma<G, kPaged, kKind>(A, Kbg, page, b, stride_b, stride_n, cbg, n, c, wv * kRowsPerWaveIter,
                                       kSelWaves * kRowsPerWaveIter, sc, (lane >> 4) == h - g * G, scale);
    __syncthreads();                                  // the score row is complete before anyone reads it
    top = select_stream<NT>(sm, sc, c, ksel, cbg, oi, os, thr_state + bh, n);
  } else {
    __syncthreads();
    const float* sc = score + (int64_t)bh * score_stride;
    const int32_t* sl = slot_in + (int64_t)bh * score_stride;
    // Flat copy of the survivors into LDS: element e lies in the piece found by a binary search over
    // the offsets.  kGatherBatch elements per thread are searched together (fixed trip count, no
    // branches) and all their loads are issued before the first is used, so the copy costs a few
    // memory round trips instead of one per element.
    int np = (int)((pg + c - 1) / S - w_first) + 1;   // pieces my group was cut into
    np = np < 1 ? 1 : (np > nseg ? nseg : np);
    np = np < kPiecesPerThread * NT ? np : kPiecesPerThread * NT;
    int topp = 1;
    while (topp < np) topp <<= 1;
    constexpr int kGatherBatch = 12;
    float my_lo = FLT_MAX, my_hi = -FLT_MAX;             // range of the elements this thread copies
    for (int e0 = tid; e0 < n_surv; e0 += kGatherBatch * NT) {
      int pc[kGatherBatch];
#pragma unroll
      for (int u = 0; u < kGatherBatch; ++u) pc[u] = 0;
      for (int half = topp >> 1; half >= 1; half >>= 1) {   // last piece with seg_off <= e (seg_off[0] = 0)
#pragma unroll
        for (int u = 0; u < kGatherBatch; ++u) {
          const int mid = pc[u] + half;
          const int e = e0 + u * NT;
          if (mid < np && seg_off[mid] <= e) pc[u] = mid;
        }
      }
      float v[kGatherBatch];
      int32_t ps[kGatherBatch];
#pragma unroll
      for (int u = 0; u < kGatherBatch; ++u) {
        const int e = e0 + u * NT;
        v[u] = 0.f;
        ps[u] = 0;
        if (e < n_surv) {
          const int64_t src = piece_lo(pc[u]) + (e - seg_off[pc[u]]);
          v[u] = sc[src];
          ps[u] = sl[src];                              // the row position, written by the scoring pass
        }
      }
#pragma unroll
      for (int u = 0; u < kGatherBatch; ++u) {
        const int e = e0 + u * NT;
        if (e < n_surv) {
          const float x = sanitize(v[u]);
          cache[e] = x;
          lslot[e] = ps[u];
          my_lo = fminf(my_lo, x);
          my_hi = fmaxf(my_hi, x);
        }
      }
    }
    __syncthreads();
    select_body<true, NT, true>(sm, cache, nullptr, n_surv, ksel, lslot, nullptr, oi, os, thr_state + bh, my_lo, my_hi,
                                0x7FFFFFFF, &top);
  }
  // ---- S4 over the rows just selected.  The barrier orders this workgroup's stores of (position, score) before
  // its loads of them, and frees the select's LDS for the partial sums.
  if (out == nullptr) return;                       // select only (the exact Top-k baseline)
  __syncthreads();
  AttendShared& as = *reinterpret_cast<AttendShared*>(cache);
  attend_rows<T, kSelWaves, kPaged>(as, V, stride_b, stride_h, stride_n, page, b, g, n, kb, oi, os, ksel > 0, top,
                                    out + (int64_t)bh * kD);
}

// ----------------------------------------------------------------------------- from the full score rows
// k_select's steps on score[b, h, 0:c] (c = the group's candidate count), then the attention.
template <typename T, bool kPaged>
__global__ __launch_bounds__(kSelThreads) void k_select_attend(
    Shape s, const float* __restrict__ score, int64_t score_stride, const int32_t* __restrict__ cand,
    const int32_t* __restrict__ cand_count, const int32_t* __restrict__ kk, int32_t* topk_idx, float* topk_score,
    int cache_elems, float* __restrict__ thr_state,
    const int32_t* __restrict__ skip_if, const T* __restrict__ V, int64_t stride_b, int64_t stride_h, int64_t stride_n,
    KvPage page, const int32_t* __restrict__ seq_lens, float* __restrict__ out) {
  __shared__ SelectShared<kSelThreads> sm;
  __shared__ AttendShared as;
  extern __shared__ float cache[];
  const int bh = head_of_block(s, blockIdx.x);
  const int b = bh / s.Hq, h = bh % s.Hq, g = h / s.G;
  const int tid = threadIdx.x;
  if (skip_if && skip_if[bh] != 0) return;          // bypassed head: its rows were written by the gate
  int c = cand_count[b * s.Hkv + g];
  c = c < 0 ? 0 : (c > s.cand_cap ? s.cand_cap : c);
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  const int ksel = kb < c ? kb : c;
  int32_t* oi = topk_idx + (int64_t)bh * s.kmax;
  float* os = topk_score + (int64_t)bh * s.kmax;
  for (int i = ksel + tid; i < s.kmax; i += kSelThreads) {   // padding
    oi[i] = -1;
    os[i] = 0.f;
  }
  float* thr_out = thr_state ? thr_state + bh : nullptr;
  float top = 0.f;
  if (ksel == 0) {
    if (thr_out && tid == 0) *thr_out = -INFINITY;
  } else {
    const float* sc = score + (int64_t)bh * score_stride;
    const int32_t* cbg = cand + ((int64_t)b * s.Hkv + g) * s.cand_cap;
    if (c <= cache_elems)
      select_body<true, kSelThreads>(sm, cache, sc, c, ksel, nullptr, cbg, oi, os, thr_out, FLT_MAX, -FLT_MAX, n, &top);
    else
      top = select_stream(sm, sc, c, ksel, cbg, oi, os, thr_out, n);
  }
  __syncthreads();                                  // this workgroup's stores of (position, score) before its loads of them
  attend_rows<T, kSelThreads / 64, kPaged>(as, V, stride_b, stride_h, stride_n, page, b, g, n, kb, oi, os, ksel > 0, top,
                                           out + (int64_t)bh * kD);
}

// ----------------------------------------------------------------------------- launchers
// Dynamic LDS of k_filter_select_attend: the survivor list (score + position per entry), reused for the attention's
// partial sums.
static int filter_select_attend_lds(const Shape& s) {
  const int list = filter_list_cap(s) * 8;
  return list > (int)sizeof(AttendShared) ? list : (int)sizeof(AttendShared);
}

// The instantiations of k_filter_select_attend: V type and K format go together (bf16 V with bf16 or FP8 keys,
// FP8 V with FP8 keys, fp16 V with fp16 keys), times paged or not, times the heads per group.
#define LFPS_FSA_FOR_EACH_G(X, TYPE, PAGED, KIND) X(TYPE, PAGED, 1, KIND) X(TYPE, PAGED, 2, KIND) X(TYPE, PAGED, 4, KIND)
#define LFPS_FSA_FOR_EACH(X)                              \
  LFPS_FSA_FOR_EACH_G(X, uint16_t, false, kKindBf16)      \
  LFPS_FSA_FOR_EACH_G(X, uint16_t, true, kKindBf16)       \
  LFPS_FSA_FOR_EACH_G(X, uint16_t, false, kKindFp8)       \
  LFPS_FSA_FOR_EACH_G(X, uint16_t, true, kKindFp8)        \
  LFPS_FSA_FOR_EACH_G(X, uint8_t, false, kKindFp8)        \
  LFPS_FSA_FOR_EACH_G(X, uint8_t, true, kKindFp8)         \
  LFPS_FSA_FOR_EACH_G(X, _Float16, false, kKindF16)       \
  LFPS_FSA_FOR_EACH_G(X, _Float16, true, kKindF16)

hipError_t configure_select_attend(const Shape& s) {
  hipError_t e = hipSuccess;
  auto raise = [&](const void* kernel, int bytes) {
    if (e == hipSuccess) e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  };
  const int fb = filter_select_attend_lds(s), sb = kCacheElems * 4;
#define LFPS_RAISE_FSA(TYPE, PAGED, GG, KIND) raise((const void*)k_filter_select_attend<TYPE, PAGED, GG, KIND>, fb);
  LFPS_FSA_FOR_EACH(LFPS_RAISE_FSA)
#undef LFPS_RAISE_FSA
#define LFPS_RAISE_SA(TYPE)                                   \
  raise((const void*)k_select_attend<TYPE, false>, sb);       \
  raise((const void*)k_select_attend<TYPE, true>, sb)
  LFPS_RAISE_SA(uint16_t);
  LFPS_RAISE_SA(_Float16);
  LFPS_RAISE_SA(uint8_t);
  LFPS_RAISE_SA(float);
#undef LFPS_RAISE_SA
  return e;
}

template <typename T>
static constexpr int v_type_code() {          // 0 bf16 (as bits), 1 FP8, 2 fp16
  return std::is_same<T, uint16_t>::value ? 0 : (std::is_same<T, uint8_t>::value ? 1 : 2);
}

hipError_t launch_filter_select_attend(const Shape& s, int dtype, float* score, const int32_t* slot_in,
                                       int64_t score_stride, const int32_t* seg_count, const int32_t* seg_rows, int nseg,
                                       const int32_t* cand, const int32_t* cand_count, const int64_t* group_start,
                                       int64_t* line_total, const int32_t* k, int32_t* topk_idx, float* topk_score,
                                       float* thr_state, const int32_t* skip_if, int32_t* rescored, const float* q,
                                       int32_t* flags, const KvView& kv, float* out, hipStream_t st) {
  const int cap = filter_list_cap(s);
  const float scale = 0.08838834764831845f;   // 1/sqrt(128)
  const bool paged = kv.page.table != nullptr;
  // the pair (V type, K format) of this cache
  int vt = -1, kind = -1;                     // vt: 0 bf16, 1 FP8, 2 fp16
  if (dtype == LFPS_BF16) {
    vt = kv.v_fp8 ? 1 : 0;
    kind = kv.k_fp8 ? kKindFp8 : kKindBf16;
    if (vt == 1 && kind != kKindFp8) return hipErrorInvalidValue;   // FP8 values come with FP8 keys
  } else if (dtype == LFPS_F16) {
    vt = 2;
    kind = kKindF16;
  } else {
    return hipErrorInvalidValue;              // the filtered pass exists for 16-bit and FP8 caches only
  }
  bool launched = false;
#define LFPS_LAUNCH_FSA(TYPE, PAGED, GG, KIND)                                                                          \
  if (!launched && vt == v_type_code<TYPE>() && paged == PAGED && s.G == GG && kind == KIND) {                        \
    hipLaunchKernelGGL((k_filter_select_attend<TYPE, PAGED, GG, KIND>), dim3(s.B * s.Hq), dim3(kFilterSelThreads),      \
                       (size_t)filter_select_attend_lds(s), st, s, score, slot_in, score_stride, seg_count, seg_rows,   \
                       nseg, cand, cand_count, group_start, line_total, k, topk_idx, topk_score, thr_state, cap,        \
                       skip_if, rescored, q, kv.k, scale, flags, (const TYPE*)kv.v, kv.stride_b, kv.stride_h,           \
                       kv.stride_n, kv.page, kv.seq_lens, out);                                                         \
    launched = true;                                                                                                    \
  }
  LFPS_FSA_FOR_EACH(LFPS_LAUNCH_FSA)
#undef LFPS_LAUNCH_FSA
  if (!launched) return hipErrorInvalidValue;
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_sa_t(const Shape& s, const float* score, int64_t score_stride, const int32_t* cand,
                              const int32_t* cand_count, const int32_t* k, int32_t* topk_idx, float* topk_score,
                              float* thr_state, const int32_t* skip_if, const KvView& kv, float* out,
                              hipStream_t st) {
  int ce = s.cand_cap < kCacheElems ? s.cand_cap : kCacheElems;
  ce = (ce + 63) & ~63;
  const T* V = (const T*)kv.v;
#define LFPS_LAUNCH_SA(PAGED)                                                                                       \
  hipLaunchKernelGGL((k_select_attend<T, PAGED>), dim3(s.B * s.Hq), dim3(kSelThreads), (size_t)ce * 4, st, s, score, \
                     score_stride, cand, cand_count, k, topk_idx, topk_score, ce, thr_state, skip_if, V,   \
                     kv.stride_b, kv.stride_h, kv.stride_n, kv.page, kv.seq_lens, out)
  if (kv.page.table) {
    LFPS_LAUNCH_SA(true);
  } else {
    LFPS_LAUNCH_SA(false);
  }
#undef LFPS_LAUNCH_SA
  return hipGetLastError();
}

hipError_t launch_select_attend(const Shape& s, int dtype, const float* score, int64_t score_stride, const int32_t* cand,
                                const int32_t* cand_count, const int32_t* k, int32_t* topk_idx, float* topk_score,
                                float* thr_state, const int32_t* skip_if, const KvView& kv, float* out,
                                hipStream_t st) {
#define LFPS_SA_ARGS s, score, score_stride, cand, cand_count, k, topk_idx, topk_score, thr_state, skip_if, kv, out, st
  if (dtype == LFPS_BF16 && kv.v_fp8) return launch_sa_t<uint8_t>(LFPS_SA_ARGS);
  if (dtype == LFPS_F16) return launch_sa_t<_Float16>(LFPS_SA_ARGS);
  if (dtype == LFPS_BF16) return launch_sa_t<uint16_t>(LFPS_SA_ARGS);
  return launch_sa_t<float>(LFPS_SA_ARGS);
#undef LFPS_SA_ARGS
}

}  // namespace lfps
