// S2 — scores q . K_j / sqrt(D) of selected rows for the G query heads that share a KV head
// (Alg. 1 line 8; Sec. 1 Step 1 restricted to the candidates).  Also the dense variant over all
// rows (the exact Top-k baseline's Step 1), and a per-head variant for arbitrary index lists.
//
// The path is bound by the bytes of the K rows it gathers; the arithmetic is kept off the
// vector ALU so it cannot become the limit:
//   bf16 cache: one wave handles 16 rows at a time with v_mfma_f32_16x16x32_bf16.  The B operand
//     is the K tile exactly as it lies in memory (each lane loads 16-byte pieces of one row),
//     so a row is fetched once for all G heads.  The A operand is
//     the query: each fp32 q is split into three bf16 terms q = q0 + q1 + q2 (24 mantissa bits),
//     and A's row 4*h + t holds term t of head h.  bf16 x bf16 products are exact in fp32, so
//     the sum D[4h+0] + D[4h+1] + D[4h+2] is the fp32-accumulated dot product with the fp32
//     query; it lands in lane group h without any cross-lane reduction.
//   fp16 cache: the same with v_mfma_f32_16x16x32_f16; the query terms are fp16 too, the second and third
//     scaled up by 2^11 and 2^22 so that they stay normal numbers, and scaled back when the three
//     D rows are added (fp16 x fp16 products are exact in fp32 as well).  |q| must stay below 65504.
//   fp32 cache: 16 lanes per row, 8 channels each, fp32 FMAs and a 4-step xor-shuffle reduce.
#include "lfps_internal.h"
#include "score_mfma.h"

namespace lfps {

// ----------------------------------------------------------------------------- bf16 / fp16 / fp8, MFMA
// grid: (tiles_x, B*Hkv).  GATHER: rows come from cand[bg, 0:count]; else rows are 0..n_b-1.
//
// Lane (j, kb) = (lane & 15, lane >> 4) supplies column j of the B operand: for MFMA step kk it
// loads the 16-byte chunk kk + 4*kb of row j, i.e. every lane walks its own contiguous 64 bytes of
// the row over the four steps (measured faster than splitting a row into four 64-byte quarters
// per step: all four loads of a tile touch both cache lines of every row).  Any assignment of
// channels to (kk, kb) is valid as long as the A operand uses the same one.
// The row ids of the next iteration are fetched, and the scores of the previous iteration stored,
// right after this iteration's loads are issued.
template <int G, bool GATHER, bool kPaged, int kKind>
__global__ __launch_bounds__(kScoreThreads) void k_group_score_bf16(Shape s, const float* __restrict__ q,
                                                                    const void* __restrict__ K, int64_t stride_b,
                                                                    int64_t stride_h, int64_t stride_n, KvPage pg,
                                                                    const int32_t* __restrict__ seq_lens,
                                                                    const int32_t* __restrict__ cand,
                                                                    const int32_t* __restrict__ cand_count,
                                                                    float* __restrict__ score, int64_t score_stride,
                                                                    float scale, int32_t* __restrict__ flags) {
  const int bg = blockIdx.y, b = bg / s.Hkv, g = bg % s.Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 15, kb = lane >> 4;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  int count = GATHER ? cand_count[bg] : n;
  if (GATHER) count = count < 0 ? 0 : (count > s.cand_cap ? s.cand_cap : count);
  const int first = (blockIdx.x * 4 + wave) * kRowsPerWaveIter;
  if (first >= count) return;

  using Op = typename KTile<kKind>::Operand;
  Op A[4];
  report_q_range(load_query_operand<G>(A, q, (int64_t)b * s.Hq + (int64_t)g * G, j, kb), flags);

  using Rows = RowMap<kPaged>;
  constexpr int ES = KTile<kKind>::kElemBytes;
  const char* Kbg = static_cast<const char*>(K) + Rows::base(b, g, stride_b, stride_h) * ES;
  const int32_t* cbg = GATHER ? cand + (int64_t)bg * s.cand_cap : nullptr;
  float* sc = score + ((int64_t)b * s.Hq + (int64_t)g * G + kb) * score_stride;   // lane group kb -> head kb
  score_slots_mfma<G, kPaged, kKind>(A, Kbg, pg, b, stride_b, stride_n, cbg, n, count, first,
                                     (int)gridDim.x * 4 * kRowsPerWaveIter, sc, kb < G, scale);
}

// ----------------------------------------------------------------------------- bf16 / fp16 / fp8, MFMA, filtered output
// The same scoring, but only rows whose score reaches a per-head threshold are written out
// (the threshold is the previous step's k-th best score minus a margin: consecutive decode steps
// select almost the same rows, the premise of the method).  Writing every score costs far more
// than its share of bytes because the small writes interleave with the row gather; survivors are
// a few per cent of the rows.
//
// Work split: the candidate slots of all groups, laid end to end, form one line [0, total); it is
// cut into equal parts of S slots, one per wave of the launch, and the launch has exactly as many
// waves as the chip holds at once.  Every wave therefore reads the same number of rows whatever
// the mix of sequence lengths, and no workgroup waits for a slot.  The candidates kernel has given
// every group its place on the line (group_start; the order of the groups on the line is the
// order in which they finished there, which changes nothing in the result) and left the line's
// length in *line_total.  A part that crosses a group boundary is handled as several pieces, one
// per group.  Piece `seg` of a group (seg = wave index minus the index of the first wave that
// touches the group) covers the group's slots [lo, hi) and appends its survivors (score, row
// position), in slot order, at offset lo of each head's score / position rows (staged in LDS,
// written when the piece is done); their number goes to seg_count[head, seg].  No atomics here:
// the lists are ascending in position and the same from run to run.
// A threshold of -inf keeps every row; NaN means there is no previous step.
constexpr int kFilterStage = 256;   // survivors one wave can hold per head before it must write them out

// kDense: the "candidates" of a group are all its rows 0..count-1 (no list is read): the exact Top-k baseline's
// scoring pass with a threshold from a sample of the rows.
template <int G, bool kPaged, int kKind, bool kDense>
__global__ __launch_bounds__(kScoreThreads, 2) void k_filter_score_bf16(
    Shape s, const float* __restrict__ q, const void* __restrict__ K, int64_t stride_b, int64_t stride_h,
    int64_t stride_n, KvPage page, const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ cand,
    const int32_t* __restrict__ cand_count, const int64_t* __restrict__ group_start,
    const int64_t* __restrict__ line_total, const float* __restrict__ thr_state, float margin,
    float* __restrict__ score, int32_t* __restrict__ slot_out, int64_t score_stride,
    int32_t* __restrict__ seg_count, int32_t* __restrict__ seg_rows_out, int min_seg_rows, int nseg, float scale,
    int32_t* __restrict__ flags) {
  __shared__ float stage_score[4][G][kFilterStage];
  __shared__ int32_t stage_slot[4][G][kFilterStage];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform values stay in scalar registers
  const int j = lane & 15, kb = lane >> 4;
  const int n_groups = s.B * s.Hkv;

  // ---- the part of this wave: S slots from wave_index * S; every wave derives the same S
  const int64_t total = *line_total;
  const int64_t n_waves = (int64_t)gridDim.x * 4;
  int64_t S = ((total + n_waves - 1) / n_waves + 63) & ~(int64_t)63;
  S = S < min_seg_rows ? min_seg_rows : S;
  if (blockIdx.x == 0 && tid == 0) *seg_rows_out = (int32_t)S;      // the select reads it
  const int64_t w = (int64_t)blockIdx.x * 4 + wave;
  const int64_t part_lo = w * S;
  const int64_t part_hi = part_lo + S < total ? part_lo + S : total;
  if (part_lo >= total) return;                          // nothing left for this wave

  const uint32_t below = (1u << j) - 1u;                // lanes of my 16-lane group with a lower row
  float* st_s = stage_score[wave][kb < G ? kb : 0];
  int32_t* st_i = stage_slot[wave][kb < G ? kb : 0];
  constexpr int T = kRowsPerWaveIter;

  // the groups that overlap my part: 64 groups are tested at a time, one per lane
  for (int g0 = 0; g0 < n_groups; g0 += 64) {
    int64_t st = 0;
    int cnt_l = 0;
    if (g0 + lane < n_groups) {
      st = group_start[g0 + lane];
      const int c = cand_count[g0 + lane];
      cnt_l = c < 0 ? 0 : (c > s.cand_cap ? s.cand_cap : c);
    }
    uint64_t hits = __ballot(cnt_l > 0 && st < part_hi && st + cnt_l > part_lo);
  while (hits) {                                          // one piece per overlapping group
    const int src = __builtin_ctzll(hits);
    hits &= hits - 1;
    const int bg = g0 + src;
    const int64_t pg = ((int64_t)__builtin_amdgcn_readlane((int)(st >> 32), src) << 32) |
                       (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)st, src);   // the group's place on the line
    const int count = __builtin_amdgcn_readlane(cnt_l, src);
    const int seg_lo = part_lo > pg ? (int)(part_lo - pg) : 0;
    const int seg_hi = part_hi - pg < count ? (int)(part_hi - pg) : count;
    const int seg = (int)(w - pg / S);

    const int b = bg / s.Hkv, g = bg % s.Hkv;
    int n = seq_lens[b];
    n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
    const int64_t head = (int64_t)b * s.Hq + (int64_t)g * G + (kb < G ? kb : 0);
    // NaN in thr_state = "no previous step": skip the group here, the unfiltered pass will take it
    bool no_history = false;
#pragma unroll
    for (int h = 0; h < G; ++h) no_history |= isnan(thr_state[(int64_t)b * s.Hq + (int64_t)g * G + h]);
    if (no_history) {
      if (j == 0 && kb < G) seg_count[head * nseg + seg] = 0;
      continue;
    }
    const float tau = kb < G ? thr_state[head] - margin : INFINITY;

    using Rows = RowMap<kPaged>;
    using Tile = KTile<kKind>;
    using Op = typename Tile::Operand;
    Op A[4];                                            // filled after the first tile's loads are on their way
    constexpr int ES = Tile::kElemBytes;
    const char* Kbg = static_cast<const char*>(K) + Rows::base(b, g, stride_b, stride_h) * ES;
    const int32_t* cbg = cand + (int64_t)bg * s.cand_cap;
    int run = 0;                                        // survivors of my head already in global memory
    int staged = 0;                                     // survivors of my head waiting in LDS

    // Survivors are staged in LDS and written out when the piece is done (or the stage is nearly
    // full).  Global stores inside the loop would share the vector-memory counter with the row
    // loads, so that every wait for a load would also wait for the stores before it.
    auto flush = [&]() {
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const int cnt_h = __shfl(staged, 16 * h);
        const int run_h = __shfl(run, 16 * h);
        float* dsc = score + ((int64_t)b * s.Hq + (int64_t)g * G + h) * score_stride + seg_lo + run_h;
        int32_t* dsl = slot_out + ((int64_t)b * s.Hq + (int64_t)g * G + h) * score_stride + seg_lo + run_h;
        for (int e = lane; e < cnt_h; e += 64) {
          dsc[e] = stage_score[wave][h][e];
          dsl[e] = stage_slot[wave][h][e];
        }
      }
      run += staged;
      staged = 0;
    };

    // Two 64-row tiles are kept in flight per wave: while tile i is multiplied, the loads of tile
    // i+1 (issued before) are still arriving.
    // ids: the row positions of the tile's 64 slots, one per lane; phys: the same rows as physical
    // rows (paged cache only; ignored otherwise)
    auto issue = [&](Tile& Bt, int (&rows)[4], int ids, int phys) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        int row = __shfl(ids, 16 * t + j);
        row = (row < 0 || row >= n) ? 0 : row;          // padding slots read row 0 and are never kept
        rows[t] = row;
        const int prow = kPaged ? __shfl(phys, 16 * t + j) : row;
        Bt.load_row(t, Kbg + Rows::offset(page, prow, stride_b, stride_n) * ES, kb);
      }
    };
    auto lookup = [&](int ids) { return Rows::phys(page, b, (ids < 0 || ids >= n) ? 0 : ids); };
    auto consume = [&](Tile& Bt, int (&rows)[4], int base_slot) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
          acc = mfma16(A[kk], Bt.operand(t, kk), acc);
        const float v = Split3<Op>::sum(acc) * scale;
        const int slot = base_slot + 16 * t + j;
        const bool pass = kb < G && slot < seg_hi && v >= tau;
        const uint32_t gm = (uint32_t)(__ballot(pass) >> (16 * kb)) & 0xFFFFu;   // my head's 16 rows
        if (pass) {
          const int o = staged + __popc(gm & below);
          st_s[o] = v;
          st_i[o] = rows[t];                            // the row position itself: the select needs no lookup
        }
        staged += __popc(gm);
      }
      // room for one more tile (64 rows) in every head's stage?  (wave-uniform test)
      if (__ballot(staged > kFilterStage - kRowsPerWaveIter)) flush();
    };
    // Slots past the end of the piece read the id of its last slot (a valid row) and are never kept:
    // no load of the loop below sits behind a branch, so the waits the compiler derives for the
    // two tiles in flight are exact counts instead of "everything outstanding".
    auto fetch_ids = [&](int base_slot) {
      const int sl = base_slot + lane;
      const int at = sl < seg_hi ? sl : seg_hi - 1;
      if constexpr (kDense) return at;
      else return cbg[at];
    };

    // Row ids are fetched three tiles ahead, always BEFORE the loads of the tile that precedes
    // their use are issued: a wait for ids then never has to wait for a tile still in flight
    // (the vector-memory counter completes in issue order).
    Tile Bt0, Bt1;
    int rows0[4], rows1[4];
    int base_slot = seg_lo;
    if constexpr (!kPaged) {
      const int ids_0 = fetch_ids(seg_lo);
      int ids_b = fetch_ids(seg_lo + T);                  // ids of the next odd tile
      int ids_a = fetch_ids(seg_lo + 2 * T);              // ids of the next even tile
      issue(Bt0, rows0, ids_0, 0);
      report_q_range(load_query_operand<G>(A, q, (int64_t)b * s.Hq + (int64_t)g * G, j, kb), flags);   // overlaps the first tile's latency
      for (; base_slot + 2 * T < seg_hi; base_slot += 2 * T) {   // at least three tiles left: no conditions inside
        issue(Bt1, rows1, ids_b, 0);
        ids_b = fetch_ids(base_slot + 3 * T);
        consume(Bt0, rows0, base_slot);
        issue(Bt0, rows0, ids_a, 0);
        ids_a = fetch_ids(base_slot + 4 * T);
        consume(Bt1, rows1, base_slot + T);
      }
      if (base_slot + T < seg_hi) {                       // two tiles left (wave-uniform)
        issue(Bt1, rows1, ids_b, 0);
        consume(Bt0, rows0, base_slot);
        consume(Bt1, rows1, base_slot + T);
      } else {
        consume(Bt0, rows0, base_slot);
      }
    } else {
      // Paged cache: a block-table lookup sits between a row id and its address.  A wait completes
      // everything older than what it waits for, so with tile i in flight every step issues, BEFORE
      // the loads of tile i+1: the ids of tile i+3 and the lookup for tile i+2 (whose ids were fetched
      // one step earlier, before the loads of tile i).  The lane shuffles that spread ids and physical
      // rows of tile i+1 over the wave come first, so that the registers can be refilled in place.
      int prow[4];
      auto aim = [&](int (&rows)[4], int ids, int phys) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int row = __shfl(ids, 16 * t + j);
          rows[t] = (row < 0 || row >= n) ? 0 : row;
          prow[t] = __shfl(phys, 16 * t + j);
        }
      };
      auto fire = [&](Tile& Bt) {
#pragma unroll
        for (int t = 0; t < 4; ++t) Bt.load_row(t, Kbg + Rows::offset(page, prow[t], stride_b, stride_n) * ES, kb);
      };
      int ids_0 = fetch_ids(seg_lo), ids_1 = fetch_ids(seg_lo + T);
      int phys_0 = lookup(ids_0), phys_1 = lookup(ids_1);
      aim(rows0, ids_0, phys_0);
      ids_0 = fetch_ids(seg_lo + 2 * T);
      __builtin_amdgcn_sched_barrier(0);
      fire(Bt0);
      report_q_range(load_query_operand<G>(A, q, (int64_t)b * s.Hq + (int64_t)g * G, j, kb), flags);
      // here and at the top of every iteration: (ids_1, phys_1) describe the next odd tile, ids_0 the next even one
      for (; base_slot + 2 * T < seg_hi; base_slot += 2 * T) {
        aim(rows1, ids_1, phys_1);
        ids_1 = fetch_ids(base_slot + 3 * T);
        phys_0 = lookup(ids_0);
        __builtin_amdgcn_sched_barrier(0);      // the instruction scheduler must not move these two loads
        fire(Bt1);                              // behind the tile's: the order is what the waits rely on
        consume(Bt0, rows0, base_slot);
        aim(rows0, ids_0, phys_0);
        ids_0 = fetch_ids(base_slot + 4 * T);
        phys_1 = lookup(ids_1);
        __builtin_amdgcn_sched_barrier(0);
        fire(Bt0);
        consume(Bt1, rows1, base_slot + T);
      }
      if (base_slot + T < seg_hi) {
        aim(rows1, ids_1, phys_1);
        fire(Bt1);
        consume(Bt0, rows0, base_slot);
        consume(Bt1, rows1, base_slot + T);
      } else {
        consume(Bt0, rows0, base_slot);
      }
      // A use of the prefetched ids on every path: without it the compiler moves the prologue's fetch of
      // ids_0 down to the loop entry, behind the first tile's loads, and the loop's first wait for it
      // becomes a wait for everything.
      asm volatile("" ::"v"(ids_0), "v"(ids_1));
    }
    flush();
    if (j == 0 && kb < G) seg_count[head * nseg + seg] = run;
  }
  }
}

// ----------------------------------------------------------------------------- fp32, vector ALU
template <int G, bool GATHER, bool kPaged>
__global__ __launch_bounds__(kScoreThreads) void k_group_score_f32(Shape s, const float* __restrict__ q,
                                                                   const float* __restrict__ K, int64_t stride_b,
                                                                   int64_t stride_h, int64_t stride_n, KvPage pg,
                                                                   const int32_t* __restrict__ seq_lens,
                                                                   const int32_t* __restrict__ cand,
                                                                   const int32_t* __restrict__ cand_count,
                                                                   float* __restrict__ score, int64_t score_stride,
                                                                   float scale, int32_t* __restrict__ flags) {
  const int bg = blockIdx.y, b = bg / s.Hkv, g = bg % s.Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 15, rs = lane >> 4;     // 16 lanes per row, 4 rows per wave instruction
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  int count = GATHER ? cand_count[bg] : n;
  if (GATHER) count = count < 0 ? 0 : (count > s.cand_cap ? s.cand_cap : count);
  const int first = (blockIdx.x * 4 + wave) * kRowsPerWaveIter;
  if (first >= count) return;

  float qr[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const float* qh = q + ((int64_t)b * s.Hq + (int64_t)g * G + h) * kD + 8 * j;
#pragma unroll
    for (int c = 0; c < 8; ++c) qr[h][c] = qh[c];
  }
  using Rows = RowMap<kPaged>;
  const float* Kbg = K + Rows::base(b, g, stride_b, stride_h);
  const int32_t* cbg = GATHER ? cand + (int64_t)bg * s.cand_cap : nullptr;
  float* sc = score + ((int64_t)b * s.Hq + (int64_t)g * G) * score_stride;
  const int step = gridDim.x * 4 * kRowsPerWaveIter;

  for (int base = first; base < count; base += step) {
    int my_row = -1;
    if (base + lane < count) my_row = GATHER ? cbg[base + lane] : base + lane;
    const bool my_ok = my_row >= 0 && my_row < n;
    const int my_phys = Rows::phys(pg, b, my_ok ? my_row : 0);
#pragma unroll 4
    for (int t = 0; t < 16; ++t) {
      const bool ok = __shfl((int)my_ok, 4 * t + rs) != 0;
      const int prow = __shfl(my_phys, 4 * t + rs);
      const float4* p = reinterpret_cast<const float4*>(Kbg + Rows::offset(pg, prow, stride_b, stride_n)) + 2 * j;
      float4 x0 = p[0], x1 = p[1];
      float acc[G];
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float a = qr[h][0] * x0.x;
        a = fmaf(qr[h][1], x0.y, a);
        a = fmaf(qr[h][2], x0.z, a);
        a = fmaf(qr[h][3], x0.w, a);
        a = fmaf(qr[h][4], x1.x, a);
        a = fmaf(qr[h][5], x1.y, a);
        a = fmaf(qr[h][6], x1.z, a);
        a = fmaf(qr[h][7], x1.w, a);
        acc[h] = a;
      }
#pragma unroll
      for (int d = 1; d < 16; d <<= 1) {
#pragma unroll
        for (int h = 0; h < G; ++h) acc[h] += __shfl_xor(acc[h], d);
      }
      int slot = base + 4 * t + rs;
      if (slot < count && j < G) {     // a candidate entry outside [0, n) scores -inf: it ranks below every row
        float v = acc[0];
#pragma unroll
        for (int h = 1; h < G; ++h) v = (j == h) ? acc[h] : v;
        sc[(int64_t)j * score_stride + slot] = ok ? v * scale : -INFINITY;
      }
    }
  }
}

// ----------------------------------------------------------------------------- per-head index lists
// Scores of idx[b,h,0:k_b] against q[b,h]; 16 lanes per row.  Used only when the caller of the
// sparse attention does not supply scores.  grid: (ceil(kmax/256), B*Hq).
template <typename T, bool kPaged>
__global__ __launch_bounds__(256) void k_head_score(Shape s, const float* __restrict__ q, const T* __restrict__ K,
                                                    int64_t stride_b, int64_t stride_h, int64_t stride_n, KvPage pg,
                                                    const int32_t* __restrict__ seq_lens,
                                                    const int32_t* __restrict__ idx, const int32_t* __restrict__ kk,
                                                    float* __restrict__ out, float scale) {
  const int bh = blockIdx.y, b = bh / s.Hq, h = bh % s.Hq, g = h / s.G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 15, rs = lane >> 4;
  int n = seq_lens[b];
  n = n < 0 ? 0 : (n > s.Lcap ? s.Lcap : n);
  int kb = kk[b];
  kb = kb < 0 ? 0 : (kb > s.kmax ? s.kmax : kb);
  const int base = (blockIdx.x * 4 + wave) * 64;
  if (base >= kb) return;
  float qr[8];
  const float* qh = q + (int64_t)bh * kD + 8 * j;
#pragma unroll
  for (int c = 0; c < 8; ++c) qr[c] = qh[c];
  using Rows = RowMap<kPaged>;
  const T* Kbg = K + Rows::base(b, g, stride_b, stride_h);
  const int my_row = (base + lane < kb) ? idx[(int64_t)bh * s.kmax + base + lane] : -1;
  const bool my_ok = my_row >= 0 && my_row < n;
  const int my_phys = Rows::phys(pg, b, my_ok ? my_row : 0);
  for (int t = 0; t < 16; ++t) {
    const bool ok = __shfl((int)my_ok, 4 * t + rs) != 0;
    const int prow = __shfl(my_phys, 4 * t + rs);
    const T* p = Kbg + Rows::offset(pg, prow, stride_b, stride_n) + 8 * j;
    float x[8];
    load8(p, x);
    float a = qr[0] * x[0];
#pragma unroll
    for (int c = 1; c < 8; ++c) a = fmaf(qr[c], x[c], a);
#pragma unroll
    for (int d = 1; d < 16; d <<= 1) a += __shfl_xor(a, d);
    int slot = base + 4 * t + rs;
    if (j == 0 && slot < kb) out[(int64_t)bh * s.kmax + slot] = ok ? a * scale : -INFINITY;
  }
}

// ----------------------------------------------------------------------------- launchers
template <int G, bool GATHER>
static hipError_t launch_gs(const Shape& s, int dtype, const float* q, const KvView& kv, const int32_t* cand,
                            const int32_t* cand_count, float* score, int64_t score_stride, int32_t* flags,
                            hipStream_t st) {
  const int rows_max = GATHER ? s.cand_cap : s.Lcap;
  const int per_block = 4 * kRowsPerWaveIter;
  int tiles = (rows_max + per_block - 1) / per_block;
  // about four workgroups (16 waves) per CU, all resident at once, but no more than there are tiles
  int want = (256 * 4 + s.B * s.Hkv - 1) / (s.B * s.Hkv);
  int gx = tiles < want ? tiles : want;
  if (gx < 1) gx = 1;
  dim3 grid(gx, s.B * s.Hkv), block(kScoreThreads);
  const float scale = 0.08838834764831845f;   // 1/sqrt(128)
#define LFPS_LAUNCH_GS(KERNEL, TYPE, ...)                                                                          \
  hipLaunchKernelGGL((KERNEL<G, GATHER, __VA_ARGS__>), grid, block, 0, st, s, q, (const TYPE*)kv.k, kv.stride_b,   \
                     kv.stride_h, kv.stride_n, kv.page, kv.seq_lens, cand, cand_count, score, score_stride, scale, \
                     flags)
  const bool paged = kv.page.table != nullptr;
  if (dtype == LFPS_BF16 && kv.k_fp8) {
    if (paged) LFPS_LAUNCH_GS(k_group_score_bf16, void, true, kKindFp8);
    else LFPS_LAUNCH_GS(k_group_score_bf16, void, false, kKindFp8);
  } else if (dtype == LFPS_BF16) {
    if (paged) LFPS_LAUNCH_GS(k_group_score_bf16, void, true, kKindBf16);
    else LFPS_LAUNCH_GS(k_group_score_bf16, void, false, kKindBf16);
  } else if (dtype == LFPS_F16) {
    if (paged) LFPS_LAUNCH_GS(k_group_score_bf16, void, true, kKindF16);
    else LFPS_LAUNCH_GS(k_group_score_bf16, void, false, kKindF16);
  } else {
    if (paged) LFPS_LAUNCH_GS(k_group_score_f32, float, true);
    else LFPS_LAUNCH_GS(k_group_score_f32, float, false);
  }
#undef LFPS_LAUNCH_GS
  return hipGetLastError();
}

hipError_t launch_group_score(const Shape& s, int dtype, const float* q, const KvView& kv, const int32_t* cand,
                              const int32_t* cand_count, float* score, int64_t score_stride, int32_t* flags,
                              hipStream_t st) {
  const bool gather = cand != nullptr;
  switch (s.G) {
    case 1: return gather ? launch_gs<1, true>(s, dtype, q, kv, cand, cand_count, score, score_stride, flags, st)
                          : launch_gs<1, false>(s, dtype, q, kv, cand, cand_count, score, score_stride, flags, st);
    case 2: return gather ? launch_gs<2, true>(s, dtype, q, kv, cand, cand_count, score, score_stride, flags, st)
                          : launch_gs<2, false>(s, dtype, q, kv, cand, cand_count, score, score_stride, flags, st);
    case 4: return gather ? launch_gs<4, true>(s, dtype, q, kv, cand, cand_count, score, score_stride, flags, st)
                          : launch_gs<4, false>(s, dtype, q, kv, cand, cand_count, score, score_stride, flags, st);
    default: return hipErrorInvalidValue;
  }
}

// Smallest part size in candidate slots, and the pieces a group can then be cut into (<= 1024).
int filter_min_seg_rows(const Shape& s) { return (((s.cand_cap + 999) / 1000) + 63) & ~63; }
int filter_nseg(const Shape& s) { return s.cand_cap / filter_min_seg_rows(s) + 2; }

template <int G, int kKind>
static hipError_t filter_resident_blocks(int out[2]) {
  int dev = 0;
  hipDeviceProp_t prop;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
  auto resident = [&](const void* kernel, int* n) {
    int per_cu = 0;
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kScoreThreads, 0);
    // two per CU is what the kernels are built for (__launch_bounds__); the FP8 variants would fit three,
    // measured slightly slower (smaller parts, no more bandwidth)
    if (per_cu > 2) per_cu = 2;
    *n = per_cu * prop.multiProcessorCount;
  };
  resident((const void*)k_filter_score_bf16<G, false, kKind, false>, &out[0]);
  resident((const void*)k_filter_score_bf16<G, true, kKind, false>, &out[1]);
  return e;
}

// Workgroups of the filtered scoring kernel that the current device holds at once (its launch size), for
// a contiguous cache (out[0]) and a paged one (out[1]); the variants differ in registers, hence in occupancy.
// k_kind: 0 bf16, 1 FP8, 2 fp16 keys.
hipError_t filter_score_blocks(const Shape& s, int k_kind, int out[2]) {
#define LFPS_RESIDENT(GG)                                                   \
  switch (k_kind) {                                                         \
    case kKindBf16: return filter_resident_blocks<GG, kKindBf16>(out);      \
    case kKindFp8: return filter_resident_blocks<GG, kKindFp8>(out);        \
    case kKindF16: return filter_resident_blocks<GG, kKindF16>(out);        \
    default: return hipErrorInvalidValue;                                   \
  }
  switch (s.G) {
    case 1: LFPS_RESIDENT(1)
    case 2: LFPS_RESIDENT(2)
    case 4: LFPS_RESIDENT(4)
    default: return hipErrorInvalidValue;
  }
#undef LFPS_RESIDENT
}

hipError_t launch_filter_score(const Shape& s, const float* q, const KvView& kv, const int32_t* cand,
                               const int32_t* cand_count, const int64_t* group_start, const int64_t* line_total,
                               const float* thr_state, float margin, float* score,
                               int32_t* slot_out, int64_t score_stride, int32_t* seg_count, int32_t* seg_rows_out,
                               int n_blocks, int32_t* flags, bool dense, int nseg, hipStream_t st) {
  if (n_blocks < 1) return hipErrorInvalidValue;
  const bool f16 = kv.f16;
  dim3 grid((unsigned)n_blocks), block(kScoreThreads);
  const float scale = 0.08838834764831845f;
#define LFPS_LAUNCH_FILTER_D(GG, PAGED, FP8, DENSE)                                                                \
  hipLaunchKernelGGL((k_filter_score_bf16<GG, PAGED, FP8, DENSE>), grid, block, 0, st, s, q, kv.k, kv.stride_b,    \
                     kv.stride_h, kv.stride_n, kv.page, kv.seq_lens, cand, cand_count, group_start, line_total,    \
                     thr_state, margin, score, slot_out, score_stride, seg_count, seg_rows_out,                    \
                     filter_min_seg_rows(s), nseg, scale, flags)
#define LFPS_LAUNCH_FILTER_P(GG, PAGED, FP8)       \
  if (dense) {                                     \
    LFPS_LAUNCH_FILTER_D(GG, PAGED, FP8, true);    \
  } else {                                         \
    LFPS_LAUNCH_FILTER_D(GG, PAGED, FP8, false);   \
  }
#define LFPS_LAUNCH_FILTER(GG)                        \
  if (kv.page.table && kv.k_fp8) {                    \
    LFPS_LAUNCH_FILTER_P(GG, true, kKindFp8);         \
  } else if (kv.page.table && f16) {                  \
    LFPS_LAUNCH_FILTER_P(GG, true, kKindF16);         \
  } else if (kv.page.table) {                         \
    LFPS_LAUNCH_FILTER_P(GG, true, kKindBf16);        \
  } else if (kv.k_fp8) {                              \
    LFPS_LAUNCH_FILTER_P(GG, false, kKindFp8);        \
  } else if (f16) {                                   \
    LFPS_LAUNCH_FILTER_P(GG, false, kKindF16);        \
  } else {                                            \
    LFPS_LAUNCH_FILTER_P(GG, false, kKindBf16);       \
  }
  switch (s.G) {
    case 1: LFPS_LAUNCH_FILTER(1); break;
    case 2: LFPS_LAUNCH_FILTER(2); break;
    case 4: LFPS_LAUNCH_FILTER(4); break;
    default: return hipErrorInvalidValue;
  }
#undef LFPS_LAUNCH_FILTER_P
#undef LFPS_LAUNCH_FILTER_D
#undef LFPS_LAUNCH_FILTER
  return hipGetLastError();
}

hipError_t launch_head_score(const Shape& s, int dtype, const float* q, const KvView& kv, const int32_t* idx,
                             const int32_t* k, float* idx_score, hipStream_t st) {
  dim3 grid((s.kmax + 255) / 256, s.B * s.Hq), block(256);
  const float scale = 0.08838834764831845f;
#define LFPS_LAUNCH_HS(TYPE, PAGED)                                                                            \
  hipLaunchKernelGGL((k_head_score<TYPE, PAGED>), grid, block, 0, st, s, q, (const TYPE*)kv.k, kv.stride_b,     \
                     kv.stride_h, kv.stride_n, kv.page, kv.seq_lens, idx, k, idx_score, scale)
  const bool paged = kv.page.table != nullptr;
  if (dtype == LFPS_BF16 && kv.k_fp8) {
    if (paged) LFPS_LAUNCH_HS(uint8_t, true);
    else LFPS_LAUNCH_HS(uint8_t, false);
  } else if (dtype == LFPS_BF16) {
    if (paged) LFPS_LAUNCH_HS(uint16_t, true);
    else LFPS_LAUNCH_HS(uint16_t, false);
  } else if (dtype == LFPS_F16) {
    if (paged) LFPS_LAUNCH_HS(_Float16, true);
    else LFPS_LAUNCH_HS(_Float16, false);
  } else {
    if (paged) LFPS_LAUNCH_HS(float, true);
    else LFPS_LAUNCH_HS(float, false);
  }
#undef LFPS_LAUNCH_HS
  return hipGetLastError();
}

}  // namespace lfps
