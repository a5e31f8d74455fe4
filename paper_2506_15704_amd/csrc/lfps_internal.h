// Internal declarations shared by the translation units of liblfps (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lfps.h"

namespace lfps {

constexpr int kD = 128;           // head_dim the kernels are written for
constexpr int kMaxSplits = 64;    // upper bound of split-K partials per head (full attention)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Where the rows of a request live when the cache is paged (table != nullptr): a pool of blocks of
// 2^shift rows, table[b*table_stride + (i >> shift)] = block of row i of request b.
struct KvPage {
  const int32_t* table;
  int32_t table_stride, shift, n_blocks;
};

// Strided view of K or V in elements, resolved for one launch.
struct KvView {
  const void* k;
  const void* v;
  int64_t stride_b, stride_h, stride_n;
  const int32_t* seq_lens;
  KvPage page;
  bool k_fp8;   // K elements are one byte (OCP FP8 E4M3)
  bool v_fp8;   // V elements are one byte; otherwise V has the cache dtype
  bool f16;     // the cache dtype is fp16 (K and V)
};

// Row addressing of the two cache layouts, chosen at compile time.  A logical row i of request b
// is first turned into a "physical row" p (an int32: i itself, or block * block_size + i % block_size;
// the only step that reads memory, and only when paged), from which the element offset follows by
// arithmetic.  Kernels translate where a row id first lives in a register and keep p from there on.
template <bool kPaged>
struct RowMap {
  __device__ __forceinline__ static int phys(const KvPage& pg, int b, int i) {
    if constexpr (!kPaged) {
      return i;
    } else {
      int blk = pg.table[(int64_t)b * pg.table_stride + (i >> pg.shift)];
      blk = blk < 0 ? 0 : (blk >= pg.n_blocks ? pg.n_blocks - 1 : blk);   // a bad entry reads a wrong block, never outside the pool
      return (blk << pg.shift) | (i & ((1 << pg.shift) - 1));
    }
  }
  // element offset of the start of (b, g)'s rows, to which offset(p) is added
  __device__ __forceinline__ static int64_t base(int b, int g, int64_t stride_b, int64_t stride_h) {
    return (kPaged ? (int64_t)0 : (int64_t)b * stride_b) + (int64_t)g * stride_h;
  }
  __device__ __forceinline__ static int64_t offset(const KvPage& pg, int p, int64_t stride_b, int64_t stride_n) {
    if constexpr (!kPaged) {
      return (int64_t)p * stride_n;
    } else {
      return (int64_t)(p >> pg.shift) * stride_b + (int64_t)(p & ((1 << pg.shift) - 1)) * stride_n;
    }
  }
};

// Shapes every kernel needs.
struct Shape {
  int32_t B, Hq, Hkv, G;
  int32_t Lcap, kmax, cand_cap;
  int32_t radius, n_recent, n_sink;
  int32_t score_stride;   // row length of the workspace score buffer [B, Hq, score_stride]
};

// ---- kernel launchers (each enqueues on `st` and returns the launch error) -------------
hipError_t configure_candidates(const Shape& s);
hipError_t configure_select(const Shape& s);
// group_start [B,Hkv] / line_total [1] (or NULL): every group adds its candidate count to *line_total
// (zero on entry) and keeps the value before the addition as its place on the line of all candidate slots.
hipError_t launch_candidates(const Shape& s, const int32_t* prev_topk, const int32_t* k, const int32_t* seq_lens,
                             int32_t* cand, int32_t* cand_count, int32_t* flags, int64_t* group_start,
                             int64_t* line_total, hipStream_t st);

// Scores of candidate rows (cand != NULL) or of all rows 0..n_b-1 (cand == NULL) for the G heads
// of each KV group.  score is [B, Hq, score_stride].
// flags: the context's status word (LFPS_FLAG_Q_RANGE is raised there).  A candidate entry outside [0, n_b)
// scores -inf.
hipError_t launch_group_score(const Shape& s, int dtype, const float* q, const KvView& kv, const int32_t* cand,
                              const int32_t* cand_count, float* score, int64_t score_stride, int32_t* flags,
                              hipStream_t st);

// Filtered scoring (bf16, fp16 or FP8 keys; the kernel keeps its first name, k_filter_score_bf16): per
// head only rows with score >= thr_state[b,h] - margin are kept, as
// (score, position) lists in at most filter_nseg(s) pieces per head.  The kernel runs with exactly
// n_blocks workgroups (filter_score_blocks: what the device holds at once) and cuts the candidate
// slots of all groups (placed on one line by the candidates kernel: group_start, line_total) into
// equal parts, one per wave; the part size of a step is written to *seg_rows_out by the scoring
// pass and read by the select, which also resets *line_total; see score.hip.
int filter_nseg(const Shape& s);
int filter_list_cap(const Shape& s);   // survivors per head the filtered select can hold
hipError_t filter_score_blocks(const Shape& s, int k_kind, int out[2]);
hipError_t launch_filter_score(const Shape& s, const float* q, const KvView& kv, const int32_t* cand,
                               const int32_t* cand_count, const int64_t* group_start, const int64_t* line_total,
                               const float* thr_state, float margin, float* score,
                               int32_t* slot_out, int64_t score_stride, int32_t* seg_count, int32_t* seg_rows_out,
                               int n_blocks, int32_t* flags, bool dense, int nseg, hipStream_t st);
// S3 + S4 of the chained steps in one kernel (select_attend.hip).  From the survivor lists of the filtered scoring
// pass: every head gets its Top-k rows (topk_idx, topk_score: both required) and its output row; a head whose list
// is short or overfull takes the unfiltered pass inside the kernel (counted in *rescored), which needs q, the K rows
// and the group's candidate list (cand; NULL = all rows 0 .. cand_count-1) and overwrites the head's score row.
hipError_t configure_select_attend(const Shape& s);
hipError_t launch_filter_select_attend(const Shape& s, int dtype, float* score, const int32_t* slot_in,
                                       int64_t score_stride, const int32_t* seg_count, const int32_t* seg_rows, int nseg,
                                       const int32_t* cand, const int32_t* cand_count, const int64_t* group_start,
                                       int64_t* line_total, const int32_t* k, int32_t* topk_idx, float* topk_score,
                                       float* thr_state, const int32_t* skip_if, int32_t* rescored, const float* q,
                                       int32_t* flags, const KvView& kv, float* out,
                                       hipStream_t st);   // out == NULL: select only

// Exact Top-k baseline, set-up of its filtered dense pass (exact_topk.hip): every group's rows 0..n_b-1 laid on the
// line (x_cnt, x_start, x_start[B*Hkv] = the line's length), a strided sample of at most ns_max rows per group
// (sized for the select's list capacity list_cap)
// (sample [B, Hkv, cand_cap], x_nsg [B*Hkv] / x_ns [B] its length) and the rank x_rank [B] whose sample score is
// taken as the threshold.
hipError_t launch_dense_prep(const Shape& s, const int32_t* seq_lens, const int32_t* k, int ns_max, int list_cap,
                             int32_t* x_cnt,
                             int64_t* x_start, int32_t* x_nsg, int32_t* x_ns, int32_t* x_rank, int32_t* sample,
                             hipStream_t st);
// From the full score rows [B, Hq, score_stride] over cand, every head.
hipError_t launch_select_attend(const Shape& s, int dtype, const float* score, int64_t score_stride, const int32_t* cand,
                                const int32_t* cand_count, const int32_t* k, int32_t* topk_idx, float* topk_score,
                                float* thr_state, const int32_t* skip_if, const KvView& kv, float* out,
                                hipStream_t st);

// Per (b, h): the k_b best of score[b,h,0:count]; count = cand_count[b, g(h)] when cand != NULL,
// else seq_lens[b].  Writes positions (ascending) and their scores.
// thr_state [B,Hq] (or NULL) receives
// each head's k-th best score.  skip_if [B,Hq] (or NULL): heads whose entry is not 0 are skipped (bypassed heads).
// seq_lens [B] (or NULL; with cand only): a selected candidate entry outside [0, n_b) is written as -1.
hipError_t launch_select(const Shape& s, const float* score, int64_t score_stride, const int32_t* cand,
                         const int32_t* count, const int32_t* k, int32_t* topk_idx, float* topk_score,
                         float* thr_state, const int32_t* skip_if, const int32_t* seq_lens, hipStream_t st);

// Scores of idx[b,h,0:k_b] rows against q[b,h] (one head at a time, no group sharing).
hipError_t launch_head_score(const Shape& s, int dtype, const float* q, const KvView& kv, const int32_t* idx,
                             const int32_t* k, float* idx_score, hipStream_t st);

// Sparse attention: one workgroup per (b, h), output row written directly.
hipError_t launch_sparse_attn(const Shape& s, int dtype, const KvView& kv, const int32_t* idx, const float* idx_score,
                              const int32_t* k, float* out, const int32_t* skip_if, hipStream_t st);

// Full attention: split partials [B*Hkv, n_split, G, D+2] + merge.
int full_attn_splits(const Shape& s);
hipError_t launch_full_attn(const Shape& s, int dtype, const float* q, const KvView& kv, float* part, int n_split,
                            hipStream_t st);
hipError_t launch_full_merge(const Shape& s, const int32_t* seq_lens, const float* part, int n_split, float* out,
                             hipStream_t st);

// Score tables (Eq. 4, 7-10): see tables.hip.  tab_ver [B*Hq, Lcap], tab_sla [B*Hq, 2*Lcap] unscaled fp32
// entries; state [B*Hq, kTableStateDoubles]; f0 / fm [B*Hq, flag_words] bitmaps written by the scan.
constexpr int kTableStateDoubles = 16;
hipError_t launch_table_flags(const Shape& s, const float* tab_ver, const float* tab_sla, const double* state,
                              const int32_t* seq_lens, uint32_t* f0, uint32_t* fm, int flag_words, double a,
                              const int32_t* gate, hipStream_t st);
hipError_t launch_table_candidates(const Shape& s, const uint32_t* f0, const uint32_t* fm, int flag_words,
                                   const int32_t* seq_lens, int32_t* cand, int32_t* cand_count, int32_t* flags,
                                   int64_t* group_start, int64_t* line_total, hipStream_t st);
hipError_t launch_table_update(const Shape& s, float* tab_ver, float* tab_sla, double* state, const int32_t* seq_lens,
                               const int32_t* idx, const float* sc, const int32_t* k, double gamma, const int32_t* gate,
                               int32_t* flags, bool distinct, hipStream_t st);   // distinct: no position twice in a head's list
hipError_t launch_table_import(const Shape& s, float* tab_ver, float* tab_sla, double* state, const int32_t* seq_lens,
                               const float* phi_ver, const float* phi_sla, hipStream_t st);
hipError_t launch_table_export(const Shape& s, const float* tab_ver, const float* tab_sla, const double* state,
                               const int32_t* seq_lens, double* phi_ver, double* phi_sla, hipStream_t st);
hipError_t launch_table_init(const Shape& s, float* tab_ver, float* tab_sla, const int32_t* seq_lens,
                             const float* score, int64_t score_stride, double gamma, int j, int n_queries,
                             hipStream_t st);
hipError_t launch_table_finish(const Shape& s, const float* tab_ver, const float* tab_sla, double* state,
                               const int32_t* seq_lens, hipStream_t st);
// Head sparsity (Eq. 5-6) and the prefill priors it needs; gate [B,Hq] marks bypassed heads, whose output
// row (vbar) and index row (-1) the kernel writes when out != NULL; thr_state (or NULL): the score filter's
// per-head history, where a bypassed head without history is given +inf.
hipError_t launch_head_sparsity(const Shape& s, int dtype, const float* q, const KvView& kv, const float* kbar,
                                const float* sigma2_hat, int n_local, float eps, float* rho, int32_t* gate,
                                const float* vbar, int32_t* topk_idx, float* topk_score, float* out, float* thr_state,
                                hipStream_t st);
hipError_t launch_prior_means(const Shape& s, int dtype, const KvView& kv, float* kbar, float* vbar, hipStream_t st);
hipError_t launch_prior_variance(const Shape& s, const float* q, const int32_t* seq_lens, const float* score,
                                 int64_t score_stride, float* sigma2_hat, hipStream_t st);

// ---- small device helpers ------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// OCP FP8 E4M3 ("FN": no infinities, one NaN pattern per sign, largest value 448) to fp32: four values of
// one dword, lowest byte first.  The hardware conversion is exact.
__device__ __forceinline__ void fp8x4_to_f32(uint32_t w, float x[4]) {
  const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
  const auto hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
  x[0] = lo[0];
  x[1] = lo[1];
  x[2] = hi[0];
  x[3] = hi[1];
}
// Eight E4M3 values as eight bf16 (exact: 3 mantissa bits fit bf16's 7, the exponent range is inside fp32's):
// the upper halves of the fp32 conversions, packed two per dword.
__device__ __forceinline__ bf16x8 fp8x8_to_bf16x8(uint32_t w0, uint32_t w1) {
  float a[4], b[4];
  fp8x4_to_f32(w0, a);
  fp8x4_to_f32(w1, b);
  auto pack = [](float lo, float hi) { return (__float_as_uint(hi) & 0xFFFF0000u) | (__float_as_uint(lo) >> 16); };
  union {
    u32x4 u;
    bf16x8 v;
  } r;
  r.u[0] = pack(a[0], a[1]);
  r.u[1] = pack(a[2], a[3]);
  r.u[2] = pack(b[0], b[1]);
  r.u[3] = pack(b[2], b[3]);
  return r.v;
}

// Eight consecutive elements of a K or V row as they are loaded (T = float, uint16_t = bf16 bits, _Float16,
// uint8_t = E4M3), converted to fp32 when used: a row waiting in registers costs 8, 4 or 2 of them.
template <typename T>
struct Raw8;
template <>
struct Raw8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = reinterpret_cast<const float4*>(p)[0];
    b = reinterpret_cast<const float4*>(p)[1];
  }
  __device__ __forceinline__ void get(float x[8]) const {
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
};
template <>
struct Raw8<uint16_t> {
  u32x4 w;
  __device__ __forceinline__ void load(const uint16_t* p) { w = *reinterpret_cast<const u32x4*>(p); }
  __device__ __forceinline__ void get(float x[8]) const {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      x[2 * c] = bf16_lo(w[c]);
      x[2 * c + 1] = bf16_hi(w[c]);
    }
  }
};
template <>
struct Raw8<_Float16> {
  f16x8 w;
  __device__ __forceinline__ void load(const _Float16* p) { w = *reinterpret_cast<const f16x8*>(p); }
  __device__ __forceinline__ void get(float x[8]) const {
#pragma unroll
    for (int c = 0; c < 8; ++c) x[c] = (float)w[c];
  }
};
template <>
struct Raw8<uint8_t> {
  uint2 w;
  __device__ __forceinline__ void load(const uint8_t* p) { w = *reinterpret_cast<const uint2*>(p); }
  __device__ __forceinline__ void get(float x[8]) const {
    fp8x4_to_f32(w.x, x);
    fp8x4_to_f32(w.y, x + 4);
  }
};
template <typename T>
__device__ __forceinline__ void load8(const T* p, float x[8]) {
  Raw8<T> r;
  r.load(p);
  r.get(x);
}

// Inclusive prefix sum over the 64 lanes of a wave, on the vector ALU alone (DPP row shifts inside each row of
// 16 lanes, then two row broadcasts for the carries); a scan by lane shuffles costs six LDS-crossbar round trips.
__device__ __forceinline__ int wave_inclusive_sum(int x) {
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);   // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);   // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false);   // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false);   // row_shr:8
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
  return x;
}

// Order-preserving map fp32 -> uint32 (larger float <=> larger key).
__device__ __forceinline__ uint32_t f2key(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

}  // namespace lfps
