// The C ABI of liblfps: context, argument validation, workspace, per-kernel timing, and the
// sequencing of the kernels for each entry point.  No arithmetic of the method lives here.
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>

#include "lfps_internal.h"

using namespace lfps;

struct lfps_ctx {
  lfps_config cfg;
  Shape shape;
  int n_split_full;
  int filter_on;       // filtered scoring inside lfps_step (bf16 / fp16 / FP8-key caches)
  int no_history;      // no chained step since creation / lfps_reset_history: no head has a remembered score
  int nseg;            // survivor pieces per head (row length of seg_count)
  int filter_blocks[2];   // launch size of the filtered scoring kernel (contiguous, paged cache): the workgroups the device holds at once
  // workspace (device)
  float* score;        // [B, Hq, score_stride]
  int32_t* slot;       // [B, Hq, score_stride] candidate slots of the filtered survivors
  int32_t* seg_count;  // [B, Hq, nseg]
  float* thr_state;    // [B, Hq] k-th best score of the previous step
  int64_t* group_start; // [B, Hkv] place of each group on the line of all candidate slots; [B*Hkv] = the line's length
  // score tables (table_mode)
  float* tab_ver;      // [B, Hq, Lcap]
  float* tab_sla;      // [B, Hq, 2*Lcap]
  double* tab_state;   // [B, Hq, kTableStateDoubles]
  uint32_t* tab_f0;    // [B, Hq, flag_words]
  uint32_t* tab_fm;    // [B, Hq, flag_words]
  int flag_words;
  int tab_updates;     // update calls since the last import / init (graph replays are not seen here: the kernel checks too)
  int tab_ready;
  int32_t* gate;       // [B, Hq] bypass marks of the current gated step
  int32_t* cand;       // [B, Hkv, cand_cap]
  int32_t* cand_count; // [B, Hkv]
  float* sel_score;    // [B, Hq, kmax]
  float* part;         // split partials of the full-attention baseline
  // exact Top-k baseline in its filtered form (x_fast): the dense rows on the line, the sample and its rank
  int x_fast;
  int32_t* x_cnt;      // [B, Hkv] rows of each group
  int32_t* x_nsg;      // [B, Hkv] sample rows of each group
  int32_t* x_ns;       // [B] the same per request
  int32_t* x_rank;     // [B] rank of the sample score taken as threshold
  int64_t* x_start;    // [B*Hkv + 1] place of each group on the line of all rows, then the line's length
  float* thr_x;        // [B, Hq] thresholds of the dense filtered pass
  int32_t* flags;      // [0] status flags, [1] part size chosen by the last filtered scoring pass, [2] heads rescored since the last poll
  int64_t ws_bytes;
  // timing
  int timing_on;
  int n_timed;
  hipEvent_t ev[LFPS_TIMING_MAX_LAUNCHES][2];
  int8_t ev_slot[LFPS_TIMING_MAX_LAUNCHES];
  int events_made;
  char err[512];
};

static thread_local char g_create_err[512] = "";

static const char* const kKernelNames[LFPS_N_KERNELS] = {
    "candidates", "gather_score", "select", "sparse_attn",
    "dense_score", "full_attn", "full_merge", "head_score", "filter_score", "filter_select",
    "table_flags", "table_candidates", "table_update", "filter_select_attend", "select_attend"};

// Margin below the previous step's k-th best score at which the filtered pass keeps a row.
static const float kFilterMargin = 0.125f;
// Exact Top-k baseline: rows sampled per KV group for the threshold, and the size from which the filtered form is used.
static const int kExactSampleRows = 32768;   // at most; the set-up kernel sizes the sample for the budget and the list
static const int64_t kExactFastMinRows = 1 << 20;

namespace {

struct Sizes {
  int32_t G, cand_cap, score_stride, n_split_full, nseg, flag_words;
  int64_t score_b, cand_b, count_b, sel_b, part_b, slot_b, seg_b, thr_b, line_b, tver_b, tsla_b, tstate_b, tflag_b, x_b, total;
};

int64_t align256(int64_t x) { return (x + 255) & ~(int64_t)255; }

int check_config(const lfps_config* c, Sizes* z, char* err, size_t errn) {
#define BAD(...)                      \
  do {                                \
    snprintf(err, errn, __VA_ARGS__); \
    return LFPS_EINVAL;               \
  } while (0)
  if (!c) BAD("config is NULL");
  if (c->batch < 1) BAD("batch must be >= 1 (got %d)", c->batch);
  if (c->n_kv_heads < 1 || c->n_q_heads < 1 || c->n_q_heads % c->n_kv_heads != 0)
    BAD("n_q_heads (%d) must be a positive multiple of n_kv_heads (%d)", c->n_q_heads, c->n_kv_heads);
  const int G = c->n_q_heads / c->n_kv_heads;
  if (G != 1 && G != 2 && G != 4) BAD("heads per KV group must be 1, 2 or 4 (got %d)", G);
  if ((int64_t)c->batch * c->n_q_heads > 65535)
    BAD("batch * n_q_heads must be <= 65535 (one grid row per head; got %d * %d)", c->batch, c->n_q_heads);
  if (c->head_dim != kD) BAD("head_dim must be %d (got %d)", kD, c->head_dim);
  if (c->kv_dtype != LFPS_F32 && c->kv_dtype != LFPS_BF16 && c->kv_dtype != LFPS_F16)
    BAD("kv_dtype must be LFPS_F32, LFPS_BF16 or LFPS_F16");
  if (c->max_seq_len < 1) BAD("max_seq_len must be >= 1");
  if (c->max_k < 1 || c->max_k > c->max_seq_len) BAD("max_k must be in [1, max_seq_len]");
  if (c->radius < 0 || c->n_recent < 0 || c->n_sink < 0) BAD("radius, n_recent, n_sink must be >= 0");
  if (c->cand_cap < 0) BAD("cand_cap must be >= 0");
  if (c->device < 0) BAD("device must be >= 0");
  if (c->table_mode != 0 && c->table_mode != 1) BAD("table_mode must be 0 or 1");
  if (c->table_mode) {
    if (!(c->table_decay > 0.f && c->table_decay < 1.f)) BAD("table_decay must lie in (0, 1) (got %g)", c->table_decay);
    if (!(c->table_a > 0.f)) BAD("table_a must be > 0 (got %g)", c->table_a);
    if (c->radius > 30) BAD("table mode supports radius <= 30 (got %d)", c->radius);
  }
  if (c->k_fp8 != 0 && c->k_fp8 != 1) BAD("k_fp8 must be 0 or 1");
  if (c->k_fp8 && c->kv_dtype != LFPS_BF16) BAD("k_fp8 needs kv_dtype = LFPS_BF16 (FP8 keys beside bf16 values)");
  if (c->v_fp8 != 0 && c->v_fp8 != 1) BAD("v_fp8 must be 0 or 1");
  if (c->v_fp8 && c->kv_dtype != LFPS_BF16) BAD("v_fp8 needs kv_dtype = LFPS_BF16");
#undef BAD
  // LDS of the candidate kernel: one bit per position beside 64 KB of staging, 160 KB per workgroup
  if (((int64_t)c->max_seq_len + 31) / 32 * 4 > 88 * 1024) {
    snprintf(err, errn, "max_seq_len %d exceeds the candidate bitmap capacity (%d positions)", c->max_seq_len,
             88 * 1024 * 8);
    return LFPS_ECAP;
  }
  int64_t bound = (int64_t)G * c->max_k * (2 * (int64_t)c->radius + 2) + c->n_recent + c->n_sink;
  if (bound > c->max_seq_len) bound = c->max_seq_len;
  z->G = G;
  if (c->table_mode) bound = c->max_seq_len;      // table candidates are not bounded by the budget
  z->cand_cap = c->cand_cap > 0 ? c->cand_cap : (int32_t)bound;
  if (z->cand_cap > c->max_seq_len) z->cand_cap = c->max_seq_len;
  z->score_stride = (c->max_seq_len + 63) & ~63;    // holds candidate scores and dense scores
  Shape s{};
  s.B = c->batch; s.Hq = c->n_q_heads; s.Hkv = c->n_kv_heads; s.G = G;
  s.Lcap = c->max_seq_len; s.kmax = c->max_k; s.cand_cap = z->cand_cap;
  z->n_split_full = full_attn_splits(s);
  z->score_b = align256((int64_t)c->batch * c->n_q_heads * z->score_stride * 4);
  z->cand_b = align256((int64_t)c->batch * c->n_kv_heads * z->cand_cap * 4);
  z->count_b = align256((int64_t)c->batch * c->n_kv_heads * 4);
  z->sel_b = align256((int64_t)c->batch * c->n_q_heads * c->max_k * 4);
  z->part_b = align256((int64_t)c->batch * c->n_kv_heads * z->n_split_full * G * (kD + 2) * 4);
  const bool filt = c->kv_dtype == LFPS_BF16 || c->kv_dtype == LFPS_F16;
  z->nseg = filter_nseg(s);
  {
    Shape sd = s;                        // the dense filtered pass of the exact Top-k baseline cuts all Lcap rows
    sd.cand_cap = s.Lcap;
    const int nd = filter_nseg(sd);
    z->nseg = nd > z->nseg ? nd : z->nseg;
  }
  z->slot_b = filt ? z->score_b : 0;
  z->seg_b = align256((int64_t)c->batch * c->n_q_heads * z->nseg * 4);
  z->thr_b = align256((int64_t)c->batch * c->n_q_heads * 4);
  z->line_b = align256(((int64_t)c->batch * c->n_kv_heads + 1) * 8);   // group_start and the line's length
  z->flag_words = ((c->max_seq_len + 63) / 64) * 2 + 2;
  const int64_t heads = (int64_t)c->batch * c->n_q_heads;
  z->tver_b = c->table_mode ? align256(heads * c->max_seq_len * 4) : 0;
  z->tsla_b = c->table_mode ? align256(heads * c->max_seq_len * 8) : 0;
  z->tstate_b = c->table_mode ? align256(heads * kTableStateDoubles * 8) : 0;
  z->tflag_b = c->table_mode ? align256(heads * z->flag_words * 4) : 0;
  z->x_b = 3 * z->count_b + 2 * align256((int64_t)c->batch * 4) + align256(((int64_t)c->batch * c->n_kv_heads + 1) * 8) + z->thr_b;
  z->total = z->score_b + z->cand_b + z->count_b + z->sel_b + z->part_b + z->slot_b + z->seg_b + z->thr_b +
             z->line_b + 256 + z->x_b + z->tver_b + z->tsla_b + z->tstate_b + 2 * z->tflag_b + z->thr_b /* gate marks */;
  return LFPS_OK;
}

int fail(lfps_ctx* ctx, int code, const char* what, hipError_t e = hipSuccess) {
  if (e != hipSuccess)
    snprintf(ctx->err, sizeof ctx->err, "%s: %s", what, hipGetErrorString(e));
  else
    snprintf(ctx->err, sizeof ctx->err, "%s", what);
  return code;
}

// Validates a cache view against a configuration; the reason of a refusal goes to err.
int check_kv_cfg(const lfps_config& cfg, char* err, size_t errn, const lfps_kv* kv, bool need_v, KvView* out) {
#define BAD(text)                  \
  do {                             \
    snprintf(err, errn, "%s", text); \
    return LFPS_EINVAL;            \
  } while (0)
  if (!kv) BAD("kv view is NULL");
  if (!kv->k) BAD("kv->k is NULL");
  if (need_v && !kv->v) BAD("kv->v is NULL");
  if (!kv->seq_lens) BAD("kv->seq_lens is NULL");
  // the strides are shared by K and V: with one-byte K elements the K rows set the alignment
  const int esz = (cfg.k_fp8 || cfg.v_fp8) ? 1 : (cfg.kv_dtype == LFPS_F32 ? 4 : 2);
  if (kv->stride_n < kD || kv->stride_b < 0 || kv->stride_h < 0)
    BAD("kv strides: stride_n must be >= head_dim, stride_b/stride_h >= 0");
  if ((kv->stride_n * esz) % 16 || (kv->stride_b * esz) % 16 || (kv->stride_h * esz) % 16 ||
      ((uintptr_t)kv->k % 16) || (kv->v && ((uintptr_t)kv->v % 16)))
    BAD("kv rows must be 16-byte aligned (base pointers and strides)");
  out->k = kv->k; out->v = kv->v;
  out->stride_b = kv->stride_b; out->stride_h = kv->stride_h; out->stride_n = kv->stride_n;
  out->seq_lens = kv->seq_lens;
  out->page = KvPage{nullptr, 0, 0, 0};
  out->k_fp8 = cfg.k_fp8 != 0;
  out->v_fp8 = cfg.v_fp8 != 0;
  out->f16 = cfg.kv_dtype == LFPS_F16;
  if (kv->block_table) {
    const int64_t bs = kv->block_size;
    if (bs < 1 || bs > 65536 || (bs & (bs - 1))) BAD("paged kv: block_size must be a power of two in [1, 65536]");
    if (kv->block_table_stride < 1 || (int64_t)kv->block_table_stride * bs < cfg.max_seq_len)
      BAD("paged kv: block_table_stride * block_size must cover max_seq_len");
    if (kv->n_blocks < 1 || (int64_t)kv->n_blocks * bs > 2147483647LL)
      BAD("paged kv: n_blocks must be >= 1 and n_blocks * block_size below 2^31");
    int shift = 0;
    while ((1 << shift) < bs) ++shift;
    out->page = KvPage{kv->block_table, kv->block_table_stride, shift, kv->n_blocks};
  }
#undef BAD
  return LFPS_OK;
}

int check_kv(lfps_ctx* ctx, const lfps_kv* kv, bool need_v, KvView* out) {
  return check_kv_cfg(ctx->cfg, ctx->err, sizeof ctx->err, kv, need_v, out);
}

// Brackets one launch with events when timing is on.
struct Timed {
  lfps_ctx* c;
  hipStream_t st;
  int i;
  Timed(lfps_ctx* ctx, int slot, hipStream_t s) : c(ctx), st(s), i(-1) {
    if (c->timing_on && c->n_timed < LFPS_TIMING_MAX_LAUNCHES) {
      i = c->n_timed++;
      c->ev_slot[i] = (int8_t)slot;
      (void)hipEventRecord(c->ev[i][0], st);
    }
  }
  ~Timed() {
    if (i >= 0) (void)hipEventRecord(c->ev[i][1], st);
  }
};

#define LAUNCH(ctx, slot, st, call)                                         \
  do {                                                                      \
    hipError_t e_;                                                          \
    {                                                                       \
      Timed t_(ctx, slot, st);                                              \
      e_ = (call);                                                          \
    }                                                                       \
    if (e_ != hipSuccess) return fail(ctx, LFPS_EHIP, kKernelNames[slot], e_); \
  } while (0)

}  // namespace

__global__ __launch_bounds__(256) void k_calib_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

extern "C" {

int lfps_calib_copy(void* dst, const void* src, int64_t bytes, void* stream) {
  if (!dst || !src || bytes < 0 || (bytes % 16) || ((uintptr_t)dst % 16) || ((uintptr_t)src % 16)) return LFPS_EINVAL;
  if (bytes == 0) return LFPS_OK;
  const int64_t n16 = bytes / 16;
  int64_t blocks = (n16 + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(k_calib_copy, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)src,
                     (uint4*)dst, n16);
  return hipGetLastError() == hipSuccess ? LFPS_OK : LFPS_EHIP;
}

int lfps_host_device_pointer(const void* host, void** dev) {
  if (!host || !dev) return LFPS_EINVAL;
  *dev = nullptr;
  hipError_t e = hipHostGetDevicePointer(dev, const_cast<void*>(host), 0);
  if (e != hipSuccess || !*dev) {
    snprintf(g_create_err, sizeof g_create_err, "hipHostGetDevicePointer: %s", hipGetErrorString(e));
    (void)hipGetLastError();
    return LFPS_EHIP;
  }
  return LFPS_OK;
}

int lfps_workspace_bytes(const lfps_config* cfg, int64_t* out) {
  Sizes z;
  int rc = check_config(cfg, &z, g_create_err, sizeof g_create_err);
  if (rc != LFPS_OK) return rc;
  if (!out) return LFPS_EINVAL;
  *out = z.total;
  return LFPS_OK;
}

int lfps_create(const lfps_config* cfg, lfps_ctx** out) {
  if (!out) {
    snprintf(g_create_err, sizeof g_create_err, "out pointer is NULL");
    return LFPS_EINVAL;
  }
  *out = nullptr;
  Sizes z;
  int rc = check_config(cfg, &z, g_create_err, sizeof g_create_err);
  if (rc != LFPS_OK) return rc;
  hipError_t e = hipSetDevice(cfg->device);
  if (e != hipSuccess) {
    snprintf(g_create_err, sizeof g_create_err, "hipSetDevice(%d): %s", cfg->device, hipGetErrorString(e));
    return LFPS_EHIP;
  }
  lfps_ctx* c = new (std::nothrow) lfps_ctx();
  if (!c) return LFPS_ENOMEM;
  c->cfg = *cfg;
  c->cfg.cand_cap = z.cand_cap;
  Shape& s = c->shape;
  s.B = cfg->batch; s.Hq = cfg->n_q_heads; s.Hkv = cfg->n_kv_heads; s.G = z.G;
  s.Lcap = cfg->max_seq_len; s.kmax = cfg->max_k; s.cand_cap = z.cand_cap;
  s.radius = cfg->radius; s.n_recent = cfg->n_recent; s.n_sink = cfg->n_sink;
  s.score_stride = z.score_stride;
  c->n_split_full = z.n_split_full;
  c->ws_bytes = z.total;
  char* base = nullptr;
  e = hipMalloc((void**)&base, (size_t)z.total);
  if (e != hipSuccess) {
    snprintf(g_create_err, sizeof g_create_err, "hipMalloc(%lld bytes): %s", (long long)z.total, hipGetErrorString(e));
    delete c;
    (void)hipGetLastError();
    return LFPS_ENOMEM;
  }
  c->score = (float*)base;
  c->cand = (int32_t*)(base + z.score_b);
  c->cand_count = (int32_t*)(base + z.score_b + z.cand_b);
  c->sel_score = (float*)(base + z.score_b + z.cand_b + z.count_b);
  c->part = (float*)(base + z.score_b + z.cand_b + z.count_b + z.sel_b);
  char* p = base + z.score_b + z.cand_b + z.count_b + z.sel_b + z.part_b;
  c->slot = z.slot_b ? (int32_t*)p : nullptr;
  p += z.slot_b;
  c->seg_count = (int32_t*)p;
  p += z.seg_b;
  c->thr_state = (float*)p;
  p += z.thr_b;
  c->group_start = (int64_t*)p;
  p += z.line_b;
  c->flags = (int32_t*)p;
  p += 256;
  {
    const int64_t per_b = align256((int64_t)cfg->batch * 4);
    c->x_cnt = (int32_t*)p;
    c->x_nsg = (int32_t*)(p + z.count_b);
    c->x_ns = (int32_t*)(p + 2 * z.count_b);
    c->x_rank = (int32_t*)(p + 2 * z.count_b + per_b);
    c->x_start = (int64_t*)(p + 2 * z.count_b + 2 * per_b);
    c->thr_x = (float*)(p + 2 * z.count_b + 2 * per_b + align256(((int64_t)cfg->batch * cfg->n_kv_heads + 1) * 8));
    p += z.x_b;
  }
  if (cfg->table_mode) {
    c->tab_ver = (float*)p;
    p += z.tver_b;
    c->tab_sla = (float*)p;
    p += z.tsla_b;
    c->tab_state = (double*)p;
    p += z.tstate_b;
    c->tab_f0 = (uint32_t*)p;
    p += z.tflag_b;
    c->tab_fm = (uint32_t*)p;
    p += z.tflag_b;
    c->flag_words = z.flag_words;
  }
  c->gate = (int32_t*)p;
  c->nseg = z.nseg;
  // The filtered pass pays off only if a head's survivors (about 1.25 x its budget) fit the select's list; with a
  // budget too large for that every head would be rescored anyway, so such a context starts with the filter off.
  c->no_history = 1;
  c->filter_on = (z.slot_b && (int64_t)cfg->max_k + cfg->max_k / 4 <= filter_list_cap(s)) ? 1 : 0;
  // The exact Top-k baseline takes the filtered scoring pass too (threshold from a sample of the rows) once the
  // contexts are large enough for the extra launches to pay: about a million rows in all.
  c->x_fast = (z.slot_b && (int64_t)cfg->batch * cfg->n_kv_heads * cfg->max_seq_len >= kExactFastMinRows) ? 1 : 0;
  e = hipMemset(c->flags, 0, 256);
  if (e == hipSuccess) e = hipMemset(c->seg_count, 0, (size_t)(z.seg_b + z.thr_b + z.line_b));   // counts, line length
  if (e == hipSuccess) e = hipMemset(c->thr_state, 0xFF, (size_t)z.thr_b);   // all-ones = NaN: "no history"
  if (e == hipSuccess && cfg->table_mode)
    e = hipMemset(c->tab_ver, 0, (size_t)(z.tver_b + z.tsla_b + z.tstate_b + 2 * z.tflag_b));
  if (e == hipSuccess) e = hipMemset(c->gate, 0, (size_t)z.thr_b);
  if (e == hipSuccess) e = configure_candidates(s);
  if (e == hipSuccess) e = configure_select(s);
  // the launch size of the filtered pass is needed whenever that pass can be switched on (lfps_set_filter)
  if (e == hipSuccess && c->slot)
    e = filter_score_blocks(s, cfg->k_fp8 ? 1 : (cfg->kv_dtype == LFPS_F16 ? 2 : 0), c->filter_blocks);
  if (e == hipSuccess && c->slot && (c->filter_blocks[0] < 1 || c->filter_blocks[1] < 1)) e = hipErrorLaunchFailure;
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    snprintf(g_create_err, sizeof g_create_err, "workspace setup: %s", hipGetErrorString(e));
    (void)hipFree(base);
    delete c;
    return LFPS_EHIP;
  }
  *out = c;
  return LFPS_OK;
}

int lfps_destroy(lfps_ctx* ctx) {
  if (!ctx) return LFPS_EINVAL;
  (void)hipSetDevice(ctx->cfg.device);
  (void)hipDeviceSynchronize();
  for (int i = 0; i < ctx->events_made; ++i) {
    (void)hipEventDestroy(ctx->ev[i][0]);
    (void)hipEventDestroy(ctx->ev[i][1]);
  }
  hipError_t e = hipFree(ctx->score);
  delete ctx;
  return e == hipSuccess ? LFPS_OK : LFPS_EHIP;
}

const char* lfps_last_error(const lfps_ctx* ctx) { return ctx ? ctx->err : g_create_err; }

int32_t lfps_cand_cap(const lfps_ctx* ctx) { return ctx ? ctx->shape.cand_cap : 0; }

const char* lfps_kernel_name(int32_t slot) {
  return (slot >= 0 && slot < LFPS_N_KERNELS) ? kKernelNames[slot] : "";
}

int lfps_candidates(lfps_ctx* ctx, const int32_t* prev_topk, const int32_t* k, const int32_t* seq_lens,
                    int32_t* cand, int32_t* cand_count, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!prev_topk || !k || !seq_lens || !cand || !cand_count)
    return fail(ctx, LFPS_EINVAL, "lfps_candidates: NULL argument");
  hipStream_t st = (hipStream_t)stream;
  LAUNCH(ctx, LFPS_KERNEL_CANDIDATES, st,
         launch_candidates(ctx->shape, prev_topk, k, seq_lens, cand, cand_count, ctx->flags, nullptr, nullptr, st));
  return LFPS_OK;
}

int lfps_score_topk(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const int32_t* cand,
                    const int32_t* cand_count, const int32_t* k, int32_t* topk_idx, float* topk_score,
                    float* cand_score, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!q || !cand || !cand_count || !k || !topk_idx) return fail(ctx, LFPS_EINVAL, "lfps_score_topk: NULL argument");
  KvView v;
  int rc = check_kv(ctx, kv, false, &v);
  if (rc != LFPS_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  const Shape& s = ctx->shape;
  float* sc = cand_score ? cand_score : ctx->score;
  const int64_t stride = cand_score ? s.cand_cap : s.score_stride;
  LAUNCH(ctx, LFPS_KERNEL_GATHER_SCORE, st,
         launch_group_score(s, ctx->cfg.kv_dtype, q, v, cand, cand_count, sc, stride, ctx->flags, st));
  LAUNCH(ctx, LFPS_KERNEL_SELECT, st,
         launch_select(s, sc, stride, cand, cand_count, k, topk_idx, topk_score, nullptr, nullptr, v.seq_lens, st));
  return LFPS_OK;
}

int lfps_sparse_attn(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const int32_t* idx, const float* idx_score,
                     const int32_t* k, float* out, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!idx || !k || !out) return fail(ctx, LFPS_EINVAL, "lfps_sparse_attn: NULL argument");
  if (!idx_score && !q) return fail(ctx, LFPS_EINVAL, "lfps_sparse_attn: q is needed when idx_score is NULL");
  KvView v;
  int rc = check_kv(ctx, kv, true, &v);
  if (rc != LFPS_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  const Shape& s = ctx->shape;
  if (!idx_score) {
    LAUNCH(ctx, LFPS_KERNEL_HEAD_SCORE, st, launch_head_score(s, ctx->cfg.kv_dtype, q, v, idx, k, ctx->sel_score, st));
    idx_score = ctx->sel_score;
  }
  LAUNCH(ctx, LFPS_KERNEL_SPARSE_ATTN, st,
         launch_sparse_attn(s, ctx->cfg.kv_dtype, v, idx, idx_score, k, out, nullptr, st));
  return LFPS_OK;
}

// Does the next chained step take the filtered kernels?  (Decides, too, whether its candidates kernel lays the
// groups on the line: only the filtered select clears the line's length again.)
static bool next_step_filtered(const lfps_ctx* ctx) { return ctx->filter_on && !ctx->no_history; }

// S2 + S3 + S4 over ctx->cand / ctx->cand_count inside the chained entry points.  With the score filter on
// (16-bit and FP8-key caches): survivors of the per-head threshold, then select and attention in one kernel, which
// also takes the unfiltered pass for the heads the filter left short.  Without it: every score, then select and
// attention; also for the first step after creation or lfps_reset_history, when no head has a remembered score and
// the filtered form would send every head through its slower in-kernel fallback.
// The candidates kernel of the same step has laid the groups on the line (group_start, line_total).
static int score_select_attend(lfps_ctx* ctx, const float* q, const KvView& v, const int32_t* k, int32_t* topk_idx,
                               float* sel, float* out, const int32_t* skip_if, hipStream_t st) {
  const Shape& s = ctx->shape;
  int64_t* line_total = ctx->group_start + (int64_t)s.B * s.Hkv;
  const bool filtered = next_step_filtered(ctx);
  ctx->no_history = 0;                       // either form leaves every selecting head's k-th best score behind
  if (filtered) {
    LAUNCH(ctx, LFPS_KERNEL_FILTER_SCORE, st,
           launch_filter_score(s, q, v, ctx->cand, ctx->cand_count, ctx->group_start, line_total, ctx->thr_state,
                               kFilterMargin, ctx->score, ctx->slot, s.score_stride, ctx->seg_count, ctx->flags + 1,
                               ctx->filter_blocks[v.page.table ? 1 : 0], ctx->flags, false, ctx->nseg, st));
    LAUNCH(ctx, LFPS_KERNEL_FILTER_SELECT_ATTEND, st,
           launch_filter_select_attend(s, ctx->cfg.kv_dtype, ctx->score, ctx->slot, s.score_stride, ctx->seg_count,
                                       ctx->flags + 1, ctx->nseg, ctx->cand, ctx->cand_count, ctx->group_start,
                                       line_total, k, topk_idx, sel, ctx->thr_state, skip_if, ctx->flags + 2, q,
                                       ctx->flags, v, out, st));
    return LFPS_OK;
  }
  LAUNCH(ctx, LFPS_KERNEL_GATHER_SCORE, st,
         launch_group_score(s, ctx->cfg.kv_dtype, q, v, ctx->cand, ctx->cand_count, ctx->score, s.score_stride,
                            ctx->flags, st));
  LAUNCH(ctx, LFPS_KERNEL_SELECT_ATTEND, st,
         launch_select_attend(s, ctx->cfg.kv_dtype, ctx->score, s.score_stride, ctx->cand, ctx->cand_count, k, topk_idx,
                              sel, ctx->thr_state, skip_if, v, out, st));
  return LFPS_OK;
}

int lfps_step(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const int32_t* prev_topk, const int32_t* k,
              int32_t* topk_idx, float* topk_score, float* out, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!q || !prev_topk || !k || !topk_idx || !out) return fail(ctx, LFPS_EINVAL, "lfps_step: NULL argument");
  const Shape& s = ctx->shape;
  {
    const int64_t nn = (int64_t)s.B * s.Hq * s.kmax;
    if ((prev_topk < topk_idx + nn) && (topk_idx < prev_topk + nn))
      return fail(ctx, LFPS_EINVAL, "lfps_step: prev_topk and topk_idx overlap");
  }
  KvView v;
  int rc = check_kv(ctx, kv, true, &v);
  if (rc != LFPS_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  float* sel = topk_score ? topk_score : ctx->sel_score;
  int64_t* line_total = ctx->group_start + (int64_t)s.B * s.Hkv;   // zero between steps: the filtered select resets it
  LAUNCH(ctx, LFPS_KERNEL_CANDIDATES, st,
         launch_candidates(s, prev_topk, k, v.seq_lens, ctx->cand, ctx->cand_count, ctx->flags,
                           next_step_filtered(ctx) ? ctx->group_start : nullptr, line_total, st));
  return score_select_attend(ctx, q, v, k, topk_idx, sel, out, nullptr, st);
}

// ---------------------------------------------------------------------------- allocation-free S4
// The scores of the selected rows (the scratch buffer between the per-head scoring kernel and the attention
// kernel, `sel_score` in a context's workspace) live in a file-scope device array here, so the call needs no
// context and allocates nothing.  The array's name is a host-side handle, not a device address: the address is
// looked up once per device and only that pointer is ever handed to a kernel.
static __device__ __align__(256) float scratch[LFPS_NOALLOC_MAX_SCORES];
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
float* g_scratch_ptr[kMaxDevices] = {};

// The current device's copy of `scratch` (each device holds its own, at its own address).
int scratch_on_current_device(int device, float** out, char* err, size_t errn) {
  if (device < 0 || device >= kMaxDevices) {
    snprintf(err, errn, "device ordinal %d is beyond the %d this entry point supports", device, kMaxDevices);
    return LFPS_EINVAL;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[device]) {
    float* p = nullptr;
    hipError_t e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      snprintf(err, errn, "hipGetSymbolAddress(scratch) on device %d: %s", device, hipGetErrorString(e));
      (void)hipGetLastError();
      return LFPS_EHIP;
    }
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return LFPS_OK;
}
}  // namespace

int lfps_sparse_attn_noalloc(const lfps_config* cfg, const float* q, const lfps_kv* kv, const int32_t* idx,
                             const int32_t* k, float* out, void* stream) {
  char* err = g_create_err;
  const size_t errn = sizeof g_create_err;
  Sizes z;
  int rc = check_config(cfg, &z, err, errn);
  if (rc != LFPS_OK) return rc;
  if (!q || !idx || !k || !out) {
    snprintf(err, errn, "lfps_sparse_attn_noalloc: NULL argument");
    return LFPS_EINVAL;
  }
  const int64_t need = (int64_t)cfg->batch * cfg->n_q_heads * cfg->max_k;
  if (need > (int64_t)LFPS_NOALLOC_MAX_SCORES) {
    snprintf(err, errn,
             "lfps_sparse_attn_noalloc: batch * n_q_heads * max_k = %lld exceeds the static scratch of %lld scores "
             "(use a context and lfps_sparse_attn for larger shapes)",
             (long long)need, (long long)LFPS_NOALLOC_MAX_SCORES);
    return LFPS_ECAP;
  }
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) {
    snprintf(err, errn, "hipGetDevice: %s", hipGetErrorString(e));
    return LFPS_EHIP;
  }
  if (dev != cfg->device) {
    snprintf(err, errn, "lfps_sparse_attn_noalloc: cfg->device is %d but the current device is %d", cfg->device, dev);
    return LFPS_EINVAL;
  }
  KvView v;
  rc = check_kv_cfg(*cfg, err, errn, kv, true, &v);
  if (rc != LFPS_OK) return rc;
  float* sel = nullptr;
  rc = scratch_on_current_device(dev, &sel, err, errn);
  if (rc != LFPS_OK) return rc;
  Shape s{};
  s.B = cfg->batch; s.Hq = cfg->n_q_heads; s.Hkv = cfg->n_kv_heads; s.G = z.G;
  s.Lcap = cfg->max_seq_len; s.kmax = cfg->max_k; s.cand_cap = z.cand_cap;
  s.radius = cfg->radius; s.n_recent = cfg->n_recent; s.n_sink = cfg->n_sink;
  s.score_stride = z.score_stride;
  hipStream_t st = (hipStream_t)stream;
  e = launch_head_score(s, cfg->kv_dtype, q, v, idx, k, sel, st);
  if (e == hipSuccess) e = launch_sparse_attn(s, cfg->kv_dtype, v, idx, sel, k, out, nullptr, st);
  if (e != hipSuccess) {
    snprintf(err, errn, "lfps_sparse_attn_noalloc: %s", hipGetErrorString(e));
    return LFPS_EHIP;
  }
  return LFPS_OK;
}

int lfps_full_attn_decode(lfps_ctx* ctx, const float* q, const lfps_kv* kv, float* out, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!q || !out) return fail(ctx, LFPS_EINVAL, "lfps_full_attn_decode: NULL argument");
  KvView v;
  int rc = check_kv(ctx, kv, true, &v);
  if (rc != LFPS_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  const Shape& s = ctx->shape;
  LAUNCH(ctx, LFPS_KERNEL_FULL_ATTN, st,
         launch_full_attn(s, ctx->cfg.kv_dtype, q, v, ctx->part, ctx->n_split_full, st));
  LAUNCH(ctx, LFPS_KERNEL_FULL_MERGE, st, launch_full_merge(s, v.seq_lens, ctx->part, ctx->n_split_full, out, st));
  return LFPS_OK;
}

int lfps_exact_topk(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const int32_t* k, int32_t* topk_idx,
                    float* topk_score, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!q || !k || !topk_idx) return fail(ctx, LFPS_EINVAL, "lfps_exact_topk: NULL argument");
  KvView v;
  int rc = check_kv(ctx, kv, false, &v);
  if (rc != LFPS_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  const Shape& s = ctx->shape;
  if (ctx->x_fast && ctx->filter_on) {      // (lfps_set_filter(ctx, 0) also selects the plain form)
    // Threshold per head from a scored sample of the rows, then one filtered pass over all rows and the select from
    // its survivors (exact_topk.hip); a head left short takes the plain pass inside the select kernel.
    Shape sd = s;
    sd.cand_cap = s.Lcap;                 // the "candidates" of the dense pass are all rows of a group
    int64_t* x_total = ctx->x_start + (int64_t)s.B * s.Hkv;
    hipError_t e = launch_dense_prep(s, v.seq_lens, k, kExactSampleRows, filter_list_cap(s), ctx->x_cnt, ctx->x_start, ctx->x_nsg, ctx->x_ns,
                                     ctx->x_rank, ctx->cand, st);
    if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_exact_topk (set-up)", e);
    LAUNCH(ctx, LFPS_KERNEL_GATHER_SCORE, st,
           launch_group_score(s, ctx->cfg.kv_dtype, q, v, ctx->cand, ctx->x_nsg, ctx->score, s.score_stride, ctx->flags,
                              st));
    LAUNCH(ctx, LFPS_KERNEL_SELECT, st,      // the rank-th best sample score of every head -> thr_x (the rows go to scratch)
           launch_select(s, ctx->score, s.score_stride, nullptr, ctx->x_ns, ctx->x_rank, ctx->slot, nullptr, ctx->thr_x,
                         nullptr, nullptr, st));
    LAUNCH(ctx, LFPS_KERNEL_FILTER_SCORE, st,
           launch_filter_score(sd, q, v, nullptr, ctx->x_cnt, ctx->x_start, x_total, ctx->thr_x, 0.f, ctx->score,
                               ctx->slot, s.score_stride, ctx->seg_count, ctx->flags + 1,
                               ctx->filter_blocks[v.page.table ? 1 : 0], ctx->flags, true, ctx->nseg, st));
    LAUNCH(ctx, LFPS_KERNEL_FILTER_SELECT_ATTEND, st,
           launch_filter_select_attend(sd, ctx->cfg.kv_dtype, ctx->score, ctx->slot, s.score_stride, ctx->seg_count,
                                       ctx->flags + 1, ctx->nseg, nullptr, ctx->x_cnt, ctx->x_start, x_total, k, topk_idx,
                                       topk_score ? topk_score : ctx->sel_score, ctx->thr_x, nullptr, nullptr, q,
                                       ctx->flags, v, nullptr, st));
    return LFPS_OK;
  }
  LAUNCH(ctx, LFPS_KERNEL_DENSE_SCORE, st,
         launch_group_score(s, ctx->cfg.kv_dtype, q, v, nullptr, nullptr, ctx->score, s.score_stride, ctx->flags, st));
  LAUNCH(ctx, LFPS_KERNEL_SELECT, st,
         launch_select(s, ctx->score, s.score_stride, nullptr, v.seq_lens, k, topk_idx, topk_score, nullptr, nullptr,
                       nullptr, st));
  return LFPS_OK;
}

// ---------------------------------------------------------------------------- score tables
static int need_tables(lfps_ctx* ctx, const char* who, bool ready) {
  if (!ctx->tab_ver) {
    snprintf(ctx->err, sizeof ctx->err, "%s: the context was created without table_mode", who);
    return LFPS_EINVAL;
  }
  if (ready && !ctx->tab_ready) {
    snprintf(ctx->err, sizeof ctx->err, "%s: the tables hold nothing yet (lfps_tables_init or lfps_tables_import first)", who);
    return LFPS_EINVAL;
  }
  return LFPS_OK;
}

int lfps_tables_init(lfps_ctx* ctx, const float* q_hist, int32_t n_queries, const lfps_kv* kv, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!q_hist) return fail(ctx, LFPS_EINVAL, "lfps_tables_init: NULL argument");
  if (n_queries < 1) return fail(ctx, LFPS_EINVAL, "lfps_tables_init: n_queries must be >= 1");
  int rc = need_tables(ctx, "lfps_tables_init", false);
  if (rc != LFPS_OK) return rc;
  KvView v;
  rc = check_kv(ctx, kv, false, &v);
  if (rc != LFPS_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  const Shape& s = ctx->shape;
  const int64_t q_stride = (int64_t)s.B * s.Hq * kD;
  for (int j = 1; j <= n_queries; ++j) {
    LAUNCH(ctx, LFPS_KERNEL_DENSE_SCORE, st,
           launch_group_score(s, ctx->cfg.kv_dtype, q_hist + (int64_t)(j - 1) * q_stride, v, nullptr, nullptr, ctx->score,
                              s.score_stride, ctx->flags, st));
    hipError_t e = launch_table_init(s, ctx->tab_ver, ctx->tab_sla, v.seq_lens, ctx->score, s.score_stride,
                                     (double)ctx->cfg.table_decay, j, n_queries, st);
    if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_tables_init", e);
  }
  hipError_t e = launch_table_finish(s, ctx->tab_ver, ctx->tab_sla, ctx->tab_state, v.seq_lens, st);
  if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_tables_init (statistics)", e);
  ctx->tab_updates = 0;
  ctx->tab_ready = 1;
  return LFPS_OK;
}

int lfps_tables_import(lfps_ctx* ctx, const float* phi_ver, const float* phi_sla, const int32_t* seq_lens,
                       void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!phi_ver || !phi_sla || !seq_lens) return fail(ctx, LFPS_EINVAL, "lfps_tables_import: NULL argument");
  int rc = need_tables(ctx, "lfps_tables_import", false);
  if (rc != LFPS_OK) return rc;
  hipError_t e = launch_table_import(ctx->shape, ctx->tab_ver, ctx->tab_sla, ctx->tab_state, seq_lens, phi_ver,
                                     phi_sla, (hipStream_t)stream);
  if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_tables_import", e);
  ctx->tab_updates = 0;
  ctx->tab_ready = 1;
  return LFPS_OK;
}

int lfps_tables_export(lfps_ctx* ctx, double* phi_ver, double* phi_sla, const int32_t* seq_lens, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!phi_ver || !phi_sla || !seq_lens) return fail(ctx, LFPS_EINVAL, "lfps_tables_export: NULL argument");
  int rc = need_tables(ctx, "lfps_tables_export", true);
  if (rc != LFPS_OK) return rc;
  hipError_t e = launch_table_export(ctx->shape, ctx->tab_ver, ctx->tab_sla, ctx->tab_state, seq_lens, phi_ver,
                                     phi_sla, (hipStream_t)stream);
  if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_tables_export", e);
  return LFPS_OK;
}

static int table_candidates_impl(lfps_ctx* ctx, const int32_t* seq_lens, int32_t* cand, int32_t* cand_count,
                                 bool for_step, const int32_t* gate, hipStream_t st) {
  const Shape& s = ctx->shape;
  LAUNCH(ctx, LFPS_KERNEL_TABLE_FLAGS, st,
         launch_table_flags(s, ctx->tab_ver, ctx->tab_sla, ctx->tab_state, seq_lens, ctx->tab_f0, ctx->tab_fm,
                            ctx->flag_words, (double)ctx->cfg.table_a, gate, st));
  LAUNCH(ctx, LFPS_KERNEL_TABLE_CANDIDATES, st,
         launch_table_candidates(s, ctx->tab_f0, ctx->tab_fm, ctx->flag_words, seq_lens, cand, cand_count, ctx->flags,
                                 for_step && next_step_filtered(ctx) ? ctx->group_start : nullptr,
                                 ctx->group_start + (int64_t)s.B * s.Hkv, st));
  return LFPS_OK;
}

static int table_update_impl(lfps_ctx* ctx, const int32_t* idx, const float* idx_score, const int32_t* k,
                             const int32_t* seq_lens, const int32_t* gate, bool distinct, hipStream_t st) {
  const Shape& s = ctx->shape;
  if (ctx->tab_updates >= s.Lcap - 1)
    return fail(ctx, LFPS_ECAP, "lfps_table_update: max_seq_len - 1 updates since the last import/init");
  LAUNCH(ctx, LFPS_KERNEL_TABLE_UPDATE, st,
         launch_table_update(s, ctx->tab_ver, ctx->tab_sla, ctx->tab_state, seq_lens, idx, idx_score, k,
                             (double)ctx->cfg.table_decay, gate, ctx->flags, distinct, st));
  ctx->tab_updates += 1;
  return LFPS_OK;
}

int lfps_table_candidates(lfps_ctx* ctx, const int32_t* seq_lens, int32_t* cand, int32_t* cand_count, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!seq_lens || !cand || !cand_count) return fail(ctx, LFPS_EINVAL, "lfps_table_candidates: NULL argument");
  int rc = need_tables(ctx, "lfps_table_candidates", true);
  if (rc != LFPS_OK) return rc;
  return table_candidates_impl(ctx, seq_lens, cand, cand_count, false, nullptr, (hipStream_t)stream);
}

int lfps_table_update(lfps_ctx* ctx, const int32_t* idx, const float* idx_score, const int32_t* k,
                      const int32_t* seq_lens, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!idx || !idx_score || !k || !seq_lens) return fail(ctx, LFPS_EINVAL, "lfps_table_update: NULL argument");
  int rc = need_tables(ctx, "lfps_table_update", true);
  if (rc != LFPS_OK) return rc;
  return table_update_impl(ctx, idx, idx_score, k, seq_lens, nullptr, false, (hipStream_t)stream);   // a caller's list
}

static int table_step_impl(lfps_ctx* ctx, const float* q, const KvView& v, const int32_t* k, int32_t* topk_idx,
                           float* topk_score, float* out, const int32_t* gate, hipStream_t st) {
  const Shape& s = ctx->shape;
  float* sel = topk_score ? topk_score : ctx->sel_score;
  int rc = table_candidates_impl(ctx, v.seq_lens, ctx->cand, ctx->cand_count, true, gate, st);
  if (rc != LFPS_OK) return rc;
  rc = score_select_attend(ctx, q, v, k, topk_idx, sel, out, gate, st);
  if (rc != LFPS_OK) return rc;
  return table_update_impl(ctx, topk_idx, sel, k, v.seq_lens, gate, true, st);   // the select's rows are distinct
}

int lfps_table_step(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const int32_t* k, int32_t* topk_idx,
                    float* topk_score, float* out, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!q || !k || !topk_idx || !out) return fail(ctx, LFPS_EINVAL, "lfps_table_step: NULL argument");
  int rc = need_tables(ctx, "lfps_table_step", true);
  if (rc != LFPS_OK) return rc;
  KvView v;
  rc = check_kv(ctx, kv, true, &v);
  if (rc != LFPS_OK) return rc;
  return table_step_impl(ctx, q, v, k, topk_idx, topk_score, out, nullptr, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------- head sparsity bypass
int lfps_priors(lfps_ctx* ctx, const float* q, const lfps_kv* kv, float* kbar, float* vbar, float* sigma2_hat,
                void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!q || !kbar || !vbar || !sigma2_hat) return fail(ctx, LFPS_EINVAL, "lfps_priors: NULL argument");
  KvView v;
  int rc = check_kv(ctx, kv, true, &v);
  if (rc != LFPS_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  const Shape& s = ctx->shape;
  hipError_t e = launch_prior_means(s, ctx->cfg.kv_dtype, v, kbar, vbar, st);
  if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_priors (means)", e);
  LAUNCH(ctx, LFPS_KERNEL_DENSE_SCORE, st,
         launch_group_score(s, ctx->cfg.kv_dtype, q, v, nullptr, nullptr, ctx->score, s.score_stride, ctx->flags, st));
  e = launch_prior_variance(s, q, v.seq_lens, ctx->score, s.score_stride, sigma2_hat, st);
  if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_priors (variance)", e);
  return LFPS_OK;
}

int lfps_head_sparsity(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const float* kbar, const float* sigma2_hat,
                       int32_t n_local, float eps, float* rho, int32_t* gate, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!q || !kbar || !sigma2_hat || !gate) return fail(ctx, LFPS_EINVAL, "lfps_head_sparsity: NULL argument");
  if (n_local < 0) return fail(ctx, LFPS_EINVAL, "lfps_head_sparsity: n_local must be >= 0");
  KvView v;
  int rc = check_kv(ctx, kv, false, &v);
  if (rc != LFPS_OK) return rc;
  hipError_t e = launch_head_sparsity(ctx->shape, ctx->cfg.kv_dtype, q, v, kbar, sigma2_hat, n_local, eps, rho, gate,
                                      nullptr, nullptr, nullptr, nullptr, nullptr, (hipStream_t)stream);
  if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_head_sparsity", e);
  return LFPS_OK;
}

int lfps_table_step_gated(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const int32_t* k, const float* kbar,
                          const float* vbar, const float* sigma2_hat, int32_t n_local, float eps, int32_t* topk_idx,
                          float* topk_score, float* out, int32_t* gate_out, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!q || !k || !kbar || !vbar || !sigma2_hat || !topk_idx || !out)
    return fail(ctx, LFPS_EINVAL, "lfps_table_step_gated: NULL argument");
  if (n_local < 0) return fail(ctx, LFPS_EINVAL, "lfps_table_step_gated: n_local must be >= 0");
  int rc = need_tables(ctx, "lfps_table_step_gated", true);
  if (rc != LFPS_OK) return rc;
  KvView v;
  rc = check_kv(ctx, kv, true, &v);
  if (rc != LFPS_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  int32_t* gate = gate_out ? gate_out : ctx->gate;
  hipError_t e = launch_head_sparsity(ctx->shape, ctx->cfg.kv_dtype, q, v, kbar, sigma2_hat, n_local, eps, nullptr,
                                      gate, vbar, topk_idx, topk_score, out, ctx->filter_on ? ctx->thr_state : nullptr, st);
  if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_table_step_gated (gate)", e);
  return table_step_impl(ctx, q, v, k, topk_idx, topk_score, out, gate, st);
}

__global__ void k_fill_f32(float* p, int n, float v) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

int lfps_set_filter(lfps_ctx* ctx, int32_t on) {
  if (!ctx) return LFPS_EINVAL;
  ctx->filter_on = (on && ctx->slot) ? 1 : 0;
  return LFPS_OK;
}

int lfps_reset_history(lfps_ctx* ctx, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  const int n = ctx->shape.B * ctx->shape.Hq;
  hipLaunchKernelGGL(k_fill_f32, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, ctx->thr_state, n,
                     __builtin_nanf(""));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_reset_history", e);
  ctx->no_history = 1;
  return LFPS_OK;
}

int lfps_copy_cand_count(lfps_ctx* ctx, int32_t* dst, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!dst) return fail(ctx, LFPS_EINVAL, "lfps_copy_cand_count: NULL argument");
  hipError_t e = hipMemcpyAsync(dst, ctx->cand_count, (size_t)ctx->shape.B * ctx->shape.Hkv * 4,
                                hipMemcpyDeviceToDevice, (hipStream_t)stream);
  if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_copy_cand_count", e);
  return LFPS_OK;
}

int lfps_poll_status(lfps_ctx* ctx, int32_t* flags, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!flags) return fail(ctx, LFPS_EINVAL, "lfps_poll_status: NULL argument");
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = hipMemcpyAsync(flags, ctx->flags, 4, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipMemsetAsync(ctx->flags, 0, 4, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_poll_status", e);
  return LFPS_OK;
}

int lfps_poll_rescored(lfps_ctx* ctx, int32_t* n_heads, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!n_heads) return fail(ctx, LFPS_EINVAL, "lfps_poll_rescored: NULL argument");
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = hipMemcpyAsync(n_heads, ctx->flags + 2, 4, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipMemsetAsync(ctx->flags + 2, 0, 4, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_poll_rescored", e);
  return LFPS_OK;
}

int lfps_timing_enable(lfps_ctx* ctx, int32_t on) {
  if (!ctx) return LFPS_EINVAL;
  if (on && ctx->events_made == 0) {
    for (int i = 0; i < LFPS_TIMING_MAX_LAUNCHES; ++i) {
      hipError_t e = hipEventCreate(&ctx->ev[i][0]);
      if (e == hipSuccess) e = hipEventCreate(&ctx->ev[i][1]);
      if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "hipEventCreate", e);
      ctx->events_made = i + 1;
    }
  }
  ctx->timing_on = on ? 1 : 0;
  return LFPS_OK;
}

int lfps_timing_read(lfps_ctx* ctx, float* ms, int32_t* launches, void* stream) {
  if (!ctx) return LFPS_EINVAL;
  if (!ms || !launches) return fail(ctx, LFPS_EINVAL, "lfps_timing_read: NULL argument");
  hipError_t e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "lfps_timing_read", e);
  for (int i = 0; i < LFPS_N_KERNELS; ++i) {
    ms[i] = 0.f;
    launches[i] = 0;
  }
  for (int i = 0; i < ctx->n_timed; ++i) {
    float t = 0.f;
    e = hipEventElapsedTime(&t, ctx->ev[i][0], ctx->ev[i][1]);
    if (e != hipSuccess) return fail(ctx, LFPS_EHIP, "hipEventElapsedTime", e);
    ms[ctx->ev_slot[i]] += t;
    launches[ctx->ev_slot[i]] += 1;
  }
  ctx->n_timed = 0;
  return LFPS_OK;
}

}  // extern "C"
