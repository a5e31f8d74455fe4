/*
 * liblfps — the decode-step hot path of LFPS ("Learn from the Past: Fast Sparse Indexing
 * for LLM Decoding") as hand-written HIP kernels for gfx950 (MI355X), behind a C ABI.
 *
 * One decode step of one attention layer, for B requests in GQA form (Hq query heads,
 * Hkv KV heads, G = Hq/Hkv heads per group, head_dim D = 128), with the KV cache resident
 * in device memory:
 *
 *   S1  candidates   previous step's per-head Top-k  ->  sorted candidate positions per KV group
 *   S2  score        q . K_j / sqrt(D) for candidate rows only (all G heads of the group)
 *   S3  select       per query head, the k best candidates  ->  Top-k index set of this step
 *   S4  sparse attn  Softmax over the selected scores, weighted sum of the selected V rows
 *
 * plus two baselines over the whole context: full attention and exact Top-k.
 *
 * Conventions
 *   - Every function returns an int status: LFPS_OK (0) or a negative lfps_status.  Nothing
 *     throws, exits, or synchronises the host (except lfps_create/destroy, lfps_timing_read and
 *     lfps_poll_status, which say so).  After lfps_create no entry point allocates memory.
 *   - All array arguments are DEVICE pointers owned by the caller, unless marked "host".
 *     The context owns only its workspace (candidate scores, split partials, event pool).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued asynchronously on it, in order.  Use one context per stream at a time.
 *   - Entry points that only enqueue kernels (the S1..S4 calls, lfps_step, the lfps_table_* steps, the
 *     baselines) keep all their state in device memory and may be recorded into a HIP graph; the ones that
 *     synchronise, copy to the host or read events (create/destroy, poll_status, timing_read) may not.
 *   - Positions and counts are int32.  A negative entry in an index array is padding.
 *   - q is fp32 [B, Hq, D].  With an fp16 cache every |q| element must stay below 65504, the fp16 range: an
 *     element beyond it is clamped to +-65504 by the scoring kernels (the scores stay finite but belong to the
 *     clamped query) and LFPS_FLAG_Q_RANGE is raised.
 *     K and V rows are D contiguous elements (bf16, fp16 or fp32); the view
 *     struct gives the element strides between requests, KV heads and rows.
 *   - Argument errors that the host can see (NULL pointers, bad shapes/strides) return
 *     LFPS_EINVAL before anything is launched.  Values that live in device memory (k, seq_lens,
 *     indices) are clamped by the kernels: k_b to [0, max_k], seq_lens to [0, max_seq_len],
 *     index entries outside [0, n_b) are ignored.
 */
#ifndef LFPS_H
#define LFPS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
#pragma GCC visibility push(default) /* the declarations below are the library's whole export list */

typedef struct lfps_ctx lfps_ctx;

typedef enum {
  LFPS_OK = 0,
  LFPS_EINVAL = -1, /* NULL pointer, unsupported shape/dtype, bad stride */
  LFPS_ECAP = -2,   /* a capacity in lfps_config cannot be met (LDS bitmap, workspace) */
  LFPS_EHIP = -3,   /* HIP runtime error; text via lfps_last_error */
  LFPS_ENOMEM = -4  /* workspace allocation failed in lfps_create */
} lfps_status;

typedef enum { LFPS_F32 = 0, LFPS_BF16 = 1, LFPS_F16 = 2 } lfps_dtype;   /* fp32, bfloat16, IEEE half */

typedef struct {
  int32_t batch;       /* B >= 1; B * Hq <= 65535 */
  int32_t n_q_heads;   /* Hq, a multiple of n_kv_heads; Hq/Hkv must be 1, 2 or 4 */
  int32_t n_kv_heads;  /* Hkv */
  int32_t head_dim;    /* D, must be 128 */
  int32_t kv_dtype;    /* lfps_dtype of the K/V cache */
  int32_t max_seq_len; /* Lcap: rows allocated per (request, KV head); n_b <= Lcap always */
  int32_t max_k;       /* kmax: row length of every Top-k array; k_b <= kmax */
  int32_t radius;      /* r >= 0: positional expansion radius around each predicted position */
  int32_t n_recent;    /* the newest n_recent rows are always candidates (>= 0) */
  int32_t n_sink;      /* the first n_sink rows are always candidates (>= 0) */
  int32_t cand_cap;    /* row length of candidate arrays; 0 = min(Lcap, G*kmax*(2r+2)+n_recent+n_sink), or Lcap in table mode */
  int32_t device;      /* HIP device ordinal */
  int32_t table_mode;  /* 1: also allocate the per-head score tables used by the lfps_table_* entry points */
  float table_decay;   /* gamma of Eq. 10 (the paper's decay factor r = 0.95); table mode needs 0 < gamma < 1 */
  float table_a;       /* a of Eq. 8 (0.2 / 0.3 in the paper); table mode needs a > 0 */
  int32_t k_fp8;       /* 1: K is stored as OCP FP8 E4M3, one byte per element (needs kv_dtype = LFPS_BF16, which then
                          describes V).  The values are used as they are; a dequantisation scale is the caller's to
                          fold into q. */
  int32_t v_fp8;       /* 1: V is stored as OCP FP8 E4M3 as well (needs kv_dtype = LFPS_BF16; a scale of V is a factor
                          on the output rows and the caller's to apply) */
} lfps_config;

/* View of the KV cache.  The struct itself is host memory; k, v, seq_lens and block_table are device
 * pointers.  seq_lens[b] = n_b, the number of valid rows of request b at this step.
 *
 * Contiguous cache (block_table == NULL): element (b, g, i, c) of K is
 *   k[b*stride_b + g*stride_h + i*stride_n + c]
 * (strides in elements, stride_n >= D, rows 16-byte aligned), same for v.  K and V share the element
 * strides also when only one of them is FP8 (cfg.k_fp8, cfg.v_fp8): an FP8 element is one byte.
 *
 * Paged cache (block_table != NULL): k and v are pools of n_blocks blocks of block_size rows, and
 * block_table[b*block_table_stride + i/block_size] names the block that holds row i of request b:
 *   k[block*stride_b + g*stride_h + (i % block_size)*stride_n + c]
 * so stride_b is the distance between blocks.  block_size is a power of two in [1, 65536];
 * block_table_stride*block_size >= max_seq_len; n_blocks*block_size < 2^31.  Table entries are
 * read by the kernels and clamped into [0, n_blocks); only the entries of rows below n_b are read,
 * and the first entry of every request (padding slots read row 0, also when n_b = 0).
 * The method itself (positions, candidates, Top-k indices) always speaks in logical rows i. */
/* Host-resident cache (the paper's placement, Sec. 4 overview: the KV cache in host memory): k and v may also
 * point to pinned host memory that the device can address (hipHostMalloc; pass what lfps_host_device_pointer
 * returns for it).  Every kernel then fetches exactly the rows it touches over the host link: the candidate rows
 * of K once per KV group, the selected rows of V per head; nothing else changes, results are bit-identical to a
 * device-resident cache.  seq_lens and block_table stay in device memory. */
typedef struct {
  const void* k;
  const void* v;
  int64_t stride_b, stride_h, stride_n;
  const int32_t* seq_lens; /* [B] */
  const int32_t* block_table; /* [B, block_table_stride] or NULL */
  int32_t block_size;
  int32_t block_table_stride;
  int32_t n_blocks;
} lfps_kv;

/* The address at which the current device sees a pinned host allocation (hipHostMalloc'ed memory, e.g. a pinned
 * torch tensor): host in, *dev out.  LFPS_EHIP if the memory is not mapped for the device. */
int lfps_host_device_pointer(const void* host, void** dev);

/* Create / destroy.  lfps_create validates the config, selects cfg->device, allocates the
 * workspace (lfps_workspace_bytes) and synchronises the device once.  *out is NULL on error. */
int lfps_create(const lfps_config* cfg, lfps_ctx** out);
int lfps_destroy(lfps_ctx* ctx);
/* Text of the last error on this context (host string owned by the context; "" if none).
 * With ctx == NULL: text of the last failure of a call that takes no context (lfps_create,
 * lfps_workspace_bytes, lfps_sparse_attn_noalloc) in this thread. */
const char* lfps_last_error(const lfps_ctx* ctx);
/* Device bytes lfps_create will allocate for this config (host out-pointer). */
int lfps_workspace_bytes(const lfps_config* cfg, int64_t* out);
/* The candidate row length in effect (cfg.cand_cap or its default). */
int32_t lfps_cand_cap(const lfps_ctx* ctx);

/* S1 — candidate set (Alg. 1 lines 6-7; Eq. 7 and Eq. 9 in their memoryless form).
 * For every (b, g):  C = clip_[0,n_b)( U_{h in g} U_{i in prev_topk[b,h,0:k_b]} {i-r, ..., i+r+1} )
 *                        U {n_b - n_recent, ..., n_b - 1} U {0, ..., n_sink - 1}
 * i.e. the previous Top-k itself (vertical pattern), the same positions shifted by +1 (slash
 * pattern, the direction Eq. 10 moves slash history), each widened by +-r (at r = 1 the offsets
 * are the {-1,0,1,2} of Sec. 4.2 stage 3).  Output is ascending and duplicate-free, hence
 * bit-reproducible.
 *   prev_topk  [B, Hq, kmax] int32, first k_b entries of a row are used, entries outside [0,n_b) ignored
 *   k          [B] int32;  seq_lens [B] int32
 *   cand       [B, Hkv, cand_cap] int32 out (entries past cand_count are left untouched)
 *   cand_count [B, Hkv] int32 out.  If a set would exceed cand_cap it is truncated to its
 *              cand_cap smallest positions and LFPS_FLAG_CAND_OVERFLOW is raised (lfps_poll_status). */
int lfps_candidates(lfps_ctx* ctx, const int32_t* prev_topk, const int32_t* k, const int32_t* seq_lens,
                    int32_t* cand, int32_t* cand_count, void* stream);

/* S2 + S3 — exact dot products over the candidates only, then the k best per query head
 * (Alg. 1 line 8; Sec. 1 Steps 1-2 restricted to the candidate set).
 * score(b,h,j) = q[b,h] . K[b,g(h),cand[b,g,j]] / sqrt(D), fp32 accumulate.
 *   cand, cand_count  as produced by lfps_candidates (ascending positions in [0, n_b)).  An entry outside
 *              [0, n_b) scores -inf: it is taken only when fewer than k_b valid candidates exist, and then
 *              written as -1 (score 0) where it would stand.
 *   topk_idx   [B, Hq, kmax] int32 out: the min(k_b, c) selected positions, ascending; rest -1.
 *              Equal scores at the cut are resolved towards the lower position.
 *   topk_score [B, Hq, kmax] fp32 out or NULL: the score of each selected position (0 for padding)
 *   cand_score [B, Hq, cand_cap] fp32 out or NULL: every candidate's score (parity/debug dump) */
int lfps_score_topk(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const int32_t* cand,
                    const int32_t* cand_count, const int32_t* k, int32_t* topk_idx, float* topk_score,
                    float* cand_score, void* stream);

/* S4 — sparse attention output (Eq. 1):  out[b,h] = sum_i softmax_i(s_i) V[b,g(h),i],  i in idx[b,h,0:k_b],
 * s_i = q.K_i/sqrt(D).  Negative entries and entries >= n_b are skipped.
 *   idx       [B, Hq, kmax] int32
 *   idx_score [B, Hq, kmax] fp32 scores of those positions, or NULL to recompute q.K from the cache
 *   out       [B, Hq, D] fp32 (zeros for a head with no valid index) */
int lfps_sparse_attn(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const int32_t* idx,
                     const float* idx_score, const int32_t* k, float* out, void* stream);

/* S4 for callers that cannot allocate device memory (code recorded into a HIP graph, serving loops and harnesses
 * that forbid hipMalloc): the same result as lfps_sparse_attn(ctx, q, kv, idx, NULL, k, out) without a context.
 * Nothing is allocated, by this call or before it: the scores of the selected rows, which lfps_sparse_attn keeps in
 * its context's workspace between its two kernels, go to a static device array of LFPS_NOALLOC_MAX_SCORES floats
 * (8 MiB, held by every GPU the library runs on until the process ends).
 *   cfg   the shapes and cache format as for lfps_create (batch, heads, head_dim, kv_dtype, k_fp8 / v_fp8,
 *         max_seq_len, max_k; the other fields must be valid but are not used); cfg->device must be the
 *         CURRENT device.  batch * n_q_heads * max_k must not exceed LFPS_NOALLOC_MAX_SCORES: LFPS_ECAP otherwise.
 *   q [B, Hq, D], idx [B, Hq, kmax], k [B], out [B, Hq, D]: device pointers owned by the caller, as for
 *         lfps_sparse_attn.
 * Errors are returned as lfps_status; their text is lfps_last_error(NULL) in the calling thread.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (different streams or
 * threads) race on it.  The array keeps the previous call's scores; nothing in it needs clearing (every entry
 * that is read has been written by the same call).  The first call on a device looks the array's address up
 * (hipGetSymbolAddress), so make that call outside stream capture. */
#define LFPS_NOALLOC_MAX_SCORES 2097152
int lfps_sparse_attn_noalloc(const lfps_config* cfg, const float* q, const lfps_kv* kv, const int32_t* idx,
                             const int32_t* k, float* out, void* stream);

/* S1..S4 in one call (Alg. 1 lines 6-8 and 10, then Eq. 1): candidates from prev_topk, score,
 * select into topk_idx (this step's index set, the next step's prev_topk), attention into out.
 * S4 reuses S3's scores, so only V rows are gathered.  prev_topk and topk_idx must not overlap.
 *   topk_score [B, Hq, kmax] fp32 out or NULL
 * With a bf16 or fp16 cache the scoring pass keeps, per head, only rows whose score reaches the k-th best
 * score of the PREVIOUS lfps_step call on this context minus a margin (the context remembers one
 * float per head); a head for which that leaves fewer than k rows is rescored without the filter
 * in the same call (by that head's workgroup of the select kernel: no extra launches).  The result is therefore
 * the same exact Top-k over the candidates whatever the remembered value is; only the time differs.  The first
 * chained step after lfps_create or lfps_reset_history has nothing remembered and takes the unfiltered kernels; that
 * is decided on the host, so a HIP graph captured from such a call replays the unfiltered form: capture a later step.  (A context whose max_k exceeds ~13 000 starts with the
 * filter off: a head's survivors would not fit the select's on-chip list.)  lfps_set_filter(ctx, 0) turns the filter off,
 * lfps_reset_history forgets the remembered scores (e.g. when the context moves to other requests). */
int lfps_step(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const int32_t* prev_topk, const int32_t* k,
              int32_t* topk_idx, float* topk_score, float* out, void* stream);

/* Baseline: full attention decode, softmax(q K^T / sqrt(D)) V over all n_b rows
 * (Sec. 1 with idx = all; the "full attention" upper bound of Sec. 5).  out [B, Hq, D] fp32. */
int lfps_full_attn_decode(lfps_ctx* ctx, const float* q, const lfps_kv* kv, float* out, void* stream);

/* Baseline: exact Top-k, Sec. 1 Steps 1-2 over all n_b keys (the "exact Top-k" upper bound of
 * Sec. 5): scores every row, selects the k_b best per head.  Outputs as lfps_score_topk.
 * Also the seed of step 0 (the previous Top-k of the first LFPS step).
 * With a 16-bit or FP8-key cache of about a million rows or more (batch * n_kv_heads * max_seq_len) and the score
 * filter on, the scores are not written out and read back: a threshold per head is taken from a scored sample of
 * the rows, one filtered pass over all rows keeps what reaches it, and heads left short are rescored the plain
 * way, so the result is the same exact Top-k either way. */
int lfps_exact_topk(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const int32_t* k, int32_t* topk_idx,
                    float* topk_score, void* stream);

/* ---- LFPS with score tables: the paper's own candidate rule (Sec. 4.2, Alg. 1 lines 5-9) --------------
 * The context (created with table_mode = 1) keeps, per query head, a vertical and a slash score table over
 * positions.  Sink rows (< n_sink) are outside the tables, as in the paper: always candidates, never
 * counted or updated.  Radius must be <= 30.  Rows appended since the last update enter the tables as zeros. */

/* Eq. 4: tables from the attention weights of the last s = n_queries prefill queries.
 *   q_hist [n_queries, B, Hq, D] fp32, q_hist[j-1] = the j-th most recent query (j = 1: the last one).
 * Query j sees rows [0, n_b - j + 1); w = softmax over the offloaded rows it sees of q.K/sqrt(D);
 *   Phi_ver(i) = 1/(2 s (1 - gamma)) sum_j w_j(i),    Phi_sla(i) = 1/(2 s (1 - gamma)) sum_j w_j(i - j + 1)
 * (the paper uses s = 32).  One dense scoring pass per query. */
int lfps_tables_init(lfps_ctx* ctx, const float* q_hist, int32_t n_queries, const lfps_kv* kv, void* stream);
/* Set / read the tables as true values per position: phi_ver, phi_sla [B, Hq, max_seq_len], rows
 * [0, seq_lens[b]) used (fp32 in, fp64 out; entries of sink rows and rows >= n_b read as 0). */
int lfps_tables_import(lfps_ctx* ctx, const float* phi_ver, const float* phi_sla, const int32_t* seq_lens,
                       void* stream);
int lfps_tables_export(lfps_ctx* ctx, double* phi_ver, double* phi_sla, const int32_t* seq_lens, void* stream);
/* S1 in table form (Eq. 7, 8, 9): per head the positions whose vertical or slash score exceeds
 * tau = a * mean / kappa of its table, widened by the offsets -r ... r+1 and kept where the vertical or the
 * slash score exceeds the table mean; union over the heads of a KV group, plus the newest n_recent and
 * the n_sink first rows.  Outputs as lfps_candidates. */
int lfps_table_candidates(lfps_ctx* ctx, const int32_t* seq_lens, int32_t* cand, int32_t* cand_count, void* stream);
/* Eq. 10: decay by gamma, slash history moved from i-1 to i, and on the selected positions
 * idx[b,h,0:k_b] (scaled scores idx_score) the softmax weight over the selected set minus 1/(2|C_2|).
 * seq_lens is the length the step saw.  The slash table has room for max_seq_len - 1 updates after an
 * import or init: the call that would exceed it returns LFPS_ECAP, and (for updates replayed from a
 * recorded graph, which the host does not see) the kernel leaves the tables alone and raises
 * LFPS_FLAG_TABLE_FULL.  The table calls keep their state in device memory and may be recorded into a graph. */
int lfps_table_update(lfps_ctx* ctx, const int32_t* idx, const float* idx_score, const int32_t* k,
                      const int32_t* seq_lens, void* stream);
/* Alg. 1 lines 5-9 then Eq. 1: table candidates, exact scores over them, per-head Top-k (fewer than k_b
 * when the candidate set is smaller: padded with -1), sparse attention, table update. */
int lfps_table_step(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const int32_t* k, int32_t* topk_idx,
                    float* topk_score, float* out, void* stream);

/* ---- Head sparsity estimate and bypass (Sec. 4.2 stage 1, Eq. 5-6, App. B.1; Alg. 1 lines 1-4) ------------
 * Priors of the prefill stage (Sec. 4.2 "Prefilling", last paragraph), from the last prefill query q:
 *   kbar, vbar  [B, Hkv, D] fp32  mean K row / V row over rows [n_sink, n_b)
 *   sigma2_hat  [B, Hq]     fp32  variance over those rows of q.K_i/sqrt(D), divided by |q|^2 */
int lfps_priors(lfps_ctx* ctx, const float* q, const lfps_kv* kv, float* kbar, float* vbar, float* sigma2_hat,
                void* stream);
/* rho[b,h] = w_sink / (w_sink + w_global + w_local)  (Eq. 6) with
 *   w_sink = sum_{i < n_sink} exp(q.K_i/sqrt(D)),  w_local = the same sum over the newest n_local rows (the paper: 6),
 *   w_global = n_b * exp(q.kbar/sqrt(D) + |q|^2 sigma2_hat / 2);   gate[b,h] = rho > eps (the paper: 0.85).
 * rho [B, Hq] fp32 or NULL; gate [B, Hq] int32. */
int lfps_head_sparsity(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const float* kbar, const float* sigma2_hat,
                       int32_t n_local, float eps, float* rho, int32_t* gate, void* stream);
/* lfps_table_step with the bypass in front (Alg. 1 in full): a head with rho > eps outputs vbar[b, g(h)],
 * selects nothing (its topk_idx row is -1), proposes no candidates and keeps its tables as they are.
 * gate_out [B, Hq] int32 or NULL receives the marks. */
int lfps_table_step_gated(lfps_ctx* ctx, const float* q, const lfps_kv* kv, const int32_t* k, const float* kbar,
                          const float* vbar, const float* sigma2_hat, int32_t n_local, float eps, int32_t* topk_idx,
                          float* topk_score, float* out, int32_t* gate_out, void* stream);

/* Switches the score filter of the chained steps on or off (on: only for caches it exists for, bf16 / fp16 / FP8
 * keys; a no-op otherwise).  lfps_reset_history makes every head start without a remembered score. */
int lfps_set_filter(lfps_ctx* ctx, int32_t on);
int lfps_reset_history(lfps_ctx* ctx, void* stream);
/* Copies the candidate counts [B, Hkv] of the last lfps_step call into dst (device, int32),
 * asynchronously on `stream` (for benchmarks: bytes moved per step). */
int lfps_copy_cand_count(lfps_ctx* ctx, int32_t* dst, void* stream);

/* Status flags raised by kernels since the last poll.  Synchronises `stream`, copies the flag
 * word to *flags (host) and clears it. */
#define LFPS_FLAG_CAND_OVERFLOW 1
#define LFPS_FLAG_TABLE_FULL 2      /* a table update was skipped: max_seq_len - 1 updates since the last import / init */
#define LFPS_FLAG_Q_RANGE 4         /* fp16 cache: a query element beyond +-65504 was clamped to the fp16 range by a
                                       scoring kernel (the scores of that head are those of the clamped query) */
int lfps_poll_status(lfps_ctx* ctx, int32_t* flags, void* stream);
/* Heads that the filtered scoring pass of lfps_step / lfps_table_step left with fewer than k rows (or more than the
 * select's list holds) and that were therefore rescored without the filter, since the last call (host out-pointer;
 * synchronises `stream` and clears the count).  Results do not depend on it: it tells how often the remembered
 * k-th score was of no use (first step after a reset, a sudden change of the query). */
int lfps_poll_rescored(lfps_ctx* ctx, int32_t* n_heads, void* stream);

/* Per-kernel timing for benchmarks.  While enabled, every kernel launch is bracketed by HIP
 * events on the launch stream (at most LFPS_TIMING_MAX_LAUNCHES launches between reads; later
 * ones go untimed).  lfps_timing_read synchronises the stream and writes, for kernel slot i,
 * the summed milliseconds to ms[i] and the number of timed launches to launches[i] (host
 * arrays of LFPS_N_KERNELS), then resets the accumulators. */
enum {
  LFPS_KERNEL_CANDIDATES = 0,
  LFPS_KERNEL_GATHER_SCORE = 1,
  LFPS_KERNEL_SELECT = 2,
  LFPS_KERNEL_SPARSE_ATTN = 3,
  LFPS_KERNEL_DENSE_SCORE = 4,
  LFPS_KERNEL_FULL_ATTN = 5,
  LFPS_KERNEL_FULL_MERGE = 6,
  LFPS_KERNEL_HEAD_SCORE = 7,
  LFPS_KERNEL_FILTER_SCORE = 8,
  LFPS_KERNEL_FILTER_SELECT = 9,
  LFPS_KERNEL_TABLE_FLAGS = 10,
  LFPS_KERNEL_TABLE_CANDIDATES = 11,
  LFPS_KERNEL_TABLE_UPDATE = 12,
  LFPS_KERNEL_FILTER_SELECT_ATTEND = 13,   /* S3 + S4 from the filtered pass's survivor lists (chained steps) */
  LFPS_KERNEL_SELECT_ATTEND = 14,          /* S3 + S4 from full score rows (heads the filter left short; unfiltered contexts) */
  LFPS_N_KERNELS = 15
};
#define LFPS_TIMING_MAX_LAUNCHES 4096
int lfps_timing_enable(lfps_ctx* ctx, int32_t on);
int lfps_timing_read(lfps_ctx* ctx, float* ms, int32_t* launches, void* stream);
const char* lfps_kernel_name(int32_t slot);

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers 16-byte aligned),
 * one 16-byte load and store per lane, grid-strided.  Not part of the method: it exists so that
 * hardware memory counters (bytes fetched / written per dispatch) can be scaled against a kernel
 * whose traffic is known exactly. */
int lfps_calib_copy(void* dst, const void* src, int64_t bytes, void* stream);

#pragma GCC visibility pop
#ifdef __cplusplus
}
#endif
#endif /* LFPS_H */
