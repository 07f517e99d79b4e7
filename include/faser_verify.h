/*
 * faser_verify -- target-side verification step of speculative decoding over a continuous
 * batch in which every request carries its own speculative length (FASER, arXiv
 * 2604.20503, Sec. 3.1), as hand-written HIP kernels for gfx950 (MI355X).
 *
 * One verification step is
 *     fsr_verify_attention  (once per transformer layer)
 *  -> fsr_spec_accept       (on the step's target / draft distributions)
 *  -> fsr_prune_compact     (drop rejected rows, re-pack the ragged batch)
 * and, for frontier (chunked) verification (Sec. 3.3), fsr_frontier_plan /
 * fsr_frontier_commit carry the per-request state from one chunk to the next without a
 * host round trip.
 *
 * Conventions for every entry point
 *   - Returns 0 (FSR_OK) or a negative FSR_E* code; fsr_last_error() gives a static,
 *     thread-local description of the last failure.  Nothing throws or aborts.
 *   - Every pointer argument is DEVICE memory owned by the caller unless its comment says
 *     "host".  The library reads the inputs and writes only the named outputs and the
 *     workspace.  Nothing is allocated or freed by these calls.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream).  No call synchronises the stream or the device.  Calls on one stream may
 *     share a workspace; calls that can overlap in time (different streams, or graphs replayed
 *     on different streams) must not: at most one call may be in flight per workspace.  (The
 *     attention kernel tags what it leaves there with the call's id: a slot written by another
 *     call turns the affected output rows into NaN instead of being summed silently.)
 *   - Ragged metadata (lengths, offsets, masks) lives on the device; the only host scalars
 *     are static shapes and capacities.  Host-detectable errors (null pointers, bad
 *     shapes, unsupported dtype/head_dim, workspace too small) are reported before
 *     anything is launched.
 *   - Ragged layout: request i owns rows cu[i] .. cu[i+1]-1 of the row-major arrays; a
 *     request with zero rows is legal everywhere and costs nothing.
 */
#ifndef FASER_VERIFY_H
#define FASER_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FSR_OK 0
#define FSR_EINVAL (-1) /* null pointer or out-of-range scalar argument */
#define FSR_ESHAPE (-2) /* inconsistent sizes */
#define FSR_EUNSUP (-3) /* dtype / head_dim / page size combination not built */
#define FSR_EWS (-4)    /* workspace missing or too small */
#define FSR_EHIP (-5)   /* HIP runtime error at launch */

enum { FSR_F32 = 0, FSR_BF16 = 1 };
enum { FSR_PROBS = 0, FSR_LOGITS = 1, FSR_GREEDY = 2 };
/* layout of a KV cache page: [H_kv][P][D] (one contiguous block per head) or [P][H_kv][D] (one per token) */
enum { FSR_KV_HEAD_MAJOR = 0, FSR_KV_TOKEN_MAJOR = 1 };

/* Static shape of one attention call. */
typedef struct fsr_attn_params {
    int32_t B;         /* requests in the batch (>= 0) */
    int32_t N_cap;     /* rows allocated in q/out; cu_q[B] <= N_cap */
    int32_t H_q;       /* query heads */
    int32_t H_kv;      /* KV heads, H_q % H_kv == 0 */
    int32_t D;         /* head dim: 64 or 128 */
    int32_t P;         /* tokens per KV page: 16 */
    int32_t max_pages; /* row stride of block_tables */
    int32_t n_pages;   /* pages in the caches (page ids are clamped into [0, n_pages)) */
    int32_t dtype;     /* FSR_F32 or FSR_BF16: element type of q, k_cache, v_cache */
    int32_t out_dtype; /* element type of out: FSR_F32 always allowed; FSR_BF16 with bf16 inputs */
    float scale;       /* softmax scale, normally 1/sqrt(D) */
    int32_t max_q_len; /* upper bound on the rows of any one request in this call (speculative
                          length + 1), or 0 if unknown.  A performance hint only: it picks the
                          register budget of the kernel; requests with more rows are still
                          computed correctly, in several passes over their keys. */
    int32_t max_workgroups; /* 0: one workgroup per compute unit of the device.  > 0: at most this
                          many -- for a call enqueued on a stream that owns only part of the
                          device (Sec. 3.3: drafting and verification share the GPU spatially), so
                          that the persistent grid matches the compute units it will get. */
    int32_t kv_layout; /* FSR_KV_HEAD_MAJOR: caches are [n_pages, H_kv, P, D];
                          FSR_KV_TOKEN_MAJOR: caches are [n_pages, P, H_kv, D] */
} fsr_attn_params;

/* Static shape of one accept call. */
typedef struct fsr_accept_params {
    int32_t B;         /* requests */
    int32_t V;         /* vocabulary size (> 0) */
    int32_t S_max;     /* max drafts per request in this call; emitted has S_max+1 columns */
    int32_t mode;      /* FSR_PROBS: rows are probabilities; FSR_LOGITS: rows are logits;
                          FSR_GREEDY: temperature 0, only the arg-max of a target row matters */
    double temperature; /* LOGITS mode: p = softmax(z / temperature), > 0; ignored in PROBS mode */
    int32_t dtype;     /* FSR_F32 (0) or FSR_BF16: element type of the p_target / p_draft rows
                          (bf16 not in FSR_GREEDY mode) */
    int32_t reserved2; /* must be 0 */
} fsr_accept_params;

/* Static shape of one compaction call. */
typedef struct fsr_prune_params {
    int32_t B;            /* requests */
    int32_t N_cap;        /* rows allocated in keep_mask / src_row / dst_row; cu_q[B] <= N_cap */
    int32_t suffix_close; /* 1: a request keeps its leading run of kept rows; 0: any subset, order kept */
    int32_t reserved;     /* must be 0 */
} fsr_prune_params;

/* Static shape of one early-exit rank check. */
typedef struct fsr_rank_params {
    int32_t B;        /* requests */
    int32_t N_cap;    /* rows allocated in logits / keep_mask; cu_q[B] <= N_cap */
    int32_t D_cap;    /* entries allocated in draft_tokens / rank; cu_d[B] <= D_cap <= 65535 */
    int32_t V;        /* scores per row (> 0) */
    int32_t K;        /* a draft passes iff fewer than K scores exceed its own (>= 0) */
    int32_t dtype;    /* FSR_F32 or FSR_BF16: element type of logits */
    int32_t reserved; /* must be 0 */
} fsr_rank_params;

/* Static description of the last failure on the calling thread ("" if none).  Host. */
const char* fsr_last_error(void);

/* Library version string.  Host. */
const char* fsr_version(void);

/*
 * Workspace bytes needed by fsr_verify_attention for shapes up to *p (host query, no GPU
 * work).  The same size covers every smaller B / N_cap / max_pages with the same heads.
 */
int fsr_attn_workspace_bytes(const fsr_attn_params* p /*host*/, size_t* out_bytes /*host*/);

/*
 * Verification attention (Sec. 2.1: the target model verifies all drafted tokens of a
 * request in one parallel pass; Sec. 3.1: each request has its own speculative length).
 *
 * For request i with c = ctx_lens[i] committed tokens and q_i = cu_q[i+1]-cu_q[i] rows in
 * this call, row j (0 <= j < q_i) is the query of the token at logical position c + j and
 * attends to positions 0 .. c + j (causal inside the suffix):
 *     out[row, h, :] = softmax_t(scale * q[row, h, :] . K_i[t, h/G, :]) . V_i[t, h/G, :]
 * with G = H_q / H_kv.  The K/V of the call's own rows must already be in the cache.
 * Logical position t of request i is stored in page block_tables[i*max_pages + t/P], slot
 * t % P.
 *
 *   q            [N_cap, H_q, D]      dtype
 *   k_cache      [n_pages, H_kv, P, D] dtype, or [n_pages, P, H_kv, D] (kv_layout)   v_cache likewise
 *   block_tables [B, max_pages] int32 (entries beyond a request's last page are not read)
 *   ctx_lens     [B] int32   tokens cached BEFORE this call's first row of the request
 *   spec_lens    [B] int32   nullable, carried for the caller's bookkeeping; cu_q decides
 *                            the number of rows (a one-shot call has spec_lens[i]+1 rows)
 *   cu_q         [B+1] int32 row offsets
 *   out          [N_cap, H_q, D] out_dtype; rows >= cu_q[B] are not written
 *   lse          [N_cap, H_q] float32, nullable: natural-log sum of exp of the scaled scores
 *   workspace    >= fsr_attn_workspace_bytes(p) bytes, 256-byte aligned
 * Softmax and accumulation are fp32; bf16 probabilities are carried as a hi+lo pair into
 * the matrix cores so the result is accurate to fp32 rounding, not bf16.
 */
int fsr_verify_attention(const void* q, const void* k_cache, const void* v_cache,
                         const int32_t* block_tables, const int32_t* ctx_lens,
                         const int32_t* spec_lens, const int32_t* cu_q, void* out, float* lse,
                         const fsr_attn_params* p /*host*/, void* workspace, size_t ws_bytes,
                         void* stream);

/*
 * fsr_verify_attention for callers that cannot allocate device memory or be handed a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * minus spec_lens and the workspace; same kernels, same results.  The partial results and arrival
 * counters that the workspace would hold live in a buffer built into the library
 * (fsr_static_scratch_bytes() bytes, about 26 MB, resident on every GPU the library runs on until the
 * process ends), laid out for a grid of at most 256 workgroups.  The call allocates and frees nothing.
 * Shapes whose scratch would not fit return FSR_EWS before anything is launched.  All calls on one
 * GPU share that buffer: calls that can overlap in time on one GPU (different streams) race; on one
 * stream they may follow each other freely (nothing needs clearing between calls).
 */
size_t fsr_static_scratch_bytes(void);
int fsr_verify_attention_static(const void* q, const void* k_cache, const void* v_cache,
                                const int32_t* block_tables, const int32_t* ctx_lens,
                                const int32_t* cu_q, void* out, float* lse,
                                const fsr_attn_params* p /*host*/, void* stream);

/*
 * Which kernel fsr_verify_attention runs for shapes *p (host query, no GPU work): FSR_PATH_STREAM,
 * the HBM-bandwidth kernel (bf16, D = 128, P = 16, H_q / H_kv <= 16, B <= 4096), or
 * FSR_PATH_GENERIC, one wavefront per (row, head) for every other supported shape (fp32 inputs,
 * D = 64, other page sizes, wider groups, larger batches): correct, but it re-reads K/V per query
 * head and row and is many times slower on large batches.  Negative on invalid shapes.
 */
#define FSR_PATH_GENERIC 0
#define FSR_PATH_STREAM 1
int fsr_attn_path(const fsr_attn_params* p /*host*/);

/*
 * Per-step schedule of the attention calls (Sec. 3.1: the batch of a verification step, with its
 * per-request speculative lengths, is fixed before the target model runs; every transformer layer
 * then sees the same lengths, row offsets and block tables).  fsr_attn_plan builds, once per step,
 * what every fsr_verify_attention call would otherwise rebuild at the start of its launch: the split
 * of the batch's K/V tiles over the workgroups and, per workgroup, the pages of its first tiles.
 * fsr_verify_attention_planned is fsr_verify_attention reading that schedule; the two give
 * bit-identical results.
 *
 *   plan        device buffer of >= fsr_attn_plan_bytes(p) bytes, 16-byte aligned, written by
 *               fsr_attn_plan (asynchronously, on `stream`) and read by the planned calls enqueued
 *               behind it.  It stays valid while block_tables, ctx_lens and cu_q keep their
 *               contents; *p must be the same in both calls (out_dtype, scale and kv_layout may
 *               differ), else the planned call returns FSR_ESHAPE / FSR_EINVAL before launching.
 * Only shapes with fsr_attn_path(p) == FSR_PATH_STREAM can be planned (FSR_EUNSUP otherwise).
 */
int fsr_attn_plan_bytes(const fsr_attn_params* p /*host*/, size_t* out_bytes /*host*/);
int fsr_attn_plan(const int32_t* block_tables, const int32_t* ctx_lens, const int32_t* cu_q,
                  const fsr_attn_params* p /*host*/, void* plan, size_t plan_bytes, void* stream);
int fsr_verify_attention_planned(const void* q, const void* k_cache, const void* v_cache,
                                 const int32_t* block_tables, const int32_t* ctx_lens,
                                 const int32_t* cu_q, void* out, float* lse,
                                 const fsr_attn_params* p /*host*/, const void* plan, void* workspace,
                                 size_t ws_bytes, void* stream);

/*
 * Cache append (Sec. 2.1 / Sec. 3.1, as fsr_kv_append) into caches stored in 8 bits: element x of a bf16 key
 * row of KV head g is stored as the E4M3 byte nearest to fl32(x / k_scale[g]) (ties to the even code, magnitudes
 * beyond 448 saturate, NaN stays NaN); values likewise with v_scale.  fsr_verify_attention_kv8 reads them back as
 * decode(byte) * scale.
 *   k_new, v_new      [N_cap, H_kv, D] bf16 (p->dtype must be FSR_BF16), D a multiple of 16
 *   k_cache, v_cache  uint8 caches in the layout p->kv_layout names, 16-byte aligned
 *   k_scale, v_scale  [H_kv] float32, device
 * Positions without a page and page ids outside the pool are skipped as in fsr_kv_append.
 */
int fsr_kv_append_kv8(const void* k_new, const void* v_new, void* k_cache, void* v_cache, const float* k_scale,
                      const float* v_scale, const int32_t* block_tables, const int32_t* ctx_lens,
                      const int32_t* cu_q, const fsr_attn_params* p /*host*/, void* stream);

/*
 * The same attention (Sec. 2.1, Sec. 3.1) over caches stored in 8 bits: every element of k_cache /
 * v_cache is one byte in the OCP E4M3 format (1 sign, 4 exponent bits with bias 7, 3 mantissa bits,
 * no infinities), and the cached key (value) it stands for is decode(byte) * k_scale[kv head]
 * (* v_scale[kv head]).  Storage only: queries, softmax and accumulation are as above (the bytes are
 * widened exactly to bf16 on the way to the matrix cores; the key scale joins the softmax scale, the
 * value scale the output).  Cache bytes per token halve, which is what bounds this kernel.
 *
 *   q                 [N_cap, H_q, D] bf16 (p->dtype must be FSR_BF16)
 *   k_cache, v_cache  [n_pages, H_kv, P, D] or [n_pages, P, H_kv, D] (kv_layout) uint8, 16-byte aligned
 *   k_scale, v_scale  [H_kv] float32, device
 *   everything else as for fsr_verify_attention (same workspace size; no spec_lens argument).
 * Needs D = 128, P = 16, H_q / H_kv <= 16, B <= 4096: FSR_EUNSUP otherwise.  Slots past a request's
 * last token may hold any bytes, NaN codes included.
 */
int fsr_verify_attention_kv8(const void* q, const void* k_cache, const void* v_cache, const float* k_scale,
                             const float* v_scale, const int32_t* block_tables, const int32_t* ctx_lens,
                             const int32_t* cu_q, void* out, float* lse, const fsr_attn_params* p /*host*/,
                             void* workspace, size_t ws_bytes, void* stream);

/*
 * fsr_verify_attention_kv8 reading a per-step schedule (Sec. 3.1: the lengths and block tables of a verification
 * step are the same for every layer): `plan` is a buffer that fsr_attn_plan has filled for the same *p, exactly as
 * for fsr_verify_attention_planned -- the schedule does not depend on how the caches are stored, so one plan serves
 * bf16 and 8-bit caches alike.  Results are bit-identical to fsr_verify_attention_kv8; errors as for the two calls
 * it combines.
 */
int fsr_verify_attention_kv8_planned(const void* q, const void* k_cache, const void* v_cache, const float* k_scale,
                                     const float* v_scale, const int32_t* block_tables, const int32_t* ctx_lens,
                                     const int32_t* cu_q, void* out, float* lse, const fsr_attn_params* p /*host*/,
                                     const void* plan, void* workspace, size_t ws_bytes, void* stream);

/*
 * Cache append (Sec. 2.1 / Sec. 3.1: the drafted tokens of a request enter the target model as
 * new positions behind its cached context).  Row j of request i (row cu_q[i] + j of k_new /
 * v_new) is the token at logical position ctx_lens[i] + j: its key and value vectors are copied,
 * bit for bit, to page block_tables[i * max_pages + t / P], slot t % P of the caches.  Call it
 * before fsr_verify_attention of the same rows (same stream).
 *
 *   k_new, v_new  [N_cap, H_kv, D] dtype; rows >= cu_q[B] are not read
 *   k_cache, v_cache, block_tables, ctx_lens, cu_q and *p as for fsr_verify_attention (H_q, scale,
 *   out_dtype, max_q_len and flags are ignored; D * element size must be a multiple of 16)
 * Positions at or beyond max_pages * P and page ids outside [0, n_pages) are skipped.
 */
int fsr_kv_append(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                  const int32_t* block_tables, const int32_t* ctx_lens, const int32_t* cu_q,
                  const fsr_attn_params* p /*host*/, void* stream);

/* Workspace bytes needed by fsr_spec_accept for shapes up to *p (host query). */
int fsr_accept_workspace_bytes(const fsr_accept_params* p /*host*/, size_t* out_bytes /*host*/);

/*
 * Accept / reject with recovery or bonus token (Sec. 2.1: accept drafted tokens until the
 * first mismatch, discard the rejected suffix, resample the first mismatched token from
 * the target; Sec. 3.3: "recovery token").  The mismatch test is that of speculative
 * sampling: draft x_n is accepted iff u_accept * q_n(x_n) < p_n(x_n) (evaluated in fp64).
 *
 * Request i has d_i = cu_d[i+1]-cu_d[i] draft rows and t_i = cu_t[i+1]-cu_t[i] target
 * rows, t_i - d_i in {0, 1}: the extra target row is the bonus row.
 *   n = number of leading accepted drafts.
 *   n < d_i            : one token from max(p_n - q_n, 0) normalised (from p_n if that is 0)
 *   n == d_i, bonus row: one token from p_{d_i}
 *   n == d_i, no bonus : no extra token (non-final frontier chunk, or rows pruned away)
 * Tokens are drawn by inverse CDF in index order with u_sample[i]: the first token whose
 * running mass (fp64) is strictly greater than u_sample[i] * total mass; zero-mass tokens
 * are never drawn.  The library draws no random numbers itself.
 *
 *   p_target     [*, V] dtype (probabilities, or logits in FSR_LOGITS mode); a bf16 value
 *                counts as the fp32 value with the same leading bits
 *   p_draft      [*, V] dtype
 *   draft_tokens [*] int32, u_accept [*] float32 in [0,1): indexed like p_draft rows
 *   u_sample     [B] float32 in [0,1)
 *   cu_t, cu_d   [B+1] int32 offsets of the call's target / draft rows
 *   t_rows       nullable [cu_t[B]] int32: call target row r is storage row t_rows[r] of
 *                p_target (identity if null)
 *   d_rows       nullable [cu_d[B]] int32: call draft row r is storage row d_rows[r] of
 *                p_draft, draft_tokens and u_accept (identity if null).  These maps are
 *                what fsr_prune_compact returns as src_row.
 *   accepted_len [B] int32 (n), n_emitted [B] int32, emitted [B, S_max+1] int32 padded -1
 * Requests with d_i > S_max or t_i - d_i outside {0,1} get accepted_len = n_emitted = -1.
 * Draft token ids are clamped into [0, V).
 * FSR_LOGITS mode: p = softmax(z / temperature) with sums in fp64 and an exponential good
 * to 5e-16 relative; a logit of -inf (a masked token) has probability exactly 0, a NaN
 * logit is treated the same way; a row needs at least one finite logit.  Only the rows
 * the outcome depends on are guaranteed to be read (target rows 0 .. n and draft rows
 * 0 .. min(n, d_i - 1)); a large call skips the later rows of requests rejected early.
 *
 * FSR_GREEDY mode (the same rule at temperature 0): draft n is accepted iff it equals the
 * arg-max token of target row n (the lowest id among equal maxima); the token after the
 * accepted run is the arg-max of the next target row (the row of the first mismatch, or
 * the bonus row).  p_target may hold probabilities or logits; p_draft, u_accept and
 * u_sample are not read and may be null.  Every target row of the call is read once.
 */
int fsr_spec_accept(const void* p_target, const void* p_draft, const int32_t* draft_tokens,
                    const float* u_accept, const float* u_sample, const int32_t* cu_t,
                    const int32_t* cu_d, const int32_t* t_rows, const int32_t* d_rows,
                    int32_t* accepted_len, int32_t* n_emitted, int32_t* emitted,
                    const fsr_accept_params* p /*host*/, void* workspace, size_t ws_bytes,
                    void* stream);

/*
 * Pruning of rejected rows and re-packing of the ragged batch (Sec. 3.2: the next layer
 * prunes the tokens of the rejected suffix and only the remaining tokens proceed;
 * Sec. 3.3: on a rejection every speculative token beyond it is discarded).
 *
 *   keep_mask  [N_cap] uint8 (non-zero = keep), cu_q [B+1] int32
 *   new_cu_q   [B+1] int32, new_q_lens [B] int32
 *   src_row    [N_cap] int32: new row -> old row for the first new_cu_q[B] entries, -1 after
 *   dst_row    [N_cap] int32: old row -> new row, -1 if dropped (rows >= cu_q[B]: -1)
 *   n_active   [1] int32, active_ids [B] int32: ascending requests with >= 1 kept row, -1 after
 *   payload_in nullable [N_cap, row_bytes]; payload_out [N_cap, row_bytes] gets the kept
 *              rows as a dense prefix (rows beyond it are not written).  row_bytes % 4 == 0.
 * No workspace is needed.
 */
int fsr_prune_compact(const uint8_t* keep_mask, const int32_t* cu_q, int32_t* new_cu_q,
                      int32_t* new_q_lens, int32_t* src_row, int32_t* dst_row, int32_t* n_active,
                      int32_t* active_ids, const void* payload_in, void* payload_out,
                      size_t row_bytes, const fsr_prune_params* p /*host*/, void* stream);

/*
 * Inverse of the compaction (Sec. 3.2 / Sec. 4: what was pruned away inside the model must be
 * back at its original row before the logits are formed, with filler in the rows that were dropped).
 * restored[r] = compact[dst_row[r]] where dst_row[r] >= 0, else every 32-bit word of the
 * row is pad_word; has_value[r] (nullable, uint8) says which.  row_bytes % 4 == 0.
 */
int fsr_prune_restore(const void* compact, const int32_t* dst_row, void* restored,
                      uint8_t* has_value, size_t row_bytes, int32_t N, uint32_t pad_word,
                      void* stream);

/*
 * Early-exit rank check (Sec. 3.2: intermediate scores predict a rejection when the draft is not
 * among their K best tokens; Sec. 4: that is decided by counting the scores above the draft's own,
 * without ever building the set of the K best).
 *
 * Request i owns the score rows cu_q[i] .. cu_q[i+1]-1 (its active query rows, q_i of them) and the
 * drafts cu_d[i] .. cu_d[i+1]-1 (d_i of them).  Row j scores the token that follows the row's
 * input, which is draft j of the request, so for j < min(q_i, d_i)
 *     rank[cu_d[i] + j] = number of v with logits[row j][v] > logits[row j][draft j]   (strictly)
 * Drafts without an active row (q_i <= j: pruned earlier) get rank -1, a draft id outside [0, V)
 * gets rank V.  keep_mask[cu_q[i]] = 1 (the row of the last committed token always stays);
 * keep_mask[cu_q[i] + j + 1] = (rank of draft j < K) for j + 1 < q_i.  The mask is not
 * suffix-closed: fsr_prune_compact (suffix_close = 1) drops everything behind the first failing
 * draft, fsr_prune_restore brings the survivors back to the original layout.
 *
 *   logits       [N_cap, V] dtype, row-major, rows contiguous
 *   draft_tokens [D_cap] int32      rank [D_cap] int32 (out; entries >= cu_d[B] not written)
 *   keep_mask    [N_cap] uint8 (out; rows >= cu_q[B] not written)
 * Reads each checked row once (4 V or 2 V bytes) and nothing else of size.  Asynchronous on
 * `stream`; needs no workspace.
 */
int fsr_topk_rank_check(const void* logits, const int32_t* draft_tokens, const int32_t* cu_q,
                        const int32_t* cu_d, int32_t* rank, uint8_t* keep_mask,
                        const fsr_rank_params* p /*host*/, void* stream);

/*
 * Keep mask after a one-shot accept step (Sec. 2.1: the rejected suffix is discarded): row j of
 * request i is kept iff j <= accepted_len[i], i.e. the rows of the last committed token and of the
 * accepted drafts survive, the rows of rejected drafts do not.  keep_mask [N_cap] uint8 in the
 * cu_q layout; rows >= cu_q[B] are not written.  Feed it to fsr_prune_compact.
 */
int fsr_survivor_mask(const int32_t* accepted_len, const int32_t* cu_q, uint8_t* keep_mask, int32_t B,
                      int32_t N_cap, void* stream);

/*
 * fsr_survivor_mask followed by fsr_prune_compact (suffix_close = 1) in one call and one launch
 * less (Sec. 2.1 / Sec. 3.2: after the accept step the rejected suffix of every request is dropped
 * and the survivors are re-packed): request i keeps its rows 0 .. accepted_len[i].  keep_mask
 * [N_cap] uint8 is an optional OUTPUT here (the mask fsr_survivor_mask would have written; may be
 * null); every other argument as in fsr_prune_compact (p->suffix_close is ignored).
 */
int fsr_survivor_compact(const int32_t* accepted_len, const int32_t* cu_q, uint8_t* keep_mask,
                         int32_t* new_cu_q, int32_t* new_q_lens, int32_t* src_row, int32_t* dst_row,
                         int32_t* n_active, int32_t* active_ids, const void* payload_in,
                         void* payload_out, size_t row_bytes, const fsr_prune_params* p /*host*/,
                         void* stream);

/*
 * Partial restore (Sec. 3.2, same passage): out[src_row[r]] = compact[r] for r < n_rows[0];
 * rows of `out` that no compacted row maps to keep their contents.  Used to put one chunk's
 * rows back into the original layout while other chunks' rows stay.  src_row [N_cap] and
 * n_rows [1] are fsr_prune_compact's src_row and &new_cu_q[B].  row_bytes % 4 == 0.
 */
int fsr_prune_scatter(const void* compact, const int32_t* src_row, const int32_t* n_rows, void* out,
                      size_t row_bytes, int32_t N_cap, void* stream);

/*
 * Frontier (chunked) verification state machine, Sec. 3.3: the suffix of every request is
 * verified in chunks; accepted tokens are committed per chunk; a rejection commits the
 * accepted prefix and the recovery token and discards every later speculative token of
 * that request.
 *
 * Per-request device state (all [B] int32, caller-allocated, set up by fsr_frontier_init):
 *   pos[i]     drafts of request i already verified;  active[i] 1 while it has rows left
 *   n_out[i]   tokens committed so far this step;  out_tokens [B, S_total_max+1] int32
 *
 * fsr_frontier_plan builds chunk k's row selections over the ORIGINAL row layout:
 *   chunk_len  [B] int32: drafts of request i to verify in this chunk (0 allowed)
 *   t_mask [N_t] uint8 over target/query rows (cu_q layout; the bonus row rides with the
 *   chunk that verifies the request's last draft), d_mask [N_d] uint8 over draft rows
 *   (cu_d layout), chunk_ctx [B] int32 = ctx_lens[i] + pos[i].
 * Feed the masks to fsr_prune_compact (suffix_close = 0) to get the chunk's offsets, row
 * maps and gathered q rows.
 *
 * fsr_frontier_commit consumes the chunk's accept results: appends emitted tokens to
 * out_tokens, advances pos by chunk_len, and clears active for requests that saw a
 * rejection or have no drafts left.
 */
int fsr_frontier_init(const int32_t* spec_lens, int32_t* pos, int32_t* active, int32_t* n_out,
                      int32_t* acc_total, int32_t* out_tokens, int32_t B, int32_t out_stride,
                      void* stream);
int fsr_frontier_plan(const int32_t* ctx_lens, const int32_t* spec_lens, const int32_t* cu_q,
                      const int32_t* cu_d, const int32_t* pos, const int32_t* active,
                      const int32_t* chunk_len, uint8_t* t_mask, uint8_t* d_mask,
                      int32_t* chunk_ctx, int32_t B, int32_t N_t_cap, int32_t N_d_cap,
                      void* stream);
int fsr_frontier_commit(const int32_t* spec_lens, const int32_t* chunk_len,
                        const int32_t* accepted_len, const int32_t* n_emitted,
                        const int32_t* emitted, int32_t emitted_stride, int32_t* pos,
                        int32_t* active, int32_t* n_out, int32_t* acc_total, int32_t* out_tokens,
                        int32_t B, int32_t out_stride, void* stream);

/* ---------------------------------------------------------------------------------------
 * Measurement aid (not a step of the verification path): one launch that reads `bytes` bytes at
 * src (device, 16-byte aligned; bytes a positive multiple of 32768) with plain 16-byte loads, eight
 * in flight per thread, `workgroups` workgroups of 256 threads striding over the buffer, and
 * writes the XOR of what each workgroup read to sink[workgroup] (device, `workgroups` words;
 * overwritten).  scatter_4k = 0: front to back.  1: the buffer's 4 KB blocks are visited in a
 * scattered order (a fixed permutation; bytes must then be a power of two) -- the granularity at
 * which a paged cache with 16-token pages stores one head's K or V bytes.  2: scattered blocks
 * again, each read as 16 rows of 256 bytes with a load taking 64 bytes of every row (K fetched
 * straight into a matrix-operand layout) instead of 1 KB of consecutive bytes.
 * bench.py times it beside the attention kernel: the rate this device delivers
 * to trivially parallel streaming reads is the practical ceiling the kernel's achieved HBM rate
 * is to be read against (the roofline fraction itself stays against the published 8 TB/s).
 * Errors: FSR_EINVAL for null or misaligned pointers, a size that is not such a multiple (or
 * not a power of two with scatter_4k != 0), or workgroups outside 1..65535.
 */
int fsr_hbm_read_probe(const void* src, size_t bytes, unsigned long long* sink, int32_t workgroups,
                       int32_t scatter_4k, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FASER_VERIFY_H */
