/*
 * memosight.h -- C ABI of the MI355X (gfx950) library for MemoSight's per-step decode hot path:
 * fused Predict+Verify attention over a paged KV cache that context compression keeps compacting,
 * the accepted-KV append, the segment -> memory-token compaction and greedy prefix acceptance.
 *
 * Conventions
 *   - Every function returns an int status: MS_OK (0) or a negative MS_ERR_* code.  Nothing throws
 *     or aborts across this boundary; ms_last_error() gives a thread-local message for the last
 *     failing call on the calling thread.
 *   - "host" pointers are ordinary CPU memory read (or written) before the call returns.
 *     "device" pointers are HIP device memory on the cache's GPU; they are only touched by work
 *     queued on `stream` (a hipStream_t passed as void*, NULL = the default stream).
 *   - Small control arrays (sequence ids, counts, ranges) are host pointers; tensors (Q, K, V,
 *     position ids, outputs, token ids) are device pointers.
 *   - The caller allocates and owns the KV pool, all tensors and workspaces; the library never
 *     frees them.  The library owns the opaque ms_cache handle, its host-side page tables and a
 *     small device mirror of them which it allocates in ms_cache_create and frees in
 *     ms_cache_destroy.  No other call allocates device memory.
 *   - Calls that take a cache are asynchronous on `stream` unless stated; all calls on one cache
 *     must be issued from one thread at a time and on one stream (or be ordered by the caller).
 *   - Tensor element type follows the cache dtype: float (MS_F32) or bfloat16 bit patterns
 *     (MS_BF16, 2 bytes, upper half of an IEEE float).  Position ids and token ids are int32.
 *
 * KV pool layout (row-major, innermost last), element = cache dtype:
 *     pool[n_layers][n_pages][n_kv_heads][2 (0 = K, 1 = V)][16 slots][head_dim]
 * Logical token t of a sequence lives in page page_table[t / 16], slot t % 16; one page table per
 * sequence serves every layer.  Cached K is stored already rotated (RoPE at its position id).
 *
 * RoPE convention (the paper names RoPE, Section 2.1.2 "Uniform Position Layout", without fixing a
 * variant; this is the rotate-half form of the model families it evaluates): element i < D/2 pairs
 * with i + D/2; inv_freq_i = float(rope_base^(-2i/D)); angle = float(pos) * inv_freq_i in fp32;
 * x'_i = x_i cos - x_{i+D/2} sin,  x'_{i+D/2} = x_{i+D/2} cos + x_i sin.
 */
#ifndef MEMOSIGHT_H
#define MEMOSIGHT_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MS_PAGE_SIZE 16
#define MS_MAX_BATCH 256        /* sequences per call */
#define MS_MAX_QUERIES 64       /* n_verify + n_foresight per sequence */

enum { MS_F32 = 0, MS_BF16 = 1 };

enum {
    MS_OK = 0,
    MS_ERR_INVALID = -1,        /* null pointer, bad size, bad flag, unknown sequence id */
    MS_ERR_OOM_PAGES = -2,      /* the pool (or a sequence's page table) cannot hold the request;
                                   the cache is left unchanged */
    MS_ERR_RANGE = -3,          /* a segment or length lies outside the sequence */
    MS_ERR_HIP = -4,            /* a HIP runtime call failed */
    MS_ERR_UNSUPPORTED = -5,    /* shape outside what the kernels are built for */
    MS_ERR_WORKSPACE = -6       /* workspace missing or too small */
};

enum {
    MS_PRE_ROTATED = 0,         /* K rows are already rotated; pos_ids is ignored (may be NULL) */
    MS_ROPE_APPLY = 1           /* rotate K rows by pos_ids before storing */
};

typedef struct ms_cache ms_cache;

typedef struct ms_cache_desc {
    int n_layers;
    int n_q_heads;              /* multiple of n_kv_heads; query head h reads KV head h / (Hq/Hkv) */
    int n_kv_heads;
    int head_dim;               /* 64 or 128 */
    int page_size;              /* must be MS_PAGE_SIZE */
    int n_pages;                /* pages per layer in the pool */
    int max_seqs;               /* sequence ids are 0 .. max_seqs-1 */
    int max_pages_per_seq;
    int dtype;                  /* MS_F32 or MS_BF16 */
    float rope_base;
    void* pool;                 /* device; ms_pool_bytes(desc) bytes; owned by the caller */
    size_t pool_bytes;
} ms_cache_desc;

/* ---- library ---------------------------------------------------------------------------- */

/* Thread-local text of the last error returned on this thread ("" if none). Never NULL. */
const char* ms_last_error(void);

/* ---- cache life cycle (Algorithm 1's KV cache S) ------------------------------------------ */

/* Bytes the pool must have for this descriptor (ignores desc->pool / pool_bytes). 0 if invalid. */
size_t ms_pool_bytes(const ms_cache_desc* desc);

/* Creates an empty cache over the caller's pool on the current HIP device: all pages free, no
 * sequences.  Allocates the device mirror of the page tables (max_seqs * (max_pages_per_seq + 1)
 * ints) and a small pinned staging ring.  Synchronous. */
int ms_cache_create(const ms_cache_desc* desc, ms_cache** out);

/* Frees the handle and what ms_cache_create allocated (not the pool).  Synchronous. */
int ms_cache_destroy(ms_cache* cache);

/* New empty sequence; *seq_id receives the lowest unused id. */
int ms_seq_create(ms_cache* cache, int* seq_id);

/* Adopts `n_pages` pages (host array, logical order) that the caller has already filled in the
 * pool as a new sequence of `length` tokens (n_pages must equal ceil(length / 16)).  Every page
 * must currently be free and appear once.  Used to hand over a prefilled or restored cache. */
int ms_seq_import(ms_cache* cache, int length, const int* pages, int n_pages, int* seq_id,
                  void* stream);

/* Releases the sequence and returns all its pages to the free set. */
int ms_seq_free(ms_cache* cache, int seq_id);

/* ---- S <- S (+) A : append KV rows (Algorithm 1, "Append to cache") ----------------------- */

/* Appends n_tok[b] rows to sequence seq_ids[b], for b = 0..B-1 in that order, in every layer.
 *   seq_ids, n_tok : host [B]
 *   k, v           : device [n_layers][sum n_tok][n_kv_heads][head_dim]
 *   pos_ids        : device [sum n_tok] int32 (ignored with MS_PRE_ROTATED)
 * A page is taken exactly when a sequence's length before a row is a multiple of 16, always the
 * lowest free page index.  If the pool cannot hold the whole call: MS_ERR_OOM_PAGES, nothing
 * changes. */
int ms_append_kv(ms_cache* cache, int B, const int* seq_ids, const int* n_tok, const void* k,
                 const void* v, const int* pos_ids, int flags, void* stream);

/* Appends the first accept_len[b] in-flight rows of each sequence (the accepted verify tokens of
 * the step; foresight rows are never stored -- Section 2.3 "MTP Attention").
 *   accept_len : host [B], 0 <= accept_len[b] <= n_q
 *   k_new,v_new: device [n_layers][B][n_q][n_kv_heads][head_dim] (K not rotated)
 *   pos_ids    : device [B][n_q]
 * Same page policy and error behaviour as ms_append_kv. */
int ms_commit_accepted(ms_cache* cache, int B, const int* seq_ids, const int* accept_len, int n_q,
                       const void* k_new, const void* v_new, const int* pos_ids, void* stream);

/* ms_commit_accepted with the accept lengths read on the device (Algorithm 1, "S <- S (+) A", without
 * the host learning how many tokens were accepted): the step's stream never has to be synchronised.
 *   accept_len : DEVICE [B] int32 (e.g. what ms_accept wrote); values are clamped to [0, n_max]
 *   n_max      : the most rows a sequence can keep (the verify block's size), 1 <= n_max <= min(n_q, 16)
 *   first_pid  : DEVICE [B] int32 or NULL; first_pid[b] += accept_len[b] (the next step's first
 *                position id, see ms_step_positions_device)
 * Same rows, same pages and same page order as ms_commit_accepted with the same accept lengths: the
 * kernel takes pages from an ascending list of the free pages in the order the host would (sequences
 * in argument order, the lowest free page whenever a row's index is a multiple of 16).  Afterwards
 * the host's lengths and page tables lag behind the device's: ms_predict_verify_attention and further
 * device-side commits go by the device's and need no catching up; every other call that reads or
 * changes lengths, page tables or the free set (ms_seq_len, ms_seq_page_table, ms_append_kv,
 * ms_compact_segment, ms_seq_free, ...) first synchronises the stream of the outstanding commits and
 * brings the host up to date (ms_cache_sync does only that).  The call needs room for the worst case
 * (n_max rows for every sequence: one page each): MS_ERR_OOM_PAGES otherwise, nothing changes.  A
 * sequence id may appear once per call; all outstanding device-side commits must be on one stream. */
int ms_commit_accepted_device(ms_cache* cache, int B, const int* seq_ids, const int* accept_len,
                              int n_q, int n_max, const void* k_new, const void* v_new,
                              const int* pos_ids, int* first_pid, void* stream);

/* Brings the host's lengths and page tables up to date with outstanding device-side commits
 * (synchronises their stream).  A no-op when there are none. */
int ms_cache_sync(ms_cache* cache);

/* ---- UpdateCache : evict a finished step, keep its memory tokens -------------------------- */

/* For b = 0..B-1 in order: logical rows [seg_begin[b], seg_begin[b] + seg_len[b]) of sequence
 * seq_ids[b] are dropped and n_mem[b] memory-token rows take their place; rows after the segment
 * (none when the segment is the cache suffix, as in Algorithm 1) keep their stored values and
 * follow.  All layers at once.  (Section 2.1.2; Algorithm 1, UpdateCache.)
 *   seq_ids, seg_begin, seg_len, n_mem : host [B]
 *   mem_k, mem_v : device [n_layers][sum n_mem][n_kv_heads][head_dim]
 *   mem_pos      : device [sum n_mem] (the memory tokens' UPL position ids; see ms_upl_positions)
 *   workspace    : device scratch, only needed when some sequence has rows after its segment:
 *                  ms_compact_workspace_bytes() bytes; may be NULL otherwise.
 * A sequence id may appear at most once per call.
 * Page policy per sequence: pages holding any row below seg_begin are kept, all later pages of
 * the sequence are released first, then rows are re-appended (memory rows, then tail rows), each
 * new page being the lowest free index.  Errors (MS_ERR_RANGE, MS_ERR_OOM_PAGES,
 * MS_ERR_WORKSPACE) leave the cache unchanged. */
int ms_compact_segment(ms_cache* cache, int B, const int* seq_ids, const int* seg_begin,
                       const int* seg_len, const int* n_mem, const void* mem_k, const void* mem_v,
                       const int* mem_pos, int flags, void* workspace, size_t ws_bytes,
                       void* stream);

/* Scratch bytes ms_compact_segment needs for the given call (0 if every segment is a suffix). */
size_t ms_compact_workspace_bytes(ms_cache* cache, int B, const int* seq_ids, const int* seg_begin,
                                  const int* seg_len);

/* ---- fused Predict+Verify attention -------------------------------------------------------- */

/* One attention layer of one decode step (Section 2.1.1 Predict and Verify, fused in one pass;
 * visibility from Section 2.3 "Compression Attention" / "MTP Attention").  For sequence
 * b = seq_ids[.], query i in [0, n_q), n_q = n_verify + n_foresight, query head h:
 *     out[b][i][h] = softmax_t(scale * rope(q[b][i][h], pos[b][i]) . k_t) . v_t
 * over t in: every cached token of the sequence (layer `layer`), the in-flight tokens
 * j < ctx_new[b][i], and the in-flight token i itself; in-flight keys are
 * rope(k_new[b][j][g], pos[b][j]).  With ctx_new == NULL the default layout is used: verify token i
 * sees the i verify tokens before it; each foresight token sees the whole verify block and no
 * other foresight token.  The cache is only read.
 *   seq_ids : host [B], B <= MS_MAX_BATCH;  n_q <= MS_MAX_QUERIES, n_verify >= 0, n_q >= 1
 *   q       : device [B][n_q][n_q_heads][head_dim]            (q, k_new, v_new, out: 16-byte aligned)
 *   k_new, v_new : device [B][n_q][n_kv_heads][head_dim]
 *   pos_ids : device [B][n_q];  ctx_new : device [B][n_q] or NULL
 *   scale   : 0 means 1/sqrt(head_dim)
 *   out     : device [B][n_q][n_q_heads][head_dim], cache dtype
 *   workspace : device, at least ms_attention_workspace_bytes(cache, B, n_q) bytes, 256-byte
 *               aligned; holds rotated queries and split-KV partial results. */
int ms_predict_verify_attention(ms_cache* cache, int layer, int B, const int* seq_ids, int n_verify,
                                int n_foresight, const void* q, const void* k_new,
                                const void* v_new, const int* pos_ids, const int* ctx_new,
                                float scale, void* out, void* workspace, size_t ws_bytes,
                                void* stream);

size_t ms_attention_workspace_bytes(ms_cache* cache, int B, int n_q);

/* ms_predict_verify_attention for callers that cannot allocate device memory or carry a workspace
 * around: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors, without the workspace: the split-KV partial results go to a fixed
 * array of MS_STATIC_SCRATCH_BYTES of device memory inside the library, which every GPU the library
 * runs on holds until the process ends.  The call allocates and frees nothing on the device.
 * A call whose ms_attention_workspace_bytes(cache, B, n_q) exceeds MS_STATIC_SCRATCH_BYTES fails
 * with MS_ERR_WORKSPACE and launches nothing (at 4 KV heads on a 256-CU part: up to 188 sequences
 * per call).  All calls on one GPU -- from any cache, stream or thread -- share the one array, which
 * keeps the last call's partials: calls that overlap in time on one GPU race; order them on one
 * stream or with events.  Nothing in the array has to start at zero. */
#define MS_STATIC_SCRATCH_BYTES (32u << 20)
int ms_predict_verify_attention_static(ms_cache* cache, int layer, int B, const int* seq_ids,
                                       int n_verify, int n_foresight, const void* q,
                                       const void* k_new, const void* v_new, const int* pos_ids,
                                       const int* ctx_new, float scale, void* out, void* stream);

/* By default attention results are reproducible to rounding only: the streaming kernel (bf16,
 * head_dim 128) lets the waves of a workgroup take KV tiles first come, first served, so the
 * order in which a row's partial sums are added varies from call to call.  on != 0 fixes the
 * assignment instead: calls with the same inputs, cache contents and page tables then return the
 * same bits, a few percent slower.  The general kernel is always reproducible. */
int ms_attention_set_deterministic(ms_cache* cache, int on);

/* Test hook for the failure path of the streaming kernel's split-KV combine.  In one launch the
 * shares of a (sequence, KV head) pair count themselves in two counters; the share that finishes
 * last waits (a few microseconds) until the others have published their partial results and folds
 * them.  If the counters are ever in a bad state the wait gives up after a bounded number of polls:
 * the pair's output rows are left unwritten, nothing faults, and the next
 * ms_predict_verify_attention call on the cache (and ms_check_integrity) returns MS_ERR_HIP and
 * puts the counters back to zero.  This call forces that condition from the host: poll_limit > 0
 * replaces the bound (0 restores the default, about a second), and every pair's "published"
 * counter is set to published_bias (0 = the healthy state) behind the work already queued on
 * `stream`. */
int ms_attention_fault_injection(ms_cache* cache, int poll_limit, int published_bias, void* stream);

/* ---- greedy longest-prefix acceptance (footnote of Section 2.1.1) -------------------------- */

/* accept_len[b] = number of leading j with draft[b][j] == target[b][j] (target[b][j] being the
 * model's argmax token for the slot draft[b][j] fills); if stop ids are given the count ends just
 * after the first accepted stop id (so a finished step is always the cache suffix, Algorithm 1).
 * next_token[b] = target[b][accept_len[b]] if accept_len[b] < n, else -1.
 *   draft, target : device [B][n] int32;  stop_ids : device [n_stop] or NULL
 *   accept_len, next_token : device [B] int32 */
int ms_accept(int B, int n, const int* draft, const int* target, const int* stop_ids, int n_stop,
              int* accept_len, int* next_token, void* stream);

/* ---- introspection (host side; synchronous where noted) ------------------------------------ */

int ms_seq_len(ms_cache* cache, int seq_id, int* len);
/* Copies up to `cap` page ids to `out` (host) and stores the page count in *n. */
int ms_seq_page_table(ms_cache* cache, int seq_id, int* out, int cap, int* n);
int ms_free_page_count(ms_cache* cache, int* n);
int ms_peak_pages(ms_cache* cache, int* n);
/* Kernels launched so far by calls on this cache (attention, append, commit, compaction, page-table
 * patches): lets a caller see how many launches a call cost. */
int ms_launch_count(ms_cache* cache, long long* n);
/* Checks: every page is free or owned exactly once, page counts match lengths, and (after
 * synchronising `stream`) the device mirror equals the host tables.  MS_OK or MS_ERR_INVALID. */
int ms_check_integrity(ms_cache* cache, void* stream);

/* ---- the decoder block around the attention (full decode step) ------------------------------
 *
 * Algorithm 1 (Appendix A) runs the whole model once per speculative step.  Around the attention
 * the block of the paper's models (Section 3.1) is: RMSNorm, Q/K/V projections, output projection,
 * residual, RMSNorm, SwiGLU MLP, residual; then the final norm, the LM head and the greedy token.
 * The projections are dense GEMMs the caller runs; these are the memory-bound pieces between them.
 * All tensors are device pointers, 16-byte aligned, rows contiguous; activations and weights are
 * bf16, the residual stream h is fp32; arithmetic is fp32.  Bad sizes or pointers return
 * MS_ERR_INVALID and launch nothing. */

/* h_out[r][:] = table[tokens[r]][:] (bf16 -> fp32), r < n.  table [vocab][hidden], tokens device
 * [n]; ids outside [0, vocab) are clamped (the caller validates them).  hidden % 8 == 0. */
int ms_embed_rows(const void* table, int vocab, int hidden, const int* tokens, int n, float* h_out,
                  void* stream);
/* h[r] += delta[r] (bf16 [n][hidden]; NULL: nothing is added), then
 * out[r] = h[r] / sqrt(mean(h[r]^2) + eps) * weight (bf16 [n][hidden]).  hidden % 8 == 0,
 * hidden <= 8192. */
int ms_add_rmsnorm(float* h, const void* delta, const void* weight, float eps, void* out, int n,
                   int hidden, void* stream);
/* out[r][i] = silu(gate_up[r][i]) * gate_up[r][inter + i]: gate_up bf16 [n][2 * inter] (the gate
 * and up projections side by side), out bf16 [n][inter].  inter % 8 == 0, n <= 65535. */
int ms_swiglu(const void* gate_up, void* out, int n, int inter, void* stream);
/* out[r] = index of the largest of logits[r][0 .. vocab) (bf16, row stride ld elements, ld % 8 ==
 * 0), the lowest index among equal maxima; NaN never wins.  out device int32 [n]. */
int ms_argmax_rows(const void* logits, int n, int vocab, long ld, int* out, void* stream);

/* Dense projection of a step's rows: C[M][N] = A[M][K] . W[N][K]^T (+ bias[N]), bf16 operands and
 * results, fp32 accumulation on the matrix cores (the model's projections inside Algorithm 1's
 * SpeculativeStep; Section 3.1 names the models).  A, W, bias, the destinations and the workspace
 * are device pointers; out and out_col are host arrays.  The N columns may go to up to 4
 * destinations: columns out_col[i] .. out_col[i + 1] are written to out[i], a row-major
 * [M][out_col[i + 1] - out_col[i]] bf16 tensor (out_col[0] = 0, out_col[n_out] = N, boundaries
 * multiples of 128) -- one fused Q/K/V projection fills three tensors.  N % 128 == 0,
 * K % (32 * split_k) == 0; A and W 16-byte, bias and destinations 8-byte aligned.
 * split_k > 1 divides K over that many workgroups per output tile (for few output tiles and a deep
 * K, such as the MLP down projection); the partial sums are added in a fixed order and the call
 * fails with MS_ERR_WORKSPACE without ms_gemm_workspace_bytes(M, N, K, split_k) bytes of 16-byte
 * aligned workspace.  With split_k == 1 that function returns what the call can use to split the
 * tiles of a partly filled last round over K (0 if the shape has none on the current device);
 * without that much workspace the call computes whole tiles throughout, with the same result up to
 * the order of the fp32 additions.  With M <= 16 and K % 128 == 0 (the step of one or two
 * sequences) the product is bound by reading W once and runs on a kernel that streams 16 weight
 * rows per wave through the matrix cores with all rows of A as the other operand; it divides K by
 * what fits its LDS share (ms_gemm_workspace_bytes covers the partial sums) and ignores split_k
 * unless the workspace is too small for that. */
size_t ms_gemm_workspace_bytes(int M, int N, int K, int split_k);
int ms_gemm_bf16(const void* a, const void* w, const void* bias, int M, int N, int K, int n_out,
                 void* const* out, const int* out_col, int split_k, void* workspace, size_t ws_bytes,
                 void* stream);

/* The MLP's gate and up projections with SwiGLU applied to the fp32 sums:
 * out[m][j] = silu(A[m] . Wg[j]) * (A[m] . Wu[j]), bf16 [M][inter].  w_gate_up is the bf16
 * [2 * inter][K] weight with the rows of both projections interleaved in blocks of 32: rows
 * 64 b .. 64 b + 32 are gate rows 32 b .. 32 b + 32, rows 64 b + 32 .. 64 b + 64 the up rows of the
 * same outputs.  inter % 64 == 0, K % 32 == 0; workspace as for ms_gemm_bf16 with N = 2 * inter and
 * split_k = 1 (optional).  M <= 16 with inter % 128 == 0 and K % 128 == 0 runs on the few-row
 * kernel of ms_gemm_bf16 when all rows of A over the whole K fit its LDS share (at K = 3584: up to
 * 8 rows, and up to 16 rows for 2 * inter >= 32768, where a workgroup takes a whole compute unit). */
int ms_gemm_swiglu_bf16(const void* a, const void* w_gate_up, int M, int inter, int K, void* out,
                        void* workspace, size_t ws_bytes, void* stream);

/* A projection together with the residual add and RMSNorm that follow it in the decoder block (the
 * MLP's down projection and the next block's input norm): delta = A[M][K] . W[N][K]^T rounded to
 * bf16, h[m] += delta[m] (device fp32 [M][N], in place), out[m] = h[m] / sqrt(mean(h[m]^2) + eps) *
 * norm_weight (bf16 [N]; out bf16 [M][N]) -- ms_gemm_bf16 without bias followed by ms_add_rmsnorm,
 * with the same bits, one launch less and no [M][N] intermediate.  K is always divided (the sum of
 * the parts and the norm share a kernel): split_k >= 2 above 16 rows, any split_k (ignored) up to
 * 16 rows with K % 128 == 0.  N % 128 == 0, N <= 8192, K % (32 * split_k) == 0; operands 16-byte
 * aligned; workspace: ms_gemm_add_rmsnorm_workspace_bytes(M, N, K, split_k) bytes, 16-byte aligned
 * (0: the shape needs split_k >= 2), MS_ERR_WORKSPACE without it. */
size_t ms_gemm_add_rmsnorm_workspace_bytes(int M, int N, int K, int split_k);
int ms_gemm_add_rmsnorm_bf16(const void* a, const void* w, int M, int N, int K, int split_k, float* h,
                             const void* norm_weight, float eps, void* out, void* workspace,
                             size_t ws_bytes, void* stream);

/* The LM head and the greedy token in one: out[m] = argmax over n of A[m] . W[n] (device int32 [M]),
 * taken on the fp32 sums, the lowest column among equal maxima, NaN never wins (a row of NaN gives
 * 0); the [M][vocab] logits are not written.  Operands as for ms_gemm_bf16 (vocab % 128 == 0,
 * K % 32 == 0); workspace: ms_lm_head_argmax_workspace_bytes(M, vocab, K) bytes, 16-byte aligned,
 * MS_ERR_WORKSPACE without it.  (The greedy token of Algorithm 1's SpeculativeStep.) */
size_t ms_lm_head_argmax_workspace_bytes(int M, int vocab, int K);
int ms_lm_head_argmax_bf16(const void* a, const void* w, int M, int vocab, int K, int* out,
                           void* workspace, size_t ws_bytes, void* stream);

/* ---- profiling ------------------------------------------------------------------------------- */

/* From now on, every stride-th ms_predict_verify_attention call on this cache that runs the
 * streaming kernel (the first such call included) opens a timed span: one pair of HIP events
 * around the launches of that call and of the span - 1 eligible calls after it (1 <= span <=
 * stride), for up to `capacity` spans; capacity 0 switches profiling off.  An event pair costs the
 * stream a few microseconds, which a span of back-to-back calls shares out and a stride keeps rare;
 * the caller keeps other work on the stream out of a span it wants to read as kernel time (a span
 * of 1 always is).  Creates the events (synchronous). */
int ms_profile_attention(ms_cache* cache, int capacity, int stride, int span);
/* Synchronises the recorded events and stores, per span in call order, its duration divided by the
 * span (milliseconds per call) in ms_out (host, up to cap entries); *n receives how many spans were
 * recorded (complete ones only: a span still open is dropped).  Resets the count. */
int ms_profile_read(ms_cache* cache, float* ms_out, int cap, int* n);

/* A plain streaming read of device memory at `src` (16-byte aligned) on `stream`: the first
 * `bytes` bytes rounded down to a multiple of 32 KiB (*bytes_read, if not NULL, receives that
 * count; less than 32 KiB launches nothing), MS_READ_PROBE_BLOCKS_PER_CU workgroups of 256 threads
 * per compute unit taking 32 KiB groups in turn with eight 16-byte loads per thread in flight,
 * non-temporal loads if `non_temporal` is not 0.  Nothing is written (`sink`, device memory of at
 * least 4 bytes per workgroup, takes a word only for data that folds to one particular value; it
 * keeps the loads alive).  What this reaches is the bandwidth a kernel that makes one pass over
 * the cache (Section 2.3: every cached token is visible to every query) can be compared with
 * besides the part's published peak.  Asynchronous; the caller times it.  MS_ERR_INVALID on a null
 * or misaligned pointer. */
#define MS_READ_PROBE_BLOCKS_PER_CU 2
int ms_hbm_read_probe(const void* src, size_t bytes, int non_temporal, void* sink, void* stream, size_t* bytes_read);

/* ---- position layout helpers (pure host integer functions) --------------------------------- */

/* Adaptive Memory Allocation: ceil(n_tokens / c).  Negative on bad input. */
int ms_ama_count(int n_tokens, int c);
/* Uniform Position Layout: the step's tokens hold PIDs first_pid .. first_pid + n_tokens - 1 and
 * are cut into groups of c (the last may be shorter); out[g] = centre PID of group g (lower middle
 * for even-sized groups).  Writes at most cap entries, returns the group count. */
int ms_upl_positions(int first_pid, int n_tokens, int c, int* out, int cap);
/* PID of <o> after a step whose last token has PID last_pid (Section 2.2): last_pid + 1. */
int ms_output_token_pid(int last_pid);
/* PIDs of d foresight tokens after a prefix ending at last_prefix_pid: last + 1 .. last + d
 * (Section 2.1.1: foresight token j stands at the position of the j-th token after the prefix and
 * predicts the token one position further). */
int ms_foresight_pids(int last_prefix_pid, int d, int* out, int cap);
/* Position ids of a whole batch's step, out[B][n_verify + n_foresight] (host): sequence b's verify
 * tokens hold first_pid[b] .. and its foresight tokens follow by the rule of ms_foresight_pids
 * (Section 2.1.1; the position rule of Section 2.2 with the verify block as the prefix).
 * Returns the number of entries written, negative on bad input. */
int ms_step_positions(int B, const int* first_pid, int n_verify, int n_foresight, int* out);
/* ms_step_positions from a DEVICE array of first position ids into a DEVICE array out[B][n_verify +
 * n_foresight]: with ms_commit_accepted_device advancing first_pid, a decode loop needs no host
 * round trip for its position ids.  Asynchronous on `stream`. */
int ms_step_positions_device(int B, const int* first_pid, int n_verify, int n_foresight, int* out,
                             void* stream);
/* Default ctx_new row for n_verify + n_foresight queries: verify token i sees the i verify tokens
 * before it, every foresight token sees the whole verify block and, like every query, itself
 * (Section 2.1.1; Section 2.3 "MTP Attention"). */
int ms_default_ctx_new(int n_verify, int n_foresight, int* out, int cap);
/* Per-position foresight step (Section 2.2 "CoT Augmentation", Section 2.3 "MTP Attention": the
 * layout the model is trained on, used at inference so that drafts survive a partial acceptance):
 * queries are the n_verify verify tokens (PIDs first_pid ..) followed by d foresight tokens for
 * every verify token j in turn, foresight k = 1..d holding PID pid_j + k and seeing verify tokens
 * 0..j (ctx_new = j + 1).  Call ms_predict_verify_attention with n_verify, n_foresight =
 * n_verify * d, these pos_ids and this ctx_new.  Either output may be NULL; at most cap entries are
 * written to each; returns n_verify * (1 + d), negative on bad input. */
int ms_per_position_layout(int first_pid, int n_verify, int d, int* pos_out, int* ctx_out, int cap);
/* Memory-token PIDs without UPL (Appendix B, "w/o UPL"): last_pid + 1 .. last_pid + n_mem, the
 * consecutive PIDs after the step's last token; <o> then takes ms_output_token_pid(last_pid +
 * n_mem).  Returns n_mem, negative on bad input. */
int ms_consecutive_memory_positions(int last_pid, int n_mem, int* out, int cap);
/* UPL for a fixed budget of n_mem memory tokens per step (Appendix B, "w/o AMA"): the step's
 * n_tokens >= 1 tokens are cut into n_mem contiguous groups at floor(g * n_tokens / n_mem); out[g] =
 * centre PID of group g (lower middle), a group left empty standing for its boundary token.
 * Returns n_mem, negative on bad input. */
int ms_upl_positions_fixed(int first_pid, int n_tokens, int n_mem, int* out, int cap);

#ifdef __cplusplus
}
#endif
#endif /* MEMOSIGHT_H */
