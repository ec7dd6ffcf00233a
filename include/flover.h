/*
 * flover.h -- C ABI of the fused decoder step of temporal fusion (Flover) on one MI355X.
 *
 * The library owns no device memory of its own: flover_init carves every buffer it will ever use
 * out of a caller-provided device arena (the paper's Buffer Manager pre-allocates all buffers once,
 * sized from max_concurrency, and never allocates during inference -- Section V-A).  All work is
 * enqueued on the caller's HIP stream.  One caller thread per context (the paper's token
 * generation thread T_I); calls are synchronous with respect to the host unless stated.
 *
 * Every function returns 0 on success or a negative FLOVER_E_* code; nothing throws or aborts
 * across this boundary.  flover_last_error() gives the text of the most recent failure.
 *
 * Pointer arguments are marked [host] or [device].  "dtype" elements are 4-byte IEEE fp32,
 * 2-byte IEEE fp16 or 2-byte bfloat16 according to flover_config.dtype.
 */
#ifndef FLOVER_H
#define FLOVER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { FLOVER_OK = 0, FLOVER_E_INVAL = -1, FLOVER_E_FULL = -2, FLOVER_E_NOMEM = -3, FLOVER_E_STATE = -4, FLOVER_E_HIP = -5 };
enum { FLOVER_ARCH_GPT = 0, FLOVER_ARCH_LLAMA = 1 };
enum { FLOVER_F32 = 0, FLOVER_F16 = 1, FLOVER_BF16 = 2 };
/* flover_config.shuffle_mode */
enum { FLOVER_SHUFFLE_SLOTS = 0, FLOVER_SHUFFLE_OFF = 1, FLOVER_SHUFFLE_BY_LENGTH = 2 };

/* slot states reported by flover_get_state */
enum { FLOVER_SLOT_EMPTY = 0, FLOVER_SLOT_READY = 1, FLOVER_SLOT_LIVE = 2, FLOVER_SLOT_DEAD = 3 };

typedef struct flover_ctx flover_ctx;

/* Model type, inference data type and request meta-specification read at launch (Section V-A). */
typedef struct flover_config {
  int32_t arch;            /* FLOVER_ARCH_*: GPT = LayerNorm, learned positions, biases, tanh-GELU;
                              LLAMA = RMSNorm, rotary embedding (rotate-half, pairs (i, i+d/2)), SwiGLU, no biases */
  int32_t dtype;           /* FLOVER_F32 | FLOVER_F16 | FLOVER_BF16: weights, KV cache and GEMM inputs */
  int32_t n_layer, hidden, n_head, head_dim, ffn, vocab;   /* hidden == n_head * head_dim; head_dim in {64,128};
                                                               n_head % 4 == 0; hidden, ffn multiples of 32 */
  int32_t max_seq;         /* slot capacity in tokens */
  int32_t max_concurrency; /* number of slots = most requests generating at once (Section V-A) */
  int32_t eos_id;          /* token that ends a request; -1 = none (Section IV) */
  int32_t shuffle_mode;    /* FLOVER_SHUFFLE_*: SLOTS = Algorithm 3 on the 0/1 occupancy array (fewest slots moved);
                              OFF = the variant without memory shuffle (Section VI-D): finished slots stay inside the
                              window as holes that the kernels still cover; BY_LENGTH = Algorithm 3 with every valid
                              entry weighted by its cached rows + 1 (the listing sums arr[i], so it already allows
                              weights): the window that leaves the fewest cached rows outside, i.e. fewest bytes moved */
  int32_t async_preprocess; /* 0: flover_add_request returns when the context cache is complete (pre-processing runs on
                               `stream`).  Non-zero: the library creates two more streams (default priority), each with
                               its own set of row buffers for the context decoder, as the paper runs pre-processing beside
                               the inference stream (Section V-B); arriving requests take them in turn, so the context
                               passes of two requests run side by side; flover_add_request returns once the passes are
                               enqueued and may be called from another thread while flover_step / flover_reorder_evict run.
                               1: the request joins the first flover_step that finds its cache complete (the iterations
                               overlap with pre-processing; which iteration a request joins depends on timing).
                               2: the next flover_step waits, on its stream, for the caches of the requests it admits, so
                               every request joins exactly where it would with 0 (same schedule, same results); only the
                               context passes of requests that arrive together overlap.  Tokens and logits of every
                               request are the same in all three modes. */
  float norm_eps;
  float rope_theta;
  void* stream;            /* hipStream_t the library enqueues on; NULL = the null stream */
  void* arena;             /* [device] 256-byte aligned; owned by the caller, must outlive the context */
  uint64_t arena_bytes;    /* >= flover_query_arena_bytes() */
} flover_config;

/* [device] pointers, dtype elements, every linear weight [out][in] with the input index contiguous,
 * per-layer tensors stacked over layers in the leading dimension.  Unused entries (by arch) may be NULL.
 * flover_init copies (and re-tiles) all of them into the arena; the caller may free them afterwards. */
typedef struct flover_weights {
  const void* wte;    /* [vocab][hidden] token embedding (GPT: also the output projection) */
  const void* wpe;    /* GPT [max_seq][hidden] learned positions */
  const void* ln1_g;  /* [L][hidden] */
  const void* ln1_b;  /* GPT [L][hidden] */
  const void* wqkv;   /* [L][3*hidden][hidden], rows: q heads, k heads, v heads */
  const void* bqkv;   /* GPT [L][3*hidden] */
  const void* wo;     /* [L][hidden][hidden] */
  const void* bo;     /* GPT [L][hidden] */
  const void* ln2_g;  /* [L][hidden] */
  const void* ln2_b;  /* GPT [L][hidden] */
  const void* w1;     /* [L][ffn][hidden]  GPT: first MLP matrix; LLAMA: gate */
  const void* b1;     /* GPT [L][ffn] */
  const void* wu;     /* LLAMA [L][ffn][hidden] up */
  const void* w2;     /* [L][hidden][ffn]  second MLP matrix / down */
  const void* b2;     /* GPT [L][hidden] */
  const void* lnf_g;  /* [hidden] */
  const void* lnf_b;  /* GPT [hidden] */
  const void* wlm;    /* LLAMA [vocab][hidden] output projection */
} flover_weights;

/* Upper bound of device memory for this configuration (Buffer Manager's calculation, Section V-A).
 * Only the shape fields of cfg are read. */
int32_t flover_query_arena_bytes(const flover_config* cfg, uint64_t* out_bytes);

/* Launcher + Buffer Manager + scheduler start (Section V-A, Algorithm 1's first lines): lays out the arena
 * (re-tiled weights, KV cache [L][K|V][slot][head][max_seq][head_dim], per-iteration buffers), copies the
 * weights in, creates the request and inference queues.  Blocks until the copies are done.
 * Errors: INVAL (bad shape / NULL required weight / misaligned arena), NOMEM (arena too small), HIP. */
int32_t flover_init(const flover_config* cfg, const flover_weights* w, flover_ctx** out_ctx);

/* Layer-by-layer hand-over, for models whose natural-layout copy would not fit in device memory beside the arena
 * (the Buffer Manager sizes everything from the model configuration, Section V-A; the 30B shape holds 65 GB of weights).
 * flover_init with EVERY per-layer pointer of `weights` NULL (ln1_g .. b2; the global tensors wte, wpe, lnf_*, wlm are
 * still taken) leaves the layers unloaded; flover_set_layer_weights then copies and re-tiles layer `layer` from w, whose
 * per-layer pointers address that ONE layer's tensors (its global pointers are ignored), and returns when the copy is
 * complete, so the caller may reuse its buffers.  Requests are refused (STATE) until every layer has been set; a layer
 * may be set again while no request is in flight.  Errors: INVAL (layer out of range, missing tensor), STATE, HIP. */
int32_t flover_set_layer_weights(flover_ctx* ctx, int32_t layer, const flover_weights* w);

/* Waits for the library's streams, releases what the context owns on the host (staging, events, the pre-processing
 * stream).  The arena is the caller's and is not touched.  ctx == NULL is a no-op. */
int32_t flover_destroy(flover_ctx* ctx);

/* Text of the last error on ctx (ctx == NULL: of the calling thread's last failed flover_init / query /
 * kernel-level call).  Owned by the library, valid until the next failing call. */
const char* flover_last_error(const flover_ctx* ctx);

/* Body of Algorithm 1 for one request (Section V-B): assign the slot adjacent to the live region
 * (hi if hi < max_concurrency, else lo-1; an empty region restarts at slot 0), copy the prompt [host] to
 * the device, run pre-processing -- the context decoder fills the slot's KV cache for prompt positions
 * 0..prompt_len-2 -- and put the request into the inference queue.  It joins the fused stream at the next
 * flover_step, which feeds prompt[prompt_len-1].  If no adjacent slot is free the request waits in the
 * request queue (FIFO) and is pre-processed by a later flover_step; *out_slot = -1 then.
 * With async_preprocess the context passes are only enqueued (on one of the library's pre-processing streams) and the
 * request joins the first flover_step that finds them complete (mode 1; a flover_step with nothing else to generate
 * waits for the oldest one) or the next flover_step, which waits for them (mode 2).  Threads: every call takes the context's scheduler lock; with async_preprocess flover_step releases it while
 * the GPU works, so ONE other thread may call flover_add_request beside the thread that drives flover_step /
 * flover_reorder_evict (the paper's pre-processing and inference threads, Section V-A).  Without async_preprocess
 * calls from several threads are serialised.
 * The prompt is copied before return.  Errors: INVAL (prompt_len < 1, max_new_tokens < 1,
 * prompt_len + max_new_tokens > max_seq, token out of range, req_id already waiting or live). */
int32_t flover_add_request(flover_ctx* ctx, uint64_t req_id, const int32_t* prompt, int32_t prompt_len,
                           int32_t max_new_tokens, int32_t* out_slot);

typedef struct flover_step_out {
  int32_t capacity;     /* in: entries each [host] array below can hold (>= max_concurrency is always enough) */
  int32_t n_live;       /* out: requests advanced in this iteration */
  uint64_t* req_id;     /* [host] out, ascending slot order */
  int32_t* slot;        /* [host] out */
  int32_t* token;       /* [host] out: the greedy token (argmax of the fp32 logits, lowest index on ties) */
  int32_t* finished;    /* [host] out: 1 if the request ended with this token (EOS or length limit, Section IV) */
  float* logits;        /* [device] optional, caller-owned [capacity][vocab] fp32: row i = logits of entry i */
} flover_step_out;

/* One iteration of Algorithm 2 (Section V-C) up to and including the detection of finished requests:
 * waiting requests take free adjacent slots and are pre-processed; every ready request is admitted
 * (Update(offset,size)); ONE launch per operation covers all live requests -- embedding, norms, the weight
 * GEMMs, rotary + KV append, ragged attention over each request's own cache length, MLP, output projection,
 * argmax.  Returns after the tokens are on the host.  n_live == 0 is not an error.  Finished requests keep
 * their slot (state DEAD) until flover_reorder_evict.  Errors: INVAL (capacity too small), HIP. */
int32_t flover_step(flover_ctx* ctx, flover_step_out* out);

typedef struct flover_reorder_out {
  int32_t capacity;        /* in: entries each [host] array can hold; must be >= max_concurrency */
  int32_t n_evicted;       /* out */
  uint64_t* evicted_req_id;/* [host] out, ascending slot order */
  int32_t mem_offset;      /* out: Algorithm 3's result, relative to the old window start */
  int32_t new_lo;          /* out: window start after the call (buffer offset, in slots) */
  int32_t new_size;        /* out: window size after the call (buffer size, in slots) */
  int32_t min_cost;        /* out: Algorithm 3's cost = number of slots that had to move */
  int32_t n_moves;         /* out */
  int32_t* move_src;       /* [host] out, absolute slot indices */
  int32_t* move_dst;       /* [host] out */
  int64_t bytes_moved;     /* out: read + written bytes of KV rows [0,len) of the moved slots */
} flover_reorder_out;

/* Pipelined form of flover_step (token return without a host wait per iteration; Algorithm 2's loop keeps the GPU
 * busy while the previous iteration's tokens travel back).  flover_step_submit admits ready requests and enqueues one
 * iteration; the tokens it will choose stay on the device as the next iteration's inputs.  Only without an
 * end-of-sequence token (eos_id < 0) is it known at submission who finishes (budget exhausted), so the scheduler
 * state -- lengths, budgets, DEAD marks -- advances at once and flover_reorder_evict / flover_add_request /
 * the next flover_step_submit may follow immediately (all work is ordered on the stream; flover_reorder_evict does not
 * wait then).  *n_live_out = rows of the iteration; 0 means nothing was enqueued (and nothing is to be collected).
 * logits: optional [device][n_live][vocab] fp32, written by this iteration; must stay valid until it is collected.
 * flover_step_collect waits for the OLDEST submitted iteration and returns what flover_step would have: rows in
 * ascending slot order at submission time, their tokens, and the finished flags decided at submission.
 * At most 3 iterations may be outstanding.  Errors: STATE (eos_id >= 0; flover_step while iterations are outstanding;
 * collect with nothing submitted), FULL (4th outstanding iteration), INVAL, HIP. */
int32_t flover_step_submit(flover_ctx* ctx, float* logits, int32_t* n_live_out);
int32_t flover_step_collect(flover_ctx* ctx, flover_step_out* out);

/* FindAndEvict's removal, Algorithm 3 and the memory shuffle (Algorithm 2's last lines, Section V-D).
 * Frees DEAD slots; over the 0/1 occupancy of the old window finds, with the sliding window of Algorithm 3
 * (first window scored too, lowest offset on ties), the region of size #valid that leaves the fewest valid
 * slots outside; copies, in one launch, the KV rows [0,len) of each outside slot into a hole inside (i-th hole
 * ascending <- i-th outside slot ascending) and moves the scheduler's record with it.  Waits for the copy.
 * With FLOVER_SHUFFLE_OFF only the empty ends of the window are dropped.  Safe to call after every step. */
int32_t flover_reorder_evict(flover_ctx* ctx, flover_reorder_out* out);

/* ------------------------------------------------------------------ inspection and test hooks (not in the paper)
 * Read-only views of the scheduler and the cache, and two hooks that let a test steer a stream. */

/* End a request as if it had produced EOS; overwrite the token a live request feeds in the next iteration
 * (teacher forcing, to re-synchronise a comparison after a near tie).  A request may be ended before it has joined an
 * iteration, also while its context passes are still queued (async_preprocess): the next flover_reorder_evict frees
 * the slot, and whatever is enqueued for that slot afterwards -- a shuffle copy into it, the context passes of its
 * next tenant on either pre-processing stream -- is ordered behind the passes already queued for it. */
int32_t flover_mark_finished(flover_ctx* ctx, uint64_t req_id);
int32_t flover_set_next_token(flover_ctx* ctx, uint64_t req_id, int32_t token);

/* Read-only snapshot.  lo_hi_wait [host][3] = window start, window end, requests waiting for a slot;
 * the other [host] arrays hold max_concurrency entries (any may be NULL). */
int32_t flover_get_state(const flover_ctx* ctx, int32_t* lo_hi_wait, int32_t* state, uint64_t* req_id, int32_t* len,
                         int32_t* next_token, int32_t* generated);

/* [device] address and byte strides of the KV cache inside the arena, for inspection by tests:
 * element (layer, k_or_v, slot, head, pos, i) lives at base + ((((layer*2+k_or_v)*C + slot)*n_head + head)*max_seq
 * + pos)*head_dim + i elements. */
int32_t flover_get_kv_cache(const flover_ctx* ctx, void** base, uint64_t* bytes);

/* Kernel launches issued by the most recent flover_step (Table I: one launch per operation however many
 * requests are live). */
int32_t flover_last_step_launches(const flover_ctx* ctx, int32_t* n);

/* ------------------------------------------------------------------ measurement hooks (not in the paper)
 * Used by the benchmark and by profiler runs only; nothing in the method depends on them. */

/* Like flover_add_request, but the slot's context cache (KV rows
 * [0, context_len)) is taken to be whatever the slot already holds -- no pre-processing kernels run.  The request
 * feeds next_token at position context_len in the next flover_step.  Meant for profiler runs in which every launch
 * must be a fused-iteration launch; results are meaningless numerically unless the caller filled the cache.
 * Errors: INVAL (context_len < 0, context_len + 1 + max_new_tokens > max_seq, bad token, duplicate id),
 * FULL (no adjacent slot free or requests already waiting; this call never queues). */
int32_t flover_add_request_cached(flover_ctx* ctx, uint64_t req_id, int32_t context_len, int32_t next_token,
                                  int32_t max_new_tokens, int32_t* out_slot);

/* Kernel timing with HIP events on the context's stream (measurement aid, not in the paper): the events take the
 * start and end time stamps of the timed kernel's own dispatch.
 * level 0 = off; 1 = sampled: the attention streaming kernel of one layer in eight (layers 0, 8, 16, ...) in every
 * iteration, and in every fourth iteration the four weight GEMMs of the middle layer (n_layer / 2) and the output
 * projection -- a timed dispatch costs about as much as a small kernel, and the layers' launches are alike;
 * 2 = the attention kernel of every layer and every weight GEMM.  The shuffle copy is timed at levels 1 and 2 (events
 * recorded before and after its launch).
 * Iterations submitted with flover_step_submit are timed too (added up when they are collected).  Setting the level
 * clears the totals.  flover_get_profile returns, for one kind, the summed duration (ms), the number of TIMED launches
 * and the summed algorithmic bytes of those launches: for attention the K and V rows [0,len) of every row; for a GEMM
 * the weight matrix; for the shuffle copy bytes read + written. */
enum { FLOVER_PROF_ATTENTION = 0, FLOVER_PROF_GEMM_QKV = 1, FLOVER_PROF_GEMM_OUT = 2, FLOVER_PROF_GEMM_FF1 = 3,
       FLOVER_PROF_GEMM_FF2 = 4, FLOVER_PROF_GEMM_LM = 5, FLOVER_PROF_COMPACT = 6, FLOVER_PROF_KINDS = 7 };
int32_t flover_set_profile(flover_ctx* ctx, int32_t level);
int32_t flover_get_profile(const flover_ctx* ctx, int32_t kind, double* ms, int64_t* launches, int64_t* bytes);

/* Plain device-to-device copy kernel of a known size (bytes % 16 == 0): the reference against which profiler byte
 * counters (FETCH_SIZE / WRITE_SIZE) are scaled.  Measurement aid only. */
int32_t flover_k_copy_probe(void* dst, const void* src, uint64_t bytes, void* stream);

/* ------------------------------------------------------------------ operation-level entry points
 * The same kernels the step uses, callable on caller-owned buffers (micro-benchmarks, unit parity).
 * All enqueue on `stream` and return without waiting unless stated. */

/* Algorithm 3 on a [host] occupancy array (0 = empty); host only. */
int32_t flover_k_find_window(const int32_t* arr, int32_t n, int32_t* mem_offset, int32_t* min_cost, int32_t* non_zero);

/* Bytes of [device] workspace flover_k_decode_attention needs for up to M rows of length <= max_len. */
int32_t flover_k_attention_workspace_bytes(int32_t M, int32_t n_head, int32_t head_dim, int32_t max_len, uint64_t* out);

/* Ragged masked self-attention of one decode iteration (the attention inside Algorithm 2's "..."):
 * for every row m and head h:  out[m][h] = softmax(q[m][h] . K[slot[m]][h][0..len[m]) / sqrt(head_dim)) V[...],
 * fp32 scores, softmax and accumulation, result rounded to dtype.
 * q, out [device][M][n_head][head_dim]; kcache, vcache [device][C][n_head][S][head_dim]; slot, len [host][M]
 * (1 <= len[m] <= S, 0 <= slot[m] < C); workspace [device].  The host arrays are consumed before return
 * (this call waits for its small host-to-device copy, not for the kernels). */
int32_t flover_k_decode_attention(int32_t dtype, const void* q, const void* kcache, const void* vcache,
                                  const int32_t* slot, const int32_t* len, int32_t M, int32_t C, int32_t n_head,
                                  int32_t head_dim, int32_t S, void* out, void* workspace, uint64_t workspace_bytes,
                                  void* stream);

/* flover_k_decode_attention for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same kernels, same arguments and results, but the workspace is a
 * FLOVER_NOALLOC_SCRATCH_BYTES array inside the library's device image (one copy per GPU, held until the process ends)
 * and the row descriptors travel as a kernel argument, so the call performs no allocation and no host-to-device copy;
 * it only enqueues on `stream` and returns.  slot, len [host][M] are consumed before return.  The device that `stream`
 * belongs to must be current.  Limits: M <= FLOVER_NOALLOC_MAX_ROWS and
 * flover_k_attention_workspace_bytes(M, n_head, head_dim, max(len)) <= FLOVER_NOALLOC_SCRATCH_BYTES, else NOMEM with
 * the sizes in flover_last_error(NULL).  Every call on a GPU uses that GPU's one array: calls that overlap on one GPU
 * (two streams, two threads) race; calls ordered on one stream do not.  Nothing in the array has to start at zero. */
#define FLOVER_NOALLOC_SCRATCH_BYTES (16u << 20)
#define FLOVER_NOALLOC_MAX_ROWS 256
int32_t flover_k_decode_attention_noalloc(int32_t dtype, const void* q, const void* kcache, const void* vcache,
                                          const int32_t* slot, const int32_t* len, int32_t M, int32_t C, int32_t n_head,
                                          int32_t head_dim, int32_t S, void* out, void* stream);

/* Bytes of [device] workspace flover_k_compact needs for n_moves moves. */
int32_t flover_k_compact_workspace_bytes(int32_t n_moves, uint64_t* out);

/* The memory-shuffle copy (Section V-D): for every move i and every (layer, K|V, head), copy rows [0,len[i]) of slot
 * src[i] to slot dst[i] in cache [device][L][2][C][n_head][S][head_dim] (elem_bytes per element), all in one launch.
 * src, dst, len [host][n_moves]; source and destination slot sets must be disjoint (INVAL otherwise). */
int32_t flover_k_compact(void* cache, int32_t L, int32_t C, int32_t n_head, int32_t S, int32_t head_dim,
                         int32_t elem_bytes, const int32_t* src, const int32_t* dst, const int32_t* len,
                         int32_t n_moves, void* workspace, uint64_t workspace_bytes, void* stream);

/* Weight GEMM of the fused rows: y[M][N] (fp32) = x[M][K] . W[N][K]^T, fp32 accumulation (MFMA for the 16-bit
 * dtypes).  W is first re-tiled into `w_tiled` (flover_k_gemm_tiled_bytes bytes, [device]) by flover_k_gemm_retile;
 * flover_k_gemm then streams the tiled copy.  x [device][Mpad][K]: rows up to M rounded up to a multiple of 128 (of 256 when
 * M > 128) must be readable (their contents do not matter);
 * workspace holds the split-K partial sums.  K % 32 == 0.  y == NULL leaves the result as partial sums in the
 * workspace (timing the streaming kernel alone). */
int32_t flover_k_gemm_tiled_bytes(int32_t dtype, int32_t N, int32_t K, uint64_t* out);
/* [host only] K slicing of the weight GEMM: *slices partial sums, each over *k_blocks_per_slice blocks of 32 input
 * features (the last slice may be shorter).  context_rows == 0: the fused iteration's slicing, a function of (dtype, N,
 * K) alone, so that a row's result cannot depend on how many rows are live; context_rows > 0: the slicing of a
 * pre-processing pass of that many rows of one request (at most 16 slices; a context may use fewer when its
 * partial-sum buffer, sized for the iteration, holds fewer at that row count). */
int32_t flover_k_gemm_plan(int32_t dtype, int32_t N, int32_t K, int32_t context_rows, int32_t* slices,
                           int32_t* k_blocks_per_slice);
int32_t flover_k_gemm_workspace_bytes(int32_t dtype, int32_t M, int32_t N, int32_t K, uint64_t* out);
int32_t flover_k_gemm_retile(int32_t dtype, const void* W, int32_t N, int32_t K, void* w_tiled, void* stream);
int32_t flover_k_gemm(int32_t dtype, const void* x, const void* w_tiled, int32_t M, int32_t N, int32_t K, float* y,
                      void* workspace, uint64_t workspace_bytes, void* stream);

/* Input half of a gated MLP over the fused rows (the MLP call of Algorithm 2 / Section V-C for LLaMA-style models):
 * act[M][F] = silu(x . Wgate^T) * (x . Wup^T), fp32 accumulation, rounded once to the model dtype -- the contraction
 * and the activation in one launch, as the fused iteration runs it.  16-bit dtypes only (fp16, bf16); F % 32 == 0 and
 * K % 512 == 0, INVAL otherwise (the step then uses flover_k_gemm's kernels and a separate activation).
 * flover_k_gated_retile writes both matrices ([device][F][K] each) into w_tiled ([device],
 * flover_k_gemm_tiled_bytes(dtype, 2F, K) bytes) with gate and up columns interleaved in tiles of 16;
 * flover_k_gated_mlp streams that copy.  x [device][Mpad][K] row-major with the rows flover_k_gemm asks for readable;
 * act [device][M][F] row-major, model dtype.
 * context_pass == 0, the fused iteration: a row's result depends on that row of x alone, not on M.  Up to 128 rows (64
 * when F > 16384) it is one launch; above that the two halves of K go through `workspace` as partial sums and the
 * activation is a second launch, with the same result bit for bit.
 * context_pass != 0, the M rows of one request's pre-processing pass (Section V-B): K is sliced by M as well, as
 * flover_k_gemm_plan reports for context rows; with one slice and more than 128 rows the activation is the epilogue of
 * the 256-row-block kernel, otherwise partial sums and a second launch.
 * workspace [device], flover_k_gated_workspace_bytes bytes (0 where one launch serves the fused iteration); NOMEM if
 * it is needed and smaller. */
int32_t flover_k_gated_retile(int32_t dtype, const void* Wgate, const void* Wup, int32_t F, int32_t K, void* w_tiled,
                              void* stream);
int32_t flover_k_gated_workspace_bytes(int32_t dtype, int32_t M, int32_t F, int32_t K, uint64_t* out);
int32_t flover_k_gated_mlp(int32_t dtype, const void* x, const void* w_tiled, int32_t M, int32_t F, int32_t K,
                           int32_t context_pass, void* act, void* workspace, uint64_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FLOVER_H */
