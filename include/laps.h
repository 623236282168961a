/*
 * laps.h - C ABI of the MI355X (gfx950) ragged-prefill hot path behind LAPS-style
 * length-aware prefill scheduling.
 *
 * The paper (LAPS, "A Length-Aware-Prefill LLM Serving System") defines the scheduling:
 * requests are classified by prompt length into a short and a long queue (Section 3.2,
 * "Mutual exclusion"), short requests are padded into a grid of (length, batch size)
 * buckets, one captured graph per bucket (Section 3.1, "Graph capture and bucketization"),
 * batches are matched to a captured shape under a memory budget or fall back to the
 * standard path (Algorithm 1), and long requests advance alone in fixed-size chunks
 * (Section 3.2, deadline-free mode).  What runs under that schedule is the prefill forward:
 * "incremental causal attention and FFN" over L new tokens that also attend to H cached
 * historical tokens (Section 2.1, latency model) - one decoder layer stack of the Qwen2.5
 * family the paper serves (Section 4.1).  This library is that forward plus the integer plan.
 *
 * Conventions
 *   - Every function returns LAPS_OK (0) or a negative LAPS_E* code; laps_last_error()
 *     gives a thread-local message for the last failure.  Nothing throws across the ABI.
 *   - "dev" pointers are device (HBM) addresses on the context's GPU; "host" pointers are
 *     ordinary host memory.  The caller owns every buffer it passes.  The library owns
 *     laps_ctx, laps_plan, laps_graph and what those allocate internally.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  laps_prefill_*,
 *     laps_graph_stage and laps_graph_replay only enqueue work: they never synchronise the
 *     stream and never allocate device memory.  The kernels they enqueue read the device arrays
 *     passed in (lengths, page tables, inputs, weights, pools) when they run, not when the call
 *     returns: keep those arrays valid and unchanged until that stream work has completed.
 *     Arrays written by work on another stream must be complete before the call (event or
 *     synchronisation on the caller's side): a page table read before it is written makes the
 *     K/V append write wherever the stale entries point.  The kernels bound what the VALUES of these
 *     arrays can reach: lengths are cut to the rows a sequence owns, a sequence whose rows do not
 *     lie inside the batch is skipped, a prefix longer than the page table can address is cut to
 *     it, and - once laps_ctx_set_pool_pages has said how many pages the pools hold - page ids
 *     outside the pools are treated as unset.  The array SIZES are the caller's responsibility.
 *   - bf16 = upper 16 bits of an IEEE float32, round-to-nearest-even on conversion.
 *   - Layer math (all accumulation fp32): r = rmsnorm(x; ln1); [q,k,v] = r W_qkv^T (+b);
 *     rotate-half RoPE with theta on q,k at absolute position prefix_len+t; causal grouped-
 *     query attention over cached prefix + new tokens, scale 1/sqrt(head_dim), query head h
 *     uses kv head h / (n_q/n_kv); x1 = x + attn W_o^T; r2 = rmsnorm(x1; ln2);
 *     y = x1 + (silu(r2 W_g^T) * (r2 W_u^T)) W_d^T.  The residual stream is fp32; q, k, v,
 *     normed rows, attention output and the MLP activation are stored as bf16.
 *
 * KV cache layout (per layer; page_size = 16 tokens):
 *     k_pool: [n_pages][n_kv_heads][16 tokens][head_dim]  bf16   (keys already rotated)
 *     v_pool: [n_pages][n_kv_heads][head_dim][16 tokens]  bf16   (transposed inside the page)
 *   page_table[s][j] is the pool page holding logical positions 16j..16j+15 of sequence s.
 *   Use laps_kv_scatter / laps_kv_gather to move token-major K/V in and out of pools.
 */
#ifndef LAPS_H
#define LAPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LAPS_OK 0
#define LAPS_EINVAL (-1) /* bad shape, unsorted grid, new_len < 1, prefix_len < 0, NULL where not allowed */
#define LAPS_ENOMEM (-2) /* host or device allocation failed, or workspace too small */
#define LAPS_EHIP (-3)   /* a HIP call failed; laps_last_error() names it */

#define LAPS_PAGE 16

typedef struct laps_ctx laps_ctx;
typedef struct laps_plan laps_plan;
typedef struct laps_graph laps_graph;

/* Shape of one decoder layer stack.  Requirements: head_dim in {64, 128}; n_q_heads a
 * multiple of n_kv_heads; hidden, n_q_heads*head_dim and intermediate multiples of 64;
 * (n_q_heads + 2 n_kv_heads)*head_dim, hidden and 2*intermediate multiples of 128;
 * page_size == 16. */
typedef struct laps_model_cfg {
    int32_t hidden, n_q_heads, n_kv_heads, head_dim, intermediate, n_layers;
    int32_t page_size;    /* must be LAPS_PAGE */
    int32_t has_qkv_bias; /* 0: b_qkv ignored */
    float rope_theta;     /* e.g. 1e6 */
    float rms_eps;        /* e.g. 1e-6 */
} laps_model_cfg;

/* Device pointers to one layer's bf16 weights, all [out, in] row-major:
 * ln1_w [hidden]; w_qkv [(n_q+2n_kv)*hd, hidden] (q heads, then k heads, then v heads);
 * b_qkv [(n_q+2n_kv)*hd] or NULL; w_o [hidden, n_q*hd]; ln2_w [hidden];
 * w_gate_up [2*intermediate, hidden] as written by laps_pack_gate_up; w_down [hidden, intermediate]. */
typedef struct laps_layer_weights {
    const void *ln1_w, *w_qkv, *b_qkv, *w_o, *ln2_w, *w_gate_up, *w_down;
} laps_layer_weights;

/* ------------------------------------------------------------------ bucket plan (host, integer)
 * Section 3.2 "Mutual exclusion" (classification by length), Section 3.1 (bucket grid, padding
 * to a bucket, grouping by the same bucket), Algorithm 1 (captured shape with depth >= batch
 * depth within the budget, else the standard path), deadline-free mode (fixed-size long chunks).
 *
 * Rules: request i is SHORT iff new_len[i] <= short_max_len (new tokens only; the cached prefix
 * does not count), else LONG.  A short request goes to the smallest length bucket >= new_len.
 * Per length bucket L_b (ascending), its requests (arrival order) are covered by graph depths
 * from `depths` with depth*L_b <= token_budget, choosing the multiset that minimises (number of
 * launches, total padded rows) and prefers larger depths first; batches are emitted larger depth
 * first and filled in arrival order.  If no depth fits the budget the bucket's requests are
 * split, in order, into the fewest contiguous groups whose un-padded token total is within the
 * budget (a single request may exceed it) and marked graph_ok = 0 (run un-captured, un-padded).
 * A long request is cut into ceil(new_len/long_chunk) chunks, all long_chunk except the last. */
typedef struct laps_plan_params {
    int32_t short_max_len;      /* >= 1 and <= len_buckets[n_len_buckets-1] */
    int32_t n_len_buckets;
    const int32_t* len_buckets; /* host, strictly ascending, >= 1 */
    int32_t n_depths;
    const int32_t* depths;      /* host, strictly ascending, >= 1 */
    int32_t token_budget;       /* M: padded new tokens one captured graph may hold, >= 1 */
    int32_t long_chunk;         /* C_l >= 1 */
} laps_plan_params;

/* new_len, prefix_len: host arrays [n_req]; new_len >= 1, prefix_len >= 0; n_req >= 0.
 * On success *out is a plan to be released with laps_plan_free.  Deterministic, no GPU use. */
int laps_plan_buckets(const laps_plan_params* params, int32_t n_req, const int32_t* new_len,
                      const int32_t* prefix_len, laps_plan** out);
void laps_plan_free(laps_plan* plan);
/* Accessors return host pointers valid until laps_plan_free (0 / NULL for a NULL plan). */
int32_t laps_plan_n_requests(const laps_plan* plan);
const int32_t* laps_plan_req_class(const laps_plan* plan);   /* [n_req] 0 short, 1 long */
const int32_t* laps_plan_req_bucket(const laps_plan* plan);  /* [n_req] length-bucket index, -1 if long */
const int32_t* laps_plan_req_batch(const laps_plan* plan);   /* [n_req] batch index, -1 if long */
const int32_t* laps_plan_req_row(const laps_plan* plan);     /* [n_req] slot inside its batch, -1 if long */
int32_t laps_plan_n_batches(const laps_plan* plan);
const int32_t* laps_plan_batch_len_bucket(const laps_plan* plan); /* [n_batches] L_b (tokens) */
const int32_t* laps_plan_batch_depth(const laps_plan* plan);      /* [n_batches] graph depth, or group size if graph_ok=0 */
const int32_t* laps_plan_batch_graph_ok(const laps_plan* plan);   /* [n_batches] */
const int32_t* laps_plan_batch_req_offset(const laps_plan* plan); /* [n_batches+1] into batch_req_ids */
const int32_t* laps_plan_batch_req_ids(const laps_plan* plan);    /* request ids, batch by batch */
int32_t laps_plan_n_long(const laps_plan* plan);
const int32_t* laps_plan_long_req(const laps_plan* plan);          /* [n_long] request id */
const int32_t* laps_plan_long_chunk_offset(const laps_plan* plan); /* [n_long+1] into long_chunk_len */
const int32_t* laps_plan_long_chunk_len(const laps_plan* plan);    /* chunk lengths, request by request */

/* ------------------------------------------------------------------ context
 * Binds a model shape to the current HIP device and builds the fp64-evaluated cos/sin table
 * for positions 0..max_positions-1 (device allocation; freed by laps_ctx_destroy). */
int laps_ctx_create(const laps_model_cfg* cfg, int32_t max_positions, laps_ctx** out);
void laps_ctx_destroy(laps_ctx* ctx);
/* Optional guard for the calls that follow on this context: the K/V pools they are given hold n_pages
 * pages each.  Page-table entries outside [0, n_pages) are then treated like unset (-1) entries - the
 * token's K/V is not written and reads fall back to page 0 - instead of addressing memory outside
 * the pools.  0 switches the check off (the default: the library does not know the pools' size).  A
 * graph keeps the value that was set when it was captured.  EINVAL on NULL or a negative count. */
int laps_ctx_set_pool_pages(laps_ctx* ctx, int32_t n_pages);
/* Bytes of scratch laps_prefill_layer / laps_prefill_stack need for up to max_tokens rows
 * (padded rows count) and max_seqs sequences.  0 on bad arguments. */
size_t laps_workspace_bytes(const laps_ctx* ctx, int32_t max_tokens, int32_t max_seqs);
/* The same figure from a model shape alone (host only; 0 on an unsupported shape).  A workspace of this size serves
 * every call with at most max_tokens rows and max_seqs sequences. */
size_t laps_workspace_bytes_for(const laps_model_cfg* cfg, int32_t max_tokens, int32_t max_seqs);

/* Interleaves gate and up projection rows in blocks of 32 so that one GEMM produces both
 * halves of the SwiGLU for the same output column in one tile: dst rows [64b, 64b+32) are
 * gate rows [32b, 32b+32), dst rows [64b+32, 64b+64) are up rows [32b, 32b+32).
 * w_gate_dev, w_up_dev: bf16 [intermediate, hidden]; dst_dev: bf16 [2*intermediate, hidden]. */
int laps_pack_gate_up(laps_ctx* ctx, const void* w_gate_dev, const void* w_up_dev, void* dst_dev, void* stream);

/* Token-major K/V <-> paged pools.  Sequence s owns rows cu_dev[s]..cu_dev[s+1]-1 of the packed
 * arrays ([n_tokens, n_kv_heads, head_dim] bf16), which map to its logical positions
 * start_pos_dev[s], start_pos_dev[s]+1, ...  page_table_dev: int32 [n_seq, max_pages]. */
int laps_kv_scatter(laps_ctx* ctx, int32_t n_seq, int32_t n_tokens, const int32_t* cu_dev,
                    const int32_t* start_pos_dev, const int32_t* page_table_dev, int32_t max_pages,
                    const void* k_src_dev, const void* v_src_dev, void* k_pool_dev, void* v_pool_dev, void* stream);
int laps_kv_gather(laps_ctx* ctx, int32_t n_seq, int32_t n_tokens, const int32_t* cu_dev,
                   const int32_t* start_pos_dev, const int32_t* page_table_dev, int32_t max_pages,
                   const void* k_pool_dev, const void* v_pool_dev, void* k_dst_dev, void* v_dst_dev, void* stream);

/* ------------------------------------------------------------------ prefill forward
 * One decoder layer over a packed ragged batch (Section 2.1: L new tokens attending to H cached
 * ones; Section 3.2: the "standard prefill kernel" that un-captured batches and long chunks use).
 *   n_seq sequences, n_tokens rows.  Sequence s owns rows cu_seqlens_dev[s] .. cu_seqlens_dev[s+1]-1;
 *   seq_len_dev (nullable) gives how many of those rows are real tokens (the rest are padding and
 *   are ignored: no KV write, output undefined); NULL means all of them.
 *   prefix_len_dev[s] = H_s cached tokens; page_table_dev[s][0..ceil((H_s+L_s)/16)) must be valid
 *   pages of this layer's pools.  The layer reads the prefix from the pools and appends the new
 *   tokens' K and V at logical positions H_s .. H_s+L_s-1 (possibly starting mid-page).
 *   x_in_dev / x_out_dev: fp32 [n_tokens, hidden]; may alias each other.
 *   workspace_dev: >= laps_workspace_bytes(ctx, n_tokens, n_seq) bytes, 256-byte aligned.
 * Errors: EINVAL on NULL / non-positive sizes; ENOMEM if the workspace is too small; EHIP. */
int laps_prefill_layer(laps_ctx* ctx, const laps_layer_weights* w, int32_t n_seq, int32_t n_tokens,
                       const int32_t* cu_seqlens_dev, const int32_t* seq_len_dev, const int32_t* prefix_len_dev,
                       const int32_t* page_table_dev, int32_t max_pages, void* k_pool_dev, void* v_pool_dev,
                       const float* x_in_dev, float* x_out_dev, void* workspace_dev, size_t workspace_bytes,
                       void* stream);

/* cfg.n_layers layers in sequence.  w: host array [n_layers]; k_pools / v_pools: host arrays
 * [n_layers] of device pool pointers (one pool pair per layer, same page table for all layers). */
int laps_prefill_stack(laps_ctx* ctx, const laps_layer_weights* w, int32_t n_seq, int32_t n_tokens,
                       const int32_t* cu_seqlens_dev, const int32_t* seq_len_dev, const int32_t* prefix_len_dev,
                       const int32_t* page_table_dev, int32_t max_pages, void* const* k_pools, void* const* v_pools,
                       const float* x_in_dev, float* x_out_dev, void* workspace_dev, size_t workspace_bytes,
                       void* stream);

/* ------------------------------------------------------------------ prefill forward without a workspace argument
 * For callers that cannot allocate device memory or may not call anything that does: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, kernels and results as
 * laps_prefill_stack, with the workspace taken from a static device array inside the library
 * (laps_static_scratch_bytes() = 128 MiB per GPU, held from library load until the process ends; its address on the
 * context's device is resolved once, in laps_ctx_create).  The call itself allocates nothing, frees nothing and
 * never synchronises.  A batch whose workspace (laps_workspace_bytes) exceeds the array is rejected with LAPS_EINVAL
 * and a message naming both sizes: at the 32B layer shape that is a few hundred rows.  The context's device must be
 * current.  Every call on a GPU uses that GPU's one array (nothing in it has to start at zero: each region is
 * written before it is read within the call), so calls that overlap in time on one GPU - two streams, two threads,
 * two contexts - race on it and must be serialised by the caller; calls on one stream are ordered by the stream. */
size_t laps_static_scratch_bytes(void);
int laps_prefill_stack_static(laps_ctx* ctx, const laps_layer_weights* w, int32_t n_seq, int32_t n_tokens,
                              const int32_t* cu_seqlens_dev, const int32_t* seq_len_dev, const int32_t* prefix_len_dev,
                              const int32_t* page_table_dev, int32_t max_pages, void* const* k_pools,
                              void* const* v_pools, const float* x_in_dev, float* x_out_dev, void* stream);

/* ------------------------------------------------------------------ launch plans (host only, no device work)
 * What the library would launch for a shape; for tests of the launch arithmetic and for tuning.
 * laps_gemm_plan_info: the projection C[m,n] = A[m,k] W[n,k]^T with the epilogue the layer driver would ask for
 * (0 = K-slice partial sums, 1 = residual add, 2 = SwiGLU) and split_k as in laps_gemm_bf16 (0 = automatic).
 * out[7] = { tile rows, tile columns, K slices, K elements per slice, epilogue the kernel applies (0 when K is
 * split), slabs kept in flight per workgroup, workgroups }.
 * laps_attn_plan_info: the attention launch of a batch shape (n_tokens rows, n_seq sequences, page tables
 * max_pages wide).  out[6] = { query rows per workgroup, bound on the (sequence, row block) work items,
 * key-range splits (1 = none), fewest 64-key tiles a split is given, bytes of the work-item table, bytes of
 * the key-split partial results (0 if tables this narrow never split) }.
 * EINVAL on NULL or unsupported shapes. */
int laps_gemm_plan_info(int32_t m, int32_t n, int32_t k, int32_t split_k, int32_t epilogue, int32_t* out);
int laps_attn_plan_info(int32_t n_seq, int32_t n_tokens, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                        int32_t max_pages, int64_t* out);

/* ------------------------------------------------------------------ captured short buckets
 * Section 3.1: one graph per (length bucket L_b, depth B_d) with fixed operator topology and
 * variable memory contents.  The graph runs the whole stack on up to depth sequences of up to
 * len_bucket tokens each, held packed (sequence after sequence, no padding between them) in a
 * [depth*len_bucket, hidden] buffer; lengths, row offsets, prefix lengths and page table live in
 * staging buffers the graph owns and every kernel reads them from there, so a replay needs no node
 * updates.  Rows past the staged total are padding: their contents are never used and their output
 * rows are unspecified (kernels skip them wherever a whole row or row tile is padding).
 * laps_graph_capture allocates the staging buffers and workspace, runs one warm-up pass on the
 * stream with all slots empty, captures and instantiates.  It synchronises the stream. */
int laps_graph_capture(laps_ctx* ctx, const laps_layer_weights* w, int32_t len_bucket, int32_t depth,
                       int32_t max_pages, void* const* k_pools, void* const* v_pools, void* stream,
                       laps_graph** out);
/* Fills slots 0..n_real-1 (n_real <= depth; remaining slots become empty).  All pointers are
 * device pointers: seq_len_dev, prefix_len_dev [n_real] (a length is clamped to [0, len_bucket] on
 * the device); page_table_dev [n_real, max_pages] with row stride max_pages; x_rows_dev fp32
 * [n_rows, hidden], the sequences' rows packed in slot order, n_rows = the sum of the lengths
 * (0 <= n_rows <= depth*len_bucket, else LAPS_EINVAL).  x_rows_dev may be NULL with n_rows 0 when the caller
 * has written laps_graph_input() in place: those rows must then be complete before this call, which reads them.
 * Enqueues two kernels that prepare everything a replay needs besides the layers themselves: lengths, row
 * offsets and the attention's work-item table (one workgroup), then per row the token's position and cache slot,
 * the copy of its input, its RMSNorm with the first layer's gain, and the page-table copy.  A replay therefore
 * starts with the first projection; replaying again without staging repeats the same batch. */
int laps_graph_stage(laps_graph* g, int32_t n_real, const int32_t* seq_len_dev, const int32_t* prefix_len_dev,
                     const int32_t* page_table_dev, const float* x_rows_dev, int32_t n_rows, void* stream);
int laps_graph_replay(laps_graph* g, void* stream);
/* Device pointer to the graph's output rows, fp32 [depth*len_bucket, hidden], packed like the input; rows
 * past the staged total hold unspecified values.  Valid until destroy. */
const float* laps_graph_output(const laps_graph* g);
/* Device pointer to the graph's input rows (same shape) for callers that write inputs in place. */
float* laps_graph_input(laps_graph* g);
/* Enqueues a device-to-device copy of output rows [0, n_rows) into dst_dev (fp32 [n_rows, hidden]). */
int laps_graph_read_output(const laps_graph* g, int32_t n_rows, float* dst_dev, void* stream);
size_t laps_graph_device_bytes(const laps_graph* g); /* staging + workspace held by this graph */
void laps_graph_destroy(laps_graph* g);

/* ------------------------------------------------------------------ single kernels (tests, roofline)
 * C[M,N] (fp32, row-major) = A[M,K] (bf16 row-major) * W[N,K]^T (bf16 row-major).  K % 64 == 0,
 * N % 64 == 0.  `split_k` 0 = automatic choice of the number of K slices.  workspace_dev must hold
 * laps_gemm_workspace_bytes(m, n, k, split_k) bytes (0 when a single slice is used; then it may be NULL). */
size_t laps_gemm_workspace_bytes(int32_t m, int32_t n, int32_t k, int32_t split_k);
int laps_gemm_bf16(laps_ctx* ctx, const void* a_dev, const void* w_dev, float* c_dev, int32_t m, int32_t n,
                   int32_t k, int32_t split_k, void* workspace_dev, size_t workspace_bytes, void* stream);
/* The same projection with the epilogue the layer driver fuses (steps x1 = x + attn W_o^T, y = x1 + act W_d^T and
 * act = silu(r2 W_g^T) * (r2 W_u^T) of the layer math above), launched as the driver launches it: inside the GEMM
 * kernel when the plan keeps K in one slice, else K-slice partial sums and the row kernel that adds them.
 *   epilogue 1: out_f32[m,n] = resid[m,n] + C (resid may alias out_f32; n <= 8192);
 *   epilogue 2: out_bf16[m,n/2] = silu(gate) * up, with W holding gate and up rows interleaved in blocks of 32 as
 *               laps_pack_gate_up writes them.
 * workspace_dev: split * m * n * 4 bytes when laps_gemm_plan_info(m, n, k, 0, epilogue) reports split > 1.
 * EINVAL on NULL / unsupported shapes or a missing operand, ENOMEM if the workspace is too small. */
int laps_gemm_epilogue_bf16(laps_ctx* ctx, const void* a_dev, const void* w_dev, int32_t m, int32_t n, int32_t k,
                            int32_t epilogue, const float* resid_dev, float* out_f32_dev, void* out_bf16_dev,
                            void* workspace_dev, size_t workspace_bytes, void* stream);
/* Ragged paged causal GQA attention alone: q_dev bf16 [n_tokens, n_q*hd] (already rotated), K/V of
 * prefix and new tokens already in the pools; out_dev bf16 [n_tokens, n_q*hd]; workspace as for
 * laps_prefill_layer. */
int laps_attention(laps_ctx* ctx, int32_t n_seq, int32_t n_tokens, const int32_t* cu_seqlens_dev,
                   const int32_t* seq_len_dev, const int32_t* prefix_len_dev, const int32_t* page_table_dev,
                   int32_t max_pages, const void* k_pool_dev, const void* v_pool_dev, const void* q_dev,
                   void* out_dev, void* workspace_dev, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------ per-kernel timing
 * When enabled, un-captured laps_prefill_* calls bracket every kernel launch with HIP events on
 * the caller's stream.  laps_prof_read synchronises those events and returns, per kernel class,
 * the summed milliseconds and the launch count since the last laps_prof_enable(ctx, 1). */
enum { LAPS_K_PREP = 0, LAPS_K_RMSNORM, LAPS_K_GEMM_QKV, LAPS_K_GEMM_O, LAPS_K_GEMM_GATEUP, LAPS_K_GEMM_DOWN,
       LAPS_K_EPI_QKV, LAPS_K_EPI_RESID, LAPS_K_EPI_SWIGLU, LAPS_K_ATTN, LAPS_K_COUNT };
int laps_prof_enable(laps_ctx* ctx, int32_t on);
int laps_prof_read(laps_ctx* ctx, double* ms_out /*[LAPS_K_COUNT]*/, int64_t* count_out /*[LAPS_K_COUNT]*/);

/* ------------------------------------------------------------------ latency model (host, double)
 * Section 2.1: T_comp(L,H) = alpha L (L + 2H) + beta L, T_mem(L,H) = gamma_w L + gamma_r H for L new and H
 * historical tokens.  Boundaries where the two meet: prefill (H = 0) max(0, (gamma_w - beta)/alpha);
 * re-prefill the positive root of alpha L^2 + (2 alpha H + beta - gamma_w) L - gamma_r H = 0, which tends
 * to gamma_r / (2 alpha) for large H.  Below the boundary a request is memory-bound ("short").
 * Both return NaN when alpha <= 0 (or H < 0). */
double laps_lm_boundary_prefill(double alpha, double beta, double gamma_w);
double laps_lm_boundary_reprefill(double alpha, double beta, double gamma_w, double gamma_r, double hist_len);
/* Section 2.1 with a constant memory term: a short batch on this hardware is bounded by streaming the layer weights
 * once per pass (floor_t, same time unit as the coefficients), which the printed T_mem does not contain.  The knee is
 * the positive root of alpha L^2 + (2 alpha H + beta - gamma_w) L - (floor_t + gamma_r H) = 0: up to that many (padded)
 * new tokens a step costs one pass over the weights, beyond it arithmetic.  floor_t = 0 gives
 * laps_lm_boundary_reprefill.  NaN when alpha <= 0, H < 0, floor_t < 0 or an argument is NaN. */
double laps_lm_knee(double alpha, double beta, double gamma_w, double gamma_r, double floor_t, double hist_len);
/* "Runtime fitting" closed into the schedule: the parameters that the classification (Section 3.2), the bucket
 * grid (Section 3.1) and Algorithm 1's batch admission take from a fit coef[4] = {alpha, beta, gamma_w, gamma_r}
 * and a measured weight-streaming floor.  knee = min(knee(H = 0), knee(H = hist_max)).
 *   short_max_len      = the largest length bucket <= knee (the smallest bucket if none is);
 *   short_token_budget = the largest captured shape len_bucket * depth <= knee over buckets <= short_max_len
 *                        (at least short_max_len * depths[0]): padded tokens per graph in latency mode;
 *   fuse_budget        = the same value: other length buckets may join a batch up to that many padded tokens.
 * EINVAL on NULL, an unsorted grid, hist_max < 0 or a fit without a knee. */
typedef struct laps_lm_params {
    int32_t short_max_len, short_token_budget, fuse_budget;
    double knee_fresh, knee_hist; /* knee at H = 0 and at H = hist_max */
} laps_lm_params;
int laps_lm_derive_params(const double* coef, double floor_t, double hist_max, int32_t n_len_buckets,
                          const int32_t* len_buckets, int32_t n_depths, const int32_t* depths, laps_lm_params* out);
/* Least-squares fit of (alpha, beta) to t_comp and (gamma_w, gamma_r) to t_mem from n samples (host arrays
 * [n]; any consistent time unit).  coef_out[4] = {alpha, beta, gamma_w, gamma_r}.  Either time array may be NULL:
 * that half is not fitted and its two outputs are left untouched.  EINVAL if n < 2, both are NULL, or the
 * samples do not vary L and H independently. */
int laps_lm_fit(int32_t n, const double* new_len, const double* hist_len, const double* t_comp, const double* t_mem,
                double* coef_out);

/* ------------------------------------------------------------------ Adaptive-Wait-Depth batching (host)
 * Algorithm 1 and Section 3.2a.  The object holds the waiting window W, the target depth D and the timer of
 * the current round; the caller owns the short queue and the clock (any origin, microseconds) and polls at
 * every event: a short request arrives, the instance becomes free, or the wake-up time of the previous poll.
 *   W starts as clip(first_slack_us, [w_min, w_max]) with first_slack_us = min_i(DDL_i - t - S_hat) over the
 *   requests known at creation (INFINITY if none); D starts as the deepest captured shape within mem_budget.
 *   mem(G) = len_bucket * depth padded tokens.  t_max_us = INFINITY disables the head-of-line cap; a request
 *   without a deadline has ddl = INFINITY.  sla_window != 0 takes, when a round's timer starts,
 *   W = clip(min(W_SLA, W_GR)) (Section 3.2a) with rate_hat (requests per microsecond) from the caller.
 *   d_regrow != 0 adds what the printed algorithm lacks, a way for D to rise again: a round that fills D while
 *   at least D more requests wait moves D to the next larger captured depth (never above its start value). */
typedef struct laps_awd laps_awd;
typedef struct {
    int32_t n_len_buckets;
    const int32_t* len_buckets; /* host, strictly ascending */
    int32_t n_depths;
    const int32_t* depths;      /* host, strictly ascending */
    int64_t mem_budget;         /* M, padded tokens; >= depths[0] * largest bucket */
    int64_t fuse_budget;        /* padded tokens up to which requests of another length bucket than the oldest
                                   one's may join the batch (shape of the largest bucket); < 0: mem_budget */
    double sigma_us;            /* slack trigger */
    double w_min_us, w_max_us;  /* 0 <= w_min <= w_max < inf */
    double s_hat_us;            /* service-time estimate of one short step */
    double t_max_us;            /* head-of-line cap, INFINITY for none */
    double delta_us;            /* safety margin of W_SLA */
    double rate_eps;            /* floor of the arrival-rate estimate, > 0 */
    int32_t sla_window;
    int32_t d_regrow;
} laps_awd_params;
enum { LAPS_AWD_WAIT = 0, LAPS_AWD_DISPATCH = 1 };
enum { LAPS_AWD_NONE = 0, LAPS_AWD_DEPTH = 1, LAPS_AWD_SLA = 2, LAPS_AWD_TMAX = 3, LAPS_AWD_WINDOW = 4 };
int laps_awd_create(const laps_awd_params* p, double first_slack_us, laps_awd** out);
void laps_awd_destroy(laps_awd* awd);
double laps_awd_window_us(const laps_awd* awd);
int32_t laps_awd_target_depth(const laps_awd* awd);
/* Per-shape service-time estimates: s_hat_us is a host array [n_len_buckets][n_depths] (copied); the estimate
 * used at a decision is then the entry of the captured shape the batch formed at that instant would run in
 * (NaN entry: the single s_hat_us of the parameters).  NULL removes the table.  EINVAL on a negative entry. */
int laps_awd_set_service_table(laps_awd* awd, const double* s_hat_us);
/* The instance is free to form the next short batch from free_at_us on (e.g. when the dispatched step ends).
 * Without this call the next round's timer may start at the dispatch itself.  EINVAL while a round collects. */
int laps_awd_begin_round(laps_awd* awd, double free_at_us);
/* One decision at now_us over the waiting short requests (host arrays [n_waiting], arrival order, all with
 * arrival <= now).  The batch is re-formed at every poll: requests of the oldest one's length bucket first,
 * then the others, passing over any that no captured shape within the budget would hold.
 * *action = LAPS_AWD_DISPATCH: take_idx[0..*n_take) index the batch in the caller's arrays, to run in the
 * captured shape (*len_bucket, *depth) (*depth >= *n_take); *reason says why; W and D are already updated.
 * *action = LAPS_AWD_WAIT: poll again at *wake_us (INFINITY if the queue is empty) or at the next arrival.
 * take_idx must hold n_waiting entries.  EINVAL on NULL / NaN / unordered arrivals / lengths outside the grid. */
int laps_awd_poll(laps_awd* awd, double now_us, double rate_hat, int32_t n_waiting, const double* arrival_us,
                  const double* ddl_us, const int32_t* new_len, int32_t* action, int32_t* n_take, int32_t* take_idx,
                  int32_t* len_bucket, int32_t* depth, int32_t* reason, double* wake_us);

/* ------------------------------------------------------------------ fixed-window dispatch of the short queue (host)
 * Section 3.2 (one class of prefill at a time; two queues) and Section 3.1 (waiting window; graph fusion), read for one
 * GPU that alternates between the queues.  At a decision instant, over the waiting short requests (host arrays
 * [n_waiting], arrival order, all arrived by now_us; need_i = the smallest length bucket >= new_len[i]):
 *   *action = LAPS_AWD_DISPATCH iff a request waits and (now - arrival[0] >= window_us, or the sum of need_i >=
 *   token_budget, or nothing_else != 0: no long request waits and no arrival is outstanding); all waiting requests then
 *   leave together, and *fused_len_bucket is the largest need_i if the sum of need_i is below merge_below (every
 *   request then runs in that one length bucket: one replay costs one pass over the weights whatever its shape), else
 *   0 (plan each bucket on its own).  Otherwise LAPS_AWD_WAIT with *wake_us = arrival[0] + window_us (INFINITY when
 *   nothing waits): run a long chunk meanwhile.  *padded_tokens = the sum of need_i.
 * EINVAL on NULL, an unsorted grid, a length outside the grid, unordered arrivals or one after now_us. */
typedef struct laps_window_params {
    int32_t n_len_buckets;
    const int32_t* len_buckets; /* host, strictly ascending */
    double window_us;           /* W >= 0 */
    int64_t token_budget;       /* padded tokens that make the queue leave at once, >= 1 */
    int64_t merge_below;        /* fuse all waiting requests into one length bucket below this many padded tokens */
} laps_window_params;
int laps_window_poll(const laps_window_params* p, double now_us, int32_t n_waiting, const double* arrival_us,
                     const int32_t* new_len, int32_t nothing_else, int32_t* action, int32_t* fused_len_bucket,
                     int64_t* padded_tokens, double* wake_us);

/* ------------------------------------------------------------------ instance-pressure controller (host)
 * Algorithm 2 (spatial disaggregation): n_total instances in a SHORT and a LONG pool.  Each control period the
 * caller passes, per instance of each pool, queue backlog q, SLA deviation e and utilisation u (host arrays);
 * psi = w_q q + w_e e - w_u u; pool pressure = nearest-rank `quantile` (0.9 in the paper) of its psi values, 0 for
 * an empty pool.  Outside the cool-down, *action = +1 (one instance LONG -> SHORT) if P_s > (1 + tau) P_l and the
 * LONG pool holds more than n_min, else -1 (SHORT -> LONG) under the mirrored condition, else 0; the object updates
 * its pool sizes, the caller chooses which instance moves.  EINVAL if the signal counts disagree with the pools. */
typedef struct laps_ctrl laps_ctrl;
typedef struct {
    int32_t n_total, n_min;
    double cool_us;  /* no move within this time of the last one */
    double tau;      /* hysteresis */
    double w_q, w_e, w_u;
    double quantile; /* (0, 1] */
    double min_pressure; /* no move unless the gaining pool's pressure exceeds this; -INFINITY = as printed */
} laps_ctrl_params;
int laps_ctrl_create(const laps_ctrl_params* p, int32_t n_short, laps_ctrl** out);
void laps_ctrl_destroy(laps_ctrl* ctrl);
int32_t laps_ctrl_n_short(const laps_ctrl* ctrl);
int laps_ctrl_step(laps_ctrl* ctrl, double now_us, int32_t n_short, const double* q_s, const double* e_s,
                   const double* u_s, int32_t n_long, const double* q_l, const double* e_l, const double* u_l,
                   int32_t* action, double* p_short, double* p_long);

const char* laps_last_error(void);
const char* laps_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LAPS_H */
