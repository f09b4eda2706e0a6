/*
 * libhmi — mixed-tenant batched forward of per-tenant transformer layers on one
 * MI355X (gfx950).
 *
 * Problem (HMI, Sec. 6 intro and Sec. 6.3): one inference batch holds requests of many
 * tenants; every request must be transformed with its own tenant's task-specific
 * parameters, and doing that tenant by tenant fragments the GPU work.  The paper
 * stacks the parameters per request and issues one batched matrix multiplication.
 * This library reaches the same result by ordering the requests by tenant and
 * running grouped GEMMs whose B operand is looked up, per segment, in a pool of
 * tenant weight images resident in HBM (optionally backed by pinned host memory
 * and filled on demand on a side stream, Sec. 5.2 / Sec. 6.2).
 *
 * Conventions for every entry point
 *   - plain C ABI; no exception crosses it; every call returns an int32 status
 *     (HMI_OK = 0, errors negative).  hmi_last_error() gives a readable reason.  A failed
 *     HIP runtime call is reported as HMI_ERR_OOM / HMI_ERR_DEVICE and taken out of the
 *     runtime's last-error state, so the caller's next hipGetLastError() does not see it.
 *   - "host" / "device" on a pointer says where the memory lives.
 *   - the library owns: the pool, its HBM slots, pinned host images, workspaces,
 *     its copy stream and events.  The caller owns x, y, index arrays, weight source
 *     buffers and the compute stream.
 *   - not thread-safe per pool; calls on one pool must come from one thread at a time.
 *     Different pools may be used from different threads at the same time.
 */
#ifndef HMI_H
#define HMI_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hmi_pool hmi_pool_t; /* opaque */

enum {
  HMI_OK = 0,
  HMI_ERR_ARG = -1,      /* null pointer, bad enum value, inconsistent config          */
  HMI_ERR_OOM = -2,      /* device or pinned-host allocation failed                    */
  HMI_ERR_TENANT = -3,   /* tenant id outside [0,max_tenants) or (tenant,layer) never loaded */
  HMI_ERR_SHAPE = -4,    /* seq_len <= 0, too many requests / tokens, wrong tensor count */
  HMI_ERR_CAPACITY = -5, /* more distinct tenants needed at once than hbm_slots         */
  HMI_ERR_DEVICE = -6    /* a HIP runtime call failed                                   */
};

enum { HMI_F32 = 0, HMI_BF16 = 1 };

/* Per-tenant block kinds.  Matrices are [out,in] row-major: Linear(a) = W a + b (Sec. 3.2.2).
 * Canonical tensor order of one (tenant, layer):
 *   FFN         w1[f,d] b1[f] w2[d,f] b2[d] ln_g[d] ln_b[d]
 *               Y = LN(X + W2 GELU(W1 X + b1) + b2)
 *   ENC_POSTLN  wqkv[3d,d] bqkv[3d] wo[d,d] bo[d] ln1_g[d] ln1_b[d] w1 b1 w2 b2 ln2_g[d] ln2_b[d]
 *               X1 = LN1(X + Attn(X));  Y = LN2(X1 + FFN(X1));  bidirectional attention
 *   DEC_PRELN   same tensors;  X1 = X + Attn(LN1(X));  Y = X1 + FFN(LN2(X1));  causal attention
 *   ADAPTER     w_down[r,d] b_down[r] w_up[d,r] b_up[d]   (r = d_ff)
 *               Y = X + Up(ReLU(Down(X)))                 (the paper's adapter, Sec. 3.2.2)
 *   ENC_ADAPTER the paper's task-adapted higher layer (Sec. 3.2.2): one ENC_POSTLN tensor set per
 *               layer shared by all tenants (hmi_pool_load_shared), and per tenant the ADAPTER
 *               tensors with r = adapter_rank, injected after the attention layer:
 *               A = Attn(X);  X1 = LN1(X + A + Up_t(ReLU(Down_t(A))));  Y = LN2(X1 + FFN(X1))
 *   DEC_ADAPTER the same for decoder-only instances: shared DEC_PRELN tensor set, tenant adapter:
 *               A = Attn(LN1(X)) causal;  X1 = X + A + Up_t(ReLU(Down_t(A)));  Y = X1 + FFN(LN2(X1))
 * Attention is per request (never across requests), softmax scale 1/sqrt(d/n_heads),
 * packed qkv in q,k,v order, head h owns columns [h*d_head,(h+1)*d_head).  GELU is the
 * exact erf form; LayerNorm uses the biased variance and ln_eps inside the square root. */
enum { HMI_BLOCK_FFN = 0, HMI_BLOCK_ENC_POSTLN = 1, HMI_BLOCK_DEC_PRELN = 2, HMI_BLOCK_ADAPTER = 3,
       HMI_BLOCK_ENC_ADAPTER = 4, HMI_BLOCK_DEC_ADAPTER = 5 };

typedef struct {
  int32_t block;        /* HMI_BLOCK_*                                                    */
  int32_t dtype;        /* HMI_F32 | HMI_BF16: storage type of weights, x and y           */
  int32_t d_model;      /* multiple of 64 (bf16) / 16 (f32), at most 2048; max_tokens * max(d_model, d_ff)
                           * element size must stay below 4 GiB (32-bit row offsets)      */
  int32_t d_ff;         /* FFN width, or adapter rank; multiple of 64 (bf16) / 16 (f32)   */
  int32_t n_heads;      /* attention blocks: d_model / n_heads must be 64; else 0         */
  int32_t n_layers;     /* per-tenant layers held per tenant (1 .. 1024)                  */
  int32_t max_tenants;  /* tenant ids live in [0, max_tenants); at most 2^24              */
  int32_t hbm_slots;    /* tenants resident in HBM at once (<= max_tenants)               */
  int32_t host_tier;    /* 1: every loaded tenant also kept in pinned host memory; HBM is
                           an LRU cache over it, misses are copied in on a side stream    */
  int32_t max_requests; /* R bound per forward call (<= 2048)                             */
  int32_t max_tokens;   /* N = sum(seq_lens) bound per forward call                       */
  float   ln_eps;
  int32_t device;       /* HIP device ordinal                                             */
  void*   compute_stream; /* hipStream_t borrowed from the caller; NULL = default stream  */
  int32_t adapter_rank; /* ENC_/DEC_ADAPTER: bottleneck width r of the per-tenant adapter, multiple
                           of 64 (bf16) / 16 (f32), <= d_ff; ignored by the other blocks      */
  int32_t max_classes;  /* > 0: tenants may own an output head with up to this many classes
                           (<= 64), see hmi_pool_load_head; 0: no heads                        */
} hmi_pool_config_t;

/* Create a pool (Sec. 4.1 "create hPLM" needs somewhere to put instances).  Allocates the
 * HBM slots (hbm_slots * n_layers images), the workspaces for max_tokens, and, with
 * host_tier, nothing per tenant yet (pinned images are allocated at load).  *out is set
 * only on HMI_OK. */
int32_t hmi_pool_create(const hmi_pool_config_t* cfg, hmi_pool_t** out);

/* Register one (tenant, layer) weight set (Sec. 5.2: a fine-tuned instance's task
 * parameters are stored once and fetched when requested).  `tensors` is a HOST array of
 * n_tensors HOST pointers in the canonical order above, each in the pool's dtype, dense
 * row-major.  The data is copied before return; the caller keeps its buffers.  Without
 * host_tier the tenant takes an HBM slot for good (HMI_ERR_CAPACITY when none is left);
 * with host_tier it goes to pinned host memory and into HBM only if a slot is free.
 * Re-loading a (tenant, layer) replaces its weights. */
int32_t hmi_pool_load_tenant(hmi_pool_t* pool, int32_t tenant_id, int32_t layer,
                             const void* const* tensors, int32_t n_tensors);

/* Pools with host_tier: create instance `tenant_id` with the task parameters of `source_tenant`, all layers (in
 * the paper instances are created from stored fine-tuned parameters, Sec. 4.1 / Sec. 5.2; here several instances
 * may be created from one stored set).  The two share one image in pinned host memory, so a tenant id space larger
 * than the pinned memory can hold still exercises the HBM cache at its real size: in HBM every tenant id has its
 * own slot, hits, misses and swap-in traffic.  Every layer of `source_tenant` must be loaded and `tenant_id` must
 * not have parameters yet, else HMI_ERR_TENANT / HMI_ERR_ARG.  Afterwards neither of the two can be loaded again
 * with hmi_pool_load_tenant (HMI_ERR_ARG).  Takes a free HBM slot if there is one, like hmi_pool_load_tenant. */
int32_t hmi_pool_alias_tenant(hmi_pool_t* pool, int32_t tenant_id, int32_t source_tenant);

/* ENC_ADAPTER / DEC_ADAPTER pools: register the parameters of `layer` that every tenant shares (the
 * higher transformer layers stay on the GPU and are reused across tenants, Sec. 3.2.2).
 * `tensors`: HOST array of the 12 ENC_POSTLN tensors as HOST pointers, pool dtype, dense
 * row-major; copied to HBM before return.  Waits for work in flight when it replaces a
 * layer that was loaded before.  Other block kinds: HMI_ERR_ARG. */
int32_t hmi_pool_load_shared(hmi_pool_t* pool, int32_t layer, const void* const* tensors,
                             int32_t n_tensors);

/* The hot path (Sec. 6.3): y[rows of request r] = block_{tenant_ids[r]}(x[rows of request r]).
 * x, y: DEVICE, [N, d_model] packed in request order (request r owns rows
 * tok_off[r] .. tok_off[r]+seq_lens[r]), pool dtype, x != y, x is not modified.
 * tenant_ids, seq_lens: HOST int32[n_requests]; copied before return.
 * Work is enqueued on compute_stream and the call returns without waiting for it.
 * Errors are detected before anything is enqueued, so y is untouched on error:
 * unknown / unloaded tenant -> HMI_ERR_TENANT; seq_len <= 0, R or N over the configured
 * bound -> HMI_ERR_SHAPE; more distinct tenants than hbm_slots -> HMI_ERR_CAPACITY;
 * ENC_/DEC_ADAPTER with the layer's shared parameters not loaded -> HMI_ERR_ARG.
 * n_requests == 0 is HMI_OK and does nothing. */
int32_t hmi_layer_forward(hmi_pool_t* pool, int32_t layer, const void* x, void* y,
                          const int32_t* tenant_ids, const int32_t* seq_lens,
                          int32_t n_requests);

/* hmi_layer_forward for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same result, but the routing arrays
 * the kernels work from (request order, segment offsets, row map, tile lists) live in a static
 * device array of the library (0.17 MB per GPU, held until the process ends) instead of the pool's
 * own allocation, and the call itself allocates and frees nothing, on the device or the host.
 * Limits: a bf16 ADAPTER pool without host_tier whose forward is one kernel (rank d_ff = 64,
 * d_model 256 / 512 / 768, n_layers = 1), else HMI_ERR_ARG; n_requests <= 256 and at most 32 768
 * tokens (and the pool's own bounds), else HMI_ERR_SHAPE.  Other arguments, errors (y untouched)
 * and asynchrony as hmi_layer_forward.  All pools on one GPU share that GPU's array: calls that
 * may overlap in time on one GPU (different streams) race; calls ordered on one stream do not.
 * Each call rewrites every entry it reads, so nothing carries over from the call before.
 * hmi_get_route and hmi_head_forward keep referring to the last call that routed inside the pool. */
int32_t hmi_layer_forward_static(hmi_pool_t* pool, int32_t layer, const void* x, void* y,
                                 const int32_t* tenant_ids, const int32_t* seq_lens,
                                 int32_t n_requests);

/* Several consecutive layers [layer_begin, layer_end) of every request's tenant in one call
 * (the paper's hPLM runs a stack of task-adapted higher layers per request, Sec. 3.3.2, and
 * prefetches layer l+1's task parameters while layer l computes, Sec. 6.2).  Same arguments,
 * errors and asynchrony as hmi_layer_forward.  The batch is routed once; between layers the
 * activations stay in fp32 inside the library and only the last layer rounds into y; with
 * host_tier the swap-in of layer l+1 is enqueued on the copy stream before layer l's
 * kernels.  hmi_layer_forward(layer) is hmi_stack_forward(layer, layer+1). */
int32_t hmi_stack_forward(hmi_pool_t* pool, int32_t layer_begin, int32_t layer_end,
                          const void* x, void* y, const int32_t* tenant_ids,
                          const int32_t* seq_lens, int32_t n_requests);

/* hmi_stack_forward with the result left unrounded: y is DEVICE float [N, d_model] whatever the
 * pool's storage type (x stays in the storage type).  The stack carries its hidden states in fp32
 * between layers; this call hands the last layer's fp32 result out instead of rounding it to bf16,
 * for callers that go on computing in fp32 (an output head, a further stack) and for checking the
 * arithmetic of a deep stack apart from the rounding of its result (half a bf16 unit is 0.0156 for
 * values of magnitude 4 to 8).  Not available from pools that run the one-kernel adapter
 * (HMI_ERR_ARG). */
int32_t hmi_stack_forward_f32(hmi_pool_t* pool, int32_t layer_begin, int32_t layer_end,
                              const void* x, float* y, const int32_t* tenant_ids,
                              const int32_t* seq_lens, int32_t n_requests);

/* Representation retrieval, GPU side (Sec. 3.3.1): the hidden states that enter the higher layers
 * are aggregated from precomputed representations of three-token fragments, one fragment centred
 * on every token.  table: DEVICE [n_entries, 3, d_model], pool dtype (row e holds the
 * representations of the first, second and third token of fragment e); frag_ids: DEVICE
 * int32 [N], the table row of the fragment centred on each token (the lookup itself runs on the
 * CPU in the paper; ids outside [0, n_entries) are clamped); seq_lens: HOST int32 [n_requests];
 * x: DEVICE [N, d_model], out.  Token i of a request is the third token of fragment i-1, the
 * second of fragment i and the first of fragment i+1 where those exist inside the request; x[i]
 * is the sum of these representations divided by their number (fp32, rounded once).  Enqueued on
 * compute_stream.  Caller owns table, frag_ids and x. */
int32_t hmi_plot_aggregate(hmi_pool_t* pool, const void* table, int32_t n_entries,
                           const int32_t* frag_ids, const int32_t* seq_lens, int32_t n_requests,
                           void* x);

/* Autoregressive decoding for bf16 DEC_PRELN and DEC_ADAPTER pools (the paper reports its GPT-style instances in
 * generated tokens per second, Sec. 7): a key/value cache of max_seqs lines ("sequence slots") of
 * max_len positions for every layer of the pool, owned by the library.  Once per pool; other
 * pools -> HMI_ERR_ARG; HMI_ERR_OOM when it does not fit. */
int32_t hmi_kv_create(hmi_pool_t* pool, int32_t max_seqs, int32_t max_len);

/* hmi_stack_forward that also records every row's key and value: request r's rows fill line
 * seq_slots[r] (HOST int32[n_requests], distinct within a call) from position 0 and set its
 * length to seq_lens[r] (<= max_len, else HMI_ERR_SHAPE).  Same results, errors and asynchrony. */
int32_t hmi_prefill(hmi_pool_t* pool, int32_t layer_begin, int32_t layer_end, const void* x, void* y,
                    const int32_t* tenant_ids, const int32_t* seq_lens, const int32_t* seq_slots,
                    int32_t n_requests);

/* One new token per request: x, y DEVICE [n_requests, d_model].  Row r passes through the layers
 * of tenant_ids[r]; in each layer its key and value are appended to line seq_slots[r] and it
 * attends to all positions of that line, itself included (causal attention over the sequence so
 * far: the result equals the last row of a full forward over the whole sequence).  The line's
 * length grows by one (beyond max_len -> HMI_ERR_SHAPE before anything is enqueued). */
int32_t hmi_decode_step(hmi_pool_t* pool, int32_t layer_begin, int32_t layer_end, const void* x, void* y,
                        const int32_t* tenant_ids, const int32_t* seq_slots, int32_t n_requests);

/* Per-tenant output heads (Sec. 3.3.2): one linear layer per tenant on the final hidden states,
 * with the tenant's own number of classes.  A classification tenant (per_token = 0) is scored on
 * the first row of each of its requests (the [CLS] token at the beginning of the sentence), a
 * tagging tenant (per_token = 1) on every row; the label is the class with the highest score
 * (lowest index on ties).  w: HOST [n_classes, d_model] row-major, b: HOST [n_classes], pool
 * dtype; copied to HBM before return (heads of all tenants stay resident: they are a few KB).
 * 1 <= n_classes <= max_classes, else HMI_ERR_SHAPE. */
int32_t hmi_pool_load_head(hmi_pool_t* pool, int32_t tenant_id, const void* w, const void* b,
                           int32_t n_classes, int32_t per_token);

/* Scores the batch of the most recent forward call on this pool (its tenant_ids and seq_lens;
 * the routing it left on the device is reused) from h: DEVICE [N, d_model], pool dtype, normally
 * that call's y.  scores: DEVICE float [N, max_classes] or NULL; labels: DEVICE int32 [N].
 * Rows without a prediction (rows after the first of a classification tenant's request) get
 * label -1 and scores -inf; columns at or beyond the tenant's class count get -inf.  Scores are
 * accumulated and compared in fp32.  Enqueued on compute_stream.  No earlier forward call ->
 * HMI_ERR_ARG; a tenant of that batch without a head -> HMI_ERR_TENANT (nothing enqueued). */
int32_t hmi_head_forward(hmi_pool_t* pool, const void* h, float* scores, int32_t* labels);

/* The grouping of the last forward call's requests by tenant (Sec. 6.3 batches the requests of
 * different instances into one set of launches; this is the order they were grouped in), for
 * bit-exact checks of the tenant-segmented router:
 * perm[R] (stable order of requests by tenant id), seg_tenant[G], seg_req_off[G+1],
 * seg_tok_off[G+1] (segment bounds in sorted requests / sorted tokens), *n_segments = G.
 * All HOST buffers sized for max_requests(+1); any may be NULL.  Waits for the router. */
int32_t hmi_get_route(hmi_pool_t* pool, int32_t* perm, int32_t* seg_tenant,
                      int32_t* seg_req_off, int32_t* seg_tok_off, int32_t* n_segments);

/* Pipelined swapping (Sec. 6.2): start bringing `layer` of these tenants into HBM on the
 * library's copy stream while the compute stream is busy with an earlier batch or layer.
 * HOST int32[n].  Tenants already resident are only marked recently used.  No-op without
 * host_tier.  Best effort: stops silently when no evictable slot is left. */
int32_t hmi_pool_prefetch(hmi_pool_t* pool, int32_t layer, const int32_t* tenant_ids, int32_t n);

/* Swapping statistics (Sec. 5.2: task parameters are brought to the GPU only when their instance
 * is requested).  Counters since creation: hits / misses count distinct (tenant, layer) lookups made by
 * forward calls; bytes_h2d counts swap-in traffic.  Any pointer may be NULL. */
int32_t hmi_pool_stats(hmi_pool_t* pool, int64_t* hits, int64_t* misses, int64_t* bytes_h2d,
                       int64_t* evictions);

/* ---- Request queue: the batch former and pipelined runner in front of a pool ----
 *
 * The paper's dispatcher appends every inference request to the last batch of its input queue and
 * opens a new batch when the maximum batch size is reached (Sec. 4.2); its scheduler runs the batches
 * in order and, while one batch computes, already loads the next batch's task parameters on the other
 * stream (coarse-grained pipelining, Sec. 6.2).  A queue does both for one pool.  Not thread-safe;
 * calls on a queue and on its pool must come from one thread at a time.  The queue owns its batch
 * buffers (x and y of max_batch_tokens rows for each of max_waiting_batches + 2 batches). */
typedef struct hmi_queue hmi_queue_t; /* opaque */

/* max_batch_requests <= the pool's max_requests, max_batch_tokens <= its max_tokens,
 * 1 <= max_waiting_batches <= 64: batches that may wait to run at any time. */
int32_t hmi_queue_create(hmi_pool_t* pool, int32_t max_batch_requests, int32_t max_batch_tokens,
                         int32_t max_waiting_batches, hmi_queue_t** out);

/* One inference request: tenant_id's instance on x_rows, DEVICE [seq_len, d_model] in the pool dtype,
 * 16-byte aligned.  The rows are not copied here: they must stay valid and unchanged until the request's
 * batch has been run (hmi_queue_run gathers the rows of all its requests with one kernel on
 * compute_stream) and that stream has passed the gather.  The request joins the last batch; a new batch is opened when
 * the last one is full: max_batch_requests requests, or not enough of max_batch_tokens left, or
 * already hbm_slots distinct tenants and this would be another one.  *ticket identifies the
 * request.  Errors change nothing: unknown / unloaded tenant -> HMI_ERR_TENANT; seq_len outside
 * [1, max_batch_tokens] -> HMI_ERR_SHAPE; a new batch is needed while max_waiting_batches are
 * waiting -> HMI_ERR_CAPACITY (run one, then push again). */
int32_t hmi_queue_push(hmi_queue_t* queue, int32_t tenant_id, int32_t seq_len, const void* x_rows,
                       int64_t* ticket);

/* Runs the oldest waiting batch through all layers of the pool (hmi_stack_forward, enqueued on
 * compute_stream), then, with host_tier, starts bringing every layer of the tenants of the next
 * waiting batch into HBM on the copy stream (hmi_pool_prefetch), so that the copies run under this
 * batch's kernels.  *batch (may be NULL) = the number of the batch that ran, counted from 0 in the
 * order the batches were opened, or -1 if none was waiting; *n_requests (may be NULL) its size. */
int32_t hmi_queue_run(hmi_queue_t* queue, int64_t* batch, int32_t* n_requests);

/* Copies the output rows of one request, DEVICE [seq_len, d_model], to y_rows (enqueued on
 * compute_stream).  The request's batch must have run, and its results are held until
 * max_waiting_batches + 1 later batches have been opened; otherwise HMI_ERR_ARG. */
int32_t hmi_queue_fetch(hmi_queue_t* queue, int64_t ticket, void* y_rows);

/* Batches waiting to run (the open one counts if it holds a request). */
int32_t hmi_queue_waiting(const hmi_queue_t* queue);

/* Reason of the last error on this queue. */
const char* hmi_queue_last_error(const hmi_queue_t* queue);

/* Waits for compute_stream, frees the batch buffers.  Destroy the queue before its pool.  NULL is fine. */
int32_t hmi_queue_destroy(hmi_queue_t* queue);

/* Per-kernel timing for measurement: while enabled, every kernel the forward calls launch
 * is bracketed by HIP events on compute_stream.  hmi_pool_profile_read waits for the
 * stream, then writes the summed milliseconds and the launch count of each kernel kind
 * (HOST arrays of HMI_KERNEL_KINDS entries, either may be NULL) and clears the record. */
enum { HMI_KERNEL_ROUTER = 0, HMI_KERNEL_GEMM = 1, HMI_KERNEL_ATTENTION = 2,
       HMI_KERNEL_LAYERNORM = 3, HMI_KERNEL_KINDS = 4 };
int32_t hmi_pool_profile(hmi_pool_t* pool, int32_t enable);
int32_t hmi_pool_profile_read(hmi_pool_t* pool, double* ms, int64_t* launches);

/* Bytes of one (tenant, layer) image in HBM (tensors padded to 256 B). */
int64_t hmi_pool_image_bytes(const hmi_pool_t* pool);

/* Static string describing the last error on this pool (or, when pool is NULL, the calling
 * thread's last create error).  Valid until the next call on the pool (by that thread). */
const char* hmi_last_error(const hmi_pool_t* pool);

/* Deletes every instance of the pool (Sec. 4.1, "delete hPLM", for all of them at once): waits
 * for both streams, then frees the HBM slots, pinned host images, workspaces, the copy stream and
 * the events.  The handle is invalid afterwards.  NULL is fine. */
int32_t hmi_pool_destroy(hmi_pool_t* pool);

#ifdef __cplusplus
}
#endif
#endif /* HMI_H */
