// Batch former and pipelined runner in front of a tenant pool.
//
// Paper passages realised here: the dispatcher appends every inference request to the last batch of
// its input queue and opens a new batch when the maximum batch size is reached (Sec. 4.2); the
// scheduler takes the batches in order and, while one batch computes, already loads the task
// parameters of the next one on the other stream (coarse-grained pipelining, Sec. 6.2).  The
// layer-ahead loading inside a batch (fine-grained pipelining) is hmi_stack_forward's.
#include "pool_internal.h"

#include <cstdarg>
#include <cstdio>
#include <new>
#include <vector>

namespace {

enum BatchState { EMPTY = 0, OPEN, CLOSED, RAN };

struct Batch {
  BatchState state = EMPTY;
  int64_t seq = -1;                 // position in the order of batches, from 0
  int32_t n_req = 0, n_tok = 0, n_distinct = 0;
  std::vector<int32_t> ids, lens, distinct;
  const void** src = nullptr;       // pinned host [max_requests]: where each request's rows are (device addresses)
  int32_t* tok_off = nullptr;       // pinned host [max_requests + 1]: first row of each request in x / y
  hipEvent_t gathered = nullptr;    // the gather kernel that reads src / tok_off has run
  char* x = nullptr;                // device [max_tokens, d]
  char* y = nullptr;
};

// x[tok_off[r] + i, :] = src[r][i, :] for every request r of a batch: one workgroup per request, 16-byte pieces.
// src and tok_off are read in place from pinned host memory (one small read each per workgroup).
__global__ __launch_bounds__(256) void gather_rows_kernel(const void* const* src, const int32_t* tok_off, char* x, int row_bytes) {
  const int r = blockIdx.x;
  const uint4* from = static_cast<const uint4*>(src[r]);
  const int first = tok_off[r];
  const size_t pieces = (size_t)(tok_off[r + 1] - first) * (size_t)(row_bytes / 16);
  uint4* to = reinterpret_cast<uint4*>(x + (size_t)first * row_bytes);
  for (size_t i = threadIdx.x; i < pieces; i += 256) to[i] = from[i];
}

}  // namespace

struct hmi_queue {
  hmi_pool_t* pool = nullptr;
  hmi_pool_config_t cfg{};
  int32_t max_req = 0, max_tok = 0, max_waiting = 0;
  size_t row_bytes = 0;
  std::vector<Batch> ring;          // max_waiting + 2 records: the waiting ones, the one that ran last, one spare
  int64_t next_seq = 0;             // sequence number of the next batch to open
  int64_t next_run = 0;             // sequence number of the next batch to run
  std::vector<uint32_t> mark;       // [tenant] sequence + 1 of the batch that saw the tenant last
  char err[256] = "";
};

namespace {

int32_t qfail(hmi_queue* q, int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(q->err, sizeof(q->err), fmt, ap);
  va_end(ap);
  if (code == HMI_ERR_OOM || code == HMI_ERR_DEVICE) (void)hipGetLastError();   // reported here: not left for the caller's next check
  return code;
}

Batch* find(hmi_queue* q, int64_t seq) {
  for (auto& b : q->ring)
    if (b.state != EMPTY && b.seq == seq) return &b;
  return nullptr;
}

int waiting(const hmi_queue* q) {
  int n = 0;
  for (auto& b : q->ring)
    if (b.state == CLOSED || (b.state == OPEN && b.n_req > 0)) ++n;
  return n;
}

// A record for a new batch: an empty one, else the oldest batch that has run (its results are given up).
Batch* take_record(hmi_queue* q) {
  Batch* best = nullptr;
  for (auto& b : q->ring) {
    if (b.state == EMPTY) return &b;
    if (b.state == RAN && (!best || b.seq < best->seq)) best = &b;
  }
  return best;
}

void open_batch(hmi_queue* q, Batch* b) {
  (void)hipEventSynchronize(b->gathered);   // the record's last gather has read its arrays (no-op for a fresh event)
  b->state = OPEN;
  b->seq = q->next_seq++;
  b->n_req = b->n_tok = b->n_distinct = 0;
  b->tok_off[0] = 0;
}

}  // namespace

extern "C" {

int32_t hmi_queue_create(hmi_pool_t* pool, int32_t max_batch_requests, int32_t max_batch_tokens,
                         int32_t max_waiting_batches, hmi_queue_t** out) {
  if (!pool || !out) return HMI_ERR_ARG;
  const hmi_pool_config_t* c = hmi_internal_config(pool);
  if (max_batch_requests < 1 || max_batch_requests > c->max_requests || max_batch_tokens < 1 ||
      max_batch_tokens > c->max_tokens || max_waiting_batches < 1 || max_waiting_batches > 64)
    return HMI_ERR_ARG;
  hmi_queue* q = new (std::nothrow) hmi_queue();
  if (!q) return HMI_ERR_OOM;
  q->pool = pool;
  q->cfg = *c;
  q->max_req = max_batch_requests;
  q->max_tok = max_batch_tokens;
  q->max_waiting = max_waiting_batches;
  q->row_bytes = (size_t)c->d_model * (c->dtype == HMI_BF16 ? 2 : 4);
  q->mark.assign(c->max_tenants, 0);
  q->ring.resize(max_waiting_batches + 2);
  if (hipSetDevice(c->device) != hipSuccess) { delete q; (void)hipGetLastError(); return HMI_ERR_DEVICE; }
  for (auto& b : q->ring) {
    b.ids.resize(max_batch_requests);
    b.lens.resize(max_batch_requests);
    b.distinct.resize(max_batch_requests);
    if (hipHostMalloc(reinterpret_cast<void**>(&b.src), sizeof(void*) * (size_t)max_batch_requests, hipHostMallocDefault) != hipSuccess ||
        hipHostMalloc(reinterpret_cast<void**>(&b.tok_off), sizeof(int32_t) * ((size_t)max_batch_requests + 1), hipHostMallocDefault) != hipSuccess ||
        hipEventCreateWithFlags(&b.gathered, hipEventDisableTiming) != hipSuccess ||
        hipMalloc(&b.x, (size_t)max_batch_tokens * q->row_bytes) != hipSuccess ||
        hipMalloc(&b.y, (size_t)max_batch_tokens * q->row_bytes) != hipSuccess) {
      hmi_queue_destroy(q);
      (void)hipGetLastError();   // reported through the status: not left behind as the runtime's last error
      return HMI_ERR_OOM;
    }
  }
  *out = q;
  return HMI_OK;
}

int32_t hmi_queue_push(hmi_queue_t* q, int32_t tenant, int32_t seq_len, const void* x_rows, int64_t* ticket) {
  if (!q) return HMI_ERR_ARG;
  if (!x_rows || !ticket) return qfail(q, HMI_ERR_ARG, "null pointer");
  if (tenant < 0 || tenant >= q->cfg.max_tenants) return qfail(q, HMI_ERR_TENANT, "tenant %d outside [0,%d)", tenant, q->cfg.max_tenants);
  if (!hmi_internal_tenant_ready(q->pool, tenant)) return qfail(q, HMI_ERR_TENANT, "tenant %d is not loaded", tenant);
  if (seq_len < 1 || seq_len > q->max_tok) return qfail(q, HMI_ERR_SHAPE, "seq_len %d outside [1,%d]", seq_len, q->max_tok);
  Batch* b = find(q, q->next_seq - 1);
  if (b && b->state != OPEN) b = nullptr;
  if (b) {
    // the batching rule: the request joins the last batch unless that batch is full (requests, tokens,
    // or more distinct tenants than the pool can hold in HBM at once)
    const bool new_tenant = q->mark[tenant] != (uint32_t)(b->seq + 1);
    if (b->n_req == q->max_req || b->n_tok + seq_len > q->max_tok || (new_tenant && b->n_distinct == q->cfg.hbm_slots)) {
      b->state = CLOSED;
      b = nullptr;
    }
  }
  if (!b) {
    if (waiting(q) >= q->max_waiting) return qfail(q, HMI_ERR_CAPACITY, "%d batches are waiting: run one first", q->max_waiting);
    b = take_record(q);
    if (!b) return qfail(q, HMI_ERR_CAPACITY, "no batch record free");
    if (hipSetDevice(q->cfg.device) != hipSuccess) return qfail(q, HMI_ERR_DEVICE, "hipSetDevice failed");
    open_batch(q, b);
  }
  b->src[b->n_req] = x_rows;
  if (q->mark[tenant] != (uint32_t)(b->seq + 1)) {
    q->mark[tenant] = (uint32_t)(b->seq + 1);
    b->distinct[b->n_distinct++] = tenant;
  }
  b->ids[b->n_req] = tenant;
  b->lens[b->n_req] = seq_len;
  b->tok_off[b->n_req + 1] = b->n_tok + seq_len;
  *ticket = b->seq * (int64_t)(1 << 20) + b->n_req;
  ++b->n_req;
  b->n_tok += seq_len;
  return HMI_OK;
}

int32_t hmi_queue_run(hmi_queue_t* q, int64_t* batch, int32_t* n_requests) {
  if (!q) return HMI_ERR_ARG;
  if (batch) *batch = -1;
  if (n_requests) *n_requests = 0;
  Batch* b = find(q, q->next_run);
  if (!b || b->n_req == 0 || (b->state != OPEN && b->state != CLOSED)) return HMI_OK;   // nothing is waiting
  b->state = CLOSED;
  const int L = q->cfg.n_layers;
  hipStream_t s = hmi_internal_compute_stream(q->pool);
  if (hipSetDevice(q->cfg.device) != hipSuccess) return qfail(q, HMI_ERR_DEVICE, "hipSetDevice failed");
  hipLaunchKernelGGL(gather_rows_kernel, dim3(b->n_req), dim3(256), 0, s, b->src, b->tok_off, b->x, (int)q->row_bytes);
  if (hipEventRecord(b->gathered, s) != hipSuccess || hipGetLastError() != hipSuccess)
    return qfail(q, HMI_ERR_DEVICE, "gathering the batch's rows failed");
  int32_t rc = hmi_stack_forward(q->pool, 0, L, b->x, b->y, b->ids.data(), b->lens.data(), b->n_req);
  if (rc != HMI_OK) {
    // cannot happen for what push admitted, short of a device error: give the batch up rather than block the queue
    snprintf(q->err, sizeof(q->err), "batch %lld failed: %s", (long long)b->seq, hmi_last_error(q->pool));
    b->state = EMPTY;
    ++q->next_run;
    return rc;
  }
  b->state = RAN;
  ++q->next_run;
  if (batch) *batch = b->seq;
  if (n_requests) *n_requests = b->n_req;
  // coarse-grained pipelining: the next waiting batch's task parameters move to HBM under this batch's kernels
  Batch* nb = find(q, q->next_run);
  if (nb && nb->n_req > 0 && q->cfg.host_tier)
    for (int l = 0; l < L; ++l) {
      rc = hmi_pool_prefetch(q->pool, l, nb->distinct.data(), nb->n_distinct);
      if (rc != HMI_OK) return qfail(q, rc, "prefetch for batch %lld failed: %s", (long long)nb->seq, hmi_last_error(q->pool));
    }
  return HMI_OK;
}

int32_t hmi_queue_fetch(hmi_queue_t* q, int64_t ticket, void* y_rows) {
  if (!q) return HMI_ERR_ARG;
  if (!y_rows || ticket < 0) return qfail(q, HMI_ERR_ARG, "null pointer or bad ticket");
  const int64_t seq = ticket >> 20;
  const int r = (int)(ticket & ((1 << 20) - 1));
  Batch* b = find(q, seq);
  if (!b || b->state != RAN || r >= b->n_req)
    return qfail(q, HMI_ERR_ARG, "batch %lld has not run yet or its results are no longer held", (long long)seq);
  if (hipSetDevice(q->cfg.device) != hipSuccess ||
      hipMemcpyAsync(y_rows, b->y + (size_t)b->tok_off[r] * q->row_bytes, (size_t)b->lens[r] * q->row_bytes,
                     hipMemcpyDeviceToDevice, hmi_internal_compute_stream(q->pool)) != hipSuccess)
    return qfail(q, HMI_ERR_DEVICE, "copy of the result rows failed");
  return HMI_OK;
}

int32_t hmi_queue_waiting(const hmi_queue_t* q) { return q ? waiting(q) : 0; }

const char* hmi_queue_last_error(const hmi_queue_t* q) { return q ? q->err : ""; }

int32_t hmi_queue_destroy(hmi_queue_t* q) {
  if (!q) return HMI_OK;
  (void)hipSetDevice(q->cfg.device);
  (void)hipStreamSynchronize(hmi_internal_compute_stream(q->pool));
  for (auto& b : q->ring) {
    (void)hipFree(b.x);
    (void)hipFree(b.y);
    if (b.src) (void)hipHostFree(b.src);
    if (b.tok_off) (void)hipHostFree(b.tok_off);
    if (b.gathered) (void)hipEventDestroy(b.gathered);
  }
  delete q;
  return HMI_OK;
}

}  // extern "C"
