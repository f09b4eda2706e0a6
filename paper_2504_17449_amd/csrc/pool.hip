// libhmi host side: the tenant pool (HBM slots, optional pinned-host tier with LRU
// swap-in on a side stream) and the per-block kernel sequence behind hmi_layer_forward.
// See include/hmi.h for the contract of every entry point.
//
// Paper passages realised here: instances are created once and their task parameters
// kept in host memory, fetched to the GPU when requested (Sec. 5.2); loading and compute
// run on different streams so that they overlap, per batch and per layer (Sec. 6.2);
// one batch mixes tenants and is executed in one set of launches (Sec. 6.3).
#include "../../include/hmi.h"
#include "hmi_kernels.h"
#include "pool_internal.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <exception>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace hmi;

namespace {

constexpr int kRing = 8;
constexpr size_t kAlign = 256;
constexpr int kArenaImages = 32;  // pinned host images per hipHostMalloc call
constexpr int kMaxTenantIds = 1 << 24;   // tenant id space of one pool
constexpr int kMaxLayers = 1024;

thread_local hmi_pool_t* g_in_creation = nullptr;   // the pool hmi_pool_create is building on this thread, if any
thread_local char g_create_error[256] = "";   // why the calling thread's last hmi_pool_create failed

// Limits of hmi_layer_forward_static and the layout of its routing arrays inside `scratch`.
constexpr int kStaticMaxRequests = 256;
constexpr int kStaticMaxTokens = 32768;
constexpr size_t kStaticTiles0 = kStaticMaxTokens / kBf16TileM0 + kStaticMaxRequests + 1;
constexpr size_t kStaticTiles1 = kStaticMaxTokens / kBf16TileM1 + kStaticMaxRequests + 1;
constexpr size_t kStaticIndexInts =              // nine per-request arrays, three of them one entry longer; three counters
    (size_t)kStaticMaxRequests * 9 + 3 + 3;
constexpr size_t kStaticScratchInts =
    kStaticIndexInts
    + kStaticMaxTokens                            // row_src
    + 2 * (kStaticTiles0 + kStaticTiles1);        // the two m-tile lists

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Events for work enqueued in order on one stream, addressed by a growing sequence
// number.  Waiting for sequence s means waiting for the newest recorded event whose
// sequence is >= s and still in the ring (a later event on the same stream implies s).
struct EventRing {
  hipEvent_t ev[kRing] = {};
  uint64_t next = 1;  // sequence the next record() will get
  bool init() {
    for (auto& e : ev)
      if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return false;
    return true;
  }
  void destroy() {
    for (auto& e : ev)
      if (e) (void)hipEventDestroy(e);
  }
  uint64_t record(hipStream_t s) {
    (void)hipEventRecord(ev[next % kRing], s);
    return next++;
  }
  hipEvent_t at_least(uint64_t seq) const {
    uint64_t newest = next - 1;
    uint64_t oldest = newest >= (uint64_t)kRing ? newest - kRing + 1 : 1;
    return ev[std::max(seq, oldest) % kRing];
  }
};

struct TensorLoc { size_t off, bytes; };

}  // namespace

// Routing arrays of hmi_layer_forward_static (0.17 MB per GPU, held until the process ends).  In host
// code this name only stands for the symbol: device_setup() asks each device for the address of its
// own copy and every use below goes through that address.
static __device__ __align__(256) int32_t scratch[kStaticScratchInts];

namespace {
// Per-device set-up, once per device and process: the kernels' dynamic-LDS limits and the number
// of compute units.  Guarded, so that pools may be created from several threads.
constexpr int kMaxDevices = 64;
std::mutex g_device_mu;
int g_device_cus[kMaxDevices] = {};        // 0 = this device has not been set up yet
int32_t* g_scratch_ptr[kMaxDevices] = {};  // each device's own copy of `scratch`

// Call with `device` current.  Returns its compute-unit count, or 0 on failure.
int device_setup(int device) {
  if (device < 0 || device >= kMaxDevices) return 0;
  std::lock_guard<std::mutex> lock(g_device_mu);
  if (g_device_cus[device] == 0) {
    int n_cu = 0;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n_cu < 1) return 0;
    init_gemm_bf16_kernels();
    init_gemm_bf16_p256_kernels();
    init_gemm_bf16_skinny_kernels();
    init_adapter_bf16_kernels();
    if (hipGetLastError() != hipSuccess) return 0;
    int32_t* ptr = nullptr;
    if (hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return 0;
    g_scratch_ptr[device] = ptr;
    g_device_cus[device] = n_cu;
  }
  return g_device_cus[device];
}
}  // namespace

struct hmi_pool {
  hmi_pool_config_t cfg{};
  int esize = 2;
  bool bf16 = true;
  std::vector<TensorLoc> tl;   // inside one (tenant, layer) image
  size_t image_bytes = 0;      // one layer
  size_t slot_stride = 0;      // all layers of a tenant
  char* d_pool = nullptr;

  // residency
  std::vector<int32_t> slot_of_tenant, tenant_of_slot;
  std::vector<uint8_t> loaded;       // [tenant*L + layer] weights registered
  std::vector<uint8_t> slot_valid;   // [slot*L + layer] HBM copy present (or in flight)
  std::vector<uint64_t> slot_stamp;  // LRU clock of last use
  std::vector<uint64_t> slot_fwd;    // forward sequence that last read the slot
  std::vector<uint64_t> slot_copy;   // copy sequence that last wrote the slot
  std::vector<int32_t> free_slots;
  uint64_t clock = 0;
  std::vector<char*> host_img;       // [tenant] pinned, all layers (host tier)
  std::vector<int32_t> alias_of;     // [tenant] the tenant whose pinned image this one shares (-1: its own)
  std::vector<int32_t> alias_count;  // [tenant] tenants that share this one's image
  std::vector<char*> arenas;
  char* arena_cur = nullptr;
  int arena_left = 0;

  // streams and ordering
  hipStream_t compute = nullptr, copy = nullptr;
  EventRing fwd_done, copy_done;
  uint64_t copy_waited_fwd = 0;     // copy stream has waited for forwards up to here
  uint64_t compute_waited_copy = 0; // compute stream has waited for copies up to here

  // staging for load_tenant without host tier
  char* stage[2] = {nullptr, nullptr};
  hipEvent_t stage_ev[2] = {};
  int stage_i = 0;

  // per-call index staging (pinned) and device index arrays
  int32_t* h_idx[4] = {};
  hipEvent_t idx_ev[4] = {};
  int idx_i = 0;
  int32_t* d_idx = nullptr;   // all device int32 routing arrays, one allocation
  Route rt{};
  int last_R = 0;
  int tile_m[2] = {256, 128};
  bool adapter_fused = false;  // bf16 adapter images keep their matrices in operand order, one kernel
  int rank = 0;                // adapter bottleneck width (ADAPTER: d_ff, ENC_ADAPTER: adapter_rank)

  // parameters shared by all tenants (ENC_ADAPTER): one encoder-layer image per layer
  std::vector<TensorLoc> stl;
  size_t shared_image_bytes = 0;
  char* d_shared = nullptr;
  std::vector<uint8_t> shared_loaded;
  Route rt_dense{};            // route for GEMMs / LayerNorms that read them

  // per-tenant output heads (max_classes > 0): all resident, [kHeadCols][d] weights + [kHeadCols] biases each
  char* d_heads = nullptr;
  size_t head_stride = 0;
  int32_t* d_head_meta = nullptr;      // [tenant] {n_classes, per_token}
  std::vector<uint8_t> head_loaded;
  std::vector<int32_t> last_distinct;  // tenants of the last routed batch
  int last_n_mtiles[2] = {0, 0};       // its m-tile counts
  int last_N = 0;                      // and rows
  float* w_scores = nullptr;           // [max_tokens, kHeadCols] raw scores

  // key/value cache for decoding (hmi_kv_create): [layer][sequence slot][k | v][head][position][64] bf16
  uint16_t* d_kv = nullptr;
  int kv_seqs = 0, kv_max_len = 0;
  std::vector<int32_t> kv_len;         // positions held per sequence slot
  std::vector<uint32_t> kv_mark;       // duplicate check per call
  uint32_t kv_epoch = 0;

  // workspaces
  char *w_qkv = nullptr, *w_ctx = nullptr, *w_hmid = nullptr, *w_act = nullptr;
  float *w_z = nullptr, *w_x1 = nullptr, *w_y32 = nullptr;
  char* w_yst = nullptr;       // inter-layer activations of a multi-layer call

  // host scratch, sized at creation: the forward calls allocate nothing
  std::vector<uint32_t> mark;       // [tenant] epoch when last seen in a batch
  std::vector<int32_t> tok_count;   // [tenant]
  std::vector<int32_t> distinct;    // capacity max_requests
  std::vector<int32_t> ones;        // [max_requests] the sequence lengths of a decode step
  uint32_t epoch = 0;

  int64_t hits = 0, misses = 0, bytes_h2d = 0, evictions = 0;

  // optional per-kernel timing (hipEvents around each launch on the compute stream)
  bool profiling = false;
  struct Span { int kind; hipEvent_t a, b; };
  std::vector<Span> spans;
  char err[256] = "";
};

namespace {

int32_t fail(hmi_pool* p, int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(p ? p->err : g_create_error, 256, fmt, ap);
  va_end(ap);
  // A failed runtime call also stays behind as the runtime's "last error", where the caller's next, unrelated check
  // (torch makes one after every operation) would find it: it has been reported through the status, so take it out.
  if (code == HMI_ERR_OOM || code == HMI_ERR_DEVICE) (void)hipGetLastError();
  return code;
}

#define HIP_TRY(p, call)                                                              \
  do {                                                                                \
    hipError_t e_ = (call);                                                           \
    if (e_ != hipSuccess)                                                             \
      return fail(p, e_ == hipErrorOutOfMemory ? HMI_ERR_OOM : HMI_ERR_DEVICE,        \
                  "%s failed: %s", #call, hipGetErrorString(e_));                     \
  } while (0)

// Canonical tensor shapes (rows, cols) per block; cols == 0 for vectors.
std::vector<std::pair<int64_t, int64_t>> tensor_shapes(const hmi_pool_config_t& c) {
  const int64_t d = c.d_model, f = c.d_ff;
  std::vector<std::pair<int64_t, int64_t>> ffn = {{f, d}, {f, 0}, {d, f}, {d, 0}};
  std::vector<std::pair<int64_t, int64_t>> out;
  switch (c.block) {
    case HMI_BLOCK_FFN:
      out = ffn; out.push_back({d, 0}); out.push_back({d, 0}); break;
    case HMI_BLOCK_ENC_POSTLN:
    case HMI_BLOCK_DEC_PRELN:
      out = {{3 * d, d}, {3 * d, 0}, {d, d}, {d, 0}, {d, 0}, {d, 0}};
      out.insert(out.end(), ffn.begin(), ffn.end());
      out.push_back({d, 0}); out.push_back({d, 0}); break;
    case HMI_BLOCK_ADAPTER:
      out = ffn; break;
    case HMI_BLOCK_ENC_ADAPTER:
    case HMI_BLOCK_DEC_ADAPTER: {
      const int64_t r = c.adapter_rank;
      out = {{r, d}, {r, 0}, {d, r}, {d, 0}}; break;
    }
  }
  return out;
}

// Tensors of the layer that all tenants of an ENC_ADAPTER pool share: an ENC_POSTLN set.
std::vector<std::pair<int64_t, int64_t>> shared_tensor_shapes(const hmi_pool_config_t& c) {
  if (c.block != HMI_BLOCK_ENC_ADAPTER && c.block != HMI_BLOCK_DEC_ADAPTER) return {};
  hmi_pool_config_t e = c;
  e.block = HMI_BLOCK_ENC_POSTLN;
  return tensor_shapes(e);
}

enum { T_W1 = 0, T_B1, T_W2, T_B2, T_LNG, T_LNB };                      // FFN / ADAPTER
enum { A_WQKV = 0, A_BQKV, A_WO, A_BO, A_LN1G, A_LN1B, A_W1, A_B1, A_W2, A_B2, A_LN2G, A_LN2B };

void free_all(hmi_pool* p) {
  if (g_in_creation == p) g_in_creation = nullptr;
  (void)hipStreamSynchronize(p->compute);
  if (p->copy) (void)hipStreamSynchronize(p->copy);
  (void)hipFree(p->d_pool);
  (void)hipFree(p->d_shared);
  (void)hipFree(p->d_heads);
  (void)hipFree(p->d_head_meta);
  (void)hipFree(p->w_scores);
  (void)hipFree(p->d_kv);
  (void)hipFree(p->d_idx);
  (void)hipFree(p->w_qkv); (void)hipFree(p->w_ctx); (void)hipFree(p->w_hmid);
  (void)hipFree(p->w_act); (void)hipFree(p->w_z); (void)hipFree(p->w_x1);
  (void)hipFree(p->w_y32); (void)hipFree(p->w_yst);
  for (char* a : p->arenas) (void)hipHostFree(a);
  for (int i = 0; i < 2; ++i) {
    if (p->stage[i]) (void)hipHostFree(p->stage[i]);
    if (p->stage_ev[i]) (void)hipEventDestroy(p->stage_ev[i]);
  }
  for (int i = 0; i < 4; ++i) {
    if (p->h_idx[i]) (void)hipHostFree(p->h_idx[i]);
    if (p->idx_ev[i]) (void)hipEventDestroy(p->idx_ev[i]);
  }
  for (auto& sp : p->spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
  p->fwd_done.destroy();
  p->copy_done.destroy();
  if (p->copy) (void)hipStreamDestroy(p->copy);
  delete p;
}

// Make the copy stream wait until every forward that read `slot` has finished.
void copy_waits_for_slot_readers(hmi_pool* p, int slot) {
  const uint64_t need = p->slot_fwd[slot];
  if (need > p->copy_waited_fwd) {
    (void)hipStreamWaitEvent(p->copy, p->fwd_done.at_least(need), 0);
    p->copy_waited_fwd = need;
  }
}

// Take a slot for `tenant`: a free one, else the least recently used slot whose stamp is
// older than `protect_from` (slots stamped at or after it belong to the batch being set
// up).  Ties on the stamp go to the lowest tenant id.  Returns -1 if none.
int acquire_slot(hmi_pool* p, int tenant, uint64_t protect_from) {
  int slot = -1;
  if (!p->free_slots.empty()) {
    slot = p->free_slots.back();
    p->free_slots.pop_back();
  } else {
    if (!p->cfg.host_tier) return -1;
    uint64_t best_stamp = ~0ull;
    int best_tenant = 0;
    for (int s = 0; s < p->cfg.hbm_slots; ++s) {
      const uint64_t st = p->slot_stamp[s];
      if (st >= protect_from) continue;
      const int tn = p->tenant_of_slot[s];
      if (st < best_stamp || (st == best_stamp && tn < best_tenant)) {
        best_stamp = st; best_tenant = tn; slot = s;
      }
    }
    if (slot < 0) return -1;
    p->slot_of_tenant[p->tenant_of_slot[slot]] = -1;
    ++p->evictions;
  }
  p->tenant_of_slot[slot] = tenant;
  p->slot_of_tenant[tenant] = slot;
  for (int l = 0; l < p->cfg.n_layers; ++l) p->slot_valid[(size_t)slot * p->cfg.n_layers + l] = 0;
  return slot;
}

// A tenant whose layers together are this small is swapped in whole: one copy of all its layers (they
// are contiguous on both sides) instead of one per layer, whose fixed cost would dominate (adapters:
// 0.2 MB per layer moved at 14 GB/s as single copies).
constexpr size_t kWholeTenantCopyBytes = 4u << 20;

// Enqueue pinned-host -> HBM copy of one (tenant, layer) image on the copy stream.
int32_t enqueue_swap_in(hmi_pool* p, int tenant, int slot, int layer) {
  copy_waits_for_slot_readers(p, slot);
  const int L = p->cfg.n_layers;
  bool whole = L > 1 && p->slot_stride <= kWholeTenantCopyBytes;
  for (int l = 0; whole && l < L; ++l) whole = p->loaded[(size_t)tenant * L + l] != 0;
  const size_t off = whole ? 0 : (size_t)layer * p->image_bytes, bytes = whole ? p->slot_stride : p->image_bytes;
  HIP_TRY(p, hipMemcpyAsync(p->d_pool + (size_t)slot * p->slot_stride + off, p->host_img[tenant] + off, bytes,
                            hipMemcpyHostToDevice, p->copy));
  if (whole) for (int l = 0; l < L; ++l) p->slot_valid[(size_t)slot * L + l] = 1;
  else p->slot_valid[(size_t)slot * L + layer] = 1;
  p->slot_copy[slot] = p->copy_done.next;  // the record() that follows this batch of copies
  p->bytes_h2d += (int64_t)bytes;
  return HMI_OK;
}

// Brackets one kernel launch with timing events when profiling is on.
struct ProfSpan {
  hmi_pool* p; hipEvent_t b = nullptr;
  ProfSpan(hmi_pool* pool, int kind) : p(pool) {
    if (!p->profiling || p->spans.size() >= 65536) return;
    hipEvent_t a;
    if (hipEventCreate(&a) != hipSuccess) return;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); b = nullptr; return; }
    (void)hipEventRecord(a, p->compute);
    p->spans.push_back({kind, a, b});
  }
  ~ProfSpan() { if (b) (void)hipEventRecord(b, p->compute); }
};

// Writes one (tenant, layer) image from the caller's canonical tensors.
void write_image(const hmi_pool* p, char* img, const void* const* tensors) {
  for (size_t i = 0; i < p->tl.size(); ++i) {
    if (p->adapter_fused && i == T_W1) pack_adapter_operand(img + p->tl[i].off, tensors[i], p->rank, p->cfg.d_model);
    else if (p->adapter_fused && i == T_W2) pack_adapter_operand(img + p->tl[i].off, tensors[i], p->cfg.d_model, p->rank);
    else memcpy(img + p->tl[i].off, tensors[i], p->tl[i].bytes);
  }
}

int bits_for(int n) {
  int b = 1;
  while ((1ll << b) < n) ++b;
  return (b + 3) / 4 * 4;
}

}  // namespace

extern "C" {

static int32_t create_impl(const hmi_pool_config_t* cfg, hmi_pool_t** out) {
  if (!cfg || !out) return fail(nullptr, HMI_ERR_ARG, "null config or out pointer");
  const hmi_pool_config_t& c = *cfg;
  if (c.block < HMI_BLOCK_FFN || c.block > HMI_BLOCK_DEC_ADAPTER) return fail(nullptr, HMI_ERR_ARG, "bad block %d", c.block);
  const bool composite = c.block == HMI_BLOCK_ENC_ADAPTER || c.block == HMI_BLOCK_DEC_ADAPTER;
  if (c.dtype != HMI_F32 && c.dtype != HMI_BF16) return fail(nullptr, HMI_ERR_ARG, "bad dtype %d", c.dtype);
  const int mult = c.dtype == HMI_BF16 ? 64 : 16;
  if (c.d_model <= 0 || c.d_ff <= 0 || c.d_model % mult || c.d_ff % mult || c.d_model > 2048)
    return fail(nullptr, HMI_ERR_ARG, "d_model/d_ff must be positive multiples of %d (d_model <= 2048)", mult);
  const bool attn = c.block == HMI_BLOCK_ENC_POSTLN || c.block == HMI_BLOCK_DEC_PRELN || composite;
  if (composite) {
    if (c.adapter_rank <= 0 || c.adapter_rank % mult || c.adapter_rank > c.d_ff)
      return fail(nullptr, HMI_ERR_ARG, "adapter_rank must be a positive multiple of %d and <= d_ff", mult);
    if ((int64_t)c.max_tokens > (int64_t)kMaxRequests * kDenseSegRows)
      return fail(nullptr, HMI_ERR_ARG, "max_tokens must be <= %d for this block", kMaxRequests * kDenseSegRows);
  }
  if (attn) {
    if (c.n_heads <= 0 || c.d_model % c.n_heads) return fail(nullptr, HMI_ERR_ARG, "n_heads must divide d_model");
    const int dh = c.d_model / c.n_heads;
    if (c.dtype == HMI_BF16 ? dh != 64 : dh > 64) return fail(nullptr, HMI_ERR_ARG, "d_head must be 64 (bf16) or <= 64 (f32)");
  }
  if (c.n_layers < 1 || c.max_tenants < 1 || c.hbm_slots < 1 || c.hbm_slots > c.max_tenants)
    return fail(nullptr, HMI_ERR_ARG, "need n_layers >= 1 and 1 <= hbm_slots <= max_tenants");
  // per-tenant and per-(tenant, layer) host tables are made here: keep their sizes sane
  if (c.max_tenants > kMaxTenantIds || c.n_layers > kMaxLayers)
    return fail(nullptr, HMI_ERR_ARG, "max_tenants must be <= %d and n_layers <= %d", kMaxTenantIds, kMaxLayers);
  if (c.max_requests < 1 || c.max_requests > kMaxRequests || c.max_tokens < c.max_requests)
    return fail(nullptr, HMI_ERR_ARG, "need 1 <= max_requests <= %d and max_tokens >= max_requests", kMaxRequests);
  if (!c.host_tier && c.hbm_slots != c.max_tenants)
    return fail(nullptr, HMI_ERR_ARG, "without host_tier every tenant needs a slot: hbm_slots must equal max_tenants");
  if (!(c.ln_eps >= 0.0f)) return fail(nullptr, HMI_ERR_ARG, "ln_eps must be >= 0");
  if (c.max_classes < 0 || c.max_classes > 64) return fail(nullptr, HMI_ERR_ARG, "max_classes must be in [0, 64]");
  // the kernels address activation rows with 32-bit byte offsets
  if ((uint64_t)c.max_tokens * (uint64_t)std::max(c.d_model, c.d_ff) * (c.dtype == HMI_BF16 ? 2u : 4u) >= (1ull << 32))
    return fail(nullptr, HMI_ERR_ARG, "max_tokens * max(d_model, d_ff) * element size must stay below 4 GiB");
  if (c.device < 0 || c.device >= kMaxDevices) return fail(nullptr, HMI_ERR_ARG, "device %d outside [0,%d)", c.device, kMaxDevices);

  hmi_pool* p = new (std::nothrow) hmi_pool();
  if (!p) return fail(nullptr, HMI_ERR_OOM, "host allocation failed");
  p->cfg = c;
  p->bf16 = c.dtype == HMI_BF16;
  p->esize = p->bf16 ? 2 : 4;
  p->tile_m[0] = p->bf16 ? kBf16TileM0 : kF32TileM;
  p->tile_m[1] = p->bf16 ? kBf16TileM1 : 0;
  p->rank = composite ? c.adapter_rank : c.d_ff;
  // The one-kernel adapter reads and writes the storage dtype: inside the shared layer it always
  // can, as a block of its own only where no fp32 activations pass between layers.
  p->adapter_fused = p->bf16 && adapter_bf16_supported(c.d_model, p->rank) &&
                     (composite || (c.block == HMI_BLOCK_ADAPTER && c.n_layers == 1));
  size_t off = 0;
  for (auto& sh : tensor_shapes(c)) {
    const size_t bytes = (size_t)sh.first * (sh.second ? sh.second : 1) * p->esize;
    p->tl.push_back({off, bytes});
    off = align_up(off + bytes, kAlign);
  }
  p->image_bytes = off;
  p->slot_stride = off * c.n_layers;
  // sizes are products of caller-given 32-bit numbers: refuse before any of them can wrap
  if ((unsigned __int128)p->slot_stride * (unsigned)c.hbm_slots >= ((unsigned __int128)1 << 46)) {
    delete p;
    return fail(nullptr, HMI_ERR_OOM, "hbm_slots x n_layers x image bytes exceeds any device");
  }
  g_in_creation = p;   // from here on an exception handler or an error path gives everything back through free_all
  off = 0;
  for (auto& sh : shared_tensor_shapes(c)) {
    const size_t bytes = (size_t)sh.first * (sh.second ? sh.second : 1) * p->esize;
    p->stl.push_back({off, bytes});
    off = align_up(off + bytes, kAlign);
  }
  p->shared_image_bytes = off;
  p->shared_loaded.assign(c.n_layers, 0);

#define CREATE_TRY(call)                                                                        \
  do {                                                                                          \
    hipError_t e_ = (call);                                                                     \
    if (e_ != hipSuccess) {                                                                     \
      int32_t rc = fail(nullptr, e_ == hipErrorOutOfMemory ? HMI_ERR_OOM : HMI_ERR_DEVICE,      \
                        "%s failed: %s", #call, hipGetErrorString(e_));                         \
      free_all(p);                                                                              \
      return rc;                                                                                \
    }                                                                                           \
  } while (0)

  CREATE_TRY(hipSetDevice(c.device));
  const int n_cu = device_setup(c.device);
  if (n_cu == 0) {
    free_all(p);
    return fail(nullptr, HMI_ERR_DEVICE, "kernel set-up on device %d failed", c.device);
  }
  p->compute = reinterpret_cast<hipStream_t>(c.compute_stream);
  CREATE_TRY(hipStreamCreateWithFlags(&p->copy, hipStreamNonBlocking));
  if (!p->fwd_done.init() || !p->copy_done.init()) {
    free_all(p);
    return fail(nullptr, HMI_ERR_DEVICE, "event creation failed");
  }
  CREATE_TRY(hipMalloc(&p->d_pool, p->slot_stride * (size_t)c.hbm_slots));
  if (p->shared_image_bytes) CREATE_TRY(hipMalloc(&p->d_shared, p->shared_image_bytes * (size_t)c.n_layers));
  if (c.max_classes > 0) {
    p->head_stride = align_up((size_t)kHeadCols * (c.d_model + 1) * p->esize, kAlign);
    CREATE_TRY(hipMalloc(&p->d_heads, p->head_stride * (size_t)c.max_tenants));
    CREATE_TRY(hipMemset(p->d_heads, 0, p->head_stride * (size_t)c.max_tenants));
    CREATE_TRY(hipMalloc(&p->w_scores, (size_t)c.max_tokens * kHeadCols * sizeof(float)));
    CREATE_TRY(hipMalloc(&p->d_head_meta, sizeof(int32_t) * 2 * (size_t)c.max_tenants));
    CREATE_TRY(hipMemset(p->d_head_meta, 0, sizeof(int32_t) * 2 * (size_t)c.max_tenants));
    p->head_loaded.assign(c.max_tenants, 0);
  }

  p->slot_of_tenant.assign(c.max_tenants, -1);
  p->tenant_of_slot.assign(c.hbm_slots, -1);
  p->loaded.assign((size_t)c.max_tenants * c.n_layers, 0);
  p->slot_valid.assign((size_t)c.hbm_slots * c.n_layers, 0);
  p->slot_stamp.assign(c.hbm_slots, 0);
  p->slot_fwd.assign(c.hbm_slots, 0);
  p->slot_copy.assign(c.hbm_slots, 0);
  for (int s = c.hbm_slots - 1; s >= 0; --s) p->free_slots.push_back(s);
  if (c.host_tier) {
    p->host_img.assign(c.max_tenants, nullptr);
    p->alias_of.assign(c.max_tenants, -1);
    p->alias_count.assign(c.max_tenants, 0);
  }
  p->mark.assign(c.max_tenants, 0);
  p->tok_count.assign(c.max_tenants, 0);
  p->distinct.reserve(c.max_requests);
  p->last_distinct.reserve(c.max_requests);
  p->ones.assign(c.max_requests, 1);

  if (!c.host_tier) {
    for (int i = 0; i < 2; ++i) {
      CREATE_TRY(hipHostMalloc(&p->stage[i], p->image_bytes, hipHostMallocDefault));
      CREATE_TRY(hipEventCreateWithFlags(&p->stage_ev[i], hipEventDisableTiming));
    }
  }
  const int Rm = c.max_requests;
  for (int i = 0; i < 4; ++i) {
    CREATE_TRY(hipHostMalloc(&p->h_idx[i], sizeof(int32_t) * 5 * Rm, hipHostMallocDefault));
    CREATE_TRY(hipEventCreateWithFlags(&p->idx_ev[i], hipEventDisableTiming));
  }

  // device routing arrays, one allocation
  const size_t MT = (size_t)c.max_tokens;
  const size_t max_tiles0 = MT / p->tile_m[0] + Rm + 1;
  const size_t max_tiles1 = p->tile_m[1] ? MT / p->tile_m[1] + Rm + 1 : 0;
  size_t n_i32 = 3 * (size_t)Rm            // ids, lens, req_slot
                 + 3 * (size_t)Rm          // req_tenant, kv_slot, kv_pos
                 + Rm + (Rm + 1)           // perm, tok_off
                 + 2 * (size_t)Rm          // seg_tenant, seg_slot
                 + 2 * ((size_t)Rm + 1)    // seg_req_off, seg_tok_off
                 + MT                      // row_src
                 + 2 * (max_tiles0 + max_tiles1) + 4   // tile lists + counters
                 + kGemmSchedInts;
  const bool dense = composite;
  const size_t dense_segs = MT / kDenseSegRows + 2;
  const size_t dense_tiles0 = MT / p->tile_m[0] + 2, dense_tiles1 = p->tile_m[1] ? MT / p->tile_m[1] + 2 : 0;
  if (dense) n_i32 += 2 * dense_segs + 1 + MT + 2 * (dense_tiles0 + dense_tiles1);
  CREATE_TRY(hipMalloc(&p->d_idx, n_i32 * sizeof(int32_t)));
  CREATE_TRY(hipMemset(p->d_idx, 0, n_i32 * sizeof(int32_t)));
  int32_t* q = p->d_idx;
  auto take = [&](size_t n) { int32_t* r = q; q += n; return r; };
  Route& rt = p->rt;
  rt.tenant_ids = take(Rm); rt.seq_lens = take(Rm); rt.req_slot = take(Rm);
  rt.req_tenant = take(Rm); rt.kv_slot = take(Rm); rt.kv_pos = take(Rm);
  rt.perm = take(Rm); rt.tok_off = take(Rm + 1);
  rt.seg_tenant = take(Rm); rt.seg_slot = take(Rm);
  rt.seg_req_off = take(Rm + 1); rt.seg_tok_off = take(Rm + 1);
  rt.row_src = take(MT);
  rt.tile_seg[0] = take(max_tiles0); rt.tile_row0[0] = take(max_tiles0);
  rt.tile_seg[1] = max_tiles1 ? take(max_tiles1) : nullptr;
  rt.tile_row0[1] = max_tiles1 ? take(max_tiles1) : nullptr;
  rt.n_segments = take(1); rt.n_tiles[0] = take(1); rt.n_tiles[1] = take(1);
  rt.gemm_sched = take(kGemmSchedInts);
  rt.tile_m[0] = p->tile_m[0]; rt.tile_m[1] = p->tile_m[1];
  rt.key_bits = bits_for(c.max_tenants);
  rt.n_cu = n_cu;
  if (dense) {
    // Route for the shared parameters: identity row map, pseudo-segments of kDenseSegRows rows
    // that all name slot 0 (the GEMMs get a slot stride of 0), tiles in row order.  Only the
    // segment offsets depend on the batch (its N); the router writes them.
    Route& rd = p->rt_dense;
    rd = rt;
    rd.seg_slot = take(dense_segs);            // stays zero
    rd.seg_tok_off = take(dense_segs);
    rd.n_segments = take(1);
    rd.row_src = take(MT);
    rd.tile_seg[0] = take(dense_tiles0); rd.tile_row0[0] = take(dense_tiles0);
    rd.tile_seg[1] = dense_tiles1 ? take(dense_tiles1) : nullptr;
    rd.tile_row0[1] = dense_tiles1 ? take(dense_tiles1) : nullptr;
    rt.dense_seg_tok_off = rd.seg_tok_off;
    rt.dense_n_segments = rd.n_segments;
    rd.dense_seg_tok_off = nullptr; rd.dense_n_segments = nullptr;
    rd.identity = 1;
    std::vector<int32_t> h(MT);
    for (size_t i = 0; i < MT; ++i) h[i] = (int32_t)i;
    CREATE_TRY(hipMemcpy(rd.row_src, h.data(), MT * sizeof(int32_t), hipMemcpyHostToDevice));
    for (int k = 0; k < 2; ++k) {
      const size_t nt = k == 0 ? dense_tiles0 : dense_tiles1;
      if (!nt) continue;
      std::vector<int32_t> seg(nt), row0(nt);
      for (size_t t = 0; t < nt; ++t) {
        row0[t] = (int32_t)(t * p->tile_m[k]);
        seg[t] = (int32_t)(t * p->tile_m[k] / kDenseSegRows);
      }
      CREATE_TRY(hipMemcpy(rd.tile_seg[k], seg.data(), nt * sizeof(int32_t), hipMemcpyHostToDevice));
      CREATE_TRY(hipMemcpy(rd.tile_row0[k], row0.data(), nt * sizeof(int32_t), hipMemcpyHostToDevice));
    }
  }

  const size_t d = c.d_model, f = c.d_ff, es = p->esize;
  CREATE_TRY(hipMalloc(&p->w_hmid, MT * f * es));
  if (c.block == HMI_BLOCK_FFN) {
    CREATE_TRY(hipMalloc(&p->w_z, MT * d * sizeof(float)));
  } else if (attn) {
    CREATE_TRY(hipMalloc(&p->w_qkv, MT * 3 * d * es));
    CREATE_TRY(hipMalloc(&p->w_ctx, MT * d * es));
    CREATE_TRY(hipMalloc(&p->w_act, MT * d * es));
    CREATE_TRY(hipMalloc(&p->w_z, MT * d * sizeof(float)));
    CREATE_TRY(hipMalloc(&p->w_x1, MT * d * sizeof(float)));
  }
  if (c.n_layers > 1) {
    CREATE_TRY(hipMalloc(&p->w_y32, MT * d * sizeof(float)));
    CREATE_TRY(hipMalloc(&p->w_yst, MT * d * es));
  }
#undef CREATE_TRY
  g_in_creation = nullptr;
  *out = p;
  return HMI_OK;
}

int32_t hmi_pool_create(const hmi_pool_config_t* cfg, hmi_pool_t** out) {
  try {
    return create_impl(cfg, out);
  } catch (const std::exception& e) {   // a host table could not be allocated: nothing may cross the C boundary
    if (g_in_creation) free_all(g_in_creation);
    return fail(nullptr, HMI_ERR_OOM, "host allocation failed: %s", e.what());
  }
}

int32_t hmi_pool_load_tenant(hmi_pool_t* p, int32_t tenant, int32_t layer,
                             const void* const* tensors, int32_t n_tensors) {
  if (!p) return HMI_ERR_ARG;
  if (!tensors) return fail(p, HMI_ERR_ARG, "null tensor list");
  if (tenant < 0 || tenant >= p->cfg.max_tenants) return fail(p, HMI_ERR_TENANT, "tenant %d outside [0,%d)", tenant, p->cfg.max_tenants);
  if (layer < 0 || layer >= p->cfg.n_layers) return fail(p, HMI_ERR_ARG, "layer %d outside [0,%d)", layer, p->cfg.n_layers);
  if (n_tensors != (int32_t)p->tl.size()) return fail(p, HMI_ERR_SHAPE, "block needs %d tensors, got %d", (int)p->tl.size(), n_tensors);
  for (int i = 0; i < n_tensors; ++i)
    if (!tensors[i]) return fail(p, HMI_ERR_ARG, "tensor %d is null", i);
  HIP_TRY(p, hipSetDevice(p->cfg.device));
  const int L = p->cfg.n_layers;

  if (p->cfg.host_tier) {
    if (p->alias_of[tenant] >= 0 || p->alias_count[tenant] > 0)
      return fail(p, HMI_ERR_ARG, "tenant %d shares its image with other tenants: it cannot be loaded again", tenant);
    if (!p->host_img[tenant]) {
      if (p->arena_left == 0) {
        char* a = nullptr;
        HIP_TRY(p, hipHostMalloc(&a, p->slot_stride * (size_t)kArenaImages, hipHostMallocDefault));
        p->arenas.push_back(a);
        p->arena_cur = a;
        p->arena_left = kArenaImages;
      }
      p->host_img[tenant] = p->arena_cur;
      p->arena_cur += p->slot_stride;
      --p->arena_left;
    }
    int slot = p->slot_of_tenant[tenant];
    if (slot >= 0 && p->slot_valid[(size_t)slot * L + layer]) {
      // replacing weights that may be in use or in flight: drain both streams first
      HIP_TRY(p, hipStreamSynchronize(p->compute));
      HIP_TRY(p, hipStreamSynchronize(p->copy));
    }
    char* img = p->host_img[tenant] + (size_t)layer * p->image_bytes;
    write_image(p, img, tensors);
    p->loaded[(size_t)tenant * L + layer] = 1;
    if (slot < 0 && !p->free_slots.empty()) slot = acquire_slot(p, tenant, 0);
    if (slot >= 0) {
      const int64_t before = p->bytes_h2d;
      int32_t rc = enqueue_swap_in(p, tenant, slot, layer);
      if (rc != HMI_OK) return rc;
      p->bytes_h2d = before;  // initial placement is not swap traffic
      p->copy_done.record(p->copy);
    }
    return HMI_OK;
  }

  int slot = p->slot_of_tenant[tenant];
  if (slot < 0) {
    slot = acquire_slot(p, tenant, 0);
    if (slot < 0) return fail(p, HMI_ERR_CAPACITY, "no HBM slot left for tenant %d", tenant);
  } else if (p->slot_valid[(size_t)slot * L + layer]) {
    HIP_TRY(p, hipStreamSynchronize(p->compute));
  }
  const int si = p->stage_i;
  p->stage_i ^= 1;
  HIP_TRY(p, hipEventSynchronize(p->stage_ev[si]));  // staging buffer free again
  write_image(p, p->stage[si], tensors);
  char* dst = p->d_pool + (size_t)slot * p->slot_stride + (size_t)layer * p->image_bytes;
  HIP_TRY(p, hipMemcpyAsync(dst, p->stage[si], p->image_bytes, hipMemcpyHostToDevice, p->copy));
  HIP_TRY(p, hipEventRecord(p->stage_ev[si], p->copy));
  p->slot_copy[slot] = p->copy_done.next;
  p->copy_done.record(p->copy);
  p->slot_valid[(size_t)slot * L + layer] = 1;
  p->loaded[(size_t)tenant * L + layer] = 1;
  return HMI_OK;
}

int32_t hmi_pool_alias_tenant(hmi_pool_t* p, int32_t tenant, int32_t source) {
  if (!p) return HMI_ERR_ARG;
  const hmi_pool_config_t& c = p->cfg;
  if (!c.host_tier) return fail(p, HMI_ERR_ARG, "tenants can share an image only in a pool with a host tier");
  if (tenant < 0 || tenant >= c.max_tenants || source < 0 || source >= c.max_tenants)
    return fail(p, HMI_ERR_TENANT, "tenant %d or %d outside [0,%d)", tenant, source, c.max_tenants);
  if (tenant == source) return fail(p, HMI_ERR_ARG, "a tenant cannot share its own image");
  const int L = c.n_layers;
  if (p->alias_of[source] >= 0) source = p->alias_of[source];
  for (int l = 0; l < L; ++l)
    if (!p->loaded[(size_t)source * L + l]) return fail(p, HMI_ERR_TENANT, "tenant %d (layer %d) is not loaded", source, l);
  if (p->host_img[tenant]) return fail(p, HMI_ERR_ARG, "tenant %d already has parameters", tenant);
  HIP_TRY(p, hipSetDevice(c.device));
  p->host_img[tenant] = p->host_img[source];
  p->alias_of[tenant] = source;
  ++p->alias_count[source];
  for (int l = 0; l < L; ++l) p->loaded[(size_t)tenant * L + l] = 1;
  if (!p->free_slots.empty()) {     // like a loaded tenant, it takes a free HBM slot while there is one
    const int slot = acquire_slot(p, tenant, 0);
    const int64_t before = p->bytes_h2d;
    for (int l = 0; l < L; ++l) {
      if (p->slot_valid[(size_t)slot * L + l]) continue;     // a whole-tenant copy brought every layer
      int32_t rc = enqueue_swap_in(p, tenant, slot, l);
      if (rc != HMI_OK) return rc;
    }
    p->bytes_h2d = before;          // initial placement is not swap traffic
    p->copy_done.record(p->copy);
  }
  return HMI_OK;
}

int32_t hmi_pool_load_shared(hmi_pool_t* p, int32_t layer, const void* const* tensors, int32_t n_tensors) {
  if (!p) return HMI_ERR_ARG;
  if (p->stl.empty()) return fail(p, HMI_ERR_ARG, "this block kind has no shared parameters");
  if (!tensors) return fail(p, HMI_ERR_ARG, "null tensor list");
  if (layer < 0 || layer >= p->cfg.n_layers) return fail(p, HMI_ERR_ARG, "layer %d outside [0,%d)", layer, p->cfg.n_layers);
  if (n_tensors != (int32_t)p->stl.size()) return fail(p, HMI_ERR_SHAPE, "the shared layer has %d tensors, got %d", (int)p->stl.size(), n_tensors);
  for (int i = 0; i < n_tensors; ++i)
    if (!tensors[i]) return fail(p, HMI_ERR_ARG, "tensor %d is null", i);
  HIP_TRY(p, hipSetDevice(p->cfg.device));
  if (p->shared_loaded[layer]) HIP_TRY(p, hipStreamSynchronize(p->compute));   // may still be read
  char* stage = nullptr;
  HIP_TRY(p, hipHostMalloc(&stage, p->shared_image_bytes, hipHostMallocDefault));
  for (int i = 0; i < n_tensors; ++i) memcpy(stage + p->stl[i].off, tensors[i], p->stl[i].bytes);
  hipError_t e = hipMemcpyAsync(p->d_shared + (size_t)layer * p->shared_image_bytes, stage, p->shared_image_bytes,
                                hipMemcpyHostToDevice, p->copy);
  if (e == hipSuccess) e = hipStreamSynchronize(p->copy);   // in HBM before return: later forwards need no event
  (void)hipHostFree(stage);
  if (e != hipSuccess) return fail(p, HMI_ERR_DEVICE, "copy of the shared layer failed: %s", hipGetErrorString(e));
  p->shared_loaded[layer] = 1;
  return HMI_OK;
}

int32_t hmi_pool_load_head(hmi_pool_t* p, int32_t tenant, const void* w, const void* b, int32_t n_classes,
                           int32_t per_token) {
  if (!p) return HMI_ERR_ARG;
  const hmi_pool_config_t& c = p->cfg;
  if (c.max_classes <= 0) return fail(p, HMI_ERR_ARG, "the pool was created without output heads (max_classes = 0)");
  if (!w || !b) return fail(p, HMI_ERR_ARG, "null head tensor");
  if (tenant < 0 || tenant >= c.max_tenants) return fail(p, HMI_ERR_TENANT, "tenant %d outside [0,%d)", tenant, c.max_tenants);
  if (n_classes < 1 || n_classes > c.max_classes) return fail(p, HMI_ERR_SHAPE, "n_classes %d outside [1,%d]", n_classes, c.max_classes);
  HIP_TRY(p, hipSetDevice(c.device));
  if (p->head_loaded[tenant]) HIP_TRY(p, hipStreamSynchronize(p->compute));   // may still be read
  char* dst = p->d_heads + (size_t)tenant * p->head_stride;
  if (p->head_loaded[tenant]) HIP_TRY(p, hipMemset(dst, 0, p->head_stride));   // rows the new head does not have
  HIP_TRY(p, hipMemcpy(dst, w, (size_t)n_classes * c.d_model * p->esize, hipMemcpyHostToDevice));
  HIP_TRY(p, hipMemcpy(dst + (size_t)kHeadCols * c.d_model * p->esize, b, (size_t)n_classes * p->esize, hipMemcpyHostToDevice));
  const int32_t meta[2] = {n_classes, per_token ? 1 : 0};
  HIP_TRY(p, hipMemcpy(p->d_head_meta + 2 * (size_t)tenant, meta, sizeof(meta), hipMemcpyHostToDevice));
  p->head_loaded[tenant] = 1;
  return HMI_OK;
}

int32_t hmi_head_forward(hmi_pool_t* p, const void* h, float* scores, int32_t* labels) {
  if (!p) return HMI_ERR_ARG;
  const hmi_pool_config_t& c = p->cfg;
  if (c.max_classes <= 0) return fail(p, HMI_ERR_ARG, "the pool was created without output heads (max_classes = 0)");
  if (!h || !labels) return fail(p, HMI_ERR_ARG, "null pointer");
  if (p->last_R <= 0) return fail(p, HMI_ERR_ARG, "no forward call has routed a batch yet");
  for (int t : p->last_distinct)
    if (!p->head_loaded[t]) return fail(p, HMI_ERR_TENANT, "tenant %d has no output head", t);
  HIP_TRY(p, hipSetDevice(c.device));
  // raw scores: grouped GEMM over the tenant route of that batch; heads are indexed by tenant, not by slot
  Route rh = p->rt;
  rh.seg_slot = p->rt.seg_tenant;
  GemmArgs g{};
  g.A = h; g.lda = c.d_model; g.C = p->w_scores; g.ldc = kHeadCols; g.out_f32 = 1;
  g.pool = p->d_heads; g.slot_stride = p->head_stride;
  g.w_off = 0; g.b_off = (size_t)kHeadCols * c.d_model * p->esize;
  g.n_out = kHeadCols; g.k = c.d_model; g.n_rows = p->last_N; g.epi = EPI_BIAS;
  g.n_mtiles_list[0] = p->last_n_mtiles[0]; g.n_mtiles_list[1] = p->last_n_mtiles[1];
  g.which_tiles = 0; g.n_mtiles = g.n_mtiles_list[0];
  if (p->bf16) launch_gemm_bf16(g, rh, p->compute); else launch_gemm_f32(g, rh, p->compute);
  HeadArgs a{};
  a.raw = p->w_scores; a.scores = scores; a.labels = labels; a.meta = p->d_head_meta; a.max_classes = c.max_classes;
  launch_head_select(a, p->rt, p->last_R, p->compute);
  HIP_TRY(p, hipGetLastError());
  return HMI_OK;
}

int32_t hmi_plot_aggregate(hmi_pool_t* p, const void* table, int32_t n_entries, const int32_t* frag_ids,
                           const int32_t* seq_lens, int32_t R, void* x) {
  if (!p) return HMI_ERR_ARG;
  if (R == 0) return HMI_OK;
  const hmi_pool_config_t& c = p->cfg;
  if (R < 0 || !table || !frag_ids || !seq_lens || !x || n_entries < 1) return fail(p, HMI_ERR_ARG, "null pointer, empty table or negative request count");
  if (R > c.max_requests) return fail(p, HMI_ERR_SHAPE, "%d requests > max_requests %d", R, c.max_requests);
  int64_t N = 0;
  for (int r = 0; r < R; ++r) {
    if (seq_lens[r] <= 0) return fail(p, HMI_ERR_SHAPE, "seq_lens[%d] = %d", r, seq_lens[r]);
    N += seq_lens[r];
    if (N > c.max_tokens) return fail(p, HMI_ERR_SHAPE, "batch has more than max_tokens = %d tokens", c.max_tokens);
  }
  HIP_TRY(p, hipSetDevice(c.device));
  // request offsets go through one of the pinned index buffers (the kernel reads them in place)
  const int bi = p->idx_i;
  p->idx_i = (p->idx_i + 1) & 3;
  HIP_TRY(p, hipEventSynchronize(p->idx_ev[bi]));
  int32_t* h = p->h_idx[bi];
  h[0] = 0;
  for (int r = 0; r < R; ++r) h[r + 1] = h[r] + seq_lens[r];
  PlotArgs a{};
  a.table = static_cast<const char*>(table); a.n_entries = n_entries; a.frag_ids = frag_ids; a.tok_off = h;
  a.x = static_cast<char*>(x); a.d = c.d_model;
  launch_plot_aggregate(a, R, p->bf16, p->compute);
  HIP_TRY(p, hipEventRecord(p->idx_ev[bi], p->compute));
  HIP_TRY(p, hipGetLastError());
  return HMI_OK;
}

int32_t hmi_pool_prefetch(hmi_pool_t* p, int32_t layer, const int32_t* ids, int32_t n) {
  if (!p) return HMI_ERR_ARG;
  if (n < 0 || (n > 0 && !ids)) return fail(p, HMI_ERR_ARG, "bad tenant list");
  if (layer < 0 || layer >= p->cfg.n_layers) return fail(p, HMI_ERR_ARG, "layer %d outside [0,%d)", layer, p->cfg.n_layers);
  if (!p->cfg.host_tier || n == 0) return HMI_OK;
  HIP_TRY(p, hipSetDevice(p->cfg.device));
  const int L = p->cfg.n_layers;
  for (int i = 0; i < n; ++i) {
    const int t = ids[i];
    if (t < 0 || t >= p->cfg.max_tenants || !p->loaded[(size_t)t * L + layer])
      return fail(p, HMI_ERR_TENANT, "tenant %d (layer %d) is not loaded", t, layer);
  }
  const uint64_t now = ++p->clock;
  for (int i = 0; i < n; ++i) {  // keep what is already here
    const int s = p->slot_of_tenant[ids[i]];
    if (s >= 0) p->slot_stamp[s] = now;
  }
  bool copied = false;
  for (int i = 0; i < n; ++i) {
    const int t = ids[i];
    int s = p->slot_of_tenant[t];
    if (s < 0) {
      s = acquire_slot(p, t, now);
      if (s < 0) break;  // best effort
      p->slot_stamp[s] = now;
    }
    if (!p->slot_valid[(size_t)s * L + layer]) {
      int32_t rc = enqueue_swap_in(p, t, s, layer);
      if (rc != HMI_OK) return rc;
      copied = true;
    }
  }
  if (copied) p->copy_done.record(p->copy);
  return HMI_OK;
}

namespace {
enum { KV_NONE = 0, KV_PREFILL = 1, KV_DECODE = 2 };
}

// The forward of layers [layer_begin, layer_end) over one batch.  kv: KV_PREFILL also stores every
// row's key and value in the request's cache line seq_slots[r] (from position 0); KV_DECODE takes
// one row per request (seq_lens == nullptr), appends it to the line and attends over the line.
static int32_t forward_impl(hmi_pool_t* p, int32_t layer_begin, int32_t layer_end, const void* x, void* y,
                            const int32_t* tenant_ids, const int32_t* seq_lens, int32_t R, int kv,
                            const int32_t* seq_slots, bool y_f32 = false) {
  if (!p) return HMI_ERR_ARG;
  if (R == 0) return HMI_OK;
  if (y_f32 && p->cfg.block == HMI_BLOCK_ADAPTER && p->adapter_fused)
    return fail(p, HMI_ERR_ARG, "fp32 output is not available from the one-kernel adapter");
  if (kv == KV_DECODE && R > 0 && R <= p->cfg.max_requests) seq_lens = p->ones.data();
  if (R > p->cfg.max_requests) return fail(p, HMI_ERR_SHAPE, "%d requests > max_requests %d", R, p->cfg.max_requests);
  if (R < 0 || !x || !y || !tenant_ids || !seq_lens) return fail(p, HMI_ERR_ARG, "null pointer or negative request count");
  if (x == y) return fail(p, HMI_ERR_ARG, "x and y must be different buffers");
  if (layer_begin < 0 || layer_end > p->cfg.n_layers || layer_begin >= layer_end)
    return fail(p, HMI_ERR_ARG, "layers [%d,%d) outside [0,%d)", layer_begin, layer_end, p->cfg.n_layers);
  const hmi_pool_config_t& c = p->cfg;
  const int L = c.n_layers;
  if (!p->stl.empty())
    for (int l = layer_begin; l < layer_end; ++l)
      if (!p->shared_loaded[l]) return fail(p, HMI_ERR_ARG, "shared parameters of layer %d were never loaded", l);

  // ---- validate, count tokens per distinct tenant
  if (++p->epoch == 0) { std::fill(p->mark.begin(), p->mark.end(), 0u); p->epoch = 1; }
  p->distinct.clear();
  int64_t N = 0;
  int max_len = 0;
  for (int r = 0; r < R; ++r) {
    const int t = tenant_ids[r], len = seq_lens[r];
    if (len <= 0) return fail(p, HMI_ERR_SHAPE, "seq_lens[%d] = %d", r, len);
    if (t < 0 || t >= c.max_tenants) return fail(p, HMI_ERR_TENANT, "tenant_ids[%d] = %d outside [0,%d)", r, t, c.max_tenants);
    for (int l = layer_begin; l < layer_end; ++l)
      if (!p->loaded[(size_t)t * L + l]) return fail(p, HMI_ERR_TENANT, "tenant %d (layer %d) was never loaded", t, l);
    if (p->mark[t] != p->epoch) { p->mark[t] = p->epoch; p->tok_count[t] = 0; p->distinct.push_back(t); }
    p->tok_count[t] += len;
    N += len;
    max_len = std::max(max_len, len);
    if (N > c.max_tokens) return fail(p, HMI_ERR_SHAPE, "batch has more than max_tokens = %d tokens", c.max_tokens);
  }
  const int G = (int)p->distinct.size();
  if (G > c.hbm_slots) return fail(p, HMI_ERR_CAPACITY, "%d distinct tenants in one batch > hbm_slots %d", G, c.hbm_slots);
  if (kv != KV_NONE) {
    if (!p->d_kv) return fail(p, HMI_ERR_ARG, "no key/value cache: call hmi_kv_create first");
    if (!seq_slots) return fail(p, HMI_ERR_ARG, "null seq_slots");
    if (++p->kv_epoch == 0) { std::fill(p->kv_mark.begin(), p->kv_mark.end(), 0u); p->kv_epoch = 1; }
    for (int r = 0; r < R; ++r) {
      const int sl = seq_slots[r];
      if (sl < 0 || sl >= p->kv_seqs) return fail(p, HMI_ERR_ARG, "seq_slots[%d] = %d outside [0,%d)", r, sl, p->kv_seqs);
      if (p->kv_mark[sl] == p->kv_epoch) return fail(p, HMI_ERR_ARG, "sequence slot %d appears twice in one batch", sl);
      p->kv_mark[sl] = p->kv_epoch;
      const int end = kv == KV_PREFILL ? seq_lens[r] : p->kv_len[sl] + 1;
      if (end > p->kv_max_len) return fail(p, HMI_ERR_SHAPE, "sequence slot %d would hold %d positions > max_len %d", sl, end, p->kv_max_len);
    }
  }
  HIP_TRY(p, hipSetDevice(c.device));

  // ---- residency of the first layer: hits first (so they cannot be chosen as victims)
  const uint64_t now = ++p->clock;
  int n_mtiles[2] = {0, 0};
  for (int t : p->distinct) {
    n_mtiles[0] += (p->tok_count[t] + p->tile_m[0] - 1) / p->tile_m[0];
    if (p->tile_m[1]) n_mtiles[1] += (p->tok_count[t] + p->tile_m[1] - 1) / p->tile_m[1];
    const int s = p->slot_of_tenant[t];
    if (s >= 0) p->slot_stamp[s] = now;
  }
  // Brings `layer` of every tenant of the batch into HBM (copy stream); returns the copy
  // sequence the compute stream has to wait for before reading those weights.
  auto make_resident = [&](int layer, bool count, uint64_t* need_out) -> int32_t {
    bool copied = false;
    uint64_t need = 0;
    for (int t : p->distinct) {
      int s = p->slot_of_tenant[t];
      const bool hit = s >= 0 && p->slot_valid[(size_t)s * L + layer];
      if (count) { if (hit) ++p->hits; else ++p->misses; }
      if (s < 0) {
        s = acquire_slot(p, t, now);
        if (s < 0) return fail(p, HMI_ERR_CAPACITY, "no evictable HBM slot for tenant %d", t);
        p->slot_stamp[s] = now;
      }
      if (!p->slot_valid[(size_t)s * L + layer]) {
        int32_t rc = enqueue_swap_in(p, t, s, layer);
        if (rc != HMI_OK) return rc;
        copied = true;
      }
      need = std::max(need, p->slot_copy[s]);
    }
    if (copied) p->copy_done.record(p->copy);
    *need_out = need;
    return HMI_OK;
  };
  // Records the end of the kernels enqueued so far and notes it as the last reader of every slot
  // this batch holds (a swap-in into one of them waits for that event).
  auto mark_slots_read = [&]() {
    const uint64_t seq = p->fwd_done.record(p->compute);
    for (int t : p->distinct) {
      const int sl = p->slot_of_tenant[t];
      if (sl >= 0) p->slot_fwd[sl] = seq;
    }
  };
  uint64_t need_copy = 0;
  {
    int32_t rc = make_resident(layer_begin, true, &need_copy);
    if (rc != HMI_OK) return rc;
  }

  // ---- index arrays to the device
  const int bi = p->idx_i;
  p->idx_i = (p->idx_i + 1) & 3;
  HIP_TRY(p, hipEventSynchronize(p->idx_ev[bi]));
  int32_t* h = p->h_idx[bi];
  const int Rm = c.max_requests;
  for (int r = 0; r < R; ++r) {
    h[r] = tenant_ids[r];
    h[Rm + r] = seq_lens[r];
    h[2 * Rm + r] = p->slot_of_tenant[tenant_ids[r]];
    if (kv != KV_NONE) {
      h[3 * Rm + r] = seq_slots[r];
      h[4 * Rm + r] = kv == KV_PREFILL ? 0 : p->kv_len[seq_slots[r]];
    }
  }
  hipStream_t s = p->compute;
  // The router reads the three index arrays straight from this pinned (device-mapped) host
  // buffer: 3 R words over the host link, instead of a staging copy that costs a copy
  // engine hand-over (about 15 us) on either side.  The event lets the buffer be reused.
  Route rt = p->rt;
  rt.tenant_ids = h; rt.seq_lens = h + Rm; rt.req_slot = h + 2 * Rm;
  if (kv != KV_NONE) { rt.kv_slot_in = h + 3 * Rm; rt.kv_pos_in = h + 4 * Rm; }
  { ProfSpan ps(p, HMI_KERNEL_ROUTER); launch_router(rt, R, s); }
  HIP_TRY(p, hipEventRecord(p->idx_ev[bi], s));
  p->last_R = R;
  p->last_distinct.assign(p->distinct.begin(), p->distinct.end());   // within the reserved capacity
  p->last_n_mtiles[0] = n_mtiles[0]; p->last_n_mtiles[1] = n_mtiles[1];
  p->last_N = (int)N;

  const int d = c.d_model, f = c.d_ff;
  const bool f32 = !p->bf16;  // fp32 pools: "storage" and fp32 coincide

  // Between the layers of one call the activations stay in fp32 (w_y32, residual operand)
  // next to a storage-dtype copy (w_yst, GEMM operand); only the last layer rounds into y.
  const void* in_st = x;        // layer input, storage dtype
  const void* in_res = x;       // layer input as residual / LayerNorm operand
  bool in_res_f32 = f32;

  // where the last layer's LayerNorm puts the result: y in the storage type, or y as fp32 on request
  float* const y_out32 = y_f32 ? static_cast<float*>(y) : nullptr;
  void* const y_outst = y_f32 ? nullptr : y;
  for (int layer = layer_begin; layer < layer_end; ++layer) {
    const bool last = layer + 1 == layer_end;
    // weights of this layer must have landed before the first kernel that reads them
    if (need_copy > p->compute_waited_copy) {
      HIP_TRY(p, hipStreamWaitEvent(s, p->copy_done.at_least(need_copy), 0));
      p->compute_waited_copy = need_copy;
    }
    // fine-grained pipelining (Sec. 6.2): start the next layer's swap-in before this
    // layer's kernels are enqueued, so that the copies run under them
    uint64_t need_next = 0;
    if (!last) {
      int32_t rc = make_resident(layer + 1, true, &need_next);
      if (rc != HMI_OK) {
        // earlier layers of this call may already be enqueued and reading their slots:
        // later evictions have to wait for them like for a completed call
        if (layer > layer_begin) mark_slots_read();
        return rc;
      }
    }

    const size_t lay = (size_t)layer * p->image_bytes;
    auto gemm = [&](const void* A, int lda, int tw, int tb, int n_out, int k, int epi, void* C, int ldc,
                    const void* resid, int ldr, bool resid_f32, bool out_f32, void* C2) {
      GemmArgs g{};
      g.A = A; g.lda = lda; g.C = C; g.ldc = ldc; g.resid = resid; g.ldr = ldr;
      g.resid_f32 = resid_f32; g.out_f32 = out_f32; g.C2 = C2;
      g.pool = p->d_pool; g.slot_stride = p->slot_stride;
      g.w_off = lay + p->tl[tw].off; g.b_off = lay + p->tl[tb].off;
      g.n_out = n_out; g.k = k; g.n_rows = (int)N; g.epi = epi;
      g.n_mtiles_list[0] = n_mtiles[0]; g.n_mtiles_list[1] = n_mtiles[1];
      g.which_tiles = 0; g.n_mtiles = n_mtiles[0];
          ProfSpan ps(p, HMI_KERNEL_GEMM);
      if (p->bf16) launch_gemm_bf16(g, rt, s); else launch_gemm_f32(g, rt, s);
    };
    auto lnorm = [&](const void* in, bool in_f32, float* out_f32, void* out_st, int tg, int tb) {
      LnArgs a{};
      a.in = in; a.in_f32 = in_f32; a.out_f32 = out_f32; a.out_st = out_st;
      a.pool = p->d_pool; a.slot_stride = p->slot_stride;
      a.g_off = lay + p->tl[tg].off; a.b_off = lay + p->tl[tb].off;
      a.d = d; a.eps = c.ln_eps; a.n_rows = (int)N; a.bf16 = p->bf16;
      ProfSpan ps(p, HMI_KERNEL_LAYERNORM);
      launch_layernorm(a, rt, s);
    };
    // the same two with the parameters all tenants share: slot stride 0, dense route
    const size_t slay = (size_t)layer * p->shared_image_bytes;
    auto sgemm = [&](const void* A, int lda, int tw, int tb, int n_out, int k, int epi, void* C, int ldc,
                     const void* resid, int ldr, bool resid_f32, bool out_f32) {
      GemmArgs g{};
      g.A = A; g.lda = lda; g.C = C; g.ldc = ldc; g.resid = resid; g.ldr = ldr;
      g.resid_f32 = resid_f32; g.out_f32 = out_f32; g.C2 = nullptr;
      g.pool = p->d_shared; g.slot_stride = 0;
      g.w_off = slay + p->stl[tw].off; g.b_off = slay + p->stl[tb].off;
      g.n_out = n_out; g.k = k; g.n_rows = (int)N; g.epi = epi;
      g.n_mtiles_list[0] = (int)((N + p->tile_m[0] - 1) / p->tile_m[0]);
      g.n_mtiles_list[1] = p->tile_m[1] ? (int)((N + p->tile_m[1] - 1) / p->tile_m[1]) : 0;
      g.which_tiles = 0; g.n_mtiles = g.n_mtiles_list[0];
          ProfSpan ps(p, HMI_KERNEL_GEMM);
      if (p->bf16) launch_gemm_bf16(g, p->rt_dense, s); else launch_gemm_f32(g, p->rt_dense, s);
    };
    auto slnorm = [&](const void* in, bool in_f32, const void* in2, float* out_f32, void* out_st, int tg, int tb,
                      float* sum_out = nullptr) {
      LnArgs a{};
      a.in = in; a.in_f32 = in_f32; a.in2 = in2; a.out_f32 = out_f32; a.out_st = out_st; a.sum_out = sum_out;
      a.pool = p->d_shared; a.slot_stride = 0;
      a.g_off = slay + p->stl[tg].off; a.b_off = slay + p->stl[tb].off;
      a.d = d; a.eps = c.ln_eps; a.n_rows = (int)N; a.bf16 = p->bf16;
      ProfSpan ps(p, HMI_KERNEL_LAYERNORM);
      launch_layernorm(a, p->rt_dense, s);
    };
    auto attention = [&](bool causal) {
      if (kv != KV_NONE) {   // decoder blocks only (hmi_kv_create refuses the others)
        KvArgs k{};
        k.qkv = p->w_qkv; k.ctx = p->w_ctx; k.d = d; k.n_heads = c.n_heads; k.max_len = p->kv_max_len;
        k.cache = p->d_kv + (size_t)layer * p->kv_seqs * 2 * (size_t)d * p->kv_max_len;
        ProfSpan ps(p, HMI_KERNEL_ATTENTION);
        if (kv == KV_PREFILL) launch_kv_store(k, rt, R, s);
        else { launch_attn_decode(k, rt, R, s); return; }
      }
      AttnArgs a{};
      a.qkv = p->w_qkv; a.ctx = p->w_ctx; a.d = d; a.n_heads = c.n_heads; a.causal = causal;
      a.R = R; a.max_len = max_len; a.bf16 = p->bf16; a.n_rows = (int)N;
      ProfSpan ps(p, HMI_KERNEL_ATTENTION);
      launch_attention(a, rt, s);
    };

    // the tenant's adapter on the attention output: w_act -> w_ctx, tenant route (composite blocks)
    auto adapter_step = [&]() {
      const int r = p->rank;
      if (p->adapter_fused) {
        AdapterArgs a{};
        a.X = p->w_act; a.Y = p->w_ctx; a.pool = p->d_pool; a.slot_stride = p->slot_stride;
        a.wd_off = lay + p->tl[T_W1].off; a.bd_off = lay + p->tl[T_B1].off;
        a.wu_off = lay + p->tl[T_W2].off; a.bu_off = lay + p->tl[T_B2].off;
        a.d = d; a.which_tiles = 1; a.n_tiles128 = n_mtiles[1];
        a.weights_once = (long long)N <= 32LL * n_mtiles[1];
        ProfSpan ps(p, HMI_KERNEL_GEMM);
        launch_adapter_bf16(a, rt, s);
      } else {
        gemm(p->w_act, d, T_W1, T_B1, r, d, EPI_BIAS_RELU, p->w_hmid, r, nullptr, 0, false, false, nullptr);
        gemm(p->w_hmid, r, T_W2, T_B2, d, r, EPI_BIAS_RESID, p->w_ctx, d, p->w_act, d, f32, f32, nullptr);
      }
    };

    switch (c.block) {
      case HMI_BLOCK_FFN:
        gemm(in_st, d, T_W1, T_B1, f, d, EPI_BIAS_GELU, p->w_hmid, f, nullptr, 0, false, false, nullptr);
        gemm(p->w_hmid, f, T_W2, T_B2, d, f, EPI_BIAS_RESID, p->w_z, d, in_res, d, in_res_f32, true, nullptr);
        lnorm(p->w_z, true, last ? y_out32 : p->w_y32, last ? y_outst : (void*)p->w_yst, T_LNG, T_LNB);
        break;
      case HMI_BLOCK_ADAPTER:
        if (p->adapter_fused) {
          AdapterArgs a{};
          a.X = x; a.Y = y; a.pool = p->d_pool; a.slot_stride = p->slot_stride;
          a.wd_off = lay + p->tl[T_W1].off; a.bd_off = lay + p->tl[T_B1].off;
          a.wu_off = lay + p->tl[T_W2].off; a.bu_off = lay + p->tl[T_B2].off;
          a.d = d; a.which_tiles = 1; a.n_tiles128 = n_mtiles[1];
          a.stream_out = 1;
          ProfSpan ps(p, HMI_KERNEL_GEMM);
          launch_adapter_bf16(a, rt, s);
          break;
        }
        gemm(in_st, d, T_W1, T_B1, f, d, EPI_BIAS_RELU, p->w_hmid, f, nullptr, 0, false, false, nullptr);
        if (last)
          gemm(p->w_hmid, f, T_W2, T_B2, d, f, EPI_BIAS_RESID, y, d, in_res, d, in_res_f32, f32 || y_f32, nullptr);
        else
          gemm(p->w_hmid, f, T_W2, T_B2, d, f, EPI_BIAS_RESID, p->w_y32, d, in_res, d, in_res_f32, true, p->w_yst);
        break;
      case HMI_BLOCK_ENC_POSTLN:
        gemm(in_st, d, A_WQKV, A_BQKV, 3 * d, d, EPI_BIAS, p->w_qkv, 3 * d, nullptr, 0, false, false, nullptr);
        attention(false);
        gemm(p->w_ctx, d, A_WO, A_BO, d, d, EPI_BIAS_RESID, p->w_z, d, in_res, d, in_res_f32, true, nullptr);
        lnorm(p->w_z, true, p->w_x1, p->bf16 ? p->w_act : nullptr, A_LN1G, A_LN1B);
        gemm(p->bf16 ? (const void*)p->w_act : (const void*)p->w_x1, d, A_W1, A_B1, f, d, EPI_BIAS_GELU,
             p->w_hmid, f, nullptr, 0, false, false, nullptr);
        gemm(p->w_hmid, f, A_W2, A_B2, d, f, EPI_BIAS_RESID, p->w_z, d, p->w_x1, d, true, true, nullptr);
        lnorm(p->w_z, true, last ? y_out32 : p->w_y32, last ? y_outst : (void*)p->w_yst, A_LN2G, A_LN2B);
        break;
      case HMI_BLOCK_DEC_ADAPTER: {
        // the decoder-only counterpart: pre-LN, causal, residual stream carried in fp32
        slnorm(in_res, in_res_f32, nullptr, nullptr, p->w_act, A_LN1G, A_LN1B);
        sgemm(p->w_act, d, A_WQKV, A_BQKV, 3 * d, d, EPI_BIAS, p->w_qkv, 3 * d, nullptr, 0, false, false);
        attention(true);
        sgemm(p->w_ctx, d, A_WO, A_BO, d, d, EPI_BIAS, p->w_act, d, nullptr, 0, false, false);
        adapter_step();                                                     // w_act -> w_ctx
        slnorm(in_res, in_res_f32, p->w_ctx, nullptr, p->w_act, A_LN2G, A_LN2B, p->w_x1);   // x1 = x + a', LN2(x1)
        sgemm(p->w_act, d, A_W1, A_B1, f, d, EPI_BIAS_GELU, p->w_hmid, f, nullptr, 0, false, false);
        if (last) sgemm(p->w_hmid, f, A_W2, A_B2, d, f, EPI_BIAS_RESID, y, d, p->w_x1, d, true, f32 || y_f32);
        else sgemm(p->w_hmid, f, A_W2, A_B2, d, f, EPI_BIAS_RESID, p->w_y32, d, p->w_x1, d, true, true);
        break;
      }
      case HMI_BLOCK_ENC_ADAPTER: {
        // the shared layer with the tenant's adapter after the attention layer (Sec. 3.2.2):
        // only the adapter step reads per-tenant parameters and follows the tenant route
        sgemm(in_st, d, A_WQKV, A_BQKV, 3 * d, d, EPI_BIAS, p->w_qkv, 3 * d, nullptr, 0, false, false);
        attention(false);
        sgemm(p->w_ctx, d, A_WO, A_BO, d, d, EPI_BIAS, p->w_act, d, nullptr, 0, false, false);
        adapter_step();                                                     // w_act -> w_ctx
        slnorm(in_res, in_res_f32, p->w_ctx, p->w_x1, p->bf16 ? p->w_act : nullptr, A_LN1G, A_LN1B);
        sgemm(p->bf16 ? (const void*)p->w_act : (const void*)p->w_x1, d, A_W1, A_B1, f, d, EPI_BIAS_GELU,
              p->w_hmid, f, nullptr, 0, false, false);
        sgemm(p->w_hmid, f, A_W2, A_B2, d, f, EPI_BIAS_RESID, p->w_z, d, p->w_x1, d, true, true);
        slnorm(p->w_z, true, nullptr, last ? y_out32 : p->w_y32, last ? y_outst : (void*)p->w_yst, A_LN2G, A_LN2B);
        break;
      }
      case HMI_BLOCK_DEC_PRELN:
        lnorm(in_res, in_res_f32, nullptr, p->w_act, A_LN1G, A_LN1B);
        gemm(p->w_act, d, A_WQKV, A_BQKV, 3 * d, d, EPI_BIAS, p->w_qkv, 3 * d, nullptr, 0, false, false, nullptr);
        attention(true);
        gemm(p->w_ctx, d, A_WO, A_BO, d, d, EPI_BIAS_RESID, p->w_x1, d, in_res, d, in_res_f32, true, nullptr);
        lnorm(p->w_x1, true, nullptr, p->w_act, A_LN2G, A_LN2B);
        gemm(p->w_act, d, A_W1, A_B1, f, d, EPI_BIAS_GELU, p->w_hmid, f, nullptr, 0, false, false, nullptr);
        if (last)
          gemm(p->w_hmid, f, A_W2, A_B2, d, f, EPI_BIAS_RESID, y, d, p->w_x1, d, true, f32 || y_f32, nullptr);
        else
          gemm(p->w_hmid, f, A_W2, A_B2, d, f, EPI_BIAS_RESID, p->w_y32, d, p->w_x1, d, true, true, nullptr);
        break;
    }
    in_st = p->w_yst;
    in_res = p->w_y32;
    in_res_f32 = true;
    need_copy = need_next;
  }
  mark_slots_read();
  HIP_TRY(p, hipGetLastError());
  if (kv == KV_PREFILL) for (int r = 0; r < R; ++r) p->kv_len[seq_slots[r]] = seq_lens[r];
  if (kv == KV_DECODE) for (int r = 0; r < R; ++r) p->kv_len[seq_slots[r]] += 1;
  return HMI_OK;
}

int32_t hmi_stack_forward(hmi_pool_t* p, int32_t layer_begin, int32_t layer_end, const void* x, void* y,
                          const int32_t* tenant_ids, const int32_t* seq_lens, int32_t R) {
  return forward_impl(p, layer_begin, layer_end, x, y, tenant_ids, seq_lens, R, KV_NONE, nullptr);
}

int32_t hmi_stack_forward_f32(hmi_pool_t* p, int32_t layer_begin, int32_t layer_end, const void* x, float* y,
                              const int32_t* tenant_ids, const int32_t* seq_lens, int32_t R) {
  return forward_impl(p, layer_begin, layer_end, x, y, tenant_ids, seq_lens, R, KV_NONE, nullptr, true);
}

int32_t hmi_kv_create(hmi_pool_t* p, int32_t max_seqs, int32_t max_len) {
  if (!p) return HMI_ERR_ARG;
  const hmi_pool_config_t& c = p->cfg;
  if ((c.block != HMI_BLOCK_DEC_PRELN && c.block != HMI_BLOCK_DEC_ADAPTER) || !p->bf16)
    return fail(p, HMI_ERR_ARG, "the key/value cache needs a bf16 DEC_PRELN or DEC_ADAPTER pool");
  if (p->d_kv) return fail(p, HMI_ERR_ARG, "the pool already has a key/value cache");
  if (max_seqs < 1 || max_len < 1) return fail(p, HMI_ERR_ARG, "max_seqs and max_len must be positive");
  HIP_TRY(p, hipSetDevice(c.device));
  const unsigned __int128 wide = (unsigned __int128)c.n_layers * (unsigned)max_seqs * 2u * (unsigned)c.d_model * (unsigned)max_len * sizeof(uint16_t);
  if (wide >= ((unsigned __int128)1 << 46)) return fail(p, HMI_ERR_OOM, "a key/value cache of that size exceeds any device");
  const size_t bytes = (size_t)wide;
  HIP_TRY(p, hipMalloc(&p->d_kv, bytes));
  p->kv_seqs = max_seqs; p->kv_max_len = max_len;
  p->kv_len.assign(max_seqs, 0);
  p->kv_mark.assign(max_seqs, 0);
  return HMI_OK;
}

int32_t hmi_prefill(hmi_pool_t* p, int32_t layer_begin, int32_t layer_end, const void* x, void* y,
                    const int32_t* tenant_ids, const int32_t* seq_lens, const int32_t* seq_slots, int32_t R) {
  return forward_impl(p, layer_begin, layer_end, x, y, tenant_ids, seq_lens, R, KV_PREFILL, seq_slots);
}

int32_t hmi_decode_step(hmi_pool_t* p, int32_t layer_begin, int32_t layer_end, const void* x, void* y,
                        const int32_t* tenant_ids, const int32_t* seq_slots, int32_t R) {
  return forward_impl(p, layer_begin, layer_end, x, y, tenant_ids, nullptr, R, KV_DECODE, seq_slots);
}

int32_t hmi_layer_forward(hmi_pool_t* p, int32_t layer, const void* x, void* y,
                          const int32_t* tenant_ids, const int32_t* seq_lens, int32_t R) {
  return hmi_stack_forward(p, layer, layer + 1, x, y, tenant_ids, seq_lens, R);
}

int32_t hmi_layer_forward_static(hmi_pool_t* p, int32_t layer, const void* x, void* y,
                                 const int32_t* tenant_ids, const int32_t* seq_lens, int32_t R) {
  if (!p) return HMI_ERR_ARG;
  if (R == 0) return HMI_OK;
  const hmi_pool_config_t& c = p->cfg;
  if (c.block != HMI_BLOCK_ADAPTER || !p->adapter_fused || c.host_tier)
    return fail(p, HMI_ERR_ARG, "hmi_layer_forward_static needs a bf16 ADAPTER pool without host tier that runs as one kernel "
                                "(rank 64, d_model 256 / 512 / 768, one layer)");
  if (R < 0 || !x || !y || !tenant_ids || !seq_lens) return fail(p, HMI_ERR_ARG, "null pointer or negative request count");
  if (x == y) return fail(p, HMI_ERR_ARG, "x and y must be different buffers");
  if (layer != 0) return fail(p, HMI_ERR_ARG, "layer %d outside [0,1)", layer);
  if (R > c.max_requests || R > kStaticMaxRequests)
    return fail(p, HMI_ERR_SHAPE, "%d requests > limit %d", R, std::min(c.max_requests, kStaticMaxRequests));
  if (++p->epoch == 0) { std::fill(p->mark.begin(), p->mark.end(), 0u); p->epoch = 1; }
  p->distinct.clear();
  const int64_t max_tokens = std::min<int64_t>(c.max_tokens, kStaticMaxTokens);
  int64_t N = 0;
  for (int r = 0; r < R; ++r) {
    const int t = tenant_ids[r], len = seq_lens[r];
    if (len <= 0) return fail(p, HMI_ERR_SHAPE, "seq_lens[%d] = %d", r, len);
    if (t < 0 || t >= c.max_tenants) return fail(p, HMI_ERR_TENANT, "tenant_ids[%d] = %d outside [0,%d)", r, t, c.max_tenants);
    if (!p->loaded[t] || p->slot_of_tenant[t] < 0) return fail(p, HMI_ERR_TENANT, "tenant %d was never loaded", t);
    if (p->mark[t] != p->epoch) { p->mark[t] = p->epoch; p->tok_count[t] = 0; p->distinct.push_back(t); }
    p->tok_count[t] += len;
    N += len;
    if (N > max_tokens) return fail(p, HMI_ERR_SHAPE, "batch has more than %d tokens", (int)max_tokens);
  }
  HIP_TRY(p, hipSetDevice(c.device));
  int32_t* const base = g_scratch_ptr[c.device];
  if (!base) return fail(p, HMI_ERR_DEVICE, "the static routing arrays of device %d were never resolved", c.device);
  int n_tiles128 = 0;
  uint64_t need_copy = 0;
  for (int t : p->distinct) {
    n_tiles128 += (p->tok_count[t] + kBf16TileM1 - 1) / kBf16TileM1;
    need_copy = std::max(need_copy, p->slot_copy[p->slot_of_tenant[t]]);
  }
  hipStream_t s = p->compute;
  if (need_copy > p->compute_waited_copy) {   // weights loaded just before this call
    HIP_TRY(p, hipStreamWaitEvent(s, p->copy_done.at_least(need_copy), 0));
    p->compute_waited_copy = need_copy;
  }
  // index arrays: through one of the pool's pinned buffers, read in place by the router
  const int bi = p->idx_i;
  p->idx_i = (p->idx_i + 1) & 3;
  HIP_TRY(p, hipEventSynchronize(p->idx_ev[bi]));
  int32_t* h = p->h_idx[bi];
  const int Rm = c.max_requests;
  for (int r = 0; r < R; ++r) {
    h[r] = tenant_ids[r];
    h[Rm + r] = seq_lens[r];
    h[2 * Rm + r] = p->slot_of_tenant[tenant_ids[r]];
  }
  // routing arrays: fixed places inside this device's copy of `scratch`; the router writes every
  // entry the adapter kernel reads, so nothing has to be cleared between calls
  int32_t* q = base;
  auto take = [&](size_t n) { int32_t* r = q; q += n; return r; };
  constexpr size_t SR = kStaticMaxRequests;
  Route rt{};
  rt.tenant_ids = h; rt.seq_lens = h + Rm; rt.req_slot = h + 2 * Rm;
  rt.req_tenant = take(SR); rt.kv_slot = take(SR); rt.kv_pos = take(SR);
  rt.perm = take(SR); rt.tok_off = take(SR + 1);
  rt.seg_tenant = take(SR); rt.seg_slot = take(SR);
  rt.seg_req_off = take(SR + 1); rt.seg_tok_off = take(SR + 1);
  rt.n_segments = take(1); rt.n_tiles[0] = take(1); rt.n_tiles[1] = take(1);
  if ((size_t)(q - base) != kStaticIndexInts) return fail(p, HMI_ERR_DEVICE, "layout of the static routing arrays is inconsistent");
  rt.row_src = take(kStaticMaxTokens);
  rt.tile_seg[0] = take(kStaticTiles0); rt.tile_row0[0] = take(kStaticTiles0);
  rt.tile_seg[1] = take(kStaticTiles1); rt.tile_row0[1] = take(kStaticTiles1);
  if ((size_t)(q - base) != kStaticScratchInts) return fail(p, HMI_ERR_DEVICE, "layout of the static routing arrays is inconsistent");
  rt.tile_m[0] = kBf16TileM0; rt.tile_m[1] = kBf16TileM1;
  rt.key_bits = p->rt.key_bits;
  rt.n_cu = p->rt.n_cu;
  launch_router(rt, R, s);
  HIP_TRY(p, hipEventRecord(p->idx_ev[bi], s));
  AdapterArgs a{};
  a.X = x; a.Y = y; a.pool = p->d_pool; a.slot_stride = p->slot_stride;
  a.wd_off = p->tl[T_W1].off; a.bd_off = p->tl[T_B1].off;
  a.wu_off = p->tl[T_W2].off; a.bu_off = p->tl[T_B2].off;
  a.d = c.d_model; a.which_tiles = 1; a.n_tiles128 = n_tiles128;
  a.stream_out = 1;
  launch_adapter_bf16(a, rt, s);
  const uint64_t seq = p->fwd_done.record(s);
  for (int t : p->distinct) p->slot_fwd[p->slot_of_tenant[t]] = seq;
  HIP_TRY(p, hipGetLastError());
  return HMI_OK;
}

int32_t hmi_get_route(hmi_pool_t* p, int32_t* perm, int32_t* seg_tenant, int32_t* seg_req_off,
                      int32_t* seg_tok_off, int32_t* n_segments) {
  if (!p) return HMI_ERR_ARG;
  HIP_TRY(p, hipSetDevice(p->cfg.device));
  HIP_TRY(p, hipStreamSynchronize(p->compute));
  const int R = p->last_R;
  int32_t G = 0;
  if (R > 0) HIP_TRY(p, hipMemcpy(&G, p->rt.n_segments, sizeof(int32_t), hipMemcpyDeviceToHost));
  if (n_segments) *n_segments = G;
  if (R == 0) return HMI_OK;
  if (perm) HIP_TRY(p, hipMemcpy(perm, p->rt.perm, sizeof(int32_t) * R, hipMemcpyDeviceToHost));
  if (seg_tenant) HIP_TRY(p, hipMemcpy(seg_tenant, p->rt.seg_tenant, sizeof(int32_t) * G, hipMemcpyDeviceToHost));
  if (seg_req_off) HIP_TRY(p, hipMemcpy(seg_req_off, p->rt.seg_req_off, sizeof(int32_t) * (G + 1), hipMemcpyDeviceToHost));
  if (seg_tok_off) HIP_TRY(p, hipMemcpy(seg_tok_off, p->rt.seg_tok_off, sizeof(int32_t) * (G + 1), hipMemcpyDeviceToHost));
  return HMI_OK;
}

int32_t hmi_pool_stats(hmi_pool_t* p, int64_t* hits, int64_t* misses, int64_t* bytes_h2d, int64_t* evictions) {
  if (!p) return HMI_ERR_ARG;
  if (hits) *hits = p->hits;
  if (misses) *misses = p->misses;
  if (bytes_h2d) *bytes_h2d = p->bytes_h2d;
  if (evictions) *evictions = p->evictions;
  return HMI_OK;
}

int32_t hmi_pool_profile(hmi_pool_t* p, int32_t enable) {
  if (!p) return HMI_ERR_ARG;
  p->profiling = enable != 0;
  return HMI_OK;
}

int32_t hmi_pool_profile_read(hmi_pool_t* p, double* ms, int64_t* launches) {
  if (!p) return HMI_ERR_ARG;
  HIP_TRY(p, hipSetDevice(p->cfg.device));
  HIP_TRY(p, hipStreamSynchronize(p->compute));
  for (int k = 0; k < HMI_KERNEL_KINDS; ++k) {
    if (ms) ms[k] = 0.0;
    if (launches) launches[k] = 0;
  }
  for (auto& sp : p->spans) {
    float t = 0.0f;
    if (hipEventElapsedTime(&t, sp.a, sp.b) == hipSuccess) {
      if (ms) ms[sp.kind] += (double)t;
      if (launches) launches[sp.kind] += 1;
    }
    (void)hipEventDestroy(sp.a);
    (void)hipEventDestroy(sp.b);
  }
  p->spans.clear();
  return HMI_OK;
}

}  // extern "C"

const hmi_pool_config_t* hmi_internal_config(const hmi_pool_t* p) { return &p->cfg; }
hipStream_t hmi_internal_compute_stream(const hmi_pool_t* p) { return p->compute; }
bool hmi_internal_tenant_ready(const hmi_pool_t* p, int32_t tenant) {
  if (tenant < 0 || tenant >= p->cfg.max_tenants) return false;
  for (int l = 0; l < p->cfg.n_layers; ++l)
    if (!p->loaded[(size_t)tenant * p->cfg.n_layers + l]) return false;
  return true;
}

extern "C" {

int64_t hmi_pool_image_bytes(const hmi_pool_t* p) { return p ? (int64_t)p->image_bytes : 0; }

const char* hmi_last_error(const hmi_pool_t* p) { return p ? p->err : g_create_error; }

int32_t hmi_pool_destroy(hmi_pool_t* p) {
  if (!p) return HMI_OK;
  (void)hipSetDevice(p->cfg.device);
  free_all(p);
  return HMI_OK;
}

}  // extern "C"
