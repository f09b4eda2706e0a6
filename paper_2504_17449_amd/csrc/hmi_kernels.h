// Internal launch interface between the pool/orchestration code and the gfx950 kernels.
// Everything here is device-pointer plumbing; the C ABI lives in include/hmi.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hmi {

constexpr int kRouterThreads = 1024;
constexpr int kMaxRequests = 2048;   // router keeps keys/values of one batch in LDS
constexpr int kDenseSegRows = 1024;  // rows per pseudo-segment of the route for shared parameters

// Output of the tenant-segmented router, all DEVICE int32 arrays.
struct Route {
  const int32_t* tenant_ids;  // [R] in: request -> tenant
  const int32_t* seq_lens;    // [R] in
  const int32_t* req_slot;    // [R] in: request -> HBM slot of its tenant (resolved on host)
  int32_t* req_tenant;        // [R]   request -> tenant (device copy of tenant_ids)
  int32_t* perm;              // [R]   sorted position -> request
  int32_t* tok_off;           // [R+1] request -> first row (original packed order)
  int32_t* seg_tenant;        // [G]
  int32_t* seg_slot;          // [G]
  int32_t* seg_req_off;       // [G+1] segment -> first sorted position
  int32_t* seg_tok_off;       // [G+1] segment -> first sorted row
  int32_t* row_src;           // [N]   sorted row -> original row
  int32_t* n_segments;        // [1]
  // m-tile work lists for two tile heights (rows of one tile never cross a segment)
  int32_t* tile_seg[2];       // [tiles] tile -> segment
  int32_t* tile_row0[2];      // [tiles] tile -> first sorted row
  int32_t* n_tiles[2];        // [1]
  int32_t tile_m[2];          // tile heights (0 = list unused)
  int32_t key_bits;           // bits needed for the largest tenant id (radix passes = bits/4)
  // scratch of the persistent GEMM: per XCD a tile-claim counter [0..7] and a count of finished
  // workgroups [8..15], then one mailbox per workgroup; all zero between launches
  int32_t* gemm_sched;
  // Decoding with a key/value cache: per request the cache line (sequence slot) and the position
  // its first row takes in it; copied from the *_in arrays (may be host memory) when those are set.
  const int32_t* kv_slot_in; const int32_t* kv_pos_in;
  int32_t* kv_slot;           // [R]
  int32_t* kv_pos;            // [R]
  // Written by the router when not null: the segment offsets of a second route over the same
  // N rows for parameters that all tenants share.  That route takes the rows in their
  // original order and cuts them into pseudo-segments of kDenseSegRows rows (the last one
  // shorter), which all name slot 0; its tile lists and row map do not depend on the batch.
  int32_t* dense_seg_tok_off;   // [ceil(N / kDenseSegRows) + 1]
  int32_t* dense_n_segments;    // [1]
  // 1 for the route of the shared parameters itself: row_src is the identity, every segment names
  // slot 0 and tile t of list k starts at row t * tile_m[k], so a kernel that is given the batch's
  // row count needs none of the arrays above (each lookup it skips is a dependent trip to L2, which
  // is most of the duration of a launch over a few hundred rows).
  int32_t identity;
  int32_t n_cu;                 // compute units of the pool's device (host side: sizes the persistent launches)
};
constexpr int kGemmSchedInts = 16 + 1024;
void launch_router(const Route& rt, int R, hipStream_t s);

// Per-device set-up of the kernels that need more than the default dynamic LDS: pool creation
// calls these once per device, with that device current, before any launch on it.
void init_gemm_bf16_kernels();
void init_gemm_bf16_p256_kernels();
void init_gemm_bf16_skinny_kernels();
void init_adapter_bf16_kernels();

enum Epilogue : int {
  EPI_BIAS = 0,        // C = acc + b                      -> storage dtype
  EPI_BIAS_GELU = 1,   // C = GELU(acc + b)                -> storage dtype
  EPI_BIAS_RELU = 2,   // C = max(acc + b, 0)              -> storage dtype
  EPI_BIAS_RESID = 3   // C = acc + b + resid              -> out_f32 ? fp32 : storage dtype
};

// Grouped GEMM: for every m-tile (segment g, rows), C[rows, :] = epi(A[rows, :] * W_g^T + b_g)
// with W_g = slot image of seg_slot[g] (+w_off), [n_out, k] row-major.  Rows are addressed
// through row_src (original packed order) in A, C and resid alike.
struct GemmArgs {
  const void* A;  int lda;            // storage dtype, [N, k]
  void* C;        int ldc;            // [N, n_out]
  void* C2;                           // optional second copy of C in the storage dtype (same ldc)
  const void* resid; int ldr;         // EPI_BIAS_RESID only
  int resid_f32;                      // residual operand is fp32 (else storage dtype)
  int out_f32;                        // write fp32 (else storage dtype)
  const char* pool; size_t slot_stride;  // HBM pool base and bytes per slot
  size_t w_off, b_off;                // byte offsets of W and bias inside a slot (layer included)
  int n_out, k;
  int n_rows;                         // rows of the whole batch (chooses between the kernels)
  int epi;
  int n_mtiles_list[2];               // exact m-tile counts of both tile lists, computed on the host
  int which_tiles;                    // set by the launcher: index into Route::tile_* ...
  int n_mtiles;                       // ... and that list's count
};

void launch_gemm_bf16(const GemmArgs& g, const Route& rt, hipStream_t s);
void launch_gemm_f32(const GemmArgs& g, const Route& rt, hipStream_t s);
// Persistent 256 x 256 tiles, 64-wide k-stages; needs n_out % 256 == 0, k % 64 == 0, k >= 192 and
// which_tiles / n_mtiles naming the list of 256-row m-tiles.
void launch_gemm_bf16_p256(const GemmArgs& g, const Route& rt, hipStream_t s);
// One wavefront per (32 rows, 32 columns) item for launches with few rows per weight matrix; needs
// k % 64 == 0, n_out % 32 == 0 and which_tiles / n_mtiles naming the list of 128-row m-tiles.
void launch_gemm_bf16_skinny(const GemmArgs& g, const Route& rt, hipStream_t s);
constexpr int kBf16TileM0 = 256, kBf16TileM1 = 128;  // heights of the two m-tile lists of bf16 pools
constexpr int kF32TileM = 64;

// Fused bottleneck adapter (bf16, rank 64): Y = X + Up_t(ReLU(Down_t(X))), rows addressed
// through row_src like the GEMMs.  Both matrices must be stored in MFMA operand order
// (pack_adapter_operand) inside the slot images.
struct AdapterArgs {
  const void* X; void* Y;             // bf16 [N, d], distinct
  const char* pool; size_t slot_stride;
  size_t wd_off, bd_off, wu_off, bu_off;  // byte offsets inside a slot (layer included)
  int d;
  int which_tiles, n_tiles128;        // index and length of the list of 128-row m-tiles
  int stream_out;                     // 1: Y is not read again soon (the caller's result): stored with the non-temporal hint
  int weights_once;                   // 1: a tenant's matrices are read by about one unit of rows (a decode step): loaded with the non-temporal hint
};
bool adapter_bf16_supported(int d, int rank);
void launch_adapter_bf16(const AdapterArgs& a, const Route& rt, hipStream_t s);
// HOST: [rows, cols] row-major bf16 -> operand order (rows % 32 == 0, cols % 16 == 0, same size).
void pack_adapter_operand(void* dst, const void* src, int rows, int cols);

// Row LayerNorm with per-tenant gain/shift looked up through the route.
// in: fp32 (in_f32) or storage dtype; writes out_f32 (fp32, may be null) and/or
// out_st (storage dtype, may be null).  All [N, d] in original packed order.
struct LnArgs {
  const void* in; int in_f32;
  const void* in2;                    // optional second addend in the storage dtype: LN(in + in2)
  float* sum_out;                     // optional: in + in2 itself, fp32 (the residual stream a pre-LN layer carries on)
  float* out_f32; void* out_st;
  const char* pool; size_t slot_stride; size_t g_off, b_off;
  int d; float eps; int n_rows; int bf16;
};
void launch_layernorm(const LnArgs& a, const Route& rt, hipStream_t s);

// Per-tenant output heads.  A head image holds kHeadCols class rows of d weights (rows at or
// beyond the tenant's class count are zero) and then kHeadCols biases, in the storage dtype, so
// that raw[row, c] = b_t[c] + W_t[c] . h[row] is a grouped GEMM with n_out = kHeadCols and fp32
// output.  launch_head_select masks raw by the tenant's {n_classes, per_token} (meta), writes the
// scores [N, max_classes] (optional) and labels[row] = first arg-max (-1: no prediction).
constexpr int kHeadCols = 64;
struct HeadArgs {
  const float* raw; float* scores; int32_t* labels;
  const int32_t* meta;
  int max_classes;
};
void launch_head_select(const HeadArgs& a, const Route& rt, int R, hipStream_t s);

// Per-request multi-head attention on packed qkv [N, 3d] (q | k | v) -> ctx [N, d].
struct AttnArgs {
  const void* qkv; void* ctx; int d; int n_heads; int causal; int R; int max_len; int bf16;
  int n_rows;  // N = total rows (fp32 kernel: one wavefront per row and head)
};
void launch_attention(const AttnArgs& a, const Route& rt, hipStream_t s);

// Aggregate of precomputed tri-gram representations: table [n_entries, 3, d] and x [N, d] in the
// storage dtype, frag_ids [N] device, tok_off [R + 1] (may be pinned host memory).
struct PlotArgs {
  const char* table; int n_entries;
  const int32_t* frag_ids; const int32_t* tok_off;
  char* x; int d;
};
void launch_plot_aggregate(const PlotArgs& a, int R, bool bf16, hipStream_t s);

// Key/value cache of one layer: [slot][k | v][head][position][64] bf16.
struct KvArgs {
  const void* qkv;     // bf16 [N, 3d] of the batch (q | k | v)
  void* ctx;           // decode: bf16 [N, d] attention output (N = R, one row per request)
  uint16_t* cache;     // the layer's lines
  int d, n_heads, max_len;
};
void launch_kv_store(const KvArgs& a, const Route& rt, int R, hipStream_t s);
void launch_attn_decode(const KvArgs& a, const Route& rt, int R, hipStream_t s);

}  // namespace hmi
