// Grouped bf16 GEMM for batches with few rows per weight matrix: decode steps (one new token per
// request, so a tenant's segment is a handful of rows) and any launch whose 256 x 256 tiles would
// leave most of the chip idle.  Such a launch is bound by streaming the weights once, so the work
// is cut into many small independent items that keep every compute unit's memory pipe full:
//
//   item = (32 rows of one segment) x (32 output columns) x (all of k), one WAVEFRONT per item,
//   five items per workgroup (three in small launches, see Ring), no workgroup barriers.
//
// A launch with so few items that they would not even give every compute unit one workgroup (a decode
// step through parameters that all tenants share: a few hundred rows in all) is bound by the latency of
// one wavefront's walk over k instead; there an item goes to a workgroup of four wavefronts that take
// a quarter of k each and add their partial sums through LDS in a fixed order.
//
// A wavefront streams its 32 weight rows and its 32 activation rows (gathered through row_src) through a
// private LDS ring of four to six stages of 64 k (direct-to-LDS copies of full 128-byte lines, all but one stage in
// flight), reads the weights back as MFMA first operands in the permuted row order that gives a lane 16
// consecutive output columns of one row, and the activations as second operands.  Items of the four row
// blocks of one 128-row tile are neighbours, so a weight panel that several row blocks need is fetched
// from HBM once.
//
// Same contract as the other grouped GEMMs (GemmArgs / Route), epilogues included.
#include "hmi_kernels.h"

#include <math.h>

namespace hmi {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

constexpr int SK = 32;                    // rows and columns of an item
constexpr int STAGE_BYTES = SK * 128;                      // per operand: 32 rows of 64 k
constexpr int KSPLIT = 4;                                  // wavefronts that share the k of one item in the split variant
// Ring depth and wavefronts per workgroup (always 160 KB of LDS, or all the split variant can use):
//   4 stages x 5 wavefronts: launches with many items (per-tenant decode steps), bound by streaming the weights;
//   6 stages x 3 wavefronts (the split variant keeps 4 stages: 5 were 3 % slower): launches with at most kDeepMaxItems items (shared layers,
//   a few hundred rows): there a launch lasts as long as one wavefront's walk over k, a chain of
//   k / 64 / (stages in flight) round trips to L2 or beyond, so more stages in flight shorten it (a decode step
//   through six shared layers: 0.699 -> 0.670 ms; 8 or 9 stages x 2 wavefronts: 0.72-0.74, 5 x 4: 0.679).
constexpr int kAuxNonTemporal = 2;   // cache-policy operand of the direct-to-LDS copy: the nt bit

template <bool SPLIT, bool DEEP>
struct Ring {
  static constexpr int STAGES = (DEEP && !SPLIT) ? 6 : 4;
  static constexpr int WAVES = SPLIT ? KSPLIT : (DEEP ? 3 : 5);
  static constexpr int X_RING = STAGES * STAGE_BYTES;      // a wavefront's ring: weight stages, then activation stages
  static constexpr int WAVE_LDS = 2 * STAGES * STAGE_BYTES;
  static constexpr int LDS_BYTES = WAVES * WAVE_LDS;
  static constexpr int INFL = STAGES - 1;                  // stages in flight
  static_assert(LDS_BYTES <= 163840 && 8 * (INFL - 1) < 64, "ring");
};
constexpr int kDeepMaxItems = 1024;
constexpr int kSplitMaxItems = 384;                        // measured: 192 items 25 -> 9 us per launch, 576 and 768 items slower with it

#define HMI_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

__device__ __forceinline__ float bf2f(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 p = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, p);
}
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

// Chunk swizzles of a 128-byte row in LDS (activation rows are read by consecutive lanes, weight rows
// in the order perm_w: either way the 16 lanes the LDS serves together hit 16 different chunks), and the
// row order of the MFMA's first operand (position i <- weight row perm_w(i)), which makes output
// register r of lane half h column 16 h + r of the item.
__device__ __forceinline__ int swz_a(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int swz_w(int row) { return ((row >> 1) & 3) | (((row >> 4) & 1) << 2); }
__device__ __forceinline__ int perm_w(int i) { return ((i >> 2) & 1) * 16 + (i >> 3) * 4 + (i & 3); }

// row_split: an item is one 32-row block of a 128-row tile (launches with full tiles but few of them);
// otherwise an item is a whole tile and its wavefront takes the tile's row blocks one after the other
// (decode steps: nearly every tile holds a single, short row block).
//
// SPLIT: the workgroup is KSPLIT wavefronts that share one item (row_split items only); wavefront w
// multiplies the w-th quarter of k.  Everything that decides whether a wavefront leaves early is the same
// for the whole workgroup, so all of them reach the barrier in front of the sum.
// WNT: the weights are per-tenant matrices that this launch reads once and the next one does not find in any cache
// (a decode step streams every present tenant's layer: gigabytes): their copies carry the non-temporal hint, which
// moves them 5 % faster (config 4's decode step 0.806 -> 0.764 ms).  Shared weights are read by every row block and again
// in the next step; with the hint that launch is 12 % slower, so the route for shared parameters keeps plain copies.
template <bool SPLIT, bool DEEP, bool WNT>
__global__ __launch_bounds__((64 * Ring<SPLIT, DEEP>::WAVES)) void gemm_bf16_skinny_kernel(GemmArgs g, Route rt, int n_items, int row_split) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  using R = Ring<SPLIT, DEEP>;
  constexpr int STAGES = R::STAGES, WAVES = R::WAVES, X_RING = R::X_RING, WAVE_LDS = R::WAVE_LDS, INFL = R::INFL;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int item = SPLIT ? (int)blockIdx.x : (int)blockIdx.x * WAVES + wave;
  if (item >= n_items) return;
  // item = (tile * NB + column block) [* 4 + row block of the 128-row tile]
  const int NB = g.n_out / SK;
  const int q = row_split ? item >> 2 : item;
  const int nb = q % NB, t = q / NB;
  const int sub_begin = row_split ? (item & 3) : 0, sub_end = row_split ? sub_begin + 1 : 4;
  // the route of the shared parameters needs no lookups: tiles in row order, identity row map, slot 0
  const bool ident = rt.identity != 0;
  int seg_end, tile_row0;
  size_t slot_base = 0;
  if (ident) {
    tile_row0 = t * rt.tile_m[g.which_tiles];
    seg_end = min(g.n_rows, (tile_row0 / kDenseSegRows + 1) * kDenseSegRows);
  } else {
    const int seg = rt.tile_seg[g.which_tiles][t];
    seg_end = rt.seg_tok_off[seg + 1];
    tile_row0 = rt.tile_row0[g.which_tiles][t];
    slot_base = (size_t)rt.seg_slot[seg] * g.slot_stride;
  }
  for (int sub = sub_begin; sub < sub_end; ++sub) {
  const int row0 = tile_row0 + SK * sub;
  const int rows = min(SK, seg_end - row0);
  if (rows <= 0) return;
  const int n0 = nb * SK;
  const int kb = g.k * 2;                               // bytes of a weight row
  const char* Wp = g.pool + slot_base + g.w_off + (size_t)n0 * kb;
  const char* Ap = reinterpret_cast<const char*>(g.A);
  const int l32 = lane & 31, lh = lane >> 5;
  // this wavefront's stages of k: all of them, or its quarter
  const int KT = SPLIT ? g.k / 64 / KSPLIT : g.k / 64;
  const int k_first = SPLIT ? wave * KT : 0;

  // copies: instruction i moves rows 8 i .. 8 i + 7 of a stage; lane l fills position (row 8 i + l / 8,
  // chunk l % 8) with the row's chunk (l % 8) ^ swizzle(row).  Rows past the end of a short row block
  // repeat its last row.
  uint32_t w_off[4], x_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = 8 * i + (lane >> 3);
    w_off[i] = (uint32_t)row * (uint32_t)kb + (((lane & 7) ^ swz_w(row)) << 4);
    const int xr = row0 + min(row, rows - 1);
    x_off[i] = (uint32_t)(ident ? xr : rt.row_src[xr]) * (uint32_t)(g.lda * 2) + (((lane & 7) ^ swz_a(row)) << 4);
  }
  unsigned char* ring = smem + wave * WAVE_LDS;
  const int my_row = ident ? row0 + min(l32, rows - 1) : rt.row_src[row0 + min(l32, rows - 1)];
  const int rw = perm_w(l32);
  const int fw_base = rw * 128 + ((lh ^ swz_w(rw)) << 4);
  const int fx_base = X_RING + l32 * 128 + ((lh ^ swz_a(l32)) << 4);

  // stage S of both operands into ring slot S mod STAGES (8 copies); past the end: an in-bounds re-read nobody consumes
#define HMI_COPY_STAGE(S)                                                                          \
  {                                                                                                \
    const int st_ = k_first + min((S), KT - 1);                                                    \
    const char* ws_ = Wp + st_ * 128;                                                              \
    const char* xs_ = Ap + st_ * 128;                                                              \
    unsigned char* dst_ = ring + ((S) % STAGES) * STAGE_BYTES;                                     \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                  \
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(ws_ + w_off[i]), (lds_ptr_t)(dst_ + i * 1024), 16, 0, WNT ? kAuxNonTemporal : 0); \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                  \
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(xs_ + x_off[i]), (lds_ptr_t)(dst_ + X_RING + i * 1024), 16, 0, 0); \
  }

  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;

#pragma unroll
  for (int p = 0; p < INFL; ++p) HMI_COPY_STAGE(p)
  for (int s = 0; s < KT; ++s) {
    HMI_WAIT_VMCNT(8 * (INFL - 1));          // stage s has landed; the copies of the INFL - 1 stages after it may be in flight
    __builtin_amdgcn_sched_barrier(0);
    const unsigned char* sb = ring + (s % STAGES) * STAGE_BYTES;
    bf16x8 fw[4], fx[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      fw[ks] = *reinterpret_cast<const bf16x8*>(sb + (fw_base ^ (ks << 5)));
      fx[ks] = *reinterpret_cast<const bf16x8*>(sb + (fx_base ^ (ks << 5)));
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[ks], fx[ks], acc, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    HMI_COPY_STAGE(s + INFL)                 // into the slot that stage s - 1 was read from
  }
#undef HMI_COPY_STAGE
  HMI_WAIT_VMCNT(0);                         // the trailing copies must have landed before the LDS is handed on
  if (SPLIT) {
    // partial sums of wavefronts 1.. go through their own (now idle) rings; wavefront 0 adds them in order
    float* red = reinterpret_cast<float*>(ring);
    if (wave != 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) red[r * 64 + lane] = acc[r];
    }
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int w = 1; w < KSPLIT; ++w) {
      const float* part = reinterpret_cast<const float*>(smem + w * WAVE_LDS);
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] += part[r * 64 + lane];
    }
  }

  // ---- epilogue: lane (row l32, half lh) holds columns n0 + 16 lh + r, r = 0..15
  if (l32 < rows) {
  const int c0 = n0 + 16 * lh;
  const u32x4* bp = reinterpret_cast<const u32x4*>(g.pool + slot_base + g.b_off + (size_t)c0 * 2);
  const u32x4 b0 = bp[0], b1 = bp[1];
  float v[16];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    v[2 * e] = acc[2 * e] + bf2f(b0[e] & 0xFFFFu);         v[2 * e + 1] = acc[2 * e + 1] + bf2f(b0[e] >> 16);
    v[8 + 2 * e] = acc[8 + 2 * e] + bf2f(b1[e] & 0xFFFFu); v[8 + 2 * e + 1] = acc[8 + 2 * e + 1] + bf2f(b1[e] >> 16);
  }
  if (g.epi == EPI_BIAS_GELU) {
#pragma unroll
    for (int r = 0; r < 16; ++r) v[r] = gelu_erf(v[r]);
  } else if (g.epi == EPI_BIAS_RELU) {
#pragma unroll
    for (int r = 0; r < 16; ++r) v[r] = fmaxf(v[r], 0.0f);
  } else if (g.epi == EPI_BIAS_RESID) {
    if (g.resid_f32) {
      const f32x4* rp = reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(g.resid) + (size_t)my_row * g.ldr + c0);
#pragma unroll
      for (int q = 0; q < 4; ++q) { const f32x4 rv = rp[q]; v[4 * q] += rv[0]; v[4 * q + 1] += rv[1]; v[4 * q + 2] += rv[2]; v[4 * q + 3] += rv[3]; }
    } else {
      const u32x4* rp = reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(g.resid) + (size_t)my_row * g.ldr + c0);
      const u32x4 r0 = rp[0], r1 = rp[1];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[2 * e] += bf2f(r0[e] & 0xFFFFu);     v[2 * e + 1] += bf2f(r0[e] >> 16);
        v[8 + 2 * e] += bf2f(r1[e] & 0xFFFFu); v[8 + 2 * e + 1] += bf2f(r1[e] >> 16);
      }
    }
  }
  u32x4 h0, h1;
#pragma unroll
  for (int e = 0; e < 4; ++e) { h0[e] = pack_bf16(v[2 * e], v[2 * e + 1]); h1[e] = pack_bf16(v[8 + 2 * e], v[8 + 2 * e + 1]); }
  const size_t o = (size_t)my_row * g.ldc + c0;
  if (g.out_f32) {
    f32x4* cp = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.C) + o);
#pragma unroll
    for (int q = 0; q < 4; ++q) cp[q] = f32x4{v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]};
  } else {
    u32x4* cp = reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(g.C) + o);
    cp[0] = h0; cp[1] = h1;
  }
  if (g.C2) {
    u32x4* cp = reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(g.C2) + o);
    cp[0] = h0; cp[1] = h1;
  }
  }   // rows of this block
  }   // row blocks of the item
}

}  // namespace

template <bool SPLIT, bool DEEP>
static void allow_ring() {
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_skinny_kernel<SPLIT, DEEP, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, Ring<SPLIT, DEEP>::LDS_BYTES);
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_skinny_kernel<SPLIT, DEEP, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, Ring<SPLIT, DEEP>::LDS_BYTES);
}

void init_gemm_bf16_skinny_kernels() {
  allow_ring<false, false>(); allow_ring<false, true>(); allow_ring<true, true>();
}

template <bool SPLIT, bool DEEP>
static void launch_ring(const GemmArgs& g, const Route& rt, hipStream_t s, long long n_items, int row_split) {
  using R = Ring<SPLIT, DEEP>;
  const unsigned blocks = SPLIT ? (unsigned)n_items : (unsigned)((n_items + R::WAVES - 1) / R::WAVES);
  if (rt.identity)
    hipLaunchKernelGGL((gemm_bf16_skinny_kernel<SPLIT, DEEP, false>), dim3(blocks), dim3(64 * R::WAVES), R::LDS_BYTES, s,
                       g, rt, (int)n_items, row_split);
  else
    hipLaunchKernelGGL((gemm_bf16_skinny_kernel<SPLIT, DEEP, true>), dim3(blocks), dim3(64 * R::WAVES), R::LDS_BYTES, s,
                       g, rt, (int)n_items, row_split);
}

// Preconditions (checked by the caller): k % 64 == 0, n_out % 32 == 0, which_tiles names the list of
// 128-row m-tiles and n_mtiles its length, all operands 16-byte aligned (lda, ldc, ldr multiples of 8).
void launch_gemm_bf16_skinny(const GemmArgs& g, const Route& rt, hipStream_t s) {
  const int row_split = g.n_rows > 32LL * g.n_mtiles ? 1 : 0;
  const long long n_items = (long long)g.n_mtiles * (g.n_out / SK) * (row_split ? 4 : 1);
  if (n_items <= 0) return;
  // few items, long k: one workgroup per item with k shared by its wavefronts
  if (row_split && n_items <= kSplitMaxItems && g.k % (64 * KSPLIT) == 0 && g.k >= 64 * KSPLIT * 2)
    return launch_ring<true, true>(g, rt, s, n_items, row_split);
  if (n_items <= kDeepMaxItems) return launch_ring<false, true>(g, rt, s, n_items, row_split);
  launch_ring<false, false>(g, rt, s, n_items, row_split);
}

}  // namespace hmi
