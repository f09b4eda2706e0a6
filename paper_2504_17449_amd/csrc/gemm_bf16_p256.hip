// Grouped bf16 GEMM, persistent workgroups, 256 x 256 tiles with 64-wide k-stages: the main
// kernel for layers whose output width is a multiple of 256.
//
// Same contract as the other grouped GEMMs (one launch multiplies every tenant segment of a
// mixed batch by that tenant's own weights, Sec. 6.3):
//      C[rows, :] = epi( A[rows, :] * W_g^T + b_g )        for every m-tile of segment g
//
// Measured facts about gfx950 that shape it
//   * An L2 channel answers one request per clock: 128 bytes if the request covers a whole
//     cache line, 64 if it covers half of one (33 TB/s against 17-20 TB/s for direct-to-LDS
//     copies that hit in L2).  Stores follow the same rule: a wavefront store that touches
//     64 different lines costs 64 requests however few bytes it carries.
//   * The matrix pipe blocks a wavefront's instruction issue for half the duration of an
//     MFMA; about four other instructions fit behind each one.
//   * LDS reads run at 256 B/clk, fragment traffic is not a bound for 64 x 128 wavefront tiles.
// Hence
//   * 256 x 256 tiles: the fewest operand bytes per FLOP the register file allows, held either by
//     8 wavefronts x 128 accumulator registers (two wavefronts per SIMD) or by 4 wavefronts x 256
//     accumulators in the AGPR half of a 512-register budget (one per SIMD); see Geo below;
//   * k-stages of 64 bf16 = 128 bytes per row: the eight lanes that copy a row fetch one
//     whole cache line, every operand request is a full line;
//   * all 160 KB of LDS are a ring of 2 activation and 3 weight stages of 32 KB; weight
//     copies (mostly L2 misses: a weight panel is shared only by the m-tiles of one
//     tenant) run two stages ahead, activation copies (mostly hits) one.  A wavefront
//     issues activation copies before weight copies, so with in-order completion "all but
//     the newest weight stage have landed" is exactly the condition for the next stage;
//   * one workgroup per compute unit walks over its share of the tiles.  Copies for the
//     next tile are issued while the current one finishes, fragment reads are double
//     buffered in registers one k-step ahead (across stage and tile boundaries), and there
//     is one barrier per stage, placed so that the MFMAs of the last k-step hide it;
//   * operand roles are swapped (weights are the MFMA's first operand, in a permuted row
//     order): a lane ends up with one row of C and 16 consecutive columns per MFMA tile;
//     bias is folded into the accumulator initialisation.  For the stores each wavefront
//     transposes its results through the part of the two idle ring slots that only its
//     own copies overwrite (no barrier), so that 16 or 32 consecutive lanes write one
//     row's 256 or 512 contiguous bytes: full-line requests again.
#include "hmi_kernels.h"

namespace hmi {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kXcds = 8;
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int WTN = 128, TN = 4;                             // a wavefront's 128 columns: four MFMA tiles
// The workgroup is NW = 8 or 4 wavefronts, NW/2 x 2 over the tile: wavefront tiles of 64 x 128 (two per SIMD,
// 128 accumulator registers each) or 128 x 128 (one per SIMD with 256 accumulators in the AGPR half of a
// 512-register budget: a third less fragment traffic per MFMA and one instruction stream per matrix pipe,
// but nothing to run while that one wavefront waits, so it pays only where the main loop is long).
template <int NW>
struct Geo {
  static constexpr int NTH = 64 * NW;
  static constexpr int WTM = BM / (NW / 2), TM = WTM / 32;  // wavefront tile rows, MFMA tiles
  static constexpr int RH = WTM / 64;                       // output-row ids a lane keeps per tile
  static constexpr int LD = BM / 8 / NW;                    // one-KB copies (8 rows x 128 B) per wavefront, operand and stage: 4 or 8
  static constexpr int WAVE_SLICE = LD * 1024;              // the part of a stage slot that one wavefront's copies fill
};
constexpr int ROW_BYTES = BK * 2;                            // 128: one cache line per row and stage
constexpr int A_STAGES = 2, W_STAGES = 3;
constexpr int STAGE_BYTES = BM * ROW_BYTES;                  // 32 KB, same for both operands
constexpr int W_RING = A_STAGES * STAGE_BYTES;               // byte offset of the weight ring
constexpr int LDS_BYTES = W_RING + W_STAGES * STAGE_BYTES;   // 163840 = all of it

__device__ __forceinline__ float bf2f(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 p = {(__bf16)lo, (__bf16)hi};                       // round to nearest even
  return __builtin_bit_cast(uint32_t, p);
}

// GELU(x) = x Phi(x) = max(x, 0) - a Phi(-a) with a = |x|.  a Phi(-a) is a smooth bump (at
// most 0.17, below 1.3e-4 beyond a = 4): Phi(-a) is replaced by a degree-6 polynomial in
// u = a/2 - 1 on [0, 4], fitted so that |a (Q(u) - Phi(-a))| <= 2e-4 everywhere (a is clamped
// at 4); GELU(0) = 0 exactly.  Ten fp32 vector-ALU operations, no transcendental.  (The same
// polynomial in packed fp16 is 1.5 % of a launch faster, but its rounding lifts the error to
// 5e-4 near x = -3.8, where the result itself is only -2e-4: not used.)
__device__ __forceinline__ float gelu_poly(float x) {
  const float a = fminf(fabsf(x), 4.0f);
  const float u = fmaf(a, 0.5f, -1.0f);
  float q = -0.0411399369f;
  q = fmaf(q, u, 0.0706263031f);
  q = fmaf(q, u, 0.0492447267f);
  q = fmaf(q, u, -0.212425632f);
  q = fmaf(q, u, 0.219460411f);
  q = fmaf(q, u, -0.108456779f);
  q = fmaf(q, u, 0.0226731103f);
  return fmaf(-a, q, fmaxf(x, 0.0f));
}

// LDS chunk swizzles (a row is 8 chunks of 16 bytes, two rows per 256-byte bank line).
// Activation rows are read by consecutive lanes in consecutive order; weight rows in the
// permuted order perm_w.  Either way the 16 lanes served together hit 16 distinct chunks.
__device__ __forceinline__ int swz_a(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int swz_w(int row) { return ((row >> 1) & 3) | (((row >> 4) & 1) << 2); }
// MFMA first-operand position i (0..31) <- weight row perm_w(i) of the 32-row tile, chosen
// so that output register r of lane half h is column 16 h + r.
__device__ __forceinline__ int perm_w(int i) { return ((i >> 2) & 1) * 16 + (i >> 3) * 4 + (i & 3); }

// Timing-only ablations of the main loop (never set by the build script's defaults; RESULTS ARE WRONG with any of them):
//   -DHMI_ABLATE_MFMA=1    no MFMA is issued (fragments are still read from LDS)
//   -DHMI_ABLATE_READS=1   no fragment is read from LDS
//   -DHMI_ABLATE_COPIES=1  the steady-state stages issue no copy (prologues and tile changes still do)
//   -DHMI_ABLATE_WAIT=n    a stage waits until all but n (instead of one) operand stages of copies have landed
// They exist so that the time of each part of a stage can be measured with the launch shapes, addresses
// and tile order of the real kernel; every access they leave in is one the real kernel makes.
#ifndef HMI_ABLATE_MFMA
#define HMI_ABLATE_MFMA 0
#endif
#ifndef HMI_ABLATE_READS
#define HMI_ABLATE_READS 0
#endif
#ifndef HMI_ABLATE_COPIES
#define HMI_ABLATE_COPIES 0
#endif
#ifndef HMI_ABLATE_WAIT
#define HMI_ABLATE_WAIT 1
#endif
#if HMI_ABLATE_MFMA || HMI_ABLATE_READS || HMI_ABLATE_COPIES || HMI_ABLATE_WAIT != 1
#warning "gemm_bf16_p256: timing-only ablation build, results are wrong"
#endif

// Results leave with the non-temporal hint: nothing in this launch reads them again, and every line of L2 they do not
// take stays with the operand panels that other workgroups of the XCD are about to ask for (measured: 1-2 % fewer
// bytes fetched, GEMM time -0.7 to -1 % on the FFN, encoder and shared-layer workloads).
#define HMI_STORE_OUT(PTR, V) __builtin_nontemporal_store((V), (PTR))
#define HMI_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | (0x7 << 4) | (0xF << 8))
#define HMI_WAIT_LGKMCNT0() __builtin_amdgcn_s_waitcnt(0xC07F)

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

// What a lane needs to know about a tile: where its copies come from and where the bias is.
constexpr int kMBlock = 8;   // m-tiles per block of a long segment's tile order

template <int NW>
struct TileRegs {
  int n0, row0, rows;
  const char* Wb;                  // first weight row of the tile: tenant's matrix + n0 rows
  const uint16_t* bias;
  uint32_t a_off[Geo<NW>::LD];     // byte offsets of this lane's activation copy sources at k = 0, plus 3072 - 1024 j
  int out_row[Geo<NW>::RH];        // where row (wavefront's first row + 64 h + lane) of the tile goes in C (row clamped to the tile)
};

template <int NW>
__device__ __forceinline__ void load_tile(const GemmArgs& g, const Route& rt, int w, int wave, int lane, TileRegs<NW>& tr) {
  constexpr int WTM = Geo<NW>::WTM, RH = Geo<NW>::RH, LD = Geo<NW>::LD;
  // Tile order: segment by segment; inside a segment n-tile by n-tile with the segment's
  // m-tiles innermost, so that the tiles which share a weight panel (and the few that
  // share an activation panel) run next to each other and the panel is fetched from HBM once.
  const int nt_n = g.n_out / BN;
  const int mt_any = w / nt_n;                               // some m-tile of the segment w falls in
  const int seg = rt.tile_seg[g.which_tiles][mt_any];
  const int s0 = rt.seg_tok_off[seg], s1 = rt.seg_tok_off[seg + 1];
  const int mt_first = mt_any - (rt.tile_row0[g.which_tiles][mt_any] - s0) / BM;
  const int mt_cnt = (s1 - s0 + BM - 1) / BM;
  const int q = w - mt_first * nt_n;
  // A long segment goes block by block of kMBlock m-tiles (the last block may be shorter): an activation panel's
  // n-tiles are then at most kMBlock tiles apart, close enough to run in the same round of the XCD's workgroups.
  const int b = q / (kMBlock * nt_n);
  const int bm = b < mt_cnt / kMBlock ? kMBlock : mt_cnt - b * kMBlock;
  const int rem = q - b * (kMBlock * nt_n);
  tr.n0 = (rem / bm) * BN;
  tr.row0 = s0 + (b * kMBlock + rem % bm) * BM;
  tr.rows = min(BM, s1 - tr.row0);
  const size_t slot_base = (size_t)rt.seg_slot[seg] * g.slot_stride;
  tr.Wb = g.pool + slot_base + g.w_off + (size_t)tr.n0 * (size_t)(g.k * 2);
  tr.bias = reinterpret_cast<const uint16_t*>(g.pool + slot_base + g.b_off);
#pragma unroll
  for (int h = 0; h < RH; ++h) tr.out_row[h] = rt.row_src[tr.row0 + min((wave >> 1) * WTM + h * 64 + lane, tr.rows - 1)];
  // lane l fills LDS position (row l/8, chunk l%8) of an 8-row block with the global chunk
  // position ^ swizzle(row): the eight lanes of a row cover its whole 128-byte line.
#pragma unroll
  for (int j = 0; j < LD; ++j) {
    const int row = (wave * LD + j) * 8 + (lane >> 3);
    const int src = rt.row_src[tr.row0 + min(row, tr.rows - 1)];
    tr.a_off[j] = (uint32_t)src * (uint32_t)(g.lda * 2) + (((lane & 7) ^ swz_a(row)) << 4) + (3072 - (j & 3) * 1024);
  }
}


// The last workgroup of an XCD to finish puts the XCD's counters back to zero for the next launch.
__device__ __forceinline__ void finish_workgroup(const Route& rt, int xcd, int n_local) {
  if (threadIdx.x == 0) {
    int* done = rt.gemm_sched + 8 + xcd;
    if (atomicAdd(done, 1) == n_local - 1) {
      __hip_atomic_store(rt.gemm_sched + xcd, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

template <int NW, int EPI, bool OUT_F32, bool RESID_F32, bool HAS_C2>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(NW / 4, NW / 4)))
void gemm_bf16_p256_kernel(GemmArgs g, Route rt, int total, int per_xcd) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int WTM = Geo<NW>::WTM, TM = Geo<NW>::TM, LD = Geo<NW>::LD, WAVE_SLICE = Geo<NW>::WAVE_SLICE;

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const int KT = g.k / BK;
  const char* Ab = reinterpret_cast<const char*>(g.A);

  // ---- this workgroup's tiles: XCD x (workgroups are dealt to XCDs round robin) owns the
  // contiguous range [x per_xcd, (x+1) per_xcd).  A workgroup's first two tiles are fixed
  // (its index inside the XCD, plus one round); from the third on it claims the next
  // unclaimed tile of the range, so that workgroups that drew cheap (short) tiles take more.
  // Wavefront 0 claims the tile after next at the start of a tile and passes the answer to
  // the other wavefronts through a mailbox in global memory (LDS has no byte to spare).
  const int n_local = gridDim.x / kXcds;
  const int xcd = blockIdx.x % kXcds;
  const int w_base = xcd * per_xcd;
  const int w_end = min(w_base + per_xcd, total);
  int* const claim_ctr = rt.gemm_sched + xcd;
  int* const mailbox = rt.gemm_sched + 16 + blockIdx.x;
  int w = w_base + blockIdx.x / kXcds;
  int w_next = w + n_local;
  if (w >= w_end) { finish_workgroup(rt, xcd, n_local); return; }
  const bool claimer = wave == 0 && lane == 0;
  int claimed = 0, mail = 0;
  if (claimer) claimed = atomicAdd(claim_ctr, 1);
  int budget = per_xcd;           // no workgroup can own more tiles than its XCD has: bounds the loop whatever the claims say

  TileRegs<NW> cur, nxt;
  load_tile(g, rt, w, wave, lane, cur);
  load_tile(g, rt, w_next < w_end ? w_next : w, wave, lane, nxt);

  // weight copies: the lane part of the source offset (plus 3072 - 1024 j) is the same for every tile
  uint32_t b_off[LD];
#pragma unroll
  for (int j = 0; j < LD; ++j) {
    const int row = (wave * LD + j) * 8 + (lane >> 3);
    b_off[j] = (uint32_t)row * (uint32_t)(g.k * 2) + (((lane & 7) ^ swz_w(row)) << 4) + (3072 - (j & 3) * 1024);
  }

  // ---- fragment read offsets inside a stage slot for the four k-steps of a stage
  // (k-step ks reads chunk (2 ks + lh) ^ swizzle: that is the k-step 0 offset with ks << 5 XORed in)
  int fx_base, fw_base;
  {
    const int rx = wm * WTM + l32;                       // + 32 i: swizzle unchanged
    const int rw = wn * WTN + perm_w(l32);               // + 32 j: swizzle unchanged
    fx_base = rx * ROW_BYTES + ((lh ^ swz_a(rx)) << 4);
    fw_base = W_RING + rw * ROW_BYTES + ((lh ^ swz_w(rw)) << 4);
  }

  // Ring bookkeeping (uniform): a_rd / w_rd are the byte offsets of the slots that hold the
  // stage being multiplied.  Activation stage s+2 and weight stage s+3 are copied into exactly
  // those slots once stage s is done, so no separate fill position is needed; a stage index
  // of KT or more means a stage of the next tile (for the last tile: an in-bounds re-read
  // of its own first stages that nobody consumes).  Needs KT >= 3, so that the copies
  // never reach the tile after next.
  int a_rd = 0, w_rd = 0;
  // Four 1 KB copies of a wavefront's slice (all of it, or half) share one LDS base (one M0 write); the
  // instruction offset j KB that separates them applies to the global address too, so
  // the lane offsets carry 3072 - j KB and the uniform base pointer -3072.
#define HMI_COPY4(SRC, VOFF, SLOT_OFF)                                                            \
  {                                                                                               \
    const char* src_ = (SRC) - 3072;                                                              \
    _Pragma("unroll") for (int q_ = 0; q_ < LD / 4; ++q_) {                                       \
      lds_ptr_t dst_ = (lds_ptr_t)(smem + (SLOT_OFF) + wave * WAVE_SLICE + q_ * 4096);            \
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(src_ + (VOFF)[4 * q_ + 0]), dst_, 16, 0, 0);    \
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(src_ + (VOFF)[4 * q_ + 1]), dst_, 16, 1024, 0); \
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(src_ + (VOFF)[4 * q_ + 2]), dst_, 16, 2048, 0); \
      __builtin_amdgcn_global_load_lds((glb_ptr_t)(src_ + (VOFF)[4 * q_ + 3]), dst_, 16, 3072, 0); \
    }                                                                                             \
  }
  static_assert(LD % 4 == 0, "HMI_COPY4 issues the copies in groups of four");

  bf16x8 fx[2][TM], fw[2][TN];
  f32x16 acc[TM][TN];

  // loads the MFMA fragments of k-step KS of the stage in slots a_rd / w_rd into register buffer B
#define HMI_READ_FRAGS(B, KS)                                                                     \
  if (!HMI_ABLATE_READS) {                                                                                               \
    const unsigned char* xa_ = smem + a_rd + (fx_base ^ ((KS) << 5));                             \
    const unsigned char* wa_ = smem + w_rd + (fw_base ^ ((KS) << 5));                             \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) fx[B][i] = *reinterpret_cast<const bf16x8*>(xa_ + i * 32 * ROW_BYTES); \
    _Pragma("unroll") for (int j = 0; j < TN; ++j) fw[B][j] = *reinterpret_cast<const bf16x8*>(wa_ + j * 32 * ROW_BYTES); \
  }
#if HMI_ABLATE_MFMA
#define HMI_MFMAS(B)   /* keeps the fragment registers (and so their reads) alive */                  \
  _Pragma("unroll") for (int i = 0; i < TM; ++i) asm volatile("" :: "v"(fx[B][i]));               \
  _Pragma("unroll") for (int j = 0; j < TN; ++j) asm volatile("" :: "v"(fw[B][j]));
#else
#define HMI_MFMAS(B)                                                                              \
  _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                  \
    _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[B][j], fx[B][i], acc[i][j], 0, 0, 0);
#endif

  // scheduling: each of the 6 fragment reads of the next k-step goes behind one MFMA of
  // this k-step (the wait for this k-step's fragments then comes before any new read)
#define HMI_SCHED_READS_THEN_MFMAS()                                                              \
  _Pragma("unroll") for (int z_ = 0; z_ < TM + TN; ++z_) {                                        \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                            \
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                            \
  }                                                                                               \
  __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - TM - TN, 0);                              \
  __builtin_amdgcn_sched_barrier(0);

  // accumulators of a tile start at its bias: lane half h of MFMA tile j holds columns
  // n0 + wn*128 + j*32 + 16 h + (0..15), the same for both m-tiles.
#define HMI_INIT_ACC(TR)                                                                          \
  _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                                \
    const int col0_ = (TR).n0 + wn * WTN + j * 32 + 16 * lh;                                      \
    const u32x4 b0_ = *reinterpret_cast<const u32x4*>((TR).bias + col0_);                         \
    const u32x4 b1_ = *reinterpret_cast<const u32x4*>((TR).bias + col0_ + 8);                     \
    _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                               \
      acc[0][j][2 * q] = bf2f(b0_[q] & 0xffffu);      acc[0][j][2 * q + 1] = bf2f(b0_[q] >> 16);  \
      acc[0][j][8 + 2 * q] = bf2f(b1_[q] & 0xffffu);  acc[0][j][8 + 2 * q + 1] = bf2f(b1_[q] >> 16); \
    }                                                                                             \
    _Pragma("unroll") for (int i = 1; i < TM; ++i) acc[i][j] = acc[0][j];                         \
  }

  // One stage.  MODE says where the copies issued after the barrier come from:
  //   0: activation stage s+2 and weight stage s+3 of the current tile
  //   1: (s = KT-3) activation stage KT-1 of the current tile, weight stage 0 of the next
  //   2: (s = KT-2) activation stage 0 and weight stage 1 of the next tile
  //   3: (s = KT-1) none: the freed slots serve the epilogue first
#define HMI_STAGE_COPIES(MODE)                                                                    \
  {                                                                                               \
    if (MODE == 0 && !HMI_ABLATE_COPIES) { HMI_COPY4(Ab + (s + 2) * ROW_BYTES, cur.a_off, fa_) HMI_COPY4(cur.Wb + (s + 3) * ROW_BYTES, b_off, W_RING + fw_) } \
    if (MODE == 1) { HMI_COPY4(Ab + (s + 2) * ROW_BYTES, cur.a_off, fa_) HMI_COPY4(nxt.Wb, b_off, W_RING + fw_) }                     \
    if (MODE == 2) { HMI_COPY4(Ab, nxt.a_off, fa_) HMI_COPY4(nxt.Wb + ROW_BYTES, b_off, W_RING + fw_) }                                \
  }
#define HMI_ITER(MODE)                                                                            \
  {                                                                                               \
    if (wave_active) {                                                                            \
      HMI_READ_FRAGS(1, 1)                                                                        \
      HMI_MFMAS(0)                                                                                \
      HMI_SCHED_READS_THEN_MFMAS()                                                                \
      HMI_READ_FRAGS(0, 2)                                                                        \
      HMI_MFMAS(1)                                                                                \
      HMI_SCHED_READS_THEN_MFMAS()                                                                \
      HMI_READ_FRAGS(1, 3)                                                                        \
      HMI_MFMAS(0)                                                                                \
      HMI_SCHED_READS_THEN_MFMAS()                                                                \
    }                                                                                             \
    HMI_WAIT_LGKMCNT0();          /* this wavefront no longer reads stage s from LDS */           \
    if (MODE == 2 && wave == 0) { HMI_WAIT_VMCNT(0); }   /* ... and its mailbox store is done */   \
    else { HMI_WAIT_VMCNT(HMI_ABLATE_WAIT * LD); }  /* its copies of stage s+1 (both operands) have landed */       \
    __builtin_amdgcn_s_barrier(); /* ... everybody's, and nobody reads stage s any more */        \
    __builtin_amdgcn_sched_barrier(0);                                                            \
    if (MODE == 1 && claimer) __hip_atomic_store(mailbox, claimed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); \
    if (MODE == 2) mail = __hip_atomic_load(mailbox, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  \
    const int fa_ = a_rd, fw_ = w_rd;                                                             \
    a_rd ^= STAGE_BYTES;                                                                          \
    w_rd = w_rd == (W_STAGES - 1) * STAGE_BYTES ? 0 : w_rd + STAGE_BYTES;                         \
    if (MODE == 3) {                                                                              \
      patch_a = fa_; patch_w = fw_;                                                               \
      if (wm * WTM < nxt.rows) HMI_READ_FRAGS(0, 0)                                               \
      __builtin_amdgcn_sched_barrier(0);                                                          \
      if (wave_active) { HMI_MFMAS(1) }                                                           \
    } else if (wave_active) {                                                                     \
      /* first fragments of stage s+1, then the last k-step's MFMAs with the copies between them */ \
      HMI_READ_FRAGS(0, 0)                                                                        \
      HMI_STAGE_COPIES(MODE)                                                                      \
      HMI_MFMAS(1)                                                                                \
      __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);                                    \
      _Pragma("unroll") for (int z_ = 0; z_ < 2 * LD; ++z_) {                                     \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                        \
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                        \
      }                                                                                           \
    } else {                                                                                      \
      HMI_STAGE_COPIES(MODE)                                                                      \
    }                                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                            \
  }

  // ---- prologue of the first tile.  Issue order W(0) A(0) W(1) A(1) W(2) is the steady
  // state's order, so the same "all but the newest weight stage" wait works from the start.
  HMI_INIT_ACC(cur)
  HMI_COPY4(cur.Wb, b_off, W_RING)
  HMI_COPY4(Ab, cur.a_off, 0)
  HMI_COPY4(cur.Wb + ROW_BYTES, b_off, W_RING + STAGE_BYTES)
  HMI_COPY4(Ab + ROW_BYTES, cur.a_off, STAGE_BYTES)
  HMI_COPY4(cur.Wb + 2 * ROW_BYTES, b_off, W_RING + 2 * STAGE_BYTES)
  HMI_WAIT_VMCNT(3 * LD);
  __builtin_amdgcn_s_barrier();
  bool wave_active = wm * WTM < cur.rows;
  if (wave_active) HMI_READ_FRAGS(0, 0)
  int patch_a = 0, patch_w = 0;

  for (;;) {
    // ================= main loop of the current tile =================
    {
      int s = 0;
      for (; s < KT - 3; ++s) HMI_ITER(0)
      HMI_ITER(1)
      HMI_ITER(2)
      HMI_ITER(3)
    }

    // ================= epilogue of the current tile =================
    // Staging patch of this wavefront: the first 4 KB of its own slice of the two slots that stage KT-1
    // occupied.  A row keeps its 16-byte chunk c at chunk position c ^ (row & 15).
    // Rows past the end of a short tile are replaced by the tile's last row of the same
    // 32-row block (same data to the same address: harmless), which keeps the code free
    // of branches so that the loads and stores of a pass are issued back to back.
    if (wave_active) {
      unsigned char* patch0 = smem + patch_a + wave * WAVE_SLICE;
      unsigned char* patch1 = smem + W_RING + patch_w + wave * WAVE_SLICE;
      // The 8 KB patch holds 32 rows of 256 bytes (rows 0-15 in patch0, 16-31 in patch1): all
      // 128 columns of an MFMA tile row as bf16, or 64 of them as fp32 (two passes).  After
      // the transposition 16 lanes hold one row's 256 contiguous bytes, 4 rows per step.
      // Results that get a residual added cross the patch in fp32 even if they are stored as
      // bf16, so that they are rounded once, after the addition.
      constexpr bool STAGE_F32 = OUT_F32 || EPI == EPI_BIAS_RESID;
      constexpr int PASSES = STAGE_F32 ? 2 : 1;
      constexpr int COLS_PER_CHUNK = STAGE_F32 ? 4 : 8;
      const int c = lane & 15;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int mbase = wm * WTM + i * 32;
        if (mbase < cur.rows) {
          if (NW == 4) {   // the row blocks still to come stay where the MFMAs left them (the AGPR half) until their turn
#pragma unroll
            for (int i2 = i + 1; i2 < TM; ++i2)
#pragma unroll
              for (int j = 0; j < TN; ++j) asm volatile("" : "+a"(acc[i2][j]));
          }
          const int rmax = min(31, cur.rows - 1 - mbase);     // last valid row of this 32-row block
          unsigned char* wrow = ((l32 & 16) ? patch1 : patch0) + (l32 & 15) * 256;
          uint32_t orow[8];                                   // row of C for each of this lane's 8 pieces
#pragma unroll
          for (int it = 0; it < 8; ++it) orow[it] = (uint32_t)__shfl(cur.out_row[i >> 1], (i & 1) * 32 + min(it * 4 + (lane >> 4), rmax), 64);
#pragma unroll
          for (int pass = 0; pass < PASSES; ++pass) {
            const int col = cur.n0 + wn * WTN + pass * 64 + c * COLS_PER_CHUNK;
            // residuals first, so that they arrive while the results cross the patch
            f32x4 rv32[(EPI == EPI_BIAS_RESID && RESID_F32) ? 8 : 1];
            u32x2 rv16[(EPI == EPI_BIAS_RESID && !RESID_F32) ? 8 : 1];
            if (EPI == EPI_BIAS_RESID) {
#pragma unroll
              for (int it = 0; it < 8; ++it) {
                if (RESID_F32) rv32[it] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(g.resid) + (size_t)orow[it] * g.ldr + col);
                else rv16[it] = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint16_t*>(g.resid) + (size_t)orow[it] * g.ldr + col);
              }
            }
            // accumulator layout -> patch
            if (STAGE_F32) {
#pragma unroll
              for (int jj = 0; jj < 2; ++jj) {
                const int j = pass * 2 + jj;
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                  f32x4 o = {acc[i][j][4 * qd], acc[i][j][4 * qd + 1], acc[i][j][4 * qd + 2], acc[i][j][4 * qd + 3]};
                  if (EPI == EPI_BIAS_GELU) { o[0] = gelu_poly(o[0]); o[1] = gelu_poly(o[1]); o[2] = gelu_poly(o[2]); o[3] = gelu_poly(o[3]); }
                  else if (EPI == EPI_BIAS_RELU) { o[0] = fmaxf(o[0], 0.f); o[1] = fmaxf(o[1], 0.f); o[2] = fmaxf(o[2], 0.f); o[3] = fmaxf(o[3], 0.f); }
                  const int c0 = jj * 8 + lh * 4 + qd;
                  *reinterpret_cast<f32x4*>(wrow + ((c0 ^ (l32 & 15)) << 4)) = o;
                }
              }
            } else {
#pragma unroll
              for (int j = 0; j < TN; ++j) {
                u32x4 h0, h1;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  float v0 = acc[i][j][2 * e], v1 = acc[i][j][2 * e + 1], v2 = acc[i][j][8 + 2 * e], v3 = acc[i][j][8 + 2 * e + 1];
                  if (EPI == EPI_BIAS_GELU) {
                    h0[e] = pack_bf16(gelu_poly(v0), gelu_poly(v1)); h1[e] = pack_bf16(gelu_poly(v2), gelu_poly(v3));
                  } else {
                    if (EPI == EPI_BIAS_RELU) { v0 = fmaxf(v0, 0.0f); v1 = fmaxf(v1, 0.0f); v2 = fmaxf(v2, 0.0f); v3 = fmaxf(v3, 0.0f); }
                    h0[e] = pack_bf16(v0, v1); h1[e] = pack_bf16(v2, v3);
                  }
                }
                const int c0 = j * 4 + lh * 2;
                *reinterpret_cast<u32x4*>(wrow + ((c0 ^ (l32 & 15)) << 4)) = h0;
                *reinterpret_cast<u32x4*>(wrow + (((c0 + 1) ^ (l32 & 15)) << 4)) = h1;
              }
            }
            HMI_WAIT_LGKMCNT0();
            // patch -> rows of C
#pragma unroll
            for (int it = 0; it < 8; ++it) {
              const int r = min(it * 4 + (lane >> 4), rmax);
              const unsigned char* rrow = ((r & 16) ? patch1 : patch0) + (r & 15) * 256;
              const size_t off = (size_t)orow[it] * g.ldc + col;
              if (STAGE_F32) {
                f32x4 v = *reinterpret_cast<const f32x4*>(rrow + ((c ^ (r & 15)) << 4));
                if (EPI == EPI_BIAS_RESID) {
                  if (RESID_F32) v += rv32[it];
                  else {
                    v[0] += bf2f(rv16[it][0] & 0xffffu); v[1] += bf2f(rv16[it][0] >> 16);
                    v[2] += bf2f(rv16[it][1] & 0xffffu); v[3] += bf2f(rv16[it][1] >> 16);
                  }
                }
                const u32x2 hh = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
                if (OUT_F32) HMI_STORE_OUT(reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.C) + off), v);
                else HMI_STORE_OUT(reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(g.C) + off), hh);
                if (HAS_C2) HMI_STORE_OUT(reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(g.C2) + off), hh);
              } else {
                const u32x4 h = *reinterpret_cast<const u32x4*>(rrow + ((c ^ (r & 15)) << 4));
                HMI_STORE_OUT(reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(g.C) + off), h);
                if (HAS_C2) HMI_STORE_OUT(reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(g.C2) + off), h);
              }
            }
          }
        }
      }
    }

    // ================= move on to the next tile =================
    w = w_next;
    if (w >= w_end || --budget <= 0) break;
    w_next = w_base + 2 * n_local + __builtin_amdgcn_readfirstlane(mail);
    if (claimer) claimed = atomicAdd(claim_ctr, 1);
    cur = nxt;
    wave_active = wm * WTM < cur.rows;
    HMI_INIT_ACC(cur)
    // the copies that were held back at the last stage (the new tile's activation stage 1
    // and weight stage 2) go into the slots the epilogue just used; a wavefront's copies
    // fill only its own slice of a slot, which is its own staging patch: no barrier
    HMI_COPY4(Ab + ROW_BYTES, cur.a_off, patch_a)
    HMI_COPY4(cur.Wb + 2 * ROW_BYTES, b_off, W_RING + patch_w)
    load_tile(g, rt, w_next < w_end ? w_next : w, wave, lane, nxt);
  }
  HMI_WAIT_VMCNT(0);   // none of this workgroup's copies may outlive it
  finish_workgroup(rt, xcd, n_local);
}

template <int NW, int EPI, bool OUT_F32, bool RESID_F32, bool HAS_C2>
void launch_one(const GemmArgs& g, const Route& rt, hipStream_t s) {
  auto kern = gemm_bf16_p256_kernel<NW, EPI, OUT_F32, RESID_F32, HAS_C2>;
  const int n_cu = rt.n_cu >= kXcds ? rt.n_cu : 256;
  const int nt_n = g.n_out / BN;
  const long long total = (long long)g.n_mtiles * nt_n;
  if (total <= 0) return;
  const int per_xcd = (int)((total + kXcds - 1) / kXcds);
  const int local = per_xcd < n_cu / kXcds ? per_xcd : n_cu / kXcds;   // workgroups per XCD: at most one per compute unit
  hipLaunchKernelGGL(kern, dim3(local * kXcds), dim3(Geo<NW>::NTH), LDS_BYTES, s, g, rt, (int)total, per_xcd);
}

template <int NW, int EPI, bool OUT_F32, bool RESID_F32, bool HAS_C2>
void allow_lds() {
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_p256_kernel<NW, EPI, OUT_F32, RESID_F32, HAS_C2>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
}

// Which geometry a launch gets (measured on the FFN and encoder workloads): launches that add a residual (output
// projection, second FFN GEMM) run with four wavefronts, 3-6 % faster there (no spills in their fp32 epilogue, a
// long main loop in the second FFN GEMM); bias-only and activation launches keep eight, whose two wavefronts per
// SIMD overlap each other's epilogue latencies (the first FFN GEMM is 11 % slower with four).
constexpr int kWavesPlain = 8, kWavesResid = 4;
}  // namespace

// every instantiation launch_gemm_bf16_p256 can pick
void init_gemm_bf16_p256_kernels() {
  allow_lds<kWavesPlain, EPI_BIAS, false, false, true>();   allow_lds<kWavesPlain, EPI_BIAS, false, false, false>();
  allow_lds<kWavesPlain, EPI_BIAS_GELU, false, false, false>();
  allow_lds<kWavesPlain, EPI_BIAS_RELU, false, false, false>();
  allow_lds<kWavesResid, EPI_BIAS_RESID, true, true, true>();   allow_lds<kWavesResid, EPI_BIAS_RESID, true, true, false>();
  allow_lds<kWavesResid, EPI_BIAS_RESID, true, false, true>();  allow_lds<kWavesResid, EPI_BIAS_RESID, true, false, false>();
  allow_lds<kWavesResid, EPI_BIAS_RESID, false, true, false>(); allow_lds<kWavesResid, EPI_BIAS_RESID, false, false, false>();
}

// Preconditions (checked by the caller): n_out % 256 == 0, k % 64 == 0, k >= 192,
// which_tiles names a list of 256-row m-tiles, all operands 16-byte aligned,
// byte offsets of A rows and of W rows inside a slot below 4 GB.
void launch_gemm_bf16_p256(const GemmArgs& g, const Route& rt, hipStream_t s) {
  const bool c2 = g.C2 != nullptr;
  switch (g.epi) {
    case EPI_BIAS:
      return c2 ? launch_one<kWavesPlain, EPI_BIAS, false, false, true>(g, rt, s) : launch_one<kWavesPlain, EPI_BIAS, false, false, false>(g, rt, s);
    case EPI_BIAS_GELU:
      return launch_one<kWavesPlain, EPI_BIAS_GELU, false, false, false>(g, rt, s);
    case EPI_BIAS_RELU:
      return launch_one<kWavesPlain, EPI_BIAS_RELU, false, false, false>(g, rt, s);
    default:
      if (g.out_f32) {
        if (g.resid_f32) return c2 ? launch_one<kWavesResid, EPI_BIAS_RESID, true, true, true>(g, rt, s) : launch_one<kWavesResid, EPI_BIAS_RESID, true, true, false>(g, rt, s);
        return c2 ? launch_one<kWavesResid, EPI_BIAS_RESID, true, false, true>(g, rt, s) : launch_one<kWavesResid, EPI_BIAS_RESID, true, false, false>(g, rt, s);
      }
      if (g.resid_f32) return launch_one<kWavesResid, EPI_BIAS_RESID, false, true, false>(g, rt, s);
      return launch_one<kWavesResid, EPI_BIAS_RESID, false, false, false>(g, rt, s);
  }
}

}  // namespace hmi
