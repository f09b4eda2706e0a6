// Grouped bf16 GEMM on the gfx950 matrix cores with fused epilogues: the dispatcher and the
// two kernels for the shapes the persistent 256 x 256 kernel (gemm_bf16_p256.hip) does not
// take: a short or odd k (k < 192 or k % 64 != 0) and output widths that are not a multiple
// of 256 (adapter ranks, small test shapes).
//
// Computes, for every m-tile the router emitted (all rows of a tile belong to one tenant
// segment g):   C[rows, :] = epi( A[rows, :] * W_g^T + b_g )
// where W_g ([n_out, k] row-major, i.e. Linear(a) = W a + b of Sec. 3.2.2) is read from
// the HBM slot of segment g.  This is the "different requests, different parameters, one
// launch" step of Sec. 6.3 without materialising per-request parameter copies.
//
// Mapping to the hardware
//   * v_mfma_f32_32x32x16_bf16: both operands are K-contiguous, which is exactly how the
//     activations ([row, k]) and the weights ([out, k]) are stored, so an operand fragment
//     is one 16-byte LDS read per lane.
//   * workgroup tile BM x BN staged through LDS; 16-byte chunks are XOR-swizzled by row so
//     that the rows a half-wavefront reads hit distinct banks.
//   * wavefronts are laid out WM x WN; each owns (BM/WM) x (BN/WN) of C in accumulators.
//   * workgroup ids are folded so that each of the 8 XCDs (which get workgroups round
//     robin) works on a contiguous range of tiles: tiles that share a weight panel or an
//     activation panel then share that XCD's L2.
// Two main loops:
//   * dma kernel (the fast path, n_out % 256 == 0): global -> LDS copies are issued as
//     direct-to-LDS loads (no staging registers), four 32-wide k-stages deep, one raw
//     s_barrier per stage, vmcnt-counted so that three stages stay in flight.
//   * staged kernel (any n_out): global -> registers -> LDS, two 64-wide k-stages.
#include "hmi_kernels.h"

namespace hmi {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte chunk (8 bf16)

constexpr int kXcds = 8;

__device__ __forceinline__ float bf2f(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) {
  __bf16 b = (__bf16)f;  // round to nearest even
  return __builtin_bit_cast(uint16_t, b);
}

// Exact GELU x * Phi(x), as in the skinny and fp32 kernels (these tiles serve odd shapes; their
// epilogue is not on the measured path).
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

// Which tile does this workgroup own.  Returns false for padding workgroups.
struct TileCoord { int mt, n0, seg, row0, rows; size_t slot_base; };
template <int BM, int BN>
__device__ __forceinline__ bool locate_tile(const GemmArgs& g, const Route& rt, TileCoord& tc) {
  const int nt_n = (g.n_out + BN - 1) / BN;
  const int total = g.n_mtiles * nt_n;
  const int per = (total + kXcds - 1) / kXcds;
  const int local = blockIdx.x / kXcds;
  const int w = (blockIdx.x % kXcds) * per + local;
  if (local >= per || w >= total) return false;
  tc.mt = w / nt_n;
  tc.n0 = (w % nt_n) * BN;
  tc.seg = rt.tile_seg[g.which_tiles][tc.mt];
  tc.row0 = rt.tile_row0[g.which_tiles][tc.mt];
  tc.rows = min(BM, rt.seg_tok_off[tc.seg + 1] - tc.row0);
  tc.slot_base = (size_t)rt.seg_slot[tc.seg] * g.slot_stride;
  return true;
}

// Epilogue.  Accumulator register r of MFMA tile (i,j) holds
//      row = 8*(r/4) + 4*(lane/32) + r%4,  column = lane%32,
// i.e. a lane owns one column of 16 rows: storing from there would be 2- or 4-byte
// scattered writes.  Instead each wavefront transposes its tile through a private LDS
// patch, 32 rows at a time: bias and activation are applied in the accumulator layout
// (bias is per column = per lane), the fp32 values go to LDS row-major, and are read back
// as 16-byte row pieces so that residual loads and result stores are full-line coalesced
// vector accesses.  No workgroup barrier is needed (the patch is wavefront-private).
constexpr int kEpiPad = 8;   // words; makes the two half-wavefronts hit different banks
template <int WTN> constexpr int epi_patch_bytes() { return 32 * (WTN + kEpiPad) * 4; }

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

template <int TM, int TN, int WTM, int WTN>
__device__ __forceinline__ void epilogue(const GemmArgs& g, f32x16 (&acc)[TM][TN], const int* rowsrc_s,
                                         float* patch /* this wavefront's LDS patch */,
                                         const uint16_t* bias, int rows, int n0, int wm, int wn,
                                         int lane) {
  constexpr int PITCH = WTN + kEpiPad;
  constexpr int LANES_PER_ROW = WTN / 4, ROWS_PER_IT = 64 / LANES_PER_ROW, ITS = 32 / ROWS_PER_IT;
  const int l32 = lane & 31, lh = lane >> 5;
  const int epi = g.epi;
  const int rcol = 4 * (lane % LANES_PER_ROW), rrow = lane / LANES_PER_ROW;
  const int gcol = n0 + wn * WTN + rcol;
  float bv[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = n0 + wn * WTN + j * 32 + l32;
    bv[j] = col < g.n_out ? bf2f(bias[col]) : 0.0f;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int mbase = wm * WTM + i * 32;
    if (mbase >= rows) break;
    // accumulator layout -> LDS patch (row-major)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = acc[i][j][r] + bv[j];
        if (epi == EPI_BIAS_GELU) v = gelu_erf(v);
        else if (epi == EPI_BIAS_RELU) v = fmaxf(v, 0.0f);
        patch[((r >> 2) * 8 + lh * 4 + (r & 3)) * PITCH + j * 32 + l32] = v;
      }
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this wavefront's LDS writes are done
    // LDS patch -> global, 16-byte row pieces.  Rows past the end of a short tile are replaced
    // by the block's last valid row (same value to the same address: harmless), so that there
    // is no branch per piece and the residual loads of a batch are issued back to back,
    // ahead of the stores.
    if (gcol < g.n_out) {
      const int rmax = min(31, rows - 1 - mbase);
      constexpr int BATCH = ITS < 8 ? ITS : 8;
#pragma unroll
      for (int it0 = 0; it0 < ITS; it0 += BATCH) {
        size_t orow[BATCH];
        f32x4 rv32[BATCH];
        u16x4 rv16[BATCH];
#pragma unroll
        for (int b = 0; b < BATCH; ++b) {
          const int lr = min((it0 + b) * ROWS_PER_IT + rrow, rmax);
          orow[b] = (size_t)rowsrc_s[mbase + lr];
          if (epi == EPI_BIAS_RESID) {
            if (g.resid_f32) rv32[b] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(g.resid) + orow[b] * g.ldr + gcol);
            else rv16[b] = *reinterpret_cast<const u16x4*>(reinterpret_cast<const uint16_t*>(g.resid) + orow[b] * g.ldr + gcol);
          }
        }
#pragma unroll
        for (int b = 0; b < BATCH; ++b) {
          const int lr = min((it0 + b) * ROWS_PER_IT + rrow, rmax);
          f32x4 v = *reinterpret_cast<const f32x4*>(patch + lr * PITCH + rcol);
          if (epi == EPI_BIAS_RESID) {
            if (g.resid_f32) v += rv32[b];
            else { v[0] += bf2f(rv16[b][0]); v[1] += bf2f(rv16[b][1]); v[2] += bf2f(rv16[b][2]); v[3] += bf2f(rv16[b][3]); }
          }
          u16x4 h;
          h[0] = f2bf(v[0]); h[1] = f2bf(v[1]); h[2] = f2bf(v[2]); h[3] = f2bf(v[3]);
          if (g.out_f32) *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.C) + orow[b] * g.ldc + gcol) = v;
          else *reinterpret_cast<u16x4*>(reinterpret_cast<uint16_t*>(g.C) + orow[b] * g.ldc + gcol) = h;
          if (g.C2) *reinterpret_cast<u16x4*>(reinterpret_cast<uint16_t*>(g.C2) + orow[b] * g.ldc + gcol) = h;
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);   // reads done before the patch is overwritten
  }
}

// ======================================================================================
// dma kernel: direct-to-LDS loads, STAGES stages of BK = 32.
// LDS stage layout: A rows then B rows, 64 bytes (4 chunks of 16 B) per row; the chunk
// stored at position p of row r is global chunk p ^ swz4(r).
// ======================================================================================
__device__ __forceinline__ int swz4(int row) { return ((row >> 1) & 3) ^ ((row >> 3) & 1); }

#define HMI_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

template <int BM, int BN, int WM, int WN, int STAGES>
__global__ __launch_bounds__(64 * WM * WN) void gemm_bf16_dma_kernel(GemmArgs g, Route rt) {
  constexpr int DBK = 32;
  constexpr int NW = WM * WN, NTH = 64 * NW;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int A_LD = BM / 16 / NW, B_LD = BN / 16 / NW;   // 1 KB (16-row) loads per wavefront
  constexpr int STAGE_BYTES = (BM + BN) * DBK * 2;
  constexpr int LOADS_PER_STAGE = A_LD + B_LD;
  static_assert(BM % (16 * NW) == 0 && BN % (16 * NW) == 0, "tile/wavefront mismatch");
  static_assert(LOADS_PER_STAGE * (STAGES - 1) < 64, "vmcnt range");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_all[];
  int* rowsrc_s = reinterpret_cast<int*>(smem_all);                      // [BM]
  unsigned char* smem = smem_all + BM * sizeof(int);                     // stages, then epilogue patches

  TileCoord tc;
  if (!locate_tile<BM, BN>(g, rt, tc)) return;
  const int rows = tc.rows, n0 = tc.n0;
  const uint16_t* W = reinterpret_cast<const uint16_t*>(g.pool + tc.slot_base + g.w_off);
  const uint16_t* bias = reinterpret_cast<const uint16_t*>(g.pool + tc.slot_base + g.b_off);
  const uint16_t* A = reinterpret_cast<const uint16_t*>(g.A);

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int wm = wave / WN, wn = wave % WN;
  const int K = g.k;

  for (int i = t; i < BM; i += NTH) rowsrc_s[i] = rt.row_src[tc.row0 + min(i, rows - 1)];
  __syncthreads();

  // Each wavefront copies A_LD + B_LD blocks of 16 rows per stage.  Lane l brings the
  // chunk that belongs at LDS position (row l/4, slot l%4) of its block.
  const uint16_t* a_src[A_LD];
  const uint16_t* b_src[B_LD];
#pragma unroll
  for (int j = 0; j < A_LD; ++j) {
    const int row = (wave * A_LD + j) * 16 + (lane >> 2);
    a_src[j] = A + (size_t)rowsrc_s[row] * g.lda + (((lane & 3) ^ swz4(row)) << 3);
  }
#pragma unroll
  for (int j = 0; j < B_LD; ++j) {
    const int row = (wave * B_LD + j) * 16 + (lane >> 2);
    b_src[j] = W + (size_t)min(n0 + row, g.n_out - 1) * K + (((lane & 3) ^ swz4(row)) << 3);
  }
  const int KT = K / DBK;

  // Copies k-stage kt into LDS buffer kt % STAGES.  Past the end it re-reads the last
  // stage (in bounds) into a buffer nobody reads any more, which keeps vmcnt uniform.
#define HMI_ISSUE_STAGE(KT_IDX)                                                                   \
  {                                                                                               \
    const int kt_ = (KT_IDX);                                                                     \
    const int kc_ = min(kt_, KT - 1) * DBK;                                                       \
    unsigned char* base_ = smem + (kt_ % STAGES) * STAGE_BYTES;                                   \
    _Pragma("unroll") for (int j = 0; j < A_LD; ++j)                                              \
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(a_src[j] + kc_),                             \
                                         (lds_ptr_t)(base_ + (wave * A_LD + j) * 1024), 16, 0, 0);\
    _Pragma("unroll") for (int j = 0; j < B_LD; ++j)                                              \
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(b_src[j] + kc_),                             \
                                         (lds_ptr_t)(base_ + BM * DBK * 2 + (wave * B_LD + j) * 1024), 16, 0, 0); \
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // Fragment read offsets (bytes inside a stage) for the two k-steps of a stage.
  int fa_off[TM][2], fb_off[TN][2];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = wm * WTM + i * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) fa_off[i][ks] = row * 64 + (((ks * 2 + lh) ^ swz4(row)) << 4);
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int row = wn * WTN + j * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) fb_off[j][ks] = BM * DBK * 2 + row * 64 + (((ks * 2 + lh) ^ swz4(row)) << 4);
  }

  const bool wave_active = wm * WTM < rows;

#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s) HMI_ISSUE_STAGE(s)

  for (int kt = 0; kt < KT; ++kt) {
    // stage kt has landed once at most STAGES-2 later stages are still in flight
    HMI_WAIT_VMCNT(LOADS_PER_STAGE * (STAGES - 2));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // every wavefront is past its reads of stage kt-1: its buffer can be refilled
    HMI_ISSUE_STAGE(kt + STAGES - 1)
    if (wave_active) {
      const unsigned char* base = smem + (kt % STAGES) * STAGE_BYTES;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        bf16x8 fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(base + fa_off[i][ks]);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(base + fb_off[j][ks]);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
#undef HMI_ISSUE_STAGE
  HMI_WAIT_VMCNT(0);   // drain the tail copies: the stage buffers are reused below
  __syncthreads();     // ... and every wavefront is done reading them
  if (!wave_active) return;
  epilogue<TM, TN, WTM, WTN>(g, acc, rowsrc_s, reinterpret_cast<float*>(smem + wave * epi_patch_bytes<WTN>()),
                             bias, rows, n0, wm, wn, lane);
}

// ======================================================================================
// staged kernel: global -> registers -> LDS, two stages of BK = 64.
// ======================================================================================
constexpr int BK = 64;          // k extent of one LDS stage (8 chunks of 8 bf16)
__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(64 * WM * WN) void gemm_bf16_kernel(GemmArgs g, Route rt) {
  constexpr int NTH = 64 * WM * WN;
  constexpr int WTM = BM / WM, WTN = BN / WN;      // wavefront tile
  constexpr int TM = WTM / 32, TN = WTN / 32;      // 32x32 MFMA tiles per wavefront
  constexpr int A_IT = BM * 8 / NTH, B_IT = BN * 8 / NTH;
  static_assert(BM * 8 % NTH == 0 && BN * 8 % NTH == 0, "tile/threads mismatch");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_all[];
  int* rowsrc_s = reinterpret_cast<int*>(smem_all);                 // [BM]
  unsigned char* smem = smem_all + BM * sizeof(int);                // stages, then epilogue patches
  uint16_t* As = reinterpret_cast<uint16_t*>(smem);                 // [2][BM*BK]
  uint16_t* Bs = As + 2 * BM * BK;                                  // [2][BN*BK]

  TileCoord tc;
  if (!locate_tile<BM, BN>(g, rt, tc)) return;
  const int rows = tc.rows, n0 = tc.n0;
  const uint16_t* W = reinterpret_cast<const uint16_t*>(g.pool + tc.slot_base + g.w_off);
  const uint16_t* bias = reinterpret_cast<const uint16_t*>(g.pool + tc.slot_base + g.b_off);
  const uint16_t* A = reinterpret_cast<const uint16_t*>(g.A);

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int wm = wave / WN, wn = wave % WN;
  const int K = g.k;

  for (int i = t; i < BM; i += NTH) rowsrc_s[i] = rt.row_src[tc.row0 + min(i, rows - 1)];
  __syncthreads();

  // ---- per-thread global source pointers and LDS destinations of the staging copies
  const uint16_t* a_src[A_IT];
  const uint16_t* b_src[B_IT];
  int a_dst[A_IT], b_dst[B_IT];
#pragma unroll
  for (int i = 0; i < A_IT; ++i) {
    const int q = t + NTH * i, row = q >> 3, c = q & 7;
    a_src[i] = A + (size_t)rowsrc_s[row] * g.lda + c * 8;
    a_dst[i] = row * BK + ((c ^ swz(row)) << 3);
  }
#pragma unroll
  for (int i = 0; i < B_IT; ++i) {
    const int q = t + NTH * i, row = q >> 3, c = q & 7;
    b_src[i] = W + (size_t)min(n0 + row, g.n_out - 1) * K + c * 8;
    b_dst[i] = row * BK + ((c ^ swz(row)) << 3);
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // A wavefront whose rows all lie beyond the tile's row count has nothing to multiply.
  const bool wave_active = wm * WTM < rows;

  {
    u32x4 ra[A_IT], rb[B_IT];
#pragma unroll
    for (int i = 0; i < A_IT; ++i) ra[i] = *reinterpret_cast<const u32x4*>(a_src[i]);
#pragma unroll
    for (int i = 0; i < B_IT; ++i) rb[i] = *reinterpret_cast<const u32x4*>(b_src[i]);
#pragma unroll
    for (int i = 0; i < A_IT; ++i) *reinterpret_cast<u32x4*>(As + a_dst[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_IT; ++i) *reinterpret_cast<u32x4*>(Bs + b_dst[i]) = rb[i];
  }
  __syncthreads();

  const int KT = K / BK;
  // One loop body, expanded with and without the multiply so that neither version has a
  // branch inside (a branch there lets the compiler sink the prefetch below the MFMAs).
  // The last iteration re-reads its own k-stage (in bounds) and parks it in the idle
  // buffer, which also keeps the body branch-free.
#define HMI_K_LOOP(ACTIVE)                                                                        \
  for (int kt = 0; kt < KT; ++kt) {                                                               \
    const int cur = kt & 1;                                                                       \
    const int k1 = min(kt + 1, KT - 1) * BK;                                                      \
    u32x4 ra[A_IT], rb[B_IT];                                                                     \
    _Pragma("unroll") for (int i = 0; i < A_IT; ++i)                                              \
        ra[i] = *reinterpret_cast<const u32x4*>(a_src[i] + k1);                                   \
    _Pragma("unroll") for (int i = 0; i < B_IT; ++i)                                              \
        rb[i] = *reinterpret_cast<const u32x4*>(b_src[i] + k1);                                   \
    __builtin_amdgcn_sched_barrier(0);                                                            \
    if (ACTIVE) {                                                                                 \
      const uint16_t* Ac = As + cur * BM * BK;                                                    \
      const uint16_t* Bc = Bs + cur * BN * BK;                                                    \
      _Pragma("unroll") for (int ks = 0; ks < BK / 16; ++ks) {                                    \
        const int chunk = ks * 2 + lh;                                                            \
        bf16x8 fa[TM], fb[TN];                                                                    \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                          \
          const int row = wm * WTM + i * 32 + l32;                                                \
          fa[i] = *reinterpret_cast<const bf16x8*>(Ac + row * BK + ((chunk ^ swz(row)) << 3));    \
        }                                                                                         \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                          \
          const int row = wn * WTN + j * 32 + l32;                                                \
          fb[j] = *reinterpret_cast<const bf16x8*>(Bc + row * BK + ((chunk ^ swz(row)) << 3));    \
        }                                                                                         \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                            \
          _Pragma("unroll") for (int j = 0; j < TN; ++j)                                          \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);\
      }                                                                                           \
    }                                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                            \
    uint16_t* An = As + (cur ^ 1) * BM * BK;                                                      \
    uint16_t* Bn = Bs + (cur ^ 1) * BN * BK;                                                      \
    _Pragma("unroll") for (int i = 0; i < A_IT; ++i)                                              \
        *reinterpret_cast<u32x4*>(An + a_dst[i]) = ra[i];                                         \
    _Pragma("unroll") for (int i = 0; i < B_IT; ++i)                                              \
        *reinterpret_cast<u32x4*>(Bn + b_dst[i]) = rb[i];                                         \
    __syncthreads();                                                                              \
  }
  if (wave_active) { HMI_K_LOOP(true) } else { HMI_K_LOOP(false) }
#undef HMI_K_LOOP

  // the loop's last barrier already separates the stage reads from the patch writes
  if (!wave_active) return;
  epilogue<TM, TN, WTM, WTN>(g, acc, rowsrc_s, reinterpret_cast<float*>(smem + wave * epi_patch_bytes<WTN>()),
                             bias, rows, n0, wm, wn, lane);
}

template <typename Kern>
void launch_kernel(Kern kern, size_t lds, int bn, int nth, const GemmArgs& g, const Route& rt, hipStream_t s) {
  const int nt_n = (g.n_out + bn - 1) / bn;
  const long long total = (long long)g.n_mtiles * nt_n;
  if (total <= 0) return;
  const int per = (int)((total + kXcds - 1) / kXcds);
  hipLaunchKernelGGL(kern, dim3(per * kXcds), dim3(nth), lds, s, g, rt);
}

template <int BM, int BN, int WM, int WN>
constexpr size_t staged_lds() {
  constexpr size_t stages = (size_t)2 * (BM + BN) * BK * 2, patches = (size_t)WM * WN * epi_patch_bytes<BN / WN>();
  return (stages > patches ? stages : patches) + BM * sizeof(int);
}
template <int BM, int BN, int WM, int WN, int STAGES>
constexpr size_t dma_lds() {
  constexpr size_t stages = (size_t)STAGES * (BM + BN) * 32 * 2, patches = (size_t)WM * WN * epi_patch_bytes<BN / WN>();
  return (stages > patches ? stages : patches) + BM * sizeof(int);
}

template <int BM, int BN, int WM, int WN>
void launch_staged(const GemmArgs& g, const Route& rt, hipStream_t s) {
  launch_kernel(gemm_bf16_kernel<BM, BN, WM, WN>, staged_lds<BM, BN, WM, WN>(), BN, 64 * WM * WN, g, rt, s);
}

template <int BM, int BN, int WM, int WN, int STAGES>
void launch_dma(const GemmArgs& g, const Route& rt, hipStream_t s) {
  launch_kernel(gemm_bf16_dma_kernel<BM, BN, WM, WN, STAGES>, dma_lds<BM, BN, WM, WN, STAGES>(), BN, 64 * WM * WN, g, rt, s);
}

}  // namespace

// the three general-tile kernels launch_gemm_bf16 can pick
void init_gemm_bf16_kernels() {
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_dma_kernel<256, 256, 4, 2, 4>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)dma_lds<256, 256, 4, 2, 4>());
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_kernel<256, 128, 4, 2>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)staged_lds<256, 128, 4, 2>());
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_kernel<256, 64, 8, 1>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)staged_lds<256, 64, 8, 1>());
}

void launch_gemm_bf16(const GemmArgs& g0, const Route& rt, hipStream_t s) {
  GemmArgs g = g0;
  // Few rows per weight matrix (a decode step: at most 32 rows per 128-row tile on average), or a small
  // launch whose 256 x 256 tiles would occupy under half of the compute units: weight streaming by
  // many small items instead.
  const long long tiles256 = (long long)g.n_mtiles_list[0] * ((g.n_out + 255) / 256);
  if (g.k % 64 == 0 && g.n_out % 32 == 0 && rt.tile_m[1] == 128 && g.n_mtiles_list[1] > 0 && g.n_rows > 0 &&
      (g.n_rows <= 32LL * g.n_mtiles_list[1] || (tiles256 < 128 && g.n_rows <= 1024))) {
    g.which_tiles = 1;
    g.n_mtiles = g.n_mtiles_list[1];
    return launch_gemm_bf16_skinny(g, rt, s);
  }
  g.which_tiles = 0;                       // the other kernels work on the list of 256-row m-tiles
  g.n_mtiles = g.n_mtiles_list[0];
  if (g.n_out % 256 == 0 && g.k % 64 == 0 && g.k >= 192) launch_gemm_bf16_p256(g, rt, s);
  else if (g.n_out % 256 == 0) launch_dma<256, 256, 4, 2, 4>(g, rt, s);
  else if (g.n_out % 128 == 0) launch_staged<256, 128, 4, 2>(g, rt, s);
  else launch_staged<256, 64, 8, 1>(g, rt, s);
}

}  // namespace hmi
