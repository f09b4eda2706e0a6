// Grouped bf16 GEMM, 256 x 256 tiles with 64-wide k-stages (the main kernel for wide layers).
//
// Same contract as the other grouped GEMMs (one launch multiplies every tenant segment of a
// mixed batch by that tenant's own weights, Sec. 6.3):
//      C[rows, :] = epi( A[rows, :] * W_g^T + b_g )        for every m-tile of segment g
//
// What bounds this kernel on gfx950 is the number of requests the L2 serves, not the matrix
// cores: an L2 channel answers one request per clock, 128 bytes if the request covers a full
// cache line, 64 if it covers half of one (measured: 33 TB/s against 17-20 TB/s for
// direct-to-LDS copies that hit in L2).  Hence
//   * 256 x 256 tiles: the fewest operand bytes per FLOP that the register file allows
//     (8 wavefronts x 128 accumulator registers);
//   * k-stages of 64 bf16 = 128 bytes per row: eight lanes of a direct-to-LDS load fetch one
//     whole cache line of a row, every request is a full line;
//   * LDS (all 160 KB) is a ring of 2 activation stages and 3 weight stages of 32 KB: the
//     weight stream, which mostly misses L2 (a weight panel is shared by the few m-tiles of
//     one tenant), runs two stages ahead, the activation stream, which mostly hits (a panel
//     is shared by all n-tiles), one stage ahead.  A wavefront issues its activation copies
//     before its weight copies, so that with in-order completion waiting for "all but the
//     newest weight stage" is exactly the condition for the next stage.
//   * Operand roles are swapped (weights are the MFMA's first operand, in a permuted row
//     order): a lane ends up with one row of C and 16 consecutive columns per MFMA tile, so
//     the epilogue stores 32-byte (bf16) or 64-byte (fp32) runs straight from registers and
//     the bias is folded into the accumulator initialisation.
//   * 16-byte chunks are XOR-swizzled so that fragment reads are bank-conflict free for
//     both row orders; workgroup ids are folded so that each XCD owns a contiguous range of
//     tiles (neighbours share panels in that XCD's L2).
#include "hmi_kernels.h"

namespace hmi {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kXcds = 8;
constexpr int BM = 256, BN = 256, BK = 64, NW = 8, NTH = 64 * NW;
constexpr int WTM = 64, WTN = 128, TM = 2, TN = 4;          // wavefront tile (4 x 2 wavefronts), MFMA tiles
constexpr int ROW_BYTES = BK * 2;                            // 128: one cache line per row and stage
constexpr int A_STAGES = 2, W_STAGES = 3;
constexpr int A_STAGE_BYTES = BM * ROW_BYTES, W_STAGE_BYTES = BN * ROW_BYTES;   // 32 KB each
constexpr int W_RING = A_STAGES * A_STAGE_BYTES;             // byte offset of the weight ring
constexpr int LDS_BYTES = W_RING + W_STAGES * W_STAGE_BYTES; // 163840 = all of it
constexpr int A_LD = BM / 8 / NW, B_LD = BN / 8 / NW;        // 1 KB (8 rows x 128 B) loads per wavefront and stage

__device__ __forceinline__ float bf2f(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 p = {(__bf16)lo, (__bf16)hi};                       // round to nearest even
  return __builtin_bit_cast(uint32_t, p);
}

// GELU(x) = x Phi(x) = max(x, 0) - a Phi(-a) with a = |x|.  a Phi(-a) is a smooth bump (at
// most 0.17, below 1.3e-4 beyond a = 4): Phi(-a) is replaced by a degree-6 polynomial in
// u = a/2 - 1 on [0, 4], fitted so that |a (Q(u) - Phi(-a))| <= 2e-4 (a tenth of the bf16
// resolution of the result at that magnitude); GELU(0) = 0 exactly.  Ten vector-ALU
// operations, no transcendental.
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

#define HMI_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

struct Tile { int n0, row0, rows; size_t slot_base; };

#ifdef HMI_EXP_CLOCK
__device__ unsigned long long hmi_dbg_clk[4];
__device__ unsigned long long hmi_dbg_wg[4096 * 4];
#endif

__device__ __forceinline__ bool locate(const GemmArgs& g, const Route& rt, Tile& tc) {
  const int nt_n = g.n_out / BN;
  const int total = g.n_mtiles * nt_n;
  const int per = (total + kXcds - 1) / kXcds;
  const int local = blockIdx.x / kXcds;
  const int w = (blockIdx.x % kXcds) * per + local;
  if (local >= per || w >= total) return false;
  const int mt = w / nt_n;
  tc.n0 = (w % nt_n) * BN;
  const int seg = rt.tile_seg[g.which_tiles][mt];
  tc.row0 = rt.tile_row0[g.which_tiles][mt];
  tc.rows = min(BM, rt.seg_tok_off[seg + 1] - tc.row0);
  tc.slot_base = (size_t)rt.seg_slot[seg] * g.slot_stride;
  return true;
}

template <int EPI, bool OUT_F32, bool RESID_F32, bool HAS_C2>
__global__ __launch_bounds__(NTH) __attribute__((amdgpu_waves_per_eu(2, 2)))
void gemm_bf16_p256_kernel(GemmArgs g, Route rt) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  Tile tc;
  if (!locate(g, rt, tc)) return;
#ifdef HMI_EXP_CLOCK
  const unsigned long long dbg_c0 = clock64(), dbg_w0 = wall_clock64();
#endif
  const int rows = tc.rows, n0 = tc.n0;
  const char* Wb = g.pool + tc.slot_base + g.w_off;
  const uint16_t* bias = reinterpret_cast<const uint16_t*>(g.pool + tc.slot_base + g.b_off);
  const char* Ab = reinterpret_cast<const char*>(g.A);

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const int K = g.k;
  const int KT = K / BK;

  // ---- global sources of this lane's direct-to-LDS copies (byte offsets at k = 0): lane l
  // fills LDS slot (row l/8, position l%8) of an 8-row block with global chunk
  // position ^ swizzle(row); the eight lanes of a row cover its whole 128-byte line.
  uint32_t a_off[A_LD], b_off[B_LD];
#pragma unroll
  for (int j = 0; j < A_LD; ++j) {
    const int row = (wave * A_LD + j) * 8 + (lane >> 3);
    const int src = rt.row_src[tc.row0 + min(row, rows - 1)];
    a_off[j] = (uint32_t)src * (uint32_t)(g.lda * 2) + (((lane & 7) ^ swz_a(row)) << 4);
  }
#pragma unroll
  for (int j = 0; j < B_LD; ++j) {
    const int row = (wave * B_LD + j) * 8 + (lane >> 3);
    b_off[j] = (uint32_t)(n0 + row) * (uint32_t)(K * 2) + (((lane & 7) ^ swz_w(row)) << 4);
  }

  // Past the end both issue macros re-read the last stage (in bounds) into a ring slot that
  // nobody reads any more, which keeps the outstanding-copy count uniform.
#define HMI_ISSUE_A(S_IDX)                                                                        \
  {                                                                                               \
    const int s_ = (S_IDX);                                                                       \
    const int kb_ = min(s_, KT - 1) * ROW_BYTES;                                                  \
    unsigned char* base_ = smem + (s_ % A_STAGES) * A_STAGE_BYTES;                                \
    _Pragma("unroll") for (int j = 0; j < A_LD; ++j)                                              \
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(Ab + kb_ + a_off[j]),                        \
                                         (lds_ptr_t)(base_ + (wave * A_LD + j) * 1024), 16, 0, 0);\
  }
#define HMI_ISSUE_W(S_IDX)                                                                        \
  {                                                                                               \
    const int s_ = (S_IDX);                                                                       \
    const int kb_ = min(s_, KT - 1) * ROW_BYTES;                                                  \
    unsigned char* base_ = smem + W_RING + (s_ % W_STAGES) * W_STAGE_BYTES;                       \
    _Pragma("unroll") for (int j = 0; j < B_LD; ++j)                                              \
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(Wb + kb_ + b_off[j]),                        \
                                         (lds_ptr_t)(base_ + (wave * B_LD + j) * 1024), 16, 0, 0);\
  }

  // ---- accumulators start at the bias: lane half h of MFMA tile j holds columns
  // n0 + wn*128 + j*32 + 16 h + (0..15), the same for both m-tiles.
  u32x4 bias_lo[TN], bias_hi[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col0 = n0 + wn * WTN + j * 32 + 16 * lh;
    bias_lo[j] = *reinterpret_cast<const u32x4*>(bias + col0);
    bias_hi[j] = *reinterpret_cast<const u32x4*>(bias + col0 + 8);
  }
  HMI_ISSUE_A(0)
  HMI_ISSUE_W(0)
  HMI_ISSUE_W(1)
  f32x16 acc[TM][TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const u32x4 b0 = bias_lo[j], b1 = bias_hi[j];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      acc[0][j][2 * q] = bf2f(b0[q] & 0xffffu);      acc[0][j][2 * q + 1] = bf2f(b0[q] >> 16);
      acc[0][j][8 + 2 * q] = bf2f(b1[q] & 0xffffu);  acc[0][j][8 + 2 * q + 1] = bf2f(b1[q] >> 16);
    }
#pragma unroll
    for (int i = 1; i < TM; ++i) acc[i][j] = acc[0][j];
  }

  // ---- fragment read offsets inside a stage for the four k-steps of a stage
  int fx_off[4], fw_off[4];
  {
    const int rx = wm * WTM + l32;                       // + 32 i: swizzle unchanged
    const int rw = wn * WTN + perm_w(l32);               // + 32 j: swizzle unchanged
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      fx_off[ks] = rx * ROW_BYTES + (((ks * 2 + lh) ^ swz_a(rx)) << 4);
      fw_off[ks] = W_RING + rw * ROW_BYTES + (((ks * 2 + lh) ^ swz_w(rw)) << 4);
    }
  }

  const bool wave_active = wm * WTM < rows;

  for (int s = 0; s < KT; ++s) {
    HMI_WAIT_VMCNT(B_LD);                                // all but the newest weight stage have landed
    __builtin_amdgcn_s_barrier();                        // ... everybody's, and stage s-1 is no longer read
    __builtin_amdgcn_sched_barrier(0);
    HMI_ISSUE_A(s + 1)
    HMI_ISSUE_W(s + 2)
    if (wave_active) {
      const unsigned char* xa = smem + (s % A_STAGES) * A_STAGE_BYTES;
      const unsigned char* wa = smem + (s % W_STAGES) * W_STAGE_BYTES;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        bf16x8 fx[TM], fw[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fx[i] = *reinterpret_cast<const bf16x8*>(xa + fx_off[ks] + i * 32 * ROW_BYTES);
#pragma unroll
        for (int j = 0; j < TN; ++j) fw[j] = *reinterpret_cast<const bf16x8*>(wa + fw_off[ks] + j * 32 * ROW_BYTES);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#ifndef HMI_EXP_NO_MFMA
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[j], fx[i], acc[i][j], 0, 0, 0);
#else
            { acc[i][j][0] += (float)fw[j][0] + (float)fx[i][0]; }
#endif
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
#undef HMI_ISSUE_A
#undef HMI_ISSUE_W
  HMI_WAIT_VMCNT(0);   // the tail copies (re-reads of the last stage) must not outlive the workgroup
#ifdef HMI_EXP_CLOCK
  if (threadIdx.x == 0 && blockIdx.x < 4096) {
    unsigned hwid, xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hwid));
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    hmi_dbg_wg[blockIdx.x * 4 + 0] = dbg_w0; hmi_dbg_wg[blockIdx.x * 4 + 1] = wall_clock64();
    hmi_dbg_wg[blockIdx.x * 4 + 2] = ((unsigned long long)xcc << 32) | hwid; hmi_dbg_wg[blockIdx.x * 4 + 3] = (unsigned long long)tc.rows;
  }
  if (threadIdx.x == 0) {
    atomicAdd(&hmi_dbg_clk[0], clock64() - dbg_c0); atomicAdd(&hmi_dbg_clk[1], wall_clock64() - dbg_w0); atomicAdd(&hmi_dbg_clk[2], 1ull);
  }
#endif
  if (!wave_active) return;
#ifdef HMI_EXP_NO_EPI
  { float sacc = 0.f;
    for (int i = 0; i < TM; ++i) for (int j = 0; j < TN; ++j) for (int r = 0; r < 16; ++r) sacc += acc[i][j][r];
    if (sacc == 12345.678f) reinterpret_cast<float*>(g.C)[0] = sacc;
    return; }
#endif

  // ---- epilogue straight from the accumulators: lane = row, 16 consecutive columns per tile
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = wm * WTM + i * 32 + l32;
    if (m >= rows) continue;
    const size_t orow = (size_t)rt.row_src[tc.row0 + m];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col0 = n0 + wn * WTN + j * 32 + 16 * lh;
      float v[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        v[r] = acc[i][j][r];
        if (EPI == EPI_BIAS_GELU) v[r] = gelu_poly(v[r]);
        else if (EPI == EPI_BIAS_RELU) v[r] = fmaxf(v[r], 0.0f);
      }
      if (EPI == EPI_BIAS_RESID) {
        if (RESID_F32) {
          const f32x4* rp = reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(g.resid) + orow * g.ldr + col0);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const f32x4 rv = rp[q];
            v[4 * q] += rv[0]; v[4 * q + 1] += rv[1]; v[4 * q + 2] += rv[2]; v[4 * q + 3] += rv[3];
          }
        } else {
          const u32x4* rp = reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(g.resid) + orow * g.ldr + col0);
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const u32x4 rv = rp[q];
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[8 * q + 2 * e] += bf2f(rv[e] & 0xffffu); v[8 * q + 2 * e + 1] += bf2f(rv[e] >> 16); }
          }
        }
      }
      u32x4 h0, h1;
      if (!OUT_F32 || HAS_C2) {
#pragma unroll
        for (int e = 0; e < 4; ++e) { h0[e] = pack_bf16(v[2 * e], v[2 * e + 1]); h1[e] = pack_bf16(v[8 + 2 * e], v[8 + 2 * e + 1]); }
      }
      if (OUT_F32) {
        f32x4* cp = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.C) + orow * g.ldc + col0);
#pragma unroll
        for (int q = 0; q < 4; ++q) { f32x4 o = {v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]}; cp[q] = o; }
      } else {
        u32x4* cp = reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(g.C) + orow * g.ldc + col0);
        cp[0] = h0; cp[1] = h1;
      }
      if (HAS_C2) {
        u32x4* cp = reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(g.C2) + orow * g.ldc + col0);
        cp[0] = h0; cp[1] = h1;
      }
    }
  }
}

template <int EPI, bool OUT_F32, bool RESID_F32, bool HAS_C2>
void launch_one(const GemmArgs& g, const Route& rt, hipStream_t s) {
  static bool attr_set = false;
  auto kern = gemm_bf16_p256_kernel<EPI, OUT_F32, RESID_F32, HAS_C2>;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    attr_set = true;
  }
  const int nt_n = g.n_out / BN;
  const long long total = (long long)g.n_mtiles * nt_n;
  if (total <= 0) return;
  const int per = (int)((total + kXcds - 1) / kXcds);
  hipLaunchKernelGGL(kern, dim3(per * kXcds), dim3(NTH), LDS_BYTES, s, g, rt);
}

}  // namespace

#ifdef HMI_EXP_CLOCK
void dbg_clock_read(unsigned long long* out) { (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(hmi_dbg_clk), 32); }
void dbg_wg_read(unsigned long long* out) { (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(hmi_dbg_wg), 4096 * 32); }
#endif

// Preconditions (checked by the caller): n_out % 256 == 0, k % 64 == 0, k >= 64,
// which_tiles names a list of 256-row m-tiles, all operands 16-byte aligned,
// byte offsets of A rows and of W rows inside a slot below 4 GB.
void launch_gemm_bf16_p256(const GemmArgs& g, const Route& rt, hipStream_t s) {
  const bool c2 = g.C2 != nullptr;
  switch (g.epi) {
    case EPI_BIAS:
      return c2 ? launch_one<EPI_BIAS, false, false, true>(g, rt, s) : launch_one<EPI_BIAS, false, false, false>(g, rt, s);
    case EPI_BIAS_GELU:
      return launch_one<EPI_BIAS_GELU, false, false, false>(g, rt, s);
    case EPI_BIAS_RELU:
      return launch_one<EPI_BIAS_RELU, false, false, false>(g, rt, s);
    default:
      if (g.out_f32) {
        if (g.resid_f32) return c2 ? launch_one<EPI_BIAS_RESID, true, true, true>(g, rt, s) : launch_one<EPI_BIAS_RESID, true, true, false>(g, rt, s);
        return c2 ? launch_one<EPI_BIAS_RESID, true, false, true>(g, rt, s) : launch_one<EPI_BIAS_RESID, true, false, false>(g, rt, s);
      }
      if (g.resid_f32) return launch_one<EPI_BIAS_RESID, false, true, false>(g, rt, s);
      return launch_one<EPI_BIAS_RESID, false, false, false>(g, rt, s);
  }
}

}  // namespace hmi
