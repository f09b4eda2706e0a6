// The paper's bottleneck adapter over a mixed-tenant batch (Sec. 3.2.2, batched as in
// Sec. 6.3), one kernel:  Y = X + Up_t(ReLU(Down_t(X))),  Down_t: d -> 64,  Up_t: 64 -> d,
// bf16 storage, fp32 accumulation, Y rounded once.
//
// With a 64-wide bottleneck the block moves 4 d bytes per token for 256 d flops per token:
// far below the machine balance, so the kernel is organised around the HBM stream and not
// around the MFMA pipes.  A workgroup (8 wavefronts, one per compute unit) walks a
// contiguous range of 32-row units of the tenant-sorted batch.  A unit's rows are copied
// straight into LDS (full 128-byte lines, rows gathered through row_src), both
// projections run out of LDS and registers, the result replaces the rows in LDS, and the
// same rows stream back out with 16-byte stores: X is read once and Y written once.
// Two row buffers alternate, so the copies of the unit after next run under this unit's
// arithmetic; wavefronts 0-3 issue the copies and wavefronts 4-7 the stores, which keeps
// each wavefront's memory counter to one kind of access (loads return in order among
// loads only).
//
// The tenant's two matrices live in registers for as long as the units stay in one
// segment: at load time they are laid out in MFMA operand order (pack_adapter_operand
// below), so a reload is a handful of 1 KB coalesced reads.
//
//   Down:  wavefront (cb, kq) multiplies the unit by column block cb of Down over its
//          quarter kq of d (k-steps 2 kq and 2 kq + 1 of every eight); the four partial sums per element meet in LDS (fixed order of
//          addition), where bias and ReLU are applied and the 32 x 64 result is rounded to
//          bf16 once, as the two-kernel path does between its GEMMs.
//   Up:    wavefront w owns output columns [w d/8, (w+1) d/8); it adds bias and the
//          unit's own rows from LDS and writes the rounded sum back in place.
#include "hmi_kernels.h"

namespace hmi {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

constexpr int RT = 32;            // rows of a unit
constexpr int RANK = 64;          // bottleneck width
constexpr int NTH = 512;
constexpr int MAX_UNITS = 64;     // units one workgroup may be handed
constexpr int PART_BYTES = 4 * RT * RANK * 4;   // four partial sums of the 32 x 64 bottleneck, fp32
constexpr int MID_BYTES = RT * RANK * 2;
constexpr int RS_BYTES = MAX_UNITS * RT * 4;
constexpr int DESC_BYTES = (MAX_UNITS * 4 + 4) * 4;

#define HMI_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

__device__ __forceinline__ float bf2f(uint32_t u16) { return __uint_as_float(u16 << 16); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

// A tenant's matrices.  In a decode step a tenant has a row or two: its 0.2 MB are read by one workgroup, once, and only push
// the shared layers' weights out of the L2s (with the hint a step through six shared layers is 3 % shorter); over a full batch
// the workgroups that hold the tenant's other rows read them again, from L2, and there the plain load is the faster one.
template <bool ONCE>
__device__ __forceinline__ bf16x8 load_w(const bf16x8* p) {
  if (ONCE) return __builtin_nontemporal_load(p);
  return *p;
}

template <int NV>
struct Shape {
  static constexpr int CH = NV * 32;          // 16-byte chunks of a row (d = 256 NV)
  static constexpr int ROWB = CH * 16;
  static constexpr int BUF = RT * ROWB;
  static constexpr int KS = NV * 16;          // 16-wide k-steps over d
  static constexpr int KSW = KS / 4;          // ... per wavefront of the down-projection
  static constexpr int NJ = RT * CH / 256;    // copies (stores) per lane and unit
  static constexpr int OFF_PART = 2 * BUF;
  static constexpr int OFF_MID = OFF_PART + PART_BYTES;
  static constexpr int OFF_RS = OFF_MID + MID_BYTES;
  static constexpr int OFF_DESC = OFF_RS + RS_BYTES;
  static constexpr int LDS = OFF_DESC + DESC_BYTES;
};

// LDS layouts (all XOR swizzles act on 16-byte chunk indices, so that the 16 lanes that
// the LDS serves together hit 16 different chunks of its 256-byte bank line):
//   row buffer   row r, position p holds the row's chunk p ^ (r & 15)
//   partial sum  [kq][row r][16 chunks of 4 fp32], chunk q at position q ^ (r & 15)
//   bottleneck   row r is 128 bytes (64 bf16), chunk c at position c ^ ((r >> 1) & 7)
// ONCE: the tenants' matrices are loaded with the non-temporal hint (load_w above); STREAM: so are the result's stores.
// Both are compile-time: a run-time choice between a hinted and a plain access to one address is merged into the plain one.
template <int NV, bool ONCE, bool STREAM>
__global__ __launch_bounds__(NTH) __attribute__((amdgpu_waves_per_eu(2, 2)))
void adapter_bf16_kernel(AdapterArgs a, Route rt) {
  using S = Shape<NV>;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 31, h = lane >> 5;     // MFMA: token row of the unit, k-half
  int* desc = reinterpret_cast<int*>(smem + S::OFF_DESC);
  int* rs = reinterpret_cast<int*>(smem + S::OFF_RS);

  // ---- which units are mine, which of them hold rows, and where those rows live
  const int U = a.n_tiles128 * 4;
  const int u_begin = (int)((long long)blockIdx.x * U / gridDim.x);
  const int u_end = (int)((long long)(blockIdx.x + 1) * U / gridDim.x);
  if (wave == 0) {
    const int u = u_begin + lane;
    int row0 = 0, rows = 0, slot = 0;
    if (u < u_end) {
      const int t = u >> 2;
      const int seg = rt.tile_seg[a.which_tiles][t];
      row0 = rt.tile_row0[a.which_tiles][t] + (u & 3) * RT;
      rows = min(RT, rt.seg_tok_off[seg + 1] - row0);
      slot = rt.seg_slot[seg];
    }
    const unsigned long long mask = __ballot(rows > 0);
    if (rows > 0) {
      const int pos = __popcll(mask & ((1ull << lane) - 1ull));
      desc[pos * 4 + 0] = row0; desc[pos * 4 + 1] = rows; desc[pos * 4 + 2] = slot;
    }
    if (lane == 0) desc[MAX_UNITS * 4] = __popcll(mask);
  }
  __syncthreads();
  const int m = desc[MAX_UNITS * 4];
  if (m == 0) return;
  for (int idx = tid; idx < m * RT; idx += NTH) {
    const int u = idx >> 5, r = idx & 31;
    rs[idx] = rt.row_src[desc[u * 4] + min(r, desc[u * 4 + 1] - 1)];   // surplus rows of a short unit repeat its last row
  }

  const int cb = wave & 1, kq = wave >> 1;    // down-projection role
  bf16x8 wd[S::KSW], wu[NV][4];
  u32x4 bu[NV][2];   // up-projection bias of my columns, packed bf16 pairs
  f32x4 bd4;

  // copies unit ui into row buffer b (wavefronts 0-3; a lane moves NJ chunks of 16 bytes)
  const char* X = reinterpret_cast<const char*>(a.X);
  char* Y = reinterpret_cast<char*>(a.Y);
  // A lane's NJ = 4 NV chunks of a unit: chunk jj * 256 + t8 with t8 = tid mod 256.  256 NV
  // chunks are exactly 8 rows, so chunk (NV g + r3) * 256 + t8 lies in row 8 g + ro[r3] at a
  // row position that does not depend on g; sw[r3] is that position swizzled for g even.
  const int t8 = tid & 255;
  int ro[NV], sw[NV];
#pragma unroll
  for (int r3 = 0; r3 < NV; ++r3) {
    const int c = r3 * 256 + t8;
    ro[r3] = c / S::CH;
    sw[r3] = ((c % S::CH) ^ ro[r3]) << 4;
  }
#define HMI_ISSUE_COPIES(UI, B)                                                                    \
  {                                                                                                \
    _Pragma("unroll") for (int g_ = 0; g_ < 4; ++g_)                                               \
      _Pragma("unroll") for (int r3 = 0; r3 < NV; ++r3) {                                          \
        const char* src_ = X + (size_t)rs[(UI) * RT + 8 * g_ + ro[r3]] * S::ROWB + (sw[r3] ^ ((g_ & 1) << 7)); \
        lds_ptr_t dst_ = (lds_ptr_t)(smem + (B) * S::BUF + ((g_ * NV + r3) * 256 + wave * 64) * 16); \
        __builtin_amdgcn_global_load_lds((glb_ptr_t)src_, dst_, 16, 0, 0);                         \
      }                                                                                            \
  }

#define HMI_LOAD_WD(SLOT)                                                                          \
  {                                                                                                \
    const bf16x8* pwd = reinterpret_cast<const bf16x8*>(a.pool + (size_t)(SLOT) * a.slot_stride + a.wd_off) + \
                        ((cb * S::KS + 2 * kq) * 64 + lane);                                       \
    _Pragma("unroll") for (int s = 0; s < S::KSW; ++s)                                             \
      wd[s] = load_w<ONCE>(pwd + ((s >> 1) * 8 + (s & 1)) * 64);   /* k-step 8 (s / 2) + 2 kq + s % 2 */ \
  }
#define HMI_LOAD_BD(SLOT)                                                                          \
  {                                                                                                \
    const u32x2 d2 = *reinterpret_cast<const u32x2*>(a.pool + (size_t)(SLOT) * a.slot_stride + a.bd_off + (tid & 15) * 8); \
    bd4 = f32x4{bf2f(d2[0] & 0xFFFFu), bf2f(d2[0] >> 16), bf2f(d2[1] & 0xFFFFu), bf2f(d2[1] >> 16)}; \
  }
#define HMI_LOAD_WU(SLOT)                                                                          \
  {                                                                                                \
    const char* base = a.pool + (size_t)(SLOT) * a.slot_stride;                                    \
    const bf16x8* pwu = reinterpret_cast<const bf16x8*>(base + a.wu_off) + (wave * NV * 4 * 64 + lane); \
    _Pragma("unroll") for (int c = 0; c < NV; ++c)                                                 \
      _Pragma("unroll") for (int s = 0; s < 4; ++s) wu[c][s] = load_w<ONCE>(pwu + (c * 4 + s) * 64); \
    _Pragma("unroll") for (int c = 0; c < NV; ++c) {                                               \
      const u32x4* pb = reinterpret_cast<const u32x4*>(base + a.bu_off + ((wave * NV + c) * 32 + h * 16) * 2); \
      bu[c][0] = pb[0]; bu[c][1] = pb[1];                                                          \
    }                                                                                              \
  }

  int cur_slot = desc[2];
  HMI_LOAD_WD(cur_slot) HMI_LOAD_BD(cur_slot) HMI_LOAD_WU(cur_slot)
  __syncthreads();   // rs complete
  if (wave < 4) {
    HMI_ISSUE_COPIES(0, 0)
    if (m > 1) HMI_ISSUE_COPIES(1, 1)
  }

  for (int i = 0; i < m; ++i) {
    const int b = i & 1;
    unsigned char* buf = smem + b * S::BUF;
    const int rows = desc[i * 4 + 1];
    // the tenant of the next unit, if it is another one: its matrices replace this unit's as
    // soon as each has been used for the last time, so that the reads run under the rest of the unit
    const int next_slot = i + 1 < m ? desc[(i + 1) * 4 + 2] : cur_slot;
    const bool reload = next_slot != cur_slot;   // same for the whole workgroup
    if (i == 0) {   // the first unit's rows must have landed (later units: see the end of the loop)
      if (wave < 4) { if (m > 1) { HMI_WAIT_VMCNT(S::NJ); } else { HMI_WAIT_VMCNT(0); } }
      __syncthreads();
    }

    // ---- Down: partial[kq] = X[32, my quarter of d] * Down[cb block, same quarter]^T
    {
      // my k-steps are 8 a + 2 kq + e (a = 0 .. KS/8 - 1, e = 0, 1): the row chunks 16 a + 4 kq + 2 e + h,
      // whose swizzled position inside the 256-byte group a is the same for every a
      f32x16 acc = {};
      const unsigned char* xr = buf + j * S::ROWB;
      const unsigned char* x0 = xr + (((4 * kq + h) ^ (j & 15)) << 4);
      const unsigned char* x1 = xr + (((4 * kq + 2 + h) ^ (j & 15)) << 4);
#pragma unroll
      for (int s = 0; s < S::KSW; ++s) {
        const bf16x8 xf = *reinterpret_cast<const bf16x8*>(((s & 1) ? x1 : x0) + (s >> 1) * 256);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wd[s], xf, acc, 0, 0, 0);
      }
      unsigned char* pr = smem + S::OFF_PART + kq * (RT * RANK * 4) + j * (RANK * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int q = cb * 8 + h * 4 + e;
        *reinterpret_cast<f32x4*>(pr + ((q ^ (j & 15)) << 4)) = f32x4{acc[4 * e], acc[4 * e + 1], acc[4 * e + 2], acc[4 * e + 3]};
      }
    }
    if (reload) HMI_LOAD_WD(next_slot)
    __syncthreads();
    // ---- bottleneck: sum of the four quarters + bias, ReLU, one rounding to bf16
    {
      const int row = tid >> 4, q = tid & 15;
      const unsigned char* pr = smem + S::OFF_PART + row * (RANK * 4) + ((q ^ (row & 15)) << 4);
      f32x4 v = *reinterpret_cast<const f32x4*>(pr);
#pragma unroll
      for (int k = 1; k < 4; ++k) v += *reinterpret_cast<const f32x4*>(pr + k * (RT * RANK * 4));
      v += bd4;
      u32x2 o;
      o[0] = pack_bf16(fmaxf(v[0], 0.0f), fmaxf(v[1], 0.0f));
      o[1] = pack_bf16(fmaxf(v[2], 0.0f), fmaxf(v[3], 0.0f));
      *reinterpret_cast<u32x2*>(smem + S::OFF_MID + row * 128 + (((q >> 1) ^ ((row >> 1) & 7)) << 4) + (q & 1) * 8) = o;
    }
    if (reload) HMI_LOAD_BD(next_slot)
    __syncthreads();
    // ---- Up: my d/8 output columns, added to the unit's rows in place
    {
      bf16x8 mf[4];
      const unsigned char* mr = smem + S::OFF_MID + j * 128;
#pragma unroll
      for (int s = 0; s < 4; ++s) mf[s] = *reinterpret_cast<const bf16x8*>(mr + (((2 * s + h) ^ ((j >> 1) & 7)) << 4));
      unsigned char* xr = buf + j * S::ROWB;
#pragma unroll
      for (int c = 0; c < NV; ++c) {
        f32x16 acc;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[2 * e] = bf2f(bu[c][0][e] & 0xFFFFu); acc[2 * e + 1] = bf2f(bu[c][0][e] >> 16);
          acc[8 + 2 * e] = bf2f(bu[c][1][e] & 0xFFFFu); acc[8 + 2 * e + 1] = bf2f(bu[c][1][e] >> 16);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wu[c][s], mf[s], acc, 0, 0, 0);
        const int p0 = (wave * NV + c) * 4 + 2 * h;
        u32x4* x0 = reinterpret_cast<u32x4*>(xr + ((p0 ^ (j & 15)) << 4));
        u32x4* x1 = reinterpret_cast<u32x4*>(xr + (((p0 + 1) ^ (j & 15)) << 4));
        const u32x4 v0 = *x0, v1 = *x1;
        u32x4 o0, o1;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o0[e] = pack_bf16(acc[2 * e] + bf2f(v0[e] & 0xFFFFu), acc[2 * e + 1] + bf2f(v0[e] >> 16));
          o1[e] = pack_bf16(acc[8 + 2 * e] + bf2f(v1[e] & 0xFFFFu), acc[8 + 2 * e + 1] + bf2f(v1[e] >> 16));
        }
        *x0 = o0; *x1 = o1;
      }
    }
    if (reload) HMI_LOAD_WU(next_slot)
    cur_slot = next_slot;
    __syncthreads();
    // ---- wavefronts 4-7 stream the finished rows out; wavefronts 0-3 make sure the next
    //      unit's rows have landed.  After the barrier the buffer is free for unit i + 2.
    if (wave >= 4) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x4 v[NV];
        int orow[NV];
#pragma unroll
        for (int r3 = 0; r3 < NV; ++r3) {
          v[r3] = *reinterpret_cast<const u32x4*>(buf + ((g * NV + r3) * 256 + t8) * 16);
          orow[r3] = rs[i * RT + 8 * g + ro[r3]];
        }
#pragma unroll
        for (int r3 = 0; r3 < NV; ++r3)
          if (8 * g + ro[r3] < rows) {
            u32x4* dst = reinterpret_cast<u32x4*>(Y + (size_t)orow[r3] * S::ROWB + (sw[r3] ^ ((g & 1) << 7)));
            // a result that goes to the caller leaves without taking lines of L2 (the adapter-only block: 4.7 -> 5.0 TB/s);
            // inside a shared layer the next kernel reads it at once, and there the plain store is the faster one
            if (STREAM) __builtin_nontemporal_store(v[r3], dst); else *dst = v[r3];
          }
      }
    } else if (i + 1 < m) {
      HMI_WAIT_VMCNT(0);
    }
    __syncthreads();
    if (wave < 4 && i + 2 < m) HMI_ISSUE_COPIES(i + 2, b)
  }
#undef HMI_ISSUE_COPIES
#undef HMI_LOAD_WD
#undef HMI_LOAD_BD
#undef HMI_LOAD_WU
}

template <int NV>
void launch_nv(const AdapterArgs& a, const Route& rt, hipStream_t s) {
  using S = Shape<NV>;
  auto kern = a.stream_out ? adapter_bf16_kernel<NV, false, true>
                           : a.weights_once ? adapter_bf16_kernel<NV, true, false> : adapter_bf16_kernel<NV, false, false>;
  const int n_cu = rt.n_cu >= 1 ? rt.n_cu : 256;
  const long long U = (long long)a.n_tiles128 * 4;
  if (U <= 0) return;
  long long grid = U < n_cu ? U : n_cu;                               // one workgroup per compute unit ...
  const long long need = (U + MAX_UNITS - 1) / MAX_UNITS;            // ... unless that hands a workgroup
  if (grid < need) grid = need;                                       //     more units than it can list
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NTH), S::LDS, s, a, rt);
}

template <int NV>
void allow_lds() {
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(adapter_bf16_kernel<NV, false, false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            Shape<NV>::LDS);
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(adapter_bf16_kernel<NV, true, false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            Shape<NV>::LDS);
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(adapter_bf16_kernel<NV, false, true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            Shape<NV>::LDS);
}

}  // namespace

void init_adapter_bf16_kernels() { allow_lds<1>(); allow_lds<2>(); allow_lds<3>(); }

// Operand order: 1 KB blocks, one per (32-row block, 16-wide k-step), k-steps innermost.
// Lane l of a block holds the 8 elements [16 s + 8 (l / 32), +8) of the block's row
// perm(l % 32), where perm places the rows so that output register r of lane half hh of
// the 32x32x16 MFMA is the block's row 16 hh + r.
void pack_adapter_operand(void* dst, const void* src, int rows, int cols) {
  uint16_t* o = static_cast<uint16_t*>(dst);
  const uint16_t* in = static_cast<const uint16_t*>(src);
  const int ks = cols / 16;
  for (int rb = 0; rb < rows / 32; ++rb)
    for (int s = 0; s < ks; ++s)
      for (int l = 0; l < 64; ++l) {
        const int i = l & 31;
        const int row = rb * 32 + ((i >> 2) & 1) * 16 + (i >> 3) * 4 + (i & 3);
        const uint16_t* from = in + (size_t)row * cols + s * 16 + 8 * (l >> 5);
        uint16_t* to = o + (((size_t)rb * ks + s) * 64 + l) * 8;
        for (int e = 0; e < 8; ++e) to[e] = from[e];
      }
}

bool adapter_bf16_supported(int d, int rank) { return rank == RANK && d % 256 == 0 && d >= 256 && d <= 768; }

// Preconditions (checked by the caller): adapter_bf16_supported(d, rank); which_tiles names
// the list of 128-row m-tiles and n_tiles128 its length; both matrices of every slot in
// the batch are in MFMA operand order; X and Y are distinct, 16-byte aligned [N, d] arrays.
void launch_adapter_bf16(const AdapterArgs& a, const Route& rt, hipStream_t s) {
  switch (a.d / 256) {
    case 1: return launch_nv<1>(a, rt, s);
    case 2: return launch_nv<2>(a, rt, s);
    default: return launch_nv<3>(a, rt, s);
  }
}

}  // namespace hmi
