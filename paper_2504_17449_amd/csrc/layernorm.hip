// Row LayerNorm with per-tenant gain and shift: y = (x - mean) / sqrt(var + eps) * g_t + b_t,
// biased variance, statistics in fp32.  One wavefront per row; the row's tenant slot is
// found by a binary search of the row's sorted position in the segment token offsets.
// Used after the residual adds of the per-tenant blocks (post-LN) or before the
// sub-layers (pre-LN); the paper leaves these to BERT / GPT's layer definitions.
// An optional second input is added first (residual stream + adapted attention output).
#include "hmi_kernels.h"

namespace hmi {
namespace {

__device__ __forceinline__ float bf2f(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

constexpr int kMaxPerLane = 32;  // d <= 2048

template <bool BF16>
__global__ __launch_bounds__(256) void layernorm_kernel(LnArgs a, Route rt) {
  const int lane = threadIdx.x & 63;
  const int srow = blockIdx.x * 4 + (threadIdx.x >> 6);  // sorted row
  if (srow >= a.n_rows) return;
  // segment of this sorted row: last g with seg_tok_off[g] <= srow
  int lo = 0, hi = rt.n_segments[0];
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (rt.seg_tok_off[mid] <= srow) lo = mid; else hi = mid;
  }
  const size_t slot_base = (size_t)rt.seg_slot[lo] * a.slot_stride;
  const size_t row = (size_t)rt.row_src[srow];
  const int d = a.d, per = (d + 63) >> 6;   // columns lane, lane + 64, ... below d

  float v[kMaxPerLane];
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < kMaxPerLane; ++i) {
    v[i] = 0.0f;
    if (i < per && lane + 64 * i < d) {
      const size_t idx = row * d + lane + 64 * i;
      if (a.in_f32) v[i] = reinterpret_cast<const float*>(a.in)[idx];
      else v[i] = BF16 ? bf2f(reinterpret_cast<const uint16_t*>(a.in)[idx])
                       : reinterpret_cast<const float*>(a.in)[idx];
      if (a.in2) v[i] += BF16 ? bf2f(reinterpret_cast<const uint16_t*>(a.in2)[idx])
                              : reinterpret_cast<const float*>(a.in2)[idx];
      if (a.sum_out) a.sum_out[idx] = v[i];
      s += v[i];
    }
  }
  const float mean = wave_sum(s) / (float)d;
  float q = 0.0f;
#pragma unroll
  for (int i = 0; i < kMaxPerLane; ++i)
    if (i < per && lane + 64 * i < d) { const float c = v[i] - mean; q += c * c; }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + a.eps);

#pragma unroll
  for (int i = 0; i < kMaxPerLane; ++i) {
    if (i < per && lane + 64 * i < d) {
      const int col = lane + 64 * i;
      float gg, bb;
      if (BF16) {
        gg = bf2f(reinterpret_cast<const uint16_t*>(a.pool + slot_base + a.g_off)[col]);
        bb = bf2f(reinterpret_cast<const uint16_t*>(a.pool + slot_base + a.b_off)[col]);
      } else {
        gg = reinterpret_cast<const float*>(a.pool + slot_base + a.g_off)[col];
        bb = reinterpret_cast<const float*>(a.pool + slot_base + a.b_off)[col];
      }
      const float y = (v[i] - mean) * rstd * gg + bb;
      const size_t idx = row * d + col;
      if (a.out_f32) a.out_f32[idx] = y;
      if (a.out_st) {
        if (BF16) reinterpret_cast<uint16_t*>(a.out_st)[idx] = f2bf(y);
        else reinterpret_cast<float*>(a.out_st)[idx] = y;
      }
    }
  }
}


typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 load4(const void* p, size_t idx, bool f32) {
  if (f32) return *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(p) + idx);
  const u16x4 h = *reinterpret_cast<const u16x4*>(reinterpret_cast<const uint16_t*>(p) + idx);
  f32x4 v = {bf2f(h[0]), bf2f(h[1]), bf2f(h[2]), bf2f(h[3])};
  return v;
}

// Vector path for d % 256 == 0: a lane owns d/256 pieces of 4 consecutive columns
// (16-byte fp32 / 8-byte bf16 accesses, a wavefront covers 1 KB / 512 B contiguous).
template <bool BF16, bool IN_F32, int NV>
__global__ __launch_bounds__(256) void layernorm_vec_kernel(LnArgs a, Route rt) {
  // The row's data is asked for first; which segment (= whose gain and shift) the row
  // belongs to is found while it is on its way, in a copy of the segment offsets that the
  // workgroup put into LDS with one coalesced read (a search through global memory is a
  // chain of ten dependent round trips per wavefront).
  __shared__ int seg_s[kMaxRequests + 1];
  const int lane = threadIdx.x & 63;
  const int srow = min(blockIdx.x * 4 + (int)(threadIdx.x >> 6), a.n_rows - 1);   // surplus wavefronts redo the last row
  const bool ident = rt.identity != 0;               // shared parameters: identity row map, slot 0, no search
  const size_t row = ident ? (size_t)srow : (size_t)rt.row_src[srow];
  constexpr int d = NV * 256;
  constexpr bool in_f32 = IN_F32 || !BF16;
  f32x4 v[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) v[i] = load4(a.in, row * d + i * 256 + lane * 4, in_f32);
  if (a.in2) {
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] += load4(a.in2, row * d + i * 256 + lane * 4, !BF16);
  }
  if (a.sum_out) {
#pragma unroll
    for (int i = 0; i < NV; ++i) *reinterpret_cast<f32x4*>(a.sum_out + row * d + i * 256 + lane * 4) = v[i];
  }
  size_t slot_base = 0;
  if (!ident) {
    const int G = rt.n_segments[0];
    for (int i = threadIdx.x; i <= G; i += 256) seg_s[i] = rt.seg_tok_off[i];
    __syncthreads();
    int lo = 0, hi = G;
    while (hi - lo > 1) {
      int mid = (lo + hi) >> 1;
      if (seg_s[mid] <= srow) lo = mid; else hi = mid;
    }
    slot_base = (size_t)rt.seg_slot[lo] * a.slot_stride;
  }
  // gain and shift are asked for before the statistics are reduced: they arrive under the reductions
  f32x4 gg[NV], bb[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    gg[i] = load4(a.pool + slot_base + a.g_off, i * 256 + lane * 4, !BF16);
    bb[i] = load4(a.pool + slot_base + a.b_off, i * 256 + lane * 4, !BF16);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < NV; ++i) s += v[i][0] + v[i][1] + v[i][2] + v[i][3];
  const float mean = wave_sum(s) / (float)d;
  float q = 0.0f;
#pragma unroll
  for (int i = 0; i < NV; ++i)
    {
#pragma unroll
      for (int e = 0; e < 4; ++e) { const float c = v[i][e] - mean; q += c * c; }
    }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + a.eps);
#pragma unroll
  for (int i = 0; i < NV; ++i)
    {
      const int col = i * 256 + lane * 4;
      f32x4 y;
#pragma unroll
      for (int e = 0; e < 4; ++e) y[e] = (v[i][e] - mean) * rstd * gg[i][e] + bb[i][e];
      const size_t idx = row * d + col;
      if (a.out_f32) *reinterpret_cast<f32x4*>(a.out_f32 + idx) = y;
      if (a.out_st) {
        if (BF16) {
          u16x4 h = {f2bf(y[0]), f2bf(y[1]), f2bf(y[2]), f2bf(y[3])};
          *reinterpret_cast<u16x4*>(reinterpret_cast<uint16_t*>(a.out_st) + idx) = h;
        } else {
          *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.out_st) + idx) = y;
        }
      }
    }
}

}  // namespace

template <int NV>
static void launch_vec(const LnArgs& a, const Route& rt, hipStream_t s, unsigned blocks) {
  if (!a.bf16) hipLaunchKernelGGL((layernorm_vec_kernel<false, true, NV>), dim3(blocks), dim3(256), 0, s, a, rt);
  else if (a.in_f32) hipLaunchKernelGGL((layernorm_vec_kernel<true, true, NV>), dim3(blocks), dim3(256), 0, s, a, rt);
  else hipLaunchKernelGGL((layernorm_vec_kernel<true, false, NV>), dim3(blocks), dim3(256), 0, s, a, rt);
}

void launch_layernorm(const LnArgs& a, const Route& rt, hipStream_t s) {
  if (a.n_rows <= 0) return;
  const unsigned blocks = (unsigned)((a.n_rows + 3) / 4);
  switch (a.d) {
    case 256: return launch_vec<1>(a, rt, s, blocks);
    case 512: return launch_vec<2>(a, rt, s, blocks);
    case 768: return launch_vec<3>(a, rt, s, blocks);
    case 1024: return launch_vec<4>(a, rt, s, blocks);
    case 2048: return launch_vec<8>(a, rt, s, blocks);
    default: break;
  }
  if (a.bf16) hipLaunchKernelGGL(layernorm_kernel<true>, dim3(blocks), dim3(256), 0, s, a, rt);
  else hipLaunchKernelGGL(layernorm_kernel<false>, dim3(blocks), dim3(256), 0, s, a, rt);
}

}  // namespace hmi
