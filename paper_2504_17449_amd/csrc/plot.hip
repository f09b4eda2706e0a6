// GPU side of the paper's representation retrieval (Sec. 3.3.1): the hidden states that enter
// the higher layers are aggregated from precomputed representations of three-token fragments.
// The lookup (fragment -> table row) happens on the CPU in the paper; this kernel gathers the
// rows and forms, for every token, the sum of its representations in the fragments that contain
// it divided by their number.
//
// One workgroup per request, one wavefront per token in turn; a lane moves 16-byte chunks of the
// up to three source vectors (third token of the previous fragment, second of its own, first of
// the next), adds in fp32 and rounds once.  HBM-bound: 3 reads and 1 write of d elements per token.
#include "hmi_kernels.h"

namespace hmi {
namespace {

typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf2f(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

template <bool BF16>
__global__ __launch_bounds__(256) void plot_aggregate_kernel(PlotArgs a) {
  constexpr int EPC = BF16 ? 8 : 4;                 // elements per 16-byte chunk
  const int r = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int start = a.tok_off[r], len = a.tok_off[r + 1] - start;
  const int chunks = a.d / EPC;
  const size_t esize = BF16 ? 2 : 4, vec = (size_t)a.d * esize;   // bytes of one representation
  for (int i = wave; i < len; i += 4) {
    // table rows of the fragments centred on tokens i-1, i, i+1, clamped into the table
    const int e1 = min(max(a.frag_ids[start + i], 0), a.n_entries - 1);
    const int e0 = i > 0 ? min(max(a.frag_ids[start + i - 1], 0), a.n_entries - 1) : -1;
    const int e2 = i < len - 1 ? min(max(a.frag_ids[start + i + 1], 0), a.n_entries - 1) : -1;
    const char* s1 = a.table + ((size_t)e1 * 3 + 1) * vec;
    const char* s0 = e0 >= 0 ? a.table + ((size_t)e0 * 3 + 2) * vec : nullptr;
    const char* s2 = e2 >= 0 ? a.table + ((size_t)e2 * 3 + 0) * vec : nullptr;
    const float scale = 1.0f / (float)(1 + (e0 >= 0) + (e2 >= 0));
    char* dst = a.x + (size_t)(start + i) * vec;
    for (int c = lane; c < chunks; c += 64) {
      float acc[8];
      if (BF16) {
        const u16x8 v1 = *reinterpret_cast<const u16x8*>(s1 + c * 16);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = bf2f(v1[e]);
        if (s0) { const u16x8 v = *reinterpret_cast<const u16x8*>(s0 + c * 16);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[e] += bf2f(v[e]); }
        if (s2) { const u16x8 v = *reinterpret_cast<const u16x8*>(s2 + c * 16);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[e] += bf2f(v[e]); }
        u16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = f2bf(acc[e] * scale);
        *reinterpret_cast<u16x8*>(dst + c * 16) = o;
      } else {
        f32x4 v = *reinterpret_cast<const f32x4*>(s1 + c * 16);
        if (s0) v += *reinterpret_cast<const f32x4*>(s0 + c * 16);
        if (s2) v += *reinterpret_cast<const f32x4*>(s2 + c * 16);
        *reinterpret_cast<f32x4*>(dst + c * 16) = v * scale;
      }
    }
  }
}

}  // namespace

void launch_plot_aggregate(const PlotArgs& a, int R, bool bf16, hipStream_t s) {
  if (R <= 0) return;
  if (bf16) hipLaunchKernelGGL(plot_aggregate_kernel<true>, dim3(R), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(plot_aggregate_kernel<false>, dim3(R), dim3(256), 0, s, a);
}

}  // namespace hmi
