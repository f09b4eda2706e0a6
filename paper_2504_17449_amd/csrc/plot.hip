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

constexpr int kIdsInLds = 2048;   // fragment ids of a request kept in LDS (longer requests read the rest from memory)

// the (up to) three source vectors of one token and its scale
struct Sources { const char* s0; const char* s1; const char* s2; float scale; };

template <bool BF16>
__device__ __forceinline__ void sum_chunk(const Sources& t, char* dst, int c) {
  if (BF16) {
    const u16x8 v1 = *reinterpret_cast<const u16x8*>(t.s1 + c * 16);
    u16x8 v0 = {}, v2 = {};
    if (t.s0) v0 = *reinterpret_cast<const u16x8*>(t.s0 + c * 16);
    if (t.s2) v2 = *reinterpret_cast<const u16x8*>(t.s2 + c * 16);
    u16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = f2bf((bf2f(v1[e]) + bf2f(v0[e]) + bf2f(v2[e])) * t.scale);
    *reinterpret_cast<u16x8*>(dst + c * 16) = o;
  } else {
    f32x4 v = *reinterpret_cast<const f32x4*>(t.s1 + c * 16);
    if (t.s0) v += *reinterpret_cast<const f32x4*>(t.s0 + c * 16);
    if (t.s2) v += *reinterpret_cast<const f32x4*>(t.s2 + c * 16);
    *reinterpret_cast<f32x4*>(dst + c * 16) = v * t.scale;
  }
}

template <bool BF16>
__global__ __launch_bounds__(256) void plot_aggregate_kernel(PlotArgs a) {
  __shared__ int ids_s[kIdsInLds];
  constexpr int EPC = BF16 ? 8 : 4;                 // elements per 16-byte chunk
  const int r = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int start = a.tok_off[r], len = a.tok_off[r + 1] - start;
  const int chunks = a.d / EPC;
  const size_t vec = (size_t)a.d * (BF16 ? 2 : 4);  // bytes of one representation
  // the request's table rows (clamped into the table), read once
  const int in_lds = min(len, kIdsInLds);
  for (int i = threadIdx.x; i < in_lds; i += 256) ids_s[i] = min(max(a.frag_ids[start + i], 0), a.n_entries - 1);
  __syncthreads();
  auto id_at = [&](int j) { return j < in_lds ? ids_s[j] : min(max(a.frag_ids[start + j], 0), a.n_entries - 1); };
  // token i is the third token of fragment i-1, the second of fragment i, the first of fragment i+1
  auto sources = [&](int i) {
    Sources t;
    t.s1 = a.table + ((size_t)id_at(i) * 3 + 1) * vec;
    t.s0 = i > 0 ? a.table + ((size_t)id_at(i - 1) * 3 + 2) * vec : nullptr;
    t.s2 = i < len - 1 ? a.table + ((size_t)id_at(i + 1) * 3 + 0) * vec : nullptr;
    t.scale = 1.0f / (float)(1 + (i > 0) + (i < len - 1));
    return t;
  };
  // one wavefront per token in turn, two tokens per trip: their six source vectors are in flight together
  for (int i = wave; i < len; i += 8) {
    const bool two = i + 4 < len;
    const Sources ta = sources(i), tb = sources(two ? i + 4 : i);
    char* da = a.x + (size_t)(start + i) * vec;
    char* db = a.x + (size_t)(start + i + 4) * vec;
    for (int c = lane; c < chunks; c += 64) {
      sum_chunk<BF16>(ta, da, c);
      if (two) sum_chunk<BF16>(tb, db, c);
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
