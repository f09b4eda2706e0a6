// Per-tenant output heads (Sec. 3.3.2 of the paper): a linear layer per tenant on the final
// hidden states, classification tenants on the first row of a request, tagging tenants on
// every row, label = class of the highest score.
//
// One workgroup per request, one wavefront per row in turn.  A lane holds d/64 elements of the
// row (k = lane + 64 j) and multiplies them with the same elements of every class's weight row
// (a tenant's head is a few KB and stays in cache across the rows of a request); a shuffle
// reduction gives the score.  HBM-bound on reading h for tagging tenants, latency-bound else.
#include "hmi_kernels.h"

#include <math.h>

namespace hmi {
namespace {

constexpr int kMaxPerLane = 32;  // d <= 2048

__device__ __forceinline__ float bf2f(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
__device__ __forceinline__ float ld(const void* p, size_t i, bool bf16) {
  return bf16 ? bf2f(reinterpret_cast<const uint16_t*>(p)[i]) : reinterpret_cast<const float*>(p)[i];
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__global__ __launch_bounds__(256) void head_kernel(HeadArgs a, Route rt) {
  const int r = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tenant = rt.req_tenant[r];
  const int n_classes = a.meta[2 * tenant], per_token = a.meta[2 * tenant + 1];
  const int start = rt.tok_off[r], len = rt.tok_off[r + 1] - start;
  const char* W = a.heads + (size_t)tenant * a.head_stride;
  const size_t esize = a.bf16 ? 2 : 4;
  const void* B = W + (size_t)a.max_classes * a.d * esize;
  const int per = a.d >> 6;
  const float ninf = -INFINITY;

  for (int i = wave; i < len; i += 4) {
    const size_t row = (size_t)start + i;
    float* srow = a.scores ? a.scores + row * a.max_classes : nullptr;
    if (!per_token && i > 0) {        // no prediction for this row
      if (srow) for (int c = lane; c < a.max_classes; c += 64) srow[c] = ninf;
      if (lane == 0) a.labels[row] = -1;
      continue;
    }
    float hv[kMaxPerLane];
#pragma unroll
    for (int j = 0; j < kMaxPerLane; ++j)
      if (j < per) hv[j] = ld(a.h, row * a.d + lane + 64 * j, a.bf16);
    float best = ninf;
    int best_c = 0;
    for (int c = 0; c < n_classes; ++c) {
      float acc = 0.0f;
#pragma unroll
      for (int j = 0; j < kMaxPerLane; ++j)
        if (j < per) acc = fmaf(hv[j], ld(W, (size_t)c * a.d + lane + 64 * j, a.bf16), acc);
      const float sc = wave_sum(acc) + ld(B, c, a.bf16);
      if (sc > best) { best = sc; best_c = c; }   // strict: the lowest index wins ties
      if (srow && lane == 0) srow[c] = sc;
    }
    if (srow) for (int c = n_classes + lane; c < a.max_classes; c += 64) srow[c] = ninf;
    if (lane == 0) a.labels[row] = best_c;
  }
}

}  // namespace

void launch_heads(const HeadArgs& a, const Route& rt, int R, hipStream_t s) {
  if (R <= 0) return;
  hipLaunchKernelGGL(head_kernel, dim3(R), dim3(256), 0, s, a, rt);
}

}  // namespace hmi
