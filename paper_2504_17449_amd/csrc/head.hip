// Per-tenant output heads (Sec. 3.3.2 of the paper): a linear layer per tenant on the final
// hidden states, classification tenants on the first row of a request, tagging tenants on
// every row, label = class of the highest score.
//
// The scores of all rows against their tenant's (zero-padded) 64 class rows are one more
// grouped GEMM over the tenant route, with fp32 output.  This kernel finishes the job: one
// workgroup per request, one wavefront per row in turn, lane c holds the row's score of class
// c; classes the tenant does not have and rows that get no prediction are masked, the label is
// a wavefront arg-max (lowest index on ties), and the scores are compacted to max_classes
// columns if the caller wants them.
#include "hmi_kernels.h"

#include <math.h>

namespace hmi {
namespace {

__global__ __launch_bounds__(256) void head_select_kernel(HeadArgs a, Route rt) {
  const int r = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tenant = rt.req_tenant[r];
  const int n_classes = a.meta[2 * tenant], per_token = a.meta[2 * tenant + 1];
  const int start = rt.tok_off[r], len = rt.tok_off[r + 1] - start;
  const float ninf = -INFINITY;
  for (int i = wave; i < len; i += 4) {
    const size_t row = (size_t)start + i;
    const bool predict = per_token || i == 0;
    float sc = (predict && lane < n_classes) ? a.raw[row * kHeadCols + lane] : ninf;
    if (a.scores && lane < a.max_classes) a.scores[row * a.max_classes + lane] = sc;
    int best = lane;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float osc = __shfl_xor(sc, o, 64);
      const int ob = __shfl_xor(best, o, 64);
      if (osc > sc || (osc == sc && ob < best)) { sc = osc; best = ob; }
    }
    if (lane == 0) a.labels[row] = predict ? best : -1;
  }
}

}  // namespace

void launch_head_select(const HeadArgs& a, const Route& rt, int R, hipStream_t s) {
  if (R <= 0) return;
  hipLaunchKernelGGL(head_select_kernel, dim3(R), dim3(256), 0, s, a, rt);
}

}  // namespace hmi
