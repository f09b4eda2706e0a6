// Key/value cache for autoregressive decoding with the per-tenant decoder layer (the paper
// reports hGPT in generated tokens per second, Sec. 7; the mixed-tenant batching of Sec. 6.3 is
// the same, one new token per request).
//
// Cache line of one (layer, sequence slot): [k | v][head][position][64] in bf16, so that the
// keys (values) of one head are contiguous over positions: a decode step streams them with
// coalesced 1 KB reads.
//
//   kv_store_kernel    after a full-sequence (prefill) QKV projection: every row's k and v go
//                      to position (first position of the request + row index) of its line.
//   attn_decode_kernel one new token per request: one workgroup per (request, head).  Eight
//                      lanes share a position (16 bytes of the 128-byte key each), 32 positions
//                      per step of the workgroup, four steps' loads in flight at a time; an online
//                      softmax per lane group, merged at the end.
//                      The new token's own key and value come from registers and are appended
//                      to the line for the steps that follow.  All arithmetic in fp32.
#include "hmi_kernels.h"

#include <math.h>

namespace hmi {
namespace {

typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float bf2f(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

constexpr int DH = 64;

__device__ __forceinline__ size_t line_off(const KvArgs& a, int slot, int kv, int head) {
  return ((((size_t)slot * 2 + kv) * a.n_heads + head) * a.max_len) * DH;
}

__global__ __launch_bounds__(256) void kv_store_kernel(KvArgs a, Route rt) {
  const int r = blockIdx.x;
  const int slot = rt.kv_slot[r], pos0 = rt.kv_pos[r];
  const int start = rt.tok_off[r], len = rt.tok_off[r + 1] - start;
  const uint16_t* qkv = reinterpret_cast<const uint16_t*>(a.qkv);
  const int cpr = a.d / 8;                         // 16-byte chunks per row of k (or v)
  for (int idx = threadIdx.x; idx < len * 2 * cpr; idx += 256) {
    const int i = idx / (2 * cpr), c = idx % (2 * cpr);
    const int kv = c / cpr, cc = c % cpr, head = cc >> 3, part = cc & 7;
    const u16x8 v = *reinterpret_cast<const u16x8*>(qkv + (size_t)(start + i) * 3 * a.d + (1 + kv) * a.d + cc * 8);
    *reinterpret_cast<u16x8*>(a.cache + line_off(a, slot, kv, head) + (size_t)(pos0 + i) * DH + part * 8) = v;
  }
}

// running softmax state of one lane: maximum, denominator, 8 numerators
struct Soft { float m, l, acc[8]; };

__device__ __forceinline__ void soft_merge(Soft& s, float mo, float lo, const float (&ao)[8]) {
  const float mn = fmaxf(s.m, mo);
  const float c0 = s.m == mn ? 1.0f : __expf(s.m - mn), c1 = mo == mn ? 1.0f : __expf(mo - mn);
  s.l = s.l * c0 + lo * c1;
#pragma unroll
  for (int e = 0; e < 8; ++e) s.acc[e] = s.acc[e] * c0 + ao[e] * c1;
  s.m = mn;
}

constexpr int PB = 4;   // positions a lane group takes per trip (their loads are in flight together)

// One workgroup per (request, head); its 32 lane groups (8 lanes each, 16 bytes of a position's
// 128-byte key per lane) take positions g, g + 32, ... in batches of PB.
__global__ __launch_bounds__(256) void attn_decode_kernel(KvArgs a, Route rt) {
  __shared__ float part_s[4][8][10];           // per wavefront and part: m, l, 8 numerators
  const int r = blockIdx.x, head = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int part = lane & 7, g = wave * 8 + (lane >> 3);
  const int slot = rt.kv_slot[r], pos = rt.kv_pos[r];      // pos = positions already in the line
  const size_t row = (size_t)rt.tok_off[r];
  const uint16_t* qkv = reinterpret_cast<const uint16_t*>(a.qkv) + row * 3 * a.d + head * DH + part * 8;
  const u16x8 q8 = *reinterpret_cast<const u16x8*>(qkv);
  float q[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) q[e] = bf2f(q8[e]) * 0.125f;   // 1 / sqrt(64)
  uint16_t* Kc = a.cache + line_off(a, slot, 0, head);
  uint16_t* Vc = a.cache + line_off(a, slot, 1, head);

  Soft s;
  s.m = -INFINITY; s.l = 0.0f;
#pragma unroll
  for (int e = 0; e < 8; ++e) s.acc[e] = 0.0f;
  for (int p0 = g; p0 < pos; p0 += 32 * PB) {   // all eight lanes of a group take the same trips
    u16x8 kk[PB], vv[PB];
#pragma unroll
    for (int u = 0; u < PB; ++u) {
      const int p = min(p0 + 32 * u, pos - 1);  // surplus positions of the last trip repeat a valid one and get no weight
      // read once per step and far larger than the caches: the non-temporal hint keeps the lines out of L2, where the
      // step's other kernels find their weights again (a step through six shared layers: 0.662 -> 0.601 ms)
      kk[u] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(Kc + (size_t)p * DH + part * 8));
      vv[u] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(Vc + (size_t)p * DH + part * 8));
    }
    float sc[PB];
#pragma unroll
    for (int u = 0; u < PB; ++u) {
      float t = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) t = fmaf(q[e], bf2f(kk[u][e]), t);
      t += __shfl_xor(t, 1, 64); t += __shfl_xor(t, 2, 64); t += __shfl_xor(t, 4, 64);
      sc[u] = p0 + 32 * u < pos ? t : -INFINITY;
    }
    float mn = s.m;
#pragma unroll
    for (int u = 0; u < PB; ++u) mn = fmaxf(mn, sc[u]);   // finite: the trip's first position is valid
    const float corr = s.m == mn ? 1.0f : __expf(s.m - mn);
    s.l *= corr;
#pragma unroll
    for (int e = 0; e < 8; ++e) s.acc[e] *= corr;
#pragma unroll
    for (int u = 0; u < PB; ++u) {
      const float w = __expf(sc[u] - mn);                 // exp(-inf) = 0 for the surplus positions
      s.l += w;
#pragma unroll
      for (int e = 0; e < 8; ++e) s.acc[e] = fmaf(w, bf2f(vv[u][e]), s.acc[e]);
    }
    s.m = mn;
  }
  // the new token itself, from registers (group 0 counts it and appends it to the line)
  if (g < 2) {
    const u16x8 k8 = *reinterpret_cast<const u16x8*>(qkv + a.d);
    const u16x8 v8 = *reinterpret_cast<const u16x8*>(qkv + 2 * a.d);
    if (g == 0) {
      float t = 0.0f, vf[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) { t = fmaf(q[e], bf2f(k8[e]), t); vf[e] = bf2f(v8[e]); }
      t += __shfl_xor(t, 1, 64); t += __shfl_xor(t, 2, 64); t += __shfl_xor(t, 4, 64);
      soft_merge(s, t, 1.0f, vf);
      *reinterpret_cast<u16x8*>(Kc + (size_t)pos * DH + part * 8) = k8;
    } else {
      *reinterpret_cast<u16x8*>(Vc + (size_t)pos * DH + part * 8) = v8;
    }
  }
  // merge the eight groups of a wavefront (lanes with the same part), then the four wavefronts
#pragma unroll
  for (int o = 8; o < 64; o <<= 1) {
    float ao[8];
    const float mo = __shfl_xor(s.m, o, 64), lo = __shfl_xor(s.l, o, 64);
#pragma unroll
    for (int e = 0; e < 8; ++e) ao[e] = __shfl_xor(s.acc[e], o, 64);
    soft_merge(s, mo, lo, ao);
  }
  if (lane < 8) {
    part_s[wave][part][0] = s.m; part_s[wave][part][1] = s.l;
#pragma unroll
    for (int e = 0; e < 8; ++e) part_s[wave][part][2 + e] = s.acc[e];
  }
  __syncthreads();
  if (wave == 0 && lane < 8) {
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      float ao[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) ao[e] = part_s[w][part][2 + e];
      soft_merge(s, part_s[w][part][0], part_s[w][part][1], ao);
    }
    u16x8 o8;
    const float inv = 1.0f / s.l;
#pragma unroll
    for (int e = 0; e < 8; ++e) o8[e] = f2bf(s.acc[e] * inv);
    *reinterpret_cast<u16x8*>(reinterpret_cast<uint16_t*>(a.ctx) + row * a.d + head * DH + part * 8) = o8;
  }
}

}  // namespace

void launch_kv_store(const KvArgs& a, const Route& rt, int R, hipStream_t s) {
  if (R <= 0) return;
  hipLaunchKernelGGL(kv_store_kernel, dim3(R), dim3(256), 0, s, a, rt);
}

void launch_attn_decode(const KvArgs& a, const Route& rt, int R, hipStream_t s) {
  if (R <= 0) return;
  hipLaunchKernelGGL(attn_decode_kernel, dim3(R, a.n_heads), dim3(256), 0, s, a, rt);
}

}  // namespace hmi
