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
//   attn_decode_kernel one new token per request: one wavefront per (request, head).  Eight
//                      lanes share a position (16 bytes of the 128-byte key each), eight
//                      positions per step; an online softmax per lane group, merged at the end.
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

__device__ __forceinline__ void soft_add(Soft& s, float score, const float (&v)[8]) {
  const float mn = fmaxf(s.m, score);
  const float corr = s.m == mn ? 1.0f : __expf(s.m - mn);
  const float p = __expf(score - mn);
  s.l = s.l * corr + p;
#pragma unroll
  for (int e = 0; e < 8; ++e) s.acc[e] = s.acc[e] * corr + p * v[e];
  s.m = mn;
}

__global__ __launch_bounds__(256) void attn_decode_kernel(KvArgs a, Route rt) {
  const int r = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int head = blockIdx.y * 4 + wave;
  if (head >= a.n_heads) return;
  const int part = lane & 7, g = lane >> 3;
  const int slot = rt.kv_slot[r], pos = rt.kv_pos[r];      // pos = positions already in the line
  const size_t row = (size_t)rt.tok_off[r];
  const uint16_t* qkv = reinterpret_cast<const uint16_t*>(a.qkv) + row * 3 * a.d + head * DH + part * 8;
  const u16x8 q8 = *reinterpret_cast<const u16x8*>(qkv);
  const u16x8 k8 = *reinterpret_cast<const u16x8*>(qkv + a.d);
  const u16x8 v8 = *reinterpret_cast<const u16x8*>(qkv + 2 * a.d);
  float q[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) q[e] = bf2f(q8[e]) * 0.125f;   // 1 / sqrt(64)
  uint16_t* Kc = a.cache + line_off(a, slot, 0, head);
  uint16_t* Vc = a.cache + line_off(a, slot, 1, head);

  Soft s;
  s.m = -INFINITY; s.l = 0.0f;
#pragma unroll
  for (int e = 0; e < 8; ++e) s.acc[e] = 0.0f;
  for (int p = g; p < pos; p += 8) {       // all eight lanes of a group take the same trips
    const u16x8 kk = *reinterpret_cast<const u16x8*>(Kc + (size_t)p * DH + part * 8);
    const u16x8 vv = *reinterpret_cast<const u16x8*>(Vc + (size_t)p * DH + part * 8);
    float sc = 0.0f, vf[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { sc = fmaf(q[e], bf2f(kk[e]), sc); vf[e] = bf2f(vv[e]); }
    sc += __shfl_xor(sc, 1, 64); sc += __shfl_xor(sc, 2, 64); sc += __shfl_xor(sc, 4, 64);
    soft_add(s, sc, vf);
  }
  {  // the new token itself (every group computes the score, group 0 counts it)
    float sc = 0.0f, vf[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { sc = fmaf(q[e], bf2f(k8[e]), sc); vf[e] = bf2f(v8[e]); }
    sc += __shfl_xor(sc, 1, 64); sc += __shfl_xor(sc, 2, 64); sc += __shfl_xor(sc, 4, 64);
    if (g == 0) soft_add(s, sc, vf);
  }
  // merge the eight groups (lanes with the same part)
#pragma unroll
  for (int o = 8; o < 64; o <<= 1) {
    const float mo = __shfl_xor(s.m, o, 64), lo = __shfl_xor(s.l, o, 64);
    const float mn = fmaxf(s.m, mo);
    const float c0 = s.m == mn ? 1.0f : __expf(s.m - mn), c1 = mo == mn ? 1.0f : __expf(mo - mn);
    s.l = s.l * c0 + lo * c1;
#pragma unroll
    for (int e = 0; e < 8; ++e) s.acc[e] = s.acc[e] * c0 + __shfl_xor(s.acc[e], o, 64) * c1;
    s.m = mn;
  }
  if (g == 0) {
    u16x8 o8;
    const float inv = 1.0f / s.l;
#pragma unroll
    for (int e = 0; e < 8; ++e) o8[e] = f2bf(s.acc[e] * inv);
    *reinterpret_cast<u16x8*>(reinterpret_cast<uint16_t*>(a.ctx) + row * a.d + head * DH + part * 8) = o8;
    *reinterpret_cast<u16x8*>(Kc + (size_t)pos * DH + part * 8) = k8;
  } else if (g == 1) {
    *reinterpret_cast<u16x8*>(Vc + (size_t)pos * DH + part * 8) = v8;
  }
}

}  // namespace

void launch_kv_store(const KvArgs& a, const Route& rt, int R, hipStream_t s) {
  if (R <= 0) return;
  hipLaunchKernelGGL(kv_store_kernel, dim3(R), dim3(256), 0, s, a, rt);
}

void launch_attn_decode(const KvArgs& a, const Route& rt, int R, hipStream_t s) {
  if (R <= 0) return;
  hipLaunchKernelGGL(attn_decode_kernel, dim3(R, (a.n_heads + 3) / 4), dim3(256), 0, s, a, rt);
}

}  // namespace hmi
