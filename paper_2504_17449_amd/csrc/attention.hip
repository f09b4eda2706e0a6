// Per-request multi-head self-attention on packed rows: ctx = softmax(Q K^T / sqrt(d_head)
// [+ causal mask]) V, one request and one head at a time, never across requests and with
// no padding keys (rows are packed).  Part of the per-tenant layer of the mixed-tenant
// forward (Sec. 6.3 gives the batching, BERT / GPT give the sub-layer).
//
// bf16 kernel (d_head = 64), one workgroup = 128 query rows of one (request, head), four
// wavefronts of 32 queries each.  Keys/values stream through LDS in blocks of 64 keys (the next
// block is loaded into registers while this one is multiplied; V is transposed in registers) with
// an online softmax.  Both products run on v_mfma_f32_32x32x16_bf16 in TRANSPOSED form so
// that every lane owns one query column throughout:
//   S^T = K Q^T   (A = K block from LDS, B = Q^T held in registers)
//   O^T = V^T P^T (A = V^T block from LDS, B = P^T = the S^T accumulators, converted in
//                  registers; the key order inside a k-step is whatever the accumulator
//                  layout gives, and V^T is read in that same order)
// so softmax statistics, the rescale of O and the final 1/l are lane-local (plus one
// exchange with the partner lane 32 apart, which holds the other half of the keys).
#include "hmi_kernels.h"

namespace hmi {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float bf2f(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

constexpr int QB = 128;       // queries per workgroup
constexpr int KB = 64;        // keys per LDS block
constexpr int DH = 64;        // head width
constexpr int VT_LD = 72;     // V^T row pitch in elements (keys), padded

__global__ __launch_bounds__(256) void attn_bf16_kernel(AttnArgs a, Route rt) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[KB * DH];      // [key][dh], swizzled chunks
  __shared__ __attribute__((aligned(16))) uint16_t Vt[DH * VT_LD];   // [dh][key]

  const int r = blockIdx.z, head = blockIdx.y, q0 = blockIdx.x * QB;
  const int start = rt.tok_off[r];
  const int len = rt.tok_off[r + 1] - start;
  if (q0 >= len) return;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6, l32 = lane & 31, lh = lane >> 5;
  const int d = a.d, ld = 3 * d;
  const uint16_t* qkv = reinterpret_cast<const uint16_t*>(a.qkv);
  const uint16_t* Qg = qkv + (size_t)start * ld + head * DH;
  const uint16_t* Kg = Qg + d;
  const uint16_t* Vg = Qg + 2 * d;

  const int q = q0 + wave * 32 + l32;            // this lane's query (request-local)
  const int qc = min(q, len - 1);
  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    qf[ks] = *reinterpret_cast<const bf16x8*>(Qg + (size_t)qc * ld + ks * 16 + lh * 8);

  f32x16 o[2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[u][i] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;

  const int q_last = min(q0 + QB, len) - 1;                    // last query of the workgroup
  const int n_keys = a.causal ? q_last + 1 : len;              // keys any query here can see
  const int wave_q_last = q0 + wave * 32 + 31;
  const bool wave_has_rows = q0 + wave * 32 < len;
  constexpr float kExpScale = 0.125f * 1.4426950408889634f;    // log2(e) / sqrt(64)

  // A key block goes global -> registers -> LDS; the registers of the next block are loaded while this
  // one is multiplied.  K: 64 keys x 8 chunks of 16 bytes, two per thread, swizzled.  V^T: thread (key
  // group kg, column pair cp) reads two columns of eight keys (4 bytes per key, a wavefront's 32 column
  // pairs cover the key's 128-byte row) and writes each column's eight keys as one 16-byte piece.
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 kreg[2];
  uint32_t vw[8];
  const int v_kg = t >> 5, v_cp = t & 31;
#define HMI_LOAD_BLOCK(K0)                                                                         \
  {                                                                                                \
    _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                                \
      const int qd = t + 256 * i, key = qd >> 3, c = qd & 7;                                       \
      kreg[i] = *reinterpret_cast<const u32x4*>(Kg + (size_t)min((K0) + key, len - 1) * ld + c * 8); \
    }                                                                                              \
    _Pragma("unroll") for (int e = 0; e < 8; ++e)                                                  \
      vw[e] = *reinterpret_cast<const uint32_t*>(Vg + (size_t)min((K0) + v_kg * 8 + e, len - 1) * ld + v_cp * 2); \
  }
  HMI_LOAD_BLOCK(0)

  for (int k0 = 0; k0 < n_keys; k0 += KB) {
    __syncthreads();  // previous block fully consumed
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int qd = t + 256 * i, key = qd >> 3, c = qd & 7;
      *reinterpret_cast<u32x4*>(Ks + key * DH + ((c ^ swz(key)) << 3)) = kreg[i];
    }
    {
      u32x4 lo, hi;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        lo[j] = (vw[2 * j] & 0xFFFFu) | (vw[2 * j + 1] << 16);
        hi[j] = (vw[2 * j] >> 16) | (vw[2 * j + 1] & 0xFFFF0000u);
      }
      *reinterpret_cast<u32x4*>(Vt + (2 * v_cp) * VT_LD + v_kg * 8) = lo;
      *reinterpret_cast<u32x4*>(Vt + (2 * v_cp + 1) * VT_LD + v_kg * 8) = hi;
    }
    if (k0 + KB < n_keys) HMI_LOAD_BLOCK(k0 + KB)   // in flight during this block's arithmetic
    __syncthreads();
    const bool skip = !wave_has_rows || (a.causal && k0 > wave_q_last);
    if (skip) continue;

    // ---- S^T = K Q^T for the two 32-key tiles of this block
    f32x16 s[2];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) s[tt][i] = 0.0f;
      const int key = tt * 32 + l32;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(Ks + key * DH + (((ks * 2 + lh) ^ swz(key)) << 3));
        s[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[tt], 0, 0, 0);
      }
    }
    // ---- mask, block max, exponentials.  s[tt][i] is key k0 + tt*32 + 8*(i/4) + 4*lh + i%4, query q.
    // The scores stay unscaled: exp((s - m) / 8) is one fma and one exp2 with c = log2(e) / 8.  Only a
    // block that reaches past the request's end or past this wavefront's first query (causal) has
    // keys to mask, which is the same for all lanes of the wavefront.
    const bool need_mask = k0 + KB > len || (a.causal && k0 + KB - 1 > q0 + wave * 32);
    if (need_mask) {
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = k0 + tt * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
          const bool ok = key < len && (!a.causal || key <= q);
          s[tt][i] = ok ? s[tt][i] : -INFINITY;
        }
    }
    float m_blk = -INFINITY;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int i = 0; i < 16; ++i) m_blk = fmaxf(m_blk, s[tt][i]);
    m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 32, 64));
    const float m_new = fmaxf(m_run, m_blk);
    // queries past the request end (or fully masked so far) keep m_new = -inf: use 0 there
    const float m_use = m_new == -INFINITY ? 0.0f : m_new;
    const float mc = m_use * kExpScale;
    const float alpha = __builtin_amdgcn_exp2f(fmaf(m_run, kExpScale, -mc));
    float psum = 0.0f;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[tt][i], kExpScale, -mc));
        s[tt][i] = p;
        psum += p;
      }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[u][i] *= alpha;

    // ---- O^T += V^T P^T, 16 keys per MFMA: k-slot (lh, e) <-> key base + 8*(e/4) + 4*lh + e%4
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int hb = 0; hb < 2; ++hb) {
        bf16x8 pf;
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[e] = (__bf16)s[tt][hb * 8 + e];
        const int kbase = tt * 32 + hb * 16 + lh * 4;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const uint16_t* vrow = Vt + (u * 32 + l32) * VT_LD + kbase;
          const bf16x4 v0 = *reinterpret_cast<const bf16x4*>(vrow);
          const bf16x4 v1 = *reinterpret_cast<const bf16x4*>(vrow + 8);
          bf16x8 vf;
#pragma unroll
          for (int e = 0; e < 4; ++e) { vf[e] = v0[e]; vf[4 + e] = v1[e]; }
          o[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[u], 0, 0, 0);
        }
      }
  }

#undef HMI_LOAD_BLOCK

  // ---- normalise and store: o[u][i] is dh = u*32 + 8*(i/4) + 4*lh + i%4 of query q
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (q < len) {
    const float inv = 1.0f / l_tot;
    uint16_t* out = reinterpret_cast<uint16_t*>(a.ctx) + (size_t)(start + q) * d + head * DH;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        ushort4 pk;
        pk.x = f2bf(o[u][g4 * 4 + 0] * inv);
        pk.y = f2bf(o[u][g4 * 4 + 1] * inv);
        pk.z = f2bf(o[u][g4 * 4 + 2] * inv);
        pk.w = f2bf(o[u][g4 * 4 + 3] * inv);
        *reinterpret_cast<ushort4*>(out + u * 32 + g4 * 8 + lh * 4) = pk;
      }
  }
}

// fp32 attention for fp32 pools: one wavefront per (row, head), keys in blocks of 64 with
// an online softmax; lane j scores key j, then lane c accumulates output column c.
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__global__ __launch_bounds__(64) void attn_f32_kernel(AttnArgs a, Route rt, int n_rows) {
  __shared__ float qs[64];
  __shared__ float ps[64];
  const int row = blockIdx.x, head = blockIdx.y, lane = threadIdx.x;
  if (row >= n_rows) return;
  int lo = 0, hi = a.R;  // request of this row: last r with tok_off[r] <= row
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (rt.tok_off[mid] <= row) lo = mid; else hi = mid;
  }
  const int start = rt.tok_off[lo], len = rt.tok_off[lo + 1] - start, qi = row - start;
  const int d = a.d, dh = d / a.n_heads, ld = 3 * d;
  const float* qkv = reinterpret_cast<const float*>(a.qkv);
  const float* Qg = qkv + (size_t)row * ld + head * dh;
  const float* Kg = qkv + (size_t)start * ld + d + head * dh;
  const float* Vg = Kg + d;
  if (lane < dh) qs[lane] = Qg[lane];
  __syncthreads();
  const int n_keys = a.causal ? qi + 1 : len;
  const float scale = 1.0f / sqrtf((float)dh);
  float m_run = -INFINITY, l_run = 0.0f, o = 0.0f;
  for (int k0 = 0; k0 < n_keys; k0 += 64) {
    const int j = k0 + lane;
    float s = -INFINITY;
    if (j < n_keys) {
      float acc = 0.0f;
      for (int c = 0; c < dh; ++c) acc = fmaf(qs[c], Kg[(size_t)j * ld + c], acc);
      s = acc * scale;
    }
    const float m_new = fmaxf(m_run, wave_max(s));
    const float alpha = expf(m_run - m_new);
    const float p = j < n_keys ? expf(s - m_new) : 0.0f;
    l_run = l_run * alpha + wave_sum(p);
    m_run = m_new;
    __syncthreads();
    ps[lane] = p;
    __syncthreads();
    o *= alpha;
    if (lane < dh) {
      const int nk = min(64, n_keys - k0);
      for (int jj = 0; jj < nk; ++jj) o = fmaf(ps[jj], Vg[(size_t)(k0 + jj) * ld + lane], o);
    }
  }
  if (lane < dh) reinterpret_cast<float*>(a.ctx)[(size_t)row * d + head * dh + lane] = o / l_run;
}

}  // namespace

void launch_attention(const AttnArgs& a, const Route& rt, hipStream_t s) {
  if (a.R <= 0) return;
  if (a.bf16) {
    dim3 grid((a.max_len + QB - 1) / QB, a.n_heads, a.R);
    hipLaunchKernelGGL(attn_bf16_kernel, grid, dim3(256), 0, s, a, rt);
  } else {
    dim3 grid(a.n_rows, a.n_heads, 1);
    hipLaunchKernelGGL(attn_f32_kernel, grid, dim3(64), 0, s, a, rt, a.n_rows);
  }
}

}  // namespace hmi
