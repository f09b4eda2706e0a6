// Tenant-segmented router: orders a batch's requests by tenant id (stable), finds the
// segments of equal tenant and their offsets, and emits the m-tile work lists and the
// sorted-row -> original-row map the grouped GEMMs consume.
//
// This is the GPU form of "stack the parameters of the adapters per request" in the
// paper's parallel adapter inference (Sec. 6.3): instead of copying a tenant's parameters
// next to every request, requests are grouped so that one segment shares one weight image.
//
// One workgroup of 1024 lanes (16 wavefronts).  The sort is an LSD radix sort, 4 bits per
// pass; within a wavefront the stable rank of an element among equal digits comes from
// ballots, across wavefronts from an exclusive scan of the per-wavefront digit counts.
// All prefix sums are wavefront shuffles-up plus a 16-entry cross-wavefront step.
#include "hmi_kernels.h"

namespace hmi {
namespace {

constexpr int kWaves = kRouterThreads / 64;
constexpr int kRounds = kMaxRequests / kRouterThreads;  // elements per lane

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int t = __shfl_up(v, o, 64);
    if (lane >= o) v += t;
  }
  return v;
}

// Exclusive prefix sum over the 1024 lanes of the workgroup; `total` gets the sum.
// Every lane must call it (it synchronises).
__device__ __forceinline__ int block_exscan(int v, int* wave_tot, int& total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int inc = wave_incl_scan(v, lane);
  if (lane == 63) wave_tot[w] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kWaves; ++i) {
    int t = wave_tot[i];
    if (i < w) base += t;
    tot += t;
  }
  __syncthreads();
  total = tot;
  return base + inc - v;
}

__global__ __launch_bounds__(kRouterThreads) void router_kernel(Route rt, int R, int key_bits) {
  __shared__ int key[2][kMaxRequests];
  __shared__ int val[2][kMaxRequests];
  __shared__ int tok_s[kMaxRequests + 1];     // request -> first original row
  __shared__ int stok_s[kMaxRequests + 1];    // sorted position -> first sorted row
  __shared__ int segtok_s[kMaxRequests + 1];  // segment -> first sorted row
  __shared__ int cnt[16 * kRounds * kWaves];
  __shared__ int wave_tot[kWaves];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int rounds = (R + kRouterThreads - 1) / kRouterThreads;

  // ---- tok_off = exclusive scan of seq_lens in arrival order.  The three input arrays may
  //      live in host memory (a round trip over the host link per dependent read), so each
  //      is read exactly once, here, all reads in flight together.
  int carry = 0;
  int slot_r[kRounds];
#pragma unroll
  for (int c = 0; c < kRounds; ++c) {
    slot_r[c] = 0;
    if (c < rounds) {
      int i = c * kRouterThreads + tid;
      int len = i < R ? rt.seq_lens[i] : 0;
      int tenant = i < R ? rt.tenant_ids[i] : 0;
      slot_r[c] = i < R ? rt.req_slot[i] : 0;
      if (rt.kv_slot_in && i < R) { rt.kv_slot[i] = rt.kv_slot_in[i]; rt.kv_pos[i] = rt.kv_pos_in[i]; }
      int tot;
      int ex = block_exscan(len, wave_tot, tot) + carry;
      if (i < R) { tok_s[i] = ex; rt.tok_off[i] = ex; rt.req_tenant[i] = tenant; key[0][i] = tenant; val[0][i] = i; }
      carry += tot;
    }
  }
  const int N = carry;
  if (tid == 0) { tok_s[R] = N; rt.tok_off[R] = N; }
  if (rt.dense_seg_tok_off) {
    const int Gd = (N + kDenseSegRows - 1) / kDenseSegRows;
    for (int g = tid; g <= Gd; g += kRouterThreads) rt.dense_seg_tok_off[g] = min(g * kDenseSegRows, N);
    if (tid == 0) rt.dense_n_segments[0] = Gd;
  }
  __syncthreads();

  // ---- stable LSD radix sort of (tenant id, request) by tenant id
  int cur = 0;
  const int ncnt = 16 * rounds * kWaves;  // <= 1024
  for (int shift = 0; shift < key_bits; shift += 4) {
    for (int i = tid; i < ncnt; i += kRouterThreads) cnt[i] = 0;
    __syncthreads();
    int digit[kRounds], rank[kRounds], k_[kRounds], v_[kRounds];
#pragma unroll
    for (int c = 0; c < kRounds; ++c) {
      digit[c] = -1; rank[c] = 0; k_[c] = 0; v_[c] = 0;
      if (c < rounds) {
        int i = c * kRouterThreads + tid;
        bool valid = i < R;
        if (valid) { k_[c] = key[cur][i]; v_[c] = val[cur][i]; }
        int dg = valid ? ((k_[c] >> shift) & 15) : 0;
        unsigned long long mask = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          bool bit = (dg >> b) & 1;
          unsigned long long bal = __ballot(valid && bit);
          mask &= bit ? bal : ~bal;
        }
        if (valid) {
          digit[c] = dg;
          rank[c] = __popcll(mask & ((1ull << lane) - 1ull));
          if (rank[c] == 0) cnt[dg * (rounds * kWaves) + c * kWaves + w] = __popcll(mask);
        }
      }
    }
    __syncthreads();
    int tot;
    int mine = tid < ncnt ? cnt[tid] : 0;
    int ex = block_exscan(mine, wave_tot, tot);
    if (tid < ncnt) cnt[tid] = ex;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kRounds; ++c) {
      if (c < rounds && digit[c] >= 0) {
        int pos = cnt[digit[c] * (rounds * kWaves) + c * kWaves + w] + rank[c];
        key[cur ^ 1][pos] = k_[c];
        val[cur ^ 1][pos] = v_[c];
      }
    }
    __syncthreads();
    cur ^= 1;
  }
  const int* sid = key[cur];
  const int* perm = val[cur];
  int* slot_s = key[cur ^ 1];   // the sort's spare buffer: request -> HBM slot
#pragma unroll
  for (int c = 0; c < kRounds; ++c) {
    int i = c * kRouterThreads + tid;
    if (c < rounds && i < R) slot_s[i] = slot_r[c];
  }
  __syncthreads();

  // ---- segments (maximal runs of one tenant) and sorted-token offsets
  int seg_carry = 0, tok_carry = 0;
  for (int c = 0; c < rounds; ++c) {
    int p = c * kRouterThreads + tid;
    bool in = p < R;
    int head = in && (p == 0 || sid[p] != sid[p - 1]);
    int len = in ? tok_s[perm[p] + 1] - tok_s[perm[p]] : 0;
    int tot_h, tot_l;
    int g = block_exscan(head, wave_tot, tot_h) + seg_carry;
    int st = block_exscan(len, wave_tot, tot_l) + tok_carry;
    if (in) {
      rt.perm[p] = perm[p];
      stok_s[p] = st;
      if (head) {
        rt.seg_tenant[g] = sid[p];
        rt.seg_slot[g] = slot_s[perm[p]];
        rt.seg_req_off[g] = p;
        rt.seg_tok_off[g] = st;
        segtok_s[g] = st;
      }
    }
    seg_carry += tot_h;
    tok_carry += tot_l;
  }
  const int G = seg_carry;
  if (tid == 0) {
    rt.seg_req_off[G] = R;
    rt.seg_tok_off[G] = N;
    segtok_s[G] = N;
    stok_s[R] = N;
    rt.n_segments[0] = G;
  }
  __syncthreads();

  // ---- m-tile work lists: tiles never straddle a segment
  for (int h = 0; h < 2; ++h) {
    const int tm = rt.tile_m[h];
    if (tm <= 0) continue;
    int tile_carry = 0;
    const int grounds = (G + kRouterThreads - 1) / kRouterThreads;
    for (int c = 0; c < grounds; ++c) {
      int g = c * kRouterThreads + tid;
      int rows = g < G ? segtok_s[g + 1] - segtok_s[g] : 0;
      int nt = (rows + tm - 1) / tm;
      int tot;
      int base = block_exscan(nt, wave_tot, tot) + tile_carry;
      for (int t = 0; t < nt; ++t) {
        rt.tile_seg[h][base + t] = g;
        rt.tile_row0[h][base + t] = segtok_s[g] + t * tm;
      }
      tile_carry += tot;
    }
    if (tid == 0) rt.n_tiles[h][0] = tile_carry;
  }

  // ---- sorted row -> original row, one wavefront per request
  for (int p = w; p < R; p += kWaves) {
    const int src0 = tok_s[perm[p]], dst0 = stok_s[p], len = stok_s[p + 1] - dst0;
    for (int i = lane; i < len; i += 64) rt.row_src[dst0 + i] = src0 + i;
  }
}

}  // namespace

void launch_router(const Route& rt, int R, hipStream_t s) {
  hipLaunchKernelGGL(router_kernel, dim3(1), dim3(kRouterThreads), 0, s, rt, R, rt.key_bits);
}

}  // namespace hmi
