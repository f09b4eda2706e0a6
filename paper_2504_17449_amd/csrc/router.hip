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

// The same for two values at once (one pair of barriers for both).
__device__ __forceinline__ void block_exscan2(int v0, int v1, int* wave_tot, int& ex0, int& ex1, int& total0, int& total1) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int inc0 = wave_incl_scan(v0, lane), inc1 = wave_incl_scan(v1, lane);
  if (lane == 63) { wave_tot[w] = inc0; wave_tot[kWaves + w] = inc1; }
  __syncthreads();
  int base0 = 0, base1 = 0, tot0 = 0, tot1 = 0;
#pragma unroll
  for (int i = 0; i < kWaves; ++i) {
    const int t0 = wave_tot[i], t1 = wave_tot[kWaves + i];
    if (i < w) { base0 += t0; base1 += t1; }
    tot0 += t0; tot1 += t1;
  }
  __syncthreads();
  total0 = tot0; total1 = tot1;
  ex0 = base0 + inc0 - v0; ex1 = base1 + inc1 - v1;
}

__global__ __launch_bounds__(kRouterThreads) void router_kernel(Route rt, int R, int key_bits) {
  __shared__ int key[2][kMaxRequests];
  __shared__ int val[2][kMaxRequests];
  __shared__ int tok_s[kMaxRequests + 1];     // request -> first original row
  __shared__ int stok_s[kMaxRequests + 1];    // sorted position -> first sorted row
  __shared__ int segtok_s[kMaxRequests + 1];  // segment -> first sorted row
  __shared__ int cnt[64 * kRounds * kWaves];   // per digit, round and wavefront: 6-bit digits at most
  __shared__ int wave_tot[2 * kWaves];

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

  // ---- stable LSD radix sort of (tenant id, request) by tenant id: as few passes as digits of at most
  //      6 bits allow (64 tenants: one pass, 1 000: two, 10 000: three), all passes equally wide
  int cur = 0;
  const int passes = (key_bits + 5) / 6;
  const int db = passes > 0 ? (key_bits + passes - 1) / passes : 0;      // bits per digit
  const int stride = rounds * kWaves;                                    // counters per digit value
  const int ncnt = (1 << db) * stride;                                   // <= 2048
  for (int shift = 0; shift < passes * db; shift += db) {
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
        int dg = valid ? ((k_[c] >> shift) & ((1 << db) - 1)) : 0;
        unsigned long long mask = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 6; ++b) {
          if (b < db) {
            bool bit = (dg >> b) & 1;
            unsigned long long bal = __ballot(valid && bit);
            mask &= bit ? bal : ~bal;
          }
        }
        if (valid) {
          digit[c] = dg;
          rank[c] = __popcll(mask & ((1ull << lane) - 1ull));
          if (rank[c] == 0) cnt[dg * stride + c * kWaves + w] = __popcll(mask);
        }
      }
    }
    __syncthreads();
    // exclusive scan over the counters in (digit, round, wavefront) order, two neighbours per lane
    int tot;
    const int c0 = 2 * tid < ncnt ? cnt[2 * tid] : 0, c1 = 2 * tid + 1 < ncnt ? cnt[2 * tid + 1] : 0;
    const int ex = block_exscan(c0 + c1, wave_tot, tot);
    if (2 * tid < ncnt) cnt[2 * tid] = ex;
    if (2 * tid + 1 < ncnt) cnt[2 * tid + 1] = ex + c0;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kRounds; ++c) {
      if (c < rounds && digit[c] >= 0) {
        int pos = cnt[digit[c] * stride + c * kWaves + w] + rank[c];
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
    int tot_h, tot_l, g, st;
    block_exscan2(head, len, wave_tot, g, st, tot_h, tot_l);
    g += seg_carry; st += tok_carry;
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

  // ---- m-tile work lists for both tile heights: tiles never straddle a segment
  {
    const int tm0 = rt.tile_m[0], tm1 = rt.tile_m[1];
    int carry0 = 0, carry1 = 0;
    int* tb0 = key[cur ^ 1];            // segment -> its first tile in list 0 / list 1 (the sort's spare buffers:
    int* tb1 = val[cur ^ 1];            // the slots kept in the first one were last read a barrier ago)
    const int grounds = (G + kRouterThreads - 1) / kRouterThreads;
    for (int c = 0; c < grounds; ++c) {
      const int g = c * kRouterThreads + tid;
      const int first = g < G ? segtok_s[g] : 0;
      const int rows = g < G ? segtok_s[g + 1] - first : 0;
      const int nt0 = tm0 > 0 ? (rows + tm0 - 1) / tm0 : 0, nt1 = tm1 > 0 ? (rows + tm1 - 1) / tm1 : 0;
      int base0, base1, tot0, tot1;
      block_exscan2(nt0, nt1, wave_tot, base0, base1, tot0, tot1);
      if (g < G) { tb0[g] = base0 + carry0; tb1[g] = base1 + carry1; }
      carry0 += tot0; carry1 += tot1;
    }
    if (tid == 0) {
      if (tm0 > 0) rt.n_tiles[0][0] = carry0;
      if (tm1 > 0) rt.n_tiles[1][0] = carry1;
    }
    __syncthreads();
    // one thread per tile, whatever the sizes of the segments (a single tenant's batch is one segment of hundreds of
    // tiles): the tile's segment is the last one whose first tile is not behind it
    for (int k = 0; k < 2; ++k) {
      const int* tb = k == 0 ? tb0 : tb1;
      const int tm = k == 0 ? tm0 : tm1, n = k == 0 ? carry0 : carry1;
      for (int t = tid; t < n; t += kRouterThreads) {
        int lo = 0, hi = G - 1;
        while (lo < hi) {
          const int mid = (lo + hi + 1) >> 1;
          if (tb[mid] <= t) lo = mid; else hi = mid - 1;
        }
        rt.tile_seg[k][t] = lo;
        rt.tile_row0[k][t] = segtok_s[lo] + (t - tb[lo]) * tm;
      }
    }
  }

  // ---- sorted row -> original row.  Wavefront w takes the sorted positions w, w + 16, ...: a lane first fetches
  //      the three numbers of one of them (a dependent chain through LDS, once for 64 positions), then the
  //      wavefront walks over those 64 with the numbers broadcast from that lane's registers.
  for (int base = 0; base < R; base += kWaves * 64) {
    const int myp = base + lane * kWaves + w;
    int src0 = 0, dst0 = 0, len = 0;
    if (myp < R) { src0 = tok_s[perm[myp]]; dst0 = stok_s[myp]; len = stok_s[myp + 1] - dst0; }
    const int mine = min(64, (R - base - w + kWaves - 1) / kWaves);      // positions of this wavefront in this batch of 1024
    for (int l = 0; l < mine; ++l) {
      const int s0 = __builtin_amdgcn_readlane(src0, l), d0 = __builtin_amdgcn_readlane(dst0, l);
      const int n = __builtin_amdgcn_readlane(len, l);
      for (int i = lane; i < n; i += 64) rt.row_src[d0 + i] = s0 + i;
    }
  }
}

}  // namespace

void launch_router(const Route& rt, int R, hipStream_t s) {
  hipLaunchKernelGGL(router_kernel, dim3(1), dim3(kRouterThreads), 0, s, rt, R, rt.key_bits);
}

}  // namespace hmi
