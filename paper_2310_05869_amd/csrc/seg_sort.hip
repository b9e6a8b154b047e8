// Algorithm 1 of the paper, the permutations P_Q and P_K: a stable ascending
// sort of 8-bit bucket codes, independently per segment (one segment per head,
// per node of the causal recursion, and per tensor Q / K).
//
// Keys have at most 256 distinct values, so one counting pass does it.  A
// segment is sorted by one workgroup of 16 waves entirely through LDS:
//   1. wave w histograms its contiguous slice of the segment (LDS atomics on
//      integers);
//   2. the 16 x 256 counters are turned into starting offsets in (bucket, wave)
//      order, which is what makes the sort stable across waves;
//   3. every wave walks its slice again in order, 64 keys at a time; a lane's
//      rank among the equal keys of its 64 is a popcount of a ballot-built peer
//      mask, so equal keys keep their original order inside the wave too.
// Traffic is 2 bytes read and 8 bytes written per key; the stage is latency
// bound, not bandwidth bound, at the sizes of interest.
#include "ha_common.h"

namespace ha {

struct SortArgs {
  const uint8_t* codes_q;
  const uint8_t* codes_k;
  int32_t* perm_q;
  int32_t* perm_k;
  int32_t* pos_k;
  const int32_t* samples;  // node mode: [total_nodes][m] sample indices ...
  int32_t* samp_blk;       // ... and where to put the sorted block of each: [BH][total_nodes][m]
  Geometry g;
  int32_t flat;  // 1: n_seg consecutive segments of seg_len keys in codes_q -> perm_q / pos_k, local indices
  int32_t seg_len;
};

constexpr int kSortWaves = 16;

__global__ __launch_bounds__(kSortWaves * 64) void seg_sort_kernel(SortArgs a) {
  __shared__ uint32_t hist[kSortWaves][256];
  __shared__ uint32_t bucket_base[256];

  const uint8_t* codes;
  int32_t* perm;
  int32_t* pos;
  int s, value_base;
  const int32_t* smp = nullptr;
  int32_t* sblk = nullptr;
  if (a.flat) {
    const int64_t off = (int64_t)blockIdx.x * a.seg_len;
    codes = a.codes_q + off;
    perm = a.perm_q + off;
    pos = a.pos_k + off;
    s = a.seg_len;
    value_base = 0;
  } else {
    const int which = blockIdx.x & 1;  // 0: queries, 1: keys
    const int rest = blockIdx.x >> 1;
    const int heap = rest % a.g.total_nodes;
    const int bh = rest / a.g.total_nodes;
    const int level = 31 - __clz(heap + 1);
    const int node = heap + 1 - (1 << level);
    const NodeRef nr = node_ref(a.g, level, node);
    s = nr.s;
    value_base = which ? nr.k_start : nr.q_start;
    codes = (which ? a.codes_k : a.codes_q) + (int64_t)bh * a.g.n + value_base;
    const int64_t off = ((int64_t)level * a.g.BH + bh) * a.g.n_cov + (int64_t)node * nr.s;
    perm = (which ? a.perm_k : a.perm_q) + off;
    pos = which ? a.pos_k + off : nullptr;
    if (which && a.samples && a.samp_blk && a.g.m > 0) {
      smp = a.samples + (int64_t)heap * a.g.m;
      sblk = a.samp_blk + ((int64_t)bh * a.g.total_nodes + heap) * a.g.m;
    }
  }

  const int tid = threadIdx.x;
  const int w = tid >> 6, lane = tid & 63;
  const int tiles = (s + 63) >> 6;
  const int tpw = (tiles + kSortWaves - 1) / kSortWaves;
  const int t0 = w * tpw;
  const int t1 = min(tiles, t0 + tpw);

  for (int i = tid; i < kSortWaves * 256; i += kSortWaves * 64) (&hist[0][0])[i] = 0;
  __syncthreads();

  for (int t = t0; t < t1; ++t) {
    const int i = t * 64 + lane;
    if (i < s) atomicAdd(&hist[w][codes[i]], 1u);
  }
  __syncthreads();

  // offsets in (bucket, wave) order
  uint32_t total = 0;
  if (tid < 256) {
    for (int ww = 0; ww < kSortWaves; ++ww) {
      const uint32_t v = hist[ww][tid];
      hist[ww][tid] = total;
      total += v;
    }
    bucket_base[tid] = total;
  }
  __syncthreads();
  if (w == 0) {
    uint32_t v[4], sum = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[j] = sum;
      sum += bucket_base[lane * 4 + j];
    }
    uint32_t incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    const uint32_t excl = incl - sum;
#pragma unroll
    for (int j = 0; j < 4; ++j) bucket_base[lane * 4 + j] = excl + v[j];
  }
  __syncthreads();

  for (int t = t0; t < t1; ++t) {
    const int i = t * 64 + lane;
    const bool valid = i < s;
    const uint32_t code = valid ? codes[i] : 0u;
    unsigned long long peers = __ballot(valid);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const bool bit = (code >> k) & 1u;
      const unsigned long long bal = __ballot(bit);
      peers &= bit ? bal : ~bal;
    }
    if (valid) {
      const uint32_t rank = __popcll(peers & ((1ull << lane) - 1ull));
      const uint32_t cnt = __popcll(peers);
      const uint32_t run = hist[w][code];
      const uint32_t dest = bucket_base[code] + run + rank;
      __builtin_amdgcn_wave_barrier();
      if (rank == cnt - 1) hist[w][code] = run + cnt;  // one lane per distinct key
      perm[dest] = value_base + i;
      if (pos) pos[i] = (int32_t)dest;
    }
    __builtin_amdgcn_wave_barrier();
  }

  // Algorithm 2's factor (1 - M_{i,l_j}) only needs the sorted block of each
  // sampled key; record it here, where the key segment's positions are at hand.
  if (sblk) {
    __threadfence_block();
    __syncthreads();
    for (int j = tid; j < a.g.m; j += kSortWaves * 64) sblk[j] = pos[smp[j]] / a.g.b;
  }
}

int launch_seg_sort_nodes(const uint8_t* codes_q, const uint8_t* codes_k, int32_t* perm_q, int32_t* perm_k,
                          int32_t* pos_k, const int32_t* samples, int32_t* samp_blk, const Geometry& g,
                          hipStream_t st) {
  if (g.levels <= 0 || g.total_nodes <= 0) return HA_OK;
  SortArgs a{codes_q, codes_k, perm_q, perm_k, pos_k, samples, samp_blk, g, 0, 0};
  dim3 grid((unsigned)(2 * g.BH * g.total_nodes)), block(kSortWaves * 64);
  hipLaunchKernelGGL(seg_sort_kernel, grid, block, 0, st, a);
  return check_launch();
}

int launch_seg_sort_flat(const uint8_t* codes, int32_t* perm, int32_t* pos, int n_seg, int seg_len,
                         hipStream_t st) {
  if (n_seg <= 0 || seg_len <= 0) return HA_OK;
  SortArgs a{};
  a.codes_q = codes;
  a.perm_q = perm;
  a.pos_k = pos;
  a.flat = 1;
  a.seg_len = seg_len;
  dim3 grid((unsigned)n_seg), block(kSortWaves * 64);
  hipLaunchKernelGGL(seg_sort_kernel, grid, block, 0, st, a);
  return check_launch();
}

}  // namespace ha
