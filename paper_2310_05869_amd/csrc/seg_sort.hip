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
// Traffic is 2 bytes read and 8 bytes written per key.
//
// Long segments (the upper levels of the causal recursion have 64 segments of
// 65536 keys) would leave most of the chip idle, so the forward pass sorts in
// chunks of kChunk keys, one workgroup each, in two launches:
//   A. every chunk's bucket counts go to a table in the workspace;
//   B. every chunk recounts per wave, finds where its buckets start (buckets
//      before it in the segment + the same bucket in earlier chunks) and
//      scatters, with the same in-wave ranking: the result is the same stable
//      order, whatever the chunking.
// A third small launch records the sorted block of every sampled key.
#include "ha_common.h"

namespace ha {

constexpr int kSortMaxLevels = 24;
constexpr int kChunk = 4096;  // keys per workgroup in the chunked passes

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
  // chunked node mode: bucket counts of every chunk, and the first workgroup of every level
  uint32_t* chunk_hist;   // [chunks][256]
  int32_t phase;          // 0: whole segments (one launch); 1: count chunks; 2: scatter chunks
  int32_t lvl_wg[kSortMaxLevels + 1];
};

constexpr int kFlatWaves = 16;   // whole-segment mode: one workgroup has to cover a long segment
constexpr int kChunkWaves = 4;   // chunked mode: many small workgroups per CU hide each other's barriers

template <int kSortWaves>
__global__ __launch_bounds__(kSortWaves * 64) void seg_sort_kernel(SortArgs a) {
  __shared__ uint32_t hist[kSortWaves][256];
  __shared__ uint32_t bucket_base[256];
  // chunked scatter: the chunk is first ordered inside LDS, then written out in that order, so
  // that a wave's 64 stores fall into a few runs of consecutive entries instead of 64 places
  constexpr bool kStaged = (kSortWaves == kChunkWaves);
  __shared__ uint32_t lbase[kStaged ? 256 : 1];        // where each bucket starts inside the chunk
  __shared__ int32_t staged[kStaged ? kChunk : 1];
  __shared__ uint8_t scode[kStaged ? kChunk : 1];

  const uint8_t* codes;
  int32_t* perm;
  int32_t* pos;
  int s, value_base;
  const int32_t* smp = nullptr;
  int32_t* sblk = nullptr;
  int chunk = 0, nchunks = 1, chunk_off = 0;
  uint32_t* seg_hist = nullptr;  // chunked: bucket counts of this segment's chunks [nchunks][256]
  if (a.flat) {
    const int64_t off = (int64_t)blockIdx.x * a.seg_len;
    codes = a.codes_q + off;
    perm = a.perm_q + off;
    pos = a.pos_k + off;
    s = a.seg_len;
    value_base = 0;
  } else if (a.phase == 0) {
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
  } else {
    // chunked: workgroups ordered (level, head, node, tensor, chunk); a segment's chunks are consecutive
    int level = 0, wg0 = 0;
#pragma unroll
    for (int l = 0; l < kSortMaxLevels; ++l)
      if (l < a.g.levels && (int)blockIdx.x >= a.lvl_wg[l]) {
        level = l;
        wg0 = a.lvl_wg[l];
      }
    const NodeRef probe = node_ref(a.g, level, 0);
    nchunks = (probe.s + kChunk - 1) / kChunk;
    const int nodes = a.g.causal ? (1 << level) : 1;
    int idx = (int)blockIdx.x - wg0;
    chunk = idx % nchunks;
    idx /= nchunks;
    const int which = idx & 1;
    idx >>= 1;
    const int node = idx % nodes;
    const int bh = idx / nodes;
    const NodeRef nr = node_ref(a.g, level, node);
    chunk_off = chunk * kChunk;
    s = min(kChunk, nr.s - chunk_off);
    value_base = (which ? nr.k_start : nr.q_start) + chunk_off;
    codes = (which ? a.codes_k : a.codes_q) + (int64_t)bh * a.g.n + value_base;
    const int64_t off = ((int64_t)level * a.g.BH + bh) * a.g.n_cov + (int64_t)node * nr.s;
    perm = (which ? a.perm_k : a.perm_q) + off;          // destinations are segment-wide
    pos = which ? a.pos_k + off + chunk_off : nullptr;    // sources are this chunk's
    seg_hist = a.chunk_hist + ((int64_t)blockIdx.x - chunk) * 256;
  }

  const int tid = threadIdx.x;
  const int w = tid >> 6, lane = tid & 63;
  const int tiles = (s + 63) >> 6;
  const int tpw = (tiles + kSortWaves - 1) / kSortWaves;
  const int t0 = w * tpw;
  const int t1 = min(tiles, t0 + tpw);

  for (int i = tid; i < kSortWaves * 256; i += kSortWaves * 64) (&hist[0][0])[i] = 0;
  __syncthreads();

  // keys are fetched eight tiles at a time, so that their loads are in flight together
  constexpr int kAhead = 8;
  for (int tb = t0; tb < t1; tb += kAhead) {
    uint32_t cv[kAhead];
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      const int i = (tb + u) * 64 + lane;
      cv[u] = (tb + u < t1 && i < s) ? codes[i] : 0xFFFFFFFFu;
    }
#pragma unroll
    for (int u = 0; u < kAhead; ++u)
      if (cv[u] != 0xFFFFFFFFu) atomicAdd(&hist[w][cv[u]], 1u);
  }
  __syncthreads();

  // offsets in (bucket, wave) order
  uint32_t total = 0;
  uint32_t before = 0;  // chunked: keys of this bucket in earlier chunks of the segment
  if (tid < 256) {
    for (int ww = 0; ww < kSortWaves; ++ww) {
      const uint32_t v = hist[ww][tid];
      hist[ww][tid] = total;
      total += v;
    }
    if (a.phase == 1) {
      seg_hist[chunk * 256 + tid] = total;
    } else if (a.phase == 2) {
      uint32_t all = 0;
      for (int c = 0; c < nchunks; ++c) {
        const uint32_t v = seg_hist[c * 256 + tid];
        if (c < chunk) before += v;
        all += v;
      }
      if (kStaged) lbase[tid] = total;  // the bucket's size in this chunk
      total = all;                      // the bucket's size in the whole segment
    }
    bucket_base[tid] = total;
  }
  if (a.phase == 1) return;
  __syncthreads();
  // exclusive prefix sums over the 256 buckets, one wave per array
  auto scan256 = [&](uint32_t* arr) {
    uint32_t v[4], sum = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[j] = sum;
      sum += arr[lane * 4 + j];
    }
    uint32_t incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    const uint32_t excl = incl - sum;
#pragma unroll
    for (int j = 0; j < 4; ++j) arr[lane * 4 + j] = excl + v[j];
  };
  if (w == 0) scan256(bucket_base);
  if (kStaged && a.phase == 2 && w == 1) scan256(lbase);
  __syncthreads();
  if (a.phase == 2 && tid < 256) bucket_base[tid] += before;
  __syncthreads();

  for (int tb = t0; tb < t1; tb += kAhead) {
    uint32_t cv[kAhead];
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      const int i = (tb + u) * 64 + lane;
      cv[u] = (tb + u < t1 && i < s) ? codes[i] : 0xFFFFFFFFu;
    }
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      if (tb + u >= t1) break;
      const int i = (tb + u) * 64 + lane;
      const bool valid = cv[u] != 0xFFFFFFFFu;
      const uint32_t code = valid ? cv[u] : 0u;
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
        if (kStaged && a.phase == 2) {
          const uint32_t lr = lbase[code] + run + rank;  // place inside the chunk's own order
          staged[lr] = value_base + i;
          scode[lr] = (uint8_t)code;
        } else {
          perm[dest] = value_base + i;
        }
        if (pos) pos[i] = (int32_t)dest;  // (chunked: pos points at this chunk's rows, dest is segment-wide)
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
  if (kStaged && a.phase == 2) {
    __syncthreads();
    for (int j = tid; j < s; j += kSortWaves * 64) {
      const uint32_t c = scode[j];
      perm[bucket_base[c] + ((uint32_t)j - lbase[c])] = staged[j];
    }
  }

  // Algorithm 2's factor (1 - M_{i,l_j}) only needs the sorted block of each
  // sampled key; record it here, where the key segment's positions are at hand.
  if (sblk) {
    __threadfence_block();
    __syncthreads();
    for (int j = tid; j < a.g.m; j += kSortWaves * 64) sblk[j] = pos[smp[j]] / a.g.b;
  }
}

// Algorithm 2's factor (1 - M_{i,l_j}): the sorted block of every sampled key, one workgroup per (head, node).
__global__ __launch_bounds__(256) void sample_block_kernel(const int32_t* __restrict__ pos_k, const int32_t* __restrict__ samples,
                                                           int32_t* __restrict__ samp_blk, Geometry g) {
  const int heap = blockIdx.x % g.total_nodes;
  const int bh = blockIdx.x / g.total_nodes;
  const int level = 31 - __clz(heap + 1);
  const int node = heap + 1 - (1 << level);
  const NodeRef nr = node_ref(g, level, node);
  const int64_t off = ((int64_t)level * g.BH + bh) * g.n_cov + (int64_t)node * nr.s;
  for (int j = threadIdx.x; j < g.m; j += blockDim.x)
    samp_blk[((int64_t)bh * g.total_nodes + heap) * g.m + j] = pos_k[off + samples[(int64_t)heap * g.m + j]] / g.b;
}

int64_t seg_sort_chunks(const Geometry& g) {
  int64_t chunks = 0;
  for (int l = 0; l < g.levels; ++l) {
    const int s = g.causal ? (g.n >> (l + 1)) : g.n;
    const int nodes = g.causal ? (1 << l) : 1;
    chunks += (int64_t)2 * g.BH * nodes * ((s + kChunk - 1) / kChunk);
  }
  return chunks;
}

int launch_seg_sort_nodes(const uint8_t* codes_q, const uint8_t* codes_k, int32_t* perm_q, int32_t* perm_k,
                          int32_t* pos_k, const int32_t* samples, int32_t* samp_blk, uint32_t* chunk_hist,
                          const Geometry& g, hipStream_t st) {
  if (g.levels <= 0 || g.total_nodes <= 0) return HA_OK;
  if (g.levels > kSortMaxLevels) return HA_ERR_SHAPE;
  SortArgs a{};
  a.codes_q = codes_q;
  a.codes_k = codes_k;
  a.perm_q = perm_q;
  a.perm_k = perm_k;
  a.pos_k = pos_k;
  a.g = g;
  a.chunk_hist = chunk_hist;
  int wg = 0;
  for (int l = 0; l < g.levels; ++l) {
    const int s = g.causal ? (g.n >> (l + 1)) : g.n;
    const int nodes = g.causal ? (1 << l) : 1;
    a.lvl_wg[l] = wg;
    wg += 2 * g.BH * nodes * ((s + kChunk - 1) / kChunk);
  }
  a.lvl_wg[g.levels] = wg;
  dim3 grid((unsigned)wg), block(kChunkWaves * 64);
  a.phase = 1;
  hipLaunchKernelGGL(seg_sort_kernel<kChunkWaves>, grid, block, 0, st, a);
  a.phase = 2;
  hipLaunchKernelGGL(seg_sort_kernel<kChunkWaves>, grid, block, 0, st, a);
  if (samples && samp_blk && g.m > 0)
    hipLaunchKernelGGL(sample_block_kernel, dim3((unsigned)(g.BH * g.total_nodes)), dim3(256), 0, st, pos_k, samples,
                       samp_blk, g);
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
  dim3 grid((unsigned)n_seg), block(kFlatWaves * 64);
  hipLaunchKernelGGL(seg_sort_kernel<kFlatWaves>, grid, block, 0, st, a);
  return check_launch();
}

}  // namespace ha
