// Algorithm 1 of the paper, the permutations P_Q and P_K: a stable ascending
// sort of 8-bit bucket codes, independently per segment (one segment per head,
// per node of the causal recursion, and per tensor Q / K).
//
// Keys have at most 256 distinct values, so one counting pass does it.
//
// Whole-segment kernel (the single-stage entry point): a segment is sorted by
// one workgroup of 16 waves entirely through LDS:
//   1. wave w histograms its contiguous slice of the segment (LDS atomics on
//      integers);
//   2. the 16 x 256 counters are turned into starting offsets in (bucket, wave)
//      order, which is what makes the sort stable across waves;
//   3. every wave walks its slice again in order, 64 keys at a time; a lane's
//      rank among the equal keys of its 64 is a popcount of a ballot-built peer
//      mask, so equal keys keep their original order inside the wave too.
//
// Long segments (the upper levels of the causal recursion have 64 segments of
// 65536 keys) would leave most of the chip idle, so the forward pass sorts in
// chunks of kChunk keys, one 4-wave workgroup each, in two launches:
//   A. every chunk's bucket counts go to a table in the workspace;
//   B. every chunk finds where its buckets start (buckets before it in the
//      segment + the same bucket in earlier chunks), ranks its keys and
//      scatters: the result is the same stable order, whatever the chunking.
// In B the peer mask of a key comes from LDS rather than from ballots: the
// lanes of a 64-key tile OR their lane bit into a 64-bit word per (wave,
// bucket) and read the word back; a counter per (wave, bucket) carries the
// number of the wave's earlier keys of the bucket, and ends up as the wave's
// bucket count, so no separate counting walk is needed.  Mask and counter
// arrays are packed (8 and 4 bytes per bucket): wider slots would put the 2^r
// buckets on a quarter of the LDS banks.  The chunk is first ordered inside LDS
// and then written out in that order, so a wave's 64 stores fall into a few
// runs of consecutive entries.  B also records the sorted block of every sampled key
// (the factor 1 - M_{i,l_j} of Algorithm 2 needs nothing else).
// Traffic per key: 1 byte read in each pass, 4 bytes written (the permutation) for queries and
// 8 (permutation and position) for keys.
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
  const int32_t* samples;  // chunked: [total_nodes][m] sample indices ...
  int32_t* samp_blk;       // ... and where to put the sorted block of each: [BH][total_nodes][m]
  Geometry g;
  int32_t seg_len;         // whole-segment mode: consecutive segments of seg_len keys in codes_q -> perm_q / pos_k
  // chunked mode: bucket counts of every chunk, and the first workgroup of every level
  uint32_t* chunk_hist;    // [chunks][256]
  int32_t lvl_wg[kSortMaxLevels + 1];
};

constexpr int kFlatWaves = 16;   // whole-segment mode: one workgroup has to cover a long segment
constexpr int kChunkWaves = 4;   // chunked mode: many small workgroups per CU hide each other's barriers

__global__ __launch_bounds__(kFlatWaves * 64) void seg_sort_kernel(SortArgs a) {
  constexpr int kSortWaves = kFlatWaves;
  __shared__ uint32_t hist[kSortWaves][256];
  __shared__ uint32_t bucket_base[256];

  const int64_t off = (int64_t)blockIdx.x * a.seg_len;
  const uint8_t* codes = a.codes_q + off;
  int32_t* perm = a.perm_q + off;
  int32_t* pos = a.pos_k + off;
  const int s = a.seg_len;

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
  if (tid < 256) {
    uint32_t total = 0;
    for (int ww = 0; ww < kSortWaves; ++ww) {
      const uint32_t v = hist[ww][tid];
      hist[ww][tid] = total;
      total += v;
    }
    bucket_base[tid] = total;
  }
  __syncthreads();
  if (w == 0) {  // exclusive prefix sums over the 256 buckets
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
        perm[dest] = i;
        pos[i] = (int32_t)dest;
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// ---------------------------------------------------------------------------
// Chunked passes.
// ---------------------------------------------------------------------------
struct ChunkRef {
  const uint8_t* codes;  // the chunk's keys
  int32_t* perm;         // the segment's permutation (destinations are segment-wide)
  int32_t* pos;          // the chunk's slice of pos_k, or null (queries)
  const uint32_t* seg_hist;  // bucket counts of the segment's chunks [nchunks][256]
  uint32_t* own_hist;        // this chunk's row of that table
  const int32_t* smp;    // key chunks with samples: the node's sample indices ...
  int32_t* sblk;         // ... and where the sorted block of each goes
  int s, value_base, chunk, nchunks, chunk_off;
};

// workgroups are ordered (level, head, node, tensor, chunk); a segment's chunks are consecutive
__device__ inline ChunkRef decode_chunk(const SortArgs& a, int wg) {
  ChunkRef c{};
  int level = 0, wg0 = 0;
#pragma unroll
  for (int l = 0; l < kSortMaxLevels; ++l)
    if (l < a.g.levels && wg >= a.lvl_wg[l]) {
      level = l;
      wg0 = a.lvl_wg[l];
    }
  const NodeRef probe = node_ref(a.g, level, 0);
  c.nchunks = (probe.s + kChunk - 1) / kChunk;
  const int nodes = a.g.causal ? (1 << level) : 1;
  int idx = wg - wg0;
  c.chunk = idx % c.nchunks;
  idx /= c.nchunks;
  const int which = idx & 1;  // 0: queries, 1: keys
  idx >>= 1;
  const int node = idx % nodes;
  const int bh = idx / nodes;
  const NodeRef nr = node_ref(a.g, level, node);
  c.chunk_off = c.chunk * kChunk;
  c.s = min(kChunk, nr.s - c.chunk_off);
  c.value_base = (which ? nr.k_start : nr.q_start) + c.chunk_off;
  c.codes = (which ? a.codes_k : a.codes_q) + (int64_t)bh * a.g.n + c.value_base;
  const int64_t off = ((int64_t)level * a.g.BH + bh) * a.g.n_cov + (int64_t)node * nr.s;
  c.perm = (which ? a.perm_k : a.perm_q) + off;
  c.pos = which ? a.pos_k + off + c.chunk_off : nullptr;
  uint32_t* seg = a.chunk_hist + ((int64_t)wg - c.chunk) * 256;
  c.seg_hist = seg;
  c.own_hist = seg + (int64_t)c.chunk * 256;
  if (which && a.samples && a.samp_blk && a.g.m > 0) {
    c.smp = a.samples + (int64_t)nr.heap * a.g.m;
    c.sblk = a.samp_blk + ((int64_t)bh * a.g.total_nodes + nr.heap) * a.g.m;
  }
  return c;
}

// Thread t of the workgroup fetches keys [16 t, 16 t + 16) of the chunk: one
// 16-byte load where the address allows it.  Keys past the chunk's end read as 0.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ inline u32x4 load_16_codes(const uint8_t* codes, int s, int t) {
  const int i0 = 16 * t;
  u32x4 v = {0, 0, 0, 0};
  if (i0 + 16 <= s && (reinterpret_cast<uintptr_t>(codes) & 15u) == 0) {
    v = *reinterpret_cast<const u32x4*>(codes + i0);
  } else {
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (i0 + j < s) v[j >> 2] |= (uint32_t)codes[i0 + j] << (8 * (j & 3));
  }
  return v;
}

// Pass A: the chunk's bucket counts.
__global__ __launch_bounds__(kChunkWaves * 64) void chunk_count_kernel(SortArgs a) {
  __shared__ uint32_t hist[256];
  const ChunkRef c = decode_chunk(a, (int)blockIdx.x);
  const int tid = threadIdx.x;
  const u32x4 v = load_16_codes(c.codes, c.s, tid);
  hist[tid] = 0;
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 16; ++j)
    if (16 * tid + j < c.s) atomicAdd(&hist[(v[j >> 2] >> (8 * (j & 3))) & 255u], 1u);
  __syncthreads();
  c.own_hist[tid] = hist[tid];
}

constexpr int kTilesPerWave = kChunk / 64 / kChunkWaves;

// LDS of pass B: the chunk's order (kChunk words, whose first quarter holds the keys
// until they are in registers), wave totals, and per (wave, bucket) a 64-bit peer
// mask (later the pair {first place, shift to the destination}) and a counter.
__host__ __device__ inline size_t chunk_scatter_lds(int nbk) {
  return (size_t)kChunk * 4 + 64 + (size_t)kChunkWaves * nbk * 12;
}

// Pass B.  nbk = number of buckets (a power of two >= every code + 1, at most 256).
__global__ __launch_bounds__(kChunkWaves * 64) void chunk_scatter_kernel(SortArgs a, int nbk) {
  extern __shared__ __attribute__((aligned(16))) unsigned char sm[];
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  uint32_t* staged = reinterpret_cast<uint32_t*>(sm);
  const uint8_t* codes_lds = sm;
  uint32_t* wave_tot = staged + kChunk;  // [2][kChunkWaves]
  unsigned long long* peers = reinterpret_cast<unsigned long long*>(wave_tot + 16);  // [kChunkWaves][nbk]
  u32x2* first = reinterpret_cast<u32x2*>(peers);                                    // the same words, after the ranking
  uint32_t* count = reinterpret_cast<uint32_t*>(peers + kChunkWaves * nbk);          // [kChunkWaves][nbk]

  const ChunkRef c = decode_chunk(a, (int)blockIdx.x);
  const int tid = threadIdx.x;
  const int w = tid >> 6, lane = tid & 63;
  const int s = c.s;

  // the bucket's keys in earlier chunks of the segment, and in the whole segment
  uint32_t before = 0, all = 0;
  if (tid < nbk) {
    for (int c0 = 0; c0 < c.nchunks; c0 += 8) {
      uint32_t v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = (c0 + u < c.nchunks) ? c.seg_hist[(int64_t)(c0 + u) * 256 + tid] : 0u;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        all += v[u];
        if (c0 + u < c.chunk) before += v[u];
      }
    }
  }
  {
    const u32x4 v = load_16_codes(c.codes, s, tid);
    *reinterpret_cast<u32x4*>(sm + 16 * tid) = v;
    for (int i = tid; i < kChunkWaves * nbk; i += kChunkWaves * 64) {
      peers[i] = 0ull;
      count[i] = 0u;
    }
  }
  __syncthreads();

  // Wave w ranks tiles [w kTilesPerWave, (w + 1) kTilesPerWave) of the chunk, in order:
  // a key's place among the wave's keys of its bucket = keys of the bucket in the wave's
  // earlier tiles (the counter) + lanes below it in its tile that hold the bucket too.
  // Afterwards the counters hold the wave's bucket counts.
  uint32_t cr[kTilesPerWave];  // bucket | place among the wave's keys of the bucket << 8
  unsigned long long* my_peers = peers + w * nbk;
  uint32_t* my_count = count + w * nbk;
  const unsigned long long lane_bit = 1ull << lane;
#pragma unroll
  for (int u = 0; u < kTilesPerWave; ++u) cr[u] = codes_lds[(w * kTilesPerWave + u) * 64 + lane] & (uint32_t)(nbk - 1);
#pragma unroll
  for (int u = 0; u < kTilesPerWave; ++u) {
    const int i = (w * kTilesPerWave + u) * 64 + lane;
    if (i < s) {
      const uint32_t code = cr[u];
      atomicOr(&my_peers[code], lane_bit);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      const unsigned long long pm = my_peers[code];  // after every lane's OR: LDS operations of a wave complete in order
      const uint32_t seen = my_count[code];
      const uint32_t rank = __popcll(pm & (lane_bit - 1ull));
      const uint32_t cnt = __popcll(pm);
      cr[u] = code | ((seen + rank) << 8);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (rank == cnt - 1) {  // one lane per distinct key
        my_peers[code] = 0ull;
        my_count[code] = seen + cnt;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  __syncthreads();

  // first places in (bucket, wave) order: exclusive sums over the buckets of the
  // chunk's counts (place inside the chunk) and of the segment's counts (destination)
  uint32_t cnt_w[kChunkWaves], mine = 0;
  if (tid < nbk) {
#pragma unroll
    for (int ww = 0; ww < kChunkWaves; ++ww) {
      cnt_w[ww] = count[ww * nbk + tid];
      mine += cnt_w[ww];
    }
  }
  uint32_t inc_l = mine, inc_g = all;  // contributions of tid >= nbk are zero
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t ul = __shfl_up(inc_l, o), ug = __shfl_up(inc_g, o);
    if (lane >= o) {
      inc_l += ul;
      inc_g += ug;
    }
  }
  if (lane == 63) {
    wave_tot[w] = inc_l;
    wave_tot[kChunkWaves + w] = inc_g;
  }
  __syncthreads();
  if (tid < nbk) {
    uint32_t lb = inc_l - mine, gb = inc_g - all + before;
#pragma unroll
    for (int ww = 0; ww < kChunkWaves; ++ww)
      if (ww < w) {
        lb += wave_tot[ww];
        gb += wave_tot[kChunkWaves + ww];
      }
    const uint32_t shift = gb - lb;  // destination in the segment = place in the chunk + shift (mod 2^32)
#pragma unroll
    for (int ww = 0; ww < kChunkWaves; ++ww) {
      first[ww * nbk + tid] = (u32x2){lb, shift};
      lb += cnt_w[ww];
    }
  }
  __syncthreads();  // (also: every wave has its keys in registers, the first quarter of `staged` is free)

  // the chunk in its own sorted order: bucket << 12 | index within the chunk
#pragma unroll
  for (int u = 0; u < kTilesPerWave; ++u) {
    const int i = (w * kTilesPerWave + u) * 64 + lane;
    if (i < s) {
      const uint32_t code = cr[u] & 255u;
      const u32x2 f = first[w * nbk + code];
      const uint32_t place = f.x + (cr[u] >> 8);
      staged[place] = (code << 12) | (uint32_t)i;
      if (c.pos) c.pos[i] = (int32_t)(place + f.y);
    }
  }
  __syncthreads();
  for (int j = tid; j < s; j += kChunkWaves * 64) {
    const uint32_t v = staged[j];
    c.perm[(uint32_t)j + first[v >> 12].y] = c.value_base + (int32_t)(v & (kChunk - 1));
  }

  // the sorted block of the node's sampled keys that fall into this chunk
  if (c.sblk) {
    __threadfence_block();  // the positions were stored by other threads of this workgroup
    __syncthreads();
    for (int j = tid; j < a.g.m; j += kChunkWaves * 64) {
      const int l = c.smp[j] - c.chunk_off;
      if (l >= 0 && l < s)
        c.sblk[j] = __hip_atomic_load(&c.pos[l], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) / a.g.b;
    }
  }
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
  if (g.levels > kSortMaxLevels || g.r < 1 || g.r > 8) return HA_ERR_SHAPE;
  SortArgs a{};
  a.codes_q = codes_q;
  a.codes_k = codes_k;
  a.perm_q = perm_q;
  a.perm_k = perm_k;
  a.pos_k = pos_k;
  a.samples = samples;
  a.samp_blk = samp_blk;
  a.g = g;
  a.chunk_hist = chunk_hist;
  int64_t wg = 0;
  for (int l = 0; l < g.levels; ++l) {
    const int s = g.causal ? (g.n >> (l + 1)) : g.n;
    const int nodes = g.causal ? (1 << l) : 1;
    a.lvl_wg[l] = (int32_t)wg;
    wg += (int64_t)2 * g.BH * nodes * ((s + kChunk - 1) / kChunk);
    if (wg > 0x7fffffff) return HA_ERR_SHAPE;
  }
  a.lvl_wg[g.levels] = (int32_t)wg;
  const int nbk = 1 << g.r;  // bucket codes of Definition 1 are below 2^r
  dim3 grid((unsigned)wg), block(kChunkWaves * 64);
  hipLaunchKernelGGL(chunk_count_kernel, grid, block, 0, st, a);
  hipLaunchKernelGGL(chunk_scatter_kernel, grid, block, chunk_scatter_lds(nbk), st, a, nbk);
  return check_launch();
}

int launch_seg_sort_flat(const uint8_t* codes, int32_t* perm, int32_t* pos, int n_seg, int seg_len,
                         hipStream_t st) {
  if (n_seg <= 0 || seg_len <= 0) return HA_OK;
  SortArgs a{};
  a.codes_q = codes;
  a.perm_q = perm;
  a.pos_k = pos;
  a.seg_len = seg_len;
  dim3 grid((unsigned)n_seg), block(kFlatWaves * 64);
  hipLaunchKernelGGL(seg_sort_kernel, grid, block, 0, st, a);
  return check_launch();
}

}  // namespace ha
