// Work decomposition and key-list construction shared by the MFMA and the
// generic attention kernels.
//
// One workgroup = one tile of QT consecutive sorted query positions inside one
// b-block of one node (node mode), or QT consecutive query rows of one diagonal
// block (exact mode).  In node mode the workgroup attends to ONE list of keys:
//   [0, nb)        the b keys of the block, M^H of Algorithm 1, bias 0
//   [nb, nkeys)    the sampled keys l_j of Algorithm 2 that are NOT in the
//                  row's own block (factor 1 - M_{i,l_j}), bias log(s/m)
// so the block part, the residual estimate and their shared normaliser come out
// of a single softmax pass: sum_block exp(S) + (s/m) sum_kept exp(S).
#pragma once

#include "ha_common.h"

namespace ha {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct TileWork {
  int bh;
  int rows_valid;    // query rows of this tile that exist
  // node mode
  int level, t, p0;  // block index within the node, first sorted position (node-local) of the tile
  NodeRef nr;
  int64_t seg_off;   // offset of the node in perm_q / perm_k / pos_k / part_*
  // exact mode
  int q0;            // first query row (within the head)
  int k0, k1;        // key rows [k0, k1) this tile attends to (before causal masking)
};

// XCD-aware ordering: consecutive workgroup ids are dealt round-robin to the 8
// XCDs, each with its own L2.  Give every XCD a contiguous range of logical
// tiles so that tiles sharing K/V (same block, same node) meet in one L2.
__device__ inline int logical_block(int bid, int total) {
  if (total % 8 != 0) return bid;
  return (bid & 7) * (total >> 3) + (bid >> 3);
}

template <int QT>
__device__ inline TileWork decode_node_tile(const AttnArgs& a, int idx) {
  const Geometry& g = a.g;
  TileWork w{};
  const int tpb = (g.b + QT - 1) / QT;  // tiles per block
  const int tiles_per_level = (g.n_cov / g.b) * tpb;
  const int tile = idx % tiles_per_level;
  const int rest = idx / tiles_per_level;
  w.bh = rest % g.BH;
  w.level = rest / g.BH;
  const int blk = tile / tpb, chunk = tile % tpb;
  const NodeRef probe = node_ref(g, w.level, 0);
  const int bpn = probe.s / g.b;  // blocks per node
  const int node = blk / bpn;
  w.t = blk % bpn;
  w.nr = node_ref(g, w.level, node);
  w.p0 = w.t * g.b + chunk * QT;
  w.rows_valid = min(QT, g.b - chunk * QT);
  w.seg_off = ((int64_t)w.level * g.BH + w.bh) * g.n_cov + (int64_t)node * w.nr.s;
  return w;
}

template <int QT>
__host__ __device__ inline int64_t node_grid(const Geometry& g) {
  const int tpb = (g.b + QT - 1) / QT;
  return (int64_t)g.levels * g.BH * (g.n_cov / g.b) * tpb;
}

template <int QT>
__device__ inline TileWork decode_exact_tile(const AttnArgs& a, int idx) {
  TileWork w{};
  const int eb = a.exact_block;
  const int tpb = (eb + QT - 1) / QT;
  const int nblk = (a.exact_rows_q + eb - 1) / eb;
  // Heavy (late) causal tiles first, and the starting tile rotated from one block to the next: the
  // workgroups of an XCD are dealt to its four shader engines in turn (workgroup i to engine i mod 4,
  // whatever their load), so a fixed order would hand one engine every fourth tile, the heaviest
  // ones, of every block (36 against 30 key tiles on average at 32 tiles per block).
  const int rest = idx / tpb;
  const int qt = tpb - 1 - (idx % tpb + rest) % tpb;
  const int blk = rest % nblk;
  w.bh = rest / nblk;
  w.q0 = blk * eb + qt * QT;
  const int blk_rows = min(eb, a.exact_rows_q - blk * eb);
  w.rows_valid = max(0, min(QT, blk_rows - qt * QT));
  w.k0 = blk * eb;
  w.k1 = min(a.exact_rows_k, (blk + 1) * eb);
  if (a.exact_causal) w.k1 = min(w.k1, w.q0 + w.rows_valid);
  return w;
}

template <int QT>
__host__ __device__ inline int64_t exact_grid(const AttnArgs& a) {
  const int eb = a.exact_block;
  const int tpb = (eb + QT - 1) / QT;
  const int nblk = (a.exact_rows_q + eb - 1) / eb;
  return (int64_t)a.g.BH * nblk * tpb;
}

constexpr int64_t kMaxGrid = 0x7fffffff;  // workgroup ids are decoded as 32-bit integers

// The first index values a thread contributes to the key list (block key `tid`, sample `tid` and
// its sorted block): fetched ahead of the list's construction so that a caller can put other
// loads of the same round trip in flight beside them.
struct KeyListHead {
  int pk0, l0, blk0;
};

template <int NT>
__device__ inline KeyListHead key_list_fetch(const AttnArgs& a, const TileWork& w) {
  const Geometry& g = a.g;
  const int tid = threadIdx.x;
  const int nb = a.use_block ? g.b : 0;
  const int m = (a.samples != nullptr) ? g.m : 0;
  KeyListHead kh{0, 0, 0};
  if (tid < nb) kh.pk0 = a.perm_k ? a.perm_k[w.seg_off + w.t * g.b + tid] : w.nr.k_start + w.t * g.b + tid;
  if (tid < m) {
    kh.l0 = a.samples[(int64_t)w.nr.heap * g.m + tid];
    if (a.samp_blk) kh.blk0 = a.samp_blk[((int64_t)w.bh * g.total_nodes + w.nr.heap) * g.m + tid];
    else kh.blk0 = (a.pos_k ? a.pos_k[w.seg_off + kh.l0] : kh.l0) / g.b;
  }
  return kh;
}

// Builds the key list of a node tile in LDS.  `list` has room for b + m entries
// rounded up to a multiple of 64; `scratch` for (NT/64 + 1) ints.  All NT
// threads call it; on return (after its final barrier) list[0..pad) holds row
// indices within the head, *nb_out the block keys and the return value nkeys.
// `kh` = key_list_fetch's values of the calling thread.
template <int NT>
__device__ inline int build_key_list(const AttnArgs& a, const TileWork& w, int32_t* list, int32_t* scratch,
                                     int* nb_out, const KeyListHead& kh) {
  const Geometry& g = a.g;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  constexpr int NW = NT / 64;
  const int nb = a.use_block ? g.b : 0;
  const int m = (a.samples != nullptr) ? g.m : 0;
  auto block_key = [&](int i) -> int {
    return a.perm_k ? a.perm_k[w.seg_off + w.t * g.b + i] : w.nr.k_start + w.t * g.b + i;
  };
  auto sample_of = [&](int j, int* blk) -> int {
    const int l = a.samples[(int64_t)w.nr.heap * g.m + j];
    if (a.samp_blk) *blk = a.samp_blk[((int64_t)w.bh * g.total_nodes + w.nr.heap) * g.m + j];
    else *blk = (a.pos_k ? a.pos_k[w.seg_off + l] : l) / g.b;
    return l;
  };
  const int pk0 = kh.pk0, l0 = kh.l0, blk0 = kh.blk0;
  if (tid < nb) list[tid] = pk0;
  for (int i = tid + NT; i < nb; i += NT) list[i] = block_key(i);
  int base = nb;
  for (int j0 = 0; j0 < m; j0 += NT) {
    const int j = j0 + tid;
    int l = l0, blk = blk0;
    bool keep = false;
    if (j < m) {
      if (j0 > 0) l = sample_of(j, &blk);
      keep = blk != w.t;  // 1 - M_{i, l_j}: same for every row of the block
    }
    const unsigned long long bal = __ballot(keep);
    if (lane == 0) scratch[wave] = __popcll(bal);
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) {
      const int c = scratch[ww];
      if (ww < wave) before += c;
      total += c;
    }
    if (keep) list[base + before + __popcll(bal & ((1ull << lane) - 1ull))] = w.nr.k_start + l;
    base += total;
    __syncthreads();
  }
  const int nkeys = base;
  const int pad = (nkeys + 63) & ~63;
  for (int i = nkeys + tid; i < pad; i += NT) list[i] = w.nr.k_start;  // loadable, masked by position
  __syncthreads();
  *nb_out = nb;
  return nkeys;
}

template <int NT>
__device__ inline int build_key_list(const AttnArgs& a, const TileWork& w, int32_t* list, int32_t* scratch,
                                     int* nb_out) {
  return build_key_list<NT>(a, w, list, scratch, nb_out, key_list_fetch<NT>(a, w));
}

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  typedef float f2 __attribute__((ext_vector_type(2)));
  const bf2 p = __builtin_convertvector((f2){lo, hi}, bf2);
  return *reinterpret_cast<const uint32_t*>(&p);
}

// One tensor element as fp32 (fp32 tensors as they are, bf16 widened): the kernels without matrix cores.
template <typename T>
__device__ inline float load_elem(const T* p);
template <>
__device__ inline float load_elem<float>(const float* p) { return *p; }
template <>
__device__ inline float load_elem<uint16_t>(const uint16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }

// Where a finished query row goes.
struct RowDest {
  bool valid;
  int64_t out_row;   // row index into out / lse (head offset included), final output
  int64_t part_row;  // row index into part_o / part_l (node mode partial)
  int row_in_head;   // exact mode: for the per-level merge
};

__device__ inline RowDest node_row_dest(const AttnArgs& a, const TileWork& w, int r_in_tile) {
  RowDest d{};
  d.valid = r_in_tile < w.rows_valid;
  const int p = w.p0 + (d.valid ? r_in_tile : 0);
  const int row = (a.scatter_out && a.perm_q) ? a.perm_q[w.seg_off + p] : w.nr.q_start + p;
  d.row_in_head = row;
  d.out_row = (int64_t)w.bh * (a.out_bh_stride / a.g.d) + row;
  d.part_row = w.seg_off + (row - w.nr.q_start);
  return d;
}

// Causal merge (Algorithm 4): the row sum of row i is the base-case row sum
// plus the row sums of the off-diagonal nodes it belongs to.  Level l touches
// row i iff i lies in the second half of its level-l node; *prow is then the
// row's index in part_o / part_l.
__device__ inline bool level_touches(const Geometry& g, int bh, int i, int l, int64_t* prow) {
  const int s = g.n >> (l + 1);
  *prow = ((int64_t)l * g.BH + bh) * g.n_cov + (int64_t)(i / (2 * s)) * s + (i % s);
  return ((i / s) & 1) != 0;
}

// Combined log row sum of the base-case result (lse_own) and the partials;
// *mx_out is the reference the weights exp(l - mx) / den are taken against.
__device__ inline float merged_lse(const AttnArgs& a, int bh, int i, float lse_own, float* mx_out,
                                   float* den_out) {
  float mx = lse_own;
  for (int l = 0; l < a.merge_levels; ++l) {
    int64_t pr;
    if (level_touches(a.g, bh, i, l, &pr)) mx = fmaxf(mx, a.part_l[pr]);
  }
  if (mx == -INFINITY) {
    *mx_out = 0.f;
    *den_out = 1.f;
    return -INFINITY;
  }
  float den = expf(lse_own - mx);
  for (int l = 0; l < a.merge_levels; ++l) {
    int64_t pr;
    if (level_touches(a.g, bh, i, l, &pr)) den += expf(a.part_l[pr] - mx);
  }
  *mx_out = mx;
  *den_out = den;
  return mx + logf(den);
}

}  // namespace ha
