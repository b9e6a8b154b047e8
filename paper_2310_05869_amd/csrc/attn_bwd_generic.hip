// Backward pass without matrix cores: the arithmetic path for HA_FP32 tensors (every product and
// sum an fp32 FMA), with the same five passes, the same work decomposition and the same outputs as
// the bf16 MFMA backward kernel, so that the host sequence is one and the same.
//
// As there, a row of the forward is one softmax over its block keys, its kept sampled keys (weight
// s/m) and, when causal, the keys of its base-case block (Algorithms 1, 2, 4), and with the final
// log row sum L_i and delta_i = <dO_i, O_i> every (query, key) pair contributes on its own:
//   P_ij = w_ij exp(<q_i, k_j> - L_i),  dV_j += P_ij dO_i,  dS_ij = P_ij (<dO_i, v_j> - delta_i),
//   dQ_i += dS_ij k_j,  dK_j += dS_ij q_i.
//
// Two neighbouring lanes own one "R row" (a query in the dQ passes, a key in the dK / dV passes), half of
// its columns each: their halves of the row, of the operand of dP and of the accumulator live in
// registers, and a dot product is the sum of the two lanes' partial sums.  The "T rows" (keys, resp.
// queries) pass through LDS as fp32 tiles of 16 rows that the lanes read at two addresses (LDS broadcast).
// The dK / dV passes run twice (dK, then dV), one accumulator row each.
#include "attn_common.h"
#include "bwd_common.h"

namespace ha {

constexpr int kGRT = 128;       // R rows per workgroup: the decomposition of the MFMA backward kernel
constexpr int kGNT = 2 * kGRT;  // threads
constexpr int kGTT = 16;        // T rows per step

__host__ __device__ inline size_t bwd_generic_lds_bytes(const Geometry& g, int d, int mode) {
  size_t s = (size_t)2 * kGTT * d * 4 + 2 * kGTT * 4 + 64;
  if (mode == kBwdDqNode) s += (size_t)(((g.b + g.m + 63) & ~63) + 64) * 4;
  return s;
}

template <typename T, int C>
__device__ inline void store_cols(T* dst, const float (&v)[C]) {
  if constexpr (sizeof(T) == 4) {
#pragma unroll
    for (int c = 0; c < C; c += 4)
      *reinterpret_cast<float4*>(reinterpret_cast<float*>(dst) + c) = make_float4(v[c], v[c + 1], v[c + 2], v[c + 3]);
  } else {
#pragma unroll
    for (int c = 0; c < C; c += 4) {
      uint2 p;
      p.x = pack_bf16x2(v[c], v[c + 1]);
      p.y = pack_bf16x2(v[c + 2], v[c + 3]);
      *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(dst) + c) = p;
    }
  }
}

// WANT_DS: accumulate dS products (dQ, or dK); otherwise P products (dV).
template <typename T, int D, int MODE, bool WANT_DS>
__global__ __launch_bounds__(kGNT) void attn_bwd_generic_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr bool kDq = (MODE == kBwdDqNode || MODE == kBwdDqExact);
  constexpr bool kExact = (MODE == kBwdDqExact || MODE == kBwdDkvExact);
  constexpr bool kSorted = (MODE == kBwdDkvBlock || MODE == kBwdDkvSamp);
  static_assert(WANT_DS || !kDq, "the dQ passes accumulate dS only");
  float* Ys = reinterpret_cast<float*>(smem);          // T rows: operand of the scores
  float* Bs = Ys + kGTT * D;                           // T rows: operand of dP (dQ passes: V) or of dV (dO)
  float* scl = Bs + kGTT * D;                          // dK / dV passes: L and delta of the T rows
  float* scd = scl + kGTT;
  int32_t* scratch = reinterpret_cast<int32_t*>(scd + kGTT);
  int32_t* list = scratch + 16;

  const AttnArgs& f = a.f;
  const Geometry& g = f.g;
  const int tid = threadIdx.x;
  const int r_in_tile = tid >> 1;          // this lane's R row within the workgroup's 128
  constexpr int C = D / 2;                 // columns per lane
  const int c0 = (tid & 1) * C;            // first of them

  // ---- which part of the problem this workgroup owns (as in the MFMA kernel) ----
  TileWork w{};
  int chunk_start = 0, chunk_len = 0, samp0 = 0, cpn_w = 0, qc_w = 0;
  int64_t samp_row0 = 0;
  int t0 = 0;
  if (MODE == kBwdDqNode || MODE == kBwdDkvBlock) {
    w = decode_node_tile<kGRT>(f, a.wg_base + blockIdx.x);
  } else if (MODE == kBwdDqExact) {
    w = decode_exact_tile<kGRT>(f, blockIdx.x);
  } else if (MODE == kBwdDkvExact) {
    const int eb = f.exact_block;
    const int tpb = (eb + kGRT - 1) / kGRT;
    const int nblk = (f.exact_rows_q + eb - 1) / eb;
    const int idx = blockIdx.x;
    const int ktile = idx % tpb;
    const int rest = idx / tpb;
    const int blk = rest % nblk;
    w.bh = rest / nblk;
    w.q0 = blk * eb + ktile * kGRT;  // first KEY row of this tile
    const int blk_rows = min(eb, f.exact_rows_q - blk * eb);
    w.rows_valid = max(0, min(kGRT, blk_rows - ktile * kGRT));
    t0 = f.exact_causal ? w.q0 : blk * eb;
    w.k0 = t0;
    w.k1 = blk * eb + blk_rows;      // queries [t0, k1)
  } else {  // kBwdDkvSamp: a slab of sampled keys over one chunk of the node's sorted queries
    const int sbid = blockIdx.x;
    int level = 0, wg0 = 0;
    int64_t srow0 = 0;
#pragma unroll
    for (int l = 0; l < kBwdMaxLevels; ++l)
      if (l < g.levels && sbid >= a.samp_wg_off[l]) {
        level = l;
        wg0 = a.samp_wg_off[l];
        srow0 = a.samp_row_off[l];
      }
    const NodeRef probe = node_ref(g, level, 0);
    const int clen = min(probe.s, kBwdChunk);
    const int cpn = (probe.s + clen - 1) / clen;
    const int spn = (g.m + kGRT - 1) / kGRT;
    const int nodes = g.causal ? (1 << level) : 1;
    int idx = sbid - wg0;
    const int slab = idx % spn;
    idx /= spn;
    qc_w = idx % cpn;
    idx /= cpn;
    const int node = idx % nodes;
    w.bh = idx / nodes;
    w.level = level;
    w.nr = node_ref(g, level, node);
    w.seg_off = ((int64_t)level * g.BH + w.bh) * g.n_cov + (int64_t)node * w.nr.s;
    chunk_start = qc_w * clen;
    chunk_len = min(clen, w.nr.s - chunk_start);
    samp0 = slab * kGRT;
    w.rows_valid = min(kGRT, g.m - samp0);
    samp_row0 = srow0;
    cpn_w = cpn;
  }

  const int64_t hs = f.q_bh_stride;
  const T* Qh = reinterpret_cast<const T*>(f.Q) + (int64_t)w.bh * hs;
  const T* Kh = reinterpret_cast<const T*>(f.K) + (int64_t)w.bh * hs;
  const T* Vh = reinterpret_cast<const T*>(f.V) + (int64_t)w.bh * hs;
  const T* Gh = reinterpret_cast<const T*>(a.dO) + (int64_t)w.bh * hs;
  const float* lse_h = a.lse + (int64_t)w.bh * g.n;
  const float* del_h = a.delta + (int64_t)w.bh * g.n;
  const T* Xh = kDq ? Qh : Kh;   // R rows: x operand of the scores
  const T* Ah = kDq ? Gh : Vh;   // R rows: operand of dP
  const T* Yh = kDq ? Kh : Qh;   // T rows: y operand of the scores
  const T* Bh = kDq ? Vh : Gh;   // T rows: operand of dP (dQ passes) / rows added into dV

  // ---- this thread's R row ----
  const bool r_valid = r_in_tile < w.rows_valid;
  const int r_use = r_valid ? r_in_tile : 0;
  int r_row;
  int64_t out_row;
  int blk_r = -1;
  if (MODE == kBwdDqNode) {
    r_row = f.perm_q[w.seg_off + w.p0 + r_use];
    out_row = (int64_t)w.bh * g.n + r_row;
  } else if (MODE == kBwdDkvBlock) {
    r_row = f.perm_k[w.seg_off + w.p0 + r_use];
    out_row = (int64_t)w.bh * g.n + r_row;
  } else if (MODE == kBwdDkvSamp) {
    const int j = samp0 + r_use;
    r_row = w.nr.k_start + f.samples[(int64_t)w.nr.heap * g.m + j];
    blk_r = f.samp_blk[((int64_t)w.bh * g.total_nodes + w.nr.heap) * g.m + j];
    const int nodes = g.causal ? (1 << w.level) : 1;
    const int node = w.nr.heap - ((1 << w.level) - 1);
    out_row = samp_row0 + ((((int64_t)w.bh * nodes + node) * cpn_w + qc_w) * g.m + j);
  } else {
    r_row = w.q0 + r_use;
    out_row = (int64_t)w.bh * g.n + r_row;
  }
  float x[C], av[WANT_DS ? C : 1], acc[C];
#pragma unroll
  for (int c = 0; c < C; ++c) {
    x[c] = load_elem<T>(Xh + (int64_t)r_row * D + c0 + c);
    if constexpr (WANT_DS) av[c] = load_elem<T>(Ah + (int64_t)r_row * D + c0 + c);
    acc[c] = 0.f;
  }
  float L_r = 0.f, del_r = 0.f;
  if (kDq) {
    L_r = lse_h[r_row];
    del_r = del_h[r_row];
  }

  // ---- the T rows ----
  int nT, nb = 0x7fffffff;
  const int32_t* tperm = nullptr;
  if (MODE == kBwdDqNode) {
    nT = build_key_list<kGNT>(f, w, list, scratch, &nb);
  } else if (MODE == kBwdDkvBlock) {
    nT = g.b;
    tperm = f.perm_q + w.seg_off + (int64_t)w.t * g.b;
  } else if (MODE == kBwdDkvSamp) {
    nT = chunk_len;
    tperm = f.perm_q + w.seg_off + chunk_start;
  } else {
    nT = max(0, w.k1 - w.k0);
  }
  const int ntiles = (nT + kGTT - 1) / kGTT;
  const float bias2 = ((MODE == kBwdDqNode || MODE == kBwdDkvSamp) && g.m > 0) ? logf((float)w.nr.s / (float)g.m) : 0.f;
  auto t_row = [&](int tpos) -> int {   // row within the head of T position tpos (clamped to an existing one)
    const int tp = min(tpos, nT - 1);
    if (kExact) return w.k0 + tp;
    if (kSorted) return tperm[tp];
    return list[tp];
  };

  for (int kt = 0; kt < ntiles; ++kt) {
    __syncthreads();
    for (int e = tid; e < kGTT * D; e += kGNT) {
      const int j = e / D, c = e % D;
      const int64_t at = (int64_t)t_row(kt * kGTT + j) * D + c;
      Ys[e] = load_elem<T>(Yh + at);
      Bs[e] = load_elem<T>(Bh + at);
    }
    if (!kDq && tid < kGTT) {
      const int row = t_row(kt * kGTT + tid);
      scl[tid] = lse_h[row];
      scd[tid] = del_h[row];
    }
    __syncthreads();
#pragma unroll 1
    for (int j = 0; j < kGTT; ++j) {
      const int tpos = kt * kGTT + j;
      bool masked = tpos >= nT;
      float bias = 0.f;
      if (MODE == kBwdDqNode) bias = (tpos >= nb) ? bias2 : 0.f;
      if (MODE == kBwdDkvSamp) {
        bias = bias2;
        masked = masked || ((chunk_start + tpos) / g.b == blk_r);  // queries of the key's own block: factor 1 - M
      }
      if (MODE == kBwdDqExact && f.exact_causal) masked = masked || (w.k0 + tpos > r_row);   // keys after the query
      if (MODE == kBwdDkvExact && f.exact_causal) masked = masked || (t0 + tpos < r_row);    // queries before the key
      const float L = kDq ? L_r : scl[j];
      const float dl = kDq ? del_r : scd[j];
      const float* yr = Ys + j * D + c0;
      const float* br = Bs + j * D + c0;
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < C; ++c) s = __builtin_fmaf(x[c], yr[c], s);
      s += __shfl_xor(s, 1);
      const float p = (masked || L == -INFINITY) ? 0.f : expf(s + bias - L);
      if constexpr (WANT_DS) {
        float dp = 0.f;
#pragma unroll
        for (int c = 0; c < C; ++c) dp = __builtin_fmaf(av[c], br[c], dp);
        dp += __shfl_xor(dp, 1);
        const float ds = p * (dp - dl);
#pragma unroll
        for (int c = 0; c < C; ++c) acc[c] = __builtin_fmaf(ds, yr[c], acc[c]);
      } else {
#pragma unroll
        for (int c = 0; c < C; ++c) acc[c] = __builtin_fmaf(p, br[c], acc[c]);
      }
    }
  }
  if (!r_valid) return;

  // ---- results: node passes write (the first level that holds the row on the pass's side) or add (later
  // levels) fp32 rows of the accumulated gradient; exact passes write the final gradient in the tensors'
  // dtype after adding the accumulated row where some level holds this row (queries: second half of the
  // node; keys: first half) ----
  if (!kExact) {
    float* dst = (WANT_DS ? a.out1 : a.out2) + out_row * D + c0;
    bool add = false;
    if (MODE == kBwdDqNode) add = node_levels_hold(g, r_row, true, w.level);
    if (MODE == kBwdDkvBlock) add = node_levels_hold(g, r_row, false, w.level);
    if (add) {
#pragma unroll
      for (int c = 0; c < C; c += 4) {
        const float4 v = *reinterpret_cast<const float4*>(dst + c);
        acc[c] += v.x;
        acc[c + 1] += v.y;
        acc[c + 2] += v.z;
        acc[c + 3] += v.w;
      }
    }
    store_cols<float, C>(dst, acc);
    return;
  }
  const float* lvl = WANT_DS ? a.lvl1 : a.lvl2;
  if (lvl != nullptr && node_levels_hold(g, r_row, kDq, g.levels)) {
    const float* pr = lvl + out_row * D + c0;
#pragma unroll
    for (int c = 0; c < C; c += 4) {
      const float4 v = *reinterpret_cast<const float4*>(pr + c);
      acc[c] += v.x;
      acc[c + 1] += v.y;
      acc[c + 2] += v.z;
      acc[c + 3] += v.w;
    }
  }
  store_cols<T, C>(reinterpret_cast<T*>(WANT_DS ? a.fin1 : a.fin2) + out_row * D + c0, acc);
}

template <typename T, int D, int MODE, bool WANT_DS>
static int launch_bwd_generic_one(const BwdArgs& a, int grid, hipStream_t st) {
  if (grid <= 0) return HA_OK;
  const size_t lds = bwd_generic_lds_bytes(a.f.g, D, MODE);
  static std::atomic<uint64_t> lds_set{0};  // per instantiation: devices on which the LDS limit is raised
  if (allow_full_lds(reinterpret_cast<const void*>(&attn_bwd_generic_kernel<T, D, MODE, WANT_DS>), lds_set) != HA_OK)
    return HA_ERR_LAUNCH;
  hipLaunchKernelGGL((attn_bwd_generic_kernel<T, D, MODE, WANT_DS>), dim3((unsigned)grid), dim3(kGNT), lds, st, a);
  return check_launch();
}

template <typename T, int D, int MODE>
static int launch_bwd_generic_pair(const BwdArgs& a, int grid, hipStream_t st) {  // dK into out1 / fin1, dV into out2 / fin2
  const int rc = launch_bwd_generic_one<T, D, MODE, true>(a, grid, st);
  return rc != HA_OK ? rc : launch_bwd_generic_one<T, D, MODE, false>(a, grid, st);
}

template <typename T, int D>
static int launch_bwd_generic_d(const BwdArgs& a, int mode, int grid, hipStream_t st) {
  switch (mode) {
    case kBwdDqNode: return launch_bwd_generic_one<T, D, kBwdDqNode, true>(a, grid, st);
    case kBwdDqExact: return launch_bwd_generic_one<T, D, kBwdDqExact, true>(a, grid, st);
    case kBwdDkvBlock: return launch_bwd_generic_pair<T, D, kBwdDkvBlock>(a, grid, st);
    case kBwdDkvSamp: return launch_bwd_generic_pair<T, D, kBwdDkvSamp>(a, grid, st);
    case kBwdDkvExact: return launch_bwd_generic_pair<T, D, kBwdDkvExact>(a, grid, st);
    default: return HA_ERR_SHAPE;
  }
}

int launch_attn_bwd_generic(const BwdArgs& a, int mode, hipStream_t st) {
  static_assert(kGRT == 128, "workgroup counts are shared with the MFMA backward kernel");
  const int64_t grid64 = bwd_grid(a, mode);
  if (grid64 > kMaxGrid) return HA_ERR_SHAPE;
  const int grid = (int)grid64;
  const int d = a.f.g.d;
  if (a.f.g.dtype != HA_FP32) return HA_ERR_DTYPE;
  if (d == 128) return launch_bwd_generic_d<float, 128>(a, mode, grid, st);
  if (d == 64) return launch_bwd_generic_d<float, 64>(a, mode, grid, st);
  return HA_ERR_SHAPE;
}

}  // namespace ha
