// bf16 MFMA backward kernel for gfx950: gradients of the HyperAttention forward
// with respect to Q, K and V, the random draws (hyperplanes, sample indices)
// and hence the permutations held fixed.
//
// Every output row of the forward is ONE softmax over a multiset of keys with
// weights: its block keys (weight 1) and its kept sampled keys (weight s/m) in
// every node the row belongs to, plus, when causal, the keys of its base-case
// block (Algorithms 1, 2 and 4 with the row sums added up).  With the final
// log row sum L_i and delta_i = <dO_i, O_i>, the gradient therefore splits into
// independent contributions of every (query, key) pair that occurs:
//   P_ij  = w_ij exp(<q_i, k_j> - L_i)
//   dV_j += P_ij dO_i
//   dS_ij = P_ij (<dO_i, v_j> - delta_i)
//   dQ_i += dS_ij k_j          dK_j += dS_ij q_i
// and each part (node block, node samples, base block) can be processed on its
// own, with the same tiles, lists and masks as in the forward.
//
// One kernel, two roles.  32 "R rows" per wave stay in registers for the whole
// pass and own the accumulators; "T rows" stream through LDS in tiles of 64:
//   dQ passes   R = queries (Q, dO, L, delta in registers), T = keys (K, V)
//   dK/dV passes R = keys (K, V in registers),  T = queries (Q, dO; L, delta in LDS)
// As in the forward the transposed products are formed (T rows along the MFMA's
// M dimension), so a lane holds 16 T rows of ONE R row, and P^T, dS^T converted
// to bf16 are directly the B operands of the accumulating products, whose A
// operands (T tile transposed) come from the transposing LDS read.
//
// The dK/dV passes run twice, once accumulating dK (scores, dP, dS) and once
// dV (scores, P): one accumulator set each, so two waves fit per SIMD.
//
// Sums over parts are taken in a fixed order, never by floating-point atomics: the node passes run
// level by level and add their fp32 rows to one accumulated row per tensor row (the first level
// that holds a row writes it), the sampled keys' rows go through a reduction of their own, and the
// base-case passes add the accumulated rows in their epilogue and write the final gradient.
#include <type_traits>

#include "attn_common.h"
#include "bwd_common.h"

namespace ha {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTT = 64;    // T rows per step
constexpr int kRT = 128;   // R rows per workgroup (4 waves x 32)
constexpr int kBNT = 256;  // threads

template <int D>
struct BwdLds {
  static constexpr int TSTR = (D + 24) * 2;     // bytes per T row: serves both the 16-byte row reads and the transposing reads
  static constexpr int TILE = kTT * TSTR;       // one tensor's tile
  static constexpr int BUF = 2 * TILE;          // y tile + bt tile
  static constexpr int SC = 2 * kTT * 4;        // per buffer: -L log2(e) and delta of the T rows
  static constexpr int EP_ROW = D * 4 + 16;
  static constexpr int EP_WAVE = 32 * EP_ROW + 256;  // rows, row ids
};

__host__ __device__ inline int bwd_list_capacity(const Geometry& g, int mode) {
  if (mode == kBwdDqNode) return ((g.b + g.m + 63) & ~63) + 64;
  return 0;
}

template <int D>
__host__ __device__ inline size_t bwd_lds_bytes(const Geometry& g, int mode) {
  return 2 * (size_t)BwdLds<D>::BUF + 2 * BwdLds<D>::SC + 64 + (size_t)bwd_list_capacity(g, mode) * 4;
}

// WHAT: which product the pass accumulates.
enum BwdWhat : int { kAccDs = 0,    // acc += Y^T dS^T : dQ (dQ passes) or dK (dK/dV passes)
                     kAccP = 1,     // acc += Bt^T P^T : dV (dK/dV passes only)
                     kAccBoth = 2 };  // dK, then dV, in one launch: the workgroup keeps its R rows and walks its T rows twice

template <int D, int MODE, int WHAT>
__global__ __launch_bounds__(kBNT, 2) void attn_bwd_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using L = BwdLds<D>;
  constexpr bool kDq = (MODE == kBwdDqNode || MODE == kBwdDqExact);
  constexpr bool kExact = (MODE == kBwdDqExact || MODE == kBwdDkvExact);
  constexpr bool kSorted = (MODE == kBwdDkvBlock || MODE == kBwdDkvSamp);  // T rows = a run of sorted query positions
  constexpr bool kLoadA = (WHAT != kAccP);  // the operand of dP is needed whenever dS is formed
  static_assert(WHAT == kAccDs || !kDq, "the dQ passes accumulate dS only");
  constexpr int KS = D / 16;
  constexpr int DT = D / 32;
  constexpr int CPR = D / 8;                 // 16-byte chunks per row
  constexpr int NKC = kTT * CPR / kBNT;      // chunks per thread and tensor

  const AttnArgs& f = a.f;
  const Geometry& g = f.g;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, h = lane >> 5;

  unsigned char* bufs = smem;
  float* sc = reinterpret_cast<float*>(smem + 2 * L::BUF);
  int32_t* scratch = reinterpret_cast<int32_t*>(smem + 2 * L::BUF + 2 * L::SC);
  int32_t* list = scratch + 16;

  // ---- which part of the problem this workgroup owns ----
  TileWork w{};
  int chunk_start = 0, chunk_len = 0, samp0 = 0;  // sampled-key pass
  int64_t samp_row0 = 0;
  int t0 = 0;                                      // exact dK/dV pass: first query row of the T range
  if (MODE == kBwdDqNode || MODE == kBwdDkvBlock) {
    w = decode_node_tile<kRT>(f, a.wg_base + logical_block(blockIdx.x, gridDim.x));
  } else if (MODE == kBwdDqExact) {
    w = decode_exact_tile<kRT>(f, logical_block(blockIdx.x, gridDim.x));
  } else if (MODE == kBwdDkvExact) {
    // key tiles of the diagonal blocks; early key tiles see the most queries
    const int eb = f.exact_block;
    const int tpb = (eb + kRT - 1) / kRT;
    const int nblk = (f.exact_rows_q + eb - 1) / eb;
    const int idx = logical_block(blockIdx.x, gridDim.x);
    const int rest = idx / tpb;
    const int ktile = (idx % tpb + rest) % tpb;  // starting tile rotated per block: see decode_exact_tile
    const int blk = rest % nblk;
    w.bh = rest / nblk;
    w.q0 = blk * eb + ktile * kRT;  // first KEY row of this tile
    const int blk_rows = min(eb, f.exact_rows_q - blk * eb);
    w.rows_valid = max(0, min(kRT, blk_rows - ktile * kRT));
    t0 = f.exact_causal ? w.q0 : blk * eb;
    w.k0 = t0;
    w.k1 = blk * eb + blk_rows;     // queries [t0, k1)
  } else {  // kBwdDkvSamp
    // (static indices only: a dynamically indexed kernel-argument array would be copied to scratch)
    const int sbid = logical_block(blockIdx.x, gridDim.x);  // slabs of one chunk meet in one L2
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
    const int cpn = (probe.s + clen - 1) / clen;        // chunks per node
    const int spn = (g.m + kRT - 1) / kRT;              // sample slabs per node
    const int nodes = g.causal ? (1 << level) : 1;
    int idx = sbid - wg0;
    const int slab = idx % spn;
    idx /= spn;
    const int qc = idx % cpn;
    idx /= cpn;
    const int node = idx % nodes;
    w.bh = idx / nodes;
    w.level = level;
    w.nr = node_ref(g, level, node);
    w.seg_off = ((int64_t)level * g.BH + w.bh) * g.n_cov + (int64_t)node * w.nr.s;
    chunk_start = qc * clen;
    chunk_len = min(clen, w.nr.s - chunk_start);
    samp0 = slab * kRT;
    w.rows_valid = min(kRT, g.m - samp0);
    samp_row0 = srow0;
    w.t = qc;  // reused: chunk index
    w.p0 = cpn;
  }

  const int64_t hs = f.q_bh_stride;
  const uint16_t* Qh = reinterpret_cast<const uint16_t*>(f.Q) + (int64_t)w.bh * hs;
  const uint16_t* Kh = reinterpret_cast<const uint16_t*>(f.K) + (int64_t)w.bh * hs;
  const uint16_t* Vh = reinterpret_cast<const uint16_t*>(f.V) + (int64_t)w.bh * hs;
  const uint16_t* Gh = reinterpret_cast<const uint16_t*>(a.dO) + (int64_t)w.bh * hs;
  const float* lse_h = a.lse + (int64_t)w.bh * g.n;
  const float* del_h = a.delta + (int64_t)w.bh * g.n;
  const uint16_t* Xh = kDq ? Qh : Kh;   // R rows: x operand of the scores
  const uint16_t* Ah = kDq ? Gh : Vh;   // R rows: operand of dP
  const uint16_t* Yh = kDq ? Kh : Qh;   // T rows: y operand of the scores
  const uint16_t* Bh = kDq ? Vh : Gh;   // T rows: operand of dP

  // ---- this lane's R row ----
  const int r_in_tile = wave * 32 + lq;
  const bool r_valid = r_in_tile < w.rows_valid;
  const int r_use = r_valid ? r_in_tile : 0;
  int r_row;             // row within the head
  int64_t out_row;       // row in out1 / out2
  int blk_r = -1;        // sampled-key pass: sorted block of this key
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
    out_row = samp_row0 + ((((int64_t)w.bh * nodes + node) * w.p0 + w.t) * g.m + j);
  } else {
    r_row = w.q0 + r_use;
    out_row = (int64_t)w.bh * g.n + r_row;
  }
  bf16x8 xreg[KS], areg[kLoadA ? KS : 1];
  {
    const u32x4* xp = reinterpret_cast<const u32x4*>(Xh + (int64_t)r_row * D + 8 * h);
    const u32x4* ap = reinterpret_cast<const u32x4*>(Ah + (int64_t)r_row * D + 8 * h);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      xreg[ks] = __builtin_bit_cast(bf16x8, xp[2 * ks]);
      if constexpr (kLoadA) areg[ks] = __builtin_bit_cast(bf16x8, ap[2 * ks]);
    }
  }
  float nl2_r = 0.f, del_r = 0.f;  // dQ passes: -L log2(e) and delta of the R row
  if (kDq) {
    const float lv = lse_h[r_row];
    nl2_r = (lv == -INFINITY) ? -INFINITY : -lv * kLog2e;
    del_r = del_h[r_row];
  }

  // ---- the T rows: the key list in LDS (dQ of a node), a run of sorted query
  // positions read through P_Q (dK/dV of a node), or a contiguous range ----
  int nT, nb = 0x7fffffff;
  const int32_t* tperm = nullptr;  // sorted passes: P_Q at T position 0
  if (MODE == kBwdDqNode) {
    nT = build_key_list<kBNT>(f, w, list, scratch, &nb);
  } else if (MODE == kBwdDkvBlock) {
    nT = g.b;
    tperm = f.perm_q + w.seg_off + (int64_t)w.t * g.b;
  } else if (MODE == kBwdDkvSamp) {
    nT = chunk_len;
    tperm = f.perm_q + w.seg_off + chunk_start;
  } else {
    nT = max(0, w.k1 - w.k0);
  }
  const int ntiles = (nT + kTT - 1) / kTT;
  const float bias2 = ((MODE == kBwdDqNode || MODE == kBwdDkvSamp) && g.m > 0) ? log2f((float)w.nr.s / (float)g.m) : 0.f;

  // ---- tile movers: rows through buffer loads (out-of-range rows read as zero) ----
  const uint32_t head_bytes = (uint32_t)(g.n * (D * 2));
  const __amdgpu_buffer_rsrc_t yrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)Yh, 0, (int)head_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t brsrc = __builtin_amdgcn_make_buffer_rsrc((void*)Bh, 0, (int)head_bytes, 0x00020000);
  u32x4 yreg[NKC], breg[NKC];
  float sc_l = 0.f, sc_d = 0.f;
  // sorted passes: the rows of the tile to be loaded next, fetched one tile ahead of its loads
  int tix[NKC], six = 0;
  auto fetch_rows = [&](int kt) {
#pragma unroll
    for (int i = 0; i < NKC; ++i) tix[i] = tperm[min(kt * kTT + (tid + i * kBNT) / CPR, nT - 1)];
    if (tid < kTT) six = tperm[min(kt * kTT + tid, nT - 1)];
  };
  auto load_tile = [&](int kt) {
#pragma unroll
    for (int i = 0; i < NKC; ++i) {
      const int c = tid + i * kBNT;
      const int row = c / CPR, col = c % CPR;
      int voff, soff;
      if (kExact) {
        voff = row * (D * 2) + col * 16;
        soff = (w.k0 + kt * kTT) * (D * 2);
      } else if (kSorted) {
        voff = tix[i] * (D * 2) + col * 16;
        soff = 0;
      } else {
        voff = list[kt * kTT + row] * (D * 2) + col * 16;
        soff = 0;
      }
      yreg[i] = __builtin_amdgcn_raw_buffer_load_b128(yrsrc, voff, soff, 0);
      breg[i] = __builtin_amdgcn_raw_buffer_load_b128(brsrc, voff, soff, 0);
    }
    if (!kDq && tid < kTT) {
      int row = kSorted ? six : min(w.k0 + kt * kTT + tid, g.n - 1);
      const float lv = lse_h[row];
      sc_l = (lv == -INFINITY) ? -INFINITY : -lv * kLog2e;
      sc_d = del_h[row];
    }
    if (kSorted && (kt + 1) * kTT < nT) fetch_rows(kt + 1);
  };
  auto store_tile = [&](int kt) {
    unsigned char* yb = bufs + (kt & 1) * L::BUF;
    unsigned char* bb = yb + L::TILE;
#pragma unroll
    for (int i = 0; i < NKC; ++i) {
      const int c = tid + i * kBNT;
      const int row = c / CPR, col = c % CPR;
      *reinterpret_cast<u32x4*>(yb + row * L::TSTR + col * 16) = yreg[i];
      *reinterpret_cast<u32x4*>(bb + row * L::TSTR + col * 16) = breg[i];
    }
    if (!kDq && tid < kTT) {
      float* s = sc + (kt & 1) * (2 * kTT);
      s[tid] = sc_l;
      s[kTT + tid] = sc_d;
    }
  };
  const int vtr_off = ((lane & 15) >> 2) * L::TSTR + ((lane & 3) * 4 + ((lane >> 4) & 1) * 16) * 2 + (4 * h) * L::TSTR;

  // One pass over the T rows: accumulate, then write the wave's rows.  `what_tag` says what is
  // accumulated (dS products or P products).
  auto run_pass = [&](auto what_tag) {
    constexpr bool kWantDs = (decltype(what_tag)::value == kAccDs);
    f32x16 acc[DT];
  #pragma unroll
    for (int dt = 0; dt < DT; ++dt)
  #pragma unroll
      for (int i = 0; i < 16; ++i) acc[dt][i] = 0.f;

    if (ntiles > 0) {
      if (kSorted) fetch_rows(0);
      load_tile(0);
      store_tile(0);
    }
    __syncthreads();

    const int r_global = r_row;  // exact passes: for the causal mask
    for (int kt = 0; kt < ntiles; ++kt) {
      const bool more = kt + 1 < ntiles;
      if (more) load_tile(kt + 1);

      const unsigned char* yb = bufs + (kt & 1) * L::BUF;
      const unsigned char* bb = yb + L::TILE;
      const float* scb = sc + (kt & 1) * (2 * kTT);

      // ---- P^T and dS^T ----
      // Masks as limits on the in-tile row offset ko = koff - 4 h of an accumulator element
      // (koff = 32 sub + 8 (i / 4) + 4 h + i % 4): masked iff ko >= hi2 (end of the T rows; keys
      // after the query), ko < lo2 (queries before the key) or mlo2 <= ko < mhi2 (queries of
      // the sampled key's own block, factor 1 - M of Algorithm 2).
      const int tbase = kt * kTT;
      int hi2 = nT - tbase - 4 * h;
      int lo2 = -0x40000000, mlo2 = 0x40000000, mhi2 = 0x40000000, nb2 = 0x40000000;
      float tile_bias = 0.f;
      if (MODE == kBwdDqNode) {
        tile_bias = (tbase >= nb) ? bias2 : 0.f;
        if (tbase < nb) nb2 = nb - tbase - 4 * h;  // tile_bias is 0 on a tile that straddles nb
      }
      if (MODE == kBwdDkvSamp) {
        tile_bias = bias2;
        mlo2 = blk_r * g.b - (chunk_start + tbase) - 4 * h;
        mhi2 = mlo2 + g.b;
      }
      if (MODE == kBwdDqExact && f.exact_causal) hi2 = min(hi2, r_global - w.k0 - tbase + 1 - 4 * h);
      if (MODE == kBwdDkvExact && f.exact_causal) lo2 = r_global - t0 - tbase - 4 * h;
      // highest / lowest ko of a lane: 59 / 0
      const bool special = __any(hi2 <= 59 || lo2 > 0 || nb2 <= 59 || (mlo2 <= 59 && mhi2 > 0));

      bf16x8 bf[2];  // B operand of the accumulating product (per half): dS^T or P^T as bf16
      // one 32-row half of the tile at a time: S^T = Y X^T and dP^T = Bt A^T, then P^T / dS^T
  #pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        f32x16 cs, es;
  #pragma unroll
        for (int i = 0; i < 16; ++i) {
          cs[i] = 0.f;
          es[i] = 0.f;
        }
        // the wave holds issue priority over its SIMD neighbour while it issues its S^T / dP^T products (measured:
        // dQ of the base case -9 %, its dK / dV -3 %; the short loops of the block passes lose 1-2 % and go without)
        constexpr bool kPrio = kExact || MODE == kBwdDkvSamp;
        if constexpr (kPrio) __builtin_amdgcn_s_setprio(1);
        {
          const unsigned char* yp0 = yb + (32 * sub + lq) * L::TSTR + 16 * h;
          const unsigned char* bp0 = bb + (32 * sub + lq) * L::TSTR + 16 * h;
  #pragma unroll
          for (int j = 0; j < KS; ++j) {
            cs = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(yp0 + 32 * j), xreg[j], cs, 0, 0, 0);
            if constexpr (kWantDs)
              es = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(bp0 + 32 * j), areg[j], es, 0, 0, 0);
          }
        }
        if constexpr (kPrio) __builtin_amdgcn_s_setprio(0);
        f32x4 nlq = {0.f, 0.f, 0.f, 0.f}, dq4 = {0.f, 0.f, 0.f, 0.f};  // -L log2(e), delta of four T rows (dK/dV passes)
  #pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          u32x4 pk, dk;
  #pragma unroll
          for (int ee = 0; ee < 4; ++ee) {
            // elements 8 jj + 2 ee, + 1: T rows 32 sub + 16 jj + 8 (ee / 2) + 4 h + 2 (ee % 2), + 1
            f32x4 nlT = {0.f, 0.f, 0.f, 0.f}, dT = {0.f, 0.f, 0.f, 0.f};
            if (!kDq && (ee % 2 == 0)) {
              const int at = 32 * sub + 16 * jj + 8 * (ee / 2) + 4 * h;
              nlq = *reinterpret_cast<const f32x4*>(scb + at);
              dq4 = *reinterpret_cast<const f32x4*>(scb + kTT + at);
            }
            nlT = nlq;
            dT = dq4;
            float pv[2], dv[2];
  #pragma unroll
            for (int z = 0; z < 2; ++z) {
              const int i = 8 * jj + 2 * ee + z;          // accumulator element
              float arg;
              float dsub;
              if (kDq) {
                arg = __builtin_fmaf(cs[i], kLog2e, nl2_r + tile_bias);
                dsub = del_r;
              } else {
                arg = __builtin_fmaf(cs[i], kLog2e, nlT[i % 4] + tile_bias);
                dsub = dT[i % 4];
              }
              if (special) {
                const int ko = 32 * sub + 8 * (i / 4) + (i % 4);
                if (MODE == kBwdDqNode && ko >= nb2) arg += bias2;
                bool msk = ko >= hi2;
                if (MODE == kBwdDkvExact) msk = msk || (ko < lo2);
                if (MODE == kBwdDkvSamp) msk = msk || ((unsigned)(ko - mlo2) < (unsigned)g.b);
                if (msk) arg = -INFINITY;
              }
              const float p = __builtin_amdgcn_exp2f(arg);
              pv[z] = p;
              dv[z] = p * (es[i] - dsub);
            }
            pk[ee] = pack_bf16x2(pv[0], pv[1]);
            dk[ee] = pack_bf16x2(dv[0], dv[1]);
          }
          bf[jj] = __builtin_bit_cast(bf16x8, kWantDs ? dk : pk);
        }
        // ---- acc^T += Y^T dS^T  or  acc^T += Bt^T P^T  for the 32 rows of this half ----
        {
          typedef short s16x4 __attribute__((ext_vector_type(4)));
          typedef short s16x8 __attribute__((ext_vector_type(8)));
          typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
          const unsigned char* tb = (kWantDs ? yb : bb) + vtr_off;
  #pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            const int j = 2 * sub + jj;
  #pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
              const unsigned char* tp = tb + (16 * j) * L::TSTR + (32 * dt) * 2;
              const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tp));
              const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tp + 8 * L::TSTR));
              const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
              acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), bf[jj], acc[dt], 0, 0, 0);
            }
          }
        }
      }
      if (more) store_tile(kt + 1);
      __syncthreads();
    }

    // ---- epilogue: the wave's 32 rows leave through an LDS transpose as whole rows.
    // Node passes write or add fp32 rows into the accumulated rows.  Exact passes (the
    // base case of Algorithm 4) write the final gradient in the tensors' dtype, after
    // adding the accumulated row where some level's node holds the row on the pass's
    // side (queries: second half of the node; keys: first half).
    unsigned char* ep = smem + wave * L::EP_WAVE;
    int64_t* ep_rows = reinterpret_cast<int64_t*>(ep + 32 * L::EP_ROW);
    if (h == 0) ep_rows[lq] = r_valid ? out_row : (int64_t)-1;
  #pragma unroll
    for (int dt = 0; dt < DT; ++dt)
  #pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int col = 32 * dt + 8 * g4 + 4 * h;
        const f32x4 v = {acc[dt][4 * g4], acc[dt][4 * g4 + 1], acc[dt][4 * g4 + 2], acc[dt][4 * g4 + 3]};
        *reinterpret_cast<f32x4*>(ep + lq * L::EP_ROW + col * 4) = v;
      }
    float* dst32 = kWantDs ? a.out1 : a.out2;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // Rows that are not stored (past the end of the tile; valid rows are a prefix) re-read the wave's first
    // row, so that every load below is unconditional and all of them are requested before the first is
    // used; only the stores sit under a branch.  With loads under a branch the compiler's wait counts
    // fall back to "everything", and each piece would also wait for the previous piece's stores.
    const int64_t row_first = ep_rows[0];
    if (row_first < 0) return;
    if (!kExact) {
      // node passes add to what earlier levels left in the row; all rows of a node lie on the same side of
      // every ancestor, so the whole workgroup either adds or writes
      bool add = false;
      if (MODE == kBwdDqNode) add = node_levels_hold(g, w.nr.q_start, true, w.level);
      if (MODE == kBwdDkvBlock) add = node_levels_hold(g, w.nr.k_start, false, w.level);
      constexpr int CH = D / 4;            // 16-byte pieces per fp32 row
      constexpr int IT = 32 * CH / 64;     // pieces per lane
      int64_t r64[IT];
      f32x4 prev[IT];
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        const int idx = lane + 64 * it;
        r64[it] = ep_rows[idx / CH];
        prev[it] = (f32x4){0.f, 0.f, 0.f, 0.f};
      }
      if (add) {
#pragma unroll
        for (int it = 0; it < IT; ++it) {
          const int ch = (lane + 64 * it) % CH;
          const int64_t rr = r64[it] >= 0 ? r64[it] : row_first;
          prev[it] = *reinterpret_cast<const f32x4*>(dst32 + rr * D + ch * 4);
        }
      }
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        const int idx = lane + 64 * it;
        const int row = idx / CH, ch = idx % CH;
        const f32x4 v = *reinterpret_cast<const f32x4*>(ep + row * L::EP_ROW + ch * 16) + prev[it];
        if (r64[it] >= 0) *reinterpret_cast<f32x4*>(dst32 + r64[it] * D + ch * 4) = v;
      }
      return;
    }
    uint16_t* dst16 = reinterpret_cast<uint16_t*>(kWantDs ? a.fin1 : a.fin2);
    const float* lvl = kWantDs ? a.lvl1 : a.lvl2;
    // the 32 rows of a wave lie in one n_min block: the node passes hold all of them or none
    const int i0 = w.q0 + 32 * __builtin_amdgcn_readfirstlane(wave);
    const bool fold = lvl != nullptr && node_levels_hold(g, i0, kDq, g.levels);
    const float* acc_rows = lvl + ((int64_t)w.bh * g.n + i0) * D;
    constexpr int CH8 = D / 8;             // 8-element pieces per row
    constexpr int IT8 = 32 * CH8 / 64;     // pieces per lane
    int64_t r64[IT8];
    f32x4 p0[IT8], p1[IT8];
#pragma unroll
    for (int it = 0; it < IT8; ++it) {
      r64[it] = ep_rows[(lane + 64 * it) / CH8];
      p0[it] = (f32x4){0.f, 0.f, 0.f, 0.f};
      p1[it] = p0[it];
    }
    if (fold) {
#pragma unroll
      for (int it = 0; it < IT8; ++it) {
        const int idx = lane + 64 * it;
        const int row = r64[it] >= 0 ? idx / CH8 : 0, ch = idx % CH8;
        const float* pp = acc_rows + (int64_t)row * D + ch * 8;
        p0[it] = *reinterpret_cast<const f32x4*>(pp);
        p1[it] = *reinterpret_cast<const f32x4*>(pp + 4);
      }
    }
#pragma unroll
    for (int it = 0; it < IT8; ++it) {
      const int idx = lane + 64 * it;
      const int row = idx / CH8, ch = idx % CH8;
      const f32x4 v0 = *reinterpret_cast<const f32x4*>(ep + row * L::EP_ROW + ch * 32) + p0[it];
      const f32x4 v1 = *reinterpret_cast<const f32x4*>(ep + row * L::EP_ROW + ch * 32 + 16) + p1[it];
      const u32x4 pk = {pack_bf16x2(v0.x, v0.y), pack_bf16x2(v0.z, v0.w), pack_bf16x2(v1.x, v1.y), pack_bf16x2(v1.z, v1.w)};
      if (r64[it] >= 0) *reinterpret_cast<u32x4*>(dst16 + r64[it] * D + ch * 8) = pk;
    }
  };
  if constexpr (WHAT == kAccBoth) {
    static_assert(WHAT != kAccBoth || !kExact, "the two-in-one form writes per-level rows only");
    run_pass(std::integral_constant<int, kAccDs>{});
    __syncthreads();  // the epilogue staged rows where the T tiles go
    run_pass(std::integral_constant<int, kAccP>{});
  } else {
    run_pass(std::integral_constant<int, WHAT>{});
  }
}

template <int D, int MODE, int WHAT>
static int launch_bwd_one(const BwdArgs& a, int grid, hipStream_t st) {
  if (grid <= 0) return HA_OK;
  size_t lds = bwd_lds_bytes<D>(a.f.g, MODE);
  if (lds < (size_t)4 * BwdLds<D>::EP_WAVE) lds = (size_t)4 * BwdLds<D>::EP_WAVE;
  static std::atomic<uint64_t> lds_set{0};  // per instantiation: devices on which the LDS limit is raised
  if (allow_full_lds(reinterpret_cast<const void*>(&attn_bwd_kernel<D, MODE, WHAT>), lds_set) != HA_OK) return HA_ERR_LAUNCH;
  hipLaunchKernelGGL((attn_bwd_kernel<D, MODE, WHAT>), dim3((unsigned)grid), dim3(kBNT), lds, st, a);
  return check_launch();
}

// dK/dV passes: two launches, dK into out1 and dV into out2
template <int D, int MODE>
static int launch_bwd_pair(const BwdArgs& a, int grid, hipStream_t st) {
  const int rc = launch_bwd_one<D, MODE, kAccDs>(a, grid, st);
  return rc != HA_OK ? rc : launch_bwd_one<D, MODE, kAccP>(a, grid, st);
}

template <int D>
static int launch_bwd_d(const BwdArgs& a, int mode, int grid, hipStream_t st) {
  switch (mode) {
    case kBwdDqNode: return launch_bwd_one<D, kBwdDqNode, kAccDs>(a, grid, st);
    case kBwdDqExact: return launch_bwd_one<D, kBwdDqExact, kAccDs>(a, grid, st);
    case kBwdDkvBlock: return launch_bwd_one<D, kBwdDkvBlock, kAccBoth>(a, grid, st);  // short T loops: one launch, shared prologue
    case kBwdDkvSamp: return launch_bwd_pair<D, kBwdDkvSamp>(a, grid, st);
    case kBwdDkvExact: return launch_bwd_pair<D, kBwdDkvExact>(a, grid, st);
    default: return HA_ERR_SHAPE;
  }
}
int64_t bwd_grid(const BwdArgs& a, int mode) {
  const Geometry& g = a.f.g;
  if (mode == kBwdDqNode || mode == kBwdDkvBlock) return g.levels > 0 ? node_grid<kRT>(g) / g.levels : 0;  // one level per launch
  if (mode == kBwdDqExact || mode == kBwdDkvExact) return exact_grid<kRT>(a.f);
  return a.samp_wg_off[g.levels];
}

int launch_attn_bwd_mfma(const BwdArgs& a, int mode, hipStream_t st) {
  if (a.f.g.dtype != HA_BF16) return HA_ERR_DTYPE;
  const int64_t grid64 = bwd_grid(a, mode);
  if (grid64 > kMaxGrid) return HA_ERR_SHAPE;
  const int grid = (int)grid64;
  if (a.f.g.d == 128) return launch_bwd_d<128>(a, mode, grid, st);
  if (a.f.g.d == 64) return launch_bwd_d<64>(a, mode, grid, st);
  return HA_ERR_SHAPE;
}

}  // namespace ha
