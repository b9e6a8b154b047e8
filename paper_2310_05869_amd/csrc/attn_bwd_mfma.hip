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
// Results leave as fp32 rows into per-part buffers; sums over parts are taken by
// separate kernels in a fixed order (no floating-point atomics anywhere).
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
  static constexpr int EP_WAVE = 32 * EP_ROW + 256;
};

__host__ __device__ inline int bwd_list_capacity(const Geometry& g, int mode) {
  if (mode == kBwdDqNode) return ((g.b + g.m + 63) & ~63) + 64;
  if (mode == kBwdDkvBlock) return ((g.b + 63) & ~63) + 64;
  if (mode == kBwdDkvSamp) return kBwdChunk;
  return 0;
}

template <int D>
__host__ __device__ inline size_t bwd_lds_bytes(const Geometry& g, int mode) {
  return 2 * (size_t)BwdLds<D>::BUF + 2 * BwdLds<D>::SC + 64 + (size_t)bwd_list_capacity(g, mode) * 4;
}

// dK/dV passes need two accumulator sets (256 registers with the operands):
// one wave per SIMD there, two in the dQ passes.
template <int MODE>
constexpr int bwd_min_waves() { return (MODE == kBwdDqNode || MODE == kBwdDqExact) ? 2 : 1; }

template <int D, int MODE>
__global__ __launch_bounds__(kBNT, bwd_min_waves<MODE>()) void attn_bwd_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using L = BwdLds<D>;
  constexpr bool kDq = (MODE == kBwdDqNode || MODE == kBwdDqExact);
  constexpr bool kExact = (MODE == kBwdDqExact || MODE == kBwdDkvExact);
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
  int t0 = 0;                                      // exact dK/dV pass: first query row of the T range
  if (MODE == kBwdDqNode || MODE == kBwdDkvBlock) {
    w = decode_node_tile<kRT>(f, logical_block(blockIdx.x, gridDim.x));
  } else if (MODE == kBwdDqExact) {
    w = decode_exact_tile<kRT>(f, logical_block(blockIdx.x, gridDim.x));
  } else if (MODE == kBwdDkvExact) {
    // key tiles of the diagonal blocks; early key tiles see the most queries
    const int eb = f.exact_block;
    const int tpb = (eb + kRT - 1) / kRT;
    const int nblk = (f.exact_rows_q + eb - 1) / eb;
    const int idx = logical_block(blockIdx.x, gridDim.x);
    const int ktile = idx % tpb;
    const int rest = idx / tpb;
    const int blk = rest % nblk;
    w.bh = rest / nblk;
    w.q0 = blk * eb + ktile * kRT;  // first KEY row of this tile
    const int blk_rows = min(eb, f.exact_rows_q - blk * eb);
    w.rows_valid = max(0, min(kRT, blk_rows - ktile * kRT));
    t0 = f.exact_causal ? w.q0 : blk * eb;
    w.k0 = t0;
    w.k1 = blk * eb + blk_rows;     // queries [t0, k1)
  } else {  // kBwdDkvSamp
    int level = 0;
    while (level + 1 < g.levels && (int)blockIdx.x >= a.samp_wg_off[level + 1]) ++level;
    const NodeRef probe = node_ref(g, level, 0);
    const int clen = min(probe.s, kBwdChunk);
    const int cpn = (probe.s + clen - 1) / clen;        // chunks per node
    const int spn = (g.m + kRT - 1) / kRT;              // sample slabs per node
    const int nodes = g.causal ? (1 << level) : 1;
    int idx = (int)blockIdx.x - a.samp_wg_off[level];
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
    out_row = w.seg_off + (r_row - w.nr.q_start);
  } else if (MODE == kBwdDkvBlock) {
    r_row = f.perm_k[w.seg_off + w.p0 + r_use];
    out_row = w.seg_off + (r_row - w.nr.k_start);
  } else if (MODE == kBwdDkvSamp) {
    const int j = samp0 + r_use;
    r_row = w.nr.k_start + f.samples[(int64_t)w.nr.heap * g.m + j];
    blk_r = f.samp_blk[((int64_t)w.bh * g.total_nodes + w.nr.heap) * g.m + j];
    const int nodes = g.causal ? (1 << w.level) : 1;
    const int node = w.nr.heap - ((1 << w.level) - 1);
    out_row = a.samp_row_off[w.level] + ((((int64_t)w.bh * nodes + node) * w.p0 + w.t) * g.m + j);
  } else {
    r_row = w.q0 + r_use;
    out_row = (int64_t)w.bh * g.n + r_row;
  }
  bf16x8 xreg[KS], areg[KS];
  {
    const u32x4* xp = reinterpret_cast<const u32x4*>(Xh + (int64_t)r_row * D + 8 * h);
    const u32x4* ap = reinterpret_cast<const u32x4*>(Ah + (int64_t)r_row * D + 8 * h);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      xreg[ks] = __builtin_bit_cast(bf16x8, xp[2 * ks]);
      areg[ks] = __builtin_bit_cast(bf16x8, ap[2 * ks]);
    }
  }
  float nl2_r = 0.f, del_r = 0.f;  // dQ passes: -L log2(e) and delta of the R row
  if (kDq) {
    const float lv = lse_h[r_row];
    nl2_r = (lv == -INFINITY) ? -INFINITY : -lv * kLog2e;
    del_r = del_h[r_row];
  }

  // ---- the T rows: a list in LDS (gathered passes) or a contiguous range ----
  int nT, nb = 0x7fffffff;
  if (MODE == kBwdDqNode) {
    nT = build_key_list<kBNT>(f, w, list, scratch, &nb);
  } else if (MODE == kBwdDkvBlock) {
    nT = g.b;
    const int pad = (nT + 63) & ~63;
    for (int i = tid; i < pad; i += kBNT) list[i] = f.perm_q[w.seg_off + w.t * g.b + min(i, nT - 1)];
    __syncthreads();
  } else if (MODE == kBwdDkvSamp) {
    nT = chunk_len;
    const int pad = (nT + 63) & ~63;
    for (int i = tid; i < pad; i += kBNT) list[i] = f.perm_q[w.seg_off + chunk_start + min(i, nT - 1)];
    __syncthreads();
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
  auto trow = [&](int tp) -> int {  // row within the head of T position tp (tp < padded length)
    if (kExact) return w.k0 + tp;
    return list[tp];
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
      } else {
        voff = list[kt * kTT + row] * (D * 2) + col * 16;
        soff = 0;
      }
      yreg[i] = __builtin_amdgcn_raw_buffer_load_b128(yrsrc, voff, soff, 0);
      breg[i] = __builtin_amdgcn_raw_buffer_load_b128(brsrc, voff, soff, 0);
    }
    if (!kDq && tid < kTT) {
      int row = trow(kt * kTT + tid);
      row = min(row, g.n - 1);
      const float lv = lse_h[row];
      sc_l = (lv == -INFINITY) ? -INFINITY : -lv * kLog2e;
      sc_d = del_h[row];
    }
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

  f32x16 acc1[DT], acc2[kDq ? 1 : DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      acc1[dt][i] = 0.f;
      if constexpr (!kDq) acc2[dt][i] = 0.f;
    }

  if (ntiles > 0) {
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

    // ---- S^T = Y X^T and dP^T = Bt A^T ----
    f32x16 c[2], e[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        c[sub][i] = 0.f;
        e[sub][i] = 0.f;
      }
    {
      const unsigned char* yp0 = yb + lq * L::TSTR + 16 * h;
      const unsigned char* bp0 = bb + lq * L::TSTR + 16 * h;
#pragma unroll
      for (int j = 0; j < KS; ++j) {
        c[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(yp0 + 32 * j), xreg[j], c[0], 0, 0, 0);
        c[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(yp0 + 32 * L::TSTR + 32 * j), xreg[j], c[1], 0, 0, 0);
        e[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(bp0 + 32 * j), areg[j], e[0], 0, 0, 0);
        e[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(bp0 + 32 * L::TSTR + 32 * j), areg[j], e[1], 0, 0, 0);
      }
    }

    // ---- P^T and dS^T ----
    const int tbase = kt * kTT;
    const bool tail = tbase + kTT > nT;
    bool special = tail;
    float tile_bias = 0.f;
    if (MODE == kBwdDqNode) {
      special = special || ((tbase < nb) && (tbase + kTT > nb));
      tile_bias = (tbase >= nb) ? bias2 : 0.f;
    }
    if (MODE == kBwdDkvSamp) tile_bias = bias2;
    if (MODE == kBwdDqExact && f.exact_causal) special = special || (w.k0 + tbase + kTT - 1 > w.q0 + wave * 32);
    if (MODE == kBwdDkvExact && f.exact_causal) special = special || (t0 + tbase < w.q0 + wave * 32 + 31);
    bool col_masked = false;  // sampled-key pass: the whole tile lies in this key's own block
    if (MODE == kBwdDkvSamp) {
      if (g.b % kTT == 0) col_masked = ((chunk_start + tbase) / g.b) == blk_r;
      else special = true;
    }

    bf16x8 pf[4], dsf[4];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        f32x4 nlT[2], dT[2];
        if (!kDq) {
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const int at = 32 * sub + 16 * jj + 8 * q + 4 * h;
            nlT[q] = *reinterpret_cast<const f32x4*>(scb + at);
            dT[q] = *reinterpret_cast<const f32x4*>(scb + kTT + at);
          }
        }
        u32x4 pk, dk;
#pragma unroll
        for (int ee = 0; ee < 4; ++ee) {
          float pv[2], dv[2];
#pragma unroll
          for (int z = 0; z < 2; ++z) {
            const int i = 8 * jj + 2 * ee + z;          // accumulator element
            const int koff = 32 * sub + 8 * (i / 4) + 4 * h + (i % 4);
            const int tp = tbase + koff;
            const int q = (i / 4) & 1;                  // which of the two f32x4 of this (sub, jj)
            float arg;
            float dsub;
            if (kDq) {
              arg = __builtin_fmaf(c[sub][i], kLog2e, nl2_r + tile_bias);
              dsub = del_r;
            } else {
              arg = __builtin_fmaf(c[sub][i], kLog2e, nlT[q][i % 4] + tile_bias);
              dsub = dT[q][i % 4];
            }
            if (special) {
              bool msk = tp >= nT;
              if (MODE == kBwdDqNode && tp >= nb && tbase < nb) arg += bias2;  // mixed tile: tile_bias is 0 there
              if (MODE == kBwdDqExact && f.exact_causal) msk = msk || (w.k0 + tp > r_global);
              if (MODE == kBwdDkvExact && f.exact_causal) msk = msk || (t0 + tp < r_global);
              if (MODE == kBwdDkvSamp && (g.b % kTT != 0)) msk = msk || (((chunk_start + tp) / g.b) == blk_r);
              if (msk) arg = -INFINITY;
            }
            if (MODE == kBwdDkvSamp && col_masked) arg = -INFINITY;
            const float p = __builtin_amdgcn_exp2f(arg);
            pv[z] = p;
            dv[z] = p * (e[sub][i] - dsub);
          }
          pk[ee] = pack_bf16x2(pv[0], pv[1]);
          dk[ee] = pack_bf16x2(dv[0], dv[1]);
        }
        pf[2 * sub + jj] = __builtin_bit_cast(bf16x8, pk);
        dsf[2 * sub + jj] = __builtin_bit_cast(bf16x8, dk);
      }

    // ---- acc1^T += Y^T dS^T ; acc2^T += Bt^T P^T ----
    {
      typedef short s16x4 __attribute__((ext_vector_type(4)));
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const unsigned char* yp = yb + vtr_off + (16 * j) * L::TSTR + (32 * dt) * 2;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(yp));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(yp + 8 * L::TSTR));
          const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          acc1[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), dsf[j], acc1[dt], 0, 0, 0);
          if constexpr (!kDq) {
            const unsigned char* bp = bb + vtr_off + (16 * j) * L::TSTR + (32 * dt) * 2;
            const s16x4 lo2 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(bp));
            const s16x4 hi2 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(bp + 8 * L::TSTR));
            const s16x8 both2 = __builtin_shufflevector(lo2, hi2, 0, 1, 2, 3, 4, 5, 6, 7);
            acc2[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both2), pf[j], acc2[dt], 0, 0, 0);
          }
        }
      }
    }
    if (more) store_tile(kt + 1);
    __syncthreads();
  }

  // ---- epilogue: the wave's 32 rows leave through an LDS transpose as whole fp32 rows ----
  unsigned char* ep = smem + wave * L::EP_WAVE;
  int64_t* ep_rows = reinterpret_cast<int64_t*>(ep + 32 * L::EP_ROW);
  if (h == 0) ep_rows[lq] = r_valid ? out_row : (int64_t)-1;
  auto drain = [&](const f32x16 (&acc)[DT], float* dst) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int col = 32 * dt + 8 * g4 + 4 * h;
        const f32x4 v = {acc[dt][4 * g4], acc[dt][4 * g4 + 1], acc[dt][4 * g4 + 2], acc[dt][4 * g4 + 3]};
        *reinterpret_cast<f32x4*>(ep + lq * L::EP_ROW + col * 4) = v;
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    constexpr int CH = D / 4;  // 16-byte pieces per fp32 row
    for (int idx = lane; idx < 32 * CH; idx += 64) {
      const int row = idx / CH, ch = idx % CH;
      const int64_t r64 = ep_rows[row];
      if (r64 >= 0)
        *reinterpret_cast<f32x4*>(dst + r64 * D + ch * 4) = *reinterpret_cast<const f32x4*>(ep + row * L::EP_ROW + ch * 16);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  drain(acc1, a.out1);
  if constexpr (!kDq) drain(acc2, a.out2);
}

template <int D, int MODE>
static int launch_bwd_one(const BwdArgs& a, int grid, hipStream_t st) {
  if (grid <= 0) return HA_OK;
  size_t lds = bwd_lds_bytes<D>(a.f.g, MODE);
  if (lds < (size_t)4 * BwdLds<D>::EP_WAVE) lds = (size_t)4 * BwdLds<D>::EP_WAVE;
  static bool configured = false;  // per instantiation
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_kernel<D, MODE>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
      (void)hipGetLastError();
      return HA_ERR_LAUNCH;
    }
    configured = true;
  }
  hipLaunchKernelGGL((attn_bwd_kernel<D, MODE>), dim3((unsigned)grid), dim3(kBNT), lds, st, a);
  return check_launch();
}

template <int D>
static int launch_bwd_d(const BwdArgs& a, int mode, int grid, hipStream_t st) {
  switch (mode) {
    case kBwdDqNode: return launch_bwd_one<D, kBwdDqNode>(a, grid, st);
    case kBwdDqExact: return launch_bwd_one<D, kBwdDqExact>(a, grid, st);
    case kBwdDkvBlock: return launch_bwd_one<D, kBwdDkvBlock>(a, grid, st);
    case kBwdDkvSamp: return launch_bwd_one<D, kBwdDkvSamp>(a, grid, st);
    case kBwdDkvExact: return launch_bwd_one<D, kBwdDkvExact>(a, grid, st);
    default: return HA_ERR_SHAPE;
  }
}

int bwd_grid(const BwdArgs& a, int mode) {
  const Geometry& g = a.f.g;
  if (mode == kBwdDqNode || mode == kBwdDkvBlock) return node_grid<kRT>(g);
  if (mode == kBwdDqExact || mode == kBwdDkvExact) return exact_grid<kRT>(a.f);
  return a.samp_wg_off[g.levels];
}

int launch_attn_bwd_mfma(const BwdArgs& a, int mode, hipStream_t st) {
  if (a.f.g.dtype != HA_BF16) return HA_ERR_DTYPE;
  const int grid = bwd_grid(a, mode);
  if (a.f.g.d == 128) return launch_bwd_d<128>(a, mode, grid, st);
  if (a.f.g.d == 64) return launch_bwd_d<64>(a, mode, grid, st);
  return HA_ERR_SHAPE;
}

}  // namespace ha
