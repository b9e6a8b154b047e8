// bf16 MFMA attention kernel for gfx950: one online-softmax pass of a tile of
// 128 queries over a list of keys.
//
//   node mode   the b x b diagonal block of the sorted attention matrix
//               (Algorithm 1's mask M^H; Section 4, Implementation Detail) and
//               the kept sampled columns of Algorithm 2 in ONE pass with a
//               shared normaliser; rows of Q, K, V are fetched through the
//               sort permutations (the "permute" is fused into the loads) and
//               the result is written back through P_Q (the inverse permute is
//               fused into the store).
//   exact mode  plain tiled softmax attention over contiguous keys with an
//               optional causal mask (Section 1.1 / 3.1): the exact baseline
//               and the n_min base case of Algorithm 4, whose epilogue also
//               folds in the per-level partial results of the recursion
//               (row sum = D_21 + D_C22 at every split).
//
// Tiling (wave64, v_mfma_f32_32x32x16_bf16):
//   * 4 waves per workgroup, 32 queries per wave, 64 keys per step.
//   * S^T = K Q^T is computed, not S: keys run along the MFMA's M dimension and
//     queries along N, so in the accumulator a lane holds 16 keys of ONE query.
//     Row max and row sum are then in-lane reductions plus a single exchange
//     with lane^32, and the accumulator registers, converted to bf16, are
//     already the B operand of O^T += V^T P^T (no LDS round trip for P).
//   * Q stays in registers for the whole pass; K (row-major, padded rows) and
//     V^T (d-major, padded rows, keys stored in the order the P registers have
//     them) are staged in LDS, double buffered; the next tile's global loads
//     are issued before the current tile's MFMAs.
//   * softmax runs in the exp2 domain in fp32; P is rounded to bf16 only as the
//     MFMA operand, the row sum uses the unrounded fp32 values.
#include "attn_common.h"

namespace ha {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kQT = 128;      // queries per workgroup
constexpr int kNT = 256;      // threads
constexpr int kKT = 64;       // keys per step

template <int D>
struct Lds {
  static constexpr int KSTR = (D + 8) * 2;        // bytes per K row (+16: conflict-free 16-byte row reads)
  static constexpr int VSTR = (D + 32) * 2;       // bytes per V row (+64: conflict-free transposing reads)
  static constexpr int K_BYTES = kKT * KSTR;
  static constexpr int V_BYTES = kKT * VSTR;
  static constexpr int BUF = K_BYTES + V_BYTES;
};

__host__ __device__ inline int list_capacity(int b, int m) { return ((b + m + 63) & ~63) + 64; }

template <int D>
__host__ __device__ inline size_t mfma_lds_bytes(int b, int m, int mode) {
  size_t s = 2 * (size_t)Lds<D>::BUF + 64;  // + wave counters
  if (mode == kModeNode) s += (size_t)list_capacity(b, m) * 4;
  return s;
}

template <int D>
struct TileRegs {
  static constexpr int CPR = D / 8;              // 16-byte chunks per K row
  static constexpr int NKC = kKT * CPR / kNT;    // K (and V) chunks per thread
};

template <int D, int MODE>
__global__ __launch_bounds__(kNT, 2) void attn_mfma_kernel(AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using L = Lds<D>;
  using TR = TileRegs<D>;
  constexpr int KS = D / 16;  // MFMA k-steps of the score product
  constexpr int DT = D / 32;  // 32-wide d tiles of the output

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, h = lane >> 5;

  unsigned char* bufs = smem;
  int32_t* scratch = reinterpret_cast<int32_t*>(smem + 2 * L::BUF);
  int32_t* list = scratch + 16;

  const int bid = logical_block(blockIdx.x, gridDim.x);
  TileWork w;
  int nb, nkeys;
  if (MODE == kModeNode) {
    w = decode_node_tile<kQT>(a, bid);
    nkeys = build_key_list<kNT>(a, w, list, scratch, &nb);
  } else {
    w = decode_exact_tile<kQT>(a, bid);
    nkeys = max(0, w.k1 - w.k0);
    nb = 0x7fffffff;
  }
  const int ntiles = (nkeys + kKT - 1) / kKT;
  const float bias2 = (MODE == kModeNode && a.g.m > 0) ? log2f((float)w.nr.s / (float)a.g.m) : 0.f;

  const uint16_t* Qh = reinterpret_cast<const uint16_t*>(a.Q) + (int64_t)w.bh * a.q_bh_stride;
  const uint16_t* Kh = reinterpret_cast<const uint16_t*>(a.K) + (int64_t)w.bh * a.k_bh_stride;
  const uint16_t* Vh = reinterpret_cast<const uint16_t*>(a.V) + (int64_t)w.bh * a.k_bh_stride;

  // ---- this lane's query row: B operand of S^T = K Q^T, kept in registers ----
  const int r_in_tile = wave * 32 + lq;
  RowDest dest;
  int qrow_load;   // row to load (always a valid row)
  int q_global;    // exact mode: row index within the head, for the causal mask
  if (MODE == kModeNode) {
    dest = node_row_dest(a, w, r_in_tile);
    const int p = w.p0 + (dest.valid ? r_in_tile : 0);
    qrow_load = a.perm_q ? a.perm_q[w.seg_off + p] : w.nr.q_start + p;
    q_global = 0;
  } else {
    dest = RowDest{};
    dest.valid = r_in_tile < w.rows_valid;
    q_global = w.q0 + r_in_tile;
    qrow_load = dest.valid ? q_global : w.q0;
    dest.row_in_head = q_global;
    dest.out_row = (int64_t)w.bh * (a.out_bh_stride / D) + q_global;
  }
  bf16x8 qreg[KS];
  {
    const u32x4* qp = reinterpret_cast<const u32x4*>(Qh + (int64_t)qrow_load * D + 8 * h);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[ks] = __builtin_bit_cast(bf16x8, qp[2 * ks]);
  }

  // ---- tile movers ----
  auto key_row = [&](int kt, int j) -> int {
    if (MODE == kModeNode) return list[kt * kKT + j];
    const int r = w.k0 + kt * kKT + j;
    return r < w.k1 ? r : w.k1 - 1;
  };
  u32x4 kreg[TR::NKC], vreg[TR::NKC];
  auto load_tile = [&](int kt) {
#pragma unroll
    for (int i = 0; i < TR::NKC; ++i) {
      const int c = tid + i * kNT;
      const int key = c / TR::CPR, col = c % TR::CPR;
      const int64_t off = (int64_t)key_row(kt, key) * D + col * 8;
      kreg[i] = *reinterpret_cast<const u32x4*>(Kh + off);
      vreg[i] = *reinterpret_cast<const u32x4*>(Vh + off);
    }
  };
  auto store_tile = [&](unsigned char* buf) {
#pragma unroll
    for (int i = 0; i < TR::NKC; ++i) {
      const int c = tid + i * kNT;
      const int key = c / TR::CPR, col = c % TR::CPR;
      *reinterpret_cast<u32x4*>(buf + key * L::KSTR + col * 16) = kreg[i];
      *reinterpret_cast<u32x4*>(buf + L::K_BYTES + key * L::VSTR + col * 16) = vreg[i];
    }
  };
  // V^T fragments come from the row-major V tile through the transposing LDS
  // read: the 16 lanes of a group fetch a 4-key x 16-d patch (lane i: key i/4,
  // d 4*(i%4)..+3) and lane n receives the 4 keys of column n.
  const int vtr_off = ((lane & 15) >> 2) * L::VSTR + ((lane & 3) * 4 + ((lane >> 4) & 1) * 16) * 2 + (4 * h) * L::VSTR;

  // ---- state ----
  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
  float m_run = -INFINITY;  // running max, log2 domain
  float l_run = 0.f;        // this lane's share of the row sum

  if (ntiles > 0) {
    load_tile(0);
    store_tile(bufs);
  }
  __syncthreads();

  const int wave_q_last = w.q0 + wave * 32 + 31;  // exact mode

  for (int kt = 0; kt < ntiles; ++kt) {
    unsigned char* buf = bufs + (kt & 1) * L::BUF;
    if (kt + 1 < ntiles) load_tile(kt + 1);

    const int key_base = kt * kKT;  // position in the key list / offset from k0
    const bool skip = (MODE == kModeExact) && a.exact_causal && (w.k0 + key_base > wave_q_last);
    if (!skip) {
      // ---- S^T tile: 64 keys x 32 queries; the two 32-key halves are
      // independent accumulators, interleaved so no MFMA waits on the previous one ----
      f32x16 c[2];
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int i = 0; i < 16; ++i) c[sub][i] = 0.f;
      {
        const unsigned char* kp0 = buf + lq * L::KSTR + 16 * h;
        const unsigned char* kp1 = kp0 + 32 * L::KSTR;
#pragma unroll
        for (int kh = 0; kh < KS; kh += 4) {
          bf16x8 kf0[4], kf1[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            kf0[j] = *reinterpret_cast<const bf16x8*>(kp0 + 32 * (kh + j));
            kf1[j] = *reinterpret_cast<const bf16x8*>(kp1 + 32 * (kh + j));
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            c[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf0[j], qreg[kh + j], c[0], 0, 0, 0);
            c[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf1[j], qreg[kh + j], c[1], 0, 0, 0);
          }
        }
      }
      // ---- masks (rare tiles only): tail of the key list, causal diagonal, and a
      // tile that straddles the block / sampled boundary ----
      const bool tail = key_base + kKT > nkeys;
      const bool mixed = (key_base < nb) && (key_base + kKT > nb);
      const bool diag = (MODE == kModeExact) && a.exact_causal && (w.k0 + key_base + kKT - 1 > w.q0 + wave * 32);
      float bias = (key_base >= nb) ? bias2 : 0.f;  // log2 domain, uniform over the tile
      if (tail || mixed || diag) {
        int lim = nkeys;
        if (MODE == kModeExact && a.exact_causal) lim = min(lim, q_global - w.k0 + 1);
        const int lim2 = lim - key_base - 4 * h;           // element i is masked iff koff_i >= lim2
        const int nb2 = mixed ? nb - key_base - 4 * h : 0x7fffffff;
        const float nat_bias = bias2 * kLn2;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int koff = 32 * sub + 8 * (i / 4) + (i % 4);
            float v = c[sub][i];
            if (koff >= nb2) v += nat_bias;
            c[sub][i] = (koff >= lim2) ? -INFINITY : v;
          }
        if (mixed) bias = 0.f;
      }
      // ---- online softmax (exp2 domain) ----
      float mx = fmaxf(c[0][0], c[1][0]);
#pragma unroll
      for (int i = 1; i < 16; ++i) mx = fmaxf(mx, fmaxf(c[0][i], c[1][i]));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, __builtin_fmaf(mx, kLog2e, bias));
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      if (__any(m_new > m_run)) {
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;
        l_run *= alpha;
      }
      m_run = m_new;
      const float shift = bias - m_use;
      bf16x8 pf[4];
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          u32x4 pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(c[sub][8 * jj + 2 * e], kLog2e, shift));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(c[sub][8 * jj + 2 * e + 1], kLog2e, shift));
            l_run += p0 + p1;
            pk[e] = pack_bf16x2(p0, p1);
          }
          pf[2 * sub + jj] = __builtin_bit_cast(bf16x8, pk);
        }
      // ---- O^T += V^T P^T ----
      // slot e of a lane's P registers holds key 8*(e/4) + 4*h + e%4 of the 16-key step
      {
        typedef short s16x4 __attribute__((ext_vector_type(4)));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
        const unsigned char* vb = buf + L::K_BYTES + vtr_off;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            const unsigned char* vp = vb + (16 * j) * L::VSTR + (32 * dt) * 2;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vp));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vp + 8 * L::VSTR));
            const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf[j], o[dt], 0, 0, 0);
          }
        }
      }
    }
    if (kt + 1 < ntiles) store_tile(bufs + ((kt + 1) & 1) * L::BUF);
    __syncthreads();
  }

  // ---- epilogue ----
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const bool empty = !(l_tot > 0.f);
  const float inv = empty ? 0.f : 1.f / l_tot;
  float lse_own = empty ? -INFINITY : (m_run + log2f(l_tot)) * kLn2;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] *= inv;

  if (!dest.valid) return;

  if (MODE == kModeNode && a.part_o != nullptr) {
    float* po = a.part_o + dest.part_row * D;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const f32x4 v = {o[dt][4 * g4], o[dt][4 * g4 + 1], o[dt][4 * g4 + 2], o[dt][4 * g4 + 3]};
        *reinterpret_cast<f32x4*>(po + 32 * dt + 8 * g4 + 4 * h) = v;
      }
    if (h == 0) a.part_l[dest.part_row] = lse_own;
    return;
  }

  if (MODE == kModeExact && a.merge_levels > 0) {
    float mx, den;
    const float Lm = merged_lse(a, w.bh, dest.row_in_head, lse_own, &mx, &den);
    const float w_own = (lse_own == -INFINITY) ? 0.f : expf(lse_own - mx) / den;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][i] *= w_own;
    for (int l = 0; l < a.merge_levels; ++l) {
      int64_t pr;
      if (!level_touches(a.g, w.bh, dest.row_in_head, l, &pr)) continue;
      const float lp = a.part_l[pr];
      if (lp == -INFINITY) continue;
      const float wl = expf(lp - mx) / den;
      const float* po = a.part_o + pr * D;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const f32x4 v = *reinterpret_cast<const f32x4*>(po + 32 * dt + 8 * g4 + 4 * h);
          o[dt][4 * g4] += wl * v.x;
          o[dt][4 * g4 + 1] += wl * v.y;
          o[dt][4 * g4 + 2] += wl * v.z;
          o[dt][4 * g4 + 3] += wl * v.w;
        }
    }
    lse_own = Lm;
  }

  if (a.out != nullptr) {
    uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + dest.out_row * D;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        u32x2 v;
        v.x = pack_bf16x2(o[dt][4 * g4], o[dt][4 * g4 + 1]);
        v.y = pack_bf16x2(o[dt][4 * g4 + 2], o[dt][4 * g4 + 3]);
        *reinterpret_cast<u32x2*>(op + 32 * dt + 8 * g4 + 4 * h) = v;
      }
  }
  if (a.lse != nullptr && h == 0) a.lse[dest.out_row] = lse_own;
}

template <int D, int MODE>
static int launch_one(const AttnArgs& a, int grid, hipStream_t st) {
  const size_t lds = mfma_lds_bytes<D>(a.g.b, a.g.m, MODE);
  static bool configured = false;  // per instantiation
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_kernel<D, MODE>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
      (void)hipGetLastError();
      return HA_ERR_LAUNCH;
    }
    configured = true;
  }
  hipLaunchKernelGGL((attn_mfma_kernel<D, MODE>), dim3((unsigned)grid), dim3(kNT), lds, st, a);
  return check_launch();
}

int launch_attn_mfma(const AttnArgs& a, int mode, hipStream_t st) {
  if (a.g.dtype != HA_BF16) return HA_ERR_DTYPE;
  const int grid = mode == kModeNode ? node_grid<kQT>(a.g) : exact_grid<kQT>(a);
  if (grid <= 0) return HA_OK;
  if (a.g.d == 128) return mode == kModeNode ? launch_one<128, kModeNode>(a, grid, st) : launch_one<128, kModeExact>(a, grid, st);
  if (a.g.d == 64) return mode == kModeNode ? launch_one<64, kModeNode>(a, grid, st) : launch_one<64, kModeExact>(a, grid, st);
  return HA_ERR_SHAPE;
}

}  // namespace ha
