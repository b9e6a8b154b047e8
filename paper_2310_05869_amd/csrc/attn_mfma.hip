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
#include <type_traits>

#include "attn_common.h"

namespace ha {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kKT = 64;       // keys per step

template <int D>
struct Lds {
  static constexpr int KSTR = (D + 8) * 2;        // bytes per K row (+16: conflict-free 16-byte row reads)
  static constexpr int VSTR = (D + 32) * 2;       // bytes per V row (+64: conflict-free transposing reads)
  static constexpr int K_BYTES = kKT * KSTR;
  static constexpr int V_BYTES = kKT * VSTR;
  static constexpr int BUF = K_BYTES + V_BYTES;
};

// Epilogue staging per wave: 32 fp32 rows (padded), 32 x kMaxFold merge weights, 32 row ids,
// kMaxFold partial-row bases.
constexpr int kMaxFold = 8;
template <int D>
struct EpLds {
  static constexpr int ROW = D * 4 + 16;
  static constexpr int WAVE = 32 * ROW + 32 * kMaxFold * 4 + 32 * 8 + kMaxFold * 8;
};

__host__ __device__ inline int list_capacity(int b, int m) { return ((b + m + 63) & ~63) + 64; }

template <int D>
__host__ __device__ inline size_t mfma_lds_bytes(int b, int m, int mode) {
  size_t s = 2 * (size_t)Lds<D>::BUF + 64;  // + wave counters
  if (mode == kModeNode) s += (size_t)list_capacity(b, m) * 4;
  return s;
}

__device__ inline float max3f(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

template <int D, int NT>
struct TileRegs {
  static constexpr int CPR = D / 8;              // 16-byte chunks per K row
  static constexpr int NKC = kKT * CPR / NT;     // K (and V) chunks per thread
};

// NW waves per workgroup (32 queries each); two waves per SIMD at d = 128, three (four-wave workgroups) at d = 64.
// STAMPS: the measuring instantiation, which also records counter readings at its phase
// boundaries (a.stamps); the product launches use STAMPS = false and carry none of it.
template <int D, int MODE, int NW, bool STAMPS = false>
__global__ __launch_bounds__(64 * NW, (D == 64 && NW == 4) ? 3 : 2) void attn_mfma_kernel(AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int kQT = 32 * NW;  // queries per workgroup
  constexpr int kNT = 64 * NW;  // threads
  using L = Lds<D>;
  using TR = TileRegs<D, kNT>;
  constexpr int KS = D / 16;  // MFMA k-steps of the score product
  constexpr int DT = D / 32;  // 32-wide d tiles of the output

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, h = lane >> 5;

  unsigned char* bufs = smem;
  int32_t* scratch = reinterpret_cast<int32_t*>(smem + 2 * L::BUF);
  int32_t* list = scratch + 16;

  long long stamp_c[5] = {0, 0, 0, 0, 0}, stamp_w = 0;
  auto stamp = [&](int i) {
    if constexpr (STAMPS) {
      __builtin_amdgcn_sched_barrier(0);
      stamp_c[i] = (long long)__builtin_readcyclecounter();
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  if constexpr (STAMPS) stamp_w = (long long)wall_clock64();
  stamp(0);

  const int bid = logical_block(blockIdx.x, gridDim.x);
  TileWork w;
  if (MODE == kModeNode) w = decode_node_tile<kQT>(a, bid);
  else w = decode_exact_tile<kQT>(a, bid);

  const uint16_t* Qh = reinterpret_cast<const uint16_t*>(a.Q) + (int64_t)w.bh * a.q_bh_stride;
  const uint16_t* Kh = reinterpret_cast<const uint16_t*>(a.K) + (int64_t)w.bh * a.k_bh_stride;
  const uint16_t* Vh = reinterpret_cast<const uint16_t*>(a.V) + (int64_t)w.bh * a.k_bh_stride;

  // ---- this lane's query row: B operand of S^T = K Q^T, kept in registers.
  // Node mode: the key list's first index values and the row's own index (through P_Q) travel
  // in one round trip; the (gathered) row is then in flight while the key list is built.
  KeyListHead klh{0, 0, 0};
  if (MODE == kModeNode) klh = key_list_fetch<kNT>(a, w);
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

  int nb, nkeys;
  if (MODE == kModeNode) {
    nkeys = build_key_list<kNT>(a, w, list, scratch, &nb, klh);
  } else {
    nkeys = max(0, w.k1 - w.k0);
    nb = 0x7fffffff;
  }
  const int ntiles = (nkeys + kKT - 1) / kKT;
  const float bias2 = (MODE == kModeNode && a.g.m > 0) ? log2f((float)w.nr.s / (float)a.g.m) : 0.f;
  stamp(1);

  // ---- tile movers ----
  // K and V rows are fetched with buffer loads: a 32-bit per-lane byte offset
  // (row * row_bytes + column, from the key list in node mode, fixed in exact
  // mode) plus a scalar offset that advances with the tile.  Offsets past the
  // end of the head's tensor return zeros (such keys are masked by position).
  const uint32_t head_bytes = (uint32_t)((MODE == kModeNode ? a.g.n : a.exact_rows_k) * (D * 2));
  const __amdgpu_buffer_rsrc_t krsrc = __builtin_amdgcn_make_buffer_rsrc((void*)Kh, 0, (int)head_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t vrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)Vh, 0, (int)head_bytes, 0x00020000);
  u32x4 kreg[TR::NKC], vreg[TR::NKC];
  auto load_rows = [&](int kt, const __amdgpu_buffer_rsrc_t& rsrc, u32x4 (&reg)[TR::NKC]) {
#pragma unroll
    for (int i = 0; i < TR::NKC; ++i) {
      const int c = tid + i * kNT;
      const int key = c / TR::CPR, col = c % TR::CPR;
      int voff, soff;
      if (MODE == kModeNode) {
        voff = list[kt * kKT + key] * (D * 2) + col * 16;
        soff = 0;
      } else {
        voff = key * (D * 2) + col * 16;
        soff = (w.k0 + kt * kKT) * (D * 2);
      }
      reg[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, soff, 0);
    }
  };
  auto store_rows = [&](unsigned char* dst, int stride, const u32x4 (&reg)[TR::NKC]) {
#pragma unroll
    for (int i = 0; i < TR::NKC; ++i) {
      const int c = tid + i * kNT;
      const int key = c / TR::CPR, col = c % TR::CPR;
      *reinterpret_cast<u32x4*>(dst + key * stride + col * 16) = reg[i];
    }
  };
  auto kbuf_at = [&](int t) -> unsigned char* { return bufs + (t & 1) * L::BUF; };
  auto vbuf_at = [&](int t) -> unsigned char* { return bufs + (t & 1) * L::BUF + L::K_BYTES; };
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
  // m_run is a reference for the exponentials, not necessarily the running
  // maximum: it is only moved (and the accumulators rescaled) when a row's tile
  // maximum exceeds it by more than 2^8, so after the first tiles the rescale is
  // skipped.  Log2 domain.
  float m_run = -INFINITY;
  float l_run = 0.f;  // this lane's share of the row sum

  // Masks of a score tile (rare tiles only): tail of the key list, causal
  // diagonal, and a tile that straddles the block / sampled boundary.  `bias` is
  // the tile-uniform log2-domain bias (log2(s/m) on sampled tiles).
  auto mask_tile = [&](f32x16 (&c)[2], int t, float& bias) {
    const int key_base = t * kKT;
    const bool tail = key_base + kKT > nkeys;
    const bool mixed = (key_base < nb) && (key_base + kKT > nb);
    const bool diag = (MODE == kModeExact) && a.exact_causal && (w.k0 + key_base + kKT - 1 > w.q0 + wave * 32);
    bias = (key_base >= nb) ? bias2 : 0.f;
    if (tail || mixed || diag) {
      int lim = nkeys;
      if (MODE == kModeExact && a.exact_causal) lim = min(lim, q_global - w.k0 + 1);
      const int lim2 = lim - key_base - 4 * h;  // element i is masked iff koff_i >= lim2
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
  };
  // row maximum of a score tile in the log2 domain (in-lane, then lane ^ 32)
  auto tile_max = [&](const f32x16 (&c)[2], float bias) -> float {
    float mx = max3f(c[0][0], c[1][0], c[0][1]);
#pragma unroll
    for (int i = 1; i < 16; ++i) {
      if (i + 1 < 16) mx = max3f(mx, c[1][i], c[0][i + 1]);
      else mx = fmaxf(mx, c[1][i]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    return __builtin_fmaf(mx, kLog2e, bias);
  };

  // Software pipeline over key tiles: while the matrix cores compute the scores
  // of tile kt+1, the vector ALU turns the scores of tile kt into bf16 weights;
  // while they accumulate P V of tile kt, the vector ALU reduces the row maximum
  // of tile kt+1.  K tile t and V tile t live in buffer (t & 1) of their kind;
  // K runs one tile ahead of V.
  f32x16 c[2];
  float bias = 0.f, t_max = -INFINITY;
  if (ntiles > 0) {
    // all three tiles are requested before any is stored: one global round trip
    u32x4 kreg1[TR::NKC];
    load_rows(0, krsrc, kreg);
    load_rows(0, vrsrc, vreg);
    if (ntiles > 1) load_rows(1, krsrc, kreg1);
    store_rows(kbuf_at(0), L::KSTR, kreg);
    store_rows(vbuf_at(0), L::VSTR, vreg);
    if (ntiles > 1) store_rows(kbuf_at(1), L::KSTR, kreg1);
  }
  __syncthreads();
  if (ntiles > 0) {
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int i = 0; i < 16; ++i) c[sub][i] = 0.f;
    const unsigned char* kp0 = kbuf_at(0) + lq * L::KSTR + 16 * h;
    const unsigned char* kp1 = kp0 + 32 * L::KSTR;
#pragma unroll
    for (int j = 0; j < KS; ++j) {
      c[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(kp0 + 32 * j), qreg[j], c[0], 0, 0, 0);
      c[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(kp1 + 32 * j), qreg[j], c[1], 0, 0, 0);
    }
    mask_tile(c, 0, bias);
    t_max = tile_max(c, bias);
    m_run = t_max;  // the first tile sets the reference: the accumulators are still zero, nothing to rescale
  }

  auto body = [&](int kt, f32x16 (&c)[2], float& bias, f32x16 (&cn)[2], float& bias_n, auto has_next) {
    constexpr bool HN = decltype(has_next)::value;
    const bool more_k = kt + 2 < ntiles;
    // The d = 64 kernels request the next tiles inside the score block (below), in the shadow of its MFMAs:
    // they then fit 168 registers (the node kernel with five spilled ones), a third workgroup per CU, and
    // take 8-10 % less (node launch, base case and exact attention alike).  At d = 128 the same move
    // measures +-0.5 % in exact mode and +7 % in node mode, whose requests first read the key list from
    // LDS: there they are issued here, ahead of the block.
    constexpr bool kRequestInBlock = D == 64;
    if constexpr (!kRequestInBlock) {
      if (more_k) load_rows(kt + 2, krsrc, kreg);
      if (HN) load_rows(kt + 1, vrsrc, vreg);
    }

    if (__any(t_max > m_run + 8.0f)) {
      const float m_new = fmaxf(m_run, t_max);
      const float alpha = __builtin_amdgcn_exp2f(m_run - ((m_new == -INFINITY) ? 0.f : m_new));
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;
      l_run *= alpha;
      m_run = m_new;
    }
    const float shift = bias - ((m_run == -INFINITY) ? 0.f : m_run);

    // ---- scores of tile kt+1 (matrix cores)  ||  weights of tile kt (vector ALU) ----
    // The wave takes issue priority over its SIMD neighbour for this block, its densest one (an MFMA and a
    // slice of exponentials per slot), and gives it back for the P V block, whose slots the neighbour's
    // vector work fills: measured -3 % on the causal base case, -2 % on the node launch (any of the
    // neighbouring placements of the two instructions measured the same; priority during P V alone: no gain;
    // the d = 64 node launch, where vector issue binds, loses 2 % with it and goes without).
    constexpr bool kPrio = D == 128 || MODE == kModeExact;
    bf16x8 pf[4];
    if constexpr (kPrio) __builtin_amdgcn_s_setprio(1);
    if constexpr (kRequestInBlock && HN) {
      // no branch here: past the end the last tile is requested again (and not stored)
      load_rows(min(kt + 2, ntiles - 1), krsrc, kreg);
      load_rows(kt + 1, vrsrc, vreg);
    }
    {
      if (HN) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
          for (int i = 0; i < 16; ++i) cn[sub][i] = 0.f;
        const unsigned char* kp0 = kbuf_at(kt + 1) + lq * L::KSTR + 16 * h;
        const unsigned char* kp1 = kp0 + 32 * L::KSTR;
        bf16x8 kf[2 * KS];
#pragma unroll
        for (int j = 0; j < KS; ++j) {
          kf[2 * j] = *reinterpret_cast<const bf16x8*>(kp0 + 32 * j);
          kf[2 * j + 1] = *reinterpret_cast<const bf16x8*>(kp1 + 32 * j);
        }
#pragma unroll
        for (int j = 0; j < KS; ++j) {
          cn[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[2 * j], qreg[j], cn[0], 0, 0, 0);
          cn[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[2 * j + 1], qreg[j], cn[1], 0, 0, 0);
        }
      }
      float ls[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          u32x4 pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(c[sub][8 * jj + 2 * e], kLog2e, shift));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(c[sub][8 * jj + 2 * e + 1], kLog2e, shift));
            ls[e] += p0 + p1;
            pk[e] = pack_bf16x2(p0, p1);
          }
          pf[2 * sub + jj] = __builtin_bit_cast(bf16x8, pk);
        }
      l_run += (ls[0] + ls[1]) + (ls[2] + ls[3]);
      // keep the weights' computation in this block, next to the MFMAs it hides behind
#pragma unroll
      for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(pf[j]));
      asm volatile("" : "+v"(l_run));
      if (HN) {
        // issue order: a few fragment reads ahead, then per MFMA one more read and
        // a slice of the vector work, which fits inside the MFMA's 32 cycles
        constexpr int kPre = 4;
        constexpr int kValu = (KS == 8) ? 5 : 18;  // d = 128: 5 measured best of 2 ... 9 (by half a percent); d = 64: 18 of 7 ... 26 (by 2 %)
        __builtin_amdgcn_sched_group_barrier(0x100, kPre, 0);
#pragma unroll
        for (int j = 0; j < 2 * KS; ++j) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (j < 2 * KS - kPre) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, kValu, 0);
        }
      }
    }
    if constexpr (kPrio) __builtin_amdgcn_s_setprio(0);
    if (HN) mask_tile(cn, kt + 1, bias_n);

    // ---- O^T += V^T P^T of tile kt (matrix cores)  ||  row maximum of tile kt+1 ----
    // slot e of a lane's P registers holds key 8*(e/4) + 4*h + e%4 of the 16-key step
    {
      typedef short s16x4 __attribute__((ext_vector_type(4)));
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
      const unsigned char* vb = vbuf_at(kt) + vtr_off;
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
      if (HN) t_max = tile_max(cn, bias_n);
      constexpr int kPreV = 8;
      __builtin_amdgcn_sched_group_barrier(0x100, kPreV, 0);
#pragma unroll
      for (int j = 0; j < 4 * DT; ++j) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (2 * j < 8 * DT - kPreV) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        if (HN) __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
      }
    }
    if (more_k) store_rows(kbuf_at(kt + 2), L::KSTR, kreg);
    if (HN) store_rows(vbuf_at(kt + 1), L::VSTR, vreg);
    __syncthreads();
  };
  // two tiles per trip so the score registers swap roles without copies.  The read / MFMA / vector-slice pipeline
  // that the sched_group_barrier calls ask for is formed where a block starts with its first fragment reads: the
  // ISA shows it for the two bodies inside the loop (kt's parity, hence every buffer address, is a constant
  // there), not for the copies of the body after the loop, which handle a list's last one or two tiles.
  f32x16 c2[2];
  float bias_b = 0.f;
  int kt = 0;
  stamp(2);
  for (; kt + 2 < ntiles; kt += 2) {
    body(kt, c, bias, c2, bias_b, std::true_type{});
    body(kt + 1, c2, bias_b, c, bias, std::true_type{});
  }
  if (kt + 2 == ntiles) {
    body(kt, c, bias, c2, bias_b, std::true_type{});
    body(kt + 1, c2, bias_b, c, bias, std::false_type{});
  } else if (kt + 1 == ntiles) {
    body(kt, c, bias, c2, bias_b, std::false_type{});
  }
  stamp(3);

  // ---- epilogue ----
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const bool empty = !(l_tot > 0.f);
  const float inv = empty ? 0.f : 1.f / l_tot;
  float lse_own = empty ? -INFINITY : (m_run + log2f(l_tot)) * kLn2;
  // Where the row goes: a partial result of the causal recursion (node mode) or
  // the final output; in exact mode the partial results of every level of
  // Algorithm 4 are folded in first (row sum = D_21 + D_C22 at every split).
  //
  // The wave's 32 rows are transposed through LDS in fp32 (free now: the last
  // barrier of the loop is behind every wave), so that rows leave, and partial
  // rows arrive, as whole 16-byte pieces on consecutive lanes.
  const bool to_partial = (MODE == kModeNode) && a.part_o != nullptr;
  unsigned char* ep = smem + wave * EpLds<D>::WAVE;
  float* ep_w = reinterpret_cast<float*>(ep + 32 * EpLds<D>::ROW);
  int64_t* ep_rows = reinterpret_cast<int64_t*>(ep + 32 * EpLds<D>::ROW + 32 * kMaxFold * 4);
  int64_t* ep_pr = ep_rows + 32;

  // Levels folded row-major below (up to kMaxFold of them).  The 32 rows of a wave
  // lie in one n_min block, so every level treats them alike: either none of
  // them belongs to its off-diagonal node, or they are 32 consecutive partial rows.
  const bool fold = MODE == kModeExact && a.merge_levels > 0;
  const bool fold_rows = fold && a.merge_levels <= kMaxFold;
  uint32_t touched = 0;
  int nfold = 0;  // number of touched levels
  int64_t pr0[kMaxFold];
  float scale_own = inv;
  if (fold_rows) {
    const int i0 = w.q0 + 32 * __builtin_amdgcn_readfirstlane(wave);
    float lp[kMaxFold];
#pragma unroll
    for (int u = 0; u < kMaxFold; ++u) {
      lp[u] = -INFINITY;
      pr0[u] = 0;
      int64_t pr;
      if (u < a.merge_levels && level_touches(a.g, w.bh, i0, u, &pr)) {
        touched |= 1u << u;
        pr0[u] = pr;
        if (dest.valid) lp[u] = a.part_l[pr + lq];
      }
    }
    float mx = lse_own;
#pragma unroll
    for (int u = 0; u < kMaxFold; ++u) mx = fmaxf(mx, lp[u]);
    float w_own = 0.f, wl[kMaxFold];
#pragma unroll
    for (int u = 0; u < kMaxFold; ++u) wl[u] = 0.f;
    if (mx != -INFINITY) {
      const float e_own = expf(lse_own - mx);
      float den = e_own;
#pragma unroll
      for (int u = 0; u < kMaxFold; ++u) {
        wl[u] = expf(lp[u] - mx);
        den += wl[u];
      }
      const float rden = 1.f / den;
      w_own = e_own * rden;
#pragma unroll
      for (int u = 0; u < kMaxFold; ++u) wl[u] *= rden;
      lse_own = mx + logf(den);
    }
    scale_own = inv * w_own;
    // weights and partial-row bases of the touched levels, compacted (the set
    // of touched levels is the same for the whole wave)
#pragma unroll
    for (int u = 0; u < kMaxFold; ++u)
      if ((touched >> u) & 1u) {
        if (h == 0) ep_w[lq * kMaxFold + nfold] = wl[u];
        if (lane == 0) ep_pr[nfold] = pr0[u];
        ++nfold;
      }
  }
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] *= scale_own;

  if (fold && !fold_rows && dest.valid) {
    // deeper recursions than kMaxFold levels: fold in the accumulator layout
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
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int64_t at = pr * D + 32 * dt + 8 * g4 + 4 * h;
          const u32x2 raw = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint16_t*>(a.part_o) + at);
          const f32x4 v = {__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xFFFF0000u),
                           __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xFFFF0000u)};
          o[dt][4 * g4] += wl * v.x;
          o[dt][4 * g4 + 1] += wl * v.y;
          o[dt][4 * g4 + 2] += wl * v.z;
          o[dt][4 * g4 + 3] += wl * v.w;
        }
    }
    lse_own = Lm;
  }
  float* lse_dst = to_partial ? a.part_l : a.lse;
  const int64_t row_dst = to_partial ? dest.part_row : dest.out_row;
  if (lse_dst != nullptr && dest.valid && h == 0) lse_dst[row_dst] = lse_own;

  unsigned char* dst_base = to_partial ? reinterpret_cast<unsigned char*>(a.part_o) : reinterpret_cast<unsigned char*>(a.out);
  if (dst_base == nullptr) return;
  const bool out_fp32 = to_partial && !a.part_bf16;  // the stage calls take their partial rows in fp32
  constexpr int rs = EpLds<D>::ROW;
  if (h == 0) ep_rows[lq] = dest.valid ? row_dst : (int64_t)-1;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int col = 32 * dt + 8 * g4 + 4 * h;
      const f32x4 v = {o[dt][4 * g4], o[dt][4 * g4 + 1], o[dt][4 * g4 + 2], o[dt][4 * g4 + 3]};
      *reinterpret_cast<f32x4*>(ep + lq * rs + col * 4) = v;
    }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  constexpr int CH = D / 8;  // 8-element pieces per row
  // NF = number of partial rows folded into every row (bf16 rows of the node launch); a compile-time
  // count, and the pieces of a lane walked in groups whose partial-row loads are ALL issued before
  // the first is consumed: one global round trip per group instead of one per piece.  The loads are
  // unconditional (a row that is not stored re-reads the wave's first row) and only the stores are
  // guarded: with loads under a branch the compiler's wait counts fall back to "everything", which
  // also waits for the previous piece's stores to reach memory.
  if (ep_rows[0] < 0) return;  // a wave whose rows all lie past the end (valid rows are a prefix)
  auto drain = [&](auto nf_tag) {
    constexpr int NF = decltype(nf_tag)::value;
    constexpr int IT = 32 * CH / 64;                 // pieces per lane
    constexpr int GROUP = NF <= 4 ? IT : IT / 2;     // 16-byte loads in flight per lane: GROUP * NF <= 32
    const uint16_t* prow[NF > 0 ? NF : 1];
#pragma unroll
    for (int c = 0; c < NF; ++c) prow[c] = reinterpret_cast<const uint16_t*>(a.part_o) + ep_pr[c] * D;
#pragma unroll
    for (int g0 = 0; g0 < IT; g0 += GROUP) {
      int64_t r64[GROUP];
      u32x4 raw[GROUP][NF > 0 ? NF : 1];
#pragma unroll
      for (int it = 0; it < GROUP; ++it) {
        const int idx = lane + 64 * (g0 + it);
        const int row = idx / CH, ch = idx % CH;
        r64[it] = ep_rows[row];
        const int row_ld = r64[it] >= 0 ? row : 0;
#pragma unroll
        for (int c = 0; c < NF; ++c) raw[it][c] = *reinterpret_cast<const u32x4*>(prow[c] + row_ld * D + ch * 8);
      }
#pragma unroll
      for (int it = 0; it < GROUP; ++it) {
        const int idx = lane + 64 * (g0 + it);
        const int row = idx / CH, ch = idx % CH;
        f32x4 v0 = *reinterpret_cast<const f32x4*>(ep + row * rs + ch * 32);
        f32x4 v1 = *reinterpret_cast<const f32x4*>(ep + row * rs + ch * 32 + 16);
#pragma unroll
        for (int c = 0; c < NF; ++c) {
          float wl = ep_w[row * kMaxFold + c];
          const u32x4 q = raw[it][c];
          f32x4 p0 = {__uint_as_float(q.x << 16), __uint_as_float(q.x & 0xFFFF0000u),
                      __uint_as_float(q.y << 16), __uint_as_float(q.y & 0xFFFF0000u)};
          f32x4 p1 = {__uint_as_float(q.z << 16), __uint_as_float(q.z & 0xFFFF0000u),
                      __uint_as_float(q.w << 16), __uint_as_float(q.w & 0xFFFF0000u)};
          if (!(wl != 0.f)) {  // a partial with an empty row sum carries no defined values
            p0 = (f32x4){0.f, 0.f, 0.f, 0.f};
            p1 = p0;
            wl = 0.f;
          }
          v0 += wl * p0;
          v1 += wl * p1;
        }
        if (r64[it] < 0) continue;
        if (out_fp32) {
          f32x4* dp = reinterpret_cast<f32x4*>(dst_base + (r64[it] * D + ch * 8) * 4);
          dp[0] = v0;
          dp[1] = v1;
          continue;
        }
        const u32x4 pk = {pack_bf16x2(v0.x, v0.y), pack_bf16x2(v0.z, v0.w), pack_bf16x2(v1.x, v1.y), pack_bf16x2(v1.z, v1.w)};
        *reinterpret_cast<u32x4*>(dst_base + (r64[it] * D + ch * 8) * 2) = pk;
        if (!to_partial && a.out_f32 != nullptr) {  // unrounded copy of the final output, for the backward's delta
          f32x4* fp = reinterpret_cast<f32x4*>(a.out_f32 + r64[it] * D + ch * 8);
          fp[0] = v0;
          fp[1] = v1;
        }
      }
    }
  };
  if (MODE == kModeExact) {
    switch (nfold) {
      case 0: drain(std::integral_constant<int, 0>{}); break;
      case 1: drain(std::integral_constant<int, 1>{}); break;
      case 2: drain(std::integral_constant<int, 2>{}); break;
      case 3: drain(std::integral_constant<int, 3>{}); break;
      case 4: drain(std::integral_constant<int, 4>{}); break;
      case 5: drain(std::integral_constant<int, 5>{}); break;
      case 6: drain(std::integral_constant<int, 6>{}); break;
      case 7: drain(std::integral_constant<int, 7>{}); break;
      default: drain(std::integral_constant<int, 8>{}); break;
    }
  } else {
    drain(std::integral_constant<int, 0>{});
  }
  if constexpr (STAMPS) {
    stamp(4);
    if (tid == 0 && a.stamps != nullptr) {
      long long* rec = a.stamps + (int64_t)kStampWords * bid;
#pragma unroll
      for (int i = 0; i < 5; ++i) rec[i] = stamp_c[i];
      rec[5] = stamp_w;
      rec[6] = (long long)wall_clock64();
      // where it ran: the hardware id register (wave, SIMD, CU, shader engine) and the XCD number
      const unsigned hw = __builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));   // HW_ID, all 32 bits
      const unsigned xcc = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));  // XCC_ID, bits 0-3
      rec[7] = (long long)(ntiles & 0xffff) | ((long long)hw << 16) | ((long long)(xcc & 15u) << 48);
    }
  }
}

template <int D, int MODE, int NW, bool STAMPS = false>
static int launch_one(const AttnArgs& a, hipStream_t st) {
  const int64_t grid = MODE == kModeNode ? node_grid<32 * NW>(a.g) : exact_grid<32 * NW>(a);
  if (grid <= 0) return HA_OK;
  if (grid > kMaxGrid) return HA_ERR_SHAPE;
  size_t lds = mfma_lds_bytes<D>(a.g.b, a.g.m, MODE);
  if (lds < (size_t)NW * EpLds<D>::WAVE) lds = (size_t)NW * EpLds<D>::WAVE;
  static std::atomic<uint64_t> lds_set{0};  // per instantiation: devices on which the LDS limit is raised
  if (allow_full_lds(reinterpret_cast<const void*>(&attn_mfma_kernel<D, MODE, NW, STAMPS>), lds_set) != HA_OK) return HA_ERR_LAUNCH;
  hipLaunchKernelGGL((attn_mfma_kernel<D, MODE, NW, STAMPS>), dim3((unsigned)grid), dim3(64 * NW), lds, st, a);
  return check_launch();
}

// Waves per workgroup: node tiles (short key loops) use 4, two workgroups per
// CU, so one workgroup's gathers overlap the other's MFMAs; exact attention and
// the causal base case (long key loops) can share each K / V tile among 8 waves.
#ifndef HA_NW_NODE
#define HA_NW_NODE 4
#endif
#ifndef HA_NW_EXACT
#define HA_NW_EXACT 4
#endif

// Exact attention over long key ranges, causal or not, shares each K / V tile among 8
// waves (one workgroup per CU): 3-4 % faster there at d = 128; the short
// loops of the base case prefer two 4-wave workgroups per CU.
constexpr int kWideExactMinRows = 8192;

int64_t attn_mfma_grid(const AttnArgs& a, int mode) {
  return mode == kModeNode ? node_grid<32 * HA_NW_NODE>(a.g) : exact_grid<32 * HA_NW_EXACT>(a);
}

int launch_attn_mfma(const AttnArgs& a, int mode, hipStream_t st) {
  if (a.g.dtype != HA_BF16) return HA_ERR_DTYPE;
  if (mode == kModeExact && a.merge_levels > 0 && !a.part_bf16) return HA_ERR_DTYPE;  // this kernel folds bf16 partial rows
  if (a.stamps != nullptr) {  // the measuring instantiations: the four-wave forms the forward pass launches
    if (a.g.d == 128)
      return mode == kModeNode ? launch_one<128, kModeNode, HA_NW_NODE, true>(a, st) : launch_one<128, kModeExact, HA_NW_EXACT, true>(a, st);
    if (a.g.d == 64)
      return mode == kModeNode ? launch_one<64, kModeNode, HA_NW_NODE, true>(a, st) : launch_one<64, kModeExact, HA_NW_EXACT, true>(a, st);
    return HA_ERR_SHAPE;
  }
  const bool wide = mode == kModeExact && a.merge_levels == 0 &&
                    a.exact_block >= kWideExactMinRows && a.exact_rows_q >= kWideExactMinRows;
  if (a.g.d == 128) {
    if (mode == kModeNode) return launch_one<128, kModeNode, HA_NW_NODE>(a, st);
    return wide ? launch_one<128, kModeExact, 8>(a, st) : launch_one<128, kModeExact, HA_NW_EXACT>(a, st);
  }
  if (a.g.d == 64) {
    if (mode == kModeNode) return launch_one<64, kModeNode, HA_NW_NODE>(a, st);
    return launch_one<64, kModeExact, HA_NW_EXACT>(a, st);  // no gain from the wide form at d = 64
  }
  return HA_ERR_SHAPE;
}

}  // namespace ha
