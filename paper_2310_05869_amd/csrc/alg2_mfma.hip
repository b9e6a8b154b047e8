// bf16 MFMA kernels for the estimator of Algorithm 2 as printed and the value
// product of Lemma 2 / Algorithm 3 (the options beside the Section 4 form):
//
//   tau role    log of the unmasked row sum <1 - M^H_j, A_j> of the rows j in T
//               (Algorithm 2's tau is their maximum): 128 rows of T per
//               workgroup against every key of the head, keys of the row's own
//               sorted block left out.
//   main role   for 128 queries of one sorted block: the masked row sum over the
//               block's keys, the capped estimate d_i over the uniform samples,
//               d~_i = masked + max(d_i, tau / kappa), and the numerator, either
//               Section 4's (block keys + (n/m) kept samples) or Lemma 2's (rows
//               of V drawn by squared norm, each with its 1 / (m p_l)).
//
// Tiling as in the forward kernel: 4 waves x 32 queries, 64 keys per step,
// S^T = K Q^T with v_mfma_f32_32x32x16_bf16 so that a lane holds 16 keys of one
// query, weights converted to bf16 in place as the B operand of O^T += V^T P^T,
// V^T fragments from the transposing LDS read.  The loop is not software
// pipelined (these are options, not the hot path): the next tile's rows are
// fetched into registers while the current tile is computed.
//
// The key list of the main role has three segments, each padded to whole tiles:
// A the block's keys, B the m uniform samples, C (Lemma 2 only) the m rows drawn
// by squared norm.  An entry is a row index, or its complement when the key is
// to be left out (padding; a sample that falls into the row's own block, the
// factor 1 - M_{i,l_j}); segment C carries a log weight per key.  One running
// reference serves all exponentials (log2 domain, lazily moved as in the forward
// kernel), so the three sums and the numerator share their scale.
#include "alg2_common.h"
#include "attn_common.h"

namespace ha {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

constexpr int kA2KT = 64;    // keys per step
constexpr int kA2QT = 128;   // queries per workgroup
constexpr int kA2NT = 256;   // threads

enum Alg2Role : int { kA2Tau = 0, kA2Main = 1 };

template <int D>
struct A2Lds {
  static constexpr int KSTR = (D + 8) * 2;    // bytes per K row (conflict-free 16-byte row reads)
  static constexpr int VSTR = (D + 32) * 2;   // bytes per V row (conflict-free transposing reads)
  static constexpr int K_BYTES = kA2KT * KSTR;
  static constexpr int V_BYTES = kA2KT * VSTR;
  static constexpr int BUF = K_BYTES + V_BYTES;
  static constexpr int AUX = 2 * kA2KT * 4;   // tau role: sorted block of every key of the two tiles in flight
  static constexpr int EP_ROW = D * 4 + 16;
  static constexpr int EP_WAVE = 32 * EP_ROW + 32 * 8;
};

__host__ __device__ inline int a2_tiles(int count) { return (count + kA2KT - 1) / kA2KT; }

// list entries (main role): segments A, B, C and the log weights of C
__host__ __device__ inline int a2_list_entries(const Geometry& g, int vnorm) {
  return (a2_tiles(g.b) + a2_tiles(g.m) * (vnorm ? 2 : 1)) * kA2KT;
}

template <int D>
__host__ __device__ inline size_t a2_lds_bytes(const Geometry& g, int role, int vnorm) {
  size_t s = 2 * (size_t)A2Lds<D>::BUF + A2Lds<D>::AUX;
  if (role == kA2Main) s += (size_t)a2_list_entries(g, vnorm) * 4 + (vnorm ? (size_t)a2_tiles(g.m) * kA2KT * 4 : 0);
  const size_t ep = 4 * (size_t)A2Lds<D>::EP_WAVE;
  return s > ep ? s : ep;
}

__device__ inline float a2_logaddexp(float x, float y) {
  const float hi = fmaxf(x, y), lo = fminf(x, y);
  if (hi == -INFINITY) return -INFINITY;
  return hi + log1pf(expf(lo - hi));
}

template <int D, int ROLE>
__global__ __launch_bounds__(kA2NT, 2) void alg2_mfma_kernel(Alg2Args a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using L = A2Lds<D>;
  constexpr int KS = D / 16;                 // MFMA k-steps of the score product
  constexpr int DT = D / 32;                 // 32-wide d tiles of the numerator
  constexpr int CPR = D / 8;                 // 16-byte chunks per row
  constexpr int NKC = kA2KT * CPR / kA2NT;   // chunks per thread and tensor
  const Geometry& g = a.g;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, h = lane >> 5;

  unsigned char* bufs = smem;
  int32_t* kblk = reinterpret_cast<int32_t*>(smem + 2 * L::BUF);  // [2][64]
  int32_t* list = kblk + 2 * kA2KT;

  // ---- which rows this workgroup owns ----
  int bh, t = 0, p0 = 0, j0 = 0, rows_valid, split = 0;
  if (ROLE == kA2Main) {
    const int tpb = (g.b + kA2QT - 1) / kA2QT;
    const int per_head = (g.n / g.b) * tpb;
    const int tile = blockIdx.x % per_head;
    bh = blockIdx.x / per_head;
    t = tile / tpb;
    const int chunk = tile % tpb;
    p0 = t * g.b + chunk * kA2QT;
    rows_valid = min(kA2QT, g.b - chunk * kA2QT);
  } else {
    // (head, 128 rows of T, one of kAlg2TauSplits ranges of key tiles)
    const int per_head = (g.m + kA2QT - 1) / kA2QT;
    split = blockIdx.x % kAlg2TauSplits;
    const int rest = blockIdx.x / kAlg2TauSplits;
    bh = rest / per_head;
    j0 = (rest % per_head) * kA2QT;
    rows_valid = min(kA2QT, g.m - j0);
  }
  // bh is a view head: one node of the level (alg2_common.h).  Row indices below are rows of the
  // real head (permutation entries already are; node-local draws get the node's first row added).
  const int64_t hb = (int64_t)bh * g.n;
  const Alg2Node nd = alg2_node(a, bh);
  const int64_t draws = ((int64_t)nd.head * a.total_nodes + nd.heap) * g.m;
  const uint16_t* Qh = reinterpret_cast<const uint16_t*>(a.Q) + (int64_t)nd.head * a.n_full * D;
  const uint16_t* Kh = reinterpret_cast<const uint16_t*>(a.K) + (int64_t)nd.head * a.n_full * D;
  const uint16_t* Vh = reinterpret_cast<const uint16_t*>(a.V) + (int64_t)nd.head * a.n_full * D;

  // ---- this lane's query row: B operand of S^T = K Q^T, kept in registers ----
  const int r_in_tile = wave * 32 + lq;
  const bool valid = r_in_tile < rows_valid;
  const int r_use = valid ? r_in_tile : 0;
  const int qrow = (ROLE == kA2Main) ? a.perm_q[hb + p0 + r_use]
                                     : nd.q_start + a.tau_rows[(int64_t)nd.heap * g.m + j0 + r_use];
  const int my_blk = (ROLE == kA2Tau) ? a.pos_q[hb + (qrow - nd.q_start)] / g.b : 0;
  bf16x8 qreg[KS];
  {
    const u32x4* qp = reinterpret_cast<const u32x4*>(Qh + (int64_t)qrow * D + 8 * h);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[ks] = __builtin_bit_cast(bf16x8, qp[2 * ks]);
  }

  // ---- the keys ----
  const int nA = (ROLE == kA2Main) ? a2_tiles(g.b) : a2_tiles(g.n);  // tau role: every key of the head, in place
  const int nB = (ROLE == kA2Main) ? a2_tiles(g.m) : 0;
  const int nC = (ROLE == kA2Main && a.vnorm) ? a2_tiles(g.m) : 0;
  const int ntiles = nA + nB + nC;
  int kt_lo = 0, kt_hi = ntiles;
  if (ROLE == kA2Tau) {
    kt_lo = (int)((int64_t)ntiles * split / kAlg2TauSplits);
    kt_hi = (int)((int64_t)ntiles * (split + 1) / kAlg2TauSplits);
  }
  const float* bias_c = reinterpret_cast<const float*>(list + (nA + nB + nC) * kA2KT);  // log2-domain weights of segment C
  if (ROLE == kA2Main) {
    int32_t* la = list;
    int32_t* lb = la + nA * kA2KT;
    int32_t* lc = lb + nB * kA2KT;
    float* bc = reinterpret_cast<float*>(lc + nC * kA2KT);
    for (int i = tid; i < nA * kA2KT; i += kA2NT) la[i] = (i < g.b) ? a.perm_k[hb + (int64_t)t * g.b + i] : ~0;
    for (int j = tid; j < nB * kA2KT; j += kA2NT) {
      int e = ~0;
      if (j < g.m) {
        const int row = nd.k_start + a.samples[(int64_t)nd.heap * g.m + j];
        e = (a.samp_blk[draws + j] == t) ? ~row : row;  // factor 1 - M_{i,l_j}
      }
      lb[j] = e;
    }
    for (int j = tid; j < nC * kA2KT; j += kA2NT) {
      lc[j] = (j < g.m) ? nd.k_start + a.vsamp[draws + j] : ~0;
      bc[j] = (j < g.m) ? a.vlogw[draws + j] * kLog2e : 0.f;
    }
    __syncthreads();
  }
  const float ratio = g.m > 0 ? (float)g.n / (float)g.m : 1.f;
  const float log2ratio = log2f(ratio);
  const float floor_term = (ROLE == kA2Main && a.kappa > 0.f)
                               ? a.log_tau[(int64_t)nd.head * a.total_nodes + nd.heap] - logf(a.kappa) : -INFINITY;
  auto need_v = [&](int kt) -> bool { return ROLE == kA2Main && (a.vnorm ? kt >= nA + nB : true); };

  // ---- tile movers (buffer loads: rows past the head read as zeros and are left out by their entries) ----
  const uint32_t head_bytes = (uint32_t)(a.n_full * (D * 2));
  const __amdgpu_buffer_rsrc_t krsrc = __builtin_amdgcn_make_buffer_rsrc((void*)Kh, 0, (int)head_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t vrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)Vh, 0, (int)head_bytes, 0x00020000);
  u32x4 kreg[NKC], vreg[NKC];
  int kb_next = -1;  // tau role: sorted block of key tid of the tile being fetched
  auto load_tile = [&](int kt) {
    const bool with_v = need_v(kt);
#pragma unroll
    for (int i = 0; i < NKC; ++i) {
      const int c = tid + i * kA2NT;
      const int key = c / CPR, col = c % CPR;
      int voff, soff;
      if (ROLE == kA2Main) {
        const int e = list[kt * kA2KT + key];
        voff = (e < 0 ? ~e : e) * (D * 2) + col * 16;
        soff = 0;
      } else {
        voff = key * (D * 2) + col * 16;
        soff = (nd.k_start + kt * kA2KT) * (D * 2);   // keys past the node's end are left out through kblk
      }
      kreg[i] = __builtin_amdgcn_raw_buffer_load_b128(krsrc, voff, soff, 0);
      if (with_v) vreg[i] = __builtin_amdgcn_raw_buffer_load_b128(vrsrc, voff, soff, 0);
    }
    if (ROLE == kA2Tau && tid < kA2KT) {
      const int key = kt * kA2KT + tid;
      kb_next = (key < g.n) ? a.pos_k[hb + key] / g.b : -1;
    }
  };
  auto store_tile = [&](int kt) {
    unsigned char* kbuf = bufs + (kt & 1) * L::BUF;
    unsigned char* vbuf = kbuf + L::K_BYTES;
    const bool with_v = need_v(kt);
#pragma unroll
    for (int i = 0; i < NKC; ++i) {
      const int c = tid + i * kA2NT;
      const int key = c / CPR, col = c % CPR;
      *reinterpret_cast<u32x4*>(kbuf + key * L::KSTR + col * 16) = kreg[i];
      if (with_v) *reinterpret_cast<u32x4*>(vbuf + key * L::VSTR + col * 16) = vreg[i];
    }
    if (ROLE == kA2Tau && tid < kA2KT) kblk[(kt & 1) * kA2KT + tid] = kb_next;
  };
  const int vtr_off = ((lane & 15) >> 2) * L::VSTR + ((lane & 3) * 4 + ((lane >> 4) & 1) * 16) * 2 + (4 * h) * L::VSTR;

  // ---- state ----
  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
  float m_run = -INFINITY;  // reference of every exponential, log2 domain
  float msum = 0.f;         // this lane's share of the masked row sum (tau role: of the unmasked one) / 2^m_run
  float dsum = 0.f;         // this lane's share of (n/m) sum of capped kept samples / 2^m_run
  float log2capw = INFINITY;  // log2 of (n/m) C_i, known once segment A is done

  if (kt_lo < kt_hi) {
    load_tile(kt_lo);
    store_tile(kt_lo);
  }
  __syncthreads();

  for (int kt = kt_lo; kt < kt_hi; ++kt) {
    const bool more = kt + 1 < kt_hi;
    if (more) load_tile(kt + 1);

    if (ROLE == kA2Main && kt == nA && nB > 0) {
      // the masked row sum is complete: the cap C_i of Algorithm 2
      const float mt = msum + __shfl_xor(msum, 32);
      const float log_masked = (mt > 0.f) ? (m_run + log2f(mt)) * kLn2 : -INFINITY;
      if (a.cap_scale > 0.f) {
        const float log_cap = logf(a.cap_scale * (float)g.m / ((float)g.n * logf((float)g.n))) + a2_logaddexp(log_masked, floor_term);
        log2capw = log_cap * kLog2e + log2ratio;
      }
    }

    const unsigned char* kbuf = bufs + (kt & 1) * L::BUF;
    const unsigned char* vbuf = kbuf + L::K_BYTES;
    // ---- scores ----
    f32x16 c[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int i = 0; i < 16; ++i) c[sub][i] = 0.f;
    {
      const unsigned char* kp0 = kbuf + lq * L::KSTR + 16 * h;
      const unsigned char* kp1 = kp0 + 32 * L::KSTR;
#pragma unroll
      for (int j = 0; j < KS; ++j) {
        c[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(kp0 + 32 * j), qreg[j], c[0], 0, 0, 0);
        c[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(kp1 + 32 * j), qreg[j], c[1], 0, 0, 0);
      }
    }
    // ---- log2-domain arguments: score + the key's log weight, -inf where the key is left out.
    // Element i of c[sub] is key 32 sub + 8 (i / 4) + 4 h + i % 4 of the tile.
    const int seg = (ROLE == kA2Tau) ? 0 : (kt < nA ? 0 : (kt < nA + nB ? 1 : 2));
    const float segbias = (seg == 1) ? log2ratio : 0.f;
    float tmax = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int at = 32 * sub + 8 * g4 + 4 * h;
        i32x4 e4;
        f32x4 b4 = {segbias, segbias, segbias, segbias};
        if (ROLE == kA2Main) {
          e4 = *reinterpret_cast<const i32x4*>(list + kt * kA2KT + at);
          if (seg == 2) b4 = *reinterpret_cast<const f32x4*>(bias_c + (kt - nA - nB) * kA2KT + at);
        } else {
          e4 = *reinterpret_cast<const i32x4*>(kblk + (kt & 1) * kA2KT + at);
        }
#pragma unroll
        for (int z = 0; z < 4; ++z) {
          const bool out_of_it = (ROLE == kA2Main) ? (e4[z] < 0) : (e4[z] < 0 || e4[z] == my_blk);
          const float v = out_of_it ? -INFINITY : __builtin_fmaf(c[sub][4 * g4 + z], kLog2e, b4[z]);
          c[sub][4 * g4 + z] = v;
          tmax = fmaxf(tmax, v);
        }
      }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    if (__any(tmax > m_run + 8.0f)) {
      const float m_new = fmaxf(m_run, tmax);
      const float alpha = __builtin_amdgcn_exp2f(m_run - ((m_new == -INFINITY) ? 0.f : m_new));
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;
      msum *= alpha;
      dsum *= alpha;
      m_run = m_new;
    }
    const float mref = (m_run == -INFINITY) ? 0.f : m_run;
    const float capw = __builtin_amdgcn_exp2f(fminf(log2capw - mref, 120.f));  // (n/m) C_i on the scale of the weights
    // ---- weights, sums, and the B operand of the numerator ----
    bf16x8 pf[4];
    float sp = 0.f, sd = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        u32x4 pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p0w = __builtin_amdgcn_exp2f(c[sub][8 * jj + 2 * e] - mref);
          const float p1w = __builtin_amdgcn_exp2f(c[sub][8 * jj + 2 * e + 1] - mref);
          sp += p0w + p1w;
          if (ROLE == kA2Main) sd += fminf(p0w, capw) + fminf(p1w, capw);
          pk[e] = pack_bf16x2(p0w, p1w);
        }
        pf[2 * sub + jj] = __builtin_bit_cast(bf16x8, pk);
      }
    if (seg == 0) msum += sp;
    if (seg == 1) dsum += sd;
    // ---- numerator: O^T += V^T P^T ----
    if (need_v(kt)) {
      typedef short s16x4 __attribute__((ext_vector_type(4)));
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
      const unsigned char* vb = vbuf + vtr_off;
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
    if (more) store_tile(kt + 1);
    __syncthreads();
  }

  // ---- results ----
  const float mt = msum + __shfl_xor(msum, 32);
  if (ROLE == kA2Tau) {
    if (valid && h == 0)
      a.log_unm_parts[((int64_t)split * g.BH + bh) * g.m + j0 + r_in_tile] = (mt > 0.f) ? (m_run + log2f(mt)) * kLn2 : -INFINITY;
    return;
  }
  const float dt_ = dsum + __shfl_xor(dsum, 32);
  const float log_masked = (mt > 0.f) ? (m_run + log2f(mt)) * kLn2 : -INFINITY;
  const float log_d = (dt_ > 0.f) ? (m_run + log2f(dt_)) * kLn2 : -INFINITY;
  const float log_dt = a2_logaddexp(log_masked, fmaxf(log_d, floor_term));   // d~_i = masked + max(d_i, tau / kappa)
  const float f = (m_run == -INFINITY || log_dt == -INFINITY) ? 0.f : expf(m_run * kLn2 - log_dt);
  const int64_t out_row = hb + (qrow - nd.q_start);
  if (valid && h == 0) a.lse[out_row] = log_dt;

  // the wave's 32 rows leave through an fp32 LDS transpose as whole 16-byte pieces
  unsigned char* ep = smem + wave * L::EP_WAVE;
  int64_t* ep_rows = reinterpret_cast<int64_t*>(ep + 32 * L::EP_ROW);
  if (h == 0) ep_rows[lq] = valid ? out_row : (int64_t)-1;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int col = 32 * dt + 8 * g4 + 4 * h;
      const f32x4 v = {o[dt][4 * g4] * f, o[dt][4 * g4 + 1] * f, o[dt][4 * g4 + 2] * f, o[dt][4 * g4 + 3] * f};
      *reinterpret_cast<f32x4*>(ep + lq * L::EP_ROW + col * 4) = v;
    }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  constexpr int CH = D / 8;  // 8-element pieces per row
  uint16_t* outp = reinterpret_cast<uint16_t*>(a.out);
  for (int idx = lane; idx < 32 * CH; idx += 64) {
    const int row = idx / CH, ch = idx % CH;
    const int64_t r64 = ep_rows[row];
    if (r64 < 0) continue;
    const f32x4 v0 = *reinterpret_cast<const f32x4*>(ep + row * L::EP_ROW + ch * 32);
    const f32x4 v1 = *reinterpret_cast<const f32x4*>(ep + row * L::EP_ROW + ch * 32 + 16);
    const u32x4 pk = {pack_bf16x2(v0.x, v0.y), pack_bf16x2(v0.z, v0.w), pack_bf16x2(v1.x, v1.y), pack_bf16x2(v1.z, v1.w)};
    *reinterpret_cast<u32x4*>(outp + r64 * D + ch * 8) = pk;
  }
}

template <int D, int ROLE>
static int launch_a2(const Alg2Args& a, int64_t grid, hipStream_t st) {
  if (grid <= 0) return HA_OK;
  if (grid > kMaxGrid) return HA_ERR_SHAPE;
  const size_t lds = a2_lds_bytes<D>(a.g, ROLE, a.vnorm);
  static std::atomic<uint64_t> lds_set{0};  // per instantiation: devices on which the LDS limit is raised
  if (allow_full_lds(reinterpret_cast<const void*>(&alg2_mfma_kernel<D, ROLE>), lds_set) != HA_OK) return HA_ERR_LAUNCH;
  hipLaunchKernelGGL((alg2_mfma_kernel<D, ROLE>), dim3((unsigned)grid), dim3(kA2NT), lds, st, a);
  return check_launch();
}

// Whether the MFMA kernels take this problem: bf16 tensors, d of 64 or 128, and a key list that fits in LDS.
bool alg2_mfma_supported(const Alg2Args& a) {
  const Geometry& g = a.g;
  if (g.dtype != HA_BF16 || (g.d != 64 && g.d != 128)) return false;
  const size_t lds = g.d == 128 ? a2_lds_bytes<128>(g, kA2Main, a.vnorm) : a2_lds_bytes<64>(g, kA2Main, a.vnorm);
  return lds <= 160 * 1024;
}

int launch_alg2_tau_mfma(const Alg2Args& a, hipStream_t st) {
  const Geometry& g = a.g;
  const int64_t grid = (int64_t)g.BH * ((g.m + kA2QT - 1) / kA2QT) * kAlg2TauSplits;
  return g.d == 128 ? launch_a2<128, kA2Tau>(a, grid, st) : launch_a2<64, kA2Tau>(a, grid, st);
}

int launch_alg2_main_mfma(const Alg2Args& a, hipStream_t st) {
  const Geometry& g = a.g;
  const int tpb = (g.b + kA2QT - 1) / kA2QT;
  const int64_t grid = (int64_t)g.BH * (g.n / g.b) * tpb;
  return g.d == 128 ? launch_a2<128, kA2Main>(a, grid, st) : launch_a2<64, kA2Main>(a, grid, st);
}

}  // namespace ha
