// fp32 attention kernel without matrix cores: the arithmetic path for HA_FP32
// tensors (all products and sums in fp32 FMA), with the same node / exact modes
// and the same outputs as the bf16 MFMA kernel.  It also accepts bf16 tensors,
// which makes it a second, independently written evaluation of the same tiles.
//
// One thread owns one query row (q and the output accumulator live in its
// registers); a workgroup of 64 rows shares 32-key tiles of K and V staged in
// LDS as fp32, which every lane reads at the same address (LDS broadcast).
#include "attn_common.h"

namespace ha {

constexpr int kGQT = 64;  // queries (= threads) per workgroup
constexpr int kGKT = 32;  // keys per step

__host__ __device__ inline size_t generic_lds_bytes(int d, int b, int m, int mode) {
  size_t s = (size_t)2 * kGKT * d * 4 + 64;
  if (mode == kModeNode) s += (size_t)(((b + m + 63) & ~63) + 64) * 4;
  return s;
}

template <typename T, int D, int MODE>
__global__ __launch_bounds__(kGQT) void attn_generic_kernel(AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* Ks = reinterpret_cast<float*>(smem);
  float* Vs = Ks + kGKT * D;
  int32_t* scratch = reinterpret_cast<int32_t*>(Vs + kGKT * D);
  int32_t* list = scratch + 16;

  const int tid = threadIdx.x;
  TileWork w;
  int nb, nkeys;
  if (MODE == kModeNode) {
    w = decode_node_tile<kGQT>(a, blockIdx.x);
    nkeys = build_key_list<kGQT>(a, w, list, scratch, &nb);
  } else {
    w = decode_exact_tile<kGQT>(a, blockIdx.x);
    nkeys = max(0, w.k1 - w.k0);
    nb = 0x7fffffff;
  }
  const int ntiles = (nkeys + kGKT - 1) / kGKT;
  const float bias = (MODE == kModeNode && a.g.m > 0) ? logf((float)w.nr.s / (float)a.g.m) : 0.f;

  const T* Qh = reinterpret_cast<const T*>(a.Q) + (int64_t)w.bh * a.q_bh_stride;
  const T* Kh = reinterpret_cast<const T*>(a.K) + (int64_t)w.bh * a.k_bh_stride;
  const T* Vh = reinterpret_cast<const T*>(a.V) + (int64_t)w.bh * a.k_bh_stride;

  RowDest dest;
  int qrow_load, q_global = 0;
  if (MODE == kModeNode) {
    dest = node_row_dest(a, w, tid);
    const int p = w.p0 + (dest.valid ? tid : 0);
    qrow_load = a.perm_q ? a.perm_q[w.seg_off + p] : w.nr.q_start + p;
  } else {
    dest = RowDest{};
    dest.valid = tid < w.rows_valid;
    q_global = w.q0 + tid;
    qrow_load = dest.valid ? q_global : w.q0;
    dest.row_in_head = q_global;
    dest.out_row = (int64_t)w.bh * (a.out_bh_stride / D) + q_global;
  }

  float q[D], o[D];
#pragma unroll
  for (int c = 0; c < D; ++c) {
    q[c] = load_elem<T>(Qh + (int64_t)qrow_load * D + c);
    o[c] = 0.f;
  }
  float m_run = -INFINITY, l_run = 0.f;

  for (int kt = 0; kt < ntiles; ++kt) {
    __syncthreads();
    for (int e = tid; e < kGKT * D; e += kGQT) {
      const int j = e / D, c = e % D;
      int krow;
      if (MODE == kModeNode) {
        krow = list[kt * kGKT + j];
      } else {
        krow = w.k0 + kt * kGKT + j;
        krow = krow < w.k1 ? krow : w.k1 - 1;
      }
      Ks[e] = load_elem<T>(Kh + (int64_t)krow * D + c);
      Vs[e] = load_elem<T>(Vh + (int64_t)krow * D + c);
    }
    __syncthreads();

    float sc[kGKT];
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < kGKT; ++j) {
      float dot = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) dot = __builtin_fmaf(q[c], Ks[j * D + c], dot);
      const int kpos = kt * kGKT + j;
      dot += (kpos >= nb) ? bias : 0.f;
      bool masked = kpos >= nkeys;
      if (MODE == kModeExact && a.exact_causal) masked = masked || (w.k0 + kpos > q_global);
      sc[j] = masked ? -INFINITY : dot;
      mx = fmaxf(mx, sc[j]);
    }
    const float m_new = fmaxf(m_run, mx);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = expf(m_run - m_use);
    l_run *= alpha;
#pragma unroll
    for (int c = 0; c < D; ++c) o[c] *= alpha;
    m_run = m_new;
#pragma unroll
    for (int j = 0; j < kGKT; ++j) {
      const float p = expf(sc[j] - m_use);
      l_run += p;
#pragma unroll
      for (int c = 0; c < D; ++c) o[c] = __builtin_fmaf(p, Vs[j * D + c], o[c]);
    }
  }

  const bool empty = !(l_run > 0.f);
  const float inv = empty ? 0.f : 1.f / l_run;
  float lse_own = empty ? -INFINITY : m_run + logf(l_run);
#pragma unroll
  for (int c = 0; c < D; ++c) o[c] *= inv;
  if (!dest.valid) return;

  if (MODE == kModeNode && a.part_o != nullptr) {
    float* po = reinterpret_cast<float*>(a.part_o) + dest.part_row * D;
#pragma unroll
    for (int c = 0; c < D; c += 4)
      *reinterpret_cast<float4*>(po + c) = make_float4(o[c], o[c + 1], o[c + 2], o[c + 3]);
    a.part_l[dest.part_row] = lse_own;
    return;
  }

  if (MODE == kModeExact && a.merge_levels > 0) {
    float mx, den;
    const float Lm = merged_lse(a, w.bh, dest.row_in_head, lse_own, &mx, &den);
    const float w_own = (lse_own == -INFINITY) ? 0.f : expf(lse_own - mx) / den;
#pragma unroll
    for (int c = 0; c < D; ++c) o[c] *= w_own;
    for (int l = 0; l < a.merge_levels; ++l) {
      int64_t pr;
      if (!level_touches(a.g, w.bh, dest.row_in_head, l, &pr)) continue;
      const float lp = a.part_l[pr];
      if (lp == -INFINITY) continue;
      const float wl = expf(lp - mx) / den;
      const float* po = reinterpret_cast<const float*>(a.part_o) + pr * D;
#pragma unroll
      for (int c = 0; c < D; c += 4) {
        const float4 v = *reinterpret_cast<const float4*>(po + c);
        o[c] += wl * v.x;
        o[c + 1] += wl * v.y;
        o[c + 2] += wl * v.z;
        o[c + 3] += wl * v.w;
      }
    }
    lse_own = Lm;
  }

  if (a.out != nullptr) {
    if (sizeof(T) == 4) {
      float* op = reinterpret_cast<float*>(a.out) + dest.out_row * D;
#pragma unroll
      for (int c = 0; c < D; c += 4)
        *reinterpret_cast<float4*>(op + c) = make_float4(o[c], o[c + 1], o[c + 2], o[c + 3]);
    } else {
      uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + dest.out_row * D;
#pragma unroll
      for (int c = 0; c < D; c += 4) {
        uint2 v;
        v.x = pack_bf16x2(o[c], o[c + 1]);
        v.y = pack_bf16x2(o[c + 2], o[c + 3]);
        *reinterpret_cast<uint2*>(op + c) = v;
      }
    }
  }
  if (a.lse != nullptr) a.lse[dest.out_row] = lse_own;
}

template <typename T, int D, int MODE>
static int launch_generic_one(const AttnArgs& a, int grid, hipStream_t st) {
  const size_t lds = generic_lds_bytes(D, a.g.b, a.g.m, MODE);
  static std::atomic<uint64_t> lds_set{0};  // per instantiation: devices on which the LDS limit is raised
  if (allow_full_lds(reinterpret_cast<const void*>(&attn_generic_kernel<T, D, MODE>), lds_set) != HA_OK) return HA_ERR_LAUNCH;
  hipLaunchKernelGGL((attn_generic_kernel<T, D, MODE>), dim3((unsigned)grid), dim3(kGQT), lds, st, a);
  return check_launch();
}

template <typename T>
static int launch_generic_t(const AttnArgs& a, int mode, int grid, hipStream_t st) {
  if (a.g.d == 128)
    return mode == kModeNode ? launch_generic_one<T, 128, kModeNode>(a, grid, st)
                             : launch_generic_one<T, 128, kModeExact>(a, grid, st);
  if (a.g.d == 64)
    return mode == kModeNode ? launch_generic_one<T, 64, kModeNode>(a, grid, st)
                             : launch_generic_one<T, 64, kModeExact>(a, grid, st);
  return HA_ERR_SHAPE;
}

int launch_attn_generic(const AttnArgs& a, int mode, hipStream_t st) {
  const int64_t grid64 = mode == kModeNode ? node_grid<kGQT>(a.g) : exact_grid<kGQT>(a);
  if (grid64 <= 0) return HA_OK;
  if (grid64 > kMaxGrid) return HA_ERR_SHAPE;
  const int grid = (int)grid64;
  if (a.g.dtype == HA_FP32) return launch_generic_t<float>(a, mode, grid, st);
  if (a.g.dtype == HA_BF16) return launch_generic_t<uint16_t>(a, mode, grid, st);
  return HA_ERR_DTYPE;
}

}  // namespace ha
