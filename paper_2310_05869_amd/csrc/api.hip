// extern "C" entry points of libhyperattn: argument validation, workspace
// layouts and the launch sequences of a forward and of a backward call.  Everything here is host
// code; it enqueues kernels on the caller's stream and returns.
//
// Launch sequence of hyperattn_forward (Algorithm 3 in its Section 4 form;
// Algorithm 4 when causal):
//   prep        R and the per-node sample indices into the workspace
//   lsh_hash    x2 (Q, K): one pass over all rows; the causal recursion reuses
//               the same codes at every node (same hyperplanes everywhere)
//   seg_sort    all nodes of all levels, Q and K, in one launch
//   attention   all nodes of all levels in one launch (block part + sampled
//               residual, shared normaliser); unmasked problem: final output;
//               causal: partial results per level, in the tensors' dtype
//   base case   causal only: exact causal attention on the n_min diagonal
//               blocks, merging the partial results of every level per row
//
// Launch sequence of hyperattn_backward (gradients of the above with the random
// draws held fixed; every (query, key) pair that occurs contributes on its own,
// given the final log row sums and delta = <dO, O>):
//   delta       row dots of dO and the forward's output
//   dQ          node passes, level by level (query tiles over their key lists),
//               into one accumulated fp32 row per query; then the base-case
//               pass, which adds that row and writes dQ
//   dK, dV      block keys of every node, level by level, into accumulated rows;
//               sampled keys of every node (partial sums per query chunk) and
//               their ordered reduction into the same rows, level by level;
//               then the base-case pass, which adds the rows and writes dK, dV
#include <cmath>
#include <cstring>

#include "ha_common.h"
#include "alg2_common.h"
#include "bwd_common.h"

namespace ha {

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Tensors and float arrays are accessed 16 bytes at a time; index arrays 4 bytes at a time.
static bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
template <typename... P>
static bool any_misaligned16(P... ptrs) { return (misaligned(ptrs, 16) || ...); }
template <typename... P>
static bool any_misaligned4(P... ptrs) { return (misaligned(ptrs, 4) || ...); }

static int make_geometry(const ha_shape* sh, const ha_params* p, Geometry* g) {
  if (!sh || !p) return HA_ERR_NULL;
  if (sh->dtype != HA_BF16 && sh->dtype != HA_FP32) return HA_ERR_DTYPE;
  if (sh->B < 0 || sh->H < 0 || sh->n < 0) return HA_ERR_SHAPE;
  if (sh->d != 64 && sh->d != 128) return HA_ERR_SHAPE;
  if (p->r < 1 || p->r > 8) return HA_ERR_SHAPE;
  if (p->b < 1 || p->b > 4096 || p->m < 0 || p->m > 4096) return HA_ERR_SHAPE;
  if ((int64_t)sh->B * sh->H > (1 << 20) || sh->n > (1 << 22)) return HA_ERR_SHAPE;
  if ((int64_t)sh->B * sh->H * sh->n > (1ll << 30)) return HA_ERR_SHAPE;  // launch grids and row ids are 32-bit
  g->BH = sh->B * sh->H;
  g->n = sh->n;
  g->d = sh->d;
  g->dtype = sh->dtype;
  g->b = p->b;
  g->m = p->m;
  g->r = p->r;
  g->causal = p->causal ? 1 : 0;
  g->n_min = p->n_min;
  g->base_len = 0;
  if (!g->causal) {
    if (sh->n % p->b != 0) return HA_ERR_SHAPE;
    g->levels = 1;
    g->total_nodes = 1;
    g->n_cov = sh->n;
  } else {
    if (p->n_min < 1) return HA_ERR_SHAPE;
    if (sh->n <= p->n_min) {
      g->levels = 0;
      g->total_nodes = 0;
      g->n_cov = 0;
      g->base_len = sh->n;
    } else {
      if (sh->n % p->n_min != 0) return HA_ERR_SHAPE;
      const int ratio = sh->n / p->n_min;
      if ((ratio & (ratio - 1)) != 0) return HA_ERR_SHAPE;
      if (p->n_min % p->b != 0) return HA_ERR_SHAPE;
      int L = 0;
      while ((1 << L) < ratio) ++L;
      g->levels = L;
      g->total_nodes = (1 << L) - 1;
      g->n_cov = sh->n / 2;
      g->base_len = p->n_min;
    }
  }
  if (g->BH == 0 || g->n == 0) {
    g->levels = 0;
    g->total_nodes = 0;
    g->n_cov = 0;
  }
  return HA_OK;
}

static void fill_layout(const Geometry& g, ha_ws_layout* l) {
  std::memset(l, 0, sizeof(*l));
  l->levels = g.levels;
  l->total_nodes = g.total_nodes;
  l->n_cov = g.n_cov;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off = align256(off + bytes);
    return at;
  };
  const size_t rows = (size_t)g.BH * g.n;
  const size_t cov = (size_t)g.levels * g.BH * g.n_cov;
  l->codes_q = take(rows);
  l->codes_k = take(rows);
  l->perm_q = take(cov * 4);
  l->perm_k = take(cov * 4);
  l->pos_k = take(cov * 4);
  l->samples = take((size_t)g.total_nodes * g.m * 4);
  l->samp_blk = take((size_t)g.BH * g.total_nodes * g.m * 4);
  l->proj = take((size_t)g.d * g.r * 4);
  l->sort_hist = take((size_t)seg_sort_chunks(g) * 256 * 4);
  const bool partials = g.causal && g.levels > 0;
  l->part_o = take(partials ? cov * g.d * (g.dtype == HA_BF16 ? 2 : 4) : 0);
  l->part_l = take(partials ? cov * 4 : 0);
  l->total_bytes = off < 256 ? 256 : off;
}

// Definition 1's hyperplane normals: Box-Muller normals from the projection
// stream, rounded to fp32 and then to bf16 (ties to even); returned as bf16 bits.
static uint16_t projection_bits(uint64_t seed, int c, int k) {
  const uint64_t ctr = 2ull * (8ull * (uint64_t)c + (uint64_t)k);
  const double u1 = ((double)(rand_u64(seed, kStreamProjection, ctr) >> 11) + 0.5) * 0x1.0p-53;
  const double u2 = ((double)(rand_u64(seed, kStreamProjection, ctr + 1) >> 11) + 0.5) * 0x1.0p-53;
  const double z = std::sqrt(-2.0 * std::log(u1)) * std::cos(2.0 * M_PI * u2);
  const float f = (float)z;
  uint32_t bits;
  std::memcpy(&bits, &f, 4);
  bits += 0x7FFFu + ((bits >> 16) & 1u);
  return (uint16_t)(bits >> 16);
}

static bool use_mfma(const Geometry& g) { return g.dtype == HA_BF16; }

// ---------------------------------------------------------------------------
// Built-in scratch of hyperattn_forward_static: a fixed device array that takes
// the place of the caller's workspace, for callers that may not allocate.  Every
// GPU the library runs on holds its own copy until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; the device
// address it returns (per device) is what kernels and copies get.
// ---------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_addr[kMaxDevices];

// Device address of `scratch` on the current device (looked up once per device).
static int static_scratch(void** addr) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HA_ERR_LAUNCH;
  void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return HA_ERR_LAUNCH;
    }
    g_scratch_addr[dev].store(p, std::memory_order_release);
  }
  *addr = p;
  return HA_OK;
}

static int run_attention(const AttnArgs& a, int mode, hipStream_t st) {
  return use_mfma(a.g) ? launch_attn_mfma(a, mode, st) : launch_attn_generic(a, mode, st);
}

// Algorithm 4's diagonal blocks: exact causal attention on every block of base_len rows, whose
// epilogue adds the row sums and outputs of the off-diagonal nodes (part_o / part_l of every level).
static AttnArgs base_case_args(const void* Q, const void* K, const void* V, void* out, float* lse, float* out_f32,
                               const Geometry& g, void* part_o, float* part_l) {
  const int64_t head_stride = (int64_t)g.n * g.d;
  AttnArgs a{};
  a.Q = Q;
  a.K = K;
  a.V = V;
  a.q_bh_stride = a.k_bh_stride = head_stride;
  a.out = out;
  a.lse = lse;
  a.out_f32 = out_f32;
  a.out_bh_stride = head_stride;
  a.part_o = part_o;
  a.part_l = part_l;
  a.part_bf16 = g.dtype == HA_BF16;
  a.g = g;
  a.exact_rows_q = a.exact_rows_k = g.n;
  a.exact_block = g.base_len;
  a.exact_causal = 1;
  a.merge_levels = g.levels;
  return a;
}

static int run_base_case(const void* Q, const void* K, const void* V, void* out, float* lse, float* out_f32,
                         const Geometry& g, void* part_o, float* part_l, hipStream_t st, long long* stamps = nullptr) {
  AttnArgs a = base_case_args(Q, K, V, out, lse, out_f32, g, part_o, part_l);
  a.stamps = stamps;
  return run_attention(a, kModeExact, st);
}

// ev, when non-null, receives 6 events recorded on the stream: start, after
// prep, after hashing, after sorting, after the node attention, after the base case.
// node_stamps / base_stamps, when non-null, select the measuring instantiation of the
// node launch / the base-case launch and receive its workgroups' stamp records.
static int forward_impl(const void* Q, const void* K, const void* V, void* out, float* lse, const ha_shape* sh,
                        const ha_params* p, const float* R_dev, const int32_t* samples_dev, void* ws,
                        size_t ws_bytes, void* stream, hipEvent_t* ev = nullptr, float* out_f32 = nullptr,
                        long long* node_stamps = nullptr, long long* base_stamps = nullptr) {
  Geometry g;
  int rc = make_geometry(sh, p, &g);
  if (rc != HA_OK) return rc;
  if (g.BH == 0 || g.n == 0) return HA_OK;
  if (!Q || !K || !V || !out || !lse) return HA_ERR_NULL;
  if (out_f32 && g.dtype != HA_BF16) return HA_ERR_DTYPE;
  if (any_misaligned16(Q, K, V, out, out_f32) || any_misaligned4(lse, R_dev, samples_dev)) return HA_ERR_ALIGN;
  ha_ws_layout lay;
  fill_layout(g, &lay);
  if (!ws) return HA_ERR_NULL;
  if (ws_bytes < lay.total_bytes || ((uintptr_t)ws & 255) != 0) return HA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  unsigned char* base = (unsigned char*)ws;
  uint8_t* codes_q = base + lay.codes_q;
  uint8_t* codes_k = base + lay.codes_k;
  int32_t* perm_q = (int32_t*)(base + lay.perm_q);
  int32_t* perm_k = (int32_t*)(base + lay.perm_k);
  int32_t* pos_k = (int32_t*)(base + lay.pos_k);
  int32_t* samples = (int32_t*)(base + lay.samples);
  int32_t* samp_blk = (int32_t*)(base + lay.samp_blk);
  float* proj = (float*)(base + lay.proj);
  void* part_o = (void*)(base + lay.part_o);
  float* part_l = (float*)(base + lay.part_l);
  const int64_t head_stride = (int64_t)g.n * g.d;
  auto mark = [&](int i) {
    if (ev) (void)hipEventRecord(ev[i], st);
  };

  mark(0);
  if (g.levels > 0) {
    uint16_t Rb[1024];
    if (!R_dev)
      for (int c = 0; c < g.d; ++c)
        for (int k = 0; k < g.r; ++k) Rb[c * g.r + k] = projection_bits(p->seed, c, k);
    rc = launch_prep(proj, R_dev, R_dev ? nullptr : Rb, samples, samples_dev, g, p->seed, st);
    if (rc != HA_OK) return rc;
    mark(1);
    rc = launch_lsh_hash(Q, codes_q, (int64_t)g.BH * g.n, g.d, g.dtype, proj, g.r, st);
    if (rc != HA_OK) return rc;
    rc = launch_lsh_hash(K, codes_k, (int64_t)g.BH * g.n, g.d, g.dtype, proj, g.r, st);
    if (rc != HA_OK) return rc;
    mark(2);
    rc = launch_seg_sort_nodes(codes_q, codes_k, perm_q, perm_k, pos_k, g.m > 0 ? samples : nullptr, samp_blk,
                               (uint32_t*)(base + lay.sort_hist), g, st);
    if (rc != HA_OK) return rc;
    mark(3);

    AttnArgs a{};
    a.Q = Q;
    a.K = K;
    a.V = V;
    a.q_bh_stride = a.k_bh_stride = head_stride;
    a.perm_q = perm_q;
    a.perm_k = perm_k;
    a.pos_k = pos_k;
    a.samples = g.m > 0 ? samples : nullptr;
    a.samp_blk = g.m > 0 ? samp_blk : nullptr;
    a.use_block = 1;
    a.out_bh_stride = head_stride;
    a.scatter_out = 1;
    a.g = g;
    if (g.causal) {
      a.part_o = part_o;
      a.part_l = part_l;
      a.part_bf16 = g.dtype == HA_BF16;
    } else {
      a.out = out;
      a.lse = lse;
      a.out_f32 = out_f32;
    }
    a.stamps = node_stamps;
    rc = run_attention(a, kModeNode, st);
    if (rc != HA_OK) return rc;
  } else {
    mark(1);
    mark(2);
    mark(3);
  }
  mark(4);
  if (g.causal) {
    rc = run_base_case(Q, K, V, out, lse, out_f32, g, part_o, part_l, st, base_stamps);
    if (rc != HA_OK) return rc;
  }
  mark(5);
  return HA_OK;
}

static int stage_geometry(Geometry* g, int groups, int n, int d, int dtype, int b, int m) {
  if (dtype != HA_BF16 && dtype != HA_FP32) return HA_ERR_DTYPE;
  if (d != 64 && d != 128) return HA_ERR_SHAPE;
  if (groups < 0 || n < 0 || b < 1 || b > 4096 || m < 0 || m > 4096) return HA_ERR_SHAPE;
  if (n % b != 0) return HA_ERR_SHAPE;
  std::memset(g, 0, sizeof(*g));
  g->BH = groups;
  g->n = n;
  g->d = d;
  g->dtype = dtype;
  g->b = b;
  g->m = m;
  g->r = 1;
  g->levels = 1;
  g->total_nodes = 1;
  g->n_cov = n;
  return HA_OK;
}

// ---------------------------------------------------------------------------
// Backward pass
// ---------------------------------------------------------------------------
// bf16 tensors: matrix cores; fp32 tensors: the fp32 FMA kernel with the same passes
static int launch_attn_bwd(const BwdArgs& a, int mode, hipStream_t st) {
  return use_mfma(a.f.g) ? launch_attn_bwd_mfma(a, mode, st) : launch_attn_bwd_generic(a, mode, st);
}

static int64_t bwd_sample_rows(const Geometry& g) {
  int64_t rows = 0;
  if (g.m <= 0) return 0;
  for (int l = 0; l < g.levels; ++l) {
    const int nodes = g.causal ? (1 << l) : 1;
    rows += (int64_t)g.BH * nodes * bwd_chunks_per_node(g, l) * g.m;
  }
  return rows;
}

static void fill_bwd_layout(const Geometry& g, ha_bwd_ws_layout* l) {
  std::memset(l, 0, sizeof(*l));
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off = align256(off + bytes);
    return at;
  };
  const size_t rows = (size_t)g.BH * g.n;
  const size_t rowb = (size_t)g.d * 4;
  l->delta = take(rows * 4);
  // accumulated node rows: dQ first, then (dQ being written out) dK in the same region, dV in the second
  l->acc_a = take(g.levels > 0 ? rows * rowb : 0);
  l->acc_b = take(g.levels > 0 ? rows * rowb : 0);
  const size_t srows = (size_t)bwd_sample_rows(g);
  l->samp_k = take(srows * rowb);
  l->samp_v = take(srows * rowb);
  l->total_bytes = off < 256 ? 256 : off;
}

// ev, when non-null, receives 8 events: start, after delta, dQ of the nodes, dQ of the base case (unmasked
// problems: its conversion), dK/dV of the block keys, of the sampled keys (with their reduction), of the base
// case, after the conversion of dK and dV (unmasked problems).
static int backward_impl(const void* Q, const void* K, const void* V, const void* out, const float* out_f32,
                         const float* lse, const void* d_out, void* dQ, void* dK, void* dV, const ha_shape* sh,
                         const ha_params* p,
                         const void* fws, size_t fws_bytes, void* bws, size_t bws_bytes, void* stream,
                         hipEvent_t* ev = nullptr) {
  Geometry g;
  int rc = make_geometry(sh, p, &g);
  if (rc != HA_OK) return rc;
  if (out_f32 && g.dtype != HA_BF16) return HA_ERR_DTYPE;
  if (g.levels > kBwdMaxLevels) return HA_ERR_SHAPE;
  if (g.BH == 0 || g.n == 0) return HA_OK;
  if (!Q || !K || !V || !out || !lse || !d_out || !dQ || !dK || !dV || !fws || !bws) return HA_ERR_NULL;
  if (any_misaligned16(Q, K, V, out, out_f32, d_out, dQ, dK, dV) || any_misaligned4(lse)) return HA_ERR_ALIGN;
  ha_ws_layout lay;
  fill_layout(g, &lay);
  ha_bwd_ws_layout bl;
  fill_bwd_layout(g, &bl);
  if (fws_bytes < lay.total_bytes || ((uintptr_t)fws & 255) != 0) return HA_ERR_WORKSPACE;
  if (bws_bytes < bl.total_bytes || ((uintptr_t)bws & 255) != 0) return HA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const unsigned char* fb = (const unsigned char*)fws;
  unsigned char* bb = (unsigned char*)bws;
  float* delta = (float*)(bb + bl.delta);
  float* acc_a = (float*)(bb + bl.acc_a);
  float* acc_b = (float*)(bb + bl.acc_b);
  float* samp_k = (float*)(bb + bl.samp_k);
  float* samp_v = (float*)(bb + bl.samp_v);
  auto mark = [&](int i) {
    if (ev) (void)hipEventRecord(ev[i], st);
  };

  BwdArgs a{};
  a.f.Q = Q;
  a.f.K = K;
  a.f.V = V;
  a.f.q_bh_stride = a.f.k_bh_stride = a.f.out_bh_stride = (int64_t)g.n * g.d;
  a.f.perm_q = (const int32_t*)(fb + lay.perm_q);
  a.f.perm_k = (const int32_t*)(fb + lay.perm_k);
  a.f.pos_k = (const int32_t*)(fb + lay.pos_k);
  a.f.samples = g.m > 0 ? (const int32_t*)(fb + lay.samples) : nullptr;
  a.f.samp_blk = g.m > 0 ? (const int32_t*)(fb + lay.samp_blk) : nullptr;
  a.f.use_block = 1;
  a.f.g = g;
  a.f.exact_rows_q = a.f.exact_rows_k = g.n;
  a.f.exact_block = g.causal ? g.base_len : g.n;
  a.f.exact_causal = g.causal;
  a.dO = d_out;
  a.lse = lse;
  a.delta = delta;
  {
    int wg = 0;
    int64_t row = 0;
    const int spn = (g.m + 127) / 128;
    for (int l = 0; l < g.levels; ++l) {
      const int nodes = g.causal ? (1 << l) : 1;
      const int cpn = bwd_chunks_per_node(g, l);
      a.samp_wg_off[l] = wg;
      a.samp_row_off[l] = row;
      wg += g.BH * nodes * cpn * spn;
      row += (int64_t)g.BH * nodes * cpn * g.m;
    }
    a.samp_wg_off[g.levels] = wg;
  }

  mark(0);
  rc = launch_bwd_delta(out, out_f32, d_out, delta, (int64_t)g.BH * g.n, g.d, g.dtype, st);
  if (rc != HA_OK) return rc;
  mark(1);
  // node passes: one launch per level, in level order, so that a row's contributions from different levels
  // are added one after the other
  const int64_t wgs_per_level = bwd_grid(a, kBwdDqNode);
  if (wgs_per_level * g.levels > 0x7fffffff) return HA_ERR_SHAPE;
  auto node_levels = [&](int mode) -> int {
    for (int l = 0; l < g.levels; ++l) {
      a.wg_base = (int32_t)(l * wgs_per_level);
      const int r = launch_attn_bwd(a, mode, st);
      if (r != HA_OK) return r;
    }
    return HA_OK;
  };
  a.out1 = acc_a;
  a.out2 = nullptr;
  rc = node_levels(kBwdDqNode);
  if (rc != HA_OK) return rc;
  mark(2);
  if (g.causal) {
    a.fin1 = dQ;
    a.lvl1 = g.levels > 0 ? acc_a : nullptr;
    rc = launch_attn_bwd(a, kBwdDqExact, st);
  } else {  // one node, no base case: its rows are the result
    rc = launch_bwd_convert(acc_a, dQ, g, st);
  }
  if (rc != HA_OK) return rc;
  mark(3);
  a.out1 = acc_a;
  a.out2 = acc_b;
  rc = node_levels(kBwdDkvBlock);
  if (rc != HA_OK) return rc;
  mark(4);
  if (g.levels > 0 && g.m > 0) {
    a.out1 = samp_k;
    a.out2 = samp_v;
    rc = launch_attn_bwd(a, kBwdDkvSamp, st);
    if (rc != HA_OK) return rc;
    for (int l = 0; l < g.levels; ++l) {
      rc = launch_bwd_sample_scatter(a, l, samp_k, samp_v, acc_a, acc_b, st);
      if (rc != HA_OK) return rc;
    }
  }
  mark(5);
  if (g.causal) {
    a.fin1 = dK;
    a.fin2 = dV;
    a.lvl1 = g.levels > 0 ? acc_a : nullptr;
    a.lvl2 = g.levels > 0 ? acc_b : nullptr;
    rc = launch_attn_bwd(a, kBwdDkvExact, st);
    if (rc != HA_OK) return rc;
  }
  mark(6);
  if (!g.causal) {
    rc = launch_bwd_convert(acc_a, dK, g, st);
    if (rc != HA_OK) return rc;
    rc = launch_bwd_convert(acc_b, dV, g, st);
    if (rc != HA_OK) return rc;
  }
  mark(7);
  return HA_OK;
}

// ---------------------------------------------------------------------------
// Algorithm 2 as printed / Lemma 2 options
// ---------------------------------------------------------------------------
static void fill_alg2_layout(const Geometry& g, const ha_ws_layout& fwd, ha_alg2_ws_layout* l) {
  std::memset(l, 0, sizeof(*l));
  size_t off = align256(fwd.total_bytes);
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off = align256(off + bytes);
    return at;
  };
  // per-level regions are sized for the largest level and reused from level to level;
  // per-node regions hold every node of every level
  const size_t view = (size_t)g.BH * g.n_cov;                                   // rows of one level
  const size_t max_nodes = g.levels > 0 ? ((size_t)1 << (g.causal ? g.levels - 1 : 0)) : 0;
  const size_t nodes_all = (size_t)g.BH * g.total_nodes;
  l->forward_bytes = fwd.total_bytes;
  l->pos_q = take(view * 4);
  l->tau_rows = take((size_t)g.total_nodes * g.m * 4);
  l->log_unmasked_t = take((size_t)g.BH * max_nodes * g.m * 4);
  l->log_tau = take(nodes_all * 4);
  l->vnorm_w = take(view * 8);
  l->vnorm_prefix = take(view * 8);
  l->vnorm_samples = take(nodes_all * g.m * 4);
  l->vnorm_logw = take(nodes_all * g.m * 4);
  l->log_unmasked_parts = take((size_t)kAlg2TauSplits * g.BH * max_nodes * g.m * 4);
  l->total_bytes = off;
}

}  // namespace ha

using namespace ha;

extern "C" {

int ha_workspace_layout(const ha_shape* shape, const ha_params* params, ha_ws_layout* layout) {
  if (!layout) return HA_ERR_NULL;
  Geometry g;
  const int rc = make_geometry(shape, params, &g);
  if (rc != HA_OK) return rc;
  fill_layout(g, layout);
  return HA_OK;
}

size_t ha_workspace_bytes(const ha_shape* shape, const ha_params* params) {
  ha_ws_layout l;
  return ha_workspace_layout(shape, params, &l) == HA_OK ? l.total_bytes : 0;
}

int hyperattn_forward(const void* Q, const void* K, const void* V, void* out, float* lse, const ha_shape* shape,
                      const ha_params* params, void* workspace, size_t workspace_bytes, void* stream) {
  return forward_impl(Q, K, V, out, lse, shape, params, nullptr, nullptr, workspace, workspace_bytes, stream);
}

size_t ha_static_scratch_bytes(void) { return kStaticScratchBytes; }

int hyperattn_forward_static(const void* Q, const void* K, const void* V, void* out, float* lse,
                             const ha_shape* shape, const ha_params* params, void* stream) {
  Geometry g;
  const int rc = make_geometry(shape, params, &g);
  if (rc != HA_OK) return rc;
  ha_ws_layout lay;
  fill_layout(g, &lay);
  if (lay.total_bytes > kStaticScratchBytes) return HA_ERR_STATIC_LIMIT;
  if (g.BH == 0 || g.n == 0) return HA_OK;
  void* ws = nullptr;
  const int rs = static_scratch(&ws);
  if (rs != HA_OK) return rs;
  // every region the kernels read is written earlier in the same call, so
  // nothing left over from the previous call has to be cleared
  return forward_impl(Q, K, V, out, lse, shape, params, nullptr, nullptr, ws, kStaticScratchBytes, stream);
}

int hyperattn_forward_ex(const void* Q, const void* K, const void* V, void* out, float* lse,
                         const ha_shape* shape, const ha_params* params, const float* R_dev,
                         const int32_t* samples_dev, void* workspace, size_t workspace_bytes, void* stream) {
  return forward_impl(Q, K, V, out, lse, shape, params, R_dev, samples_dev, workspace, workspace_bytes, stream);
}

int hyperattn_forward_timed(const void* Q, const void* K, const void* V, void* out, float* lse,
                            const ha_shape* shape, const ha_params* params, void* workspace,
                            size_t workspace_bytes, void* stream, float* stage_ms_host) {
  if (!stage_ms_host) return HA_ERR_NULL;
  hipEvent_t ev[6];
  for (int i = 0; i < 6; ++i)
    if (hipEventCreate(&ev[i]) != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(ev[j]);
      return HA_ERR_LAUNCH;
    }
  int rc = forward_impl(Q, K, V, out, lse, shape, params, nullptr, nullptr, workspace, workspace_bytes, stream, ev);
  for (int i = 0; i < 6; ++i) stage_ms_host[i] = 0.f;
  Geometry g;
  const bool ran = rc == HA_OK && make_geometry(shape, params, &g) == HA_OK && g.BH > 0 && g.n > 0;
  if (ran) {
    if (hipEventSynchronize(ev[5]) != hipSuccess) rc = HA_ERR_LAUNCH;
    for (int i = 0; i < 5 && rc == HA_OK; ++i)
      if (hipEventElapsedTime(&stage_ms_host[i], ev[i], ev[i + 1]) != hipSuccess) rc = HA_ERR_LAUNCH;
    if (rc == HA_OK && hipEventElapsedTime(&stage_ms_host[5], ev[0], ev[5]) != hipSuccess) rc = HA_ERR_LAUNCH;
  }
  for (int i = 0; i < 6; ++i) (void)hipEventDestroy(ev[i]);
  return rc;
}

int ha_forward_workgroups(const ha_shape* shape, const ha_params* params, int64_t* node_wgs, int64_t* base_wgs) {
  if (!node_wgs || !base_wgs) return HA_ERR_NULL;
  Geometry g;
  const int rc = make_geometry(shape, params, &g);
  if (rc != HA_OK) return rc;
  *node_wgs = *base_wgs = 0;
  if (g.BH == 0 || g.n == 0 || !use_mfma(g)) return HA_OK;
  AttnArgs a{};
  a.g = g;
  if (g.levels > 0) *node_wgs = attn_mfma_grid(a, kModeNode);
  if (g.causal) {
    const AttnArgs e = base_case_args(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, g, nullptr, nullptr);
    *base_wgs = attn_mfma_grid(e, kModeExact);
  }
  return HA_OK;
}

int hyperattn_forward_stamped(const void* Q, const void* K, const void* V, void* out, float* lse,
                              const ha_shape* shape, const ha_params* params, void* workspace,
                              size_t workspace_bytes, void* stream, int64_t* node_stamps_dev,
                              size_t node_stamps_bytes, int64_t* base_stamps_dev, size_t base_stamps_bytes) {
  if (!shape) return HA_ERR_NULL;
  if (shape->dtype != HA_BF16) return HA_ERR_DTYPE;  // the instrumented kernel is the MFMA kernel
  int64_t node_wgs = 0, base_wgs = 0;
  const int rc = ha_forward_workgroups(shape, params, &node_wgs, &base_wgs);
  if (rc != HA_OK) return rc;
  const size_t rec = (size_t)kStampWords * sizeof(int64_t);
  if ((node_wgs > 0 && !node_stamps_dev) || (base_wgs > 0 && !base_stamps_dev)) return HA_ERR_NULL;
  if (node_stamps_bytes < (size_t)node_wgs * rec || base_stamps_bytes < (size_t)base_wgs * rec) return HA_ERR_WORKSPACE;
  if ((((uintptr_t)node_stamps_dev) | ((uintptr_t)base_stamps_dev)) & 7) return HA_ERR_ALIGN;
  static_assert(sizeof(long long) == sizeof(int64_t), "stamp words are 64-bit");
  return forward_impl(Q, K, V, out, lse, shape, params, nullptr, nullptr, workspace, workspace_bytes, stream, nullptr,
                      nullptr, node_wgs > 0 ? reinterpret_cast<long long*>(node_stamps_dev) : nullptr,
                      base_wgs > 0 ? reinterpret_cast<long long*>(base_stamps_dev) : nullptr);
}

static int exact_forward_impl(const void* Q, const void* K, const void* V, void* out, float* lse, float* out_f32,
                              const ha_shape* sh, int causal, void* stream) {
  if (!sh) return HA_ERR_NULL;
  if (sh->dtype != HA_BF16 && sh->dtype != HA_FP32) return HA_ERR_DTYPE;
  if (sh->B < 0 || sh->H < 0 || sh->n < 0 || (sh->d != 64 && sh->d != 128)) return HA_ERR_SHAPE;
  if ((int64_t)sh->B * sh->H > (1 << 20) || sh->n > (1 << 22)) return HA_ERR_SHAPE;
  if ((int64_t)sh->B * sh->H * sh->n > (1ll << 30)) return HA_ERR_SHAPE;
  if (sh->B == 0 || sh->H == 0 || sh->n == 0) return HA_OK;
  if (!Q || !K || !V || !out || !lse) return HA_ERR_NULL;
  if (out_f32 && sh->dtype != HA_BF16) return HA_ERR_DTYPE;
  if (any_misaligned16(Q, K, V, out, out_f32) || any_misaligned4(lse)) return HA_ERR_ALIGN;
  AttnArgs a{};
  a.Q = Q;
  a.K = K;
  a.V = V;
  a.q_bh_stride = a.k_bh_stride = a.out_bh_stride = (int64_t)sh->n * sh->d;
  a.out = out;
  a.lse = lse;
  a.out_f32 = out_f32;
  a.g.BH = sh->B * sh->H;
  a.g.n = sh->n;
  a.g.d = sh->d;
  a.g.dtype = sh->dtype;
  a.g.b = 1;
  a.exact_rows_q = a.exact_rows_k = sh->n;
  a.exact_block = sh->n;
  a.exact_causal = causal ? 1 : 0;
  a.merge_levels = 0;
  return run_attention(a, kModeExact, (hipStream_t)stream);
}

int exact_attn_forward(const void* Q, const void* K, const void* V, void* out, float* lse, const ha_shape* sh,
                       int causal, void* stream) {
  return exact_forward_impl(Q, K, V, out, lse, nullptr, sh, causal, stream);
}

int exact_attn_forward_train(const void* Q, const void* K, const void* V, void* out, float* lse, float* out_f32,
                             const ha_shape* sh, int causal, void* stream) {
  return exact_forward_impl(Q, K, V, out, lse, out_f32, sh, causal, stream);
}

int ha_make_projection(uint64_t seed, int32_t d, int32_t r, float* R_host) {
  if (!R_host) return HA_ERR_NULL;
  if (d < 1 || d > 128 || r < 1 || r > 8) return HA_ERR_SHAPE;
  for (int c = 0; c < d; ++c)
    for (int k = 0; k < r; ++k) {
      const uint32_t bits = (uint32_t)projection_bits(seed, c, k) << 16;
      std::memcpy(&R_host[c * r + k], &bits, 4);
    }
  return HA_OK;
}

int ha_make_samples(uint64_t seed, int32_t level, int32_t node, int32_t n_keys, int32_t m, int32_t* idx_host) {
  if (m > 0 && !idx_host) return HA_ERR_NULL;
  if (level < 0 || level > 30 || node < 0 || node >= (1 << level) || n_keys < 1 || m < 0) return HA_ERR_SHAPE;
  for (int j = 0; j < m; ++j) idx_host[j] = sample_index(seed, level, node, n_keys, j);
  return HA_OK;
}

int ha_lsh_hash(const void* X, uint8_t* codes, int64_t rows, int32_t d, int32_t dtype, const float* R_dev,
                int32_t r, void* stream) {
  if (dtype != HA_BF16 && dtype != HA_FP32) return HA_ERR_DTYPE;
  if (rows < 0 || (d != 64 && d != 128) || r < 1 || r > 8) return HA_ERR_SHAPE;
  if (rows == 0) return HA_OK;
  if (!X || !codes || !R_dev) return HA_ERR_NULL;
  if (any_misaligned16(X) || any_misaligned4(R_dev)) return HA_ERR_ALIGN;
  return launch_lsh_hash(X, codes, rows, d, dtype, R_dev, r, (hipStream_t)stream);
}

int ha_seg_sort(const uint8_t* codes, int32_t* perm, int32_t* pos, int32_t n_seg, int32_t seg_len,
                void* stream) {
  if (n_seg < 0 || seg_len < 0 || seg_len > (1 << 24)) return HA_ERR_SHAPE;
  if (n_seg == 0 || seg_len == 0) return HA_OK;
  if (!codes || !perm || !pos) return HA_ERR_NULL;
  if (any_misaligned4(perm, pos)) return HA_ERR_ALIGN;
  return launch_seg_sort_flat(codes, perm, pos, n_seg, seg_len, (hipStream_t)stream);
}

int ha_gather_rows(const void* src, const int32_t* idx, void* dst, int32_t groups, int32_t n, int32_t d,
                   int32_t dtype, void* stream) {
  if (dtype != HA_BF16 && dtype != HA_FP32) return HA_ERR_DTYPE;
  if (groups < 0 || n < 0 || (d != 64 && d != 128)) return HA_ERR_SHAPE;
  if (groups == 0 || n == 0) return HA_OK;
  if (!src || !idx || !dst) return HA_ERR_NULL;
  if (any_misaligned16(src, dst) || any_misaligned4(idx)) return HA_ERR_ALIGN;
  return launch_gather_rows(src, idx, dst, groups, n, d, dtype, (hipStream_t)stream);
}

int ha_block_attn(const void* Qs, const void* Ks, const void* Vs, float* o_b, float* lse_b, int32_t groups,
                  int32_t n, int32_t d, int32_t dtype, int32_t b, void* stream) {
  Geometry g;
  const int rc = stage_geometry(&g, groups, n, d, dtype, b, 0);
  if (rc != HA_OK) return rc;
  if (groups == 0 || n == 0) return HA_OK;
  if (!Qs || !Ks || !Vs || !o_b || !lse_b) return HA_ERR_NULL;
  if (any_misaligned16(Qs, Ks, Vs, o_b) || any_misaligned4(lse_b)) return HA_ERR_ALIGN;
  AttnArgs a{};
  a.Q = Qs;
  a.K = Ks;
  a.V = Vs;
  a.q_bh_stride = a.k_bh_stride = a.out_bh_stride = (int64_t)n * d;
  a.use_block = 1;
  a.part_o = o_b;
  a.part_l = lse_b;
  a.g = g;
  return run_attention(a, kModeNode, (hipStream_t)stream);
}

int ha_sampled_attn(const void* Qs, const void* K, const void* V, const int32_t* samples, const int32_t* pos_k,
                    float* o_r, float* lse_r, int32_t groups, int32_t n, int32_t d, int32_t dtype, int32_t b,
                    int32_t m, void* stream) {
  Geometry g;
  const int rc = stage_geometry(&g, groups, n, d, dtype, b, m);
  if (rc != HA_OK) return rc;
  if (groups == 0 || n == 0) return HA_OK;
  if (!Qs || !K || !V || !o_r || !lse_r || !pos_k || (m > 0 && !samples)) return HA_ERR_NULL;
  if (any_misaligned16(Qs, K, V, o_r) || any_misaligned4(lse_r, pos_k, samples)) return HA_ERR_ALIGN;
  AttnArgs a{};
  a.Q = Qs;
  a.K = K;
  a.V = V;
  a.q_bh_stride = a.k_bh_stride = a.out_bh_stride = (int64_t)n * d;
  a.pos_k = pos_k;
  a.samples = m > 0 ? samples : nullptr;
  a.use_block = 0;
  a.part_o = o_r;
  a.part_l = lse_r;
  a.g = g;
  return run_attention(a, kModeNode, (hipStream_t)stream);
}

int ha_merge_unpermute(const float* o_b, const float* lse_b, const float* o_r, const float* lse_r,
                       const int32_t* perm_q, void* out, float* lse, int32_t groups, int32_t n, int32_t d,
                       int32_t dtype, void* stream) {
  if (dtype != HA_BF16 && dtype != HA_FP32) return HA_ERR_DTYPE;
  if (groups < 0 || n < 0 || (d != 64 && d != 128)) return HA_ERR_SHAPE;
  if (groups == 0 || n == 0) return HA_OK;
  if (!o_b || !lse_b || !o_r || !lse_r || !perm_q || !out || !lse) return HA_ERR_NULL;
  if (any_misaligned16(o_b, o_r, out) || any_misaligned4(lse_b, lse_r, perm_q, lse)) return HA_ERR_ALIGN;
  return launch_merge_unpermute(o_b, lse_b, o_r, lse_r, perm_q, out, lse, groups, n, d, dtype,
                                (hipStream_t)stream);
}

int ha_backward_workspace_layout(const ha_shape* shape, const ha_params* params, ha_bwd_ws_layout* layout) {
  if (!layout) return HA_ERR_NULL;
  Geometry g;
  const int rc = make_geometry(shape, params, &g);
  if (rc != HA_OK) return rc;
  fill_bwd_layout(g, layout);
  return HA_OK;
}

size_t ha_backward_workspace_bytes(const ha_shape* shape, const ha_params* params) {
  ha_bwd_ws_layout l;
  return ha_backward_workspace_layout(shape, params, &l) == HA_OK ? l.total_bytes : 0;
}

int hyperattn_forward_train(const void* Q, const void* K, const void* V, void* out, float* lse, float* out_f32,
                            const ha_shape* shape, const ha_params* params, void* workspace,
                            size_t workspace_bytes, void* stream) {
  return forward_impl(Q, K, V, out, lse, shape, params, nullptr, nullptr, workspace, workspace_bytes, stream, nullptr,
                      out_f32);
}

int hyperattn_backward(const void* Q, const void* K, const void* V, const void* out, const float* out_f32,
                       const float* lse, const void* d_out, void* dQ, void* dK, void* dV, const ha_shape* shape,
                       const ha_params* params, const void* fwd_workspace, size_t fwd_workspace_bytes,
                       void* bwd_workspace, size_t bwd_workspace_bytes, void* stream) {
  return backward_impl(Q, K, V, out, out_f32, lse, d_out, dQ, dK, dV, shape, params, fwd_workspace,
                       fwd_workspace_bytes, bwd_workspace, bwd_workspace_bytes, stream);
}

int hyperattn_backward_timed(const void* Q, const void* K, const void* V, const void* out, const float* out_f32,
                             const float* lse, const void* d_out, void* dQ, void* dK, void* dV, const ha_shape* shape,
                             const ha_params* params, const void* fwd_workspace, size_t fwd_workspace_bytes,
                             void* bwd_workspace, size_t bwd_workspace_bytes, void* stream, float* stage_ms_host) {
  if (!stage_ms_host) return HA_ERR_NULL;
  constexpr int NE = 8;
  hipEvent_t ev[NE];
  for (int i = 0; i < NE; ++i)
    if (hipEventCreate(&ev[i]) != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(ev[j]);
      return HA_ERR_LAUNCH;
    }
  int rc = backward_impl(Q, K, V, out, out_f32, lse, d_out, dQ, dK, dV, shape, params, fwd_workspace,
                         fwd_workspace_bytes, bwd_workspace, bwd_workspace_bytes, stream, ev);
  for (int i = 0; i < NE; ++i) stage_ms_host[i] = 0.f;
  Geometry g;
  const bool ran = rc == HA_OK && make_geometry(shape, params, &g) == HA_OK && g.BH > 0 && g.n > 0;
  if (ran) {
    if (hipEventSynchronize(ev[NE - 1]) != hipSuccess) rc = HA_ERR_LAUNCH;
    for (int i = 0; i < NE - 1 && rc == HA_OK; ++i)
      if (hipEventElapsedTime(&stage_ms_host[i], ev[i], ev[i + 1]) != hipSuccess) rc = HA_ERR_LAUNCH;
    if (rc == HA_OK && hipEventElapsedTime(&stage_ms_host[NE - 1], ev[0], ev[NE - 1]) != hipSuccess) rc = HA_ERR_LAUNCH;
  }
  for (int i = 0; i < NE; ++i) (void)hipEventDestroy(ev[i]);
  return rc;
}

int exact_attn_backward(const void* Q, const void* K, const void* V, const void* out, const float* out_f32,
                        const float* lse, const void* d_out, void* dQ, void* dK, void* dV, const ha_shape* sh, int causal,
                        void* workspace, size_t workspace_bytes, void* stream) {
  if (!sh) return HA_ERR_NULL;
  // exact attention is the causal recursion that never splits (n_min = n), or its unmasked twin
  ha_params p;
  std::memset(&p, 0, sizeof(p));
  p.b = 1;
  p.m = 0;
  p.r = 1;
  p.causal = 1;
  p.n_min = sh->n > 0 ? sh->n : 1;
  Geometry g;
  int rc = make_geometry(sh, &p, &g);
  if (rc != HA_OK) return rc;
  if (out_f32 && g.dtype != HA_BF16) return HA_ERR_DTYPE;
  if (g.BH == 0 || g.n == 0) return HA_OK;
  if (!Q || !K || !V || !out || !lse || !d_out || !dQ || !dK || !dV || !workspace) return HA_ERR_NULL;
  if (any_misaligned16(Q, K, V, out, out_f32, d_out, dQ, dK, dV) || any_misaligned4(lse)) return HA_ERR_ALIGN;
  ha_bwd_ws_layout bl;
  fill_bwd_layout(g, &bl);
  if (workspace_bytes < bl.total_bytes || ((uintptr_t)workspace & 255) != 0) return HA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  unsigned char* bb = (unsigned char*)workspace;
  BwdArgs a{};
  a.f.Q = Q;
  a.f.K = K;
  a.f.V = V;
  a.f.q_bh_stride = a.f.k_bh_stride = a.f.out_bh_stride = (int64_t)g.n * g.d;
  a.f.g = g;
  a.f.exact_rows_q = a.f.exact_rows_k = g.n;
  a.f.exact_block = g.n;
  a.f.exact_causal = causal ? 1 : 0;
  a.dO = d_out;
  a.lse = lse;
  a.delta = (float*)(bb + bl.delta);
  rc = launch_bwd_delta(out, out_f32, d_out, (float*)(bb + bl.delta), (int64_t)g.BH * g.n, g.d, g.dtype, st);
  if (rc != HA_OK) return rc;
  a.fin1 = dQ;
  rc = launch_attn_bwd(a, kBwdDqExact, st);
  if (rc != HA_OK) return rc;
  a.fin1 = dK;
  a.fin2 = dV;
  return launch_attn_bwd(a, kBwdDkvExact, st);
}

size_t exact_attn_backward_workspace_bytes(const ha_shape* sh) {
  if (!sh) return 0;
  ha_params p;
  std::memset(&p, 0, sizeof(p));
  p.b = 1;
  p.r = 1;
  p.causal = 1;
  p.n_min = sh->n > 0 ? sh->n : 1;
  return ha_backward_workspace_bytes(sh, &p);
}

int ha_alg2_workspace_layout(const ha_shape* shape, const ha_params* params, ha_alg2_ws_layout* layout) {
  if (!layout) return HA_ERR_NULL;
  Geometry g;
  const int rc = make_geometry(shape, params, &g);
  if (rc != HA_OK) return rc;
  ha_ws_layout fwd;
  fill_layout(g, &fwd);
  fill_alg2_layout(g, fwd, layout);
  return HA_OK;
}

size_t ha_alg2_workspace_bytes(const ha_shape* shape, const ha_params* params) {
  ha_alg2_ws_layout l;
  return ha_alg2_workspace_layout(shape, params, &l) == HA_OK ? l.total_bytes : 0;
}

int hyperattn_forward_alg2(const void* Q, const void* K, const void* V, void* out, float* lse, const ha_shape* shape,
                           const ha_params* params, const ha_alg2_options* opt, void* workspace,
                           size_t workspace_bytes, void* stream) {
  if (!opt) return HA_ERR_NULL;
  Geometry g;
  int rc = make_geometry(shape, params, &g);
  if (rc != HA_OK) return rc;
  if (g.BH == 0 || g.n == 0) return HA_OK;
  if (!Q || !K || !V || !out || !lse || !workspace) return HA_ERR_NULL;
  if (any_misaligned16(Q, K, V, out) || any_misaligned4(lse)) return HA_ERR_ALIGN;
  ha_ws_layout lay;
  fill_layout(g, &lay);
  ha_alg2_ws_layout al;
  fill_alg2_layout(g, lay, &al);
  if (workspace_bytes < al.total_bytes || ((uintptr_t)workspace & 255) != 0) return HA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  unsigned char* base = (unsigned char*)workspace;
  void* part_o = (void*)(base + lay.part_o);
  float* part_l = (float*)(base + lay.part_l);
  if (g.levels > 0) {
    // hash, sort and draws exactly as the forward does them
    uint16_t Rb[1024];
    for (int c = 0; c < g.d; ++c)
      for (int k = 0; k < g.r; ++k) Rb[c * g.r + k] = projection_bits(params->seed, c, k);
    float* proj = (float*)(base + lay.proj);
    int32_t* samples = (int32_t*)(base + lay.samples);
    rc = launch_prep(proj, nullptr, Rb, samples, nullptr, g, params->seed, st);
    if (rc != HA_OK) return rc;
    uint8_t* codes_q = base + lay.codes_q;
    uint8_t* codes_k = base + lay.codes_k;
    rc = launch_lsh_hash(Q, codes_q, (int64_t)g.BH * g.n, g.d, g.dtype, proj, g.r, st);
    if (rc != HA_OK) return rc;
    rc = launch_lsh_hash(K, codes_k, (int64_t)g.BH * g.n, g.d, g.dtype, proj, g.r, st);
    if (rc != HA_OK) return rc;
    rc = launch_seg_sort_nodes(codes_q, codes_k, (int32_t*)(base + lay.perm_q), (int32_t*)(base + lay.perm_k),
                               (int32_t*)(base + lay.pos_k), g.m > 0 ? samples : nullptr,
                               (int32_t*)(base + lay.samp_blk), (uint32_t*)(base + lay.sort_hist), g, st);
    if (rc != HA_OK) return rc;
    // Algorithm 2 on every node, one level at a time: the unmasked problem is its own single node;
    // a causal problem's level l holds 2^l off-diagonal nodes per head (Algorithm 4), whose results
    // go to the per-level partial outputs that the base case adds up below
    const size_t esz = g.dtype == HA_BF16 ? 2 : 4;
    for (int level = 0; level < g.levels; ++level) {
      const int nodes = g.causal ? (1 << level) : 1;
      const int s_rows = g.causal ? (g.n >> (level + 1)) : g.n;
      const size_t lvl = (size_t)level * g.BH * g.n_cov;   // first entry of the level in the per-level arrays
      Alg2Args a{};
      a.Q = Q;
      a.K = K;
      a.V = V;
      a.out = g.causal ? (void*)((unsigned char*)part_o + lvl * g.d * esz) : out;
      a.lse = g.causal ? part_l + lvl : lse;
      a.g = g;
      a.g.BH = g.BH * nodes;
      a.g.n = s_rows;
      a.n_full = g.n;
      a.nodes = nodes;
      a.level = level;
      a.causal = g.causal;
      a.heads = g.BH;
      a.total_nodes = g.total_nodes;
      a.perm_q = (const int32_t*)(base + lay.perm_q) + lvl;
      a.perm_k = (const int32_t*)(base + lay.perm_k) + lvl;
      a.pos_k = (const int32_t*)(base + lay.pos_k) + lvl;
      a.samples = samples;
      a.samp_blk = (const int32_t*)(base + lay.samp_blk);
      a.pos_q = (int32_t*)(base + al.pos_q);
      a.tau_rows = (int32_t*)(base + al.tau_rows);
      a.log_unm_t = (float*)(base + al.log_unmasked_t);
      a.log_tau = (float*)(base + al.log_tau);
      a.vw = (double*)(base + al.vnorm_w);
      a.vprefix = (double*)(base + al.vnorm_prefix);
      a.vsamp = (int32_t*)(base + al.vnorm_samples);
      a.vlogw = (float*)(base + al.vnorm_logw);
      a.log_unm_parts = (float*)(base + al.log_unmasked_parts);
      a.seed = params->seed;
      a.cap_scale = opt->cap_scale;
      a.kappa = opt->kappa;
      a.vnorm = opt->vnorm_sampling ? 1 : 0;
      rc = launch_alg2(a, st);
      if (rc != HA_OK) return rc;
    }
  }
  if (g.causal) return run_base_case(Q, K, V, out, lse, nullptr, g, part_o, part_l, st);
  return HA_OK;
}

const char* ha_strerror(int status) {
  switch (status) {
    case HA_OK: return "ok";
    case HA_ERR_NULL: return "a required pointer is NULL";
    case HA_ERR_DTYPE: return "unsupported dtype";
    case HA_ERR_SHAPE: return "unsupported shape or parameters";
    case HA_ERR_WORKSPACE: return "workspace too small or misaligned";
    case HA_ERR_LAUNCH: return "HIP launch failed";
    case HA_ERR_STATIC_LIMIT:
      return "the problem needs more scratch than the built-in array holds (ha_static_scratch_bytes): call "
             "hyperattn_forward with a workspace";
    case HA_ERR_ALIGN: return "a tensor is not 16-byte aligned (or an index / float array not 4-byte aligned)";
    default: return "unknown status";
  }
}

}  // extern "C"
