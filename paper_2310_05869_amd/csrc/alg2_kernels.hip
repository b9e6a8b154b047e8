// The estimator of Algorithm 2 as printed, and Lemma 2 / Algorithm 3's value
// product, as options beside the Section 4 form the main path implements:
//   tau      = max over a random row subset T of the unmasked row sum <1 - M^H_j, A_j>
//   C_i      = cap_scale * m / (n ln n) * (masked row sum_i + tau / kappa)
//   d_i      = (n/m) sum_j (1 - M_{i,l_j}) min(exp<q_i,k_{l_j}>, C_i)
//   d~_i     = masked row sum_i + max(d_i, tau / kappa)
//   out_i    = (1 / d~_i) sum_r exp<q_i,k_{l'_r}> v_{l'_r} / (m p_{l'_r}),  l'_r ~ p_l ~ |V_l|^2   (Lemma 2)
//         or = (1 / d~_i) (masked part + (n/m) sum_j (1 - M) exp<q_i,k_{l_j}> v_{l_j})                (Section 4)
// The constants the paper leaves open (the Theta in C_i, kappa) are the caller's.
// A launch sequence handles one level of nodes (alg2_common.h): the unmasked problem, or one
// level of Algorithm 4's off-diagonal nodes, every node with its own draws.  The kernels here are plain fp32 FMA code (one thread per query row,
// K / V rows staged through LDS): they serve fp32 tensors and whatever the bf16 matrix-core
// forms of the two heavy steps (alg2_mfma.hip) do not take; the draws, weights and prefix
// sums are computed here for both.
//
// Lemma 2's rows are drawn with p_l = |V_l|^2 / |V|_F^2 (V the node's value rows) by inverting
// the cumulative distribution in fp64: draw r of head bh at the node with heap index h takes the
// uniform u in (0, 1) formed by the top 53 bits of counter (h * heads + bh) * m + r of stream 2
// and is the first l whose inclusive prefix sum of squared norms exceeds u |V|_F^2.
#include "attn_common.h"
#include "alg2_common.h"

namespace ha {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint64_t kStreamTauRows = 0;
constexpr uint64_t kStreamVnorm = 2;

template <typename T>
__device__ inline float elem(const T* p);
template <>
__device__ inline float elem<float>(const float* p) { return *p; }
template <>
__device__ inline float elem<uint16_t>(const uint16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }

__global__ void alg2_prep_kernel(Alg2Args a) {
  const Geometry& g = a.g;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  // rows of T of every node of this level: counter heap * m + j of the stream
  if (t < (int64_t)a.nodes * g.m) {
    const int node = (int)(t / g.m), j = (int)(t % g.m);
    const int heap = (1 << a.level) - 1 + node;
    const uint64_t hi = rand_u64(a.seed, kStreamTauRows, (uint64_t)heap * g.m + j) >> 32;
    a.tau_rows[(int64_t)heap * g.m + j] = (int32_t)((hi * (uint64_t)g.n) >> 32);
  }
  // pos_q = P_Q^-1, node-local
  if (t < (int64_t)g.BH * g.n) {
    const int vh = (int)(t / g.n);
    const Alg2Node nd = alg2_node(a, vh);
    a.pos_q[(int64_t)vh * g.n + (a.perm_q[t] - nd.q_start)] = (int32_t)(t % g.n);
  }
}

// Squared row norms of V in fp64 (one thread per row); 64 rows per workgroup come in through LDS
// so that the global loads are coalesced.
constexpr int kVwRows = 64;

template <typename T, int D>
__global__ __launch_bounds__(256) void vnorm_weight_kernel(Alg2Args a) {
  constexpr int kRowBytes = D * (int)sizeof(T);
  constexpr int kStride = kRowBytes + 4;  // odd number of words: the 64 row readers hit 64 banks
  __shared__ __attribute__((aligned(16))) unsigned char tile[kVwRows * kStride];
  const Geometry& g = a.g;
  // one workgroup per 64 consecutive keys of one node (g.n need not be a multiple of 64)
  const int per_node = (g.n + kVwRows - 1) / kVwRows;
  const int vh = blockIdx.x / per_node;
  const int l0 = (blockIdx.x % per_node) * kVwRows;
  const Alg2Node nd = alg2_node(a, vh);
  const int nrows = min(kVwRows, g.n - l0);
  const int64_t row0 = (int64_t)vh * g.n + l0;   // in the view
  const unsigned char* src = reinterpret_cast<const unsigned char*>(a.V) +
                             ((int64_t)nd.head * a.n_full + nd.k_start + l0) * kRowBytes;
  for (int e = threadIdx.x; e < nrows * (kRowBytes / 4); e += 256) {
    const int r = e / (kRowBytes / 4), w = e % (kRowBytes / 4);
    *reinterpret_cast<uint32_t*>(tile + r * kStride + 4 * w) = *reinterpret_cast<const uint32_t*>(src + (int64_t)e * 4);
  }
  __syncthreads();
  if (threadIdx.x >= 64) return;  // the first wave sums the rows (whole waves leave; no partial wave)
  const bool active = (int)threadIdx.x < nrows;
  const T* v = reinterpret_cast<const T*>(tile + (active ? threadIdx.x : 0) * kStride);
  double w = 0.0;
  for (int c = 0; c < D; ++c) {
    const double x = (double)elem<T>(v + c);
    w = w + x * x;  // the product of two fp32-representable values is exact in fp64
  }
  const int64_t row = row0 + (active ? threadIdx.x : 0);
  if (active) a.vw[row] = w;
}

constexpr int kScanThreads = 1024;

// Inclusive prefix sums of the squared norms of one head, in fp64 and in a fixed order (a thread
// sums its run of rows, the threads' sums are scanned, every thread then walks its run again).
__global__ __launch_bounds__(kScanThreads) void vnorm_scan_kernel(Alg2Args a) {
  __shared__ double part[kScanThreads];
  const Geometry& g = a.g;
  const int bh = blockIdx.x;
  const int tid = threadIdx.x;
  const int per = (g.n + kScanThreads - 1) / kScanThreads;
  const int lo = min(g.n, tid * per), hi = min(g.n, lo + per);
  const double* w = a.vw + (int64_t)bh * g.n;
  double sum = 0.0;
  for (int l = lo; l < hi; ++l) sum += w[l];
  part[tid] = sum;
  __syncthreads();
  for (int off = 1; off < kScanThreads; off <<= 1) {
    double v = 0.0;
    if (tid >= off) v = part[tid - off];
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  double run = tid > 0 ? part[tid - 1] : 0.0;
  for (int l = lo; l < hi; ++l) {
    run += w[l];
    a.vprefix[(int64_t)bh * g.n + l] = run;
  }
}

__global__ void vnorm_sample_kernel(Alg2Args a) {
  const Geometry& g = a.g;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (int64_t)g.BH * g.m) return;
  const int vh = (int)(t / g.m), r = (int)(t % g.m);
  const Alg2Node nd = alg2_node(a, vh);
  const double* prefix = a.vprefix + (int64_t)vh * g.n;
  const double total = prefix[g.n - 1];
  const uint64_t ctr = ((uint64_t)nd.heap * a.heads + nd.head) * g.m + r;
  const double u = ((double)(rand_u64(a.seed, kStreamVnorm, ctr) >> 11) + 0.5) * 0x1.0p-53;
  int lo;
  double p;
  if (total > 0.0) {
    const double target = u * total;
    int hi = g.n - 1;  // first l with prefix[l] > target
    lo = 0;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (prefix[mid] > target) hi = mid;
      else lo = mid + 1;
    }
    p = a.vw[(int64_t)vh * g.n + lo] / total;
  } else {  // V = 0: every choice gives the same (zero) product; uniform
    lo = min(g.n - 1, (int)(u * (double)g.n));
    p = 1.0 / (double)g.n;
  }
  const int64_t at = ((int64_t)nd.head * a.total_nodes + nd.heap) * g.m + r;
  a.vsamp[at] = lo;
  a.vlogw[at] = (float)(-log((double)g.m * p));
}

// log of the unmasked row sum of the rows T_j: one workgroup per head and kTauRows of them.
// Key rows pass through LDS in tiles (coalesced loads, every key element serves several rows);
// a thread owns one key of the tile for some of the rows and keeps their running log sums.
constexpr int kTauRows = 8;

template <typename T, int D>
__global__ __launch_bounds__(256) void alg2_tau_kernel(Alg2Args a) {
  constexpr int kKeys = sizeof(T) == 2 ? 128 : 64;   // keys per tile
  constexpr int kGroups = 256 / kKeys;               // thread groups, each with its own rows
  constexpr int kRpt = kTauRows / kGroups;           // rows per thread
  constexpr int kRowBytes = D * (int)sizeof(T);
  constexpr int kStride = kRowBytes + 4;             // odd number of words: no bank conflicts between the keys
  __shared__ __attribute__((aligned(16))) unsigned char tile[kKeys * kStride];
  __shared__ __attribute__((aligned(16))) float qs[kTauRows][D];
  __shared__ float red_m[kTauRows][kKeys], red_s[kTauRows][kKeys];
  __shared__ int blk_of[kTauRows];
  const Geometry& g = a.g;
  const int groups_per_head = (g.m + kTauRows - 1) / kTauRows;
  const int bh = blockIdx.x / groups_per_head, j0 = (blockIdx.x % groups_per_head) * kTauRows;
  const int nr = min(kTauRows, g.m - j0);
  const int64_t hb = (int64_t)bh * g.n;   // bh: view head (one node)
  const Alg2Node nd = alg2_node(a, bh);
  const int32_t* trows = a.tau_rows + (int64_t)nd.heap * g.m;
  const T* Qh = reinterpret_cast<const T*>(a.Q) + ((int64_t)nd.head * a.n_full + nd.q_start) * D;
  const unsigned char* Kh = reinterpret_cast<const unsigned char*>(a.K) + ((int64_t)nd.head * a.n_full + nd.k_start) * kRowBytes;
  const int tid = threadIdx.x;
  for (int e = tid; e < kTauRows * D; e += 256) {
    const int r = e / D, c = e % D;
    qs[r][c] = r < nr ? elem<T>(Qh + (int64_t)trows[j0 + r] * D + c) : 0.f;
  }
  if (tid < kTauRows) blk_of[tid] = tid < nr ? a.pos_q[hb + trows[j0 + tid]] / g.b : -1;
  const int k = tid % kKeys, grp = tid / kKeys;
  float mx[kRpt], sum[kRpt];
#pragma unroll
  for (int r = 0; r < kRpt; ++r) {
    mx[r] = -INFINITY;
    sum[r] = 0.f;
  }
  for (int l0 = 0; l0 < g.n; l0 += kKeys) {
    const int cnt = min(kKeys, g.n - l0);
    __syncthreads();
    for (int e = tid; e < cnt * (kRowBytes / 4); e += 256) {
      const int r = e / (kRowBytes / 4), w = e % (kRowBytes / 4);
      *reinterpret_cast<uint32_t*>(tile + r * kStride + 4 * w) =
          *reinterpret_cast<const uint32_t*>(Kh + (int64_t)l0 * kRowBytes + (int64_t)e * 4);
    }
    __syncthreads();
    if (k >= cnt) continue;
    const int kblk = a.pos_k[hb + l0 + k] / g.b;
    const T* kr = reinterpret_cast<const T*>(tile + k * kStride);
    float s[kRpt];
#pragma unroll
    for (int r = 0; r < kRpt; ++r) s[r] = 0.f;
    // ascending columns, one fused multiply-add each (the scores of an fp32 dot product); four columns
    // per step so that a row of q is read 16 bytes at a time
#pragma unroll 4
    for (int c = 0; c < D; c += 4) {
      float x[4];
      if (sizeof(T) == 2) {
        const uint32_t lo = *reinterpret_cast<const uint32_t*>(kr + c), hi = *reinterpret_cast<const uint32_t*>(kr + c + 2);
        x[0] = __uint_as_float(lo << 16);
        x[1] = __uint_as_float(lo & 0xFFFF0000u);
        x[2] = __uint_as_float(hi << 16);
        x[3] = __uint_as_float(hi & 0xFFFF0000u);
      } else {
#pragma unroll
        for (int z = 0; z < 4; ++z) x[z] = elem<T>(kr + c + z);
      }
#pragma unroll
      for (int r = 0; r < kRpt; ++r) {
        const float4 qv = *reinterpret_cast<const float4*>(&qs[grp * kRpt + r][c]);
        s[r] = __builtin_fmaf(qv.x, x[0], s[r]);
        s[r] = __builtin_fmaf(qv.y, x[1], s[r]);
        s[r] = __builtin_fmaf(qv.z, x[2], s[r]);
        s[r] = __builtin_fmaf(qv.w, x[3], s[r]);
      }
    }
#pragma unroll
    for (int r = 0; r < kRpt; ++r) {
      if (kblk == blk_of[grp * kRpt + r]) continue;  // 1 - M (rows beyond nr have block -1 and are dropped below)
      if (s[r] > mx[r]) {
        sum[r] = sum[r] * expf(mx[r] - s[r]) + 1.f;
        mx[r] = s[r];
      } else {
        sum[r] += expf(s[r] - mx[r]);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < kRpt; ++r) {
    red_m[grp * kRpt + r][k] = mx[r];
    red_s[grp * kRpt + r][k] = sum[r];
  }
  __syncthreads();
  if (tid < nr) {
    float M = -INFINITY;
    for (int t = 0; t < kKeys; ++t) M = fmaxf(M, red_m[tid][t]);
    float S = 0.f;
    for (int t = 0; t < kKeys; ++t)
      if (red_m[tid][t] > -INFINITY) S += red_s[tid][t] * expf(red_m[tid][t] - M);
    a.log_unm_t[(int64_t)bh * g.m + j0 + tid] = (M == -INFINITY) ? -INFINITY : M + logf(S);
  }
}

__device__ inline float logaddexpf(float x, float y) {
  const float hi = fmaxf(x, y), lo = fminf(x, y);
  if (hi == -INFINITY) return -INFINITY;
  return hi + log1pf(expf(lo - hi));
}

// log tau = the largest log unmasked row sum over the rows of T, one workgroup per head; where the
// sums came in over ranges of keys they are added up first (and kept in log_unm_t).
__global__ __launch_bounds__(256) void alg2_tau_max_kernel(Alg2Args a) {
  __shared__ float red[256];
  const Geometry& g = a.g;
  const int bh = blockIdx.x;
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < g.m; j += 256) {
    float v;
    if (a.tau_splits > 0) {
      v = -INFINITY;
      for (int sp = 0; sp < a.tau_splits; ++sp) v = logaddexpf(v, a.log_unm_parts[((int64_t)sp * g.BH + bh) * g.m + j]);
      a.log_unm_t[(int64_t)bh * g.m + j] = v;
    } else {
      v = a.log_unm_t[(int64_t)bh * g.m + j];
    }
    mx = fmaxf(mx, v);
  }
  red[threadIdx.x] = mx;
  __syncthreads();
  for (int s = 128; s >= 1; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const Alg2Node nd = alg2_node(a, bh);
    a.log_tau[(int64_t)nd.head * a.total_nodes + nd.heap] = red[0];
  }
}

constexpr int kA2Rows = 64;  // query rows (threads) per workgroup
constexpr int kA2Tile = 32;  // key rows per LDS tile

// One thread per query row; 64 consecutive sorted positions of one block per workgroup.
template <typename T, int D>
__global__ __launch_bounds__(kA2Rows) void alg2_main_kernel(Alg2Args a) {
  __shared__ float Ks[kA2Tile * D];
  __shared__ float Vs[kA2Tile * D];
  __shared__ int32_t rows[kA2Tile];
  __shared__ float bias[kA2Tile];
  const Geometry& g = a.g;
  const int tid = threadIdx.x;
  const int tpb = (g.b + kA2Rows - 1) / kA2Rows;
  const int tile = blockIdx.x % ((g.n / g.b) * tpb);
  const int bh = blockIdx.x / ((g.n / g.b) * tpb);
  const int t = tile / tpb, chunk = tile % tpb;
  const int p0 = t * g.b + chunk * kA2Rows;
  const bool valid = chunk * kA2Rows + tid < g.b;
  const int64_t hb = (int64_t)bh * g.n;   // bh: view head (one node); perm values are rows of the real head
  const Alg2Node nd = alg2_node(a, bh);
  const int qrow = a.perm_q[hb + (valid ? p0 + tid : p0)];
  const T* Qh = reinterpret_cast<const T*>(a.Q) + (int64_t)nd.head * a.n_full * D;
  const T* Kh = reinterpret_cast<const T*>(a.K) + (int64_t)nd.head * a.n_full * D;
  const T* Vh = reinterpret_cast<const T*>(a.V) + (int64_t)nd.head * a.n_full * D;
  const int64_t draws = ((int64_t)nd.head * a.total_nodes + nd.heap) * g.m;   // this node's entries of the per-node arrays

  float q[D], o[D];
#pragma unroll
  for (int c = 0; c < D; ++c) {
    q[c] = elem<T>(Qh + (int64_t)qrow * D + c);
    o[c] = 0.f;
  }
  float M = -INFINITY;      // reference of every exponential below
  float msum = 0.f;         // masked row sum / e^M
  float dsum = 0.f;         // sum of (capped) kept samples / e^M
  const float ratio = g.m > 0 ? (float)g.n / (float)g.m : 0.f;
  const float log_tau = a.log_tau[(int64_t)nd.head * a.total_nodes + nd.heap];
  const float floor_term = a.kappa > 0.f ? log_tau - logf(a.kappa) : -INFINITY;

  auto rescale_to = [&](float m_new) {
    if (m_new > M) {
      const float f = expf(M - m_new);  // M = -inf gives 0 with all sums 0
      msum *= f;
      dsum *= f;
#pragma unroll
      for (int c = 0; c < D; ++c) o[c] *= f;
      M = m_new;
    }
  };
  // stage `cnt` key rows (indices and per-row log weights already in LDS) as fp32
  auto stage = [&](int cnt, bool with_v) {
    for (int e = tid; e < cnt * D; e += kA2Rows) {
      const int j = e / D, c = e % D;
      Ks[e] = elem<T>(Kh + (int64_t)rows[j] * D + c);
      if (with_v) Vs[e] = elem<T>(Vh + (int64_t)rows[j] * D + c);
    }
  };

  // ---- pass 1: the keys of this block (mask M^H) ----
  for (int k0 = 0; k0 < g.b; k0 += kA2Tile) {
    const int cnt = min(kA2Tile, g.b - k0);
    __syncthreads();
    if (tid < cnt) rows[tid] = a.perm_k[hb + t * g.b + k0 + tid];
    __syncthreads();
    stage(cnt, !a.vnorm);
    __syncthreads();
    for (int j = 0; j < cnt; ++j) {
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) s = __builtin_fmaf(q[c], Ks[j * D + c], s);
      rescale_to(s);
      const float p = expf(s - M);
      msum += p;
      if (!a.vnorm) {
#pragma unroll
        for (int c = 0; c < D; ++c) o[c] = __builtin_fmaf(p, Vs[j * D + c], o[c]);
      }
    }
  }
  const float log_masked = (msum > 0.f) ? M + logf(msum) : -INFINITY;
  const bool capped = a.cap_scale > 0.f && g.m > 0;
  const float log_cap = capped ? logf(a.cap_scale * (float)g.m / ((float)g.n * logf((float)g.n))) + logaddexpf(log_masked, floor_term)
                               : INFINITY;

  // ---- pass 2: the uniform samples of Algorithm 2 (row-sum estimate; Section 4's numerator) ----
  for (int j0 = 0; j0 < g.m; j0 += kA2Tile) {
    const int cnt = min(kA2Tile, g.m - j0);
    __syncthreads();
    if (tid < cnt) {
      rows[tid] = nd.k_start + a.samples[(int64_t)nd.heap * g.m + j0 + tid];
      bias[tid] = (a.samp_blk[draws + j0 + tid] == t) ? -INFINITY : 0.f;  // factor 1 - M_{i,l_j}
    }
    __syncthreads();
    stage(cnt, !a.vnorm);
    __syncthreads();
    for (int j = 0; j < cnt; ++j) {
      if (bias[j] == -INFINITY) continue;
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) s = __builtin_fmaf(q[c], Ks[j * D + c], s);
      rescale_to(s);
      dsum += expf(fminf(s, log_cap) - M);
      if (!a.vnorm) {
        const float p = ratio * expf(s - M);
#pragma unroll
        for (int c = 0; c < D; ++c) o[c] = __builtin_fmaf(p, Vs[j * D + c], o[c]);
      }
    }
  }

  // ---- pass 3: the value rows drawn by squared norm (Lemma 2), each with its 1 / (m p_l) ----
  if (a.vnorm) {
    for (int j0 = 0; j0 < g.m; j0 += kA2Tile) {
      const int cnt = min(kA2Tile, g.m - j0);
      __syncthreads();
      if (tid < cnt) {
        rows[tid] = nd.k_start + a.vsamp[draws + j0 + tid];
        bias[tid] = a.vlogw[draws + j0 + tid];
      }
      __syncthreads();
      stage(cnt, true);
      __syncthreads();
      for (int j = 0; j < cnt; ++j) {
        float s = bias[j];
#pragma unroll
        for (int c = 0; c < D; ++c) s = __builtin_fmaf(q[c], Ks[j * D + c], s);
        rescale_to(s);
        const float p = expf(s - M);
#pragma unroll
        for (int c = 0; c < D; ++c) o[c] = __builtin_fmaf(p, Vs[j * D + c], o[c]);
      }
    }
  }

  const float log_d = (dsum > 0.f) ? M + logf(dsum * ratio) : -INFINITY;
  const float log_dt = logaddexpf(log_masked, fmaxf(log_d, floor_term));
  const float f = (M == -INFINITY || log_dt == -INFINITY) ? 0.f : expf(M - log_dt);
  if (!valid) return;
  const int64_t orow = hb + (qrow - nd.q_start);
  a.lse[orow] = log_dt;
  if (sizeof(T) == 4) {
    float* op = reinterpret_cast<float*>(a.out) + orow * D;
#pragma unroll
    for (int c = 0; c < D; ++c) op[c] = o[c] * f;
  } else {
    uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + orow * D;
#pragma unroll
    for (int c = 0; c < D; c += 2) *reinterpret_cast<uint32_t*>(op + c) = pack_bf16x2(o[c] * f, o[c + 1] * f);
  }
}

template <typename T>
static int launch_alg2_t(const Alg2Args& a_in, hipStream_t st) {
  const Geometry& g = a_in.g;
  Alg2Args a = a_in;
  const bool mfma = alg2_mfma_supported(a);
  a.tau_splits = mfma ? kAlg2TauSplits : 0;
  const int64_t rows = (int64_t)g.BH * g.n;
  int64_t prep = rows > (int64_t)a.nodes * g.m ? rows : (int64_t)a.nodes * g.m;
  hipLaunchKernelGGL(alg2_prep_kernel, dim3((unsigned)((prep + 255) / 256)), dim3(256), 0, st, a);
  if (a.vnorm && g.m > 0) {
    const unsigned vw_grid = (unsigned)((int64_t)g.BH * ((g.n + kVwRows - 1) / kVwRows));
    if (g.d == 128) hipLaunchKernelGGL((vnorm_weight_kernel<T, 128>), dim3(vw_grid), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((vnorm_weight_kernel<T, 64>), dim3(vw_grid), dim3(256), 0, st, a);
    hipLaunchKernelGGL(vnorm_scan_kernel, dim3((unsigned)g.BH), dim3(kScanThreads), 0, st, a);
    hipLaunchKernelGGL(vnorm_sample_kernel, dim3((unsigned)(((int64_t)g.BH * g.m + 255) / 256)), dim3(256), 0, st, a);
  }
  if (g.m > 0) {
    if (mfma) {
      const int rc = launch_alg2_tau_mfma(a, st);
      if (rc != HA_OK) return rc;
    } else {
      const unsigned tau_grid = (unsigned)((int64_t)g.BH * ((g.m + kTauRows - 1) / kTauRows));
      if (g.d == 128) hipLaunchKernelGGL((alg2_tau_kernel<T, 128>), dim3(tau_grid), dim3(256), 0, st, a);
      else hipLaunchKernelGGL((alg2_tau_kernel<T, 64>), dim3(tau_grid), dim3(256), 0, st, a);
    }
  }
  hipLaunchKernelGGL(alg2_tau_max_kernel, dim3((unsigned)g.BH), dim3(256), 0, st, a);
  if (mfma) return launch_alg2_main_mfma(a, st);
  const int tpb = (g.b + kA2Rows - 1) / kA2Rows;
  const unsigned grid = (unsigned)((int64_t)g.BH * (g.n / g.b) * tpb);
  if (g.d == 128)
    hipLaunchKernelGGL((alg2_main_kernel<T, 128>), dim3(grid), dim3(kA2Rows), 0, st, a);
  else
    hipLaunchKernelGGL((alg2_main_kernel<T, 64>), dim3(grid), dim3(kA2Rows), 0, st, a);
  return check_launch();
}

int launch_alg2(const Alg2Args& a, hipStream_t st) {
  if (a.g.d != 64 && a.g.d != 128) return HA_ERR_SHAPE;
  if (a.g.dtype == HA_BF16) return launch_alg2_t<uint16_t>(a, st);
  if (a.g.dtype == HA_FP32) return launch_alg2_t<float>(a, st);
  return HA_ERR_DTYPE;
}

}  // namespace ha
