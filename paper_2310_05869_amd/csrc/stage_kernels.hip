// Small streaming kernels around the attention kernels:
//   prep            puts the call's random draws into the workspace: the
//                   hyperplane matrix R (Definition 1) and the per-node sample
//                   indices l_1..l_m (Algorithm 2), either derived from the
//                   seed or copied from caller-supplied device arrays
//   gather_rows     the row permutation of Section 4 ("permuting n rows") as a
//                   stage of its own
//   merge_unpermute Algorithm 2's last step (row sum = block part + estimate)
//                   applied to two partial results, with the inverse permutation
// The production path fuses the gather into the attention kernel's loads and
// the merge into its single softmax pass; these kernels exist so that each
// stage can be checked and timed alone.
#include "ha_common.h"

namespace ha {

struct PrepArgs {
  float* R_ws;
  const float* R_dev;
  int32_t* samples_ws;
  const int32_t* samples_dev;
  Geometry g;
  uint64_t seed;
  uint16_t Rb[1024];  // seed-derived R as bf16 bit patterns, [c*r + k]
};

__global__ __launch_bounds__(256) void prep_kernel(PrepArgs a) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int nR = a.g.d * a.g.r;
  if (i < nR) a.R_ws[i] = a.R_dev ? a.R_dev[i] : __uint_as_float((uint32_t)a.Rb[i] << 16);
  const int64_t nS = (int64_t)a.g.total_nodes * a.g.m;
  if (i < nS && a.g.levels > 0) {
    const int heap = (int)(i / a.g.m);
    const int j = (int)(i % a.g.m);
    const int level = 31 - __clz(heap + 1);
    const int node = heap + 1 - (1 << level);
    const NodeRef nr = node_ref(a.g, level, node);
    int32_t v;
    if (a.samples_dev) {
      v = a.samples_dev[i];
      v = v < 0 ? 0 : (v >= nr.s ? nr.s - 1 : v);  // never index outside the node
    } else {
      v = sample_index(a.seed, level, node, nr.s, j);
    }
    a.samples_ws[i] = v;
  }
}

int launch_prep(float* R_ws, const float* R_dev, const uint16_t* R_bf16_host, int32_t* samples_ws,
                const int32_t* samples_dev, const Geometry& g, uint64_t seed, hipStream_t st) {
  PrepArgs a{};
  a.R_ws = R_ws;
  a.R_dev = R_dev;
  a.samples_ws = samples_ws;
  a.samples_dev = samples_dev;
  a.g = g;
  a.seed = seed;
  if (R_bf16_host)
    for (int i = 0; i < g.d * g.r; ++i) a.Rb[i] = R_bf16_host[i];
  int64_t work = (int64_t)g.total_nodes * g.m;
  if (work < g.d * g.r) work = g.d * g.r;
  dim3 grid((unsigned)((work + 255) / 256)), block(256);
  hipLaunchKernelGGL(prep_kernel, grid, block, 0, st, a);
  return check_launch();
}

// ---------------------------------------------------------------------------
// 16 bytes per lane; a row of `chunks` 16-byte pieces is read and written by
// consecutive lanes.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ src,
                                                           const int32_t* __restrict__ idx,
                                                           uint4* __restrict__ dst, int64_t total_rows, int n,
                                                           int chunks) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t total = total_rows * chunks;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int64_t row = i / chunks;
    const int c = (int)(i % chunks);
    const int64_t g = row / n;
    const int64_t srow = g * n + idx[row];
    dst[i] = src[srow * chunks + c];
  }
}

int launch_gather_rows(const void* src, const int32_t* idx, void* dst, int groups, int n, int d, int dtype,
                       hipStream_t st) {
  const int64_t rows = (int64_t)groups * n;
  if (rows <= 0) return HA_OK;
  const int chunks = d * (dtype == HA_BF16 ? 2 : 4) / 16;
  int64_t blocks = (rows * chunks + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const uint4*)src, idx,
                     (uint4*)dst, rows, n, chunks);
  return check_launch();
}

// ---------------------------------------------------------------------------
__device__ inline uint32_t pack_bf16x2(float a, float b) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  typedef float f2 __attribute__((ext_vector_type(2)));
  const bf2 p = __builtin_convertvector((f2){a, b}, bf2);
  return *reinterpret_cast<const uint32_t*>(&p);
}

// One lane per 4 consecutive elements of a row.
__global__ __launch_bounds__(256) void merge_unpermute_kernel(const float4* __restrict__ o_b,
                                                               const float* __restrict__ lse_b,
                                                               const float4* __restrict__ o_r,
                                                               const float* __restrict__ lse_r,
                                                               const int32_t* __restrict__ perm_q, void* out,
                                                               float* lse, int64_t total_rows, int n, int d,
                                                               int dtype) {
  const int q4 = d / 4;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t total = total_rows * q4;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int64_t row = i / q4;
    const int c = (int)(i % q4);
    const float lb = lse_b[row], lr = lse_r[row];
    const float mx = fmaxf(lb, lr);
    float wb = 0.f, wr = 0.f, L = -INFINITY;
    if (mx > -INFINITY) {
      const float eb = expf(lb - mx), er = expf(lr - mx);
      const float den = eb + er;
      wb = eb / den;
      wr = er / den;
      L = mx + logf(den);
    }
    const float4 a = o_b[i], b = o_r[i];
    float4 o;
    o.x = wb * a.x + wr * b.x;
    o.y = wb * a.y + wr * b.y;
    o.z = wb * a.z + wr * b.z;
    o.w = wb * a.w + wr * b.w;
    const int64_t g = row / n;
    const int64_t drow = g * n + perm_q[row];
    if (dtype == HA_BF16) {
      uint2 v;
      v.x = pack_bf16x2(o.x, o.y);
      v.y = pack_bf16x2(o.z, o.w);
      reinterpret_cast<uint2*>(out)[drow * q4 + c] = v;
    } else {
      reinterpret_cast<float4*>(out)[drow * q4 + c] = o;
    }
    if (c == 0) lse[drow] = L;
  }
}

int launch_merge_unpermute(const float* o_b, const float* lse_b, const float* o_r, const float* lse_r,
                           const int32_t* perm_q, void* out, float* lse, int groups, int n, int d, int dtype,
                           hipStream_t st) {
  const int64_t rows = (int64_t)groups * n;
  if (rows <= 0) return HA_OK;
  int64_t blocks = (rows * (d / 4) + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(merge_unpermute_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const float4*)o_b, lse_b,
                     (const float4*)o_r, lse_r, perm_q, out, lse, rows, n, d, dtype);
  return check_launch();
}

}  // namespace ha
