// Small kernels around the backward passes: delta_i = <dO_i, O_i>, the ordered
// reduction of the sampled keys' gradients of one level into the accumulated
// key rows, and the conversion of accumulated rows to the tensors' dtype
// (unmasked problems, whose single node holds the whole result).
// Every sum is taken in a fixed order: results are bit-reproducible.
#include "attn_common.h"
#include "bwd_common.h"

namespace ha {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// One group of D/8 lanes per row; 8 elements per lane.  O is read from its
// unrounded fp32 copy when there is one: with the bf16 tensor, delta carries the
// output's rounding error, which matters where <dO_i, v_j> - delta_i cancels
// (rows whose weight sits on few keys).
template <int D>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const uint16_t* __restrict__ O, const float* __restrict__ O32,
                                                        const uint16_t* __restrict__ G, float* __restrict__ delta,
                                                        int64_t rows) {
  constexpr int LPR = D / 8;  // lanes per row
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t row = t / LPR;
  const int part = (int)(t % LPR);
  float s = 0.f;
  if (row < rows) {
    const u32x4 g = *reinterpret_cast<const u32x4*>(G + row * D + part * 8);
    float o[8];
    if (O32 != nullptr) {
      const f32x4 a = *reinterpret_cast<const f32x4*>(O32 + row * D + part * 8);
      const f32x4 b = *reinterpret_cast<const f32x4*>(O32 + row * D + part * 8 + 4);
      o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
      o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    } else {
      const u32x4 ob = *reinterpret_cast<const u32x4*>(O + row * D + part * 8);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        o[2 * e] = __uint_as_float(ob[e] << 16);
        o[2 * e + 1] = __uint_as_float(ob[e] & 0xFFFF0000u);
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      s = __builtin_fmaf(o[2 * e], __uint_as_float(g[e] << 16), s);
      s = __builtin_fmaf(o[2 * e + 1], __uint_as_float(g[e] & 0xFFFF0000u), s);
    }
  }
#pragma unroll
  for (int off = LPR / 2; off >= 1; off >>= 1) s += __shfl_xor(s, off);
  if (row < rows && part == 0) delta[row] = s;
}

// fp32 tensors: the same dot product, straight from O and dO.
template <int D>
__global__ __launch_bounds__(256) void bwd_delta_f32_kernel(const float* __restrict__ O, const float* __restrict__ G,
                                                            float* __restrict__ delta, int64_t rows) {
  constexpr int LPR = D / 8;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t row = t / LPR;
  const int part = (int)(t % LPR);
  float s = 0.f;
  if (row < rows) {
#pragma unroll
    for (int e = 0; e < 8; ++e) s = __builtin_fmaf(O[row * D + part * 8 + e], G[row * D + part * 8 + e], s);
  }
#pragma unroll
  for (int off = LPR / 2; off >= 1; off >>= 1) s += __shfl_xor(s, off);
  if (row < rows && part == 0) delta[row] = s;
}

int launch_bwd_delta(const void* O, const float* O_f32, const void* dO, float* delta, int64_t rows, int d, int dtype,
                     hipStream_t st) {
  if (rows <= 0) return HA_OK;
  const int lpr = d / 8;
  const int64_t threads = rows * lpr;
  const unsigned grid = (unsigned)((threads + 255) / 256);
  if (dtype == HA_FP32) {
    if (d == 128)
      hipLaunchKernelGGL((bwd_delta_f32_kernel<128>), dim3(grid), dim3(256), 0, st, (const float*)O, (const float*)dO, delta, rows);
    else if (d == 64)
      hipLaunchKernelGGL((bwd_delta_f32_kernel<64>), dim3(grid), dim3(256), 0, st, (const float*)O, (const float*)dO, delta, rows);
    else
      return HA_ERR_SHAPE;
    return check_launch();
  }
  if (d == 128)
    hipLaunchKernelGGL((bwd_delta_kernel<128>), dim3(grid), dim3(256), 0, st, (const uint16_t*)O, O_f32, (const uint16_t*)dO, delta, rows);
  else if (d == 64)
    hipLaunchKernelGGL((bwd_delta_kernel<64>), dim3(grid), dim3(256), 0, st, (const uint16_t*)O, O_f32, (const uint16_t*)dO, delta, rows);
  else
    return HA_ERR_SHAPE;
  return check_launch();
}

// Sampled keys' gradients of one level into the accumulated key rows.  One wave per sample j
// of a (head, node of the level); a lane owns four columns of dK (lanes < d/4) or of dV (the
// next d/4 lanes).  A key may be drawn more than once: the FIRST sample that
// drew a key ("owner") adds, in increasing sample order, the sums of every
// sample of that key, each taken over the node's query chunks in a fixed order;
// the other samples of the key do nothing.  One writer per row and a fixed
// order of additions: reproducible bit for bit.
constexpr int kScatterWaves = 4;

__global__ __launch_bounds__(64 * kScatterWaves) void bwd_sample_scatter_kernel(BwdArgs a, int level,
                                                                                const float* __restrict__ samp_k,
                                                                                const float* __restrict__ samp_v,
                                                                                float* part_k, float* part_v) {
  __shared__ int32_t keys[4096];
  const Geometry& g = a.f.g;
  const int d = g.d, m = g.m;
  const int groups = (m + kScatterWaves - 1) / kScatterWaves;
  const int grp = blockIdx.x % groups;
  const int rest = blockIdx.x / groups;
  const int nodes = g.causal ? (1 << level) : 1;
  const int bh = rest / nodes;
  const int node = rest % nodes;
  const int heap = (1 << level) - 1 + node;
  const NodeRef nr = node_ref(g, level, node);
  const int cpn = bwd_chunks_per_node(g, level);
  const int64_t key_row0 = (int64_t)bh * g.n + nr.k_start;  // the node's first key in the accumulated rows
  int64_t lvl_row0 = 0;
#pragma unroll
  for (int l = 0; l < kBwdMaxLevels; ++l)
    if (l == level) lvl_row0 = a.samp_row_off[l];
  const int64_t row0 = lvl_row0 + ((int64_t)bh * nodes + node) * cpn * m;

  for (int j = threadIdx.x; j < m; j += blockDim.x) keys[j] = a.f.samples[(int64_t)heap * m + j];
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int j = grp * kScatterWaves + (threadIdx.x >> 6);
  if (j >= m) return;
  const int key = keys[j];
  // an earlier sample of the same key owns it
  for (int base = 0; base < j; base += 64) {
    const int jj = base + lane;
    if (__any(jj < j && keys[jj] == key)) return;
  }
  const int q4 = d / 4;  // column quads per row
  const bool active = lane < 2 * q4;
  const float* src = lane < q4 ? samp_k : samp_v;
  float* dst = lane < q4 ? part_k : part_v;
  const int c4 = (lane % q4) * 4;
  f32x4 total = {0.f, 0.f, 0.f, 0.f};
  for (int base = j; base < m; base += 64) {
    const int jl = base + lane;
    unsigned long long same = __ballot(jl < m && keys[jl] == key);
    while (same) {
      const int jj = base + __builtin_ctzll(same);
      same &= same - 1;
      if (active) {
        const float* p = src + (row0 + jj) * d + c4;
        const int64_t step = (int64_t)m * d;
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0, s2 = s0, s3 = s0;
        int qc = 0;
        for (; qc + 4 <= cpn; qc += 4) {
          s0 += *reinterpret_cast<const f32x4*>(p + (qc + 0) * step);
          s1 += *reinterpret_cast<const f32x4*>(p + (qc + 1) * step);
          s2 += *reinterpret_cast<const f32x4*>(p + (qc + 2) * step);
          s3 += *reinterpret_cast<const f32x4*>(p + (qc + 3) * step);
        }
        for (; qc < cpn; ++qc) s0 += *reinterpret_cast<const f32x4*>(p + qc * step);
        total += (s0 + s1) + (s2 + s3);
      }
    }
  }
  if (active) {
    f32x4* out = reinterpret_cast<f32x4*>(dst + (key_row0 + key) * d + c4);
    *out = *out + total;
  }
}

int launch_bwd_sample_scatter(const BwdArgs& a, int level, const float* samp_k, const float* samp_v, float* acc_k,
                              float* acc_v, hipStream_t st) {
  const Geometry& g = a.f.g;
  if (g.m <= 0 || level < 0 || level >= g.levels) return HA_OK;
  const int nodes = g.causal ? (1 << level) : 1;
  const int groups = (g.m + kScatterWaves - 1) / kScatterWaves;
  const int64_t grid = (int64_t)g.BH * nodes * groups;
  if (grid > kMaxGrid) return HA_ERR_SHAPE;
  hipLaunchKernelGGL(bwd_sample_scatter_kernel, dim3((unsigned)grid), dim3(64 * kScatterWaves), 0, st, a, level, samp_k,
                     samp_v, acc_k, acc_v);
  return check_launch();
}

// Accumulated fp32 rows to the tensors' dtype.
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_convert_kernel(const float* __restrict__ acc, T* __restrict__ dst, int64_t rows) {
  constexpr int LPR = D / 8;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t row = t / LPR;
  const int piece = (int)(t % LPR);
  if (row >= rows) return;
  const f32x4 v0 = *reinterpret_cast<const f32x4*>(acc + row * D + piece * 8);
  const f32x4 v1 = *reinterpret_cast<const f32x4*>(acc + row * D + piece * 8 + 4);
  if constexpr (sizeof(T) == 4) {
    *reinterpret_cast<f32x4*>(dst + row * D + piece * 8) = v0;
    *reinterpret_cast<f32x4*>(dst + row * D + piece * 8 + 4) = v1;
  } else {
    const u32x4 pk = {pack_bf16x2(v0.x, v0.y), pack_bf16x2(v0.z, v0.w), pack_bf16x2(v1.x, v1.y), pack_bf16x2(v1.z, v1.w)};
    *reinterpret_cast<u32x4*>(dst + row * D + piece * 8) = pk;
  }
}

int launch_bwd_convert(const float* acc, void* dst, const Geometry& g, hipStream_t st) {
  const int64_t rows = (int64_t)g.BH * g.n;
  if (rows <= 0) return HA_OK;
  const int lpr = g.d / 8;
  const unsigned grid = (unsigned)((rows * lpr + 255) / 256);
  const bool f32 = g.dtype == HA_FP32;
  if (g.d == 128 && f32)
    hipLaunchKernelGGL((bwd_convert_kernel<float, 128>), dim3(grid), dim3(256), 0, st, acc, (float*)dst, rows);
  else if (g.d == 64 && f32)
    hipLaunchKernelGGL((bwd_convert_kernel<float, 64>), dim3(grid), dim3(256), 0, st, acc, (float*)dst, rows);
  else if (g.d == 128)
    hipLaunchKernelGGL((bwd_convert_kernel<uint16_t, 128>), dim3(grid), dim3(256), 0, st, acc, (uint16_t*)dst, rows);
  else if (g.d == 64)
    hipLaunchKernelGGL((bwd_convert_kernel<uint16_t, 64>), dim3(grid), dim3(256), 0, st, acc, (uint16_t*)dst, rows);
  else
    return HA_ERR_SHAPE;
  return check_launch();
}

}  // namespace ha
