// sortLSH hashing (Definition 1 of the paper; Algorithm 1, "hash rows of Q, K").
//
// code(x) = Gray-sequence position of the word whose bit k is [<x, R[:,k]> > 0].
//
// The stage is a pure stream over X (d*esz bytes in, 1 byte out per row), so the
// layout is chosen for HBM: every lane issues 16-byte loads, a row is spread
// over LPR = d*esz/16 consecutive lanes and a wave covers 64/LPR whole rows per
// load instruction (fully coalesced 1 KiB).  Each lane multiplies its 16 bytes
// of the row with its slice of R held in registers as fp64 and the LPR partial
// sums of the (up to 8) projections are combined by a transposing butterfly:
// each exchange halves the number of values a lane carries, so 8 values cost 8
// exchanges instead of 8*log2(LPR).
//
// Accumulation is fp64: inputs are bf16 or fp32 and R is fp32, so every product
// is exact in fp64 and the sum carries a relative error of about d * 2^-53.  A
// sign can therefore differ from an infinitely precise evaluation only for
// projections that are zero to ~1e-13, which keeps bucket codes reproducible
// against any fp64 reference.
#include "ha_common.h"

namespace ha {

template <typename T>
struct Elem;
template <>
struct Elem<uint16_t> {  // bf16 bit patterns
  static constexpr int kPerLane = 8;
  __device__ static void unpack(const uint4& raw, double* x) {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = (double)__uint_as_float(w[i] << 16);
      x[2 * i + 1] = (double)__uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
};
template <>
struct Elem<float> {
  static constexpr int kPerLane = 4;
  __device__ static void unpack(const uint4& raw, double* x) {
    x[0] = (double)__uint_as_float(raw.x);
    x[1] = (double)__uint_as_float(raw.y);
    x[2] = (double)__uint_as_float(raw.z);
    x[3] = (double)__uint_as_float(raw.w);
  }
};

// Sum v[k] over the LPR lanes of a row; lane l ends with projection (l / (LPR/8)) & 7.
template <int LPR>
__device__ inline double reduce_transposed(const double* v, int l) {
  constexpr int W1 = LPR / 2, W2 = LPR / 4, W3 = LPR / 8;
  const bool u1 = (l & W1) != 0;
  double w4[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const double keep = u1 ? v[4 + j] : v[j];
    const double send = u1 ? v[j] : v[4 + j];
    w4[j] = keep + __shfl_xor(send, W1);
  }
  const bool u2 = (l & W2) != 0;
  double w2[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const double keep = u2 ? w4[2 + j] : w4[j];
    const double send = u2 ? w4[j] : w4[2 + j];
    w2[j] = keep + __shfl_xor(send, W2);
  }
  const bool u3 = (l & W3) != 0;
  const double keep = u3 ? w2[1] : w2[0];
  const double send = u3 ? w2[0] : w2[1];
  double w = keep + __shfl_xor(send, W3);
#pragma unroll
  for (int o = W3 / 2; o >= 1; o >>= 1) w += __shfl_xor(w, o);
  return w;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void lsh_hash_kernel(const T* __restrict__ X, uint8_t* __restrict__ codes,
                                                        int64_t rows, const float* __restrict__ R, int r) {
  constexpr int EPL = Elem<T>::kPerLane;
  constexpr int LPR = D / EPL;   // lanes per row: 8, 16 or 32
  constexpr int RPW = 64 / LPR;  // rows per wave and load
  constexpr int W3 = LPR / 8;
  constexpr int U = 4;           // loads in flight per lane
  const int lane = threadIdx.x & 63;
  const int l = lane % LPR;
  const int jrow = lane / LPR;
  const int c0 = l * EPL;

  double Rr[EPL][8];
#pragma unroll
  for (int e = 0; e < EPL; ++e)
#pragma unroll
    for (int k = 0; k < 8; ++k) Rr[e][k] = (k < r) ? (double)R[(c0 + e) * r + k] : 0.0;

  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  const int64_t ngroups = (rows + RPW - 1) / RPW;

  for (int64_t g0 = wave; g0 < ngroups; g0 += nwaves * U) {
    uint4 raw[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t row = (g0 + u * nwaves) * RPW + jrow;
      raw[u] = make_uint4(0, 0, 0, 0);
      if (row < rows) raw[u] = *reinterpret_cast<const uint4*>(X + row * D + c0);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t grp = g0 + u * nwaves;
      if (grp >= ngroups) break;  // wave-uniform
      double x[EPL];
      Elem<T>::unpack(raw[u], x);
      double acc[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[k] = 0.0;
#pragma unroll
      for (int e = 0; e < EPL; ++e)
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = __builtin_fma(x[e], Rr[e][k], acc[k]);
      const double p = reduce_transposed<LPR>(acc, l);
      const unsigned long long bal = __ballot(p > 0.0);  // 0 and NaN give bit 0
      if (l == 0) {
        const int64_t row = grp * RPW + jrow;
        if (row < rows) {
          const uint32_t rowbits = (uint32_t)(bal >> (jrow * LPR));
          uint32_t word = 0;
          for (int k = 0; k < r; ++k) word |= ((rowbits >> (k * W3)) & 1u) << k;
          // position in the reflected Gray sequence: the i with i ^ (i >> 1) == word
          uint32_t idx = word;
          idx ^= idx >> 1;
          idx ^= idx >> 2;
          idx ^= idx >> 4;
          codes[row] = (uint8_t)idx;
        }
      }
    }
  }
}

int launch_lsh_hash(const void* X, uint8_t* codes, int64_t rows, int d, int dtype, const float* R_dev, int r,
                    hipStream_t st) {
  if (rows <= 0) return HA_OK;
  if (dtype == HA_BF16) return launch_lsh_hash_mfma(X, codes, rows, d, R_dev, r, st);  // matrix-core path
  const int esz = dtype == HA_BF16 ? 2 : 4;
  const int rpw = 64 / (d * esz / 16);
  const int64_t ngroups = (rows + rpw - 1) / rpw;
  int64_t blocks = (ngroups + 4 * 4 - 1) / (4 * 4);  // 4 waves per block, 4 groups per wave and trip
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  dim3 grid((unsigned)blocks), block(256);
  if (dtype == HA_BF16 && d == 128)
    hipLaunchKernelGGL((lsh_hash_kernel<uint16_t, 128>), grid, block, 0, st, (const uint16_t*)X, codes, rows, R_dev, r);
  else if (dtype == HA_BF16 && d == 64)
    hipLaunchKernelGGL((lsh_hash_kernel<uint16_t, 64>), grid, block, 0, st, (const uint16_t*)X, codes, rows, R_dev, r);
  else if (dtype == HA_FP32 && d == 128)
    hipLaunchKernelGGL((lsh_hash_kernel<float, 128>), grid, block, 0, st, (const float*)X, codes, rows, R_dev, r);
  else if (dtype == HA_FP32 && d == 64)
    hipLaunchKernelGGL((lsh_hash_kernel<float, 64>), grid, block, 0, st, (const float*)X, codes, rows, R_dev, r);
  else
    return HA_ERR_SHAPE;
  return check_launch();
}

}  // namespace ha
