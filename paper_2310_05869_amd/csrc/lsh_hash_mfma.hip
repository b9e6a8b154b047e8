// sortLSH hashing of bf16 rows (Definition 1; Algorithm 1, "hash rows of Q, K")
// at HBM speed: the r projections of 32 rows are one chain of bf16 MFMAs, and
// only the rare rows whose sign that arithmetic cannot certify are redone in
// exact fp64.
//
//   P   = X R          32 rows x 32 columns (r of them real) per wave and trip
//   P'  = |X| |R|      same shape: sum_c |x_c R_ck|, the scale of the rounding error
//
// A wave reads 32 rows straight from global memory in the MFMA's operand layout
// (lane l: row l%32, 8 consecutive elements starting at 16*ks + 8*(l/32)); R
// and |R| sit in registers as the other operand.  The products are formed as
// R^T X^T so that a lane ends up with the projections of ONE row.  bf16 x bf16 products are exact; the
// fp32 accumulation of the d products deviates from the exact sum by far less
// than 2^-14 * P' (d <= 128 terms, fp32 unit roundoff 2^-24 per add, with a 4x
// margin for the matrix core's internal order).  So sign(P) is certified
// wherever |P| > 2^-14 P'; any row with an uncertified projection (a fraction
// of a percent of rows) is recomputed by the whole wave in fp64, whose sum of
// exact products carries a relative error of about d * 2^-53.  The resulting
// codes are those of an fp64 evaluation, bit for bit, except for projections
// that vanish to ~1e-13.
//
// If R holds values that are not bf16-representable (caller-supplied
// hyperplanes), every row takes the fp64 path.
#include "ha_common.h"

namespace ha {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Two packed non-negative bf16 values times 2^-14 (exact: exponent minus 14);
// values below 2^-112 become zero.
__device__ inline uint32_t scale_bf16x2_down14(uint32_t v) {
  const uint32_t lo = v & 0xFFFFu, hi = v >> 16;
  const uint32_t sub = 14u << 7;
  const uint32_t lo2 = lo >= sub + 0x80u ? lo - sub : 0u;
  const uint32_t hi2 = hi >= sub + 0x80u ? hi - sub : 0u;
  return lo2 | (hi2 << 16);
}

template <int D>
__global__ __launch_bounds__(256) void lsh_hash_mfma_kernel(const uint16_t* __restrict__ X,
                                                             uint8_t* __restrict__ codes, int64_t rows,
                                                             const float* __restrict__ R, int r) {
  constexpr int KS = D / 16;
  constexpr int EL = D / 64;  // elements per lane on the fp64 path
  const int lane = threadIdx.x & 63;
  const int n = lane & 31, h = lane >> 5;

  // matrix operands R^T and |R|^T as bf16: projection n (zero for n >= r)
  u32x4 rb[KS], rabs[KS];
  bool exact = true;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    uint32_t pk[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      uint32_t lo = 0, hi = 0;
      if (n < r) {
        lo = __float_as_uint(R[(16 * ks + 8 * h + 2 * e2) * r + n]);
        hi = __float_as_uint(R[(16 * ks + 8 * h + 2 * e2 + 1) * r + n]);
      }
      exact = exact && ((lo & 0xFFFFu) == 0) && ((hi & 0xFFFFu) == 0);
      pk[e2] = (lo >> 16) | (hi & 0xFFFF0000u);
    }
    rb[ks] = (u32x4){pk[0], pk[1], pk[2], pk[3]};
    rabs[ks] = rb[ks] & 0x7FFF7FFFu;
  }
  // |R| * 2^-14, so that the second MFMA chain yields the doubt threshold itself
  // (entries below 2^-112 drop out of it; their products are far below any rounding error)
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int e = 0; e < 4; ++e) rabs[ks][e] = scale_bf16x2_down14(rabs[ks][e]);
  const bool all_exact = __all(exact);

  // for the fp64 path: R in fp32, eight columns per row (zero beyond r), and one
  // row of X per wave
  __shared__ __attribute__((aligned(16))) float Rs[D * 8];
  __shared__ __attribute__((aligned(16))) uint16_t xrow[4][D];
  const int wv = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < D * 8; i += blockDim.x) Rs[i] = (i % 8) < r ? R[(i / 8) * r + (i % 8)] : 0.f;
  __syncthreads();

  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  const int64_t ngroups = (rows + 31) / 32;

  auto load_group = [&](int64_t g, u32x4 (&xa)[KS]) {
    int64_t lrow = g * 32 + n;
    if (lrow >= rows) lrow = rows - 1;
    const u32x4* xp = reinterpret_cast<const u32x4*>(X + lrow * D + 8 * h);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) xa[ks] = xp[2 * ks];
  };
  const uint32_t mask_r = (1u << r) - 1u;
  auto trip = [&](int64_t g, u32x4 (&xa)[KS], u32x4 (&xn)[KS]) {
    const int64_t row0 = g * 32;
    // unconditional (past the end: this trip's own rows again, a cache hit), so
    // the count of loads in flight is the same on every path and the waits
    // before the MFMAs below leave the two younger groups in flight
    load_group(g + 2 * nwaves < ngroups ? g + 2 * nwaves : g, xn);

    f32x16 p, pa;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      p[i] = 0.f;
      pa[i] = 0.f;
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      p = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, rb[ks]), __builtin_bit_cast(bf16x8, xa[ks]),
                                                  p, 0, 0, 0);
      const u32x4 ax = xa[ks] & 0x7FFF7FFFu;
      pa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, rabs[ks]), __builtin_bit_cast(bf16x8, ax),
                                                   pa, 0, 0, 0);
    }

    // The product is taken transposed (R^T X^T), so accumulator element i < 4 of
    // lane (n, h) is projection 4 h + i of row n: every lane forms one nibble of
    // its row's sign word, and the two halves of the wave swap nibbles.
    uint32_t nib = 0;
    bool lane_doubt = !all_exact;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool real = 4 * h + i < r;
      nib |= (p[i] > 0.f ? 1u : 0u) << i;
      lane_doubt = lane_doubt || (real && !(fabsf(p[i]) > pa[i]));
    }
    nib <<= 4 * h;
    uint32_t my_word = (nib | (uint32_t)__shfl_xor((int)nib, 32)) & mask_r;
    const unsigned long long dbal = __ballot(lane_doubt);
    const uint32_t doubt_rows = (uint32_t)dbal | (uint32_t)(dbal >> 32);
    const int64_t left = rows - row0;
    // a wave-uniform row mask, held in scalar registers
    uint32_t redo = __builtin_amdgcn_readfirstlane(doubt_rows);
    if (left < 32) redo &= (1u << left) - 1u;

    // Exact fp64 evaluation of the doubtful rows, one row at a time by the whole
    // wave: the two lanes that hold row j hand it over through LDS, then lane l
    // multiplies elements EL*l .. EL*l + EL - 1 with their rows of R.
    while (redo) {
      const int j = __builtin_ctz(redo);
      redo &= redo - 1;
      if (n == j) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) *reinterpret_cast<u32x4*>(&xrow[wv][16 * ks + 8 * h]) = xa[ks];
      }
      __builtin_amdgcn_wave_barrier();  // LDS serves one wave's requests in order
      double acc[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[k] = 0.0;
#pragma unroll
      for (int e = 0; e < EL; ++e) {
        const double x = (double)__uint_as_float((uint32_t)xrow[wv][lane * EL + e] << 16);
        const f32x4 r0 = *reinterpret_cast<const f32x4*>(&Rs[(lane * EL + e) * 8]);
        const f32x4 r1 = *reinterpret_cast<const f32x4*>(&Rs[(lane * EL + e) * 8 + 4]);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          acc[k] = __builtin_fma(x, (double)r0[k], acc[k]);
          acc[4 + k] = __builtin_fma(x, (double)r1[k], acc[4 + k]);
        }
      }
      __builtin_amdgcn_wave_barrier();
      // transposing butterfly over the 64 lanes: 8 -> 4 -> 2 -> 1 values, then plain
      const bool u1 = (lane & 32) != 0;
      double w4[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const double keep = u1 ? acc[4 + q] : acc[q];
        const double send = u1 ? acc[q] : acc[4 + q];
        w4[q] = keep + __shfl_xor(send, 32);
      }
      const bool u2 = (lane & 16) != 0;
      double w2[2];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const double keep = u2 ? w4[2 + q] : w4[q];
        const double send = u2 ? w4[q] : w4[2 + q];
        w2[q] = keep + __shfl_xor(send, 16);
      }
      const bool u3 = (lane & 8) != 0;
      double ws = (u3 ? w2[1] : w2[0]) + __shfl_xor(u3 ? w2[0] : w2[1], 8);
      ws += __shfl_xor(ws, 4);
      ws += __shfl_xor(ws, 2);
      ws += __shfl_xor(ws, 1);
      // lane l now holds projection (l >> 3) & 7
      const unsigned long long bal = __ballot(ws > 0.0);
      uint32_t word = 0;
#pragma unroll
      for (int k = 0; k < 8; ++k) word |= (uint32_t)((bal >> (8 * k)) & 1ull) << k;
      if (lane == j) my_word = word & mask_r;
    }

    if (lane < 32 && row0 + lane < rows) {
      // position in the reflected Gray sequence: the i with i ^ (i >> 1) == word
      uint32_t idx = my_word;
      idx ^= idx >> 1;
      idx ^= idx >> 2;
      idx ^= idx >> 4;
      codes[row0 + lane] = (uint8_t)idx;
    }
  };
  // the rows of the next two trips are in flight while the current one is
  // processed; three register sets rotate so nothing is copied
  u32x4 xa[KS], xb[KS], xc[KS];
  int64_t g = wave;
  if (g >= ngroups) return;
  load_group(g, xa);
  load_group(g + nwaves < ngroups ? g + nwaves : g, xb);
  while (g < ngroups) {
    trip(g, xa, xc);
    g += nwaves;
    if (g >= ngroups) break;
    trip(g, xb, xa);
    g += nwaves;
    if (g >= ngroups) break;
    trip(g, xc, xb);
    g += nwaves;
  }
}

#ifndef HA_HASH_BLOCKS
#define HA_HASH_BLOCKS 512
#endif
// resident-sized grid (two 4-wave blocks per CU): every wave streams many 32-row groups
constexpr int kHashBlocks = HA_HASH_BLOCKS;

int launch_lsh_hash_mfma(const void* X, uint8_t* codes, int64_t rows, int d, const float* R_dev, int r,
                         hipStream_t st) {
  if (rows <= 0) return HA_OK;
  const int64_t ngroups = (rows + 31) / 32;
  int64_t blocks = (ngroups + 3) / 4;
  if (blocks > kHashBlocks) blocks = kHashBlocks;
  dim3 grid((unsigned)blocks), block(256);
  if (d == 128)
    hipLaunchKernelGGL((lsh_hash_mfma_kernel<128>), grid, block, 0, st, (const uint16_t*)X, codes, rows, R_dev, r);
  else if (d == 64)
    hipLaunchKernelGGL((lsh_hash_mfma_kernel<64>), grid, block, 0, st, (const uint16_t*)X, codes, rows, R_dev, r);
  else
    return HA_ERR_SHAPE;
  return check_launch();
}

}  // namespace ha
