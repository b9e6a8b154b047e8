// sortLSH hashing of bf16 rows (Definition 1; Algorithm 1, "hash rows of Q, K")
// at HBM speed: the r projections of 32 rows are one chain of bf16 MFMAs, and
// only the rare rows whose sign that arithmetic cannot certify are redone in
// exact fp64.
//
//   P   = X R          32 rows x 32 columns (r of them real) per wave and trip
//   P'  = |X| |R|      same shape: sum_c |x_c R_ck|, the scale of the rounding error
//
// A wave reads 32 rows straight from global memory in the MFMA's A layout
// (lane l: row l%32, 8 consecutive elements starting at 16*ks + 8*(l/32)); R
// and |R| sit in registers as B operands.  bf16 x bf16 products are exact; the
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

  // B operands: R and |R| as bf16, column n (zero for n >= r)
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
    if (g + nwaves < ngroups) load_group(g + nwaves, xn);

    f32x16 p, pa;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      p[i] = 0.f;
      pa[i] = 0.f;
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      p = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xa[ks]), __builtin_bit_cast(bf16x8, rb[ks]),
                                                  p, 0, 0, 0);
      const u32x4 ax = xa[ks] & 0x7FFF7FFFu;
      pa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ax), __builtin_bit_cast(bf16x8, rabs[ks]),
                                                   pa, 0, 0, 0);
    }

    // Accumulator element i of lane (n, h) is row 8*(i/4) + 4*h + i%4, column n:
    // a ballot over the wave yields the sign word of row j_lo = 8*(i/4) + i%4 in
    // its low half and of row j_lo + 4 in its high half.  The words are uniform
    // values, dropped into lane j of my_word; doubt is collected as a row mask.
    uint32_t my_word = 0;
    uint32_t doubt_rows = all_exact ? 0u : 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const unsigned long long sign = __ballot(p[i] > 0.f);
      const unsigned long long doubt = __ballot(!(fabsf(p[i]) > pa[i]));
      const int j_lo = 8 * (i / 4) + (i % 4);
      asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(my_word) : "s"((uint32_t)sign & mask_r), "n"(j_lo));
      asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(my_word) : "s"((uint32_t)(sign >> 32) & mask_r), "n"(j_lo + 4));
      if ((uint32_t)doubt & mask_r) doubt_rows |= 1u << j_lo;
      if ((uint32_t)(doubt >> 32) & mask_r) doubt_rows |= 1u << (j_lo + 4);
    }
    const int64_t left = rows - row0;
    unsigned long long redo = doubt_rows;
    if (left < 32) redo &= (1ull << left) - 1ull;

    // exact fp64 evaluation of the doubtful rows, one row at a time by the whole wave
    while (redo) {
      const int j = __ffsll((long long)redo) - 1;
      redo &= redo - 1;
      const uint16_t* xr = X + (row0 + j) * D + lane * EL;
      double acc[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[k] = 0.0;
#pragma unroll
      for (int e = 0; e < EL; ++e) {
        const double x = (double)__uint_as_float((uint32_t)xr[e] << 16);
#pragma unroll
        for (int k = 0; k < 8; ++k)
          if (k < r) acc[k] = __builtin_fma(x, (double)R[(lane * EL + e) * r + k], acc[k]);
      }
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
      for (int k = 0; k < r; ++k) word |= (uint32_t)((bal >> (8 * k)) & 1ull) << k;
      if (lane == j) my_word = word;
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
  // rows of the next trip are requested before the current trip is processed;
  // two trips per loop pass so the two register sets swap roles without copies
  u32x4 xa[KS], xb[KS];
  int64_t g = wave;
  if (g < ngroups) load_group(g, xa);
  for (; g + nwaves < ngroups; g += 2 * nwaves) {
    trip(g, xa, xb);
    trip(g + nwaves, xb, xa);
  }
  if (g < ngroups) trip(g, xa, xb);
}

int launch_lsh_hash_mfma(const void* X, uint8_t* codes, int64_t rows, int d, const float* R_dev, int r,
                         hipStream_t st) {
  if (rows <= 0) return HA_OK;
  const int64_t ngroups = (rows + 31) / 32;
  int64_t blocks = (ngroups + 3) / 4;
  if (blocks > 2048) blocks = 2048;
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
