// Measurement aids, not part of the method: the matrix-core and HBM rates this
// GPU sustains on code that does nothing else, so that a kernel's achieved rate
// can be set against an attainable figure as well as the published peak.
//
//   MFMA   every wave runs independent chains of v_mfma_f32_32x32x16_bf16 (the
//          instruction the attention kernels use) over eight register-resident
//          operand pairs of pseudo-random values; the rate depends on how long the
//          probe runs (the chip lowers its clock within milliseconds under this
//          load), so `iters` should give a duration like the kernel's it is set against.
//   HBM    a grid-stride read of a buffer (16 bytes per lane and step), and a
//          copy of its first half onto its second.
// Both time themselves with events on the given stream and wait for it.
#include "ha_common.h"

namespace ha {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kChains = 4;       // independent accumulators per wave
constexpr int kPerIter = 8;      // MFMAs per chain and loop trip

constexpr int kOperands = 8;     // operand pairs a wave rotates through

// bf16 pair with pseudo-random sign, mantissa and an exponent in [2^-3, 2): operands that differ
// from one instruction to the next, as a kernel's do (constant operands toggle no wires and
// flatter the rate)
__device__ inline uint32_t rate_operand_bits(uint32_t seed) {
  uint32_t v = 0;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    seed = seed * 1664525u + 1013904223u;
    const uint32_t b = ((seed >> 31) << 15) | ((0x7Cu + ((seed >> 20) & 3u)) << 7) | ((seed >> 8) & 0x7Fu);
    v |= b << (16 * half);
  }
  return v;
}

__global__ __launch_bounds__(256) void mfma_rate_kernel(float* out, int iters) {
  f32x16 acc[kChains];
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
  bf16x8 x[kOperands], y[kOperands];
#pragma unroll
  for (int u = 0; u < kOperands; ++u) {
    u32x4 xb, yb;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      xb[i] = rate_operand_bits((threadIdx.x * 64u + u * 8u + i) * 2654435761u);
      yb[i] = rate_operand_bits((threadIdx.x * 64u + u * 8u + i + 4u) * 2246822519u);
    }
    x[u] = __builtin_bit_cast(bf16x8, xb);
    y[u] = __builtin_bit_cast(bf16x8, yb);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < kPerIter; ++u)
#pragma unroll
      for (int c = 0; c < kChains; ++c)
        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[(u + c) % kOperands], y[(u + 2 * c) % kOperands], acc[c], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[c][i];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void read_rate_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* flag) {
  u32x4 acc = {0, 0, 0, 0};
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) acc ^= src[i];
  // the sum is data dependent, so the loads cannot be dropped; it is written only for one value
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) *flag = 1u;
}

__global__ __launch_bounds__(256) void copy_rate_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// ---------------------------------------------------------------------------
// Issue-rate probes: shader cycles per instruction of what the attention loop is
// made of, alone and next to each other, read from the shader clock by one wave
// while every CU runs the same code.  They answer which of the three things a
// 64-key tile needs per wave -- 32 MFMAs, about 140 vector instructions of
// softmax work, 32 KiB of operand fragments from LDS -- the loop runs out of
// first.
// ---------------------------------------------------------------------------
enum IssueProbe : int {
  kProbeExp, kProbeFma, kProbeCvtPk, kProbeMax3, kProbeMfma, kProbeMfmaFma4, kProbeMfmaFma7, kProbeMfmaExpFma3,
  kProbeMfmaExpFma4, kProbeSplitMfmaValu, kProbeLdsRead128, kProbeLdsReadTr64, kProbeLdsWrite128, kProbeCount
};

#define HA_REP8(x) x x x x x x x x
#define HA_EXP(r) asm volatile("v_exp_f32 %0, %0" : "+v"(r));
#define HA_FMA(r) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(r) : "v"(k1), "v"(k2));
#define HA_MAX3(r) asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(r) : "v"(k1), "v"(k2));
#define HA_CVT(r) asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(k1), "v"(k2));
#define HA_MFMA(acc) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));

constexpr int kProbeIters = 1000;

// 8 waves per workgroup (two per SIMD), one workgroup per CU.  out[probe * 2 + 0 / 1] = cycles the
// first wave of each half of workgroup 0 took for kProbeIters trips.
template <int P>
__global__ __launch_bounds__(512) void issue_probe_kernel(long long* out, float* sink) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[65536];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float r[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = threadIdx.x * 0.001f + i * 0.01f - 0.5f;
  float k1 = 0.999f, k2 = -0.001f;
  asm volatile("" : "+v"(k1), "+v"(k2));
  f32x16 acc0, acc1;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    acc0[i] = 0.f;
    acc1[i] = 0.f;
  }
  bf16x8 a, b;
  {
    u32x4 xb, yb;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      xb[i] = rate_operand_bits((threadIdx.x * 8u + i) * 2654435761u);
      yb[i] = rate_operand_bits((threadIdx.x * 8u + i + 4u) * 2246822519u);
    }
    a = __builtin_bit_cast(bf16x8, xb);
    b = __builtin_bit_cast(bf16x8, yb);
  }
  for (int i = threadIdx.x; i < 16384; i += 512) reinterpret_cast<uint32_t*>(lds)[i] = i * 2654435761u;
  __syncthreads();
  u32x4 lacc = {0, 0, 0, 0};
  const unsigned char* lp = lds + wave * 8192 + lane * 16;
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
  const long long c0 = clock64();
  for (int it = 0; it < kProbeIters; ++it) {
    if (P == kProbeExp) { HA_REP8(HA_EXP(r[0]) HA_EXP(r[1]) HA_EXP(r[2]) HA_EXP(r[3]) HA_EXP(r[4]) HA_EXP(r[5]) HA_EXP(r[6]) HA_EXP(r[7])) }
    if (P == kProbeFma) { HA_REP8(HA_FMA(r[0]) HA_FMA(r[1]) HA_FMA(r[2]) HA_FMA(r[3]) HA_FMA(r[4]) HA_FMA(r[5]) HA_FMA(r[6]) HA_FMA(r[7])) }
    if (P == kProbeCvtPk) { HA_REP8(HA_CVT(r[0]) HA_CVT(r[1]) HA_CVT(r[2]) HA_CVT(r[3]) HA_CVT(r[4]) HA_CVT(r[5]) HA_CVT(r[6]) HA_CVT(r[7])) }
    if (P == kProbeMax3) { HA_REP8(HA_MAX3(r[0]) HA_MAX3(r[1]) HA_MAX3(r[2]) HA_MAX3(r[3]) HA_MAX3(r[4]) HA_MAX3(r[5]) HA_MAX3(r[6]) HA_MAX3(r[7])) }
    if (P == kProbeMfma) { HA_REP8(HA_MFMA(acc0) HA_MFMA(acc1)) }
    if (P == kProbeMfmaFma4) { HA_REP8(HA_MFMA(acc0) HA_FMA(r[0]) HA_FMA(r[1]) HA_FMA(r[2]) HA_FMA(r[3]) HA_MFMA(acc1) HA_FMA(r[4]) HA_FMA(r[5]) HA_FMA(r[6]) HA_FMA(r[7])) }
    if (P == kProbeMfmaFma7) { HA_REP8(HA_MFMA(acc0) HA_FMA(r[0]) HA_FMA(r[1]) HA_FMA(r[2]) HA_FMA(r[3]) HA_FMA(r[4]) HA_FMA(r[5]) HA_FMA(r[6]) HA_MFMA(acc1) HA_FMA(r[7]) HA_FMA(r[0]) HA_FMA(r[1]) HA_FMA(r[2]) HA_FMA(r[3]) HA_FMA(r[4]) HA_FMA(r[5])) }
    if (P == kProbeMfmaExpFma3) { HA_REP8(HA_MFMA(acc0) HA_EXP(r[0]) HA_FMA(r[1]) HA_FMA(r[2]) HA_FMA(r[3]) HA_MFMA(acc1) HA_EXP(r[4]) HA_FMA(r[5]) HA_FMA(r[6]) HA_FMA(r[7])) }
    if (P == kProbeMfmaExpFma4) { HA_REP8(HA_MFMA(acc0) HA_EXP(r[0]) HA_FMA(r[1]) HA_FMA(r[2]) HA_FMA(r[3]) HA_FMA(r[4]) HA_MFMA(acc1) HA_EXP(r[5]) HA_FMA(r[6]) HA_FMA(r[7]) HA_FMA(r[1]) HA_FMA(r[2])) }
    if (P == kProbeSplitMfmaValu) {  // waves 0-3: 16 MFMAs; waves 4-7: the vector work of half a tile (16 exp + 48 others)
      if (wave < 4) { HA_REP8(HA_MFMA(acc0) HA_MFMA(acc1)) }
      else { HA_REP8(HA_EXP(r[0]) HA_FMA(r[1]) HA_FMA(r[2]) HA_FMA(r[3]) HA_EXP(r[4]) HA_FMA(r[5]) HA_FMA(r[6]) HA_FMA(r[7])) }
    }
    if (P == kProbeLdsRead128) {
#pragma unroll
      for (int u = 0; u < 8; ++u) lacc ^= *reinterpret_cast<const u32x4*>(lp + u * 1024);
      asm volatile("" : "+v"(lacc));
    }
    if (P == kProbeLdsReadTr64) {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + wave * 8192 + u * 512 + lane * 8));
        lacc.x ^= (uint32_t)(unsigned short)v.x | ((uint32_t)(unsigned short)v.y << 16);
        lacc.y ^= (uint32_t)(unsigned short)v.z | ((uint32_t)(unsigned short)v.w << 16);
      }
      asm volatile("" : "+v"(lacc));
    }
    if (P == kProbeLdsWrite128) {
#pragma unroll
      for (int u = 0; u < 8; ++u) *reinterpret_cast<u32x4*>(lds + wave * 8192 + u * 1024 + lane * 16) = lacc;
      asm volatile("" : "+v"(lacc)::"memory");
    }
  }
  const long long c1 = clock64();
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += r[i];
#pragma unroll
  for (int i = 0; i < 16; ++i) s += acc0[i] + acc1[i];
  s += (float)(lacc.x ^ lacc.y ^ lacc.z ^ lacc.w) + (float)lds[threadIdx.x];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (blockIdx.x == 0 && lane == 0 && (wave == 0 || wave == 4)) out[P * 2 + (wave >> 2)] = c1 - c0;
}

template <int P>
static void launch_issue_probe(long long* out, float* sink, hipStream_t st) {
  hipLaunchKernelGGL(issue_probe_kernel<P>, dim3(256), dim3(512), 0, st, out, sink);
  if constexpr (P + 1 < kProbeCount) launch_issue_probe<P + 1>(out, sink, st);
}

struct EventPair {
  hipEvent_t a = nullptr, b = nullptr;
  bool ok;
  EventPair() { ok = hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess; }
  ~EventPair() {
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
  }
};

}  // namespace ha

using namespace ha;

extern "C" int ha_measure_mfma_rate(void* buf, size_t bytes, int32_t iters, float* tflops, void* stream) {
  if (!buf || !tflops) return HA_ERR_NULL;
  const int grid = 512;  // two 4-wave workgroups per CU
  if (bytes < (size_t)grid * 256 * sizeof(float)) return HA_ERR_WORKSPACE;
  if (iters < 1 || iters > (1 << 20)) return HA_ERR_SHAPE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  EventPair ev;
  if (!ev.ok) return HA_ERR_LAUNCH;
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(grid), dim3(256), 0, st, static_cast<float*>(buf), 16);  // warm-up
  if (hipEventRecord(ev.a, st) != hipSuccess) return HA_ERR_LAUNCH;
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(grid), dim3(256), 0, st, static_cast<float*>(buf), iters);
  if (hipEventRecord(ev.b, st) != hipSuccess || hipEventSynchronize(ev.b) != hipSuccess) return HA_ERR_LAUNCH;
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess || !(ms > 0.f)) return HA_ERR_LAUNCH;
  const double flop = (double)grid * 4 * iters * kPerIter * kChains * (2.0 * 32 * 32 * 16);
  *tflops = (float)(flop / (ms * 1e-3) / 1e12);
  return check_launch();
}

extern "C" int ha_measure_hbm_rate(void* buf, size_t bytes, float* read_gbs, float* copy_gbs, void* stream) {
  if (!buf || !read_gbs || !copy_gbs) return HA_ERR_NULL;
  if (bytes < (1u << 20) || (reinterpret_cast<uintptr_t>(buf) & 15u)) return HA_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  EventPair ev;
  if (!ev.ok) return HA_ERR_LAUNCH;
  const size_t half16 = bytes / 32;            // 16-byte pieces in each half
  u32x4* lo = static_cast<u32x4*>(buf);
  u32x4* hi = lo + half16;
  uint32_t* flag = reinterpret_cast<uint32_t*>(hi);  // never written in practice; the copy overwrites it anyway
  const int grid = 2048;
  constexpr int kReps = 5;  // the fastest repetition counts (the first warms up)
  float ms = 0.f, best = 0.f;
  for (int rep = 0; rep < kReps; ++rep) {
    if (hipEventRecord(ev.a, st) != hipSuccess) return HA_ERR_LAUNCH;
    hipLaunchKernelGGL(read_rate_kernel, dim3(grid), dim3(256), 0, st, lo, half16, flag);
    if (hipEventRecord(ev.b, st) != hipSuccess || hipEventSynchronize(ev.b) != hipSuccess) return HA_ERR_LAUNCH;
    if (hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess || !(ms > 0.f)) return HA_ERR_LAUNCH;
    if (rep == 0 || ms < best) best = ms;
  }
  *read_gbs = (float)((double)half16 * 16 / (best * 1e-3) / 1e9);
  for (int rep = 0; rep < kReps; ++rep) {
    if (hipEventRecord(ev.a, st) != hipSuccess) return HA_ERR_LAUNCH;
    hipLaunchKernelGGL(copy_rate_kernel, dim3(grid), dim3(256), 0, st, lo, hi, half16);
    if (hipEventRecord(ev.b, st) != hipSuccess || hipEventSynchronize(ev.b) != hipSuccess) return HA_ERR_LAUNCH;
    if (hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess || !(ms > 0.f)) return HA_ERR_LAUNCH;
    if (rep == 0 || ms < best) best = ms;
  }
  *copy_gbs = (float)((double)half16 * 32 / (best * 1e-3) / 1e9);
  return check_launch();
}

extern "C" int32_t ha_issue_probe_count(void) { return kProbeCount; }

extern "C" int ha_measure_issue_rates(void* buf, size_t bytes, float* cycles_host, void* stream) {
  if (!buf || !cycles_host) return HA_ERR_NULL;
  const size_t need = 4096 + (size_t)256 * 512 * sizeof(float);
  if (bytes < need || (reinterpret_cast<uintptr_t>(buf) & 15u)) return HA_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  long long* out = static_cast<long long*>(buf);
  float* sink = reinterpret_cast<float*>(static_cast<unsigned char*>(buf) + 4096);
  launch_issue_probe<0>(out, sink, st);
  if (check_launch() != HA_OK) return HA_ERR_LAUNCH;
  long long host[kProbeCount * 2];
  if (hipMemcpyAsync(host, out, sizeof(host), hipMemcpyDeviceToHost, st) != hipSuccess) return HA_ERR_LAUNCH;
  if (hipStreamSynchronize(st) != hipSuccess) return HA_ERR_LAUNCH;
  // cycles per loop trip of the first wave of each half of the workgroup
  for (int i = 0; i < kProbeCount * 2; ++i) cycles_host[i] = (float)((double)host[i] / kProbeIters);
  return HA_OK;
}
