// Declarations shared by the backward-pass kernels and their host driver.
#pragma once

#include "ha_common.h"

namespace ha {

// Passes of the MFMA backward kernel.
enum BwdMode : int32_t {
  kBwdDqNode = 0,    // dQ of the node parts: query tiles over their key lists (block keys + kept samples)
  kBwdDqExact = 1,   // dQ of exact attention / the causal base case
  kBwdDkvBlock = 2,  // dK, dV of the block keys of every node: key tiles over the queries of their block
  kBwdDkvSamp = 3,   // dK, dV of the sampled keys of every node: sample slabs over chunks of the node's queries
  kBwdDkvExact = 4,  // dK, dV of exact attention / the causal base case
};

constexpr int kBwdMaxLevels = 24;
constexpr int kBwdChunk = 2048;  // sorted query positions per workgroup of the sampled-key pass

struct BwdArgs {
  AttnArgs f;          // tensors, permutations, samples and geometry as in the forward
  const void* dO;      // [BH][n][d], dtype of the tensors
  const float* lse;    // final log row sums [BH][n]
  const float* delta;  // <dO_i, O_i> [BH][n]
  float* out1;         // fp32 rows: dQ (dQ passes) or dK (dK/dV passes)
  float* out2;         // fp32 rows: dV (dK/dV passes)
  // exact passes write the final gradients (tensors' dtype) instead: fin1 = dQ or dK, fin2 = dV,
  // after adding the rows of the per-level buffers lvl1 / lvl2 (null: nothing to add)
  void* fin1;
  void* fin2;
  const float* lvl1;
  const float* lvl2;
  // sampled-key pass: first workgroup and first output row of every level
  int32_t samp_wg_off[kBwdMaxLevels + 1];
  int64_t samp_row_off[kBwdMaxLevels];
};

// Chunks of sorted query positions per node at a level, for the sampled-key pass.
__host__ __device__ inline int bwd_chunks_per_node(const Geometry& g, int level) {
  const int s = g.causal ? (g.n >> (level + 1)) : g.n;
  const int clen = s < kBwdChunk ? s : kBwdChunk;
  return (s + clen - 1) / clen;
}

int64_t bwd_grid(const BwdArgs& a, int mode);  // workgroups of a pass (128 R rows each), the same for both kernels
int launch_attn_bwd_mfma(const BwdArgs& a, int mode, hipStream_t st);     // bf16 tensors
int launch_attn_bwd_generic(const BwdArgs& a, int mode, hipStream_t st);  // fp32 tensors
// delta_i = <dO_i, O_i>; bf16 tensors: O from its unrounded fp32 copy when O_f32 is non-null, else from the tensor
int launch_bwd_delta(const void* O, const float* O_f32, const void* dO, float* delta, int64_t rows, int d, int dtype,
                     hipStream_t st);
int launch_bwd_sample_scatter(const BwdArgs& a, const float* samp_k, const float* samp_v, float* part_k,
                              float* part_v, hipStream_t st);
// dst (the tensors' dtype, g.dtype) = base + sum over the levels whose node holds the row on the given side
// (query_side: second half of the node; key side: first half)
int launch_bwd_combine(const float* base, const float* part, void* dst, const Geometry& g, int query_side,
                       hipStream_t st);

}  // namespace ha
