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
  // Node passes (one launch per level, in level order) accumulate fp32 rows [BH][n][d], natural row
  // order: out1 = dQ (dQ pass) or dK (dK/dV passes), out2 = dV.  The first level that holds a row on
  // the pass's side writes it, later levels add to it.  The sampled-key pass writes its own rows
  // (per level, head, node, query chunk, sample) into out1 / out2 instead.
  float* out1;
  float* out2;
  int32_t wg_base;     // node passes: first workgroup of the launch's level in the all-level numbering
  // exact passes write the final gradients (tensors' dtype): fin1 = dQ or dK, fin2 = dV, after adding
  // the accumulated node rows lvl1 / lvl2 (null: none) where some level holds the row on that side
  void* fin1;
  void* fin2;
  const float* lvl1;
  const float* lvl2;
  // sampled-key pass: first workgroup and first output row of every level
  int32_t samp_wg_off[kBwdMaxLevels + 1];
  int64_t samp_row_off[kBwdMaxLevels];
};

// Whether row i of a head lies, at some level l in [0, upto), on the given side of its level-l node of
// Algorithm 4 (query side: second half; key side: first half): whether a node pass before level `upto`
// has a contribution for it.  Unmasked problems have one node that holds every row on both sides.
__host__ __device__ inline bool node_levels_hold(const Geometry& g, int i, bool query_side, int upto) {
  if (!g.causal) return upto > 0;
  for (int l = 0; l < upto; ++l) {
    const bool second = ((i / (g.n >> (l + 1))) & 1) != 0;
    if (second == query_side) return true;
  }
  return false;
}

// Chunks of sorted query positions per node at a level, for the sampled-key pass.
__host__ __device__ inline int bwd_chunks_per_node(const Geometry& g, int level) {
  const int s = g.causal ? (g.n >> (level + 1)) : g.n;
  const int clen = s < kBwdChunk ? s : kBwdChunk;
  return (s + clen - 1) / clen;
}

// workgroups of a launch (128 R rows each), the same for both kernels; node passes: of one level
int64_t bwd_grid(const BwdArgs& a, int mode);
int launch_attn_bwd_mfma(const BwdArgs& a, int mode, hipStream_t st);     // bf16 tensors
int launch_attn_bwd_generic(const BwdArgs& a, int mode, hipStream_t st);  // fp32 tensors
// delta_i = <dO_i, O_i>; bf16 tensors: O from its unrounded fp32 copy when O_f32 is non-null, else from the tensor
int launch_bwd_delta(const void* O, const float* O_f32, const void* dO, float* delta, int64_t rows, int d, int dtype,
                     hipStream_t st);
// adds the sampled keys' sums of one level into the accumulated key rows acc_k / acc_v [BH][n][d]
int launch_bwd_sample_scatter(const BwdArgs& a, int level, const float* samp_k, const float* samp_v, float* acc_k,
                              float* acc_v, hipStream_t st);
// dst (the tensors' dtype, g.dtype) = acc, row by row (unmasked problems: the one node's rows are the result)
int launch_bwd_convert(const float* acc, void* dst, const Geometry& g, hipStream_t st);

}  // namespace ha
