// Arguments of the Algorithm 2 / Lemma 2 option kernels and their launcher.
#pragma once

#include "ha_common.h"

namespace ha {

constexpr int kAlg2TauSplits = 8;  // key ranges the tau rows' sums are split over, for enough workgroups

// One launch sequence handles one LEVEL of the problem as a batch of independent unmasked
// nodes: the unmasked problem is one level of one node per head; level l of a causal problem
// (Algorithm 4) has 2^l nodes per head, node j with queries [(2j+1)s, (2j+2)s) and keys
// [2js, (2j+1)s) of its head, s = n >> (l+1).  `g` describes that batch: g.BH = heads x nodes
// per head, g.n = s rows per node; the arrays marked [view] are laid out [g.BH][g.n] (or
// [g.BH][m]) for the level being processed.
struct Alg2Args {
  const void* Q;           // whole tensors [heads][n_full][d]
  const void* K;
  const void* V;
  void* out;               // [view][d]: the final output (unmasked) or the level's partial outputs
  float* lse;              // [view]: log d~
  Geometry g;
  int32_t n_full;          // rows per head of Q, K, V
  int32_t nodes;           // nodes per head at this level (1 for the unmasked problem)
  int32_t level;
  int32_t causal;          // node j's rows start at (2j+1)s / 2js instead of 0
  int32_t heads;           // real heads (B*H)
  int32_t total_nodes;     // nodes per head over all levels
  const int32_t* perm_q;   // [view] rows (within the head) in sorted order
  const int32_t* perm_k;
  const int32_t* pos_k;    // [view] sorted position (within the node) of each key
  const int32_t* samples;  // [total_nodes][m] node-local key indices
  const int32_t* samp_blk; // [heads][total_nodes][m]
  int32_t* pos_q;          // [view]
  int32_t* tau_rows;       // [total_nodes][m] node-local query indices
  float* log_unm_t;        // [view heads][m]
  float* log_unm_parts;    // [kAlg2TauSplits][view heads][m]: the same over ranges of keys (matrix-core form)
  int32_t tau_splits;      // 0: log_unm_t is final; else the number of key ranges to combine
  float* log_tau;          // [heads][total_nodes]
  double* vw;              // [view] squared norms of the value rows
  double* vprefix;         // [view] their inclusive prefix sums
  int32_t* vsamp;          // [heads][total_nodes][m] node-local key indices
  float* vlogw;            // [heads][total_nodes][m]
  uint64_t seed;
  float cap_scale, kappa;
  int32_t vnorm;
};

// Where view head `vh` of a level sits: its real head, node, heap index and first query / key row.
struct Alg2Node {
  int32_t head, node, heap, q_start, k_start;
};
__host__ __device__ inline Alg2Node alg2_node(const Alg2Args& a, int vh) {
  Alg2Node x;
  x.head = vh / a.nodes;
  x.node = vh % a.nodes;
  x.heap = (1 << a.level) - 1 + x.node;
  x.q_start = a.causal ? (2 * x.node + 1) * a.g.n : 0;
  x.k_start = a.causal ? (2 * x.node) * a.g.n : 0;
  return x;
}

int launch_alg2(const Alg2Args& a, hipStream_t st);

// bf16 matrix-core forms of the two heavy steps (alg2_mfma.hip); the fp32 FMA kernels take what they do not
bool alg2_mfma_supported(const Alg2Args& a);
int launch_alg2_tau_mfma(const Alg2Args& a, hipStream_t st);
int launch_alg2_main_mfma(const Alg2Args& a, hipStream_t st);

}  // namespace ha
