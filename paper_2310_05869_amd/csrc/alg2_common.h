// Arguments of the Algorithm 2 / Lemma 2 option kernels and their launcher.
#pragma once

#include "ha_common.h"

namespace ha {

constexpr int kAlg2TauSplits = 8;  // key ranges the tau rows' sums are split over, for enough workgroups

struct Alg2Args {
  const void* Q;
  const void* K;
  const void* V;
  void* out;
  float* lse;
  Geometry g;
  const int32_t* perm_q;   // [BH][n]
  const int32_t* perm_k;
  const int32_t* pos_k;
  const int32_t* samples;  // [m]
  const int32_t* samp_blk; // [BH][m]
  int32_t* pos_q;          // [BH][n]
  int32_t* tau_rows;       // [m]
  float* log_unm_t;        // [BH][m]
  float* log_unm_parts;    // [kAlg2TauSplits][BH][m]: the same over ranges of keys (matrix-core form)
  int32_t tau_splits;      // 0: log_unm_t is final; else the number of key ranges to combine
  float* log_tau;          // [BH]
  double* vw;              // [BH][n] squared norms of the value rows
  double* vprefix;         // [BH][n] their inclusive prefix sums
  int32_t* vsamp;          // [BH][m]
  float* vlogw;            // [BH][m]
  uint64_t seed;
  float cap_scale, kappa;
  int32_t vnorm;
};

int launch_alg2(const Alg2Args& a, hipStream_t st);

// bf16 matrix-core forms of the two heavy steps (alg2_mfma.hip); the fp32 FMA kernels take what they do not
bool alg2_mfma_supported(const Alg2Args& a);
int launch_alg2_tau_mfma(const Alg2Args& a, hipStream_t st);
int launch_alg2_main_mfma(const Alg2Args& a, hipStream_t st);

}  // namespace ha
