// Shared declarations of the HIP side of the HyperAttention library (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "hyperattn.h"

namespace ha {

// ---------------------------------------------------------------------------
// Counter-based generator of the method's random draws (hyperplanes of
// Definition 1, sample indices of Algorithm 2).  SplitMix64's output function
// keyed by (seed, stream) and indexed by a counter; integer-only, so the host
// and the device produce the same indices.
// ---------------------------------------------------------------------------
__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__host__ __device__ inline uint64_t rand_u64(uint64_t seed, uint64_t stream, uint64_t ctr) {
  const uint64_t g = 0x9E3779B97F4A7C15ull;
  const uint64_t key = mix64(seed + g * (stream + 1));
  return mix64(key + g * (ctr + 1));
}
constexpr uint64_t kStreamProjection = 1;
constexpr uint64_t kStreamSamples = 2;  // + heap index (1-based) of the node

__host__ __device__ inline int32_t sample_index(uint64_t seed, int level, int node, int n_keys, int j) {
  const uint64_t stream = kStreamSamples + (1ull << level) + (uint64_t)node;
  const uint64_t hi = rand_u64(seed, stream, (uint64_t)j) >> 32;
  return (int32_t)((hi * (uint64_t)n_keys) >> 32);
}

// ---------------------------------------------------------------------------
// Geometry of one forward call, shared by host validation and kernels.
// Unmasked problem: one level, one node of s = n rows per head.
// Causal problem (Algorithm 4): level l has 2^l nodes of s = n >> (l+1) rows;
// node j takes queries [(2j+1)s, (2j+2)s) and keys [2js, (2j+1)s).
// ---------------------------------------------------------------------------
struct Geometry {
  int32_t BH, n, d, dtype;
  int32_t b, m, r, causal, n_min;
  int32_t levels;       // node levels (0 if causal and n <= n_min)
  int32_t total_nodes;  // per head
  int32_t n_cov;        // rows covered per level per head
  int32_t base_len;     // causal: rows of one exact diagonal block (n if n <= n_min)
};

struct NodeRef {
  int32_t s;        // rows (queries = keys) in the node
  int32_t q_start;  // first query row within the head
  int32_t k_start;  // first key row within the head
  int32_t heap;     // 0-based heap index: (1 << level) - 1 + node
};

__host__ __device__ inline NodeRef node_ref(const Geometry& g, int level, int node) {
  NodeRef nr;
  if (g.causal) {
    nr.s = g.n >> (level + 1);
    nr.q_start = (2 * node + 1) * nr.s;
    nr.k_start = (2 * node) * nr.s;
  } else {
    nr.s = g.n;
    nr.q_start = 0;
    nr.k_start = 0;
  }
  nr.heap = (1 << level) - 1 + node;
  return nr;
}

// ---------------------------------------------------------------------------
// Arguments of the attention kernels (MFMA and generic share them).
// ---------------------------------------------------------------------------
enum AttnMode : int32_t {
  kModeNode = 0,   // unmasked node(s): block keys by list + kept sampled keys
  kModeExact = 1,  // contiguous keys, optional causal mask (exact attention / causal base case)
};

struct AttnArgs {
  const void* Q;  // [BH][rows_q][d]
  const void* K;  // [BH][rows_k][d]
  const void* V;
  int64_t q_bh_stride, k_bh_stride;  // elements between heads
  // node mode
  const int32_t* perm_q;   // [levels][BH][n_cov] or null (sorted position == row)
  const int32_t* perm_k;   // same, or null
  const int32_t* pos_k;    // [levels][BH][n_cov]; null => pos == row
  const int32_t* samples;  // [total_nodes][m] node-local key indices; null or m == 0 => none
  const int32_t* samp_blk; // [BH][total_nodes][m] sorted block of each sampled key; null => look up pos_k
  int32_t use_block;       // 0: residual part alone
  // outputs
  void* out;        // final output in dtype (may be null)
  float* lse;       // final log row sum (may be null)
  float* out_f32;   // optional unrounded copy of the final output (bf16 tensors; may be null)
  void* part_o;     // outputs [levels][BH][n_cov][d] (node mode when non-null; merged in by the base case):
                    // bf16 if part_bf16, else fp32
  float* part_l;
  int32_t part_bf16;
  int64_t out_bh_stride;  // elements between heads of `out` ; lse stride = out_bh_stride / d
  int32_t scatter_out;    // node mode: 1 => write row perm_q[p], 0 => write sorted position p
  Geometry g;
  // exact mode
  int32_t exact_rows_q, exact_rows_k;  // rows per head (full problem)
  int32_t exact_block;                 // rows per independent diagonal block (== rows for full attention)
  int32_t exact_causal;
  int32_t merge_levels;                // exact mode: merge part_o/part_l of this many levels into the result
  // measurement only (null in every product call): kStampWords 64-bit words per workgroup, indexed by the
  // workgroup's logical tile number, written by the instrumented instantiation of the MFMA kernel
  long long* stamps;
};

// Words of a workgroup's stamp record: shader-clock readings at entry, after the key list is built,
// before the tile loop (first scores done), after the loop and at the end; the constant-rate
// counter at entry and at the end; the number of key tiles.
constexpr int kStampWords = HA_STAMP_WORDS;

// launchers (defined in the .hip files)
int launch_lsh_hash(const void* X, uint8_t* codes, int64_t rows, int d, int dtype, const float* R_dev,
                    int r, hipStream_t st);
int launch_lsh_hash_mfma(const void* X, uint8_t* codes, int64_t rows, int d, const float* R_dev, int r,
                         hipStream_t st);
int launch_seg_sort_nodes(const uint8_t* codes_q, const uint8_t* codes_k, int32_t* perm_q, int32_t* perm_k,
                          int32_t* pos_k, const int32_t* samples, int32_t* samp_blk, uint32_t* chunk_hist,
                          const Geometry& g, hipStream_t st);
int64_t seg_sort_chunks(const Geometry& g);  // rows of 256 counters the chunked sort needs
int launch_seg_sort_flat(const uint8_t* codes, int32_t* perm, int32_t* pos, int n_seg, int seg_len,
                         hipStream_t st);
int launch_prep(float* R_ws, const float* R_dev, const uint16_t* R_bf16_host, int32_t* samples_ws,
                const int32_t* samples_dev, const Geometry& g, uint64_t seed, hipStream_t st);
int launch_attn_mfma(const AttnArgs& a, int mode, hipStream_t st);
int64_t attn_mfma_grid(const AttnArgs& a, int mode);  // workgroups of the four-wave launch of that mode
int launch_attn_generic(const AttnArgs& a, int mode, hipStream_t st);
int launch_gather_rows(const void* src, const int32_t* idx, void* dst, int groups, int n, int d, int dtype,
                       hipStream_t st);
int launch_merge_unpermute(const float* o_b, const float* lse_b, const float* o_r, const float* lse_r,
                           const int32_t* perm_q, void* out, float* lse, int groups, int n, int d, int dtype,
                           hipStream_t st);

inline int check_launch() { return hipGetLastError() == hipSuccess ? HA_OK : HA_ERR_LAUNCH; }

// Lets kernel `fn` use up to 160 KiB of dynamic LDS on the current device.  The
// attribute is per device; `done` (one per kernel instantiation) remembers the
// devices already set, so concurrent callers and several devices are both fine.
inline int allow_full_lds(const void* fn, std::atomic<uint64_t>& done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return HA_ERR_LAUNCH;
  const uint64_t bit = 1ull << (dev & 63);
  if (dev < 64 && (done.load(std::memory_order_acquire) & bit)) return HA_OK;
  if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
    (void)hipGetLastError();
    return HA_ERR_LAUNCH;
  }
  if (dev < 64) done.fetch_or(bit, std::memory_order_release);
  return HA_OK;
}

}  // namespace ha
