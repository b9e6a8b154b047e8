/*
 * hyperattn.h - C ABI of the MI355X (gfx950) HyperAttention forward library.
 *
 * HyperAttention (arXiv 2310.05869) approximates softmax attention
 * Att = D^-1 A V, A = exp(Q K^T) (Section 1.1; no 1/sqrt(d) factor: fold any
 * scale into Q or K) in near-linear time:
 *   1. sortLSH (Definition 1, Algorithm 1): every row of Q and K is hashed by r
 *      random hyperplanes; the sign word's position in the reflected Gray code is
 *      the bucket; a stable sort by bucket gives permutations P_Q, P_K and the
 *      mask M^H = 1{floor(P_Q(i)/b) == floor(P_K(j)/b)}: the b x b diagonal
 *      blocks of the sorted attention matrix, which are computed exactly;
 *   2. the rest of each row is estimated from m key indices drawn uniformly
 *      with replacement, one set shared by all rows and reused for the value
 *      product (Algorithm 2 without its caps, as in the Implementation Detail
 *      paragraph of Section 4): weight (#keys/m), samples that fall in the row's
 *      own block contribute nothing;
 *   3. both parts share one normaliser: row sum = block part + estimate;
 *   4. causal masking (Section 3.1, Algorithm 4): recursive halving; the
 *      off-diagonal block (Q_2, K_1, V_1) of every split is an unmasked problem
 *      handled by 1-3, diagonal blocks of n_min rows are exact causal
 *      attention, and a row's partial results are combined by their row sums.
 *
 * Conventions for every entry point
 *   - Tensors are contiguous [B, H, n, d] in DEVICE memory, caller-owned, of the
 *     dtype in ha_shape (HA_BF16: 16-bit bfloat; HA_FP32: IEEE float).  `lse` is
 *     float [B, H, n], natural log of the (estimated) row sum.  Tensors start at a
 *     16-byte boundary, float and index arrays at a 4-byte one (HA_ERR_ALIGN).
 *   - The library allocates no device memory, never synchronises and enqueues
 *     only on `stream` (a hipStream_t passed as void*; NULL = the null stream).
 *     Scratch comes from the caller: `workspace` of at least
 *     ha_workspace_bytes() bytes, 256-byte aligned, device memory.  Two calls may
 *     overlap only if they use different workspaces.
 *   - Inputs are not modified; outputs must not alias inputs.
 *   - Return value: HA_OK (0) or a negative ha_status; nothing aborts.  Argument
 *     errors are detected on the host before anything is enqueued.
 *   - Same inputs, parameters and seed give bit-identical outputs (no floating
 *     point atomics anywhere).
 *   - Pointers named *_host are host memory, everything else is device memory.
 */
#ifndef HYPERATTN_H
#define HYPERATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { HA_BF16 = 0, HA_FP32 = 1 } ha_dtype;

typedef enum {
  HA_OK = 0,
  HA_ERR_NULL = -1,      /* a required pointer is NULL */
  HA_ERR_DTYPE = -2,     /* dtype is neither HA_BF16 nor HA_FP32 */
  HA_ERR_SHAPE = -3,     /* shape or parameters outside what is supported (see each call) */
  HA_ERR_WORKSPACE = -4, /* workspace too small or not 256-byte aligned */
  HA_ERR_LAUNCH = -5,    /* the HIP runtime refused a launch (hipGetLastError) */
  HA_ERR_ALIGN = -6,     /* a tensor does not start at a 16-byte boundary, or a float / index array at a 4-byte one */
  HA_ERR_STATIC_LIMIT = -7 /* hyperattn_forward_static: the problem needs more than ha_static_scratch_bytes() of scratch */
} ha_status;

/* [B, H, n, d]; d must be 64 or 128; n <= 2^22; B*H <= 2^20. */
typedef struct {
  int32_t B, H, n, d;
  int32_t dtype; /* ha_dtype */
} ha_shape;

/* b: block size of the sorted diagonal blocks; m: sampled key columns per node
 * (0 = block part only); r: LSH hyperplanes, 1..8; causal: 0/1; n_min: causal
 * recursion stops (exact causal attention) at n <= n_min; seed: selects the
 * hyperplanes and the sample indices. */
typedef struct {
  int32_t b, m, r, causal, n_min;
  uint64_t seed;
} ha_params;

/* Byte offsets of the regions of the workspace, for inspection after a forward
 * call (stage-by-stage parity checks).  `levels` is 1 for the unmasked problem
 * and log2(n / n_min) for the causal one (0 if n <= n_min); n_cov is the number
 * of query (= key) rows all nodes of one level cover per head: n (unmasked) or
 * n/2 (causal).  Node j of level l has s = n_cov >> l rows (causal) and owns
 * entries [j*s, (j+1)*s) of its level's arrays.
 *   codes_q, codes_k  uint8  [B*H][n]                 bucket index of each row
 *   perm_q, perm_k    int32  [levels][B*H][n_cov]     row (index within the head) at each sorted position
 *   pos_k             int32  [levels][B*H][n_cov]     sorted position (within the node) of each key
 *   samples           int32  [total_nodes][m]         l_1..l_m of each node, heap order (level l node j -> 2^l - 1 + j)
 *   samp_blk          int32  [B*H][total_nodes][m]    floor(pos_k[l_j] / b): the sorted block each sampled key falls in
 *   proj              float  [d][r]                   hyperplane matrix R
 *   sort_hist         uint32 [chunks][256]            scratch of the sort: bucket counts per 4096-key chunk
 *   part_o            dtype  [levels][B*H][n_cov][d]   causal only: per-level partial outputs (normalised), in the tensors' dtype
 *   part_l            float  [levels][B*H][n_cov]      causal only: log of the per-level partial row sums
 */
typedef struct {
  int32_t levels, total_nodes;
  int64_t n_cov;
  size_t codes_q, codes_k, perm_q, perm_k, pos_k, samples, samp_blk, proj, sort_hist, part_o, part_l;
  size_t total_bytes;
} ha_ws_layout;

/* Host only.  Validates shape/params as hyperattn_forward does and fills
 * *layout.  Returns HA_OK or the error hyperattn_forward would return. */
int ha_workspace_layout(const ha_shape* shape, const ha_params* params, ha_ws_layout* layout);

/* Host only.  Bytes of workspace hyperattn_forward needs; 0 if shape/params are invalid. */
size_t ha_workspace_bytes(const ha_shape* shape, const ha_params* params);

/* HyperAttention forward (Algorithm 3 in its Section 4 form; Algorithm 4 when
 * params->causal).  out: [B,H,n,d] of shape->dtype; lse: float [B,H,n].
 * HA_ERR_SHAPE unless: d in {64,128}; 1 <= r <= 8; b >= 1; 0 <= m <= 4096;
 * b <= 4096; B*H <= 2^20, n <= 2^22 and B*H*n <= 2^30; unmasked: n % b == 0; causal: n_min >= 1 and either n <= n_min
 * (plain exact causal attention) or n / n_min is a power of two with
 * n_min % b == 0.  The hyperplanes and sample indices are those
 * ha_make_projection / ha_make_samples return for params->seed. */
int hyperattn_forward(const void* Q, const void* K, const void* V, void* out, float* lse,
                      const ha_shape* shape, const ha_params* params,
                      void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): hyperattn_forward with the workspace taken from an array built
 * into the library (device memory of the code object, ha_static_scratch_bytes()
 * = 32 MiB per GPU, held until the process ends).  Same kernels, same results,
 * bit for bit, as hyperattn_forward.  The call allocates and frees nothing; the
 * array's device address is looked up once per device on the first call there.
 * Problems whose ha_workspace_bytes() exceeds the array return
 * HA_ERR_STATIC_LIMIT before anything is enqueued.  All calls on one GPU share
 * the one array: calls that overlap in time on one GPU (different streams or
 * host threads) race and must be serialised by the caller.  Nothing is kept in
 * the array between calls. */
int hyperattn_forward_static(const void* Q, const void* K, const void* V, void* out, float* lse,
                             const ha_shape* shape, const ha_params* params, void* stream);

/* Host only.  Size in bytes of the built-in array hyperattn_forward_static uses. */
size_t ha_static_scratch_bytes(void);

/* Same, with the random draws supplied by the caller: R_dev is float [d][r]
 * (NULL = derive from the seed); samples_dev is int32 [total_nodes][m] in heap
 * order, node-local key indices in [0, s) (NULL = derive from the seed).  Both
 * are device memory and are copied into the workspace on `stream`.  The call
 * never reads device memory on the host, so it cannot reject an index outside
 * [0, s): such an index is clamped into the node by the copying kernel (no
 * access outside the node's keys can result); validate on the host beforehand
 * if the indices come from elsewhere (the Python binding does). */
int hyperattn_forward_ex(const void* Q, const void* K, const void* V, void* out, float* lse,
                         const ha_shape* shape, const ha_params* params,
                         const float* R_dev, const int32_t* samples_dev,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Measurement variant of hyperattn_forward (same computation, same launches):
 * HIP events are recorded on `stream` between the stages, the call WAITS for the
 * last one, and stage_ms_host[0..5] (host memory) receive the elapsed
 * milliseconds of: [0] random draws into the workspace, [1] sortLSH hashing of Q
 * and K, [2] the sort (Algorithm 1's permutations), [3] block + sampled
 * attention of all nodes, [4] the exact causal base case with the Algorithm 4
 * merge (0 when not causal), [5] the whole call.  Unlike every other entry
 * point this one synchronises with the stream. */
int hyperattn_forward_timed(const void* Q, const void* K, const void* V, void* out, float* lse,
                            const ha_shape* shape, const ha_params* params,
                            void* workspace, size_t workspace_bytes, void* stream,
                            float* stage_ms_host);

/* Measurement variant of hyperattn_forward for bf16 tensors (same computation and
 * results; HA_ERR_DTYPE otherwise): the two attention launches of the forward pass
 * (all nodes of Section 4.1 / Algorithm 4; the causal base case) run an instrumented
 * instantiation of the same kernel, in which every workgroup also writes HA_STAMP_WORDS
 * 64-bit words into device memory, indexed by its tile number:
 *   [0] shader-clock reading at entry, [1] once its key list (block keys + kept
 *   samples) is built, [2] before the loop over key tiles (rows gathered, first
 *   score tile done), [3] after the loop, [4] at the end (results stored);
 *   [5], [6] the constant-rate counter (100 MHz) at entry and at the end;
 *   [7] bits 0-15 the number of 64-key tiles of the workgroup; bits 16-47 the hardware id
 *   register of its first wave (bits 8-11 of that value: CU, 13-15: shader engine);
 *   bits 48-51 the number of its XCD.
 * ha_forward_workgroups gives the number of records of either launch (0 for a launch
 * the problem does not have, and for fp32 tensors); node_stamps_dev / base_stamps_dev
 * are device memory of at least that many records (sizes in bytes, checked:
 * HA_ERR_WORKSPACE), 8-byte aligned, owned by the caller, and may be NULL where the
 * count is 0.  Asynchronous on `stream` like hyperattn_forward. */
#define HA_STAMP_WORDS 8
int ha_forward_workgroups(const ha_shape* shape, const ha_params* params, int64_t* node_wgs, int64_t* base_wgs);
int hyperattn_forward_stamped(const void* Q, const void* K, const void* V, void* out, float* lse,
                              const ha_shape* shape, const ha_params* params,
                              void* workspace, size_t workspace_bytes, void* stream,
                              int64_t* node_stamps_dev, size_t node_stamps_bytes,
                              int64_t* base_stamps_dev, size_t base_stamps_bytes);

/* Plain exact attention D^-1 A V (Section 1.1), or D_C^-1 (M^C . A) V with
 * M^C_ij = 1{i >= j} (Section 3.1) when causal != 0; the denominator of the
 * speed-up ratio.  Any n >= 1; d in {64,128}.  Needs no workspace. */
int exact_attn_forward(const void* Q, const void* K, const void* V, void* out, float* lse,
                       const ha_shape* shape, int causal, void* stream);

/* Host only.  The r hyperplane normals used for `seed` (Definition 1 read as
 * sign-of-Gaussian-projection LSH): R_host[c*r + k], c < d, k < r, i.i.d. N(0,1)
 * rounded to bf16-representable floats.  Entry (c,k) depends on (seed,c,k) only. */
int ha_make_projection(uint64_t seed, int32_t d, int32_t r, float* R_host);

/* Host only.  The m key indices, i.i.d. uniform on [0, n_keys) with
 * replacement (Algorithm 2), that node `node` of recursion level `level` uses
 * (level 0, node 0 for the unmasked problem); shared by all batches and heads. */
int ha_make_samples(uint64_t seed, int32_t level, int32_t node, int32_t n_keys, int32_t m,
                    int32_t* idx_host);

/* ---- single stages, for stage-by-stage parity and profiling ---------------- */

/* sortLSH hashing (Definition 1; Algorithm 1 "hash rows of Q, K"): codes[i] =
 * Gray-sequence position of the sign word of X[i,:] R.  X: [rows][d] of dtype,
 * R_dev: float [d][r], codes: uint8 [rows].  The codes equal those of an fp64
 * evaluation of the projections: bf16 rows are projected on the matrix cores in
 * fp32 together with a bound on the accumulation error, and every row with a
 * projection inside that bound is recomputed in fp64 (exact products); fp32 rows
 * are accumulated in fp64 throughout. */
int ha_lsh_hash(const void* X, uint8_t* codes, int64_t rows, int32_t d, int32_t dtype,
                const float* R_dev, int32_t r, void* stream);

/* Algorithm 1's permutation: n_seg independent segments of seg_len consecutive
 * codes each; stable ascending sort.  perm[g*seg_len + p] = index (within the
 * segment) of the row at sorted position p; pos = inverse.  seg_len <= 2^24. */
int ha_seg_sort(const uint8_t* codes, int32_t* perm, int32_t* pos, int32_t n_seg,
                int32_t seg_len, void* stream);

/* Row permutation ("permuting n rows", Section 4): dst[g][p][:] = src[g][idx[g*n + p]][:]
 * for g < groups, p < n; rows of d elements of dtype. */
int ha_gather_rows(const void* src, const int32_t* idx, void* dst, int32_t groups, int32_t n,
                   int32_t d, int32_t dtype, void* stream);

/* Block-diagonal part alone on inputs ALREADY in sorted order (Section 4,
 * Implementation Detail: i-th group of b sorted queries against the i-th group
 * of b sorted keys).  Qs,Ks,Vs: [groups][n][d]; o_b float [groups][n][d] and
 * lse_b float [groups][n], both in sorted order. */
int ha_block_attn(const void* Qs, const void* Ks, const void* Vs, float* o_b, float* lse_b,
                  int32_t groups, int32_t n, int32_t d, int32_t dtype, int32_t b, void* stream);

/* Sampled residual part alone (Algorithm 2's estimator with shared indices):
 * Qs in sorted order [groups][n][d]; K, V in ORIGINAL order [groups][n][d];
 * samples int32 [m] (original key indices), pos_k int32 [groups][n].  Sample j
 * is skipped for the rows of block floor(pos_k[l_j]/b).  o_r float
 * [groups][n][d], lse_r float [groups][n] (includes log(n/m); -inf and zero
 * row where nothing is kept), sorted order. */
int ha_sampled_attn(const void* Qs, const void* K, const void* V, const int32_t* samples,
                    const int32_t* pos_k, float* o_r, float* lse_r, int32_t groups, int32_t n,
                    int32_t d, int32_t dtype, int32_t b, int32_t m, void* stream);

/* Shared normaliser and inverse permutation: L = log(exp lse_b + exp lse_r),
 * out[g][perm_q[g*n+p]] = exp(lse_b-L) o_b[g][p] + exp(lse_r-L) o_r[g][p],
 * lse[g][perm_q[..]] = L.  out is of dtype. */
int ha_merge_unpermute(const float* o_b, const float* lse_b, const float* o_r, const float* lse_r,
                       const int32_t* perm_q, void* out, float* lse, int32_t groups, int32_t n,
                       int32_t d, int32_t dtype, void* stream);

/* ------------------------------------------------------------------------
 * Backward pass (Section 4.2 times forward + backward; the backward is the
 * derivative of the forward above with the random draws, and so the
 * permutations, held fixed).  bf16 tensors run on the matrix cores; fp32 tensors
 * take the same passes in fp32 FMA arithmetic.
 *
 * Because every output row is one softmax over the union of its parts (block
 * keys, kept samples weighted s/m, base-case keys; Algorithms 1, 2, 4), with
 * L = lse and delta_i = <d_out_i, out_i>:
 *   P_ij = w_ij exp(<q_i,k_j> - L_i),  dV_j = sum_i P_ij d_out_i,
 *   dS_ij = P_ij (<d_out_i, v_j> - delta_i),  dQ_i = sum_j dS_ij k_j,  dK_j = sum_i dS_ij q_i.
 *
 * hyperattn_forward_train: hyperattn_forward that also writes out_f32 (device
 * fp32 [B][H][n][d]; NULL: none), the output before its rounding to bf16.  The
 * backward forms delta from it: with the bf16 tensor alone delta carries the
 * output's rounding error (2^-9 relative), which dominates dQ and dK on rows
 * whose weight sits on few keys, where <d_out_i, v_j> - delta_i cancels.
 * exact_attn_forward_train: the same for exact attention.
 *
 * hyperattn_backward: Q, K, V, out, d_out, dQ, dK, dV are device pointers to
 * contiguous [B][H][n][d] of shape->dtype; lse device fp32 [B][H][n]; out_f32 as written
 * by hyperattn_forward_train, or NULL (delta then comes from out; fp32 tensors:
 * must be NULL, HA_ERR_DTYPE otherwise).  out and lse are the
 * results of hyperattn_forward on the same Q, K, V, shape and params, and
 * fwd_workspace is that call's workspace, unmodified since (it holds the sort
 * permutations and sample indices; only read here).  bwd_workspace: device,
 * 256-byte aligned, >= ha_backward_workspace_bytes(); overwritten.  All
 * caller-owned; nothing is allocated; kernels are enqueued on `stream` and the
 * call returns without waiting.  Sums over parts are taken in a fixed order
 * (the node parts level by level into one accumulated fp32 row per tensor row):
 * same inputs give bit-identical gradients.
 * Errors: HA_ERR_NULL, HA_ERR_DTYPE, HA_ERR_SHAPE (as hyperattn_forward; more
 * than 24 recursion levels), HA_ERR_WORKSPACE, HA_ERR_LAUNCH.
 *
 * hyperattn_backward_timed: the same, and WAITS for the stream; stage_ms_host
 * (host, 8 floats) receives the times between events on the stream: delta, dQ
 * of the nodes, dQ of the base case (unmasked problems: conversion of the one
 * node's rows), dK/dV of the block keys, dK/dV of the sampled keys with their
 * reduction, dK/dV of the base case, conversion of dK and dV (unmasked problems
 * only; the causal base-case passes write the final tensors themselves), total.
 *
 * exact_attn_backward: gradients of exact_attn_forward (Section 1.1; causal:
 * Section 3.1), the denominator of the forward + backward speed-up.  workspace
 * >= exact_attn_backward_workspace_bytes(shape). */
typedef struct {
  size_t delta;                      /* fp32 [B*H][n] */
  size_t acc_a, acc_b;               /* fp32 [B*H][n][d] each: the node parts' rows, added up level by level
                                        (acc_a: dQ, afterwards dK; acc_b: dV) */
  size_t samp_k, samp_v;             /* fp32 rows of the sampled keys per (level, head, node, query chunk, sample) */
  size_t total_bytes;
} ha_bwd_ws_layout;

int ha_backward_workspace_layout(const ha_shape* shape, const ha_params* params, ha_bwd_ws_layout* layout);
size_t ha_backward_workspace_bytes(const ha_shape* shape, const ha_params* params);
int hyperattn_forward_train(const void* Q, const void* K, const void* V, void* out, float* lse, float* out_f32,
                            const ha_shape* shape, const ha_params* params, void* workspace,
                            size_t workspace_bytes, void* stream);
int exact_attn_forward_train(const void* Q, const void* K, const void* V, void* out, float* lse, float* out_f32,
                             const ha_shape* shape, int causal, void* stream);
int hyperattn_backward(const void* Q, const void* K, const void* V, const void* out, const float* out_f32,
                       const float* lse, const void* d_out, void* dQ, void* dK, void* dV, const ha_shape* shape,
                       const ha_params* params, const void* fwd_workspace, size_t fwd_workspace_bytes,
                       void* bwd_workspace, size_t bwd_workspace_bytes, void* stream);
int hyperattn_backward_timed(const void* Q, const void* K, const void* V, const void* out, const float* out_f32,
                             const float* lse, const void* d_out, void* dQ, void* dK, void* dV, const ha_shape* shape,
                             const ha_params* params, const void* fwd_workspace, size_t fwd_workspace_bytes,
                             void* bwd_workspace, size_t bwd_workspace_bytes, void* stream, float* stage_ms_host);
int exact_attn_backward(const void* Q, const void* K, const void* V, const void* out, const float* out_f32,
                        const float* lse, const void* d_out, void* dQ, void* dK, void* dV, const ha_shape* shape, int causal,
                        void* workspace, size_t workspace_bytes, void* stream);
size_t exact_attn_backward_workspace_bytes(const ha_shape* shape);

/* ------------------------------------------------------------------------
 * Algorithm 2 as printed and Lemma 2 / Algorithm 3, as options (the Section 4
 * form above leaves them out); both dtypes (bf16 tensors on the matrix cores,
 * weights rounded to bf16 as operands like in the forward; fp32 tensors in
 * plain fp32 arithmetic).  Causal problems run them at every off-diagonal node of
 * Algorithm 4 ("the unmasked algorithm on Q_2, K_1"): below, n is then the
 * node's size s, every node has its own subset T, index set and value rows
 * (counters offset by the node's heap index 2^level - 1 + node), the diagonal
 * blocks are exact and the results are added up as in hyperattn_forward.
 *   tau   = max over m rows drawn uniformly (with replacement) of the unmasked row sum
 *   C_i   = cap_scale * m / (n ln n) * (masked row sum_i + tau / kappa)     cap_scale <= 0: no cap
 *   d_i   = (n/m) sum_j (1 - M_{i,l_j}) min(exp<q_i,k_{l_j}>, C_i)
 *   d~_i  = masked row sum_i + max(d_i, tau / kappa)                         kappa <= 0: no lower cap
 *   out_i = (1/d~_i) sum_r exp<q_i,k_{l'_r}> v_{l'_r} / (m p_{l'_r}),  l'_r drawn with p_l ~ |V_l|^2   (vnorm_sampling)
 *        or (1/d~_i) (masked part + (n/m) sum_j (1 - M_{i,l_j}) exp<q_i,k_{l_j}> v_{l_j})             (otherwise)
 * lse receives log d~.  The constants the paper leaves open (the Theta of C_i,
 * kappa) are the caller's.  Lemma 2's rows are drawn with p_l = |V_l|^2 / |V|_F^2
 * by inverting the cumulative distribution in fp64 (draw r of head bh: first l
 * whose inclusive prefix sum of squared norms exceeds u |V|_F^2, u in (0,1) from
 * the top 53 bits of counter (heap * B*H + bh) * m + r of stream 2; T uses counter
 * heap * m + j of stream 0).
 * workspace: device, 256-byte aligned, >= ha_alg2_workspace_bytes(); it starts
 * with the forward's layout (ha_workspace_layout) followed by the regions below
 * ("per level": sized for the largest level and reused from level to level, so
 * after the call they hold the last, deepest level; "per node": every node of
 * every level, nodes in heap order).  Errors as hyperattn_forward. */
typedef struct {
  float cap_scale;
  float kappa;
  int32_t vnorm_sampling;
} ha_alg2_options;

typedef struct {
  size_t forward_bytes;      /* the forward's regions come first */
  size_t pos_q;              /* per level, int32 [B*H][n_cov]: inverse of perm_q within the node */
  size_t tau_rows;           /* per node, int32 [total_nodes][m]: the rows of T (node-local) */
  size_t log_unmasked_t;     /* per level, float [B*H * nodes][m]: log of their unmasked row sums */
  size_t log_tau;            /* per node, float [B*H][total_nodes] */
  size_t vnorm_w;            /* per level, double [B*H][n_cov]: |V_l|^2 of the nodes' value rows */
  size_t vnorm_prefix;       /* per level, double [B*H][n_cov]: inclusive prefix sums within the node */
  size_t vnorm_samples;      /* per node, int32 [B*H][total_nodes][m]: l'_r (node-local) */
  size_t vnorm_logw;         /* per node, float [B*H][total_nodes][m]: log(1 / (m p_{l'_r})) */
  size_t log_unmasked_parts; /* per level, float [8][B*H * nodes][m]: scratch, the unmasked row sums of T over eight ranges of keys */
  size_t total_bytes;
} ha_alg2_ws_layout;

int ha_alg2_workspace_layout(const ha_shape* shape, const ha_params* params, ha_alg2_ws_layout* layout);
size_t ha_alg2_workspace_bytes(const ha_shape* shape, const ha_params* params);
int hyperattn_forward_alg2(const void* Q, const void* K, const void* V, void* out, float* lse,
                           const ha_shape* shape, const ha_params* params, const ha_alg2_options* options,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Measurement aids (no passage of the paper: they serve the roofline report).
 * Both run on `stream`, time themselves with events and WAIT for the stream;
 * `buf` is caller-owned device memory that they overwrite.
 *
 * ha_measure_mfma_rate: bf16 matrix-core rate of register-resident chains of the
 * 32x32x16 MFMA the attention kernels use, over operands that change from one
 * instruction to the next, `iters` loop trips per wave (1..2^20; 1000 take about
 * 1.2 ms, and the rate falls with the duration as the chip lowers its clock), in
 * TFLOP/s.  buf >= 512 KiB.
 * ha_measure_hbm_rate: GB/s of a streaming read of the first half of buf, and of
 * a copy of the first half onto the second (read + written bytes counted).
 * buf 16-byte aligned, bytes >= 1 MiB; use a buffer well beyond the caches.
 * Errors: HA_ERR_NULL, HA_ERR_WORKSPACE (buf too small / misaligned),
 * HA_ERR_SHAPE (iters), HA_ERR_LAUNCH. */
int ha_measure_mfma_rate(void* buf, size_t bytes, int32_t iters, float* tflops, void* stream);
int ha_measure_hbm_rate(void* buf, size_t bytes, float* read_gbs, float* copy_gbs, void* stream);

/* Issue-rate probes (measurement aid): what one trip of small instruction loops costs in
 * shader-clock cycles on this GPU, every CU running the same loop in one workgroup of eight
 * waves (two per SIMD).  cycles_host (host memory) receives 2 * ha_issue_probe_count() floats:
 * for probe p, [2p] is the first wave of the workgroup's first half, [2p+1] of its second half.
 * A trip holds, in this order of p: 64 v_exp_f32; 64 v_fma_f32; 64 v_cvt_pk_bf16_f32; 64
 * v_max3_f32; 16 v_mfma_f32_32x32x16_bf16; 16 MFMAs with 4 fma each; with 7 fma each; with 1 exp
 * + 3 fma each; with 1 exp + 4 fma each; waves 0-3 16 MFMAs while waves 4-7 issue 16 exp + 48 fma;
 * 8 ds_read_b128 per wave (64 KiB read per trip and workgroup); 8 ds_read_b64_tr_b16 (32 KiB);
 * 8 ds_write_b128 (64 KiB).  buf: device memory, 16-byte aligned, >= 1 MiB, overwritten.
 * WAITS for the stream.  Errors: HA_ERR_NULL, HA_ERR_WORKSPACE, HA_ERR_LAUNCH. */
int32_t ha_issue_probe_count(void);
int ha_measure_issue_rates(void* buf, size_t bytes, float* cycles_host, void* stream);

/* Text for an ha_status value. */
const char* ha_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* HYPERATTN_H */
