/*
 * bastion_tv.h -- C ABI of the MI355X (gfx950) tree-verify library for budget-aware tree
 * speculative decoding: best-first tree build, tree-masked attention, acceptance walk.
 *
 * Conventions shared by every entry point
 *   - Unless a parameter says HOST, every pointer is a DEVICE pointer owned by the caller.
 *     The library allocates no caller-visible memory; scratch space is the caller's `ws`
 *     (size from the matching *_workspace() query, 256-byte aligned).  A workspace must be
 *     zero-filled once, before its first use; every call leaves it ready for the next one (the
 *     data flag aside, see btv_workspace_status).  A workspace serves one call at a time.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work; outputs are valid once the caller has synchronised the stream.
 *   - Return value: BTV_OK, or a negative btv_status.  All argument checks run on the host
 *     before anything is launched; btv_last_error() returns a thread-local message.
 *     Nothing throws, nothing aborts.
 *   - Tree encoding: M draft nodes in best-first (topological) order, parent[i] in
 *     {-1} u [0, i); -1 marks a child of the root.  The root is the last validated token
 *     and already lives in the KV prefix.  Data-dependent violations cannot be seen by the
 *     host: kernels treat an out-of-range parent as -1 (so no access leaves its buffer) and
 *     raise a flag in the workspace that btv_workspace_status() reports.
 *   - dtype: BTV_F32 or BTV_BF16 (storage type of Q, K, V, O or of the logits).
 *   - Limits: 1 <= M <= BTV_MAX_NODES, D in {64, 128}, Hq % Hkv == 0, Hq/Hkv <= 16, L >= 0,
 *     1 <= B <= BTV_MAX_DEPTH, V >= 1.
 */
#ifndef BASTION_TV_H
#define BASTION_TV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BTV_OK = 0,
    BTV_EINVAL = -1,      /* null pointer, bad shape, unsupported dtype or limit exceeded */
    BTV_EWORKSPACE = -2,  /* workspace missing, misaligned or too small */
    BTV_EHIP = -3,        /* a HIP runtime call or kernel launch failed */
    BTV_EDATA = -4        /* btv_workspace_status(): a kernel saw invalid data (e.g. parent[i] >= i) */
} btv_status;

enum { BTV_F32 = 0, BTV_BF16 = 1 };
enum { BTV_MAX_NODES = 256, BTV_MAX_DEPTH = 16, BTV_PAGE = 16, BTV_ANC_WORDS = 8 };

const char *btv_last_error(void);
int btv_version(void);

/* Synchronises `stream`, reads the data-error flag that kernels of the last call using `ws`
 * may have raised, clears it, and returns BTV_OK or BTV_EDATA.  Optional. */
int btv_workspace_status(void *ws, void *stream);

/* ---------------------------------------------------------------------------------------------
 * tree_build -- best-first expansion at a fixed budget (Sec. 3.3, Prop. 3.3; Algorithm 1's
 * frontier rule without the early stop; path score of Eq. 1; surrogate of Eq. 3).
 *
 * marginals [B,V] fp32 row-major: position-wise draft probabilities q_1..q_B (non-negative,
 * finite).  Emits the N prefixes of the candidate lattice with the largest path score
 * rho = prod_k q_k(x_k), in non-increasing order of rho; rho of a child is one fp32 multiply
 * rho(parent) * q.  Ties: shallower first, then smaller rank path, where a token's rank at a
 * position is its index in that position's list sorted by (probability desc, token id asc).
 *
 * Outputs (all [N] unless noted; entries past *n_out are left untouched):
 *   parent  -1 = child of the root, else index of the parent node (< own index)
 *   token   vocabulary id;  depth (optional, may be NULL) 1-based;  rho (optional) fp32 score
 *   n_out   [1] = min(N, number of prefixes in the lattice)
 *   ahat    [1] optional: 1 + sum of rho (the root counts 1), fp32
 * ------------------------------------------------------------------------------------------- */
size_t btv_tree_build_workspace(int B, int V, int N);
int btv_tree_build(const float *marginals, int B, int V, int N,
                   int32_t *parent, int32_t *token, int32_t *depth, float *rho,
                   int32_t *n_out, float *ahat, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * tree_build_adaptive -- Algorithm 1 with its early stop: the budget is chosen online (Sec. 3.4,
 * Eq. 6, Prop. 3.4).  Same expansion and outputs as btv_tree_build with N = N_max, but after the
 * N-th node is popped the estimated speedup  S(N) = Ahat(T_N) * L_AR / C(N)  is compared with the
 * best so far: the node is kept while S strictly improves, and the tree before the first
 * non-improvement is returned (*n_out = N*).  The first node is always kept.
 *   cost   [N_max] fp64 DEVICE: cost[N-1] = C(N) = T_draft + T_aux + T_verify(N), the estimated
 *          latency of one cycle at budget N, any unit, positive and finite (btv_verify_cost gives
 *          the T_verify term).  A non-positive or NaN entry stops the expansion there and raises
 *          the data flag (btv_workspace_status).
 *   L_AR   HOST: latency of one autoregressive target step, same unit, > 0.
 *   s_best [1] fp64 DEVICE, optional: S(N*).
 * The comparison is made in fp64 as  Ahat(N) * C(N*) > Ahat(N*) * C(N)  (no division per node).
 * Workspace: btv_tree_build_workspace(B, V, N_max).
 * ------------------------------------------------------------------------------------------- */
int btv_tree_build_adaptive(const float *marginals, int B, int V, int N_max, const double *cost,
                            double L_AR, int32_t *parent, int32_t *token, int32_t *depth, float *rho,
                            int32_t *n_out, float *ahat, double *s_best, void *ws, size_t ws_bytes,
                            void *stream);

/* tree_build with the choice of expansion made by the caller (tests, tuning): the results are
 * those of btv_tree_build (cost == NULL) or btv_tree_build_adaptive (cost != NULL, with L_AR and
 * s_best as there), whichever expansion runs.
 *   algo  0 = the library chooses from the depth the tree can reach, 1 = the one-wavefront
 *         best-first expansion (Algorithm 1's frontier loop), 2 = the level-synchronous one.
 * Workspace: btv_tree_build_workspace(B, V, N). */
int btv_tree_build_tuned(const float *marginals, int B, int V, int N, const double *cost,
                         double L_AR, int algo, int32_t *parent, int32_t *token,
                         int32_t *depth_out, float *rho, int32_t *n_out, float *ahat,
                         double *s_best, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Batches of requests in one launch (the ragged batch of the paged attention entry point, for the
 * steps before and after it).  Requests are independent; request r owns the output rows
 * q_offset[r] .. q_offset[r+1]-1 (the same array the paged attention takes).
 *
 * tree_build_batch: marginals [batch,B,V] fp32; n_nodes [batch] int32 DEVICE = budget N_r of each
 *   request, 0 <= N_r <= min(N_max, q_offset[r+1]-q_offset[r]); parent/token/depth/rho [total]
 *   written at q_offset[r] with node ids local to the request; n_out, ahat [batch].  N_max HOST:
 *   upper bound of any N_r (sizes the top lists and the workspace).  A request that violates
 *   the bounds gets n_out = 0 and raises the data flag.
 * tree_accept_greedy_batch: logits [total_M + batch, V]: request r owns rows q_offset[r]+r ..
 *   q_offset[r+1]+r, its root row first; parent/token [total_M] local ids; path [total_M] written at
 *   q_offset[r]; n_acc, bonus [batch]; argmax_out [total_M + batch] optional.  M_max HOST: upper
 *   bound of any request's node count (<= BTV_MAX_NODES); a request with no node or more than
 *   M_max gets n_acc = 0 and raises the data flag.
 * ------------------------------------------------------------------------------------------- */
size_t btv_tree_build_batch_workspace(int batch, int B, int V, int N_max);
int btv_tree_build_batch(const float *marginals, int batch, int B, int V, const int32_t *n_nodes,
                         const int32_t *q_offset, int N_max, int32_t *parent, int32_t *token,
                         int32_t *depth, float *rho, int32_t *n_out, float *ahat, void *ws,
                         size_t ws_bytes, void *stream);
size_t btv_tree_accept_batch_workspace(int batch, int total_M, int V);
int btv_tree_accept_greedy_batch(const void *logits, int dtype, const int32_t *parent,
                                 const int32_t *token, const int32_t *q_offset, int batch,
                                 int total_M, int M_max, int V, int32_t *path, int32_t *n_acc,
                                 int32_t *bonus, int32_t *argmax_out, void *ws, size_t ws_bytes,
                                 void *stream);

/* ---------------------------------------------------------------------------------------------
 * stream_read -- measurement aid, not part of the method: reads `bytes` bytes at src once with
 * all CUs (16-byte loads, nothing else), so that a benchmark can time what a plain streaming read
 * achieves on the machine it runs on and quote kernels against that beside the datasheet peak.
 *   src DEVICE, 16-byte aligned, bytes a multiple of 16; sink DEVICE, >= 16384 bytes, receives
 *   a checksum word per workgroup (xor-accumulated: its content is of no use).
 * ------------------------------------------------------------------------------------------- */
int btv_stream_read(const void *src, size_t bytes, void *sink, size_t sink_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * mfma_peak -- measurement aid, not part of the method: `workgroups` workgroups of 8 wavefronts
 * each run `iters` rounds of four independent 32x32x16 bf16 matrix-core instructions on
 * register-resident operands, so that a benchmark can time what the matrix cores sustain on the
 * machine it runs on.  *flops (HOST) receives the number of floating-point operations the launch
 * performs (2 per multiply-add); sink DEVICE, >= 16384 bytes, receives checksum words of no use.
 * ------------------------------------------------------------------------------------------- */
int btv_mfma_peak(int workgroups, int iters, void *sink, size_t sink_bytes, double *flops,
                  void *stream);

/* ---------------------------------------------------------------------------------------------
 * tree_build_beam -- the beam-search tree that Sec. 4.3 compares best-first expansion with:
 * depth by depth, of all one-token extensions of the prefixes kept at the previous depth, the
 * `width` with the largest path score (Eq. 1) are kept: a width x depth rectangle below the
 * root; width 1 is the single greedy chain.  Order within a depth (and of the node numbers):
 * rho descending, then the parent's place in the previous depth, then the token's rank at its
 * position (probability descending, token id ascending).  A depth with fewer than `width`
 * extensions keeps them all.
 *   marginals [B,V] fp32; only the first `depth` rows are read.  1 <= width <= 16,
 *   1 <= depth <= B <= BTV_MAX_DEPTH, so at most 256 nodes.
 *   parent, token, depth_out, rho: [width*depth] as for btv_tree_build; n_out [1]; ahat [1].
 * Workspace: btv_tree_build_workspace(depth, V, width).
 * ------------------------------------------------------------------------------------------- */
int btv_tree_build_beam(const float *marginals, int B, int V, int width, int depth,
                        int32_t *parent, int32_t *token, int32_t *depth_out, float *rho,
                        int32_t *n_out, float *ahat, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * verify_cost -- HOST function, no GPU work: the verifier cost model of App. E.  FLOPs and
 * memory traffic of one target forward pass over s newly verified tokens with c cached tokens
 * (non-fused attention: the score matrix counts as activation traffic; elementwise work is
 * left out), the roofline time R = max(FLOPs / peak_flops, Bytes / bandwidth) and the
 * statically calibrated estimate calib_scale * R + calib_offset (Sec. 3.4).
 *   layers, h (hidden), nq, nkv (heads), d (head dim), hffn, V (vocabulary), bp (bytes/element)
 *   out [4] HOST: FLOPs, Bytes, R, calibrated latency.  Returns BTV_OK or BTV_EINVAL.
 * ------------------------------------------------------------------------------------------- */
int btv_verify_cost(double s, double c, double layers, double h, double nq, double nkv, double d,
                    double hffn, double V, double bp, double peak_flops, double bandwidth,
                    double calib_scale, double calib_offset, double *out);

/* ---------------------------------------------------------------------------------------------
 * Latency calibration -- HOST functions, no GPU work (Sec. 5.2).
 * calib_fit_linear: the static per-(GPU, target) calibration, read as the least-squares line
 *   obs ~ calib_scale * pred + calib_offset  through n >= 2 (roofline prediction, measured
 *   latency) pairs; pred, obs HOST [n].  BTV_EINVAL when the predictions are all equal.
 * calib_ema_update: the online bias  *c <- (1 - alpha) * *c + alpha * obs / pred,  alpha in
 *   [0, 1], pred > 0; the caller keeps c (start at 1) and passes pred = bare roofline time for
 *   the EMA variant or the statically calibrated time for the EMA+Calib variant.
 * verify_cost_curve: the controller's cost curve (Eq. 6 denominator) for N = 1..N_max draft
 *   nodes:  cost[N-1] = t_other + c_ema * (calib_scale * R(N + 1) + calib_offset),  R as in
 *   btv_verify_cost with s = N + 1 (the verifier also processes the root); t_other =
 *   T_draft + T_aux.  cost HOST [N_max]; copy it to the device for btv_tree_build_adaptive.
 * ------------------------------------------------------------------------------------------- */
int btv_calib_fit_linear(const double *pred, const double *obs, int n, double *calib_scale,
                         double *calib_offset);
int btv_calib_ema_update(double *c, double alpha, double obs, double pred);
int btv_verify_cost_curve(int N_max, double c, double layers, double h, double nq, double nkv,
                          double d, double hffn, double V, double bp, double peak_flops,
                          double bandwidth, double calib_scale, double calib_offset, double c_ema,
                          double t_other, double *cost);

/* ---------------------------------------------------------------------------------------------
 * ancestor mask -- the verification mask of App. C ("Linearization and verification mask")
 * as a bitset: bit a of anc[i] is set iff a is i or an ancestor of i.
 * anc [M, BTV_ANC_WORDS] uint32, word w holds nodes 32w..32w+31.
 * ------------------------------------------------------------------------------------------- */
int btv_tree_ancestor_mask(const int32_t *parent, int M, uint32_t *anc, void *ws, size_t ws_bytes,
                           void *stream);

/* ---------------------------------------------------------------------------------------------
 * tree_verify_attn -- tree-masked attention of one layer (App. C): node i attends to the L
 * prefix rows of the KV cache and to the tree rows of its ancestors and itself.
 *   O[i,h,:] = sum_j softmax_j(scale * Q[i,h,:].K[j,g,:]) V[j,g,:],  g = h / (Hq/Hkv),
 *   j over 0..L-1 and L+a for a in anc(i).
 * Q, O [M,Hq,D]; K, V [L+M,Hkv,D] (tree node a at row L+a); all row-major, contiguous, of
 * `dtype`, 16-byte aligned; softmax and accumulation in fp32.  scale <= 0 selects 1/sqrt(D).
 * Workspace: ancestor bitmasks and split-K partial results.
 * ------------------------------------------------------------------------------------------- */
size_t btv_tree_verify_attn_workspace(int M, int L, int Hq, int Hkv, int D, int dtype);
int btv_tree_verify_attn(const void *Q, const void *K, const void *V, const int32_t *parent,
                         int M, int L, int Hq, int Hkv, int D, int dtype, float scale,
                         void *O, void *ws, size_t ws_bytes, void *stream);

/* btv_tree_verify_attn for callers that cannot allocate or hand over a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation): the same operation, the
 * same kernels, with the scratch memory (ancestor bitmasks, split-K partial results, flags) in an
 * array that is part of the library itself, 32 MiB per GPU, held until the process ends.  The
 * call allocates and frees nothing and synchronises nothing.
 *   status   [1] uint32 DEVICE, optional: kernels OR their data-error bits into it (non-zero =
 *            what btv_workspace_status would report as BTV_EDATA); the caller clears it.
 *   Shapes whose scratch need (btv_tree_verify_attn_workspace) exceeds the array are refused with
 *   BTV_EWORKSPACE and nothing is launched; every shape with M * Hq <= 4096 rows fits.
 *   All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *   streams, two threads) race and give wrong results; calls on one stream are safe.
 * All other arguments and errors as for btv_tree_verify_attn. */
int btv_tree_verify_attn_noalloc(const void *Q, const void *K, const void *V, const int32_t *parent,
                                 int M, int L, int Hq, int Hkv, int D, int dtype, float scale,
                                 void *O, uint32_t *status, void *stream);

/* Ragged batch over a paged KV cache (BTV_PAGE-token blocks), bf16 only.
 *   Q, O        [total_M, Hq, D]; request r owns rows q_offset[r] .. q_offset[r+1]-1
 *   Kpool,Vpool [num_blocks, BTV_PAGE, Hkv, D]
 *   block_table [batch, max_blocks] int32: logical block b of request r is pool block
 *               block_table[r*max_blocks + b]; sequence position j lives in block j/BTV_PAGE at
 *               slot j%BTV_PAGE; tree node a of request r sits at position prefix_len[r] + a
 *   q_offset    [batch+1] int32, prefix_len [batch] int32 (device)
 *   parent      [total_M] int32, indices local to each request
 *   M_max, L_max  HOST upper bounds on any request's node count / prefix length (they size the
 *               grid and the workspace); a request exceeding them, or whose L+M exceeds
 *               max_blocks*BTV_PAGE, is skipped and flagged (see btv_workspace_status).
 * Block ids outside [0, num_blocks) are clamped, so no access leaves the pools. */
size_t btv_tree_verify_attn_paged_workspace(int batch, int M_max, int L_max, int Hq, int Hkv, int D);
int btv_tree_verify_attn_paged(const void *Q, const void *Kpool, const void *Vpool, int num_blocks,
                               const int32_t *block_table, int max_blocks, const int32_t *q_offset,
                               const int32_t *prefix_len, const int32_t *parent, int batch,
                               int total_M, int M_max, int L_max, int Hq, int Hkv, int D,
                               float scale, void *O, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * tree_verify_attn over an FP8 KV cache -- the same operation (App. C) with K and V stored as
 * 8-bit floats; App. E prices the cache by a bytes-per-element factor and fixes no precision.
 *   K8, V8      [L+M,Hkv,D] (or the paged pools [num_blocks, BTV_PAGE, Hkv, D]) of one byte per
 *               element in the OCP E4M3 encoding (sign, 4 exponent bits of bias 7, 3 fraction
 *               bits, subnormals, no infinities, 0x7F / 0xFF = NaN)
 *   k_scale, v_scale   one positive finite factor per tensor: element x stands for x * k_scale
 *               (keys), x * v_scale (values)
 *   Q, O        bf16, as above.  D = 128 only.
 *   O[i,h,:] = v_scale * sum_j softmax_j(scale * k_scale * Q[i,h,:].K8[j,g,:]) V8[j,g,:]
 * The codes are converted exactly (every E4M3 number is a bf16 number) and the two factors are
 * applied in fp32 to the scores and to the normalised sum, so the result differs from the bf16
 * entry point on the same numbers only by rounding order.  A NaN code makes the rows that see it
 * NaN.  All other arguments, the workspace contents and the error behaviour are those of
 * btv_tree_verify_attn / btv_tree_verify_attn_paged; the workspace queries return 0 for shapes
 * that are not built.
 * ------------------------------------------------------------------------------------------- */
size_t btv_tree_verify_attn_fp8kv_workspace(int M, int L, int Hq, int Hkv, int D);
int btv_tree_verify_attn_fp8kv(const void *Q, const void *K8, const void *V8, float k_scale,
                               float v_scale, const int32_t *parent, int M, int L, int Hq, int Hkv,
                               int D, float scale, void *O, void *ws, size_t ws_bytes, void *stream);
size_t btv_tree_verify_attn_paged_fp8kv_workspace(int batch, int M_max, int L_max, int Hq, int Hkv,
                                                  int D);
int btv_tree_verify_attn_paged_fp8kv(const void *Q, const void *K8pool, const void *V8pool,
                                     float k_scale, float v_scale, int num_blocks,
                                     const int32_t *block_table, int max_blocks,
                                     const int32_t *q_offset, const int32_t *prefix_len,
                                     const int32_t *parent, int batch, int total_M, int M_max,
                                     int L_max, int Hq, int Hkv, int D, float scale, void *O,
                                     void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * tree_accept -- the walk that commits the longest accepted root-to-node path (App. C,
 * "Acceptance"; Sec. 3.1).  logits [M+1,V] of `dtype`: row 0 is the root, row 1+i node i.
 *
 * greedy (temperature 0): t[r] = argmax_v logits[r,v] (lowest v on ties); from the root follow
 * the child whose token equals t[row of the current node] until none does.
 *   path [M] accepted node ids in root-to-leaf order (first *n_acc valid), n_acc [1],
 *   bonus [1] = t[row of the last accepted node] (the token that seeds the next cycle),
 *   argmax_out [M+1] optional.
 *   One launch: every workgroup leaves the best of its part of the rows in 8-byte words of its
 *   own in the workspace, and the workgroup with the highest index collects them (it waits for
 *   words still empty, for one second of wall clock at most: past that it raises the data flag)
 *   and does the walk; the words are back at zero when the call has run.
 *
 * stochastic (temperature 1): token-level rejection sampling of the target distribution
 * p = softmax(logits row) against the draft marginal q of the child's depth, children tried in
 * node order, one uniform each: accept iff u*q[x] < p[x]; on rejection p <- norm(max(p-q,0))
 * (unchanged if that is all zero) and q[x] <- 0, q renormalised; when no child is accepted the
 * bonus token is the inverse-CDF sample of p with the next uniform.  uniforms [M+1] fp32 in
 * [0,1), consumed in order.  marginals [B,V] fp32 as given to tree_build.
 *   Four small launches ahead of the walk prepare the root's row (softmax numerators and their
 *   (e, q) pairs sorted by q/e) on many CUs when the root has 6 children or more; the walk
 *   itself is one workgroup; one small launch after it draws the bonus token (bonus is valid
 *   when it has run, like every output: in stream order).
 * ------------------------------------------------------------------------------------------- */
size_t btv_tree_accept_workspace(int M, int V, int stochastic);
int btv_tree_accept_greedy(const void *logits, int dtype, const int32_t *parent, const int32_t *token,
                           int M, int V, int32_t *path, int32_t *n_acc, int32_t *bonus,
                           int32_t *argmax_out, void *ws, size_t ws_bytes, void *stream);
/* btv_tree_accept_greedy with the collecting workgroup's wait limit given by the caller (tests of
 * that path): wait_ticks in ticks of the 100 MHz wall clock; negative = give up before the first
 * look, which gives the outputs of logit rows whose argmax is 0 everywhere, raises the data flag
 * and leaves the workspace dirty (zero-fill it again before its next use).  Every kernel ends
 * normally. */
int btv_tree_accept_greedy_tuned(const void *logits, int dtype, const int32_t *parent,
                                 const int32_t *token, int M, int V, int32_t *path, int32_t *n_acc,
                                 int32_t *bonus, int32_t *argmax_out, void *ws, size_t ws_bytes,
                                 void *stream, long long wait_ticks);
int btv_tree_accept_stochastic(const void *logits, int dtype, const float *marginals, int B,
                               const int32_t *parent, const int32_t *token, int M, int V,
                               const float *uniforms, int32_t *path, int32_t *n_acc, int32_t *bonus,
                               void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Greedy acceptance straight from the final hidden states: the LM head of App. E (2*s*h*V FLOPs,
 * s*V logits of activation traffic) fused with the top-1 of App. C "Acceptance", so the logits
 * are never written:  t[r] = argmax_v sum_k hidden[r,k] * W[v,k]  (lowest v on ties), then the
 * same walk as btv_tree_accept_greedy.
 *   hidden [M+1, h] bf16 (row 0 = root, row 1+i = node i; final norm already applied)
 *   W      [V, h]   bf16, row-major (one row per token); both DEVICE, 16-byte aligned
 *   h      a multiple of 128
 * Products are exact in fp32 and accumulated in fp32 on the matrix cores; two tokens whose
 * logits differ by less than that rounding (about 1e-6 of sum_k |hidden*W|) can swap.
 * Outputs and errors as for btv_tree_accept_greedy.
 * ------------------------------------------------------------------------------------------- */
size_t btv_tree_accept_lm_head_workspace(int M, int V);
int btv_tree_accept_greedy_lm_head(const void *hidden, const void *W, int h, const int32_t *parent,
                                   const int32_t *token, int M, int V, int32_t *path,
                                   int32_t *n_acc, int32_t *bonus, int32_t *argmax_out, void *ws,
                                   size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * kv_commit -- makes the KV cache ready for the next cycle (App. C, "Acceptance"): behind the L
 * prefix rows only the rows of the accepted nodes are needed, in path order.  In every layer, in K
 * and in V, the row at sequence position L + path[j] is moved to position L + j for j < *n_acc;
 * positions from L + *n_acc on hold nothing of use afterwards.  In place.
 *   K, V     [layers][>= L+M rows][row_bytes]; layer l starts layer_stride_bytes * l after the base;
 *            row_bytes = Hkv * D * element size, a multiple of 16, at most 32768; 16-byte aligned
 *   path     [M] int32, n_acc [1] int32 (device): as written by tree_accept (node ids in
 *            root-to-leaf order, hence increasing, path[j] >= j).  A path that breaks this
 *            gives unspecified rows L .. L+M-1, nothing else is touched (ids are clamped).
 *   new_len  [1] int32 optional: L + *n_acc
 * The paged form does the same for a batch of requests over block pools laid out
 * [layers][num_blocks][BTV_PAGE][row_bytes] with the block table and prefix lengths of
 * btv_tree_verify_attn_paged; n_acc, new_len [batch].  Paths: with q_offset ([batch+1], the array
 * the other batch calls take; total_M = q_offset[batch]) request r's ids start at path[q_offset[r]],
 * exactly as btv_tree_accept_greedy_batch writes them; with q_offset NULL they start at
 * path[r * M_max] (total_M is ignored).  ws (optional) receives the data flag when a request's
 * n_acc, offsets or prefix length are out of range (that request is left untouched).
 * ------------------------------------------------------------------------------------------- */
int btv_kv_commit(void *K, void *V, int layers, long long layer_stride_bytes, int L, int M, int row_bytes,
                  const int32_t *path, const int32_t *n_acc, int32_t *new_len, void *stream);
int btv_kv_commit_paged(void *Kpool, void *Vpool, int layers, long long layer_stride_bytes, int num_blocks,
                        const int32_t *block_table, int max_blocks, const int32_t *prefix_len,
                        const int32_t *path, const int32_t *q_offset, int total_M, const int32_t *n_acc,
                        int batch, int M_max, int row_bytes, int32_t *new_len, void *ws, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Tuning and test form of btv_tree_verify_attn / btv_tree_verify_attn_fp8kv (App. C; bf16 Q and O):
 * the same operation with the two choices the library otherwise makes itself passed explicitly, so
 * that a test can run every kernel shape and split count on any input, and a tuner can sweep them.
 *   kv_fp8   0: K, V bf16, the two scales are ignored;  1: E4M3 codes with k_scale, v_scale
 *   nsplit   number of pieces the key range is cut into (0 = the library's choice; the library
 *            rounds pieces to whole tiles, so fewer may result)
 *   shape    0 = the library's choice; 1, 2, 3 = workgroups of 64, 128, 256 packed query rows
 *            (3 is not built for an FP8 cache: BTV_EINVAL)
 * The workspace query takes the same nsplit and shape as the call it sizes.
 * ------------------------------------------------------------------------------------------- */
size_t btv_tree_verify_attn_tuned_workspace(int M, int L, int Hq, int Hkv, int D, int kv_fp8,
                                            int nsplit, int shape);
int btv_tree_verify_attn_tuned(const void *Q, const void *K, const void *V, int kv_fp8, float k_scale,
                               float v_scale, const int32_t *parent, int M, int L, int Hq, int Hkv,
                               int D, float scale, int nsplit, int shape, void *O, void *ws,
                               size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BASTION_TV_H */
