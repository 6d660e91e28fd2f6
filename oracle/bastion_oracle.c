/*
 * CPU oracle for the tree-verify path of budget-aware tree speculative decoding.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow and meant to be checked against the paper by eye.
 * It shares no code with the HIP library and must never be reached from the product path:
 * only the tests, the smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * Every function cites the passage of the paper it follows.  Floating point is fp64,
 * except where a floating-point value decides an integer output that the HIP path must
 * reproduce bit for bit (the path score rho, which orders the tree): there both sides
 * use one IEEE fp32 multiply per tree edge, as stated below.
 *
 * Pins (tests/, run with -m "not gpu"):
 *   orc_tree_build       brute-force enumeration of all prefixes (Prop. 3.3), closed forms,
 *                        Monte-Carlo self-verification (Prop. 3.2)
 *   orc_tree_build_adaptive  exhaustive argmax of the estimated speedup over all budgets on concave/convex
 *                        inputs (Prop. 3.4), prefix property against orc_tree_build, hand-made cost curves
 *   orc_tree_build_beam  hand-worked example, width 1 = per-position argmax chain, full-width = whole lattice,
 *                        per-depth top-w of explicitly enumerated extensions (numpy sort), Prop. 3.3 upper bound
 *   orc_verify_cost      the per-module tables of App. E summed by hand for a small configuration
 *   orc_calib_fit        exact recovery of a planted line, numpy's polynomial fit, zero-gradient of the residual
 *   orc_calib_ema        closed form of the geometric approach to a constant ratio
 *   orc_cost_curve       assembled by hand from orc_verify_cost's pinned totals
 *   orc_kv_commit        array gather by a library routine (numpy indexing), identity and chain cases
 *   orc_tree_attn        library causal attention over each root-to-node path, chain/star cases
 *   orc_fp8_e4m3_decode  a library conversion (torch's float8_e4m3fn) over all 256 codes, the format's named values
 *   orc_tree_attn_fp8kv  library attention over values decoded and scaled by that library, scale-folding identities
 *   orc_ancestor_mask    reachability by explicit path enumeration
 *   orc_accept_greedy    brute force over all root-to-node paths, planted paths
 *   orc_lm_head_argmax   library matrix product + argmax (numpy, fp64), planted winners, exact ties, one-hot rows
 *   orc_accept_stochastic  closed-form special cases and an empirical chi-square test of the
 *                        single-child case; the multi-child rule is not given by the paper:
 *                        parity unpinned beyond those cases.
 */
#define _GNU_SOURCE
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------------
 * Per-position ranking of the drafter's marginals (Sec. 3.3: candidate lattice of the top
 * tokens at each position).  rank r of position k = r-th token when sorted by probability
 * descending, token id ascending on equal probability.
 * ---------------------------------------------------------------------------------------- */
static int cmp_prob_desc_id_asc(const void *a, const void *b, void *ctx)
{
    const float *q = (const float *)ctx;
    int32_t ia = *(const int32_t *)a, ib = *(const int32_t *)b;
    if (q[ia] > q[ib]) return -1;
    if (q[ia] < q[ib]) return 1;
    return (ia > ib) - (ia < ib);
}

/* order[k*V + r] = token id of rank r at position k */
void orc_rank_tokens(const float *marg, int B, int V, int32_t *order)
{
    for (int k = 0; k < B; ++k) {
        int32_t *o = order + (size_t)k * V;
        for (int v = 0; v < V; ++v) o[v] = v;
        qsort_r(o, (size_t)V, sizeof(int32_t), cmp_prob_desc_id_asc, (void *)(marg + (size_t)k * V));
    }
}

/* ------------------------------------------------------------------------------------------
 * Best-first expansion at a fixed budget N (Sec. 3.3 Prop. 3.3; Algorithm 1 without the
 * early stop).  A candidate is a prefix of the lattice: (parent node, rank at its depth).
 * Path score (Eq. 1): rho(root) = 1, rho(child) = rho(parent) * q_depth(token), evaluated as
 * one fp32 multiply per edge.  N counts draft (non-root) nodes; Ahat = 1 + sum rho (Eq. 3,
 * the root contributes 1).
 *
 * Selection order (the paper leaves ties open): rho descending, then depth ascending, then
 * the rank path (r_1..r_d) lexicographically ascending.  The frontier is the set of prefixes
 * whose parent is in the tree and whose previous sibling (rank-1) is in the tree; it is kept
 * as a plain array and scanned linearly for the best element.
 * ---------------------------------------------------------------------------------------- */
typedef struct { float rho; int32_t depth, parent, rank; } cand_t;

static int rank_path(const int32_t *parent, const int32_t *rank, const int32_t *depth, int32_t p, int32_t r,
                     int32_t *out)
{   /* rank path of the candidate (parent node p, rank r); returns its length */
    int d = (p < 0) ? 1 : depth[p] + 1;
    out[d - 1] = r;
    for (int32_t a = p; a >= 0; a = parent[a]) out[depth[a] - 1] = rank[a];
    return d;
}

static int cand_before(const cand_t *a, const cand_t *b, const int32_t *parent, const int32_t *rank,
                       const int32_t *depth, int B)
{
    if (a->rho != b->rho) return a->rho > b->rho;
    if (a->depth != b->depth) return a->depth < b->depth;
    int32_t pa[64], pb[64];
    (void)B;
    int d = rank_path(parent, rank, depth, a->parent, a->rank, pa);
    rank_path(parent, rank, depth, b->parent, b->rank, pb);
    for (int i = 0; i < d; ++i)
        if (pa[i] != pb[i]) return pa[i] < pb[i];
    return 0;
}

/* The tree under construction plus its frontier.  The frontier holds every prefix that may be selected next:
 * its parent is in the tree and so is its previous sibling.  It is kept sorted in selection order (best first) by
 * insertion, so selecting is taking the head. */
typedef struct {
    const float *marg; const int32_t *order; int B, V;
    int32_t *parent, *token, *depth, *rank; float *rho;
    int n;                       /* nodes in the tree */
    cand_t *front; int nf;       /* sorted frontier */
} build_t;

/* Path score of the prefix "child of node p with rank r" (Eq. 1): the parent's score times the marginal of the
 * token of that rank at the child's depth, as one rounded fp32 multiply (the root scores 1). */
static float prefix_score(const build_t *b, int32_t p, int32_t r)
{
    int d = (p < 0) ? 0 : b->depth[p];                       /* 0-based position of the child's token */
    float q = b->marg[(size_t)d * b->V + b->order[(size_t)d * b->V + r]];
    volatile float s = ((p < 0) ? 1.0f : b->rho[p]) * q;
    return s;
}

static void frontier_insert(build_t *b, int32_t p, int32_t r)
{
    cand_t c = { prefix_score(b, p, r), (p < 0) ? 1 : b->depth[p] + 1, p, r };
    int at = b->nf;
    while (at > 0 && cand_before(&c, &b->front[at - 1], b->parent, b->rank, b->depth, b->B)) {
        b->front[at] = b->front[at - 1];
        --at;
    }
    b->front[at] = c;
    ++b->nf;
}

/* Budget controller (Sec. 3.4, Eq. 6): would the tree with one more node of score `rho_next` have a strictly
 * better estimated speedup  S = Ahat * L_AR / C(size)  than the best seen so far?  Updates *s_best when it does,
 * and *margin with the relative distance between the two quotients (how close the decision was). */
static int controller_keeps(double ahat_with, double L_AR, double cost_at_size, double *s_best, double *margin)
{
    double s = ahat_with * L_AR / cost_at_size;
    if (*s_best > -INFINITY) {
        double rel = fabs(s - *s_best) / fmax(fabs(s), 1e-300);
        if (rel < *margin) *margin = rel;
    }
    if (!(s > *s_best)) return 0;
    *s_best = s;
    return 1;
}

/* Core of both builders.  cost == NULL: fixed budget N (Prop. 3.3).  Otherwise the budget is chosen online
 * (Algorithm 1): cost[k-1] is the estimated cycle latency C(k) = T_draft + T_aux + T_verify(k) supplied by the
 * caller, and growth ends at the first node that does not strictly improve the estimated speedup; that node is
 * not part of the returned tree.  Ahat, S in fp64.  s_best: best estimated speedup (-inf when no node was kept);
 * margin: the smallest relative distance between compared quotients. */
static int tree_build_core(const float *marg, int B, int V, int N, const double *cost, double L_AR, int32_t *parent,
                           int32_t *token, int32_t *depth, float *rho, int32_t *rank, double *ahat, double *s_best,
                           double *margin)
{
    if (B < 1 || B > 64 || V < 1 || N < 0) return -1;
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * V);
    orc_rank_tokens(marg, B, V, order);
    build_t b = { marg, order, B, V, parent, token, depth, rank, rho, 0,
                  (cand_t *)malloc(sizeof(cand_t) * (size_t)(N + 2)), 0 };
    double a = 1.0, sb = -INFINITY, mg = INFINITY;           /* the root alone: Ahat = 1 */
    frontier_insert(&b, -1, 0);                              /* the root's most probable child */
    while (b.n < N && b.nf > 0) {
        cand_t u = b.front[0];                               /* the best prefix not yet in the tree */
        if (cost && !controller_keeps(a + (double)u.rho, L_AR, cost[b.n], &sb, &mg)) break;
        for (int j = 1; j < b.nf; ++j) b.front[j - 1] = b.front[j];
        --b.nf;
        int i = b.n++;
        parent[i] = u.parent; rank[i] = u.rank; depth[i] = u.depth; rho[i] = u.rho;
        token[i] = order[(size_t)(u.depth - 1) * V + u.rank];
        a += (double)u.rho;
        /* what becomes selectable through u: its own best extension, and the sibling ranked right after it */
        if (u.depth < B) frontier_insert(&b, i, 0);
        if (u.rank + 1 < V) frontier_insert(&b, u.parent, u.rank + 1);
    }
    if (ahat) *ahat = a;
    if (s_best) *s_best = sb;
    if (margin) *margin = mg;
    free(order); free(b.front);
    return b.n;
}

/* Returns the number of nodes emitted (= N unless the lattice has fewer prefixes), or -1 on bad arguments.
 * parent[i] = -1 for children of the root; depth is 1-based; rank[i] = sibling rank of node i. */
int orc_tree_build(const float *marg, int B, int V, int N, int32_t *parent, int32_t *token, int32_t *depth,
                   float *rho, int32_t *rank, double *ahat)
{
    return tree_build_core(marg, B, V, N, NULL, 0.0, parent, token, depth, rho, rank, ahat, NULL, NULL);
}

/* Algorithm 1: budget chosen online, at most N_max nodes.  cost[0..N_max-1] > 0.  Returns N*. */
int orc_tree_build_adaptive(const float *marg, int B, int V, int N_max, const double *cost, double L_AR,
                            int32_t *parent, int32_t *token, int32_t *depth, float *rho, int32_t *rank,
                            double *ahat, double *s_best, double *margin)
{
    if (!cost || !(L_AR > 0.0)) return -1;
    for (int i = 0; i < N_max; ++i)
        if (!(cost[i] > 0.0)) return -1;
    return tree_build_core(marg, B, V, N_max, cost, L_AR, parent, token, depth, rho, rank, ahat, s_best, margin);
}

/* ------------------------------------------------------------------------------------------
 * Beam-search tree (Sec. 4.3, the comparison topology): depth by depth, of all one-token extensions of the
 * prefixes kept at the previous depth, the `width` with the largest path score (Eq. 1) are kept, which gives a
 * width x depth rectangle below the root; width 1 is the single greedy chain.  Every extension of every kept
 * prefix is enumerated (all V tokens) and the list is sorted.  Order within a depth (the paper is silent):
 * rho descending, then the parent's place in the previous depth ascending, then the token's rank at that
 * position ascending (probability descending, token id ascending).  Nodes are numbered depth by depth in that
 * order.  A depth with fewer than `width` extensions keeps them all.  Returns the node count.
 * ---------------------------------------------------------------------------------------- */
typedef struct { float rho; int32_t parent_place, rank; } beam_cand_t;

static int cmp_beam(const void *a, const void *b)
{
    const beam_cand_t *x = (const beam_cand_t *)a, *y = (const beam_cand_t *)b;
    if (x->rho != y->rho) return x->rho > y->rho ? -1 : 1;
    if (x->parent_place != y->parent_place) return x->parent_place < y->parent_place ? -1 : 1;
    return (x->rank > y->rank) - (x->rank < y->rank);
}

int orc_tree_build_beam(const float *marg, int B, int V, int width, int depth_max, int32_t *parent, int32_t *token,
                        int32_t *depth, float *rho, int32_t *rank, double *ahat)
{
    if (B < 1 || V < 1 || width < 1 || depth_max < 1 || depth_max > B) return -1;
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * V);
    beam_cand_t *cand = (beam_cand_t *)malloc(sizeof(beam_cand_t) * (size_t)width * V);
    orc_rank_tokens(marg, B, V, order);
    int n = 0, first = 0, kept = 1;          /* previous depth: nodes first .. first + kept - 1 (depth 0: the root) */
    double a = 1.0;
    for (int k = 0; k < depth_max; ++k) {
        size_t nc = 0;
        for (int b = 0; b < kept; ++b) {
            float prho = (k == 0) ? 1.0f : rho[first + b];
            for (int r = 0; r < V; ++r) {
                volatile float child = prho * marg[(size_t)k * V + order[(size_t)k * V + r]];   /* one fp32 multiply */
                cand[nc++] = (beam_cand_t){ child, b, r };
            }
        }
        qsort(cand, nc, sizeof(beam_cand_t), cmp_beam);
        int keep = nc < (size_t)width ? (int)nc : width;
        for (int i = 0; i < keep; ++i) {
            parent[n + i] = (k == 0) ? -1 : first + cand[i].parent_place;
            rank[n + i] = cand[i].rank;
            token[n + i] = order[(size_t)k * V + cand[i].rank];
            depth[n + i] = k + 1;
            rho[n + i] = cand[i].rho;
            a += (double)cand[i].rho;
        }
        first = n; kept = keep; n += keep;
    }
    *ahat = a;
    free(order); free(cand);
    return n;
}

/* ------------------------------------------------------------------------------------------
 * Verifier cost model (App. E): FLOPs and memory traffic of one target forward pass over s newly
 * verified tokens with c cached tokens, as the sums of the per-module entries of the appendix's two
 * tables (a multiply-accumulate counts 2 FLOPs; elementwise work is left out; non-fused attention,
 * so the score matrix counts as activation traffic), the roofline time
 *     R = max(FLOPs / peak_flops, Bytes / bandwidth)
 * and the statically calibrated estimate  T = calib_scale * R + calib_offset  (Sec. 3.4: "a linear
 * calibration").  hq = nq*d, hkv = nkv*d.  out[0] = FLOPs, out[1] = Bytes, out[2] = R, out[3] = T.
 * ---------------------------------------------------------------------------------------- */
void orc_verify_cost(double s, double c, double layers, double h, double nq, double nkv, double d, double hffn,
                     double V, double bp, double peak_flops, double bandwidth, double calib_scale,
                     double calib_offset, double *out)
{
    double hq = nq * d, hkv = nkv * d;
    /* FLOPs per layer, module by module */
    double f_qproj = 2 * s * h * hq, f_kvproj = 4 * s * h * hkv, f_scores = 2 * s * (c + s) * hq;
    double f_pv = 2 * s * (c + s) * hq, f_oproj = 2 * s * hq * h, f_gateup = 4 * s * h * hffn, f_down = 2 * s * hffn * h;
    double f_lmhead = 2 * s * h * V;
    double flops = layers * (f_qproj + f_kvproj + f_scores + f_pv + f_oproj + f_gateup + f_down) + f_lmhead;
    /* traffic in elements, module by module */
    double w_embed_lm = V * h + h * V, w_attn = 2 * h * hq + 2 * h * hkv, w_ffn = 3 * h * hffn;
    double kv_read = 2 * c * hkv, kv_write = 2 * s * hkv;
    double a_attn = 2 * s * h + 4 * s * hq + 2 * s * hkv + 2 * nq * s * (c + s), a_ffn = 2 * s * h + 4 * s * hffn;
    double a_lm = s * h + s * V;
    double bytes = bp * (w_embed_lm + layers * (w_attn + w_ffn) + layers * (kv_read + kv_write) +
                         layers * (a_attn + a_ffn) + a_lm);
    double r = fmax(flops / peak_flops, bytes / bandwidth);
    out[0] = flops; out[1] = bytes; out[2] = r; out[3] = calib_scale * r + calib_offset;
}

/* ------------------------------------------------------------------------------------------
 * Calibration of the latency estimate (Sec. 5.2).
 *
 * Static: "a per-(GPU, target) linear calibration" of the roofline prediction against measured latency.  The
 * paper does not name the fit; it is read as the ordinary least-squares line  obs ~ scale * pred + offset,
 * written here from the normal equations with centred sums.  Fewer than two points, or predictions that are all
 * equal, leave the slope undetermined: return -1.
 *
 * Online: one multiplicative bias updated as  c <- (1 - alpha) c + alpha (obs / pred);  the corrected estimate
 * is c * pred, where pred is the bare roofline time (EMA) or the statically calibrated one (EMA+Calib).  The
 * start value is not given; callers pass it (1 = no correction).
 * ---------------------------------------------------------------------------------------- */
int orc_calib_fit(const double *pred, const double *obs, int n, double *scale, double *offset)
{
    if (n < 2) return -1;
    double mp = 0, mo = 0;
    for (int i = 0; i < n; ++i) { mp += pred[i]; mo += obs[i]; }
    mp /= n; mo /= n;
    double spp = 0, spo = 0;
    for (int i = 0; i < n; ++i) { spp += (pred[i] - mp) * (pred[i] - mp); spo += (pred[i] - mp) * (obs[i] - mo); }
    if (!(spp > 0)) return -1;
    *scale = spo / spp;
    *offset = mo - *scale * mp;
    return 0;
}

double orc_calib_ema(double c, double alpha, double obs, double pred)
{
    return (1.0 - alpha) * c + alpha * (obs / pred);
}

/* Cost curve handed to the budget controller (Eq. 6 denominator): for N = 1..N_max,
 *     C(N) = T_other + c_ema * (calib_scale * R(N + 1) + calib_offset),
 * where R is the roofline time of the model above.  N counts draft nodes, the verifier also processes the root,
 * hence s = N + 1 new tokens.  T_other = T_draft + T_aux. */
void orc_cost_curve(int N_max, double c, double layers, double h, double nq, double nkv, double d, double hffn,
                    double V, double bp, double peak_flops, double bandwidth, double calib_scale, double calib_offset,
                    double c_ema, double t_other, double *cost)
{
    for (int n = 1; n <= N_max; ++n) {
        double out[4];
        orc_verify_cost((double)n + 1.0, c, layers, h, nq, nkv, d, hffn, V, bp, peak_flops, bandwidth, calib_scale,
                        calib_offset, out);
        cost[n - 1] = t_other + c_ema * out[3];
    }
}

/* ------------------------------------------------------------------------------------------
 * Tree-masked attention (App. C, "Linearization and verification mask"): node i attends to
 * the L prefix rows of the KV cache and to the tree rows of its own ancestors and itself,
 * nothing else.  For query head h (KV head h / (Hq/Hkv)):
 *     O[i,h] = sum_j softmax_j( scale * Q[i,h].K[j] ) V[j],   j over  0..L-1, then L+a for a on
 *     the root-to-i path.
 * Written as the definition: gather the visible rows, scores, max-subtracted softmax, weighted sum.
 *
 * Inputs are fp32 arrays holding the exact stored values (bf16-rounded when the HIP path runs in
 * bf16).  K/V row j lives at physical row  j                       if block_table == NULL,
 *                                          block_table[j/page]*page + j%page   otherwise.
 * pairs: npairs x 2 (node, head) to evaluate, or NULL for all (node-major, head-minor).
 * O: fp64 [npairs or M*Hq, D].
 * ---------------------------------------------------------------------------------------- */
static inline size_t phys_row(int j, const int32_t *block_table, int page)
{
    return block_table ? (size_t)block_table[j / page] * (size_t)page + (size_t)(j % page) : (size_t)j;
}

int orc_tree_attn(const float *Q, const float *K, const float *V, const int32_t *parent, int M, int L, int Hq,
                  int Hkv, int D, double scale, const int32_t *block_table, int page, const int32_t *pairs,
                  int npairs, double *O, int nthreads)
{
    if (M < 0 || L < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv || D < 1) return -1;
    for (int i = 0; i < M; ++i)
        if (parent[i] < -1 || parent[i] >= i) return -2;
    int total = pairs ? npairs : M * Hq;
    int G = Hq / Hkv;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
#endif
    for (int t = 0; t < total; ++t) {
        int i = pairs ? pairs[2 * t] : t / Hq;
        int h = pairs ? pairs[2 * t + 1] : t % Hq;
        int g = h / G;
        /* visible rows: the prefix, then the root-to-i path in path order */
        int np = 0;
        for (int a = i; a >= 0; a = parent[a]) ++np;
        int nvis = L + np;
        int *vis = (int *)malloc(sizeof(int) * (size_t)(nvis > 0 ? nvis : 1));
        double *s = (double *)malloc(sizeof(double) * (size_t)(nvis > 0 ? nvis : 1));
        for (int j = 0; j < L; ++j) vis[j] = j;
        { int k = nvis; for (int a = i; a >= 0; a = parent[a]) vis[--k] = L + a; }
        const float *q = Q + ((size_t)i * Hq + h) * D;
        double m = -INFINITY;
        for (int j = 0; j < nvis; ++j) {
            const float *k = K + (phys_row(vis[j], block_table, page) * Hkv + g) * D;
            double acc = 0.0;
            for (int d = 0; d < D; ++d) acc += (double)q[d] * (double)k[d];
            s[j] = acc * scale;
            if (s[j] > m) m = s[j];
        }
        double z = 0.0;
        for (int j = 0; j < nvis; ++j) { s[j] = exp(s[j] - m); z += s[j]; }
        double *o = O + (size_t)t * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int j = 0; j < nvis; ++j) {
            const float *v = V + (phys_row(vis[j], block_table, page) * Hkv + g) * D;
            double p = s[j] / z;
            for (int d = 0; d < D; ++d) o[d] += p * (double)v[d];
        }
        free(vis); free(s);
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * FP8 KV cache (a storage variant of the same attention; the paper fixes no KV precision, App. E
 * only carries a bytes-per-element factor).  Cache elements are 8-bit floats in the OCP "E4M3"
 * encoding: 1 sign bit, 4 exponent bits with bias 7, 3 fraction bits; exponent field 0 holds the
 * subnormals f/8 * 2^-6; there are no infinities; exponent 15 with fraction 7 is NaN, every other
 * pattern is finite (largest 448).  A stored element x stands for the number  x * k_scale  (keys)
 * or  x * v_scale  (values), one scale per tensor.
 * ---------------------------------------------------------------------------------------- */
void orc_fp8_e4m3_decode(const uint8_t *code, size_t n, float *out)
{
    for (size_t i = 0; i < n; ++i) {
        int c = code[i], e = (c >> 3) & 15, f = c & 7;
        double v;
        if (e == 15 && f == 7) v = NAN;
        else if (e == 0) v = ldexp((double)f / 8.0, -6);
        else v = ldexp(1.0 + (double)f / 8.0, e - 7);
        out[i] = (float)((c & 128) ? -v : v);      /* every finite value is exact in fp32 */
    }
}

/* Attention by its definition over the numbers the cache stands for:
 * scores scale * Q.(k_scale K8) and values v_scale V8.  The decoded elements go through
 * orc_tree_attn unchanged, with the two per-tensor factors applied in fp64 where the definition
 * has them (on the score and on the weighted sum), so nothing is rounded in between. */
int orc_tree_attn_fp8kv(const float *Q, const uint8_t *K8, const uint8_t *V8, size_t kv_elems, double k_scale,
                        double v_scale, const int32_t *parent, int M, int L, int Hq, int Hkv, int D, double scale,
                        const int32_t *block_table, int page, const int32_t *pairs, int npairs, double *O,
                        int nthreads)
{
    float *K = (float *)malloc(sizeof(float) * (kv_elems ? kv_elems : 1));
    float *V = (float *)malloc(sizeof(float) * (kv_elems ? kv_elems : 1));
    if (!K || !V) { free(K); free(V); return -9; }
    orc_fp8_e4m3_decode(K8, kv_elems, K);
    orc_fp8_e4m3_decode(V8, kv_elems, V);
    int rc = orc_tree_attn(Q, K, V, parent, M, L, Hq, Hkv, D, scale * k_scale, block_table, page, pairs, npairs, O,
                           nthreads);
    if (rc == 0) {
        size_t total = (size_t)(pairs ? npairs : M * Hq) * (size_t)D;
        for (size_t i = 0; i < total; ++i) O[i] *= v_scale;
    }
    free(K); free(V);
    return rc;
}

/* ------------------------------------------------------------------------------------------
 * Greedy acceptance (App. C, "Acceptance"; Sec. 3.1): the target's top-1 token at every tree
 * row, then the longest root-to-node path whose tokens are what the target itself would have
 * produced.  logits row 0 belongs to the root, row 1+i to node i.  Ties in the argmax go to
 * the lowest token id (the paper is silent).  bonus = the target's token at the last accepted
 * node (the token that seeds the next cycle).
 * ---------------------------------------------------------------------------------------- */
void orc_row_argmax(const float *logits, int rows, int V, int32_t *t)
{
    for (int r = 0; r < rows; ++r) {
        const float *x = logits + (size_t)r * V;
        int best = 0;
        for (int v = 1; v < V; ++v)
            if (x[v] > x[best]) best = v;
        t[r] = best;
    }
}

/* ------------------------------------------------------------------------------------------
 * Target tokens straight from the final hidden states (the LM head of App. E, 2*s*h*V FLOPs, followed by the
 * top-1 of App. C "Acceptance"):  logit[r, v] = sum_k hidden[r, k] * W[v, k],  t[r] = argmax_v logit[r, v], lowest
 * v on ties.  hidden [R, h] and W [V, h] are fp32 arrays holding the exact stored values (bf16-rounded when the
 * HIP path runs in bf16); every logit is accumulated in fp64 in index order.  margin[r] (optional) = best logit
 * minus the best logit of any other token (0 on an exact tie): rows with a margin below the other side's rounding
 * error have no unique answer and parity tests leave them out.
 * ---------------------------------------------------------------------------------------- */
void orc_lm_head_argmax(const float *hidden, const float *W, int R, int h, int V, int32_t *t, double *margin,
                        int nthreads)
{
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
#endif
    for (int r = 0; r < R; ++r) {
        const float *x = hidden + (size_t)r * h;
        double best = -INFINITY, second = -INFINITY;
        int arg = 0;
        for (int v = 0; v < V; ++v) {
            const float *w = W + (size_t)v * h;
            double z = 0.0;
            for (int k = 0; k < h; ++k) z += (double)x[k] * (double)w[k];
            if (z > best) { second = best; best = z; arg = v; }
            else if (z > second) second = z;
        }
        t[r] = arg;
        if (margin) margin[r] = (V > 1) ? best - second : INFINITY;
    }
}

/* returns n_acc; path[0..n_acc) = accepted node ids in root-to-leaf order */
int orc_accept_greedy(const float *logits, const int32_t *parent, const int32_t *token, int M, int V,
                      int32_t *path, int32_t *bonus, int32_t *t_out /* [M+1] or NULL */)
{
    int32_t *t = (int32_t *)malloc(sizeof(int32_t) * (size_t)(M + 1));
    orc_row_argmax(logits, M + 1, V, t);
    int cur = -1, n = 0;
    for (;;) {
        int next = -1;
        for (int c = 0; c < M; ++c)
            if (parent[c] == cur && token[c] == t[cur + 1]) { next = c; break; }
        if (next < 0) break;
        path[n++] = next;
        cur = next;
    }
    *bonus = t[cur + 1];
    if (t_out) memcpy(t_out, t, sizeof(int32_t) * (size_t)(M + 1));
    free(t);
    return n;
}

/* ------------------------------------------------------------------------------------------
 * Stochastic acceptance at temperature 1.  The paper states only that decoding preserves the
 * target distribution and cites standard speculative sampling (Sec. 2.1); the rule used here
 * is the reading fixed for this build: token-level rejection of each child, in sibling order,
 * of the target probability p against the draft marginal q of the child's depth, with the
 * residual update on rejection and the bonus token drawn from what is left of p.
 *
 *   cur = root; d = 0
 *   loop: p = softmax(logits[row(cur)]);  q = marginals[d] (copy)
 *         for each child c of cur in node order (= sibling rank order):
 *             x = token[c]; u = next uniform
 *             accept c if  u * q[x] < p[x]           (u < min(1, p/q); q[x] == 0 accepts iff p[x] > 0)
 *             else p = max(p - q, 0), renormalised (kept as is if it sums to 0);
 *                  q[x] = 0, renormalised (left all-zero if it sums to 0)
 *         no child accepted (or d == B): bonus = smallest v with cumsum(p)[v] > u (next uniform), stop.
 *
 * Uniforms are consumed strictly in order.  margin_out receives the smallest relative distance
 * of any accept/reject decision from its threshold and gap_out the absolute distance of the
 * bonus draw from the nearer CDF step, so a caller can discard inputs whose outcome depends on
 * the last bits of a vocabulary-wide sum.
 * ---------------------------------------------------------------------------------------- */
int orc_accept_stochastic(const float *logits, const float *marg, int B, const int32_t *parent,
                          const int32_t *token, const int32_t *depth, int M, int V, const float *uniforms,
                          int32_t *path, int32_t *bonus, int32_t *n_uniforms_used, double *margin_out,
                          double *gap_out)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    double *q = (double *)malloc(sizeof(double) * (size_t)V);
    double *r = (double *)malloc(sizeof(double) * (size_t)V);
    int cur = -1, n = 0, ui = 0, d = 0;
    double margin = INFINITY, bgap = INFINITY;
    (void)depth;   /* the depth of cur is tracked by the walk itself */
    for (;;) {
        /* target distribution at the current node: softmax of its logits row */
        const float *x = logits + (size_t)(cur + 1) * V;
        double mx = -INFINITY, z = 0.0;
        for (int v = 0; v < V; ++v) if ((double)x[v] > mx) mx = (double)x[v];
        for (int v = 0; v < V; ++v) { p[v] = exp((double)x[v] - mx); z += p[v]; }
        for (int v = 0; v < V; ++v) p[v] /= z;
        int accepted = -1;
        if (d < B) {
            for (int v = 0; v < V; ++v) q[v] = (double)marg[(size_t)d * V + v];
            for (int c = 0; c < M; ++c) {
                if (parent[c] != cur) continue;
                int tk = token[c];
                double u = (double)uniforms[ui++];
                double lhs = u * q[tk], rhs = p[tk];
                if (!(lhs == 0.0 && rhs == 0.0)) {
                    double rel = fabs(lhs - rhs) / (rhs > 0.0 ? rhs : lhs);
                    if (rel < margin) margin = rel;
                }
                if (lhs < rhs) { accepted = c; break; }
                /* rejected: residual target, and the draft without the tried token */
                double zr = 0.0, zq = 0.0;
                for (int v = 0; v < V; ++v) { double t = p[v] - q[v]; r[v] = t > 0.0 ? t : 0.0; zr += r[v]; }
                if (zr > 0.0) for (int v = 0; v < V; ++v) p[v] = r[v] / zr;
                q[tk] = 0.0;
                for (int v = 0; v < V; ++v) zq += q[v];
                if (zq > 0.0) for (int v = 0; v < V; ++v) q[v] /= zq;
            }
        }
        if (accepted >= 0) { path[n++] = accepted; cur = accepted; ++d; continue; }
        /* bonus token by inverse CDF of what is left of p */
        double u = (double)uniforms[ui++], c = 0.0;
        int b = -1, last_pos = 0;
        for (int v = 0; v < V; ++v) {
            if (p[v] > 0.0) last_pos = v;
            double c2 = c + p[v];
            if (b < 0 && c2 > u) {
                b = v;
                double gap = fmin(c2 - u, u - c);
                bgap = gap;
            }
            c = c2;
        }
        if (b < 0) b = last_pos;   /* u beyond the rounded total: last token with mass */
        *bonus = b;
        break;
    }
    if (n_uniforms_used) *n_uniforms_used = ui;
    if (margin_out) *margin_out = margin;
    if (gap_out) *gap_out = bgap;
    free(p); free(q); free(r);
    return n;
}

/* ------------------------------------------------------------------------------------------
 * Verification mask as a bitset (App. C, "Linearization and verification mask"): bit a of
 * anc[i] is set iff tree node a is i itself or an ancestor of i.  words = 32-bit words per row.
 * ---------------------------------------------------------------------------------------- */
int orc_ancestor_mask(const int32_t *parent, int M, int words, uint32_t *anc)
{
    for (int i = 0; i < M; ++i) {
        if (parent[i] < -1 || parent[i] >= i) return -2;
        for (int w = 0; w < words; ++w) anc[(size_t)i * words + w] = 0u;
        for (int a = i; a >= 0; a = parent[a]) {
            if (a / 32 >= words) return -1;
            anc[(size_t)i * words + a / 32] |= 1u << (a % 32);
        }
    }
    return 0;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------
 * KV commit (App. C, "Acceptance": the cache is reordered and cropped so that it holds the shared
 * prefix followed only by the accepted path).  Sequence position L + j takes the row of position
 * L + path[j] for j < n_acc, in every layer, for K and for V alike; positions from L + n_acc on are
 * dead afterwards.  Written as the definition: the accepted rows are first copied out, then written
 * back, so the order of the moves cannot matter.
 * cache: [layers][layer_stride bytes]; position p of a layer lives at byte offset
 *     p * row_bytes                                                  if block_table == NULL,
 *     (block_table[p / page] * page + p % page) * row_bytes          otherwise.
 * Returns the new length L + n_acc, or -1 on bad arguments.
 * ---------------------------------------------------------------------------------------- */
long long orc_kv_commit(unsigned char *cache, int layers, long long layer_stride, int L, int M, int row_bytes,
                        const int32_t *path, int n_acc, const int32_t *block_table, int page)
{
    if (layers < 0 || L < 0 || M < 0 || row_bytes < 1 || n_acc < 0 || n_acc > M) return -1;
    for (int j = 0; j < n_acc; ++j)
        if (path[j] < 0 || path[j] >= M) return -1;
    unsigned char *tmp = (unsigned char *)malloc((size_t)(n_acc > 0 ? n_acc : 1) * (size_t)row_bytes);
    for (int l = 0; l < layers; ++l) {
        unsigned char *base = cache + (size_t)l * (size_t)layer_stride;
        for (int j = 0; j < n_acc; ++j)
            memcpy(tmp + (size_t)j * row_bytes, base + phys_row(L + path[j], block_table, page) * (size_t)row_bytes,
                   (size_t)row_bytes);
        for (int j = 0; j < n_acc; ++j)
            memcpy(base + phys_row(L + j, block_table, page) * (size_t)row_bytes, tmp + (size_t)j * row_bytes,
                   (size_t)row_bytes);
    }
    free(tmp);
    return (long long)L + n_acc;
}
