/*
 * radar_oracle.c -- TEST INFRASTRUCTURE, not the product.
 *
 * A plain, slow, host-only statement of what the RADAR speculative-sampling hot
 * path computes, written from the paper (arXiv 2512.14069) so that the HIP
 * library can be checked against it.  Nothing in the product path may call,
 * link or import this file; only tests, the smoke check and the benchmark's
 * cpu_baseline leg do.  It shares no code, header, table or helper with the
 * HIP sources.
 *
 * Arithmetic: inputs are what the device sees (bf16 for attention operands,
 * fp32 for logits, scores and uniforms); every sum, exp and log is taken in
 * fp64 and results are rounded once to the output type (bf16 round-to-nearest-
 * even for attention, fp32 for scores).  Order comparisons between raw logits
 * are exact fp32 comparisons.
 *
 * The paper states the operations in words and formulas only (it prints no listing
 * and no worked numbers), so each function below is the plain definition of
 * the sentence it cites:
 *   - tree attention: Sec. 1 and Sec. 3 (the serialized tree is checked by the
 *     target in one forward pass whose attention is masked by the tree);
 *   - draft expansion: Sec. 2.3 (confidence scores as proxy, reordering and
 *     pruning) and App. A.1 (k tokens -> k*k candidates -> top-k confidences);
 *   - acceptance: Sec. 3, Eq. 1 (accept probability) and Eq. 2 (residual),
 *     with the tree form implied by Sec. 4.3, Eq. 11-13;
 *   - acceptance-length distribution: Sec. 4.3, Eq. 11-13 written out;
 *   - prediction-model step: Sec. 4.2 with the architecture of App. A.3 (the
 *     standard LSTM cell, pinned to a library LSTM in tests/test_oracle_policy.py).
 * Parity pins: tests/test_oracle_*.py (brute force, closed forms, invariants,
 * library routines).  Fidelity to the authors' unpublished code for the points
 * the paper leaves open (root is node 0, pool contents, serialized order,
 * multi-child rejection rule) is "parity unpinned": pinned to the stated
 * readings only.
 *
 * Loops over independent units carry OpenMP pragmas; they do not change any
 * result (each unit is computed by one thread with the same serial code).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_ARG -1
#define ORACLE_BAD_TREE -2

/* ------------------------------------------------------------------ helpers */

static double bf16_to_double(uint16_t h)
{
    uint32_t bits = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* fp64 -> bf16, round to nearest, ties to even, done on the exact value
 * (not via an intermediate fp32 rounding). */
static uint16_t double_to_bf16(double x)
{
    if (isnan(x)) return 0x7fc0;
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    if (isinf(a)) return sign | 0x7f80;
    if (a == 0.0) return sign;
    int e;
    double m = frexp(a, &e);          /* a = m * 2^e, m in [0.5,1) */
    int E = e - 1;                    /* a = (2m) * 2^E, 2m in [1,2) */
    if (E < -126) E = -126;           /* subnormal range: fixed exponent */
    /* mantissa step of bf16 at exponent E is 2^(E-7) */
    double q = ldexp(a, 7 - E);       /* a / step */
    double r = nearbyint(q);          /* default rounding mode: ties to even */
    (void)m;
    double v = ldexp(r, E - 7);
    if (v >= ldexp(1.0, 128)) return sign | 0x7f80;
    float f = (float)v;               /* exact: v has <= 8 significant bits */
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    return (uint16_t)(bits >> 16) | sign;
}

int radar_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void radar_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

uint16_t radar_oracle_round_bf16(double x) { return double_to_bf16(x); }

/* --------------------------------------------------------- tree attention
 *
 * Sec. 1 / Sec. 3: the draft tree is laid out as a sequence and verified in
 * one target pass with masked attention.  Node i of sequence b may look at
 *   - every prefix position 0 .. ctx_lens[b]-1 of the KV cache, and
 *   - the cache rows of itself and of its ancestors (cache row ctx_lens[b]+a
 *     holds tree node a), found by following parents[] up to the root (-1).
 * Query head h uses KV head h / (Hq/Hkv).
 *
 * q, out      : bf16 [B][T][Hq][D]
 * k_cache, v_cache : bf16 [B][Hkv][S][D]
 * parents     : i32 [B][T], parents[b][0] = -1, 0 <= parents[b][i] < i
 * ctx_lens    : i32 [B];  n_nodes : i32 [B] or NULL (= T for every b)
 * lse_out     : f32 [B][T][Hq] or NULL (natural-log sum of exp of scaled scores)
 * Rows i >= n_nodes[b] of out are zero and of lse_out are 0.
 */
int radar_oracle_tree_attention(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache,
                                const int32_t *parents, const int32_t *ctx_lens, const int32_t *n_nodes,
                                uint16_t *out, float *lse_out,
                                int B, int T, int Hq, int Hkv, int D, int S, float scale)
{
    if (B < 0 || T < 1 || Hq < 1 || Hkv < 1 || D < 1 || S < 1 || Hq % Hkv != 0) return ORACLE_BAD_ARG;
    const int G = Hq / Hkv;
    int status = ORACLE_OK;

    for (int b = 0; b < B; ++b) {
        int nn = n_nodes ? n_nodes[b] : T;
        int L = ctx_lens[b];
        if (nn < 0 || nn > T || L < 0 || L + nn > S) return ORACLE_BAD_ARG;
        for (int i = 0; i < nn; ++i) {
            int p = parents[(size_t)b * T + i];
            if (!((i == 0 && p == -1) || (i > 0 && p >= 0 && p < i))) return ORACLE_BAD_TREE;
        }
    }

#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int ih = 0; ih < T * Hq; ++ih) {
            const int i = ih / Hq, h = ih % Hq;
            const int nn = n_nodes ? n_nodes[b] : T;
            const int L = ctx_lens[b];
            uint16_t *o = out + (((size_t)b * T + i) * Hq + h) * D;
            if (i >= nn) {
                for (int d = 0; d < D; ++d) o[d] = 0;
                if (lse_out) lse_out[((size_t)b * T + i) * Hq + h] = 0.0f;
                continue;
            }
            /* allowed key rows: prefix, then self and ancestors */
            int nkeys = L;
            int *rows = (int *)malloc(sizeof(int) * (size_t)(L + T));
            double *s = (double *)malloc(sizeof(double) * (size_t)(L + T));
            double *acc = (double *)calloc((size_t)D, sizeof(double));
            for (int j = 0; j < L; ++j) rows[j] = j;
            for (int a = i; a >= 0; a = parents[(size_t)b * T + a]) rows[nkeys++] = L + a;

            const uint16_t *qv = q + (((size_t)b * T + i) * Hq + h) * D;
            const uint16_t *kb = k_cache + ((size_t)b * Hkv + h / G) * (size_t)S * D;
            const uint16_t *vb = v_cache + ((size_t)b * Hkv + h / G) * (size_t)S * D;

            double m = -INFINITY;
            for (int j = 0; j < nkeys; ++j) {
                const uint16_t *kr = kb + (size_t)rows[j] * D;
                double dot = 0.0;
                for (int d = 0; d < D; ++d) dot += bf16_to_double(qv[d]) * bf16_to_double(kr[d]);
                s[j] = (double)scale * dot;
                if (s[j] > m) m = s[j];
            }
            double denom = 0.0;
            for (int j = 0; j < nkeys; ++j) {
                double w = exp(s[j] - m);
                denom += w;
                const uint16_t *vr = vb + (size_t)rows[j] * D;
                for (int d = 0; d < D; ++d) acc[d] += w * bf16_to_double(vr[d]);
            }
            for (int d = 0; d < D; ++d) o[d] = double_to_bf16(acc[d] / denom);
            if (lse_out) lse_out[((size_t)b * T + i) * Hq + h] = (float)(m + log(denom));
            free(rows); free(s); free(acc);
        }
    }
    return status;
}

/* ------------------------------------------------------------ row helpers */

/* total order used for every selection: larger value first, then lower index */
static int better(float va, int ia, float vb, int ib)
{
    return (va > vb) || (va == vb && ia < ib);
}

/* natural-log sum of exp of x[0..V) * inv_temp, in fp64 */
static double row_lse(const float *x, int V, double inv_temp)
{
    double m = -INFINITY;
    for (int v = 0; v < V; ++v) if ((double)x[v] * inv_temp > m) m = (double)x[v] * inv_temp;
    double sum = 0.0;
    for (int v = 0; v < V; ++v) sum += exp((double)x[v] * inv_temp - m);
    return m + log(sum);
}

static int row_argmax(const float *x, int V)
{
    int best = 0;
    for (int v = 1; v < V; ++v) if (better(x[v], v, x[best], best)) best = v;
    return best;
}

/* --------------------------------------------------------- draft expansion
 *
 * App. A.1: one draft call turns each of the F frontier nodes into k candidate
 * children (its k most likely next tokens); of the F*k candidates the k with
 * the highest confidence become the next frontier, and their confidences are
 * what the prediction model sees (Sec. 4.2, Eq. 3: k scores in [0,1]).
 * Sec. 2.3: confidence stands in for acceptance probability and is what the
 * tree is later reordered and pruned by.  Confidence of a node is the product
 * of the draft probabilities along its path, kept as a sum of logs:
 *   cum(child) = parent_scores[f] + (logit - logsumexp(row f)).
 *
 * logits        : f32 [F][V]
 * parent_scores : f32 [F]   cumulative log-prob of each frontier node
 * parent_pool_idx : i32 [F] pool index of each frontier node (-1 = tree root)
 * Outputs (candidate c = f*k + r, r-th best token of row f):
 *   cand_tokens i32 [F*k], cand_scores f32 [F*k]
 *   frontier_pool_idx / frontier_tokens / frontier_scores / frontier_conf [k]:
 *     the min(k, F*k) best candidates by (score desc, candidate index asc);
 *     conf = exp(score)
 *   pool_*[pool_count + c] = (token, score, parent_pool_idx[f]) for every c.
 */
int radar_oracle_draft_expand(const float *logits, const float *parent_scores, const int32_t *parent_pool_idx,
                              int F, int V, int k, int pool_count, int pool_capacity,
                              int32_t *cand_tokens, float *cand_scores,
                              int32_t *frontier_pool_idx, int32_t *frontier_tokens,
                              float *frontier_scores, float *frontier_conf,
                              int32_t *pool_tokens, float *pool_scores, int32_t *pool_parents)
{
    if (F < 1 || V < 1 || k < 1 || k > V || pool_count < 0 || pool_count + F * k > pool_capacity)
        return ORACLE_BAD_ARG;

#pragma omp parallel for schedule(dynamic)
    for (int f = 0; f < F; ++f) {
        const float *x = logits + (size_t)f * V;
        const double lse = row_lse(x, V, 1.0);
        unsigned char *taken = (unsigned char *)calloc((size_t)V, 1);
        for (int r = 0; r < k; ++r) {
            int best = -1;
            for (int v = 0; v < V; ++v) {
                if (taken[v]) continue;
                if (best < 0 || better(x[v], v, x[best], best)) best = v;
            }
            taken[best] = 1;
            cand_tokens[f * k + r] = best;
            cand_scores[f * k + r] = (float)((double)parent_scores[f] + ((double)x[best] - lse));
        }
        free(taken);
    }

    const int C = F * k;
    for (int c = 0; c < C; ++c) {
        pool_tokens[pool_count + c] = cand_tokens[c];
        pool_scores[pool_count + c] = cand_scores[c];
        pool_parents[pool_count + c] = parent_pool_idx[c / k];
    }

    unsigned char *used = (unsigned char *)calloc((size_t)C, 1);
    for (int r = 0; r < k; ++r) {
        int best = -1;
        for (int c = 0; c < C; ++c) {
            if (used[c]) continue;
            if (best < 0 || better(cand_scores[c], c, cand_scores[best], best)) best = c;
        }
        if (best < 0) { /* fewer than k candidates cannot happen (C >= k) */
            free(used);
            return ORACLE_BAD_ARG;
        }
        used[best] = 1;
        frontier_pool_idx[r] = pool_count + best;
        frontier_tokens[r] = cand_tokens[best];
        frontier_scores[r] = cand_scores[best];
        frontier_conf[r] = (float)exp((double)cand_scores[best]);
    }
    free(used);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ rerank
 *
 * Sec. 1 / Sec. 2.3 (dynamic trees are reordered and pruned by confidence): once drafting stops, the
 * candidates gathered over all draft calls are ordered by confidence and only
 * the best N are kept; together with the root they form the tree the target
 * verifies.  Order: (score desc, pool index asc).  Node 0 is the root
 * (token root_token, score 0, depth 0, parent -1); the candidate of rank r is
 * node 1+r.  A pool parent of -1 maps to node 0.  Because a child's score never
 * exceeds its parent's and the parent was created first, a kept node's parent
 * is kept and precedes it; if the input breaks that, ORACLE_BAD_TREE.
 *
 * Outputs sized N+1: tree_tokens, tree_parents, tree_scores, tree_depth,
 * tree_pool_idx (pool index a node came from, -1 for the root); *n_nodes_out =
 * 1 + min(N, pool_count).  Entries past n_nodes are token -1, parent -1,
 * score 0, depth 0, pool_idx -1.
 */
int radar_oracle_draft_rerank(const int32_t *pool_tokens, const float *pool_scores, const int32_t *pool_parents,
                              int pool_count, int N, int32_t root_token,
                              int32_t *tree_tokens, int32_t *tree_parents, float *tree_scores,
                              int32_t *tree_depth, int32_t *tree_pool_idx, int32_t *n_nodes_out)
{
    if (pool_count < 0 || N < 0) return ORACLE_BAD_ARG;
    const int keep = pool_count < N ? pool_count : N;
    for (int i = 0; i <= N; ++i) {
        tree_tokens[i] = -1; tree_parents[i] = -1; tree_scores[i] = 0.0f; tree_depth[i] = 0; tree_pool_idx[i] = -1;
    }
    tree_tokens[0] = root_token;
    *n_nodes_out = 1 + keep;

    unsigned char *used = (unsigned char *)calloc((size_t)(pool_count > 0 ? pool_count : 1), 1);
    int *node_of = (int *)malloc(sizeof(int) * (size_t)(pool_count > 0 ? pool_count : 1));
    for (int c = 0; c < pool_count; ++c) node_of[c] = -1;
    int status = ORACLE_OK;
    for (int r = 0; r < keep; ++r) {
        int best = -1;
        for (int c = 0; c < pool_count; ++c) {
            if (used[c]) continue;
            if (best < 0 || better(pool_scores[c], c, pool_scores[best], best)) best = c;
        }
        used[best] = 1;
        node_of[best] = 1 + r;
        tree_tokens[1 + r] = pool_tokens[best];
        tree_scores[1 + r] = pool_scores[best];
        tree_pool_idx[1 + r] = best;
        int pp = pool_parents[best];
        int pn = (pp < 0) ? 0 : ((pp < pool_count) ? node_of[pp] : -1);
        if (pn < 0 || pn >= 1 + r) { status = ORACLE_BAD_TREE; break; }   /* parent missing, itself, or ranked later */
        tree_parents[1 + r] = pn;
        tree_depth[1 + r] = tree_depth[pn] + 1;
    }
    free(used); free(node_of);
    return status;
}

/* ------------------------------------------------------------- acceptance
 *
 * Row r of target_logits is the target model's next-token distribution after
 * the path ending in node r (row 0: after the root).  The walk starts at the
 * root, which is always kept.
 *
 * mode 0 (greedy; the temperature-0 setting of App. Table 7): descend to the
 * child whose token equals the argmax of the current row (lowest index among
 * equal logits); stop when no child matches.  bonus = argmax of the last row.
 *
 * mode 1 (Sec. 3, Eq. 1-2, "strict speculative sampling"): p = softmax(row /
 * temperature).  The children of a node are fixed tokens (the draft's top-k),
 * i.e. each proposal is a point mass, so Eq. 1 gives accept probability
 * p'(tok) under the current residual p', and Eq. 2's residual after a
 * rejection is p' with tok removed and renormalised.  With R the mass of the
 * children rejected so far this reads: child c (ascending node index) is
 * accepted iff uniforms[c] < p(tok_c) / (1 - R); otherwise R += p(tok_c).
 * This makes "accept child j" disjoint events of probability p(tok_j), which
 * is the additive P_rej = 1 - sum_j P_acc(l_j | v) of Eq. 13.  When no child
 * is accepted (or the node is a leaf, R = 0) the bonus token is drawn from the
 * residual by inverse CDF with uniforms[T]: the smallest v, not a rejected
 * child token, whose running residual mass exceeds uniforms[T] * (1 - R).
 * Sec. 3: every cycle emits the accepted tokens plus this one.
 *
 * target_logits f32 [B][T][V]; draft_tokens, parents i32 [B][T];
 * n_nodes i32 [B] or NULL; uniforms f32 [B][T+1] (mode 1).
 * accept_len i32 [B] (# accepted draft nodes, root not counted);
 * accept_path i32 [B][D_max+1]: node indices from the root, padded with -1;
 * bonus_token i32 [B].  A path longer than D_max is ORACLE_BAD_ARG.
 */
int radar_oracle_verify_accept(const float *target_logits, const int32_t *draft_tokens, const int32_t *parents,
                               const int32_t *n_nodes, const float *uniforms,
                               int B, int T, int V, int D_max, int mode, float temperature,
                               int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token)
{
    if (B < 0 || T < 1 || V < 1 || D_max < 0 || (mode != 0 && mode != 1)) return ORACLE_BAD_ARG;
    if (mode == 1 && (!(temperature > 0.0f) || uniforms == NULL)) return ORACLE_BAD_ARG;
    int status = ORACLE_OK;

#pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        const int nn = n_nodes ? n_nodes[b] : T;
        const int32_t *par = parents + (size_t)b * T;
        const int32_t *tok = draft_tokens + (size_t)b * T;
        int32_t *path = accept_path + (size_t)b * (D_max + 1);
        for (int d = 0; d <= D_max; ++d) path[d] = -1;
        accept_len[b] = 0;
        bonus_token[b] = -1;
        if (nn < 1 || nn > T) { status = ORACLE_BAD_ARG; continue; }

        int cur = 0, len = 0;
        path[0] = 0;
        if (mode == 0) {
            for (;;) {
                const float *x = target_logits + ((size_t)b * T + cur) * V;
                const int want = row_argmax(x, V);
                int next = -1;
                for (int c = cur + 1; c < nn; ++c)
                    if (par[c] == cur && tok[c] == want) { next = c; break; }
                if (next < 0) { bonus_token[b] = want; break; }
                if (len + 1 > D_max) { status = ORACLE_BAD_ARG; break; }
                cur = next; path[++len] = cur;
            }
        } else {
            const double inv_t = 1.0 / (double)temperature;
            const float *u = uniforms + (size_t)b * (T + 1);
            unsigned char *rejected = (unsigned char *)calloc((size_t)V, 1);
            for (;;) {
                const float *x = target_logits + ((size_t)b * T + cur) * V;
                const double lse = row_lse(x, V, inv_t);
                double R = 0.0;
                int next = -1;
                memset(rejected, 0, (size_t)V);
                for (int c = cur + 1; c < nn; ++c) {
                    if (par[c] != cur) continue;
                    if (rejected[tok[c]]) continue;          /* repeated sibling token: already refused */
                    const double pc = exp((double)x[tok[c]] * inv_t - lse);
                    if ((double)u[c] * (1.0 - R) < pc) { next = c; break; }
                    R += pc;
                    rejected[tok[c]] = 1;
                }
                if (next >= 0) {
                    if (len + 1 > D_max) { status = ORACLE_BAD_ARG; break; }
                    cur = next; path[++len] = cur;
                    continue;
                }
                /* residual draw */
                const double target = (double)u[T] * (1.0 - R);
                double cdf = 0.0;
                int pick = -1, last_pos = -1;
                for (int v = 0; v < V; ++v) {
                    if (rejected[v]) continue;
                    const double pv = exp((double)x[v] * inv_t - lse);
                    if (pv > 0.0) last_pos = v;
                    cdf += pv;
                    if (cdf > target) { pick = v; break; }
                }
                bonus_token[b] = pick >= 0 ? pick : last_pos;
                break;
            }
            free(rejected);
        }
        accept_len[b] = len;
    }
    return status;
}

/* ---------------------------------------------- acceptance-length distribution
 *
 * Sec. 4.3, Eq. 11-13: the distribution of the acceptance length of one draft
 * tree under the sampling rule above, without drawing anything.  With
 * P_acc(child | parent) = p_parent(token of child) (children are fixed tokens,
 * see mode 1 above):
 *   reach(root) = 1,  reach(v) = reach(parent) * p_parent(tok_v)
 *   P_stop(v)   = reach(v) * (1 - sum over children c of p_v(tok_c))      (Eq. 12-13)
 *   dist[i]     = sum of P_stop(v) over the nodes v of depth i            (Eq. 11)
 * A child whose token repeats an earlier sibling's is never reached (reach 0)
 * and takes no mass from its parent.  Nodes at depth D_max stop with all the
 * mass that reaches them; deeper nodes are never reached (the walk is cut
 * there, as in radar_oracle_verify_accept).
 *
 * dist f64 [B][D_max+1]; every row sums to 1.
 */
int radar_oracle_accept_length_distribution(const float *target_logits, const int32_t *draft_tokens,
                                            const int32_t *parents, const int32_t *n_nodes,
                                            int B, int T, int V, int D_max, float temperature, double *dist)
{
    if (B < 0 || T < 1 || V < 1 || D_max < 0 || !(temperature > 0.0f)) return ORACLE_BAD_ARG;
    int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        const int nn = n_nodes ? n_nodes[b] : T;
        const int32_t *par = parents + (size_t)b * T;
        const int32_t *tok = draft_tokens + (size_t)b * T;
        double *out = dist + (size_t)b * (D_max + 1);
        for (int d = 0; d <= D_max; ++d) out[d] = 0.0;
        if (nn < 1 || nn > T) { status = ORACLE_BAD_ARG; continue; }
        const double inv_t = 1.0 / (double)temperature;
        double *reach = (double *)calloc((size_t)nn, sizeof(double));
        double *kids = (double *)calloc((size_t)nn, sizeof(double));     /* mass handed to children */
        int *depth = (int *)calloc((size_t)nn, sizeof(int));
        reach[0] = 1.0;
        for (int v = 1; v < nn; ++v) {
            const int p = par[v];
            if (p < 0 || p >= v) { status = ORACLE_BAD_TREE; continue; }
            depth[v] = depth[p] + 1;
            if (depth[v] > D_max || tok[v] < 0 || tok[v] >= V) continue;          /* never reached */
            int dup = 0;
            for (int o = p + 1; o < v; ++o) dup |= (par[o] == p && tok[o] == tok[v]);
            if (dup) continue;
            const float *x = target_logits + ((size_t)b * T + p) * V;
            const double pc = exp((double)x[tok[v]] * inv_t - row_lse(x, V, inv_t));
            reach[v] = reach[p] * pc;
            kids[p] += pc;
        }
        for (int v = 0; v < nn; ++v) {
            if (depth[v] > D_max) continue;
            double stay = 1.0 - kids[v];
            if (stay < 0.0) stay = 0.0;
            out[depth[v]] += reach[v] * stay;
        }
        free(reach); free(kids); free(depth);
    }
    return status;
}

/* Margins that tell a test whether a sampling-mode case is decided far from
 * a rounding boundary (so that an fp32 device path must take the same
 * decisions).  For sequence b, walking exactly as above:
 *   margins[2b]   = min over tried children of |u[c]*(1-R) - p(tok_c)|
 *   margins[2b+1] = min(|cdf(pick) - target|, |cdf(pick) - p(pick) - target|)
 * Both are +inf when nothing of that kind was evaluated.
 */
int radar_oracle_accept_margins(const float *target_logits, const int32_t *draft_tokens, const int32_t *parents,
                                const int32_t *n_nodes, const float *uniforms,
                                int B, int T, int V, float temperature, double *margins)
{
    if (!(temperature > 0.0f) || uniforms == NULL) return ORACLE_BAD_ARG;
    for (int b = 0; b < B; ++b) {
        const int nn = n_nodes ? n_nodes[b] : T;
        const int32_t *par = parents + (size_t)b * T;
        const int32_t *tok = draft_tokens + (size_t)b * T;
        const double inv_t = 1.0 / (double)temperature;
        const float *u = uniforms + (size_t)b * (T + 1);
        unsigned char *rejected = (unsigned char *)calloc((size_t)V, 1);
        double m_acc = INFINITY, m_cdf = INFINITY;
        int cur = 0;
        for (;;) {
            const float *x = target_logits + ((size_t)b * T + cur) * V;
            const double lse = row_lse(x, V, inv_t);
            double R = 0.0;
            int next = -1;
            memset(rejected, 0, (size_t)V);
            for (int c = cur + 1; c < nn; ++c) {
                if (par[c] != cur || rejected[tok[c]]) continue;
                const double pc = exp((double)x[tok[c]] * inv_t - lse);
                const double gap = fabs((double)u[c] * (1.0 - R) - pc);
                if (gap < m_acc) m_acc = gap;
                if ((double)u[c] * (1.0 - R) < pc) { next = c; break; }
                R += pc;
                rejected[tok[c]] = 1;
            }
            if (next >= 0) { cur = next; continue; }
            const double target = (double)u[T] * (1.0 - R);
            double cdf = 0.0;
            for (int v = 0; v < V; ++v) {
                if (rejected[v]) continue;
                const double pv = exp((double)x[v] * inv_t - lse);
                cdf += pv;
                if (cdf > target) {
                    double g1 = fabs(cdf - target), g0 = fabs(cdf - pv - target);
                    m_cdf = g1 < g0 ? g1 : g0;
                    break;
                }
            }
            break;
        }
        free(rejected);
        margins[2 * b] = m_acc;
        margins[2 * b + 1] = m_cdf;
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------- prediction-model step */

static double sigmoid_d(double x) { return 1.0 / (1.0 + exp(-x)); }

/* One call of the prediction model (Sec. 4.2; architecture per App. A.3): a
 * single-layer LSTM cell over the k confidences, whose new hidden vector is
 * joined with those same k inputs and passed through a two-layer perceptron
 * (ReLU between the layers) to two logits; softmax gives the probability of
 * action 0 (stop drafting) and action 1 (call the draft model again), Eq. 5.
 * The state (h, c) starts at zero at the first draft step of a cycle and is
 * handed from call to call.
 *
 * The paper names the parts but not the cell's equations or a parameter
 * layout; this is the standard LSTM cell
 *     i = sigm(Wi x + Ui h + bi + di)   f = sigm(Wf x + Uf h + bf + df)
 *     g = tanh(Wg x + Ug h + bg + dg)   o = sigm(Wo x + Uo h + bo + do)
 *     c' = f*c + i*g                    h' = o * tanh(c')
 * with the four blocks stacked in the order i, f, g, o along the rows of
 * w_ih [4H][k], w_hh [4H][H], b_ih [4H], b_hh [4H] (two bias vectors, added),
 * then  z = relu(w1 [h'; x] + b1),  w1 [M][H+k] with the hidden part first,
 * logits = w2 z + b2,  w2 [2][M].  Dropout (training only) is absent.
 *
 * action: with uniforms == NULL, 1 iff logits[1] > logits[0] (a tie stops);
 * otherwise 1 iff uniforms[b] < probs[1] (a draw from the policy, Eq. 5).
 * Parameters and inputs are fp32 values, all arithmetic fp64; h_out, c_out,
 * logits, probs are fp64.  h_in / c_in NULL means the zero state.
 */
int radar_oracle_policy_step(const float *conf, const float *h_in, const float *c_in,
                             const float *w_ih, const float *w_hh, const float *b_ih, const float *b_hh,
                             const float *w1, const float *b1, const float *w2, const float *b2,
                             const float *uniforms, int B, int k, int H, int M,
                             double *h_out, double *c_out, double *logits, double *probs, int32_t *action)
{
    if (B < 0 || k < 1 || H < 1 || M < 1) return ORACLE_BAD_ARG;
    if (!conf || !w_ih || !w_hh || !b_ih || !b_hh || !w1 || !b1 || !w2 || !b2) return ORACLE_BAD_ARG;
    for (int b = 0; b < B; ++b) {
        const float *x = conf + (size_t)b * k;
        double *gate = (double *)calloc((size_t)4 * H, sizeof(double));
        double *hn = (double *)calloc((size_t)H, sizeof(double));
        double *z = (double *)calloc((size_t)M, sizeof(double));
        for (int r = 0; r < 4 * H; ++r) {
            double a = (double)b_ih[r] + (double)b_hh[r];
            for (int j = 0; j < k; ++j) a += (double)w_ih[(size_t)r * k + j] * (double)x[j];
            if (h_in)
                for (int j = 0; j < H; ++j) a += (double)w_hh[(size_t)r * H + j] * (double)h_in[(size_t)b * H + j];
            gate[r] = a;
        }
        for (int u = 0; u < H; ++u) {
            const double ig = sigmoid_d(gate[u]);
            const double fg = sigmoid_d(gate[H + u]);
            const double gg = tanh(gate[2 * H + u]);
            const double og = sigmoid_d(gate[3 * H + u]);
            const double c_prev = c_in ? (double)c_in[(size_t)b * H + u] : 0.0;
            const double cn = fg * c_prev + ig * gg;
            hn[u] = og * tanh(cn);
            if (c_out) c_out[(size_t)b * H + u] = cn;
            if (h_out) h_out[(size_t)b * H + u] = hn[u];
        }
        for (int m = 0; m < M; ++m) {
            double a = (double)b1[m];
            const float *row = w1 + (size_t)m * (H + k);
            for (int j = 0; j < H; ++j) a += (double)row[j] * hn[j];
            for (int j = 0; j < k; ++j) a += (double)row[H + j] * (double)x[j];
            z[m] = a > 0.0 ? a : 0.0;
        }
        double l[2];
        for (int a2 = 0; a2 < 2; ++a2) {
            double a = (double)b2[a2];
            for (int m = 0; m < M; ++m) a += (double)w2[(size_t)a2 * M + m] * z[m];
            l[a2] = a;
        }
        const double mx = l[0] > l[1] ? l[0] : l[1];
        const double e0 = exp(l[0] - mx), e1 = exp(l[1] - mx);
        const double p0 = e0 / (e0 + e1), p1 = e1 / (e0 + e1);
        if (logits) { logits[2 * b] = l[0]; logits[2 * b + 1] = l[1]; }
        if (probs) { probs[2 * b] = p0; probs[2 * b + 1] = p1; }
        if (action) action[b] = uniforms ? ((double)uniforms[b] < p1) : (l[1] > l[0]);
        free(gate); free(hn); free(z);
    }
    return ORACLE_OK;
}

/* ------------------------------------- verification with draft distributions
 *
 * Sec. 3, Eq. 1-2 as printed: every drafted token was DRAWN from a draft
 * distribution q, is accepted with probability min(1, p(x)/q(x)), and after a
 * rejection the target distribution is replaced by the normalised positive part
 * of p - q.  On a tree the rule is applied child by child to the running
 * residual (the paper states the chain; this is the reading for several
 * children, the one that keeps the output distributed exactly as p):
 *
 *   at node v:  r = p_v = softmax(target row v / temperature)
 *   for each child c of v, ascending node index, x = tok_c,
 *       q_c = softmax(draft row q_rows[c] / draft_temperature):
 *       accept c  iff  uniforms[c] * q_c(x) < r(x)        (prob. min(1, r(x)/q_c(x)))
 *       else          r = max(0, r - q_c) / sum_x max(0, r(x) - q_c(x))       (Eq. 2)
 *   none accepted (or a leaf, or depth D_max reached): the bonus token is the
 *   inverse CDF of r at uniforms[T], scanning token ids upwards.
 *
 * The code keeps the unnormalised residual u (r = u / W, W = sum u), so that
 * the test reads uniforms[c] * W * q_c(x) < u(x) and a rejection is
 * u = max(0, u - W q_c).  Should W reach 0 (p fully covered, possible only
 * through rounding) the bonus is drawn from p_v itself.
 *
 * draft_logits f32 [B][Tq][V]; q_rows i32 [B][T] (row of draft_logits for each
 * node; entry 0 unused) or NULL (Tq == T, row c for node c).
 * margins f64 [B][2] or NULL: smallest |uniforms[c] * W * q - u| / (W * max(q, tiny))
 * over the tests taken, i.e. the distance of a uniform from its threshold, and the
 * distance of the bonus draw from the nearest CDF step, relative to W.
 */
int radar_oracle_verify_accept_q(const float *target_logits, const float *draft_logits, const int32_t *q_rows,
                                 const int32_t *draft_tokens, const int32_t *parents, const int32_t *n_nodes,
                                 const float *uniforms, int B, int T, int Tq, int V, int D_max,
                                 float temperature, float draft_temperature,
                                 int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token, double *margins)
{
    if (B < 0 || T < 1 || Tq < 1 || V < 1 || D_max < 0) return ORACLE_BAD_ARG;
    if (!(temperature > 0.0f) || !(draft_temperature > 0.0f) || !uniforms) return ORACLE_BAD_ARG;
    if (!q_rows && Tq != T) return ORACLE_BAD_ARG;
    int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        const int nn = n_nodes ? n_nodes[b] : T;
        const int32_t *par = parents + (size_t)b * T;
        const int32_t *tok = draft_tokens + (size_t)b * T;
        const float *un = uniforms + (size_t)b * (T + 1);
        int32_t *path = accept_path + (size_t)b * (D_max + 1);
        for (int d = 0; d <= D_max; ++d) path[d] = -1;
        accept_len[b] = 0;
        bonus_token[b] = -1;
        double m_acc = INFINITY, m_cdf = INFINITY;
        if (margins) { margins[2 * b] = m_acc; margins[2 * b + 1] = m_cdf; }
        if (nn < 1 || nn > T) { status = ORACLE_BAD_ARG; continue; }
        double *u = (double *)malloc((size_t)V * sizeof(double));
        double *q = (double *)malloc((size_t)V * sizeof(double));
        const double inv_t = 1.0 / (double)temperature, inv_td = 1.0 / (double)draft_temperature;
        int cur = 0, len = 0;
        path[0] = 0;
        for (;;) {
            const float *x = target_logits + ((size_t)b * T + cur) * V;
            const double lse = row_lse(x, V, inv_t);
            for (int t = 0; t < V; ++t) u[t] = exp((double)x[t] * inv_t - lse);
            double W = 1.0;
            int next = -1;
            for (int c = cur + 1; c < nn && len < D_max; ++c) {
                if (par[c] != cur) continue;
                const int xr = tok[c];
                const int row = q_rows ? q_rows[(size_t)b * T + c] : c;
                if (xr < 0 || xr >= V || row < 0 || row >= Tq) { status = ORACLE_BAD_ARG; continue; }
                const float *y = draft_logits + ((size_t)b * Tq + row) * V;
                const double lse_q = row_lse(y, V, inv_td);
                for (int t = 0; t < V; ++t) q[t] = exp((double)y[t] * inv_td - lse_q);
                const double lhs = (double)un[c] * W * q[xr];
                const double denom = W * (q[xr] > 1e-300 ? q[xr] : 1e-300);
                if (fabs(lhs - u[xr]) / denom < m_acc) m_acc = fabs(lhs - u[xr]) / denom;
                if (lhs < u[xr]) { next = c; break; }
                double Wn = 0.0;
                for (int t = 0; t < V; ++t) {
                    const double r = u[t] - W * q[t];
                    u[t] = r > 0.0 ? r : 0.0;
                    Wn += u[t];
                }
                W = Wn;
                if (!(W > 0.0)) break;
            }
            if (next >= 0) { cur = next; path[++len] = cur; continue; }
            if (!(W > 0.0)) {                                  /* covered completely: fall back to p_v */
                for (int t = 0; t < V; ++t) u[t] = exp((double)x[t] * inv_t - lse);
                W = 1.0;
            }
            const double target = (double)un[T] * W;
            double cdf = 0.0;
            int pick = -1, last_pos = -1;
            for (int t = 0; t < V; ++t) {
                if (u[t] > 0.0) last_pos = t;
                const double before = cdf;
                cdf += u[t];
                if (cdf > target) {
                    pick = t;
                    const double d1 = (cdf - target) / W, d0 = (target - before) / W;
                    m_cdf = d1 < d0 ? d1 : d0;
                    break;
                }
            }
            bonus_token[b] = pick >= 0 ? pick : last_pos;
            break;
        }
        accept_len[b] = len;
        if (margins) { margins[2 * b] = m_acc; margins[2 * b + 1] = m_cdf; }
        free(u); free(q);
    }
    return status;
}
