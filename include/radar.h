/*
 * radar.h -- C ABI of the MI355X (gfx950) hot path of RADAR's speculative-
 * sampling loop (arXiv 2512.14069).
 *
 * One decode cycle of the paper's pipeline (Sec. 4.1, App. A.1) runs, on the
 * device, three data-parallel pieces of work that this library provides:
 *
 *   radar_draft_expand   after every draft-model call: vocabulary-wide top-k,
 *                        cumulative log-probability ("confidence") scoring and
 *                        choice of the next frontier (App. A.1; Sec. 4.2 Eq. 3)
 *   radar_draft_rerank   when drafting stops: keep the best N candidates and
 *                        emit the serialized draft tree (Sec. 1, Sec. 2.3)
 *   radar_tree_attention inside every target layer: each tree node attends to
 *                        the prefix KV cache plus its own ancestors (Sec. 1,
 *                        Sec. 3: one parallel target pass over the tree)
 *   radar_verify_accept  after the target pass: greedy or rejection-sampling
 *                        walk down the tree (Sec. 3, Eq. 1-2; Sec. 4.3 Eq. 13)
 * and, around them, radar_policy_step (the prediction model's continue / stop
 * decision after each draft call, Sec. 4.2) and
 * radar_accept_length_distribution (Sec. 4.3, Eq. 11-13).
 *
 * Conventions for every call
 *   - Tensor arguments are DEVICE pointers owned by the caller; descriptors
 *     are HOST structs read during the call; scalars are passed by value.
 *   - A call validates what the host can see, enqueues its kernels on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and returns
 *     without synchronising.  Outputs are valid once the stream has reached
 *     the end of the enqueued work.  A call consists of kernel launches
 *     only, so it may be made on a stream that is being captured into a HIP
 *     graph (radar_workspace_init stays outside the capture; make each entry
 *     point's first call on a device outside a capture as well: it sets the
 *     kernels' launch attributes).
 *   - No call allocates or frees memory.  Scratch memory is a caller-owned
 *     device workspace whose size the matching *_workspace_bytes query gives.
 *     A workspace must be passed once through radar_workspace_init before its
 *     first use (it holds arrival counters that the kernels leave zeroed
 *     again); it may then be reused by any number of calls of the SAME entry
 *     point with the SAME descriptor on ONE stream.  Where the counters sit
 *     depends on the entry point and on the shape, so a workspace that goes
 *     over to another entry point or another descriptor is passed through
 *     radar_workspace_init again first.  Calls that share a workspace on
 *     different streams race.
 *   - Return value: RADAR_OK or a negative radar_status.  Nothing is printed,
 *     thrown or aborted.  On an error no kernel has been launched.
 *   - Device data is not validated (that would need a synchronisation).  The
 *     kernels stay in bounds and terminate for any content: a parent index
 *     that is not smaller than its child simply ends that node's ancestor
 *     chain; token ids outside [0,V) are not dereferenced.
 *     radar_debug_validate_tree checks a parent array on request.
 *
 * Tree convention (the paper leaves it open): a serialized tree has T_max row
 * slots per sequence of which the first n_nodes[b] are used; node 0 is the
 * root, i.e. the token the target produced last ("can" in App. A.1), with
 * parents[0] = -1; for i > 0, 0 <= parents[i] < i.
 */
#ifndef RADAR_H
#define RADAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t radar_status;
#define RADAR_OK                    0
#define RADAR_INVALID_ARG          -1   /* null pointer, non-positive size, inconsistent sizes   */
#define RADAR_UNSUPPORTED_SHAPE    -2   /* outside the compiled limits listed at each call      */
#define RADAR_WORKSPACE_TOO_SMALL  -3
#define RADAR_HIP_ERROR            -4   /* a HIP runtime call failed (launch, attribute query)  */

#define RADAR_T_MAX        64    /* most tree rows per sequence (one 64-bit ancestor word)  */
#define RADAR_K_MAX        16    /* largest branching factor k                              */
#define RADAR_F_MAX        64    /* most frontier rows per expand call                      */
#define RADAR_POOL_MAX   4096    /* most pooled candidates radar_draft_rerank accepts       */

/* Text for a status code; never NULL; static storage. */
const char *radar_status_string(radar_status status);

/* Library version: major * 10000 + minor * 100 + patch. */
int radar_version(void);

/* Zero a workspace before its first use.  `bytes` is the full size that was
 * allocated (what the *_workspace_bytes query returned, or more; at least 4096).
 * Enqueues one kernel. */
radar_status radar_workspace_init(void *workspace, size_t bytes, void *stream);

/* --------------------------------------------------------------------------
 * Tree-verify attention (Sec. 1 and Sec. 3: the target model checks the whole
 * serialized draft tree in one pass whose attention is masked by the tree).
 *
 * For sequence b, node i < n_nodes[b] and query head h:
 *     out[b,i,h,:] = softmax_j( scale * <q[b,i,h,:], k[b,h/G,j,:]> ) . v[b,h/G,j,:]
 * over cache rows j in [0, ctx_lens[b])  (the prefix)  and  j = ctx_lens[b] + a
 * for a = i and every ancestor a of i (cache row ctx_lens[b]+a holds the key /
 * value of tree node a: the verify pass appends the tree to the cache before
 * attention).  G = Hq / Hkv.  Rotary embedding, if any, is already applied.
 * Inputs and output are bf16, scores / softmax / accumulation fp32.
 * Rows i >= n_nodes[b] of out (and lse) are written as zero.
 *
 * Limits: D in {64, 128}; Hq % Hkv == 0; 1 <= T_max <= RADAR_T_MAX;
 *         ctx_lens[b] + n_nodes[b] <= S_max (caller's contract).
 * Strides are in elements; the innermost (D) axis is contiguous; a stride of
 * 0 means "dense" ([B,T_max,Hq,D] for q / out, [B,Hkv,S_max,D] for caches).
 * All bf16 base pointers and strides must keep rows 16-byte aligned.
 */
typedef struct radar_attn_desc {
    int32_t B, T_max, Hq, Hkv, D, S_max;
    int64_t q_stride_b, q_stride_t, q_stride_h;
    int64_t kv_stride_b, kv_stride_h, kv_stride_s;
    int64_t out_stride_b, out_stride_t, out_stride_h;
    float   softmax_scale;      /* 0 => 1/sqrt(D); must not be negative */
    int32_t keys_per_split;     /* 0 => chosen by the library; else a multiple of 64: cache rows one
                                   workgroup streams before partial results are merged */
} radar_attn_desc;

size_t radar_tree_attention_workspace_bytes(const radar_attn_desc *desc);

/* q, out: bf16 [B,T_max,Hq,D]; k_cache, v_cache: bf16 [B,Hkv,S_max,D];
 * parents: i32 [B,T_max]; ctx_lens: i32 [B]; n_nodes: i32 [B] or NULL (= T_max
 * everywhere); lse_out: f32 [B,T_max,Hq] or NULL (natural-log sum of exp of the
 * scaled scores over the allowed set). */
radar_status radar_tree_attention(const void *q, const void *k_cache, const void *v_cache,
                                  const int32_t *parents, const int32_t *ctx_lens, const int32_t *n_nodes,
                                  void *out, float *lse_out, const radar_attn_desc *desc,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* --------------------------------------------------------------------------
 * Draft expansion, one call per draft-model call (App. A.1; Sec. 2.3).
 *
 * Row f of `logits` is the draft model's output for frontier node f.  For each
 * row the k best tokens under the order (logit descending, token id ascending)
 * become candidate children c = f*k + r with
 *     cand_scores[c] = parent_scores[f] + (logit - logsumexp(row f))
 * i.e. the log of the path's cumulative draft probability.  The k best of the
 * F*k candidates under (score descending, c ascending) are the next frontier;
 * frontier_conf = exp(score) are the k confidences in [0,1] that the paper's
 * prediction model reads (Sec. 4.2, Eq. 3).  Every candidate is appended to
 * the pool at index pool_count + c with its parent's pool index, for the final
 * rerank.  Requires F*k >= k, i.e. always k frontier outputs.
 *
 * Limits: 1 <= F <= RADAR_F_MAX; 1 <= k <= min(RADAR_K_MAX, V);
 *         pool_count + F*k <= pool_capacity.  -inf logits are legal; NaN
 *         logits and rows that are entirely -inf give unspecified results.
 */
typedef struct radar_expand_desc {
    int32_t F, V, k;
    int32_t pool_count;      /* candidates already in the pool (host-tracked: grows by F*k per call) */
    int32_t pool_capacity;   /* length of the three pool arrays */
} radar_expand_desc;

/* One workspace serves every draft call of a cycle: the expansion family
 * (radar_draft_expand, _policy, _cycle, _batch) keeps its arrival counters at
 * fixed places at the head of the workspace and leaves them zero, and rewrites
 * everything else before reading it, so calls with different descriptors (F = 1
 * for the root, then F = k; a growing pool_count) and different members of the
 * family may follow each other on one stream without radar_workspace_init in
 * between, provided the workspace has the size the largest of them asks for
 * and, for radar_draft_expand_batch, B stays the same (sequence b's counters
 * sit where another B keeps other data). */
size_t radar_draft_expand_workspace_bytes(const radar_expand_desc *desc);

/* logits f32 [F,V]; parent_scores f32 [F]; parent_pool_idx i32 [F] (-1 = root);
 * cand_tokens i32 [F*k]; cand_scores f32 [F*k];
 * frontier_pool_idx i32 [k]; frontier_tokens i32 [k]; frontier_scores f32 [k];
 * frontier_conf f32 [k];  pool_tokens i32, pool_scores f32, pool_parents i32
 * [pool_capacity] (entries [pool_count, pool_count+F*k) are written).
 * frontier_scores / frontier_pool_idx may be passed as the next call's
 * parent_scores / parent_pool_idx. */
radar_status radar_draft_expand(const float *logits, const float *parent_scores, const int32_t *parent_pool_idx,
                                int32_t *cand_tokens, float *cand_scores,
                                int32_t *frontier_pool_idx, int32_t *frontier_tokens,
                                float *frontier_scores, float *frontier_conf,
                                int32_t *pool_tokens, float *pool_scores, int32_t *pool_parents,
                                const radar_expand_desc *desc,
                                void *workspace, size_t workspace_bytes, void *stream);

/* radar_draft_expand for callers that cannot allocate or hand over a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels with
 * their scratch memory in a device array that this library holds itself,
 * RADAR_NOALLOC_SCRATCH_BYTES on every GPU it runs on, until the process ends.  Inputs and
 * outputs are the caller's, exactly as for radar_draft_expand; there is no workspace argument
 * and nothing is allocated or freed, by this call or by anything it calls.
 * Limits: those of radar_draft_expand, and radar_draft_expand_workspace_bytes(desc) <=
 * RADAR_NOALLOC_SCRATCH_BYTES (F = 10, V = 128256 needs 0.06 MB; about F * V <= 25 M logits
 * fit), else RADAR_UNSUPPORTED_SHAPE and nothing is launched.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two threads) race and give unspecified results; calls that follow each other on one
 * stream, or are ordered by events, are fine, whatever their shapes.  The stream must belong to
 * the current device.  The first call on a device looks the array up and enqueues one extra
 * fill kernel that clears it; make that call outside a graph capture. */
#define RADAR_NOALLOC_SCRATCH_BYTES (1u << 20)
radar_status radar_draft_expand_noalloc(const float *logits, const float *parent_scores, const int32_t *parent_pool_idx,
                                        int32_t *cand_tokens, float *cand_scores,
                                        int32_t *frontier_pool_idx, int32_t *frontier_tokens,
                                        float *frontier_scores, float *frontier_conf,
                                        int32_t *pool_tokens, float *pool_scores, int32_t *pool_parents,
                                        const radar_expand_desc *desc, void *stream);

/* --------------------------------------------------------------------------
 * Rerank, once per cycle (Sec. 1 / Sec. 2.3: the dynamic tree is reordered
 * and pruned by confidence).
 *
 * Orders the pool by (score descending, pool index ascending), keeps the first
 * min(N, pool_count) and emits the tree to verify: node 0 is the root
 * (root_token, score 0, depth 0, parent -1), the candidate of rank r is node
 * 1+r, parents are re-indexed to node numbers (pool parent -1 => node 0),
 * depth = depth(parent) + 1.  Scores never grow from parent to child, so a kept
 * node's parent is kept and has a smaller node number; should the input break
 * that, the node's parent is written as -2 and its depth as 0.
 * Outputs are N+1 long; slots past n_nodes hold token -1, parent -1, score 0,
 * depth 0, pool_idx -1.  *n_nodes_out (device) = 1 + min(N, pool_count).
 *
 * Limits: 0 <= pool_count <= RADAR_POOL_MAX; 0 <= N < RADAR_T_MAX.
 */
size_t radar_draft_rerank_workspace_bytes(int32_t pool_count, int32_t N);

radar_status radar_draft_rerank(const int32_t *pool_tokens, const float *pool_scores, const int32_t *pool_parents,
                                int32_t pool_count, int32_t N, int32_t root_token,
                                int32_t *tree_tokens, int32_t *tree_parents, float *tree_scores,
                                int32_t *tree_depth, int32_t *tree_pool_idx, int32_t *n_nodes_out,
                                void *workspace, size_t workspace_bytes, void *stream);

/* --------------------------------------------------------------------------
 * Verification walk (Sec. 3, Eq. 1-2; tree form per Sec. 4.3, Eq. 11-13).
 *
 * Row r of target_logits is the target's next-token distribution after the
 * path ending in node r.  Starting at the root:
 *   mode RADAR_ACCEPT_GREEDY   descend to the child whose token is the argmax of
 *       the current row (lowest token id among equal logits, lowest node index
 *       among equal tokens); stop when none matches; bonus = that argmax.
 *   mode RADAR_ACCEPT_SAMPLE   p = softmax(row / temperature).  The children
 *       are fixed tokens (point-mass proposals), so Eq. 1 accepts child c with
 *       the residual probability of its token: visiting children in ascending
 *       node index with R = mass of those already rejected, accept iff
 *       uniforms[b,c] * (1 - R) < p(tok_c), else R += p(tok_c).  If none is
 *       accepted the bonus token is the inverse CDF, at uniforms[b,T_max] *
 *       (1 - R), of p with the rejected tokens removed (Eq. 2), scanning token
 *       ids upwards.  A leaf has R = 0.
 * accept_len[b] = number of accepted draft nodes (root excluded, <= depth);
 * accept_path[b,:] = node indices from the root, padded with -1, D_max+1 long;
 * a walk that would exceed D_max stops there.  bonus_token[b] = the extra token
 * every cycle emits (Sec. 3: between 1 and t+1 tokens per cycle).
 *
 * Limits: 1 <= T_max <= RADAR_T_MAX; 0 <= D_max < RADAR_T_MAX; V >= 1;
 *         temperature > 0 and uniforms != NULL in sampling mode.
 */
#define RADAR_ACCEPT_GREEDY 0
#define RADAR_ACCEPT_SAMPLE 1

typedef struct radar_accept_desc {
    int32_t B, T_max, V, D_max;
    int32_t mode;
    float   temperature;
} radar_accept_desc;

size_t radar_verify_accept_workspace_bytes(const radar_accept_desc *desc);

/* target_logits f32 [B,T_max,V]; draft_tokens, parents i32 [B,T_max];
 * n_nodes i32 [B] or NULL; uniforms f32 [B,T_max+1] or NULL (greedy);
 * accept_len i32 [B]; accept_path i32 [B,D_max+1]; bonus_token i32 [B]. */
radar_status radar_verify_accept(const float *target_logits, const int32_t *draft_tokens, const int32_t *parents,
                                 const int32_t *n_nodes, const float *uniforms,
                                 int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token,
                                 const radar_accept_desc *desc,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* --------------------------------------------------------------------------
 * Acceptance-length distribution of a draft tree (Sec. 4.3, Eq. 11-13): what
 * the walk above would return as accept_len, as a distribution over the
 * uniforms, computed without drawing.  With P_acc(child | parent) =
 * p_parent(token of child), p = softmax(row / temperature):
 *   reach(root) = 1, reach(v) = reach(parent) * p_parent(tok_v);
 *   P_stop(v) = reach(v) * (1 - sum over children c of p_v(tok_c))  (Eq. 12-13);
 *   dist[b,i] = sum of P_stop(v) over nodes of depth i              (Eq. 11).
 * A child that repeats an earlier sibling's token is never reached; nodes at
 * depth D_max keep all the mass that reaches them and deeper nodes get none
 * (the cut radar_verify_accept makes).  Every row of dist sums to 1.
 *
 * dist f64 [B,D_max+1] (device); the other tensors as for radar_verify_accept;
 * desc->mode is ignored, desc->temperature must be > 0.  Workspace: what
 * radar_verify_accept_workspace_bytes(desc) gives; one kernel is enqueued. */
radar_status radar_accept_length_distribution(const float *target_logits, const int32_t *draft_tokens,
                                              const int32_t *parents, const int32_t *n_nodes, double *dist,
                                              const radar_accept_desc *desc,
                                              void *workspace, size_t workspace_bytes, void *stream);

/* --------------------------------------------------------------------------
 * Verification with draft distributions (Sec. 3, Eq. 1-2 as printed): for
 * trees whose tokens were DRAWN from the draft model's distributions rather
 * than picked as its top-k.  With p_v = softmax(target row v / temperature),
 * q_c = softmax(draft row q_rows[c] / draft_temperature) the distribution node
 * c's token was drawn from, and r the running residual at node v (r = p_v at
 * first):
 *   for each child c of v in ascending node index, x = its token:
 *     accept c  iff  uniforms[b,c] * q_c(x) < r(x)          (probability min(1, r(x)/q_c(x)), Eq. 1)
 *     otherwise     r <- max(0, r - q_c), renormalised       (Eq. 2)
 *   when no child is accepted (or v is a leaf, or the walk is D_max deep) the
 *   bonus token is the inverse CDF of r at uniforms[b,T_max], scanning token ids
 *   upwards.  Should the residual vanish (p_v <= the rejected proposals
 *   everywhere, possible only through rounding) the bonus is drawn from p_v.
 * On a chain this is exactly the paper's procedure; for several children it is
 * the recursive form that keeps the emitted tokens distributed as the target's.
 * Children may repeat a token.  Outputs as for radar_verify_accept.
 *
 * target_logits f32 [B,T_max,V]; draft_logits f32 [B,Tq,V]; q_rows i32 [B,T_max]
 * (row of draft_logits per node, entry 0 unused; siblings drawn from one
 * distribution may share a row) or NULL (Tq == T_max, node c uses row c);
 * draft_tokens, parents i32 [B,T_max]; n_nodes i32 [B] or NULL; uniforms f32
 * [B,T_max+1].  Nodes whose token or draft row is out of range are skipped.
 * Limits: T_max <= RADAR_T_MAX; V <= 1048576; B * (T_max + Tq) <= 65535;
 *         both temperatures > 0.  Two or three kernels are enqueued.  The shared walk needs its
 *         B * G workgroups resident together; the library sizes G from the occupancy the runtime
 *         reports for the device (CUs x workgroups per CU) and bounds every wait (about 100 us by
 *         default): where other work keeps some of them from running, the wait ends and the
 *         fall-back described at walk_spin_limit redoes the sequence.  On a GPU that is shared as a
 *         rule, pass walk_spin_limit < 0 (single-workgroup walk, no waiting at all). */
typedef struct radar_accept_q_desc {
    int32_t B, T_max, Tq, V, D_max;
    float   temperature, draft_temperature;
    int32_t walk_spin_limit;    /* 0: the library's choice.  The walk of one sequence is shared by several
                                   workgroups that meet at a counter after every rejection; the wait there is
                                   bounded, and a sequence whose workgroups gave up is redone by a single one
                                   (same results).  > 0: polls (about 0.4 us each) before giving up (tests
                                   pass 1 to force that path; the default is 256); < 0: single-workgroup
                                   walk only */
} radar_accept_q_desc;

size_t radar_verify_accept_q_workspace_bytes(const radar_accept_q_desc *desc);

radar_status radar_verify_accept_q(const float *target_logits, const float *draft_logits, const int32_t *q_rows,
                                   const int32_t *draft_tokens, const int32_t *parents, const int32_t *n_nodes,
                                   const float *uniforms,
                                   int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token,
                                   const radar_accept_q_desc *desc,
                                   void *workspace, size_t workspace_bytes, void *stream);

/* --------------------------------------------------------------------------
 * Prediction-model step (Sec. 4.2, Eq. 3-5; architecture per App. A.3): after a
 * draft-model call, decide from the k frontier confidences whether to call the
 * draft model again.
 *
 * A single-layer LSTM cell reads x = the k confidences (frontier_conf of
 * radar_draft_expand) and the state (h, c); the new hidden vector is joined
 * with x and passed through a two-layer perceptron with ReLU to two logits:
 *     [i f g o] = w_ih x + b_ih + w_hh h + b_hh      (four blocks of H rows, this order)
 *     c' = sigm(f) * c + sigm(i) * tanh(g);   h' = sigm(o) * tanh(c')
 *     logits = w2 relu(w1 [h'; x] + b1) + b2;   probs = softmax(logits)
 * Index 0 is "stop drafting", index 1 "call the draft model again" (Eq. 5).
 * action[b] = 1 iff logits[b,1] > logits[b,0] (a tie stops), or, when uniforms
 * is given, 1 iff uniforms[b] < probs[b,1] (a draw from the policy).
 * The state starts at zero at the first draft step of a cycle (h_in = c_in =
 * NULL) and is handed from call to call; h_out / c_out may be h_in / c_in.
 * Training-time dropout has no counterpart here.  All arithmetic is fp32.
 *
 * Parameters are DEVICE arrays of fp32 in row-major [out, in] order (the
 * layout in which the common deep-learning toolkits keep an LSTM layer and a
 * linear layer, so trained weights can be handed over unchanged):
 *   w_ih [4H,k]  w_hh [4H,H]  b_ih, b_hh [4H]  w1 [M,H+k]  b1 [M]  w2 [2,M]  b2 [2]
 * Limits: H == 128; 1 <= k <= RADAR_K_MAX; 1 <= M <= 128; w_hh, h_in 16-byte aligned.
 * conf f32 [B,k]; h_in, c_in, h_out, c_out f32 [B,H]; logits, probs f32 [B,2];
 * action i32 [B]; uniforms f32 [B] or NULL.  One kernel, no workspace. */
typedef struct radar_policy_params {
    const float *w_ih, *w_hh, *b_ih, *b_hh;   /* LSTM cell   */
    const float *w1, *b1, *w2, *b2;           /* perceptron  */
    int32_t k, H, M;
} radar_policy_params;

radar_status radar_policy_step(const float *conf, const float *h_in, const float *c_in,
                               const radar_policy_params *params, const float *uniforms,
                               float *h_out, float *c_out, float *logits, float *probs, int32_t *action,
                               int32_t B, void *stream);

/* radar_draft_expand followed, in the same launch, by radar_policy_step on the
 * frontier_conf it has just written (batch of one: a drafting loop has one
 * frontier and one policy state).  Results are those of the two calls made one
 * after the other, bit for bit; the second launch and its latency are saved
 * (the paper's T_p, Sec. 4.2 Eq. 8-9, is mostly that).  params->k must equal
 * desc->k.  io is a HOST struct of DEVICE pointers: h_in, c_in f32 [H] or both
 * NULL (zero state); uniform f32 [1] or NULL (argmax action); h_out, c_out f32
 * [H] (may be h_in, c_in); logits, probs f32 [2]; action i32 [1].  Workspace and
 * all other arguments as for radar_draft_expand. */
typedef struct radar_policy_io {
    const float *h_in, *c_in, *uniform;
    float *h_out, *c_out, *logits, *probs;
    int32_t *action;
} radar_policy_io;

radar_status radar_draft_expand_policy(const float *logits, const float *parent_scores, const int32_t *parent_pool_idx,
                                       int32_t *cand_tokens, float *cand_scores,
                                       int32_t *frontier_pool_idx, int32_t *frontier_tokens,
                                       float *frontier_scores, float *frontier_conf,
                                       int32_t *pool_tokens, float *pool_scores, int32_t *pool_parents,
                                       const radar_expand_desc *desc,
                                       const radar_policy_params *params, const radar_policy_io *io,
                                       void *workspace, size_t workspace_bytes, void *stream);

/* --------------------------------------------------------------------------
 * A whole drafting cycle without the host in the loop (Sec. 4.1-4.2: after
 * every draft call the prediction model decides whether another one follows;
 * App. latency table: the decision and its round trip are what T_p pays for).
 *
 * The decision stays on the device: a radar_cycle_state in DEVICE memory holds
 * "stopped", the number of pooled candidates and the number of draft calls
 * made.  The host enqueues the longest cycle it allows (t_max draft calls,
 * Sec. 4.2) once -- directly or captured in a HIP graph -- and never reads a
 * result in between:
 *   radar_cycle_begin          resets the state (one small kernel, no memset);
 *       not needed before a cycle whose first draft call is made through
 *       radar_draft_expand_cycle with desc->pool_count == 0: that call starts
 *       the cycle itself (it ignores what the state holds and writes all of it)
 *   radar_draft_expand_cycle   one draft call's expansion; does NOTHING (every
 *       workgroup leaves at once, no output is touched) when the state says
 *       stopped; otherwise radar_draft_expand with the pool count taken from
 *       the state, followed, when params != NULL, by radar_policy_step on the
 *       new confidences as in radar_draft_expand_policy; then the state's pool
 *       count grows by F*k, steps_done by one, and action 0 sets stopped.
 *       Pass params = io = NULL for the last allowed draft call (no decision
 *       is needed after it).  desc->pool_count is the LARGEST count the state
 *       can hold when this call runs (what it would be had every earlier call
 *       run): the capacity check uses it, and a state outside [0, that] makes
 *       the call a no-op.  With desc->pool_count == 0 the call is the first
 *       of a cycle and always runs.
 *   radar_draft_rerank_cycle   radar_draft_rerank over the candidates the state
 *       counts (at most pool_count_max).
 * Because a skipped call leaves its outputs alone, the frontier arrays chained
 * from call to call still hold the last executed call's values.  All other
 * arguments, limits and the workspace are those of the plain calls. */
typedef struct radar_cycle_state {
    int32_t stopped;        /* 1 once a decision said "stop" */
    int32_t pool_count;     /* candidates pooled so far */
    int32_t steps_done;     /* draft calls whose expansion ran */
    int32_t last_action;    /* last decision (0 stop, 1 continue), -1 before the first */
} radar_cycle_state;

radar_status radar_cycle_begin(radar_cycle_state *state, void *stream);

radar_status radar_draft_expand_cycle(const float *logits, const float *parent_scores, const int32_t *parent_pool_idx,
                                      int32_t *cand_tokens, float *cand_scores,
                                      int32_t *frontier_pool_idx, int32_t *frontier_tokens,
                                      float *frontier_scores, float *frontier_conf,
                                      int32_t *pool_tokens, float *pool_scores, int32_t *pool_parents,
                                      const radar_expand_desc *desc,
                                      const radar_policy_params *params, const radar_policy_io *io,
                                      radar_cycle_state *state,
                                      void *workspace, size_t workspace_bytes, void *stream);

radar_status radar_draft_rerank_cycle(const int32_t *pool_tokens, const float *pool_scores, const int32_t *pool_parents,
                                      const radar_cycle_state *state, int32_t pool_count_max, int32_t N,
                                      int32_t root_token,
                                      int32_t *tree_tokens, int32_t *tree_parents, float *tree_scores,
                                      int32_t *tree_depth, int32_t *tree_pool_idx, int32_t *n_nodes_out,
                                      void *workspace, size_t workspace_bytes, void *stream);

/* --------------------------------------------------------------------------
 * One draft call for B sequences in ONE launch (the batch the other two steps
 * already take; Sec. 4.1-4.2: every sequence runs its own cycle and stops at
 * its own draft call, which is what makes the batch's trees ragged).
 *
 * Sequence b is an independent radar_draft_expand_cycle (states != NULL),
 * radar_draft_expand_policy (states == NULL, params != NULL) or
 * radar_draft_expand (both NULL): same results, same limits.  Every array of
 * those calls gains a leading dimension B, densely packed:
 * logits [B,F,V]; parent_scores, parent_pool_idx [B,F]; cand_* [B,F*k];
 * frontier_* [B,k]; pool_* [B,pool_capacity]; states [B]; and in io: h_in,
 * c_in, h_out, c_out [B,H], uniform [B], logits, probs [B,2], action [B].
 * desc (F, V, k, pool_count, pool_capacity) is shared by all sequences:
 * without states every sequence's pool holds desc->pool_count candidates; with
 * states each holds its own state's count, desc->pool_count being the largest
 * any may have, and a sequence whose state says stopped is skipped (its
 * workgroups leave at once) while the others run.  The model's weights
 * (params) are shared.
 * Small batches are one launch; a batch of at least 4 Mi logits (B*F*V) is
 * two: a streaming kernel over all sequences, then one workgroup per sequence
 * (which also runs the prediction model's step when params != NULL).  Integer results are the same
 * either way; scores may differ in the last bit (the sums are grouped differently).
 * Limits: 1 <= B <= 65535.  The workspace is sized by
 * radar_draft_expand_batch_workspace_bytes(desc, B) (equal to
 * radar_draft_expand_workspace_bytes(desc) for B = 1).
 */
size_t radar_draft_expand_batch_workspace_bytes(const radar_expand_desc *desc, int32_t B);

radar_status radar_draft_expand_batch(const float *logits, const float *parent_scores, const int32_t *parent_pool_idx,
                                      int32_t *cand_tokens, float *cand_scores,
                                      int32_t *frontier_pool_idx, int32_t *frontier_tokens,
                                      float *frontier_scores, float *frontier_conf,
                                      int32_t *pool_tokens, float *pool_scores, int32_t *pool_parents,
                                      const radar_expand_desc *desc, int32_t B,
                                      const radar_policy_params *params, const radar_policy_io *io,
                                      radar_cycle_state *states,
                                      void *workspace, size_t workspace_bytes, void *stream);

/* radar_draft_rerank for B sequences in one launch: pool_* [B,pool_capacity];
 * root_tokens i32 [B]; tree_* [B,N+1]; n_nodes_out i32 [B], i.e. the parents,
 * tokens and n_nodes arrays that radar_tree_attention and radar_verify_accept
 * take for a batch with T_max = N+1.  states == NULL: every pool holds
 * pool_count candidates; states [B]: each holds its own state's count, at most
 * pool_count.  Limits: those of radar_draft_rerank; pool_count <= pool_capacity;
 * 1 <= B <= 65535.  Workspace as for radar_draft_rerank. */
radar_status radar_draft_rerank_batch(const int32_t *pool_tokens, const float *pool_scores, const int32_t *pool_parents,
                                      const radar_cycle_state *states, int32_t pool_count, int32_t pool_capacity,
                                      int32_t B, int32_t N, const int32_t *root_tokens,
                                      int32_t *tree_tokens, int32_t *tree_parents, float *tree_scores,
                                      int32_t *tree_depth, int32_t *tree_pool_idx, int32_t *n_nodes_out,
                                      void *workspace, size_t workspace_bytes, void *stream);

/* Counts, per call, the nodes i < n_nodes[b] whose parent breaks the tree
 * convention; *bad_count_out (device i32) is overwritten.  parents i32
 * [B,T_max]; n_nodes i32 [B] or NULL. */
radar_status radar_debug_validate_tree(const int32_t *parents, const int32_t *n_nodes, int32_t B, int32_t T_max,
                                       int32_t *bad_count_out, void *stream);

/* --------------------------------------------------------------------------
 * Measurement support (not part of the method; for benchmarks that report
 * achieved bandwidth per kernel as the paper's Table 5 reports time per
 * stage).  Between radar_profile_begin and radar_profile_end every kernel the
 * library launches, from any thread, carries a pair of HIP events stamped
 * with the dispatch's own begin and end on the device, i.e. the duration a
 * kernel trace shows, without launch gaps or event overhead.
 *
 * radar_profile_begin(max_launches) creates max_launches event pairs (host
 * objects; 1 <= max_launches <= 2^20) and starts recording; launches beyond
 * that number run unrecorded.  radar_profile_end stops recording, waits for
 * the recorded kernels, writes one entry per kernel name into out[0..capacity)
 * (HOST memory; names beyond capacity are dropped), stores the number of
 * entries in *n_out and destroys the events.  These two calls are the only
 * ones that create or destroy anything and that synchronise.  Neither may
 * run while another thread is inside a call of this library: a launch that
 * has taken its event pair must have been issued before radar_profile_end
 * destroys the events. */
typedef struct radar_kernel_time {
    char name[48];      /* "expand", "expand_stream", "expand_finish", "rerank", "accept",
                           "accept_length_distribution", "tree_attn_group_share",
                           "tree_attn_merge", ... */
    int64_t calls;
    double total_us;
    double min_us;
    double max_us;
} radar_kernel_time;

radar_status radar_profile_begin(int32_t max_launches);
radar_status radar_profile_end(radar_kernel_time *out, int32_t capacity, int32_t *n_out);

/* Measurement support: reads `bytes` (a multiple of 16 is read; src 16-byte aligned, DEVICE
 * memory) once with 16-byte loads from every CU and keeps nothing -- the time a pure streaming
 * read of that size takes on this chip, against which the streaming kernels above (logits
 * passes, KV passes) are priced besides the nominal peak.  sink: DEVICE u32 or NULL, written
 * practically never (it only keeps the loads alive).  One kernel ("hbm_read_probe" in the
 * timing table); enqueues and returns. */
radar_status radar_probe_hbm_read(const void *src, size_t bytes, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RADAR_H */
