/*
 * CPU oracle for tree-verification attention and tree acceptance.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of what
 * the verification pass computes.  It exists so the tests, the smoke check and the
 * benchmark's CPU-baseline leg can compare the GPU library against it.  No product
 * code path may call it, and it shares no code with the GPU library.
 *
 * What it follows:
 *  - Tree attention: the target model validates every path of the draft tree in one
 *    pass under a tree attention mask (paper, Section 2, "tree of candidate tokens");
 *    contemplate rows are extra rows of that tree, one hanging off the node whose
 *    future it predicts (Section 3.1, Figure 4), and only contemplate rows may attend
 *    to the soft-prompt slots prepended to the KV cache (Section 3.1).
 *    The mask is written out from that definition as a dense 0/1 matrix and the
 *    attention is ordinary max-subtracted softmax attention under it.
 *  - Acceptance: draft tokens are checked in order, the first rejected one is
 *    replaced by a token from the target's corrected distribution, and the output law
 *    equals the target model's (Section 2, steps 3-4; Section 5).  The rule is the
 *    speculative-sampling rule of the literature the paper cites there, generalised
 *    to sibling lists; temperature 0 is greedy matching (Section 4).  RULE_SAMPLE_MATCH
 *    is the literal reading of step 3 instead: the target's token is sampled at each node
 *    and a draft child is accepted iff it proposed exactly that token.
 *
 * Every pin of these functions lives in tests/ (closed forms, textbook special
 * cases, brute force, exact enumeration of the output law).  No function here is
 * "parity unpinned".
 *
 * No blocking, fusion or reordering: loops are written in the order of the
 * definition.  OpenMP, when enabled, only distributes independent (row, head)
 * pairs over host threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_BAD_TREE 1
#define ORACLE_BAD_ARG 2
#define ORACLE_NOMEM 3

#define KIND_NODE 0
#define KIND_CONTEMPLATE 1

#define RULE_GREEDY 0
#define RULE_DETERMINISTIC 1
#define RULE_DRAFT_WOR 2
#define RULE_DRAFT_WR 3
#define RULE_SAMPLE_MATCH 4

#define FINAL_BONUS 0
#define FINAL_RESIDUAL 1

/* ---------------------------------------------------------------------------
 * Mask (Section 3.1 and Figure 4 caption; Section 2 tree attention).
 *
 * Query row i may look at new row j exactly when j lies on the chain
 * i, parent[i], parent[parent[i]], ..., root.  A draft node never hangs off a
 * contemplate row (so the nodes' representations are those of plain tree
 * verification).  anc is M x M, row major, anc[i*M + j] in {0,1}.
 * ------------------------------------------------------------------------- */
int oracle_ancestor_matrix(int M, const int32_t* parent, const uint8_t* kind, uint8_t* anc)
{
    if (M < 1 || !parent || !kind || !anc) return ORACLE_BAD_ARG;
    for (int i = 0; i < M; ++i) {
        if (kind[i] != KIND_NODE && kind[i] != KIND_CONTEMPLATE) return ORACLE_BAD_TREE;
        if (parent[i] < -1 || parent[i] >= i) return ORACLE_BAD_TREE;
        if (parent[i] >= 0 && kind[i] == KIND_NODE && kind[parent[i]] == KIND_CONTEMPLATE)
            return ORACLE_BAD_TREE;
    }
    memset(anc, 0, (size_t)M * (size_t)M);
    for (int i = 0; i < M; ++i) {
        int j = i;
        while (j >= 0) {
            anc[(size_t)i * M + j] = 1;
            j = parent[j];
        }
    }
    return ORACLE_OK;
}

/* Full visibility matrix vis[i][k], k over the P cached rows then the M new rows.
 * Cached rows [0, s) are soft-prompt slots: visible to contemplate rows only. */
int oracle_visibility_matrix(int M, int P, int s, const int32_t* parent, const uint8_t* kind,
                             uint8_t* vis /* [M][P+M] */)
{
    if (P < 0 || s < 0 || s > P) return ORACLE_BAD_ARG;
    uint8_t* anc = (uint8_t*)malloc((size_t)M * (size_t)M);
    if (!anc) return ORACLE_NOMEM;
    int rc = oracle_ancestor_matrix(M, parent, kind, anc);
    if (rc != ORACLE_OK) { free(anc); return rc; }
    const size_t L = (size_t)P + (size_t)M;
    for (int i = 0; i < M; ++i) {
        for (int k = 0; k < P; ++k)
            vis[i * L + k] = (uint8_t)((k >= s) || (kind[i] == KIND_CONTEMPLATE));
        for (int j = 0; j < M; ++j)
            vis[i * L + P + j] = anc[(size_t)i * M + j];
    }
    free(anc);
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Dense masked attention for one sequence, fp64.
 *
 *   q   [M][Hq][D]       this step's query rows (after positional encoding)
 *   k,v [P+M][Hkv][D]    cached prefix rows then this step's M new rows
 *   out [M][Hq][D]
 *   lse [Hq][M] or NULL  log-sum-exp of the scaled visible scores
 *
 * Query head h reads KV head h / (Hq / Hkv).
 * out[i,h,:] = sum_{k visible to i} softmax_k(scale * q[i,h].K[k,g]) * V[k,g,:]
 * ------------------------------------------------------------------------- */
int oracle_tree_attention(int M, int Hq, int Hkv, int D, int P, int s, double scale,
                          const double* q, const double* k, const double* v,
                          const int32_t* parent, const uint8_t* kind,
                          double* out, double* lse)
{
    if (M < 1 || Hq < 1 || Hkv < 1 || D < 1 || Hq % Hkv != 0 || !q || !k || !v || !out)
        return ORACLE_BAD_ARG;
    const int G = Hq / Hkv;
    const size_t L = (size_t)P + (size_t)M;
    uint8_t* vis = (uint8_t*)malloc((size_t)M * L);
    if (!vis) return ORACLE_NOMEM;
    int rc = oracle_visibility_matrix(M, P, s, parent, kind, vis);
    if (rc != ORACLE_OK) { free(vis); return rc; }
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel for collapse(2) schedule(static)
#endif
    for (int h = 0; h < Hq; ++h) {
        for (int i = 0; i < M; ++i) {
            double* score = (double*)malloc(L * sizeof(double));
            if (!score) { failed = 1; continue; }
            const int g = h / G;
            const double* qi = q + ((size_t)i * Hq + h) * D;
            double mx = -INFINITY;
            for (size_t t = 0; t < L; ++t) {
                if (!vis[i * L + t]) { score[t] = -INFINITY; continue; }
                const double* kt = k + (t * Hkv + g) * D;
                double dot = 0.0;
                for (int d = 0; d < D; ++d) dot += qi[d] * kt[d];
                score[t] = scale * dot;
                if (score[t] > mx) mx = score[t];
            }
            double denom = 0.0;
            for (size_t t = 0; t < L; ++t) {
                score[t] = vis[i * L + t] ? exp(score[t] - mx) : 0.0;
                denom += score[t];
            }
            double* oi = out + ((size_t)i * Hq + h) * D;
            for (int d = 0; d < D; ++d) oi[d] = 0.0;
            for (size_t t = 0; t < L; ++t) {
                if (!vis[i * L + t]) continue;
                const double w = score[t] / denom;
                const double* vt = v + (t * Hkv + g) * D;
                for (int d = 0; d < D; ++d) oi[d] += w * vt[d];
            }
            if (lse) lse[(size_t)h * M + i] = mx + log(denom);
            free(score);
        }
    }
    free(vis);
    return failed ? ORACLE_NOMEM : ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Tree acceptance for one sequence (Section 2, steps 3-4, applied along the tree).
 * ------------------------------------------------------------------------- */

/* prob[v] = softmax(logits / temp)[v], max-subtracted, fp64 */
static void softmax_row(const float* logits, int V, double temp, double* prob)
{
    double mx = -INFINITY;
    for (int v = 0; v < V; ++v) {
        const double z = (double)logits[v] / temp;
        if (z > mx) mx = z;
    }
    double sum = 0.0;
    for (int v = 0; v < V; ++v) {
        prob[v] = exp((double)logits[v] / temp - mx);
        sum += prob[v];
    }
    for (int v = 0; v < V; ++v) prob[v] /= sum;
}

static int argmax_row(const float* logits, int V)
{
    int best = 0;
    for (int v = 1; v < V; ++v)
        if (logits[v] > logits[best]) best = v;   /* lowest index wins ties */
    return best;
}

/* first v whose running sum exceeds u; if rounding leaves none, the last v with mass */
static int inverse_cdf(const double* prob, int V, double u)
{
    double run = 0.0;
    int last = -1;
    for (int v = 0; v < V; ++v) {
        if (prob[v] > 0.0) last = v;
        run += prob[v];
        if (run > u) return v;
    }
    return last;
}

/*
 *   T, V                number of draft nodes, vocabulary size
 *   temp                sampling temperature (rule GREEDY ignores it)
 *   target_logits [T][V]  target model's next-token logits at each node
 *   draft_logits  [T][V]  draft model's logits at each node (DRAFT_* rules), else NULL
 *   token  [T]          token drafted at each node (token[0]: the root's, already committed)
 *   parent [T]          parent node, -1 for the root, parent[i] < i
 *   uniforms [2T]       uniforms[c] decides node c's test, uniforms[T+n] the final draw at stop node n
 *   con_anchor [C]      node each contemplate row belongs to, or NULL
 * Outputs:
 *   path [T]            accepted node indices, root first; entries past n_accepted are -1
 *   n_accepted          accepted draft tokens (root not counted)
 *   final_token         bonus token (no rejection at the stop node) or residual token
 *   final_kind          FINAL_BONUS / FINAL_RESIDUAL
 *   last_node           last accepted node (= path[n_accepted])
 *   selected_con        first c with con_anchor[c] == last_node, else -1: whose future prediction to keep
 */
int oracle_tree_accept(int T, int V, int C, double temp, int rule,
                       const float* target_logits, const float* draft_logits,
                       const int32_t* token, const int32_t* parent, const float* uniforms,
                       const int32_t* con_anchor,
                       int32_t* path, int32_t* n_accepted, int32_t* final_token,
                       int32_t* final_kind, int32_t* last_node, int32_t* selected_con)
{
    if (T < 1 || V < 1 || !target_logits || !token || !parent || !path || !n_accepted ||
        !final_token || !final_kind || !last_node)
        return ORACLE_BAD_ARG;
    if (rule < RULE_GREEDY || rule > RULE_SAMPLE_MATCH) return ORACLE_BAD_ARG;
    if (rule != RULE_GREEDY && (!(temp > 0.0) || !uniforms)) return ORACLE_BAD_ARG;
    const int use_draft = (rule == RULE_DRAFT_WOR || rule == RULE_DRAFT_WR);
    if (use_draft && !draft_logits) return ORACLE_BAD_ARG;
    if (parent[0] != -1) return ORACLE_BAD_TREE;
    for (int i = 1; i < T; ++i)
        if (parent[i] < 0 || parent[i] >= i) return ORACLE_BAD_TREE;
    for (int i = 0; i < T; ++i)
        if (token[i] < 0 || token[i] >= V) return ORACLE_BAD_ARG;

    double* p = (double*)malloc((size_t)V * sizeof(double));
    double* q = use_draft ? (double*)malloc((size_t)V * sizeof(double)) : NULL;
    if (!p || (use_draft && !q)) { free(p); free(q); return ORACLE_NOMEM; }

    for (int i = 0; i < T; ++i) path[i] = -1;
    int cur = 0, len = 0;
    path[0] = 0;
    int rejected_any = 0;
    int sampled = -1;
    for (;;) {
        rejected_any = 0;
        int next = -1;
        if (rule == RULE_SAMPLE_MATCH) {
            /* the literal reading of Section 2, step 3: draw the target's own token at this node
             * (inverse CDF with the node's uniform); a child is accepted iff it proposed that token */
            softmax_row(target_logits + (size_t)cur * V, V, temp, p);
            sampled = inverse_cdf(p, V, (double)uniforms[T + cur]);
            for (int c = cur + 1; c < T && next < 0; ++c) {
                if (parent[c] != cur) continue;
                if (token[c] == sampled) next = c; else rejected_any = 1;
            }
        } else if (rule == RULE_GREEDY) {
            const int best = argmax_row(target_logits + (size_t)cur * V, V);
            for (int c = cur + 1; c < T && next < 0; ++c) {
                if (parent[c] != cur) continue;
                if (token[c] == best) next = c; else rejected_any = 1;
            }
        } else {
            softmax_row(target_logits + (size_t)cur * V, V, temp, p);
            if (use_draft) softmax_row(draft_logits + (size_t)cur * V, V, temp, q);
            for (int c = cur + 1; c < T && next < 0; ++c) {   /* children in proposal order */
                if (parent[c] != cur) continue;
                const int x = token[c];
                const double u = (double)uniforms[c];
                int accept;
                if (rule == RULE_DETERMINISTIC) accept = (u < p[x]);
                else accept = (u * q[x] < p[x]);
                if (accept) { next = c; break; }
                rejected_any = 1;
                if (rule == RULE_DETERMINISTIC) {
                    /* the proposal was the point mass on x: the corrected law drops x */
                    p[x] = 0.0;
                    double sum = 0.0;
                    for (int v = 0; v < V; ++v) sum += p[v];
                    if (sum > 0.0) for (int v = 0; v < V; ++v) p[v] /= sum;
                } else {
                    /* corrected law: positive part of (target - draft), renormalised */
                    double sum = 0.0;
                    for (int v = 0; v < V; ++v) {
                        const double r = p[v] - q[v];
                        sum += (r > 0.0) ? r : 0.0;
                    }
                    if (sum > 0.0) {
                        for (int v = 0; v < V; ++v) {
                            const double r = p[v] - q[v];
                            p[v] = ((r > 0.0) ? r : 0.0) / sum;
                        }
                    }
                    if (rule == RULE_DRAFT_WOR) {
                        /* siblings were drawn without replacement: x leaves the draft law */
                        q[x] = 0.0;
                        double qs = 0.0;
                        for (int v = 0; v < V; ++v) qs += q[v];
                        if (qs > 0.0) for (int v = 0; v < V; ++v) q[v] /= qs;
                    }
                }
            }
        }
        if (next < 0) break;
        cur = next;
        path[++len] = cur;
    }

    if (rule == RULE_GREEDY) {
        *final_token = argmax_row(target_logits + (size_t)cur * V, V);
    } else if (rule == RULE_SAMPLE_MATCH) {
        *final_token = sampled;          /* the target's token at the stop node, matched by no child */
    } else {
        /* p now holds the law to draw from at the stop node: the target's own law if
         * nothing was rejected there, the last corrected law otherwise */
        *final_token = inverse_cdf(p, V, (double)uniforms[T + cur]);
    }
    *final_kind = rejected_any ? FINAL_RESIDUAL : FINAL_BONUS;
    *n_accepted = len;
    *last_node = cur;
    if (selected_con) {
        *selected_con = -1;
        if (con_anchor)
            for (int c = 0; c < C; ++c)
                if (con_anchor[c] == cur) { *selected_con = c; break; }
    }
    free(p);
    free(q);
    return ORACLE_OK;
}

/* The same call repeated over n independent sets of uniforms (everything else fixed):
 * lets a test integrate the output law over a grid of uniforms. out_* are [n]. */
int oracle_tree_accept_many(int n, int T, int V, double temp, int rule,
                            const float* target_logits, const float* draft_logits,
                            const int32_t* token, const int32_t* parent,
                            const float* uniforms /* [n][2T] */,
                            int32_t* out_n_accepted, int32_t* out_final_token,
                            int32_t* out_final_kind, int32_t* out_last_node)
{
    int32_t* path = (int32_t*)malloc((size_t)T * sizeof(int32_t));
    if (!path) return ORACLE_NOMEM;
    int rc = ORACLE_OK;
    for (int i = 0; i < n && rc == ORACLE_OK; ++i) {
        rc = oracle_tree_accept(T, V, 0, temp, rule, target_logits, draft_logits, token, parent,
                                uniforms + (size_t)i * 2 * T, NULL, path,
                                out_n_accepted + i, out_final_token + i, out_final_kind + i,
                                out_last_node + i, NULL);
    }
    free(path);
    return rc;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
