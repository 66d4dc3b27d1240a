/*
 * specvlm_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, fp64 CPU definition of the target model's verification step
 * over a draft token tree (SpecVLM, Sec. 3.1: the target "verifies" the
 * drafted tokens in one forward pass and the incorrect ones are discarded;
 * Sec. 4.1: the draft is an EAGLE-2 style token tree, Top-K 10, 60 tokens,
 * depth 7).  The paper never writes these steps as formulas, so every
 * function below is the plain mathematical definition of what that sentence
 * requires, written out without blocking, fusion or reordering:
 *
 *   oracle_ancestors      ancestor-or-self sets of a parent array
 *   oracle_tree_attn      softmax attention where tree node i sees the whole
 *                         committed prefix plus its own ancestors-or-self
 *   oracle_node_argmax    greedy (temperature 0) target token per node,
 *                         lowest index on ties
 *   oracle_tree_accept    longest root path whose drafted tokens equal the
 *                         target's greedy tokens ("lossless" verification)
 *   oracle_tree_accept_sample  the same walk at temperature > 0: each child is
 *                         accepted with its residual target probability
 *                         (speculative sampling with fixed candidates)
 *   oracle_kv_compact     move the accepted path's K/V rows to the front of
 *                         the tree region (read-all-then-write)
 *   oracle_head_argmax    the output head applied to the nodes' hidden states, fused
 *                         with the greedy choice (the logits are never stored)
 *   oracle_visual_pool, oracle_visual_prune
 *                         the two parameter-free visual token compressors of the draft side
 *   oracle_topk_logprob, oracle_tree_select, oracle_tree_finalize
 *                         the draft side: Top-K expansion of a level, choice of
 *                         the next level's nodes, and the final tree
 *
 * Pinned by tests/test_oracle_*.py against: textbook causal attention (chain
 * tree), plain decode attention (one node), a numpy brute force with a
 * materialised mask, hand-worked fixtures under tests/golden/, the closed form
 * sigma = alpha(1-alpha^gamma)/(1-alpha) of Sec. 3.1, exhaustive path
 * enumeration on tiny trees, and, for the sampling walk, the exact output
 * distribution (it must equal the target's), its zero-temperature limit (the
 * greedy walk) and hand-computed acceptance thresholds; for the draft-side
 * growth, a hand-worked fixture, scipy's log_softmax / logsumexp and numpy's
 * stable sort, closed forms (uniform logits, probabilities summing to one) and
 * enumeration of all token sequences (an exhaustively expanded tree must hold
 * exactly the most probable sequences); for the fused head, numpy's float64 matmul
 * + argmax, one-hot head rows, integer-valued inputs whose fp32 logits are exact
 * (then it must agree with oracle_node_argmax on the stored logits) and duplicate rows;
 * for the compressors, numpy's reshape-mean and fancy indexing, ratio 1 = identity, constant
 * inputs, and the mean's linearity.
 *
 * Only tests/, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code with the HIP library.
 *
 * Element types: dtype 0 = bf16 stored as uint16 bit patterns, dtype 1 =
 * IEEE fp32.  Both convert to double exactly, so the oracle sees exactly the
 * bits the GPU sees.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double elem_as_double(const void *base, int dtype, int64_t idx)
{
    if (dtype == 1)
        return (double)((const float *)base)[idx];
    uint32_t w = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* Number of threads an OpenMP parallel region will use here (1 without OpenMP). */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Ancestor-or-self sets.  parent[0] = -1 (root), 0 <= parent[i] < i otherwise.
 * anc[i*n + j] = 1 iff j is i or an ancestor of i.  depth[i] = edges from root.
 * Returns 0, or 1 when the parent array is not a topologically ordered tree.
 */
int oracle_ancestors(int n, const int32_t *parent, uint8_t *anc, int32_t *depth)
{
    if (n < 1 || parent[0] != -1)
        return 1;
    for (int i = 1; i < n; ++i)
        if (parent[i] < 0 || parent[i] >= i)
            return 1;
    memset(anc, 0, (size_t)n * (size_t)n);
    for (int i = 0; i < n; ++i) {
        int d = 0;
        for (int t = i; t != -1; t = parent[t]) {
            anc[(size_t)i * n + t] = 1;
            if (t != i)
                ++d;
        }
        depth[i] = d;
    }
    return 0;
}

/* Logical cache slot -> element offset of that token's row for KV head hk. */
static int64_t kv_row_offset(int b, int hk, int slot,
                             int64_t kv_sb, int64_t kv_sh, int64_t kv_st,
                             const int32_t *block_table, int block_size, int max_blocks)
{
    if (block_table) {
        int blk = block_table[(int64_t)b * max_blocks + slot / block_size];
        return (int64_t)blk * kv_sb + (int64_t)hk * kv_sh + (int64_t)(slot % block_size) * kv_st;
    }
    return (int64_t)b * kv_sb + (int64_t)hk * kv_sh + (int64_t)slot * kv_st;
}

/*
 * Tree-masked attention (definition).  For request b, query head h, tree node
 * i < num_nodes[b]:
 *     J(i) = {0..P_b-1}  U  {P_b + j : j ancestor-or-self of i}
 *     s_j  = scale * sum_d q[b,i,h,d] * K[b,kv(h),j,d]          kv(h) = h / (Hq/Hkv)
 *     o    = sum_J exp(s_j - M) V_j / sum_J exp(s_j - M),        M = max_J s_j
 *     lse  = M + ln sum_J exp(s_j - M)
 * q is [B,N_max,Hq,D] through element strides (q_sb,q_sn,q_sh); K/V are either
 * contiguous (block_table NULL: kv_sb is the request stride) or paged
 * (kv_sb is the block stride).  Outputs: o [B,N_max,Hq,D] dense doubles,
 * lse [B,Hq,N_max] doubles (may be NULL).  Rows i >= num_nodes[b] are set to 0.
 * num_nodes NULL means every request has N_max nodes.
 * Returns 0, 1 on a malformed tree, 2 on allocation failure.
 */
int oracle_tree_attn(int dtype, int B, int Hq, int Hkv, int D, int N_max, double scale,
                     const void *q, int64_t q_sb, int64_t q_sn, int64_t q_sh,
                     const void *k, const void *v,
                     int64_t kv_sb, int64_t kv_sh, int64_t kv_st,
                     const int32_t *block_table, int block_size, int max_blocks,
                     const int32_t *prefix_len, const int32_t *num_nodes,
                     const int32_t *parent, double *o, double *lse)
{
    int status = 0;
    int group = Hq / Hkv;
    for (int b = 0; b < B; ++b) {
        int n = num_nodes ? num_nodes[b] : N_max;
        int P = prefix_len[b];
        uint8_t *anc = malloc((size_t)n * n);
        int32_t *depth = malloc(sizeof(int32_t) * n);
        if (!anc || !depth) {
            free(anc); free(depth);
            return 2;
        }
        if (oracle_ancestors(n, parent + (int64_t)b * N_max, anc, depth)) {
            free(anc); free(depth);
            return 1;
        }
#pragma omp parallel for schedule(dynamic, 1)
        for (int h = 0; h < Hq; ++h) {
            int hk = h / group;
            int S = P + n;
            double *s = malloc(sizeof(double) * S);
            double *acc = malloc(sizeof(double) * D);
            if (!s || !acc) {
#pragma omp atomic write
                status = 2;
                free(s); free(acc);
                continue;
            }
            for (int i = 0; i < N_max; ++i) {
                double *orow = o + (((int64_t)b * N_max + i) * Hq + h) * D;
                if (i >= n) {
                    for (int d = 0; d < D; ++d) orow[d] = 0.0;
                    if (lse) lse[((int64_t)b * Hq + h) * N_max + i] = 0.0;
                    continue;
                }
                int64_t qoff = (int64_t)b * q_sb + (int64_t)i * q_sn + (int64_t)h * q_sh;
                /* scores over the visible set, maximum */
                double M = -INFINITY;
                for (int j = 0; j < S; ++j) {
                    int visible = (j < P) || anc[(size_t)i * n + (j - P)];
                    if (!visible) { s[j] = -INFINITY; continue; }
                    int64_t koff = kv_row_offset(b, hk, j, kv_sb, kv_sh, kv_st,
                                                 block_table, block_size, max_blocks);
                    double dot = 0.0;
                    for (int d = 0; d < D; ++d)
                        dot += elem_as_double(q, dtype, qoff + d) * elem_as_double(k, dtype, koff + d);
                    s[j] = scale * dot;
                    if (s[j] > M) M = s[j];
                }
                /* softmax-weighted sum of V rows */
                double Z = 0.0;
                for (int d = 0; d < D; ++d) acc[d] = 0.0;
                for (int j = 0; j < S; ++j) {
                    int visible = (j < P) || anc[(size_t)i * n + (j - P)];
                    if (!visible) continue;
                    double w = exp(s[j] - M);
                    Z += w;
                    int64_t voff = kv_row_offset(b, hk, j, kv_sb, kv_sh, kv_st,
                                                 block_table, block_size, max_blocks);
                    for (int d = 0; d < D; ++d)
                        acc[d] += w * elem_as_double(v, dtype, voff + d);
                }
                for (int d = 0; d < D; ++d) orow[d] = acc[d] / Z;
                if (lse) lse[((int64_t)b * Hq + h) * N_max + i] = M + log(Z);
            }
            free(s); free(acc);
        }
        free(anc); free(depth);
        if (status) return status;
    }
    return status;
}

/*
 * Greedy target token per node (temperature 0):
 *     amax[b,i] = min { v : logits[b,i,v] = max_v' logits[b,i,v'] }
 * Values compare as real numbers (so -0 equals +0).  Precondition: no NaN.
 * An all -inf row gives index 0.  Rows i >= num_nodes[b] give -1.
 * logits are addressed as b*stride_b + i*stride_n + v (elements).
 */
int oracle_node_argmax(int dtype, int B, int N_max, int V, const void *logits,
                       int64_t stride_b, int64_t stride_n,
                       const int32_t *num_nodes, int32_t *amax)
{
#pragma omp parallel for collapse(2)
    for (int b = 0; b < B; ++b) {
        for (int i = 0; i < N_max; ++i) {
            int n = num_nodes ? num_nodes[b] : N_max;
            if (i >= n) { amax[(int64_t)b * N_max + i] = -1; continue; }
            int64_t off = (int64_t)b * stride_b + (int64_t)i * stride_n;
            int best = 0;
            double bestv = elem_as_double(logits, dtype, off);
            for (int v = 1; v < V; ++v) {
                double x = elem_as_double(logits, dtype, off + v);
                if (x > bestv) { bestv = x; best = v; }
            }
            amax[(int64_t)b * N_max + i] = best;
        }
    }
    return 0;
}

/*
 * Greedy acceptance walk.  Node 0 is the root (a token the target already
 * committed; Fig. 3: the target's first token initialises the tree); its draft
 * token is not matched.  For i >= 1:
 *     match(i) = draft_tok[i] == amax[parent[i]]
 *     ok(0) = true, ok(i) = ok(parent[i]) and match(i)
 *     best = the ok node of greatest depth, lowest node index on ties
 * path = root..best = a_0..a_m (padded with -1 up to path_cap),
 * accept_len = m, bonus_tok = amax[best],
 * committed_tok = draft_tok[a_1..a_m] then bonus_tok (padded with -1).
 * Returns 0, 1 on a malformed tree, 3 if a path would not fit in path_cap.
 */
int oracle_tree_accept(int B, int N_max, int path_cap,
                       const int32_t *parent, const int32_t *draft_tok, const int32_t *amax,
                       const int32_t *num_nodes,
                       int32_t *accept_len, int32_t *path, int32_t *bonus_tok,
                       int32_t *committed_tok)
{
    for (int b = 0; b < B; ++b) {
        int n = num_nodes ? num_nodes[b] : N_max;
        const int32_t *par = parent + (int64_t)b * N_max;
        const int32_t *tok = draft_tok + (int64_t)b * N_max;
        const int32_t *am = amax + (int64_t)b * N_max;
        if (n < 1 || par[0] != -1) return 1;
        int *ok = malloc(sizeof(int) * n);
        int *depth = malloc(sizeof(int) * n);
        ok[0] = 1; depth[0] = 0;
        int best = 0;
        for (int i = 1; i < n; ++i) {
            if (par[i] < 0 || par[i] >= i) { free(ok); free(depth); return 1; }
            depth[i] = depth[par[i]] + 1;
            ok[i] = ok[par[i]] && (tok[i] == am[par[i]]);
            if (ok[i] && depth[i] > depth[best]) best = i;   /* strict: ties keep the lower index */
        }
        int m = depth[best];
        if (m + 1 > path_cap) { free(ok); free(depth); return 3; }
        int32_t *prow = path + (int64_t)b * path_cap;
        int32_t *crow = committed_tok + (int64_t)b * path_cap;
        for (int j = 0; j < path_cap; ++j) { prow[j] = -1; crow[j] = -1; }
        int t = best;
        for (int j = m; j >= 0; --j) { prow[j] = t; t = par[t]; }
        for (int j = 1; j <= m; ++j) crow[j - 1] = tok[prow[j]];
        crow[m] = am[best];
        accept_len[b] = m;
        bonus_tok[b] = am[best];
        free(ok); free(depth);
    }
    return 0;
}

/*
 * Sampling-based acceptance walk (temperature > 0).  The paper names speculative
 * sampling as the rule that discards drafted tokens (Sec. 3.1) and evaluates
 * temperature 1 with the same Top-K tree (Sec. 4.1) without writing the tree form
 * out.  The reading taken here: the children of a tree node are a FIXED candidate
 * list (top-K expansion, not draws from the draft distribution), so each candidate
 * is a point-mass proposal and the speculative-sampling rule
 *     accept x with probability min(1, p(x)/q(x)),  else  p <- norm(max(p - q, 0))
 * becomes, at the current node cur with target distribution
 *     p = softmax(logits[cur] / temperature):
 *     for each child c of cur, in increasing node index:
 *         x = draft_tok[c]
 *         accept c (cur <- c, restart with c's own distribution) when
 *             u_accept[c] < p(x) / (1 - sum of p over tokens already rejected at cur)
 *         (a token already rejected at cur has residual probability 0: rejected again);
 *         otherwise x joins the rejected set of cur
 *     no child accepted: stop.
 * The bonus token is drawn from the residual distribution at the final node
 * (p with its rejected tokens zeroed, renormalised) by inverse CDF in vocabulary
 * order: the lowest v with  sum_{v' <= v, v' not rejected} p(v') > u_bonus * residual mass.
 * Each emitted token is then distributed exactly as the target's own sample.
 *
 * u_accept [B,N_max] and u_bonus [B] are uniform numbers in [0,1) supplied by the
 * caller.  A child whose token is outside [0,V) is rejected.  Walking stops when
 * the path holds path_cap nodes.  Outputs as oracle_tree_accept, plus (each
 * optional) what a caller needs to tell decisions that a lower-precision
 * evaluation might take differently:
 *   margin_accept[b]  smallest |u - threshold| over the accept comparisons taken
 *   margin_bonus[b]   distance (as probability of the residual distribution)
 *                     from the drawn position to the nearer edge of the bonus
 *                     token's CDF interval
 *   bonus_alt[b]      the token on the other side of that edge (the bonus token
 *                     itself when there is none)
 * Returns 0, 1 on a malformed tree, 2 on allocation failure.
 */
int oracle_tree_accept_sample(int dtype, int B, int N_max, int V, int path_cap,
                              const int32_t *parent, const int32_t *draft_tok,
                              const void *logits, int64_t stride_b, int64_t stride_n,
                              const int32_t *num_nodes, double temperature,
                              const float *u_accept, const float *u_bonus,
                              int32_t *accept_len, int32_t *path, int32_t *bonus_tok,
                              int32_t *committed_tok, double *margin_accept, double *margin_bonus,
                              int32_t *bonus_alt)
{
    double *e = malloc(sizeof(double) * (size_t)V);
    uint8_t *rejected = malloc((size_t)V);
    if (!e || !rejected) { free(e); free(rejected); return 2; }
    int rc = 0;
    for (int b = 0; b < B && !rc; ++b) {
        int n = num_nodes ? num_nodes[b] : N_max;
        const int32_t *par = parent + (int64_t)b * N_max;
        const int32_t *tok = draft_tok + (int64_t)b * N_max;
        if (n < 1 || par[0] != -1) { rc = 1; break; }
        for (int i = 1; i < n; ++i) if (par[i] < 0 || par[i] >= i) rc = 1;
        if (rc) break;
        int32_t *prow = path + (int64_t)b * path_cap;
        int32_t *crow = committed_tok + (int64_t)b * path_cap;
        for (int j = 0; j < path_cap; ++j) { prow[j] = -1; crow[j] = -1; }
        double mg = 1.0;
        int cur = 0, m = 0;
        prow[0] = 0;
        double Z = 0.0, rej_mass = 0.0;
        for (;;) {
            /* unnormalised target distribution at cur: e[v] = exp((l_v - max) / T) */
            const int64_t row = (int64_t)b * stride_b + (int64_t)cur * stride_n;
            double mx = -INFINITY;
            for (int v = 0; v < V; ++v) { double l = elem_as_double(logits, dtype, row + v); if (l > mx) mx = l; }
            Z = 0.0;
            for (int v = 0; v < V; ++v) {
                e[v] = exp((elem_as_double(logits, dtype, row + v) - mx) / temperature);
                Z += e[v];
                rejected[v] = 0;
            }
            rej_mass = 0.0;
            int next = -1;
            if (m + 1 < path_cap) {
                for (int c = cur + 1; c < n && next < 0; ++c) {
                    if (par[c] != cur) continue;
                    const int x = tok[c];
                    const int live = x >= 0 && x < V && !rejected[x];
                    const double a = live ? e[x] / (Z - rej_mass) : 0.0;     /* residual probability of x */
                    const double u = (double)u_accept[(int64_t)b * N_max + c];
                    if (live && fabs(u - a) < mg) mg = fabs(u - a);   /* a dead token is rejected in any precision */
                    if (u < a) {
                        next = c;
                    } else if (live) {
                        rejected[x] = 1;
                        rej_mass += e[x];
                    }
                }
            }
            if (next < 0) break;
            cur = next;
            prow[++m] = cur;
        }
        /* bonus token: inverse CDF over the residual distribution at cur */
        const double total = Z - rej_mass;
        const double t = (double)u_bonus[b] * total;
        double cum = 0.0, lo = 0.0;
        int pick = -1, last_live = -1, prev_live = -1;
        for (int v = 0; v < V && pick < 0; ++v) {
            if (rejected[v] || !(e[v] > 0.0)) continue;
            lo = cum;
            cum += e[v];
            prev_live = last_live;
            last_live = v;
            if (cum > t) pick = v;
        }
        if (pick < 0) { pick = last_live; }               /* rounding left t at the very end */
        {
            int next_live = -1;
            for (int v = pick + 1; v < V && next_live < 0; ++v)
                if (!rejected[v] && e[v] > 0.0) next_live = v;
            const double d_lo = (t - lo) / total, d_hi = (cum - t) / total;
            int alt = d_lo <= d_hi ? prev_live : next_live;
            if (alt < 0) alt = pick;
            if (margin_bonus) margin_bonus[b] = alt == pick ? 1.0 : (d_lo <= d_hi ? d_lo : d_hi);
            if (bonus_alt) bonus_alt[b] = alt;
        }
        for (int j = 1; j <= m; ++j) crow[j - 1] = tok[prow[j]];
        crow[m] = pick;
        accept_len[b] = m;
        bonus_tok[b] = pick;
        if (margin_accept) margin_accept[b] = mg;
    }
    free(e); free(rejected);
    return rc;
}

/*
 * ---- draft-side tree growth (Sec. 4.1: "following EAGLE-2, the draft uses tree
 * attention with Top-K = 10, total tokens = 60, depth = 7") ----------------------
 * The paper gives the three numbers only; the growth rule is the one of the
 * method it follows: a node's value is the sum of the draft's log-probabilities
 * along its root path; every level expands the Top-K most valuable nodes of the
 * previous level by their Top-K tokens; at the end the `total` most valuable
 * candidates form the tree.  Three definitions:
 *
 * oracle_topk_logprob: for each row r of logits [R,V] (row stride stride_r),
 *     lse_r = ln sum_v exp(l_v),
 *     token[r,0..K-1] = the K tokens of greatest logit, greater first, the lower
 *                       token first among equal logits,
 *     score[r,k] = cum[r] + l_{token[r,k]} - lse_r      (cum NULL means 0).
 * Returns 0, or 5 when K > V.
 */
int oracle_topk_logprob(int dtype, int R, int V, int K, const void *logits, int64_t stride_r,
                        const double *cum, double *score, int32_t *token, double *lse)
{
    if (K > V || K < 1) return 5;
    uint8_t *taken = malloc((size_t)V);
    if (!taken) return 2;
    for (int r = 0; r < R; ++r) {
        const int64_t row = (int64_t)r * stride_r;
        double mx = -INFINITY;
        for (int v = 0; v < V; ++v) { double l = elem_as_double(logits, dtype, row + v); if (l > mx) mx = l; }
        double z = 0.0;
        for (int v = 0; v < V; ++v) z += exp(elem_as_double(logits, dtype, row + v) - mx);
        const double l_r = mx + log(z);
        if (lse) lse[r] = l_r;
        memset(taken, 0, (size_t)V);
        for (int k = 0; k < K; ++k) {
            int best = -1;
            double bv = 0.0;
            for (int v = 0; v < V; ++v) {
                if (taken[v]) continue;
                const double l = elem_as_double(logits, dtype, row + v);
                if (best < 0 || l > bv) { best = v; bv = l; }     /* strict: ties keep the lower token */
            }
            taken[best] = 1;
            token[(int64_t)r * K + k] = best;
            score[(int64_t)r * K + k] = (cum ? cum[r] : 0.0) + bv - l_r;
        }
    }
    free(taken);
    return 0;
}

/*
 * oracle_tree_select: the M most valuable of C scored candidates, per request.
 * Candidate i beats candidate j when score[i] > score[j], or when the scores are
 * equal and i < j.  Scores are fp32 values and are compared as they are (this
 * is a decision, so it is taken on the stored numbers).  sel[b,0..] lists the
 * winners in increasing candidate index, -1 padded; count[b] = min(M, C_b);
 * gap[b] (optional) = score of the last winner minus score of the best loser
 * (+inf when nobody loses).  num_cand NULL means C candidates everywhere.
 */
int oracle_tree_select(int B, int C, int M, const float *score, const int32_t *num_cand,
                       int32_t *sel, int32_t *count, double *gap)
{
    for (int b = 0; b < B; ++b) {
        const int c = num_cand ? num_cand[b] : C;
        const float *sc = score + (int64_t)b * C;
        int32_t *out = sel + (int64_t)b * M;
        int n = 0;
        double worst_in = INFINITY, best_out = -INFINITY;
        for (int i = 0; i < c; ++i) {
            int beaten_by = 0;
            for (int j = 0; j < c; ++j)
                if (sc[j] > sc[i] || (sc[j] == sc[i] && j < i)) ++beaten_by;
            if (beaten_by < M) {
                out[n++] = i;
                if ((double)sc[i] < worst_in) worst_in = sc[i];
            } else if ((double)sc[i] > best_out) {
                best_out = sc[i];
            }
        }
        for (int j = n; j < M; ++j) out[j] = -1;
        if (count) count[b] = n;
        if (gap) gap[b] = best_out == -INFINITY ? INFINITY : worst_in - best_out;
    }
    return 0;
}

/*
 * oracle_tree_finalize: turn the candidates of a finished growth into the draft
 * tree that the target verifies.  Candidate i has a score, a token and a parent
 * candidate cand_parent[i] < i (-1: a child of the root).  The N_max - 1 most
 * valuable candidates (rule of oracle_tree_select) become nodes 1.., in
 * increasing candidate index -- which is a topological order because a parent
 * precedes its children -- and node 0 is the root carrying root_token:
 *     node_cand[b,j]  candidate behind node j (-1 for the root, -1 padding)
 *     parent[b,j]     node index of its parent (-1 for the root)
 *     draft_tok[b,j]  its token
 *     num_nodes[b]    1 + number of selected candidates
 * A child never outscores its parent when scores are sums of log-probabilities,
 * so the selection is closed under "parent of"; returns 4 if it is not, 1 if a
 * cand_parent entry is not below its own index.
 */
int oracle_tree_finalize(int B, int C, int N_max, const float *cand_score, const int32_t *cand_parent,
                         const int32_t *cand_token, const int32_t *num_cand, const int32_t *root_token,
                         int32_t *parent, int32_t *draft_tok, int32_t *node_cand, int32_t *num_nodes,
                         double *gap)
{
    const int M = N_max - 1;
    int32_t *sel = malloc(sizeof(int32_t) * (size_t)(M > 0 ? M : 1));
    int32_t *node_of = malloc(sizeof(int32_t) * (size_t)(C > 0 ? C : 1));
    if (!sel || !node_of) { free(sel); free(node_of); return 2; }
    int rc = 0;
    for (int b = 0; b < B && !rc; ++b) {
        const int c = num_cand ? num_cand[b] : C;
        int32_t cnt = 0;
        if (M > 0)
            oracle_tree_select(1, C, M, cand_score + (int64_t)b * C, &c, sel, &cnt, gap ? gap + b : NULL);
        else if (gap) gap[b] = INFINITY;
        int32_t *par = parent + (int64_t)b * N_max, *tok = draft_tok + (int64_t)b * N_max;
        int32_t *nc = node_cand + (int64_t)b * N_max;
        for (int j = 0; j < N_max; ++j) { par[j] = -1; tok[j] = -1; nc[j] = -1; }
        for (int i = 0; i < c; ++i) node_of[i] = -1;
        tok[0] = root_token[b];
        for (int j = 0; j < cnt; ++j) node_of[sel[j]] = j + 1;
        for (int j = 0; j < cnt; ++j) {
            const int i = sel[j];
            const int cp = cand_parent[(int64_t)b * C + i];
            if (cp >= i) { rc = 1; break; }
            if (cp >= 0 && node_of[cp] < 0) { rc = 4; break; }
            nc[j + 1] = i;
            par[j + 1] = cp < 0 ? 0 : node_of[cp];
            tok[j + 1] = cand_token[(int64_t)b * C + i];
        }
        num_nodes[b] = cnt + 1;
    }
    free(sel); free(node_of);
    return rc;
}

/*
 * ---- parameter-free visual token compressors (Sec. 3.4, the elastic vision compressor:
 * pruning discards a random subset of the tokens, pooling is a plain operator; Table 4 uses ratios 2x .. 30x) ------------------------------------------
 * They shorten the visual prefix the DRAFT reads (the target keeps the full sequence, which is what
 * keeps decoding lossless).  The paper fixes neither the pooling window nor what happens to a ragged
 * tail; the reading here: average pooling along the token sequence with window = stride = ratio, the
 * last window shorter when the length is not a multiple (mean over the tokens it has):
 *     y[b,j,:] = mean_{t = j*ratio .. min((j+1)*ratio, T_b) - 1} x[b,t,:],   j < ceil(T_b / ratio)
 * and pruning keeps the tokens whose indices the caller drew (any order, repeats allowed):
 *     y[b,j,:] = x[b, keep[b,j], :]            (keep[b,j] = -1: row j is padding and left untouched)
 * Output in double (pool) / bit copies (prune).  out_tokens[b] = ceil(T_b / ratio).
 */
int oracle_visual_pool(int dtype, int B, int T, int E, int ratio, const void *x, int64_t x_stride_b,
                       int64_t x_stride_t, const int32_t *num_tokens, double *y, int32_t *out_tokens)
{
    if (ratio < 1) return 1;
    const int Tp = (T + ratio - 1) / ratio;
    for (int b = 0; b < B; ++b) {
        const int tb = num_tokens ? num_tokens[b] : T;
        if (tb < 0 || tb > T) return 1;
        const int nb = (tb + ratio - 1) / ratio;
        if (out_tokens) out_tokens[b] = nb;
        for (int j = 0; j < nb; ++j) {
            const int t0 = j * ratio, t1 = (j + 1) * ratio < tb ? (j + 1) * ratio : tb;
            for (int e = 0; e < E; ++e) {
                double acc = 0.0;
                for (int t = t0; t < t1; ++t)
                    acc += elem_as_double(x, dtype, (int64_t)b * x_stride_b + (int64_t)t * x_stride_t + e);
                y[((int64_t)b * Tp + j) * E + e] = acc / (double)(t1 - t0);
            }
        }
    }
    return 0;
}

int oracle_visual_prune(int elem_bytes, int B, int T, int T_keep, int E, const void *x, int64_t x_stride_b,
                        int64_t x_stride_t, const int32_t *keep, void *y)
{
    for (int b = 0; b < B; ++b)
        for (int j = 0; j < T_keep; ++j) {
            const int t = keep[(int64_t)b * T_keep + j];
            if (t == -1) continue;
            if (t < 0 || t >= T) return 1;
            memcpy((char *)y + ((int64_t)b * T_keep + j) * E * elem_bytes,
                   (const char *)x + ((int64_t)b * x_stride_b + (int64_t)t * x_stride_t) * elem_bytes,
                   (size_t)E * elem_bytes);
        }
    return 0;
}

/*
 * ---- output head fused with the greedy choice (Fig. 3: the output head is shared by target and
 * draft; temperature 0, Sec. 4.1) ----------------------------------------------------------------
 * The target's logits of node i are the head matrix applied to its last hidden state,
 *     logit[b,i,v] = sum_e hidden[b,i,e] * W[v,e]                     (W is [V,E], row v = token v)
 * and the greedy token is amax[b,i] = the lowest v holding the row's greatest logit.  This is
 * oracle_node_argmax applied to logits that are never stored.  Everything in double (products of
 * bf16 or fp32 inputs are exact in double; the sum is rounded as double).  Optional outputs:
 *     max_logit[b,i]  the greatest logit
 *     gap[b,i]        greatest minus second greatest logit over DIFFERENT tokens (0 on an exact tie,
 *                     +inf when V == 1): a comparison partner that accumulates in lower precision
 *                     can only be held to rows whose gap exceeds its rounding error
 *     second[b,i]     the token holding the second greatest logit (lowest index on ties), -1 if V == 1
 * Rows i >= num_nodes[b] get amax -1.  hidden element (b,i,e) at b*h_stride_b + i*h_stride_n + e.
 */
int oracle_head_argmax(int dtype, int B, int N_max, int E, int V, const void *hidden, int64_t h_stride_b,
                       int64_t h_stride_n, const void *W, int64_t w_stride_v, const int32_t *num_nodes,
                       int32_t *amax, double *max_logit, double *gap, int32_t *second)
{
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int i = 0; i < N_max; ++i) {
            const int64_t o = (int64_t)b * N_max + i;
            const int n = num_nodes ? num_nodes[b] : N_max;
            if (i >= n) {
                amax[o] = -1;
                if (max_logit) max_logit[o] = 0.0;
                if (gap) gap[o] = INFINITY;
                if (second) second[o] = -1;
                continue;
            }
            const int64_t h0 = (int64_t)b * h_stride_b + (int64_t)i * h_stride_n;
            int best = -1, sec = -1;
            double bv = 0.0, sv = 0.0;
            for (int v = 0; v < V; ++v) {
                double acc = 0.0;
                for (int e = 0; e < E; ++e)
                    acc += elem_as_double(hidden, dtype, h0 + e) * elem_as_double(W, dtype, (int64_t)v * w_stride_v + e);
                if (best < 0 || acc > bv) {            /* strict: ties keep the lower token */
                    sec = best; sv = bv;
                    best = v; bv = acc;
                } else if (sec < 0 || acc > sv) {
                    sec = v; sv = acc;
                }
            }
            amax[o] = best;
            if (max_logit) max_logit[o] = bv;
            if (gap) gap[o] = sec < 0 ? INFINITY : bv - sv;
            if (second) second[o] = sec;
        }
    return 0;
}

/*
 * KV compaction of the accepted path, for all layers, KV heads and both K and V:
 *     cache[P_b + j] <- cache_old[P_b + a_j]   j = 0..m     (read all, then write)
 *     new_prefix_len[b] = P_b + m + 1
 * The paper does not describe this step; it is what any tree verifier must do
 * so that the cache holds only committed tokens.  Rows are copied as raw bytes.
 * Layer l's cache starts layer_stride elements after layer l-1's.
 * moved_idx (may be NULL) [B,path_cap,2] receives (src_slot, dst_slot), -1 padded.
 * new_prefix_len may alias prefix_len.
 */
int oracle_kv_compact(int L, int B, int Hkv, int D, int elem_bytes,
                      void *k, void *v, int64_t layer_stride,
                      int64_t kv_sb, int64_t kv_sh, int64_t kv_st,
                      const int32_t *block_table, int block_size, int max_blocks,
                      const int32_t *prefix_len, const int32_t *path, int path_cap,
                      const int32_t *accept_len, int32_t *new_prefix_len, int32_t *moved_idx)
{
    size_t row_bytes = (size_t)D * elem_bytes;
    for (int b = 0; b < B; ++b) {
        int P = prefix_len[b];
        int m = accept_len[b];
        const int32_t *prow = path + (int64_t)b * path_cap;
        if (m < 0 || m + 1 > path_cap) return 3;
        if (moved_idx)
            for (int j = 0; j < path_cap; ++j) {
                moved_idx[((int64_t)b * path_cap + j) * 2 + 0] = j <= m ? P + prow[j] : -1;
                moved_idx[((int64_t)b * path_cap + j) * 2 + 1] = j <= m ? P + j : -1;
            }
        unsigned char *tmp = malloc(row_bytes * (size_t)(m + 1));
        if (!tmp) return 2;
        for (int l = 0; l < L; ++l)
            for (int which = 0; which < 2; ++which) {
                unsigned char *base = (unsigned char *)(which ? v : k) +
                                      (size_t)l * layer_stride * elem_bytes;
                for (int hk = 0; hk < Hkv; ++hk) {
                    for (int j = 0; j <= m; ++j) {
                        int64_t off = kv_row_offset(b, hk, P + prow[j], kv_sb, kv_sh, kv_st,
                                                    block_table, block_size, max_blocks);
                        memcpy(tmp + row_bytes * j, base + off * elem_bytes, row_bytes);
                    }
                    for (int j = 0; j <= m; ++j) {
                        int64_t off = kv_row_offset(b, hk, P + j, kv_sb, kv_sh, kv_st,
                                                    block_table, block_size, max_blocks);
                        memcpy(base + off * elem_bytes, tmp + row_bytes * j, row_bytes);
                    }
                }
            }
        free(tmp);
    }
    for (int b = 0; b < B; ++b)
        new_prefix_len[b] = prefix_len[b] + accept_len[b] + 1;
    return 0;
}
