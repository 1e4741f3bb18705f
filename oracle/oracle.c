/*
 * CPU oracle for the tree-verification step of speculative decoding
 * (paper Section 3.1: the target model scores a whole draft tree in one pass,
 * then keeps the longest accepted prefix; Section 3.2: image embeddings are
 * ordinary context positions; Eq. 1: softmax attention).
 *
 * THIS IS TEST INFRASTRUCTURE. It is a plain, slow, direct transcription of the
 * definitions, in fp64, with no tiling, no online softmax and no bit tricks. It
 * shares no code with the HIP library and must never be linked, imported or
 * called by the product path; only the tests, the smoke check and the
 * benchmark's CPU-baseline leg use it.
 *
 * Every function takes host pointers. All reals are computed in double; inputs
 * arrive as float (bf16 storage is widened to float by the caller, which is
 * exact).
 *
 * Pins (tests that tie each function to something other than itself):
 *   oracle_tree_validate / oracle_tree_mask  closed forms for chain and star
 *       trees, popcount = depth + 1, brute-force reachability on random trees.
 *   oracle_tree_attention  chain tree = textbook causal attention (independent
 *       fp64 routine), one-node tree = decode attention, needle keys, the
 *       closed form for R identical keys plus one unique key (paper Eq. 3-4),
 *       zero keys = mean of visible values, convex-hull bounds, GQA = MHA with
 *       repeated heads, permutation invariance, split merge by log-sum-exp.
 *   oracle_row_argmax  planted maxima, ties, signed zeros, NaN rule, numpy.
 *   oracle_tree_accept  brute-force enumeration of root-to-leaf paths (a
 *       separate implementation in another language), forced full/zero
 *       acceptance, structural invariants of the returned path.
 *   oracle_tree_accept_sample  exact output distribution by enumeration of the
 *       decision tree (a separate implementation) equals the target softmax at
 *       every emitted position, Monte-Carlo chi-square of the same, temperature
 *       -> 0 equals the greedy rule, u = 0 / u -> 1 extremes, duplicate sibling
 *       tokens, inverse-CDF sampling against numpy's searchsorted.
 *   oracle_tree_accept_sample_check  admits the walk's own outcome and nothing else at
 *       eps = 0; hand-worked knife-edge cases for eps > 0.
 *   oracle_draft_expand  numpy stable argsort and an independent log-softmax for tokens
 *       and scores, a hand-worked example, brute-force frontier.
 *   oracle_draft_tree_build  exhaustive search over ancestor-closed subsets on tiny
 *       candidate sets (the selection maximises total probability), K = 1 gives a chain,
 *       structural invariants, a hand-worked example.
 *   oracle_compress_attention  an independent fp64 softmax-attention routine, the paper's
 *       closed form for R identical keys plus one unique key (Eq. 3-4), hand-worked
 *       weights, zero keys = mean over exactly r values, untouched slots beyond r.
 *   oracle_kv_commit  an out-of-place gather from a pristine copy of the cache
 *       (numpy fancy indexing), identity on a chain path, untouched bytes
 *       outside the destination rows, and the closed loop: attention over the
 *       committed cache equals attention over the accepted tokens' rows taken
 *       from the original cache.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum {
    ORACLE_OK = 0,
    ORACLE_BAD_ROOT = 1,   /* parent[0] != -1 */
    ORACLE_BAD_PARENT = 2, /* parent[i] outside [0, i) for some i >= 1 */
    ORACLE_BAD_SIZE = 3,
    ORACLE_BAD_PATH = 4    /* accepted path is not root, then strictly increasing node ids */
};

/* Section 3.1, "draft tree": node 0 is the root (the last committed token), every
 * other node names an earlier node as its parent. Returns ORACLE_OK or the first
 * violation found. */
int oracle_tree_validate(const int32_t* parent, int32_t T) {
    if (T < 1 || T > 64) return ORACLE_BAD_SIZE;
    if (parent[0] != -1) return ORACLE_BAD_ROOT;
    for (int32_t i = 1; i < T; ++i)
        if (parent[i] < 0 || parent[i] >= i) return ORACLE_BAD_PARENT;
    return ORACLE_OK;
}

/* Ancestor-or-self sets of the draft tree. mask[i] has bit j set iff node j is i
 * or an ancestor of i; depth[i] is the number of edges from the root. */
int oracle_tree_mask(const int32_t* parent, int32_t T, uint64_t* mask, int32_t* depth) {
    int rc = oracle_tree_validate(parent, T);
    if (rc != ORACLE_OK) return rc;
    for (int32_t i = 0; i < T; ++i) {
        uint64_t m = 0;
        int32_t hops = 0;
        int32_t j = i;
        while (j != -1) {
            m |= (uint64_t)1 << j;
            j = parent[j];
            if (j != -1) ++hops;
        }
        mask[i] = m;
        depth[i] = hops;
    }
    return ORACLE_OK;
}

/* Where logical token `tok` of KV head `kvh` starts inside a cache.
 * Contiguous: kvh * stride_head + tok * stride_tok (the base pointer is the
 * sequence's). Paged: block = block_table[tok / block_size], then
 * block * stride_block + kvh * stride_head + (tok % block_size) * stride_tok. */
typedef struct {
    int32_t paged;
    int64_t stride_head, stride_tok;
    const int32_t* block_table;
    int32_t block_size;
    int64_t stride_block;
} oracle_kv_layout;

static int64_t token_offset(const oracle_kv_layout* L, int32_t kvh, int32_t tok) {
    if (!L->paged) return (int64_t)kvh * L->stride_head + (int64_t)tok * L->stride_tok;
    int32_t blk = L->block_table[tok / L->block_size];
    return (int64_t)blk * L->stride_block + (int64_t)kvh * L->stride_head +
           (int64_t)(tok % L->block_size) * L->stride_tok;
}

/* Tree-masked attention for one sequence (Eq. 1 with the usual scale, restricted to
 * the keys a node may see). The cache holds S prefix tokens followed by the T tree
 * nodes' own keys/values at logical slots S .. S+T-1. Node i, query head h sees
 * every prefix key and the tree keys of i's ancestor-or-self set; it reads KV
 * head h / (Hq / Hkv).
 *
 *   s_j   = scale * <q[i,h,:], K[kv,j,:]>            for visible j
 *   w_j   = exp(s_j - max_j s_j)
 *   out[i,h,:] = sum_j w_j V[kv,j,:] / sum_j w_j      (ascending j)
 *
 * Keys that are not visible are skipped, never multiplied by zero, so whatever
 * they hold (NaN included) cannot reach the output.
 *
 * q   [T][Hq][d] float, out [T][Hq][d] double; only heads h_begin <= h < h_end are
 * computed (lets a caller spread heads over threads). */
int oracle_tree_attention(const float* q, const float* k_cache, const float* v_cache,
                          int32_t T, int32_t Hq, int32_t Hkv, int32_t d, int32_t S, double scale,
                          const int32_t* parent, int32_t paged, int64_t stride_head,
                          int64_t stride_tok, const int32_t* block_table, int32_t block_size,
                          int64_t stride_block, int32_t h_begin, int32_t h_end, double* out) {
    uint64_t mask[64];
    int32_t depth[64];
    int rc = oracle_tree_mask(parent, T, mask, depth);
    if (rc != ORACLE_OK) return rc;
    if (Hkv < 1 || Hq % Hkv != 0 || d < 1 || S < 0) return ORACLE_BAD_SIZE;
    oracle_kv_layout L = {paged, stride_head, stride_tok, block_table, block_size, stride_block};
    const int32_t group = Hq / Hkv;
    const int32_t n = S + T;
    double* s = (double*)malloc(sizeof(double) * (size_t)n);
    unsigned char* vis = (unsigned char*)malloc((size_t)n);
    if (!s || !vis) { free(s); free(vis); return ORACLE_BAD_SIZE; }
    for (int32_t i = 0; i < T; ++i) {
        for (int32_t j = 0; j < n; ++j)
            vis[j] = (j < S) ? 1 : (unsigned char)((mask[i] >> (j - S)) & 1u);
        for (int32_t h = h_begin; h < h_end; ++h) {
            const int32_t kv = h / group;
            const float* qv = q + ((int64_t)i * Hq + h) * d;
            double m = -INFINITY;
            for (int32_t j = 0; j < n; ++j) {
                if (!vis[j]) continue;
                const float* kj = k_cache + token_offset(&L, kv, j);
                double dot = 0.0;
                for (int32_t c = 0; c < d; ++c) dot += (double)qv[c] * (double)kj[c];
                s[j] = scale * dot;
                if (s[j] > m) m = s[j];
            }
            double* o = out + ((int64_t)i * Hq + h) * d;
            for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
            double denom = 0.0;
            for (int32_t j = 0; j < n; ++j) {
                if (!vis[j]) continue;
                const double w = exp(s[j] - m);
                const float* vj = v_cache + token_offset(&L, kv, j);
                denom += w;
                for (int32_t c = 0; c < d; ++c) o[c] += w * (double)vj[c];
            }
            for (int32_t c = 0; c < d; ++c) o[c] /= denom;
        }
    }
    free(s);
    free(vis);
    return ORACLE_OK;
}

/* Greedy choice of the target model at one node: the first index holding the row
 * maximum. A plain left-to-right scan with strict '>' in fp32, so ties (signed
 * zeros included) keep the lowest index and NaN never replaces the incumbent. */
int64_t oracle_row_argmax(const float* logits, int64_t V) {
    int64_t best = 0;
    for (int64_t t = 1; t < V; ++t)
        if (logits[t] > logits[best]) best = t;
    return best;
}

/* Greedy (temperature 0) acceptance over the tree. Section 3.1 accepts a draft
 * token with probability min(1, p/p_hat) and on rejection resamples from the
 * normalised positive part of p - p_hat; at temperature 0 the target's p is one-hot
 * at its argmax, so a child is accepted iff its token equals the argmax of its
 * parent's logits, and the token emitted after the last accepted node (the "bonus")
 * is that node's own argmax. accepted_len counts accepted draft tokens only (the
 * paper's acceptance length excludes the bonus token).
 *
 * amax[i]: argmax of node i's logits. draft[i]: node i's draft token (draft[0], the
 * root's already committed token, is ignored).
 * Result: best = accepted node of greatest depth (ties: lowest index);
 * accepted_len = depth[best]; path[0..accepted_len] = root .. best, remaining
 * path entries -1; bonus = amax[best]. */
int oracle_tree_accept(const int32_t* amax, const int32_t* draft, const int32_t* parent, int32_t T,
                       int32_t* accepted_len, int32_t* path, int32_t* bonus) {
    uint64_t mask[64];
    int32_t depth[64];
    unsigned char ok[64];
    int rc = oracle_tree_mask(parent, T, mask, depth);
    if (rc != ORACLE_OK) return rc;
    ok[0] = 1;
    for (int32_t i = 1; i < T; ++i)
        ok[i] = (unsigned char)(ok[parent[i]] && draft[i] == amax[parent[i]]);
    int32_t best = 0;
    for (int32_t i = 1; i < T; ++i)
        if (ok[i] && depth[i] > depth[best]) best = i;
    *accepted_len = depth[best];
    for (int32_t k = 0; k < T; ++k) path[k] = -1;
    for (int32_t j = best; j != -1; j = parent[j]) path[depth[j]] = j;
    *bonus = amax[best];
    return ORACLE_OK;
}

/* Commit of the accepted path into a pre-allocated KV cache (Section 3.1: the draft
 * tokens after the first rejected one are discarded; Appendix A: the cache is
 * allocated once, so keeping the accepted tokens means moving their rows).
 *
 * Before the call the cache of one sequence holds S prefix tokens and the T tree
 * nodes' rows at logical slots S .. S+T-1 (node i at S+i). path[0..accepted_len]
 * is the accepted root-to-node path (path[0] = 0, node ids strictly increasing,
 * as oracle_tree_accept returns it). After the call slot S+k holds the row of node
 * path[k] for k = 0 .. accepted_len, i.e. the sequence's context is the old prefix
 * plus the accepted tokens in order, and *new_prefix = S + accepted_len + 1.
 * Rows are moved as bytes, one k after the other in ascending order; since
 * path[k] >= k no source row is overwritten before it is read. Slots above
 * S + accepted_len keep whatever they held.
 *
 * `cache` is one tensor (K or V) of one layer and one sequence (contiguous) or the
 * block pool (paged); offsets are in elements of elem_bytes bytes. */
int oracle_kv_commit(unsigned char* cache, int32_t elem_bytes, int32_t Hkv, int32_t d, int32_t S,
                     int32_t T, const int32_t* path, int32_t accepted_len, int32_t paged,
                     int64_t stride_head, int64_t stride_tok, const int32_t* block_table,
                     int32_t block_size, int64_t stride_block, int32_t* new_prefix) {
    if (T < 1 || T > 64 || S < 0) return ORACLE_BAD_SIZE;
    if (accepted_len < 0 || accepted_len >= T || path[0] != 0) return ORACLE_BAD_PATH;
    for (int32_t k = 1; k <= accepted_len; ++k)
        if (path[k] <= path[k - 1] || path[k] >= T) return ORACLE_BAD_PATH;
    oracle_kv_layout L = {paged, stride_head, stride_tok, block_table, block_size, stride_block};
    const size_t row_bytes = (size_t)d * (size_t)elem_bytes;
    for (int32_t kvh = 0; kvh < Hkv; ++kvh)
        for (int32_t k = 1; k <= accepted_len; ++k) {
            const int64_t src = token_offset(&L, kvh, S + path[k]);
            const int64_t dst = token_offset(&L, kvh, S + k);
            if (src != dst) memmove(cache + dst * elem_bytes, cache + src * elem_bytes, row_bytes);
        }
    *new_prefix = S + accepted_len + 1;
    return ORACLE_OK;
}

/* Stochastic acceptance over a draft tree (Section 3.1: a draft token is accepted with
 * probability min(1, p/p_hat); after a rejection the target distribution is replaced by
 * norm(max(0, p - p_hat)) and, when no candidate is left, the next token is drawn from it).
 * Reading for a tree whose candidates come from a deterministic top-k expansion
 * (Appendix A): the proposal for a candidate is a point mass on its token, p_hat = 1 there
 * and 0 elsewhere. So, standing at node `cur` with target distribution
 * p = softmax(logits[cur] / temperature):
 *   - the children of cur are tried in ascending node order; child c with token x is
 *     accepted iff u_accept[c] < r(x), r = the current residual distribution;
 *   - a rejected token is removed: r(x) = 0 and r is renormalised (that is
 *     norm(max(0, r - p_hat)) for a point mass); a sibling that repeats a removed token, or
 *     names a token outside the vocabulary, has probability 0;
 *   - an accepted child becomes cur (with a fresh p from its own logits row);
 *   - when no child is accepted (or cur is a leaf) the bonus token is drawn from r by
 *     inverting its cumulative sum in index order with u_bonus:
 *     bonus = min{ j : sum_{i<=j} r_i > u_bonus * sum_i r_i }.
 * Every step is an exact rejection scheme, so the emitted tokens are distributed as the
 * target's own sampling would be.
 *
 * u_accept[T] and u_bonus are uniforms in [0,1) supplied by the caller. *margin receives
 * the smallest distance between a uniform and the threshold it was compared with
 * (accept tests: |u - r(x)|; bonus: distance of u_bonus to the two cumulative sums that
 * bracket it, relative to the total), so that a caller comparing against an fp32
 * implementation can tell a knife-edge decision from a wrong one. */
int oracle_tree_accept_sample(const float* logits, int64_t ld, int32_t V, double temperature,
                              const int32_t* draft, const int32_t* parent, int32_t T,
                              const double* u_accept, double u_bonus, int32_t* accepted_len,
                              int32_t* path, int32_t* bonus, double* margin) {
    int rc = oracle_tree_validate(parent, T);
    if (rc != ORACLE_OK) return rc;
    if (V < 1 || !(temperature > 0.0)) return ORACLE_BAD_SIZE;
    double* e = (double*)malloc((size_t)V * sizeof(double));
    if (!e) return ORACLE_BAD_SIZE;
    for (int32_t k = 0; k < T; ++k) path[k] = -1;
    double mg = 1.0;
    int32_t cur = 0, len = 0;
    path[0] = 0;
    for (;;) {
        const float* row = logits + (int64_t)cur * ld;
        double m = -INFINITY;
        for (int32_t j = 0; j < V; ++j) {
            double z = (double)row[j] / temperature;
            if (z > m) m = z;
        }
        for (int32_t j = 0; j < V; ++j) e[j] = exp((double)row[j] / temperature - m);
        int32_t next = -1;
        for (int32_t c = cur + 1; c < T && next < 0; ++c) {
            if (parent[c] != cur) continue;
            double total = 0.0; /* residual mass, summed afresh */
            for (int32_t j = 0; j < V; ++j) total += e[j];
            const int32_t x = draft[c];
            const double r = (x >= 0 && x < V && total > 0.0) ? e[x] / total : 0.0;
            const double dist = fabs(u_accept[c] - r);
            if (dist < mg) mg = dist;
            if (u_accept[c] < r) next = c;
            else if (x >= 0 && x < V) e[x] = 0.0;
        }
        if (next >= 0) {
            cur = next;
            path[++len] = cur;
            continue;
        }
        double total = 0.0;
        for (int32_t j = 0; j < V; ++j) total += e[j];
        const double target = u_bonus * total;
        double acc = 0.0;
        int32_t pick = -1, last_pos = -1;
        for (int32_t j = 0; j < V; ++j) {
            if (e[j] > 0.0) last_pos = j;
            const double before = acc;
            acc += e[j];
            if (acc > target) {
                pick = j;
                const double d0 = (target - before) / total, d1 = (acc - target) / total;
                if (before > 0.0 && d0 < mg) mg = d0;
                if (d1 < mg) mg = d1;
                break;
            }
        }
        if (pick < 0) pick = last_pos; /* u_bonus * total rounded up to the whole mass */
        *bonus = pick;
        break;
    }
    *accepted_len = len;
    *margin = mg;
    free(e);
    return ORACLE_OK;
}

/* Is (accepted_len, path, bonus) an outcome of the stochastic acceptance above when every
 * comparison of a uniform with its threshold is allowed to be off by `eps` (absolute, in
 * probability)? The walk is replayed along the claimed path with the same rule, same order,
 * same fp64 arithmetic as oracle_tree_accept_sample:
 *   - a child tried before the claimed next node must have been rejected: u >= r(x) - eps;
 *   - the claimed next node must be a child of the current one, accepted: u < r(x) + eps;
 *   - after the last node of the path every child must have been rejected, and the bonus
 *     token must carry weight and bracket the target: with C the cumulative sum of the
 *     residual r in index order, C(bonus-1) - eps <= u_bonus and u_bonus < C(bonus) + eps.
 * With eps = 0 exactly one outcome passes: the one oracle_tree_accept_sample returns (except
 * that a u_bonus so close to 1 that u_bonus * total rounds up to the whole mass makes that
 * routine fall back to the last weighted token; here any eps > 0 admits it). An fp32
 * implementation whose probabilities are within eps of the exact ones must pass with that eps.
 * *worst receives the largest amount by which a comparison was on the wrong side (<= 0 when
 * every exact comparison agrees). Returns ORACLE_OK or ORACLE_BAD_PATH. */
int oracle_tree_accept_sample_check(const float* logits, int64_t ld, int32_t V, double temperature,
                                    const int32_t* draft, const int32_t* parent, int32_t T,
                                    const double* u_accept, double u_bonus, int32_t accepted_len,
                                    const int32_t* path, int32_t bonus, double eps, double* worst) {
    int rc = oracle_tree_validate(parent, T);
    if (rc != ORACLE_OK) return rc;
    if (V < 1 || !(temperature > 0.0)) return ORACLE_BAD_SIZE;
    if (accepted_len < 0 || accepted_len >= T || path[0] != 0) return ORACLE_BAD_PATH;
    double* e = (double*)malloc((size_t)V * sizeof(double));
    if (!e) return ORACLE_BAD_SIZE;
    double w = -1.0;
    int ok = 1;
    for (int32_t k = 0; k <= accepted_len && ok; ++k) {
        const int32_t cur = path[k];
        const int32_t want = (k < accepted_len) ? path[k + 1] : -1;
        if (cur < 0 || cur >= T) { ok = 0; break; }
        if (want >= 0 && (want <= cur || want >= T || parent[want] != cur)) { ok = 0; break; }
        const float* row = logits + (int64_t)cur * ld;
        double m = -INFINITY;
        for (int32_t j = 0; j < V; ++j) {
            double z = (double)row[j] / temperature;
            if (z > m) m = z;
        }
        for (int32_t j = 0; j < V; ++j) e[j] = exp((double)row[j] / temperature - m);
        for (int32_t c = cur + 1; c < T; ++c) {
            if (parent[c] != cur) continue;
            double total = 0.0;
            for (int32_t j = 0; j < V; ++j) total += e[j];
            const int32_t x = draft[c];
            const double r = (x >= 0 && x < V && total > 0.0) ? e[x] / total : 0.0;
            if (c == want) {
                const double off = u_accept[c] - r; /* accepted needs u < r */
                if (off > w) w = off;
                if (!(u_accept[c] < r + eps)) ok = 0;
                break;
            }
            const double off = r - u_accept[c]; /* rejected needs u >= r */
            if (off > w) w = off;
            if (!(u_accept[c] >= r - eps)) ok = 0;
            if (x >= 0 && x < V) e[x] = 0.0;
        }
        if (want < 0 && ok) {
            double total = 0.0;
            for (int32_t j = 0; j < V; ++j) total += e[j];
            if (bonus < 0 || bonus >= V || !(e[bonus] > 0.0) || !(total > 0.0)) { ok = 0; break; }
            double before = 0.0;
            for (int32_t j = 0; j < bonus; ++j) before += e[j];
            const double lo = before / total, hi = (before + e[bonus]) / total;
            const double off_lo = lo - u_bonus;  /* needs C(bonus-1) <= u */
            const double off_hi = u_bonus - hi;  /* needs u < C(bonus)  */
            if (off_lo > w) w = off_lo;
            if (off_hi > w) w = off_hi;
            if (!(u_bonus >= lo - eps) || !(u_bonus < hi + eps)) ok = 0;
        }
    }
    for (int32_t k = accepted_len + 1; k < T && ok; ++k)
        if (path[k] != -1) ok = 0;
    *worst = w;
    free(e);
    return ok ? ORACLE_OK : ORACLE_BAD_PATH;
}

/* ---------------------------------------------------------------------------------------
 * Draft-tree construction. Section 3.1 adopts the context-aware dynamic draft tree of
 * EAGLE-2; Appendix A fixes its hyper-parameters (30 draft tokens, depth 3, 8 nodes kept
 * per expansion). The published procedure, restated:
 *   - every tree node carries the sum of the draft model's log-probabilities along its
 *     path from the root (its score; the root has 0);
 *   - an expansion step takes the current frontier (the root at first, then K nodes),
 *     gives every frontier node its K most likely next tokens as children (candidates),
 *     child score = frontier node's score + log softmax(draft logits of that node)[token],
 *     and keeps the K best-scored of the new candidates as the next frontier;
 *   - after the last step the N best-scored candidates over all levels are the draft
 *     tree. A child never scores above its parent, so that set is closed under taking
 *     parents; among such closed sets of N nodes it has the largest total probability.
 * The draft model's forward pass is outside this path: its logits are inputs.
 * ------------------------------------------------------------------------------------ */

/* One expansion step for one sequence.
 * logits [F][ld] (V used): draft logits at the F frontier nodes; cum_in [F]: their scores.
 * Candidate f*K + r is the r-th most likely token of frontier node f (larger logit first,
 * equal logits: lower token id first): cand_token, cand_score = cum_in[f] + logit -
 * logsumexp(row f). frontier [min(K, F*K)]: the candidates kept for the next step, i.e.
 * the best by (score descending, candidate index ascending), listed in ascending candidate
 * index. *cut_gap = score of the worst kept candidate minus score of the best dropped one
 * (+inf if nothing is dropped): how far the selection is from flipping. */
int oracle_draft_expand(const float* logits, int64_t ld, int32_t V, const float* cum_in, int32_t F,
                        int32_t K, int32_t* cand_token, double* cand_score, int32_t* frontier,
                        double* cut_gap) {
    if (F < 1 || K < 1 || K > V || K > 64 || F > 64) return ORACLE_BAD_SIZE;
    unsigned char* taken = (unsigned char*)calloc((size_t)V, 1);
    if (!taken) return ORACLE_BAD_SIZE;
    for (int32_t f = 0; f < F; ++f) {
        const float* row = logits + (int64_t)f * ld;
        double m = -INFINITY;
        for (int32_t j = 0; j < V; ++j)
            if ((double)row[j] > m) m = (double)row[j];
        double s = 0.0;
        for (int32_t j = 0; j < V; ++j) s += exp((double)row[j] - m);
        const double lse = m + log(s);
        memset(taken, 0, (size_t)V);
        for (int32_t r = 0; r < K; ++r) {
            int32_t best = -1;
            for (int32_t j = 0; j < V; ++j)
                if (!taken[j] && (best < 0 || row[j] > row[best])) best = j;
            taken[best] = 1;
            cand_token[f * K + r] = best;
            cand_score[f * K + r] = (double)cum_in[f] + ((double)row[best] - lse);
        }
    }
    free(taken);
    const int32_t C = F * K, keep = K < C ? K : C;
    unsigned char kept[64 * 64];
    memset(kept, 0, sizeof kept);
    double worst_kept = INFINITY;
    for (int32_t r = 0; r < keep; ++r) {
        int32_t best = -1;
        for (int32_t c = 0; c < C; ++c)
            if (!kept[c] && (best < 0 || cand_score[c] > cand_score[best])) best = c;
        kept[best] = 1;
        worst_kept = cand_score[best];
    }
    double best_dropped = -INFINITY;
    int32_t n = 0;
    for (int32_t c = 0; c < C; ++c) {
        if (kept[c]) frontier[n++] = c;
        else if (cand_score[c] > best_dropped) best_dropped = cand_score[c];
    }
    *cut_gap = (keep < C) ? worst_kept - best_dropped : INFINITY;
    return ORACLE_OK;
}

/* The final selection for one sequence.
 * M candidates (all levels, in the order they were created): token, score (fp32 as the
 * caller stores it; compared as such), parent candidate (-1: child of the root, else an
 * earlier candidate). Picks the min(N, M) best by (score descending, index ascending) and
 * emits them as a tree in ascending candidate order behind the root (node 0, token
 * root_token): parent[] / tokens[] / node_cand[] (candidate index of each node, -1 for the
 * root) of *T_out = picked + 1 nodes. Parents precede children, and levels stay together
 * when the caller appended candidates level by level.
 * ORACLE_BAD_PARENT: a cand_parent outside [-1, index), or a picked candidate whose parent
 * was not picked (only possible when a child scores above its parent: not a sum of
 * log-probabilities). */
int oracle_draft_tree_build(const int32_t* cand_token, const float* cand_score, const int32_t* cand_parent,
                            int32_t M, int32_t N, int32_t root_token, int32_t* parent, int32_t* tokens,
                            int32_t* node_cand, int32_t* T_out) {
    if (M < 1 || M > 4096 || N < 1 || N > 63) return ORACLE_BAD_SIZE;
    for (int32_t c = 0; c < M; ++c)
        if (cand_parent[c] < -1 || cand_parent[c] >= c) return ORACLE_BAD_PARENT;
    unsigned char* picked = (unsigned char*)calloc((size_t)M, 1);
    int32_t* node_of = (int32_t*)malloc((size_t)M * sizeof(int32_t));
    if (!picked || !node_of) return ORACLE_BAD_SIZE;
    const int32_t take = N < M ? N : M;
    for (int32_t r = 0; r < take; ++r) {
        int32_t best = -1;
        for (int32_t c = 0; c < M; ++c)
            if (!picked[c] && (best < 0 || cand_score[c] > cand_score[best])) best = c;
        picked[best] = 1;
    }
    int rc = ORACLE_OK;
    int32_t t = 0;
    parent[0] = -1;
    tokens[0] = root_token;
    node_cand[0] = -1;
    for (int32_t c = 0; c < M && rc == ORACLE_OK; ++c) {
        if (!picked[c]) continue;
        ++t;
        node_of[c] = t;
        const int32_t pc = cand_parent[c];
        if (pc >= 0 && !picked[pc]) rc = ORACLE_BAD_PARENT;
        parent[t] = pc < 0 ? 0 : node_of[pc];
        tokens[t] = cand_token[c];
        node_cand[t] = c;
    }
    *T_out = take + 1;
    free(picked);
    free(node_of);
    return rc;
}

/* Compression attention of the vision adaptor (Section 4.1, Fig. 3: a small fixed number of
 * trained query vectors cross-attend to the image's visual features, the keys and values;
 * every query sees every image embedding; Eq. 1 with a softmax scale).
 * The projections and the rest of the adaptor's encoder layer are outside this path: q, K, V
 * arrive already projected.
 *
 *   s_j = scale * <q[i,h,:], K[kv,j,:]>,  j = 0 .. r-1,  kv = h / (Hq / Hkv)
 *   out[i,h,:] = sum_j exp(s_j - max s) V[kv,j,:] / sum_j exp(s_j - max s)      (ascending j)
 *
 * q [nq][Hq][d] float, out [nq][Hq][d] double; K / V addressed like the tree attention's
 * caches (contiguous or paged); r >= 1 keys; slots beyond r are never read. */
int oracle_compress_attention(const float* q, const float* k_cache, const float* v_cache, int32_t nq,
                              int32_t Hq, int32_t Hkv, int32_t d, int32_t r, double scale, int32_t paged,
                              int64_t stride_head, int64_t stride_tok, const int32_t* block_table,
                              int32_t block_size, int64_t stride_block, double* out) {
    if (nq < 1 || Hkv < 1 || Hq % Hkv != 0 || d < 1 || r < 1) return ORACLE_BAD_SIZE;
    oracle_kv_layout L = {paged, stride_head, stride_tok, block_table, block_size, stride_block};
    const int32_t group = Hq / Hkv;
    double* s = (double*)malloc(sizeof(double) * (size_t)r);
    if (!s) return ORACLE_BAD_SIZE;
    for (int32_t i = 0; i < nq; ++i)
        for (int32_t h = 0; h < Hq; ++h) {
            const int32_t kv = h / group;
            const float* qv = q + ((int64_t)i * Hq + h) * d;
            double m = -INFINITY;
            for (int32_t j = 0; j < r; ++j) {
                const float* kj = k_cache + token_offset(&L, kv, j);
                double dot = 0.0;
                for (int32_t c = 0; c < d; ++c) dot += (double)qv[c] * (double)kj[c];
                s[j] = scale * dot;
                if (s[j] > m) m = s[j];
            }
            double* o = out + ((int64_t)i * Hq + h) * d;
            for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
            double denom = 0.0;
            for (int32_t j = 0; j < r; ++j) {
                const double w = exp(s[j] - m);
                const float* vj = v_cache + token_offset(&L, kv, j);
                denom += w;
                for (int32_t c = 0; c < d; ++c) o[c] += w * (double)vj[c];
            }
            for (int32_t c = 0; c < d; ++c) o[c] /= denom;
        }
    free(s);
    return ORACLE_OK;
}
