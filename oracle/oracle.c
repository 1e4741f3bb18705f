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
