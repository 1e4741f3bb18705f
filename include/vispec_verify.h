/*
 * libvispec_verify — tree verification for speculative decoding on MI355X (gfx950).
 *
 * The target model of a speculative decoder scores a whole draft token tree in one
 * forward pass and keeps the longest accepted root-to-node path (paper Section 3.1;
 * image embeddings are ordinary context positions, Section 3.2, so the KV cache the
 * tree attends to is dominated by thousands of image tokens). This library is that
 * step's data-parallel part:
 *
 *   vs_tree_mask_build        ancestor-or-self bit masks and depths of a draft tree
 *   vs_tree_verify_attention  softmax attention (paper Eq. 1, with the usual scale)
 *                             of the T tree queries over prefix + visible tree keys
 *   vs_tree_accept            vocab-wide argmax per node, longest accepted path and
 *                             bonus token (Section 3.1 at temperature 0)
 *   vs_tree_accept_sample     the same walk at a temperature > 0: accept with probability
 *                             min(1, p/p_hat), residual resampling (Section 3.1)
 *   vs_draft_expand /         builds the draft tree that the next step verifies: top-K
 *   vs_draft_tree_build       expansion scored by cumulative log-probability, best-N selection
 *                             (Section 3.1's dynamic draft tree, Appendix A's parameters)
 *   vs_compress_attention     the vision adaptor's attention: a few learnable queries over the
 *                             image embeddings (Section 4.1, Fig. 3)
 *   vs_tree_kv_commit         keeps the accepted path's K/V rows, in order, behind the
 *                             prefix of the pre-allocated cache (Section 3.1, Appendix A)
 *
 * Conventions
 *   - C ABI, no exceptions cross it. Every function returns an int32 vs_error
 *     (0 = VS_OK, negative = error found on the host before anything was enqueued).
 *   - Unless a parameter says "host", every data pointer is a DEVICE pointer owned by
 *     the caller; the library neither allocates nor frees device memory. Scratch
 *     comes from a caller-supplied workspace sized by the matching *_workspace_bytes.
 *   - Calls enqueue kernels on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and return without synchronising. Outputs are valid once the
 *     stream has been synchronised. Calls that share a workspace must be ordered on
 *     one stream.
 *   - Data-dependent problems (a malformed tree, a prefix length outside the cache, a
 *     block id outside the pool) cannot be seen by the host. The kernels report them
 *     per sequence in the optional device array `status` (vs_status, 0 = ok), never
 *     read out of bounds, and leave that sequence's outputs unspecified.
 *   - A tree has T nodes, 1 <= T <= 64. Node 0 is the root: the last committed token,
 *     whose K/V are not yet part of the prefix. parent[0] = -1 and 0 <= parent[i] < i.
 */
#ifndef VISPEC_VERIFY_H
#define VISPEC_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VS_VERSION 100 /* major*10000 + minor*100 + patch */
#define VS_MAX_TREE 64

typedef enum vs_error {
    VS_OK = 0,
    VS_ERR_NULL = -1,      /* a required pointer is NULL */
    VS_ERR_SHAPE = -2,     /* B < 1, T outside [1,64], Hq % Hkv != 0, unsupported head_dim, V < 1 ... */
    VS_ERR_DTYPE = -3,     /* dtype is neither VS_BF16 nor VS_F32 */
    VS_ERR_WORKSPACE = -4, /* workspace NULL or smaller than *_workspace_bytes reports */
    VS_ERR_HIP = -5,       /* the HIP runtime refused a launch */
    VS_ERR_LAYOUT = -6,    /* strides / alignment / paging parameters not supported */
    VS_ERR_NO_DEVICE = -7  /* no usable gfx950 device */
} vs_error;

/* Per-sequence result codes written by the kernels into `status`. */
typedef enum vs_status {
    VS_STATUS_OK = 0,
    VS_STATUS_BAD_ROOT = 1,   /* parent[0] != -1 */
    VS_STATUS_BAD_PARENT = 2, /* some parent[i], i >= 1, outside [0, i) */
    VS_STATUS_BAD_PREFIX = 3, /* prefix_len < 0, > max_prefix_len, or prefix_len + T beyond the cache */
    VS_STATUS_BAD_BLOCK = 4,  /* a block-table entry in use lies outside [0, num_blocks) */
    VS_STATUS_BAD_PATH = 5,   /* accepted_len outside [0, T) or path not 0 followed by increasing node ids */
    VS_STATUS_BAD_CANDIDATE = 6 /* draft tree: cand_parent outside [-1, index), or a selected candidate whose
                                   parent was not selected (a child scoring above its parent) */
} vs_status;

typedef enum vs_dtype { VS_BF16 = 0, VS_F32 = 1 } vs_dtype;

/* Which attention kernel to run. AUTO picks MFMA for bf16 and GENERIC for fp32. */
typedef enum vs_attn_impl { VS_IMPL_AUTO = 0, VS_IMPL_GENERIC = 1, VS_IMPL_MFMA = 2 } vs_attn_impl;

/* How the MFMA kernels are scheduled. LOOP streams 64-key tiles through LDS and runs a tile's
 * three stages (scores, softmax, output update) back to back; PIPELINED overlaps the matrix-core
 * work of the neighbouring tiles with the current tile's softmax (launches with many units);
 * RESIDENT keeps a split's whole key range (at most 192 keys) in LDS and splits the
 * keys once more among the waves of a workgroup (latency-bound launches with few units);
 * BALANCED is the pipelined kernel on a batch whose sequences differ in length: the kernels read
 * the prefix lengths, lay all sequences' keys end to end and give every workgroup an equal share
 * of them (a share may end one sequence and begin the next), instead of cutting every sequence
 * into the same number of splits sized for the longest allowed one (at most 64 sequences; bf16;
 * `num_splits`, if not 0, is the number of shares per KV head and row group, at most 64).
 * Same results up to fp32 rounding. AUTO chooses from the shape. */
typedef enum vs_attn_schedule {
    VS_SCHED_AUTO = 0,
    VS_SCHED_LOOP = 1,
    VS_SCHED_PIPELINED = 2,
    VS_SCHED_RESIDENT = 3,
    VS_SCHED_BALANCED = 4
} vs_attn_schedule;

int32_t vs_version(void);
const char* vs_strerror(int32_t err);       /* static string for a vs_error */
const char* vs_status_string(int32_t code); /* static string for a vs_status */

/* Host twin of the kernels' tree check: `parent` is a HOST array of T entries.
 * Returns the vs_status the kernels would report for this tree (VS_STATUS_OK,
 * VS_STATUS_BAD_ROOT, VS_STATUS_BAD_PARENT), or VS_ERR_NULL / VS_ERR_SHAPE. */
int32_t vs_tree_validate_host(const int32_t* parent, int32_t T);

/*
 * Ancestor masks of B draft trees (Section 3.1: the draft tree proposes several
 * candidate tokens per position; a node may attend to itself and its ancestors only).
 *   parent  [B,T] int32   in   parent[b][0] = -1, 0 <= parent[b][i] < i
 *   mask    [B,T] uint64  out  bit j of mask[b][i] set iff j == i or j is an ancestor of i
 *   depth   [B,T] int32   out  edges from the root (root = 0)
 *   status  [B]   int32   out, optional (may be NULL)
 * An invalid tree gets its status set and its mask/depth rows zero-filled.
 */
int32_t vs_tree_mask_build(const int32_t* parent, int32_t B, int32_t T, uint64_t* mask,
                           int32_t* depth, int32_t* status, void* stream);

/*
 * Attention problem description (host struct, read during the call only).
 *
 * Query head h reads KV head h / (Hq / Hkv). Each sequence's cache holds its
 * prefix_len[b] context tokens (image and text alike) followed by the T tree nodes'
 * own K/V at logical token slots prefix_len[b] .. prefix_len[b]+T-1, written by the
 * caller before the call (the pre-allocated cache of the paper's Appendix A used the
 * way a verify forward uses it). Whatever lies beyond slot prefix_len+T-1 is never
 * read into the result. All K/V values in slots that are read must be finite.
 *
 * Element offset of (sequence b, KV head kv, logical token t, channel c):
 *   contiguous (paged = 0):  b*stride_seq + kv*stride_head + t*stride_tok + c
 *   paged      (paged = 1):  blk*stride_block + kv*stride_head + (t % block_size)*stride_tok + c
 *                            with blk = block_table[b*max_blocks + t / block_size]
 * The same layout applies to k_cache and v_cache. Channels are contiguous.
 */
typedef struct vs_attn_desc {
    int32_t B;              /* sequences, >= 1 */
    int32_t T;              /* tree nodes per sequence incl. root, 1..64 */
    int32_t Hq;             /* query heads */
    int32_t Hkv;            /* KV heads, divides Hq */
    int32_t d;              /* head_dim: 64 or 128 */
    int32_t dtype;          /* vs_dtype of q, k_cache, v_cache and out */
    float softmax_scale;    /* > 0, multiplies q.k before softmax (Eq. 1 omits it) */
    int32_t max_prefix_len; /* host-side upper bound on every prefix_len[b]; sizes the launch */
    int32_t paged;          /* 0 contiguous, 1 paged */
    int32_t block_size;     /* paged: tokens per block, power of two >= 16 */
    int32_t max_blocks;     /* paged: row length of block_table */
    int32_t num_blocks;     /* paged: blocks in the pool (for the bounds check) */
    int64_t capacity;       /* contiguous: token slots per sequence (for the bounds check) */
    int64_t stride_seq;     /* contiguous */
    int64_t stride_block;   /* paged */
    int64_t stride_head;
    int64_t stride_tok;
    const int32_t* block_table; /* paged: device [B, max_blocks] */
    int32_t impl;           /* vs_attn_impl */
    int32_t num_splits;     /* key splits per (sequence, KV head); 0 = choose */
    int32_t rows_per_wave;  /* MFMA path: 32-row blocks per wave, 1 or 2; 0 = choose */
    int32_t waves_per_group; /* MFMA path: waves per workgroup, 1, 2, 4 or 8; 0 = choose */
    int32_t schedule;       /* MFMA path: vs_attn_schedule; PIPELINED needs rows_per_wave 0 or 1
                               and waves_per_group 0, 4 or 8; RESIDENT needs rows_per_wave 0 or 1 and
                               waves_per_group 0 or 8, and never puts more than 192 keys into a split
                               (num_splits is raised where it asks for more) */
} vs_attn_desc;

/* What a call with this descriptor would launch (for tests and reports). */
typedef struct vs_attn_plan {
    int32_t impl;            /* VS_IMPL_GENERIC or VS_IMPL_MFMA */
    int32_t num_splits;      /* upper bound on key splits per (sequence, KV head); BALANCED: shares per (KV head, row group) */
    int32_t keys_per_split;  /* BALANCED: 0, the shares are sized from the prefix lengths at run time */
    int32_t row_groups;      /* workgroups that share one (sequence, KV head, split) */
    int32_t waves_per_group;
    int32_t rows_per_wave;   /* 32-row blocks per wave (MFMA path) */
    int32_t workgroups;      /* main kernel grid size */
    int32_t combine;         /* 1 if a split-combine kernel follows */
    int32_t schedule;        /* VS_SCHED_LOOP, _PIPELINED, _RESIDENT or _BALANCED (MFMA path), else 0 */
} vs_attn_plan;

int32_t vs_attention_plan(const vs_attn_desc* desc, vs_attn_plan* plan); /* both host */
size_t vs_attention_workspace_bytes(const vs_attn_desc* desc);           /* 0 on invalid desc */

/*
 * Tree-masked attention (Eq. 1 restricted by tree ancestry; Sections 3.1-3.2).
 * For node i of sequence b and query head h the visible keys are all prefix tokens
 * plus the tree slots of i's ancestor-or-self set; the result is
 *   out[b,i,h,:] = sum_j softmax_j(softmax_scale * q[b,i,h,:].K[j,:]) V[j,:]
 * with fp32 accumulation, rounded to the storage dtype (nearest even).
 *   q           [B,T,Hq,d]  in, dense
 *   k_cache, v_cache        in, layout per desc
 *   prefix_len  [B] int32   in
 *   tree_parent [B,T] int32 in
 *   tree_mask   [B,T] uint64 in, optional: vs_tree_mask_build's output for the same
 *               trees; NULL = derive the masks from tree_parent inside the kernel
 *   out         [B,T,Hq,d]  out, dense
 *   status      [B] int32   out, optional
 *   workspace   device scratch of at least vs_attention_workspace_bytes(desc) bytes
 *               (may be NULL when that is 0), 256-byte aligned
 * bf16 MFMA path needs 16-byte aligned q/k/v/out and strides that are multiples of 8.
 */
int32_t vs_tree_verify_attention(const vs_attn_desc* desc, const void* q, const void* k_cache,
                                 const void* v_cache, const int32_t* prefix_len,
                                 const int32_t* tree_parent, const uint64_t* tree_mask, void* out,
                                 int32_t* status, void* workspace, size_t workspace_bytes,
                                 void* stream);

/*
 * Compression attention of the vision adaptor (Section 4.1, Fig. 3: the adaptor owns a small,
 * fixed number of trained query vectors; the image's visual features are the keys and the values
 * of its attention, whose outputs are the few compressed image tokens the draft model reads;
 * Eq. 1 with the softmax scale). Every query sees every image embedding and nothing else. The adaptor's projections and the rest of its
 * encoder layer are outside this library: q, k, v arrive projected.
 * The descriptor is read as for vs_tree_verify_attention with these meanings: T = number of
 * learnable queries (1..64; the paper studies 1 to 64), max_prefix_len = the largest kv_len
 * (>= 1), k / v = the image embeddings' keys and values in either cache layout.
 *   q        [B,T,Hq,d]  in  (a caller with one shared query set passes B copies)
 *   kv_len   [B] int32   in, number of image embeddings of each image, 1 <= kv_len <= max_prefix_len;
 *            anything else is reported as VS_STATUS_BAD_PREFIX
 *   out      [B,T,Hq,d]  out, the compressed image tokens before the output projection
 *   status, workspace (vs_compress_attention_workspace_bytes), stream: as above
 * Runs the same kernels as the verification call (no tree slots, no mask).
 */
size_t vs_compress_attention_workspace_bytes(const vs_attn_desc* desc);     /* 0 on invalid desc */

int32_t vs_compress_attention(const vs_attn_desc* desc, const void* q, const void* k, const void* v,
                              const int32_t* kv_len, void* out, int32_t* status, void* workspace,
                              size_t workspace_bytes, void* stream);

size_t vs_accept_workspace_bytes(int32_t B, int32_t T, int32_t V);

/*
 * Greedy acceptance (Section 3.1 at temperature 0: a draft token is kept iff it is the
 * target's argmax at its parent; the token after the last kept node is that node's own
 * argmax. The acceptance length counts draft tokens only, Section 5.1 "Metrics").
 *   logits       [B,T,ld_logits] fp32 in; row (b,i) = target logits at node i; ld_logits >= V
 *   draft_tokens [B,T] int32 in; entry 0 (the root's committed token) is ignored
 *   parent       [B,T] int32 in
 *   accepted_len [B] int32 out; depth of the deepest accepted node (ties: lowest index)
 *   path         [B,T] int32 out; path[b][0..accepted_len[b]] = root .. that node, rest -1
 *   bonus_token  [B] int32 out; argmax at the last node of the path
 *   row_argmax   [B,T] int32 out, optional; first index of each row's maximum
 *                (strict '>' scan: ties and signed zeros keep the lowest index, NaN never
 *                displaces a value, a NaN in column 0 is never displaced)
 *   status       [B] int32 out, optional
 *   workspace    at least vs_accept_workspace_bytes(B,T,V) bytes, 256-byte aligned
 */
int32_t vs_tree_accept(const float* logits, int64_t ld_logits, int32_t V,
                       const int32_t* draft_tokens, const int32_t* parent, int32_t B, int32_t T,
                       int32_t* accepted_len, int32_t* path, int32_t* bonus_token,
                       int32_t* row_argmax, int32_t* status, void* workspace,
                       size_t workspace_bytes, void* stream);

/*
 * vs_tree_accept for callers that cannot allocate or hand over device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments, results and error
 * codes as vs_tree_accept, minus the workspace: the per-chunk scan results live in a static device
 * array inside the library (VS_ACCEPT_NOALLOC_MAX_BYTES per GPU, held until the process ends). The
 * call allocates nothing and frees nothing.
 *   - Sizes whose workspace would exceed the array (vs_accept_workspace_bytes(B,T,V) >
 *     VS_ACCEPT_NOALLOC_MAX_BYTES, about 131000 (row, 4096-logit chunk) pairs; C5's 16 x 60 rows of
 *     152064 logits need 292 KB) return VS_ERR_WORKSPACE: use vs_tree_accept for those.
 *   - All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different
 *     streams, different threads) race and must be ordered by the caller. Calls on different
 *     GPUs are independent. Nothing in the array has to be cleared between calls.
 *   - The first call on a device looks up the array's address (no allocation); make it outside
 *     graph capture.
 */
#define VS_ACCEPT_NOALLOC_MAX_BYTES (1u << 20)
int32_t vs_tree_accept_noalloc(const float* logits, int64_t ld_logits, int32_t V,
                               const int32_t* draft_tokens, const int32_t* parent, int32_t B, int32_t T,
                               int32_t* accepted_len, int32_t* path, int32_t* bonus_token,
                               int32_t* row_argmax, int32_t* status, void* stream);

size_t vs_accept_sample_workspace_bytes(int32_t B, int32_t T, int32_t V); /* 0 for unsupported sizes */

/*
 * Stochastic acceptance (Section 3.1: a draft token is accepted with probability
 * min(1, p/p_hat); after a rejection the target distribution becomes norm(max(0, p - p_hat)),
 * and when no candidate is left the next token is drawn from it). The candidates of a tree
 * built by deterministic top-k expansion (Appendix A) are point-mass proposals, so, standing
 * at a node with residual distribution r (initially softmax(logits / temperature) of that
 * node's row): its children are tried in ascending node order; child c with token x is
 * accepted iff u_accept[c] < r(x) and becomes the current node; a rejected token is removed
 * from r, which is renormalised (a sibling repeating a removed token, or naming a token
 * outside [0, V), has probability 0); when no child is accepted the bonus token is
 * min{ j : sum_{i<=j} r_i > u_bonus * sum_i r_i }. The emitted tokens are distributed exactly
 * as sampling from the target would distribute them. The random numbers are inputs, so the
 * call is a deterministic function of its arguments.
 *   logits       [B,T,ld_logits] fp32 in; every row needs at least one finite entry, -inf
 *                entries have probability 0, no NaN; ld_logits >= V; V <= 8388608
 *   temperature  > 0, finite
 *   draft_tokens [B,T] int32 in; entry 0 is ignored
 *   parent       [B,T] int32 in
 *   u_accept     [B,T] fp32 in, uniform in [0,1); entry 0 is ignored
 *   u_bonus      [B] fp32 in, uniform in [0,1)
 *   accepted_len [B] int32 out; number of accepted draft tokens
 *   path         [B,T] int32 out; path[b][0..accepted_len[b]] = root .. last accepted node, rest -1
 *   bonus_token  [B] int32 out
 *   status       [B] int32 out, optional
 *   workspace    at least vs_accept_sample_workspace_bytes(B,T,V) bytes, 256-byte aligned
 * Arithmetic is fp32 (exp2 of the hardware, sums over 4096-entry chunks merged per row), so a
 * uniform that lies within ~1e-5 of its threshold may fall on the other side than in exact
 * arithmetic; either outcome is a valid draw.
 */
int32_t vs_tree_accept_sample(const float* logits, int64_t ld_logits, int32_t V, float temperature,
                              const int32_t* draft_tokens, const int32_t* parent,
                              const float* u_accept, const float* u_bonus, int32_t B, int32_t T,
                              int32_t* accepted_len, int32_t* path, int32_t* bonus_token,
                              int32_t* status, void* workspace, size_t workspace_bytes,
                              void* stream);

/*
 * Draft-tree construction (Section 3.1: the context-aware dynamic draft tree of EAGLE-2;
 * Appendix A: N = 30 draft tokens, depth 3, K = 8 nodes kept per expansion). A candidate's
 * score is the sum of the draft model's log-probabilities on its path from the root. The draft
 * model itself is not part of this library: the caller runs it on the current frontier and
 * passes its logits. Candidates of all levels live in three caller-owned arrays
 * cand_token / cand_score / cand_parent of cand_capacity entries per sequence.
 *
 * vs_draft_expand, one expansion step:
 *   logits        [B,F,ld_logits] fp32 in; row (b,f) = draft logits at frontier node f; no NaN;
 *                 1 <= F <= 64, 1 <= K <= 16, F*K <= 1024, K <= V <= ld_logits
 *   cum_in        [B,F] fp32 in, scores of the frontier nodes; NULL = all 0 (the root)
 *   frontier_cand [B,F] int32 in, candidate index of each frontier node; NULL = all -1 (the root)
 *   cand_base     where this step's F*K candidates go: candidate cand_base + f*K + r is the r-th
 *                 most likely token of frontier node f (larger logit first, equal logits: lower
 *                 token id first); cand_base + F*K <= cand_capacity
 *   cand_token / cand_score / cand_parent  [B,cand_capacity] out at those positions:
 *                 token id; cum_in + logit - logsumexp(row); frontier_cand of the node
 *   next_frontier_cand [B,min(K,F*K)] int32 out: the step's best candidates by (score descending,
 *                 index ascending), listed in ascending candidate index
 *   next_cum      [B,min(K,F*K)] fp32 out: their scores (the next step's cum_in)
 *   workspace     at least vs_draft_expand_workspace_bytes(B,F,V,K) bytes, 256-byte aligned
 * Tokens are exact; scores are fp32 (log-sum-exp over 4096-entry chunks), so two candidates
 * whose exact scores differ by less than ~1e-5 may swap places at the cut.
 *
 * vs_draft_tree_build, the final selection over the first M candidates (1 <= M <= 2048,
 * 1 <= N <= 63; scores without NaN): the min(N, M) best by (score descending, index ascending)
 * become nodes 1.. in ascending candidate order behind the root (node 0). With candidates
 * appended level by level that is level order, and a parent always precedes its children.
 *   root_token    [B] int32 in or NULL (then draft_tokens[b][0] = -1)
 *   parent        [B,N+1] int32 out, the tree_parent array of the verification calls
 *   draft_tokens  [B,N+1] int32 out
 *   node_cand     [B,N+1] int32 out, candidate index of every node (-1 for the root)
 *   num_nodes     [B] int32 out: min(N, M) + 1; entries beyond it are -1; 0 on a bad status
 *   status        [B] int32 out, optional: VS_STATUS_BAD_CANDIDATE if a cand_parent is not in
 *                 [-1, own index) or the selection is not closed under taking parents
 */
size_t vs_draft_expand_workspace_bytes(int32_t B, int32_t F, int32_t V, int32_t K); /* 0 for unsupported sizes */

int32_t vs_draft_expand(const float* logits, int64_t ld_logits, int32_t V, const float* cum_in,
                        const int32_t* frontier_cand, int32_t B, int32_t F, int32_t K,
                        int32_t cand_base, int32_t cand_capacity, int32_t* cand_token,
                        float* cand_score, int32_t* cand_parent, int32_t* next_frontier_cand,
                        float* next_cum, void* workspace, size_t workspace_bytes, void* stream);

int32_t vs_draft_tree_build(const int32_t* cand_token, const float* cand_score,
                            const int32_t* cand_parent, int32_t B, int32_t M, int32_t cand_capacity,
                            int32_t N, const int32_t* root_token, int32_t* parent,
                            int32_t* draft_tokens, int32_t* node_cand, int32_t* num_nodes,
                            int32_t* status, void* stream);

/*
 * KV caches of one or more layers that share a layout (host struct, read during the call).
 * Element offset of (layer l, sequence b, KV head kv, logical token t, channel c) in k_cache
 * and in v_cache: l*stride_layer + the offset vs_attn_desc documents. Every stride times
 * the element size, and d times the element size, must be a multiple of 16 bytes; the
 * cache pointers must be 16-byte aligned.
 */
typedef struct vs_kv_desc {
    int32_t B;              /* sequences */
    int32_t T;              /* tree nodes per sequence incl. root, 1..64 */
    int32_t Hkv;
    int32_t d;
    int32_t dtype;          /* vs_dtype of the caches */
    int32_t num_layers;     /* >= 1 */
    int64_t stride_layer;   /* elements between consecutive layers' caches */
    int32_t paged, block_size, max_blocks, num_blocks;
    int64_t capacity, stride_seq, stride_block, stride_head, stride_tok;
    const int32_t* block_table; /* paged: device [B, max_blocks], shared by all layers */
} vs_kv_desc;

/*
 * Commit of the accepted path (Section 3.1: draft tokens after the first rejected one are
 * discarded; Appendix A: the cache is pre-allocated, so the accepted tokens' rows move).
 * Before the call sequence b's cache holds prefix_len[b] context tokens and node i's K/V at
 * logical slot prefix_len[b] + i. For every layer and KV head, the K and V rows of node
 * path[b][k] move to slot prefix_len[b] + k, k = 1 .. accepted_len[b] (bit-exact copies;
 * slots above prefix_len[b] + accepted_len[b] keep what they held), and
 * new_prefix_len[b] = prefix_len[b] + accepted_len[b] + 1: the context of the next step is the
 * old prefix, the root and the accepted draft tokens in order. The bonus token is not in the
 * cache yet; it is the next step's root.
 *   k_cache, v_cache        in/out, layout per desc
 *   prefix_len     [B] int32     in
 *   path           [B,T] int32   in, as vs_tree_accept writes it
 *   accepted_len   [B] int32     in
 *   new_prefix_len [B] int32     out; must not overlap prefix_len
 *   status         [B] int32     out, optional
 * A sequence with a malformed path, a prefix length beyond the cache or a block id outside
 * the pool is reported in status, keeps its cache and gets new_prefix_len[b] = prefix_len[b].
 */
int32_t vs_tree_kv_commit(const vs_kv_desc* desc, void* k_cache, void* v_cache, const int32_t* prefix_len,
                          const int32_t* path, const int32_t* accepted_len, int32_t* new_prefix_len,
                          int32_t* status, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VISPEC_VERIFY_H */
