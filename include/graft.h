/*
 * graft.h - C ABI of the hybrid-tree verification hot path for MI355X (gfx950).
 *
 * One decoding round of prune-then-graft speculative decoding verifies a
 * hybrid tree: retained draft nodes plus retrieved continuations appended
 * into the slots pruning released (paper Sec. 3; App. A, Alg. 1 loop body and
 * Alg. 2 last steps).  This library is the data-parallel part of that round:
 *
 *     graft_retrieve         ranked continuation chains to graft
 *     graft_build_tree_mask  flattened parent list -> ancestor masks, positions, paths
 *     graft_tree_attn        tree-masked GQA attention over a paged KV cache (per layer)
 *     graft_accept           greedy acceptance walk
 *
 * and the steps on either side of it in the decoding loop (App. A, Alg. 1 and 2):
 *
 *     graft_prune_select     confidence gates and the choice of the retained draft nodes
 *     graft_matrix_retrieve  the method's retrieval: a rank template filled by lookups
 *                            in the GPU-resident transition matrix, appended to the tree
 *     graft_matrix_update    refresh of the matrix rows from the verification logits
 *     graft_kv_compact       cache update: the accepted path becomes an ordinary prefix
 *
 * Conventions shared by every call
 *  - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *    never allocates, frees or keeps them.  Scratch memory comes from
 *    caller-provided workspaces whose sizes the *_workspace_bytes functions
 *    (pure host functions) return.
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *    only enqueue kernels: they never synchronize and never copy to the host.
 *  - Return value: GRAFT_OK or a GRAFT_ERR_* code.  Arguments are validated on
 *    the host before anything is launched; on error nothing is launched.
 *  - Data-dependent faults (a length out of range, an ill-formed tree) cannot be
 *    seen by the host.  They are reported per sequence in a caller-provided
 *    int32 status[B] device array as GRAFT_STATUS_* bit flags, and the outputs of
 *    that sequence are still fully defined (documented per call).
 *  - Tree convention: node 0 is the root = the current token x_t (retrieval and
 *    drafting are both rooted at it, Sec. 3.2), parent[0] = -1, and every other
 *    node's parent has a smaller index (the flattened parent-child order of
 *    Sec. 3.3).  Nodes >= n_nodes[b] are padding.  K_max <= GRAFT_MAX_NODES.
 *  - Integers are int32_t, masks uint64_t, all arrays dense row-major with the
 *    shapes given in brackets.
 */
#ifndef GRAFT_H
#define GRAFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GRAFT_MAX_NODES   128   /* tree slots per sequence, root included          */
#define GRAFT_MASK_WORDS  2     /* uint64 words per ancestor mask (bit j of word j/64) */
#define GRAFT_MAX_CHAINS  8     /* C: chains returned per sequence                  */
#define GRAFT_MAX_NGRAM   32    /* n_max: longest suffix matched                    */
#define GRAFT_PAGE_SIZE   16    /* tokens per KV page                               */
#define GRAFT_ARGMAX_CHUNKS 16  /* vocabulary chunks per logits row in graft_accept */
#define GRAFT_MAX_SUCCESSORS 16 /* k: successors per row of the transition matrix   */
#define GRAFT_MAX_CHECKPOINTS 16 /* pruning checkpoints per call                     */

/* return codes */
#define GRAFT_OK             0
#define GRAFT_ERR_NULL       1   /* a required pointer is NULL                       */
#define GRAFT_ERR_SHAPE      2   /* a size or stride is outside the supported range  */
#define GRAFT_ERR_DTYPE      3   /* unknown dtype enum                               */
#define GRAFT_ERR_WORKSPACE  4   /* workspace NULL or smaller than *_workspace_bytes */
#define GRAFT_ERR_HIP        5   /* a launch failed; see graft_last_hip_error()      */

/* per-sequence status bit flags (device side) */
#define GRAFT_STATUS_BAD_LENGTH     1  /* ctx_len / tail_len outside [0, L_max] / [0, tail_max] */
#define GRAFT_STATUS_BAD_TREE       2  /* n_nodes outside [1, K_max], parent[0] != -1, or parent[i] not in [0, i) */
#define GRAFT_STATUS_PATH_OVERFLOW  4  /* a path deeper than depth_cap or more leaves than n_leaf_max */

/* element types of Q / K / V / O */
#define GRAFT_F32   0
#define GRAFT_BF16  1

/* Raw hipError_t of the last failed launch on this thread (0 if none). */
int32_t graft_last_hip_error(void);

/* Library version as major*10000 + minor*100 + patch. */
int32_t graft_version(void);

/*
 * graft_retrieve - suffix n-gram lookup over the whole context token buffer.
 *
 * This is the prompt-lookup / suffix-matching form of retrieval that the paper
 * positions its method against (Sec. 3.2 first paragraph) and names as the
 * online n-gram branch to add (Sec. 6, limitations and future work); the
 * chains it returns are what gets grafted into the released slots (Sec. 3.2
 * merge step; the append step of App. A Alg. 2).
 *
 * For sequence b let L = ctx_len[b] and q = ctx[b,0..L) followed by
 * tail[b,0..tail_len[b]) (the tokens on the tree path from below the root to
 * the node the chains will hang from; tail may be NULL = empty).  A position
 * e, 1 <= e <= L-1, is a hit when the longest l <= min(n_max, e) such that
 * ctx[b,e-l..e) equals the last l tokens of q satisfies l >= n_min.  Hits are
 * ranked by (l descending, e descending) - longest match first, most recent
 * first - and for the best C of them the library returns
 *     chain_pos   [B,C]    e                       (-1 if fewer than C hits)
 *     chain_match [B,C]    l                       (0)
 *     chain_len   [B,C]    min(m, L - e)           (0)
 *     chain_tok   [B,C,m]  ctx[b,e..e+chain_len), then -1 padding (all -1)
 *     n_hits      [B]      total number of hits
 * The end of the buffer (e = L) is never a candidate and duplicate
 * continuations are not merged.
 *
 * ctx [B,L_max], ctx_len [B], tail [B,tail_max] or NULL, tail_len [B] or NULL.
 * Requires 1 <= n_min <= n_max <= GRAFT_MAX_NGRAM, 1 <= C <= GRAFT_MAX_CHAINS,
 * m >= 1, B >= 1, L_max >= 1, L_max < 2^30.
 * status[b] = GRAFT_STATUS_BAD_LENGTH if ctx_len[b] or tail_len[b] is out of
 * range; that sequence then reports no hits.
 */
int32_t graft_retrieve(const int32_t* ctx, const int32_t* ctx_len, int32_t B, int32_t L_max,
                       const int32_t* tail, const int32_t* tail_len, int32_t tail_max,
                       int32_t n_min, int32_t n_max, int32_t C, int32_t m,
                       int32_t* chain_tok, int32_t* chain_len, int32_t* chain_pos,
                       int32_t* chain_match, int32_t* n_hits, int32_t* status, void* stream);

/*
 * graft_build_tree_mask - the rebuild step: from the flattened hybrid tree's
 * parent list to the three things the verifier needs, position ids, ancestor
 * masks and the node indices of every candidate path (Sec. 3.3, hybrid-tree
 * verification; App. A Alg. 2, last step).
 *
 *     mask  [B,K_max,GRAFT_MASK_WORDS]  bit j set iff j == i or j is an ancestor of i
 *     depth [B,K_max]                   edges from the root
 *     pos   [B,K_max]                   prefix_len[b] + depth   (position id)
 *     paths [B,n_leaf_max,depth_cap+1]  optional (NULL to skip): one row per leaf
 *                                       in increasing leaf index, node indices
 *                                       root..leaf, -1 padded; unused rows -1
 * Padding nodes get mask 0, depth -1, pos -1.  A leaf deeper than depth_cap
 * gets an all -1 row and leaves beyond n_leaf_max are dropped; both raise
 * GRAFT_STATUS_PATH_OVERFLOW.  An ill-formed tree raises GRAFT_STATUS_BAD_TREE and
 * gives mask 0 and -1 everywhere else for that sequence.
 *
 * parent [B,K_max], n_nodes [B], prefix_len [B].  1 <= K_max <= GRAFT_MAX_NODES;
 * with paths: n_leaf_max >= 1, 0 <= depth_cap < GRAFT_MAX_NODES.
 */
int32_t graft_build_tree_mask(const int32_t* parent, const int32_t* n_nodes, const int32_t* prefix_len,
                              int32_t B, int32_t K_max,
                              uint64_t* mask, int32_t* pos, int32_t* depth,
                              int32_t* paths, int32_t n_leaf_max, int32_t depth_cap,
                              int32_t* status, void* stream);

/*
 * graft_tree_attn - the attention inside the verification pass over the hybrid
 * tree (Sec. 3.3: the target model scores all tree nodes at once under the
 * usual ancestor mask; the long-context runs use scaled dot-product attention,
 * Sec. 3.3, long-context adaptation).  One call = one layer.
 *
 * For sequence b, node i < n_nodes[b], query head h (KV head g = h / (Hq/Hkv)):
 *     S   = {prefix tokens 0..P-1} U {tree slot j : bit j of mask[b,i] set},  P = prefix_len[b]
 *     out[b,i,h,:] = sum_{t in S} softmax_t( scale * q[b,i,h,:] . k_t[g,:] ) * v_t[g,:]
 * i.e. causal attention of node i over the prefix and its own root-to-node
 * path.  Tree slot j is logical token P + j of the sequence: the K/V of all
 * tree tokens, the root's included, sit in the same paged cache right after
 * the prefix.  Rows of padding nodes are written as zeros.  No rotary
 * embedding is applied here: q and k arrive already position-encoded (the
 * position ids come from graft_build_tree_mask).
 *
 * q, out     [B,K_max,Hq,D]   dtype elements
 * k_cache, v_cache            paged; element d of KV head g of the token at
 *                             in-page offset o of physical page p is at index
 *                             p*page_stride + o*token_stride + g*head_stride + d
 *                             (strides in elements; the D elements contiguous)
 * block_table [B,max_pages]   physical page of each logical page; logical token
 *                             t is in page block_table[b, t/page_size] at offset
 *                             t % page_size.  (P + n_nodes[b]) <= max_pages*page_size
 *                             is the caller's responsibility.
 * prefix_len [B], n_nodes [B], mask [B,K_max,GRAFT_MASK_WORDS] (from graft_build_tree_mask)
 * scale                       softmax scale, normally 1/sqrt(D)
 * dtype                       GRAFT_F32: fp32 storage and arithmetic throughout.
 *                             GRAFT_BF16: bf16 storage, fp32 scores/softmax/accumulation,
 *                             probabilities rounded to bf16 for the P.V product; where the
 *                             keys are split over workgroups, each split's normalised
 *                             partial row passes through memory as fp16 scaled by a power
 *                             of two to its largest entry: 11 bits for entries within
 *                             2^-14 of the row's largest (finer than the bf16 rounding of
 *                             the result), an absolute 2^-25 of it below that.
 * workspace                   at least graft_tree_attn_workspace_bytes(...) bytes,
 *                             256-byte aligned; contents are scratch.  The size is 0 (and
 *                             workspace may be NULL) for the fp32 / D = 64 path and where
 *                             the keys of a sequence are not split over workgroups.
 *
 * Requires D in {64,128}, Hq % Hkv == 0, Hq/Hkv <= 16, page_size == GRAFT_PAGE_SIZE,
 * 1 <= K_max <= GRAFT_MAX_NODES, 1 <= max_pages <= 262144 (4 Mi tokens),
 * token_stride, head_stride and page_stride multiples of 8 elements,
 * token_stride < 2^26, all sizes positive.  The workspace size depends on the
 * device the calling thread has current (its compute-unit count picks the split), so
 * graft_tree_attn_workspace_bytes is a host function but not a pure one.
 */
size_t graft_tree_attn_workspace_bytes(int32_t B, int32_t K_max, int32_t Hq, int32_t Hkv, int32_t D,
                                       int32_t max_pages, int32_t dtype);

int32_t graft_tree_attn(const void* q, const void* k_cache, const void* v_cache,
                        int64_t page_stride, int64_t token_stride, int64_t head_stride,
                        const int32_t* block_table, int32_t max_pages,
                        const int32_t* prefix_len, const int32_t* n_nodes, const uint64_t* mask,
                        int32_t B, int32_t K_max, int32_t Hq, int32_t Hkv, int32_t D, int32_t page_size,
                        float scale, int32_t dtype, void* out,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * graft_attn_profile_events - measurement hook for benchmarks (not part of the
 * method).  start_events / stop_events are host arrays of n hipEvent_t created by
 * the caller.  While set, the i-th graft_tree_attn call made afterwards on this
 * host thread (i < n) attaches start_events[i] / stop_events[i] to the dispatch of
 * its main attention kernel (not the split-merge kernel): after the stream has
 * been synchronised their elapsed time is that kernel's own duration.  n = 0
 * clears the hook.  The arrays must stay alive until it is cleared.
 */
int32_t graft_attn_profile_events(void** start_events, void** stop_events, int32_t n);

/*
 * graft_accept - the acceptance step under greedy decoding: the unchanged
 * speculative rule (Sec. 3.3; the path-selection step of App. A Alg. 1;
 * App. B.4) specialised to the greedy setting of the main results (Sec. 4).
 *
 * t*[i] = the target's greedy token after node i.  Two modes:
 *   logits == NULL : target_ids [B,K_max] is an INPUT holding t*.
 *   logits != NULL : logits [B,K_max,V] fp32; t*[i] = index of the first maximum
 *                    of row i (inputs assumed NaN-free) and target_ids is an
 *                    OUTPUT receiving t* (-1 for padding nodes); needs workspace.
 * The root is accepted; node i > 0 is accepted iff its parent is accepted and
 * tokens[b,i] == t*[parent[i]].  best = accepted node of greatest depth not
 * exceeding depth_cap (smallest index on ties).
 *     accept_len [B]              depth of best (root and bonus token not counted)
 *     best_node  [B]
 *     path       [B,depth_cap+1]  node indices root..best, -1 padded
 *     out_tokens [B,depth_cap+1]  tokens of path[1..], then the bonus token t*[best], -1 padded
 * An accepted node deeper than depth_cap raises GRAFT_STATUS_PATH_OVERFLOW.  An
 * ill-formed tree raises GRAFT_STATUS_BAD_TREE with accept_len 0, best_node -1,
 * path/out_tokens (and target_ids in logits mode) all -1.
 *
 * parent, tokens [B,K_max], n_nodes [B].  0 <= depth_cap < GRAFT_MAX_NODES,
 * logits mode: V >= 1, workspace >= graft_accept_workspace_bytes(B,K_max,V).
 */
size_t graft_accept_workspace_bytes(int32_t B, int32_t K_max, int32_t V);

int32_t graft_accept(const int32_t* parent, const int32_t* tokens, const int32_t* n_nodes,
                     const float* logits, int32_t V, int32_t* target_ids,
                     int32_t B, int32_t K_max, int32_t depth_cap,
                     int32_t* accept_len, int32_t* best_node, int32_t* path, int32_t* out_tokens,
                     int32_t* status, void* workspace, size_t workspace_bytes, void* stream);

/*
 * graft_accept_noalloc - graft_accept for callers that cannot allocate device memory or
 * carry a workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, outputs, status flags and error codes as graft_accept
 * without the workspace pair.  In logits mode the argmax partials (one (value, index) pair
 * per GRAFT_ARGMAX_CHUNKS-th of every logits row) go to a 1 MiB array that is part of the
 * library's device image (each GPU the library runs on holds its own copy until the process
 * ends); its address is looked up on the first call per device, on the calling thread's
 * current device.  The call allocates nothing and frees nothing.
 *   - B * K_max <= GRAFT_NOALLOC_MAX_ROWS in logits mode, else GRAFT_ERR_WORKSPACE (nothing is
 *     launched); target_ids mode has no such limit (it needs no scratch).
 *   - GRAFT_ERR_HIP if the array's address cannot be obtained (graft_last_hip_error()).
 *   - All calls on one GPU share the array: calls that may overlap in time on the same GPU
 *     (different streams, different threads) race on it and must be ordered by the caller.
 *     Nothing in it has to start at zero: every entry read by a call is written by that call.
 */
#define GRAFT_NOALLOC_MAX_ROWS 8192

int32_t graft_accept_noalloc(const int32_t* parent, const int32_t* tokens, const int32_t* n_nodes,
                             const float* logits, int32_t V, int32_t* target_ids,
                             int32_t B, int32_t K_max, int32_t depth_cap,
                             int32_t* accept_len, int32_t* best_node, int32_t* path, int32_t* out_tokens,
                             int32_t* status, void* stream);

/*
 * graft_matrix_retrieve - the retrieval branch of the method (Sec. 3.2, the paragraphs
 * on the GPU-resident adjacency matrix and on the stage-adaptive templates:
 * x_u = M[x_F(u), r_u]; App. A.1; the template traversal and append steps of App. A
 * Alg. 2).
 *
 *     M          [V,k]  int32 successor ids, -1 = empty entry (read only)
 *     tpl_parent [N]    parent template node of node u, -1 = the tree's root; < u
 *     tpl_rank   [N]    successor rank r_u, 0 <= r_u < k
 *     n_ret      [B]    template nodes to take for sequence b (a stage's template is a
 *                       prefix of the envelope), 0 <= n_ret[b] <= N
 *     tokens, parent [B,K_max], n_nodes [B]   IN/OUT: the retained draft nodes on entry
 *                       (root = tokens[b,0]); node n_nodes[b] + u receives token x_u and
 *                       parent (tpl_parent[u] < 0 ? 0 : n_nodes[b] + tpl_parent[u]);
 *                       n_nodes[b] grows by n_ret[b].  Entries past the new end are not
 *                       touched.
 * A lookup from a token outside [0,V) or of an empty entry gives -1, and so do all
 * descendants (such nodes stay in the tree; they can never be accepted).
 * status [B]: GRAFT_STATUS_BAD_LENGTH if n_nodes[b] < 1, n_ret[b] outside [0,N] or the
 * tree would exceed K_max; GRAFT_STATUS_BAD_TREE if one of the first n_ret[b] template
 * nodes breaks the rules above.  In both cases the sequence is left as it was.
 *
 * 1 <= N <= GRAFT_MAX_NODES, 1 <= k <= GRAFT_MAX_SUCCESSORS, V >= 1, K_max <= GRAFT_MAX_NODES.
 */
int32_t graft_matrix_retrieve(const int32_t* M, int32_t V, int32_t k,
                              const int32_t* tpl_parent, const int32_t* tpl_rank, int32_t N,
                              const int32_t* n_ret, int32_t B, int32_t K_max,
                              int32_t* tokens, int32_t* parent, int32_t* n_nodes, int32_t* status,
                              void* stream);

/*
 * graft_matrix_update - M[x_i] <- argtop-k(p_{i+1}) for every verified node, accepted
 * or rejected (Sec. 3.3, warm-up and online update, last equation; the matrix update
 * equation and step of App. A Alg. 1).  The order of the probabilities is the order of
 * the logits: no softmax.
 *
 *     tokens [B,K_max], n_nodes [B]   the verified tree
 *     logits [B,K_max,V] fp32         target logits per node (inputs assumed NaN-free)
 *     M      [V,k] int32              IN/OUT: row tokens[b,i] becomes the k ids with the
 *                                     largest logits of node i, largest first, equal
 *                                     logits in order of id (-0.0 equals +0.0)
 *     target_ids [B,K_max]            OUT: the first of the k ids (the greedy token that
 *                                     graft_accept takes as input), -1 for padding nodes
 * Where a token occurs at several nodes the node with the largest (b, i) decides its
 * row; tokens outside [0,V) are skipped.  The same scan of the logits serves the
 * acceptance step: call graft_accept with this target_ids.
 *
 * 1 <= k <= GRAFT_MAX_SUCCESSORS, k <= V, B * K_max <= 65536,
 * workspace >= graft_matrix_update_workspace_bytes(B,K_max,V,k), 8-byte aligned.
 */
size_t graft_matrix_update_workspace_bytes(int32_t B, int32_t K_max, int32_t V, int32_t k);

int32_t graft_matrix_update(const int32_t* tokens, const int32_t* n_nodes, const float* logits, int32_t V,
                            int32_t B, int32_t K_max, int32_t* M, int32_t k, int32_t* target_ids,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * graft_kv_compact - the cache update step of App. A Alg. 1 (the KV/input update
 * column of the runtime table in App. D).  During
 * verification tree node j has its key and value at logical position P + j.  For
 * k = 1 .. accept_len[b], position P + k takes the key and value rows (all KV heads)
 * of position P + path[b,k]; path[b,0] = 0 is the root and stays.  Every row is read
 * before any row of the same sequence and layer is written.
 *
 *     k_cache, v_cache   paged caches as in graft_tree_attn (IN/OUT); layer l of
 *                        n_layers starts layer_stride elements after layer l - 1
 *     block_table [B,max_pages], prefix_len [B]
 *     path [B,depth_cap+1], accept_len [B]   as written by graft_accept
 *     new_prefix_len [B] OUT: prefix_len + accept_len + 1 (root and accepted nodes; the
 *                        bonus token has no key yet).  Must not overlap prefix_len
 *                        (workgroups still read the old length while it is written):
 *                        an overlap is rejected with GRAFT_ERR_SHAPE
 * status [B]: GRAFT_STATUS_BAD_TREE if path does not start at 0, does not increase
 * strictly or reaches K_max; GRAFT_STATUS_BAD_LENGTH if prefix_len < 0, accept_len
 * outside [0,depth_cap] or a position lies beyond the block table.  Then nothing of
 * that sequence is moved and new_prefix_len = prefix_len.
 *
 * dtype GRAFT_F32 or GRAFT_BF16 (element size only), D in {64,128}, strides as in
 * graft_tree_attn, 0 <= depth_cap < GRAFT_MAX_NODES, 1 <= n_layers <= 65535.
 */
int32_t graft_kv_compact(void* k_cache, void* v_cache, int64_t layer_stride, int32_t n_layers,
                         int64_t page_stride, int64_t token_stride, int64_t head_stride,
                         const int32_t* block_table, int32_t max_pages,
                         const int32_t* prefix_len, const int32_t* path, const int32_t* accept_len,
                         int32_t B, int32_t depth_cap, int32_t K_max, int32_t Hkv, int32_t D, int32_t dtype,
                         int32_t* new_prefix_len, int32_t* status, void* stream);

/*
 * graft_prune_select - dynamic-depth pruning applied to a finished draft tree (Sec. 3.1:
 * cumulative path score S_{d,j} = S_{d-1,F(j)} + log q(x_{d,j} | .), confidence
 * c_d = exp(max_j S_{d,j}), gate g_d = 1[c_d > tau_d]; the budget resolution and
 * top-K_draft selection steps of App. A Alg. 2; App. E: the batched implementation
 * builds the whole static tree first and gates afterwards).
 *
 *     parent, tokens [B,K_max], n_nodes [B]   the draft tree
 *     logq [B,K_max] fp32   log-probability of each node given its parent, <= 0 (the
 *                           root's entry is ignored: its score is 0)
 *     chk_depth, chk_log_tau, chk_keep, chk_ret [n_chk]   checkpoints in the order they are
 *                           tried: tree depth looked at, LOG of the threshold tau_d, draft
 *                           nodes kept and retrieval slots announced when pruned there
 * Scores are accumulated in fp32 from the root downwards.  Gate c is open when some node
 * of depth chk_depth[c] has S > chk_log_tau[c] (the inequality c_d > tau_d taken in the
 * log domain; a depth without nodes is closed).  stage [B] = first closed checkpoint, or
 * n_chk when all are open (then every node is kept and n_ret = 0).  Otherwise the tree
 * ends at the closed checkpoint (Sec. 3.1: no deeper expansion; Alg. 2 prunes at the
 * stage's depth first): of the nodes of depth <= chk_depth[stage] the chk_keep[stage]
 * (at least 1, at most all of them) with the largest scores are kept, equal scores in
 * index order, and n_ret [B] = chk_ret[stage].
 *     out_index  [B,K_max]  old index of each kept node, in old order; -1 past the end
 *     out_tokens, out_parent [B,K_max]   the kept tree, parents re-indexed; -1 past the end
 *     out_n_nodes [B]
 * The outputs must not overlap the inputs.  status [B]: GRAFT_STATUS_BAD_TREE for an
 * ill-formed tree or when a kept node's parent was not kept (only possible with positive
 * logq); then out_n_nodes = 0, stage = -1, n_ret = 0 and the output rows are -1.
 *
 * 0 <= n_chk <= GRAFT_MAX_CHECKPOINTS, K_max <= GRAFT_MAX_NODES.
 */
int32_t graft_prune_select(const int32_t* parent, const int32_t* tokens, const float* logq,
                           const int32_t* n_nodes, int32_t B, int32_t K_max,
                           const int32_t* chk_depth, const float* chk_log_tau, const int32_t* chk_keep,
                           const int32_t* chk_ret, int32_t n_chk,
                           int32_t* out_parent, int32_t* out_tokens, int32_t* out_index, int32_t* out_n_nodes,
                           int32_t* stage, int32_t* n_ret, int32_t* status, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GRAFT_H */
