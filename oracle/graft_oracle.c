/*
 * CPU oracle for the hybrid-tree verification step of prune-then-graft
 * speculative decoding ("Draft Less, Retrieve More", method Graft).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP sources and must never be called from the product path; only
 * the tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Each function is an exact definition (no approximation), so
 * each is written as that definition, in fp64 where floating point appears:
 *
 *   oracle_retrieve         suffix n-gram lookup over the context buffer: the
 *                           prompt-lookup / suffix-matching family the paper
 *                           contrasts itself with (Sec. 3.2, first paragraph)
 *                           and names as its online n-gram branch (Sec. 6,
 *                           limitations).  Brute-force scan of every position.
 *   oracle_build_tree_mask  position ids, ancestor masks and candidate path
 *                           indices rebuilt from the flattened parent list
 *                           (Sec. 3.3, hybrid-tree verification; App. A,
 *                           Alg. 2 last step).  Parent walk per node.
 *   oracle_tree_attn        what the tree-attention pass must produce: for
 *                           every node, ordinary causal attention of that
 *                           node's query over the prefix followed by its own
 *                           root-to-node path (Sec. 3.3).  Computed per path,
 *                           deliberately without any mask.
 *   oracle_accept           greedy form of the unchanged acceptance rule
 *                           (Sec. 3.3; greedy decoding as in Sec. 4; App. B.4).
 *
 *   oracle_matrix_retrieve  the method's own retrieval: a static template over
 *                           successor ranks filled by lookups in the transition
 *                           matrix and appended to the retained draft nodes
 *                           (Sec. 3.2; App. A.1; App. A Alg. 2).
 *   oracle_matrix_update    refresh of the matrix rows of all verified nodes
 *                           from the target logits (Sec. 3.3 last equation).
 *   oracle_kv_compact       cache update after acceptance (App. A Alg. 1).
 *   oracle_prune_select     confidence gates and top-K_draft selection on a
 *                           finished draft tree (Sec. 3.1; App. A Alg. 2; App. E).
 *
 * Pins (tests/test_oracle_*.py): brute force in pure Python on tiny inputs,
 * planted-span closed forms, chain/star closed forms, comparison with a
 * library causal-attention routine on chain trees, masked-softmax
 * reformulation, losslessness against plain greedy decoding of a toy target,
 * monotonicity (App. B.1 Prop. 1, B.2 Prop. 2); for the last four: hand-worked
 * fixtures, enumeration of rank paths under an explicit successor function,
 * a library stable sort, the gather definition on a snapshot, and equality of
 * the accepted leaf's attention before and after the cache update.  No function
 * is unpinned.  (The rank paths of the retrieval templates themselves are an
 * input: the paper prints only their per-depth counts, which are pinned.)
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC graft_oracle.c -o libgraft_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ST_BAD_LENGTH = 1, ST_BAD_TREE = 2, ST_PATH_OVERFLOW = 4 };
enum { DT_F32 = 0, DT_BF16 = 1 };
enum { MASK_WORDS = 2 };

/* ------------------------------------------------------------------ */
/* retrieval                                                           */
/* ------------------------------------------------------------------ */
typedef struct { int32_t e; int32_t len; } hit_t;

static int hit_cmp(const void* a, const void* b) {
    const hit_t* x = (const hit_t*)a;
    const hit_t* y = (const hit_t*)b;
    if (x->len != y->len) return (x->len > y->len) ? -1 : 1;   /* longer match first */
    if (x->e != y->e) return (x->e > y->e) ? -1 : 1;           /* then most recent   */
    return 0;
}

/*
 * For sequence b: L = ctx_len[b], query string q = ctx[0..L) ++ tail[0..tail_len[b]).
 * A position e (1 <= e <= L-1) is a hit when the longest l <= min(n_max, e)
 * with ctx[e-l..e) equal to the last l tokens of q has l >= n_min.  Hits are
 * ranked by (l descending, e descending); the best C are returned with the
 * (at most m) tokens that follow e.  The end of the buffer itself (e == L) is
 * not a candidate: it has no continuation.
 */
void oracle_retrieve(const int32_t* ctx, const int32_t* ctx_len, int32_t B, int32_t L_max,
                     const int32_t* tail, const int32_t* tail_len, int32_t tail_max,
                     int32_t n_min, int32_t n_max, int32_t C, int32_t m,
                     int32_t* chain_tok, int32_t* chain_len, int32_t* chain_pos,
                     int32_t* chain_match, int32_t* n_hits, int32_t* status) {
    for (int32_t b = 0; b < B; ++b) {
        int32_t* tok = chain_tok + (size_t)b * C * m;
        for (int32_t i = 0; i < C * m; ++i) tok[i] = -1;
        for (int32_t c = 0; c < C; ++c) {
            chain_len[b * C + c] = 0;
            chain_pos[b * C + c] = -1;
            chain_match[b * C + c] = 0;
        }
        n_hits[b] = 0;
        status[b] = 0;
        int32_t L = ctx_len[b];
        int32_t T = (tail != NULL && tail_len != NULL) ? tail_len[b] : 0;
        if (L < 0 || L > L_max || T < 0 || T > tail_max) { status[b] = ST_BAD_LENGTH; continue; }
        const int32_t* x = ctx + (size_t)b * L_max;
        const int32_t* tl = (T > 0) ? tail + (size_t)b * tail_max : NULL;
        int32_t QL = L + T;
        hit_t* hits = (hit_t*)malloc(sizeof(hit_t) * (size_t)(L > 0 ? L : 1));
        int32_t nh = 0;
        for (int32_t e = 1; e <= L - 1; ++e) {
            int32_t cap = n_max < e ? n_max : e;
            int32_t best = 0;
            for (int32_t l = cap; l >= 1; --l) {
                int ok = 1;
                for (int32_t j = 0; j < l; ++j) {
                    int32_t qi = QL - l + j;                       /* index into q */
                    int32_t qv = (qi < L) ? x[qi] : tl[qi - L];
                    if (x[e - l + j] != qv) { ok = 0; break; }
                }
                if (ok) { best = l; break; }
            }
            if (best >= n_min && best >= 1) { hits[nh].e = e; hits[nh].len = best; ++nh; }
        }
        qsort(hits, (size_t)nh, sizeof(hit_t), hit_cmp);
        n_hits[b] = nh;
        for (int32_t c = 0; c < C && c < nh; ++c) {
            int32_t e = hits[c].e;
            int32_t cl = (L - e) < m ? (L - e) : m;
            chain_pos[b * C + c] = e;
            chain_match[b * C + c] = hits[c].len;
            chain_len[b * C + c] = cl;
            for (int32_t j = 0; j < cl; ++j) tok[c * m + j] = x[e + j];
        }
        free(hits);
    }
}

/* ------------------------------------------------------------------ */
/* tree bookkeeping                                                    */
/* ------------------------------------------------------------------ */
/* Node 0 is the root (parent -1); every other node's parent has a smaller index. */
static int tree_ok(const int32_t* parent, int32_t n, int32_t K_max) {
    if (n < 1 || n > K_max) return 0;
    if (parent[0] != -1) return 0;
    for (int32_t i = 1; i < n; ++i)
        if (parent[i] < 0 || parent[i] >= i) return 0;
    return 1;
}

/*
 * mask[b][i] = bit set of {i} and all ancestors of i (two 64-bit words, bit j
 * of word j/64); depth[i] = edges to the root; pos[i] = prefix_len[b] +
 * depth[i].  paths (optional): one row per leaf (node without children), in
 * increasing leaf index, listing the node indices root..leaf, -1 padded, row
 * width depth_cap+1.  A leaf deeper than depth_cap gets an all -1 row and
 * leaves beyond n_leaf_max are dropped; both set ST_PATH_OVERFLOW.
 * An ill-formed tree sets ST_BAD_TREE and yields mask 0, pos/depth/paths -1.
 */
void oracle_build_tree_mask(const int32_t* parent, const int32_t* n_nodes, const int32_t* prefix_len,
                            int32_t B, int32_t K_max, uint64_t* mask, int32_t* pos, int32_t* depth,
                            int32_t* paths, int32_t n_leaf_max, int32_t depth_cap, int32_t* status) {
    for (int32_t b = 0; b < B; ++b) {
        const int32_t* par = parent + (size_t)b * K_max;
        uint64_t* mk = mask + (size_t)b * K_max * MASK_WORDS;
        int32_t* ps = pos + (size_t)b * K_max;
        int32_t* dp = depth + (size_t)b * K_max;
        int32_t width = depth_cap + 1;
        int32_t* pt = paths ? paths + (size_t)b * n_leaf_max * width : NULL;
        status[b] = 0;
        for (int32_t i = 0; i < K_max; ++i) {
            mk[i * MASK_WORDS] = 0; mk[i * MASK_WORDS + 1] = 0;
            ps[i] = -1; dp[i] = -1;
        }
        if (pt) for (int32_t i = 0; i < n_leaf_max * width; ++i) pt[i] = -1;
        int32_t n = n_nodes[b];
        if (!tree_ok(par, n, K_max)) { status[b] = ST_BAD_TREE; continue; }
        for (int32_t i = 0; i < n; ++i) {
            int32_t d = -1;
            for (int32_t j = i; j != -1; j = par[j]) {
                mk[i * MASK_WORDS + (j >> 6)] |= (uint64_t)1 << (j & 63);
                ++d;
            }
            dp[i] = d;
            ps[i] = prefix_len[b] + d;
        }
        if (pt) {
            int32_t row = 0;
            for (int32_t i = 0; i < n; ++i) {
                int is_leaf = 1;
                for (int32_t c = i + 1; c < n; ++c) if (par[c] == i) { is_leaf = 0; break; }
                if (!is_leaf) continue;
                if (row >= n_leaf_max) { status[b] |= ST_PATH_OVERFLOW; break; }
                if (dp[i] > depth_cap) { status[b] |= ST_PATH_OVERFLOW; ++row; continue; }
                int32_t k = dp[i];
                for (int32_t j = i; j != -1; j = par[j]) pt[row * width + k--] = j;
                ++row;
            }
        }
    }
}

/* ------------------------------------------------------------------ */
/* attention                                                           */
/* ------------------------------------------------------------------ */
static double load_elem(const void* base, int64_t idx, int dtype) {
    if (dtype == DT_F32) return (double)((const float*)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t*)base)[idx] << 16;   /* bf16 widens exactly */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/*
 * One output row per (b, node i, query head h): the sequence attended to is
 *   S = prefix positions 0..P-1, then the tree slots on the path root..i;
 * tree slot j is logical token P+j of sequence b.  Token t lives in page
 * block_table[b][t / page_size] at in-page offset t % page_size; element d of
 * KV head g of that token is at  page*page_stride + off*token_stride +
 * g*head_stride + d.  score_t = (q . k_t) * scale, weights = softmax over S,
 * out = sum_t w_t v_t, all in fp64.  KV head of query head h is h / (Hq/Hkv).
 *
 * rows == NULL: every (b,i,h) is computed into out[B][K_max][Hq][D] (rows of
 * padding nodes and of ill-formed trees are zero).  Otherwise rows holds
 * n_rows triples (b,i,h) and out is [n_rows][D].
 */
void oracle_tree_attn(const void* q, const void* k_cache, const void* v_cache, int32_t dtype,
                      int64_t page_stride, int64_t token_stride, int64_t head_stride,
                      const int32_t* block_table, int32_t max_pages,
                      const int32_t* prefix_len, const int32_t* n_nodes, const int32_t* parent,
                      int32_t B, int32_t K_max, int32_t Hq, int32_t Hkv, int32_t D, int32_t page_size,
                      double scale, const int32_t* rows, int64_t n_rows, double* out) {
    int64_t total = rows ? n_rows : (int64_t)B * K_max * Hq;
    int32_t G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < total; ++r) {
        int32_t b, i, h;
        if (rows) { b = rows[3 * r]; i = rows[3 * r + 1]; h = rows[3 * r + 2]; }
        else { b = (int32_t)(r / ((int64_t)K_max * Hq)); i = (int32_t)((r / Hq) % K_max); h = (int32_t)(r % Hq); }
        double* o = out + r * D;
        for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
        const int32_t* par = parent + (size_t)b * K_max;
        int32_t n = n_nodes[b];
        if (!tree_ok(par, n, K_max) || i >= n) continue;
        int32_t P = prefix_len[b];
        int32_t g = h / G;
        /* the path root..i as tree slots */
        int32_t plen = 0;
        for (int32_t j = i; j != -1; j = par[j]) ++plen;
        int32_t* seq = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P + plen));
        for (int32_t t = 0; t < P; ++t) seq[t] = t;
        { int32_t k = P + plen - 1; for (int32_t j = i; j != -1; j = par[j]) seq[k--] = P + j; }
        int32_t n_tok = P + plen;
        double* s = (double*)malloc(sizeof(double) * (size_t)n_tok);
        int64_t qoff = (((int64_t)b * K_max + i) * Hq + h) * D;
        double mx = -INFINITY;
        for (int32_t t = 0; t < n_tok; ++t) {
            int32_t tk = seq[t];
            int64_t base = (int64_t)block_table[(size_t)b * max_pages + tk / page_size] * page_stride
                         + (int64_t)(tk % page_size) * token_stride + (int64_t)g * head_stride;
            double acc = 0.0;
            for (int32_t d = 0; d < D; ++d)
                acc += load_elem(q, qoff + d, dtype) * load_elem(k_cache, base + d, dtype);
            s[t] = acc * scale;
            if (s[t] > mx) mx = s[t];
        }
        double den = 0.0;
        for (int32_t t = 0; t < n_tok; ++t) { s[t] = exp(s[t] - mx); den += s[t]; }
        for (int32_t t = 0; t < n_tok; ++t) {
            int32_t tk = seq[t];
            int64_t base = (int64_t)block_table[(size_t)b * max_pages + tk / page_size] * page_stride
                         + (int64_t)(tk % page_size) * token_stride + (int64_t)g * head_stride;
            double wgt = s[t] / den;
            for (int32_t d = 0; d < D; ++d) o[d] += wgt * load_elem(v_cache, base + d, dtype);
        }
        free(s);
        free(seq);
    }
}

/* ------------------------------------------------------------------ */
/* acceptance                                                          */
/* ------------------------------------------------------------------ */
/*
 * t*[i] = the target's greedy token after node i: target_ids[i] when logits
 * is NULL, else the index of the first maximum of logits[b][i][0..V) (and it
 * is written back to target_ids).  The root is always accepted; node i > 0 is
 * accepted when its parent is accepted and tokens[i] == t*[parent[i]].  best =
 * the accepted node of greatest depth not exceeding depth_cap (smallest index
 * on ties); accept_len = depth of best (root and bonus token not counted);
 * path = node indices root..best; out_tokens = the tokens of path[1..] then
 * the bonus token t*[best]; both rows have width depth_cap+1, -1 padded.  An
 * accepted node deeper than depth_cap sets ST_PATH_OVERFLOW.
 */
void oracle_accept(const int32_t* parent, const int32_t* tokens, const int32_t* n_nodes,
                   const float* logits, int32_t V, int32_t* target_ids,
                   int32_t B, int32_t K_max, int32_t depth_cap,
                   int32_t* accept_len, int32_t* best_node, int32_t* path, int32_t* out_tokens,
                   int32_t* status) {
    int32_t width = depth_cap + 1;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t* par = parent + (size_t)b * K_max;
        const int32_t* tok = tokens + (size_t)b * K_max;
        int32_t* ts = target_ids + (size_t)b * K_max;
        int32_t* pth = path + (size_t)b * width;
        int32_t* ot = out_tokens + (size_t)b * width;
        status[b] = 0;
        accept_len[b] = 0;
        best_node[b] = -1;
        for (int32_t k = 0; k < width; ++k) { pth[k] = -1; ot[k] = -1; }
        int32_t n = n_nodes[b];
        if (!tree_ok(par, n, K_max)) {
            status[b] = ST_BAD_TREE;
            if (logits) for (int32_t i = 0; i < K_max; ++i) ts[i] = -1;
            continue;
        }
        if (logits) {
            for (int32_t i = 0; i < K_max; ++i) {
                ts[i] = -1;
                if (i >= n) continue;
                const float* row = logits + ((size_t)b * K_max + i) * V;
                int32_t arg = 0;
                for (int32_t v = 1; v < V; ++v) if (row[v] > row[arg]) arg = v;
                ts[i] = arg;
            }
        }
        int* ok = (int*)malloc(sizeof(int) * (size_t)n);
        int32_t* dp = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
        ok[0] = 1; dp[0] = 0;
        int32_t best = 0;
        for (int32_t i = 1; i < n; ++i) {
            dp[i] = dp[par[i]] + 1;
            ok[i] = ok[par[i]] && tok[i] == ts[par[i]];
            if (ok[i]) {
                if (dp[i] > depth_cap) status[b] |= ST_PATH_OVERFLOW;
                else if (dp[i] > dp[best]) best = i;
            }
        }
        accept_len[b] = dp[best];
        best_node[b] = best;
        { int32_t k = dp[best]; for (int32_t j = best; j != -1; j = par[j]) pth[k--] = j; }
        for (int32_t k = 1; k <= dp[best]; ++k) ot[k - 1] = tok[pth[k]];
        ot[dp[best]] = ts[best];
        free(ok);
        free(dp);
    }
}

/* ================================================================== */
/* Steps around the verification pass (the method's own retrieval, the */
/* matrix refresh, the cache update).  Same rules as above: plain       */
/* definitions, test infrastructure only.                               */
/* ================================================================== */

/* ------------------------------------------------------------------ */
/* retrieval from the transition matrix                                */
/* ------------------------------------------------------------------ */
/*
 * The retrieval branch of the method (Sec. 3.2, stage-adaptive templates,
 * equation x_u = M[x_F(u), r_u]; App. A.1; the template traversal and append
 * steps of App. A Alg. 2).
 *
 * M is the matrix of successor ids, int32 [V][k].  The template has N nodes;
 * node u has parent tpl_parent[u] (an earlier template node, or -1 for the
 * root of the tree) and successor rank tpl_rank[u].  For sequence b the first
 * n_ret[b] template nodes are taken (a stage's template is a prefix of the
 * envelope), filled in order, and appended behind the n_nodes[b] retained
 * draft nodes: merged node n_nodes[b] + u gets token x_u and parent
 * (tpl_parent[u] < 0 ? 0 : n_nodes[b] + tpl_parent[u]); n_nodes[b] grows by
 * n_ret[b].  The root token is tokens[b][0].  A lookup from a token outside
 * [0, V) or of an empty matrix entry (-1) gives -1, and so do all of its
 * descendants (such a node stays in the tree and can never be accepted).
 * n_ret[b] outside [0, N], a tree that would exceed K_max, or n_nodes[b] < 1
 * set ST_BAD_LENGTH; a template node (among the first n_ret[b]) whose parent
 * is not an earlier node or -1, or whose rank is outside [0, k), sets
 * ST_BAD_TREE.  Either way the sequence is left as it was.
 */
void oracle_matrix_retrieve(const int32_t* M, int32_t V, int32_t k,
                            const int32_t* tpl_parent, const int32_t* tpl_rank, int32_t N,
                            const int32_t* n_ret, int32_t B, int32_t K_max,
                            int32_t* tokens, int32_t* parent, int32_t* n_nodes, int32_t* status) {
    int32_t* x = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    for (int32_t b = 0; b < B; ++b) {
        int32_t* tok = tokens + (size_t)b * K_max;
        int32_t* par = parent + (size_t)b * K_max;
        int32_t nd = n_nodes[b], nr = n_ret[b];
        status[b] = 0;
        if (nd < 1 || nr < 0 || nr > N || nd + nr > K_max) { status[b] = ST_BAD_LENGTH; continue; }
        int ok = 1;
        for (int32_t u = 0; u < nr; ++u)
            if (tpl_parent[u] < -1 || tpl_parent[u] >= u || tpl_rank[u] < 0 || tpl_rank[u] >= k) ok = 0;
        if (!ok) { status[b] = ST_BAD_TREE; continue; }
        for (int32_t u = 0; u < nr; ++u) {
            int32_t f = tpl_parent[u];
            int32_t from = f < 0 ? tok[0] : x[f];
            int32_t r = tpl_rank[u];
            x[u] = (from >= 0 && from < V) ? M[(size_t)from * k + r] : -1;
            tok[nd + u] = x[u];
            par[nd + u] = f < 0 ? 0 : nd + f;
        }
        n_nodes[b] = nd + nr;
    }
    free(x);
}

/* ------------------------------------------------------------------ */
/* refresh of the transition matrix                                    */
/* ------------------------------------------------------------------ */
/*
 * M[x_i] <- argtop-k(p_{i+1}) over every verified node, accepted or rejected
 * (Sec. 3.3, warm-up and online update, last equation; the matrix update
 * equation and step of App. A Alg. 1).  The ranking of the softmax distribution is the ranking of the
 * logits, so no softmax is taken.
 *
 * For b = 0..B-1 and i = 0..n_nodes[b]-1 in this order: row tokens[b][i] of M
 * becomes the k ids with the largest logits[b][i][.], largest first, equal
 * logits in order of id.  Nodes are processed in order, so when a token occurs
 * at several nodes the last one (largest b, then largest i) stays.  Tokens
 * outside [0, V) are skipped.  target_ids[b][i] = the first of the k ids (the
 * greedy token that the acceptance step uses), -1 for i >= n_nodes[b].
 */
void oracle_matrix_update(const int32_t* tokens, const int32_t* n_nodes, const float* logits, int32_t V,
                          int32_t B, int32_t K_max, int32_t* M, int32_t k, int32_t* target_ids) {
    int32_t* best = (int32_t*)malloc(sizeof(int32_t) * (size_t)k);
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t i = 0; i < K_max; ++i) {
            target_ids[(size_t)b * K_max + i] = -1;
            if (i >= n_nodes[b]) continue;
            const float* row = logits + ((size_t)b * K_max + i) * V;
            /* k rounds of "largest not yet taken" */
            for (int32_t j = 0; j < k; ++j) {
                int32_t arg = -1;
                for (int32_t v = 0; v < V; ++v) {
                    int taken = 0;
                    for (int32_t t = 0; t < j; ++t) if (best[t] == v) taken = 1;
                    if (taken) continue;
                    if (arg < 0 || row[v] > row[arg]) arg = v;
                }
                best[j] = arg;                 /* -1 only when k > V */
            }
            target_ids[(size_t)b * K_max + i] = best[0];
            int32_t x = tokens[(size_t)b * K_max + i];
            if (x < 0 || x >= V) continue;
            for (int32_t j = 0; j < k; ++j) M[(size_t)x * k + j] = best[j];
        }
    }
    free(best);
}

/* ------------------------------------------------------------------ */
/* cache update after acceptance                                       */
/* ------------------------------------------------------------------ */
/*
 * The cache update step of App. A Alg. 1 (the KV/input update column of the
 * runtime table, App. D).  During verification
 * tree node j has its key and value at logical position P + j.  Afterwards the
 * cache must hold the accepted path as an ordinary prefix: for k = 1 ..
 * accept_len, position P + k takes the key and value rows (all KV heads) of
 * position P + path[k]; path[0] = 0 is the root, already in place.  Done out
 * of place here: all rows are read before any is written.  The new prefix
 * length is P + accept_len + 1 (root and accepted nodes; the bonus token has
 * no key yet).  The caches of n_layers layers lie layer_stride elements apart.
 *
 * path must start at 0 and increase strictly with path[k] < K_max, else the
 * sequence is left untouched with ST_BAD_TREE; P < 0, accept_len outside
 * [0, depth_cap] or a position beyond the block table give ST_BAD_LENGTH.
 */
void oracle_kv_compact(void* k_cache, void* v_cache, int32_t dtype, int64_t layer_stride, int32_t n_layers,
                       int64_t page_stride, int64_t token_stride, int64_t head_stride,
                       const int32_t* block_table, int32_t max_pages, int32_t page_size,
                       const int32_t* prefix_len, const int32_t* path, const int32_t* accept_len,
                       int32_t B, int32_t depth_cap, int32_t K_max, int32_t Hkv, int32_t D,
                       int32_t* new_prefix_len, int32_t* status) {
    const size_t es = dtype == DT_F32 ? 4 : 2;
    const size_t row = (size_t)D * es;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t P = prefix_len[b], a = accept_len[b];
        const int32_t* pth = path + (size_t)b * (depth_cap + 1);
        const int32_t* table = block_table + (size_t)b * max_pages;
        status[b] = 0;
        new_prefix_len[b] = P;
        if (P < 0 || a < 0 || a > depth_cap) { status[b] = ST_BAD_LENGTH; continue; }
        int ok = pth[0] == 0;
        for (int32_t k = 1; k <= a && ok; ++k) ok = pth[k] > pth[k - 1] && pth[k] < K_max;
        if (!ok) { status[b] = ST_BAD_TREE; continue; }
        if (a > 0 && (int64_t)P + pth[a] >= (int64_t)max_pages * page_size) { status[b] = ST_BAD_LENGTH; continue; }
        new_prefix_len[b] = P + a + 1;
        if (a == 0) continue;
        unsigned char* tmp = (unsigned char*)malloc((size_t)a * Hkv * row);
        for (int32_t l = 0; l < n_layers; ++l) {
            for (int side = 0; side < 2; ++side) {
                unsigned char* base = (unsigned char*)(side ? v_cache : k_cache) + (size_t)l * layer_stride * es;
                for (int32_t k = 1; k <= a; ++k) {                        /* read everything ... */
                    int32_t t = P + pth[k];
                    int64_t off = (int64_t)table[t / page_size] * page_stride + (int64_t)(t % page_size) * token_stride;
                    for (int32_t g = 0; g < Hkv; ++g)
                        memcpy(tmp + ((size_t)(k - 1) * Hkv + g) * row, base + (off + g * head_stride) * es, row);
                }
                for (int32_t k = 1; k <= a; ++k) {                        /* ... then write */
                    int32_t t = P + k;
                    int64_t off = (int64_t)table[t / page_size] * page_stride + (int64_t)(t % page_size) * token_stride;
                    for (int32_t g = 0; g < Hkv; ++g)
                        memcpy(base + (off + g * head_stride) * es, tmp + ((size_t)(k - 1) * Hkv + g) * row, row);
                }
            }
        }
        free(tmp);
    }
}

/* ------------------------------------------------------------------ */
/* confidence gates and selection of the retained draft nodes          */
/* ------------------------------------------------------------------ */
/*
 * Dynamic-depth pruning on a finished draft tree (Sec. 3.1: cumulative path
 * score S_{d,j} = S_{d-1,F(j)} + log q, confidence
 * c_d = exp(max_j S_{d,j}), gate g_d = 1[c_d > tau_d]; the budget resolution
 * and top-K_draft selection steps of App. A Alg. 2; App. E: in the batched
 * implementation the whole static tree is built
 * first and the gates are applied afterwards).
 *
 * logq[b][i] is the draft model's log-probability of node i given its parent
 * (node 0, the root, has score 0 whatever logq[b][0] holds).  Scores are
 * accumulated in fp32 from the root downwards, S_i = S_parent(i) + logq_i, in
 * that order, because they decide a selection.  Checkpoint c looks at tree
 * depth chk_depth[c]; the gate is taken in the log domain, max_j S_{d,j} >
 * chk_log_tau[c] (the same inequality as c_d > tau_d, without rounding an
 * exponential); a depth without nodes has confidence 0 (gate closed).  The
 * stage is the first checkpoint whose gate is closed.  A closed gate ends the
 * draft tree at its checkpoint: nothing deeper is expanded (Sec. 3.1; Alg. 2
 * prunes the tree at the stage's depth before it keeps the best K_draft), so
 * of a finished static tree only the nodes of depth <= chk_depth[c] are
 * candidates.  The stage keeps the chk_keep[c] candidates with the largest
 * scores (equal scores: smaller index first, so that a parent comes before its
 * child) and announces chk_ret[c] retrieval slots.  If every gate is open,
 * stage = n_chk, all nodes stay and n_ret = 0.
 *
 * The kept nodes are written in their old order: out_index[new] = old index,
 * out_tokens, out_parent (re-indexed), out_n_nodes; entries past the end are
 * -1.  An ill-formed tree, or a kept node whose parent was not kept (possible
 * only with positive logq), gives ST_BAD_TREE with out_n_nodes = 0, stage = -1.
 */
void oracle_prune_select(const int32_t* parent, const int32_t* tokens, const float* logq,
                         const int32_t* n_nodes, int32_t B, int32_t K_max,
                         const int32_t* chk_depth, const float* chk_log_tau, const int32_t* chk_keep,
                         const int32_t* chk_ret, int32_t n_chk,
                         int32_t* out_parent, int32_t* out_tokens, int32_t* out_index, int32_t* out_n_nodes,
                         int32_t* stage, int32_t* n_ret, int32_t* status) {
    float* S = (float*)malloc(sizeof(float) * (size_t)K_max);
    int32_t* dp = (int32_t*)malloc(sizeof(int32_t) * (size_t)K_max);
    int32_t* newi = (int32_t*)malloc(sizeof(int32_t) * (size_t)K_max);
    for (int32_t b = 0; b < B; ++b) {
        const int32_t* par = parent + (size_t)b * K_max;
        const int32_t* tok = tokens + (size_t)b * K_max;
        const float* lq = logq + (size_t)b * K_max;
        int32_t* op = out_parent + (size_t)b * K_max;
        int32_t* ot = out_tokens + (size_t)b * K_max;
        int32_t* oi = out_index + (size_t)b * K_max;
        const int32_t n = n_nodes[b];
        for (int32_t i = 0; i < K_max; ++i) { op[i] = -1; ot[i] = -1; oi[i] = -1; }
        status[b] = 0; out_n_nodes[b] = 0; stage[b] = -1; n_ret[b] = 0;
        if (!tree_ok(par, n, K_max)) { status[b] = ST_BAD_TREE; continue; }
        S[0] = 0.0f; dp[0] = 0;
        for (int32_t i = 1; i < n; ++i) { S[i] = S[par[i]] + lq[i]; dp[i] = dp[par[i]] + 1; }
        int32_t st = n_chk;
        for (int32_t c = 0; c < n_chk && st == n_chk; ++c) {
            int open = 0;
            for (int32_t i = 0; i < n; ++i)
                if (dp[i] == chk_depth[c] && S[i] > chk_log_tau[c]) open = 1;
            if (!open) st = c;
        }
        /* candidates: the nodes the pruned tree still has (depth <= the stage's depth) */
        const int32_t dlim = st == n_chk ? K_max : chk_depth[st];
        int32_t n_cand = 0;
        for (int32_t i = 0; i < n; ++i)
            if (dp[i] <= dlim) ++n_cand;
        int32_t keep = st == n_chk ? n : chk_keep[st];
        if (keep > n_cand) keep = n_cand;
        if (keep < 1) keep = 1;
        /* candidate i is kept when fewer than `keep` candidates come before it in (score, index) order */
        int32_t cnt = 0;
        int ok = 1;
        for (int32_t i = 0; i < n; ++i) {
            int32_t before = 0;
            for (int32_t j = 0; j < n; ++j)
                if (dp[j] <= dlim && (S[j] > S[i] || (S[j] == S[i] && j < i))) ++before;
            newi[i] = (dp[i] <= dlim && before < keep) ? cnt++ : -1;
            if (newi[i] >= 0 && i > 0 && newi[par[i]] < 0) ok = 0;
        }
        if (!ok) { status[b] = ST_BAD_TREE; continue; }
        for (int32_t i = 0; i < n; ++i) {
            if (newi[i] < 0) continue;
            oi[newi[i]] = i;
            ot[newi[i]] = tok[i];
            op[newi[i]] = i == 0 ? -1 : newi[par[i]];
        }
        out_n_nodes[b] = cnt;
        stage[b] = st;
        n_ret[b] = st == n_chk ? 0 : chk_ret[st];
    }
    free(S); free(dp); free(newi);
}
