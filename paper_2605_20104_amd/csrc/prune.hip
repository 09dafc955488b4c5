// graft_prune_select: confidence gates and selection of the retained draft nodes.
//
// One 128-thread workgroup per sequence, one thread per tree slot, everything in LDS; the call
// is launch-latency bound like the mask rebuild, so what counts is the number of dependent LDS
// round trips and barriers.  The cumulative scores decide a selection, so they are accumulated
// exactly as the definition says, S_i = S_parent + log q_i in fp32 from the root downwards: a
// thread records its ancestors while it walks up to measure its depth (one byte each, 16 of them)
// and then adds their log q from the root down, all reads in flight at once; only a tree deeper
// than that takes one round per depth through LDS.  A node's place in the (score, index) order
// is counted directly: score and index make one 64-bit key (the float's bits made monotonic,
// then the index so that equal scores keep index order, parents before children), a node's rank
// is the number of larger keys - one 64-bit compare per pair, no sort.
#include "common.h"

namespace graft {

constexpr int PS_THREADS = GRAFT_MAX_NODES;
constexpr int PS_PATH = 16;                        // ancestors a thread records (deeper trees: rounds)

__global__ __launch_bounds__(PS_THREADS) void prune_select_kernel(
    const int32_t* __restrict__ parent, const int32_t* __restrict__ tokens, const float* __restrict__ logq,
    const int32_t* __restrict__ n_nodes, int32_t K_max, const int32_t* __restrict__ chk_depth,
    const float* __restrict__ chk_log_tau, const int32_t* __restrict__ chk_keep,
    const int32_t* __restrict__ chk_ret, int32_t n_chk, int32_t* __restrict__ out_parent,
    int32_t* __restrict__ out_tokens, int32_t* __restrict__ out_index, int32_t* __restrict__ out_n_nodes,
    int32_t* __restrict__ stage, int32_t* __restrict__ n_ret, int32_t* __restrict__ status) {
    const int b = blockIdx.x, i = threadIdx.x;
    const int lane = i & 63, wave = i >> 6;
    __shared__ int32_t par[PS_THREADS];
    __shared__ float lqs[PS_THREADS];                                   // log q of every node
    __shared__ float S[PS_THREADS];                                     // scores (deep trees only)
    __shared__ __attribute__((aligned(16))) unsigned char anc[PS_THREADS][PS_PATH];   // anc[i][k]: ancestor at distance k
    __shared__ __attribute__((aligned(16))) u64 keys[PS_THREADS];
    __shared__ int32_t newi[PS_THREADS];
    __shared__ int32_t old_of[PS_THREADS];
    __shared__ int32_t wave_cnt[PS_THREADS / 64];
    __shared__ int32_t c_depth[GRAFT_MAX_CHECKPOINTS], c_keep[GRAFT_MAX_CHECKPOINTS], c_ret[GRAFT_MAX_CHECKPOINTS];
    __shared__ float c_tau[GRAFT_MAX_CHECKPOINTS];
    __shared__ unsigned gates_open, any_deep, orphan;
    __shared__ int32_t n_cand_s;
    __shared__ int32_t or_bad[2];
    const size_t row = static_cast<size_t>(b) * K_max;

    // every input is requested at once: one trip to memory (the checkpoint parameters included,
    // thread c takes checkpoint c)
    const int32_t n = n_nodes[b];
    const bool n_ok = n >= 1 && n <= K_max;
    const int32_t p = i < K_max ? parent[row + i] : -1;
    const float lq_in = i < K_max ? logq[row + i] : 0.0f;
    if (i < n_chk) {
        c_depth[i] = chk_depth[i];
        c_tau[i] = chk_log_tau[i];
        c_keep[i] = chk_keep[i];
        c_ret[i] = chk_ret[i];
    }
    if (i == 0) { gates_open = 0u; any_deep = 0u; orphan = 0u; n_cand_s = 0; }
    bool bad = !n_ok;
    if (n_ok && i < n) bad = (i == 0) ? (p != -1) : (p < 0 || p >= i);
    par[i] = p;
    lqs[i] = (i > 0 && n_ok && i < n) ? lq_in : 0.0f;
    int any_bad = workgroup_or_128(bad, or_bad) ? 1 : 0;

    int32_t st = -1, cnt = 0, nret = 0;
    bool kept = false;
    if (!any_bad) {
        // depth by a walk up, which also records the ancestors: anc[i][0] = i, ..., anc[i][d] = 0
        int32_t d = -1;
        if (i < n) {
            for (int32_t j = i; j != -1; j = par[j]) {
                ++d;
                if (d < PS_PATH) anc[i][d] = static_cast<unsigned char>(j);
            }
        }
        if (i < n && d >= PS_PATH) any_deep = 1u;            // same value from every writer
        __syncthreads();
        float s_i = 0.0f;
        if (any_deep == 0u) {                                // uniform
            // S_i = (((0 + q[a_{d-1}]) + q[a_{d-2}]) + ...) + q[a_0]: the additions of the definition, in its order
            const uint4 a4 = *reinterpret_cast<const uint4*>(&anc[i][0]);
            const unsigned aw[4] = {a4.x, a4.y, a4.z, a4.w};
            float q[PS_PATH];
#pragma unroll
            for (int k = 0; k < PS_PATH; ++k) q[k] = lqs[(aw[k >> 2] >> (8 * (k & 3))) & (PS_THREADS - 1)];
#pragma unroll
            for (int k = PS_PATH - 1; k >= 0; --k)
                if (k < d) s_i += q[k];
        } else {
            // a tree deeper than the recorded paths: one round per depth
            if (i == 0) S[0] = 0.0f;
            for (int32_t r = 1; __syncthreads_or(d >= r ? 1 : 0); ++r)
                if (d == r) S[i] = S[p] + lqs[i];
            // the barrier that ended the loop also made the last round's scores visible
            s_i = i < n ? S[i] : 0.0f;
        }
        // gate c is open when some node of its depth has a score above its threshold; the first
        // closed gate is the stage.  All gates at once: the nodes set the bits of the gates they open.
        unsigned mine = 0u;
        for (int32_t c = 0; c < n_chk; ++c)
            if (i < n && d == c_depth[c] && s_i > c_tau[c]) mine |= 1u << c;
        if (mine != 0u) atomicOr(&gates_open, mine);
        __syncthreads();
        st = __builtin_ctz(~gates_open | (1u << n_chk));     // first gate that nobody opened, n_chk if none
        // A closed gate ends the draft tree at its checkpoint (Sec. 3.1; App. A Alg. 2 prunes at
        // the stage's depth before it keeps the best K_draft): only nodes of depth <= dlim are
        // candidates.  Non-candidates get the key 0, below every candidate's.
        const int32_t dlim = st == n_chk ? K_max : c_depth[st];
        const bool cand = i < n && d <= dlim;
        // (score, index) as one key: the float's bits made monotonic (scores are NaN-free; -0 is
        // folded into +0 first), then the index complemented so that a smaller index ranks higher
        const unsigned sb = __float_as_uint(s_i + 0.0f);
        const unsigned mono = (sb & 0x80000000u) ? ~sb : (sb | 0x80000000u);
        const u64 key = cand ? ((static_cast<u64>(mono) << 32) | static_cast<u64>(0xffffffffu - static_cast<unsigned>(i))) : 0ull;
        keys[i] = key;
        if (cand) atomicAdd(&n_cand_s, 1);
        __syncthreads();
        const int32_t n_cand = n_cand_s;
        int32_t keep = st == n_chk ? n : c_keep[st];
        keep = keep > n_cand ? n_cand : keep;
        keep = keep < 1 ? 1 : keep;
        nret = st == n_chk ? 0 : c_ret[st];
        if (cand) {
            int32_t before = 0;
            for (int32_t j0 = 0; j0 < n; j0 += 8) {          // eight keys per round of (broadcast) LDS reads
                u64 kj[8];
#pragma unroll
                for (int u = 0; u < 8; u += 2) {
                    const uint4 t = *reinterpret_cast<const uint4*>(&keys[(j0 + u) & (PS_THREADS - 1)]);
                    kj[u] = (static_cast<u64>(t.y) << 32) | t.x;
                    kj[u + 1] = (static_cast<u64>(t.w) << 32) | t.z;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) before += (j0 + u < n && kj[u] > key) ? 1 : 0;
            }
            kept = before < keep;
        }
        // new index = number of kept nodes with a smaller old index
        const u64 ballot = __ballot(kept);
        if (lane == 0) wave_cnt[wave] = __popcll(ballot);
        __syncthreads();
        int32_t rank = __popcll(ballot & ((1ull << lane) - 1));
        if (wave == 1) rank += wave_cnt[0];
        cnt = wave_cnt[0] + wave_cnt[1];
        newi[i] = kept ? rank : -1;
        if (kept) old_of[rank] = i;
        __syncthreads();
        if (kept && i > 0 && newi[p] < 0) orphan = 1u;       // a kept node lost its parent
        __syncthreads();
        any_bad = orphan != 0u ? 1 : 0;
    }
    if (any_bad) {
        if (i < K_max) { out_parent[row + i] = -1; out_tokens[row + i] = -1; out_index[row + i] = -1; }
        if (i == 0) { out_n_nodes[b] = 0; stage[b] = -1; n_ret[b] = 0; status[b] = GRAFT_STATUS_BAD_TREE; }
        return;
    }
    if (i < K_max) {                                  // thread i writes entry i of the new tree
        int32_t oi = -1, ot = -1, op = -1;
        if (i < cnt) {
            oi = old_of[i];
            ot = tokens[row + oi];
            op = oi == 0 ? -1 : newi[par[oi]];
        }
        out_index[row + i] = oi;
        out_tokens[row + i] = ot;
        out_parent[row + i] = op;
    }
    if (i == 0) { out_n_nodes[b] = cnt; stage[b] = st; n_ret[b] = nret; status[b] = 0; }
}

}  // namespace graft

extern "C" int32_t graft_prune_select(const int32_t* parent, const int32_t* tokens, const float* logq,
                                      const int32_t* n_nodes, int32_t B, int32_t K_max,
                                      const int32_t* chk_depth, const float* chk_log_tau,
                                      const int32_t* chk_keep, const int32_t* chk_ret, int32_t n_chk,
                                      int32_t* out_parent, int32_t* out_tokens, int32_t* out_index,
                                      int32_t* out_n_nodes, int32_t* stage, int32_t* n_ret, int32_t* status,
                                      void* stream) {
    if (!parent || !tokens || !logq || !n_nodes || !out_parent || !out_tokens || !out_index || !out_n_nodes ||
        !stage || !n_ret || !status)
        return GRAFT_ERR_NULL;
    if (n_chk > 0 && (!chk_depth || !chk_log_tau || !chk_keep || !chk_ret)) return GRAFT_ERR_NULL;
    if (B < 1 || K_max < 1 || K_max > GRAFT_MAX_NODES || n_chk < 0 || n_chk > GRAFT_MAX_CHECKPOINTS)
        return GRAFT_ERR_SHAPE;
    hipLaunchKernelGGL(graft::prune_select_kernel, dim3(B), dim3(graft::PS_THREADS), 0,
                       static_cast<hipStream_t>(stream), parent, tokens, logq, n_nodes, K_max, chk_depth,
                       chk_log_tau, chk_keep, chk_ret, n_chk, out_parent, out_tokens, out_index, out_n_nodes,
                       stage, n_ret, status);
    return graft::check_launch();
}
