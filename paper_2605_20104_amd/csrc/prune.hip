// graft_prune_select: confidence gates and selection of the retained draft nodes.
//
// One 128-thread workgroup per sequence, one thread per tree slot, everything in LDS; the
// call is launch-latency bound like the mask rebuild.  The cumulative scores decide a
// selection, so they are accumulated exactly as the definition says, S_i = S_parent + log q_i
// in fp32 from the root downwards: one round per depth.  A node's place in the (score,
// index) order is counted directly (n compares per node), which needs no sort and keeps
// equal scores in index order, parents before children.
#include "common.h"

namespace graft {

constexpr int PS_THREADS = GRAFT_MAX_NODES;

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
    __shared__ float S[PS_THREADS];
    __shared__ int32_t newi[PS_THREADS];
    __shared__ int32_t dep[PS_THREADS];
    __shared__ int32_t old_of[PS_THREADS];
    __shared__ int32_t wave_cnt[PS_THREADS / 64];
    const size_t row = static_cast<size_t>(b) * K_max;

    const int32_t n = n_nodes[b];
    const bool n_ok = n >= 1 && n <= K_max;
    const int32_t p = i < K_max ? parent[row + i] : -1;
    bool bad = !n_ok;
    if (n_ok && i < n) bad = (i == 0) ? (p != -1) : (p < 0 || p >= i);
    par[i] = p;
    int any_bad = __syncthreads_or(bad ? 1 : 0);

    int32_t st = -1, cnt = 0, nret = 0;
    bool kept = false;
    if (!any_bad) {
        // depth by a walk, scores by one round per depth
        int32_t d = -1;
        if (i < n) for (int32_t j = i; j != -1; j = par[j]) ++d;
        const float lq = (i > 0 && i < n) ? logq[row + i] : 0.0f;
        if (i == 0) S[0] = 0.0f;
        for (int32_t r = 1; __syncthreads_or(d >= r ? 1 : 0); ++r)
            if (d == r) S[i] = S[p] + lq;
        // the barrier that ended the loop also made the last round's scores visible
        const float s_i = i < n ? S[i] : 0.0f;
        st = n_chk;
        for (int32_t c = 0; c < n_chk; ++c) {
            const bool open = i < n && d == chk_depth[c] && s_i > chk_log_tau[c];
            if (__syncthreads_or(open ? 1 : 0) == 0) { st = c; break; }
        }
        // A closed gate ends the draft tree at its checkpoint (Sec. 3.1; App. A Alg. 2 prunes at
        // the stage's depth before it keeps the best K_draft): only nodes of depth <= dlim are
        // candidates.  Non-candidates get a score below every real one so that the counting
        // loop needs no second array (real scores are finite sums of finite inputs; NaN-free).
        const int32_t dlim = st == n_chk ? K_max : chk_depth[st];
        const bool cand = i < n && d <= dlim;
        dep[i] = d;
        const int32_t n_cand = __syncthreads_count(cand ? 1 : 0);
        int32_t keep = st == n_chk ? n : chk_keep[st];
        keep = keep > n_cand ? n_cand : keep;
        keep = keep < 1 ? 1 : keep;
        nret = st == n_chk ? 0 : chk_ret[st];
        if (cand) {
            int32_t before = 0;
            for (int32_t j = 0; j < n; ++j) {
                const float s_j = S[j];
                before += (dep[j] <= dlim && (s_j > s_i || (s_j == s_i && j < i))) ? 1 : 0;
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
        any_bad = __syncthreads_or((kept && i > 0 && newi[p] < 0) ? 1 : 0);   // a kept node lost its parent
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
