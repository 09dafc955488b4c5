// graft_matrix_retrieve and graft_matrix_update: the transition matrix M[V][k] of successor
// ids that the method keeps in GPU memory.
//
// Retrieval is a gather along a static template: one 128-thread workgroup per sequence, one
// thread per template node.  A node can be filled once its parent's token is known, so the
// template is filled in rounds, one per depth: every round is one dependent lookup in M, and
// the nodes of a depth are looked up together.  The call is bound by those dependent
// round trips (nine for the paper's templates), not by bandwidth.
//
// The refresh ranks every verified node's logits row.  Like the argmax of the acceptance
// step it is one HBM scan of the logits (4 V bytes per node): GRAFT_ARGMAX_CHUNKS workgroups
// per row; a workgroup finds a threshold from its threads' maxima, collects the few elements
// above it and picks its chunk's k best from those in k rounds.  A key packs (logit,
// id) into 64 bits so that "larger logit first, then smaller id" is one unsigned compare.
// A one-wavefront kernel per node then merges the chunks, writes the greedy token and, if
// no later node carries the same token, the matrix row.
#include "common.h"

namespace graft {

constexpr int MR_THREADS = GRAFT_MAX_NODES;
constexpr int MU_THREADS = 256;
constexpr int MU_WAVES = MU_THREADS / 64;

__global__ __launch_bounds__(MR_THREADS) void matrix_retrieve_kernel(
    const int32_t* __restrict__ M, int32_t V, int32_t k, const int32_t* __restrict__ tpl_parent,
    const int32_t* __restrict__ tpl_rank, int32_t N, const int32_t* __restrict__ n_ret, int32_t K_max,
    int32_t* __restrict__ tokens, int32_t* __restrict__ parent, int32_t* __restrict__ n_nodes,
    int32_t* __restrict__ status) {
    const int b = blockIdx.x, u = threadIdx.x;
    __shared__ int32_t x[GRAFT_MAX_NODES];        // token of template node u
    __shared__ int32_t done[GRAFT_MAX_NODES];
    int32_t* tok = tokens + static_cast<size_t>(b) * K_max;
    int32_t* par = parent + static_cast<size_t>(b) * K_max;
    const int32_t nd = n_nodes[b], nr = n_ret[b];
    if (nd < 1 || nr < 0 || nr > N || nd + nr > K_max) {       // uniform over the workgroup
        if (u == 0) status[b] = GRAFT_STATUS_BAD_LENGTH;
        return;
    }
    const bool mine = u < nr;
    const int32_t f = mine ? tpl_parent[u] : -1;
    const int32_t r = mine ? tpl_rank[u] : 0;
    const int bad = mine && (f < -1 || f >= u || r < 0 || r >= k);
    if (__syncthreads_or(bad)) {
        if (u == 0) status[b] = GRAFT_STATUS_BAD_TREE;
        return;
    }
    const int32_t root = tok[0];
    done[u] = 0;
    __syncthreads();
    // rounds: a node is filled in the round after its parent's (at most nr rounds; the
    // workgroup stops as soon as every node is filled)
    bool filled = !mine;
    for (int round = 0; round < nr; ++round) {
        const bool ready = !filled && (f < 0 || done[f] != 0);
        int32_t from = 0;
        if (ready) from = f < 0 ? root : x[f];
        __syncthreads();                            // all reads of done/x of this round before its writes
        if (ready) {
            const int32_t v = (from >= 0 && from < V) ? M[static_cast<size_t>(from) * k + r] : -1;
            x[u] = v;
            done[u] = 1;
            tok[nd + u] = v;
            par[nd + u] = f < 0 ? 0 : nd + f;
            filled = true;
        }
        if (__syncthreads_and(filled)) break;
    }
    if (u == 0) {
        n_nodes[b] = nd + nr;
        status[b] = 0;
    }
}

// ---- refresh ------------------------------------------------------------------------------

// (logit, id) -> key: larger logit = larger key; among equal logits the smaller id is larger.
__device__ __forceinline__ u64 rank_key(float v, int32_t id) {
    v += 0.0f;                                      // -0.0 -> +0.0: they compare equal
    const unsigned bits = __float_as_uint(v);
    const unsigned ord = (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
    return (static_cast<u64>(ord) << 32) | static_cast<u64>(0xffffffffu - static_cast<unsigned>(id));
}
__device__ __forceinline__ int32_t key_id(u64 key) {
    return static_cast<int32_t>(0xffffffffu - static_cast<unsigned>(key & 0xffffffffu));
}

// The thread's KK best keys, best first.  Almost every element fails the first test (one
// float compare against the value of the worst kept key; equal values go on to the exact
// 64-bit compare because the id decides then).
template <int KK>
__device__ __forceinline__ void topk_insert(u64 (&top)[KK], float& worst, float v, int32_t id) {
    if (v >= worst) {
        u64 key = rank_key(v, id);
        if (key > top[KK - 1]) {
#pragma unroll
            for (int j = 0; j < KK; ++j) {
                if (key > top[j]) { const u64 t = top[j]; top[j] = key; key = t; }
            }
            // value of the new worst key (-inf while fewer than KK have been seen)
            const unsigned ord = static_cast<unsigned>(top[KK - 1] >> 32);
            const unsigned bits = (ord & 0x80000000u) ? (ord & 0x7fffffffu) : ~ord;
            worst = top[KK - 1] == 0 ? -INFINITY : __uint_as_float(bits);
        }
    }
}

// The scan of one thread's share of a chunk.  take(value, id) is called for every element in
// order of id.
template <class Take>
__device__ __forceinline__ void scan_chunk(const float* __restrict__ row, int32_t V, int32_t q0, int32_t q1,
                                           int tid, Take&& take) {
    if (V % 4 == 0) {                               // every row start is 16-byte aligned
        const float4* row4 = reinterpret_cast<const float4*>(row);
        constexpr int U = 4;                        // 16-byte loads in flight per thread
        for (int32_t qd = q0 + tid; qd < q1; qd += U * MU_THREADS) {
            float4 x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int32_t qu = qd + u * MU_THREADS;
                x[u] = row4[qu < q1 ? qu : qd];     // a lane past the end re-reads its first quad (skipped below)
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int32_t qu = qd + u * MU_THREADS;
                if (qu < q1) {
                    take(x[u].x, qu * 4);
                    take(x[u].y, qu * 4 + 1);
                    take(x[u].z, qu * 4 + 2);
                    take(x[u].w, qu * 4 + 3);
                }
            }
        }
    } else {
        const int32_t e0 = q0 * 4, e1 = (q1 * 4) < V ? (q1 * 4) : V;
        for (int32_t e = e0 + tid; e < e1; e += MU_THREADS) take(row[e], e);
    }
}

// k rounds over the workgroup: every wavefront offers its best remaining key, the owner of
// the round's winner (keys are unique: the id is part of them) pops it.  Returns how many of
// this thread's keys were taken.
template <int KK>
__device__ __forceinline__ int select_rounds(u64 (&top)[KK], int k, u64 (&red)[2][MU_WAVES], u64* out,
                                             int tid, int lane, int wave) {
    int taken = 0;
    for (int j = 0; j < k; ++j) {
        const u64 wmax = wave_max_u64(top[0]);
        if (lane == 0) red[j & 1][wave] = wmax;
        __syncthreads();
        u64 gmax = red[j & 1][0];
#pragma unroll
        for (int w = 1; w < MU_WAVES; ++w) gmax = red[j & 1][w] > gmax ? red[j & 1][w] : gmax;
        if (tid == 0) out[j] = gmax;
        if (gmax != 0 && top[0] == gmax) {
#pragma unroll
            for (int t = 0; t + 1 < KK; ++t) top[t] = top[t + 1];
            top[KK - 1] = 0;
            ++taken;
        }
    }
    return taken;
}

// Chunk scan: workgroup (chunk, node, sequence) -> its chunk's k best keys, best first.
//
// Fast path (aligned rows whose chunk fits in registers, MU_REG_QUADS 16-byte loads per
// thread, all issued before anything else):
//   1. every thread takes the maximum of its elements (one max3 per two elements);
//   2. every wavefront finds the k-th largest of its 64 maxima (k rounds of a float max in
//      registers; equal maxima leave together, which only lowers the result) and T is the
//      largest of the four: at least k elements are >= T, so every one of the chunk's k
//      best is >= T;
//   3. the elements >= T (normally a dozen or two) are appended to a list in LDS as keys;
//   4. one wavefront picks the result from the list in k rounds.
// If the list overflows (long runs of equal values) or the chunk does not fit, the
// workgroup takes the exact streaming path: per-thread sorted lists of KK >= k keys.
constexpr int MU_REG_QUADS = 12;                    // covers V <= 196608
constexpr int MU_LIST = 256;                        // four candidates per lane of the last wavefront

template <int KK>
__global__ __launch_bounds__(MU_THREADS) void topk_chunk_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ n_nodes, int32_t K_max, int32_t V,
    int32_t k, u64* __restrict__ partial) {
    const int chunk = blockIdx.x, i = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    u64* out = partial + ((static_cast<size_t>(b) * K_max + i) * GRAFT_ARGMAX_CHUNKS + chunk) * k;
    const int32_t n = n_nodes[b];
    if (i >= n || n > K_max) {                      // padding node
        if (tid < k) out[tid] = 0;
        return;
    }
    const int32_t quads = (V + 3) / 4;
    const int32_t per = (quads + GRAFT_ARGMAX_CHUNKS - 1) / GRAFT_ARGMAX_CHUNKS;
    const int32_t q0 = chunk * per;
    const int32_t q1 = (q0 + per) < quads ? (q0 + per) : quads;
    const float* row = logits + (static_cast<size_t>(b) * K_max + i) * V;
    __shared__ u64 red[2][MU_WAVES];
    __shared__ u64 list[MU_LIST];
    __shared__ int32_t list_n;

    bool exact = true;
    if (V % 4 == 0 && per <= MU_REG_QUADS * MU_THREADS) {           // uniform over the grid
        const float4* row4 = reinterpret_cast<const float4*>(row);
        float4 x[MU_REG_QUADS];
#pragma unroll
        for (int u = 0; u < MU_REG_QUADS; ++u) {
            const int32_t qu = q0 + tid + u * MU_THREADS;
            x[u] = qu < q1 ? row4[qu] : float4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        }
        if (tid == 0) list_n = 0;
        float m = -INFINITY;
#pragma unroll
        for (int u = 0; u < MU_REG_QUADS; ++u)
            m = __builtin_fmaxf(__builtin_fmaxf(__builtin_fmaxf(m, x[u].x), __builtin_fmaxf(x[u].y, x[u].z)), x[u].w);
        // T = the largest over the wavefronts of "k-th largest of the wavefront's maxima"
        float mm = m, tw = -INFINITY;
        for (int j = 0; j < k; ++j) {
            tw = wave_max_f32(mm);
            if (mm == tw) mm = -INFINITY;
        }
        __shared__ float tws[MU_WAVES];
        if (lane == 0) tws[wave] = tw;
        __syncthreads();                                             // also orders list_n = 0 before the appends
        const float T = __builtin_fmaxf(__builtin_fmaxf(tws[0], tws[1]), __builtin_fmaxf(tws[2], tws[3]));
#pragma unroll
        for (int u = 0; u < MU_REG_QUADS; ++u) {
            const int32_t qu = q0 + tid + u * MU_THREADS;
            if (qu < q1) {
                const float e[4] = {x[u].x, x[u].y, x[u].z, x[u].w};
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    if (e[t] >= T) {
                        const int slot = atomicAdd(&list_n, 1);
                        if (slot < MU_LIST) list[slot] = rank_key(e[t], qu * 4 + t);
                    }
                }
            }
        }
        __syncthreads();
        const int32_t nl = list_n;
        if (nl <= MU_LIST) {                                         // uniform
            if (wave == 0) {
                u64 c4[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) c4[t] = (lane + t * 64) < nl ? list[lane + t * 64] : 0;
#pragma unroll
                for (int a = 0; a < 3; ++a)
#pragma unroll
                    for (int t = 0; t + 1 < 4 - a; ++t)
                        if (c4[t + 1] > c4[t]) { const u64 sw = c4[t]; c4[t] = c4[t + 1]; c4[t + 1] = sw; }
                for (int j = 0; j < k; ++j) {
                    const u64 gmax = wave_max_u64(c4[0]);
                    if (lane == 0) out[j] = gmax;
                    if (gmax != 0 && c4[0] == gmax) { c4[0] = c4[1]; c4[1] = c4[2]; c4[2] = c4[3]; c4[3] = 0; }
                }
            }
            exact = false;
        }
        __syncthreads();
    }
    if (!exact) return;

    // exact streaming path: per-thread sorted lists of KK keys
    u64 top[KK];
#pragma unroll
    for (int j = 0; j < KK; ++j) top[j] = 0;
    float worst = -INFINITY;
    scan_chunk(row, V, q0, q1, tid, [&](float v, int32_t id) { topk_insert<KK>(top, worst, v, id); });
    select_rounds<KK>(top, k, red, out, tid, lane, wave);
}

// One wavefront per node: merge the chunks' keys, write the greedy token and the matrix row.
__global__ __launch_bounds__(64) void matrix_update_merge_kernel(
    const int32_t* __restrict__ tokens, const int32_t* __restrict__ n_nodes, int32_t V, int32_t B,
    int32_t K_max, int32_t k, const u64* __restrict__ partial, int32_t* __restrict__ M,
    int32_t* __restrict__ target_ids) {
    const int node = blockIdx.x;                    // b * K_max + i
    const int b = node / K_max, i = node - b * K_max;
    const int lane = threadIdx.x;
    const int32_t n = n_nodes[b];
    if (i >= n || n > K_max) {
        if (lane == 0) target_ids[node] = -1;
        return;
    }
    // GRAFT_ARGMAX_CHUNKS * k <= 256 candidates: four per lane, kept sorted
    const u64* cand = partial + static_cast<size_t>(node) * GRAFT_ARGMAX_CHUNKS * k;
    const int n_cand = GRAFT_ARGMAX_CHUNKS * k;
    u64 c[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) c[t] = (lane + 64 * t) < n_cand ? cand[lane + 64 * t] : 0;
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int t = 0; t + 1 < 4 - a; ++t)
            if (c[t + 1] > c[t]) { const u64 s = c[t]; c[t] = c[t + 1]; c[t + 1] = s; }
    // is this the last node (largest b, then i) carrying its token?
    const int32_t x = tokens[node];
    bool later = false;
    const int total = B * K_max;
    for (int o = node + 1 + lane; o < total; o += 64) {
        const int ob = o / K_max, oi = o - ob * K_max;
        const int32_t on = n_nodes[ob];
        if (oi < on && on <= K_max && tokens[o] == x) later = true;
    }
    const bool write_row = x >= 0 && x < V && __builtin_amdgcn_ballot_w64(later) == 0;
    for (int j = 0; j < k; ++j) {
        const u64 gmax = wave_max_u64(c[0]);
        if (lane == 0) {
            const int32_t id = gmax != 0 ? key_id(gmax) : -1;
            if (j == 0) target_ids[node] = id;
            if (write_row) M[static_cast<size_t>(x) * k + j] = id;
        }
        if (gmax != 0 && c[0] == gmax) { c[0] = c[1]; c[1] = c[2]; c[2] = c[3]; c[3] = 0; }
    }
}

}  // namespace graft

extern "C" int32_t graft_matrix_retrieve(const int32_t* M, int32_t V, int32_t k,
                                         const int32_t* tpl_parent, const int32_t* tpl_rank, int32_t N,
                                         const int32_t* n_ret, int32_t B, int32_t K_max,
                                         int32_t* tokens, int32_t* parent, int32_t* n_nodes, int32_t* status,
                                         void* stream) {
    if (!M || !tpl_parent || !tpl_rank || !n_ret || !tokens || !parent || !n_nodes || !status) return GRAFT_ERR_NULL;
    if (V < 1 || k < 1 || k > GRAFT_MAX_SUCCESSORS || N < 1 || N > GRAFT_MAX_NODES || B < 1 || K_max < 1 ||
        K_max > GRAFT_MAX_NODES)
        return GRAFT_ERR_SHAPE;
    hipLaunchKernelGGL(graft::matrix_retrieve_kernel, dim3(B), dim3(graft::MR_THREADS), 0,
                       static_cast<hipStream_t>(stream), M, V, k, tpl_parent, tpl_rank, N, n_ret, K_max,
                       tokens, parent, n_nodes, status);
    return graft::check_launch();
}

extern "C" size_t graft_matrix_update_workspace_bytes(int32_t B, int32_t K_max, int32_t V, int32_t k) {
    if (B < 1 || K_max < 1 || K_max > GRAFT_MAX_NODES || V < 1 || k < 1 || k > GRAFT_MAX_SUCCESSORS) return 0;
    return static_cast<size_t>(B) * K_max * GRAFT_ARGMAX_CHUNKS * k * sizeof(unsigned long long);
}

extern "C" int32_t graft_matrix_update(const int32_t* tokens, const int32_t* n_nodes, const float* logits,
                                       int32_t V, int32_t B, int32_t K_max, int32_t* M, int32_t k,
                                       int32_t* target_ids, void* workspace, size_t workspace_bytes,
                                       void* stream) {
    using namespace graft;
    if (!tokens || !n_nodes || !logits || !M || !target_ids) return GRAFT_ERR_NULL;
    if (B < 1 || B > 65535 || K_max < 1 || K_max > GRAFT_MAX_NODES || V < 1 || k < 1 ||
        k > GRAFT_MAX_SUCCESSORS || k > V || static_cast<int64_t>(B) * K_max > 65536)
        return GRAFT_ERR_SHAPE;
    const size_t need = graft_matrix_update_workspace_bytes(B, K_max, V, k);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<size_t>(workspace) & 7) != 0)
        return GRAFT_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    u64* partial = static_cast<u64*>(workspace);
    dim3 grid(GRAFT_ARGMAX_CHUNKS, K_max, B);
    if (k <= 4) hipLaunchKernelGGL(topk_chunk_kernel<4>, grid, dim3(MU_THREADS), 0, s, logits, n_nodes, K_max, V, k, partial);
    else if (k <= 8) hipLaunchKernelGGL(topk_chunk_kernel<8>, grid, dim3(MU_THREADS), 0, s, logits, n_nodes, K_max, V, k, partial);
    else hipLaunchKernelGGL(topk_chunk_kernel<16>, grid, dim3(MU_THREADS), 0, s, logits, n_nodes, K_max, V, k, partial);
    int32_t rc = check_launch();
    if (rc != GRAFT_OK) return rc;
    hipLaunchKernelGGL(matrix_update_merge_kernel, dim3(B * K_max), dim3(64), 0, s, tokens, n_nodes, V, B, K_max, k,
                       partial, M, target_ids);
    return check_launch();
}
