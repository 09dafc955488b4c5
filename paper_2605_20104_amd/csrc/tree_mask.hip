// graft_build_tree_mask: parent list -> ancestor bitmasks, depths, position ids, leaf paths.
//
// One 128-thread workgroup (two wavefronts) per sequence, one thread per tree
// slot.  The parent list sits in LDS; each thread walks its own ancestor chain
// (at most K steps), so the whole call is a few hundred LDS reads deep and
// launch-latency bound.  Leaves are ranked with a wavefront ballot + popcount.
#include "common.h"

namespace graft {

constexpr int TM_THREADS = GRAFT_MAX_NODES;

__global__ __launch_bounds__(TM_THREADS) void tree_mask_kernel(
    const int32_t* __restrict__ parent, const int32_t* __restrict__ n_nodes,
    const int32_t* __restrict__ prefix_len, int32_t K_max,
    u64* __restrict__ mask, int32_t* __restrict__ pos, int32_t* __restrict__ depth,
    int32_t* __restrict__ paths, int32_t n_leaf_max, int32_t depth_cap, int32_t* __restrict__ status) {
    const int b = blockIdx.x;
    const int i = threadIdx.x;
    __shared__ int32_t par[TM_THREADS];
    __shared__ int32_t has_child[TM_THREADS];
    __shared__ int32_t wave_leaves[TM_THREADS / 64];
    __shared__ int32_t or_bad[2], or_over[2];

    const int32_t n = n_nodes[b];
    const int32_t P = prefix_len[b];          // with the other inputs: one trip to memory for all of them
    const bool n_ok = n >= 1 && n <= K_max;
    const int32_t p = i < K_max ? parent[static_cast<size_t>(b) * K_max + i] : -1;
    bool bad = !n_ok;
    if (n_ok && i < n) bad = (i == 0) ? (p != -1) : (p < 0 || p >= i);
    par[i] = p;
    has_child[i] = 0;
    const bool any_bad = workgroup_or_128(bad, or_bad);

    const int32_t width = depth_cap + 1;
    int32_t* paths_b = paths ? paths + static_cast<size_t>(b) * n_leaf_max * width : nullptr;
    u64* mask_b = mask + static_cast<size_t>(b) * K_max * GRAFT_MASK_WORDS;

    if (any_bad) {
        if (i < K_max) {
            mask_b[i * GRAFT_MASK_WORDS] = 0;
            mask_b[i * GRAFT_MASK_WORDS + 1] = 0;
            pos[static_cast<size_t>(b) * K_max + i] = -1;
            depth[static_cast<size_t>(b) * K_max + i] = -1;
        }
        if (paths_b)
            for (int k = i; k < n_leaf_max * width; k += TM_THREADS) paths_b[k] = -1;
        if (i == 0) status[b] = GRAFT_STATUS_BAD_TREE;
        return;
    }

    // the path table starts as all -1 (consecutive addresses, all threads; these stores are on
    // their way during the walk below); the barriers of the leaf ranking order them before the
    // leaves' own entries
    if (paths_b)
        for (int k = i; k < n_leaf_max * width; k += TM_THREADS) paths_b[k] = -1;

    int32_t d = -1;
    if (i < K_max) {
        // (the walk's dependent chain is the LDS read of the parent alone: the mask bits are set in
        //  32-bit words, off that chain)
        unsigned w0 = 0, w1 = 0, w2 = 0, w3 = 0;              // mask bits 0..31, 32..63, 64..95, 96..127
        if (i < n) {
            for (int32_t j = i; j != -1;) {
                const int32_t up = par[j];
                const unsigned bit = 1u << (j & 31);
                const int word = j >> 5;
                w0 |= word == 0 ? bit : 0u;
                w1 |= word == 1 ? bit : 0u;
                w2 |= word == 2 ? bit : 0u;
                w3 |= word == 3 ? bit : 0u;
                ++d;
                j = up;
            }
        }
        mask_b[i * GRAFT_MASK_WORDS] = (static_cast<u64>(w1) << 32) | w0;
        mask_b[i * GRAFT_MASK_WORDS + 1] = (static_cast<u64>(w3) << 32) | w2;
        depth[static_cast<size_t>(b) * K_max + i] = d;
        pos[static_cast<size_t>(b) * K_max + i] = i < n ? P + d : -1;
    }

    int overflow = 0;
    if (paths_b) {
        if (i > 0 && i < n) has_child[p] = 1;          // same value from every writer
        __syncthreads();
        const bool leaf = i < n && has_child[i] == 0;
        const u64 ballot = __ballot(leaf);
        const int lane = i & 63, wave = i >> 6;
        if (lane == 0) wave_leaves[wave] = __popcll(ballot);
        __syncthreads();
        int32_t rank = __popcll(ballot & ((1ull << lane) - 1));
        if (wave == 1) rank += wave_leaves[0];
        if (leaf) {
            if (rank >= n_leaf_max) {
                overflow = 1;                          // dropped
            } else {
                int32_t* row = paths_b + static_cast<size_t>(rank) * width;
                if (d > depth_cap) {
                    overflow = 1;                      // its row stays -1
                } else {
                    int32_t k = d;
                    for (int32_t j = i; j != -1; j = par[j]) row[k--] = j;
                }
            }
        }
    }
    const bool any_over = workgroup_or_128(overflow != 0, or_over);
    if (i == 0) status[b] = any_over ? GRAFT_STATUS_PATH_OVERFLOW : 0;
}

}  // namespace graft

extern "C" int32_t graft_build_tree_mask(const int32_t* parent, const int32_t* n_nodes,
                                         const int32_t* prefix_len, int32_t B, int32_t K_max,
                                         uint64_t* mask, int32_t* pos, int32_t* depth, int32_t* paths,
                                         int32_t n_leaf_max, int32_t depth_cap, int32_t* status,
                                         void* stream) {
    if (!parent || !n_nodes || !prefix_len || !mask || !pos || !depth || !status) return GRAFT_ERR_NULL;
    if (B < 1 || K_max < 1 || K_max > GRAFT_MAX_NODES) return GRAFT_ERR_SHAPE;
    if (paths && (n_leaf_max < 1 || n_leaf_max > GRAFT_MAX_NODES || depth_cap < 0 ||
                  depth_cap >= GRAFT_MAX_NODES))
        return GRAFT_ERR_SHAPE;
    hipLaunchKernelGGL(graft::tree_mask_kernel, dim3(B), dim3(graft::TM_THREADS), 0,
                       static_cast<hipStream_t>(stream), parent, n_nodes, prefix_len, K_max,
                       reinterpret_cast<graft::u64*>(mask), pos, depth, paths, n_leaf_max, depth_cap,
                       status);
    return graft::check_launch();
}
