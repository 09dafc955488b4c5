// graft_kv_compact: after acceptance the accepted path's keys and values move from their
// tree slots to the positions right behind the prefix, in every layer's paged cache.
//
// The rows to move are few (accept_len * Hkv * D elements per layer and side), so the call is
// a scatter of short copies, bound by memory latency.  One thread owns one 16-byte column
// of a token row (a fixed KV head and element range) for one sequence and layer and walks
// the path in order, eight rows at a time: all eight (K and V: sixteen loads) are in flight
// before the first store.  Doing this in place is safe because the path increases strictly:
// position P + k is written by the thread that alone reads this column, and only after it
// has read every source P + path[k'] with k' <= k + 7; later sources lie beyond P + k + 7.
#include "common.h"

namespace graft {

constexpr int KC_THREADS = 256;
constexpr int KC_BATCH = 8;

struct CompactParams {
    void* k;
    void* v;
    const int32_t* block_table;
    const int32_t* prefix_len;
    const int32_t* path;
    const int32_t* accept_len;
    int32_t* new_prefix_len;
    int32_t* status;
    int64_t layer_stride, page_stride, token_stride, head_stride;   // in elements
    int32_t max_pages, depth_cap, K_max, Hkv, D, elem_bytes, cols_per_head;
};

__global__ __launch_bounds__(KC_THREADS) void kv_compact_kernel(CompactParams p) {
    const int b = blockIdx.z, layer = blockIdx.y;
    const int col = blockIdx.x * KC_THREADS + threadIdx.x;          // 16-byte column of a token row
    __shared__ int32_t pth[GRAFT_MAX_NODES];
    __shared__ int32_t verdict;
    const int32_t P = p.prefix_len[b], a = p.accept_len[b];
    const int32_t* path_b = p.path + static_cast<size_t>(b) * (p.depth_cap + 1);
    const bool len_ok = P >= 0 && a >= 0 && a <= p.depth_cap;
    if (len_ok)
        for (int k = threadIdx.x; k <= a; k += KC_THREADS) pth[k] = path_b[k];
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t st = 0;
        if (!len_ok) {
            st = GRAFT_STATUS_BAD_LENGTH;
        } else {
            bool ok = pth[0] == 0;
            for (int k = 1; k <= a && ok; ++k) ok = pth[k] > pth[k - 1] && pth[k] < p.K_max;
            if (!ok) st = GRAFT_STATUS_BAD_TREE;
            else if (a > 0 && static_cast<int64_t>(P) + pth[a] >= static_cast<int64_t>(p.max_pages) * GRAFT_PAGE_SIZE)
                st = GRAFT_STATUS_BAD_LENGTH;
        }
        verdict = st;
        if (layer == 0 && blockIdx.x == 0) {
            p.status[b] = st;
            p.new_prefix_len[b] = st == 0 ? P + a + 1 : P;
        }
    }
    __syncthreads();
    if (verdict != 0 || a == 0) return;
    const int g = col / p.cols_per_head;
    if (g >= p.Hkv) return;
    const int64_t col_off = (static_cast<int64_t>(g) * p.head_stride) * p.elem_bytes +
                            static_cast<int64_t>(col - g * p.cols_per_head) * 16;
    const int32_t* table = p.block_table + static_cast<size_t>(b) * p.max_pages;
    unsigned char* kb = static_cast<unsigned char*>(p.k) + static_cast<int64_t>(layer) * p.layer_stride * p.elem_bytes + col_off;
    unsigned char* vb = static_cast<unsigned char*>(p.v) + static_cast<int64_t>(layer) * p.layer_stride * p.elem_bytes + col_off;
    auto row_off = [&](int32_t t) {
        return (static_cast<int64_t>(table[t >> 4]) * p.page_stride + static_cast<int64_t>(t & 15) * p.token_stride) *
               p.elem_bytes;
    };
    for (int k0 = 1; k0 <= a; k0 += KC_BATCH) {
        uint4 kr[KC_BATCH], vr[KC_BATCH];
#pragma unroll
        for (int j = 0; j < KC_BATCH; ++j) {
            if (k0 + j <= a) {
                const int64_t src = row_off(P + pth[k0 + j]);
                kr[j] = *reinterpret_cast<const uint4*>(kb + src);
                vr[j] = *reinterpret_cast<const uint4*>(vb + src);
            }
        }
#pragma unroll
        for (int j = 0; j < KC_BATCH; ++j) {
            if (k0 + j <= a) {
                const int64_t dst = row_off(P + k0 + j);
                *reinterpret_cast<uint4*>(kb + dst) = kr[j];
                *reinterpret_cast<uint4*>(vb + dst) = vr[j];
            }
        }
    }
}

}  // namespace graft

extern "C" int32_t graft_kv_compact(void* k_cache, void* v_cache, int64_t layer_stride, int32_t n_layers,
                                    int64_t page_stride, int64_t token_stride, int64_t head_stride,
                                    const int32_t* block_table, int32_t max_pages,
                                    const int32_t* prefix_len, const int32_t* path, const int32_t* accept_len,
                                    int32_t B, int32_t depth_cap, int32_t K_max, int32_t Hkv, int32_t D,
                                    int32_t dtype, int32_t* new_prefix_len, int32_t* status, void* stream) {
    using namespace graft;
    if (!k_cache || !v_cache || !block_table || !prefix_len || !path || !accept_len || !new_prefix_len || !status)
        return GRAFT_ERR_NULL;
    if (dtype != GRAFT_F32 && dtype != GRAFT_BF16) return GRAFT_ERR_DTYPE;
    const int32_t es = dtype == GRAFT_F32 ? 4 : 2;
    // 16-byte columns: every stride must keep them aligned
    const int64_t align = 16 / es;
    if (B < 1 || B > 65535 || n_layers < 1 || n_layers > 65535 || depth_cap < 0 || depth_cap >= GRAFT_MAX_NODES ||
        K_max < 1 || K_max > GRAFT_MAX_NODES || Hkv < 1 || Hkv > 65535 || (D != 64 && D != 128) || max_pages < 1 ||
        page_stride < 1 || token_stride < D || head_stride < D || layer_stride < 0 ||
        (n_layers > 1 && layer_stride < 1) || page_stride % align != 0 || token_stride % align != 0 ||
        head_stride % align != 0 || layer_stride % align != 0)
        return GRAFT_ERR_SHAPE;
    if ((reinterpret_cast<size_t>(k_cache) | reinterpret_cast<size_t>(v_cache)) & 15) return GRAFT_ERR_SHAPE;
    // Every workgroup of a sequence reads prefix_len[b] when it starts and one of them writes
    // new_prefix_len[b]: the two arrays must not share memory.
    if (new_prefix_len < prefix_len + B && prefix_len < new_prefix_len + B) return GRAFT_ERR_SHAPE;
    CompactParams p{};
    p.k = k_cache; p.v = v_cache; p.block_table = block_table; p.prefix_len = prefix_len; p.path = path;
    p.accept_len = accept_len; p.new_prefix_len = new_prefix_len; p.status = status;
    p.layer_stride = layer_stride; p.page_stride = page_stride; p.token_stride = token_stride;
    p.head_stride = head_stride; p.max_pages = max_pages; p.depth_cap = depth_cap; p.K_max = K_max;
    p.Hkv = Hkv; p.D = D; p.elem_bytes = es; p.cols_per_head = D * es / 16;
    const int cols = Hkv * p.cols_per_head;
    dim3 grid((cols + KC_THREADS - 1) / KC_THREADS, n_layers, B);
    hipLaunchKernelGGL(kv_compact_kernel, grid, dim3(KC_THREADS), 0, static_cast<hipStream_t>(stream), p);
    return check_launch();
}
