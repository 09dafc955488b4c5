// graft_accept: greedy acceptance walk over the verified hybrid tree.
//
// Two kernels.  In logits mode an argmax kernel scans every node's logits row
// once (an HBM scan: V*4 bytes per node), GRAFT_ARGMAX_CHUNKS workgroups per row
// so that even one sequence fills the chip; each writes its chunk's (value,
// first index) to the workspace.  The walk kernel (one 128-thread workgroup per
// sequence, one thread per node) folds the chunk partials into the target's
// greedy token per node, checks each node's whole ancestor chain, and a
// workgroup-wide max over (depth, -index) picks the deepest accepted node.
#include <mutex>

#include "common.h"

namespace graft {

constexpr int AM_THREADS = 256;
constexpr int AC_THREADS = GRAFT_MAX_NODES;

struct ArgPartial { float val; int32_t idx; };

// "first maximum": larger value wins, equal values keep the smaller index.
__device__ __forceinline__ void arg_take(float& bv, int32_t& bi, float v, int32_t i) {
    if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
}

__global__ __launch_bounds__(AM_THREADS) void argmax_chunk_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ n_nodes, int32_t K_max, int32_t V,
    ArgPartial* __restrict__ partial) {
    const int chunk = blockIdx.x, i = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x;
    ArgPartial* out = partial + (static_cast<size_t>(b) * K_max + i) * GRAFT_ARGMAX_CHUNKS + chunk;
    const int32_t n = n_nodes[b];
    if (i >= n || n > K_max) {                   // padding node: nothing to scan
        if (tid == 0) { out->val = -INFINITY; out->idx = 0x7fffffff; }
        return;
    }
    // chunk boundaries in units of 4 elements so that aligned rows can use 16-byte loads
    const int32_t quads = (V + 3) / 4;
    const int32_t per = (quads + GRAFT_ARGMAX_CHUNKS - 1) / GRAFT_ARGMAX_CHUNKS;
    const int32_t q0 = chunk * per;
    const int32_t q1 = (q0 + per) < quads ? (q0 + per) : quads;
    const float* row = logits + (static_cast<size_t>(b) * K_max + i) * V;
    float bv = -INFINITY;
    int32_t bi = 0x7fffffff;
    const bool vec = (V % 4 == 0);               // then every row start is 16-byte aligned
    if (vec) {
        const float4* row4 = reinterpret_cast<const float4*>(row);
        constexpr int U = 4;                         // 16-byte loads in flight per thread
        for (int32_t qd = q0 + tid; qd < q1; qd += U * AM_THREADS) {
            float4 x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int32_t qu = qd + u * AM_THREADS;
                x[u] = row4[qu < q1 ? qu : qd];      // a lane past the end re-reads its first quad (skipped below)
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int32_t qu = qd + u * AM_THREADS;
                if (qu < q1) {
                    const int32_t base = qu * 4;
                    arg_take(bv, bi, x[u].x, base);
                    arg_take(bv, bi, x[u].y, base + 1);
                    arg_take(bv, bi, x[u].z, base + 2);
                    arg_take(bv, bi, x[u].w, base + 3);
                }
            }
        }
    } else {
        const int32_t e0 = q0 * 4, e1 = (q1 * 4) < V ? (q1 * 4) : V;
        for (int32_t e = e0 + tid; e < e1; e += AM_THREADS) arg_take(bv, bi, row[e], e);
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        float ov = __shfl_xor(bv, s);
        int32_t oi = __shfl_xor(bi, s);
        arg_take(bv, bi, ov, oi);
    }
    __shared__ float sv[AM_THREADS / 64];
    __shared__ int32_t si[AM_THREADS / 64];
    if ((tid & 63) == 0) { sv[tid >> 6] = bv; si[tid >> 6] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < AM_THREADS / 64; ++w) arg_take(bv, bi, sv[w], si[w]);
        out->val = bv;
        out->idx = bi;
    }
}

__global__ __launch_bounds__(AC_THREADS) void accept_walk_kernel(
    const int32_t* __restrict__ parent, const int32_t* __restrict__ tokens,
    const int32_t* __restrict__ n_nodes, const ArgPartial* __restrict__ partial,
    int32_t* __restrict__ target_ids, int32_t K_max, int32_t depth_cap,
    int32_t* __restrict__ accept_len, int32_t* __restrict__ best_node, int32_t* __restrict__ path,
    int32_t* __restrict__ out_tokens, int32_t* __restrict__ status) {
    const int b = blockIdx.x;
    const int i = threadIdx.x;
    __shared__ int32_t par[AC_THREADS];
    __shared__ int32_t tok[AC_THREADS];
    __shared__ int32_t tstar[AC_THREADS];
    __shared__ u64 red[AC_THREADS / 64];
    __shared__ int32_t best_d;
    __shared__ int32_t or_bad[2], or_over[2];

    const int32_t n = n_nodes[b];
    const bool n_ok = n >= 1 && n <= K_max;
    const size_t row = static_cast<size_t>(b) * K_max;
    const int32_t p = i < K_max ? parent[row + i] : -1;
    bool bad = !n_ok;
    if (n_ok && i < n) bad = (i == 0) ? (p != -1) : (p < 0 || p >= i);
    par[i] = p;
    tok[i] = i < K_max ? tokens[row + i] : -1;
    // (requested with the other inputs: one trip to memory for all of them)
    const int32_t ts_given = (!partial && i < K_max) ? target_ids[row + i] : -1;
    const bool any_bad = workgroup_or_128(bad, or_bad);

    const int32_t width = depth_cap + 1;
    int32_t* path_b = path + static_cast<size_t>(b) * width;
    int32_t* out_b = out_tokens + static_cast<size_t>(b) * width;
    if (any_bad) {
        for (int k = i; k < width; k += AC_THREADS) { path_b[k] = -1; out_b[k] = -1; }
        if (partial && i < K_max) target_ids[row + i] = -1;
        if (i == 0) { accept_len[b] = 0; best_node[b] = -1; status[b] = GRAFT_STATUS_BAD_TREE; }
        return;
    }

    // the target's greedy token after each node
    int32_t ts = -1;
    if (i < K_max) {
        if (partial) {
            if (i < n) {
                const ArgPartial* pr = partial + (row + i) * GRAFT_ARGMAX_CHUNKS;
                float bv = pr[0].val;
                int32_t bi = pr[0].idx;
                for (int c = 1; c < GRAFT_ARGMAX_CHUNKS; ++c) arg_take(bv, bi, pr[c].val, pr[c].idx);
                ts = bi;
            }
            target_ids[row + i] = ts;
        } else {
            ts = ts_given;
        }
    }
    tstar[i] = ts;
    __syncthreads();

    // accepted iff every node on the path below the root carries its parent's greedy token
    bool ok = i < n;
    int32_t d = 0;
    if (ok) {
        for (int32_t j = i; j != 0; j = par[j]) {
            ok = ok && tok[j] == tstar[par[j]];
            ++d;
        }
    }
    const int over = (ok && d > depth_cap) ? 1 : 0;
    // key: depth first, then smaller index; 0 = not a candidate (the root gives key >= 1)
    u64 key = (ok && d <= depth_cap) ? ((static_cast<u64>(d) << 8) | static_cast<u64>(255 - i)) : 0;
    u64 wmax = wave_max_u64(key);
    if ((i & 63) == 0) red[i >> 6] = wmax;
    const bool any_over = workgroup_or_128(over != 0, or_over);
    const u64 gmax = red[0] > red[1] ? red[0] : red[1];
    if (key == gmax) {                           // unique: the index is part of the key
        accept_len[b] = d;
        best_node[b] = i;
        status[b] = any_over ? GRAFT_STATUS_PATH_OVERFLOW : 0;
        best_d = d;
        int32_t k = d;
        for (int32_t j = i; j != -1; j = par[j]) {
            path_b[k] = j;
            if (k > 0) out_b[k - 1] = tok[j];
            --k;
        }
        out_b[d] = ts;
    }
    __syncthreads();
    // the padding behind the path: all threads, not one after the other
    for (int32_t k = best_d + 1 + i; k < width; k += AC_THREADS) { path_b[k] = -1; out_b[k] = -1; }
}

// ---- graft_accept_noalloc: the argmax partials live in a file-scope device array ----------
// In host code the array's name is only a stand-in for the symbol: the device address is
// asked for once per device (hipGetSymbolAddress with that device current; every GPU holds its
// own copy at its own address) and that pointer is what the kernels get.
constexpr int NA_MAX_ROWS = GRAFT_NOALLOC_MAX_ROWS;   // B * K_max logits rows per call
constexpr int NA_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[static_cast<size_t>(NA_MAX_ROWS) * GRAFT_ARGMAX_CHUNKS *
                                                       sizeof(ArgPartial)];   // 1 MiB
static void* g_scratch_ptr[NA_MAX_DEVICES];
static std::mutex g_scratch_lock;

// Device address of `scratch` on the current device, or nullptr (with the HIP error recorded).
static ArgPartial* scratch_on_current_device() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= NA_MAX_DEVICES)) e = hipErrorInvalidDevice;
    if (e == hipSuccess) {
        std::lock_guard<std::mutex> hold(g_scratch_lock);
        if (!g_scratch_ptr[dev]) {
            void* ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e == hipSuccess && !ptr) e = hipErrorInvalidSymbol;
            if (e == hipSuccess) g_scratch_ptr[dev] = ptr;
        }
        if (e == hipSuccess) return static_cast<ArgPartial*>(g_scratch_ptr[dev]);
    }
    (void)hipGetLastError();
    set_last_hip_error(static_cast<int32_t>(e));
    return nullptr;
}

static int32_t accept_impl(const int32_t* parent, const int32_t* tokens, const int32_t* n_nodes,
                           const float* logits, int32_t V, int32_t* target_ids, int32_t B, int32_t K_max,
                           int32_t depth_cap, int32_t* accept_len, int32_t* best_node, int32_t* path,
                           int32_t* out_tokens, int32_t* status, ArgPartial* ws, hipStream_t s) {
    const ArgPartial* partial = nullptr;
    if (logits) {
        hipLaunchKernelGGL(argmax_chunk_kernel, dim3(GRAFT_ARGMAX_CHUNKS, K_max, B), dim3(AM_THREADS), 0, s,
                           logits, n_nodes, K_max, V, ws);
        int32_t rc = check_launch();
        if (rc != GRAFT_OK) return rc;
        partial = ws;
    }
    hipLaunchKernelGGL(accept_walk_kernel, dim3(B), dim3(AC_THREADS), 0, s, parent, tokens, n_nodes, partial,
                       target_ids, K_max, depth_cap, accept_len, best_node, path, out_tokens, status);
    return check_launch();
}

static int32_t accept_args_ok(const int32_t* parent, const int32_t* tokens, const int32_t* n_nodes,
                              const int32_t* target_ids, int32_t B, int32_t K_max, int32_t depth_cap,
                              const int32_t* accept_len, const int32_t* best_node, const int32_t* path,
                              const int32_t* out_tokens, const int32_t* status) {
    if (!parent || !tokens || !n_nodes || !target_ids || !accept_len || !best_node || !path ||
        !out_tokens || !status)
        return GRAFT_ERR_NULL;
    if (B < 1 || B > 65535 || K_max < 1 || K_max > GRAFT_MAX_NODES || depth_cap < 0 ||
        depth_cap >= GRAFT_MAX_NODES)
        return GRAFT_ERR_SHAPE;
    return GRAFT_OK;
}

}  // namespace graft

extern "C" size_t graft_accept_workspace_bytes(int32_t B, int32_t K_max, int32_t V) {
    if (B < 1 || K_max < 1 || V < 1) return 0;
    return static_cast<size_t>(B) * K_max * GRAFT_ARGMAX_CHUNKS * sizeof(graft::ArgPartial);
}

extern "C" int32_t graft_accept(const int32_t* parent, const int32_t* tokens, const int32_t* n_nodes,
                                const float* logits, int32_t V, int32_t* target_ids, int32_t B,
                                int32_t K_max, int32_t depth_cap, int32_t* accept_len,
                                int32_t* best_node, int32_t* path, int32_t* out_tokens, int32_t* status,
                                void* workspace, size_t workspace_bytes, void* stream) {
    const int32_t rc = graft::accept_args_ok(parent, tokens, n_nodes, target_ids, B, K_max, depth_cap, accept_len,
                                             best_node, path, out_tokens, status);
    if (rc != GRAFT_OK) return rc;
    if (logits) {
        if (V < 1) return GRAFT_ERR_SHAPE;
        if (!workspace || workspace_bytes < graft_accept_workspace_bytes(B, K_max, V))
            return GRAFT_ERR_WORKSPACE;
    }
    return graft::accept_impl(parent, tokens, n_nodes, logits, V, target_ids, B, K_max, depth_cap, accept_len,
                              best_node, path, out_tokens, status, static_cast<graft::ArgPartial*>(workspace),
                              static_cast<hipStream_t>(stream));
}

extern "C" int32_t graft_accept_noalloc(const int32_t* parent, const int32_t* tokens, const int32_t* n_nodes,
                                        const float* logits, int32_t V, int32_t* target_ids, int32_t B,
                                        int32_t K_max, int32_t depth_cap, int32_t* accept_len,
                                        int32_t* best_node, int32_t* path, int32_t* out_tokens,
                                        int32_t* status, void* stream) {
    const int32_t rc = graft::accept_args_ok(parent, tokens, n_nodes, target_ids, B, K_max, depth_cap, accept_len,
                                             best_node, path, out_tokens, status);
    if (rc != GRAFT_OK) return rc;
    graft::ArgPartial* ws = nullptr;
    if (logits) {
        if (V < 1) return GRAFT_ERR_SHAPE;
        if (static_cast<int64_t>(B) * K_max > graft::NA_MAX_ROWS) return GRAFT_ERR_WORKSPACE;   // beyond the static scratch
        ws = graft::scratch_on_current_device();
        if (!ws) return GRAFT_ERR_HIP;
    }
    return graft::accept_impl(parent, tokens, n_nodes, logits, V, target_ids, B, K_max, depth_cap, accept_len,
                              best_node, path, out_tokens, status, ws, static_cast<hipStream_t>(stream));
}
