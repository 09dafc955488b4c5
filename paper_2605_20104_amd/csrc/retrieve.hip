// graft_retrieve: suffix n-gram lookup over the context token buffer.
//
// One 1024-thread workgroup per sequence.  The buffer is at most a few hundred
// KB, so the call is latency-bound, not bandwidth-bound: what matters is one
// launch, coalesced independent loads, and an exact total order on the hits.
//
//   1. the query (last n_max tokens of context ++ tail) goes to LDS, reversed;
//   2. every thread scans positions tid, tid+1024, ... eight at a time (eight
//      independent coalesced loads in flight), and only where the token equals
//      the query's last token walks backwards to measure the match length;
//   3. a hit is the 64-bit key (match_len << 32 | e); each thread keeps its own
//      best C keys in registers (unrolled insertion, no dynamic indexing);
//   4. C rounds of workgroup-wide max pick the global ranking: keys are unique
//      because e is, so exactly one thread owns each round's winner, writes that
//      chain and pops it.
#include "common.h"

namespace graft {

constexpr int RT_THREADS = 1024;
constexpr int RT_WAVES = RT_THREADS / 64;
constexpr int RT_UNROLL = 8;

__global__ __launch_bounds__(RT_THREADS) void retrieve_kernel(
    const int32_t* __restrict__ ctx, const int32_t* __restrict__ ctx_len, int32_t L_max,
    const int32_t* __restrict__ tail, const int32_t* __restrict__ tail_len, int32_t tail_max,
    int32_t n_min, int32_t n_max, int32_t C, int32_t m,
    int32_t* __restrict__ chain_tok, int32_t* __restrict__ chain_len, int32_t* __restrict__ chain_pos,
    int32_t* __restrict__ chain_match, int32_t* __restrict__ n_hits, int32_t* __restrict__ status) {
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    __shared__ int32_t q_rev[GRAFT_MAX_NGRAM];   // q_rev[j] = j-th token from the end of the query
    __shared__ u64 red[RT_WAVES];
    __shared__ int32_t red_cnt[RT_WAVES];

    const int32_t L = ctx_len[b];
    const int32_t T = (tail != nullptr && tail_len != nullptr) ? tail_len[b] : 0;
    const bool bad = L < 0 || L > L_max || T < 0 || T > tail_max;

    // defaults: no chain
    int32_t* tok_b = chain_tok + static_cast<size_t>(b) * C * m;
    for (int i = tid; i < C * m; i += RT_THREADS) tok_b[i] = -1;
    if (bad) {                                   // uniform over the workgroup
        if (tid < C) {
            chain_len[b * C + tid] = 0;
            chain_pos[b * C + tid] = -1;
            chain_match[b * C + tid] = 0;
        }
        if (tid == 0) { n_hits[b] = 0; status[b] = GRAFT_STATUS_BAD_LENGTH; }
        return;
    }
    const int32_t* x = ctx + static_cast<size_t>(b) * L_max;
    const int32_t QL = L + T;
    const int32_t nq = n_max < QL ? n_max : QL;
    if (tid < nq) {
        int32_t qi = QL - 1 - tid;
        q_rev[tid] = qi < L ? x[qi] : tail[static_cast<size_t>(b) * tail_max + (qi - L)];
    }
    __syncthreads();
    const int32_t q_last = nq > 0 ? q_rev[0] : 0;

    u64 top[GRAFT_MAX_CHAINS];
#pragma unroll
    for (int k = 0; k < GRAFT_MAX_CHAINS; ++k) top[k] = 0;
    int32_t my_hits = 0;

    // position i holds the token right before continuation start e = i + 1, 1 <= e <= L-1
    const int32_t last_i = L - 2;
    for (int32_t base = tid; base <= last_i; base += RT_THREADS * RT_UNROLL) {
        int32_t v[RT_UNROLL];
#pragma unroll
        for (int u = 0; u < RT_UNROLL; ++u) {
            int32_t i = base + u * RT_THREADS;
            v[u] = i <= last_i ? x[i] : 0;
        }
#pragma unroll
        for (int u = 0; u < RT_UNROLL; ++u) {
            int32_t i = base + u * RT_THREADS;
            if (i <= last_i && v[u] == q_last) {
                int32_t e = i + 1;
                int32_t cap = n_max < e ? n_max : e;
                int32_t l = 1;
                while (l < cap && x[e - 1 - l] == q_rev[l]) ++l;
                if (l >= n_min) {
                    ++my_hits;
                    u64 key = (static_cast<u64>(l) << 32) | static_cast<u64>(e);
#pragma unroll
                    for (int k = 0; k < GRAFT_MAX_CHAINS; ++k) {
                        if (key > top[k]) { u64 t = top[k]; top[k] = key; key = t; }
                    }
                }
            }
        }
    }

    // total number of hits
    int32_t cnt = my_hits;
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) cnt += __shfl_xor(cnt, s);
    if (lane == 0) red_cnt[wave] = cnt;
    __syncthreads();
    if (tid == 0) {
        int32_t total = 0;
        for (int w = 0; w < RT_WAVES; ++w) total += red_cnt[w];
        n_hits[b] = total;
        status[b] = 0;
    }

    // global ranking: C rounds of workgroup-wide max over the threads' current best keys
    for (int c = 0; c < C; ++c) {
        u64 wmax = wave_max_u64(top[0]);
        if (lane == 0) red[wave] = wmax;
        __syncthreads();
        u64 gmax = 0;
#pragma unroll
        for (int w = 0; w < RT_WAVES; ++w) gmax = red[w] > gmax ? red[w] : gmax;
        __syncthreads();
        if (gmax == 0) {                         // fewer than C hits: remaining chains stay empty
            if (tid == 0) {
                for (int cc = c; cc < C; ++cc) {
                    chain_len[b * C + cc] = 0;
                    chain_pos[b * C + cc] = -1;
                    chain_match[b * C + cc] = 0;
                }
            }
            break;
        }
        if (top[0] == gmax) {                    // exactly one thread: e is unique
            int32_t e = static_cast<int32_t>(gmax & 0xffffffffu);
            int32_t l = static_cast<int32_t>(gmax >> 32);
            int32_t cl = (L - e) < m ? (L - e) : m;
            chain_pos[b * C + c] = e;
            chain_match[b * C + c] = l;
            chain_len[b * C + c] = cl;
            for (int j = 0; j < cl; ++j) tok_b[c * m + j] = x[e + j];
#pragma unroll
            for (int k = 0; k + 1 < GRAFT_MAX_CHAINS; ++k) top[k] = top[k + 1];
            top[GRAFT_MAX_CHAINS - 1] = 0;
        }
    }
}

}  // namespace graft

extern "C" int32_t graft_retrieve(const int32_t* ctx, const int32_t* ctx_len, int32_t B, int32_t L_max,
                                  const int32_t* tail, const int32_t* tail_len, int32_t tail_max,
                                  int32_t n_min, int32_t n_max, int32_t C, int32_t m,
                                  int32_t* chain_tok, int32_t* chain_len, int32_t* chain_pos,
                                  int32_t* chain_match, int32_t* n_hits, int32_t* status, void* stream) {
    if (!ctx || !ctx_len || !chain_tok || !chain_len || !chain_pos || !chain_match || !n_hits || !status)
        return GRAFT_ERR_NULL;
    if ((tail == nullptr) != (tail_len == nullptr)) return GRAFT_ERR_NULL;
    if (B < 1 || L_max < 1 || L_max >= (1 << 30) || n_min < 1 || n_min > n_max ||
        n_max > GRAFT_MAX_NGRAM || C < 1 || C > GRAFT_MAX_CHAINS || m < 1 || m > (1 << 20) ||
        tail_max < 0 || (tail != nullptr && tail_max < 1))
        return GRAFT_ERR_SHAPE;
    hipLaunchKernelGGL(graft::retrieve_kernel, dim3(B), dim3(graft::RT_THREADS), 0,
                       static_cast<hipStream_t>(stream), ctx, ctx_len, L_max, tail, tail_len, tail_max,
                       n_min, n_max, C, m, chain_tok, chain_len, chain_pos, chain_match, n_hits, status);
    return graft::check_launch();
}
