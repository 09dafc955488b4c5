// graft_retrieve: suffix n-gram lookup over the context token buffer.
//
// One 1024-thread workgroup per sequence.  The buffer is at most a few hundred
// KB, so the call is latency-bound, not bandwidth-bound: what matters is one
// launch, few dependent memory round trips, and an exact total order on the hits.
//
//   1. the query (last n_max tokens of context ++ tail) goes to LDS, reversed;
//   2. the context passes through LDS in chunks of 16384 tokens (two buffers: 128 KB of the
//      compute unit's 160).  The loads run two chunks (32 per thread, independent and
//      coalesced) ahead of the scan and the first two are issued before anything else, so
//      a 32K-token context costs one exposed memory round trip and two passes of the scan.  Every thread looks at positions tid, tid+1024, ... of
//      the chunk and, where the token equals the query's last token, walks backwards
//      through LDS to measure the match length (the previous chunk is still in the
//      other buffer);
//   3. a hit is the 64-bit key (match_len << 32 | e); each thread keeps its own
//      best C keys in registers (unrolled insertion, no dynamic indexing);
//   4. ranking without memory traffic: each wavefront extracts its best C keys (keys are
//      unique because e is, so exactly one lane owns a maximum and pops it), wavefront 0
//      merges the 16 x C survivors the same way, and C x m threads then copy the chains
//      in one round trip.
#include "common.h"

namespace graft {

constexpr int RT_THREADS = 1024;
constexpr int RT_WAVES = RT_THREADS / 64;
constexpr int RT_UNROLL = 16;
constexpr int RT_CHUNK = RT_THREADS * RT_UNROLL;      // tokens per LDS buffer
constexpr int RT_AHEAD = 2;                           // chunks the loads run ahead of the scan

__global__ __launch_bounds__(RT_THREADS) void retrieve_kernel(
    const int32_t* __restrict__ ctx, const int32_t* __restrict__ ctx_len, int32_t L_max,
    const int32_t* __restrict__ tail, const int32_t* __restrict__ tail_len, int32_t tail_max,
    int32_t n_min, int32_t n_max, int32_t C, int32_t m,
    int32_t* __restrict__ chain_tok, int32_t* __restrict__ chain_len, int32_t* __restrict__ chain_pos,
    int32_t* __restrict__ chain_match, int32_t* __restrict__ n_hits, int32_t* __restrict__ status) {
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    __shared__ int32_t buf[2][RT_CHUNK];         // two context chunks
    __shared__ int32_t q_rev[GRAFT_MAX_NGRAM];   // q_rev[j] = j-th token from the end of the query
    __shared__ u64 red[RT_WAVES * GRAFT_MAX_CHAINS];   // per-wavefront best keys
    __shared__ u64 win[GRAFT_MAX_CHAINS];              // the C winners
    __shared__ int32_t red_cnt[RT_WAVES];

    // the first chunks do not wait for the length: every index below L_max is readable
    const int32_t* x = ctx + static_cast<size_t>(b) * L_max;
    int32_t v[RT_AHEAD][RT_UNROLL];
#pragma unroll
    for (int k = 0; k < RT_AHEAD; ++k)
#pragma unroll
        for (int u = 0; u < RT_UNROLL; ++u) {
            const int32_t i = k * RT_CHUNK + tid + u * RT_THREADS;
            v[k][u] = i < L_max ? x[i] : 0;
        }

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
    const int32_t QL = L + T;
    const int32_t nq = n_max < QL ? n_max : QL;
    if (tid < nq) {
        int32_t qi = QL - 1 - tid;
        q_rev[tid] = qi < L ? x[qi] : tail[static_cast<size_t>(b) * tail_max + (qi - L)];
    }

    u64 top[GRAFT_MAX_CHAINS];
#pragma unroll
    for (int k = 0; k < GRAFT_MAX_CHAINS; ++k) top[k] = 0;
    int32_t my_hits = 0;

    // position i holds the token right before continuation start e = i + 1, 1 <= e <= L-1
    const int32_t last_i = L - 2;
    const int32_t n_chunks = last_i >= 0 ? last_i / RT_CHUNK + 1 : 0;
    for (int32_t c0 = 0; c0 < n_chunks; c0 += RT_AHEAD) {
#pragma unroll
        for (int k = 0; k < RT_AHEAD; ++k) {
            const int32_t c = c0 + k;
            if (c >= n_chunks) continue;              // uniform over the workgroup (no break: k must stay a constant)
            int32_t* cur = buf[c & 1];
#pragma unroll
            for (int u = 0; u < RT_UNROLL; ++u) cur[tid + u * RT_THREADS] = v[k][u];
            __syncthreads();                      // chunk c (and q_rev) visible; chunk c - 1 still in the other buffer
            const int32_t q_last = nq > 0 ? q_rev[0] : 0;
            // When a hit needs at least two matching tokens, the token before position i is
            // tested as well before the (divergent) walk: with frequent tokens at the end of
            // the query almost every wavefront would otherwise enter every walk.
            const bool two = n_min >= 2;
            const int32_t q_prev = nq > 1 ? q_rev[1] : 0;
            unsigned cand = 0;
#pragma unroll
            for (int u = 0; u < RT_UNROLL; ++u) {
                const int32_t i = c * RT_CHUNK + tid + u * RT_THREADS;
                const int32_t ip = i - 1;
                const int32_t prev = ip >= 0 ? buf[(ip / RT_CHUNK) & 1][ip % RT_CHUNK] : -1;
                if (i <= last_i && v[k][u] == q_last && (!two || (ip >= 0 && prev == q_prev))) cand |= 1u << u;
            }
            // one candidate per lane and pass (usually a single pass): the walk and the insertion
            // below exist once in the code and run once per pass, whatever slot the candidate is in
            while (cand != 0) {
                const int u = __builtin_ctz(cand);
                cand &= cand - 1;
                const int32_t i = c * RT_CHUNK + tid + u * RT_THREADS;
                {
                    const int32_t e = i + 1;
                    const int32_t cap = n_max < e ? n_max : e;
                    int32_t l = 1;
                    while (l < cap) {
                        const int32_t pos = e - 1 - l;            // >= 0, at most n_max - 1 before i
                        if (buf[(pos / RT_CHUNK) & 1][pos % RT_CHUNK] != q_rev[l]) break;
                        ++l;
                    }
                    if (l >= n_min) {
                        ++my_hits;
                        u64 key = (static_cast<u64>(l) << 32) | static_cast<u64>(e);
#pragma unroll
                        for (int kk = 0; kk < GRAFT_MAX_CHAINS; ++kk) {
                            if (key > top[kk]) { u64 t = top[kk]; top[kk] = key; key = t; }
                        }
                    }
                }
            }
            if (c + RT_AHEAD < n_chunks) {        // this slot's registers are free: fetch RT_AHEAD chunks ahead
#pragma unroll
                for (int u = 0; u < RT_UNROLL; ++u) {
                    const int32_t i = (c + RT_AHEAD) * RT_CHUNK + tid + u * RT_THREADS;
                    v[k][u] = i < L_max ? x[i] : 0;
                }
            }
            __syncthreads();                      // all walks done before chunk c + 1 overwrites chunk c - 1
        }
    }

    // ---- ranking: every wavefront extracts its own best C keys (keys are unique because e is,
    //      so exactly one lane owns each maximum and pops it), then wavefront 0 merges the
    //      16 x C survivors.  No memory access between the rounds.
    int32_t cnt = my_hits;
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) cnt += __shfl_xor(cnt, s);
    if (lane == 0) red_cnt[wave] = cnt;
    for (int c = 0; c < C; ++c) {
        const u64 wmax = wave_max_u64(top[0]);
        if (lane == 0) red[wave * GRAFT_MAX_CHAINS + c] = wmax;
        if (wmax != 0 && top[0] == wmax) {
#pragma unroll
            for (int k = 0; k + 1 < GRAFT_MAX_CHAINS; ++k) top[k] = top[k + 1];
            top[GRAFT_MAX_CHAINS - 1] = 0;
        }
    }
    __syncthreads();
    if (wave == 0) {
        // lane l holds candidates l and l + 64 of the RT_WAVES * C survivors (sorted pair)
        const int n_cand = RT_WAVES * C;
        u64 k0 = 0, k1 = 0;
        if (lane < n_cand) k0 = red[(lane / C) * GRAFT_MAX_CHAINS + lane % C];
        if (lane + 64 < n_cand) k1 = red[((lane + 64) / C) * GRAFT_MAX_CHAINS + (lane + 64) % C];
        if (k1 > k0) { const u64 t = k0; k0 = k1; k1 = t; }
        for (int c = 0; c < C; ++c) {
            const u64 gmax = wave_max_u64(k0);
            if (lane == 0) win[c] = gmax;
            if (gmax != 0 && k0 == gmax) { k0 = k1; k1 = 0; }
        }
        if (lane == 0) {
            int32_t total = 0;
            for (int w = 0; w < RT_WAVES; ++w) total += red_cnt[w];
            n_hits[b] = total;
            status[b] = 0;
        }
    }
    __syncthreads();
    // ---- outputs: chain c starts at e = low word of win[c]; all copies in one round trip
    if (tid < C) {
        const u64 key = win[tid];
        const int32_t e = static_cast<int32_t>(key & 0xffffffffu);
        const int32_t l = static_cast<int32_t>(key >> 32);
        const int32_t cl = key == 0 ? 0 : ((L - e) < m ? (L - e) : m);
        chain_pos[b * C + tid] = key == 0 ? -1 : e;
        chain_match[b * C + tid] = l;
        chain_len[b * C + tid] = cl;
    }
    for (int i = tid; i < C * m; i += RT_THREADS) {
        const int c = i / m, jj = i - c * m;
        const u64 key = win[c];
        const int32_t e = static_cast<int32_t>(key & 0xffffffffu);
        if (key != 0 && e + jj < L) tok_b[i] = x[e + jj];
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
