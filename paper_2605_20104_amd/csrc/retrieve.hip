// graft_retrieve: suffix n-gram lookup over the context token buffer.
//
// One 1024-thread workgroup per sequence.  The buffer is at most a few hundred
// KB, so the call is latency-bound, not bandwidth-bound: what matters is one
// launch, few dependent memory round trips, and an exact total order on the hits.
//
//   1. the context passes through LDS in chunks of 16384 tokens (two buffers, a ring: 128 KB of
//      the compute unit's 160).  The lengths are requested first and the first two chunks right
//      behind them, before the lengths are back (every index below L_max is readable); a thread
//      loads groups of four consecutive tokens with 16-byte loads.  Both chunks and the tail go to
//      LDS at once, and the query (last n_max tokens of context ++ tail, reversed) is read from
//      there: a context of up to 32768 tokens costs one memory round trip and three barriers
//      before the ranking;
//   2. scan: one compare per token against the query's last token, and a wavefront in which no
//      lane has it goes on (in text it is rare).  Otherwise the lanes test the token before as
//      well (in a register, or for the first of a group in LDS) where a hit needs two tokens, and
//      a candidate's match length is measured backwards through the ring, eight tokens per round
//      of independent reads;
//   3. a hit is the 64-bit key (match_len << 32 | e); each thread keeps its own best C keys in
//      registers (unrolled insertion, no dynamic indexing);
//   4. ranking without memory traffic.  The threads that have hits append their best C keys to a
//      short list in LDS (one 64-bit atomic reserves the places and counts the hits) and every
//      key counts how many of the list are larger: that is its rank (keys are unique because e
//      is).  A list that overflows (periodic text, tiny alphabets) takes the tournament instead:
//      each wavefront extracts its best C keys (exactly one lane owns a maximum and pops it),
//      wavefront 0 merges the 16 x C survivors the same way.  C x m threads then copy the chains,
//      from LDS where the chunk that holds them is still there.
//
// Measured on a 32768-token context (cycle stamps): with one position per lane and load, a
// dependent query load, a tournament in all 16 wavefronts and a serial backward walk the kernel
// took 10.4 us; 2.3 us of that were the tournament (its vector instructions, issued by 16
// wavefronts that almost never hold a hit), 2 x 1.5 us the walks of the single wavefront per chunk
// that had a candidate (250 instructions of signed index arithmetic and per-token branches per
// round), 0.5 us each the dependent query load, the second chunk's barrier pair and the chain
// copy from memory.  This form takes 6.1 us.
#include "common.h"

namespace graft {

constexpr int RT_THREADS = 1024;
constexpr int RT_WAVES = RT_THREADS / 64;
constexpr int RT_GROUPS = 4;                          // groups of four consecutive tokens per thread and chunk
constexpr int RT_UNROLL = 4 * RT_GROUPS;
constexpr int RT_CHUNK = RT_THREADS * RT_UNROLL;      // tokens per LDS buffer
// Four consecutive tokens.  The context rows are only known to be 4-byte aligned (L_max is any
// number), which the hardware's vector loads accept.
struct __attribute__((packed, aligned(4))) Tok4 { int32_t t[4]; };

// Thread tid's group u of a chunk starts at token (u * RT_THREADS + tid) * 4 of the chunk: one
// 16-byte load per lane, consecutive lanes consecutive addresses; a group past the end of the row
// is read token by token.
__device__ __forceinline__ Tok4 load_group(const int32_t* __restrict__ x, int32_t i0, int32_t L_max) {
    Tok4 r;
    if (i0 + 3 < L_max) {
        r = *reinterpret_cast<const Tok4*>(x + i0);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) r.t[j] = (i0 + j) < L_max ? x[i0 + j] : 0;
    }
    return r;
}
constexpr int RT_AHEAD = 2;                           // chunks the loads run ahead of the scan
constexpr int RT_LIST = 128;                          // keys the ranking list holds before the tournament takes over
constexpr int RT_WALK = 8;                            // tokens compared per round of the backward match

__global__ __launch_bounds__(RT_THREADS) void retrieve_kernel(
    const int32_t* __restrict__ ctx, const int32_t* __restrict__ ctx_len, int32_t L_max,
    const int32_t* __restrict__ tail, const int32_t* __restrict__ tail_len, int32_t tail_max,
    int32_t n_min, int32_t n_max, int32_t C, int32_t m,
    int32_t* __restrict__ chain_tok, int32_t* __restrict__ chain_len, int32_t* __restrict__ chain_pos,
    int32_t* __restrict__ chain_match, int32_t* __restrict__ n_hits, int32_t* __restrict__ status) {
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    __shared__ __attribute__((aligned(16))) int32_t buf[2][RT_CHUNK];   // two context chunks
    __shared__ int32_t q_rev[GRAFT_MAX_NGRAM + RT_WALK];   // q_rev[j] = j-th token from the end of the query (the
                                                           // backward match reads up to RT_WALK entries past n_max - 1 and ignores them)
    __shared__ u64 red[RT_WAVES * GRAFT_MAX_CHAINS];   // per-wavefront best keys
    __shared__ u64 win[GRAFT_MAX_CHAINS];              // the C winners
    __shared__ u64 list[RT_LIST];                      // best keys of the threads that have hits
    __shared__ u64 counts;                             // low word: keys appended to the list, high word: hits
    __shared__ int32_t tail_s[RT_THREADS];             // the first RT_THREADS tail tokens

    // the lengths first, the first chunks right behind them: they do not wait for the length, every
    // index below L_max is readable
    const int32_t L = ctx_len[b];
    const int32_t T = (tail != nullptr && tail_len != nullptr) ? tail_len[b] : 0;
    const int32_t* x = ctx + static_cast<size_t>(b) * L_max;
    Tok4 v[RT_AHEAD][RT_GROUPS];
#pragma unroll
    for (int k = 0; k < RT_AHEAD; ++k)
#pragma unroll
        for (int u = 0; u < RT_GROUPS; ++u) v[k][u] = load_group(x, k * RT_CHUNK + (u * RT_THREADS + tid) * 4, L_max);
    const int32_t tail_tok = (tail != nullptr && tid < tail_max) ? tail[static_cast<size_t>(b) * tail_max + tid] : 0;
    if (tid == 0) counts = 0;
    if (tid < GRAFT_MAX_CHAINS) win[tid] = 0;

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
    // Both chunks in flight go to LDS at once (the two buffers are a ring: the token at position p
    // sits at flat index p mod 2 RT_CHUNK), and so do the tail tokens; the query is then read from
    // there: no second trip to memory unless it lies beyond the first two chunks.
    int32_t* ring = &buf[0][0];
#pragma unroll
    for (int k = 0; k < RT_AHEAD; ++k)
#pragma unroll
        for (int u = 0; u < RT_GROUPS; ++u)
            if (k * RT_CHUNK + u * RT_THREADS * 4 < L_max)       // uniform: nothing past the row's end is ever read
                *reinterpret_cast<int4*>(ring + k * RT_CHUNK + (u * RT_THREADS + tid) * 4) =
                    int4{v[k][u].t[0], v[k][u].t[1], v[k][u].t[2], v[k][u].t[3]};
    tail_s[tid] = tail_tok;
    __syncthreads();
    const int32_t QL = L + T;
    const int32_t nq = n_max < QL ? n_max : QL;
    if (tid < nq) {
        const int32_t qi = QL - 1 - tid;
        int32_t q;
        if (qi < L) q = qi < RT_AHEAD * RT_CHUNK ? ring[qi] : x[qi];
        else q = (qi - L) < RT_THREADS ? tail_s[qi - L] : tail[static_cast<size_t>(b) * tail_max + (qi - L)];
        q_rev[tid] = q;
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
            if (c >= RT_AHEAD) {                  // (the first RT_AHEAD chunks are in LDS already)
                int32_t* cur = buf[c & 1];
#pragma unroll
                for (int u = 0; u < RT_GROUPS; ++u)
                    *reinterpret_cast<int4*>(cur + (u * RT_THREADS + tid) * 4) =
                        int4{v[k][u].t[0], v[k][u].t[1], v[k][u].t[2], v[k][u].t[3]};
                __syncthreads();                  // chunk c visible; chunk c - 1 still in the other buffer
            } else if (c == 0) {
                __syncthreads();                  // q_rev visible
            }
            const int32_t q_last = nq > 0 ? q_rev[0] : 0;
            // When a hit needs at least two matching tokens, the token before position i is
            // tested as well before the (divergent) walk: with frequent tokens at the end of
            // the query almost every wavefront would otherwise enter every walk.  Inside a
            // group that token is in a register; the one before the group comes from LDS.
            const bool two = n_min >= 2;
            const int32_t q_prev = nq > 1 ? q_rev[1] : 0;
            unsigned cand = 0;                    // bit 4 u + j: token j of group u is a candidate
#pragma unroll
            for (int u = 0; u < RT_GROUPS; ++u) {
                const int32_t i0 = c * RT_CHUNK + (u * RT_THREADS + tid) * 4;
                if (c * RT_CHUNK + u * RT_THREADS * 4 > last_i) continue;        // uniform: the whole group row is past the end
                // in text the query's last token is rare: one compare per token, and a wavefront in
                // which no lane has it skips the rest
                const bool any = (v[k][u].t[0] == q_last) | (v[k][u].t[1] == q_last) | (v[k][u].t[2] == q_last) |
                                 (v[k][u].t[3] == q_last);
                if (__builtin_amdgcn_ballot_w64(any) == 0) continue;
                const int32_t ip = i0 - 1;
                int32_t prev = ip >= 0 ? buf[(ip / RT_CHUNK) & 1][ip % RT_CHUNK] : ~q_prev;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int32_t t = v[k][u].t[j];
                    if (i0 + j <= last_i && t == q_last && (!two || (i0 + j >= 1 && prev == q_prev))) cand |= 1u << (4 * u + j);
                    prev = t;
                }
            }
            // one candidate per lane and pass (usually a single pass): the walk and the insertion
            // below exist once in the code and run once per pass, whatever slot the candidate is in
            while (cand != 0) {
                const int bit = __builtin_ctz(cand);
                cand &= cand - 1;
                const int32_t i = c * RT_CHUNK + ((bit >> 2) * RT_THREADS + tid) * 4 + (bit & 3);
                {
                    const int32_t e = i + 1;
                    const int32_t cap = n_max < e ? n_max : e;
                    // token e - 1 matches q_rev[0]; tokens e - 1 - j, j = 1 .. cap - 1, are compared RT_WALK at
                    // a time (independent LDS reads; they lie at most n_max - 1 before i: this chunk or the one before)
                    int32_t l = 1;
                    for (int32_t base = 1; base < cap; base += RT_WALK) {
                        unsigned eq = 0;                 // bit jj: token e - 1 - (base + jj) continues the match
#pragma unroll
                        for (int jj = 0; jj < RT_WALK; ++jj) {
                            // (positions before the buffer's start wrap to some other token of the ring: masked below)
                            const unsigned pos = static_cast<unsigned>(e - 1 - base - jj) & (2u * RT_CHUNK - 1u);
                            eq |= (ring[pos] == q_rev[base + jj] && base + jj < cap) ? 1u << jj : 0u;
                        }
                        const int run = __builtin_ctz(~eq);          // matching tokens at the front of this round (<= RT_WALK)
                        l += run;
                        if (run < RT_WALK) break;
                    }
                    if (l >= n_min) {
                        ++my_hits;
                        u64 key = (static_cast<u64>(l) << 32) | static_cast<u64>(e);
                        // (only the best C of a thread can be among the best C overall)
#pragma unroll
                        for (int kk = 0; kk < GRAFT_MAX_CHAINS; ++kk) {
                            if (kk >= C) break;          // uniform
                            if (key > top[kk]) { u64 t = top[kk]; top[kk] = key; key = t; }
                        }
                    }
                }
            }
            if (c + RT_AHEAD < n_chunks) {        // this slot's registers are free: fetch RT_AHEAD chunks ahead
#pragma unroll
                for (int u = 0; u < RT_GROUPS; ++u)
                    v[k][u] = load_group(x, (c + RT_AHEAD) * RT_CHUNK + (u * RT_THREADS + tid) * 4, L_max);
            }
            if (c + 1 >= RT_AHEAD && c + 1 < n_chunks)
                __syncthreads();                  // all walks done before chunk c + 1 overwrites chunk c - 1
        }
    }

    // ---- ranking.  Threads with hits append their best C keys (top[] is sorted, so its first
    //      min(my_hits, C) entries) to the list; the append order does not matter, a key's rank
    //      is the number of larger keys.
    if (my_hits > 0) {
        const int32_t k = my_hits < C ? my_hits : C;
        const u64 before = atomicAdd(&counts, (static_cast<u64>(my_hits) << 32) | static_cast<u64>(k));
        const int32_t off = static_cast<int32_t>(before & 0xffffffffu);
#pragma unroll
        for (int j = 0; j < GRAFT_MAX_CHAINS; ++j)
            if (j < k && off + j < RT_LIST) list[off + j] = top[j];
    }
    __syncthreads();                              // (also orders the zeroing of win[] when no chunk was scanned)
    const u64 counted = counts;
    const int32_t n_list = static_cast<int32_t>(counted & 0xffffffffu);
    if (n_list <= RT_LIST) {                      // uniform over the workgroup
        if (tid < n_list) {
            const u64 key = list[tid];
            int32_t rank = 0;
            for (int32_t i0 = 0; i0 < n_list; i0 += 8) {          // eight independent reads per round
#pragma unroll
                for (int u = 0; u < 8; ++u) rank += (i0 + u < n_list && list[(i0 + u) & (RT_LIST - 1)] > key) ? 1 : 0;
            }
            if (rank < C) win[rank] = key;
        }
    } else {
        // the list overflowed: every wavefront extracts its own best C keys (keys are unique because
        // e is, so exactly one lane owns each maximum and pops it), then wavefront 0 merges the
        // 16 x C survivors.  No memory access between the rounds.
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
        }
    }
    if (tid == 0) {
        n_hits[b] = static_cast<int32_t>(counted >> 32);
        status[b] = 0;
    }
    __syncthreads();
    // ---- outputs: chain c starts at e = low word of win[c]; the last two chunks scanned are still in LDS
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
        if (key != 0 && e + jj < L) {
            const int32_t pos = e + jj, ch = pos / RT_CHUNK;
            tok_b[i] = (ch < n_chunks && ch + 2 >= n_chunks) ? buf[ch & 1][pos % RT_CHUNK] : x[pos];
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
