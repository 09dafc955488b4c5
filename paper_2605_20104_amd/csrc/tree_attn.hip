// graft_tree_attn: tree-masked GQA attention over a paged KV cache.
//
// Two code paths.
//
// (1) bf16, D = 128: split-KV MFMA kernel + log-sum-exp combine.
//     All R = K_max * (Hq/Hkv) query rows of one KV head share every K/V element
//     that is streamed, so K and V are read from HBM once per head; the
//     arithmetic intensity is R flop per byte, which puts the tree-verify shapes
//     (R = 160..768) around the MFMA/HBM ridge of the chip.
//       grid  = (splits * row_tiles, Hkv, B), 512 threads = 8 wavefronts,
//               one workgroup per CU, two wavefronts per SIMD (<= 256 VGPRs each)
//               so that one wavefront's softmax VALU work overlaps the other's MFMAs.
//       rows  : a wavefront owns 16*MB query rows (MB <= 3 MFMA row blocks);
//               wavefronts 0..3 take MBA blocks and 4..7 take MBB <= MBA, so that
//               e.g. 320 rows = 16 * 4 * (3 + 2) load the four SIMDs evenly.  Q stays
//               in registers for the whole kernel, O accumulates in registers as
//               O^T tiles.
//       K/V   : 64-token stages (4 pages) go global -> LDS directly (no register
//               staging), double buffered, one barrier per stage; K rows are
//               XOR-swizzled at 16 B and V rows at 32 B so that the MFMA operand
//               reads spread over all banks.
//       QK^T  : S^T = K * Q^T with v_mfma_f32_16x16x32_bf16, so each lane holds
//               scores of ONE query row (column l%16): the row max needs only two
//               cross-lane steps and the probabilities are already laid out as
//               the B operand of the second product (no LDS round trip).
//       PV    : O^T = V^T * P^T; the V^T operand (contraction over tokens, which
//               are strided in memory) comes from the gfx950 LDS transpose read
//               ds_read_b64_tr_b16: a 16-lane group turns a 4-token x 16-dim
//               block into "lane = dim, 4 tokens packed".
//       mask  : only sub-tiles that reach past the prefix take the masked path
//               (ancestor bits from graft_build_tree_mask); the prefix is dense.
//       softmax: running max with a lazy threshold (the accumulators are only
//               rescaled when the row max grows by more than 2^8), exp2 with the
//               scale folded into one FMA.
//     Partials (unnormalised O, max, sum) go to the workspace; a small combine
//     kernel merges the splits and writes bf16.
//
// (2) everything else (fp32 storage, or D = 64): a plain one-workgroup-per-
//     (node, head) kernel in fp32.  It serves the tiny fp32 configuration and as
//     an independent GPU cross-check of path (1).
#include "common.h"

namespace graft {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int AT_THREADS = 512;
constexpr int AT_WAVES = 8;
constexpr int AT_STAGE = 64;        // tokens per LDS stage (4 pages)
constexpr int AT_SUB = 32;          // tokens per softmax step
constexpr int AT_D = 128;
constexpr int AT_ROW_BYTES = AT_D * 2;
constexpr int AT_MAX_BLOCKS = 24;      // 16-row blocks per workgroup: 4 * (3 + 3)
constexpr int AT_MAX_SPLITS = 64;
constexpr float AT_LAZY_LOG2 = 8.0f;   // rescale only when the max grows by more than 2^8

struct AttnParams {
    const void* q;
    const void* k;
    const void* v;
    void* out;
    const int32_t* block_table;
    const int32_t* prefix_len;
    const int32_t* n_nodes;
    const u64* mask;
    float* ws_o;        // [B][Hkv][splits][R_pad][D]
    float* ws_ml;       // [B][Hkv][splits][R_pad][2]  (max in log2 units, sum)
    int64_t page_stride, token_stride, head_stride;
    int32_t max_pages, B, K_max, Hq, Hkv, G, R, R_pad, n_splits, n_row_tiles;
    float scale;        // softmax scale
    float scale_log2e;  // scale * log2(e)
};

__device__ __forceinline__ float bf16_bits_to_float(unsigned short b) {
    return __uint_as_float(static_cast<unsigned>(b) << 16);
}
__device__ __forceinline__ unsigned short float_to_bf16_bits(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);           // round to nearest even (finite inputs)
    return static_cast<unsigned short>(u >> 16);
}

// ---------------------------------------------------------------------------
// path (1): MFMA split-KV kernel
// ---------------------------------------------------------------------------
// One 32-token sub-tile for the MB row blocks of this wavefront.
template <int MB>
__device__ __forceinline__ void attn_subtile(
    const unsigned char* __restrict__ Ks, const unsigned char* __restrict__ Vs,
    const bf16x8 (&qreg)[MB][4], floatx4 (&o)[MB][8], float (&m_run)[MB], float (&l_run)[MB],
    float c_log2, float lazy_raw, int lane,
    bool masked, int t_sub0, int P, int n, int r_base, int R, int G, const unsigned* __restrict__ Ms) {
    const int l16 = lane & 15, lg = lane >> 4;

    // ---- S^T = K Q^T : s[rb][c][i] = score of row (rb, l16) and token 16c + 4lg + i
    floatx4 s[MB][2];
#pragma unroll
    for (int rb = 0; rb < MB; ++rb) {
        s[rb][0] = floatx4{0.f, 0.f, 0.f, 0.f};
        s[rb][1] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int row = 16 * c + l16;
#pragma unroll
        for (int ds = 0; ds < 4; ++ds) {
            const int chunk = (4 * ds + lg) ^ l16;
            const bf16x8 ka = *reinterpret_cast<const bf16x8*>(Ks + row * AT_ROW_BYTES + chunk * 16);
#pragma unroll
            for (int rb = 0; rb < MB; ++rb)
                s[rb][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qreg[rb][ds], s[rb][c], 0, 0, 0);
        }
    }

    // ---- online softmax per row block
    bf16x8 pb[MB];
#pragma unroll
    for (int rb = 0; rb < MB; ++rb) {
        if (masked) {                                     // wavefront-uniform; branch-free inside
            const int r = r_base + rb * 16 + l16;
            const int node = r / G;
            const bool live = r < R && node < n;
            const int nd = live ? node : 0;
            const unsigned w0 = live ? Ms[4 * nd + 0] : 0u, w1 = live ? Ms[4 * nd + 1] : 0u;
            const unsigned w2 = live ? Ms[4 * nd + 2] : 0u, w3 = live ? Ms[4 * nd + 3] : 0u;
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int j0 = t_sub0 + 16 * c + 4 * lg - P;          // tree slot of element i = 0
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int j = j0 + i;
                    const int wi = (j >> 5) & 3;
                    const unsigned word = wi == 0 ? w0 : (wi == 1 ? w1 : (wi == 2 ? w2 : w3));
                    const bool bit = (word >> (j & 31)) & 1u;
                    const bool valid = (j < 0) | ((j < n) & bit);
                    s[rb][c][i] = valid ? s[rb][c][i] : -INFINITY;
                }
            }
        }
        float mx = fmaxf(fmaxf(fmaxf(s[rb][0][0], s[rb][0][1]), fmaxf(s[rb][0][2], s[rb][0][3])),
                         fmaxf(fmaxf(s[rb][1][0], s[rb][1][1]), fmaxf(s[rb][1][2], s[rb][1][3])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        // lazy running max: all four lane groups of a row see the same mx and m_run
        const bool grow = mx > m_run[rb] + lazy_raw;      // also true on the first finite tile
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {      // wavefront-uniform branch
            const float m_new = grow ? mx : m_run[rb];
            float a = grow ? __builtin_amdgcn_exp2f((m_run[rb] - m_new) * c_log2) : 1.0f;
            if (m_run[rb] == -INFINITY) a = 0.0f;
            l_run[rb] *= a;
#pragma unroll
            for (int db = 0; db < 8; ++db) o[rb][db] *= a;
            m_run[rb] = m_new;
        }
        const float mref = (m_run[rb] == -INFINITY) ? 0.0f : m_run[rb];
        const float neg = -mref * c_log2;
        float lsum = 0.f;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[rb][c][i], c_log2, neg));
                lsum += e;
                pb[rb][4 * c + i] = static_cast<__bf16>(e);
            }
        l_run[rb] += lsum;
    }

    // ---- O^T += V^T P^T ; V^T operand through the LDS transpose read
#pragma unroll
    for (int db = 0; db < 8; ++db) {
        bf16x8 va;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int row = 16 * c + 4 * lg + (l16 >> 2);
            const int seg = db ^ (row & 7);
            const unsigned char* ptr = Vs + row * AT_ROW_BYTES + seg * 32 + 8 * (l16 & 3);
            const short4_t r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (short4_t __attribute__((address_space(3)))*)(ptr));
            const bf16x4 rb4 = __builtin_bit_cast(bf16x4, r);
            va[4 * c + 0] = rb4[0];
            va[4 * c + 1] = rb4[1];
            va[4 * c + 2] = rb4[2];
            va[4 * c + 3] = rb4[3];
        }
#pragma unroll
        for (int rb = 0; rb < MB; ++rb)
            o[rb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb[rb], o[rb][db], 0, 0, 0);
    }
}

struct SplitRange { int st0, st1, P, n, total; };

constexpr int AT_MAX_SPLIT_PAGES = 4096;          // block-table entries of one split kept in LDS
constexpr int AT_NBUF = 4;                         // LDS stage buffers: 3 stages in flight + 1 in use
constexpr int AT_STAGE_BYTES = 2 * AT_STAGE * AT_ROW_BYTES;   // K rows then V rows
constexpr int AT_LOADS_PER_STAGE = 4;              // global->LDS instructions per wavefront per stage

// Global -> LDS without passing through registers: each lane's 16 bytes land at
// (wavefront-uniform LDS base) + lane * 16, so the swizzled LDS layout is produced by
// choosing which global chunk each lane fetches.  One wavefront moves 4 token rows
// (1 KB) of K or of V per instruction; 8 wavefronts x 2 x (K,V) = one 64-token stage.
// The block-table entries of the split were copied to LDS (Tb) up front, so the lookup is
// an LDS read and nothing but the transfers themselves occupies the vector memory counter.
//
// The transfer is issued through inline assembly on purpose: the kernel keeps several stages
// in flight and waits for them with explicit s_waitcnt vmcnt(N); transfers the compiler knows
// about make it drain the whole vector memory counter before every LDS read and barrier.
__device__ __forceinline__ void load_global_to_lds_b128(const void* gptr, unsigned lds_addr) {
    // LDS address of lane l = M0 + 16 * l (M0 write needs one wait state before its use).
    // M0 is a reserved register the compiler sets up itself right before each of its own uses.
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_addr), "v"(gptr)
                 : "memory");
}

__device__ __forceinline__ unsigned lds_address(const void* p) {
    return static_cast<unsigned>(reinterpret_cast<size_t>(
        (const __attribute__((address_space(3))) unsigned char*)(p)));
}

__device__ __forceinline__ void stage_loads(const AttnParams& p, const SplitRange& sr, int st, int wave_u,
                                            int lane, const int32_t* __restrict__ Tb, int g,
                                            unsigned char* buf) {
    const int l16 = lane & 15;
    const unsigned lds_base = __builtin_amdgcn_readfirstlane(lds_address(buf));
    const int last = sr.total - 1;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int slot = 2 * wave_u + j;                         // 1 KB slot = 4 token rows
        const int row = 4 * slot + (lane >> 4);                  // token row within the stage
        const int pg = (st - sr.st0) * (AT_STAGE / GRAFT_PAGE_SIZE) + (slot >> 2);   // uniform, split-local
        int t = st * AT_STAGE + row;
        t = t < last ? t : last;                                 // rows past the end re-read the last token
        const int64_t off = static_cast<int64_t>(Tb[pg]) * p.page_stride +
                            static_cast<int64_t>(t & 15) * p.token_stride +
                            static_cast<int64_t>(g) * p.head_stride;
        const int kchunk = l16 ^ (row & 15);
        const int vchunk = (((l16 >> 1) ^ (row & 7)) << 1) | (l16 & 1);
        const __bf16* ksrc = static_cast<const __bf16*>(p.k) + off + kchunk * 8;
        const __bf16* vsrc = static_cast<const __bf16*>(p.v) + off + vchunk * 8;
        const unsigned lds = lds_base + slot * 1024;
        load_global_to_lds_b128(ksrc, lds);
        load_global_to_lds_b128(vsrc, lds + AT_STAGE * AT_ROW_BYTES);
    }
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also drain the
// vector memory counter and with it the global->LDS transfers of the stages still in flight.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// s_waitcnt vmcnt(N) only (expcnt / lgkmcnt fields left at "no wait")
#define GRAFT_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(0x0F70 | ((N) & 15) | (((N) >> 4) << 14))

template <int MB>
__device__ __forceinline__ void attn_wave_main(const AttnParams& p, const SplitRange& sr, int r_base,
                                               int split, int g, int b, unsigned char* kv0, unsigned char* kv1,
                                               unsigned char* kv2, unsigned char* kv3,
                                               const unsigned* __restrict__ Ms, const int32_t* __restrict__ Tb) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_u = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lg = lane >> 4;
    constexpr int MBX = MB > 0 ? MB : 1;

    unsigned char* const bufs[AT_NBUF] = {kv0, kv1, kv2, kv3};
    const int n_st = sr.st1 - sr.st0;
    // pipeline prologue: the first three stages start streaming before anything else
#pragma unroll
    for (int k = 0; k < AT_NBUF - 1; ++k)
        if (k < n_st) stage_loads(p, sr, sr.st0 + k, wave_u, lane, Tb, g, bufs[k]);

    // ---- Q rows of this wavefront stay in registers (B operand of S^T = K Q^T)
    bf16x8 qreg[MBX][4];
    floatx4 o[MBX][8];
    float m_run[MBX], l_run[MBX];
#pragma unroll
    for (int rb = 0; rb < MB; ++rb) {
        const int r = r_base + rb * 16 + l16;
        if (r < p.R) {
            const int i = r / p.G, hl = r - i * p.G;
            const __bf16* qp = static_cast<const __bf16*>(p.q) +
                ((static_cast<size_t>(b) * p.K_max + i) * p.Hq + (g * p.G + hl)) * AT_D + lg * 8;
#pragma unroll
            for (int ds = 0; ds < 4; ++ds) qreg[rb][ds] = *reinterpret_cast<const bf16x8*>(qp + 32 * ds);
        } else {
#pragma unroll
            for (int ds = 0; ds < 4; ++ds)
#pragma unroll
                for (int t = 0; t < 8; ++t) qreg[rb][ds][t] = static_cast<__bf16>(0.0f);
        }
        m_run[rb] = -INFINITY;
        l_run[rb] = 0.f;
#pragma unroll
        for (int db = 0; db < 8; ++db) o[rb][db] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // Q must have landed before the loop: a pending compiler-tracked load would make every
    // iteration drain the vector memory counter (and the stages in flight with it).
    GRAFT_WAIT_VMCNT(0);
    const float c_log2 = p.scale_log2e;
    const float lazy_raw = AT_LAZY_LOG2 / c_log2;

    // ---- software pipeline over 64-token stages: stage k lives in buffer k % 4, loads run
    //      three stages ahead; before a stage is used every wavefront waits for its own
    //      loads of that stage (the younger stages' loads stay in flight) and meets the
    //      others at one barrier, which also frees the buffer consumed one stage earlier.
    for (int base = 0; base < n_st; base += AT_NBUF) {
#pragma unroll
        for (int i = 0; i < AT_NBUF; ++i) {
            const int idx = base + i;
            if (idx >= n_st) break;
            const int younger = n_st - 1 - idx;                  // stages already issued after this one
            if (younger >= 2) GRAFT_WAIT_VMCNT(2 * AT_LOADS_PER_STAGE);
            else if (younger == 1) GRAFT_WAIT_VMCNT(AT_LOADS_PER_STAGE);
            else GRAFT_WAIT_VMCNT(0);
            lds_barrier();
            if (idx + AT_NBUF - 1 < n_st)
                stage_loads(p, sr, sr.st0 + idx + AT_NBUF - 1, wave_u, lane, Tb, g,
                            bufs[(i + AT_NBUF - 1) % AT_NBUF]);
            if (MB > 0) {
                const int st = sr.st0 + idx;
#pragma unroll 1
                for (int sub = 0; sub < 2; ++sub) {
                    const int t_sub0 = st * AT_STAGE + sub * AT_SUB;
                    if (t_sub0 < sr.total)
                        attn_subtile<MBX>(bufs[i] + sub * AT_SUB * AT_ROW_BYTES,
                                          bufs[i] + AT_STAGE * AT_ROW_BYTES + sub * AT_SUB * AT_ROW_BYTES, qreg, o,
                                          m_run, l_run, c_log2, lazy_raw, lane, t_sub0 + AT_SUB > sr.P, t_sub0,
                                          sr.P, sr.n, r_base, p.R, p.G, Ms);
                }
            }
        }
    }

    // ---- partial results: unnormalised O, running max (log2 units), running sum
    const size_t part = ((static_cast<size_t>(b) * p.Hkv + g) * p.n_splits + split) * p.R_pad;
#pragma unroll
    for (int rb = 0; rb < MB; ++rb) {
        const int r = r_base + rb * 16 + l16;
        float l = l_run[rb];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        float* op = p.ws_o + (part + r) * AT_D + 4 * lg;
#pragma unroll
        for (int db = 0; db < 8; ++db)       // o[rb][db][i] = O[r][16 db + 4 lg + i]
            *reinterpret_cast<floatx4*>(op + 16 * db) = o[rb][db];
        if (lg == 0) {
            float* ml = p.ws_ml + (part + r) * 2;
            ml[0] = m_run[rb] == -INFINITY ? -INFINITY : m_run[rb] * c_log2;
            ml[1] = l;
        }
    }
}

// Wavefronts 0..3 own MBA row blocks each, wavefronts 4..7 own MBB (<= MBA): with the
// usual round-robin placement every SIMD hosts one wavefront of each kind, so a row
// count like 320 = 16 * (4*3 + 4*2) is balanced over the four SIMDs.
template <int MBA, int MBB>
__global__ __launch_bounds__(AT_THREADS) void tree_attn_mfma_kernel(AttnParams p) {
    // Four separate arrays on purpose: the compiler tracks pending global->LDS transfers per
    // LDS variable, so reads of one stage buffer do not wait for transfers into the others.
    __shared__ __attribute__((aligned(1024))) unsigned char kv0[AT_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char kv1[AT_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char kv2[AT_STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char kv3[AT_STAGE_BYTES];
    __shared__ unsigned Ms[GRAFT_MAX_NODES * GRAFT_MASK_WORDS * 2];   // ancestor masks as 32-bit words
    __shared__ int32_t Tb[AT_MAX_SPLIT_PAGES];                         // this split's block-table entries

    const int tid = threadIdx.x, wave = tid >> 6;
    const int split = blockIdx.x % p.n_splits, rt = blockIdx.x / p.n_splits;
    const int g = blockIdx.y, b = blockIdx.z;

    SplitRange sr;
    int n = p.n_nodes[b];
    if (n < 1 || n > p.K_max) n = 0;
    const int cap = p.max_pages * GRAFT_PAGE_SIZE;
    int P = p.prefix_len[b];
    P = P < 0 ? 0 : (P > cap ? cap : P);
    sr.n = n;
    sr.P = P;
    sr.total = n ? ((P + n) < cap ? (P + n) : cap) : 0;
    const int n_stages = (sr.total + AT_STAGE - 1) / AT_STAGE;
    const int spt = (n_stages + p.n_splits - 1) / p.n_splits;
    sr.st0 = split * spt;
    sr.st1 = (sr.st0 + spt) < n_stages ? (sr.st0 + spt) : n_stages;
    if (sr.st1 < sr.st0) sr.st1 = sr.st0;

    if (tid < p.K_max * GRAFT_MASK_WORDS * 2)
        Ms[tid] = reinterpret_cast<const unsigned*>(p.mask)[static_cast<size_t>(b) * p.K_max * GRAFT_MASK_WORDS * 2 + tid];
    {
        const int32_t* table = p.block_table + static_cast<size_t>(b) * p.max_pages;
        const int first_pg = sr.st0 * (AT_STAGE / GRAFT_PAGE_SIZE);
        const int n_pg = (sr.st1 - sr.st0) * (AT_STAGE / GRAFT_PAGE_SIZE);
        const int last_pg = (sr.total - 1) >> 4;
        for (int k = tid; k < n_pg; k += AT_THREADS) {
            const int pg = first_pg + k;
            Tb[k] = table[pg < last_pg ? pg : last_pg];
        }
    }
    __syncthreads();

    const int tile_base = rt * (AT_WAVES / 2) * 16 * (MBA + MBB);
    if (wave < AT_WAVES / 2) {
        attn_wave_main<MBA>(p, sr, tile_base + wave * 16 * MBA, split, g, b, kv0, kv1, kv2, kv3, Ms, Tb);
    } else {
        attn_wave_main<MBB>(p, sr, tile_base + (AT_WAVES / 2) * 16 * MBA + (wave - AT_WAVES / 2) * 16 * MBB,
                            split, g, b, kv0, kv1, kv2, kv3, Ms, Tb);
    }
}

// Merge the splits of one output row: out = sum_s w_s O_s / sum_s w_s l_s, w_s = 2^(m_s - max m).
__global__ __launch_bounds__(AT_THREADS) void tree_attn_combine_kernel(AttnParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t row = static_cast<int64_t>(blockIdx.x) * AT_WAVES + wave;   // over B*K_max*Hq
    const int64_t n_rows = static_cast<int64_t>(p.B) * p.K_max * p.Hq;
    if (row >= n_rows) return;
    const int h = static_cast<int>(row % p.Hq);
    const int i = static_cast<int>((row / p.Hq) % p.K_max);
    const int b = static_cast<int>(row / (static_cast<int64_t>(p.Hq) * p.K_max));
    unsigned short* outp = static_cast<unsigned short*>(p.out) + row * AT_D + 2 * lane;
    int n = p.n_nodes[b];
    if (n < 1 || n > p.K_max) n = 0;
    if (i >= n) {
        *reinterpret_cast<unsigned*>(outp) = 0u;
        return;
    }
    const int g = h / p.G, r = i * p.G + (h - g * p.G);
    const size_t base = (static_cast<size_t>(b) * p.Hkv + g) * p.n_splits * p.R_pad + r;
    float mmax = -INFINITY;
    for (int s = 0; s < p.n_splits; ++s)
        mmax = fmaxf(mmax, p.ws_ml[(base + static_cast<size_t>(s) * p.R_pad) * 2]);
    float acc0 = 0.f, acc1 = 0.f, den = 0.f;
    for (int s = 0; s < p.n_splits; ++s) {
        const size_t idx = base + static_cast<size_t>(s) * p.R_pad;
        const float m = p.ws_ml[idx * 2], l = p.ws_ml[idx * 2 + 1];
        if (m == -INFINITY) continue;                       // wavefront-uniform
        const float w = __builtin_amdgcn_exp2f(m - mmax);
        const float2 ov = *reinterpret_cast<const float2*>(p.ws_o + idx * AT_D + 2 * lane);
        acc0 += w * ov.x;
        acc1 += w * ov.y;
        den += w * l;
    }
    const float inv = den > 0.f ? 1.0f / den : 0.f;
    const unsigned lo = float_to_bf16_bits(acc0 * inv), hi = float_to_bf16_bits(acc1 * inv);
    *reinterpret_cast<unsigned*>(outp) = lo | (hi << 16);
}

// ---------------------------------------------------------------------------
// path (2): plain fp32 kernel, one workgroup per (head, node, sequence)
// ---------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ float load_as_float(const T* p, int64_t i);
template <> __device__ __forceinline__ float load_as_float<float>(const float* p, int64_t i) { return p[i]; }
template <> __device__ __forceinline__ float load_as_float<unsigned short>(const unsigned short* p, int64_t i) {
    return bf16_bits_to_float(p[i]);
}
template <typename T> __device__ __forceinline__ void store_from_float(T* p, int64_t i, float v);
template <> __device__ __forceinline__ void store_from_float<float>(float* p, int64_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void store_from_float<unsigned short>(unsigned short* p, int64_t i, float v) {
    p[i] = float_to_bf16_bits(v);
}

__device__ __forceinline__ float block_max_256(float v, float* red) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v = fmaxf(v, __shfl_xor(v, s));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
__device__ __forceinline__ float block_sum_256(float v, float* red) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

constexpr int SM_THREADS = 256;

template <typename T, int D>
__global__ __launch_bounds__(SM_THREADS) void tree_attn_simple_kernel(AttnParams p) {
    const int h = blockIdx.x, i = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x;
    __shared__ float qs[D];
    __shared__ float ps[SM_THREADS];
    __shared__ float accs[SM_THREADS];
    __shared__ float red[SM_THREADS / 64];
    const int64_t row = (static_cast<int64_t>(b) * p.K_max + i) * p.Hq + h;
    T* outp = static_cast<T*>(p.out) + row * D;
    int n = p.n_nodes[b];
    if (n < 1 || n > p.K_max) n = 0;
    if (i >= n) {
        if (tid < D) store_from_float<T>(outp, tid, 0.f);
        return;
    }
    const int cap = p.max_pages * GRAFT_PAGE_SIZE;
    int P = p.prefix_len[b];
    P = P < 0 ? 0 : (P > cap ? cap : P);
    const int total = (P + n) < cap ? (P + n) : cap;
    const int g = h / p.G;
    const T* qp = static_cast<const T*>(p.q) + row * D;
    const T* kc = static_cast<const T*>(p.k);
    const T* vc = static_cast<const T*>(p.v);
    const int32_t* table = p.block_table + static_cast<size_t>(b) * p.max_pages;
    const u64* mp = p.mask + (static_cast<size_t>(b) * p.K_max + i) * GRAFT_MASK_WORDS;
    const u64 mk0 = mp[0], mk1 = mp[1];
    if (tid < D) qs[tid] = load_as_float<T>(qp, tid);
    __syncthreads();

    constexpr int PARTS = SM_THREADS / D;
    const int d = tid % D, part = tid / D;
    float acc = 0.f, m_run = -INFINITY, l_run = 0.f;
    for (int t0 = 0; t0 < total; t0 += SM_THREADS) {
        const int t = t0 + tid;
        bool valid = t < P;
        if (!valid && t < total) {
            const int j = t - P;
            valid = ((j < 64 ? mk0 : mk1) >> (j & 63)) & 1ull;
        }
        float s = -INFINITY;
        if (valid) {
            const int64_t base = static_cast<int64_t>(table[t / GRAFT_PAGE_SIZE]) * p.page_stride +
                                 static_cast<int64_t>(t % GRAFT_PAGE_SIZE) * p.token_stride +
                                 static_cast<int64_t>(g) * p.head_stride;
            float dot = 0.f;
#pragma unroll 8
            for (int e = 0; e < D; ++e) dot = __builtin_fmaf(qs[e], load_as_float<T>(kc, base + e), dot);
            s = dot * p.scale;
        }
        const float mt = block_max_256(s, red);
        const float m_new = fmaxf(m_run, mt);
        const float pr = (valid && m_new != -INFINITY) ? __expf(s - m_new) : 0.f;
        const float alpha = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
        ps[tid] = pr;
        const float lsum = block_sum_256(pr, red);        // its barriers also publish ps[]
        acc *= alpha;
        l_run = l_run * alpha + lsum;
        const int lim = (total - t0) < SM_THREADS ? (total - t0) : SM_THREADS;
        for (int tt = part; tt < lim; tt += PARTS) {
            const float pp = ps[tt];
            if (pp != 0.f) {
                const int tk = t0 + tt;
                const int64_t base = static_cast<int64_t>(table[tk / GRAFT_PAGE_SIZE]) * p.page_stride +
                                     static_cast<int64_t>(tk % GRAFT_PAGE_SIZE) * p.token_stride +
                                     static_cast<int64_t>(g) * p.head_stride;
                acc = __builtin_fmaf(pp, load_as_float<T>(vc, base + d), acc);
            }
        }
        m_run = m_new;
        __syncthreads();
    }
    accs[tid] = acc;
    __syncthreads();
    if (tid < D) {
        float sum = 0.f;
#pragma unroll
        for (int k = 0; k < PARTS; ++k) sum += accs[k * D + tid];
        store_from_float<T>(outp, tid, l_run > 0.f ? sum / l_run : 0.f);
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct AttnPlan {
    bool mfma;
    int mba, mbb, n_row_tiles, n_splits, r_pad;
    size_t ws_o_bytes, ws_bytes;
};

static AttnPlan make_plan(int32_t B, int32_t K_max, int32_t Hq, int32_t Hkv, int32_t D, int32_t max_pages,
                          int32_t dtype) {
    AttnPlan pl{};
    pl.mfma = (dtype == GRAFT_BF16 && D == AT_D);
    if (!pl.mfma) return pl;
    const int R = K_max * (Hq / Hkv);
    const int blocks = (R + 15) / 16;                            // 16-row MFMA blocks
    pl.n_row_tiles = (blocks + AT_MAX_BLOCKS - 1) / AT_MAX_BLOCKS;
    const int per_tile = (blocks + pl.n_row_tiles - 1) / pl.n_row_tiles;
    const int per_simd = (per_tile + 3) / 4;                     // blocks per SIMD = MBA + MBB
    pl.mba = (per_simd + 1) / 2;
    pl.mbb = per_simd / 2;
    pl.r_pad = pl.n_row_tiles * 64 * (pl.mba + pl.mbb);
    const int stages = (max_pages * GRAFT_PAGE_SIZE + AT_STAGE - 1) / AT_STAGE;
    const int units = B * Hkv * pl.n_row_tiles;
    int splits = (256 + units - 1) / units;                      // one workgroup per CU
    if (splits > stages) splits = stages;
    if (splits > AT_MAX_SPLITS) splits = AT_MAX_SPLITS;
    if (splits < 1) splits = 1;
    const int min_splits = (stages * (AT_STAGE / GRAFT_PAGE_SIZE) + AT_MAX_SPLIT_PAGES - 1) / AT_MAX_SPLIT_PAGES;
    if (splits < min_splits) splits = min_splits;       // a split's block-table slice must fit in LDS
    pl.n_splits = splits;
    const size_t rows = static_cast<size_t>(B) * Hkv * splits * pl.r_pad;
    pl.ws_o_bytes = rows * AT_D * sizeof(float);
    pl.ws_bytes = pl.ws_o_bytes + rows * 2 * sizeof(float);
    return pl;
}

static bool attn_shape_ok(int32_t B, int32_t K_max, int32_t Hq, int32_t Hkv, int32_t D, int32_t max_pages) {
    return B >= 1 && B <= 65535 && K_max >= 1 && K_max <= GRAFT_MAX_NODES && Hq >= 1 && Hkv >= 1 &&
           Hkv <= 65535 && Hq % Hkv == 0 && Hq / Hkv <= 16 && (D == 64 || D == 128) && max_pages >= 1 &&
           max_pages <= (1 << 26);
}

// Profiling hook state (per host thread): event pairs recorded around the main kernel.
static thread_local hipEvent_t* g_prof_start = nullptr;
static thread_local hipEvent_t* g_prof_stop = nullptr;
static thread_local int32_t g_prof_n = 0, g_prof_i = 0;

static void prof_record(bool start, hipStream_t s) {
    if (g_prof_i < g_prof_n) {
        (void)hipEventRecord(start ? g_prof_start[g_prof_i] : g_prof_stop[g_prof_i], s);
        if (!start) ++g_prof_i;
    }
}

template <int MBA, int MBB>
static void launch_mfma(const AttnParams& p, dim3 grid, hipStream_t s) {
    hipLaunchKernelGGL((tree_attn_mfma_kernel<MBA, MBB>), grid, dim3(AT_THREADS), 0, s, p);
}

}  // namespace graft

extern "C" size_t graft_tree_attn_workspace_bytes(int32_t B, int32_t K_max, int32_t Hq, int32_t Hkv,
                                                  int32_t D, int32_t max_pages, int32_t dtype) {
    if (!graft::attn_shape_ok(B, K_max, Hq, Hkv, D, max_pages)) return 0;
    if (dtype != GRAFT_F32 && dtype != GRAFT_BF16) return 0;
    return graft::make_plan(B, K_max, Hq, Hkv, D, max_pages, dtype).ws_bytes;
}

extern "C" int32_t graft_attn_profile_events(void** start_events, void** stop_events, int32_t n) {
    if (n < 0 || (n > 0 && (!start_events || !stop_events))) return GRAFT_ERR_NULL;
    graft::g_prof_start = reinterpret_cast<hipEvent_t*>(start_events);
    graft::g_prof_stop = reinterpret_cast<hipEvent_t*>(stop_events);
    graft::g_prof_n = n;
    graft::g_prof_i = 0;
    return GRAFT_OK;
}

extern "C" int32_t graft_tree_attn(const void* q, const void* k_cache, const void* v_cache,
                                   int64_t page_stride, int64_t token_stride, int64_t head_stride,
                                   const int32_t* block_table, int32_t max_pages,
                                   const int32_t* prefix_len, const int32_t* n_nodes, const uint64_t* mask,
                                   int32_t B, int32_t K_max, int32_t Hq, int32_t Hkv, int32_t D,
                                   int32_t page_size, float scale, int32_t dtype, void* out,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    using namespace graft;
    if (!q || !k_cache || !v_cache || !block_table || !prefix_len || !n_nodes || !mask || !out)
        return GRAFT_ERR_NULL;
    if (dtype != GRAFT_F32 && dtype != GRAFT_BF16) return GRAFT_ERR_DTYPE;
    if (!attn_shape_ok(B, K_max, Hq, Hkv, D, max_pages) || page_size != GRAFT_PAGE_SIZE ||
        page_stride < 1 || token_stride < D || head_stride < D || token_stride % 8 != 0 ||
        head_stride % 8 != 0 || page_stride % 8 != 0 || !(scale > 0.f) || !(scale < 1e30f))
        return GRAFT_ERR_SHAPE;
    const AttnPlan pl = make_plan(B, K_max, Hq, Hkv, D, max_pages, dtype);
    if (pl.ws_bytes > 0 && (!workspace || workspace_bytes < pl.ws_bytes)) return GRAFT_ERR_WORKSPACE;

    AttnParams p{};
    p.q = q; p.k = k_cache; p.v = v_cache; p.out = out;
    p.block_table = block_table; p.prefix_len = prefix_len; p.n_nodes = n_nodes;
    p.mask = reinterpret_cast<const u64*>(mask);
    p.page_stride = page_stride; p.token_stride = token_stride; p.head_stride = head_stride;
    p.max_pages = max_pages; p.B = B; p.K_max = K_max; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv;
    p.R = K_max * p.G;
    p.scale = scale;
    p.scale_log2e = scale * 1.4426950408889634f;
    hipStream_t s = static_cast<hipStream_t>(stream);

    if (!pl.mfma) {
        dim3 grid(Hq, K_max, B);
        prof_record(true, s);
        if (dtype == GRAFT_F32) {
            if (D == 64) hipLaunchKernelGGL((tree_attn_simple_kernel<float, 64>), grid, dim3(SM_THREADS), 0, s, p);
            else hipLaunchKernelGGL((tree_attn_simple_kernel<float, 128>), grid, dim3(SM_THREADS), 0, s, p);
        } else {
            hipLaunchKernelGGL((tree_attn_simple_kernel<unsigned short, 64>), grid, dim3(SM_THREADS), 0, s, p);
        }
        prof_record(false, s);
        return check_launch();
    }

    p.R_pad = pl.r_pad; p.n_splits = pl.n_splits; p.n_row_tiles = pl.n_row_tiles;
    p.ws_o = static_cast<float*>(workspace);
    p.ws_ml = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + pl.ws_o_bytes);
    dim3 grid(pl.n_splits * pl.n_row_tiles, Hkv, B);
    prof_record(true, s);
    switch (pl.mba * 4 + pl.mbb) {
        case 1 * 4 + 0: launch_mfma<1, 0>(p, grid, s); break;
        case 1 * 4 + 1: launch_mfma<1, 1>(p, grid, s); break;
        case 2 * 4 + 1: launch_mfma<2, 1>(p, grid, s); break;
        case 2 * 4 + 2: launch_mfma<2, 2>(p, grid, s); break;
        case 3 * 4 + 2: launch_mfma<3, 2>(p, grid, s); break;
        default: launch_mfma<3, 3>(p, grid, s); break;
    }
    prof_record(false, s);
    int32_t rc = check_launch();
    if (rc != GRAFT_OK) return rc;
    const int64_t n_rows = static_cast<int64_t>(B) * K_max * Hq;
    hipLaunchKernelGGL(tree_attn_combine_kernel, dim3(static_cast<unsigned>((n_rows + AT_WAVES - 1) / AT_WAVES)),
                       dim3(AT_THREADS), 0, s, p);
    return check_launch();
}
