// graft_tree_attn: tree-masked GQA attention over a paged KV cache.
//
// Two code paths.
//
// (1) bf16, D = 128: split-KV MFMA kernel + log-sum-exp combine.
//     All R = K_max * (Hq/Hkv) query rows of one KV head share every K/V element
//     that is streamed, so K and V are read from HBM once per head; the
//     arithmetic intensity is R flop per byte, which puts the tree-verify shapes
//     (R = 160..768) around the MFMA/HBM ridge of the chip.
//       grid  : one workgroup of 256 threads (4 wavefronts, one per SIMD, 512
//               registers each) per (row tile, split, KV head, sequence); the
//               host plan sizes it to about one workgroup per compute unit.
//       rows  : a wavefront owns 16*MB query rows (MB <= 5 MFMA row blocks).  Its
//               O^T accumulators and the Q operand live in hand-placed AccVGPRs
//               and are only touched by inline-asm MFMAs inside the loop.
//       K/V   : 64-token stages (4 pages) go global -> LDS directly (no register
//               staging) into a ring of four buffers, two stages in flight, one
//               LDS-only barrier per stage; K rows are XOR-swizzled at 16 B and
//               V rows at 32 B so that the MFMA operand reads spread over all banks.
//       QK^T  : X^T = K * Q'^T - m with v_mfma_f32_16x16x32_bf16, where
//               Q' = bf16(Q * scale * log2 e) and the negated row reference m is
//               the accumulator input: the result is the argument of exp2.  Each
//               lane holds exponents of ONE query row (column l%16), and the
//               packed probabilities are already laid out as the B operand of
//               the second product (no LDS round trip).
//       PV    : O^T += V^T * P^T; the V^T operand (contraction over tokens, which
//               are strided in memory) comes from the gfx950 LDS transpose read
//               ds_read_b64_tr_b16: a 16-lane group turns a 4-token x 16-dim
//               block into "lane = dim, 4 tokens packed".  Row sums: one more
//               MFMA per row block with an all-ones A operand.
//       pipeline: over 32-token sub-tiles, MFMAs of one sub-tile interleaved slot
//               by slot with the exp2 / pack / max work of its neighbours; the
//               MFMA operands are read from LDS two groups ahead, across the
//               boundary between the two regions of a step.
//       mask  : only sub-tiles that reach past the prefix take the masked path
//               (ancestor bits from graft_build_tree_mask); the prefix is dense.
//       softmax: a row's reference is the maximum of the first sub-tile that gives
//               it a finite score and is kept while later exponents stay below
//               2^24; beyond that the wavefront switches to an exact online
//               softmax loop that rescales the accumulators.
//     With one split per (sequence, KV head) the rows are normalised and written as
//     bf16 straight from the accumulators.  Otherwise partials (reference, sum, and
//     O / sum as fp16 rows with a per-row scale) go to the workspace; a small combine
//     kernel merges the splits and writes bf16.
//
// (2) everything else (fp32 storage, or D = 64): a plain one-workgroup-per-
//     (node, head) kernel in fp32.  It serves the tiny fp32 configuration and as
//     an independent GPU cross-check of path (1).
#include <type_traits>

#include <hip/hip_ext.h>

#include "common.h"

namespace graft {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

constexpr int AT_THREADS = 256;
constexpr int AT_WAVES = 4;
constexpr int AT_STAGE = 64;        // tokens per LDS stage (4 pages)
constexpr int AT_SUB = 32;          // tokens per softmax step
constexpr int AT_D = 128;
constexpr int AT_ROW_BYTES = AT_D * 2;
constexpr int AT_MAX_MB = 5;            // 16-row MFMA blocks per wavefront (5 * 48 = 240 of 256 AccVGPRs)
constexpr int AT_MAX_SPLITS = 64;
constexpr float AT_LAZY_LOG2 = 24.0f;  // a row keeps its reference while exponents stay below 2^24

struct AttnParams {
    const void* q;
    const void* k;
    const void* v;
    void* out;
    const int32_t* block_table;
    const int32_t* prefix_len;
    const int32_t* n_nodes;
    const u64* mask;
    unsigned short* ws_o;   // fp16 [B][Hkv][splits][R_pad/16][D/32] blocks of 1 KB: [lane][2][4], lane = MFMA
                            // accumulator lane, two adjacent 16-dim tiles per block
    float* ws_ml;       // [B][Hkv][splits][R_pad][4]  (max in log2 units, sum, scale of the stored row, 0)
    int64_t page_stride, token_stride, head_stride;
    int32_t max_pages, B, K_max, Hq, Hkv, G, R, R_pad, n_splits, n_row_tiles;
    int32_t g_magic;    // ceil(2^16 / G): r / G == (r * g_magic) >> 16 for r < 4096, G <= 16
    float scale;        // softmax scale
    float scale_log2e;  // scale * log2(e)
#ifdef GRAFT_ATTN_STAMPS
    unsigned long long* stamps;   // timing build: AT_STAMPS values per workgroup, or null
#endif
};

// Timing build (-DGRAFT_ATTN_STAMPS, a library of its own: see build.py): the MFMA kernel
// records when each workgroup passed the points below and writes them to a buffer the caller
// registered with graft_attn_stamp_buffer().  Times are values of the 100 MHz real-time counter
// (the first absolute, the others relative to it), two entries are the core-clock counter at
// both ends of the stage loop, which gives the clock the loop ran at.  Without the flag the
// macros are empty and the kernel is unchanged.
constexpr int AT_STAMPS = 24;
enum AttnStamp {
    AT_TS_START = 0,          // first instruction of the workgroup (absolute)
    AT_TS_LENGTHS = 1,        // lengths known
    AT_TS_TABLE_REQ = 2,      // block-table entries requested
    AT_TS_Q_DONE = 3,         // Q converted
    AT_TS_TABLE_LDS = 4,      // table and masks stored to LDS
    AT_TS_STAGE0_REQ = 5,     // transfers of stage 0 issued
    AT_TS_ZEROED = 6,         // accumulators zeroed, stage 1 issued (in front of the barrier)
    AT_TS_LOOP = 7,           // stage loop entered
    AT_TS_STAGE0 = 8,         // first stage arrived
    AT_TS_LOOP_END = 9,       // stage loop left
    AT_TS_END = 10,           // results written
    AT_TS_CYCLES_LOOP = 11,   // core-clock counter at AT_TS_LOOP
    AT_TS_CYCLES_END = 12,    // core-clock counter at AT_TS_LOOP_END
    AT_TS_STAGES = 13,        // stages of this workgroup
    AT_TS_VALID = 14,         // 1
    AT_TS_WAIT_CYCLES = 15,   // core-clock cycles wavefront 0 waited for its transfers of a stage, summed
    AT_TS_BARRIER_CYCLES = 16,  // ... and at the stage barriers (reading the counter costs some 50 cycles itself)
};
#ifdef GRAFT_ATTN_STAMPS
#define GRAFT_STAMPS_BEGIN()                                \
    unsigned long long at_stamp[AT_STAMPS] = {};            \
    at_stamp[AT_TS_START] = __builtin_amdgcn_s_memrealtime()
#define GRAFT_STAMP(k) (at_stamp[k] = __builtin_amdgcn_s_memrealtime() - at_stamp[AT_TS_START])
#define GRAFT_STAMP_CYCLES(k) (at_stamp[k] = __builtin_readcyclecounter())
#define GRAFT_SPAN_BEGIN() const unsigned long long at_span0 = __builtin_readcyclecounter()
#define GRAFT_SPAN_SPLIT(k) const unsigned long long at_span1 = __builtin_readcyclecounter(); at_stamp[k] += at_span1 - at_span0
#define GRAFT_SPAN_END(k) (at_stamp[k] += __builtin_readcyclecounter() - at_span1)
#define GRAFT_STAMPS_WRITE(p, n_stages)                                                     \
    do {                                                                                    \
        GRAFT_STAMP(AT_TS_END);                                                             \
        at_stamp[AT_TS_STAGES] = static_cast<unsigned long long>(n_stages);                 \
        at_stamp[AT_TS_VALID] = 1;                                                          \
        if (threadIdx.x == 0 && (p).stamps)                                                 \
            for (int at_k = 0; at_k < AT_STAMPS; ++at_k)                                    \
                (p).stamps[static_cast<size_t>(blockIdx.x) * AT_STAMPS + at_k] = at_stamp[at_k]; \
    } while (0)
#else
#define GRAFT_STAMPS_BEGIN() ((void)0)
#define GRAFT_STAMP(k) ((void)0)
#define GRAFT_STAMP_CYCLES(k) ((void)0)
#define GRAFT_SPAN_BEGIN() ((void)0)
#define GRAFT_SPAN_SPLIT(k) ((void)0)
#define GRAFT_SPAN_END(k) ((void)0)
#define GRAFT_STAMPS_WRITE(p, n_stages) ((void)0)
#endif

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
struct SplitRange { int st0, st1, P, n, total; };

constexpr int AT_MAX_SPLIT_PAGES = 4096;          // block-table entries of one split kept in LDS
constexpr int AT_NBUF = 4;                         // LDS stage buffers
constexpr int AT_STAGE_BYTES = 2 * AT_STAGE * AT_ROW_BYTES;   // K rows then V rows
constexpr int AT_LOADS_PER_STAGE = 8;              // global->LDS instructions per wavefront per stage

// Global -> LDS without passing through registers: each lane's 16 bytes land at
// (wavefront-uniform LDS base) + lane * 16, so the swizzled LDS layout is produced by
// choosing which global chunk each lane fetches.  One instruction moves 4 token rows (1 KB)
// of K or of V; 4 wavefronts x 4 x (K,V) = one 64-token stage.
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

// Same with the global address given as (wavefront-uniform 64-bit base) + (32-bit byte offset
// of the lane).
__device__ __forceinline__ void load_global_to_lds_b128(const void* base, unsigned lane_off, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(lane_off), "s"(base)
                 : "memory");
}

__device__ __forceinline__ unsigned lds_address(const void* p) {
    return static_cast<unsigned>(reinterpret_cast<size_t>(
        (const __attribute__((address_space(3))) unsigned char*)(p)));
}

// s_waitcnt vmcnt(N) only (expcnt / lgkmcnt fields left at "no wait")
#define GRAFT_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(0x0F70 | ((N) & 15) | (((N) >> 4) << 14))

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also drain the
// vector memory counter and with it the global->LDS transfers of the stages still in flight.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- MFMA issue through inline assembly, accumulators in fixed AccVGPRs ----------------
// With 512 registers per lane available the register allocator rotates MFMA accumulators
// between register sets, parks them in AccVGPRs and copies them back for every vector ALU
// use.  Here the placement is part of the design and is done by hand:
//   O^T accumulators of row block rb, dim block db : a[32 rb + 4 db .. +3], accumulated in
//       place and never touched by the vector ALUs inside the fast loop;
//   Q^T operand of row block rb < QA, dim step ds   : a[32 MB + 16 rb + 4 ds .. +3];
//   row sums of row block rb < 4                     : a[48 MB + 4 rb .. +3] (a fifth row block's
//       are in VGPRs: 48 * 5 + 16 = 256 is the whole AccVGPR file);
//   score tiles, probabilities, K/V operands        : VGPRs chosen by the compiler.
// The compiler itself uses no AccVGPR in this kernel (VGPR-to-AccVGPR spilling is switched
// off in the build, and the kernel must compile without spills); the asm statement in
// reserve_acc_registers() lists the hand-managed ones as clobbered so that they are counted in
// the kernel's register allocation; it is repeated inside the loops so that the compiler never
// parks a value of its own in one of them across the MFMAs.  asm volatile statements keep
// their relative order, which also pins the MFMA sequence.
// Hazards handled by construction: no vector ALU, LDS or memory instruction touches an MFMA
// result within 16 instructions of the MFMA (the pipeline regions are far apart and explicit
// s_nop guards the other places), dependent MFMAs on one accumulator are at least two
// instructions apart, AccVGPR writes are followed by s_nop before an MFMA reads them, an MFMA
// that may have a vector ALU write of one of its VGPR sources right in front of it (the first
// of a pipeline region, all of the slow path) begins with s_nop 1, and constants used as MFMA
// sources are made opaque to the compiler.  The build checks the generated assembly for the
// source-write distance, for compiler use of the hand-managed registers and for spills.
#define GRAFT_ACC_BLOCK_0 "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15", "a16", "a17", "a18", "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31", "a32", "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", "a45", "a46", "a47"
#define GRAFT_ACC_BLOCK_1 "a48", "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", "a58", "a59", "a60", "a61", "a62", "a63", "a64", "a65", "a66", "a67", "a68", "a69", "a70", "a71", "a72", "a73", "a74", "a75", "a76", "a77", "a78", "a79", "a80", "a81", "a82", "a83", "a84", "a85", "a86", "a87", "a88", "a89", "a90", "a91", "a92", "a93", "a94", "a95"
#define GRAFT_ACC_BLOCK_2 "a96", "a97", "a98", "a99", "a100", "a101", "a102", "a103", "a104", "a105", "a106", "a107", "a108", "a109", "a110", "a111", "a112", "a113", "a114", "a115", "a116", "a117", "a118", "a119", "a120", "a121", "a122", "a123", "a124", "a125", "a126", "a127", "a128", "a129", "a130", "a131", "a132", "a133", "a134", "a135", "a136", "a137", "a138", "a139", "a140", "a141", "a142", "a143"
#define GRAFT_ACC_BLOCK_3 "a144", "a145", "a146", "a147", "a148", "a149", "a150", "a151", "a152", "a153", "a154", "a155", "a156", "a157", "a158", "a159", "a160", "a161", "a162", "a163", "a164", "a165", "a166", "a167", "a168", "a169", "a170", "a171", "a172", "a173", "a174", "a175", "a176", "a177", "a178", "a179", "a180", "a181", "a182", "a183", "a184", "a185", "a186", "a187", "a188", "a189", "a190", "a191"
#define GRAFT_ACC_BLOCK_4 "a192", "a193", "a194", "a195", "a196", "a197", "a198", "a199", "a200", "a201", "a202", "a203", "a204", "a205", "a206", "a207", "a208", "a209", "a210", "a211", "a212", "a213", "a214", "a215", "a216", "a217", "a218", "a219", "a220", "a221", "a222", "a223", "a224", "a225", "a226", "a227", "a228", "a229", "a230", "a231", "a232", "a233", "a234", "a235", "a236", "a237", "a238", "a239"
#define GRAFT_ACC_BLOCK_5 "a240", "a241", "a242", "a243", "a244", "a245", "a246", "a247", "a248", "a249", "a250", "a251", "a252", "a253", "a254", "a255"

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}
#define GRAFT_CONST(name, ic) constexpr int name = decltype(ic)::value

template <int MB> constexpr int q_in_acc() { return MB; }   // row blocks with Q^T in AccVGPRs (all, for MB <= 5)
constexpr int L_IN_ACC = 4;                                  // row blocks with their row sums in AccVGPRs
template <int MB> constexpr int acc_used() { return 32 * MB + 16 * q_in_acc<MB>() + 4 * (MB < L_IN_ACC ? MB : L_IN_ACC); }
constexpr int o_reg(int rb, int db) { return 32 * rb + 4 * db; }
template <int MB> constexpr int q_reg(int rb, int ds) { return 32 * MB + 16 * rb + 4 * ds; }
template <int MB> constexpr int l_reg(int rb) { return 48 * MB + 4 * rb; }

template <int MB>
__device__ __forceinline__ void reserve_acc_registers() {
    asm volatile("" ::: GRAFT_ACC_BLOCK_0);
    if constexpr (acc_used<MB>() > 48) asm volatile("" ::: GRAFT_ACC_BLOCK_1);
    if constexpr (acc_used<MB>() > 96) asm volatile("" ::: GRAFT_ACC_BLOCK_2);
    if constexpr (acc_used<MB>() > 144) asm volatile("" ::: GRAFT_ACC_BLOCK_3);
    if constexpr (acc_used<MB>() > 192) asm volatile("" ::: GRAFT_ACC_BLOCK_4);
    if constexpr (acc_used<MB>() > 240) asm volatile("" ::: GRAFT_ACC_BLOCK_5);
}

template <int R> __device__ __forceinline__ void acc_set(float v) {
    asm volatile("v_accvgpr_write_b32 a[%0], %1" : : "n"(R), "v"(v));
}
template <int R> __device__ __forceinline__ void acc_set_bits(unsigned v) {
    asm volatile("v_accvgpr_write_b32 a[%0], %1" : : "n"(R), "v"(v));
}
template <int R> __device__ __forceinline__ float acc_get() {
    float v;
    asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(v) : "n"(R));
    return v;
}
template <int R> __device__ __forceinline__ void acc_scale(float a) {
    float t;
    asm volatile("v_accvgpr_read_b32 %0, a[%1]\n\ts_nop 1\n\tv_mul_f32 %0, %0, %2\n\ts_nop 1\n\tv_accvgpr_write_b32 a[%1], %0"
                 : "=&v"(t)
                 : "n"(R), "v"(a));
}
// The compiler does not know that these asm statements are MFMAs, so it inserts none of the
// wait states an MFMA needs after a vector ALU write of one of its VGPR sources (2 for the
// A and B operands, 1 for C: measured on gfx950, a shorter distance makes the MFMA read the
// old register contents).  Two mechanisms cover this: GUARD = true puts s_nop 1 in front of
// the MFMA (used wherever the preceding instructions are the compiler's choice and the cost
// does not matter), and the build checks the generated assembly of this file and fails if
// any MFMA has a vector ALU write of one of its sources within the two preceding
// instructions.  Constants used as MFMA sources are made opaque to the compiler so that it
// cannot rematerialise them in front of the statement.
#define GRAFT_MFMA_GUARD "s_nop 1\n\t"
// exponent tile (VGPRs) = K operand (VGPRs) x Q'^T operand (fixed AccVGPRs) + C, where C is the
// tile being accumulated or, for the first dim step, the row's negated reference.
template <int QR, bool GUARD = false>
__device__ __forceinline__ void mfma_x_first(floatx4& d, const bf16x8& ka, const floatx4& c) {
    if constexpr (GUARD)
        asm volatile(GRAFT_MFMA_GUARD "v_mfma_f32_16x16x32_bf16 %0, %1, a[%2:%3], %4"
                     : "=&v"(d) : "v"(ka), "n"(QR), "n"(QR + 3), "v"(c));
    else
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, a[%2:%3], %4"
                     : "=&v"(d) : "v"(ka), "n"(QR), "n"(QR + 3), "v"(c));
}
template <int QR, bool GUARD = false>
__device__ __forceinline__ void mfma_x_next(floatx4& d, const bf16x8& ka) {
    if constexpr (GUARD)
        asm volatile(GRAFT_MFMA_GUARD "v_mfma_f32_16x16x32_bf16 %0, %1, a[%2:%3], %0"
                     : "+v"(d) : "v"(ka), "n"(QR), "n"(QR + 3));
    else
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, a[%2:%3], %0" : "+v"(d) : "v"(ka), "n"(QR), "n"(QR + 3));
}
// O^T tile (fixed AccVGPRs) += V^T operand (VGPRs) x P^T operand (VGPRs)
template <int OR, bool GUARD = false>
__device__ __forceinline__ void mfma_o(const bf16x8& va, const uintx4& pb) {
    if constexpr (GUARD)
        asm volatile(GRAFT_MFMA_GUARD "v_mfma_f32_16x16x32_bf16 a[%0:%1], %2, %3, a[%0:%1]"
                     : : "n"(OR), "n"(OR + 3), "v"(va), "v"(pb));
    else
        asm volatile("v_mfma_f32_16x16x32_bf16 a[%0:%1], %2, %3, a[%0:%1]"
                     : : "n"(OR), "n"(OR + 3), "v"(va), "v"(pb));
}
// row sums += ones x P^T operand: every element of the tile ends up holding the row's sum.
// In AccVGPRs a[LR .. LR+3], or (a fifth row block) in VGPRs.
template <int LR, bool GUARD = false>
__device__ __forceinline__ void mfma_rowsum_acc(const bf16x8& ones, const uintx4& pb) {
    if constexpr (GUARD)
        asm volatile(GRAFT_MFMA_GUARD "v_mfma_f32_16x16x32_bf16 a[%0:%1], %2, %3, a[%0:%1]" : : "n"(LR), "n"(LR + 3), "v"(ones), "v"(pb));
    else
        asm volatile("v_mfma_f32_16x16x32_bf16 a[%0:%1], %2, %3, a[%0:%1]" : : "n"(LR), "n"(LR + 3), "v"(ones), "v"(pb));
}
template <bool GUARD = false>
__device__ __forceinline__ void mfma_rowsum(floatx4& l, const bf16x8& ones, const uintx4& pb) {
    if constexpr (GUARD)
        asm volatile(GRAFT_MFMA_GUARD "v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(l) : "v"(ones), "v"(pb));
    else
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(l) : "v"(ones), "v"(pb));
}
// Two fp32 -> one packed pair of bf16 (round to nearest even): v_cvt_pk_bf16_f32.
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
    typedef float floatx2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(unsigned, __builtin_convertvector(floatx2{lo, hi}, bf16x2));
}
// A register holding a bit pattern the compiler cannot see through (so it is kept, not
// rematerialised in front of an MFMA that reads it).
__device__ __forceinline__ unsigned opaque_bits(unsigned v) {
    unsigned r;
    asm volatile("v_mov_b32 %0, %1" : "=v"(r) : "s"(v));
    return r;
}
#define GRAFT_MFMA_SETTLE() asm volatile("s_nop 15\n\ts_nop 7" ::: "memory")
// An empty asm that reads x: the registers of x stay allocated up to this point.  Used in the
// slow path after a group of MFMAs so that their source registers are not reused in between.
// (Not inside the pipeline regions: a use of an operand buffer after its reload has been
// issued makes the compiler wait for that reload, which undoes the prefetch.)
#define GRAFT_KEEP(x) asm volatile("" : : "v"(x))

// What one wavefront keeps in VGPRs for its 16*MB query rows (O^T and Q'^T are in AccVGPRs).
// Exponents are in log2 units throughout: Q' = bf16(Q * scale * log2 e), so that the MFMA
// result q'.k - m_ref is directly the argument of exp2.
template <int MB>
struct WaveRows {
    floatx4 negm[MB];       // {-m_ref} x 4: accumulator input of the first QK^T step (0 while unset);
                            // m_ref is the reference max of the row in log2 units
    floatx4 lsum_v;         // row sums of a fifth row block (the others' are in AccVGPRs)
    float thr[MB];          // an exponent above this needs attention: -inf while the row has no reference
                            // yet, else the lazy bound
    float thr_min;          // the smallest of thr[]: one compare of the largest new exponent against it
                            // decides whether any row needs attention (the rows are then looked at one by one)
    __device__ __forceinline__ bool unset(int rb) const { return thr[rb] == -INFINITY; }
    __device__ __forceinline__ float m_ref(int rb) const { return unset(rb) ? -INFINITY : -negm[rb][0]; }
};

// LDS byte offsets of this lane's MFMA operands inside a 32-token sub-tile.
// K group g = (c, ds): rows 16c + l16, 16-byte chunk (4ds + lg) ^ l16.
__device__ __forceinline__ bf16x8 load_k_operand(const unsigned char* Ks, int g, int l16, int lg) {
    const int c = g >> 2, ds = g & 3;
    return *reinterpret_cast<const bf16x8*>(Ks + (16 * c + l16) * AT_ROW_BYTES + (((4 * ds + lg) ^ l16) * 16));
}
// V^T operand of dim block db through the LDS transpose read: a 16-lane group turns the
// 4-token x 16-dim block (tokens 16c + 4lg .. +3, dims 16db .. +15) into "lane = dim, 4 tokens".
// (half c = tokens 16c .. 16c + 15 of the sub-tile: one transpose read, elements 4c .. 4c + 3)
template <int C>
__device__ __forceinline__ void load_v_half(bf16x8& va, const unsigned char* Vs, int db, int l16, int lg) {
    // row 16C + 4lg + (l16 >> 2), 32-byte segment db ^ (row & 7): the segment is bits 5-7 of the
    // address, row & 7 does not depend on C, and sub-tiles start at multiples of 256 bytes, so
    // the address is the lane's base (which carries row & 7 in those bits) XOR db << 5, plus a
    // constant for C that fits the read's offset field: one vector instruction per dim block.
    const int row0 = 4 * lg + (l16 >> 2);
    const unsigned base = lds_address(Vs) + row0 * AT_ROW_BYTES + ((row0 & 7) << 5) + 8 * (l16 & 3);
    const short4_t r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (short4_t __attribute__((address_space(3)))*)(static_cast<size_t>((base ^ (db << 5)) + C * 16 * AT_ROW_BYTES)));
    const bf16x4 r4 = __builtin_bit_cast(bf16x4, r);
    va[4 * C + 0] = r4[0];
    va[4 * C + 1] = r4[1];
    va[4 * C + 2] = r4[2];
    va[4 * C + 3] = r4[3];
}
__device__ __forceinline__ bf16x8 load_v_operand(const unsigned char* Vs, int db, int l16, int lg) {
    bf16x8 va;
    load_v_half<0>(va, Vs, db, l16, lg);
    load_v_half<1>(va, Vs, db, l16, lg);
    return va;
}

// The vector ALUs are the scarce resource of the pipeline: next to one MFMA the wavefront
// can issue one exponential, or two plain vector instructions, without delaying the next
// MFMA.  Region 1 therefore exponentiates only the first rows_early<MB>() row blocks; the
// last ("late") row block's probabilities are computed one region earlier, in region 2,
// whose other vector work (the maximum scan) leaves slots free.
template <int MB> constexpr int rows_early() { return MB >= 2 ? MB - 1 : MB; }
// The two pipeline regions share a ring of four MFMA operand buffers.  Operand g of a region
// (eight per region) lives in ring[g & 3] and is read from LDS read_ahead<MB>() groups before
// its MFMAs; the last groups of a region read the first operands of the region that follows
// (K after V after K ...), so the LDS latency never shows at a region's start.  The exception
// is the first region of a stage (FIRST): the stage is only known to have landed after the
// barrier in front of it, so it reads its own first operands and the region before it (LAST)
// reads nothing ahead.
// How many groups (of MB MFMAs, 16.4 cycles each) an operand is read from LDS ahead of its use.
// Three (the most the ring allows) was measured 2 % slower than two with three row blocks.
template <int MB> constexpr int read_ahead() { return 2; }

// Pipeline region 1: the matrix cores compute the exponents of the NEXT sub-tile
// (X^T = K Q'^T - m_ref into xn) while the vector ALUs turn the CURRENT sub-tile's exponents
// xc into probabilities (pb, packed bf16) for the early row blocks.  One MFMA and one
// exponential per slot; sched_barrier pins the interleaving because the wavefront issues in
// order.
template <int MB, bool FIRST>
__device__ __forceinline__ void region_qk_exp(const unsigned char* __restrict__ Ks,
                                              const unsigned char* __restrict__ Vnext, const WaveRows<MB>& w,
                                              floatx4 (&xn)[MB][2], const floatx4 (&xc)[MB][2],
                                              uintx4 (&pb)[MB], bf16x8 (&ring)[4], int lane) {
    constexpr int E = rows_early<MB>();
    constexpr int PF = read_ahead<MB>();
    const int l16 = lane & 15, lg = lane >> 4;
    constexpr bool LATE = E < MB;
    constexpr int H = (E + 1) / 2;
    // Exponentials waiting to be packed.  Pair p = groups 2p (-> e0[p & 1]) and 2p + 1 (-> e1).
    // With a late row block its slots do the packing, two per slot so that no slot holds more
    // than 8 cycles of vector work: rows < H of pair p in group 2p + 1, the others in group
    // 2p + 2 (hence two copies of e0).  Without one, a pair is packed next to the exponential
    // one group later.
    float e0[2][E], e1[E];
    if constexpr (FIRST) {
        ring[0] = load_k_operand(Ks, 0, l16, lg);
        ring[1] = load_k_operand(Ks, 1, l16, lg);
        if constexpr (PF > 2) ring[2] = load_k_operand(Ks, 2, l16, lg);
    }
    static_for<0, 8>([&](auto g_) {
        GRAFT_CONST(g, g_);
        constexpr int c = g >> 2, ds = g & 3;
        if constexpr (g + PF < 8) ring[(g + PF) & 3] = load_k_operand(Ks, g + PF, l16, lg);
        else ring[(g + PF) & 3] = load_v_operand(Vnext, g + PF - 8, l16, lg);
        static_for<0, MB>([&](auto rb_) {
            GRAFT_CONST(rb, rb_);
            constexpr bool guard = (g == 0 && rb == 0);
            if constexpr (ds == 0) mfma_x_first<q_reg<MB>(rb, 0), guard>(xn[rb][c], ring[g & 3], w.negm[rb]);
            else mfma_x_next<q_reg<MB>(rb, ds), guard>(xn[rb][c], ring[g & 3]);
            if constexpr (rb < E) {
                if constexpr (!LATE && (g & 1) == 0 && g >= 2)
                    pb[rb][(g - 2) >> 1] = pack_bf16(e0[((g - 2) >> 1) & 1][rb], e1[rb]);
                const float pe = __builtin_amdgcn_exp2f(xc[rb][c][ds]);
                if constexpr (g & 1) e1[rb] = pe;
                else e0[(g >> 1) & 1][rb] = pe;
            } else if constexpr (g & 1) {           // late slot of group 2p + 1: rows < H of pair p
                constexpr int pr = g >> 1;
#pragma unroll
                for (int r = 0; r < H; ++r) pb[r][pr] = pack_bf16(e0[pr & 1][r], e1[r]);
            } else if constexpr (g >= 2) {          // late slot of group 2p + 2: the other rows of pair p
                constexpr int pr = (g - 2) >> 1;
#pragma unroll
                for (int r = H; r < E; ++r) pb[r][pr] = pack_bf16(e0[pr & 1][r], e1[r]);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    });
#pragma unroll
    for (int rb = LATE ? H : 0; rb < E; ++rb) pb[rb][3] = pack_bf16(e0[1][rb], e1[rb]);
    __builtin_amdgcn_sched_barrier(0);
}

// Probabilities of the late row block from its exponents, outside the pipeline: after the
// exponents were changed behind region 2's back (ancestor masking, a new reference).
template <int MB>
__device__ __forceinline__ void late_probabilities(const floatx4 (&x)[MB][2], uintx4& pl) {
    if constexpr (rows_early<MB>() < MB) {
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float p0 = __builtin_amdgcn_exp2f(x[MB - 1][e >> 2][e & 3]);
            const float p1 = __builtin_amdgcn_exp2f(x[MB - 1][e >> 2][(e & 3) + 1]);
            pl[e >> 1] = pack_bf16(p0, p1);
        }
    }
}

// Pipeline region 2: the matrix cores run O^T += V^T P^T and the row sums of the CURRENT
// sub-tile (probabilities: pb for the early row blocks, pl_cur for the late one) while the
// vector ALUs scan the NEXT sub-tile's exponents xn for their lane-local maxima (first half
// of the region) and turn the late row block's into probabilities pl_next (second half;
// speculative: the caller redoes them when the scan or the masking changes the exponents).
// Returns whether any lane saw an exponent above its row's threshold (wavefront-uniform).
template <int MB, bool LAST>
__device__ __forceinline__ bool region_pv_max(const unsigned char* __restrict__ Vs,
                                              const unsigned char* __restrict__ Knext, WaveRows<MB>& w,
                                              const uintx4 (&pb)[MB], const uintx4& pl_cur, uintx4& pl_next,
                                              const floatx4 (&xn)[MB][2], const bf16x8& ones, float ninf,
                                              float (&lm)[MB], bf16x8 (&ring)[4], int lane) {
    constexpr int E = rows_early<MB>();
    constexpr int PF = read_ahead<MB>();
    constexpr bool LATE = E < MB;
    constexpr bool INLOOP = LATE && MB >= 3;     // three free slots per group are needed
    const int l16 = lane & 15, lg = lane >> 4;
    float le0 = 0.f, le1 = 0.f;
    unsigned long long above = 0;
    static_for<0, 8>([&](auto db_) {
        GRAFT_CONST(db, db_);
        static_for<0, MB>([&](auto rb_) {
            GRAFT_CONST(rb, rb_);
            if constexpr (rb < E) mfma_o<o_reg(rb, db), (db == 0 && rb == 0)>(ring[db & 3], pb[rb]);
            else mfma_o<o_reg(rb, db), (db == 0 && rb == 0)>(ring[db & 3], pl_cur);
            // The slot's vector work, at most 8 cycles of it where the slots suffice.
            // LDS reads of the operand two groups ahead: one half in each of the first two slots.
            if constexpr (rb == 0) {
                if constexpr (db + PF < 8) load_v_half<0>(ring[(db + PF) & 3], Vs, db + PF, l16, lg);
                else if constexpr (!LAST) ring[(db + PF) & 3] = load_k_operand(Knext, db + PF - 8, l16, lg);
            }
            if constexpr (rb == (MB > 1 ? 1 : 0) && db + PF < 8) load_v_half<1>(ring[(db + PF) & 3], Vs, db + PF, l16, lg);
            if constexpr (db < 4) {
                // maximum scan, two exponents of one row block per instruction; slot 0 is left
                // to the LDS read where there are five slots (row blocks 0 and 1 go to slots 1, 2)
                static_for<0, MB>([&](auto r_) {
                    GRAFT_CONST(r, r_);
                    constexpr int slot = MB == 5 ? (r == 0 ? 1 : (r == 1 ? 2 : r)) : r;
                    if constexpr (slot == rb) {
                        const float a = xn[r][db >> 1][2 * (db & 1)], b = xn[r][db >> 1][2 * (db & 1) + 1];
                        // (the three-operand form also for the first pair: a plain two-operand
                        // maximum would first canonicalise both inputs, two more instructions)
                        lm[r] = __builtin_fmaxf(__builtin_fmaxf(db == 0 ? ninf : lm[r], a), b);
                    }
                });
            }
            if constexpr (db == 4 && rb == (MB >= 4 ? 0 : MB - 1)) {
                // the scan is complete: one compare for all row blocks, long before the branch on
                // it at the end of the region (a branch on a fresh vector compare would stall)
                float lmax = lm[0];
#pragma unroll
                for (int r = 1; r < MB; ++r) lmax = __builtin_fmaxf(lmax, lm[r]);
                above = __builtin_amdgcn_ballot_w64(lmax > w.thr_min);
                asm volatile("" : "+s"(above));
            }
            if constexpr (db < 4) {
            } else if constexpr (INLOOP && (rb == MB - 3 || rb == MB - 2)) {
                // late row block: element 2 (db - 4) + {0, 1} of its 8; the pair is packed in
                // the slot after its second exponential
                constexpr int e = 2 * (db - 4) + (rb - (MB - 3));
                const float pe = __builtin_amdgcn_exp2f(xn[MB - 1][e >> 2][e & 3]);
                if constexpr (rb == MB - 3) le0 = pe;
                else le1 = pe;
            } else if constexpr (INLOOP && rb == MB - 1) {
                pl_next[db - 4] = pack_bf16(le0, le1);
                // (pinned here: the caller overwrites pl_next on some paths, and the compiler
                //  would otherwise move these exponentials to the paths that do not)
                asm volatile("" : "+v"(pl_next[db - 4]));
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    });
    if constexpr (LATE && !INLOOP) late_probabilities<MB>(xn, pl_next);
    static_for<0, MB>([&](auto rb_) {
        GRAFT_CONST(rb, rb_);
        if constexpr (rb >= L_IN_ACC) mfma_rowsum(w.lsum_v, ones, rb < E ? pb[rb] : pl_cur);
        else if constexpr (rb < E) mfma_rowsum_acc<l_reg<MB>(rb)>(ones, pb[rb]);
        else mfma_rowsum_acc<l_reg<MB>(rb)>(ones, pl_cur);
    });
    const bool any = above != 0;
#pragma unroll
    for (int rb = 0; rb < E; ++rb) GRAFT_KEEP(pb[rb]);
    GRAFT_KEEP(pl_cur);
    return any;
}

// Ancestor masking of an exponent tile that reaches past the prefix (tree slots and the
// tail): masked entries become -inf; the lane-local maxima are recomputed.
template <int MB>
__device__ __forceinline__ bool apply_tree_mask(floatx4 (&x)[MB][2], const WaveRows<MB>& w, float (&lm)[MB],
                                                int lane, int t_sub0, int P, int n, int r_base, int R, int g_magic,
                                                const unsigned* __restrict__ Ms) {
    const int l16 = lane & 15, lg = lane >> 4;
    bool grow = false;
#pragma unroll
    for (int rb = 0; rb < MB; ++rb) {
        const int r = r_base + rb * 16 + l16;
        const int node = (r * g_magic) >> 16;              // r / G
        const bool live = r < R && node < n;
        const int nd = live ? node : 0;
        unsigned wd[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) wd[k] = live ? Ms[4 * nd + k] : 0u;
        float mx = -INFINITY;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            reserve_acc_registers<MB>();                      // no temporaries of the compiler's in the accumulators
            const int j0 = t_sub0 + 16 * c + 4 * lg - P;      // tree slot of element i = 0
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int j = j0 + i;
                const int wi = (j >> 5) & 3;
                const unsigned word = wi == 0 ? wd[0] : (wi == 1 ? wd[1] : (wi == 2 ? wd[2] : wd[3]));
                const bool bit = (word >> (j & 31)) & 1u;
                const bool valid = (j < 0) | ((j < n) & bit);
                x[rb][c][i] = valid ? x[rb][c][i] : -INFINITY;
                mx = fmaxf(mx, x[rb][c][i]);
            }
        }
        lm[rb] = mx;
        grow = grow || (mx > w.thr[rb]);
    }
    return __builtin_amdgcn_ballot_w64(grow) != 0;
}

// Some lane saw an exponent above its row's threshold.  Rows without a reference take the
// tile's row maximum as their reference: nothing has been accumulated for them yet, so only
// the pending exponents are re-based.  Returns true when a row that already has a reference
// exceeded the lazy bound: the caller then leaves the fast loop (that needs a rescale of O).
template <int MB>
__device__ __forceinline__ bool set_references(float (&lm)[MB], WaveRows<MB>& w, floatx4 (&x)[MB][2]) {
    bool raise = false;
#pragma unroll
    for (int rb = 0; rb < MB; ++rb) {
        float mx = lm[rb];
        mx = rows_max_f32(mx);
        lm[rb] = mx;                                      // now the row maximum, same in the row's 4 lanes
        raise = raise || (!w.unset(rb) && mx > w.thr[rb]);
    }
    if (__builtin_amdgcn_ballot_w64(raise) != 0) return true;
#pragma unroll
    for (int rb = 0; rb < MB; ++rb) {
        if (w.unset(rb) && lm[rb] > -INFINITY) {
            w.negm[rb] = floatx4{-lm[rb], -lm[rb], -lm[rb], -lm[rb]};
            w.thr[rb] = AT_LAZY_LOG2;
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int i = 0; i < 4; ++i) x[rb][c][i] -= lm[rb];
        }
    }
    float tm = w.thr[0];
#pragma unroll
    for (int rb = 1; rb < MB; ++rb) tm = fminf(tm, w.thr[rb]);
    w.thr_min = tm;
    return false;
}

// Slow path (exact running max, classic online softmax): raise every row's reference to
// the maximum seen so far, rescaling O and the row sums.  lm holds the row maxima of x.
template <int MB>
__device__ __forceinline__ void raise_references(const float (&lm)[MB], WaveRows<MB>& w, floatx4 (&x)[MB][2]) {
    GRAFT_MFMA_SETTLE();
    static_for<0, MB>([&](auto rb_) {
        GRAFT_CONST(rb, rb_);
        const float mx = lm[rb];
        const bool unset = w.unset(rb);
        const bool move = (!unset && mx > 0.0f) || (unset && mx > -INFINITY);
        if (__builtin_amdgcn_ballot_w64(move) != 0) {
            // rows that do not move get a = 1 and a zero shift
            const float shift = move ? mx : 0.0f;
            const float a = move ? (unset ? 0.0f : __builtin_amdgcn_exp2f(-mx)) : 1.0f;
            if (move) {
                const float nm = (unset ? 0.0f : w.negm[rb][0]) - mx;
                w.negm[rb] = floatx4{nm, nm, nm, nm};
                w.thr[rb] = AT_LAZY_LOG2;
            }
            if constexpr (rb >= L_IN_ACC) w.lsum_v *= a;
            else
                static_for<0, 4>([&](auto k_) {
                    GRAFT_CONST(k, k_);
                    acc_scale<l_reg<MB>(rb) + k>(a);
                });
            static_for<0, 32>([&](auto k_) {
                GRAFT_CONST(k, k_);
                acc_scale<32 * rb + k>(a);
            });
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int i = 0; i < 4; ++i) x[rb][c][i] -= shift;
        }
    });
    GRAFT_MFMA_SETTLE();
}

// Slow-path building blocks: the same arithmetic as the pipeline regions, one thing at a time.
template <int MB>
__device__ __forceinline__ void qk_only(const unsigned char* __restrict__ Ks, const WaveRows<MB>& w,
                                        floatx4 (&x)[MB][2], int lane) {
    const int l16 = lane & 15, lg = lane >> 4;
    static_for<0, 8>([&](auto g_) {
        GRAFT_CONST(g, g_);
        const bf16x8 ka = load_k_operand(Ks, g, l16, lg);
        static_for<0, MB>([&](auto rb_) {
            GRAFT_CONST(rb, rb_);
            if constexpr ((g & 3) == 0) mfma_x_first<q_reg<MB>(rb, 0), true>(x[rb][g >> 2], ka, w.negm[rb]);
            else mfma_x_next<q_reg<MB>(rb, (g & 3)), true>(x[rb][g >> 2], ka);
            asm volatile("s_nop 7" ::: "memory");
        });
        asm volatile("s_nop 15" ::: "memory");
        GRAFT_KEEP(ka);
    });
    GRAFT_MFMA_SETTLE();
}
template <int MB>
__device__ __forceinline__ void exp_only(const floatx4 (&x)[MB][2], uintx4 (&pb)[MB]) {
#pragma unroll
    for (int rb = 0; rb < MB; ++rb)
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float p0 = __builtin_amdgcn_exp2f(x[rb][e >> 2][e & 3]);
            const float p1 = __builtin_amdgcn_exp2f(x[rb][e >> 2][(e & 3) + 1]);
            pb[rb][e >> 1] = pack_bf16(p0, p1);
        }
}
template <int MB>
__device__ __forceinline__ void pv_only(const unsigned char* __restrict__ Vs, WaveRows<MB>& w,
                                        const uintx4 (&pb)[MB], const bf16x8& ones, int lane) {
    const int l16 = lane & 15, lg = lane >> 4;
    static_for<0, 8>([&](auto db_) {
        GRAFT_CONST(db, db_);
        const bf16x8 va = load_v_operand(Vs, db, l16, lg);
        static_for<0, MB>([&](auto rb_) {
            GRAFT_CONST(rb, rb_);
            mfma_o<o_reg(rb, db), true>(va, pb[rb]);
            asm volatile("s_nop 7" ::: "memory");
        });
        asm volatile("s_nop 15" ::: "memory");
        GRAFT_KEEP(va);
    });
    static_for<0, MB>([&](auto rb_) {
        GRAFT_CONST(rb, rb_);
        if constexpr (rb >= L_IN_ACC) mfma_rowsum<true>(w.lsum_v, ones, pb[rb]);
        else mfma_rowsum_acc<l_reg<MB>(rb), true>(ones, pb[rb]);
        asm volatile("s_nop 7" ::: "memory");
    });
    GRAFT_MFMA_SETTLE();
#pragma unroll
    for (int rb = 0; rb < MB; ++rb) GRAFT_KEEP(pb[rb]);
}

// One split only: O / l as bf16, straight from the accumulators.  Lane (l16, lg) holds row l16 of
// each row block, dims 16 db + 4 lg .. +3 of dim block db.  Rows of absent nodes are zeros.
template <int MB>
__device__ __forceinline__ void store_rows(const AttnParams& p, const WaveRows<MB>& w, int b, int g, int r_base,
                                           int n, int lane) {
    const int l16 = lane & 15, lg = lane >> 4;
    static_for<0, MB>([&](auto rb_) {
        GRAFT_CONST(rb, rb_);
        const int r = r_base + rb * 16 + l16;
        float l;
        if constexpr (rb >= L_IN_ACC) l = w.lsum_v[0];
        else l = acc_get<l_reg<MB>(rb)>();
        const int i = (r * p.g_magic) >> 16, hl = r - i * p.G;                  // i = r / G
        const bool keep = i < n && l > 0.f;
        const float inv_l = keep ? 1.0f / l : 0.f;
        unsigned short* outp = static_cast<unsigned short*>(p.out) +
            ((static_cast<int64_t>(b) * p.K_max + i) * p.Hq + g * p.G + hl) * AT_D + 4 * lg;
        static_for<0, 8>([&](auto db_) {
            GRAFT_CONST(db, db_);
            float o[4];
            static_for<0, 4>([&](auto k_) {
                GRAFT_CONST(k, k_);
                const float v = acc_get<o_reg(rb, db) + k>();
                o[k] = keep ? v * inv_l : 0.f;
            });
            if (r < p.R) *reinterpret_cast<uint2*>(outp + 16 * db) = uint2{pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3])};
        });
    });
}

// Rounds q * f to bf16 for two packed bf16 values.
__device__ __forceinline__ unsigned scale_bf16_pair(unsigned q2, float f) {
    return pack_bf16(__uint_as_float(q2 << 16) * f, __uint_as_float(q2 & 0xffff0000u) * f);
}

template <int MB>
__global__ __launch_bounds__(AT_THREADS) void tree_attn_mfma_kernel(AttnParams p) {
    __shared__ __attribute__((aligned(1024))) unsigned char kv[AT_NBUF][AT_STAGE_BYTES];
    __shared__ unsigned Ms[GRAFT_MAX_NODES * GRAFT_MASK_WORDS * 2];   // ancestor masks as 32-bit words
    __shared__ int32_t Tb[AT_MAX_SPLIT_PAGES];                         // this split's block-table entries

    reserve_acc_registers<MB>();
    GRAFT_STAMPS_BEGIN();
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_u = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lg = lane >> 4;
    // Workgroups go to the 8 XCDs (each with its own L2) round-robin by their linear index.
    // The row tiles of one (sequence, KV head, split) read the same keys and values: they get
    // the same XCD and neighbouring slots on it, so that they run side by side and all but the
    // first reader find the stage in that XCD's L2.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int rt = slot % p.n_row_tiles;
    const int unit = (slot / p.n_row_tiles) * 8 + xcd;           // over B * Hkv * n_splits
    if (unit >= p.B * p.Hkv * p.n_splits) return;                 // grid padding (whole workgroup)
    const int split = unit % p.n_splits;
    const int g = (unit / p.n_splits) % p.Hkv, b = unit / (p.n_splits * p.Hkv);

    // The set-up is a chain of dependent trips to memory (lengths -> block table -> first
    // keys), so everything that does not depend on the lengths is requested alongside them:
    // the lengths first (vector memory returns in order, and they are waited for first), then
    // this wavefront's Q rows and the sequence's ancestor masks.
    const int n_raw = p.n_nodes[b];
    const int P_raw = p.prefix_len[b];
    // Q rows of this wavefront (rows past R read row 0 and are zeroed when converted)
    const int r_base = rt * (AT_WAVES * 16 * MB) + wave_u * (16 * MB);
    uintx4 qd[MB][4];
#pragma unroll
    for (int rb = 0; rb < MB; ++rb) {
        const int r = r_base + rb * 16 + l16;
        const int rc = r < p.R ? r : 0;
        const int i = (rc * p.g_magic) >> 16, hl = rc - i * p.G;     // i = rc / G
        const __bf16* qp = static_cast<const __bf16*>(p.q) +
            ((static_cast<size_t>(b) * p.K_max + i) * p.Hq + (g * p.G + hl)) * AT_D + lg * 8;
#pragma unroll
        for (int ds = 0; ds < 4; ++ds) qd[rb][ds] = *reinterpret_cast<const uintx4*>(qp + 32 * ds);
    }

    // ancestor masks as 32-bit words: two rounds of 256 cover the 64 nodes x 4 x 64 bits
    static_assert(GRAFT_MAX_NODES * GRAFT_MASK_WORDS * 2 <= 2 * AT_THREADS, "mask words per thread");
    const int n_mask_words = p.K_max * GRAFT_MASK_WORDS * 2;
    const unsigned* mask_words = reinterpret_cast<const unsigned*>(p.mask) + static_cast<size_t>(b) * n_mask_words;
    const unsigned mw0 = tid < n_mask_words ? mask_words[tid] : 0u;
    const unsigned mw1 = tid + AT_THREADS < n_mask_words ? mask_words[tid + AT_THREADS] : 0u;

    SplitRange sr;
    int n = n_raw;
    if (n < 1 || n > p.K_max) n = 0;
    const int cap = p.max_pages * GRAFT_PAGE_SIZE;
    int P = P_raw;
    P = P < 0 ? 0 : (P > cap ? cap : P);
    sr.n = n;
    sr.P = P;
    sr.total = n ? ((P + n) < cap ? (P + n) : cap) : 0;
    const int n_stages = (sr.total + AT_STAGE - 1) / AT_STAGE;
    const int spt = (n_stages + p.n_splits - 1) / p.n_splits;
    sr.st0 = split * spt;
    sr.st1 = (sr.st0 + spt) < n_stages ? (sr.st0 + spt) : n_stages;
    if (sr.st1 < sr.st0) sr.st1 = sr.st0;
    const int n_st = sr.st1 - sr.st0;
#ifdef GRAFT_ATTN_STAMPS
    asm volatile("" : : "s"(n_st));              // (the stamp is taken when the lengths are there)
#endif
    GRAFT_STAMP(AT_TS_LENGTHS);

    // this split's block-table entries: the first 1024 are requested before anything is
    // stored (one trip for all of them), a longer split takes the plain loop for the rest.
    // The pages of this wavefront's first two stages are also requested on their own, as
    // scalars: with them the first transfers can be issued without a trip through LDS and a
    // barrier.
    int32_t tbv[4];
    const int n_pg = n_st * (AT_STAGE / GRAFT_PAGE_SIZE);
    const int32_t* table = p.block_table + static_cast<size_t>(b) * p.max_pages;
    const int first_pg = sr.st0 * (AT_STAGE / GRAFT_PAGE_SIZE);
    const int last_pg = (sr.total - 1) >> 4;
    int32_t first_pages[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int pg = first_pg + 4 * u + wave_u;
        first_pages[u] = (4 * u + wave_u) < n_pg ? table[pg < last_pg ? pg : last_pg] : 0;
    }
    {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int pg = first_pg + tid + u * AT_THREADS;
            tbv[u] = (tid + u * AT_THREADS) < n_pg ? table[pg < last_pg ? pg : last_pg] : 0;
        }
    }
    GRAFT_STAMP(AT_TS_TABLE_REQ);
    // ---- this wavefront's rows: Q' = bf16(Q * scale * log2 e) into AccVGPRs.  Done here, while
    //      the table entries are on their way (Q was requested before them and vector memory
    //      returns in order).
    const float c_log2 = p.scale_log2e;
    WaveRows<MB> w;
    static_for<0, MB>([&](auto rb_) {
        GRAFT_CONST(rb, rb_);
        const float c_row = (r_base + rb * 16 + l16) < p.R ? c_log2 : 0.0f;
        static_for<0, 16>([&](auto k_) {
            GRAFT_CONST(k, k_);
            acc_set_bits<q_reg<MB>(rb, 0) + k>(scale_bf16_pair(qd[rb][k >> 2][k & 3], c_row));
        });
        w.thr[rb] = -INFINITY;
        w.thr_min = -INFINITY;
        w.negm[rb] = floatx4{0.f, 0.f, 0.f, 0.f};
    });
    GRAFT_STAMP(AT_TS_Q_DONE);
    // Everything that came from memory goes to LDS now, so that no load the compiler tracks is
    // outstanding when the first transfers are issued (it counts its own loads only, and a
    // wait for one of them behind the transfers would wait for the transfers as well).
    if (tid < n_mask_words) Ms[tid] = mw0;
    if (tid + AT_THREADS < n_mask_words) Ms[tid + AT_THREADS] = mw1;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (tid + u * AT_THREADS < n_pg) Tb[tid + u * AT_THREADS] = tbv[u];
    for (int k = tid + 4 * AT_THREADS; k < n_pg; k += AT_THREADS) {
        const int pg = first_pg + k;
        Tb[k] = table[pg < last_pg ? pg : last_pg];
    }

    // ---- stage pipeline: stage k (split-local) lives in kv[k & 3]; its loads are issued two
    //      stages ahead.  advance(k) = wait for this wavefront's loads of stage k (the next
    //      stage's stay in flight), meet the others, then start stage k + 2.
    const unsigned kv_base = __builtin_amdgcn_readfirstlane(lds_address(&kv[0][0]));
    const int last_tok = sr.total - 1;
    // A wavefront moves one page per stage: page 4 * stage + wave, 16 token rows of K and of V,
    // four rows (1 KB) per instruction.  Lane (lg, l16) of instruction j fetches 16-byte chunk
    // l16 of row 4 j + lg; which chunk of the row that is (the XOR swizzle) depends on the lane
    // and on j only, so the lane's byte offsets inside a page are loop-invariant.
    unsigned koff[4], voff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 4 * j + lg;                                  // token row within the page
        const int kchunk = l16 ^ row;
        const int vchunk = (((l16 >> 1) ^ (row & 7)) << 1) | (l16 & 1);
        const unsigned row_off = static_cast<unsigned>(row) * static_cast<unsigned>(p.token_stride) * 2u;
        koff[j] = row_off + kchunk * 16;
        voff[j] = row_off + vchunk * 16;
    }
    auto issue_page = [&](int k, int page) {
        const unsigned buf = kv_base + (k & (AT_NBUF - 1)) * AT_STAGE_BYTES + wave_u * 4096;
        const int t_page = (sr.st0 + k) * AT_STAGE + 16 * wave_u;   // first token of this wavefront's page
        const int64_t page_off = (static_cast<int64_t>(page) * p.page_stride + static_cast<int64_t>(g) * p.head_stride) * 2;
        const unsigned char* kp = static_cast<const unsigned char*>(p.k) + page_off;
        const unsigned char* vp = static_cast<const unsigned char*>(p.v) + page_off;
        if (t_page + 15 <= last_tok) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                load_global_to_lds_b128(kp, koff[j], buf + j * 1024);
                load_global_to_lds_b128(vp, voff[j], buf + AT_STAGE * AT_ROW_BYTES + j * 1024);
            }
        } else {
            // the page holding the last token, or a page past it (its table entry then repeats
            // the last page): rows past the end re-read the last token, whose values are finite
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int row = 4 * j + lg;
                int t = t_page + row;
                t = t < last_tok ? t : last_tok;
                const int kchunk = l16 ^ row;
                const int vchunk = (((l16 >> 1) ^ (row & 7)) << 1) | (l16 & 1);
                const unsigned row_off = static_cast<unsigned>(t & 15) * static_cast<unsigned>(p.token_stride) * 2u;
                load_global_to_lds_b128(kp, row_off + kchunk * 16, buf + j * 1024);
                load_global_to_lds_b128(vp, row_off + vchunk * 16, buf + AT_STAGE * AT_ROW_BYTES + j * 1024);
            }
        }
    };
    // The first stage starts here, before the rest of the set-up: its flight time covers the
    // zeroing of the accumulators and the barrier.  The second follows after the zeroing: all
    // workgroups start at the same time, and the memory system delivers their first stages
    // sooner when the requests for the second ones are not queued in between.
    int next_issue = 0;                          // stages are issued in order, each once
    GRAFT_STAMP(AT_TS_TABLE_LDS);
    if (n_st > 0) {
        issue_page(0, __builtin_amdgcn_readfirstlane(first_pages[0]));
        next_issue = 1;
    }
    GRAFT_STAMP(AT_TS_STAGE0_REQ);

    // O^T and the row sums to zero
    static_for<0, MB>([&](auto rb_) {
        GRAFT_CONST(rb, rb_);
        if constexpr (rb >= L_IN_ACC) w.lsum_v = floatx4{0.f, 0.f, 0.f, 0.f};
        else
            static_for<0, 4>([&](auto k_) {
                GRAFT_CONST(k, k_);
                acc_set<l_reg<MB>(rb) + k>(0.0f);
            });
        static_for<0, 32>([&](auto k_) {
            GRAFT_CONST(k, k_);
            acc_set<32 * rb + k>(0.0f);
        });
    });
    // the first pipeline step multiplies zero probabilities with whatever buffer 3 holds: make it zeros
    for (int k = tid; k < AT_STAGE * AT_ROW_BYTES / 16; k += AT_THREADS)
        reinterpret_cast<uint4*>(&kv[AT_NBUF - 1][AT_STAGE * AT_ROW_BYTES])[k] = uint4{0u, 0u, 0u, 0u};
    if (n_st > 1) {
        issue_page(1, __builtin_amdgcn_readfirstlane(first_pages[1]));
        next_issue = 2;
    }
    GRAFT_STAMP(AT_TS_ZEROED);
    lds_barrier();                               // (LDS only: the transfers stay in flight)

    int tb_next = Tb[2 * 4 + wave_u];            // the next stage's table entry is read one stage early
    auto issue_stage = [&](int k) {
        const int page = __builtin_amdgcn_readfirstlane(tb_next);
        const int nxt = (k + 1) * 4 + wave_u;
        tb_next = Tb[nxt < AT_MAX_SPLIT_PAGES ? nxt : AT_MAX_SPLIT_PAGES - 1];
        issue_page(k, page);
    };
    // arrive(k): wait for this wavefront's transfers of stage k (those of stage k + 1 stay in
    // flight) and meet the other wavefronts.  After it stage k can be read and the buffer of
    // stage k + 2 (last read in step k - 1) can be refilled.  advance(k) also starts stage k + 2.
    auto arrive = [&](int k) {
        GRAFT_SPAN_BEGIN();
        if (k + 1 < n_st) GRAFT_WAIT_VMCNT(AT_LOADS_PER_STAGE);
        else GRAFT_WAIT_VMCNT(0);
        GRAFT_SPAN_SPLIT(AT_TS_WAIT_CYCLES);
        lds_barrier();
        GRAFT_SPAN_END(AT_TS_BARRIER_CYCLES);
    };
    // The compute unit's address path takes about 16 cycles per 1 KB transfer, and a wavefront
    // that issues waits for its turn: four wavefronts issuing their 8 transfers at the same
    // time hold each other up for about 500 cycles.  So only the first two issue right after
    // the barrier; the other two issue in the middle of the stage (the target buffer is free
    // during the whole stage), when the first two are computing.
    const bool early_wave = wave_u < 2;
    auto issue_upto = [&](int s) {
        while (next_issue <= s && next_issue < n_st) issue_stage(next_issue++);
    };
    auto advance = [&](int k) {
        arrive(k);
        if (early_wave) issue_upto(k + 2);
    };

    // Only the transfers of stages 0 and 1 are in flight here, and the first advance() waits
    // for stage 0 alone.
    GRAFT_MFMA_SETTLE();

    uintx4 ones_bits;
#pragma unroll
    for (int t = 0; t < 4; ++t) ones_bits[t] = opaque_bits(0x3f803f80u);    // 1.0 in both bf16 halves
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);
    constexpr int K_OFF = 0, V_OFF = AT_STAGE * AT_ROW_BYTES, SUB = AT_SUB * AT_ROW_BYTES;

    // ---- fast loop, software pipelined over 32-token sub-tiles.  Step j: region 1 computes
    //      the exponents of sub-tile j while exponentiating sub-tile j-1 (-> pb); region 2
    //      accumulates P.V and the row sums of sub-tile j-1 while scanning the maxima of
    //      sub-tile j.  Exponents ping-pong between xa (even j) and xb (odd j).  The first
    //      step exponentiates -inf (zero probabilities against the zero-filled buffer 3), the
    //      last (drain) step computes exponents nobody uses.  A row's reference is the row
    //      maximum of the first tile that gives it a finite score and is kept while later
    //      exponents stay below AT_LAZY_LOG2; otherwise the wavefront leaves for the slow loop
    //      below (exact running max, rescaling O with the vector ALUs).
    floatx4 xa[MB][2], xb[MB][2];
    uintx4 pb[MB];
    uintx4 pla = uintx4{0u, 0u, 0u, 0u}, plb = pla;   // late row block's probabilities: even / odd sub-tiles
    float lm[MB];
    const float ninf = __uint_as_float(opaque_bits(0xff800000u));
    bf16x8 ring[4];            // MFMA operands read ahead from LDS (see the regions)
#pragma unroll
    for (int rb = 0; rb < MB; ++rb)
#pragma unroll
        for (int c = 0; c < 2; ++c) xb[rb][c] = floatx4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};

    GRAFT_STAMP(AT_TS_LOOP);
    GRAFT_STAMP_CYCLES(AT_TS_CYCLES_LOOP);
    const int n_sub = 2 * n_st;
    int j = 0;                 // sub-tile whose exponents are pending when the fast loop is left
    bool slow = false;
    for (int k = 0; k <= n_st; ++k) {
        reserve_acc_registers<MB>();    // nothing of the compiler's may live in the hand-managed AccVGPRs here
        const bool live = k < n_st;
        // (transfers of stage k + 2: see advance(); issuing them inside the MFMA regions was
        //  measured slower, a transfer issued while MFMAs are in flight stalls the wavefront)
        if (live) advance(k);
#ifdef GRAFT_ATTN_STAMPS
        if (k == 0) GRAFT_STAMP(AT_TS_STAGE0);
#endif
        const unsigned char* cur = kv[k & (AT_NBUF - 1)];
        const unsigned char* prev = kv[(k - 1) & (AT_NBUF - 1)];
        const int t0 = (sr.st0 + k) * AT_STAGE;
        // even sub-tile of stage k
        // (the late row block's probabilities of the odd sub-tile before, plb, are consumed
        //  while those of this even sub-tile, pla, are produced; and the other way round below)
        region_qk_exp<MB, true>(cur + K_OFF, prev + V_OFF + SUB, w, xa, xb, pb, ring, lane);
        bool grow = region_pv_max<MB, false>(prev + V_OFF + SUB, cur + K_OFF + SUB, w, pb, plb, pla, xa, ones, ninf, lm, ring, lane);
        if (!live) break;
        // (where the exponents change after region 2 has turned the late row block's into
        //  probabilities, those are redone)
        if (__builtin_expect(t0 + AT_SUB > sr.P, 0)) {
            grow = apply_tree_mask<MB>(xa, w, lm, lane, t0, sr.P, sr.n, r_base, p.R, p.g_magic, Ms);
            late_probabilities<MB>(xa, pla);
        }
        if (__builtin_expect(grow, 0)) {
            if (set_references<MB>(lm, w, xa)) { slow = true; j = 2 * k; break; }
            late_probabilities<MB>(xa, pla);
        }
        if (!early_wave) issue_upto(k + 2);
        // odd sub-tile of stage k
        region_qk_exp<MB, false>(cur + K_OFF + SUB, cur + V_OFF, w, xb, xa, pb, ring, lane);
        grow = region_pv_max<MB, true>(cur + V_OFF, nullptr, w, pb, pla, plb, xb, ones, ninf, lm, ring, lane);
        if (__builtin_expect(t0 + 2 * AT_SUB > sr.P, 0)) {
            grow = apply_tree_mask<MB>(xb, w, lm, lane, t0 + AT_SUB, sr.P, sr.n, r_base, p.R, p.g_magic, Ms);
            late_probabilities<MB>(xb, plb);
        }
        if (__builtin_expect(grow, 0)) {
            if (set_references<MB>(lm, w, xb)) {
                slow = true;
                j = 2 * k + 1;
#pragma unroll
                for (int rb = 0; rb < MB; ++rb)
#pragma unroll
                    for (int c = 0; c < 2; ++c) xa[rb][c] = xb[rb][c];
                break;
            }
            late_probabilities<MB>(xb, plb);
        }
    }

    // ---- slow loop (rare): xa holds the exponents of sub-tile j against the old references and
    //      lm their row maxima.  One sub-tile at a time, exact running max.
    if (slow) {
        issue_upto((j >> 1) + 2);       // a late-issuing wavefront may have left before its turn
        while (true) {
            reserve_acc_registers<MB>();
            const unsigned char* cur = kv[(j >> 1) & (AT_NBUF - 1)] + (j & 1) * SUB;
            raise_references<MB>(lm, w, xa);
            exp_only<MB>(xa, pb);
            pv_only<MB>(cur + V_OFF, w, pb, ones, lane);
            ++j;
            if (j >= n_sub) break;
            if ((j & 1) == 0) {
                advance(j >> 1);
                issue_upto((j >> 1) + 2);
            }
            qk_only<MB>(kv[(j >> 1) & (AT_NBUF - 1)] + (j & 1) * SUB + K_OFF, w, xa, lane);
#pragma unroll
            for (int rb = 0; rb < MB; ++rb) {
                float mx = -INFINITY;
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int i = 0; i < 4; ++i) mx = fmaxf(mx, xa[rb][c][i]);
                lm[rb] = mx;
            }
            const int t_sub0 = sr.st0 * AT_STAGE + j * AT_SUB;
            if (t_sub0 + AT_SUB > sr.P)
                apply_tree_mask<MB>(xa, w, lm, lane, t_sub0, sr.P, sr.n, r_base, p.R, p.g_magic, Ms);
#pragma unroll
            for (int rb = 0; rb < MB; ++rb) {
                float mx = lm[rb];
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                lm[rb] = mx;
            }
        }
    }
    GRAFT_MFMA_SETTLE();
    GRAFT_STAMP(AT_TS_LOOP_END);
    GRAFT_STAMP_CYCLES(AT_TS_CYCLES_END);

    if (p.n_splits == 1) {
        // ---- one split: this workgroup holds the whole result of its rows
        // (the lane index goes through an empty asm: otherwise the compiler keeps the row
        //  addressing it computed for the Q loads in registers across the whole loop, registers
        //  that the loop does not have)
        int lane_out = lane;
        asm volatile("" : "+v"(lane_out));
        store_rows<MB>(p, w, b, g, r_base, sr.n, lane_out);
        GRAFT_STAMPS_WRITE(p, n_st);
        return;
    }
    // ---- partial results.  Per row and split: the reference max m (log2 units), the row sum l
    //      and O / l, which is a convex combination of V rows, stored as fp16 after an exact
    //      scaling by a power of two 2^-e that brings the row's largest magnitude into
    //      [0.5, 1): eleven significant bits relative to the row's largest entry, eight times
    //      finer than the bf16 rounding of the final output, at half the bytes of fp32 for the
    //      round trip through memory that the splits cost.  The rows are written as the
    //      accumulator tiles lie in the registers (two 16 x 16 tiles side by side, 16 bytes per
    //      lane), so that every store instruction fills 1 KB of consecutive addresses.
    typedef float floatx2 __attribute__((ext_vector_type(2)));
    typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
    const size_t part = ((static_cast<size_t>(b) * p.Hkv + g) * p.n_splits + split) * p.R_pad;
    static_for<0, MB>([&](auto rb_) {
        GRAFT_CONST(rb, rb_);
        const int r0 = r_base + rb * 16;                          // first row of this 16-row block
        float l;
        if constexpr (rb >= L_IN_ACC) l = w.lsum_v[0];
        else l = acc_get<l_reg<MB>(rb)>();
        const float inv_l = l > 0.f ? 1.0f / l : 0.f;
        float ov[32];
        static_for<0, 32>([&](auto k_) {
            GRAFT_CONST(k, k_);
            ov[k] = acc_get<o_reg(rb, 0) + k>();
        });
        float amax = 0.f;
#pragma unroll
        for (int k = 0; k < 32; ++k) amax = fmaxf(amax, fabsf(ov[k]));
        amax = rows_max_f32(amax);                                // the row's, same in its four lanes
        // biased exponent of the normalised row maximum, kept where 2^e and 2^-e are normal numbers
        // (a zero row, or values at the ends of the fp32 range, keep a scale they can live with)
        int ex = static_cast<int>((__float_as_uint(amax * inv_l) >> 23) & 0xffu);
        ex = ex < 2 ? 126 : (ex > 252 ? 252 : ex);
        const float pow2e = __uint_as_float(static_cast<unsigned>(ex + 1) << 23);      // 2^(ex - 126)
        const float f = inv_l * __uint_as_float(static_cast<unsigned>(253 - ex) << 23);  // 2^-(ex - 126) / l
        unsigned short* op = p.ws_o + (part + r0) * AT_D + 8 * lane;
        static_for<0, 4>([&](auto dp_) {
            GRAFT_CONST(dp, dp_);
            uintx4 t;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                t[k] = __builtin_bit_cast(unsigned, __builtin_convertvector(
                           floatx2{ov[8 * dp + 2 * k] * f, ov[8 * dp + 2 * k + 1] * f}, halfx2));
            *reinterpret_cast<uintx4*>(op + 512 * dp) = t;
        });
        if (lg == 0)
            *reinterpret_cast<floatx4*>(p.ws_ml + (part + r0 + l16) * 4) = floatx4{w.m_ref(rb), l, pow2e, 0.f};
    });
    GRAFT_STAMPS_WRITE(p, n_st);
}

// Merge the splits of two adjacent 16-row x 16-dim output tiles:
// out = sum_s w_s l_s 2^e_s o_s / sum_s w_s l_s with w_s = 2^(m_s - max m), o_s the stored
// fp16 rows.  Lane (l16, lg) owns row l16, dims 4 lg .. +3 of both tiles, exactly the 16 bytes
// it wrote of every split's block, so a split is one 1 KB read per wavefront.  The kernel is
// a chain of memory round trips, not a stream, so a wavefront takes at most U splits (U = 2,
// 4, 8 or 16, the smallest that covers them: registers, and with them the wavefronts in
// flight, go with U) and has all their loads in flight at once (a split without keys has
// weight 0 and a zero block); with more than 16 splits, up to four wavefronts share a tile
// pair and the first of them merges their sums through LDS.
constexpr int CB_MAX_SPLITS = 16;
constexpr int CB_MAX_WAVES = 8;          // per workgroup; the host picks a multiple of the wavefronts per tile pair

template <int U>
__global__ __launch_bounds__(64 * CB_MAX_WAVES) void tree_attn_combine_kernel(AttnParams p, int32_t n_tiles, int32_t wpt) {
    typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
    constexpr int CB_SPLITS = U;
    // (m, den, acc[8]) per lane of the helper wavefronts (only U = 16 has helpers)
    __shared__ float xch[U == CB_MAX_SPLITS ? CB_MAX_WAVES : 1][10][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, lg = lane >> 4;
    const int n_blk = p.R_pad >> 4;                                           // 16-row blocks per (b, g)
    const int tiles_per_wg = (blockDim.x >> 6) / wpt;
    const int tile = static_cast<int>(blockIdx.x) * tiles_per_wg + wave / wpt;   // over B*Hkv*n_blk*4
    const int part_i = wave % wpt;                                            // which CB_SPLITS splits
    const int dp = tile & 3;                                                  // dims 32 dp .. 32 dp + 31
    const int blk = (tile >> 2) % n_blk;
    const int bg = (tile >> 2) / n_blk;                                       // b * Hkv + g
    const int g = bg % p.Hkv, b = bg / p.Hkv;
    const int r = blk * 16 + l16;
    const bool live = tile < n_tiles && r < p.R;                              // not a padding row or tile
    const int ns = p.n_splits;
    const int s0 = part_i * CB_SPLITS;

    float m_run = -INFINITY, den = 0.f;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int n = 0;
    if (live) {
        n = p.n_nodes[b];                                                     // needed only at the end
        const size_t base = static_cast<size_t>(bg) * ns * p.R_pad + blk * 16;     // row index of split 0
        const float* mlrow = p.ws_ml + (base + l16) * 4;
        const size_t ml_stride = static_cast<size_t>(p.R_pad) * 4;
        const unsigned short* otile = p.ws_o + base * AT_D + 512 * dp + 8 * lane;
        const size_t o_stride = static_cast<size_t>(p.R_pad) * AT_D;
        uintx4 ov[CB_SPLITS];
        floatx4 ml[CB_SPLITS];
#pragma unroll
        for (int u = 0; u < CB_SPLITS; ++u) {
            ov[u] = uintx4{0u, 0u, 0u, 0u};
            ml[u] = floatx4{-INFINITY, 0.f, 0.f, 0.f};
            if ((s0 + u) < ns) {                                              // uniform: nothing is read twice
                ov[u] = *reinterpret_cast<const uintx4*>(otile + (s0 + u) * o_stride);
                ml[u] = *reinterpret_cast<const floatx4*>(mlrow + (s0 + u) * ml_stride);
            }
        }
#pragma unroll
        for (int u = 0; u < CB_SPLITS; ++u)
            if ((s0 + u) < ns) m_run = fmaxf(m_run, ml[u][0]);
#pragma unroll
        for (int u = 0; u < CB_SPLITS; ++u) {
            const bool on = (s0 + u) < ns && ml[u][0] > -INFINITY;
            const float wl = on ? __builtin_amdgcn_exp2f(ml[u][0] - m_run) * ml[u][1] : 0.f;
            den += wl;
            const float wu = wl * ml[u][2];
            const halfx8 h = __builtin_bit_cast(halfx8, ov[u]);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += wu * static_cast<float>(h[e]);
        }
    }
    if (U == CB_MAX_SPLITS && wpt > 1) {                                      // uniform over the workgroup
        if (part_i > 0) {
            xch[wave][0][lane] = m_run;
            xch[wave][1][lane] = den;
#pragma unroll
            for (int e = 0; e < 8; ++e) xch[wave][2 + e][lane] = acc[e];
        }
        __syncthreads();
        if (part_i > 0) return;
        float m_all = m_run;
        for (int k = 1; k < wpt; ++k) m_all = fmaxf(m_all, xch[wave + k][0][lane]);
        const float keep = m_run > -INFINITY ? __builtin_amdgcn_exp2f(m_run - m_all) : 0.f;
        den *= keep;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= keep;
        for (int k = 1; k < wpt; ++k) {
            const float mk = xch[wave + k][0][lane];
            const float wk = mk > -INFINITY ? __builtin_amdgcn_exp2f(mk - m_all) : 0.f;
            den += wk * xch[wave + k][1][lane];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += wk * xch[wave + k][2 + e][lane];
        }
    }
    if (!live) return;
    const int i = (r * p.g_magic) >> 16, hl = r - i * p.G;                     // i = r / G
    unsigned short* outp = static_cast<unsigned short*>(p.out) +
        ((static_cast<int64_t>(b) * p.K_max + i) * p.Hq + g * p.G + hl) * AT_D + 32 * dp + 4 * lg;
    if (n < 1 || n > p.K_max) n = 0;
    const float inv = den > 0.f ? 1.0f / den : 0.f;
    unsigned o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        o[k] = float_to_bf16_bits(acc[2 * k] * inv) | (float_to_bf16_bits(acc[2 * k + 1] * inv) << 16);
    if (i >= n) o[0] = o[1] = o[2] = o[3] = 0u;   // rows of absent nodes are zeros whatever their Q rows held
    *reinterpret_cast<uint2*>(outp) = uint2{o[0], o[1]};          // dims 32 dp + 4 lg .. +3
    *reinterpret_cast<uint2*>(outp + 16) = uint2{o[2], o[3]};     // dims 32 dp + 16 + 4 lg .. +3
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
    int mb, n_row_tiles, n_splits, r_pad;
    size_t ws_o_bytes, ws_bytes;
};

// Compute units of the current device (256 when it cannot be asked, e.g. without a GPU).
static int device_compute_units() {
    static int cached = 0;
    if (cached == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cached = n;
        else
            cached = 256;
        (void)hipGetLastError();
    }
    return cached;
}

#ifdef GRAFT_ATTN_STAMPS
static thread_local int g_force_splits = 0, g_force_row_tiles = 0;
#endif

// Launch shape of the MFMA path.  One workgroup per compute unit is resident at a time, so
// the job runs in ceil(workgroups / CUs) rounds, each as long as one workgroup's pass: a
// fixed part (set-up, Q conversion, writing the partial results) plus its stages.  The
// numbers are cycles measured on MI355X (per stage about 680 MB + 1100, fixed about
// 3300 MB + 8000); the plan takes the row tiling (MB <= 5 row blocks per wavefront) and the
// number of splits (<= 64, each with at most AT_MAX_SPLIT_PAGES pages) that make the
// estimate smallest.  It depends on the capacity max_pages, not on the actual lengths.
static AttnPlan make_plan(int32_t B, int32_t K_max, int32_t Hq, int32_t Hkv, int32_t D, int32_t max_pages,
                          int32_t dtype) {
    AttnPlan pl{};
    pl.mfma = (dtype == GRAFT_BF16 && D == AT_D);
    if (!pl.mfma) return pl;
    const int R = K_max * (Hq / Hkv);
    const int rows_per_mb = AT_WAVES * 16;                       // rows a workgroup covers per MB
    const int64_t stages = (static_cast<int64_t>(max_pages) * GRAFT_PAGE_SIZE + AT_STAGE - 1) / AT_STAGE;
    const int64_t min_splits = (stages * (AT_STAGE / GRAFT_PAGE_SIZE) + AT_MAX_SPLIT_PAGES - 1) / AT_MAX_SPLIT_PAGES;
    const int64_t cus = device_compute_units();
    const int rt_min = (R + rows_per_mb * AT_MAX_MB - 1) / (rows_per_mb * AT_MAX_MB);
    const int rt_max = (R + rows_per_mb - 1) / rows_per_mb;
    double best = -1.0;
    for (int rt = rt_min; rt <= rt_max && rt <= rt_min + 3; ++rt) {
        const int mb = (R + rt * rows_per_mb - 1) / (rt * rows_per_mb);
        const double c_stage = 680.0 * mb + 1100.0, c_fixed = 3300.0 * mb + 8000.0;
        const int64_t units = static_cast<int64_t>(B) * Hkv * rt;
        int64_t s_hi = stages < AT_MAX_SPLITS ? stages : AT_MAX_SPLITS;
        if (s_hi < 1) s_hi = 1;
        for (int64_t sp = min_splits < 1 ? 1 : min_splits; sp <= s_hi; ++sp) {
            const int64_t rounds = (units * sp + cus - 1) / cus;
            const int64_t per = (stages + sp - 1) / sp;
            const double cost = rounds * (c_fixed + per * c_stage) + 300.0 * sp;
            if (best < 0.0 || cost < best) {
                best = cost;
                pl.n_row_tiles = rt;
                pl.mb = mb;
                pl.n_splits = static_cast<int>(sp);
            }
        }
    }
#ifdef GRAFT_ATTN_STAMPS
    // timing build: a plan held fixed by the caller (to compare runs that differ in nothing else)
    if (g_force_splits >= (min_splits < 1 ? 1 : min_splits) && g_force_splits <= (stages < AT_MAX_SPLITS ? stages : AT_MAX_SPLITS) &&
        g_force_row_tiles >= rt_min && g_force_row_tiles <= rt_max) {
        pl.n_splits = g_force_splits;
        pl.n_row_tiles = g_force_row_tiles;
        pl.mb = (R + pl.n_row_tiles * rows_per_mb - 1) / (pl.n_row_tiles * rows_per_mb);
    }
#endif
    pl.r_pad = pl.n_row_tiles * pl.mb * rows_per_mb;
    if (pl.n_splits > 1) {                                       // one split needs no workspace and no merge
        const size_t rows = static_cast<size_t>(B) * Hkv * pl.n_splits * pl.r_pad;
        pl.ws_o_bytes = rows * AT_D * sizeof(unsigned short);   // fp16 rows
        pl.ws_bytes = pl.ws_o_bytes + rows * 4 * sizeof(float);
    }
    return pl;
}

static bool attn_shape_ok(int32_t B, int32_t K_max, int32_t Hq, int32_t Hkv, int32_t D, int32_t max_pages) {
    return B >= 1 && B <= 65535 && K_max >= 1 && K_max <= GRAFT_MAX_NODES && Hq >= 1 && Hkv >= 1 &&
           Hkv <= 65535 && Hq % Hkv == 0 && Hq / Hkv <= 16 && (D == 64 || D == 128) && max_pages >= 1 &&
           max_pages <= AT_MAX_SPLITS * AT_MAX_SPLIT_PAGES;    // 64 splits x 4096 pages = 4 Mi tokens
}

// Profiling hook state (per host thread): event pairs attached to the main kernel's dispatch
// (hipExtLaunchKernelGGL: the events then carry the kernel's own begin and end time stamps,
// without the dispatch latency that events recorded around a launch would include).
static thread_local hipEvent_t* g_prof_start = nullptr;
static thread_local hipEvent_t* g_prof_stop = nullptr;
static thread_local int32_t g_prof_n = 0, g_prof_i = 0;
#ifdef GRAFT_ATTN_STAMPS
static thread_local unsigned long long* g_stamps = nullptr;      // device buffer of the timing build
static thread_local size_t g_stamps_bytes = 0;
#endif

template <class Kernel>
static void launch_main(Kernel kernel, dim3 grid, dim3 block, hipStream_t s, const AttnParams& p) {
    if (g_prof_i < g_prof_n) {
        hipExtLaunchKernelGGL(kernel, grid, block, 0, s, g_prof_start[g_prof_i], g_prof_stop[g_prof_i], 0, p);
        ++g_prof_i;
    } else {
        hipLaunchKernelGGL(kernel, grid, block, 0, s, p);
    }
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

#ifdef GRAFT_ATTN_STAMPS
namespace graft {
// Timing build only: what the matrix cores of this chip deliver on a plain stream of independent
// v_mfma_f32_16x16x32_bf16 with operands of a given distribution (the clock under such a load
// depends on what the operands hold).  Every wavefront loads eight operands (64 lanes x 16 bytes
// each, the same for all wavefronts) and runs iters rounds of eight MFMAs on eight accumulators;
// every wavefront records real-time and core-clock counters around its loop (the wavefronts of a
// SIMD do not share the matrix core evenly: the oldest one runs first).
__global__ __launch_bounds__(1024) void mfma_calibration_kernel(const uintx4* __restrict__ operands, float* __restrict__ sink,
                                                               int iters, unsigned long long* __restrict__ stamps) {
    const int lane = threadIdx.x & 63;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        a[j] = __builtin_bit_cast(bf16x8, operands[j * 64 + lane]);
        b[j] = __builtin_bit_cast(bf16x8, operands[(4 + j) * 64 + lane]);
    }
    floatx4 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
    const unsigned long long r0 = __builtin_amdgcn_s_memrealtime(), c0 = __builtin_readcyclecounter();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j & 3], b[(j >> 1) & 3], acc[j], 0, 0, 0);
    }
    const unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) t += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    sink[static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x] = t;
    if (lane == 0) {
        unsigned long long* st = stamps + 4 * (static_cast<size_t>(blockIdx.x) * (blockDim.x >> 6) + (threadIdx.x >> 6));
        st[0] = r0;
        st[1] = r1;
        st[2] = c1 - c0;
        st[3] = 1;
    }
}
}  // namespace graft

// operands: 8 x 64 x 16 bytes; sink: n_workgroups * threads floats; stamps: 4 values per wavefront
// (real-time counter before and after the loop, core-clock cycles of the loop, 1).  threads is 256
// (one wavefront per SIMD), 512, 768 or 1024 (four).  All device memory, all the caller's.
extern "C" int32_t graft_mfma_calibration(const void* operands, float* sink, unsigned long long* stamps,
                                          int32_t n_workgroups, int32_t threads, int32_t iters, void* stream) {
    if (!operands || !sink || !stamps) return GRAFT_ERR_NULL;
    if (n_workgroups < 1 || n_workgroups > (1 << 20) || (threads != 256 && threads != 512 && threads != 768 && threads != 1024) || iters < 1 || iters > (1 << 24))
        return GRAFT_ERR_SHAPE;
    hipLaunchKernelGGL(graft::mfma_calibration_kernel, dim3(n_workgroups), dim3(threads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const graft::uintx4*>(operands), sink, iters, stamps);
    return graft::check_launch();
}

// Timing build only (not part of the library's interface): device buffer that the MFMA kernel of
// this host thread's following graft_tree_attn calls fills with AT_STAMPS 64-bit values per
// workgroup; a call whose grid does not fit the buffer records nothing.  Null switches it off.
extern "C" int32_t graft_attn_stamp_buffer(void* device_buffer, size_t bytes) {
    graft::g_stamps = static_cast<unsigned long long*>(device_buffer);
    graft::g_stamps_bytes = device_buffer ? bytes : 0;
    return GRAFT_OK;
}
extern "C" int32_t graft_attn_stamp_count(void) { return graft::AT_STAMPS; }
// Holds the launch plan of this host thread's following calls (workspace query included) at
// n_splits splits and n_row_tiles row tiles where the shape allows them; zeros give the plan
// back to the cost model.
extern "C" int32_t graft_attn_force_plan(int32_t n_splits, int32_t n_row_tiles) {
    graft::g_force_splits = n_splits;
    graft::g_force_row_tiles = n_row_tiles;
    return GRAFT_OK;
}
#endif

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
        page_stride < 1 || token_stride < D || token_stride >= (1 << 26) || head_stride < D || token_stride % 8 != 0 ||
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
    p.g_magic = (65536 + p.G - 1) / p.G;
    p.scale = scale;
    p.scale_log2e = scale * 1.4426950408889634f;
    hipStream_t s = static_cast<hipStream_t>(stream);

    if (!pl.mfma) {
        dim3 grid(Hq, K_max, B);
        if (dtype == GRAFT_F32) {
            if (D == 64) launch_main(tree_attn_simple_kernel<float, 64>, grid, dim3(SM_THREADS), s, p);
            else launch_main(tree_attn_simple_kernel<float, 128>, grid, dim3(SM_THREADS), s, p);
        } else {
            launch_main(tree_attn_simple_kernel<unsigned short, 64>, grid, dim3(SM_THREADS), s, p);
        }
        return check_launch();
    }

    p.R_pad = pl.r_pad; p.n_splits = pl.n_splits; p.n_row_tiles = pl.n_row_tiles;
    p.ws_o = static_cast<unsigned short*>(workspace);
    p.ws_ml = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + pl.ws_o_bytes);
    const int64_t n_units = static_cast<int64_t>(B) * Hkv * pl.n_splits;
    dim3 grid(static_cast<unsigned>(((n_units + 7) / 8) * 8 * pl.n_row_tiles));
#ifdef GRAFT_ATTN_STAMPS
    p.stamps = static_cast<size_t>(grid.x) * AT_STAMPS * sizeof(unsigned long long) <= g_stamps_bytes ? g_stamps : nullptr;
#endif
    switch (pl.mb) {
        case 1: launch_main(tree_attn_mfma_kernel<1>, grid, dim3(AT_THREADS), s, p); break;
        case 2: launch_main(tree_attn_mfma_kernel<2>, grid, dim3(AT_THREADS), s, p); break;
        case 3: launch_main(tree_attn_mfma_kernel<3>, grid, dim3(AT_THREADS), s, p); break;
        case 4: launch_main(tree_attn_mfma_kernel<4>, grid, dim3(AT_THREADS), s, p); break;
        default: launch_main(tree_attn_mfma_kernel<5>, grid, dim3(AT_THREADS), s, p); break;
    }
    int32_t rc = check_launch();
    if (rc != GRAFT_OK || pl.n_splits == 1) return rc;
    // wpt wavefronts per tile pair (cb_u splits each); as many tile pairs per workgroup as
    // make the workgroups one round (or, capped, a few whole rounds) over the compute units
    const int64_t n_tiles = static_cast<int64_t>(B) * Hkv * (pl.r_pad / 16) * (AT_D / 32);
    if (n_tiles > (1 << 30)) return GRAFT_ERR_SHAPE;
    const int cb_u = pl.n_splits > 8 ? 16 : (pl.n_splits > 4 ? 8 : (pl.n_splits > 2 ? 4 : 2));
    const int wpt = (pl.n_splits + cb_u - 1) / cb_u;                       // 1 .. 4
    const int64_t cus = device_compute_units();
    int64_t tpw = (n_tiles + cus - 1) / cus;                               // tile pairs per workgroup
    const int64_t tpw_max = CB_MAX_WAVES / wpt;
    tpw = tpw < 1 ? 1 : (tpw > tpw_max ? tpw_max : tpw);
    const dim3 cgrid(static_cast<unsigned>((n_tiles + tpw - 1) / tpw)), cblock(static_cast<unsigned>(64 * tpw * wpt));
    const int32_t nt = static_cast<int32_t>(n_tiles);
    switch (cb_u) {
        case 2: hipLaunchKernelGGL(tree_attn_combine_kernel<2>, cgrid, cblock, 0, s, p, nt, wpt); break;
        case 4: hipLaunchKernelGGL(tree_attn_combine_kernel<4>, cgrid, cblock, 0, s, p, nt, wpt); break;
        case 8: hipLaunchKernelGGL(tree_attn_combine_kernel<8>, cgrid, cblock, 0, s, p, nt, wpt); break;
        default: hipLaunchKernelGGL(tree_attn_combine_kernel<16>, cgrid, cblock, 0, s, p, nt, wpt); break;
    }
    return check_launch();
}
