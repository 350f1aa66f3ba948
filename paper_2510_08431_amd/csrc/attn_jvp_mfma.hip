// bf16 matrix-core (MFMA) streaming kernel for attention forward + JVP (paper Alg. 2), head dimension 128 or 64.
//
// One workgroup = 4 wavefronts = 128 query rows; each wavefront owns 32 query rows for the whole
// key/value sweep.  All contractions of Alg. 2's inner loop run on v_mfma_f32_32x32x16_bf16 in the
// TRANSPOSED orientation: S^T = K Q^T, tS^T = K tQ^T + tK Q^T, O^T += V^T P~^T,
// (A+B)^T += tV^T P~^T + V^T H~^T.  In that orientation a lane's MFMA result registers all belong
// to ONE query (column = lane % 32), so
//   * row max / row sums are in-lane reductions plus one exchange between lane l and l^32,
//   * any per-row factor is a per-lane scalar,
//   * P~^T and H~^T feed the next MFMA as its B operand straight from registers (the contraction
//     index - the key position - may be enumerated in any order as long as both operands agree,
//     and V^T is fetched from LDS in exactly the order the result registers happen to hold).
// A and B of Alg. 2 share one accumulator: they carry the same rescale factor and are only added.
//
// Key/value blocks (32 rows x 128 bf16 per tensor) are copied HBM -> LDS with 128-bit direct-to-LDS loads
// into two rings of 4 stages each (K|tK: 16 KiB per stage, V|tV: 16 KiB per stage, 128 KiB in all), K four
// blocks and V three blocks ahead of the block being accumulated, XOR-swizzled so that both the row-wise
// 128-bit reads (K, tK as MFMA A operand) and the transposing 64-bit reads (V, tV) spread over all banks.  (The fp16
// copies of V, tV are stored transposed by the pre-pass, block by block, and are read row-wise like K.)
// Q and tQ fragments stay in registers (in the AGPR half of the file: only MFMA instructions read them); they reach
// them through LDS, and the results leave through LDS, so that every global load and store moves whole rows.
//
// Software pipeline inside a wavefront (there is one wavefront per SIMD, so matrix and vector work
// overlap only through the order of issue, fixed here by scheduling fences): the score MFMAs of block
// b+1 run over block b's softmax arithmetic, the value MFMAs of block b over the fetch of block b+1's
// scores from the accumulation registers; LDS fragments are requested several MFMAs ahead of their use.
//
// Four instantiations differ in how the weights P~ and H~ enter the three value contractions: single bf16
// terms (MODE_BF16), hi + lo bf16 pairs (MODE_BF16_SPLIT), or fp16 terms against power-of-two-scaled fp16
// copies of V and tV that a pre-pass left in the caller's workspace (MODE_F16 with a sampled, fixed exponent
// reference; MODE_F16_ONLINE with a running one, for peaked rows).  On the fp16 path the host launches MODE_F16,
// MODE_F16_ONLINE and MODE_BF16_SPLIT in turn; per-tile flags in the workspace say which of them finishes a tile.
//
// Numerics: bf16 operands, fp32 accumulation; softmax in base 2 with scale*log2(e) folded into one FMA.
// The fast sweep fixes the exponent reference m per row after the first block (all of Alg. 2's rescale
// factors become 1, so the accumulators are only ever written by MFMAs), checks at the end that this was
// safe, and otherwise redoes the tile with Alg. 2's running maximum (bf16 weights) or leaves it to the bf16-pair
// launch (fp16 weights).  H~ = P~ o tS is formed as
// P~ o (tS - ctr) with a per-row constant ctr near rowsum(P o tS): tP does not change when a constant is
// added to a row of tS, and a small |tS - ctr| on the keys that carry the weight keeps the rounding of H~
// from surviving the B - r O cancellation.
#include "launchers.h"
#include "f16_scales.h"
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <type_traits>
#include <utility>

namespace attn_jvp {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int BR = 128, BC = 32, NSTAGE = 4, NTHREADS = 256;
// Geometry for head dimension DH (128 or 64): LDS rows of DH bf16, a tensor's 32-row block, a ring stage (X | tX), the
// two rings.  DH = 128: 256-byte rows, 8 KiB blocks, 128 KiB of LDS; DH = 64: half of each.
template <int DH>
struct Geo {
    static_assert(DH == 128 || DH == 64, "head dimensions built natively");
    static constexpr int ROW_BYTES = DH * 2;
    static constexpr int TENSOR_BYTES = BC * ROW_BYTES;
    static constexpr int KV_STAGE_BYTES = 2 * TENSOR_BYTES;        // K|tK or V|tV
    static constexpr int V_RING_BASE = NSTAGE * KV_STAGE_BYTES;    // K ring first, V ring behind it
    static constexpr int RING_BYTES = 2 * NSTAGE * KV_STAGE_BYTES;
    static constexpr int LDS_BYTES = RING_BYTES + 1024;           // + a KiB where prefetches land that nobody reads
    static constexpr int LANES_PER_ROW = ROW_BYTES / 16;           // 16-byte chunks of a row
    static constexpr int ROWS_PER_COPY = 64 / LANES_PER_ROW;       // rows one direct-to-LDS instruction (64 x 16 B) moves
    static constexpr int COPIES_PER_WAVE = BC / ROWS_PER_COPY / 4; // ... and how many of them a wave issues per tensor block
    // swizzles, applied to the 16-byte chunk index of a row (on the global side of the copies): K, tK for row-wise
    // 128-bit reads, V, tV for the transposing 64-bit reads
    static __device__ __forceinline__ int k_swizzle(int row) { return DH == 128 ? (row & 15) : ((row >> 1) & 7); }
    static __device__ __forceinline__ int v_swizzle(int row) { return DH == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }
};
constexpr int PRESCAN_BLOCKS = NSTAGE;   // key blocks sampled for the fp16 path's exponent reference: the first four, which start the K ring anyway

// nothing may be scheduled across a fence: the instruction order between fences is the issue order
#define FENCE() __builtin_amdgcn_sched_barrier(0)
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)
// Score products of the main loop, with the result in ARITHMETIC registers.  The vector ALU reads every score, and
// the compiler, once a kernel uses accumulation registers at all, places every MFMA result there: 32 single-register
// copies per key block to get the scores out.  Written as assembly, the MFMA delivers them where they are needed.
// The compiler does not see inside: it still orders the LDS reads that produce operand `a` (they are register
// operands of the statement), but it knows nothing of the 11 wait states an 8-pass MFMA needs before the vector ALU
// may read its result; the loop provides them itself (SCORE_RESULTS_LAND and what follows it) after the last score
// product of a block.
// Nor does it know that the result registers are busy until then: a result lane nobody reads later would be handed
// to the next LDS load at once, which the MFMA would then overwrite.  Every lane of s and ts is therefore read
// through a pinned copy after the wait (the hand-over in phase 2), and the build checks the compiled assembly for
// both kinds of accident (lint_mfma_asm.py).
// `b` (a Q or tQ fragment) lives in accumulation registers.  SMFMA0 starts a chain (C = 0), SMFMA continues it.
#define SMFMA0(a, b, c) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(c) : "a"(a), "a"(b))
#define SMFMA(a, b, c) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "a"(a), "a"(b))
// 5 wait states of its own; the other 6 or more of the 11 are the instructions that follow in every instantiation
// (LDS reads, the wait for the copies, the barrier, the first value MFMA) before the first hand-over copy: the
// build's check of the compiled assembly counts them, so a schedule that came out shorter would fail the build.
#define SCORE_RESULTS_LAND() asm volatile("s_nop 4" ::: "memory")
// value contractions: bf16 or fp16 operands (the fragments are carried as raw 128-bit registers)
#define VMFMA(a, b, c)                                                                                          \
    (F16 ? __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0) \
         : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0))

template <int N, typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl<N>(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr) {
    return *reinterpret_cast<__attribute__((address_space(3))) const bf16x8*>((uintptr_t)addr);
}
__device__ __forceinline__ s16x4 lds_read_tr_b64(uint32_t addr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        reinterpret_cast<__attribute__((address_space(3))) s16x4*>((uintptr_t)addr));
}
__device__ __forceinline__ float xhalf_max(float x) {   // max of lane l and lane l^32, in both
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    float d;   // as assembly: fmaxf would first canonicalise both halves (two more instructions)
    asm("v_max_f32 %0, %1, %2" : "=v"(d) : "v"(r[0]), "v"(r[1]));
    return d;
}
__device__ __forceinline__ float xhalf_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint32_t pack_f16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}
// fp32 a * b + c with a taken from one half of a packed fp16 pair (a mixed-precision fused multiply-add: the
// conversion rides along, so reading the weights back AS ROUNDED costs no instruction of its own).  `b` is a
// wave-uniform fp32 value in a scalar register for the *_s forms.
__device__ __forceinline__ float mix_lo(uint32_t h2, float b, float c) {
    float d;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(h2), "v"(b), "v"(c));
    return d;
}
__device__ __forceinline__ float mix_hi(uint32_t h2, float b, float c) {
    float d;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(h2), "v"(b), "v"(c));
    return d;
}
__device__ __forceinline__ float mix_lo_s(uint32_t h2, float b, float c) {
    float d;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(h2), "s"(b), "v"(c));
    return d;
}
__device__ __forceinline__ float mix_hi_s(uint32_t h2, float b, float c) {
    float d;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(h2), "s"(b), "v"(c));
    return d;
}
// element-wise product of two packed fp16 pairs, each rounded to fp16 (denormal results kept)
__device__ __forceinline__ uint32_t pk_mul_f16(uint32_t a, uint32_t b) {
    uint32_t d;
    asm("v_pk_mul_f16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
__device__ __forceinline__ bf16x8 as_bf16x8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    u32x4 u = {a, b, c, d};
    return __builtin_bit_cast(bf16x8, u);
}
__device__ __forceinline__ bf16x8 join_tr(s16x4 a, s16x4 b) {
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7));
}

// 128-bit direct-to-LDS loads (64 lanes x 16 B land at lds_base + 16 * lane; M0 carries lds_base).  Written as
// inline assembly on purpose: the compiler orders LDS reads it cannot prove disjoint behind EVERY outstanding
// direct-to-LDS load it knows of (a full vmcnt(0) wait before each transposing read), which would serialise the
// ring.  Here the kernel does its own accounting: these are the only vector-memory loads in flight during the
// sweep, each wave issues them in program order, and explicit s_waitcnt vmcnt(N) + barriers publish a stage before
// anyone reads it.  M0 is not used by anything else in this kernel.
__device__ __forceinline__ void load_lds_b128(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_base), "v"(gptr) : "memory");
}
// same with a uniform 64-bit base (scalar registers) and a per-lane 32-bit byte offset
__device__ __forceinline__ void load_lds_b128(const void* uniform_base, uint32_t lane_off, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_base), "v"(lane_off), "s"(uniform_base) : "memory");
}
#define ATTN_JVP_LOAD_LDS(g, l) load_lds_b128((g), __builtin_amdgcn_readfirstlane(l))

// Copy one 32-row block of a tensor pair (X, tX) into an LDS stage (X at stage_base, tX TENSOR_BYTES above).
// Each direct-to-LDS instruction moves 64 x 16 B = 4 rows of 256 bytes (8 of 128); the LDS side is linear in the lane
// id, so the swizzle is applied by choosing which 16-byte chunk of the row each lane fetches (Geo::k_swizzle for K, tK:
// row-wise b128 reads; Geo::v_swizzle (VSWZ) for V, tV: transposing b64 reads).  Rows past Lkv re-read the last valid
// row (finite values; their scores are masked to -inf).
template <int DH, bool VSWZ, bool WITH_TANGENT>
__device__ __forceinline__ void issue_pair_clamped(const char* Xh, const char* tXh, long row_stride, int j0, int Lkv,
                                                   uint32_t stage_base, int wave, int lane) {
    using G = Geo<DH>;
#pragma unroll
    for (int i = 0; i < G::COPIES_PER_WAVE; ++i) {
        const int rowblk = wave * G::COPIES_PER_WAVE + i;
        const int row = rowblk * G::ROWS_PER_COPY + lane / G::LANES_PER_ROW;
        const int pc = lane % G::LANES_PER_ROW;
        int grow = j0 + row;
        grow = grow < Lkv ? grow : Lkv - 1;
        const long goff = (long)grow * row_stride + ((pc ^ (VSWZ ? G::v_swizzle(row) : G::k_swizzle(row))) << 4);
        const uint32_t dst = stage_base + rowblk * 1024;
        ATTN_JVP_LOAD_LDS(Xh + goff, dst);
        if constexpr (WITH_TANGENT) ATTN_JVP_LOAD_LDS(tXh + goff, dst + G::TENSOR_BYTES);
    }
}
// The fp16 copies of V and tV that the pre-pass leaves in the workspace are stored TRANSPOSED, key block by key block:
// block j of a head is [DH][32] fp16 (64-byte rows, one per column of V; 32 * DH * 2 bytes = TENSOR_BYTES, the last
// block zero-filled past Lkv), and inside a row the 32 keys stand in the order in which the score MFMAs leave them in
// a lane's result registers: position 16 t2 + 8 g + t holds key 16 t2 + 4 g + (t & 3) + 8 (t >> 2).  The A operand of
// a value MFMA (32 columns of V x 16 keys; lane (c, g) feeds column c, contraction indices 8 g .. 8 g + 7) is then ONE
// 16-byte read, chunk 2 t2 + g of row c, where the row-major bf16 blocks need two transposing 8-byte reads.  A stage
// holds the block as it is in memory, except that 16-byte chunk q of row r sits at chunk q ^ ((r >> 2) & 3): the 16
// lanes that a 128-bit read serves together (consecutive c) then cover all 64 banks.  As with the other copies the
// swizzle is applied on the global side; the byte offset of a lane inside a 1-KiB piece (16 rows) is fixed.
__device__ __forceinline__ uint32_t v16t_lane_offset(int lane) {
    return (uint32_t)(lane >> 2) * 64 + (uint32_t)(((lane & 3) ^ ((lane >> 4) & 3)) << 4);
}
template <int DH, bool WITH_TANGENT>
__device__ __forceinline__ void issue_pair_v16t(const char* Xh, const char* tXh, int blk, int n_blocks, uint32_t stage_base,
                                                int wave, int lane) {
    using G = Geo<DH>;
    const int b = blk < n_blocks ? blk : n_blocks - 1;      // past the end: any finite data (the weights there are zero)
    const uint32_t lo = v16t_lane_offset(lane);
#pragma unroll
    for (int i = 0; i < G::COPIES_PER_WAVE; ++i) {
        const int piece = wave * G::COPIES_PER_WAVE + i;
        const long goff = (long)b * G::TENSOR_BYTES + piece * 1024 + lo;
        const uint32_t dst = stage_base + piece * 1024;
        ATTN_JVP_LOAD_LDS(Xh + goff, dst);
        if constexpr (WITH_TANGENT) ATTN_JVP_LOAD_LDS(tXh + goff, dst + G::TENSOR_BYTES);
    }
}
// Same copy for a block known to lie entirely inside the sequence: the per-lane byte offsets (row and swizzled
// chunk) never change, so they are computed once and only the uniform block base advances.
struct LaneOffsets { uint32_t k[2], v[2]; };
template <int DH, bool V16T>
__device__ __forceinline__ LaneOffsets make_lane_offsets(int wave, int lane, int k_stride, int v_stride) {
    using G = Geo<DH>;
    LaneOffsets o = {};
#pragma unroll
    for (int i = 0; i < G::COPIES_PER_WAVE; ++i) {
        const int row = (wave * G::COPIES_PER_WAVE + i) * G::ROWS_PER_COPY + lane / G::LANES_PER_ROW;
        const int pc = lane % G::LANES_PER_ROW;
        o.k[i] = row * k_stride + ((pc ^ G::k_swizzle(row)) << 4);
        o.v[i] = V16T ? (wave * G::COPIES_PER_WAVE + i) * 1024 + v16t_lane_offset(lane)
                      : row * v_stride + ((pc ^ G::v_swizzle(row)) << 4);
    }
    return o;
}

// MODE selects how the weights P~ and H~ enter the three value contractions:
//   MODE_BF16      one bf16 term each: Alg. 2's 6 matrix products per key block, 8-bit weights;
//   MODE_BF16_SPLIT hi + lo bf16 pairs: 9 products, ~16-bit weights, no extra memory;
//   MODE_F16       one fp16 term each against fp16 copies of V, tV (made by the pre-pass, scaled per head by
//                  powers of two so that nothing over- or underflows): 6 products, 11-bit weights;
//   MODE_F16_ONLINE the same, with a running exponent reference.
// In both fp16 modes the row sums l and r are taken over the weights as rounded to fp16, so what comes out is the
// exact JVP of an attention whose probabilities and centred tangent scores are each off by 2^-11 relative; lse
// carries that rounding of l (at most 2^-11 absolute, far less when many keys share the weight).
//
// ZT ("zero key/value tangents", cross-attention onto a context that does not depend on the differentiated
// variable; template value TAN_QUERY): tK = tV = 0 are not passed at all.  tS = scale tQ K^T and tO = tP V then need 4 of the 6 products, and
// only K and V are streamed; the stage layout stays the same, the tangent halves are simply never written or read.
constexpr int MODE_BF16 = 0, MODE_BF16_SPLIT = 1, MODE_F16 = 2, MODE_F16_ONLINE = 3;
// MODE_F16_ONLINE: fp16 weights as MODE_F16, but the exponent reference follows the running row maximum (Alg. 2's
// rescaling, done lazily) instead of being fixed from a sample: the tier for the tiles MODE_F16 declines or abandons.
constexpr float ONLINE_SLACK = 8.f;   // binades by which a block's maximum may exceed the running one before m moves
// A move costs a wave about 600 instructions (check, new centre, rescale of 128 accumulator registers), and a row of
// the stress workload moves 3.3 times with 4 binades of slack, 2.0 times with 8: about 100 us per tile.  Below this
// many key blocks (5120 keys) the bf16 pairs (9 products, but 11 us of fixed cost per tile) finish a tile as soon as
// the sampled-reference kernel's wasted pre-scan plus the online kernel, so declined tiles go straight to them
// (measured, logit std 8, 16 heads: 4096 keys 0.49 ms pairs / 0.52 online, 6144 keys 1.06 / 0.96, 8192 1.86 / 1.64).
constexpr int ONLINE_MIN_BLOCKS = 160;     // (ATTN_JVP_FLAG_F16_ALWAYS sets this aside)
constexpr int LOCKSTEP_MIN_BLOCKS = 1024;            // tiles of at least 1.3 ms: a wasted wait is at most 8 % of one
constexpr unsigned long long LOCKSTEP_WAIT_TICKS = 10000;   // 100 us of the 100 MHz wall clock
constexpr int LOCKSTEP_MAX_POLLS = 2048;
constexpr int STAGGER_TICKS = 32;   // start offset between neighbouring resident workgroups of an XCD (0.32 us; 31 steps = 10 us)
// The fp16 path costs a pre-pass per call (two small launches, ~20 us plus the conversion of V and tV) and a key sample per
// tile; per key block it is a quarter faster than the bf16 pairs.  It pays from 2048 keys on, and from 256 keys on when
// the call has at least four tiles per compute unit to spread the pre-pass over (measured per tile, 12 tiles per unit:
// 8 key blocks 24.8 against 27.9 us, 16 blocks 33.6 against 37.8 us); below that the bf16 pairs run unless the caller insists.
constexpr int F16_MIN_KEYS = 2048, F16_MIN_KEYS_MANY_TILES = 256, F16_MANY_TILES_PER_CU = 4;

// TAN selects which tangents exist: TAN_ALL (tQ, tK, tV), TAN_QUERY (tQ only: "ZT" below, zero key/value tangents)
// or TAN_NONE (plain attention forward, O and lse only: 2 of the 6 products; same code path, nothing else changes).
constexpr int TAN_NONE = 0, TAN_QUERY = 1, TAN_ALL = 2;

// One query tile (128 rows of one head), start to finish.  `vw` is the tile's index in the launch's list of
// (head, query tile) pairs as a one-workgroup-per-tile launch would number its workgroups; n_tiles their count.
template <int MODE, int TAN, int DH>
__device__ __forceinline__ void attn_jvp_tile(
    const __hip_bfloat16* __restrict__ Q, const __hip_bfloat16* __restrict__ K, const void* __restrict__ V,
    const __hip_bfloat16* __restrict__ tQ, const __hip_bfloat16* __restrict__ tK, const void* __restrict__ tV,
    void* __restrict__ O, void* __restrict__ tO, float* __restrict__ LSE,
    int Lq, int Lkv, float scale, int q_tiles, const float* __restrict__ stats, int* __restrict__ wg_flags,
    int H, int blhd, int out_bf16, int d_out, int out_blhd, int online_min_blocks, int lockstep_slots,
    const int vw, const int n_tiles) {
    using G = Geo<DH>;
    constexpr int D = DH, ROW_BYTES = G::ROW_BYTES, TENSOR_BYTES = G::TENSOR_BYTES, KV_STAGE_BYTES = G::KV_STAGE_BYTES;
    constexpr int V_RING_BASE = G::V_RING_BASE;
    constexpr int NT = DH / 16;             // score steps per key block (16 of the head dimension each)
    constexpr int NDB = DH / 32;            // 32-wide column blocks of the accumulators
    constexpr int NG = 2 * NDB;             // value groups per key block: (half of the block's keys) x (column block)
    constexpr bool SPLIT = MODE == MODE_BF16_SPLIT;
    constexpr bool F16 = MODE == MODE_F16 || MODE == MODE_F16_ONLINE;   // fp16 weights and value operands
    constexpr bool PRESCAN = MODE == MODE_F16;                          // fixed reference from a key sample
    constexpr bool ONLINE = MODE == MODE_F16_ONLINE;                    // reference follows the running maximum
    constexpr bool ZT = TAN != TAN_ALL;          // no key/value tangents
    constexpr bool PRIMAL = TAN == TAN_NONE;     // no tangents at all
    // Hand-over between the launches of the fp16 path, which follow each other on one stream: the fp16 kernel
    // writes wg_flags[workgroup] = 1 for every tile it declines or abandons (0 otherwise) and stores nothing for
    // those; the online fp16 kernel works on exactly the tiles flagged 1 and sets 3 (done), or 2 if it has to
    // abandon one itself; the bf16-pair kernel, given the flags, works on exactly the tiles flagged 2.
    if constexpr (ONLINE) {
        if (wg_flags[vw] != 1) return;
        // Lock-step start of the tiles that share an XCD's L2 (lockstep_slots = workgroups an XCD holds at a time, 0 =
        // off).  The tiles of this tier take different times (moves of the reference), and over many rounds of
        // tiles the workgroups of an XCD drift apart until each streams K and V from memory on its own.  Each
        // working workgroup takes a ticket of its XCD and waits until its round of lockstep_slots tickets is
        // complete, i.e. until the neighbours it will share its key stream with have started too.  The wait is
        // bounded twice (wall clock and iteration count), so it ends whatever the other workgroups do: the last,
        // partial round of a launch simply waits out the limit once.
        if (lockstep_slots > 0) {
            if (threadIdx.x == 0) {
                int* ticket = wg_flags + ((n_tiles * 4 + 255) & ~255) / 4 + (vw & 7) * 16;
                const int mine = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const int full = (mine / lockstep_slots + 1) * lockstep_slots;
                const unsigned long long t0 = wall_clock64();
                for (int it = 0; it < LOCKSTEP_MAX_POLLS; ++it) {
                    if (__hip_atomic_load(ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= full) break;
                    if (wall_clock64() - t0 > LOCKSTEP_WAIT_TICKS) break;
                    __builtin_amdgcn_s_sleep(32);
                }
            }
            __syncthreads();
        }
    } else if constexpr (!F16) {
        if (wg_flags != nullptr && wg_flags[vw] != 2) return;
    }
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;

    // (an opaque copy of the thread index: with resident workgroups this function is the body of a loop over tiles, and
    // everything derived from the lane id would otherwise be hoisted out of that loop and kept in registers across
    // tiles, on top of what a tile needs anyway)
    unsigned tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 31;          // query column of this lane in every MFMA result
    const int g = lane >> 5;          // which half of the contraction index this lane feeds
    // Workgroups are dealt to the 8 XCDs round-robin by index.  Give XCD x the x-th contiguous eighth of the
    // (head, query tile) list, so that neighbouring tiles, whose output rows are neighbours in memory, are written
    // through the same L2: measured, this halves the kernel's HBM write traffic (0.81 -> 0.41 GB on the video
    // workload, the algorithmic 0.40) at unchanged run time.  (It does not reduce the K/V fetch traffic: a head's
    // K and V do not fit an L2, so every round of 32 co-resident workgroups streams them again either way.)
    const int n_wg = n_tiles;
    const int bid = (n_wg & 7) == 0 ? (vw & 7) * (n_wg >> 3) + (vw >> 3) : vw;
    const long bh = bid / q_tiles;
    const int q0 = (bid % q_tiles) * BR + wave * 32;

    // Memory layout of the caller's tensors: [B,H,L,d] (rows of a head contiguous) or [B,L,H,d] (rows of a head H*d
    // apart).  Element offset of row r of head (b, h): head_base + r * row_elems.  The fp16 copies of V, tV in the
    // workspace are always [B,H,L,d].
    const int row_elems = blhd ? H * D : D;
    const long bidx = bh / H, hidx = bh % H;
    const long q_base = blhd ? (bidx * Lq * H + hidx) * D : bh * (long)Lq * D;
    const long kv_base = blhd ? (bidx * Lkv * H + hidx) * D : bh * (long)Lkv * D;
    const int k_stride = row_elems * 2;                                  // bytes between key rows
    const int n_blocks = (Lkv + BC - 1) / BC;
    const int v_stride = F16 ? ROW_BYTES : k_stride;                     // (fp16 copies: whole transposed blocks, see issue_pair_v16t)
    const long v_base = F16 ? bh * (long)n_blocks * (BC * D) : kv_base;
    const char* Kh = reinterpret_cast<const char*>(K) + kv_base * 2;
    const char* tKh = reinterpret_cast<const char*>(tK) + kv_base * 2;
    const char* Vh = static_cast<const char*>(V) + v_base * 2;           // bf16, or the fp16 copies
    const char* tVh = static_cast<const char*>(tV) + v_base * 2;

    // block x: K|tK in K-ring stage x & 3, V|tV in V-ring stage x & 3
    auto copy_k = [&](int blk) __attribute__((always_inline)) {
        issue_pair_clamped<DH, false, !ZT>(Kh, tKh, k_stride, blk * BC, Lkv, lds0 + (uint32_t)(blk & 3) * KV_STAGE_BYTES, wave, lane);
    };
    auto copy_v = [&](int blk) __attribute__((always_inline)) {
        const uint32_t stage = lds0 + V_RING_BASE + (uint32_t)(blk & 3) * KV_STAGE_BYTES;
        if constexpr (F16) issue_pair_v16t<DH, !ZT>(Vh, tVh, blk, n_blocks, stage, wave, lane);
        else issue_pair_clamped<DH, true, !ZT>(Vh, tVh, v_stride, blk * BC, Lkv, stage, wave, lane);
    };
    // Tile start.  One round trip to memory brings in K(0..3) (K ring, all four stages) and the tile's 128 rows of Q and
    // tQ, which are staged through the V ring's area (64 KiB, not needed yet) so that they, too, come as whole
    // rows: fetched straight into the MFMA operand layout, every load instruction of a wave would touch 32 rows with
    // 32 bytes each, and the tile start took 4.7 us instead of one memory latency.  Staged like four 32-row K blocks
    // per tensor (same swizzle), wave w then reads its rows (block w) with the K fragment addresses.  V(0..2) are
    // requested once everyone has read its fragments (rows past the end are clamped, so all copies are unconditional).
    constexpr uint32_t Q_STAGE = V_RING_BASE, TQ_STAGE = V_RING_BASE + 4 * TENSOR_BYTES;
    const int qrow = q0 + c;
    {
        const char* Qh = reinterpret_cast<const char*>(Q) + q_base * 2;
        const char* tQh = reinterpret_cast<const char*>(tQ) + q_base * 2;
        const int tile_row0 = q0 - wave * 32;
        copy_k(0); copy_k(1); copy_k(2); copy_k(3);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < G::COPIES_PER_WAVE; ++i) {
                const int rowblk = wave * G::COPIES_PER_WAVE + i;
                const int row = rowblk * G::ROWS_PER_COPY + lane / G::LANES_PER_ROW;
                const int pc = lane % G::LANES_PER_ROW;
                int grow = tile_row0 + 32 * j + row;
                grow = grow < Lq ? grow : Lq - 1;
                const long goff = (long)grow * k_stride + ((pc ^ G::k_swizzle(row)) << 4);
                ATTN_JVP_LOAD_LDS(Qh + goff, lds0 + Q_STAGE + (uint32_t)j * TENSOR_BYTES + rowblk * 1024);
                if constexpr (!PRIMAL) ATTN_JVP_LOAD_LDS(tQh + goff, lds0 + TQ_STAGE + (uint32_t)j * TENSOR_BYTES + rowblk * 1024);
            }
    }
    auto start_v_ring = [&]() __attribute__((always_inline)) { copy_v(0); copy_v(1); copy_v(2); };

    // per-lane LDS read addresses within stage 0 of the K ring / of the V ring; stage and tensor offsets are
    // 16-bit immediates of the read instructions
    uint32_t kaddr0[NT], vaddr0[F16 ? 2 : NDB];
#pragma unroll
    for (int t = 0; t < NT; ++t) kaddr0[t] = lds0 + c * ROW_BYTES + (((2 * t + g) ^ G::k_swizzle(c)) << 4);
    if constexpr (F16) {
        // transposed fp16 blocks: chunk 2 t2 + g of row c (of column block db: + 32 db rows, an immediate), swizzled
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) vaddr0[t2] = lds0 + V_RING_BASE + c * 64 + (((2 * t2 + g) ^ ((c >> 2) & 3)) << 4);
    } else {
        // transposing read: the lane fetches 4 consecutive columns, 32 db + 16 hb + 4 (i & 3) .. +3, of key row
        // 4 g + (i >> 2) (+ 8 for the second read of a fragment, + 16 for the block's second half); the row's 64-byte
        // segments (32 columns) are swizzled by v_swizzle(row) >> 2, which those row offsets do not change
        const int i = lane & 15, hb = (lane >> 4) & 1;
        const int vrow = 4 * g + (i >> 2);
        const uint32_t rowpart = vrow * ROW_BYTES + (2 * hb + ((i & 3) >> 1)) * 16 + 8 * (i & 1);
#pragma unroll
        for (int db = 0; db < NDB; ++db) vaddr0[db] = lds0 + V_RING_BASE + rowpart + ((db ^ (G::v_swizzle(vrow) >> 2)) << 6);
    }

    // Q^T / tQ^T as MFMA B operand: lane (c, g) holds row q0+c, elements 16t + 8g .. +7
    bf16x8 qf[NT], tqf[NT];
    {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // K(0..3), Q and tQ are in
        __syncthreads();
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            qf[t] = lds_read_b128(kaddr0[t] + Q_STAGE + (uint32_t)wave * TENSOR_BYTES);
            if constexpr (!PRIMAL) tqf[t] = lds_read_b128(kaddr0[t] + TQ_STAGE + (uint32_t)wave * TENSOR_BYTES);
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {   // keep them in accumulation registers: only MFMAs read them
            asm volatile("" : "+a"(qf[t]));
            if constexpr (!PRIMAL) asm volatile("" : "+a"(tqf[t]));
        }
        __syncthreads();                                    // everyone has its fragments: the V ring's area is free
        if constexpr (!PRESCAN) start_v_ring();             // (the sampled-reference kernel first decides whether it takes the tile)
    }

    f32x16 accO[NDB], accAB[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) { accO[db][e] = 0.f; accAB[db][e] = 0.f; }

    const float c2 = scale * 1.4426950408889634f;   // scores -> base-2 exponent
    float m;                  // per-row exponent reference, fixed for the fast sweep
    float l_part2 = 0.f, r_part2 = 0.f;
    float l_part, r_part;     // this lane's share of rowsum(P~) and of gH * rowsum(H~), H~ = P~ o (tS - ctr)
    // fp16 path: the O accumulator holds 2^-eV O~, the A+B accumulator 2^-eA (A+B), H~ is formed times gH = 2^(eV-eA)
    float gO = 1.f, gAB = 1.f, gH = 1.f;
    if constexpr (F16) {
        const F16Scales sc = f16_scales(stats + bh * 8, scale);
        gO = ldexpf(1.f, sc.eV);
        gAB = ldexpf(1.f, sc.eA);
        gH = ldexpf(1.f, sc.eV - sc.eA);
    }
    const float scale_h = scale * gH;
    float ctr_h;              // gH * ctr, ctr = per-row centre subtracted from the scaled tangent scores

    uint32_t wp[8], wh[8];                              // P~^T, H~^T as packed bf16 pairs, result-register order
    uint32_t wpl[SPLIT ? 8 : 1], whl[SPLIT ? 8 : 1];    // their low-order parts

    // Scores (raw, fp32) of two key blocks at a time, in ordinary registers: the score products of block b+1 write one
    // pair of buffers while the softmax of block b still reads the other, so the scores are used where the matrix
    // pipe delivers them and nothing is copied (block x lives in buffer x & 1).
    f32x16 sbuf0, sbuf1, tsbuf0, tsbuf1;
    auto SV = [&](auto Bc) __attribute__((always_inline)) -> f32x16& { if constexpr (decltype(Bc)::value == 0) return sbuf0; else return sbuf1; };
    auto TSV = [&](auto Bc) __attribute__((always_inline)) -> f32x16& { if constexpr (decltype(Bc)::value == 0) return tsbuf0; else return tsbuf1; };
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;

    // Softmax arithmetic of one pair of score elements (2j, 2j+1) -> packed weights, cut into five parts of at most
    // six vector instructions so that the pipelined sweep can put one part behind each MFMA:
    //   bf16 weights: 0: P~ = exp2(S c2 - m)   1: H~ = P~ (tS scale - ctr)   2: row sums   3: pack P~ (hi, lo)
    //                 4: pack H~ (hi, lo)
    //   fp16 weights: 0: P~ = exp2(S c2 - m)   1: pack P~16, pack u16 = tS scale - ctr   2, 3: -
    //                 4: H~16 = P~16 x u16 (one packed multiply), l += P~16, r += H~16
    f32x4 sp0a, sp1a;   // (the exponentials of pairs 0-3 are taken ahead of the rest of their softmax: one set per pair)
    float sh0, sh1;
    uint32_t uh;        // fp16 weights: the pair's centred, scaled tangent scores as packed fp16
    float one = 1.f;   // kept in a scalar register as an opaque operand of the mixed multiply-adds
    asm volatile("" : "+s"(one));
    auto softmax_part = [&](auto J, auto PART, auto Bc) __attribute__((always_inline)) {
        constexpr int j = decltype(J)::value, e = 2 * j, part = decltype(PART)::value;
        const f32x16& sv = SV(Bc);
        const f32x16& tsv = TSV(Bc);
        constexpr int jj = j & 3;
        if constexpr (part == 0) {
            sp0a[jj] = __builtin_amdgcn_exp2f(fmaf(sv[e], c2, -m));
            sp1a[jj] = __builtin_amdgcn_exp2f(fmaf(sv[e + 1], c2, -m));
            // fp16 weights: everything downstream (l, H~, r) is formed from P~ AS ROUNDED to fp16, and r from H~ as
            // rounded, so that the result is the exact JVP of a softmax whose probabilities and centred tangent
            // scores are off by 2^-11 relative.  With unrounded values in l, r and H~ but rounded ones in the
            // products, B - (r/l) O would keep the rounding of a dominant key's weight times its tangent score,
            // which is not small on peaked rows.  The mixed-precision multiply-adds read the packed halves
            // directly, so this costs no instruction.
        } else if constexpr (part == 1) {
            if constexpr (F16) wp[j] = pack_f16(sp0a[jj], sp1a[jj]);   // behind the scale-and-centre of part 1: the exponentials have landed
            if constexpr (!PRIMAL) {
                if constexpr (F16) {
                    // H~16 = P~16 (x) u16, u = tS scale - ctr rounded to fp16 first: one packed multiply for the pair
                    uh = pack_f16(fmaf(tsv[e], scale_h, -ctr_h), fmaf(tsv[e + 1], scale_h, -ctr_h));
                } else {
                    sh0 = sp0a[jj] * fmaf(tsv[e], scale_h, -ctr_h);
                    sh1 = sp1a[jj] * fmaf(tsv[e + 1], scale_h, -ctr_h);
                }
            }
        } else if constexpr (part == 2) {
            if constexpr (F16) {
                if constexpr (PRIMAL) {
                    l_part = mix_lo_s(wp[j], one, l_part);      // two chains: low halves, high halves
                    l_part2 = mix_hi_s(wp[j], one, l_part2);
                }   // (with tangents: in part 4, between the packed product and the sums that read it)
            } else {
                l_part += sp0a[jj] + sp1a[jj];
                if constexpr (!PRIMAL) r_part += sh0 + sh1;
            }
        } else if constexpr (part == 3) {
            if constexpr (!F16) {
                const uint32_t ph = pack_bf16(sp0a[jj], sp1a[jj]);
                wp[j] = ph;
                if constexpr (SPLIT)   // lo = x - hi (exact in fp32), rounded to bf16
                    wpl[j] = pack_bf16(sp0a[jj] - __uint_as_float(ph << 16), sp1a[jj] - __uint_as_float(ph & 0xffff0000u));
            }
        } else if constexpr (part == 4 && !PRIMAL) {
            uint32_t hh;
            if constexpr (F16) {
                hh = pk_mul_f16(wp[j], uh);
                l_part = mix_lo_s(wp[j], one, l_part);      // two chains: low halves, high halves
                l_part2 = mix_hi_s(wp[j], one, l_part2);
            } else {
                hh = pack_bf16(sh0, sh1);
            }
            wh[j] = hh;
            if constexpr (SPLIT)
                whl[j] = pack_bf16(sh0 - __uint_as_float(hh << 16), sh1 - __uint_as_float(hh & 0xffff0000u));
            if constexpr (F16) {
                r_part = mix_lo_s(hh, one, r_part);
                r_part2 = mix_hi_s(hh, one, r_part2);
            }
        }
    };
    auto softmax_pair = [&](auto J, auto Bc) __attribute__((always_inline)) {
        static_for<5>([&](auto PART) { softmax_part(J, PART, Bc); });
    };
    // the part(s) that go behind MFMA number `slot` of the `n_slots` a pair has to itself
    auto softmax_slot = [&](auto J, auto SLOT, auto NSLOTS, auto Bc) __attribute__((always_inline)) {
        constexpr int slot = decltype(SLOT)::value, n_slots = decltype(NSLOTS)::value;
        if constexpr (n_slots >= 5) {
            if constexpr (slot < 5) softmax_part(J, SLOT, Bc);
        } else if constexpr (n_slots == 4) {
            if constexpr (slot == 0) softmax_part(J, std::integral_constant<int, 0>{}, Bc);
            if constexpr (slot == 1) { softmax_part(J, std::integral_constant<int, 1>{}, Bc); softmax_part(J, std::integral_constant<int, 2>{}, Bc); }
            if constexpr (slot == 2) softmax_part(J, std::integral_constant<int, 3>{}, Bc);
            if constexpr (slot == 3) softmax_part(J, std::integral_constant<int, 4>{}, Bc);
        } else if constexpr (n_slots == 3) {
            if constexpr (slot == 0) softmax_part(J, std::integral_constant<int, 0>{}, Bc);
            if constexpr (slot == 1) { softmax_part(J, std::integral_constant<int, 1>{}, Bc); softmax_part(J, std::integral_constant<int, 3>{}, Bc); }
            if constexpr (slot == 2) { softmax_part(J, std::integral_constant<int, 2>{}, Bc); softmax_part(J, std::integral_constant<int, 4>{}, Bc); }
        } else if constexpr (n_slots == 1) {
            if constexpr (slot == 0) static_for<5>([&](auto PART) { softmax_part(J, PART, Bc); });
        } else {
            static_assert(n_slots == 2, "a pair gets 1, 2, 3, 4 or at least 5 MFMA slots");
            if constexpr (slot == 0) { softmax_part(J, std::integral_constant<int, 0>{}, Bc); softmax_part(J, std::integral_constant<int, 1>{}, Bc); }
            if constexpr (slot == 1) {
                softmax_part(J, std::integral_constant<int, 2>{}, Bc); softmax_part(J, std::integral_constant<int, 3>{}, Bc);
                softmax_part(J, std::integral_constant<int, 4>{}, Bc);
            }
        }
    };

    // parts 1-4 of a pair whose exponentials (part 0) were taken earlier, spread over the `n_slots` MFMAs of one value group
    auto softmax_late_slot = [&](auto J, auto SLOT, auto NSLOTS, auto Bc) __attribute__((always_inline)) {
        constexpr int slot = decltype(SLOT)::value, n_slots = decltype(NSLOTS)::value;
        using P1 = std::integral_constant<int, 1>;
        using P2 = std::integral_constant<int, 2>;
        using P3 = std::integral_constant<int, 3>;
        using P4 = std::integral_constant<int, 4>;
        if constexpr (n_slots >= 4) {
            if constexpr (slot < 4) softmax_part(J, std::integral_constant<int, slot + 1>{}, Bc);
        } else if constexpr (n_slots == 3) {
            if constexpr (slot == 0) softmax_part(J, P1{}, Bc);
            if constexpr (slot == 1) { softmax_part(J, P2{}, Bc); softmax_part(J, P3{}, Bc); }
            if constexpr (slot == 2) softmax_part(J, P4{}, Bc);
        } else if constexpr (n_slots == 2) {
            if constexpr (slot == 0) { softmax_part(J, P1{}, Bc); softmax_part(J, P2{}, Bc); }
            if constexpr (slot == 1) { softmax_part(J, P3{}, Bc); softmax_part(J, P4{}, Bc); }
        } else {
            static_assert(n_slots == 1, "a value group has 1, 2, 3 or at least 4 MFMAs");
            if constexpr (slot == 0) { softmax_part(J, P1{}, Bc); softmax_part(J, P2{}, Bc); softmax_part(J, P3{}, Bc); softmax_part(J, P4{}, Bc); }
        }
    };

    auto mask_scores = [&](int blk, auto Bc) __attribute__((always_inline)) {   // keys past Lkv: P~ = 0, tangent score 0
        f32x16& sv = SV(Bc);
        f32x16& tsv = TSV(Bc);
        const int jbase = blk * BC + 4 * g;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int jj = jbase + 8 * (e >> 2) + (e & 3);
            if (jj >= Lkv) { sv[e] = -INFINITY; tsv[e] = 0.f; }
        }
    };
    auto plain_scores = [&](uint32_t stage_off, auto Bc) __attribute__((always_inline)) {   // unscheduled: prologue, safe sweep
        f32x16 s, ts;
#pragma unroll
        for (int e = 0; e < 16; ++e) { s[e] = 0.f; ts[e] = 0.f; }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const bf16x8 kf = lds_read_b128(kaddr0[t] + stage_off);
            s = MFMA(kf, qf[t], s);
            if constexpr (!PRIMAL) ts = MFMA(kf, tqf[t], ts);
            if constexpr (!ZT) ts = MFMA(lds_read_b128(kaddr0[t] + stage_off + TENSOR_BYTES), qf[t], ts);
        }
        SV(Bc) = s;
        TSV(Bc) = ts;
        // (in arithmetic registers from here on: the pipelined sweep carries these buffers round its loop, and a value
        // that enters the loop in accumulation registers is kept there, with copies in and out at every turn)
        asm volatile("" : "+v"(SV(Bc)), "+v"(TSV(Bc)));
    };
    // Row maximum of the 16 scores a lane holds, times c2.  Written with the three-operand maximum as assembly: the
    // compiler's own fmaxf first canonicalises every operand it did not produce itself (one extra v_max per score).
    auto row_max = [&](auto Bc) __attribute__((always_inline)) -> float {
        const f32x16& sv = SV(Bc);
        auto max3 = [](float a, float b, float c) __attribute__((always_inline)) {
            float d;
            asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
            return d;
        };
        const float t0 = max3(sv[0], sv[1], sv[2]), t1 = max3(sv[3], sv[4], sv[5]), t2_ = max3(sv[6], sv[7], sv[8]);
        const float t3 = max3(sv[9], sv[10], sv[11]), t4 = max3(sv[12], sv[13], sv[14]);
        const float u0 = max3(t0, t1, t2_), u1 = max3(t3, t4, sv[15]);
        return xhalf_max(max3(u0, u1, u1)) * c2;
    };
    // A operand of a value MFMA (32 columns of V x 16 keys): one 128-bit read of a transposed fp16 block, or two
    // transposing 64-bit reads of a row-major bf16 block (rows 8 apart)
    auto read_v_fragment = [&](uint32_t a) __attribute__((always_inline)) -> bf16x8 {
        if constexpr (F16) return lds_read_b128(a);
        else return join_tr(lds_read_tr_b64(a), lds_read_tr_b64(a + 8 * ROW_BYTES));
    };
    auto plain_values = [&](uint32_t stage_off) __attribute__((always_inline)) {   // unscheduled: safe sweep
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
            const bf16x8 pb = as_bf16x8(wp[4 * t2], wp[4 * t2 + 1], wp[4 * t2 + 2], wp[4 * t2 + 3]);
            bf16x8 hb8 = pb;
            if constexpr (!PRIMAL) hb8 = as_bf16x8(wh[4 * t2], wh[4 * t2 + 1], wh[4 * t2 + 2], wh[4 * t2 + 3]);
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                const uint32_t a = F16 ? vaddr0[t2] + stage_off + db * (32 * 64) : vaddr0[db] + stage_off + t2 * 16 * ROW_BYTES;
                const bf16x8 vf = read_v_fragment(a);
                bf16x8 tvf = vf;   // placeholder when there is no tV
                if constexpr (!ZT) tvf = read_v_fragment(a + TENSOR_BYTES);
                accO[db] = VMFMA(vf, pb, accO[db]);
                if constexpr (!ZT) accAB[db] = VMFMA(tvf, pb, accAB[db]);
                if constexpr (!PRIMAL) accAB[db] = VMFMA(vf, hb8, accAB[db]);
                if constexpr (SPLIT) {
                    const bf16x8 pl8 = as_bf16x8(wpl[4 * t2], wpl[4 * t2 + 1], wpl[4 * t2 + 2], wpl[4 * t2 + 3]);
                    accO[db] = VMFMA(vf, pl8, accO[db]);
                    if constexpr (!ZT) accAB[db] = VMFMA(tvf, pl8, accAB[db]);
                    if constexpr (!PRIMAL) {
                        const bf16x8 hl8 = as_bf16x8(whl[4 * t2], whl[4 * t2 + 1], whl[4 * t2 + 2], whl[4 * t2 + 3]);
                        accAB[db] = VMFMA(vf, hl8, accAB[db]);
                    }
                }
            }
        }
    };

    // ================================ fast sweep ================================
    // Alg. 2 with the running maximum replaced by a per-row exponent reference m fixed before the sweep; Alg. 2's
    // rescale factors are then all exp(0) = 1 and no accumulator is ever rewritten.  The sweep verifies at its end
    // that exp2(S c2 - m) stayed representable (see the check below).  ctr is fixed to block 0's value of
    // rowsum(P o tS).  The loop body is straight-line code.
    //   bf16 weights: m = block-0 maximum + 40 binades; fine while later scores exceed it by < ~100 binades.
    //   fp16 weights: H~ (up to 2^8 P~ after scaling) must stay below 2^16, so P~ below 2^7, and the keys that carry
    //   the sum must stay inside the fp16 range below that (weights under 2^-25 round to zero), so m has to be close
    //   to the true maximum: m = maximum over the first four key blocks (128 keys, which are in the K ring anyway)
    //   + (2.7 sigma - 6) binades, sigma = the row's sampled score spread: the true maximum, which rarely exceeds
    //   the sampled one by more than 2.7 sigma, then gets a weight of at most 2^6.  (If the first keys are not
    //   typical of the rest, the end-of-sweep checks notice and the tile is redone with a running reference.)
    //   fp16 weights, online: m = running maximum + 1 binade, moved (with a rescale of everything accumulated)
    //   when a block's maximum exceeds the running one by more than ONLINE_SLACK: weights stay below 2^7, and
    //   keys more than 23 binades (16 nats) below the running maximum drop out of the fp16 range.
    constexpr float REF_HEADROOM = PRESCAN ? 6.f : ONLINE ? 1.f : 40.f;
    constexpr float F16_MAX_GAP = 10.f;
    float headroom = REF_HEADROOM;
    float m_scan = -INFINITY;
    if constexpr (PRESCAN) {
        float sum1 = 0.f, sum2 = 0.f;   // first and second moment of the sampled raw scores (full blocks only)
        int n_stat = 0;
        // the sample: K(0..3), which sit in the four stages of the K ring
        const int ns = n_blocks < PRESCAN_BLOCKS ? n_blocks : PRESCAN_BLOCKS;
        // Two samples per step, software-pipelined: the sixteen fragment reads of a pair go out together, and the
        // MFMAs of pair p+1 run while the vector unit works through the statistics of pair p.
        auto scan_one = [&](const float (&x)[16], int blk) __attribute__((always_inline)) {
            f32x16& sv = SV(B1{});      // (as scratch: the sweep has not started)
            f32x16& tsv = TSV(B1{});
#pragma unroll
            for (int e = 0; e < 16; ++e) { sv[e] = x[e]; tsv[e] = 0.f; }
            if ((blk + 1) * BC > Lkv) {
                mask_scores(blk, B1{});
            } else {
                float a1 = 0.f, a2 = 0.f;
#pragma unroll
                for (int e = 0; e < 16; ++e) { a1 += sv[e]; a2 = fmaf(sv[e], sv[e], a2); }
                sum1 += a1; sum2 += a2; n_stat += BC;
            }
            float t0 = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
            float t1 = fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7]));
            float t2_ = fmaxf(fmaxf(sv[8], sv[9]), fmaxf(sv[10], sv[11]));
            float t3 = fmaxf(fmaxf(sv[12], sv[13]), fmaxf(sv[14], sv[15]));
            m_scan = fmaxf(m_scan, fmaxf(fmaxf(t0, t1), fmaxf(t2_, t3)));   // this lane's half of the row, raw
        };
        f32x16 s0, s1;
        auto scores_of_pair = [&](int i) __attribute__((always_inline)) {   // samples i and i+1 (or i twice)
            const uint32_t off0 = (uint32_t)i * KV_STAGE_BYTES, off1 = (uint32_t)(i + 1 < ns ? i + 1 : i) * KV_STAGE_BYTES;
            bf16x8 ka[NT], kb[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) { ka[t] = lds_read_b128(kaddr0[t] + off0); kb[t] = lds_read_b128(kaddr0[t] + off1); }
            FENCE();   // all sixteen reads in flight before the first MFMA waits for one
#pragma unroll
            for (int e = 0; e < 16; ++e) { s0[e] = 0.f; s1[e] = 0.f; }
#pragma unroll
            for (int t = 0; t < NT; ++t) { s0 = MFMA(ka[t], qf[t], s0); s1 = MFMA(kb[t], qf[t], s1); }
            FENCE();
        };
        scores_of_pair(0);
        for (int i = 0; i < ns; i += 2) {
            float x0[16], x1[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) { x0[e] = s0[e]; x1[e] = s1[e]; }
#pragma unroll
            for (int e = 0; e < 16; ++e) asm volatile("" : "+v"(x0[e]), "+v"(x1[e]));   // copied out before s0, s1 are reused
            FENCE();
            if (i + 2 < ns) scores_of_pair(i + 2);
            scan_one(x0, i);
            if (i + 1 < ns) scan_one(x1, i + 1);
        }
        m_scan = xhalf_max(m_scan) * c2;
        // Is a fixed reference good enough for this row?  For scores with standard deviation sigma the maximum
        // over all keys exceeds the maximum over a few hundred sampled keys by ~1.2 sigma, rarely by more than
        // 2.7 sigma.  The wider that uncertainty, the higher the reference has to sit and the less of the fp16
        // range is left below it for the keys that carry the sum (which spread over more binades, too): rows with
        // 2.7 sigma above F16_MAX_GAP binades (logit standard deviation above ~2.5) are left to the kernel with the
        // running reference.  The same rule is applied when the sample covers every block and its maximum is exact,
        // so that the kernel a row gets does not depend on the length of the key sequence.  A wrong guess costs
        // time only: the end-of-sweep check catches overflow.
        bool risky = false;
        if (n_stat >= BC) {
            const float inv_n = 1.f / (float)n_stat;
            const float mean = xhalf_sum(sum1) * inv_n;
            const float var = fmaxf(xhalf_sum(sum2) * inv_n - mean * mean, 0.f);
            const float reach = 2.7f * __builtin_sqrtf(var) * fabsf(c2);   // how far above the sampled maximum the true one may sit, in binades
            risky = !(reach <= F16_MAX_GAP);   // NaN counts as risky
            // The reference sits as LOW as the row's own spread allows (true maximum at weight 2^7 at most, one binade
            // kept in hand), not a fixed 6 binades above the sampled maximum: a row whose sample happens to contain
            // an outlying maximum would otherwise push the keys that carry its sum below the fp16 range.
            headroom = fminf(fmaxf(reach - 6.f, -6.f), REF_HEADROOM);
        }
        // the workgroup's vote, through a word of the V ring's last stage (nothing is there yet; the K ring is live)
        volatile __attribute__((address_space(3))) int* flag =
            (volatile __attribute__((address_space(3))) int*)(uintptr_t)(lds0 + V_RING_BASE + 3 * KV_STAGE_BYTES);
        if (tid == 0) *flag = 0;
        __syncthreads();
        if (__builtin_amdgcn_ballot_w64(risky) != 0 && lane == 0) *flag = 1;
        __syncthreads();
        const bool decline = *flag != 0;
        __syncthreads();
        if (decline) {                       // uniform over the workgroup; nothing is in flight
            if (tid == 0) wg_flags[vw] = n_blocks >= online_min_blocks ? 1 : 2;
            return;
        }
        start_v_ring();
    }
    {
        plain_scores(0, B0{});
        if (n_blocks == 1) mask_scores(0, B0{});
        m = (PRESCAN ? m_scan : row_max(B0{})) + headroom;
        const f32x16& sv = SV(B0{});
        const f32x16& tsv = TSV(B0{});
        float lb = 0.f, rb = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float pe = __builtin_amdgcn_exp2f(fmaf(sv[e], c2, -m));
            lb += pe;
            rb = fmaf(pe, tsv[e] * scale_h, rb);
        }
        const float lb_row = xhalf_sum(lb);
        ctr_h = lb_row > 0.f ? xhalf_sum(rb) / lb_row : 0.f;
        l_part = 0.f;
        r_part = 0.f;
        static_for<4>([&](auto J) { softmax_pair(J, B0{}); });   // pairs 0-3 of block 0; pairs 4-7 follow in iteration 0
        // V(0) and V(1) have landed (the first iteration reads V(0) before its own barrier, and publishes V(1) with
        // it); the copies of V(2), issued last, may still be under way
        // (a wave issues G::COPIES_PER_WAVE instructions per tensor block)
        if constexpr (G::COPIES_PER_WAVE * (ZT ? 1 : 2) == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else if constexpr (G::COPIES_PER_WAVE * (ZT ? 1 : 2) == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(1)" ::: "memory");
        __syncthreads();
    }

    // ---- online reference (MODE_F16_ONLINE).  Checked once per block, when the scores of block b+1 have been handed
    // over (middle of iteration b's phase 2).  If a row's block maximum exceeds its running maximum by more than the
    // slack, that row's reference moves there, and with it the tangent-score centre moves to the running value of
    // rowsum(P o tS) (a dominant key has appeared: centring on it keeps its H~ small and exactly representable):
    // Alg. 2's rescale, plus B <- B - (ctr_new - ctr_old) O~ as in the safe sweep.  l and r are complete up to block
    // b at that point and are rescaled at once; the accumulators still receive the rest of block b, weighted in the
    // old frame, and are rescaled at the end of the iteration.  Rare: a cold path.
    bool pend = false;
    float pend_alpha = 1.f, pend_da = 0.f;
    auto online_check = [&](auto Bc) __attribute__((always_inline)) {
        const f32x16& sv = SV(Bc);
        const f32x16& tsv = TSV(Bc);
        const float mb = row_max(Bc);
        const bool upd = mb > (m - REF_HEADROOM) + ONLINE_SLACK;
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(upd) != 0, 0)) {
            const float m_new = upd ? mb + REF_HEADROOM : m;
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);
            float lb = 0.f, rb = 0.f;
            // (an opaque copy of the new reference: seeing the same expression here and in the softmax that follows,
            // the compiler would otherwise hoist that softmax's exponentials out of their slots behind the MFMAs
            // into one block after this branch)
            float m_cold = m_new;
            asm volatile("" : "+v"(m_cold));
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float pe = __builtin_amdgcn_exp2f(fmaf(sv[e], c2, -m_cold));
                lb += pe;
                if constexpr (!PRIMAL) rb = fmaf(pe, fmaf(tsv[e], scale_h, -ctr_h), rb);
            }
            l_part = (l_part + l_part2) * alpha; l_part2 = 0.f;
            r_part = (r_part + r_part2) * alpha; r_part2 = 0.f;
            const float l_row = xhalf_sum(l_part + lb);
            const float r_row = xhalf_sum(r_part + rb);
            const float delta = upd ? r_row / l_row : 0.f;      // gH * (running rowsum(P o tS) minus ctr)
            ctr_h += delta;
            r_part = fmaf(-delta, l_part, r_part);
            pend_alpha = alpha;
            pend_da = delta * alpha;
            pend = true;
            m = m_new;
        }
    };
    auto online_apply = [&]() __attribute__((always_inline)) {
        if (__builtin_expect(pend, 0)) {
            // (the empty statements tie the accumulators to the accumulation registers on entry and exit, so that
            // the copies to and from arithmetic registers stay inside this block)
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                asm volatile("" : "+a"(accO[db]), "+a"(accAB[db]));
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    if constexpr (!PRIMAL) accAB[db][e] = fmaf(accAB[db][e], pend_alpha, -pend_da * accO[db][e]);
                    accO[db][e] *= pend_alpha;
                }
                asm volatile("" : "+a"(accO[db]), "+a"(accAB[db]));
            }
            pend = false;
        }
    };

    // ---- pipelined sweep.  Iteration b (U = b & 3 selects the ring stages at compile time):
    //   phase 1: score MFMAs of block b+1, block b's softmax arithmetic underneath;
    //   middle : wait for the copies issued two iterations ago, workgroup barrier, issue K(b+4) and V(b+3);
    //   phase 2: value MFMAs of block b, fetch of block b+1's scores underneath.
    // LDS fragments are requested well ahead of the MFMA that consumes them: the first KPRE score steps of the
    // next iteration during phase 2, the first VPRE value groups during phase 1, the rest KPRE steps / VPRE
    // groups ahead inside their own phase, through small register rings.
    constexpr int KPRE = 3, KRING = KPRE + 1, VPRE = 2, VRING = VPRE + 1;
    constexpr int KFIRST = NG == 8 ? 2 : 1;   // value group after which the next iteration's first score fragments are requested
    static_assert(KPRE < NT && KFIRST + KPRE <= NG && VPRE < NG, "the fragment rings fit the key block's steps and groups");
    const LaneOffsets lofs = make_lane_offsets<DH, F16>(wave, lane, k_stride, v_stride);
    const int n_full = Lkv / BC;                       // blocks that need no row clamping
    bf16x8 kfr[KRING], tkfr[KRING], vfr[VRING], tvfr[VRING];
    auto read_k = [&](auto T, auto ST) __attribute__((always_inline)) {     // score step T of the block in K stage ST
        constexpr int t = decltype(T)::value;
        constexpr int off = decltype(ST)::value * KV_STAGE_BYTES;
        // (the tangent fragment first: LDS reads return in order, so the wait in front of the step's first product,
        // which takes the K fragment, covers both and the third product needs none of its own)
        if constexpr (!ZT) tkfr[t % KRING] = lds_read_b128(kaddr0[t] + off + TENSOR_BYTES);
        kfr[t % KRING] = lds_read_b128(kaddr0[t] + off);
    };
    auto read_v = [&](auto Gi, auto ST) __attribute__((always_inline)) {    // value group Gi of the block in V stage ST
        constexpr int gi = decltype(Gi)::value;
        constexpr int t2 = gi / NDB, db = gi % NDB;
        constexpr int off = decltype(ST)::value * KV_STAGE_BYTES + (F16 ? db * (32 * 64) : t2 * 16 * ROW_BYTES);
        const uint32_t a = vaddr0[F16 ? t2 : db] + off;
        if constexpr (!ZT) tvfr[gi % VRING] = read_v_fragment(a + TENSOR_BYTES);
        vfr[gi % VRING] = read_v_fragment(a);
    };

    // The copies of iteration b: K(b+4) into K stage b & 3, V(b+3) into V stage (b+3) & 3, as 8 direct-to-LDS
    // instructions per wave (4 at head dimension 64).  They are issued ONE per value group in phase 2, not back to back: the vector memory
    // pipe takes ~16 cycles per 1 KiB instruction and all four waves pass the barrier together, so a burst would
    // stall the in-order instruction stream behind the queue.
    auto issue_copy_piece = [&](auto FULLc, auto IDX, int b) __attribute__((always_inline)) {
        constexpr int idx = decltype(IDX)::value;
        constexpr int i = idx >> 2, which = idx & 3;      // row group of this wave; 0 K, 1 tK, 2 V, 3 tV
        static_assert(i < G::COPIES_PER_WAVE, "one piece per value group covers exactly the iteration's copies");
        if constexpr (ZT && (which & 1)) return;          // no tangent tensors to copy
        const int blk = which < 2 ? b + 4 : b + 3;
        const char* base = which == 0 ? Kh : which == 1 ? tKh : which == 2 ? Vh : tVh;
        const uint32_t dst = lds0 + (which < 2 ? 0 : V_RING_BASE) + (uint32_t)(blk & 3) * KV_STAGE_BYTES +
                             (which & 1) * TENSOR_BYTES + (wave * G::COPIES_PER_WAVE + i) * 1024;
        if constexpr (F16 && which >= 2) {                 // a whole transposed block of the fp16 copies: nothing to clamp but the block index
            const int bc = decltype(FULLc)::value ? blk : (blk < n_blocks ? blk : n_blocks - 1);
            load_lds_b128(base + (long)bc * TENSOR_BYTES, lofs.v[i], __builtin_amdgcn_readfirstlane(dst));
        } else if constexpr (decltype(FULLc)::value) {
            const uint32_t lo = which < 2 ? lofs.k[i] : lofs.v[i];
            load_lds_b128(base + (long)blk * (BC * (which < 2 ? k_stride : v_stride)), lo, __builtin_amdgcn_readfirstlane(dst));
        } else {
            const int row = (wave * G::COPIES_PER_WAVE + i) * G::ROWS_PER_COPY + lane / G::LANES_PER_ROW;
            const int pc = lane % G::LANES_PER_ROW;
            int grow = blk * BC + row;
            grow = grow < Lkv ? grow : Lkv - 1;
            const int chunk = pc ^ (which < 2 ? G::k_swizzle(row) : G::v_swizzle(row));
            ATTN_JVP_LOAD_LDS(base + (long)grow * (which < 2 ? k_stride : v_stride) + (chunk << 4), dst);
        }
    };

    // Vector work is spread so that no MFMA has more than ~6 vector instructions behind it (beyond that the single
    // wavefront of a SIMD stops overlapping them with the matrix pipe):
    //   phase 1 of iteration b  : weights of pairs 4-7 of block b   (its scores were produced in iteration b-1)
    //   phase 2, groups 0-3     : exponentials of pairs 0-3 of block b+1 (one pair per group), straight from the
    //                             registers its score products wrote in phase 1
    //   phase 2, groups 4-7     : rest of the softmax of those pairs, which writes the packed weights (their
    //                             registers were consumed by groups 0-3)
    auto iteration = [&](auto Uc, auto FULLc, int b) __attribute__((always_inline)) {
        constexpr int U = decltype(Uc)::value;
        constexpr bool FULL = decltype(FULLc)::value;
        constexpr int PRODUCTS = PRIMAL ? 1 : ZT ? 2 : 3;         // matrix products per score step / per weight term
        constexpr int GROUP_MFMAS = SPLIT ? 2 * PRODUCTS : PRODUCTS;
        constexpr int SPP = NT / 4;                                // phase 1: score steps per pair of score elements (2, or 1 at head dimension 64)
        constexpr int PPG = 8 / NG;                                // phase 2: pairs per value group in each half of the groups (1, or 2)
        using NS_P1 = std::integral_constant<int, SPP * PRODUCTS>;
        using NS_P2 = std::integral_constant<int, GROUP_MFMAS>;
        using K1 = std::integral_constant<int, (U + 1) & 3>;    // K stage of block b+1
        using K2 = std::integral_constant<int, (U + 2) & 3>;    // K stage of block b+2
        using V0 = std::integral_constant<int, U>;              // V stage of block b
        using Bcur = std::integral_constant<int, U & 1>;        // score buffers of block b
        using Bnext = std::integral_constant<int, (U + 1) & 1>; // ... of block b+1, written in phase 1
        f32x16& s = SV(Bnext{});
        f32x16& ts = TSV(Bnext{});
        // ---- phase 1
        static_for<NT>([&](auto T) {
            constexpr int t = decltype(T)::value;
            using J = std::integral_constant<int, 4 + t / SPP>;
            constexpr int s0 = (t % SPP) * PRODUCTS;
            if constexpr (t == 0) SMFMA0(kfr[t % KRING], qf[t], s); else SMFMA(kfr[t % KRING], qf[t], s);
            softmax_slot(J{}, std::integral_constant<int, s0>{}, NS_P1{}, Bcur{});
            FENCE();
            if constexpr (!PRIMAL) {
                if constexpr (t == 0) SMFMA0(kfr[t % KRING], tqf[t], ts); else SMFMA(kfr[t % KRING], tqf[t], ts);
                softmax_slot(J{}, std::integral_constant<int, s0 + 1>{}, NS_P1{}, Bcur{});
                FENCE();
            }
            if constexpr (!ZT) {
                SMFMA(tkfr[t % KRING], qf[t], ts);
                softmax_slot(J{}, std::integral_constant<int, s0 + 2>{}, NS_P1{}, Bcur{});
                FENCE();
            }
            if constexpr (t + KPRE < NT) read_k(std::integral_constant<int, t + KPRE>{}, K1{});
            if constexpr (t >= NT - VPRE) read_v(std::integral_constant<int, t - (NT - VPRE)>{}, V0{});
            FENCE();
        });
        // ---- middle
        SCORE_RESULTS_LAND();
        // all but the newest copies (8 instructions per wave and iteration, 4 without tangents) landed: K(b+2), V(b+1) are in
        // (G::COPIES_PER_WAVE instructions per tensor block: 8 per iteration at head dimension 128, 4 at 64, half without tangents)
        if constexpr (G::COPIES_PER_WAVE * (ZT ? 2 : 4) == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else if constexpr (G::COPIES_PER_WAVE * (ZT ? 2 : 4) == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
        // ... and visible to all waves after the barrier; all waves are done with K(b) and V(b-1).  A bare barrier:
        // the LDS reads still in flight (first value fragments of block b) read stages nobody overwrites yet.
        __builtin_amdgcn_s_barrier();
        FENCE();
        // ---- phase 2
        static_for<NG>([&](auto Gc) {
            constexpr int gi = decltype(Gc)::value;     // group = (t2, db)
            constexpr int t2 = gi / NDB, db = gi % NDB;
            const bf16x8 pb = as_bf16x8(wp[4 * t2], wp[4 * t2 + 1], wp[4 * t2 + 2], wp[4 * t2 + 3]);
            bf16x8 hb8 = pb;
            if constexpr (!PRIMAL) hb8 = as_bf16x8(wh[4 * t2], wh[4 * t2 + 1], wh[4 * t2 + 2], wh[4 * t2 + 3]);
            // vector work behind MFMA number `slot` of this group
            auto behind = [&](auto SLOT) __attribute__((always_inline)) {
                constexpr int slot = decltype(SLOT)::value;
                if constexpr (gi < NG / 2) {
                    // first touch of block b+1's scores (behind the second MFMA of a group where there is one: the
                    // score products' results have landed by then; the build's assembly check counts the wait states)
                    constexpr int first = GROUP_MFMAS >= 3 ? 1 : 0;
                    // (head dimension 64: two pairs per group, the second one behind the next MFMA where there is one)
                    if constexpr (PPG == 2 && GROUP_MFMAS >= first + 2 && slot == first + 1)
                        softmax_part(std::integral_constant<int, 2 * gi + 1>{}, std::integral_constant<int, 0>{}, Bnext{});
                    if constexpr (slot == first) {
                        if constexpr (gi == 0) {
                            // (every lane of the new scores counts as read here, used or not: the score products of the
                            // last iteration's unused block past the end still write their registers, which must not
                            // have been handed to something else in the meantime)
                            if constexpr (PRIMAL) asm volatile("" : "+v"(s));
                            else asm volatile("" : "+v"(s), "+v"(ts));
                            if constexpr (!FULL) {
                                // tail iterations only: keys past Lkv (a ragged last block, or the unused block past the end)
                                if ((b + 2) * BC > Lkv) mask_scores(b + 1, Bnext{});
                            }
                            if constexpr (ONLINE) online_check(Bnext{});
                        }
                        softmax_part(std::integral_constant<int, PPG * gi>{}, std::integral_constant<int, 0>{}, Bnext{});
                        if constexpr (PPG == 2 && GROUP_MFMAS < first + 2)
                            softmax_part(std::integral_constant<int, 2 * gi + 1>{}, std::integral_constant<int, 0>{}, Bnext{});
                    }
                } else if constexpr (PPG == 1) {
                    softmax_late_slot(std::integral_constant<int, gi - NG / 2>{}, SLOT, NS_P2{}, Bnext{});
                } else {
                    // two pairs per group: their eight late parts in order, dealt evenly over the group's MFMAs
                    static_for<8>([&](auto Kc) {
                        constexpr int k = decltype(Kc)::value;
                        if constexpr (k * GROUP_MFMAS / 8 == slot)
                            softmax_part(std::integral_constant<int, 2 * (gi - NG / 2) + k / 4>{}, std::integral_constant<int, 1 + k % 4>{}, Bnext{});
                    });
                }
            };
            accO[db] = VMFMA(vfr[gi % VRING], pb, accO[db]);
            behind(std::integral_constant<int, 0>{});
            FENCE();
            if constexpr (!ZT) {
                accAB[db] = VMFMA(tvfr[gi % VRING], pb, accAB[db]);
                behind(std::integral_constant<int, 1>{});
                FENCE();
            }
            if constexpr (!PRIMAL) {
                accAB[db] = VMFMA(vfr[gi % VRING], hb8, accAB[db]);
                behind(std::integral_constant<int, PRODUCTS - 1>{});
            }
            if constexpr (SPLIT) {
                const bf16x8 pl8 = as_bf16x8(wpl[4 * t2], wpl[4 * t2 + 1], wpl[4 * t2 + 2], wpl[4 * t2 + 3]);
                FENCE();
                accO[db] = VMFMA(vfr[gi % VRING], pl8, accO[db]);
                behind(std::integral_constant<int, PRODUCTS>{});
                if constexpr (!ZT) {
                    FENCE();
                    accAB[db] = VMFMA(tvfr[gi % VRING], pl8, accAB[db]);
                    behind(std::integral_constant<int, PRODUCTS + 1>{});
                }
                if constexpr (!PRIMAL) {
                    const bf16x8 hl8 = as_bf16x8(whl[4 * t2], whl[4 * t2 + 1], whl[4 * t2 + 2], whl[4 * t2 + 3]);
                    FENCE();
                    accAB[db] = VMFMA(vfr[gi % VRING], hl8, accAB[db]);
                    behind(std::integral_constant<int, 2 * PRODUCTS - 1>{});
                }
            }
            FENCE();
            issue_copy_piece(FULLc, Gc, b);
            if constexpr (gi + VPRE < NG) read_v(std::integral_constant<int, gi + VPRE>{}, V0{});
            if constexpr (gi >= KFIRST && gi < KFIRST + KPRE) read_k(std::integral_constant<int, gi - KFIRST>{}, K2{});
            FENCE();
        });
        if constexpr (ONLINE) online_apply();     // block b is complete: move the accumulators to the new frame, if any
    };

    {
        static_for<KPRE>([&](auto T) { read_k(T, std::integral_constant<int, 1>{}); });   // K(1), landed in the prologue
        FENCE();
        using FY = std::integral_constant<bool, true>;
        using FN = std::integral_constant<bool, false>;
        using U0 = std::integral_constant<int, 0>;
        using U1 = std::integral_constant<int, 1>;
        using U2 = std::integral_constant<int, 2>;
        using U3 = std::integral_constant<int, 3>;
        int b = 0;
        // main loop: every block copied inside it (up to K(b+7)) is a full block
        if (b + 8 <= n_full) {
            do {
                iteration(U0{}, FY{}, b);
                iteration(U1{}, FY{}, b + 1);
                iteration(U2{}, FY{}, b + 2);
                iteration(U3{}, FY{}, b + 3);
                b += 4;
            } while (b + 8 <= n_full);
        }
        // tail (at most 8 blocks, b is a multiple of 4 here): clamped copies, and masking of the keys past Lkv in
        // the scores fetched for block b+1.  Straight-line nested code, not a loop over a switch: around a loop
        // the register allocator moved the accumulators at every iteration.
        auto tail = [&](auto self, auto K, int bb) __attribute__((always_inline)) -> void {
            constexpr int k = decltype(K)::value;
            if constexpr (k < 8) {
                if (bb < n_blocks) {
                    iteration(std::integral_constant<int, k & 3>{}, FN{}, bb);
                    self(self, std::integral_constant<int, k + 1>{}, bb + 1);
                }
            }
        };
        tail(tail, std::integral_constant<int, 0>{}, b);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        // Resident workgroups: while this tile's results are checked, turned round and stored, bring the next tile's
        // Q and tQ rows into the L2 (one 128-byte line per lane and tensor, as a direct-to-LDS load of 16 bytes of it
        // into a spare KiB that nobody reads).  The next tile's first loads then wait for the L2, not for memory:
        // measured on the cross-attention workload, 2.0 us instead of 3.6 us from a tile's start to its Q fragments.
        // (Its start waits for all vector memory operations, so nothing of this is in flight beyond it; the last tile
        // of a workgroup requests nothing.)
        if (vw + (int)gridDim.x < n_tiles) {
            const int vn = vw + (int)gridDim.x;
            const int bidn = (n_wg & 7) == 0 ? (vn & 7) * (n_wg >> 3) + (vn >> 3) : vn;
            const long bhn = bidn / q_tiles;
            const int rown0 = (bidn % q_tiles) * BR;
            const long qbn = blhd ? ((bhn / H) * Lq * H + bhn % H) * D : bhn * (long)Lq * D;
            constexpr int LINES = ROW_BYTES / 128;                 // 128-byte lines per row (2, or 1 at head dimension 64)
#pragma unroll
            for (int u = 0; u < (BR * LINES + NTHREADS - 1) / NTHREADS; ++u) {
                const int idx = (int)tid + NTHREADS * u;
                if (idx < BR * LINES) {
                    int row = rown0 + idx / LINES;
                    row = row < Lq ? row : Lq - 1;
                    const long off = (qbn + (long)row * row_elems) * 2 + (idx % LINES) * 128;
                    ATTN_JVP_LOAD_LDS(reinterpret_cast<const char*>(Q) + off, lds0 + G::RING_BYTES);
                    if constexpr (!PRIMAL) ATTN_JVP_LOAD_LDS(reinterpret_cast<const char*>(tQ) + off, lds0 + G::RING_BYTES);
                    // ... and the first four key blocks of its head (the same 128 rows of K and tK), if it is another head
                    if (bhn != bh) {
                        int krow = idx / LINES;
                        krow = krow < Lkv ? krow : Lkv - 1;
                        const long kbn = blhd ? ((bhn / H) * Lkv * H + bhn % H) * D : bhn * (long)Lkv * D;
                        const long koff = (kbn + (long)krow * row_elems) * 2 + (idx % LINES) * 128;
                        ATTN_JVP_LOAD_LDS(reinterpret_cast<const char*>(K) + koff, lds0 + G::RING_BYTES);
                        if constexpr (!ZT) ATTN_JVP_LOAD_LDS(reinterpret_cast<const char*>(tK) + koff, lds0 + G::RING_BYTES);
                    }
                }
            }
        }
    }

    // Did the fixed exponent reference hold?  Row sums beyond 2^60 (or not finite) mean some score exceeded the
    // reference by ~100 binades.  Then the WHOLE workgroup redoes its tile with Alg. 2's running maximum.
    {
        const float l_chk = xhalf_sum(l_part + l_part2), r_chk = xhalf_sum(r_part + r_part2);
        bool bad = !(l_chk < 0x1p60f) || !(fabsf(r_chk) < 0x1p100f);
        // Sampled reference: weights below 2^-25 round to zero in fp16, so up to Lkv 2^-25 of weight may be missing
        // from a row's sums; the row is good when that is at most 2^-10 of its l.  (A reference that sits too high
        // for a row, e.g. because the sample caught an outlying maximum, shows up here.)
        if constexpr (PRESCAN) bad = bad || !(l_chk >= (float)Lkv * 0x1p-15f);
        // (fp16 weights: l and r are summed from the weights as rounded to fp16, so a weight that overflowed to inf,
        // or a 0 x inf in H~16, shows in l or r and fails the tests above; V16 and tV16 are finite by their scaling,
        // and finite fp16 operands cannot overflow the fp32 accumulators.  The accumulators need no scan of their own.)
        __syncthreads();                       // everyone is done with the rings
        volatile __attribute__((address_space(3))) int* flag =
            (volatile __attribute__((address_space(3))) int*)(uintptr_t)lds0;
        if (tid == 0) *flag = 0;
        __syncthreads();
        if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0) *flag = 1;
        __syncthreads();
        const bool redo = *flag != 0;
        __syncthreads();
        if constexpr (F16) {
            // the fp16 kernels do not repair: they hand the tile to the launch that follows (online fp16, then bf16 pairs)
            if (tid == 0)
                wg_flags[vw] = redo ? (ONLINE || n_blocks < online_min_blocks ? 2 : 1) : (ONLINE ? 3 : 0);
            if (redo) return;
        } else if (__builtin_expect(redo, 0)) {
            // ============================ safe sweep (rare) ============================
            // Alg. 2 as printed: per block, running maximum, rescale of every accumulator, no overlap.
            // ctr follows the running value of rowsum(P o tS): B <- B - (ctr_new - ctr_old) O~ keeps it exact.
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) { accO[db][e] = 0.f; accAB[db][e] = 0.f; }
            m = -INFINITY; l_part = 0.f; r_part = 0.f; l_part2 = 0.f; r_part2 = 0.f; ctr_h = 0.f; headroom = 0.f;
            copy_k(0); copy_v(0);
            for (int b = 0; b < n_blocks; ++b) {
                const uint32_t off = (uint32_t)(b & 3) * KV_STAGE_BYTES;
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
                copy_k(b + 1); copy_v(b + 1);
                plain_scores(off, B0{});
                if ((b + 1) * BC > Lkv) mask_scores(b, B0{});
                const f32x16& sv = SV(B0{});
                const f32x16& tsv = TSV(B0{});
                const float tmax = row_max(B0{});
                const float m_new = fmaxf(m, tmax);
                const float alpha = __builtin_amdgcn_exp2f(m - m_new);
                m = m_new;
                float lb = 0.f, rb = 0.f;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float pe = __builtin_amdgcn_exp2f(fmaf(sv[e], c2, -m));
                    lb += pe;
                    rb = fmaf(pe, fmaf(tsv[e], scale_h, -ctr_h), rb);
                }
                l_part = (l_part + l_part2) * alpha; l_part2 = 0.f;
                r_part = (r_part + r_part2) * alpha; r_part2 = 0.f;
                const float l_row = xhalf_sum(l_part + lb);
                const float r_row = xhalf_sum(r_part + rb);
                const float delta = r_row / l_row;          // gH * (running rowsum(P o tS) minus ctr)
                ctr_h += delta;
                r_part = fmaf(-delta, l_part, r_part);
                const float da = delta * alpha;
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        if constexpr (!PRIMAL) accAB[db][e] = fmaf(accAB[db][e], alpha, -da * accO[db][e]);
                        accO[db][e] *= alpha;
                    }
                static_for<8>([&](auto P) { softmax_pair(P, B0{}); });
                plain_values(off);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
    }

    // ---- epilogue: O = O~/l, lse = m + log l, tO = (A + B - (r/l) O~) / l  (r and B both relative to ctr).
    // With accO = O~/gO, accAB = (A+B)/gAB and r_part summing gH H~ (gH = gO/gAB) this is gAB (accAB - mu accO) / l.
    const float l_row = xhalf_sum(l_part + l_part2);
    const float r_row = xhalf_sum(r_part + r_part2);
    const float inv_l = 1.f / l_row;
    const float mu = r_row * inv_l;
    const float fo = gO * inv_l, ft = gAB * inv_l;
    // Outputs: rows d_out elements wide in the caller's layout.  d_out = 128 unless the inputs are zero-padded
    // copies of a smaller head dimension: then only the first d_out columns exist (and are stored).
    //
    // A lane holds 16 scattered 16-byte pieces of ONE row per tensor, so storing from the accumulators directly puts
    // only 32 contiguous bytes per row into each store instruction.  Measured, such a 128 KiB tile takes a compute
    // unit 3.6 us to write (18 us when all units write at once), against 1.1 us (5.4 us) when every instruction
    // writes whole rows.  Each wave therefore turns its 32 x 128 results round through its own 32 KiB of the (now
    // idle) LDS: written as held (row c, 16-byte chunk 8 db + 2 v4 + g, at chunk position chunk ^ c so that neither
    // direction meets bank conflicts), read back two whole rows per instruction.  LDS operations of one wave execute
    // in order, so the wave needs no barrier of its own; the workgroup barrier at the end keeps the next tile's
    // first copies (resident workgroups) off the staging areas of waves that are still reading.
    {
        typedef __attribute__((address_space(3))) f32x4 lds_float4;
        constexpr uint32_t OUT_ROW_BYTES = DH * 4;                 // a row of fp32 results
        constexpr int OUT_CHUNKS = DH / 4;                         // ... in 16-byte chunks (32, or 16 at head dimension 64)
        constexpr int ROWS_PER_STORE = 64 / OUT_CHUNKS;            // rows one store instruction covers (2, or 4)
        const uint32_t stage_o = lds0 + (uint32_t)wave * (64u * OUT_ROW_BYTES), stage_t = stage_o + 32u * OUT_ROW_BYTES;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                float4 o4, t4;
                const float a0 = accO[db][4 * v4], a1 = accO[db][4 * v4 + 1], a2 = accO[db][4 * v4 + 2], a3 = accO[db][4 * v4 + 3];
                o4.x = a0 * fo; o4.y = a1 * fo; o4.z = a2 * fo; o4.w = a3 * fo;
                t4.x = (accAB[db][4 * v4] - mu * a0) * ft;
                t4.y = (accAB[db][4 * v4 + 1] - mu * a1) * ft;
                t4.z = (accAB[db][4 * v4 + 2] - mu * a2) * ft;
                t4.w = (accAB[db][4 * v4 + 3] - mu * a3) * ft;
                const uint32_t at = (uint32_t)c * OUT_ROW_BYTES + (uint32_t)(((8 * db + 2 * v4 + g) ^ (c & (OUT_CHUNKS - 1))) << 4);
                *reinterpret_cast<lds_float4*>((uintptr_t)(stage_o + at)) = f32x4{o4.x, o4.y, o4.z, o4.w};
                if constexpr (!PRIMAL) *reinterpret_cast<lds_float4*>((uintptr_t)(stage_t + at)) = f32x4{t4.x, t4.y, t4.z, t4.w};
            }
        // m carries `headroom` binades that l_row lacks: take them out of both before adding (exact scalings)
        if (g == 0 && qrow < Lq)
            LSE[bh * Lq + qrow] = ((m - headroom) + __builtin_amdgcn_logf(l_row * __builtin_amdgcn_exp2f(headroom))) * 0.6931471805599453f;
        const int o_row = out_blhd ? H * d_out : d_out;
        const long o_base = out_blhd ? (bidx * Lq * H + hidx) * d_out : bh * (long)Lq * d_out;
        const int chunk = lane % OUT_CHUNKS;         // 16-byte chunk of the row this lane stores: columns 4 chunk .. +3
        if (4 * chunk < d_out) {
#pragma unroll
            for (int i = 0; i < 32 / ROWS_PER_STORE; ++i) {
                const int r = ROWS_PER_STORE * i + lane / OUT_CHUNKS;      // row of the wave's 32
                const int row = q0 + r;
                const uint32_t at = (uint32_t)r * OUT_ROW_BYTES + (uint32_t)((chunk ^ (r & (OUT_CHUNKS - 1))) << 4);
                const f32x4 ov = *reinterpret_cast<const lds_float4*>((uintptr_t)(stage_o + at));
                f32x4 tv_ = ov;
                if constexpr (!PRIMAL) tv_ = *reinterpret_cast<const lds_float4*>((uintptr_t)(stage_t + at));
                const float4 o4 = make_float4(ov[0], ov[1], ov[2], ov[3]), t4 = make_float4(tv_[0], tv_[1], tv_[2], tv_[3]);
                if (row < Lq) {
                    const long off = o_base + (long)row * o_row + 4 * chunk;
                    if (out_bf16) {      // uniform; four bf16 = 8 bytes per lane and tensor
                        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(O) + off) = make_uint2(pack_bf16(o4.x, o4.y), pack_bf16(o4.z, o4.w));
                        if constexpr (!PRIMAL)
                            *reinterpret_cast<uint2*>(static_cast<uint16_t*>(tO) + off) = make_uint2(pack_bf16(t4.x, t4.y), pack_bf16(t4.z, t4.w));
                    } else {
                        *reinterpret_cast<float4*>(static_cast<float*>(O) + off) = o4;
                        if constexpr (!PRIMAL) *reinterpret_cast<float4*>(static_cast<float*>(tO) + off) = t4;
                    }
                }
            }
        }
        __syncthreads();
    }
}

// The launch: workgroup w does tiles w, w + gridDim.x, w + 2 gridDim.x, ...  With one workgroup per tile (gridDim.x
// = n_tiles) that is one tile each, handed out by the hardware as compute units fall free; with fewer, the workgroups
// stay resident and walk through their tiles themselves: no workgroup launch between tiles, the tile-independent
// set-up is done once, and a tile's output stores drain while the next tile's first loads are already queued
// behind them.  A tile ends with every wave past a workgroup barrier that follows its last LDS read, on every
// path, so the next tile may start filling LDS at once.  Since gridDim.x is then a multiple of 8, tile w + k gridDim.x
// runs on the same XCD as tile w, as the tile map in attn_jvp_tile assumes.
template <int MODE, int TAN, int DH>
__global__ __launch_bounds__(NTHREADS, DH == 64 ? 2 : 1) void attn_jvp_mfma_kernel(
    const __hip_bfloat16* __restrict__ Q, const __hip_bfloat16* __restrict__ K, const void* __restrict__ V,
    const __hip_bfloat16* __restrict__ tQ, const __hip_bfloat16* __restrict__ tK, const void* __restrict__ tV,
    void* __restrict__ O, void* __restrict__ tO, float* __restrict__ LSE,
    int Lq, int Lkv, float scale, int q_tiles, const float* __restrict__ stats, int* __restrict__ wg_flags,
    int H, int blhd, int out_bf16, int d_out, int out_blhd, int online_min_blocks, int lockstep_slots, int n_tiles,
    int stagger_ticks) {
    // Resident workgroups all start together and their tiles take the same time, so without this every compute unit
    // would write its 128 KiB of results in the same few microseconds, round after round, and wait for memory while
    // the matrix pipes idle (measured 8 us per tile, against 1-2 us for a compute unit that writes alone).  The
    // workgroups of an XCD therefore start stagger_ticks (of the 100 MHz wall clock) apart; the offsets persist, and
    // each unit's stores fall into the others' sweeps.  Bounded by the clock; costs the last offset once per launch.
    if (stagger_ticks > 0) {
        const unsigned long long t0 = wall_clock64();
        const unsigned long long wait = (unsigned long long)((blockIdx.x >> 3) & 31) * (unsigned)stagger_ticks;
        while (wall_clock64() - t0 < wait) __builtin_amdgcn_s_sleep(8);
    }
    for (int vw = blockIdx.x; vw < n_tiles; vw += gridDim.x)
        attn_jvp_tile<MODE, TAN, DH>(Q, K, V, tQ, tK, tV, O, tO, LSE, Lq, Lkv, scale, q_tiles, stats, wg_flags, H, blhd, out_bf16,
                                 d_out, out_blhd, online_min_blocks, lockstep_slots, vw, n_tiles);
    // (a hand-over launch may have requested lines for a next tile that turned out not to be its own: no direct-to-LDS
    // load is left in flight when the wave ends)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

}  // namespace

// scale > 0: the kernel masks padded keys with a raw score of -inf and takes row maxima before scaling.
// tk and tv are either both given or both absent (zero key/value tangents); single bf16 weights (FAST) are not built
// for the latter.
// Head dimensions 128 and 64 are built natively; 32 and 96 run on zero-padded copies (to 64 and 128 columns), which
// need the caller's workspace.
static bool padded_head_dim(const Problem& p) {
    return (p.d == 32 || p.d == 96) && p.workspace != nullptr &&
           (reinterpret_cast<uintptr_t>(p.workspace) & 255u) == 0 &&
           p.workspace_bytes >= pad_workspace_bytes(p.B, p.H, p.Lq, p.Lkv, p.d);
}
bool mfma_bf16_supports(const Problem& p) {
    const bool zt = p.tk == nullptr && p.tv == nullptr;     // (the API admits absent tangents only as tk+tv or tq+tk+tv)
    return p.in_dtype == 0 && (p.d == 128 || p.d == 64 || padded_head_dim(p)) && p.scale > 0.f && !(zt && (p.flags & 1));
}

// Dynamic-LDS limit of every instantiation a call may launch, raised once per device and before anything is enqueued.
template <int DH>
static hipError_t prepare_kernels(int dev) {
    const void* kernels[] = {
        (const void*)attn_jvp_mfma_kernel<MODE_BF16, TAN_ALL, DH>,
        (const void*)attn_jvp_mfma_kernel<MODE_BF16_SPLIT, TAN_NONE, DH>, (const void*)attn_jvp_mfma_kernel<MODE_BF16_SPLIT, TAN_QUERY, DH>,
        (const void*)attn_jvp_mfma_kernel<MODE_BF16_SPLIT, TAN_ALL, DH>,
        (const void*)attn_jvp_mfma_kernel<MODE_F16, TAN_NONE, DH>, (const void*)attn_jvp_mfma_kernel<MODE_F16, TAN_QUERY, DH>,
        (const void*)attn_jvp_mfma_kernel<MODE_F16, TAN_ALL, DH>,
        (const void*)attn_jvp_mfma_kernel<MODE_F16_ONLINE, TAN_NONE, DH>, (const void*)attn_jvp_mfma_kernel<MODE_F16_ONLINE, TAN_QUERY, DH>,
        (const void*)attn_jvp_mfma_kernel<MODE_F16_ONLINE, TAN_ALL, DH>};
    for (const void* k : kernels) {
        const hipError_t e = ensure_dynamic_lds(k, Geo<DH>::LDS_BYTES, dev);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <int DH>
static hipError_t launch_dh(const Problem& p_in) {
    int dev = 0, cus = 0;
    {   // everything that can fail without a launch comes first: a failure here leaves nothing enqueued
        hipError_t e = device_cus(&dev, &cus);
        if (e == hipSuccess) e = prepare_kernels<DH>(dev);
        if (e != hipSuccess) return e;
        const long long tiles = (long long)((p_in.Lq + BR - 1) / BR) * p_in.B * p_in.H;
        if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    }
    Problem p = p_in;
    if (p_in.d != DH) {      // run on zero-padded copies of the inputs; o, to keep the caller's width and layout
        hipError_t e = launch_pad_inputs(p_in, &p);
        if (e != hipSuccess) return e;
    }
    const int q_tiles = (p.Lq + BR - 1) / BR;
    const long long blocks = (long long)q_tiles * p.B * p.H;
    int lockstep = 0;   // set for the online launch below
    // The launch that does (nearly) all the tiles runs with resident workgroups, one per compute unit, each walking
    // through its share of the tiles, when there are at least two tiles per unit.  The hand-over launches do the
    // same on sequences below LOCKSTEP_MIN_BLOCKS key blocks, without the staggered start: they usually find nothing
    // to do, and a workgroup that looks at a dozen flags costs far less than a dozen workgroups that are launched
    // (with all of a compute unit's LDS and registers each) to look at one (cross-attention workload: 13 + 9 us for
    // the two launches with one workgroup per tile).  On longer sequences, where their tiles take milliseconds and
    // differ in length, they keep one workgroup per tile, which the hardware balances.
    bool resident = false;
    const bool short_tiles = (p.Lkv + BC - 1) / BC < LOCKSTEP_MIN_BLOCKS;
    auto launch = [&](auto kern, const void* v, const void* tv, const float* stats, int* wg_flags) -> hipError_t {
        constexpr int WG_PER_CU = DH == 64 ? 2 : 1;       // what the kernel's registers and LDS allow
        const bool follower = !resident && wg_flags != nullptr;      // a hand-over launch of the fp16 path
        const bool res = (resident || (follower && short_tiles)) && cus % 8 == 0 && blocks >= 2LL * WG_PER_CU * cus &&
                         !(p.flags & 16);   // 16: ATTN_JVP_FLAG_NO_RESIDENT
        const long long grid = res ? (long long)WG_PER_CU * cus : blocks;
        const int stagger = res && !follower ? STAGGER_TICKS : 0;
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NTHREADS), Geo<DH>::LDS_BYTES, p.stream,
                           (const __hip_bfloat16*)p.q, (const __hip_bfloat16*)p.k, v,
                           (const __hip_bfloat16*)p.tq, (const __hip_bfloat16*)p.tk, tv,
                           p.o, p.to, p.lse, p.Lq, p.Lkv, p.scale, q_tiles, stats, wg_flags, p.H, p.layout, p.out_dtype,
                           p.d_out, p.out_layout, (p.flags & 4) ? 0 : ONLINE_MIN_BLOCKS,   // F16_ALWAYS: never the pairs first
                           lockstep, (int)blocks, stagger);
        return hipGetLastError();
    };
    // fp16 value path when the caller lent enough scratch (and did not ask for another variant) and the call is
    // large enough to amortise its per-call pre-pass (see F16_MIN_KEYS)
    const bool f16 = !(p.flags & 3) && p.workspace != nullptr && (long long)p.B * p.H <= 65535 &&   // pre-pass grid.y
                     (p.Lkv >= F16_MIN_KEYS || (p.flags & 4) ||
                      (p.Lkv >= F16_MIN_KEYS_MANY_TILES && blocks >= (long long)F16_MANY_TILES_PER_CU * cus)) &&
                     p.workspace_bytes >= f16_workspace_bytes(p.B, p.H, p.Lq, p.Lkv, p.d) &&
                     (reinterpret_cast<uintptr_t>(p.workspace) & 255u) == 0;
    F16Workspace ws{};
    if (f16) {
        hipError_t e = launch_f16_prepass(p, cus, &ws);
        if (e != hipSuccess) return e;
        if ((p.Lkv + BC - 1) / BC < LOCKSTEP_MIN_BLOCKS || (p.flags & 8)) ws.lockstep_slots = 0;
    }
    MainKernelTimer timer(p);
    hipError_t e;
    // fp16 path: every tile is finished by exactly one of three launches.  The fp16 kernel with its sampled, fixed
    // reference flags the tiles it declines (scores too spread out) or abandons (overflow found at the end of its
    // sweep); the online fp16 kernel does those, unless it meets an overflow itself (tangent scores beyond the fp16
    // range), which it flags for the bf16-pair kernel; each returns at once from the tiles that are not its own.
    auto run = [&](auto tan, const void* tv, const void* tv16) -> hipError_t {
        constexpr int T = decltype(tan)::value;
        resident = true;
        if (!f16) return launch(attn_jvp_mfma_kernel<MODE_BF16_SPLIT, T, DH>, p.v, tv, nullptr, nullptr);
        hipError_t err = launch(attn_jvp_mfma_kernel<MODE_F16, T, DH>, ws.v16, tv16, ws.stats, ws.wg_flags);
        resident = false;
        lockstep = ws.lockstep_slots;
        if (err == hipSuccess) err = launch(attn_jvp_mfma_kernel<MODE_F16_ONLINE, T, DH>, ws.v16, tv16, ws.stats, ws.wg_flags);
        lockstep = 0;
        if (err == hipSuccess) err = launch(attn_jvp_mfma_kernel<MODE_BF16_SPLIT, T, DH>, p.v, tv, nullptr, ws.wg_flags);
        return err;
    };
    if (p.tq == nullptr) {             // no tangents at all: plain attention forward
        e = run(std::integral_constant<int, TAN_NONE>{}, nullptr, nullptr);
    } else if (p.tk == nullptr) {      // zero key/value tangents
        e = run(std::integral_constant<int, TAN_QUERY>{}, nullptr, nullptr);
    } else if (p.flags & 1) {
        resident = true;
        e = launch(attn_jvp_mfma_kernel<MODE_BF16, TAN_ALL, DH>, p.v, p.tv, nullptr, nullptr);
    } else {
        e = run(std::integral_constant<int, TAN_ALL>{}, p.tv, ws.tv16);
    }
    return timer.finish(e);
}

hipError_t launch_mfma_bf16(const Problem& p) {
    if (!mfma_bf16_supports(p)) return hipErrorInvalidValue;
    return p.d <= 64 ? launch_dh<64>(p) : launch_dh<128>(p);     // 32 runs on copies padded to 64 columns, 96 to 128
}

}  // namespace attn_jvp
