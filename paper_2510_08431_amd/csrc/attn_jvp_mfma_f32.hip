// fp32 matrix-core streaming kernel for attention forward + JVP (paper App. C.1, Alg. 2) on gfx950.
//
// The path for fp32 inputs at head dims 32, 64, 96, 128: every product runs on v_mfma_f32_32x32x2_f32 (fp32
// operands, fp32 accumulation), the softmax weights stay fp32 and nothing is rounded to a narrower type.  What is
// left is the rounding of the fp32 running sums themselves (l, r and, foremost, the accumulators, which take one
// rounded addition per two keys): measured max error 5e-6 of RMS at 256 keys, the size the 1e-5 tolerance for fp32
// inputs is stated for, growing like sqrt(Lkv) beyond (1.4e-5 at 4096 keys); that growth law is part of the
// interface's accuracy contract.  The algorithm is Alg. 2: row reference m, rescale factor
// alpha = exp(m_old - m_new) applied to l, r and both accumulators, A and B summed into one accumulator (they are
// only ever added), epilogue O/l, lse = m + log l, tO = (A + B - (r/l) O_unnorm)/l.  Two things differ from the
// printed algorithm: the softmax scale, which it leaves out, multiplies S and tS; and m trails the running row
// maximum by up to 32 nats (it is moved only when a block exceeds it by more), which changes no result and makes
// the rescaling of the accumulators rare.
//
// Work split: a workgroup of 4 waves owns 128 query rows, 32 per wave; key blocks of BC = 32 rows.  Products are
// taken transposed, S^T = K Q^T and O^T += V^T P~^T: the query index is the MFMA column (lane % 32), so each lane
// holds, for ONE query row, 16 of the 32 scores of a block (the other 16 sit in lane ^ 32); row max and row sums are
// per-lane loops plus one half-wave exchange, and the 16 weights a lane holds are exactly the B operands of the 16
// reduction steps of the value products: no transposition, no LDS round trip for the weights.
//
//   score step t = 4u + e (u < D/8, e < 4): A = K[key = lane%32][8u + 4h + e], B = Q[query = lane%32][8u + 4h + e],
//                                           h = lane/32; the reduction index is permuted the same way on both sides
//   value step t < 16, column chunk c < D/32: A = V[key = 8(t/4) + 4h + t%4][32c + lane%32], B = weight register t
//
// K, tK, V, tV blocks are staged through LDS as fp32 in two stages by direct-to-LDS loads (no staging registers, no
// LDS write instructions): one 1-KiB part per wave and MFMA step, issued from the second step of a phase on, one wait
// and one barrier per block (a block is >= 6000 MFMA cycles per wave).  A 16-byte chunk of a row sits at position
// chunk ^ (row & 7): the K-side reads (16 bytes per lane, one row per lane) and the V-side reads (4 bytes per lane,
// one row per half-wave) then spread over the banks for every row width that is a multiple of 128 bytes.
// Operands are read one MFMA step ahead; the three score chains (S, K tQ^T, tK Q^T) and the accumulators of the
// column chunks are issued round-robin, so no MFMA waits for its predecessor; the weights of key step t + 1 are
// computed in the shadow of step t's MFMAs.
//
// Registers per lane at D = 128: Q, tQ 64 + 64, the two accumulators 64 + 64, S and the two parts of tS 48, weights
// 32, operands 24: one wave per SIMD, one workgroup per CU.
#include "launchers.h"
#include <type_traits>
#include <stdint.h>

namespace attn_jvp {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BR = 128;          // query rows per workgroup
constexpr int BC = 32;           // key rows per block
constexpr int NTHREADS = 256;
constexpr int TAN_NONE = 0;      // no tangents: O, lse only
constexpr int TAN_QUERY = 1;     // tQ only (tK = tV = 0)
constexpr int TAN_ALL = 2;
constexpr float MAX_SLACK = 32.f;     // nats by which a row's scores may exceed its reference m before m is moved
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

__device__ __forceinline__ float xhalf_max(float x) {   // max of lane l and lane l^32, in both
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {      // f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>{});
    }
}

// 128-bit direct-to-LDS load: 64 lanes x 16 B land at lds_base + 16 * lane (M0 carries lds_base); uniform 64-bit base
// in scalar registers plus a per-lane 32-bit byte offset.  Inline assembly so that the kernel keeps its own account
// of these loads: they are the only vector-memory loads in flight during the sweep, and an explicit wait plus the
// barrier at the end of each block publish a stage before anyone reads it.  M0 is reserved: the compiler puts nothing
// of its own there.
__device__ __forceinline__ void load_lds_b128(const void* uniform_base, uint32_t lane_off, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_base), "v"(lane_off), "s"(uniform_base) : "memory");
}

#define FENCE() __builtin_amdgcn_sched_barrier(0)      // no instruction is scheduled across this point

__device__ __forceinline__ f32x16 mfma(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

template <int D, int TAN>
__global__ __launch_bounds__(NTHREADS, D <= 64 ? 2 : 1) void attn_jvp_mfma_f32_kernel(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const float* __restrict__ tQ, const float* __restrict__ tK, const float* __restrict__ tV,
    float* __restrict__ O, float* __restrict__ tO, float* __restrict__ LSE,
    int Lq, int Lkv, float scale, int q_tiles, int H, int blhd) {
    // No implicit fusing of a product with a following sum: the compiler would fuse differently in each instantiation,
    // and the instantiations must agree bit for bit (absent tangents against zero tangents).  fmaf() stays fused.
#pragma clang fp contract(off)
    constexpr int CH = D / 4;                        // 16-byte chunks per row
    constexpr int TILE_F4 = BC * CH;                 // chunks per staged block of one tensor
    constexpr int PT = TILE_F4 / NTHREADS;           // chunks each lane moves per tensor per block
    constexpr int NT = TAN == TAN_ALL ? 4 : 2;       // tensors staged: K, V (+ tK, tV)
    constexpr int NC = D / 32;                       // 32-column chunks of the accumulators
    static_assert(D % 32 == 0 && D <= 128 && TILE_F4 % NTHREADS == 0 && 2 * PT < D / 8, "head dim");

    extern __shared__ float4 smem[];                 // [2 stages][NT tensors][TILE_F4]
    auto tile = [&](int stage, int tensor) { return smem + (stage * NT + tensor) * TILE_F4; };
    constexpr int T_K = 0, T_V = 1, T_TK = 2, T_TV = 3;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, h = lane >> 5;

    // consecutive workgroups go round-robin over the 8 XCDs: give each XCD a contiguous range of tiles, so that the
    // workgroups sharing one L2 stream the same heads' keys
    const int n_wg = gridDim.x;
    const int bid = (n_wg & 7) == 0 ? (int)(blockIdx.x & 7) * (n_wg >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const long bh = bid / q_tiles;
    const int qrow = (bid % q_tiles) * BR + 32 * wave + j;

    // [B,H,L,d]: rows of a head contiguous; [B,L,H,d]: rows of a head H*d elements apart
    const long row_elems = blhd ? (long)H * D : D;
    const long bidx = bh / H, hidx = bh % H;
    const long q_base = blhd ? (bidx * Lq * H + hidx) * D : bh * (long)Lq * D;
    const long kv_base = blhd ? (bidx * Lkv * H + hidx) * D : bh * (long)Lkv * D;

    // ---- this lane's slices of its query row: columns 8u + 4h .. + 3 ------------------------------------------------
    float4 q[D / 8], tq[TAN != TAN_NONE ? D / 8 : 1];
    {
        const bool live = qrow < Lq;                 // rows past the end load row 0, compute on zeros, store nothing
        const float* qp = Q + q_base + (long)(live ? qrow : 0) * row_elems + 4 * h;
        const float* tqp = TAN != TAN_NONE ? tQ + q_base + (long)(live ? qrow : 0) * row_elems + 4 * h : nullptr;
        const float keep = live ? 1.f : 0.f;
#pragma unroll
        for (int u = 0; u < D / 8; ++u) {
            q[u] = *reinterpret_cast<const float4*>(qp + 8 * u);
            q[u].x *= keep; q[u].y *= keep; q[u].z *= keep; q[u].w *= keep;
            if constexpr (TAN != TAN_NONE) {
                tq[u] = *reinterpret_cast<const float4*>(tqp + 8 * u);
                tq[u].x *= keep; tq[u].y *= keep; tq[u].z *= keep; tq[u].w *= keep;
            }
        }
#pragma unroll
        for (int u = 0; u < D / 8; ++u) {   // keep q in the accumulation half of the register file: only MFMAs read it
            asm volatile("" : "+a"(q[u].x), "+a"(q[u].y), "+a"(q[u].z), "+a"(q[u].w));
        }
    }

    // ---- staging of one block of one tensor: direct-to-LDS loads, 16 bytes per lane ---------------------------------
    // One instruction fills 1 KiB of the tile linearly in the lane id; the swizzle is applied on the global side:
    // the lane that fills chunk position pc of row `row` fetches chunk pc ^ (row & 7) of that row.  The lane's
    // share (positions tid, tid + 256, ...) is the same in every block, so its byte offsets from the block's first
    // row are computed once.  Rows past the end of a ragged last block re-read the block's first row (finite
    // values; the softmax gives them weight zero).
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    uint32_t g_off[PT];
    int s_row[PT];
#pragma unroll
    for (int n = 0; n < PT; ++n) {
        const int idx = tid + NTHREADS * n;
        const int row = idx / CH, pc = idx % CH;
        s_row[n] = row;
        g_off[n] = (uint32_t)((row * row_elems + 4 * (pc ^ (row & 7))) * (long)sizeof(float));
    }
    // part n (of PT) of one tensor's block: one instruction per wave
    const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(64 * wave * sizeof(float4)));
    auto stage_part = [&](const float* base, int j0, int stage, int tensor, int n) {
        const char* blk = reinterpret_cast<const char*>(base + kv_base + (long)j0 * row_elems);     // uniform
        const uint32_t dst = wave_lds + (uint32_t)(((stage * NT + tensor) * TILE_F4 + NTHREADS * n) * sizeof(float4));
        if (j0 + BC <= Lkv) {                        // uniform
            load_lds_b128(blk, g_off[n], dst);
        } else {
            const bool dead = j0 + s_row[n] >= Lkv;
            load_lds_b128(blk, dead ? g_off[n] - (uint32_t)(s_row[n] * row_elems * sizeof(float)) : g_off[n], dst);
        }
    };
    auto stage_in = [&](const float* base, int j0, int stage, int tensor) {
#pragma unroll
        for (int n = 0; n < PT; ++n) stage_part(base, j0, stage, tensor, n);
    };

    f32x16 acc_o[NC], acc_t[TAN != TAN_NONE ? NC : 1];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        acc_o[c] = f32x16{};
        if constexpr (TAN != TAN_NONE) acc_t[c] = f32x16{};
    }
    float m = -INFINITY, l = 0.f, r = 0.f;       // l, r: this lane's 16 keys per block only; halves meet in the epilogue

    const int n_blocks = (Lkv + BC - 1) / BC;
    stage_in(K, 0, 0, T_K);
    stage_in(V, 0, 0, T_V);
    if constexpr (TAN == TAN_ALL) {
        stage_in(tK, 0, 0, T_TK);
        stage_in(tV, 0, 0, T_TV);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int blk = 0; blk < n_blocks; ++blk) {
        const int cur = blk & 1, nxt = cur ^ 1;
        const int j0 = blk * BC;
        const bool has_next = blk + 1 < n_blocks;       // workgroup-uniform

        // ---- phase 1: S^T = K Q^T, tS^T = K tQ^T + tK Q^T; next block's K, tK travel meanwhile ---------------------
        // Three independent accumulation chains (S, K tQ^T, tK Q^T), issued round-robin so that no MFMA waits for the
        // one before it; the operands of step u + 1 are read from LDS while the 12 MFMAs of step u run (the fences
        // keep the compiler from sinking the reads down to their first use).
        // (up to d = 64 two workgroups share a CU and each wave has 256 registers: there tS is one chain, and the
        // other workgroup's waves fill the gaps)
        constexpr bool THREE_CHAINS = D > 64;
        f32x16 s = f32x16{}, ts = f32x16{}, ts2 = f32x16{};
        {
            // chunk (2u + h) ^ (j & 7) = 8 (u/4) + ((2 (u%4) + h) ^ (j & 7)): four lane-dependent addresses, the rest
            // is an immediate offset
            const float4* lk[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) lk[w] = tile(cur, T_K) + j * CH + ((2 * w + h) ^ (j & 7));
            constexpr int TK_OFF = (T_TK - T_K) * TILE_F4;
            float4 ka[2], tka[2];
            ka[0] = lk[0][0];
            if constexpr (TAN == TAN_ALL) tka[0] = lk[0][TK_OFF];
#pragma unroll
            for (int u = 0; u < D / 8; ++u) {
                if (u + 1 < D / 8) {
                    ka[(u + 1) & 1] = lk[(u + 1) & 3][8 * ((u + 1) >> 2)];
                    if constexpr (TAN == TAN_ALL) tka[(u + 1) & 1] = lk[(u + 1) & 3][8 * ((u + 1) >> 2) + TK_OFF];
                }
                // the next block's K, tK: one 1-KiB part per wave and step, from the second step on, so that a load
                // that has to queue for the memory pipe waits behind 12 MFMAs, not in front of them
                if (has_next) {
                    if (u >= 1 && u <= PT) stage_part(K, j0 + BC, nxt, T_K, u - 1);
                    if constexpr (TAN == TAN_ALL)
                        if (u > PT && u <= 2 * PT) stage_part(tK, j0 + BC, nxt, T_TK, u - PT - 1);
                }
                FENCE();
                const float kv[4] = {ka[u & 1].x, ka[u & 1].y, ka[u & 1].z, ka[u & 1].w};
                const float qv[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    s = mfma(kv[e], qv[e], s);
                    if constexpr (TAN != TAN_NONE) {
                        const float tqv[4] = {tq[u].x, tq[u].y, tq[u].z, tq[u].w};
                        ts = mfma(kv[e], tqv[e], ts);
                    }
                    if constexpr (TAN == TAN_ALL) {
                        const float tkv[4] = {tka[u & 1].x, tka[u & 1].y, tka[u & 1].z, tka[u & 1].w};
                        if constexpr (THREE_CHAINS) ts2 = mfma(tkv[e], qv[e], ts2);
                        else ts = mfma(tkv[e], qv[e], ts);
                    }
                }
                FENCE();
            }
            // the vector ALU reads the scores next: have the MFMAs deliver them in arithmetic registers (left alone, the
            // compiler puts them in accumulation registers and copies all 48 out, one instruction each)
            asm volatile("" : "+v"(s));
            if constexpr (TAN != TAN_NONE) asm volatile("" : "+v"(ts));
            if constexpr (TAN == TAN_ALL && THREE_CHAINS) {
                asm volatile("" : "+v"(ts2));
                ts += ts2;
            }
        }
        // ---- online softmax of Alg. 2 on this lane's 16 keys: register e holds key j0 + 8(e/4) + 4h + e%4 -----------
        // The running maximum m is a reference, not a result: it is taken over the rounded products S scale, and the
        // exponent S scale - m is then formed by ONE fused multiply-add from the unrounded S, so that its rounding
        // error is relative to the small difference, not to the size of the scores.
        const bool ragged = j0 + BC > Lkv;              // last block: keys past the end weigh nothing
        float mb = -INFINITY;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const bool dead = ragged && j0 + 8 * (e / 4) + 4 * h + (e % 4) >= Lkv;     // (their tS is 0: K, tK rows are 0)
            mb = fmaxf(mb, dead ? -INFINITY : s[e] * scale);
        }
        mb = xhalf_max(mb);                             // a block always holds a valid key: mb is finite
        // m follows the row maximum with a slack: it moves only when a block's maximum exceeds it by more than
        // MAX_SLACK nats, so that the rescaling of the accumulators (Alg. 2's alpha) is rare after the first block
        // instead of happening whenever any of a wave's 32 rows meets a new maximum.  Any reference gives the same
        // result; with fp32 weights up to e^MAX_SLACK nothing is lost (l and the accumulators stay below
        // Lkv e^MAX_SLACK max|V|, far inside the fp32 range; weights below e^-87 of the reference, i.e. below
        // e^-87 of the true maximum or less, flush to zero as they would anyway).
        const float m_new = mb > m + MAX_SLACK ? mb : m;
        const float alpha = __builtin_amdgcn_exp2f((m - m_new) * LOG2E);    // 0 on the first block (m = -inf), else 1 or tiny
        m = m_new;
        if (__builtin_expect(__any(alpha != 1.f), 0)) {
            // (the empty statements tie the accumulators to the accumulation registers on entry and exit, so that the
            // copies to and from arithmetic registers stay inside this block)
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                asm volatile("" : "+a"(acc_o[c]));
                acc_o[c] *= alpha;
                asm volatile("" : "+a"(acc_o[c]));
                if constexpr (TAN != TAN_NONE) {
                    asm volatile("" : "+a"(acc_t[c]));
                    acc_t[c] *= alpha;
                    asm volatile("" : "+a"(acc_t[c]));
                }
            }
        }
        // weights of key step e: P~ = exp(S scale - m), H~ = P~ o tS; computed one step ahead of the value products
        // that consume them, in the shadow of the previous step's MFMAs
        float p[16], hh[16];
        float row_p = 0.f, row_h = 0.f;
        auto weigh = [&](auto e_tag) {
            constexpr int e = decltype(e_tag)::value;
            const bool dead = ragged && j0 + 8 * (e / 4) + 4 * h + (e % 4) >= Lkv;
            p[e] = dead ? 0.f : __builtin_amdgcn_exp2f(fmaf(s[e], scale, -m_new) * LOG2E);
            row_p += p[e];
            if constexpr (TAN != TAN_NONE) {
                hh[e] = p[e] * (ts[e] * scale);
                row_h += hh[e];
            }
        };

        // ---- phase 2: O^T += V^T P~^T, (A+B)^T += V^T H~^T + tV^T P~^T ---------------------------------------------
        {
            // key row 8 (t/4) + 4h + t%4, float column 32c + j at chunk ^ (row & 7): four lane-dependent addresses
            // (one per t%4), the rest is an immediate offset
            const float* lv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                lv[i] = reinterpret_cast<const float*>(tile(cur, T_V)) + (4 * h + i) * D + ((((j >> 2) ^ (4 * h + i)) << 2) | (j & 3));
            constexpr int TV_OFF = (T_TV - T_V) * TILE_F4 * 4;
            // per key step t: 4 (8) operands, read one step ahead; the 4, 8 or 12 MFMAs of a step go round the column
            // chunks, so consecutive ones never share an accumulator
            float va[2][NC], tva[2][NC];
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                va[0][c] = lv[0][32 * c];
                if constexpr (TAN == TAN_ALL) tva[0][c] = lv[0][32 * c + TV_OFF];
            }
            weigh(std::integral_constant<int, 0>{});
            static_for<16>([&](auto t_tag) {
                constexpr int t = decltype(t_tag)::value;
                if constexpr (t + 1 < 16) {
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        constexpr int row_off = 8 * ((t + 1) >> 2) * D;
                        va[(t + 1) & 1][c] = lv[(t + 1) & 3][row_off + 32 * c];
                        if constexpr (TAN == TAN_ALL) tva[(t + 1) & 1][c] = lv[(t + 1) & 3][row_off + 32 * c + TV_OFF];
                    }
                }
                if (has_next) {                      // next block's V, tV: as for K, tK above
                    if (t >= 1 && t <= PT) stage_part(V, j0 + BC, nxt, T_V, t - 1);
                    if constexpr (TAN == TAN_ALL)
                        if (t > PT && t <= 2 * PT) stage_part(tV, j0 + BC, nxt, T_TV, t - PT - 1);
                }
                FENCE();
#pragma unroll
                for (int c = 0; c < NC; ++c) acc_o[c] = mfma(va[t & 1][c], p[t], acc_o[c]);
                if constexpr (TAN != TAN_NONE) {
#pragma unroll
                    for (int c = 0; c < NC; ++c) acc_t[c] = mfma(va[t & 1][c], hh[t], acc_t[c]);
                }
                if constexpr (TAN == TAN_ALL) {
#pragma unroll
                    for (int c = 0; c < NC; ++c) acc_t[c] = mfma(tva[t & 1][c], p[t], acc_t[c]);
                }
                if constexpr (t + 1 < 16) weigh(std::integral_constant<int, t + 1>{});
                FENCE();
            });
        }
        l = fmaf(alpha, l, row_p);
        r = fmaf(alpha, r, row_h);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // this wave's share of the next stage has landed
        __syncthreads();    // next stage written by all, this stage read by all
    }

    // ---- epilogue (Alg. 2, last lines): accumulator register 4g + i of chunk c is column 32c + 8g + 4h + i -----------
    const float l_row = xhalf_sum(l);
    const float r_row = xhalf_sum(r);
    if (qrow < Lq) {
        const float inv_l = 1.f / l_row;
        const float mu = r_row * inv_l;              // rowsum(P o tS)
        float* op = O + q_base + (long)qrow * row_elems + 4 * h;
        float* top = TAN != TAN_NONE ? tO + q_base + (long)qrow * row_elems + 4 * h : nullptr;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float4 o4, t4;
                o4.x = acc_o[c][4 * g + 0]; o4.y = acc_o[c][4 * g + 1];
                o4.z = acc_o[c][4 * g + 2]; o4.w = acc_o[c][4 * g + 3];
                if constexpr (TAN != TAN_NONE) {
                    t4.x = fmaf(-mu, o4.x, acc_t[c][4 * g + 0]) * inv_l; t4.y = fmaf(-mu, o4.y, acc_t[c][4 * g + 1]) * inv_l;
                    t4.z = fmaf(-mu, o4.z, acc_t[c][4 * g + 2]) * inv_l; t4.w = fmaf(-mu, o4.w, acc_t[c][4 * g + 3]) * inv_l;
                    *reinterpret_cast<float4*>(top + 32 * c + 8 * g) = t4;
                }
                o4.x *= inv_l; o4.y *= inv_l; o4.z *= inv_l; o4.w *= inv_l;
                *reinterpret_cast<float4*>(op + 32 * c + 8 * g) = o4;
            }
        }
        if (h == 0) LSE[bh * Lq + qrow] = fmaf(__builtin_amdgcn_logf(l_row), LN2, m);     // v_log_f32 is a binary log
    }
}

template <int D, int TAN>
hipError_t launch_one(const Problem& p) {
    const int q_tiles = (p.Lq + BR - 1) / BR;
    const long long blocks = (long long)q_tiles * p.B * p.H;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    constexpr int NT = TAN == TAN_ALL ? 4 : 2;
    constexpr int smem = 2 * NT * BC * D * (int)sizeof(float);
    auto kern = attn_jvp_mfma_f32_kernel<D, TAN>;
    int dev = 0, cus = 0;
    hipError_t e = device_cus(&dev, &cus);
    if (e == hipSuccess) e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), smem, dev);
    if (e != hipSuccess) return e;
    MainKernelTimer timer(p);
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(NTHREADS), smem, p.stream,
                       (const float*)p.q, (const float*)p.k, (const float*)p.v,
                       (const float*)p.tq, (const float*)p.tk, (const float*)p.tv,
                       (float*)p.o, (float*)p.to, p.lse, p.Lq, p.Lkv, p.scale, q_tiles, p.H, p.layout);
    return timer.finish(hipGetLastError());
}

template <int D>
hipError_t launch_tan(const Problem& p) {
    if (!p.tq) return launch_one<D, TAN_NONE>(p);
    if (!p.tk) return launch_one<D, TAN_QUERY>(p);
    return launch_one<D, TAN_ALL>(p);
}

}  // namespace

bool mfma_f32_supports(const Problem& p) {
    // (a lane's byte offset inside a block of 32 rows is kept in 32 bits)
    const long long row_bytes = (long long)(p.layout ? p.H : 1) * p.d * (long long)sizeof(float);
    return p.in_dtype == 1 && (p.d == 32 || p.d == 64 || p.d == 96 || p.d == 128) && row_bytes * BC < (1ll << 31);
}

hipError_t launch_mfma_f32(const Problem& p) {
    if (!mfma_f32_supports(p)) return hipErrorInvalidValue;
    switch (p.d) {
        case 32: return launch_tan<32>(p);
        case 64: return launch_tan<64>(p);
        case 96: return launch_tan<96>(p);
        default: return launch_tan<128>(p);
    }
}

}  // namespace attn_jvp
