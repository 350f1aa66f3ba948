// fp32 matrix-core streaming kernel for attention forward + JVP (paper App. C.1, Alg. 2) on gfx950.
//
// The path for fp32 inputs at head dims 32, 64, 96, 128: every product runs on v_mfma_f32_32x32x2_f32 (fp32
// operands, fp32 accumulation), the softmax weights stay fp32 and nothing is rounded to a narrower type, so the
// fp32 tolerance is met at matrix-core speed.  The algorithm is Alg. 2 as printed: running row max m, rescale factor
// alpha = exp(m_old - m_new) applied to l, r and both accumulators, A and B summed into one accumulator (they are
// only ever added), epilogue O/l, lse = m + log l, tO = (A + B - (r/l) O_unnorm)/l.  The softmax scale, which
// Alg. 2 leaves out, multiplies S and tS.
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
// K, tK, V, tV blocks are staged through LDS as fp32 in two stages: global -> registers at the start of a phase,
// registers -> LDS at its end, one barrier per block (a block is >= 6000 MFMA cycles per wave, so neither the loads
// nor the barrier are on the critical path).  16-byte chunks of a row are stored at chunk ^ (row & 7): the K-side
// reads (16 bytes per lane, one row per lane) and the V-side reads (4 bytes per lane, one row per half-wave) are
// then free of bank conflicts for every row width that is a multiple of 128 bytes.
//
// Registers per lane at D = 128: Q, tQ 64 + 64, the two accumulators 64 + 64, S, tS (overwritten by P~, H~) 32,
// staging 32: one wave per SIMD, one workgroup per CU.
#include "launchers.h"

namespace attn_jvp {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BR = 128;          // query rows per workgroup
constexpr int BC = 32;           // key rows per block
constexpr int NTHREADS = 256;
constexpr int TAN_NONE = 0;      // no tangents: O, lse only
constexpr int TAN_QUERY = 1;     // tQ only (tK = tV = 0)
constexpr int TAN_ALL = 2;
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
__device__ __forceinline__ f32x16 mfma(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

template <int D, int TAN>
__global__ __launch_bounds__(NTHREADS) void attn_jvp_mfma_f32_kernel(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const float* __restrict__ tQ, const float* __restrict__ tK, const float* __restrict__ tV,
    float* __restrict__ O, float* __restrict__ tO, float* __restrict__ LSE,
    int Lq, int Lkv, float scale, int q_tiles, int H, int blhd) {
    constexpr int CH = D / 4;                        // 16-byte chunks per row
    constexpr int TILE_F4 = BC * CH;                 // chunks per staged block of one tensor
    constexpr int PT = TILE_F4 / NTHREADS;           // chunks each lane moves per tensor per block
    constexpr int NT = TAN == TAN_ALL ? 4 : 2;       // tensors staged: K, V (+ tK, tV)
    constexpr int NC = D / 32;                       // 32-column chunks of the accumulators
    static_assert(D % 32 == 0 && D <= 128 && TILE_F4 % NTHREADS == 0, "head dim");

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
        for (int u = 0; u < D / 8; ++u) {   // keep them in the accumulation half of the register file: only MFMAs read them
            asm volatile("" : "+a"(q[u].x), "+a"(q[u].y), "+a"(q[u].z), "+a"(q[u].w));
            if constexpr (TAN != TAN_NONE) asm volatile("" : "+a"(tq[u].x), "+a"(tq[u].y), "+a"(tq[u].z), "+a"(tq[u].w));
        }
    }

    // ---- staging of one block of one tensor: coalesced 16-byte global reads, swizzled LDS writes -------------------
    auto fetch = [&](const float* base, int j0, float4 (&regs)[PT]) {
#pragma unroll
        for (int n = 0; n < PT; ++n) {
            const int idx = tid + NTHREADS * n;
            const int row = idx / CH, ch = idx % CH;
            const int krow = j0 + row < Lkv ? j0 + row : Lkv - 1;     // rows past the end: any valid row (zeroed in stash)
            regs[n] = *reinterpret_cast<const float4*>(base + kv_base + (long)krow * row_elems + 4 * ch);
        }
    };
    auto stash = [&](float4* dst, int j0, const float4 (&regs)[PT]) {
#pragma unroll
        for (int n = 0; n < PT; ++n) {
            const int idx = tid + NTHREADS * n;
            const int row = idx / CH, ch = idx % CH;
            const bool live = j0 + row < Lkv;        // rows past the end are stored as zeros and masked in the softmax
            float4 v = regs[n];
            v.x = live ? v.x : 0.f; v.y = live ? v.y : 0.f; v.z = live ? v.z : 0.f; v.w = live ? v.w : 0.f;
            dst[row * CH + (ch ^ (row & 7))] = v;
        }
    };

    f32x16 acc_o[NC], acc_t[TAN != TAN_NONE ? NC : 1];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        acc_o[c] = f32x16{};
        if constexpr (TAN != TAN_NONE) acc_t[c] = f32x16{};
    }
    float m = -INFINITY, l = 0.f, r = 0.f;       // l, r: this lane's 16 keys per block only; halves meet in the epilogue

    const int n_blocks = (Lkv + BC - 1) / BC;
    {
        float4 a[PT], b[PT];
        fetch(K, 0, a);
        fetch(V, 0, b);
        stash(tile(0, T_K), 0, a);
        stash(tile(0, T_V), 0, b);
        if constexpr (TAN == TAN_ALL) {
            fetch(tK, 0, a);
            fetch(tV, 0, b);
            stash(tile(0, T_TK), 0, a);
            stash(tile(0, T_TV), 0, b);
        }
    }
    __syncthreads();

    for (int blk = 0; blk < n_blocks; ++blk) {
        const int cur = blk & 1, nxt = cur ^ 1;
        const int j0 = blk * BC;
        const bool has_next = blk + 1 < n_blocks;       // workgroup-uniform
        float4 st_a[PT], st_b[PT];

        // ---- phase 1: S^T = K Q^T, tS^T = K tQ^T + tK Q^T; next block's K, tK travel meanwhile ---------------------
        if (has_next) {
            fetch(K, j0 + BC, st_a);
            if constexpr (TAN == TAN_ALL) fetch(tK, j0 + BC, st_b);
        }
        f32x16 s = f32x16{}, ts = f32x16{};
        {
            // chunk (2u + h) ^ (j & 7) = 8 (u/4) + ((2 (u%4) + h) ^ (j & 7)): four lane-dependent addresses, the rest
            // is an immediate offset
            const float4* lk[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) lk[w] = tile(cur, T_K) + j * CH + ((2 * w + h) ^ (j & 7));
            constexpr int TK_OFF = (T_TK - T_K) * TILE_F4;
#pragma unroll
            for (int u = 0; u < D / 8; ++u) {
                const float4 ka = lk[u & 3][8 * (u >> 2)];
                float4 tka;
                if constexpr (TAN == TAN_ALL) tka = lk[u & 3][8 * (u >> 2) + TK_OFF];
                const float kv[4] = {ka.x, ka.y, ka.z, ka.w};
                const float qv[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    s = mfma(kv[e], qv[e], s);
                    if constexpr (TAN != TAN_NONE) {
                        const float tqv[4] = {tq[u].x, tq[u].y, tq[u].z, tq[u].w};
                        ts = mfma(kv[e], tqv[e], ts);
                    }
                    if constexpr (TAN == TAN_ALL) {
                        const float tkv[4] = {tka.x, tka.y, tka.z, tka.w};
                        ts = mfma(tkv[e], qv[e], ts);
                    }
                }
            }
        }
        if (has_next) {
            stash(tile(nxt, T_K), j0 + BC, st_a);
            if constexpr (TAN == TAN_ALL) stash(tile(nxt, T_TK), j0 + BC, st_b);
        }

        // ---- online softmax of Alg. 2 on this lane's 16 keys: register e holds key j0 + 8(e/4) + 4h + e%4 -----------
        if (has_next) {
            fetch(V, j0 + BC, st_a);
            if constexpr (TAN == TAN_ALL) fetch(tV, j0 + BC, st_b);
        }
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
        const float m_new = fmaxf(m, mb);
        const float alpha = __builtin_amdgcn_exp2f((m - m_new) * LOG2E);    // 0 on the first block (m = -inf)
        m = m_new;
        if (__builtin_expect(__any(alpha != 1.f), 0)) {     // rare after the first blocks
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
        float p[16], hh[16];
        float row_p = 0.f, row_h = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const bool dead = ragged && j0 + 8 * (e / 4) + 4 * h + (e % 4) >= Lkv;
            p[e] = dead ? 0.f : __builtin_amdgcn_exp2f(fmaf(s[e], scale, -m_new) * LOG2E);
            row_p += p[e];
            if constexpr (TAN != TAN_NONE) {
                hh[e] = p[e] * (ts[e] * scale);
                row_h += hh[e];
            }
        }
        l = fmaf(alpha, l, row_p);
        r = fmaf(alpha, r, row_h);

        // ---- phase 2: O^T += V^T P~^T, (A+B)^T += V^T H~^T + tV^T P~^T ---------------------------------------------
        {
            // key row 8 (t/4) + 4h + t%4, float column 32c + j at chunk ^ (row & 7): four lane-dependent addresses
            // (one per t%4), the rest is an immediate offset
            const float* lv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                lv[i] = reinterpret_cast<const float*>(tile(cur, T_V)) + (4 * h + i) * D + ((((j >> 2) ^ (4 * h + i)) << 2) | (j & 3));
            constexpr int TV_OFF = (T_TV - T_V) * TILE_F4 * 4;
#pragma unroll
            for (int t = 0; t < 16; ++t) {
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int off = 8 * (t >> 2) * D + 32 * c;
                    const float va = lv[t & 3][off];
                    acc_o[c] = mfma(va, p[t], acc_o[c]);
                    if constexpr (TAN != TAN_NONE) acc_t[c] = mfma(va, hh[t], acc_t[c]);
                    if constexpr (TAN == TAN_ALL) acc_t[c] = mfma(lv[t & 3][off + TV_OFF], p[t], acc_t[c]);
                }
            }
        }
        if (has_next) {
            stash(tile(nxt, T_V), j0 + BC, st_a);
            if constexpr (TAN == TAN_ALL) stash(tile(nxt, T_TV), j0 + BC, st_b);
        }
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
                    t4.x = (acc_t[c][4 * g + 0] - mu * o4.x) * inv_l; t4.y = (acc_t[c][4 * g + 1] - mu * o4.y) * inv_l;
                    t4.z = (acc_t[c][4 * g + 2] - mu * o4.z) * inv_l; t4.w = (acc_t[c][4 * g + 3] - mu * o4.w) * inv_l;
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
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
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
    return p.in_dtype == 1 && (p.d == 32 || p.d == 64 || p.d == 96 || p.d == 128);
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
