// bf16 matrix-core (MFMA) streaming kernel for attention forward + JVP (paper Alg. 2), d = 128.
//
// One workgroup = 4 wavefronts = 128 query rows; each wavefront owns 32 query rows for the whole
// key/value sweep.  All six contractions of Alg. 2's inner loop run on v_mfma_f32_32x32x16_bf16
// in the TRANSPOSED orientation: S^T = K Q^T, tS^T = K tQ^T + tK Q^T, O^T += V^T P~^T,
// (A+B)^T += tV^T P~^T + V^T H~^T.  In that orientation a lane's MFMA result registers all belong
// to ONE query (column = lane % 32), so
//   * row max / row sums are in-lane reductions plus one exchange between lane l and l^32,
//   * the rescale factor exp(m_old - m_new) is a per-lane scalar,
//   * P~^T and H~^T feed the next MFMA as its B operand straight from registers (the contraction
//     index - the key position - may be enumerated in any order as long as both operands agree,
//     and V^T is fetched from LDS in exactly the order the result registers happen to hold).
// A and B of Alg. 2 share one accumulator: they carry the same rescale factor and are only added.
//
// Key/value tiles (K, tK, V, tV: 64 rows x 128 bf16 each) are copied HBM -> LDS with 128-bit
// direct-to-LDS loads, double buffered (2 x 64 KiB), XOR-swizzled so that both the row-wise
// 128-bit reads (K, tK as MFMA A operand) and the transposing 64-bit reads (V, tV) spread over
// all banks.  Q and tQ fragments stay in registers.
//
// Numerics: bf16 operands, fp32 accumulation; softmax in base 2 with scale*log2(e) folded into one
// FMA; the running maximum m is raised only when some row's tile maximum exceeds it (wave-uniform
// branch), which is Alg. 2's update whenever it fires and leaves m_new = m_old otherwise.
// H~ = P~ o tS is formed as P~ o (tS - ctr) with a per-row constant ctr that follows the running value of
// rowsum(P o tS): tP does not change when a constant is added to a row of tS, and a small |tS - ctr| on
// the keys that carry the weight keeps the bf16 rounding of H~ from surviving the B - r O cancellation.
#include "launchers.h"
#include <hip/hip_bf16.h>
#include <stdint.h>

namespace attn_jvp {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int D = 128;
constexpr int BR = 128;              // query rows per workgroup (32 per wavefront)
constexpr int BC = 64;               // key rows per LDS stage
constexpr int NTHREADS = 256;
constexpr int ROW_BYTES = D * 2;     // 256
constexpr int TILE_BYTES = BC * ROW_BYTES;   // 16 KiB per tensor per stage
constexpr int STAGE_BYTES = 4 * TILE_BYTES;  // K, tK, V, tV
constexpr int LDS_BYTES = 2 * STAGE_BYTES;   // 128 KiB

typedef __attribute__((address_space(3))) char lds_char;

__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr) {
    return *reinterpret_cast<__attribute__((address_space(3))) const bf16x8*>((uintptr_t)addr);
}
__device__ __forceinline__ s16x4 lds_read_tr_b64(uint32_t addr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        reinterpret_cast<__attribute__((address_space(3))) s16x4*>((uintptr_t)addr));
}
__device__ __forceinline__ float xhalf_max(float x) {   // max of lane l and lane l^32, in both
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
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

// Copy one 64-row tile of one tensor into LDS.  Each direct-to-LDS instruction moves 64 x 16 B =
// 4 rows; the LDS side is linear in the lane id, so the swizzle is applied by choosing which
// 16-byte chunk of the row each lane fetches.  vswz = false: chunk ^= row & 15 (row-wise b128
// reads); vswz = true: chunk ^= (row & 3) << 2 (transposing b64 reads).  Rows past Lkv re-read
// the last valid row (finite values; their scores are masked to -inf).
template <bool VSWZ>
__device__ __forceinline__ void issue_tile_load(const char* gbase, int j0, int Lkv, uint32_t lds_tensor_base,
                                                int wave, int lane) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int rowblk = wave * 4 + i;
        const int row = rowblk * 4 + (lane >> 4);
        const int pc = lane & 15;
        const int lc = VSWZ ? (pc ^ ((row & 3) << 2)) : (pc ^ (row & 15));
        int grow = j0 + row;
        grow = grow < Lkv ? grow : Lkv - 1;
        const char* g = gbase + (long)grow * ROW_BYTES + lc * 16;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                         (__attribute__((address_space(3))) void*)(uintptr_t)(lds_tensor_base + rowblk * 1024),
                                         16, 0, 0);
    }
}

// SPLIT: P~ (for O) and H~ (for B) enter their contractions as hi + lo bf16 terms, two more MFMAs per V fragment:
// 8 matrix products per key tile instead of Alg. 2's 6, in exchange for ~16-bit instead of 8-bit weights.
template <bool SPLIT>
__global__ __launch_bounds__(NTHREADS, 1) void attn_jvp_mfma_kernel(
    const __hip_bfloat16* __restrict__ Q, const __hip_bfloat16* __restrict__ K, const __hip_bfloat16* __restrict__ V,
    const __hip_bfloat16* __restrict__ tQ, const __hip_bfloat16* __restrict__ tK, const __hip_bfloat16* __restrict__ tV,
    float* __restrict__ O, float* __restrict__ tO, float* __restrict__ LSE,
    int Lq, int Lkv, float scale, int q_tiles) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c = lane & 31;          // query column of this lane in every MFMA result
    const int g = lane >> 5;          // which half of the contraction index this lane feeds

    const int bid = blockIdx.x;
    const long bh = bid / q_tiles;
    const int q0 = (bid % q_tiles) * BR + wave * 32;

    const char* Kh = reinterpret_cast<const char*>(K) + bh * (long)Lkv * ROW_BYTES;
    const char* tKh = reinterpret_cast<const char*>(tK) + bh * (long)Lkv * ROW_BYTES;
    const char* Vh = reinterpret_cast<const char*>(V) + bh * (long)Lkv * ROW_BYTES;
    const char* tVh = reinterpret_cast<const char*>(tV) + bh * (long)Lkv * ROW_BYTES;

    const int n_tiles = (Lkv + BC - 1) / BC;

    // prefetch tile 0 while Q is being fetched
    issue_tile_load<false>(Kh, 0, Lkv, lds0 + 0 * TILE_BYTES, wave, lane);
    issue_tile_load<false>(tKh, 0, Lkv, lds0 + 1 * TILE_BYTES, wave, lane);
    issue_tile_load<true>(Vh, 0, Lkv, lds0 + 2 * TILE_BYTES, wave, lane);
    issue_tile_load<true>(tVh, 0, Lkv, lds0 + 3 * TILE_BYTES, wave, lane);

    // Q^T / tQ^T as MFMA B operand: lane (c, g) holds row q0+c, elements 16t + 8g .. +7
    const int qrow = q0 + c;
    const int qrow_ld = qrow < Lq ? qrow : Lq - 1;
    bf16x8 qf[8], tqf[8];
    {
        const bf16x8* qp = reinterpret_cast<const bf16x8*>(Q + (bh * Lq + qrow_ld) * D + 8 * g);
        const bf16x8* tqp = reinterpret_cast<const bf16x8*>(tQ + (bh * Lq + qrow_ld) * D + 8 * g);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            qf[t] = qp[2 * t];
            tqf[t] = tqp[2 * t];
        }
    }

    // per-lane LDS read offsets (relative to a tensor's tile base)
    uint32_t kaddr[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) kaddr[t] = c * ROW_BYTES + (((2 * t + g) ^ (c & 15)) << 4);
    uint32_t vaddr[4];
    {
        const int i = lane & 15, hb = (lane >> 4) & 1;
        const uint32_t rowpart = (4 * g + (i >> 2)) * ROW_BYTES + (2 * hb + ((i & 3) >> 1)) * 16 + 8 * (i & 1);
#pragma unroll
        for (int db = 0; db < 4; ++db) vaddr[db] = rowpart + ((db ^ (i >> 2)) << 6);
    }

    f32x16 accO[4], accAB[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) { accO[db][e] = 0.f; accAB[db][e] = 0.f; }

    const float c2 = scale * 1.4426950408889634f;   // scores -> base-2 exponent
    float m = -INFINITY;      // running max of c2 * s_raw, identical in lanes l and l^32
    float l_part = 0.f;       // this lane's share of the row sum of P~
    float r_part = 0.f;       // this lane's share of the row sum of H~ = P~ o (tS - ctr)
    float ctr = 0.f;          // per-row constant subtracted from tS before H~ is rounded to bf16

    for (int j = 0; j < n_tiles; ++j) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();   // tile j is in LDS for every wave; every wave is done with the other stage
        if (j + 1 < n_tiles) {
            const uint32_t nb = lds0 + ((j + 1) & 1) * STAGE_BYTES;
            const int j0n = (j + 1) * BC;
            issue_tile_load<false>(Kh, j0n, Lkv, nb + 0 * TILE_BYTES, wave, lane);
            issue_tile_load<false>(tKh, j0n, Lkv, nb + 1 * TILE_BYTES, wave, lane);
            issue_tile_load<true>(Vh, j0n, Lkv, nb + 2 * TILE_BYTES, wave, lane);
            issue_tile_load<true>(tVh, j0n, Lkv, nb + 3 * TILE_BYTES, wave, lane);
        }
        const uint32_t sb = lds0 + (j & 1) * STAGE_BYTES;
        const bool tail = (j + 1) * BC > Lkv;

#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            // ---- scores: S^T, tS^T for 32 keys x 32 queries
            f32x16 s, ts;
#pragma unroll
            for (int e = 0; e < 16; ++e) { s[e] = 0.f; ts[e] = 0.f; }
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const bf16x8 kf = lds_read_b128(sb + 0 * TILE_BYTES + kb * 32 * ROW_BYTES + kaddr[t]);
                const bf16x8 tkf = lds_read_b128(sb + 1 * TILE_BYTES + kb * 32 * ROW_BYTES + kaddr[t]);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], s, 0, 0, 0);
                ts = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, tqf[t], ts, 0, 0, 0);
                ts = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tkf, qf[t], ts, 0, 0, 0);
            }
            if (tail) {   // keys past Lkv: score -inf (P~ = 0), tangent score 0
                const int jbase = j * BC + kb * 32 + 4 * g;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int jj = jbase + 8 * (e >> 2) + (e & 3);
                    if (jj >= Lkv) { s[e] = -INFINITY; ts[e] = 0.f; }
                }
            }
            // ---- online softmax (base 2) with re-centred tangent scores
            float tmax = s[0];
#pragma unroll
            for (int e = 1; e < 16; ++e) tmax = fmaxf(tmax, s[e]);
            tmax = xhalf_max(tmax) * c2;
            const bool raise = __builtin_amdgcn_ballot_w64(tmax > m) != 0;   // wave-uniform
            float alpha = 1.f;
            if (raise) {
                const float m_new = fmaxf(m, tmax);
                alpha = __builtin_amdgcn_exp2f(m - m_new);   // exp2(-inf) = 0 on the first block
                m = m_new;
            }
            float p[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) p[e] = __builtin_amdgcn_exp2f(fmaf(s[e], c2, -m));
            if (raise) {
                // Some row's maximum moved, so every accumulator is touched anyway: use the pass to move the
                // centring constant ctr of ALL 32 rows to the current estimate of mu = rowsum(P o tS) (this block
                // included, taken before H~ is rounded).  Exact in real arithmetic for any ctr:
                //   sum_j P~_j (tS_j - ctr_new) V_j = sum_j P~_j (tS_j - ctr_old) V_j - (ctr_new - ctr_old) O~.
                float lb = 0.f, rb = 0.f;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    lb += p[e];
                    rb = fmaf(p[e], fmaf(ts[e], scale, -ctr), rb);
                }
                l_part *= alpha;
                r_part *= alpha;
                const float l_row = xhalf_sum(l_part + lb);
                const float r_row = xhalf_sum(r_part + rb);
                const float delta = r_row / l_row;          // mu estimate minus ctr
                ctr += delta;
                r_part = fmaf(-delta, l_part, r_part);
                const float da = delta * alpha;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        accAB[db][e] = fmaf(accAB[db][e], alpha, -da * accO[db][e]);
                        accO[db][e] *= alpha;
                    }
            }
            uint32_t pp[8], pq[8], hp[8], hq[8];   // P~^T, H~^T (hi, lo) as packed bf16 pairs, in result-register order
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                const float h0 = p[e] * fmaf(ts[e], scale, -ctr);
                const float h1 = p[e + 1] * fmaf(ts[e + 1], scale, -ctr);
                l_part += p[e] + p[e + 1];
                r_part += h0 + h1;
                if (SPLIT) {
                    // hi = x rounded to bf16, lo = x - hi (exact in fp32) rounded to bf16
                    const uint32_t ph = pack_bf16(p[e], p[e + 1]);
                    pp[e >> 1] = ph;
                    pq[e >> 1] = pack_bf16(p[e] - __uint_as_float(ph << 16), p[e + 1] - __uint_as_float(ph & 0xffff0000u));
                    const uint32_t hh = pack_bf16(h0, h1);
                    hp[e >> 1] = hh;
                    hq[e >> 1] = pack_bf16(h0 - __uint_as_float(hh << 16), h1 - __uint_as_float(hh & 0xffff0000u));
                } else {
                    pp[e >> 1] = pack_bf16(p[e], p[e + 1]);
                    hp[e >> 1] = pack_bf16(h0, h1);
                }
            }
            // ---- value contractions
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
                u32x4 pu = {pp[4 * t2], pp[4 * t2 + 1], pp[4 * t2 + 2], pp[4 * t2 + 3]};
                u32x4 hu = {hp[4 * t2], hp[4 * t2 + 1], hp[4 * t2 + 2], hp[4 * t2 + 3]};
                const bf16x8 pb = __builtin_bit_cast(bf16x8, pu);
                const bf16x8 hb8 = __builtin_bit_cast(bf16x8, hu);
                bf16x8 hl8 = hb8, pl8 = pb;
                if (SPLIT) {
                    u32x4 lu = {hq[4 * t2], hq[4 * t2 + 1], hq[4 * t2 + 2], hq[4 * t2 + 3]};
                    hl8 = __builtin_bit_cast(bf16x8, lu);
                    u32x4 ql = {pq[4 * t2], pq[4 * t2 + 1], pq[4 * t2 + 2], pq[4 * t2 + 3]};
                    pl8 = __builtin_bit_cast(bf16x8, ql);
                }
                const uint32_t rb = sb + (kb * 32 + t2 * 16) * ROW_BYTES;
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const s16x4 v0 = lds_read_tr_b64(rb + 2 * TILE_BYTES + vaddr[db]);
                    const s16x4 v1 = lds_read_tr_b64(rb + 2 * TILE_BYTES + 8 * ROW_BYTES + vaddr[db]);
                    const s16x4 w0 = lds_read_tr_b64(rb + 3 * TILE_BYTES + vaddr[db]);
                    const s16x4 w1 = lds_read_tr_b64(rb + 3 * TILE_BYTES + 8 * ROW_BYTES + vaddr[db]);
                    typedef __attribute__((ext_vector_type(8))) short s16x8;
                    const s16x8 vv = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
                    const s16x8 ww = __builtin_shufflevector(w0, w1, 0, 1, 2, 3, 4, 5, 6, 7);
                    const bf16x8 vf = __builtin_bit_cast(bf16x8, vv);
                    const bf16x8 tvf = __builtin_bit_cast(bf16x8, ww);
                    accO[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb, accO[db], 0, 0, 0);
                    accAB[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tvf, pb, accAB[db], 0, 0, 0);
                    accAB[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, hb8, accAB[db], 0, 0, 0);
                    if (SPLIT) {
                        accO[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pl8, accO[db], 0, 0, 0);
                        accAB[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, hl8, accAB[db], 0, 0, 0);
                    }
                }
            }
        }
    }

    // ---- epilogue: O = O~/l, lse = m + log l, tO = (A + B - (r/l) O~) / l  (r and B both relative to ctr)
    const float l_row = xhalf_sum(l_part);
    const float r_row = xhalf_sum(r_part);
    const float inv_l = 1.f / l_row;
    const float mu = r_row * inv_l;
    if (qrow < Lq) {
        float* Op = O + (bh * Lq + qrow) * D + 4 * g;
        float* tOp = tO + (bh * Lq + qrow) * D + 4 * g;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                float4 o4, t4;
                const float a0 = accO[db][4 * v4], a1 = accO[db][4 * v4 + 1], a2 = accO[db][4 * v4 + 2], a3 = accO[db][4 * v4 + 3];
                o4.x = a0 * inv_l; o4.y = a1 * inv_l; o4.z = a2 * inv_l; o4.w = a3 * inv_l;
                t4.x = (accAB[db][4 * v4] - mu * a0) * inv_l;
                t4.y = (accAB[db][4 * v4 + 1] - mu * a1) * inv_l;
                t4.z = (accAB[db][4 * v4 + 2] - mu * a2) * inv_l;
                t4.w = (accAB[db][4 * v4 + 3] - mu * a3) * inv_l;
                *reinterpret_cast<float4*>(Op + 32 * db + 8 * v4) = o4;
                *reinterpret_cast<float4*>(tOp + 32 * db + 8 * v4) = t4;
            }
        if (g == 0) LSE[bh * Lq + qrow] = (m + __builtin_amdgcn_logf(l_row)) * 0.6931471805599453f;
    }
}

}  // namespace

bool mfma_bf16_supports(const Problem& p) {
    return p.in_dtype == 0 && p.out_dtype == 0 && p.d == D;
}

hipError_t launch_mfma_bf16(const Problem& p) {
    if (!mfma_bf16_supports(p)) return hipErrorInvalidValue;
    const int q_tiles = (p.Lq + BR - 1) / BR;
    const long long blocks = (long long)q_tiles * p.B * p.H;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    auto launch = [&](auto kern) -> hipError_t {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(NTHREADS), LDS_BYTES, p.stream,
                           (const __hip_bfloat16*)p.q, (const __hip_bfloat16*)p.k, (const __hip_bfloat16*)p.v,
                           (const __hip_bfloat16*)p.tq, (const __hip_bfloat16*)p.tk, (const __hip_bfloat16*)p.tv,
                           (float*)p.o, (float*)p.to, p.lse, p.Lq, p.Lkv, p.scale, q_tiles);
        return hipGetLastError();
    };
    if (p.flags & 1) return launch(attn_jvp_mfma_kernel<false>);
    return launch(attn_jvp_mfma_kernel<true>);
}

}  // namespace attn_jvp
