// fp32 vector-ALU streaming kernel for attention forward + JVP (paper Alg. 2).
//
// Reference-grade GPU path: every product and sum is an fp32 FMA on the vector ALU, so it meets
// the fp32 tolerance, and it accepts bf16 inputs too (upcast exactly).  It is the path for fp32
// inputs and head dims the matrix-core kernel does not cover; it is not tuned for speed.
//
// Work split: a workgroup of 256 lanes owns BR = 64 query rows (16 for d = 256); each row is shared by 4 (16)
// neighbouring lanes, lane part p holding the float4 chunks p, p+4, p+8, ... of q, tq and of the
// accumulators.  Key/value tiles of BC = 32 rows (K, tK, V, tV) are staged in LDS as fp32.
// Per tile: partial dot products reduced over the 4 lanes -> S, tS; row max; P~ = exp(S - m);
// l, r, O, A+B updated with the rescale factor exp(m_old - m_new) exactly as in Alg. 2, except
// that A and B share one accumulator (they are only ever added).  Epilogue as in Alg. 2.
#include "launchers.h"
#include <hip/hip_bf16.h>

namespace attn_jvp {
namespace {

constexpr int BC = 32;       // key rows per tile
constexpr int NTHREADS = 256;
// lanes sharing one query row: 4 up to d = 128, 16 for d = 256 (keeps q, tq and the two accumulators of a lane at 64
// registers; with 4 lanes the d = 256 kernel spilled and ran 14x slower per flop)
constexpr int lanes_per_row(int d) { return d > 128 ? 16 : 4; }

template <typename T> struct Ld;
template <> struct Ld<float> {
    static __device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
};
template <> struct Ld<__hip_bfloat16> {
    static __device__ __forceinline__ float4 load4(const __hip_bfloat16* p) {
        uint2 raw = *reinterpret_cast<const uint2*>(p);
        float4 r;
        r.x = __uint_as_float(raw.x << 16);
        r.y = __uint_as_float(raw.x & 0xffff0000u);
        r.z = __uint_as_float(raw.y << 16);
        r.w = __uint_as_float(raw.y & 0xffff0000u);
        return r;
    }
};

template <typename TOut> __device__ __forceinline__ void store4(TOut* p, float4 x);
template <> __device__ __forceinline__ void store4<float>(float* p, float4 x) { *reinterpret_cast<float4*>(p) = x; }
template <> __device__ __forceinline__ void store4<__hip_bfloat16>(__hip_bfloat16* p, float4 x) {
    p[0] = __float2bfloat16(x.x); p[1] = __float2bfloat16(x.y);
    p[2] = __float2bfloat16(x.z); p[3] = __float2bfloat16(x.w);
}

template <typename TIn, typename TOut, int D>
__global__ __launch_bounds__(NTHREADS) void attn_jvp_fp32_kernel(
    const TIn* __restrict__ Q, const TIn* __restrict__ K, const TIn* __restrict__ V,
    const TIn* __restrict__ tQ, const TIn* __restrict__ tK, const TIn* __restrict__ tV,
    TOut* __restrict__ O, TOut* __restrict__ tO, float* __restrict__ LSE,
    int Lq, int Lkv, float scale, int H, int blhd) {
    constexpr int LPR = lanes_per_row(D);
    constexpr int BR = NTHREADS / LPR;          // query rows per workgroup
    constexpr int NCH = D / (4 * LPR);          // float4 chunks per lane
    extern __shared__ float4 smem[];            // 4 tiles of BC x D floats
    float4* sK = smem;
    float4* stK = sK + BC * D / 4;
    float4* sV = stK + BC * D / 4;
    float4* stV = sV + BC * D / 4;

    const int tid = threadIdx.x;
    const int part = tid % LPR;
    const int row_in_blk = tid / LPR;
    const long bh = blockIdx.y;
    const int q0 = blockIdx.x * BR;
    const int qrow = q0 + row_in_blk;
    const int qrow_ld = qrow < Lq ? qrow : Lq - 1;          // ragged last block: duplicate a valid row, never stored

    // [B,H,L,d]: rows of a head contiguous; [B,L,H,d]: rows of a head H*d elements apart
    const int row_elems = blhd ? H * D : D;
    const long bidx = bh / H, hidx = bh % H;
    const long q_base = blhd ? (bidx * Lq * H + hidx) * D : bh * (long)Lq * D;
    const long kv_base = blhd ? (bidx * Lkv * H + hidx) * D : bh * (long)Lkv * D;
    const TIn* Qb = Q + q_base + (long)qrow_ld * row_elems;
    const TIn* tQb = tQ + q_base + (long)qrow_ld * row_elems;
    const TIn* Kb = K + kv_base;
    const TIn* tKb = tK + kv_base;
    const TIn* Vb = V + kv_base;
    const TIn* tVb = tV + kv_base;

    float4 q[NCH], tq[NCH], acc_o[NCH], acc_ab[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        q[c] = Ld<TIn>::load4(Qb + 4 * (part + LPR * c));
        tq[c] = tQ ? Ld<TIn>::load4(tQb + 4 * (part + LPR * c)) : make_float4(0.f, 0.f, 0.f, 0.f);   // absent: zero
        acc_o[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        acc_ab[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float m = -INFINITY, l = 0.f, r = 0.f;

    for (int j0 = 0; j0 < Lkv; j0 += BC) {
        __syncthreads();                        // previous tile fully consumed
        for (int idx = tid; idx < BC * D / 4; idx += NTHREADS) {
            int rr = idx / (D / 4), cc = idx % (D / 4);
            int krow = j0 + rr;
            krow = krow < Lkv ? krow : Lkv - 1;  // pad rows duplicate the last key; masked below
            long off = (long)krow * row_elems + 4 * cc;
            sK[idx] = Ld<TIn>::load4(Kb + off);
            stK[idx] = tK ? Ld<TIn>::load4(tKb + off) : make_float4(0.f, 0.f, 0.f, 0.f);   // absent tangents are zero
            sV[idx] = Ld<TIn>::load4(Vb + off);
            stV[idx] = tV ? Ld<TIn>::load4(tVb + off) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        __syncthreads();

        float s[BC], ts[BC];
        float tile_max = -INFINITY;
#pragma unroll
        for (int j = 0; j < BC; ++j) {
            float a = 0.f, b = 0.f;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                float4 kk = sK[j * (D / 4) + part + LPR * c];
                float4 tk = stK[j * (D / 4) + part + LPR * c];
                a = fmaf(q[c].x, kk.x, a); a = fmaf(q[c].y, kk.y, a); a = fmaf(q[c].z, kk.z, a); a = fmaf(q[c].w, kk.w, a);
                b = fmaf(tq[c].x, kk.x, b); b = fmaf(tq[c].y, kk.y, b); b = fmaf(tq[c].z, kk.z, b); b = fmaf(tq[c].w, kk.w, b);
                b = fmaf(q[c].x, tk.x, b); b = fmaf(q[c].y, tk.y, b); b = fmaf(q[c].z, tk.z, b); b = fmaf(q[c].w, tk.w, b);
            }
#pragma unroll
            for (int o = 1; o < LPR; o <<= 1) { a += __shfl_xor(a, o); b += __shfl_xor(b, o); }
            bool valid = (j0 + j) < Lkv;
            s[j] = valid ? a * scale : -INFINITY;
            ts[j] = valid ? b * scale : 0.f;
            tile_max = fmaxf(tile_max, s[j]);
        }
        const float m_new = fmaxf(m, tile_max);
        const float alpha = expf(m - m_new);    // exp(-inf) = 0 on the first tile
        float row_p = 0.f, row_h = 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            acc_o[c].x *= alpha; acc_o[c].y *= alpha; acc_o[c].z *= alpha; acc_o[c].w *= alpha;
            acc_ab[c].x *= alpha; acc_ab[c].y *= alpha; acc_ab[c].z *= alpha; acc_ab[c].w *= alpha;
        }
#pragma unroll
        for (int j = 0; j < BC; ++j) {
            const float p = expf(s[j] - m_new);
            const float h = p * ts[j];
            row_p += p;
            row_h += h;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                float4 vv = sV[j * (D / 4) + part + LPR * c];
                float4 tv = stV[j * (D / 4) + part + LPR * c];
                acc_o[c].x = fmaf(p, vv.x, acc_o[c].x); acc_o[c].y = fmaf(p, vv.y, acc_o[c].y);
                acc_o[c].z = fmaf(p, vv.z, acc_o[c].z); acc_o[c].w = fmaf(p, vv.w, acc_o[c].w);
                acc_ab[c].x = fmaf(p, tv.x, acc_ab[c].x); acc_ab[c].y = fmaf(p, tv.y, acc_ab[c].y);
                acc_ab[c].z = fmaf(p, tv.z, acc_ab[c].z); acc_ab[c].w = fmaf(p, tv.w, acc_ab[c].w);
                acc_ab[c].x = fmaf(h, vv.x, acc_ab[c].x); acc_ab[c].y = fmaf(h, vv.y, acc_ab[c].y);
                acc_ab[c].z = fmaf(h, vv.z, acc_ab[c].z); acc_ab[c].w = fmaf(h, vv.w, acc_ab[c].w);
            }
        }
        l = alpha * l + row_p;
        r = alpha * r + row_h;
        m = m_new;
    }

    if (qrow < Lq) {
        const float inv_l = 1.f / l;
        const float mu = r * inv_l;             // rowsum(P o tS)
        TOut* Ob = O + q_base + (long)qrow * row_elems;
        TOut* tOb = tO + q_base + (long)qrow * row_elems;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            float4 o4 = acc_o[c], ab = acc_ab[c], t4;
            t4.x = (ab.x - mu * o4.x) * inv_l; t4.y = (ab.y - mu * o4.y) * inv_l;
            t4.z = (ab.z - mu * o4.z) * inv_l; t4.w = (ab.w - mu * o4.w) * inv_l;
            o4.x *= inv_l; o4.y *= inv_l; o4.z *= inv_l; o4.w *= inv_l;
            store4<TOut>(Ob + 4 * (part + LPR * c), o4);
            if (tO) store4<TOut>(tOb + 4 * (part + LPR * c), t4);   // no tangent asked for: nothing to store
        }
        if (part == 0) LSE[bh * Lq + qrow] = m + logf(l);
    }
}

template <typename TIn, typename TOut, int D>
hipError_t launch_one(const Problem& p) {
    constexpr int BR = NTHREADS / lanes_per_row(D);
    dim3 grid((p.Lq + BR - 1) / BR, p.B * p.H);
    size_t smem = 4ull * BC * D * sizeof(float);
    auto kern = attn_jvp_fp32_kernel<TIn, TOut, D>;
    int dev = 0, cus = 0;
    hipError_t e = device_cus(&dev, &cus);
    if (e == hipSuccess) e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)smem, dev);
    if (e != hipSuccess) return e;
    MainKernelTimer timer(p);
    hipLaunchKernelGGL(kern, grid, dim3(NTHREADS), smem, p.stream,
                       (const TIn*)p.q, (const TIn*)p.k, (const TIn*)p.v,
                       (const TIn*)p.tq, (const TIn*)p.tk, (const TIn*)p.tv,
                       (TOut*)p.o, (TOut*)p.to, p.lse, p.Lq, p.Lkv, p.scale, p.H, p.layout);
    return timer.finish(hipGetLastError());
}

template <typename TIn, typename TOut>
hipError_t launch_d(const Problem& p) {
    switch (p.d) {
        case 32: return launch_one<TIn, TOut, 32>(p);
        case 64: return launch_one<TIn, TOut, 64>(p);
        case 128: return launch_one<TIn, TOut, 128>(p);
        case 256: return launch_one<TIn, TOut, 256>(p);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool fp32_vector_supports(const Problem& p) {
    return (p.d == 32 || p.d == 64 || p.d == 128 || p.d == 256) && (long)p.B * p.H <= 65535;
}

hipError_t launch_fp32_vector(const Problem& p) {
    if (!fp32_vector_supports(p)) return hipErrorInvalidValue;
    if (p.in_dtype == 1) return launch_d<float, float>(p);                      // fp32 in -> fp32 out either way
    if (p.out_dtype == 0) return launch_d<__hip_bfloat16, float>(p);
    return launch_d<__hip_bfloat16, __hip_bfloat16>(p);
}

}  // namespace attn_jvp
