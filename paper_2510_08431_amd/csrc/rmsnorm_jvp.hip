// RMS normalisation with gain and its Jacobian-vector product, one pass over the rows (paper App. C.2, the RMSNorm
// layer restructured for JVP mode; used as the QK-normalisation in front of the attention kernel).
//
//     r = rsqrt(mean(x^2) + eps)      y = cast(x r) w      ty = cast(tx r - x r^3 mean(x tx)) w
//
// where cast() rounds to the input dtype before the gain is applied, as the layer does (it normalises in fp32,
// casts back, then multiplies by the weight); for fp32 inputs the casts are no-ops.
//
// Bound: HBM.  Each row is read once (x, tx) and written once (y, ty): 4 d sizeof(T) bytes per row.  A row is
// spread over d * sizeof(T) / 16 adjacent lanes, 16 bytes per lane per tensor, so every access is a full-width
// coalesced 128-bit access; the two row sums are reduced with lane shuffles inside that group.  Each lane keeps
// ROWS_IN_FLIGHT independent rows in flight to cover memory latency.
#include "launchers.h"
#include <hip/hip_bf16.h>
#include <stdint.h>

namespace attn_jvp {
namespace {

#ifndef RMSNORM_JVP_THREADS
#define RMSNORM_JVP_THREADS 256
#endif
#ifndef RMSNORM_JVP_ROWS_IN_FLIGHT
#define RMSNORM_JVP_ROWS_IN_FLIGHT 2
#endif
constexpr int NTHREADS = RMSNORM_JVP_THREADS;
constexpr int ROWS_IN_FLIGHT = RMSNORM_JVP_ROWS_IN_FLIGHT;

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// 16 bytes of T <-> floats.  Rows are streamed once and never re-read by this kernel: non-temporal loads and stores
// (measured +5 % over plain ones on the video workload's q tensor).
template <typename T> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void load(const float* p, float (&f)[4]) {
        const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
        f[0] = v[0]; f[1] = v[1]; f[2] = v[2]; f[3] = v[3];
    }
    static __device__ __forceinline__ void store(float* p, const float (&f)[4]) {
        const f32x4 v = {f[0], f[1], f[2], f[3]};
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p));
    }
    static __device__ __forceinline__ float round(float x) { return x; }
};
template <> struct Vec16<__hip_bfloat16> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void load(const __hip_bfloat16* p, float (&f)[8]) {
        const u32x4 vv = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
        const uint32_t w[4] = {vv[0], vv[1], vv[2], vv[3]};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ float round(float x) { return (float)(__bf16)x; }   // round to nearest even
    static __device__ __forceinline__ void store(__hip_bfloat16* p, const float (&f)[8]) {
        typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
        bf16x8 v;
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (__bf16)f[i];
        __builtin_nontemporal_store(v, reinterpret_cast<bf16x8*>(p));
    }
};

template <typename T, int D>
__global__ __launch_bounds__(NTHREADS) void rmsnorm_jvp_kernel(const T* X, const T* tX, const float* __restrict__ W,
                                                               T* Y, T* tY, long rows, float eps) {
    // X/Y and tX/tY may be the same arrays (in place): no __restrict__ on them; a lane reads every element it
    // later writes before its first store, and no lane touches another lane's elements
    using V = Vec16<T>;
    constexpr int N = V::N;
    constexpr int LPR = D / N;                      // lanes per row
    constexpr int ROWS_PER_PASS = NTHREADS / LPR;
    static_assert(LPR >= 1 && LPR <= 64 && (LPR & (LPR - 1)) == 0, "a row must fit a power-of-two lane group of one wave");
    const int sub = threadIdx.x % LPR;
    const long row0 = (long)blockIdx.x * (ROWS_PER_PASS * ROWS_IN_FLIGHT) + threadIdx.x / LPR;

    float w[N];
#pragma unroll
    for (int i = 0; i < N; i += 4) {
        const float4 v = *reinterpret_cast<const float4*>(W + sub * N + i);
        w[i] = v.x; w[i + 1] = v.y; w[i + 2] = v.z; w[i + 3] = v.w;
    }

    float x[ROWS_IN_FLIGHT][N], t[ROWS_IN_FLIGHT][N];
#pragma unroll
    for (int u = 0; u < ROWS_IN_FLIGHT; ++u) {      // all loads first: 2 * ROWS_IN_FLIGHT requests in flight per lane
        long row = row0 + (long)u * ROWS_PER_PASS;
        row = row < rows ? row : rows - 1;          // rows past the end re-read the last row and are not stored
        V::load(X + row * D + sub * N, x[u]);
        V::load(tX + row * D + sub * N, t[u]);
    }
#pragma unroll
    for (int u = 0; u < ROWS_IN_FLIGHT; ++u) {
        float ss = 0.f, st = 0.f;
#pragma unroll
        for (int i = 0; i < N; ++i) { ss = fmaf(x[u][i], x[u][i], ss); st = fmaf(x[u][i], t[u][i], st); }
#pragma unroll
        for (int o = 1; o < LPR; o <<= 1) { ss += __shfl_xor(ss, o); st += __shfl_xor(st, o); }
        const float r = 1.0f / sqrtf(ss * (1.0f / D) + eps);
        const float c = r * r * r * (st * (1.0f / D));
        float y[N], ty[N];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            y[i] = V::round(x[u][i] * r) * w[i];
            ty[i] = V::round(fmaf(t[u][i], r, -x[u][i] * c)) * w[i];
        }
        const long row = row0 + (long)u * ROWS_PER_PASS;
        if (row < rows) {
            V::store(Y + row * D + sub * N, y);
            V::store(tY + row * D + sub * N, ty);
        }
    }
}

template <typename T, int D>
hipError_t launch_one(const RmsNormProblem& p) {
    constexpr int LPR = D / Vec16<T>::N;
    constexpr long rows_per_block = (NTHREADS / LPR) * ROWS_IN_FLIGHT;
    const long blocks = (p.rows + rows_per_block - 1) / rows_per_block;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((rmsnorm_jvp_kernel<T, D>), dim3((unsigned)blocks), dim3(NTHREADS), 0, p.stream,
                       static_cast<const T*>(p.x), static_cast<const T*>(p.tx), p.w, static_cast<T*>(p.y),
                       static_cast<T*>(p.ty), p.rows, p.eps);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_d(const RmsNormProblem& p) {
    switch (p.d) {
        case 64: return launch_one<T, 64>(p);
        case 128: return launch_one<T, 128>(p);
        case 256: return launch_one<T, 256>(p);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool rmsnorm_jvp_supports(const RmsNormProblem& p) { return p.d == 64 || p.d == 128 || p.d == 256; }

hipError_t launch_rmsnorm_jvp(const RmsNormProblem& p) {
    return p.dtype == 0 ? launch_d<__hip_bfloat16>(p) : launch_d<float>(p);
}

}  // namespace attn_jvp
