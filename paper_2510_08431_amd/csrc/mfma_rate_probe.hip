// Measurement aid, not part of the attention path: back-to-back 8-pass matrix-core instructions
// (v_mfma_f32_32x32x16_bf16 / _f16) on every compute unit, one wavefront per SIMD, operands taken from a caller's
// buffer.  What it is for: the rate a CDNA4 chip sustains on dense MFMAs depends on the operand VALUES (all-zero
// operands toggle no multiplier inputs and run at full clock; random operands pull the clock down to the power
// limit), so the published peak, which assumes the full clock, is not what any kernel working on real data can
// reach.  Timing this loop on the data distribution of a workload gives the rate that bounds it on the chip at hand.
#include "launchers.h"
#include <stdint.h>

namespace attn_jvp {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int PROBE_SETS = 8;          // operand sets of 256 lanes x 16 bytes: four A operands, four B operands
constexpr int PROBE_MFMAS_PER_ITER = 16;

// Four independent accumulation chains; the A operand rotates over four register sets so that the multiplier inputs
// change with every instruction, as they do when an operand streams from LDS.
template <bool F16>
__global__ __launch_bounds__(256, 1) void mfma_rate_probe_kernel(const u32x4* __restrict__ operands,
                                                                 float* __restrict__ out, int iters) {
    u32x4 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = operands[(2 * i) * 256 + threadIdx.x];
        b[i] = operands[(2 * i + 1) * 256 + threadIdx.x];
    }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (F16)
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a[(i + j) & 3]),
                                                                    __builtin_bit_cast(f16x8, b[j]), acc[j], 0, 0, 0);
                else
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[(i + j) & 3]),
                                                                     __builtin_bit_cast(bf16x8, b[j]), acc[j], 0, 0, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

hipError_t launch_mfma_rate_probe(const void* operands, float* out, int f16, int iters, hipStream_t stream,
                                  long long* mfmas_per_wave, int* waves) {
    int dev = 0, cus = 0;
    hipError_t e = device_cus(&dev, &cus);
    if (e != hipSuccess) return e;
    if (mfmas_per_wave) *mfmas_per_wave = (long long)iters * PROBE_MFMAS_PER_ITER;
    if (waves) *waves = cus * 4;
    const u32x4* ops = static_cast<const u32x4*>(operands);
    if (f16) mfma_rate_probe_kernel<true><<<dim3(cus), dim3(256), 0, stream>>>(ops, out, iters);
    else mfma_rate_probe_kernel<false><<<dim3(cus), dim3(256), 0, stream>>>(ops, out, iters);
    return hipGetLastError();
}

}  // namespace attn_jvp
