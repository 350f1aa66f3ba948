// Internal: launcher entry points shared by the C-ABI translation unit and the kernel files.
#pragma once
#include <hip/hip_runtime.h>

namespace attn_jvp {

struct Problem {
    const void *q, *k, *v, *tq, *tk, *tv;
    void *o, *to;
    float* lse;
    int B, H, Lq, Lkv, d;
    float scale;
    int in_dtype;   // 0 bf16, 1 fp32
    int out_dtype;  // 0 fp32, 1 same as input
    hipStream_t stream;
    int flags;      // ATTN_JVP_FLAG_*
};

// Each returns hipSuccess/hip error of the launch, or hipErrorInvalidValue when the
// (dtype, d) combination is not built for that kernel.
hipError_t launch_fp32_vector(const Problem& p);
hipError_t launch_mfma_bf16(const Problem& p);
bool mfma_bf16_supports(const Problem& p);
bool fp32_vector_supports(const Problem& p);

}  // namespace attn_jvp
