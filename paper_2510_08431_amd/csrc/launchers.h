// Internal: launcher entry points shared by the C-ABI translation unit and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

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
    void* workspace;        // optional device scratch for the fp16 value path (may be null)
    size_t workspace_bytes;
    hipEvent_t ev_start, ev_stop;   // optional: recorded around the main kernel (may be null)
};

// Records the caller's optional timing events around the main kernel's launch.
struct MainKernelTimer {
    const Problem& p;
    hipError_t err;
    explicit MainKernelTimer(const Problem& prob) : p(prob), err(hipSuccess) {
        if (p.ev_start) err = hipEventRecord(p.ev_start, p.stream);
    }
    hipError_t finish(hipError_t launch_err) {
        if (err != hipSuccess) return err;
        if (launch_err != hipSuccess) return launch_err;
        return p.ev_stop ? hipEventRecord(p.ev_stop, p.stream) : hipSuccess;
    }
};

// Each returns hipSuccess/hip error of the launch, or hipErrorInvalidValue when the
// (dtype, d) combination is not built for that kernel.
hipError_t launch_fp32_vector(const Problem& p);
hipError_t launch_mfma_bf16(const Problem& p);
bool mfma_bf16_supports(const Problem& p);
bool fp32_vector_supports(const Problem& p);

// fp16 value path: bytes of device scratch it needs, and the pre-pass that fills it (per-head statistics at the
// start of the workspace, then the scaled fp16 copies of V and tV)
size_t f16_workspace_bytes(int B, int H, int Lkv, int d);
hipError_t launch_f16_prepass(const Problem& p, float** stats_out, const void** v16_out, const void** tv16_out);

}  // namespace attn_jvp
