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
    int layout;     // 0: q, k, v, tq, tk, tv are [B,H,L,d]; 1: they are [B,L,H,d].  lse is [B,H,Lq] either way
    int d_out;      // width of the rows of o, to (= d, except when the inputs are zero-padded copies of a smaller d)
    int out_layout; // layout of o, to (= layout, except for the same case)
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

// Facts about the current device and one-time set-up, cached per device; none of it touches a stream, and every
// launcher calls it BEFORE its first enqueue, so that a failure here leaves nothing launched.
//   device_cus: index of the current device and its number of compute units (queried once per device);
//   ensure_dynamic_lds: raises a kernel's dynamic-LDS limit (hipFuncSetAttribute) once per (kernel, device).
hipError_t device_cus(int* dev, int* cus);
hipError_t ensure_dynamic_lds(const void* kern, int bytes, int dev);

// Each returns hipSuccess/hip error of the launch, or hipErrorInvalidValue when the
// (dtype, d) combination is not built for that kernel.
hipError_t launch_fp32_vector(const Problem& p);
hipError_t launch_mfma_bf16(const Problem& p);
hipError_t launch_mfma_f32(const Problem& p);
bool mfma_bf16_supports(const Problem& p);
bool mfma_f32_supports(const Problem& p);
bool fp32_vector_supports(const Problem& p);

constexpr int MFMA_TILE_ROWS = 128;   // query rows per workgroup of the MFMA kernel

// fp16 value path: bytes of device scratch it needs, and the pre-pass that fills it.  Workspace layout, each part
// rounded up to 256 bytes: per-head statistics (8 floats per head) | one int per MFMA workgroup (hand-over flags
// between the launches of the fp16 path: sampled-reference fp16, online fp16, bf16 pairs) followed by 512 bytes of
// lock-step tickets (one counter per XCD, 64 bytes apart) | scaled fp16 copy of V | scaled fp16 copy of tV (both as
// whole 32-key blocks, each block transposed to [d][32]; see convert_values_kernel) | partial
// statistics (8 floats per head and 1024-row block) that the pre-pass's first kernel hands to its second.
struct F16Workspace {
    float* stats;
    int* wg_flags;
    const void* v16;
    const void* tv16;
    int lockstep_slots;   // workgroups of the sweep kernel an XCD holds at a time (its tickets follow the flags, zeroed)
};
size_t f16_workspace_bytes(int B, int H, int Lq, int Lkv, int d);

// Head dimensions the MFMA kernel is not built for (32 and 96): the inputs are first copied, zero-padded to the next
// width it is built for (64 and 128 columns), into the front of the workspace ([B,H,L,width] bf16 each, absent
// tangents skipped); the padded columns add exact zeros to every product.  Width, bytes of that area, and the copy.
constexpr int MFMA_HEAD_DIM = 128;
inline int padded_head_dim_of(int d) { return d <= 64 ? 64 : MFMA_HEAD_DIM; }
size_t pad_workspace_bytes(int B, int H, int Lq, int Lkv, int d);
hipError_t launch_pad_inputs(const Problem& p, Problem* padded);
hipError_t launch_f16_prepass(const Problem& p, int cus, F16Workspace* out);

// Measurement aid: back-to-back MFMAs on every compute unit with the caller's operand values (mfma_rate_probe.hip).
// operands: 8 x 256 x 16 bytes; out: 256 floats per compute unit.  Reports how many MFMAs a wave issues and how many
// waves run, so that the caller can turn a measured time into a rate.
hipError_t launch_mfma_rate_probe(const void* operands, float* out, int f16, int iters, hipStream_t stream,
                                  long long* mfmas_per_wave, int* waves);

// RMS normalisation with gain + JVP over `rows` rows of length d
struct RmsNormProblem {
    const void *x, *tx;
    const float* w;
    void *y, *ty;
    long rows;
    int d;
    float eps;
    int dtype;      // 0 bf16, 1 fp32 (x, tx, y, ty)
    hipStream_t stream;
};
bool rmsnorm_jvp_supports(const RmsNormProblem& p);
hipError_t launch_rmsnorm_jvp(const RmsNormProblem& p);

}  // namespace attn_jvp
