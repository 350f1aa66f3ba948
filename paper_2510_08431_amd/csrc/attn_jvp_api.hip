// C-ABI entry points: argument validation, kernel choice, launch.  No allocation; the only state is what is cached
// per device at first use (compute-unit count, raised LDS limits, the address of the static scratch array).
#include "../../include/attn_jvp.h"
#include "launchers.h"
#include <cmath>
#include <cstdint>
#include <mutex>
#include <set>
#include <utility>

using attn_jvp::Problem;

// Scratch of attn_jvp_fwd_static: device memory that belongs to the library.  Every GPU the library runs on holds its own
// copy of this array, at its own address, from the first use until the process ends.  The name below is a host-side
// stand-in, not a device address: host code only ever uses the per-device pointer hipGetSymbolAddress returns.
static __device__ __align__(256) unsigned char scratch[ATTN_JVP_STATIC_SCRATCH_BYTES];

namespace attn_jvp {
namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_setup_mutex;
int g_cus[MAX_DEVICES];                         // 0 = not queried yet
void* g_scratch[MAX_DEVICES];                   // device address of `scratch` on each device, null = not looked up yet
std::set<std::pair<const void*, int>> g_lds_set;   // (kernel, device) pairs whose dynamic-LDS limit has been raised
}  // namespace

hipError_t device_cus(int* dev, int* cus) {
    hipError_t e = hipGetDevice(dev);
    if (e != hipSuccess) return e;
    if (*dev < 0 || *dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    if (g_cus[*dev] == 0) {
        int n = 0;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, *dev);
        if (e != hipSuccess) return e;
        if (n <= 0) return hipErrorInvalidDevice;
        g_cus[*dev] = n;
    }
    *cus = g_cus[*dev];
    return hipSuccess;
}

hipError_t ensure_dynamic_lds(const void* kern, int bytes, int dev) {
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    if (g_lds_set.count({kern, dev})) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) g_lds_set.insert({kern, dev});
    return e;
}

// Address of the static scratch array on the current device (looked up once per device, with that device current).
static hipError_t static_scratch(void** ptr) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    if (g_scratch[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr || (reinterpret_cast<uintptr_t>(p) & 255u)) return hipErrorInvalidSymbol;
        g_scratch[dev] = p;
    }
    *ptr = g_scratch[dev];
    return hipSuccess;
}
}  // namespace attn_jvp

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int run(const void* q, const void* k, const void* v, const void* tq, const void* tk, const void* tv,
        void* o, void* to, float* lse, int B, int H, int Lq, int Lkv, int d, float scale,
        const attn_jvp_opts* opts, bool use_static_scratch = false) {
    attn_jvp_opts def = {};
    def.in_dtype = ATTN_JVP_BF16;
    def.out_dtype = ATTN_JVP_OUT_FP32;
    if (!opts) opts = &def;

    if (!q || !k || !v || !o || !lse) return ATTN_JVP_NULL_PTR;
    if ((tk == nullptr) != (tv == nullptr)) return ATTN_JVP_NULL_PTR;   // zero key/value tangents come as a pair
    if (!tq && tk) return ATTN_JVP_NULL_PTR;                            // no query tangent: no tangents at all
    if (tq && !to) return ATTN_JVP_NULL_PTR;                            // `to` may be NULL only when there is no tangent
    if (B <= 0 || H <= 0 || Lq <= 0 || Lkv <= 0 || d <= 0) return ATTN_JVP_BAD_SHAPE;
    if (!std::isfinite(scale)) return ATTN_JVP_BAD_SHAPE;
    // element counts must stay far below 2^62 so that byte offsets fit in 64 bits; B*H must fit a grid dimension
    const long double elems = (long double)B * H * (long double)(Lq > Lkv ? Lq : Lkv) * d;
    if (elems > 4.0e18L || (long long)B * H > 0x7fffffffLL) return ATTN_JVP_BAD_SHAPE;
    if (opts->in_dtype != ATTN_JVP_BF16 && opts->in_dtype != ATTN_JVP_FP32) return ATTN_JVP_UNSUPPORTED;
    if (opts->out_dtype != ATTN_JVP_OUT_FP32 && opts->out_dtype != ATTN_JVP_OUT_INPUT) return ATTN_JVP_UNSUPPORTED;
    if (opts->layout != ATTN_JVP_LAYOUT_BHLD && opts->layout != ATTN_JVP_LAYOUT_BLHD) return ATTN_JVP_UNSUPPORTED;
    if (opts->reserved != 0) return ATTN_JVP_UNSUPPORTED;
    if (opts->flags & ~(ATTN_JVP_FLAG_FAST | ATTN_JVP_FLAG_NO_F16 | ATTN_JVP_FLAG_F16_ALWAYS | ATTN_JVP_FLAG_NO_LOCKSTEP | ATTN_JVP_FLAG_NO_RESIDENT)) return ATTN_JVP_UNSUPPORTED;
    if (opts->workspace && (reinterpret_cast<uintptr_t>(opts->workspace) & 255u)) return ATTN_JVP_MISALIGNED;
    const void* ptrs[] = {q, k, v, tq, tk, tv, o, to, lse};   // (NULL passes the alignment test)
    for (const void* p : ptrs)
        if (!aligned16(p)) return ATTN_JVP_MISALIGNED;

    void* workspace = opts->workspace;
    size_t workspace_bytes = opts->workspace ? opts->workspace_bytes : 0;
    if (use_static_scratch) {
        if (opts->workspace) return ATTN_JVP_UNSUPPORTED;      // this entry point brings its own scratch
        const size_t need = opts->in_dtype == ATTN_JVP_BF16 ? attn_jvp_workspace_bytes(B, H, Lq, Lkv, d) : 0;
        if (need > (size_t)ATTN_JVP_STATIC_SCRATCH_BYTES) return ATTN_JVP_TOO_LARGE;
        if (need > 0) {
            if (attn_jvp::static_scratch(&workspace) != hipSuccess) return ATTN_JVP_LAUNCH_FAILED;
            workspace_bytes = ATTN_JVP_STATIC_SCRATCH_BYTES;
        }
    }

    Problem p{q, k, v, tq, tk, tv, o, to, lse, B, H, Lq, Lkv, d, scale,
              opts->in_dtype, opts->out_dtype, static_cast<hipStream_t>(opts->stream), opts->flags,
              workspace, workspace_bytes,
              static_cast<hipEvent_t>(opts->timing_events[0]), static_cast<hipEvent_t>(opts->timing_events[1]),
              opts->layout, d, opts->layout};

    const bool f32 = opts->in_dtype == ATTN_JVP_FP32;
    const bool mfma_ok = f32 ? attn_jvp::mfma_f32_supports(p) : attn_jvp::mfma_bf16_supports(p);
    int kernel = opts->kernel;
    if (kernel == ATTN_JVP_KERNEL_AUTO) kernel = mfma_ok ? ATTN_JVP_KERNEL_MFMA : ATTN_JVP_KERNEL_FP32;

    hipError_t e;
    if (kernel == ATTN_JVP_KERNEL_MFMA) {
        if (!mfma_ok) return ATTN_JVP_UNSUPPORTED;
        e = f32 ? attn_jvp::launch_mfma_f32(p) : attn_jvp::launch_mfma_bf16(p);
    } else if (kernel == ATTN_JVP_KERNEL_FP32) {
        if (!attn_jvp::fp32_vector_supports(p)) return ATTN_JVP_UNSUPPORTED;
        e = attn_jvp::launch_fp32_vector(p);
    } else {
        return ATTN_JVP_UNSUPPORTED;
    }
    return e == hipSuccess ? ATTN_JVP_OK : ATTN_JVP_LAUNCH_FAILED;
}

}  // namespace

extern "C" {

int attn_jvp_fwd(const void* q, const void* k, const void* v, const void* tq, const void* tk, const void* tv,
                 void* o, void* to, float* lse, int B, int H, int Lq, int Lkv, int d, float scale) {
    return run(q, k, v, tq, tk, tv, o, to, lse, B, H, Lq, Lkv, d, scale, nullptr);
}

int attn_jvp_fwd_ex(const void* q, const void* k, const void* v, const void* tq, const void* tk, const void* tv,
                    void* o, void* to, float* lse, int B, int H, int Lq, int Lkv, int d, float scale,
                    const attn_jvp_opts* opts) {
    return run(q, k, v, tq, tk, tv, o, to, lse, B, H, Lq, Lkv, d, scale, opts);
}

int attn_jvp_fwd_static(const void* q, const void* k, const void* v, const void* tq, const void* tk, const void* tv,
                        void* o, void* to, float* lse, int B, int H, int Lq, int Lkv, int d, float scale,
                        const attn_jvp_opts* opts) {
    return run(q, k, v, tq, tk, tv, o, to, lse, B, H, Lq, Lkv, d, scale, opts, true);
}

size_t attn_jvp_static_scratch_bytes(void) { return ATTN_JVP_STATIC_SCRATCH_BYTES; }

int attn_jvp_rmsnorm_fwd(const void* x, const void* tx, const float* w, void* y, void* ty,
                         long long rows, int d, float eps, int dtype, void* stream) {
    if (!x || !tx || !w || !y || !ty) return ATTN_JVP_NULL_PTR;
    if (rows <= 0 || d <= 0 || !std::isfinite(eps) || eps < 0.f) return ATTN_JVP_BAD_SHAPE;
    if ((long double)rows * d > 4.0e18L) return ATTN_JVP_BAD_SHAPE;
    if (dtype != ATTN_JVP_BF16 && dtype != ATTN_JVP_FP32) return ATTN_JVP_UNSUPPORTED;
    const void* ptrs[] = {x, tx, w, y, ty};
    for (const void* p : ptrs)
        if (!aligned16(p)) return ATTN_JVP_MISALIGNED;
    attn_jvp::RmsNormProblem p{x, tx, w, y, ty, (long)rows, d, eps, dtype, static_cast<hipStream_t>(stream)};
    if (!attn_jvp::rmsnorm_jvp_supports(p)) return ATTN_JVP_UNSUPPORTED;
    return attn_jvp::launch_rmsnorm_jvp(p) == hipSuccess ? ATTN_JVP_OK : ATTN_JVP_LAUNCH_FAILED;
}

int attn_jvp_mfma_rate_probe(const void* operands, float* out, int f16, int iters, void* stream,
                             long long* mfmas_per_wave, int* waves) {
    if (!operands || !out) return ATTN_JVP_NULL_PTR;
    if (iters <= 0 || iters > ATTN_JVP_RATE_PROBE_MAX_ITERS) return ATTN_JVP_BAD_SHAPE;
    if (!aligned16(operands) || !aligned16(out)) return ATTN_JVP_MISALIGNED;
    return attn_jvp::launch_mfma_rate_probe(operands, out, f16 != 0, iters, static_cast<hipStream_t>(stream),
                                            mfmas_per_wave, waves) == hipSuccess ? ATTN_JVP_OK : ATTN_JVP_LAUNCH_FAILED;
}

size_t attn_jvp_workspace_bytes(int B, int H, int Lq, int Lkv, int d) {
    if (B <= 0 || H <= 0 || Lq <= 0 || Lkv <= 0) return 0;
    if (d != 128 && d != 32 && d != 64 && d != 96) return 0;
    if (d == 32 || d == 96)                 // zero-padded copies of the inputs in front of the fp16 path's scratch
        return attn_jvp::pad_workspace_bytes(B, H, Lq, Lkv, d) + attn_jvp::f16_workspace_bytes(B, H, Lq, Lkv, attn_jvp::padded_head_dim_of(d));
    return attn_jvp::f16_workspace_bytes(B, H, Lq, Lkv, d);
}

const char* attn_jvp_strerror(int code) {
    switch (code) {
        case ATTN_JVP_OK: return "ok";
        case ATTN_JVP_NULL_PTR: return "a required pointer is NULL";
        case ATTN_JVP_BAD_SHAPE: return "a dimension is not positive, the shape is too large, or scale is not finite";
        case ATTN_JVP_UNSUPPORTED: return "unsupported head dim, dtype, kernel choice or option";
        case ATTN_JVP_MISALIGNED: return "a pointer is not 16-byte aligned";
        case ATTN_JVP_LAUNCH_FAILED: return "the HIP runtime refused a set-up call or the kernel launch";
        case ATTN_JVP_TOO_LARGE: return "the shape needs more scratch than the library's static array holds";
        default: return "unknown attn_jvp error code";
    }
}

int attn_jvp_version(void) { return 200; }  // 0.2.0

}  // extern "C"
