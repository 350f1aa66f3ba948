/*
 * attn_jvp.h - C ABI of the MI355X (gfx950) fused attention forward + Jacobian-vector product.
 *
 * Operation (paper App. C.1: the equations defining S, P, O and tS, tP, tO; Alg. 2 is the
 * streaming procedure that evaluates them without forming the Lq x Lkv matrices).
 * Per (batch b, head h), with s = `scale`:
 *
 *     S  = s Q K^T            P  = softmax_rows(S)          O  = P V
 *     tS = s (tQ K^T + Q tK^T)
 *     tP = P o tS - P o rowsum(P o tS)                      tO = tP V + P tV
 *     lse_i = log sum_j exp(S_ij)                           (the L of Alg. 2's epilogue)
 *
 * Non-causal, no mask, no dropout; Lq and Lkv are independent (self- and cross-attention).
 * The paper writes S = Q K^T without a softmax scale; here the caller's constant `scale`
 * multiplies both S and tS.
 *
 * Memory: every pointer is a DEVICE pointer owned by the caller; the library allocates
 * nothing.  What it keeps between calls is cached per device at first use: the compute-unit
 * count, the raised dynamic-LDS limits of its kernels and the address of the static scratch
 * array of attn_jvp_fwd_static.  attn_jvp_fwd and attn_jvp_fwd_ex need no workspace; if the
 * caller lends one (attn_jvp_opts.workspace, see attn_jvp_workspace_bytes) the bf16 kernel
 * uses its faster fp16-value path (6 instead of 9 matrix products per key block).
 *   q, tq        [B, H, Lq,  d]  contiguous, row-major, d fastest (or [B, Lq, H, d], see attn_jvp_opts.layout)
 *   k, v, tk, tv [B, H, Lkv, d]  same
 *   o, to        [B, H, Lq,  d]  float32 (or the input dtype, see attn_jvp_opts.out_dtype), same layout as q
 *   lse          [B, H, Lq]      float32, natural log
 * Inputs are never written.  Outputs must not alias inputs or one another.  All pointers
 * must be 16-byte aligned.
 * tk and tv may BOTH be NULL: zero key/value tangents.  The paper's kernel serves self- and cross-attention (Sec. 3.2,
 * Flash Attention paragraph); in cross-attention onto a context that does not depend on the differentiated variable
 * the keys and values carry no tangent, which is App. C.1's equations with tK = tV = 0.
 * The result is bit-identical to passing zero tensors; the MFMA kernel then streams only K and V and runs 4 of the
 * 6 matrix products (tS = s tQ K^T, tO = tP V).
 * tq, tk and tv may ALL be NULL: no tangents, the plain attention forward that Alg. 2 extends (2 of the 6 products).
 * o and lse are the same bits as with tangents; `to` is not written and may be NULL.
 *
 * Execution: a call validates its arguments on the host, enqueues its kernels on the given
 * HIP stream and returns without synchronising.  A return value of 0 means "enqueued".
 * Codes 1-4 and 6 come from the host-side checks: nothing was launched and the outputs are
 * untouched.  Everything else that can fail without a launch (device query, LDS limits, grid
 * sizes, the static scratch's address) is also done before the first enqueue and returns
 * ATTN_JVP_LAUNCH_FAILED with nothing launched.  Only when the HIP runtime refuses an enqueue
 * in the middle of a call (the fp16 value path enqueues up to eight kernels) may earlier
 * kernels of that call already be on the stream; the outputs are then unspecified.  No
 * exception or abort crosses this boundary.  Results are deterministic (the only atomics are order-independent maxima in the
 * fp16 path's pre-pass).
 */
#ifndef ATTN_JVP_H_
#define ATTN_JVP_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* error codes */
#define ATTN_JVP_OK            0
#define ATTN_JVP_NULL_PTR      1  /* a required pointer is NULL (tangents may be absent only as tk+tv or tq+tk+tv) */
#define ATTN_JVP_BAD_SHAPE     2  /* B, H, Lq, Lkv or d <= 0, a product overflows, or scale is not finite */
#define ATTN_JVP_UNSUPPORTED   3  /* head dim / dtype / kernel choice not built */
#define ATTN_JVP_MISALIGNED    4  /* a pointer is not 16-byte aligned */
#define ATTN_JVP_LAUNCH_FAILED 5  /* the HIP runtime refused a set-up call or a launch */
#define ATTN_JVP_TOO_LARGE     6  /* attn_jvp_fwd_static only: the shape needs more than ATTN_JVP_STATIC_SCRATCH_BYTES */

/* size of the library's static device scratch array (attn_jvp_fwd_static): 200 MiB per GPU */
#define ATTN_JVP_STATIC_SCRATCH_BYTES (200u << 20)

/* attn_jvp_opts.in_dtype / out_dtype */
#define ATTN_JVP_BF16 0
#define ATTN_JVP_FP32 1
#define ATTN_JVP_OUT_FP32  0      /* o, to are float32 (default; the accumulators' own precision) */
#define ATTN_JVP_OUT_INPUT 1      /* o, to have the input dtype (bf16 outputs carry the bf16 rounding of each element,
                                     up to 2^-8 of its value: more than the kernels' own error) */

/* attn_jvp_opts.layout */
#define ATTN_JVP_LAYOUT_BHLD 0    /* [B, H, L, d] (default) */
#define ATTN_JVP_LAYOUT_BLHD 1    /* [B, L, H, d]: what a sequence-to-head all-to-all (Ulysses context parallelism,
                                     paper Sec. 3.2) leaves on each GPU, consumed and produced without a transpose.
                                     lse stays [B, H, Lq]. */

/* attn_jvp_opts.kernel */
#define ATTN_JVP_KERNEL_AUTO 0    /* bf16, scale > 0 and d in {64, 128} (or d in {32, 96} with a workspace) -> bf16 MFMA kernel;
                                     fp32 and d in {32, 64, 96, 128} -> fp32 MFMA kernel; everything else -> vector kernel */
#define ATTN_JVP_KERNEL_FP32 1    /* fp32 vector-ALU streaming kernel: any dtype, d in {32, 64, 128, 256}, slow */
#define ATTN_JVP_KERNEL_MFMA 2    /* matrix-core kernels.
                                     bf16 inputs: scale > 0, d in {64, 128} (built natively); d in {32, 96} given a
                                     workspace of attn_jvp_workspace_bytes(...): the inputs are first copied there
                                     zero-padded to 64 and 128 columns (exact: the padding adds zeros to every
                                     product; half and a quarter of the matrix work are then spent on zeros).
                                     fp32 inputs: d in {32, 64, 96, 128}, any finite scale, fp32 outputs; fp32 operands
                                     and fp32 accumulation throughout (Alg. 2 as printed), no workspace, flags ignored.
                                     Accuracy contract of this path: l, r and the accumulators are fp32 running sums
                                     over the keys, so max |x - x_exact| / RMS(x) of o and to is within 1e-5 up to
                                     256 keys and grows like sqrt(Lkv) beyond: within 1.5e-5 sqrt(Lkv / 256)
                                     (measured on unit-variance scores: 5e-6 at 256 keys, 1.4e-5 at 4096); rows on
                                     which one key carries the weight add up to 40 x 2^-24 x max|S| (the rounding of
                                     the fp32 score itself, which the exponential turns into a relative error) */

/* attn_jvp_opts.flags */
#define ATTN_JVP_FLAG_FAST 1      /* EXPERIMENTAL, outside the accuracy contract (O within 1e-2, tO within 2e-2 of RMS): kept for
                                     measurements only.
                                     MFMA kernel only (not with absent tangents): round the weights P~ and H~ = P~ o tS to ONE bf16 term each
                                     (6 matrix products per key tile, as Alg. 2 counts them) instead of the default
                                     hi + lo bf16 pairs in all three value contractions (9 products) or the fp16 value path.  Faster; the
                                     8-bit rounding then shows in the results: max errors up to ~2e-2 of RMS(O) and
                                     a few 1e-2 of RMS(tO) on rows where few keys carry the weight. */

#define ATTN_JVP_FLAG_NO_F16 2    /* MFMA kernel only: do not use the fp16 value path even if a workspace is given */
#define ATTN_JVP_FLAG_F16_ALWAYS 4 /* MFMA kernel only: use the fp16 value path (given a workspace) for short key
                                     sequences too; without it Lkv < 2048 (Lkv < 256 when the call has at least four
                                     query tiles per compute unit) takes the bf16 pairs, which are faster
                                     there (the fp16 path's pre-pass and key sampling do not pay off), and so do
                                     tiles with widely spread scores below ~5k keys */

#define ATTN_JVP_FLAG_NO_LOCKSTEP 8 /* MFMA kernel only: on the fp16 path's running-reference tier (key sequences of
                                     32768 keys or more), do not hold back the start of a query tile until the
                                     tiles that will share its XCD's L2 have started too (a wait of at most
                                     100 us per tile).  Results are identical either way; the wait keeps those
                                     tiles in step on their key/value stream (measured 273 against 329 ms on
                                     the 75600-key stress workload).  For callers that run other kernels on the
                                     same GPU at the same time, where an XCD does not hold a full round of
                                     this kernel's workgroups and every wait would run to its limit.
                                     Hardware assumption behind the wait and behind the kernel's tile map, which
                                     nothing checks at run time: workgroup w of a launch runs on XCD w mod 8, and
                                     the GPU is otherwise idle.  If it does not hold, only speed is lost. */

#define ATTN_JVP_FLAG_NO_RESIDENT 16 /* MFMA kernel only: launch one workgroup per 128-row query tile and let the hardware hand
                                     them out, instead of one resident workgroup per compute unit that walks through
                                     its share of the tiles (the default from two tiles per compute unit on).
                                     Results are identical.  For callers that run other kernels on the same GPU at
                                     the same time: resident workgroups assume they get a compute unit each. */

typedef struct attn_jvp_opts {
    int    in_dtype;        /* ATTN_JVP_BF16 or ATTN_JVP_FP32: dtype of q, k, v, tq, tk, tv */
    int    out_dtype;       /* ATTN_JVP_OUT_FP32 or ATTN_JVP_OUT_INPUT: dtype of o, to */
    void*  stream;          /* hipStream_t; NULL = the default stream */
    int    kernel;          /* ATTN_JVP_KERNEL_* */
    int    flags;           /* bitwise OR of ATTN_JVP_FLAG_*; unknown bits are rejected */
    void*  workspace;       /* optional DEVICE scratch, 256-byte aligned, or NULL.  Contents are overwritten; it
                               must stay untouched until the call's work on `stream` has finished.  With at least
                               attn_jvp_workspace_bytes(...) bytes the MFMA kernel runs its fp16 value path: V, tV
                               are first copied there as per-head power-of-two-scaled fp16, and the weights P~, H~
                               enter the value contractions as single fp16 terms (6 matrix products per key block,
                               11-bit weights) against an exponent reference sampled before the sweep.  Query
                               tiles whose scores are too spread out for that (standard deviation of a row's
                               scaled scores above ~2.5) are done by a second launch with a running reference.
                               On this path the row sums are taken over the weights as rounded, so o, to are
                               the exact result for probabilities off by 2^-11 and centred tangent scores off by 2^-10 relative, and
                               lse carries the rounding of l (at most 2^-11 absolute).  Without a workspace, and for
                               Lkv < 2048 (Lkv < 256 for calls with at least four 128-row query tiles per compute
                               unit): hi + lo bf16 pairs everywhere (9 products, ~16-bit weights). */
    size_t workspace_bytes; /* size of `workspace` */
    void*  timing_events[2]; /* optional hipEvent_t pair (created by the caller, with timing enabled), or NULL:
                               [0] is recorded on `stream` immediately before the main attention kernel and [1]
                               immediately after it, so a profiler can time that kernel apart from the fp16
                               path's pre-pass kernels, which are enqueued before [0] */
    int    layout;          /* ATTN_JVP_LAYOUT_*: memory layout of q, k, v, tq, tk, tv, o, to */
    int    reserved;        /* must be zero */
} attn_jvp_opts;

/*
 * Alg. 2 with bf16 inputs, float32 o/to/lse, on the default stream, kernel chosen automatically.
 * Returns ATTN_JVP_OK or an error code above.
 * This call passes no workspace, so at d = 128 it runs the hi + lo bf16-pair kernel: 9 matrix products per key
 * block where the fp16 value path runs 6, i.e. about 1.35x the time on long key sequences (measured on the
 * 32760-token self-attention shape, B = 1, H = 12: 20.4-21.4 ms against 14.7-15.7 ms; 37-39 % against 50-53 % of the
 * bf16 matrix peak, over the boxes of one pool).  Callers that want the faster path lend a workspace through attn_jvp_fwd_ex, or call
 * attn_jvp_fwd_static, which brings its own.
 */
int attn_jvp_fwd(const void* q, const void* k, const void* v,
                 const void* tq, const void* tk, const void* tv,
                 void* o, void* to, float* lse,
                 int B, int H, int Lq, int Lkv, int d, float scale);

/* Same operation with explicit dtype, stream and kernel choice. opts == NULL means the defaults of attn_jvp_fwd. */
int attn_jvp_fwd_ex(const void* q, const void* k, const void* v,
                    const void* tq, const void* tk, const void* tv,
                    void* o, void* to, float* lse,
                    int B, int H, int Lq, int Lkv, int d, float scale,
                    const attn_jvp_opts* opts);

/*
 * attn_jvp_fwd_ex with the library's own scratch in place of a caller-lent workspace: for callers that cannot
 * allocate device memory (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
 * The scratch is a static device array of ATTN_JVP_STATIC_SCRATCH_BYTES (200 MiB: enough for the fp16 value path
 * up to B*H*Lkv = 409 000 keys at d = 128, e.g. the 32760-token shape with 12 heads); every GPU the library is
 * used on holds its copy from the first use until the process ends.  The call allocates nothing (no hipMalloc,
 * no hipFree, no allocating library routine) and is otherwise attn_jvp_fwd_ex: same arguments, same kernels, same
 * results bit for bit as attn_jvp_fwd_ex with a workspace of attn_jvp_workspace_bytes(...).
 * opts may be NULL (defaults); opts->workspace must be NULL (ATTN_JVP_UNSUPPORTED otherwise).  Shapes whose
 * attn_jvp_workspace_bytes(...) exceeds the array are rejected with ATTN_JVP_TOO_LARGE before anything is
 * launched.  All calls on one GPU share that GPU's array: calls whose work overlaps in time (different
 * streams, different host threads) race on it and must be serialised by the caller; calls on one stream are
 * ordered and safe.  The array keeps the last call's contents; the kernels re-initialise what they read
 * (statistics, tile flags and tickets are cleared by the call's own first kernels).
 */
int attn_jvp_fwd_static(const void* q, const void* k, const void* v,
                        const void* tq, const void* tk, const void* tv,
                        void* o, void* to, float* lse,
                        int B, int H, int Lq, int Lkv, int d, float scale,
                        const attn_jvp_opts* opts);

/* ATTN_JVP_STATIC_SCRATCH_BYTES as the loaded library was built with. */
size_t attn_jvp_static_scratch_bytes(void);

/*
 * Bytes of scratch the MFMA kernel can use for this shape (0 if it has no use for any).  d = 128: the fp16 value
 * path's 2 fp16 copies of V and tV (Lkv rounded up to a multiple of 32 keys: they are kept as whole 32-key blocks), 32 bytes of statistics per (batch, head), 4 bytes per 128-row query tile and
 * 32 bytes per (batch, head) and 1024 rows of the longer sequence, each part rounded up to 256 bytes, and 512 bytes
 * of counters (d = 64 likewise, with its own row width).  d in {32, 96}: in front of that, bf16 copies of the six inputs
 * zero-padded to 64 and 128 columns (without them the MFMA kernel does not take these head dimensions), and the
 * rest sized for the padded width.  Pure host arithmetic.
 */
size_t attn_jvp_workspace_bytes(int B, int H, int Lq, int Lkv, int d);

/*
 * RMS normalisation with gain and its JVP, the QK-normalisation in front of the attention (paper App. C.2, the
 * RMSNorm layer restructured for JVP mode).  For each of `rows` rows of length d:
 *
 *     r = 1 / sqrt(mean(x^2) + eps)     y = cast(x r) w     ty = cast(tx r - x r^3 mean(x tx)) w
 *
 * cast() rounds to the dtype of x before the gain is applied, as the layer does (normalise in float32, cast back,
 * multiply by the weight); y, ty are rounded once more on storing.  x, tx, y, ty: [rows, d] contiguous DEVICE
 * arrays of `dtype` (ATTN_JVP_BF16 or ATTN_JVP_FP32), 16-byte aligned; w: [d] float32 DEVICE array.  d in
 * {64, 128, 256}.  y may be x and ty may be tx (in place); no other overlap.  eps >= 0.  Enqueues one kernel on
 * `stream` (hipStream_t, NULL = default) and returns an ATTN_JVP_* code without synchronising; on a non-zero
 * return nothing was launched.
 */
int attn_jvp_rmsnorm_fwd(const void* x, const void* tx, const float* w, void* y, void* ty,
                         long long rows, int d, float eps, int dtype, void* stream);

/* Measurement aid (no passage of the paper: it prices the kernels above).  Runs `iters` x 16 back-to-back
 * v_mfma_f32_32x32x16_bf16 (f16 = 0) or _f16 (f16 != 0) instructions per wavefront, one wavefront per SIMD on every
 * compute unit, on the operand VALUES the caller supplies, asynchronously on `stream`; the caller times it (events on
 * that stream).  The rate a chip sustains on dense matrix instructions depends on those values: all-zero operands run
 * at the full clock, random ones at the clock the power limit leaves.
 *   operands  device, 8 x 256 x 16 bytes (eight sets of one 16-byte fragment per lane: four A and four B operands,
 *             bf16 or fp16 bit patterns), 16-byte aligned, read only;
 *   out       device, 256 floats per compute unit (sums of the accumulators, so that the work is observable);
 *   iters     1 .. ATTN_JVP_RATE_PROBE_MAX_ITERS (bounds the run time to about a second);
 *   mfmas_per_wave, waves   host, optional: instructions each wavefront issues, and how many wavefronts run;
 *             flops = 32768 x mfmas_per_wave x waves.
 * Errors as above (NULL_PTR, BAD_SHAPE, MISALIGNED from host checks; LAUNCH_FAILED). */
#define ATTN_JVP_RATE_PROBE_MAX_ITERS 2000000
int attn_jvp_mfma_rate_probe(const void* operands, float* out, int f16, int iters, void* stream,
                             long long* mfmas_per_wave, int* waves);

/* Static, NUL-terminated description of an error code (never NULL). */
const char* attn_jvp_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int attn_jvp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ATTN_JVP_H_ */
