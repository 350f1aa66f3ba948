// Pre-pass of the fp16 value path: per-head statistics, then V, tV -> scaled, block-transposed fp16 copies in the workspace.
// Two memory-bound launches (coalesced 128-bit accesses).  The first reads V and tV once (their largest magnitudes
// fix the scales of the fp16 copies) and every 16th row of Q, tQ, K, tK (their row norms only steer how the tangent
// weights are scaled; an estimate is enough, see f16_scales.h), and leaves one partial result per block; the second
// reduces a head's partials, converts, and clears the lock-step tickets.  No atomics, nothing to zero beforehand.
#include "launchers.h"
#include "f16_scales.h"
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace attn_jvp {
namespace {

constexpr int ROWS_PER_BLOCK = 1024;     // rows of a tensor one block of the statistics kernel looks at

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// 16-byte load of data that this kernel reads exactly once
__device__ __forceinline__ uint4 ld16(const __hip_bfloat16* p) {
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}

struct StatsArgs {
    const __hip_bfloat16* x[6];   // V, tV, Q, tQ, K, tK
    int L[6];
    int H, blhd;                  // layout of the tensors: [B,H,L,d] or [B,L,H,d]
};

// element offset of row `row` of head `bh` in a tensor with L rows of DH elements per head
template <int DH>
__device__ __forceinline__ long row_offset(long bh, int row, int L, int H, int blhd) {
    return blhd ? (((bh / H) * L + row) * H + bh % H) * (long)DH : (bh * L + row) * (long)DH;
}

constexpr int NORM_ROW_STEP = 16;   // row norms of Q, tQ, K, tK are taken from every 16th row (and the last one)

// One launch for all six tensors: blockIdx.z selects the tensor, blockIdx.x a range of ROWS_PER_BLOCK rows.
// Slot 0, 1: abs max of V, tV over every element; slots 2..5: largest squared row norm of Q, tQ, K, tK over the
// sampled rows.  Every block writes its result (zero for an empty range or an absent tensor) to
// partials[(head * gridDim.x + blockIdx.x) * 8 + tensor]: nothing needs clearing, and no two blocks share a word.
// A row of DH bf16 is read by DH / 8 adjacent lanes (16 bytes each); 256 threads cover 16 rows per pass (32 at DH = 64).
template <int DH>
__global__ __launch_bounds__(256) void head_stats_kernel(StatsArgs a, float* __restrict__ partials) {
    constexpr int LPR = DH / 8;              // lanes per row
    constexpr int RPP = 256 / LPR;           // rows per pass of the block
    const int which = blockIdx.z;
    const int L = a.L[which];
    const int row0 = blockIdx.x * ROWS_PER_BLOCK;
    const long bh = blockIdx.y;
    float* out = partials + (bh * gridDim.x + blockIdx.x) * 8 + which;
    if (row0 >= L || a.x[which] == nullptr) {         // absent tangents leave their statistic at zero
        if (threadIdx.x == 0) *out = 0.f;
        return;
    }
    const __hip_bfloat16* __restrict__ X = a.x[which];
    const int sub = threadIdx.x % LPR;
    const int r_in = threadIdx.x / LPR;
    float best = 0.f;
    auto fold = [&](const uint4& w) {
        const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
        float v = 0.f;
        if (which < 2) {
#pragma unroll
            for (int i = 0; i < 4; ++i) v = fmaxf(v, fmaxf(fabsf(bf16_lo(ws[i])), fabsf(bf16_hi(ws[i]))));
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) { const float c = bf16_lo(ws[i]), e = bf16_hi(ws[i]); v = fmaf(c, c, fmaf(e, e, v)); }
            // row norm^2: sum over the lanes of the row
            v += __shfl_xor(v, 1); v += __shfl_xor(v, 2); v += __shfl_xor(v, 4);
            if constexpr (LPR == 16) v += __shfl_xor(v, 8);
        }
        best = fmaxf(best, v);
    };
    if (which < 2) {
        for (int rr = r_in; rr < ROWS_PER_BLOCK; rr += 4 * RPP) {
            uint4 w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {            // four independent 16-byte loads in flight per lane
                const int row = row0 + rr + RPP * u;
                w[u] = row < L ? ld16(X + row_offset<DH>(bh, row, L, a.H, a.blhd) + sub * 8) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) fold(w[u]);
        }
    } else {
        // the block's 64 sampled rows (row0, row0 + 16, ...) in one round of loads, plus the tensor's last row, taken
        // by the block whose range holds it
        constexpr int NU = ROWS_PER_BLOCK / NORM_ROW_STEP / RPP;     // loads per lane: 4, or 2 at DH = 64
        uint4 w[NU];
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int row = row0 + NORM_ROW_STEP * (r_in + RPP * u);
            w[u] = row < L ? ld16(X + row_offset<DH>(bh, row, L, a.H, a.blhd) + sub * 8) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < NU; ++u) fold(w[u]);
        if (L - 1 >= row0 && L - 1 < row0 + ROWS_PER_BLOCK && r_in == 0) fold(ld16(X + row_offset<DH>(bh, L - 1, L, a.H, a.blhd) + sub * 8));
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) best = fmaxf(best, __shfl_xor(best, o));
    __shared__ float wave_best[4];
    if ((threadIdx.x & 63) == 0) wave_best[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) *out = fmaxf(fmaxf(wave_best[0], wave_best[1]), fmaxf(wave_best[2], wave_best[3]));
}

// Reduces the head's partial statistics (NaN in an input gives NaN here and ends in the bf16-pair fallback), leaves
// them in stats[head * 8 ..] for the sweep kernels (block 0 of each head), clears the lock-step tickets (block 0 of
// head 0), then converts its share of the head's V, tV to scaled fp16, TRANSPOSED key block by key block, which is how
// the sweep kernels want them: block j of a head is [DH][32] fp16, and within a row position 16 t2 + 8 g + t holds key
// 32 j + 16 t2 + 4 g + (t & 3) + 8 (t >> 2) (the order in which a score MFMA leaves the keys in a lane's registers, so
// that the matching operand of a value MFMA is 16 contiguous bytes); keys past Lkv are stored as zeros.
// One key block per pass of the workgroup: 32 rows are read whole (16 bytes per lane), converted into an LDS tile
// [key][DH + 4] (the padding spreads the transposed reads over the banks), and written out as 16-byte pieces.
template <int DH>
__global__ __launch_bounds__(256) void convert_values_kernel(const __hip_bfloat16* __restrict__ V,
                                                             const __hip_bfloat16* __restrict__ tV,
                                                             const float* __restrict__ partials, int n_partials,
                                                             float* __restrict__ stats, float* __restrict__ tickets,
                                                             __half* __restrict__ V16,
                                                             __half* __restrict__ tV16, int n_blocks, float scale,
                                                             int Lkv, int H, int blhd) {
    constexpr int LPR = DH / 8;              // 16-byte chunks per source row
    constexpr int TILE_ROW = DH + 4;         // halves per row of the LDS tile
    constexpr int IN_CHUNKS = 32 * LPR / 256, OUT_CHUNKS = DH * 4 / 256;   // per thread and tensor
    const long bh = blockIdx.y;
    __shared__ float head_stats[8];
    __shared__ __half tile[2][32 * TILE_ROW];
    if (threadIdx.x < 64) {          // lane t % 8 of the first wave takes statistic t % 8 of every 8th partial
        const int which = threadIdx.x & 7;
        float best = 0.f;
        for (int p = threadIdx.x >> 3; p < n_partials; p += 8) {
            const float v = partials[(bh * n_partials + p) * 8 + which];
            best = (v > best || v != v) ? v : best;      // a NaN sticks
        }
#pragma unroll
        for (int o = 8; o < 64; o <<= 1) {
            const float other = __shfl_xor(best, o);
            best = (other > best || other != other) ? other : best;
        }
        if (threadIdx.x < 8) {
            head_stats[which] = which < 6 ? best : 0.f;
            if (blockIdx.x == 0) stats[bh * 8 + which] = which < 6 ? best : 0.f;
        }
    }
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 128) tickets[threadIdx.x] = 0.f;
    __syncthreads();
    const F16Scales sc = f16_scales(head_stats, scale);
    const float gain[2] = {ldexpf(1.f, -sc.eV), ldexpf(1.f, -sc.eA)};
    const __hip_bfloat16* src[2] = {V, tV};
    __half* dst[2] = {V16, tV16};
    const int n_tensors = tV != nullptr ? 2 : 1;         // uniform: tV is absent when the caller passes no key/value tangents
    for (int blk = blockIdx.x; blk < n_blocks; blk += gridDim.x) {
        for (int x = 0; x < n_tensors; ++x) {
#pragma unroll
            for (int u = 0; u < IN_CHUNKS; ++u) {
                const int q = threadIdx.x + 256 * u, row = q / LPR, sub = q % LPR;
                const int key = blk * 32 + row;
                uint4 a = make_uint4(0, 0, 0, 0);
                if (key < Lkv) a = *reinterpret_cast<const uint4*>(src[x] + row_offset<DH>(bh, key, Lkv, H, blhd) + sub * 8);
                const uint32_t aw[4] = {a.x, a.y, a.z, a.w};
                alignas(16) __half2 h[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) h[j] = __floats2half2_rn(bf16_lo(aw[j]) * gain[x], bf16_hi(aw[j]) * gain[x]);
                uint2* t = reinterpret_cast<uint2*>(&tile[x][row * TILE_ROW + sub * 8]);     // rows are 8-byte aligned
                t[0] = reinterpret_cast<const uint2*>(h)[0];
                t[1] = reinterpret_cast<const uint2*>(h)[1];
            }
        }
        __syncthreads();
        for (int x = 0; x < n_tensors; ++x) {
#pragma unroll
            for (int u = 0; u < OUT_CHUNKS; ++u) {
                const int o = threadIdx.x + 256 * u, col = o >> 2, chunk = o & 3;    // 16-byte piece `chunk` of row `col`
                const int key0 = 16 * (chunk >> 1) + 4 * (chunk & 1);
                alignas(16) __half v[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) v[t] = tile[x][(key0 + (t & 3) + 8 * (t >> 2)) * TILE_ROW + col];
                *reinterpret_cast<uint4*>(dst[x] + ((bh * n_blocks + blk) * (long)(32 * DH)) + o * 8) = *reinterpret_cast<const uint4*>(v);
            }
        }
        __syncthreads();
    }
}

}  // namespace

namespace {
struct Layout {
    size_t stats_bytes, flags_bytes, vals_bytes, partials_bytes;
    int n_partials;     // blocks of ROWS_PER_BLOCK rows that cover the longer of the two sequences
};
Layout layout(int B, int H, int Lq, int Lkv, int d) {
    const size_t heads = (size_t)B * H;
    const size_t tiles = heads * (size_t)((Lq + MFMA_TILE_ROWS - 1) / MFMA_TILE_ROWS);
    const int Lmax = Lq > Lkv ? Lq : Lkv;
    const int np = (Lmax + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    auto up = [](size_t n) { return (n + 255) & ~(size_t)255; };
    const size_t key_blocks = (size_t)((Lkv + 31) / 32);     // the fp16 copies are whole 32-key blocks
    return {up(heads * 8 * sizeof(float)), up(tiles * sizeof(int)) + 512, up(heads * key_blocks * 32 * d * sizeof(__half)),
            up(heads * (size_t)np * 8 * sizeof(float)), np};
}
struct PadArgs {
    const __hip_bfloat16* src[6];   // q, k, v, tq, tk, tv (null = absent)
    __hip_bfloat16* dst[6];
    int L[6];
    int H, d, blhd;
    int D;                          // width of the zero-padded copies (64 or 128)
};

// dst[B,H,L,D] = src rows (any layout) followed by zeros.  One thread per 16-byte chunk of dst; blockIdx.z = tensor.
__global__ __launch_bounds__(256) void pad_inputs_kernel(PadArgs a, long heads) {
    const int which = blockIdx.z;
    if (a.src[which] == nullptr) return;
    const int L = a.L[which];
    const int cpr = a.D / 8;                    // chunks per padded row
    const long n_chunks = heads * L * cpr;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n_chunks; i += (long)gridDim.x * blockDim.x) {
        const int c = (int)(i % cpr);
        const long hr = i / cpr;                // head * L + row
        const long bh = hr / L;
        const int row = (int)(hr % L);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (c * 8 < a.d) {
            const long src = a.blhd ? (((bh / a.H) * L + row) * a.H + bh % a.H) * (long)a.d : hr * (long)a.d;
            v = *reinterpret_cast<const uint4*>(a.src[which] + src + c * 8);
        }
        *reinterpret_cast<uint4*>(a.dst[which] + i * 8) = v;
    }
}

}  // namespace

size_t pad_workspace_bytes(int B, int H, int Lq, int Lkv, int d) {
    const size_t heads = (size_t)B * H, D = (size_t)padded_head_dim_of(d);
    auto up = [](size_t n) { return (n + 255) & ~(size_t)255; };
    return 2 * up(heads * Lq * D * 2) + 4 * up(heads * Lkv * D * 2);
}

hipError_t launch_pad_inputs(const Problem& p, Problem* padded) {
    const size_t heads = (size_t)p.B * p.H, D = (size_t)padded_head_dim_of(p.d);
    auto up = [](size_t n) { return (n + 255) & ~(size_t)255; };
    const size_t qb = up(heads * p.Lq * D * 2), kb = up(heads * p.Lkv * D * 2);
    char* ws = static_cast<char*>(p.workspace);
    PadArgs a;
    const void* srcs[6] = {p.q, p.k, p.v, p.tq, p.tk, p.tv};
    const size_t offs[6] = {0, 2 * qb, 2 * qb + kb, qb, 2 * qb + 2 * kb, 2 * qb + 3 * kb};
    for (int i = 0; i < 6; ++i) {
        a.src[i] = static_cast<const __hip_bfloat16*>(srcs[i]);
        a.dst[i] = reinterpret_cast<__hip_bfloat16*>(ws + offs[i]);
        a.L[i] = (i == 0 || i == 3) ? p.Lq : p.Lkv;
    }
    a.H = p.H; a.d = p.d; a.blhd = p.layout; a.D = (int)D;
    const int Lmax = p.Lq > p.Lkv ? p.Lq : p.Lkv;
    long blocks = ((long)heads * Lmax * (long)(D / 8) + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(pad_inputs_kernel, dim3((unsigned)blocks, 1, 6), dim3(256), 0, p.stream, a, (long)heads);
    *padded = p;
    auto at = [&](int i) -> const void* { return srcs[i] ? static_cast<const void*>(a.dst[i]) : nullptr; };
    padded->q = at(0); padded->k = at(1); padded->v = at(2); padded->tq = at(3); padded->tk = at(4); padded->tv = at(5);
    padded->d = (int)D;
    padded->layout = 0;
    padded->workspace = ws + pad_workspace_bytes(p.B, p.H, p.Lq, p.Lkv, p.d);
    padded->workspace_bytes = p.workspace_bytes - pad_workspace_bytes(p.B, p.H, p.Lq, p.Lkv, p.d);
    return hipGetLastError();
}

size_t f16_workspace_bytes(int B, int H, int Lq, int Lkv, int d) {
    const Layout l = layout(B, H, Lq, Lkv, d);
    return l.stats_bytes + l.flags_bytes + 2 * l.vals_bytes + l.partials_bytes;
}

hipError_t launch_f16_prepass(const Problem& p, int cus, F16Workspace* out) {
    const size_t heads = (size_t)p.B * p.H;
    const Layout l = layout(p.B, p.H, p.Lq, p.Lkv, p.d);
    char* ws = static_cast<char*>(p.workspace);
    float* stats = reinterpret_cast<float*>(ws);
    int* wg_flags = reinterpret_cast<int*>(ws + l.stats_bytes);
    __half* V16 = reinterpret_cast<__half*>(ws + l.stats_bytes + l.flags_bytes);
    __half* tV16 = reinterpret_cast<__half*>(ws + l.stats_bytes + l.flags_bytes + l.vals_bytes);
    float* partials = reinterpret_cast<float*>(ws + l.stats_bytes + l.flags_bytes + 2 * l.vals_bytes);
    // tickets of the online tier's lock-step start: 8 XCDs x one counter per 64 bytes, after the flags
    float* tickets = reinterpret_cast<float*>(ws + l.stats_bytes + l.flags_bytes - 512);
    out->lockstep_slots = cus % 8 == 0 ? cus / 8 : 0;   // one workgroup per compute unit, eight XCDs
    StatsArgs sa;
    const void* xs[6] = {p.v, p.tv, p.q, p.tq, p.k, p.tk};
    for (int i = 0; i < 6; ++i) {
        sa.x[i] = static_cast<const __hip_bfloat16*>(xs[i]);
        sa.L[i] = (i == 2 || i == 3) ? p.Lq : p.Lkv;
    }
    sa.H = p.H;
    sa.blhd = p.layout;
    auto bf = [](const void* x) { return static_cast<const __hip_bfloat16*>(x); };
    if (p.d == 64)
        hipLaunchKernelGGL(head_stats_kernel<64>, dim3(l.n_partials, (unsigned)heads, 6), dim3(256), 0, p.stream, sa, partials);
    else
        hipLaunchKernelGGL(head_stats_kernel<128>, dim3(l.n_partials, (unsigned)heads, 6), dim3(256), 0, p.stream, sa, partials);
    const int n_blocks = (p.Lkv + 31) / 32;
    int cx = n_blocks < 512 ? n_blocks : 512;
    if (p.d == 64)
        hipLaunchKernelGGL(convert_values_kernel<64>, dim3(cx, (unsigned)heads), dim3(256), 0, p.stream, bf(p.v), bf(p.tv), partials,
                           l.n_partials, stats, tickets, V16, tV16, n_blocks, p.scale, p.Lkv, p.H, p.layout);
    else
        hipLaunchKernelGGL(convert_values_kernel<128>, dim3(cx, (unsigned)heads), dim3(256), 0, p.stream, bf(p.v), bf(p.tv), partials,
                           l.n_partials, stats, tickets, V16, tV16, n_blocks, p.scale, p.Lkv, p.H, p.layout);
    out->stats = stats;
    out->wg_flags = wg_flags;
    out->v16 = V16;
    out->tv16 = tV16;
    return hipGetLastError();
}

}  // namespace attn_jvp
