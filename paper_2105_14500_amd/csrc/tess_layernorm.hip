// Local parts of the layer normalisation of a hidden dimension that is spread over the q
// processors of a grid row (Section 3.2, "Other procedure"): per-row sum and sum of squares
// of this processor's [m, w] block, and the normalisation of the block once the sums have
// been reduced over the grid row.  Both are streaming kernels bound by HBM bandwidth:
// row_sums reads 2 (bf16) or 4 (fp32) bytes per element and writes 8 bytes per row;
// normalize reads and writes one element each.
#include "tess_internal.h"

namespace tess {

typedef uint32_t u32x4_ln __attribute__((ext_vector_type(4)));
typedef float floatx4_ln __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// One wavefront per row, four rows per workgroup.  Lanes stride over 16-byte chunks of the
// row (fully coalesced); a ragged head or tail and unaligned rows fall back to elements.
template <bool F32>
__global__ __launch_bounds__(256) void tess_row_sums_kernel(const void* x, int64_t m, int64_t w,
                                                            int64_t ldx, int accumulate, float* out)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= m) return;
    constexpr int EPC = F32 ? 4 : 8;                       // elements per 16-byte chunk
    const char* base = (const char*)x + row * ldx * (F32 ? 4 : 2);
    const bool vec = ((reinterpret_cast<uintptr_t>(base) & 15u) == 0);
    float s1 = 0.0f, s2 = 0.0f;
    int64_t done = 0;
    if (vec) {
        const int64_t chunks = w / EPC;
        for (int64_t c = lane; c < chunks; c += 64) {
            if (F32) {
                const floatx4_ln v = ((const floatx4_ln*)base)[c];
#pragma unroll
                for (int e = 0; e < 4; ++e) { s1 += v[e]; s2 = fmaf(v[e], v[e], s2); }
            } else {
                const u32x4_ln v = ((const u32x4_ln*)base)[c];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float lo = __uint_as_float(v[e] << 16), hi = __uint_as_float(v[e] & 0xffff0000u);
                    s1 += lo; s2 = fmaf(lo, lo, s2);
                    s1 += hi; s2 = fmaf(hi, hi, s2);
                }
            }
        }
        done = chunks * EPC;
    }
    for (int64_t u = done + lane; u < w; u += 64) {
        const float v = F32 ? ((const float*)base)[u]
                            : __uint_as_float(((uint32_t)((const uint16_t*)base)[u]) << 16);
        s1 += v;
        s2 = fmaf(v, v, s2);
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    if (lane == 0) {
        float* o = out + 2 * row;
        o[0] = accumulate ? o[0] + s1 : s1;
        o[1] = accumulate ? o[1] + s2 : s2;
    }
}

// xhat = (x - S1/n) / sqrt(S2/n - (S1/n)^2 + eps), one wavefront per row.
template <bool F32>
__global__ __launch_bounds__(256) void tess_normalize_kernel(const void* x, int64_t m, int64_t w,
                                                             int64_t ldx, const float* sums,
                                                             float inv_n, float eps, void* out,
                                                             int64_t ldo)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= m) return;
    const float mean = sums[2 * row] * inv_n;
    // E[X^2] - E[X]^2 is a variance: rounding can push the difference below zero for rows
    // whose mean is large against their spread
    const float var = fmaxf(fmaf(-mean, mean, sums[2 * row + 1] * inv_n), 0.0f);
    const float rstd = 1.0f / sqrtf(var + eps);
    constexpr int EPC = F32 ? 4 : 8;
    const char* src = (const char*)x + row * ldx * (F32 ? 4 : 2);
    char* dst = (char*)out + row * ldo * (F32 ? 4 : 2);
    const bool vec = (((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) == 0);
    int64_t done = 0;
    if (vec) {
        const int64_t chunks = w / EPC;
        for (int64_t c = lane; c < chunks; c += 64) {
            if (F32) {
                floatx4_ln v = ((const floatx4_ln*)src)[c];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (v[e] - mean) * rstd;
                ((floatx4_ln*)dst)[c] = v;
            } else {
                const u32x4_ln v = ((const u32x4_ln*)src)[c];
                u32x4_ln o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float lo = (__uint_as_float(v[e] << 16) - mean) * rstd;
                    const float hi = (__uint_as_float(v[e] & 0xffff0000u) - mean) * rstd;
                    typedef __bf16 bf16x2_ln __attribute__((ext_vector_type(2)));
                    typedef float floatx2_ln __attribute__((ext_vector_type(2)));
                    const floatx2_ln p = {lo, hi};
                    o[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2_ln));
                }
                ((u32x4_ln*)dst)[c] = o;
            }
        }
        done = chunks * EPC;
    }
    for (int64_t u = done + lane; u < w; u += 64) {
        if (F32) {
            ((float*)dst)[u] = (((const float*)src)[u] - mean) * rstd;
        } else {
            const float v = (__uint_as_float(((uint32_t)((const uint16_t*)src)[u]) << 16) - mean) * rstd;
            ((__bf16*)dst)[u] = (__bf16)v;
        }
    }
}

// Element u of a row of 2- or 4-byte values as fp32.
template <bool F32>
__device__ __forceinline__ float ln_load(const char* row, int64_t u)
{
    return F32 ? ((const float*)row)[u] : __uint_as_float(((uint32_t)((const uint16_t*)row)[u]) << 16);
}

// Backward partial sums of one block: per row sum(xhat * g) and sum(g).  One wavefront per
// row, 16-byte chunks when both rows are aligned.
template <bool F32>
__global__ __launch_bounds__(256) void tess_row_sums_bwd_kernel(const void* xhat, const void* g,
                                                                int64_t m, int64_t w, int64_t ldx,
                                                                int64_t ldg, int accumulate, float* out)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= m) return;
    constexpr int EPC = F32 ? 4 : 8, ES = F32 ? 4 : 2;
    const char* xr = (const char*)xhat + row * ldx * ES;
    const char* gr = (const char*)g + row * ldg * ES;
    const bool vec = (((reinterpret_cast<uintptr_t>(xr) | reinterpret_cast<uintptr_t>(gr)) & 15u) == 0);
    float a = 0.0f, b = 0.0f;
    int64_t done = 0;
    if (vec) {
        const int64_t chunks = w / EPC;
        for (int64_t c = lane; c < chunks; c += 64) {
            if (F32) {
                const floatx4_ln xv = ((const floatx4_ln*)xr)[c], gv = ((const floatx4_ln*)gr)[c];
#pragma unroll
                for (int e = 0; e < 4; ++e) { a = fmaf(xv[e], gv[e], a); b += gv[e]; }
            } else {
                const u32x4_ln xv = ((const u32x4_ln*)xr)[c], gv = ((const u32x4_ln*)gr)[c];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float xl = __uint_as_float(xv[e] << 16), xh = __uint_as_float(xv[e] & 0xffff0000u);
                    const float gl = __uint_as_float(gv[e] << 16), gh = __uint_as_float(gv[e] & 0xffff0000u);
                    a = fmaf(xl, gl, a); b += gl;
                    a = fmaf(xh, gh, a); b += gh;
                }
            }
        }
        done = chunks * EPC;
    }
    for (int64_t u = done + lane; u < w; u += 64) {
        const float xv = ln_load<F32>(xr, u), gv = ln_load<F32>(gr, u);
        a = fmaf(xv, gv, a);
        b += gv;
    }
    a = wave_sum(a);
    b = wave_sum(b);
    if (lane == 0) {
        float* o = out + 2 * row;
        o[0] = accumulate ? o[0] + a : a;
        o[1] = accumulate ? o[1] + b : b;
    }
}

// X' = (g - (xhat * A + B) / n) * rstd with the reduced backward sums A, B and rstd from the
// reduced forward sums.  Element-wise per lane (the kernel is bound by its three streams).
template <bool F32>
__global__ __launch_bounds__(256) void tess_layernorm_bwd_kernel(const void* xhat, const void* g,
                                                                 int64_t m, int64_t w, int64_t ldx,
                                                                 int64_t ldg, const float* sums_bwd,
                                                                 const float* sums_fwd, float inv_n,
                                                                 float eps, void* out, int64_t ldo)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= m) return;
    const float mean = sums_fwd[2 * row] * inv_n;
    const float var = fmaxf(fmaf(-mean, mean, sums_fwd[2 * row + 1] * inv_n), 0.0f);
    const float rstd = 1.0f / sqrtf(var + eps);
    const float A = sums_bwd[2 * row] * inv_n, Bc = sums_bwd[2 * row + 1] * inv_n;
    constexpr int EPC = F32 ? 4 : 8, ES = F32 ? 4 : 2;
    const char* xr = (const char*)xhat + row * ldx * ES;
    const char* gr = (const char*)g + row * ldg * ES;
    char* dst = (char*)out + row * ldo * ES;
    const bool vec = (((reinterpret_cast<uintptr_t>(xr) | reinterpret_cast<uintptr_t>(gr) |
                        reinterpret_cast<uintptr_t>(dst)) & 15u) == 0);
    int64_t done = 0;
    if (vec) {
        const int64_t chunks = w / EPC;
        for (int64_t c = lane; c < chunks; c += 64) {
            if (F32) {
                const floatx4_ln xv = ((const floatx4_ln*)xr)[c], gv = ((const floatx4_ln*)gr)[c];
                floatx4_ln o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (gv[e] - fmaf(xv[e], A, Bc)) * rstd;
                ((floatx4_ln*)dst)[c] = o;
            } else {
                const u32x4_ln xv = ((const u32x4_ln*)xr)[c], gv = ((const u32x4_ln*)gr)[c];
                u32x4_ln o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float xl = __uint_as_float(xv[e] << 16), xh = __uint_as_float(xv[e] & 0xffff0000u);
                    const float gl = __uint_as_float(gv[e] << 16), gh = __uint_as_float(gv[e] & 0xffff0000u);
                    typedef __bf16 bf16x2_ln __attribute__((ext_vector_type(2)));
                    typedef float floatx2_ln __attribute__((ext_vector_type(2)));
                    const floatx2_ln p = {(gl - fmaf(xl, A, Bc)) * rstd, (gh - fmaf(xh, A, Bc)) * rstd};
                    o[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2_ln));
                }
                ((u32x4_ln*)dst)[c] = o;
            }
        }
        done = chunks * EPC;
    }
    for (int64_t u = done + lane; u < w; u += 64) {
        const float v = (ln_load<F32>(gr, u) - fmaf(ln_load<F32>(xr, u), A, Bc)) * rstd;
        if (F32) ((float*)dst)[u] = v;
        else ((__bf16*)dst)[u] = (__bf16)v;
    }
}

hipError_t launch_row_sums_bwd(const void* xhat, const void* g, int64_t m, int64_t w, int64_t ldx,
                               int64_t ldg, int in_f32, int accumulate, float* out, hipStream_t s)
{
    const dim3 grid((unsigned)((m + 3) / 4)), block(256);
    if (in_f32) hipLaunchKernelGGL(tess_row_sums_bwd_kernel<true>, grid, block, 0, s, xhat, g, m, w, ldx, ldg, accumulate, out);
    else hipLaunchKernelGGL(tess_row_sums_bwd_kernel<false>, grid, block, 0, s, xhat, g, m, w, ldx, ldg, accumulate, out);
    return hipGetLastError();
}

hipError_t launch_layernorm_bwd(const void* xhat, const void* g, int64_t m, int64_t w, int64_t ldx,
                                int64_t ldg, int in_f32, const float* sums_bwd, const float* sums_fwd,
                                float inv_n, float eps, void* out, int64_t ldo, hipStream_t s)
{
    const dim3 grid((unsigned)((m + 3) / 4)), block(256);
    if (in_f32) hipLaunchKernelGGL(tess_layernorm_bwd_kernel<true>, grid, block, 0, s, xhat, g, m, w, ldx, ldg, sums_bwd, sums_fwd, inv_n, eps, out, ldo);
    else hipLaunchKernelGGL(tess_layernorm_bwd_kernel<false>, grid, block, 0, s, xhat, g, m, w, ldx, ldg, sums_bwd, sums_fwd, inv_n, eps, out, ldo);
    return hipGetLastError();
}

hipError_t launch_row_sums(const void* x, int64_t m, int64_t w, int64_t ldx, int in_f32,
                           int accumulate, float* out, hipStream_t s)
{
    const dim3 grid((unsigned)((m + 3) / 4)), block(256);
    if (in_f32) hipLaunchKernelGGL(tess_row_sums_kernel<true>, grid, block, 0, s, x, m, w, ldx, accumulate, out);
    else hipLaunchKernelGGL(tess_row_sums_kernel<false>, grid, block, 0, s, x, m, w, ldx, accumulate, out);
    return hipGetLastError();
}

hipError_t launch_normalize(const void* x, int64_t m, int64_t w, int64_t ldx, int in_f32,
                            const float* sums, float inv_n, float eps, void* out, int64_t ldo,
                            hipStream_t s)
{
    const dim3 grid((unsigned)((m + 3) / 4)), block(256);
    if (in_f32) hipLaunchKernelGGL(tess_normalize_kernel<true>, grid, block, 0, s, x, m, w, ldx, sums, inv_n, eps, out, ldo);
    else hipLaunchKernelGGL(tess_normalize_kernel<false>, grid, block, 0, s, x, m, w, ldx, sums, inv_n, eps, out, ldo);
    return hipGetLastError();
}

}  // namespace tess
