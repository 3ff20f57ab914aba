// Fused epilogues of the bf16 matrix-core GEMMs: what happens to 4 consecutive output columns of one
// row on their way from the float32 accumulators to memory (bias, GELU, GELU', residual add/subtract).
#pragma once
#include "mfma.h"

namespace rev {

// Normal CDF for the bf16 GELU epilogues: Phi(x) = 1/2 + x * P(x^2) on |x| <= 3.8 with a degree-6 minimax-fitted P
// (absolute error < 6.5e-5 there; plain FMAs, no transcendental), and exactly 0 / 1 beyond, so that gelu(x) is exactly
// 0 for x < -3.8 (the true value is below 2.8e-4 in magnitude and shrinking) and exactly x for x > 3.8.  The bound is an
// absolute one: relative to the small negative-tail values of gelu it is not small (4.6 % at x = -3).
// The density, needed by the derivative only, is one exp.
__device__ __forceinline__ float gelu_cdf(float x) {
    const float xc = fminf(fmaxf(x, -3.8f), 3.8f);
    const float u = xc * xc;
    float p = 3.665773107e-08f;
    p = p * u - 2.272460051e-06f;
    p = p * u + 6.068476796e-05f;
    p = p * u - 9.315473144e-04f;
    p = p * u + 9.316634387e-03f;
    p = p * u - 6.571978331e-02f;
    p = p * u + 3.986767530e-01f;
    float r = 0.5f + xc * p;
    r = x < -3.8f ? 0.f : r;
    r = x > 3.8f ? 1.f : r;
    return r;
}
__device__ __forceinline__ float gelu_pdf(float x) { return 0.39894228040143268f * __expf(-0.5f * x * x); }

typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4_t ld_bf16x4(const void* p) {
    const u32x2_t u = *reinterpret_cast<const u32x2_t*>(p);
    f32x4_t r;
    r[0] = __uint_as_float(u[0] << 16);
    r[1] = __uint_as_float(u[0] & 0xFFFF0000u);
    r[2] = __uint_as_float(u[1] << 16);
    r[3] = __uint_as_float(u[1] & 0xFFFF0000u);
    return r;
}
__device__ __forceinline__ void st_bf16x4(void* p, f32x4_t v) {
    bf16x4_t b;
#pragma unroll
    for (int e = 0; e < 4; ++e) b[e] = (__bf16)v[e];
    *reinterpret_cast<bf16x4_t*>(p) = b;
}

// The epilogue operand of 4 consecutive output columns n..n+3 of row m (residual stream or saved
// pre-activation), loaded ahead of the arithmetic so that all loads of a panel are in flight together.
template <int KIND>
__device__ __forceinline__ f32x4_t epi_load4(const Epi& e, int m, int n) {
    const int64_t idx = (int64_t)m * e.ldo + n;
    if (KIND == EPI_RESIDUAL) return *reinterpret_cast<const f32x4_t*>(e.res + idx);
    if (KIND == EPI_GELU_BWD) {
        // the 4 bf16 values stay packed (2 registers) until epi_store4 unpacks them
        const u32x2_t u = *reinterpret_cast<const u32x2_t*>(reinterpret_cast<const bf16*>(e.aux) + idx);
        return f32x4_t{__uint_as_float(u[0]), __uint_as_float(u[1]), 0.f, 0.f};
    }
    return f32x4_t{0.f, 0.f, 0.f, 0.f};
}

// 4 consecutive output columns n..n+3 of row m; `opnd` is what epi_load4 returned for them
// (returns the float32 values behind the stored output, for the fused column sums)
template <int KIND>
__device__ __forceinline__ f32x4_t epi_store4(const Epi& e, int m, int n, f32x4_t acc, f32x4_t bv, f32x4_t opnd) {
    const int64_t idx = (int64_t)m * e.ldo + n;
    if (KIND == EPI_BIAS || KIND == EPI_BIAS_GELU || KIND == EPI_RESIDUAL) acc += bv;
    if (KIND == EPI_BIAS) {
        st_bf16x4(reinterpret_cast<bf16*>(e.out) + idx, acc);
    } else if (KIND == EPI_BIAS_GELU) {
        if (e.out != nullptr) st_bf16x4(reinterpret_cast<bf16*>(e.out) + idx, acc);   // the pre-activation is optional
        f32x4_t a;
#pragma unroll
        for (int k = 0; k < 4; ++k) a[k] = acc[k] * gelu_cdf(acc[k]);
        st_bf16x4(reinterpret_cast<bf16*>(e.out2) + idx, a);
    } else if (KIND == EPI_RESIDUAL) {
        *reinterpret_cast<f32x4_t*>(e.outf + idx) = opnd + e.sign * acc;
    } else if (KIND == EPI_GELU_BWD) {
        const unsigned u0 = __float_as_uint(opnd[0]), u1 = __float_as_uint(opnd[1]);
        const f32x4_t h = {__uint_as_float(u0 << 16), __uint_as_float(u0 & 0xFFFF0000u),
                           __uint_as_float(u1 << 16), __uint_as_float(u1 & 0xFFFF0000u)};
        f32x4_t o;
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = acc[k] * (gelu_cdf(h[k]) + h[k] * gelu_pdf(h[k]));
        st_bf16x4(reinterpret_cast<bf16*>(e.out) + idx, o);
        return o;
    } else if (KIND == EPI_PLAIN) {
        st_bf16x4(reinterpret_cast<bf16*>(e.out) + idx, acc);
    } else {
        *reinterpret_cast<f32x4_t*>(e.outf + idx) = acc;
    }
    return acc;
}

}  // namespace rev
