// Per-element arithmetic of the group-wise rational function (FlashKAT paper,
// Eq. "pade"), shared by the elementwise kernels and the fused GR-KAN layer
// kernel.  Device code only.
#ifndef GRKAN_ELEM_H_
#define GRKAN_ELEM_H_

#include <hip/hip_runtime.h>

namespace grkan {

// --------------------------------------------------------------------------
// coefficients of one group for numerator degree M and denominator degree N
// (scalar registers when the group is wave-uniform, vector registers in the
// flat walk).  Entries no kernel reads cost nothing: everything is unrolled.
// --------------------------------------------------------------------------
template <int M, int N> struct Coef {
    float a[M + 1];  // a_0 .. a_M
    float b[N];      // b_1 .. b_N  (b[j - 1] = b_j)
    float da[M + 1]; // i * a_i, the coefficients of P'  (da[0] unused)
    float db[N];     // j * b_j, the coefficients of Aden'
    double bd[N];    // b_j in double, for the float32-I/O kernels (see aden_of)
};

template <int M, int N>
__device__ __forceinline__ Coef<M, N> load_coef(const float *__restrict__ A, const float *__restrict__ B, int g)
{
    const float *a = A + (size_t)g * (M + 1);
    const float *b = B + (size_t)g * N;
    Coef<M, N> c;
#pragma unroll
    for (int i = 0; i <= M; ++i) {
        c.a[i] = a[i];
        c.da[i] = i >= 2 ? (float)i * a[i] : a[i];
    }
#pragma unroll
    for (int j = 0; j < N; ++j) {
        c.b[j] = b[j];
        c.db[j] = j >= 1 ? (float)(j + 1) * b[j] : b[j];
        c.bd[j] = (double)b[j];
    }
    return c;
}

// --------------------------------------------------------------------------
// per-element arithmetic (float32)
// --------------------------------------------------------------------------

// Aden = x (b_1 + b_2 x + ... + b_N x^(N-1)) by Horner.
//
// WIDE = true (float32 I/O): in double, rounded once to float32.  Q = 1 + |Aden|
// sits in every result as 1/Q or 1/Q^2, and next to a real root of the
// denominator polynomial at |x| of a few units Aden is a small difference of
// large monomials: in float32 its absolute error eps * sum |b_j||x|^j would be a
// relative error of that size in Q ~ 1 and, since those are exactly the
// elements where P/Q^2 is huge, would dominate the error of the summed
// b-gradients whatever the summation order (measured: 100x on their mean
// absolute error with N(0,1) coefficients).  Double FMA issues at the unpacked
// float32 rate on this chip, and the float32-I/O kernels are bound by HBM, so
// this is free there.
// WIDE = false (16-bit I/O): in float32.  That backward kernel is bound by
// the vector ALU (the conversions and double compares cost it 12 %), and its
// outputs are rounded to 8 or 11 significant bits anyway.
template <bool WIDE, int M, int N> __device__ __forceinline__ float aden_of(float x, const Coef<M, N> &c)
{
    if constexpr (WIDE) {
        const double xd = (double)x;
        double h = c.bd[N - 1];
#pragma unroll
        for (int j = N - 2; j >= 0; --j)
            h = fma(h, xd, c.bd[j]);
        return (float)(h * xd);
    } else {
        float h = c.b[N - 1];
#pragma unroll
        for (int j = N - 2; j >= 0; --j)
            h = fmaf(h, x, c.b[j]);
        return h * x;
    }
}

template <int M, int N> __device__ __forceinline__ float numerator_of(float x, const Coef<M, N> &c)
{
    float p = c.a[M];
#pragma unroll
    for (int i = M - 1; i >= 0; --i)
        p = fmaf(p, x, c.a[i]);
    return p;
}

// Q = 1 + |Aden| for the forward pass.  WIDE = false: Aden = x h(x) is not needed by itself there, and
// |x h| = |x| |h|, so the product and the addition are one fused multiply-add (one instruction and
// one rounding fewer).
template <bool WIDE, int M, int N> __device__ __forceinline__ float q_of(float x, const Coef<M, N> &c)
{
    if constexpr (WIDE) {
        return 1.0f + fabsf(aden_of<true>(x, c));
    } else {
        float h = c.b[N - 1];
#pragma unroll
        for (int j = N - 2; j >= 0; --j)
            h = fmaf(h, x, c.b[j]);
        return fmaf(fabsf(h), fabsf(x), 1.0f);
    }
}

// Eq. "pade": P by Horner in float32, Q as above, and one hardware
// reciprocal (1 ulp) instead of a division.
template <bool WIDE, int M, int N> __device__ __forceinline__ float fwd_elem(float x, const Coef<M, N> &c)
{
    const float p = numerator_of(x, c);
    const float q = q_of<WIDE>(x, c);
    return p * __builtin_amdgcn_rcpf(q);
}

} // namespace grkan
#endif // GRKAN_ELEM_H_
