// The paper's Algorithm 1 (KAT's original backward pass) as a measurement
// baseline: one thread per element, coefficients re-read from global memory by
// every thread, ten global float atomics per element.  Deliberately not
// optimised -- it is the "before" of the paper's comparison, kept out of the
// product path (see include/grkan_alg1.h).
#include <hip/hip_runtime.h>

#include "../../include/grkan_alg1.h"

namespace {

constexpr int kBlock = 256; // S_block of Algorithm 1

__global__ __launch_bounds__(kBlock) void grkan_alg1_kernel(const float *x, const float *dy, const float *A,
                                                            const float *B, float *dx, float *dA, float *dB,
                                                            int64_t n_elem, int32_t D, int32_t dg)
{
    const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= n_elem)
        return;
    const int k = (int)((e % D) / dg); // the element's group
    const float *a = A + (size_t)k * 6;
    const float *b = B + (size_t)k * 4;
    const float xv = x[e];
    const float d = dy[e];

    float xp[6];
    xp[0] = 1.0f;
    for (int i = 1; i < 6; ++i)
        xp[i] = xp[i - 1] * xv;
    float P = 0.0f, dP = 0.0f, Ad = 0.0f, dAd = 0.0f;
    for (int i = 0; i < 6; ++i)
        P += a[i] * xp[i];
    for (int i = 1; i < 6; ++i)
        dP += (float)i * a[i] * xp[i - 1];
    for (int j = 1; j <= 4; ++j)
        Ad += b[j - 1] * xp[j];
    for (int j = 1; j <= 4; ++j)
        dAd += (float)j * b[j - 1] * xp[j - 1];
    const float Q = 1.0f + fabsf(Ad);
    const float s = Ad > 0.0f ? 1.0f : (Ad < 0.0f ? -1.0f : 0.0f);

    dx[e] = d * (dP / Q - s * dAd * P / (Q * Q));
    for (int i = 0; i < 6; ++i)
        atomicAdd(&dA[k * 6 + i], d * xp[i] / Q);
    for (int j = 1; j <= 4; ++j)
        atomicAdd(&dB[k * 4 + (j - 1)], -d * xp[j] * s * P / (Q * Q));
}

} // namespace

extern "C" grkan_status_t grkan_alg1_bwd(const float *x, const float *dy, const float *A, const float *B,
                                         float *dx, float *dA, float *dB,
                                         int64_t rows, int32_t D, int32_t G, void *hip_stream)
{
    if (rows < 0 || D <= 0 || G <= 0 || D % G != 0)
        return GRKAN_ERR_SHAPE;
    if (!A || !B || !dA || !dB || (rows > 0 && (!x || !dy || !dx)))
        return GRKAN_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(dy) | reinterpret_cast<uintptr_t>(dx) |
         reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B) | reinterpret_cast<uintptr_t>(dA) |
         reinterpret_cast<uintptr_t>(dB)) % 4 != 0)
        return GRKAN_ERR_ALIGN;
    if (rows > (((int64_t)1 << 40) - 1) / D)
        return GRKAN_ERR_UNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (hipMemsetAsync(dA, 0, (size_t)G * 6 * sizeof(float), stream) != hipSuccess ||
        hipMemsetAsync(dB, 0, (size_t)G * 4 * sizeof(float), stream) != hipSuccess)
        return GRKAN_ERR_LAUNCH;
    const int64_t n_elem = rows * (int64_t)D;
    if (n_elem == 0)
        return GRKAN_OK;
    const int64_t blocks = (n_elem + kBlock - 1) / kBlock;
    if (blocks > 0x7fffffff)
        return GRKAN_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(grkan_alg1_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, stream, x, dy, A, B, dx, dA, dB,
                       n_elem, D, D / G);
    return hipGetLastError() == hipSuccess ? GRKAN_OK : GRKAN_ERR_LAUNCH;
}
