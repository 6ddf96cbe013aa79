// Fused GR-KAN layer on gfx950 (MI355X): out = W F(x) (+ bias) in one kernel
// (FlashKAT paper, Sec. "Kolmogorov-Arnold Transformer", Eq. "GR_KAN" with the
// group-wise rational function F of Eq. "pade").
//
// Run as two kernels, F(x) is written to HBM and read back by the matrix
// product.  Here the rational function is the prologue of the matrix product's
// token operand: x is loaded, F is evaluated in float32 registers, rounded to
// bfloat16 and written to LDS, from where the matrix cores consume it.  F(x)
// never exists in HBM.
//
// Geometry (one workgroup = 4 wavefronts, one per SIMD, up to 512 registers each):
//   * a workgroup owns a tile of BM = 16 MT tokens x BN = 64 NT output channels
//     and sweeps the whole contraction dimension K = D_in;
//   * wavefront w owns the 16 NT channels [16 NT w, 16 NT (w + 1)) of the tile for
//     all BM tokens: MT x NT accumulators of v_mfma_f32_16x16x32_bf16, the
//     weights as the row operand, F(x) as the column operand, so that a lane
//     ends up with four consecutive output channels of one token;
//   * W streams through LDS in stages of 32 k (64 bytes per row), double
//     buffered through registers; x in pairs of stages (64 k = one 128-byte line
//     per token), so that F of the next pair is computed while the matrix cores
//     work on the current one; rows are padded by 16 bytes so that the 16 lanes
//     of an operand read hit 16 different 16-byte bank groups;
//   * the coefficient group of a stage is wave-uniform (d_g is a multiple of 32),
//     so the coefficients live in scalar registers.
//
// The tile is wide in the channel direction on purpose: every token-operand
// element costs about 16 vector-ALU issue slots (F) once per workgroup that
// consumes it, against BN / 512 matrix-core cycles per lane; only from
// BN = 512 up does the matrix work outlast the evaluation of F.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/grkan.h"
#include "grkan_elem.h"

namespace grkan {
namespace lin {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

typedef const __attribute__((address_space(1))) char *gcptr_t;
typedef __attribute__((address_space(1))) char *gptr_t;
typedef __attribute__((address_space(3))) char *lptr_t;

constexpr int kThreads = 256;
constexpr int kMT = 7;                 // 16-token sub-tiles per workgroup: BM = 112
constexpr int kBM = 16 * kMT;
constexpr int kXRows = 128;            // rows of an x buffer (all 128 loader lanes write; BM are read)
constexpr int kXPitch = 144;           // 64 k (128 B) + 16 B pad
constexpr int kWPitch = 80;            // 32 k (64 B) + 16 B pad
constexpr int kXBuf = kXRows * kXPitch; // 18432

struct LinArgs {
    const char *x;     // bfloat16 [rows, K]
    const char *W;     // bfloat16 [Nout, K]
    const float *bias; // float32 [Nout] or NULL
    char *out;         // OUT [rows, Nout]
    const float *A;    // [G, m + 1]
    const float *B;    // [G, n]
    int64_t rows;
    int32_t K;
    int32_t Nout;
    int32_t dgc;       // channels per coefficient group (a multiple of 32)
    int32_t mblocks;   // ceil(rows / BM)
    int32_t nblocks;   // ceil(Nout / BN)
};

__device__ __forceinline__ uint64_t uniform_u64(uint64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ u32x4 gload16(uint64_t uniform_base, uint32_t lane_off)
{
    return *(const __attribute__((address_space(1))) u32x4 *)((gcptr_t)uniform_u64(uniform_base) + lane_off);
}

__device__ __forceinline__ bf16x8 lds_read16(uint32_t addr)
{
    return *(const __attribute__((address_space(3))) bf16x8 *)(uintptr_t)addr;
}

__device__ __forceinline__ void lds_write16(uint32_t addr, u32x4 v)
{
    *(__attribute__((address_space(3))) u32x4 *)(uintptr_t)addr = v;
}

// two bfloat16 of one word -> float32, F, -> one word of two bfloat16 (round to nearest even)
template <int M, int N> __device__ __forceinline__ uint32_t rational_pair(uint32_t w, const Coef<M, N> &c)
{
    const float lo = __builtin_bit_cast(float, w << 16);
    const float hi = __builtin_bit_cast(float, w & 0xffff0000u);
    f32x2 y;
    y[0] = fwd_elem<false, M, N>(lo, c);
    y[1] = fwd_elem<false, M, N>(hi, c);
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(y, bf16x2));
}

template <typename OUT> struct OutPack;
template <> struct OutPack<float> {
    static __device__ __forceinline__ void store(gptr_t p, f32x4 v)
    {
        *(__attribute__((address_space(1))) f32x4 *)p = v;
    }
};
struct bf16_out {
    uint16_t bits;
};
template <> struct OutPack<bf16_out> {
    static __device__ __forceinline__ void store(gptr_t p, f32x4 v)
    {
        f32x2 a, b;
        a[0] = v[0];
        a[1] = v[1];
        b[0] = v[2];
        b[1] = v[3];
        u32x2 r;
        r[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2));
        r[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(b, bf16x2));
        *(__attribute__((address_space(1))) u32x2 *)p = r;
    }
};

// NT: 16-channel sub-tiles per wavefront (BN = 64 NT).  NEDGE: the last channel
// block may be partial (weight rows are clamped, stores predicated).
template <int NT, typename OUT, bool NEDGE, int M, int N>
__global__ __launch_bounds__(kThreads, 1) void grkan_linear_fwd_kernel(const LinArgs a)
{
    constexpr int MT = kMT;
    constexpr int WN = 16 * NT;
    constexpr int BN = 4 * WN;
    constexpr int kWBuf = BN * kWPitch;
    constexpr uint32_t kWs0 = 2 * kXBuf;
    extern __shared__ __align__(16) char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // workgroup -> (token block, channel block): the channel blocks of one token block run on one
    // XCD (workgroups go round-robin over the 8 XCDs), so that they share its L2 copy of the x rows
    const int xcd = (int)blockIdx.x & 7;
    const int slot = (int)blockIdx.x >> 3;
    const int nb = slot % a.nblocks;
    const int mb = (slot / a.nblocks) * 8 + xcd;
    if (mb >= a.mblocks)
        return;
    const int64_t m0 = (int64_t)mb * kBM;
    const int32_t n0 = nb * BN;
    const uint32_t K2 = (uint32_t)a.K * 2u; // bytes per row of x and W

    // ---- x loader: waves 0, 1 take the first 32 k of a pair for rows 0..127, waves 2, 3 the last 32
    const int xhalf = wave >> 1;
    const int xrow = (wave & 1) * 64 + lane;
    int64_t xg = m0 + xrow;
    if (xg > a.rows - 1)
        xg = a.rows - 1; // rows past the end read the last row (never stored)
    const uint64_t x_base = reinterpret_cast<uint64_t>(a.x) + (uint64_t)m0 * K2 + (uint64_t)xhalf * 64u;
    const uint32_t x_lane = (uint32_t)((xg - m0) * (int64_t)K2);
    uint32_t x_dst = lds0 + (uint32_t)xrow * kXPitch + (uint32_t)xhalf * 64u; // + buffer

    // ---- W loader: unit i * 256 + tid -> row i * 64 + tid / 4, 16-byte piece tid % 4
    const int wrow = tid >> 2;
    const int wkg = tid & 3;
    const uint64_t w_base = reinterpret_cast<uint64_t>(a.W) + (uint64_t)n0 * K2;
    uint32_t w_lane[NEDGE ? NT : 1];
    if constexpr (NEDGE) {
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            int r = i * 64 + wrow;
            if (n0 + r > a.Nout - 1)
                r = a.Nout - 1 - n0;
            w_lane[i] = (uint32_t)r * K2 + (uint32_t)wkg * 16u;
        }
    } else {
        w_lane[0] = (uint32_t)wrow * K2 + (uint32_t)wkg * 16u;
    }
    const uint32_t w_dst = lds0 + kWs0 + (uint32_t)wrow * kWPitch + (uint32_t)wkg * 16u; // + buffer + i * 64 rows

    auto w_load = [&](int i, uint32_t kbyte) -> u32x4 {
        if constexpr (NEDGE)
            return gload16(w_base + kbyte, w_lane[i]);
        else
            return gload16(w_base + kbyte + (uint64_t)i * 64u * K2, w_lane[0]);
    };

    // ---- operand reads: lane -> row lane % 16 of a 16-row sub-tile, 16-byte piece lane / 16
    const uint32_t xf_base = lds0 + (uint32_t)(lane & 15) * kXPitch + (uint32_t)(lane >> 4) * 16u;
    const uint32_t wf_base =
        lds0 + kWs0 + (uint32_t)(wave * WN + (lane & 15)) * kWPitch + (uint32_t)(lane >> 4) * 16u;

    f32x4 acc[NT][MT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            acc[nt][mt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    const int32_t n_pairs = a.K >> 6;
    const uint32_t k_last_stage = K2 - 64u;  // byte offset of the last 32-k stage in a row
    const uint32_t k_last_pair = K2 - 128u;

    // coefficients of the group the wave's next F work lies in
    int g_cur = (xhalf * 32) / a.dgc;
    Coef<M, N> c = load_coef<M, N>(a.A, a.B, g_cur);
    auto coef_for = [&](uint32_t kbyte_pair) {
        const int g = (int)((kbyte_pair / 2u + (uint32_t)xhalf * 32u) / (uint32_t)a.dgc);
        if (g != g_cur) {
            g_cur = g;
            c = load_coef<M, N>(a.A, a.B, g);
        }
    };

    u32x4 xq[4];  // this lane's 32 k of the pair F works on next
    u32x4 wr[NT]; // this lane's pieces of the next W stage

    // ---- prologue: pair 0 and stage 0 into LDS, pair 1 and stage 1 into registers
#pragma unroll
    for (int u = 0; u < 4; ++u)
        xq[u] = gload16(x_base, x_lane + (uint32_t)u * 16u);
#pragma unroll
    for (int i = 0; i < NT; ++i)
        wr[i] = w_load(i, 0);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        u32x4 y;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            y[j] = rational_pair<M, N>(xq[u][j], c);
        lds_write16(x_dst + (uint32_t)u * 16u, y);
    }
#pragma unroll
    for (int i = 0; i < NT; ++i)
        lds_write16(w_dst + (uint32_t)i * 64u * kWPitch, wr[i]);
    {
        const uint32_t kp = n_pairs > 1 ? 128u : k_last_pair;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            xq[u] = gload16(x_base + kp, x_lane + (uint32_t)u * 16u);
        coef_for(kp);
#pragma unroll
        for (int i = 0; i < NT; ++i)
            wr[i] = w_load(i, 64u);
    }
    __syncthreads();

    // One stage: the matrix products of stage s = 2 p + Q from LDS, and beside them the
    // hand-over of stage s + 1 (registers -> LDS; its successor s + 2 -> registers) and half of
    // F for pair p + 1.  Addresses past the end of K are clamped to the last stage / pair: the
    // surplus loads read valid memory and what they bring is never consumed.
    auto stage = [&](auto Qc, uint32_t xsel_read, uint32_t xsel_write, uint32_t kbyte_stage2, uint32_t kbyte_pair2) {
        constexpr int Q = decltype(Qc)::value;
        const uint32_t xb = xf_base + xsel_read + (uint32_t)Q * 64u;
        const uint32_t wb = wf_base + (uint32_t)Q * kWBuf;
        const uint32_t wd = w_dst + (uint32_t)(1 - Q) * kWBuf;
        bf16x8 xf[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            xf[mt] = lds_read16(xb + (uint32_t)mt * 16u * kXPitch);
        bf16x8 wf = lds_read16(wb);
        u32x4 y0, y1;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            bf16x8 wf_next = wf;
            if (nt + 1 < NT)
                wf_next = lds_read16(wb + (uint32_t)(nt + 1) * 16u * kWPitch);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xf[mt], acc[nt][mt], 0, 0, 0);
            // stage s + 1 of W: registers -> LDS, then stage s + 2 -> registers
            lds_write16(wd + (uint32_t)nt * 64u * kWPitch, wr[nt]);
            wr[nt] = w_load(nt, kbyte_stage2);
            // F on this stage's share of pair p + 1: words 8 Q' .. of the lane's 16 words
#pragma unroll
            for (int j = nt; j < 8; j += NT) {
                const uint32_t r = rational_pair<M, N>(xq[2 * Q + (j >> 2)][j & 3], c);
                if (j < 4)
                    y0[j] = r;
                else
                    y1[j - 4] = r;
            }
            wf = wf_next;
        }
        lds_write16(x_dst + xsel_write + (uint32_t)(2 * Q) * 16u, y0);
        lds_write16(x_dst + xsel_write + (uint32_t)(2 * Q + 1) * 16u, y1);
        xq[2 * Q] = gload16(x_base + kbyte_pair2, x_lane + (uint32_t)(2 * Q) * 16u);
        xq[2 * Q + 1] = gload16(x_base + kbyte_pair2, x_lane + (uint32_t)(2 * Q + 1) * 16u);
        __syncthreads();
    };

    uint32_t xsel = 0; // buffer the matrix products read
    for (int32_t p = 0; p < n_pairs; ++p) {
        const uint32_t s2 = (uint32_t)(2 * p + 2) * 64u; // byte offset of stage 2 p + 2
        const uint32_t s3 = s2 + 64u;
        const uint32_t p2 = (uint32_t)(p + 2) * 128u;
        const uint32_t kb2 = s2 < k_last_stage ? s2 : k_last_stage;
        const uint32_t kb3 = s3 < k_last_stage ? s3 : k_last_stage;
        const uint32_t kp2 = p2 < k_last_pair ? p2 : k_last_pair;
        stage(std::integral_constant<int, 0>{}, xsel, kXBuf - xsel, kb2, kp2);
        stage(std::integral_constant<int, 1>{}, xsel, kXBuf - xsel, kb3, kp2);
        // F of pair p + 2 (computed during pair p + 1) uses the group of that pair
        coef_for(kp2);
        xsel = kXBuf - xsel;
    }

    // ---- epilogue: lane holds channels n0 + wave WN + nt 16 + (lane / 16) 4 + 0..3 of token m0 + mt 16 + lane % 16
    const int32_t o_lane = n0 + wave * WN + (lane >> 4) * 4;
    constexpr int ES = (int)sizeof(OUT);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int32_t o = o_lane + nt * 16;
        if (NEDGE && o >= a.Nout)
            continue;
        f32x4 bv = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (a.bias)
            bv = *(const f32x4 *)(a.bias + o);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int64_t token = m0 + mt * 16 + (lane & 15);
            if (token < a.rows)
                OutPack<OUT>::store((gptr_t)(a.out + (token * a.Nout + o) * ES), acc[nt][mt] + bv);
        }
    }
}

// --------------------------------------------------------------------------
// host side
// --------------------------------------------------------------------------
using LinKernel = void (*)(const LinArgs);

template <typename OUT> static LinKernel select_kernel(int nt, bool nedge)
{
    switch (nt) {
    case 6: return grkan_linear_fwd_kernel<6, OUT, false, 5, 4>;
    case 3:
        return nedge ? grkan_linear_fwd_kernel<3, OUT, true, 5, 4> : grkan_linear_fwd_kernel<3, OUT, false, 5, 4>;
    }
    return nullptr;
}

static size_t lds_bytes(int nt) { return (size_t)2 * kXBuf + (size_t)2 * (64 * nt) * kWPitch; }

// The kernels use more LDS than the default limit for dynamic shared memory; raise it once per
// kernel and device.
static bool allow_lds(const void *kernel, size_t bytes)
{
    static std::mutex mu;
    static const void *done[64][16];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return false;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < 16; ++i) {
        if (done[dev][i] == kernel)
            return true;
        if (!done[dev][i]) {
            if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
                return false;
            done[dev][i] = kernel;
            return true;
        }
    }
    return false;
}

} // namespace lin
} // namespace grkan

using namespace grkan::lin;

extern "C" grkan_status_t grkan_linear_fwd(const void *x, const float *A, const float *B, const void *W,
                                           const float *bias, void *out,
                                           int64_t rows, int32_t D_in, int32_t D_out, int32_t G,
                                           int32_t m, int32_t n, grkan_dtype_t io, grkan_dtype_t out_dtype,
                                           void *hip_stream)
{
    if (io != GRKAN_BF16 || (out_dtype != GRKAN_BF16 && out_dtype != GRKAN_F32))
        return GRKAN_ERR_DTYPE;
    if (m != 5 || n != 4)
        return GRKAN_ERR_DEGREE;
    if (rows < 0 || D_in <= 0 || D_out <= 0 || G <= 0 || D_in % G != 0)
        return GRKAN_ERR_SHAPE;
    if (!A || !B || !W || (rows > 0 && (!x || !out)))
        return GRKAN_ERR_NULL;
    // 128-bit loads of x and W rows, 64/128-bit stores of four output channels, vector load of the bias
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(out) |
         reinterpret_cast<uintptr_t>(bias)) % 16 != 0 ||
        (reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) % 4 != 0)
        return GRKAN_ERR_ALIGN;
    const int32_t dg = D_in / G;
    // the contraction runs in pairs of 32-k stages with one coefficient group per stage and wave;
    // a lane stores four consecutive channels
    if (D_in % 64 != 0 || dg % 32 != 0 || D_out % 4 != 0)
        return GRKAN_ERR_UNSUPPORTED;
    if (rows > (INT64_MAX / 8) / (D_in > D_out ? D_in : D_out) || (int64_t)D_in * 2 * 128 >= ((int64_t)1 << 32))
        return GRKAN_ERR_UNSUPPORTED;
    if (rows == 0)
        return GRKAN_OK;

    const int nt = D_out % 384 == 0 ? 6 : 3;
    const int bn = 64 * nt;
    const bool nedge = D_out % bn != 0;
    const LinKernel kernel = out_dtype == GRKAN_BF16 ? select_kernel<bf16_out>(nt, nedge) : select_kernel<float>(nt, nedge);
    if (!kernel)
        return GRKAN_ERR_LAUNCH;
    const size_t lds = lds_bytes(nt);
    if (!allow_lds(reinterpret_cast<const void *>(kernel), lds))
        return GRKAN_ERR_LAUNCH;

    LinArgs a;
    a.x = static_cast<const char *>(x);
    a.W = static_cast<const char *>(W);
    a.bias = bias;
    a.out = static_cast<char *>(out);
    a.A = A;
    a.B = B;
    a.rows = rows;
    a.K = D_in;
    a.Nout = D_out;
    a.dgc = dg;
    const int64_t mblocks = (rows + kBM - 1) / kBM;
    const int64_t nblocks = (D_out + bn - 1) / bn;
    const int64_t grid = ((mblocks + 7) / 8) * 8 * nblocks;
    if (mblocks > INT32_MAX / 2 || grid > INT32_MAX)
        return GRKAN_ERR_UNSUPPORTED;
    a.mblocks = (int32_t)mblocks;
    a.nblocks = (int32_t)nblocks;
    void *args[] = {&a};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3((unsigned)grid), dim3(kThreads),
                                         args, lds, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? GRKAN_OK : GRKAN_ERR_LAUNCH;
}
