// GR-KAN group-wise rational function on gfx950 (MI355X): kernels and C ABI.
//
// The function and its gradients are those of the FlashKAT paper
// (Eq. "pade"; Eq. "grad_a", "grad_b", "grad_x", summed as in Eq. "accum" and
// "accum2").  The paper's own backward kernel (its Algorithm 2) accumulates the
// coefficient gradients per thread block and then issues one atomic add per
// block; here there are no atomics at all:
//
//   stage 1  Each lane streams 128-bit vectors of x and dy, writes dx, and
//            keeps the m + 1 + n partial sums (ten for the paper's degrees) in
//            registers for the whole kernel.
//            Group walk (long, line-aligned group segments): one wavefront =
//            one group, coefficients in scalar registers; the wavefront folds
//            its sums with DPP row/bank operations, the workgroup folds its
//            wavefronts through LDS.  Flat walk (short segments): wavefronts
//            read whole rows or column blocks of whole groups, each lane holds
//            the coefficients of its fixed column's group, and the workgroup
//            folds lanes -> runs -> groups through LDS.  Either way one row of m + 1 + n floats per (workgroup,
//            group) goes to a workspace.
//   stage 2  one wavefront per group adds that group's workspace rows in a
//            fixed order (in double) and overwrites dA / dB.
//
// Every order is fixed by the launch geometry, which is a pure function of
// shape, alignment and device, so dA / dB are bit-identical from run to run.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdlib>
#include <mutex>
#include <tuple>
#include <type_traits>
#include <vector>

#include "grkan_elem.h"
#include "grkan_plan.h"

namespace grkan {

// Eq. "grad_x", "grad_a", "grad_b" for one element; returns dx and adds this
// element's M + 1 + N terms to acc (acc[0..M] numerator, acc[M+1..M+N]
// denominator, the latter with the opposite sign until negate_b_sums is
// applied).  P/Q^2 is formed as (P r) r with r = 1/Q, so Q^2 is never computed.
template <bool WIDE, int M, int N>
__device__ __forceinline__ float bwd_elem(float x, float d, const Coef<M, N> &c, float (&acc)[M + 1 + N])
{
    // x^k: squares for even k, one more factor x for odd k
    constexpr int K = M > N ? M : N;
    float pw[K + 1];
    pw[0] = 1.0f;
    pw[1] = x;
#pragma unroll
    for (int k = 2; k <= K; ++k)
        pw[k] = (k % 2 == 0) ? pw[k / 2] * pw[k / 2] : pw[k - 1] * x;

    const float p = numerator_of(x, c);

    float dp = c.da[M];
#pragma unroll
    for (int i = M - 1; i >= 1; --i)
        dp = fmaf(dp, x, c.da[i]);

    const float aden = aden_of<WIDE>(x, c);

    float dh = c.db[N - 1];
#pragma unroll
    for (int j = N - 2; j >= 0; --j)
        dh = fmaf(dh, x, c.db[j]);

    const float q = 1.0f + fabsf(aden);
    const float r = __builtin_amdgcn_rcpf(q);

    const float t = d * r; // dy / Q
    acc[0] += t;
#pragma unroll
    for (int i = 1; i <= M; ++i)
        acc[i] = fmaf(t, pw[i], acc[i]);

    // s / Q with s = sign(Aden), sign(0) = 0: r > 0, so the sign is copied onto it bitwise
    const float sr = aden != 0.0f ? __builtin_copysignf(r, aden) : 0.0f;
    // acc[M+1..] collect +dy s P x^j / Q^2; the minus sign of Eq. "grad_b" is
    // applied once per lane after the loop (negate_b_sums)
    const float wb = t * (p * sr); // (dy / Q) (P s / Q) = dy s P / Q^2
#pragma unroll
    for (int j = 1; j <= N; ++j)
        acc[M + j] = fmaf(wb, pw[j], acc[M + j]);

    // dx = dy (P'/Q - s Aden' P/Q^2) = (dy/Q) P' - (dy s P/Q^2) Aden'
    const float dx = fmaf(t, dp, -(wb * dh));
    return dx;
}

// Global-memory (address space 1) byte pointers.  The loop-carried chunk base
// is wave-uniform; passing its two halves through readfirstlane keeps it in
// scalar registers, so that the memory instructions take the "scalar base +
// 32-bit lane offset" form and the vector ALU does no address arithmetic in the
// steady state.  The explicit address space keeps these global_* instructions
// (a pointer rebuilt from integers would otherwise be treated as generic).
typedef const __attribute__((address_space(1))) char *gcptr_t;
typedef __attribute__((address_space(1))) char *gptr_t;

// Marks a lane value as redefined at this point (no instruction is emitted).  Used on the 32-bit lane
// offset at the top of the streaming loops: its zero-extension then stays inside the loop body, where
// the address "scalar base + 32-bit lane offset" is recognised as such; hoisted out of the loop it would
// become a 64-bit lane value and every access would pay a 64-bit vector addition.
__device__ __forceinline__ void keep_in_loop(uint32_t &v) { asm volatile("" : "+v"(v)); }

// The instruction scheduler may not move anything across this point.  Placed after the prefetch loads:
// left alone, the scheduler sinks them into the arithmetic of the chunk before (dozens of instructions
// later), which shortens the time they have to arrive.
__device__ __forceinline__ void issue_before_what_follows() { __builtin_amdgcn_sched_barrier(0); }

__device__ __forceinline__ uint64_t uniform_u64(uint64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

template <int M, int N> __device__ __forceinline__ void negate_b_sums(float (&acc)[M + 1 + N])
{
#pragma unroll
    for (int k = M + 1; k < M + 1 + N; ++k)
        acc[k] = -acc[k];
}

// --------------------------------------------------------------------------
// vector memory access: VEC elements of IO per lane, one instruction
// --------------------------------------------------------------------------
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// tags of the two 16-bit I/O formats (the arithmetic is float32 for both)
struct bf16_t {
    uint16_t bits;
};
struct f16_t {
    uint16_t bits;
};

// two 16-bit elements of one 32-bit word -> float32 (element 0 in the low half)
template <typename IO> __device__ __forceinline__ void widen_pair(uint32_t w, float &lo, float &hi)
{
    if constexpr (std::is_same_v<IO, bf16_t>) {
        // bfloat16 -> float32 is a 16-bit shift
        lo = __builtin_bit_cast(float, w << 16);
        hi = __builtin_bit_cast(float, w & 0xffff0000u);
    } else {
        const f16x2 h = __builtin_bit_cast(f16x2, w);
        lo = (float)h[0];
        hi = (float)h[1];
        // keep the two conversions as instructions of their own: folded into mixed-precision FMAs
        // (one per use of x) they cost the backward kernel registers and time
        asm volatile("" : "+v"(lo), "+v"(hi));
    }
}

// two float32 -> one word of two 16-bit elements, round to nearest even
template <typename IO> __device__ __forceinline__ uint32_t narrow_pair(float lo, float hi)
{
    f32x2 f;
    f[0] = lo;
    f[1] = hi;
    if constexpr (std::is_same_v<IO, bf16_t>)
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
    else
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2));
}

template <typename IO> __device__ __forceinline__ float widen_one(uint16_t v)
{
    if constexpr (std::is_same_v<IO, bf16_t>)
        return __builtin_bit_cast(float, (uint32_t)v << 16);
    else
        return (float)__builtin_bit_cast(_Float16, v);
}

template <typename IO> __device__ __forceinline__ uint16_t narrow_one(float v)
{
    if constexpr (std::is_same_v<IO, bf16_t>)
        return __builtin_bit_cast(uint16_t, static_cast<__bf16>(v));
    else
        return __builtin_bit_cast(uint16_t, static_cast<_Float16>(v));
}

template <int BYTES> struct RawOf;
template <> struct RawOf<16> { using type = u32x4; };
template <> struct RawOf<8> { using type = u32x2; };
template <> struct RawOf<4> { using type = uint32_t; };
template <> struct RawOf<2> { using type = uint16_t; };

template <int BYTES> __device__ __forceinline__ uint32_t raw_word(const typename RawOf<BYTES>::type &r, int i)
{
    if constexpr (BYTES == 16 || BYTES == 8)
        return r[i];
    else
        return (uint32_t)r;
}

// A lane's vector as it sits in memory (raw bits), so that a prefetched vector
// can sit in registers untouched while the wave works on the current one:
// converting at load time would make the wave wait for the data immediately.
template <typename IO, int VEC> using RawT = typename RawOf<(int)sizeof(IO) * VEC>::type;

template <typename IO, int VEC> __device__ __forceinline__ RawT<IO, VEC> load_raw(gcptr_t p)
{
    using Raw = RawT<IO, VEC>;
    return __builtin_nontemporal_load((const __attribute__((address_space(1))) Raw *)p);
}

// Reads a loaded vector at this point (no instruction is emitted), so that the wait for its load is
// placed here and not at its first real use further down.
template <typename IO, int VEC> __device__ __forceinline__ void arrived(const RawT<IO, VEC> &r)
{
    const uint32_t w = raw_word<(int)sizeof(IO) * VEC>(r, 0);
    asm volatile("" : : "v"(w));
}

template <typename IO, int VEC> __device__ __forceinline__ void unpack(const RawT<IO, VEC> &r, float (&out)[VEC])
{
    constexpr int BYTES = (int)sizeof(IO) * VEC;
    if constexpr (sizeof(IO) == 4) {
#pragma unroll
        for (int i = 0; i < VEC; ++i)
            out[i] = __builtin_bit_cast(float, raw_word<BYTES>(r, i));
    } else if constexpr (VEC == 1) {
        out[0] = widen_one<IO>(r);
    } else {
        // two elements per 32-bit word
#pragma unroll
        for (int i = 0; i < VEC / 2; ++i)
            widen_pair<IO>(raw_word<BYTES>(r, i), out[2 * i], out[2 * i + 1]);
    }
}

template <typename IO, int VEC> __device__ __forceinline__ void load_vec(gcptr_t p, float (&out)[VEC])
{
    unpack<IO, VEC>(load_raw<IO, VEC>(p), out);
}

template <typename IO, int VEC> __device__ __forceinline__ void store_vec(gptr_t p, const float (&in)[VEC])
{
    constexpr int BYTES = (int)sizeof(IO) * VEC;
    using Raw = typename RawOf<BYTES>::type;
    Raw r;
    if constexpr (sizeof(IO) == 4) {
        if constexpr (VEC == 1) {
            r = __builtin_bit_cast(uint32_t, in[0]);
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                r[i] = __builtin_bit_cast(uint32_t, in[i]);
        }
    } else if constexpr (VEC == 1) {
        r = narrow_one<IO>(in[0]);
    } else {
#pragma unroll
        for (int i = 0; i < VEC / 2; ++i) {
            const uint32_t w = narrow_pair<IO>(in[2 * i], in[2 * i + 1]);
            if constexpr (VEC == 2)
                r = w;
            else
                r[i] = w;
        }
    }
    __builtin_nontemporal_store(r, (__attribute__((address_space(1))) Raw *)p);
}

// --------------------------------------------------------------------------
// wavefront sum with DPP: quad swaps, half-row and row mirrors, then the two
// row broadcasts; the total of all 64 lanes ends in lane 63.
// --------------------------------------------------------------------------
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp_get(float v)
{
    // lanes whose row is masked off receive 0
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false));
}

__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_get<0xB1, 0xf>(v);  // quad_perm [1,0,3,2]
    v += dpp_get<0x4E, 0xf>(v);  // quad_perm [2,3,0,1]
    v += dpp_get<0x141, 0xf>(v); // row_half_mirror
    v += dpp_get<0x140, 0xf>(v); // row_mirror: every lane of a row holds the row's sum
    v += dpp_get<0x142, 0xa>(v); // row_bcast:15 into rows 1 and 3
    v += dpp_get<0x143, 0xc>(v); // row_bcast:31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// --------------------------------------------------------------------------
// kernels
// --------------------------------------------------------------------------
struct FwdArgs {
    const char *x;
    char *y;
    const float *A;
    const float *B;
    int32_t dgc; // channels per coefficient group (walk.dg is the walk's: a whole row in the flat walk)
    Walk walk;
};

struct BwdArgs {
    const char *x;
    const char *dy;
    char *dx;
    const float *A;
    const float *B;
    float *partial; // [G][workspace rows per group][m + 1 + n]
    int32_t dgc;    // channels per coefficient group (walk.dg is the walk's: a whole row in the flat walk,
                    // a column block of the group when the plan splits groups)
    Walk walk;
};

// Forward.  In fixed-column mode a wave prefetches: the loads of its next chunk
// are issued before the arithmetic on the current one, so every resident wave
// always has one chunk of loads in flight.  The persistent grid is then sized
// so that the chip as a whole keeps about 4 MB of loads in flight (measured
// optimum of this memory system for a streaming read/write mix; both deeper
// per-wave prefetch and more resident waves were measured slower).
template <typename IO, int VEC, bool FIXED, bool LANECOEF, int M, int N>
__global__ __launch_bounds__(kThreadsPerWg) void grkan_fwd_kernel(const FwdArgs a)
{
    static_assert(FIXED || !LANECOEF, "per-lane coefficients need fixed columns");
    const Walk &p = a.walk;
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const WaveId id = wave_id(p, (int32_t)blockIdx.x, wv);
    // group walk: the coefficient group that holds the wave's column block (scalar registers; the
    // block is the group itself unless the plan splits groups); flat walk: the group of this lane's
    // fixed column inside the wave's block of whole groups (vector registers)
    int cg;
    if constexpr (LANECOEF)
        cg = (int)(((uint32_t)id.g * (uint32_t)p.dg + fixed_lane_col(p, id.w, lane).ccol * (uint32_t)p.vec) /
                   (uint32_t)a.dgc);
    else
        cg = p.dg == a.dgc ? id.g : (int)((uint32_t)id.g * (uint32_t)p.dg / (uint32_t)a.dgc);
    const Coef<M, N> c = load_coef<M, N>(a.A, a.B, cg);
    const int32_t n_it = full_visits(p, id.w);
    const bool tail = owns_tail(p, id.w) && lane < p.rem;
    constexpr int64_t ES = sizeof(IO);
    constexpr bool WIDE = sizeof(IO) == 4; // see aden_of
    const uint64_t x0 = reinterpret_cast<uint64_t>(a.x);
    const uint64_t y0 = reinterpret_cast<uint64_t>(a.y);

    auto one = [&](uint64_t off) {
        float xv[VEC], yv[VEC];
        load_vec<IO, VEC>((gcptr_t)(x0 + off), xv);
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            yv[e] = fwd_elem<WIDE, M, N>(xv[e], c);
        store_vec<IO, VEC>((gptr_t)(y0 + off), yv);
    };

    if constexpr (FIXED) {
        const uint64_t base0 = (uint64_t)(fixed_base0(p, id.g, id.w) * ES);
        const uint64_t step = (uint64_t)(fixed_step(p) * ES);
        uint32_t lo = fixed_lane_offset(p, id.w, lane) * (uint32_t)ES;
        // chunk `i` of this wave: scalar base + lane offset
        auto xin = [&](int32_t i) { return (gcptr_t)uniform_u64(x0 + base0 + (uint64_t)(uint32_t)i * step) + lo; };
        auto yout = [&](int32_t i) { return (gptr_t)uniform_u64(y0 + base0 + (uint64_t)(uint32_t)i * step) + lo; };

        // chunk i: raw bits in, results out
        auto work = [&](const RawT<IO, VEC> &rx, int32_t i) {
            float xs[VEC], yv[VEC];
            unpack<IO, VEC>(rx, xs);
#pragma unroll
            for (int e = 0; e < VEC; ++e)
                yv[e] = fwd_elem<WIDE, M, N>(xs[e], c);
            store_vec<IO, VEC>(yout(i), yv);
        };
        if (n_it > 0) {
            // Two register sets take turns, so nothing is copied from "next" to "current" and the loop
            // body has no conditional load.  Per half trip: issue the loads of the following chunk
            // (raw, untouched), work on the current one, then wait for those loads before issuing any
            // more - one chunk of loads in flight per wave, which is what the persistent grid is sized for.
            RawT<IO, VEC> ra = load_raw<IO, VEC>(xin(0));
            arrived<IO, VEC>(ra); // the loop is entered, like re-entered, with nothing to wait for
            int32_t it = 0;
            for (; it + 2 < n_it; it += 2) {
                keep_in_loop(lo);
                const RawT<IO, VEC> rb = load_raw<IO, VEC>(xin(it + 1));
                issue_before_what_follows();
                work(ra, it);
                arrived<IO, VEC>(rb);
                ra = load_raw<IO, VEC>(xin(it + 2));
                issue_before_what_follows();
                work(rb, it + 1);
                arrived<IO, VEC>(ra);
            }
            if (it + 1 < n_it) {
                const RawT<IO, VEC> rb = load_raw<IO, VEC>(xin(it + 1));
                issue_before_what_follows();
                work(ra, it);
                work(rb, it + 1);
            } else {
                work(ra, it);
            }
        }
        if (tail)
            one(base0 + (uint64_t)(uint32_t)n_it * step + lo);
    } else {
        LanePos s = lane_start(p, id.w, lane);
        for (int32_t it = 0; it < n_it; ++it) {
            one((uint64_t)(elem_offset(p, id.g, s) * ES));
            lane_advance(p, s);
        }
        if (tail)
            one((uint64_t)(elem_offset(p, id.g, s) * ES));
    }
}

// Backward, stage 1 (see the file header).
template <typename IO, int VEC, bool FIXED, bool LANECOEF, int M, int N>
__global__ __launch_bounds__(kThreadsPerWg) void grkan_bwd_stage1_kernel(const BwdArgs a)
{
    static_assert(FIXED || !LANECOEF, "per-lane coefficients need fixed columns");
    const Walk &p = a.walk;
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const WaveId id = wave_id(p, (int32_t)blockIdx.x, wv);
    int cg;
    if constexpr (LANECOEF)
        cg = (int)(((uint32_t)id.g * (uint32_t)p.dg + fixed_lane_col(p, id.w, lane).ccol * (uint32_t)p.vec) /
                   (uint32_t)a.dgc);
    else
        cg = p.dg == a.dgc ? id.g : (int)((uint32_t)id.g * (uint32_t)p.dg / (uint32_t)a.dgc);
    const Coef<M, N> c = load_coef<M, N>(a.A, a.B, cg);
    const int32_t n_it = full_visits(p, id.w);
    const bool tail = owns_tail(p, id.w) && lane < p.rem;
    constexpr int64_t ES = sizeof(IO);
    constexpr bool WIDE = sizeof(IO) == 4; // see aden_of
    const uint64_t x0 = reinterpret_cast<uint64_t>(a.x);
    const uint64_t dy0 = reinterpret_cast<uint64_t>(a.dy);
    const uint64_t dx0 = reinterpret_cast<uint64_t>(a.dx);

    constexpr int kNumCoef = M + 1 + N; // sums per group
    float acc[kNumCoef];
#pragma unroll
    for (int k = 0; k < kNumCoef; ++k)
        acc[k] = 0.0f;

    auto one = [&](uint64_t off) {
        float xv[VEC], dv[VEC], ov[VEC];
        load_vec<IO, VEC>((gcptr_t)(x0 + off), xv);
        load_vec<IO, VEC>((gcptr_t)(dy0 + off), dv);
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            ov[e] = bwd_elem<WIDE, M, N>(xv[e], dv[e], c, acc);
        store_vec<IO, VEC>((gptr_t)(dx0 + off), ov);
    };

    if constexpr (FIXED) {
        const uint64_t base0 = (uint64_t)(fixed_base0(p, id.g, id.w) * ES);
        const uint64_t step = (uint64_t)(fixed_step(p) * ES);
        uint32_t lo = fixed_lane_offset(p, id.w, lane) * (uint32_t)ES;
        // chunk `i` of this wave: scalar base + lane offset
        auto xin = [&](int32_t i) { return (gcptr_t)uniform_u64(x0 + base0 + (uint64_t)(uint32_t)i * step) + lo; };
        auto dyin = [&](int32_t i) { return (gcptr_t)uniform_u64(dy0 + base0 + (uint64_t)(uint32_t)i * step) + lo; };
        auto dxout = [&](int32_t i) { return (gptr_t)uniform_u64(dx0 + base0 + (uint64_t)(uint32_t)i * step) + lo; };

        // chunk i: raw bits in, dx out, sums updated
        auto work = [&](const RawT<IO, VEC> &rx, const RawT<IO, VEC> &rd, int32_t i) {
            float xs[VEC], ds[VEC], ov[VEC];
            unpack<IO, VEC>(rx, xs);
            unpack<IO, VEC>(rd, ds);
#pragma unroll
            for (int e = 0; e < VEC; ++e)
                ov[e] = bwd_elem<WIDE, M, N>(xs[e], ds[e], c, acc);
            store_vec<IO, VEC>(dxout(i), ov);
        };
        if (n_it > 0) {
            // Two register sets take turns, so nothing is copied from "next" to "current" and the loop
            // body has no conditional load.  Per half trip: issue the loads of the following chunk
            // (raw, untouched), work on the current one, then wait for those loads before issuing any
            // more - one chunk of loads in flight per wave, which is what the persistent grid is sized for.
            RawT<IO, VEC> xa = load_raw<IO, VEC>(xin(0));
            RawT<IO, VEC> da = load_raw<IO, VEC>(dyin(0));
            arrived<IO, VEC>(xa); // the loop is entered, like re-entered, with nothing to wait for
            arrived<IO, VEC>(da);
            int32_t it = 0;
            for (; it + 2 < n_it; it += 2) {
                keep_in_loop(lo);
                const RawT<IO, VEC> xb = load_raw<IO, VEC>(xin(it + 1));
                const RawT<IO, VEC> db = load_raw<IO, VEC>(dyin(it + 1));
                issue_before_what_follows();
                work(xa, da, it);
                arrived<IO, VEC>(xb);
                arrived<IO, VEC>(db);
                xa = load_raw<IO, VEC>(xin(it + 2));
                da = load_raw<IO, VEC>(dyin(it + 2));
                issue_before_what_follows();
                work(xb, db, it + 1);
                arrived<IO, VEC>(xa);
                arrived<IO, VEC>(da);
            }
            if (it + 1 < n_it) {
                const RawT<IO, VEC> xb = load_raw<IO, VEC>(xin(it + 1));
                const RawT<IO, VEC> db = load_raw<IO, VEC>(dyin(it + 1));
                issue_before_what_follows();
                work(xa, da, it);
                work(xb, db, it + 1);
            } else {
                work(xa, da, it);
            }
        }
        if (tail)
            one(base0 + (uint64_t)(uint32_t)n_it * step + lo);
    } else {
        LanePos s = lane_start(p, id.w, lane);
        for (int32_t it = 0; it < n_it; ++it) {
            one((uint64_t)(elem_offset(p, id.g, s) * ES));
            lane_advance(p, s);
        }
        if (tail)
            one((uint64_t)(elem_offset(p, id.g, s) * ES));
    }

    negate_b_sums<M, N>(acc);
    if constexpr (!LANECOEF) {
        // registers -> wavefront (DPP) -> workgroup (LDS) -> one workspace row per group
        __shared__ float wave_part[kWavesPerWg][kNumCoef];
#pragma unroll
        for (int k = 0; k < kNumCoef; ++k) {
            const float s = wave_sum(acc[k]);
            if (lane == 0)
                wave_part[wv][k] = s;
        }
        __syncthreads();
        const int tid = threadIdx.x;
        if (tid < p.k * kNumCoef) {
            const int gl = tid / kNumCoef;
            const int kc = tid - gl * kNumCoef;
            // waves gl, gl + k, gl + 2k, ... of this workgroup hold group (bundle * k + gl)
            float s = 0.0f;
            for (int sub = 0; sub < p.ns; ++sub)
                s += wave_part[sub * p.k + gl][kc];
            const int32_t bundle = (int32_t)blockIdx.x % p.nb;
            const int32_t wgi = (int32_t)blockIdx.x / p.nb;
            const int64_t g = (int64_t)bundle * p.k + gl;
            a.partial[(g * p.wg_per_bundle + wgi) * kNumCoef + kc] = s;
        }
    } else {
        // Flat walk: the 256 lanes of the workgroup hold consecutive vectors of
        // the rows of its column block, so lanes of one coefficient group form
        // runs of vt = d_g / vec lanes (a group can own several runs when the
        // block's row is shorter than the workgroup).  registers -> LDS -> one sum
        // per run (fixed lane order) -> one sum per group (fixed run order) -> one
        // workspace row per workgroup for every group of the block, zeros
        // included, so that stage 2 needs no map of who wrote what.
        __shared__ float lane_part[kNumCoef][kThreadsPerWg];
        __shared__ float run_part[kThreadsPerWg + 1][kNumCoef];
        const int tid = threadIdx.x;
#pragma unroll
        for (int k = 0; k < kNumCoef; ++k)
            lane_part[k][tid] = acc[k];
        __syncthreads();
        const uint32_t vt = (uint32_t)a.dgc / (uint32_t)p.vec; // lanes per run
        const uint32_t V = (uint32_t)p.v;                       // vectors per row of the walk's column block
        const uint32_t Gb = (uint32_t)p.dg / (uint32_t)a.dgc;   // coefficient groups per column block
        const uint32_t c0 = ((uint32_t)id.wg_index * kThreadsPerWg) % V; // column of lane 0
        const uint32_t u0 = c0 / vt;                            // first (unwrapped) run
        const uint32_t n_runs = (c0 + kThreadsPerWg - 1) / vt - u0 + 1;
        for (uint32_t item = tid; item < n_runs * kNumCoef; item += kThreadsPerWg) {
            const uint32_t r = item / kNumCoef, k = item - r * kNumCoef;
            const uint32_t first = (u0 + r) * vt; // unwrapped column where run r starts
            const uint32_t lo = first > c0 ? first - c0 : 0;
            const uint32_t hi = first + vt - c0 < (uint32_t)kThreadsPerWg ? first + vt - c0 : (uint32_t)kThreadsPerWg;
            float s = 0.0f;
            for (uint32_t l = lo; l < hi; ++l)
                s += lane_part[k][l];
            run_part[r][k] = s;
        }
        __syncthreads();
        for (uint32_t item = tid; item < Gb * kNumCoef; item += kThreadsPerWg) {
            const uint32_t g = item / kNumCoef, k = item - g * kNumCoef;
            // run r belongs to group (u0 + r) mod Gb of this block
            float s = 0.0f;
            for (uint32_t r = (g + Gb - u0 % Gb) % Gb; r < n_runs; r += Gb)
                s += run_part[r][k];
            const int64_t gg = (int64_t)id.g * Gb + g; // the group's index in A, B and the workspace
            a.partial[(gg * p.wg_per_bundle + id.wg_index) * kNumCoef + k] = s;
        }
    }
}

// Stage 2.  One workgroup per group, of one wavefront when the group has at
// most 64 workspace rows and of four otherwise (the flat walk leaves one row
// per stage-1 workgroup; reading hundreds of rows with 64 lanes is a chain of
// dependent memory latencies).  Thread t adds rows t, t + T, ... in double; the
// T thread sums go through LDS, each block of 64 of them is added in thread
// order, then the blocks in block order.  Every order is fixed by T and the row
// count; dA / dB are overwritten.
constexpr int kStage2MaxThreads = 4 * kWave;

static int stage2_threads(int32_t rows_per_group) { return rows_per_group > kWave ? kStage2MaxThreads : kWave; }

template <int M, int N>
__global__ __launch_bounds__(kStage2MaxThreads) void grkan_bwd_stage2_kernel(const float *__restrict__ partial,
                                                                             int32_t rows_per_group,
                                                                             float *__restrict__ dA,
                                                                             float *__restrict__ dB)
{
    constexpr int kNumCoef = M + 1 + N;
    constexpr int kBlocks = kStage2MaxThreads / kWave;
    __shared__ double thread_sum[kNumCoef][kStage2MaxThreads];
    __shared__ double block_sum[kNumCoef][kBlocks];
    const int g = blockIdx.x;
    const int tid = threadIdx.x;
    const int T = blockDim.x; // 64 or 256
    const float *base = partial + (size_t)g * rows_per_group * kNumCoef;

    double s[kNumCoef];
#pragma unroll
    for (int k = 0; k < kNumCoef; ++k)
        s[k] = 0.0;
    for (int r = tid; r < rows_per_group; r += T) {
#pragma unroll
        for (int k = 0; k < kNumCoef; ++k)
            s[k] += (double)base[(size_t)r * kNumCoef + k];
    }
#pragma unroll
    for (int k = 0; k < kNumCoef; ++k)
        thread_sum[k][tid] = s[k];
    __syncthreads();
    const int nblocks = T / kWave;
    if (tid < kNumCoef * nblocks) {
        const int k = tid / nblocks, b = tid - k * nblocks;
        double t = 0.0;
        for (int l = 0; l < kWave; ++l)
            t += thread_sum[k][b * kWave + l];
        block_sum[k][b] = t;
    }
    __syncthreads();
    if (tid < kNumCoef) {
        double t = 0.0;
        for (int b = 0; b < nblocks; ++b)
            t += block_sum[tid][b];
        if (tid <= M)
            dA[g * (M + 1) + tid] = (float)t;
        else
            dB[g * N + (tid - (M + 1))] = (float)t;
    }
}

// --------------------------------------------------------------------------
// host side
// --------------------------------------------------------------------------
struct DeviceInfo {
    bool ready = false;
    int num_cu = 0;
};

static std::mutex g_mu;
static DeviceInfo g_dev[64];

static bool device_info(int *dev_out, DeviceInfo *out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return false;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_dev[dev].ready) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            return false;
        g_dev[dev].num_cu = n;
        g_dev[dev].ready = true;
    }
    *dev_out = dev;
    *out = g_dev[dev];
    return true;
}

// Experiment overrides of the persistent grid sizes (workgroups per compute
// unit; 0 = the built-in choice).  The two environment variables are read once,
// when the library is loaded; grkan_tuning_override replaces them at run time.
static int env_int(const char *name)
{
    const char *s = std::getenv(name);
    if (!s || !*s)
        return 0;
    const int v = std::atoi(s);
    return v > 0 ? v : 0;
}

static std::atomic<int> g_fwd_wg_per_cu{env_int("GRKAN_FWD_WG_PER_CU")};
static std::atomic<int> g_bwd_wg_per_cu{env_int("GRKAN_BWD_WG_PER_CU")};

static int32_t common_alignment(std::initializer_list<const void *> ptrs)
{
    uintptr_t bits = 16;
    for (const void *q : ptrs)
        bits |= reinterpret_cast<uintptr_t>(q);
    return (int32_t)(bits & (~bits + 1)); // lowest set bit, at most 16
}

// Kernel selection: the variant for (degrees, dtype, vector width, walk mode)
// as a plain function pointer, so that one code path can both query its
// occupancy and launch it.
using FwdKernel = void (*)(const FwdArgs);
using BwdKernel = void (*)(const BwdArgs);
using Stage2Kernel = void (*)(const float *, int32_t, float *, float *);

template <typename IO, int VEC, int M, int N> static FwdKernel fwd_variant(bool fixed, bool lane_coef)
{
    if (lane_coef)
        return grkan_fwd_kernel<IO, VEC, true, true, M, N>;
    return fixed ? grkan_fwd_kernel<IO, VEC, true, false, M, N> : grkan_fwd_kernel<IO, VEC, false, false, M, N>;
}
template <typename IO, int VEC, int M, int N> static BwdKernel bwd_variant(bool fixed, bool lane_coef)
{
    if (lane_coef)
        return grkan_bwd_stage1_kernel<IO, VEC, true, true, M, N>;
    return fixed ? grkan_bwd_stage1_kernel<IO, VEC, true, false, M, N>
                 : grkan_bwd_stage1_kernel<IO, VEC, false, false, M, N>;
}

template <int M, int N> static FwdKernel select_fwd(grkan_dtype_t io, int vec, bool fixed, bool lane_coef)
{
    switch (io) {
    case GRKAN_F32:
        switch (vec) {
        case 4: return fwd_variant<float, 4, M, N>(fixed, lane_coef);
        case 2: return fwd_variant<float, 2, M, N>(fixed, lane_coef);
        case 1: return fwd_variant<float, 1, M, N>(fixed, lane_coef);
        }
        break;
    case GRKAN_BF16:
        switch (vec) {
        case 8: return fwd_variant<bf16_t, 8, M, N>(fixed, lane_coef);
        case 4: return fwd_variant<bf16_t, 4, M, N>(fixed, lane_coef);
        case 2: return fwd_variant<bf16_t, 2, M, N>(fixed, lane_coef);
        case 1: return fwd_variant<bf16_t, 1, M, N>(fixed, lane_coef);
        }
        break;
    case GRKAN_F16:
        switch (vec) {
        case 8: return fwd_variant<f16_t, 8, M, N>(fixed, lane_coef);
        case 4: return fwd_variant<f16_t, 4, M, N>(fixed, lane_coef);
        case 2: return fwd_variant<f16_t, 2, M, N>(fixed, lane_coef);
        case 1: return fwd_variant<f16_t, 1, M, N>(fixed, lane_coef);
        }
        break;
    }
    return nullptr;
}

template <int M, int N> static BwdKernel select_bwd(grkan_dtype_t io, int vec, bool fixed, bool lane_coef)
{
    switch (io) {
    case GRKAN_F32:
        switch (vec) {
        case 4: return bwd_variant<float, 4, M, N>(fixed, lane_coef);
        case 2: return bwd_variant<float, 2, M, N>(fixed, lane_coef);
        case 1: return bwd_variant<float, 1, M, N>(fixed, lane_coef);
        }
        break;
    case GRKAN_BF16:
        switch (vec) {
        case 8: return bwd_variant<bf16_t, 8, M, N>(fixed, lane_coef);
        case 4: return bwd_variant<bf16_t, 4, M, N>(fixed, lane_coef);
        case 2: return bwd_variant<bf16_t, 2, M, N>(fixed, lane_coef);
        case 1: return bwd_variant<bf16_t, 1, M, N>(fixed, lane_coef);
        }
        break;
    case GRKAN_F16:
        switch (vec) {
        case 8: return bwd_variant<f16_t, 8, M, N>(fixed, lane_coef);
        case 4: return bwd_variant<f16_t, 4, M, N>(fixed, lane_coef);
        case 2: return bwd_variant<f16_t, 2, M, N>(fixed, lane_coef);
        case 1: return bwd_variant<f16_t, 1, M, N>(fixed, lane_coef);
        }
        break;
    }
    return nullptr;
}

// The degrees the library is built for.  (5, 4) is the paper's; (3, 2) and
// (7, 6) are the neighbouring "numerator one degree above the denominator"
// units of the same family.
struct DegreeOps {
    int m, n;
    FwdKernel (*fwd)(grkan_dtype_t, int, bool, bool);
    BwdKernel (*bwd)(grkan_dtype_t, int, bool, bool);
    Stage2Kernel stage2;
};

template <int M, int N> static constexpr DegreeOps degree_entry()
{
    static_assert(M + 1 + N <= kMaxCoef, "workspace rows are sized for kMaxCoef sums");
    return DegreeOps{M, N, select_fwd<M, N>, select_bwd<M, N>, grkan_bwd_stage2_kernel<M, N>};
}

static const DegreeOps kDegrees[] = {degree_entry<5, 4>(), degree_entry<3, 2>(), degree_entry<7, 6>()};

static const DegreeOps *degree_ops(int m, int n)
{
    for (const DegreeOps &d : kDegrees)
        if (d.m == m && d.n == n)
            return &d;
    return nullptr;
}

// Workgroups of a kernel that fit on one compute unit at once (cached per
// kernel and device).  A persistent grid larger than that would leave
// workgroups queued behind the resident ones.
static int resident_wg_per_cu(const void *kernel, int dev)
{
    static std::mutex mu;
    static std::vector<std::tuple<const void *, int, int>> cache;
    std::lock_guard<std::mutex> lock(mu);
    for (const auto &e : cache)
        if (std::get<0>(e) == kernel && std::get<1>(e) == dev)
            return std::get<2>(e);
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, kThreadsPerWg, 0) != hipSuccess || n <= 0)
        return 0;
    cache.emplace_back(kernel, dev, n);
    return n;
}

// Workgroups (of 4 waves) per compute unit the persistent grids are sized for.
// With one chunk of loads in flight per wave (1 KB forward, 2 KB backward),
// 4 and 2 workgroups per unit put about 4 MB of loads in flight on 256 units,
// which is where the HBM-bound kernels were measured fastest (a backward pass
// that sweeps whole rows as one stream - no column blocks - measured best at 3).  The bfloat16 backward pass moves half the
// bytes for the same arithmetic and is bound by the vector ALU instead: it
// takes every wave slot it can get (requests are clamped to the kernel's real
// occupancy).  The overrides above apply to both walks.
struct Want {
    int group_walk;
    int flat_walk;
};

static Want fwd_want(grkan_dtype_t)
{
    const int e = g_fwd_wg_per_cu.load(std::memory_order_relaxed);
    return e ? Want{e, e} : Want{4, 4};
}

static Want bwd_want(grkan_dtype_t io)
{
    const int e = g_bwd_wg_per_cu.load(std::memory_order_relaxed);
    if (e)
        return Want{e, e};
    return io == GRKAN_F32 ? Want{2, 3} : Want{8, 8}; // both 16-bit formats are ALU-bound
}

// Plans the launch with the wanted workgroups per unit, then clamps to what
// the selected kernel can keep resident and re-plans if needed.
template <typename Select>
static grkan_status_t plan_resident(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io, int32_t align,
                                    const DeviceInfo &info, int dev, Want want, bool forward, Select select,
                                    grkan_plan_t *pl, Walk *walk, const void **kernel)
{
    int per_cu = want.group_walk;
    grkan_status_t st = make_plan(rows, D, G, io, align, info.num_cu, per_cu, forward, pl, walk);
    if (st != GRKAN_OK)
        return st;
    // one sweep over whole rows (flat walk without column blocks, or a single unsplit group) against
    // several interleaved column streams: the two were measured best at different grid sizes
    const bool rows_walk = (pl->lane_coef ? pl->column_split : G * pl->column_split) == 1;
    if (rows_walk && want.flat_walk != per_cu) {
        grkan_plan_t alt;
        if (make_plan(rows, D, G, io, align, info.num_cu, want.flat_walk, forward, &alt, nullptr) == GRKAN_OK &&
            alt.lane_coef == pl->lane_coef) {
            per_cu = want.flat_walk;
            st = make_plan(rows, D, G, io, align, info.num_cu, per_cu, forward, pl, walk);
            if (st != GRKAN_OK)
                return st;
        }
    }
    *kernel = reinterpret_cast<const void *>(select(io, pl->vec, pl->fixed_col != 0, pl->lane_coef != 0));
    if (!*kernel)
        return GRKAN_ERR_LAUNCH;
    const int fit = resident_wg_per_cu(*kernel, dev);
    if (fit <= 0)
        return GRKAN_ERR_LAUNCH;
    if (fit < per_cu) {
        const int32_t was_flat = pl->lane_coef;
        st = make_plan(rows, D, G, io, align, info.num_cu, fit, forward, pl, walk);
        if (st != GRKAN_OK)
            return st;
        *kernel = reinterpret_cast<const void *>(select(io, pl->vec, pl->fixed_col != 0, pl->lane_coef != 0));
        if (!*kernel || (pl->lane_coef != was_flat && resident_wg_per_cu(*kernel, dev) <= 0))
            return GRKAN_ERR_LAUNCH;
    }
    return GRKAN_OK;
}

static grkan_status_t check_common(int64_t rows, int32_t D, int32_t G, int32_t m, int32_t n, grkan_dtype_t io,
                                   const DegreeOps **ops)
{
    *ops = degree_ops(m, n);
    if (!*ops)
        return GRKAN_ERR_DEGREE;
    return check_shape(rows, D, G, io);
}

// rows of `coefs` floats, one per (group, workgroup that holds a part of it)
static size_t workspace_for(const grkan_plan_t &pl, int32_t G, int coefs)
{
    return (size_t)G * (size_t)pl.partials_per_group * (size_t)coefs * sizeof(float);
}

} // namespace grkan

using namespace grkan;

extern "C" size_t grkan_bwd_workspace_bytes(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io)
{
    if (check_shape(rows, D, G, io) != GRKAN_OK)
        return 0;
    int dev;
    DeviceInfo info;
    if (!device_info(&dev, &info))
        return 0;
    size_t need = 16; // never zero, so that callers can always allocate it
    // the query names no degrees: the bound covers every built (m, n), whose kernels differ in occupancy
    for (const DegreeOps &ops : kDegrees) {
        for (int align = elem_size(io); align <= 16; align *= 2) {
            grkan_plan_t pl;
            const void *kernel = nullptr;
            if (plan_resident(rows, D, G, io, align, info, dev, bwd_want(io), false, ops.bwd, &pl, nullptr, &kernel) !=
                GRKAN_OK)
                return 0;
            const size_t b = workspace_for(pl, G, ops.m + 1 + ops.n);
            need = b > need ? b : need;
        }
    }
    return need;
}

extern "C" void grkan_tuning_override(int32_t fwd_wg_per_cu, int32_t bwd_wg_per_cu)
{
    g_fwd_wg_per_cu.store(fwd_wg_per_cu > 0 ? fwd_wg_per_cu : 0, std::memory_order_relaxed);
    g_bwd_wg_per_cu.store(bwd_wg_per_cu > 0 ? bwd_wg_per_cu : 0, std::memory_order_relaxed);
}

extern "C" grkan_status_t grkan_device_query(int32_t *out)
{
    if (!out)
        return GRKAN_ERR_NULL;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess)
        return GRKAN_ERR_LAUNCH;
    const hipDeviceAttribute_t what[4] = {hipDeviceAttributeMultiprocessorCount, hipDeviceAttributeClockRate,
                                          hipDeviceAttributeMemoryClockRate, hipDeviceAttributeMemoryBusWidth};
    for (int i = 0; i < 4; ++i) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, what[i], dev) != hipSuccess)
            return GRKAN_ERR_LAUNCH;
        out[i] = v;
    }
    return GRKAN_OK;
}

extern "C" grkan_status_t grkan_fwd(const void *x, const float *A, const float *B, void *y,
                                    int64_t rows, int32_t D, int32_t G, int32_t m, int32_t n,
                                    grkan_dtype_t io, void *hip_stream)
{
    const DegreeOps *ops = nullptr;
    grkan_status_t st = check_common(rows, D, G, m, n, io, &ops);
    if (st != GRKAN_OK)
        return st;
    if (!A || !B || (rows > 0 && (!x || !y)))
        return GRKAN_ERR_NULL;
    const int es = elem_size(io);
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y)) % es != 0 ||
        (reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) % 4 != 0)
        return GRKAN_ERR_ALIGN;
    if (rows == 0)
        return GRKAN_OK;

    int dev;
    DeviceInfo info;
    if (!device_info(&dev, &info))
        return GRKAN_ERR_LAUNCH;
    grkan_plan_t pl;
    FwdArgs a;
    const void *kernel = nullptr;
    st = plan_resident(rows, D, G, io, common_alignment({x, y}), info, dev, fwd_want(io), true, ops->fwd, &pl,
                       &a.walk, &kernel);
    if (st != GRKAN_OK)
        return st;
    a.x = static_cast<const char *>(x);
    a.y = static_cast<char *>(y);
    a.A = A;
    a.B = B;
    a.dgc = D / G;
    void *args[] = {&a};
    const hipError_t e = hipLaunchKernel(kernel, dim3(pl.grid), dim3(kThreadsPerWg), args, 0,
                                         static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? GRKAN_OK : GRKAN_ERR_LAUNCH;
}

namespace grkan {

// Scratch of the allocation-free entry point: the workspace rows of stage 1,
// in a fixed array in device memory (one copy per GPU the library runs on, held
// until the process ends).  In host code the array's name is only a handle for
// the symbol; its address on a device comes from hipGetSymbolAddress, once per
// device, and only that pointer is ever handed to a kernel.
constexpr size_t kScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

static std::mutex g_scratch_mu;
static void *g_scratch_ptr[64]; // per device, filled on the first call there

// `dev` must be the current device.
static grkan_status_t scratch_of_device(int dev, void **out)
{
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr)
            return GRKAN_ERR_LAUNCH;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return GRKAN_OK;
}

// Both backward entry points.  own_scratch: the workspace is the library's
// fixed array (then `workspace` / `workspace_bytes` are ignored).
static grkan_status_t bwd_impl(const void *x, const void *dy, const float *A, const float *B,
                               void *dx, float *dA, float *dB,
                               void *workspace, size_t workspace_bytes, bool own_scratch,
                               int64_t rows, int32_t D, int32_t G, int32_t m, int32_t n,
                               grkan_dtype_t io, void *hip_stream)
{
    const DegreeOps *ops = nullptr;
    grkan_status_t st = check_common(rows, D, G, m, n, io, &ops);
    if (st != GRKAN_OK)
        return st;
    if (!A || !B || !dA || !dB || (rows > 0 && (!x || !dy || !dx)))
        return GRKAN_ERR_NULL;
    const int es = elem_size(io);
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(dy) | reinterpret_cast<uintptr_t>(dx)) % es != 0 ||
        (reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B) | reinterpret_cast<uintptr_t>(dA) |
         reinterpret_cast<uintptr_t>(dB)) % 4 != 0)
        return GRKAN_ERR_ALIGN;

    int dev;
    DeviceInfo info;
    if (!device_info(&dev, &info))
        return GRKAN_ERR_LAUNCH;
    grkan_plan_t pl;
    BwdArgs a;
    const void *kernel = nullptr;
    st = plan_resident(rows, D, G, io, common_alignment({x, dy, dx}), info, dev, bwd_want(io), false, ops->bwd, &pl,
                       &a.walk, &kernel);
    if (st != GRKAN_OK)
        return st;
    const size_t need = workspace_for(pl, G, m + 1 + n);
    if (own_scratch) {
        if (need > kScratchBytes)
            return GRKAN_ERR_SCRATCH_LIMIT;
        st = scratch_of_device(dev, &workspace);
        if (st != GRKAN_OK)
            return st;
    } else if (need > 0 &&
               (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 16 != 0)) {
        return GRKAN_ERR_WORKSPACE;
    }

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    a.x = static_cast<const char *>(x);
    a.dy = static_cast<const char *>(dy);
    a.dx = static_cast<char *>(dx);
    a.A = A;
    a.B = B;
    a.partial = static_cast<float *>(workspace);
    a.dgc = D / G;
    if (pl.grid > 0) {
        void *args[] = {&a};
        if (hipLaunchKernel(kernel, dim3(pl.grid), dim3(kThreadsPerWg), args, 0, stream) != hipSuccess)
            return GRKAN_ERR_LAUNCH;
    }
    // Stage 1 writes every workspace row stage 2 reads (one per workgroup and group, zeros included),
    // so nothing has to be cleared beforehand; with no rows there are no workspace rows and stage 2
    // writes zeros.
    const float *partial = a.partial;
    int32_t rows_per_group = pl.partials_per_group;
    void *args2[] = {&partial, &rows_per_group, &dA, &dB};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(ops->stage2), dim3(G),
                                         dim3(stage2_threads(rows_per_group)), args2, 0, stream);
    return e == hipSuccess ? GRKAN_OK : GRKAN_ERR_LAUNCH;
}

} // namespace grkan

extern "C" grkan_status_t grkan_bwd(const void *x, const void *dy, const float *A, const float *B,
                                    void *dx, float *dA, float *dB,
                                    void *workspace, size_t workspace_bytes,
                                    int64_t rows, int32_t D, int32_t G, int32_t m, int32_t n,
                                    grkan_dtype_t io, void *hip_stream)
{
    return bwd_impl(x, dy, A, B, dx, dA, dB, workspace, workspace_bytes, false, rows, D, G, m, n, io, hip_stream);
}

extern "C" grkan_status_t grkan_bwd_noalloc(const void *x, const void *dy, const float *A, const float *B,
                                            void *dx, float *dA, float *dB,
                                            int64_t rows, int32_t D, int32_t G, int32_t m, int32_t n,
                                            grkan_dtype_t io, void *hip_stream)
{
    return bwd_impl(x, dy, A, B, dx, dA, dB, nullptr, 0, true, rows, D, G, m, n, io, hip_stream);
}
