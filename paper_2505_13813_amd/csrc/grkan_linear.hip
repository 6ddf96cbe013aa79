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
// Geometry:
//   * a workgroup of NW wavefronts (8: two per SIMD, or 4) owns a tile of BM = 112
//     tokens x BN = 16 NW NT output channels (768 for the wide variant) and sweeps
//     the whole contraction dimension K = D_in; one workgroup per compute unit;
//   * wavefront w owns the 16 NT channels [16 NT w, 16 NT (w + 1)) of the tile for
//     all BM tokens: 7 x NT accumulators of v_mfma_f32_16x16x32_bf16, the
//     weights as the row operand, F(x) as the column operand, so that a lane
//     ends up with four consecutive output channels of one token;
//   * W streams through LDS in stages of 32 k (64 bytes per row) by LDS-direct
//     loads, two buffers; every wave fetches exactly the rows it multiplies, so the
//     weights need no barrier, only the wave's own load counter; rows are 64 bytes
//     apart, unpadded, with the 16-byte pieces of a row permuted so that an operand
//     read (16 rows at one piece index) hits 16 different bank groups;
//   * x goes memory -> registers -> F -> LDS in pairs of stages (64 k = one
//     128-byte line per token): F of the next pair is computed, in pieces placed
//     between the matrix instructions, while the matrix cores work on the current
//     one; one barrier per pair; rows padded by 16 bytes;
//   * the coefficient group of a wave's share of a pair is wave-uniform (d_g is a
//     multiple of 32), so the coefficients live in scalar registers;
//   * the output tile leaves through LDS in whole rows (bias added, rounded).
//
// The tile is wide in the channel direction on purpose: every token-operand
// element costs about 13 vector instructions (F) once per workgroup that
// consumes it, and on this chip only about two vector instructions per matrix
// instruction issue for free in its shadow (measured: each further one costs the
// SIMD about 5 clocks).  At BN = 768 there are 2.1 per matrix instruction from F
// alone; a narrower tile would be bound by the vector ALU, not the matrix cores.
#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>

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

constexpr int kMT = 7;                 // 16-token sub-tiles per workgroup: BM = 112
constexpr int kBM = 16 * kMT;
constexpr int kXRows = 128;            // rows of an x buffer (all 128 loader lanes write; BM are read)
constexpr int kXPitch = 144;           // 64 k (128 B) + 16 B pad
constexpr int kWRow = 64;              // 32 k per row of a W buffer, no padding (pieces permuted instead)
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
    int32_t wtiles;    // packed W only: 16-row tiles per stage, nblocks * BN / 16
};

__device__ __forceinline__ uint64_t uniform_u64(uint64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// 16 bytes from "wave-uniform base + 32-bit lane offset" (the form the memory instructions take a
// scalar base register pair for)
__device__ __forceinline__ u32x4 gload16(uint64_t uniform_base, uint32_t lane_off)
{
    return *(const __attribute__((address_space(1))) u32x4 *)((gcptr_t)uniform_base + lane_off);
}

// Marks a lane value as redefined here (no instruction): its zero-extension to 64 bits then stays
// next to the access that uses it, where "scalar base + 32-bit lane offset" is recognised; hoisted
// out of the loop it would turn every access into a 64-bit vector addition.
__device__ __forceinline__ void keep_in_loop(uint32_t &v) { asm volatile("" : "+v"(v)); }

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

// One matrix instruction, D = A B + D with D a 16 x 16 float32 tile (4 registers per lane), A the
// weights (16 channels x 32 k), B the token operand (32 k x 16 tokens).  Written as inline assembly
// so that the accumulators are pinned to the accumulation registers (AGPR = true) or to ordinary
// vector registers (the tiles that do not fit the 256 accumulation registers): left to the register
// allocator, a kernel that needs more than 256 registers shuffles hundreds of values between the
// two files per stage.
template <bool AGPR> __device__ __forceinline__ void mfma_16x16x32(f32x4 &acc, const bf16x8 &a, const bf16x8 &b)
{
    if constexpr (AGPR)
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
    else
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}

// Waits until at most N of this wave's vector-memory loads (LDS-direct ones included) are in flight.
template <int N> __device__ __forceinline__ void wait_loads()
{
    static_assert(N >= 0 && N < 64, "the counter has six bits");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Nothing may be moved across this point by the instruction scheduler.
__device__ __forceinline__ void fence_schedule() { __builtin_amdgcn_sched_barrier(0); }

template <int I, int N, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// F of the two bfloat16 of one word, cut into seven pieces of about four vector instructions, one
// to follow each matrix instruction of a 7-tile step: the matrix core works for 16 cycles per
// instruction, in whose shadow the same wavefront can issue three to four other instructions.
struct PairState {
    float x0, x1, p0, p1, h0, h1;
};

template <int S> __device__ __forceinline__ void rational_piece(PairState &t, uint32_t w, const Coef<5, 4> &c, uint32_t &out)
{
    if constexpr (S == 0) {
        t.x0 = __builtin_bit_cast(float, w << 16);
        t.x1 = __builtin_bit_cast(float, w & 0xffff0000u);
        t.p0 = fmaf(c.a[5], t.x0, c.a[4]);
        t.p1 = fmaf(c.a[5], t.x1, c.a[4]);
    } else if constexpr (S == 1) {
        t.p0 = fmaf(t.p0, t.x0, c.a[3]);
        t.p1 = fmaf(t.p1, t.x1, c.a[3]);
        t.h0 = fmaf(c.b[3], t.x0, c.b[2]);
        t.h1 = fmaf(c.b[3], t.x1, c.b[2]);
    } else if constexpr (S == 2) {
        t.p0 = fmaf(t.p0, t.x0, c.a[2]);
        t.p1 = fmaf(t.p1, t.x1, c.a[2]);
        t.h0 = fmaf(t.h0, t.x0, c.b[1]);
        t.h1 = fmaf(t.h1, t.x1, c.b[1]);
    } else if constexpr (S == 3) {
        t.p0 = fmaf(t.p0, t.x0, c.a[1]);
        t.p1 = fmaf(t.p1, t.x1, c.a[1]);
        t.h0 = fmaf(t.h0, t.x0, c.b[0]);
        t.h1 = fmaf(t.h1, t.x1, c.b[0]);
    } else if constexpr (S == 4) {
        t.p0 = fmaf(t.p0, t.x0, c.a[0]);
        t.p1 = fmaf(t.p1, t.x1, c.a[0]);
        t.h0 = fmaf(fabsf(t.h0), fabsf(t.x0), 1.0f); // Q = 1 + |x h| (as q_of<false>)
        t.h1 = fmaf(fabsf(t.h1), fabsf(t.x1), 1.0f);
    } else if constexpr (S == 5) {
        t.h0 = __builtin_amdgcn_rcpf(t.h0);
        t.h1 = __builtin_amdgcn_rcpf(t.h1);
    } else {
        f32x2 y;
        y[0] = t.p0 * t.h0;
        y[1] = t.p1 * t.h1;
        out = __builtin_bit_cast(uint32_t, __builtin_convertvector(y, bf16x2));
    }
}

template <typename OUT> struct OutPack;
template <> struct OutPack<float> {
    static __device__ __forceinline__ void store(gptr_t p, f32x4 v)
    {
        *(__attribute__((address_space(1))) f32x4 *)p = v;
    }
    static __device__ __forceinline__ void to_lds(uint32_t addr, f32x4 v)
    {
        *(__attribute__((address_space(3))) f32x4 *)(uintptr_t)addr = v;
    }
};
struct bf16_out {
    uint16_t bits;
};
template <> struct OutPack<bf16_out> {
    static __device__ __forceinline__ u32x2 pack(f32x4 v)
    {
        f32x2 a, b;
        a[0] = v[0];
        a[1] = v[1];
        b[0] = v[2];
        b[1] = v[3];
        u32x2 r;
        r[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2));
        r[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(b, bf16x2));
        return r;
    }
    static __device__ __forceinline__ void store(gptr_t p, f32x4 v)
    {
        *(__attribute__((address_space(1))) u32x2 *)p = pack(v);
    }
    static __device__ __forceinline__ void to_lds(uint32_t addr, f32x4 v)
    {
        *(__attribute__((address_space(3))) u32x2 *)(uintptr_t)addr = pack(v);
    }
};

// Number of multiples of `period` in [lo, hi] (the x refills, one per stage start, among a range of steps).
constexpr int multiples_in(int lo, int hi, int period)
{
    int n = 0;
    for (int t = lo; t <= hi; ++t)
        if (t % period == 0)
            ++n;
    return n;
}

// NW: wavefronts per workgroup (4: one per SIMD; 8: two per SIMD, each with half the registers, so
// that one wavefront's waits at memory instructions and barriers are covered by the other's matrix
// instructions).  NT: 16-channel sub-tiles per wavefront (BN = 16 NW NT).  NEDGE: the last channel
// block may be partial (weight rows are clamped, stores predicated).
//
// PACKED: a.W is the copy grkan_linear_pack_w makes of the weights, in which the 1 KB a weight fetch
// brings (16 rows x 32 k, pieces already permuted) is contiguous: the fetch then reads eight whole
// cache lines in sequence instead of sixteen half lines D_in * 2 bytes apart (5 - 8 % of the kernel's
// time at the wide layer).  Rows past Nout are zeros there.
template <int NW, int NT, typename OUT, bool NEDGE, bool PACKED, int M, int N>
__global__ __launch_bounds__(64 * NW, 1) void grkan_linear_fwd_kernel(const LinArgs a)
{
    static_assert(M == 5 && N == 4 && kMT == 7, "rational_piece is written for degrees (5, 4) and 7-tile steps");
    static_assert(NW == 4 || NW == 8, "4 or 8 wavefronts");
    constexpr int MT = kMT;
    // Accumulator tiles pinned to accumulation registers; the rest live in vector registers.  One wave
    // per SIMD has 256 of each kind; with two waves per SIMD the compiler splits a wave's 256
    // registers evenly, 128 accumulation registers (32 tiles) and 128 vector registers.
    constexpr int kAgprTiles = NW == 8 ? 32 : 64;
    constexpr int WN = 16 * NT;
    constexpr int BN = NW * WN;
    constexpr int U = 16 / NW;   // 16-byte pieces of x a lane holds per pair of stages
    constexpr int PPS = U / 2;   // ... of which it works on per stage
    constexpr int kWBuf = BN * kWRow;
    constexpr uint32_t kWs0 = 2 * kXBuf;
    // How many 16-row sub-tiles a weight fetch runs ahead of the step that multiplies with it.  The two
    // W buffers are a ring of 2 NT slots per wave, and a slot is free once the step that used it has
    // been issued, so anything up to 2 NT - 2 is possible.  Measured at the wide layer (NT = 6),
    // same box: 4 -> 152 us (every step waits for its sub-tile), 5 -> 147, 6 -> 149.7, 7 -> 147.4 (*),
    // 8 -> 148.0 (*), 10 -> 152.7 (*) ((*) another box, where 6 gave 146.6): more requests in flight
    // than needed slow everything down, as in the elementwise kernels.
    // With the packed weights a fetch is cheaper on the memory side and one step more ahead pays
    // (same box: 5 -> 137.6 us, 6 -> 134.9, 8 -> 134.5).
    constexpr int kAhead = NT == 6 ? (PACKED ? 6 : 5) : NT;
    constexpr int kStep0 = 4 * NT; // an arbitrary stage start, for counting in absolute steps
    extern __shared__ __align__(16) char smem[];
    const lptr_t lds = (lptr_t)smem;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;

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

    // ---- x loader.  A pair of stages needs 128 rows x 128 bytes of x: 16 units of (16 rows, one
    // 64-byte half), one load instruction each, four lanes per row, so that a load touches sixteen
    // 64-byte segments (with one lane per row it would touch 64 and keep the address path of the
    // vector cache busy four times as long).  Wave w takes units U w .. U w + U - 1; unit q is half
    // q / 8 (wave-uniform: one coefficient group per wave and pair), rows 16 (q % 8) + lane / 4,
    // bytes 16 (lane % 4) .. of the half.
    const int xhalf = (wave * U) >> 3;
    const int xrow0 = ((wave * U) & 7) * 16 + (lane >> 2);
    const uint64_t x_base = reinterpret_cast<uint64_t>(a.x) + (uint64_t)m0 * K2 + (uint64_t)xhalf * 64u;
    uint32_t x_lane[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        int64_t xg = m0 + xrow0 + 16 * u;
        if (xg > a.rows - 1)
            xg = a.rows - 1; // rows past the end read the last row (never stored)
        x_lane[u] = (uint32_t)((xg - m0) * (int64_t)K2) + (uint32_t)(lane & 3) * 16u;
    }
    // + buffer + 16 u rows
    const uint32_t x_dst = lds0 + (uint32_t)xrow0 * kXPitch + (uint32_t)xhalf * 64u + (uint32_t)(lane & 3) * 16u;
    constexpr uint32_t kXPieceStep = 16u * kXPitch;

    // ---- W loader: LDS-direct loads.  One wave instruction brings 16 rows x 64 bytes (32 k) and
    // lands them in LDS as 1024 contiguous bytes, lane l at byte 16 l: row l / 4 of the 16, slot
    // l % 4 of the row.  Instruction i of wave w covers rows WN w + 16 i + 0..15 of the channel
    // block: the rows whose products this very wave computes, so that the weights need no barrier
    // at all - a wave waits for its own loads and reads what they brought.  Which 16-byte piece of its row a lane fetches is permuted (slot = piece xor g(row)) so
    // that the operand reads below, 16 rows at one piece index, fall into 16 different 16-byte bank
    // groups although rows are 64 bytes apart; g depends on the low four row bits only, i.e. on
    // the lane.
    const uint32_t w_g = (uint32_t)((lane >> 4) ^ (lane >> 3)) & 3u;
    const uint64_t w_base = PACKED ? reinterpret_cast<uint64_t>(a.W) + ((uint64_t)(n0 >> 4) + (uint32_t)(NT * wave)) * 1024u
                                   : reinterpret_cast<uint64_t>(a.W) + (uint64_t)n0 * K2;
    constexpr int kWLanes = PACKED ? 1 : (NEDGE ? NT : 1);
    uint32_t w_lane[kWLanes];
    if constexpr (PACKED) {
        w_lane[0] = (uint32_t)lane * 16u;
    } else if constexpr (NEDGE) {
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            int r = WN * wave + 16 * i + (lane >> 2);
            if (n0 + r > a.Nout - 1)
                r = a.Nout - 1 - n0;
            w_lane[i] = (uint32_t)r * K2 + (((uint32_t)lane & 3u) ^ w_g) * 16u;
        }
    } else {
        w_lane[0] = (uint32_t)(WN * wave + (lane >> 2)) * K2 + (((uint32_t)lane & 3u) ^ w_g) * 16u;
    }
    const uint64_t w_stage_bytes = (uint64_t)(uint32_t)a.wtiles * 1024u; // packed: bytes per stage of 32 k
    // stage at byte offset kbyte of the rows -> W buffer `buf`
    auto w_fetch = [&](int i, uint32_t kbyte, int buf) {
        const lptr_t dst = lds + kWs0 + (uint32_t)buf * kWBuf + (uint32_t)(NT * wave + i) * 1024u;
        gcptr_t src;
        if constexpr (PACKED)
            src = (gcptr_t)(w_base + (uint64_t)(kbyte >> 6) * w_stage_bytes + (uint32_t)i * 1024u) + w_lane[0];
        else if constexpr (NEDGE)
            src = (gcptr_t)(w_base + kbyte) + w_lane[i];
        else
            src = (gcptr_t)(w_base + kbyte + (uint64_t)i * 16u * K2) + w_lane[0];
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                         (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
    };

    // ---- operand reads: lane -> row lane % 16 of a 16-row sub-tile, 16-byte piece lane / 16
    const uint32_t xf_base = lds0 + (uint32_t)(lane & 15) * kXPitch + (uint32_t)(lane >> 4) * 16u;
    // row r = wave WN + nt 16 + lane % 16: g(r) = ((r >> 2) ^ (r >> 1)) & 3 with r mod 16 = lane % 16
    const uint32_t wf_g = (uint32_t)(((lane & 15) >> 2) ^ ((lane & 15) >> 1)) & 3u;
    const uint32_t wf_base =
        lds0 + kWs0 + (uint32_t)(wave * WN + (lane & 15)) * kWRow + (((uint32_t)(lane >> 4)) ^ wf_g) * 16u;

    f32x4 acc[NT][MT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            acc[nt][mt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    // The contraction runs over pairs of stages (64 k = 128 bytes of a row) in rotated order: this
    // workgroup starts at pair `rot` and wraps around.  Rows of x and W are K2 bytes apart, which for
    // the model shapes is a multiple of 16 cache lines, so the same 128 bytes of every row sit in one
    // L2 channel; workgroups that all walk K from 0 would hammer one channel at a time.  With the
    // workgroups of an XCD started at different pairs their fetches spread over all channels.  The
    // order of summation of an output stays fixed by the shape (it is the rotation of its token block).
    const int32_t n_pairs = a.K >> 6;
    const uint32_t rot = ((uint32_t)mb >> 3) % (uint32_t)n_pairs;
    auto next_pair = [&](uint32_t pp) { return pp + 1u == (uint32_t)n_pairs ? 0u : pp + 1u; };

    // Coefficients of the group the wave's next F work lies in: wave-uniform, in scalar registers,
    // reloaded once per pair.  They are read through the constant address space (nothing writes A
    // and B while the kernel runs): the compiler then uses scalar loads and waits for them at their
    // first use, a stage later.  Read through the generic pointers inside the loop, it cannot show
    // that nothing has written them since the kernel started and would fetch them through the
    // vector memory path, into vector registers, with a wait on the vector-memory counter (and so on
    // the x and W loads just issued) in front of the first use.  (A quotient of an integer division
    // is formed by vector instructions, hence the readfirstlane.)
    typedef const __attribute__((address_space(4))) float *cfloat_ptr;
    Coef<M, N> c, c_next;
    auto coef_for = [&](Coef<M, N> &dst, uint32_t kbyte_pair) {
        const int g = __builtin_amdgcn_readfirstlane((int)((kbyte_pair / 2u + (uint32_t)xhalf * 32u) / (uint32_t)a.dgc));
        const cfloat_ptr pa = (cfloat_ptr)(uintptr_t)(a.A + (size_t)g * (M + 1));
        const cfloat_ptr pb = (cfloat_ptr)(uintptr_t)(a.B + (size_t)g * N);
#pragma unroll
        for (int i = 0; i <= M; ++i)
            dst.a[i] = pa[i];
#pragma unroll
        for (int i = 0; i < N; ++i)
            dst.b[i] = pb[i];
    };
    uint32_t pp = rot; // the pair the matrix products work on
    coef_for(c, pp * 128u);

    u32x4 xq[U]; // this lane's 16-byte pieces (8 k each, of U rows) of the pair F works on next

    // ---- prologue: the first stage of W and F(first pair) into LDS, the first half of the second pair into registers
#pragma unroll
    for (int i = 0; i < (kAhead < NT ? kAhead : NT); ++i)
        w_fetch(i, pp * 128u, 0);
#pragma unroll
    for (int i = 0; i < kAhead - NT; ++i)
        w_fetch(i, pp * 128u + 64u, 1);
#pragma unroll
    for (int u = 0; u < U; ++u)
        xq[u] = gload16(x_base + pp * 128u, x_lane[u]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        u32x4 y;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            y[j] = rational_pair<M, N>(xq[u][j], c);
        lds_write16(x_dst + (uint32_t)u * kXPieceStep, y);
    }
    {
        const uint32_t kp = next_pair(pp) * 128u;
#pragma unroll
        for (int u = 0; u < PPS; ++u)
            xq[u] = gload16(x_base + kp, x_lane[u]);
        coef_for(c, kp);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // One stage: the matrix products of stage s = 2 p + Q from LDS.  Beside them: the next stage of
    // W goes from memory straight into the other W buffer, one 16-row sub-tile per step; one half of
    // the x registers is refilled (the half that was consumed one stage ago); F is evaluated on the
    // other half, which holds 16 k of pair p + 1, and written to the other x buffer.
    //
    // Waiting.  A wave's loads complete in the order they were issued (x refill, then the sub-tiles
    // 0 .. NT - 1 of a stage), and the weights are the wave's own, so a sub-tile is waited for just
    // before its first read, two steps ahead of its use, by the number of younger loads that may stay
    // in flight: there is no point in a stage at which all loads must have arrived, and a fetch has
    // most of a stage to complete.  (Issued all at once at the start of a stage, or two per step, the
    // fetches stalled the issuing wave for hundreds of cycles each: the path that forms the
    // addresses of a 16-row gather is the narrow one.)  The F values are shared between the waves:
    // one barrier per pair, after its second stage - what a stage writes is read from the next pair
    // on, and the buffer it writes to was last read in the pair before, which ended with a barrier.
    // The barrier is written in assembly, with a wait for this wave's LDS writes only: the
    // compiler's own would wait for the loads in flight as well.  The loads issued during the last
    // pair (for pairs that would come after it) wrap around to valid memory; what they bring is
    // never consumed.
    // The order of the instructions is the one written here: every matrix instruction is followed
    // by a piece of F and a scheduling fence (see rational_piece).
    bf16x8 xf[MT]; // token operands of a stage, one per 16-token sub-tile
    bf16x8 wf[3];  // ring of weight operands
    auto stage = [&](auto Qc, uint32_t xsel_read, uint32_t xsel_write, uint32_t kbyte_stage0, uint32_t kbyte_stage1, uint32_t kbyte_stage2,
                     uint32_t kbyte_refill, uint32_t kbyte_coef) {
        constexpr int Q = decltype(Qc)::value;
        constexpr int kWords = 4 * PPS;                       // words (pairs of elements) F works on per stage and lane
        constexpr int kPairsPerStep = (kWords + NT - 1) / NT;
        const uint32_t xb = xf_base + xsel_read + (uint32_t)Q * 64u;
        const uint32_t wb = wf_base + (uint32_t)Q * kWBuf;
        // The second stage of a pair finds its first operands already on their way: the first stage
        // reads them during its last two steps, each register as soon as its last use has been
        // issued (the x values of the pair are all in LDS, the weights are the wave's own).  The
        // first stage of a pair follows a barrier and reads its operands here.
        constexpr bool kHandOver = NT == 6; // the register ring below frees slots 0 and 1 in steps NT - 2 and NT - 1
        if constexpr (!(kHandOver && Q == 1)) {
            // sub-tiles 0 and 1 of this stage have arrived when at most the loads issued after the
            // fetch of sub-tile 1 are in flight: kAhead - 2 fetches and the x refills between them
            wait_loads<kAhead - 2 + PPS * multiples_in(kStep0 + 1 - kAhead + 1, kStep0 - 1, NT)>();
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                xf[mt] = lds_read16(xb + (uint32_t)mt * 16u * kXPitch);
            // weight operands two steps ahead of their use (an LDS read takes longer than the 7 matrix
            // instructions of one step)
            wf[0] = lds_read16(wb);
            if constexpr (NT > 1)
                wf[1] = lds_read16(wb + 16u * kWRow);
        }
        // refill the pieces that were consumed one stage ago
#pragma unroll
        for (int u = 0; u < PPS; ++u) {
            keep_in_loop(x_lane[(1 - Q) * PPS + u]);
            xq[(1 - Q) * PPS + u] = gload16(x_base + kbyte_refill, x_lane[(1 - Q) * PPS + u]);
        }
#pragma unroll
        for (int i = 0; i < kWLanes; ++i)
            keep_in_loop(w_lane[i]);
        u32x4 y[PPS];
        fence_schedule();
        static_for<0, NT>([&](auto ntc) {
            constexpr int nt = decltype(ntc)::value;
            // the fetch of this step: the sub-tile kAhead steps on, into the slot of the ring whose
            // sub-tile was multiplied two steps ago
            if constexpr (nt + kAhead < NT)
                w_fetch(nt + kAhead, kbyte_stage0, Q);
            else if constexpr (nt + kAhead < 2 * NT)
                w_fetch(nt + kAhead - NT, kbyte_stage1, 1 - Q);
            else
                w_fetch(nt + kAhead - 2 * NT, kbyte_stage2, Q);
            // A sub-tile is read two steps ahead of its use; its fetch was issued kAhead steps before
            // that use, and younger than it are the kAhead - 2 fetches since and the x refills of the
            // stage starts in between.
            if constexpr (nt + 2 < NT) {
                wait_loads<kAhead - 2 + PPS * multiples_in(kStep0 + nt + 2 - kAhead + 1, kStep0 + nt, NT)>();
                wf[(nt + 2) % 3] = lds_read16(wb + (uint32_t)(nt + 2) * 16u * kWRow);
            } else if constexpr (kHandOver && Q == 0) {
                // sub-tile nt + 2 - NT (0, then 1) of the next stage
                wait_loads<kAhead - 2 + PPS * multiples_in(kStep0 + nt + 2 - kAhead + 1, kStep0 + nt, NT)>();
                wf[(nt + 2) % 3] = lds_read16(wf_base + (uint32_t)(1 - Q) * kWBuf + (uint32_t)(nt + 2 - NT) * 16u * kWRow);
            }
            fence_schedule();
            PairState ps[kPairsPerStep];
            uint32_t res[kPairsPerStep];
            static_for<0, MT>([&](auto mtc) {
                constexpr int mt = decltype(mtc)::value;
                mfma_16x16x32<(nt * MT + mt) < kAgprTiles>(acc[nt][mt], wf[nt % 3], xf[mt]);
                // The coefficients F needs from the next pair on are requested right after the first
                // matrix instruction of the pair: scalar loads and LDS reads share a counter that can
                // only be waited on as a whole while a scalar load is in flight, and the next wait
                // for an LDS operand is two steps away.
                if constexpr (Q == 0 && nt == 0 && mt == 0)
                    coef_for(c_next, kbyte_coef);
                if constexpr (kHandOver && Q == 0 && nt == NT - 1)
                    xf[mt] = lds_read16(xf_base + xsel_read + 64u + (uint32_t)mt * 16u * kXPitch);
                // F on this step's share: words nt, nt + NT, .. of the lane's words of this stage
                static_for<0, kPairsPerStep>([&](auto ic) {
                    constexpr int j = nt + decltype(ic)::value * NT;
                    if constexpr (j < kWords)
                        rational_piece<mt>(ps[decltype(ic)::value], xq[Q * PPS + (j >> 2)][j & 3], c, res[decltype(ic)::value]);
                });
                fence_schedule();
            });
            static_for<0, kPairsPerStep>([&](auto ic) {
                constexpr int j = nt + decltype(ic)::value * NT;
                if constexpr (j < kWords)
                    y[j >> 2][j & 3] = res[decltype(ic)::value];
            });
        });
#pragma unroll
        for (int u = 0; u < PPS; ++u)
            lds_write16(x_dst + xsel_write + (uint32_t)(Q * PPS + u) * kXPieceStep, y[u]);
        if constexpr (Q == 1)
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    };

    uint32_t xsel = 0; // buffer the matrix products read
    for (int32_t p = 0; p < n_pairs; ++p) {
        const uint32_t p1 = next_pair(pp);
        const uint32_t p2 = next_pair(p1);
        // first stage of the pair (the weight fetches run kAhead sub-tiles ahead, into the next stage
        // and the one after it): refill pieces 2, 3 with the next pair; F on pieces 0, 1 of the next pair
        stage(std::integral_constant<int, 0>{}, xsel, kXBuf - xsel, pp * 128u, pp * 128u + 64u, p1 * 128u, p1 * 128u, p2 * 128u);
        // second stage: refill pieces 0, 1 with the pair after the next; F on pieces 2, 3 of the next
        // pair.  (The coefficients requested in the first stage
        // are for F during the next pair, which works on the pair after it.)
        stage(std::integral_constant<int, 1>{}, xsel, kXBuf - xsel, pp * 128u + 64u, p1 * 128u, p1 * 128u + 64u, p2 * 128u, 0u);
        c = c_next;
        xsel = kXBuf - xsel;
        pp = p1;
    }

    // the matrix instructions above are opaque to the compiler's hazard tracking: let the last of
    // them drain before their results are read
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");

    // ---- epilogue: lane holds channels n0 + wave WN + nt 16 + (lane / 16) 4 + 0..3 of token m0 + mt 16 + lane % 16
    constexpr int ES = (int)sizeof(OUT);
    if constexpr (!NEDGE) {
        // Through LDS, so that every store instruction of a wavefront covers 1 KB of one output row:
        // stored straight from the accumulator layout a row would receive its cache lines in 32-byte
        // parts, from different wavefronts at different times, and lines leave the L2 partly written
        // (measured: 1.9 times the output's bytes written to memory).  The tile goes through in
        // passes of as many 16-token sub-tiles as the operand buffers (no longer needed) hold.
        constexpr int kRowB = (BN + 16) * ES; // the padding spreads 8 (float32: 4) tokens over the 64 banks
        constexpr int kFit = (2 * kXBuf + 2 * kWBuf) / (16 * kRowB);
        static_assert(kFit >= 1, "one 16-token sub-tile must fit the operand buffers");
        constexpr int kPasses = (MT + kFit - 1) / kFit;
        constexpr int MTP = (MT + kPasses - 1) / kPasses;
        constexpr int CPR = BN * ES / 16; // 16-byte chunks per row
        f32x4 bv[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            bv[nt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            if (a.bias)
                bv[nt] = *(const f32x4 *)(a.bias + n0 + wave * WN + nt * 16 + (lane >> 4) * 4);
        }
        // every fetch into the operand buffers has landed (the last stages prefetch past the end of
        // the walk, which wraps around) and every wavefront has read its last operands
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        const uint32_t lane_dst = lds0 + (uint32_t)(lane & 15) * kRowB + (uint32_t)(wave * WN + (lane >> 4) * 4) * ES;
        char *const out_tile = a.out + ((int64_t)m0 * a.Nout + n0) * ES;
        static_for<0, kPasses>([&](auto PASS) {
            constexpr int P0 = PASS.value * MTP;
            constexpr int NM = (MT - P0) < MTP ? (MT - P0) : MTP;
            if constexpr (P0 > 0)
                __syncthreads(); // the previous pass has been read out
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int mt = 0; mt < NM; ++mt)
                    OutPack<OUT>::to_lds(lane_dst + (uint32_t)(mt * 16) * kRowB + (uint32_t)(nt * 16) * ES,
                                         acc[nt][P0 + mt] + bv[nt]);
            __syncthreads();
            constexpr int kChunks = NM * 16 * CPR;
#pragma unroll 4
            for (int c = tid; c < kChunks; c += 64 * NW) {
                const int r = c / CPR;
                const int col = c - r * CPR;
                const int64_t trow = (int64_t)(P0 * 16 + r);
                if (m0 + trow < a.rows) {
                    const u32x4 v = *(const __attribute__((address_space(3))) u32x4 *)(uintptr_t)(
                        lds0 + (uint32_t)r * kRowB + (uint32_t)col * 16u);
                    *(__attribute__((address_space(1))) u32x4 *)(gptr_t)(out_tile + trow * a.Nout * ES + col * 16) = v;
                }
            }
        });
    } else {
        const int32_t o_lane = n0 + wave * WN + (lane >> 4) * 4;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int32_t o = o_lane + nt * 16;
            if (o >= a.Nout)
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
}

// --------------------------------------------------------------------------
// host side
// --------------------------------------------------------------------------
using LinKernel = void (*)(const LinArgs);

// Tile variants: (waves, 16-channel sub-tiles per wave) -> channels per workgroup
//   (8, 6): 768  two waves per SIMD, the variant for wide layers
//   (8, 3): 384  two waves per SIMD (one wave per SIMD with six sub-tiles was 12 % slower: a single
//                 wave cannot cover its own waits)
//   (4, 3): 192  also with a partial last channel block
struct Variant {
    int nw, nt;
    int bn() const { return 16 * nw * nt; }
};

static Variant pick_variant(int32_t D_out)
{
    if (D_out % 768 == 0)
        return Variant{8, 6};
    if (D_out % 384 == 0)
        return Variant{8, 3};
    return Variant{4, 3};
}

template <typename OUT, bool PACKED> static LinKernel select_kernel(Variant v, bool nedge)
{
    if (v.nw == 8 && v.nt == 6)
        return grkan_linear_fwd_kernel<8, 6, OUT, false, PACKED, 5, 4>;
    if (v.nw == 8 && v.nt == 3)
        return grkan_linear_fwd_kernel<8, 3, OUT, false, PACKED, 5, 4>;
    if (v.nw == 4 && v.nt == 3)
        return nedge ? grkan_linear_fwd_kernel<4, 3, OUT, true, PACKED, 5, 4>
                     : grkan_linear_fwd_kernel<4, 3, OUT, false, PACKED, 5, 4>;
    return nullptr;
}

static size_t lds_bytes(Variant v) { return (size_t)2 * kXBuf + (size_t)2 * v.bn() * kWRow; }

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

// The packed copy of the weights: for stage s (32 k), 16-row tile t and lane l, the 16 bytes lane l of
// a weight fetch brings - row 16 t + l / 4, piece (l % 4) xor g(l) of that row's 64 bytes of stage
// s - at ((s T + t) 64 + l) 16, T tiles per stage.  Rows past D_out are zeros.
__global__ __launch_bounds__(256) void grkan_linear_pack_w_kernel(const char *__restrict__ W, char *__restrict__ Wp,
                                                                    int32_t K, int32_t Nout, int32_t wtiles,
                                                                    int64_t pieces)
{
    const uint32_t K2 = (uint32_t)K * 2u;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < pieces; idx += (int64_t)gridDim.x * 256) {
        const uint32_t l = (uint32_t)(idx & 63);
        const int64_t st = idx >> 6;
        const int64_t stage = st / wtiles;
        const int32_t t = (int32_t)(st - stage * wtiles);
        const int32_t r = 16 * t + (int32_t)(l >> 2);
        const uint32_t g = ((l >> 4) ^ (l >> 3)) & 3u;
        u32x4 v = u32x4{0u, 0u, 0u, 0u};
        if (r < Nout)
            v = *(const u32x4 *)(W + (int64_t)r * K2 + stage * 64 + (int64_t)(((l & 3u) ^ g) * 16u));
        *(u32x4 *)(Wp + idx * 16) = v;
    }
}

// tiles per stage of the packed copy: whole channel blocks of the tile variant the layer runs with
static int64_t packed_tiles(int32_t D_out)
{
    const int bn = pick_variant(D_out).bn();
    return ((int64_t)D_out + bn - 1) / bn * (bn / 16);
}

static grkan_status_t linear_shape_status(int64_t rows, int32_t D_in, int32_t D_out, int32_t G)
{
    if (rows < 0 || D_in <= 0 || D_out <= 0 || G <= 0 || D_in % G != 0)
        return GRKAN_ERR_SHAPE;
    const int32_t dg = D_in / G;
    // the contraction runs in pairs of 32-k stages with one coefficient group per stage and wave;
    // a lane stores four consecutive channels
    if (D_in % 64 != 0 || dg % 32 != 0 || D_out % 4 != 0)
        return GRKAN_ERR_UNSUPPORTED;
    // 32-bit lane offsets inside a tile: up to 128 rows of x and up to 768 rows of W, D_in * 2 bytes apart
    if (rows > (INT64_MAX / 8) / (D_in > D_out ? D_in : D_out) || (int64_t)D_in * 2 * 768 >= ((int64_t)1 << 32))
        return GRKAN_ERR_UNSUPPORTED;
    return GRKAN_OK;
}

static grkan_status_t linear_fwd_impl(const void *x, const float *A, const float *B, const void *W, bool packed,
                                      const float *bias, void *out, int64_t rows, int32_t D_in, int32_t D_out,
                                      int32_t G, int32_t m, int32_t n, grkan_dtype_t io, grkan_dtype_t out_dtype,
                                      void *hip_stream)
{
    if (io != GRKAN_BF16 || (out_dtype != GRKAN_BF16 && out_dtype != GRKAN_F32))
        return GRKAN_ERR_DTYPE;
    if (m != 5 || n != 4)
        return GRKAN_ERR_DEGREE;
    const grkan_status_t shape = linear_shape_status(rows, D_in, D_out, G);
    if (shape != GRKAN_OK && shape != GRKAN_ERR_UNSUPPORTED)
        return shape;
    if (!A || !B || !W || (rows > 0 && (!x || !out)))
        return GRKAN_ERR_NULL;
    // 128-bit loads of x and W rows, 64/128-bit stores of four output channels, vector load of the bias
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(out) |
         reinterpret_cast<uintptr_t>(bias)) % 16 != 0 ||
        (reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) % 4 != 0)
        return GRKAN_ERR_ALIGN;
    if (shape != GRKAN_OK)
        return shape;
    if (rows == 0)
        return GRKAN_OK;

    const Variant v = pick_variant(D_out);
    const int bn = v.bn();
    const bool nedge = D_out % bn != 0;
    LinKernel kernel;
    if (packed)
        kernel = out_dtype == GRKAN_BF16 ? select_kernel<bf16_out, true>(v, nedge) : select_kernel<float, true>(v, nedge);
    else
        kernel = out_dtype == GRKAN_BF16 ? select_kernel<bf16_out, false>(v, nedge) : select_kernel<float, false>(v, nedge);
    if (!kernel)
        return GRKAN_ERR_LAUNCH;
    const size_t lds = lds_bytes(v);
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
    a.dgc = D_in / G;
    const int64_t mblocks = (rows + kBM - 1) / kBM;
    const int64_t nblocks = (D_out + bn - 1) / bn;
    const int64_t grid = ((mblocks + 7) / 8) * 8 * nblocks;
    if (mblocks > INT32_MAX / 2 || grid > INT32_MAX)
        return GRKAN_ERR_UNSUPPORTED;
    a.mblocks = (int32_t)mblocks;
    a.nblocks = (int32_t)nblocks;
    a.wtiles = (int32_t)packed_tiles(D_out);
    void *args[] = {&a};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3((unsigned)grid), dim3(64 * v.nw),
                                         args, lds, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? GRKAN_OK : GRKAN_ERR_LAUNCH;
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
    return linear_fwd_impl(x, A, B, W, false, bias, out, rows, D_in, D_out, G, m, n, io, out_dtype, hip_stream);
}

extern "C" grkan_status_t grkan_linear_fwd_packed(const void *x, const float *A, const float *B, const void *Wp,
                                                  const float *bias, void *out,
                                                  int64_t rows, int32_t D_in, int32_t D_out, int32_t G,
                                                  int32_t m, int32_t n, grkan_dtype_t io, grkan_dtype_t out_dtype,
                                                  void *hip_stream)
{
    return linear_fwd_impl(x, A, B, Wp, true, bias, out, rows, D_in, D_out, G, m, n, io, out_dtype, hip_stream);
}

extern "C" size_t grkan_linear_packed_w_bytes(int32_t D_in, int32_t D_out)
{
    if (D_in <= 0 || D_out <= 0 || D_in % 64 != 0 || D_out % 4 != 0 || (int64_t)D_in * 2 * 768 >= ((int64_t)1 << 32))
        return 0;
    return (size_t)(D_in / 32) * (size_t)packed_tiles(D_out) * 1024u;
}

extern "C" grkan_status_t grkan_linear_pack_w(const void *W, void *Wp, int32_t D_in, int32_t D_out, void *hip_stream)
{
    if (D_in <= 0 || D_out <= 0)
        return GRKAN_ERR_SHAPE;
    const size_t bytes = grkan_linear_packed_w_bytes(D_in, D_out);
    if (bytes == 0)
        return GRKAN_ERR_UNSUPPORTED;
    if (!W || !Wp)
        return GRKAN_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(Wp)) % 16 != 0)
        return GRKAN_ERR_ALIGN;
    const int64_t pieces = (int64_t)(bytes / 16);
    const int64_t want = (pieces + 255) / 256;
    const unsigned grid = (unsigned)(want < 8192 ? want : 8192);
    const char *w_arg = static_cast<const char *>(W);
    char *wp_arg = static_cast<char *>(Wp);
    int32_t tiles = (int32_t)packed_tiles(D_out);
    int64_t n_pieces = pieces;
    void *args[] = {&w_arg, &wp_arg, &D_in, &D_out, &tiles, &n_pieces};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(grkan_linear_pack_w_kernel), dim3(grid), dim3(256),
                                         args, 0, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? GRKAN_OK : GRKAN_ERR_LAUNCH;
}
