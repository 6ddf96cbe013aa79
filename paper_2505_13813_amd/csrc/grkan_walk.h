// Index arithmetic shared by the HIP kernels and the host-side cover check.
//
// The [rows, D] array is cut by channel group (FlashKAT paper, Eq. "GR_KAN":
// channel c uses the coefficients of group c div d_g).  Group g owns a slab of
// rows x d_g elements, seen as rows * v vectors of `vec` elements
// (v = d_g / vec), numbered t = row * v + col.  A wavefront is bound to one
// group for the whole kernel, so the coefficients are wave-uniform and the m + 1 + n
// coefficient-gradient partial sums can be reduced across the wavefront
// without regard to group boundaries.  Wave w of the Wg waves of a group visits
// the 64-vector chunks w, w + Wg, w + 2 Wg, ... of that numbering.
//
// When 64 * Wg is a multiple of v ("fixed column" mode, which the host plan
// arranges whenever it can) a lane keeps its column and its row offset inside
// the chunk for the whole kernel and only a wave-uniform base advances.
//
// The same walk with a single group of D channels (or a few column blocks of
// whole coefficient groups) is the "flat" walk: wavefronts then read
// contiguous kilobytes whatever d_g is, and because columns are fixed each
// lane belongs to one coefficient group for the whole kernel and keeps that
// group's coefficients in vector registers.  Likewise a walk group can be a
// column block of one coefficient group (few, long groups are cut up).
#ifndef GRKAN_WALK_H_
#define GRKAN_WALK_H_

#include <stdint.h>

#if defined(__HIPCC__)
#define GRKAN_HD __host__ __device__ inline
#else
#define GRKAN_HD inline
#endif

// Integer division is expanded into vector instructions, which leaves even a
// wave-uniform quotient in vector registers; on the device the quotient is
// moved back to a scalar register so that everything derived from it (loop
// counts, base addresses) stays scalar.  On the host this is the identity.
#if defined(__HIP_DEVICE_COMPILE__)
#define GRKAN_UNIFORM(x) __builtin_amdgcn_readfirstlane((int)(x))
#else
#define GRKAN_UNIFORM(x) ((int)(x))
#endif

namespace grkan {

constexpr int kWave = 64;       // CDNA wavefront width
constexpr int kMaxCoef = 14;    // most sums per group over the built degrees: (m, n) = (7, 6) -> m + 1 + n
constexpr int kLineBytes = 128; // cache line the bundling rule is built around

// Launch geometry in the form the kernels consume (all wave-uniform).
struct Walk {
    int64_t rows;
    int32_t D;
    int32_t G;
    int32_t dg;            // channels per group
    int32_t vec;           // elements per vector
    int32_t v;             // vectors per row segment of a group
    int32_t k;             // groups per workgroup
    int32_t ns;            // waves of a workgroup that share one group
    int32_t nb;            // bundles = G / k
    int32_t wg_per_bundle; // workgroups per bundle
    int32_t Wg;            // waves per group = wg_per_bundle * ns (< 2^25)
    int32_t dq;            // (64 * Wg) div v : rows a lane advances per visit
    int32_t dr;            // (64 * Wg) mod v : columns a lane advances per visit (0 in fixed mode)
    int64_t n_full;        // chunks of a group with all 64 lanes in range
    int32_t visits_base;   // n_full div Wg : full chunks every wave visits (< 2^31 - 1)
    int32_t visits_rem;    // n_full mod Wg : waves below this index visit one more
    int32_t rem;           // lanes in range in the last, partial chunk (0 = none)
};

// Which group and which wave-of-the-group a wavefront is.
struct WaveId {
    int32_t g;
    int32_t g_local; // index of the group inside the workgroup's bundle
    int32_t wg_index; // index of the workgroup inside its bundle
    int32_t w;       // index of the wave among the Wg waves of its group
};

GRKAN_HD WaveId wave_id(const Walk &p, int32_t block, int32_t wave_in_wg)
{
    WaveId id;
    id.wg_index = GRKAN_UNIFORM(block / p.nb);
    const int32_t bundle = block - id.wg_index * p.nb;
    const int32_t sub = GRKAN_UNIFORM(wave_in_wg / p.k);
    id.g_local = wave_in_wg - sub * p.k;
    id.g = bundle * p.k + id.g_local;
    id.w = id.wg_index * p.ns + sub;
    return id;
}

// Number of full chunks wave w visits: chunks w, w + Wg, ... below n_full.
GRKAN_HD int32_t full_visits(const Walk &p, int32_t w)
{
    return p.visits_base + (w < p.visits_rem ? 1 : 0);
}

// Does wave w own the partial last chunk?  (It then comes right after its
// full visits: n_full = w + full_visits * Wg.)
GRKAN_HD bool owns_tail(const Walk &p, int32_t w)
{
    return p.rem != 0 && p.visits_rem == w;
}

// Position of a lane at its first visit: row and column (in vectors) inside
// the group's slab.
struct LanePos {
    int64_t row;
    int32_t col;
};

GRKAN_HD LanePos lane_start(const Walk &p, int32_t w, int32_t lane)
{
    const uint32_t t = (uint32_t)w * kWave + (uint32_t)lane;
    const uint32_t row = t / (uint32_t)p.v;
    LanePos s;
    s.row = row;
    s.col = (int32_t)(t - row * (uint32_t)p.v);
    return s;
}

// One visit later (general mode; in fixed mode dr == 0 and only row moves).
GRKAN_HD void lane_advance(const Walk &p, LanePos &s)
{
    s.row += p.dq;
    s.col += p.dr;
    if (s.col >= p.v) {
        s.col -= p.v;
        s.row += 1;
    }
}

// Element offset of a lane position in the [rows, D] array.
GRKAN_HD int64_t elem_offset(const Walk &p, int32_t g, const LanePos &s)
{
    return s.row * (int64_t)p.D + (int64_t)g * p.dg + (int64_t)s.col * p.vec;
}

// Fixed-column mode: the wave-uniform base (element offset of the chunk's
// first row, column 0 of the group) at visit 0, its step per visit, and the
// lane's constant offset relative to that base.
GRKAN_HD int64_t fixed_base0(const Walk &p, int32_t g, int32_t w)
{
    const uint32_t row0 = (uint32_t)GRKAN_UNIFORM(((uint32_t)w * kWave) / (uint32_t)p.v);
    return (int64_t)row0 * p.D + (int64_t)g * p.dg;
}

GRKAN_HD int64_t fixed_step(const Walk &p) { return (int64_t)p.dq * p.D; }

// Column (in vectors, inside the walk group's row segment) a lane keeps in
// fixed-column mode, and the rows it sits below the chunk's first row.
struct LaneCol {
    uint32_t rrow;
    uint32_t ccol;
};

GRKAN_HD LaneCol fixed_lane_col(const Walk &p, int32_t w, int32_t lane)
{
    const uint32_t row0 = (uint32_t)GRKAN_UNIFORM(((uint32_t)w * kWave) / (uint32_t)p.v);
    const uint32_t c0 = (uint32_t)w * kWave - row0 * (uint32_t)p.v;
    const uint32_t cl = c0 + (uint32_t)lane;
    LaneCol lc;
    lc.rrow = cl / (uint32_t)p.v;
    lc.ccol = cl - lc.rrow * (uint32_t)p.v;
    return lc;
}

GRKAN_HD uint32_t fixed_lane_offset(const Walk &p, int32_t w, int32_t lane)
{
    const LaneCol lc = fixed_lane_col(p, w, lane);
    return lc.rrow * (uint32_t)p.D + lc.ccol * (uint32_t)p.vec;
}

} // namespace grkan
#endif // GRKAN_WALK_H_
