// Host-only launch planning for the GR-KAN kernels and the cover check the
// CPU tests run on it.  No HIP calls here.
#include "grkan_plan.h"

#include <cstring>
#include <numeric>
#include <vector>

namespace grkan {

int elem_size(grkan_dtype_t io) { return io == GRKAN_F32 ? 4 : 2; } // bfloat16 and float16: 2

grkan_status_t check_shape(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io)
{
    if (io != GRKAN_F32 && io != GRKAN_BF16 && io != GRKAN_F16)
        return GRKAN_ERR_DTYPE;
    if (rows < 0 || D <= 0 || G <= 0 || D % G != 0)
        return GRKAN_ERR_SHAPE;
    // element offsets are 64-bit, but keep rows * D well inside int64
    if (rows > (INT64_MAX / 8) / D)
        return GRKAN_ERR_UNSUPPORTED;
    return GRKAN_OK;
}

static int pick_vec(int32_t dg, int es, int32_t align_bytes)
{
    for (int vec = 16 / es; vec > 1; vec /= 2)
        if (dg % vec == 0 && align_bytes >= vec * es)
            return vec;
    return 1;
}

// Plan of the group walk over `Gw` groups of `dgw` channels with vectors of
// `vec` elements (Gw = 1, dgw = D describes the flat walk over whole rows).
static grkan_status_t plan_walk(int64_t rows, int32_t D, int32_t Gw, int32_t vec, int es, int32_t num_cu,
                                int32_t wg_per_cu, grkan_plan_t *out)
{
    const int32_t dg = D / Gw;
    const int32_t v = dg / vec;
    const int32_t nw = kWavesPerWg;

    // Adjacent groups share a workgroup when one group's row segment is not a
    // whole number of cache lines, so that the waves touching the two halves
    // of a line sit on the same compute unit (and the same XCD's L2).
    int32_t k = 1;
    while (((int64_t)k * dg * es) % kLineBytes != 0 && 2 * k <= nw && Gw % (2 * k) == 0)
        k *= 2;
    const int32_t ns = nw / k;
    const int32_t nb = Gw / k;

    const int64_t n_vec = rows * (int64_t)v;          // vectors per group
    const int64_t n_chunks = (n_vec + kWave - 1) / kWave;
    const int64_t capacity = (int64_t)num_cu * wg_per_cu;
    int64_t base = capacity / nb;
    if (base < 1)
        base = 1;
    const int64_t by_work = (n_chunks + ns - 1) / ns;  // more workgroups would have idle waves

    // fixed-column mode needs 64 * Wg = 64 * wpb * ns to be a multiple of v
    const int64_t q = v / std::gcd((int64_t)v, (int64_t)kWave);
    const int64_t q2 = q / std::gcd(q, (int64_t)ns);
    const int64_t rrow_max = ((int64_t)v - 1 + (kWave - 1)) / v;
    const bool offsets_fit = (rrow_max * D + dg) * (int64_t)es < ((int64_t)1 << 32);

    int64_t wpb = base < by_work ? base : by_work;
    int32_t fixed = 0;
    if (rows == 0) {
        wpb = 0;
    } else if (offsets_fit) {
        if (wpb >= q2) {
            wpb -= wpb % q2;
            fixed = 1;
        } else if (q2 <= 4 * base) {
            wpb = q2; // a few idle or queued workgroups are cheaper than the general walk
            fixed = 1;
        }
    }
    if (wpb * nb > INT32_MAX || wpb * ns >= ((int64_t)1 << 25))
        return GRKAN_ERR_UNSUPPORTED;

    out->vec = vec;
    out->vecs_per_segment = v;
    out->waves_per_wg = nw;
    out->groups_per_wg = k;
    out->waves_per_group_in_wg = ns;
    out->wg_per_bundle = (int32_t)wpb;
    out->grid = (int32_t)(wpb * nb);
    out->fixed_col = fixed;
    out->chunk_stride = wpb * ns;
    out->partials_per_group = (int32_t)wpb;
    out->lane_coef = 0;
    out->column_split = 1;
    return GRKAN_OK;
}

// How many column blocks each group is cut into for the backward group walk.
// With one or two groups the waves sweep whole rows (or half rows) in step,
// which this memory system serves 5 % slower than four to eight interleaved
// column streams (measured at [50432, 3072]: 5.8 TB/s with G = 1 or 2 against
// 6.1-6.2 TB/s with G = 4 or 8).  Few, long groups are therefore walked as
// G * split narrower ones that share the coefficients of their parent; the
// blocks stay a whole number of cache lines, at least three, and of vectors.
static int32_t pick_column_split(int32_t G, int32_t dg, int32_t vec, int es)
{
    int32_t split = 1;
    while ((int64_t)G * split < 4) {
        const int32_t next = split * 2;
        if (dg % next != 0)
            break;
        const int64_t bytes = (int64_t)(dg / next) * es;
        if (bytes % kLineBytes != 0 || bytes < 3 * kLineBytes || (dg / next) % vec != 0)
            break;
        split = next;
    }
    return split;
}

grkan_status_t make_plan(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io, int32_t align_bytes,
                         int32_t num_cu, int32_t wg_per_cu, bool forward, grkan_plan_t *out, Walk *walk)
{
    grkan_status_t st = check_shape(rows, D, G, io);
    if (st != GRKAN_OK)
        return st;
    if (!out)
        return GRKAN_ERR_NULL;
    const int es = elem_size(io);
    if (align_bytes < es || num_cu <= 0 || wg_per_cu <= 0)
        return GRKAN_ERR_ALIGN;

    const int32_t dg = D / G;
    const int32_t vec = pick_vec(dg, es, align_bytes);

    // Wavefronts bound to one group read that group's row segments; measured on
    // MI355X this streams at full speed for segments of 384 bytes and more but
    // loses 18 % at 192 bytes and 40 % at 96 bytes.  Short or line-straddling
    // segments therefore take the flat walk over whole rows (if its columns can
    // be fixed), with the coefficients held per lane.  The forward pass, which
    // has nothing to reduce and so gains nothing from group-bound waves, always
    // prefers the flat walk (measured 2-6 % faster); the backward pass keeps the
    // group walk for long segments (scalar-register coefficients, short
    // epilogue: measured 6-10 % faster there).
    const int64_t seg_bytes = (int64_t)dg * es;
    const bool short_segments = G > 1 && (forward || seg_bytes < 3 * kLineBytes || seg_bytes % kLineBytes != 0);
    if (short_segments && rows > 0) {
        // The backward pass prefers the flat walk over a few column blocks of whole groups to one
        // sweep over whole rows, for the reason given at pick_column_split; the forward pass, one
        // read and one write per element, was measured no faster that way.
        const int32_t blocks_to_try[] = {8, 4, 2, 1};
        for (int32_t blocks : blocks_to_try) {
            if (blocks > 1) {
                const int64_t block_bytes = (int64_t)(D / blocks) * es;
                if (forward || G % blocks != 0 || block_bytes % kLineBytes != 0 || block_bytes < 3 * kLineBytes)
                    continue;
            }
            st = plan_walk(rows, D, blocks, vec, es, num_cu, wg_per_cu, out);
            if (st == GRKAN_OK && out->fixed_col && out->groups_per_wg == 1) {
                out->lane_coef = 1;
                out->column_split = blocks;
                // every workgroup of a block writes one row for each group of that block
                out->partials_per_group = out->wg_per_bundle;
                if (walk)
                    return walk_from_plan(rows, D, G, io, *out, walk);
                return GRKAN_OK;
            }
        }
    }
    const int32_t split = forward ? 1 : pick_column_split(G, dg, vec, es);
    st = plan_walk(rows, D, G * split, vec, es, num_cu, wg_per_cu, out);
    if (st != GRKAN_OK)
        return st;
    out->column_split = split;
    out->partials_per_group *= split; // workspace rows per coefficient group
    if (walk)
        return walk_from_plan(rows, D, G, io, *out, walk);
    return GRKAN_OK;
}

grkan_status_t walk_from_plan(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io,
                              const grkan_plan_t &pl, Walk *walk)
{
    grkan_status_t st = check_shape(rows, D, G, io);
    if (st != GRKAN_OK)
        return st;
    if (pl.vec <= 0 || (D / G) % pl.vec != 0)
        return GRKAN_ERR_SHAPE;
    if (pl.column_split < 1 || (pl.lane_coef ? G % pl.column_split != 0 : (D / G) % pl.column_split != 0))
        return GRKAN_ERR_SHAPE;
    // groups of the walk: column blocks of whole coefficient groups (flat walk) or of one group each
    const int32_t Gw = pl.lane_coef ? pl.column_split : G * pl.column_split;
    const int32_t dg = D / Gw;
    if (pl.vecs_per_segment != dg / pl.vec || pl.groups_per_wg <= 0 ||
        Gw % pl.groups_per_wg != 0 || pl.waves_per_wg != kWavesPerWg || pl.waves_per_wg % pl.groups_per_wg != 0 ||
        pl.waves_per_group_in_wg != pl.waves_per_wg / pl.groups_per_wg || pl.wg_per_bundle < 0 ||
        (pl.lane_coef && !pl.fixed_col))
        return GRKAN_ERR_SHAPE;
    walk->rows = rows;
    walk->D = D;
    walk->G = Gw;
    walk->dg = dg;
    walk->vec = pl.vec;
    walk->v = pl.vecs_per_segment;
    walk->k = pl.groups_per_wg;
    walk->ns = pl.waves_per_group_in_wg;
    walk->nb = Gw / pl.groups_per_wg;
    walk->wg_per_bundle = pl.wg_per_bundle;
    const int64_t Wg = (int64_t)pl.wg_per_bundle * walk->ns;
    if (Wg >= ((int64_t)1 << 25))
        return GRKAN_ERR_UNSUPPORTED;
    walk->Wg = (int32_t)Wg;
    walk->dq = Wg ? (int32_t)((kWave * Wg) / walk->v) : 0;
    walk->dr = Wg ? (int32_t)((kWave * Wg) % walk->v) : 0;
    const int64_t n_vec = rows * (int64_t)walk->v;
    walk->n_full = n_vec / kWave;
    const int64_t visits = Wg ? walk->n_full / Wg : 0;
    if (visits >= INT32_MAX - 1)
        return GRKAN_ERR_UNSUPPORTED;
    walk->visits_base = (int32_t)visits;
    walk->visits_rem = Wg ? (int32_t)(walk->n_full % Wg) : 0;
    walk->rem = (int32_t)(n_vec % kWave);
    if (rows > 0 && Wg == 0)
        return GRKAN_ERR_SHAPE; // a plan with no waves cannot cover a non-empty array
    return GRKAN_OK;
}

// Visit every (block, wave, lane, visit) exactly as the kernels do and count.
static int64_t cover_errors(const Walk &p, bool fixed, int es)
{
    const int64_t n_total = p.rows * (int64_t)p.D / p.vec;
    std::vector<uint8_t> seen((size_t)n_total, 0);
    int64_t bad = 0;
    const int64_t total_elems = p.rows * (int64_t)p.D;
    const int32_t nw = p.k * p.ns;
    const int32_t grid = p.nb * p.wg_per_bundle;

    auto visit = [&](int32_t g, int64_t off) {
        if (off < 0 || off + p.vec > total_elems || off % p.vec != 0) {
            ++bad;
            return;
        }
        const int64_t c = off % p.D;
        if (c < (int64_t)g * p.dg || c + p.vec > (int64_t)(g + 1) * p.dg) {
            ++bad;
            return;
        }
        uint8_t &s = seen[(size_t)(off / p.vec)];
        if (s)
            ++bad;
        s = 1;
    };

    for (int32_t b = 0; b < grid; ++b) {
        for (int32_t wv = 0; wv < nw; ++wv) {
            const WaveId id = wave_id(p, b, wv);
            const int32_t n_it = full_visits(p, id.w);
            const bool tail = owns_tail(p, id.w);
            if (fixed) {
                const int64_t base0 = fixed_base0(p, id.g, id.w);
                const int64_t step = fixed_step(p);
                for (int32_t lane = 0; lane < kWave; ++lane) {
                    const uint64_t lo_bytes = (uint64_t)fixed_lane_offset(p, id.w, lane) * (uint64_t)es;
                    if (lo_bytes >> 32) {
                        ++bad; // the kernels hold this offset in 32 bits
                        continue;
                    }
                    const int64_t lo = (int64_t)(lo_bytes / es);
                    for (int32_t it = 0; it < n_it; ++it)
                        visit(id.g, base0 + (int64_t)it * step + lo);
                    if (tail && lane < p.rem)
                        visit(id.g, base0 + (int64_t)n_it * step + lo);
                }
            } else {
                for (int32_t lane = 0; lane < kWave; ++lane) {
                    LanePos s = lane_start(p, id.w, lane);
                    for (int32_t it = 0; it < n_it; ++it) {
                        visit(id.g, elem_offset(p, id.g, s));
                        lane_advance(p, s);
                    }
                    if (tail && lane < p.rem)
                        visit(id.g, elem_offset(p, id.g, s));
                }
            }
        }
    }
    for (uint8_t s : seen)
        if (!s)
            ++bad;
    return bad;
}

} // namespace grkan

extern "C" grkan_status_t grkan_plan(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io,
                                     int32_t align_bytes, int32_t num_cu, int32_t wg_per_cu,
                                     int32_t forward, grkan_plan_t *plan)
{
    return grkan::make_plan(rows, D, G, io, align_bytes, num_cu, wg_per_cu, forward != 0, plan, nullptr);
}

extern "C" int64_t grkan_plan_cover_errors(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io,
                                           const grkan_plan_t *plan)
{
    if (!plan)
        return 1;
    grkan::Walk w;
    if (grkan::walk_from_plan(rows, D, G, io, *plan, &w) != GRKAN_OK)
        return 1;
    if (rows * (int64_t)D > ((int64_t)1 << 28))
        return -1;
    if (plan->fixed_col && w.dr != 0)
        return 1;
    return grkan::cover_errors(w, plan->fixed_col != 0, grkan::elem_size(io));
}

extern "C" const char *grkan_status_string(grkan_status_t s)
{
    switch (s) {
    case GRKAN_OK: return "ok";
    case GRKAN_ERR_NULL: return "null pointer";
    case GRKAN_ERR_SHAPE: return "bad shape (need rows >= 0, D > 0, G > 0, D % G == 0)";
    case GRKAN_ERR_DEGREE: return "unsupported degrees (built: (m, n) = (5, 4), (3, 2), (7, 6))";
    case GRKAN_ERR_ALIGN: return "pointer not aligned to its element size";
    case GRKAN_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case GRKAN_ERR_DTYPE: return "unknown dtype";
    case GRKAN_ERR_LAUNCH: return "HIP launch or query failed";
    case GRKAN_ERR_UNSUPPORTED:
        return "shape or type outside what the kernels cover (index range; grkan_linear_fwd: see its conditions)";
    case GRKAN_ERR_SCRATCH_LIMIT: return "the shape needs more workspace than the 4 MiB scratch of grkan_bwd_noalloc";
    }
    return "unknown status";
}
