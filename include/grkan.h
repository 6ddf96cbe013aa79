/*
 * grkan.h - C ABI of the MI355X (gfx950) GR-KAN group-wise rational function.
 *
 * The operation is the safe Pade activation unit of the FlashKAT paper
 * (Sec. "Kolmogorov-Arnold Transformer", Eq. "pade"), applied group-wise over
 * channels, and its backward pass (Sec. "Gradient Computations", Eq. "grad_a",
 * "grad_b", "grad_x", summed as in Eq. "accum" and "accum2"):
 *
 *     channel c of a row uses coefficient row g = c div d_g,  d_g = D / G
 *     P(x)    = a_{g,0} + a_{g,1} x + ... + a_{g,m} x^m          (the paper: m = 5)
 *     Aden(x) = b_{g,1} x + ... + b_{g,n} x^n    (the paper writes A(x); n = 4)
 *     F(x)    = P(x) / (1 + |Aden(x)|)
 *
 * Common conventions of every entry point
 *   - x, y, dy, dx: DEVICE pointers to contiguous row-major [rows, D] arrays of
 *     the I/O dtype `io` (the paper's [B, N, d] tensor with B and N flattened).
 *   - A: DEVICE pointer, float32 [G, m+1], A[g*(m+1) + i] = a_{g,i}, i = 0..m.
 *     B: DEVICE pointer, float32 [G, n], B[g*n + (j-1)] = b_{g,j}, j = 1..n
 *     (there is no b_0).  Coefficients and their gradients are float32 for
 *     every I/O dtype; all arithmetic is float32 (the denominator polynomial
 *     is evaluated in double for float32 I/O).
 *   - The caller owns every buffer.  The library never allocates, frees or
 *     keeps device memory.
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and return without synchronising.  The
 *     status reports argument and launch errors only.
 *   - Built degrees: (m, n) = (5, 4), the paper's, and its neighbours (3, 2)
 *     and (7, 6); any other pair returns GRKAN_ERR_DEGREE.
 *   - D % G != 0 is GRKAN_ERR_SHAPE.  rows == 0 is valid.
 *   - Pointers must be aligned to the element size.  16-byte aligned tensors
 *     with d_g a multiple of 4 (float32) or 8 (16-bit formats) take the fast
 *     128-bit path; anything else silently takes a narrower-vector variant.
 */
#ifndef GRKAN_H_
#define GRKAN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GRKAN_F32 = 0,  /* x, y, dy, dx are float32 */
    GRKAN_BF16 = 1, /* x, y, dy, dx are bfloat16; outputs rounded to nearest even */
    GRKAN_F16 = 2   /* x, y, dy, dx are IEEE binary16; outputs rounded to nearest even,
                       results beyond 65504 in magnitude become infinities */
} grkan_dtype_t;

typedef enum {
    GRKAN_OK = 0,
    GRKAN_ERR_NULL = 1,      /* a required pointer is NULL */
    GRKAN_ERR_SHAPE = 2,     /* rows < 0, D <= 0, G <= 0 or D % G != 0 */
    GRKAN_ERR_DEGREE = 3,    /* (m, n) is not one of the built degree pairs */
    GRKAN_ERR_ALIGN = 4,     /* a pointer is not aligned to its element size */
    GRKAN_ERR_WORKSPACE = 5, /* workspace missing or smaller than required */
    GRKAN_ERR_DTYPE = 6,     /* unknown grkan_dtype_t */
    GRKAN_ERR_LAUNCH = 7,    /* the HIP runtime rejected a launch or query */
    GRKAN_ERR_UNSUPPORTED = 8, /* shape outside what the kernels index (see grkan_plan), or outside the shapes and
                                  types grkan_linear_fwd is built for */
    GRKAN_ERR_SCRATCH_LIMIT = 9 /* grkan_bwd_noalloc: the shape needs more workspace than the built-in scratch */
} grkan_status_t;

/* Human-readable name of a status; never NULL; static storage. */
const char *grkan_status_string(grkan_status_t status);

/*
 * Launch geometry the backward (and forward) pass uses for one shape.  Host
 * logic only; exposed so that callers and tests can see how a shape is cut.
 *
 * Two walks exist.  Group walk (lane_coef = 0): one wavefront owns one group g
 * and walks that group's [rows x d_g] slab in chunks of 64 vectors;
 * `wg_per_bundle * waves_per_group_in_wg` wavefronts share a group, and a
 * workgroup holds `groups_per_wg` adjacent groups.  Flat walk (lane_coef = 1),
 * chosen by the forward pass always and by the backward pass when a group's
 * row segment is shorter than 384 bytes or not a whole number of 128-byte
 * lines: wavefronts walk whole rows, or in the backward pass column blocks of
 * whole groups (the plan is that of `column_split` groups of D / column_split
 * channels), and every lane keeps the coefficients of the group its fixed
 * column belongs to.  In the backward pass a group walk over fewer than four
 * groups cuts each group into `column_split` column blocks that are walked
 * like groups of their own.
 */
typedef struct {
    int32_t vec;                  /* elements per lane per memory access */
    int32_t vecs_per_segment;     /* d_g / column_split / vec (D / column_split / vec in the flat walk) */
    int32_t waves_per_wg;         /* wavefronts in a workgroup */
    int32_t groups_per_wg;        /* adjacent groups that share a workgroup */
    int32_t waves_per_group_in_wg;/* waves_per_wg / groups_per_wg */
    int32_t wg_per_bundle;        /* workgroups that share one bundle of groups */
    int32_t grid;                 /* workgroups launched = (walk groups / groups_per_wg) * wg_per_bundle,
                                     walk groups = G * column_split (column_split in the flat walk) */
    int32_t fixed_col;            /* 1: every lane keeps its column for the whole kernel */
    int64_t chunk_stride;         /* 64-vector chunks between two visits of one wavefront */
    int32_t partials_per_group;   /* rows of m+1+n floats each group contributes to the workspace */
    int32_t lane_coef;            /* 1: flat walk with per-lane coefficients (then fixed_col = 1) */
    int32_t column_split;         /* backward pass only (1 otherwise).  Group walk: column blocks per group, each
                                     walked like a group of its own (fewer than four groups).  Flat walk:
                                     column blocks per row, each of whole groups and walked on its own */
} grkan_plan_t;

/*
 * Pure host function: the plan for a shape on a device with `num_cu` compute
 * units that keeps `wg_per_cu` workgroups of this kernel resident per unit.
 * `align_bytes` is the largest power of two (<= 16) that divides every tensor
 * pointer.  `forward` != 0 plans the forward pass (which prefers the flat walk
 * for every shape), 0 the backward pass.  Returns GRKAN_OK or the argument error.
 */
grkan_status_t grkan_plan(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io,
                          int32_t align_bytes, int32_t num_cu, int32_t wg_per_cu,
                          int32_t forward, grkan_plan_t *plan);

/*
 * Pure host function used by the tests: walks the plan exactly as the kernels
 * do and checks that every vector of the [rows, D] array is visited exactly
 * once and in bounds.  Returns 0 when the cover is exact, a positive count of
 * offending vectors otherwise, -1 if the shape is too large to simulate
 * (rows * D > 2^28).
 */
int64_t grkan_plan_cover_errors(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io,
                                const grkan_plan_t *plan);

/*
 * Bytes of device workspace grkan_bwd needs for this shape on the current
 * device (an upper bound over every alignment of the tensors and every built
 * degree pair).  Needs a HIP device; returns 0 on any error.
 */
size_t grkan_bwd_workspace_bytes(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io);

/*
 * What the HIP runtime reports about the current device, for measurement code
 * that prices a run against the hardware (no operation of the paper):
 * out[0] = compute units, out[1] = engine clock in kHz, out[2] = memory clock
 * in kHz, out[3] = memory bus width in bits.  `out` is a HOST pointer to four
 * int32.  Returns GRKAN_ERR_NULL or GRKAN_ERR_LAUNCH (a query failed).
 */
grkan_status_t grkan_device_query(int32_t *out);

/*
 * For experiments and tests (no operation of the paper): workgroups per compute
 * unit the persistent grids of the forward and of the backward pass are sized
 * for; 0 restores the built-in choice.  The environment variables
 * GRKAN_FWD_WG_PER_CU and GRKAN_BWD_WG_PER_CU give the initial values and are
 * read once, when the library is loaded.  Results do not depend on the setting
 * beyond the summation order of dA / dB; grkan_bwd_workspace_bytes follows it.
 */
void grkan_tuning_override(int32_t fwd_wg_per_cu, int32_t bwd_wg_per_cu);

/*
 * Forward (Eq. "pade"):  y[r, c] = P_g(x[r, c]) / (1 + |Aden_g(x[r, c])|).
 * y may alias x.
 */
grkan_status_t grkan_fwd(const void *x, const float *A, const float *B, void *y,
                         int64_t rows, int32_t D, int32_t G, int32_t m, int32_t n,
                         grkan_dtype_t io, void *hip_stream);

/*
 * Backward (Eq. "grad_x", "grad_a", "grad_b", "accum", "accum2").  Nothing is
 * saved from the forward pass; P, Aden and Q are recomputed from x.
 *
 *   dx[r, c]  = dy * ( P'/Q - s * Aden' * P / Q^2 ),   s = sign(Aden), s(0) = 0
 *   dA[g, i]  = sum over all rows and the d_g channels of group g of  dy * x^i / Q
 *   dB[g, j-1]= sum over the same elements of                       -dy * x^j * s * P / Q^2
 *
 * dA (float32 [G, m+1]) and dB (float32 [G, n]) are OVERWRITTEN with the sums.
 * The sums use no atomic operations and a fixed order: for one build, device,
 * shape and pointer alignment the results are bit-identical from run to run.
 * dx may alias dy or x.  `workspace` is device scratch of at least
 * grkan_bwd_workspace_bytes() bytes, 16-byte aligned, that must stay untouched
 * until the enqueued work has finished; its contents afterwards are unspecified.
 */
grkan_status_t grkan_bwd(const void *x, const void *dy, const float *A, const float *B,
                         void *dx, float *dA, float *dB,
                         void *workspace, size_t workspace_bytes,
                         int64_t rows, int32_t D, int32_t G, int32_t m, int32_t n,
                         grkan_dtype_t io, void *hip_stream);

/*
 * The GR-KAN layer in one kernel (Sec. "Kolmogorov-Arnold Transformer", Eq. "GR_KAN" with F of Eq. "pade"):
 *
 *     out[r, o] = sum_c W[o, c] * F_{g(c)}(x[r, c])  (+ bias[o]),   g(c) = c div d_g, d_g = D_in / G
 *
 * The rational function is evaluated in float32 on the way into the matrix
 * cores, rounded to bfloat16 (nearest even) and multiplied with bfloat16 weights
 * with float32 accumulation (v_mfma_f32_16x16x32_bf16); F(x) is never written
 * to memory.  (The equation has no bias; bias == NULL gives the equation.)
 *
 *   x    DEVICE, bfloat16 [rows, D_in], contiguous, 16-byte aligned   (io must be GRKAN_BF16)
 *   A, B DEVICE, float32 [G, m+1] / [G, n] as for grkan_fwd; (m, n) must be (5, 4)
 *   W    DEVICE, bfloat16 [D_out, D_in] row-major (the paper's W in R^{d_out x d_in}), 16-byte aligned
 *   bias DEVICE, float32 [D_out], 16-byte aligned, or NULL
 *   out  DEVICE, [rows, D_out] of out_dtype (GRKAN_BF16: rounded to nearest even; GRKAN_F32), 16-byte
 *        aligned; must not overlap x or W
 *
 * Shapes: D_in a multiple of 64 (and below 2^32 / 1536), d_g a multiple of 32 and D_out
 * a multiple of 4 (of the paper's model table: both layers of KAT-B and the second
 * layer of KAT-T and KAT-S; their first layers have groups of 24 and 48 channels);
 * anything else returns GRKAN_ERR_UNSUPPORTED and the caller runs grkan_fwd
 * followed by its own matrix product.  Asynchronous on hip_stream, caller-owned memory, no
 * workspace, results independent of the launch (fixed summation order per
 * output).  The first call of a kernel variant on a device raises that kernel's
 * dynamic-LDS limit (no allocation).
 * Sizing: a workgroup owns 112 rows x one channel block (768, 384 or 192
 * channels) and walks the whole of D_in by itself, so the kernel is at its best
 * from about as many such tiles as the chip has compute units (at 3072 -> 768:
 * from about 20,000 rows); far below that, grkan_fwd and a library product are
 * the faster route.
 */
grkan_status_t grkan_linear_fwd(const void *x, const float *A, const float *B, const void *W,
                                const float *bias, void *out,
                                int64_t rows, int32_t D_in, int32_t D_out, int32_t G,
                                int32_t m, int32_t n, grkan_dtype_t io, grkan_dtype_t out_dtype,
                                void *hip_stream);

/*
 * The same layer with the weights in a packed copy, for callers whose weights do
 * not change between calls (inference): the kernel's weight fetches then read
 * whole cache lines in sequence (5 - 8 % of the layer's time at the paper's wide
 * layer).  Results are bit-identical to grkan_linear_fwd (same arithmetic, same
 * summation order).
 *
 * grkan_linear_packed_w_bytes: size of the packed copy of a [D_out, D_in]
 *   bfloat16 matrix, or 0 if grkan_linear_fwd does not cover the shape.
 * grkan_linear_pack_w: writes it (one small kernel on hip_stream).
 *   W  DEVICE, bfloat16 [D_out, D_in] row-major, 16-byte aligned
 *   Wp DEVICE, grkan_linear_packed_w_bytes(D_in, D_out) bytes, 16-byte aligned, caller-owned.
 *   Layout: T = D_out rounded up to whole channel blocks of the kernel's tile, in
 *   units of 16 rows; for stage s (32 consecutive k), tile t and l = 0..63 the 16
 *   bytes at ((s T + t) 64 + l) 16 are row 16 t + l / 4, bytes
 *   64 s + 16 ((l mod 4) xor g) .. + 15 of W, g = ((l >> 4) xor (l >> 3)) and 3;
 *   rows past D_out are zeros.  The layout is tied to this library's build.
 * grkan_linear_fwd_packed: as grkan_linear_fwd with Wp in place of W.
 */
size_t grkan_linear_packed_w_bytes(int32_t D_in, int32_t D_out);
grkan_status_t grkan_linear_pack_w(const void *W, void *Wp, int32_t D_in, int32_t D_out, void *hip_stream);
grkan_status_t grkan_linear_fwd_packed(const void *x, const float *A, const float *B, const void *Wp,
                                       const float *bias, void *out,
                                       int64_t rows, int32_t D_in, int32_t D_out, int32_t G,
                                       int32_t m, int32_t n, grkan_dtype_t io, grkan_dtype_t out_dtype,
                                       void *hip_stream);

/*
 * grkan_bwd for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and kernels as grkan_bwd (bit-identical
 * outputs), minus the workspace: the workspace rows live in a fixed array of
 * GRKAN_NOALLOC_SCRATCH_BYTES (4 MiB) of device memory that belongs to the
 * library (one copy on every GPU it runs on, held until the process ends).
 * The call allocates and frees nothing.
 *
 *   - A shape whose workspace (grkan_bwd_workspace_bytes: G * rows per group *
 *     (m+1+n) * 4 bytes; 20 KB at the paper's KAT-B shape, 0.2 MB for 64 groups)
 *     exceeds the array returns GRKAN_ERR_SCRATCH_LIMIT and enqueues nothing.
 *   - Every call on one GPU uses that GPU's one array: calls whose kernels can
 *     overlap on a GPU (different streams, several host threads) race on it and
 *     give wrong dA / dB.  Calls on one stream are safe.  The array keeps the
 *     last call's rows; nothing in it has to start at zero, because stage 1
 *     writes every row stage 2 reads.
 *   - The first call on a device looks the array's address up (no allocation);
 *     make that call outside a graph capture.
 */
#define GRKAN_NOALLOC_SCRATCH_BYTES ((size_t)4 << 20)
grkan_status_t grkan_bwd_noalloc(const void *x, const void *dy, const float *A, const float *B,
                                 void *dx, float *dA, float *dB,
                                 int64_t rows, int32_t D, int32_t G, int32_t m, int32_t n,
                                 grkan_dtype_t io, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GRKAN_H_ */
