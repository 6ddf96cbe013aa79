// Host-side launch planning (declarations).  See grkan_walk.h for the walk the
// plan parameterises.
#ifndef GRKAN_PLAN_H_
#define GRKAN_PLAN_H_

#include "../../include/grkan.h"
#include "grkan_walk.h"

namespace grkan {

constexpr int kWavesPerWg = 4; // 256 threads per workgroup
constexpr int kThreadsPerWg = kWavesPerWg * kWave;

int elem_size(grkan_dtype_t io);
grkan_status_t check_shape(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io);

// Fills the public plan and (optionally) the kernel-side walk parameters.
grkan_status_t make_plan(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io, int32_t align_bytes,
                         int32_t num_cu, int32_t wg_per_cu, bool forward, grkan_plan_t *out, Walk *walk);

// Rebuilds the walk parameters from a public plan (validating it).
grkan_status_t walk_from_plan(int64_t rows, int32_t D, int32_t G, grkan_dtype_t io,
                              const grkan_plan_t &pl, Walk *walk);

} // namespace grkan
#endif // GRKAN_PLAN_H_
