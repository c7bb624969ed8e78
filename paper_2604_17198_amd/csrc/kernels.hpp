// Launchers of the HIP kernels (one translation unit per kernel family).
#pragma once
#include "common.hpp"

namespace nacho {

// Algorithm 1 for boundaries 0..P.  `queries` (device, may be NULL) overrides
// the built-in queries; otherwise Q_p = min(p*grain, total) when grain > 0 and
// floor(p*total/P) when grain == 0 (total = total_unscaled * cost_scale).
hipError_t launch_partition(const DevOperands &ops, int64_t cost_scale, int64_t P, int64_t grain,
                            const int64_t *queries, int64_t total_unscaled,
                            int32_t *coord, int32_t *posn, int64_t *cost, hipStream_t stream);

// Items one wavefront can stage for SpMV (partition work must not exceed it).
int spmv_capacity(int dtype);
hipError_t launch_spmv_exec(int dtype, const int32_t *pos, const int32_t *crd, const void *val,
                            const void *x, void *y, int64_t n_rows, int64_t nnz,
                            const int32_t *coord, const int32_t *posn, int64_t P,
                            void *carry_val, int32_t *carry_row, hipStream_t stream);
hipError_t launch_spmv_fixup(int dtype, void *y, int64_t P, const void *carry_val,
                             const int32_t *carry_row, hipStream_t stream);

}  // namespace nacho
