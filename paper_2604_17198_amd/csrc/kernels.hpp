// Launchers of the HIP kernels (one translation unit per kernel family).
#pragma once
#include "common.hpp"

namespace nacho {

// Algorithm 1 for boundaries 0..P.  `queries` (device, may be NULL) overrides
// the built-in queries; otherwise Q_p = min(p*grain, total) when grain > 0 and
// floor(p*total/P) when grain == 0 (total = total_unscaled * cost_scale).
// `clear_words` (may be NULL): n_clear 64-bit words the kernel sets to zero on the side, and
// `clear_status` (may be NULL) a status word it sets to NACHO_OK: the state of the kernels that
// follow it in a fused call.
hipError_t launch_partition(const DevOperands &ops, int64_t cost_scale, int64_t P, int64_t grain,
                            const int64_t *queries, int64_t total_unscaled,
                            int32_t *coord, int32_t *posn, int64_t *cost, hipStream_t stream,
                            unsigned long long *clear_words = nullptr, int64_t n_clear = 0,
                            int32_t *clear_status = nullptr);

// Items one wavefront can stage for SpMV (partition work must not exceed it).
int spmv_capacity(int dtype);
// `grain` > 0: the partitions come from the fixed-grain queries Q_p = min(p * grain, nnz)
// (the kernel then deals the partitions of long rows out by XCD); 0: any partitions.
hipError_t launch_spmv_exec(int dtype, const int32_t *pos, const int32_t *crd, const void *val,
                            const void *x, void *y, int64_t n_rows, int64_t nnz,
                            const int32_t *coord, const int32_t *posn, int64_t P,
                            void *carry_val, int32_t *carry_row, int64_t grain, hipStream_t stream);
hipError_t launch_spmv_fixup(int dtype, void *y, int64_t P, const void *carry_val,
                             const int32_t *carry_row, const int32_t *pos, int64_t grain, hipStream_t stream);

// ---- SpMM (lane per column of B, n <= 64) -----------------------------------
int spmm_capacity(int dtype);
hipError_t launch_spmm_exec(int dtype, const int32_t *pos, const int32_t *crd, const void *val,
                            const void *B, int n, int64_t ldb, void *C, int64_t ldc,
                            const int32_t *coord, const int32_t *posn, int64_t P, void *carry_val,
                            int32_t *carry_row, hipStream_t stream);
// `grain` > 0: fixed-grain partitions of `grain` non-zeros (run lengths then come from `pos`).
hipError_t launch_spmm_fixup(int dtype, void *C, int64_t ldc, int n, int64_t P, const void *carry_val,
                             const int32_t *carry_row, const int32_t *pos, int64_t grain, hipStream_t stream);

// ---- k-way union addition ---------------------------------------------------
enum { SPADD_VECTOR = 0, SPADD_CSR = 1, SPADD_DCSR = 2 };
constexpr int kSpaddCap = 4096;         // entries of all operands one partition (workgroup) stages

struct SpaddValues { const void *v[NACHO_MAX_OPERANDS]; };
struct SpaddOut {
    int32_t *pos0, *crd0, *pos1, *crd1;
    void *val;
    int64_t cap_rows, cap_nnz;
    int64_t *counts;
    int32_t *status;
};
int spadd_capacity(int fmt);
// 64-bit words of prefix-sum state a call with P partitions uses.
int64_t spadd_state_words(int64_t P);
// Count, prefix sum and fill in one kernel, one workgroup per partition.  `multiply`: the k-way
// intersection with products instead of the union with sums (vectors and CSR only).
hipError_t launch_spadd(int fmt, int dtype, bool multiply, const DevOperands &ops, const SpaddValues &vals,
                        int64_t P, const int32_t *coord, const int32_t *posn, unsigned long long *tile_state,
                        const SpaddOut &out, hipStream_t s);

}  // namespace nacho
