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
// `row_cost` (one CSR operand with built-in queries only): every row costs that many units on top of its
// stored non-zeros (in the units of a non-zero before cost_scale); total_unscaled stays the non-zero count.
// `zero_rows` (may be NULL; one CSR operand with built-in queries only, i.e. the fused SpMV and
// SpMM calls): the kernel also sets to zero the rows of a dense result whose operand row is empty.
struct ZeroRows {
    void *base;          // row r of the result: `width` elements of `elem` bytes from base + r * ld * elem
    int64_t ld;
    int32_t width, elem;
};
hipError_t launch_partition(const DevOperands &ops, int64_t cost_scale, int64_t P, int64_t grain,
                            const int64_t *queries, int64_t total_unscaled,
                            int32_t *coord, int32_t *posn, int64_t *cost, hipStream_t stream,
                            unsigned long long *clear_words = nullptr, int64_t n_clear = 0,
                            int32_t *clear_status = nullptr, const ZeroRows *zero_rows = nullptr,
                            int64_t row_cost = 0);

hipError_t launch_partition_csr64(const int64_t *pos, const int32_t *crd, int64_t n_rows, int64_t nnz, int64_t P,
                                  int32_t *coord, int64_t *posn, int64_t *cost, hipStream_t stream);

// Items one wavefront can stage for SpMV (partition work must not exceed it).
int spmv_capacity(int dtype);
// `grain` > 0: the partitions come from the fixed-grain queries Q_p = min(p * grain, nnz)
// (the kernel then deals the partitions of long rows out by XCD); 0: any partitions.
hipError_t launch_spmv_exec(int dtype, const int32_t *pos, const int32_t *crd, const void *val,
                            const void *x, void *y, int64_t n_rows, int64_t nnz,
                            const int32_t *coord, const int32_t *posn, int64_t P,
                            void *carry_val, int32_t *carry_row, int64_t grain, hipStream_t stream);
// (coord == nullptr with grain > 0: the fused form, every wavefront searches its own boundaries)
hipError_t launch_zero_vector(int dtype, void *y, int64_t n, hipStream_t stream);
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
enum { SPADD_VECTOR = 0, SPADD_CSR = 1, SPADD_DCSR = 2, SPADD_COO = 3, SPADD_CSF3 = 4 };

struct SpaddValues { const void *v[NACHO_MAX_OPERANDS]; };
struct SpaddOut {
    int32_t *pos0, *crd0, *pos1, *crd1;
    void *val;
    int64_t cap_rows, cap_nnz;
    int32_t *pos2, *crd2;        // third-order tensors: the innermost level (crd1 / pos2: the fibres)
    int64_t cap_fibres;
    int64_t *counts;
    int32_t *status;
};
// Entries of all operands one partition (workgroup) may hold.
int spadd_capacity(int fmt, int dtype);
// Workgroups of the merge kernel that run on one compute unit at a time.
int spadd_resident();
// Wavefronts of one of its workgroups (the instrumented build logs one record per wavefront).
int spadd_wavefronts();
// 64-bit words of prefix-sum state a call with P partitions uses.
int64_t spadd_state_words(int64_t P);
// The partition table a merge kernel that searches its own boundaries fills, and the total cost Q*.
struct SpaddSearch {
    int32_t *coord, *posn;
    int64_t *cost;
    int64_t total;
};
// Sparse vectors, union: as launch_spadd, but without a partition kernel before it -- every workgroup
// searches its two boundaries (equal-share queries over P partitions) and stores them in the table.
// The prefix-sum state and the status word must be zero when the kernel starts.
hipError_t launch_spadd_vector_search(int dtype, const DevOperands &ops, const SpaddValues &vals, int64_t P,
                                      const SpaddSearch &search, unsigned long long *tile_state, const SpaddOut &out,
                                      hipStream_t s);
// Count, prefix sum and fill in one kernel, one workgroup per partition.  `multiply`: the k-way
// intersection with products instead of the union with sums (vectors and CSR only).
hipError_t launch_spadd(int fmt, int dtype, bool multiply, const DevOperands &ops, const SpaddValues &vals,
                        int64_t P, const int32_t *coord, const int32_t *posn, unsigned long long *tile_state,
                        const SpaddOut &out, hipStream_t s);

// ---- recursive partitioning for an outer intersection (DCSR products) -----------
// Memoised row loop of Section 3.3, all arrays on the device:
//   rows[i']                    coordinate of the i'-th row all operands store
//   start[t * stride + i']      position in operand t's crd / val of that row's first entry
//   cost[t * (stride + 1) + x]  entries operand t stores in the intersected rows before row x
//                               (x <= stride; rows past the last intersected one hold nothing)
//   head[0] = number M of intersected rows, head[1 + t] = cost[t][stride]
struct RemapArrays {
    int32_t *rows, *start, *cost, *head;
    int64_t stride;
};
// 32-bit words of scratch a prefix sum over `batch` arrays of n items uses.
int64_t remap_scan_words(int64_t n, int batch);
// flags[e] = all operands store row crd0_0[e]; qpos[(t-1) * count_0 + e] = its position in operand t.
// posn0: boundaries of a P0-way partition of the operands' level-0 coordinate arrays.
hipError_t launch_rows_match(const DevOperands &ops, int64_t P0, const int32_t *posn0, int32_t *flags,
                             int32_t *qpos, hipStream_t s);
// rows, start and the per-row entry counts (in r.cost, which must be zero beforehand), head[0]
hipError_t launch_remap_rows(const DevOperands &ops, const int32_t *flags, const int32_t *qpos,
                             const RemapArrays &r, int32_t *tsum, hipStream_t s);
// r.cost: per-row counts -> exclusive prefix sums (in place), head[1 + t]
hipError_t launch_remap_costs(int k, const RemapArrays &r, int32_t *tsum, hipStream_t s);
// Result rows that hold an entry: pos_full[0 .. head[0]] over the intersected rows -> out.pos0 / crd0 /
// pos1 / counts (counts_in = {rows, nnz} of the remapped result).
hipError_t launch_compact_rows(const RemapArrays &r, const int32_t *pos_full,
                               const int64_t *counts_in, const SpaddOut &out, int32_t *tsum, hipStream_t s);
// plan[0..2] = {partitions of the remapped nest, intersected rows, remapped total cost}, computed on the
// device from r.head: capacity = entries one partition may hold, round = resident workgroups of the
// chip (the count is rounded up to whole rounds when P_min == 0), P_max = what the launches are sized for.
hipError_t launch_remap_plan(int k, const RemapArrays &r, int64_t capacity, int64_t round, int64_t P_min,
                             int64_t P_max, int64_t *plan, hipStream_t s);
hipError_t launch_empty_result(const SpaddOut &out, int64_t *info, hipStream_t s);

// ---- measurement aids: kernels of known traffic (streaming read, copy, independent gathers) ----
hipError_t launch_probe_read(const void *src, size_t bytes, void *sink, hipStream_t s);
hipError_t launch_probe_copy(void *dst, const void *src, size_t bytes, hipStream_t s);
hipError_t launch_probe_gather(const void *table, size_t window_bytes, int64_t gathers, void *sink, hipStream_t s);

// ---- debug aid: the preconditions of the operands, checked on the device -----------
hipError_t launch_validate(const DevOperands &ops, int32_t *status, int64_t *info, hipStream_t s);

}  // namespace nacho
