// Recursive partitioning (Section 3.3, Algorithm 2) for a product whose OUTER
// level is a sparse intersection: the Hadamard product of k DCSR matrices.
//
// Hierarchical skipping (rows that not every operand stores are never
// coiterated) makes the plain non-zero count of Section 4.2.2 the wrong cost,
// so the row loop is run first, on its own partitions, and memoises the cost
// of the loop below it:
//   1. the rows all operands store are found (a k-way intersection of the
//      level-0 coordinate arrays, partitioned by Algorithm 1 on those arrays);
//   2. for the i'-th such row, T[i'] = C_j(N_j | i) is stored -- here per
//      operand, S_t[i'] = number of entries operand t stores in the row, so that
//      T = sum_t S_t -- together with the position of the row's first entry in
//      every operand;
//   3. exclusive prefix sums turn S_t into the remapped cost function
//      C'_i(x) = T'[x] = sum_t S_t'[x].
// The remapped nest (i' dense over the intersected rows, then the column
// intersection) has no skipping left: it is what the partition kernel and the
// merge kernel run on, each operand seen as a CSR matrix over i' whose pos
// array is S_t' and whose row i' starts at the stored position in crd/val.
// Finally the rows of the result that received no entry are dropped.
//
// The prefix sums are the backend capability of Section 4.1: here two kernels,
// per-tile sums, then every tile adds up the sums of the tiles before it and
// scans its own items (no chain between workgroups).
#include "common.hpp"
#include "kernels.hpp"

namespace nacho {

namespace {

// ---- rows all operands store -----------------------------------------------
struct RowArrays {
    int32_t k;
    const int32_t *crd0[NACHO_MAX_OPERANDS];
};

// One workgroup per partition of the level-0 coordinate arrays.  Equal
// coordinates of different operands fall in one partition (Section 6), so every
// row of operand 0 in the partition looks for itself in the partition's segment
// of every other operand.  flags[e] = 1 when all operands store row crd0_0[e];
// qpos[(t-1) * count0 + e] = position of that row in operand t >= 1.
__global__ void __launch_bounds__(256)
rows_match_kernel(RowArrays rows, const int32_t *__restrict__ posn0, int32_t *__restrict__ flags,
                  int32_t *__restrict__ qpos, int64_t count0)
{
    const int64_t p = blockIdx.x;
    const int k = rows.k;
    const int a0 = posn0[p * k], b0 = posn0[(p + 1) * k];
    for (int e = a0 + (int)threadIdx.x; e < b0; e += (int)blockDim.x) {
        const int x = rows.crd0[0][e];
        bool all = true;
        for (int t = 1; t < k; ++t) {
            const int lo = posn0[p * k + t], hi = posn0[(p + 1) * k + t];
            const int q = lower_bound_global(rows.crd0[t], lo, hi, x);
            const bool hit = q < hi && rows.crd0[t][q] == x;
            all = all && hit;
            qpos[(int64_t)(t - 1) * count0 + e] = q;
        }
        flags[e] = all ? 1 : 0;
    }
}

// ---- exclusive prefix sums --------------------------------------------------
constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;                        // consecutive items of a thread
constexpr int kScanTile = kScanThreads * kScanItems;  // items of a workgroup

__device__ inline int block_sum(int v, int *lds)
{
    v = wave_sum<int>(v);
    __syncthreads();                                  // lds may still be read from an earlier call
    if (lane_id() == 0) lds[threadIdx.x / NACHO_WAVE] = v;
    __syncthreads();
    int s = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / NACHO_WAVE; ++w) s += lds[w];
    return s;
}

// tsum[b * n_tiles + tile] = sum of the items of the tile, for every array b of a batch
template <class In>
__global__ void __launch_bounds__(kScanThreads)
scan_sums_kernel(In in, int64_t n, int64_t n_tiles, int32_t *__restrict__ tsum)
{
    __shared__ int lds[kScanThreads / NACHO_WAVE];
    const int b = blockIdx.y;
    const int64_t tile = blockIdx.x;
    int s = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        const int64_t i = tile * kScanTile + (int64_t)j * kScanThreads + threadIdx.x;
        if (i < n) s += in.load(b, i);
    }
    s = block_sum(s, lds);
    if (threadIdx.x == 0) tsum[(int64_t)b * n_tiles + tile] = s;
}

// Item i of array b receives out.store(b, i, sum of the items before it, item);
// the last tile reports the total through out.finish.
template <class In, class Out>
__global__ void __launch_bounds__(kScanThreads)
scan_apply_kernel(In in, Out out, int64_t n, int64_t n_tiles, const int32_t *__restrict__ tsum)
{
    __shared__ int lds[kScanThreads / NACHO_WAVE];
    const int b = blockIdx.y;
    const int64_t tile = blockIdx.x;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / NACHO_WAVE;
    int part = 0;
    for (int64_t j = tid; j < tile; j += kScanThreads) part += tsum[(int64_t)b * n_tiles + j];
    const int offset = block_sum(part, lds);          // items of the tiles before this one
    int v[kScanItems], sum = 0;
    const int64_t first = tile * kScanTile + (int64_t)tid * kScanItems;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        v[j] = first + j < n ? in.load(b, first + j) : 0;
        sum += v[j];
    }
    const int incl = wave_inclusive_scan(sum);
    __syncthreads();
    if (lane == NACHO_WAVE - 1) lds[wave] = incl;
    __syncthreads();
    int excl = offset + incl - sum;
#pragma unroll
    for (int w = 0; w < kScanThreads / NACHO_WAVE; ++w)
        if (w < wave) excl += lds[w];
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (first + j < n) out.store(b, first + j, excl, v[j]);
        excl += v[j];
    }
    if (tile == n_tiles - 1 && tid == kScanThreads - 1) out.finish(b, excl);
}

struct ArrayIn {
    const int32_t *base;
    int64_t stride;
    __device__ int load(int b, int64_t i) const { return base[(int64_t)b * stride + i]; }
};

// S_t: in place, n + 1 results per array (the last one is the total, also kept in head[1 + t])
struct CostOut {
    int32_t *base;
    int64_t stride, n;
    int32_t *head;
    __device__ void store(int b, int64_t i, int before, int) const { base[(int64_t)b * stride + i] = before; }
    __device__ void finish(int b, int total) const
    {
        base[(int64_t)b * stride + n] = total;
        head[1 + b] = total;
    }
};

// Second stage of the row loop: the i'-th intersected row (i' = number of
// flagged rows before it) stores its coordinate, and per operand the position
// of its first entry and its number of entries.
struct RemapOut {
    int32_t k;
    const int32_t *crd0_0;
    const int32_t *qpos;
    int64_t count0;
    const int32_t *pos1[NACHO_MAX_OPERANDS];
    int32_t *rows;      // [M]
    int32_t *start;     // [k][stride]
    int32_t *len;       // [k][stride + 1]
    int64_t stride;
    int32_t *head;      // head[0] = M
    __device__ void store(int, int64_t e, int before, int flag) const
    {
        if (!flag) return;
        rows[before] = crd0_0[e];
        for (int t = 0; t < k; ++t) {
            const int q = t == 0 ? (int)e : qpos[(int64_t)(t - 1) * count0 + e];
            const int a = pos1[t][q], z = pos1[t][q + 1];
            start[(int64_t)t * stride + before] = a;
            len[(int64_t)t * (stride + 1) + before] = z - a;
        }
    }
    __device__ void finish(int, int total) const { head[0] = total; }
};

// Rows of the remapped result that hold an entry (the first head[0] rows exist)
struct KeepIn {
    const int32_t *pos_full;
    const int32_t *head;
    __device__ int load(int, int64_t i) const { return i < head[0] && pos_full[i + 1] > pos_full[i] ? 1 : 0; }
};

struct CompactOut {
    const int32_t *rows, *pos_full;
    const int64_t *counts_in;      // {rows, nnz} of the remapped result
    SpaddOut out;
    __device__ void store(int, int64_t i, int before, int keep) const
    {
        if (keep && before < out.cap_rows) {
            out.crd0[before] = rows[i];
            out.pos1[before] = pos_full[i];
        }
    }
    __device__ void finish(int, int total) const
    {
        const int64_t nnz = counts_in[1];
        out.pos0[0] = 0;
        out.pos0[1] = total;
        if (total <= out.cap_rows) out.pos1[total] = (int32_t)nnz;
        else *out.status = NACHO_ERR_CAPACITY;
        out.counts[0] = total;
        out.counts[1] = nnz;
    }
};

// What the kernels after the row loop need to know, left where they can read it: the number of
// partitions of the remapped nest (the rule of the fused calls: enough partitions that one fits a
// workgroup, a whole number of rounds of resident workgroups, at least what the caller asked for),
// the number of intersected rows and the remapped total cost.
__global__ void remap_plan_kernel(const int32_t *__restrict__ head, int k, int64_t capacity, int64_t round,
                                  int64_t P_min, int64_t P_max, int64_t *__restrict__ plan)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    int64_t total = 0;
    for (int t = 0; t < k; ++t) total += head[1 + t];
    int64_t need = total > 0 ? (total + capacity - 1) / capacity : 1;
    if (P_min == 0 && need > round) need = (need + round - 1) / round * round;
    int64_t P = P_min > need ? P_min : need;
    if (P > P_max) P = P_max;
    plan[0] = P;
    plan[1] = head[0];
    plan[2] = total;
}

__global__ void empty_result_kernel(SpaddOut out, int64_t *info)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        out.pos0[0] = 0;
        out.pos0[1] = 0;
        out.pos1[0] = 0;
        out.counts[0] = 0;
        out.counts[1] = 0;
        *out.status = NACHO_OK;
        info[0] = info[1] = info[2] = 0;
    }
}

int64_t tiles_of(int64_t n) { return n > 0 ? (n + kScanTile - 1) / kScanTile : 1; }

template <class In, class Out>
hipError_t scan(const In &in, const Out &out, int64_t n, int batch, int32_t *tsum, hipStream_t s)
{
    const int64_t n_tiles = tiles_of(n);
    const dim3 grid((unsigned)n_tiles, (unsigned)batch);
    hipLaunchKernelGGL((scan_sums_kernel<In>), grid, dim3(kScanThreads), 0, s, in, n, n_tiles, tsum);
    hipLaunchKernelGGL((scan_apply_kernel<In, Out>), grid, dim3(kScanThreads), 0, s, in, out, n, n_tiles, tsum);
    return hipGetLastError();
}

}  // namespace

int64_t remap_scan_words(int64_t n, int batch) { return tiles_of(n) * batch; }

hipError_t launch_rows_match(const DevOperands &ops, int64_t P0, const int32_t *posn0, int32_t *flags,
                             int32_t *qpos, hipStream_t s)
{
    RowArrays rows;
    rows.k = ops.k;
    for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) rows.crd0[t] = t < ops.k ? ops.lvl[t][0].crd : nullptr;
    hipLaunchKernelGGL(rows_match_kernel, dim3((unsigned)P0), dim3(256), 0, s, rows, posn0, flags, qpos,
                       ops.lvl[0][0].count);
    return hipGetLastError();
}

hipError_t launch_remap_rows(const DevOperands &ops, const int32_t *flags, const int32_t *qpos,
                             const RemapArrays &r, int32_t *tsum, hipStream_t s)
{
    ArrayIn in;
    in.base = flags;
    in.stride = 0;
    RemapOut out;
    out.k = ops.k;
    out.crd0_0 = ops.lvl[0][0].crd;
    out.qpos = qpos;
    out.count0 = ops.lvl[0][0].count;
    for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) out.pos1[t] = t < ops.k ? ops.lvl[t][1].pos : nullptr;
    out.rows = r.rows;
    out.start = r.start;
    out.len = r.cost;
    out.stride = r.stride;
    out.head = r.head;
    return scan(in, out, ops.lvl[0][0].count, 1, tsum, s);
}

hipError_t launch_remap_costs(int k, const RemapArrays &r, int32_t *tsum, hipStream_t s)
{
    ArrayIn in;
    in.base = r.cost;
    in.stride = r.stride + 1;
    CostOut out;
    out.base = r.cost;
    out.stride = r.stride + 1;
    out.n = r.stride;
    out.head = r.head;
    return scan(in, out, r.stride, k, tsum, s);
}

hipError_t launch_compact_rows(const RemapArrays &r, const int32_t *pos_full,
                               const int64_t *counts_in, const SpaddOut &out, int32_t *tsum, hipStream_t s)
{
    KeepIn in;
    in.pos_full = pos_full;
    in.head = r.head;
    CompactOut o;
    o.rows = r.rows;
    o.pos_full = pos_full;
    o.counts_in = counts_in;
    o.out = out;
    return scan(in, o, r.stride, 1, tsum, s);       // (over the upper bound of the rows; those past head[0] count as empty)
}

hipError_t launch_remap_plan(int k, const RemapArrays &r, int64_t capacity, int64_t round, int64_t P_min,
                             int64_t P_max, int64_t *plan, hipStream_t s)
{
    hipLaunchKernelGGL(remap_plan_kernel, dim3(1), dim3(64), 0, s, r.head, k, capacity, round, P_min, P_max, plan);
    return hipGetLastError();
}

hipError_t launch_empty_result(const SpaddOut &out, int64_t *info, hipStream_t s)
{
    hipLaunchKernelGGL(empty_result_kernel, dim3(1), dim3(64), 0, s, out, info);
    return hipGetLastError();
}

}  // namespace nacho
