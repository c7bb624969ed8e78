// Partition kernel: one wavefront runs one boundary search (Section 3.2,
// Algorithm 1) with the non-zero-count cost of Section 4.2.2, in position
// space with tracked search windows (Section 4.2.3).
//
// What differs from the paper's per-thread nested binary search (an outer
// search over coordinates, one inner search per operand per probe): the chain
// of dependent memory accesses is what a boundary costs on this machine, so the
// 64 lanes of a wavefront shorten it.
//   * Dense level (rows of CSR): a 64-ary search, 64 candidate coordinates per
//     round, ceil(log64(N+1)) rounds, one pos load per operand and round.
//   * Compressed level: every round each operand's current window is sampled at
//     64 evenly spaced positions (one load per lane and operand).  A sample's
//     own position is its exact lower bound in its operand; in the other
//     operands its lower bound is bracketed by the two neighbouring samples.
//     That gives a lower and an upper bound of the cost of every sampled
//     coordinate; samples whose upper bound is <= the residual query are not
//     after the boundary, samples whose lower bound exceeds it are after it, and
//     every window shrinks to the bracket of the largest / smallest such sample.
//     Once every window holds <= 64 entries the bounds are exact and the round
//     returns the boundary.  A boundary over 10M + 1M + 100k entries takes about
//     seven rounds, i.e. seven dependent loads instead of several hundred.
//     (With five to eight operands the K * K rank searches per round outgrow the
//     registers and the instruction cache; those calls use the 64-ary search over
//     coordinates with one lower-bound search per operand and probe, inside
//     tracked windows, throughout.)
//   * Coordinate lists (COO): both levels are searched as one level of (row,
//     column) pairs with 64-bit coordinates.
//   * One CSR operand (SpMV, SpMM): no search at all, see partition_csr1_kernel.
// The result is the coordinate and the positions the serial search returns: the
// highest coordinate whose cost does not exceed the residual query (it is then
// a stored coordinate), and for every operand the position of its first entry
// that is not before that coordinate.
#include "common.hpp"
#include "kernels.hpp"
#include "search.hpp"

namespace nacho {

namespace {

// Words of the call's later kernels that the partition kernel clears on the side
// (it is the first kernel of every fused call): thread i clears word i.
struct ClearWords {
    unsigned long long *words;
    int64_t n;
    int32_t *status;
    __device__ void run(int64_t i) const
    {
        if (i < n) words[i] = 0ull;
        if (i == 0 && status) *status = NACHO_OK;
    }
};

}  // namespace

// (declared in kernels.hpp) rows of a dense result that the one-pass CSR kernel sets to zero
// because the operand stores nothing in them
__device__ inline void zero_row(const ZeroRows &z, int64_t r, int lane_in_row, int lanes)
{
    char *row = static_cast<char *>(z.base) + r * z.ld * z.elem;
    for (int c = lane_in_row; c < z.width; c += lanes) {
        if (z.elem == 8) reinterpret_cast<double *>(row)[c] = 0.0;
        else reinterpret_cast<float *>(row)[c] = 0.0f;
    }
}

// One wavefront searches one boundary.
// kMode: 0 = vectors, CSR, DCSR; 1 = coordinate lists; 2 = three compressed levels (CSF).  The
// last two are instantiations of their own: the other formats keep their register budget.
template <int K, int kMode>
__global__ void __launch_bounds__(256)
partition_kernel(DevOperands ops, int64_t cost_scale, int64_t P, int64_t grain,
                 const int64_t *__restrict__ queries, int64_t total_unscaled,
                 int32_t *__restrict__ coord, int32_t *__restrict__ posn, int64_t *__restrict__ cost,
                 ClearWords clear)
{
    clear.run((int64_t)blockIdx.x * blockDim.x + threadIdx.x);
    if (ops.dyn_plan) {                      // sizes left on the device by earlier kernels of the call
        P = ops.dyn_plan[0];
        total_unscaled = ops.dyn_plan[2];
    }
    const int64_t b = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / NACHO_WAVE;
    if (b > P) return;                       // whole wavefront leaves together
    int found[K];
    search_boundary<K, kMode>(ops, cost_scale, P, grain, queries, total_unscaled, coord, posn, cost, b, found);
}

// ---- one CSR operand: all boundaries in one pass over the rows ---------------
// With a single operand the search of Algorithm 1 has a closed form (the CSR
// cost functions of Section 4.2.2): boundary b lies in the row r with
// pos[r] <= Q_b < pos[r+1], at position Q_b.  Instead of P searches over pos,
// every row finds the boundaries that fall inside it: the queries are a
// monotone function of b with a cheap inverse, so row r owns the boundaries
// b_first(pos[r]) .. b_first(pos[r+1]) - 1, where b_first(y) is the first
// boundary whose query reaches y.  One coalesced pass over pos, no dependent
// loads; a row with many boundaries is written by its whole wavefront.
namespace {

// Built-in queries in unscaled units.  grain_u > 0: Q_b = min(b * grain_u, total);
// grain_u == 0: Q_b = floor(b * total / P).
struct QueryRule {
    int64_t P, total, grain_u;
    __device__ int64_t query(int64_t b) const
    {
        if (grain_u > 0) { const int64_t q = b * grain_u; return q < total ? q : total; }
        return equal_query(b, total, P);
    }
    // least b in [0, P] whose query is >= y, for 0 <= y <= total
    __device__ int64_t first_reaching(int64_t y) const
    {
        int64_t b;
        if (grain_u > 0 && (grain_u & (grain_u - 1)) == 0)           // a power of two (the built-in grains are)
            b = (y + grain_u - 1) >> (63 - __clzll((long long)grain_u));
        else if (grain_u > 0 && grain_u < 0x7fffffffLL && y < 0x7fffffffLL)
            b = ((uint32_t)y + (uint32_t)grain_u - 1u) / (uint32_t)grain_u;
        else if (grain_u > 0) b = (y + grain_u - 1) / grain_u;
        else if (total <= 0) b = 0;
        else if (total < 0x7fffffffLL && P < 0x7fffffffLL)          // (the product fits 64 bits: no 128-bit division)
            b = (int64_t)(((uint64_t)y * (uint64_t)P + (uint64_t)total - 1u) / (uint64_t)total);
        else b = (int64_t)(((__int128)y * P + total - 1) / total);
        return b < P ? b : P;
    }
};

// row_cost > 0: the row-aware variant of the cost (Section 4.2.2 remarks that the non-zero count only
// approximates the run time): every row costs row_cost units on top of its stored non-zeros,
// charged in front of its first column, C_i(r) = pos[r] + row_cost * r.  Row r then owns the queries in
// [C_i(r), C_i(r + 1)) -- empty rows own some too -- and a boundary with R = Q - C_i(r) left lies at the
// row's start when R < row_cost, else at the entry of rank R - row_cost (an entry in column 0 shares
// the coordinate of the row's own units: the boundary's cost is then C_i(r)).
// PosT: type of the operand's positions and of the stored ones (int64_t: operands of 2^31 entries or more).
template <typename PosT>
__global__ void __launch_bounds__(256)
partition_csr1_kernel(const PosT *__restrict__ pos, const int32_t *__restrict__ crd, int64_t n_rows,
                      int64_t count, QueryRule rule, int64_t cost_scale, int64_t row_cost,
                      int32_t *__restrict__ coord,
                      PosT *__restrict__ posn, int64_t *__restrict__ cost, ClearWords clear, ZeroRows zero)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    clear.run(i);
    const int lane = lane_id();
    const int64_t P = rule.P;
    const PosT p0 = pos[0];
    // As boundary i: everything that does not depend on the row.  Boundaries that
    // are not searched (the origin, the end, queries that reach past the work) are
    // complete here.
    if (i <= P) {
        const int64_t q = rule.query(i);
        if (i == 0 || i == P || q >= rule.total) {
            const bool end = i != 0;
            coord[i * 2 + 0] = end ? (int32_t)n_rows : 0;
            coord[i * 2 + 1] = 0;
            posn[i * 2 + 0] = end ? (PosT)n_rows : 0;
            posn[i * 2 + 1] = end ? (PosT)count : 0;
            cost[i] = end ? rule.total * cost_scale : 0;
        } else if (row_cost == 0) {
            coord[i * 2 + 1] = crd[p0 + q];
            posn[i * 2 + 1] = (PosT)(p0 + q);
            cost[i] = q * cost_scale;
        }
    }
    // As row i: the row fields of the boundaries that fall inside it.
    int64_t b_lo = 0, b_hi = 0;
    bool empty_row = false;
    if (i < n_rows) {
        const int64_t a = (int64_t)(pos[i] - p0) + row_cost * i, e = (int64_t)(pos[i + 1] - p0) + row_cost * (i + 1);
        empty_row = pos[i + 1] == pos[i];
        if (e > a) {
            b_lo = rule.first_reaching(a);
            b_hi = rule.first_reaching(e);
            if (b_lo < 1) b_lo = 1;                 // boundary 0 is the origin by definition
            // (b < b_hi means Q_b < C_i(r + 1) <= total and b < P: interior)
        }
    }
    // row r writes the row fields of boundary b
    auto write_boundary = [&](int64_t b, int32_t r) {
        coord[b * 2 + 0] = r;
        posn[b * 2 + 0] = r;
        if (row_cost > 0) {
            const int64_t start = (int64_t)(pos[r] - p0) + row_cost * r;      // C_i(r)
            const int64_t Q = rule.query(b), R = Q - start;
            PosT at = pos[r];
            int32_t x1 = 0;
            if (R >= row_cost) {
                at += (PosT)(R - row_cost);
                x1 = crd[at];
            }
            coord[b * 2 + 1] = x1;
            posn[b * 2 + 1] = at;
            cost[b] = (x1 > 0 ? Q : start) * cost_scale;
        }
    };
    // a row with a few boundaries writes them itself (all rows of the wavefront at once); a row with
    // many is written by its whole wavefront
    constexpr int kFew = 4;
    const int64_t mine = b_hi - b_lo;
    if (mine > 0 && mine <= kFew)
        for (int64_t b = b_lo; b < b_hi; ++b) write_boundary(b, (int32_t)i);
    unsigned long long todo = __ballot(mine > kFew);
    while (todo) {
        const int src = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        const int64_t lo = __shfl((long long)b_lo, src, NACHO_WAVE);
        const int64_t hi = __shfl((long long)b_hi, src, NACHO_WAVE);
        const int32_t r = (int32_t)(i - lane + src);
        for (int64_t b = lo + lane; b < hi; b += NACHO_WAVE) write_boundary(b, r);
    }
    // Rows without entries: their row of the result is zero, and the executing
    // wavefronts may then step over them however many there are.
    if (zero.base) {
        if (zero.width == 1) {
            if (empty_row) zero_row(zero, i, 0, 1);
        } else {
            unsigned long long left = __ballot(empty_row);
            while (left) {
                const int src = __ffsll((long long)left) - 1;
                left &= left - 1;
                zero_row(zero, i - lane + src, lane, NACHO_WAVE);
            }
        }
    }
}

}  // namespace

// One CSR operand whose positions are 64-bit: the same one-pass kernel, equal-share queries.
hipError_t launch_partition_csr64(const int64_t *pos, const int32_t *crd, int64_t n_rows, int64_t nnz, int64_t P,
                                  int32_t *coord, int64_t *posn, int64_t *cost, hipStream_t stream)
{
    ClearWords clear;
    clear.words = nullptr;
    clear.n = 0;
    clear.status = nullptr;
    ZeroRows zero;
    zero.base = nullptr;
    zero.ld = 0;
    zero.width = zero.elem = 0;
    QueryRule rule;
    rule.P = P;
    rule.total = nnz;
    rule.grain_u = 0;
    const int64_t threads = n_rows > P + 1 ? n_rows : P + 1;
    hipLaunchKernelGGL(partition_csr1_kernel<int64_t>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream,
                       pos, crd, n_rows, nnz, rule, (int64_t)1, (int64_t)0, coord, posn, cost, clear, zero);
    return hipGetLastError();
}

hipError_t launch_partition(const DevOperands &ops, int64_t cost_scale, int64_t P, int64_t grain,
                            const int64_t *queries, int64_t total_unscaled,
                            int32_t *coord, int32_t *posn, int64_t *cost, hipStream_t stream,
                            unsigned long long *clear_words, int64_t n_clear, int32_t *clear_status,
                            const ZeroRows *zero_rows, int64_t row_cost)
{
    ClearWords clear;
    clear.words = clear_words;
    clear.n = clear_words ? n_clear : 0;
    clear.status = clear_status;
    ZeroRows zero;
    zero.base = nullptr;
    zero.ld = 0;
    zero.width = zero.elem = 0;
    if (zero_rows) zero = *zero_rows;
    if (ops.k == 1 && ops.d == 2 && ops.lvl[0][0].kind == NACHO_DENSE && !queries && !ops.start[0] &&
        (grain == 0 || grain % cost_scale == 0)) {
        QueryRule rule;
        rule.P = P;
        rule.total = total_unscaled + row_cost * ops.lvl[0][0].extent;
        rule.grain_u = grain / cost_scale;
        const int64_t n_rows = ops.lvl[0][0].extent;
        int64_t threads = n_rows > P + 1 ? n_rows : P + 1;
        if (clear.n > threads) threads = clear.n;
        hipLaunchKernelGGL(partition_csr1_kernel<int32_t>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream,
                           ops.lvl[0][1].pos, ops.lvl[0][1].crd, n_rows, ops.lvl[0][1].count, rule, cost_scale,
                           row_cost, coord, posn, cost, clear, zero);
        return hipGetLastError();
    }
    if (zero_rows || row_cost != 0) return hipErrorInvalidValue;      // only the one-pass kernel above does these
    int64_t waves = P + 1;
    if (clear.n > waves * NACHO_WAVE) waves = (clear.n + NACHO_WAVE - 1) / NACHO_WAVE;
    const int waves_per_block = 256 / NACHO_WAVE;
    const unsigned grid = (unsigned)((waves + waves_per_block - 1) / waves_per_block);
    // instantiated for 1, 2, 3, 4 and 8 operands so that small calls keep their state in registers
    if (ops.d == 3) {
        if (ops.k <= 2)
            hipLaunchKernelGGL((partition_kernel<2, 2>), dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                               queries, total_unscaled, coord, posn, cost, clear);
        else if (ops.k <= 4)
            hipLaunchKernelGGL((partition_kernel<4, 2>), dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                               queries, total_unscaled, coord, posn, cost, clear);
        else
            hipLaunchKernelGGL((partition_kernel<8, 2>), dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                               queries, total_unscaled, coord, posn, cost, clear);
        return hipGetLastError();
    }
    if (ops.lvl[0][0].kind == NACHO_NONUNIQUE) {
        if (ops.k <= 2)
            hipLaunchKernelGGL((partition_kernel<2, 1>), dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                               queries, total_unscaled, coord, posn, cost, clear);
        else if (ops.k <= 4)
            hipLaunchKernelGGL((partition_kernel<4, 1>), dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                               queries, total_unscaled, coord, posn, cost, clear);
        else
            hipLaunchKernelGGL((partition_kernel<8, 1>), dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                               queries, total_unscaled, coord, posn, cost, clear);
        return hipGetLastError();
    }
    if (ops.k <= 1)
        hipLaunchKernelGGL((partition_kernel<1, 0>), dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                           queries, total_unscaled, coord, posn, cost, clear);
    else if (ops.k <= 2)
        hipLaunchKernelGGL((partition_kernel<2, 0>), dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                           queries, total_unscaled, coord, posn, cost, clear);
    else if (ops.k <= 3)
        hipLaunchKernelGGL((partition_kernel<3, 0>), dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                           queries, total_unscaled, coord, posn, cost, clear);
    else if (ops.k <= 4)
        hipLaunchKernelGGL((partition_kernel<4, 0>), dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                           queries, total_unscaled, coord, posn, cost, clear);
    else
        hipLaunchKernelGGL((partition_kernel<8, 0>), dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                           queries, total_unscaled, coord, posn, cost, clear);
    return hipGetLastError();
}

}  // namespace nacho
