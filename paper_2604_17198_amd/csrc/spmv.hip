// SpMV execution: one wavefront per partition (the compute kernel of Section
// 4.4 with loop bounds taken from the stored partitions), plus the carry
// fix-up for rows split across partitions.
//
// Partition p owns the stored non-zeros at positions [n_p, n_{p+1}) of A.  Its
// wavefront
//   1. streams crd/val of that range (read once: non-temporal loads, so that
//      the L2 is left to x), gathers x and leaves the products in LDS;
//   2. walks the rows that overlap the range (their pos entries staged in LDS),
//      one lane per row; rows with many products are summed by the whole
//      wavefront instead;
//   3. stores y[r] for every row that STARTS inside the partition (a row that
//      ends later gets its first piece here), and hands the piece of the one
//      row that started earlier to the fix-up pass as a carry.
// The fix-up pass adds the carries of a row, in a fixed order, to y[r].  There
// are no floating-point atomics anywhere: results repeat bit for bit.
#include <type_traits>

#include "common.hpp"
#include "kernels.hpp"

namespace nacho {

namespace {

constexpr int kLongRow = 192;  // products per row above which the wavefront sums it together

// kDealt: the partitions come from fixed-grain queries (grain > 0) and are dealt out by XCD; the
// instantiation without it serves arbitrary partition tables (caller's P, the row-aware cost).
// kFused (with kDealt): there is no partition table; the wavefront finds its own two boundaries, the
// search of Algorithm 1 for one CSR operand (Section 4.2.2: the row with pos[r] <= Q < pos[r + 1], at
// position Q) with the fixed-grain queries Q_b = min(b * grain, nnz), as a 64-ary search over pos.
template <typename T, int G, int RBLK, bool kDealt, bool kFused = false>
__global__ void __launch_bounds__(NACHO_WAVE)
spmv_exec_kernel(const int32_t *__restrict__ pos, const int32_t *__restrict__ crd,
                 const T *__restrict__ val, const T *__restrict__ x, T *__restrict__ y,
                 int nnz, const int32_t *__restrict__ coord, const int32_t *__restrict__ posn,
                 T *__restrict__ carry_val, int32_t *__restrict__ carry_row, int n_rows, int grain, WaveLog wlog)
{
    const WaveStamp stamp = wave_begin();
    __shared__ T prod[G + 8];
    __shared__ int32_t spos[RBLK + 1];

    const int lane = threadIdx.x;
    // Which partition this workgroup executes.  Workgroups are handed to the 8
    // XCDs in turn (workgroup w runs on XCD w mod 8) and every XCD has its own
    // L2, which x does not fit.  The partitions that lie inside one long row are
    // therefore dealt out so that XCD j gets the j-th eighth of the row, in
    // ascending order: its gathers then stay inside one eighth of x (columns
    // are sorted inside a row), which its L2 holds.  With fixed-grain queries
    // the partitions inside row r are first = ceil(pos[r] / grain) .. end - 1 =
    // floor(pos[r+1] / grain) - 1.  Among the workgroups first .. end - 1 those
    // with index = j (mod 8) take, in order, the j-th stretch of these
    // partitions (stretches as long as there are such workgroups): a
    // permutation of first .. end - 1; everything else keeps its index.
    int p = blockIdx.x;
    // (fused search) boundary b: its row and its position
    auto boundary = [&](int b, int from, int &r, int &n) {
        const long long Q = (long long)b * grain;
        if (b == 0) { r = 0; n = pos[0]; }
        else if (Q >= nnz) { r = n_rows; n = pos[0] + nnz; }
        else {
            n = pos[0] + (int)Q;
            r = pos[from + 1] > n ? from : first_row_past(pos, from, n_rows, n);
        }
    };
    int r_own = 0, n_own = 0;
    if (kFused) boundary(p, 0, r_own, n_own);
    if (kDealt) {
        const int r = kFused ? r_own : coord[2 * p];
        if (r < n_rows) {
            const int base = pos[0];
            const int first = ((pos[r] - base) + grain - 1) / grain;
            const int end = (pos[r + 1] - base) / grain;
            if (end - first >= 4 && p >= first && p < end) {
                const int j = p & 7;
                int before = 0, mine = 0;              // partitions of the stretches before stretch j; first workgroup of j
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) {
                    const int f = first + ((jj - first) & 7);      // first workgroup >= first with index = jj (mod 8)
                    const int cnt = f < end ? (end - f + 7) >> 3 : 0;
                    if (jj < j) before += cnt;
                    if (jj == j) mine = f;
                }
                p = first + before + ((p - mine) >> 3);
            }
        }
    }
    // k = 1, d = 2: coord[b*2 + 0] = row, posn[b*2 + 1] = position in crd/val
    int r0, r1, n0, n1;
    if (kFused) {
        // (a dealt partition lies in the row of the one it was dealt for)
        if (p == (int)blockIdx.x) { r0 = r_own; n0 = n_own; }
        else boundary(p, r_own < n_rows ? r_own : 0, r0, n0);
        boundary(p + 1, r0 < n_rows ? r0 : 0, r1, n1);
    } else {
        r0 = coord[2 * p]; r1 = coord[2 * p + 2];
        n0 = posn[2 * p + 1]; n1 = posn[2 * p + 3];
    }
    const int pr0 = pos[r0], pr1 = pos[r1];
    const bool has_head = n0 > pr0;                    // row r0 started in an earlier partition
    const int next_first = (n1 > pr1) ? r1 + 1 : r1;   // first row that starts after this partition
    const int nrows = next_first - r0;                 // rows overlapping or starting here
    const int a0 = n0;                                 // prod[i] belongs to position a0 + i
    // pos entries of the first row block, requested before the streamed data
    int nr = nrows < RBLK ? nrows : RBLK;
    if (nrows > 0)
        for (int i = lane; i <= nr; i += NACHO_WAVE) spos[i] = pos[r0 + i];

    // Lane l takes positions n0 + l, n0 + 64 + l, ...: consecutive lanes hold
    // consecutive non-zeros, so inside a dense row the 64 gathers of one
    // instruction fall into few cache lines of x (columns are sorted).  All
    // streamed loads are issued before the first gather, all gathers before the
    // first LDS store, so one wavefront keeps its whole window in flight.
    constexpr int kIter = G / NACHO_WAVE;
    int c[kIter];
    T v[kIter];
#pragma unroll
    for (int j = 0; j < kIter; ++j) {
        const int idx = n0 + j * NACHO_WAVE + lane;
        c[j] = 0;
        v[j] = T(0);
        if (idx < n1) {
            c[j] = __builtin_nontemporal_load(crd + idx);
            v[j] = __builtin_nontemporal_load(val + idx);
        }
    }
    T xv[kIter];
#pragma unroll
    for (int j = 0; j < kIter; ++j) {
        const int idx = n0 + j * NACHO_WAVE + lane;
        xv[j] = idx < n1 ? x[c[j]] : T(0);
    }
#pragma unroll
    for (int j = 0; j < kIter; ++j) {
        const int idx = n0 + j * NACHO_WAVE + lane;
        if (idx < n1) prod[idx - a0] = v[j] * xv[j];
    }
    __syncthreads();

    for (int rb = 0; rb < nrows; rb += RBLK) {
        if (rb > 0) {
            nr = nrows - rb < RBLK ? nrows - rb : RBLK;
            __syncthreads();
            for (int i = lane; i <= nr; i += NACHO_WAVE) spos[i] = pos[r0 + rb + i];
            __syncthreads();
            // A block of rows without entries: empty rows are zero already (the partition
            // kernel wrote them), so the wavefront steps over them, however many there are.
            const int q = spos[0];
            if (q == spos[nr]) {
                if (q >= n1) break;                     // every product of the partition is summed
                rb = first_row_past(pos, r0 + rb + nr, r0 + nrows, q) - r0 - RBLK;
                continue;
            }
        }
        for (int rr0 = 0; rr0 < nr; rr0 += NACHO_WAVE) {
            const int rr = rr0 + lane;
            const bool valid = rr < nr;
            const int a = valid ? spos[rr] : 0;
            const int b = valid ? spos[rr + 1] : 0;
            const int lo = (a > n0 ? a : n0) - a0;
            const int hi = (b < n1 ? b : n1) - a0;
            const int len = valid && hi > lo ? hi - lo : 0;
            T sum = T(0);
            if (len < kLongRow)
                for (int i = lo; i < lo + len; ++i) sum += prod[i];
            unsigned long long heavy = __ballot(len >= kLongRow);
            while (heavy) {
                const int L = __ffsll((long long)heavy) - 1;
                heavy &= heavy - 1;
                const int llo = __shfl(lo, L, NACHO_WAVE), lhi = __shfl(hi, L, NACHO_WAVE);
                T s = T(0);
                for (int i = llo + lane; i < lhi; i += NACHO_WAVE) s += prod[i];
                s = wave_sum(s);
                if (lane == L) sum = s;
            }
            if (valid) {
                const int r = r0 + rb + rr;
                if (has_head && r == r0) carry_val[p] = sum;
                else y[r] = sum;
            }
        }
    }
    if (lane == 0) carry_row[p] = has_head ? r0 : -1;
    wave_end(wlog, blockIdx.x, stamp, (uint32_t)(n1 - n0), (uint32_t)nrows);
}

// Carry fix-up, one lane per partition.  The carries of a row sit in
// consecutive partitions; the wavefront that holds the first carry of a row adds
// the whole run to y[row]: a segmented sum over its own 64 lanes, plus a walk
// over the following partitions when the run goes on past the wavefront's last
// lane.  One writer per row and a fixed order of additions.
template <typename T>
__global__ void __launch_bounds__(256)
spmv_fixup_kernel(T *__restrict__ y, int P, const T *__restrict__ carry_val,
                  const int32_t *__restrict__ carry_row, const int32_t *__restrict__ pos, int grain)
{
    const int p = (int)((int64_t)blockIdx.x * blockDim.x + threadIdx.x);
    const int lane = lane_id();
    const int p_first = p - lane;                      // partition of lane 0
    if (p_first >= P) return;                          // whole wavefront leaves together
    const int r = p < P ? carry_row[p] : -1;
    T v = r >= 0 ? carry_val[p] : T(0);
    int before = __shfl_up(r, 1, NACHO_WAVE);
    if (lane == 0) before = p_first > 0 ? carry_row[p_first - 1] : -1;
    const bool head = r >= 0 && r != before;           // first carry of its row
    const bool first_here = r != before || lane == 0;  // first lane of its segment in this wavefront
    const unsigned long long starts = __ballot(first_here);
    const unsigned long long upto = lane == NACHO_WAVE - 1 ? ~0ull : ((2ull << lane) - 1ull);
    const int start = 63 - __clzll((long long)(starts & upto));
    const unsigned long long after = starts & ~upto;
    const int end = after ? __ffsll((long long)after) - 2 : NACHO_WAVE - 1;   // last lane of the segment
    // inclusive sum inside the segment
#pragma unroll
    for (int o = 1; o < NACHO_WAVE; o <<= 1) {
        const T left = __shfl_up(v, o, NACHO_WAVE);
        if (lane - o >= start) v += left;
    }
    const bool owned = __shfl((int)head, start, NACHO_WAVE) != 0;   // the run starts in this wavefront
    // a run that reaches the last lane may go on in the next wavefronts
    const int r_last = __shfl(r, NACHO_WAVE - 1, NACHO_WAVE);
    const bool last_owned = __shfl((int)owned, NACHO_WAVE - 1, NACHO_WAVE) != 0;
    // (the writer's element of y is requested now, beside the loads of the tail)
    const bool writer = r >= 0 && owned && lane == end;
    const T y_old = writer ? y[r] : T(0);
    T tail = T(0);
    if (r_last >= 0 && last_owned && grain > 0) {
        // fixed-grain partitions: the carries of row r come from the partitions that
        // start strictly inside it, floor(pos[r] / grain) + 1 .. ceil(pos[r+1] / grain) - 1,
        // so the rest of the run is known without looking: independent loads, eight
        // chunks of 64 in flight, added in a fixed order
        const int base = pos[0];
        int last = ((pos[r_last + 1] - base) + grain - 1) / grain - 1;
        if (last > P - 1) last = P - 1;
        T acc[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc[u] = T(0);
        for (int q0 = p_first + NACHO_WAVE; q0 <= last; q0 += 8 * NACHO_WAVE) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int q = q0 + u * NACHO_WAVE + lane;
                if (q <= last) acc[u] += carry_val[q];
            }
        }
        tail = wave_sum(((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7])));
    } else if (r_last >= 0 && last_owned) {
        // chunks of 64 partitions, loaded in batches: two chunks first (most runs end
        // there), then sixteen at a time (a row of a million non-zeros has thousands of
        // carries; every batch is one round trip)
        int e = p_first + NACHO_WAVE;
        bool more = true;
        auto walk = [&](auto batch_tag) {
            constexpr int kBatch = decltype(batch_tag)::value;
            int rr[kBatch];
            T vv[kBatch];
#pragma unroll
            for (int c = 0; c < kBatch; ++c) {
                const int q = e + c * NACHO_WAVE + lane;
                rr[c] = q < P ? carry_row[q] : -1;
                vv[c] = q < P ? carry_val[q] : T(0);
            }
#pragma unroll
            for (int c = 0; c < kBatch; ++c) {
                if (!more) break;
                const unsigned long long m = __ballot(rr[c] == r_last);
                const int cnt = m == ~0ull ? NACHO_WAVE : __ffsll((long long)~m) - 1;   // leading lanes of the run
                tail += wave_sum(lane < cnt ? vv[c] : T(0));
                more = cnt == NACHO_WAVE;
            }
            e += kBatch * NACHO_WAVE;
        };
        walk(std::integral_constant<int, 2>());
        while (more) walk(std::integral_constant<int, 16>());
    }
    if (writer) y[r] = y_old + (v + (end == NACHO_WAVE - 1 ? tail : T(0)));
}

constexpr int kGrainF64 = 512, kRowsF64 = 512;
constexpr int kGrainF32 = 1024, kRowsF32 = 1024;

}  // namespace

int spmv_capacity(int dtype) { return dtype == NACHO_F64 ? kGrainF64 : kGrainF32; }

hipError_t launch_spmv_exec(int dtype, const int32_t *pos, const int32_t *crd, const void *val,
                            const void *x, void *y, int64_t n_rows, int64_t nnz,
                            const int32_t *coord, const int32_t *posn, int64_t P,
                            void *carry_val, int32_t *carry_row, int64_t grain, hipStream_t stream)
{
#define NACHO_SPMV_LAUNCH(T, G, R, DEALT, FUSED)                                                        \
    hipLaunchKernelGGL((spmv_exec_kernel<T, G, R, DEALT, FUSED>), dim3((unsigned)P), dim3(NACHO_WAVE), 0, stream, \
                       pos, crd, (const T *)val, (const T *)x, (T *)y, (int)nnz, coord, posn, (T *)carry_val,    \
                       carry_row, (int)n_rows, (int)grain, nacho_host::wave_log())
    const bool fused = grain > 0 && coord == nullptr;       // no table: the wavefronts search their boundaries
    if (dtype == NACHO_F64) {
        if (fused) NACHO_SPMV_LAUNCH(double, kGrainF64, kRowsF64, true, true);
        else if (grain > 0) NACHO_SPMV_LAUNCH(double, kGrainF64, kRowsF64, true, false);
        else NACHO_SPMV_LAUNCH(double, kGrainF64, kRowsF64, false, false);
    } else {
        if (fused) NACHO_SPMV_LAUNCH(float, kGrainF32, kRowsF32, true, true);
        else if (grain > 0) NACHO_SPMV_LAUNCH(float, kGrainF32, kRowsF32, true, false);
        else NACHO_SPMV_LAUNCH(float, kGrainF32, kRowsF32, false, false);
    }
#undef NACHO_SPMV_LAUNCH
    return hipGetLastError();
}

namespace {
__global__ void __launch_bounds__(256) zero_words_kernel(uint32_t *__restrict__ dst, int64_t n_words)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += (int64_t)gridDim.x * blockDim.x)
        dst[i] = 0u;
}
}  // namespace

// y = 0 (the fused form has no partition kernel to write the zeros of the rows A stores nothing in)
hipError_t launch_zero_vector(int dtype, void *y, int64_t n, hipStream_t stream)
{
    const int64_t words = n * (dtype == NACHO_F64 ? 2 : 1);
    if (words == 0) return hipSuccess;
    int64_t blocks = (words + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (uint32_t *)y, words);
    return hipGetLastError();
}

hipError_t launch_spmv_fixup(int dtype, void *y, int64_t P, const void *carry_val,
                             const int32_t *carry_row, const int32_t *pos, int64_t grain, hipStream_t stream)
{
    const unsigned grid = (unsigned)((P + 255) / 256);
    if (dtype == NACHO_F64)
        hipLaunchKernelGGL((spmv_fixup_kernel<double>), dim3(grid), dim3(256), 0, stream,
                           (double *)y, (int)P, (const double *)carry_val, carry_row, pos, (int)grain);
    else
        hipLaunchKernelGGL((spmv_fixup_kernel<float>), dim3(grid), dim3(256), 0, stream,
                           (float *)y, (int)P, (const float *)carry_val, carry_row, pos, (int)grain);
    return hipGetLastError();
}

}  // namespace nacho
