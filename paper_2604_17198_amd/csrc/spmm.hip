// SpMM execution, C = A B with A in CSR and B, C dense row-major: one wavefront
// per partition, one lane per column of B (n <= 64), loop order i -> j -> k with
// the dense k innermost (the broadcast rule of Section 4.2.2 scales the cost of
// every stored non-zero by n, so the partitions are those of SpMV).
//
// The wavefront stages its partition's crd/val and the pos entries of its rows
// in LDS, then streams over the non-zeros sixteen at a time: sixteen rows of B are
// requested (one 4n-byte coalesced load each) before the first is consumed.  A
// row of C is stored by the partition in which the row starts; the partial row
// of a partition that starts inside a row goes to the carry buffer and is added
// by the fix-up pass in a fixed order.
#include "common.hpp"
#include "kernels.hpp"

namespace nacho {

namespace {

constexpr int kUnroll = 16;

template <typename T, int G, int RBLK>
__global__ void __launch_bounds__(NACHO_WAVE)
spmm_exec_kernel(const int32_t *__restrict__ pos, const int32_t *__restrict__ crd,
                 const T *__restrict__ val, const T *__restrict__ B, int n, int64_t ldb,
                 T *__restrict__ C, int64_t ldc, const int32_t *__restrict__ coord,
                 const int32_t *__restrict__ posn, T *__restrict__ carry_val,
                 int32_t *__restrict__ carry_row, WaveLog wlog)
{
    const WaveStamp stamp = wave_begin();
    __shared__ int32_t s_crd[G];
    __shared__ T s_val[G];
    __shared__ int32_t spos[RBLK + 1];

    const int p = blockIdx.x;
    const int lane = threadIdx.x;
    const bool col = lane < n;
    const int r0 = coord[2 * p], r1 = coord[2 * p + 2];
    const int n0 = posn[2 * p + 1], n1 = posn[2 * p + 3];
    const int pr0 = pos[r0], pr1 = pos[r1];
    const bool has_head = n0 > pr0;
    const int next_first = (n1 > pr1) ? r1 + 1 : r1;
    const int nrows = next_first - r0;

    for (int i = lane; i < n1 - n0; i += NACHO_WAVE) {
        s_crd[i] = crd[n0 + i];
        s_val[i] = val[n0 + i];
    }
    int blk0 = r0;                                     // spos[i] = pos[blk0 + i]
    {
        const int cnt = nrows < RBLK ? nrows : RBLK;
        if (nrows > 0)
            for (int i = lane; i <= cnt; i += NACHO_WAVE) spos[i] = pos[blk0 + i];
    }
    __syncthreads();

    T acc = T(0);
    int cur = r0;                                      // row being accumulated
    int cur_end = n1;                                  // its end inside the partition
    if (nrows > 0) { const int e = spos[1]; cur_end = e < n1 ? e : n1; }

    // store row `cur` (to C, or to the carry buffer when the row started in an earlier partition)
    auto store = [&]() {
        if (has_head && cur == r0) { if (col) carry_val[(int64_t)p * NACHO_WAVE + lane] = acc; }
        else if (col) C[(int64_t)cur * ldc + lane] = acc;
        acc = T(0);
    };
    // move on to the row that holds position q (cur_end <= q < n1).  The rows in between are
    // empty: their rows of C are zero already (the partition kernel wrote them), so they are
    // stepped over however many there are.
    int win = nrows < RBLK ? nrows : RBLK;             // rows whose pos entries are staged: blk0 .. blk0 + win
    auto advance = [&](int q) {
        ++cur;
        const int idx = cur + 1 - blk0;
        if (idx <= win) {
            const int e = spos[idx];
            if (e > q) {                               // the next row holds q: the common case
                cur_end = e < n1 ? e : n1;
                return;
            }
        }
        if (spos[win] > q) {
            while (spos[cur + 1 - blk0] <= q) ++cur;   // inside the window: at most RBLK cheap steps
        } else {                                       // beyond the staged window: search pos, restage
            cur = first_row_past(pos, blk0 + win, next_first, q);
            __syncthreads();
            blk0 = cur;
            const int left = next_first - blk0;
            win = left < RBLK ? left : RBLK;
            for (int i = lane; i <= win; i += NACHO_WAVE) spos[i] = pos[blk0 + i];
            __syncthreads();
        }
        const int e = spos[cur + 1 - blk0];
        cur_end = e < n1 ? e : n1;
    };

    for (int q0 = n0; q0 < n1; q0 += kUnroll) {
        T b[kUnroll], v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int q = q0 + u;
            const bool in = q < n1;
            const int c = in ? s_crd[q - n0] : 0;
            v[u] = in ? s_val[q - n0] : T(0);
            b[u] = (in && col) ? B[(int64_t)c * ldb + lane] : T(0);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int q = q0 + u;
            if (q < n1) {
                if (q >= cur_end) { store(); advance(q); }
                acc += v[u] * b[u];
            }
        }
    }
    // the row of the last non-zero (or, for a partition without work that starts inside a
    // row, a zero carry); every row after it up to the next partition is empty
    if (cur < next_first) store();
    if (lane == 0) carry_row[p] = has_head ? r0 : -1;
    wave_end(wlog, blockIdx.x, stamp, (uint32_t)(n1 - n0), (uint32_t)nrows);
}

template <typename T>
__global__ void __launch_bounds__(256)
spmm_fixup_kernel(T *__restrict__ C, int64_t ldc, int n, int P, const T *__restrict__ carry_val,
                  const int32_t *__restrict__ carry_row, const int32_t *__restrict__ pos, int grain)
{
    const int p = (int)(((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / NACHO_WAVE);
    if (p >= P) return;
    const int lane = lane_id();
    const int r = carry_row[p];
    if (r < 0) return;
    if (p > 0 && carry_row[p - 1] == r) return;
    int e = p + 1;
    if (grain > 0) {
        // fixed-grain partitions: the carries of row r come from the partitions that start
        // strictly inside it, the last one being ceil(pos[r+1] / grain) - 1
        e = ((pos[r + 1] - pos[0]) + grain - 1) / grain;
        if (e > P) e = P;
    } else for (;;) {
        const int q = e + lane;
        const bool same = q < P && carry_row[q] == r;
        const unsigned long long m = __ballot(same);
        if (m == ~0ull) { e += NACHO_WAVE; continue; }
        e += __ffsll((long long)~m) - 1;
        break;
    }
    if (lane >= n) return;
    // 32 independent partial sums keep 32 carry rows in flight (a row of hundreds of
    // thousands of non-zeros has hundreds of carries); the order of the additions is
    // fixed, so the result repeats bit for bit
    constexpr int kAcc = 32;
    T s[kAcc];
#pragma unroll
    for (int u = 0; u < kAcc; ++u) s[u] = T(0);
    int q = p;
    for (; q + kAcc <= e; q += kAcc) {
#pragma unroll
        for (int u = 0; u < kAcc; ++u) s[u] += carry_val[(int64_t)(q + u) * NACHO_WAVE + lane];
    }
    for (; q < e; ++q) s[(q - p) & (kAcc - 1)] += carry_val[(int64_t)q * NACHO_WAVE + lane];
#pragma unroll
    for (int w = kAcc / 2; w > 0; w >>= 1)
#pragma unroll
        for (int u = 0; u < w; ++u) s[u] += s[u + w];
    C[(int64_t)r * ldc + lane] += s[0];
}

constexpr int kGrain = 512, kRows = 512;

}  // namespace

int spmm_capacity(int dtype) { (void)dtype; return kGrain; }

hipError_t launch_spmm_exec(int dtype, const int32_t *pos, const int32_t *crd, const void *val,
                            const void *B, int n, int64_t ldb, void *C, int64_t ldc,
                            const int32_t *coord, const int32_t *posn, int64_t P, void *carry_val,
                            int32_t *carry_row, hipStream_t stream)
{
    if (dtype == NACHO_F64)
        hipLaunchKernelGGL((spmm_exec_kernel<double, kGrain, kRows>), dim3((unsigned)P), dim3(NACHO_WAVE),
                           0, stream, pos, crd, (const double *)val, (const double *)B, n, ldb,
                           (double *)C, ldc, coord, posn, (double *)carry_val, carry_row, nacho_host::wave_log());
    else
        hipLaunchKernelGGL((spmm_exec_kernel<float, kGrain, kRows>), dim3((unsigned)P), dim3(NACHO_WAVE),
                           0, stream, pos, crd, (const float *)val, (const float *)B, n, ldb,
                           (float *)C, ldc, coord, posn, (float *)carry_val, carry_row, nacho_host::wave_log());
    return hipGetLastError();
}

hipError_t launch_spmm_fixup(int dtype, void *C, int64_t ldc, int n, int64_t P, const void *carry_val,
                             const int32_t *carry_row, const int32_t *pos, int64_t grain, hipStream_t stream)
{
    const unsigned grid = (unsigned)((P * NACHO_WAVE + 255) / 256);
    if (dtype == NACHO_F64)
        hipLaunchKernelGGL((spmm_fixup_kernel<double>), dim3(grid), dim3(256), 0, stream, (double *)C, ldc,
                           n, (int)P, (const double *)carry_val, carry_row, pos, (int)grain);
    else
        hipLaunchKernelGGL((spmm_fixup_kernel<float>), dim3(grid), dim3(256), 0, stream, (float *)C, ldc,
                           n, (int)P, (const float *)carry_val, carry_row, pos, (int)grain);
    return hipGetLastError();
}

}  // namespace nacho
