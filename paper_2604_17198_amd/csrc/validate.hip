// Debug aid, not on the hot path: checks on the device the preconditions the
// other entry points rely on without looking (sorted, duplicate-free
// coordinates inside every segment, coordinates inside the extents, monotone
// pos arrays that start at 0 and end at the level's count).
#include "common.hpp"
#include "kernels.hpp"

namespace nacho {

namespace {

struct Report {
    int32_t *status;     // NACHO_ERR_INVALID_ARG on a violation (left alone otherwise)
    int64_t *info;       // {operand, level, position} of one violation (any of them)
    __device__ void bad(int t, int m, int64_t at) const
    {
        *status = NACHO_ERR_INVALID_ARG;
        if (info) {
            info[0] = t;
            info[1] = m;
            info[2] = at;
        }
    }
};

// One compressed level of one operand: thread i checks parent i's pos entries, a wavefront
// walks every segment (64 neighbouring pairs of coordinates at a time).
__global__ void __launch_bounds__(256)
check_compressed_kernel(const int32_t *__restrict__ pos, const int32_t *__restrict__ crd, int64_t parents,
                        int64_t count, int64_t extent, int t, int m, Report rep)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = lane_id();
    int a = 0, b = 0;
    bool ok = true;
    if (i < parents) {
        a = pos[i];
        b = pos[i + 1];
        ok = a >= 0 && a <= b && b <= count;
        if (i == 0 && a != 0) ok = false;
        if (i == parents - 1 && b != count) ok = false;
        if (!ok) rep.bad(t, m, i);
    }
    unsigned long long todo = __ballot(i < parents && ok && b > a);
    while (todo) {
        const int src = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        const int lo = __shfl(a, src, NACHO_WAVE), hi = __shfl(b, src, NACHO_WAVE);
        for (int q = lo + lane; q < hi; q += NACHO_WAVE) {
            const int c = crd[q];
            if (c < 0 || (int64_t)c >= extent || (q > lo && crd[q - 1] >= c)) rep.bad(t, m, q);
        }
    }
}

// A coordinate list: (row, column) pairs strictly ascending, inside the extents.
__global__ void __launch_bounds__(256)
check_pairs_kernel(const int32_t *__restrict__ rows, const int32_t *__restrict__ cols, int64_t count,
                   int64_t n_rows, int64_t n_cols, int t, Report rep)
{
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= count) return;
    const int r = rows[q], c = cols[q];
    if (r < 0 || (int64_t)r >= n_rows) rep.bad(t, 0, q);
    if (c < 0 || (int64_t)c >= n_cols) rep.bad(t, 1, q);
    if (q > 0) {
        const int pr = rows[q - 1], pc = cols[q - 1];
        if (pr > r) rep.bad(t, 0, q);
        else if (pr == r && pc >= c) rep.bad(t, 1, q);
    }
}

__global__ void set_ok_kernel(int32_t *status, int64_t *info)
{
    *status = NACHO_OK;
    if (info) info[0] = info[1] = info[2] = -1;
}

}  // namespace

hipError_t launch_validate(const DevOperands &ops, int32_t *status, int64_t *info, hipStream_t s)
{
    Report rep;
    rep.status = status;
    rep.info = info;
    hipLaunchKernelGGL(set_ok_kernel, dim3(1), dim3(1), 0, s, status, info);
    for (int t = 0; t < ops.k; ++t) {
        if (ops.lvl[t][0].kind == NACHO_NONUNIQUE) {
            const int64_t n = ops.lvl[t][0].count;
            if (n > 0)
                hipLaunchKernelGGL(check_pairs_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                                   ops.lvl[t][0].crd, ops.lvl[t][1].crd, n, ops.lvl[t][0].extent,
                                   ops.lvl[t][1].extent, t, rep);
            continue;
        }
        int64_t parents = 1;                         // entries of the level above
        for (int m = 0; m < ops.d; ++m) {
            const DevLevel &L = ops.lvl[t][m];
            if (L.kind == NACHO_DENSE) {
                parents *= L.extent;
                continue;
            }
            if (parents > 0)
                hipLaunchKernelGGL(check_compressed_kernel, dim3((unsigned)((parents + 255) / 256)), dim3(256), 0, s,
                                   L.pos, L.crd, parents, L.count, L.extent, t, m, rep);
            parents = L.count;
        }
    }
    return hipGetLastError();
}

}  // namespace nacho
