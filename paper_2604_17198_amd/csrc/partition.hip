// Partition kernel: one wavefront runs one boundary search (Section 3.2,
// Algorithm 1) with the non-zero-count cost of Section 4.2.2, in position
// space with tracked search windows (Section 4.2.3).
//
// What differs from the paper's per-thread binary search: the 64 lanes of a
// wavefront probe 64 candidate coordinates per round (a 64-ary search), so a
// level of extent N takes ceil(log64(N+1)) rounds instead of log2(N).  Each
// lane evaluates the cost of its candidate with one lower-bound search per
// operand inside that operand's tracked window; the window shrinks to the
// bracketing lanes' positions after every round.  The result is the same
// coordinate and the same positions the serial search returns: the highest
// coordinate whose cost does not exceed the residual query.
#include "common.hpp"
#include "kernels.hpp"

namespace nacho {

namespace {

struct LevelResult {
    int64_t x;  // chosen coordinate
    int64_t c;  // C_m(x | prefix), unscaled
};

// One level of Algorithm 1.  seg_lo/seg_hi: every operand's segment at this
// level.  On return p[t] = position of operand t's first entry with coordinate
// >= x inside its segment.  All arguments are wave-uniform.
template <bool kLast>
__device__ LevelResult search_level(const DevOperands &ops, int m, int64_t R,
                                    const int *seg_lo, const int *seg_hi, int *p)
{
    const int lane = lane_id();
    const int k = ops.k;
    const int64_t N = ops.lvl[0][m].extent;
    const bool dense = ops.lvl[0][m].kind == NACHO_DENSE;

    // Cost of the entries before a position, relative to the segment start.
    int base[NACHO_MAX_OPERANDS];
#pragma unroll
    for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
        if (t >= k) break;
        if (kLast) base[t] = seg_lo[t];
        else base[t] = ops.lvl[t][m + 1].pos[dense ? 0 : seg_lo[t]];
    }

    if (kLast && !dense) {
        // Exactly one operand with a non-empty segment: the residual indexes it.
        int nonempty = 0, which = 0;
#pragma unroll
        for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
            if (t >= k) break;
            if (seg_hi[t] > seg_lo[t]) { ++nonempty; which = t; }
        }
        if (nonempty == 1 && R < (int64_t)(seg_hi[which] - seg_lo[which])) {
#pragma unroll
            for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
                if (t >= k) break;
                p[t] = seg_lo[t];
            }
            p[which] = seg_lo[which] + (int)R;
            LevelResult r;
            r.x = ops.lvl[which][m].crd[p[which]];
            r.c = R;
            return r;
        }
    }

    int64_t low = 0, high = N, c_low = 0;
    int wl[NACHO_MAX_OPERANDS], wh[NACHO_MAX_OPERANDS];  // tracked windows [wl, wh]
#pragma unroll
    for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
        if (t >= k) break;
        wl[t] = seg_lo[t];
        wh[t] = seg_hi[t];
    }
    while (low < high) {
        const int64_t span = high - low;
        const int64_t step = (span + NACHO_WAVE - 1) / NACHO_WAVE;
        int64_t x = low + (int64_t)(lane + 1) * step;
        if (x > high) x = high;
        int ip[NACHO_MAX_OPERANDS];
        int64_t c = 0;
#pragma unroll
        for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
            if (t >= k) break;
            int q;
            if (dense) q = (int)x;
            else q = lower_bound_global(ops.lvl[t][m].crd, wl[t], wh[t], x);
            ip[t] = q;
            c += kLast ? (int64_t)(q - base[t]) : (int64_t)(ops.lvl[t][m + 1].pos[q] - base[t]);
        }
        const unsigned long long ok = __ballot(c <= R);   // a prefix of the lanes (monotone cost)
        const int n = __popcll(ok);
        if (n > 0) {
            low = __shfl(x, n - 1, NACHO_WAVE);
            c_low = __shfl(c, n - 1, NACHO_WAVE);
        }
        if (n < NACHO_WAVE) high = __shfl(x, n, NACHO_WAVE) - 1;
#pragma unroll
        for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
            if (t >= k) break;
            const int lo_new = __shfl(ip[t], n > 0 ? n - 1 : 0, NACHO_WAVE);
            const int hi_new = __shfl(ip[t], n < NACHO_WAVE ? n : NACHO_WAVE - 1, NACHO_WAVE);
            if (n > 0) wl[t] = lo_new;
            if (n < NACHO_WAVE) wh[t] = hi_new;
        }
    }
#pragma unroll
    for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
        if (t >= k) break;
        p[t] = dense ? (int)low : wl[t];
    }
    LevelResult r;
    r.x = low;
    r.c = c_low;
    return r;
}

}  // namespace

__global__ void __launch_bounds__(256)
partition_kernel(DevOperands ops, int64_t cost_scale, int64_t P, int64_t grain,
                 const int64_t *__restrict__ queries, int64_t total_unscaled, int32_t *__restrict__ coord, int32_t *__restrict__ posn,
                 int64_t *__restrict__ cost)
{
    const int64_t b = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / NACHO_WAVE;
    if (b > P) return;                      // whole wavefront leaves together
    const int lane = lane_id();
    const int k = ops.k, d = ops.d;

    const int64_t total_scaled = total_unscaled * cost_scale;
    int64_t Q;
    if (queries) Q = queries[b];
    else if (grain > 0) Q = b * grain < total_scaled ? b * grain : total_scaled;
    else Q = equal_query(b, total_scaled, P);
    if (Q < 0) Q = 0;
    const int64_t Qu = Q / cost_scale;

    int32_t *cb = coord + b * d;
    int32_t *pb = posn + b * (int64_t)k * d;

    if (b == 0 || b == P || Qu >= total_unscaled) {
        const bool end = (b != 0);
        if (lane == 0) {
            for (int m = 0; m < d; ++m) cb[m] = 0;
            if (end) cb[0] = (int32_t)ops.lvl[0][0].extent;
            for (int t = 0; t < k; ++t)
                for (int m = 0; m < d; ++m) {
                    const DevLevel &L = ops.lvl[t][m];
                    int32_t at = 0;
                    if (end) at = (L.kind == NACHO_DENSE) ? (int32_t)L.extent : (int32_t)L.count;
                    pb[t * d + m] = at;
                }
            cost[b] = end ? total_scaled : 0;
        }
        return;
    }

    int seg_lo[NACHO_MAX_OPERANDS], seg_hi[NACHO_MAX_OPERANDS], p[NACHO_MAX_OPERANDS];
#pragma unroll
    for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
        if (t >= k) break;
        const DevLevel &L = ops.lvl[t][0];
        seg_lo[t] = 0;
        seg_hi[t] = (L.kind == NACHO_DENSE) ? (int)L.extent : (int)L.count;
    }
    int64_t R = Qu;
    if (d == 1) {
        LevelResult r = search_level<true>(ops, 0, R, seg_lo, seg_hi, p);
        R -= r.c;
        if (lane == 0) {
            cb[0] = (int32_t)r.x;
            for (int t = 0; t < k; ++t) pb[t] = p[t];
        }
    } else {
        LevelResult r0 = search_level<false>(ops, 0, R, seg_lo, seg_hi, p);
        R -= r0.c;
        const bool dense0 = ops.lvl[0][0].kind == NACHO_DENSE;
        int p0[NACHO_MAX_OPERANDS];
#pragma unroll
        for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
            if (t >= k) break;
            p0[t] = p[t];
            const DevLevel &L0 = ops.lvl[t][0];
            const int32_t *pos1 = ops.lvl[t][1].pos;
            bool present;
            if (dense0) present = r0.x < L0.extent;
            else present = p[t] < seg_hi[t] && (int64_t)L0.crd[p[t]] == r0.x;
            const int lo1 = pos1[p[t]];
            seg_lo[t] = lo1;
            seg_hi[t] = present ? pos1[p[t] + 1] : lo1;
        }
        LevelResult r1 = search_level<true>(ops, 1, R, seg_lo, seg_hi, p);
        R -= r1.c;
        if (lane == 0) {
            cb[0] = (int32_t)r0.x;
            cb[1] = (int32_t)r1.x;
            for (int t = 0; t < k; ++t) {
                pb[t * 2 + 0] = p0[t];
                pb[t * 2 + 1] = p[t];
            }
        }
    }
    if (lane == 0) cost[b] = (Qu - R) * cost_scale;
}

hipError_t launch_partition(const DevOperands &ops, int64_t cost_scale, int64_t P, int64_t grain,
                            const int64_t *queries, int64_t total_unscaled,
                            int32_t *coord, int32_t *posn, int64_t *cost, hipStream_t stream)
{
    const int64_t waves = P + 1;
    const int waves_per_block = 256 / NACHO_WAVE;
    const unsigned grid = (unsigned)((waves + waves_per_block - 1) / waves_per_block);
    hipLaunchKernelGGL(partition_kernel, dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                       queries, total_unscaled, coord, posn, cost);
    return hipGetLastError();
}

}  // namespace nacho
