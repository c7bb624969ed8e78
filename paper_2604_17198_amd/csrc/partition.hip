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
// The result is the coordinate and the positions the serial search returns: the
// highest coordinate whose cost does not exceed the residual query (it is then
// a stored coordinate), and for every operand the position of its first entry
// that is not before that coordinate.
#include "common.hpp"
#include "kernels.hpp"

namespace nacho {

namespace {

struct LevelResult {
    int64_t x;  // chosen coordinate
    int64_t c;  // C_m(x | prefix), unscaled
};

__device__ inline int64_t wave_max64(int64_t v)
{
#pragma unroll
    for (int off = NACHO_WAVE / 2; off > 0; off >>= 1) {
        const int64_t o = __shfl_xor((long long)v, off, NACHO_WAVE);
        v = o > v ? o : v;
    }
    return v;
}
__device__ inline int64_t wave_min64(int64_t v)
{
#pragma unroll
    for (int off = NACHO_WAVE / 2; off > 0; off >>= 1) {
        const int64_t o = __shfl_xor((long long)v, off, NACHO_WAVE);
        v = o < v ? o : v;
    }
    return v;
}

// Dense level (level 0 of CSR operands): position == coordinate, cost through
// the next level's pos array.  64-ary search over [0, N].
template <int K>
__device__ LevelResult dense_search(const DevOperands &ops, int m, int64_t R, int *p)
{
    const int lane = lane_id();
    const int k = ops.k;
    const int64_t N = ops.lvl[0][m].extent;
    int64_t low = 0, high = N, c_low = 0;
    while (low < high) {
        const int64_t span = high - low;
        const int64_t step = (span + NACHO_WAVE - 1) / NACHO_WAVE;
        int64_t x = low + (int64_t)(lane + 1) * step;
        if (x > high) x = high;
        int64_t c = 0;
#pragma unroll
        for (int t = 0; t < K; ++t) {
            if (t >= k) break;
            const int32_t *pos = ops.lvl[t][m + 1].pos;
            c += (int64_t)(pos[x] - pos[0]);
        }
        const unsigned long long ok = __ballot(c <= R);   // a prefix of the lanes (monotone cost)
        const int n = __popcll(ok);
        if (n > 0) {
            low = __shfl((long long)x, n - 1, NACHO_WAVE);
            c_low = __shfl((long long)c, n - 1, NACHO_WAVE);
        }
        if (n < NACHO_WAVE) high = __shfl((long long)x, n, NACHO_WAVE) - 1;
    }
#pragma unroll
    for (int t = 0; t < K; ++t) {
        if (t >= k) break;
        p[t] = (int)low;
    }
    LevelResult r;
    r.x = low;
    r.c = c_low;
    return r;
}

// 64-ary search over coordinates with one lower-bound search per operand and
// probe inside tracked windows [wl, wh] (the specialised search of Section
// 4.2.3, 64 probes per round).  Lower bounds are clamped to the windows, which
// is exact as long as the windows bracket the boundary's positions.  c_low is
// the cost at coordinate 0 under that clamping.  Used when the sampled search
// below stops making progress.
template <bool kLast, int K>
__device__ LevelResult tracked_search(const DevOperands &ops, int m, int64_t R, const int *base,
                                      int *wl, int *wh, int64_t c_low, int *p)
{
    const int lane = lane_id();
    const int k = ops.k;
    int64_t low = 0, high = ops.lvl[0][m].extent;
    while (low < high) {
        const int64_t span = high - low;
        const int64_t step = (span + NACHO_WAVE - 1) / NACHO_WAVE;
        int64_t x = low + (int64_t)(lane + 1) * step;
        if (x > high) x = high;
        int ip[K];
        int64_t c = 0;
#pragma unroll
        for (int t = 0; t < K; ++t) {
            if (t >= k) break;
            const int q = lower_bound_global(ops.lvl[t][m].crd, wl[t], wh[t], x);
            ip[t] = q;
            c += kLast ? (int64_t)(q - base[t]) : (int64_t)(ops.lvl[t][m + 1].pos[q] - base[t]);
        }
        const unsigned long long ok = __ballot(c <= R);
        const int n = __popcll(ok);
        if (n > 0) {
            low = __shfl((long long)x, n - 1, NACHO_WAVE);
            c_low = __shfl((long long)c, n - 1, NACHO_WAVE);
        }
        if (n < NACHO_WAVE) high = __shfl((long long)x, n, NACHO_WAVE) - 1;
#pragma unroll
        for (int t = 0; t < K; ++t) {
            if (t >= k) break;
            const int lo_new = __shfl(ip[t], n > 0 ? n - 1 : 0, NACHO_WAVE);
            const int hi_new = __shfl(ip[t], n < NACHO_WAVE ? n : NACHO_WAVE - 1, NACHO_WAVE);
            if (n > 0) wl[t] = lo_new;
            if (n < NACHO_WAVE) wh[t] = hi_new;
        }
    }
#pragma unroll
    for (int t = 0; t < K; ++t) {
        if (t >= k) break;
        p[t] = wl[t];
    }
    LevelResult r;
    r.x = low;
    r.c = c_low;
    return r;
}

// Compressed level.  seg_lo/seg_hi: every operand's segment.  Requires
// 0 <= R < total cost of the segments (an interior query), so the boundary is a
// stored coordinate.  Invariant of the windows [l, h]: the position of the
// boundary coordinate x in operand t lies in [l_t, h_t], and so does the
// position of x + 1.  With that, clamping any coordinate's lower bounds into
// the windows preserves "cost <= R  <=>  coordinate <= x".
template <bool kLast, int K>
__device__ LevelResult sampled_search(const DevOperands &ops, int m, int64_t R,
                                      const int *seg_lo, const int *seg_hi, int *p)
{
    const int lane = lane_id();
    const int k = ops.k;
    int base[K], l[K], h[K], cl[K], ch[K];          // costs relative to the segment start
#pragma unroll
    for (int t = 0; t < K; ++t) {
        l[t] = h[t] = cl[t] = ch[t] = base[t] = 0;  // operands beyond k: empty windows, no cost
        if (t < k) {
            l[t] = seg_lo[t];
            h[t] = seg_hi[t];
            if (kLast) {
                base[t] = seg_lo[t];
                ch[t] = seg_hi[t] - seg_lo[t];
            } else {
                const int32_t *pos = ops.lvl[t][m + 1].pos;
                base[t] = pos[seg_lo[t]];
                ch[t] = pos[seg_hi[t]] - base[t];
            }
        }
    }
    // position of sample j of a window (l, w): every entry when w <= 64, else 64 evenly spaced ones
    auto sample_pos = [](int lo, int w, int j) -> int {
        return lo + (w <= NACHO_WAVE ? j : (int)(((int64_t)j * w) >> 6));
    };
    int64_t prev_total = INT64_MAX;
    for (;;) {
        int v[K], ca[K], cb[K], w[K], mt[K];
        bool all_small = true;
        int64_t total = 0;
#pragma unroll
        for (int t = 0; t < K; ++t) {
            w[t] = h[t] - l[t];
            mt[t] = w[t] < NACHO_WAVE ? w[t] : NACHO_WAVE;
            total += w[t];
            if (w[t] > NACHO_WAVE) all_small = false;
            const bool valid = lane < mt[t];
            const int s = valid ? sample_pos(l[t], w[t], lane) : l[t];
            v[t] = INT32_MAX;
            cb[t] = s - base[t];
            ca[t] = s + 1 - base[t];
            if (t < k) {
                if (valid) v[t] = ops.lvl[t][m].crd[s];
                if (!kLast) {
                    const int32_t *pos = ops.lvl[t][m + 1].pos;
                    cb[t] = valid ? pos[s] - base[t] : 0;
                    ca[t] = valid ? pos[s + 1] - base[t] : 0;
                }
            }
        }
        if (!all_small && total >= prev_total) {
            int64_t c0 = 0;
#pragma unroll
            for (int t = 0; t < K; ++t) c0 += cl[t];
            return tracked_search<kLast, K>(ops, m, R, base, l, h, c0, p);
        }
        prev_total = total;

        // rank of every sample of t among the samples of u: K*(K-1) binary searches
        // over the lanes, advanced in lockstep so their shuffles overlap
        int lo[K][K], hi[K][K];
#pragma unroll
        for (int t = 0; t < K; ++t)
#pragma unroll
            for (int u = 0; u < K; ++u) { lo[t][u] = 0; hi[t][u] = mt[u]; }
#pragma unroll
        for (int it = 0; it < 7; ++it) {
#pragma unroll
            for (int t = 0; t < K; ++t)
#pragma unroll
                for (int u = 0; u < K; ++u) {
                    if (u == t) continue;
                    const int mid = (lo[t][u] + hi[t][u]) >> 1;
                    const int xs = __shfl(v[u], mid & (NACHO_WAVE - 1), NACHO_WAVE);
                    const bool go = lo[t][u] < hi[t][u];
                    const bool right = xs < v[t];
                    lo[t][u] = (go && right) ? mid + 1 : lo[t][u];
                    hi[t][u] = (go && !right) ? mid : hi[t][u];
                }
        }
        // bounds of the cost of every sampled coordinate
        int64_t best_le = -1, best_gt = INT64_MAX;
#pragma unroll
        for (int t = 0; t < K; ++t) {
            int64_t glo = cb[t], ghi = cb[t];       // own operand: the sample's position is exact
#pragma unroll
            for (int u = 0; u < K; ++u) {
                if (u == t) continue;
                const int c = lo[t][u];             // u's samples below this coordinate
                int costA, costB;
                if (kLast) {
                    const int posA = c == 0 ? l[u] : sample_pos(l[u], w[u], c - 1) + 1;
                    const int posB = c == mt[u] ? h[u] : sample_pos(l[u], w[u], c);
                    costA = posA - base[u];
                    costB = posB - base[u];
                } else {
                    const int a = __shfl(ca[u], (c - 1) & (NACHO_WAVE - 1), NACHO_WAVE);
                    const int bq = __shfl(cb[u], c & (NACHO_WAVE - 1), NACHO_WAVE);
                    costA = c == 0 ? cl[u] : a;
                    costB = c == mt[u] ? ch[u] : bq;
                }
                glo += costA;
                ghi += costB;
            }
            const bool valid = lane < mt[t];
            const int64_t vv = v[t];
            if (valid && ghi <= R && vv > best_le) best_le = vv;
            if (valid && glo > R && vv < best_gt) best_gt = vv;
        }
        const int64_t vminus = wave_max64(best_le);     // largest sample known not to be after the boundary
        const int64_t vplus = wave_min64(best_gt);      // smallest sample known to be after it

#pragma unroll
        for (int u = 0; u < K; ++u) {
            const bool in = lane < mt[u];
            int nl = l[u], ncl = cl[u], nh = h[u], nch = ch[u];
            if (vminus >= 0) {
                const int c = __popcll(__ballot(in && (int64_t)v[u] < vminus));
                const bool eq = __ballot(in && (int64_t)v[u] == vminus) != 0ull;
                const int sc = c < mt[u] ? sample_pos(l[u], w[u], c) : h[u];
                const int sp = c > 0 ? sample_pos(l[u], w[u], c - 1) + 1 : l[u];
                nl = eq ? sc : sp;
                if (kLast) ncl = nl - base[u];
                else {
                    const int e = __shfl(cb[u], c & (NACHO_WAVE - 1), NACHO_WAVE);
                    const int a = __shfl(ca[u], (c - 1) & (NACHO_WAVE - 1), NACHO_WAVE);
                    ncl = eq ? e : (c == 0 ? cl[u] : a);
                }
            }
            if (vplus != INT64_MAX) {
                const int c = __popcll(__ballot(in && (int64_t)v[u] < vplus));
                nh = c == mt[u] ? h[u] : sample_pos(l[u], w[u], c);
                if (kLast) nch = nh - base[u];
                else {
                    const int e = __shfl(cb[u], c & (NACHO_WAVE - 1), NACHO_WAVE);
                    nch = c == mt[u] ? ch[u] : e;
                }
            }
            l[u] = nl; cl[u] = ncl; h[u] = nh; ch[u] = nch;
        }
        if (all_small) {
            if (vminus < 0) {                           // cannot happen for an interior query
#pragma unroll
                for (int t = 0; t < K; ++t) {
                    if (t < k) { l[t] = seg_lo[t]; h[t] = seg_hi[t]; }
                }
                return tracked_search<kLast, K>(ops, m, R, base, l, h, 0, p);
            }
            LevelResult r;
            r.x = vminus;
            r.c = 0;
#pragma unroll
            for (int t = 0; t < K; ++t) {
                if (t < k) p[t] = l[t];
                r.c += cl[t];
            }
            return r;
        }
    }
}

// One level of Algorithm 1.  On return p[t] = position of operand t's first
// entry with coordinate >= x inside its segment.  All arguments are wave-uniform.
template <bool kLast, int K>
__device__ LevelResult search_level(const DevOperands &ops, int m, int64_t R,
                                    const int *seg_lo, const int *seg_hi, int *p)
{
    const int k = ops.k;
    if (ops.lvl[0][m].kind == NACHO_DENSE) return dense_search<K>(ops, m, R, p);

    int64_t total = 0;
    int nonempty = 0, which = 0;
#pragma unroll
    for (int t = 0; t < K; ++t) {
        if (t >= k) break;
        if (seg_hi[t] > seg_lo[t]) { ++nonempty; which = t; }
        if (kLast) total += seg_hi[t] - seg_lo[t];
        else total += ops.lvl[t][m + 1].pos[seg_hi[t]] - ops.lvl[t][m + 1].pos[seg_lo[t]];
    }
    if (R >= total) {
        // the query reaches past this level's segments: highest coordinate is the extent
#pragma unroll
        for (int t = 0; t < K; ++t) {
            if (t >= k) break;
            p[t] = seg_hi[t];
        }
        LevelResult r;
        r.x = ops.lvl[0][m].extent;
        r.c = total;
        return r;
    }
    if (kLast && nonempty == 1) {
        // exactly one operand with a non-empty segment: the residual indexes it
#pragma unroll
        for (int t = 0; t < K; ++t) {
            if (t >= k) break;
            p[t] = seg_lo[t];
        }
        p[which] = seg_lo[which] + (int)R;
        LevelResult r;
        r.x = ops.lvl[which][m].crd[p[which]];
        r.c = R;
        return r;
    }
    return sampled_search<kLast, K>(ops, m, R, seg_lo, seg_hi, p);
}

}  // namespace

template <int K>
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

    int seg_lo[K], seg_hi[K], p[K];
#pragma unroll
    for (int t = 0; t < K; ++t) {
        if (t >= k) break;
        const DevLevel &L = ops.lvl[t][0];
        seg_lo[t] = 0;
        seg_hi[t] = (L.kind == NACHO_DENSE) ? (int)L.extent : (int)L.count;
    }
    int64_t R = Qu;
    if (d == 1) {
        LevelResult r = search_level<true, K>(ops, 0, R, seg_lo, seg_hi, p);
        R -= r.c;
        if (lane == 0) {
            cb[0] = (int32_t)r.x;
            for (int t = 0; t < k; ++t) pb[t] = p[t];
        }
    } else {
        LevelResult r0 = search_level<false, K>(ops, 0, R, seg_lo, seg_hi, p);
        R -= r0.c;
        const bool dense0 = ops.lvl[0][0].kind == NACHO_DENSE;
        int p0[K];
#pragma unroll
        for (int t = 0; t < K; ++t) {
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
        LevelResult r1 = search_level<true, K>(ops, 1, R, seg_lo, seg_hi, p);
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
    // instantiated for 1, 2, 3, 4 and 8 operands so that small calls keep their state in registers
    if (ops.k <= 1)
        hipLaunchKernelGGL(partition_kernel<1>, dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                           queries, total_unscaled, coord, posn, cost);
    else if (ops.k <= 2)
        hipLaunchKernelGGL(partition_kernel<2>, dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                           queries, total_unscaled, coord, posn, cost);
    else if (ops.k <= 3)
        hipLaunchKernelGGL(partition_kernel<3>, dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                           queries, total_unscaled, coord, posn, cost);
    else if (ops.k <= 4)
        hipLaunchKernelGGL(partition_kernel<4>, dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                           queries, total_unscaled, coord, posn, cost);
    else
        hipLaunchKernelGGL(partition_kernel<8>, dim3(grid), dim3(256), 0, stream, ops, cost_scale, P, grain,
                           queries, total_unscaled, coord, posn, cost);
    return hipGetLastError();
}

}  // namespace nacho
