// The boundary search of Algorithm 1 (Section 3.2) as one wavefront runs it, for the partition
// kernel and for kernels that search their own boundaries: see partition.hip for the method.
#pragma once
#include "common.hpp"
#include "kernels.hpp"

namespace nacho {

namespace {

struct LevelResult {
    int64_t x;  // chosen coordinate
    int64_t c;  // C_m(x | prefix), unscaled
};

// How a compressed level's coordinates are read.  Plain: one int32 array.  Pairs: the level is
// the list of (row, column) pairs of a coordinate-list (COO) operand, i.e. both of its levels
// taken together as one sorted, duplicate-free level with the 64-bit coordinate row << 32 | column
// (Algorithm 1 on the two levels and on this one level find the same boundary: the highest row
// whose cost fits, then the highest column inside it, is the highest pair whose cost fits).
struct PlainCoords {
    typedef int type;
    static constexpr type kNone = INT32_MAX;            // no coordinate
    __device__ static type load(const DevOperands &ops, int t, int m, int at) { return ops.lvl[t][m].crd[at]; }
    __device__ static int64_t extent(const DevOperands &ops, int m) { return ops.lvl[0][m].extent; }
};
struct PairCoords {
    typedef long long type;
    static constexpr type kNone = INT64_MAX;
    __device__ static type load(const DevOperands &ops, int t, int, int at)
    {
        return ((long long)ops.lvl[t][0].crd[at] << 32) | (long long)(unsigned)ops.lvl[t][1].crd[at];
    }
    __device__ static int64_t extent(const DevOperands &ops, int) { return ops.lvl[0][0].extent << 32; }
};

// The value lane `from` holds (`from` the same in every lane), through a scalar register.
__device__ inline int lane_value(int x, int from) { return __builtin_amdgcn_readlane(x, from); }
__device__ inline long long lane_value(long long x, int from)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(unsigned long long)x, from);
    const int hi = __builtin_amdgcn_readlane((int)(x >> 32), from);
    return ((long long)hi << 32) | (long long)lo;
}

// Least position in [lo, hi) of operand t whose coordinate is >= x; hi if there is none.
template <class Acc>
__device__ inline int lower_bound_level(const DevOperands &ops, int t, int m, int shift, int lo, int hi, int64_t x)
{
    while (lo < hi) {
        const int mid = lo + ((hi - lo) >> 1);
        if ((int64_t)Acc::load(ops, t, m, mid + shift) < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Cost of the entries before position q of a level that is not the last one: the start of
// q's segment one level down -- or, kDeep (level 0 of a three-level operand), the start two
// levels down, where the non-zeros are.
template <bool kDeep>
__device__ inline int cost_at(const DevOperands &ops, int t, int m, int q)
{
    const int v = ops.lvl[t][m + 1].pos[q];
    return kDeep ? ops.lvl[t][m + 2].pos[v] : v;
}

// Dense level (level 0 of CSR operands): position == coordinate, cost through
// the next level's pos array.  64-ary search over [0, N].
template <int K>
__device__ __forceinline__ LevelResult dense_search(const DevOperands &ops, int m, int64_t R, int *p)
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
            low = lane_value((long long)x, n - 1);
            c_low = lane_value((long long)c, n - 1);
        }
        if (n < NACHO_WAVE) high = lane_value((long long)x, n) - 1;
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

// (In all searches of a compressed level, sh[t] is added to operand t's positions
// where its coordinates are read: the offset between the positions the cost is
// counted in and the storage of a remapped operand's row, 0 otherwise.)
//
// 64-ary search over coordinates with one lower-bound search per operand and
// probe inside tracked windows [wl, wh] (the specialised search of Section
// 4.2.3, 64 probes per round).  Lower bounds are clamped to the windows, which
// is exact as long as the windows bracket the boundary's positions.  c_low is
// the cost at coordinate 0 under that clamping.  Used when the sampled search
// below stops making progress.
template <bool kLast, int K, class Acc = PlainCoords, bool kDeep = false>
__device__ __forceinline__ LevelResult tracked_search(const DevOperands &ops, int m, int64_t R, const int *base,
                                      int *wl, int *wh, int64_t c_low, int *p, const int *sh)
{
    const int lane = lane_id();
    const int k = ops.k;
    int64_t low = 0, high = Acc::extent(ops, m);
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
            const int q = lower_bound_level<Acc>(ops, t, m, sh[t], wl[t], wh[t], x);
            ip[t] = q;
            c += kLast ? (int64_t)(q - base[t]) : (int64_t)(cost_at<kDeep>(ops, t, m, q) - base[t]);
        }
        const unsigned long long ok = __ballot(c <= R);
        const int n = __popcll(ok);
        if (n > 0) {
            low = lane_value((long long)x, n - 1);
            c_low = lane_value((long long)c, n - 1);
        }
        if (n < NACHO_WAVE) high = lane_value((long long)x, n) - 1;
#pragma unroll
        for (int t = 0; t < K; ++t) {
            if (t >= k) break;
            const int lo_new = lane_value(ip[t], n > 0 ? n - 1 : 0);
            const int hi_new = lane_value(ip[t], n < NACHO_WAVE ? n : NACHO_WAVE - 1);
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

// How many of the wavefront's 64 values xs -- ascending with the lane, lanes past the valid ones hold
// the largest value there is -- are smaller than this lane's key.  Three levels of a 4-ary search: the
// values of lanes 15, 31, 47 (through scalar registers) pick sixteen lanes, three shuffles their
// quarter, three more count inside it; the last lane of a quarter is a pivot that was compared
// before, but for lane 63.  (A binary search is a chain of seven dependent shuffles and twice the
// instructions; these rank searches were half of a round's time, and the kernel is bound by the
// instructions its wavefronts issue.)
template <typename CoordT>
__device__ inline int rank_among(CoordT xs, CoordT key)
{
    int sixteen = 0;
#pragma unroll
    for (int g = 0; g < 3; ++g) sixteen += lane_value(xs, 16 * g + 15) < key ? 1 : 0;
    const int b1 = sixteen * 16;
    int quarter = 0;
#pragma unroll
    for (int g = 0; g < 3; ++g) quarter += __shfl(xs, b1 + 4 * g + 3, NACHO_WAVE) < key ? 1 : 0;
    const int b2 = b1 + quarter * 4;
    int n = b2 + (lane_value(xs, NACHO_WAVE - 1) < key ? 1 : 0);
#pragma unroll
    for (int i = 0; i < 3; ++i) n += __shfl(xs, b2 + i, NACHO_WAVE) < key ? 1 : 0;
    return n;
}

// Search windows of one compressed level: for operand t the boundary's position
// lies in [l, h]; cl/ch are the costs of the entries before l / before h,
// relative to the segment start (base = cost offset of the segment start).
template <int K>
struct Windows {
    int base[K], l[K], h[K], cl[K], ch[K];
};

template <bool kLast, int K, bool kDeep = false>
__device__ inline void windows_init(const DevOperands &ops, int m, const int *seg_lo, const int *seg_hi,
                                    Windows<K> &W)
{
#pragma unroll
    for (int t = 0; t < K; ++t) {
        W.l[t] = W.h[t] = W.cl[t] = W.ch[t] = W.base[t] = 0;   // operands beyond k: empty, no cost
        if (t < ops.k) {
            W.l[t] = seg_lo[t];
            W.h[t] = seg_hi[t];
            if (kLast) {
                W.base[t] = seg_lo[t];
                W.ch[t] = seg_hi[t] - seg_lo[t];
            } else {
                W.base[t] = cost_at<kDeep>(ops, t, m, seg_lo[t]);
                W.ch[t] = cost_at<kDeep>(ops, t, m, seg_hi[t]) - W.base[t];
            }
        }
    }
}

// Compressed level.  Requires 0 <= R_lo <= R_hi < total cost of the segments
// (interior queries), so the boundaries are stored coordinates.  Invariant of
// the windows [l, h]: for every query R in [R_lo, R_hi] the position of its
// boundary coordinate x in operand t lies in [l_t, h_t], and so does the
// position of x + 1.  With that, clamping any coordinate's lower bounds into
// the windows preserves "cost <= R  <=>  coordinate <= x".
// Runs until the boundary of query R is found.
template <bool kLast, int K, class Acc = PlainCoords, bool kDeep = false>
__device__ __forceinline__ LevelResult sampled_search(const DevOperands &ops, int m, int64_t R64, Windows<K> &W,
                                                      int *p, const int *sh)
{
    typedef typename Acc::type CoordT;
    // costs, positions and coordinates all fit 32 bits (the operands hold fewer than
    // 2^31 entries together; INT32_MAX is no coordinate)
    const int R_lo = (int)R64, R_hi = (int)R64;      // (the bounds below are written for a range of queries)
    const int lane = lane_id();
    const int k = ops.k;
    int base[K], l[K], h[K], cl[K], ch[K];
#pragma unroll
    for (int t = 0; t < K; ++t) {
        base[t] = W.base[t]; l[t] = W.l[t]; h[t] = W.h[t]; cl[t] = W.cl[t]; ch[t] = W.ch[t];
    }
    LevelResult r;
    r.x = 0;
    r.c = 0;
    // position of sample j of a window (l, w): every entry when w <= 64, else 64 evenly spaced ones
    // (j * w / 64 with w = 128 q + r is 2 j q + j r / 64: two 24-bit products, no 64-bit one)
    auto sample_pos = [](int lo, int w, int j) -> int {
        const int spread = 2 * __mul24(j, w >> 7) + (__mul24(j, w & 127) >> 6);
        return lo + (w <= NACHO_WAVE ? j : spread);
    };
    int prev_total = INT32_MAX;
    for (;;) {
        CoordT v[K];
        int ca[K], cb[K], w[K], mt[K];
        bool all_small = true;
        int total = 0;
#pragma unroll
        for (int t = 0; t < K; ++t) {
            w[t] = h[t] - l[t];
            mt[t] = w[t] < NACHO_WAVE ? w[t] : NACHO_WAVE;
            total += w[t];
            if (w[t] > NACHO_WAVE) all_small = false;
        }
        if (!all_small && total >= prev_total) {
            int64_t c0 = 0;
#pragma unroll
            for (int t = 0; t < K; ++t) c0 += cl[t];
            return tracked_search<kLast, K, Acc, kDeep>(ops, m, R64, base, l, h, c0, p, sh);
        }
        prev_total = total;
#pragma unroll
        for (int t = 0; t < K; ++t) {
            const bool valid = lane < mt[t];
            const int s = valid ? sample_pos(l[t], w[t], lane) : l[t];
            v[t] = Acc::kNone;
            cb[t] = s - base[t];
            ca[t] = s + 1 - base[t];
            if (t < k) {
                if (valid) v[t] = Acc::load(ops, t, m, s + sh[t]);
                if (!kLast) {
                    cb[t] = valid ? cost_at<kDeep>(ops, t, m, s) - base[t] : 0;
                    ca[t] = valid ? cost_at<kDeep>(ops, t, m, s + 1) - base[t] : 0;
                }
            }
        }

        // Bounds of the cost of every sampled coordinate, from the rank lo_t[u] of the sample
        // among the samples of every other operand u.  Inside one operand the
        // samples ascend with the lane and so do both bounds, so the samples whose
        // upper bound is within the query are a prefix of the lanes and those whose
        // lower bound exceeds it a suffix: one ballot each finds the largest / smallest
        // such sample, no reduction over the wavefront.
        CoordT vminus = -1, vplus = Acc::kNone;
        auto bounds_of = [&](int t, const int (&lo_t)[K]) {
            int glo = cb[t], ghi = cb[t];           // own operand: the sample's position is exact
#pragma unroll
            for (int u = 0; u < K; ++u) {
                if (u == t) continue;
                const int c = lo_t[u];              // u's samples below this coordinate
                // cost before u's sample c - 1 ... before its sample c: what the lanes c - 1 and c hold
                // (with positions as costs, the last level, these are the samples' positions)
                const int a = __shfl(ca[u], (c - 1) & (NACHO_WAVE - 1), NACHO_WAVE);
                const int bq = __shfl(cb[u], c & (NACHO_WAVE - 1), NACHO_WAVE);
                const int costA = c == 0 ? cl[u] : a;
                const int costB = c == mt[u] ? ch[u] : bq;
                glo += costA;
                ghi += costB;
            }
            const bool valid = lane < mt[t];
            const int n_le = __popcll(__ballot(valid && ghi <= R_lo));   // lanes 0 .. n_le - 1
            const int n_in = __popcll(__ballot(valid && glo <= R_hi));   // lanes n_in .. mt - 1 are after
            if (n_le > 0) {
                const CoordT cand = lane_value(v[t], n_le - 1);
                vminus = cand > vminus ? cand : vminus;  // largest sample not after the first boundary
            }
            if (n_in < mt[t]) {
                const CoordT cand = lane_value(v[t], n_in);
                vplus = cand < vplus ? cand : vplus;     // smallest sample after the last boundary
            }
        };
        // rank of every sample of t among the samples of u (lanes past mt[u] hold kNone, which is
        // smaller than no key: a rank never exceeds mt[u]); one operand at a time, ranks and bounds
#pragma unroll
        for (int t = 0; t < K; ++t) {
            int lo_t[K];
#pragma unroll
            for (int u = 0; u < K; ++u) lo_t[u] = u == t ? 0 : rank_among<CoordT>(v[u], v[t]);
            bounds_of(t, lo_t);
        }

#pragma unroll
        for (int u = 0; u < K; ++u) {
            const bool in = lane < mt[u];
            int nl = l[u], ncl = cl[u], nh = h[u], nch = ch[u];
            if (vminus >= 0) {
                const int c = __popcll(__ballot(in && v[u] < vminus));
                const bool eq = __ballot(in && v[u] == vminus) != 0ull;
                const int sc = c < mt[u] ? sample_pos(l[u], w[u], c) : h[u];
                const int sp = c > 0 ? sample_pos(l[u], w[u], c - 1) + 1 : l[u];
                nl = eq ? sc : sp;
                if (kLast) ncl = nl - base[u];
                else {
                    const int e = lane_value(cb[u], c & (NACHO_WAVE - 1));
                    const int a = lane_value(ca[u], (c - 1) & (NACHO_WAVE - 1));
                    ncl = eq ? e : (c == 0 ? cl[u] : a);
                }
            }
            if (vplus != Acc::kNone) {
                const int c = __popcll(__ballot(in && v[u] < vplus));
                nh = c == mt[u] ? h[u] : sample_pos(l[u], w[u], c);
                if (kLast) nch = nh - base[u];
                else {
                    const int e = lane_value(cb[u], c & (NACHO_WAVE - 1));
                    nch = c == mt[u] ? ch[u] : e;
                }
            }
            l[u] = nl; cl[u] = ncl; h[u] = nh; ch[u] = nch;
        }
        if (all_small) {
            if (vminus < 0) {                           // cannot happen for an interior query
                int64_t c0 = 0;
#pragma unroll
                for (int t = 0; t < K; ++t) {
                    l[t] = W.l[t]; h[t] = W.h[t];
                    c0 += W.cl[t];
                }
                return tracked_search<kLast, K, Acc, kDeep>(ops, m, R64, base, l, h, c0, p, sh);
            }
            r.x = vminus;
#pragma unroll
            for (int t = 0; t < K; ++t) {
                if (t < k) p[t] = l[t];
                r.c += cl[t];
            }
            return r;
        }
    }
}

// One level of Algorithm 1 for one query, starting from windows that bracket the
// boundary.  `total` = cost of the level's whole segments.  On return p[t] =
// position of operand t's first entry with coordinate >= x inside its segment.
template <bool kLast, int K, class Acc = PlainCoords, bool kDeep = false>
__device__ __forceinline__ LevelResult compressed_level(const DevOperands &ops, int m, int64_t R, int64_t total,
                                        const int *seg_lo, const int *seg_hi, Windows<K> &W, int *p,
                                        const int *sh)
{
    const int k = ops.k;
    LevelResult r;
    if (R >= total) {
        // the query reaches past this level's segments: highest coordinate is the extent
#pragma unroll
        for (int t = 0; t < K; ++t)
            if (t < k) p[t] = seg_hi[t];
        r.x = Acc::extent(ops, m);
        r.c = total;
        return r;
    }
    int nonempty = 0, which = 0;
#pragma unroll
    for (int t = 0; t < K; ++t)
        if (t < k && seg_hi[t] > seg_lo[t]) { ++nonempty; which = t; }
    if (kLast && nonempty == 1) {
        // exactly one operand with a non-empty segment: the residual indexes it
#pragma unroll
        for (int t = 0; t < K; ++t)
            if (t < k) p[t] = seg_lo[t];
        int at = 0;                                    // (no array is indexed by `which`: they stay in registers)
#pragma unroll
        for (int t = 0; t < K; ++t)
            if (t == which) {
                p[t] = seg_lo[t] + (int)R;
                at = p[t] + sh[t];
            }
        r.x = Acc::load(ops, which, m, at);
        r.c = R;
        return r;
    }
    if constexpr (K > 4) {
        // many operands: the sampled search would carry K * K rank searches per round and a
        // code size no instruction cache holds; the coordinate search with tracked windows
        // is the faster one there (8 operands of 2.5M entries: 275 us against 394 us)
        int64_t c0 = 0;
#pragma unroll
        for (int t = 0; t < K; ++t) c0 += W.cl[t];
        return tracked_search<kLast, K, Acc, kDeep>(ops, m, R, W.base, W.l, W.h, c0, p, sh);
    }
    return sampled_search<kLast, K, Acc, kDeep>(ops, m, R, W, p, sh);
}

template <bool kLast, int K>
__device__ inline int64_t level_total(const DevOperands &ops, int m, const int *seg_lo, const int *seg_hi)
{
    int64_t total = 0;
#pragma unroll
    for (int t = 0; t < K; ++t)
        if (t < ops.k) {
            if (kLast) total += seg_hi[t] - seg_lo[t];
            else total += ops.lvl[t][m + 1].pos[seg_hi[t]] - ops.lvl[t][m + 1].pos[seg_lo[t]];
        }
    return total;
}

// One wavefront searches boundary b (0 <= b <= P) and stores its coordinate, positions and cost.
// kMode: 0 = vectors, CSR, DCSR; 1 = coordinate lists; 2 = three compressed levels (CSF).
// found[t] (operands of one level only): operand t's position of the boundary, in every lane.
template <int K, int kMode>
__device__ inline void search_boundary(const DevOperands &ops, int64_t cost_scale, int64_t P, int64_t grain,
                                                const int64_t *__restrict__ queries, int64_t total_unscaled,
                                                int32_t *__restrict__ coord, int32_t *__restrict__ posn,
                                                int64_t *__restrict__ cost, int64_t b, int (&found)[K])
{
    const int lane = lane_id();
    const int k = ops.k, d = ops.d;
#pragma unroll
    for (int t = 0; t < K; ++t) found[t] = 0;
    const int64_t total_scaled = total_unscaled * cost_scale;
    const bool dense0 = ops.lvl[0][0].kind == NACHO_DENSE;
    constexpr bool pairs = kMode == 1;                              // coordinate lists (COO), d == 2
    constexpr bool csf3 = kMode == 2;                               // three compressed levels, d == 3

    int64_t Q = 0;
    if (queries) Q = queries[b];
    else if (grain > 0) Q = b * grain < total_scaled ? b * grain : total_scaled;
    else Q = equal_query(b, total_scaled, P);
    if (Q < 0) Q = 0;
    const int64_t Qu = Q / cost_scale;
    const bool interior = b > 0 && b < P && Qu < total_unscaled;

    // level-0 segments and, for a compressed level 0, the windows the search starts from
    int seg0_lo[K], seg0_hi[K];
#pragma unroll
    for (int t = 0; t < K; ++t) {
        seg0_lo[t] = seg0_hi[t] = 0;
        if (t < k) {
            const DevLevel &L = ops.lvl[t][0];
            seg0_hi[t] = (L.kind == NACHO_DENSE) ? (int)L.extent : (int)L.count;
        }
    }
    int no_shift[K];
#pragma unroll
    for (int t = 0; t < K; ++t) no_shift[t] = 0;
    Windows<K> W0;
    if (!dense0 && interior) {
        if (pairs) windows_init<true, K>(ops, 0, seg0_lo, seg0_hi, W0);
        else if (csf3) windows_init<false, K, true>(ops, 0, seg0_lo, seg0_hi, W0);
        else if (d == 1) windows_init<true, K>(ops, 0, seg0_lo, seg0_hi, W0);
        else windows_init<false, K>(ops, 0, seg0_lo, seg0_hi, W0);
    }

    {
        int32_t *cb = coord + b * d;
        int32_t *pb = posn + b * (int64_t)k * d;
        if (!interior) {
            const bool end = (b != 0);
            if (lane == 0) {
                for (int m = 0; m < d; ++m) cb[m] = 0;
                if (end) cb[0] = (int32_t)level0_extent(ops);
                for (int t = 0; t < k; ++t)
                    for (int m = 0; m < d; ++m) {
                        const DevLevel &L = ops.lvl[t][m];
                        int32_t at = 0;
                        if (end) at = (L.kind == NACHO_DENSE) ? (int32_t)L.extent : (int32_t)L.count;
                        if (end && ops.dyn_head) at = m == 0 ? (int32_t)level0_extent(ops) : (int32_t)last_count(ops, t);
                        pb[t * d + m] = at;
                    }
                cost[b] = end ? total_scaled : 0;
            }
            if (end && d == 1) {
#pragma unroll
                for (int t = 0; t < K; ++t)
                    if (t < k) found[t] = (int)ops.lvl[t][0].count;
            }
            return;
        }
        int seg_lo[K], seg_hi[K], p[K];
        int64_t R = Qu;
        if (pairs) {
            // one search over the (row, column) pairs; the row-level position of an operand is
            // that of its first entry in the boundary's row
            Windows<K> W = W0;
            LevelResult r = compressed_level<true, K, PairCoords>(ops, 0, R, total_unscaled, seg0_lo, seg0_hi, W, p,
                                                                  no_shift);
            R -= r.c;
            const int x0 = (int)(r.x >> 32), x1 = (int)(r.x & 0xffffffffLL);
            int mine = 0, row_at = 0;
#pragma unroll
            for (int t = 0; t < K; ++t)
                if (t < k && lane == t) mine = p[t];
            if (lane < k) row_at = lower_bound_global(ops.lvl[lane][0].crd, 0, mine, x0);
            if (lane < k) {
                pb[lane * 2 + 0] = row_at;
                pb[lane * 2 + 1] = mine;
            }
            if (lane == 0) {
                cb[0] = x0;
                cb[1] = x1;
            }
        } else if (csf3) {
            // three compressed levels: Algorithm 1 level by level; a level's cost counts the
            // non-zeros below its entries (two pos arrays down at level 0, one at level 1)
            int p0[K], p1[K];
            Windows<K> W = W0;
            LevelResult r0 = compressed_level<false, K, PlainCoords, true>(ops, 0, R, total_unscaled, seg0_lo, seg0_hi,
                                                                           W, p, no_shift);
            R -= r0.c;
            int64_t tot1 = 0;
#pragma unroll
            for (int t = 0; t < K; ++t) {
                p0[t] = 0;
                seg_lo[t] = seg_hi[t] = 0;
                if (t < k) {
                    p0[t] = p[t];
                    const int32_t *pos1 = ops.lvl[t][1].pos;
                    const bool present = p[t] < seg0_hi[t] && (int64_t)ops.lvl[t][0].crd[p[t]] == r0.x;
                    seg_lo[t] = pos1[p[t]];
                    seg_hi[t] = present ? pos1[p[t] + 1] : seg_lo[t];
                    tot1 += ops.lvl[t][2].pos[seg_hi[t]] - ops.lvl[t][2].pos[seg_lo[t]];
                }
            }
            Windows<K> W1;
            windows_init<false, K>(ops, 1, seg_lo, seg_hi, W1);
            LevelResult r1 = compressed_level<false, K>(ops, 1, R, tot1, seg_lo, seg_hi, W1, p, no_shift);
            R -= r1.c;
            int64_t tot2 = 0;
#pragma unroll
            for (int t = 0; t < K; ++t) {
                p1[t] = 0;
                if (t < k) {
                    p1[t] = p[t];
                    const int32_t *pos2 = ops.lvl[t][2].pos;
                    const bool present = p[t] < seg_hi[t] && (int64_t)ops.lvl[t][1].crd[p[t]] == r1.x;
                    const int lo2 = pos2[p[t]];
                    seg_hi[t] = present ? pos2[p[t] + 1] : lo2;     // (level-1 bounds are used up)
                    seg_lo[t] = lo2;
                    tot2 += seg_hi[t] - seg_lo[t];
                } else {
                    seg_lo[t] = seg_hi[t] = 0;
                }
            }
            Windows<K> W2;
            windows_init<true, K>(ops, 2, seg_lo, seg_hi, W2);
            LevelResult r2 = compressed_level<true, K>(ops, 2, R, tot2, seg_lo, seg_hi, W2, p, no_shift);
            R -= r2.c;
            if (lane == 0) {
                cb[0] = (int32_t)r0.x;
                cb[1] = (int32_t)r1.x;
                cb[2] = (int32_t)r2.x;
#pragma unroll
                for (int t = 0; t < K; ++t)
                    if (t < k) {
                        pb[t * 3 + 0] = p0[t];
                        pb[t * 3 + 1] = p1[t];
                        pb[t * 3 + 2] = p[t];
                    }
            }
        } else if (d == 1) {
            Windows<K> W = W0;
            LevelResult r = compressed_level<true, K>(ops, 0, R, total_unscaled, seg0_lo, seg0_hi, W, p, no_shift);
            R -= r.c;
#pragma unroll
            for (int t = 0; t < K; ++t)
                if (t < k) found[t] = p[t];
            if (lane == 0) {
                cb[0] = (int32_t)r.x;
#pragma unroll
                for (int t = 0; t < K; ++t)
                    if (t < k) pb[t] = p[t];
            }
        } else {
            LevelResult r0;
            if (dense0) r0 = dense_search<K>(ops, 0, R, p);
            else {
                Windows<K> W = W0;
                r0 = compressed_level<false, K>(ops, 0, R, total_unscaled, seg0_lo, seg0_hi, W, p, no_shift);
            }
            R -= r0.c;
            int p0[K], sh[K];
#pragma unroll
            for (int t = 0; t < K; ++t) {
                p0[t] = 0;
                sh[t] = 0;
                seg_lo[t] = seg_hi[t] = 0;
                if (t < k) {
                    p0[t] = p[t];
                    const DevLevel &L0 = ops.lvl[t][0];
                    const int32_t *pos1 = ops.lvl[t][1].pos;
                    bool present;
                    if (dense0) present = r0.x < L0.extent;
                    else present = p[t] < seg0_hi[t] && (int64_t)L0.crd[p[t]] == r0.x;
                    const int lo1 = pos1[p[t]];
                    seg_lo[t] = lo1;
                    seg_hi[t] = present ? pos1[p[t] + 1] : lo1;
                    if (present && ops.start[t]) sh[t] = ops.start[t][p[t]] - lo1;   // remapped row
                }
            }
            Windows<K> W1;
            windows_init<true, K>(ops, 1, seg_lo, seg_hi, W1);
            const int64_t tot1 = level_total<true, K>(ops, 1, seg_lo, seg_hi);
            LevelResult r1 = compressed_level<true, K>(ops, 1, R, tot1, seg_lo, seg_hi, W1, p, sh);
            R -= r1.c;
            if (lane == 0) {
                cb[0] = (int32_t)r0.x;
                cb[1] = (int32_t)r1.x;
#pragma unroll
                for (int t = 0; t < K; ++t)
                    if (t < k) {
                        pb[t * 2 + 0] = p0[t];
                        pb[t * 2 + 1] = p[t];
                    }
            }
        }
        if (lane == 0) cost[b] = (Qu - R) * cost_scale;
    }
}

}  // namespace

}  // namespace nacho
