// k-way sparse union addition: assembly (count), prefix sum, compute (fill)
// -- Section 4.3 and 4.4, pipeline of Figure 7(a) -- one wavefront per partition.
//
// A partition owns, in every operand t, the stored entries at last-level
// positions [q_t(p), q_t(p+1)) found by the partition search; because the
// search runs in coordinate space, entries with equal coordinates in different
// operands always fall in the same partition (Section 6, merge-path paragraph),
// so a partition's output is independent of its neighbours: there is no carry.
//
// Per partition the wavefront
//   1. stages the operands' coordinate segments in LDS as sorted runs of keys
//      (vectors: the index; matrices: row<<32 | column, the row of every entry
//      recovered from the pos array with a marker + running-maximum scan);
//   2. merges the k runs with a tree of stable two-way merges (merge-path split
//      per lane, serial merge of each lane's share), ties kept in operand order;
//   3. marks the first entry of every group of equal keys; the number of marks
//      is the partition's output count (assembly), their prefix ranks are the
//      write offsets inside the partition (compute);
//   4. in the compute pass writes coordinate and the sum of the group's values
//      (added in operand order) at partition_offset + rank, and the hierarchical
//      arrays (crd0/pos1 of a DCSR result, pos of a CSR result) for the rows
//      whose first output entry it owns -- one writer per row.
#include "common.hpp"
#include "kernels.hpp"

namespace nacho {

namespace {

template <int FMT> struct KeyOf { typedef uint64_t type; };
template <> struct KeyOf<SPADD_VECTOR> { typedef uint32_t type; };

template <int FMT> struct Cap { static constexpr int value = kSpaddCapMatrix; };
template <> struct Cap<SPADD_VECTOR> { static constexpr int value = kSpaddCapVector; };

// Stable two-way merge of the adjacent sorted runs [lo, mid) and [mid, hi) of
// (sk, sp) into the same range of (dk, dp).  Every lane finds the merge-path
// split of its first output and merges its share serially.
template <typename KeyT>
__device__ inline void merge_runs(const KeyT *sk, const uint16_t *sp, KeyT *dk, uint16_t *dp,
                                  int lo, int mid, int hi, int lane)
{
    const int nA = mid - lo, nB = hi - mid, n = nA + nB;
    const KeyT *A = sk + lo, *B = sk + mid;
    const int vt = (n + NACHO_WAVE - 1) / NACHO_WAVE;
    int d0 = lane * vt;
    if (d0 > n) d0 = n;
    int d1 = d0 + vt;
    if (d1 > n) d1 = n;
    int l = d0 - nB > 0 ? d0 - nB : 0, h = d0 < nA ? d0 : nA;
    while (l < h) {
        const int m = (l + h) >> 1;
        if (A[m] <= B[d0 - 1 - m]) l = m + 1; else h = m;
    }
    int i = l, j = d0 - l;
    KeyT ka = i < nA ? A[i] : KeyT(0), kb = j < nB ? B[j] : KeyT(0);
    for (int o = d0; o < d1; ++o) {
        const bool takeA = (j >= nB) || (i < nA && ka <= kb);
        dk[lo + o] = takeA ? ka : kb;
        dp[lo + o] = takeA ? sp[lo + i] : sp[mid + j];
        if (takeA) { ++i; if (i < nA) ka = A[i]; }
        else { ++j; if (j < nB) kb = B[j]; }
    }
}

// Does boundary b fall strictly inside a row, i.e. does some operand hold an
// entry of the boundary's row before the boundary?  (Then the row's first
// output entry belongs to an earlier partition.)
template <int FMT>
__device__ inline bool row_continues(const DevOperands &ops, const int32_t *coord, const int32_t *posn,
                                     int64_t b)
{
    const int k = ops.k;
    const int x0 = coord[b * 2];
    bool cont = false;
    for (int t = 0; t < k; ++t) {
        const int i0 = posn[(b * k + t) * 2 + 0];
        const int q = posn[(b * k + t) * 2 + 1];
        bool present;
        if (FMT == SPADD_CSR) present = (int64_t)x0 < ops.lvl[t][0].extent;
        else present = (int64_t)i0 < ops.lvl[t][0].count && ops.lvl[t][0].crd[i0] == x0;
        if (present && q > ops.lvl[t][1].pos[i0]) cont = true;
    }
    return cont;
}

template <int FMT, typename T, bool kFill>
__global__ void __launch_bounds__(NACHO_WAVE)
spadd_kernel(DevOperands ops, SpaddValues vals, MergePlan plan,
             const int32_t *__restrict__ coord, const int32_t *__restrict__ posn,
             int32_t *__restrict__ cnt_nnz, int32_t *__restrict__ cnt_rows,   // count: out; fill: exclusive offsets
             SpaddOut out)
{
    typedef typename KeyOf<FMT>::type KeyT;
    constexpr int CAP = Cap<FMT>::value;
    constexpr int D = FMT == SPADD_VECTOR ? 1 : 2;
    __shared__ KeyT keys[2][CAP];
    __shared__ uint16_t pay[2][CAP];
    __shared__ int32_t rowtmp[FMT == SPADD_VECTOR ? 1 : CAP];
    __shared__ int32_t soff[NACHO_MAX_OPERANDS + 1];

    const int64_t p = blockIdx.x;
    const int lane = threadIdx.x;
    const int k = ops.k;

    // ---- 1. segments of this partition --------------------------------------
    int q_lo[NACHO_MAX_OPERANDS], off[NACHO_MAX_OPERANDS + 1];
    off[0] = 0;
#pragma unroll
    for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
        if (t >= k) { off[t + 1] = off[t]; q_lo[t] = 0; continue; }
        q_lo[t] = posn[(p * k + t) * D + (D - 1)];
        const int q_hi = posn[((p + 1) * k + t) * D + (D - 1)];
        off[t + 1] = off[t] + (q_hi - q_lo[t]);
    }
    int n = 0;                     // <= CAP by the host's choice of the partition count
#pragma unroll
    for (int t = 0; t <= NACHO_MAX_OPERANDS; ++t) {
        if (lane == 0) soff[t] = off[t];
        if (t == k) n = off[t];
    }

    if (n > CAP || n < 0) {
        // only possible when an operand violates its preconditions (unsorted or
        // repeated coordinates): refuse the partition instead of overrunning LDS
        if (lane == 0) {
            if (kFill) *out.status = NACHO_ERR_INVALID_ARG;
            else { cnt_nnz[p] = 0; if (FMT == SPADD_DCSR) cnt_rows[p] = 0; }
        }
        return;
    }
#pragma unroll
    for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
        if (t >= k) break;
        const int nt = off[t + 1] - off[t];
        const int32_t *crd = ops.lvl[t][D - 1].crd;
        KeyT *kb = keys[plan.leaf_buf[t]] + off[t];
        uint16_t *pb = pay[plan.leaf_buf[t]] + off[t];
        if (D == 1) {
            for (int i = lane; i < nt; i += NACHO_WAVE) {
                kb[i] = (KeyT)(uint32_t)crd[q_lo[t] + i];
                pb[i] = (uint16_t)(off[t] + i);
            }
        } else {
            // rows overlapping [q_lo, q_hi): mark each row's first entry, then a running maximum
            const int32_t *pos1 = ops.lvl[t][1].pos;
            const int qh = q_lo[t] + nt;
            const int i_lo = posn[(p * k + t) * 2 + 0];
            int i_hi = posn[((p + 1) * k + t) * 2 + 0] + 1;
            const int i_max = FMT == SPADD_CSR ? (int)ops.lvl[t][0].extent : (int)ops.lvl[t][0].count;
            if (i_hi > i_max) i_hi = i_max;
            int32_t *mark = rowtmp + off[t];
            for (int i = lane; i < nt; i += NACHO_WAVE) mark[i] = 0;
            __syncthreads();
            if (nt > 0)
                for (int i = i_lo + lane; i < i_hi; i += NACHO_WAVE) {
                    const int a = pos1[i], b = pos1[i + 1];
                    const int s = a > q_lo[t] ? a : q_lo[t];
                    if (b > s && s < qh) {
                        const int row = FMT == SPADD_CSR ? i : ops.lvl[t][0].crd[i];
                        mark[s - q_lo[t]] = row + 1;
                    }
                }
            __syncthreads();
            const int chunk = (nt + NACHO_WAVE - 1) / NACHO_WAVE;
            const int c0 = lane * chunk < nt ? lane * chunk : nt;
            const int c1 = c0 + chunk < nt ? c0 + chunk : nt;
            int run = 0;
            for (int i = c0; i < c1; ++i) run = max(run, mark[i]);
            int incl = run;                               // inclusive running maximum over lanes
#pragma unroll
            for (int o = 1; o < NACHO_WAVE; o <<= 1) {
                const int v = __shfl_up(incl, o, NACHO_WAVE);
                if (lane >= o) incl = max(incl, v);
            }
            int before = __shfl_up(incl, 1, NACHO_WAVE);
            if (lane == 0) before = 0;
            run = before;
            for (int i = c0; i < c1; ++i) {
                run = max(run, mark[i]);
                const uint32_t row = (uint32_t)(run - 1);
                kb[i] = (KeyT)(((uint64_t)row << 32) | (uint32_t)crd[q_lo[t] + i]);
                pb[i] = (uint16_t)(off[t] + i);
            }
            __syncthreads();
        }
    }
    __syncthreads();

    // ---- 2. merge tree --------------------------------------------------------
    for (int e = 0; e < plan.n_nodes; ++e) {
        const int ob = plan.out_buf[e];
        merge_runs<KeyT>(keys[1 - ob], pay[1 - ob], keys[ob], pay[ob],
                         soff[plan.a[e]], soff[plan.m[e]], soff[plan.b[e]], lane);
        __syncthreads();
    }
    const KeyT *mk = keys[0];
    const uint16_t *mp = pay[0];

    // ---- 3./4. heads, ranks, output -------------------------------------------
    bool cont = false;                 // the partition starts inside a row whose head is elsewhere
    if (D == 2) cont = row_continues<FMT>(ops, coord, posn, p);
    const int64_t base_nnz = kFill ? (int64_t)cnt_nnz[p] : 0;
    const int64_t base_rows = (kFill && FMT == SPADD_DCSR) ? (int64_t)cnt_rows[p] : 0;
    int heads = 0, rheads = 0;
    for (int i0 = 0; i0 < n; i0 += NACHO_WAVE) {
        const int i = i0 + lane;
        const bool valid = i < n;
        const KeyT key = valid ? mk[i] : KeyT(0);
        const KeyT prev = (valid && i > 0) ? mk[i - 1] : KeyT(0);
        const bool head = valid && (i == 0 || key != prev);
        const unsigned long long hm = __ballot(head);
        const int j = heads + __popcll(hm & ((1ull << lane) - 1));
        bool rhead = false;
        int jr = 0;
        if (FMT == SPADD_DCSR) {
            rhead = head && (i == 0 ? !cont : (uint32_t)(key >> 32) != (uint32_t)((uint64_t)prev >> 32));
            const unsigned long long rm = __ballot(rhead);
            jr = rheads + __popcll(rm & ((1ull << lane) - 1));
            rheads += __popcll(rm);
        }
        if (kFill && FMT == SPADD_CSR && valid) rowtmp[i] = j;   // heads before item i
        if (kFill && head) {
            // sum of the group, in operand order (the merge is stable)
            T sum = T(0);
            int g = i;
            do {
                const int idx = mp[g];
                int t_off = 0, t_q = q_lo[0];
                const void *t_v = vals.v[0];
#pragma unroll
                for (int s = 1; s < NACHO_MAX_OPERANDS; ++s)
                    if (s < k && idx >= off[s]) { t_off = off[s]; t_q = q_lo[s]; t_v = vals.v[s]; }
                sum += static_cast<const T *>(t_v)[t_q + (idx - t_off)];
                ++g;
            } while (g < n && mk[g] == key);
            const int64_t w = base_nnz + j;
            if (w < out.cap_nnz) {
                out.crd1[w] = (int32_t)(uint32_t)key;
                static_cast<T *>(out.val)[w] = sum;
            }
            if (FMT == SPADD_DCSR && rhead) {
                const int64_t wr = base_rows + jr;
                if (wr < out.cap_rows) {
                    out.crd0[wr] = (int32_t)(uint32_t)((uint64_t)key >> 32);
                    out.pos1[wr] = (int32_t)w;
                }
            }
        }
        heads += __popcll(hm);
    }
    if (!kFill) {
        if (lane == 0) {
            cnt_nnz[p] = heads;
            if (FMT == SPADD_DCSR) cnt_rows[p] = rheads;
        }
        return;
    }
    if (FMT == SPADD_CSR) {
        // pos of every row that starts inside this partition: offset of the first
        // output entry whose row is not smaller
        __syncthreads();
        const int first = coord[p * 2] + (cont ? 1 : 0);
        const int next_first = coord[(p + 1) * 2] + (row_continues<FMT>(ops, coord, posn, p + 1) ? 1 : 0);
        for (int r = first + lane; r < next_first; r += NACHO_WAVE) {
            const KeyT want = (KeyT)((uint64_t)(uint32_t)r << 32);
            int l = 0, h = n;
            while (l < h) {
                const int m = (l + h) >> 1;
                if (mk[m] < want) l = m + 1; else h = m;
            }
            out.pos1[r] = (int32_t)(base_nnz + (l < n ? rowtmp[l] : heads));
        }
    }
}

// Exclusive prefix sums of the per-partition counts (in place), totals, output
// tails and the capacity check.  One workgroup.
__global__ void __launch_bounds__(1024)
spadd_scan_kernel(int fmt, int64_t P, int32_t *__restrict__ cnt_nnz, int32_t *__restrict__ cnt_rows,
                  int64_t n_rows, SpaddOut out)
{
    __shared__ long long part_nnz[1024];
    __shared__ long long part_rows[1024];
    const int tid = threadIdx.x;
    const int64_t chunk = (P + 1023) / 1024;
    const int64_t b = (int64_t)tid * chunk < P ? (int64_t)tid * chunk : P;
    const int64_t e = b + chunk < P ? b + chunk : P;
    long long s_nnz = 0, s_rows = 0;
    for (int64_t i = b; i < e; ++i) {
        s_nnz += cnt_nnz[i];
        if (fmt == SPADD_DCSR) s_rows += cnt_rows[i];
    }
    part_nnz[tid] = s_nnz;
    part_rows[tid] = s_rows;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {          // Hillis-Steele inclusive scan
        long long a = 0, r = 0;
        if (tid >= o) { a = part_nnz[tid - o]; r = part_rows[tid - o]; }
        __syncthreads();
        part_nnz[tid] += a;
        part_rows[tid] += r;
        __syncthreads();
    }
    long long run_nnz = part_nnz[tid] - s_nnz, run_rows = part_rows[tid] - s_rows;
    for (int64_t i = b; i < e; ++i) {
        const int c = cnt_nnz[i];
        cnt_nnz[i] = (int32_t)run_nnz;
        run_nnz += c;
        if (fmt == SPADD_DCSR) {
            const int r = cnt_rows[i];
            cnt_rows[i] = (int32_t)run_rows;
            run_rows += r;
        }
    }
    if (tid == 1023) {
        const long long total_nnz = part_nnz[1023];
        const long long total_rows = fmt == SPADD_DCSR ? part_rows[1023] : (fmt == SPADD_CSR ? n_rows : 1);
        out.counts[0] = total_rows;
        out.counts[1] = total_nnz;
        const bool fits = total_nnz <= out.cap_nnz && (fmt != SPADD_DCSR || total_rows <= out.cap_rows);
        *out.status = fits ? NACHO_OK : NACHO_ERR_CAPACITY;
        if (fmt == SPADD_VECTOR) { out.pos1[0] = 0; out.pos1[1] = (int32_t)total_nnz; }
        if (fmt == SPADD_CSR) out.pos1[n_rows] = (int32_t)total_nnz;
        if (fmt == SPADD_DCSR) {
            out.pos0[0] = 0;
            out.pos0[1] = (int32_t)total_rows;
            if (total_rows <= out.cap_rows) out.pos1[total_rows] = (int32_t)total_nnz;
        }
    }
}

template <int FMT, typename T>
void launch_pair(bool fill, const DevOperands &ops, const SpaddValues &vals, const MergePlan &plan,
                 const int32_t *coord, const int32_t *posn, int64_t P, int32_t *cnt_nnz,
                 int32_t *cnt_rows, const SpaddOut &out, hipStream_t s)
{
    if (fill)
        hipLaunchKernelGGL((spadd_kernel<FMT, T, true>), dim3((unsigned)P), dim3(NACHO_WAVE), 0, s, ops,
                           vals, plan, coord, posn, cnt_nnz, cnt_rows, out);
    else
        hipLaunchKernelGGL((spadd_kernel<FMT, T, false>), dim3((unsigned)P), dim3(NACHO_WAVE), 0, s, ops,
                           vals, plan, coord, posn, cnt_nnz, cnt_rows, out);
}

}  // namespace

int spadd_capacity(int fmt) { return fmt == SPADD_VECTOR ? kSpaddCapVector : kSpaddCapMatrix; }

hipError_t launch_spadd_pass(bool fill, int fmt, int dtype, const DevOperands &ops,
                             const SpaddValues &vals, const MergePlan &plan, const int32_t *coord,
                             const int32_t *posn, int64_t P, int32_t *cnt_nnz, int32_t *cnt_rows,
                             const SpaddOut &out, hipStream_t s)
{
#define NACHO_SPADD_CASE(F)                                                                          \
    if (fmt == F) {                                                                                  \
        if (dtype == NACHO_F64) launch_pair<F, double>(fill, ops, vals, plan, coord, posn, P, cnt_nnz, cnt_rows, out, s); \
        else launch_pair<F, float>(fill, ops, vals, plan, coord, posn, P, cnt_nnz, cnt_rows, out, s); \
    }
    NACHO_SPADD_CASE(SPADD_VECTOR)
    NACHO_SPADD_CASE(SPADD_CSR)
    NACHO_SPADD_CASE(SPADD_DCSR)
#undef NACHO_SPADD_CASE
    return hipGetLastError();
}

hipError_t launch_spadd_scan(int fmt, int64_t P, int32_t *cnt_nnz, int32_t *cnt_rows, int64_t n_rows,
                             const SpaddOut &out, hipStream_t s)
{
    hipLaunchKernelGGL(spadd_scan_kernel, dim3(1), dim3(1024), 0, s, fmt, P, cnt_nnz, cnt_rows, n_rows, out);
    return hipGetLastError();
}

}  // namespace nacho
