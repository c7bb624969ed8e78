// k-way sparse union addition: assembly (count), prefix sum and compute (fill)
// of Section 4.3 / 4.4 (pipeline of Figure 7(a)) in ONE kernel, one wavefront
// per partition.
//
// A partition owns, in every operand t, the stored entries at last-level
// positions [q_t(p), q_t(p+1)) found by the partition search; because the
// search runs in coordinate space, entries with equal coordinates in different
// operands always fall in the same partition (Section 6, merge-path paragraph),
// so a partition's output is independent of its neighbours: there is no carry.
//
// Per partition the wavefront
//   1. stages the operands' coordinate segments (and values) in LDS as sorted
//      runs of keys (vectors: the index; matrices: row<<32 | column, the row of
//      every entry recovered from the pos array with a marker + running-maximum
//      scan); all global loads are issued in batches before they are consumed;
//   2. merges the k runs with a tree of stable two-way merges (merge-path split
//      per lane, serial merge of each lane's share), ties kept in operand order;
//   3. assembly: marks the first entry of every group of equal keys; the number
//      of marks is the partition's output count (and the number of rows whose
//      first output entry lies in the partition);
//   4. prefix sum: publishes its counts and adds up the counts of all earlier
//      partitions with a decoupled look-back over a per-partition state word
//      (partitions are handed out through an atomic ticket, so every partition a
//      wavefront waits for has already started; the wait is bounded anyway);
//   5. compute: writes coordinate and the sum of each group's values (added in
//      operand order) at offset + rank, and the hierarchical arrays (crd0/pos1 of
//      a DCSR result, pos of a CSR result) for the rows whose first output entry
//      it owns -- exactly one writer per row.
// What differs from the paper's three kernels: the inputs are read once instead
// of twice and there is no separate scan launch; the arithmetic is the same.
#include "common.hpp"
#include "kernels.hpp"

namespace nacho {

namespace {

template <int FMT> struct KeyOf { typedef uint64_t type; };
template <> struct KeyOf<SPADD_VECTOR> { typedef uint32_t type; };

template <int FMT> struct Cap { static constexpr int value = kSpaddCapMatrix; };
template <> struct Cap<SPADD_VECTOR> { static constexpr int value = kSpaddCapVector; };

// state word of a partition: bits 63..62 status, 61..31 rows, 30..0 nnz
constexpr unsigned long long kStatusShift = 62;
constexpr unsigned long long kAggregate = 1ull, kInclusive = 2ull;
constexpr int kSpinLimit = 1 << 20;   // look-back polls before a wavefront gives up
constexpr int kWavesPerGroup = 4;     // partitions handed out per ticket

__device__ inline unsigned long long pack_state(unsigned long long status, long long rows, long long nnz)
{
    return (status << kStatusShift) | ((unsigned long long)rows << 31) | (unsigned long long)nnz;
}

// Stable two-way merge of the adjacent sorted runs [lo, mid) and [mid, hi) of
// (sk, sv) into the same range of (dk, dv).  Every lane finds the merge-path
// split of its first output and merges its share serially.
template <typename KeyT, typename T>
__device__ inline void merge_runs(const KeyT *sk, const T *sv, KeyT *dk, T *dv,
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
        dv[lo + o] = takeA ? sv[lo + i] : sv[mid + j];
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

template <int FMT, typename T>
__global__ void __launch_bounds__(kWavesPerGroup * NACHO_WAVE)
spadd_kernel(DevOperands ops, SpaddValues vals, MergePlan plan, int64_t P,
             const int32_t *__restrict__ coord, const int32_t *__restrict__ posn,
             unsigned long long *__restrict__ tile_state, unsigned int *__restrict__ ticket,
             SpaddOut out)
{
    typedef typename KeyOf<FMT>::type KeyT;
    constexpr int CAP = Cap<FMT>::value;
    constexpr int D = FMT == SPADD_VECTOR ? 1 : 2;
    constexpr int U = 8;                       // global loads in flight per lane and batch
    // every wavefront of the workgroup owns a private slice of LDS and works on
    // its own partition; only the ticket is shared
    __shared__ KeyT s_keys[kWavesPerGroup][2][CAP];
    __shared__ T s_lval[kWavesPerGroup][2][CAP];
    __shared__ int32_t s_rowtmp[kWavesPerGroup][FMT == SPADD_VECTOR ? 1 : CAP];
    __shared__ int32_t s_soff[kWavesPerGroup][NACHO_MAX_OPERANDS + 1];
    __shared__ unsigned int s_tile;
    __shared__ unsigned long long s_cnt[kWavesPerGroup];   // per-wavefront counts (rows<<31 | nnz)
    __shared__ unsigned long long s_base;                  // the workgroup's exclusive prefix

    const int lane = lane_id();
    const int wave = threadIdx.x / NACHO_WAVE;
    const int k = ops.k;
    // One ticket per workgroup hands out kWavesPerGroup consecutive partitions:
    // a partition's predecessors belong to workgroups that drew earlier tickets
    // (or to earlier wavefronts of the same workgroup), so they are all running.
    if (threadIdx.x == 0) s_tile = atomicAdd(ticket, 1u);
    __syncthreads();
    const int64_t group = s_tile;
    const int64_t p = group * kWavesPerGroup + wave;
    const bool active = p < P;                 // idle wavefronts of the last workgroup only keep the barriers
    KeyT (*keys)[CAP] = s_keys[wave];
    T (*lval)[CAP] = s_lval[wave];
    int32_t *rowtmp = s_rowtmp[wave];
    int32_t *soff = s_soff[wave];

    // ---- 1. segments of this partition --------------------------------------
    int q_lo[NACHO_MAX_OPERANDS], off[NACHO_MAX_OPERANDS + 1];
    off[0] = 0;
#pragma unroll
    for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
        if (t >= k || !active) { off[t + 1] = off[t]; q_lo[t] = 0; continue; }
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
    // Only an operand that violates its preconditions (unsorted or repeated
    // coordinates) can overflow the staging buffer: such a partition contributes
    // nothing and the call reports INVALID_ARG, but the look-back chain goes on.
    const bool broken = n > CAP || n < 0;
    if (broken) n = 0;

#pragma unroll
    for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
        if (t >= k) break;
        const int nt = broken ? 0 : off[t + 1] - off[t];
        const int32_t *crd = ops.lvl[t][D - 1].crd + q_lo[t];
        const T *val = static_cast<const T *>(vals.v[t]) + q_lo[t];
        KeyT *kb = keys[plan.leaf_buf[t]] + off[t];
        T *vb = lval[plan.leaf_buf[t]] + off[t];
        if (D == 2) {
            // rows overlapping [q_lo, q_hi): mark each row's first entry, then a running maximum
            const int32_t *pos1 = ops.lvl[t][1].pos;
            const int32_t *crd0 = ops.lvl[t][0].crd;
            const int ql = q_lo[t], qh = ql + nt;
            const int i_lo = posn[(p * k + t) * 2 + 0];
            int i_hi = posn[((p + 1) * k + t) * 2 + 0] + 1;
            const int i_max = FMT == SPADD_CSR ? (int)ops.lvl[t][0].extent : (int)ops.lvl[t][0].count;
            if (i_hi > i_max) i_hi = i_max;
            int32_t *mark = rowtmp + off[t];
            for (int i = lane; i < nt; i += NACHO_WAVE) mark[i] = 0;
            wave_sync();
            if (nt > 0)
                for (int i0 = i_lo + lane; i0 < i_hi; i0 += NACHO_WAVE * 4) {
                    int a[4], b[4], row[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int i = i0 + u * NACHO_WAVE;
                        if (i < i_hi) {
                            a[u] = pos1[i];
                            b[u] = pos1[i + 1];
                            row[u] = FMT == SPADD_CSR ? i : crd0[i];
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int i = i0 + u * NACHO_WAVE;
                        if (i < i_hi) {
                            const int s = a[u] > ql ? a[u] : ql;
                            if (b[u] > s && s < qh) mark[s - ql] = row[u] + 1;
                        }
                    }
                }
            wave_sync();
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
                mark[i] = run;
            }
            wave_sync();
        }
        const int32_t *mark = rowtmp + (D == 2 ? off[t] : 0);
        for (int i0 = lane; i0 < nt; i0 += NACHO_WAVE * U) {
            int c[U];
            T v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u * NACHO_WAVE;
                if (i < nt) { c[u] = crd[i]; v[u] = val[i]; }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u * NACHO_WAVE;
                if (i < nt) {
                    if (D == 1) kb[i] = (KeyT)(uint32_t)c[u];
                    else kb[i] = (KeyT)(((uint64_t)(uint32_t)(mark[i] - 1) << 32) | (uint32_t)c[u]);
                    vb[i] = v[u];
                }
            }
        }
    }
    wave_sync();

    // ---- 2. merge tree --------------------------------------------------------
    if (!broken)
        for (int e = 0; e < plan.n_nodes; ++e) {
            const int ob = plan.out_buf[e];
            merge_runs<KeyT, T>(keys[1 - ob], lval[1 - ob], keys[ob], lval[ob],
                                soff[plan.a[e]], soff[plan.m[e]], soff[plan.b[e]], lane);
            wave_sync();
        }
    const KeyT *mk = keys[0];
    const T *mv = lval[0];

    // ---- 3. assembly: count group heads and row heads ---------------------------
    bool cont = false;                 // the partition starts inside a row whose head is elsewhere
    if (D == 2 && active) cont = row_continues<FMT>(ops, coord, posn, p);
    int heads = 0, rheads = 0;
    for (int i0 = 0; i0 < n; i0 += NACHO_WAVE) {
        const int i = i0 + lane;
        const bool valid = i < n;
        const KeyT key = valid ? mk[i] : KeyT(0);
        const KeyT prev = (valid && i > 0) ? mk[i - 1] : KeyT(0);
        const bool head = valid && (i == 0 || key != prev);
        heads += __popcll(__ballot(head));
        if (FMT == SPADD_DCSR) {
            const bool rhead = head && (i == 0 ? !cont : (uint32_t)((uint64_t)key >> 32) != (uint32_t)((uint64_t)prev >> 32));
            rheads += __popcll(__ballot(rhead));
        }
    }

    // ---- 4. prefix sum: one decoupled look-back per workgroup ---------------------
    // The wavefronts pool their counts; wavefront 0 publishes the workgroup's
    // aggregate, walks back over earlier workgroups' state words (64 per round,
    // nearest first) up to the nearest known inclusive prefix, and publishes its
    // own inclusive prefix.
    if (lane == 0) s_cnt[wave] = pack_state(0, rheads, heads);
    __syncthreads();
    if (wave == 0) {
        unsigned long long tot = 0;
#pragma unroll
        for (int w = 0; w < kWavesPerGroup; ++w) tot += s_cnt[w];
        long long b_rows = 0, b_nnz = 0;
        bool gave_up = false;
        if (group > 0) {
            if (lane == 0)
                __hip_atomic_store(&tile_state[group], (kAggregate << kStatusShift) | tot, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            int64_t first = group - 1;      // lane L looks at workgroup first - L
            int spins = 0;
            for (;;) {
                const int64_t j = first - lane;
                unsigned long long s = pack_state(kInclusive, 0, 0);     // before workgroup 0: nothing
                if (j >= 0) s = __hip_atomic_load(&tile_state[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const unsigned long long st = s >> kStatusShift;
                const unsigned long long incl = __ballot(st == kInclusive);
                const int stop = incl ? __ffsll((long long)incl) - 1 : NACHO_WAVE;   // nearest inclusive
                const unsigned long long need = stop >= NACHO_WAVE - 1 ? ~0ull : ((2ull << stop) - 1);
                if (__ballot(st == 0) & need) {            // a needed predecessor has not published yet
                    if (++spins > kSpinLimit) { gave_up = true; break; }
                    __builtin_amdgcn_s_sleep(8);
                    continue;
                }
                const bool use = lane <= stop;
                b_nnz += wave_sum<long long>(use ? (long long)(s & 0x7fffffffull) : 0ll);
                b_rows += wave_sum<long long>(use ? (long long)((s >> 31) & 0x7fffffffull) : 0ll);
                if (stop < NACHO_WAVE) break;
                first -= NACHO_WAVE;
            }
        }
        const long long t_nnz = (long long)(tot & 0x7fffffffull), t_rows = (long long)((tot >> 31) & 0x7fffffffull);
        if (lane == 0) {
            __hip_atomic_store(&tile_state[group], pack_state(kInclusive, b_rows + t_rows, b_nnz + t_nnz),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_base = pack_state(0, b_rows, b_nnz);
            if (gave_up) *out.status = NACHO_ERR_HIP;
            if (group == (P + kWavesPerGroup - 1) / kWavesPerGroup - 1) {
                // totals, tails and the capacity verdict (the only writer of these words)
                const long long total_nnz = b_nnz + t_nnz;
                const long long total_rows = FMT == SPADD_DCSR ? b_rows + t_rows
                                                               : (FMT == SPADD_CSR ? ops.lvl[0][0].extent : 1);
                out.counts[0] = total_rows;
                out.counts[1] = total_nnz;
                const bool fits = total_nnz <= out.cap_nnz && (FMT != SPADD_DCSR || total_rows <= out.cap_rows);
                if (!fits) *out.status = NACHO_ERR_CAPACITY;
                if (FMT == SPADD_VECTOR) { out.pos1[0] = 0; out.pos1[1] = (int32_t)total_nnz; }
                if (FMT == SPADD_CSR) out.pos1[ops.lvl[0][0].extent] = (int32_t)total_nnz;
                if (FMT == SPADD_DCSR) {
                    out.pos0[0] = 0;
                    out.pos0[1] = (int32_t)total_rows;
                    if (total_rows <= out.cap_rows) out.pos1[total_rows] = (int32_t)total_nnz;
                }
            }
        }
    }
    __syncthreads();
    unsigned long long mine = s_base;
#pragma unroll
    for (int w = 0; w < kWavesPerGroup; ++w)
        if (w < wave) mine += s_cnt[w];
    const long long base_nnz = (long long)(mine & 0x7fffffffull);
    const long long base_rows = (long long)((mine >> 31) & 0x7fffffffull);
    if (broken && lane == 0) *out.status = NACHO_ERR_INVALID_ARG;
    if (!active) return;                       // no barrier below this point

    // ---- 5. compute: write the partition's output ------------------------------
    int hcount = 0, rcount = 0;
    for (int i0 = 0; i0 < n; i0 += NACHO_WAVE) {
        const int i = i0 + lane;
        const bool valid = i < n;
        const KeyT key = valid ? mk[i] : KeyT(0);
        const KeyT prev = (valid && i > 0) ? mk[i - 1] : KeyT(0);
        const bool head = valid && (i == 0 || key != prev);
        const unsigned long long hm = __ballot(head);
        const int j = hcount + __popcll(hm & ((1ull << lane) - 1));
        bool rhead = false;
        int jr = 0;
        if (FMT == SPADD_DCSR) {
            rhead = head && (i == 0 ? !cont : (uint32_t)((uint64_t)key >> 32) != (uint32_t)((uint64_t)prev >> 32));
            const unsigned long long rm = __ballot(rhead);
            jr = rcount + __popcll(rm & ((1ull << lane) - 1));
            rcount += __popcll(rm);
        }
        if (FMT == SPADD_CSR && valid) rowtmp[i] = j;       // heads before item i
        if (head) {
            T sum = mv[i];                                  // group sum in operand order (stable merge)
            for (int g = i + 1; g < n && mk[g] == key; ++g) sum += mv[g];
            const long long w = base_nnz + j;
            if (w < out.cap_nnz) {
                out.crd1[w] = (int32_t)(uint32_t)key;
                static_cast<T *>(out.val)[w] = sum;
            }
            if (FMT == SPADD_DCSR && rhead) {
                const long long wr = base_rows + jr;
                if (wr < out.cap_rows) {
                    out.crd0[wr] = (int32_t)(uint32_t)((uint64_t)key >> 32);
                    out.pos1[wr] = (int32_t)w;
                }
            }
        }
        hcount += __popcll(hm);
    }
    if (FMT == SPADD_CSR) {
        // pos of every row that starts inside this partition: offset of the first
        // output entry whose row is not smaller
        wave_sync();
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

// Clears the look-back state of a call: P state words, the ticket and the status.
__global__ void __launch_bounds__(256)
spadd_reset_kernel(int64_t P, unsigned long long *__restrict__ tile_state,
                   unsigned int *__restrict__ ticket, int32_t *__restrict__ status)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < P) tile_state[i] = 0ull;
    if (i == 0) { *ticket = 0u; *status = NACHO_OK; }
}

template <int FMT, typename T>
void launch_one(const DevOperands &ops, const SpaddValues &vals, const MergePlan &plan, int64_t P,
                const int32_t *coord, const int32_t *posn, unsigned long long *tile_state,
                unsigned int *ticket, const SpaddOut &out, hipStream_t s)
{
    const unsigned grid = (unsigned)((P + kWavesPerGroup - 1) / kWavesPerGroup);
    hipLaunchKernelGGL((spadd_kernel<FMT, T>), dim3(grid), dim3(kWavesPerGroup * NACHO_WAVE), 0, s, ops, vals,
                       plan, P, coord, posn, tile_state, ticket, out);
}

}  // namespace

int spadd_capacity(int fmt) { return fmt == SPADD_VECTOR ? kSpaddCapVector : kSpaddCapMatrix; }

hipError_t launch_spadd_reset(int64_t P, unsigned long long *tile_state, unsigned int *ticket,
                              int32_t *status, hipStream_t s)
{
    const unsigned grid = (unsigned)((P + 255) / 256);
    hipLaunchKernelGGL(spadd_reset_kernel, dim3(grid ? grid : 1), dim3(256), 0, s, P, tile_state, ticket, status);
    return hipGetLastError();
}

hipError_t launch_spadd(int fmt, int dtype, const DevOperands &ops, const SpaddValues &vals,
                        const MergePlan &plan, int64_t P, const int32_t *coord, const int32_t *posn,
                        unsigned long long *tile_state, unsigned int *ticket, const SpaddOut &out,
                        hipStream_t s)
{
#define NACHO_SPADD_CASE(F)                                                                          \
    if (fmt == F) {                                                                                  \
        if (dtype == NACHO_F64) launch_one<F, double>(ops, vals, plan, P, coord, posn, tile_state, ticket, out, s); \
        else launch_one<F, float>(ops, vals, plan, P, coord, posn, tile_state, ticket, out, s);      \
    }
    NACHO_SPADD_CASE(SPADD_VECTOR)
    NACHO_SPADD_CASE(SPADD_CSR)
    NACHO_SPADD_CASE(SPADD_DCSR)
#undef NACHO_SPADD_CASE
    return hipGetLastError();
}

}  // namespace nacho
