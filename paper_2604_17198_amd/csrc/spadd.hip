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
// The union is formed by cross-ranking instead of a serial k-finger merge: the
// work per entry is constant, every lane works on its own entries, and the only
// data-dependent loops are binary searches of fixed depth done by the SMALLER
// run of every pair of runs.
// Per partition the wavefront
//   1. stages the operands' coordinate segments in LDS as k sorted runs of keys
//      (vectors: the index; matrices: row<<32 | column, the row of every entry
//      recovered from the pos array with a marker + running-maximum scan);
//   2. ranks: for every pair of runs the entries of the smaller run search the
//      larger one.  The position found is the number of entries of the larger
//      run that precede the entry in the stable k-way merge (ties in operand
//      order); it also leaves a mark at the first entry of the larger run that
//      comes after it, so one prefix sum over the marks gives every entry of
//      the larger run the number of smaller-run entries before it.  An entry
//      that meets an equal key in an operand with a smaller index is flagged as
//      a duplicate.  Own position + searched positions + summed marks = the
//      entry's slot in the merged order; a 16-bit descriptor (run, position in
//      the run, duplicate flag) is scattered to that slot;
//   3. assembly: walks the merged order; a slot that is not a duplicate is the
//      HEAD of its coordinate.  The number of heads is the partition's output
//      count (and a head whose predecessor lies in another row starts a row);
//   4. prefix sum: publishes its counts and adds up the counts of all earlier
//      partitions with a decoupled look-back over a state word per workgroup;
//   5. compute: walks the merged order again and writes, for every head,
//      coordinate and value (its own value plus the duplicates that follow it,
//      i.e. in operand order) at offset + rank, and the hierarchical arrays
//      (crd0/pos1 of a DCSR result, pos of a CSR result) for the rows whose
//      first output entry the partition owns -- exactly one writer per row.
// What differs from the paper's three kernels: the inputs are read once instead
// of twice and there is no separate scan launch; the arithmetic is the same.
//
// The grid is persistent: at most as many workgroups as the device can hold at
// once, workgroup b taking groups b, b + grid, b + 2 grid, ...  Every group a
// look-back waits for is therefore owned by a resident workgroup that reaches it
// before anything later, so the waits end without an atomic hand-out of work.
#include "common.hpp"
#include "kernels.hpp"

namespace nacho {

namespace {

template <int FMT> struct KeyOf { typedef uint64_t type; };
template <> struct KeyOf<SPADD_VECTOR> { typedef uint32_t type; };

template <int FMT> struct Cap { static constexpr int value = kSpaddCapMatrix; };
template <> struct Cap<SPADD_VECTOR> { static constexpr int value = kSpaddCapVector; };

// state word of a workgroup: bits 63..62 status, 61..31 rows, 30..0 nnz
constexpr unsigned long long kStatusShift = 62;
constexpr unsigned long long kAggregate = 1ull, kInclusive = 2ull;
constexpr int kSpinLimit = 1 << 20;   // look-back polls before a wavefront gives up
constexpr int kWavesPerGroup = 4;     // partitions per workgroup (one look-back for all of them)
constexpr int kLook = 8;              // predecessors a lane examines per look-back round

__device__ inline unsigned long long pack_state(unsigned long long status, long long rows, long long nnz)
{
    return (status << kStatusShift) | ((unsigned long long)rows << 31) | (unsigned long long)nnz;
}

__device__ inline int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

template <typename KeyT> __device__ inline uint32_t row_of(KeyT k) { return (uint32_t)((uint64_t)k >> 32); }

// Number of keys of the sorted run seg[0, n) that are smaller than key[i], for
// NI keys per lane at once (n >= 1, the same for all lanes).  Binary lifting:
// the loop count depends on n only, and the NI chains of LDS reads overlap.
template <typename KeyT, int NI>
__device__ inline void run_lower_bound(const KeyT *seg, int n, const KeyT (&key)[NI], int (&lb)[NI])
{
#pragma unroll
    for (int i = 0; i < NI; ++i) lb[i] = 0;
    for (int step = 1 << (31 - __builtin_clz((unsigned)n)); step > 0; step >>= 1) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int j = lb[i] + step;
            const KeyT v = seg[(j <= n ? j : n) - 1];
            lb[i] = (j <= n && v < key[i]) ? j : lb[i];
        }
    }
}

// Per-wavefront LDS state of one partition.
constexpr int kPadShift = 4;    // one unused word after every 16: a lane's 16 consecutive words start on its own bank
template <int CAP> struct Padded { static constexpr int value = CAP + (CAP >> kPadShift); };
__device__ inline int pad(int x) { return x + (x >> kPadShift); }

template <typename KeyT, int CAP>
struct WaveTile {
    KeyT keys[CAP];                       // the k runs, one after the other
    int32_t marks[Padded<CAP>::value];    // staging: row markers; then marks -> their prefix sum; then heads before a slot
    uint16_t direct[CAP];                 // searched positions of an entry (bits 0..14) | duplicate (bit 15)
    uint16_t info[CAP];                   // merged order: position in keys (0..9) | run (11..13) | duplicate (15)
    unsigned long long sval[NACHO_MAX_OPERANDS];   // address of the value of run t's first entry
    int32_t soff[NACHO_MAX_OPERANDS + 1];          // start of run t in keys
};
static_assert(kSpaddCapVector <= 1024 && kSpaddCapMatrix <= 1024, "info packs a 10-bit position");

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

// Is run u the larger one of the pair (t, u)?  (Ties: the higher index.)
__device__ inline bool larger_run(int nu, int u, int nt, int t) { return nu > nt || (nu == nt && u > t); }

// Ranking of NI consecutive 64-entry blocks of run t, starting at entry r0:
// searches in every larger run.
template <typename KeyT, int NI, typename Tile>
__device__ inline void rank_blocks(Tile &w, int k, int t, int r0, int lane)
{
    const int off_t = uni(w.soff[t]), nt = uni(w.soff[t + 1]) - off_t;
    KeyT key[NI];
    bool valid[NI];
    int direct[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int il = r0 + i * NACHO_WAVE + lane;
        valid[i] = il < nt;
        key[i] = valid[i] ? w.keys[off_t + il] : KeyT(0);
        direct[i] = 0;
    }
    for (int u = 0; u < k; ++u) {
        const int off_u = uni(w.soff[u]), nu = uni(w.soff[u + 1]) - off_u;
        if (u == t || !larger_run(nu, u, nt, t)) continue;
        int lb[NI];
        run_lower_bound<KeyT, NI>(w.keys + off_u, nu, key, lb);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const KeyT at = w.keys[off_u + (lb[i] < nu ? lb[i] : nu - 1)];
            const int eq = (lb[i] < nu && at == key[i]) ? 1 : 0;
            if (u < t) {
                // run u wins ties: its equal entry precedes this one, which is a duplicate
                direct[i] += lb[i] + eq;
                direct[i] |= eq << 15;
                if (valid[i] && lb[i] + eq < nu) atomicAdd(&w.marks[pad(off_u + lb[i] + eq)], 1);
            } else {
                // this entry precedes u's entries from position lb on; an equal one there is a duplicate
                direct[i] += lb[i];
                if (valid[i] && lb[i] < nu) atomicAdd(&w.marks[pad(off_u + lb[i])], 1 + (eq << 16));
            }
        }
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int il = r0 + i * NACHO_WAVE + lane;
        if (valid[i]) w.direct[off_t + il] = (uint16_t)direct[i];
    }
}

template <int FMT, typename T>
__global__ void __launch_bounds__(kWavesPerGroup * NACHO_WAVE)
spadd_kernel(DevOperands ops, SpaddValues vals, int64_t P, int64_t n_groups,
             const int32_t *__restrict__ coord, const int32_t *__restrict__ posn,
             unsigned long long *__restrict__ tile_state, SpaddOut out)
{
    typedef typename KeyOf<FMT>::type KeyT;
    constexpr int CAP = Cap<FMT>::value;
    constexpr int D = FMT == SPADD_VECTOR ? 1 : 2;
    constexpr int U = 8;                       // global loads in flight per lane and batch
    constexpr int PER_LANE = CAP / NACHO_WAVE; // consecutive entries a lane scans
    typedef WaveTile<KeyT, CAP> Tile;
    // every wavefront of the workgroup owns a private slice of LDS and works on
    // its own partition; only the look-back is shared
    __shared__ Tile s_tile[kWavesPerGroup];
    __shared__ unsigned long long s_cnt[2][kWavesPerGroup];   // per-wavefront counts (rows<<31 | nnz)
    __shared__ unsigned long long s_base[2];                  // the workgroup's exclusive prefix

    const int lane = lane_id();
    const int wave = threadIdx.x / NACHO_WAVE;
    const int k = ops.k;
    const unsigned long long below = (1ull << lane) - 1ull;
    Tile &w = s_tile[wave];
    KeyT *keys = w.keys;
    int parity = 0;

    for (int64_t group = blockIdx.x; group < n_groups; group += gridDim.x, parity ^= 1) {
        const int64_t p = group * kWavesPerGroup + wave;
        const bool active = p < P;             // idle wavefronts of the last workgroup only keep the barriers

        // ---- 1. segments of this partition ----------------------------------
        int q_lo[NACHO_MAX_OPERANDS], off[NACHO_MAX_OPERANDS + 1];
        off[0] = 0;
#pragma unroll
        for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
            if (t >= k || !active) { off[t + 1] = off[t]; q_lo[t] = 0; continue; }
            q_lo[t] = posn[(p * k + t) * D + (D - 1)];
            const int q_hi = posn[((p + 1) * k + t) * D + (D - 1)];
            off[t + 1] = off[t] + (q_hi - q_lo[t]);
        }
        int n = off[NACHO_MAX_OPERANDS];       // <= CAP by the host's choice of the partition count
        // Only an operand that violates its preconditions (unsorted or repeated
        // coordinates) can overflow the staging buffer: such a partition contributes
        // nothing and the call reports INVALID_ARG, but the look-back chain goes on.
        bool broken = n > CAP || n < 0;
#pragma unroll
        for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) broken = broken || off[t + 1] < off[t];
        if (broken) {
            n = 0;
#pragma unroll
            for (int t = 0; t <= NACHO_MAX_OPERANDS; ++t) off[t] = 0;
        }
        wave_sync();                           // the previous partition's LDS reads are done
#pragma unroll
        for (int t = 0; t <= NACHO_MAX_OPERANDS; ++t) {
            if (lane == 0) {
                w.soff[t] = off[t];
                if (t < NACHO_MAX_OPERANDS)
                    w.sval[t] = (unsigned long long)(uintptr_t)(static_cast<const T *>(vals.v[t]) + q_lo[t]);
            }
        }

#pragma unroll
        for (int t = 0; t < NACHO_MAX_OPERANDS; ++t) {
            if (t >= k) break;
            const int nt = off[t + 1] - off[t];
            const int32_t *crd = ops.lvl[t][D - 1].crd + q_lo[t];
            KeyT *kb = keys + off[t];
            if (D == 2) {
                // rows overlapping [q_lo, q_hi): mark each row's first entry, then a running maximum
                const int32_t *pos1 = ops.lvl[t][1].pos;
                const int32_t *crd0 = ops.lvl[t][0].crd;
                const int ql = q_lo[t], qh = ql + nt;
                int32_t *mark = w.marks + off[t];
                for (int i = lane; i < nt; i += NACHO_WAVE) mark[i] = 0;
                wave_sync();
                if (nt > 0) {
                    const int i_lo = posn[(p * k + t) * 2 + 0];
                    int i_hi = posn[((p + 1) * k + t) * 2 + 0] + 1;
                    const int i_max = FMT == SPADD_CSR ? (int)ops.lvl[t][0].extent : (int)ops.lvl[t][0].count;
                    if (i_hi > i_max) i_hi = i_max;
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
                }
                wave_sync();
                const int chunk = (nt + NACHO_WAVE - 1) / NACHO_WAVE;
                const int c0 = lane * chunk < nt ? lane * chunk : nt;
                const int c1 = c0 + chunk < nt ? c0 + chunk : nt;
                int run = 0;
                for (int i = c0; i < c1; ++i) run = max(run, mark[i]);
                int incl = run;                           // inclusive running maximum over lanes
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
            const int32_t *mark = w.marks + (D == 2 ? off[t] : 0);
            for (int i0 = lane; i0 < nt; i0 += NACHO_WAVE * U) {
                int c[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int i = i0 + u * NACHO_WAVE;
                    if (i < nt) c[u] = crd[i];
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int i = i0 + u * NACHO_WAVE;
                    if (i < nt) {
                        if (D == 1) kb[i] = (KeyT)(uint32_t)c[u];
                        else kb[i] = (KeyT)(((uint64_t)(uint32_t)(mark[i] - 1) << 32) | (uint32_t)c[u]);
                    }
                }
            }
        }
        wave_sync();

        // ---- 2. ranks: slot of every entry in the merged order -----------------------
        for (int i = lane; i < Padded<CAP>::value; i += NACHO_WAVE) w.marks[i] = 0;
        wave_sync();
        int n_max = 0, t_max = 0;              // the largest run searches nothing
        for (int t = 0; t < k; ++t) {
            const int nt = uni(w.soff[t + 1]) - uni(w.soff[t]);
            if (t == 0 || larger_run(nt, t, n_max, t_max)) { n_max = nt; t_max = t; }
        }
        for (int t = 0; t < k; ++t) {
            if (t == t_max) continue;
            const int nt = uni(w.soff[t + 1]) - uni(w.soff[t]);
            int r0 = 0;
            for (; r0 + 2 * NACHO_WAVE < nt; r0 += 4 * NACHO_WAVE) rank_blocks<KeyT, 4>(w, k, t, r0, lane);
            for (; r0 < nt; r0 += NACHO_WAVE) rank_blocks<KeyT, 1>(w, k, t, r0, lane);
        }
        wave_sync();
        {
            // inclusive prefix sum of the marks (low halves) over all runs at once; a
            // lane owns PER_LANE consecutive words, the flags in the high halves stay
            int v[PER_LANE], sum = 0;
            const int at = lane * (PER_LANE + (PER_LANE >> kPadShift));
#pragma unroll
            for (int j = 0; j < PER_LANE; ++j) {
                v[j] = w.marks[at + j];
                sum += v[j] & 0xffff;
            }
            int run = wave_inclusive_scan(sum) - sum;
#pragma unroll
            for (int j = 0; j < PER_LANE; ++j) {
                run += v[j] & 0xffff;
                w.marks[at + j] = (v[j] & 0xffff0000) | run;
            }
        }
        wave_sync();
        for (int t = 0; t < k; ++t) {
            const int off_t = uni(w.soff[t]), nt = uni(w.soff[t + 1]) - off_t;
            const int before_run = off_t > 0 ? (w.marks[pad(off_t - 1)] & 0xffff) : 0;
            for (int il = lane; il < nt; il += NACHO_WAVE) {
                const int c = off_t + il;
                const int mk = w.marks[pad(c)];
                const int d = t == t_max ? 0 : (int)w.direct[c];
                const int slot = il + (d & 0x7fff) + ((mk & 0xffff) - before_run);
                const int dup = ((d >> 15) | ((unsigned)mk >> 16)) != 0 ? 1 : 0;
                w.info[slot] = (uint16_t)(c | (t << 11) | (dup << 15));
            }
        }
        wave_sync();

        // ---- 3. assembly: count heads and row heads -------------------------------------
        bool cont = false;                 // the partition starts inside a row whose head is elsewhere
        if (D == 2 && active) cont = row_continues<FMT>(ops, coord, posn, p);
        int heads = 0, rheads = 0;
        for (int i0 = 0; i0 < n; i0 += NACHO_WAVE) {
            const int i = i0 + lane;
            const bool valid = i < n;
            const int inf = valid ? (int)w.info[i] : 0x8000;
            const bool head = !(inf >> 15);
            heads += __popcll(__ballot(head));
            if (FMT == SPADD_DCSR) {
                const uint32_t row = row_of(keys[inf & 1023]);
                const uint32_t prow = (valid && i > 0) ? row_of(keys[w.info[i - 1] & 1023]) : 0u;
                const bool rhead = head && (i == 0 ? !cont : row != prow);
                rheads += __popcll(__ballot(rhead));
            }
        }

        // ---- 4. prefix sum: one decoupled look-back per workgroup ------------------
        // The wavefronts pool their counts; wavefront 0 publishes the workgroup's
        // aggregate, walks back over earlier workgroups' state words (64 per round,
        // nearest first) up to the nearest known inclusive prefix, and publishes its
        // own inclusive prefix.
        if (lane == 0) s_cnt[parity][wave] = pack_state(0, rheads, heads);
        __syncthreads();
        if (wave == 0) {
            unsigned long long tot = 0;
#pragma unroll
            for (int ww = 0; ww < kWavesPerGroup; ++ww) tot += s_cnt[parity][ww];
            long long b_rows = 0, b_nnz = 0;
            bool gave_up = false;
            if (group > 0) {
                if (lane == 0)
                    __hip_atomic_store(&tile_state[group], (kAggregate << kStatusShift) | tot, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                // Every round looks at the kLook * 64 nearest predecessors not yet summed,
                // lane L at the kLook consecutive ones from first - L * kLook downwards,
                // all loads in flight together: when many workgroups start at the same
                // time none of them has an inclusive prefix to offer, and the sum has to
                // reach far back.
                int64_t first = group - 1;
                int spins = 0;
                for (;;) {
                    unsigned long long s[kLook];
#pragma unroll
                    for (int j = 0; j < kLook; ++j) {
                        const int64_t g = first - ((int64_t)lane * kLook + j);
                        s[j] = pack_state(kInclusive, 0, 0);                 // before group 0: nothing
                        if (g >= 0) s[j] = __hip_atomic_load(&tile_state[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    // per lane: states up to and including its nearest inclusive one
                    long long l_nnz = 0, l_rows = 0;
                    bool l_incl = false, l_missing = false;
#pragma unroll
                    for (int j = 0; j < kLook; ++j) {
                        const unsigned long long st = s[j] >> kStatusShift;
                        if (!l_incl) {
                            if (st == 0) l_missing = true;
                            l_nnz += (long long)(s[j] & 0x7fffffffull);
                            l_rows += (long long)((s[j] >> 31) & 0x7fffffffull);
                            if (st == kInclusive) l_incl = true;
                        }
                    }
                    const unsigned long long incl = __ballot(l_incl);
                    const int stop = incl ? __ffsll((long long)incl) - 1 : NACHO_WAVE;   // lane of the nearest inclusive
                    const unsigned long long need = stop >= NACHO_WAVE - 1 ? ~0ull : ((2ull << stop) - 1);
                    if (__ballot(l_missing) & need) {          // a needed predecessor has not published yet
                        if (++spins > kSpinLimit) { gave_up = true; break; }
                        __builtin_amdgcn_s_sleep(4);
                        continue;
                    }
                    const bool use = lane <= stop;
                    b_nnz += wave_sum<long long>(use ? l_nnz : 0ll);
                    b_rows += wave_sum<long long>(use ? l_rows : 0ll);
                    if (stop < NACHO_WAVE) break;
                    first -= NACHO_WAVE * kLook;
                }
            }
            const long long t_nnz = (long long)(tot & 0x7fffffffull), t_rows = (long long)((tot >> 31) & 0x7fffffffull);
            if (lane == 0) {
                __hip_atomic_store(&tile_state[group], pack_state(kInclusive, b_rows + t_rows, b_nnz + t_nnz),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_base[parity] = pack_state(0, b_rows, b_nnz);
                if (gave_up) *out.status = NACHO_ERR_HIP;
                if (group == n_groups - 1) {
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
        unsigned long long mine = s_base[parity];
#pragma unroll
        for (int ww = 0; ww < kWavesPerGroup; ++ww)
            if (ww < wave) mine += s_cnt[parity][ww];
        const long long base_nnz = (long long)(mine & 0x7fffffffull);
        const long long base_rows = (long long)((mine >> 31) & 0x7fffffffull);
        if (broken && lane == 0) *out.status = NACHO_ERR_INVALID_ARG;
        if (!active) continue;

        // ---- 5. compute: write the partition's output ------------------------------
        int hcount = 0, rcount = 0;
        for (int i0 = 0; i0 < n; i0 += NACHO_WAVE) {
            const int i = i0 + lane;
            const bool valid = i < n;
            const int inf = valid ? (int)w.info[i] : 0x8000;
            const bool head = !(inf >> 15);
            const unsigned long long hm = __ballot(head);
            const int j = hcount + __popcll(hm & below);
            const KeyT key = keys[inf & 1023];
            bool rhead = false;
            int jr = 0;
            if (FMT == SPADD_DCSR) {
                const uint32_t prow = (valid && i > 0) ? row_of(keys[w.info[i - 1] & 1023]) : 0u;
                rhead = head && (i == 0 ? !cont : row_of(key) != prow);
                const unsigned long long rm = __ballot(rhead);
                jr = rcount + __popcll(rm & below);
                rcount += __popcll(rm);
            }
            if (FMT == SPADD_CSR && valid) w.marks[i] = j;      // heads before slot i
            if (head) {
                // the head's own value, then its duplicates in merged (= operand) order
                const int t = (inf >> 11) & 7;
                T sum = reinterpret_cast<const T *>((uintptr_t)w.sval[t])[(inf & 1023) - w.soff[t]];
                for (int g = i + 1; g < n; ++g) {
                    const int ig = w.info[g];
                    if (!(ig >> 15)) break;
                    const int tg = (ig >> 11) & 7;
                    sum += reinterpret_cast<const T *>((uintptr_t)w.sval[tg])[(ig & 1023) - w.soff[tg]];
                }
                const long long wpos = base_nnz + j;
                if (wpos < out.cap_nnz) {
                    out.crd1[wpos] = (int32_t)(uint32_t)key;
                    static_cast<T *>(out.val)[wpos] = sum;
                }
                if (FMT == SPADD_DCSR && rhead) {
                    const long long wr = base_rows + jr;
                    if (wr < out.cap_rows) {
                        out.crd0[wr] = (int32_t)row_of(key);
                        out.pos1[wr] = (int32_t)wpos;
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
                int l = 0, h = n;
                while (l < h) {
                    const int m = (l + h) >> 1;
                    if (row_of(keys[w.info[m] & 1023]) < (uint32_t)r) l = m + 1; else h = m;
                }
                out.pos1[r] = (int32_t)(base_nnz + (l < n ? w.marks[l] : heads));
            }
        }
    }
}

// Clears the look-back state of a call: one state word per workgroup, and the status.
__global__ void __launch_bounds__(256)
spadd_reset_kernel(int64_t n_groups, unsigned long long *__restrict__ tile_state,
                   int32_t *__restrict__ status)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_groups) tile_state[i] = 0ull;
    if (i == 0) *status = NACHO_OK;
}

// Workgroups of this kernel the device holds at once (per device, asked once).
template <int FMT, typename T>
int64_t resident_groups()
{
    static int64_t cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, spadd_kernel<FMT, T>,
                                                         kWavesPerGroup * NACHO_WAVE, 0) != hipSuccess)
            return 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cached[dev] = (int64_t)per_cu * cus;
    }
    return cached[dev];
}

template <int FMT, typename T>
hipError_t launch_one(const DevOperands &ops, const SpaddValues &vals, int64_t P, const int32_t *coord,
                      const int32_t *posn, unsigned long long *tile_state, const SpaddOut &out, hipStream_t s)
{
    const int64_t n_groups = (P + kWavesPerGroup - 1) / kWavesPerGroup;
    const int64_t resident = resident_groups<FMT, T>();
    if (resident < 1) return hipErrorUnknown;
    const unsigned grid = (unsigned)(n_groups < resident ? n_groups : resident);
    hipLaunchKernelGGL((spadd_kernel<FMT, T>), dim3(grid), dim3(kWavesPerGroup * NACHO_WAVE), 0, s, ops, vals,
                       P, n_groups, coord, posn, tile_state, out);
    return hipGetLastError();
}

}  // namespace

int spadd_capacity(int fmt) { return fmt == SPADD_VECTOR ? kSpaddCapVector : kSpaddCapMatrix; }

int64_t spadd_groups(int64_t P) { return (P + kWavesPerGroup - 1) / kWavesPerGroup; }

hipError_t launch_spadd_reset(int64_t P, unsigned long long *tile_state, int32_t *status, hipStream_t s)
{
    const int64_t n_groups = spadd_groups(P);
    const unsigned grid = (unsigned)((n_groups + 255) / 256);
    hipLaunchKernelGGL(spadd_reset_kernel, dim3(grid ? grid : 1), dim3(256), 0, s, n_groups, tile_state, status);
    return hipGetLastError();
}

hipError_t launch_spadd(int fmt, int dtype, const DevOperands &ops, const SpaddValues &vals, int64_t P,
                        const int32_t *coord, const int32_t *posn, unsigned long long *tile_state,
                        const SpaddOut &out, hipStream_t s)
{
#define NACHO_SPADD_CASE(F)                                                                          \
    if (fmt == F) {                                                                                  \
        if (dtype == NACHO_F64) return launch_one<F, double>(ops, vals, P, coord, posn, tile_state, out, s); \
        return launch_one<F, float>(ops, vals, P, coord, posn, tile_state, out, s);                  \
    }
    NACHO_SPADD_CASE(SPADD_VECTOR)
    NACHO_SPADD_CASE(SPADD_CSR)
    NACHO_SPADD_CASE(SPADD_DCSR)
#undef NACHO_SPADD_CASE
    return hipErrorInvalidValue;
}

}  // namespace nacho
