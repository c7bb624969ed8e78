// k-way sparse union addition: assembly (count), prefix sum and compute (fill)
// of Section 4.3 / 4.4 (pipeline of Figure 7(a)) in ONE kernel, one workgroup
// of eight wavefronts per partition.
//
// A partition owns, in every operand t, the stored entries at last-level
// positions [q_t(p), q_t(p+1)) found by the partition search; because the
// search runs in coordinate space, entries with equal coordinates in different
// operands always fall in the same partition (Section 6, merge-path paragraph),
// so a partition's output is independent of its neighbours: there is no carry.
// Inside the workgroup the entries are dealt out thread by thread (entry c of
// the partition belongs to thread c mod 512), so the eight wavefronts carry
// exactly the same load whatever the operands look like.
//
// The union is formed by cross-ranking instead of a serial k-finger merge: the
// work per entry is constant, every lane works on its own entries, and the only
// data-dependent loops are binary searches of fixed depth done by the SMALLER
// run of every pair of runs.
// Per partition the workgroup
//   1. stages the operands' coordinate segments in LDS as k sorted runs of keys
//      (vectors: the index; matrices: row<<32 | column, the row of every entry
//      recovered from the pos array with a marker + latest-marker scan, or read
//      from the stored rows of a coordinate list);
//   2. ranks: for every pair of runs the entries of the smaller run search the
//      larger one.  The position found is the number of entries of the larger
//      run that precede the entry in the stable k-way merge (ties in operand
//      order); it also leaves a mark at the first entry of the larger run that
//      comes after it, so one prefix sum over the marks gives every entry of
//      the larger run the number of smaller-run entries before it.  An entry
//      that meets an equal key in an operand with a smaller index is flagged as
//      a duplicate.  Own position + searched positions + summed marks = the
//      entry's slot in the merged order; a 16-bit descriptor (position in the
//      runs, duplicate flag) is scattered to that slot.  The partition's output
//      counts are known at this point already (an entry is emitted iff no
//      earlier operand stores its key; DCSR: the searches also settle which
//      entry starts a row) and are published for the prefix sum right away;
//   3. assembly: walks the merged order; a slot that is not a duplicate is the
//      HEAD of its coordinate (and a head whose predecessor lies in another row
//      starts a row); every slot keeps the number of heads (and row heads)
//      before it;
//   4. prefix sum: reads the counts of everything before the partition (two
//      levels, see below; requested before the assembly, consumed after it);
//      the loads of the values are in flight meanwhile;
//   5. compute: every thread goes back to its own entries (values in its
//      registers, coordinates re-read from the keys).  A head writes coordinate and value at
//      offset + heads before its slot; its value is its own plus the
//      duplicates in the slots that follow it, i.e. in operand order
//      (duplicates hand their values over through LDS).  The hierarchical
//      arrays (crd0/pos1 of a DCSR result, pos of a CSR result) are written for
//      the rows whose first output entry the partition owns -- exactly one
//      writer per row.
// Every loop over a partition's entries is unrolled over the 8 entries of a
// thread, so that the LDS and global accesses of a stage are in flight together.
// What differs from the paper's three kernels: the inputs are read once instead
// of twice and there is no separate scan launch; the arithmetic is the same.
//
// Workgroup p handles partition p and waits, when it looks up its offset, only
// for workgroups with a smaller index.  Workgroups are handed to every XCD in
// index order, so the unfinished workgroup with the smallest index is always
// running and waits for nobody: the waits end.  (Every wait is bounded all the
// same; a wavefront that gives up reports NACHO_ERR_HIP.)
#include "common.hpp"
#include "kernels.hpp"

namespace nacho {

namespace {

template <int FMT> struct KeyOf { typedef uint64_t type; };
template <> struct KeyOf<SPADD_VECTOR> { typedef uint32_t type; };

constexpr int kWaves = 8;                          // wavefronts per workgroup
constexpr int kThreads = kWaves * NACHO_WAVE;
constexpr int kPerThread = 8;                      // entries of a thread: c = r * kThreads + tid, r < kPerThread
constexpr int kTile = kThreads * kPerThread;       // entries a partition may hold
static_assert(kTile == kSpaddCap, "capacity told to the host");
static_assert(kTile <= 4096, "descriptors pack a 12-bit position");

// Prefix sum over the workgroups' counts, two levels and no chains: a workgroup
// publishes the counts of its partition in a 32-bit word; the last workgroup
// of every chunk of kChunk workgroups also publishes the chunk's total.  The
// offset of a workgroup is the sum of the totals of the chunks before its own
// plus the sum of the words of the workgroups before it in its chunk: all of
// them plain reads of words that their owners publish without waiting for
// anybody (a word) or after one such wait (a total).
//   word:  bit 31 published, bits 14..27 rows, bits 0..13 nnz
//   total: bit 63 published, bits 31..61 rows, bits 0..30 nnz
constexpr int kChunk = 512;           // workgroups per chunk
constexpr int kSpinLimit = 1 << 20;   // polls before a wavefront gives up
constexpr unsigned kWordValid = 0x80000000u;
constexpr unsigned long long kTotalValid = 1ull << 63;

__device__ inline unsigned long long pack_counts(long long rows, long long nnz)
{
    return ((unsigned long long)rows << 31) | (unsigned long long)nnz;
}

__device__ inline int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

template <typename KeyT> __device__ inline uint32_t row_of(KeyT k) { return (uint32_t)((uint64_t)k >> 32); }

// Number of keys of the sorted run seg[0, n) that are smaller than key[i], for
// NI keys per lane at once (n >= 1, the same for all lanes).  Quaternary lifting
// (32-bit keys):
// every level tries to advance by one, two or three steps (three independent LDS
// reads), the steps shrink by four from level to level -- floor(log4 n) + 1
// dependent rounds instead of floor(log2 n) + 1, and what a partition's ranking
// costs is the length of that chain.  The loop count depends on n only.
template <typename KeyT, int NI>
__device__ inline void run_lower_bound(const KeyT *seg, int n, const KeyT (&key)[NI], int (&lb)[NI])
{
#pragma unroll
    for (int i = 0; i < NI; ++i) lb[i] = 0;
    if (sizeof(KeyT) == 8) {
        // 64-bit keys: three probes per level would cost the registers that keep three
        // workgroups on a CU; plain binary lifting
        for (int step = 1 << (31 - __builtin_clz((unsigned)n)); step > 0; step >>= 1) {
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int j = lb[i] + step;
                const KeyT v = seg[(j <= n ? j : n) - 1];
                lb[i] = (j <= n && v < key[i]) ? j : lb[i];
            }
        }
        return;
    }
    for (int step = 1 << ((31 - __builtin_clz((unsigned)n)) & ~1); step > 0; step >>= 2) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int j1 = lb[i] + step, j2 = j1 + step, j3 = j2 + step;
            const KeyT v1 = seg[(j1 <= n ? j1 : n) - 1];
            const KeyT v2 = seg[(j2 <= n ? j2 : n) - 1];
            const KeyT v3 = seg[(j3 <= n ? j3 : n) - 1];
            // (the run is sorted: a later probe is below the key only if the earlier ones are)
            const int adv = ((j1 <= n && v1 < key[i]) ? 1 : 0) + ((j2 <= n && v2 < key[i]) ? 1 : 0) +
                            ((j3 <= n && v3 < key[i]) ? 1 : 0);
            lb[i] += adv * step;
        }
    }
}

// LDS state of one partition.
constexpr int kPadShift = 3;    // one unused word after every 8: a thread's 8 consecutive words start on its own bank
static_assert((1 << kPadShift) == kPerThread, "the padding follows the words of a thread");
constexpr int kPadded = kTile + (kTile >> kPadShift);
__device__ inline int pad(int x) { return x + (x >> kPadShift); }

// Word of an entry in `marks` while the ranks are formed:
//   bits  0..15  marks left at this entry by smaller runs (then their prefix sum over the tile)
//   bits 16..19  number of equal keys met in operands with a smaller index (> 0: duplicate)
//   bits 20..31  sum of the positions this entry found in larger runs (< kTile)
constexpr int kDupShift = 16, kDirectShift = 20;
// (the count of equal keys stays below 8: bit 19 is free)
//   bit  19      DCSR: some other run holds an entry of this entry's row that precedes it in the merged order
constexpr uint32_t kRowLater = 1u << 19;
// Word of a merged slot (in the memory of the ranking words, which are dead by then):
//   bits  0..11  position of the slot's entry in keys      } written when the ranks are known
//   bit   12     the entry is a duplicate                  }
//   bits 13..21  emitted entries before the slot           } added by the assembly
//   bits 22..30  row heads before the slot (DCSR)          } (counts inside the slot's wavefront share)
//   bit   31     the slot's entry is emitted
constexpr uint32_t kSlotPos = 0xfffu, kSlotDup = 1u << 12, kSlotEmit = 1u << 31;
constexpr int kSlotHeads = 13, kSlotRows = 22;
static_assert(kTile / kWaves <= 512, "the counts inside a share take 9 bits");
template <typename KeyT, typename T>
struct Tile {
    union {
        KeyT keys[kTile];                 // the k runs, one after the other
        T dupval[sizeof(T) <= sizeof(KeyT) ? kTile : 1];   // later: values of duplicates by merged slot
    };
    T dupval_wide[sizeof(T) <= sizeof(KeyT) ? 1 : kTile];
    uint32_t marks[kPadded];              // staging: row markers; ranking words (padded); slot words
    unsigned long long scrd[NACHO_MAX_OPERANDS];   // address of crd of run t, biased so that [c] is entry c of keys
    unsigned long long sval[NACHO_MAX_OPERANDS];   // the same for the values
    unsigned long long sstart[NACHO_MAX_OPERANDS]; // remapped operands: address of start[t] and of pos of run t
    unsigned long long spos[NACHO_MAX_OPERANDS];
    int32_t soff[NACHO_MAX_OPERANDS + 1];          // start of run t in keys
    uint32_t srun[NACHO_MAX_OPERANDS];             // start of run t | marks summed before it << 16
    uint32_t wave_x[kWaves];                       // per-wavefront partial of a scan across the workgroup
    uint32_t emit_total;                           // emitted entries | rows started << 16 (known after the ranking)
    unsigned long long wave_cnt[kWaves];           // per-wavefront counts of the assembly (rows << 31 | nnz)
    unsigned long long share_off[kWaves + 1];      // offset of every wavefront's share of the merged order
                                                   // (rows << 31 | nnz; the last one: end of the partition)
    __device__ T *dups() { return sizeof(T) <= sizeof(KeyT) ? dupval : dupval_wide; }
};

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

// Ranking of NI consecutive 64-entry blocks of run t, starting at entry r0,
// against the larger run u: one search per entry.
// kRows (DCSR): the searches also settle which entry is the first of its row in the merged
// order.  An entry that finds an entry of its own row right before its place in run u is not;
// and if the entry of u at its place is u's first of that row, that one is not (unless it is the
// same coordinate in an operand with a smaller index, which precedes this entry).
template <typename KeyT, int NI, bool kRows, typename TileT>
__device__ inline void rank_blocks(TileT &w, int t, int u, int r0, int lane)
{
    const int off_t = uni(w.soff[t]), nt = uni(w.soff[t + 1]) - off_t;
    const int off_u = uni(w.soff[u]), nu = uni(w.soff[u + 1]) - off_u;
    KeyT key[NI];
    bool valid[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int il = r0 + i * NACHO_WAVE + lane;
        valid[i] = il < nt;
        key[i] = valid[i] ? w.keys[off_t + il] : KeyT(0);
    }
    int lb[NI];
    run_lower_bound<KeyT, NI>(w.keys + off_u, nu, key, lb);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        if (!valid[i]) continue;
        const int il = r0 + i * NACHO_WAVE + lane;
        const KeyT at = w.keys[off_u + (lb[i] < nu ? lb[i] : nu - 1)];
        const unsigned eq = (lb[i] < nu && at == key[i]) ? 1u : 0u;
        if (kRows) {
            const uint32_t rw = row_of(key[i]);
            const bool row_before = lb[i] > 0 && row_of(w.keys[off_u + lb[i] - 1]) == rw;
            if (row_before) atomicOr(&w.marks[pad(off_t + il)], kRowLater);
            else if (lb[i] < nu && row_of(at) == rw && !(eq && u < t))
                atomicOr(&w.marks[pad(off_u + lb[i])], kRowLater);
        }
        if (u < t) {
            // run u wins ties: its equal entry precedes this one, which is a duplicate
            if (lb[i] + (int)eq < nu) atomicAdd(&w.marks[pad(off_u + lb[i] + (int)eq)], 1u);
            atomicAdd(&w.marks[pad(off_t + il)], (((unsigned)lb[i] + eq) << kDirectShift) + (eq << kDupShift));
        } else {
            // this entry precedes u's entries from position lb on; an equal one there is a duplicate
            if (lb[i] < nu) atomicAdd(&w.marks[pad(off_u + lb[i])], 1u + (eq << kDupShift));
            if (lb[i] > 0) atomicAdd(&w.marks[pad(off_t + il)], (unsigned)lb[i] << kDirectShift);
        }
    }
}

// kMul: the k-way intersection with products (an entry is emitted when all k
// operands store its coordinate, Section 2.1) instead of the union with sums;
// the partitions, the ranks and the prefix sum are the same.
// kMapped: the operands are remapped ones (Section 3.3): CSR over the rows all
// operands store, positions counted over those rows only; the entries of row
// i' of operand t are read from start[t][i'] on.
// (second launch bound, wavefronts per SIMD the register budget must allow: the remapped
// variant is held to the three workgroups per CU that its LDS footprint allows)
template <int FMT, typename T, int K, bool kMul, bool kMapped>
__global__ void __launch_bounds__(kThreads, kMapped ? 6 : 1)
spadd_kernel(DevOperands ops, SpaddValues vals, int64_t P, int64_t n_chunks,
             const int32_t *__restrict__ coord, const int32_t *__restrict__ posn,
             unsigned long long *__restrict__ tile_state, SpaddOut out)
{
    typedef typename KeyOf<FMT>::type KeyT;
    constexpr int D = FMT == SPADD_VECTOR ? 1 : 2;
    constexpr bool kCoo = FMT == SPADD_COO;    // coordinate lists: the row of an entry is stored with it
    constexpr int R = kPerThread;
    constexpr int kShare = kTile / kWaves;     // merged slots a wavefront walks in the assembly
    __shared__ Tile<KeyT, T> w;
    uint32_t *slotw = w.marks;              // slot words (once the ranking words are dead)

    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int wave = tid / NACHO_WAVE;
    const int k = ops.k;                       // <= K
    const unsigned long long below = (1ull << lane) - 1ull;
    KeyT *keys = w.keys;
    const int64_t p = blockIdx.x;              // the partition of this workgroup, p < P

    // ---- 1. segments of this partition ----------------------------------
    int q_lo[K], off[K + 1];
    off[0] = 0;
#pragma unroll
    for (int t = 0; t < K; ++t) {
        if (t >= k) { off[t + 1] = off[t]; q_lo[t] = 0; continue; }
        q_lo[t] = posn[(p * k + t) * D + (D - 1)];
        const int q_hi = posn[((p + 1) * k + t) * D + (D - 1)];
        off[t + 1] = off[t] + (q_hi - q_lo[t]);
    }
    int n = off[K];                            // <= kTile by the host's choice of the partition count
    // Only an operand that violates its preconditions (unsorted or repeated
    // coordinates) can overflow the staging buffer: such a partition contributes
    // nothing and the call reports INVALID_ARG, but the prefix sum goes on.
    bool broken = n > kTile || n < 0;
#pragma unroll
    for (int t = 0; t < K; ++t) broken = broken || off[t + 1] < off[t];
    if (broken) {
        n = 0;
#pragma unroll
        for (int t = 0; t <= K; ++t) off[t] = 0;
    }
    if (tid == 0) {
        w.emit_total = 0;
#pragma unroll
        for (int t = 0; t <= K; ++t) {
            w.soff[t] = off[t];
            if (t < K) {
                const int32_t *crd_t = t < k ? ops.lvl[t][D - 1].crd : nullptr;
                w.scrd[t] = (unsigned long long)(uintptr_t)(crd_t + q_lo[t] - off[t]);
                w.sval[t] = (unsigned long long)(uintptr_t)(static_cast<const T *>(vals.v[t]) + q_lo[t] - off[t]);
                if (kCoo) {
                    const int32_t *rows_t = t < k ? ops.lvl[t][0].crd : nullptr;
                    w.sstart[t] = (unsigned long long)(uintptr_t)(rows_t + q_lo[t] - off[t]);
                }
                if (kMapped) {
                    w.sstart[t] = (unsigned long long)(uintptr_t)(t < k ? ops.start[t] : nullptr);
                    w.spos[t] = (unsigned long long)(uintptr_t)(t < k ? ops.lvl[t][1].pos : nullptr);
                }
            }
        }
    }
    __syncthreads();

    // run and column of every entry of this thread
    int tr[R], col[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int c = r * kThreads + tid;
        int t = 0;
#pragma unroll
        for (int u = 1; u < K; ++u) t += c >= off[u] ? 1 : 0;
        tr[r] = t;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int c = r * kThreads + tid;
        col[r] = 0;
        if (!kMapped && c < n) col[r] = reinterpret_cast<const int32_t *>((uintptr_t)w.scrd[tr[r]])[c];
    }

    uint32_t row[D == 2 ? R : 1];
    unsigned rowfirst = 0;                     // bit j: entry tid * R + j is the first of its row in its run
    if (kCoo) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int c = r * kThreads + tid;
            row[r] = 0;
            if (c < n) row[r] = (uint32_t)reinterpret_cast<const int32_t *>((uintptr_t)w.sstart[tr[r]])[c];
        }
    }
    if (D == 2 && !kCoo) {
        // rows overlapping [q_lo, q_hi) of every run: mark each row's first entry
        // (word of the entry in marks), then hand every entry the latest marker
        // at or before it.  The first entry of every run carries a marker, so no
        // row leaks from one run into the next.
        for (int i = tid; i < kPadded; i += kThreads) w.marks[i] = 0;
        __syncthreads();
#pragma unroll
        for (int t = 0; t < K; ++t) {
            if (t >= k) break;
            const int nt = off[t + 1] - off[t];
            if (nt == 0) continue;
            const int32_t *pos1 = ops.lvl[t][1].pos;
            const int32_t *crd0 = ops.lvl[t][0].crd;
            const int ql = q_lo[t], qh = ql + nt;
            const int i_lo = posn[(p * k + t) * 2 + 0];
            int i_hi = posn[((p + 1) * k + t) * 2 + 0] + 1;
            const int i_max = FMT == SPADD_CSR ? (int)ops.lvl[t][0].extent : (int)ops.lvl[t][0].count;
            if (i_hi > i_max) i_hi = i_max;
            for (int i0 = i_lo + tid; i0 < i_hi; i0 += kThreads * 4) {
                int a[4], b[4], rw[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = i0 + u * kThreads;
                    if (i < i_hi) {
                        a[u] = pos1[i];
                        b[u] = pos1[i + 1];
                        rw[u] = FMT == SPADD_CSR ? i : crd0[i];
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = i0 + u * kThreads;
                    if (i < i_hi) {
                        const int s = a[u] > ql ? a[u] : ql;
                        if (b[u] > s && s < qh) w.marks[pad(off[t] + s - ql)] = (uint32_t)(rw[u] + 1);
                    }
                }
            }
        }
        __syncthreads();
        {
            uint32_t v[R], cur = 0;
            const int at = tid * (R + 1);
#pragma unroll
            for (int j = 0; j < R; ++j) {
                v[j] = w.marks[at + j];
                cur = v[j] ? v[j] : cur;
                if (FMT == SPADD_DCSR && v[j]) rowfirst |= 1u << j;
            }
            uint32_t incl = cur;                      // latest marker up to the end of this thread's words
#pragma unroll
            for (int o = 1; o < NACHO_WAVE; o <<= 1) {
                const uint32_t left = __shfl_up(incl, o, NACHO_WAVE);
                if (lane >= o && incl == 0) incl = left;
            }
            if (lane == NACHO_WAVE - 1) w.wave_x[wave] = incl;
            __syncthreads();
            uint32_t carry = 0;                       // latest marker of the earlier wavefronts
#pragma unroll
            for (int ww = 0; ww < kWaves; ++ww)
                if (ww < wave && w.wave_x[ww]) carry = w.wave_x[ww];
            cur = __shfl_up(incl, 1, NACHO_WAVE);
            if (lane == 0) cur = 0;
            if (cur == 0) cur = carry;
#pragma unroll
            for (int j = 0; j < R; ++j) {
                cur = v[j] ? v[j] : cur;
                w.marks[at + j] = cur;
            }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < R; ++r) row[r] = w.marks[pad(r * kThreads + tid)] - 1u;
        __syncthreads();                           // markers are read: the ranking may clear them
    }
    int sh[kMapped ? R : 1];                   // remapped: storage position - counted position of an entry
    if (kMapped) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int c = r * kThreads + tid;
            sh[r] = 0;
            if (c < n) {
                const int32_t *st = reinterpret_cast<const int32_t *>((uintptr_t)w.sstart[tr[r]]);
                const int32_t *ps = reinterpret_cast<const int32_t *>((uintptr_t)w.spos[tr[r]]);
                sh[r] = st[row[D == 2 ? r : 0]] - ps[row[D == 2 ? r : 0]];
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int c = r * kThreads + tid;
            if (c < n) col[r] = reinterpret_cast<const int32_t *>((uintptr_t)w.scrd[tr[r]])[c + sh[r]];
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int c = r * kThreads + tid;
        if (c < n) {
            if (D == 1) keys[c] = (KeyT)(uint32_t)col[r];
            else keys[c] = (KeyT)(((uint64_t)row[r] << 32) | (uint32_t)col[r]);
        }
    }

    // ---- 2. ranks: slot of every entry in the merged order -----------------------
    bool cont = false;                     // the partition starts inside a row whose head is elsewhere
    if (D == 2 && !kCoo) cont = row_continues<FMT>(ops, coord, posn, p);
    for (int i = tid; i < kPadded; i += kThreads) w.marks[i] = 0;
    __syncthreads();
    int n_max = 0, t_max = 0;                  // the largest run searches nothing
#pragma unroll
    for (int t = 0; t < K; ++t) {
        const int nt = off[t + 1] - off[t];
        if (t == 0 || (t < k && larger_run(nt, t, n_max, t_max))) { n_max = nt; t_max = t; }
    }
    {
        // every pair (smaller run t, larger run u) and every block of t is a unit of
        // work; the units are dealt out to the wavefronts in turn
        int unit = 0;
        for (int t = 0; t < k; ++t) {
            if (t == t_max) continue;
            const int nt = uni(w.soff[t + 1]) - uni(w.soff[t]);
            for (int u = 0; u < k; ++u) {
                if (u == t || !larger_run(uni(w.soff[u + 1]) - uni(w.soff[u]), u, nt, t)) continue;
                int r0 = 0;
                // a long run is searched four blocks at a time (the chains of LDS reads
                // overlap), a short one block by block (more wavefronts share it)
                constexpr int kB = 4;
                for (; nt > 8 * NACHO_WAVE && r0 + (kB / 2) * NACHO_WAVE < nt; r0 += kB * NACHO_WAVE, ++unit)
                    if ((unit & (kWaves - 1)) == wave) rank_blocks<KeyT, kB, FMT == SPADD_DCSR>(w, t, u, r0, lane);
                for (; r0 < nt; r0 += NACHO_WAVE, ++unit)
                    if ((unit & (kWaves - 1)) == wave) rank_blocks<KeyT, 1, FMT == SPADD_DCSR>(w, t, u, r0, lane);
            }
        }
    }
    __syncthreads();
    {
        // inclusive prefix sum of the marks (bits 0..15) over all runs at once; a
        // thread owns R consecutive words, the other bits stay
        uint32_t v[R];
        int sum = 0, emitted = 0;
        const int at = tid * (R + 1);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            v[j] = w.marks[at + j];
            sum += (int)(v[j] & 0xffffu);
            // entry tid * R + j is emitted when no operand before its own stores its key
            // (kMul: when all k - 1 operands before its own do)
            const int met = (int)((v[j] >> kDupShift) & 0x7u);
            const bool out_entry = tid * R + j < n && (kMul ? met == k - 1 : met == 0);
            // (counted over the wavefront with ballots: no vector registers at this crowded point)
            emitted += __popcll(__ballot(out_entry));
            // DCSR: a row of the output starts at the emitted entry that is the first of its row in
            // its own run and has no entry of that row before it in any other run
            if (FMT == SPADD_DCSR)
                emitted += __popcll(__ballot(out_entry && ((rowfirst >> j) & 1u) && !(v[j] & kRowLater))) << 16;
        }
        const int incl = wave_inclusive_scan(sum);
        if (lane == NACHO_WAVE - 1) w.wave_x[wave] = (uint32_t)incl;
        if (lane == 0) atomicAdd(&w.emit_total, (uint32_t)emitted);    // both counts stay below 2^13
        __syncthreads();
        if (tid == 0) {
            // The partition's output counts are known here, long before its offset is needed:
            // published now, the workgroups after this one rarely find them missing.
            const unsigned e = w.emit_total;
            unsigned e_rows = e >> 16;
            if (FMT == SPADD_DCSR && n > 0 && cont) e_rows -= 1;      // the first row's head is elsewhere
            unsigned int *words = reinterpret_cast<unsigned int *>(tile_state + n_chunks);
            __hip_atomic_store(&words[p], kWordValid | (e_rows << 14) | (e & 0xffffu), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
        int run = incl - sum;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww)
            if (ww < wave) run += (int)w.wave_x[ww];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            run += (int)(v[j] & 0xffffu);
            w.marks[at + j] = (v[j] & 0xffff0000u) | (uint32_t)run;
        }
    }
    __syncthreads();
    if (tid < K) {
        const int o = w.soff[tid];
        w.srun[tid] = (uint32_t)o | ((o > 0 ? (w.marks[pad(o - 1)] & 0xffffu) : 0u) << 16);
    }
    __syncthreads();
    int slot[R];                               // merged slot | duplicate << 15
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int c = r * kThreads + tid;
        const uint32_t mk = w.marks[pad(c)];
        const uint32_t sr = w.srun[tr[r]];
        const int m = (c - (int)(sr & 0xffffu)) + (int)(mk >> kDirectShift) + ((int)(mk & 0xffffu) - (int)(sr >> 16));
        const int dup = ((mk >> kDupShift) & 0x7u) ? 0x8000 : 0;
        slot[r] = m | dup;
    }
    __syncthreads();                           // all ranking words are read: the assembly may overwrite them
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int c = r * kThreads + tid;
        if (c < n) slotw[slot[r] & 0x7fff] = (uint32_t)c | ((slot[r] & 0x8000) ? kSlotDup : 0u);
    }
    __syncthreads();

    // ---- 3. assembly: heads and row heads before every merged slot ------------------
    // wavefront v walks the slots v * kShare .. (v + 1) * kShare - 1; the counts in
    // the words are relative to the start of that share
    // Wavefront 0 asks for the counts of the workgroups before this one in its chunk already
    // now: they were published long ago as a rule, and the answer travels during the assembly.
    unsigned early[kChunk / NACHO_WAVE];
    {
        const unsigned int *words = reinterpret_cast<const unsigned int *>(tile_state + n_chunks);
        const int64_t c0 = (p / kChunk) * kChunk;
        const int m = (int)(p - c0);
#pragma unroll
        for (int i = 0; i < kChunk / NACHO_WAVE; ++i) {
            const int j = i * NACHO_WAVE + lane;
            early[i] = kWordValid;
            if (wave == 0 && i * NACHO_WAVE < m && j < m)
                early[i] = __hip_atomic_load(&words[c0 + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    int heads = 0, rheads = 0;
#pragma unroll
    for (int b = 0; b < kShare / NACHO_WAVE; ++b) {
        const int i = wave * kShare + b * NACHO_WAVE + lane;
        if (i - lane >= n) break;
        const bool valid = i < n;
        const uint32_t inf = valid ? slotw[i] : kSlotDup;
        bool head = !(inf & kSlotDup);         // emitted entries: heads; kMul: heads followed by k - 1 duplicates
        if (kMul) {
            head = head && i + k - 1 < n;
#pragma unroll
            for (int g = 1; g < K; ++g)
                if (g < k && head) head = (slotw[i + g < kTile ? i + g : kTile - 1] & kSlotDup) != 0;
        }
        const unsigned long long hm = __ballot(head);
        uint32_t word = inf | ((uint32_t)(heads + __popcll(hm & below)) << kSlotHeads) | (head ? kSlotEmit : 0u);
        heads += __popcll(hm);
        bool rhead = false;
        if (FMT == SPADD_DCSR) {
            const uint32_t rw = row_of(keys[inf & kSlotPos]);
            const uint32_t prow = (valid && i > 0) ? row_of(keys[slotw[i - 1] & kSlotPos]) : 0u;
            rhead = head && (i == 0 ? !cont : rw != prow);
            const unsigned long long rm = __ballot(rhead);
            word |= (uint32_t)(rheads + __popcll(rm & below)) << kSlotRows;
            rheads += __popcll(rm);
        }
        // (a DCSR union emits every head: the top bit says instead that the head starts a row)
        if (FMT == SPADD_DCSR) word = (word & ~kSlotEmit) | (rhead ? kSlotEmit : 0u);
        if (valid) slotw[i] = word;
    }
    if (lane == 0) w.wave_cnt[wave] = pack_counts(rheads, heads);

    // the values of this thread's entries: in flight during the prefix look-up
    T val[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int c = r * kThreads + tid;
        val[r] = T(0);
        if (c < n) val[r] = reinterpret_cast<const T *>((uintptr_t)w.sval[tr[r]])[c + (kMapped ? sh[kMapped ? r : 0] : 0)];
    }
    __syncthreads();

    // ---- 4. prefix sum over the workgroups ------------------------------------
    // Wavefront 0 publishes the partition's counts and reads the counts of
    // everything before the partition.
    if (wave == 0) {
        unsigned long long tot = 0;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) tot += w.wave_cnt[ww];
        long long b_rows = 0, b_nnz = 0;
        bool gave_up = false;
        const long long t_nnz = (long long)(tot & 0x7fffffffull), t_rows = (long long)((tot >> 31) & 0x7fffffffull);
        unsigned long long *totals = tile_state;                                        // one per chunk
        unsigned int *words = reinterpret_cast<unsigned int *>(tile_state + n_chunks);   // one per workgroup
        // (the workgroup's own word was published after the ranking)
        const int64_t chunk = p / kChunk, c0 = chunk * kChunk;
        {
            // words of the workgroups before this one in its chunk, all loads in flight together
            const int m = (int)(p - c0);
            int spins = 0;
            for (bool first = true;; first = false) {
                unsigned v[kChunk / NACHO_WAVE];
                bool missing = false;
#pragma unroll
                for (int i = 0; i < kChunk / NACHO_WAVE; ++i) {
                    const int j = i * NACHO_WAVE + lane;
                    v[i] = first ? early[i] : kWordValid;
                    if (!first && i * NACHO_WAVE < m && j < m)
                        v[i] = __hip_atomic_load(&words[c0 + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                int l_nnz = 0, l_rows = 0;
#pragma unroll
                for (int i = 0; i < kChunk / NACHO_WAVE; ++i) {
                    missing = missing || !(v[i] & kWordValid);
                    l_nnz += (int)(v[i] & 0x3fffu);
                    l_rows += (int)((v[i] >> 14) & 0x3fffu);
                }
                if (__ballot(missing)) {                   // a predecessor has not published yet
                    if (++spins > kSpinLimit) { gave_up = true; break; }
                    __builtin_amdgcn_s_sleep(16);
                    continue;
                }
                b_nnz = wave_sum<int>(l_nnz);
                b_rows = wave_sum<int>(l_rows);
                break;
            }
        }
        if (!gave_up && (p == c0 + kChunk - 1 || p == P - 1) && lane == 0)
            __hip_atomic_store(&totals[chunk], kTotalValid | pack_counts(b_rows + t_rows, b_nnz + t_nnz),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (!gave_up && chunk > 0) {
            // totals of the chunks before this one
            int spins = 0;
            long long c_nnz = 0, c_rows = 0;
            for (int64_t first = 0; first < chunk && !gave_up; ) {
                const int64_t j = first + lane;
                unsigned long long s = kTotalValid;
                if (j < chunk) s = __hip_atomic_load(&totals[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (__ballot(!(s & kTotalValid))) {
                    if (++spins > kSpinLimit) { gave_up = true; break; }
                    __builtin_amdgcn_s_sleep(16);
                    continue;
                }
                c_nnz += wave_sum<long long>((long long)(s & 0x7fffffffull));
                c_rows += wave_sum<long long>((long long)((s >> 31) & 0x7fffffffull));
                first += NACHO_WAVE;
            }
            b_nnz += c_nnz;
            b_rows += c_rows;
        }
        if (lane == 0) {
            unsigned long long at = pack_counts(b_rows, b_nnz);
#pragma unroll
            for (int ww = 0; ww < kWaves; ++ww) {
                w.share_off[ww] = at;
                at += w.wave_cnt[ww];
            }
            w.share_off[kWaves] = at;
            if (gave_up) *out.status = NACHO_ERR_HIP;
            if (broken) *out.status = NACHO_ERR_INVALID_ARG;
            if (p == P - 1) {
                // totals, tails and the capacity verdict (the only writer of these words)
                const long long total_nnz = b_nnz + t_nnz;
                const long long total_rows = FMT == SPADD_DCSR ? b_rows + t_rows
                                                               : (FMT == SPADD_CSR ? ops.lvl[0][0].extent : 1);
                out.counts[0] = total_rows;
                out.counts[1] = total_nnz;
                const bool fits = total_nnz <= out.cap_nnz && (FMT != SPADD_DCSR || total_rows <= out.cap_rows);
                if (!fits) *out.status = NACHO_ERR_CAPACITY;
                if (FMT == SPADD_VECTOR || kCoo) { out.pos1[0] = 0; out.pos1[1] = (int32_t)total_nnz; }
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
    // ---- 5. compute: write the partition's output ------------------------------
    if (FMT == SPADD_CSR) {
        // pos of every row that starts inside this partition: offset of the first
        // output entry whose row is not smaller
        const int first = coord[p * 2] + (cont ? 1 : 0);
        const int next_first = coord[(p + 1) * 2] + (row_continues<FMT>(ops, coord, posn, p + 1) ? 1 : 0);
        for (int rr = first + tid; rr < next_first; rr += kThreads) {
            int l = 0, h = n;
            while (l < h) {
                const int m = (l + h) >> 1;
                if (row_of(keys[slotw[m] & kSlotPos]) < (uint32_t)rr) l = m + 1; else h = m;
            }
            long long at = (long long)(w.share_off[kWaves] & 0x7fffffffull);   // past the partition's last entry
            if (l < n)
                at = (long long)((slotw[l] >> kSlotHeads) & 0x1ffu) +
                     (long long)(w.share_off[l / kShare] & 0x7fffffffull);
            out.pos1[rr] = (int32_t)at;
        }
    }
    // columns (and rows) come back from the keys: not held in registers through the stages above
    int colr[R];
    uint32_t rowr[D == 2 ? R : 1];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int c = r * kThreads + tid;
        const KeyT key = c < n ? keys[c] : KeyT(0);
        colr[r] = (int)(uint32_t)key;
        if (D == 2) rowr[r] = row_of(key);
    }
    if (sizeof(T) <= sizeof(KeyT)) __syncthreads();   // keys are read: the duplicates' values may overwrite them
    T *dv = w.dups();
#pragma unroll
    for (int r = 0; r < R; ++r)
        if (slot[r] & 0x8000) dv[slot[r] & 0x7fff] = val[r];
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int c = r * kThreads + tid;
        if (c >= n || (slot[r] & 0x8000)) continue;
        const int m = slot[r];
        const uint32_t word = slotw[m];
        if (FMT != SPADD_DCSR && !(word & kSlotEmit)) continue;   // (kMul: a head that not every operand matches)
        T sum = val[r];                    // then the duplicates, which follow in operand order
        if (kMul) {
#pragma unroll
            for (int g = 1; g < K; ++g)
                if (g < k) sum *= dv[m + g];
        } else {
            bool more = true;
#pragma unroll
            for (int g = 1; g < K; ++g) {
                more = more && m + g < n && (slotw[m + g < kTile ? m + g : kTile - 1] & kSlotDup);
                if (more) sum += dv[m + g];
            }
        }
        const unsigned long long so = w.share_off[m / kShare];
        const long long wpos = (long long)((word >> kSlotHeads) & 0x1ffu) + (long long)(so & 0x7fffffffull);
        const long long wr = (long long)((word >> kSlotRows) & 0x1ffu) + (long long)((so >> 31) & 0x7fffffffull);
        if (wpos < out.cap_nnz) {
            out.crd1[wpos] = colr[r];
            if (kCoo) out.crd0[wpos] = (int32_t)rowr[r];
            static_cast<T *>(out.val)[wpos] = sum;
        }
        if (FMT == SPADD_DCSR && (word & kSlotEmit)) {
            if (wr < out.cap_rows) {
                out.crd0[wr] = (int32_t)rowr[r];
                out.pos1[wr] = (int32_t)wpos;
            }
        }
    }
}

int64_t chunks_of(int64_t P) { return (P + kChunk - 1) / kChunk; }

template <int FMT, typename T, int K, bool kMul, bool kMapped>
hipError_t launch_k(const DevOperands &ops, const SpaddValues &vals, int64_t P, const int32_t *coord,
                    const int32_t *posn, unsigned long long *tile_state, const SpaddOut &out, hipStream_t s)
{
    hipLaunchKernelGGL((spadd_kernel<FMT, T, K, kMul, kMapped>), dim3((unsigned)P), dim3(kThreads), 0, s, ops, vals,
                       P, chunks_of(P), coord, posn, tile_state, out);
    return hipGetLastError();
}

// instantiated for up to 2, 3, 4 and 8 operands: the per-entry loops over the runs are unrolled
template <int FMT, typename T, bool kMul, bool kMapped = false>
hipError_t launch_one(const DevOperands &ops, const SpaddValues &vals, int64_t P, const int32_t *coord,
                      const int32_t *posn, unsigned long long *tile_state, const SpaddOut &out, hipStream_t s)
{
    if (ops.k <= 2) return launch_k<FMT, T, 2, kMul, kMapped>(ops, vals, P, coord, posn, tile_state, out, s);
    if (ops.k <= 3) return launch_k<FMT, T, 3, kMul, kMapped>(ops, vals, P, coord, posn, tile_state, out, s);
    if (ops.k <= 4) return launch_k<FMT, T, 4, kMul, kMapped>(ops, vals, P, coord, posn, tile_state, out, s);
    return launch_k<FMT, T, 8, kMul, kMapped>(ops, vals, P, coord, posn, tile_state, out, s);
}

}  // namespace

int spadd_capacity(int fmt) { (void)fmt; return kSpaddCap; }

// 64-bit words of look-up state: one per chunk, then one 32-bit word per workgroup
int64_t spadd_state_words(int64_t P) { return chunks_of(P) + (P + 1) / 2; }

hipError_t launch_spadd(int fmt, int dtype, bool multiply, const DevOperands &ops, const SpaddValues &vals,
                        int64_t P, const int32_t *coord, const int32_t *posn, unsigned long long *tile_state,
                        const SpaddOut &out, hipStream_t s)
{
#define NACHO_SPADD_CASE(F, M)                                                                       \
    if (fmt == F && multiply == M) {                                                                 \
        if (dtype == NACHO_F64) return launch_one<F, double, M>(ops, vals, P, coord, posn, tile_state, out, s); \
        return launch_one<F, float, M>(ops, vals, P, coord, posn, tile_state, out, s);               \
    }
    NACHO_SPADD_CASE(SPADD_VECTOR, false)
    NACHO_SPADD_CASE(SPADD_CSR, false)
    NACHO_SPADD_CASE(SPADD_DCSR, false)
    NACHO_SPADD_CASE(SPADD_VECTOR, true)
    NACHO_SPADD_CASE(SPADD_COO, false)
    NACHO_SPADD_CASE(SPADD_COO, true)
    if (fmt == SPADD_CSR && multiply && ops.start[0]) {       // remapped operands of a DCSR product
        if (dtype == NACHO_F64)
            return launch_one<SPADD_CSR, double, true, true>(ops, vals, P, coord, posn, tile_state, out, s);
        return launch_one<SPADD_CSR, float, true, true>(ops, vals, P, coord, posn, tile_state, out, s);
    }
    NACHO_SPADD_CASE(SPADD_CSR, true)
#undef NACHO_SPADD_CASE
    return hipErrorInvalidValue;    // (a DCSR product reaches this kernel as remapped CSR operands)
}

}  // namespace nacho
