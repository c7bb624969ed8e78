// k-way sparse union addition (and intersection product): assembly (count),
// prefix sum and compute (fill) of Section 4.3 / 4.4 (pipeline of Figure 7(a))
// in ONE kernel, one workgroup of eight wavefronts per partition.
//
// A partition owns, in every operand t, the stored entries at last-level
// positions [q_t(p), q_t(p+1)) found by the partition search; because the
// search runs in coordinate space, entries with equal coordinates in different
// operands always fall in the same partition (Section 6, merge-path paragraph),
// so a partition's output is independent of its neighbours: there is no carry.
//
// Inside the workgroup the k sorted runs are merged the way the partition
// search splits the whole problem, one level down: every thread owns the same
// number of consecutive places of the merged order, finds where its share
// starts with a diagonal search over the two runs it merges (the search of
// Section 3.2 for two one-level operands, in LDS) and then merges its places
// serially, a two-finger loop without branches.  More than two runs are merged
// pairwise in rounds (adjacent runs, so ties stay in operand order).  What a
// lane executes does not depend on how the entries are spread over the
// operands, so the eight wavefronts carry the same load whatever the operands
// look like.
// Per partition the workgroup
//   1. stages the operands' coordinate segments in LDS as k sorted runs of keys
//      (vectors: the index; matrices: row<<32 | column, the row of every entry
//      recovered from the pos array with a marker + latest-marker scan, or read
//      from the stored rows of a coordinate list; third-order tensors: the
//      16-byte key (i<<32 | j, k), fibre and slice of every entry recovered by
//      two such passes), every run followed by a sentinel, and the values
//      beside them;
//   2. merges the runs pairwise, in place, values moving with their keys;
//   3. assembly: walks the merged order, place m = j * 512 + thread; a place
//      whose key differs from the one before it is the HEAD of its coordinate
//      (and a head whose predecessor lies in another row starts a row); its
//      value is its own plus the equal keys that follow it, i.e. in operand
//      order.  Heads are counted with ballots, per block of 64 places;
//   4. prefix sum: publishes the partition's counts and reads the counts of
//      everything before the partition (two levels, see below);
//   5. compute: every head writes coordinate and value at offset + heads before
//      it -- consecutive lanes write consecutive words.  The hierarchical
//      arrays (crd0/pos1 of a DCSR result, pos of a CSR result, crd1/pos2 and
//      crd0/pos1 of a third-order result) are written for the rows (fibres,
//      slices) whose first output entry the partition owns -- exactly one
//      writer each.
// What differs from the paper's three kernels: the inputs are read once instead
// of twice and there is no separate scan launch; the arithmetic is the same.
//
// Workgroup p handles partition p and waits, when it looks up its offset, only
// for workgroups with a smaller index.  Workgroups are handed to every XCD in
// index order, so the unfinished workgroup with the smallest index is always
// running and waits for nobody: the waits end.  (Every wait is bounded all the
// same; a wavefront that gives up reports NACHO_ERR_HIP and writes nothing.)
#include "common.hpp"
#include "kernels.hpp"
#include "search.hpp"

namespace nacho {

namespace {

// Key of a third-order tensor's entry: (i, j) above k, compared lexicographically.
struct alignas(16) Key3 {
    uint64_t hi, lo;                                   // i << 32 | j,  k
    __device__ bool operator==(const Key3 &o) const { return hi == o.hi && lo == o.lo; }
    __device__ bool operator!=(const Key3 &o) const { return hi != o.hi || lo != o.lo; }
    __device__ bool operator<(const Key3 &o) const { return hi < o.hi || (hi == o.hi && lo < o.lo); }
    __device__ bool operator<=(const Key3 &o) const { return hi < o.hi || (hi == o.hi && lo <= o.lo); }
};
// c ? a : b, member by member (a conditional over the whole struct goes through memory)
template <typename KeyT> __device__ inline KeyT pick(bool c, const KeyT &a, const KeyT &b) { return c ? a : b; }
template <> __device__ inline Key3 pick<Key3>(bool c, const Key3 &a, const Key3 &b)
{
    return Key3{c ? a.hi : b.hi, c ? a.lo : b.lo};
}
template <int FMT> struct KeyOf { typedef uint64_t type; };
template <> struct KeyOf<SPADD_VECTOR> { typedef uint32_t type; };
template <> struct KeyOf<SPADD_CSF3> { typedef Key3 type; };
// The key no entry reaches (coordinates stay below 2^31).
template <typename KeyT> __device__ constexpr KeyT key_sentinel() { return ~KeyT(0); }
template <> __device__ constexpr Key3 key_sentinel<Key3>() { return Key3{~0ull, ~0ull}; }

#ifndef NACHO_MERGE_WAVES
#define NACHO_MERGE_WAVES 8
#endif
constexpr int kWaves = NACHO_MERGE_WAVES;           // wavefronts per workgroup
constexpr int kThreads = kWaves * NACHO_WAVE;
constexpr int kMaxRuns = NACHO_MAX_OPERANDS;
constexpr int kSlack = 4 * kMaxRuns;               // sentinels, gaps left by merged runs, reads past the last run
// (word 0 of the staged keys is a sentinel, run t is staged from word off[t] + t + 1 on, one
// word after every run holds its sentinel; the last word of the arrays takes the stores of the
// threads that have no entry)

// Places of the merged order a thread owns.  Odd: thread i's places start at word
// i * kIpt of the LDS arrays, and an odd stride spreads the lanes of a wavefront
// over all banks.  Chosen so that three workgroups fit the LDS of a compute unit (the
// scalar registers of the kernel allow no more than three anyway).
template <typename KeyT, typename T> struct Shape {
    static constexpr int kIpt = (sizeof(KeyT) + sizeof(T) <= 8) ? 11 : (sizeof(KeyT) > 8 ? 5 : 7);
    static constexpr int kTile = kThreads * kIpt;
    // entries a partition may hold: every round of pairwise merges hands out whole threads per pair
    // (at most kMaxRuns / 2 pairs), and all of them must fit the workgroup
    static constexpr int kCapacity = kIpt * (kThreads - kMaxRuns / 2);
    static constexpr int kBlocks = kTile / NACHO_WAVE;     // blocks of 64 places
};

// Prefix sum over the workgroups' counts, two levels and no chains: a workgroup
// publishes the counts of its partition in a 32-bit word; the last workgroup
// of every chunk of kChunk workgroups also publishes the chunk's total.  The
// offset of a workgroup is the sum of the totals of the chunks before its own
// plus the sum of the words of the workgroups before it in its chunk: all of
// them plain reads of words that their owners publish without waiting for
// anybody (a word) or after one such wait (a total).
//   word:  bit 31 published, bits 14..27 rows, bits 0..13 nnz
//   total: bit 63 published, bits 31..61 rows, bits 0..30 nnz
// Workgroups per chunk.  Vectors: a large chunk, so that few totals are read (their workgroups run
// nearly in step and a total is there early).  Matrices and tensors: a small one; their partitions
// take unequal time, the waiting wavefronts poll the words of their chunk, and hundreds of them on
// the same 2 KB of words measured a sixth slower than on 256 bytes each.
constexpr int kChunkVector = 512, kChunkOther = 64;
constexpr int chunk_size(int fmt) { return fmt == SPADD_VECTOR ? kChunkVector : kChunkOther; }
constexpr int word_loads(int chunk) { return (chunk + NACHO_WAVE - 1) / NACHO_WAVE; }   // words of a chunk a lane reads
constexpr int kSpinLimit = 1 << 14;   // polls (each a sleep + one round trip to memory: tens of milliseconds in all)
constexpr unsigned kWordValid = 0x80000000u;
constexpr unsigned long long kTotalValid = 1ull << 63;
static_assert(kThreads * 11 < (1 << 14), "a partition's counts fit the 14-bit fields of its word");

__device__ inline unsigned long long pack_counts(long long rows, long long nnz)
{
    return ((unsigned long long)rows << 31) | (unsigned long long)nnz;
}

// Level-0 coordinate and innermost coordinate of a key.
template <typename KeyT> __device__ inline uint32_t row_of(KeyT k) { return (uint32_t)((uint64_t)k >> 32); }
__device__ inline uint32_t row_of(const Key3 &k) { return (uint32_t)(k.hi >> 32); }
template <typename KeyT> __device__ inline uint32_t col_of(KeyT k) { return (uint32_t)k; }
__device__ inline uint32_t col_of(const Key3 &k) { return (uint32_t)k.lo; }

// Pointers into the operands' and the result's arrays are global-memory pointers (the loads and
// stores below then need no address-space check).
#define NACHO_GLOBAL __attribute__((address_space(1)))
template <typename U> __device__ inline const NACHO_GLOBAL U *global_ptr(unsigned long long a)
{
    return reinterpret_cast<const NACHO_GLOBAL U *>(a);
}
template <typename U> __device__ inline NACHO_GLOBAL U *global_out(U *p)
{
    return reinterpret_cast<NACHO_GLOBAL U *>(reinterpret_cast<uintptr_t>(p));
}

// LDS state of one partition.  Word 0 of `keys` is a sentinel, run t is staged from word
// off[t] + t + 1 on and is followed by its sentinel; the last word of keys / vals takes the
// stores of threads that have no entry.
template <typename KeyT, typename T, int TILE>
struct Tile {
    KeyT keys[TILE + kSlack + 1];         // the k runs, then the merged order
    union {
        T vals[TILE + kSlack + 1];        // the values, word for word beside the keys
        uint32_t marks[TILE + kSlack + 1];    // staging (matrices): row markers, before the values are stored
    };
    unsigned long long blk_emit[TILE / NACHO_WAVE];    // per block of 64 merged places: which are emitted
    uint32_t blk_cnt[TILE / NACHO_WAVE];  // emitted entries of the block | rows it starts << 16
    uint32_t blk_loc[TILE / NACHO_WAVE];  // emitted entries | rows started, before the block inside the partition
    uint32_t blk_cnt2[TILE / NACHO_WAVE]; // third-order tensors: slices (level-0 coordinates) the block starts
    uint32_t blk_loc2[TILE / NACHO_WAVE]; // ... and those started before the block inside the partition
    unsigned long long scrd[kMaxRuns];    // address of crd of run t, biased so that [c] is entry c of the partition
    unsigned long long sval[kMaxRuns];    // the same for the values
    unsigned long long sstart[kMaxRuns];  // remapped operands: address of start[t]; coordinate lists: of the rows
    unsigned long long spos[kMaxRuns];    // remapped operands: address of pos of run t
    int32_t soff[kMaxRuns + 1];           // start of run t among the partition's entries
    uint32_t wave_x[kWaves];              // per-wavefront partial of a scan across the workgroup
    long long base_nnz, base_rows, base_slices;    // output offsets of the partition (known after the prefix sum)
    uint32_t tile_cnt;                    // emitted entries | rows started of the partition
    uint32_t tile_cnt2;                   // slices started (third-order tensors)
    uint32_t early_hits;                  // early count: entries found to repeat a key (union) / found everywhere (product)
    int32_t gave_up;
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

// Byte offset of a value in `vals` from the byte offset of its key in `keys` (the two arrays hold
// entry c at index c).
template <int KB, int VB> __device__ inline int value_offset(int src)
{
    if constexpr (KB == VB) return src;
    else if constexpr (KB > VB) return (int)((unsigned)src / (unsigned)(KB / VB));
    else return src * (VB / KB);
}

// Third-order tensors: does boundary b fall strictly inside a fibre (i, j) / inside a slice i, i.e. does
// some operand hold an entry of the boundary's fibre / slice before the boundary?
__device__ inline void csf3_continues(const DevOperands &ops, const int32_t *coord, const int32_t *posn, int64_t b,
                                      bool &fibre, bool &slice)
{
    const int k = ops.k;
    const int x0 = coord[b * 3], x1 = coord[b * 3 + 1];
    fibre = slice = false;
    for (int t = 0; t < k; ++t) {
        const int i0 = posn[(b * k + t) * 3 + 0], f0 = posn[(b * k + t) * 3 + 1], q = posn[(b * k + t) * 3 + 2];
        if ((int64_t)i0 >= ops.lvl[t][0].count || ops.lvl[t][0].crd[i0] != x0) continue;
        const int32_t *pos1 = ops.lvl[t][1].pos, *pos2 = ops.lvl[t][2].pos;
        if (q > pos2[pos1[i0]]) slice = true;
        if (f0 < pos1[i0 + 1] && ops.lvl[t][1].crd[f0] == x1 && q > pos2[f0]) fibre = true;
    }
}

// One thread's share of the stable merge of the sorted runs X = keys[sx, sx + nx)
// and Y = keys[sy, sy + ny) (nx, ny > 0), each followed by a sentinel key that no
// entry reaches: places d0 .. d0 + IPT - 1 of the merged order (X first on
// ties).  `steps` >= number of bits of min(nx, ny).  Places past nx + ny come
// out as garbage.  Reads only.  All positions are kept as byte offsets into the
// LDS arrays (kb = keys, vb = vals).
template <typename KeyT, typename T, int IPT>
__device__ inline void merge_share(const char *kb, const char *vb, int sx, int nx, int sy, int ny, int d0,
                                   int steps, KeyT (&ok)[IPT], T (&ov)[IPT])
{
    constexpr int KB = (int)sizeof(KeyT);
    // The diagonal: how many of the first d0 places come from X -- the search of Section 3.2 on two
    // one-level operands: the highest c in [lo, hi] such that X[c - 1] comes before Y[d0 - c]
    // (true for every c up to the answer, false beyond it), by binary lifting.
    const int lo = d0 - ny > 0 ? d0 - ny : 0, hi = d0 < nx ? d0 : nx;
    int pos = lo * KB;
    const int hib = hi * KB;
    const int bx = (sx - 1) * KB;              // X[c - 1] lives at bx + c * KB
    const int by = (sy + d0) * KB;             // Y[d0 - c] at by - c * KB
    for (int step = KB << (steps - 1); step >= KB; step >>= 1) {
        int cand = pos + step;
        cand = cand < hib ? cand : hib;
        const KeyT xv = *reinterpret_cast<const KeyT *>(kb + bx + cand);
        const KeyT yv = *reinterpret_cast<const KeyT *>(kb + by - cand);
        pos = xv <= yv ? cand : pos;
    }
    int xi = sx * KB + pos, yi = by - pos;
    KeyT xk = *reinterpret_cast<const KeyT *>(kb + xi), yk = *reinterpret_cast<const KeyT *>(kb + yi);
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
        const bool tx = xk <= yk;              // (an exhausted run shows its sentinel)
        const int src = tx ? xi : yi;
        ok[j] = pick<KeyT>(tx, xk, yk);
        const int vsrc = value_offset<KB, (int)sizeof(T)>(src);
        ov[j] = *reinterpret_cast<const T *>(vb + vsrc);
        const KeyT nk = *reinterpret_cast<const KeyT *>(kb + src + KB);
        xi += tx ? KB : 0;
        yi += tx ? 0 : KB;
        xk = pick<KeyT>(tx, nk, xk);
        yk = pick<KeyT>(tx, yk, nk);
    }
}


// Number of keys of the sorted run keys[s, s + n) (followed by its sentinel) that are
// smaller than `key` (n >= 1): binary lifting, `bits` >= number of bits of n.
template <typename KeyT>
__device__ inline int run_lower_bound(const KeyT *keys, int s, int n, int bits, KeyT key)
{
    int pos = 0;
    for (int step = 1 << (bits - 1); step > 0; step >>= 1) {
        const int cand = pos + step;
        const int at = cand < n ? cand : n;
        pos = keys[s + at - 1] < key ? at : pos;
    }
    return pos;
}

// Prefix look-up, first level: the 14-bit fields of the words of workgroups c0 .. c0 + m - 1 (m <= kChunk)
// summed over the wavefront, once every one of them is published.  `early` holds the words as they were
// when the wavefront asked for them ahead of time (kUseEarly), else the first round loads them too.
// Returns false when the wavefront gives up waiting.
template <bool kUseEarly, int kWordLoads>
__device__ inline bool sum_words(const unsigned int *words, int64_t c0, int m, const unsigned (&early)[kWordLoads],
                                 int lane, long long &lo14, long long &hi14)
{
    // (a word that has been seen published is not read again: a waiting wavefront only polls the words
    // it still misses -- hundreds of waiting workgroups re-reading whole chunks would load the fabric
    // that the publishing stores travel on)
    unsigned v[kWordLoads];
#pragma unroll
    for (int i = 0; i < kWordLoads; ++i) {
        const int j = i * NACHO_WAVE + lane;
        const bool mine = i * NACHO_WAVE < m && j < m;
        v[i] = mine ? 0u : kWordValid;
        if (kUseEarly && mine) v[i] = early[i];
    }
    for (int spins = 0;; ++spins) {
        bool missing = false;
#pragma unroll
        for (int i = 0; i < kWordLoads; ++i) {
            if (i * NACHO_WAVE < m && !(v[i] & kWordValid))
                v[i] = __hip_atomic_load(&words[c0 + i * NACHO_WAVE + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            missing = missing || !(v[i] & kWordValid);
        }
        if (__ballot(missing) == 0ull) break;
        if (spins > kSpinLimit) return false;      // a predecessor has not published yet
        __builtin_amdgcn_s_sleep(16);
    }
    int l_lo = 0, l_hi = 0;
#pragma unroll
    for (int i = 0; i < kWordLoads; ++i) {
        l_lo += (int)(v[i] & 0x3fffu);
        l_hi += (int)((v[i] >> 14) & 0x3fffu);
    }
    lo14 = wave_sum<int>(l_lo);
    hi14 = wave_sum<int>(l_hi);
    return true;
}

// Second level: the two 31-bit fields of the totals of chunks 0 .. chunk - 1, summed, once published.
template <int kChunk>
__device__ inline bool sum_totals(const unsigned long long *totals, const unsigned int *words, int64_t chunk, int lane,
                                  long long &lo31, long long &hi31)
{
    // A total that its chunk's last workgroup has not published yet (that workgroup first has to get to
    // its own prefix sum) is not waited for: the words of that chunk are summed here -- they may all be
    // there long before, published early.
    long long c_lo = 0, c_hi = 0;
    const unsigned none[word_loads(kChunk)] = {};
    for (int64_t first = 0; first < chunk; first += NACHO_WAVE) {
        const int64_t j = first + lane;
        unsigned long long s = kTotalValid;
        if (j < chunk) s = __hip_atomic_load(&totals[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool there = (s & kTotalValid) != 0;
        c_lo += wave_sum<long long>(there ? (long long)(s & 0x7fffffffull) : 0ll);
        c_hi += wave_sum<long long>(there ? (long long)((s >> 31) & 0x7fffffffull) : 0ll);
        unsigned long long missing = __ballot(!there);
        while (missing) {                          // (uniform)
            const int64_t jm = first + (__ffsll((long long)missing) - 1);
            missing &= missing - 1;
            long long l = 0, h = 0;
            if (!sum_words<false, word_loads(kChunk)>(words, jm * kChunk, kChunk, none, lane, l, h)) return false;
            c_lo += l;
            c_hi += h;
        }
    }
    lo31 = c_lo;
    hi31 = c_hi;
    return true;
}

// kMul: the k-way intersection with products (an entry is emitted when all k
// operands store its coordinate, Section 2.1) instead of the union with sums;
// the partitions, the merge and the prefix sum are the same.
// kMapped: the operands are remapped ones (Section 3.3): CSR over the rows all
// operands store, positions counted over those rows only; the entries of row
// i' of operand t are read from start[t][i'] on.
// kSearch (sparse vectors): there is no partition kernel before this one; wavefronts 0 and 1 of the
// workgroup search its two boundaries themselves (Algorithm 1, equal-share queries) and store them in
// the partition table on the way -- the search fused into the executing kernel.
template <int FMT, typename T, int K, bool kMul, bool kMapped, bool kSearch = false>
__global__ void __launch_bounds__(kThreads)
spadd_kernel(DevOperands ops, SpaddValues vals, int64_t P, int64_t n_chunks,
             const int32_t *__restrict__ coord, const int32_t *__restrict__ posn,
             unsigned long long *__restrict__ tile_state, SpaddOut out, WaveLog wlog, SpaddSearch search)
{
    static_assert(!kSearch || (FMT == SPADD_VECTOR && !kMapped), "the fused search is built for sparse vectors");
    const WaveStamp stamp = wave_begin();
    if (kMapped && ops.dyn_plan) {
        // the number of partitions is a result of earlier kernels of the call: the launch is sized for
        // an upper bound and the workgroups past the last partition have nothing to do
        P = ops.dyn_plan[0];
        if ((int64_t)blockIdx.x >= P) return;
    }
    typedef typename KeyOf<FMT>::type KeyT;
    typedef Shape<KeyT, T> S;
    constexpr int D = FMT == SPADD_VECTOR ? 1 : (FMT == SPADD_CSF3 ? 3 : 2);
    constexpr int kChunk = chunk_size(FMT), kWordLoads = word_loads(kChunk);
    constexpr bool kCsf = FMT == SPADD_CSF3;   // third-order tensors: three compressed levels
    constexpr bool kCoo = FMT == SPADD_COO;    // coordinate lists: the row of an entry is stored with it
    constexpr int R = S::kIpt;
    constexpr int NB = S::kBlocks;
    constexpr int NR = K <= 2 ? 2 : (K <= 4 ? 4 : 8);     // runs of the merge tree (a power of two)
    constexpr KeyT kSentinel = key_sentinel<KeyT>();
    static_assert(!kCsf || R <= 5, "the slice bits of a thread's places start at bit 27");
    constexpr int kDummy = S::kTile + kSlack;  // word of keys / vals nobody reads
    __shared__ Tile<KeyT, T, S::kTile> w;

    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int wave = tid / NACHO_WAVE;
    const int k = ops.k;                       // <= K
    KeyT *keys = w.keys;
    const int64_t p = blockIdx.x;              // the partition of this workgroup, p < P

    // ---- 1. segments of this partition ----------------------------------
    int q_lo[K], off[K + 1];
    off[0] = 0;
    if constexpr (kSearch) {
        __shared__ int own_bounds[2][K];
        if (wave < 2) {                        // (whole wavefronts)
            int found[K];
            search_boundary<K, 0>(ops, 1, P, 0, nullptr, search.total, search.coord, search.posn, search.cost,
                                  p + wave, found);
            if (lane == 0) {
#pragma unroll
                for (int t = 0; t < K; ++t) own_bounds[wave][t] = found[t];
            }
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < K; ++t) {
            q_lo[t] = t < k ? own_bounds[0][t] : 0;
            off[t + 1] = off[t] + (t < k ? own_bounds[1][t] - q_lo[t] : 0);
        }
    } else {
#pragma unroll
        for (int t = 0; t < K; ++t) {
            if (t >= k) { off[t + 1] = off[t]; q_lo[t] = 0; continue; }
            q_lo[t] = posn[(p * k + t) * D + (D - 1)];
            const int q_hi = posn[((p + 1) * k + t) * D + (D - 1)];
            off[t + 1] = off[t] + (q_hi - q_lo[t]);
        }
    }
    int n = off[K];                            // <= kCapacity by the host's choice of the partition count
    // Only an operand that violates its preconditions (unsorted or repeated
    // coordinates) can overflow the staging buffer: such a partition contributes
    // nothing and the call reports INVALID_ARG, but the prefix sum goes on.
    bool broken = n > S::kCapacity || n < 0;
#pragma unroll
    for (int t = 0; t < K; ++t) broken = broken || off[t + 1] < off[t];
    if (broken) {
        n = 0;
#pragma unroll
        for (int t = 0; t <= K; ++t) off[t] = 0;
    }
    // Vectors: key = the stored index and nothing else, so keys and values are copied as they are -- by
    // the memory pipeline itself, global memory to LDS (one instruction moves 64 words of one run, no
    // register in between, no address arithmetic per entry); the wavefronts share the stretches of
    // 64 words of every run among them.
    constexpr bool kDirect = D == 1 && !kMapped;
    if constexpr (kDirect) {
        typedef __attribute__((address_space(3))) uint32_t lds_word;
        if (tid == 0) w.gave_up = 0;
        const int wv = __builtin_amdgcn_readfirstlane(wave);
        constexpr int kValWords = (int)sizeof(T) / 4;
#pragma unroll
        for (int t = 0; t < K; ++t) {
            if (t >= k) break;
            const int nt = off[t + 1] - off[t];
            const int slot = off[t] + t + 1;
            const NACHO_GLOBAL uint32_t *ksrc = global_ptr<uint32_t>((unsigned long long)(uintptr_t)(ops.lvl[t][0].crd + q_lo[t]));
            const NACHO_GLOBAL uint32_t *vsrc =
                global_ptr<uint32_t>((unsigned long long)(uintptr_t)(static_cast<const T *>(vals.v[t]) + q_lo[t]));
            lds_word *kdst = (lds_word *)(keys + slot);
            lds_word *vdst = (lds_word *)(w.vals + slot);
            // (the wavefront that starts on a run rotates with the run: short runs do not all land on wavefront 0)
            for (int c = ((wv + kWaves - (t & (kWaves - 1))) & (kWaves - 1)) * NACHO_WAVE; c < nt; c += kThreads)
                if (c + lane < nt) __builtin_amdgcn_global_load_lds(ksrc + c + lane, kdst + c, 4, 0, 0);
            const int nw = nt * kValWords;
            for (int c = ((wv + kWaves - (t & (kWaves - 1))) & (kWaves - 1)) * NACHO_WAVE; c < nw; c += kThreads)
                if (c + lane < nw) __builtin_amdgcn_global_load_lds(vsrc + c + lane, vdst + c, 4, 0, 0);
        }
        int sentinel_at = 0;
#pragma unroll
        for (int t = 0; t < K; ++t)
            if (tid == t) sentinel_at = off[t + 1] + t + 1;
        if (tid < K) keys[sentinel_at] = kSentinel;
        if (tid == K) keys[0] = kSentinel;
    } else {
        if (tid == 0) {
            w.gave_up = 0;
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
                    if (kCsf) w.sstart[t] = (unsigned long long)(uintptr_t)(t < k ? ops.lvl[t][1].crd : nullptr);
                }
            }
        }
        __syncthreads();

        // run and column of every entry this thread stages: entry c = r * kThreads + tid.  A thread
        // without an entry (c >= n) goes through the motions on the partition's last entry and stores
        // to the dummy word: no branches around the loads.
        int tr[R], col[R];
        T val[R];
        uint32_t row[D >= 2 ? R : 1];              // level-0 coordinate of every entry (matrices, tensors)
        uint32_t mid[D == 3 ? R : 1];              // level-1 coordinate (third-order tensors)
        const int last = n - 1;
    #pragma unroll
        for (int r = 0; r < R; ++r) {
            const int c = r * kThreads + tid;
            const int cc = c < last ? c : last;
            int t = 0;
    #pragma unroll
            for (int u = 1; u < K; ++u) t += cc >= off[u] ? 1 : 0;
            tr[r] = t;
            col[r] = 0;
            val[r] = T(0);
            if (D >= 2) row[r] = 0;
            if (D == 3) mid[r] = 0;
        }
        if (n > 0) {
    #pragma unroll
            for (int r = 0; r < R; ++r) {
                const int c = r * kThreads + tid;
                const int cc = c < last ? c : last;
                if (!kMapped) {
                    col[r] = global_ptr<int32_t>(w.scrd[tr[r]])[cc];
                    // the values: requested now, stored beside the keys once the markers are done with
                    val[r] = global_ptr<T>(w.sval[tr[r]])[cc];
                }
                if (kCoo) row[r] = (uint32_t)global_ptr<int32_t>(w.sstart[tr[r]])[cc];
            }
        }

        // Matrices: the first 512 rows of every run (as a rule all of them) are asked for together with
        // the entries, one round trip to memory instead of two.
        constexpr bool kRowsAhead = D == 2 && !kCoo && K <= 4;      // (with eight runs the registers for it cost a workgroup per CU)
        int ahead_a[kRowsAhead ? K : 1], ahead_b[kRowsAhead ? K : 1], ahead_row[kRowsAhead ? K : 1];
        if constexpr (kRowsAhead) {
    #pragma unroll
            for (int t = 0; t < K; ++t) {
                ahead_a[t] = ahead_b[t] = ahead_row[t] = 0;
                if (t >= k) continue;
                const int i = posn[(p * k + t) * D] + tid;
                int i_hi = posn[((p + 1) * k + t) * D] + 1;
                const int i_max = (FMT == SPADD_CSR) ? (int)ops.lvl[t][0].extent : (int)ops.lvl[t][0].count;
                if (i_hi > i_max) i_hi = i_max;
                if (i < i_hi && off[t + 1] > off[t]) {
                    ahead_a[t] = ops.lvl[t][1].pos[i];
                    ahead_b[t] = ops.lvl[t][1].pos[i + 1];
                    ahead_row[t] = (FMT == SPADD_CSR) ? i : ops.lvl[t][0].crd[i];
                }
            }
        }

        if constexpr (D >= 2 && !kCoo) {
            // Segments of an upper level overlapping [q_lo, q_hi) of every run: mark each segment's
            // first entry (word of the entry in marks) with a value, then hand every entry the latest
            // marker at or before it.  The first entry of every run carries a marker, so nothing leaks
            // from one run into the next.  Matrices: the segments are the rows, the value the row's
            // coordinate.  Third-order tensors, two passes: the fibres (value: the fibre's position,
            // whose coordinate j is then read from the level-1 coordinates), then the slices (value: i).
            auto parents = [&](const int lv, uint32_t (&res)[R]) {
                for (int i = tid; i < S::kTile; i += kThreads) w.marks[i] = 0;
                __syncthreads();
    #pragma unroll
                for (int t = 0; t < K; ++t) {
                    if (t >= k) break;
                    const int nt = off[t + 1] - off[t];
                    if (nt == 0) continue;
                    const int32_t *pos_a = ops.lvl[t][1].pos;                       // children of level 0
                    const int32_t *pos_b = D == 3 ? ops.lvl[t][2].pos : nullptr;    // children of level 1
                    const int32_t *crd0 = ops.lvl[t][0].crd;
                    const int ql = q_lo[t], qh = ql + nt;
                    const int i_lo = posn[(p * k + t) * D + lv];
                    int i_hi = posn[((p + 1) * k + t) * D + lv] + 1;
                    const int i_max = (FMT == SPADD_CSR) ? (int)ops.lvl[t][0].extent : (int)ops.lvl[t][lv].count;
                    if (i_hi > i_max) i_hi = i_max;
                    if constexpr (kRowsAhead) {
                        // (a thread without a row holds a = b = 0: no mark)
                        const int s = ahead_a[t] > ql ? ahead_a[t] : ql;
                        if (ahead_b[t] > s && s < qh) w.marks[off[t] + s - ql] = (uint32_t)(ahead_row[t] + 1);
                    }
                    for (int i0 = i_lo + tid + (kRowsAhead ? kThreads : 0); i0 < i_hi; i0 += kThreads * 4) {
                        int a[4], b[4], rw[4];
    #pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const int i = i0 + u * kThreads;
                            if (i < i_hi) {
                                if (D == 2) { a[u] = pos_a[i]; b[u] = pos_a[i + 1]; }
                                else if (lv == 1) { a[u] = pos_b[i]; b[u] = pos_b[i + 1]; }
                                else { a[u] = pos_b[pos_a[i]]; b[u] = pos_b[pos_a[i + 1]]; }
                                rw[u] = (FMT == SPADD_CSR || lv == 1) ? i : crd0[i];
                            }
                        }
    #pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const int i = i0 + u * kThreads;
                            if (i < i_hi) {
                                const int s = a[u] > ql ? a[u] : ql;
                                if (b[u] > s && s < qh) w.marks[off[t] + s - ql] = (uint32_t)(rw[u] + 1);
                            }
                        }
                    }
                }
                __syncthreads();
                {
                    // latest marker at or before every word; a thread owns R consecutive words
                    uint32_t v[R], cur = 0;
                    const int at = tid * R;
    #pragma unroll
                    for (int j = 0; j < R; ++j) {
                        v[j] = w.marks[at + j];
                        cur = v[j] ? v[j] : cur;
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
                for (int r = 0; r < R; ++r) {
                    const int c = r * kThreads + tid;
                    res[r] = w.marks[c < last ? c : (last > 0 ? last : 0)] - 1u;
                }
                __syncthreads();                       // markers are read: the next pass / the values may overwrite them
            };
            if constexpr (D == 3) {
                uint32_t fibre[R];
                parents(1, fibre);
                if (n > 0) {
    #pragma unroll
                    for (int r = 0; r < R; ++r) mid[D == 3 ? r : 0] = (uint32_t)global_ptr<int32_t>(w.sstart[tr[r]])[fibre[r]];
                }
            }
            parents(0, row);
        }
        if (kMapped && n > 0) {
            // storage position - counted position of every entry, then its column and value
            int sh[R];
    #pragma unroll
            for (int r = 0; r < R; ++r) {
                const int32_t NACHO_GLOBAL *st = global_ptr<int32_t>(w.sstart[tr[r]]);
                const int32_t NACHO_GLOBAL *ps = global_ptr<int32_t>(w.spos[tr[r]]);
                sh[r] = st[row[D == 2 ? r : 0]] - ps[row[D == 2 ? r : 0]];
            }
    #pragma unroll
            for (int r = 0; r < R; ++r) {
                const int c = r * kThreads + tid;
                const int cc = c < last ? c : last;
                col[r] = global_ptr<int32_t>(w.scrd[tr[r]])[cc + sh[r]];
                val[r] = global_ptr<T>(w.sval[tr[r]])[cc + sh[r]];
            }
        }
    #pragma unroll
        for (int r = 0; r < R; ++r) {
            const int c = r * kThreads + tid;
            const int slot = c < n ? c + tr[r] + 1 : kDummy;
            if constexpr (D == 1) keys[slot] = (KeyT)(uint32_t)col[r];
            else if constexpr (D == 2) keys[slot] = (KeyT)(((uint64_t)row[r] << 32) | (uint32_t)col[r]);
            else keys[slot] = Key3{((uint64_t)row[r] << 32) | (uint64_t)mid[r], (uint64_t)(uint32_t)col[r]};
            w.vals[slot] = val[r];
        }
        if (tid < K) keys[w.soff[tid + 1] + tid + 1] = kSentinel;
        if (tid == K) keys[0] = kSentinel;
    }
    bool cont = false;                     // the partition starts inside a row (fibre) whose head is elsewhere
    bool cont_slice = false;               // third-order tensors: ... inside a slice whose head is elsewhere
    if (D == 2 && !kCoo) cont = row_continues<FMT>(ops, coord, posn, p);
    if (kCsf) csf3_continues(ops, coord, posn, p, cont, cont_slice);
    if (tid == 0) w.early_hits = 0;
    __syncthreads();

    // ---- 1b. the partition's output count, early, when it is cheap to get -----------------
    // The workgroups behind this one wait for its count (stage 4), so it is worth knowing before the
    // merge: the union emits one entry per DISTINCT key, n minus the entries whose key an earlier
    // run stores as well (or: a later run -- whichever direction needs fewer look-ups); the product
    // emits the entries of the shortest run that every other run stores.  Each such entry costs one
    // binary search per other run; done only when that is at most two searches per thread (one
    // operand dominates the partition), otherwise the count is published after the assembly.
    bool published = false;                // (uniform)
    if (FMT != SPADD_DCSR && !kCsf) {
        int cost_fwd = 0, cost_bwd = 0, n_min = n, t_min = 0;
#pragma unroll
        for (int t = 0; t < K; ++t) {
            const int nt = off[t + 1] - off[t];
            cost_fwd += nt * t;
            cost_bwd += t < k ? nt * (k - 1 - t) : 0;
            if (t < k && nt < n_min) { n_min = nt; t_min = t; }
        }
        const bool fwd = cost_fwd <= cost_bwd;
        const int cost = kMul ? n_min * (k - 1) : (fwd ? cost_fwd : cost_bwd);
        if (cost <= 2 * kThreads) {
            published = true;
            uint32_t hits = 0;
#pragma unroll
            for (int t = 0; t < K; ++t) {
                if (t >= k) break;
                const int nt = off[t + 1] - off[t];
                if (kMul ? t != t_min : (fwd ? t == 0 : t == k - 1)) continue;      // (uniform)
                for (int i0 = 0; i0 < nt; i0 += kThreads) {
                    const int i = i0 + tid;
                    const KeyT key = keys[off[t] + t + 1 + (i < nt ? i : 0)];
                    bool any = false, all = true;
#pragma unroll
                    for (int u = 0; u < K; ++u) {
                        if (u >= k || u == t) continue;
                        if (!kMul && (fwd ? u > t : u < t)) continue;
                        const int nu = off[u + 1] - off[u];
                        bool hit = false;
                        if (nu > 0) {                                              // (uniform)
                            const int bits = 32 - __builtin_clz((unsigned)nu);
                            const int at = run_lower_bound<KeyT>(keys, off[u] + u + 1, nu, bits, key);
                            hit = keys[off[u] + u + 1 + at] == key;                // (past the run: its sentinel)
                        }
                        any = any || hit;
                        all = all && hit;
                    }
                    hits += (uint32_t)__popcll(__ballot(i < nt && (kMul ? all : any)));
                }
            }
            if (lane == 0 && hits) atomicAdd(&w.early_hits, hits);
            __syncthreads();
            if (tid == 0) {
                const uint32_t e = kMul ? w.early_hits : (uint32_t)n - w.early_hits;
                unsigned int *words = reinterpret_cast<unsigned int *>(tile_state + n_chunks);
                __hip_atomic_store(&words[p], kWordValid | e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }

    // ---- 2. merge: adjacent runs pairwise, in rounds, in place -------------------
    // (all of this is uniform over the workgroup except the thread's own share)
    int rs[NR], rn[NR];                        // start and length of the runs still to be merged
    if (K == 3) {
        // three operands: the lone run is the one that makes the first round the shorter one
        const bool front = off[3] - off[2] < off[1] - off[0];       // (-, a), (b, c)  rather than  (a, b), (c, -)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int t = front ? g - 1 : g;
            rs[g] = 1;
            rn[g] = 0;
#pragma unroll
            for (int u = 0; u < 3; ++u)
                if (u == t) { rs[g] = off[u] + u + 1; rn[g] = off[u + 1] - off[u]; }
        }
    } else {
#pragma unroll
        for (int g = 0; g < NR; ++g) {
            rs[g] = g < K ? off[g] + g + 1 : 1;
            rn[g] = g < K ? off[g + 1] - off[g] : 0;
        }
    }
    const char *kb = reinterpret_cast<const char *>(w.keys);
    const char *vb = reinterpret_cast<const char *>(w.vals);
#pragma unroll
    for (int s = 1; s < NR; s <<= 1) {
        int t_base = 0, steps = 0;
        int msx = 1, mnx = 0, msy = 1, mny = 0, md0 = -1;
#pragma unroll
        for (int g = 0; g < NR; g += 2 * s) {
            const int nx = rn[g], ny = rn[g + s];
            if (nx > 0 && ny > 0) {
                const int tg = (nx + ny + R - 1) / R;              // threads of this pair
                const int lesser = nx < ny ? nx : ny;
                const int bits = 32 - __builtin_clz((unsigned)lesser);
                steps = bits > steps ? bits : steps;
                if (tid >= t_base && tid < t_base + tg) {
                    msx = rs[g]; mnx = nx; msy = rs[g + s]; mny = ny;
                    md0 = (tid - t_base) * R;
                }
                t_base += tg;
            }
        }
        if (t_base > 0) {                      // (uniform) some pair has two non-empty sides
            KeyT ok[R];
            T ov[R];
            if (md0 >= 0) merge_share<KeyT, T, R>(kb, vb, msx, mnx, msy, mny, md0, steps, ok, ov);
            __syncthreads();                   // every share is read: the merged runs may overwrite their sources
            if (md0 >= 0) {
                const int left = mnx + mny - md0;
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    const int slot = j < left ? msx + md0 + j : kDummy;
                    keys[slot] = ok[j];
                    w.vals[slot] = ov[j];
                }
                if (md0 == 0) keys[msx + mnx + mny] = kSentinel;
            }
            __syncthreads();
        }
#pragma unroll
        for (int g = 0; g < NR; g += 2 * s) {
            if (rn[g] == 0) rs[g] = rs[g + s];
            rn[g] += rn[g + s];
        }
    }
    const int mb = rs[0];                      // the merged order: keys[mb + m], m < n; keys[mb - 1] is a sentinel
    if (tid < K) keys[mb + n + tid] = kSentinel;           // (equal-key look-ahead of the last places)
    __syncthreads();

    // ---- 3. assembly: heads (and row heads) of the merged order ---------------------
    // place m = j * kThreads + tid; block b = m / 64 = j * kWaves + wave
    // Wavefront 0 asks for the counts of the workgroups before this one in its chunk already
    // now: they were published long ago as a rule, and the answer travels during the assembly.
    unsigned early[kWordLoads];
    {
        const unsigned int *words = reinterpret_cast<const unsigned int *>(tile_state + n_chunks);
        const int64_t c0 = (p / kChunk) * kChunk;
        const int m = (int)(p - c0);
#pragma unroll
        for (int i = 0; i < kWordLoads; ++i) {
            const int j = i * NACHO_WAVE + lane;
            early[i] = kWordValid;
            if (wave == 0 && i * NACHO_WAVE < m && j < m)
                early[i] = __hip_atomic_load(&words[c0 + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    KeyT hk[R];                                // key of the place
    T hv[R];                                   // its value with the equal keys after it folded in
    unsigned long long em[R];                  // (uniform) the emitted places of the thread's block
    unsigned long long rm[(FMT == SPADD_DCSR || kCsf) ? R : 1];      // (uniform) the places that start a row / fibre
    unsigned long long sm[kCsf ? R : 1];       // (uniform) third-order tensors: the places that start a slice
    uint32_t mine = 0;                         // bit j: place j is emitted; bit 16 + j: it starts a row (fibre);
                                               // bit 27 + j: it starts a slice
    uint32_t logged_items = 0, logged_rows = 0;    // (instrumented build) places / row heads this wavefront walked
    {
        const KeyT *mk = keys + mb + tid;      // (all reads below stay inside the arrays: the slack)
        const T *mv = w.vals + mb + tid;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int m = j * kThreads + tid;
            const KeyT k0 = mk[j * kThreads];
            const KeyT kp = mk[j * kThreads - 1];
            const bool head = m < n && k0 != kp;
            T sum = mv[j * kThreads];
            bool emit = head;
            if (kMul) {
                // all k operands store the coordinate: k - 1 equal keys follow the head
                emit = head && mk[j * kThreads + k - 1] == k0;
#pragma unroll
                for (int g = 1; g < K; ++g)
                    if (g < k) sum *= mv[j * kThreads + g];
            } else {
                // (an operand stores a coordinate once: at most k - 1 equal keys follow, and what lies
                // past the last place is sentinels)
#pragma unroll
                for (int g = 1; g < K; ++g) {
                    const bool eq = mk[j * kThreads + g] == k0;
                    if (K > 4 && g >= 2 && __ballot(eq) == 0ull) break;    // (uniform) nobody has more equal keys
                    const T v = mv[j * kThreads + g];
                    sum = eq ? sum + v : sum;
                }
            }
            em[j] = __ballot(emit);
            if (kInstrument) logged_items += (uint32_t)__popcll(__ballot(m < n));
            mine |= emit ? 1u << j : 0u;
            uint32_t cnt = (uint32_t)__popcll(em[j]);
            if (FMT == SPADD_DCSR) {
                const bool rhead = emit && (m == 0 ? !cont : row_of(k0) != row_of(kp));
                rm[j] = __ballot(rhead);
                mine |= rhead ? 0x10000u << j : 0u;
                cnt |= (uint32_t)__popcll(rm[j]) << 16;
                if (kInstrument) logged_rows += (uint32_t)__popcll(rm[j]);
            }
            if constexpr (kCsf) {
                const bool fhead = emit && (m == 0 ? !cont : k0.hi != kp.hi);
                const bool shead = emit && (m == 0 ? !cont_slice : row_of(k0) != row_of(kp));
                rm[j] = __ballot(fhead);
                sm[j] = __ballot(shead);
                mine |= (fhead ? 0x10000u << j : 0u) | (shead ? 0x8000000u << j : 0u);
                cnt |= (uint32_t)__popcll(rm[j]) << 16;
                if (lane == 0) w.blk_cnt2[j * kWaves + wave] = (uint32_t)__popcll(sm[j]);
                if (kInstrument) logged_rows += (uint32_t)__popcll(rm[j]);
            }
            hk[j] = k0;
            hv[j] = sum;
            // (the folded value is formed here and now: left to the compiler, the additions sink to
            // the stores of stage 5 and the words they read stay in registers until then)
            asm volatile("" : "+v"(hv[j]));
            if (lane == 0) {
                w.blk_cnt[j * kWaves + wave] = cnt;
                if (FMT == SPADD_CSR) w.blk_emit[j * kWaves + wave] = em[j];
            }
            // (the places are taken one after the other: requesting the words of all of them
            // at once would cost the registers that keep four workgroups on a compute unit)
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    __syncthreads();

    // ---- 4. prefix sum over the workgroups ------------------------------------
    // Wavefront 0 adds up the blocks, publishes the partition's counts and reads the
    // counts of everything before the partition.
    if (wave == 0) {
        // exclusive prefix over the blocks (two per lane: NB <= 128)
        const int b0 = 2 * lane, b1 = 2 * lane + 1;
        const uint32_t c0v = b0 < NB ? w.blk_cnt[b0 < NB ? b0 : 0] : 0u;
        const uint32_t c1v = b1 < NB ? w.blk_cnt[b1 < NB ? b1 : 0] : 0u;
        const int incl = wave_inclusive_scan((int)(c0v + c1v));      // both halves stay below 2^16
        const uint32_t excl = (uint32_t)incl - (c0v + c1v);
        const uint32_t tile_cnt = (uint32_t)__shfl(incl, NACHO_WAVE - 1, NACHO_WAVE);
        if (b0 < NB) w.blk_loc[b0] = excl;
        if (b1 < NB) w.blk_loc[b1] = excl + c0v;
        const long long t_nnz = (long long)(tile_cnt & 0xffffu), t_rows = (long long)(tile_cnt >> 16);
        long long t_slices = 0;
        if (kCsf) {
            const uint32_t s0v = b0 < NB ? w.blk_cnt2[b0 < NB ? b0 : 0] : 0u;
            const uint32_t s1v = b1 < NB ? w.blk_cnt2[b1 < NB ? b1 : 0] : 0u;
            const int incl2 = wave_inclusive_scan((int)(s0v + s1v));
            if (b0 < NB) w.blk_loc2[b0] = (uint32_t)incl2 - (s0v + s1v);
            if (b1 < NB) w.blk_loc2[b1] = (uint32_t)incl2 - s1v;
            t_slices = (long long)__shfl(incl2, NACHO_WAVE - 1, NACHO_WAVE);
        }
        // state of the call: one total per chunk, one 32-bit word per workgroup; third-order tensors keep
        // a second such pair behind the first for the slices
        const int64_t state_half = n_chunks + (P + 1) / 2;
        unsigned long long *totals = tile_state;
        unsigned int *words = reinterpret_cast<unsigned int *>(tile_state + n_chunks);
        unsigned long long *totals2 = tile_state + state_half;
        unsigned int *words2 = reinterpret_cast<unsigned int *>(tile_state + state_half + n_chunks);
        if (lane == 0 && !published)
            __hip_atomic_store(&words[p], kWordValid | ((unsigned)t_rows << 14) | (unsigned)t_nnz, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        if (kCsf && lane == 0)
            __hip_atomic_store(&words2[p], kWordValid | (unsigned)t_slices, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        long long b_rows = 0, b_nnz = 0, b_slices = 0, unused = 0;
        const int64_t chunk = p / kChunk, c0 = chunk * kChunk;
        // words of the workgroups before this one in its chunk, all loads in flight together
        bool ok = sum_words<true, kWordLoads>(words, c0, (int)(p - c0), early, lane, b_nnz, b_rows);
        if (kCsf && ok) ok = sum_words<false, kWordLoads>(words2, c0, (int)(p - c0), early, lane, b_slices, unused);
        if (ok && (p == c0 + kChunk - 1 || p == P - 1) && lane == 0) {
            __hip_atomic_store(&totals[chunk], kTotalValid | pack_counts(b_rows + t_rows, b_nnz + t_nnz),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (kCsf)
                __hip_atomic_store(&totals2[chunk], kTotalValid | pack_counts(0, b_slices + t_slices),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (ok && chunk > 0) {
            // totals of the chunks before this one
            long long c_nnz = 0, c_rows = 0, c_slices = 0;
            ok = sum_totals<kChunk>(totals, words, chunk, lane, c_nnz, c_rows);
            if (kCsf && ok) ok = sum_totals<kChunk>(totals2, words2, chunk, lane, c_slices, unused);
            b_nnz += c_nnz;
            b_rows += c_rows;
            b_slices += c_slices;
        }
        const bool gave_up = !ok;
        if (lane == 0) {
            w.base_nnz = b_nnz;
            w.base_rows = b_rows;
            w.base_slices = b_slices;
            w.tile_cnt = tile_cnt;
            // a status once set to an error stays: the errors are ordered, the gravest wins
            if (gave_up) {
                w.gave_up = 1;
                atomicMin(out.status, (int32_t)NACHO_ERR_HIP);
            } else if (broken) {
                atomicMin(out.status, (int32_t)NACHO_ERR_INVALID_ARG);
            }
            if (p == P - 1 && !gave_up) {
                // totals, tails and the capacity verdict (the only writer of these words)
                const long long total_nnz = b_nnz + t_nnz;
                const long long total_rows = (FMT == SPADD_DCSR || kCsf) ? b_rows + t_rows
                                                               : (FMT == SPADD_CSR ? level0_extent(ops) : 1);
                const long long total_slices = b_slices + t_slices;
                bool fits = total_nnz <= out.cap_nnz && (FMT != SPADD_DCSR || total_rows <= out.cap_rows);
                if (kCsf) {
                    // third-order tensors: {slices, fibres, entries}; the tails of the three pos arrays
                    out.counts[0] = total_slices;
                    out.counts[1] = total_rows;
                    out.counts[2] = total_nnz;
                    fits = fits && total_slices <= out.cap_rows && total_rows <= out.cap_fibres;
                    out.pos0[0] = 0;
                    out.pos0[1] = (int32_t)total_slices;
                    if (total_slices <= out.cap_rows) out.pos1[total_slices] = (int32_t)total_rows;
                    if (total_rows <= out.cap_fibres) out.pos2[total_rows] = (int32_t)total_nnz;
                } else {
                    out.counts[0] = total_rows;
                    out.counts[1] = total_nnz;
                }
                if (!fits) atomicMin(out.status, (int32_t)NACHO_ERR_CAPACITY);
                if (FMT == SPADD_VECTOR || kCoo) { out.pos1[0] = 0; out.pos1[1] = (int32_t)total_nnz; }
                if (FMT == SPADD_CSR) out.pos1[level0_extent(ops)] = (int32_t)total_nnz;
                if (FMT == SPADD_DCSR) {
                    out.pos0[0] = 0;
                    out.pos0[1] = (int32_t)total_rows;
                    if (total_rows <= out.cap_rows) out.pos1[total_rows] = (int32_t)total_nnz;
                }
            }
        }
    }
    __syncthreads();
    if (w.gave_up) {                           // no offset: nothing of this partition may be written
        wave_end(wlog, (long long)p * kWaves + wave, stamp, logged_items, logged_rows);
        return;
    }
    // ---- 5. compute: write the partition's output ------------------------------
    // (the partition's offsets are uniform: the stores address base + a small per-lane offset)
    const long long base_nnz = ((long long)__builtin_amdgcn_readfirstlane((int)(w.base_nnz >> 32)) << 32) |
                               (unsigned)__builtin_amdgcn_readfirstlane((int)(w.base_nnz & 0xffffffffll));
    const long long room_ll = out.cap_nnz - base_nnz;
    const int room = room_ll < 0 ? 0 : (room_ll > 0x7fffffffll ? 0x7fffffff : (int)room_ll);
    if (FMT == SPADD_CSR) {
        // pos of every row that starts inside this partition: offset of the first
        // output entry whose row is not smaller
        const int first = coord[p * 2] + (cont ? 1 : 0);
        const int next_first = coord[(p + 1) * 2] + (row_continues<FMT>(ops, coord, posn, p + 1) ? 1 : 0);
        const int t_nnz = (int)(w.tile_cnt & 0xffffu);
        for (int rr = first + tid; rr < next_first; rr += kThreads) {
            int l = 0, h = n;
            while (l < h) {
                const int m = (l + h) >> 1;
                if (row_of(keys[mb + m]) < (uint32_t)rr) l = m + 1; else h = m;
            }
            // emitted entries before place l
            int at = t_nnz;
            if (l < n) {
                const int b = l / NACHO_WAVE;
                at = (int)(w.blk_loc[b] & 0xffffu) +
                     __popcll(w.blk_emit[b] & ((1ull << (l & (NACHO_WAVE - 1))) - 1ull));
            }
            out.pos1[rr] = (int32_t)(base_nnz + at);
        }
    }
    NACHO_GLOBAL int32_t *crd_out = global_out(kCsf ? out.crd2 : out.crd1) + base_nnz;
    NACHO_GLOBAL T *val_out = global_out(static_cast<T *>(out.val)) + base_nnz;
    NACHO_GLOBAL int32_t *row_out = kCoo ? global_out(out.crd0) + base_nnz : nullptr;
    long long base_rows = 0;
    int room_rows = 0;
    if (FMT == SPADD_DCSR || kCsf) {
        base_rows = ((long long)__builtin_amdgcn_readfirstlane((int)(w.base_rows >> 32)) << 32) |
                    (unsigned)__builtin_amdgcn_readfirstlane((int)(w.base_rows & 0xffffffffll));
        const long long rr_ll = (kCsf ? out.cap_fibres : out.cap_rows) - base_rows;
        room_rows = rr_ll < 0 ? 0 : (rr_ll > 0x7fffffffll ? 0x7fffffff : (int)rr_ll);
    }
    long long base_slices = 0;
    int room_slices = 0;
    if (kCsf) {
        base_slices = ((long long)__builtin_amdgcn_readfirstlane((int)(w.base_slices >> 32)) << 32) |
                      (unsigned)__builtin_amdgcn_readfirstlane((int)(w.base_slices & 0xffffffffll));
        const long long ss_ll = out.cap_rows - base_slices;
        room_slices = ss_ll < 0 ? 0 : (ss_ll > 0x7fffffffll ? 0x7fffffff : (int)ss_ll);
    }
#pragma unroll
    for (int j = 0; j < R; ++j) {
        if (em[j] == 0ull) continue;           // (uniform)
        const uint32_t loc_b = w.blk_loc[j * kWaves + wave];
        const int loc = (int)(loc_b & 0xffffu) +
                        (int)__builtin_amdgcn_mbcnt_hi((unsigned)(em[j] >> 32),
                                                       __builtin_amdgcn_mbcnt_lo((unsigned)em[j], 0u));
        if ((mine >> j & 1u) && loc < room) {
            crd_out[loc] = (int32_t)col_of(hk[j]);
            if (kCoo) row_out[loc] = (int32_t)row_of(hk[j]);
            val_out[loc] = hv[j];
        }
        if (FMT == SPADD_DCSR) {
            const int rloc = (int)(loc_b >> 16) +
                             (int)__builtin_amdgcn_mbcnt_hi((unsigned)(rm[j] >> 32),
                                                            __builtin_amdgcn_mbcnt_lo((unsigned)rm[j], 0u));
            if ((mine >> (16 + j) & 1u) && rloc < room_rows) {
                global_out(out.crd0)[base_rows + rloc] = (int32_t)row_of(hk[j]);
                global_out(out.pos1)[base_rows + rloc] = (int32_t)(base_nnz + loc);
            }
        }
        if constexpr (kCsf) {
            // a fibre head writes its j and where its entries start; a slice head its i and where its fibres start
            const int floc = (int)(loc_b >> 16) +
                             (int)__builtin_amdgcn_mbcnt_hi((unsigned)(rm[j] >> 32),
                                                            __builtin_amdgcn_mbcnt_lo((unsigned)rm[j], 0u));
            if ((mine >> (16 + j) & 1u) && floc < room_rows) {
                global_out(out.crd1)[base_rows + floc] = (int32_t)(uint32_t)hk[j].hi;
                global_out(out.pos2)[base_rows + floc] = (int32_t)(base_nnz + loc);
            }
            const int sloc = (int)w.blk_loc2[j * kWaves + wave] +
                             (int)__builtin_amdgcn_mbcnt_hi((unsigned)(sm[j] >> 32),
                                                            __builtin_amdgcn_mbcnt_lo((unsigned)sm[j], 0u));
            if ((mine >> (27 + j) & 1u) && sloc < room_slices) {
                global_out(out.crd0)[base_slices + sloc] = (int32_t)row_of(hk[j]);
                global_out(out.pos1)[base_slices + sloc] = (int32_t)(base_rows + floc);
            }
        }
    }
    wave_end(wlog, (long long)p * kWaves + wave, stamp, logged_items, logged_rows);
}

int64_t chunks_of(int64_t P, int chunk) { return (P + chunk - 1) / chunk; }

template <int FMT, typename T, int K, bool kMul, bool kMapped>
hipError_t launch_k(const DevOperands &ops, const SpaddValues &vals, int64_t P, const int32_t *coord,
                    const int32_t *posn, unsigned long long *tile_state, const SpaddOut &out, hipStream_t s)
{
    hipLaunchKernelGGL((spadd_kernel<FMT, T, K, kMul, kMapped>), dim3((unsigned)P), dim3(kThreads), 0, s, ops, vals,
                       P, chunks_of(P, chunk_size(FMT)), coord, posn, tile_state, out, nacho_host::wave_log(),
                       SpaddSearch{});
    return hipGetLastError();
}

template <typename T, int K>
hipError_t launch_search_k(const DevOperands &ops, const SpaddValues &vals, int64_t P, const SpaddSearch &search,
                           unsigned long long *tile_state, const SpaddOut &out, hipStream_t s)
{
    hipLaunchKernelGGL((spadd_kernel<SPADD_VECTOR, T, K, false, false, true>), dim3((unsigned)P), dim3(kThreads), 0, s,
                       ops, vals, P, chunks_of(P, chunk_size(SPADD_VECTOR)), search.coord, search.posn, tile_state,
                       out, nacho_host::wave_log(), search);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_search_one(const DevOperands &ops, const SpaddValues &vals, int64_t P, const SpaddSearch &search,
                             unsigned long long *tile_state, const SpaddOut &out, hipStream_t s)
{
    if (ops.k <= 2) return launch_search_k<T, 2>(ops, vals, P, search, tile_state, out, s);
    if (ops.k <= 3) return launch_search_k<T, 3>(ops, vals, P, search, tile_state, out, s);
    if (ops.k <= 4) return launch_search_k<T, 4>(ops, vals, P, search, tile_state, out, s);
    return launch_search_k<T, 8>(ops, vals, P, search, tile_state, out, s);
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

// Workgroups of the merge kernel a compute unit holds at a time: its registers allow seven
// wavefronts per SIMD.
int spadd_resident() { return 28 / kWaves; }
int spadd_wavefronts() { return kWaves; }

int spadd_capacity(int fmt, int dtype)
{
    if (fmt == SPADD_VECTOR)
        return dtype == NACHO_F64 ? Shape<uint32_t, double>::kCapacity : Shape<uint32_t, float>::kCapacity;
    if (fmt == SPADD_CSF3)
        return dtype == NACHO_F64 ? Shape<Key3, double>::kCapacity : Shape<Key3, float>::kCapacity;
    return dtype == NACHO_F64 ? Shape<uint64_t, double>::kCapacity : Shape<uint64_t, float>::kCapacity;
}

// 64-bit words of look-up state: one per chunk, then one 32-bit word per workgroup -- twice (third-order
// tensors count slices in the second set); sized for the smaller chunk, which covers both
int64_t spadd_state_words(int64_t P) { return 2 * (chunks_of(P, kChunkOther) + (P + 1) / 2); }

hipError_t launch_spadd_vector_search(int dtype, const DevOperands &ops, const SpaddValues &vals, int64_t P,
                                      const SpaddSearch &search, unsigned long long *tile_state, const SpaddOut &out,
                                      hipStream_t s)
{
    if (dtype == NACHO_F64) return launch_search_one<double>(ops, vals, P, search, tile_state, out, s);
    return launch_search_one<float>(ops, vals, P, search, tile_state, out, s);
}

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
    NACHO_SPADD_CASE(SPADD_CSF3, false)
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
