// Shared device helpers of the nacho HIP library (gfx950, 64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "nacho.h"

#define NACHO_WAVE 64

namespace nacho {

// Device-side copy of the operands' level descriptors (passed by value as a
// kernel argument; k <= NACHO_MAX_OPERANDS, d <= NACHO_MAX_LEVELS).
struct DevLevel {
    int32_t kind;
    int32_t pad_;
    int64_t extent;
    const int32_t *pos;
    const int32_t *crd;
    int64_t count;
};
struct DevOperands {
    int32_t k, d;
    DevLevel lvl[NACHO_MAX_OPERANDS][NACHO_MAX_LEVELS];
    // Remapped operands (Section 3.3; dense level 0 over the intersected rows): the entries of
    // row i' of operand t are stored from position start[t][i'] of crd / val on, while the
    // level-1 pos array counts only the entries of the intersected rows.  NULL otherwise.
    const int32_t *start[NACHO_MAX_OPERANDS];
    // Remapped operands only: their sizes are results of earlier kernels of the same call and are
    // read on the device.  dyn_head[0] = rows all operands store (the extent of the dense level),
    // dyn_head[1 + t] = entries operand t stores in them (the count of its compressed level);
    // dyn_plan[0] = partitions of the remapped nest, dyn_plan[2] = its total cost.  The extents and
    // counts in lvl[][] are upper bounds then (what the launches are sized for).  NULL otherwise.
    const int32_t *dyn_head;
    const int64_t *dyn_plan;
};

// Extent of the dense level 0 / count of the last level of operand t: the stored ones, or (remapped
// operands) the values earlier kernels of the call left on the device.
__device__ inline int64_t level0_extent(const DevOperands &ops)
{
    return ops.dyn_head ? (int64_t)ops.dyn_head[0] : ops.lvl[0][0].extent;
}
__device__ inline int64_t last_count(const DevOperands &ops, int t)
{
    return ops.dyn_head ? (int64_t)ops.dyn_head[1 + t] : ops.lvl[t][ops.d - 1].count;
}

// floor(p * total / P) for 0 <= p <= P < 2^31 without leaving int64.
__host__ __device__ inline int64_t equal_query(int64_t p, int64_t total, int64_t P)
{
    int64_t q = total / P, r = total % P;
    return p * q + (p * r) / P;
}

__device__ inline int lane_id() { return (int)(threadIdx.x & (NACHO_WAVE - 1)); }

// Orders the LDS traffic of ONE wavefront: writes issued before it are visible
// to reads of other lanes of the same wavefront issued after it.  (The LDS
// executes a wavefront's instructions in order; this keeps the compiler from
// moving accesses across the point.)  It does not synchronise wavefronts.
__device__ inline void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Butterfly sum over the 64 lanes in a fixed order: every lane ends with the
// same bits, and the same inputs always give the same result.
template <typename T>
__device__ inline T wave_sum(T v)
{
#pragma unroll
    for (int off = NACHO_WAVE / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, NACHO_WAVE);
    return v;
}

__device__ inline int wave_max(int v)
{
#pragma unroll
    for (int off = NACHO_WAVE / 2; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off, NACHO_WAVE));
    return v;
}

// Inclusive prefix sum over the lanes of a wavefront.
__device__ inline int wave_inclusive_scan(int v)
{
    const int lane = lane_id();
#pragma unroll
    for (int off = 1; off < NACHO_WAVE; off <<= 1) {
        int n = __shfl_up(v, off, NACHO_WAVE);
        if (lane >= off) v += n;
    }
    return v;
}

// Least position in [lo, hi) whose coordinate is >= x; hi if there is none.
__device__ inline int lower_bound_global(const int32_t *__restrict__ crd, int lo, int hi, int64_t x)
{
    while (lo < hi) {
        int mid = lo + ((hi - lo) >> 1);
        if ((int64_t)crd[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// First row t in [lo, hi) with pos[t + 1] > q, found by the whole wavefront (64 probes
// per round).  Requires pos[hi] > q.  Rows lo .. t - 1 then hold nothing at or after q.
__device__ inline int first_row_past(const int32_t *__restrict__ pos, int lo, int hi, int q)
{
    const int lane = lane_id();
    while (hi - lo > 1) {
        const int span = hi - lo;
        const int step = (span + NACHO_WAVE - 1) / NACHO_WAVE;
        int t = lo + lane * step;
        if (lane == NACHO_WAVE - 1 || t > hi - 1) t = hi - 1;
        const unsigned long long past = __ballot(pos[t + 1] > q);    // a suffix of the lanes, never empty
        const int L = __ffsll((long long)past) - 1;
        const int t_hit = __shfl(t, L, NACHO_WAVE);
        const int t_prev = __shfl(t, L > 0 ? L - 1 : 0, NACHO_WAVE);
        if (L > 0) lo = t_prev + 1;
        hi = t_hit + 1;
    }
    return lo;
}

// ---- instrumented build (-DNACHO_INSTRUMENT): what every wavefront did, and when -----------
// The executing kernels take a log descriptor as their last argument.  In the ordinary build the
// flag below is false and every use of it folds away; in the instrumented build lane 0 of
// wavefront i of a launch fills record i (if the caller gave a buffer): the items and rows it
// worked on, its first and last time stamp (constant 100 MHz counter, comparable across the
// chip), its shader-clock cycles and where it ran.
#ifdef NACHO_INSTRUMENT
constexpr bool kInstrument = true;
#else
constexpr bool kInstrument = false;
#endif
struct WaveRecord {
    unsigned long long t_begin, t_end;   // wall_clock64()
    unsigned long long cycles;           // clock64() span
    uint32_t items, rows;                // work items (stored non-zeros / merged places) and rows touched
    uint32_t hw_id, xcc_id;              // HW_ID and XCC_ID registers of the wavefront
};
struct WaveLog {
    WaveRecord *rec;
    long long capacity;
};
struct WaveStamp { unsigned long long t, c; };
__device__ inline WaveStamp wave_begin()
{
    WaveStamp s = {0ull, 0ull};
    if (kInstrument) { s.t = wall_clock64(); s.c = clock64(); }
    return s;
}
__device__ inline void wave_end(const WaveLog &log, long long index, const WaveStamp &s, uint32_t items,
                                uint32_t rows)
{
    if (!kInstrument) return;
    if (log.rec == nullptr || index >= log.capacity || lane_id() != 0) return;
    WaveRecord r;
    r.t_begin = s.t;
    r.t_end = wall_clock64();
    r.cycles = clock64() - s.c;
    r.items = items;
    r.rows = rows;
    uint32_t hw = 0, xcc = 0;
#ifdef NACHO_INSTRUMENT
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
#endif
    r.hw_id = hw;
    r.xcc_id = xcc;
    log.rec[index] = r;
}

}  // namespace nacho

// Host-side bookkeeping shared by the translation units.
namespace nacho_host {

struct Profiler {
    static constexpr int kMax = 16;
    bool enabled = false;
    int n = 0;
    hipEvent_t ev[kMax + 1] = {};
    const char *name[kMax] = {};
    bool created = false;
    hipStream_t stream = nullptr;
};
Profiler &profiler();
// Call before the first kernel of an entry point, then after every kernel.
void profile_begin(hipStream_t s);
void profile_mark(const char *kernel_name);

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Where the executing kernels of an instrumented build log their wavefronts (null otherwise).
nacho::WaveLog &wave_log();

}  // namespace nacho_host
