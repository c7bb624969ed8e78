// Measurement aids, not part of the hot path: three kernels of known traffic
// that a benchmark times on the same GPU, in the same run, to put the machine's
// own ceilings beside the roofline fractions of the executing kernels -- a
// streaming read, a copy, and independent 8-byte gathers over a window of a
// given size (what a CSR row-major SpMV does to x once per stored non-zero).
#include "common.hpp"
#include "kernels.hpp"

namespace nacho {

namespace {

constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 8;
typedef unsigned int word4 __attribute__((ext_vector_type(4)));      // a 16-byte word

// every thread reads kProbeUnroll 16-byte words per round, a workgroup a contiguous stretch
__global__ void __launch_bounds__(kProbeThreads)
probe_read_kernel(const word4 *__restrict__ src, int64_t n16, unsigned long long *__restrict__ sink)
{
    unsigned long long acc = 0;
    const int64_t per_block = (int64_t)kProbeThreads * kProbeUnroll;
    for (int64_t base = (int64_t)blockIdx.x * per_block; base < n16; base += (int64_t)gridDim.x * per_block) {
        word4 v[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            const int64_t i = base + (int64_t)u * kProbeThreads + threadIdx.x;
            v[u] = i < n16 ? __builtin_nontemporal_load(src + i) : word4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9e3779b97f4a7c15ull) *sink = acc;      // (keeps the loads alive; practically never taken)
}

__global__ void __launch_bounds__(kProbeThreads)
probe_copy_kernel(word4 *__restrict__ dst, const word4 *__restrict__ src, int64_t n16)
{
    const int64_t per_block = (int64_t)kProbeThreads * kProbeUnroll;
    for (int64_t base = (int64_t)blockIdx.x * per_block; base < n16; base += (int64_t)gridDim.x * per_block) {
        word4 v[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            const int64_t i = base + (int64_t)u * kProbeThreads + threadIdx.x;
            v[u] = i < n16 ? __builtin_nontemporal_load(src + i) : word4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            const int64_t i = base + (int64_t)u * kProbeThreads + threadIdx.x;
            if (i < n16) __builtin_nontemporal_store(v[u], dst + i);
        }
    }
}

// `per_thread` independent gathers of one 8-byte word each, at pseudo-random places of the
// first `words` words of the table (a counter-based hash of the gather's number: every lane
// of a wavefront lands in another cache line)
__global__ void __launch_bounds__(kProbeThreads)
probe_gather_kernel(const unsigned long long *__restrict__ table, unsigned long long words, int per_thread,
                    unsigned long long *__restrict__ sink)
{
    unsigned long long acc = 0;
    const unsigned long long t = (unsigned long long)blockIdx.x * kProbeThreads + threadIdx.x;
    for (int r0 = 0; r0 < per_thread; r0 += kProbeUnroll) {
        unsigned long long v[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            unsigned long long h = (t * (unsigned long long)per_thread + (unsigned long long)(r0 + u)) *
                                   0x9e3779b97f4a7c15ull;
            h ^= h >> 29;
            h *= 0xbf58476d1ce4e5b9ull;
            h ^= h >> 32;
            v[u] = table[h % words];
        }
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) acc += v[u];
    }
    if (acc == 0x9e3779b97f4a7c15ull) *sink = acc;
}

unsigned probe_grid(int64_t items_per_block_round, int64_t items)
{
    int64_t blocks = (items + items_per_block_round - 1) / items_per_block_round;
    const int64_t cap = 256 * 32;                       // a few workgroups per compute unit, grid-stride beyond
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (unsigned)blocks;
}

}  // namespace

hipError_t launch_probe_read(const void *src, size_t bytes, void *sink, hipStream_t s)
{
    const int64_t n16 = (int64_t)(bytes / 16);
    hipLaunchKernelGGL(probe_read_kernel, dim3(probe_grid((int64_t)kProbeThreads * kProbeUnroll, n16)),
                       dim3(kProbeThreads), 0, s, static_cast<const word4 *>(src), n16,
                       static_cast<unsigned long long *>(sink));
    return hipGetLastError();
}

hipError_t launch_probe_copy(void *dst, const void *src, size_t bytes, hipStream_t s)
{
    const int64_t n16 = (int64_t)(bytes / 16);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(probe_grid((int64_t)kProbeThreads * kProbeUnroll, n16)),
                       dim3(kProbeThreads), 0, s, static_cast<word4 *>(dst), static_cast<const word4 *>(src), n16);
    return hipGetLastError();
}

hipError_t launch_probe_gather(const void *table, size_t window_bytes, int64_t gathers, void *sink, hipStream_t s)
{
    const unsigned long long words = window_bytes / 8;
    const int per_thread = 64;
    int64_t threads = (gathers + per_thread - 1) / per_thread;
    const unsigned grid = (unsigned)((threads + kProbeThreads - 1) / kProbeThreads);
    hipLaunchKernelGGL(probe_gather_kernel, dim3(grid), dim3(kProbeThreads), 0, s,
                       static_cast<const unsigned long long *>(table), words, per_thread,
                       static_cast<unsigned long long *>(sink));
    return hipGetLastError();
}

}  // namespace nacho
