// C-ABI entry points: argument checks, workspace carving, kernel sequencing.
// Nothing here computes; every step of the hot path runs in the kernels.
#include <cstring>
#include <mutex>

#include "common.hpp"
#include "kernels.hpp"

namespace nacho_host {

Profiler &profiler()
{
    static Profiler p;
    return p;
}

nacho::WaveLog &wave_log()
{
    static nacho::WaveLog log = {nullptr, 0};
    return log;
}

void profile_begin(hipStream_t s)
{
    Profiler &p = profiler();
    if (!p.enabled) return;
    if (!p.created) {
        for (int i = 0; i <= Profiler::kMax; ++i) (void)hipEventCreate(&p.ev[i]);
        p.created = true;
    }
    p.n = 0;
    p.stream = s;
    (void)hipEventRecord(p.ev[0], s);
}

void profile_mark(const char *kernel_name)
{
    Profiler &p = profiler();
    if (!p.enabled || p.n >= Profiler::kMax) return;
    p.name[p.n] = kernel_name;
    ++p.n;
    (void)hipEventRecord(p.ev[p.n], p.stream);
}

}  // namespace nacho_host

using namespace nacho;
using namespace nacho_host;

namespace {

enum Format { FMT_BAD = 0, FMT_VECTOR, FMT_CSR, FMT_DCSR, FMT_COO, FMT_CSF3 };

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

Format tensor_format(const nacho_tensor &t)
{
    if (t.nlevels == 1 && t.lvl[0].kind == NACHO_COMPRESSED) return FMT_VECTOR;
    if (t.nlevels == 2 && t.lvl[0].kind == NACHO_DENSE && t.lvl[1].kind == NACHO_COMPRESSED) return FMT_CSR;
    if (t.nlevels == 2 && t.lvl[0].kind == NACHO_COMPRESSED && t.lvl[1].kind == NACHO_COMPRESSED) return FMT_DCSR;
    if (t.nlevels == 2 && t.lvl[0].kind == NACHO_NONUNIQUE && t.lvl[1].kind == NACHO_SINGLETON) return FMT_COO;
    if (t.nlevels == 3 && t.lvl[0].kind == NACHO_COMPRESSED && t.lvl[1].kind == NACHO_COMPRESSED &&
        t.lvl[2].kind == NACHO_COMPRESSED)
        return FMT_CSF3;
    return FMT_BAD;
}

// Checks shapes and pointers of the operands of one call; fills the device
// descriptor and the total number of stored non-zeros.
int32_t check_operands(const nacho_tensor *ops, int32_t k, bool need_arrays, DevOperands *dev,
                       int64_t *total_nnz, Format *fmt_out)
{
    if (!ops || k < 1) return NACHO_ERR_INVALID_ARG;
    if (k > NACHO_MAX_OPERANDS) return NACHO_ERR_UNSUPPORTED;
    const Format fmt = tensor_format(ops[0]);
    if (fmt == FMT_BAD) return NACHO_ERR_UNSUPPORTED;
    std::memset(dev, 0, sizeof(*dev));
    dev->k = k;
    dev->d = ops[0].nlevels;
    int64_t total = 0;
    for (int t = 0; t < k; ++t) {
        if (tensor_format(ops[t]) != fmt) return NACHO_ERR_INVALID_ARG;
        for (int m = 0; m < ops[t].nlevels; ++m) {
            const nacho_level &L = ops[t].lvl[m];
            if (L.extent < 0 || L.extent > 0x7fffffffLL) return NACHO_ERR_INVALID_ARG;
            if (L.extent != ops[0].lvl[m].extent) return NACHO_ERR_INVALID_ARG;
            DevLevel &D = dev->lvl[t][m];
            D.kind = L.kind;
            D.extent = L.extent;
            if (L.kind == NACHO_NONUNIQUE || L.kind == NACHO_SINGLETON) {
                // a coordinate list: one row and one column coordinate per stored non-zero
                if (L.count < 0 || L.count > 0x7fffffffLL || L.count != ops[t].lvl[0].count)
                    return NACHO_ERR_INVALID_ARG;
                if (need_arrays && L.count > 0 && (!L.crd || !aligned16(L.crd))) return NACHO_ERR_INVALID_ARG;
                D.crd = L.crd;
                D.count = L.count;
            } else if (L.kind == NACHO_COMPRESSED) {
                if (L.count < 0 || L.count > 0x7fffffffLL) return NACHO_ERR_INVALID_ARG;
                if (need_arrays && (!L.pos || (L.count > 0 && !L.crd))) return NACHO_ERR_INVALID_ARG;
                if (need_arrays && !aligned16(L.crd)) return NACHO_ERR_INVALID_ARG;
                D.pos = L.pos;
                D.crd = L.crd;
                D.count = L.count;
            }
        }
        total += ops[t].lvl[ops[t].nlevels - 1].count;
    }
    if (total > 0x7fffffffLL) return NACHO_ERR_INVALID_ARG;
    *total_nnz = total;
    if (fmt_out) *fmt_out = fmt;
    return NACHO_OK;
}

struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *p) : base(static_cast<char *>(p)) {}
    template <typename T> T *take(size_t n)
    {
        off = align_up(off, 256);
        T *r = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += n * sizeof(T);
        return r;
    }
};

struct PartsWs {
    int32_t *coord;
    int32_t *posn;
    int64_t *cost;
};

PartsWs carve_parts(Carver &c, int64_t P, int k, int d)
{
    PartsWs w;
    w.coord = c.take<int32_t>((size_t)(P + 1) * d);
    w.posn = c.take<int32_t>((size_t)(P + 1) * k * d);
    w.cost = c.take<int64_t>((size_t)(P + 1));
    return w;
}

size_t dtype_size(int32_t dtype) { return dtype == NACHO_F64 ? 8 : 4; }

struct CarryWs {
    PartsWs parts;
    void *carry_val;
    int32_t *carry_row;
    size_t bytes;
};

// SpMV: one carry value per partition; SpMM: one 64-wide carry row per partition.
CarryWs carve_carry(void *ws, int64_t P, int32_t dtype, int width)
{
    Carver c(ws);
    CarryWs w;
    w.parts = carve_parts(c, P, 1, 2);
    w.carry_val = c.take<char>((size_t)P * width * dtype_size(dtype));
    w.carry_row = c.take<int32_t>((size_t)P);
    w.bytes = align_up(c.off, 256);
    return w;
}

struct SpaddWs {
    PartsWs parts;
    unsigned long long *tile_state;   // prefix-sum state of the call
    size_t bytes;
};

SpaddWs carve_spadd(void *ws, int64_t P, int k, int d)
{
    Carver c(ws);
    SpaddWs w;
    w.parts = carve_parts(c, P, k, d);
    w.tile_state = c.take<unsigned long long>((size_t)spadd_state_words(P));
    w.bytes = align_up(c.off, 256);
    return w;
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Compute units of the current device (256 on an MI355X), asked once.
int compute_units()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

// Workspace of a DCSR product (recursive partitioning, Section 3.3)
constexpr int64_t kRowGrain = 2048;     // level-0 coordinates of all operands per partition of the row loop
struct RemapWs {
    int64_t P0, Pmax, Mmax, count0;
    PartsWs parts0;                  // partitions of the row loop
    int32_t *flags, *qpos, *tsum;
    RemapArrays remap;
    int64_t *info;                   // {partitions, intersected rows, remapped total cost} of the last call
    PartsWs parts;                   // partitions of the remapped nest
    unsigned long long *tile_state;
    int32_t *pos_full;
    int64_t *counts;
    size_t bytes;
};

int spadd_fmt(Format f)
{
    if (f == FMT_CSF3) return SPADD_CSF3;
    return f == FMT_VECTOR ? SPADD_VECTOR : (f == FMT_CSR ? SPADD_CSR : (f == FMT_COO ? SPADD_COO : SPADD_DCSR));
}

// Partitions a fused call uses: at least P, and enough that one partition's work
// (ideal share + k - 1 by the tightness bound of Section 3.2.2) fits a wavefront.
int64_t fused_partitions(int32_t op, Format fmt, int32_t dtype, int32_t k, int64_t total_nnz, int64_t P)
{
    int64_t cap;
    if (op == NACHO_OP_SPMV) cap = spmv_capacity(dtype);
    else if (op == NACHO_OP_SPMM) cap = spmm_capacity(dtype);
    else cap = spadd_capacity(spadd_fmt(fmt), dtype) - k;
    int64_t need = total_nnz > 0 ? ceil_div(total_nnz, cap) : 1;
    if (P == 0 && op != NACHO_OP_SPMV && op != NACHO_OP_SPMM) {
        // The merge kernel keeps spadd_resident() workgroups per compute unit, and its partitions all
        // take about the same time: they run in rounds of that many workgroups per unit.  With the
        // partition count a whole number of rounds the last round is as full as the others.
        const int64_t round = (int64_t)compute_units() * spadd_resident();
        if (need > round) need = ceil_div(need, round) * round;
    }
    return P > need ? P : need;
}

RemapWs carve_remap(void *ws, const nacho_tensor *ops, int k, int32_t dtype, int64_t total_nnz, int64_t P)
{
    Carver c(ws);
    RemapWs w;
    int64_t rows_total = 0;
    w.count0 = ops[0].lvl[0].count;
    w.Mmax = w.count0;
    for (int t = 0; t < k; ++t) {
        rows_total += ops[t].lvl[0].count;
        if (ops[t].lvl[0].count < w.Mmax) w.Mmax = ops[t].lvl[0].count;
    }
    w.P0 = rows_total > 0 ? ceil_div(rows_total, kRowGrain) : 1;
    // the remapped cost never exceeds the stored non-zeros: enough partitions for any outcome
    w.Pmax = fused_partitions(NACHO_OP_SPADD, FMT_CSR, dtype, k, total_nnz, P);
    w.parts0 = carve_parts(c, w.P0, k, 1);
    w.flags = c.take<int32_t>((size_t)w.count0);
    w.qpos = c.take<int32_t>((size_t)w.count0 * (k - 1));
    int64_t sw = remap_scan_words(w.count0, 1);
    if (remap_scan_words(w.Mmax + 1, k) > sw) sw = remap_scan_words(w.Mmax + 1, k);
    w.tsum = c.take<int32_t>((size_t)sw);
    w.remap.stride = w.Mmax;
    w.remap.rows = c.take<int32_t>((size_t)w.Mmax);
    w.remap.start = c.take<int32_t>((size_t)w.Mmax * k);
    w.remap.cost = c.take<int32_t>((size_t)(w.Mmax + 1) * k);
    w.remap.head = c.take<int32_t>(1 + NACHO_MAX_OPERANDS);
    w.info = c.take<int64_t>(4);
    w.parts = carve_parts(c, w.Pmax, k, 2);
    w.tile_state = c.take<unsigned long long>((size_t)spadd_state_words(w.Pmax));
    w.pos_full = c.take<int32_t>((size_t)w.Mmax + 1);
    w.counts = c.take<int64_t>(2);
    w.bytes = align_up(c.off, 256);
    return w;
}


// The three launches of y = A x on a carved workspace (caller's or the built-in one).
int32_t spmv_enqueue(const nacho_tensor *A, const DevOperands &dev, int64_t nnz, const void *x, void *y,
                     int32_t dtype, int64_t P, int64_t Pe, const CarryWs &w, hipStream_t s, int64_t row_cost = 0)
{
    const int64_t n_rows = A->lvl[0].extent;
    profile_begin(s);
    // (fixed-grain queries make the partitions inside a row arithmetic in pos, which the executing
    // kernel uses to deal them out; with a row cost the boundaries are no longer multiples of the grain
    // in pos, and the equally spaced queries are used)
    const int64_t grain = (P == 0 && row_cost == 0) ? spmv_capacity(dtype) : 0;
    // (the partition kernel also writes the zeros of the rows A stores nothing in)
    ZeroRows zero;
    zero.base = y;
    zero.ld = 1;
    zero.width = 1;
    zero.elem = (int32_t)dtype_size(dtype);
    if (launch_partition(dev, 1, Pe, grain, nullptr, nnz, w.parts.coord, w.parts.posn, w.parts.cost, s, nullptr, 0,
                         nullptr, &zero, row_cost) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("partition");
    if (launch_spmv_exec(dtype, A->lvl[1].pos, A->lvl[1].crd, A->val, x, y, n_rows, nnz,
                         w.parts.coord, w.parts.posn, Pe, w.carry_val, w.carry_row, grain, s) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("spmv_exec");
    if (launch_spmv_fixup(dtype, y, Pe, w.carry_val, w.carry_row, A->lvl[1].pos, grain, s) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("spmv_fixup");
    return NACHO_OK;
}

// Scratch memory of nacho_spmv_static: one array per GPU inside the loaded code object, alive
// until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address on the current device is looked up once per device and
// that pointer is what the kernels get.
constexpr size_t kStaticScratchBytes = 8u << 20;
constexpr int kMaxDevices = 64;
}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxDevices] = {};

int32_t static_scratch(void **base)
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return NACHO_ERR_HIP;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return NACHO_ERR_HIP;
        g_scratch_ptr[device] = p;
    }
    *base = g_scratch_ptr[device];
    return NACHO_OK;
}
}  // namespace

extern "C" {

int32_t nacho_version(void) { return 100; }

const char *nacho_status_string(int32_t status)
{
    switch (status) {
    case NACHO_OK: return "ok";
    case NACHO_ERR_INVALID_ARG: return "invalid argument";
    case NACHO_ERR_UNSUPPORTED: return "unsupported format or operand count";
    case NACHO_ERR_WORKSPACE: return "workspace too small";
    case NACHO_ERR_CAPACITY: return "output capacity too small";
    case NACHO_ERR_HIP: return "HIP call failed";
    case NACHO_ERR_TOO_LARGE: return "operands need more than the built-in scratch memory of the no-allocation entry point";
    default: return "unknown status";
    }
}

int64_t nacho_num_partitions(int32_t op, const nacho_tensor *ops, int32_t k, int32_t dtype,
                             int64_t n_dense, int64_t P)
{
    (void)n_dense;
    if (P < 0 || (dtype != NACHO_F32 && dtype != NACHO_F64)) return 0;
    DevOperands dev;
    int64_t total = 0;
    Format fmt;
    if (check_operands(ops, k, false, &dev, &total, &fmt) != NACHO_OK) return 0;
    switch (op) {
    case NACHO_OP_PARTITION: return P;
    case NACHO_OP_SPMV:
    case NACHO_OP_SPMM:
        if (k != 1 || fmt != FMT_CSR) return 0;
        return fused_partitions(op, fmt, dtype, k, total, P);
    case NACHO_OP_SPADD:
    case NACHO_OP_SPMUL:      // (a DCSR product: an upper bound, the count depends on the intersected rows)
        if (fmt == FMT_CSF3 && op == NACHO_OP_SPMUL) return 0;
        return fused_partitions(NACHO_OP_SPADD, fmt, dtype, k, total, P);
    default: return 0;
    }
}

int32_t nacho_workspace_bytes(int32_t op, const nacho_tensor *ops, int32_t k, int32_t dtype,
                              int64_t n_dense, int64_t P, size_t *bytes)
{
    if (!bytes || P < 0) return NACHO_ERR_INVALID_ARG;
    if (dtype != NACHO_F32 && dtype != NACHO_F64) return NACHO_ERR_INVALID_ARG;
    DevOperands dev;
    int64_t total = 0;
    Format fmt;
    int32_t rc = check_operands(ops, k, false, &dev, &total, &fmt);
    if (rc != NACHO_OK) return rc;
    switch (op) {
    case NACHO_OP_PARTITION: *bytes = 0; return NACHO_OK;
    case NACHO_OP_SPMV:
    case NACHO_OP_SPMM: {
        if (k != 1 || fmt != FMT_CSR) return NACHO_ERR_UNSUPPORTED;
        const int64_t Pe = fused_partitions(op, fmt, dtype, k, total, P);
        *bytes = carve_carry(nullptr, Pe, dtype, op == NACHO_OP_SPMM ? NACHO_WAVE : 1).bytes;
        return NACHO_OK;
    }
    case NACHO_OP_SPMUL:
        if (fmt == FMT_CSF3) return NACHO_ERR_UNSUPPORTED;
        if (fmt == FMT_DCSR && k > 1) {
            *bytes = carve_remap(nullptr, ops, k, dtype, total, P).bytes;
            return NACHO_OK;
        }
        /* fall through: the pipeline of the union */
    case NACHO_OP_SPADD: {
        const int64_t Pe = fused_partitions(NACHO_OP_SPADD, fmt, dtype, k, total, P);
        *bytes = carve_spadd(nullptr, Pe, k, dev.d).bytes;
        return NACHO_OK;
    }
    default: return NACHO_ERR_UNSUPPORTED;
    }
}

int32_t nacho_workspace_parts(int32_t op, const nacho_tensor *ops, int32_t k, int32_t dtype,
                              int64_t n_dense, int64_t P, void *ws, size_t ws_bytes,
                              nacho_parts *parts, int64_t *grain, void *hip_stream)
{
    if (!parts || !ws || P < 0) return NACHO_ERR_INVALID_ARG;
    if (dtype != NACHO_F32 && dtype != NACHO_F64) return NACHO_ERR_INVALID_ARG;
    DevOperands dev;
    int64_t total = 0;
    Format fmt;
    int32_t rc = check_operands(ops, k, false, &dev, &total, &fmt);
    if (rc != NACHO_OK) return rc;
    PartsWs w;
    int64_t Pe = 0, g = 0;
    size_t need = 0;
    switch (op) {
    case NACHO_OP_SPMV:
    case NACHO_OP_SPMM: {
        if (k != 1 || fmt != FMT_CSR) return NACHO_ERR_UNSUPPORTED;
        if (op == NACHO_OP_SPMM && n_dense < 1) return NACHO_ERR_INVALID_ARG;
        Pe = fused_partitions(op, fmt, dtype, k, total, P);
        CarryWs c = carve_carry(ws, Pe, dtype, op == NACHO_OP_SPMM ? NACHO_WAVE : 1);
        w = c.parts;
        need = c.bytes;
        if (P == 0) g = op == NACHO_OP_SPMV ? (int64_t)spmv_capacity(dtype) : (int64_t)spmm_capacity(dtype) * n_dense;
        break;
    }
    case NACHO_OP_SPMUL:
        if (fmt == FMT_DCSR && k > 1) {
            RemapWs c = carve_remap(ws, ops, k, dtype, total, P);
            if (ws_bytes < c.bytes) return NACHO_ERR_WORKSPACE;
            // (the partition count of this call is a result of its kernels: read back behind them)
            int64_t info[4];
            hipStream_t s = static_cast<hipStream_t>(hip_stream);
            if (hipMemcpyAsync(info, c.info, sizeof(info), hipMemcpyDeviceToHost, s) != hipSuccess ||
                hipStreamSynchronize(s) != hipSuccess)
                return NACHO_ERR_HIP;
            if (info[0] < 0 || info[0] > c.Pmax) return NACHO_ERR_INVALID_ARG;   // no call has run on ws
            w = c.parts;
            Pe = info[0];
            need = c.bytes;
            break;
        }
        /* fall through */
    case NACHO_OP_SPADD: {
        Pe = fused_partitions(NACHO_OP_SPADD, fmt, dtype, k, total, P);
        SpaddWs c = carve_spadd(ws, Pe, k, dev.d);
        w = c.parts;
        need = c.bytes;
        break;
    }
    default: return NACHO_ERR_UNSUPPORTED;
    }
    if (ws_bytes < need) return NACHO_ERR_WORKSPACE;
    parts->k = k;
    parts->d = dev.d;
    parts->P = Pe;
    parts->coord = w.coord;
    parts->posn = w.posn;
    parts->cost = w.cost;
    if (grain) *grain = g;
    return NACHO_OK;
}

int32_t nacho_partition(const nacho_tensor *ops, int32_t k, int64_t cost_scale, int64_t P,
                        const int64_t *queries, const nacho_parts *out,
                        void *ws, size_t ws_bytes, void *hip_stream)
{
    (void)ws;
    (void)ws_bytes;
    if (!out || !out->coord || !out->posn || !out->cost) return NACHO_ERR_INVALID_ARG;
    if (P < 1 || P > 0x7ffffff0LL || cost_scale < 1) return NACHO_ERR_INVALID_ARG;
    DevOperands dev;
    int64_t total = 0;
    int32_t rc = check_operands(ops, k, true, &dev, &total, nullptr);
    if (rc != NACHO_OK) return rc;
    if (out->k != k || out->d != dev.d || out->P != P) return NACHO_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    profile_begin(s);
    if (launch_partition(dev, cost_scale, P, 0, queries, total, out->coord, out->posn, out->cost, s) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("partition");
    return NACHO_OK;
}

int32_t nacho_partition_csr64(const int64_t *pos, const int32_t *crd, int64_t n_rows, int64_t n_cols, int64_t nnz,
                              int64_t P, int32_t *coord, int64_t *posn, int64_t *cost, void *hip_stream)
{
    if (!pos || !coord || !posn || !cost) return NACHO_ERR_INVALID_ARG;
    if (n_rows < 0 || n_rows > 0x7ffffff0LL || n_cols < 0 || n_cols > 0x7ffffff0LL || nnz < 0) return NACHO_ERR_INVALID_ARG;
    if (P < 1 || P > 0x7ffffff0LL) return NACHO_ERR_INVALID_ARG;
    if (nnz > 0 && (!crd || !aligned16(crd))) return NACHO_ERR_INVALID_ARG;
    if (nnz > ((int64_t)1 << 62) / P) return NACHO_ERR_INVALID_ARG;         // (p * nnz is formed in 128 bits, kept sane)
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    profile_begin(s);
    if (launch_partition_csr64(pos, crd, n_rows, nnz, P, coord, posn, cost, s) != hipSuccess) return NACHO_ERR_HIP;
    profile_mark("partition");
    return NACHO_OK;
}

int32_t nacho_spmv(const nacho_tensor *A, const void *x, void *y, int32_t dtype, int64_t P,
                   void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!A || !x || !y || P < 0) return NACHO_ERR_INVALID_ARG;
    if (dtype != NACHO_F32 && dtype != NACHO_F64) return NACHO_ERR_INVALID_ARG;
    DevOperands dev;
    int64_t nnz = 0;
    Format fmt;
    int32_t rc = check_operands(A, 1, true, &dev, &nnz, &fmt);
    if (rc != NACHO_OK) return rc;
    if (fmt != FMT_CSR) return NACHO_ERR_UNSUPPORTED;
    if (nnz > 0 && (!A->val || !aligned16(A->val))) return NACHO_ERR_INVALID_ARG;
    const int64_t Pe = fused_partitions(NACHO_OP_SPMV, fmt, dtype, 1, nnz, P);
    CarryWs w = carve_carry(ws, Pe, dtype, 1);
    if (!ws || ws_bytes < w.bytes) return NACHO_ERR_WORKSPACE;
    return spmv_enqueue(A, dev, nnz, x, y, dtype, P, Pe, w, static_cast<hipStream_t>(hip_stream));
}

int32_t nacho_spmv_fused(const nacho_tensor *A, const void *x, void *y, int32_t dtype, void *ws, size_t ws_bytes,
                         void *hip_stream)
{
    if (!A || !x || !y) return NACHO_ERR_INVALID_ARG;
    if (dtype != NACHO_F32 && dtype != NACHO_F64) return NACHO_ERR_INVALID_ARG;
    DevOperands dev;
    int64_t nnz = 0;
    Format fmt;
    int32_t rc = check_operands(A, 1, true, &dev, &nnz, &fmt);
    if (rc != NACHO_OK) return rc;
    if (fmt != FMT_CSR) return NACHO_ERR_UNSUPPORTED;
    if (nnz > 0 && (!A->val || !aligned16(A->val))) return NACHO_ERR_INVALID_ARG;
    const int64_t Pe = fused_partitions(NACHO_OP_SPMV, fmt, dtype, 1, nnz, 0);
    CarryWs w = carve_carry(ws, Pe, dtype, 1);
    if (!ws || ws_bytes < w.bytes) return NACHO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int64_t n_rows = A->lvl[0].extent;
    const int64_t grain = spmv_capacity(dtype);
    profile_begin(s);
    if (launch_zero_vector(dtype, y, n_rows, s) != hipSuccess) return NACHO_ERR_HIP;
    profile_mark("zero_y");
    if (launch_spmv_exec(dtype, A->lvl[1].pos, A->lvl[1].crd, A->val, x, y, n_rows, nnz, nullptr, nullptr, Pe,
                         w.carry_val, w.carry_row, grain, s) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("spmv_exec_fused");
    if (launch_spmv_fixup(dtype, y, Pe, w.carry_val, w.carry_row, A->lvl[1].pos, grain, s) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("spmv_fixup");
    return NACHO_OK;
}

int32_t nacho_spmv_static(const nacho_tensor *A, const void *x, void *y, int32_t dtype, int64_t P,
                          void *hip_stream)
{
    if (!A || !x || !y || P < 0) return NACHO_ERR_INVALID_ARG;
    if (dtype != NACHO_F32 && dtype != NACHO_F64) return NACHO_ERR_INVALID_ARG;
    DevOperands dev;
    int64_t nnz = 0;
    Format fmt;
    int32_t rc = check_operands(A, 1, true, &dev, &nnz, &fmt);
    if (rc != NACHO_OK) return rc;
    if (fmt != FMT_CSR) return NACHO_ERR_UNSUPPORTED;
    if (nnz > 0 && (!A->val || !aligned16(A->val))) return NACHO_ERR_INVALID_ARG;
    const int64_t Pe = fused_partitions(NACHO_OP_SPMV, fmt, dtype, 1, nnz, P);
    // sizes first: nothing is touched when the call does not fit the built-in scratch memory
    if (carve_carry(nullptr, Pe, dtype, 1).bytes > kStaticScratchBytes) return NACHO_ERR_TOO_LARGE;
    void *base = nullptr;
    rc = static_scratch(&base);
    if (rc != NACHO_OK) return rc;
    CarryWs w = carve_carry(base, Pe, dtype, 1);
    // (every word of the table and of the carries that a kernel reads is written earlier in the
    // same call, so nothing of the previous call's contents needs clearing)
    return spmv_enqueue(A, dev, nnz, x, y, dtype, P, Pe, w, static_cast<hipStream_t>(hip_stream));
}

size_t nacho_static_scratch_bytes(void) { return kStaticScratchBytes; }

// Partitions of the row-aware calls: at least P, and enough that a partition's cost (non-zeros +
// row_cost per row) fits what one wavefront stages.
static int64_t rowcost_partitions(int32_t dtype, int64_t nnz, int64_t n_rows, int64_t row_cost, int64_t P)
{
    const int64_t total = nnz + row_cost * n_rows;
    const int64_t need = total > 0 ? ceil_div(total, spmv_capacity(dtype)) : 1;
    return P > need ? P : need;
}

int64_t nacho_rowcost_partitions(const nacho_tensor *A, int32_t dtype, int64_t row_cost, int64_t P)
{
    if (!A || P < 0 || row_cost < 0 || row_cost > 64 || (dtype != NACHO_F32 && dtype != NACHO_F64)) return 0;
    DevOperands dev;
    int64_t nnz = 0;
    Format fmt;
    if (check_operands(A, 1, false, &dev, &nnz, &fmt) != NACHO_OK || fmt != FMT_CSR) return 0;
    return rowcost_partitions(dtype, nnz, A->lvl[0].extent, row_cost, P);
}

int32_t nacho_partition_rowcost(const nacho_tensor *A, int64_t row_cost, int64_t P, const nacho_parts *out,
                                void *hip_stream)
{
    if (!out || !out->coord || !out->posn || !out->cost) return NACHO_ERR_INVALID_ARG;
    if (P < 1 || P > 0x7ffffff0LL || row_cost < 0 || row_cost > 64) return NACHO_ERR_INVALID_ARG;
    DevOperands dev;
    int64_t total = 0;
    Format fmt;
    int32_t rc = check_operands(A, 1, true, &dev, &total, &fmt);
    if (rc != NACHO_OK) return rc;
    if (fmt != FMT_CSR) return NACHO_ERR_UNSUPPORTED;
    if (out->k != 1 || out->d != 2 || out->P != P) return NACHO_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    profile_begin(s);
    if (launch_partition(dev, 1, P, 0, nullptr, total, out->coord, out->posn, out->cost, s, nullptr, 0, nullptr,
                         nullptr, row_cost) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("partition");
    return NACHO_OK;
}

int32_t nacho_spmv_rowcost(const nacho_tensor *A, const void *x, void *y, int32_t dtype, int64_t row_cost,
                           int64_t P, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!A || !x || !y || P < 0 || row_cost < 0 || row_cost > 64) return NACHO_ERR_INVALID_ARG;
    if (dtype != NACHO_F32 && dtype != NACHO_F64) return NACHO_ERR_INVALID_ARG;
    DevOperands dev;
    int64_t nnz = 0;
    Format fmt;
    int32_t rc = check_operands(A, 1, true, &dev, &nnz, &fmt);
    if (rc != NACHO_OK) return rc;
    if (fmt != FMT_CSR) return NACHO_ERR_UNSUPPORTED;
    if (nnz > 0 && (!A->val || !aligned16(A->val))) return NACHO_ERR_INVALID_ARG;
    const int64_t Pe = rowcost_partitions(dtype, nnz, A->lvl[0].extent, row_cost, P);
    CarryWs w = carve_carry(ws, Pe, dtype, 1);
    if (!ws || ws_bytes < w.bytes) return NACHO_ERR_WORKSPACE;
    // (P as passed on: with a row cost the call always uses the equally spaced queries)
    return spmv_enqueue(A, dev, nnz, x, y, dtype, Pe, Pe, w, static_cast<hipStream_t>(hip_stream), row_cost);
}

int32_t nacho_spmm(const nacho_tensor *A, const void *B, int64_t n, int64_t ldb, void *C, int64_t ldc,
                   int32_t dtype, int64_t P, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!A || !B || !C || P < 0) return NACHO_ERR_INVALID_ARG;
    if (dtype != NACHO_F32 && dtype != NACHO_F64) return NACHO_ERR_INVALID_ARG;
    if (n < 1 || ldb < n || ldc < n) return NACHO_ERR_INVALID_ARG;
    if (n > (int64_t)1 << 20) return NACHO_ERR_UNSUPPORTED;     // (costs are n per non-zero: n * nnz stays far below 2^63)
    DevOperands dev;
    int64_t nnz = 0;
    Format fmt;
    int32_t rc = check_operands(A, 1, true, &dev, &nnz, &fmt);
    if (rc != NACHO_OK) return rc;
    if (fmt != FMT_CSR) return NACHO_ERR_UNSUPPORTED;
    if (nnz > 0 && !A->val) return NACHO_ERR_INVALID_ARG;
    const int64_t Pe = fused_partitions(NACHO_OP_SPMM, fmt, dtype, 1, nnz, P);
    CarryWs w = carve_carry(ws, Pe, dtype, NACHO_WAVE);
    if (!ws || ws_bytes < w.bytes) return NACHO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    profile_begin(s);
    // cost of a stored non-zero = n (broadcast over the dense loop); queries are multiples of n
    const int64_t grain = (P == 0) ? (int64_t)spmm_capacity(dtype) * n : 0;
    ZeroRows zero;                      // rows of C whose row of A is empty
    zero.base = C;
    zero.ld = ldc;
    zero.width = (int32_t)n;
    zero.elem = (int32_t)dtype_size(dtype);
    if (launch_partition(dev, n, Pe, grain, nullptr, nnz, w.parts.coord, w.parts.posn, w.parts.cost, s, nullptr, 0,
                         nullptr, &zero) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("partition");
    // The executing kernel gives every lane of a wavefront one column of B: wider operands go through it
    // in stretches of 64 columns.  The partitions are the same for every stretch (the queries are multiples
    // of n, so no boundary falls inside the dense loop), and so are the carry buffers, which the stretches
    // use one after the other on the stream.
    const size_t elem = dtype_size(dtype);
    for (int64_t j0 = 0; j0 < n; j0 += NACHO_WAVE) {
        const int width = (int)(n - j0 < NACHO_WAVE ? n - j0 : NACHO_WAVE);
        const void *Bj = static_cast<const char *>(B) + (size_t)j0 * elem;
        void *Cj = static_cast<char *>(C) + (size_t)j0 * elem;
        if (launch_spmm_exec(dtype, A->lvl[1].pos, A->lvl[1].crd, A->val, Bj, width, ldb, Cj, ldc,
                             w.parts.coord, w.parts.posn, Pe, w.carry_val, w.carry_row, s) != hipSuccess)
            return NACHO_ERR_HIP;
        profile_mark("spmm_exec");
        if (launch_spmm_fixup(dtype, Cj, ldc, width, Pe, w.carry_val, w.carry_row, A->lvl[1].pos, grain / n, s) !=
            hipSuccess)
            return NACHO_ERR_HIP;
        profile_mark("spmm_fixup");
    }
    return NACHO_OK;
}

// Product of k >= 2 DCSR matrices: the rows are intersected first and the cost
// function of the row loop is remapped (Section 3.3, Algorithm 2); the remapped
// nest then runs through the partition and merge kernels of the CSR product.
static int32_t dcsr_product(const nacho_tensor *ops, int32_t k, int32_t dtype, int64_t P, const DevOperands &dev,
                            int64_t total, const SpaddValues &vals, const SpaddOut &o, void *ws,
                            size_t ws_bytes, hipStream_t s)
{
    RemapWs w = carve_remap(ws, ops, k, dtype, total, P);
    if (!ws || ws_bytes < w.bytes) return NACHO_ERR_WORKSPACE;
    profile_begin(s);
    bool empty = false;
    for (int t = 0; t < k; ++t)
        if (ops[t].lvl[0].count == 0 || ops[t].lvl[1].count == 0) empty = true;
    if (empty) {
        // (an operand without rows or entries: known from the descriptors)
        if (launch_empty_result(o, w.info, s) != hipSuccess) return NACHO_ERR_HIP;
        profile_mark("empty_result");
        return NACHO_OK;
    }
    // 1. the row loop on its own partitions (Algorithm 1 on the level-0 coordinate arrays)
    DevOperands rows;
    std::memset(&rows, 0, sizeof(rows));
    rows.k = k;
    rows.d = 1;
    int64_t rows_total = 0;
    for (int t = 0; t < k; ++t) {
        rows.lvl[t][0] = dev.lvl[t][0];
        rows_total += dev.lvl[t][0].count;
    }
    // (the partition kernel also zeroes the per-row counts; the array starts on a 256-byte
    // boundary and so does whatever follows it, so whole 64-bit words may be cleared)
    const int64_t cost_words = ((int64_t)(w.Mmax + 1) * k + 1) / 2;
    if (launch_partition(rows, 1, w.P0, 0, nullptr, rows_total, w.parts0.coord, w.parts0.posn, w.parts0.cost,
                         s, reinterpret_cast<unsigned long long *>(w.remap.cost), cost_words) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("rows_partition");
    if (launch_rows_match(dev, w.P0, w.parts0.posn, w.flags, w.qpos, s) != hipSuccess) return NACHO_ERR_HIP;
    profile_mark("rows_match");
    // 2. T (per operand) and the rows' places, 3. its prefix sums: the remapped cost function
    if (launch_remap_rows(dev, w.flags, w.qpos, w.remap, w.tsum, s) != hipSuccess) return NACHO_ERR_HIP;
    profile_mark("remap_rows");
    if (launch_remap_costs(k, w.remap, w.tsum, s) != hipSuccess) return NACHO_ERR_HIP;
    profile_mark("remap_costs");
    // The size of the remapped space (rows all operands store, entries in them) stays on the device:
    // everything below is launched for the upper bounds the workspace was carved for, reads the real
    // sizes there, and lets the surplus workgroups leave at once.  The call never waits for the stream.
    const int64_t capacity = spadd_capacity(SPADD_CSR, dtype) - k;
    if (launch_remap_plan(k, w.remap, capacity, (int64_t)compute_units() * spadd_resident(), P, w.Pmax, w.info,
                          s) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("remap_plan");
    DevOperands mapped;
    std::memset(&mapped, 0, sizeof(mapped));
    mapped.k = k;
    mapped.d = 2;
    for (int t = 0; t < k; ++t) {
        mapped.lvl[t][0].kind = NACHO_DENSE;
        mapped.lvl[t][0].extent = w.Mmax;                       // (upper bound; the real extent is dyn_head[0])
        mapped.lvl[t][1].kind = NACHO_COMPRESSED;
        mapped.lvl[t][1].extent = dev.lvl[t][1].extent;
        mapped.lvl[t][1].pos = w.remap.cost + (size_t)t * (w.Mmax + 1);
        mapped.lvl[t][1].crd = dev.lvl[t][1].crd;
        mapped.lvl[t][1].count = dev.lvl[t][1].count;           // (upper bound; dyn_head[1 + t])
        mapped.start[t] = w.remap.start + (size_t)t * w.Mmax;
    }
    mapped.dyn_head = w.remap.head;
    mapped.dyn_plan = w.info;
    SpaddOut mo = o;                        // the remapped result: CSR over the intersected rows
    mo.pos0 = nullptr;
    mo.crd0 = nullptr;
    mo.pos1 = w.pos_full;
    mo.cap_rows = w.Mmax;
    mo.counts = w.counts;
    if (launch_partition(mapped, 1, w.Pmax, 0, nullptr, total, w.parts.coord, w.parts.posn, w.parts.cost, s,
                         w.tile_state, spadd_state_words(w.Pmax), o.status) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("partition");
    if (launch_spadd(SPADD_CSR, dtype, true, mapped, vals, w.Pmax, w.parts.coord, w.parts.posn, w.tile_state, mo,
                     s) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("spmul_merge");
    if (launch_compact_rows(w.remap, w.pos_full, w.counts, o, w.tsum, s) != hipSuccess) return NACHO_ERR_HIP;
    profile_mark("rows_compact");
    return NACHO_OK;
}

// nacho_spadd_k and nacho_spmul_k: the same pipeline, sums over the union or products over the intersection
static int32_t sparse_combine(bool multiply, const nacho_tensor *ops, int32_t k, int32_t dtype, int64_t P,
                       const nacho_sparse_out *out, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!out || P < 0) return NACHO_ERR_INVALID_ARG;
    if (dtype != NACHO_F32 && dtype != NACHO_F64) return NACHO_ERR_INVALID_ARG;
    DevOperands dev;
    int64_t total = 0;
    Format fmt;
    int32_t rc = check_operands(ops, k, true, &dev, &total, &fmt);
    if (rc != NACHO_OK) return rc;
    if (fmt == FMT_CSF3 && multiply) return NACHO_ERR_UNSUPPORTED;      // third-order tensors: partition and union
    // (the product of one operand is the operand: the union's pipeline copies it)
    if (multiply && fmt == FMT_DCSR && k == 1) multiply = false;
    SpaddValues vals;
    std::memset(&vals, 0, sizeof(vals));
    for (int t = 0; t < k; ++t) {
        const int64_t nt = ops[t].lvl[dev.d - 1].count;
        if (nt > 0 && !ops[t].val) return NACHO_ERR_INVALID_ARG;
        vals.v[t] = ops[t].val;
    }
    if (!out->counts || !out->status || !out->pos1 || out->cap_nnz < 0 || out->cap_rows < 0)
        return NACHO_ERR_INVALID_ARG;
    if (out->cap_nnz > 0 && ((fmt != FMT_CSF3 && !out->crd1) || !out->val)) return NACHO_ERR_INVALID_ARG;
    if (fmt == FMT_DCSR && (!out->pos0 || (out->cap_rows > 0 && !out->crd0))) return NACHO_ERR_INVALID_ARG;
    if (fmt == FMT_COO && out->cap_nnz > 0 && !out->crd0) return NACHO_ERR_INVALID_ARG;
    if (fmt == FMT_CSF3 && (!out->pos0 || !out->pos2 || out->cap_fibres < 0 || (out->cap_rows > 0 && !out->crd0) ||
                            (out->cap_fibres > 0 && !out->crd1) || (out->cap_nnz > 0 && !out->crd2)))
        return NACHO_ERR_INVALID_ARG;
    const int64_t Pe = fused_partitions(NACHO_OP_SPADD, fmt, dtype, k, total, P);
    SpaddWs w = carve_spadd(ws, Pe, k, dev.d);
    const bool recursive = multiply && fmt == FMT_DCSR && k > 1;    // (its own workspace layout)
    if (!recursive && (!ws || ws_bytes < w.bytes)) return NACHO_ERR_WORKSPACE;
    SpaddOut o;
    o.pos0 = out->pos0; o.crd0 = out->crd0; o.pos1 = out->pos1; o.crd1 = out->crd1; o.val = out->val;
    o.cap_rows = out->cap_rows; o.cap_nnz = out->cap_nnz; o.counts = out->counts; o.status = out->status;
    o.pos2 = fmt == FMT_CSF3 ? out->pos2 : nullptr;
    o.crd2 = fmt == FMT_CSF3 ? out->crd2 : nullptr;
    o.cap_fibres = fmt == FMT_CSF3 ? out->cap_fibres : 0;
    const int f = spadd_fmt(fmt);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // a product of DCSR operands intersects the OUTER level
    if (multiply && fmt == FMT_DCSR) return dcsr_product(ops, k, dtype, P, dev, total, vals, o, ws, ws_bytes, s);
    profile_begin(s);
    // the partition kernel also clears the prefix-sum state and the status word of the call
    if (launch_partition(dev, 1, Pe, 0, nullptr, total, w.parts.coord, w.parts.posn, w.parts.cost, s,
                         w.tile_state, spadd_state_words(Pe), o.status) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark("partition");
    if (launch_spadd(f, dtype, multiply, dev, vals, Pe, w.parts.coord, w.parts.posn, w.tile_state, o, s) != hipSuccess)
        return NACHO_ERR_HIP;
    profile_mark(multiply ? "spmul_merge" : "spadd_merge");
    return NACHO_OK;
}

int32_t nacho_spadd_k(const nacho_tensor *ops, int32_t k, int32_t dtype, int64_t P,
                      const nacho_sparse_out *out, void *ws, size_t ws_bytes, void *hip_stream)
{
    return sparse_combine(false, ops, k, dtype, P, out, ws, ws_bytes, hip_stream);
}

int32_t nacho_spadd_fused(const nacho_tensor *ops, int32_t k, int32_t dtype, int64_t P, const nacho_sparse_out *out,
                          void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!out || P < 0) return NACHO_ERR_INVALID_ARG;
    if (dtype != NACHO_F32 && dtype != NACHO_F64) return NACHO_ERR_INVALID_ARG;
    DevOperands dev;
    int64_t total = 0;
    Format fmt;
    int32_t rc = check_operands(ops, k, true, &dev, &total, &fmt);
    if (rc != NACHO_OK) return rc;
    if (fmt != FMT_VECTOR) return NACHO_ERR_UNSUPPORTED;
    SpaddValues vals;
    std::memset(&vals, 0, sizeof(vals));
    for (int t = 0; t < k; ++t) {
        if (ops[t].lvl[0].count > 0 && !ops[t].val) return NACHO_ERR_INVALID_ARG;
        vals.v[t] = ops[t].val;
    }
    if (!out->counts || !out->status || !out->pos1 || out->cap_nnz < 0) return NACHO_ERR_INVALID_ARG;
    if (out->cap_nnz > 0 && (!out->crd1 || !out->val)) return NACHO_ERR_INVALID_ARG;
    const int64_t Pe = fused_partitions(NACHO_OP_SPADD, fmt, dtype, k, total, P);
    SpaddWs w = carve_spadd(ws, Pe, k, dev.d);
    if (!ws || ws_bytes < w.bytes) return NACHO_ERR_WORKSPACE;
    SpaddOut o;
    std::memset(&o, 0, sizeof(o));
    o.pos1 = out->pos1; o.crd1 = out->crd1; o.val = out->val;
    o.cap_nnz = out->cap_nnz; o.counts = out->counts; o.status = out->status;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    profile_begin(s);
    // no partition kernel: the prefix-sum state and the status word are cleared by fill kernels
    if (launch_zero_vector(NACHO_F64, w.tile_state, spadd_state_words(Pe), s) != hipSuccess) return NACHO_ERR_HIP;
    if (launch_zero_vector(NACHO_F32, o.status, 1, s) != hipSuccess) return NACHO_ERR_HIP;
    profile_mark("clear_state");
    SpaddSearch search;
    search.coord = w.parts.coord; search.posn = w.parts.posn; search.cost = w.parts.cost; search.total = total;
    if (launch_spadd_vector_search(dtype, dev, vals, Pe, search, w.tile_state, o, s) != hipSuccess) return NACHO_ERR_HIP;
    profile_mark("spadd_merge_fused");
    return NACHO_OK;
}

int32_t nacho_spmul_k(const nacho_tensor *ops, int32_t k, int32_t dtype, int64_t P,
                      const nacho_sparse_out *out, void *ws, size_t ws_bytes, void *hip_stream)
{
    return sparse_combine(true, ops, k, dtype, P, out, ws, ws_bytes, hip_stream);
}

int32_t nacho_validate(const nacho_tensor *ops, int32_t k, int32_t *status, int64_t *info, void *hip_stream)
{
    if (!status) return NACHO_ERR_INVALID_ARG;
    DevOperands dev;
    int64_t total = 0;
    int32_t rc = check_operands(ops, k, true, &dev, &total, nullptr);
    if (rc != NACHO_OK) return rc;
    if (launch_validate(dev, status, info, static_cast<hipStream_t>(hip_stream)) != hipSuccess) return NACHO_ERR_HIP;
    return NACHO_OK;
}

int32_t nacho_probe(int32_t kind, void *dst, const void *src, size_t bytes, int64_t gathers, void *hip_stream)
{
    if (!src || !dst || bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u))
        return NACHO_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    switch (kind) {
    case NACHO_PROBE_READ: e = launch_probe_read(src, bytes, dst, s); break;
    case NACHO_PROBE_COPY: e = launch_probe_copy(dst, src, bytes, s); break;
    case NACHO_PROBE_GATHER:
        if (gathers < 1) return NACHO_ERR_INVALID_ARG;
        e = launch_probe_gather(src, bytes, gathers, dst, s);
        break;
    default: return NACHO_ERR_INVALID_ARG;
    }
    return e == hipSuccess ? NACHO_OK : NACHO_ERR_HIP;
}

int32_t nacho_instrument(void *records, int64_t capacity)
{
    if (!kInstrument) return NACHO_ERR_UNSUPPORTED;
    if (capacity < 0 || (capacity > 0 && !records)) return NACHO_ERR_INVALID_ARG;
    wave_log().rec = static_cast<WaveRecord *>(records);
    wave_log().capacity = records ? capacity : 0;
    return NACHO_OK;
}

int32_t nacho_instrument_record_bytes(void) { return (int32_t)sizeof(WaveRecord); }

int32_t nacho_merge_wavefronts(void) { return spadd_wavefronts(); }

int32_t nacho_profile_enable(int32_t on)
{
    profiler().enabled = on != 0;
    profiler().n = 0;
    return NACHO_OK;
}

int32_t nacho_profile_read(float *ms, const char **names, int32_t max_n)
{
    Profiler &p = profiler();
    if (!p.enabled || p.n == 0) return 0;
    if (hipEventSynchronize(p.ev[p.n]) != hipSuccess) return NACHO_ERR_HIP;
    for (int i = 0; i < p.n && i < max_n; ++i) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, p.ev[i], p.ev[i + 1]) != hipSuccess) return NACHO_ERR_HIP;
        if (ms) ms[i] = t;
        if (names) names[i] = p.name[i];
    }
    return p.n;
}

}  // extern "C"
