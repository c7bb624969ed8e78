/*
 * nacho.h -- C ABI of the MI355X (gfx950) library for provably load-balanced
 * partitioning of sparse tensor algebra and the partitioned kernels it balances.
 *
 * The operations follow the paper "Partitioning Unstructured Sparse Tensor
 * Algebra for Load-Balanced Parallel Execution":
 *   - nacho_partition : Section 3.2, Algorithm 1 (hierarchical search) with the
 *                       non-zero-count cost functions of Section 4.2.2, stored
 *                       in position space (Section 4.2, 4.2.3);
 *   - nacho_spmv/spmm : the compute kernel of Section 4.4 for y_i = A_ij x_j and
 *                       C_ik = A_ij B_jk (cost scaled by the broadcast extent,
 *                       Section 4.2.2, second listing);
 *   - nacho_spadd_k   : partition -> assembly (count) -> prefix sum -> compute
 *                       (Section 4.3, 4.4, pipeline of Figure 7(a)) for the
 *                       k-operand union of sparse vectors, CSR, DCSR or COO
 *                       matrices (Section 2.1, 2.2);
 *   - nacho_spmul_k   : the same pipeline for the k-operand intersection with
 *                       products (Section 2.1); DCSR operands intersect on the
 *                       outer level and take the recursive partitioning of
 *                       Section 3.3 (Algorithm 2);
 *   - nacho_validate  : debug aid, checks the preconditions below on the device.
 *
 * Conventions that hold for every entry point
 *   * Descriptor structs (nacho_tensor, nacho_parts, nacho_sparse_out) live in
 *     HOST memory and are read during the call only.
 *   * Every array pointer inside them, and every `void*`/typed array argument
 *     that is not explicitly marked "host", is a DEVICE pointer owned by the
 *     caller.  The library allocates and frees nothing; scratch memory comes
 *     from the `ws` argument, sized by nacho_workspace_bytes().
 *   * A call only enqueues kernels on `hip_stream` (a hipStream_t passed as
 *     void*; NULL is the default stream) and returns without synchronising
 *     (nacho_workspace_parts, which launches nothing, reads one word back for a
 *     DCSR product and waits for it).
 *   * Indices and positions are int32; costs are int64.  Preconditions (not
 *     checked): coordinates sorted and unique inside each segment, `pos`
 *     non-decreasing with pos[0] = 0, sum of the operands' nnz < 2^31, all
 *     operands of one call share the same level kinds and extents.
 *   * `crd`, `val` and dense operand arrays must be 16-byte aligned.
 *   * The return value is a status code.  Argument errors are detected on the
 *     host before anything is launched (nothing is written then); a failed HIP
 *     launch maps to NACHO_ERR_HIP.
 *   * Calls that share a workspace or an output must not overlap in time.
 */
#ifndef NACHO_H
#define NACHO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NACHO_OK = 0,
    NACHO_ERR_INVALID_ARG = -1, /* null pointer, bad count, misaligned array, mismatched operands */
    NACHO_ERR_UNSUPPORTED = -2, /* level formats / operand count outside what is implemented      */
    NACHO_ERR_WORKSPACE = -3,   /* ws_bytes smaller than nacho_workspace_bytes() reports           */
    NACHO_ERR_CAPACITY = -4,    /* sparse output larger than the caller's capacity                 */
    NACHO_ERR_HIP = -5,         /* a HIP call failed                                               */
    NACHO_ERR_TOO_LARGE = -6    /* nacho_spmv_static: the call needs more than the built-in scratch */
} nacho_status;

typedef enum { NACHO_F32 = 0, NACHO_F64 = 1 } nacho_dtype;
typedef enum { NACHO_DENSE = 0, NACHO_COMPRESSED = 1, NACHO_NONUNIQUE = 2, NACHO_SINGLETON = 3 } nacho_level_kind;
typedef enum {
    NACHO_OP_PARTITION = 0, NACHO_OP_SPMV = 1, NACHO_OP_SPMM = 2, NACHO_OP_SPADD = 3, NACHO_OP_SPMUL = 4
} nacho_op;

#define NACHO_MAX_OPERANDS 8
#define NACHO_MAX_LEVELS 3

/* One level of a tensor's coordinate hierarchy (Section 4.2.1).
 *   DENSE:      every coordinate in [0, extent) is present; pos, crd are NULL.
 *   COMPRESSED: pos[parent] .. pos[parent+1] delimit the sorted coordinates
 *               crd[] stored below `parent` (a top level has one parent, so
 *               pos has 2 entries).  `count` is the number of entries of crd.
 *   NONUNIQUE:  a top compressed level whose sorted coordinates may repeat, one
 *               entry per stored non-zero (the row level of a coordinate list);
 *               crd[count]; pos is not read.
 *   SINGLETON:  one coordinate per entry of the level above: crd[count], the
 *               same count (the column level of a coordinate list).            */
typedef struct {
    int32_t kind;       /* nacho_level_kind                                    */
    int64_t extent;     /* N_m, at most 2^31 - 1                               */
    const int32_t *pos; /* device, [parents + 1]                               */
    const int32_t *crd; /* device, [count]                                     */
    int64_t count;      /* stored coordinates at this level (COMPRESSED only)  */
} nacho_level;

/* A sparse operand.  Supported shapes:
 *   sparse vector  nlevels = 1  {COMPRESSED}
 *   CSR            nlevels = 2  {DENSE, COMPRESSED}
 *   DCSR           nlevels = 2  {COMPRESSED, COMPRESSED}
 *   CSF            nlevels = 3  {COMPRESSED, COMPRESSED, COMPRESSED}: third-order
 *                  tensors (nacho_partition and nacho_spadd_k)
 *   COO            nlevels = 2  {NONUNIQUE, SINGLETON}: entries sorted by (row,
 *                  column), no pair twice (nacho_partition, nacho_spadd_k,
 *                  nacho_spmul_k)
 * `val` (device, one value per innermost coordinate) may be NULL for
 * nacho_partition. */
typedef struct {
    int32_t nlevels;
    nacho_level lvl[NACHO_MAX_LEVELS];
    const void *val;
} nacho_tensor;

/* Stored result of the search (Section 4.2.3: the positions found by the
 * search are kept for the assembly and compute stages).  P partitions have
 * P + 1 boundaries; boundary 0 is the origin, boundary P the end of the
 * iteration space, and partition p spans boundaries p .. p+1.
 *   coord[b*d + m]          coordinate x_m of boundary b
 *   posn[(b*k + t)*d + m]   for operand t: position of the first level-m entry
 *                           that is not before the boundary (DENSE level: x_m)
 *   cost[b]                 C(x) of boundary b = work strictly before it      */
typedef struct {
    int32_t k, d;
    int64_t P;
    int32_t *coord; /* device, [(P+1) * d]     */
    int32_t *posn;  /* device, [(P+1) * k * d] */
    int64_t *cost;  /* device, [P+1]           */
} nacho_parts;

/* Caller-allocated sparse result of nacho_spadd_k, in the operands' format.
 *   vector: crd1[cap_nnz], val[cap_nnz]; pos1[2] = {0, nnz}
 *   CSR:    pos1[n_rows+1], crd1[cap_nnz], val[cap_nnz]
 *   DCSR:   pos0[2] = {0, rows}, crd0[cap_rows], pos1[cap_rows+1], crd1, val
 *   COO:    crd0[cap_nnz] (rows), crd1[cap_nnz] (columns), val[cap_nnz];
 *           pos1[2] = {0, nnz}; cap_rows is not used
 *   CSF (third order, three compressed levels): pos0[2] = {0, slices},
 *           crd0[cap_rows] (i), pos1[cap_rows+1], crd1[cap_fibres] (j),
 *           pos2[cap_fibres+1], crd2[cap_nnz] (k), val[cap_nnz]
 * counts[0] = stored rows (DCSR; n_rows for CSR; 1 for a vector), counts[1] =
 * nnz; for CSF counts = {slices, fibres, nnz}.  counts always has room for
 * three words.  pos2, crd2 and cap_fibres are read for CSF only.  *status is
 * set to NACHO_OK, or to NACHO_ERR_CAPACITY when cap_rows, cap_fibres or
 * cap_nnz is too small (then nothing is written beyond the capacities; counts
 * still hold the required sizes).  The sums of the operands' counts are always
 * sufficient capacities. */
typedef struct {
    int32_t *pos0;
    int32_t *crd0;
    int32_t *pos1;
    int32_t *crd1;
    void *val;
    int64_t cap_rows, cap_nnz;
    int64_t *counts; /* device, [3] */
    int32_t *status; /* device, [1] */
    int32_t *pos2;   /* CSF only */
    int32_t *crd2;   /* CSF only */
    int64_t cap_fibres;
} nacho_sparse_out;

/* Library version (major*10000 + minor*100 + patch) and a static string for a status. */
int32_t nacho_version(void);
const char *nacho_status_string(int32_t status);

/* Number of partitions a fused call uses for these operands (host descriptors;
 * only counts/extents are read) when the caller asks for `P` (0 = automatic).
 * Fused calls never use fewer partitions than needed for one partition's work
 * to fit the staging buffer of its wavefront (SpMV, SpMM) or workgroup (SpAdd,
 * SpMul), so the result is >= P.  For a DCSR product it is an upper bound (the
 * count depends on the rows the operands share).  `n_dense`: SpMM's dense
 * extent (0 otherwise).  Returns 0 on bad input. */
int64_t nacho_num_partitions(int32_t op, const nacho_tensor *ops, int32_t k, int32_t dtype,
                             int64_t n_dense, int64_t P);

/* Bytes of device workspace `op` needs for these operands (host descriptors;
 * only counts/extents are read).  `P` as passed to the call (0 = automatic),
 * `n_dense` = columns of B for SpMM (0 otherwise).  NACHO_OP_SPADD sizes
 * nacho_spadd_k, NACHO_OP_SPMUL nacho_spmul_k. */
int32_t nacho_workspace_bytes(int32_t op, const nacho_tensor *ops, int32_t k, int32_t dtype,
                              int64_t n_dense, int64_t P, size_t *bytes);

/*
 * Algorithm 1 for all P+1 boundaries of a P-way partition, one independent
 * search per interior boundary (Section 3.2; Section 4.2.3).
 *   ops[k]        coiterated operands (1 <= k <= NACHO_MAX_OPERANDS)
 *   cost_scale    >= 1; every stored non-zero costs this much (the extent of a
 *                 broadcast dense inner loop, Section 4.2.2).  Queries are then
 *                 interpreted in scaled units and boundaries never fall inside
 *                 the dense loop: the boundary of query Q is that of
 *                 floor(Q / cost_scale) in unscaled units.
 *   P             number of partitions (>= 1)
 *   queries       device int64[P+1] or NULL.  NULL: Q_p = floor(p*Q_total/P).
 *                 Entries 0 and P are ignored (origin / end); an interior
 *                 query >= Q_total yields the end boundary.
 *   out           coord/posn/cost arrays of the sizes documented above
 * Errors: INVALID_ARG (null/size/kind), UNSUPPORTED (format), WORKSPACE, HIP.
 */
int32_t nacho_partition(const nacho_tensor *ops, int32_t k, int64_t cost_scale, int64_t P,
                        const int64_t *queries, const nacho_parts *out,
                        void *ws, size_t ws_bytes, void *hip_stream);

/*
 * nacho_partition for ONE CSR operand whose positions are 64-bit: operands of
 * 2^31 stored non-zeros or more, which the int32 descriptors above cannot
 * describe (Section 4.2.2's CSR cost functions, C_i(x) = pos[x] and the count
 * of the row's entries before a column; equal-share queries
 * Q_p = floor(p * nnz / P)).
 *   pos     device int64[n_rows + 1], non-decreasing, pos[0] = 0, pos[n_rows] = nnz
 *   crd     device int32[nnz], 16-byte aligned
 *   coord   device int32[(P+1) * 2]   (row, column) of every boundary
 *   posn    device int64[(P+1) * 2]   (row, position of the first entry not
 *           before the boundary)
 *   cost    device int64[P+1]
 * Rows and columns stay below 2^31.  Enqueues only.  Errors: INVALID_ARG, HIP.
 */
int32_t nacho_partition_csr64(const int64_t *pos, const int32_t *crd, int64_t n_rows, int64_t n_cols, int64_t nnz,
                              int64_t P, int32_t *coord, int64_t *posn, int64_t *cost, void *hip_stream);

/*
 * Where a fused call keeps its stored partitions (Section 4.2.3: the positions
 * found by the search are kept for the assembly and compute stages).  Fills
 * `parts` (host struct) with the number of partitions the fused call `op` uses
 * for these operands and with DEVICE pointers into the workspace `ws` the call
 * was (or will be) given; the table is valid once that call has run.  Nothing
 * is launched.  One case waits: for nacho_spmul_k on DCSR operands the number of
 * partitions is a result of the call's own kernels; it is read back on
 * `hip_stream` (the stream that call was enqueued on) and the function returns
 * once the stream has reached that point.  `hip_stream` is not used otherwise.  `grain` (host, may be NULL) receives G when the call uses the
 * fixed-grain queries Q_p = min(p*G, Q_total) (SpMV and SpMM with P = 0; G is
 * in scaled units, a multiple of n_dense for SpMM), 0 when it uses
 * Q_p = floor(p*Q_total/P).  Arguments as for nacho_workspace_bytes.
 */
int32_t nacho_workspace_parts(int32_t op, const nacho_tensor *ops, int32_t k, int32_t dtype,
                              int64_t n_dense, int64_t P, void *ws, size_t ws_bytes,
                              nacho_parts *parts /* host */, int64_t *grain /* host */, void *hip_stream);

/*
 * y = A x with A in CSR (Section 4.2.2 uses this expression for the broadcast
 * rule; the cost of a partition is its number of stored non-zeros of A, the
 * dense x is only located into).  One wavefront executes one partition; a row
 * split across partitions is completed by a deterministic carry fix-up pass.
 *   A      CSR, val of type `dtype`;  x[n_cols], y[n_rows] of type `dtype`
 *   P      0 = automatic, else the minimum number of partitions
 * Every y[i] is written (exactly 0 for an empty row).
 */
int32_t nacho_spmv(const nacho_tensor *A, const void *x, void *y, int32_t dtype, int64_t P,
                   void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Row-aware cost (a variant; Section 4.2.2 remarks that the non-zero count only
 * approximates the run time, and a partition of 512 one-entry rows does more
 * than one of a single 512-entry row).  Every row of A costs `row_cost` units
 * (0 .. 64) on top of its stored non-zeros, charged in front of its first
 * column: C_i(r) = pos[r] + row_cost * r, C_j(x | r) = (x > 0 ? row_cost : 0) +
 * entries of row r with column < x -- monotone and hierarchically consistent
 * (Section 3.1), so Algorithm 1 applies unchanged; a boundary may fall at
 * (r, 0), also in an empty row.  row_cost = 0 is the paper's cost.
 *   nacho_partition_rowcost   boundaries of one CSR operand, queries
 *                             floor(p * total / P) with total = nnz + row_cost * rows;
 *                             `out` as for nacho_partition (k = 1, d = 2)
 *   nacho_spmv_rowcost        y = A x on those partitions; uses
 *                             nacho_rowcost_partitions(A, dtype, row_cost, P)
 *                             partitions (at least P, and enough that a
 *                             partition's cost fits one wavefront) and needs the
 *                             workspace nacho_workspace_bytes reports for
 *                             NACHO_OP_SPMV with that partition count
 * Errors as for nacho_partition / nacho_spmv.
 */
int64_t nacho_rowcost_partitions(const nacho_tensor *A, int32_t dtype, int64_t row_cost, int64_t P);
int32_t nacho_partition_rowcost(const nacho_tensor *A, int64_t row_cost, int64_t P, const nacho_parts *out,
                                void *hip_stream);
int32_t nacho_spmv_rowcost(const nacho_tensor *A, const void *x, void *y, int32_t dtype, int64_t row_cost,
                           int64_t P, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * nacho_spmv without a partition pass (a P-free, fused search-in-execute form):
 * there is no partition table; every wavefront of the executing kernel finds its
 * own two boundaries -- Algorithm 1 for one CSR operand with the fixed-grain
 * queries Q_b = min(b * G, nnz), G = one wavefront's capacity, i.e. the row with
 * pos[r] <= Q_b < pos[r+1] by a 64-ary search over pos -- and y is cleared by a
 * small fill kernel first.  Same partitions, same arithmetic and the same result
 * as nacho_spmv with P = 0; it trades the partition kernel's one pass over pos
 * for two searches per wavefront (a measured variant, not the default).
 * Workspace: nacho_workspace_bytes(NACHO_OP_SPMV, ..., P = 0).
 */
int32_t nacho_spmv_fused(const nacho_tensor *A, const void *x, void *y, int32_t dtype, void *ws, size_t ws_bytes,
                         void *hip_stream);

/*
 * nacho_spadd_k on sparse vectors without a partition pass (the fused
 * search-in-execute form of the merge path; the paper's partitions "computed in
 * parallel" with the kernel they balance, Sections 1 and 2.1): every workgroup
 * of the merge kernel searches its own two boundaries with Algorithm 1
 * (Section 3.2; wavefront 0 the lower one, wavefront 1 the upper one, equal-share
 * queries Q_p = floor(p Q* / P)) and stores them in the partition table of the
 * workspace, which nacho_workspace_parts returns as after nacho_spadd_k; two
 * small fill kernels clear the prefix-sum state and the status word first.  Same
 * partitions, same result arrays, counts and status as nacho_spadd_k; other
 * formats: NACHO_ERR_UNSUPPORTED.  A measured variant, not the default: a
 * boundary search is as long as a workgroup's whole merge, and here every
 * workgroup waits for two of them.  Workspace: nacho_workspace_bytes(NACHO_OP_SPADD, ...).
 */
int32_t nacho_spadd_fused(const nacho_tensor *ops, int32_t k, int32_t dtype, int64_t P, const nacho_sparse_out *out,
                          void *ws, size_t ws_bytes, void *hip_stream);

/*
 * nacho_spmv for callers that cannot allocate device memory or pass a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc).  Same operation, arguments, results and status codes as nacho_spmv,
 * but the partition table and the carries live in a scratch array that is part of
 * the library's code object (one copy per GPU, nacho_static_scratch_bytes() bytes,
 * held until the process ends) instead of a caller's workspace.  The call
 * allocates and frees nothing and only enqueues.  A matrix whose partitions do
 * not fit that array (about 36 bytes per partition, i.e. per 512 fp64 / 1024 fp32
 * non-zeros, or per requested partition when P is given) is refused with
 * NACHO_ERR_TOO_LARGE before anything is launched.  All calls on one GPU share
 * the array: two calls that overlap in time on one GPU (different streams or
 * threads) race; calls on one stream are ordered and safe.  The first call on a
 * device looks the array's address up (hipGetSymbolAddress), once.
 */
int32_t nacho_spmv_static(const nacho_tensor *A, const void *x, void *y, int32_t dtype, int64_t P,
                          void *hip_stream);
size_t nacho_static_scratch_bytes(void);

/*
 * C = A B with A in CSR and B, C dense row-major (loop order i -> j -> k, dense
 * k innermost; cost of a stored non-zero = n, the broadcast extent).
 *   B[n_cols(A) x n] leading dimension ldb,  C[n_rows(A) x n] leading dimension
 *   ldc (elements); n >= 1.  The executing kernel covers 64 columns at a time:
 *   a wider B goes through it in stretches of 64 columns over the same
 *   partitions (A is then read once per stretch).
 */
int32_t nacho_spmm(const nacho_tensor *A, const void *B, int64_t n, int64_t ldb,
                   void *C, int64_t ldc, int32_t dtype, int64_t P,
                   void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Z = sum_t ops[t]: the union of k sparse vectors, CSR, DCSR or COO matrices
 * or third-order CSF tensors with sorted output coordinates; coinciding values
 * are added in operand order.  Two kernels: the partition search, then one
 * merge kernel whose workgroup p stages, merges, assembles and writes
 * partition p.
 *
 * Where workgroup p writes depends on what the workgroups before it emit, and
 * it learns that inside the kernel: every workgroup publishes its counts in
 * the workspace and reads those of its predecessors, polling a bounded number
 * of times for the ones not there yet.  This relies on the GPU starting the
 * workgroups of a launch in the order of their indices, so that a workgroup
 * only ever waits for workgroups that are already running or done; HIP does
 * not promise that order, every AMD GPU so far keeps it.  Should a wait run
 * out all the same (about 2^14 polls of a few hundred nanoseconds each), the
 * workgroup writes nothing and *status becomes NACHO_ERR_HIP: the output is
 * then incomplete and the call must be repeated.  Among several conditions the
 * gravest (lowest) status wins.
 */
int32_t nacho_spadd_k(const nacho_tensor *ops, int32_t k, int32_t dtype, int64_t P,
                      const nacho_sparse_out *out, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Z = prod_t ops[t] over the INTERSECTION of the operands' stored coordinates:
 * the k-way product of sparse vectors (the three-finger loop of Section 2.1,
 * z_i = a_i b_i c_i) or the Hadamard product of k CSR matrices.  The
 * intersection is on the innermost level, so the partitions are those of
 * Algorithm 1 on the operands' non-zero counts, exactly as for nacho_spadd_k
 * (Section 3.3: only an outer intersection needs the recursive partitioning);
 * an entry is emitted when all k operands store its coordinate, its value is
 * the product in operand order.  Same arguments, output layout, status and
 * capacity rules as nacho_spadd_k (min_t nnz_t is always a sufficient cap_nnz).
 *
 * DCSR operands intersect on the OUTER level as well, and rows that not every
 * operand stores are skipped with everything below them, so the plain non-zero
 * count is the wrong cost.  The call then follows the recursive partitioning of
 * Section 3.3 (Algorithm 2): a first, separately partitioned loop intersects
 * the operands' row coordinates and memoises, for the i'-th row all operands
 * store, T[i'] = the number of entries the operands store in it; the prefix sum
 * T' is the remapped cost function C'_i(x) = T'[x]; Algorithm 1 on the
 * remapped nest (i' over the intersected rows, then the columns) gives the
 * partitions of the product.  A row of the result is stored only when it holds
 * an entry (min_t rows_t is always a sufficient cap_rows).  The stored
 * partitions (nacho_workspace_parts with NACHO_OP_SPMUL, after the call) are
 * those of the remapped nest, a CSR-like space: coord = (i', j), posn[..][0] =
 * i', posn[..][1] = the number of entries the operand stores in the
 * intersected rows before the boundary.  Workspace: nacho_workspace_bytes with
 * NACHO_OP_SPMUL.  Like every other call this one only enqueues: the size of the
 * remapped space stays on the device, the kernels after the row loop are launched
 * for upper bounds (the sizes the workspace is carved for) and read the real
 * sizes there.
 */
int32_t nacho_spmul_k(const nacho_tensor *ops, int32_t k, int32_t dtype, int64_t P,
                      const nacho_sparse_out *out, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Debug aid, not part of the hot path: checks on the device the preconditions
 * that the other entry points rely on without looking -- pos arrays start at 0,
 * never decrease and end at the level's count; coordinates lie inside the
 * extents and ascend strictly inside every segment (coordinate lists: the
 * (row, column) pairs ascend strictly).  Enqueues only.  *status (device)
 * becomes NACHO_OK or NACHO_ERR_INVALID_ARG; info (device int64[3], may be
 * NULL) = {operand, level, position} of one violation, {-1, -1, -1} if none.
 * The return value covers what the host can see (null pointers, kinds, counts).
 */
int32_t nacho_validate(const nacho_tensor *ops, int32_t k, int32_t *status /* device */,
                       int64_t *info /* device */, void *hip_stream);

/*
 * Machine ceilings for benchmarks (not part of the hot path): kernels of known
 * traffic, timed by the caller on the same GPU in the same run.  Enqueues only.
 *   NACHO_PROBE_READ    reads `bytes` of src once (dst: 8 writable device bytes)
 *   NACHO_PROBE_COPY    copies `bytes` from src to dst
 *   NACHO_PROBE_GATHER  `gathers` independent 8-byte loads at pseudo-random places
 *                       of the first `bytes` of src (dst: 8 writable device bytes):
 *                       what a row-major CSR SpMV does to x per stored non-zero
 * src, dst: device, 16-byte aligned; bytes >= 16.
 */
typedef enum { NACHO_PROBE_READ = 0, NACHO_PROBE_COPY = 1, NACHO_PROBE_GATHER = 2 } nacho_probe_kind;
int32_t nacho_probe(int32_t kind, void *dst, const void *src, size_t bytes, int64_t gathers, void *hip_stream);

/*
 * Per-wavefront measurements (not part of the hot path; benchmarks and tests of
 * the load balance use it).  Only the instrumented build of the library
 * (libnacho_instr.so, the same sources compiled with -DNACHO_INSTRUMENT) records
 * anything; the ordinary build returns NACHO_ERR_UNSUPPORTED.  After
 * nacho_instrument(records, capacity), wavefront i of every launch of an
 * executing kernel (SpMV, SpMM: workgroup i; the merge kernel: workgroup i / 8,
 * wavefront i % 8) overwrites record i < capacity of the caller's DEVICE buffer
 * when it ends; records = NULL switches the log off.  A record is
 * nacho_instrument_record_bytes() = 40 bytes:
 *   uint64 t_begin, t_end   constant 100 MHz counter, comparable across the chip
 *   uint64 cycles           shader clock cycles between the two
 *   uint32 items, rows      stored non-zeros (merge kernel: merged places) and rows
 *                           (merge kernel: output rows started) the wavefront worked on
 *   uint32 hw_id, xcc_id    where it ran (HW_ID and XCC_ID hardware registers)
 */
int32_t nacho_instrument(void *records /* device */, int64_t capacity);
int32_t nacho_instrument_record_bytes(void);
/* Wavefronts per workgroup (= per partition) of the merge kernel of nacho_spadd_k / nacho_spmul_k. */
int32_t nacho_merge_wavefronts(void);

/*
 * Per-kernel timing for benchmarks (not part of the hot path).  While enabled,
 * every fused call brackets each of its kernels with HIP events on the call's
 * stream.  nacho_profile_read synchronises on those events and returns the
 * number of kernels of the last call; ms[i] and names[i] (static strings,
 * host) are filled for i < min(n, max_n).
 */
int32_t nacho_profile_enable(int32_t on);
int32_t nacho_profile_read(float *ms /* host */, const char **names /* host */, int32_t max_n);

#ifdef __cplusplus
}
#endif
#endif /* NACHO_H */
