/*
 * libsparsecontract -- sparse-times-dense tensor contractions on one AMD MI355X (gfx950),
 * executed under the fused / fissioned loop nests of "SparseAuto: An Auto-Scheduler for
 * Sparse Tensor Computations Using Recursive Loop Nest Restructuring" (arXiv 2311.09549).
 *
 * The library executes a schedule; it does not search the space of schedules (the
 * compile-time stages of the auto-scheduler of Section 5 are not part of it).  The caller
 * names the expression and the schedule class, or lets the library's run-time stage pick
 * among the schedules it has kernels for (SC_SCHED_AUTO):
 *
 *   kernel 6 of Table 2   A(i,l,m)   = B(i,j,k) * C(j,l) * D(k,m)                    ("ttmc3")
 *   MTTKRP (Section 6)    A(i,r)     = B(i,j,k) * C(j,r) * D(k,r)                    ("mttkrp3")
 *   kernel 1 of Table 2   A(i,l)     = S(i,j) * X(i,k) * Y(j,k) * Z(j,l)             ("sddmm_spmm")
 *   order-4 TTM chain     A(i,l,m,n) = B(i,j,k,p) * C(j,l) * D(k,m) * E(p,n)         ("ttmc4")
 *   kernel 5 of Table 2   A(l,m,n)   = B(i,j,k) * C(i,l) * D(j,m) * E(k,n)           ("ttmc_all")
 *   kernel 8 of Table 2   A(i,m)     = B(i,j,k) * C(j,r) * D(k,r) * E(r,m)           ("mttkrp_gemm")
 *   kernel 2 of Table 2   A(i,m)     = S(i,j) * X(i,k) * Y(j,k) * Z(j,l) * E(l,m)    ("sddmm_spmm_gemm")
 *
 * Index names are free; the FIRST operand on the right-hand side is the sparse one, its
 * first index must be the first output index (except in kernel 5, whose output has no
 * sparse index), and the remaining operands are dense row-major matrices passed in
 * expression order.  Anything outside this family is rejected with SC_ERR_EXPR_UNSUPPORTED.
 *
 * Conventions
 *   - Every function returns an sc_status (0 = SC_OK), never throws, never aborts,
 *     never prints.
 *   - All views are BORROWED: the caller owns every buffer and keeps it alive for the
 *     duration of the call (sc_execute: until the work queued on the stream has run).
 *   - Coordinates and positions are int32 (as in the generated code of Figure 1b);
 *     values are fp32 or fp64; dense operands are row-major with leading dimension `ld`
 *     (in elements), the rank index contiguous; the output is dense, row-major, last
 *     index fastest, and is fully overwritten (rows of empty slices become +0).
 *   - `on_device` says whether the pointers of a view are host (0) or device (1) memory.
 *   - sc_execute allocates nothing, never synchronises and launches only on the stream
 *     it is given.  sc_plan_create allocates the plan-owned device tables: tile records and,
 *     for the kernels that use them, walk tables (4 bytes per stored nonzero and per node of
 *     the level above, see sc_plan_create).
 */
#ifndef SPARSECONTRACT_H
#define SPARSECONTRACT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SC_OK = 0,
    SC_ERR_NULL,              /* a required pointer argument is NULL */
    SC_ERR_BAD_ORDER,         /* sparse order outside 2..4, or it disagrees with the expression */
    SC_ERR_BAD_DTYPE,         /* unknown dtype, or operands of different dtypes */
    SC_ERR_BAD_DIMS,          /* a dimension, nnz or node count is negative / inconsistent / overflows int32 */
    SC_ERR_BAD_POS,           /* a pos array is not monotone, has an empty node, or has wrong end points */
    SC_ERR_CRD_RANGE,         /* a coordinate is outside [0, dim) */
    SC_ERR_UNSORTED,          /* coordinates are not in lexicographic order */
    SC_ERR_DUPLICATE,         /* the same coordinate is stored twice */
    SC_ERR_EXPR_PARSE,        /* the expression string is not well-formed index notation */
    SC_ERR_EXPR_UNSUPPORTED,  /* well-formed, but not a member of the supported family */
    SC_ERR_SCHED_UNSUPPORTED, /* schedule kind / fuse depth / intermediate name not available */
    SC_ERR_SHAPE_MISMATCH,    /* operand shapes disagree with the expression or with the plan */
    SC_ERR_WORKSPACE_SMALL,   /* workspace_bytes < sc_plan_workspace_bytes() */
    SC_ERR_DEVICE,            /* no usable GPU, a HIP call failed, or a host view was given where a device view is needed */
    SC_ERR_ALLOC              /* host allocation failed */
} sc_status;

typedef enum { SC_F32 = 0, SC_F64 = 1 } sc_dtype;

/* Schedule classes of Section 4.2: LINEAR = the perfectly nested default nest, run
 * unfactored (every stored entry times one element of every factor for every combination
 * of the dense output indices): the baseline of the other two, any rank, fp32 / fp64, no
 * temporary, no workspace, sums combined with atomics (deterministic must be 0);
 * FISSIONED = producer and consumer split, the temporary fully materialised (in the
 * workspace, in HBM); FUSED = producer and consumer fused under their common outer
 * loops, the live temporary kept on chip (registers / LDS);
 * AUTO = the library picks: it evaluates the cost expressions of the candidate schedules it has kernels
 * for (iteration count and memory traffic, with the concrete node counts and ranks of the operands)
 * and takes the one of least predicted time among those whose on-chip temporary leaves room for at
 * least two workgroups per compute unit -- the run-time stage of Section 5, with "auxiliary memory
 * below half of the last-level cache" read as "below half of a compute unit's LDS".  sc_plan_chosen
 * and sc_plan_describe report the decision. */
typedef enum { SC_SCHED_LINEAR = 0, SC_SCHED_FUSED = 1, SC_SCHED_FISSIONED = 2, SC_SCHED_AUTO = 3 } sc_sched_kind;

typedef struct sc_plan sc_plan;

/* Sorted coordinate list (Section 2.1): crd[m][z] is the mode-m coordinate of stored
 * entry z; entries are in strictly increasing lexicographic order (mode 0 slowest). */
typedef struct {
    int32_t order;            /* 2..4 */
    int64_t dims[4];
    int64_t nnz;
    sc_dtype dtype;
    const int32_t *crd[4];
    const void *vals;         /* nnz values of `dtype` */
    int32_t on_device;
} sc_coo_view;

/* Compressed sparse fiber tree (Section 2.1), every level compressed:
 *   level 0:  crd[0][s], s < nfib[0]          -- the non-empty top-level slices
 *   level m:  pos[m][p] .. pos[m][p+1]        -- children of node p of level m-1  (nfib[m-1]+1 entries)
 *             crd[m][c], c < nfib[m]          -- coordinate of node c
 *   leaves:   nfib[order-1] == nnz; vals[z] belongs to leaf z.
 * pos[0] is unused (may be NULL).  No node is empty. */
typedef struct {
    int32_t order;
    int64_t dims[4];
    int64_t nnz;
    sc_dtype dtype;
    int64_t nfib[4];
    const int32_t *pos[4];
    const int32_t *crd[4];
    const void *vals;
    int32_t on_device;
} sc_csf_view;

/* Row-major dense matrix: element (r, c) at data[r * ld + c]. */
typedef struct {
    const void *data;
    int64_t rows, cols, ld;
    sc_dtype dtype;
} sc_dense_view;

/* A schedule in closed form (the loopfuse directive of Section 4.4 with the split
 * positions fixed by the expression family): its class, and for each temporary its name
 * and the number of leading common loops fused.
 *   n_intermediates  0 (LINEAR), 1 (orders 2, 3) or 2 (order 4); 0 is also accepted for
 *                    FUSED / FISSIONED and means "the derived ones".
 *   intermediate[t]  optional text such as "T(i,j,m)" or "T1(i,j,k,n)"; when given, its
 *                    index set must equal the one Section 4.2 derives (indices of the
 *                    producer that also occur in the consumer or the output).
 *   fuse_depth[t]    how many leading sparse loops producer and consumer share (the fused prefix of
 *                    Section 4.2).  FISSIONED and AUTO: must be 0.  FUSED: 0 = the depth the library's
 *                    kernel for this expression is built at, or that depth itself (order-3 and order-4
 *                    TTM chains 1: the temporaries of a chunk of a slice in LDS; MTTKRP and the
 *                    SDDMM -> SpMM pair 2: the temporary of one fiber / one stored entry in
 *                    registers); any other value returns SC_ERR_SCHED_UNSUPPORTED rather than being
 *                    ignored.  sc_plan_describe reports the on-chip granularity.
 *   deterministic    0: partial sums of rows that span work tiles are combined with
 *                    floating-point atomics (order may vary from run to run).
 *                    1: every tile stores its piece of such a row in the workspace and a last
 *                    kernel adds the pieces in tile order, so two executions of a plan give
 *                    bit-identical results.  Available for both schedules of the SDDMM -> SpMM
 *                    pair, of the MTTKRP and of the order-3 TTM chain (any supported rank, fp32 /
 *                    fp64) and of the fp32 order-4 TTM chain; under FISSIONED the rows of the
 *                    temporaries that span tiles are treated the same way.  The fp64 order-4
 *                    chain returns SC_ERR_SCHED_UNSUPPORTED.  sc_plan_workspace_bytes then
 *                    includes the pieces. */
typedef struct {
    sc_sched_kind kind;
    int32_t n_intermediates;
    const char *intermediate[2];
    int32_t fuse_depth[2];
    int32_t deterministic;
} sc_schedule;

/* Library version. */
sc_status sc_version(int *major, int *minor);

/* Static English text for a status code (never NULL). */
const char *sc_status_string(sc_status s);

/* Host helper, off the hot path.  Counts the nodes of every CSF level of a sorted,
 * duplicate-free HOST coordinate list (Section 2.1).  Validates order, dims, coordinate
 * ranges, ordering and uniqueness.  nfib_out[m] receives the node count of level m. */
sc_status sc_coo_to_csf_sizes(const sc_coo_view *coo, int64_t nfib_out[4]);

/* Host helper, off the hot path.  Fills a caller-allocated HOST CSF view: the caller sets
 * out->pos[m] (nfib[m-1]+1 int32, m >= 1) and out->crd[m] (nfib[m] int32) to writable host
 * arrays sized from sc_coo_to_csf_sizes, and out->vals either to NULL (the leaf order of a
 * sorted coordinate list IS the CSF leaf order, so the COO value array can be reused) or to
 * a writable array of nnz values, which is then filled.  order, dims, nnz, dtype, nfib and
 * on_device(=0) are written by the call. */
sc_status sc_coo_to_csf(const sc_coo_view *coo, sc_csf_view *out);

/* Validates everything and prepares execution (Section 4.2 for the derivation of the
 * temporaries; Table 2 for the nests).  `expr` is index notation such as
 * "A(i,l,m)=B(i,j,k)*C(j,l)*D(k,m)".  `sparse` may be a host or a device view: its pos
 * arrays (and, for host views, its crd arrays) are checked and the equal-work tile tables
 * are built from them.  Of `factors` only rows / cols / dtype are read.  If a GPU is
 * present the tile tables are uploaded into plan-owned device memory, together with the
 * walk tables of the kernels that use them (the leaf traversal of the FISSIONED schedules,
 * the matrix-core kernels of the TTM chains): a copy of the coordinates of the walked levels
 * with the end-of-node bit folded into bit 31 (4 bytes per stored nonzero, and per node of
 * the level above for the order-4 chain) and 2 bytes per tile and lane group.  Those kernels
 * read the copy instead of the view's arrays of these levels, which is why an execution
 * must be given the view the plan was made from.  Without a GPU the plan is still created
 * (for validation, sizing and description) but cannot execute. */
sc_status sc_plan_create(sc_plan **out, const char *expr, const sc_csf_view *sparse,
                         const sc_dense_view *factors, int32_t nfactors, const sc_schedule *sched);

/* Bytes of device workspace sc_execute needs: the temporaries of the `where` nests of Section 4.2
 * when the schedule materialises them (FISSIONED: T(i,j,m), T1/T2, the sampled values of kernel 1
 * of Table 2), plus the stored row pieces of a deterministic schedule; 0 is possible. */
sc_status sc_plan_workspace_bytes(const sc_plan *plan, size_t *bytes);

/* Human-readable description: the forall/where text of the nest (Section 4.2 notation),
 * the temporaries with their shapes, the flop and compulsory-byte model, tile counts.
 * Always NUL-terminates; truncates to n-1 characters. */
sc_status sc_plan_describe(const sc_plan *plan, char *buf, size_t n);

/* What the plan runs: the schedule class (never SC_SCHED_AUTO: the class the evaluator settled on
 * when AUTO was asked for) and, for the all-mode TTMC, which of the three schedules of Table 2,
 * kernel 5 (1..3; 0 for the other expressions).  Either pointer may be NULL. */
sc_status sc_plan_chosen(const sc_plan *plan, sc_sched_kind *kind, int32_t *table2_schedule);

/* Model figures of the planned schedule: flops (multiply = 1, add = 1) and compulsory HBM
 * bytes (every input array and the output touched once; temporaries of a FISSIONED
 * schedule written once and read once).  Either pointer may be NULL. */
sc_status sc_plan_model(const sc_plan *plan, double *flops, double *bytes);

/* Where FISSIONED temporary `index` lives inside the workspace: byte offset, rows (one per
 * node of the sparse prefix level it is attached to) and columns.  For FUSED plans returns
 * SC_ERR_SCHED_UNSUPPORTED (the temporary never exists in memory). */
sc_status sc_plan_intermediate(const sc_plan *plan, int32_t index, size_t *offset_bytes,
                               int64_t *rows, int64_t *cols);

/* Runs the planned contraction -- the loop nest of its schedule: the perfectly nested default
 * of Section 3 (LINEAR), or the producer / consumer nests of Section 3.1 and Table 2 fused under
 * their common loops or split -- on `hip_stream` (a hipStream_t; NULL = the default stream).
 * `sparse` and every factor must be DEVICE views with the shapes the plan was made for, and
 * `sparse` must have the very pos and crd arrays the plan was built from (tile tables, the list of
 * rows to zero and the numbering of row pieces all come from them; only node counts are
 * re-checked here, so a different tensor of equal node counts gives wrong results); vals and the
 * factor values are free to change between executions.  Every factor spans less than 2 GiB
 * (rows x ld x element size; SC_ERR_SHAPE_MISMATCH otherwise, before anything is launched).
 * `out` is device memory for the whole dense result;
 * `workspace` is device memory of at least sc_plan_workspace_bytes() bytes, 256-byte
 * aligned (may be NULL when that is 0).  Asynchronous: returns after queueing. */
sc_status sc_execute(const sc_plan *plan, const sc_csf_view *sparse, const sc_dense_view *factors,
                     int32_t nfactors, void *out, void *workspace, size_t workspace_bytes,
                     void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): sc_execute with the workspace taken from a fixed array
 * of SC_STATIC_WORKSPACE_BYTES bytes inside the library's device image instead of a caller buffer.
 * Same arguments, checks, kernels and results as sc_execute otherwise.  Calls no hipMalloc /
 * hipFree or any other allocating routine; the array's device address is looked up once per GPU
 * (at the first sc_plan_create or sc_execute_static on that GPU) and the array stays resident on
 * every GPU the library has run on until the process ends.  A plan whose
 * sc_plan_workspace_bytes() exceeds SC_STATIC_WORKSPACE_BYTES is refused with
 * SC_ERR_WORKSPACE_SMALL before anything is launched.  All calls on one GPU share the array, which
 * keeps the contents of the last call (the kernels clear what they need to start from zero):
 * executions that overlap on one GPU (two streams, two plans) race on it -- serialise them, or use
 * sc_execute with separate workspaces. */
#define SC_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)
sc_status sc_execute_static(const sc_plan *plan, const sc_csf_view *sparse, const sc_dense_view *factors,
                            int32_t nfactors, void *out, void *hip_stream);

/* Optional per-kernel timing.  With profiling on, sc_execute brackets each kernel it
 * launches with plan-owned HIP events on the caller's stream; after the caller has
 * synchronised the stream, sc_plan_kernel_time reports the elapsed milliseconds of launch
 * `index` of the most recent sc_execute and its name (name may be NULL).  With profiling off an
 * execution writes nothing that belongs to the plan, so one plan may execute on several streams
 * at once (with separate workspaces and outputs); with profiling on, executions of a plan must
 * not overlap. */
sc_status sc_plan_set_profiling(sc_plan *plan, int32_t on);
sc_status sc_plan_kernel_count(const sc_plan *plan, int32_t *count);
sc_status sc_plan_kernel_time(const sc_plan *plan, int32_t index, char *name, size_t name_len, float *ms);

/* Work-tile introspection (for tests and reports).  A plan cuts the stored nonzeros into
 * contiguous tiles of roughly equal work; rec receives {n0, n1, a0, na, b0, nb, c0, nc, flags}:
 * the leaf range [n0, n1) and, for each CSF level above the leaves (a = parents of the
 * leaves, b = the level above, c = the one above that), the first node and the node count
 * the tile touches; flag bit 2*lvl is set when the first node of that level also has leaves
 * in an earlier tile, bit 2*lvl+1 when the last node also has leaves in a later tile. */
sc_status sc_plan_tile_count(const sc_plan *plan, int64_t *count);
sc_status sc_plan_tile(const sc_plan *plan, int64_t index, int32_t rec[9]);

/* Process-global tuning knobs for experiments; sc_plan_create copies them into the plan it
 * makes, and executions read only that copy (changing a knob never affects an existing plan; set
 * them from one thread, before creating plans).  Names:
 * "tile_leaves", "tile_nodes_a", "tile_nodes_b" (upper bounds on the leaves / level-a /
 * level-b nodes of one work tile; 0 restores the built-in choice), "tile_interleave"
 * (stride of the order in which tiles are handed to workgroups; 1 = tensor order),
 * "persistent_per_cu" (workgroups per compute unit launched by the kernels that loop over
 * tiles; 0 = as many as fit).  Unknown names give
 * SC_ERR_EXPR_PARSE; sc_plan_create rejects caps whose on-chip buffers do not fit. */
sc_status sc_tuning_set(const char *name, int64_t value);

/* Measurement aid, not part of the contraction path: queues a plain streaming copy of
 * `bytes` bytes (a multiple of 16) from `src` to `dst` (both device, 16-byte aligned, not
 * overlapping) on `hip_stream`.  Hardware counters of memory traffic are calibrated against
 * this kernel, whose traffic is known: `bytes` read and `bytes` written.  Returns
 * SC_ERR_NULL for NULL pointers, SC_ERR_BAD_DIMS for a size or pointer that is not a multiple of 16,
 * SC_ERR_DEVICE when the launch fails. */
sc_status sc_stream_copy(void *dst, const void *src, size_t bytes, void *hip_stream);

/* Frees the plan and its device tables (the tile tables cut from the CSF levels of Section 2.1 at
 * plan creation).  NULL is accepted.  Work queued by sc_execute must have finished. */
sc_status sc_plan_destroy(sc_plan *plan);

#ifdef __cplusplus
}
#endif
#endif /* SPARSECONTRACT_H */
