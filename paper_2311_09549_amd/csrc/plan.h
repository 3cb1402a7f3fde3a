// Internal definitions shared by the host planner and the HIP launchers of
// libsparsecontract.  Not part of the public C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/sparsecontract.h"

namespace sck {

enum Kind { K_TTMC3 = 0, K_MTTKRP3 = 1, K_SDDMM_SPMM = 2, K_TTMC4 = 3, K_TTMC_ALL = 4, K_MTTKRP_GEMM = 5, K_SDDMM_SPMM_GEMM = 6 };

// One work tile: a contiguous range of leaves (stored nonzeros) together with the range
// of CSF nodes that contain them at every level above.  Level "a" is the parent level of
// the leaves, "b" the level above it, "c" the one above that (unused levels are zero).
//   order 2: a = rows
//   order 3: a = (i,j) fibers, b = slices
//   order 4: a = (i,j,k) fibers, b = (i,j) fibers, c = slices
// A node that also has leaves outside [n0, n1) is "partial"; flag bit 2*lvl says the first
// node of that level continues from the previous tile, bit 2*lvl+1 that the last node
// continues into the next tile (lvl: a = 0, b = 1, c = 2).
struct TileRec {
    int32_t n0, n1;
    int32_t a0, na;
    int32_t b0, nb;
    int32_t c0, nc;
    int32_t flags;
    int32_t pad[3];
};
static_assert(sizeof(TileRec) == 48, "TileRec layout");

// Per-level caps of a tile (upper bounds on leaves / nodes it may hold); they size the LDS
// arrays of the kernels.
struct TileCaps {
    int32_t tn;  // leaves
    int32_t ta;  // level-a nodes
    int32_t tb;  // level-b nodes (order 4 only; for order 3 the slice count is bounded by ta)
};

constexpr int kMaxLaunches = 12;

// Deterministic schedules: an output row whose slice spans several tiles is not updated with
// atomics; every tile stores its piece of the row in a slot of the workspace (the two slot
// numbers of a tile for output rows are in TileRec::pad[0] / pad[1], -1 = none; the pieces of one row occupy
// consecutive slots in tile order) and two last kernels add the pieces of each row in that
// order: first in segments of kFixSegment pieces (many workgroups per heavy row), then the
// segment sums.  Both are described by the same record.
struct FixRec {
    int32_t row;     // destination row: segment number (first pass) or coordinate of the slice (second pass)
    int32_t first;   // first source row: slot (first pass) or segment (second pass)
    int32_t count;   // number of source rows
    int32_t pad;
};
constexpr int kFixSegment = 64;

// The rows of one level that span several tiles under a deterministic schedule.
struct FixLevel {
    std::vector<FixRec> fix;      // second pass: one record per spanning row
    std::vector<FixRec> segs;     // first pass: its pieces in segments
    FixRec *d_fix = nullptr;      // plan-owned device copies
    FixRec *d_segs = nullptr;
    int64_t n_slots = 0;          // pieces in the workspace
    int64_t rowlen = 0;           // elements per row
    size_t slot_offset = 0;       // byte offsets inside the workspace: the pieces ...
    size_t seg_offset = 0;        // ... and the segment sums
};

// Process-global tuning overrides (0 = use the built-in choice); a plan copies them when it is created.
struct Tuning {
    int32_t tn = 0, ta = 0, tb = 0;
    int32_t interleave = 0;  // stride of the tile upload order (0 = built-in)
    int32_t per_cu = 0;      // workgroups per compute unit of the persistent kernels (0 = as many as fit)
};

// HIP events around every launch of the most recent execution (sc_plan_set_profiling).
struct ProfileState {
    bool on = false;
    int32_t n_launch = 0;
    const char *launch_name[kMaxLaunches];
    hipEvent_t ev_begin[kMaxLaunches];
    hipEvent_t ev_end[kMaxLaunches];
};

// Walk tables: what the segmented walks of a tile need to know about the node boundaries, worked out
// once when the plan is made instead of by every tile of every execution.
//   rec[0]   one word per stored nonzero: its last coordinate, bit 31 set when it is the last of its fiber
//   rec[1]   one word per node of level "a": its coordinate, bit 31 set when it is the last child of its parent
//   heads    per tile (in the order of the device tile table) one 16-bit entry per lane group of the leaf walk,
//            then one per lane group of the walk one level up: the tile-local index of the node that holds the
//            first child of the group's chunk (chunks of walk_chunk children), bit 15 set when that node began
//            in an earlier chunk
// The lane-group counts and batch sizes are those of the kernel the plan dispatches to.
struct WalkShape {
    int32_t levels = 0;          // 0 = the plan's kernels keep no walk tables
    int32_t groups[2] = {0, 0};  // lane groups of the leaf walk / of the walk over level-a nodes
    int32_t batch[2] = {1, 1};   // children a lane group takes per step (chunks are multiples of it)
};

struct WalkTables {
    WalkShape shape;
    uint32_t *d_rec[2] = {nullptr, nullptr};
    uint16_t *d_heads = nullptr;
    int32_t heads_per_tile = 0;
};

// Children per lane group for a tile of n children: a multiple of the batch size u.
__host__ __device__ inline int walk_chunk(int n, int groups, int u)
{
    const int q = ((n + groups - 1) / groups + u - 1) / u * u;
    return q > u ? q : u;
}

struct Intermediate {
    std::string name;   // e.g. "T(i,j,m)"
    size_t offset = 0;  // byte offset inside the workspace (FISSIONED only)
    int64_t rows = 0, cols = 0;
};

}  // namespace sck

struct sc_plan {
    sck::Kind kind;
    sc_dtype dtype;
    int32_t order;
    int64_t dims[4];
    int64_t nnz;
    int64_t nfib[4];
    int32_t nfactors;
    int32_t slot_of_factor[4];   // canonical slot -> position in the caller's factor array
    int64_t frows[4], fcols[4];  // canonical slots
    int64_t out_elems;
    int64_t out_row_elems;       // elements of one output row (per top-level slice)

    sc_sched_kind sched;
    int32_t fuse_depth[2];
    int32_t n_inter;
    sck::Intermediate inter[2];

    sck::TileCaps caps;
    std::vector<sck::TileRec> tiles;  // host copy
    sck::TileRec *d_tiles = nullptr;  // plan-owned device copy
    bool has_device = false;

    // Output rows that no kernel overwrites completely: rows of empty slices, and (atomic
    // schedules) rows whose slice spans several tiles.  When they are few, only they are zeroed
    // before the kernels run; otherwise the whole output is.
    std::vector<int32_t> zero_rows;
    int32_t *d_zero_rows = nullptr;   // plan-owned device copy
    bool zero_selective = false;

    size_t ws_bytes = 0;
    bool deterministic = false;
    sck::FixLevel det_top;   // output rows (slices) that span tiles; slot numbers in TileRec::pad[0] / pad[1]
    sck::FixLevel det_a;     // FISSIONED, order >= 3: rows of the first temporary (leaf fibers) that span tiles; a
                             // tile's pieces are numbered TileRec::pad[2] (first fiber, if it continues from the
                             // previous tile) and the next number (last fiber, if it continues into the next)
    sck::FixLevel det_b;     // FISSIONED, order 4: rows of the second temporary (level-b nodes) that span tiles,
                             // numbered the same way from slot_b[tile]
    std::vector<int32_t> slot_b;
    int32_t *d_slot_b = nullptr;   // plan-owned device copy, in the order of the device tile table
    sck::WalkTables walk;          // plan-owned device tables of the segmented walks (kernels that use them)
    double model_flops = 0, model_bytes = 0;
    std::string text;  // description

    // All-mode TTMC (kernel 5 of Table 2): the sparse part runs as an inner plan of the order-3 chain
    // S(i,m,n) = B(i,j,k) D(j,m) E(k,n) over the same tensor; the contraction with C(i,l) is a grid-wide
    // reduction through per-workgroup slots of the workspace.
    sc_plan *inner = nullptr;          // owned
    int32_t k5_variant = 0;            // which schedule of Table 2: 1, 2 or 3
    size_t k5_s_offset = 0;            // S, dims[0] x (M N) (variants 2, 3)
    size_t k5_inner_ws_offset = 0;     // workspace of the inner plan
    size_t k5_partials_offset = 0;     // k5_nchunks x L x (M N)
    int64_t k5_nchunks = 0, k5_chunk = 0;
    bool k5_mfma_reduce = false;       // the contraction over the first mode runs on the matrix cores (fp32, L in {16, 32, 64, 128}, M N a multiple of 64)

    // Trailing dense product (kernels 8 and 2 of Table 2): the sparse part runs as an inner plan (MTTKRP, or kernel 1)
    // whose rows, one per coordinate of the first mode, pass through the workspace.
    size_t tg_rows_offset = 0, tg_inner_ws_offset = 0;

    // Snapshot of the tuning knobs and of the device the plan was made on (taken once, at plan
    // creation): an execution reads only these, never process-global state.
    sck::Tuning tune;
    int32_t n_cu = 256;                 // compute units of the device (hipDeviceProp; the value without a device is MI355X's)
    int64_t lds_per_cu = 160 * 1024;    // LDS bytes per compute unit

    // Per-kernel timing (optional).  The record lives behind a pointer: an execution with profiling
    // off writes nothing that belongs to the plan, so such executions of one plan may overlap on
    // several streams; with profiling on they must not.
    sck::ProfileState *prof = nullptr;
};

namespace sck {

Tuning &tuning();

// Workgroups using `lds` bytes of LDS each that one compute unit holds at a time: the unit's LDS
// (160 KB on MI355X) is handed out in units of 1280 bytes (measured: a fifth workgroup of 31,880
// bytes fits, one of 32,232 does not).  The kernels here are bound by latency, and their time
// falls almost in proportion to this number, so tile sizes are chosen to land just below a step.
inline int lds_workgroups_per_cu(size_t lds, int64_t lds_per_cu = 160 * 1024)
{
    const size_t unit = 1280;
    const size_t need = std::max<size_t>(unit, (lds + unit - 1) / unit * unit);
    return (int)std::max<size_t>(1, std::min<size_t>(8, (size_t)lds_per_cu / need));
}


// Built-in tile caps for a contraction (host side; the kernels size their LDS from them).
TileCaps default_caps(Kind kind, sc_dtype dtype, sc_sched_kind sched, const int64_t *fcols);

// True when the plan's kernels walk contiguous runs of tiles and therefore want the device tile
// table in tensor order rather than interleaved.
bool plan_wants_tensor_order(const sc_plan *plan);

// Tiles per workgroup of the kernel that writes the plan's output rows when that kernel is persistent over contiguous
// runs of tiles (the matrix-core kernels); 0 for the kernels that take one tile per workgroup.  Within a run a slice that
// continues from tile to tile stays in registers and is stored once; only a slice that crosses a run's end is added
// atomically, so only those rows have to start from zero.  The launchers use the same number.
int plan_output_run(const sc_plan *plan);

// True for the FUSED order-3 chains that run the matrix-core kernel for rank pairs beyond 16 x 16 (kernels_ttmc3w.hip).
bool plan_uses_wide_ttmc3(const sc_plan *plan);

// True when the kernels of the plan can run without floating-point atomics (FUSED schedules of
// the kernels that emit one piece per tile and shared row).
bool plan_supports_deterministic(const sc_plan *plan);

// Lane-group layout of the walks of the kernels the plan dispatches to (levels = 0: no walk tables).
WalkShape plan_walk_shape(const sc_plan *plan);

// Dynamic LDS bytes the fused / fissioned kernels of a plan need (used for validation).
size_t lds_bytes_needed(const sc_plan *plan);

// Argument checks of an execution followed by launch_plan (shared by the execute entry points).
sc_status execute_checked(const sc_plan *plan, const sc_csf_view *sparse, const sc_dense_view *factors, int32_t nfactors, void *out,
                          void *workspace, size_t workspace_bytes, hipStream_t stream);

// Device address of the library's fixed scratch array on the current device (static_scratch.hip).
void *static_scratch(sc_status *st);

sc_status launch_plan(const sc_plan *plan, const sc_csf_view *sp, const sc_dense_view *fac /*canonical order*/,
                      void *out, void *workspace, hipStream_t stream);

// Per-family pieces behind the three functions above (one kernel file each).
TileCaps order2_caps(sc_dtype dtype, const int64_t *fcols);
size_t order2_lds_bytes_needed(const sc_plan *plan);
// LINEAR schedule (kernels_linear.hip): the unfactored nest, every expression family.
size_t linear_lds_bytes(const sc_plan *plan);
sc_status launch_linear(const sc_plan *plan, const sc_csf_view *sp, const sc_dense_view *fac, void *out, hipStream_t stream);
sc_status launch_order2(const sc_plan *plan, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *workspace,
                        hipStream_t stream);
sc_status launch_ttmc_all(const sc_plan *plan, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *workspace,
                          hipStream_t stream);
sc_status launch_trailing_gemm(const sc_plan *plan, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *workspace,
                               hipStream_t stream);
TileCaps order4_caps(sc_dtype dtype, const int64_t *fcols);
size_t order4_lds_bytes_needed(const sc_plan *plan);
sc_status launch_order4(const sc_plan *plan, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *workspace,
                        hipStream_t stream);

}  // namespace sck
