// Leaf traversal of the FISSIONED schedules of order >= 3: the producer half of a split nest
// (Section 3.1, Algorithm 1 with nothing fused), materialising the temporary
//     T(f,:) = sum_{z in fiber f} vals[z] * F(crd[z],:)
// with one W-wide row per leaf fiber f (position-compressed along the sparse levels).
//
// The stage streams crd/vals once, gathers cached factor rows and writes T once, so it is
// bound by memory traffic.  What limits it in practice is the number of vector-memory
// instructions, not bytes: a lane group that stores its own 16..128-byte row whenever a
// fiber ends issues one mostly-masked store per step.  The kernel therefore collects the
// rows of a tile in LDS and writes them out at the end with full-width stores:
//
//   stage    one LDS record per nonzero {factor row offset | end-of-fiber bit, value}: the
//            coordinates come from the plan's walk tables with the end bits in them, and so does
//            the fiber at the head of every lane group's chunk; no fiber bounds are read and
//            nothing is marked at run time
//   walk     the shared branch-free leaf walk: a lane group of LG = W / VEC lanes owns a
//            contiguous chunk of nonzeros, keeps U gathers in flight and writes the running
//            sum to the current fiber's row of the LDS tile after every nonzero; chunk heads
//            are combined after a barrier without atomics
//   flush    rows leave LDS as contiguous 16-byte-per-lane stores; the (at most two) rows
//            shared with neighbouring tiles are added atomically to pre-zeroed memory
#include "leaf_walk.h"

namespace sck {

constexpr int LNT = 256;  // threads per workgroup of the traversal kernel

// 16-byte store with the non-temporal hint: rows of T are written once and not read by this kernel.
typedef unsigned int leaf_u32x4 __attribute__((ext_vector_type(4)));
template <typename T, typename PK>
__device__ __forceinline__ void nt_store16(T *dst, const PK &v)
{
    static_assert(sizeof(PK) == 16, "pack size");
    __builtin_nontemporal_store(__builtin_bit_cast(leaf_u32x4, v), reinterpret_cast<leaf_u32x4 *>(dst));
}

struct LeafArgs {
    const uint32_t *rec;     // the plan's walk table: last coordinate of every nonzero | end-of-fiber bit 31
    const uint16_t *heads;   // ... and per tile the chunk heads of the lane groups
    int32_t heads_per_tile;
    const void *vals;
    const void *F;
    int64_t ldF;
    void *Tout;
    void *partials;   // deterministic schedules: slots for the pieces of rows that span tiles, else null
    int32_t tn, ta;
    int32_t ntiles;
};

template <typename T>
__host__ __device__ constexpr size_t leaf_lds_bytes(int W, int tn, int ta)
{
    const int groups = LNT / (W / (16 / (int)sizeof(T)));
    return (size_t)(ta + 1 + groups) * leaf_row_stride<T>(W) * sizeof(T) + (size_t)padded(tn + 8) * sizeof(LeafRec<T>) + (size_t)groups * 4 + 64;
}

// Global reads of one tile's staging, held in registers until the tile's turn.
template <typename T>
struct LeafStage {
    static constexpr int MAXR = 4;   // tn <= MAXR * LNT
    uint32_t kk[MAXR];
    T vv[MAXR];
    uint32_t hd;
};

// Issues every global read of a tile's staging at once (clamped indices keep the redundant
// ones in bounds), so the staging costs one memory latency, not one per loop trip.
template <typename T>
__device__ __forceinline__ void leaf_issue(const LeafArgs &a, const TileRec &t, int tile, int groups, int tid, LeafStage<T> &s)
{
    const T *vals = static_cast<const T *>(a.vals);
    const int nchild = t.n1 - t.n0;
#pragma unroll
    for (int r = 0; r < LeafStage<T>::MAXR; ++r) {
        const int c = t.n0 + min(tid + r * LNT, nchild - 1);
        s.kk[r] = a.rec[c];
        s.vv[r] = vals[c];
    }
    s.hd = a.heads[(int64_t)tile * a.heads_per_tile + min(tid, groups - 1)];
}

// Workgroup b handles tiles b, b + gridDim.x, ... (the launch is persistent for wide rows and
// has one workgroup per tile for narrow ones).  While one tile is walked, the staging reads of
// the next are already in flight, and the row stores of the previous tile drain behind them.
// DET: the deterministic variant (the pieces of a row shared with a neighbouring tile go to the
// tile's slots instead of being added atomically).
template <typename T, int W, bool DET>
__global__ void __launch_bounds__(LNT) leaf_traverse_kernel(LeafArgs a, const TileRec *__restrict__ tiles)
{
    // `tiles` is a separate restrict-qualified argument so that the tile records stay scalar
    // loads inside the loop (nothing the kernel stores can alias them).
    constexpr int VEC = VecWidth<T>::value;
    constexpr int LG = W / VEC;
    constexpr int G = LNT / LG;
    constexpr int U = 4;   // as in leaf_traverse_walk_shape
    static_assert(W % VEC == 0 && (LG & (LG - 1)) == 0 && LG <= 64, "row width");
    using P = Pack<T, VEC>;
    using Rec = LeafRec<T>;
    using Stage = LeafStage<T>;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int RS = leaf_row_stride<T>(W);
    T *row_s = reinterpret_cast<T *>(smem);                                    // (ta + 1) rows of RS
    T *carry_s = row_s + (size_t)(a.ta + 1) * RS;                              // G rows of RS
    Rec *rec_s = reinterpret_cast<Rec *>(carry_s + (size_t)G * RS);            // padded(tn + 8)
    uint32_t *chunk_s = reinterpret_cast<uint32_t *>(rec_s + padded(a.tn + 8));   // G: chunk heads

    const int tid = threadIdx.x;
    const int g = tid / LG, li = tid % LG;
    const uint32_t rowF = (uint32_t)(a.ldF * sizeof(T));
    const int stride = gridDim.x, last = a.ntiles - 1;

    int nx = blockIdx.x + stride;                 // the launch has at most ntiles workgroups
    TileRec t = tiles[blockIdx.x];
    TileRec t1 = tiles[min(nx, last)];
    Stage st;
    leaf_issue(a, t, (int)blockIdx.x, G, tid, st);
    // First tile: wait here, so that the loop body itself never waits on staging registers
    // (a wait there would also wait for the previous tile's row stores): vmcnt(0).
    __builtin_amdgcn_s_waitcnt(0x0F70);

    for (;;) {
        const int nchild = t.n1 - t.n0;
        const int na = t.na;
        const int q = leaf_chunk<U>(nchild, G);   // nonzeros per lane group, multiple of U

        // ---- stage: registers -> LDS ----
#pragma unroll
        for (int r = 0; r < Stage::MAXR; ++r) {
            const int c = tid + r * LNT;
            if (c < nchild) {
                Rec rec;
                // the tile's last nonzero closes the fiber it is in as far as this tile goes
                rec.koff = (st.kk[r] & 0x7fffffffu) * rowF | (st.kk[r] & 0x80000000u) | (c == nchild - 1 ? 0x80000000u : 0u);
                rec.v = st.vv[r];
                rec_s[pidx(c)] = rec;
            }
        }
        if (tid < G) chunk_s[tid] = st.hd;
        if (tid < U) {  // dummies completing the last batch: value 0, row 0, no mark
            Rec rec;
            rec.koff = 0;
            rec.v = T(0);
            rec_s[pidx(nchild + tid)] = rec;
        }
        __syncthreads();

        // ---- reads of the next tile (and the record of the one after) go out now ----
        const bool more = nx < a.ntiles;
        Stage sn;
        if (more) leaf_issue(a, t1, nx, G, tid, sn);
        const TileRec t2 = tiles[min(nx + stride, last)];

        // ---- walk ----
        const uint32_t done = table_walk<T, W, U>(row_s, carry_s, rec_s, chunk_s, a.F, g, li, q, nchild);
        // The prefetched registers are complete here, before any store is queued behind
        // them (waits count loads and stores in issue order): vmcnt(0), other counters free.
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        table_combine<T, W>(row_s, carry_s, chunk_s, done, g, li);
        __syncthreads();

        // ---- flush ----
        T *Tout = static_cast<T *>(a.Tout) + (int64_t)t.a0 * W;
        // Rows that only this tile holds leave in batches: the LDS reads of a batch are issued
        // together, then its stores (no branch inside).  The at most two rows shared with a
        // neighbouring tile are handled after the loop.
        const bool sh0 = (t.flags & 1) != 0, sh1 = (t.flags & 2) != 0;
        constexpr int FB = 8;
        for (int r0 = g; r0 < na; r0 += FB * G) {
            P rows[FB];
#pragma unroll
            for (int k = 0; k < FB; ++k) rows[k] = *reinterpret_cast<const P *>(row_s + min(r0 + k * G, na - 1) * RS + li * VEC);
#pragma unroll
            for (int k = 0; k < FB; ++k) {
                const int r = r0 + k * G;
                if (r < na && !(r == 0 && sh0) && !(r == na - 1 && sh1)) nt_store16(Tout + (int64_t)r * W + li * VEC, rows[k]);
            }
        }
        {
            // first row (continues from the previous tile) by lane group 0, last row (continues
            // into the next tile) by the lane group that would have stored it
            const bool first = sh0 && g == 0;
            const bool last = sh1 && !(sh0 && na == 1) && g == (na - 1) % G;
            if (first || last) {
                const int r = first ? 0 : na - 1;
                // a group can hold both roles only when they are different rows: do them in turn
                for (int pass = 0; pass < 2; ++pass) {
                    const int rr = pass == 0 ? r : na - 1;
                    if (pass == 1 && !(first && last)) break;
                    const P row = *reinterpret_cast<const P *>(row_s + rr * RS + li * VEC);
                    T *dst = Tout + (int64_t)rr * W + li * VEC;
                    if (DET) {
                        // the piece of the tile's first fiber is numbered pad[2], that of its last fiber follows
                        const int slot = t.pad[2] + ((rr == 0 && sh0) ? 0 : (sh0 ? 1 : 0));
                        *reinterpret_cast<P *>(static_cast<T *>(a.partials) + (int64_t)slot * W + li * VEC) = row;
                    } else {
#pragma unroll
                        for (int i = 0; i < VEC; ++i) atomic_add(dst + i, row.v[i]);
                    }
                }
            }
        }
        if (!more) break;
        t = t1;
        t1 = t2;
        st = sn;
        nx += stride;
    }
}

namespace {
template <typename T, int W>
sc_status leaf_traverse(const sc_plan *p, Launcher &ln, const void *vals, const sc_dense_view &F, void *Tout, void *partials, const char *name)
{
    const int ntiles = (int)p->tiles.size();
    if (ntiles == 0) return SC_OK;
    // factor rows are addressed with 31-bit byte offsets (bit 31 marks fiber ends)
    if ((uint64_t)F.rows * (uint64_t)F.ld * sizeof(T) >= (1ull << 31)) return SC_ERR_SHAPE_MISMATCH;
    if (p->caps.tn > LeafStage<float>::MAXR * LNT || p->caps.ta > (int)kChunkRow) return SC_ERR_SCHED_UNSUPPORTED;   // staging registers, row numbers of the chunk heads
    // the plan's walk tables must have been made for this kernel's lane groups
    const WalkShape want = leaf_traverse_walk_shape(p->dtype, W);
    const WalkTables &wt = p->walk;
    if (!wt.d_rec[0] || !wt.d_heads || wt.shape.groups[0] != want.groups[0] || wt.shape.batch[0] != want.batch[0]) return SC_ERR_SCHED_UNSUPPORTED;
    LeafArgs a = {};
    a.rec = wt.d_rec[0]; a.heads = wt.d_heads; a.heads_per_tile = wt.heads_per_tile;
    a.vals = vals;
    a.F = F.data;
    a.ldF = F.ld;
    a.Tout = Tout;
    a.partials = partials;
    a.tn = p->caps.tn; a.ta = p->caps.ta;
    if (!partials) {   // rows shared between tiles are added atomically: they start from zero
        ln.begin("zero_shared_rows");
        zero_shared_rows_kernel<T><<<(ntiles + 3) / 4, NT, 0, ln.stream>>>(p->d_tiles, ntiles, 0, static_cast<T *>(Tout), W);
        ln.end();
    }
    ln.begin(name);
    // Wide rows (LDS lets at most three workgroups reside on a compute unit): persistent launch, as
    // many workgroups as fit on the chip at once, each looping over tiles.  Narrow rows: one
    // workgroup per tile, which lets the dispatcher even out tiles of different cost (measured 5 to
    // 9 % faster on the order-3 chain with 16-wide rows and the order-4 chain with 8-wide rows, 10 %
    // slower on the 32-wide rows of the MTTKRP).
    a.ntiles = ntiles;
    const size_t lds = leaf_lds_bytes<T>(W, a.tn, a.ta);
    const int fit = lds_workgroups_per_cu(lds, p->lds_per_cu);
    const int per_cu = p->tune.per_cu > 0 ? std::min(p->tune.per_cu, 16) : fit;
    const int blocks = (p->tune.per_cu == 0 && fit > 3) ? ntiles : std::min(ntiles, p->n_cu * per_cu);
    if (partials)
        leaf_traverse_kernel<T, W, true><<<blocks, LNT, lds, ln.stream>>>(a, p->d_tiles);
    else
        leaf_traverse_kernel<T, W, false><<<blocks, LNT, lds, ln.stream>>>(a, p->d_tiles);
    ln.end();
    return ln.status;
}
}  // namespace

size_t leaf_traverse_lds_bytes(const sc_plan *p, int W)
{
    if (p->caps.tn > LeafStage<float>::MAXR * LNT || p->caps.ta > (int)kChunkRow) return SIZE_MAX;   // staging registers, row numbers of the chunk heads
    return p->dtype == SC_F64 ? leaf_lds_bytes<double>(W, p->caps.tn, p->caps.ta) : leaf_lds_bytes<float>(W, p->caps.tn, p->caps.ta);
}

WalkShape leaf_traverse_walk_shape(sc_dtype dtype, int W)
{
    WalkShape w;
    const int vec = dtype == SC_F64 ? 2 : 4;   // elements per 16-byte lane
    if (W < vec || W % vec) return w;
    w.levels = 1;
    w.groups[0] = LNT / (W / vec);
    w.batch[0] = 4;   // U of the kernel
    return w;
}

sc_status launch_leaf_producer(const sc_plan *p, Launcher &ln, const void *vals, const sc_dense_view &F, void *Tout, int W, const char *name,
                               void *partials)
{
    const bool f64 = p->dtype == SC_F64;
#define SC_LEAF(WW)                                                                                   \
    case WW:                                                                                          \
        return f64 ? leaf_traverse<double, WW>(p, ln, vals, F, Tout, partials, name) \
                   : leaf_traverse<float, WW>(p, ln, vals, F, Tout, partials, name);
    switch (W) {
        SC_LEAF(8)
        SC_LEAF(16)
        SC_LEAF(32)
        SC_LEAF(64)
        SC_LEAF(128)
    default: return SC_ERR_SCHED_UNSUPPORTED;
    }
#undef SC_LEAF
}

}  // namespace sck
