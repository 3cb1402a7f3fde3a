// HIP kernels of libsparsecontract for gfx950 (CDNA4, 64-wide wavefronts).
//
// Every kernel works on one "tile": a contiguous run of stored nonzeros (CSF leaves)
// together with the CSF nodes above them (plan.h, TileRec).  Tiles are cut at plan time so
// that each holds about the same number of nonzeros whatever the slice / fiber lengths;
// heavy slices and fibers are therefore split across workgroups, and the pieces are
// recombined at the end (inside a workgroup: parked in LDS and added by one owner in a fixed
// order; between workgroups: atomic adds on pre-zeroed output rows, or plan-numbered slots
// added by a last kernel under a deterministic schedule).
//
// Inside a tile the nests of Table 2 run as a chain of segmented reductions, one per CSF
// level, each of the form
//     out(parent, :) = sum over children c of parent:  f( in(c, :), Factor(crd[c], :) )
// A "lane group" of LG = W / VEC adjacent lanes owns VEC consecutive elements of the
// W-wide row; a workgroup holds G = 256 / LG lane groups and each walks a contiguous chunk
// of the tile's children, keeping the running sum of the current parent in registers and
// flushing it when the walk crosses a parent boundary.  Coordinates, values and boundary
// positions are staged into LDS with coalesced loads first.
//
// Because every stage is linear in its input, a node that is cut by a chunk or tile
// boundary is simply treated as two nodes: each piece is pushed through the consumer
// separately and only the final output rows need recombining.
#include "leaf_walk.h"

namespace sck {

// ------------------------------------------------------------------------------------------
// Order-3 kernels:  T(f, x) = sum_{k' in fiber f} B * D(k, x)   then
//   hadamard:  A(i, r)    += C(j, r) * T(f, r)                      (MTTKRP)
//   outer:     A(i, l, m) += C(j, l) * T(f, m)                      (kernel 6 of Table 2)
// The MTTKRP and the fp32 16 x 16 outer product have kernels of their own (below and in
// kernels_ttmc3.hip); order3_kernel is the general outer-product kernel for every other rank
// and for fp64:
//   MODE 0: fused (T lives in LDS for the tile)      -- FUSED schedule
//   MODE 2: consumer only, T read back from HBM      -- FISSIONED, second kernel (the first is
//           the leaf traversal of kernels_traverse.hip)
// Its producer is the shared leaf walk (leaf_walk.h); its consumer gives every thread a set of
// output elements (l, m) and lets it run over the tile's slices and fibers in order: one
// global update per tile, slice and element, an atomic add (or, under a deterministic
// schedule, a store to the tile's slot) if the slice is shared with another tile.
// ------------------------------------------------------------------------------------------
struct Order3Args {
    const TileRec *tiles;
    const int32_t *crd1, *pos2, *crd2, *pos3, *crd3;
    const void *vals;
    const void *C;  // factor on mode 1 (rows = J)
    const void *D;  // factor on mode 2 (rows = K)
    int64_t ldC, ldD;
    int32_t L;      // columns of C (outer only)
    void *T;        // temporary rows (the traversal kernel writes them, the consumers read them)
    void *A;
    void *partials; // deterministic schedules: slots for the pieces of rows that span tiles, else null
    int32_t tn, ta, tb;  // caps used to carve LDS
};

// `crow_l`: columns of C when the consumer runs on the matrix cores (it then keeps the tile's C rows in LDS), else 0
template <typename T>
__host__ __device__ constexpr size_t order3_lds_bytes(int W, int tn, int ta, int crow_l = 0)
{
    return leaf_walk_lds_bytes<T>(W, tn, ta, NT) + (size_t)(3 * ta + 8) * 4 + 64 + (crow_l ? (size_t)ta * (crow_l + 4) * 4 + 16 : 0);
}

// fp32 outer products whose ranks are multiples of the 16 x 16 MFMA tile (other than the 16 x 16 case, which has a
// kernel of its own) run the consumer of order3_kernel on the matrix cores.
__host__ __device__ constexpr bool order3_mfma_ranks(int L, int W)
{
    return W % 16 == 0 && (L == 16 || L == 32 || L == 64 || L == 128) && !(L == 16 && W == 16);
}

typedef float o3_floatx4 __attribute__((ext_vector_type(4)));

template <typename T, int W, int MODE, bool MF = false>
__global__ void __launch_bounds__(NT) order3_kernel(Order3Args a)
{
    constexpr int VEC = VecWidth<T>::value;
    constexpr int LG = W / VEC;   // lanes per row
    constexpr int G = NT / LG;    // lane groups per workgroup
    constexpr int U = 4;          // gathers in flight per lane
    constexpr int RS = leaf_row_stride<T>(W);
    static_assert(W % VEC == 0 && (LG & (LG - 1)) == 0 && LG <= 64, "row width");
    using P = Pack<T, VEC>;
    using Rec = LeafRec<T>;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    T *row_s = reinterpret_cast<T *>(smem);                                    // (ta + 1) rows of RS: T
    T *carry_s = row_s + (size_t)(a.ta + 1) * RS;                              // G rows of RS
    Rec *rec_s = reinterpret_cast<Rec *>(carry_s + (size_t)G * RS);            // padded(tn + 8)
    int *ba_s = reinterpret_cast<int *>(rec_s + padded(a.tn + 8));             // ta + 2: first nonzero of each fiber (tile-local)
    int *chunk_lr = ba_s + a.ta + 2;                                           // G
    int *crda_s = chunk_lr + G;          // ta: j of each fiber
    int *bb_s = crda_s + a.ta;           // ta + 2: first fiber of each slice (tile-local)
    int *crdb_s = bb_s + a.ta + 2;       // ta: output row of each slice
    // MF: C rows of the tile's fibers, ta rows of L + 4 floats (16-byte aligned)
    float *crow_s = reinterpret_cast<float *>(smem + ((order3_lds_bytes<T>(W, a.tn, a.ta) + 15) & ~(size_t)15));

    const TileRec t = a.tiles[blockIdx.x];
    const int tid = threadIdx.x;
    const int nchild = t.n1 - t.n0;
    const int na = t.na, nb = t.nb;
    const int g = tid / LG, li = tid % LG;
    const int q = leaf_chunk<U>(nchild, G);

    // ---- stage ----
    if (MODE == 0) {
        const T *vals = static_cast<const T *>(a.vals);
        const uint32_t rowD = (uint32_t)(a.ldD * sizeof(T));
        for (int c = tid; c < nchild; c += NT) {
            Rec rec;
            rec.koff = (uint32_t)a.crd3[t.n0 + c] * rowD;
            rec.v = vals[t.n0 + c];
            rec_s[pidx(c)] = rec;
        }
        if (tid < U) {  // dummies completing the last batch: value 0, row 0, no mark
            Rec rec;
            rec.koff = 0;
            rec.v = T(0);
            rec_s[pidx(nchild + tid)] = rec;
        }
        for (int i = tid; i <= na; i += NT) ba_s[i] = min(max(a.pos3[t.a0 + i], t.n0), t.n1) - t.n0;
    } else {
        // A fiber cut by a tile boundary has one complete row in the workspace; the tile in which
        // it starts consumes it, the tiles it continues into skip it (cf0 below).
        const T *Tg = static_cast<const T *>(a.T) + (int64_t)t.a0 * W;
        for (int r = g; r < na; r += G)
            *reinterpret_cast<P *>(row_s + r * RS + li * VEC) = *reinterpret_cast<const P *>(Tg + (int64_t)r * W + li * VEC);
    }
    for (int i = tid; i < na; i += NT) crda_s[i] = a.crd2[t.a0 + i];
    for (int i = tid; i <= nb; i += NT) bb_s[i] = min(max(a.pos2[t.b0 + i], t.a0), t.a0 + na) - t.a0;
    for (int i = tid; i < nb; i += NT) crdb_s[i] = a.crd1[t.b0 + i];
    __syncthreads();

    if constexpr (MF) {
        // C rows -> LDS, 16 bytes per lane, consecutive lanes on consecutive pieces of a row
        const int LS = a.L + 4, vpr = a.L / 4;
        const int sh = vpr == 4 ? 2 : vpr == 8 ? 3 : vpr == 16 ? 4 : 5;
        const float *Cg = static_cast<const float *>(a.C);
#pragma unroll 4
        for (int idx = tid; idx < (na << sh); idx += NT) {
            const int f = idx >> sh, q4 = (idx & (vpr - 1)) * 4;
            *reinterpret_cast<o3_floatx4 *>(crow_s + f * LS + q4) = *reinterpret_cast<const o3_floatx4 *>(Cg + (int64_t)crda_s[f] * a.ldC + q4);
        }
    }

    // ---- producer: the shared leaf walk, leaves -> rows of T in LDS ----
    if (MODE == 0) {
        leaf_mark(rec_s, ba_s, chunk_lr, tid, NT, na, q);
        __syncthreads();
        const LeafCarry st = leaf_walk<T, W, U>(row_s, carry_s, rec_s, ba_s, chunk_lr, a.D, g, li, q, nchild);
        __syncthreads();
        leaf_combine<T, W>(row_s, carry_s, ba_s, chunk_lr, st, g, li, q);
        __syncthreads();
    }

    // ---- consumer: rows of T -> A.  Every thread owns output elements (l, m) and runs over the
    // tile's slices and fibers in order: one update per tile, slice and element. ----
    const int cf0 = (MODE == 2 && (t.flags & 1)) ? 1 : 0;
    const T *C = static_cast<const T *>(a.C);
    T *A = static_cast<T *>(a.A);
    const int L = a.L;
    if constexpr (MF) {
        // Matrix cores: A(i, l, m) = sum_f C(j_f, l) * T(f, m) per slice is an (L x Kf) * (Kf x W) product.  A
        // wavefront owns output tiles of 16 (l) x 16 (m) for every slice of the work tile, so no sums cross
        // wavefronts; four fibers per v_mfma_f32_16x16x4_f32, operand A = T (m along the rows), operand B = the
        // C rows (l along the columns), both read from LDS; a lane ends up with four consecutive m of one l.
        if (MODE != 0) __syncthreads();   // (the fused path has passed a barrier since the C rows were written)
        const int lane = tid % 64, wave = tid / 64;
        const int kk = lane / 16, col = lane % 16;
        const int LS = L + 4;
        constexpr int NTM = W / 16;
        const int ntile = (L / 16) * NTM;
        float *Af = reinterpret_cast<float *>(A);
        for (int ot = wave; ot < ntile; ot += NT / 64) {
            const int lt = ot / NTM, mt = ot % NTM;
            for (int ls = 0; ls < nb; ++ls) {
                const int f0 = max(bb_s[ls], ls == 0 ? cf0 : 0), f1 = bb_s[ls + 1];
                const bool first_shared = ls == 0 && (t.flags & 4), last_shared = ls == nb - 1 && (t.flags & 8);
                if (f0 >= f1 && !(a.partials && (first_shared || last_shared))) continue;
                o3_floatx4 acc = {0.f, 0.f, 0.f, 0.f};
                for (int fb = f0; fb < f1; fb += 4) {
                    const int lf = fb + kk;
                    const int lfc = min(lf, f1 - 1);   // lanes past the slice read a valid fiber and are zeroed
                    const float tvr = reinterpret_cast<const float *>(row_s)[lfc * RS + mt * 16 + col];
                    const float cv = crow_s[lfc * LS + lt * 16 + col];
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(lf < f1 ? tvr : 0.f, cv, acc, 0, 0, 0);
                }
                // acc[r] = A(l = 16 lt + col, m = 16 mt + 4 kk + r)
                const int64_t eoff = (int64_t)(lt * 16 + col) * W + mt * 16 + 4 * kk;
                if (!first_shared && !last_shared) {
                    *reinterpret_cast<o3_floatx4 *>(Af + (int64_t)crdb_s[ls] * L * W + eoff) = acc;
                } else if (a.partials) {
                    *reinterpret_cast<o3_floatx4 *>(static_cast<float *>(a.partials) + (int64_t)(first_shared ? t.pad[0] : t.pad[1]) * L * W + eoff) = acc;
                } else {
                    float *dst = Af + (int64_t)crdb_s[ls] * L * W + eoff;
#pragma unroll
                    for (int r = 0; r < 4; ++r) atomic_add(dst + r, acc[r]);
                }
            }
        }
        return;
    }
    for (int e = tid; e < L * W; e += NT) {
        const int l = e / W, m = e % W;
        for (int ls = 0; ls < nb; ++ls) {
            const int f0 = max(bb_s[ls], ls == 0 ? cf0 : 0), f1 = bb_s[ls + 1];
            const bool first_shared = ls == 0 && (t.flags & 4), last_shared = ls == nb - 1 && (t.flags & 8);
            // nothing of this slice is consumed here (only the fiber that an earlier tile owns): no
            // update, except that a deterministic schedule still expects the tile's (zero) piece
            if (f0 >= f1 && !(a.partials && (first_shared || last_shared))) continue;
            T acc = T(0);
            for (int lf = f0; lf < f1; ++lf) acc += C[(int64_t)crda_s[lf] * a.ldC + l] * row_s[lf * RS + m];
            T *dst = A + (int64_t)crdb_s[ls] * L * W + e;
            if (!first_shared && !last_shared) {
                *dst = acc;
            } else if (a.partials) {
                // deterministic: the tile's piece of this row goes to its slot (a tile whose only
                // slice continues on both sides has one piece, numbered as its first)
                static_cast<T *>(a.partials)[(int64_t)(first_shared ? t.pad[0] : t.pad[1]) * L * W + e] = acc;
            } else {
                atomic_add(dst, acc);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// MTTKRP, FUSED at fiber granularity: one walk over the nonzeros keeps the fiber sum T(r)
// and the slice sum A(i, r) in registers (Table 2, kernel 8 producer: t += B * D, then
// A += t * C at the end of each fiber).
//
// Staging turns the tile's CSF arrays into per-nonzero LDS arrays (read four nonzeros at a time):
//   koff  byte offset of the D row to gather
//   v     the stored value
//   e     byte offset of the C row if this nonzero is the last of its fiber (in the tile), else -1
//   send  one bit: this nonzero is the last of its slice (in the tile)
// so the walk needs no boundary cursors or searches: a lane group reads these per
// nonzero, gathers D (and C when e >= 0, in the same batch of loads) and updates two
// register accumulators; the slice it is in is a counter that starts from chunk_ls0.
// Fibers / slices cut by a chunk boundary are described by small per-group tables
// (chunk_coff, chunk_ls) filled during staging.  12 bytes of LDS per nonzero (fp32) let
// eight workgroups share a compute unit; the walk is bound by gather latency, and the
// kernel's time fell almost in proportion as the workgroups per unit went from 4 to 7.
// ------------------------------------------------------------------------------------------
// LDS index of nonzero c in the per-nonzero arrays: groups of four stay contiguous and
// 16-byte aligned, and one group of padding after every eight spreads the lane groups of a
// wavefront (whose chunks start a multiple of 32 nonzeros apart) over the banks.
__host__ __device__ constexpr int nz_vec(int c4) { return c4 + (c4 >> 3); }           // c4 = c / 4
__host__ __device__ constexpr int nz_idx(int c) { return 4 * nz_vec(c >> 2) + (c & 3); }
__host__ __device__ constexpr int nz_padded(int n) { return 4 * (nz_vec((n + 3) >> 2) + 1); }

// W = rank; a lane group is W / (16 / sizeof(T)) lanes, and there is one parked row and one
// entry of each chunk table per lane group.
template <typename T>
__host__ __device__ constexpr size_t mttkrp_lds_bytes(int W, int tn, int ta, int tb)
{
    const int groups = NT / (W / (16 / (int)sizeof(T)));
    const int pn = nz_padded(tn + 8);
    return (size_t)NT * 16 + (size_t)pn * (sizeof(T) + 8) + (size_t)((tn + 8 + 31) / 32 + 1) * 4 + (size_t)(2 * tb + 4 * groups) * 4 + 64;
}

// DET: the deterministic variant (pieces of rows that span tiles go to plan-numbered slots).  A
// separate instantiation, so that the atomic variant keeps its 64 registers (8 waves per SIMD).
template <typename T, int W, bool DET>
__global__ void __launch_bounds__(NT) mttkrp3_fused_kernel(Order3Args a)
{
    constexpr int VEC = VecWidth<T>::value;
    constexpr int LG = W / VEC;
    constexpr int G = NT / LG;
    using P = Pack<T, VEC>;
    using Acc = AccVec<T, VEC>;
    struct alignas(16) Val4 { T v[4]; };
    struct alignas(16) Int4 { int32_t v[4]; };

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int pn = nz_padded(a.tn + 8);
    T *slot_s = reinterpret_cast<T *>(smem);                       // NT * VEC: one parked row per lane group
    T *v_s = slot_s + NT * VEC;                                    // pn: stored values
    uint32_t *koff_s = reinterpret_cast<uint32_t *>(v_s + pn);     // pn: byte offset of the D row
    int32_t *e_s = reinterpret_cast<int32_t *>(koff_s + pn);       // pn: byte offset of the C row at a fiber end, else -1
    uint32_t *send_s = reinterpret_cast<uint32_t *>(e_s + pn);     // one bit per nonzero: last of its slice
    const int nsend = (a.tn + 8 + 31) / 32 + 1;
    int *slo_s = reinterpret_cast<int *>(send_s + nsend);          // tb: first nonzero of each slice
    int *crdb_s = slo_s + a.tb;                                    // tb: output row of each slice
    int *chunk_coff = crdb_s + a.tb;                               // G: C row of the fiber a chunk ends inside, else -1
    int *chunk_ls = chunk_coff + G;                                // G: slice a chunk ends inside, else -1
    int *chunk_ls0 = chunk_ls + G;                                 // G: slice holding the first nonzero of a chunk
    int *slot_id = chunk_ls0 + G;                                  // G

    const TileRec t = a.tiles[blockIdx.x];
    const int tid = threadIdx.x;
    const int nchild = t.n1 - t.n0;
    const int na = t.na, nb = t.nb;
    constexpr int U = 4;                          // gathers kept in flight per lane = nonzeros per LDS read
    const int q = max(((nchild + G - 1) / G + U - 1) / U * U, U);   // nonzeros per lane group, multiple of U
    const uint32_t rowD = (uint32_t)(a.ldD * sizeof(T)), rowC = (uint32_t)(a.ldC * sizeof(T));

    // ---- stage 1: per-nonzero arrays, per-fiber and per-slice ranges (kept in registers) ----
    {
        const T *vals = static_cast<const T *>(a.vals);
        for (int c = tid; c < nchild; c += NT) {
            const int p = nz_idx(c);
            koff_s[p] = (uint32_t)a.crd3[t.n0 + c] * rowD;
            v_s[p] = vals[t.n0 + c];
            e_s[p] = -1;
        }
        if (tid < U) {  // dummies that complete the last batch: value 0, row 0, no marks
            const int p = nz_idx(nchild + tid);
            koff_s[p] = 0;
            v_s[p] = T(0);
            e_s[p] = -1;
        }
        if (tid < nsend) send_s[tid] = 0;
        P z;
#pragma unroll
        for (int i = 0; i < VEC; ++i) z.v[i] = T(0);
        reinterpret_cast<P *>(slot_s)[tid] = z;
        if (tid < G) {
            slot_id[tid] = -1;
            chunk_coff[tid] = -1;
            chunk_ls[tid] = -1;
        }
    }
    constexpr int MAXF = 2;  // fibers per thread: ta <= MAXF * NT
    int f_lo[MAXF], f_hi[MAXF];
    uint32_t f_off[MAXF];
#pragma unroll
    for (int r = 0; r < MAXF; ++r) {
        const int i = tid + r * NT;
        f_lo[r] = f_hi[r] = 0;
        f_off[r] = 0;
        if (i < na) {
            f_lo[r] = min(max(a.pos3[t.a0 + i], t.n0), t.n1) - t.n0;
            f_hi[r] = min(max(a.pos3[t.a0 + i + 1], t.n0), t.n1) - t.n0;
            f_off[r] = (uint32_t)a.crd2[t.a0 + i] * rowC;
        }
    }
    int s_lo = 0, s_hi = 0;
    if (tid < nb) {
        const int flo = min(max(a.pos2[t.b0 + tid], t.a0), t.a0 + na);
        const int fhi = min(max(a.pos2[t.b0 + tid + 1], t.a0), t.a0 + na);
        s_lo = min(max(a.pos3[flo], t.n0), t.n1) - t.n0;
        s_hi = min(max(a.pos3[fhi], t.n0), t.n1) - t.n0;
        slo_s[tid] = s_lo;
        crdb_s[tid] = a.crd1[t.b0 + tid];
    }
    __syncthreads();

    // ---- stage 2: mark fiber ends, slice ends and the nodes cut by chunk boundaries ----
#pragma unroll
    for (int r = 0; r < MAXF; ++r)
        if (f_hi[r] > f_lo[r]) {
            e_s[nz_idx(f_hi[r] - 1)] = (int32_t)f_off[r];
            for (int m = f_lo[r] / q + 1; m * q < f_hi[r]; ++m) chunk_coff[m - 1] = (int32_t)f_off[r];
        }
    if (s_hi > s_lo) {
        atomicOr(&send_s[(s_hi - 1) >> 5], 1u << ((s_hi - 1) & 31));
        for (int m = (s_lo + q - 1) / q; m * q < s_hi; ++m) {
            chunk_ls0[m] = tid;
            if (m * q > s_lo) chunk_ls[m - 1] = tid;
        }
    }
    __syncthreads();

    const int g = tid / LG, li = tid % LG;
    // uniform base + 32-bit per-lane byte offset: one address add per gather
    const char *Cb = static_cast<const char *>(a.C);
    const char *Db = static_cast<const char *>(a.D);
    const uint32_t lo = (uint32_t)li * 16u;
    T *A = static_cast<T *>(a.A);
    auto slice_shared = [&](int ls) { return (ls == 0 && (t.flags & 4)) || (ls == nb - 1 && (t.flags & 8)); };
    auto direct = [&](int ls, const P &row) {
        T *dst = A + (int64_t)crdb_s[ls] * W + li * VEC;
        if (!slice_shared(ls)) {
            *reinterpret_cast<P *>(dst) = row;
        } else if (DET) {
            // deterministic: the tile's one piece of this row goes to its slot (a tile whose only
            // slice continues on both sides has one piece, numbered as its first)
            const int slot = (ls == 0 && (t.flags & 4)) ? t.pad[0] : t.pad[1];
            *reinterpret_cast<P *>(static_cast<T *>(a.partials) + (int64_t)slot * W + li * VEC) = row;
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) atomic_add(dst + i, row.v[i]);
        }
    };

    // A lane group whose chunk starts inside a slice keeps that slice's piece ("head") in
    // registers when the slice ends; a chunk that ends inside a slice parks its running sum
    // ("tail") in its LDS row together with a flag telling whether the slice began in this
    // chunk.  After the barrier the group holding a head adds the tails of the chunks before
    // it, back to the one in which the slice began, and issues the tile's single update of
    // that output row.  (LDS float atomics for this measured about a quarter of the kernel.)
    const int gs = g * q, ge = min(gs + q, nchild);
    int head_ls = -1;
    P headv;
#pragma unroll
    for (int i = 0; i < VEC; ++i) headv.v[i] = T(0);
    if (gs < ge) {
        int ls = chunk_ls0[g];                     // slice of the nonzero the walk is at
        bool started = slo_s[ls] == gs;            // the current slice starts in this chunk
        Acc tsum, asum;
        tsum.clear();
        asum.clear();
        auto emit = [&](int s, bool whole) {
            P o;
#pragma unroll
            for (int i = 0; i < VEC; ++i) o.v[i] = asum.v[i];
            if (whole) {
                direct(s, o);
            } else {
                headv = o;
                head_ls = s;
            }
        };
        // Chunks start at multiples of U and the entries up to the next multiple of U past
        // the tile's last nonzero are zero-valued dummies, so every batch is a full,
        // branch-free group of U gathers (the compiler can then keep all of them in flight).
        for (int c = gs; c < ge; c += U) {
            const int pv = nz_vec(c >> 2);
            const Int4 kk = reinterpret_cast<const Int4 *>(koff_s)[pv];
            const Val4 vv = reinterpret_cast<const Val4 *>(v_s)[pv];
            const Int4 ee = reinterpret_cast<const Int4 *>(e_s)[pv];
            const uint32_t sbits = send_s[c >> 5] >> (c & 31);   // the batch's four bits share a word
            P d[U], cc[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                d[u] = *reinterpret_cast<const P *>(Db + ((uint32_t)kk.v[u] + lo));
                if (ee.v[u] >= 0) cc[u] = *reinterpret_cast<const P *>(Cb + ((uint32_t)ee.v[u] + lo));   // read only where loaded
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) tsum.v[i] += vv.v[u] * d[u].v[i];
                if (ee.v[u] >= 0) {   // the fiber ends here: through the consumer, under the lane mask
#pragma unroll
                    for (int i = 0; i < VEC; ++i) {
                        asum.v[i] += tsum.v[i] * cc[u].v[i];
                        tsum.v[i] = T(0);
                    }
                    if ((sbits >> u) & 1u) {   // a slice can only end where a fiber ends
                        emit(ls, started);
                        asum.clear();
                        started = true;
                        ++ls;
                    }
                }
            }
        }
        const int co = chunk_coff[g];
        if (co >= 0) {  // the chunk ends inside a fiber: push its piece through the consumer
            const P cl = *reinterpret_cast<const P *>(Cb + ((uint32_t)co + lo));
#pragma unroll
            for (int i = 0; i < VEC; ++i) asum.v[i] += tsum.v[i] * cl.v[i];
        }
        if (chunk_ls[g] >= 0) {  // ... and inside a slice: park the tail
            P o;
#pragma unroll
            for (int i = 0; i < VEC; ++i) o.v[i] = asum.v[i];
            *reinterpret_cast<P *>(slot_s + g * W + li * VEC) = o;
            if (li == 0) slot_id[g] = started ? 1 : 0;
        }
    }
    __syncthreads();
    if (head_ls >= 0) {
        for (int h = g - 1; h >= 0; --h) {
            const P tl = *reinterpret_cast<const P *>(slot_s + h * W + li * VEC);
#pragma unroll
            for (int i = 0; i < VEC; ++i) headv.v[i] += tl.v[i];
            if (slot_id[h] != 0) break;   // the slice began in chunk h
        }
        direct(head_ls, headv);
    }
}

// ------------------------------------------------------------------------------------------
// MTTKRP, FISSIONED, second kernel: A(i, r) = sum_{fibers f of slice i} C(j_f, r) * T(f, r) with T
// read back from the workspace (the consumer of the split nest, Section 3.1).  The same walk
// as the fused kernel one level up: the children are the tile's fibers (their T rows are
// contiguous in memory, 16 bytes per lane), the parents its slices.  One 8-byte LDS record
// per fiber {C row offset, slice id at slice end}; slice pieces cut by chunk boundaries are
// parked and summed by the group where the slice ends.  A fiber that continues from the
// previous tile belongs to the tile it starts in and is skipped here.
// ------------------------------------------------------------------------------------------
struct FibRec {
    uint32_t coff;
    int32_t s;
};

template <typename T>
__host__ __device__ constexpr size_t hadamard_lds_bytes(int ta, int tb)
{
    return (size_t)NT * 16 + (size_t)padded(ta + 8) * sizeof(FibRec) + (size_t)(2 * tb + 2 * (NT / 2)) * 4 + 64;
}

template <typename T, int W, bool DET>
__global__ void __launch_bounds__(NT) hadamard_consume_kernel(Order3Args a)
{
    constexpr int VEC = VecWidth<T>::value;
    constexpr int LG = W / VEC;
    constexpr int G = NT / LG;
    constexpr int GMAX = NT / 2;
    constexpr int U = 4;
    static_assert(G <= GMAX, "lane group count");
    using P = Pack<T, VEC>;
    using Acc = AccVec<T, VEC>;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    T *slot_s = reinterpret_cast<T *>(smem);                                   // NT * VEC: one parked row per lane group
    FibRec *rec_s = reinterpret_cast<FibRec *>(slot_s + NT * VEC);             // padded(ta + 8)
    int *slo_s = reinterpret_cast<int *>(rec_s + padded(a.ta + 8));            // tb: first fiber of each slice
    int *crdb_s = slo_s + a.tb;                                                // tb: output row of each slice
    int *chunk_ls = crdb_s + a.tb;                                             // GMAX
    int *slot_id = chunk_ls + GMAX;                                            // GMAX

    const TileRec t = a.tiles[blockIdx.x];
    const int tid = threadIdx.x;
    const int cf0 = (t.flags & 1) ? 1 : 0;
    const int na = t.na, nb = t.nb;
    const int nfib = na - cf0;                    // fibers this tile consumes; may be 0
    const int q = max(((nfib + G - 1) / G + U - 1) / U * U, U);
    const uint32_t rowC = (uint32_t)(a.ldC * sizeof(T));

    // ---- stage: every global read before the first use ----
    {
        constexpr int MAXF = 2;   // ta <= MAXF * NT
        int cj[MAXF];
#pragma unroll
        for (int r = 0; r < MAXF; ++r) cj[r] = a.crd2[t.a0 + min(cf0 + tid + r * NT, na - 1)];
        const int sb = t.b0 + min(tid, nb - 1);
        const int p_lo = a.pos2[sb], p_hi = a.pos2[sb + 1], ci = a.crd1[sb];
#pragma unroll
        for (int r = 0; r < MAXF; ++r) {
            const int f = tid + r * NT;
            if (f < nfib + U) {   // the records past the last fiber complete the last batch: row 0 of C, no mark
                FibRec rec;
                rec.coff = f < nfib ? (uint32_t)cj[r] * rowC : 0u;
                rec.s = -1;
                rec_s[pidx(f)] = rec;
            }
        }
        if (tid < GMAX) {
            slot_id[tid] = -1;
            chunk_ls[tid] = -1;
        }
        int s_lo = 0, s_hi = 0;
        if (tid < nb) {
            s_lo = max(min(max(p_lo, t.a0), t.a0 + na) - t.a0, cf0) - cf0;
            s_hi = max(min(max(p_hi, t.a0), t.a0 + na) - t.a0, cf0) - cf0;
            slo_s[tid] = s_lo;
            crdb_s[tid] = ci;
        }
        __syncthreads();
        if (s_hi > s_lo) {
            rec_s[pidx(s_hi - 1)].s = tid;
            for (int m = s_lo / q + 1; m * q < s_hi; ++m) chunk_ls[m - 1] = tid;
        }
        if (DET && tid < nb && s_hi == s_lo) {
            // Nothing of this slice is consumed here (its only fiber in the tile belongs to an earlier
            // tile), so the walk emits nothing for it; the plan still counts a piece of this tile.
            const bool first_shared = tid == 0 && (t.flags & 4), last_shared = tid == nb - 1 && (t.flags & 8);
            if (first_shared || last_shared) {
                T *slot = static_cast<T *>(a.partials) + (int64_t)(first_shared ? t.pad[0] : t.pad[1]) * W;
                for (int i = 0; i < W; ++i) slot[i] = T(0);
            }
        }
    }
    __syncthreads();

    const int g = tid / LG, li = tid % LG;
    const char *Cb = static_cast<const char *>(a.C);
    const uint32_t lo = (uint32_t)li * 16u;
    const T *Tg = static_cast<const T *>(a.T) + (int64_t)(t.a0 + cf0) * W + li * VEC;
    T *A = static_cast<T *>(a.A);
    auto slice_shared = [&](int ls) { return (ls == 0 && (t.flags & 4)) || (ls == nb - 1 && (t.flags & 8)); };
    auto direct = [&](int ls, const P &row) {
        T *dst = A + (int64_t)crdb_s[ls] * W + li * VEC;
        if (!slice_shared(ls)) {
            *reinterpret_cast<P *>(dst) = row;
        } else if (DET) {
            const int slot = (ls == 0 && (t.flags & 4)) ? t.pad[0] : t.pad[1];
            *reinterpret_cast<P *>(static_cast<T *>(a.partials) + (int64_t)slot * W + li * VEC) = row;
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) atomic_add(dst + i, row.v[i]);
        }
    };

    const int gs = g * q, ge = min(gs + q, nfib);
    int head_ls = -1;
    P headv;
#pragma unroll
    for (int i = 0; i < VEC; ++i) headv.v[i] = T(0);
    if (gs < ge) {
        bool started = (gs == 0) || (rec_s[pidx(gs - 1)].s >= 0);   // the current slice starts in this chunk
        Acc asum;
        asum.clear();
        for (int c = gs; c < ge; c += U) {
            FibRec r[U];
            P tt[U], cc[U];
#pragma unroll
            for (int u = 0; u < U; ++u) r[u] = rec_s[pidx(c + u)];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                tt[u] = *reinterpret_cast<const P *>(Tg + (int64_t)min(c + u, nfib - 1) * W);   // clamped: rows past the tile are never used
                cc[u] = *reinterpret_cast<const P *>(Cb + (r[u].coff + lo));
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) asum.v[i] += tt[u].v[i] * cc[u].v[i];
                if (r[u].s >= 0) {
                    P o;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) o.v[i] = asum.v[i];
                    if (started) {
                        direct(r[u].s, o);
                    } else {
                        headv = o;
                        head_ls = r[u].s;
                    }
                    asum.clear();
                    started = true;
                }
            }
        }
        if (chunk_ls[g] >= 0) {   // the chunk ends inside a slice: park the tail
            P o;
#pragma unroll
            for (int i = 0; i < VEC; ++i) o.v[i] = asum.v[i];
            *reinterpret_cast<P *>(slot_s + g * W + li * VEC) = o;
            if (li == 0) slot_id[g] = started ? 1 : 0;
        }
    }
    __syncthreads();
    if (head_ls >= 0) {
        for (int h = g - 1; h >= 0; --h) {
            const P tl = *reinterpret_cast<const P *>(slot_s + h * W + li * VEC);
#pragma unroll
            for (int i = 0; i < VEC; ++i) headv.v[i] += tl.v[i];
            if (slot_id[h] != 0) break;   // the slice began in chunk h
        }
        direct(head_ls, headv);
    }
}

// ------------------------------------------------------------------------------------------
// host side: caps, LDS sizing, dispatch
// ------------------------------------------------------------------------------------------
namespace {

int64_t producer_width(const sc_plan *p)
{
    switch (p->kind) {
    case K_TTMC3: return p->fcols[1];
    case K_MTTKRP3: return p->fcols[0];
    default: return 0;
    }
}

// ------------------------------------------------------------------------------------------
// Deterministic schedules, last two kernels: add rows of `src` in a fixed order and write the
// sum to a row of `dst` (nothing else writes it).  First pass: the pieces of every output row
// that spans several tiles, in segments (dst = segment sums); second pass: the segment sums of
// each such row, into the output.  One workgroup per record; when a row is narrower than the
// workgroup, NT / rowlen lanes share the source rows round robin and their sums are added in
// lane order, so the order of additions is fixed by the plan.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(NT) fixup_rows_kernel(const FixRec *__restrict__ fix, const T *__restrict__ srcbase, T *dstbase, int rowlen)
{
    __shared__ T lane_sum[NT];
    const FixRec f = fix[blockIdx.x];
    const int tid = threadIdx.x;
    const T *src = srcbase + (int64_t)f.first * rowlen;
    T *dst = dstbase + (int64_t)f.row * rowlen;
    if (rowlen <= NT / 2) {
        const int lanes = NT / rowlen;
        const int lane = tid / rowlen, e = tid % rowlen;
        T s = T(0);
        if (lane < lanes) {
#pragma unroll 4
            for (int p = lane; p < f.count; p += lanes) s += src[(int64_t)p * rowlen + e];
        }
        lane_sum[tid] = s;
        __syncthreads();
        if (tid < rowlen) {
            T tot = lane_sum[tid];
            for (int l = 1; l < lanes; ++l) tot += lane_sum[l * rowlen + tid];
            dst[tid] = tot;
        }
    } else {
        for (int e = tid; e < rowlen; e += NT) {
            T s = T(0);
#pragma unroll 8
            for (int p = 0; p < f.count; ++p) s += src[(int64_t)p * rowlen + e];
            dst[e] = s;
        }
    }
}

template <typename T, int W>
sc_status run_order3(const sc_plan *p, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *ws, hipStream_t stream)
{
    const bool had = p->kind == K_MTTKRP3;
    const bool mfma = !had && sizeof(T) == 4 && W == 16 && p->fcols[0] == 16;
    // Range checks come before the first launch, so that a refused execution leaves the output untouched.
    // Factor rows are addressed with 32-bit byte offsets; the fused MTTKRP walk keeps the C row's offset in a
    // signed record (negative = "no fiber ends here"), and the leaf walk of the general kernel marks fiber
    // ends in bit 31 of the D row's offset: 31 bits there.
    for (int s = 0; s < 2; ++s)
        if ((uint64_t)fac[s].rows * (uint64_t)fac[s].ld * sizeof(T) >= (1ull << 32)) return SC_ERR_SHAPE_MISMATCH;
    if (p->sched == SC_SCHED_FUSED && had && (uint64_t)fac[0].rows * (uint64_t)fac[0].ld * sizeof(T) >= (1ull << 31))
        return SC_ERR_SHAPE_MISMATCH;
    if (!(p->sched == SC_SCHED_FUSED && had) && (uint64_t)fac[1].rows * (uint64_t)fac[1].ld * sizeof(T) >= (1ull << 31))
        return SC_ERR_SHAPE_MISMATCH;
    Launcher ln{p, stream};
    launch_output_zero<T>(ln, p, static_cast<T *>(out));
    const int ntiles = (int)p->tiles.size();
    if (ntiles == 0) return ln.status;
    Order3Args a;
    a.tiles = p->d_tiles;
    a.crd1 = sp->crd[0]; a.pos2 = sp->pos[1]; a.crd2 = sp->crd[1]; a.pos3 = sp->pos[2]; a.crd3 = sp->crd[2];
    a.vals = sp->vals;
    a.C = fac[0].data; a.ldC = fac[0].ld;
    a.D = fac[1].data; a.ldD = fac[1].ld;
    a.L = (int32_t)p->fcols[0];
    a.T = ws ? static_cast<char *>(ws) + p->inter[0].offset : nullptr;
    a.A = out;
    a.partials = p->deterministic && ws ? static_cast<char *>(ws) + p->det_top.slot_offset : nullptr;
    a.tn = p->caps.tn; a.ta = p->caps.ta; a.tb = p->caps.tb;
    constexpr bool can_mf = sizeof(T) == 4 && W % 16 == 0;
    const bool mf = can_mf && !had && !mfma && order3_mfma_ranks(a.L, W);
    const size_t lds = order3_lds_bytes<T>(W, a.tn, a.ta, mf ? a.L : 0);
    if (p->sched == SC_SCHED_FUSED) {
        if (had) {
            ln.begin("mttkrp3_fused");
            if (a.partials)
                mttkrp3_fused_kernel<T, W, true><<<ntiles, NT, mttkrp_lds_bytes<T>(W, a.tn, a.ta, a.tb), stream>>>(a);
            else
                mttkrp3_fused_kernel<T, W, false><<<ntiles, NT, mttkrp_lds_bytes<T>(W, a.tn, a.ta, a.tb), stream>>>(a);
        } else if (mfma) {
            ln.status = launch_ttmc3_mfma(p, ln, sp, fac, nullptr, out, a.partials);
            if (ln.status != SC_OK) return ln.status;
            return launch_fixup(p, ln, p->det_top, ws, out);
        } else if (plan_uses_wide_ttmc3(p)) {
            if constexpr (sizeof(T) == 4) {
                ln.status = launch_ttmc3_wide(p, ln, sp, fac, nullptr, out);
                return ln.status;
            }
        } else {
            if constexpr (can_mf) {
                if (mf) {
                    ln.begin("ttmc3_fused_mfma_tiles");
                    order3_kernel<T, W, 0, true><<<ntiles, NT, lds, stream>>>(a);
                    ln.end();
                    return launch_fixup(p, ln, p->det_top, ws, out);
                }
            }
            ln.begin("ttmc3_fused_valu");
            order3_kernel<T, W, 0><<<ntiles, NT, lds, stream>>>(a);
        }
        ln.end();
        return launch_fixup(p, ln, p->det_top, ws, out);
    } else {
        void *partials_a = p->deterministic && ws ? static_cast<char *>(ws) + p->det_a.slot_offset : nullptr;
        sc_status st = launch_leaf_producer(p, ln, sp->vals, fac[1], a.T, W, "order3_traverse", partials_a);
        if (st != SC_OK) return st;
        st = launch_fixup(p, ln, p->det_a, ws, a.T);   // deterministic: the rows of T that span tiles
        if (st != SC_OK) return st;
        if (had) {
            if (a.ta > 2 * NT - 4 || a.tb > NT) return SC_ERR_SCHED_UNSUPPORTED;   // staging registers of the consumer
            ln.begin("mttkrp3_consume");
            if (a.partials)
                hadamard_consume_kernel<T, W, true><<<ntiles, NT, hadamard_lds_bytes<T>(a.ta, a.tb), stream>>>(a);
            else
                hadamard_consume_kernel<T, W, false><<<ntiles, NT, hadamard_lds_bytes<T>(a.ta, a.tb), stream>>>(a);
        } else if (mfma) {
            ln.status = launch_ttmc3_mfma(p, ln, sp, fac, a.T, out, a.partials);
            if (ln.status != SC_OK) return ln.status;
            return launch_fixup(p, ln, p->det_top, ws, out);
        } else if (plan_uses_wide_ttmc3(p)) {
            if constexpr (sizeof(T) == 4) {
                ln.status = launch_ttmc3_wide(p, ln, sp, fac, a.T, out);
                return ln.status;
            }
        } else {
            if constexpr (can_mf) {
                if (mf) {
                    ln.begin("ttmc3_consume_mfma_tiles");
                    order3_kernel<T, W, 2, true><<<ntiles, NT, lds, stream>>>(a);
                    ln.end();
                    return launch_fixup(p, ln, p->det_top, ws, out);
                }
            }
            ln.begin("ttmc3_consume_valu");
            order3_kernel<T, W, 2><<<ntiles, NT, lds, stream>>>(a);
        }
        ln.end();
        return launch_fixup(p, ln, p->det_top, ws, out);
    }
    return ln.status;
}

template <typename T>
sc_status dispatch_order3(const sc_plan *p, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *ws, hipStream_t stream)
{
    switch (producer_width(p)) {
    case 8: return run_order3<T, 8>(p, sp, fac, out, ws, stream);
    case 16: return run_order3<T, 16>(p, sp, fac, out, ws, stream);
    case 32: return run_order3<T, 32>(p, sp, fac, out, ws, stream);
    case 64: return run_order3<T, 64>(p, sp, fac, out, ws, stream);
    case 128: return run_order3<T, 128>(p, sp, fac, out, ws, stream);
    default: return SC_ERR_SCHED_UNSUPPORTED;
    }
}

bool uses_register_fused_mttkrp(const sc_plan *p) { return p->kind == K_MTTKRP3 && p->sched == SC_SCHED_FUSED; }

}  // namespace

TileCaps default_caps(Kind kind, sc_dtype dtype, sc_sched_kind sched, const int64_t *fcols)
{
    TileCaps c{0, 0, 0};
    const int e = dtype == SC_F64 ? 8 : 4;
    switch (kind) {
    case K_TTMC3:
    case K_MTTKRP3: {
        const int64_t w = kind == K_TTMC3 ? fcols[1] : fcols[0];
        if (!(w == 8 || w == 16 || w == 32 || w == 64 || w == 128) || !rank_ok(w, dtype)) return c;
        c.tn = 1024;
        if (kind == K_MTTKRP3 && sched == SC_SCHED_FUSED) {
            // fiber sums live in registers: only boundary tables limit the node counts
            c.ta = 512;
            c.tb = 128;
        } else if (kind == K_MTTKRP3) {
            // keep the T rows of a tile within 32 KB of LDS
            // (at most 508 fibers: the traversal and consumer kernels stage two or three per thread)
            c.ta = (int32_t)std::max<int64_t>(32, std::min<int64_t>(508, (32 * 1024) / (w * e)));
            c.tb = std::min(c.ta, NT);   // the consumer stages one slice per thread
        } else {
            // smaller tiles (T rows within 16 KB) let more workgroups share a CU, which measured
            // faster than larger tiles for the outer-product consumer
            c.tn = 512;
            c.ta = (int32_t)std::max<int64_t>(32, std::min<int64_t>(512, (16 * 1024) / (w * e)));
            c.tb = c.ta;
            if (dtype == SC_F32 && order3_mfma_ranks((int)fcols[0], (int)w)) {
                // matrix-core consumers (the kernel for rank pairs beyond 16 x 16, and the general kernel under a
                // deterministic schedule): T rows and C rows of a tile share about 26 KB; 768 nonzeros and 112 fibers
                // measured best on the uniform 11.5 M-nonzero case at 16 x 32
                c.tn = 768;
                c.ta = (int32_t)std::max<int64_t>(16, std::min<int64_t>(256, (26 * 1024) / ((w + 4 + fcols[0] + 4) * 4)));
                c.tb = c.ta;
            }
            if (dtype == SC_F32 && fcols[0] == 16 && fcols[1] == 16) {
                // matrix-core kernel: measured best on the 30 M-nonzero workload; 224 rows keep the
                // workgroup's LDS (31,328 bytes) just below the size at which five fit a compute unit
                c.tn = 768;
                c.ta = 224;
                c.tb = 64;
            }
        }
        break;
    }
    case K_SDDMM_SPMM: return order2_caps(dtype, fcols);
    case K_TTMC4: return order4_caps(dtype, fcols);
    case K_TTMC_ALL:
    case K_MTTKRP_GEMM:
    case K_SDDMM_SPMM_GEMM: break;   // tiles belong to the inner plan
    }
    return c;
}

bool plan_supports_deterministic(const sc_plan *p)
{
    if (p->kind == K_SDDMM_SPMM) return true;   // both schedules: the sampled values have one writer each
    if (p->kind == K_MTTKRP3 || p->kind == K_TTMC3) return true;   // both schedules
    return plan_wants_tensor_order(p);   // order 4: the fp32 matrix-core kernels, both schedules
}

sc_status launch_fixup(const sc_plan *p, Launcher &ln, const FixLevel &lv, void *ws, void *dst)
{
    if (!p->deterministic || lv.fix.empty()) return ln.status;
    const int rowlen = (int)lv.rowlen;
    char *slots = static_cast<char *>(ws) + lv.slot_offset;
    char *segs = static_cast<char *>(ws) + lv.seg_offset;
    ln.begin("fixup_segments");
    if (p->dtype == SC_F64)
        fixup_rows_kernel<double><<<(int)lv.segs.size(), NT, 0, ln.stream>>>(lv.d_segs, reinterpret_cast<const double *>(slots),
                                                                            reinterpret_cast<double *>(segs), rowlen);
    else
        fixup_rows_kernel<float><<<(int)lv.segs.size(), NT, 0, ln.stream>>>(lv.d_segs, reinterpret_cast<const float *>(slots),
                                                                           reinterpret_cast<float *>(segs), rowlen);
    ln.end();
    ln.begin("fixup_rows");
    if (p->dtype == SC_F64)
        fixup_rows_kernel<double><<<(int)lv.fix.size(), NT, 0, ln.stream>>>(lv.d_fix, reinterpret_cast<const double *>(segs),
                                                                           static_cast<double *>(dst), rowlen);
    else
        fixup_rows_kernel<float><<<(int)lv.fix.size(), NT, 0, ln.stream>>>(lv.d_fix, reinterpret_cast<const float *>(segs),
                                                                          static_cast<float *>(dst), rowlen);
    ln.end();
    return ln.status;
}

// Order-3 chains whose ranks are multiples of the MFMA tile (other than 16 x 16) run the kernel that keeps a slice's
// output tiles in registers across the work tiles of a run (FUSED, and as the consumer behind the leaf traversal);
// deterministic plans stay with the general kernel.
bool plan_uses_wide_ttmc3(const sc_plan *p)
{
    return p->kind == K_TTMC3 && p->dtype == SC_F32 && (p->sched == SC_SCHED_FUSED || p->sched == SC_SCHED_FISSIONED) &&
           !p->deterministic && ttmc3_wide_ranks(p->fcols[0], p->fcols[1]);
}

bool plan_wants_tensor_order(const sc_plan *p)
{
    if (p->dtype != SC_F32 || p->sched == SC_SCHED_LINEAR) return false;
    if (plan_uses_wide_ttmc3(p)) return true;
    if (p->kind == K_TTMC3) return p->fcols[0] == 16 && p->fcols[1] == 16;
    return p->kind == K_TTMC4 && p->fcols[0] <= 16 && p->fcols[1] == 8 && p->fcols[2] == 8;   // the matrix-core kernels of the order-4 chain
}

int plan_output_run(const sc_plan *p)
{
    if (p->sched != SC_SCHED_FUSED && p->sched != SC_SCHED_FISSIONED) return 0;
    if (p->deterministic) return 0;   // one tile per workgroup, pieces in slots: no row is added to
    const bool fused = p->sched == SC_SCHED_FUSED;
    if (plan_uses_wide_ttmc3(p)) return ttmc3_wide_run(p);
    if (p->kind == K_TTMC3 && plan_wants_tensor_order(p)) return ttmc3_mfma_run(p, false);
    if (p->kind == K_TTMC4 && plan_wants_tensor_order(p)) return ttmc4_mfma_run(p, fused ? 0 : 2, false);
    return 0;
}

WalkShape plan_walk_shape(const sc_plan *p)
{
    if (p->sched == SC_SCHED_LINEAR) return WalkShape{};
    if (p->kind == K_TTMC4 && plan_wants_tensor_order(p)) return ttmc4_mfma_walk_shape();   // its leaf level also serves the traversal kernel
    if (plan_uses_wide_ttmc3(p) && p->sched == SC_SCHED_FUSED) return ttmc3_wide_walk_shape((int)p->fcols[1]);
    if (p->kind == K_TTMC3 && p->sched == SC_SCHED_FUSED && plan_wants_tensor_order(p)) return ttmc3_mfma_walk_shape();
    // FISSIONED, order >= 3: the leaf traversal, whose rows are as wide as the last factor
    if (p->sched == SC_SCHED_FISSIONED && (p->kind == K_TTMC3 || p->kind == K_MTTKRP3))
        return leaf_traverse_walk_shape(p->dtype, (int)p->fcols[1]);
    if (p->sched == SC_SCHED_FISSIONED && p->kind == K_TTMC4) return leaf_traverse_walk_shape(p->dtype, (int)p->fcols[2]);
    return WalkShape{};
}

size_t lds_bytes_needed(const sc_plan *p)
{
    if (p->sched == SC_SCHED_LINEAR) return linear_lds_bytes(p);
    switch (p->kind) {
    case K_TTMC3:
    case K_MTTKRP3:
        if (uses_register_fused_mttkrp(p)) {
            // one thread stages at most two fibers and one slice
            if (p->caps.ta > 2 * NT || p->caps.tb > NT) return SIZE_MAX;
            const int w = (int)producer_width(p);
            return p->dtype == SC_F64 ? mttkrp_lds_bytes<double>(w, p->caps.tn, p->caps.ta, p->caps.tb)
                                      : mttkrp_lds_bytes<float>(w, p->caps.tn, p->caps.ta, p->caps.tb);
        }
        if (plan_uses_wide_ttmc3(p))
            return p->sched == SC_SCHED_FUSED ? ttmc3_wide_lds_bytes(p)
                                              : std::max(ttmc3_wide_lds_bytes(p), leaf_traverse_lds_bytes(p, (int)producer_width(p)));
        if (p->kind == K_TTMC3 && plan_wants_tensor_order(p)) {
            if (!ttmc3_mfma_caps_ok(p)) return SIZE_MAX;
            if (p->sched != SC_SCHED_FISSIONED) return ttmc3_mfma_lds_bytes(p);
            return std::max(ttmc3_mfma_lds_bytes(p), leaf_traverse_lds_bytes(p, 16));
        }
        if (p->kind == K_MTTKRP3) {
            // FISSIONED MTTKRP: leaf traversal, then the Hadamard consumer (two fibers and one slice staged per thread)
            if (p->caps.ta > 2 * NT - 4 || p->caps.tb > NT) return SIZE_MAX;
            const size_t cons = p->dtype == SC_F64 ? hadamard_lds_bytes<double>(p->caps.ta, p->caps.tb)
                                                   : hadamard_lds_bytes<float>(p->caps.ta, p->caps.tb);
            return std::max(cons, leaf_traverse_lds_bytes(p, (int)producer_width(p)));
        }
        {
            // general outer-product kernel, fused or as the consumer behind the leaf traversal
            const bool mf = p->kind == K_TTMC3 && p->dtype == SC_F32 && order3_mfma_ranks((int)p->fcols[0], (int)producer_width(p));
            const size_t own = p->dtype == SC_F64 ? order3_lds_bytes<double>((int)producer_width(p), p->caps.tn, p->caps.ta)
                                                  : order3_lds_bytes<float>((int)producer_width(p), p->caps.tn, p->caps.ta, mf ? (int)p->fcols[0] : 0);
            if (p->sched != SC_SCHED_FISSIONED) return own;
            return std::max(own, leaf_traverse_lds_bytes(p, (int)producer_width(p)));
        }
    case K_SDDMM_SPMM: return order2_lds_bytes_needed(p);
    case K_TTMC4: return order4_lds_bytes_needed(p);
    default: return 0;
    }
}

sc_status launch_plan(const sc_plan *p, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *ws, hipStream_t stream)
{
    if (p->prof && p->prof->on) p->prof->n_launch = 0;
    if (p->sched == SC_SCHED_LINEAR && !p->inner) return launch_linear(p, sp, fac, out, stream);
    switch (p->kind) {
    case K_TTMC3:
    case K_MTTKRP3:
        return p->dtype == SC_F64 ? dispatch_order3<double>(p, sp, fac, out, ws, stream)
                                  : dispatch_order3<float>(p, sp, fac, out, ws, stream);
    case K_SDDMM_SPMM: return launch_order2(p, sp, fac, out, ws, stream);
    case K_TTMC4: return launch_order4(p, sp, fac, out, ws, stream);
    case K_TTMC_ALL: return launch_ttmc_all(p, sp, fac, out, ws, stream);
    case K_MTTKRP_GEMM:
    case K_SDDMM_SPMM_GEMM: return launch_trailing_gemm(p, sp, fac, out, ws, stream);
    default: return SC_ERR_SCHED_UNSUPPORTED;

    }
}

}  // namespace sck

// ------------------------------------------------------------------------------------------
// plain streaming copy (calibration of memory-traffic counters)
// ------------------------------------------------------------------------------------------
namespace sck {
__global__ void __launch_bounds__(NT) stream_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x; i < n; i += (int64_t)gridDim.x * NT) dst[i] = src[i];
}
}  // namespace sck

extern "C" sc_status sc_stream_copy(void *dst, const void *src, size_t bytes, void *hip_stream)
{
    if (!dst || !src) return SC_ERR_NULL;
    if (bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) % 16 != 0) return SC_ERR_BAD_DIMS;
    if (bytes == 0) return SC_OK;
    const int64_t n = (int64_t)(bytes / 16);
    const int blocks = (int)std::min<int64_t>((n + sck::NT - 1) / sck::NT, 256 * 32);
    sck::stream_copy_kernel<<<blocks, sck::NT, 0, (hipStream_t)hip_stream>>>(static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), n);
    return hipGetLastError() == hipSuccess ? SC_OK : SC_ERR_DEVICE;
}
