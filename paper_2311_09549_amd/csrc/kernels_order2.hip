// Order-2 kernels: Table 2, kernel 1 <SDDMM,SpMM>
//     A(i,l) = sum_j S(i,j) * ( sum_k X(i,k) * Y(j,k) ) * Z(j,l)
// under the paper's chosen nest  i, j' < t ; k: t += S*X*Y , l: A += t*Z >.
//
// MODE 0 (FUSED): the sampled value t stays a register scalar; one walk over the stored
//                 entries of S gathers X(i,:), Y(j,:) and Z(j,:), reduces the dot product
//                 across the lane group and accumulates t * Z(j,:) into the row sum.
// MODE 1 (FISSIONED, first kernel, SDDMM):  t(z) written to the workspace, one per entry.
// MODE 2 (FISSIONED, second kernel, SpMM):  A(i,:) += t(z) * Z(j,:) with t read back.
//
// Work is cut into equal-nnz tiles (rows are level "a" of the tile record); a lane group of
// LG = W / VEC lanes owns one stored entry per step (W = K = L).  Staging builds one LDS
// record per entry {X row offset, Y row offset, Z row offset, value} plus a row-end mark, so
// the walk is a branch-free batch of gathers followed by arithmetic.
#include "device_common.h"

namespace sck {

struct Order2Args {
    const TileRec *tiles;
    const int32_t *crd1, *pos2, *crd2;
    const void *vals;
    const void *X, *Y, *Z;
    int64_t ldX, ldY, ldZ;
    void *T;   // sampled values, one per stored entry (MODE 1 writes, MODE 2 reads)
    void *A;
    void *partials;   // deterministic schedules: slots for the pieces of rows that span tiles, else null
    int32_t tn, ta;
};

template <typename T>
struct alignas(sizeof(T) == 4 ? 16 : 8) SdRec {
    uint32_t xoff, yoff, zoff;
    T v;
};

template <typename T>
__host__ __device__ constexpr size_t order2_lds_bytes(int tn, int ta)
{
    return (size_t)NT * 16 + (size_t)padded(tn + 8) * (sizeof(SdRec<T>) + 4) + (size_t)(3 * ta + 8) * 4 + 2 * NT * 4 + 64;
}

template <typename T, int W, int MODE>
__global__ void __launch_bounds__(NT) sddmm_spmm_kernel(Order2Args a)
{
    constexpr int VEC = VecWidth<T>::value;
    constexpr int LG = W / VEC;
    constexpr int G = NT / LG;
    constexpr int U = 4;
    static_assert(W % VEC == 0 && (LG & (LG - 1)) == 0 && LG <= 64, "row width");
    using P = Pack<T, VEC>;
    using Acc = AccVec<T, VEC>;
    using Rec = SdRec<T>;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    T *slot_s = reinterpret_cast<T *>(smem);                         // NT * VEC
    Rec *rec_s = reinterpret_cast<Rec *>(slot_s + NT * VEC);         // padded(tn + 8)
    int *end_s = reinterpret_cast<int *>(rec_s + padded(a.tn + 8));  // padded(tn + 8): local row if the entry ends its row
    int *ba_s = end_s + padded(a.tn + 8);                            // ta + 2: first entry of each row (tile-local)
    uint32_t *xrow_s = reinterpret_cast<uint32_t *>(ba_s + a.ta + 2);  // ta: byte offset of X(i,:)
    int *crda_s = reinterpret_cast<int *>(xrow_s + a.ta);            // ta: output row
    int *chunk_ls = crda_s + a.ta;                                   // NT
    int *slot_id = chunk_ls + NT;                                    // NT

    const TileRec t = a.tiles[blockIdx.x];
    const int tid = threadIdx.x;
    const int nchild = t.n1 - t.n0;
    const int na = t.na;
    const int q = max(((nchild + G - 1) / G + U - 1) / U * U, U);   // entries per lane group, multiple of U
    const uint32_t rowX = (uint32_t)(a.ldX * sizeof(T)), rowY = (uint32_t)(a.ldY * sizeof(T)), rowZ = (uint32_t)(a.ldZ * sizeof(T));

    // ---- stage 1: row tables, marks cleared ----
    for (int i = tid; i <= na; i += NT) ba_s[i] = min(max(a.pos2[t.a0 + i], t.n0), t.n1) - t.n0;
    if (tid == 0) ba_s[na + 1] = INT_MAX;
    for (int i = tid; i < na; i += NT) {
        const int row = a.crd1[t.a0 + i];
        crda_s[i] = row;
        xrow_s[i] = (uint32_t)row * rowX;
    }
    for (int c = tid; c < nchild + U; c += NT) end_s[pidx(c)] = -1;
    {
        P z;
#pragma unroll
        for (int i = 0; i < VEC; ++i) z.v[i] = T(0);
        reinterpret_cast<P *>(slot_s)[tid] = z;
        slot_id[tid] = -1;
        chunk_ls[tid] = -1;
    }
    __syncthreads();

    // ---- stage 2: one record per entry; row ends and rows cut by chunk boundaries ----
    {
        const T *vals = static_cast<const T *>(MODE == 2 ? a.T : a.vals);
        const int c0 = 4 * tid;
        if (c0 < nchild) {
            int lr = find_segment(ba_s, na, c0);
            int rend = ba_s[lr + 1];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int c = c0 + r;
                if (c < nchild) {
                    while (c >= rend) {
                        ++lr;
                        rend = ba_s[lr + 1];
                    }
                    const uint32_t j = (uint32_t)a.crd2[t.n0 + c];
                    Rec rec;
                    rec.xoff = xrow_s[lr];
                    rec.yoff = j * rowY;
                    rec.zoff = j * rowZ;
                    rec.v = vals[t.n0 + c];
                    rec_s[pidx(c)] = rec;
                }
            }
        }
        if (tid < U) {  // dummies completing the last batch
            Rec rec;
            rec.xoff = rec.yoff = rec.zoff = 0;
            rec.v = T(0);
            rec_s[pidx(nchild + tid)] = rec;
        }
        for (int i = tid; i < na; i += NT) {
            const int lo = ba_s[i], hi = ba_s[i + 1];
            if (hi > lo) {
                end_s[pidx(hi - 1)] = i;
                for (int m = lo / q + 1; m * q < hi; ++m) chunk_ls[m - 1] = i;
            }
        }
    }
    __syncthreads();

    const int g = tid / LG, li = tid % LG;
    const char *Xb = static_cast<const char *>(a.X) + li * 16;
    const char *Yb = static_cast<const char *>(a.Y) + li * 16;
    const char *Zb = static_cast<const char *>(a.Z) + li * 16;
    T *A = static_cast<T *>(a.A);
    auto row_shared = [&](int lr) { return (lr == 0 && (t.flags & 1)) || (lr == na - 1 && (t.flags & 2)); };
    auto direct = [&](int lr, const P &row) {
        T *dst = A + (int64_t)crda_s[lr] * W + li * VEC;
        if (!row_shared(lr)) {
            *reinterpret_cast<P *>(dst) = row;
        } else if (a.partials) {
            // deterministic: the tile's one piece of this row goes to its slot (a tile whose only
            // row continues on both sides has one piece, numbered as its first)
            const int slot = (lr == 0 && (t.flags & 1)) ? t.pad[0] : t.pad[1];
            *reinterpret_cast<P *>(static_cast<T *>(a.partials) + (int64_t)slot * W + li * VEC) = row;
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) atomic_add(dst + i, row.v[i]);
        }
    };

    // A lane group whose chunk starts inside a row keeps that row's piece ("head") in registers
    // when the row ends; a chunk that ends inside a row parks its running sum ("tail") in its
    // LDS row together with a flag telling whether the row began in this chunk.  After the
    // barrier the group holding a head adds the tails of the chunks before it, back to the one
    // in which the row began, and issues the tile's single update of that output row: no LDS
    // atomics, and a fixed order of additions.
    const int gs = g * q, ge = min(gs + q, nchild);
    int head_lr = -1;
    P headv;
#pragma unroll
    for (int i = 0; i < VEC; ++i) headv.v[i] = T(0);
    if (gs < ge) {
        bool started = (gs == 0) || (end_s[pidx(gs - 1)] >= 0);  // the current row starts in this chunk
        Acc asum;
        asum.clear();
        auto emit = [&](int lr, bool whole) {
            P o;
#pragma unroll
            for (int i = 0; i < VEC; ++i) o.v[i] = asum.v[i];
            if (whole) {
                direct(lr, o);
            } else {
                headv = o;
                head_lr = lr;
            }
        };
        for (int c = gs; c < ge; c += U) {
            Rec r[U];
            int e[U];
            P x[U], y[U], z[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                r[u] = rec_s[pidx(c + u)];
                e[u] = end_s[pidx(c + u)];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (MODE < 2) {
                    x[u] = *reinterpret_cast<const P *>(Xb + r[u].xoff);
                    y[u] = *reinterpret_cast<const P *>(Yb + r[u].yoff);
                }
                if (MODE != 1) z[u] = *reinterpret_cast<const P *>(Zb + r[u].zoff);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                T tv = r[u].v;
                if (MODE < 2) {
                    T p = T(0);
#pragma unroll
                    for (int i = 0; i < VEC; ++i) p += x[u].v[i] * y[u].v[i];
#pragma unroll
                    for (int m = LG / 2; m >= 1; m >>= 1) p += __shfl_xor(p, m, LG);
                    tv *= p;
                }
                if (MODE == 1) {
                    if (li == 0 && c + u < nchild) static_cast<T *>(a.T)[t.n0 + c + u] = tv;
                } else {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) asum.v[i] += tv * z[u].v[i];
                    if (e[u] >= 0) {
                        emit(e[u], started);
                        asum.clear();
                        started = true;
                    }
                }
            }
        }
        if (MODE != 1 && chunk_ls[g] >= 0) {  // the chunk ends inside a row: park the tail
            P o;
#pragma unroll
            for (int i = 0; i < VEC; ++i) o.v[i] = asum.v[i];
            *reinterpret_cast<P *>(slot_s + g * W + li * VEC) = o;
            if (li == 0) slot_id[g] = started ? 1 : 0;
        }
    }
    if (MODE == 1) return;
    __syncthreads();
    if (head_lr >= 0) {
        for (int h = g - 1; h >= 0; --h) {
            const P tl = *reinterpret_cast<const P *>(slot_s + h * W + li * VEC);
#pragma unroll
            for (int i = 0; i < VEC; ++i) headv.v[i] += tl.v[i];
            if (slot_id[h] != 0) break;   // the row began in chunk h
        }
        direct(head_lr, headv);
    }
}

namespace {

template <typename T, int W>
sc_status run_order2(const sc_plan *p, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *ws, hipStream_t stream)
{
    Launcher ln{p, stream};
    launch_output_zero<T>(ln, p, static_cast<T *>(out));
    const int ntiles = (int)p->tiles.size();
    if (ntiles == 0) return ln.status;
    // rows are addressed with 32-bit byte offsets
    for (int s = 0; s < 3; ++s)
        if ((uint64_t)fac[s].rows * (uint64_t)fac[s].ld * sizeof(T) >= (1ull << 32)) return SC_ERR_SHAPE_MISMATCH;
    Order2Args a;
    a.tiles = p->d_tiles;
    a.crd1 = sp->crd[0]; a.pos2 = sp->pos[1]; a.crd2 = sp->crd[1];
    a.vals = sp->vals;
    a.X = fac[0].data; a.ldX = fac[0].ld;
    a.Y = fac[1].data; a.ldY = fac[1].ld;
    a.Z = fac[2].data; a.ldZ = fac[2].ld;
    a.T = ws ? static_cast<char *>(ws) + p->inter[0].offset : nullptr;
    a.A = out;
    a.partials = p->deterministic && ws ? static_cast<char *>(ws) + p->det_top.slot_offset : nullptr;
    a.tn = p->caps.tn; a.ta = p->caps.ta;
    const size_t lds = order2_lds_bytes<T>(a.tn, a.ta);
    if (p->sched == SC_SCHED_FUSED) {
        ln.begin("sddmm_spmm_fused");
        sddmm_spmm_kernel<T, W, 0><<<ntiles, NT, lds, stream>>>(a);
        ln.end();
    } else {
        ln.begin("sddmm_traverse");
        sddmm_spmm_kernel<T, W, 1><<<ntiles, NT, lds, stream>>>(a);
        ln.end();
        ln.begin("spmm_consume");
        sddmm_spmm_kernel<T, W, 2><<<ntiles, NT, lds, stream>>>(a);
        ln.end();
    }
    return launch_fixup(p, ln, p->det_top, ws, out);
}

template <typename T>
sc_status dispatch_order2(const sc_plan *p, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *ws, hipStream_t stream)
{
    switch (p->fcols[0]) {
    case 16: return run_order2<T, 16>(p, sp, fac, out, ws, stream);
    case 32: return run_order2<T, 32>(p, sp, fac, out, ws, stream);
    case 64: return run_order2<T, 64>(p, sp, fac, out, ws, stream);
    case 128: return run_order2<T, 128>(p, sp, fac, out, ws, stream);
    default: return SC_ERR_SCHED_UNSUPPORTED;
    }
}

}  // namespace

TileCaps order2_caps(sc_dtype dtype, const int64_t *fcols)
{
    TileCaps c{0, 0, 0};
    const int64_t k = fcols[0], l = fcols[2];
    // one lane group covers both the dot-product width and the output width
    if (k != l || !(k == 16 || k == 32 || k == 64 || k == 128) || !rank_ok(k, dtype)) return c;
    c.tn = 1024;
    c.ta = 512;
    return c;
}

size_t order2_lds_bytes_needed(const sc_plan *p)
{
    if (p->caps.tn > 4 * NT) return SIZE_MAX;  // staging gives every thread four consecutive entries
    return p->dtype == SC_F64 ? order2_lds_bytes<double>(p->caps.tn, p->caps.ta) : order2_lds_bytes<float>(p->caps.tn, p->caps.ta);
}

sc_status launch_order2(const sc_plan *p, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *ws, hipStream_t stream)
{
    return p->dtype == SC_F64 ? dispatch_order2<double>(p, sp, fac, out, ws, stream)
                              : dispatch_order2<float>(p, sp, fac, out, ws, stream);
}

}  // namespace sck
