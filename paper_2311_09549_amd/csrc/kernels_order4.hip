// Order-4 TTM chain  A(i,l,m,n) = sum_{j,k,p} B(i,j,k,p) * C(j,l) * D(k,m) * E(p,n)
// under the two-level nest obtained by applying the split-and-fuse step of Section 4.2 twice
// (same shape as the second schedule of Table 2, kernel 5):
//     T1(f3, n)    = sum_{p' in f3} B * E(p, n)              f3 = (i,j,k) fiber
//     T2(f2, m, n) = sum_{f3 in f2} D(k, m) * T1(f3, n)      f2 = (i,j) fiber
//     A(i, l, m, n) = sum_{f2 in slice i} C(j, l) * T2(f2, m, n)
//
// The fp32 case has a matrix-core kernel of its own (kernels_ttmc4.hip); order4_kernel is the
// general kernel for fp64:
// MODE 0 (FUSED):      all three stages per tile, T1 and T2 live in LDS.
// MODE 2 (FISSIONED):  T1 rows (from the workspace) -> T2 rows (to the workspace).
// MODE 3 (FISSIONED):  T2 rows (from the workspace) -> A.
// (The first FISSIONED kernel, leaves -> T1, is the leaf traversal with W = N.)
// The last stage gives every thread a set of output elements and lets it run over the tile's
// slices and f2 fibers in order.
#include "device_common.h"

namespace sck {

struct Order4Args {
    const TileRec *tiles;
    const int32_t *crd1, *pos2, *crd2, *pos3, *crd3, *pos4, *crd4;
    const void *vals;
    const void *C, *D, *E;
    int64_t ldC, ldD, ldE;
    int32_t L;
    void *T1, *T2;
    void *A;
    int32_t tn, ta, tb;
};

template <typename T>
__host__ __device__ constexpr size_t order4_lds_bytes(int N, int W2, int L, int tn, int ta, int tb)
{
    return (size_t)ta * N * sizeof(T) + (size_t)tb * W2 * sizeof(T) + (size_t)padded(tn) * (4 + sizeof(T)) +
           (size_t)(2 * ta + 4 * tb + 16) * 4 + 64;
}

template <typename T, int N, int M, int MODE>
__global__ void __launch_bounds__(NT) order4_kernel(Order4Args a)
{
    constexpr int VEC = VecWidth<T>::value;
    constexpr int W2 = M * N;
    constexpr int LGA = N / VEC, GA = NT / LGA;     // leaf stage: lanes per T1 row, lane groups
    constexpr int LGB = W2 / VEC, GB = NT / LGB;    // middle stage: lanes per T2 row
    constexpr int NPM = N / VEC;                    // lanes per m inside a T2 row
    static_assert(N % VEC == 0 && W2 % VEC == 0 && LGB <= 64 && (LGA & (LGA - 1)) == 0 && (LGB & (LGB - 1)) == 0, "ranks");
    using P = Pack<T, VEC>;
    using Acc = AccVec<T, VEC>;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int L = a.L;
    T *T1_s = reinterpret_cast<T *>(smem);              // ta * N
    T *T2_s = T1_s + (size_t)a.ta * N;                  // tb * W2
    T *val_s = T2_s + (size_t)a.tb * W2;                // padded(tn)
    int *crd_s = reinterpret_cast<int *>(val_s + padded(a.tn));
    int *ba_s = crd_s + padded(a.tn);   // ta + 2   f3 boundaries (leaf offsets)
    int *crda_s = ba_s + a.ta + 2;      // ta       k of each f3
    int *bb_s = crda_s + a.ta;          // tb + 2   f2 boundaries (f3 offsets)
    int *crdb_s = bb_s + a.tb + 2;      // tb       j of each f2
    int *bc_s = crdb_s + a.tb;          // tb + 2   slice boundaries (f2 offsets)
    int *crdc_s = bc_s + a.tb + 2;      // tb       i of each slice

    const TileRec t = a.tiles[blockIdx.x];
    const int tid = threadIdx.x;
    const int nchild = t.n1 - t.n0;
    const int na = t.na, nb = t.nb, nc = t.nc;

    // ---- stage ----
    if (MODE == 0) {
        const T *vals = static_cast<const T *>(a.vals);
        for (int i = tid; i < nchild; i += NT) {
            crd_s[pidx(i)] = a.crd4[t.n0 + i];
            val_s[pidx(i)] = vals[t.n0 + i];
        }
        for (int i = tid; i <= na; i += NT) ba_s[i] = min(max(a.pos4[t.a0 + i], t.n0), t.n1) - t.n0;
        if (tid == 0) ba_s[na + 1] = INT_MAX;
    }
    if (MODE != 3) {
        for (int i = tid; i < na; i += NT) crda_s[i] = a.crd3[t.a0 + i];
        for (int i = tid; i <= nb; i += NT) bb_s[i] = min(max(a.pos3[t.b0 + i], t.a0), t.a0 + na) - t.a0;
        if (tid == 0) {
            bb_s[nb + 1] = INT_MAX;
            // T1 -> T2 kernel: an f3 fiber that continues from the previous tile is consumed by
            // the tile it starts in
            if (MODE == 2 && (t.flags & 1)) bb_s[0] = 1;
        }
    }
    if (MODE != 2) {
        for (int i = tid; i < nb; i += NT) crdb_s[i] = a.crd2[t.b0 + i];
        for (int i = tid; i <= nc; i += NT) bc_s[i] = min(max(a.pos2[t.c0 + i], t.b0), t.b0 + nb) - t.b0;
        if (tid == 0) {
            bc_s[nc + 1] = INT_MAX;
            if (MODE == 3 && (t.flags & 4)) bc_s[0] = 1;   // likewise for f2 fibers in the T2 -> A kernel
        }
        for (int i = tid; i < nc; i += NT) crdc_s[i] = a.crd1[t.c0 + i];
    }
    {
        P z;
#pragma unroll
        for (int i = 0; i < VEC; ++i) z.v[i] = T(0);
        if (MODE == 2) {
            const P *Tg = reinterpret_cast<const P *>(static_cast<const T *>(a.T1) + (int64_t)t.a0 * N);
            for (int i = tid; i < na * LGA; i += NT) reinterpret_cast<P *>(T1_s)[i] = Tg[i];
        } else if (MODE == 0) {
            for (int i = tid; i < na * LGA; i += NT) reinterpret_cast<P *>(T1_s)[i] = z;
        }
        if (MODE == 3) {
            const P *Tg = reinterpret_cast<const P *>(static_cast<const T *>(a.T2) + (int64_t)t.b0 * W2);
            for (int i = tid; i < nb * LGB; i += NT) reinterpret_cast<P *>(T2_s)[i] = Tg[i];
        } else {
            for (int i = tid; i < nb * LGB; i += NT) reinterpret_cast<P *>(T2_s)[i] = z;
        }
    }
    __syncthreads();

    // ---- stage A: leaves -> T1_s ----
    if (MODE == 0) {
        const T *E = static_cast<const T *>(a.E);
        const int g = tid / LGA, li = tid % LGA;
        const int q = (nchild + GA - 1) / GA;
        const int gs = g * q, ge = min(gs + q, nchild);
        struct Item { T v; P d; };
        seg_walk<8, Acc, Item>(
            gs, ge, ba_s, na,
            [&](int c) {
                Item it;
                it.v = val_s[pidx(c)];
                it.d = *reinterpret_cast<const P *>(E + (int64_t)crd_s[pidx(c)] * a.ldE + li * VEC);
                return it;
            },
            [&](Acc &acc, const Item &it) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc.v[i] += it.v * it.d.v[i];
            },
            [&](int lp, const Acc &acc, bool whole) {
                T *dst = T1_s + lp * N + li * VEC;
                if (whole) {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) dst[i] = acc.v[i];
                } else {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) atomic_add(dst + i, acc.v[i]);
                }
            });
        __syncthreads();
    }

    // ---- stage B: T1_s -> T2_s   (outer product with the D row of each f3 fiber) ----
    if (MODE != 3) {
        const T *D = static_cast<const T *>(a.D);
        const int g = tid / LGB, li = tid % LGB;
        const int m = li / NPM, nv = (li % NPM) * VEC;
        const int cf0 = (MODE == 2 && (t.flags & 1)) ? 1 : 0;
        const int nfib = na - cf0;
        const int q = max((nfib + GB - 1) / GB, 1);
        const int gs = cf0 + g * q, ge = min(gs + q, na);
        struct Item { T d; P t1; };
        seg_walk<4, Acc, Item>(
            gs, ge, bb_s, nb,
            [&](int lf) {
                Item it;
                it.d = D[(int64_t)crda_s[lf] * a.ldD + m];
                it.t1 = *reinterpret_cast<const P *>(T1_s + lf * N + nv);
                return it;
            },
            [&](Acc &acc, const Item &it) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc.v[i] += it.d * it.t1.v[i];
            },
            [&](int lp, const Acc &acc, bool whole) {
                T *dst = T2_s + lp * W2 + li * VEC;
                if (whole) {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) dst[i] = acc.v[i];
                } else {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) atomic_add(dst + i, acc.v[i]);
                }
            });
        __syncthreads();
    }

    if (MODE == 2) {
        // write the tile's T2 rows; rows shared with a neighbouring tile are added atomically
        T *Tg = static_cast<T *>(a.T2) + (int64_t)t.b0 * W2;
        for (int i = tid; i < nb * LGB; i += NT) {
            const int lf = i / LGB;
            const bool shared = (lf == 0 && (t.flags & 4)) || (lf == nb - 1 && (t.flags & 8));
            const P v = reinterpret_cast<const P *>(T2_s)[i];
            if (!shared) {
                reinterpret_cast<P *>(Tg)[i] = v;
            } else {
#pragma unroll
                for (int x = 0; x < VEC; ++x) atomic_add(Tg + (int64_t)i * VEC + x, v.v[x]);
            }
        }
        return;
    }

    // ---- stage C: T2_s -> A ----
    const int cf0 = (MODE == 3 && (t.flags & 4)) ? 1 : 0;
    const T *C = static_cast<const T *>(a.C);
    T *A = static_cast<T *>(a.A);
    const int rowA = L * W2;
    auto slice_shared = [&](int ls) { return (ls == 0 && (t.flags & 16)) || (ls == nc - 1 && (t.flags & 32)); };

    for (int e = tid; e < rowA; e += NT) {
        const int l = e / W2, x = e % W2;
        for (int ls = 0; ls < nc; ++ls) {
            const int f0 = max(bc_s[ls], cf0), f1 = bc_s[ls + 1];
            if (f0 >= f1) continue;
            T acc = T(0);
            for (int lf = f0; lf < f1; ++lf) acc += C[(int64_t)crdb_s[lf] * a.ldC + l] * T2_s[lf * W2 + x];
            T *dst = A + (int64_t)crdc_s[ls] * rowA + e;
            if (!slice_shared(ls)) *dst = acc; else atomic_add(dst, acc);
        }
    }
}

namespace {

template <typename T, int N, int M>
sc_status run_order4(const sc_plan *p, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *ws, hipStream_t stream)
{
    Launcher ln{p, stream};
    launch_output_zero<T>(ln, p, static_cast<T *>(out));
    const int ntiles = (int)p->tiles.size();
    if (ntiles == 0) return ln.status;
    Order4Args a;
    a.tiles = p->d_tiles;
    a.crd1 = sp->crd[0]; a.pos2 = sp->pos[1]; a.crd2 = sp->crd[1]; a.pos3 = sp->pos[2]; a.crd3 = sp->crd[2];
    a.pos4 = sp->pos[3]; a.crd4 = sp->crd[3];
    a.vals = sp->vals;
    a.C = fac[0].data; a.ldC = fac[0].ld;
    a.D = fac[1].data; a.ldD = fac[1].ld;
    a.E = fac[2].data; a.ldE = fac[2].ld;
    a.L = (int32_t)p->fcols[0];
    a.T1 = ws ? static_cast<char *>(ws) + p->inter[0].offset : nullptr;
    a.T2 = ws ? static_cast<char *>(ws) + p->inter[1].offset : nullptr;
    a.A = out;
    a.tn = p->caps.tn; a.ta = p->caps.ta; a.tb = p->caps.tb;
    const size_t lds = order4_lds_bytes<T>(N, M * N, a.L, a.tn, a.ta, a.tb);
    const bool mfma = sizeof(T) == 4 && a.L <= 16 && M == 8 && N == 8;   // the matrix-core kernel (fp32, M = N = 8)
    if (p->sched == SC_SCHED_FUSED) {
        if (mfma) {
            void *partials = p->deterministic && ws ? static_cast<char *>(ws) + p->det_top.slot_offset : nullptr;
            ln.status = launch_ttmc4_mfma(p, ln, sp, fac, 0, nullptr, nullptr, out, partials);   // dedicated matrix-core kernel
            if (ln.status != SC_OK) return ln.status;
            return launch_fixup(p, ln, p->det_top, ws, out);
        } else {
            ln.begin("ttmc4_fused_valu");
            order4_kernel<T, N, M, 0><<<ntiles, NT, lds, stream>>>(a);
        }
        ln.end();
    } else {
        // deterministic (matrix-core kernels): each kernel stores its pieces of the rows that span tiles
        // in slots, and a fix-up adds them in tile order before the next kernel reads the rows
        const bool det = p->deterministic && ws && mfma;
        char *wsb = static_cast<char *>(ws);
        sc_status st = launch_leaf_producer(p, ln, sp->vals, fac[2], a.T1, (int)N, "ttmc4_traverse",
                                            det ? wsb + p->det_a.slot_offset : nullptr);
        if (st != SC_OK) return st;
        if (det) {
            st = launch_fixup(p, ln, p->det_a, ws, a.T1);
            if (st != SC_OK) return st;
        } else {
            ln.begin("zero_shared_rows_t2");
            zero_shared_rows_kernel<T><<<(ntiles + 3) / 4, NT, 0, stream>>>(p->d_tiles, ntiles, 1, static_cast<T *>(a.T2), M * N);
            ln.end();
        }
        if (mfma) {
            st = launch_ttmc4_mfma(p, ln, sp, fac, 1, a.T1, a.T2, out, det ? wsb + p->det_b.slot_offset : nullptr);
            if (st != SC_OK) return st;
            if (det) {
                st = launch_fixup(p, ln, p->det_b, ws, a.T2);
                if (st != SC_OK) return st;
            }
            ln.status = launch_ttmc4_mfma(p, ln, sp, fac, 2, a.T1, a.T2, out, det ? wsb + p->det_top.slot_offset : nullptr);
            if (ln.status != SC_OK || !det) return ln.status;
            return launch_fixup(p, ln, p->det_top, ws, out);
        }
        ln.begin("ttmc4_middle");
        order4_kernel<T, N, M, 2><<<ntiles, NT, lds, stream>>>(a);
        ln.end();
        ln.begin("ttmc4_consume_valu");
        order4_kernel<T, N, M, 3><<<ntiles, NT, lds, stream>>>(a);
        ln.end();
    }
    return ln.status;
}

}  // namespace

TileCaps order4_caps(sc_dtype dtype, const int64_t *fcols)
{
    TileCaps c{0, 0, 0};
    // instantiated: M = N = 8 (fp32 on matrix cores, fp64 general kernel) and M = N = 16 (fp32, general kernel); any L up to 16
    if (fcols[0] < 1 || fcols[0] > 16) return c;
    if (fcols[1] == 16 && fcols[2] == 16 && dtype == SC_F32) {
        c.tn = 512; c.ta = 256; c.tb = 24;   // T2 rows of 1 KB: 24 of them next to 256 T1 rows
        return c;
    }
    if (fcols[1] != 8 || fcols[2] != 8) return c;
    if (dtype == SC_F64) {
        c.tn = 512; c.ta = 256; c.tb = 40;
    } else {
        // the largest tile with which four workgroups of the matrix-core kernel fit a compute unit
        // (40,784 bytes of LDS each); measured best on the 50 M-nonzero workload
        c.tn = 768; c.ta = 384; c.tb = 78;
    }
    return c;
}

size_t order4_lds_bytes_needed(const sc_plan *p)
{
    const int N = (int)p->fcols[2], W2 = (int)(p->fcols[1] * p->fcols[2]), L = (int)p->fcols[0];
    const size_t own = p->dtype == SC_F64 ? order4_lds_bytes<double>(N, W2, L, p->caps.tn, p->caps.ta, p->caps.tb)
                                          : order4_lds_bytes<float>(N, W2, L, p->caps.tn, p->caps.ta, p->caps.tb);
    if (p->dtype == SC_F32 && p->fcols[0] <= 16 && p->fcols[1] == 8 && p->fcols[2] == 8) {
        if (!ttmc4_mfma_caps_ok(p)) return SIZE_MAX;
        if (p->sched != SC_SCHED_FISSIONED) return ttmc4_mfma_lds_bytes(p);
        return std::max(ttmc4_mfma_lds_bytes(p), leaf_traverse_lds_bytes(p, N));
    }
    if (p->sched != SC_SCHED_FISSIONED) return own;
    return std::max(own, leaf_traverse_lds_bytes(p, N));  // the leaf traversal is the first FISSIONED kernel
}

sc_status launch_order4(const sc_plan *p, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *ws, hipStream_t stream)
{
    if (p->fcols[1] == 16 && p->fcols[2] == 16 && p->dtype == SC_F32) return run_order4<float, 16, 16>(p, sp, fac, out, ws, stream);
    if (p->fcols[1] != 8 || p->fcols[2] != 8) return SC_ERR_SCHED_UNSUPPORTED;
    return p->dtype == SC_F64 ? run_order4<double, 8, 8>(p, sp, fac, out, ws, stream)
                              : run_order4<float, 8, 8>(p, sp, fac, out, ws, stream);
}

}  // namespace sck
