// LINEAR schedule: the perfectly nested default loop nest of an expression (Section 3, the nest a
// tensor compiler emits before any split), run as it stands: every stored entry is multiplied
// with one element of every factor for every combination of the dense output indices, nothing is
// factored out.  It is the baseline the fused and fissioned nests are compared with
// (nnz * L * M multiply-adds for the order-3 chain instead of M * (nnz + F * L), Section 1), not
// a tuned kernel: one workgroup per tile of nonzeros, one thread per dense output element, the
// partial sum of an output row kept in a register while the tile stays inside one slice and added
// atomically to the zeroed output when the slice changes.
//
//   order 3 chain   A(i,l,m)   += B(i,j,k)   * C(j,l) * D(k,m)
//   MTTKRP          A(i,r)     += B(i,j,k)   * C(j,r) * D(k,r)
//   order 4 chain   A(i,l,m,n) += B(i,j,k,p) * C(j,l) * D(k,m) * E(p,n)
//   SDDMM -> SpMM   A(i,l)     += S(i,j) * X(i,k) * Y(j,k) * Z(j,l)      (loops k and l both inside)
#include "device_common.h"

namespace sck {

namespace {

constexpr int LIN_TN = 1024;   // nonzeros per tile at most (LDS: five words per nonzero)

struct LinArgs {
    const int32_t *pos[4];
    const int32_t *crd[4];
    const void *vals;
    const void *F[3];
    int64_t ld[3];
    int32_t cols[3];
    void *A;
    int32_t order, kind, row_elems;
};

// Last node x in [lo, lo + n) with pos[x] <= z: the parent of child z among the tile's nodes.
__device__ __forceinline__ int32_t parent_in(const int32_t *pos, int32_t lo, int32_t n, int32_t z)
{
    int32_t a = lo, b = lo + n - 1;
    while (a < b) {
        const int32_t mid = (a + b + 1) >> 1;
        if (pos[mid] <= z) a = mid; else b = mid - 1;
    }
    return a;
}

template <typename T>
__global__ void __launch_bounds__(NT) linear_kernel(LinArgs a, const TileRec *__restrict__ tiles)
{
    __shared__ int32_t c0_s[LIN_TN], c1_s[LIN_TN], c2_s[LIN_TN], c3_s[LIN_TN];
    __shared__ T v_s[LIN_TN];
    const TileRec t = tiles[blockIdx.x];
    const int tid = threadIdx.x;
    const int nchild = t.n1 - t.n0;
    const int d = a.order;
    const T *vals = static_cast<const T *>(a.vals);

    // coordinates of every nonzero of the tile: the leaf's own, then its ancestors' (found among the
    // tile's nodes of each level)
    for (int c = tid; c < nchild; c += NT) {
        const int32_t z = t.n0 + c;
        int32_t co[4] = {0, 0, 0, 0};
        co[d - 1] = a.crd[d - 1][z];
        const int32_t xa = parent_in(a.pos[d - 1], t.a0, t.na, z);
        co[d - 2] = a.crd[d - 2][xa];
        if (d >= 3) {
            const int32_t xb = parent_in(a.pos[d - 2], t.b0, t.nb, xa);
            co[d - 3] = a.crd[d - 3][xb];
            if (d == 4) {
                const int32_t xc = parent_in(a.pos[1], t.c0, t.nc, xb);
                co[0] = a.crd[0][xc];
            }
        }
        c0_s[c] = co[0]; c1_s[c] = co[1]; c2_s[c] = co[2]; c3_s[c] = co[3];
        v_s[c] = vals[z];
    }
    __syncthreads();

    const int E = a.row_elems;
    // E >= NT: a thread owns elements tid, tid + NT, ... and walks all nonzeros for each;
    // E <  NT: NT / E sets of E threads share the nonzeros (set s takes nonzeros s, s + sets, ...)
    const int sets = E >= NT ? 1 : NT / E;
    const int s = E >= NT ? 0 : tid / E;
    if (s >= sets) return;
    const T *F0 = static_cast<const T *>(a.F[0]), *F1 = static_cast<const T *>(a.F[1]), *F2 = static_cast<const T *>(a.F[2]);
    T *A = static_cast<T *>(a.A);
    for (int e = E >= NT ? tid : tid % E; e < E; e += (E >= NT ? NT : E)) {
        T acc = T(0);
        int32_t cur = -1;
        for (int c = s; c < nchild; c += sets) {
            const int32_t i = c0_s[c];
            if (i != cur) {
                if (cur >= 0) atomic_add(A + (int64_t)cur * E + e, acc);
                acc = T(0);
                cur = i;
            }
            const T v = v_s[c];
            switch (a.kind) {
            case K_TTMC3: {
                const int l = e / a.cols[1], m = e % a.cols[1];
                acc += v * F0[(int64_t)c1_s[c] * a.ld[0] + l] * F1[(int64_t)c2_s[c] * a.ld[1] + m];
                break;
            }
            case K_MTTKRP3:
                acc += v * F0[(int64_t)c1_s[c] * a.ld[0] + e] * F1[(int64_t)c2_s[c] * a.ld[1] + e];
                break;
            case K_TTMC4: {
                const int mn = a.cols[1] * a.cols[2];
                const int l = e / mn, m = (e / a.cols[2]) % a.cols[1], n = e % a.cols[2];
                acc += v * F0[(int64_t)c1_s[c] * a.ld[0] + l] * F1[(int64_t)c2_s[c] * a.ld[1] + m] * F2[(int64_t)c3_s[c] * a.ld[2] + n];
                break;
            }
            default: {   // K_SDDMM_SPMM: X(i,k) Y(j,k) Z(j,l), the k loop inside the l loop
                const T *x = F0 + (int64_t)i * a.ld[0], *y = F1 + (int64_t)c1_s[c] * a.ld[1];
                const T zl = F2[(int64_t)c1_s[c] * a.ld[2] + e];
                for (int k = 0; k < a.cols[0]; ++k) acc += v * x[k] * y[k] * zl;
                break;
            }
            }
        }
        if (cur >= 0) atomic_add(A + (int64_t)cur * E + e, acc);
    }
}

}  // namespace

size_t linear_lds_bytes(const sc_plan *p)
{
    if (p->caps.tn > LIN_TN) return SIZE_MAX;
    return (size_t)LIN_TN * (16 + (p->dtype == SC_F64 ? 8 : 4));
}

sc_status launch_linear(const sc_plan *p, const sc_csf_view *sp, const sc_dense_view *fac, void *out, hipStream_t stream)
{
    Launcher ln{p, stream};
    if (p->dtype == SC_F64)
        launch_output_zero<double>(ln, p, static_cast<double *>(out));
    else
        launch_output_zero<float>(ln, p, static_cast<float *>(out));
    const int ntiles = (int)p->tiles.size();
    if (ntiles == 0) return ln.status;
    if (p->caps.tn > LIN_TN) return SC_ERR_SCHED_UNSUPPORTED;
    LinArgs a = {};
    for (int m = 0; m < 4; ++m) {
        a.pos[m] = sp->pos[m];
        a.crd[m] = sp->crd[m];
    }
    a.vals = sp->vals;
    for (int s = 0; s < p->nfactors; ++s) {
        a.F[s] = fac[s].data;
        a.ld[s] = fac[s].ld;
        a.cols[s] = (int32_t)fac[s].cols;
    }
    a.A = out;
    a.order = p->order;
    a.kind = (int32_t)p->kind;
    a.row_elems = (int32_t)p->out_row_elems;
    ln.begin("linear_nest");
    if (p->dtype == SC_F64)
        linear_kernel<double><<<ntiles, NT, 0, stream>>>(a, p->d_tiles);
    else
        linear_kernel<float><<<ntiles, NT, 0, stream>>>(a, p->d_tiles);
    ln.end();
    return ln.status;
}

}  // namespace sck
