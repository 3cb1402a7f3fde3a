// All-mode TTMC, kernel 5 of Table 2 (the running example of Sections 1 and 3):
//     A(l,m,n) = sum_ijk B(i,j,k) * C(i,l) * D(j,m) * E(k,n)
// under the three schedules Table 2 lists for it.  The output carries no sparse index, so whatever
// the nest produces per slice (or per fiber) has to be reduced over the whole grid; that last
// contraction is what this file adds.  The sparse part reuses the order-3 TTM chain
//     S(i,m,n) = sum_jk B(i,j,k) * D(j,m) * E(k,n)
// of the library (an inner plan over the same tensor with factors D and E):
//
//   schedule 2 (default)  i,n < T_m; j' < t; k': t += B E, m: T_m += t D >, m,l: A += T_m C >
//                         inner plan FUSED (t and T_m on chip) or FISSIONED (t(i,j,n) in the
//                         workspace), then mode0_reduce: A(l,:) += C(i,l) * S(i,:)
//   schedule 3            i,m,n < t; j',k': t += B D E, l: A += t C >
//                         inner plan LINEAR (the unfactored nest per slice), then mode0_reduce
//   schedule 1            i,j',n < t; k': t += B E, m,l: A += t C D >
//                         leaf traversal of the inner plan (t(i,j,:) per fiber in the workspace), then
//                         fiber_reduce: A(l,m,n) += C(i,l) * D(j,m) * t(f,n) over all fibers
//
// Both reductions are deterministic: a workgroup sums a contiguous chunk of slices (fibers) into an
// L x (M N) tile in registers and stores it in its own slot of the workspace; sum_partials adds the
// slots in chunk order.  The reduction over i is a dense (L x I) * (I x MN) product with I large:
// 2 L flops per 4-byte element of S read.  In fp32 with L in {16, 32, 64, 128} and M N a multiple of 64 it runs
// on the matrix cores with all of L per workgroup, so that S is read once whatever L is; the other cases
// (fp64, other ranks) run on the vector ALUs, a thread per column with 16 values of l in registers.
#include "device_common.h"

namespace sck {

namespace {

constexpr int KB_L = 16;     // output slabs (values of l) one thread accumulates
constexpr int KR_ROWS = 64;  // rows of C staged per pass of mode0_reduce

struct K5Args {
    const void *C;
    int64_t ldC;
    const void *D;
    int64_t ldD;
    const void *S;          // mode0_reduce: I x MN, row-major; fiber_reduce: t rows, F x N
    const int32_t *crd1, *pos2, *crd2;   // fiber_reduce: slices and fibers of the tensor
    void *partials;         // nchunks x L x MN
    int64_t rows;           // I (mode0_reduce) or F (fiber_reduce)
    int32_t nslices;        // fiber_reduce: non-empty slices
    int32_t L, M, N, MN;
    int32_t chunk;          // rows (slices / fibers) per workgroup
};

// partial(b, l, c) = sum_{i in chunk b} C(i,l) * S(i,c); thread = column c, KB_L values of l in registers
template <typename T>
__global__ void __launch_bounds__(NT) mode0_reduce_kernel(K5Args a)
{
    __shared__ T c_s[KR_ROWS * KB_L];
    const int tid = threadIdx.x;
    const int c = blockIdx.y * NT + tid;
    const int l0 = blockIdx.z * KB_L;
    const int nl = min(KB_L, a.L - l0);
    const int64_t r0 = (int64_t)blockIdx.x * a.chunk, r1 = min(r0 + a.chunk, a.rows);
    const T *C = static_cast<const T *>(a.C);
    const T *S = static_cast<const T *>(a.S);
    T acc[KB_L];
#pragma unroll
    for (int l = 0; l < KB_L; ++l) acc[l] = T(0);
    for (int64_t rb = r0; rb < r1; rb += KR_ROWS) {
        const int nr = (int)min<int64_t>(KR_ROWS, r1 - rb);
        __syncthreads();
        for (int e = tid; e < KR_ROWS * KB_L; e += NT) {
            const int r = e / KB_L, l = e % KB_L;
            c_s[e] = (r < nr && l < nl) ? C[(rb + r) * a.ldC + l0 + l] : T(0);
        }
        __syncthreads();
        if (c < a.MN) {
            for (int r = 0; r < nr; ++r) {
                const T s = S[(rb + r) * (int64_t)a.MN + c];
#pragma unroll
                for (int l = 0; l < KB_L; ++l) acc[l] += c_s[r * KB_L + l] * s;
            }
        }
    }
    if (c < a.MN) {
        T *P = static_cast<T *>(a.partials) + (int64_t)blockIdx.x * a.L * a.MN;
        for (int l = 0; l < nl; ++l) P[(int64_t)(l0 + l) * a.MN + c] = acc[l];
    }
}

// The same partial sums on the matrix cores, fp32, L = 16 LT in {16, 32, 64, 128}, M N a multiple of 64: a workgroup takes all of L
// for 64 columns (a wavefront for 16 of them), so S is read once instead of once per 16 values of l; four slices per
// v_mfma_f32_16x16x4_f32 with C^T as operand A (l along the rows) and S as operand B, both straight from global memory
// (a lane's 16 neighbours read 64 contiguous bytes of a row).
typedef float k5_floatx4 __attribute__((ext_vector_type(4)));
template <int LT>
__global__ void __launch_bounds__(NT) mode0_reduce_mfma_kernel(K5Args a)
{
    constexpr int UK = 4;   // steps of four slices whose operand reads are issued together
    const int tid = threadIdx.x;
    const int wave = tid / 64, lane = tid % 64, kk = lane / 16, col = lane % 16;
    const int c = blockIdx.y * 64 + wave * 16 + col;   // < M N: the launch has M N / 64 workgroups along y
    const int64_t r0 = (int64_t)blockIdx.x * a.chunk, r1 = min(r0 + a.chunk, a.rows);
    const float *C = static_cast<const float *>(a.C) + col;
    const float *S = static_cast<const float *>(a.S) + c;
    k5_floatx4 acc[LT];
#pragma unroll
    for (int lt = 0; lt < LT; ++lt) acc[lt] = k5_floatx4{0.f, 0.f, 0.f, 0.f};
    for (int64_t rb = r0; rb < r1; rb += 4 * UK) {
        float sv[UK], cv[UK][LT];
#pragma unroll
        for (int u = 0; u < UK; ++u) {
            const int64_t row = rb + 4 * u + kk, rc = min(row, r1 - 1);   // lanes past the chunk read its last slice and are zeroed
            const bool ok = row < r1;
            const float s = S[rc * (int64_t)a.MN];
            sv[u] = ok ? s : 0.f;
#pragma unroll
            for (int lt = 0; lt < LT; ++lt) {
                const float v = C[rc * a.ldC + lt * 16];
                cv[u][lt] = ok ? v : 0.f;
            }
        }
#pragma unroll
        for (int u = 0; u < UK; ++u)
#pragma unroll
            for (int lt = 0; lt < LT; ++lt) acc[lt] = __builtin_amdgcn_mfma_f32_16x16x4f32(cv[u][lt], sv[u], acc[lt], 0, 0, 0);
    }
    // acc[lt][r] = partial(l = 16 lt + 4 kk + r, column c)
    float *P = static_cast<float *>(a.partials) + (int64_t)blockIdx.x * a.L * a.MN + c;
#pragma unroll
    for (int lt = 0; lt < LT; ++lt)
#pragma unroll
        for (int r = 0; r < 4; ++r) P[(int64_t)(lt * 16 + 4 * kk + r) * a.MN] = acc[lt][r];
}

// partial(b, l, (m,n)) = sum_{fibers f in chunk b} C(i_f,l) * D(j_f,m) * t(f,n); thread = (m,n)
template <typename T>
__global__ void __launch_bounds__(NT) fiber_reduce_kernel(K5Args a)
{
    __shared__ int s_first;
    const int tid = threadIdx.x;
    const int c = blockIdx.y * NT + tid;
    const int l0 = blockIdx.z * KB_L;
    const int nl = min(KB_L, a.L - l0);
    const int64_t f0 = (int64_t)blockIdx.x * a.chunk, f1 = min(f0 + a.chunk, a.rows);
    const T *C = static_cast<const T *>(a.C);
    const T *D = static_cast<const T *>(a.D);
    const T *Tt = static_cast<const T *>(a.S);
    if (tid == 0) {   // slice that holds fiber f0: last s with pos2[s] <= f0
        int lo = 0, hi = a.nslices;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (a.pos2[mid] <= f0) lo = mid; else hi = mid;
        }
        s_first = lo;
    }
    __syncthreads();
    int s = s_first;
    int64_t s_end = a.pos2[s + 1];
    const int m = c < a.MN ? c / a.N : 0, n = c < a.MN ? c % a.N : 0;
    T acc[KB_L];
#pragma unroll
    for (int l = 0; l < KB_L; ++l) acc[l] = T(0);
    T crow[KB_L];
    auto load_c = [&](int slice) {
        const int64_t i = a.crd1[slice];
#pragma unroll
        for (int l = 0; l < KB_L; ++l) crow[l] = l < nl ? C[i * a.ldC + l0 + l] : T(0);
    };
    load_c(s);
    for (int64_t f = f0; f < f1; ++f) {
        if (f >= s_end) {   // uniform: every thread walks the same fibers
            ++s;
            s_end = a.pos2[s + 1];
            load_c(s);
        }
        const int64_t j = a.crd2[f];
        const T dt = D[j * a.ldD + m] * Tt[f * a.N + n];
#pragma unroll
        for (int l = 0; l < KB_L; ++l) acc[l] += crow[l] * dt;
    }
    if (c < a.MN) {
        T *P = static_cast<T *>(a.partials) + (int64_t)blockIdx.x * a.L * a.MN;
        for (int l = 0; l < nl; ++l) P[(int64_t)(l0 + l) * a.MN + c] = acc[l];
    }
}

// LINEAR: the perfectly nested loop of Figure 2a, nothing factored out: every stored entry is multiplied with one
// element of each of the three factors for every (l, m, n).  A workgroup walks a contiguous chunk of fibers; a
// thread owns KB_L output elements e = (l, m, n) of one block of KB_L * NT elements (blockIdx.y) and keeps their
// sums in registers; the partial tiles of the chunks are added by sum_partials like those of the other schedules.
template <typename T>
__global__ void __launch_bounds__(NT) linear_all_kernel(K5Args a, const int32_t *__restrict__ pos3, const int32_t *__restrict__ crd3,
                                                        const T *__restrict__ vals, const T *__restrict__ E, int64_t ldE)
{
    __shared__ int s_first;
    const int tid = threadIdx.x;
    const int64_t elems = (int64_t)a.L * a.MN;
    const int64_t f0 = (int64_t)blockIdx.x * a.chunk, f1 = min(f0 + a.chunk, a.rows);
    const T *C = static_cast<const T *>(a.C);
    const T *D = static_cast<const T *>(a.D);
    if (tid == 0) {   // slice that holds fiber f0: last s with pos2[s] <= f0
        int lo = 0, hi = a.nslices;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (a.pos2[mid] <= f0) lo = mid; else hi = mid;
        }
        s_first = lo;
    }
    __syncthreads();
    int l[KB_L], m[KB_L], n[KB_L];
    bool ok[KB_L];
    T acc[KB_L];
#pragma unroll
    for (int r = 0; r < KB_L; ++r) {
        const int64_t e = ((int64_t)blockIdx.y * KB_L + r) * NT + tid;
        ok[r] = e < elems;
        const int64_t ec = ok[r] ? e : 0;
        l[r] = (int)(ec / a.MN);
        m[r] = (int)((ec % a.MN) / a.N);
        n[r] = (int)(ec % a.N);
        acc[r] = T(0);
    }
    int s = s_first;
    int64_t s_end = a.pos2[s + 1];
    int64_t i = a.crd1[s];
    for (int64_t f = f0; f < f1; ++f) {
        if (f >= s_end) {   // uniform: every thread walks the same fibers
            ++s;
            s_end = a.pos2[s + 1];
            i = a.crd1[s];
        }
        const int64_t j = a.crd2[f];
        for (int z = pos3[f]; z < pos3[f + 1]; ++z) {
            const int64_t k = crd3[z];
            const T v = vals[z];
#pragma unroll
            for (int r = 0; r < KB_L; ++r) acc[r] += v * C[i * a.ldC + l[r]] * D[j * a.ldD + m[r]] * E[k * ldE + n[r]];
        }
    }
    T *P = static_cast<T *>(a.partials) + (int64_t)blockIdx.x * elems;
#pragma unroll
    for (int r = 0; r < KB_L; ++r)
        if (ok[r]) P[((int64_t)blockIdx.y * KB_L + r) * NT + tid] = acc[r];
}

// A(e) = sum over chunks b of partial(b, e), in an order fixed by the launch: a workgroup owns 64 output
// elements, its four wavefronts take the chunks round robin and their sums are added in wavefront order.
// Every output element is written.
template <typename T>
__global__ void __launch_bounds__(NT) sum_partials_kernel(const T *__restrict__ partials, int nchunks, int64_t elems, T *__restrict__ out)
{
    __shared__ T part_s[NT];
    const int lane = threadIdx.x % 64, part = threadIdx.x / 64;
    const int64_t e = (int64_t)blockIdx.x * 64 + lane;
    T s = T(0);
    if (e < elems) {
#pragma unroll 4
        for (int b = part; b < nchunks; b += NT / 64) s += partials[(int64_t)b * elems + e];
    }
    part_s[threadIdx.x] = s;
    __syncthreads();
    if (part == 0 && e < elems) {
        T tot = part_s[lane];
        for (int w = 1; w < NT / 64; ++w) tot += part_s[w * 64 + lane];
        out[e] = tot;
    }
}

template <typename T>
sc_status run_ttmc_all(const sc_plan *p, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *ws, hipStream_t stream)
{
    const sc_plan *in = p->inner;
    const sc_dense_view inner_fac[2] = {fac[1], fac[2]};
    char *wsb = static_cast<char *>(ws);
    const int L = (int)p->fcols[0], M = (int)p->fcols[1], N = (int)p->fcols[2], MN = M * N;
    const int64_t elems = (int64_t)L * MN;
    Launcher ln{p, stream};
    K5Args a = {};
    a.C = fac[0].data; a.ldC = fac[0].ld;
    a.D = fac[1].data; a.ldD = fac[1].ld;
    a.L = L; a.M = M; a.N = N; a.MN = MN;
    a.partials = wsb + p->k5_partials_offset;
    a.chunk = (int32_t)p->k5_chunk;
    const dim3 grid((unsigned)p->k5_nchunks, (unsigned)((MN + NT - 1) / NT), (unsigned)((L + KB_L - 1) / KB_L));
    if (p->nnz == 0) {   // nothing stored: the output is zero
        launch_fill<T>(ln, static_cast<T *>(out), elems, "fill_output");
        return ln.status;
    }
    if (p->k5_variant == 0) {
        // the unfactored nest over all stored entries
        a.crd1 = sp->crd[0]; a.pos2 = sp->pos[1]; a.crd2 = sp->crd[1];
        a.rows = p->nfib[1];
        a.nslices = (int32_t)p->nfib[0];
        const dim3 lgrid((unsigned)p->k5_nchunks, (unsigned)((elems + (int64_t)KB_L * NT - 1) / ((int64_t)KB_L * NT)), 1);
        ln.begin("ttmc_all_linear_nest");
        linear_all_kernel<T><<<lgrid, NT, 0, stream>>>(a, sp->pos[2], sp->crd[2], static_cast<const T *>(sp->vals),
                                                       static_cast<const T *>(fac[2].data), fac[2].ld);
        ln.end();
    } else if (p->k5_variant == 1) {
        // t(f,:) per fiber by the leaf traversal of the inner plan (its first FISSIONED kernel), then the fiber reduction
        Launcher li{in, stream};
        void *T1 = wsb + p->k5_inner_ws_offset + in->inter[0].offset;
        void *partials_a = in->deterministic ? wsb + p->k5_inner_ws_offset + in->det_a.slot_offset : nullptr;
        sc_status st = launch_leaf_producer(in, li, sp->vals, fac[2], T1, N, "ttmc_all_traverse", partials_a);
        if (st != SC_OK) return st;
        st = launch_fixup(in, li, in->det_a, wsb + p->k5_inner_ws_offset, T1);
        if (st != SC_OK) return st;
        a.S = T1;
        a.crd1 = sp->crd[0]; a.pos2 = sp->pos[1]; a.crd2 = sp->crd[1];
        a.rows = p->nfib[1];
        a.nslices = (int32_t)p->nfib[0];
        ln.begin("ttmc_all_fiber_reduce");
        fiber_reduce_kernel<T><<<grid, NT, 0, stream>>>(a);
        ln.end();
    } else {
        void *S = wsb + p->k5_s_offset;
        const sc_status st = launch_plan(in, sp, inner_fac, S, wsb + p->k5_inner_ws_offset, stream);
        if (st != SC_OK) return st;
        a.S = S;
        a.rows = p->dims[0];
        if (p->k5_mfma_reduce) {
            if constexpr (sizeof(T) == 4) {
                if (MN % 64 != 0) return SC_ERR_SCHED_UNSUPPORTED;
                const dim3 mgrid((unsigned)p->k5_nchunks, (unsigned)(MN / 64), 1);
                ln.begin("ttmc_all_mode0_reduce_mfma");
                if (L == 16) mode0_reduce_mfma_kernel<1><<<mgrid, NT, 0, stream>>>(a);
                else if (L == 32) mode0_reduce_mfma_kernel<2><<<mgrid, NT, 0, stream>>>(a);
                else if (L == 64) mode0_reduce_mfma_kernel<4><<<mgrid, NT, 0, stream>>>(a);
                else if (L == 128) mode0_reduce_mfma_kernel<8><<<mgrid, NT, 0, stream>>>(a);
                else return SC_ERR_SCHED_UNSUPPORTED;
                ln.end();
            } else {
                return SC_ERR_SCHED_UNSUPPORTED;
            }
        } else {
            ln.begin("ttmc_all_mode0_reduce");
            mode0_reduce_kernel<T><<<grid, NT, 0, stream>>>(a);
            ln.end();
        }
    }
    ln.begin("ttmc_all_sum_partials");
    sum_partials_kernel<T><<<(unsigned)((elems + 63) / 64), NT, 0, stream>>>(static_cast<const T *>(a.partials), (int)p->k5_nchunks, elems,
                                                                               static_cast<T *>(out));
    ln.end();
    return ln.status;
}

}  // namespace

sc_status launch_ttmc_all(const sc_plan *p, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *ws, hipStream_t stream)
{
    if (!p->inner) return SC_ERR_SCHED_UNSUPPORTED;
    return p->dtype == SC_F64 ? run_ttmc_all<double>(p, sp, fac, out, ws, stream) : run_ttmc_all<float>(p, sp, fac, out, ws, stream);
}

}  // namespace sck
