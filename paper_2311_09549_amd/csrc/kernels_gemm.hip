// Trailing dense matrix product of kernels 8 <MTTKRP,GEMM> and 2 <SDDMM,SpMM,GEMM> of Table 2:
//     A(i,m) = sum_r P(i,r) * E(r,m)
// where P (one row per coordinate of the first mode) is what the sparse part of the nest leaves per
// slice -- the MTTKRP row, or the row of kernel 1 -- computed by an inner plan of the library into
// the workspace.  This stage is a plain dense product (I x R) * (R x M), the GEMM-shaped consumer
// of the two-level nests of Table 2 (temporary T_l, then m,l: A_im += T_l F_lm), so it runs on the
// matrix cores: v_mfma_f32_16x16x4_f32, one wavefront per 16 rows of P, all of E's columns in
// turn.  fp64, and ranks that are not multiples of the MFMA tile, take the vector-ALU kernel.
#include "device_common.h"

namespace sck {

namespace {

typedef float gemm_floatx4 __attribute__((ext_vector_type(4)));

struct GemmArgs {
    const void *P;     // I x R, row-major, leading dimension ldP
    const void *E;     // R x M, row-major, leading dimension ldE
    void *A;           // I x M, row-major, dense
    int64_t rows, ldP, ldE;
    int32_t R, M;
};

// fp32, R a multiple of 4, M a multiple of 16.  A wavefront owns rows [i0, i0 + 16); operand A of the
// MFMA is the 16 x 4 block P(i0 + col, r0 + kk), operand B the 4 x 16 block E(r0 + kk, m0 + col)
// (lane = 16 * kk + col); the lane then holds A(i0 + 4 * kk + r, m0 + col) for r = 0..3.
__global__ void __launch_bounds__(NT) rows_gemm_mfma_kernel(GemmArgs a)
{
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const int col = lane % 16, kk = lane / 16;
    const int64_t i0 = ((int64_t)blockIdx.x * (NT / 64) + wave) * 16;
    if (i0 >= a.rows) return;   // whole wavefronts leave: no barrier follows
    const float *P = static_cast<const float *>(a.P);
    const float *E = static_cast<const float *>(a.E);
    float *A = static_cast<float *>(a.A);
    const int64_t prow = min(i0 + col, a.rows - 1);   // rows past the end read a valid row and are not stored
    for (int m0 = 0; m0 < a.M; m0 += 16) {
        gemm_floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int r0 = 0; r0 < a.R; r0 += 4) {
            const float pv = P[prow * a.ldP + r0 + kk];
            const float ev = E[(int64_t)(r0 + kk) * a.ldE + m0 + col];
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(pv, ev, acc, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t i = i0 + 4 * kk + r;
            if (i < a.rows) A[i * a.M + m0 + col] = acc[r];
        }
    }
}

// Any precision and shape: a thread per output element, rows of E read through the cache.
template <typename T>
__global__ void __launch_bounds__(NT) rows_gemm_valu_kernel(GemmArgs a)
{
    const T *P = static_cast<const T *>(a.P);
    const T *E = static_cast<const T *>(a.E);
    T *A = static_cast<T *>(a.A);
    const int64_t total = a.rows * a.M;
    for (int64_t e = (int64_t)blockIdx.x * NT + threadIdx.x; e < total; e += (int64_t)gridDim.x * NT) {
        const int64_t i = e / a.M;
        const int m = (int)(e % a.M);
        T s = T(0);
        for (int r = 0; r < a.R; ++r) s += P[i * a.ldP + r] * E[(int64_t)r * a.ldE + m];
        A[e] = s;
    }
}

}  // namespace

sc_status launch_trailing_gemm(const sc_plan *p, const sc_csf_view *sp, const sc_dense_view *fac, void *out, void *ws, hipStream_t stream)
{
    const sc_plan *in = p->inner;
    if (!in) return SC_ERR_SCHED_UNSUPPORTED;
    char *wsb = static_cast<char *>(ws);
    void *P = wsb + p->tg_rows_offset;
    // the sparse part: the producer's rows, one per coordinate of the first mode (rows of empty slices are +0)
    const sc_status st = launch_plan(in, sp, fac, P, wsb + p->tg_inner_ws_offset, stream);
    if (st != SC_OK) return st;
    const int last = p->nfactors - 1;
    GemmArgs a;
    a.P = P;
    a.E = fac[last].data;
    a.A = out;
    a.rows = p->dims[0];
    a.R = (int32_t)p->fcols[last - 1];
    a.M = (int32_t)p->fcols[last];
    a.ldP = a.R;
    a.ldE = fac[last].ld;
    Launcher ln{p, stream};
    if (p->dtype == SC_F32 && a.R % 4 == 0 && a.M % 16 == 0) {
        ln.begin("trailing_gemm_mfma");
        const int64_t waves = (a.rows + 15) / 16;
        rows_gemm_mfma_kernel<<<(unsigned)((waves + NT / 64 - 1) / (NT / 64)), NT, 0, stream>>>(a);
    } else {
        ln.begin("trailing_gemm_valu");
        const int64_t total = a.rows * a.M;
        const int blocks = (int)std::min<int64_t>((total + NT - 1) / NT, (int64_t)p->n_cu * 32);
        if (p->dtype == SC_F64) rows_gemm_valu_kernel<double><<<blocks, NT, 0, stream>>>(a);
        else rows_gemm_valu_kernel<float><<<blocks, NT, 0, stream>>>(a);
    }
    ln.end();
    return ln.status;
}

}  // namespace sck
