// Trailing dense matrix product of kernels 8 <MTTKRP,GEMM> and 2 <SDDMM,SpMM,GEMM> of Table 2:
//     A(i,m) = sum_r P(i,r) * E(r,m)
// where P (one row per coordinate of the first mode) is what the sparse part of the nest leaves per
// slice -- the MTTKRP row, or the row of kernel 1 -- computed by an inner plan of the library into
// the workspace.  This stage is a plain dense product (I x R) * (R x M), the GEMM-shaped consumer
// of the two-level nests of Table 2 (temporary T_l, then m,l: A_im += T_l F_lm), so it runs on the
// matrix cores: v_mfma_f32_16x16x4_f32, a wavefront per block of 16 rows of P, all of E's columns in
// turn.  It moves I * (R + M) elements for 2 I R M flops, so at these ranks it is bound by memory
// traffic; what the kernel has to get right is 16-byte accesses on both sides.  fp64, and ranks
// that are not multiples of the MFMA tile, take the vector-ALU kernel.
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

// fp32, R a multiple of 16, M a multiple of 16, R * M * 4 <= 32 KB.  A wavefront owns rows [i0, i0 + 16) and
// runs over blocks of 16 rows.  The sum over r may be taken in any order, so the four k-slots of an MFMA step
// are given the four quarters of r: lane (col, kk) holds P(i0 + col, kk * R/4 + t) for t = 0 .. R/4 - 1, a
// contiguous run of its row read with 16-byte loads (the 16 rows of a block are one contiguous piece of P), and
// step t multiplies it with E(kk * R/4 + t, m0 + col), read from a copy of E in LDS.  The lane ends up with
// A(i0 + 4 * kk + r, m0 + col), r = 0..3; the four column tiles of a 64-wide output are exchanged through LDS so
// that every lane stores 16 contiguous bytes.
template <int R>
__global__ void __launch_bounds__(NT) rows_gemm_mfma_kernel(GemmArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char gemm_smem[];
    float *E_s = reinterpret_cast<float *>(gemm_smem);                    // R x M
    float *out_s = E_s + R * a.M;                                         // per wavefront 16 x M (rows padded by 4)
    constexpr int RQ = R / 4;
    const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const int col = lane % 16, kk = lane / 16;
    const float *P = static_cast<const float *>(a.P);
    const float *E = static_cast<const float *>(a.E);
    float *A = static_cast<float *>(a.A);
    for (int e = threadIdx.x; e < R * a.M; e += NT) E_s[e] = E[(int64_t)(e / a.M) * a.ldE + e % a.M];
    __syncthreads();
    const int MS = a.M + 4;
    float *my_out = out_s + wave * 16 * MS;
    const int64_t nblocks = (a.rows + 15) / 16;
    for (int64_t b = (int64_t)blockIdx.x * (NT / 64) + wave; b < nblocks; b += (int64_t)gridDim.x * (NT / 64)) {
        const int64_t i0 = b * 16;
        const int64_t prow = min(i0 + col, a.rows - 1);   // rows past the end read a valid row and are not stored
        float pv[RQ];
#pragma unroll
        for (int t = 0; t < RQ; t += 4) {
            const gemm_floatx4 v = *reinterpret_cast<const gemm_floatx4 *>(P + prow * a.ldP + kk * RQ + t);
            pv[t] = v[0]; pv[t + 1] = v[1]; pv[t + 2] = v[2]; pv[t + 3] = v[3];
        }
        for (int m0 = 0; m0 < a.M; m0 += 16) {
            gemm_floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < RQ; ++t) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(pv[t], E_s[(kk * RQ + t) * a.M + m0 + col], acc, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) my_out[(4 * kk + r) * MS + m0 + col] = acc[r];
        }
        __builtin_amdgcn_wave_barrier();
        // 16 rows x M floats leave as 16-byte pieces, consecutive lanes on consecutive pieces of a row
        const int vpr = a.M / 4;
        for (int v = lane; v < 16 * vpr; v += 64) {
            const int r = v / vpr, c4 = v % vpr;
            if (i0 + r < a.rows)
                *reinterpret_cast<gemm_floatx4 *>(A + (i0 + r) * a.M + 4 * c4) = *reinterpret_cast<const gemm_floatx4 *>(my_out + r * MS + 4 * c4);
        }
        __builtin_amdgcn_wave_barrier();
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
    const size_t lds = (size_t)a.R * a.M * 4 + (size_t)(NT / 64) * 16 * (a.M + 4) * 4;
    const bool mfma = p->dtype == SC_F32 && (a.R == 16 || a.R == 32 || a.R == 64 || a.R == 128) && a.M % 16 == 0 && lds <= 60 * 1024 &&
                      (reinterpret_cast<uintptr_t>(P) % 16) == 0;
    if (mfma) {
        ln.begin("trailing_gemm_mfma");
        const int64_t nblocks = (a.rows + 15) / 16;
        const unsigned grid = (unsigned)std::min<int64_t>((nblocks + NT / 64 - 1) / (NT / 64), (int64_t)p->n_cu * 8);
        switch (a.R) {
        case 16: rows_gemm_mfma_kernel<16><<<grid, NT, lds, stream>>>(a); break;
        case 32: rows_gemm_mfma_kernel<32><<<grid, NT, lds, stream>>>(a); break;
        case 64: rows_gemm_mfma_kernel<64><<<grid, NT, lds, stream>>>(a); break;
        default: rows_gemm_mfma_kernel<128><<<grid, NT, lds, stream>>>(a); break;
        }
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
