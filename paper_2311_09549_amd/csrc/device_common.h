// Device-side helpers and launch utilities shared by the kernel files of libsparsecontract.
// Not part of the public C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>

#include "plan.h"

namespace sck {

constexpr int NT = 256;  // threads per workgroup

template <typename T, int N>
struct alignas(sizeof(T) * N) Pack {
    T v[N];
};

template <typename T>
struct VecWidth {
    static constexpr int value = 16 / (int)sizeof(T);
};

// Padded LDS index: spreads chunk starts that are a multiple of 32 words apart over banks.
__device__ __forceinline__ int pidx(int i) { return i + (i >> 5); }
__host__ __device__ constexpr int padded(int n) { return n + (n >> 5) + 1; }

template <typename T>
__device__ __forceinline__ void atomic_add(T *p, T v)
{
    atomicAdd(p, v);
}

// Largest lp in [0, np) with bnd[lp] <= x  (bnd[0] <= x < bnd[np] assumed).
__device__ __forceinline__ int find_segment(const int *bnd, int np, int x)
{
    int lo = 0, hi = np;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (bnd[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// ------------------------------------------------------------------------------------------
// fill
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(NT) fill_zero_kernel(T *__restrict__ p, int64_t n)
{
    constexpr int VEC = VecWidth<T>::value;
    const int64_t nvec = n / VEC;
    Pack<T, VEC> z;
#pragma unroll
    for (int i = 0; i < VEC; ++i) z.v[i] = T(0);
    for (int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * NT)
        reinterpret_cast<Pack<T, VEC> *>(p)[i] = z;
    for (int64_t i = nvec * VEC + (int64_t)blockIdx.x * NT + threadIdx.x; i < n; i += (int64_t)gridDim.x * NT) p[i] = T(0);
}

// Zeroes the rows of a W-wide temporary that are shared between tiles (the first node of a
// tile that continues from the previous tile), so that the tiles can add their pieces
// atomically.  `level` selects which node level the rows belong to (0 = a, 1 = b).
template <typename T>
__global__ void __launch_bounds__(NT) zero_shared_rows_kernel(const TileRec *__restrict__ tiles, int ntiles, int level,
                                                              T *__restrict__ rows, int W)
{
    const int per = NT / 64;
    const int t = blockIdx.x * per + threadIdx.x / 64;
    if (t >= ntiles) return;
    const TileRec tr = tiles[t];
    const bool shared = (tr.flags >> (2 * level)) & 1;
    if (!shared) return;
    const int64_t row = level == 0 ? tr.a0 : tr.b0;
    for (int x = threadIdx.x % 64; x < W; x += 64) rows[row * W + x] = T(0);
}

// ------------------------------------------------------------------------------------------
// segmented walk of one lane group over children [gs, ge) of a tile
//   bnd[lp] = first child (tile-local) of local parent lp; bnd[np] = child count; bnd[np+1] = INT_MAX
//   load(c)            -> Item   (issues the memory reads for child c)
//   apply(acc, item)             (adds child contribution into acc)
//   emit(lp, acc, whole)         (parent lp finished or chunk ended; `whole` = the parent lies
//                                 entirely inside this lane group's chunk)
// ------------------------------------------------------------------------------------------
template <int U, typename Acc, typename Item, typename Load, typename Apply, typename Emit>
__device__ __forceinline__ void seg_walk(int gs, int ge, const int *bnd, int np, Load load, Apply apply, Emit emit)
{
    if (gs >= ge) return;
    int lp = find_segment(bnd, np, gs);
    int pend = bnd[lp + 1];
    bool whole = bnd[lp] >= gs;
    Acc acc;
    acc.clear();
    for (int c = gs; c < ge; c += U) {
        Item it[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            it[u] = load(min(c + u, ge - 1));   // unconditional: keeps all U gathers of a batch in flight
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (c + u < ge) {
                apply(acc, it[u]);
                if (c + u + 1 == pend) {
                    emit(lp, acc, whole);
                    acc.clear();
                    whole = true;
                    ++lp;
                    pend = bnd[lp + 1];
                }
            }
    }
    if (bnd[lp] < ge) emit(lp, acc, false);
}

template <typename T, int VEC>
struct AccVec {
    T v[VEC];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = T(0);
    }
};

// ------------------------------------------------------------------------------------------
// host-side launch helpers
// ------------------------------------------------------------------------------------------
inline bool rank_ok(int64_t w, sc_dtype dt)
{
    const int vec = dt == SC_F64 ? 2 : 4;
    if (w % vec) return false;
    const int64_t lg = w / vec;
    return lg >= 1 && lg <= 64 && (lg & (lg - 1)) == 0;
}

struct Launcher {
    const sc_plan *plan;
    hipStream_t stream;
    sc_status status = SC_OK;
    bool timed() const { return plan->prof && plan->prof->on && plan->prof->n_launch < kMaxLaunches; }
    void begin(const char *name)
    {
        if (!timed()) return;
        ProfileState &pr = *plan->prof;
        pr.launch_name[pr.n_launch] = name;
        if (hipEventRecord(pr.ev_begin[pr.n_launch], stream) != hipSuccess) status = SC_ERR_DEVICE;
    }
    void end()
    {
        if (hipGetLastError() != hipSuccess) status = SC_ERR_DEVICE;
        if (!timed()) return;
        ProfileState &pr = *plan->prof;
        if (hipEventRecord(pr.ev_end[pr.n_launch], stream) != hipSuccess) status = SC_ERR_DEVICE;
        pr.n_launch++;
    }
};

template <typename T>
inline void launch_fill(Launcher &ln, T *p, int64_t n, const char *name)
{
    if (n <= 0) return;
    const int64_t nvec = (n + VecWidth<T>::value - 1) / VecWidth<T>::value;
    const int blocks = (int)std::min<int64_t>((nvec + NT - 1) / NT, (int64_t)ln.plan->n_cu * 16);
    ln.begin(name);
    fill_zero_kernel<T><<<blocks, NT, 0, ln.stream>>>(p, n);
    ln.end();
}

// Zeroes the listed rows of the output (16-byte stores; rows are a multiple of 16 bytes long).
template <typename T>
__global__ void __launch_bounds__(NT) zero_rows_kernel(const int32_t *__restrict__ rows, int64_t nvec, int vec_per_row, T *out, int64_t rowlen)
{
    constexpr int VEC = VecWidth<T>::value;
    Pack<T, VEC> z;
#pragma unroll
    for (int i = 0; i < VEC; ++i) z.v[i] = T(0);
    for (int64_t i = (int64_t)blockIdx.x * NT + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * NT) {
        const int64_t r = rows[i / vec_per_row];
        reinterpret_cast<Pack<T, VEC> *>(out + r * rowlen)[i % vec_per_row] = z;
    }
}

// First launch of every execution: the output rows that the kernels do not overwrite completely
// become zero (the rows the plan lists, or the whole output when they are many).
template <typename T>
inline void launch_output_zero(Launcher &ln, const sc_plan *p, T *out)
{
    constexpr int VEC = VecWidth<T>::value;
    if (!p->zero_selective || p->out_row_elems % VEC != 0) {
        launch_fill<T>(ln, out, p->out_elems, "fill_output");
        return;
    }
    const int vpr = (int)(p->out_row_elems / VEC);
    const int64_t nvec = (int64_t)p->zero_rows.size() * vpr;
    ln.begin("zero_output_rows");
    if (nvec > 0) {
        const int blocks = (int)std::min<int64_t>((nvec + NT - 1) / NT, (int64_t)p->n_cu * 16);
        zero_rows_kernel<T><<<blocks, NT, 0, ln.stream>>>(p->d_zero_rows, nvec, vpr, out, p->out_row_elems);
    }
    ln.end();
}

// Leaf traversal of the FISSIONED schedules of order >= 3 (its own kernel file); W = row width of
// the temporary it writes.
size_t leaf_traverse_lds_bytes(const sc_plan *p, int W);
// `partials`: deterministic schedules only (else null): slots for the pieces of rows that span tiles.
WalkShape leaf_traverse_walk_shape(sc_dtype dtype, int W);
sc_status launch_leaf_producer(const sc_plan *p, Launcher &ln, const void *vals, const sc_dense_view &F, void *Tout, int W, const char *name,
                               void *partials);

// Order-3 TTM chain on matrix cores (fp32, L = M = 16; its own kernel file): the FUSED schedule (T == nullptr)
// or the consumer kernel of the FISSIONED one.
size_t ttmc3_mfma_lds_bytes(const sc_plan *p);
WalkShape ttmc3_mfma_walk_shape();
bool ttmc3_mfma_caps_ok(const sc_plan *p);
int ttmc3_mfma_run(const sc_plan *p, bool one_tile_per_workgroup);
// `partials`: deterministic schedules only (else null): slots for the pieces of rows that span tiles.
sc_status launch_ttmc3_mfma(const sc_plan *p, Launcher &ln, const sc_csf_view *sp, const sc_dense_view *fac, const void *T, void *out,
                            void *partials);

// Last kernels of a deterministic stage: add the stored pieces of every row of the level that spans tiles
// (dst = the output for the top level, the temporary for level a).
sc_status launch_fixup(const sc_plan *p, Launcher &ln, const FixLevel &lv, void *workspace, void *dst);

// Order-4 TTM chain on matrix cores (fp32, M = N = 8, L <= 16; its own kernel file): mode 0 the FUSED schedule,
// modes 1 and 2 the second and third kernel of the FISSIONED one.
// kernels_ttmc3w.hip: order-3 chain on matrix cores for rank pairs that are multiples of 16 (other than 16 x 16), fused and
// the consumer kernel of the FISSIONED schedule
bool ttmc3_wide_ranks(int64_t L, int64_t W);
WalkShape ttmc3_wide_walk_shape(int W);
size_t ttmc3_wide_lds_bytes(const sc_plan *p);
int ttmc3_wide_run(const sc_plan *p);
sc_status launch_ttmc3_wide(const sc_plan *p, Launcher &ln, const sc_csf_view *sp, const sc_dense_view *fac, const void *T, void *out);

size_t ttmc4_mfma_lds_bytes(const sc_plan *p);
WalkShape ttmc4_mfma_walk_shape();
bool ttmc4_mfma_caps_ok(const sc_plan *p);
int ttmc4_mfma_run(const sc_plan *p, int mode, bool one_tile_per_workgroup);
sc_status launch_ttmc4_mfma(const sc_plan *p, Launcher &ln, const sc_csf_view *sp, const sc_dense_view *fac, int mode, const void *T1,
                            void *T2, void *out, void *partials);

}  // namespace sck
