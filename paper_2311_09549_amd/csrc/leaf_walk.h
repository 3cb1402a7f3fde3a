// Leaf walk shared by the kernels that start from the leaf level of a CSF tile:
//     row(f,:) = sum_{z in fiber f, z in tile} vals[z] * F(crd[z],:)      (rows kept in LDS)
// the producer of a split nest (Section 3.1) at the granularity of one work tile.
//
// LDS layout the caller provides:
//   row_s    (ta + 1) rows of RS floats (leaf_row_stride: 16-byte aligned, wide rows padded so
//            that they spread over banks); the extra row absorbs the writes of the padding records
//   carry_s  one row of RS per lane group
//   rec_s    padded(tn + 8) records {factor row byte offset | end-of-fiber bit 31, value}
//   ba_s     ta + 2 ints: first nonzero (tile-local) of each fiber, ba_s[na] = nonzeros in tile
//   chunk_lr one int per lane group: fiber holding the first nonzero of the group's chunk
//
// A lane group of LG = W / VEC lanes owns a contiguous chunk of q nonzeros (q a multiple of
// U) and keeps U gathers in flight.  The walk has no branches: after every nonzero the
// running sum is written to the current fiber's row (the last write of a fiber leaves its
// sum) and a fiber end only changes registers.  A chunk that starts inside a fiber writes
// that fiber's running sum to its carry row instead.  After a barrier the group in which
// such a fiber ends adds the carry rows of the chunks the fiber passed through to the row
// (it is then the row's only writer); there are no LDS atomics, which measured several
// times slower on this chip than the extra barrier and the short serial loop.
#pragma once

#include "device_common.h"

namespace sck {

template <typename T>
struct alignas(sizeof(T) == 4 ? 8 : 16) LeafRec {
    uint32_t koff;  // byte offset of the factor row; bit 31 set when the nonzero ends its fiber
    T v;
};

// Rows of 64 bytes or more are padded by 16 bytes, which spreads consecutive rows over the
// LDS banks; narrower rows are packed.
template <typename T>
__host__ __device__ constexpr int leaf_row_stride(int W)
{
    return W + (W * (int)sizeof(T) >= 64 ? 16 / (int)sizeof(T) : 0);
}

// LDS bytes of row_s + carry_s + rec_s + ba_s + chunk_lr for a workgroup of `nthreads`.
template <typename T>
__host__ __device__ constexpr size_t leaf_walk_lds_bytes(int W, int tn, int ta, int nthreads)
{
    const int groups = nthreads / (W / (16 / (int)sizeof(T)));
    return (size_t)(ta + 1 + groups) * leaf_row_stride<T>(W) * sizeof(T) + (size_t)padded(tn + 8) * sizeof(LeafRec<T>) +
           (size_t)(ta + 2) * 4 + (size_t)groups * 4;
}

// Nonzeros per lane group for a tile of `nchild` nonzeros: a multiple of U.
template <int U>
__device__ __forceinline__ int leaf_chunk(int nchild, int groups)
{
    return walk_chunk(nchild, groups, U);
}

// Marks fiber ends in the records and notes the fiber at the head of every chunk.  Runs
// after the records and ba_s are in LDS (barrier before and after).
template <typename T>
__device__ __forceinline__ void leaf_mark(LeafRec<T> *rec_s, const int *ba_s, int *chunk_lr, int tid, int nthreads, int na, int q)
{
    for (int i = tid; i < na; i += nthreads) {
        const int lo = ba_s[i], hi = ba_s[i + 1];
        if (hi <= lo) continue;   // cannot happen: a tile lists only nodes with leaves inside it
        rec_s[pidx(hi - 1)].koff |= 0x80000000u;
        for (int m = (lo + q - 1) / q; m * q < hi; ++m) chunk_lr[m] = i;
    }
}

// What a lane group remembers between the walk and the combine step.
struct LeafCarry {
    int lr0;      // fiber at the head of the chunk
    bool head;    // that fiber began in an earlier chunk
    bool owner;   // ... and ends in this chunk (or the tile ends inside it): this group sums it
};

template <typename T, int W, int U>
__device__ __forceinline__ LeafCarry leaf_walk(T *row_s, T *carry_s, const LeafRec<T> *rec_s, const int *ba_s, const int *chunk_lr,
                                               const void *F, int g, int li, int q, int nchild)
{
    constexpr int VEC = VecWidth<T>::value;
    constexpr int RS = leaf_row_stride<T>(W);
    using P = Pack<T, VEC>;
    LeafCarry st{0, false, false};
    const int gs = g * q, ge = min(gs + q, nchild);
    if (gs >= ge) return st;
    const char *Fb = static_cast<const char *>(F);
    const uint32_t lo16 = (uint32_t)li * 16u;
    st.lr0 = chunk_lr[g];
    st.head = ba_s[st.lr0] != gs;
    T *rowp = row_s + st.lr0 * RS + li * VEC;
    T *const row0 = rowp;
    T *dst = st.head ? carry_s + g * RS + li * VEC : rowp;
    T acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = T(0);
    for (int c = gs; c < ge; c += U) {
        LeafRec<T> r[U];
        P d[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = rec_s[pidx(c + u)];
#pragma unroll
        for (int u = 0; u < U; ++u) d[u] = *reinterpret_cast<const P *>(Fb + ((r[u].koff & 0x7fffffffu) + lo16));
#pragma unroll
        for (int u = 0; u < U; ++u) {
            P o;
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                acc[i] += r[u].v * d[u].v[i];
                o.v[i] = acc[i];
            }
            *reinterpret_cast<P *>(dst) = o;
            const bool end = (int32_t)r[u].koff < 0;
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = end ? T(0) : acc[i];
            rowp = end ? rowp + RS : rowp;
            dst = end ? rowp : dst;
        }
    }
    // the head fiber ended here if the row pointer moved; a fiber still open at the tile's
    // last nonzero "ends" there as far as this tile goes
    st.owner = st.head && (rowp != row0 || ge == nchild);
    return st;
}

// After a barrier: the owner adds the carry rows of the chunks its head fiber passed through.
template <typename T, int W>
__device__ __forceinline__ void leaf_combine(T *row_s, const T *carry_s, const int *ba_s, const int *chunk_lr, const LeafCarry &st, int g,
                                             int li, int q)
{
    constexpr int VEC = VecWidth<T>::value;
    constexpr int RS = leaf_row_stride<T>(W);
    using P = Pack<T, VEC>;
    if (!st.owner) return;
    const int start = ba_s[st.lr0];
    P sum = *reinterpret_cast<const P *>(carry_s + g * RS + li * VEC);
    // chunks g-1, g-2, ... that begin after the fiber's first nonzero lie entirely inside it
    for (int h = g - 1; h >= 0 && h * q > start; --h) {
        const P c = *reinterpret_cast<const P *>(carry_s + h * RS + li * VEC);
#pragma unroll
        for (int i = 0; i < VEC; ++i) sum.v[i] += c.v[i];
    }
    T *dst = row_s + st.lr0 * RS + li * VEC;
    const P base = *reinterpret_cast<const P *>(dst);   // the piece written by the chunk in which the fiber starts
#pragma unroll
    for (int i = 0; i < VEC; ++i) sum.v[i] += base.v[i];
    *reinterpret_cast<P *>(dst) = sum;
}

// ---- the same walk driven by the plan's walk tables ----
// The records already carry the end-of-fiber bits (the plan's copy of the coordinates has them, and
// the stage sets the bit of the tile's last nonzero), and chunk_s holds, per lane group, the plan's
// entry for the tile: row of the fiber at the head of the chunk | bit 15 when that fiber began in an
// earlier chunk.  No fiber bounds are staged and nothing is marked at run time.  After its walk a
// group replaces its entry by the same word with bit 16 set when a fiber ended inside the chunk;
// the combine step reads the entries of the chunks before its own to find the carry rows that
// belong to its head fiber: those of the chunks that began inside the fiber and saw no end.
constexpr uint32_t kChunkHead = 0x8000u, kChunkEnded = 0x10000u, kChunkRow = 0x7fffu;

template <typename T, int W, int U>
__device__ __forceinline__ uint32_t table_walk(T *row_s, T *carry_s, const LeafRec<T> *rec_s, uint32_t *chunk_s, const void *F, int g, int li,
                                               int q, int nchild)
{
    constexpr int VEC = VecWidth<T>::value;
    constexpr int RS = leaf_row_stride<T>(W);
    using P = Pack<T, VEC>;
    const int gs = g * q, ge = min(gs + q, nchild);
    if (gs >= ge) return 0;
    const char *Fb = static_cast<const char *>(F);
    const uint32_t lo16 = (uint32_t)li * 16u;
    const uint32_t entry = chunk_s[g];
    const bool head = (entry & kChunkHead) != 0;
    T *rowp = row_s + (entry & kChunkRow) * RS + li * VEC;
    T *const row0 = rowp;
    T *dst = head ? carry_s + g * RS + li * VEC : rowp;
    T acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = T(0);
    for (int c = gs; c < ge; c += U) {
        LeafRec<T> r[U];
        P d[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = rec_s[pidx(c + u)];
#pragma unroll
        for (int u = 0; u < U; ++u) d[u] = *reinterpret_cast<const P *>(Fb + ((r[u].koff & 0x7fffffffu) + lo16));
#pragma unroll
        for (int u = 0; u < U; ++u) {
            P o;
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                acc[i] += r[u].v * d[u].v[i];
                o.v[i] = acc[i];
            }
            *reinterpret_cast<P *>(dst) = o;
            const bool end = (int32_t)r[u].koff < 0;
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = end ? T(0) : acc[i];
            rowp = end ? rowp + RS : rowp;
            dst = end ? rowp : dst;
        }
    }
    const uint32_t done = entry | (rowp != row0 ? kChunkEnded : 0u);
    if (li == 0) chunk_s[g] = done;
    return done;
}

// After a barrier: the group in which a head fiber ends adds the carry rows of the chunks the fiber
// passed through to the fiber's row (it is then the row's only writer).
template <typename T, int W>
__device__ __forceinline__ void table_combine(T *row_s, const T *carry_s, const uint32_t *chunk_s, uint32_t done, int g, int li)
{
    constexpr int VEC = VecWidth<T>::value;
    constexpr int RS = leaf_row_stride<T>(W);
    using P = Pack<T, VEC>;
    if ((done & (kChunkHead | kChunkEnded)) != (kChunkHead | kChunkEnded)) return;
    P sum = *reinterpret_cast<const P *>(carry_s + g * RS + li * VEC);
    for (int h = g - 1; h >= 0; --h) {
        const uint32_t e = chunk_s[h];
        // a chunk in which a fiber ended, or which began with the fiber, wrote its piece to the row itself
        if ((e & (kChunkHead | kChunkEnded)) != kChunkHead) break;
        const P c = *reinterpret_cast<const P *>(carry_s + h * RS + li * VEC);
#pragma unroll
        for (int i = 0; i < VEC; ++i) sum.v[i] += c.v[i];
    }
    T *dst = row_s + (done & kChunkRow) * RS + li * VEC;
    const P base = *reinterpret_cast<const P *>(dst);   // the piece written by the chunk in which the fiber starts
#pragma unroll
    for (int i = 0; i < VEC; ++i) sum.v[i] += base.v[i];
    *reinterpret_cast<P *>(dst) = sum;
}

}  // namespace sck
