// Order-4 TTM chain on matrix cores, fp32, M = N = 8, L <= 16; MODE 0 is the FUSED schedule in one
// kernel, MODE 1 and 2 are the second and third kernel of the FISSIONED schedule (T1 rows read from
// the workspace and T2 rows written to it; T2 rows read from the workspace):
//     A(i,l,m,n) = sum_{j,k,p} B(i,j,k,p) * C(j,l) * D(k,m) * E(p,n)
// under the two-level nest obtained by applying the split-and-fuse step of Section 4.2 twice
// (the shape of the second schedule of Table 2, kernel 5):
//     T1(f3, n)    = sum_{p' in f3} B * E(p, n)              f3 = (i,j,k) fiber
//     T2(f2, m, n) = sum_{f3 in f2} D(k, m) * T1(f3, n)      f2 = (i,j) fiber
//     A(i, l, m, n) = sum_{f2 in slice i} C(j, l) * T2(f2, m, n)
// Both temporaries live in LDS for the nodes of one tile.
//
//   stage    every global read of the tile is issued before the first is used; the coordinates of
//            the two walked levels come from the plan's walk tables, with the end-of-fiber bits in
//            them, as do the fibers at the heads of the lane groups' chunks: no fiber bounds are
//            read and nothing is marked at run time
//   leaves   the shared branch-free leaf walk with 8-wide rows (2 lanes per nonzero) -> T1 rows
//   middle   the same walk one level up: children are the f3 fibers (their T1 row comes from
//            LDS, the D row is gathered), a group of 16 lanes owns a chunk of children and
//            keeps the 64-wide running sum of the current f2 fiber -> T2 rows
//   consume  A(i, l, mn) = sum_f2 T2(f2, mn) * C(j, l): wavefront w owns the 16 columns
//            mn = 16 w .. 16 w + 15 for every slice of the tile (four f2 fibers per
//            v_mfma_f32_16x16x4_f32, l padded to 16), so no sums cross wavefronts; a lane ends
//            up with four consecutive mn of one l, i.e. one 16-byte store
//   carry    a workgroup owns a contiguous run of tiles; the sum of a slice that continues
//            into the next tile stays in registers, so a heavy slice costs one global update
//            per workgroup; only a slice that crosses the run's ends is added atomically to
//            the zeroed output
#include <type_traits>

#include "leaf_walk.h"

namespace sck {

struct Ttmc4Args {
    const int32_t *crd1, *pos2, *crd2;
    const uint32_t *rec3, *rec4;   // the plan's walk tables: coordinates of the f3 fibers / of the nonzeros | end-of-parent bit 31
    const uint16_t *heads;         // per tile: T4_G1 chunk heads of the leaf walk, then T4_G2 of the middle walk
    int32_t heads_per_tile;
    const float *vals;
    const float *C, *D, *E;
    int64_t ldC, ldD, ldE;
    const float *T1;   // MODE 1: materialised T1, one 8-wide row per f3 fiber
    float *T2;         // MODE 1 writes, MODE 2 reads: one 64-wide row per f2 fiber
    float *A;
    float *partials;   // deterministic schedules: slots for the pieces of rows that span tiles (runs are single tiles then), else null
    const int32_t *slot_b;   // deterministic MODE 1: first slot of each tile's pieces of T2 rows
    int32_t L;
    int32_t tn, ta, tb;
    int32_t ntiles, run;   // tiles in the plan; tiles per workgroup
};

constexpr int T4_N = 8, T4_M = 8, T4_W2 = T4_M * T4_N;
constexpr int T4_RS1 = leaf_row_stride<float>(T4_N);
constexpr int T4_RS2 = leaf_row_stride<float>(T4_W2);
constexpr int T4_G1 = NT / (T4_N / 4);     // lane groups of the leaf walk (2 lanes each)
constexpr int T4_LG2 = T4_W2 / 4;          // lanes per T2 row
constexpr int T4_G2 = NT / T4_LG2;         // lane groups of the middle walk
constexpr int T4_U1 = 4, T4_U2 = 4;          // children a lane group of the leaf / middle walk takes per step
constexpr int T4_MAXR = 3;                 // tn <= T4_MAXR * NT
constexpr int T4_MAXA = 2;                 // ta + 1 <= T4_MAXA * NT, tb + 1 <= NT
constexpr int T4_TR1 = 3;                  // MODE 1: T1 rows copied per 2-lane group, ta <= T4_TR1 * G1
constexpr int T4_TR2 = 5;                  // MODE 2: T2 rows copied per 16-lane group, tb <= T4_TR2 * G2
static_assert(NT / 64 == T4_W2 / 16, "one wavefront per 16 columns of a T2 row");

// What the leaf stage needs besides the T1 rows (carry rows, nonzero records, fiber bounds,
// chunk heads) is dead before the first T2 row is written, and shares its space with the T2
// rows.  The kernel is bound by latency and its time falls almost in proportion to the
// workgroups that fit a compute unit, so LDS bytes are what to save.
__host__ __device__ constexpr size_t ttmc4_leaf_scratch_bytes(int tn, int ta)
{
    return (size_t)T4_G1 * T4_RS1 * 4 + (size_t)padded(tn + 8) * sizeof(LeafRec<float>) + (size_t)T4_G1 * 4;
}

__host__ __device__ constexpr size_t ttmc4_shared_bytes(int tn, int ta, int tb)
{
    const size_t leaf = ttmc4_leaf_scratch_bytes(tn, ta);
    const size_t rows2 = (size_t)(tb + 1 + T4_G2) * T4_RS2 * 4;
    return ((leaf > rows2 ? leaf : rows2) + 15) / 16 * 16;
}

// The third kernel of the FISSIONED schedule (mode 2) reads finished T2 rows and has no T1 rows.
__host__ __device__ constexpr size_t ttmc4_lds_bytes(int tn, int ta, int tb, int mode = 0)
{
    return (size_t)(mode == 2 ? 0 : (ta + 1) * T4_RS1 * 4) + ttmc4_shared_bytes(tn, ta, tb) + (size_t)(ta + 4) * 4 + (size_t)T4_G2 * 4 +
           (size_t)tb * 4 + (size_t)(tb + 2) * 4 + (size_t)tb * 4 + 64;
}

typedef float t4_floatx4 __attribute__((ext_vector_type(4)));

// DET: the deterministic variants (pieces of rows that span tiles go to plan-numbered slots: rows of A in
// MODE 0 and 2, rows of T2 in MODE 1).
template <int MODE, bool DET>
__global__ void __launch_bounds__(NT) ttmc4_mfma_kernel(Ttmc4Args a, const TileRec *__restrict__ tiles)
{
    using P = Pack<float, 4>;
    using Rec = LeafRec<float>;
    constexpr int U1 = T4_U1, U2 = T4_U2;
    constexpr int RS1 = T4_RS1, RS2 = T4_RS2;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *row1_s = reinterpret_cast<float *>(smem);                          // (ta + 1) rows of RS1: T1
    unsigned char *shared_s = reinterpret_cast<unsigned char *>(row1_s + (MODE == 2 ? (size_t)0 : (size_t)(a.ta + 1) * RS1));
    // leaf stage (dead once the T1 rows are complete) ...
    float *carry1_s = reinterpret_cast<float *>(shared_s);                    // G1 rows of RS1
    Rec *rec_s = reinterpret_cast<Rec *>(carry1_s + (size_t)T4_G1 * RS1);     // padded(tn + 8)
    uint32_t *chunk1_s = reinterpret_cast<uint32_t *>(rec_s + padded(a.tn + 8));   // G1: chunk heads of the leaf walk
    // ... and, in the same space, what the middle walk and the consumer use
    float *row2_s = reinterpret_cast<float *>(shared_s);                      // (tb + 1) rows of RS2: T2
    float *carry2_s = row2_s + (size_t)(a.tb + 1) * RS2;                      // G2 rows of RS2
    uint32_t *krec_s = reinterpret_cast<uint32_t *>(shared_s + ttmc4_shared_bytes(a.tn, a.ta, a.tb));   // ta + 4: D row offset of each f3 | end-of-f2 bit 31
    uint32_t *chunk2_s = krec_s + a.ta + 4;                                   // G2: chunk heads of the middle walk
    uint32_t *coff2_s = chunk2_s + T4_G2;                                     // tb: byte offset of C(j,:) per f2
    int *bc_s = reinterpret_cast<int *>(coff2_s + a.tb);                      // tb + 2: first f2 of each slice
    int *crdc_s = bc_s + a.tb + 2;                                            // tb: output row of each slice

    const int tid = threadIdx.x;
    const int L = a.L;
    const int rowA = L * T4_W2;
    const uint32_t rowE = (uint32_t)(a.ldE * 4), rowD = (uint32_t)(a.ldD * 4), rowC = (uint32_t)(a.ldC * 4);
    const int first = blockIdx.x * a.run, lastp1 = min(first + a.run, a.ntiles);
    auto uni = [](int x) { return __builtin_amdgcn_readfirstlane(x); };
    const int wave = uni(tid / 64), lane = tid % 64;
    const int kk = lane / 16, col = lane % 16;
    t4_floatx4 carry = {0.f, 0.f, 0.f, 0.f};   // this wavefront's columns of the slice continuing from the previous tile
    bool chain_shared = false;                 // that slice began before this workgroup's run

    // Global reads of one tile's staging, held in registers: they are issued while the previous
    // tile of the run is still being worked on.
    struct Stage {
        uint32_t pp[T4_MAXR];
        float vv[T4_MAXR];
        uint32_t k3[T4_MAXA];
        int j2, p2, i1;
        uint32_t hd;
        P t1row[MODE == 1 ? T4_TR1 : 1], t2row[MODE == 2 ? T4_TR2 : 1];
    };
    auto issue = [&](const TileRec &t, int tile, Stage &s) {
        const int nchild = t.n1 - t.n0;
        const int na = t.na, nb = t.nb, nc = t.nc;
        if (MODE == 0) {
#pragma unroll
            for (int r = 0; r < T4_MAXR; ++r) {
                const int c = t.n0 + min(tid + r * NT, nchild - 1);
                s.pp[r] = a.rec4[c];
                s.vv[r] = a.vals[c];
            }
        }
        if (MODE != 2) {
#pragma unroll
            for (int r = 0; r < T4_MAXA; ++r) s.k3[r] = a.rec3[t.a0 + min(tid + r * NT, na - 1)];
            s.hd = a.heads[(int64_t)tile * a.heads_per_tile + min(tid, T4_G1 + T4_G2 - 1)];
        }
        if (MODE != 1) {
            s.j2 = a.crd2[t.b0 + min(tid, nb - 1)];
            s.p2 = a.pos2[t.c0 + min(tid, nc)];
            s.i1 = a.crd1[t.c0 + min(tid, nc - 1)];
        }
        if (MODE == 1) {
#pragma unroll
            for (int r = 0; r < T4_TR1; ++r) {
                const int f = min(tid / 2 + r * T4_G1, na - 1);
                s.t1row[r] = *reinterpret_cast<const P *>(a.T1 + (int64_t)(t.a0 + f) * T4_N + (tid % 2) * 4);
            }
        }
        if (MODE == 2) {
#pragma unroll
            for (int r = 0; r < T4_TR2; ++r) {
                const int f = min(tid / T4_LG2 + r * T4_G2, nb - 1);
                s.t2row[r] = *reinterpret_cast<const P *>(a.T2 + (int64_t)(t.b0 + f) * T4_W2 + (tid % T4_LG2) * 4);
            }
        }
    };
    TileRec t = tiles[first];   // a launched workgroup has at least one tile
    Stage st;
    issue(t, first, st);

    for (int tile = first; tile < lastp1; ++tile) {
        const TileRec tn = tiles[min(tile + 1, lastp1 - 1)];
        const bool in_f = (t.flags & 16) != 0, out_f = (t.flags & 32) != 0;
        if (tile == first && in_f) chain_shared = true;
        const int nchild = t.n1 - t.n0;
        const int na = t.na, nb = t.nb, nc = t.nc;
        const int q1 = leaf_chunk<U1>(nchild, T4_G1);
        const int q2 = leaf_chunk<U2>(na, T4_G2);

        // ---- stage: registers -> LDS ----
        {
            const uint32_t(&pp)[T4_MAXR] = st.pp;
            const float(&vv)[T4_MAXR] = st.vv;
            const uint32_t(&k3)[T4_MAXA] = st.k3;
            const int j2 = st.j2, p2 = st.p2, i1 = st.i1;
            const auto &t1row = st.t1row;
            const auto &t2row = st.t2row;
            if (MODE == 0) {
#pragma unroll
                for (int r = 0; r < T4_MAXR; ++r) {
                    const int c = tid + r * NT;
                    if (c < nchild) {
                        Rec rec;
                        // the tile's last nonzero closes the fiber it is in as far as this tile goes
                        rec.koff = (pp[r] & 0x7fffffffu) * rowE | (pp[r] & 0x80000000u) | (c == nchild - 1 ? 0x80000000u : 0u);
                        rec.v = vv[r];
                        rec_s[pidx(c)] = rec;
                    }
                }
                if (tid < U1) {  // dummies completing the last batch of the leaf walk
                    Rec rec;
                    rec.koff = 0;
                    rec.v = 0.f;
                    rec_s[pidx(nchild + tid)] = rec;
                }
                if (tid < T4_G1) chunk1_s[tid] = st.hd;
            }
            // A node cut by a tile boundary has one complete row in the workspace; the tile in
            // which it starts consumes it, the tiles it continues into see a zero row.
            if (MODE == 1) {
#pragma unroll
                for (int r = 0; r < T4_TR1; ++r) {
                    const int f = tid / 2 + r * T4_G1;
                    if (f < na) {
                        P v = t1row[r];
                        if (f == 0 && (t.flags & 1)) v = P{{0.f, 0.f, 0.f, 0.f}};
                        *reinterpret_cast<P *>(row1_s + f * RS1 + (tid % 2) * 4) = v;
                    }
                }
            }
            if (MODE == 2) {
#pragma unroll
                for (int r = 0; r < T4_TR2; ++r) {
                    const int f = tid / T4_LG2 + r * T4_G2;
                    if (f < nb) {
                        P v = t2row[r];
                        if (f == 0 && (t.flags & 4)) v = P{{0.f, 0.f, 0.f, 0.f}};
                        *reinterpret_cast<P *>(row2_s + f * RS2 + (tid % T4_LG2) * 4) = v;
                    }
                }
            }
            if (MODE != 2) {
#pragma unroll
                for (int r = 0; r < T4_MAXA; ++r) {
                    const int i = tid + r * NT;
                    if (i < na) krec_s[i] = (k3[r] & 0x7fffffffu) * rowD | (k3[r] & 0x80000000u) | (i == na - 1 ? 0x80000000u : 0u);
                }
                if (tid < U2) krec_s[na + tid] = 0;   // dummies of the middle walk
                if (tid >= T4_G1 && tid < T4_G1 + T4_G2) chunk2_s[tid - T4_G1] = st.hd;
            }
            if (MODE != 1) {
                if (tid < nb) coff2_s[tid] = (uint32_t)j2 * rowC;
                if (tid <= nc) bc_s[tid] = min(max(p2, t.b0), t.b0 + nb) - t.b0;
                if (tid < nc) crdc_s[tid] = i1;
            }
        }
        __syncthreads();

        // ---- the next tile's reads go out now and land while this tile is worked on ----
        Stage sn;
        if (tile + 1 < lastp1) issue(tn, tile + 1, sn);
        // FUSED: the C rows of the tile's f2 fibers are fetched ahead of the consumer (16 lanes per row, rows
        // tid / 16 + 16 r; their offsets are in LDS by now) and are parked in the space of the T1 rows as soon
        // as those are dead.  The consumer then reads both operands of its MFMAs from LDS instead of gathering
        // C in its inner loop, where the gather's latency was paid once per block of fibers.
        const bool c_in_lds = MODE == 0 && (a.tb + 15) * 16 <= (a.ta + 1) * RS1;   // 15 rows of slack: the consumer reads past a slice's last fiber
        float cval[T4_TR2];
        if (c_in_lds) {
            const char *Cl = reinterpret_cast<const char *>(a.C) + min(tid % 16, L - 1) * 4;
#pragma unroll
            for (int r = 0; r < T4_TR2; ++r) cval[r] = *reinterpret_cast<const float *>(Cl + coff2_s[min(tid / 16 + r * T4_G2, nb - 1)]);
        }

        // ---- leaves -> T1 rows ----
        if (MODE == 0) {
            const int g = tid / 2, li = tid % 2;
            const uint32_t done = table_walk<float, T4_N, U1>(row1_s, carry1_s, rec_s, chunk1_s, a.E, g, li, q1, nchild);
            __syncthreads();
            table_combine<float, T4_N>(row1_s, carry1_s, chunk1_s, done, g, li);
            __syncthreads();
        }

        // ---- f3 fibers -> T2 rows: T2(f2, m, :) += D(k, m) * T1(f3, :) ----
        if (MODE != 2) {
            const int g = tid / T4_LG2, li = tid % T4_LG2;
            const int m = li / 2, nq = (li % 2) * 4;
            const char *Db = reinterpret_cast<const char *>(a.D) + m * 4;
            uint32_t done = 0;
            const int gs = g * q2, ge = min(gs + q2, na);
            if (gs < ge) {
                const uint32_t entry = chunk2_s[g];
                float *rowp = row2_s + (entry & kChunkRow) * RS2 + li * 4;
                float *const row0 = rowp;
                float *dst = (entry & kChunkHead) ? carry2_s + g * RS2 + li * 4 : rowp;
                float acc[4] = {0.f, 0.f, 0.f, 0.f};
                for (int c = gs; c < ge; c += U2) {
                    uint32_t kr[U2];
                    P t1[U2];
                    float d[U2];
#pragma unroll
                    for (int u = 0; u < U2; ++u) {
                        kr[u] = krec_s[c + u];
                        t1[u] = *reinterpret_cast<const P *>(row1_s + (c + u) * RS1 + nq);
                    }
#pragma unroll
                    for (int u = 0; u < U2; ++u) d[u] = *reinterpret_cast<const float *>(Db + (kr[u] & 0x7fffffffu));
#pragma unroll
                    for (int u = 0; u < U2; ++u) {
                        P o;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            acc[i] += d[u] * t1[u].v[i];
                            o.v[i] = acc[i];
                        }
                        *reinterpret_cast<P *>(dst) = o;
                        const bool end = (int32_t)kr[u] < 0;
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[i] = end ? 0.f : acc[i];
                        rowp = end ? rowp + RS2 : rowp;
                        dst = end ? rowp : dst;
                    }
                }
                done = entry | (rowp != row0 ? kChunkEnded : 0u);
                if (li == 0) chunk2_s[g] = done;
            }
            __syncthreads();
            if (c_in_lds) {   // the T1 rows are dead: their space takes the C rows (l >= L padded with zeros)
                const int l = tid % 16;
#pragma unroll
                for (int r = 0; r < T4_TR2; ++r) {
                    const int f = tid / 16 + r * T4_G2;
                    if (f < nb) row1_s[f * 16 + l] = l < L ? cval[r] : 0.f;
                }
            }
            table_combine<float, T4_W2>(row2_s, carry2_s, chunk2_s, done, g, li);
            __syncthreads();
        }

        if (MODE == 1) {
            // write the tile's T2 rows; rows shared with a neighbouring tile are added atomically to
            // pre-zeroed memory
            const int g = tid / T4_LG2, li = tid % T4_LG2;
            float *Tg = a.T2 + (int64_t)t.b0 * T4_W2;
            for (int r = g; r < nb; r += T4_G2) {
                const P row = *reinterpret_cast<const P *>(row2_s + r * RS2 + li * 4);
                float *dst = Tg + (int64_t)r * T4_W2 + li * 4;
                const bool shared = (r == 0 && (t.flags & 4)) || (r == nb - 1 && (t.flags & 8));
                if (!shared) {
                    // written once, read by the next kernel only: non-temporal
                    __builtin_nontemporal_store(__builtin_bit_cast(t4_floatx4, row), reinterpret_cast<t4_floatx4 *>(dst));
                } else if (DET) {
                    // the piece of the tile's first node is numbered slot_b[tile], that of its last node follows
                    const int slot = a.slot_b[tile] + ((r == 0 && (t.flags & 4)) ? 0 : ((t.flags & 4) >> 2));
                    *reinterpret_cast<P *>(a.partials + (int64_t)slot * T4_W2 + li * 4) = row;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) atomic_add(dst + i, row.v[i]);
                }
            }
        }

        // ---- consume: T2 rows x gathered C rows -> A ----
        if (MODE != 1) {
            const bool lval = col < L;
            const char *Cb = reinterpret_cast<const char *>(a.C) + min(col, L - 1) * 4;
            const bool last_tile = tile + 1 == lastp1;
            auto emit = [&](const t4_floatx4 &v, int ls, bool atomic) {
                // v[r] = A(l = col, mn = 16 wave + 4 kk + r)
                if (!lval) return;
                float *dst = a.A + (int64_t)uni(crdc_s[ls]) * rowA + col * T4_W2 + wave * 16 + 4 * kk;
                if (!atomic) {
                    *reinterpret_cast<t4_floatx4 *>(dst) = v;
                } else if (DET) {
                    // deterministic: this tile's piece of the row goes to its slot (a tile whose only
                    // slice continues on both sides has one piece, numbered as its first)
                    const int slot = (ls == 0 && in_f) ? t.pad[0] : t.pad[1];
                    *reinterpret_cast<t4_floatx4 *>(a.partials + (int64_t)slot * rowA + col * T4_W2 + wave * 16 + 4 * kk) = v;
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) atomic_add(dst + r, v[r]);
                }
            };
            // the loop is compiled once per source of the C rows: with a run-time choice inside it the two reads
            // merge into one generic-address load, whose wait also covers every global read in flight
            auto slices = [&](auto c_rows_in_lds) {
                constexpr bool CL = decltype(c_rows_in_lds)::value;
                for (int ls = 0; ls < nc; ++ls) {
                    const int f0 = uni(bc_s[ls]), f1 = uni(bc_s[ls + 1]);
                    t4_floatx4 acc = {0.f, 0.f, 0.f, 0.f};
                    constexpr int UB = 4;   // 4-fiber blocks whose operand reads are issued together
                    for (int fb = f0; fb < f1; fb += 4 * UB) {
                        float cv[UB], tv[UB];
                        if (CL) {
                            // both operands at fixed distances from one address per lane: lanes past the slice read
                            // rows of the next slice or unused rows of the same arrays, and both values are dropped
                            const float *t2p = row2_s + (fb + kk) * RS2 + wave * 16 + col;
                            const float *c1p = row1_s + (fb + kk) * 16 + col;
#pragma unroll
                            for (int ub = 0; ub < UB; ++ub) {
                                const bool in_slice = fb + 4 * ub + kk < f1;
                                const float tvr = t2p[ub * 4 * RS2], cvr = c1p[ub * 64];
                                tv[ub] = in_slice ? tvr : 0.f;
                                cv[ub] = in_slice ? cvr : 0.f;   // rows l >= L of C are zeros in LDS
                            }
                        } else {
#pragma unroll
                            for (int ub = 0; ub < UB; ++ub) {
                                const int lf = fb + 4 * ub + kk;
                                const int lfc = min(lf, f1 - 1);   // lanes past the slice read a valid fiber and are zeroed
                                const float tvr = row2_s[lfc * RS2 + wave * 16 + col];
                                const float cvr = *reinterpret_cast<const float *>(Cb + coff2_s[lfc]);
                                tv[ub] = lf < f1 ? tvr : 0.f;
                                cv[ub] = lval ? cvr : 0.f;
                            }
                        }
#pragma unroll
                        for (int ub = 0; ub < UB; ++ub)
                            if (fb + 4 * ub < f1) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(tv[ub], cv[ub], acc, 0, 0, 0);
                    }
                    const bool incoming = ls == 0 && in_f, outgoing = ls == nc - 1 && out_f;
                    if (incoming) acc += carry;
                    if (outgoing) {
                        if (last_tile) emit(acc, ls, true);   // continues in another workgroup's run
                        else carry = acc;
                    } else {
                        emit(acc, ls, incoming && chain_shared);
                        if (incoming) chain_shared = false;
                    }
                }
            };
            if (MODE == 0 && c_in_lds) slices(std::true_type{});
            else slices(std::false_type{});
        }
        __syncthreads();
        if (tile + 1 < lastp1) {
            t = tn;
            st = sn;
        }
    }  // tiles of the run
}

WalkShape ttmc4_mfma_walk_shape()
{
    WalkShape w;
    w.levels = 2;
    w.groups[0] = T4_G1; w.groups[1] = T4_G2;
    w.batch[0] = T4_U1; w.batch[1] = T4_U2;
    return w;
}

size_t ttmc4_mfma_lds_bytes(const sc_plan *p) { return ttmc4_lds_bytes(p->caps.tn, p->caps.ta, p->caps.tb); }

bool ttmc4_mfma_caps_ok(const sc_plan *p)
{
    return p->caps.tn <= T4_MAXR * NT && p->caps.ta + 1 <= T4_MAXA * NT && p->caps.ta <= T4_TR1 * T4_G1 && p->caps.tb <= T4_TR2 * T4_G2 &&
           p->caps.tb >= 1;
}

// Tiles per workgroup.  Several runs per resident workgroup slot: shorter runs even out the tiles' different costs,
// longer ones save row updates; six per slot measured best for the fused kernel (24 per compute unit), 32 per compute
// unit for the two kernels of the FISSIONED schedule.  A deterministic schedule takes one tile per workgroup, so that
// the pieces are the ones the plan numbered.
int ttmc4_mfma_run(const sc_plan *p, int mode, bool one_tile_per_workgroup)
{
    const int ntiles = (int)p->tiles.size();
    if (ntiles == 0 || one_tile_per_workgroup) return 1;
    const int fit = lds_workgroups_per_cu(ttmc4_lds_bytes(p->caps.tn, p->caps.ta, p->caps.tb, mode), p->lds_per_cu);
    const int per_cu = p->tune.per_cu > 0 ? std::min(p->tune.per_cu, 64) : (mode == 0 ? 6 * fit : 32);
    const int want = std::min(ntiles, p->n_cu * per_cu);
    return (ntiles + want - 1) / want;
}

sc_status launch_ttmc4_mfma(const sc_plan *p, Launcher &ln, const sc_csf_view *sp, const sc_dense_view *fac, int mode, const void *T1,
                            void *T2, void *out, void *partials)
{
    // mode 0: FUSED schedule; 1: T1 -> T2 and 2: T2 -> A of the FISSIONED schedule
    const int ntiles = (int)p->tiles.size();
    if (ntiles == 0) return SC_OK;
    if (!ttmc4_mfma_caps_ok(p) || p->fcols[0] > 16 || p->fcols[1] != T4_M || p->fcols[2] != T4_N) return SC_ERR_SCHED_UNSUPPORTED;
    // E and D rows are addressed with 31-bit byte offsets (bit 31 marks node ends), C rows with 32-bit ones
    if ((uint64_t)fac[2].rows * (uint64_t)fac[2].ld * 4 >= (1ull << 31)) return SC_ERR_SHAPE_MISMATCH;
    if ((uint64_t)fac[1].rows * (uint64_t)fac[1].ld * 4 >= (1ull << 31)) return SC_ERR_SHAPE_MISMATCH;
    if ((uint64_t)fac[0].rows * (uint64_t)fac[0].ld * 4 >= (1ull << 32)) return SC_ERR_SHAPE_MISMATCH;
    Ttmc4Args a;
    a.crd1 = sp->crd[0]; a.pos2 = sp->pos[1]; a.crd2 = sp->crd[1];
    // the two walked levels are read from the plan's walk tables
    if (!p->walk.d_rec[0] || !p->walk.d_rec[1] || !p->walk.d_heads || p->walk.heads_per_tile < T4_G1 + T4_G2) return SC_ERR_SCHED_UNSUPPORTED;
    a.rec4 = p->walk.d_rec[0]; a.rec3 = p->walk.d_rec[1];
    a.heads = p->walk.d_heads; a.heads_per_tile = p->walk.heads_per_tile;
    a.vals = static_cast<const float *>(sp->vals);
    a.C = static_cast<const float *>(fac[0].data); a.ldC = fac[0].ld;
    a.D = static_cast<const float *>(fac[1].data); a.ldD = fac[1].ld;
    a.E = static_cast<const float *>(fac[2].data); a.ldE = fac[2].ld;
    a.T1 = static_cast<const float *>(T1);
    a.T2 = static_cast<float *>(T2);
    a.A = static_cast<float *>(out);
    a.L = (int32_t)p->fcols[0];
    a.tn = p->caps.tn; a.ta = p->caps.ta; a.tb = p->caps.tb;
    // persistent launch over contiguous runs of tiles (the tile table of such a plan is in tensor order)
    const size_t lds = ttmc4_lds_bytes(a.tn, a.ta, a.tb, mode);
    a.partials = static_cast<float *>(partials);
    a.slot_b = p->d_slot_b;
    if (partials && mode == 1 && !p->d_slot_b) return SC_ERR_SCHED_UNSUPPORTED;
    a.ntiles = ntiles;
    a.run = ttmc4_mfma_run(p, mode, partials != nullptr);
    const int blocks = (ntiles + a.run - 1) / a.run;
    if (mode == 0) {
        ln.begin("ttmc4_fused_mfma");
        if (partials)
            ttmc4_mfma_kernel<0, true><<<blocks, NT, lds, ln.stream>>>(a, p->d_tiles);
        else
            ttmc4_mfma_kernel<0, false><<<blocks, NT, lds, ln.stream>>>(a, p->d_tiles);
    } else if (mode == 1) {
        ln.begin("ttmc4_middle");
        if (partials)
            ttmc4_mfma_kernel<1, true><<<blocks, NT, lds, ln.stream>>>(a, p->d_tiles);
        else
            ttmc4_mfma_kernel<1, false><<<blocks, NT, lds, ln.stream>>>(a, p->d_tiles);
    } else {
        ln.begin("ttmc4_consume_mfma");
        if (partials)
            ttmc4_mfma_kernel<2, true><<<blocks, NT, lds, ln.stream>>>(a, p->d_tiles);
        else
            ttmc4_mfma_kernel<2, false><<<blocks, NT, lds, ln.stream>>>(a, p->d_tiles);
    }
    ln.end();
    return ln.status;
}

}  // namespace sck
