// TTM chain of order 3 on matrix cores (Table 2, kernel 6 <SpTTM, TTM>), fp32, L = M = 16; the FUSED
// schedule in one kernel and, with FUSED = false, the consumer half of the FISSIONED schedule (the
// rows of T then come from the workspace instead of the leaf walk):
//     T(f,:)   = sum_{k' in fiber f} B * D(k,:)              (producer, leaf traversal)
//     A(i,:,:) += C(j,:)^T (x) T(f,:)   over the fibers of slice i   (consumer, rank-1 updates)
// The temporary of the `where` nest lives in LDS for the fibers of one tile; the consumer is a
// (16 x Kf) * (Kf x 16) product per slice, Kf = fibers of the slice, on v_mfma_f32_16x16x4_f32.
//
//   stage    every global read of the tile is issued before the first is used; records
//            {D row offset | end-of-fiber bit, value} per nonzero (the coordinates come from the
//            plan's walk tables with the end bits in them, as do the fibers at the heads of the
//            lane groups' chunks), C row offset per fiber, slice bounds and output rows go to LDS
//   walk     the shared branch-free leaf walk (a group of 4 lanes per nonzero chunk, U gathers
//            in flight, running sums written to the fibers' LDS rows, chunk heads combined
//            after a barrier without atomics)
//   consume  each wavefront takes a contiguous quarter of the tile's fibers and runs over the
//            slice segments inside it, four fibers per MFMA; operand A is T (m along the
//            rows), operand B the gathered C rows (l along the columns), so a lane ends up
//            with four consecutive m of one l: one 16-byte store per lane, 1 KB per slice.
//            A slice that begins and ends inside a wavefront's fibers is stored directly; the
//            piece of a slice that continues from / into another wavefront or tile is parked
//            in LDS (at most one head and one tail piece per wavefront, plain stores).
//   combine  wavefront 0 adds the parked pieces in fiber order and stores every slice that
//            ends in the tile.  A workgroup owns a contiguous run of tiles, and the sum of a
//            slice that continues into the next tile stays in wavefront 0's registers, so a
//            heavy slice costs one global update per workgroup instead of one per tile; only a
//            slice that crosses the run's ends is added atomically to the zeroed output.  No
//            LDS atomics are involved (they measured several times slower than this scheme).
#include "leaf_walk.h"

namespace sck {

struct Ttmc3Args {
    const int32_t *crd1, *pos2, *crd2;
    const uint32_t *rec3;    // FUSED: the plan's walk table, last coordinate of every nonzero | end-of-fiber bit 31
    const uint16_t *heads;   // ... and per tile the chunk heads of the T3_G lane groups
    int32_t heads_per_tile;
    const float *vals;
    const float *C, *D;
    int64_t ldC, ldD;
    const float *T;   // FISSIONED consumer: the materialised temporary, one 16-wide row per fiber
    float *A;
    float *partials;   // deterministic schedules: slots for the pieces of rows that span tiles (runs are single tiles then), else null
    int32_t tn, ta, tb;
    int32_t ntiles, run;   // tiles in the plan; tiles per workgroup
};

using Ttmc3Rec = LeafRec<float>;

constexpr int T3_W = 16;            // row width of T (= M) and of C rows (= L)
constexpr int T3_RS = leaf_row_stride<float>(T3_W);   // LDS row stride in floats
constexpr int T3_LG = 4;            // lanes per row
constexpr int T3_G = NT / T3_LG;    // lane groups per workgroup
constexpr int T3_WAVES = NT / 64;
constexpr int T3_MAXR = 4;          // tn <= T3_MAXR * NT
constexpr int T3_U = 8;             // nonzeros a lane group of the leaf walk takes per step

// The carry rows and the nonzero records are dead once the T rows of a tile are complete;
// the pieces that the consumer parks (WAVES x {head, tail} x 256 floats) reuse their space.
// The kernel is bound by latency and its time falls almost in proportion to the workgroups
// that fit a compute unit, so LDS bytes are what to save.
__host__ __device__ constexpr size_t ttmc3_scratch_bytes(int tn)
{
    const size_t walk = (size_t)T3_G * T3_RS * 4 + (size_t)padded(tn + 8) * sizeof(Ttmc3Rec);
    const size_t park = (size_t)(2 * T3_WAVES) * 256 * 4;
    return walk > park ? walk : park;
}

__host__ __device__ constexpr size_t ttmc3_lds_bytes(int tn, int ta, int tb)
{
    return (size_t)(ta + 1) * T3_RS * 4 + ttmc3_scratch_bytes(tn) + (size_t)(T3_G + ta + 2 * tb + 2) * 4 + T3_WAVES * 16 + 64;
}

typedef float t3_floatx4 __attribute__((ext_vector_type(4)));

// DET: the deterministic variant (pieces of rows that span tiles go to plan-numbered slots), a
// separate instantiation so that the atomic variant keeps its register budget.
template <bool FUSED, bool DET>
__global__ void __launch_bounds__(NT, 5) ttmc3_mfma_kernel(Ttmc3Args a, const TileRec *__restrict__ tiles)
{
    constexpr int U = T3_U;
    constexpr int RS = T3_RS;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *row_s = reinterpret_cast<float *>(smem);                                      // (ta + 1) rows of RS
    float *carry_s = row_s + (size_t)(a.ta + 1) * RS;                                    // G rows of RS
    Ttmc3Rec *rec_s = reinterpret_cast<Ttmc3Rec *>(carry_s + (size_t)T3_G * RS);         // padded(tn + 8)
    float *part_s = carry_s;                                                             // WAVES x {head, tail} x 256, once carry_s and rec_s are dead
    uint32_t *chunk_s = reinterpret_cast<uint32_t *>(reinterpret_cast<unsigned char *>(carry_s) + ttmc3_scratch_bytes(a.tn));   // G: chunk heads of the leaf walk
    uint32_t *coff_s = chunk_s + T3_G;                                                   // ta: byte offset of C(j,:)
    int *bb_s = reinterpret_cast<int *>(coff_s + a.ta);                                  // tb + 2: first fiber of each slice
    int *crdb_s = bb_s + a.tb + 2;                                                       // tb: output row of each slice
    int *meta_s = crdb_s + a.tb;                                                         // WAVES x 4: head slice, head ends, tail slice

    const int tid = threadIdx.x;
    const int first = blockIdx.x * a.run, lastp1 = min(first + a.run, a.ntiles);
    t3_floatx4 carry = {0.f, 0.f, 0.f, 0.f};   // wavefront 0: sum so far of the slice that continues from the previous tile
    bool chain_shared = false;                 // that slice began before this workgroup's run
    // Global reads of one tile's staging, all issued before the first is used.
    constexpr int TR = (NT + T3_G - 1) / T3_G;   // T rows copied per lane group: ta <= TR * G
    struct Stage {
        uint32_t kk[T3_MAXR];
        float vv[T3_MAXR];
        uint32_t hd;
        Pack<float, 4> trow[FUSED ? 1 : TR];
        int cj, ps, ci;
    };
    auto issue = [&](const TileRec &t, int tile, Stage &s) {
        const int nchild = t.n1 - t.n0;
        const int na = t.na, nb = t.nb;
        if (FUSED) {
#pragma unroll
            for (int r = 0; r < T3_MAXR; ++r) {
                const int c = t.n0 + min(tid + r * NT, nchild - 1);
                s.kk[r] = a.rec3[c];
                s.vv[r] = a.vals[c];
            }
            s.hd = a.heads[(int64_t)tile * a.heads_per_tile + min(tid, T3_G - 1)];
        } else {
#pragma unroll
            for (int r = 0; r < TR; ++r) {
                const int f = min(tid / T3_LG + r * T3_G, na - 1);
                s.trow[r] = *reinterpret_cast<const Pack<float, 4> *>(a.T + (int64_t)(t.a0 + f) * T3_W + (tid % T3_LG) * 4);
            }
        }
        s.cj = a.crd2[t.a0 + min(tid, na - 1)];
        s.ps = a.pos2[t.b0 + min(tid, nb)];
        s.ci = a.crd1[t.b0 + min(tid, nb - 1)];
    };
    TileRec t = tiles[first];   // a launched workgroup has at least one tile
    Stage st;
    issue(t, first, st);

    for (int tile = first; tile < lastp1; ++tile) {
    const TileRec tn = tiles[min(tile + 1, lastp1 - 1)];
    const bool in_f = (t.flags & 4) != 0, out_f = (t.flags & 8) != 0;
    if (tile == first && in_f) chain_shared = true;
    const int nchild = t.n1 - t.n0;
    const int na = t.na, nb = t.nb;
    const int q = leaf_chunk<U>(nchild, T3_G);   // nonzeros per lane group, multiple of U
    const uint32_t rowD = (uint32_t)(a.ldD * 4), rowC = (uint32_t)(a.ldC * 4);

    // ---- stage 1: registers -> LDS ----
    {
        const uint32_t(&kk)[T3_MAXR] = st.kk;
        const float(&vv)[T3_MAXR] = st.vv;
        const auto &trow = st.trow;
        const int cj = st.cj, ps = st.ps, ci = st.ci;
        if (FUSED) {
#pragma unroll
            for (int r = 0; r < T3_MAXR; ++r) {
                const int c = tid + r * NT;
                if (c < nchild) {
                    Ttmc3Rec rec;
                    // the tile's last nonzero closes the fiber it is in as far as this tile goes
                    rec.koff = (kk[r] & 0x7fffffffu) * rowD | (kk[r] & 0x80000000u) | (c == nchild - 1 ? 0x80000000u : 0u);
                    rec.v = vv[r];
                    rec_s[pidx(c)] = rec;
                }
            }
            if (tid < U) {  // dummies completing the last batch: value 0, row 0, no mark
                Ttmc3Rec rec;
                rec.koff = 0;
                rec.v = 0.f;
                rec_s[pidx(nchild + tid)] = rec;
            }
            if (tid < T3_G) chunk_s[tid] = st.hd;
        } else {
            // A fiber cut by a tile boundary has one complete row in the workspace; the tile in
            // which it starts consumes it, the tiles it continues into see a zero row.
#pragma unroll
            for (int r = 0; r < TR; ++r) {
                const int f = tid / T3_LG + r * T3_G;
                if (f < na) {
                    Pack<float, 4> v = trow[r];
                    if (f == 0 && (t.flags & 1)) v = Pack<float, 4>{{0.f, 0.f, 0.f, 0.f}};
                    *reinterpret_cast<Pack<float, 4> *>(row_s + f * RS + (tid % T3_LG) * 4) = v;
                }
            }
        }
        if (tid < na) coff_s[tid] = (uint32_t)cj * rowC;
        if (tid <= nb) bb_s[tid] = min(max(ps, t.a0), t.a0 + na) - t.a0;
        if (tid < nb) crdb_s[tid] = ci;
    }
    __syncthreads();

    // ---- consumer kernel: the next tile's reads go out now and land while this tile is worked on
    // (the fused kernel has no registers to spare for that: it measured slower with spills) ----
    Stage sn;
    if (!FUSED && tile + 1 < lastp1) issue(tn, tile + 1, sn);

    // ---- walk (leaves -> T rows in LDS), combine ----
    if (FUSED) {
        const int g = tid / T3_LG, li = tid % T3_LG;
        const uint32_t done = table_walk<float, T3_W, U>(row_s, carry_s, rec_s, chunk_s, a.D, g, li, q, nchild);
        __syncthreads();
        table_combine<float, T3_W>(row_s, carry_s, chunk_s, done, g, li);
        __syncthreads();
    }

    // ---- consume: T rows (LDS) x gathered C rows -> A ----
    // Loop bounds come from LDS; readfirstlane tells the compiler they are wavefront-uniform.
    auto uni = [](int x) { return __builtin_amdgcn_readfirstlane(x); };
    const int wave = uni(tid / 64), lane = tid % 64;
    const int kk = lane / 16, col = lane % 16;
    const int qf = max((((na + 3) / 4) + T3_WAVES - 1) / T3_WAVES * 4, 4);   // fibers per wavefront, multiple of 4
    const int ws = wave * qf, we = min(ws + qf, na);
    const char *Cb = reinterpret_cast<const char *>(a.C) + col * 4;
    int head_ls = -1, head_ends = 0, tail_ls = -1;
    if (ws < we) {
        int ls = 0;
        while (uni(bb_s[ls + 1]) <= ws) ++ls;   // slice holding fiber ws (bb_s[nb] = na > ws ends the scan)
        int f = ws;
        while (f < we) {
            const int s_lo = uni(bb_s[ls]), s_hi = uni(bb_s[ls + 1]);
            const int se = min(s_hi, we);
            t3_floatx4 acc = {0.f, 0.f, 0.f, 0.f};
            constexpr int UB = 4;   // 4-fiber blocks whose operand reads are issued together
            for (int fb = f; fb < se; fb += 4 * UB) {
                float cv[UB], tv[UB];
#pragma unroll
                for (int ub = 0; ub < UB; ++ub) {
                    const int lf = fb + 4 * ub + kk;
                    const int lfc = min(lf, se - 1);   // lanes past the segment read a valid fiber and are zeroed
                    const float tvr = row_s[lfc * RS + col];
                    cv[ub] = *reinterpret_cast<const float *>(Cb + coff_s[lfc]);
                    tv[ub] = lf < se ? tvr : 0.f;
                }
#pragma unroll
                for (int ub = 0; ub < UB; ++ub)
                    if (fb + 4 * ub < se) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(tv[ub], cv[ub], acc, 0, 0, 0);
            }
            // acc[r] = A(l = col, m = 4 kk + r)
            const bool starts = s_lo >= ws && !(ls == 0 && in_f);      // the slice's first fiber is here
            const bool ends = s_hi <= we && !(ls == nb - 1 && out_f);  // ... and its last one
            if (starts && ends) {
                *reinterpret_cast<t3_floatx4 *>(a.A + (int64_t)uni(crdb_s[ls]) * 256 + col * 16 + 4 * kk) = acc;   // sole writer
            } else if (!starts) {
                *reinterpret_cast<t3_floatx4 *>(part_s + (2 * wave) * 256 + col * 16 + 4 * kk) = acc;
                head_ls = ls;
                head_ends = ends;
            } else {
                *reinterpret_cast<t3_floatx4 *>(part_s + (2 * wave + 1) * 256 + col * 16 + 4 * kk) = acc;
                tail_ls = ls;
            }
            f = se;
            ++ls;
        }
    }
    if (lane == 0) {
        meta_s[4 * wave] = head_ls;
        meta_s[4 * wave + 1] = head_ends;
        meta_s[4 * wave + 2] = tail_ls;
    }
    __syncthreads();

    // ---- combine ----
    if (wave == 0) {
        auto emit = [&](const t3_floatx4 &v, int ls, bool atomic) {
            float *dst = a.A + (int64_t)uni(crdb_s[ls]) * 256 + lane * 4;
            if (!atomic) {
                *reinterpret_cast<t3_floatx4 *>(dst) = v;
            } else if (DET) {
                // deterministic: this tile's piece of the row goes to its slot (a tile whose only
                // slice continues on both sides has one piece, numbered as its first)
                const int slot = (ls == 0 && in_f) ? t.pad[0] : t.pad[1];
                *reinterpret_cast<t3_floatx4 *>(a.partials + (int64_t)slot * 256 + lane * 4) = v;
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) atomic_add(dst + r, v[r]);
            }
        };
        t3_floatx4 acc = carry;   // zero unless a slice continues from the previous tile of the run
        if (!in_f) acc = t3_floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < T3_WAVES; ++w) {
            const int hl = uni(meta_s[4 * w]), he = uni(meta_s[4 * w + 1]), tl = uni(meta_s[4 * w + 2]);
            if (hl >= 0) {
                acc += *reinterpret_cast<const t3_floatx4 *>(part_s + (2 * w) * 256 + lane * 4);
                if (he) {
                    const bool incoming = hl == 0 && in_f;
                    emit(acc, hl, incoming && chain_shared);
                    if (incoming) chain_shared = false;
                    acc = t3_floatx4{0.f, 0.f, 0.f, 0.f};
                }
            }
            if (tl >= 0) acc = *reinterpret_cast<const t3_floatx4 *>(part_s + (2 * w + 1) * 256 + lane * 4);
        }
        if (out_f) {
            if (tile + 1 == lastp1) emit(acc, nb - 1, true);   // continues in another workgroup's run
            else carry = acc;
        }
    }
    __syncthreads();
    if (tile + 1 < lastp1) {
        if (FUSED) issue(tn, tile + 1, sn);
        t = tn;
        st = sn;
    }
    }  // tiles of the run
}

WalkShape ttmc3_mfma_walk_shape()
{
    WalkShape w;
    w.levels = 1;
    w.groups[0] = T3_G;
    w.batch[0] = T3_U;
    return w;
}

size_t ttmc3_mfma_lds_bytes(const sc_plan *p) { return ttmc3_lds_bytes(p->caps.tn, p->caps.ta, p->caps.tb); }

bool ttmc3_mfma_caps_ok(const sc_plan *p)
{
    return p->caps.tn <= T3_MAXR * NT && p->caps.ta <= NT && p->caps.tb + 1 <= NT && p->caps.tb >= 1;
}

// Tiles per workgroup: four runs per resident workgroup slot (shorter runs even out the tiles' different costs); a
// deterministic schedule takes one tile per workgroup, so that the pieces are the ones the plan numbered.
int ttmc3_mfma_run(const sc_plan *p, bool one_tile_per_workgroup)
{
    const int ntiles = (int)p->tiles.size();
    if (ntiles == 0 || one_tile_per_workgroup) return 1;
    const int fit = lds_workgroups_per_cu(ttmc3_lds_bytes(p->caps.tn, p->caps.ta, p->caps.tb), p->lds_per_cu);
    const int per_cu = p->tune.per_cu > 0 ? std::min(p->tune.per_cu, 64) : 4 * fit;
    const int want = std::min(ntiles, p->n_cu * per_cu);
    return (ntiles + want - 1) / want;
}

sc_status launch_ttmc3_mfma(const sc_plan *p, Launcher &ln, const sc_csf_view *sp, const sc_dense_view *fac, const void *T, void *out,
                            void *partials)
{
    // T == nullptr: FUSED schedule; otherwise the consumer kernel of the FISSIONED schedule
    const int ntiles = (int)p->tiles.size();
    if (ntiles == 0) return SC_OK;
    if (!ttmc3_mfma_caps_ok(p)) return SC_ERR_SCHED_UNSUPPORTED;
    // D rows are addressed with 31-bit byte offsets (bit 31 marks fiber ends), C rows with 32-bit ones
    if ((uint64_t)fac[1].rows * (uint64_t)fac[1].ld * 4 >= (1ull << 31)) return SC_ERR_SHAPE_MISMATCH;
    if ((uint64_t)fac[0].rows * (uint64_t)fac[0].ld * 4 >= (1ull << 32)) return SC_ERR_SHAPE_MISMATCH;
    Ttmc3Args a;
    a.crd1 = sp->crd[0]; a.pos2 = sp->pos[1]; a.crd2 = sp->crd[1];
    a.rec3 = nullptr; a.heads = nullptr; a.heads_per_tile = 0;
    if (T == nullptr) {   // the leaf level is read from the plan's walk tables
        const WalkTables &wt = p->walk;
        if (!wt.d_rec[0] || !wt.d_heads || wt.shape.groups[0] != T3_G || wt.shape.batch[0] != T3_U) return SC_ERR_SCHED_UNSUPPORTED;
        a.rec3 = wt.d_rec[0]; a.heads = wt.d_heads; a.heads_per_tile = wt.heads_per_tile;
    }
    a.vals = static_cast<const float *>(sp->vals);
    a.C = static_cast<const float *>(fac[0].data); a.ldC = fac[0].ld;
    a.D = static_cast<const float *>(fac[1].data); a.ldD = fac[1].ld;
    a.T = static_cast<const float *>(T);
    a.A = static_cast<float *>(out);
    a.tn = p->caps.tn; a.ta = p->caps.ta; a.tb = p->caps.tb;
    // persistent launch over contiguous runs of tiles (the tile table of such a plan is in tensor order)
    const size_t lds = ttmc3_lds_bytes(a.tn, a.ta, a.tb);
    a.partials = static_cast<float *>(partials);
    a.ntiles = ntiles;
    a.run = ttmc3_mfma_run(p, partials != nullptr);
    const int blocks = (ntiles + a.run - 1) / a.run;
    if (T == nullptr) {
        ln.begin("ttmc3_fused_mfma");
        if (partials)
            ttmc3_mfma_kernel<true, true><<<blocks, NT, lds, ln.stream>>>(a, p->d_tiles);
        else
            ttmc3_mfma_kernel<true, false><<<blocks, NT, lds, ln.stream>>>(a, p->d_tiles);
    } else {
        ln.begin("ttmc3_consume_mfma");
        if (partials)
            ttmc3_mfma_kernel<false, true><<<blocks, NT, lds, ln.stream>>>(a, p->d_tiles);
        else
            ttmc3_mfma_kernel<false, false><<<blocks, NT, lds, ln.stream>>>(a, p->d_tiles);
    }
    ln.end();
    return ln.status;
}

}  // namespace sck
