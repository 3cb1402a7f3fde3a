// TTM chain of order 3 on matrix cores for fp32 ranks that are multiples of the 16 x 16 MFMA tile (Table 2,
// kernel 6 <SpTTM, TTM>; also the sparse part of kernel 5's second schedule): the FUSED schedule in one kernel and,
// with FUSED = false, the consumer half of the FISSIONED schedule (the rows of T then come from the workspace):
//     T(f,:)    = sum_{k' in fiber f} B * D(k,:)                       (producer, leaf walk; W = 16 MT columns)
//     A(i,:,:) += C(j,:)^T (x) T(f,:)   over the fibers of slice i     (consumer; L = 16 LT rows of C)
// The consumer of a slice is an (L x Kf) * (Kf x W) product, Kf = fibers of the slice.  Its LT x MT output tiles
// are dealt out to the four wavefronts of a workgroup once and for all, so no sum crosses wavefronts, and a
// workgroup owns a contiguous run of tiles: the tiles of a slice that continues into the next work tile stay in
// the accumulator registers.  A slice therefore costs one store of its L x W row per workgroup it passes through
// (atomic only when it crosses the ends of a run), where a kernel that works tile by tile pays one atomic row
// update per tile: with rows of 4 to 64 KB and 16 to 128 fibers per tile that update was most of its time.
//
//   stage    every global read of the tile is issued before the first is used, one tile ahead; records
//            {D row offset | end-of-fiber bit, value} per nonzero and the chunk heads come from the plan's walk tables
//   C rows   the C rows of the tile's fibers go to LDS with 16-byte loads (operand B of every MFMA of the tile)
//   walk     the shared branch-free leaf walk -> T rows in LDS (operand A)
//   consume  per slice segment, four fibers per v_mfma_f32_16x16x4_f32 and output tile; a wavefront reads MTW + LTW
//            operands per step for its MTW x LTW tiles; a lane ends up with four consecutive m of one l
#include "leaf_walk.h"

namespace sck {

struct Ttmc3wArgs {
    const int32_t *crd1, *pos2, *crd2;
    const uint32_t *rec3;    // the plan's walk table: last coordinate of every nonzero | end-of-fiber bit 31
    const uint16_t *heads;   // ... and per tile the chunk heads of the lane groups
    int32_t heads_per_tile;
    const float *vals;
    const float *C, *D;
    int64_t ldC, ldD;
    const float *T;   // FISSIONED consumer: the materialised temporary, one W-wide row per fiber
    float *A;
    int32_t tn, ta, tb;
    int32_t ntiles, run;   // tiles in the plan; tiles per workgroup
};

constexpr int T3W_U = 4;      // nonzeros a lane group of the leaf walk takes per step
constexpr int T3W_MAXR = 4;   // tn <= T3W_MAXR * NT; ta, tb + 1 <= NT

__host__ __device__ constexpr int t3w_groups(int W) { return NT / (W / 4); }

__host__ __device__ constexpr size_t ttmc3w_lds_bytes(int L, int W, int tn, int ta, int tb)
{
    const int RS = leaf_row_stride<float>(W);
    return (size_t)(ta + 1 + t3w_groups(W)) * RS * 4 + (size_t)padded(tn + 8) * sizeof(LeafRec<float>) + (size_t)t3w_groups(W) * 4 +
           (size_t)(ta + 4) * (L + 4) * 4 + (size_t)(ta + 2 * tb + 4) * 4 + 64;
}

typedef float t3w_floatx4 __attribute__((ext_vector_type(4)));

template <int LT, int MT, bool FUSED>
__global__ void __launch_bounds__(NT) ttmc3_wide_kernel(Ttmc3wArgs a, const TileRec *__restrict__ tiles)
{
    constexpr int L = 16 * LT, W = 16 * MT;
    constexpr int U = T3W_U;
    constexpr int RS = leaf_row_stride<float>(W), LS = L + 4;
    constexpr int LG = W / 4, G = NT / LG;
    // the four wavefronts over the output tiles: WM of them along m, WL along l
    constexpr int WM = MT < 4 ? MT : 4, WL = 4 / WM;
    constexpr int MTW = MT / WM, LTW = LT >= WL ? LT / WL : 1;
    static_assert(MT % WM == 0 && (LT % WL == 0 || LT < WL), "tile split");
    using Rec = LeafRec<float>;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *row_s = reinterpret_cast<float *>(smem);                                  // (ta + 1) rows of RS: T
    float *carry_s = row_s + (size_t)(a.ta + 1) * RS;                                // G rows of RS
    float *crow_s = carry_s + (size_t)G * RS;                                        // (ta + 4) rows of LS: C rows of the fibers (16-byte aligned)
    Rec *rec_s = reinterpret_cast<Rec *>(crow_s + (size_t)(a.ta + 4) * LS);          // padded(tn + 8)
    uint32_t *chunk_s = reinterpret_cast<uint32_t *>(rec_s + padded(a.tn + 8));      // G: chunk heads
    int *cj_s = reinterpret_cast<int *>(chunk_s + G);                                // ta: j of each fiber
    int *bb_s = cj_s + a.ta;                                                         // tb + 2: first fiber of each slice
    int *crdb_s = bb_s + a.tb + 2;                                                   // tb: output row of each slice

    const int tid = threadIdx.x;
    const int first = blockIdx.x * a.run, lastp1 = min(first + a.run, a.ntiles);
    auto uni = [](int x) { return __builtin_amdgcn_readfirstlane(x); };
    const int wave = uni(tid / 64), lane = tid % 64;
    const int kk = lane / 16, col = lane % 16;
    const int wm = wave % WM, wl = wave / WM;
    const bool wave_active = wl * LTW < LT;   // fewer output tiles than wavefronts: the others only produce
    const uint32_t rowD = (uint32_t)(a.ldD * 4);

    t3w_floatx4 acc[MTW][LTW];   // this wavefront's tiles of the current slice; they live across work tiles
#pragma unroll
    for (int x = 0; x < MTW; ++x)
#pragma unroll
        for (int y = 0; y < LTW; ++y) acc[x][y] = t3w_floatx4{0.f, 0.f, 0.f, 0.f};
    bool chain_shared = false;   // the slice in the accumulators began before this workgroup's run

    struct Stage {
        uint32_t kk[T3W_MAXR];
        float vv[T3W_MAXR];
        uint32_t hd;
        int cj, ps, ci;
    };
    auto issue = [&](const TileRec &t, int tile, Stage &s) {
        const int nchild = t.n1 - t.n0;
        if (FUSED) {
#pragma unroll
            for (int r = 0; r < T3W_MAXR; ++r) {
                const int c = t.n0 + min(tid + r * NT, nchild - 1);
                s.kk[r] = a.rec3[c];
                s.vv[r] = a.vals[c];
            }
            s.hd = a.heads[(int64_t)tile * a.heads_per_tile + min(tid, G - 1)];
        }
        s.cj = a.crd2[t.a0 + min(tid, t.na - 1)];
        s.ps = a.pos2[t.b0 + min(tid, t.nb)];
        s.ci = a.crd1[t.b0 + min(tid, t.nb - 1)];
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
        const int q = leaf_chunk<U>(nchild, G);

        // ---- stage: registers -> LDS ----
        if (FUSED) {
#pragma unroll
            for (int r = 0; r < T3W_MAXR; ++r) {
                const int c = tid + r * NT;
                if (c < nchild) {
                    Rec rec;
                    // the tile's last nonzero closes the fiber it is in as far as this tile goes
                    rec.koff = (st.kk[r] & 0x7fffffffu) * rowD | (st.kk[r] & 0x80000000u) | (c == nchild - 1 ? 0x80000000u : 0u);
                    rec.v = st.vv[r];
                    rec_s[pidx(c)] = rec;
                }
            }
            if (tid < U) {  // dummies completing the last batch: value 0, row 0, no mark
                Rec rec;
                rec.koff = 0;
                rec.v = 0.f;
                rec_s[pidx(nchild + tid)] = rec;
            }
            if (tid < G) chunk_s[tid] = st.hd;
        }
        if (tid < na) cj_s[tid] = st.cj;
        if (tid <= nb) bb_s[tid] = min(max(st.ps, t.a0), t.a0 + na) - t.a0;
        if (tid < nb) crdb_s[tid] = st.ci;
        __syncthreads();

        // ---- the next tile's reads go out now and land while this tile is worked on ----
        Stage sn;
        if (tile + 1 < lastp1) issue(tn, tile + 1, sn);

        // ---- C rows of the tile's fibers -> LDS, 16 bytes per lane, consecutive lanes on consecutive pieces of a row ----
        {
            constexpr int VPR = L / 4;   // 16-byte pieces per row
#pragma unroll 4
            for (int idx = tid; idx < na * VPR; idx += NT) {
                const int f = idx / VPR, q4 = (idx % VPR) * 4;
                *reinterpret_cast<t3w_floatx4 *>(crow_s + f * LS + q4) =
                    *reinterpret_cast<const t3w_floatx4 *>(a.C + (int64_t)cj_s[f] * a.ldC + q4);
            }
        }

        // ---- T rows of the tile's fibers: the leaf walk (FUSED), or the rows the traversal kernel left in the workspace.  A fiber
        // cut by a tile boundary has one complete row there; the tile in which it starts consumes it, the tiles it continues
        // into see a zero row. ----
        if (!FUSED) {
            constexpr int VPR = W / 4;
            const float *Tg = a.T + (int64_t)t.a0 * W;
#pragma unroll 4
            for (int idx = tid; idx < na * VPR; idx += NT) {
                const int f = idx / VPR, q4 = (idx % VPR) * 4;
                t3w_floatx4 v = *reinterpret_cast<const t3w_floatx4 *>(Tg + (int64_t)f * W + q4);
                if (f == 0 && (t.flags & 1)) v = t3w_floatx4{0.f, 0.f, 0.f, 0.f};
                *reinterpret_cast<t3w_floatx4 *>(row_s + f * RS + q4) = v;
            }
            __syncthreads();
        } else {
            const int g = tid / LG, li = tid % LG;
            const uint32_t done = table_walk<float, W, U>(row_s, carry_s, rec_s, chunk_s, a.D, g, li, q, nchild);
            __syncthreads();
            table_combine<float, W>(row_s, carry_s, chunk_s, done, g, li);
            __syncthreads();
        }

        // ---- consume: T rows x C rows -> the wavefront's output tiles, slice by slice ----
        if (wave_active) {
            const bool last_tile = tile + 1 == lastp1;
            auto emit = [&](int ls, bool atomic) {
                float *row = a.A + (int64_t)uni(crdb_s[ls]) * (L * W);
#pragma unroll
                for (int x = 0; x < MTW; ++x)
#pragma unroll
                    for (int y = 0; y < LTW; ++y) {
                        // acc[r] = A(l = 16 lt + col, m = 16 mt + 4 kk + r)
                        const int mt = wm + WM * x, lt = wl * LTW + y;
                        float *dst = row + (lt * 16 + col) * W + mt * 16 + 4 * kk;
                        if (!atomic) {
                            *reinterpret_cast<t3w_floatx4 *>(dst) = acc[x][y];
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r) atomic_add(dst + r, acc[x][y][r]);
                        }
                        acc[x][y] = t3w_floatx4{0.f, 0.f, 0.f, 0.f};
                    }
            };
            for (int ls = 0; ls < nb; ++ls) {
                const int f0 = uni(bb_s[ls]), f1 = uni(bb_s[ls + 1]);
                for (int fb = f0; fb < f1; fb += 4) {
                    const int lf = fb + kk;
                    const int lfc = min(lf, f1 - 1);   // lanes past the slice read a valid fiber and are zeroed
                    const float *tp = row_s + lfc * RS + wm * 16 + col;
                    const float *cp = crow_s + lfc * LS + wl * LTW * 16 + col;
                    float tv[MTW], cv[LTW];
#pragma unroll
                    for (int x = 0; x < MTW; ++x) {
                        const float v = tp[x * WM * 16];
                        tv[x] = lf < f1 ? v : 0.f;
                    }
#pragma unroll
                    for (int y = 0; y < LTW; ++y) cv[y] = cp[y * 16];
#pragma unroll
                    for (int x = 0; x < MTW; ++x)
#pragma unroll
                        for (int y = 0; y < LTW; ++y) acc[x][y] = __builtin_amdgcn_mfma_f32_16x16x4f32(tv[x], cv[y], acc[x][y], 0, 0, 0);
                }
                const bool incoming = ls == 0 && in_f, outgoing = ls == nb - 1 && out_f;
                if (outgoing) {
                    if (last_tile) emit(ls, true);   // continues in another workgroup's run
                } else {
                    emit(ls, incoming && chain_shared);
                    if (incoming) chain_shared = false;
                }
            }
        }
        __syncthreads();
        if (tile + 1 < lastp1) {
            t = tn;
            st = sn;
        }
    }  // tiles of the run
}

namespace {

template <int LT, int MT>
void launch_wide(const Ttmc3wArgs &a, const TileRec *tiles, int blocks, size_t lds, hipStream_t stream)
{
    if (a.T)
        ttmc3_wide_kernel<LT, MT, false><<<blocks, NT, lds, stream>>>(a, tiles);
    else
        ttmc3_wide_kernel<LT, MT, true><<<blocks, NT, lds, stream>>>(a, tiles);
}

template <int LT>
bool dispatch_m(int MT, const Ttmc3wArgs &a, const TileRec *tiles, int blocks, size_t lds, hipStream_t stream)
{
    switch (MT) {
    case 1: if constexpr (LT != 1) { launch_wide<LT, 1>(a, tiles, blocks, lds, stream); return true; } return false;
    case 2: launch_wide<LT, 2>(a, tiles, blocks, lds, stream); return true;
    case 4: launch_wide<LT, 4>(a, tiles, blocks, lds, stream); return true;
    case 8: launch_wide<LT, 8>(a, tiles, blocks, lds, stream); return true;
    default: return false;
    }
}

}  // namespace

// Ranks the kernel is instantiated for: L, W in {16, 32, 64, 128}, not both 16 (that case has a kernel of its own).
bool ttmc3_wide_ranks(int64_t L, int64_t W)
{
    auto ok = [](int64_t x) { return x == 16 || x == 32 || x == 64 || x == 128; };
    return ok(L) && ok(W) && !(L == 16 && W == 16);
}

WalkShape ttmc3_wide_walk_shape(int W)
{
    WalkShape w;
    w.levels = 1;
    w.groups[0] = t3w_groups(W);
    w.batch[0] = T3W_U;
    return w;
}

size_t ttmc3_wide_lds_bytes(const sc_plan *p)
{
    if (p->caps.tn > T3W_MAXR * NT || p->caps.ta > NT || p->caps.tb + 1 > NT || p->caps.tb < 1) return SIZE_MAX;
    return ttmc3w_lds_bytes((int)p->fcols[0], (int)p->fcols[1], p->caps.tn, p->caps.ta, p->caps.tb);
}

// Tiles per workgroup: four runs per resident workgroup slot.
int ttmc3_wide_run(const sc_plan *p)
{
    const int ntiles = (int)p->tiles.size();
    if (ntiles == 0) return 1;
    const size_t lds = ttmc3w_lds_bytes((int)p->fcols[0], (int)p->fcols[1], p->caps.tn, p->caps.ta, p->caps.tb);
    const int fit = lds_workgroups_per_cu(lds, p->lds_per_cu);
    const int per_cu = p->tune.per_cu > 0 ? std::min(p->tune.per_cu, 64) : 4 * fit;
    const int want = std::min(ntiles, p->n_cu * per_cu);
    return (ntiles + want - 1) / want;
}

sc_status launch_ttmc3_wide(const sc_plan *p, Launcher &ln, const sc_csf_view *sp, const sc_dense_view *fac, const void *T, void *out)
{
    // T == nullptr: FUSED schedule; otherwise the consumer kernel of the FISSIONED schedule
    const int ntiles = (int)p->tiles.size();
    if (ntiles == 0) return SC_OK;
    const int L = (int)p->fcols[0], W = (int)p->fcols[1];
    if (!ttmc3_wide_ranks(L, W) || ttmc3_wide_lds_bytes(p) == SIZE_MAX) return SC_ERR_SCHED_UNSUPPORTED;
    // D rows are addressed with 31-bit byte offsets (bit 31 marks fiber ends)
    if ((uint64_t)fac[1].rows * (uint64_t)fac[1].ld * 4 >= (1ull << 31)) return SC_ERR_SHAPE_MISMATCH;
    Ttmc3wArgs a;
    a.crd1 = sp->crd[0]; a.pos2 = sp->pos[1]; a.crd2 = sp->crd[1];
    a.rec3 = nullptr; a.heads = nullptr; a.heads_per_tile = 0;
    if (T == nullptr) {   // the leaf level is read from the plan's walk tables
        const WalkTables &wt = p->walk;
        const WalkShape want = ttmc3_wide_walk_shape(W);
        if (!wt.d_rec[0] || !wt.d_heads || wt.shape.groups[0] != want.groups[0] || wt.shape.batch[0] != want.batch[0]) return SC_ERR_SCHED_UNSUPPORTED;
        a.rec3 = wt.d_rec[0]; a.heads = wt.d_heads; a.heads_per_tile = wt.heads_per_tile;
    }
    a.T = static_cast<const float *>(T);
    a.vals = static_cast<const float *>(sp->vals);
    a.C = static_cast<const float *>(fac[0].data); a.ldC = fac[0].ld;
    a.D = static_cast<const float *>(fac[1].data); a.ldD = fac[1].ld;
    a.A = static_cast<float *>(out);
    a.tn = p->caps.tn; a.ta = p->caps.ta; a.tb = p->caps.tb;
    // persistent launch over contiguous runs of tiles (the tile table of such a plan is in tensor order)
    const size_t lds = ttmc3w_lds_bytes(L, W, a.tn, a.ta, a.tb);
    a.ntiles = ntiles;
    a.run = ttmc3_wide_run(p);
    const int blocks = (ntiles + a.run - 1) / a.run;
    ln.begin(T ? "ttmc3_consume_mfma_wide" : "ttmc3_fused_mfma_wide");
    bool ok = false;
    switch (L / 16) {
    case 1: ok = dispatch_m<1>(W / 16, a, p->d_tiles, blocks, lds, ln.stream); break;
    case 2: ok = dispatch_m<2>(W / 16, a, p->d_tiles, blocks, lds, ln.stream); break;
    case 4: ok = dispatch_m<4>(W / 16, a, p->d_tiles, blocks, lds, ln.stream); break;
    case 8: ok = dispatch_m<8>(W / 16, a, p->d_tiles, blocks, lds, ln.stream); break;
    default: break;
    }
    ln.end();
    return ok ? ln.status : SC_ERR_SCHED_UNSUPPORTED;
}

}  // namespace sck
