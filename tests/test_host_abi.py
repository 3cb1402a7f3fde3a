"""Host side of the C ABI, without a GPU: the library loads and exports every declared
symbol, COO -> CSF conversion, validation / error codes, derived temporaries, tile tables."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2311_09549_amd import binding as sc
from paper_2311_09549_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _status(fn, *args, **kw):
    try:
        fn(*args, **kw)
    except sc.ScError as e:
        return sc.STATUS_NAMES[e.status]
    return "SC_OK"


def _small(cid=3, scale=0.002):
    cfg = synth.config(cid, scale)
    data = synth.generate(cfg)
    csf = sc.coo_to_csf(list(data["coords"]), data["vals"], cfg["dims"])
    return cfg, data, csf


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "sparsecontract.h")).read()
    declared = sorted(set(re.findall(r"\b(sc_[a-z_0-9]+)\s*\(", hdr)) - {"sc_status"})  # the type name occurs in a comment
    assert set(declared) == set(sc.EXPORTS)
    lib = ctypes.CDLL(sc.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert sc.version() == (0, 1)
    assert sc.status_string(0) == "ok" and "unknown" in sc.status_string(99)


def test_coo_to_csf_matches_numpy_prefix_structure():
    for cid, scale in [(1, 1.0), (2, 0.002), (4, 0.002), (5, 0.01)]:
        cfg = synth.config(cid, scale)
        data = synth.generate(cfg)
        coords, dims = data["coords"], cfg["dims"]
        csf = sc.coo_to_csf(list(coords), data["vals"], dims)
        order = len(dims)
        key = np.zeros(coords.shape[1], dtype=np.int64)
        for m in range(order):
            key = key * dims[m] + coords[m]
            uniq, first = np.unique(key, return_index=True)
            assert csf.nfib[m] == uniq.size
            np.testing.assert_array_equal(csf.crd[m], coords[m][first])   # coordinate of each node
            if m:
                # children of node p of level m-1 are the level-m nodes sharing its prefix
                parent_key = uniq // dims[m]
                starts = np.searchsorted(parent_key, prev_uniq)
                np.testing.assert_array_equal(csf.pos[m][:-1], starts)
                assert csf.pos[m][-1] == uniq.size
            prev_uniq = uniq
        assert csf.nnz == coords.shape[1] and csf.vals is not None


def test_coo_validation_errors():
    dims = (4, 5, 6)
    good = [np.array([0, 0, 1], np.int32), np.array([1, 2, 0], np.int32), np.array([3, 3, 5], np.int32)]
    vals = np.ones(3, np.float32)
    assert sc.coo_to_csf_sizes(good, vals, dims) == [2, 3, 3]
    unsorted = [good[0][::-1].copy(), good[1][::-1].copy(), good[2][::-1].copy()]
    assert _status(sc.coo_to_csf_sizes, unsorted, vals, dims) == "SC_ERR_UNSORTED"
    dup = [np.array([0, 0], np.int32), np.array([1, 1], np.int32), np.array([3, 3], np.int32)]
    assert _status(sc.coo_to_csf_sizes, dup, vals[:2], dims) == "SC_ERR_DUPLICATE"
    rng = [np.array([0], np.int32), np.array([5], np.int32), np.array([0], np.int32)]
    assert _status(sc.coo_to_csf_sizes, rng, vals[:1], dims) == "SC_ERR_CRD_RANGE"
    assert _status(sc.coo_to_csf_sizes, good, vals, (4, 5, 0)) == "SC_ERR_BAD_DIMS"
    assert _status(sc.coo_to_csf_sizes, good[:1], vals, (4,)) == "SC_ERR_BAD_ORDER"
    v = sc.coo_view(good, vals, dims)
    v.dtype = 7
    nf = (ctypes.c_int64 * 4)()
    assert sc.lib().sc_coo_to_csf_sizes(ctypes.byref(v), nf) == sc.STATUS_NAMES.index("SC_ERR_BAD_DTYPE")
    assert sc.lib().sc_coo_to_csf_sizes(None, nf) == sc.STATUS_NAMES.index("SC_ERR_NULL")


def test_empty_tensor_converts_and_plans():
    dims = (4, 5, 6)
    empty = [np.zeros(0, np.int32)] * 3
    csf = sc.coo_to_csf(empty, np.zeros(0, np.float32), dims)
    assert csf.nfib == (0, 0, 0) and [int(p[0]) for p in csf.pos[1:]] == [0, 0]
    plan = sc.plan_create("A(i,l,m)=B(i,j,k)*C(j,l)*D(k,m)", csf,
                          [sc.dense_view(None, "f32", 5, 8), sc.dense_view(None, "f32", 6, 8)], sc.schedule("fused"))
    assert sc.plan_tile_count(plan) == 0


@pytest.mark.parametrize("cid,scale,temps", [
    (1, 1.0, ["T(i,j,m)"]), (2, 0.002, ["T(i,j,r)"]), (4, 0.002, ["T(i,j)"]), (5, 0.01, ["T1(i,j,k,n)", "T2(i,j,m,n)"])])
def test_derived_temporaries_and_workspace(cid, scale, temps):
    """The temporaries' index sets follow from the split positions (Section 4.2): indices of
    the producer that also occur in the consumer or the output."""
    cfg, data, csf = _small(cid, scale)
    plan = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fissioned", temps, [0] * len(temps)))
    text = sc.plan_describe(plan)
    for t in temps:
        assert t in text
    esz = 8 if cfg["dtype"] == "f64" else 4
    order = len(cfg["dims"])
    ranks = cfg["ranks"]
    if cfg["kind"] == "ttmc4":
        shapes = [(csf.nfib[2], ranks[2]), (csf.nfib[1], ranks[1] * ranks[2])]
    elif cfg["kind"] == "sddmm_spmm":
        shapes = [(csf.nnz, 1)]
    else:
        shapes = [(csf.nfib[order - 2], ranks[-1])]
    need = 0
    for t, (rows, cols) in enumerate(shapes):
        off, r, c = sc.plan_intermediate(plan, t)
        assert (r, c) == (rows, cols) and off == need and off % 256 == 0
        need += (rows * cols * esz + 255) // 256 * 256
    assert sc.plan_workspace_bytes(plan) == need
    # same index set in another order is accepted; a wrong set, a wrong count or a fuse depth are not
    assert _status(sc.plan_create, cfg["expr"], csf, data["factors"],
                   sc.schedule("fissioned", [temps[0].replace("(i,j", "(j,i")] + temps[1:], [0] * len(temps))) == "SC_OK"
    assert _status(sc.plan_create, cfg["expr"], csf, data["factors"],
                   sc.schedule("fissioned", ["T(i,q)"] + temps[1:], [0] * len(temps))) == "SC_ERR_SCHED_UNSUPPORTED"
    assert _status(sc.plan_create, cfg["expr"], csf, data["factors"],
                   sc.schedule("fissioned", temps + ["X(i)"], [0] * (len(temps) + 1))) in ("SC_ERR_SCHED_UNSUPPORTED",)
    assert _status(sc.plan_create, cfg["expr"], csf, data["factors"],
                   sc.schedule("fissioned", temps, [1] * len(temps))) == "SC_ERR_SCHED_UNSUPPORTED"
    # FUSED: the fuse depth is 0 (the library's) or the depth its kernel is built at; other depths are refused, not ignored
    built = 2 if cfg["kind"] in ("mttkrp3", "sddmm_spmm") else 1
    fused = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fused", temps, [built] * len(temps)))
    assert sc.plan_workspace_bytes(fused) == 0
    assert _status(sc.plan_intermediate, fused, 0) == "SC_ERR_SCHED_UNSUPPORTED"
    assert sc.plan_chosen(fused) == ("fused", 0)
    for depth in (1, 2, 3):
        if depth != built:
            assert _status(sc.plan_create, cfg["expr"], csf, data["factors"],
                           sc.schedule("fused", temps, [depth] * len(temps))) == "SC_ERR_SCHED_UNSUPPORTED"


def test_expression_family():
    cfg, data, csf = _small(3, 0.002)
    f = data["factors"]
    ok = sc.schedule("fused")
    # free index names, factors in either order, "+=" accepted
    assert _status(sc.plan_create, "Out(a,x,y) += Bt(a,b,c) * Dm(c,y) * Cm(b,x)", csf, [f[1], f[0]], ok) == "SC_OK"
    assert _status(sc.plan_create, "A(i,l,m)=B(i,j,k)*C(j,l)*D(k,m", csf, f, ok) == "SC_ERR_EXPR_PARSE"
    assert _status(sc.plan_create, "A(i,l,m)=B(i,j,k)*C(j,l)+D(k,m)", csf, f, ok) == "SC_ERR_EXPR_PARSE"
    assert _status(sc.plan_create, "A(l,m,i)=B(i,j,k)*C(j,l)*D(k,m)", csf, f, ok) == "SC_ERR_EXPR_UNSUPPORTED"
    assert _status(sc.plan_create, "A(l,m,n)=B(i,j,k)*C(i,l)*D(j,m)", csf, f, ok) == "SC_ERR_EXPR_UNSUPPORTED"
    assert _status(sc.plan_create, "A(i,m,l)=B(i,j,k)*C(j,l)*D(k,m)", csf, f, ok) == "SC_ERR_EXPR_UNSUPPORTED"
    assert _status(sc.plan_create, "A(i,l)=B(i,j)*C(j,l)", csf, f[:1], ok) == "SC_ERR_EXPR_UNSUPPORTED"
    assert _status(sc.plan_create, "A(i,l,m,n)=B(i,j,k,p)*C(j,l)*D(k,m)*E(p,n)", csf, f + [f[0]], ok) == "SC_ERR_BAD_ORDER"
    assert _status(sc.plan_create, cfg["expr"], csf, f[:1], ok) == "SC_ERR_SHAPE_MISMATCH"
    assert _status(sc.plan_create, cfg["expr"], csf, [f[1], f[0]], ok) == "SC_ERR_SHAPE_MISMATCH"   # rows != dims
    assert _status(sc.plan_create, cfg["expr"], csf, [f[0].astype(np.float64), f[1]], ok) == "SC_ERR_BAD_DTYPE"
    assert _status(sc.plan_create, cfg["expr"], csf, f, sc.schedule("linear", deterministic=True)) == "SC_ERR_SCHED_UNSUPPORTED"
    assert _status(sc.plan_create, cfg["expr"], csf, f, sc.Schedule(kind=7)) == "SC_ERR_SCHED_UNSUPPORTED"
    assert _status(sc.plan_create, cfg["expr"], csf, f, sc.Schedule(kind=sc.SC_SCHED_FUSED, deterministic=2)) == "SC_ERR_SCHED_UNSUPPORTED"
    odd = np.ones((cfg["dims"][2], 12), np.float32)   # a rank no kernel is instantiated for
    assert _status(sc.plan_create, cfg["expr"], csf, [f[0], odd], ok) == "SC_ERR_SCHED_UNSUPPORTED"


def test_structure_validation_errors():
    cfg, data, csf = _small(3, 0.002)
    f, ok = data["factors"], sc.schedule("fused")

    def broken(mutate):
        c = sc.Csf(csf.order, csf.dims, csf.nnz, csf.dtype_code, csf.nfib, [None] + [p.copy() for p in csf.pos[1:]],
                   [x.copy() for x in csf.crd], csf.vals, False)
        mutate(c)
        return _status(sc.plan_create, cfg["expr"], c, f, ok)

    def swap_pos(c): c.pos[2][3], c.pos[2][4] = c.pos[2][4], c.pos[2][3]
    def empty_node(c): c.pos[1][2] = c.pos[1][1]
    def bad_end(c): c.pos[2][-1] += 1
    def crd_range(c): c.crd[2][5] = cfg["dims"][2]
    def crd_neg(c): c.crd[1][0] = -1
    def unsorted_leaf(c):
        lo, hi = c.pos[2][np.argmax(np.diff(c.pos[2]) >= 2)], 0
        c.crd[2][lo], c.crd[2][lo + 1] = c.crd[2][lo + 1], c.crd[2][lo]
    def dup_leaf(c):
        lo = c.pos[2][np.argmax(np.diff(c.pos[2]) >= 2)]
        c.crd[2][lo + 1] = c.crd[2][lo]
    def dup_slice(c): c.crd[0][1] = c.crd[0][0]
    def nfib_mismatch(c): c.nfib = (c.nfib[0], c.nfib[1], c.nfib[2] - 1)
    def too_many_slices(c): c.dims = (c.nfib[0] - 1,) + tuple(c.dims[1:])

    assert broken(swap_pos) == "SC_ERR_BAD_POS"
    assert broken(empty_node) == "SC_ERR_BAD_POS"
    assert broken(bad_end) == "SC_ERR_BAD_POS"
    assert broken(crd_range) == "SC_ERR_CRD_RANGE"
    assert broken(crd_neg) == "SC_ERR_CRD_RANGE"
    assert broken(unsorted_leaf) == "SC_ERR_UNSORTED"
    assert broken(dup_leaf) == "SC_ERR_DUPLICATE"
    assert broken(dup_slice) == "SC_ERR_DUPLICATE"
    assert broken(nfib_mismatch) == "SC_ERR_BAD_DIMS"
    assert broken(too_many_slices) in ("SC_ERR_BAD_DIMS", "SC_ERR_CRD_RANGE")
    assert sc.lib().sc_plan_create(None, b"x", None, None, 0, None) == sc.STATUS_NAMES.index("SC_ERR_NULL")

    # Node counts are checked before any array is sized from them, for device views too (whose arrays would
    # have to be copied first): a negative or oversized count is an error status, never an exception that
    # crosses the C boundary.
    def device_view(nfib):
        c = sc.Csf(csf.order, csf.dims, csf.nnz, csf.dtype_code, nfib, csf.pos, csf.crd, csf.vals, True)
        return _status(sc.plan_create, cfg["expr"], c, f, ok)

    assert device_view((-5, csf.nfib[1], csf.nfib[2])) == "SC_ERR_BAD_DIMS"
    assert device_view((csf.nfib[0], -1, csf.nfib[2])) == "SC_ERR_BAD_DIMS"
    assert device_view((csf.nfib[0], csf.nfib[2] + 1, csf.nfib[2])) == "SC_ERR_BAD_DIMS"
    assert device_view((csf.nfib[0], csf.nfib[1], csf.nfib[2] + 7)) == "SC_ERR_BAD_DIMS"


def test_factors_of_2_gib_or_more_are_refused_at_plan_time():
    """Factor rows are addressed with 31-bit byte offsets (bit 31 is the end-of-node mark of the walks):
    a factor that spans 2 GiB or more is refused when the plan is made, for every schedule."""
    cfg, data, csf = _small(2, 0.002)
    J, K = cfg["dims"][1], cfg["dims"][2]
    for which in ("fused", "fissioned"):
        # bare shapes (no data): C with 2^31 bytes of rows x cols
        big_rows = (1 << 31) // (32 * 4)
        c2 = sc.Csf(csf.order, (csf.dims[0], big_rows, K), csf.nnz, csf.dtype_code, csf.nfib, csf.pos, csf.crd, csf.vals, False)
        fac = [sc.dense_view(None, "f32", rows=big_rows, cols=32), sc.dense_view(None, "f32", rows=K, cols=32)]
        assert _status(sc.plan_create, cfg["expr"], c2, fac, sc.schedule(which)) == "SC_ERR_SHAPE_MISMATCH"
        fac = [sc.dense_view(None, "f32", rows=big_rows - 1, cols=32), sc.dense_view(None, "f32", rows=K, cols=32)]
        c3 = sc.Csf(csf.order, (csf.dims[0], big_rows - 1, K), csf.nnz, csf.dtype_code, csf.nfib, csf.pos, csf.crd, csf.vals, False)
        assert _status(sc.plan_create, cfg["expr"], c3, fac, sc.schedule(which)) == "SC_OK"


@pytest.mark.parametrize("cid,scale,which", [(2, 0.004, "fused"), (2, 0.004, "fissioned"), (3, 0.003, "fused"),
                                             (4, 0.003, "fused"), (5, 0.004, "fused"), (1, 1.0, "fissioned")])
def test_tiles_partition_the_nonzeros(cid, scale, which):
    """Tiles are contiguous, cover every nonzero once, respect their caps, and their node
    ranges and continuation flags agree with the CSF pos arrays."""
    cfg, data, csf = _small(cid, scale)
    plan = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule(which))
    nt = sc.plan_tile_count(plan)
    recs = np.array([sc.plan_tile(plan, i) for i in range(nt)])
    text = sc.plan_describe(plan)
    caps = [int(x) for x in re.search(r"tiles: \d+ \(<= (\d+) leaves, <= (\d+) level-a", text).groups()]
    order = csf.order
    assert recs[0, 0] == 0 and recs[-1, 1] == csf.nnz
    np.testing.assert_array_equal(recs[1:, 0], recs[:-1, 1])
    sizes = recs[:, 1] - recs[:, 0]
    assert sizes.min() >= 1 and sizes.max() <= caps[0]
    assert recs[:, 3].max() <= caps[1]
    levels = [(order - 1, 2, 3)] + ([(order - 2, 4, 5)] if order >= 3 else []) + ([(order - 3, 6, 7)] if order >= 4 else [])
    # leaf index -> node index at each level above
    idx_lo, idx_hi = recs[:, 0].copy(), recs[:, 1] - 1
    lo_leaf, hi_leaf = recs[:, 0], recs[:, 1]
    for depth, (lvl, c0, cn) in enumerate(levels):
        pos = csf.pos[lvl]
        first = np.searchsorted(pos, idx_lo, side="right") - 1
        last = np.searchsorted(pos, idx_hi, side="right") - 1
        np.testing.assert_array_equal(recs[:, c0], first)
        np.testing.assert_array_equal(recs[:, cn], last - first + 1)
        # leaf range covered by the first / last node, to check the continuation flags
        start_leaf, end_leaf = pos[first], pos[last + 1]
        for deeper in range(lvl + 1, order):
            start_leaf, end_leaf = csf.pos[deeper][start_leaf], csf.pos[deeper][end_leaf]
        np.testing.assert_array_equal((recs[:, 8] >> (2 * depth)) & 1, (start_leaf < lo_leaf).astype(int))
        np.testing.assert_array_equal((recs[:, 8] >> (2 * depth + 1)) & 1, (end_leaf > hi_leaf).astype(int))
        idx_lo, idx_hi = first, last


def test_tuning_knobs_and_lds_limit():
    cfg, data, csf = _small(3, 0.003)
    try:
        sc.tuning_set("tile_leaves", 256)
        plan = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fused"))
        recs = np.array([sc.plan_tile(plan, i) for i in range(sc.plan_tile_count(plan))])
        assert (recs[:, 1] - recs[:, 0]).max() <= 256
        sc.tuning_set("tile_nodes_a", 1 << 14)   # T rows would not fit in LDS
        assert _status(sc.plan_create, cfg["expr"], csf, data["factors"], sc.schedule("fused")) == "SC_ERR_SCHED_UNSUPPORTED"
        assert _status(sc.tuning_set, "no_such_knob", 1) == "SC_ERR_EXPR_PARSE"
        sc.tuning_set("persistent_per_cu", 2)
        sc.tuning_set("tile_interleave", 8)
        assert _status(sc.tuning_set, "persistent_per_cu", -1) == "SC_ERR_BAD_DIMS"
    finally:
        for k in ("tile_leaves", "tile_nodes_a", "tile_nodes_b", "persistent_per_cu", "tile_interleave"):
            sc.tuning_set(k, 0)


def test_execute_without_gpu_or_with_host_views_is_refused():
    cfg, data, csf = _small(3, 0.002)
    plan = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fused"))
    out = np.zeros(synth.output_shape(cfg), np.float32)
    # host views are never executable: the library has no CPU path
    assert _status(sc.execute, plan, csf, data["factors"], out) == "SC_ERR_DEVICE"


def test_model_counts():
    cfg, data, csf = _small(3, 0.002)
    plan = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fused"))
    flops, byts = sc.plan_model(plan)
    L, M = cfg["ranks"]
    assert flops == 2 * M * csf.nnz + 2 * L * M * csf.nfib[1]
    fis = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fissioned"))
    assert sc.plan_model(fis)[1] == byts + 2 * csf.nfib[1] * M * 4


def test_stream_copy_argument_checks():
    """The calibration copy validates its arguments on the host before any launch."""
    lib = sc.lib()
    buf = np.zeros(64, dtype=np.uint8)
    p = buf.ctypes.data & ~15
    assert lib.sc_stream_copy(None, ctypes.c_void_p(p), ctypes.c_size_t(16), None) == sc.STATUS_NAMES.index("SC_ERR_NULL")
    assert lib.sc_stream_copy(ctypes.c_void_p(p + 16), ctypes.c_void_p(p), ctypes.c_size_t(12), None) == sc.STATUS_NAMES.index("SC_ERR_BAD_DIMS")
    assert lib.sc_stream_copy(ctypes.c_void_p(p + 17), ctypes.c_void_p(p), ctypes.c_size_t(16), None) == sc.STATUS_NAMES.index("SC_ERR_BAD_DIMS")
    assert lib.sc_stream_copy(ctypes.c_void_p(p + 16), ctypes.c_void_p(p), ctypes.c_size_t(0), None) == 0


@pytest.mark.parametrize("which", ["fused", "fissioned"])
@pytest.mark.parametrize("cid,dtype,ranks", [
    (2, "f32", (8,)), (2, "f32", (16,)), (2, "f32", (32,)), (2, "f32", (64,)), (2, "f64", (8,)), (2, "f64", (64,)),
    (3, "f32", (8, 16)), (3, "f32", (16, 16)), (3, "f32", (16, 64)), (3, "f64", (16, 16)),
    (4, "f32", (16, 16)), (4, "f32", (128, 128)), (4, "f64", (64, 64)),
    (5, "f32", (4, 8, 8)), (5, "f32", (16, 8, 8)), (5, "f64", (8, 8, 8))])
def test_built_in_tile_caps_fit_every_supported_rank(cid, dtype, ranks, which):
    """The built-in tile caps must satisfy the LDS and staging limits of every kernel a plan
    launches, for every rank / dtype combination the library accepts."""
    cfg = synth.config(cid, 0.002)
    cfg["dtype"], cfg["ranks"] = dtype, ranks
    data = synth.generate(cfg)
    csf = sc.coo_to_csf(list(data["coords"]), data["vals"], cfg["dims"])
    plan = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule(which))
    assert sc.plan_tile_count(plan) > 0


@pytest.mark.parametrize("cid,scale", [(1, 1.0), (2, 0.004), (3, 0.003), (4, 0.003), (5, 0.004)])
def test_deterministic_plan_numbers_the_pieces_of_rows_that_span_tiles(cid, scale):
    """Host side of the deterministic schedules: slots are consecutive per row, in tile order,
    and the workspace holds exactly the pieces."""
    cfg, data, csf = _small(cid, scale)
    plain = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fused"))
    det = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fused", deterministic=True))
    assert sc.plan_tile_count(det) == sc.plan_tile_count(plain)
    assert sc.plan_workspace_bytes(plain) == 0
    text = sc.plan_describe(det)
    assert "deterministic:" in text
    rows, pieces = (int(x) for x in re.search(r"deterministic: (\d+) output rows span several tiles; their (\d+) pieces", text).groups())
    # count them again from the tile table: a tile's first top-level node continues from the
    # previous tile (one piece), its last continues into the next (one piece, unless it is that same node)
    in_bit, out_bit, ntop_i = {"ttmc4": (16, 32, 7), "sddmm_spmm": (1, 2, 3)}.get(cfg["kind"], (4, 8, 5))
    want_pieces = want_rows = 0
    for i in range(sc.plan_tile_count(det)):
        rec = sc.plan_tile(det, i)
        fl, ntop = rec[8], rec[ntop_i]
        if fl & in_bit:
            want_pieces += 1
        if (fl & out_bit) and not ((fl & in_bit) and ntop == 1):
            want_pieces += 1
            want_rows += 1
    assert (rows, pieces) == (want_rows, want_pieces) and pieces >= 2 * rows > 0
    elem = 8 if cfg["dtype"] == "f64" else 4
    row_bytes = int(np.prod(synth.output_shape(cfg)[1:])) * elem
    segments = int(re.search(r"\((\d+) segments of at most 64\)", text).group(1))
    assert rows <= segments <= rows + pieces // 64
    # the pieces, then (256-byte aligned) one partial sum per segment
    assert sc.plan_workspace_bytes(det) == ((pieces * row_bytes + 255) & ~255) + segments * row_bytes


def test_deterministic_is_refused_where_no_kernel_provides_it():
    cfg = synth.config(5, 0.004)
    cfg["dtype"] = "f64"   # the fp64 order-4 kernel sums with LDS atomics
    data = synth.generate(cfg)
    csf = sc.coo_to_csf(list(data["coords"]), data["vals"], cfg["dims"])
    for which in ("fused", "fissioned"):
        assert _status(sc.plan_create, cfg["expr"], csf, data["factors"], sc.schedule(which, deterministic=True)) == "SC_ERR_SCHED_UNSUPPORTED"


def test_deterministic_fissioned_order4_plan_numbers_the_rows_of_both_temporaries():
    cfg, data, csf = _small(5, 0.004)
    det = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fissioned", deterministic=True))
    plain = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fissioned"))
    text = sc.plan_describe(det)
    found = {name: (int(r), int(p)) for r, name, p in re.findall(r"deterministic: (\d+) rows of (T\d)\S* span several tiles; (\d+) pieces", text)}
    want = {"T1": [0, 0], "T2": [0, 0]}
    for i in range(sc.plan_tile_count(det)):
        rec = sc.plan_tile(det, i)
        fl, na, nb = rec[8], rec[3], rec[5]
        for name, bit_in, bit_out, n in (("T1", 1, 2, na), ("T2", 4, 8, nb)):
            if fl & bit_in:
                want[name][1] += 1
            if (fl & bit_out) and not ((fl & bit_in) and n == 1):
                want[name][1] += 1
                want[name][0] += 1
    for name in ("T1", "T2"):
        assert found.get(name, (0, 0)) == tuple(want[name])
    assert want["T2"][0] > 0   # the skewed tensor has level-b nodes cut by tile boundaries
    assert sc.plan_workspace_bytes(det) > sc.plan_workspace_bytes(plain) > 0


@pytest.mark.parametrize("cid,scale", [(1, 1.0), (2, 0.004), (3, 0.003)])
def test_deterministic_fissioned_plan_also_numbers_the_rows_of_the_temporary(cid, scale):
    cfg, data, csf = _small(cid, scale)
    det = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fissioned", deterministic=True))
    plain = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fissioned"))
    text = sc.plan_describe(det)
    m = re.search(r"deterministic: (\d+) rows of T\S* span several tiles; (\d+) pieces \((\d+) segments\)", text)
    rows, pieces, segments = (int(x) for x in m.groups()) if m else (0, 0, 0)   # no line when no fiber spans tiles
    want_rows = want_pieces = 0
    for i in range(sc.plan_tile_count(det)):
        rec = sc.plan_tile(det, i)
        fl, na = rec[8], rec[3]
        if fl & 1:
            want_pieces += 1
        if (fl & 2) and not ((fl & 1) and na == 1):
            want_pieces += 1
            want_rows += 1
    assert (rows, pieces) == (want_rows, want_pieces)
    assert sc.plan_workspace_bytes(det) > sc.plan_workspace_bytes(plain) > 0


@pytest.mark.parametrize("cid,scale", [(1, 1.0), (2, 0.002), (3, 0.002), (4, 0.002), (5, 0.002)])
def test_linear_plan_counts_the_unfactored_nest(cid, scale):
    """LINEAR plans: no temporary, no workspace, and the flop model is the unfactored count
    (a multiply per operand and an add, for every stored entry and every combination of the
    dense output indices; Section 1 gives nnz * L * M for the order-3 chain)."""
    cfg, data, csf = _small(cid, scale)
    plan = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("linear"))
    ranks = [f.shape[1] for f in data["factors"]]
    nnz = csf.nnz
    want = {"ttmc3": 3 * ranks[0] * ranks[1] * nnz, "mttkrp3": 3 * ranks[0] * nnz,
            "sddmm_spmm": 4 * ranks[0] * ranks[2] * nnz if cfg["kind"] == "sddmm_spmm" else 0,
            "ttmc4": 4 * int(np.prod(ranks)) * nnz}[cfg["kind"]]
    assert sc.plan_model(plan)[0] == want
    assert sc.plan_workspace_bytes(plan) == 0
    text = sc.plan_describe(plan)
    assert "LINEAR" in text and "temporary 0" not in text
    fused = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fused"))
    assert sc.plan_model(fused)[0] < want or cfg["dims"][0] < 300


def test_all_mode_ttmc_plans():
    """Kernel 5 of Table 2: classification, the three schedules picked by naming their temporaries, the
    iteration counts of their nests (the same closed forms the counted twins reproduce), refusals."""
    cfg = synth.config(6, 0.005)
    data = synth.generate(cfg)
    csf = sc.coo_to_csf(list(data["coords"]), data["vals"], cfg["dims"])
    nnz, S, F = csf.nnz, csf.nfib[0], csf.nfib[1]
    L, M, N = cfg["ranks"]
    want = {1: 2 * N * nnz + 3 * L * M * N * F, 2: 2 * N * nnz + 2 * M * N * F + 2 * L * M * N * S, 3: 3 * M * N * nnz + 2 * L * M * N * S}
    cases = [("fused", [], 2), ("fissioned", [], 2), ("fused", ["T2(i,m,n)", "T1(i,j,n)"], 2), ("fissioned", ["T(i,j,n)"], 1),
             ("fused", ["T(i,m,n)"], 3), ("fused", ["Q(n,m,i)"], 3)]
    for which, names, variant in cases:
        plan = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule(which, names, [0] * len(names)))
        text = sc.plan_describe(plan)
        assert f"kernel 5, schedule {variant}" in text, text
        assert sc.plan_model(plan)[0] == want[variant]
        ws = sc.plan_workspace_bytes(plan)
        tiles_elems = cfg["dims"][0] * M * N * 4
        assert ws >= (F * N * 4 if variant == 1 else tiles_elems)
        assert sc.plan_tile_count(plan) > 0
    # index names are free; a factor per mode in any order
    plan = sc.plan_create("Out(a,b,c)=X(p,q,r)*W(r,c)*U(p,a)*V(q,b)", csf, [data["factors"][2], data["factors"][0], data["factors"][1]],
                          sc.schedule("fused"))
    assert "kernel 5, schedule 2" in sc.plan_describe(plan)
    lin = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("linear"))
    assert sc.plan_model(lin)[0] == 4 * L * M * N * nnz and "Figure 2a" in sc.plan_describe(lin)
    bad = [("linear", ["T(i,m,n)"]), ("fused", ["T(i,j,n)"]), ("fissioned", ["T(i,m,n)"]), ("fused", ["T(i,j,m)"]), ("fused", ["T(i,j,n)", "T(i,j,n)"])]
    for which, names in bad:
        assert _status(sc.plan_create, cfg["expr"], csf, data["factors"], sc.schedule(which, names, [0] * len(names))) == "SC_ERR_SCHED_UNSUPPORTED"
    assert _status(sc.plan_create, cfg["expr"], csf, data["factors"], sc.schedule("fused", ["T(i,m,n)"], [0], deterministic=True)) == "SC_ERR_SCHED_UNSUPPORTED"
    # not in the family: an output index that is a sparse index but not the first, or two factors on one mode
    for expr in ("A(l,j,n)=B(i,j,k)*C(i,l)*D(j,m)*E(k,n)", "A(l,m,n)=B(i,j,k)*C(i,l)*D(i,m)*E(k,n)", "A(m,l,n)=B(i,j,k)*C(i,l)*D(j,m)*E(k,n)"):
        assert _status(sc.plan_create, expr, csf, data["factors"], sc.schedule("fused")) == "SC_ERR_EXPR_UNSUPPORTED"
    # shapes: the factor on mode 0 has one row per coordinate of mode 0
    wrong = [data["factors"][1], data["factors"][1], data["factors"][2]]
    assert _status(sc.plan_create, cfg["expr"], csf, wrong, sc.schedule("fused")) == "SC_ERR_SHAPE_MISMATCH"


def test_cost_evaluator_picks_a_schedule():
    """SC_SCHED_AUTO (run-time stage of Section 5): the class of least predicted time among those with kernels
    for the ranks; the decision and the candidates' figures are in the description."""
    for cid, scale in [(1, 1.0), (2, 0.004), (3, 0.003), (4, 0.003), (5, 0.004)]:
        cfg, data, csf = _small(cid, scale)
        plan = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("auto"))
        assert sc.plan_chosen(plan) == ("fused", 0), cid           # same iterations as FISSIONED, fewer bytes
        text = sc.plan_describe(plan)
        assert "cost evaluator" in text and text.count("candidate") == 3 and "<- chosen" in text
        ref = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("fused"))
        assert sc.plan_model(plan) == sc.plan_model(ref) and sc.plan_workspace_bytes(plan) == sc.plan_workspace_bytes(ref)
    # ranks no factored kernel is built for: only the unfactored nest can run them, and AUTO says so
    cfg, data, csf = _small(3, 0.003)
    odd = [np.ascontiguousarray(np.resize(f, (f.shape[0], 24))) for f in data["factors"]]
    assert _status(sc.plan_create, cfg["expr"], csf, odd, sc.schedule("fused")) == "SC_ERR_SCHED_UNSUPPORTED"
    plan = sc.plan_create(cfg["expr"], csf, odd, sc.schedule("auto"))
    assert sc.plan_chosen(plan) == ("linear", 0)
    assert "no kernel for these ranks" in sc.plan_describe(plan)
    # ... unless the caller also asks for a reproducible result, which the unfactored nest cannot give
    assert _status(sc.plan_create, cfg["expr"], csf, odd, sc.schedule("auto", deterministic=True)) == "SC_ERR_SCHED_UNSUPPORTED"
    # AUTO takes no temporaries or depths from the caller
    assert _status(sc.plan_create, cfg["expr"], csf, data["factors"], sc.schedule("auto", ["T(i,j,m)"], [0])) == "SC_ERR_SCHED_UNSUPPORTED"

    # all-mode TTMC: the three schedules of Table 2 compete; the second has the fewest iterations wherever slices
    # hold several fibers, and the third takes over when the second has no kernel for the ranks
    cfg = synth.config(6, 0.005)
    data = synth.generate(cfg)
    csf = sc.coo_to_csf(list(data["coords"]), data["vals"], cfg["dims"])
    plan = sc.plan_create(cfg["expr"], csf, data["factors"], sc.schedule("auto"))
    assert sc.plan_chosen(plan) == ("fused", 2)
    assert sc.plan_describe(plan).count("candidate Table 2 schedule") == 4
    odd = [data["factors"][0]] + [np.ascontiguousarray(np.resize(f, (f.shape[0], 24))) for f in data["factors"][1:]]
    plan = sc.plan_create(cfg["expr"], csf, odd, sc.schedule("auto"))
    assert sc.plan_chosen(plan) == ("fused", 3)
    assert _status(sc.plan_create, cfg["expr"], csf, odd, sc.schedule("auto", deterministic=True)) == "SC_ERR_SCHED_UNSUPPORTED"
