"""Pins of the CPU oracle against things other than itself (no GPU needed).

The paper prints no numeric tensor values for these contractions, so the
oracle is pinned by construction: hand-computed worked examples
(tests/golden), brute-force dense einsum on tiny tensors, linearity, closed
forms, reduction to library routines (scipy SpMM, dense matmul), invariance
under COO permutation, and fused-vs-fissioned agreement through the named
intermediates (Section 4.2).  Shapes are deliberately non-square with distinct
extents per index so that a transposed operand or swapped index cannot pass.
"""
import json
import os

import numpy as np
import pytest
import scipy.sparse as sp

HERE = os.path.dirname(os.path.abspath(__file__))

EINSUM = {
    "ttmc3": "ijk,jl,km->ilm",
    "mttkrp3": "ijk,jr,kr->ir",
    "ttmc4": "ijkp,jl,km,pn->ilmn",
    "ttmc_all": "ijk,il,jm,kn->lmn",
    "mttkrp_gemm": "ijk,jr,kr,rm->im",
    "sddmm_spmm_gemm": "ij,ik,jk,jl,lm->im",
}


def _random_case(kind, rng, dims, nnz, ranks, empty_rows=()):
    order = len(dims)
    space = int(np.prod(dims))
    flat = rng.choice(space, size=nnz, replace=False)
    coords = np.array(np.unravel_index(flat, dims), dtype=np.int32)
    keep = ~np.isin(coords[0], list(empty_rows))
    coords = coords[:, keep]
    vals = rng.uniform(-1, 1, coords.shape[1])
    if kind == "ttmc3":
        shapes = [(dims[1], ranks[0]), (dims[2], ranks[1])]
    elif kind == "mttkrp3":
        shapes = [(dims[1], ranks[0]), (dims[2], ranks[0])]
    elif kind == "sddmm_spmm":
        shapes = [(dims[0], ranks[0]), (dims[1], ranks[0]), (dims[1], ranks[1])]
    elif kind == "ttmc_all":
        shapes = [(dims[0], ranks[0]), (dims[1], ranks[1]), (dims[2], ranks[2])]
    elif kind == "mttkrp_gemm":
        shapes = [(dims[1], ranks[0]), (dims[2], ranks[0]), (ranks[0], ranks[1])]
    elif kind == "sddmm_spmm_gemm":
        shapes = [(dims[0], ranks[0]), (dims[1], ranks[0]), (dims[1], ranks[1]), (ranks[1], ranks[2])]
    else:
        shapes = [(dims[1], ranks[0]), (dims[2], ranks[1]), (dims[3], ranks[2])]
    factors = [rng.standard_normal(s) for s in shapes]
    assert order == coords.shape[0]
    return coords, vals, factors


def _dense(coords, vals, dims):
    B = np.zeros(dims)
    np.add.at(B, tuple(coords), vals)
    return B


def _brute(kind, coords, vals, dims, factors):
    B = _dense(coords, vals, dims)
    if kind == "sddmm_spmm_gemm":
        X, Y, Z, F = factors
        return ((B * (X @ Y.T)) @ Z) @ F
    if kind == "sddmm_spmm":
        X, Y, Z = factors
        return (B * (X @ Y.T)) @ Z
    return np.einsum(EINSUM[kind], B, *factors)


CASES = [
    ("ttmc3", (5, 6, 7), 60, (2, 3)),
    ("ttmc3", (4, 9, 3), 108, (3, 2)),   # every coordinate stored: full slices
    ("mttkrp3", (5, 6, 7), 70, (3,)),
    ("sddmm_spmm", (6, 7), 20, (3, 4)),
    ("ttmc4", (3, 4, 5, 6), 90, (2, 3, 4)),
    ("ttmc_all", (5, 6, 7), 60, (2, 3, 4)),
    ("ttmc_all", (4, 3, 9), 108, (4, 2, 3)),   # every coordinate stored
    ("mttkrp_gemm", (5, 6, 7), 70, (3, 4)),
    ("sddmm_spmm_gemm", (6, 7), 20, (3, 4, 2)),
]


def test_golden_worked_examples(oracle):
    g = json.load(open(os.path.join(HERE, "golden", "worked_examples.json")))
    for kind in ("ttmc3", "mttkrp3", "sddmm_spmm", "ttmc4", "ttmc_all", "mttkrp_gemm", "sddmm_spmm_gemm"):
        e = g[kind]
        A = oracle.contract(kind, np.array(e["coords"]), np.array(e["vals"], float), e["dims"],
                            [np.array(f, float) for f in e["factors"]])
        assert np.array_equal(A, np.array(e["expected"], float)), kind


@pytest.mark.parametrize("kind,dims,nnz,ranks", CASES)
def test_bruteforce_dense_einsum(oracle, kind, dims, nnz, ranks):
    rng = np.random.default_rng(7)
    coords, vals, factors = _random_case(kind, rng, dims, nnz, ranks, empty_rows=(1,))
    A = oracle.contract(kind, coords, vals, dims, factors)
    ref = _brute(kind, coords, vals, dims, factors)
    assert A.shape == ref.shape
    np.testing.assert_allclose(A, ref, rtol=0, atol=1e-12 * max(1.0, np.abs(ref).max()))
    if kind != "ttmc_all":   # (its output has no sparse index)
        assert np.all(A[1] == 0.0)  # the emptied slice gives an exactly-zero row


@pytest.mark.parametrize("kind,dims,nnz,ranks", CASES)
def test_single_and_multi_thread_agree(oracle, kind, dims, nnz, ranks):
    rng = np.random.default_rng(8)
    coords, vals, factors = _random_case(kind, rng, dims, nnz, ranks)
    a1 = oracle.contract(kind, coords, vals, dims, factors, nthreads=1)
    a4 = oracle.contract(kind, coords, vals, dims, factors, nthreads=4)
    assert np.array_equal(a1, a4)  # rows are disjoint: threading cannot change rounding


@pytest.mark.parametrize("kind,dims,nnz,ranks", CASES)
def test_linearity_in_each_factor(oracle, kind, dims, nnz, ranks):
    rng = np.random.default_rng(9)
    coords, vals, factors = _random_case(kind, rng, dims, nnz, ranks)
    alpha, beta = 0.75, -1.5
    for n in range(len(factors)):
        other = rng.standard_normal(factors[n].shape)
        f_a = list(factors)
        f_b = list(factors); f_b[n] = other
        f_mix = list(factors); f_mix[n] = alpha * factors[n] + beta * other
        lhs = oracle.contract(kind, coords, vals, dims, f_mix)
        rhs = alpha * oracle.contract(kind, coords, vals, dims, f_a) + beta * oracle.contract(kind, coords, vals, dims, f_b)
        np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-11)
    # ... and in the sparse values
    lhs = oracle.contract(kind, coords, 3.0 * vals, dims, factors)
    np.testing.assert_allclose(lhs, 3.0 * oracle.contract(kind, coords, vals, dims, factors), rtol=0, atol=1e-11)


@pytest.mark.parametrize("kind,dims,nnz,ranks", CASES)
def test_coo_permutation_invariance(oracle, kind, dims, nnz, ranks):
    rng = np.random.default_rng(10)
    coords, vals, factors = _random_case(kind, rng, dims, nnz, ranks)
    perm = rng.permutation(coords.shape[1])
    a = oracle.contract(kind, coords, vals, dims, factors)
    b = oracle.contract(kind, coords[:, perm], vals[perm], dims, factors)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)


def test_all_ones_factors_give_slice_sums(oracle):
    rng = np.random.default_rng(11)
    dims = (5, 6, 7)
    coords, vals, _ = _random_case("ttmc3", rng, dims, 50, (2, 3))
    slice_sum = np.bincount(coords[0], weights=vals, minlength=dims[0])
    A = oracle.contract_ttmc3(coords, vals, dims, np.ones((6, 2)), np.ones((7, 3)))
    np.testing.assert_allclose(A, np.broadcast_to(slice_sum[:, None, None], A.shape), atol=1e-13)
    A = oracle.contract_mttkrp3(coords, vals, dims, np.ones((6, 4)), np.ones((7, 4)))
    np.testing.assert_allclose(A, np.broadcast_to(slice_sum[:, None], A.shape), atol=1e-13)


def test_one_hot_factors_pick_entries(oracle):
    # C = I_J and D = I_K  =>  A(i,l,m) = B(i,l,m)
    rng = np.random.default_rng(12)
    dims = (4, 5, 6)
    coords, vals, _ = _random_case("ttmc3", rng, dims, 40, (5, 6))
    A = oracle.contract_ttmc3(coords, vals, dims, np.eye(5), np.eye(6))
    np.testing.assert_array_equal(A, _dense(coords, vals, dims))
    # order 4 likewise
    dims4 = (3, 4, 2, 5)
    coords4, vals4, _ = _random_case("ttmc4", rng, dims4, 30, (4, 2, 5))
    A4 = oracle.contract_ttmc4(coords4, vals4, dims4, np.eye(4), np.eye(2), np.eye(5))
    np.testing.assert_array_equal(A4, _dense(coords4, vals4, dims4))


def test_identity_C_reduces_to_spttm_via_scipy(oracle):
    # C = I  =>  A(i,j,m) = sum_k B(i,j,k) D(k,m): one sparse (IJ x K) matrix times D
    rng = np.random.default_rng(13)
    dims = (5, 6, 7)
    coords, vals, _ = _random_case("ttmc3", rng, dims, 80, (6, 3))
    D = rng.standard_normal((7, 3))
    A = oracle.contract_ttmc3(coords, vals, dims, np.eye(6), D)
    rows = coords[0].astype(np.int64) * 6 + coords[1]
    Bm = sp.coo_matrix((vals, (rows, coords[2])), shape=(30, 7)).tocsr()
    np.testing.assert_allclose(A.reshape(30, 3), Bm @ D, atol=1e-13)


def test_spmm_special_cases(oracle):
    # Figure 1b loop against scipy, and the order-3 kernels with a unit last mode against it
    rng = np.random.default_rng(14)
    I, J, K = 9, 11, 4
    coords, vals, _ = _random_case("sddmm_spmm", rng, (I, J), 40, (2, 2))
    C = rng.standard_normal((J, K))
    ref = sp.coo_matrix((vals, (coords[0], coords[1])), shape=(I, J)).tocsr() @ C
    np.testing.assert_allclose(oracle.contract_spmm(coords, vals, (I, J), C), ref, atol=1e-13)
    c3 = np.vstack([coords, np.zeros((1, coords.shape[1]), dtype=np.int32)])
    A = oracle.contract_ttmc3(c3, vals, (I, J, 1), C, np.ones((1, 1)))
    np.testing.assert_allclose(A[:, :, 0], ref, atol=1e-13)
    A = oracle.contract_mttkrp3(c3, vals, (I, J, 1), C, np.ones((1, K)))
    np.testing.assert_allclose(A, ref, atol=1e-13)


def test_sddmm_spmm_with_dense_ones_is_xytz(oracle):
    rng = np.random.default_rng(15)
    I, J, K, L = 5, 6, 3, 4
    ii, jj = np.meshgrid(np.arange(I), np.arange(J), indexing="ij")
    coords = np.array([ii.ravel(), jj.ravel()], dtype=np.int32)
    X, Y, Z = rng.standard_normal((I, K)), rng.standard_normal((J, K)), rng.standard_normal((J, L))
    A = oracle.contract_sddmm_spmm(coords, np.ones(I * J), (I, J), X, Y, Z)
    np.testing.assert_allclose(A, (X @ Y.T) @ Z, atol=1e-12)


def test_order4_with_unit_last_mode_is_order3(oracle):
    rng = np.random.default_rng(16)
    dims = (4, 5, 6)
    coords, vals, (C, D) = _random_case("ttmc3", rng, dims, 50, (2, 3))
    c4 = np.vstack([coords, np.zeros((1, coords.shape[1]), dtype=np.int32)])
    A4 = oracle.contract_ttmc4(c4, vals, dims + (1,), C, D, np.full((1, 1), 2.0))
    np.testing.assert_allclose(A4[..., 0], 2.0 * oracle.contract_ttmc3(coords, vals, dims, C, D), atol=1e-13)


def test_abs_bound_dominates_and_matches_bruteforce(oracle):
    rng = np.random.default_rng(17)
    for kind, dims, nnz, ranks in CASES:
        coords, vals, factors = _random_case(kind, rng, dims, nnz, ranks)
        bound = oracle.abs_bound(kind, coords, vals, dims, factors)
        ref = _brute(kind, coords, np.abs(vals), dims, [np.abs(f) for f in factors])
        np.testing.assert_allclose(bound, ref, atol=1e-12 * max(1.0, ref.max()))
        assert np.all(np.abs(oracle.contract(kind, coords, vals, dims, factors)) <= bound + 1e-14)


# --- named intermediates of the fissioned schedules --------------------------------------------

def test_prefix_structure_matches_numpy_unique(oracle):
    rng = np.random.default_rng(18)
    dims = (6, 5, 7)
    coords, vals, _ = _random_case("ttmc3", rng, dims, 90, (2, 2))
    pre, inv = oracle.prefixes(coords, dims, 2)
    pairs = np.unique(np.stack([coords[0], coords[1]], axis=1), axis=0)
    np.testing.assert_array_equal(pre.T, pairs)
    np.testing.assert_array_equal(pre[:, inv], coords[:2])


def test_leaf_intermediate_and_fissioned_agreement_order3(oracle):
    rng = np.random.default_rng(19)
    dims = (5, 6, 7)
    coords, vals, (C, D) = _random_case("ttmc3", rng, dims, 100, (2, 3))
    pre, T = oracle.intermediate_leaf(coords, vals, dims, D)   # T(i,j,m)
    # dense definition T(i,j,m) = sum_k B(i,j,k) D(k,m), restricted to stored (i,j)
    Td = np.einsum("ijk,km->ijm", _dense(coords, vals, dims), D)
    np.testing.assert_allclose(T, Td[pre[0], pre[1]], atol=1e-13)
    # D = ones => row sums are the fiber sums of vals
    _, Tones = oracle.intermediate_leaf(coords, vals, dims, np.ones((7, 1)))
    fib = np.zeros(pre.shape[1]); np.add.at(fib, oracle.prefixes(coords, dims, 2)[1], vals)
    np.testing.assert_allclose(Tones[:, 0], fib, atol=1e-13)
    # fissioned consumer  A(i,l,m) = sum_j T(i,j,m) C(j,l)  equals the linear nest
    A = np.zeros((dims[0], C.shape[1], D.shape[1]))
    np.add.at(A, pre[0], C[pre[1]][:, :, None] * T[:, None, :])
    np.testing.assert_allclose(A, oracle.contract_ttmc3(coords, vals, dims, C, D), atol=1e-12)
    # MTTKRP: A(i,r) = sum_j T(i,j,r) C(j,r)
    Cr = rng.standard_normal((6, 3))
    Am = np.zeros((dims[0], 3)); np.add.at(Am, pre[0], Cr[pre[1]] * T)
    np.testing.assert_allclose(Am, oracle.contract_mttkrp3(coords, vals, dims, Cr, D), atol=1e-12)


def test_two_level_intermediates_order4(oracle):
    rng = np.random.default_rng(20)
    dims = (3, 4, 5, 6)
    coords, vals, (C, D, E) = _random_case("ttmc4", rng, dims, 120, (2, 3, 4))
    B = _dense(coords, vals, dims)
    pre3, T1 = oracle.intermediate_leaf(coords, vals, dims, E)          # T1(i,j,k,n)
    np.testing.assert_allclose(T1, np.einsum("ijkp,pn->ijkn", B, E)[pre3[0], pre3[1], pre3[2]], atol=1e-13)
    pre2, T2 = oracle.intermediate_t2_order4(coords, vals, dims, D, E)  # T2(i,j,m,n)
    np.testing.assert_allclose(T2, np.einsum("ijkp,km,pn->ijmn", B, D, E)[pre2[0], pre2[1]], atol=1e-13)
    # T2 from T1 (second-level producer), then the final consumer
    key2 = pre3[0] * dims[1] + pre3[1]
    _, inv2 = np.unique(key2, return_inverse=True)
    T2b = np.zeros_like(T2); np.add.at(T2b, inv2, D[pre3[2]][:, :, None] * T1[:, None, :])
    np.testing.assert_allclose(T2b, T2, atol=1e-13)
    A = np.zeros((dims[0], 2, 3, 4)); np.add.at(A, pre2[0], C[pre2[1]][:, :, None, None] * T2[:, None, :, :])
    np.testing.assert_allclose(A, oracle.contract_ttmc4(coords, vals, dims, C, D, E), atol=1e-12)


def test_sampled_intermediate(oracle):
    rng = np.random.default_rng(21)
    dims = (6, 7)
    coords, vals, (X, Y, Z) = _random_case("sddmm_spmm", rng, dims, 25, (3, 4))
    t = oracle.intermediate_sampled(coords, vals, X, Y)
    ref = (_dense(coords, vals, dims) * (X @ Y.T))[coords[0], coords[1]]
    np.testing.assert_allclose(t, ref, atol=1e-13)
    A = sp.coo_matrix((t, (coords[0], coords[1])), shape=dims).tocsr() @ Z
    np.testing.assert_allclose(A, oracle.contract_sddmm_spmm(coords, vals, dims, X, Y, Z), atol=1e-12)


def test_out_of_range_coordinate_is_rejected(oracle):
    with pytest.raises(ValueError):
        oracle.contract_ttmc3(np.array([[0], [9], [0]], dtype=np.int32), np.ones(1), (2, 2, 2),
                              np.ones((2, 1)), np.ones((2, 1)))


def test_ttmc_all_is_the_mode0_contraction_of_kernel6(oracle):
    """Kernel 5 = kernel 6 (whose oracle is pinned above and against scipy) followed by the dense
    contraction of the remaining sparse mode: A(l,m,n) = sum_i C(i,l) * [sum_jk B(i,j,k) D(j,m) E(k,n)]."""
    rng = np.random.default_rng(31)
    dims, ranks = (6, 5, 7), (3, 2, 4)
    coords, vals, (C, D, E) = _random_case("ttmc_all", rng, dims, 80, ranks, empty_rows=(2,))
    A = oracle.contract("ttmc_all", coords, vals, dims, [C, D, E])
    S = oracle.contract("ttmc3", coords, vals, dims, [D, E])          # S(i,m,n)
    np.testing.assert_allclose(A, np.einsum("il,imn->lmn", C, S), rtol=0, atol=1e-12)
    # and it reduces to a dense triple product when one factor is all ones along a unit rank
    ones = np.ones((dims[0], 1))
    A1 = oracle.contract("ttmc_all", coords, vals, dims, [ones, D, E])
    np.testing.assert_allclose(A1[0], D.T @ _dense(coords, vals, dims).sum(axis=0) @ E, rtol=0, atol=1e-12)


def test_ttmc_all_closed_forms(oracle):
    rng = np.random.default_rng(32)
    dims = (4, 5, 6)
    coords, vals, _ = _random_case("ttmc_all", rng, dims, 50, (2, 3, 4))
    # all-ones factors: every output element is the sum of all stored values
    f1 = [np.ones((dims[0], 2)), np.ones((dims[1], 3)), np.ones((dims[2], 4))]
    A = oracle.contract("ttmc_all", coords, vals, dims, f1)
    np.testing.assert_allclose(A, np.full((2, 3, 4), vals.sum()), rtol=0, atol=1e-12)
    # identity factors: the output is the dense operand itself (distinct extents: a transposed mode cannot pass)
    A = oracle.contract("ttmc_all", coords, vals, dims, [np.eye(d) for d in dims])
    assert np.array_equal(A, _dense(coords, vals, dims))


def test_ttmc_all_slice_intermediate(oracle):
    """T(i,m,n) of the second and third schedule of Table 2, kernel 5, against dense einsum, and the
    output rebuilt from it (fissioned = fused = linear, Section 4.1)."""
    rng = np.random.default_rng(33)
    dims, ranks = (7, 4, 5), (3, 2, 4)
    coords, vals, (C, D, E) = _random_case("ttmc_all", rng, dims, 60, ranks, empty_rows=(3,))
    pre, T = oracle.intermediate_slice_ttmc_all(coords, vals, dims, D, E)
    dense_T = np.einsum("ijk,jm,kn->imn", _dense(coords, vals, dims), D, E)
    assert np.array_equal(pre[0], np.unique(coords[0]))
    np.testing.assert_allclose(T, dense_T[pre[0]], rtol=0, atol=1e-12)
    A = oracle.contract("ttmc_all", coords, vals, dims, [C, D, E])
    np.testing.assert_allclose(np.einsum("sl,smn->lmn", C[pre[0]], T), A, rtol=0, atol=1e-12)
    # first schedule: t(i,j,n) per fiber, then A(l,m,n) += t * C(i,l) * D(j,m)
    pre2, t = oracle.intermediate_leaf(coords, vals, dims, E)
    np.testing.assert_allclose(np.einsum("fl,fm,fn->lmn", C[pre2[0]], D[pre2[1]], t), A, rtol=0, atol=1e-12)


def test_trailing_gemm_kernels_are_their_producers_times_the_last_factor(oracle):
    """Kernels 8 and 2 of Table 2 = the MTTKRP / kernel 1 (pinned above) followed by a dense matrix
    product with the last factor (numpy matmul), on non-square shapes."""
    rng = np.random.default_rng(41)
    dims = (6, 5, 7)
    coords, vals, (C, D, E) = _random_case("mttkrp_gemm", rng, dims, 90, (3, 5), empty_rows=(4,))
    A = oracle.contract("mttkrp_gemm", coords, vals, dims, [C, D, E])
    np.testing.assert_allclose(A, oracle.contract("mttkrp3", coords, vals, dims, [C, D]) @ E, rtol=0, atol=1e-12)
    assert np.all(A[4] == 0)
    dims = (7, 6)
    coords, vals, (X, Y, Z, F) = _random_case("sddmm_spmm_gemm", rng, dims, 25, (3, 4, 5), empty_rows=(2,))
    A = oracle.contract("sddmm_spmm_gemm", coords, vals, dims, [X, Y, Z, F])
    np.testing.assert_allclose(A, oracle.contract("sddmm_spmm", coords, vals, dims, [X, Y, Z]) @ F, rtol=0, atol=1e-12)
    assert np.all(A[2] == 0)
    # an identity last factor leaves the producer's result
    A = oracle.contract("sddmm_spmm_gemm", coords, vals, dims, [X, Y, Z, np.eye(4)])
    np.testing.assert_allclose(A, oracle.contract("sddmm_spmm", coords, vals, dims, [X, Y, Z]), rtol=0, atol=1e-13)
