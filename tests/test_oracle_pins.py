"""Pins for the CPU oracle: everything here checks the oracle against something other
than itself - numbers the paper prints, closed forms, structural invariants, degenerate
cases, and brute-force dense products computed with numpy / scipy."""
from __future__ import annotations

import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import synth
from helpers import (blockgroupcoo_to_dense, check_groupcoo_invariants, coo_to_dense,
                     groupcoo_to_dense, read_golden, to_f32)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _matrix_with_occupancy(occ, K, seed=0):
    rng = np.random.default_rng(seed)
    row = np.repeat(np.arange(len(occ)), occ).astype(np.int32)
    col = np.concatenate([rng.choice(K, size=k, replace=False) for k in occ]).astype(np.int32)
    val = rng.standard_normal(row.shape[0]).astype(np.float32)
    perm = rng.permutation(row.shape[0])
    return row[perm], col[perm], val[perm]


# --------------------------------------------------------------------------- #
# Section 4.1 / 4.2 worked example
# --------------------------------------------------------------------------- #
def test_worked_example_occ_3112():
    rows = read_golden(os.path.join(GOLDEN, "groupcoo_worked_example.txt"))
    occ = [int(x) for x in next(r for r in rows if r[0] == "occ")[1:]]
    row, col, val = _matrix_with_occupancy(occ, K=6)
    for r in (r for r in rows if r[0] == "g"):
        g, groups, padding, F = (int(x) for x in r[1:])
        g_used, AM, AK, AV = oracle.coo_to_groupcoo(len(occ), 6, row, col, val, g)
        assert g_used == g and AM.shape[0] == groups
        assert AK.size - row.shape[0] == padding
        assert oracle.indirect_access_cost(occ, g) == F
        assert F == AM.size + AK.size        # one scatter per group, one gather per slot
        check_groupcoo_invariants(len(occ), 6, row, col, val, g, AM, AK, AV)
    for r in (r for r in rows if r[0] == "AM"):
        g = int(r[1])
        _, AM, _, _ = oracle.coo_to_groupcoo(len(occ), 6, row, col, val, g)
        assert AM.tolist() == [int(x) for x in r[2:]]


def test_g1_is_coo_and_gmax_is_ell():
    """Section 4.1: group size 1 is COO, group size max occupancy is ELL."""
    M, K = 37, 53
    row, col, val = synth.random_coo(M, K, 300, seed=3)
    order = np.lexsort((np.arange(row.size), col, row))
    g, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, 1)
    assert np.array_equal(AM, row[order])
    assert np.array_equal(AK[:, 0], col[order])
    assert np.array_equal(AV[:, 0].view(np.uint32), val[order].view(np.uint32))
    occ = np.bincount(row, minlength=M)
    g, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, int(occ.max()))
    assert np.array_equal(AM, np.flatnonzero(occ))        # one group per non-empty row
    for p, i in enumerate(AM):                             # ELL row = sorted columns + padding
        cols = np.sort(col[row == i])
        assert np.array_equal(AK[p, :cols.size], cols)
        assert np.all(AK[p, cols.size:] == cols[-1])
        assert np.all(AV[p, cols.size:].view(np.uint32) == 0)


def test_canonical_order_matches_lexsort():
    rng = np.random.default_rng(5)
    row = rng.integers(0, 9, 500).astype(np.int32)
    col = rng.integers(0, 7, 500).astype(np.int32)     # many duplicates: ties by position
    perm = oracle.canonical_order(9, 7, row, col)
    assert np.array_equal(perm, np.lexsort((np.arange(500), col, row)))


@pytest.mark.parametrize("g", [1, 2, 3, 4, 7, 16, 64])
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_groupcoo_invariants_and_roundtrip(g, dtype):
    M, K = 61, 45
    row, col, val = synth.zipf_rows_coo(M, K, 1.2, 6.0, seed=g, dtype=dtype, values="normal")
    # add empty rows, explicit zeros and duplicate coordinates
    keep = (row % 5) != 2
    row, col, val = row[keep], col[keep], val[keep].copy()
    val[::11] = 0.0
    row = np.concatenate([row, row[:7]])
    col = np.concatenate([col, col[:7]])
    val = np.concatenate([val, val[:7] * 2])
    st = synth.storage_array(val, dtype)
    g_used, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, st, g)
    check_groupcoo_invariants(M, K, row, col, st, g, AM, AK, AV)
    A1 = coo_to_dense(M, K, row, col, val.astype(np.float64))
    A2 = groupcoo_to_dense(M, K, AM, AK, to_f32(AV, dtype).astype(np.float64))
    assert np.array_equal(A1, A2) or np.allclose(A1, A2, rtol=0, atol=1e-12)


def test_groupcoo_errors_and_empty():
    with pytest.raises(oracle.OracleError) as e:
        oracle.coo_to_groupcoo(4, 4, [0, 4], [0, 0], np.ones(2, np.float32), 2)
    assert e.value.code == oracle.ERR_OUT_OF_RANGE
    with pytest.raises(oracle.OracleError):
        oracle.coo_to_groupcoo(4, 4, [0, 1], [0, -1], np.ones(2, np.float32), 2)
    g, AM, AK, AV = oracle.coo_to_groupcoo(4, 4, [], [], np.zeros(0, np.float32), 2)
    assert AM.shape == (0,) and AK.shape == (0, 2) and AV.shape == (0, 2)
    g, AM, AK, AV = oracle.coo_to_groupcoo(4, 4, [], [], np.zeros(0, np.float32), None)
    assert g == 1


# --------------------------------------------------------------------------- #
# Section 4.2: group size
# --------------------------------------------------------------------------- #
def test_group_size_matches_the_papers_choices():
    gold = {r[0]: r[1:] for r in read_golden(os.path.join(GOLDEN, "ablation_shape.txt"))}
    M, K = int(gold["M"][0]), int(gold["K"][0])
    bM, bK = (int(x) for x in gold["block"])
    density = 1.0 - int(gold["sparsity_percent"][0]) / 100.0
    S_rows = round(density * M * K)
    assert oracle.default_group_size(S_rows, M) == int(gold["group_size_rows"][0])
    S_blocks = round(density * (M // bM) * (K // bK))
    assert oracle.default_group_size(S_blocks, M // bM) == int(gold["group_size_block_rows"][0])


def test_group_size_rule_properties():
    rng = np.random.default_rng(0)
    for _ in range(300):
        n = int(rng.integers(1, 10**6))
        S = int(rng.integers(0, 10**9))
        g = oracle.default_group_size(S, n)
        assert g >= 1 and (g & (g - 1)) == 0
        if S >= 2 * n:                   # nearest power of two in log2: g/sqrt2 <= g* < g*sqrt2
            gs = oracle.gstar(S, n)
            assert g / np.sqrt(2) <= gs * (1 + 1e-12) and gs < g * np.sqrt(2) * (1 + 1e-12)
        else:
            assert g == 1
    assert oracle.default_group_size(0, 10) == 1
    # exact interval edges: S = 2n rounds up to 2, S = 2n-1 stays at 1; S = 8n -> 4
    assert oracle.default_group_size(2 * 1000 - 1, 1000) == 1
    assert oracle.default_group_size(2 * 1000, 1000) == 2
    assert oracle.default_group_size(8 * 1000 - 1, 1000) == 2
    assert oracle.default_group_size(8 * 1000, 1000) == 4


def test_relaxed_cost_and_gstar():
    S, n = 12345.0, 321.0
    gs = oracle.gstar(S, n)
    assert gs == pytest.approx(np.sqrt(S / n), rel=1e-15)
    f0 = oracle.relaxed_cost(S, n, gs)
    assert f0 == pytest.approx(S + n + 2 * np.sqrt(S * n), rel=1e-12)   # minimum value
    for eps in (0.9, 0.99, 1.01, 1.1):
        assert oracle.relaxed_cost(S, n, gs * eps) > f0
    # ceil(x) <= x + 1  =>  F(g) <= relaxed cost, with equality never exceeded
    rng = np.random.default_rng(1)
    occ = rng.integers(0, 40, 200)
    for g in (1, 2, 3, 5, 8, 16, 40):
        F = oracle.indirect_access_cost(occ, g)
        assert F == (g + 1) * int(np.sum(-(-occ // g)))
        assert F <= oracle.relaxed_cost(occ.sum(), occ.size, g) + 1e-9


def test_heuristic_is_near_the_brute_force_optimum():
    """Section 4.2 calls g* 'nearly optimal' for F(g); report the ratio, require only a
    loose bound so a broken rule (e.g. S/n instead of sqrt) fails."""
    rng = np.random.default_rng(2)
    for mean in (3, 16, 100):
        occ = rng.poisson(mean, 500)
        best = min(oracle.indirect_access_cost(occ, g) for g in range(1, int(occ.max()) + 1))
        g = oracle.default_group_size(int(occ.sum()), occ.size)
        assert oracle.indirect_access_cost(occ, g) <= 1.35 * best


def test_memory_ratio_69_percent():
    """Section 6.5: GroupCOO (g = 16) takes 69 % of COO's memory on the ablation matrix.
    Holds only with 32-bit indices and 32-bit values and one AM entry per group."""
    gold = {r[0]: r[1:] for r in read_golden(os.path.join(GOLDEN, "ablation_shape.txt"))}
    M, K = int(gold["M"][0]), int(gold["K"][0])
    bM, bK = (int(x) for x in gold["block"])
    row, col, val = synth.random_block_coo(M, K, bM, bK, seed=0, dtype="f32",
                                           block_density=0.10)
    g, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, None)
    assert g == int(gold["group_size_rows"][0])
    assert AK.size == row.size                                   # no padding on this matrix
    coo_bytes = row.nbytes + col.nbytes + val.nbytes
    ratio = (AM.nbytes + AK.nbytes + AV.nbytes) / coo_bytes
    assert round(100 * ratio) == int(gold["groupcoo_over_coo_memory_percent"][0])
    assert ratio == pytest.approx((4 / 16 + 4 + 4) / 12)


# --------------------------------------------------------------------------- #
# BlockGroupCOO
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("bM,bK,g", [(2, 2, 1), (4, 2, 2), (2, 8, 3), (8, 8, 4)])
def test_blockgroupcoo_structure_and_roundtrip(bM, bK, g):
    M, K = 8 * bM, 6 * bK
    row, col, val = synth.random_block_coo(M, K, bM, bK, seed=bM + g, dtype="bf16",
                                           block_density=0.4, fill=0.7)
    st = synth.storage_array(val, "bf16")
    g_used, AM, AK, AV = oracle.coo_to_blockgroupcoo(M, K, row, col, st, bM, bK, g)
    G = AM.shape[0]
    assert AK.shape == (G, g) and AV.shape == (G, g, bM, bK)
    blocks = np.unique(np.stack([row // bM, col // bK], 1), axis=0)     # sorted (br, bc)
    occ = np.bincount(blocks[:, 0], minlength=M // bM)
    assert G == int(np.sum((occ + g - 1) // g))
    assert np.all(np.diff(AM) >= 0)
    # the sequence of real blocks equals the sorted distinct block list
    real = []
    for p in range(G):
        j = p - int(np.searchsorted(AM, AM[p]))
        nreal = min(g, occ[AM[p]] - j * g)
        for q in range(g):
            if q < nreal:
                real.append((AM[p], AK[p, q]))
            else:
                assert AK[p, q] == AK[p, nreal - 1]
                assert not AV[p, q].any()
    assert np.array_equal(np.array(real), blocks)
    A1 = coo_to_dense(M, K, row, col, val.astype(np.float64))
    A2 = blockgroupcoo_to_dense(M, K, bM, bK, AM, AK, to_f32(AV, "bf16").astype(np.float64))
    assert np.array_equal(A1, A2)


def test_block_1x1_is_groupcoo_and_g1_is_blockcoo():
    M, K = 24, 30
    row, col, val = synth.random_coo(M, K, 150, seed=9)
    g1, AM1, AK1, AV1 = oracle.coo_to_groupcoo(M, K, row, col, val, 4)
    g2, AM2, AK2, AV2 = oracle.coo_to_blockgroupcoo(M, K, row, col, val, 1, 1, 4)
    assert np.array_equal(AM1, AM2) and np.array_equal(AK1, AK2)
    assert np.array_equal(AV1.view(np.uint32), AV2.reshape(AV1.shape).view(np.uint32))
    # g = 1: BlockCOO - one (block row, block col) per stored block, sorted
    row, col, val = synth.random_block_coo(M, K, 4, 5, seed=1, dtype="f32", block_density=0.3)
    g, AM, AK, AV = oracle.coo_to_blockgroupcoo(M, K, row, col, val, 4, 5, 1)
    blocks = np.unique(np.stack([row // 4, col // 5], 1), axis=0)
    assert np.array_equal(np.stack([AM, AK[:, 0]], 1), blocks)


def test_block_errors():
    one = np.ones(2, np.float32)
    with pytest.raises(oracle.OracleError) as e:
        oracle.coo_to_blockgroupcoo(8, 8, [1, 1], [2, 2], one, 2, 2, 1)
    assert e.value.code == oracle.ERR_DUPLICATE
    with pytest.raises(oracle.OracleError) as e:
        oracle.coo_to_blockgroupcoo(9, 8, [1, 2], [2, 2], one, 2, 2, 1)
    assert e.value.code == oracle.ERR_UNSUPPORTED
    with pytest.raises(oracle.OracleError) as e:
        oracle.coo_to_blockgroupcoo(8, 8, [1, 8], [2, 2], one, 2, 2, 1)
    assert e.value.code == oracle.ERR_OUT_OF_RANGE
    # an explicit zero still marks its block
    g, AM, AK, AV = oracle.coo_to_blockgroupcoo(8, 8, [5], [2], np.zeros(1, np.float32), 2, 2, 1)
    assert AM.tolist() == [2] and AK.tolist() == [[1]]
    # default group size uses blocks per block row
    row, col, val = synth.random_block_coo(4096, 4096, 32, 32, seed=0, dtype="f32",
                                           block_density=0.10, fill=0.02)
    g, AM, AK, AV = oracle.coo_to_blockgroupcoo(4096, 4096, row, col, val, 32, 32, None)
    assert g == 4


# --------------------------------------------------------------------------- #
# SpMM against dense products
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("g", [1, 2, 5, 8])
def test_spmm_groupcoo_equals_dense_gemm(g):
    M, K, N = 23, 31, 9                       # all different: a transposed operand fails
    row, col, val = synth.random_coo(M, K, 200, seed=g)
    row = np.concatenate([row, row[:5]])      # duplicates are summed (Section 3.1)
    col = np.concatenate([col, col[:5]])
    val = np.concatenate([val, val[:5]])
    B = np.random.default_rng(g).standard_normal((K, N)).astype(np.float32)
    _, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, g)
    C = oracle.spmm_groupcoo(M, K, N, AM, AK, AV, B)
    A = coo_to_dense(M, K, row, col, val.astype(np.float64))
    assert np.allclose(C, A @ B.astype(np.float64), rtol=1e-13, atol=1e-13)
    # accumulate into an existing C
    C0 = np.random.default_rng(1).standard_normal((M, N))
    C2 = oracle.spmm_groupcoo(M, K, N, AM, AK, AV, B, C_init=C0)
    assert np.allclose(C2, C0 + A @ B.astype(np.float64), rtol=1e-13, atol=1e-13)


def test_spmm_groupcoo_medium_against_scipy_and_g_invariance():
    M, K, N = 700, 900, 33
    row, col, val = synth.zipf_rows_coo(M, K, 1.2, 16.0, seed=4, values="inv_deg")
    B = synth.round_to_dtype(np.random.default_rng(3).standard_normal((K, N)), "f32")
    ref = sp.csr_matrix((val.astype(np.float64), (row, col)), shape=(M, K)) @ B.astype(np.float64)
    results = []
    for g in (1, 2, 4, 16, 128):
        _, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, g)
        C = oracle.spmm_groupcoo(M, K, N, AM, AK, AV, B)
        assert np.allclose(C, ref, rtol=1e-12, atol=1e-13)
        results.append(C)
        # a padding slot may point at any valid column without changing the result
        occ = np.bincount(row, minlength=M)
        AK2 = AK.copy()
        for p in range(AM.shape[0]):
            j = p - int(np.searchsorted(AM, AM[p]))
            nreal = min(g, occ[AM[p]] - j * g)
            AK2[p, nreal:] = (AK2[p, nreal:] + 17) % K
        assert np.array_equal(oracle.spmm_groupcoo(M, K, N, AM, AK2, AV, B), C)
    for C in results[1:]:
        assert np.allclose(C, results[0], rtol=1e-12, atol=1e-14)
    # linearity in B
    _, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, 4)
    B2 = np.random.default_rng(8).standard_normal((K, N)).astype(np.float32)
    lhs = oracle.spmm_groupcoo(M, K, N, AM, AK, AV, B) + oracle.spmm_groupcoo(M, K, N, AM, AK, AV, B2)
    both = sp.csr_matrix((val.astype(np.float64), (row, col)), shape=(M, K)) @ \
        (B.astype(np.float64) + B2.astype(np.float64))
    assert np.allclose(lhs, both, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("bM,bK,g", [(2, 3, 1), (4, 4, 2), (8, 2, 3)])
def test_spmm_blockgroupcoo_equals_dense_gemm(bM, bK, g):
    M, K, N = 6 * bM, 5 * bK, 7
    row, col, val = synth.random_block_coo(M, K, bM, bK, seed=g, dtype="bf16",
                                           block_density=0.5, sigma=1.0, fill=0.8)
    st = synth.storage_array(val, "bf16")
    B = synth.round_to_dtype(np.random.default_rng(g).standard_normal((K, N)), "bf16")
    _, AM, AK, AV = oracle.coo_to_blockgroupcoo(M, K, row, col, st, bM, bK, g)
    C = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, to_f32(AV, "bf16"), B)
    A = coo_to_dense(M, K, row, col, val.astype(np.float64))
    assert np.allclose(C, A @ B.astype(np.float64), rtol=1e-13, atol=1e-13)
    C0 = np.ones((M, N))
    C2 = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, to_f32(AV, "bf16"), B, C_init=C0)
    assert np.allclose(C2, 1.0 + A @ B.astype(np.float64), rtol=1e-13, atol=1e-13)


def test_spmm_handles_empty_format():
    C = oracle.spmm_groupcoo(3, 4, 5, np.zeros(0, np.int32), np.zeros((0, 2), np.int32),
                             np.zeros((0, 2), np.float32), np.ones((4, 5), np.float32))
    assert C.shape == (3, 5) and not C.any()


def test_scatter_and_gather_counts():
    """Section 6.5 listing: COO issues NNZ*N scatter updates, GroupCOO (NNZ/g)*N; with
    padding the exact counts are G*N scatters and g*G*N gathers = F(g)*N in total."""
    M, K, N, g = 50, 50, 8, 4
    row, col, val = synth.random_coo(M, K, 400, seed=0)
    _, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, g)
    occ = np.bincount(row, minlength=M)
    assert (AM.size + AK.size) * N == oracle.indirect_access_cost(occ, g) * N
    _, AM1, AK1, _ = oracle.coo_to_groupcoo(M, K, row, col, val, 1)
    assert AM1.size * N == row.size * N


# --------------------------------------------------------------------------- #
# Section 4.2, last paragraph: the powers of two around g*
# --------------------------------------------------------------------------- #
def test_enclosing_powers_of_two():
    # the paper's two cases (Section 6.5): g* = 20.2 lies between 16 and 32, g* = 3.58 between 2 and 4
    assert oracle.enclosing_powers_of_two(1677722, 4096) == (16, 32)
    assert oracle.enclosing_powers_of_two(1638, 128) == (2, 4)
    assert oracle.enclosing_powers_of_two(16 * 7, 7) == (4, 4)      # g* = 4 exactly
    assert oracle.enclosing_powers_of_two(3, 7) == (1, 1)           # g* < 1: group size 1
    assert oracle.enclosing_powers_of_two(0, 5) == (1, 1)
    rng = np.random.default_rng(0)
    for _ in range(2000):
        n = int(rng.integers(1, 1 << 20))
        S = int(rng.integers(n, n << 12))                 # g* in [1, 64]
        lo, hi = oracle.enclosing_powers_of_two(S, n)
        # the definition, in rationals: lo^2 <= S/n <= hi^2, both powers of two, hi/lo in {1, 2}
        assert lo & (lo - 1) == 0 and hi & (hi - 1) == 0 and hi in (lo, 2 * lo)
        assert lo * lo * n <= S <= hi * hi * n
        assert (hi == lo) == (lo * lo * n == S)
        assert oracle.default_group_size(S, n) in (lo, hi)    # the nearest of the two in log2
        gs = np.sqrt(S / n)
        if abs(np.log2(gs) - round(np.log2(gs))) > 1e-9:      # away from exact powers: plain floats agree
            assert lo == 2 ** int(np.floor(np.log2(gs))) and hi == 2 * lo


# --------------------------------------------------------------------------- #
# product with the transposed matrix over the same format
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("g", [1, 3, 4, 16])
def test_spmm_groupcoo_transposed_equals_dense_gemm(g):
    M, K, N = 23, 31, 7                                    # M != K != N: a swapped operand cannot pass
    rng = np.random.default_rng(g)
    row, col, val = synth.random_coo(M, K, 120, seed=g, dtype="f32")
    E = rng.standard_normal((M, N)).astype(np.float32)
    _, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, g)
    D = oracle.spmm_groupcoo_transposed(M, K, N, AM, AK, AV, E)
    A = coo_to_dense(M, K, row, col, val.astype(np.float64))
    assert np.allclose(D, A.T @ E.astype(np.float64), rtol=1e-12, atol=1e-12)
    # accumulating into an existing D
    D0 = rng.standard_normal((K, N))
    D2 = oracle.spmm_groupcoo_transposed(M, K, N, AM, AK, AV, E, D_init=D0)
    assert np.allclose(D2, D0 + A.T @ E.astype(np.float64), rtol=1e-12, atol=1e-12)
    # adjoint identity with the forward product: <A B, E> = <B, A^T E>
    B = rng.standard_normal((K, N)).astype(np.float32)
    C = oracle.spmm_groupcoo(M, K, N, AM, AK, AV, B)
    assert np.isclose(np.sum(C * E), np.sum(B.astype(np.float64) * D), rtol=1e-11)


def test_spmm_groupcoo_transposed_medium_against_scipy():
    M, K, N = 3000, 2000, 48
    row, col, val = synth.zipf_rows_coo(M, K, 1.2, 8.0, seed=2, dtype="f32", values="normal")
    row = np.concatenate([row, row[:100]])                 # duplicates add up
    col = np.concatenate([col, col[:100]])
    val = np.concatenate([val, val[:100]])
    E = np.random.default_rng(1).standard_normal((M, N)).astype(np.float32)
    want = sp.csr_matrix((val.astype(np.float64), (row, col)), shape=(M, K)).T @ E.astype(np.float64)
    for g in (1, 4, 7):
        _, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, g)
        D = oracle.spmm_groupcoo_transposed(M, K, N, AM, AK, AV, E)
        assert np.allclose(D, want, rtol=1e-11, atol=1e-11)
    # a padding slot's column does not matter (its value is zero)
    _, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, 4)
    AK2 = AK.copy()
    AK2[AV == 0] = 0
    assert np.allclose(oracle.spmm_groupcoo_transposed(M, K, N, AM, AK2, AV, E), want, rtol=1e-11, atol=1e-11)


# --------------------------------------------------------------------------- #
# GroupCOO of the transposed matrix, built from the format
# --------------------------------------------------------------------------- #
def test_real_slots_by_hand():
    AK = np.array([[2, 5, 5], [7, 7, 7], [1, 1, 4], [3, 3, 3]], dtype=np.int32)
    AV = np.array([[1, 2, 0], [3, 0, 0], [0, 5, 6], [0, 0, 9]], dtype=np.float32)
    want = np.array([[1, 1, 0], [1, 0, 0],
                     [1, 1, 1],            # a zero in slot 0 is an entry; the repeated column carries 5
                     [1, 0, 1]], dtype=bool)   # a +0 repeat is dropped, the nonzero repeat after it is kept
    assert np.array_equal(oracle.groupcoo_real_slots(AK, AV), want)
    AVn = AV.copy()
    AVn[1, 1] = -0.0                       # -0 is not the padding pattern
    assert oracle.groupcoo_real_slots(AK, AVn)[1, 1]
    # 16-bit values
    assert np.array_equal(oracle.groupcoo_real_slots(AK, AV.astype(np.float16)), want)


@pytest.mark.parametrize("g,g_t", [(1, 1), (4, 4), (3, 5), (16, 2)])
def test_groupcoo_transpose_is_the_format_of_the_transposed_matrix(g, g_t):
    M, K = 37, 23                                          # M != K
    row, col, val = synth.zipf_rows_coo(M, K, 1.2, 4.0, seed=g, dtype="f32", values="normal")
    row = np.concatenate([row, row[:9]])                   # repeated coordinates stay separate entries
    col = np.concatenate([col, col[:9]])
    val = np.concatenate([val, 2 * val[:9]])
    _, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, g)
    assert int(oracle.groupcoo_real_slots(AK, AV).sum()) == row.size
    gt, AMt, AKt, AVt = oracle.groupcoo_transpose(M, K, AM, AK, AV, g_t)
    assert gt == g_t
    # the matrix it holds is the transpose, value for value
    A = coo_to_dense(M, K, row, col, val.astype(np.float64))
    assert np.array_equal(groupcoo_to_dense(K, M, AMt, AKt, AVt.astype(np.float64)), A.T)
    # and it is a valid GroupCOO of the exchanged coordinates (structure checked independently)
    check_groupcoo_invariants(K, M, col, row, val, g_t, AMt, AKt, AVt)
    # the same arrays as converting the exchanged COO directly: entries with equal coordinates
    # keep their order, because the format stores them in input order
    _, AMd, AKd, AVd = oracle.coo_to_groupcoo(K, M, col, row, val, g_t)
    assert np.array_equal(AMt, AMd) and np.array_equal(AKt, AKd)
    assert np.array_equal(AVt.view(np.uint32), AVd.view(np.uint32))


def test_groupcoo_transpose_twice_is_the_identity():
    M, K = 50, 64
    row, col, val = synth.random_coo(M, K, 400, seed=5, dtype="f16")
    val = synth.storage_array(val, "f16")
    g, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, 4)
    _, AMt, AKt, AVt = oracle.groupcoo_transpose(M, K, AM, AK, AV, 8)
    g2, AM2, AK2, AV2 = oracle.groupcoo_transpose(K, M, AMt, AKt, AVt, 4)
    assert g2 == g and np.array_equal(AM2, AM) and np.array_equal(AK2, AK)
    assert np.array_equal(AV2.view(np.uint16), AV.view(np.uint16))
    # default group size: the Section 4.2 rule on the entries and the rows of A^T
    gd, *_ = oracle.groupcoo_transpose(M, K, AM, AK, AV)
    assert gd == oracle.default_group_size(400, K)


def test_groupcoo_transpose_product_agrees_with_the_transposed_product():
    M, K, N = 40, 30, 5
    row, col, val = synth.random_coo(M, K, 300, seed=8, dtype="f32")
    E = np.random.default_rng(0).standard_normal((M, N)).astype(np.float32)
    _, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, val, 4)
    _, AMt, AKt, AVt = oracle.groupcoo_transpose(M, K, AM, AK, AV, 4)
    D1 = oracle.spmm_groupcoo_transposed(M, K, N, AM, AK, AV, E)
    D2 = oracle.spmm_groupcoo(K, M, N, AMt, AKt, AVt, E)
    assert np.allclose(D1, D2, rtol=1e-12, atol=1e-12)
