"""CPU pins for the sparse-convolution oracle (Section 6.4: point-cloud convolution as the
indirect Einsum Out[MAPX[p,q], m] += MAPV[p,q] * In[MAPY[p,q], c] * Weight[MAPZ[p], c, m]).

The paper prints no worked numbers for this operator, so the pins are what the mathematics
fixes: the dense definition sum_z Map[:, :, z] @ In @ W[z], special cases that are a plain
GEMM, a plain SpMM and a dense 1-D correlation, and the structure of the grouped format.
"""
from __future__ import annotations

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import synth


def _dense_map(X, Y, Z, mx, my, mz, mv):
    D = np.zeros((X, Y, Z))
    np.add.at(D, (mx, my, mz), mv.astype(np.float64))
    return D


def _case(seed, X=13, Y=11, Z=5, nnz=60, C=6, M=7):
    rng = np.random.default_rng(seed)
    mx = rng.integers(0, X, nnz).astype(np.int32)
    my = rng.integers(0, Y, nnz).astype(np.int32)
    mz = rng.integers(0, Z, nnz).astype(np.int32)
    mv = rng.normal(size=nnz).astype(np.float32)
    In = rng.normal(size=(Y, C)).astype(np.float32)
    W = rng.normal(size=(Z, C, M)).astype(np.float32)
    return X, Y, Z, mx, my, mz, mv, In, W


@pytest.mark.parametrize("g", [1, 2, 3, 8, 64])
def test_spconv_equals_the_dense_definition(g):
    X, Y, Z, mx, my, mz, mv, In, W = _case(g)
    g_used, MZ, MX, MY, MV = oracle.map_to_groupcoo(X, Y, Z, mx, my, mz, mv, g)
    got = oracle.spconv_groupcoo(X, In.shape[1], W.shape[2], MZ, MX, MY, MV, In, W)
    D = _dense_map(X, Y, Z, mx, my, mz, mv)
    want = np.einsum("xyz,yc,zcm->xm", D, In.astype(np.float64), W.astype(np.float64))
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_transposed_weight_or_swapped_xy_is_detected():
    X, Y, Z, mx, my, mz, mv, In, W = _case(3, X=9, Y=9, C=5, M=5)
    _, MZ, MX, MY, MV = oracle.map_to_groupcoo(X, Y, Z, mx, my, mz, mv, 4)
    got = oracle.spconv_groupcoo(X, 5, 5, MZ, MX, MY, MV, In, W)
    D = _dense_map(X, Y, Z, mx, my, mz, mv)
    In64, W64 = In.astype(np.float64), W.astype(np.float64)
    wrong_w = np.einsum("xyz,yc,zmc->xm", D, In64, W64)
    wrong_xy = np.einsum("yxz,yc,zcm->xm", D, In64, W64)
    right = np.einsum("xyz,yc,zcm->xm", D, In64, W64)
    assert np.abs(got - right).max() < 1e-12
    assert np.abs(got - wrong_w).max() > 1e-3 and np.abs(got - wrong_xy).max() > 1e-3


def test_identity_map_is_a_plain_gemm():
    rng = np.random.default_rng(0)
    P, C, M = 17, 9, 4
    ar = np.arange(P, dtype=np.int32)
    In = rng.normal(size=(P, C)).astype(np.float32)
    W = rng.normal(size=(1, C, M)).astype(np.float32)
    _, MZ, MX, MY, MV = oracle.map_to_groupcoo(P, P, 1, ar, ar, np.zeros(P, np.int32),
                                               np.ones(P, np.float32), 4)
    got = oracle.spconv_groupcoo(P, C, M, MZ, MX, MY, MV, In, W)
    np.testing.assert_allclose(got, In.astype(np.float64) @ W[0].astype(np.float64), rtol=1e-13)


def test_one_channel_unit_weight_is_a_plain_spmv():
    X, Y, Z, mx, my, mz, mv, In, W = _case(5, C=1, M=1, nnz=80)
    W[:] = 1.0
    _, MZ, MX, MY, MV = oracle.map_to_groupcoo(X, Y, Z, mx, my, mz, mv, 4)
    got = oracle.spconv_groupcoo(X, 1, 1, MZ, MX, MY, MV, In, W)
    A = sp.coo_matrix((mv.astype(np.float64), (mx, my)), shape=(X, Y)).tocsr()
    np.testing.assert_allclose(got, A @ In.astype(np.float64), rtol=1e-12, atol=1e-13)


def test_full_1d_grid_is_a_dense_correlation():
    """Every voxel of a 1-D line occupied, kernel of 3 taps: the sparse convolution is the
    textbook 'same' correlation out[i] = sum_d in[i + d - 1] * w[d]."""
    P = 12
    rng = np.random.default_rng(1)
    sig = rng.normal(size=P).astype(np.float32)
    w = rng.normal(size=3).astype(np.float32)
    mx, my, mz = [], [], []
    for i in range(P):
        for d in range(3):
            j = i + d - 1
            if 0 <= j < P:
                mx.append(i), my.append(j), mz.append(d)
    mx, my, mz = (np.array(a, np.int32) for a in (mx, my, mz))
    _, MZ, MX, MY, MV = oracle.map_to_groupcoo(P, P, 3, mx, my, mz, np.ones(mx.size, np.float32), 4)
    got = oracle.spconv_groupcoo(P, 1, 1, MZ, MX, MY, MV, sig[:, None], w[:, None, None])[:, 0]
    want = np.correlate(sig.astype(np.float64), w.astype(np.float64), mode="same")
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("g,dtype", [(1, "f32"), (3, "f16"), (4, "bf16"), (16, "f16")])
def test_grouped_map_structure(g, dtype):
    P, mx, my, mz, mv = synth.voxel_kernel_map(7, 0.4, seed=g, dtype=dtype, values="normal")
    Z = 27
    st = synth.storage_array(mv, dtype)
    g_used, MZ, MX, MY, MV = oracle.map_to_groupcoo(P, P, Z, mx, my, mz, st, g)
    G = MZ.shape[0]
    occ = np.bincount(mz, minlength=Z)
    assert g_used == g and G == int(np.sum(-(-occ // g)))
    assert np.all(np.diff(MZ) >= 0)                                   # grouped along z
    assert np.array_equal(np.bincount(MZ, minlength=Z), -(-occ // g))
    # real slots, read group by group, are the entries in (z, x, position) order
    order = np.lexsort((np.arange(mx.size), mx, mz))
    zero_bits = np.zeros((), st.dtype)
    slot = 0
    e = 0
    for p in range(G):
        n_real = min(g, occ[MZ[p]] - (np.sum(MZ[:p] == MZ[p]) * g))
        for q in range(g):
            if q < n_real:
                src = order[e]
                assert (MZ[p], MX[p, q], MY[p, q]) == (mz[src], mx[src], my[src])
                assert MV[p, q] == st[src]
                e += 1
            else:                                                     # padding
                assert MV[p, q].tobytes() == zero_bits.tobytes()
                assert (MX[p, q], MY[p, q]) == (MX[p, n_real - 1], MY[p, n_real - 1])
            slot += 1
    assert e == mx.size


def test_default_group_size_uses_offsets_as_rows_and_result_is_g_invariant():
    P, mx, my, mz, mv = synth.voxel_kernel_map(8, 0.5, seed=2, dtype="f32", values="normal")
    rng = np.random.default_rng(0)
    In = rng.normal(size=(P, 4)).astype(np.float32)
    W = rng.normal(size=(27, 4, 3)).astype(np.float32)
    g0, *fmt0 = oracle.map_to_groupcoo(P, P, 27, mx, my, mz, mv, None)
    assert g0 == oracle.default_group_size(mx.size, 27)
    ref = oracle.spconv_groupcoo(P, 4, 3, *fmt0, In, W)
    for g in (1, 5, 32):
        _, *fmt = oracle.map_to_groupcoo(P, P, 27, mx, my, mz, mv, g)
        np.testing.assert_allclose(oracle.spconv_groupcoo(P, 4, 3, *fmt, In, W), ref, rtol=1e-11, atol=1e-12)


def test_accumulates_into_initial_output_and_rejects_bad_coordinates():
    X, Y, Z, mx, my, mz, mv, In, W = _case(9)
    _, *fmt = oracle.map_to_groupcoo(X, Y, Z, mx, my, mz, mv, 4)
    base = np.random.default_rng(1).normal(size=(X, W.shape[2]))
    a = oracle.spconv_groupcoo(X, In.shape[1], W.shape[2], *fmt, In, W)
    b = oracle.spconv_groupcoo(X, In.shape[1], W.shape[2], *fmt, In, W, Out_init=base)
    np.testing.assert_allclose(b, a + base, rtol=1e-12, atol=1e-12)
    for arr, bound in ((mx, X), (my, Y), (mz, Z)):
        saved = arr[3]
        arr[3] = bound
        with pytest.raises(oracle.OracleError):
            oracle.map_to_groupcoo(X, Y, Z, mx, my, mz, mv, 4)
        arr[3] = saved
    g, MZ, MX, MY, MV = oracle.map_to_groupcoo(X, Y, Z, mx[:0], my[:0], mz[:0], mv[:0], 4)
    assert MZ.size == 0 and MX.shape == (0, 4)
    assert np.all(oracle.spconv_groupcoo(X, In.shape[1], W.shape[2], MZ, MX, MY, MV, In, W) == 0)


def test_voxel_map_properties():
    """The synthetic kernel map: the centre offset is the identity, offsets d and -d are
    transposes of each other, and for one offset every output has at most one input."""
    P, mx, my, mz, _ = synth.voxel_kernel_map(9, 0.35, seed=4)
    centre = mz == 13
    assert centre.sum() == P and np.array_equal(mx[centre], my[centre])
    for z in range(27):
        a = set(zip(mx[mz == z].tolist(), my[mz == z].tolist()))
        b = set(zip(my[mz == 26 - z].tolist(), mx[mz == 26 - z].tolist()))
        assert a == b
        assert len(set(mx[mz == z].tolist())) == int((mz == z).sum())
