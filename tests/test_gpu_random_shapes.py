"""Seeded random-shape sweep: many small problems with awkward sizes (N not a multiple of
the vector width, single rows, empty rows, g larger than any row, block rows without blocks)
through conversion and SpMM, each compared with the oracle."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import RTOL, assert_format_equal, coo_to_device, values_to_torch
from helpers import assert_spmm_close, to_f32

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", range(40))
def test_random_groupcoo_problem(seed):
    import paper_2510_17505_amd as I
    rng = np.random.default_rng(1000 + seed)
    M = int(rng.integers(1, 400))
    K = int(rng.integers(1, 400))
    N = int(rng.choice([1, 2, 3, 4, 7, 8, 12, 16, 31, 32, 64, 100, 128, 129, 256, 260, 513]))
    dtype = ["f32", "f16", "bf16"][seed % 3]
    g = int(rng.choice([0, 1, 2, 3, 4, 5, 8, 16, 33, 64, 200]))
    density = float(rng.choice([0.0, 0.002, 0.02, 0.2, 0.9]))
    nnz = int(density * M * K)
    print(f"[random groupcoo] seed={seed} M={M} K={K} N={N} g={g} {dtype} nnz={nnz}", flush=True)
    row, col, val = synth.random_coo(M, K, nnz, seed, dtype)
    if nnz > 4 and seed % 4 == 0:            # duplicates
        row = np.concatenate([row, row[:3]]); col = np.concatenate([col, col[:3]])
        val = np.concatenate([val, val[:3]])
    st = synth.storage_array(val, dtype)
    want = oracle.coo_to_groupcoo(M, K, row, col, st, g or None)
    A = I.insum_coo_to_groupcoo(M, K, *coo_to_device(row, col, val, dtype), g=g)
    assert_format_equal(A.g, A.AM, A.AK, A.AV, want)
    B = synth.round_to_dtype(rng.standard_normal((K, N)), dtype)
    gg, AM, AK, AV = want
    av = to_f32(AV, dtype)
    C0 = synth.round_to_dtype(rng.standard_normal((M, N)), dtype) if seed % 2 else None
    C64 = oracle.spmm_groupcoo(M, K, N, AM, AK, av, B, C_init=None if C0 is None else C0.astype(np.float64))
    absprod = oracle.spmm_groupcoo(M, K, N, AM, AK, np.abs(av), np.abs(B),
                                   C_init=None if C0 is None else np.abs(C0).astype(np.float64))
    Bd = values_to_torch(B, dtype)
    if C0 is None:
        C = I.insum_spmm_groupcoo(A, Bd)
    else:
        C = values_to_torch(C0, dtype)
        I.insum_spmm_groupcoo(A, Bd, C_out=C, accumulate=True)
    assert_spmm_close(C.float().cpu().numpy(), C64, absprod, RTOL[dtype], f"seed {seed}", out_dtype=dtype)
    # the product with the transposed matrix over the same arrays
    E = synth.round_to_dtype(rng.standard_normal((M, N)), dtype)
    D64 = oracle.spmm_groupcoo_transposed(M, K, N, AM, AK, av, E)
    absD = oracle.spmm_groupcoo_transposed(M, K, N, AM, AK, np.abs(av), np.abs(E))
    D = I.insum_spmm_groupcoo_transposed(A, values_to_torch(E, dtype),
                                         out_dtype=torch.float32 if seed % 2 else None)
    assert_spmm_close(D.float().cpu().numpy(), D64, absD, RTOL[dtype], f"transposed, seed {seed}",
                      out_dtype=None if seed % 2 else dtype)


@pytest.mark.parametrize("seed", range(12))
def test_random_skewed_block_rows_with_and_without_plan(seed):
    """Block rows of very different lengths (one holds hundreds of blocks, some none): with a
    plan the long one is split into chunks, without it one workgroup walks it."""
    import paper_2510_17505_amd as I
    rng = np.random.default_rng(4000 + seed)
    bM, bK = [(32, 32), (64, 32), (32, 64), (64, 64)][seed % 4]
    nbr = int(rng.integers(1, 7))
    nbc = int(rng.integers(300, 700))
    N = int(rng.choice([8, 64, 136, 256, 264, 520]))
    g = int(rng.choice([1, 2, 3, 4, 8, 70]))
    dtype = ["bf16", "f16"][seed % 2]
    occ = rng.integers(0, 6, nbr)
    occ[int(rng.integers(0, nbr))] = int(rng.integers(150, nbc))
    M, K = nbr * bM, nbc * bK
    print(f"[random skewed blocks] seed={seed} b={bM}x{bK} rows={occ.tolist()} N={N} g={g} {dtype}", flush=True)
    AMl, AKl, AVl = [], [], []
    for r, k in enumerate(occ):
        if k == 0:
            continue
        cols = np.sort(rng.choice(nbc, size=int(k), replace=False))
        ng = -(-int(k) // g)
        ak = np.concatenate([cols, np.full(ng * g - k, cols[-1])]).reshape(ng, g)
        av = synth.round_to_dtype(rng.standard_normal((ng, g, bM, bK)) * 0.5, dtype)
        av.reshape(ng * g, bM, bK)[int(k):] = 0.0
        AMl += [r] * ng
        AKl.append(ak)
        AVl.append(av)
    AM = np.array(AMl, dtype=np.int32)
    AK = np.concatenate(AKl).astype(np.int32)
    AV = np.concatenate(AVl)
    B = synth.round_to_dtype(rng.standard_normal((K, N)), dtype)
    C64 = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, AV, B)
    absprod = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, np.abs(AV), np.abs(B))
    A = I.BlockGroupCOO(M, K, bM, bK, g, torch.from_numpy(AM).cuda(), torch.from_numpy(AK).cuda(),
                        values_to_torch(AV, dtype))
    Bd = values_to_torch(B, dtype)
    planned = I.insum_spmm_blockgroupcoo(A, Bd)
    assert_spmm_close(planned.float().cpu().numpy(), C64, absprod, RTOL[dtype], f"planned, seed {seed}",
                      out_dtype=dtype)
    assert torch.equal(planned, I.insum_spmm_blockgroupcoo(A, Bd))
    unplanned = I.insum_spmm_blockgroupcoo(A, Bd, plan=False)
    assert_spmm_close(unplanned.float().cpu().numpy(), C64, absprod, RTOL[dtype], f"unplanned, seed {seed}",
                      out_dtype=dtype)


@pytest.mark.parametrize("seed", range(30))
def test_random_blockgroupcoo_problem(seed):
    import paper_2510_17505_amd as I
    rng = np.random.default_rng(2000 + seed)
    bM = int(rng.choice([1, 2, 8, 16, 32, 32, 64, 64]))
    bK = int(rng.choice([1, 4, 16, 32, 32, 64, 64, 96, 128]))
    M = bM * int(rng.integers(1, 9))
    K = bK * int(rng.integers(1, 12))
    N = int(rng.choice([1, 5, 8, 16, 24, 64, 128, 136, 256, 264, 512, 520]))
    dtype = ["bf16", "f16", "f32"][seed % 3]
    g = int(rng.choice([0, 1, 2, 3, 4, 8, 70]))
    density = float(rng.choice([0.0, 0.1, 0.5, 1.0]))
    print(f"[random blockgroupcoo] seed={seed} M={M} K={K} N={N} b={bM}x{bK} g={g} {dtype} d={density}", flush=True)
    row, col, val = synth.random_block_coo(M, K, bM, bK, seed, dtype, block_density=density, sigma=0.5,
                                           fill=1.0 if seed % 2 else 0.6)
    st = synth.storage_array(val, dtype)
    want = oracle.coo_to_blockgroupcoo(M, K, row, col, st, bM, bK, g or None)
    A = I.insum_coo_to_blockgroupcoo(M, K, *coo_to_device(row, col, val, dtype), bM, bK, g=g)
    assert_format_equal(A.g, A.AM, A.AK, A.AV, want)
    B = synth.round_to_dtype(rng.standard_normal((K, N)), dtype)
    gg, AM, AK, AV = want
    av = to_f32(AV, dtype)
    C64 = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, av, B)
    absprod = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, np.abs(av), np.abs(B))
    C = I.insum_spmm_blockgroupcoo(A, values_to_torch(B, dtype))
    assert_spmm_close(C.float().cpu().numpy(), C64, absprod, RTOL[dtype], f"seed {seed}")


@pytest.mark.parametrize("seed", range(40))
def test_random_sparse_convolution_problem(seed):
    """Random maps (repeated triples, repeated (x, z) pairs with different y, empty offsets,
    sparse and dense occupancy, all three schedules), channel counts on and off the matrix-core
    conditions, unit and general values, fresh and accumulated output."""
    import paper_2510_17505_amd as I
    from gpu_util import bits, storage_to_torch, torch_to_storage
    rng = np.random.default_rng(3000 + seed)
    X = int(rng.integers(1, 700))
    Y = int(rng.integers(1, 700))
    Z = int(rng.choice([1, 2, 3, 8, 27, 27, 40, 125]))
    C = int(rng.choice([8, 16, 24, 32, 40, 64, 72, 128, 136, 256, 12, 20, 264]))
    M = int(rng.choice([1, 8, 31, 32, 64, 65, 96, 128, 130, 200, 256]))
    dtype = ["f16", "bf16", "f32"][seed % 3] if seed % 5 else "f16"
    g = int(rng.choice([0, 1, 2, 3, 8, 16, 32, 33, 64, 256]))
    density = float(rng.choice([0.0005, 0.01, 0.05, 0.3, 0.8]))
    nnz = int(density * X * Z) + int(rng.integers(0, 3))
    unit = bool(seed % 2)
    print(f"[random spconv] seed={seed} X={X} Y={Y} Z={Z} C={C} M={M} g={g} {dtype} nnz={nnz} unit={unit}",
          flush=True)
    mx = rng.integers(0, X, nnz).astype(np.int32)
    my = rng.integers(0, Y, nnz).astype(np.int32)
    mz = rng.integers(0, Z, nnz).astype(np.int32)
    mv = np.ones(nnz, np.float32) if unit else synth.round_to_dtype(rng.standard_normal(nnz), dtype)
    st = synth.storage_array(mv, dtype)
    want = oracle.map_to_groupcoo(X, Y, Z, mx, my, mz, st, g or None)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    Map = I.insum_map_to_groupcoo(X, Y, Z, dev(mx), dev(my), dev(mz), storage_to_torch(st, dtype), g)
    gg, MZ, MX, MY, MV = want
    assert Map.g == gg and Map.G == MZ.shape[0]
    assert np.array_equal(Map.MAPZ.cpu().numpy(), MZ) and np.array_equal(Map.MAPX.cpu().numpy(), MX)
    assert np.array_equal(Map.MAPY.cpu().numpy(), MY)
    assert np.array_equal(bits(torch_to_storage(Map.MAPV)), bits(MV))
    In = synth.round_to_dtype(rng.standard_normal((Y, C)), dtype)
    W = synth.round_to_dtype(rng.standard_normal((Z, C, M)), dtype)
    mv32 = to_f32(MV, dtype)
    O0 = rng.standard_normal((X, M)).astype(np.float32) if seed % 3 == 0 else None
    O64 = oracle.spconv_groupcoo(X, C, M, MZ, MX, MY, mv32, In, W, Out_init=O0)
    absprod = oracle.spconv_groupcoo(X, C, M, MZ, MX, MY, np.abs(mv32), np.abs(In), np.abs(W),
                                     Out_init=None if O0 is None else np.abs(O0))
    if O0 is None:
        Out = I.insum_spconv_groupcoo(Map, values_to_torch(In, dtype), values_to_torch(W, dtype))
    else:
        Out = torch.from_numpy(O0.copy()).cuda()
        I.insum_spconv_groupcoo(Map, values_to_torch(In, dtype), values_to_torch(W, dtype), Out=Out,
                                accumulate=True)
    assert_spmm_close(Out.cpu().numpy(), O64, absprod, 1e-5, f"seed {seed}")
