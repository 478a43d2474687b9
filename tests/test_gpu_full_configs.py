"""The five benchmark workloads at full size, in the launch configuration bench.py times
(default group size, library conversion feeding library SpMM): conversion bit-exact and
SpMM within tolerance of the fp64 oracle on every output element."""
from __future__ import annotations

import time

import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import RTOL, assert_format_equal, coo_to_device, values_to_torch
from helpers import assert_spmm_close, to_f32

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

EXPECTED_G = {"cfg1": 2, "cfg2": 16, "cfg3": 4, "cfg3_f16": 4, "cfg4": 4, "cfg5": 4}


@pytest.mark.parametrize("name", synth.CONFIG_NAMES + ("cfg3_f16",))   # + the fp16 twin of cfg3
def test_full_config(name):
    import paper_2510_17505_amd as I
    t0 = time.time()
    print(f"[full config] {name}: generating", flush=True)
    cfg = synth.make_config(name)
    M, K, N, dt = cfg["M"], cfg["K"], cfg["N"], cfg["a_dtype"]
    st = synth.storage_array(cfg["val"], dt)
    dev = coo_to_device(cfg["row"], cfg["col"], cfg["val"], dt)
    print(f"[full config] {name}: nnz={cfg['row'].size}, converting on the GPU ({time.time()-t0:.1f}s)", flush=True)
    if cfg["kind"] == "group":
        A = I.insum_coo_to_groupcoo(M, K, *dev, g=0)
        print(f"[full config] {name}: oracle conversion ({time.time()-t0:.1f}s)", flush=True)
        want = oracle.coo_to_groupcoo(M, K, cfg["row"], cfg["col"], st, None)
    else:
        A = I.insum_coo_to_blockgroupcoo(M, K, *dev, cfg["bM"], cfg["bK"], g=0)
        print(f"[full config] {name}: oracle conversion ({time.time()-t0:.1f}s)", flush=True)
        want = oracle.coo_to_blockgroupcoo(M, K, cfg["row"], cfg["col"], st, cfg["bM"], cfg["bK"], None)
    assert A.g == EXPECTED_G[name]
    assert_format_equal(A.g, A.AM, A.AK, A.AV, want)
    del dev
    g, AM, AK, AV = want
    av = to_f32(AV, dt)
    print(f"[full config] {name}: G={AM.size}, SpMM on the GPU ({time.time()-t0:.1f}s)", flush=True)
    Bd = values_to_torch(cfg["B"], cfg["b_dtype"])
    if cfg["kind"] == "group":
        C = I.insum_spmm_groupcoo(A, Bd)
    else:
        C = I.insum_spmm_blockgroupcoo(A, Bd)
    torch.cuda.synchronize()
    got = C.float().cpu().numpy()
    del C, Bd, A
    print(f"[full config] {name}: oracle SpMM ({time.time()-t0:.1f}s)", flush=True)
    if cfg["kind"] == "group":
        C64 = oracle.spmm_groupcoo(M, K, N, AM, AK, av, cfg["B"])
        absprod = oracle.spmm_groupcoo(M, K, N, AM, AK, np.abs(av), np.abs(cfg["B"]))
    else:
        C64 = oracle.spmm_blockgroupcoo(M, K, N, cfg["bM"], cfg["bK"], AM, AK, av, cfg["B"])
        absprod = oracle.spmm_blockgroupcoo(M, K, N, cfg["bM"], cfg["bK"], AM, AK, np.abs(av),
                                            np.abs(cfg["B"]))
    print(f"[full config] {name}: comparing ({time.time()-t0:.1f}s)", flush=True)
    assert_spmm_close(got, C64, absprod, RTOL[dt], name)
    print(f"[full config] {name}: ok ({time.time()-t0:.1f}s)", flush=True)


@pytest.mark.parametrize("name", ["cfg2", "cfg3"])
def test_full_config_transposed_format(name):
    """GroupCOO of A^T built from the format at full size.  These matrices have no repeated
    coordinates, so the expected arrays are the oracle's conversion of the exchanged COO (the
    identity the CPU pins establish for the oracle's own transpose)."""
    import paper_2510_17505_amd as I
    cfg = synth.make_config(name)
    M, K, dt = cfg["M"], cfg["K"], cfg["a_dtype"]
    print(f"[full config] {name}: transposed format, nnz={cfg['row'].size}", flush=True)
    A = I.insum_coo_to_groupcoo(M, K, *coo_to_device(cfg["row"], cfg["col"], cfg["val"], dt), g=0)
    At = I.insum_groupcoo_transpose(A)
    del A
    want = oracle.coo_to_groupcoo(K, M, cfg["col"], cfg["row"], synth.storage_array(cfg["val"], dt), None)
    assert_format_equal(At.g, At.AM, At.AK, At.AV, want)
    # and both routes to A^T E at full size, every element against the oracle's transposed Einsum
    N = cfg["N"]
    print(f"[full config] {name}: A^T E on the GPU, two routes", flush=True)
    g, AM, AK, AV = oracle.coo_to_groupcoo(M, K, cfg["row"], cfg["col"], synth.storage_array(cfg["val"], dt), None)
    av = to_f32(AV, dt)
    E = synth.round_to_dtype(np.random.default_rng(5).standard_normal((M, N)).astype(np.float32), dt)
    Ed = values_to_torch(E, dt)
    through_copy = I.insum_spmm_groupcoo(At, Ed).float().cpu().numpy()
    del At
    A = I.insum_coo_to_groupcoo(M, K, *coo_to_device(cfg["row"], cfg["col"], cfg["val"], dt), g=0)
    with_atomics = I.insum_spmm_groupcoo_transposed(A, Ed).float().cpu().numpy()
    del A, Ed
    print(f"[full config] {name}: oracle A^T E", flush=True)
    D64 = oracle.spmm_groupcoo_transposed(M, K, N, AM, AK, av, E)
    absprod = oracle.spmm_groupcoo_transposed(M, K, N, AM, AK, np.abs(av), np.abs(E))
    assert_spmm_close(through_copy, D64, absprod, RTOL[dt], name + " through the transposed format",
                      out_dtype=dt if dt != "f32" else None)
    assert_spmm_close(with_atomics, D64, absprod, RTOL[dt], name + " with atomics",
                      out_dtype=dt if dt != "f32" else None)


def test_more_than_2_to_31_slots():
    """Maximum sizes: a caller-built GroupCOO matrix with 2^31 + 192 slots (the conversion takes
    fewer than 2^31 entries, the SpMM any G < 2^40), so that slot numbers pass the range of 32-bit
    integers inside the kernel.  Values are multiples of 1/8 in [-1, 1]; every element of C
    against the oracle."""
    import psutil
    import paper_2510_17505_amd as I
    free, _ = torch.cuda.mem_get_info()
    if free < (40 << 30) or psutil.virtual_memory().available < (64 << 30):
        pytest.skip("needs 40 GB of device memory and 64 GB of host memory")
    g, G = 64, (1 << 25) + 3
    M, K, N = 1 << 20, 4096, 8
    print(f"[max sizes] G={G} g={g}: {G * g} slots, generating", flush=True)
    rng = np.random.default_rng(0)
    AM = (np.arange(G, dtype=np.int64) * M // G).astype(np.int32)
    AK = rng.integers(0, K, size=(G, g), dtype=np.int32)
    AV = rng.integers(-8, 9, size=(G, g), dtype=np.int8).astype(np.float16) / np.float16(8)
    B = synth.round_to_dtype(rng.standard_normal((K, N)).astype(np.float32), "f16")
    print("[max sizes] SpMM on the GPU", flush=True)
    A = I.GroupCOO(M, K, g, torch.from_numpy(AM).cuda(), torch.from_numpy(AK).cuda(), torch.from_numpy(AV).cuda())
    C = I.insum_spmm_groupcoo(A, values_to_torch(B, "f16"), out_dtype=torch.float32)
    torch.cuda.synchronize()
    got = C.cpu().numpy()
    del A, C
    torch.cuda.empty_cache()
    print("[max sizes] oracle", flush=True)
    av = AV.astype(np.float32)
    del AV
    C64 = oracle.spmm_groupcoo(M, K, N, AM, AK, av, B)
    np.abs(av, out=av)
    absprod = oracle.spmm_groupcoo(M, K, N, AM, AK, av, np.abs(B))
    assert_spmm_close(got, C64, absprod, RTOL["f16"], "2^31 + 192 slots")


def test_block_format_with_more_than_2_to_31_values():
    """Maximum sizes for the block kernel: 524 292 blocks of 64 x 64 = 2^31 + 16 384 stored values,
    so that element offsets into AV pass the range of 32-bit integers (DMA sources, chunk bases).
    Values are multiples of 1/4 (exact in bf16); with and without a work plan, every element."""
    import psutil
    import paper_2510_17505_amd as I
    free, _ = torch.cuda.mem_get_info()
    if free < (24 << 30) or psutil.virtual_memory().available < (48 << 30):
        pytest.skip("needs 24 GB of device memory and 48 GB of host memory")
    bM = bK = 64
    g, nbr, per_row, nbc = 4, 8192, 64, 1024
    G = nbr * per_row // g + 1                       # one group more than 2^31 values
    M, K, N = (nbr + 1) * bM, nbc * bK, 16
    rng = np.random.default_rng(0)
    AM = np.concatenate([np.repeat(np.arange(nbr, dtype=np.int32), per_row // g), np.array([nbr], dtype=np.int32)])
    cols = np.sort(rng.permuted(np.tile(np.arange(nbc, dtype=np.int32), (nbr + 1, 1)), axis=1)[:, :per_row], axis=1)
    AK = np.concatenate([cols[:nbr].reshape(-1, g), cols[nbr, :g].reshape(1, g)])   # ascending inside a block row
    print(f"[max sizes] block format: {G * g} blocks, {G * g * bM * bK} values", flush=True)
    AVf = rng.integers(-4, 5, size=(G, g, bM, bK), dtype=np.int8).astype(np.float32) / 4
    B = synth.round_to_dtype(rng.standard_normal((K, N)).astype(np.float32), "bf16")
    A = I.BlockGroupCOO(M, K, bM, bK, g, torch.from_numpy(AM).cuda(), torch.from_numpy(AK).cuda(),
                        values_to_torch(AVf, "bf16"))
    Bd = values_to_torch(B, "bf16")
    planned = I.insum_spmm_blockgroupcoo(A, Bd, out_dtype=torch.float32).cpu().numpy()
    unplanned = I.insum_spmm_blockgroupcoo(A, Bd, out_dtype=torch.float32, plan=False).cpu().numpy()
    del A
    torch.cuda.empty_cache()
    print("[max sizes] block format: oracle", flush=True)
    C64 = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, AVf, B)
    np.abs(AVf, out=AVf)
    absprod = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, AVf, np.abs(B))
    assert_spmm_close(planned, C64, absprod, RTOL["bf16"], "2^31 + 16384 values, planned")
    assert_spmm_close(unplanned, C64, absprod, RTOL["bf16"], "2^31 + 16384 values, block rows in index order")


def test_output_with_more_than_2_to_31_elements():
    """Maximum sizes: C has 2^21 x 1032 = 2^31 + 2^24 elements, so element offsets into C pass
    the range of 32-bit integers.  The first and last 500 rows and 2 000 random rows are compared
    with the oracle (run on those rows' entries); rows without entries must be zero everywhere."""
    import paper_2510_17505_amd as I
    free, _ = torch.cuda.mem_get_info()
    if free < (16 << 30):
        pytest.skip("needs 16 GB of device memory")
    M, K, N, nnz = 1 << 21, 2048, 1032, 4_000_000
    rng = np.random.default_rng(0)
    row = rng.integers(0, M, nnz).astype(np.int32)
    col = rng.integers(0, K, nnz).astype(np.int32)
    val = synth.round_to_dtype(rng.standard_normal(nnz).astype(np.float32), "f16")
    B = synth.round_to_dtype(rng.standard_normal((K, N)).astype(np.float32), "f16")
    print(f"[max sizes] C with {M * N} elements", flush=True)
    A = I.insum_coo_to_groupcoo(M, K, *coo_to_device(row, col, val, "f16"), g=4)
    C = I.insum_spmm_groupcoo(A, values_to_torch(B, "f16"))
    torch.cuda.synchronize()
    sample = np.unique(np.concatenate([np.arange(500), np.arange(M - 500, M), rng.integers(0, M, 2000)]))
    keep = np.isin(row, sample)
    remap = -np.ones(M, dtype=np.int64)
    remap[sample] = np.arange(sample.size)
    g, AM, AK, AV = oracle.coo_to_groupcoo(sample.size, K, remap[row[keep]].astype(np.int32), col[keep],
                                           synth.storage_array(val[keep], "f16"), 4)
    av = to_f32(AV, "f16")
    C64 = oracle.spmm_groupcoo(sample.size, K, N, AM, AK, av, B)
    absprod = oracle.spmm_groupcoo(sample.size, K, N, AM, AK, np.abs(av), np.abs(B))
    got = C[torch.from_numpy(sample).cuda()].float().cpu().numpy()
    assert_spmm_close(got, C64, absprod, RTOL["f16"], "sampled rows", out_dtype="f16")
    empty = torch.from_numpy(np.bincount(row, minlength=M) == 0).cuda()
    assert bool((C[empty] == 0).all()) and not bool(torch.isnan(C).any())


def test_conversion_at_the_largest_matrix_shape():
    """Maximum sizes: M = K = 2^31 - 1 (62-bit sort keys, per-row arrays of 2^31 entries) with a
    few thousand entries, some in the first and last rows and columns: bit-exact."""
    import psutil
    import paper_2510_17505_amd as I
    free, _ = torch.cuda.mem_get_info()
    if free < (40 << 30) or psutil.virtual_memory().available < (40 << 30):
        pytest.skip("needs 40 GB of device memory and 40 GB of host memory")
    M = K = (1 << 31) - 1
    nnz = 5000
    rng = np.random.default_rng(0)
    row = rng.integers(0, M, nnz).astype(np.int32)
    col = rng.integers(0, K, nnz).astype(np.int32)
    row[:50], row[50:100], row[100:140] = M - 1, 0, M - 2
    col[:25], col[50:75] = K - 1, 0
    val = rng.standard_normal(nnz).astype(np.float32)
    print(f"[max sizes] conversion with M = K = {M}", flush=True)
    A = I.insum_coo_to_groupcoo(M, K, *coo_to_device(row, col, val, "f32"), g=4)
    want = oracle.coo_to_groupcoo(M, K, row, col, val, 4)
    assert_format_equal(A.g, A.AM, A.AK, A.AV, want)


@pytest.mark.parametrize("M,K", [((1 << 31) - 32, 128), (128, (1 << 31) - 32)])
def test_block_conversion_at_the_largest_extents(M, K):
    """Maximum sizes: 2^26 - 1 block rows (or block columns) of 32 x 32 blocks, a few hundred
    stored blocks that include the first and the last block row and column: bit-exact.  (The
    other extent is small because the oracle keeps a table over the whole block grid.)"""
    import paper_2510_17505_amd as I
    bM = bK = 32
    rng = np.random.default_rng(M % 1000)
    nbr, nbc = M // bM, K // bK
    br, bc = rng.integers(0, nbr, 300), rng.integers(0, nbc, 300)
    br[:20], br[20:40] = nbr - 1, 0
    bc[:10], bc[20:30] = nbc - 1, 0
    key = np.unique(br.astype(np.int64) * nbc + bc)
    rows, cols = [], []
    for r, c in zip(key // nbc, key % nbc):
        pos = rng.choice(bM * bK, size=7, replace=False)
        rows.append(r * bM + pos // bK)
        cols.append(c * bK + pos % bK)
    row, col = np.concatenate(rows).astype(np.int32), np.concatenate(cols).astype(np.int32)
    val = synth.round_to_dtype(rng.standard_normal(row.size).astype(np.float32), "bf16")
    perm = rng.permutation(row.size)
    row, col, val = row[perm], col[perm], val[perm]
    print(f"[max sizes] block conversion, M={M} K={K}", flush=True)
    want = oracle.coo_to_blockgroupcoo(M, K, row, col, synth.storage_array(val, "bf16"), bM, bK, None)
    A = I.insum_coo_to_blockgroupcoo(M, K, *coo_to_device(row, col, val, "bf16"), bM, bK, g=0)
    assert_format_equal(A.g, A.AM, A.AK, A.AV, want)


def test_map_conversion_at_the_largest_point_count():
    """Maximum sizes: a kernel map over 2^31 - 1 points (keys z * X + x of 36 bits): bit-exact."""
    import paper_2510_17505_amd as I
    rng = np.random.default_rng(3)
    X, n = (1 << 31) - 1, 4000
    mx, my = rng.integers(0, X, n).astype(np.int32), rng.integers(0, X, n).astype(np.int32)
    mz = rng.integers(0, 27, n).astype(np.int32)
    mx[:30], mx[30:60], mz[:15] = X - 1, 0, 26
    mv = synth.round_to_dtype(rng.standard_normal(n).astype(np.float32), "f16")
    g, MZ, MX, MY, MV = oracle.map_to_groupcoo(X, X, 27, mx, my, mz, synth.storage_array(mv, "f16"), None)
    Map = I.insum_map_to_groupcoo(X, X, 27, torch.from_numpy(mx).cuda(), torch.from_numpy(my).cuda(),
                                  torch.from_numpy(mz).cuda(), values_to_torch(mv, "f16"))
    assert Map.g == g and np.array_equal(Map.MAPZ.cpu().numpy(), MZ)
    assert np.array_equal(Map.MAPX.cpu().numpy(), MX) and np.array_equal(Map.MAPY.cpu().numpy(), MY)
    assert np.array_equal(Map.MAPV.cpu().numpy().view(np.uint16), MV.view(np.uint16))
