"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element, on the same seeded inputs.  Conversion must match bit for bit; SpMM must stay
within rtol = 1e-5 (fp32) / 2e-2 (fp16, bf16 with fp32 accumulation) of the fp64 oracle,
both relative to max|C| and componentwise against (|A| |B|)."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import (RTOL, TORCH_DTYPE, assert_format_equal, coo_to_device, storage_to_torch,
                      values_to_torch)
from helpers import assert_spmm_close, to_f32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def I():
    import paper_2510_17505_amd as lib
    assert torch.cuda.is_available()
    return lib


def _say(msg):
    print(msg, flush=True)


# --------------------------------------------------------------------------- #
# conversion: bit exact
# --------------------------------------------------------------------------- #
GROUP_CASES = [
    # M, K, nnz-ish, g, dtype, kind
    (1, 1, 1, 1, "f32", "uniform"),
    (5, 7, 12, 2, "f32", "uniform"),
    (61, 45, 300, 3, "f16", "zipf"),
    (512, 512, 2621, 0, "f32", "uniform"),
    (1000, 777, 20000, 4, "bf16", "zipf"),
    (3000, 5000, 60000, 16, "f16", "uniform"),
    (4096, 64, 30000, 7, "f32", "dups"),
    (20000, 30000, 250000, 0, "f32", "zipf"),
    (300, 100000, 90000, 64, "f32", "hub"),
]


def _group_case(M, K, nnz, kind, dtype, seed):
    if kind == "zipf":
        row, col, val = synth.zipf_rows_coo(M, K, 1.2, max(1.0, nnz / M), seed, dtype, "normal")
    else:
        row, col, val = synth.random_coo(M, K, nnz, seed, dtype)
    if kind == "dups":      # duplicate coordinates and explicit zeros
        row = np.concatenate([row, row[:500]])
        col = np.concatenate([col, col[:500]])
        val = np.concatenate([val, -val[:500]])
        val[::13] = 0.0
    if kind == "hub":       # one very long row, many empty rows
        keep = row % 7 == 0
        extra = np.arange(0, K, 3, dtype=np.int32)
        row = np.concatenate([row[keep], np.full(extra.size, 123, np.int32)])
        col = np.concatenate([col[keep], extra])
        val = synth.round_to_dtype(np.random.default_rng(seed).standard_normal(row.size), dtype)
        perm = np.random.default_rng(seed + 1).permutation(row.size)
        row, col, val = row[perm], col[perm], val[perm]
    return row, col, val


@pytest.mark.parametrize("M,K,nnz,g,dtype,kind", GROUP_CASES)
def test_coo_to_groupcoo_bit_exact(I, M, K, nnz, g, dtype, kind):
    _say(f"[groupcoo convert] M={M} K={K} nnz~{nnz} g={g} {dtype} {kind}")
    row, col, val = _group_case(M, K, nnz, kind, dtype, seed=nnz)
    want = oracle.coo_to_groupcoo(M, K, row, col, synth.storage_array(val, dtype), g or None)
    got = I.insum_coo_to_groupcoo(M, K, *coo_to_device(row, col, val, dtype), g=g)
    assert_format_equal(got.g, got.AM, got.AK, got.AV, want)
    # same call twice gives the same bits (no dependence on atomics' order)
    again = I.insum_coo_to_groupcoo(M, K, *coo_to_device(row, col, val, dtype), g=g)
    assert torch.equal(again.AK, got.AK) and torch.equal(again.AM, got.AM)


@pytest.mark.parametrize("M,K,nnz,g,dtype,kind", GROUP_CASES)
def test_groupcoo_transpose_bit_exact(I, M, K, nnz, g, dtype, kind):
    _say(f"[groupcoo transpose] M={M} K={K} nnz~{nnz} g={g} {dtype} {kind}")
    row, col, val = _group_case(M, K, nnz, kind, dtype, seed=nnz)
    A = I.insum_coo_to_groupcoo(M, K, *coo_to_device(row, col, val, dtype), g=g)
    g_o, AM, AK, AV = oracle.coo_to_groupcoo(M, K, row, col, synth.storage_array(val, dtype), g or None)
    for g_t in (0, 3):
        want = oracle.groupcoo_transpose(M, K, AM, AK, AV, g_t or None)
        got = I.insum_groupcoo_transpose(A, g=g_t)
        assert (got.M, got.K) == (K, M)
        assert_format_equal(got.g, got.AM, got.AK, got.AV, want)


def test_groupcoo_transpose_then_spmm_is_the_transposed_product(I):
    M, K, N = 5000, 3000, 72
    _say("[groupcoo transpose + spmm]")
    row, col, val = synth.zipf_rows_coo(M, K, 1.2, 6.0, 11, "f32", "normal")
    A = I.insum_coo_to_groupcoo(M, K, *coo_to_device(row, col, val, "f32"), g=4)
    At = I.insum_groupcoo_transpose(A)
    E = np.random.default_rng(3).standard_normal((M, N)).astype(np.float32)
    D = I.insum_spmm_groupcoo(At, torch.from_numpy(E).cuda())
    AM, AK, AV = A.AM.cpu().numpy(), A.AK.cpu().numpy(), A.AV.cpu().numpy()
    D64 = oracle.spmm_groupcoo_transposed(M, K, N, AM, AK, AV, E)
    absprod = oracle.spmm_groupcoo_transposed(M, K, N, AM, AK, np.abs(AV), np.abs(E))
    assert_spmm_close(D.cpu().numpy(), D64, absprod, RTOL["f32"], "A^T E through the transposed format")
    # no atomics on this route: the same bits every time
    assert torch.equal(D, I.insum_spmm_groupcoo(At, torch.from_numpy(E).cuda()))


def test_groupcoo_transpose_edge_cases(I):
    dev = "cuda"
    e = torch.zeros(0, dtype=torch.int32, device=dev)
    A0 = I.insum_coo_to_groupcoo(10, 20, e, e, torch.zeros(0, device=dev), g=4)
    At = I.insum_groupcoo_transpose(A0, g=2)
    assert (At.M, At.K, At.G, At.g) == (20, 10, 0, 2)
    # a caller-built format with a row index outside the matrix is reported, not followed
    bad = I.GroupCOO(4, 6, 2, torch.tensor([0, 9], dtype=torch.int32, device=dev),
                     torch.tensor([[1, 2], [3, 3]], dtype=torch.int32, device=dev),
                     torch.tensor([[1.0, 2.0], [3.0, 0.0]], device=dev))
    with pytest.raises(I.InsumError) as ex:
        I.insum_groupcoo_transpose(bad)
    assert ex.value.status == 2


def test_coo_to_groupcoo_edge_cases(I):
    dev = "cuda"
    e = torch.zeros(0, dtype=torch.int32, device=dev)
    f = I.insum_coo_to_groupcoo(10, 10, e, e, torch.zeros(0, device=dev), g=4)
    assert f.G == 0 and f.g == 4
    f = I.insum_coo_to_groupcoo(10, 10, e, e, torch.zeros(0, device=dev), g=0)
    assert f.g == 1
    row = torch.tensor([0, 10], dtype=torch.int32, device=dev)
    col = torch.tensor([0, 0], dtype=torch.int32, device=dev)
    with pytest.raises(I.InsumError) as ex:
        I.insum_coo_to_groupcoo(10, 10, row, col, torch.ones(2, device=dev), g=2)
    assert ex.value.status == 2
    with pytest.raises(I.InsumError) as ex:
        I.insum_coo_to_groupcoo(10, 10, col, row - 11, torch.ones(2, device=dev), g=2)
    assert ex.value.status == 2


BLOCK_CASES = [
    # M, K, bM, bK, g, dtype, density, fill
    (64, 64, 32, 32, 1, "bf16", 0.5, 1.0),
    (256, 384, 32, 32, 4, "bf16", 0.3, 1.0),
    (512, 256, 64, 64, 0, "f16", 0.4, 0.6),
    (96, 160, 8, 16, 3, "f32", 0.3, 0.5),
    (120, 90, 4, 2, 2, "f16", 0.2, 0.9),
    (2048, 2048, 32, 32, 0, "bf16", 0.1, 1.0),
    (50, 70, 1, 1, 4, "f32", 0.1, 1.0),
]


@pytest.mark.parametrize("M,K,bM,bK,g,dtype,density,fill", BLOCK_CASES)
def test_coo_to_blockgroupcoo_bit_exact(I, M, K, bM, bK, g, dtype, density, fill):
    _say(f"[blockgroupcoo convert] M={M} K={K} b={bM}x{bK} g={g} {dtype}")
    row, col, val = synth.random_block_coo(M, K, bM, bK, seed=M + bK, dtype=dtype,
                                           block_density=density, fill=fill)
    want = oracle.coo_to_blockgroupcoo(M, K, row, col, synth.storage_array(val, dtype), bM, bK, g or None)
    got = I.insum_coo_to_blockgroupcoo(M, K, *coo_to_device(row, col, val, dtype), bM, bK, g=g)
    assert_format_equal(got.g, got.AM, got.AK, got.AV, want)


def test_coo_to_blockgroupcoo_zipf_rows_and_errors(I):
    M = K = 1024
    row, col, val = synth.random_block_coo(M, K, 64, 64, seed=5, dtype="bf16", zipf_alpha=1.0,
                                           zipf_mean=4.0)
    want = oracle.coo_to_blockgroupcoo(M, K, row, col, synth.storage_array(val, "bf16"), 64, 64, None)
    got = I.insum_coo_to_blockgroupcoo(M, K, *coo_to_device(row, col, val, "bf16"), 64, 64, g=0)
    assert_format_equal(got.g, got.AM, got.AK, got.AV, want)
    r, c, v = coo_to_device(np.array([1, 1, 5]), np.array([2, 2, 3]), np.ones(3, np.float32), "f32")
    with pytest.raises(I.InsumError) as ex:
        I.insum_coo_to_blockgroupcoo(8, 8, r, c, v, 2, 2, g=1)
    assert ex.value.status == 3          # duplicate
    with pytest.raises(I.InsumError) as ex:
        I.insum_coo_to_blockgroupcoo(9, 8, r, c, v, 2, 2, g=1)
    assert ex.value.status == 5          # not divisible
    r2 = torch.tensor([1, 8], dtype=torch.int32, device="cuda")
    with pytest.raises(I.InsumError) as ex:
        I.insum_coo_to_blockgroupcoo(8, 8, r2, c[:2], v[:2], 2, 2, g=1)
    assert ex.value.status == 2          # out of range


# --------------------------------------------------------------------------- #
# SpMM over GroupCOO
# --------------------------------------------------------------------------- #
def _oracle_group_spmm(M, K, N, fmt, dtype, B, C0=None):
    g, AM, AK, AV = fmt
    av = to_f32(AV, dtype)
    C64 = oracle.spmm_groupcoo(M, K, N, AM, AK, av, B, C_init=C0)
    absprod = oracle.spmm_groupcoo(M, K, N, AM, AK, np.abs(av), np.abs(B),
                                   C_init=None if C0 is None else np.abs(C0))
    return C64, absprod


def _gpu_group_format(I, M, K, fmt, dtype):
    g, AM, AK, AV = fmt
    return I.GroupCOO(M, K, g, torch.from_numpy(AM).cuda(), torch.from_numpy(AK).cuda(),
                      storage_to_torch(AV, dtype))


SPMM_GROUP_CASES = [
    # M, K, N, nnz, g, dtype, kind
    (37, 53, 9, 300, 2, "f32", "uniform"),        # scalar path, N < 16
    (37, 53, 1, 300, 4, "f32", "uniform"),
    (200, 300, 100, 3000, 3, "f32", "uniform"),   # g not a power of two
    (512, 512, 64, 2621, 2, "f32", "uniform"),    # cfg1 shape
    (3000, 2000, 128, 50000, 4, "f32", "zipf"),   # cfg3 shape, several runs
    (3000, 2000, 130, 50000, 4, "f32", "zipf"),   # N not a multiple of 4 -> scalar path
    (3000, 2000, 132, 50000, 8, "f32", "zipf"),   # ragged last lanes
    (1000, 4096, 256, 100000, 16, "f16", "uniform"),   # cfg2 shape
    (1000, 4096, 256, 100000, 16, "bf16", "uniform"),
    (1000, 1000, 600, 20000, 4, "f32", "uniform"),     # two column tiles
    (1000, 1000, 1032, 20000, 1, "f16", "uniform"),    # g = 1 (COO), three column tiles
    (300, 100000, 128, 90000, 4, "f32", "hub"),        # one row spanning many runs
    (300, 100000, 64, 90000, 32, "f16", "hub"),
    (5000, 5000, 32, 4000, 4, "f32", "uniform"),       # mostly empty rows
    (64, 64, 24, 4096, 64, "bf16", "uniform"),         # dense matrix, g = row length
    (64, 4096, 128, 60000, 128, "f32", "uniform"),     # g larger than a sub-wave batch
    (2, 3, 5, 6, 1, "f32", "uniform"),                 # tiny dense
    (100000, 50, 16, 3000, 4, "f32", "uniform"),       # long runs of empty rows to zero-fill
]


@pytest.mark.parametrize("M,K,N,nnz,g,dtype,kind", SPMM_GROUP_CASES)
def test_spmm_groupcoo_parity(I, M, K, N, nnz, g, dtype, kind):
    _say(f"[spmm groupcoo] M={M} K={K} N={N} nnz~{nnz} g={g} {dtype} {kind}")
    row, col, val = _group_case(M, K, nnz, kind, dtype, seed=N + g)
    fmt = oracle.coo_to_groupcoo(M, K, row, col, synth.storage_array(val, dtype), g)
    B = synth.round_to_dtype(np.random.default_rng(N).standard_normal((K, N)), dtype)
    C64, absprod = _oracle_group_spmm(M, K, N, fmt, dtype, B)
    A = _gpu_group_format(I, M, K, fmt, dtype)
    Bd = values_to_torch(B, dtype)
    C = I.insum_spmm_groupcoo(A, Bd)
    assert C.dtype == TORCH_DTYPE[dtype]
    assert_spmm_close(C.float().cpu().numpy(), C64, absprod, RTOL[dtype], "C=A*B")
    # bit-reproducible (no floating-point atomics)
    C2 = I.insum_spmm_groupcoo(A, Bd)
    assert torch.equal(C, C2)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_spmm_groupcoo_accumulate_strides_and_f32_out(I, dtype):
    M, K, N, g = 700, 900, 96, 4
    row, col, val = synth.zipf_rows_coo(M, K, 1.2, 8.0, seed=2, dtype=dtype, values="normal")
    keep = row % 4 != 1                       # empty rows must keep their old contents
    row, col, val = row[keep], col[keep], val[keep]
    fmt = oracle.coo_to_groupcoo(M, K, row, col, synth.storage_array(val, dtype), g)
    B = synth.round_to_dtype(np.random.default_rng(0).standard_normal((K, N)), dtype)
    C0 = synth.round_to_dtype(np.random.default_rng(1).standard_normal((M, N)), dtype)
    C64, absprod = _oracle_group_spmm(M, K, N, fmt, dtype, B, C0.astype(np.float64))
    A = _gpu_group_format(I, M, K, fmt, dtype)
    # B and C are column slices of wider buffers: ldb, ldc > N
    Bw = torch.zeros((K, N + 32), dtype=TORCH_DTYPE[dtype], device="cuda")
    Bw[:, :N] = values_to_torch(B, dtype)
    Cw = torch.full((M, N + 16), 7.0, dtype=TORCH_DTYPE[dtype], device="cuda")
    Cw[:, :N] = values_to_torch(C0, dtype)
    I.insum_spmm_groupcoo(A, Bw[:, :N], C_out=Cw[:, :N], accumulate=True)
    assert_spmm_close(Cw[:, :N].float().cpu().numpy(), C64, absprod, RTOL[dtype], "C+=A*B")
    assert torch.all(Cw[:, N:] == 7.0), "wrote outside the N columns"
    # fp32 output for 16-bit inputs
    C64b, absb = _oracle_group_spmm(M, K, N, fmt, dtype, B)
    Cf = I.insum_spmm_groupcoo(A, Bw[:, :N], out_dtype=torch.float32)
    assert Cf.dtype == torch.float32
    assert_spmm_close(Cf.cpu().numpy(), C64b, absb, RTOL[dtype] if dtype != "f32" else 1e-5, "f32 out")


def test_spmm_groupcoo_empty_format_and_errors(I):
    A = I.GroupCOO(6, 5, 2, torch.zeros(0, dtype=torch.int32, device="cuda"),
                   torch.zeros((0, 2), dtype=torch.int32, device="cuda"),
                   torch.zeros((0, 2), device="cuda"))
    B = torch.ones((5, 12), device="cuda")
    C = torch.full((6, 12), 3.0, device="cuda")
    I.insum_spmm_groupcoo(A, B, C_out=C)
    assert not C.any()
    A2 = I.GroupCOO(6, 5, 2, torch.zeros(1, dtype=torch.int32, device="cuda"),
                    torch.zeros((1, 2), dtype=torch.int32, device="cuda"),
                    torch.zeros((1, 2), dtype=torch.float16, device="cuda"))
    with pytest.raises(I.InsumError) as ex:
        I.insum_spmm_groupcoo(A2, B)            # fp16 A with fp32 B
    assert ex.value.status == 5
    with pytest.raises(I.InsumError) as ex:     # workspace too small
        A3 = I.GroupCOO(6, 5, 2, A2.AM, A2.AK, torch.zeros((1, 2), device="cuda"))
        I.insum_spmm_groupcoo(A3, B, workspace=torch.empty(8, dtype=torch.uint8, device="cuda"))
    assert ex.value.status == 4


# --------------------------------------------------------------------------- #
# SpMM over BlockGroupCOO
# --------------------------------------------------------------------------- #
def _oracle_block_spmm(M, K, N, bM, bK, fmt, dtype, B, C0=None):
    g, AM, AK, AV = fmt
    av = to_f32(AV, dtype)
    C64 = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, av, B, C_init=C0)
    absprod = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, np.abs(av), np.abs(B),
                                        C_init=None if C0 is None else np.abs(C0))
    return C64, absprod


def _gpu_block_format(I, M, K, bM, bK, fmt, dtype):
    g, AM, AK, AV = fmt
    return I.BlockGroupCOO(M, K, bM, bK, g, torch.from_numpy(AM).cuda(), torch.from_numpy(AK).cuda(),
                           storage_to_torch(AV, dtype))


SPMM_BLOCK_CASES = [
    # M, K, N, bM, bK, g, dtype, density
    (64, 64, 64, 32, 32, 1, "bf16", 1.0),
    (256, 384, 256, 32, 32, 4, "bf16", 0.3),
    (256, 384, 512, 32, 32, 4, "f16", 0.3),
    (512, 512, 264, 64, 64, 4, "bf16", 0.4),      # ragged column tile
    (512, 512, 1000, 64, 64, 2, "f16", 0.3),
    (512, 1024, 128, 64, 32, 3, "bf16", 0.3),
    (256, 512, 72, 32, 16, 4, "bf16", 0.5),
    (256, 1024, 320, 32, 128, 2, "f16", 0.5),     # two k-chunks per block
    (256, 768, 64, 64, 48, 4, "bf16", 0.5),       # bK = 48 is not a multiple of 32 -> general kernel
    (2048, 2048, 512, 32, 32, 4, "bf16", 0.1),    # cfg4 shape, smaller
    (2048, 2048, 1024, 64, 64, 4, "bf16", 0.05),  # cfg5 shape, smaller; empty block rows
    (96, 160, 40, 8, 16, 3, "f32", 0.4),          # general kernel
    (120, 90, 33, 4, 2, 2, "f16", 0.3),
    (128, 128, 50, 16, 16, 2, "bf16", 0.5),
    (256, 256, 36, 32, 32, 4, "bf16", 0.5),       # N % 8 != 0 -> general kernel
    (128, 4800, 256, 32, 32, 1, "bf16", 0.9),     # ~135 blocks per block row: several 64-slot batches
    (128, 4800, 264, 32, 32, 7, "f16", 0.9),      # g not a power of two, ragged tile
    (128, 4800, 256, 32, 32, 128, "bf16", 0.9),   # g > 64: whole batches of padding
    (192, 6400, 512, 64, 64, 3, "bf16", 0.8),     # 80 blocks x 2 k-chunks per block row
    (64, 64, 8, 64, 64, 4, "bf16", 1.0),          # one block, N = 8 (a single 16-byte chunk)
    (512, 1024, 512, 128, 64, 2, "bf16", 0.5),    # 128-row blocks (four MFMA row tiles)
    (256, 768, 200, 128, 32, 3, "f16", 0.6),
]


@pytest.mark.parametrize("M,K,N,bM,bK,g,dtype,density", SPMM_BLOCK_CASES)
def test_spmm_blockgroupcoo_parity(I, M, K, N, bM, bK, g, dtype, density):
    _say(f"[spmm blockgroupcoo] M={M} K={K} N={N} b={bM}x{bK} g={g} {dtype}")
    row, col, val = synth.random_block_coo(M, K, bM, bK, seed=N + bK, dtype=dtype,
                                           block_density=density, sigma=0.5)
    fmt = oracle.coo_to_blockgroupcoo(M, K, row, col, synth.storage_array(val, dtype), bM, bK, g)
    B = synth.round_to_dtype(np.random.default_rng(N).standard_normal((K, N)), dtype)
    C64, absprod = _oracle_block_spmm(M, K, N, bM, bK, fmt, dtype, B)
    A = _gpu_block_format(I, M, K, bM, bK, fmt, dtype)
    Bd = values_to_torch(B, dtype)
    C = I.insum_spmm_blockgroupcoo(A, Bd)
    assert_spmm_close(C.float().cpu().numpy(), C64, absprod, RTOL[dtype], "C=A*B")
    assert torch.equal(C, I.insum_spmm_blockgroupcoo(A, Bd))


@pytest.mark.parametrize("bM,bK,N", [(32, 32, 256), (64, 64, 520), (8, 8, 40)])
def test_spmm_blockgroupcoo_accumulate_and_f32_out(I, bM, bK, N):
    M, K, g, dtype = 8 * bM, 12 * bK, 4, "bf16"
    row, col, val = synth.random_block_coo(M, K, bM, bK, seed=1, dtype=dtype, block_density=0.3,
                                           sigma=0.5)
    keep = (row // bM) != 2                      # an empty block row keeps its old contents
    row, col, val = row[keep], col[keep], val[keep]
    fmt = oracle.coo_to_blockgroupcoo(M, K, row, col, synth.storage_array(val, dtype), bM, bK, g)
    B = synth.round_to_dtype(np.random.default_rng(0).standard_normal((K, N)), dtype)
    C0 = synth.round_to_dtype(np.random.default_rng(1).standard_normal((M, N)), dtype)
    C64, absprod = _oracle_block_spmm(M, K, N, bM, bK, fmt, dtype, B, C0.astype(np.float64))
    A = _gpu_block_format(I, M, K, bM, bK, fmt, dtype)
    Bw = torch.zeros((K, N + 64), dtype=torch.bfloat16, device="cuda")
    Bw[:, :N] = values_to_torch(B, dtype)
    Cw = torch.full((M, N + 8), 7.0, dtype=torch.bfloat16, device="cuda")
    Cw[:, :N] = values_to_torch(C0, dtype)
    I.insum_spmm_blockgroupcoo(A, Bw[:, :N], C_out=Cw[:, :N], accumulate=True)
    assert_spmm_close(Cw[:, :N].float().cpu().numpy(), C64, absprod, RTOL[dtype], "C+=A*B")
    assert torch.all(Cw[:, N:] == 7.0)
    C64b, absb = _oracle_block_spmm(M, K, N, bM, bK, fmt, dtype, B)
    Cf = I.insum_spmm_blockgroupcoo(A, Bw[:, :N], out_dtype=torch.float32)
    assert_spmm_close(Cf.cpu().numpy(), C64b, absb, RTOL[dtype], "f32 out")


@pytest.mark.parametrize("bM,bK,N", [(32, 32, 256), (8, 8, 40)])
def test_spmm_blockgroupcoo_repeated_block_column_is_taken_as_padding(I, bM, bK, N):
    """The precondition stated in the header: among the real slots of a block row the block
    columns are strictly increasing, and a slot that repeats the column of the slot before it in
    its group is padding.  A hand-built format that breaks it (a repeated column with nonzero
    values) is therefore multiplied as if that slot were zero - on both kernels."""
    M, K, g, dtype = 2 * bM, 6 * bK, 3, "bf16"
    rng = np.random.default_rng(bM)
    AM = np.array([0, 1], dtype=np.int32)
    AK = np.array([[1, 4, 4], [0, 2, 5]], dtype=np.int32)          # group 0 repeats block column 4
    AV = synth.round_to_dtype(rng.standard_normal((2, g, bM, bK)) * 0.5, dtype)
    B = synth.round_to_dtype(rng.standard_normal((K, N)), dtype)
    A = I.BlockGroupCOO(M, K, bM, bK, g, torch.from_numpy(AM).cuda(), torch.from_numpy(AK).cuda(),
                        values_to_torch(AV, dtype))
    got = I.insum_spmm_blockgroupcoo(A, values_to_torch(B, dtype)).float().cpu().numpy()
    as_padding = AV.copy()
    as_padding[0, 2] = 0.0
    C64 = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, as_padding, B)
    absprod = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, np.abs(as_padding), np.abs(B))
    assert_spmm_close(got, C64, absprod, RTOL[dtype], "repeated column skipped")
    literal = oracle.spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, AV, B)   # the Einsum taken literally
    assert np.abs(literal - C64).max() > 0.1                              # ... differs: hence the precondition


def _hub_block_coo(nbr, nbc, bM, bK, occ, seed, dtype):
    """Block rows with the given numbers of blocks, block columns uniform without repetition."""
    rng = np.random.default_rng(seed)
    rows, cols = [], []
    for r, k in enumerate(occ):
        bc = np.sort(rng.choice(nbc, size=int(k), replace=False))
        rr = (r * bM + np.arange(bM))[None, :, None] + np.zeros((int(k), 1, bK), np.int64)
        cc = (bc[:, None, None] * bK + np.arange(bK)[None, None, :]) + np.zeros((1, bM, 1), np.int64)
        rows.append(rr.reshape(-1))
        cols.append(cc.reshape(-1))
    row = np.concatenate(rows).astype(np.int32)
    col = np.concatenate(cols).astype(np.int32)
    val = synth.round_to_dtype(rng.standard_normal(row.size) * 0.5, dtype)
    perm = rng.permutation(row.size)
    return row[perm], col[perm], val[perm]


@pytest.mark.parametrize("bM,bK,N,g,dtype,out32,accumulate", [
    (32, 32, 264, 3, "bf16", False, False),    # ragged column tile, g not a power of two
    (64, 64, 512, 4, "f16", True, True),       # fp32 C, accumulating: only the last chunk adds the old C
])
def test_spmm_blockgroupcoo_hub_block_row_is_split_by_the_plan(I, bM, bK, N, g, dtype, out32, accumulate):
    """One block row holds more than 2 000 blocks: the plan cuts it into chunks that different
    workgroups multiply; their fp32 tiles are added in a fixed order.  Checked against the
    oracle with and without the plan, and on repeated calls that reuse the plan."""
    nbr, nbc = 6, 2300
    occ = [3, 2100, 0, 40, 1, 700]
    M, K = nbr * bM, nbc * bK
    row, col, val = _hub_block_coo(nbr, nbc, bM, bK, occ, seed=bM + N, dtype=dtype)
    _say(f"[spmm blockgroupcoo hub] b={bM}x{bK} N={N} g={g} {dtype} nnz={row.size}")
    fmt = oracle.coo_to_blockgroupcoo(M, K, row, col, synth.storage_array(val, dtype), bM, bK, g)
    B = synth.round_to_dtype(np.random.default_rng(N).standard_normal((K, N)), dtype)
    C0 = synth.round_to_dtype(np.random.default_rng(1).standard_normal((M, N)), "f32" if out32 else dtype)
    C64, absprod = _oracle_block_spmm(M, K, N, bM, bK, fmt, dtype, B, C0.astype(np.float64) if accumulate else None)
    A = _gpu_block_format(I, M, K, bM, bK, fmt, dtype)
    Bd = values_to_torch(B, dtype)
    odt = torch.float32 if out32 else TORCH_DTYPE[dtype]

    def run(**kw):
        C = values_to_torch(C0, "f32" if out32 else dtype)
        I.insum_spmm_blockgroupcoo(A, Bd, C_out=C, accumulate=accumulate, **kw)
        assert C.dtype == odt
        return C

    ws = I.insum_spmm_blockgroupcoo_plan(A, N)
    assert ws is not None
    planned = run(workspace=ws)
    assert_spmm_close(planned.float().cpu().numpy(), C64, absprod, RTOL[dtype], "planned")
    for _ in range(3):                      # the plan (and its arrival counters) serve later calls unchanged
        assert torch.equal(planned, run(workspace=ws))
    unplanned = run(plan=False)
    assert_spmm_close(unplanned.float().cpu().numpy(), C64, absprod, RTOL[dtype], "no workspace")
    junk = torch.randint(0, 255, (ws.numel(),), dtype=torch.uint8, device="cuda")
    assert torch.equal(unplanned, run(workspace=junk))       # not a plan: ignored
    other = I.insum_spmm_blockgroupcoo_plan(A, N)            # a second plan of the same matrix
    assert torch.equal(planned, run(workspace=other))


def test_spmm_blockgroupcoo_plan_orders_rows_without_changing_results(I):
    """Zipf block rows, none long enough to be split: with a plan the block rows are issued
    longest first, each still summed by one workgroup in the same order -> identical bits."""
    M = K = 4096
    N, bM, bK, g = 1024, 64, 64, 4
    row, col, val = synth.random_block_coo(M, K, bM, bK, seed=3, dtype="bf16", zipf_alpha=1.0,
                                           zipf_mean=6.0, sigma=0.5)
    A = I.insum_coo_to_blockgroupcoo(M, K, *coo_to_device(row, col, val, "bf16"), bM, bK, g=g)
    Bd = values_to_torch(synth.round_to_dtype(np.random.default_rng(0).standard_normal((K, N)), "bf16"), "bf16")
    assert torch.equal(I.insum_spmm_blockgroupcoo(A, Bd), I.insum_spmm_blockgroupcoo(A, Bd, plan=False))
    assert N in A.plans


# --------------------------------------------------------------------------- #
# robustness
# --------------------------------------------------------------------------- #
def test_spmm_groupcoo_hub_rows_large(I):
    """Rank-size-like degree distribution: a few rows hold most of the nonzeros, so single
    rows span hundreds of work ranges and the seam pass does most of the reduction."""
    M, K, N, g = 4096, 1 << 18, 128, 4
    rng = np.random.default_rng(7)
    occ = np.minimum((K // 2) // np.arange(1, M + 1), K // 2).astype(np.int64)   # 131072, 65536, ...
    occ[64:] = rng.integers(0, 4, M - 64)
    row = np.repeat(np.arange(M, dtype=np.int32), occ)
    col = np.concatenate([rng.choice(K, size=int(k), replace=False) for k in occ]).astype(np.int32)
    val = rng.standard_normal(row.size).astype(np.float32)
    perm = rng.permutation(row.size)
    row, col, val = row[perm], col[perm], val[perm]
    _say(f"[spmm groupcoo hub] nnz={row.size}")
    fmt = oracle.coo_to_groupcoo(M, K, row, col, val, g)
    A = I.insum_coo_to_groupcoo(M, K, *coo_to_device(row, col, val, "f32"), g=g)
    assert_format_equal(A.g, A.AM, A.AK, A.AV, fmt)
    B = np.random.default_rng(1).standard_normal((K, N)).astype(np.float32)
    C64, absprod = _oracle_group_spmm(M, K, N, fmt, "f32", B)
    C = I.insum_spmm_groupcoo(A, values_to_torch(B, "f32"))
    assert_spmm_close(C.cpu().numpy(), C64, absprod, RTOL["f32"], "hub rows")


@pytest.mark.parametrize("M,N,dtype", [(1 << 17, 128, "f32"), (100_003, 72, "f16"), (70_000, 33, "f32")])
def test_spmm_groupcoo_long_runs_of_empty_rows(I, M, N, dtype):
    """Nonzeros only in the first and the last 1 % of the rows plus a few isolated rows: nearly all
    of C is zero-fill, most of it in aligned chunks that the second launch clears in parallel,
    the ragged ends of every gap by the wavefront that sees the jump."""
    K, g = 5000, 4
    rng = np.random.default_rng(M % 1000)
    lo = rng.integers(0, M // 100, 20_000)
    hi = M - 1 - rng.integers(0, M // 100, 20_000)
    lone = np.array([M // 3, M // 3 + 63, M // 3 + 64, M // 3 + 129, M // 2, M // 2 + 1000], dtype=np.int64)
    row = np.concatenate([lo, hi, lone]).astype(np.int32)
    col = rng.integers(0, K, row.size).astype(np.int32)
    val = synth.round_to_dtype(rng.standard_normal(row.size), dtype)
    _say(f"[spmm groupcoo gaps] M={M} N={N} {dtype} nnz={row.size}")
    fmt = oracle.coo_to_groupcoo(M, K, row, col, synth.storage_array(val, dtype), g)
    B = synth.round_to_dtype(np.random.default_rng(N).standard_normal((K, N)), dtype)
    C64, absprod = _oracle_group_spmm(M, K, N, fmt, dtype, B)
    A = _gpu_group_format(I, M, K, fmt, dtype)
    C = torch.full((M, N), 3.0, dtype=TORCH_DTYPE[dtype], device="cuda")       # every element must be overwritten
    I.insum_spmm_groupcoo(A, values_to_torch(B, dtype), C_out=C)
    assert_spmm_close(C.float().cpu().numpy(), C64, absprod, RTOL[dtype], "gaps", out_dtype=dtype)
    # accumulate: untouched rows keep their contents
    C2 = torch.full((M, N), 3.0, dtype=TORCH_DTYPE[dtype], device="cuda")
    I.insum_spmm_groupcoo(A, values_to_torch(B, dtype), C_out=C2, accumulate=True)
    empty = np.ones(M, bool)
    empty[row] = False
    assert torch.all(C2[torch.from_numpy(empty).cuda()] == 3.0)


def test_spmm_calls_can_be_captured_in_a_hip_graph(I):
    """Neither SpMM call allocates, synchronises or clears memory with a memset node, so a
    caller may capture it.  The graph is replayed several times with eager work in between and
    every replay must reproduce the eager result bit for bit."""
    M, K, N = 1024, 2048, 256
    row, col, val = synth.zipf_rows_coo(M, K, 1.2, 12.0, seed=3, dtype="f16", values="normal")
    A = I.insum_coo_to_groupcoo(M, K, *coo_to_device(row, col, val, "f16"), g=4)
    rb, cb, vb = synth.random_block_coo(M, K, 32, 32, seed=4, dtype="f16", block_density=0.2, sigma=0.5)
    Ab = I.insum_coo_to_blockgroupcoo(M, K, *coo_to_device(rb, cb, vb, "f16"), 32, 32, g=4)
    Bd = values_to_torch(synth.round_to_dtype(np.random.default_rng(0).standard_normal((K, N)), "f16"), "f16")
    ws = torch.empty(I.insum_spmm_groupcoo_workspace_bytes(M, N, A.G, A.g), dtype=torch.uint8, device="cuda")
    C1 = torch.empty((M, N), dtype=torch.float16, device="cuda")
    C2 = torch.empty((M, N), dtype=torch.float16, device="cuda")
    ref1 = I.insum_spmm_groupcoo(A, Bd, workspace=ws).clone()
    ref2 = I.insum_spmm_blockgroupcoo(Ab, Bd).clone()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            I.insum_spmm_groupcoo(A, Bd, C_out=C1, workspace=ws)
            I.insum_spmm_blockgroupcoo(Ab, Bd, C_out=C2)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        C1.fill_(float("nan"))
        C2.fill_(float("nan"))
        ws.random_(0, 255)                       # stale scratch contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C1, ref1), f"GroupCOO replay {rep} differs"
        assert torch.equal(C2, ref2), f"BlockGroupCOO replay {rep} differs"
        _ = I.insum_spmm_groupcoo(A, Bd, workspace=ws)   # eager work between replays
        torch.cuda.synchronize()


def test_planned_block_spmm_and_transposed_product_in_a_hip_graph(I):
    """The planned block SpMM with a split block row (partial tiles, arrival counters that the
    last chunk resets) and the transposed product (its clearing pass is a kernel, not a memset)
    under graph capture: every replay reproduces the eager result - bit for bit for the planned
    SpMM, to summation order for the atomics of the transposed product."""
    bM = bK = 32
    nbr, nbc, N = 5, 1500, 256
    row, col, val = _hub_block_coo(nbr, nbc, bM, bK, [2, 1300, 0, 30, 400], seed=9, dtype="bf16")
    M, K = nbr * bM, nbc * bK
    Ab = I.insum_coo_to_blockgroupcoo(M, K, *coo_to_device(row, col, val, "bf16"), bM, bK, g=4)
    Bd = values_to_torch(synth.round_to_dtype(np.random.default_rng(0).standard_normal((K, N)), "bf16"), "bf16")
    plan = I.insum_spmm_blockgroupcoo_plan(Ab, N)
    assert plan is not None
    ref = I.insum_spmm_blockgroupcoo(Ab, Bd, workspace=plan).clone()
    r2, c2, v2 = synth.zipf_rows_coo(2000, 1500, 1.2, 8.0, seed=4, dtype="f32", values="normal")
    A = I.insum_coo_to_groupcoo(2000, 1500, *coo_to_device(r2, c2, v2, "f32"), g=4)
    E = torch.randn((2000, 96), device="cuda")
    refT = I.insum_spmm_groupcoo_transposed(A, E).clone()
    C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    D = torch.empty((1500, 96), device="cuda")
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            I.insum_spmm_blockgroupcoo(Ab, Bd, C_out=C, workspace=plan)
            I.insum_spmm_groupcoo_transposed(A, E, D_out=D)
    torch.cuda.current_stream().wait_stream(side)
    scale = float(refT.abs().max())
    for rep in range(4):
        C.fill_(float("nan"))
        D.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, ref), f"planned block SpMM, replay {rep}"
        assert float((D - refT).abs().max()) <= 1e-5 * scale, f"transposed product, replay {rep}"
        _ = I.insum_spmm_blockgroupcoo(Ab, Bd, workspace=plan)   # eager use of the same plan between replays
        torch.cuda.synchronize()


def test_calls_on_two_streams_do_not_disturb_each_other(I):
    """The SpMM entry points keep no state outside their arguments: calls issued on two streams,
    each with its own workspace (and its own plan for the block kernel), may overlap on the GPU and
    still give the bits of the same calls made one after the other."""
    M, K, N = 3000, 2500, 256
    r1, c1, v1 = synth.zipf_rows_coo(M, K, 1.2, 10.0, seed=1, dtype="f32", values="normal")
    A1 = I.insum_coo_to_groupcoo(M, K, *coo_to_device(r1, c1, v1, "f32"), g=4)
    B1 = torch.randn((K, N), device="cuda")
    bM = bK = 32
    rb, cb, vb = _hub_block_coo(6, 900, bM, bK, [5, 700, 1, 30, 0, 250], seed=2, dtype="bf16")
    Mb, Kb = 6 * bM, 900 * bK
    A2 = I.insum_coo_to_blockgroupcoo(Mb, Kb, *coo_to_device(rb, cb, vb, "bf16"), bM, bK, g=4)
    B2 = torch.randn((Kb, N), device="cuda").bfloat16()
    ws = [torch.empty(I.insum_spmm_groupcoo_workspace_bytes(M, N, A1.G, A1.g), dtype=torch.uint8, device="cuda")
          for _ in range(2)]
    plans = [I.insum_spmm_blockgroupcoo_plan(A2, N) for _ in range(2)]
    ref1 = I.insum_spmm_groupcoo(A1, B1, workspace=ws[0]).clone()
    ref2 = I.insum_spmm_blockgroupcoo(A2, B2, workspace=plans[0]).clone()
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [[], []]
    for rep in range(6):
        for i, st in enumerate(streams):
            with torch.cuda.stream(st):
                outs[i].append((I.insum_spmm_groupcoo(A1, B1, workspace=ws[i]).clone(),
                                I.insum_spmm_blockgroupcoo(A2, B2, workspace=plans[i]).clone()))
    torch.cuda.synchronize()
    for i in range(2):
        for c1_, c2_ in outs[i]:
            assert torch.equal(c1_, ref1) and torch.equal(c2_, ref2)


TRANSPOSED_CASES = [
    # M, K, N, nnz, g, dtype, kind, out32
    (37, 53, 9, 300, 2, "f32", "uniform", False),        # scalar path
    (3000, 2000, 128, 50000, 4, "f32", "zipf", False),   # cfg3 shape
    (3000, 2000, 130, 50000, 4, "f32", "zipf", False),   # N not a multiple of 4
    (1000, 4096, 256, 100000, 16, "f16", "uniform", False),
    (1000, 4096, 256, 100000, 16, "bf16", "uniform", True),
    (300, 100000, 64, 90000, 32, "f16", "hub", False),   # one long row of A = one row of E used 30 000 times
    (4096, 64, 40, 30000, 7, "f32", "dups", False),      # few columns: every row of D receives ~500 atomics per element
    (1000, 1000, 1032, 20000, 1, "f16", "uniform", True),    # several column tiles
]


@pytest.mark.parametrize("M,K,N,nnz,g,dtype,kind,out32", TRANSPOSED_CASES)
def test_spmm_groupcoo_transposed_parity(I, M, K, N, nnz, g, dtype, kind, out32):
    """D = A^T E over the same stored format (the derivative of the SpMM with respect to its dense
    operand), against the oracle's fp64 Einsum with the dense operands exchanged."""
    _say(f"[spmm groupcoo transposed] M={M} K={K} N={N} nnz~{nnz} g={g} {dtype} {kind}")
    row, col, val = _group_case(M, K, nnz, kind, dtype, seed=N + g)
    fmt = oracle.coo_to_groupcoo(M, K, row, col, synth.storage_array(val, dtype), g)
    _, AM, AK, AV = fmt
    av = to_f32(AV, dtype)
    E = synth.round_to_dtype(np.random.default_rng(N).standard_normal((M, N)), dtype)
    D0 = synth.round_to_dtype(np.random.default_rng(N + 1).standard_normal((K, N)), "f32" if out32 else dtype)
    D64 = oracle.spmm_groupcoo_transposed(M, K, N, AM, AK, av, E)
    absprod = oracle.spmm_groupcoo_transposed(M, K, N, AM, AK, np.abs(av), np.abs(E))
    A = _gpu_group_format(I, M, K, fmt, dtype)
    Ed = values_to_torch(E, dtype)
    odt = torch.float32 if out32 else TORCH_DTYPE[dtype]
    D = torch.full((K, N), 5.0, dtype=odt, device="cuda")            # must be overwritten everywhere
    I.insum_spmm_groupcoo_transposed(A, Ed, D_out=D)
    assert_spmm_close(D.float().cpu().numpy(), D64, absprod, RTOL[dtype], "D=A^T E",
                      out_dtype=None if out32 else dtype)
    Dacc = values_to_torch(D0, "f32" if out32 else dtype)
    I.insum_spmm_groupcoo_transposed(A, Ed, D_out=Dacc, accumulate=True)
    assert_spmm_close(Dacc.float().cpu().numpy(), D64 + D0.astype(np.float64), absprod + np.abs(D0), RTOL[dtype],
                      "D+=A^T E", out_dtype=None if out32 else dtype)


def test_spmm_groupcoo_transposed_is_the_gradient_of_the_forward_product(I):
    """<A B, E> = <B, A^T E> with both sides from the library (fp32), and strided operands."""
    M, K, N, g = 900, 1300, 96, 4
    row, col, val = synth.zipf_rows_coo(M, K, 1.2, 10.0, seed=11, dtype="f32", values="normal")
    A = I.insum_coo_to_groupcoo(M, K, *coo_to_device(row, col, val, "f32"), g=g)
    rng = np.random.default_rng(5)
    Bw = torch.from_numpy(rng.standard_normal((K, N + 32)).astype(np.float32)).cuda()
    Ew = torch.from_numpy(rng.standard_normal((M, N + 8)).astype(np.float32)).cuda()
    B, E = Bw[:, :N], Ew[:, :N]
    C = I.insum_spmm_groupcoo(A, B)
    Dw = torch.full((K, N + 4), 7.0, device="cuda")
    I.insum_spmm_groupcoo_transposed(A, E, D_out=Dw[:, :N])
    lhs = float((C.double() * E.double()).sum())
    rhs = float((B.double() * Dw[:, :N].double()).sum())
    assert abs(lhs - rhs) <= 1e-5 * float((C.double().abs() * E.double().abs()).sum())
    assert torch.all(Dw[:, N:] == 7.0)
    # empty format: D = 0, or D unchanged when accumulating
    A0 = I.GroupCOO(M, K, 4, torch.zeros(0, dtype=torch.int32, device="cuda"),
                    torch.zeros((0, 4), dtype=torch.int32, device="cuda"), torch.zeros((0, 4), device="cuda"))
    assert torch.all(I.insum_spmm_groupcoo_transposed(A0, E.contiguous()) == 0)


def test_choose_group_size_times_the_neighbours(I):
    """Section 4.2: the candidates are timed on the caller's operands; the chosen g is one of
    them, and converting with it gives the oracle's format and product."""
    M, K, N = 4096, 4096, 256
    row, col, val = synth.random_coo(M, K, 400_000, seed=2, dtype="f16", sigma=0.02)    # g* ~ 9.9
    rd, cd, vd = coo_to_device(row, col, val, "f16")
    B = synth.round_to_dtype(np.random.default_rng(3).standard_normal((K, N)), "f16")
    Bd = values_to_torch(B, "f16")
    best, times = I.insum_choose_group_size(M, K, rd, cd, vd, Bd, repeats=5)
    cand = I.insum_group_size_candidates(row.size, M)
    _say(f"[choose g] candidates {cand} ms {times} -> {best}")
    assert cand == [4, 8, 16] and sorted(times) == cand and best in cand
    assert all(t > 0 for t in times.values()) and times[best] == min(times.values())
    fmt = oracle.coo_to_groupcoo(M, K, row, col, synth.storage_array(val, "f16"), best)
    A = I.insum_coo_to_groupcoo(M, K, rd, cd, vd, g=best)
    assert_format_equal(A.g, A.AM, A.AK, A.AV, fmt)
    C64, absprod = _oracle_group_spmm(M, K, N, fmt, "f16", B)
    assert_spmm_close(I.insum_spmm_groupcoo(A, Bd).float().cpu().numpy(), C64, absprod, RTOL["f16"], "chosen g",
                      out_dtype="f16")
