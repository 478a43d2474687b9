"""insum_spmm_groupcoo_noalloc (the entry point for callers that cannot allocate) against
insum_spmm_groupcoo, through the C ABI, on calls in a row that share the library's device
array: a large input first, then smaller ones that find the earlier call's partial sums
still in the array."""
from __future__ import annotations

import ctypes

import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import RTOL, coo_to_device, values_to_torch
from helpers import assert_spmm_close

pytestmark = pytest.mark.gpu

_DT = {"f32": 0, "f16": 1, "bf16": 2}


def _abi():
    import paper_2510_17505_amd as I
    lib = ctypes.CDLL(I.library_path())
    i64, i32, p, ci = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int
    common = [i64, i64, i64, i64, i32, p, p, p, ci, p, i64, ci, p, i64, ci, ci]
    lib.insum_spmm_groupcoo.restype = ci
    lib.insum_spmm_groupcoo.argtypes = common + [p, ctypes.c_size_t, p]
    lib.insum_spmm_groupcoo_noalloc.restype = ci
    lib.insum_spmm_groupcoo_noalloc.argtypes = common + [p]
    lib.insum_spmm_groupcoo_workspace_bytes.restype = ctypes.c_size_t
    lib.insum_spmm_groupcoo_workspace_bytes.argtypes = [i64, i64, i64, i32]
    return I, lib


def _hub_coo(M, K, mean, hubs, seed, dtype):
    """Zipf rows plus a few rows long enough to span many work ranges (they exercise the
    partial sums that live in the device array)."""
    row, col, val = synth.zipf_rows_coo(M, K, 1.2, mean, seed, dtype, "normal")
    rng = np.random.default_rng(seed + 100)
    extra_r, extra_c = [], []
    for h, length in hubs:
        extra_r.append(np.full(length, h, np.int32))
        extra_c.append(rng.choice(K, size=length, replace=False).astype(np.int32))
    row = np.concatenate([row] + extra_r)
    col = np.concatenate([col] + extra_c)
    val = np.concatenate([val, synth.round_to_dtype(rng.standard_normal(row.size - val.size), dtype)])
    perm = rng.permutation(row.size)
    return row[perm], col[perm], val[perm]


def _run_pair(I, lib, M, K, N, g, dtype, row, col, val, seed, accumulate, expect_equal):
    A = I.insum_coo_to_groupcoo(M, K, *coo_to_device(row, col, val, dtype), g=g)
    Bh = synth.round_to_dtype(np.random.default_rng(seed).standard_normal((K, N)), dtype)
    B = values_to_torch(Bh, dtype)
    C0h = synth.round_to_dtype(np.random.default_rng(seed + 1).standard_normal((M, N)), dtype)
    C_ref = values_to_torch(C0h, dtype)
    C_new = C_ref.clone()
    ws = torch.empty(lib.insum_spmm_groupcoo_workspace_bytes(M, N, A.G, A.g), dtype=torch.uint8, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    args = (M, K, N, A.G, A.g, A.AM.data_ptr(), A.AK.data_ptr(), A.AV.data_ptr(), _DT[dtype],
            B.data_ptr(), B.stride(0), _DT[dtype], None, N, _DT[dtype], int(accumulate))

    def with_c(c):
        return args[:12] + (c.data_ptr(),) + args[13:]

    assert lib.insum_spmm_groupcoo(*with_c(C_ref), ws.data_ptr(), ws.numel(), s) == 0
    assert lib.insum_spmm_groupcoo_noalloc(*with_c(C_new), s) == 0
    torch.cuda.synchronize()
    got, ref = C_new.float().cpu().numpy(), C_ref.float().cpu().numpy()
    if expect_equal:
        assert np.array_equal(got, ref), "same plan, same kernels: results must be identical"
    # and to the parity bar against the fp64 definition
    fmt_AM, fmt_AK = A.AM.cpu().numpy(), A.AK.cpu().numpy()
    AV = A.AV.float().cpu().numpy()
    C64 = oracle.spmm_groupcoo(M, K, N, fmt_AM, fmt_AK, AV, Bh, C_init=C0h if accumulate else None)
    absprod = oracle.spmm_groupcoo(M, K, N, fmt_AM, fmt_AK, np.abs(AV), np.abs(Bh),
                                   C_init=np.abs(C0h) if accumulate else None)
    assert_spmm_close(got, C64, absprod, RTOL[dtype], f"noalloc {dtype} M={M} N={N}",
                      out_dtype=dtype)
    scale = float(np.abs(C64).max())
    assert float(np.abs(got - ref).max()) <= RTOL[dtype] * scale


def test_noalloc_matches_the_workspace_entry_point_on_calls_in_a_row():
    I, lib = _abi()
    # 1. large fp16 input: the usual number of work ranges would need 64 MiB of partial sums,
    #    so this call runs with fewer ranges (32 MiB array) - compared within tolerance.
    M, K, N = 200_000, 40_000, 256
    row, col, val = _hub_coo(M, K, 11.0, [(17, 30_000), (150_000, 9_000)], 3, "f16")
    print(f"[noalloc] call 1: f16 M={M} K={K} N={N} nnz={row.size}", flush=True)
    _run_pair(I, lib, M, K, N, 4, "f16", row, col, val, 5, False, expect_equal=False)
    # 2. smaller fp32 input right after it: same plan in both entry points -> identical bits
    M, K, N = 20_000, 30_000, 128
    row, col, val = _hub_coo(M, K, 8.0, [(0, 20_000), (19_999, 5_000)], 4, "f32")
    print(f"[noalloc] call 2: f32 M={M} K={K} N={N} nnz={row.size}", flush=True)
    _run_pair(I, lib, M, K, N, 4, "f32", row, col, val, 6, False, expect_equal=True)
    # 3. smaller again, accumulating into C, ragged N (scalar path), g not a power of two
    M, K, N = 700, 900, 50
    row, col, val = _hub_coo(M, K, 6.0, [(3, 800)], 5, "f32")
    print(f"[noalloc] call 3: f32 M={M} K={K} N={N} nnz={row.size} accumulate", flush=True)
    _run_pair(I, lib, M, K, N, 3, "f32", row, col, val, 7, True, expect_equal=True)


def test_noalloc_rejects_what_it_cannot_serve():
    _, lib = _abi()
    call = lib.insum_spmm_groupcoo_noalloc
    # a row of partial sums wider than the array: N > 4 194 304 (no device work is started)
    assert call(1, 1, 5_000_000, 1, 1, 8, 8, 8, 0, 8, 5_000_000, 0, 8, 5_000_000, 0, 0, None) == 4
    assert call(4, 4, 4, 1, 0, 0, 0, 0, 0, 0, 4, 0, 0, 4, 0, 0, None) == 1      # g <= 0
    assert call(4, 4, 4, 1, 2, 8, 8, 8, 0, 8, 4, 1, 8, 4, 0, 0, None) == 5      # mixed dtypes
