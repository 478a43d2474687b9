"""GPU parity of the sparse-convolution path (Section 6.4) against the CPU oracle: the grouping
of the kernel map is compared bit for bit, the convolution element by element.

Tolerance: inputs are exact in their storage type, products of two 16-bit values are exact in
fp32, and every sum (over channels on the matrix cores, over contributions through fp32
atomics, in any order) is an fp32 sum of at most C + (entries per output) terms, so the error
is bounded by that count times 2^-24 times sum |v| |In| |W|: 1e-5 of the absolute-value
product covers C = 128 with 27 offsets, with the fp64 oracle as the exact side.
"""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import paper_2510_17505_amd as I
import synth
from gpu_util import TORCH_DTYPE, bits, storage_to_torch, torch_to_storage, values_to_torch
from helpers import assert_spmm_close

pytestmark = pytest.mark.gpu
RTOL = 1e-5


def _i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def _features(rows, cols, seed, dtype, lead=None):
    rng = np.random.default_rng(seed)
    x = synth.round_to_dtype(rng.normal(0.0, 1.0, size=(rows, cols) if lead is None else (lead, rows, cols))
                             .astype(np.float32), dtype)
    return x


def _convert_both(X, Y, Z, mx, my, mz, mv, dtype, g):
    st = synth.storage_array(mv, dtype)
    want = oracle.map_to_groupcoo(X, Y, Z, mx, my, mz, st, g)
    got = I.insum_map_to_groupcoo(X, Y, Z, _i32(mx), _i32(my), _i32(mz), storage_to_torch(st, dtype), g or 0)
    return got, want


def _assert_map_equal(got, want):
    g, MZ, MX, MY, MV = want
    assert got.g == g and got.G == MZ.shape[0]
    assert tuple(got.MAPX.shape) == MX.shape and tuple(got.MAPV.shape) == MV.shape
    assert np.array_equal(got.MAPZ.cpu().numpy(), MZ), "MAPZ differs"
    assert np.array_equal(got.MAPX.cpu().numpy(), MX), "MAPX differs"
    assert np.array_equal(got.MAPY.cpu().numpy(), MY), "MAPY differs"
    assert np.array_equal(bits(torch_to_storage(got.MAPV)), bits(MV)), "MAPV differs"


def _random_map(seed, X, Y, Z, nnz):
    rng = np.random.default_rng(seed)
    return (rng.integers(0, X, nnz).astype(np.int32), rng.integers(0, Y, nnz).astype(np.int32),
            rng.integers(0, Z, nnz).astype(np.int32), rng.normal(size=nnz).astype(np.float32))


# ------------------------------------------------------------------------------------------- #
# grouping of the kernel map: bit-exact
# ------------------------------------------------------------------------------------------- #
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("g", [None, 1, 3, 32, 100])
def test_map_grouping_voxel(dtype, g):
    P, mx, my, mz, mv = synth.voxel_kernel_map(12, 0.35, seed=3, dtype=dtype, values="normal")
    got, want = _convert_both(P, P, 27, mx, my, mz, mv, dtype, g)
    _assert_map_equal(got, want)
    if g is None:
        assert got.g == oracle.default_group_size(mx.size, 27)
    g_cnt, G_cnt = I.insum_map_count_groups(P, P, 27, _i32(mx), _i32(my), _i32(mz), g or 0)
    assert (g_cnt, G_cnt) == (got.g, got.G)


@pytest.mark.parametrize("X,Y,Z,nnz,g", [(1, 1, 1, 5, 2), (50, 70, 5000, 3000, 4), (3000, 11, 2, 40000, 64),
                                         (17, 19, 9, 1, 8)])
def test_map_grouping_random_shapes(X, Y, Z, nnz, g):
    """Repeated triples, empty offsets, more offsets than the LDS histogram holds, one entry."""
    mx, my, mz, mv = _random_map(nnz, X, Y, Z, nnz)
    mv = synth.round_to_dtype(mv, "f16")
    got, want = _convert_both(X, Y, Z, mx, my, mz, mv, "f16", g)
    _assert_map_equal(got, want)
    assert I.insum_map_count_groups(X, Y, Z, _i32(mx), _i32(my), _i32(mz), g) == (g, got.G)


def test_map_grouping_errors_and_empty():
    X, Y, Z = 10, 12, 4
    mx, my, mz, mv = _random_map(0, X, Y, Z, 50)
    mv = synth.round_to_dtype(mv, "f16")
    for arr, bound in ((mx, X), (my, Y), (mz, Z)):
        for badval in (bound, -1):
            a = arr.copy()
            a[7] = badval
            args = [_i32(a if arr is t else t) for t in (mx, my, mz)]
            with pytest.raises(I.InsumError) as e:
                I.insum_map_to_groupcoo(X, Y, Z, *args, values_to_torch(mv, "f16"), 4)
            assert e.value.status == 2
    empty = I.insum_map_to_groupcoo(X, Y, Z, _i32(mx[:0]), _i32(my[:0]), _i32(mz[:0]),
                                    values_to_torch(mv[:0], "f16"), 4)
    assert empty.G == 0 and empty.g == 4
    Out = I.insum_spconv_groupcoo(empty, values_to_torch(_features(Y, 8, 0, "f16"), "f16"),
                                  values_to_torch(_features(8, 16, 1, "f16", lead=Z), "f16"))
    assert Out.shape == (X, 16) and torch.all(Out == 0)


# ------------------------------------------------------------------------------------------- #
# the convolution
# ------------------------------------------------------------------------------------------- #
def _run_conv(X, Y, Z, mx, my, mz, mv, C, M, dtype, g, seed=0, ld_in=None, accumulate=False):
    In = _features(Y, C, seed + 1, dtype)
    W = _features(C, M, seed + 2, dtype, lead=Z)
    got_map, want_map = _convert_both(X, Y, Z, mx, my, mz, mv, dtype, g)
    _, MZ, MX, MY, MV = want_map
    MV32 = oracle.bf16_bits_to_f32(MV) if dtype == "bf16" else MV.astype(np.float32)
    init = None
    Out = None
    if accumulate:
        init = np.random.default_rng(seed + 3).normal(size=(X, M)).astype(np.float32)
        Out = torch.from_numpy(init.copy()).cuda()
    want = oracle.spconv_groupcoo(X, C, M, MZ, MX, MY, MV32, In, W, Out_init=init)
    absprod = oracle.spconv_groupcoo(X, C, M, MZ, MX, MY, np.abs(MV32), np.abs(In), np.abs(W),
                                     Out_init=None if init is None else np.abs(init))
    In_d = values_to_torch(In, dtype)
    if ld_in is not None:
        buf = torch.full((Y, ld_in), float("nan"), dtype=TORCH_DTYPE[dtype], device="cuda")
        buf[:, :C] = In_d
        In_d = buf[:, :C]
    got = I.insum_spconv_groupcoo(got_map, In_d, values_to_torch(W, dtype), Out, accumulate)
    torch.cuda.synchronize()
    assert got.dtype == torch.float32
    assert_spmm_close(got.cpu().numpy(), want, absprod, RTOL, f"spconv {dtype} C={C} M={M} g={got_map.g}")
    return got_map


@pytest.mark.parametrize("values", ["ones", "normal"])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("C,M", [(128, 128), (64, 64), (32, 96), (256, 256), (16, 32), (8, 8), (72, 100),
                                 (256, 40), (128, 160)])
def test_spconv_voxel_mfma(dtype, C, M, values):
    """Matrix-core path: every instantiation (C up to 32 / 64 / 128 / 256), channel counts that
    end inside a k-step, output widths that end inside a column block or need several m-tiles;
    map values all one (a plain convolution, its own kernel variant) and general."""
    P, mx, my, mz, mv = synth.voxel_kernel_map(14, 0.3, seed=C + M, dtype=dtype, values=values)
    _run_conv(P, P, 27, mx, my, mz, mv, C, M, dtype, None, seed=C)


def test_spconv_one_value_differs_from_one():
    """A single map value other than 1 switches the whole call to the general variant."""
    P, mx, my, mz, mv = synth.voxel_kernel_map(14, 0.3, seed=5, dtype="f16")
    mv = mv.copy()
    mv[mv.size // 2] = -2.5
    _run_conv(P, P, 27, mx, my, mz, mv, 64, 64, "f16", None, seed=7)


@pytest.mark.parametrize("g", [1, 2, 5, 16, 32, 48, 256])
def test_spconv_group_sizes(g):
    """Tiles of 32 slots that span several groups and several offsets (g below 32 or not a
    divisor of 32), padding inside tiles, groups longer than a tile."""
    P, mx, my, mz, mv = synth.voxel_kernel_map(10, 0.4, seed=g, dtype="f16", values="normal")
    _run_conv(P, P, 27, mx, my, mz, mv, 64, 64, "f16", g, seed=g)


def test_spconv_many_offsets_few_entries():
    """More offsets than slots per tile: most tiles hold several offsets, each a reload of the
    weight fragments."""
    X, Y, Z = 300, 200, 500
    mx, my, mz, mv = _random_map(5, X, Y, Z, 4000)
    _run_conv(X, Y, Z, mx, my, mz, synth.round_to_dtype(mv, "bf16"), 32, 64, "bf16", 4, seed=1)


def test_spconv_repeated_output_rows_and_binary_values():
    """All entries of an offset scatter into a handful of output rows (atomics on the same
    address from one wavefront), values all one as in a plain convolution."""
    X, Y, Z = 4, 1000, 3
    rng = np.random.default_rng(0)
    nnz = 5000
    mx = rng.integers(0, X, nnz).astype(np.int32)
    my = rng.integers(0, Y, nnz).astype(np.int32)
    mz = rng.integers(0, Z, nnz).astype(np.int32)
    _run_conv(X, Y, Z, mx, my, mz, np.ones(nnz, np.float32), 64, 128, "f16", 32, seed=2)


@pytest.mark.parametrize("dtype,C,M,g", [("f32", 24, 40, 8), ("f32", 128, 128, None), ("f16", 12, 20, 4),
                                         ("bf16", 264, 16, 16), ("f16", 36, 300, 3)])
def test_spconv_general_kernel(dtype, C, M, g):
    """fp32 inputs, channel counts that are not a multiple of 8 or exceed 256."""
    P, mx, my, mz, mv = synth.voxel_kernel_map(9, 0.4, seed=C, dtype=dtype, values="normal")
    _run_conv(P, P, 27, mx, my, mz, mv, C, M, dtype, g, seed=M)


def test_spconv_strided_input_and_accumulate():
    P, mx, my, mz, mv = synth.voxel_kernel_map(11, 0.35, seed=8, dtype="f16", values="normal")
    _run_conv(P, P, 27, mx, my, mz, mv, 64, 96, "f16", None, seed=4, ld_in=80, accumulate=True)
    _run_conv(P, P, 27, mx, my, mz, mv, 64, 96, "f16", None, seed=5, ld_in=68)   # ld_in % 8 != 0: general


def test_spconv_identity_map_is_a_gemm_on_the_device():
    """Independent of the oracle: one offset, identity map, unit values -> In @ W[0]."""
    P, C, M = 1000, 128, 128
    ar = torch.arange(P, dtype=torch.int32, device="cuda")
    Map = I.insum_map_to_groupcoo(P, P, 1, ar, ar, torch.zeros_like(ar),
                                  torch.ones(P, dtype=torch.float16, device="cuda"), 32)
    In = values_to_torch(_features(P, C, 0, "f16"), "f16")
    W = values_to_torch(_features(C, M, 1, "f16", lead=1), "f16")
    got = I.insum_spconv_groupcoo(Map, In, W)
    want = In.double() @ W[0].double()
    assert torch.allclose(got.double(), want, rtol=0, atol=1e-5 * float(want.abs().max()) * 4)


def test_spconv_argument_errors():
    P, mx, my, mz, mv = synth.voxel_kernel_map(6, 0.4, seed=1, dtype="f16")
    Map = I.insum_map_to_groupcoo(P, P, 27, _i32(mx), _i32(my), _i32(mz), values_to_torch(mv, "f16"), 8)
    In = values_to_torch(_features(P, 16, 0, "f16"), "f16")
    W = values_to_torch(_features(16, 16, 0, "f16", lead=27), "f16")
    from paper_2510_17505_amd import api
    Out = torch.empty((P, 16), dtype=torch.float32, device="cuda")
    need = I.insum_spconv_groupcoo_workspace_bytes(Map, 16, 16, torch.float16)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")

    def call(**kw):
        a = dict(X=P, Y=P, Z=27, C=16, M=16, G=Map.G, g=Map.g, MAPZ=Map.MAPZ.data_ptr(), MAPX=Map.MAPX.data_ptr(),
                 MAPY=Map.MAPY.data_ptr(), MAPV=Map.MAPV.data_ptr(), In=In.data_ptr(), ld_in=16,
                 W=W.data_ptr(), dt=1, Out=Out.data_ptr(), ld_out=16, acc=0, reuse=0, ws=ws.data_ptr(),
                 ws_bytes=ws.numel(),
                 stream=0)
        a.update(kw)
        return api._conv(*a.values())

    assert call() == 0
    assert call(g=0) == 1 and call(ld_in=8) == 1 and call(ld_out=8) == 1 and call(dt=7) == 1
    assert call(MAPZ=0) == 1 and call(In=0) == 1 and call(Out=0) == 1 and call(C=-1) == 1
    assert call(ws_bytes=need - 1) == 4 and call(ws=0) == 4          # workspace too small / missing
    torch.cuda.synchronize()


def test_spconv_full_size_properties_and_samples():
    """The benchmark workload (96^3 grid, 30 % occupancy, 128 -> 128 channels, fp16): sampled
    output rows against the oracle evaluated on just the entries that reach them, and the
    column sums of Out against sum_z (column sums of gathered In) @ W[z] in fp64."""
    P, mx, my, mz, mv = synth.voxel_kernel_map(96, 0.3, seed=0, dtype="f16")
    C = M = 128
    In = _features(P, C, 1, "f16")
    W = _features(C, M, 2, "f16", lead=27) * np.float32(0.125)
    W = synth.round_to_dtype(W, "f16")
    Map = I.insum_map_to_groupcoo(P, P, 27, _i32(mx), _i32(my), _i32(mz), values_to_torch(mv, "f16"))
    assert Map.g == oracle.default_group_size(mx.size, 27)
    got = I.insum_spconv_groupcoo(Map, values_to_torch(In, "f16"), values_to_torch(W, "f16")).cpu().numpy()
    rng = np.random.default_rng(0)
    rows = np.unique(rng.integers(0, P, 200))
    sel = np.isin(mx, rows)
    remap = -np.ones(P, dtype=np.int64)
    remap[rows] = np.arange(rows.size)
    _, MZ, MX, MY, MV = oracle.map_to_groupcoo(rows.size, P, 27, remap[mx[sel]], my[sel], mz[sel], mv[sel], 8)
    want = oracle.spconv_groupcoo(rows.size, C, M, MZ, MX, MY, MV, In, W)
    absprod = oracle.spconv_groupcoo(rows.size, C, M, MZ, MX, MY, np.abs(MV), np.abs(In), np.abs(W))
    assert_spmm_close(got[rows], want, absprod, RTOL, "sampled rows")
    In64, W64 = In.astype(np.float64), W.astype(np.float64)
    colsum = np.zeros(M)
    abssum = np.zeros(M)
    for z in range(27):
        s = mz == z
        colsum += In64[my[s]].sum(axis=0) @ W64[z]
        abssum += np.abs(In64[my[s]]).sum(axis=0) @ np.abs(W64[z])
    err = np.abs(got.astype(np.float64).sum(axis=0) - colsum)
    assert np.all(err <= 1e-5 * abssum), float((err / abssum).max())


def test_spconv_full_size_every_element():
    """The benchmark workload again, every element of Out against the oracle run over the whole
    map (about 75 GFLOP of fp64 loops on the host cores: the slow one of the two full-size tests)."""
    P, mx, my, mz, mv = synth.voxel_kernel_map(96, 0.3, seed=0, dtype="f16")
    C = M = 128
    In = _features(P, C, 1, "f16")
    W = synth.round_to_dtype(_features(C, M, 2, "f16", lead=27) * np.float32(0.125), "f16")
    st = synth.storage_array(mv, "f16")
    g, MZ, MX, MY, MV = oracle.map_to_groupcoo(P, P, 27, mx, my, mz, st, None)
    Map = I.insum_map_to_groupcoo(P, P, 27, _i32(mx), _i32(my), _i32(mz), values_to_torch(mv, "f16"))
    assert Map.g == g and np.array_equal(Map.MAPZ.cpu().numpy(), MZ)
    assert np.array_equal(Map.MAPX.cpu().numpy(), MX) and np.array_equal(Map.MAPY.cpu().numpy(), MY)
    print(f"[spconv full] P={P} entries={mx.size} g={g}: oracle over the whole map ...", flush=True)
    mvf = MV.astype(np.float32)
    want = oracle.spconv_groupcoo(P, C, M, MZ, MX, MY, mvf, In, W)
    absprod = oracle.spconv_groupcoo(P, C, M, MZ, MX, MY, np.abs(mvf), np.abs(In), np.abs(W))
    print("[spconv full] library ...", flush=True)
    Ind, Wd = values_to_torch(In, "f16"), values_to_torch(W, "f16")
    ws = torch.empty(max(1, I.insum_spconv_groupcoo_workspace_bytes(Map, C, M, Ind.dtype)), dtype=torch.uint8,
                     device="cuda")
    got = I.insum_spconv_groupcoo(Map, Ind, Wd, workspace=ws)
    assert_spmm_close(got.cpu().numpy(), want, absprod, RTOL, "whole output")
    again = I.insum_spconv_groupcoo(Map, Ind, Wd, workspace=ws, reuse_map_tables=True)
    assert_spmm_close(again.cpu().numpy(), want, absprod, RTOL, "whole output, tables reused")


@pytest.mark.parametrize("order,values", [("morton", "ones"), ("lex", "normal")])
def test_spconv_surface_cloud(order, values):
    """A point cloud on surfaces (planes and sphere shells), where whole 32-point tiles miss
    most stencil offsets - the passes the output-stationary kernel skips - every element."""
    P, mx, my, mz, mv = synth.surface_kernel_map(48, 4, 1, seed=2, dtype="f16", values=values, order=order)
    C, M = 64, 96
    print(f"[spconv surfaces] {order} {values}: P={P} entries={mx.size}", flush=True)
    In = _features(P, C, 1, "f16")
    W = synth.round_to_dtype(_features(C, M, 2, "f16", lead=27) * np.float32(0.125), "f16")
    g, MZ, MX, MY, MV = oracle.map_to_groupcoo(P, P, 27, mx, my, mz, synth.storage_array(mv, "f16"), None)
    Map = I.insum_map_to_groupcoo(P, P, 27, _i32(mx), _i32(my), _i32(mz), values_to_torch(mv, "f16"))
    assert Map.g == g and np.array_equal(Map.MAPX.cpu().numpy(), MX) and np.array_equal(Map.MAPY.cpu().numpy(), MY)
    mvf = MV.astype(np.float32)
    want = oracle.spconv_groupcoo(P, C, M, MZ, MX, MY, mvf, In, W)
    absprod = oracle.spconv_groupcoo(P, C, M, MZ, MX, MY, np.abs(mvf), np.abs(In), np.abs(W))
    Ind, Wd = values_to_torch(In, "f16"), values_to_torch(W, "f16")
    ws = torch.empty(max(1, I.insum_spconv_groupcoo_workspace_bytes(Map, C, M, Ind.dtype)), dtype=torch.uint8,
                     device="cuda")
    got = I.insum_spconv_groupcoo(Map, Ind, Wd, workspace=ws)
    assert_spmm_close(got.cpu().numpy(), want, absprod, RTOL, "surface cloud")


@pytest.mark.parametrize("values", ["ones", "normal"])
def test_spconv_reuses_the_map_tables_across_layers(values):
    """Three layers over one kernel map: the later calls skip the table build and must still
    match the oracle, with other features, weights and channel counts."""
    P, mx, my, mz, mv = synth.voxel_kernel_map(13, 0.3, seed=11, dtype="f16", values=values)
    st = synth.storage_array(mv, "f16")
    _, MZ, MX, MY, MV = oracle.map_to_groupcoo(P, P, 27, mx, my, mz, st, None)
    Map = I.insum_map_to_groupcoo(P, P, 27, _i32(mx), _i32(my), _i32(mz), storage_to_torch(st, "f16"))
    shapes = ((64, 96), (64, 96), (128, 32), (32, 256))
    ws = torch.empty(max(I.insum_spconv_groupcoo_workspace_bytes(Map, C, M, torch.float16) for C, M in shapes),
                     dtype=torch.uint8, device="cuda")
    for layer, (C, M) in enumerate(shapes):
        reuse = layer > 0
        In = _features(P, C, 20 + layer, "f16")
        W = _features(C, M, 30 + layer, "f16", lead=27)
        got = I.insum_spconv_groupcoo(Map, values_to_torch(In, "f16"), values_to_torch(W, "f16"),
                                      workspace=ws, reuse_map_tables=reuse)
        want = oracle.spconv_groupcoo(P, C, M, MZ, MX, MY, MV.astype(np.float32), In, W)
        absprod = oracle.spconv_groupcoo(P, C, M, MZ, MX, MY, np.abs(MV.astype(np.float32)), np.abs(In), np.abs(W))
        assert_spmm_close(got.cpu().numpy(), want, absprod, RTOL, f"layer {layer}")


def test_spconv_call_can_be_captured_in_a_hip_graph():
    """The convolution neither allocates nor synchronises nor clears memory with a memset node.
    On a map without repeated (x, z) pairs the output-stationary schedule uses no atomics, so
    every replay (with stale workspace contents and eager work in between) must reproduce the
    eager result bit for bit."""
    P, mx, my, mz, mv = synth.voxel_kernel_map(16, 0.3, seed=21, dtype="f16")
    Map = I.insum_map_to_groupcoo(P, P, 27, _i32(mx), _i32(my), _i32(mz), values_to_torch(mv, "f16"))
    In = values_to_torch(_features(P, 64, 1, "f16"), "f16")
    W = values_to_torch(_features(64, 128, 2, "f16", lead=27), "f16")
    need = I.insum_spconv_groupcoo_workspace_bytes(Map, 64, 128, torch.float16)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    ref = I.insum_spconv_groupcoo(Map, In, W, workspace=ws).clone()
    Out = torch.empty_like(ref)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            I.insum_spconv_groupcoo(Map, In, W, Out=Out, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        Out.fill_(float("nan"))
        ws.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Out, ref), f"replay {rep} differs"
        _ = I.insum_spconv_groupcoo(Map, In, W, workspace=ws)
        torch.cuda.synchronize()
