"""ctypes binding of libinsum.so (see include/insum.h for the contract of every call)."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field

import torch

from . import _build

_i64, _i32, _p = C.c_int64, C.c_int32, C.c_void_p

OK, ERR_INVALID_ARG, ERR_OUT_OF_RANGE, ERR_DUPLICATE, ERR_CAPACITY, ERR_UNSUPPORTED, ERR_HIP = range(7)
_DTYPE = {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}


def _load() -> C.CDLL:
    if not os.path.exists(_build.LIB):
        _build.build()          # raises if hipcc is missing or compilation fails
    return C.CDLL(_build.LIB)


_lib = _load()


def library_path() -> str:
    return _build.LIB


def _sig(name, restype, argtypes):
    fn = getattr(_lib, name)
    fn.restype = restype
    fn.argtypes = argtypes
    return fn


_version = _sig("insum_version", C.c_int, [])
_status_string = _sig("insum_status_string", C.c_char_p, [C.c_int])
_default_g = _sig("insum_default_group_size", _i32, [_i64, _i64])
_cost = _sig("insum_indirect_access_cost", _i64, [_i64, _p, _i32])
_cand = _sig("insum_group_size_candidates", _i32, [_i64, _i64, _p])
_choose_ws = _sig("insum_choose_group_size_workspace_bytes", C.c_size_t, [_i64, _i64, _i64, C.c_int])
_choose = _sig("insum_choose_group_size", C.c_int,
               [_i64, _i64, _i64, _i64, _p, _p, _p, C.c_int, _p, _i64, _p, _i64, C.c_int, _i32,
                _p, _p, _p, _p, _p, C.c_size_t, _p])
_g_ws = _sig("insum_coo_to_groupcoo_workspace_bytes", C.c_size_t, [_i64, _i64])
_g_conv = _sig("insum_coo_to_groupcoo", C.c_int,
               [_i64, _i64, _i64, _p, _p, _p, C.c_int, _i32, _p, _p, _p, _p, _p, _i64,
                _p, C.c_size_t, _p])
_gt_ws = _sig("insum_groupcoo_transpose_workspace_bytes", C.c_size_t, [_i64, _i64, _i64, _i32])
_gt = _sig("insum_groupcoo_transpose", C.c_int,
           [_i64, _i64, _i64, _i32, _p, _p, _p, C.c_int, _i32, _p, _p, _p, _p, _p, _p, _i64,
            _p, C.c_size_t, _p])
_b_ws = _sig("insum_coo_to_blockgroupcoo_workspace_bytes", C.c_size_t, [_i64, _i64, _i64, _i32, _i32])
_b_conv = _sig("insum_coo_to_blockgroupcoo", C.c_int,
               [_i64, _i64, _i64, _p, _p, _p, C.c_int, _i32, _i32, _i32, _p, _p, _p, _p, _p, _i64,
                _p, C.c_size_t, _p])
_sg_ws = _sig("insum_spmm_groupcoo_workspace_bytes", C.c_size_t, [_i64, _i64, _i64, _i32])
_sg = _sig("insum_spmm_groupcoo", C.c_int,
           [_i64, _i64, _i64, _i64, _i32, _p, _p, _p, C.c_int, _p, _i64, C.c_int,
            _p, _i64, C.c_int, C.c_int, _p, C.c_size_t, _p])
_sg_na = _sig("insum_spmm_groupcoo_noalloc", C.c_int,
              [_i64, _i64, _i64, _i64, _i32, _p, _p, _p, C.c_int, _p, _i64, C.c_int,
               _p, _i64, C.c_int, C.c_int, _p])
_sgt_ws = _sig("insum_spmm_groupcoo_transposed_workspace_bytes", C.c_size_t, [_i64, _i64, C.c_int])
_sgt = _sig("insum_spmm_groupcoo_transposed", C.c_int,
            [_i64, _i64, _i64, _i64, _i32, _p, _p, _p, C.c_int, _p, _i64, C.c_int,
             _p, _i64, C.c_int, C.c_int, _p, C.c_size_t, _p])
_sb_ws = _sig("insum_spmm_blockgroupcoo_workspace_bytes", C.c_size_t,
              [_i64, _i64, _i64, _i32, _i32, _i32])
_sb = _sig("insum_spmm_blockgroupcoo", C.c_int,
           [_i64, _i64, _i64, _i64, _i32, _i32, _i32, _p, _p, _p, C.c_int, _p, _i64, C.c_int,
            _p, _i64, C.c_int, C.c_int, _p, C.c_size_t, _p])
_sb_plan = _sig("insum_spmm_blockgroupcoo_plan", C.c_int,
                [_i64, _i64, _i64, _i64, _i32, _i32, _i32, _p, _p, C.c_size_t, _p])
_m_ws = _sig("insum_map_to_groupcoo_workspace_bytes", C.c_size_t, [_i64, _i64])
_m_conv = _sig("insum_map_to_groupcoo", C.c_int,
               [_i64, _i64, _i64, _i64, _p, _p, _p, _p, C.c_int, _i32, _p, _p, _p, _p, _p, _p, _i64,
                _p, C.c_size_t, _p])
_conv_ws = _sig("insum_spconv_groupcoo_workspace_bytes", C.c_size_t,
                [_i64, _i64, _i64, _i64, _i64, _i32, C.c_int])
_conv = _sig("insum_spconv_groupcoo", C.c_int,
             [_i64, _i64, _i64, _i64, _i64, _i64, _i32, _p, _p, _p, _p, _p, _i64, _p, C.c_int,
              _p, _i64, C.c_int, C.c_int, _p, C.c_size_t, _p])


class InsumError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"{where}: {insum_status_string(status)} (status {status})")
        self.status = status


def _check(status: int, where: str):
    if status != OK:
        raise InsumError(status, where)


def _dev(t: torch.Tensor, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t


def _ptr(t) -> int:
    return 0 if t is None or t.numel() == 0 else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def insum_version() -> int:
    return int(_version())


def insum_status_string(status: int) -> str:
    return _status_string(int(status)).decode()


def insum_default_group_size(S: int, n: int) -> int:
    return int(_default_g(int(S), int(n)))


def insum_indirect_access_cost(occ, g: int) -> int:
    arr = (C.c_int64 * len(occ))(*[int(x) for x in occ])
    return int(_cost(len(occ), C.cast(arr, _p), int(g)))


def insum_group_size_candidates(S: int, n: int) -> list:
    out = (C.c_int32 * 3)()
    k = int(_cand(int(S), int(n), C.cast(out, _p)))
    return [int(out[i]) for i in range(k)]


def insum_choose_group_size(M: int, K: int, row, col, val, B: torch.Tensor, C_out: torch.Tensor | None = None,
                            repeats: int = 5):
    """Times the GroupCOO SpMM for the candidate group sizes of Section 4.2 on (row, col, val) x B.
    Returns (best_g, {g: ms per launch})."""
    row, col, val = _dev(row, "row"), _dev(col, "col"), _dev(val, "val")
    assert B.is_cuda and B.dim() == 2 and B.shape[0] == K and B.stride(1) == 1 and B.dtype == val.dtype
    N, nnz = B.shape[1], row.numel()
    C_out = _out(C_out, M, N, B.dtype, B.device, False)
    ws = torch.empty(int(_choose_ws(M, N, nnz, _DTYPE[val.dtype])), dtype=torch.uint8, device=B.device)
    best, n = _i32(0), _i32(0)
    cand, ms = (C.c_int32 * 3)(), (C.c_float * 3)()
    _check(_choose(M, K, N, nnz, _ptr(row), _ptr(col), _ptr(val), _DTYPE[val.dtype], _ptr(B), B.stride(0),
                   _ptr(C_out), C_out.stride(0), _DTYPE[C_out.dtype], int(repeats), C.addressof(best),
                   C.cast(cand, _p), C.cast(ms, _p), C.addressof(n), _ptr(ws), ws.numel(), _stream()),
           "insum_choose_group_size")
    return best.value, {int(cand[i]): float(ms[i]) for i in range(n.value)}


@dataclass
class GroupCOO:
    M: int
    K: int
    g: int
    AM: torch.Tensor   # int32 [G]
    AK: torch.Tensor   # int32 [G, g]
    AV: torch.Tensor   # dtype [G, g]

    @property
    def G(self) -> int:
        return int(self.AM.shape[0])


@dataclass
class BlockGroupCOO:
    M: int
    K: int
    bM: int
    bK: int
    g: int
    AM: torch.Tensor   # int32 [G]          block rows
    AK: torch.Tensor   # int32 [G, g]       block columns
    AV: torch.Tensor   # dtype [G, g, bM, bK]
    plans: dict = field(default_factory=dict, repr=False)   # N -> planned workspace (see insum_spmm_blockgroupcoo_plan)

    @property
    def G(self) -> int:
        return int(self.AM.shape[0])


@dataclass
class MapGroupCOO:
    X: int
    Y: int
    Z: int
    g: int
    MAPZ: torch.Tensor   # int32 [G]      kernel offset of each group
    MAPX: torch.Tensor   # int32 [G, g]   output points
    MAPY: torch.Tensor   # int32 [G, g]   input points
    MAPV: torch.Tensor   # dtype [G, g]

    @property
    def G(self) -> int:
        return int(self.MAPZ.shape[0])


def insum_coo_to_groupcoo(M: int, K: int, row, col, val, g: int = 0) -> GroupCOO:
    row, col, val = _dev(row, "row"), _dev(col, "col"), _dev(val, "val")
    assert row.dtype == torch.int32 and col.dtype == torch.int32 and val.dtype in _DTYPE
    nnz = row.numel()
    assert col.numel() == nnz and val.numel() == nnz
    dev = val.device
    ws = torch.empty(int(_g_ws(M, nnz)), dtype=torch.uint8, device=dev)
    g_used, G = _i32(0), _i64(0)
    # One fill call into buffers sized by the bound G <= nnz/g + min(M, nnz) (insum.h); the
    # results are views of the first G groups.
    g_eff = int(g) if g else insum_default_group_size(nnz, M)
    cap = nnz // g_eff + min(M, nnz)
    AM = torch.empty(cap, dtype=torch.int32, device=dev)
    AK = torch.empty((cap, g_eff), dtype=torch.int32, device=dev)
    AV = torch.empty((cap, g_eff), dtype=val.dtype, device=dev)
    if nnz:
        _check(_g_conv(M, K, nnz, _ptr(row), _ptr(col), _ptr(val), _DTYPE[val.dtype], int(g),
                       C.addressof(g_used), C.addressof(G), _ptr(AM), _ptr(AK), _ptr(AV), cap,
                       _ptr(ws), ws.numel(), _stream()), "insum_coo_to_groupcoo")
    else:
        g_used.value = g_eff
    AM, AK, AV = AM[:G.value], AK[:G.value], AV[:G.value]
    return GroupCOO(M, K, g_used.value, AM, AK, AV)


def insum_groupcoo_transpose(A: GroupCOO, g: int = 0) -> GroupCOO:
    """GroupCOO of A^T built on the device from the GroupCOO of A, in one fill call: the outputs
    are sized by the bounds of insum.h for the largest group size the call can choose (the number
    of entries, which decides the default group size, is at most the number of slots), and the
    result is a view of the first G groups."""
    dev = A.AV.device
    slots = A.G * A.g
    ws = torch.empty(max(1, int(_gt_ws(A.M, A.K, A.G, A.g))), dtype=torch.uint8, device=dev)
    g_used, G, entries = _i32(0), _i64(0), _i64(0)
    g_max = int(g) if g else insum_default_group_size(slots, A.K)
    cap = slots + min(A.K, slots)                       # groups: entries/g + min(K, entries), any g >= 1
    AM = torch.empty(cap, dtype=torch.int32, device=dev)
    flat = slots + min(A.K, slots) * g_max              # slots of the result: cap(g) * g for g <= g_max
    AK = torch.empty(flat, dtype=torch.int32, device=dev)
    AV = torch.empty(flat, dtype=A.AV.dtype, device=dev)
    _check(_gt(A.M, A.K, A.G, A.g, _ptr(A.AM), _ptr(A.AK), _ptr(A.AV), _DTYPE[A.AV.dtype], int(g),
               C.addressof(g_used), C.addressof(G), C.addressof(entries), _ptr(AM), _ptr(AK), _ptr(AV),
               cap, _ptr(ws), ws.numel(), _stream()), "insum_groupcoo_transpose")
    n, gu = G.value, g_used.value
    return GroupCOO(A.K, A.M, gu, AM[:n], AK[:n * gu].view(n, gu), AV[:n * gu].view(n, gu))


def insum_coo_to_blockgroupcoo(M: int, K: int, row, col, val, bM: int, bK: int, g: int = 0) -> BlockGroupCOO:
    row, col, val = _dev(row, "row"), _dev(col, "col"), _dev(val, "val")
    assert row.dtype == torch.int32 and col.dtype == torch.int32 and val.dtype in _DTYPE
    nnz = row.numel()
    assert col.numel() == nnz and val.numel() == nnz
    dev = val.device
    ws = torch.empty(int(_b_ws(M, K, nnz, bM, bK)), dtype=torch.uint8, device=dev)
    g_used, G = _i32(0), _i64(0)
    args = (M, K, nnz, _ptr(row), _ptr(col), _ptr(val), _DTYPE[val.dtype], int(bM), int(bK), int(g),
            C.addressof(g_used), C.addressof(G))
    _check(_b_conv(*args, 0, 0, 0, 0, _ptr(ws), ws.numel(), _stream()),
           "insum_coo_to_blockgroupcoo(count)")
    AM = torch.empty(G.value, dtype=torch.int32, device=dev)
    AK = torch.empty((G.value, g_used.value), dtype=torch.int32, device=dev)
    AV = torch.empty((G.value, g_used.value, bM, bK), dtype=val.dtype, device=dev)
    if G.value:
        _check(_b_conv(*args, _ptr(AM), _ptr(AK), _ptr(AV), G.value, _ptr(ws), ws.numel(), _stream()),
               "insum_coo_to_blockgroupcoo(fill)")
    return BlockGroupCOO(M, K, bM, bK, g_used.value, AM, AK, AV)


def insum_spmm_groupcoo_workspace_bytes(M: int, N: int, G: int, g: int) -> int:
    return int(_sg_ws(M, N, G, g))


def insum_spmm_blockgroupcoo_workspace_bytes(M: int, N: int, G: int, g: int, bM: int, bK: int) -> int:
    return int(_sb_ws(M, N, G, g, bM, bK))


def _out(C_out, M, N, dtype, dev, accumulate):
    if C_out is None:
        if accumulate:
            raise ValueError("accumulate=True needs an existing C")
        C_out = torch.empty((M, N), dtype=dtype, device=dev)
    assert C_out.is_cuda and C_out.dim() == 2 and C_out.shape == (M, N) and C_out.stride(1) == 1
    return C_out


def insum_spmm_groupcoo(A: GroupCOO, B: torch.Tensor, C_out: torch.Tensor | None = None,
                        accumulate: bool = False, out_dtype=None, workspace=None) -> torch.Tensor:
    """C = A @ B (or C += A @ B) with A in GroupCOO.  B: [K, N] row-major device tensor."""
    assert B.is_cuda and B.dim() == 2 and B.shape[0] == A.K and B.stride(1) == 1
    N = B.shape[1]
    C_out = _out(C_out, A.M, N, out_dtype or B.dtype, B.device, accumulate)
    if workspace is None:
        workspace = torch.empty(insum_spmm_groupcoo_workspace_bytes(A.M, N, A.G, A.g),
                                dtype=torch.uint8, device=B.device)
    st = _sg(A.M, A.K, N, A.G, A.g, _ptr(A.AM), _ptr(A.AK), _ptr(A.AV), _DTYPE[A.AV.dtype],
             _ptr(B), B.stride(0), _DTYPE[B.dtype], _ptr(C_out), C_out.stride(0),
             _DTYPE[C_out.dtype], int(bool(accumulate)), _ptr(workspace), workspace.numel(), _stream())
    _check(st, "insum_spmm_groupcoo")
    return C_out


def insum_spmm_groupcoo_noalloc(A: GroupCOO, B: torch.Tensor, C_out: torch.Tensor,
                                accumulate: bool = False) -> torch.Tensor:
    """insum_spmm_groupcoo without a workspace; C_out is required (the call allocates nothing)."""
    assert B.is_cuda and B.dim() == 2 and B.shape[0] == A.K and B.stride(1) == 1
    N = B.shape[1]
    assert C_out.is_cuda and C_out.dim() == 2 and C_out.shape == (A.M, N) and C_out.stride(1) == 1
    st = _sg_na(A.M, A.K, N, A.G, A.g, _ptr(A.AM), _ptr(A.AK), _ptr(A.AV), _DTYPE[A.AV.dtype],
                _ptr(B), B.stride(0), _DTYPE[B.dtype], _ptr(C_out), C_out.stride(0),
                _DTYPE[C_out.dtype], int(bool(accumulate)), _stream())
    _check(st, "insum_spmm_groupcoo_noalloc")
    return C_out


def insum_spmm_groupcoo_transposed(A: GroupCOO, E: torch.Tensor, D_out: torch.Tensor | None = None,
                                   accumulate: bool = False, out_dtype=None, workspace=None) -> torch.Tensor:
    """D = A^T @ E (or D += A^T @ E) over the same GroupCOO arrays.  E: [M, N] row-major."""
    assert E.is_cuda and E.dim() == 2 and E.shape[0] == A.M and E.stride(1) == 1
    N = E.shape[1]
    D_out = _out(D_out, A.K, N, out_dtype or E.dtype, E.device, accumulate)
    nws = int(_sgt_ws(A.K, N, _DTYPE[D_out.dtype]))
    if workspace is None and nws:
        workspace = torch.empty(nws, dtype=torch.uint8, device=E.device)
    st = _sgt(A.M, A.K, N, A.G, A.g, _ptr(A.AM), _ptr(A.AK), _ptr(A.AV), _DTYPE[A.AV.dtype],
              _ptr(E), E.stride(0), _DTYPE[E.dtype], _ptr(D_out), D_out.stride(0), _DTYPE[D_out.dtype],
              int(bool(accumulate)), _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream())
    _check(st, "insum_spmm_groupcoo_transposed")
    return D_out


def insum_spmm_blockgroupcoo_plan(A: BlockGroupCOO, N: int) -> torch.Tensor | None:
    """Builds the work plan of A for dense width N in a fresh workspace and returns it (None for
    shapes that take no plan).  The plan stays valid while A.AM is unchanged."""
    nws = insum_spmm_blockgroupcoo_workspace_bytes(A.M, N, A.G, A.g, A.bM, A.bK)
    if nws == 0:
        return None
    ws = torch.empty(nws, dtype=torch.uint8, device=A.AM.device)
    _check(_sb_plan(A.M, A.K, N, A.G, A.g, A.bM, A.bK, _ptr(A.AM), _ptr(ws), ws.numel(), _stream()),
           "insum_spmm_blockgroupcoo_plan")
    return ws


def insum_spmm_blockgroupcoo(A: BlockGroupCOO, B: torch.Tensor, C_out: torch.Tensor | None = None,
                             accumulate: bool = False, out_dtype=None, workspace=None,
                             plan: bool = True) -> torch.Tensor:
    """C = A @ B (or C += A @ B) with A in BlockGroupCOO.  `workspace`: a planned workspace from
    insum_spmm_blockgroupcoo_plan; when it is None and `plan` is true, the plan for this N is
    built on first use and kept in A.plans; plan=False passes no workspace at all."""
    assert B.is_cuda and B.dim() == 2 and B.shape[0] == A.K and B.stride(1) == 1
    N = B.shape[1]
    C_out = _out(C_out, A.M, N, out_dtype or B.dtype, B.device, accumulate)
    if workspace is None and plan and A.G:
        if N not in A.plans:
            A.plans[N] = insum_spmm_blockgroupcoo_plan(A, N)
        workspace = A.plans[N]
    st = _sb(A.M, A.K, N, A.G, A.g, A.bM, A.bK, _ptr(A.AM), _ptr(A.AK), _ptr(A.AV),
             _DTYPE[A.AV.dtype], _ptr(B), B.stride(0), _DTYPE[B.dtype], _ptr(C_out),
             C_out.stride(0), _DTYPE[C_out.dtype], int(bool(accumulate)), _ptr(workspace),
             0 if workspace is None else workspace.numel(), _stream())
    _check(st, "insum_spmm_blockgroupcoo")
    return C_out


def insum_map_to_groupcoo(X: int, Y: int, Z: int, mx, my, mz, mv, g: int = 0) -> MapGroupCOO:
    """Groups the kernel map Map[x, y, z] of a sparse convolution along its offsets z."""
    mx, my, mz, mv = _dev(mx, "mx"), _dev(my, "my"), _dev(mz, "mz"), _dev(mv, "mv")
    assert mx.dtype == my.dtype == mz.dtype == torch.int32 and mv.dtype in _DTYPE
    nnz = mx.numel()
    assert my.numel() == nnz and mz.numel() == nnz and mv.numel() == nnz
    dev = mv.device
    ws = torch.empty(int(_m_ws(Z, nnz)), dtype=torch.uint8, device=dev)
    g_used, G = _i32(0), _i64(0)
    g_eff = int(g) if g else insum_default_group_size(nnz, Z)
    cap = nnz // g_eff + min(Z, nnz)            # bound on G stated in insum.h
    MAPZ = torch.empty(cap, dtype=torch.int32, device=dev)
    MAPX = torch.empty((cap, g_eff), dtype=torch.int32, device=dev)
    MAPY = torch.empty((cap, g_eff), dtype=torch.int32, device=dev)
    MAPV = torch.empty((cap, g_eff), dtype=mv.dtype, device=dev)
    if nnz:
        _check(_m_conv(X, Y, Z, nnz, _ptr(mx), _ptr(my), _ptr(mz), _ptr(mv), _DTYPE[mv.dtype], int(g),
                       C.addressof(g_used), C.addressof(G), _ptr(MAPZ), _ptr(MAPX), _ptr(MAPY), _ptr(MAPV),
                       cap, _ptr(ws), ws.numel(), _stream()), "insum_map_to_groupcoo")
    else:
        g_used.value = g_eff
    n = G.value
    return MapGroupCOO(X, Y, Z, g_used.value, MAPZ[:n], MAPX[:n], MAPY[:n], MAPV[:n])


def insum_map_count_groups(X: int, Y: int, Z: int, mx, my, mz, g: int = 0):
    """Count mode of insum_map_to_groupcoo: returns (g_used, G) without writing the format."""
    nnz = mx.numel()
    ws = torch.empty(int(_m_ws(Z, nnz)), dtype=torch.uint8, device=mx.device)
    g_used, G = _i32(0), _i64(0)
    dummy = torch.zeros(max(nnz, 1), dtype=torch.float16, device=mx.device)
    _check(_m_conv(X, Y, Z, nnz, _ptr(mx), _ptr(my), _ptr(mz), _ptr(dummy), 1, int(g),
                   C.addressof(g_used), C.addressof(G), 0, 0, 0, 0, 0, _ptr(ws), ws.numel(), _stream()),
           "insum_map_to_groupcoo(count)")
    return g_used.value, G.value


def insum_spconv_groupcoo_workspace_bytes(Map: MapGroupCOO, C_in: int, M_out: int, dtype) -> int:
    return int(_conv_ws(Map.X, Map.Z, C_in, M_out, Map.G, Map.g, _DTYPE[dtype]))


def insum_spconv_groupcoo(Map: MapGroupCOO, In: torch.Tensor, W: torch.Tensor,
                          Out: torch.Tensor | None = None, accumulate: bool = False,
                          workspace=None, reuse_map_tables: bool = False) -> torch.Tensor:
    """Out[MAPX[p,q], m] (+)= MAPV[p,q] * In[MAPY[p,q], c] * W[MAPZ[p], c, m]; Out is fp32 [X, M]."""
    assert In.is_cuda and In.dim() == 2 and In.shape[0] == Map.Y and In.stride(1) == 1
    assert W.is_cuda and W.dim() == 3 and W.is_contiguous() and W.shape[0] == Map.Z
    assert W.shape[1] == In.shape[1] and W.dtype == In.dtype
    assert Map.G == 0 or Map.MAPV.dtype == In.dtype
    Cc, M = int(W.shape[1]), int(W.shape[2])
    Out = _out(Out, Map.X, M, torch.float32, In.device, accumulate)
    assert Out.dtype == torch.float32
    nws = insum_spconv_groupcoo_workspace_bytes(Map, Cc, M, In.dtype)
    if workspace is None and nws:
        if reuse_map_tables:
            raise ValueError("reuse_map_tables=True needs the workspace of the earlier call")
        workspace = torch.empty(nws, dtype=torch.uint8, device=In.device)
    st = _conv(Map.X, Map.Y, Map.Z, Cc, M, Map.G, Map.g, _ptr(Map.MAPZ), _ptr(Map.MAPX), _ptr(Map.MAPY),
               _ptr(Map.MAPV), _ptr(In), In.stride(0), _ptr(W), _DTYPE[In.dtype], _ptr(Out), Out.stride(0),
               int(bool(accumulate)), int(bool(reuse_map_tables)), _ptr(workspace),
               0 if workspace is None else workspace.numel(), _stream())
    _check(st, "insum_spconv_groupcoo")
    return Out
