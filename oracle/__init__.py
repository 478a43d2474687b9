"""ctypes front end of the C oracle (``insum_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the HIP library and its
Python binding never do.  The functions below marshal numpy arrays and call the C
loops; the definitions they implement are cited in the C file's header.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import build as _build

_lib = C.CDLL(_build())

_i64 = C.c_int64
_p = C.c_void_p


def _ptr(a):
    return a.ctypes.data_as(_p)


_lib.oracle_canonical_order.restype = C.c_int
_lib.oracle_canonical_order.argtypes = [_i64, _i64, _i64, _p, _p, _p]
_lib.oracle_indirect_access_cost.restype = _i64
_lib.oracle_indirect_access_cost.argtypes = [_i64, _p, _i64]
_lib.oracle_relaxed_cost.restype = C.c_double
_lib.oracle_relaxed_cost.argtypes = [C.c_double] * 3
_lib.oracle_gstar.restype = C.c_double
_lib.oracle_gstar.argtypes = [C.c_double] * 2
_lib.oracle_default_group_size.restype = _i64
_lib.oracle_default_group_size.argtypes = [_i64, _i64]
_lib.oracle_groupcoo_num_groups.restype = _i64
_lib.oracle_groupcoo_num_groups.argtypes = [_i64, _i64, _p, _i64, _p]
_lib.oracle_coo_to_groupcoo.restype = C.c_int
_lib.oracle_coo_to_groupcoo.argtypes = [_i64, _i64, _i64, _p, _p, _p, C.c_int, _i64, _p, _p, _p]
_lib.oracle_nonzero_blocks.restype = C.c_int
_lib.oracle_nonzero_blocks.argtypes = [_i64, _i64, _i64, _p, _p, _i64, _i64, _p, _p, _p, _p]
_lib.oracle_coo_to_blockgroupcoo.restype = C.c_int
_lib.oracle_coo_to_blockgroupcoo.argtypes = [_i64, _i64, _i64, _p, _p, _p, C.c_int, _i64, _i64,
                                             _i64, _i64, _p, _p, _i64, _p, _p, _p]
_lib.oracle_spmm_groupcoo.restype = None
_lib.oracle_spmm_groupcoo.argtypes = [_i64] * 5 + [_p, _p, _p, _p, _i64, _p, _i64]
_lib.oracle_spmm_groupcoo_transposed.restype = None
_lib.oracle_spmm_groupcoo_transposed.argtypes = [_i64] * 5 + [_p, _p, _p, _p, _i64, _p, _i64]
_lib.oracle_enclosing_powers_of_two.restype = None
_lib.oracle_enclosing_powers_of_two.argtypes = [_i64, _i64, _p, _p]
_lib.oracle_spmm_blockgroupcoo.restype = None
_lib.oracle_spmm_blockgroupcoo.argtypes = [_i64] * 7 + [_p, _p, _p, _p, _i64, _p, _i64]
_lib.oracle_map_order.restype = C.c_int
_lib.oracle_map_order.argtypes = [_i64, _i64, _i64, _i64, _p, _p, _p, _p]
_lib.oracle_map_num_groups.restype = _i64
_lib.oracle_map_num_groups.argtypes = [_i64, _i64, _p, _i64, _p]
_lib.oracle_map_to_groupcoo.restype = C.c_int
_lib.oracle_map_to_groupcoo.argtypes = [_i64, _i64, _i64, _i64, _p, _p, _p, _p, C.c_int, _i64, _p, _p, _p, _p]
_lib.oracle_spconv_groupcoo.restype = None
_lib.oracle_spconv_groupcoo.argtypes = [_i64, _i64, _i64, _i64, _p, _p, _p, _p, _p, _i64, _p, _p, _i64]
_lib.oracle_num_threads.restype = C.c_int

ERR_OUT_OF_RANGE = 2
ERR_DUPLICATE = 3
ERR_UNSUPPORTED = 5


class OracleError(ValueError):
    def __init__(self, code: int):
        super().__init__(f"oracle error code {code}")
        self.code = code


def _coords(row, col):
    row = np.ascontiguousarray(row, dtype=np.int32)
    col = np.ascontiguousarray(col, dtype=np.int32)
    assert row.shape == col.shape and row.ndim == 1
    return row, col


def num_threads() -> int:
    return int(_lib.oracle_num_threads())


def canonical_order(M, K, row, col) -> np.ndarray:
    row, col = _coords(row, col)
    perm = np.empty(row.shape[0], dtype=np.int64)
    rc = _lib.oracle_canonical_order(M, K, row.shape[0], _ptr(row), _ptr(col), _ptr(perm))
    if rc:
        raise OracleError(rc)
    return perm


def indirect_access_cost(occ, g: int) -> int:
    occ = np.ascontiguousarray(occ, dtype=np.int64)
    return int(_lib.oracle_indirect_access_cost(occ.shape[0], _ptr(occ), int(g)))


def relaxed_cost(S: float, n: float, g: float) -> float:
    return float(_lib.oracle_relaxed_cost(float(S), float(n), float(g)))


def gstar(S: float, n: float) -> float:
    return float(_lib.oracle_gstar(float(S), float(n)))


def default_group_size(S: int, n: int) -> int:
    return int(_lib.oracle_default_group_size(int(S), int(n)))


def enclosing_powers_of_two(S: int, n: int):
    """(lo, hi): the powers of two below and above g* = sqrt(S/n) (equal when g* is one itself)."""
    lo, hi = C.c_int64(0), C.c_int64(0)
    _lib.oracle_enclosing_powers_of_two(int(S), int(n), C.addressof(lo), C.addressof(hi))
    return int(lo.value), int(hi.value)


def coo_to_groupcoo(M, K, row, col, val, g=None):
    """val: numpy array in its storage type (float32, float16 or uint16 bf16 bits).
    Returns (g, AM[G], AK[G,g], AV[G,g]) with AV in the same storage type."""
    row, col = _coords(row, col)
    val = np.ascontiguousarray(val)
    nnz = row.shape[0]
    assert val.shape == (nnz,) and val.dtype.itemsize in (2, 4)
    if np.any((row < 0) | (row >= M)) or np.any((col < 0) | (col >= K)):
        raise OracleError(ERR_OUT_OF_RANGE)
    if g is None or g == 0:
        g = default_group_size(nnz, M)
    occ = np.empty(max(M, 1), dtype=np.int64)
    G = int(_lib.oracle_groupcoo_num_groups(M, nnz, _ptr(row), int(g), _ptr(occ)))
    AM = np.empty(G, dtype=np.int32)
    AK = np.empty((G, g), dtype=np.int32)
    AV = np.empty((G, g), dtype=val.dtype)
    rc = _lib.oracle_coo_to_groupcoo(M, K, nnz, _ptr(row), _ptr(col), _ptr(val),
                                     val.dtype.itemsize, int(g), _ptr(AM), _ptr(AK), _ptr(AV))
    if rc:
        raise OracleError(rc)
    return int(g), AM, AK, AV


def groupcoo_real_slots(AK, AV) -> np.ndarray:
    """Boolean [G, g]: which slots of a GroupCOO matrix hold entries.  Section 4.1 pads the last
    group of a row; by this build's reading a padding slot has value +0 (all bits zero) and
    repeats the column of the slot to its left, so padding is recognised from the arrays alone:
    slot q > 0 is padding when its value bits are zero and AK[p, q] == AK[p, q - 1].  (A stored
    +0 entry that repeats the coordinate of the entry before it looks the same and is treated
    the same; it contributes nothing to any product.)"""
    AK = np.asarray(AK)
    bits = np.ascontiguousarray(AV).view({2: np.uint16, 4: np.uint32}[np.asarray(AV).dtype.itemsize])
    real = np.ones(AK.shape, dtype=bool)
    G, g = AK.shape
    for p_ in range(G):
        for q in range(1, g):
            real[p_, q] = not (bits[p_, q] == 0 and AK[p_, q] == AK[p_, q - 1])
    return real


def groupcoo_transpose(M, K, AM, AK, AV, g_t=None):
    """GroupCOO of A^T (K rows, M columns) from the GroupCOO of A: the entries of A, read off the
    format in slot order with padding left out, with row and column exchanged, grouped again as
    Section 4.1 prescribes.  Returns (g_t, AM_t, AK_t, AV_t)."""
    AM, AK, AV = np.asarray(AM), np.asarray(AK), np.ascontiguousarray(AV)
    real = groupcoo_real_slots(AK, AV)
    rows, cols, vals = [], [], []
    for p_ in range(AK.shape[0]):
        for q in range(AK.shape[1]):
            if real[p_, q]:
                rows.append(AK[p_, q])      # the column of A is the row of A^T
                cols.append(AM[p_])
                vals.append(AV[p_, q])
    return coo_to_groupcoo(K, M, np.array(rows, dtype=np.int32), np.array(cols, dtype=np.int32),
                           np.array(vals, dtype=AV.dtype), g_t)


def coo_to_blockgroupcoo(M, K, row, col, val, bM, bK, g=None):
    """Returns (g, AM[G], AK[G,g], AV[G,g,bM,bK]); AM/AK hold block coordinates."""
    row, col = _coords(row, col)
    val = np.ascontiguousarray(val)
    nnz = row.shape[0]
    assert val.shape == (nnz,) and val.dtype.itemsize in (2, 4)
    if bM <= 0 or bK <= 0 or M % bM or K % bK:
        raise OracleError(ERR_UNSUPPORTED)
    nbr = M // bM
    blk_row = np.empty(max(nnz, 1), dtype=np.int32)
    blk_col = np.empty(max(nnz, 1), dtype=np.int32)
    occ = np.zeros(max(nbr, 1), dtype=np.int64)
    nb = _i64(0)
    rc = _lib.oracle_nonzero_blocks(M, K, nnz, _ptr(row), _ptr(col), bM, bK, C.byref(nb),
                                    _ptr(blk_row), _ptr(blk_col), _ptr(occ))
    if rc:
        raise OracleError(rc)
    nb = nb.value
    if g is None or g == 0:
        g = default_group_size(nb, nbr)
    G = int(np.sum((occ[:nbr] + g - 1) // g)) if nbr else 0
    AM = np.empty(G, dtype=np.int32)
    AK = np.empty((G, g), dtype=np.int32)
    AV = np.empty((G, g, bM, bK), dtype=val.dtype)
    rc = _lib.oracle_coo_to_blockgroupcoo(M, K, nnz, _ptr(row), _ptr(col), _ptr(val),
                                          val.dtype.itemsize, bM, bK, int(g), nb,
                                          _ptr(blk_row), _ptr(blk_col), G,
                                          _ptr(AM), _ptr(AK), _ptr(AV))
    if rc:
        raise OracleError(rc)
    return int(g), AM, AK, AV


def _f32(a):
    a = np.asarray(a)
    assert a.dtype in (np.float32, np.float16), "pass values as float32/float16 (bf16: upcast first)"
    return np.ascontiguousarray(a, dtype=np.float32)


def spmm_groupcoo(M, K, N, AM, AK, AV, B, C_init=None) -> np.ndarray:
    """fp64 result of C[AM[p], n] += AV[p,q] * B[AK[p,q], n] (C starts at C_init or zero)."""
    AM = np.ascontiguousarray(AM, dtype=np.int32)
    AK = np.ascontiguousarray(AK, dtype=np.int32)
    AV = _f32(AV)
    B = _f32(B)
    G = AM.shape[0]
    g = AK.shape[1] if AK.ndim == 2 else 1
    assert AK.size == G * g and AV.size == G * g and B.shape == (K, N)
    Cd = np.zeros((M, N), dtype=np.float64) if C_init is None else \
        np.array(C_init, dtype=np.float64, order="C")
    assert Cd.shape == (M, N)
    if G:
        assert AM.min() >= 0 and AM.max() < M and AK.min() >= 0 and AK.max() < K
    _lib.oracle_spmm_groupcoo(M, K, N, G, g, _ptr(AM), _ptr(AK), _ptr(AV), _ptr(B), N, _ptr(Cd), N)
    return Cd


def spmm_groupcoo_transposed(M, K, N, AM, AK, AV, E, D_init=None) -> np.ndarray:
    """fp64 result of D[AK[p,q], n] += AV[p,q] * E[AM[p], n] (D = A^T E; starts at D_init or zero)."""
    AM = np.ascontiguousarray(AM, dtype=np.int32)
    AK = np.ascontiguousarray(AK, dtype=np.int32)
    AV = _f32(AV)
    E = _f32(E)
    G = AM.shape[0]
    g = AK.shape[1] if AK.ndim == 2 else 1
    assert AK.size == G * g and AV.size == G * g and E.shape == (M, N)
    Dd = np.zeros((K, N), dtype=np.float64) if D_init is None else \
        np.array(D_init, dtype=np.float64, order="C")
    assert Dd.shape == (K, N)
    if G:
        assert AM.min() >= 0 and AM.max() < M and AK.min() >= 0 and AK.max() < K
    _lib.oracle_spmm_groupcoo_transposed(M, K, N, G, g, _ptr(AM), _ptr(AK), _ptr(AV), _ptr(E), N, _ptr(Dd), N)
    return Dd


def spmm_blockgroupcoo(M, K, N, bM, bK, AM, AK, AV, B, C_init=None) -> np.ndarray:
    AM = np.ascontiguousarray(AM, dtype=np.int32)
    AK = np.ascontiguousarray(AK, dtype=np.int32)
    AV = _f32(AV)
    B = _f32(B)
    G = AM.shape[0]
    g = AK.shape[1] if AK.ndim == 2 else 1
    assert AK.size == G * g and AV.size == G * g * bM * bK and B.shape == (K, N)
    Cd = np.zeros((M, N), dtype=np.float64) if C_init is None else \
        np.array(C_init, dtype=np.float64, order="C")
    assert Cd.shape == (M, N)
    if G:
        assert AM.min() >= 0 and (AM.max() + 1) * bM <= M
        assert AK.min() >= 0 and (AK.max() + 1) * bK <= K
    _lib.oracle_spmm_blockgroupcoo(M, K, N, G, g, bM, bK, _ptr(AM), _ptr(AK), _ptr(AV), _ptr(B),
                                   N, _ptr(Cd), N)
    return Cd


def map_to_groupcoo(X, Y, Z, mx, my, mz, mv, g=None):
    """Kernel map (COO of the 3-D tensor Map[x, y, z]) -> groups along z.
    Returns (g, MAPZ[G], MAPX[G,g], MAPY[G,g], MAPV[G,g])."""
    mx = np.ascontiguousarray(mx, dtype=np.int32)
    my = np.ascontiguousarray(my, dtype=np.int32)
    mz = np.ascontiguousarray(mz, dtype=np.int32)
    mv = np.ascontiguousarray(mv)
    nnz = mx.shape[0]
    assert my.shape == (nnz,) and mz.shape == (nnz,) and mv.shape == (nnz,) and mv.dtype.itemsize in (2, 4)
    if nnz and (mx.min() < 0 or mx.max() >= X or my.min() < 0 or my.max() >= Y or mz.min() < 0 or mz.max() >= Z):
        raise OracleError(ERR_OUT_OF_RANGE)
    if g is None or g == 0:
        g = default_group_size(nnz, Z)
    occ = np.empty(max(Z, 1), dtype=np.int64)
    G = int(_lib.oracle_map_num_groups(Z, nnz, _ptr(mz), int(g), _ptr(occ)))
    MAPZ = np.empty(G, dtype=np.int32)
    MAPX = np.empty((G, g), dtype=np.int32)
    MAPY = np.empty((G, g), dtype=np.int32)
    MAPV = np.empty((G, g), dtype=mv.dtype)
    rc = _lib.oracle_map_to_groupcoo(X, Y, Z, nnz, _ptr(mx), _ptr(my), _ptr(mz), _ptr(mv), mv.dtype.itemsize,
                                     int(g), _ptr(MAPZ), _ptr(MAPX), _ptr(MAPY), _ptr(MAPV))
    if rc:
        raise OracleError(rc)
    return int(g), MAPZ, MAPX, MAPY, MAPV


def spconv_groupcoo(X, C_in, M_out, MAPZ, MAPX, MAPY, MAPV, In, W, Out_init=None) -> np.ndarray:
    """fp64 result of Out[MAPX[p,q], m] += MAPV[p,q] * In[MAPY[p,q], c] * W[MAPZ[p], c, m]."""
    MAPZ = np.ascontiguousarray(MAPZ, dtype=np.int32)
    MAPX = np.ascontiguousarray(MAPX, dtype=np.int32)
    MAPY = np.ascontiguousarray(MAPY, dtype=np.int32)
    MAPV = _f32(MAPV)
    In = _f32(In)
    W = _f32(W)
    G = MAPZ.shape[0]
    g = MAPX.shape[1] if MAPX.ndim == 2 else 1
    assert MAPX.size == G * g and MAPY.size == G * g and MAPV.size == G * g
    assert In.ndim == 2 and In.shape[1] == C_in and W.ndim == 3 and W.shape[1:] == (C_in, M_out)
    Out = np.zeros((X, M_out), dtype=np.float64) if Out_init is None else \
        np.array(Out_init, dtype=np.float64, order="C")
    if G:
        assert MAPX.min() >= 0 and MAPX.max() < X and MAPY.min() >= 0 and MAPY.max() < In.shape[0]
        assert MAPZ.min() >= 0 and MAPZ.max() < W.shape[0]
    _lib.oracle_spconv_groupcoo(C_in, M_out, G, g, _ptr(MAPZ), _ptr(MAPX), _ptr(MAPY), _ptr(MAPV),
                                _ptr(In), C_in, _ptr(W), _ptr(Out), M_out)
    return Out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact upcast of bf16 bit patterns (uint16) to float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)
