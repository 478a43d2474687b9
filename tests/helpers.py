"""Test-side utilities: independent decoders and the parity criterion.

Nothing here is shared with the oracle's C code or with the HIP path; the decoders are
deliberately written with different primitives (numpy scatter-add on dense matrices).
"""
from __future__ import annotations

import numpy as np


def read_golden(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            rows.append(line.split())
    return rows


def to_f32(a: np.ndarray, dtype: str) -> np.ndarray:
    """Storage array -> exact float32 values."""
    if dtype == "bf16":
        return (np.ascontiguousarray(a, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)
    return np.asarray(a).astype(np.float32)


def coo_to_dense(M, K, row, col, val64):
    A = np.zeros((M, K), dtype=np.float64)
    np.add.at(A, (row, col), val64)
    return A


def groupcoo_to_dense(M, K, AM, AK, AV64):
    A = np.zeros((M, K), dtype=np.float64)
    G, g = AK.shape
    np.add.at(A, (np.repeat(AM, g), AK.reshape(-1)), AV64.reshape(-1))
    return A


def blockgroupcoo_to_dense(M, K, bM, bK, AM, AK, AV64):
    A = np.zeros((M, K), dtype=np.float64)
    G, g = AK.shape
    for p in range(G):
        for q in range(g):
            r0, c0 = AM[p] * bM, AK[p, q] * bK
            A[r0:r0 + bM, c0:c0 + bK] += AV64[p, q]
    return A


def check_groupcoo_invariants(M, K, row, col, val, g, AM, AK, AV):
    """Structure of Section 4.1: fixed group length, one row per group, rows ascending,
    every input entry exactly once among the real slots, padding only at the tail of a
    row's last group with value +0 (all bits zero)."""
    G = AM.shape[0]
    assert AK.shape == (G, g) and AV.shape == (G, g)
    occ = np.bincount(row, minlength=M)
    assert G == int(np.sum((occ + g - 1) // g))
    assert np.all(np.diff(AM) >= 0)
    if G:
        assert AK.min() >= 0 and AK.max() < K
    groups_of_row = np.bincount(AM, minlength=M)
    assert np.array_equal(groups_of_row, (occ + g - 1) // g)
    # number of real slots in each group: full except the last group of its row
    first_group = np.concatenate([[0], np.cumsum(groups_of_row)[:-1]])
    j = np.arange(G) - first_group[AM]                      # index of the group in its row
    real = np.minimum(g, occ[AM] - j * g)
    assert np.all(real >= 1)
    slot = np.arange(g)[None, :]
    is_real = slot < real[:, None]
    raw = AV.view(np.uint16 if AV.dtype.itemsize == 2 else np.uint32)
    assert np.all(raw[~is_real] == 0), "padding value must be +0"
    last_real_col = AK[np.arange(G), real - 1]
    assert np.all((AK == last_real_col[:, None])[~is_real]), "padding repeats last real column"
    # multiset of (row, col, value bits) is preserved
    got = np.stack([np.repeat(AM, g)[is_real.reshape(-1)].astype(np.int64),
                    AK.reshape(-1)[is_real.reshape(-1)].astype(np.int64),
                    raw.reshape(-1)[is_real.reshape(-1)].astype(np.int64)], axis=1)
    vraw = np.ascontiguousarray(val).view(np.uint16 if val.dtype.itemsize == 2 else np.uint32)
    want = np.stack([row.astype(np.int64), col.astype(np.int64), vraw.astype(np.int64)], axis=1)
    got = got[np.lexsort(got.T[::-1])]
    want = want[np.lexsort(want.T[::-1])]
    assert np.array_equal(got, want)
    # inside a row the columns are non-decreasing across consecutive real slots
    flat_row = np.repeat(AM, g)[is_real.reshape(-1)]
    flat_col = AK.reshape(-1)[is_real.reshape(-1)]
    same = flat_row[1:] == flat_row[:-1]
    assert np.all(flat_col[1:][same] >= flat_col[:-1][same])


def assert_spmm_close(C_got, C64, absprod64, rtol, what="", out_dtype=None):
    """Parity criterion: max error relative to max|C| and a componentwise bound against
    (|A| |B|), which does not suffer from cancellation.  A result stored as fp16 cannot be
    closer to the exact value than half the spacing of fp16 subnormals (2^-25) wherever that
    value is below the normal range, so out_dtype="f16" adds that much to the bound."""
    C_got = np.asarray(C_got, dtype=np.float64)
    E = np.abs(C_got - C64)
    scale = max(float(np.max(np.abs(C64))) if C64.size else 0.0, 1e-300)
    assert not np.any(np.isnan(C_got)), f"{what}: NaN in result"
    worst = float(E.max()) if E.size else 0.0
    assert worst <= rtol * scale, f"{what}: max err {worst:.3e} > {rtol} * {scale:.3e}"
    bound = rtol * absprod64 + (2.0 ** -25 if out_dtype == "f16" else 1e-30)
    bad = E > bound
    assert not bad.any(), (f"{what}: {int(bad.sum())} elements exceed the componentwise bound; "
                           f"worst ratio {float((E / bound).max()):.3f}")
