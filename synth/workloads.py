"""Seeded generators for the five benchmark workloads and for small test matrices.

The workloads stand in for the matrices the paper evaluates on (pruned weight
matrices and graph adjacency matrices, Section 6 "Case Study: Structured SpMM" /
"Unstructured SpMM"), which are not available here.  Every generator returns
plain numpy arrays:

    row, col : int32 COO coordinates (in a shuffled, non-canonical order)
    val      : float32 values that are exactly representable in ``a_dtype``
    B        : float32 dense operand, exactly representable in ``b_dtype``

16-bit tensors are drawn in fp32 and rounded once (round-to-nearest-even), so both
the oracle and the GPU path consume bit-identical inputs.
"""
from __future__ import annotations

import numpy as np

CONFIG_NAMES = ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5")


# --------------------------------------------------------------------------- #
# storage types
# --------------------------------------------------------------------------- #
def _round_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> nearest-even bf16, returned as fp32 (finite inputs only)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32 array to ``dtype`` ('f32' | 'f16' | 'bf16'); result stays fp32."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        return _round_bf16(x)
    raise ValueError(f"unknown dtype {dtype!r}")


def storage_array(x: np.ndarray, dtype: str) -> np.ndarray:
    """The in-memory representation of already-rounded values: float32, float16,
    or the uint16 bit patterns of bf16."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == "f32":
        return np.ascontiguousarray(x)
    if dtype == "f16":
        y = x.astype(np.float16)
        assert np.array_equal(y.astype(np.float32), x), "values not exact in f16"
        return y
    if dtype == "bf16":
        u = np.ascontiguousarray(x).view(np.uint32)
        assert not np.any(u & 0xFFFF), "values not exact in bf16"
        return (u >> 16).astype(np.uint16)
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------- #
# bounded Zipf
# --------------------------------------------------------------------------- #
def _zipf_pmf(alpha: float, kmax: int) -> np.ndarray:
    k = np.arange(1, kmax + 1, dtype=np.float64)
    w = k ** (-alpha)
    return w / w.sum()


def bounded_zipf_kmax(alpha: float, target_mean: float, limit: int = 1 << 20) -> int:
    """Smallest kmax such that P(k) ~ k^-alpha on [1, kmax] has mean >= target_mean."""
    num = 0.0
    den = 0.0
    for k in range(1, limit + 1):
        w = float(k) ** (-alpha)
        num += k * w
        den += w
        if num / den >= target_mean:
            return k
    raise ValueError("target mean not reachable")


def bounded_zipf_sample(rng: np.random.Generator, alpha: float, kmax: int, size: int) -> np.ndarray:
    p = _zipf_pmf(alpha, kmax)
    return rng.choice(np.arange(1, kmax + 1), size=size, p=p).astype(np.int64)


# --------------------------------------------------------------------------- #
# small test matrices
# --------------------------------------------------------------------------- #
def _streams(seed: int, n: int = 4):
    return [np.random.default_rng(s) for s in np.random.SeedSequence(seed).spawn(n)]


def _shuffle(rng, row, col, val):
    perm = rng.permutation(row.shape[0])
    return row[perm], col[perm], val[perm]


def random_coo(M: int, K: int, nnz: int, seed: int, dtype: str = "f32", sigma: float = 1.0,
               shuffle: bool = True):
    """nnz distinct positions uniform over the M x K grid, values N(0, sigma)."""
    r_pos, r_val, _, r_perm = _streams(seed)
    nnz = min(nnz, M * K)
    flat = r_pos.choice(M * K, size=nnz, replace=False) if nnz else np.zeros(0, np.int64)
    row = (flat // K).astype(np.int32)
    col = (flat % K).astype(np.int32)
    val = round_to_dtype(r_val.normal(0.0, sigma, size=nnz).astype(np.float32), dtype)
    if shuffle:
        row, col, val = _shuffle(r_perm, row, col, val)
    return row, col, val


def zipf_rows_coo(M: int, K: int, alpha: float, mean: float, seed: int, dtype: str = "f32",
                  values: str = "inv_deg", kmax: int | None = None, shuffle: bool = True):
    """Row occupancies iid bounded Zipf, columns iid uniform with duplicates inside a
    row removed; values 1/occ_row ('inv_deg') or N(0,1) ('normal')."""
    r_pos, r_val, _, r_perm = _streams(seed)
    if kmax is None:
        kmax = bounded_zipf_kmax(alpha, mean)
    kmax = min(kmax, K)
    occ = bounded_zipf_sample(r_pos, alpha, kmax, M)
    row = np.repeat(np.arange(M, dtype=np.int64), occ)
    col = r_pos.integers(0, K, size=row.shape[0], dtype=np.int64)
    key = np.unique(row * K + col)
    row = (key // K).astype(np.int32)
    col = (key % K).astype(np.int32)
    occ2 = np.bincount(row, minlength=M)
    if values == "inv_deg":
        val = (1.0 / occ2[row]).astype(np.float32)
    else:
        val = r_val.normal(0.0, 1.0, size=row.shape[0]).astype(np.float32)
    val = round_to_dtype(val, dtype)
    if shuffle:
        row, col, val = _shuffle(r_perm, row, col, val)
    return row, col, val


def _expand_blocks(brow, bcol, bM, bK, r_val, sigma, dtype):
    nb = brow.shape[0]
    rr = (brow[:, None, None].astype(np.int64) * bM + np.arange(bM)[None, :, None])
    cc = (bcol[:, None, None].astype(np.int64) * bK + np.arange(bK)[None, None, :])
    row = np.broadcast_to(rr, (nb, bM, bK)).reshape(-1).astype(np.int32)
    col = np.broadcast_to(cc, (nb, bM, bK)).reshape(-1).astype(np.int32)
    val = round_to_dtype(r_val.normal(0.0, sigma, size=row.shape[0]).astype(np.float32), dtype)
    return row, col, val


def random_block_coo(M: int, K: int, bM: int, bK: int, seed: int, dtype: str = "bf16",
                     block_density: float | None = None, zipf_alpha: float | None = None,
                     zipf_mean: float | None = None, sigma: float = 0.02,
                     fill: float = 1.0, shuffle: bool = True):
    """Block-sparse matrix as element COO.  Nonzero blocks are either chosen uniformly
    (``block_density``) or per block-row with bounded-Zipf counts (``zipf_alpha``,
    ``zipf_mean``).  ``fill`` < 1 keeps only that fraction of each block's elements
    (tests only; the benchmark workloads use dense blocks)."""
    r_pos, r_val, _, r_perm = _streams(seed)
    nbr, nbc = M // bM, K // bK
    if zipf_alpha is None:
        nblk = int(round(block_density * nbr * nbc))
        flat = r_pos.choice(nbr * nbc, size=nblk, replace=False) if nblk else np.zeros(0, np.int64)
        brow, bcol = flat // nbc, flat % nbc
    else:
        kmax = min(bounded_zipf_kmax(zipf_alpha, zipf_mean), nbc)
        occ = bounded_zipf_sample(r_pos, zipf_alpha, kmax, nbr)
        brow = np.repeat(np.arange(nbr, dtype=np.int64), occ)
        bcol = np.concatenate([r_pos.choice(nbc, size=int(k), replace=False) for k in occ]) \
            if nbr else np.zeros(0, np.int64)
    row, col, val = _expand_blocks(brow, bcol, bM, bK, r_val, sigma, dtype)
    if fill < 1.0 and row.shape[0]:
        keep = r_pos.random(row.shape[0]) < fill
        row, col, val = row[keep], col[keep], val[keep]
    if shuffle:
        row, col, val = _shuffle(r_perm, row, col, val)
    return row, col, val


def voxel_kernel_map(grid: int, density: float, seed: int, kernel: int = 3, dtype: str = "f16",
                     values: str = "ones", shuffle: bool = True):
    """Kernel map of a submanifold sparse convolution on a synthetic point cloud: voxels of a
    grid^3 volume are occupied independently with probability `density`; for every occupied
    voxel x and every offset z of the kernel^3 stencil whose neighbour y is occupied the map
    holds the entry (x, y, z).  Stands in for the voxelised indoor scans of Section 6.4.
    Returns (P, mx, my, mz, mv): number of points and the COO arrays of Map[x, y, z]."""
    r_pos = _streams(seed)[0]
    occ = r_pos.random((grid, grid, grid)) < density
    return _kernel_map_of(occ, seed, kernel, dtype, values, shuffle)


def _morton_order(coords: np.ndarray) -> np.ndarray:
    """Permutation that lists voxel coordinates [P, 3] (each below 2^21) in Z-curve order."""
    def spread(v):   # put two zero bits between the bits of v
        v = v.astype(np.uint64)
        v = (v | (v << np.uint64(32))) & np.uint64(0x1F00000000FFFF)
        v = (v | (v << np.uint64(16))) & np.uint64(0x1F0000FF0000FF)
        v = (v | (v << np.uint64(8))) & np.uint64(0x100F00F00F00F00F)
        v = (v | (v << np.uint64(4))) & np.uint64(0x10C30C30C30C30C3)
        v = (v | (v << np.uint64(2))) & np.uint64(0x1249249249249249)
        return v
    code = spread(coords[:, 0]) | (spread(coords[:, 1]) << np.uint64(1)) | (spread(coords[:, 2]) << np.uint64(2))
    return np.argsort(code, kind="stable")


def surface_kernel_map(grid: int, planes: int, spheres: int, seed: int, kernel: int = 3, dtype: str = "f16",
                       values: str = "ones", shuffle: bool = True, order: str = "morton"):
    """The same for a point cloud that lies on surfaces, as a scanned room does (walls, floor,
    furniture): the occupied voxels of a grid^3 volume are those within half a voxel of one of
    `planes` random planes (the first three axis-aligned) or `spheres` random sphere shells.
    Points are numbered along the Z-curve of their voxels (`order="morton"`, how point-cloud
    libraries commonly sort voxels) or lexicographically (`order="lex"`): with the former,
    consecutive points are neighbours on a surface and mostly see the same stencil offsets
    occupied."""
    rng = _streams(seed)[0]
    ax = np.arange(grid, dtype=np.float32)
    X, Y, Z = np.meshgrid(ax, ax, ax, indexing="ij")
    occ = np.zeros((grid, grid, grid), dtype=bool)
    for i in range(planes):
        if i < 3:
            n = np.zeros(3, dtype=np.float32)
            n[i] = 1.0
        else:
            n = rng.standard_normal(3).astype(np.float32)
            n /= np.linalg.norm(n)
        c = rng.uniform(0.25 * grid, 0.75 * grid, size=3).astype(np.float32)
        occ |= np.abs(n[0] * (X - c[0]) + n[1] * (Y - c[1]) + n[2] * (Z - c[2])) < 0.5
    for _ in range(spheres):
        c = rng.uniform(0.3 * grid, 0.7 * grid, size=3).astype(np.float32)
        r = rng.uniform(0.15 * grid, 0.3 * grid)
        occ |= np.abs(np.sqrt((X - c[0]) ** 2 + (Y - c[1]) ** 2 + (Z - c[2]) ** 2) - r) < 0.5
    return _kernel_map_of(occ, seed, kernel, dtype, values, shuffle, order)


def _kernel_map_of(occ: np.ndarray, seed: int, kernel: int, dtype: str, values: str, shuffle: bool,
                   order: str = "lex"):
    """(P, mx, my, mz, mv) of the kernel^3 stencil over the occupied voxels `occ` [grid]^3."""
    _, r_val, _, r_perm = _streams(seed)
    grid = occ.shape[0]
    coords = np.argwhere(occ).astype(np.int64)                     # [P, 3], lexicographic
    if order == "morton":
        coords = coords[_morton_order(coords)]
    P = coords.shape[0]
    half = kernel // 2
    index = -np.ones((grid + 2 * half,) * 3, dtype=np.int64)       # lookup table with a halo
    index[coords[:, 0] + half, coords[:, 1] + half, coords[:, 2] + half] = np.arange(P)
    xs, ys, zs = [], [], []
    z = 0
    for dx in range(-half, half + 1):
        for dy in range(-half, half + 1):
            for dz in range(-half, half + 1):
                nb = index[coords[:, 0] + half + dx, coords[:, 1] + half + dy, coords[:, 2] + half + dz]
                hit = nb >= 0
                xs.append(np.flatnonzero(hit))
                ys.append(nb[hit])
                zs.append(np.full(int(hit.sum()), z))
                z += 1
    mx = np.concatenate(xs).astype(np.int32)
    my = np.concatenate(ys).astype(np.int32)
    mz = np.concatenate(zs).astype(np.int32)
    if values == "ones":
        mv = np.ones(mx.shape[0], dtype=np.float32)
    else:
        mv = r_val.normal(0.0, 1.0, size=mx.shape[0]).astype(np.float32)
    mv = round_to_dtype(mv, dtype)
    if shuffle:
        perm = r_perm.permutation(mx.shape[0])
        mx, my, mz, mv = mx[perm], my[perm], mz[perm], mv[perm]
    return P, mx, my, mz, mv


def dense_operand(K: int, N: int, seed: int, dtype: str) -> np.ndarray:
    rng = _streams(seed)[2]
    return round_to_dtype(rng.standard_normal((K, N), dtype=np.float32), dtype)


# --------------------------------------------------------------------------- #
# the five benchmark workloads
# --------------------------------------------------------------------------- #
def make_config(name: str, seed: int = 0, shuffle: bool = True) -> dict:
    """Build one of the five workloads.  Keys: kind ('group'|'block'), M, K, N, row,
    col, val, a_dtype, B, b_dtype, c_dtype, and bM/bK for block workloads."""
    if name == "cfg1":   # 512x512 fp32, 1% density, N=64
        M = K = 512
        N = 64
        nnz = int(round(0.01 * M * K))
        row, col, val = random_coo(M, K, nnz, seed, "f32", 1.0, shuffle)
        cfg = dict(kind="group", M=M, K=K, N=N, a_dtype="f32", b_dtype="f32", c_dtype="f32")
    elif name == "cfg2":  # weight-sparsity shape: 4096^2 fp16, 90% sparse, N=256
        M = K = 4096
        N = 256
        nnz = int(round(0.10 * M * K))
        row, col, val = random_coo(M, K, nnz, seed, "f16", 0.02, shuffle)
        cfg = dict(kind="group", M=M, K=K, N=N, a_dtype="f16", b_dtype="f16", c_dtype="f16")
    elif name in ("cfg3", "cfg3_f16"):  # graph aggregation shape: 2^20 rows, Zipf(1.2) degrees, mean 16, N=128
        M = K = 1 << 20
        N = 128
        dt = "f32" if name == "cfg3" else "f16"    # the paper reports this experiment in both precisions
        row, col, val = zipf_rows_coo(M, K, 1.2, 16.0, seed, dt, "inv_deg", None, shuffle)
        cfg = dict(kind="group", M=M, K=K, N=N, a_dtype=dt, b_dtype=dt, c_dtype=dt)
    elif name == "cfg3_wide":
        # cfg3's generator with four times as many columns: B is 2 GiB, of which the 256 MB
        # Infinity Cache can hold an eighth, so the gathers have to come from HBM itself.
        M, K, N = 1 << 20, 1 << 22, 128
        row, col, val = zipf_rows_coo(M, K, 1.2, 16.0, seed, "f32", "inv_deg", None, shuffle)
        cfg = dict(kind="group", M=M, K=K, N=N, a_dtype="f32", b_dtype="f32", c_dtype="f32")
    elif name == "cfg4":  # 8192^2 bf16, 32x32 blocks, 10% of blocks, N=512
        M = K = 8192
        N = 512
        row, col, val = random_block_coo(M, K, 32, 32, seed, "bf16", block_density=0.10,
                                         sigma=0.02, shuffle=shuffle)
        cfg = dict(kind="block", M=M, K=K, N=N, bM=32, bK=32,
                   a_dtype="bf16", b_dtype="bf16", c_dtype="bf16")
    elif name == "cfg5":  # 32768^2 bf16, 64x64 blocks, Zipf(1.0) blocks per block-row, 2%, N=1024
        M = K = 32768
        N = 1024
        row, col, val = random_block_coo(M, K, 64, 64, seed, "bf16", zipf_alpha=1.0,
                                         zipf_mean=0.02 * (K // 64), sigma=0.02, shuffle=shuffle)
        cfg = dict(kind="block", M=M, K=K, N=N, bM=64, bK=64,
                   a_dtype="bf16", b_dtype="bf16", c_dtype="bf16")
    else:
        raise ValueError(f"unknown config {name!r}")
    cfg.update(name=name, row=row, col=col, val=val, seed=seed,
               B=dense_operand(cfg["K"], cfg["N"], seed, cfg["b_dtype"]))
    return cfg
