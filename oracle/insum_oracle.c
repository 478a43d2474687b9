/*
 * CPU oracle for the Insum SpMM hot path.  TEST INFRASTRUCTURE ONLY: nothing in the
 * product (the HIP library and its Python binding) may include, link or call this file.
 *
 * Everything here is the plain definition from the paper, written as loops:
 *   - indirect-Einsum semantics (output starts at zero, colliding writes are summed):
 *     Section 3.1 "Extending Einsums with Indirect Indexing";
 *   - GroupCOO and BlockGroupCOO (fixed-length groups along rows / block rows, the row
 *     coordinate stored once per group, padding inside the last group of a row):
 *     Section 4.1 "Grouping", the GroupCOO equation and the BlockCOO / BlockGroupCOO
 *     figure captions;
 *   - the indirect-access count F(g), its relaxation and g* = sqrt(S/n):
 *     Section 4.2 "Choosing Group Size";
 *   - SpMM: the GroupCOO and BlockGroupCOO Einsums of Section 4.1, one update of the output
 *     per stored slot; the product with the transposed matrix over the same format (the
 *     derivative of the SpMM with respect to its dense operand, cf. Section 5.1);
 *   - point-cloud sparse convolution as an indirect Einsum grouped by kernel offset:
 *     Section 6.4 "Case Study: Point Cloud Sparse Convolution".
 *
 * Where the paper is silent the oracle takes these readings (listed again in the
 * design notes): entries are ordered by (row, column, input position); padding slots
 * hold value +0 and repeat the column of the last real entry of their group; rows
 * without entries produce no group; duplicate coordinates stay separate entries in
 * GroupCOO and are an error in BlockGroupCOO; the default group size is the power of
 * two nearest to g* in log2.
 *
 * Floating point: SpMM accumulates in fp64.  Inputs arrive as fp32 arrays that hold the
 * (already rounded) fp32 / fp16 / bf16 values exactly.  Format conversion moves bytes
 * and does no arithmetic on values.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------------------ */
/* canonical order                                                                       */
/* ------------------------------------------------------------------------------------ */
typedef struct {
    int64_t key_hi; /* row (or block row)            */
    int64_t key_lo; /* column (or block column, ...) */
    int64_t pos;    /* input position: final tie-break */
} sort_item;

static int cmp_item(const void* a, const void* b) {
    const sort_item* x = (const sort_item*)a;
    const sort_item* y = (const sort_item*)b;
    if (x->key_hi != y->key_hi) return x->key_hi < y->key_hi ? -1 : 1;
    if (x->key_lo != y->key_lo) return x->key_lo < y->key_lo ? -1 : 1;
    if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
    return 0;
}

/* perm[i] = input position of the i-th entry in (row, col, position) order.
 * Returns 0, or 2 if a coordinate is outside [0,M) x [0,K). */
int oracle_canonical_order(int64_t M, int64_t K, int64_t nnz, const int32_t* row,
                           const int32_t* col, int64_t* perm) {
    sort_item* it = (sort_item*)malloc(sizeof(sort_item) * (size_t)(nnz > 0 ? nnz : 1));
    for (int64_t i = 0; i < nnz; ++i) {
        if (row[i] < 0 || row[i] >= M || col[i] < 0 || col[i] >= K) {
            free(it);
            return 2;
        }
        it[i].key_hi = row[i];
        it[i].key_lo = col[i];
        it[i].pos = i;
    }
    qsort(it, (size_t)nnz, sizeof(sort_item), cmp_item);
    for (int64_t i = 0; i < nnz; ++i) perm[i] = it[i].pos;
    free(it);
    return 0;
}

/* ------------------------------------------------------------------------------------ */
/* group size (Section 4.2)                                                               */
/* ------------------------------------------------------------------------------------ */

/* F(g) = (g + 1) * sum_i ceil(occ_i / g): scatters through AM plus gathers through AK. */
int64_t oracle_indirect_access_cost(int64_t n, const int64_t* occ, int64_t g) {
    int64_t groups = 0;
    for (int64_t i = 0; i < n; ++i) groups += (occ[i] + g - 1) / g;
    return (g + 1) * groups;
}

/* Relaxed cost with ceil(x) ~ x + 1:  S + S/g + n*g + n. */
double oracle_relaxed_cost(double S, double n, double g) { return S + S / g + n * g + n; }

/* Real-valued minimiser of the relaxed cost. */
double oracle_gstar(double S, double n) { return sqrt(S / n); }

/* Power of two nearest to g* in log2:  g = 2^e with e = round(log2(S/n) / 2), i.e. the
 * e >= 0 with  n * 2^(2e-1) <= S < n * 2^(2e+1)  (e = 0 when S < 2n).  Integers only. */
int64_t oracle_default_group_size(int64_t S, int64_t n) {
    if (S <= 0 || n <= 0) return 1;
    int e = 0;
    while (e < 30) {
        /* upper edge of the interval that rounds to e */
        __int128 hi = (__int128)n << (2 * e + 1);
        if ((__int128)S < hi) break;
        ++e;
    }
    return (int64_t)1 << e;
}

/* The two powers of two that enclose g* = sqrt(S/n) (Section 4.2: g* is rounded "to the nearest
 * power-of-two values", plural, and the better of them is kept):  lo = 2^a with a the largest
 * integer such that 4^a * n <= S (at least 1), hi = lo when g* is exactly lo, else 2 * lo. */
void oracle_enclosing_powers_of_two(int64_t S, int64_t n, int64_t* lo, int64_t* hi) {
    *lo = 1;
    *hi = 1;
    if (S <= 0 || n <= 0) return;
    int a = 0;
    while (a < 30 && ((__int128)n << (2 * (a + 1))) <= (__int128)S) ++a;
    *lo = (int64_t)1 << a;
    const __int128 at_lo = (__int128)n << (2 * a);
    *hi = (at_lo >= (__int128)S) ? *lo : 2 * *lo;   /* S <= n * lo^2: g* <= lo (g* < 1 clamps to 1) */
}

/* ------------------------------------------------------------------------------------ */
/* COO -> GroupCOO (Section 4.1)                                                          */
/* ------------------------------------------------------------------------------------ */

/* occ[i] = entries in row i; returns G = sum_i ceil(occ_i / g). */
int64_t oracle_groupcoo_num_groups(int64_t M, int64_t nnz, const int32_t* row, int64_t g,
                                   int64_t* occ) {
    for (int64_t i = 0; i < M; ++i) occ[i] = 0;
    for (int64_t e = 0; e < nnz; ++e) occ[row[e]] += 1;
    int64_t G = 0;
    for (int64_t i = 0; i < M; ++i) G += (occ[i] + g - 1) / g;
    return G;
}

/* Fills AM[G], AK[G*g], AV[G*g] (elem_size bytes per value, copied bit for bit).
 * Returns 0 on success, 2 for an out-of-range coordinate. */
int oracle_coo_to_groupcoo(int64_t M, int64_t K, int64_t nnz, const int32_t* row,
                           const int32_t* col, const void* val, int elem_size, int64_t g,
                           int32_t* AM, int32_t* AK, void* AV) {
    int64_t* perm = (int64_t*)malloc(sizeof(int64_t) * (size_t)(nnz > 0 ? nnz : 1));
    int rc = oracle_canonical_order(M, K, nnz, row, col, perm);
    if (rc) {
        free(perm);
        return rc;
    }
    const char* vin = (const char*)val;
    char* vout = (char*)AV;
    int64_t p = 0; /* next group to emit */
    int64_t e = 0; /* next sorted entry  */
    while (e < nnz) {
        const int32_t i = row[perm[e]];
        int64_t end = e;
        while (end < nnz && row[perm[end]] == i) ++end; /* entries e..end-1 form row i */
        while (e < end) {
            /* one group: up to g entries of row i, then padding */
            AM[p] = i;
            int32_t last_col = 0;
            for (int64_t q = 0; q < g; ++q) {
                if (e < end) {
                    last_col = col[perm[e]];
                    AK[p * g + q] = last_col;
                    memcpy(vout + (size_t)(p * g + q) * elem_size,
                           vin + (size_t)perm[e] * elem_size, (size_t)elem_size);
                    ++e;
                } else {
                    AK[p * g + q] = last_col;                                   /* padding */
                    memset(vout + (size_t)(p * g + q) * elem_size, 0, (size_t)elem_size); /* +0 */
                }
            }
            ++p;
        }
    }
    free(perm);
    return 0;
}

/* ------------------------------------------------------------------------------------ */
/* COO -> BlockGroupCOO (Section 4.1, "Group+Blocking")                                   */
/* ------------------------------------------------------------------------------------ */

/* Sorted list of distinct nonzero blocks.  Returns 0, 2 (coordinate out of range),
 * 3 (duplicate coordinate) or 5 (M or K not a multiple of the block shape).
 * blk_row / blk_col must hold nnz entries; *num_blocks receives the count;
 * occ[M/bM] receives the blocks per block row. */
int oracle_nonzero_blocks(int64_t M, int64_t K, int64_t nnz, const int32_t* row,
                          const int32_t* col, int64_t bM, int64_t bK, int64_t* num_blocks,
                          int32_t* blk_row, int32_t* blk_col, int64_t* occ) {
    if (bM <= 0 || bK <= 0 || M % bM || K % bK) return 5;
    int64_t* perm = (int64_t*)malloc(sizeof(int64_t) * (size_t)(nnz > 0 ? nnz : 1));
    int rc = oracle_canonical_order(M, K, nnz, row, col, perm);
    if (rc) {
        free(perm);
        return rc;
    }
    for (int64_t e = 1; e < nnz; ++e)
        if (row[perm[e]] == row[perm[e - 1]] && col[perm[e]] == col[perm[e - 1]]) {
            free(perm);
            return 3;
        }
    /* collect (block row, block col) of every entry, sort, keep distinct ones */
    sort_item* it = (sort_item*)malloc(sizeof(sort_item) * (size_t)(nnz > 0 ? nnz : 1));
    for (int64_t e = 0; e < nnz; ++e) {
        it[e].key_hi = row[e] / bM;
        it[e].key_lo = col[e] / bK;
        it[e].pos = 0;
    }
    qsort(it, (size_t)nnz, sizeof(sort_item), cmp_item);
    int64_t nb = 0;
    for (int64_t i = 0; i < M / bM; ++i) occ[i] = 0;
    for (int64_t e = 0; e < nnz; ++e) {
        if (e == 0 || it[e].key_hi != it[e - 1].key_hi || it[e].key_lo != it[e - 1].key_lo) {
            blk_row[nb] = (int32_t)it[e].key_hi;
            blk_col[nb] = (int32_t)it[e].key_lo;
            occ[it[e].key_hi] += 1;
            ++nb;
        }
    }
    *num_blocks = nb;
    free(it);
    free(perm);
    return 0;
}

/* Fills AM[G], AK[G*g], AV[G*g*bM*bK] from the block list produced above (blocks sorted
 * by (block row, block col)).  AV is zero-filled first; every input entry is then copied
 * to its place inside its block. */
int oracle_coo_to_blockgroupcoo(int64_t M, int64_t K, int64_t nnz, const int32_t* row,
                                const int32_t* col, const void* val, int elem_size, int64_t bM,
                                int64_t bK, int64_t g, int64_t num_blocks,
                                const int32_t* blk_row, const int32_t* blk_col, int64_t G,
                                int32_t* AM, int32_t* AK, void* AV) {
    (void)M;
    const int64_t nbc = K / bK;
    const int64_t nbr = M / bM;
    char* vout = (char*)AV;
    const char* vin = (const char*)val;
    memset(vout, 0, (size_t)(G * g * bM * bK) * elem_size);
    /* slot_of[block row * nbc + block col] = flat slot p*g+q of that block, or -1 */
    int64_t* slot_of = (int64_t*)malloc(sizeof(int64_t) * (size_t)(nbr * nbc > 0 ? nbr * nbc : 1));
    for (int64_t i = 0; i < nbr * nbc; ++i) slot_of[i] = -1;
    int64_t p = 0, b = 0;
    while (b < num_blocks) {
        const int32_t i = blk_row[b];
        int64_t end = b;
        while (end < num_blocks && blk_row[end] == i) ++end;
        while (b < end) {
            AM[p] = i;
            int32_t last_col = 0;
            for (int64_t q = 0; q < g; ++q) {
                if (b < end) {
                    last_col = blk_col[b];
                    slot_of[(int64_t)i * nbc + last_col] = p * g + q;
                    ++b;
                }
                AK[p * g + q] = last_col; /* real block column, or repeated for padding */
            }
            ++p;
        }
    }
    if (p != G) {
        free(slot_of);
        return 4;
    }
    for (int64_t e = 0; e < nnz; ++e) {
        const int64_t s = slot_of[(int64_t)(row[e] / bM) * nbc + col[e] / bK];
        const int64_t off = ((s * bM + row[e] % bM) * bK + col[e] % bK);
        memcpy(vout + (size_t)off * elem_size, vin + (size_t)e * elem_size, (size_t)elem_size);
    }
    free(slot_of);
    return 0;
}

/* ------------------------------------------------------------------------------------ */
/* SpMM (fp64 accumulate)                                                                 */
/* ------------------------------------------------------------------------------------ */

static void column_slice(int64_t N, int64_t* n0, int64_t* n1) {
#ifdef _OPENMP
    const int t = omp_get_thread_num(), T = omp_get_num_threads();
#else
    const int t = 0, T = 1;
#endif
    *n0 = N * t / T;
    *n1 = N * (t + 1) / T;
}

/* The GroupCOO Einsum of Section 4.1,  C[AM[p], n] += AV[p,q] * B[AK[p,q], n],  taken as it
 * stands: one update of C per stored slot (p, q) and column n, slots in storage order.
 * C is not cleared here: the caller passes zeros (plain Einsum) or the matrix to
 * accumulate into.  Threads own disjoint column ranges, so there are no races and
 * the summation order per output element is fixed. */
void oracle_spmm_groupcoo(int64_t M, int64_t K, int64_t N, int64_t G, int64_t g,
                          const int32_t* AM, const int32_t* AK, const float* AV,
                          const float* B, int64_t ldb, double* C, int64_t ldc) {
    (void)M;
    (void)K;
#pragma omp parallel
    {
        int64_t n0, n1;
        column_slice(N, &n0, &n1);
        for (int64_t slot = 0; slot < G * g; ++slot) {
            const double a = (double)AV[slot];
            const float* brow = B + (int64_t)AK[slot] * ldb;
            double* crow = C + (int64_t)AM[slot / g] * ldc;
            for (int64_t n = n0; n < n1; ++n) crow[n] += a * (double)brow[n];
        }
    }
}

/* The same Einsum with the roles of the dense operands exchanged - the product with the
 * transposed matrix over the same stored format, which is what differentiating the SpMM with
 * respect to B gives (Section 5.1 names autodiff as a use of the Einsum form):
 *     D[AK[p,q], n] += AV[p,q] * E[AM[p], n]        (D = A^T * E;  E is M x N, D is K x N)
 * Slots in storage order, one update each.  D is not cleared here. */
void oracle_spmm_groupcoo_transposed(int64_t M, int64_t K, int64_t N, int64_t G, int64_t g,
                                     const int32_t* AM, const int32_t* AK, const float* AV,
                                     const float* E, int64_t lde, double* D, int64_t ldd) {
    (void)M;
    (void)K;
#pragma omp parallel
    {
        int64_t n0, n1;
        column_slice(N, &n0, &n1);
        for (int64_t slot = 0; slot < G * g; ++slot) {
            const double a = (double)AV[slot];
            const float* erow = E + (int64_t)AM[slot / g] * lde;
            double* drow = D + (int64_t)AK[slot] * ldd;
            for (int64_t n = n0; n < n1; ++n) drow[n] += a * (double)erow[n];
        }
    }
}

/* C[AM[p]*bM + bm, n] += sum_{q,bk} AV[p,q,bm,bk] * B[AK[p,q]*bK + bk, n]. */
void oracle_spmm_blockgroupcoo(int64_t M, int64_t K, int64_t N, int64_t G, int64_t g,
                               int64_t bM, int64_t bK, const int32_t* AM, const int32_t* AK,
                               const float* AV, const float* B, int64_t ldb, double* C,
                               int64_t ldc) {
    (void)M;
    (void)K;
#pragma omp parallel
    {
        int64_t n0, n1;
        column_slice(N, &n0, &n1);
        for (int64_t p = 0; p < G; ++p)
            for (int64_t q = 0; q < g; ++q)
                for (int64_t bm = 0; bm < bM; ++bm)
                    for (int64_t bk = 0; bk < bK; ++bk) {
                        const double a = (double)AV[((p * g + q) * bM + bm) * bK + bk];
                        const float* brow = B + ((int64_t)AK[p * g + q] * bK + bk) * ldb;
                        double* crow = C + ((int64_t)AM[p] * bM + bm) * ldc;
                        for (int64_t n = n0; n < n1; ++n) crow[n] += a * (double)brow[n];
                    }
    }
}

/* ------------------------------------------------------------------------------------ */
/* Point-cloud sparse convolution (Section 6.4)                                           */
/*   Out[MAPX[p,q], m] += MAPV[p,q] * sum_c In[MAPY[p,q], c] * W[MAPZ[p], c, m]           */
/* The map is a 3-D sparse tensor Map[x, y, z] stored as COO and grouped along z (the     */
/* kernel offset): every group holds g (x, y, value) triples of one offset.               */
/* ------------------------------------------------------------------------------------ */

/* perm[i] = input position of the i-th entry in (z, x, position) order.  Returns 0, or 2
 * when a coordinate is out of range. */
int oracle_map_order(int64_t X, int64_t Y, int64_t Z, int64_t nnz, const int32_t* mx,
                     const int32_t* my, const int32_t* mz, int64_t* perm) {
    sort_item* it = (sort_item*)malloc(sizeof(sort_item) * (size_t)(nnz > 0 ? nnz : 1));
    for (int64_t i = 0; i < nnz; ++i) {
        if (mx[i] < 0 || mx[i] >= X || my[i] < 0 || my[i] >= Y || mz[i] < 0 || mz[i] >= Z) {
            free(it);
            return 2;
        }
        it[i].key_hi = mz[i];
        it[i].key_lo = mx[i];
        it[i].pos = i;
    }
    qsort(it, (size_t)nnz, sizeof(sort_item), cmp_item);
    for (int64_t i = 0; i < nnz; ++i) perm[i] = it[i].pos;
    free(it);
    return 0;
}

/* occ[z] = entries with offset z; returns G = sum_z ceil(occ_z / g). */
int64_t oracle_map_num_groups(int64_t Z, int64_t nnz, const int32_t* mz, int64_t g, int64_t* occ) {
    for (int64_t z = 0; z < Z; ++z) occ[z] = 0;
    for (int64_t e = 0; e < nnz; ++e) occ[mz[e]] += 1;
    int64_t G = 0;
    for (int64_t z = 0; z < Z; ++z) G += (occ[z] + g - 1) / g;
    return G;
}

/* Fills MAPZ[G], MAPX[G*g], MAPY[G*g], MAPV[G*g].  Padding slots (tail of the last group
 * of an offset) hold value +0 and repeat the x and y of the last real entry of the group. */
int oracle_map_to_groupcoo(int64_t X, int64_t Y, int64_t Z, int64_t nnz, const int32_t* mx,
                           const int32_t* my, const int32_t* mz, const void* mv, int elem_size,
                           int64_t g, int32_t* MAPZ, int32_t* MAPX, int32_t* MAPY, void* MAPV) {
    int64_t* perm = (int64_t*)malloc(sizeof(int64_t) * (size_t)(nnz > 0 ? nnz : 1));
    int rc = oracle_map_order(X, Y, Z, nnz, mx, my, mz, perm);
    if (rc) {
        free(perm);
        return rc;
    }
    const char* vin = (const char*)mv;
    char* vout = (char*)MAPV;
    int64_t p = 0, e = 0;
    while (e < nnz) {
        const int32_t z = mz[perm[e]];
        int64_t end = e;
        while (end < nnz && mz[perm[end]] == z) ++end;
        while (e < end) {
            MAPZ[p] = z;
            int32_t last_x = 0, last_y = 0;
            for (int64_t q = 0; q < g; ++q) {
                if (e < end) {
                    last_x = mx[perm[e]];
                    last_y = my[perm[e]];
                    memcpy(vout + (size_t)(p * g + q) * elem_size, vin + (size_t)perm[e] * elem_size,
                           (size_t)elem_size);
                    ++e;
                } else {
                    memset(vout + (size_t)(p * g + q) * elem_size, 0, (size_t)elem_size);
                }
                MAPX[p * g + q] = last_x;
                MAPY[p * g + q] = last_y;
            }
            ++p;
        }
    }
    free(perm);
    return 0;
}

/* Out[MAPX[p,q], m] += MAPV[p,q] * sum_c In[MAPY[p,q], c] * W[MAPZ[p], c, m]  in fp64.
 * Out is not cleared here.  Threads own disjoint ranges of m. */
void oracle_spconv_groupcoo(int64_t C, int64_t M, int64_t G, int64_t g, const int32_t* MAPZ,
                            const int32_t* MAPX, const int32_t* MAPY, const float* MAPV,
                            const float* In, int64_t ld_in, const float* W, double* Out,
                            int64_t ld_out) {
#pragma omp parallel
    {
        int64_t m0, m1;
        column_slice(M, &m0, &m1);
        for (int64_t p = 0; p < G; ++p)
            for (int64_t q = 0; q < g; ++q) {
                const double v = (double)MAPV[p * g + q];
                const float* in = In + (int64_t)MAPY[p * g + q] * ld_in;
                const float* w = W + (int64_t)MAPZ[p] * C * M;
                double* out = Out + (int64_t)MAPX[p * g + q] * ld_out;
                for (int64_t m = m0; m < m1; ++m) {
                    double acc = 0.0;
                    for (int64_t c = 0; c < C; ++c) acc += (double)in[c] * (double)w[c * M + m];
                    out[m] += v * acc;
                }
            }
    }
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
