/*
 * insum.h - C ABI of the MI355X (gfx950) library for sparse x dense matrix multiply
 * written as an indirect Einsum over fixed-length sparse formats.
 *
 *     GroupCOO       C[AM[p], n]          += AV[p,q]       * B[AK[p,q], n]
 *     BlockGroupCOO  C[AM[p]*bM + bm, n]  += AV[p,q,bm,bk] * B[AK[p,q]*bK + bk, n]
 *
 * (paper: Section 3.1 for the Einsum semantics, Section 4.1 for both formats and both
 * Einsums, Section 4.2 for the group size, Section 6.5 for the GroupCOO SpMM loop.)
 *
 * Conventions that hold for every call unless a comment says otherwise
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory.  The library never frees anything and keeps no state
 *     between calls.
 *   - All matrices are row-major.  B is K x N with leading dimension ldb (elements),
 *     C is M x N with leading dimension ldc.  Indices are int32; M, K, N, nnz < 2^31.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued on it; SpMM calls never synchronise, conversion calls synchronise the
 *     stream (they return counts to the host).
 *   - Every function returns an insum_status and never throws or aborts.  After a
 *     non-OK status the output buffers hold unspecified data.
 */
#ifndef INSUM_H
#define INSUM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    INSUM_OK = 0,
    INSUM_ERR_INVALID_ARG = 1,  /* null pointer, negative size, bad enum, misaligned    */
    INSUM_ERR_OUT_OF_RANGE = 2, /* a coordinate lies outside [0,M) x [0,K)              */
    INSUM_ERR_DUPLICATE = 3,    /* block conversion: the same (row, col) appears twice  */
    INSUM_ERR_CAPACITY = 4,     /* an output or workspace buffer is too small           */
    INSUM_ERR_UNSUPPORTED = 5,  /* dtype or shape combination that is not implemented   */
    INSUM_ERR_HIP = 6           /* a HIP runtime call failed                            */
} insum_status;

typedef enum { INSUM_F32 = 0, INSUM_F16 = 1, INSUM_BF16 = 2 } insum_dtype;

/* Library version (major*10000 + minor*100 + patch) and a static description of a
 * status code.  Host only. */
int insum_version(void);
const char* insum_status_string(int status);

/* ---------------------------------------------------------------------------------- */
/* Group size (Section 4.2)                                                            */
/* ---------------------------------------------------------------------------------- */

/* Default group size: the power of two nearest (in log2) to g* = sqrt(S / n), where S
 * is the number of stored entries (blocks for the block format) and n the number of
 * rows (block rows), empty ones included.  Host only, integer arithmetic.  Returns 1
 * when S <= 0 or n <= 0. */
int32_t insum_default_group_size(int64_t S, int64_t n);

/* F(g) = (g + 1) * sum_i ceil(occ_i / g): the number of indirect accesses (one scatter
 * per group through AM, g gathers per group through AK).  `occ` is a host array of n
 * row occupancies.  Returns -1 for invalid arguments and when F(g) does not fit 64 bits. */
int64_t insum_indirect_access_cost(int64_t n, const int64_t* occ, int32_t g);

/* The group sizes Section 4.2 considers for a matrix with S stored entries in n rows: the
 * default above and its two power-of-two neighbours (so both powers of two that enclose g* are
 * among them), ascending, at most three, written to out3.  Returns their number.  Host only. */
int32_t insum_group_size_candidates(int64_t S, int64_t n, int32_t* out3);

/* Bytes of device workspace insum_choose_group_size needs.  Host only. */
size_t insum_choose_group_size_workspace_bytes(int64_t M, int64_t N, int64_t nnz, insum_dtype dt);

/*
 * Group size by measurement (Section 4.2, last paragraph: the powers of two next to g* are
 * tried and the fastest is kept).  For every candidate of
 * insum_group_size_candidates(nnz, M) the COO matrix is converted to GroupCOO and
 * insum_spmm_groupcoo is run on the caller's operands: one untimed launch, then `repeats`
 * launches between two HIP events on `stream`.
 *
 *   row, col, val, dt   device; the matrix, as for insum_coo_to_groupcoo
 *   B, ldb              device dt[K, ldb]; C, ldc, c_dt: device output, overwritten (C = A*B)
 *   best_g              host out: the candidate with the smallest time per launch (the smaller
 *                       one on a tie); the default group size when there is nothing to time
 *   candidates, candidate_ms, num_candidates   host out, optional (NULL): what was tried and
 *                       the milliseconds per launch of each (3 entries each)
 *   workspace           device, at least insum_choose_group_size_workspace_bytes(...) bytes
 *
 * Synchronises the stream several times.  The formats it builds live in the workspace only:
 * convert again with the chosen g.
 */
insum_status insum_choose_group_size(int64_t M, int64_t K, int64_t N, int64_t nnz,
                                     const int32_t* row, const int32_t* col, const void* val,
                                     insum_dtype dt, const void* B, int64_t ldb,
                                     void* C, int64_t ldc, insum_dtype c_dt, int32_t repeats,
                                     int32_t* best_g, int32_t* candidates, float* candidate_ms,
                                     int32_t* num_candidates,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------- */
/* COO -> GroupCOO (Section 4.1, "Grouping")                                           */
/* ---------------------------------------------------------------------------------- */

/* Bytes of device workspace the conversion below needs for a matrix with M rows and nnz
 * entries.  Host only. */
size_t insum_coo_to_groupcoo_workspace_bytes(int64_t M, int64_t nnz);

/*
 * Converts an element-wise COO matrix into GroupCOO with group size g.
 *
 *   row, col  device int32[nnz]   coordinates, any order, duplicates allowed (they stay
 *                                 separate entries)
 *   val       device dt[nnz]      values; copied bit for bit
 *   g         group size, or 0 for insum_default_group_size(nnz, M)
 *   g_used    host out            the group size that was used
 *   num_groups host out           G = sum over rows of ceil(occ_row / g)
 *   AM        device int32[capacity_groups]      row of each group (non-decreasing)
 *   AK        device int32[capacity_groups * g]  columns, row-major [G, g]
 *   AV        device dt[capacity_groups * g]     values,  row-major [G, g]
 *   workspace device scratch of at least insum_coo_to_groupcoo_workspace_bytes(M, nnz)
 *
 * Layout produced: rows ascending; inside a row entries ascending by (column, input
 * position); a row with occ entries owns ceil(occ/g) consecutive groups; only the last
 * group of a row is padded, and a padding slot has value +0 and repeats the column of
 * the last real entry of its group.  Rows without entries own no group.
 *
 * Count mode: pass AM = AK = AV = NULL (capacity_groups ignored) to obtain g_used and
 * num_groups only.  Fill mode returns INSUM_ERR_CAPACITY, with num_groups set, when
 * capacity_groups < G.  G never exceeds nnz/g + min(M, nnz).
 * The call synchronises `stream` before it returns.
 */
insum_status insum_coo_to_groupcoo(int64_t M, int64_t K, int64_t nnz,
                                   const int32_t* row, const int32_t* col, const void* val,
                                   insum_dtype dt, int32_t g,
                                   int32_t* g_used, int64_t* num_groups,
                                   int32_t* AM, int32_t* AK, void* AV, int64_t capacity_groups,
                                   void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of device workspace insum_groupcoo_transpose needs.  Host only; 0 for invalid sizes. */
size_t insum_groupcoo_transpose_workspace_bytes(int64_t M, int64_t K, int64_t G, int32_t g);

/*
 * GroupCOO of A^T (K rows, M columns) from the GroupCOO of A: a second, column-grouped copy of
 * the matrix, for callers that multiply by A^T many times (the backward pass of a layer whose
 * forward pass is the Section 4.1 SpMM).  insum_spmm_groupcoo on the result computes A^T * E
 * without atomics and in a fixed summation order, several times faster than
 * insum_spmm_groupcoo_transposed on the original arrays.
 *
 *   AM, AK, AV, dt, G, g   device; the format of A as produced by insum_coo_to_groupcoo
 *   g_t        group size of the result, or 0 for insum_default_group_size(entries, K)
 *   g_used, num_groups      host out, as for insum_coo_to_groupcoo
 *   num_entries             host out, optional (NULL): entries found in the format
 *   AM_t, AK_t, AV_t, capacity_groups   device outputs, as for insum_coo_to_groupcoo
 *                           (num_groups never exceeds entries/g_t + min(K, entries), and
 *                           entries <= G * g); all NULL = count mode
 *   workspace  device, at least insum_groupcoo_transpose_workspace_bytes(M, K, G, g) bytes
 *
 * The entries are read off the format in slot order with row and column exchanged and grouped
 * again by the rule of insum_coo_to_groupcoo (so entries with the same coordinates keep their
 * order).  Padding is recognised by the pattern that conversion writes: a slot other than the
 * first of its group whose value bits are all zero and whose column equals that of the slot to
 * its left.  A stored +0 entry that repeats the coordinates of the entry before it has the same
 * pattern and is left out with the padding; no product changes by that.
 * Statuses as for insum_coo_to_groupcoo (INSUM_ERR_OUT_OF_RANGE for an AM outside [0, M) or an
 * AK outside [0, K)); G * g must be below 2^31.  Synchronises `stream`.
 */
insum_status insum_groupcoo_transpose(int64_t M, int64_t K, int64_t G, int32_t g,
                                      const int32_t* AM, const int32_t* AK, const void* AV,
                                      insum_dtype dt, int32_t g_t,
                                      int32_t* g_used, int64_t* num_groups, int64_t* num_entries,
                                      int32_t* AM_t, int32_t* AK_t, void* AV_t,
                                      int64_t capacity_groups,
                                      void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------- */
/* COO -> BlockGroupCOO (Section 4.1, "Group+Blocking")                                */
/* ---------------------------------------------------------------------------------- */

size_t insum_coo_to_blockgroupcoo_workspace_bytes(int64_t M, int64_t K, int64_t nnz,
                                                  int32_t bM, int32_t bK);

/*
 * Converts an element-wise COO matrix into BlockGroupCOO with bM x bK blocks grouped
 * along block rows.  Arguments as above, except:
 *
 *   bM, bK    block shape; M % bM == 0 and K % bK == 0 (else INSUM_ERR_UNSUPPORTED)
 *   g         group size, or 0 for insum_default_group_size(#nonzero blocks, M / bM)
 *   AM        device int32[capacity_groups]        block row of each group
 *   AK        device int32[capacity_groups * g]    block columns [G, g]
 *   AV        device dt[capacity_groups*g*bM*bK]   block values [G, g, bM, bK], bk fastest
 *
 * A block is stored when at least one input entry falls inside it (a zero-valued entry
 * still counts); positions of a stored block without an entry hold +0.  Blocks are
 * ordered by (block row, block column) and grouped like the entries of GroupCOO;
 * padding blocks are all +0 and repeat the last real block column of their group.
 * The same (row, col) given twice is INSUM_ERR_DUPLICATE.
 * Count mode and capacity behaviour as for insum_coo_to_groupcoo.  A count call leaves its
 * sorted entries in the workspace; a fill call with the same arguments (sizes, pointers, dtype,
 * block shape) and the same workspace goes on from them instead of sorting again, so between
 * such a pair neither the workspace nor row / col / val may be modified.  The fill call
 * consumes them: a second fill call sorts afresh.
 */
insum_status insum_coo_to_blockgroupcoo(int64_t M, int64_t K, int64_t nnz,
                                        const int32_t* row, const int32_t* col, const void* val,
                                        insum_dtype dt, int32_t bM, int32_t bK, int32_t g,
                                        int32_t* g_used, int64_t* num_groups,
                                        int32_t* AM, int32_t* AK, void* AV,
                                        int64_t capacity_groups,
                                        void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------- */
/* SpMM over GroupCOO (Section 4.1 equation; loop nest of the Section 6.5 listing)     */
/* ---------------------------------------------------------------------------------- */

/* Bytes of device workspace insum_spmm_groupcoo needs (partial sums of rows whose groups
 * are shared between two wavefront work ranges).  Host only. */
size_t insum_spmm_groupcoo_workspace_bytes(int64_t M, int64_t N, int64_t G, int32_t g);

/*
 * C = A * B (accumulate == 0) or C += A * B (accumulate != 0), A given in GroupCOO.
 *
 *   M, K, N < 2^31, G < 2^40 (else INSUM_ERR_INVALID_ARG).
 *   AM, AK, AV  device; layout as produced by insum_coo_to_groupcoo.  AM must be
 *               non-decreasing, 0 <= AM[p] < M, 0 <= AK[p,q] < K (not checked).
 *   a_dt, b_dt, c_dt  supported: a_dt == b_dt in {F32, F16, BF16}; c_dt == b_dt or F32.
 *               Products and sums are formed in fp32; C is rounded once
 *               (round-to-nearest-even) when c_dt is a 16-bit type.
 *   B           device b_dt[K, ldb];  C  device c_dt[M, ldc];  ldb, ldc >= N.
 *   accumulate  0: every element of C[0:M, 0:N] is written (rows without groups become
 *               zero); 1: existing C is read and added to.
 *   workspace   device scratch, at least insum_spmm_groupcoo_workspace_bytes(...) bytes.
 *
 * B is assumed finite: a slot with value zero contributes nothing.  The result does not
 * depend on run-to-run timing (no floating-point atomics are used).  Asynchronous.
 */
insum_status insum_spmm_groupcoo(int64_t M, int64_t K, int64_t N, int64_t G, int32_t g,
                                 const int32_t* AM, const int32_t* AK, const void* AV,
                                 insum_dtype a_dt,
                                 const void* B, int64_t ldb, insum_dtype b_dt,
                                 void* C, int64_t ldc, insum_dtype c_dt, int accumulate,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * insum_spmm_groupcoo for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (without the workspace), same kernels and same results up to fp32 summation
 * order.  The partial sums of rows shared between work ranges live in a device array of
 * 32 MiB that is part of the library image (every GPU the library runs on holds its copy
 * until the process ends); the call performs no allocation and no free, and does not
 * synchronise.  The work is cut into fewer ranges when the usual number of them would not
 * fit the array; INSUM_ERR_CAPACITY when even one range does not fit (N above 4 194 304).
 * The device that owns `stream` must be the current device.  All calls on one GPU share the
 * array: calls that may overlap on one GPU (different streams, several host threads) race
 * and must be serialised by the caller.
 */
insum_status insum_spmm_groupcoo_noalloc(int64_t M, int64_t K, int64_t N, int64_t G, int32_t g,
                                         const int32_t* AM, const int32_t* AK, const void* AV,
                                         insum_dtype a_dt,
                                         const void* B, int64_t ldb, insum_dtype b_dt,
                                         void* C, int64_t ldc, insum_dtype c_dt, int accumulate,
                                         void* stream);

/* ---------------------------------------------------------------------------------- */
/* Product with the transposed matrix over the same stored GroupCOO format             */
/*     D[AK[p,q], n] += AV[p,q] * E[AM[p], n]          (D = A^T * E)                   */
/* The Section 4.1 Einsum with the dense operands exchanged: the derivative of the     */
/* SpMM with respect to B (Section 5.1 names autodiff as a use of the Einsum form).    */
/* ---------------------------------------------------------------------------------- */

/* Bytes of device workspace the call below needs: K x N fp32 sums when D is a 16-bit type,
 * 0 when D is fp32.  Host only. */
size_t insum_spmm_groupcoo_transposed_workspace_bytes(int64_t K, int64_t N, insum_dtype d_dt);

/*
 * D = A^T * E (accumulate == 0) or D += A^T * E, A (M x K) given in GroupCOO exactly as for
 * insum_spmm_groupcoo - no second, transposed copy of A is needed.
 *
 *   E   device e_dt[M, lde], lde >= N;   D   device d_dt[K, ldd], ldd >= N
 *   a_dt == e_dt in {F32, F16, BF16}; d_dt == e_dt or F32.
 *   workspace   device, at least insum_spmm_groupcoo_transposed_workspace_bytes(...) bytes
 *               (may be NULL when that is 0)
 *
 * A group's row of E is read once for its g slots; the contributions to a row of D are
 * added in memory with hardware fp32 atomic adds (the format has no index by column).  So:
 * products and sums are fp32, the order of the additions varies from run to run (results are
 * reproducible up to fp32 summation order), a 16-bit D is summed in the fp32 workspace and
 * rounded once, and with accumulate == 0 every element of D[0:K, 0:N] is written.  Slots with
 * value zero contribute nothing; E is assumed finite.  Asynchronous.
 */
insum_status insum_spmm_groupcoo_transposed(int64_t M, int64_t K, int64_t N, int64_t G, int32_t g,
                                            const int32_t* AM, const int32_t* AK, const void* AV,
                                            insum_dtype a_dt,
                                            const void* E, int64_t lde, insum_dtype e_dt,
                                            void* D, int64_t ldd, insum_dtype d_dt, int accumulate,
                                            void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------- */
/* SpMM over BlockGroupCOO (Section 4.1, BlockGroupCOO Einsum)                         */
/* ---------------------------------------------------------------------------------- */

/* Bytes of device workspace that hold a work plan (below) for these sizes; 0 for shapes that
 * take no plan.  Host only. */
size_t insum_spmm_blockgroupcoo_workspace_bytes(int64_t M, int64_t N, int64_t G, int32_t g,
                                                int32_t bM, int32_t bK);

/*
 * Optional, once per matrix and dense width N: writes a work plan for insum_spmm_blockgroupcoo
 * into `workspace` (device, at least insum_spmm_blockgroupcoo_workspace_bytes(...) bytes).
 * The plan depends on AM only (which groups belong to which block row): it lists the block rows
 * longest first - the order in which the matrix cores are kept busiest when block rows differ
 * in length, as the fixed-length groups of Section 4.1 allow - and cuts a block row that is
 * much longer than the mean load of a workgroup into chunks that are multiplied by different
 * workgroups and added up in a fixed order.  A plan stays valid for every later SpMM call with
 * the same M, N, G, g, bM, AM pointer and AM contents; it must be rebuilt when AM changes.
 * Asynchronous; returns INSUM_OK without touching the workspace for shapes that take no plan.
 */
insum_status insum_spmm_blockgroupcoo_plan(int64_t M, int64_t K, int64_t N, int64_t G, int32_t g,
                                           int32_t bM, int32_t bK, const int32_t* AM,
                                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * C = A * B or C += A * B with A in BlockGroupCOO (layout as produced by
 * insum_coo_to_blockgroupcoo; M % bM == 0, K % bK == 0).
 *
 *   a_dt == b_dt in {F32, F16, BF16}; c_dt == b_dt or F32.  Products are exact, sums are
 *   formed in fp32 on the matrix cores (MFMA) when bM is 32, 64 or 128, bK is a multiple
 *   of 32, N and ldb are multiples of 8, ldc is a multiple of 8 (4 for fp32 C) and B, AV, C
 *   are 16-byte aligned; other shapes, and a_dt == b_dt == F32, run on a slower general
 *   kernel with the same results up to summation order.
 *   Among the real slots of a block row the block columns must be strictly increasing (as
 *   insum_coo_to_blockgroupcoo produces them): a slot that repeats the block column of the
 *   slot before it in its group is taken to be padding and is skipped whatever its values.
 *   B is assumed finite.
 *   workspace   NULL (workspace_bytes 0), or device memory of at least
 *               insum_spmm_blockgroupcoo_workspace_bytes(...) bytes.  When it holds a plan made
 *               by insum_spmm_blockgroupcoo_plan for the same M, N, G, g, bM and AM pointer the
 *               call follows it (and uses the rest of the workspace for the partial tiles of
 *               split block rows: calls that share a workspace must not overlap); contents
 *               that are not such a plan are ignored and block rows are processed whole, in
 *               index order.  Results with and without a plan agree up to fp32 summation
 *               order, and each is reproducible from run to run.
 *
 * Other arguments and behaviour as for insum_spmm_groupcoo.  Asynchronous.
 */
insum_status insum_spmm_blockgroupcoo(int64_t M, int64_t K, int64_t N, int64_t G, int32_t g,
                                      int32_t bM, int32_t bK,
                                      const int32_t* AM, const int32_t* AK, const void* AV,
                                      insum_dtype a_dt,
                                      const void* B, int64_t ldb, insum_dtype b_dt,
                                      void* C, int64_t ldc, insum_dtype c_dt, int accumulate,
                                      void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------- */
/* Point-cloud sparse convolution (Section 6.4)                                        */
/*   Out[MAPX[p,q], m] += MAPV[p,q] * In[MAPY[p,q], c] * Weight[MAPZ[p], c, m]         */
/* The kernel map Map[x, y, z] (output point x receives input point y through kernel   */
/* offset z) is a 3-D sparse tensor in COO, grouped along z with group size g.         */
/* ---------------------------------------------------------------------------------- */

size_t insum_map_to_groupcoo_workspace_bytes(int64_t Z, int64_t nnz);

/*
 * Groups a kernel map along its offset dimension.
 *
 *   mx, my, mz  device int32[nnz]  coordinates: 0 <= mx < X, 0 <= my < Y, 0 <= mz < Z, any
 *                                  order, repeated triples stay separate entries
 *   mv          device dt[nnz]     values (1 for a plain convolution); copied bit for bit
 *   g           group size, or 0 for insum_default_group_size(nnz, Z)
 *   MAPZ        device int32[capacity_groups]      offset of each group (non-decreasing)
 *   MAPX, MAPY  device int32[capacity_groups * g]  output / input point of each slot, [G, g]
 *   MAPV        device dt[capacity_groups * g]     values, [G, g]
 *   workspace   device scratch, at least insum_map_to_groupcoo_workspace_bytes(Z, nnz)
 *
 * Layout produced: offsets ascending; inside an offset entries ascending by (x, input
 * position); an offset with occ entries owns ceil(occ/g) consecutive groups; a padding slot
 * (tail of the last group of an offset) has value +0 and repeats the x and y of the last
 * real entry of its group.  G never exceeds nnz/g + min(Z, nnz).
 * Count mode (MAPZ = MAPX = MAPY = MAPV = NULL), capacity behaviour, status codes and
 * synchronisation as for insum_coo_to_groupcoo.
 */
insum_status insum_map_to_groupcoo(int64_t X, int64_t Y, int64_t Z, int64_t nnz,
                                   const int32_t* mx, const int32_t* my, const int32_t* mz,
                                   const void* mv, insum_dtype dt, int32_t g,
                                   int32_t* g_used, int64_t* num_groups,
                                   int32_t* MAPZ, int32_t* MAPX, int32_t* MAPY, void* MAPV,
                                   int64_t capacity_groups,
                                   void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of device workspace insum_spconv_groupcoo needs for these sizes (an inverse table of
 * the map, transposed weights and a list of repeated (x, z) pairs); 0 when the shape runs on
 * the scatter kernels, which need none.  Host only. */
size_t insum_spconv_groupcoo_workspace_bytes(int64_t X, int64_t Z, int64_t C, int64_t M,
                                             int64_t G, int32_t g, insum_dtype dt);

/*
 * Out = conv (accumulate == 0) or Out += conv (accumulate != 0) with the grouped map above.
 *
 *   MAPZ, MAPX, MAPY, MAPV  device; layout as produced by insum_map_to_groupcoo (any order of
 *               groups and slots is accepted; coordinates are not checked)
 *   In          device dt[Y, ld_in]   input features, C channels per point, ld_in >= C
 *   W           device dt[Z, C, M]    one C x M weight matrix per kernel offset, m fastest
 *   dt          type of MAPV, In and W: F32, F16 or BF16
 *   Out         device float[X, ld_out]  output features, M channels per point, fp32
 *   workspace   device scratch, at least insum_spconv_groupcoo_workspace_bytes(...) bytes
 *               (INSUM_ERR_CAPACITY otherwise); may be NULL when that is 0
 *   reuse_map_tables  0: the call derives its tables from the map.  Nonzero: the caller
 *               guarantees that `workspace` (same address) still holds what an earlier call
 *               with the same X, Z, G, g, dt and the same MAPZ/MAPX/MAPY/MAPV contents left
 *               there (the layers of a network that share one kernel map), so that step is
 *               skipped.  In, W, Out, C, M and accumulate may differ between such calls; the
 *               workspace must be large enough for each of them, and every one of them must
 *               be a shape with a nonzero insum_spconv_groupcoo_workspace_bytes.
 *
 * Products are exact and sums are formed in fp32.  16-bit types with C a multiple of 8, at
 * most 256, ld_in a multiple of 8 and In 16-byte aligned run on the matrix cores, in one of
 * two schedules: when the map holds at least X*Z/16 slots, by output point with the sums
 * kept in registers and stored once (only repeated (x, z) pairs use atomics); otherwise by
 * slot with fp32 atomic adds into Out.  Everything else runs on a general scatter kernel.
 * The order of the fp32 additions differs between schedules and, where atomics are used,
 * from run to run: results are reproducible up to fp32 summation order.
 * A slot with value zero contributes nothing; In and W are assumed finite.  Asynchronous.
 */
insum_status insum_spconv_groupcoo(int64_t X, int64_t Y, int64_t Z, int64_t C, int64_t M,
                                   int64_t G, int32_t g,
                                   const int32_t* MAPZ, const int32_t* MAPX, const int32_t* MAPY,
                                   const void* MAPV, const void* In, int64_t ld_in, const void* W,
                                   insum_dtype dt, float* Out, int64_t ld_out, int accumulate,
                                   int reuse_map_tables,
                                   void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* INSUM_H */
