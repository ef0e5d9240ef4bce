/*
 * smat.h -- C ABI of the MI355X (gfx950) blocked SpMM library.
 *
 * The library computes C = A * B for a sparse A given in CSR and a dense B
 * (paper, Background section: C in F^{M x N}, A in F^{M x K} sparse, B in
 * F^{K x N} dense).  Following the paper's pipeline (Overview section), A is
 * preprocessed once: its rows are permuted, A' = P A, so that fewer h x w
 * blocks of the fixed grid hold a nonzero (Preprocessing section), A' is
 * stored as BCSR (Data Structures section) and every multiplication then
 * walks the stored blocks of each block row and multiplies each with the
 * matching rows of B on the matrix units (Implementation section, Alg. 1).
 *
 * Conventions for every entry point
 *   - returns a smat_status_t, never throws or aborts; on error the out
 *     parameters are left untouched and smat_last_error() holds a message
 *     (thread local, valid until the next call on the same thread);
 *   - pointers marked HOST are ordinary host memory, pointers marked DEVICE
 *     are device memory of the current HIP device, owned by the caller;
 *   - inputs are borrowed for the duration of the call only: the handle keeps
 *     its own host copies and the device workspace passed to smat_bind_device;
 *   - the library never allocates or frees device memory;
 *   - there is no CPU fallback: smat_spmm needs a bound handle and a gfx950
 *     device, anything else is an error.
 */
#ifndef SMAT_H
#define SMAT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct smat_handle smat_handle_t;   /* opaque, owned by the library */

typedef enum {
    SMAT_OK = 0,
    SMAT_ERR_INVALID_ARG = 1,   /* null pointer, negative size, bad option value      */
    SMAT_ERR_BAD_CSR = 2,       /* row_ptr not monotone, column out of range or not
                                   strictly ascending inside a row                     */
    SMAT_ERR_UNSUPPORTED = 3,   /* block size other than 16x16, sizes beyond the limits */
    SMAT_ERR_ALLOC = 4,         /* host allocation failed                               */
    SMAT_ERR_NOT_BOUND = 5,     /* smat_spmm before smat_bind_device                    */
    SMAT_ERR_HIP = 6            /* a HIP runtime call failed; text in smat_last_error   */
} smat_status_t;

/* Storage type of A and B: the operand types of the gfx950 matrix units (the paper's
 * Introduction claims every precision the matrix units accept).  fp16 and bf16 take two
 * bytes per value; SMAT_E4M3 and SMAT_E5M2 are the OCP 8-bit floating-point formats (1-4-3
 * bits, bias 7, no infinities; 1-5-2 bits, bias 15) and SMAT_I8 is a two's complement byte.
 * C is fp32 (fp32 accumulation) for the floating-point types and int32 (int32 accumulation,
 * wrapping on overflow) for SMAT_I8. */
typedef enum { SMAT_F16 = 0, SMAT_BF16 = 1, SMAT_E4M3 = 2, SMAT_E5M2 = 3, SMAT_I8 = 4 } smat_dtype_t;

typedef struct {
    int block_h;        /* block height; only 16 is accepted                            */
    int block_w;        /* block width;  only 16 is accepted                            */
    int reorder;        /* 0: keep the row order (P = I); 1: Jaccard clustering, kept
                           only if it yields strictly fewer blocks than the identity;
                           2: the same, then the columns of P A are clustered in the same
                           way (a column's pattern being the block rows it touches) and
                           that column order Q is kept only if P A Q has strictly fewer
                           blocks still -- the variant the paper tried and set aside
                           (Preprocessing section); B is not moved: the kernel fetches
                           its rows through Q                                            */
    int tau_permille;   /* merge threshold of the clustering in 1/1000, 0..1000: a row w
                           joins a cluster with column union pc iff
                           1 - |w n pc| / |w u pc| < tau_permille / 1000                 */
    int dense_tiles;    /* block-dense regions (sixteen block rows sharing most of their
                           block columns) have a kernel of their own that stages panels of
                           B in LDS: 0 = take it where an estimate says it is faster,
                           1 = take it wherever it applies, -1 = never.  It reads B in
                           whole block columns, so it is not used once reorder = 2 has
                           kept a column order, and 1 together with reorder = 2 is refused */
    int concurrent_streams; /* 1..16: on how many streams smat_spmm calls on this handle may be in
                           flight at the same time with the full choice of launches.  A launch
                           with few block-dense tiles splits every tile over several workgroups
                           and keeps their partial tiles in the workspace; each of the first
                           concurrent_streams distinct streams the handle sees owns an area of
                           32 MiB for them (part of smat_device_bytes when the matrix has
                           block-dense parts).  Calls on further streams are still correct:
                           they run such launches unsplit                                    */
} smat_options_t;

/* Default options: 16 x 16 blocks, reordering on, tau = 0.7, dense_tiles = 0, concurrent_streams = 2. */
void smat_default_options(smat_options_t *opt);

/*
 * Preprocessing (Overview and Preprocessing sections): CSR -> row permutation
 * that lowers the number of nonzero blocks -> BCSR structure.
 *
 *   M, K      rows / columns of A, 0 <= M < 2^31 - 16, 0 <= K < 2^24
 *   row_ptr   HOST int64[M+1], row_ptr[0] == 0, non-decreasing
 *   col_idx   HOST int32[nnz], strictly ascending inside each row, 0 <= col < K
 *   vals      HOST values [nnz], bit patterns of dtype: two bytes each for fp16 / bf16,
 *             one byte each for the 8-bit types; a stored value of 0 still counts as a
 *             nonzero of the pattern
 *   opt       may be NULL (defaults)
 *   out       receives a new handle; release it with smat_destroy
 *
 * The row "pattern" used by the clustering is the set of block columns
 * floor(c / 16) a row touches.  Clusters are opened by the lowest unclustered
 * row and scanned in ascending row order with the cluster union updated after
 * every merge; clusters are concatenated in creation order; perm[new] = old.
 * Runs on the host, integer arithmetic only.
 */
smat_status_t smat_preprocess(int64_t M, int64_t K,
                              const int64_t *row_ptr, const int32_t *col_idx, const void *vals,
                              smat_dtype_t dtype, const smat_options_t *opt,
                              smat_handle_t **out);

/* Sizes and counts of the preprocessed matrix: number of block rows ceil(M/16),
 * number of stored blocks n_e (Eq. 2 bounds it), n_e under the identity order,
 * and whether the identity order was kept.  Any out pointer may be NULL. */
smat_status_t smat_get_info(const smat_handle_t *h, int64_t *n_block_rows, int64_t *n_blocks,
                            int64_t *n_blocks_identity, int *used_identity);

/* Shape and storage type the handle was made for (what smat_spmm expects of B and C): rows M
 * and columns K of A, and the smat_dtype_t.  Any out pointer may be NULL. */
smat_status_t smat_get_dims(const smat_handle_t *h, int64_t *M, int64_t *K, int *dtype);

/* perm: HOST int32[M], perm[new_row] = old_row (A' = P A, Overview section). */
smat_status_t smat_export_perm(const smat_handle_t *h, int32_t *perm);

/* Column order of the row + column variant (reorder = 2): HOST int32[K], col_perm[new] = old;
 * the identity when no column order was kept.  With one, the block structure and the values of
 * smat_export_bcsr are those of P A Q.  n_blocks_rows_only (may be NULL) receives the number of
 * blocks of P A. */
smat_status_t smat_export_col_perm(const smat_handle_t *h, int32_t *col_perm, int64_t *n_blocks_rows_only);

/* Canonical BCSR of A' (Data Structures section), all HOST, caller allocated:
 *   row_ptr int32[n_block_rows+1]  offsets into col_idx per block row
 *   col_idx int32[n_blocks]        block column of each block, ascending per block row
 *   vals    [n_blocks*256] values of the handle's dtype (2 or 1 bytes each), one 16x16
 *           block after the other, row-major, zero filled
 * vals may be NULL to export the structure only. */
smat_status_t smat_export_bcsr(const smat_handle_t *h, int32_t *row_ptr, int32_t *col_idx, void *vals);

/* Bytes of device workspace smat_bind_device needs for this handle. */
smat_status_t smat_device_bytes(const smat_handle_t *h, size_t *bytes);

/* What one multiplication has to read from the device copy of the matrix (host
 * counts, known after smat_preprocess).  The device copy groups the consecutive
 * stored blocks of a block row into "packs" of at most 32 occupied columns (a
 * column of a block is occupied when it holds a stored entry); one matrix
 * instruction per 16 output columns multiplies a pack, and columns that hold
 * nothing are neither stored nor fetched from B.  Two full blocks make a pack.
 * A block row whose occupied columns hold hardly more than one stored entry each (at most
 * 9/8 on average; 3/2 when the values of the whole matrix kept by column would exceed 192 MB)
 * is kept by entry instead: packs of 32 stored entries, one value and one
 * named row of B per entry, expanded into the instruction's operand in registers.
 *   n_packs       packs of the whole matrix
 *   value_bytes   bytes of block values over all packs
 *   table_bytes   bytes of the per-pack tables naming the rows of B, plus the
 *                 launch table and the row permutation
 *   n_columns     rows of B named by the tables: the occupied columns over all stored
 *                 blocks (the stored entries, in block rows kept by entry); each is
 *                 fetched once per output tile
 * Any out pointer may be NULL. */
smat_status_t smat_get_layout_info(const smat_handle_t *h, int64_t *n_packs, int64_t *value_bytes,
                                   int64_t *table_bytes, int64_t *n_columns);

/*
 * Copies the preprocessed matrix into caller-owned device memory and builds the
 * device-side block values there (the kernel's own layout: packs of blocks, the
 * table of B rows per pack, and a launch table of the block rows).
 *
 *   dev_workspace  DEVICE, 256-byte aligned, at least smat_device_bytes() bytes,
 *                  must stay alive and untouched until smat_destroy
 *   stream         hipStream_t (NULL = default stream); the call enqueues copies
 *                  and kernels on it and returns after they have completed
 */
smat_status_t smat_bind_device(smat_handle_t *h, void *dev_workspace, size_t bytes, void *stream);

/* Reads the device-side block values back and returns them in the canonical
 * layout of smat_export_bcsr (vals: HOST [n_blocks*256] values of the handle's dtype); used to verify
 * the device-side conversion.  Synchronises the stream. */
smat_status_t smat_export_device_vals(const smat_handle_t *h, void *vals, void *stream);

/*
 * C = A * B on the device (Implementation section, Alg. 1: per output tile, loop
 * over the stored blocks of the block row, multiply-accumulate on the matrix
 * units), fp32 accumulation (int32 for SMAT_I8), rows of C in the ORIGINAL row order of A.
 *
 *   dB   DEVICE, K x N row-major, element type = dtype of the handle, leading
 *        dimension ldb >= N (in elements); the padding between rows may be read (whatever it
 *        holds never reaches C), nothing outside the ((K-1)*ldb + N) elements is touched
 *   dC   DEVICE, M x N row-major fp32 (int32 for SMAT_I8), leading dimension ldc >= N; every
 *        element of the M x N window is overwritten (rows of A without entries give 0)
 *   N    >= 1 (N = 0 is a no-op); any value, any alignment: wide vector loads
 *        are used when N, ldb and the base address allow it
 *   stream  hipStream_t; the call only enqueues work (no synchronisation)
 *
 * Stream-ordered and re-entrant: calls on different handles, and calls on the SAME handle on
 * different streams with different C, may be in flight at the same time (from one host thread
 * or several).  The only state a call uses besides its arguments is an area of partial tiles
 * for launches with few block-dense tiles; every stream has its own (option concurrent_streams),
 * and a call on a stream without one runs such a launch unsplit -- the same product, summed in
 * another order.  For a given handle, stream and arguments the result is bitwise reproducible.
 * Limits: the bytes of B that are addressed, ((K-1)*ldb + N) * bytes per value, must stay below 2 GiB;
 * ldb < 2^23; N <= 1048560.
 */
smat_status_t smat_spmm(const smat_handle_t *h, const void *dB, int64_t ldb,
                        void *dC, int64_t ldc, int64_t N, void *stream);

/*
 * smat_spmm for callers that cannot allocate device memory and cannot give the handle's workspace
 * the areas for partial tiles either: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Same arguments, same product, same kernels.  The partial
 * tiles of a launch that splits its block-dense tiles live in an array of 16 MiB that is part of
 * the library's device code (one copy per GPU, held from the first use of the library on that
 * GPU until the process ends); the call allocates and frees nothing, on the device or through
 * any library.  smat_bind_device looks the array's address up for its device.
 *   - a launch whose partial tiles would exceed the 16 MiB is refused with SMAT_ERR_UNSUPPORTED
 *     before anything is enqueued (smat_spmm takes it);
 *   - every call on a GPU uses that GPU's one array, whatever the handle or stream: calls that
 *     overlap in time on one GPU race -- order them on one stream, or with events.  The array
 *     keeps what the last call left; nothing in it has to start at zero, every partial tile is
 *     written in full before it is read.
 */
smat_status_t smat_spmm_static(const smat_handle_t *h, const void *dB, int64_t ldb,
                               void *dC, int64_t ldc, int64_t N, void *stream);

/* Frees the host state of the handle (never device memory).  NULL is allowed. */
void smat_destroy(smat_handle_t *h);

/* Message of the last error on the calling thread ("" if none). */
const char *smat_last_error(void);

/* Name of the SpMM kernel variant chosen by the last smat_spmm on this thread
 * (for profiles and logs). */
const char *smat_last_kernel(void);

#ifdef __cplusplus
}
#endif
#endif /* SMAT_H */
