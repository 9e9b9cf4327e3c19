/*
 * vbr_spmm.h -- C ABI of the blocked sparse-times-dense path for one MI355X (gfx950).
 *
 * The path, after "Blocking Techniques for Sparse Matrix Multiplication on Tensor
 * Accelerators" (arXiv 2202.05868):
 *
 *   sa1_reorder   1-SA row reordering: quotient rows over a regular column partition (section
 *                 3.1, Eq. 4), grouping of identical quotient rows (Algorithm 1 applied to
 *                 quotient rows, hash of Eq. 5), greedy merge with pattern update (Algorithm 2)
 *                 under the two-step merge condition (section 3.2: Jaccard similarity, Eq. 3,
 *                 and the limit lambda <= lambda0 / (1 - tau/2) that gives Theorem 1).
 *   vbr_build     row partition + column partition -> variable-block-row matrix that keeps
 *                 only the nonzero blocks, zero-filled (section 2, section 3.1 last paragraph).
 *   vbr_spmm      C = A.B, every stored block multiplied as a small dense product on the
 *                 matrix units (section 4.4.1), in one launch per kernel class the matrix
 *                 needs (at most nine: see vbr_get_launches below).
 *
 * sa1_reorder and vbr_build are deterministic integer host code.  vbr_spmm runs on the GPU.
 * All pointers are HOST pointers unless the name ends in _dev.  Nothing is retained from the
 * caller's arrays after a call returns, except the device buffer handed to vbr_upload.
 * No call throws or aborts; every call returns 0 (VBR_OK) or a negative error code.
 * Calls on distinct handles may run concurrently; a handle is not internally locked.
 */
#ifndef VBR_SPMM_H
#define VBR_SPMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    VBR_OK = 0,
    VBR_EINVAL = -1,       /* bad argument, non-canonical CSR, perm not a bijection, ... */
    VBR_ENOMEM = -2,       /* host allocation failed */
    VBR_EHIP = -3,         /* a HIP runtime call failed (vbr_last_hip_error has its code) */
    VBR_ESTATE = -4,       /* call out of order (e.g. vbr_spmm before vbr_upload) */
    VBR_EUNSUPPORTED = -5  /* valid input the GPU path does not take (see vbr_upload) */
};

enum { VBR_F16 = 0, VBR_BF16 = 1 };

/*
 * Sparse matrix in CSR (section 2), borrowed from the caller, host memory.
 * Canonical form is required: row_ptr[0] == 0, row_ptr non-decreasing, row_ptr[n_rows] == nnz,
 * column indices strictly increasing inside a row and in [0, n_cols).  Every stored entry is a
 * structural nonzero, whatever its value.
 */
typedef struct vbr_csr {
    int64_t n_rows, n_cols, nnz;
    const int64_t *row_ptr;   /* [n_rows + 1] */
    const int32_t *col_idx;   /* [nnz] */
    const void *vals;         /* [nnz] 16-bit patterns of type dtype; may be NULL for sa1_reorder */
    int32_t dtype;            /* VBR_F16 or VBR_BF16 */
} vbr_csr_t;

typedef struct vbr vbr_t;     /* host handle of a built VBR matrix, owned by the library */

/*
 * 1-SA (Algorithm 2 with the merge condition of section 3.2) on the quotient rows of `csr`
 * over column blocks of width col_block (n_cols % col_block must be 0).
 *
 *   tau         Jaccard threshold in [0, 1].  A row joins a group when
 *               |P & v| / |P | v| >= tau (one binary64 division; two empty patterns are similar)
 *               and |P | v| <= floor(lambda0 / (1 - tau/2)), lambda0 = blocks of the group's seed.
 *   perm        out [n_rows]: perm[new position] = original row.  Groups are numbered in seed
 *               order (by smallest original row), rows ascend inside a group.
 *   row_groups  out, room for n_rows + 1 entries: row_groups[g] = first position of group g,
 *               row_groups[*n_groups] = n_rows.
 * Identical quotient rows are grouped first and visited as one row, in order of their
 * smallest member (section 3.1).  csr->vals is not read.
 */
int sa1_reorder(const vbr_csr_t *csr, int32_t col_block, double tau,
                int32_t *perm, int32_t *row_groups, int32_t *n_groups);

/*
 * Build the VBR matrix of `csr` for ANY valid row partition (perm a bijection of the rows,
 * row_groups strictly increasing from 0 to n_rows) and the regular column partition of width
 * col_block.  Per group the stored blocks are the column blocks that hold at least one entry of
 * the group's rows, ascending; a block of group g is the h_g x col_block window of the permuted
 * matrix, zero-filled (section 2: fill-in).  Values are packed in the layout the kernel reads.
 * On success *out is a new handle; free it with vbr_free.
 */
int vbr_build(const vbr_csr_t *csr, const int32_t *perm, const int32_t *row_groups,
              int32_t n_groups, int32_t col_block, vbr_t **out);

/*
 * Views of the index arrays, valid until vbr_free.  Any out pointer may be NULL.
 *   row_groups [n_groups + 1], perm [n_rows]          as given to vbr_build
 *   blk_ptr    [n_groups + 1]   blocks of group g are blk_ptr[g] .. blk_ptr[g+1]-1
 *   blk_col    [n_blocks]       column block of each stored block, ascending inside a group
 *   blk_off    [n_blocks + 1]   running element offset; block b holds h_g * col_block elements
 */
int vbr_get_index(const vbr_t *v, const int32_t **row_groups, const int32_t **perm,
                  const int64_t **blk_ptr, const int32_t **blk_col, const int64_t **blk_off,
                  int64_t *n_groups, int64_t *n_blocks, int64_t *stored_elems);

/* Copy stored block `blk` out of the packed kernel layout: dst[h_g * col_block] 16-bit, row-major. */
int vbr_unpack_block(const vbr_t *v, int64_t blk, void *dst);

/*
 * Check of a built matrix against itself: every index the kernels use (B rows of the gather lists,
 * value offsets of tiles and panels, row positions, the schedule's class ranges, the sections of the
 * device buffer) lies inside what it indexes.  VBR_OK, or VBR_EINVAL at the first violation.  vbr_build
 * produces matrices that pass; the tests call this on every matrix they build.
 */
int vbr_audit(const vbr_t *v);

/* Bytes of device memory vbr_upload needs (a multiple of 256, never 0). */
int64_t vbr_device_bytes(const vbr_t *v);

/*
 * Copy the packed matrix and its schedule into buf_dev (device memory of the current device,
 * allocated by the caller, at least vbr_device_bytes(v) bytes, 256-byte aligned) on hip_stream
 * (a hipStream_t, NULL = default stream) and wait for the copy.  The handle keeps the pointer;
 * the buffer must outlive every vbr_spmm on this handle.  The library allocates no device memory.
 * Any col_block >= 1 is taken; widths that are multiples of 8 take the fast gather path.
 * For a matrix that needs more than one kind of kernel, the first upload of a handle also creates,
 * on the current device, three streams of default priority and four events (vbr_free destroys
 * them): a multiply of several launches spreads them over these streams, see vbr_spmm.
 */
int vbr_upload(vbr_t *v, void *buf_dev, void *hip_stream);

/*
 * C = A.B on the GPU (section 4.4.1), asynchronous on hip_stream, no synchronisation; one to
 * VBR_MAX_LAUNCHES kernel launches (vbr_get_launches lists them), no allocation, no memset.
 * Several launches of one call write disjoint rows of C and do not depend on each other: the
 * first runs on hip_stream, the others on the handle's own streams, which first wait for an event
 * recorded on hip_stream and which hip_stream then waits for, so the call is ordered against
 * earlier and later work on hip_stream like a single launch (measured on RMAT graphs: 0 to 13 %
 * shorter than the launches one behind the other).  Two calls on ONE handle from different streams
 * at the same time would share these streams and events: give each concurrent caller its own
 * handle.  With the environment variable VBR_SPMM_SERIAL set (read once), every launch stays on
 * hip_stream.
 *   B_dev  K x N row-major, 16-bit type of the matrix, leading dimension ldb (elements)
 *   C_dev  n_rows x N row-major fp32, leading dimension ldc (elements); OVERWRITTEN (beta = 0),
 *          rows in ORIGINAL row order (the reordering is internal); rows without entries get 0
 * Requires N >= 0, N % 8 == 0, ldb >= N, ldb % 8 == 0, ldc >= N, ldc % 4 == 0, B_dev and C_dev
 * 16-byte aligned (else VBR_EINVAL), and ldb < 2^26 (inside a granule of 32 B rows lanes use 32-bit
 * byte offsets; else VBR_EUNSUPPORTED); B itself may be larger than 4 GiB.  Products are exact, sums
 * are fp32 on the matrix units.
 * B and C must not overlap each other or the uploaded buffer.
 * Non-finite values: the zero fill-in of a stored block is multiplied like any other value, so a
 * NaN or Inf in B row k reaches every C row whose group stores the column block of k (the
 * format's semantics).  For groups lower than 16 rows, which are multiplied in slabs of 16 rows
 * cut across group boundaries, it reaches the rows of the slabs that hold such a group when the
 * slabs share whole column blocks (panels), and only the rows of the slabs one of whose rows has
 * an entry in column k itself when they gather single columns.  B rows of column blocks that no
 * group stores are never read.
 */
int vbr_spmm(const vbr_t *v, const void *B_dev, int64_t ldb, float *C_dev, int64_t ldc,
             int64_t N, void *hip_stream);

/*
 * The kernel launches one vbr_spmm call with dense width N issues, in issue order (for reporting;
 * vbr_spmm itself launches from the same plan).  Rows of groups lower than 16 rows are multiplied
 * 128 at a time, by the panel kernel (their slabs of 16 rows share the B rows of the union of their
 * column blocks) or by the tile kernel on column-gathered slabs (every slab loads exactly the B rows
 * of the columns its rows touch), whichever packing needs fewer loads; the other groups by the tile
 * kernel, on whole column blocks or, where the blocks are mostly fill-in, on the columns the rows
 * of a tile touch (VBR_LAUNCH_GATHER_*), either in one launch per class of tile
 * height that occurs (1, 2, 3-4, 5-8 slabs of 16 rows) or, for small matrices, in one launch that
 * mixes the classes: between 0 and VBR_MAX_LAUNCHES launches.  kinds / tiles / workgroups (each
 * room for VBR_MAX_LAUNCHES entries, any may be NULL) receive the kernel, the number of row tiles
 * or panels, and the grid size of each launch.
 */
enum { VBR_MAX_LAUNCHES = 9 };
enum {
    VBR_LAUNCH_PANEL = 0, VBR_LAUNCH_TILE_1 = 1, VBR_LAUNCH_TILE_2 = 2, VBR_LAUNCH_TILE_4 = 3,
    VBR_LAUNCH_TILE_8 = 4, VBR_LAUNCH_TILE_MIXED = 5,
    VBR_LAUNCH_GATHER_1 = 6, VBR_LAUNCH_GATHER_2 = 7, VBR_LAUNCH_GATHER_4 = 8, VBR_LAUNCH_GATHER_8 = 9
};
int vbr_get_launches(const vbr_t *v, int64_t N, int32_t *n_launches, int32_t *kinds, int64_t *tiles,
                     int64_t *workgroups);

/* Number of workgroup tiles and K-steps of the schedule (for reporting). */
int vbr_get_schedule(const vbr_t *v, int64_t *n_tiles, int64_t *n_ksteps, int64_t *packed_elems);

/*
 * K-steps (32 gathered B rows each) every workgroup tile walks, for judging the balance of the
 * schedule: the tiles in launch order of their classes, then the column-gathered slabs, then the
 * panels.  Returns their number; fills out[0 .. min(number, cap) - 1] when out is not NULL.
 */
int64_t vbr_get_tile_ksteps(const vbr_t *v, int64_t *out, int64_t cap);

void vbr_free(vbr_t *v);

/*
 * Blocking curve (sections 2.2 and 4.3.1): run 1-SA once per threshold taus[0 .. n_taus-1] and
 * report, per threshold, what the VBR matrix of that blocking would hold, without building it:
 *   n_groups[i]       row groups
 *   n_blocks[i]       stored (nonzero) blocks
 *   stored_elems[i]   nonzero area: sum over stored blocks of height * col_block
 *   sum_heights[i]    sum over stored blocks of their height
 * so that the in-block density after blocking is rho' = nnz / stored_elems[i] and the average
 * height of the nonzero blocks is Delta'_H = sum_heights[i] / n_blocks[i] (section 2.2).
 * *selected is the index of the blocking whose Delta'_H is nearest to target_height (the rule of
 * sections 4.3.2 and 4.4.2: take the blocking with Delta'_H ~ Delta), compared exactly in integers; of equally
 * near ones the first in the order given; a blocking without blocks is never selected unless
 * none has any (then 0).  Any out array may be NULL.  target_height > 0.
 */
int sa1_blocking_curve(const vbr_csr_t *csr, int32_t col_block, const double *taus, int32_t n_taus,
                       int64_t target_height, int64_t *n_groups, int64_t *n_blocks,
                       int64_t *stored_elems, int64_t *sum_heights, int32_t *selected);

/*
 * Comparator: C = A.B straight from the CSR matrix on the GPU, one fp32 accumulator per output
 * element, no blocking and no matrix units.  It stands where the sparse-library routine stands
 * in the comparison of section 4.4.2 and is not part of the blocked path.
 *   csr_spmm_create   validates the host CSR (canonical form as above) and keeps a copy
 *   csr_device_bytes  device bytes csr_upload needs (multiple of 256, never 0)
 *   csr_upload        copies it into buf_dev (caller-allocated, 256-byte aligned) on hip_stream and waits
 *   csr_spmm          asynchronous on hip_stream; same B / C / N / ldb / ldc rules as vbr_spmm
 */
typedef struct csr_dev csr_dev_t;
int csr_spmm_create(const vbr_csr_t *csr, csr_dev_t **out);
int64_t csr_device_bytes(const csr_dev_t *h);
int csr_upload(csr_dev_t *h, void *buf_dev, void *hip_stream);
int csr_spmm(const csr_dev_t *h, const void *B_dev, int64_t ldb, float *C_dev, int64_t ldc,
             int64_t N, void *hip_stream);
void csr_free(csr_dev_t *h);

/*
 * Measured denominators (not part of the path; nothing in vbr_spmm calls them): one launch of a
 * small loop that keeps ONE unit of the compute units busy, at four workgroups of four waves per
 * compute unit.  The caller times the launch with events on hip_stream; *work receives what one
 * launch performs (floating-point operations for the VBR_PROBE_MFMA_* kinds, bytes otherwise), so
 * rate = *work / time.  They price the kernel of section 4.4.1 against what the chip delivers:
 * the issue rate of the matrix instructions, the rate at which operands leave LDS, the rate of
 * 16-byte-per-lane direct-to-LDS loads from cache-resident memory, and a copy through HBM.
 *   buf_dev  caller-allocated device memory, 256-byte aligned, buf_bytes >= 1 MiB; the copy kind
 *            copies its first half onto its second half; the other kinds only read it, apart from
 *            a result word at its start that is never actually written
 *   iters    loop count of the kernel (ignored by VBR_PROBE_HBM_COPY), > 0
 * VBR_EINVAL for an unknown kind or a bad buffer.  Asynchronous; allocates nothing.
 */
enum {
    VBR_PROBE_MFMA_16X16X32 = 0,   /* v_mfma_f32_16x16x32_f16, 4 independent accumulators per wave */
    VBR_PROBE_MFMA_16X16X16 = 1,   /* v_mfma_f32_16x16x16_f16 */
    VBR_PROBE_MFMA_32X32X16 = 2,   /* v_mfma_f32_32x32x16_f16, 2 independent accumulators per wave */
    VBR_PROBE_LDS_TR_B64 = 3,      /* ds_read_b64_tr_b16 in the kernels' swizzled row pattern */
    VBR_PROBE_LDS_B64 = 4,         /* ds_read_b64, consecutive addresses */
    VBR_PROBE_LDS_B128 = 5,        /* ds_read_b128, consecutive addresses */
    VBR_PROBE_LDS_DMA = 6,         /* global_load_lds_dwordx4 out of a region of at most 2 MiB */
    VBR_PROBE_HBM_COPY = 7         /* 16 bytes per lane streaming copy */
};
int vbr_probe_launch(int32_t kind, void *buf_dev, int64_t buf_bytes, int32_t iters, void *hip_stream,
                     double *work);

const char *vbr_strerror(int code);
int vbr_last_hip_error(void);   /* hipError_t of the last failing HIP call on this thread */

#ifdef __cplusplus
}
#endif
#endif /* VBR_SPMM_H */
