/*
 * cer.h -- C ABI of the MI355X (gfx950) CER / CSER matrix-product library.
 *
 * The library stores a quantized, low-entropy weight matrix W (m rows, n columns, every element
 * one of K codebook values) in the two formats of Wiedemann, Mueller, Samek, "Compact and
 * Computationally Efficient Representation of Deep Neural Networks":
 *
 *   CER  (Compressed Entropy Row,          Section III-A): Omega, colI, OmegaPtr, rowPtr
 *   CSER (Compressed Shared Elements Row,  Section III-A): the same plus OmegaI
 *
 * and computes Y = W.X on the GPU from those arrays (Appendix A-C, Algorithms 3 and 4): per row,
 * the inputs selected by the groups of column indices, each weighted by its group's value; the
 * most frequent value Omega[0] owns no indices and is handled by a constant term (Appendix
 * A-A1).  The paper's algorithm sums a group's inputs first and multiplies the sum once.  On
 * MI355X a multiply-add costs what an add costs, and what the format saves is the bytes it does
 * not read; the default kernels therefore form the same sum with one multiply-add per indexed
 * element (the element's weight comes from the group boundaries without any search), a variant
 * that sums first is kept for the batched product, and wide batches of matrices that are not
 * sparse enough are multiplied from the decoded matrix on the matrix cores -- cer_matmul_path
 * tells which.
 *
 * Conventions
 *   - Every function returns CER_OK (0) or a negative CER_E_* code; nothing aborts or throws
 *     across this boundary.  cer_strerror() names a code; cer_last_hip_error() returns the HIP
 *     error number behind the calling thread's most recent CER_E_HIP.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory on the
 *     device that was current when the handle was created.  Matrices are row-major fp32.
 *   - A handle is immutable after creation: any number of threads / streams may use it
 *     concurrently for matmul, decode and inspection.  Free it exactly once.
 *   - A handle made by cer_encode is a CER handle, one made by cser_encode a CSER handle; the
 *     cer_matmul / cer_decode calls accept only the former, cser_matmul / cser_decode only the
 *     latter (CER_E_FORMAT otherwise).  Inspection calls and cer_free accept both.
 */
#ifndef CER_H_
#define CER_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cer_matrix cer_handle_t; /* opaque */

enum {
    CER_OK = 0,
    CER_E_INVALID = -1,         /* null pointer, non-positive size, unknown selector */
    CER_E_NOT_IN_CODEBOOK = -2, /* a matrix element equals no codebook value */
    CER_E_BAD_CODEBOOK = -3,    /* duplicate, NaN or infinite codebook value */
    CER_E_TOO_LARGE = -4,       /* n, the number of indexed elements or of groups exceeds 32 bits */
    CER_E_NOMEM = -5,           /* host allocation failed */
    CER_E_HIP = -6,             /* a HIP call failed, or the handle has no device copy */
    CER_E_FORMAT = -7           /* CER handle given to a cser_* call or the reverse */
};

/* selectors of cer_get_array */
enum {
    CER_ARRAY_OMEGA = 0,    /* fp32 [K]      distinct values, most frequent first */
    CER_ARRAY_COLI = 1,     /* uint [nnz]    column indices, grouped by row then by value */
    CER_ARRAY_OMEGAPTR = 2, /* uint [G+1]    group boundaries into colI, leading 0 */
    CER_ARRAY_ROWPTR = 3,   /* uint [m+1]    row boundaries into OmegaPtr, leading 0 */
    CER_ARRAY_OMEGAI = 4,   /* uint [G]      CSER only: index into Omega of each group */
    CER_ARRAY_COUNT = 5     /* int64 [K]     occurrences of Omega[k] in W (not part of the format) */
};

/*
 * cer_encode / cser_encode -- dense matrix + codebook -> CER / CSER handle (Section III-A, the
 * four format steps; CSER paragraph).  Host-side, O(m.n); not part of the timed product, as in
 * the paper's experiments (Section V).
 *
 *   W_host    [m][n] fp32, host, row-major, borrowed for the duration of the call
 *   codebook  [K] fp32, host, distinct finite values; every element of W must equal one of them
 *             bit for bit, except that -0.0 and +0.0 are the same value (stored as +0.0)
 *   out       receives the handle; owned by the caller until cer_free
 *
 * The arrays are defined as follows (all indices 0-based):
 *   Omega     codebook values that occur in W, by occurrence count, highest first; equal counts
 *             keep codebook order.  Omega[0] (whatever its value) is never indexed.
 *   colI      for each row, for rank k = 1, 2, ...: the ascending columns holding Omega[k].
 *   OmegaPtr  OmegaPtr[0] = 0; one entry per group = number of indices emitted so far.
 *             CER: a row emits groups for ranks 1..kmax (kmax = highest rank present in it); an
 *             absent rank repeats the previous pointer.  CSER: present ranks only.
 *   OmegaI    CSER: the rank of each group.
 *   rowPtr    rowPtr[0] = 0; rowPtr[r+1] = number of groups emitted up to and including row r.
 *   widths    Omega fp32; each index array is stored in the smallest of 8/16/32 bits that holds
 *             its largest possible value: colI n-1, OmegaPtr nnz, rowPtr G, OmegaI K-1 (Section V).
 *
 * If a HIP device is present the arrays are also uploaded to the current device (one
 * allocation; colI and OmegaI at their minimal width, the pointer arrays as uint32, followed by
 * two arrays derived from them on the device: 8 bytes per row that name the row's first group
 * and first colI position, and, for 2 - 256 values, the rank table described at cer_matmul_ex);
 * with no device the handle is host-only and *_matmul returns CER_E_HIP.
 * m = 0 or n = 0 is allowed (empty arrays).  Errors: CER_E_INVALID, CER_E_BAD_CODEBOOK,
 * CER_E_NOT_IN_CODEBOOK, CER_E_TOO_LARGE, CER_E_NOMEM, CER_E_HIP (upload failed).
 */
int cer_encode(const float* W_host, int64_t m, int64_t n, const float* codebook, int32_t K,
               cer_handle_t** out);
int cser_encode(const float* W_host, int64_t m, int64_t n, const float* codebook, int32_t K,
                cer_handle_t** out);

/*
 * cer_matmul / cser_matmul -- Y = W.X from the encoded arrays (Algorithm 3 / Algorithm 4; the
 * constant Omega[0].sum_i X[i,l] of Appendix A-A1 is added when Omega[0] != 0).
 *
 *   X_dev   [n][batch] fp32, device, row-major, read only
 *   Y_dev   [m][batch] fp32, device, row-major, fully overwritten (no accumulation into Y)
 *   batch   number of columns of X (L in the paper), >= 1
 *   stream  a hipStream_t passed as void*; NULL = the default stream
 *
 * Work is enqueued on `stream` and the call returns without synchronising.  The caller keeps
 * ownership of X and Y and must keep them alive until the stream has run the work.  When
 * Omega[0] != 0 and batch > 1 (or X does not fit in LDS) a stream-ordered temporary of batch floats
 * (plus partial sums) is allocated and released on `stream`, and so is one for a batched product
 * of a matrix with split rows (cer_long_row_parts > 0); kernels 2, 3 and 5 have temporaries of
 * their own (a tile-major copy of X; the decoded matrix; strips x m x batch partial sums).
 * Otherwise (and when cer_matmul_path reports kernel 0 or 1) the call only launches kernels and may be recorded into a HIP graph
 * after one eager call on the device.
 * fp32 arithmetic; the summation order differs from a sequential loop.  With Omega[0] != 0 the
 * rounding error is relative to sum|w||x| + |Omega[0]|.sum|x|: Appendix A-A1 adds that term and
 * subtracts it again inside the groups' weights.
 * Errors: CER_E_INVALID (null pointers, batch < 1), CER_E_FORMAT, CER_E_HIP.
 */
int cer_matmul(const cer_handle_t* h, const float* X_dev, float* Y_dev, int64_t batch, void* stream);
int cser_matmul(const cer_handle_t* h, const float* X_dev, float* Y_dev, int64_t batch, void* stream);

/*
 * cer_matmul_noalloc -- the same product for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Accepts CER and CSER
 * handles.  It calls no allocating routine: the one temporary a product can need here, the column
 * sums of X for a non-zero most frequent value (batch floats plus partial sums), lives in a fixed
 * 2 MiB device array that is part of the library's code object (one per GPU, kept until the process
 * ends), and only kernels that need no other temporary are chosen: the batch-1 kernels, the batched
 * kernel that gathers from L2 with every row whole, the LDS-resident kernel for batches of one tile;
 * never the decode + dense route.  Y equals cer_matmul's within the same error bound (bit for bit
 * where both run the same kernel).  A product whose column sums would not fit the array (batch above
 * about 260 000 columns with Omega[0] != 0) is refused with CER_E_TOO_LARGE.
 * All calls on one GPU share the array: two such calls that overlap in time on one GPU (different
 * streams or threads) race when Omega[0] != 0; calls on one stream are ordered and safe.  Nothing in
 * the array has to survive between calls, and every word a call reads it has written before.
 * Arguments, stream semantics and the other errors are those of cer_matmul.
 */
int cer_matmul_noalloc(const cer_handle_t* h, const float* X_dev, float* Y_dev, int64_t batch, void* stream);

/*
 * cer_trim -- gives the device memory of released temporaries back to the system.  The products and
 * conversions that need a temporary (see each call) take it, ordered on the caller's stream, from
 * a memory pool of the library's own on the current device; the pool keeps what it has handed out
 * once, because getting a few hundred megabytes from the system again costs more than the product
 * that needs them.  Its size settles at the largest amount in use at one time.  cer_trim releases
 * whatever is not in use at the moment of the call on the current device; it does not synchronise
 * and may be called at any time.  Errors: CER_E_HIP.
 */
int cer_trim(void);

/*
 * cer_matmul_path -- which kernel cer_matmul / cser_matmul runs for this handle and batch:
 *   0  CER_PATH_GEMV: batch-1 kernel, always taken for batch 1: X staged in LDS per workgroup (read
 *      from global memory when it does not fit), one wave per row (4 or 8 waves per row in matrices
 *      of at most two rows per compute unit), colI read with 16-byte loads, the weight of every
 *      position derived from a bitmap of the group boundaries, one multiply-add per position.
 *      Handles of 2 - 256 values with X in LDS use their rank table (below) to find the boundaries
 *   4  CER_PATH_GEMV_EXPAND: an earlier batch-1 kernel, only on request: the group values are
 *      expanded per colI position into LDS and every input is multiplied by its position's value;
 *      needs X to fit in LDS
 *   1  CER_PATH_GEMM: batched kernel that gathers rows of X from L2, one wave per (row, tile of batch
 *      columns: 32 when a row of X is a whole number of 128-byte lines, else 32, 64 or 128 by the
 *      cache lines the gathers touch; any width and 4-byte aligned X / Y are served by 16-byte
 *      gathers).  By default the group values are expanded per colI position into LDS and every
 *      gathered row is multiplied by its position's value; with CER_OPT_SUM_THEN_MULTIPLY the
 *      gathered rows of a group are summed first and multiplied once (slower on MI355X)
 *   2  CER_PATH_XTILE: batched kernel with the input resident in LDS -- the reuse of input elements
 *      that the paper's Section V-C names as the missing optimisation: a tile of 4 or 8 batch columns
 *      of all n input rows is staged once per workgroup and serves many rows of W.  Applicable when
 *      n.16 bytes fit in LDS (n <= about 10000), K <= 64 and no row has more than 63 groups;
 *      for a batch of more than one tile a stream-ordered temporary of about the size of X is
 *      used (a tile-major copy of X).
 *   3  CER_PATH_DENSE: decode + dense: the matrix is decoded into a stream-ordered temporary of 4.m.n
 *      bytes and multiplied on the fp32 matrix cores.  Chosen when the estimated time of the gathers
 *      (max(4.batch, 128) bytes per indexed element through the L1/L2 path) exceeds that of the
 *      decode and the dense contraction: wide batches of matrices with more than about one
 *      indexed element in five, any batch > 1 of matrices with most elements indexed.  The
 *      arithmetic is then that of a dense fp32 product (same error bound), not Algorithm 3 / 4.
 *   5  CER_PATH_STRIP: batched kernel with strips of 1024 input rows resident in LDS; needs the strip-major
 *      index of cer_prepare_strips.  For a handle that has it the library chooses this kernel where its
 *      estimated duration is below that of kernels 1 and 3: wide batches of large matrices (AlexNet-fc6
 *      shape, batch 32 / 64 / 128: 30 / 46 / 78 us against 33 / 57 / 107 us with kernel 1)
 * On MI355X kernel 2 beats kernel 1 for narrow batches of large matrices (kernel 1 moves a whole
 * 128-byte line per index however narrow the batch) and loses for wide ones (random LDS gathers
 * are bank-conflict bound): it is chosen when it is applicable, batch <= 8 and the matrix holds
 * at least 2.5 million indices.
 * Errors: CER_E_INVALID, CER_E_HIP (no device copy).
 */
int cer_matmul_path(const cer_handle_t* h, int64_t batch);

/*
 * cer_matmul_ex -- cer_matmul / cser_matmul (it accepts handles of both formats) with the caller's
 * choices instead of the library's; the result is the same Y within the same error bound.  The
 * library reads no environment variable: this call is the only way to steer it.
 *   opts->path       CER_PATH_AUTO, or the kernel to prefer (numbering of cer_matmul_path).  A
 *                    preferred kernel is taken whenever it is applicable to the handle and the batch
 *                    (0 / 4 for batch 1, 1 / 2 / 3 / 5 for batch > 1); where it is not, the library
 *                    chooses as cer_matmul does.  cer_matmul_path_ex tells which kernel will run.
 *   opts->tile_cols  kernel 1, batch a multiple of 4 with 16-byte aligned X and Y: batch columns per
 *                    tile, 8, 16, 32, 64 or 128; 0 = the library's choice
 *   opts->flags      CER_OPT_SUM_THEN_MULTIPLY    kernel 1: the variant that sums a group's gathered
 *                                                 rows before its one multiplication
 *                    CER_OPT_ROWS_WHOLE           kernel 1: rows in their own order and never in parts
 *                                                 (see cer_long_row_parts); kernel 0: a row is never
 *                                                 shared between waves
 *                    CER_OPT_X_FROM_GLOBAL        kernel 0: gather X from global memory, no LDS copy
 *                    CER_OPT_ONE_COLUMN_PER_LANE  kernel 1, ragged batch widths: one batch column per
 *                                                 lane instead of 16-byte gathers
 *                    CER_OPT_SHORT_CHUNKS / CER_OPT_LONG_CHUNKS  kernel 1: group values expanded 512 /
 *                                                 2048 positions at a time (default: by the average row)
 *                    CER_OPT_NO_RANK_TABLE        kernels 0 and 1: find the group boundaries through rowPtr and
 *                                                 OmegaPtr even when the handle has a rank table
 *                                                 (a derived array of handles with 2 - 256 values:
 *                                                 per row its first colI position and the end of the
 *                                                 group of every rank, at a fixed stride, 4 bytes per
 *                                                 row and rank; it lets a wave fetch all boundaries
 *                                                 of its row with its first memory request; kernel 1
 *                                                 uses it for handles of 2 - 64 values)
 * opts == NULL is cer_matmul's behaviour.  Errors: those of cer_matmul; CER_E_INVALID also for an
 * undefined path, tile width or flag.
 */
enum { CER_PATH_AUTO = -1, CER_PATH_GEMV = 0, CER_PATH_GEMM = 1, CER_PATH_XTILE = 2, CER_PATH_DENSE = 3,
       CER_PATH_GEMV_EXPAND = 4, CER_PATH_STRIP = 5 };
enum { CER_OPT_SUM_THEN_MULTIPLY = 1, CER_OPT_ROWS_WHOLE = 2, CER_OPT_X_FROM_GLOBAL = 4,
       CER_OPT_ONE_COLUMN_PER_LANE = 8, CER_OPT_SHORT_CHUNKS = 16, CER_OPT_LONG_CHUNKS = 32,
       CER_OPT_NO_RANK_TABLE = 64 };
typedef struct {
    int32_t path;
    int32_t tile_cols;
    uint32_t flags;
    uint32_t reserved; /* 0 */
} cer_matmul_opts_t;
int cer_matmul_ex(const cer_handle_t* h, const float* X_dev, float* Y_dev, int64_t batch, void* stream,
                  const cer_matmul_opts_t* opts);
int cer_matmul_path_ex(const cer_handle_t* h, int64_t batch, const cer_matmul_opts_t* opts);

/*
 * cer_prepare_strips -- builds, once per handle, the strip-major index that kernel 5 (CER_PATH_STRIP) needs: the
 * column-blocked reuse of input elements (Section V-C).  X is cut into equally long strips of at most 1024 consecutive rows; for
 * every strip and every row of W the index lists the row's indexed elements whose column falls into the strip, each
 * as 16 bits: the rank of the element's value in Omega (6 bits) and the column inside the strip (10 bits), in chunks
 * of eight entries (the last chunk of a strip's share of a row is filled up with entries of rank 0, whose weight
 * Omega[0] - Omega[0] is zero).  It is DERIVED from the format arrays (which stay as they are): 2 bytes per indexed
 * element, up to 14 bytes of padding and a 4-byte pointer per strip and row, in device memory of its own.  Kernel 5
 * copies one strip of 32 batch columns into LDS per workgroup (128 KB), multiplies every element of the strip's share
 * of its rows by Omega[rank] - Omega[0], and leaves one partial sum per strip and row in a stream-ordered temporary
 * of strips x m x batch floats, which a second kernel adds up in strip order (the result does not depend on the
 * launch).  Applicable to codebooks of at most 64 values (CER_E_TOO_LARGE otherwise) and batches of
 * 2 columns or more (a last tile of fewer than 32 columns costs what a full one costs; batches of up to 16 columns
 * run a variant that moves half as much through LDS; widths that are not multiples of 4, and X / Y that are only
 * 4-byte aligned, are read and written in smaller pieces).  Once the index exists, cer_matmul / cser_matmul choose kernel 5 by
 * themselves where they expect it to be the fastest (cer_matmul_path tells); cer_matmul_ex can prefer or avoid it.
 * Not thread-safe against products running on the same handle: call it before the handle is shared.  A second call
 * is a no-op.  Errors: CER_E_INVALID, CER_E_TOO_LARGE, CER_E_NOMEM, CER_E_HIP (no device copy, allocation failed).
 */
int cer_prepare_strips(cer_handle_t* h);

/*
 * cer_decode / cser_decode -- arrays -> dense matrix (Section III-A: the arrays
 * determine M).  W_host_out: [m][n] fp32, host, written completely; equals the encoder's input bit
 * for bit (with -0.0 returned as +0.0).  Host-side.  Errors: CER_E_INVALID, CER_E_FORMAT.
 */
int cer_decode(const cer_handle_t* h, float* W_host_out);
int cser_decode(const cer_handle_t* h, float* W_host_out);

/*
 * Inspection (host copies of the arrays of Section III-A; lengths as in the proofs of Theorems 1
 * and 2, with the pointer arrays' leading zeros included).
 *
 * cer_get_array: *host_ptr is borrowed and valid until cer_free; *len = number of elements,
 * *elem_bits = 8, 16 or 32 (unsigned integers), 32 for OMEGA (fp32), 64 for COUNT (int64).
 * CER_ARRAY_OMEGAI on a CER handle yields len 0.  cer_get_dims: any output pointer may be NULL;
 * nnz = len(colI), groups = len(OmegaPtr) - 1.  cer_storage_bits = sum over the format's arrays
 * of length x width (negative code on error).  cer_get_stats: entropy H = -sum p_k log2 p_k of
 * the element distribution (Section III), p0 = share of Omega[0], k_bar = mean number of
 * non-empty groups per row, k_tilde = mean number of empty (padding) groups per row (Theorem 1).
 */
int cer_get_array(const cer_handle_t* h, int which, const void** host_ptr, int64_t* len,
                  int32_t* elem_bits);
int cer_get_dims(const cer_handle_t* h, int64_t* m, int64_t* n, int32_t* K, int64_t* nnz,
                 int64_t* groups, int32_t* is_cser);
int64_t cer_storage_bits(const cer_handle_t* h);
int cer_get_stats(const cer_handle_t* h, double* H, double* p0, double* k_bar, double* k_tilde);

/*
 * cer_clone_device -- a second handle with the same host arrays and its own, freshly allocated
 * device copy on the current device.  Lets a benchmark rotate over more encoded bytes than the
 * GPU's caches hold.  The clone has no strip-major index, whether the original has one or not
 * (cer_prepare_strips builds it per handle).  Errors: CER_E_INVALID, CER_E_NOMEM, CER_E_HIP.
 */
int cer_clone_device(const cer_handle_t* h, cer_handle_t** out);

/* Bytes of the format arrays on the device (colI at its width + uint32 OmegaPtr and rowPtr + OmegaI
 * + Omega): the algorithmic traffic of one product; 0 for a host-only handle.  (A product that goes
 * through the rank table reads that table -- 4 bytes per row and rank, rounded up to a power of two
 * ranks -- in place of OmegaPtr, rowPtr and OmegaI.) */
int64_t cer_device_bytes(const cer_handle_t* h);

/* Matrices with rows of unequal length (longest row above twice the average and at least 2048
 * indexed elements, average row at least 256 unless a row is split): the batched product takes
 * the rows in descending order of length.  When a row holds more than 3 P indexed elements,
 * P = 1.5 x the average rounded up to a multiple of 2048, the rows of more than 2 P elements
 * are served in parts of P elements, so that one long row does not outlast the rest of the
 * launch; such a product uses a stream-ordered temporary of batch floats per part.  Returns
 * the number of parts beyond the rows' first ones (0: no row is split; also for host-only
 * handles). */
int64_t cer_long_row_parts(const cer_handle_t* h);

/* Frees host and device memory.  NULL is allowed. */
void cer_free(cer_handle_t* h);

/*
 * dense_matmul -- the plain dense fp32 product Y = W.X (Algorithm 1) as a HIP kernel on the same
 * device: the baseline the CER / CSER speed-up is quoted against.
 *   W_dev [m][n], X_dev [n][batch], Y_dev [m][batch]: fp32, device, row-major; Y overwritten.
 * Enqueued on `stream`, no synchronisation.  Errors: CER_E_INVALID, CER_E_HIP.
 */
int dense_matmul(const float* W_dev, const float* X_dev, float* Y_dev, int64_t m, int64_t n,
                 int64_t batch, void* stream);

/*
 * CSR comparator (Section III-A "Sparse format", Algorithm 2): the paper's main sparse baseline in
 * the same harness.  csr_encode stores the elements different from 0.0 in row-major order (values
 * fp32, column indices at the minimal 8/16/32-bit width, row pointers; on the device the row
 * pointers are uint32); csr_matmul computes Y = W.X from them (one multiply-add per stored
 * element); csr_decode rebuilds the dense matrix (-0.0 comes back as +0.0).  Pointer, layout,
 * stream and error conventions are those of cer_encode / cer_matmul / cer_decode.
 * csr_get_array selectors: 0 values (fp32 [nnz]), 1 colI (uint [nnz]), 2 rowPtr (uint [m+1]).
 */
typedef struct csr_matrix csr_handle_t; /* opaque */
int csr_encode(const float* W_host, int64_t m, int64_t n, csr_handle_t** out);
int csr_matmul(const csr_handle_t* h, const float* X_dev, float* Y_dev, int64_t batch, void* stream);
int csr_decode(const csr_handle_t* h, float* W_host_out);
int csr_get_array(const csr_handle_t* h, int which, const void** host_ptr, int64_t* len, int32_t* elem_bits);
int64_t csr_storage_bits(const csr_handle_t* h);
int64_t csr_device_bytes(const csr_handle_t* h);
int csr_clone_device(const csr_handle_t* h, csr_handle_t** out);
void csr_free(csr_handle_t* h);

/*
 * Cost model (host-side analytics; Sections III-B, IIII and V): elementary operations of ONE
 * matrix-vector product (batch 1) per format, the storage of the format, and the energy that
 * Table I (45 nm CMOS, pJ) assigns to those operations -- reads and writes priced by the width of
 * the value and the size of the array that holds it, 32-bit float add 0.9 pJ, mul 3.7 pJ.
 *   CER_COUNT_THEOREM  counts as Eq. (2), (4), (10), (12) price them (proofs of Theorems 1, 2)
 *   CER_COUNT_EXAMPLE  the hand count of Section III-B: both ends of a row's pointer range are read
 *                      and summing k terms costs k - 1 additions (dense 48, CSR 32, CER 24 for the
 *                      example row)
 * A non-zero most frequent value adds n input reads, n + m additions, one multiplication and one
 * Omega read (Appendix A-A1).  Errors: CER_E_INVALID.
 */
enum { CER_COUNT_THEOREM = 0, CER_COUNT_EXAMPLE = 1 };
typedef struct {
    int64_t read_weight;   /* dense elements / CSR values */
    int64_t read_omega, read_colI, read_omegaPtr, read_rowPtr, read_omegaI;
    int64_t read_input;    /* elements of the input vector */
    int64_t mul, add, write;
    int64_t storage_bits;
    double energy_pj;
} cer_cost_t;
int cer_cost_model(const cer_handle_t* h, int convention, cer_cost_t* out);
int csr_cost_model(const csr_handle_t* h, int convention, cer_cost_t* out);
int dense_cost_model(int64_t m, int64_t n, int convention, cer_cost_t* out);

/*
 * Device front-end -- for a weight matrix that already lives in GPU memory (Section V-B: weights
 * are quantized, then converted losslessly into the format).
 *
 * cer_encode_device: as cer_encode / cser_encode, but W_dev is a DEVICE pointer to the row-major
 * m x n fp32 matrix (borrowed for the call, never written) and the whole conversion runs in HIP
 * kernels on `stream`; only the encoded arrays travel to the host (the handle's host mirror).
 * `codebook` is a HOST array of K <= 256 values (CER_E_TOO_LARGE above that); `format` is
 * CER_FORMAT_CER or CER_FORMAT_CSER.  The handle is identical, array for array and bit for bit, to
 * the one cer_encode / cser_encode builds from the same matrix.  The call returns after the stream
 * has drained.  Errors: those of cer_encode, CER_E_HIP (also: no device).
 *
 * cer_quantize_uniform: the uniform quantizer.  Takes the range [w_min, w_max] of the `count`
 * elements at W_dev, places K = 2^bits (1 <= bits <= 8) equidistant points on it, both ends
 * included, and maps every element to its nearest point.  All arithmetic is IEEE binary32 with one
 * rounding per operation: step = (w_max - w_min) / (K - 1); point_j = w_min + j.step (the last
 * point is w_max itself); code = clamp(round_half_even((w - w_min) / step), 0, K - 1).  A constant
 * array has the single point w_min (K = 1).  Outputs, each optional (NULL): codes_dev (device,
 * one byte per element), Wq_dev (device, fp32, the quantized values; must not overlap W_dev),
 * codebook_out (host, room for 2^bits floats), K_out (host).  Returns after the stream has
 * drained.  Errors: CER_E_INVALID (null W_dev, bits out of range, count < 0, NaN or infinite
 * weight), CER_E_BAD_CODEBOOK (range so narrow that two points coincide), CER_E_HIP.
 *
 * cer_quantize_encode_device: both steps in one call; the quantized matrix is never materialised
 * in fp32.  Same result as cer_quantize_uniform followed by cer_encode_device on Wq_dev with the
 * returned codebook.
 *
 * cer_decode_device: the handle's device arrays -> dense matrix in device memory (W_dev_out:
 * [m][n] fp32, row-major, written completely; CER and CSER handles alike).  Same values as
 * cer_decode / cser_decode.  Enqueued on `stream`, no synchronisation.  Errors: CER_E_INVALID,
 * CER_E_HIP (no device copy, wrong device).
 */
enum { CER_FORMAT_CER = 0, CER_FORMAT_CSER = 1 };
int cer_encode_device(const float* W_dev, int64_t m, int64_t n, const float* codebook, int32_t K,
                      int32_t format, void* stream, cer_handle_t** out);
int cer_quantize_uniform(const float* W_dev, int64_t count, int32_t bits, uint8_t* codes_dev,
                         float* Wq_dev, float* codebook_out, int32_t* K_out, void* stream);
int cer_quantize_encode_device(const float* W_dev, int64_t m, int64_t n, int32_t bits, int32_t format,
                               void* stream, float* codebook_out, int32_t* K_out, cer_handle_t** out);
int cer_decode_device(const cer_handle_t* h, float* W_dev_out, void* stream);

/*
 * cer_stream_copy -- plain device-to-device copy of `bytes` bytes (rounded down to a multiple of
 * 16; both pointers 16-byte aligned) by a simple HIP kernel.  A measurement aid: a kernel of
 * exactly known memory traffic against which hardware byte counters (and the attainable copy
 * bandwidth) are calibrated.  Enqueued on `stream`, no synchronisation.  Errors: CER_E_INVALID,
 * CER_E_HIP.
 */
int cer_stream_copy(void* dst_dev, const void* src_dev, int64_t bytes, void* stream);

/*
 * cer_stream_read -- reads `bytes` bytes (rounded down to a multiple of 16; src_dev 16-byte aligned)
 * with 16-byte loads and nothing else, in the launch shape of the batch-1 product kernel (256
 * workgroups of 1024 threads); sink_dev receives 16 KiB of folded words that keep the loads alive.
 * A measurement aid: what one launch that only streams as many bytes as a product reads costs on
 * this machine -- the ceiling against which the product kernel's time is read.  Enqueued on
 * `stream`, no synchronisation.  Errors: CER_E_INVALID, CER_E_HIP.
 */
int cer_stream_read(const void* src_dev, int64_t bytes, void* sink_dev, void* stream);

const char* cer_strerror(int code);
int cer_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CER_H_ */
