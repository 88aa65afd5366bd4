/*
 * libcsr5 -- CSR5 sparse matrix-vector multiply for AMD MI355X (gfx950).
 *
 * C ABI.  The operation is the one the paper states in Section 1: y = A*x with
 * A an m x n sparse matrix given in CSR (Section 2.1), computed on the CSR5
 * format of Section 3 by the algorithm of Section 4.
 *
 * Every array argument is a DEVICE pointer (memory of the current HIP device)
 * unless a comment says "host".  Indices are int32 and values fp64 in the csr5_
 * entry points; csr5s_ is the single-precision and csr5l_ the 64-bit-index
 * variant of the conversion, and their handles go through the same calls.  A
 * handle is tied to the device that was current when it was made: call with that
 * device current (csr5_spmv* return CSR5_EINVAL otherwise) and with pointers to
 * its memory.  The tile
 * width omega is fixed to 64, the wavefront width (Section 3.2); sigma, the tile
 * height, is chosen per matrix.  T = omega*sigma nonzeros per tile,
 * p = ceil(nnz/T) tiles, p_c = floor(nnz/T) complete tiles (Section 3.1, 3.3).
 *
 * Error behaviour: every function returns CSR5_OK (0) or a negative code; none
 * aborts or throws.  On failure csr5_convert* sets *out to NULL.
 *
 * Streams: the *_ex calls enqueue their kernels on the given HIP stream
 * (hipStream_t passed as void*, NULL = the default stream) and return without
 * waiting unless stated otherwise.
 */
#ifndef CSR5_H
#define CSR5_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct csr5_handle_s *csr5_handle_t; /* opaque; owned by the library */

enum {
    CSR5_OK = 0,
    CSR5_EINVAL = -1, /* bad argument (null pointer, negative size, inconsistent row_ptr) */
    CSR5_ENOMEM = -2, /* allocation failed or workspace too small */
    CSR5_EHIP = -3,   /* a HIP runtime call or kernel launch failed */
    CSR5_ERANGE = -4  /* sigma outside [CSR5_SIGMA_MIN, CSR5_SIGMA_MAX], or matrix beyond the stated limits */
};

/* value types: the csr5_ entry points take double, the csr5s_ ones float */
#define CSR5_DTYPE_F64 0
#define CSR5_DTYPE_F32 1

#define CSR5_OMEGA 64
#define CSR5_SIGMA_MIN 1
#define CSR5_SIGMA_MAX 48

/* csr5_convert_ex flags */
#define CSR5_FLAG_NONE 0u
#define CSR5_FLAG_NO_HOST_CHECK 1u /* do not wait for the device-side checks of the input: only enqueue */
/* Measurement aids (they fix what the library otherwise chooses by the matrix's size, see csr5_spmv):
 * a matrix whose cross-tile sums go through the auxiliary array adds them ... */
#define CSR5_FLAG_AUX_TWO_KERNELS 2u /* ... always with the second kernel */
#define CSR5_FLAG_AUX_ONE_KERNEL 4u  /* ... inside the tile kernel whenever the handle has the words for it
                                        (8 <= sigma <= 32, at most 32768 tiles).  Not both; unknown bits: CSR5_EINVAL. */

/* bits of the device-side status word reported by csr5_status */
#define CSR5_STATUS_BAD_ROW_PTR 1u /* row_ptr decreasing or outside [0, nnz] */
#define CSR5_STATUS_BAD_COL_IDX 2u /* a column index outside [0, n) */
#define CSR5_STATUS_HAS_DIRTY 4u   /* informational: some tile holds an empty row */
#define CSR5_STATUS_HAS_EMPTY_ROWS 8u /* informational: the matrix has a row without nonzeros */

/* ==========================================================================
 * 1. The method: conversion (Section 3), SpMV (Section 4), back-conversion
 *    (Section 3.6), release.
 * ========================================================================== */

/*
 * sigma from nnz/row (Section 3.2): the paper's four-way rule with bounds
 * <r, s, t, u> = <16, 16, 256, 16> measured on MI355X (nnz/row is the integer
 * quotient nnz/m; on this GPU the best sigma turned out not to depend on it).
 * One addition: when nnz/row <= t and the matrix would have fewer than 12288
 * tiles at that sigma, sigma = 8 (a small matrix needs the parallelism more than
 * the amortisation).  Pure host arithmetic.
 */
int32_t csr5_sigma_auto(int64_t nnz, int64_t m);

/*
 * Bytes of device workspace csr5_convert_ex needs for a matrix of m rows and
 * nnz nonzeros at the given sigma (0 = the value csr5_sigma_auto picks).  An
 * upper bound computable on the host: tile_ptr (p+1 words) + tile_desc
 * (p_c*W*64 words) + empty_offset_ptr (p_c+1 words) + empty_offset (at most
 * min(m + p_c, p_c*T) words) + the SpMV's four auxiliary arrays (p+1 doubles each) + one
 * word per tile saying how far into its first row the tile starts (p+1) + for
 * 8 <= sigma <= 32 a copy of the last 160 (col_idx, val) pairs in CSR order of every
 * 4th complete tile (every 2nd for sigma > 16) and of the last one (1920 bytes each;
 * the last 32 pairs, 384 bytes, when nnz exceeds 28 million; it lets a tile finish
 * a row that began in the previous tile without a second kernel) + for 8 <= sigma <= 32
 * and at most 32768 tiles what the one-kernel form of the auxiliary-array path
 * needs (per tile two words naming the groups of tiles its first row touches; per
 * group of 4 tiles, 2 for sigma > 16, and with each of the four auxiliary arrays,
 * an 8-byte meeting word and a counter) + the conversion's scratch
 * (p_c/8192 + 1 + 8192 words) + a status word, each rounded up to 256 bytes.
 * Returns 0 for invalid arguments.
 */
size_t csr5_workspace_bytes(int32_t m, int32_t nnz, int32_t sigma);

/*
 * CSR -> CSR5 (Sections 3.3-3.5; the four steps of Section 5.4).
 *
 *   m, n, nnz   matrix shape, all >= 0, nnz < 2^31, m <= 2^31 - 2 (else CSR5_ERANGE).
 *   row_ptr     int32[m+1], row_ptr[0] = 0, row_ptr[m] = nnz, non-decreasing.
 *               BORROWED: read now and again by every csr5_spmv (the format
 *               keeps it unchanged, Section 1); must outlive the handle.
 *   col_idx     int32[nnz], values in [0, n).  Any int32-aligned address (a view into a
 *               larger array is fine); a 16-byte aligned one lets the SpMV read it with
 *               wider loads.
 *   val         double[nnz].
 *               Both MODIFIED IN PLACE: inside every complete tile the entries
 *               go from CSR order to tile column-major order (Section 3.1);
 *               the entries after the last complete tile stay.  The caller keeps
 *               ownership of the memory, must keep it alive for the handle's
 *               lifetime, and gets CSR order back with csr5_to_csr.
 *   out         receives the handle.  The handle owns tile_ptr, tile_desc
 *               (bit_flag, y_offset, seg_offset packed as in Section 3.5) and
 *               empty_offset with its per-tile start array.
 *
 * csr5_convert picks sigma itself, allocates with hipMalloc, runs on the default
 * stream and waits for the conversion's device-side checks of the input
 * (row_ptr[0] = 0, row_ptr[m] = nnz, non-decreasing; column indices in range):
 * it BLOCKS, and returns CSR5_EINVAL (col_idx and val restored to CSR order)
 * when one of them fails.  The conversion kernels stay inside the arrays
 * whatever row_ptr holds.
 *
 * csr5_convert_ex: sigma = 0 means automatic.  If workspace != NULL the
 * handle's arrays are carved from it (workspace_bytes must be at least
 * csr5_workspace_bytes(m, nnz, sigma); the memory stays the caller's and must
 * outlive the handle), and no allocation happens on the device.  Without
 * CSR5_FLAG_NO_HOST_CHECK it blocks and validates like csr5_convert.  With the
 * flag it only enqueues work: consistency of row_ptr and the range of col_idx
 * are still checked on the device; read the verdict with csr5_status.
 */
int csr5_convert(int32_t m, int32_t n, int32_t nnz, const int32_t *row_ptr, int32_t *col_idx,
                 double *val, csr5_handle_t *out);
int csr5_convert_ex(int32_t m, int32_t n, int32_t nnz, const int32_t *row_ptr, int32_t *col_idx,
                    double *val, int32_t sigma, void *workspace, size_t workspace_bytes,
                    void *hip_stream, uint32_t flags, csr5_handle_t *out);

/*
 * y = A*x (Section 4: Algorithm 8 per complete tile; the entries after the last
 * complete tile by a row-wise SIMD reduction).  A tile's first segment, when it
 * continues a row of an earlier tile, is completed in one of two ways, fixed per
 * matrix at conversion: if every tile can get at the head of its first row
 * (8 <= sigma <= 32; every 4th tile, every 2nd for sigma > 16, starts at most 160
 * entries into a row -- 32 in a matrix of more than 28 million nonzeros -- and
 * re-reads them, the others start at most a tile's length into a row and are
 * handed the sum by the neighbouring tile of their workgroup; in particular
 * every matrix without a row longer than 33, and up to 28 million nonzeros every
 * matrix without a row longer than 161), it adds the head itself and stores the
 * finished row, and the SpMV is ONE kernel; otherwise those segments go through
 * an auxiliary array (Section 4's "global auxiliary array").  Its sums are added
 * to y by a second small kernel, or, where that is faster (8 <= sigma <= 32 and
 * at most 6144 tiles, or at most 32768 tiles and fewer than 64 nonzeros per row
 * on average), inside the tile kernel: the tiles of a workgroup settle their
 * common rows through LDS, workgroups meet at a word of the array per row (one
 * atomic exchange each when the row touches two workgroups' tiles, a counter
 * otherwise), nobody waits, and whoever comes last stores the row -- again ONE
 * kernel.  Which of these, and whether rows without nonzeros need
 * their zeros written, is in the conversion's status word: the library launches
 * only what the matrix needs once the host has seen that word (csr5_convert and
 * csr5_convert_ex without CSR5_FLAG_NO_HOST_CHECK read it; after an asynchronous
 * conversion call csr5_status once), and everything until then -- same result,
 * a few microseconds slower.
 * x double[n], y double[m]; y is overwritten (rows without nonzeros get 0).  x
 * and y must not overlap.  Asynchronous.  Summation order differs from CSR
 * order; rows that the second kernel sums with more than one wavefront and
 * rows cut inside the incomplete tile are added up atomically, so their last
 * bits may differ between runs (the one-kernel forms add in a fixed order).  The handle holds four auxiliary arrays, taken
 * in turn by successive calls: up to four SpMVs on ONE handle may be in flight at
 * the same time (on different streams); a fifth must be ordered after the first.
 */
int csr5_spmv(csr5_handle_t h, const double *x, double *y);
int csr5_spmv_ex(csr5_handle_t h, const double *x, double *y, void *hip_stream);

/*
 * For callers that cannot allocate (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): csr5_spmv_ex with the auxiliary array
 * of the cross-tile sums taken from a fixed array in the library's device image
 * (CSR5_STATIC_SCRATCH_BYTES per GPU, held until the process ends) instead of
 * the handle's own.  No hipMalloc, hipFree or other allocating call is made.
 * Same arguments, same result and same error codes as csr5_spmv_ex (double
 * precision, either index width), plus CSR5_ERANGE when the handle has more than
 * CSR5_STATIC_MAX_TILES tiles (p, the incomplete tile included).  A matrix that
 * takes the auxiliary-array path always gets the two-kernel form here (the
 * one-kernel form keeps words of its own between calls, which a shared array
 * cannot promise).  Every slot the second kernel reads has been written by the
 * first, so nothing needs clearing between calls.  All calls on one GPU share the array, whatever their handle:
 * calls that overlap in time on one GPU race; order them (one stream, or events).
 */
#define CSR5_STATIC_SCRATCH_BYTES (4u << 20)
#define CSR5_STATIC_MAX_TILES (CSR5_STATIC_SCRATCH_BYTES / 8u - 1u)
int csr5_spmv_static(csr5_handle_t h, const double *x, double *y, void *hip_stream);

/*
 * CSR5 -> CSR (Section 3.6): transposes col_idx and val of every complete tile
 * back to CSR order, in place.  The handle stays valid only for csr5_free.
 */
int csr5_to_csr(csr5_handle_t h, void *hip_stream);

/* Releases the handle and whatever it allocated; never touches the caller's
 * arrays or workspace.  NULL is accepted. */
int csr5_free(csr5_handle_t h);

/* ==========================================================================
 * 2. Variants of the same calls: single precision, 64-bit indices.
 * ========================================================================== */

/*
 * Single-precision variant (the paper's Figure 3 is single precision): same
 * format, same kernels instantiated for float.  val, x and y are float arrays;
 * a handle made by csr5s_convert_ex is accepted by csr5s_spmv_ex,
 * csr5_to_csr and all the introspection calls (and csr5s_spmv_profile), and refused
 * (CSR5_EINVAL) by the double-precision SpMV calls, and vice versa.  Everything
 * said above about arguments, ownership and errors applies.
 */
int csr5s_convert_ex(int32_t m, int32_t n, int32_t nnz, const int32_t *row_ptr, int32_t *col_idx,
                     float *val, int32_t sigma, void *workspace, size_t workspace_bytes,
                     void *hip_stream, uint32_t flags, csr5_handle_t *out);
int csr5s_spmv_ex(csr5_handle_t h, const float *x, float *y, void *hip_stream);


/*
 * 64-bit index variant (Section 3.3 mentions it for tile_ptr: a 63-bit row
 * index with the top bit as the empty-row flag), for matrices of 2^31 nonzeros
 * and more: row_ptr is int64[m+1], nnz is int64, and the handle's tile_ptr and
 * empty_offset_ptr have 8-byte entries (tile_ptr: bit 63 is the flag).  Rows,
 * columns and the other arrays are as above (m, n < 2^31; col_idx, tile_desc
 * and empty_offset are 32-bit), values are double.  Limits: at most 2^26 - 5
 * tiles (one wavefront each; a grid holds fewer than 2^32 threads), which is
 * 68 G nonzeros at sigma = 16, and m + tiles < 2^32 - 512; beyond them
 * CSR5_ERANGE (csr5l_workspace_bytes: 0).
 * The handle is accepted by csr5_spmv, csr5_spmv_ex, csr5_spmv_profile,
 * csr5_to_csr, csr5_status, csr5_get_info, csr5_read_array (8-byte entries for
 * arrays 0 and 2) and csr5_free; csr5_get_arrays refuses it, csr5l_get_arrays
 * refuses a 32-bit one.  Everything else said for csr5_convert_ex applies.
 */
size_t csr5l_workspace_bytes(int32_t m, int64_t nnz, int32_t sigma);
int csr5l_convert_ex(int32_t m, int32_t n, int64_t nnz, const int64_t *row_ptr, int32_t *col_idx,
                     double *val, int32_t sigma, void *workspace, size_t workspace_bytes,
                     void *hip_stream, uint32_t flags, csr5_handle_t *out);
int csr5l_get_arrays(csr5_handle_t h, const uint64_t **tile_ptr, const uint32_t **tile_desc,
                     const int64_t **empty_offset_ptr, const int32_t **empty_offset);

/* ==========================================================================
 * 3. Introspection: the conversion's verdict on its input, the format's
 *    geometry and arrays (what the parity tests compare).
 * ========================================================================== */

/*
 * Waits for the conversion's stream and returns the device-side status word
 * (CSR5_STATUS_* bits) in *status (host).  BAD_* bits mean the input violated
 * the contract; results are then undefined (but conversion stays in bounds).
 * The handle remembers what it read: later csr5_spmv* calls launch only the
 * kernels this matrix needs.
 */
int csr5_status(csr5_handle_t h, uint32_t *status);

/*
 * Introspection (used by the parity tests).  All outputs are host scalars and
 * may be NULL.  empty_offset_len needs the device's count and therefore waits
 * for the conversion's stream.
 */
int csr5_get_info(csr5_handle_t h, int32_t *omega, int32_t *sigma, int32_t *p, int32_t *p_complete,
                  int32_t *desc_words_per_lane, int32_t *empty_offset_len);

/* m and n of the handle's matrix (host scalars, may be NULL). */
int csr5_get_shape(csr5_handle_t h, int32_t *m, int32_t *n);

/*
 * Device pointers to the handle's arrays (valid until csr5_free):
 *   tile_ptr          uint32[p+1]   bit 31 = tile holds an empty row (Section 3.3)
 *   tile_desc         uint32[p_c*W*64]; word k of column i of tile t at (t*W+k)*64+i;
 *                     bits [0,sigma) bit_flag, then 6 bits seg_offset, then
 *                     ceil(log2(64*sigma)) bits y_offset (Section 3.5)
 *   empty_offset_ptr  int32[p_c+1]  start of tile t's entries in empty_offset
 *   empty_offset      int32[empty_offset_len] (Algorithm 7), one per segment of
 *                     every tile whose tile_ptr has bit 31 set
 * Any output pointer may be NULL.
 */
int csr5_get_arrays(csr5_handle_t h, const uint32_t **tile_ptr, const uint32_t **tile_desc,
                    const int32_t **empty_offset_ptr, const int32_t **empty_offset);

/*
 * Copies one of the handle's arrays to HOST memory (blocking; waits for the
 * conversion's stream).  which: 0 tile_ptr, 1 tile_desc, 2 empty_offset_ptr,
 * 3 empty_offset.  dst_host must hold `bytes` bytes; bytes must not exceed the
 * array's size (empty_offset: 4*empty_offset_len), else CSR5_EINVAL.
 */
enum { CSR5_ARRAY_TILE_PTR = 0, CSR5_ARRAY_TILE_DESC = 1, CSR5_ARRAY_EMPTY_OFFSET_PTR = 2,
       CSR5_ARRAY_EMPTY_OFFSET = 3 };
int csr5_read_array(csr5_handle_t h, int which, void *dst_host, size_t bytes);

/* Static description of an error code. */
const char *csr5_strerror(int code);

/* ==========================================================================
 * 4. Measurement aids.  NOT part of the method: bench.py and the comparison of
 *    Section 5.5 use them; nothing else in the library depends on them.
 * ========================================================================== */

/*
 * Measurement helper: launches each of the SpMV's two kernels `reps` times in a
 * row on the stream, HIP events before and after each series, waits, and returns
 * the mean duration per launch in milliseconds: ms[0] the tile kernel (all
 * complete tiles plus the workgroup for the incomplete one), ms[1] the carry
 * fix-up (0 when this matrix does not need it or settles its carries inside the
 * tile kernel).  ms is a host array of 2 floats.
 * A full SpMV follows the two series, so y ends up holding A*x as after
 * csr5_spmv.  csr5s_spmv_profile: the same for a single-precision handle.
 */
int csr5_spmv_profile(csr5_handle_t h, const double *x, double *y, void *hip_stream, int reps,
                      float *ms);
int csr5s_spmv_profile(csr5_handle_t h, const float *x, float *y, void *hip_stream, int reps,
                       float *ms);

/*
 * Measurement helper: what the memory system alone charges for this matrix's tile
 * streams.  A kernel with one wavefront per complete tile, in the SpMV's tile
 * order, that only reads the tile's col_idx, val and descriptors (the bytes the
 * per-column loop of Algorithm 8 streams) is launched `reps` times in a row, then
 * `reps` times again with every wavefront also storing one value to each row its
 * tile starts (the write stream of y).  ms[0], ms[1]: mean duration per launch in
 * milliseconds of the two series (HIP events, as above; waits for the stream).
 * The tile kernel cannot be faster than ms[1]; the distance is what its gathers,
 * its LDS traffic and its arithmetic cost.  y (device, y_bytes bytes: at least m
 * values of the handle's value type, CSR5_EINVAL if fewer) is OVERWRITTEN WITH
 * MEANINGLESS VALUES.  Works on handles of every variant; col_idx and val must
 * be 16-byte aligned (CSR5_EINVAL otherwise, also for a matrix without a
 * complete tile).  ms is a host array of 2 floats.
 */
int csr5_stream_floor(csr5_handle_t h, void *y, size_t y_bytes, void *hip_stream, int reps, float *ms);

/*
 * CSR row-block baselines on the plain CSR arrays (Section 2.2.1): CSR-scalar is
 * Algorithm 1 with one thread per row; CSR-vector reduces each row with
 * lanes_per_row lanes (2, 4, ..., 64; 0 = smallest power of two >= nnz/m).
 * They exist for the iteration-scenario comparison of Section 5.5 (cost of
 * staying in CSR against converting to CSR5) and do not touch any handle.
 * y double[m] is overwritten.  Asynchronous on the stream.
 */
int csr5_baseline_csr_scalar(int32_t m, const int32_t *row_ptr, const int32_t *col_idx, const double *val,
                             const double *x, double *y, void *hip_stream);
int csr5_baseline_csr_vector(int32_t m, int32_t nnz, const int32_t *row_ptr, const int32_t *col_idx,
                             const double *val, const double *x, double *y, int32_t lanes_per_row,
                             void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CSR5_H */
