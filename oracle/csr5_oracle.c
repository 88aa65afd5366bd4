/*
 * CPU oracle for CSR5 (Liu & Vinter, ICS'15).  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, sequential, obviously-correct C written from the paper's definitions.
 * It exists to check the HIP library: only the tests, the smoke entry and the
 * benchmark's cpu_baseline leg may call it.  It shares no code with the HIP
 * path and is never used to produce a product result.
 *
 * Conventions where the paper leaves a choice open are stated at each function.
 * All of them are pinned by CPU tests against brute force, closed forms and the
 * values the paper's text gives for its 8x8 example (Section 3).
 *
 * Types: indices int32, tile_ptr/tile_desc uint32, values fp64.
 * omega = tile width, sigma = tile height, T = omega*sigma nonzeros per tile,
 * p = ceil(nnz/T) tiles, p_c = floor(nnz/T) complete tiles (Section 3.1, 3.3).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define DIRTY 0x80000000u

/* ------------------------------------------------------------------ */
/* Algorithm 1 (Section 2.2.1): y[i] = sum_j val[j] * x[col_idx[j]],    */
/* one row after the other, entries in CSR order, empty row -> 0.       */
/* abs_sum[i] = sum_j |val[j] * x[col_idx[j]]| feeds the tolerance.     */
/* ------------------------------------------------------------------ */
void oracle_csr_spmv(int32_t m, const int32_t *row_ptr, const int32_t *col_idx,
                     const double *val, const double *x, double *y, double *abs_sum)
{
    for (int32_t i = 0; i < m; i++) {
        double acc = 0.0, mag = 0.0;
        for (int32_t j = row_ptr[i]; j < row_ptr[i + 1]; j++) {
            double prod = val[j] * x[col_idx[j]];
            acc = acc + prod;
            mag = mag + (prod < 0 ? -prod : prod);
        }
        y[i] = acc;
        if (abs_sum) abs_sum[i] = mag;
    }
}

/* The same rows by the same loop, rows shared among the host's cores (each row is
 * still summed sequentially in CSR order, so the result is bit-identical to
 * oracle_csr_spmv).  Exists for the benchmark's all-cores CPU figure only.
 * Returns the number of threads that took part. */
#ifdef _OPENMP
#include <omp.h>
#endif
int32_t oracle_csr_spmv_all_cores(int32_t m, const int32_t *row_ptr, const int32_t *col_idx,
                                  const double *val, const double *x, double *y, double *abs_sum)
{
    int32_t threads = 1;
#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        threads = omp_get_num_threads();
#endif
#pragma omp for schedule(dynamic, 1024)
        for (int32_t i = 0; i < m; i++)
            oracle_csr_spmv(1, row_ptr + i, col_idx, val, x, y + i, abs_sum ? abs_sum + i : 0);
    }
    return threads;
}

/* The "binary_search" of Algorithms 4 and 7 is not defined in the paper.  With
 * empty rows several row_ptr entries are equal, so it is read as an upper
 * bound: the number of entries of row_ptr[0..m] that are <= key.  Minus one,
 * that is the last row r with row_ptr[r] <= key: the non-empty row that owns
 * nonzero `key` when key < nnz, and m when key >= nnz.                      */
static int64_t count_le(const int32_t *row_ptr, int32_t m, int64_t key)
{
    int64_t lo = 0, hi = (int64_t)m + 1;           /* answer in [lo, hi] */
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if ((int64_t)row_ptr[mid] <= key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

/* number of tiles and of complete tiles */
int64_t oracle_num_tiles(int64_t nnz, int32_t omega, int32_t sigma)
{
    int64_t T = (int64_t)omega * sigma;
    return (nnz + T - 1) / T;
}
int64_t oracle_num_complete_tiles(int64_t nnz, int32_t omega, int32_t sigma)
{
    return nnz / ((int64_t)omega * sigma);
}

/* ------------------------------------------------------------------ */
/* Algorithm 4 (Section 3.3): tile_ptr[0..p].                           */
/* First loop: row of the first nonzero of every tile.  Second loop:    */
/* tile tid is flagged (top bit, so that "-0" exists) when some row in  */
/* the inclusive range tile_ptr[tid] .. tile_ptr[tid+1] is empty.  The  */
/* printed loop reads row_ptr[rid+1] at rid = m for the last tile; the  */
/* range is clamped to rid <= m-1.  tile_ptr[p] never carries the flag. */
/* ------------------------------------------------------------------ */
void oracle_tile_ptr(int32_t m, int32_t nnz, const int32_t *row_ptr,
                     int32_t omega, int32_t sigma, uint32_t *tile_ptr)
{
    int64_t T = (int64_t)omega * sigma;
    int64_t p = oracle_num_tiles(nnz, omega, sigma);
    for (int64_t tid = 0; tid <= p; tid++) {
        int64_t bnd = tid * T;
        tile_ptr[tid] = (uint32_t)(count_le(row_ptr, m, bnd) - 1);
    }
    for (int64_t tid = 0; tid < p; tid++) {
        int64_t first = tile_ptr[tid] & ~DIRTY;
        int64_t last = tile_ptr[tid + 1] & ~DIRTY;
        if (last > (int64_t)m - 1) last = (int64_t)m - 1;
        for (int64_t rid = first; rid <= last; rid++) {
            if (row_ptr[rid] == row_ptr[rid + 1]) {
                tile_ptr[tid] |= DIRTY;
                break;
            }
        }
    }
}

/* ------------------------------------------------------------------ */
/* Section 3.4, first part: bit_flag for the complete tiles.            */
/* Built as in Algorithm 3 step 1 (flag[row_ptr[i]] = TRUE for every    */
/* row; an empty row re-flags the position its right neighbour owns, or */
/* nnz itself, which is outside), then read out column-major: flag j of */
/* column i of tile tid is the CSR position tid*T + i*sigma + j.  The   */
/* first flag of every tile is forced TRUE.                             */
/* Output: bit_flag[(tid*omega + i)*sigma + j] as bytes 0/1.            */
/* ------------------------------------------------------------------ */
void oracle_bit_flag(int32_t m, int32_t nnz, const int32_t *row_ptr,
                     int32_t omega, int32_t sigma, uint8_t *bit_flag)
{
    int64_t T = (int64_t)omega * sigma;
    int64_t pc = oracle_num_complete_tiles(nnz, omega, sigma);
    uint8_t *flat = (uint8_t *)calloc((size_t)nnz + 1, 1);
    for (int32_t i = 0; i < m; i++)
        flat[row_ptr[i]] = 1;                 /* row_ptr[i] == nnz lands on the spare slot */
    for (int64_t tid = 0; tid < pc; tid++)
        for (int32_t i = 0; i < omega; i++)
            for (int32_t j = 0; j < sigma; j++)
                bit_flag[(tid * omega + i) * sigma + j] = flat[tid * T + (int64_t)i * sigma + j];
    for (int64_t tid = 0; tid < pc; tid++)
        bit_flag[tid * omega * sigma] = 1;
    free(flat);
}

/* ------------------------------------------------------------------ */
/* y_offset and seg_offset of every complete tile, from what Section    */
/* 3.4 says they mean (Algorithm 5 computes the same two arrays with a  */
/* prefix sum and a segmented sum):                                     */
/*   y_offset[i]   = number of TRUE flags in the tile's columns before  */
/*                   column i (the forced first flag counts): the       */
/*                   segment, counted from the tile's first row, that   */
/*                   the first flag of column i opens;                  */
/*   seg_offset[i] = for a column that holds a TRUE flag, how many      */
/*                   columns directly to its right hold none (their     */
/*                   partial sums belong to this column's last          */
/*                   segment); 0 for a column without a flag.           */
/* Outputs are [pc][omega] int32.                                       */
/* ------------------------------------------------------------------ */
void oracle_y_seg_offset(int64_t pc, int32_t omega, int32_t sigma, const uint8_t *bit_flag,
                         int32_t *y_offset, int32_t *seg_offset)
{
    uint8_t *has_flag = (uint8_t *)malloc((size_t)omega);
    for (int64_t tid = 0; tid < pc; tid++) {
        const uint8_t *tile_flags = bit_flag + tid * omega * sigma;
        int32_t flags_before = 0;
        for (int32_t col = 0; col < omega; col++) {
            int32_t here = 0;
            for (int32_t j = 0; j < sigma; j++) here += tile_flags[col * sigma + j];
            y_offset[tid * omega + col] = flags_before;
            flags_before += here;
            has_flag[col] = (uint8_t)(here > 0);
        }
        for (int32_t col = 0; col < omega; col++) {
            int32_t empty_to_the_right = 0;
            if (has_flag[col])
                for (int32_t nb = col + 1; nb < omega && !has_flag[nb]; nb++) empty_to_the_right++;
            seg_offset[tid * omega + col] = empty_to_the_right;
        }
    }
    free(has_flag);
}

/* ceil(log2(v)) for v >= 1 */
static int32_t ceil_log2(int64_t v)
{
    int32_t b = 0;
    while (((int64_t)1 << b) < v) b++;
    return b;
}

int32_t oracle_desc_bits(int32_t omega, int32_t sigma)
{
    /* Section 3.5: sigma flag bits + ceil(log2 omega) + ceil(log2(omega*sigma)) */
    return sigma + ceil_log2(omega) + ceil_log2((int64_t)omega * sigma);
}
int32_t oracle_desc_words(int32_t omega, int32_t sigma)
{
    return (oracle_desc_bits(omega, sigma) + 31) / 32;
}

static void put_bits(uint32_t *words, int32_t pos, int32_t nbits, uint64_t value)
{
    for (int32_t b = 0; b < nbits; b++)
        if ((value >> b) & 1u)
            words[(pos + b) / 32] |= (uint32_t)1 << ((pos + b) % 32);
}

/* ------------------------------------------------------------------ */
/* Section 3.5: one bit-field per tile column.  The paper fixes the     */
/* three fields and their widths, not their order.  Layout used here:   */
/* bits [0, sigma) = bit_flag (bit j = row j of the column), then       */
/* seg_offset (ceil(log2 omega) bits), then y_offset                    */
/* (ceil(log2(omega*sigma)) bits), as a little-endian number of         */
/* W = ceil(bits/32) words; word k of column i of tile tid is stored at */
/* tile_desc[(tid*W + k)*omega + i] so that a SIMD unit reads word k of */
/* all its columns contiguously.  Unused high bits are zero.            */
/* ------------------------------------------------------------------ */
void oracle_pack_desc(int64_t pc, int32_t omega, int32_t sigma, const uint8_t *bit_flag,
                      const int32_t *y_offset, const int32_t *seg_offset, uint32_t *tile_desc)
{
    int32_t sbits = ceil_log2(omega);
    int32_t ybits = ceil_log2((int64_t)omega * sigma);
    int32_t W = oracle_desc_words(omega, sigma);
    uint32_t words[8];
    for (int64_t tid = 0; tid < pc; tid++) {
        for (int32_t i = 0; i < omega; i++) {
            memset(words, 0, sizeof words);
            for (int32_t j = 0; j < sigma; j++)
                put_bits(words, j, 1, bit_flag[(tid * omega + i) * sigma + j]);
            put_bits(words, sigma, sbits, (uint64_t)seg_offset[tid * omega + i]);
            put_bits(words, sigma + sbits, ybits, (uint64_t)y_offset[tid * omega + i]);
            for (int32_t k = 0; k < W; k++)
                tile_desc[(tid * W + k) * omega + i] = words[k];
        }
    }
}

/* ------------------------------------------------------------------ */
/* empty_offset (Section 3.4; Algorithm 7 builds the same array with a  */
/* binary search per flag).  In a tile that holds an empty row, segment */
/* number s no longer is row tile_ptr + s, so the format stores, for    */
/* every TRUE flag of such a tile in CSR order, which row the flagged   */
/* nonzero belongs to, relative to the tile's first row.  The owner of  */
/* nonzero q is the row r with row_ptr[r] <= q < row_ptr[r+1]; flags    */
/* are visited in increasing q, so one row cursor that only moves       */
/* forward finds them all.  The per-tile arrays are concatenated;       */
/* empty_offset_ptr[tid] (exclusive prefix sum of the per-tile lengths, */
/* 0 for tiles without an empty row, int32[pc+1]) says where tile tid's */
/* entries start -- the paper does not say how they are laid out.       */
/* Call with empty_offset == NULL to get only empty_offset_ptr.         */
/* ------------------------------------------------------------------ */
void oracle_empty_offset(int32_t m, int32_t nnz, const int32_t *row_ptr, int32_t omega,
                         int32_t sigma, const uint32_t *tile_ptr, const uint8_t *bit_flag,
                         int32_t *empty_offset_ptr, int32_t *empty_offset)
{
    int64_t T = (int64_t)omega * sigma;
    int64_t pc = oracle_num_complete_tiles(nnz, omega, sigma);
    int32_t written = 0;
    int32_t owner = 0;                         /* row cursor, never moves back */
    (void)m;
    for (int64_t tid = 0; tid < pc; tid++) {
        empty_offset_ptr[tid] = written;
        if (!(tile_ptr[tid] & DIRTY)) continue;
        int32_t first_row = (int32_t)(tile_ptr[tid] & ~DIRTY);
        for (int64_t q = tid * T; q < (tid + 1) * T; q++) {      /* CSR order = bit_flag's order */
            if (!bit_flag[q]) continue;
            if (empty_offset) {
                while (row_ptr[owner + 1] <= q) owner++;         /* q < nnz = row_ptr[m]: stops at a row < m */
                empty_offset[written] = owner - first_row;
            }
            written++;
        }
    }
    empty_offset_ptr[pc] = written;
}

/* ------------------------------------------------------------------ */
/* Section 3.1: col_idx and val of every complete tile go from          */
/* row-major (CSR order: column i holds CSR offsets i*sigma..+sigma-1)  */
/* to column-major, the order Algorithm 8 reads: entry (i, j) at        */
/* tid*T + j*omega + i.  The incomplete last tile is left untouched.    */
/* Out of place here; the product does it in place.                     */
/* ------------------------------------------------------------------ */
void oracle_transpose(int32_t nnz, int32_t omega, int32_t sigma, const int32_t *col_in,
                      const double *val_in, int32_t *col_out, double *val_out)
{
    int64_t T = (int64_t)omega * sigma;
    int64_t pc = oracle_num_complete_tiles(nnz, omega, sigma);
    for (int64_t tid = 0; tid < pc; tid++)
        for (int32_t i = 0; i < omega; i++)
            for (int32_t j = 0; j < sigma; j++) {
                col_out[tid * T + (int64_t)j * omega + i] = col_in[tid * T + (int64_t)i * sigma + j];
                val_out[tid * T + (int64_t)j * omega + i] = val_in[tid * T + (int64_t)i * sigma + j];
            }
    for (int64_t k = pc * T; k < nnz; k++) {
        col_out[k] = col_in[k];
        val_out[k] = val_in[k];
    }
}

/* ------------------------------------------------------------------ */
/* Section 3.2: sigma from nnz/row with the four hardware constants.    */
/* nnz/row is taken as the integer quotient; an empty matrix gives r.   */
/* ------------------------------------------------------------------ */
int32_t oracle_sigma_rule(int64_t nnz, int64_t m, int32_t r, int32_t s, int32_t t, int32_t u)
{
    if (m <= 0 || nnz <= 0) return r;
    int64_t q = nnz / m;
    if (q <= r) return r;
    if (q <= s) return (int32_t)q;
    if (q <= t) return s;
    return u;
}

/* Algorithm 6: fast segmented sum through an inclusive prefix-sum scan. */
static void fast_segmented_sum(double *in, const int32_t *seg_offset, int32_t length, double *tmp)
{
    memcpy(tmp, in, (size_t)length * sizeof(double));
    for (int32_t i = 1; i < length; i++) in[i] = in[i - 1] + in[i];    /* inclusive scan */
    for (int32_t i = 0; i < length; i++)
        in[i] = in[i + seg_offset[i]] - in[i] + tmp[i];
    /* the loop above runs left to right and reads in[i + seg_offset[i]] with
       seg_offset >= 0, i.e. entries not yet overwritten, except in[i] itself */
}

/* ------------------------------------------------------------------ */
/* Algorithm 8 + Section 4 text: SpMV on the CSR5 arrays, tile by tile, */
/* sequentially; y is zeroed first and every store is an addition, so   */
/* the "atomic add" of the first/last segment is just "+=".  This is a  */
/* check that the descriptors suffice to compute y; the reference value */
/* for y is Algorithm 1 above.                                          */
/*                                                                      */
/* Per column i: walk the sigma entries; a TRUE flag closes what came   */
/* before it: nothing (flag in row 0), a red sub-segment if it is the   */
/* column's first flag (handed to slot i-1 of tmp), else a green        */
/* segment (stored directly, column's segment counter advances).  What  */
/* follows the last flag is the blue sub-segment; a column without any  */
/* flag is entirely red.  Column i's last segment then receives blue[i] */
/* plus the fast segmented sum of tmp at i.  A column without flags     */
/* stores nothing.  Segment number s of a tile maps to row              */
/* tile_ptr + s, or tile_ptr + empty_offset[s] in a dirty tile.         */
/* The nonzeros after the last complete tile are added row by row.      */
/* ------------------------------------------------------------------ */
void oracle_csr5_spmv(int32_t m, int32_t nnz, const int32_t *row_ptr, int32_t omega,
                      int32_t sigma, const uint32_t *tile_ptr, const uint32_t *tile_desc,
                      const int32_t *empty_offset_ptr, const int32_t *empty_offset,
                      const int32_t *col_t, const double *val_t, const double *x, double *y)
{
    int64_t T = (int64_t)omega * sigma;
    int64_t pc = oracle_num_complete_tiles(nnz, omega, sigma);
    int32_t sbits = ceil_log2(omega);
    int32_t ybits = ceil_log2((int64_t)omega * sigma);
    int32_t W = oracle_desc_words(omega, sigma);
    /* tmp has one guard slot in front: column 0 never hands anything to "slot -1"
       for a well-formed descriptor, but a malformed one must not corrupt memory */
    double *tmp_base = (double *)calloc((size_t)(omega + 2), sizeof(double));
    double *tmp = tmp_base + 1;
    double *scratch = (double *)malloc(sizeof(double) * (size_t)(omega + 1));
    double *last_tmp = (double *)malloc(sizeof(double) * (size_t)omega);
    int32_t *seg_off = (int32_t *)malloc(sizeof(int32_t) * (size_t)omega);
    int32_t *last_seg = (int32_t *)malloc(sizeof(int32_t) * (size_t)omega);
    uint8_t *has_flag = (uint8_t *)malloc((size_t)omega);

    for (int32_t r = 0; r < m; r++) y[r] = 0.0;

    for (int64_t tid = 0; tid < pc; tid++) {
        int64_t row0 = tile_ptr[tid] & ~DIRTY;
        int dirty = (tile_ptr[tid] & DIRTY) != 0;
        const int32_t *eo = dirty ? empty_offset + empty_offset_ptr[tid] : NULL;
        for (int32_t i = 0; i < omega; i++) tmp[i] = 0.0;
        for (int32_t i = 0; i < omega; i++) {
            /* unpack column i */
            uint64_t lo = 0, hi = 0;          /* up to 128 bits */
            for (int32_t k = 0; k < W && k < 4; k++) {
                uint64_t w = tile_desc[(tid * W + k) * omega + i];
                if (k < 2) lo |= w << (32 * k); else hi |= w << (32 * (k - 2));
            }
#define GETBIT(b) ((((b) < 64 ? (lo >> (b)) : (hi >> ((b) - 64))) & 1u))
            int32_t so = 0, yo = 0;
            for (int32_t b = 0; b < sbits; b++) so |= (int32_t)GETBIT(sigma + b) << b;
            for (int32_t b = 0; b < ybits; b++) yo |= (int32_t)GETBIT(sigma + sbits + b) << b;
            seg_off[i] = so;
            double sum = 0.0;
            int seen = 0;
            int32_t seg = yo;
            for (int32_t j = 0; j < sigma; j++) {
                if (GETBIT(j)) {
                    if (seen) {                          /* end of a green segment */
                        int64_t row = row0 + (dirty ? eo[seg] : seg);
                        y[row] += sum;
                        seg = seg + 1;
                    } else if (j > 0) {                  /* end of a red sub-segment */
                        tmp[i - 1] = sum;
                    }
                    sum = 0.0;
                    seen = 1;
                }
                int64_t ptr = tid * T + (int64_t)j * omega + i;
                sum = sum + val_t[ptr] * x[col_t[ptr]];
            }
#undef GETBIT
            has_flag[i] = (uint8_t)seen;
            if (seen) {
                last_tmp[i] = sum;                       /* end of a blue sub-segment */
                last_seg[i] = seg;
            } else {
                last_tmp[i] = 0.0;
                tmp[i - 1] = sum;                        /* whole column is red */
            }
        }
        fast_segmented_sum(tmp, seg_off, omega, scratch);
        for (int32_t i = 0; i < omega; i++) {
            if (!has_flag[i]) continue;
            last_tmp[i] = last_tmp[i] + tmp[i];
            int64_t row = row0 + (dirty ? eo[last_seg[i]] : last_seg[i]);
            y[row] += last_tmp[i];
        }
    }
    /* incomplete last tile: rows from tile_ptr[pc], entries from pc*T (Section 4) */
    if (pc * T < nnz) {
        int64_t first = tile_ptr[pc] & ~DIRTY;
        for (int64_t r = first; r < m; r++) {
            int64_t b = row_ptr[r] > pc * T ? row_ptr[r] : pc * T;
            double sum = 0.0;
            for (int64_t k = b; k < row_ptr[r + 1]; k++) sum = sum + val_t[k] * x[col_t[k]];
            y[r] += sum;
        }
    }
    free(tmp_base); free(scratch); free(last_tmp); free(seg_off); free(last_seg); free(has_flag);
}
