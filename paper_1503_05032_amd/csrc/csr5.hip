// libcsr5: CSR -> CSR5 conversion and CSR5 SpMV for gfx950 (MI355X).
//
// Follows Liu & Vinter, "CSR5: An Efficient Storage Format for Cross-Platform
// Sparse Matrix-Vector Multiplication" (ICS'15): format in Section 3, SpMV in
// Section 4.  omega = 64 = one wavefront per tile, one lane per tile column.
//
// What is different from the paper's own GPU design, and why, is said at each
// kernel.  The C ABI is declared in include/csr5.h.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <new>
#include <type_traits>

#include "csr5.h"

namespace {

constexpr int OMEGA = CSR5_OMEGA;
constexpr int SBITS = 6;  // ceil(log2 omega)
constexpr uint32_t BAD_BITS = CSR5_STATUS_BAD_ROW_PTR | CSR5_STATUS_BAD_COL_IDX;
// Internal status bit (not reported): some COMPLETE tile is marked, so the
// empty_offset layout has to be scanned.  Set by the descriptor step of k_transpose only; the scan
// kernels decide on it, and nothing in their own launches changes it.
constexpr uint32_t STATUS_SCAN_NEEDED = 1u << 16;
// Internal status bit: some tile (the incomplete one included) starts further
// into a row than the look-behind can make up for, so the SpMV sends its
// cross-tile sums through the auxiliary array (see k_spmv and k_tile_ptr).
constexpr uint32_t STATUS_NEEDS_CARRY = 1u << 17;
// Internal status bit: some first tile of a workgroup (or the incomplete tile)
// starts more than LOOK entries into a row: the look-behind of this matrix reads
// the far part of the records too (see below).
constexpr uint32_t STATUS_FAR_HEADS = 1u << 18;
// A tile whose first segment continues a row of the previous tile completes
// that row itself when it can get at the row's head.  The tiles of one
// workgroup of the tile kernel are neighbours and hand the finished head over
// through LDS (any head that began inside the previous tile).  The first tile of
// a workgroup sums the head itself, from a copy of the last LOOK_MAX entries of
// the tile before it that the conversion keeps in CSR order next to the format
// (in the transposed tile they are spread over sigma cache lines each for val
// and col_idx; re-reading them there cost 16 % more memory traffic).  The last
// LOOK = 32 of them are three cache lines, read without first asking how long
// the head is (a dependent load at that point costs more than the lines); the
// LOOK_FAR = 128 before them are read only by a tile whose head is longer than
// LOOK.  One record per workgroup of tiles (tile_group_waves), none for
// sigma < LOOK_MIN_SIGMA, where the matrices are small, nor for
// sigma > LOOK_MAX_SIGMA, where the tile kernel has no registers to spare (those
// matrices always take the auxiliary-array path).
constexpr int LOOK = 32;
constexpr int LOOK_FAR = 128;
constexpr int LOOK_MAX = LOOK + LOOK_FAR;
// Heads longer than LOOK are re-read only in matrices of at most this many
// nonzeros; larger ones take the auxiliary array and its second kernel instead.
// The far part costs the tile kernel 5-8 % on matrices with 64- and 128-entry
// rows, the second kernel about 3 us and a launch: measured at 8 to 60 M
// nonzeros, re-reading wins up to 24 M (5-9 % of the SpMV), is level at 32 M and
// loses beyond (3-5 %).
constexpr int64_t LOOK_FAR_MAX_NNZ = 28 * 1000 * 1000;
// The three instantiations of the tile kernel: cross-tile sums through the
// auxiliary array and a second kernel; by look-behind; through the auxiliary array
// inside the one kernel (see "One-launch form of the auxiliary-array path" below).
constexpr int MODE_CARRY = 0, MODE_LOOK = 1, MODE_ONE = 2;
// The one-launch form saves the second kernel (3 us and a launch) and pays for
// one or two atomics with a return value per group of tiles (0.2-1 ns of kernel
// time each, whenever they are sent).  Measured against the
// two-kernel form: matrices of a few thousand tiles gain 10-20 % whatever their
// rows look like (a dense 2000 x 2000 matrix 14.9 -> 12.0 us); with rows of 701
// or 2000 entries throughout the gain is gone at 6 M nonzeros and turns into a
// loss of 4-13 % at 8-21 M; matrices whose rows are short on average and that
// take this path for a few long rows still gain at 17 M (power-law: 2.7 %) and are
// level at 34 M.  Hence: up to ONE_LAUNCH_ANY_TILES tiles always, up to
// ONE_LAUNCH_MAX_TILES when the average row is shorter than ONE_LAUNCH_SHORT_ROWS.
constexpr int ONE_LAUNCH_ANY_TILES = 6144;
constexpr int ONE_LAUNCH_MAX_TILES = 32768;
constexpr int ONE_LAUNCH_SHORT_ROWS = 64;
constexpr int LOOK_MIN_SIGMA = 8, LOOK_MAX_SIGMA = 32;
constexpr bool look_sigma(int sigma) { return sigma >= LOOK_MIN_SIGMA && sigma <= LOOK_MAX_SIGMA; }
constexpr bool one_launch_fits(int sigma, int64_t tiles) { return look_sigma(sigma) && tiles <= ONE_LAUNCH_MAX_TILES; }
// Tiles (= wavefronts) per workgroup of the tile kernel and of the transposition,
// chosen so the LDS buffer stays under 40 KB.
constexpr int tile_group_waves(int sigma) { return sigma <= 16 ? 4 : (sigma <= 32 ? 2 : 1); }
// One record per group of tiles, holding the last LOOK_MAX entries, in CSR
// order, of the group's last tile (of the last complete tile, for the last
// group).  Near part first: LOOK values (8 bytes each, 4 used in single
// precision) followed by LOOK column indices, contiguous, so that a tile fetches
// it with one run of three cache lines; then the far part, LOOK_FAR values and
// LOOK_FAR column indices (entry j of the far part is entry T - LOOK_MAX + j of
// the tile, entry i of the near part entry T - LOOK + i).  Record of tile t:
// number t / tile_group_waves.  Strides of the two views of the record array
// (last_val points at a record's first byte, last_col at its near indices):
// A matrix too large for far heads (LOOK_FAR_MAX_NNZ) keeps the near part only.
constexpr int NEAR_REC_BYTES = LOOK * 8 + LOOK * 4;
constexpr int LAST_REC_BYTES = LOOK_MAX * 8 + LOOK_MAX * 4;
constexpr int record_bytes(int64_t nnz) { return nnz <= LOOK_FAR_MAX_NNZ ? LAST_REC_BYTES : NEAR_REC_BYTES; }
// where a record's far part begins, counted from last_val / last_col of the record
template <typename VT> constexpr int far_val_at() { return (LOOK * 8 + LOOK * 4) / int(sizeof(VT)); }
constexpr int FAR_COL_AT = (LOOK * 8 + LOOK * 4 + LOOK_FAR * 8 - LOOK * 8) / 4;
constexpr uint32_t STATUS_PUBLIC = 0xffu;
constexpr int NUM_XCD = 8;  // MI355X: 8 accelerator dies, each with its own L2

// sigma rule constants <r, s, t, u> for MI355X (Section 3.2 leaves them to the
// hardware; measured with calibrate.py, see csr5_sigma_auto).  On this GPU the
// best sigma does not depend on nnz/row at all for matrices that fill the chip
// (16 wins by 2-3 % from 1 to 256 nonzeros per row), so r = s = u.
constexpr int RULE_R = 16, RULE_S = 16, RULE_T = 256, RULE_U = 16;
// What does matter is the number of tiles: the chip holds 256 CUs x 16
// wavefronts of this kernel, and below about three rounds of them the ramp-up and
// the last partial round dominate; such a matrix gets the smaller tile.  Placed
// with matrices of 8 and of 27 entries per row at 8 to 40 M nonzeros: at sigma 16
// the 27-per-row ones win from 12 M nonzeros on (7 % at 14 M), the 8-per-row
// ones are within 2 % either way between 12 M and 20 M.
constexpr int64_t RULE_MIN_TILES = 3 * 256 * 16;
constexpr int RULE_SIGMA_SMALL = 8;

// Index width of row_ptr, tile_ptr and empty_offset_ptr.  int32 is the layout the
// paper describes first (tile_ptr: 31-bit row index, top bit = "tile holds an
// empty row"); int64 is its 64-bit variant (Section 3.3: 63-bit index plus the
// flag bit) for matrices of 2^31 nonzeros and more, which this GPU's memory holds
// many times over.  Row and column indices stay below 2^31 in both.
template <typename IT> struct Index;
template <> struct Index<int32_t> {
    using tp_t = uint32_t;
    static constexpr tp_t DIRTY = 0x80000000u, ROWMASK = 0x7fffffffu;
};
template <> struct Index<int64_t> {
    using tp_t = uint64_t;
    static constexpr tp_t DIRTY = 0x8000000000000000ull, ROWMASK = 0x7fffffffffffffffull;
};

inline int ceil_log2_host(int64_t v) {
    int b = 0;
    while ((int64_t(1) << b) < v) b++;
    return b;
}

constexpr int MEET_STRIDE_WORDS = 1;

struct Geom {
    int32_t sigma, T, W, ybits;
    int32_t p, pc;
};

inline Geom make_geom(int64_t nnz, int sigma) {
    Geom g;
    g.sigma = sigma;
    g.T = OMEGA * sigma;
    g.ybits = ceil_log2_host(int64_t(OMEGA) * sigma);
    g.W = (sigma + SBITS + g.ybits + 31) / 32;
    g.p = int32_t((nnz + g.T - 1) / g.T);
    g.pc = int32_t(nnz / g.T);
    return g;
}

inline size_t align256(size_t b) { return (b + 255) & ~size_t(255); }
// one slot of the cross-tile sums of an SpMV: carry, then (one-launch form) the meeting words and the counters
// (meeting words and counters: one per group of tiles, the incomplete tile being a group of its own)
inline size_t tile_groups(const Geom& g, int waves) { return (size_t(g.pc) + waves - 1) / waves + 1; }
inline size_t slot_off_meet(const Geom& g) { return align256((size_t(g.p) + 1) * 8); }
inline size_t slot_off_arrived(const Geom& g, int waves) { return slot_off_meet(g) + align256(tile_groups(g, waves) * 8 * MEET_STRIDE_WORDS); }
inline size_t slot_bytes_one(const Geom& g, int waves) { return slot_off_arrived(g, waves) + align256(tile_groups(g, waves) * 4); }

// ----------------------------------------------------------------------------
// device helpers
// ----------------------------------------------------------------------------

// Number of entries of a[0..len) that are <= key ("upper bound").  This is the
// binary search of Algorithms 4 and 7: with empty rows several row_ptr entries
// are equal, and count-1 is then the non-empty row that owns nonzero `key`.
template <typename IT>
__device__ __forceinline__ int count_le(const IT* __restrict__ a, int len, int64_t key) {
    int lo = 0, hi = len;
    while (lo < hi) {
        int mid = lo + ((hi - lo) >> 1);
        if (int64_t(a[mid]) <= key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (OMEGA - 1); }

// Group of tiles (= workgroup of the tile kernel) that holds a nonzero: tile t of
// the complete tiles belongs to group t / waves, the incomplete tile is a group
// of its own behind them.
__device__ __forceinline__ int tile_group_of(int64_t entry, int T, int pc, int waves) {
    const int64_t t = entry / T;
    return t < int64_t(pc) ? int(t / waves) : (pc + waves - 1) / waves;
}
// "nobody has been here yet" in the meeting words of the one-launch SpMV (a NaN pattern no sum is stored as)
constexpr uint64_t MEET_EMPTY = 0xfff8c5125eaf0001ull;
// Distance, in 8-byte words, between the meeting words of neighbouring groups.
constexpr int MEET_STRIDE = MEET_STRIDE_WORDS;
__device__ __forceinline__ uint64_t* meet_at(uint64_t* meet, uint32_t g) { return meet + size_t(g) * MEET_STRIDE; }

// Sets a bit of the status word.  Hundreds of thousands of threads may want the
// same bit, and atomics on one address are served one after the other, so look
// first: after the first few, everybody finds it set.
__device__ __forceinline__ void raise_status(uint32_t* status, uint32_t bit) {
    if ((__hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bit) != bit) atomicOr(status, bit);
}

// Native global floating-point atomic add (fp64 or fp32), no return value.
template <typename VT>
__device__ __forceinline__ void atomic_add_fp(VT* addr, VT v) {
    __hip_atomic_fetch_add(addr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Which tiles a workgroup takes.  Workgroups are dealt round-robin to the 8
// XCDs (workgroup w runs on XCD w mod 8), each with its own L2.  Three orders,
// chosen per matrix at launch (measured on stencil, power-law and banded random
// matrices from 3 M to 2.2 G nonzeros; the crossovers sat at the same places in
// all families):
//  * contiguous (chunk = 0): XCD k gets the k-th eighth of the tiles, so
//    neighbouring tiles, which gather neighbouring parts of x, share one L2.
//    Wins by 1-14 % while x is at most about 9 MiB, i.e. while the part of x one
//    XCD works on stays in its L2 next to the streamed tiles; beyond that it
//    loses 2-9 %: eight distant streams cost more than a shared sweep.
//  * plain (chunk = 1): workgroup w takes tiles 4w..4w+3; all XCDs sweep the same
//    region, and expensive stretches (a long row's tiles) are spread evenly.
//    But neighbouring tiles then sit on different XCDs, and when a tile holds
//    fewer rows than a cache line of y (16), every line of y is written piecewise
//    from several L2s: 8 % slower on a matrix with 350 nonzeros per row.
//  * chunked (chunk = 16): runs of 16 workgroups go to the XCDs in turn; as good
//    as plain on regular matrices and without its piecewise writes.  Also the
//    choice when x is so small (below 2.5 MB) that it stays in every L2 anyway:
//    1-4 % faster than contiguous there.
constexpr size_t XCD_CONTIGUOUS_MIN_X_BYTES = 2500u * 1000u;
constexpr size_t XCD_CONTIGUOUS_MAX_X_BYTES = 10u * 1000u * 1000u;
constexpr uint32_t XCD_CHUNK = 16;
constexpr int Y_LINE_ROWS = 16;            // 128-byte line / 8-byte value

__device__ __forceinline__ uint32_t xcd_order(uint32_t w, uint32_t nb, uint32_t chunk) {
    const uint32_t xcd = w % NUM_XCD, k = w / NUM_XCD;
    if (chunk == 0) {
        const uint32_t per = nb / NUM_XCD, rem = nb % NUM_XCD;
        return xcd * per + (xcd < rem ? xcd : rem) + k;
    }
    // a permutation of [0, full); the ragged rest keeps the plain order
    const uint32_t full = (nb / (NUM_XCD * chunk)) * (NUM_XCD * chunk);
    if (w >= full) return w;
    return (k / chunk) * (NUM_XCD * chunk) + xcd * chunk + (k % chunk);
}

// ----------------------------------------------------------------------------
// Conversion step 2a: tile_ptr (Algorithm 4, first loop).  One thread per
// tile boundary.  The same launch clears the flag words the next kernel ORs
// into, and the status word, and notes for every tile how many entries of its
// first row lie before it (tile_head, an auxiliary array of the SpMV).
// ----------------------------------------------------------------------------
template <typename IT>
__global__ void __launch_bounds__(256)
k_tile_ptr(int m, const IT* __restrict__ row_ptr, int T, int p, int pc, int group, int record_reach,
           typename Index<IT>::tp_t* __restrict__ tile_ptr, uint32_t* __restrict__ tile_head,
           uint32_t* __restrict__ wg_far, uint32_t* __restrict__ desc, size_t ndesc,
           uint32_t* __restrict__ arrived, uint64_t* __restrict__ meet, size_t slot_bytes, int slots,
           uint2* __restrict__ span, uint32_t* __restrict__ status) {
    using tp_t = typename Index<IT>::tp_t;
    size_t gid = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
    size_t stride = size_t(gridDim.x) * blockDim.x;
    for (size_t k = gid; k < ndesc; k += stride) desc[k] = 0u;
    // the one-launch SpMV finds its counters at zero and its meeting places empty, and leaves them so
    const size_t groups = (size_t(pc) + group - 1) / group + 1;         // one word of each per group of tiles
    for (int slot = 0; slot < slots; slot++) {
        for (size_t t = gid; t < groups; t += stride) arrived[slot * (slot_bytes / 4) + t] = 0u;
        for (size_t w = gid; w < groups * MEET_STRIDE; w += stride) meet[slot * (slot_bytes / 8) + w] = MEET_EMPTY;
    }
    if (gid == 0) *status = 0u;
    int far = 0, far_heads = 0;
    for (size_t t = gid; t <= size_t(p); t += stride) {
        int64_t bnd = int64_t(t) * T;
        const int row = count_le(row_ptr, m + 1, bnd) - 1;
        tile_ptr[t] = tp_t(row) & Index<IT>::ROWMASK;
        // how far into its first row the tile starts (0: the row starts with the
        // tile), saturated at 32 bits: what the SpMV needs to know about the
        // boundary, so that it does not have to look into row_ptr itself
        int64_t head = 0;
        if (t < size_t(p) && row >= 0 && row < m) head = bnd - int64_t(row_ptr[row]);
        tile_head[t] = uint32_t(head < 0 ? 0 : (head > int64_t(0xffffffffu) ? int64_t(0xffffffffu) : head));
        // for the one-launch SpMV: the groups of tiles that row touches (first, how many)
        if (slots > 0) {
            uint2 sp = {0u, 1u};
            if (row >= 0 && row < m) {
                const int64_t rs = int64_t(row_ptr[row]), re = int64_t(row_ptr[row + 1]);
                if (re > rs && rs >= 0) {
                    const int g0 = tile_group_of(rs, T, pc, group), g1 = tile_group_of(re - 1, T, pc, group);
                    if (g1 >= g0) sp = uint2{uint32_t(g0), uint32_t(g1 - g0 + 1)};
                }
            }
            span[t] = sp;
        }
        // Can the tile kernel complete that row on its own?  The first tile of a
        // workgroup (and the workgroup of the incomplete tile) re-reads the head
        // from the previous tile's record: at most record_reach entries (LOOK_MAX,
        // or LOOK in a large matrix, see LOOK_FAR_MAX_NNZ).  The other
        // tiles are handed their neighbour's last segment, which is the whole
        // head if the row began inside (or with) that neighbour: at most T entries.
        const bool from_record = (t % size_t(group)) == 0 || t >= size_t(pc);
        far |= int(head > (from_record ? int64_t(record_reach) : int64_t(T)));
        far_heads |= int(from_record && head > int64_t(LOOK));
    }
    // "Some tile starts too far into a row" (the SpMV then needs its
    // carry array) does not go to the status word from here -- this launch also
    // clears that word, and thousands of workgroups saying so would queue at it --
    // but into one word per workgroup, which the scan kernel collects.
    far = __syncthreads_or(far);
    far_heads = __syncthreads_or(far_heads);
    if (threadIdx.x == 0) wg_far[blockIdx.x] = uint32_t(far != 0) | (uint32_t(far_heads != 0) << 1);   // bit 0, bit 1
}

// What the workgroups of k_tile_ptr (nwg of them) found about the tiles' heads
// (bit 0: some tile starts too far into a row for the tile kernel alone; bit 1:
// some workgroup's first tile starts more than LOOK entries into a row) goes to
// the status word, once.  Every thread of the workgroup must call this.
__device__ __forceinline__ uint32_t any_tile_far(const uint32_t* __restrict__ wg_far, int nwg, uint32_t* status) {
    int far = 0, far_heads = 0;
    for (int w = threadIdx.x; w < nwg; w += blockDim.x) {
        const uint32_t bits = wg_far[w];
        far |= int(bits & 1u);
        far_heads |= int(bits & 2u);
    }
    far = __syncthreads_or(far);
    far_heads = __syncthreads_or(far_heads);
    const uint32_t raise = (far ? STATUS_NEEDS_CARRY : 0u) | (far_heads ? STATUS_FAR_HEADS : 0u);
    if (raise && threadIdx.x == 0) atomicOr(status, raise);
    return raise;
}

// ----------------------------------------------------------------------------
// Conversion steps 2b + 3a, one thread per matrix row (the first workgroup also
// passes on what k_tile_ptr noted about the tiles' heads).
//  * empty row   -> mark the tile whose row range holds it (Algorithm 4, second
//    loop, turned inside out: the printed loop walks each tile's rows, which
//    serialises on a tile that spans millions of empty rows).  An empty row
//    sitting at entry position a lies in the inclusive range
//    [tile_ptr[t], tile_ptr[t+1]] of exactly one tile, the one that holds entry
//    a - 1: tiles that start at or after a begin with a later row, tiles that
//    end before a - 1 end with an earlier one.  Rows before the first nonzero
//    (a = 0) lie in no tile's range.
//  * other rows  -> set the bit_flag of the row's first nonzero (Section 3.4;
//    the scatter of Algorithm 3 step 1) directly inside the packed descriptor.
// Also validates row_ptr.
// ----------------------------------------------------------------------------
template <typename IT>
__global__ void __launch_bounds__(256)
k_rows(int m, IT nnz, const IT* __restrict__ row_ptr, int sigma, int T, int W, int p, int pc,
       typename Index<IT>::tp_t* tile_ptr, uint32_t* desc, const uint32_t* __restrict__ wg_far, int nwg,
       uint32_t* status) {
    using tp_t = typename Index<IT>::tp_t;
    constexpr tp_t DIRTY = Index<IT>::DIRTY;
    // what k_tile_ptr found about the tiles' heads, for the transposition that follows
    if (blockIdx.x == 0) any_tile_far(wg_far, nwg, status);
    const int lane = lane_id();
    const int64_t g = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const bool in = g < int64_t(m);                       // every lane stays for the shuffles below
    const int r = in ? int(g) : 0;
    IT a = 0, b = 0;
    if (in) { a = row_ptr[r]; b = row_ptr[r + 1]; }
    const bool bad = in && ((a < 0) || (b < a) || (b > nnz) || (r == 0 && a != 0) || (r == m - 1 && b != nnz));
    if (bad) raise_status(status, CSR5_STATUS_BAD_ROW_PTR);
    // Empty row: mark its tile.  Neighbouring empty rows aim at the same tile, so
    // only the first lane of such a run goes on, and it looks before the atomic (a
    // tile whose range holds millions of empty rows would otherwise receive
    // millions of atomics on one word).  The status bits that say "some tile is
    // marked" are set once, by the scan that follows; only rows before the first
    // nonzero mark no tile, and row 0 speaks for them.
    const bool empty = in && !bad && a == b;
    if (empty && r == 0) raise_status(status, CSR5_STATUS_HAS_EMPTY_ROWS);
    const bool nonempty = in && !bad && a != b;
    const IT a_tile = nonempty ? IT(a / T) : IT(0);
    const int a_off = nonempty ? int(a - a_tile * T) : 0;
    const int t = (empty && a > 0) ? int((a - 1) / T) : -1 - lane;
    const int tprev = __shfl_up(t, 1, OMEGA);
    if (t >= 0 && t < p && (lane == 0 || tprev != t) &&
        !(__hip_atomic_load(&tile_ptr[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & DIRTY))
        __hip_atomic_fetch_or(&tile_ptr[t], DIRTY, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // The flag of the row's first nonzero.  Short rows put the flags of several
    // consecutive rows, i.e. lanes, into one descriptor word, and atomics on one
    // word are served one after the other (2 M rows of a power-law matrix: 75 us).
    // So the lanes that aim at the same word merge their bits first (the rows are
    // in order, hence those lanes are neighbours) and the last of them issues one OR.
    const bool sets = in && !bad && a != b && int64_t(a) < int64_t(pc) * T;
    uint64_t word = ~uint64_t(lane);                      // no real word index, different in every lane
    uint32_t bits = 0;
    if (sets) {
        const int tile = int(a_tile);
        const int w = a_off;
        const int i = w / sigma;
        const int j = w - i * sigma;
        word = (uint64_t(tile) * W + (j >> 5)) * OMEGA + i;
        bits = 1u << (j & 31);
    }
#pragma unroll
    for (int d = 1; d < OMEGA; d <<= 1) {
        const uint32_t up = __shfl_up(bits, d, OMEGA);
        const uint64_t wup = __shfl_up(word, d, OMEGA);
        if (lane >= d && wup == word) bits |= up;
    }
    const uint64_t wnext = __shfl_down(word, 1, OMEGA);
    if (sets && (lane == OMEGA - 1 || wnext != word)) atomicOr(&desc[word], bits);
}


// ----------------------------------------------------------------------------
// empty_offset layout: exclusive prefix sum of the per-tile segment counts
// (non-zero only for tiles with an empty row); the array has p_c + 1 entries.
// Nothing to scan when no tile is marked (status bit from the descriptor step of k_transpose).  Up to
// SCAN_SINGLE tiles one workgroup walks the array chunk by chunk; beyond that
// every chunk gets a workgroup (local scan + chunk total) and a second launch
// adds to every chunk the sum of the totals before it.
// ----------------------------------------------------------------------------
constexpr uint32_t MAX_TILE_PTR_WG = 8192;     // workgroups of k_tile_ptr
constexpr uint32_t CARRY_SLOTS = 4;            // carry arrays per handle = SpMVs of one handle that may overlap
constexpr int SCAN_THREADS = 1024, SCAN_ITEMS = 8, SCAN_CHUNK = SCAN_THREADS * SCAN_ITEMS;
constexpr int SCAN_SINGLE = 4 * SCAN_CHUNK;

// Exclusive scan of a[base .. base + SCAN_CHUNK) (entries at or beyond len count
// as 0) by one workgroup of SCAN_THREADS threads, in place, plus `carry`;
// returns the chunk's total to every thread.
template <typename IT>
__device__ IT scan_chunk(IT* __restrict__ a, int64_t base, int64_t len, IT carry) {
    __shared__ IT wave_sum[SCAN_THREADS / OMEGA];
    __shared__ IT chunk_total;
    const int lane = lane_id(), wave = threadIdx.x / OMEGA;
    const int64_t idx0 = base + int64_t(threadIdx.x) * SCAN_ITEMS;
    IT local[SCAN_ITEMS];
    IT s = 0;
#pragma unroll
    for (int q = 0; q < SCAN_ITEMS; q++) {
        IT v = (idx0 + q < len) ? a[idx0 + q] : IT(0);
        local[q] = s;
        s += v;
    }
    IT incl = s;
#pragma unroll
    for (int d = 1; d < OMEGA; d <<= 1) {
        IT up = __shfl_up(incl, d, OMEGA);
        if (lane >= d) incl += up;
    }
    if (lane == OMEGA - 1) wave_sum[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        IT v = (lane < SCAN_THREADS / OMEGA) ? wave_sum[lane] : IT(0);
        IT ws = v;
#pragma unroll
        for (int d = 1; d < SCAN_THREADS / OMEGA; d <<= 1) {
            IT up = __shfl_up(ws, d, OMEGA);
            if (lane >= d) ws += up;
        }
        if (lane < SCAN_THREADS / OMEGA) wave_sum[lane] = ws - v;  // exclusive
        if (lane == SCAN_THREADS / OMEGA - 1) chunk_total = ws;
    }
    __syncthreads();
    const IT excl = carry + wave_sum[wave] + incl - s;
#pragma unroll
    for (int q = 0; q < SCAN_ITEMS; q++)
        if (idx0 + q < len) a[idx0 + q] = excl + local[q];
    const IT total = chunk_total;
    __syncthreads();                                    // the shared words are reused by the next call
    return total;
}

// The last words of the scan: the total number of entries, and the status bits
// for a marked incomplete tile (it has no descriptor, so the descriptor step never sees
// it).  One thread.
template <typename IT>
__device__ __forceinline__ void scan_epilogue(int pc, int p, IT total, IT* __restrict__ eop,
                                              const typename Index<IT>::tp_t* __restrict__ tile_ptr,
                                              uint32_t* __restrict__ status) {
    eop[pc] = total;
    if (p > pc && (tile_ptr[pc] & Index<IT>::DIRTY))
        atomicOr(status, CSR5_STATUS_HAS_DIRTY | CSR5_STATUS_HAS_EMPTY_ROWS);
}

template <typename IT>
__global__ void __launch_bounds__(SCAN_THREADS)
k_scan_eop(int pc, int p, IT* __restrict__ eop, const typename Index<IT>::tp_t* __restrict__ tile_ptr,
           uint32_t* __restrict__ status) {
    IT total = 0;
    if (*status & STATUS_SCAN_NEEDED)
        for (int64_t base = 0; base < pc; base += SCAN_CHUNK) total += scan_chunk(eop, base, int64_t(pc), total);
    if (threadIdx.x == 0) scan_epilogue(pc, p, total, eop, tile_ptr, status);
}

// more than SCAN_SINGLE tiles, step 1: workgroup b scans chunk b on its own
template <typename IT>
__global__ void __launch_bounds__(SCAN_THREADS)
k_scan_chunks(int pc, IT* __restrict__ eop, IT* __restrict__ chunk_sum, const uint32_t* __restrict__ status) {
    if (!(*status & STATUS_SCAN_NEEDED)) return;
    const IT total = scan_chunk(eop, int64_t(blockIdx.x) * SCAN_CHUNK, int64_t(pc), IT(0));
    if (threadIdx.x == 0) chunk_sum[blockIdx.x] = total;
}

// step 2: workgroup b sums the totals of the chunks before its own (at most
// SCAN_CHUNK of them) and adds that to its chunk; the last one finishes the array
template <typename IT>
__global__ void __launch_bounds__(SCAN_THREADS)
k_scan_finish(int pc, int p, IT* __restrict__ eop, const IT* __restrict__ chunk_sum,
              const typename Index<IT>::tp_t* __restrict__ tile_ptr, uint32_t* __restrict__ status) {
    const int b = blockIdx.x, last = int(gridDim.x) - 1;
    if (!(*status & STATUS_SCAN_NEEDED)) {
        if (b == last && threadIdx.x == 0) scan_epilogue(pc, p, IT(0), eop, tile_ptr, status);
        return;
    }
    __shared__ IT wave_part[SCAN_THREADS / OMEGA];
    __shared__ IT before;
    const int lane = lane_id(), wave = threadIdx.x / OMEGA;
    IT part = 0;
    for (int c = threadIdx.x; c < b; c += SCAN_THREADS) part += chunk_sum[c];
#pragma unroll
    for (int d = OMEGA / 2; d >= 1; d >>= 1) part += __shfl_down(part, d, OMEGA);
    if (lane == 0) wave_part[wave] = part;
    __syncthreads();
    if (threadIdx.x == 0) {
        IT sum = 0;
        for (int k = 0; k < SCAN_THREADS / OMEGA; k++) sum += wave_part[k];
        before = sum;
    }
    __syncthreads();
    const IT offset = before;
    if (offset != 0) {
        const int64_t i0 = int64_t(b) * SCAN_CHUNK + int64_t(threadIdx.x) * SCAN_ITEMS;
#pragma unroll
        for (int q = 0; q < SCAN_ITEMS; q++)
            if (i0 + q < pc) eop[i0 + q] += offset;
    }
    if (b == last && threadIdx.x == 0) scan_epilogue(pc, p, IT(offset + chunk_sum[b]), eop, tile_ptr, status);
}

// ----------------------------------------------------------------------------
// empty_offset values (Algorithm 7), one thread per matrix row instead of one
// sequential walk per tile: a non-empty row whose first nonzero lies in a
// marked complete tile is segment number  y_offset[column] + (flags below it in
// the column)  of that tile, and its entry is  row - tile_ptr.  Segment 0 of a
// marked tile may start with the forced flag (a row continued from the previous
// tile, which is then the tile's first row): its entry is 0 and is written by
// the extra p_c threads at the end of the grid.
// ----------------------------------------------------------------------------
template <typename IT>
__global__ void __launch_bounds__(256)
k_empty_offset(int m, const IT* __restrict__ row_ptr, int sigma, int T, int W, int pc,
               const typename Index<IT>::tp_t* __restrict__ tile_ptr, const uint32_t* __restrict__ desc,
               const IT* __restrict__ eop, int32_t* __restrict__ eo,
               const uint32_t* __restrict__ status) {
    using tp_t = typename Index<IT>::tp_t;
    constexpr tp_t DIRTY = Index<IT>::DIRTY, ROWMASK = Index<IT>::ROWMASK;
    uint32_t st = *status;
    if (!(st & CSR5_STATUS_HAS_DIRTY) || (st & BAD_BITS)) return;
    int64_t g = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (g >= int64_t(m)) {
        int64_t t = g - m;
        if (t < pc && (tile_ptr[t] & DIRTY)) eo[eop[t]] = 0;
        return;
    }
    int r = int(g);
    IT a = row_ptr[r], b = row_ptr[r + 1];
    if (a == b || int64_t(a) >= int64_t(pc) * T) return;
    int tile = int(a / T);
    tp_t tp = tile_ptr[tile];
    if (!(tp & DIRTY)) return;
    int w = int(a - IT(tile) * T);
    int i = w / sigma;
    int j = w - i * sigma;
    size_t base = size_t(tile) * W * OMEGA + i;
    uint64_t lo = desc[base];
    if (W > 1) lo |= uint64_t(desc[base + OMEGA]) << 32;
    uint64_t hi = (W > 2) ? desc[base + 2 * OMEGA] : 0u;
    int ysh = sigma + SBITS;
    uint64_t yo = lo >> ysh;
    if (W > 2) yo |= hi << (64 - ysh);
    // y_offset occupies every bit above seg_offset (unused high bits are zero)
    uint64_t below = lo & ((uint64_t(1) << j) - 1);
    int seg = int(yo) + __popcll(below);
    eo[eop[tile] + seg] = int32_t(int64_t(r) - int64_t(tp & ROWMASK));
}

// ----------------------------------------------------------------------------
// Conversion step 4 (Section 3.1): in-place transposition of col_idx and val
// inside every complete tile, one wavefront per tile.  The tile is read in CSR
// order (lane-contiguous), parked in LDS, and written back column-major
// (lane-contiguous again), so both HBM directions are fully coalesced and each
// lane happens to write exactly the addresses it read.  LDS rows are padded to
// an odd pitch to avoid bank conflicts on the strided LDS read.  BACK = the
// inverse permutation (CSR5 -> CSR, Section 3.6).  The last block also checks
// the column indices of the incomplete tile.  The forward pass also keeps, per
// workgroup, a copy of its last tile's last LOOK entries in CSR order when asked to.
// ----------------------------------------------------------------------------
template <int SIGMA>
struct TransposeShape {
    static constexpr int WAVES = tile_group_waves(SIGMA);
    static constexpr int PITCH = SIGMA | 1;
};

// Orders LDS traffic between the lanes of ONE wavefront: LDS instructions of a
// wavefront execute in order, so what is needed is that the compiler keeps the
// stores before and the loads after this point.
__device__ __forceinline__ void wave_sync_lds() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int SIGMA, bool BACK, typename VT>
__global__ void __launch_bounds__(TransposeShape<SIGMA>::WAVES * OMEGA)
k_transpose(int pc, int n, int64_t nnz, int32_t* __restrict__ col_idx, VT* __restrict__ val,
            uint32_t* __restrict__ status, int32_t* __restrict__ last_col, VT* __restrict__ last_val, int rec_bytes,
            const void* __restrict__ tile_ptr, uint32_t* __restrict__ desc, void* __restrict__ eop, int wide) {
    constexpr int T = OMEGA * SIGMA;
    constexpr int YBITS = 32 - __builtin_clz(uint32_t(T - 1));        // ceil(log2(64*sigma))
    constexpr int W = (SIGMA + SBITS + YBITS + 31) / 32;
    constexpr int PITCH = TransposeShape<SIGMA>::PITCH;
    constexpr int WAVES = TransposeShape<SIGMA>::WAVES;
    __shared__ double lds[WAVES][OMEGA * PITCH];
    const int wave = threadIdx.x / OMEGA, lane = lane_id();
    const int tile = blockIdx.x * WAVES + wave;
    const bool active = tile < pc;                 // uniform per wavefront
    const size_t base = size_t(active ? tile : 0) * T;
    VT* buf = reinterpret_cast<VT*>(lds[wave]);
    int32_t* ibuf = reinterpret_cast<int32_t*>(lds[wave]);
    bool bad = false;
    // The copy of the tile's last entries is for the SpMV's look-behind, which a
    // matrix with a tile far into a row never uses (the scan kernel has said so by now).
    // Only a group's last tile is looked at from outside its workgroup; the last
    // complete tile also by the workgroup of the incomplete one.
    const uint32_t st_heads = *status;
    const bool keep_last = !BACK && last_val && last_col && !(st_heads & STATUS_NEEDS_CARRY) &&
                           (wave == WAVES - 1 || tile == pc - 1);
    const bool keep_far = keep_last && (st_heads & STATUS_FAR_HEADS) && rec_bytes == LAST_REC_BYTES;   // nobody reads the far part otherwise
    const size_t rec = size_t(tile) / WAVES;

    // ---- conversion step 3b rides along (forward pass): the tile's flag words,
    // as k_rows left them, are asked for now and turned into descriptors below
    uint64_t flags = 0;
    bool marked = false;
    const size_t dbase = size_t(active ? tile : 0) * W * OMEGA + lane;
    if constexpr (!BACK) {
        if (active && desc) {
            flags = desc[dbase];
            if (SIGMA > 32) flags |= uint64_t(desc[dbase + OMEGA]) << 32;
            marked = wide ? (static_cast<const uint64_t*>(tile_ptr)[tile] >> 63) != 0
                          : (static_cast<const uint32_t*>(tile_ptr)[tile] >> 31) != 0;
        }
    }

    // ---- val: HBM -> registers -> LDS -> registers -> HBM
    VT v[SIGMA];
    if (active) {
#pragma unroll
        for (int k = 0; k < SIGMA; k++) v[k] = __builtin_nontemporal_load(&val[base + k * OMEGA + lane]);
        // the tile's last LOOK_MAX entries, still in CSR order (entry k*64 + lane of
        // the tile is v[k] here), for the SpMV's look-behind: near part, far part
        if constexpr (!BACK && look_sigma(SIGMA)) {
            if (keep_last) {
                VT* const near_v = last_val + rec * size_t(rec_bytes / int(sizeof(VT)));
                VT* const far_v = near_v + far_val_at<VT>();
                if (lane >= OMEGA - LOOK) near_v[lane - (OMEGA - LOOK)] = v[SIGMA - 1];
                if (keep_far) {
                    if (lane >= OMEGA - LOOK) far_v[lane - (OMEGA - LOOK)] = v[SIGMA - 3];
                    else far_v[LOOK_FAR - LOOK + lane] = v[SIGMA - 1];
                    far_v[LOOK + lane] = v[SIGMA - 2];
                }
            }
        }
        if (!BACK) {
#pragma unroll
            for (int k = 0; k < SIGMA; k++) {
                int e = k * OMEGA + lane;          // CSR offset inside the tile
                buf[(e / SIGMA) * PITCH + (e % SIGMA)] = v[k];
            }
        } else {
#pragma unroll
            for (int j = 0; j < SIGMA; j++) buf[lane * PITCH + j] = v[j];
        }
    }
    wave_sync_lds();    // every wavefront works in its own LDS slice
    if (active) {
        if (!BACK) {
#pragma unroll
            for (int j = 0; j < SIGMA; j++) v[j] = buf[lane * PITCH + j];
        } else {
#pragma unroll
            for (int k = 0; k < SIGMA; k++) {
                int e = k * OMEGA + lane;
                v[k] = buf[(e / SIGMA) * PITCH + (e % SIGMA)];
            }
        }
#pragma unroll
        for (int k = 0; k < SIGMA; k++) __builtin_nontemporal_store(v[k], &val[base + k * OMEGA + lane]);
    }
    wave_sync_lds();    // every wavefront works in its own LDS slice
    // ---- col_idx, same path through the same LDS buffer
    int32_t c[SIGMA];
    if (active) {
#pragma unroll
        for (int k = 0; k < SIGMA; k++) {
            c[k] = __builtin_nontemporal_load(&col_idx[base + k * OMEGA + lane]);
            bad |= (c[k] < 0) | (c[k] >= n);
        }
        if constexpr (!BACK && look_sigma(SIGMA)) {
            if (keep_last) {
                int32_t* const near_c = last_col + rec * size_t(rec_bytes / 4);
                int32_t* const far_c = near_c + FAR_COL_AT;
                if (lane >= OMEGA - LOOK) near_c[lane - (OMEGA - LOOK)] = c[SIGMA - 1];
                if (keep_far) {
                    if (lane >= OMEGA - LOOK) far_c[lane - (OMEGA - LOOK)] = c[SIGMA - 3];
                    else far_c[LOOK_FAR - LOOK + lane] = c[SIGMA - 1];
                    far_c[LOOK + lane] = c[SIGMA - 2];
                }
            }
        }
        if (!BACK) {
#pragma unroll
            for (int k = 0; k < SIGMA; k++) {
                int e = k * OMEGA + lane;
                ibuf[(e / SIGMA) * PITCH + (e % SIGMA)] = c[k];
            }
        } else {
#pragma unroll
            for (int j = 0; j < SIGMA; j++) ibuf[lane * PITCH + j] = c[j];
        }
    }
    wave_sync_lds();    // every wavefront works in its own LDS slice
    if (active) {
        if (!BACK) {
#pragma unroll
            for (int j = 0; j < SIGMA; j++) c[j] = ibuf[lane * PITCH + j];
        } else {
#pragma unroll
            for (int k = 0; k < SIGMA; k++) {
                int e = k * OMEGA + lane;
                c[k] = ibuf[(e / SIGMA) * PITCH + (e % SIGMA)];
            }
        }
#pragma unroll
        for (int k = 0; k < SIGMA; k++) __builtin_nontemporal_store(c[k], &col_idx[base + k * OMEGA + lane]);
    }
    if (!BACK && blockIdx.x == gridDim.x - 1) {
        for (size_t e = size_t(pc) * T + threadIdx.x; e < size_t(nnz); e += blockDim.x) {
            int32_t ce = col_idx[e];
            bad |= (ce < 0) | (ce >= n);
        }
    }
    if (!BACK && bad) raise_status(status, CSR5_STATUS_BAD_COL_IDX);

    // ---- conversion step 3b, lane = tile column: forced first flag, y_offset =
    // exclusive scan of the columns' flag counts, seg_offset = run of flag-less
    // columns to the right (Algorithm 5; the scan and the run length are wavefront
    // operations here), packing (Section 3.5), and the tile's segment count for
    // the empty_offset layout.
    if constexpr (!BACK) {
        if (desc) {                                        // uniform over the grid
            if (active) {
                if (lane == 0) flags |= 1u;
                const int cnt = __popcll(flags);
                int incl = cnt;
#pragma unroll
                for (int d = 1; d < OMEGA; d <<= 1) {
                    const int up = __shfl_up(incl, d, OMEGA);
                    if (lane >= d) incl += up;
                }
                const uint32_t yo = uint32_t(incl - cnt);
                const int total = __shfl(incl, OMEGA - 1, OMEGA);
                const uint64_t heads = __ballot(cnt > 0);
                const uint64_t right = (lane == OMEGA - 1) ? 0ull : (heads >> (lane + 1));
                uint32_t so = 0;
                if (cnt > 0) so = right ? uint32_t(__builtin_ctzll(right)) : uint32_t(OMEGA - 1 - lane);
                // little-endian bit field: flags | seg_offset << sigma | y_offset << (sigma+6)
                constexpr int YSH = SIGMA + SBITS;  // <= 54
                const uint64_t lo = flags | (uint64_t(so) << SIGMA) | (uint64_t(yo) << YSH);
                const uint64_t hi = (YSH + YBITS > 64) ? (uint64_t(yo) >> (64 - YSH)) : 0ull;
                desc[dbase] = uint32_t(lo);
                if (W > 1) desc[dbase + OMEGA] = uint32_t(lo >> 32);
                if (W > 2) desc[dbase + 2 * OMEGA] = uint32_t(hi);
                if (lane == 0) {
                    if (wide) static_cast<int64_t*>(eop)[tile] = marked ? total : 0;
                    else static_cast<int32_t*>(eop)[tile] = marked ? total : 0;
                }
            }
            // "some tile is marked" (and hence "some row is empty"): once per workgroup, not
            // once per tile -- everything that aims at the one status word queues up
            __shared__ int wg_met_marked;
            if (threadIdx.x == 0) wg_met_marked = 0;
            __syncthreads();
            if (active && marked && lane == 0) wg_met_marked = 1;
            __syncthreads();
            if (threadIdx.x == 0 && wg_met_marked)
                raise_status(status, CSR5_STATUS_HAS_DIRTY | CSR5_STATUS_HAS_EMPTY_ROWS | STATUS_SCAN_NEEDED);
        }
    }
}

// ----------------------------------------------------------------------------
// CSR5 SpMV (Algorithm 8), one wavefront per complete tile, lane i = column i.
//
// Lane i streams its sigma (val, col_idx) pairs -- at each step j the 64 lanes
// read 64 consecutive entries -- gathers x, and walks its bit_flag word: a set
// flag closes the running sum either as the column's "red" head (belongs to a
// segment opened by an earlier column) or as a "green" complete segment that is
// stored straight to y[tile_ptr + y_offset + k].  What follows the last flag is
// the "blue" tail.
//
// In-tile segmented sum (the step of Algorithm 8 that calls Algorithm 6).
// Algorithm 6 computes it as a difference of two prefix sums over the whole
// tile, which loses the accuracy of a small row sitting after large ones.  Here: red partials are shifted one
// lane down (tmp[i] = red[i+1], the printed tmp[i-1] <- sum) and summed by a
// segmented suffix scan made of six wavefront shuffles, the segments being
// delimited by the ballot of "column has a flag".  The range it sums for a head
// column i is exactly tmp[i .. i+seg_offset[i]], the value Algorithm 6 defines;
// seg_offset itself is not read (the ballot carries the same information).
//
// Cross-tile (Section 4 offers atomic adds or a global auxiliary array; device
// wide fp64 atomics are resolved on the memory side of the eight L2s on this
// chip and, at two per tile, measured slower than everything else in the kernel
// together).  Only segment 0 of a tile can continue a row that an earlier tile
// opened (it does iff the tile's first nonzero is not its row's first:
// row_ptr[tile_ptr] != tile*T).  Two ways, chosen per MATRIX during conversion
// (status word), so that both tiles at a boundary decide alike without talking
// to each other:
//  * every tile can get at the head of its first row: it adds the head to its
//    segment 0 and stores the finished row; the previous tile does not store its
//    last segment.  That segment IS the head when the row began inside the
//    previous tile, and inside a workgroup (four neighbouring tiles up to
//    sigma = 16, two up to 32) it is handed over through LDS behind one barrier.
//    The workgroup's first tile sums the head itself, from a CSR-order copy of the
//    last LOOK_MAX = 160 entries of the previous workgroup's last tile (one extra
//    gather for heads up to 32 entries, three beyond).  So the condition is: no
//    first tile of a workgroup starts more than 160 entries into a row, and no
//    other tile more than a tile's length.  Such a matrix needs no second kernel.
//  * otherwise: the auxiliary array.  Segment 0 goes to carry[tile]; the tile that
//    holds the row's first nonzero stores the row's base value, and k_spmv_fixup
//    adds the carries afterwards.  Or, for matrices where that is faster (the
//    host decides, see ONE_LAUNCH_ANY_TILES), inside this kernel: the tiles of a
//    workgroup settle their common rows through LDS, workgroups meet per row at a
//    word of the auxiliary memory, and whoever comes last stores the row (see
//    "One-launch form of the auxiliary-array path" above spmv_tail).
// The third template argument (MODE) is the way: MODE_LOOK, MODE_CARRY, MODE_ONE.
// y needs no zero-fill.  Rows that receive carries from more than one wavefront
// of k_spmv_fixup, and rows cut by 64-entry chunks of the incomplete tile, are
// summed with atomic adds, in whatever order they arrive: their last bits can
// differ from run to run.  Everything else is summed in a fixed order.
//
// Workgroup 0 handles the entries after the last complete tile when there are
// any (early, so that its dependent searches hide behind the tiles); workgroups
// after the tiles write the zeros of rows without nonzeros when the matrix has
// such rows.
// ----------------------------------------------------------------------------
template <int SIGMA>
struct FlagWord {
    using type = typename std::conditional<(SIGMA > 32), uint64_t, uint32_t>::type;
};

// Sum over the 64 lanes; every lane gets the total.
template <typename VT>
__device__ __forceinline__ VT wave_sum(VT v) {
#pragma unroll
    for (int d = OMEGA / 2; d >= 1; d >>= 1) v += __shfl_xor(v, d, OMEGA);
    return v;
}

// The last `count` (<= LOOK_MAX) entries of a complete tile, read from the
// CSR-order record of its last entries (near part: the last LOOK; far part: the
// LOOK_FAR before them): every lane multiplies up to three of them by their x
// and the wavefront sums the products.  This is how the incomplete tile's
// workgroup completes a row that began shortly before it, instead of handing its
// part to a second kernel (the first tile of a workgroup does the same inside
// k_spmv).  last_col, last_val: the record's two views.
template <typename VT>
__device__ __forceinline__ VT look_behind(const int32_t* __restrict__ last_col, const VT* __restrict__ last_val,
                                          const VT* __restrict__ x, int count, int lane) {
    VT prod = VT(0);
    const int near_n = count < LOOK ? count : LOOK;
    if (lane >= LOOK - near_n && lane < LOOK) prod = last_val[lane] * x[last_col[lane]];
    if (count > LOOK) {                                   // uniform
        const int32_t* const far_c = last_col + FAR_COL_AT;
        const VT* const far_v = last_val + far_val_at<VT>();
        const int first = LOOK_FAR - (count - LOOK);      // far entries first .. LOOK_FAR - 1 belong to the head
#pragma unroll
        for (int j = lane; j < LOOK_FAR; j += OMEGA)
            if (j >= first) prod = fma(far_v[j], x[far_c[j]], prod);
    }
    return wave_sum(prod);
}

// ----------------------------------------------------------------------------
// One-launch form of the auxiliary-array path (Section 4: the sums of a row that
// spans tiles meet in a global auxiliary array).  The tiles of a workgroup are
// neighbours and settle the rows that cross between them through LDS.  A row that
// crosses workgroups is settled through memory without anybody waiting.  Groups:
// tile t of the complete tiles belongs to group t / waves, the incomplete tile is
// a group of its own behind them; span[t] (conversion) says for the row that holds
// tile t's first entry in which group it starts and how many groups it touches.
//  * Two groups (nearly all such rows): each swaps its part into meet[first group]
//    with one atomic exchange.  Whoever gets EMPTY back was first and is done;
//    whoever gets the other's part back adds the two, stores the row and puts
//    EMPTY back.  One memory round trip, and the value travels inside the atomic,
//    so nothing has to be ordered.
//  * More groups: the first group leaves its part in meet[first group], every
//    later group its part in carry[group]; each then counts itself in at
//    arrived[first group], and whoever finds that all the others have been there
//    adds the parts up, in group order, stores the row and resets the two words.
//    A part must have reached memory before its group is counted, and is read by
//    a wavefront of another XCD, whose L2 knows nothing of it: parts and counters
//    are written and read with device-scope atomic accesses (which pass the L2s),
//    and the wait between "part written" and "counted" is the plain wait for the
//    wavefront's outstanding memory operations.  (A release fence would also
//    write back every dirty line of the L2, the rows of y included: measured once
//    per tile, it made the kernel eleven times slower.)
// Either way the parts are added in group order: the result does not depend on
// who came last.
// ----------------------------------------------------------------------------
// A part as the 64-bit word of meet[]: a double's bits (with the one NaN pattern
// that means EMPTY replaced by another NaN), a float's bits under a tag.
__device__ __forceinline__ uint64_t meet_word(double v) {
    const uint64_t b = uint64_t(__double_as_longlong(v));
    return b == MEET_EMPTY ? 0x7ff8000000000000ull : b;
}
__device__ __forceinline__ uint64_t meet_word(float v) { return (1ull << 32) | uint64_t(__float_as_uint(v)); }
template <typename VT> __device__ __forceinline__ VT meet_value(uint64_t w);
template <> __device__ __forceinline__ double meet_value<double>(uint64_t w) { return __longlong_as_double(static_cast<long long>(w)); }
template <> __device__ __forceinline__ float meet_value<float>(uint64_t w) { return __uint_as_float(uint32_t(w)); }

__device__ __forceinline__ uint64_t swap_in(uint64_t* slot, uint64_t w) {
    return __hip_atomic_exchange(slot, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <typename T>
__device__ __forceinline__ void publish(T* slot, T v) {
    __hip_atomic_store(slot, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// lane 0 of a wavefront, after publish() and wait_for_memory(): count this group
// in at `counter`; returns how many were there before
__device__ __forceinline__ uint32_t count_in(uint32_t* counter) {
    return __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Barrier of the workgroup that orders LDS only: the wavefronts exchange their
// sums through LDS, and a wavefront's atomics to memory may still be on their way.
__device__ __forceinline__ void meet_at_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ void wait_for_memory() {
    __builtin_amdgcn_s_waitcnt(0);          // every counter at zero: loads, stores and LDS of this wavefront are done
    asm volatile("" ::: "memory");
}

// The whole wavefront: row R spans groups g0..g1 (three or more) and all of them have published.
template <typename VT>
__device__ __forceinline__ void assemble_row(const VT* piece_in, uint64_t* meet, uint32_t* arrived,
                                             int g0, int g1, VT* __restrict__ y, uint32_t R, int m, int lane) {
    VT sum = VT(0);
    for (int g = g0 + 1 + lane; g <= g1; g += OMEGA)
        sum += __hip_atomic_load(piece_in + g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sum = wave_sum(sum);
    if (lane == 0) {
        sum = meet_value<VT>(__hip_atomic_load(meet_at(meet, g0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) + sum;
        if (R < uint32_t(m)) y[R] = sum;
        publish(meet_at(meet, g0), MEET_EMPTY);
        publish(arrived + g0, 0u);
    }
}

constexpr int TAIL_MAX_CHUNKS = (CSR5_SIGMA_MAX * OMEGA) / OMEGA + 1;   // 64-entry chunks in < one tile

// Entries after the last complete tile (Section 4, last paragraph: a CSR-vector
// style pass).  64 consecutive entries per wavefront step; the row of each entry
// comes from a binary search (so runs of empty rows cost nothing); a shuffle
// scan sums runs of equal row.  A row that lies inside one 64-entry chunk is
// stored directly.  A row cut by a chunk boundary is accumulated in LDS, in the
// slot of the chunk it starts in (at most one row starts in a chunk and leaves
// it), and stored at the end.  The part of a row that began in the complete
// tiles is treated like a tile's segment 0: completed here when the row began at
// most LOOK entries earlier, handed to carry[pc] otherwise.
template <typename VT, typename IT>
__device__ void spmv_tail(int m, IT nnz, IT first, uint32_t row_first,
                          const IT* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                          const VT* __restrict__ val, const VT* __restrict__ x,
                          VT* __restrict__ y, VT* __restrict__ carry_slot,
                          VT* piece_in, uint64_t* meet, uint32_t* arrived, uint2 row_span,
                          const int32_t* __restrict__ last_col, const VT* __restrict__ last_val) {
    __shared__ VT acc[TAIL_MAX_CHUNKS];
    __shared__ int acc_row[TAIL_MAX_CHUNKS];
    __shared__ VT acc_first;
    const int lane = lane_id();
    const int wave = threadIdx.x / OMEGA, nwaves = blockDim.x / OMEGA;
    for (int q = threadIdx.x; q < TAIL_MAX_CHUNKS; q += blockDim.x) { acc[q] = VT(0); acc_row[q] = -1; }
    if (threadIdx.x == 0) acc_first = VT(0);
    __syncthreads();
    int row_lo = row_first > uint32_t(m) ? m : int(row_first);
    const int span = int(nnz - first);                   // < one tile
    const int nchunks = (span + OMEGA - 1) / OMEGA;
    for (int q = wave; q < nchunks && q < TAIL_MAX_CHUNKS; q += nwaves) {
        // 64-bit: with 32-bit indices and nnz within 64 of 2^31 these would overflow
        const int64_t chunk_lo = int64_t(first) + q * OMEGA;
        const int64_t e = chunk_lo + lane;
        const bool live = e < nnz;
        int row = -2 - lane;                         // distinct keys for dead lanes
        VT prod = VT(0);
        if (live) {
            row = row_lo + count_le(row_ptr + row_lo, m + 1 - row_lo, e) - 1;
            prod = val[e] * x[col_idx[e]];
        }
#pragma unroll
        for (int d = 1; d < OMEGA; d <<= 1) {
            VT up = __shfl_up(prod, d, OMEGA);
            int rup = __shfl_up(row, d, OMEGA);
            if (lane >= d && rup == row) prod += up;
        }
        int rnext = __shfl_down(row, 1, OMEGA);
        bool run_end = live && ((lane == OMEGA - 1) || (rnext != row));
        if (run_end && row >= 0 && row < m) {
            IT rs = row_ptr[row], re = row_ptr[row + 1];
            if (rs >= chunk_lo && re <= chunk_lo + OMEGA) {
                y[row] = prod;                       // the whole row lies in this chunk
            } else if (rs < first) {
                atomicAdd(&acc_first, prod);         // continues a row of the complete tiles
            } else {
                int q1 = int((rs - first) / OMEGA);  // chunk the row starts in
                if (q1 >= 0 && q1 < TAIL_MAX_CHUNKS) {
                    atomicAdd(&acc[q1], prod);
                    acc_row[q1] = row;
                }
            }
        }
    }
    __syncthreads();
    for (int q = threadIdx.x; q < TAIL_MAX_CHUNKS; q += blockDim.x)
        if (acc_row[q] >= 0) y[acc_row[q]] = acc[q];
    if (threadIdx.x < OMEGA && piece_in) {               // first wavefront, one-launch form: this is the last group of its first row
        if (row_lo < m && first > 0 && row_ptr[row_lo] < first) {
            const int g0 = int(row_span.x), g1 = g0 + int(row_span.y) - 1;
            if (row_span.y == 2u) {
                uint64_t other = MEET_EMPTY;
                if (lane == 0) other = swap_in(meet_at(meet, g0), meet_word(acc_first));
                if (lane == 0 && other != MEET_EMPTY) {
                    y[row_lo] = meet_value<VT>(other) + acc_first;
                    publish(meet_at(meet, g0), MEET_EMPTY);
                }
            } else {
                uint32_t before = 0;
                if (lane == 0) {
                    publish(piece_in + g1, acc_first);
                    wait_for_memory();
                    before = count_in(arrived + g0);
                }
                if (__shfl(before, 0, OMEGA) == uint32_t(g1 - g0))
                    assemble_row<VT>(piece_in, meet, arrived, g0, g1, y, uint32_t(row_lo), m, lane);
            }
        }
    } else if (threadIdx.x < OMEGA) {                    // first wavefront
        VT carried = acc_first;
        if (last_col && row_lo < m && first > 0) {       // last_col: entries of the last complete tile, or null
            const IT rs = row_ptr[row_lo];
            if (rs < first && first - rs <= IT(LOOK_MAX)) {  // the first row began shortly before: finish it here
                const VT head = look_behind<VT>(last_col, last_val, x, int(first - rs), lane);
                if (lane == 0) y[row_lo] = head + acc_first;
                carried = VT(0);
            }
        }
        if (lane == 0) *carry_slot = carried;
    }
}

template <int SIGMA, typename VT, typename IT, int MODE>
__global__ void __launch_bounds__(TransposeShape<SIGMA>::WAVES * OMEGA)
k_spmv(int m, IT nnz, int pc, int p, uint32_t nb_tiles, uint32_t has_tail, uint32_t xcd_chunk, uint32_t far_mode,
       int rec_bytes, const IT* __restrict__ row_ptr, const typename Index<IT>::tp_t* __restrict__ tile_ptr,
       const uint32_t* __restrict__ tile_desc, const IT* __restrict__ eop,
       const int32_t* __restrict__ eo, const int32_t* __restrict__ col_idx,
       const VT* __restrict__ val, const VT* __restrict__ x, VT* __restrict__ y,
       VT* __restrict__ carry, uint64_t* __restrict__ meet, uint32_t* __restrict__ arrived,
       const uint2* __restrict__ span, const uint32_t* __restrict__ status, const uint32_t* __restrict__ tile_head,
       const int32_t* __restrict__ last_col, const VT* __restrict__ last_val) {
    constexpr bool CAN_LOOK = MODE == MODE_LOOK;
    constexpr bool ONE = MODE == MODE_ONE;
    constexpr bool MEET = CAN_LOOK || ONE;      // the wavefronts of a workgroup meet at one barrier
    constexpr int T = OMEGA * SIGMA;
    constexpr int YBITS = 32 - __builtin_clz(uint32_t(T - 1));        // ceil(log2(64*sigma))
    constexpr int W = (SIGMA + SBITS + YBITS + 31) / 32;
    constexpr int YSH = SIGMA + SBITS;
    constexpr int WAVES = TransposeShape<SIGMA>::WAVES;
    constexpr int PITCH = TransposeShape<SIGMA>::PITCH;
    using flag_t = typename FlagWord<SIGMA>::type;
    using tp_t = typename Index<IT>::tp_t;
    // one slot per tile entry: a column index on the way in, an x value on the way back,
    // a segment sum at the end (so single precision needs half the space)
    __shared__ VT lds[WAVES][OMEGA * PITCH];
    __shared__ VT last_sum[WAVES];    // look-behind inside a workgroup: every tile's last segment, for the next tile

    const uint32_t st = *status;      // consulted below, after the streaming loads are in flight
    // Rows that cross a tile boundary are completed by look-behind in the whole
    // matrix or nowhere: both tiles at a boundary must decide alike.
    // CAN_LOOK = false is the instantiation for matrices the host knows to need
    // the carry array: the same kernel without the look-behind's loads.
    const bool look = CAN_LOOK && last_col != nullptr && !(st & STATUS_NEEDS_CARRY);

    if (blockIdx.x < has_tail) {      // workgroup 0: incomplete last tile
        if (st & BAD_BITS) return;
        const tp_t first_row = tile_ptr[pc] & Index<IT>::ROWMASK;
        spmv_tail<VT, IT>(m, nnz, IT(pc) * T, first_row > tp_t(m) ? uint32_t(m) : uint32_t(first_row),
                          row_ptr, col_idx, val, x, y, carry + pc,
                          ONE ? carry : nullptr, meet, arrived, ONE ? span[pc] : uint2{0u, 1u},
                          (look && pc > 0) ? last_col + size_t((pc - 1) / WAVES) * size_t(rec_bytes / 4) : nullptr,
                          (look && pc > 0) ? last_val + size_t((pc - 1) / WAVES) * size_t(rec_bytes / int(sizeof(VT))) : nullptr);
        return;
    }
    if (blockIdx.x >= has_tail + nb_tiles) {   // workgroups after the tiles: the zeros of rows without nonzeros
        if ((st & BAD_BITS) || !(st & CSR5_STATUS_HAS_EMPTY_ROWS)) return;
        const uint32_t b = blockIdx.x - has_tail - nb_tiles, nb = gridDim.x - has_tail - nb_tiles;
        const int64_t stride = int64_t(nb) * blockDim.x;
        for (int64_t r = int64_t(b) * blockDim.x + threadIdx.x; r < int64_t(m); r += stride)
            if (row_ptr[r] == row_ptr[r + 1]) y[r] = VT(0);
        return;
    }
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / OMEGA);
    const int tile = int(xcd_order(blockIdx.x - has_tail, nb_tiles, xcd_chunk)) * WAVES + wave;
    // (every wavefront of a tile workgroup passes exactly one barrier, see below)
    if (tile >= pc) {
        if constexpr (MEET) __syncthreads();
        return;
    }

    // How far into its first row the tile starts, and the next tile into its own
    // (tile_head: entries of a tile's first row that lie before the tile; p + 1
    // entries, 0 at p).  The same for every lane: scalar loads.
    const uint32_t head_len = tile_head[tile];
    const uint32_t next_head = tile_head[tile + 1];
    // One-launch form of the auxiliary-array path: the rows that cross this tile's
    // two boundaries (first group, number of groups), and the row of the second.
    uint2 span_in = {0u, 1u}, span_out = {0u, 1u};
    uint32_t out_row = 0;
    if constexpr (ONE) {
        span_in = span[tile];
        span_out = span[tile + 1];
        const typename Index<IT>::tp_t next_wide = tile_ptr[tile + 1] & Index<IT>::ROWMASK;
        out_row = next_wide < typename Index<IT>::tp_t(m) ? uint32_t(next_wide) : 0u;
    }

    // ---- look-behind, first part: the previous tile's last LOOK entries, whether
    // or not this tile turns out to need them (asking first would put a dependent
    // load in front of these, and everything the wavefront loads later waits for
    // them in turn).  Lanes LOOK.. repeat the addresses of lanes 0..LOOK-1.
    // Only the first tile of a workgroup needs them: the others get the finished
    // sum of their row's head from the wavefront next door (last_sum).  A head
    // longer than LOOK also takes the far part of the record, two entries per lane.
    VT head_v = VT(0), head_x = VT(0), far_v0 = VT(0), far_v1 = VT(0), far_prod = VT(0);
    int32_t head_c = 0, far_c0 = 0, far_c1 = 0;
    // far_mode, from the host: 0 = this matrix has no such head (nobody waits for
    // head_len then), 1 = it has, or the host does not know yet.  (Taking the far
    // part without asking whenever the matrix has such heads was slower than
    // asking: 114 against 110 us on a 53 M-nonzero matrix of 128-entry rows.)
    const bool far_head = CAN_LOOK && look && wave == 0 && far_mode != 0u && head_len > uint32_t(LOOK) &&
                          rec_bytes == LAST_REC_BYTES;      // uniform (the last test cannot fail: such a matrix has no long head in look mode)
    if constexpr (CAN_LOOK) {
        if (wave == 0) {
            const size_t rec = size_t(tile > 0 ? tile - 1 : 0) / WAVES;      // the group before this one
            const int32_t* const near_c = last_col + rec * size_t(rec_bytes / 4);
            const VT* const near_v = last_val + rec * size_t(rec_bytes / int(sizeof(VT)));
            head_c = near_c[lane & (LOOK - 1)];
            head_v = near_v[lane & (LOOK - 1)];
        }
    }

    // ---- stream the tile.  val: at step j the 64 lanes read 64 consecutive
    // doubles, lane i keeping entry (column i, step j).  col_idx is not needed by
    // its owner lane at all (see the gather below), so it is read with 16-byte
    // loads in plain memory order: 4 steps of the tile per instruction.
    const size_t tile_base = size_t(tile) * T;
    constexpr int NC4 = (SIGMA + 3) / 4;                  // 16-byte col loads per lane
    typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
    i32x4 c4[NC4];
    if ((reinterpret_cast<uintptr_t>(col_idx) & 15) == 0) {   // uniform
        const i32x4* col4 = reinterpret_cast<const i32x4*>(col_idx + tile_base);
#pragma unroll
        for (int q = 0; q < NC4; q++) {
            const int e4 = q * OMEGA + lane;              // index of the int4 inside the tile
            c4[q] = (SIGMA % 4 == 0 || e4 < T / 4) ? __builtin_nontemporal_load(&col4[e4]) : i32x4{0, 0, 0, 0};
        }
    } else {      // col_idx is a view at an odd offset into a caller's array: the same four entries, one by one
        const int32_t* col1 = col_idx + tile_base;
#pragma unroll
        for (int q = 0; q < NC4; q++) {
            const int e4 = q * OMEGA + lane;
            c4[q] = i32x4{0, 0, 0, 0};
            if (SIGMA % 4 == 0 || e4 < T / 4) {
                c4[q].x = __builtin_nontemporal_load(&col1[4 * e4 + 0]);
                c4[q].y = __builtin_nontemporal_load(&col1[4 * e4 + 1]);
                c4[q].z = __builtin_nontemporal_load(&col1[4 * e4 + 2]);
                c4[q].w = __builtin_nontemporal_load(&col1[4 * e4 + 3]);
            }
        }
    }
    VT v[SIGMA];
#pragma unroll
    for (int j = 0; j < SIGMA; j++) v[j] = __builtin_nontemporal_load(&val[tile_base + j * OMEGA + lane]);

    // ---- descriptor
    const tp_t tp = tile_ptr[tile];
    const bool dirty = (tp & Index<IT>::DIRTY) != 0;
    const tp_t row0_wide = tp & Index<IT>::ROWMASK;
    const uint32_t row0 = uint32_t(row0_wide);
    const uint32_t* dp = tile_desc + size_t(tile) * W * OMEGA + lane;
    uint64_t lo = __builtin_nontemporal_load(dp);
    if (W > 1) lo |= uint64_t(__builtin_nontemporal_load(dp + OMEGA)) << 32;
    uint64_t hi = 0;
    if (W > 2) hi = __builtin_nontemporal_load(dp + 2 * OMEGA);
    constexpr int FLAG_BITS = 8 * int(sizeof(flag_t));
    constexpr flag_t FLAG_MASK = (SIGMA == FLAG_BITS) ? ~flag_t(0) : flag_t((flag_t(1) << (SIGMA % FLAG_BITS)) - 1);
    const flag_t flags = flag_t(lo) & FLAG_MASK;
    uint32_t yo = uint32_t(lo >> YSH);
    if (W > 2) yo |= uint32_t(hi << (64 - YSH));
    // empty_offset slice of a tile that holds empty rows (Algorithm 8, where y_offset is replaced by empty_offset[y_offset])
    const int32_t* eo_t = nullptr;
    uint32_t nseg_t = 0;
    if (dirty) {
        IT e0 = eop[tile], e1 = eop[tile + 1];
        eo_t = eo + e0;
        nseg_t = uint32_t(e1 - e0);
    }
    // look-behind, the far part of the record.  Asked for only here, behind the
    // tile's own loads: the decision needs head_len, and a wait for it further up
    // would hold back the stream of every tile, also of those that never take it.
    if constexpr (CAN_LOOK) {
        if (far_head) {
            const size_t rec = size_t(tile - 1) / WAVES;                  // tile > 0: it has a head
            const int32_t* const far_c = last_col + rec * size_t(rec_bytes / 4) + FAR_COL_AT;
            const VT* const far_v = last_val + rec * size_t(rec_bytes / int(sizeof(VT))) + far_val_at<VT>();
            far_c0 = far_c[lane];
            far_c1 = far_c[OMEGA + lane];
            far_v0 = far_v[lane];
            far_v1 = far_v[OMEGA + lane];
        }
    }
    if ((st & BAD_BITS) || row0_wide >= tp_t(m)) {        // rejected input: gather and store nothing
        if constexpr (MEET) __syncthreads();
        return;
    }
    // Does segment 0 continue a row that an earlier tile opened?  Then either this
    // tile gets hold of the row's head (see `look`) and stores the finished row,
    // or its part goes through the carry array.
    // The mirror image: when the next tile (or the incomplete tile's workgroup)
    // completes this tile's last row, this tile must not store its part of it.
    const bool cont0 = head_len != 0;
    const bool skip_last = look && next_head != 0;
    const bool fetch_head = look && cont0 && wave == 0;   // uniform; the head is then at most LOOK_MAX entries long
    // the last min(head_len, LOOK) of the near LOOK entries belong to the head
    const bool head_lane = fetch_head && lane < LOOK && lane >= LOOK - int(head_len < uint32_t(LOOK) ? head_len : uint32_t(LOOK));

    // ---- gather x.  Lane i owns the CSR entries i*sigma .. i*sigma+sigma-1 of the
    // tile, so at a fixed step the 64 lanes would gather from 64 unrelated
    // places.  Consecutive CSR entries, however, have increasing and often
    // adjacent columns.  So the column indices are laid out in LDS in CSR order
    // (entry (i, j) at i*PITCH + j, rows padded to an odd pitch), read back so
    // that lane L holds CSR entries k*64+L (64 consecutive entries per gather
    // instruction: few distinct cache lines), x is gathered in that order, and
    // the values return through the same LDS buffer to the owner lanes.
    VT* const xb = reinterpret_cast<VT*>(lds[wave]);
    int32_t* const cb = reinterpret_cast<int32_t*>(lds[wave]);
    VT xv[SIGMA];
    {
#pragma unroll
        for (int q = 0; q < NC4; q++) {
            const int m0 = (q * OMEGA + lane) * 4;        // memory offset inside the tile = j*64 + i
            const int j = m0 / OMEGA, i0 = m0 % OMEGA;
            if (SIGMA % 4 == 0 || m0 < T) {
                cb[(i0 + 0) * PITCH + j] = c4[q].x;
                cb[(i0 + 1) * PITCH + j] = c4[q].y;
                cb[(i0 + 2) * PITCH + j] = c4[q].z;
                cb[(i0 + 3) * PITCH + j] = c4[q].w;
            }
        }
        wave_sync_lds();
        int32_t c[SIGMA];
#pragma unroll
        for (int k = 0; k < SIGMA; k++) {
            const int e = k * OMEGA + lane;
            c[k] = cb[(e / SIGMA) * PITCH + (e % SIGMA)];
        }
        wave_sync_lds();
        // All gathers of the tile are in flight together up to sigma = 32.  Beyond
        // that they go in groups of 16 (8 from sigma = 47 on): each gather holds four registers (address and
        // result) next to the tile's 2*sigma value registers, and with all of them
        // at once the kernel ran out of the 256 a wavefront can have (sigma >= 42:
        // spills into accumulator registers, one wavefront per SIMD).
        constexpr int GROUP = SIGMA > 46 ? 8 : (SIGMA > 32 ? 16 : SIGMA);
        // (without the look-behind the record holds nothing: the conversion did not fill it)
        VT far_x0 = VT(0), far_x1 = VT(0);
        if constexpr (CAN_LOOK) {
            if (wave == 0) {
                head_x = x[look ? head_c : 0];
                if (far_head) {
                    far_x0 = x[far_c0];
                    far_x1 = x[far_c1];
                }
            }
        }
#pragma unroll
        for (int k0 = 0; k0 < SIGMA; k0 += GROUP) {
#pragma unroll
            for (int k = k0; k < k0 + GROUP && k < SIGMA; k++) xv[k] = x[c[k]];
#pragma unroll
            for (int k = k0; k < k0 + GROUP && k < SIGMA; k++) {
                const int e = k * OMEGA + lane;
                xb[(e / SIGMA) * PITCH + (e % SIGMA)] = xv[k];
            }
            wave_sync_lds();
        }
#pragma unroll
        for (int j = 0; j < SIGMA; j++) xv[j] = xb[lane * PITCH + j];
        wave_sync_lds();
        if constexpr (CAN_LOOK) {
            if (far_head) {     // far entries first .. LOOK_FAR - 1 belong to the head (none when it is short); lane holds entries lane and lane + 64
                const int first = LOOK_FAR + LOOK - int(head_len);
                if (lane >= first) far_prod = far_v0 * far_x0;
                if (lane + OMEGA >= first) far_prod = fma(far_v1, far_x1, far_prod);
            }
        }
    }

    // ---- per-column walk.  Finished segment sums are parked in LDS (the buffer
    // is free again), slot = segment number inside the tile, and written to y
    // afterwards, 64 consecutive segments per store instruction.
    VT* const yb = xb;                                // T <= 64*PITCH slots
    VT sum = VT(0), red = VT(0);
    bool seen = false;
    uint32_t seg = yo;
#pragma unroll
    for (int j = 0; j < SIGMA; j++) {
        if ((flags >> j) & 1) {
            if (seen) {                                   // a green segment ends
                if (seg < uint32_t(T)) yb[seg] = sum;
                seg++;
            } else {                                      // the red head ends (empty when j == 0)
                red = sum;
                seen = true;
            }
            sum = VT(0);
        }
        sum = fma(v[j], xv[j], sum);
    }
    VT blue = sum;
    if (!seen) { red = sum; blue = VT(0); }                 // whole column is red

    // ---- in-tile segmented sum of the red partials
    uint64_t heads = __ballot(seen);                      // bit 0 is always set
    VT tmp = __shfl_down(red, 1, OMEGA);
    if (lane == OMEGA - 1) tmp = VT(0);
    uint64_t right = (lane == OMEGA - 1) ? 0ull : (heads >> (lane + 1));
    int end = right ? (lane + __builtin_ctzll(right)) : (OMEGA - 1);   // last lane of my segment
#pragma unroll
    for (int d = 1; d < OMEGA; d <<= 1) {
        VT dn = __shfl_down(tmp, d, OMEGA);
        if (lane + d <= end) tmp += dn;
    }
    if (seen && seg < uint32_t(T)) yb[seg] = blue + tmp;
    // number of segments of the tile = flags before the last column + its own
    uint32_t nseg = __shfl(seen ? seg + 1 : seg, OMEGA - 1, OMEGA);
    if (nseg > uint32_t(T)) nseg = T;
    if (dirty && nseg > nseg_t) nseg = nseg_t;            // cannot happen for a consistent format
    wave_sync_lds();

    // The head of the tile's first row.  Tiles of one workgroup are neighbours: a
    // tile's last segment, which the tile itself does not store when the row goes
    // on (skip_last), is the head its successor needs, finished (in look-behind
    // mode a row begins at most LOOK entries before a tile, so inside the previous
    // one).  It crosses through LDS; the workgroup's first tile has no neighbour
    // here and sums its head from the previous tile's record.
    VT head = VT(0);
    if constexpr (CAN_LOOK) {
        if (lane == 0) last_sum[wave] = nseg ? yb[nseg - 1] : VT(0);     // (nseg >= 1: a tile's first flag is forced)
        __syncthreads();
        if (wave == 0) head = wave_sum(head_lane ? fma(head_v, head_x, far_prod) : far_prod);
        else if (look && cont0) head = last_sum[wave - 1];
    }

    // One-launch form.  What the tiles before this one, inside the workgroup, hold
    // of its first row comes through LDS: a tile that lies wholly inside the row
    // passes on what it got plus its own sum, the tile the row starts in its last
    // segment.  `outside`: the row began before the workgroup.
    bool store_first = true, drop_last = false, pub_in = false, pub_out = false, pub_out_first = false;
    uint32_t before_in = 0, before_out = 0;
    uint64_t other_in = MEET_EMPTY, other_out = MEET_EMPTY;
    VT part_in = VT(0), part_out = VT(0);
    const int group = tile / WAVES;
    if constexpr (ONE) {
        __shared__ VT first_sum[WAVES];
        __shared__ int inside_row[WAVES];
        const bool goes_on = next_head != 0;                       // the last segment's row continues in the next tile
        const bool last_of_group = wave == WAVES - 1 || tile + 1 >= pc;
        const bool leaves = nseg == 1 && goes_on;                  // the tile's only segment goes on
        // Parts that do not depend on the neighbours set out before the barrier: the
        // last segment of the group's last tile, and the first tile's first segment
        // when its row ends there.
        const bool early_out = nseg > 1 && goes_on && last_of_group;
        const bool early_in = wave == 0 && cont0 && !leaves;
        if (lane == 0) {
            first_sum[wave] = nseg ? yb[0] : VT(0);
            last_sum[wave] = nseg ? yb[nseg - 1] : VT(0);
            inside_row[wave] = (nseg == 1 && cont0) ? 1 : 0;
            if (early_in) {
                part_in = first_sum[wave];
                if (span_in.y == 2u) other_in = swap_in(meet_at(meet, span_in.x), meet_word(part_in));
                else publish(carry + group, part_in);
            }
            if (early_out) {
                part_out = last_sum[wave];
                if (span_out.y == 2u) other_out = swap_in(meet_at(meet, group), meet_word(part_out));
                else publish(meet_at(meet, group), meet_word(part_out));
            }
        }
        meet_at_barrier();
        bool outside = false;
        if (cont0) {
            outside = true;
            for (int v = wave - 1; v >= 0; v--) {
                if (inside_row[v]) {
                    head += first_sum[v];
                } else {
                    head += last_sum[v];
                    outside = false;
                    break;
                }
            }
        }
        store_first = !leaves && !(cont0 && outside);
        drop_last = goes_on;
        // the group's part of a row that came in from outside: published where the row ends, or by the group's last tile
        pub_in = cont0 && outside && (!leaves || last_of_group);
        // the group's part of a row that began inside it and leaves it
        pub_out_first = leaves && last_of_group && !(cont0 && outside);
        pub_out = pub_out_first || early_out;
        if (lane == 0 && (pub_in || pub_out)) {
            const bool late_in = pub_in && !early_in, late_out = pub_out_first;
            if (late_in || late_out) {
                const VT whole = first_sum[wave] + head;
                if (late_in) part_in = whole;
                if (late_out) part_out = whole;
            }
            const bool count_in_row = pub_in && span_in.y != 2u, count_out_row = pub_out && span_out.y != 2u;
            if (late_in && !count_in_row) other_in = swap_in(meet_at(meet, span_in.x), meet_word(part_in));
            if (late_out && !count_out_row) other_out = swap_in(meet_at(meet, group), meet_word(part_out));
            if (count_in_row || count_out_row) {
                if (late_in && count_in_row) publish(carry + group, part_in);
                if (late_out && count_out_row) publish(meet_at(meet, group), meet_word(part_out));
                wait_for_memory();
                if (count_in_row) before_in = count_in(arrived + span_in.x);
                if (count_out_row) before_out = count_in(arrived + group);
            }
        }
    }

    // ---- write the tile's rows.  Segment s is row tile_ptr + s, or
    // tile_ptr + empty_offset[s] when the tile holds empty rows.  In the
    // two-kernel form segment 0 goes to the carry array when it continues an
    // earlier tile's row.
    for (uint32_t s0 = 0; s0 < nseg; s0 += OMEGA) {
        const uint32_t sg = s0 + lane;
        if (sg < nseg) {
            VT value = yb[sg];
            const uint32_t row = row0 + (dirty ? uint32_t(eo_t[sg]) : sg);
            bool mine;
            if constexpr (ONE) {
                if (sg == 0) value += head;
                mine = sg == 0 ? store_first : !(drop_last && sg == nseg - 1);
            } else {
                if (sg == 0) {
                    carry[tile] = (cont0 && !look) ? value : VT(0);
                    value += head;                         // 0 unless this tile completes the row
                }
                mine = (sg != 0 || !cont0 || look) && !(skip_last && sg == nseg - 1);
            }
            if (mine && row < uint32_t(m)) y[row] = value;
        }
    }
    if constexpr (ONE) {
        // (the answers come back while the rows above are stored)
        const uint32_t row_out = pub_out_first ? row0 : out_row;
        if (pub_in && span_in.y == 2u) {               // two groups: the second to come stores the row
            if (lane == 0 && other_in != MEET_EMPTY) {
                if (row0 < uint32_t(m)) y[row0] = meet_value<VT>(other_in) + part_in;
                publish(meet_at(meet, span_in.x), MEET_EMPTY);
            }
        } else if (pub_in && __shfl(before_in, 0, OMEGA) == span_in.y - 1u) {
            assemble_row<VT>(carry, meet, arrived, int(span_in.x), int(span_in.x + span_in.y) - 1, y, row0, m, lane);
        }
        if (pub_out && span_out.y == 2u) {
            if (lane == 0 && other_out != MEET_EMPTY) {
                if (row_out < uint32_t(m)) y[row_out] = part_out + meet_value<VT>(other_out);
                publish(meet_at(meet, group), MEET_EMPTY);
            }
        } else if (pub_out && __shfl(before_out, 0, OMEGA) == span_out.y - 1u) {
            assemble_row<VT>(carry, meet, arrived, group, group + int(span_out.y) - 1, y, row_out, m, lane);
        }
    }
}

// ----------------------------------------------------------------------------
// Second launch of an SpMV, needed only when some tile starts more than LOOK
// entries into a row: adds the carries (the global auxiliary array of Section 4).
// One thread per tile, tiles in order across the lanes.  Tiles whose first row
// is the same row R form a run (a row longer than a tile); a shuffle scan sums
// the carries of a run and its last lane adds the total to y[R], which already
// holds the part computed by the tile R starts in.  A run wholly inside one
// wavefront is a plain read-modify-write (nobody else touches y[R] now); a run
// cut by a wavefront boundary uses atomic adds, which commute.
// ----------------------------------------------------------------------------
template <typename VT, typename IT>
__global__ void __launch_bounds__(256)
k_spmv_fixup(int m, int ntiles,
             const typename Index<IT>::tp_t* __restrict__ tile_ptr, const VT* __restrict__ carry,
             VT* __restrict__ y, const uint32_t* __restrict__ status) {
    // rows are below 2^31 whatever the index width; 0xfff... marks "no tile"
    auto first_row = [&](int t) -> uint32_t {
        auto v = tile_ptr[t] & Index<IT>::ROWMASK;
        return v > 0x7fffffffu ? 0x7fffffffu : uint32_t(v);
    };
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = lane_id();
    const int t0 = gid - lane;                            // first tile of this wavefront
    const bool live = gid < ntiles;
    // Everything that does not depend on other loads is requested at once: the
    // kernel is a chain of memory round trips and nothing else.
    const uint32_t st = *status;
    const uint32_t R = live ? first_row(gid) : (0xfffffff0u - uint32_t(lane));
    VT cs = live ? carry[gid] : VT(0);
    const uint32_t r_after = (gid + 1 < ntiles) ? first_row(gid + 1) : 0xffffffffu;
    const uint32_t r_before = (t0 > 0 && t0 < ntiles) ? first_row(t0 - 1) : 0xffffffffu;
    if ((st & BAD_BITS) || t0 >= ntiles) return;
#pragma unroll
    for (int d = 1; d < OMEGA; d <<= 1) {
        VT up = __shfl_up(cs, d, OMEGA);
        uint32_t rup = __shfl_up(R, d, OMEGA);
        if (lane >= d && rup == R) cs += up;
    }
    const uint32_t rnext = __shfl_down(R, 1, OMEGA);
    const uint32_t rfirst = __shfl(R, 0, OMEGA);
    const bool run_end = live && ((lane == OMEGA - 1) || (rnext != R));
    if (run_end && cs != VT(0) && R < uint32_t(m)) {
        const bool ext_left = (rfirst == R) && (r_before == R);
        const bool ext_right = (lane == OMEGA - 1) && (r_after == R);
        if (ext_left || ext_right) atomic_add_fp(&y[R], cs);
        else y[R] += cs;
    }
}

// ----------------------------------------------------------------------------
// Measurement aid: what the memory system charges for the tile kernel's streams
// alone.  One wavefront per complete tile, the same workgroup shape and tile
// order as the tile kernel's most common instantiation; it reads the tile's
// col_idx, val and descriptors with 16-byte non-temporal loads (all of a tile in
// flight at once up to sigma = 16) and, if asked, stores one value to every row
// the tile starts (the rows of y that tile's wavefront writes in an SpMV).  No
// gathers, no LDS, no arithmetic to speak of.
// ----------------------------------------------------------------------------
constexpr int FLOOR_WAVES = 4;
constexpr int FLOOR_LOADS = 12;            // 16-byte loads per lane and round

template <typename VT, typename IT>
__global__ void __launch_bounds__(FLOOR_WAVES * OMEGA)
k_stream_floor(int m, int pc, int sigma, int W, uint32_t nb_tiles, uint32_t xcd_chunk, int write_y,
               const typename Index<IT>::tp_t* __restrict__ tile_ptr, const uint32_t* __restrict__ tile_desc,
               const int32_t* __restrict__ col_idx, const VT* __restrict__ val, VT* __restrict__ y) {
    typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / OMEGA);
    const int tile = int(xcd_order(blockIdx.x, nb_tiles, xcd_chunk)) * FLOOR_WAVES + wave;
    if (tile >= pc) return;
    const int T = OMEGA * sigma;
    // the three streams of a tile as one sequence of 16-byte pieces
    const i32x4* c4 = reinterpret_cast<const i32x4*>(col_idx + size_t(tile) * T);
    const i32x4* v4 = reinterpret_cast<const i32x4*>(val + size_t(tile) * T);
    const i32x4* d4 = reinterpret_cast<const i32x4*>(tile_desc + size_t(tile) * W * OMEGA);
    const int n_c = T / 4, n_v = T * int(sizeof(VT)) / 16, n_d = W * OMEGA / 4;
    const int total = n_c + n_v + n_d;
    int32_t acc = 0;
    for (int base = 0; base < total; base += OMEGA * FLOOR_LOADS) {
        i32x4 r[FLOOR_LOADS];
#pragma unroll
        for (int u = 0; u < FLOOR_LOADS; u++) {
            const int idx = base + u * OMEGA + lane;
            const i32x4* src = idx < n_c ? c4 + idx : (idx < n_c + n_v ? v4 + (idx - n_c) : d4 + (idx - n_c - n_v));
            r[u] = i32x4{0, 0, 0, 0};
            if (idx < total) r[u] = __builtin_nontemporal_load(src);
        }
#pragma unroll
        for (int u = 0; u < FLOOR_LOADS; u++) acc ^= r[u].x ^ r[u].y ^ r[u].z ^ r[u].w;
    }
    if (write_y) {
        const uint32_t r0 = uint32_t(tile_ptr[tile] & Index<IT>::ROWMASK);
        uint32_t r1 = uint32_t(tile_ptr[tile + 1] & Index<IT>::ROWMASK);
        if (r1 > uint32_t(m)) r1 = uint32_t(m);
        for (uint32_t r = r0 + lane; r < r1; r += OMEGA) y[r] = VT(acc);
    } else if (acc == 0x5a17c0de) {
        y[0] = VT(acc);                    // keeps the loads alive; practically never taken (y is scratch here)
    }
}

template <int SIGMA, typename VT, typename IT, int MODE>
hipError_t launch_spmv(const Geom& g, int m, int n, IT nnz, const IT* row_ptr,
                       const typename Index<IT>::tp_t* tile_ptr,
                       const uint32_t* tile_desc, const IT* eop, const int32_t* eo,
                       const int32_t* col_idx, const VT* val, const VT* x, VT* y,
                       VT* carry, uint64_t* meet, uint32_t* arrived, const uint2* span, const uint32_t* status, const uint32_t* tile_head, const int32_t* last_col,
                       const VT* last_val, bool zero_rows, uint32_t far_mode, hipStream_t s) {
    constexpr int WAVES = TransposeShape<SIGMA>::WAVES;
    uint32_t nb_tiles = uint32_t((g.pc + WAVES - 1) / WAVES);
    uint32_t has_tail = (int64_t(g.pc) * g.T < nnz) ? 1u : 0u;
    // rows without nonzeros: up to 512 workgroups stride over the rows
    size_t nb_zero = zero_rows ? (size_t(m) + WAVES * OMEGA - 1) / (WAVES * OMEGA) : 0;
    if (nb_zero > 512) nb_zero = 512;
    uint32_t nb = nb_tiles + has_tail + uint32_t(nb_zero);
    if (nb == 0) return hipSuccess;
    const size_t x_bytes = size_t(n) * sizeof(VT);
    uint32_t xcd_chunk = 0;                                        // contiguous eighths
    if (x_bytes > XCD_CONTIGUOUS_MAX_X_BYTES)                      // x too large for that to pay
        xcd_chunk = (int64_t(nnz) / (m > 0 ? m : 1) <= g.T / Y_LINE_ROWS) ? 1u : XCD_CHUNK;
    else if (x_bytes < XCD_CONTIGUOUS_MIN_X_BYTES)                 // x at home in every L2
        xcd_chunk = XCD_CHUNK;
    hipLaunchKernelGGL((k_spmv<SIGMA, VT, IT, MODE>), dim3(nb), dim3(WAVES * OMEGA), 0, s, m, nnz, g.pc, g.p, nb_tiles, has_tail,
                       xcd_chunk, far_mode, record_bytes(int64_t(nnz)), row_ptr, tile_ptr, tile_desc, eop, eo, col_idx, val, x, y, carry,
                       meet, arrived, span, status, tile_head, last_col, last_val);
    return hipGetLastError();
}

template <int SIGMA, bool BACK, typename VT>
hipError_t launch_transpose(const Geom& g, int n, int64_t nnz, int32_t* col_idx, VT* val,
                            uint32_t* status, int32_t* last_col, VT* last_val, const void* tile_ptr,
                            uint32_t* desc, void* eop, int wide, hipStream_t s) {
    constexpr int WAVES = TransposeShape<SIGMA>::WAVES;
    uint32_t nb = uint32_t((g.pc + WAVES - 1) / WAVES);
    if (nb == 0) nb = BACK ? 0 : 1;   // forward pass still validates the tail's columns
    if (nb == 0) return hipSuccess;
    hipLaunchKernelGGL((k_transpose<SIGMA, BACK, VT>), dim3(nb), dim3(WAVES * OMEGA), 0, s, g.pc, n, nnz,
                       col_idx, val, status, last_col, last_val, record_bytes(nnz), tile_ptr, desc, eop, wide);
    return hipGetLastError();
}

// ----------------------------------------------------------------------------
// CSR row-block baselines (Section 2.2.1), for the iteration-scenario comparison
// of Section 5.5: the cost of staying in CSR.  They read the untouched CSR
// arrays and have nothing to do with the CSR5 path.
//  * CSR-scalar (Algorithm 1): one thread per row.
//  * CSR-vector: LANES lanes per row (a power of two up to the wavefront),
//    lane-strided loads, shuffle reduction.
// ----------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_csr_scalar(int m, const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
             const double* __restrict__ val, const double* __restrict__ x, double* __restrict__ y) {
    const int64_t g = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (g >= int64_t(m)) return;
    const int r = int(g);
    double acc = 0.0;
    for (int k = row_ptr[r], e = row_ptr[r + 1]; k < e; k++) acc = fma(val[k], x[col_idx[k]], acc);
    y[r] = acc;
}

template <int LANES>
__global__ void __launch_bounds__(256)
k_csr_vector(int m, const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
             const double* __restrict__ val, const double* __restrict__ x, double* __restrict__ y) {
    const int64_t gid = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t r = gid / LANES;
    const int sub = int(gid % LANES);
    double acc = 0.0;
    if (r < int64_t(m))
        for (int64_t k = int64_t(row_ptr[r]) + sub, e = row_ptr[r + 1]; k < e; k += LANES)
            acc = fma(val[k], x[col_idx[k]], acc);
#pragma unroll
    for (int d = LANES / 2; d >= 1; d >>= 1) acc += __shfl_down(acc, d, LANES);
    if (r < int64_t(m) && sub == 0) y[r] = acc;
}

#define CSR5_FOR_SIGMA(X)                                                                          \
    X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15) X(16) X(17)   \
    X(18) X(19) X(20) X(21) X(22) X(23) X(24) X(25) X(26) X(27) X(28) X(29) X(30) X(31) X(32)      \
    X(33) X(34) X(35) X(36) X(37) X(38) X(39) X(40) X(41) X(42) X(43) X(44) X(45) X(46) X(47) X(48)

}  // namespace

// ----------------------------------------------------------------------------
// Scratch of csr5_spmv_static, the SpMV entry point that allocates nothing: the
// cross-tile auxiliary array lives here instead of in the handle.  Every GPU the
// library runs on holds its own copy of this array until the process ends.  In
// host code the array's NAME is only a stand-in; the memory is reached through
// the address hipGetSymbolAddress returns for the current device, resolved once
// per device (static_scratch) and passed to the kernels as an argument.
// ----------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[CSR5_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::atomic<void*> scratch_ptr[MAX_DEVICES];

// Address of `scratch` on device `dev`, which must be the current device.
// Threads that race here resolve the same address.
int static_scratch(int dev, void** out) {
    if (dev < 0 || dev >= MAX_DEVICES) return CSR5_ERANGE;
    void* p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return CSR5_EHIP;
        }
        scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return CSR5_OK;
}

}  // namespace

// ----------------------------------------------------------------------------
// handle
// ----------------------------------------------------------------------------
struct csr5_handle_s {
    int32_t m, n;
    int64_t nnz;
    Geom g;
    bool wide;             // 64-bit row_ptr, tile_ptr and empty_offset_ptr (csr5l_convert_ex)
    const void* row_ptr;   // int32_t* or int64_t*
    int32_t* col_idx;
    void* val;             // double* or float*, see dtype
    int dtype;             // CSR5_DTYPE_F64 / CSR5_DTYPE_F32
    void* tile_ptr;        // uint32_t* or uint64_t*
    uint32_t* tile_desc;
    void* eop;             // int32_t* or int64_t*
    int32_t* eo;
    uint32_t* status;
    // Cross-tile sums of an SpMV: one 8-byte entry per tile (incomplete one included),
    // CARRY_SLOTS such arrays taken in turn by successive calls, so that up to that
    // many SpMVs on one handle may be in flight at once (on different streams).
    void* carry;
    size_t carry_slot_bytes;
    std::atomic<uint32_t> carry_turn;
    uint32_t* tile_head;   // per tile: entries of its first row that lie before it, saturated at 32 bits
    int aux_form;          // 0: the size rule decides how the auxiliary-array path adds its sums; 1: always the second kernel; 2: inside the tile kernel wherever span exists
    uint2* span;           // per tile: the groups of tiles that row touches (first, how many); NULL where the one-launch SpMV cannot run
    // CSR-order copy of the last LOOK entries of every tile group's last tile (NULL for
    // small and for large sigma): two views of one array of LAST_REC_BYTES-byte records
    int32_t* last_col;
    void* last_val;
    void* owned;           // hipMalloc'ed block, or NULL when a workspace was given
    hipStream_t conv_stream;
    int device;            // HIP device that was current at conversion
    bool in_csr5_order;
    // The device-side status word once the host has read it (-1 before): tells
    // csr5_spmv* which launches this matrix needs.  Unknown means all of them.
    std::atomic<int32_t> status_host;
};

namespace {

struct Layout {
    size_t off_tile_ptr, off_tile_head, off_span, off_desc, off_eop, off_eo, off_carry, off_last, off_scan, off_wg_far, off_status, total;
    bool has_last;
    size_t ndesc, eo_cap, carry_slot_bytes;
};

Layout make_layout(int32_t m, int64_t nnz, const Geom& g, bool wide) {
    Layout L;
    const size_t isz = wide ? 8 : 4;   // bytes of one tile_ptr / empty_offset_ptr entry
    L.ndesc = size_t(g.pc) * g.W * OMEGA;
    size_t cap_a = size_t(m) + size_t(g.pc);
    size_t cap_b = size_t(g.pc) * g.T;
    L.eo_cap = cap_a < cap_b ? cap_a : cap_b;
    size_t o = 0;
    L.off_tile_ptr = o; o += align256((size_t(g.p) + 1) * isz);
    L.off_tile_head = o; o += align256((size_t(g.p) + 1) * 4);
    L.off_span = o;     o += one_launch_fits(g.sigma, g.p) ? align256((size_t(g.p) + 1) * 8) : 0;
    L.off_desc = o;     o += align256(L.ndesc * 4);
    L.off_eop = o;      o += align256((size_t(g.pc) + 1) * isz);
    L.off_eo = o;       o += align256(L.eo_cap * 4);
    // one slot per SpMV in flight: carry; where the one-launch form may run, also the meeting words and the counters
    L.carry_slot_bytes = align256((size_t(g.p) + 1) * 8);
    if (one_launch_fits(g.sigma, g.p)) L.carry_slot_bytes = slot_bytes_one(g, tile_group_waves(g.sigma));
    L.off_carry = o;    o += L.carry_slot_bytes * CARRY_SLOTS;
    L.has_last = look_sigma(g.sigma) && g.pc > 0;
    const size_t groups = (size_t(g.pc) + tile_group_waves(g.sigma) - 1) / tile_group_waves(g.sigma);
    L.off_last = o;     o += L.has_last ? align256(groups * size_t(record_bytes(nnz))) : 0;
    L.off_scan = o;     o += align256((size_t(g.pc) / SCAN_CHUNK + 1) * isz);   // chunk totals of the scan
    L.off_wg_far = o;   o += align256(size_t(MAX_TILE_PTR_WG) * 4);              // one word per workgroup of k_tile_ptr
    L.off_status = o;   o += 256;
    L.total = o;
    return L;
}

// Largest matrix the launches can address: one wavefront per tile and at most
// 2^32 - 1 threads in a grid; the row-parallel kernels add p_c threads to m, and
// all of them form m + 1 in 32 bits.
bool geometry_fits(int64_t m, int64_t nnz, int sigma) {
    if (m > int64_t(INT32_MAX) - 1) return false;
    const int64_t T = int64_t(OMEGA) * sigma;
    const int64_t p = (nnz + T - 1) / T;
    return p < (int64_t(1) << 26) - 4 && m + p < (int64_t(1) << 32) - 512;
}

}  // namespace

extern "C" {

const char* csr5_strerror(int code) {
    switch (code) {
        case CSR5_OK: return "ok";
        case CSR5_EINVAL: return "invalid argument";
        case CSR5_ENOMEM: return "out of memory or workspace too small";
        case CSR5_EHIP: return "HIP runtime error";
        case CSR5_ERANGE: return "sigma out of range, or matrix too large for the index width";
        default: return "unknown error";
    }
}

int32_t csr5_sigma_auto(int64_t nnz, int64_t m) {
    if (m <= 0 || nnz <= 0) return RULE_R;
    int64_t q = nnz / m;
    if (q > RULE_T) return RULE_U;
    int32_t sigma = q <= RULE_R ? RULE_R : (q <= RULE_S ? int32_t(q) : RULE_S);
    if (sigma > RULE_SIGMA_SMALL && nnz < RULE_MIN_TILES * OMEGA * sigma) sigma = RULE_SIGMA_SMALL;
    return sigma;
}

size_t csr5_workspace_bytes(int32_t m, int32_t nnz, int32_t sigma) {
    if (m < 0 || nnz < 0) return 0;
    if (sigma == 0) sigma = csr5_sigma_auto(nnz, m);
    if (sigma < CSR5_SIGMA_MIN || sigma > CSR5_SIGMA_MAX || !geometry_fits(m, nnz, sigma)) return 0;
    Geom g = make_geom(nnz, sigma);
    return make_layout(m, nnz, g, false).total;
}

size_t csr5l_workspace_bytes(int32_t m, int64_t nnz, int32_t sigma) {
    if (m < 0 || nnz < 0) return 0;
    if (sigma == 0) sigma = csr5_sigma_auto(nnz, m);
    if (sigma < CSR5_SIGMA_MIN || sigma > CSR5_SIGMA_MAX || !geometry_fits(m, nnz, sigma)) return 0;
    Geom g = make_geom(nnz, sigma);
    return make_layout(m, nnz, g, true).total;
}

}  // extern "C"

template <typename VT, typename IT>
static int convert_impl(int32_t m, int32_t n, IT nnz, const IT* row_ptr, int32_t* col_idx,
                        VT* val, int32_t sigma, void* workspace, size_t workspace_bytes,
                        void* hip_stream, uint32_t flags, csr5_handle_t* out) {
    using tp_t = typename Index<IT>::tp_t;
    constexpr bool wide = sizeof(IT) == 8;
    if (!out) return CSR5_EINVAL;
    *out = nullptr;
    if (m < 0 || n < 0 || nnz < 0) return CSR5_EINVAL;
    if (!row_ptr) return CSR5_EINVAL;                      // row_ptr has m+1 >= 1 entries
    if (nnz > 0 && (!col_idx || !val || m == 0 || n == 0)) return CSR5_EINVAL;
    // natural alignment of every element is all the kernels need (the SpMV reads
    // col_idx sixteen bytes at a time when its base allows that, else four)
    if ((reinterpret_cast<uintptr_t>(col_idx) & 3) || (reinterpret_cast<uintptr_t>(val) & (sizeof(VT) - 1)) ||
        (reinterpret_cast<uintptr_t>(row_ptr) & (sizeof(IT) - 1))) return CSR5_EINVAL;
    if (sigma == 0) sigma = csr5_sigma_auto(nnz, m);
    if (sigma < CSR5_SIGMA_MIN || sigma > CSR5_SIGMA_MAX) return CSR5_ERANGE;
    if (!geometry_fits(m, nnz, sigma)) return CSR5_ERANGE;
    if ((flags & ~(CSR5_FLAG_NO_HOST_CHECK | CSR5_FLAG_AUX_TWO_KERNELS | CSR5_FLAG_AUX_ONE_KERNEL)) ||
        ((flags & CSR5_FLAG_AUX_TWO_KERNELS) && (flags & CSR5_FLAG_AUX_ONE_KERNEL))) return CSR5_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    Geom g = make_geom(nnz, sigma);
    Layout L = make_layout(m, nnz, g, wide);
    csr5_handle_s* h = new (std::nothrow) csr5_handle_s();
    if (!h) return CSR5_ENOMEM;
    char* basep = nullptr;
    if (workspace) {
        if (workspace_bytes < L.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) {
            delete h;
            return workspace_bytes < L.total ? CSR5_ENOMEM : CSR5_EINVAL;
        }
        basep = static_cast<char*>(workspace);
        h->owned = nullptr;
    } else {
        void* ptr = nullptr;
        if (hipMalloc(&ptr, L.total) != hipSuccess) {
            (void)hipGetLastError();
            delete h;
            return CSR5_ENOMEM;
        }
        basep = static_cast<char*>(ptr);
        h->owned = ptr;
    }
    h->m = m; h->n = n; h->nnz = nnz; h->g = g; h->wide = wide;
    h->row_ptr = row_ptr; h->col_idx = col_idx; h->val = val;
    h->dtype = std::is_same<VT, float>::value ? CSR5_DTYPE_F32 : CSR5_DTYPE_F64;
    h->tile_ptr = basep + L.off_tile_ptr;
    h->tile_desc = reinterpret_cast<uint32_t*>(basep + L.off_desc);
    h->eop = basep + L.off_eop;
    h->eo = reinterpret_cast<int32_t*>(basep + L.off_eo);
    h->carry = basep + L.off_carry;
    h->carry_slot_bytes = L.carry_slot_bytes;
    h->carry_turn.store(0, std::memory_order_relaxed);
    h->tile_head = reinterpret_cast<uint32_t*>(basep + L.off_tile_head);
    h->aux_form = (flags & CSR5_FLAG_AUX_TWO_KERNELS) ? 1 : ((flags & CSR5_FLAG_AUX_ONE_KERNEL) ? 2 : 0);
    h->span = one_launch_fits(g.sigma, g.p) ? reinterpret_cast<uint2*>(basep + L.off_span) : nullptr;
    h->last_val = L.has_last ? basep + L.off_last : nullptr;                               // record + 0
    h->last_col = L.has_last ? reinterpret_cast<int32_t*>(basep + L.off_last + LOOK * 8) : nullptr;
    h->status = reinterpret_cast<uint32_t*>(basep + L.off_status);
    h->conv_stream = s;
    if (hipGetDevice(&h->device) != hipSuccess) {
        if (h->owned) (void)hipFree(h->owned);
        delete h;
        return CSR5_EHIP;
    }
    h->in_csr5_order = true;
    h->status_host.store(-1, std::memory_order_relaxed);
    {   // set-up time on this device: resolve the static scratch's address now, so
        // that csr5_spmv_static has nothing left to look up (failure is reported there)
        void* unused = nullptr;
        (void)static_scratch(h->device, &unused);
    }
    tp_t* const tile_ptr = static_cast<tp_t*>(h->tile_ptr);
    IT* const eop = static_cast<IT*>(h->eop);

    hipError_t e = hipSuccess;
    uint32_t* const wg_far = reinterpret_cast<uint32_t*>(basep + L.off_wg_far);
    int n_far_wg = 0;
    {   // step 2a (+ clearing)
        size_t work = L.ndesc > size_t(g.p) + 1 ? L.ndesc : size_t(g.p) + 1;
        size_t nb = (work + 255) / 256;
        if (nb > MAX_TILE_PTR_WG) nb = MAX_TILE_PTR_WG;
        // only the workgroups that hold tile boundaries (thread g of the grid takes tile g first) have anything to say
        const size_t with_tiles = (size_t(g.p) + 1 + 255) / 256;
        n_far_wg = int(with_tiles < nb ? with_tiles : nb);
        hipLaunchKernelGGL(k_tile_ptr<IT>, dim3(uint32_t(nb)), dim3(256), 0, s, m, row_ptr, g.T, g.p, g.pc,
                           tile_group_waves(g.sigma), int64_t(nnz) <= LOOK_FAR_MAX_NNZ ? LOOK_MAX : LOOK, tile_ptr, h->tile_head, wg_far, h->tile_desc, L.ndesc,
                           reinterpret_cast<uint32_t*>(basep + L.off_carry + slot_off_arrived(g, tile_group_waves(g.sigma))),
                           reinterpret_cast<uint64_t*>(basep + L.off_carry + slot_off_meet(g)), L.carry_slot_bytes,
                           one_launch_fits(g.sigma, g.p) ? int(CARRY_SLOTS) : 0, reinterpret_cast<uint2*>(basep + L.off_span), h->status);
        e = hipGetLastError();
    }
    if (e == hipSuccess && m > 0) {   // steps 2b + 3a
        hipLaunchKernelGGL(k_rows<IT>, dim3(uint32_t((size_t(m) + 255) / 256)), dim3(256), 0, s, m, nnz,
                           row_ptr, g.sigma, g.T, g.W, g.p, g.pc, tile_ptr, h->tile_desc, wg_far, n_far_wg, h->status);
        e = hipGetLastError();
    }
    if (e == hipSuccess && nnz > 0) {   // steps 3b (descriptors, inside the same kernel) + 4
        switch (sigma) {
#define X(S) case S: e = launch_transpose<S, false, VT>(g, n, nnz, col_idx, val, h->status, h->last_col,      \
                                                        static_cast<VT*>(h->last_val), tile_ptr, h->tile_desc, \
                                                        eop, wide ? 1 : 0, s); break;
            CSR5_FOR_SIGMA(X)
#undef X
            default: e = hipErrorInvalidValue;
        }
    }
    if (e == hipSuccess && g.pc <= SCAN_SINGLE) {
        hipLaunchKernelGGL(k_scan_eop<IT>, dim3(1), dim3(SCAN_THREADS), 0, s, g.pc, g.p, eop, tile_ptr, h->status);
        e = hipGetLastError();
    } else if (e == hipSuccess) {
        IT* chunk_sum = reinterpret_cast<IT*>(basep + L.off_scan);
        const int nchunks = (g.pc + SCAN_CHUNK - 1) / SCAN_CHUNK;      // <= 2^26 / 2^13 = SCAN_CHUNK
        hipLaunchKernelGGL(k_scan_chunks<IT>, dim3(nchunks), dim3(SCAN_THREADS), 0, s, g.pc, eop, chunk_sum, h->status);
        e = hipGetLastError();
        if (e == hipSuccess) {
            hipLaunchKernelGGL(k_scan_finish<IT>, dim3(nchunks), dim3(SCAN_THREADS), 0, s, g.pc, g.p, eop, chunk_sum,
                               tile_ptr, h->status);
            e = hipGetLastError();
        }
    }
    if (e == hipSuccess && g.pc > 0 && m > 0) {
        size_t threads = size_t(m) + size_t(g.pc);
        hipLaunchKernelGGL(k_empty_offset<IT>, dim3(uint32_t((threads + 255) / 256)), dim3(256), 0, s, m,
                           row_ptr, g.sigma, g.T, g.W, g.pc, tile_ptr, h->tile_desc, eop, h->eo,
                           h->status);
        e = hipGetLastError();
    }
    if (e != hipSuccess) {
        (void)hipStreamSynchronize(s);
        if (h->owned) (void)hipFree(h->owned);
        delete h;
        return CSR5_EHIP;
    }
    if (!(flags & CSR5_FLAG_NO_HOST_CHECK)) {
        // blocking variant: wait for the device-side verdict; on bad input undo the
        // transposition and refuse
        uint32_t st = 0;
        int rc = csr5_status(h, &st);
        if (rc == CSR5_OK && (st & BAD_BITS)) {
            (void)csr5_to_csr(h, hip_stream);
            (void)hipStreamSynchronize(s);
            rc = CSR5_EINVAL;
        }
        if (rc != CSR5_OK) {
            if (h->owned) (void)hipFree(h->owned);
            delete h;
            return rc;
        }
    }
    *out = h;
    return CSR5_OK;
}

extern "C" {

int csr5_convert_ex(int32_t m, int32_t n, int32_t nnz, const int32_t* row_ptr, int32_t* col_idx,
                    double* val, int32_t sigma, void* workspace, size_t workspace_bytes,
                    void* hip_stream, uint32_t flags, csr5_handle_t* out) {
    return convert_impl<double, int32_t>(m, n, nnz, row_ptr, col_idx, val, sigma, workspace, workspace_bytes,
                                         hip_stream, flags, out);
}

int csr5l_convert_ex(int32_t m, int32_t n, int64_t nnz, const int64_t* row_ptr, int32_t* col_idx,
                     double* val, int32_t sigma, void* workspace, size_t workspace_bytes,
                     void* hip_stream, uint32_t flags, csr5_handle_t* out) {
    return convert_impl<double, int64_t>(m, n, nnz, row_ptr, col_idx, val, sigma, workspace, workspace_bytes,
                                         hip_stream, flags, out);
}

int csr5s_convert_ex(int32_t m, int32_t n, int32_t nnz, const int32_t* row_ptr, int32_t* col_idx,
                     float* val, int32_t sigma, void* workspace, size_t workspace_bytes,
                     void* hip_stream, uint32_t flags, csr5_handle_t* out) {
    return convert_impl<float, int32_t>(m, n, nnz, row_ptr, col_idx, val, sigma, workspace, workspace_bytes,
                                        hip_stream, flags, out);
}

int csr5_convert(int32_t m, int32_t n, int32_t nnz, const int32_t* row_ptr, int32_t* col_idx,
                 double* val, csr5_handle_t* out) {
    return csr5_convert_ex(m, n, nnz, row_ptr, col_idx, val, 0, nullptr, 0, nullptr, CSR5_FLAG_NONE, out);
}

}  // extern "C"

// One SpMV: the tile kernel, then the carry fix-up if this matrix needs it.
// `which` selects the launches (measurement only): bit 0 the tile kernel, bit 1
// the fix-up.
constexpr int LAUNCH_TILES = 1, LAUNCH_FIXUP = 2, LAUNCH_BOTH = 3;

template <typename VT, typename IT>
static int spmv_launch_it(csr5_handle_t h, const VT* x, VT* y, hipStream_t s, int which, void* carry_mem) {
    using tp_t = typename Index<IT>::tp_t;
    const IT* row_ptr = static_cast<const IT*>(h->row_ptr);
    const tp_t* tile_ptr = static_cast<const tp_t*>(h->tile_ptr);
    const IT* eop = static_cast<const IT*>(h->eop);
    hipError_t e = hipSuccess;
    // a whole SpMV takes the next of the handle's carry arrays; partial launches (measurement) the first
    const uint32_t turn = (which == LAUNCH_BOTH) ? h->carry_turn.fetch_add(1, std::memory_order_relaxed) % CARRY_SLOTS : 0u;
    VT* carry = static_cast<VT*>(carry_mem ? carry_mem : static_cast<void*>(static_cast<char*>(h->carry) + turn * h->carry_slot_bytes));
    // What the matrix needs beyond its tiles is known once the host has seen the
    // status word of the conversion; until then everything is launched (the
    // kernels look at the status word themselves and return at once if idle).
    const int32_t known = h->status_host.load(std::memory_order_relaxed);
    const bool zero_rows = known < 0 || (uint32_t(known) & CSR5_STATUS_HAS_EMPTY_ROWS);
    const bool carries = known < 0 || (uint32_t(known) & STATUS_NEEDS_CARRY) || !h->last_col;
    // the instantiation without the look-behind when the matrix is known not to use it
    const bool can_look = h->last_col && (known < 0 || !(uint32_t(known) & STATUS_NEEDS_CARRY));
    // can the look-behind of this matrix need the far part of the records
    const uint32_t far_mode = (known < 0 || (uint32_t(known) & STATUS_FAR_HEADS)) ? 1u : 0u;
    // The auxiliary-array path in one launch: when the matrix is known to take that
    // path, is small enough for it to pay, and the call uses the handle's own slot
    // (whose counters the conversion cleared).
    const bool one_pays = h->g.p <= ONE_LAUNCH_ANY_TILES || h->nnz / (h->m > 0 ? h->m : 1) < ONE_LAUNCH_SHORT_ROWS;
    const bool one = !carry_mem && known >= 0 && !can_look && h->span &&
                     (h->aux_form == 2 || (h->aux_form == 0 && one_pays));
    uint64_t* const meet = reinterpret_cast<uint64_t*>(reinterpret_cast<char*>(carry) + slot_off_meet(h->g));
    uint32_t* const arrived = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(carry) + slot_off_arrived(h->g, tile_group_waves(h->g.sigma)));
#define ARGS h->g, h->m, h->n, IT(h->nnz), row_ptr, tile_ptr, h->tile_desc, eop, h->eo, h->col_idx,              \
             static_cast<const VT*>(h->val), x, y, carry, meet, arrived, h->span, h->status, h->tile_head, h->last_col, \
             static_cast<const VT*>(h->last_val), zero_rows, far_mode, s
    if (which & LAUNCH_TILES) {
#define X(S) case S:                                                                                  \
        if (look_sigma(S) && can_look) e = launch_spmv<S, VT, IT, look_sigma(S) ? MODE_LOOK : MODE_CARRY>(ARGS); \
        else if (look_sigma(S) && one) e = launch_spmv<S, VT, IT, look_sigma(S) ? MODE_ONE : MODE_CARRY>(ARGS);  \
        else e = launch_spmv<S, VT, IT, MODE_CARRY>(ARGS);                                            \
        break;
        switch (h->g.sigma) {
            CSR5_FOR_SIGMA(X)
            default: e = hipErrorInvalidValue;
        }
#undef X
#undef ARGS
    }
    if (e != hipSuccess) return CSR5_EHIP;
    if ((which & LAUNCH_FIXUP) && carries && !one && h->g.p > 0) {
        int ntiles = h->g.p;                                  // one thread per tile
        size_t nb = (size_t(ntiles) + 255) / 256;
        hipLaunchKernelGGL((k_spmv_fixup<VT, IT>), dim3(uint32_t(nb)), dim3(256), 0, s, h->m, ntiles,
                           tile_ptr, carry, y, h->status);
        if (hipGetLastError() != hipSuccess) return CSR5_EHIP;
    }
    return CSR5_OK;
}

// The 64-bit index variant exists for double only.
template <typename VT>
static int spmv_launch(csr5_handle_t h, const VT* x, VT* y, hipStream_t s, int which = LAUNCH_BOTH,
                       void* carry_mem = nullptr) {
    if constexpr (std::is_same<VT, double>::value) {
        if (h->wide) return spmv_launch_it<double, int64_t>(h, x, y, s, which, carry_mem);
    }
    if (h->wide) return CSR5_EINVAL;
    return spmv_launch_it<VT, int32_t>(h, x, y, s, which, carry_mem);
}

template <typename VT>
static int spmv_checked(csr5_handle_t h, const VT* x, VT* y, void* hip_stream, bool static_carry = false) {
    constexpr int want = std::is_same<VT, float>::value ? CSR5_DTYPE_F32 : CSR5_DTYPE_F64;
    if (!h || !h->in_csr5_order || h->dtype != want) return CSR5_EINVAL;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return CSR5_EHIP;
    if (dev != h->device) return CSR5_EINVAL;              // the handle's arrays live on another device
    if (h->m > 0 && !y) return CSR5_EINVAL;
    if (h->nnz > 0 && !x) return CSR5_EINVAL;
    void* carry_mem = nullptr;
    if (static_carry) {
        // one 8-byte slot per tile, the incomplete one included, in the static array
        if ((size_t(h->g.p) + 1) * 8 > size_t(CSR5_STATIC_SCRATCH_BYTES)) return CSR5_ERANGE;
        const int rc = static_scratch(dev, &carry_mem);
        if (rc != CSR5_OK) return rc;
    }
    if (h->m == 0) return CSR5_OK;
    return spmv_launch<VT>(h, x, y, static_cast<hipStream_t>(hip_stream), LAUNCH_BOTH, carry_mem);
}

template <typename VT>
static int spmv_profile(csr5_handle_t h, const VT* x, VT* y, void* hip_stream, int reps, float* ms) {
    constexpr int want = std::is_same<VT, float>::value ? CSR5_DTYPE_F32 : CSR5_DTYPE_F64;
    if (!h || !h->in_csr5_order || h->dtype != want || !ms || reps <= 0 || reps > 100000) return CSR5_EINVAL;
    if (h->m == 0 || !y || (h->nnz > 0 && !x)) return CSR5_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // Each kernel is launched `reps` times in a row between two events: consecutive
    // launches hide each other's dispatch latency, so elapsed / reps is the kernel's
    // duration (an event pair around a single launch would add that latency).
    // What the repeated launches leave in y is overwritten by the full SpMV at the end.
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    int rc = CSR5_OK;
    for (int k = 0; k < 3 && rc == CSR5_OK; k++)
        if (hipEventCreate(&ev[k]) != hipSuccess) rc = CSR5_EHIP;
    if (rc == CSR5_OK && hipEventRecord(ev[0], s) != hipSuccess) rc = CSR5_EHIP;
    for (int r = 0; rc == CSR5_OK && r < reps; r++) rc = spmv_launch<VT>(h, x, y, s, LAUNCH_TILES);
    if (rc == CSR5_OK && hipEventRecord(ev[1], s) != hipSuccess) rc = CSR5_EHIP;
    for (int r = 0; rc == CSR5_OK && r < reps; r++) rc = spmv_launch<VT>(h, x, y, s, LAUNCH_FIXUP);
    if (rc == CSR5_OK && hipEventRecord(ev[2], s) != hipSuccess) rc = CSR5_EHIP;
    if (rc == CSR5_OK) rc = spmv_launch<VT>(h, x, y, s);
    if (hipStreamSynchronize(s) != hipSuccess && rc == CSR5_OK) rc = CSR5_EHIP;
    float a = 0.f, b = 0.f;
    if (rc == CSR5_OK && (hipEventElapsedTime(&a, ev[0], ev[1]) != hipSuccess ||
                          hipEventElapsedTime(&b, ev[1], ev[2]) != hipSuccess))
        rc = CSR5_EHIP;
    for (int k = 0; k < 3; k++)
        if (ev[k]) (void)hipEventDestroy(ev[k]);
    if (rc == CSR5_OK) {
        ms[0] = a / float(reps);   // tile kernel
        ms[1] = b / float(reps);   // carry fix-up
    }
    return rc;
}

template <typename VT, typename IT>
static int stream_floor(csr5_handle_t h, VT* y, hipStream_t s, int reps, float* ms) {
    using tp_t = typename Index<IT>::tp_t;
    const Geom& g = h->g;
    const uint32_t nb_tiles = uint32_t((g.pc + FLOOR_WAVES - 1) / FLOOR_WAVES);
    // the tile order the SpMV uses for this matrix
    const size_t x_bytes = size_t(h->n) * sizeof(VT);
    uint32_t xcd_chunk = 0;
    if (x_bytes > XCD_CONTIGUOUS_MAX_X_BYTES)
        xcd_chunk = (h->nnz / (h->m > 0 ? h->m : 1) <= g.T / Y_LINE_ROWS) ? 1u : XCD_CHUNK;
    else if (x_bytes < XCD_CONTIGUOUS_MIN_X_BYTES)
        xcd_chunk = XCD_CHUNK;
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    int rc = CSR5_OK;
    for (int k = 0; k < 3 && rc == CSR5_OK; k++)
        if (hipEventCreate(&ev[k]) != hipSuccess) rc = CSR5_EHIP;
    for (int pass = 0; pass < 2 && rc == CSR5_OK; pass++) {      // reads only, then reads and the rows of y
        if (hipEventRecord(ev[pass], s) != hipSuccess) rc = CSR5_EHIP;
        for (int r = 0; rc == CSR5_OK && r < reps; r++) {
            hipLaunchKernelGGL((k_stream_floor<VT, IT>), dim3(nb_tiles), dim3(FLOOR_WAVES * OMEGA), 0, s, h->m, g.pc,
                               g.sigma, g.W, nb_tiles, xcd_chunk, pass, static_cast<const tp_t*>(h->tile_ptr),
                               h->tile_desc, h->col_idx, static_cast<const VT*>(h->val), y);
            if (hipGetLastError() != hipSuccess) rc = CSR5_EHIP;
        }
    }
    if (rc == CSR5_OK && hipEventRecord(ev[2], s) != hipSuccess) rc = CSR5_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess && rc == CSR5_OK) rc = CSR5_EHIP;
    float a = 0.f, b = 0.f;
    if (rc == CSR5_OK && (hipEventElapsedTime(&a, ev[0], ev[1]) != hipSuccess ||
                          hipEventElapsedTime(&b, ev[1], ev[2]) != hipSuccess))
        rc = CSR5_EHIP;
    for (int k = 0; k < 3; k++)
        if (ev[k]) (void)hipEventDestroy(ev[k]);
    if (rc == CSR5_OK) {
        ms[0] = a / float(reps);
        ms[1] = b / float(reps);
    }
    return rc;
}

extern "C" {

int csr5_stream_floor(csr5_handle_t h, void* y, size_t y_bytes, void* hip_stream, int reps, float* ms) {
    if (!h || !h->in_csr5_order || !y || !ms || reps <= 0 || reps > 100000) return CSR5_EINVAL;
    if (h->g.pc == 0 || h->m == 0) return CSR5_EINVAL;                     // no complete tile: nothing to stream
    if (y_bytes < size_t(h->m) * (h->dtype == CSR5_DTYPE_F32 ? 4 : 8)) return CSR5_EINVAL;
    if ((reinterpret_cast<uintptr_t>(h->col_idx) & 15) || (reinterpret_cast<uintptr_t>(h->val) & 15)) return CSR5_EINVAL;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return CSR5_EHIP;
    if (dev != h->device) return CSR5_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (h->dtype == CSR5_DTYPE_F32) return h->wide ? CSR5_EINVAL : stream_floor<float, int32_t>(h, static_cast<float*>(y), s, reps, ms);
    return h->wide ? stream_floor<double, int64_t>(h, static_cast<double*>(y), s, reps, ms)
                   : stream_floor<double, int32_t>(h, static_cast<double*>(y), s, reps, ms);
}

int csr5_spmv_ex(csr5_handle_t h, const double* x, double* y, void* hip_stream) {
    return spmv_checked<double>(h, x, y, hip_stream);
}
int csr5_spmv(csr5_handle_t h, const double* x, double* y) { return spmv_checked<double>(h, x, y, nullptr); }
int csr5_spmv_static(csr5_handle_t h, const double* x, double* y, void* hip_stream) {
    return spmv_checked<double>(h, x, y, hip_stream, true);
}
int csr5s_spmv_ex(csr5_handle_t h, const float* x, float* y, void* hip_stream) {
    return spmv_checked<float>(h, x, y, hip_stream);
}
int csr5_spmv_profile(csr5_handle_t h, const double* x, double* y, void* hip_stream, int reps, float* ms) {
    return spmv_profile<double>(h, x, y, hip_stream, reps, ms);
}
int csr5s_spmv_profile(csr5_handle_t h, const float* x, float* y, void* hip_stream, int reps, float* ms) {
    return spmv_profile<float>(h, x, y, hip_stream, reps, ms);
}

int csr5_to_csr(csr5_handle_t h, void* hip_stream) {
    if (!h) return CSR5_EINVAL;
    if (!h->in_csr5_order) return CSR5_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipSuccess;
    if (h->nnz > 0) {
        switch (h->g.sigma) {
#define X(S) case S: e = (h->dtype == CSR5_DTYPE_F32)                                                            \
        ? launch_transpose<S, true, float>(h->g, h->n, h->nnz, h->col_idx, static_cast<float*>(h->val), h->status,     \
                                           nullptr, nullptr, nullptr, nullptr, nullptr, 0, s)                           \
        : launch_transpose<S, true, double>(h->g, h->n, h->nnz, h->col_idx, static_cast<double*>(h->val), h->status,   \
                                            nullptr, nullptr, nullptr, nullptr, nullptr, 0, s);                         \
        break;
            CSR5_FOR_SIGMA(X)
#undef X
            default: e = hipErrorInvalidValue;
        }
    }
    if (e != hipSuccess) return CSR5_EHIP;
    h->in_csr5_order = false;
    return CSR5_OK;
}

int csr5_free(csr5_handle_t h) {
    if (!h) return CSR5_OK;
    int rc = CSR5_OK;
    if (h->owned && hipFree(h->owned) != hipSuccess) rc = CSR5_EHIP;
    delete h;
    return rc;
}

int csr5_status(csr5_handle_t h, uint32_t* status) {
    if (!h || !status) return CSR5_EINVAL;
    if (hipMemcpyAsync(status, h->status, 4, hipMemcpyDeviceToHost, h->conv_stream) != hipSuccess) return CSR5_EHIP;
    if (hipStreamSynchronize(h->conv_stream) != hipSuccess) return CSR5_EHIP;
    h->status_host.store(int32_t(*status & 0x7fffffffu), std::memory_order_relaxed);
    *status &= STATUS_PUBLIC;
    return CSR5_OK;
}

int csr5_get_info(csr5_handle_t h, int32_t* omega, int32_t* sigma, int32_t* p, int32_t* p_complete,
                  int32_t* desc_words_per_lane, int32_t* empty_offset_len) {
    if (!h) return CSR5_EINVAL;
    if (omega) *omega = OMEGA;
    if (sigma) *sigma = h->g.sigma;
    if (p) *p = h->g.p;
    if (p_complete) *p_complete = h->g.pc;
    if (desc_words_per_lane) *desc_words_per_lane = h->g.W;
    if (empty_offset_len) {
        int64_t v = 0;
        const size_t isz = h->wide ? 8 : 4;   // little-endian host: a 4-byte count lands in the low half
        const char* src = static_cast<const char*>(h->eop) + size_t(h->g.pc) * isz;
        if (hipMemcpyAsync(&v, src, isz, hipMemcpyDeviceToHost, h->conv_stream) != hipSuccess) return CSR5_EHIP;
        if (hipStreamSynchronize(h->conv_stream) != hipSuccess) return CSR5_EHIP;
        if (v < 0 || v > INT32_MAX) return CSR5_ERANGE;
        *empty_offset_len = int32_t(v);
    }
    return CSR5_OK;
}

int csr5_get_shape(csr5_handle_t h, int32_t* m, int32_t* n) {
    if (!h) return CSR5_EINVAL;
    if (m) *m = h->m;
    if (n) *n = h->n;
    return CSR5_OK;
}

int csr5_get_arrays(csr5_handle_t h, const uint32_t** tile_ptr, const uint32_t** tile_desc,
                    const int32_t** empty_offset_ptr, const int32_t** empty_offset) {
    if (!h || h->wide) return CSR5_EINVAL;
    if (tile_ptr) *tile_ptr = static_cast<const uint32_t*>(h->tile_ptr);
    if (tile_desc) *tile_desc = h->tile_desc;
    if (empty_offset_ptr) *empty_offset_ptr = static_cast<const int32_t*>(h->eop);
    if (empty_offset) *empty_offset = h->eo;
    return CSR5_OK;
}

int csr5l_get_arrays(csr5_handle_t h, const uint64_t** tile_ptr, const uint32_t** tile_desc,
                     const int64_t** empty_offset_ptr, const int32_t** empty_offset) {
    if (!h || !h->wide) return CSR5_EINVAL;
    if (tile_ptr) *tile_ptr = static_cast<const uint64_t*>(h->tile_ptr);
    if (tile_desc) *tile_desc = h->tile_desc;
    if (empty_offset_ptr) *empty_offset_ptr = static_cast<const int64_t*>(h->eop);
    if (empty_offset) *empty_offset = h->eo;
    return CSR5_OK;
}

int csr5_baseline_csr_scalar(int32_t m, const int32_t* row_ptr, const int32_t* col_idx, const double* val,
                             const double* x, double* y, void* hip_stream) {
    if (m < 0 || !row_ptr || (m > 0 && !y)) return CSR5_EINVAL;
    if (m == 0) return CSR5_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(k_csr_scalar, dim3(uint32_t((size_t(m) + 255) / 256)), dim3(256), 0, s, m, row_ptr,
                       col_idx, val, x, y);
    return hipGetLastError() == hipSuccess ? CSR5_OK : CSR5_EHIP;
}

int csr5_baseline_csr_vector(int32_t m, int32_t nnz, const int32_t* row_ptr, const int32_t* col_idx,
                             const double* val, const double* x, double* y, int32_t lanes_per_row,
                             void* hip_stream) {
    if (m < 0 || nnz < 0 || !row_ptr || (m > 0 && !y)) return CSR5_EINVAL;
    if (m == 0) return CSR5_OK;
    if (lanes_per_row == 0) {   // smallest power of two >= nnz/row, between 2 and 64
        int64_t q = nnz / m;
        lanes_per_row = 2;
        while (lanes_per_row < 64 && lanes_per_row < q) lanes_per_row *= 2;
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    size_t threads = size_t(m) * size_t(lanes_per_row);
    dim3 grid(uint32_t((threads + 255) / 256)), block(256);
    if (threads / 256 >= 0x7fffffffull) return CSR5_EINVAL;
    switch (lanes_per_row) {
#define X(L) case L: hipLaunchKernelGGL(k_csr_vector<L>, grid, block, 0, s, m, row_ptr, col_idx, val, x, y); break;
        X(2) X(4) X(8) X(16) X(32) X(64)
#undef X
        default: return CSR5_EINVAL;
    }
    return hipGetLastError() == hipSuccess ? CSR5_OK : CSR5_EHIP;
}

int csr5_read_array(csr5_handle_t h, int which, void* dst_host, size_t bytes) {
    if (!h || (!dst_host && bytes)) return CSR5_EINVAL;
    const void* src = nullptr;
    size_t have = 0;
    switch (which) {
        case CSR5_ARRAY_TILE_PTR: src = h->tile_ptr; have = (size_t(h->g.p) + 1) * (h->wide ? 8 : 4); break;
        case CSR5_ARRAY_TILE_DESC: src = h->tile_desc; have = size_t(h->g.pc) * h->g.W * OMEGA * 4; break;
        case CSR5_ARRAY_EMPTY_OFFSET_PTR: src = h->eop; have = (size_t(h->g.pc) + 1) * (h->wide ? 8 : 4); break;
        case CSR5_ARRAY_EMPTY_OFFSET: {
            int32_t len = 0;
            int rc = csr5_get_info(h, nullptr, nullptr, nullptr, nullptr, nullptr, &len);
            if (rc != CSR5_OK) return rc;
            src = h->eo; have = size_t(len) * 4;
            break;
        }
        default: return CSR5_EINVAL;
    }
    if (bytes > have) return CSR5_EINVAL;
    if (bytes == 0) return CSR5_OK;
    if (hipMemcpyAsync(dst_host, src, bytes, hipMemcpyDeviceToHost, h->conv_stream) != hipSuccess) return CSR5_EHIP;
    if (hipStreamSynchronize(h->conv_stream) != hipSuccess) return CSR5_EHIP;
    return CSR5_OK;
}

}  // extern "C"
