// Transposition of a CSR matrix on the device: for every column the list of (row, value) pairs
// of its stored cells.  Used by the left_mm variant of the Outer template (Table 1),
// which accumulates into output row j over the stored cells of COLUMN j: with the transposed
// pattern it becomes the right_mm traversal (one group of lanes owns an output row, no atomics on
// the output).  A counting sort by column in two levels, so that all counting happens in LDS:
//   1. the columns are cut into at most 1024 ranges of 2^s columns; blocks of rows count their
//      cells per range (LDS histogram), an exclusive scan over (range, block) gives every block
//      its place in every range, and the blocks write (column, row, value) there;
//   2. one block per range counts its cells per column (LDS), scans the counts -- these are the
//      column offsets of the transposed matrix -- and moves (row, value) to their final places.
// Matrices with more than 1024 * 8192 columns take the plain form instead: one global atomic per
// cell for the counts and one for the places.  The order of the cells inside a column is
// whatever the atomics produce.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>

#include "runtime.h"

namespace {

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 8;
constexpr int SCAN_CHUNK = SCAN_THREADS * SCAN_ITEMS;

template <typename T>
__global__ void __launch_bounds__(256) zero_kernel(T *__restrict__ p, long long n)
{
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256)
        p[i] = 0;
}

// cnt[c] = number of stored cells in column c (indices outside [0, n) are ignored)
template <typename RP>
__global__ void __launch_bounds__(256) count_kernel(const int *__restrict__ colidx, long long nnz, long long n,
                                                    RP *__restrict__ cnt)
{
    for (long long p = (long long)blockIdx.x * 256 + threadIdx.x; p < nnz; p += (long long)gridDim.x * 256) {
        const long long c = colidx[p];
        if (c >= 0 && c < n)
            atomicAdd(&cnt[c], (RP)1);
    }
}

// exclusive prefix sum of the block's thread values; returns this thread's offset, *total = block sum
template <typename RP, int NT = SCAN_THREADS>
__device__ __forceinline__ RP block_exclusive_scan(RP v, RP *total)
{
    __shared__ RP wsum[NT / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    RP inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const RP t = __shfl_up(inc, d, 64);
        if (lane >= d)
            inc += t;
    }
    __syncthreads();                      // (wsum may still be read from the previous call)
    if (lane == 63)
        wsum[wave] = inc;
    __syncthreads();
    RP before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
        if (w < wave)
            before += wsum[w];
        all += wsum[w];
    }
    *total = all;
    return before + inc - v;
}

// phase A: bsum[b] = sum of the counts of chunk b
template <typename RP>
__global__ void __launch_bounds__(SCAN_THREADS) scan_sums_kernel(const RP *__restrict__ cnt, long long n,
                                                                 RP *__restrict__ bsum)
{
    const long long base = (long long)blockIdx.x * SCAN_CHUNK + (long long)threadIdx.x * SCAN_ITEMS;
    RP s = 0;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i)
        if (base + i < n)
            s += cnt[base + i];
    RP total;
    (void)block_exclusive_scan(s, &total);
    if (threadIdx.x == 0)
        bsum[blockIdx.x] = total;
}

// phase B (one block): bsum becomes its own exclusive prefix sum
template <typename RP>
__global__ void __launch_bounds__(SCAN_THREADS) scan_bsums_kernel(RP *__restrict__ bsum, long long nb)
{
    RP carry = 0;
    for (long long b0 = 0; b0 < nb; b0 += SCAN_THREADS) {
        const long long i = b0 + threadIdx.x;
        const RP v = i < nb ? bsum[i] : 0;
        RP total;
        const RP off = block_exclusive_scan(v, &total);
        if (i < nb)
            bsum[i] = carry + off;
        carry += total;
    }
}

// phase C: next[c] = sum of the values before c (in place); the same goes to copy[c] and the grand
// total to copy[n] (copy may be null) and to *total (may be null)
template <typename RP>
__global__ void __launch_bounds__(SCAN_THREADS) scan_apply_kernel(RP *__restrict__ next, long long n,
                                                                  const RP *__restrict__ bsum, RP *__restrict__ tptr,
                                                                  RP *__restrict__ total_out)
{
    const long long base = (long long)blockIdx.x * SCAN_CHUNK + (long long)threadIdx.x * SCAN_ITEMS;
    RP v[SCAN_ITEMS];
    RP s = 0;
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        v[i] = base + i < n ? next[base + i] : 0;
        s += v[i];
    }
    RP total;
    RP off = block_exclusive_scan(s, &total) + bsum[blockIdx.x];
#pragma unroll
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        if (base + i < n) {
            next[base + i] = off;
            if (tptr)
                tptr[base + i] = off;
        }
        off += v[i];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == SCAN_THREADS - 1) {
        if (tptr)
            tptr[n] = off;                // (the last thread's running offset has passed every entry)
        if (total_out)
            *total_out = off;
    }
}

// ---- two-level form -------------------------------------------------------------------------
struct __attribute__((aligned(16))) Cell {       // one stored cell between the two levels: one 16-byte store
    int col, row;
    double val;
};
constexpr int RANGE_THREADS = 1024;       // level 2
constexpr int PART_THREADS = 1024;        // level 1: 64 rows in flight per block
constexpr int MAX_RANGES = 1024;
constexpr int MAX_RANGE_SHIFT = 13;       // 8192 columns per range: 32 KB of LDS counters

// level 1, counting: hist[range * nblk + block] = cells of the block's rows in the column range
template <typename RP, typename XRP>
__global__ void __launch_bounds__(PART_THREADS) part_hist_kernel(const XRP *__restrict__ rowptr, const int *__restrict__ colidx,
                                                        long long m, long long n, long long nnz, long long rows_per_block,
                                                        int shift, int nranges, RP *__restrict__ hist)
{
    __shared__ unsigned int cnt[MAX_RANGES];
    for (int i = threadIdx.x; i < nranges; i += PART_THREADS)
        cnt[i] = 0;
    __syncthreads();
    const int k = threadIdx.x & 15;
    const long long row0 = (long long)blockIdx.x * rows_per_block;
    for (long long lr = threadIdx.x >> 4; lr < rows_per_block && row0 + lr < m; lr += PART_THREADS / 16) {
        const long long row = row0 + lr;
        long long rs = (long long)rowptr[row], re = (long long)rowptr[row + 1];
        rs = rs < 0 ? 0 : (rs > nnz ? nnz : rs);
        re = re < rs ? rs : (re > nnz ? nnz : re);
        for (long long e = rs + k; e < re; e += 16) {
            const long long c = colidx[e];
            if (c >= 0 && c < n)
                atomicAdd(&cnt[c >> shift], 1u);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nranges; i += PART_THREADS)
        hist[(long long)i * gridDim.x + blockIdx.x] = (RP)cnt[i];
}

// level 1, moving: the same walk; every cell goes to the next free place of its block inside its range
template <typename RP, typename XRP>
__global__ void __launch_bounds__(PART_THREADS) part_move_kernel(const XRP *__restrict__ rowptr, const int *__restrict__ colidx,
                                                        const double *__restrict__ vals, long long m, long long n,
                                                        long long nnz, long long rows_per_block,
                                                        int shift, int nranges, const RP *__restrict__ place,
                                                        Cell *__restrict__ cells)
{
    __shared__ RP cursor[MAX_RANGES];
    for (int i = threadIdx.x; i < nranges; i += PART_THREADS)
        cursor[i] = place[(long long)i * gridDim.x + blockIdx.x];
    __syncthreads();
    const int k = threadIdx.x & 15;
    const long long row0 = (long long)blockIdx.x * rows_per_block;
    for (long long lr = threadIdx.x >> 4; lr < rows_per_block && row0 + lr < m; lr += PART_THREADS / 16) {
        const long long row = row0 + lr;
        long long rs = (long long)rowptr[row], re = (long long)rowptr[row + 1];
        rs = rs < 0 ? 0 : (rs > nnz ? nnz : rs);
        re = re < rs ? rs : (re > nnz ? nnz : re);
        for (long long e = rs + k; e < re; e += 16) {
            const long long c = colidx[e];
            if (c < 0 || c >= n)
                continue;
            const long long pos = (long long)atomicAdd(&cursor[c >> shift], (RP)1);
            if (pos >= 0 && pos < nnz) {  // (always, unless the arrays change while the call runs)
                cells[pos] = Cell{(int)c, (int)row, vals[e]};
            }
        }
    }
}

// level 2: one block per column range
template <typename RP>
__global__ void __launch_bounds__(RANGE_THREADS) range_sort_kernel(const Cell *__restrict__ cells, const RP *__restrict__ place,
                                                                  const RP *__restrict__ total, long long nblk, int shift,
                                                                  long long n, long long nnz, RP *__restrict__ tptr,
                                                                  int *__restrict__ trow, double *__restrict__ tval)
{
    extern __shared__ unsigned int colcnt[];          // 2^shift counters, then cursors
    const int width = 1 << shift;
    const long long b = blockIdx.x;
    long long s0 = (long long)place[b * nblk];
    long long s1 = b + 1 < gridDim.x ? (long long)place[(b + 1) * nblk] : (long long)*total;
    s0 = s0 < 0 ? 0 : (s0 > nnz ? nnz : s0);
    s1 = s1 < s0 ? s0 : (s1 > nnz ? nnz : s1);
    const long long cbase = b << shift;
    for (int i = threadIdx.x; i < width; i += RANGE_THREADS)
        colcnt[i] = 0;
    __syncthreads();
    for (long long p = s0 + threadIdx.x; p < s1; p += RANGE_THREADS) {
        const long long cl = (long long)cells[p].col - cbase;
        if (cl >= 0 && cl < width)
            atomicAdd(&colcnt[cl], 1u);
    }
    __syncthreads();
    unsigned int carry = 0;
    for (int j0 = 0; j0 < width; j0 += RANGE_THREADS) {
        const int j = j0 + threadIdx.x;
        const unsigned int v = j < width ? colcnt[j] : 0u;
        unsigned int tot;
        const unsigned int off = block_exclusive_scan<unsigned int, RANGE_THREADS>(v, &tot) + carry;
        if (j < width) {
            colcnt[j] = off;
            if (cbase + j < n)
                tptr[cbase + j] = (RP)(s0 + off);
        }
        carry += tot;
    }
    if (b == gridDim.x - 1 && threadIdx.x == 0)
        tptr[n] = (RP)s1;
    __syncthreads();
    for (long long p = s0 + threadIdx.x; p < s1; p += RANGE_THREADS) {
        const Cell c = cells[p];
        const long long cl = (long long)c.col - cbase;
        if (cl < 0 || cl >= width)
            continue;
        const long long pos = s0 + (long long)atomicAdd(&colcnt[cl], 1u);
        if (pos < s1) {
            trow[pos] = c.row;
            tval[pos] = c.val;
        }
    }
}

// scatter: cell e of row i in column c goes to slot next[c]++ of column c.  16 lanes per row.
template <typename RP, typename XRP>
__global__ void __launch_bounds__(256) scatter_kernel(const XRP *__restrict__ rowptr, const int *__restrict__ colidx,
                                                      const double *__restrict__ vals, long long m, long long n,
                                                      long long nnz, RP *__restrict__ next, int *__restrict__ trow,
                                                      double *__restrict__ tval)
{
    const int k = threadIdx.x & 15;
    const long long row = ((long long)blockIdx.x * 256 + threadIdx.x) >> 4;
    if (row >= m)
        return;
    long long rs = (long long)rowptr[row], re = (long long)rowptr[row + 1];
    rs = rs < 0 ? 0 : (rs > nnz ? nnz : rs);
    re = re < rs ? rs : (re > nnz ? nnz : re);
    for (long long e = rs + k; e < re; e += 16) {
        const long long c = colidx[e];
        if (c < 0 || c >= n)
            continue;
        const long long pos = (long long)atomicAdd(&next[c], (RP)1);
        if (pos >= 0 && pos < nnz) {      // (always, unless the arrays change while the call runs)
            trow[pos] = (int)row;
            tval[pos] = vals[e];
        }
    }
}

inline unsigned grid_for(long long items)
{
    return (unsigned)std::max<long long>(1, std::min<long long>((items + 255) / 256, 8192));
}

struct Shape {                   // launch shape of the two-level form
    bool two_level;
    int shift, nranges;
    long long rows_per_block, nblk, nhist;
};

Shape shape_of(long long m, long long n, long long nnz)
{
    Shape s = {};
    int shift = 0;
    while (((n + (1LL << shift) - 1) >> shift) > MAX_RANGES)
        ++shift;
    const char *plain = std::getenv("FUSE_TRANSPOSE_PLAIN");        // (tests: the plain form on small inputs)
    s.two_level = shift <= MAX_RANGE_SHIFT && nnz < 4294967296LL && !(plain && plain[0] == '1');
    s.shift = shift;
    s.nranges = (int)((n + (1LL << shift) - 1) >> shift);
    // few, large blocks of rows: a block's cells of one range land next to each other (longer runs of writes)
    const long long want = std::max<long long>(1, std::min<long long>(512, (m + 15) / 16));
    s.rows_per_block = (m + want - 1) / want;
    s.nblk = (m + s.rows_per_block - 1) / s.rows_per_block;
    s.nhist = (long long)s.nranges * s.nblk;
    return s;
}

size_t align16(size_t b) { return (b + 15) / 16 * 16; }

template <typename RP, typename XRP>
int transpose_typed(const void *rowptr, const int *colidx, const double *vals, long long m, long long n, long long nnz,
                    char *scratch, void *tptr_, int *trow, double *tval, hipStream_t stream)
{
    RP *tptr = (RP *)tptr_;
    const Shape sh = shape_of(m, n, nnz);
    if (!sh.two_level) {
        RP *next = (RP *)scratch, *bsum = (RP *)(scratch + align16((size_t)n * sizeof(RP)));
        const long long nb = (n + SCAN_CHUNK - 1) / SCAN_CHUNK;
        zero_kernel<RP><<<grid_for(n), 256, 0, stream>>>(next, n);
        count_kernel<RP><<<grid_for(nnz), 256, 0, stream>>>(colidx, nnz, n, next);
        scan_sums_kernel<RP><<<(unsigned)nb, SCAN_THREADS, 0, stream>>>(next, n, bsum);
        scan_bsums_kernel<RP><<<1, SCAN_THREADS, 0, stream>>>(bsum, nb);
        scan_apply_kernel<RP><<<(unsigned)nb, SCAN_THREADS, 0, stream>>>(next, n, bsum, tptr, (RP *)nullptr);
        const long long gs = (m * 16 + 255) / 256;
        scatter_kernel<RP, XRP><<<(unsigned)gs, 256, 0, stream>>>((const XRP *)rowptr, colidx, vals, m, n, nnz, next, trow, tval);
        return hipGetLastError() == hipSuccess ? 0 : -1;
    }
    // scratch: hist | block sums of its scan | grand total | the cells by range
    const long long nb = (sh.nhist + SCAN_CHUNK - 1) / SCAN_CHUNK;
    char *q = scratch;
    RP *hist = (RP *)q;              q += align16((size_t)sh.nhist * sizeof(RP));
    RP *bsum = (RP *)q;              q += align16((size_t)nb * sizeof(RP));
    RP *total = (RP *)q;             q += 16;
    Cell *cells = (Cell *)q;
    part_hist_kernel<RP, XRP><<<(unsigned)sh.nblk, PART_THREADS, 0, stream>>>((const XRP *)rowptr, colidx, m, n, nnz, sh.rows_per_block,
                                                                    sh.shift, sh.nranges, hist);
    scan_sums_kernel<RP><<<(unsigned)nb, SCAN_THREADS, 0, stream>>>(hist, sh.nhist, bsum);
    scan_bsums_kernel<RP><<<1, SCAN_THREADS, 0, stream>>>(bsum, nb);
    scan_apply_kernel<RP><<<(unsigned)nb, SCAN_THREADS, 0, stream>>>(hist, sh.nhist, bsum, (RP *)nullptr, total);
    part_move_kernel<RP, XRP><<<(unsigned)sh.nblk, PART_THREADS, 0, stream>>>((const XRP *)rowptr, colidx, vals, m, n, nnz,
                                                                    sh.rows_per_block, sh.shift, sh.nranges, hist, cells);
    range_sort_kernel<RP><<<(unsigned)sh.nranges, RANGE_THREADS, (size_t)4 << sh.shift, stream>>>(
        cells, hist, total, sh.nblk, sh.shift, n, nnz, tptr, trow, tval);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace

namespace fuse {

namespace {
__global__ void __launch_bounds__(256) iota_kernel(double *__restrict__ dst, long long n)
{
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256)
        dst[i] = (double)i;
}
}  // namespace

// dst[i] = i as a double (exact below 2^53): "values" that make the transposition carry every cell's place in the
// original arrays along, i.e. produce the permutation instead of permuted values
int iota_launch(double *dst, long long n, hipStream_t stream)
{
    if (n <= 0)
        return 0;
    const long long blocks = (n + 255) / 256;
    iota_kernel<<<(unsigned)(blocks < 4096 ? blocks : 4096), 256, 0, stream>>>(dst, n);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

namespace {
__global__ void __launch_bounds__(256) gather_kernel(double *__restrict__ dst, const double *__restrict__ src,
                                                     const double *__restrict__ perm, long long n)
{
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
        long long p = (long long)__builtin_nontemporal_load(&perm[i]);
        p = p < 0 ? 0 : (p < n ? p : n - 1);               // (a foreign pattern cannot lead outside the array)
        dst[i] = src[p];
    }
}
}  // namespace

// dst[i] = src[perm[i]] for a permutation stored as doubles: the values of a matrix in the order of a prepared pattern
int gather_launch(double *dst, const double *src, const double *perm, long long n, hipStream_t stream)
{
    if (n <= 0)
        return 0;
    const long long blocks = (n + 255) / 256;
    gather_kernel<<<(unsigned)(blocks < 8192 ? blocks : 8192), 256, 0, stream>>>(dst, src, perm, n);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

size_t transpose_scratch_bytes(long long m, long long n, long long nnz, int rowptr_is64)
{
    const size_t rpb = rowptr_is64 ? 8 : 4;
    const Shape sh = shape_of(m, n, nnz);
    if (!sh.two_level)
        return align16((size_t)n * rpb) + align16((size_t)((n + SCAN_CHUNK - 1) / SCAN_CHUNK) * rpb);
    const long long nb = (sh.nhist + SCAN_CHUNK - 1) / SCAN_CHUNK;
    return align16((size_t)sh.nhist * rpb) + align16((size_t)nb * rpb) + 16 + (size_t)nnz * sizeof(Cell);
}

int transpose_launch(const void *rowptr, int rowptr_is64, const int *colidx, const double *vals, long long m, long long n,
                     long long nnz, void *scratch, void *tptr, int *trow, double *tval, hipStream_t stream)
{
    if (m <= 0 || n <= 0 || m > 2147483647LL / 16)
        return -1;
    if (rowptr_is64)
        return transpose_typed<unsigned long long, long long>(rowptr, colidx, vals, m, n, nnz, (char *)scratch, tptr, trow, tval,
                                                              stream);
    return transpose_typed<unsigned int, int>(rowptr, colidx, vals, m, n, nnz, (char *)scratch, tptr, trow, tval, stream);
}

}  // namespace fuse
