// Pattern transposition of a CSR matrix on the device: for every column the list of (row, cell
// index) pairs of its stored cells.  Used by the left_mm variant of the Outer template (Table 1),
// which accumulates into output row j over the stored cells of COLUMN j: with the transposed
// pattern it becomes the right_mm traversal (one group of lanes owns an output row, no atomics on
// the output).  A counting sort by column: count, exclusive scan, scatter.  The order of the cells
// inside a column is whatever the scatter's atomics produce.
#include <hip/hip_runtime.h>

#include <algorithm>

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
template <typename RP>
__device__ __forceinline__ RP block_exclusive_scan(RP v, RP *total)
{
    __shared__ RP wsum[SCAN_THREADS / 64];
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
    for (int w = 0; w < SCAN_THREADS / 64; ++w) {
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

// phase C: tptr[c] = next[c] = number of stored cells in the columns before c; tptr[n] = their total
template <typename RP>
__global__ void __launch_bounds__(SCAN_THREADS) scan_apply_kernel(RP *__restrict__ next, long long n,
                                                                  const RP *__restrict__ bsum, RP *__restrict__ tptr)
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
            tptr[base + i] = off;
        }
        off += v[i];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == SCAN_THREADS - 1)
        tptr[n] = off;                    // (the last thread's running offset has passed every column)
}

// scatter: cell e of row i in column c goes to slot next[c]++ of column c.  16 lanes per row.
template <typename RP, typename XRP>
__global__ void __launch_bounds__(256) scatter_kernel(const XRP *__restrict__ rowptr, const int *__restrict__ colidx,
                                                      long long m, long long n, long long nnz, RP *__restrict__ next,
                                                      int *__restrict__ trow, RP *__restrict__ tperm)
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
            tperm[pos] = (RP)e;
        }
    }
}

template <typename RP, typename XRP>
int transpose_typed(const void *rowptr, const int *colidx, long long m, long long n, long long nnz, void *next_,
                    void *bsum_, void *tptr_, int *trow, void *tperm_, hipStream_t stream)
{
    RP *next = (RP *)next_, *bsum = (RP *)bsum_, *tptr = (RP *)tptr_, *tperm = (RP *)tperm_;
    const long long nb = (n + SCAN_CHUNK - 1) / SCAN_CHUNK;
    auto grid = [](long long items) { return (unsigned)std::max<long long>(1, std::min<long long>((items + 255) / 256, 8192)); };
    zero_kernel<RP><<<grid(n), 256, 0, stream>>>(next, n);
    count_kernel<RP><<<grid(nnz), 256, 0, stream>>>(colidx, nnz, n, next);
    scan_sums_kernel<RP><<<(unsigned)nb, SCAN_THREADS, 0, stream>>>(next, n, bsum);
    scan_bsums_kernel<RP><<<1, SCAN_THREADS, 0, stream>>>(bsum, nb);
    scan_apply_kernel<RP><<<(unsigned)nb, SCAN_THREADS, 0, stream>>>(next, n, bsum, tptr);
    const long long gs = (m * 16 + 255) / 256;
    scatter_kernel<RP, XRP><<<(unsigned)gs, 256, 0, stream>>>((const XRP *)rowptr, colidx, m, n, nnz, next, trow, tperm);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace

namespace fuse {

size_t transpose_scan_blocks(long long n) { return (size_t)((n + SCAN_CHUNK - 1) / SCAN_CHUNK); }

int transpose_launch(const void *rowptr, int rowptr_is64, const int *colidx, long long m, long long n, long long nnz,
                     void *next, void *bsum, void *tptr, int *trow, void *tperm, hipStream_t stream)
{
    if (m <= 0 || n <= 0 || m > 2147483647LL || (m * 16 + 255) / 256 > 2147483647LL)
        return -1;
    if (rowptr_is64)
        return transpose_typed<unsigned long long, long long>(rowptr, colidx, m, n, nnz, next, bsum, tptr, trow, tperm, stream);
    return transpose_typed<unsigned int, int>(rowptr, colidx, m, n, nnz, next, bsum, tptr, trow, tperm, stream);
}

}  // namespace fuse
