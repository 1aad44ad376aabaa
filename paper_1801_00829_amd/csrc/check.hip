// Structure check of a CSR matrix on the device (kernel of fuse_check_csr).
#include <hip/hip_runtime.h>

#include "runtime.h"

namespace {

// bad[0]: first row whose two offsets are out of order or outside [0, nnz]
// bad[1]: first row that stores a column index outside [0, cols)
// bad[2]: first row whose column indices are not strictly ascending
// bad[3]: bit 0: rowptr[0] != 0, bit 1: rowptr[rows] != nnz
// A wave takes one row at a time (its lanes stride over the row's cells), so a few very long rows
// do not serialise on one lane; no cell is read before the row's offsets are known to lie inside
// the arrays.
template <typename RP>
__global__ void __launch_bounds__(256) check_csr_kernel(const RP *__restrict__ rowptr, const int *__restrict__ colidx,
                                                        long long rows, long long cols, long long nnz,
                                                        unsigned long long *__restrict__ bad)
{
    const int lane = threadIdx.x & 63;
    const long long wave = ((long long)blockIdx.x * 256 + threadIdx.x) >> 6;
    const long long nwaves = ((long long)gridDim.x * 256) >> 6;
    if (wave == 0 && lane == 0) {
        unsigned long long f = 0;
        if ((long long)rowptr[0] != 0)
            f |= 1;
        if ((long long)rowptr[rows] != nnz)
            f |= 2;
        if (f)
            atomicOr(&bad[3], f);
    }
    for (long long r = wave; r < rows; r += nwaves) {
        const long long s = (long long)rowptr[r], e = (long long)rowptr[r + 1];
        if (s < 0 || e < s || e > nnz) {
            if (lane == 0)
                atomicMin(&bad[0], (unsigned long long)r);
            continue;
        }
        bool range = false, order = false;
        for (long long p = s + lane; p < e; p += 64) {
            const int c = colidx[p];
            range |= c < 0 || (long long)c >= cols;
            if (p > s)
                order |= colidx[p - 1] >= c;
        }
        if (range)
            atomicMin(&bad[1], (unsigned long long)r);
        if (order)
            atomicMin(&bad[2], (unsigned long long)r);
    }
}

}  // namespace

namespace fuse {

int check_csr_launch(const void *rowptr, int rowptr_is64, const int *colidx, long long rows, long long cols,
                     long long nnz, unsigned long long *bad, hipStream_t stream)
{
    const long long want = (rows + 3) / 4;            // 4 waves per block, one row per wave and step
    const unsigned gx = (unsigned)(want < 1 ? 1 : (want > 8192 ? 8192 : want));
    if (rowptr_is64)
        check_csr_kernel<long long><<<gx, 256, 0, stream>>>((const long long *)rowptr, colidx, rows, cols, nnz, bad);
    else
        check_csr_kernel<int><<<gx, 256, 0, stream>>>((const int *)rowptr, colidx, rows, cols, nnz, bad);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace fuse
