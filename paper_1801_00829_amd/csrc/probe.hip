// Bandwidth probes: a plain copy and a read-only reduction over 16-byte
// vectors.  They give the achievable HBM ceiling of the device and calibrate
// profiler byte counters against a transfer of known size.
#include <hip/hip_runtime.h>

#include "../../include/fuse.h"

namespace {

typedef double double2_t __attribute__((ext_vector_type(2)));

__global__ void __launch_bounds__(256) probe_copy_kernel(double2_t *__restrict__ dst,
                                                         const double2_t *__restrict__ src, long long nvec)
{
    const long long stride = (long long)gridDim.x * 256;
    long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < nvec; i += 4 * stride) {
        double2_t a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a;
        dst[i + stride] = b;
        dst[i + 2 * stride] = c;
        dst[i + 3 * stride] = d;
    }
    for (; i < nvec; i += stride)
        dst[i] = src[i];
}

__global__ void __launch_bounds__(256) probe_read_kernel(const double2_t *__restrict__ src, long long nvec,
                                                         double *__restrict__ sink)
{
    const long long stride = (long long)gridDim.x * 256;
    long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    double acc = 0.0;
    for (; i + 7 * stride < nvec; i += 8 * stride) {
        double2_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            acc += v[u].x + v[u].y;
    }
    for (; i < nvec; i += stride)
        acc += src[i].x + src[i].y;
    if (acc == 123.456789)   // keeps the loads alive; practically never true
        sink[0] = acc;
}

// Gather of whole table rows at random: a group of 8 consecutive lanes reads row idx[k] of the table
// (EPL 16-byte vectors per lane, vector e * 8 + lane, so that a load instruction of the group covers 128
// contiguous bytes) for 4 values of k at a time, all loads issued before any is used -- the access pattern
// of the Outer template's V_j fetch without any of its arithmetic, i.e. the rate at which this device
// serves such gathers from a table of the given size (L2, memory-side cache or HBM resident).
template <int EPL>
__global__ void __launch_bounds__(256) probe_gather_kernel(const double2_t *__restrict__ table, long long ldv, int nvec,
                                                           const int *__restrict__ idx, long long count,
                                                           double *__restrict__ sink)
{
    constexpr int G = 8, UNR = 4;
    const int lig = threadIdx.x & (G - 1);
    const long long ngroups = (long long)gridDim.x * (256 / G);
    long long k = (long long)blockIdx.x * (256 / G) + threadIdx.x / G;
    double acc = 0.0;
    for (; k < count; k += ngroups * UNR) {
        double2_t v[UNR][EPL];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const long long kk = k + u * ngroups;
            const long long row = kk < count ? idx[kk] : idx[k];
            const double2_t *p = table + row * ldv;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const int c = e * G + lig;
                v[u][e] = p[c < nvec ? c : nvec - 1];          // redirected, not predicated: every lane loads
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int e = 0; e < EPL; ++e)
                acc += v[u][e].x + v[u][e].y;
    }
    if (acc == 123.456789)
        sink[0] = acc;
}

}  // namespace

extern "C" int fuse_probe_gather(const double *table, int64_t rows, int64_t row_doubles, int64_t ld,
                                 const int32_t *idx, int64_t count, int blocks, double *sink, void *stream)
{
    if (!table || !idx || !sink || rows < 1 || row_doubles < 2 || (row_doubles & 1) || row_doubles > 128 ||
        ld < row_doubles || (ld & 1) || count < 0 || blocks < 1 || ((uintptr_t)table & 15u))
        return FUSE_EINVAL;
    if (count == 0)
        return FUSE_OK;
    const int nvec = (int)(row_doubles / 2), epl = (nvec + 7) / 8;
    const double2_t *t = (const double2_t *)table;
    hipStream_t s = (hipStream_t)stream;
#define FUSE_GATHER_CASE(E) case E: probe_gather_kernel<E><<<blocks, 256, 0, s>>>(t, ld / 2, nvec, idx, count, sink); break;
    switch (epl) {
        FUSE_GATHER_CASE(1) FUSE_GATHER_CASE(2) FUSE_GATHER_CASE(3) FUSE_GATHER_CASE(4)
        FUSE_GATHER_CASE(5) FUSE_GATHER_CASE(6) FUSE_GATHER_CASE(7) FUSE_GATHER_CASE(8)
    default: return FUSE_EINVAL;
    }
#undef FUSE_GATHER_CASE
    return hipGetLastError() == hipSuccess ? FUSE_OK : FUSE_ERUNTIME;
}

extern "C" int fuse_probe_copy(double *dst, const double *src, int64_t n_doubles, int blocks, void *stream)
{
    if (!dst || !src || n_doubles < 0 || (n_doubles & 1) || blocks < 1)
        return FUSE_EINVAL;
    if (((uintptr_t)dst | (uintptr_t)src) & 15u)
        return FUSE_EINVAL;
    probe_copy_kernel<<<blocks, 256, 0, (hipStream_t)stream>>>((double2_t *)dst, (const double2_t *)src,
                                                              n_doubles / 2);
    return hipGetLastError() == hipSuccess ? FUSE_OK : FUSE_ERUNTIME;
}

extern "C" int fuse_probe_read(const double *src, int64_t n_doubles, int blocks, double *sink, void *stream)
{
    if (!src || !sink || n_doubles < 0 || (n_doubles & 1) || blocks < 1 || ((uintptr_t)src & 15u))
        return FUSE_EINVAL;
    probe_read_kernel<<<blocks, 256, 0, (hipStream_t)stream>>>((const double2_t *)src, n_doubles / 2, sink);
    return hipGetLastError() == hipSuccess ? FUSE_OK : FUSE_ERUNTIME;
}
