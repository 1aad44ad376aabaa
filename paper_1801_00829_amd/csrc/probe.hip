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

}  // namespace

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
