// Fixed device workspace of the entry point that allocates nothing (fuse_magg_noalloc):
// the block partials and the arrival counter of a full aggregate live in a file-scope
// device array instead of the per-stream workspace that the other entry points hipMalloc.
//
// Every GPU holds its own copy of the array at its own address until the process ends.  The
// array's name is only a host-side handle: its device address is asked for once per device
// (hipGetSymbolAddress, with that device current) and kept; kernels and launches get that
// address, never the name.  All calls on one GPU share the array, so calls of this entry point
// that overlap on one GPU (two streams, two host threads) race; calls on one stream are ordered.
#include <hip/hip_runtime.h>

#include <mutex>
#include <string>

#include "../../include/fuse.h"
#include "runtime.h"

namespace {

constexpr size_t kTicketBytes = 256;                                     // arrival counter (first word) + padding
constexpr size_t kScratchBytes = kTicketBytes + FUSE_NOALLOC_MAX_PARTIALS * sizeof(double);

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// The arrival counter must be zero when a full aggregate starts.  A finished launch leaves it at zero,
// but the array keeps whatever the last call left (a launch that was aborted, another user of the
// array), so every call clears it on its own stream first -- with a kernel, not a memset, so that the
// call can be recorded into a HIP graph.
__global__ void __launch_bounds__(64) noalloc_reset_kernel(unsigned int *ticket)
{
    ticket[threadIdx.x] = 0u;                                            // 64 words = kTicketBytes
}

std::mutex g_mu;
constexpr int kMaxDevices = 64;
unsigned char *g_ptr[kMaxDevices];                                       // device address of `scratch`, per device

}  // namespace

namespace fuse {

int noalloc_workspace(hipStream_t stream, Workspace &ws, std::string &err)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        err = std::string("fuse_magg_noalloc: hipGetDevice: ") + (e != hipSuccess ? hipGetErrorString(e) : "device index out of range");
        return FUSE_ERUNTIME;
    }
    unsigned char *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        if (!g_ptr[dev]) {
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));            // the current device's copy
            if (e != hipSuccess || !p) {
                err = std::string("fuse_magg_noalloc: hipGetSymbolAddress: ") + hipGetErrorString(e);
                return FUSE_ERUNTIME;
            }
            g_ptr[dev] = static_cast<unsigned char *>(p);
        }
        ptr = g_ptr[dev];
    }
    noalloc_reset_kernel<<<1, 64, 0, stream>>>(reinterpret_cast<unsigned int *>(ptr));
    e = hipGetLastError();
    if (e != hipSuccess) {
        err = std::string("fuse_magg_noalloc: clearing the arrival counter: ") + hipGetErrorString(e);
        return FUSE_ERUNTIME;
    }
    ws.ticket = reinterpret_cast<unsigned int *>(ptr);
    ws.partials = reinterpret_cast<double *>(ptr + kTicketBytes);
    ws.partial_doubles = FUSE_NOALLOC_MAX_PARTIALS;
    return 0;
}

// ticket[0 .. 64) = 0 on `stream` (the arrival counter of a freshly allocated per-stream workspace: cleared by a
// kernel on the caller's stream, like every other operation of a call, not by a host-synchronous memset)
int reset_ticket_launch(unsigned int *ticket, hipStream_t stream)
{
    noalloc_reset_kernel<<<1, 64, 0, stream>>>(ticket);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace fuse
