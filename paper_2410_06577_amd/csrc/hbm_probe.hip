// Measurement aid, not part of the recurrence: a plain streaming kernel with a chosen mix of reads and writes, so that
// the bandwidth figures of the scan and decode kernels can be set beside what the memory system of the same GPU gives a
// kernel that does nothing else (the published peak is not reachable by any access mix).  Every lane adds up one 16-byte
// unit from each of `reads_per_write` input streams and writes one unit; all accesses are coalesced and streaming.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace rodimus {
namespace {

typedef float floatx4_t __attribute__((ext_vector_type(4)));

template <int kReads>
__global__ __launch_bounds__(256) void hbm_stream_probe_kernel(const floatx4_t *__restrict__ src, floatx4_t *__restrict__ dst, size_t units)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < units; i += stride) {
        floatx4_t acc = {1.f, 2.f, 3.f, 4.f};
#pragma unroll
        for (int r = 0; r < kReads; ++r) acc += __builtin_nontemporal_load(src + (size_t)r * units + i);
        __builtin_nontemporal_store(acc, dst + i);
    }
}

}  // namespace

hipError_t launch_hbm_stream_probe(const void *src, void *dst, size_t units, int reads_per_write, int workgroups, hipStream_t stream)
{
    if (units == 0) return hipSuccess;
    const dim3 grid((unsigned)workgroups), block(256);
    const floatx4_t *s = static_cast<const floatx4_t *>(src);
    floatx4_t *d = static_cast<floatx4_t *>(dst);
    switch (reads_per_write) {
    case 0: hipLaunchKernelGGL(hbm_stream_probe_kernel<0>, grid, block, 0, stream, s, d, units); break;
    case 1: hipLaunchKernelGGL(hbm_stream_probe_kernel<1>, grid, block, 0, stream, s, d, units); break;
    case 2: hipLaunchKernelGGL(hbm_stream_probe_kernel<2>, grid, block, 0, stream, s, d, units); break;
    case 4: hipLaunchKernelGGL(hbm_stream_probe_kernel<4>, grid, block, 0, stream, s, d, units); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace rodimus
