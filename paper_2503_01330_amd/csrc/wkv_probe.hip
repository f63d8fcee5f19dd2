// A plain streaming read with a chosen launch shape: the yardstick the benchmark holds the decode
// step against.  It moves no result anywhere and is no part of the method (Algorithm 1 has no such
// step); it answers one question: how fast can THIS grid pull THIS many bytes out of memory when
// it does nothing else -- the achievable fraction of the 8 TB/s a launch of that size can reach.
#include "../../include/wkv.h"
#include "wkv_internal.h"

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Workgroup b reads the b-th contiguous share of the buffer, 16 bytes per lane and load, DEPTH
// loads in flight per lane; consecutive lanes read consecutive 16-byte pieces (a wave instruction
// covers 1 KiB, as the row loads of the decode kernel do).
template <bool NT, int DEPTH>
__global__ __launch_bounds__(1024)
void wkv_probe_read_kernel(const u32x4_t* __restrict__ src, size_t per_group, uint32_t* __restrict__ sink)
{
    const u32x4_t* p = src + (size_t)blockIdx.x * per_group;
    const size_t nt = blockDim.x;
    uint32_t acc = 0;
    for (size_t i = threadIdx.x; i < per_group; i += DEPTH * nt) {
        u32x4_t x[DEPTH];
#pragma unroll
        for (int k = 0; k < DEPTH; ++k) {
            const size_t j = i + k * nt;
            const u32x4_t* a = p + (j < per_group ? j : i);      // past the end: a harmless repeat
            x[k] = NT ? __builtin_nontemporal_load(a) : *a;
        }
#pragma unroll
        for (int k = 0; k < DEPTH; ++k) acc ^= x[k].x ^ x[k].y ^ x[k].z ^ x[k].w;
    }
    if (acc == 0x9E3779B9u && sink) sink[0] = acc;               // keeps the loads alive; practically never taken
}

}  // namespace

hipError_t wkv_launch_probe_read(const void* src, size_t bytes, int workgroups, int threads, bool nontemporal,
                                 void* sink, hipStream_t stream)
{
    const size_t per_group = bytes / 16 / (size_t)workgroups;
    const u32x4_t* s = static_cast<const u32x4_t*>(src);
    if (nontemporal)
        hipLaunchKernelGGL((wkv_probe_read_kernel<true, 4>), dim3(workgroups), dim3(threads), 0, stream, s, per_group,
                           static_cast<uint32_t*>(sink));
    else
        hipLaunchKernelGGL((wkv_probe_read_kernel<false, 4>), dim3(workgroups), dim3(threads), 0, stream, s, per_group,
                           static_cast<uint32_t*>(sink));
    return hipGetLastError();
}
