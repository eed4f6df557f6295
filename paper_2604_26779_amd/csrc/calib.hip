// Plain streaming kernels of known size: the measured HBM ceiling that roofline figures are read
// against, and the reference against which hardware traffic counters are scaled.
#include "common.h"

namespace specv {

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// every workgroup walks the buffer with a grid stride; 16 bytes per lane, 4 loads in flight per lane
__global__ __launch_bounds__(256) void calib_read_kernel(const u32x4_t* __restrict__ src, int64_t n16, unsigned int* __restrict__ sink)
{
    int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    u32x4_t acc = {0u, 0u, 0u, 0u};
    for (; i + 3 * stride < n16; i += 4 * stride) {
        u32x4_t a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride);
        u32x4_t c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    unsigned int r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (r == 0x9e3779b9u) sink[0] = r;          // practically never: keeps the loads alive
}

__global__ __launch_bounds__(256) void calib_copy_kernel(u32x4_t* __restrict__ dst, const u32x4_t* __restrict__ src, int64_t n16)
{
    int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace specv

extern "C" spec_status spec_calib_read(const void* dev_src, size_t bytes, void* dev_sink4, int32_t workgroups, void* stream)
{
    using namespace specv;
    if (!dev_src || !dev_sink4 || bytes < 16 || workgroups < 1 || ((uintptr_t)dev_src & 15)) { set_error("spec_calib_read: bad argument"); return SPEC_EINVAL; }
    calib_read_kernel<<<workgroups, 256, 0, (hipStream_t)stream>>>((const u32x4_t*)dev_src, (int64_t)(bytes / 16), (unsigned int*)dev_sink4);
    SPEC_LAUNCH_CHECK("calib_read_kernel");
    return SPEC_OK;
}

extern "C" spec_status spec_calib_copy(void* dev_dst, const void* dev_src, size_t bytes, int32_t workgroups, void* stream)
{
    using namespace specv;
    if (!dev_src || !dev_dst || bytes < 16 || workgroups < 1 || (((uintptr_t)dev_src | (uintptr_t)dev_dst) & 15)) { set_error("spec_calib_copy: bad argument"); return SPEC_EINVAL; }
    calib_copy_kernel<<<workgroups, 256, 0, (hipStream_t)stream>>>((u32x4_t*)dev_dst, (const u32x4_t*)dev_src, (int64_t)(bytes / 16));
    SPEC_LAUNCH_CHECK("calib_copy_kernel");
    return SPEC_OK;
}
