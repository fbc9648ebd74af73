// Measurement aids, not part of the finalization pass: a plain copy kernel of known size (to
// calibrate the FETCH_SIZE / WRITE_SIZE hardware counters) and a plain read-and-sum kernel (the
// read-only streaming ceiling of the device, for comparison with the vocabulary reduction).
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t probe_u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void jot_probe_copy_kernel(const probe_u32x4* __restrict__ src,
                                                             probe_u32x4* __restrict__ dst, int64_t n_vec)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < n_vec; k += stride)
        dst[k] = src[k];
}

__global__ __launch_bounds__(256) void jot_probe_read_kernel(const probe_u32x4* __restrict__ src,
                                                             int64_t n_vec, uint32_t* __restrict__ out)
{
    // n_vec is a multiple of 2048 = 256 threads x 8 vectors, so every batch is whole
    const int64_t stride = (int64_t)gridDim.x * 256 * 8;
    uint32_t acc = 0;
    for (int64_t k = (int64_t)blockIdx.x * 256 * 8 + threadIdx.x; k < n_vec; k += stride) {
        probe_u32x4 w[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) w[u] = __builtin_nontemporal_load(src + k + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += w[u].x ^ w[u].y ^ w[u].z ^ w[u].w;
    }
    if (acc == 0x9e3779b9u) out[0] = acc;     // practically never true: keeps the loads alive
}

extern "C" {

// Copies `bytes` (multiple of 16) from src_dev to dst_dev.  Returns the hipError_t of the launch.
int jot_probe_copy(const void* src_dev, void* dst_dev, int64_t bytes, void* stream)
{
    if (bytes <= 0 || bytes % 16) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(jot_probe_copy_kernel, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const probe_u32x4*>(src_dev), static_cast<probe_u32x4*>(dst_dev), bytes / 16);
    return (int)hipGetLastError();
}

// Reads `bytes` (multiple of 32768) from src_dev; out_dev is a 4-byte device scratch word.
int jot_probe_read(const void* src_dev, int64_t bytes, void* out_dev, void* stream)
{
    if (bytes <= 0 || bytes % 32768) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(jot_probe_read_kernel, dim3(256 * 8), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const probe_u32x4*>(src_dev), bytes / 16, static_cast<uint32_t*>(out_dev));
    return (int)hipGetLastError();
}

}  // extern "C"
