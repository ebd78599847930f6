// Two measurement helpers behind the C ABI, used by the benchmark to put the kernels' figures
// next to what this card reaches in practice: a pure streaming read and a bf16 MFMA issue loop.
// They compute nothing of the method.
#include "ls_internal.hpp"

namespace ls {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Every thread strides over the buffer in 16-byte pieces; the XOR of what it read goes to sink
// only under a condition the data never meets, so the loads cannot be dropped.
__global__ void __launch_bounds__(256) stream_read_kernel(const u32x4 *__restrict__ src, size_t n16, u32x4 *sink)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    u32x4 acc = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        acc ^= __builtin_nontemporal_load(src + i);
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = acc;
}

// 512 threads per workgroup (two waves per SIMD), four independent accumulator chains per wave.
__global__ void __launch_bounds__(512) mfma_loop_kernel(int iters, float *sink)
{
    bf16x8 a, b;
    const uint16_t one = 0x3f80;
    const uint16_t ones[8] = {one, one, one, one, one, one, one, one};
    __builtin_memcpy(&a, ones, 16);
    __builtin_memcpy(&b, ones, 16);
    floatx16 c[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[k][r] = 0.f;
    for (int i = 0; i < iters; ++i)
#pragma unroll
        for (int k = 0; k < 4; ++k) c[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[k], 0, 0, 0);
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[k][r];
    if (s == 12345.f) sink[0] = s;
}

}  // namespace

hipError_t launch_probe_stream_read(const void *src, size_t bytes, void *sink, hipStream_t stream)
{
    int cus = 256;
    int dev = 0;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    hipLaunchKernelGGL(stream_read_kernel, dim3(cus * 8), dim3(256), 0, stream, (const u32x4 *)src, bytes / 16,
                       (u32x4 *)sink);
    return hipGetLastError();
}

hipError_t launch_probe_mfma_loop(int iters, float *sink, int *flops_per_iter_per_cu, hipStream_t stream)
{
    int cus = 256;
    int dev = 0;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(cus), dim3(512), 0, stream, iters, sink);
    // 8 waves x 4 chains x one 32x32x16 MFMA (2*32*32*16 flop) per iteration and workgroup
    if (flops_per_iter_per_cu) *flops_per_iter_per_cu = 8 * 4 * 2 * 32 * 32 * 16;
    return hipGetLastError();
}

}  // namespace ls
