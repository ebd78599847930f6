// Measurement helpers for the benchmark, built into a library of their own (libls_probe.so): what
// this card reaches in practice on a pure streaming read and on a bf16 MFMA issue loop, to put
// next to the kernels' figures.  They compute nothing of the method and are not part of the
// attention library or its header.
#include <hip/hip_runtime.h>
#include <stdint.h>

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

// The same loop on operands that differ from lane to lane and from one instruction to the next
// (hashed sign and mantissa bits, magnitudes in [1, 2)): what the matrix cores sustain when their
// inputs toggle as real keys and values do.  With constant operands the loop above draws far less
// power and holds a higher clock.
__device__ inline uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
__global__ void __launch_bounds__(512) mfma_loop_varied_kernel(int iters, float *sink)
{
    bf16x8 a[4], b[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        uint16_t av[8], bv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t h = mix32((threadIdx.x * 4u + k) * 8u + e + 0x9e3779b9u * (blockIdx.x + 1u));
            av[e] = (uint16_t)(0x3f80u | (h & 0x807fu));          // +-[1, 2)
            bv[e] = (uint16_t)(0x3f80u | ((h >> 16) & 0x807fu));
        }
        __builtin_memcpy(&a[k], av, 16);
        __builtin_memcpy(&b[k], bv, 16);
    }
    floatx16 c[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[k][r] = 0.f;
    for (int i = 0; i < iters; i += 4)  // iters is a multiple of 4
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int k = 0; k < 4; ++k)
                c[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[k], b[(k + r) & 3], c[k], 0, 0, 0);
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[k][r];
    if (s == 12345.f) sink[0] = s;
}

}  // namespace

extern "C" {

// Reads `bytes` (>= 16, 16-byte aligned DEVICE memory) once with every compute unit; writes nothing
// but, possibly, 16 bytes at `sink` (DEVICE).  Returns 0, or -1 on a bad argument / launch error.
int ls_probe_stream_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (!src || !sink || bytes < 16 || ((uintptr_t)src & 15u) || ((uintptr_t)sink & 15u)) return -1;
    int cus = 256, dev = 0;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    hipLaunchKernelGGL(stream_read_kernel, dim3(cus * 8), dim3(256), 0, (hipStream_t)stream, (const u32x4 *)src,
                       bytes / 16, (u32x4 *)sink);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// `iters` rounds of independent bf16 32x32x16 MFMAs from two waves per SIMD on every compute unit;
// *flops_out (HOST, may be NULL) receives the flop count of the launch.
int ls_probe_mfma_loop(int32_t iters, void *sink, int64_t *flops_out, void *stream)
{
    if (!sink || iters <= 0 || iters > (1 << 24)) return -1;
    int cus = 256, dev = 0;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(cus), dim3(512), 0, (hipStream_t)stream, iters, (float *)sink);
    // 8 waves x 4 chains x one 32x32x16 MFMA (2*32*32*16 flop) per iteration and workgroup
    if (flops_out) *flops_out = (int64_t)8 * 4 * 2 * 32 * 32 * 16 * iters * cus;
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// The same launch shape and flop count with operands that vary per lane and per instruction;
// iters must be a multiple of 4.
int ls_probe_mfma_loop_varied(int32_t iters, void *sink, int64_t *flops_out, void *stream)
{
    if (!sink || iters <= 0 || iters > (1 << 24) || iters % 4) return -1;
    int cus = 256, dev = 0;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    hipLaunchKernelGGL(mfma_loop_varied_kernel, dim3(cus), dim3(512), 0, (hipStream_t)stream, iters, (float *)sink);
    if (flops_out) *flops_out = (int64_t)8 * 4 * 2 * 32 * 32 * 16 * iters * cus;
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // extern "C"
