// Measured ceilings of the machine, as kernels of the library's own so that the figures
// quoted beside the nominal peaks can be reproduced: a loop of nothing but bf16 matrix
// instructions (on operands of normal-distributed or of constant bits: the chip's clock
// depends on how many bits toggle) and a read-only stream over device memory.
// Measurement aids: they compute nothing of the method.
#include "en_device.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Counter-based bits (a 32-bit mix of the argument): the operands only have to look like
// data, i.e. toggle about half of their bits from one matrix instruction to the next.
__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// A bf16 value with random sign and mantissa and an exponent of 2^-2 .. 2^1 (the bulk of a
// unit normal distribution), or the constant 0.5.
__device__ __forceinline__ bf16_t operand_value(uint32_t key, int constant)
{
    const uint32_t h = mix32(key);
    const uint16_t bits = constant ? 0x3f00 : (uint16_t)((h & 0x807f) | ((0x7d + ((h >> 8) & 3)) << 7));
    return __builtin_bit_cast(bf16_t, bits);
}

constexpr int MFMA_PER_ITER = 8;

// Every wave: `iters` rounds of 8 matrix instructions 32x32x16 over 4 independent accumulators,
// 4 A fragments and 2 B fragments taking turns (so that operand bits change between
// instructions as they do in a real product). Two waves per SIMD.
__global__ __launch_bounds__(512) void mfma_only_kernel(float *sink, int iters, int constant)
{
    // More than half of a compute unit's LDS: workgroups cannot share a compute unit, so that a launch
    // of one workgroup per compute unit really occupies every one of them (two waves per SIMD).
    __shared__ char one_workgroup_per_cu[96 * 1024];
    if (iters < 0)
        one_workgroup_per_cu[threadIdx.x] = (char)constant;      // never: keeps the array
    const uint32_t t = blockIdx.x * 512 + threadIdx.x;
    bf16x8 a[4], b[2];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int k = 0; k < 4; ++k)
            a[k][j] = operand_value(t * 64 + k * 8 + j, constant);
#pragma unroll
        for (int k = 0; k < 2; ++k)
            b[k][j] = operand_value(t * 64 + 32 + k * 8 + j, constant);
    }
    f32x16 acc[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            acc[k][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < MFMA_PER_ITER; ++m)
            acc[m % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m % 4], b[(m / 4) % 2], acc[m % 4], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            s += acc[k][e];
    if (s == 1.2345e-30f)              // never true for these operands; keeps the loop alive
        sink[t] = s + (float)one_workgroup_per_cu[threadIdx.x];
}

// Read-only stream: every lane loads 16 bytes per step, four steps in flight, whole workgroups
// walk the buffer with the grid's stride; what is read is folded into one word per lane that
// is (practically never) written.
__global__ __launch_bounds__(256) void read_stream_kernel(const u32x4 *src, size_t n16, uint32_t *sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t f = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 v0 = __builtin_nontemporal_load(src + i);
        const u32x4 v1 = __builtin_nontemporal_load(src + i + stride);
        const u32x4 v2 = __builtin_nontemporal_load(src + i + 2 * stride);
        const u32x4 v3 = __builtin_nontemporal_load(src + i + 3 * stride);
        f ^= v0.x ^ v0.y ^ v0.z ^ v0.w ^ v1.x ^ v1.y ^ v1.z ^ v1.w ^ v2.x ^ v2.y ^ v2.z ^ v2.w ^ v3.x ^ v3.y ^ v3.z ^ v3.w;
    }
    for (; i < n16; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(src + i);
        f ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (f == 0x9e3779b9u)              // data-dependent and practically never true
        sink[threadIdx.x] = f;
}

}  // namespace

int en_launch_ceiling_mfma(float *sink_dev, int n_workgroups, int iters, int constant, void *stream)
{
    hipLaunchKernelGGL(mfma_only_kernel, dim3(n_workgroups), dim3(512), 0, (hipStream_t)stream, sink_dev, iters, constant);
    return (int)hipGetLastError();
}

int en_launch_ceiling_read(const void *src_dev, size_t bytes, void *sink_dev, int n_workgroups, void *stream)
{
    hipLaunchKernelGGL(read_stream_kernel, dim3(n_workgroups), dim3(256), 0, (hipStream_t)stream,
                       (const u32x4 *)src_dev, bytes / 16, (uint32_t *)sink_dev);
    return (int)hipGetLastError();
}
