// Device side of the counter-based input generator (see moe_inputs/__init__.py
// for the recipe).  Test/benchmark harness code: fills tensors in HBM so that
// multi-gigabyte synthetic weights never cross PCIe.  Not part of the MoE library.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ float element(uint64_t key, uint64_t i, float scale)
{
    int32_t s = 0;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        uint64_t r = mix64(key + (3ull * i + (uint64_t)(j + 1)) * 0x9E3779B97F4A7C15ull);
        s += (int32_t)(r & 0xFFFF) + (int32_t)((r >> 16) & 0xFFFF) + (int32_t)((r >> 32) & 0xFFFF) +
             (int32_t)(r >> 48);
    }
    return __int2float_rn(s - 6 * 65535) * scale;
}

__global__ void fill_normal(void *out, int bf16, uint64_t key, uint64_t start, uint64_t count, float scale)
{
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) {
        float v = element(key, start + i, scale);
        if (bf16) {
            uint32_t b = __float_as_uint(v);
            b = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
            static_cast<uint16_t *>(out)[i] = (uint16_t)b;
        } else {
            static_cast<float *>(out)[i] = v;
        }
    }
}

// plain copy, 16 bytes per lane, grid-stride: the yardstick for HBM counters and for the
// achievable copy bandwidth of the box
__global__ void copy_16B(const uint4 *__restrict__ src, uint4 *__restrict__ dst, uint64_t n16)
{
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride)
        dst[i] = src[i];
}

}  // namespace

// Copies `bytes` (a multiple of 16) from src to dst, both device pointers.
extern "C" int moe_inputs_copy(void *dst, const void *src, uint64_t bytes, void *stream)
{
    if (bytes == 0 || bytes % 16 != 0)
        return bytes == 0 ? 0 : -1;
    hipLaunchKernelGGL(copy_16B, dim3(256 * 32), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// out: device pointer to `count` elements (fp32, or bf16 when bf16 != 0) that receive
// flat elements [start, start+count) of the stream identified by `key`.
extern "C" int moe_inputs_fill_normal(void *out, int bf16, uint64_t key, uint64_t start, uint64_t count,
                                      float scale, void *stream)
{
    if (count == 0)
        return 0;
    uint64_t blocks = (count + 255) / 256;
    if (blocks > 65536)
        blocks = 65536;
    hipLaunchKernelGGL(fill_normal, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), out,
                       bf16, key, start, count, scale);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}
