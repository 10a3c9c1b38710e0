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

// Read yardstick: each workgroup (4 wavefronts) streams its own region of `region` bytes from memory into LDS
// with 16-byte buffer loads, 32 of them in flight per wavefront, rows of `row_bytes` (a multiple of 128) taken
// 128 rows x 128 bytes at a time: the access pattern of a weight panel.  Nothing is computed.
constexpr int kStreamWaves = 4, kStreamDepth = 8;
__global__ __launch_bounds__(kStreamWaves * 64) void stream_read(const unsigned char *__restrict__ src, uint64_t region,
                                                                int row_bytes, int panels, unsigned *__restrict__ out)
{
    __shared__ __attribute__((aligned(1024))) unsigned char lds[kStreamWaves * 4096];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned char *p = src + (uint64_t)blockIdx.x * region + (uint64_t)(wave * 32 + lane / 8) * row_bytes + (lane % 8) * 16;
    for (int pn = 0; pn < panels; ++pn) {
        for (int koff = 0; koff < row_bytes; koff += 128) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p + (uint64_t)j * 8 * row_bytes + koff),
                                                 (__attribute__((address_space(3))) void *)(lds + (wave * 4 + j) * 1024), 16, 0, 0);
            __builtin_amdgcn_s_waitcnt(0x0F70 | (((kStreamDepth - 1) * 4) & 15) | ((((kStreamDepth - 1) * 4) >> 4) << 14)); // vmcnt
        }
        p += (uint64_t)kStreamWaves * 32 * row_bytes;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0)
    __syncthreads();
    if (out)
        out[blockIdx.x * kStreamWaves * 64 + tid] = lds[tid];
}

}  // namespace

// Launches `workgroups` workgroups that each read `panels` panels of 128 rows x row_bytes from their own region of
// `region` bytes of src (device pointer, at least workgroups * region bytes).  Returns the bytes one workgroup reads
// (0: bad arguments, -1: launch failed).
extern "C" int64_t moe_inputs_stream_read(const void *src, uint64_t region, int row_bytes, int panels, int workgroups,
                                          void *stream)
{
    const uint64_t panel = (uint64_t)kStreamWaves * 32 * row_bytes;
    if (!src || row_bytes <= 0 || row_bytes % 128 != 0 || panels <= 0 || workgroups <= 0 || panel * panels > region)
        return 0;
    hipLaunchKernelGGL(stream_read, dim3(workgroups), dim3(kStreamWaves * 64), 0, static_cast<hipStream_t>(stream),
                       static_cast<const unsigned char *>(src), region, row_bytes, panels, (unsigned *)nullptr);
    return hipGetLastError() == hipSuccess ? (int64_t)(panel * panels) : -1;
}

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
