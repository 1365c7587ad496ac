// Device twin of pier_inputs/generator.py: fills a buffer with N(0, std) deviates
// from Philox4x32-10 + Box-Muller, addressed by (seed, stream, step, element index).
// Input synthesis for tests and benchmarks only; no optimizer arithmetic here.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

struct U4 { uint32_t x, y, z, w; };

__device__ __forceinline__ U4 philox4x32_10(U4 c, uint32_t k0, uint32_t k1)
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        if (r) { k0 += W0; k1 += W1; }
        const uint32_t hi0 = __umulhi(M0, c.x), lo0 = M0 * c.x;
        const uint32_t hi1 = __umulhi(M1, c.z), lo1 = M1 * c.z;
        c = U4{hi1 ^ c.y ^ k0, lo1, hi0 ^ c.w ^ k1, lo0};
    }
    return c;
}

__device__ __forceinline__ float uniform(uint32_t x)
{
    return (static_cast<float>(x >> 9) + 0.5f) * 1.1920928955078125e-07f;  // 2^-23
}

__device__ __forceinline__ void box_muller(uint32_t xa, uint32_t xb, float& z0, float& z1)
{
    const float r = sqrtf(-2.0f * logf(uniform(xa)));
    const float ang = 6.283185307179586f * uniform(xb);
    float s, c;
    sincosf(ang, &s, &c);
    z0 = r * c;
    z1 = r * s;
}

__device__ __forceinline__ unsigned short to_bf16(float f)
{
    uint32_t b = __float_as_uint(f);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return static_cast<unsigned short>(b >> 16);
}

template <bool BF16>
__global__ __launch_bounds__(256) void fill_normal(void* dst, int64_t n, int64_t first_elem,
                                                   uint64_t seed, uint32_t stream_id, uint32_t step,
                                                   float std_)
{
    // one Philox block (4 elements) per thread; first_elem is a multiple of 4
    const int64_t nblk = (n + 3) >> 2;
    for (int64_t b = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; b < nblk;
         b += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const uint64_t blk = static_cast<uint64_t>((first_elem >> 2) + b);
        const U4 x = philox4x32_10(U4{static_cast<uint32_t>(blk), static_cast<uint32_t>(blk >> 32), step, stream_id},
                                   static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32));
        float z[4];
        box_muller(x.x, x.y, z[0], z[1]);
        box_muller(x.z, x.w, z[2], z[3]);
        const int64_t e = b << 2;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (e + k < n) {
                const float val = std_ * z[k];
                if constexpr (BF16) static_cast<unsigned short*>(dst)[e + k] = to_bf16(val);
                else static_cast<float*>(dst)[e + k] = val;
            }
        }
    }
}

}  // namespace

// dst: device pointer to n elements (fp32, or bf16 when is_bf16 != 0), which are the
// elements [first_elem, first_elem + n) of draw (seed, stream_id, step); first_elem
// must be a multiple of 4.  Returns the hipError_t of the launch as int.
extern "C" int pier_inputs_fill_normal(void* dst, int64_t n, int64_t first_elem, int is_bf16,
                                       uint64_t seed, uint32_t stream_id, uint32_t step, float std_,
                                       void* hip_stream)
{
    if (n <= 0) return 0;
    if (!dst || first_elem < 0 || (first_elem & 3)) return static_cast<int>(hipErrorInvalidValue);
    const int64_t nblk = (n + 3) >> 2;
    const int grid = static_cast<int>(nblk / 256 + 1 < 65536 * 4 ? nblk / 256 + 1 : 65536 * 4);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (is_bf16) hipLaunchKernelGGL(fill_normal<true>, dim3(grid), dim3(256), 0, s, dst, n, first_elem, seed, stream_id, step, std_);
    else hipLaunchKernelGGL(fill_normal<false>, dim3(grid), dim3(256), 0, s, dst, n, first_elem, seed, stream_id, step, std_);
    return static_cast<int>(hipGetLastError());
}

// Pinned host memory of exactly the size asked for.  (torch's pinned allocator rounds requests
// up to a power of two - 26.6 GB becomes 32 GiB - and a process here may pin about 66 GiB in
// all, so the two host arrays of the 7B configuration are allocated through these instead.)
extern "C" int pier_inputs_host_alloc(void** out, size_t bytes)
{
    if (!out) return static_cast<int>(hipErrorInvalidValue);
    *out = nullptr;
    return static_cast<int>(hipHostMalloc(out, bytes ? bytes : 16, hipHostMallocDefault));
}

extern "C" int pier_inputs_host_free(void* p)
{
    return p ? static_cast<int>(hipHostFree(p)) : 0;
}

// Device memory of exactly the size asked for, as its own allocation (torch's caching allocator
// hands out pieces of larger segments, so the extent of a torch tensor's underlying allocation
// says nothing about the tensor).
extern "C" int pier_inputs_device_alloc(void** out, size_t bytes)
{
    if (!out) return static_cast<int>(hipErrorInvalidValue);
    *out = nullptr;
    return static_cast<int>(hipMalloc(out, bytes ? bytes : 16));
}

extern "C" int pier_inputs_device_free(void* p)
{
    return p ? static_cast<int>(hipFree(p)) : 0;
}
