// Device twin of the seeded synthetic-logits definition (input tooling only).
//
// Stand-in for ComputeLogits(L) of Algorithm 2.  Integer arithmetic only, so the values
// equal the host implementation bit for bit:
//   e   = (step * batch + b) * n_tokens + t
//   z_k = mix(seed + (3 e + k + 1) * 0x9E3779B97F4A7C15),  k = 0, 1, 2   (splitmix64 finaliser)
//   S   = sum of the twelve 16-bit fields of z_0, z_1, z_2
//   x   = (S - 393210) * (sigma / 65536)          exact in fp32 for sigma a power of two
//   bf16 = round-to-nearest-even of the fp32 bits
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ uint32_t fields16(uint64_t z)
{
    return (uint32_t)(z & 0xFFFF) + (uint32_t)((z >> 16) & 0xFFFF) + (uint32_t)((z >> 32) & 0xFFFF) +
           (uint32_t)(z >> 48);
}

template <typename OutT>
__global__ void __launch_bounds__(256)
gen_logits_kernel(OutT* __restrict__ out, uint64_t seed, uint64_t step, int32_t batch, int32_t n_tokens,
                  int64_t row_stride, float scale)
{
    const int32_t b = blockIdx.y;
    const uint64_t row_base = (step * (uint64_t)batch + (uint64_t)b) * (uint64_t)n_tokens;
    for (int32_t t = blockIdx.x * blockDim.x + threadIdx.x; t < n_tokens; t += gridDim.x * blockDim.x) {
        const uint64_t e = row_base + (uint64_t)t;
        uint32_t s = 0;
#pragma unroll
        for (uint64_t k = 1; k <= 3; ++k) s += fields16(mix64(seed + (3ull * e + k) * 0x9E3779B97F4A7C15ull));
        const float x = (float)((int32_t)s - 393210) * scale;
        if constexpr (sizeof(OutT) == 4) {
            out[(int64_t)b * row_stride + t] = x;
        } else {
            uint32_t u = __float_as_uint(x);
            u += 0x7FFFu + ((u >> 16) & 1u);
            out[(int64_t)b * row_stride + t] = (OutT)(u >> 16);
        }
    }
}

}  // namespace

// out: device pointer to [batch, row_stride] elements (float for dtype 0, 16-bit bf16 patterns
// for dtype 1).  Enqueues on `stream`; returns the hipError_t of the launch (0 = success).
extern "C" int tdfa_workload_gen_logits(void* out, uint64_t seed, uint64_t step, int32_t batch,
                                        int32_t n_tokens, int64_t row_stride, float sigma, int dtype,
                                        void* stream)
{
    if (batch <= 0 || n_tokens <= 0) return 0;
    if (!out || row_stride < n_tokens || batch > 65535) return (int)hipErrorInvalidValue;
    const float scale = sigma / 65536.0f;
    int gx = (n_tokens + 255) / 256;
    if (gx > 1024) gx = 1024;
    dim3 grid(gx, batch);
    if (dtype == 0)
        gen_logits_kernel<float><<<grid, 256, 0, (hipStream_t)stream>>>((float*)out, seed, step, batch, n_tokens,
                                                                        row_stride, scale);
    else
        gen_logits_kernel<uint16_t><<<grid, 256, 0, (hipStream_t)stream>>>((uint16_t*)out, seed, step, batch,
                                                                           n_tokens, row_stride, scale);
    return (int)hipGetLastError();
}
