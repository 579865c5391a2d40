// Row-wise kernels of the decoder forward: embedding gather, RMSNorm fused with the
// head/tail split that produces the matrix-core B operand, buffer clearing.
#include "launch.h"

namespace spd {

__global__ void embed_gather_kernel(const uint16_t *__restrict__ E, const int32_t *__restrict__ tokens,
                                    int d, int vocab, float *__restrict__ h) {
    int row = blockIdx.x;
    int tok = min(max(tokens[row], 0), vocab - 1);                    // never read outside the table
    const uint16_t *src = E + (size_t)tok * d;
    float *dst = h + (size_t)row * d;
    for (int k = threadIdx.x * 8; k < d; k += blockDim.x * 8) {      // d % 8 == 0
        uint4 v = *reinterpret_cast<const uint4 *>(src + k);
        float4 a = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y)};
        float4 b = {bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
        *reinterpret_cast<float4 *>(dst + k) = a;
        *reinterpret_cast<float4 *>(dst + k + 4) = b;
    }
}

hipError_t launch_embed_gather(const void *embed_bf16, const int32_t *tokens, int rows, int d, int vocab,
                               float *h, hipStream_t stream) {
    hipLaunchKernelGGL(embed_gather_kernel, dim3(rows), dim3(256), 0, stream,
                       (const uint16_t *)embed_bf16, tokens, d, vocab, h);
    return hipGetLastError();
}

// y = x / sqrt(mean(x^2) + eps) * gain, float32; written as bf16 head + tail in B-operand order.
__global__ __launch_bounds__(256) void rmsnorm_pack_kernel(const float *__restrict__ h,
                                                           const float *__restrict__ gain, int d, float eps,
                                                           uint16_t *__restrict__ xpack) {
    const int row = blockIdx.x;
    const float *x = h + (size_t)row * d;
    float ss = 0.f;
    for (int k = threadIdx.x * 4; k < d; k += 256 * 4) {              // d % 4 == 0
        float4 v = *reinterpret_cast<const float4 *>(x + k);
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    __shared__ float part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    float total = (part[0] + part[1]) + (part[2] + part[3]);
    float inv = 1.0f / sqrtf(total / (float)d + eps);
    const int KS = d / 32;
    for (int k = threadIdx.x * 4; k < d; k += 256 * 4) {
        float4 v = *reinterpret_cast<const float4 *>(x + k);
        float4 g = *reinterpret_cast<const float4 *>(gain + k);
        float y[4] = {v.x * inv * g.x, v.y * inv * g.y, v.z * inv * g.z, v.w * inv * g.w};
        union { uint2 v; uint16_t h[4]; } hi, lo;
#pragma unroll
        for (int e = 0; e < 4; ++e) split_hi_lo(y[e], hi.h[e], lo.h[e]);
        // 4 consecutive k stay inside one 8-element lane slot
        *reinterpret_cast<uint2 *>(xpack + xpack_index(row, k, KS, 0)) = hi.v;
        *reinterpret_cast<uint2 *>(xpack + xpack_index(row, k, KS, 1)) = lo.v;
    }
}

hipError_t launch_rmsnorm_pack(const float *h, const float *gain, int rows, int d, float eps,
                               void *xpack, hipStream_t stream) {
    hipLaunchKernelGGL(rmsnorm_pack_kernel, dim3(rows), dim3(256), 0, stream, h, gain, d, eps,
                       (uint16_t *)xpack);
    return hipGetLastError();
}

__global__ void fill_zero_kernel(uint4 *p, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) p[i] = uint4{0, 0, 0, 0};
}

hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t stream) {
    size_t n16 = bytes / 16;                                           // callers pass multiples of 16
    if (n16 == 0) return hipSuccess;
    unsigned grid = (unsigned)((n16 + 255) / 256);
    if (grid > 4096) grid = 4096;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, stream, (uint4 *)p, n16);
    return hipGetLastError();
}

}  // namespace spd
