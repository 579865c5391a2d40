// Row-wise kernels of the decoder forward: the input rows (embedding gather or caller's
// embedding rows) with the first RMSNorm's operand, and buffer clearing.
#include "launch.h"

namespace spd {

// One workgroup per input row.  Writes the float32 residual row h, the packed three-term bf16
// operand of (h * gain) for the first QKV projection, and sum(h^2) of the row
// (the RMSNorm scale itself is applied inside that projection).
__global__ __launch_bounds__(256) void input_rows_kernel(const uint16_t *__restrict__ E,
                                                         const int32_t *__restrict__ tokens, int M, int token_stride,
                                                         const float *__restrict__ embeds, int d, int vocab,
                                                         const float *__restrict__ gain, float *__restrict__ h,
                                                         uint16_t *__restrict__ xpack, float *__restrict__ ssq) {
    const int row = blockIdx.x;
    const int KS = d / 32;
    const uint16_t *src_tok = nullptr;
    if (tokens) {
        // row = seq * M + i; the ids of one sequence are token_stride apart from the next one's
        int tok = tokens[(size_t)(row / M) * token_stride + row % M];
        tok = min(max(tok, 0), vocab - 1);                            // never read outside the table
        src_tok = E + (size_t)tok * d;
    }
    const float *src_row = embeds ? embeds + (size_t)row * d : nullptr;
    float *dst = h + (size_t)row * d;
    float ss = 0.f;
#pragma unroll 4
    for (int k = threadIdx.x * 4; k < d; k += 256 * 4) {              // d % 32 == 0
        float4 v;
        if (src_tok) {
            uint2 p = *reinterpret_cast<const uint2 *>(src_tok + k);
            v = float4{bf16_lo(p.x), bf16_hi(p.x), bf16_lo(p.y), bf16_hi(p.y)};
        } else {
            v = *reinterpret_cast<const float4 *>(src_row + k);
        }
        *reinterpret_cast<float4 *>(dst + k) = v;
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        float4 g = *reinterpret_cast<const float4 *>(gain + k);
        float y[4] = {v.x * g.x, v.y * g.y, v.z * g.z, v.w * g.w};
        union { uint2 v; uint16_t h[4]; } term[kTerms];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint16_t t3[kTerms];
            split3(y[e], t3);
#pragma unroll
            for (int t = 0; t < kTerms; ++t) term[t].h[e] = t3[t];
        }
        // 4 consecutive k stay inside one 8-element lane slot
#pragma unroll
        for (int t = 0; t < kTerms; ++t) *reinterpret_cast<uint2 *>(xpack + xpack_index(row, k, KS, t)) = term[t].v;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    __shared__ float part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) ssq[(size_t)row * (d / 16)] = (part[0] + part[1]) + (part[2] + part[3]);   // part 0 of [rows][d / 16]
}

hipError_t launch_input_rows(const void *embed_bf16, const int32_t *tokens, int M, int token_stride,
                             const float *embeds, int rows, int d, int vocab, const float *gain, float *h,
                             void *xpack, float *ssq, hipStream_t stream) {
    if ((!tokens) == (!embeds) || M < 1 || token_stride < M) return hipErrorInvalidValue;
    hipLaunchKernelGGL(input_rows_kernel, dim3(rows), dim3(256), 0, stream, (const uint16_t *)embed_bf16,
                       tokens, M, token_stride, embeds, d, vocab, gain, h, (uint16_t *)xpack, ssq);
    return hipGetLastError();
}

// ---- KV lengths kept on the device ---------------------------------------------------------
__global__ void lens_add_kernel(int32_t *lens, int n, int delta) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) lens[i] += delta;
}

hipError_t launch_lens_add(int32_t *lens, int n, int delta, hipStream_t stream) {
    hipLaunchKernelGGL(lens_add_kernel, dim3((n + 63) / 64), dim3(64), 0, stream, lens, n, delta);
    return hipGetLastError();
}

// End of a speculative-decoding block, one thread per sequence: emit d_1 .. d_k and y, make y the
// first token of the next verify call, hand the draft its next two inputs and roll both KV
// lengths back by the gamma - k rejected positions.
__global__ void block_commit_kernel(CommitArgs a) {
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= a.n_seqs) return;
    const int G = a.gamma;
    const int k = min(max(a.n_accepted[s], 0), G);
    const int y = a.next_token[s];
    int32_t *vt = a.verify_tokens + (size_t)s * (G + 1);
    if (a.out_tokens) {
        int n = a.n_out[s];
        for (int j = 0; j <= k; ++j)
            if (n + j < a.out_capacity) a.out_tokens[(size_t)s * a.out_capacity + n + j] = (j < k) ? vt[1 + j] : y;
        a.n_out[s] = min(n + k + 1, a.out_capacity);
    }
    a.draft_in[2 * s + 0] = vt[k];             // token before y: d_k, or t when nothing was accepted
    a.draft_in[2 * s + 1] = y;
    vt[0] = y;
    a.target_lens[s] -= G - k;
    a.draft_lens[s] -= G - k;
}

hipError_t launch_block_commit(const CommitArgs &a, hipStream_t stream) {
    if (a.n_seqs < 1 || a.gamma < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(block_commit_kernel, dim3((a.n_seqs + 63) / 64), dim3(64), 0, stream, a);
    return hipGetLastError();
}

// ---- KV cache read-out (inspection: tests, the benchmark's CPU baseline) -------------------
// K[pos][head][d] and V[pos][head][d] of one (layer, sequence) as float32, from the cache's own layouts:
// K bf16 [head][pos][dh], V bf16 [head][v_stride / 32][dh][32].
__global__ void kv_export_kernel(const uint16_t *__restrict__ Kc, const uint16_t *__restrict__ Vt, int H, int dh, int max_positions,
                                 int pos0, int n, float *__restrict__ k_out, float *__restrict__ v_out) {
    const size_t total = (size_t)n * H * dh;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int d = (int)(i % dh), h = (int)((i / dh) % H), p = (int)(i / ((size_t)dh * H));
        const int pos = pos0 + p;
        k_out[i] = bf16_bits_to_f32(Kc[((size_t)h * max_positions + pos) * dh + d]);
        v_out[i] = bf16_bits_to_f32(Vt[(((size_t)h * ((max_positions + 31) / 32) + (pos >> 5)) * dh + d) * 32 + (pos & 31)]);
    }
}

hipError_t launch_kv_export(const void *k_cache, const void *v_cache, int H, int dh, int max_positions, int pos0, int n,
                            float *k_out, float *v_out, hipStream_t stream) {
    if (n < 1 || pos0 < 0 || pos0 + n > max_positions) return hipErrorInvalidValue;
    const size_t total = (size_t)n * H * dh;
    unsigned grid = (unsigned)((total + 255) / 256);
    if (grid > 4096) grid = 4096;
    hipLaunchKernelGGL(kv_export_kernel, dim3(grid), dim3(256), 0, stream, (const uint16_t *)k_cache, (const uint16_t *)v_cache, H, dh,
                       max_positions, pos0, n, k_out, v_out);
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
