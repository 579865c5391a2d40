// RoPE + KV-cache append + causal attention of M <= 8 new queries per sequence over
// the cached prefix (image rows + text + already accepted tokens), split over the
// key range ("split-KV") with a deterministic second-stage combine.
//
// Grid of the first stage: (key split, head, sequence).  Each workgroup
//   1. rotates q and k of its head for the M new positions (half-split RoPE pairing,
//      table of cos/sin per position), rounds the new k, v to bf16 -- the cache
//      precision -- and, if it owns the position, appends them to the cache;
//   2. scores its slice of cached keys (16-byte loads, one key per 16 or 8 lanes,
//      partial dot products reduced with wavefront shuffles) plus the new keys that
//      fall into its slice (causal mask among the new positions);
//   3. softmax statistics of the slice (max, sum) with wavefront reductions;
//   4. weighted sum of its slice of V.
// The second stage merges the slices of a (sequence, head) in a fixed order and
// writes the result as bf16 head + tail in B-operand order for the O projection.
#include "launch.h"

namespace spd {

constexpr int kSplitMax = 256;       // keys per workgroup (upper bound of split_len)

template <int DH>
__global__ __launch_bounds__(256) void attention_partial_kernel(AttnArgs a) {
    constexpr int LG = DH / 8;        // lanes that share one key row (16 B each)
    constexpr int PPW = 64 / LG;      // keys per wave per iteration
    constexpr int HALF = DH / 2;
    const int sp = blockIdx.x, hh = blockIdx.y, seq = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int li = lane % LG, lg = lane / LG;
    const int M = a.M, H = a.H;
    const int P = a.lens.len[seq];                  // cached positions before this call
    const int L = a.split_len;
    const int lo = sp * L;                          // this workgroup's key range [lo, hi)
    const int hi = min(lo + L, P + M);
    const size_t part_idx = ((size_t)seq * H + hh) * a.n_split + sp;

    if (hi <= lo) {                                 // empty slice: neutral element of the merge
        for (int i = tid; i < 8 * DH; i += 256) a.part_o[part_idx * 8 * DH + i] = 0.f;
        if (tid < 8) {
            a.part_ml[(part_idx * 8 + tid) * 2 + 0] = -INFINITY;
            a.part_ml[(part_idx * 8 + tid) * 2 + 1] = 0.f;
        }
        return;
    }

    __shared__ float qs[8][DH];
    __shared__ float kf[8][DH];
    __shared__ float vf[8][DH];
    __shared__ float sc[8][kSplitMax];
    __shared__ float red_o[4][8][DH];
    __shared__ float ml[8][2];

    const size_t HD = (size_t)H * DH;
    uint16_t *Kc = (uint16_t *)a.k_cache + ((size_t)seq * H + hh) * a.max_positions * DH;
    uint16_t *Vc = (uint16_t *)a.v_cache + ((size_t)seq * H + hh) * a.max_positions * DH;
    const float scale = 1.0f / sqrtf((float)DH);

    // ---- 1. RoPE on q, k of the new rows; bf16 rounding of new k, v; cache append -------
    for (int idx = tid; idx < 8 * HALF; idx += 256) {
        int i = idx / HALF, j = idx % HALF;
        if (i < M) {
            int pos = P + i;
            const float *row = a.qkv + (size_t)(seq * M + i) * 3 * HD + (size_t)hh * DH;
            float c = a.rope[((size_t)pos * HALF + j) * 2 + 0];
            float s = a.rope[((size_t)pos * HALF + j) * 2 + 1];
            float q1 = row[j], q2 = row[j + HALF];
            float k1 = row[HD + j], k2 = row[HD + j + HALF];
            float v1 = row[2 * HD + j], v2 = row[2 * HD + j + HALF];
            qs[i][j] = (q1 * c - q2 * s) * scale;
            qs[i][j + HALF] = (q2 * c + q1 * s) * scale;
            uint16_t kb1 = f32_to_bf16_bits(k1 * c - k2 * s);
            uint16_t kb2 = f32_to_bf16_bits(k2 * c + k1 * s);
            uint16_t vb1 = f32_to_bf16_bits(v1), vb2 = f32_to_bf16_bits(v2);
            kf[i][j] = bf16_bits_to_f32(kb1);
            kf[i][j + HALF] = bf16_bits_to_f32(kb2);
            vf[i][j] = bf16_bits_to_f32(vb1);
            vf[i][j + HALF] = bf16_bits_to_f32(vb2);
            if (pos >= lo && pos < hi) {            // exactly one slice owns each new position
                Kc[(size_t)pos * DH + j] = kb1;
                Kc[(size_t)pos * DH + j + HALF] = kb2;
                Vc[(size_t)pos * DH + j] = vb1;
                Vc[(size_t)pos * DH + j + HALF] = vb2;
            }
        } else {
            qs[i][j] = 0.f; qs[i][j + HALF] = 0.f;
            kf[i][j] = 0.f; kf[i][j + HALF] = 0.f;
            vf[i][j] = 0.f; vf[i][j + HALF] = 0.f;
        }
    }
    __syncthreads();

    // ---- 2. scores ----------------------------------------------------------------------
    const int c1 = min(hi, P);                      // cached keys of this slice: [lo, c1)
    {
        float qreg[8][8];
#pragma unroll
        for (int m = 0; m < 8; ++m)
#pragma unroll
            for (int e = 0; e < 8; ++e) qreg[m][e] = qs[m][li * 8 + e];
        for (int base = lo + w * PPW; base < c1; base += 4 * PPW) {
            int p = base + lg;
            bool valid = p < c1;
            uint4 kv = valid ? *reinterpret_cast<const uint4 *>(Kc + (size_t)p * DH + li * 8) : uint4{0, 0, 0, 0};
            float k[8] = {bf16_lo(kv.x), bf16_hi(kv.x), bf16_lo(kv.y), bf16_hi(kv.y),
                          bf16_lo(kv.z), bf16_hi(kv.z), bf16_lo(kv.w), bf16_hi(kv.w)};
            float s[8];
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                float acc = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc += k[e] * qreg[m][e];
                s[m] = acc;
            }
#pragma unroll
            for (int o = LG / 2; o > 0; o >>= 1)
#pragma unroll
                for (int m = 0; m < 8; ++m) s[m] += __shfl_xor(s[m], o);
            if (valid && li < 8) {
                // lane li of the group stores query li's score (all lanes hold all sums)
                float mine = s[0];
#pragma unroll
                for (int m = 1; m < 8; ++m) mine = (li == m) ? s[m] : mine;
                sc[li][p - lo] = mine;
            }
        }
    }
    if (tid < 64) {                                 // new keys: query m sees new key j iff j <= m
        int m = tid >> 3, j = tid & 7;
        int p = P + j;
        if (j < M && p >= lo && p < hi) {
            float acc = -INFINITY;
            if (j <= m) {
                acc = 0.f;
                for (int e = 0; e < DH; ++e) acc += qs[m][e] * kf[j][e];
            }
            sc[m][p - lo] = acc;
        }
    }
    __syncthreads();

    // ---- 3. softmax statistics of the slice ---------------------------------------------
    const int n_here = hi - lo;
    {
        int m = tid >> 5, t = tid & 31;
        float mx = -INFINITY;
        for (int i = t; i < n_here; i += 32) mx = fmaxf(mx, sc[m][i]);
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        float mref = (mx == -INFINITY) ? 0.f : mx;
        float sum = 0.f;
        for (int i = t; i < n_here; i += 32) {
            float e = expf(sc[m][i] - mref);
            sc[m][i] = e;
            sum += e;
        }
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        if (t == 0) { ml[m][0] = mx; ml[m][1] = sum; }
    }
    __syncthreads();

    // ---- 4. weighted sum of V --------------------------------------------------------------
    float o[8][8];
#pragma unroll
    for (int m = 0; m < 8; ++m)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[m][e] = 0.f;
    for (int base = lo + w * PPW; base < c1; base += 4 * PPW) {
        int p = base + lg;
        if (p < c1) {
            uint4 vv = *reinterpret_cast<const uint4 *>(Vc + (size_t)p * DH + li * 8);
            float v[8] = {bf16_lo(vv.x), bf16_hi(vv.x), bf16_lo(vv.y), bf16_hi(vv.y),
                          bf16_lo(vv.z), bf16_hi(vv.z), bf16_lo(vv.w), bf16_hi(vv.w)};
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                float pr = sc[m][p - lo];
#pragma unroll
                for (int e = 0; e < 8; ++e) o[m][e] += pr * v[e];
            }
        }
    }
    if (w == 0 && lg == 0) {                        // new values held in LDS
        for (int j = 0; j < M; ++j) {
            int p = P + j;
            if (p >= lo && p < hi) {
#pragma unroll
                for (int m = 0; m < 8; ++m) {
                    float pr = sc[m][p - lo];
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[m][e] += pr * vf[j][li * 8 + e];
                }
            }
        }
    }
#pragma unroll
    for (int off = LG; off < 64; off <<= 1)
#pragma unroll
        for (int m = 0; m < 8; ++m)
#pragma unroll
            for (int e = 0; e < 8; ++e) o[m][e] += __shfl_xor(o[m][e], off);
    if (lg == 0) {
#pragma unroll
        for (int m = 0; m < 8; ++m)
#pragma unroll
            for (int e = 0; e < 8; ++e) red_o[w][m][li * 8 + e] = o[m][e];
    }
    __syncthreads();
    for (int i = tid; i < 8 * DH; i += 256) {
        int m = i / DH, dd = i % DH;
        float sum = (red_o[0][m][dd] + red_o[1][m][dd]) + (red_o[2][m][dd] + red_o[3][m][dd]);
        a.part_o[part_idx * 8 * DH + i] = sum;
    }
    if (tid < 8) {
        a.part_ml[(part_idx * 8 + tid) * 2 + 0] = ml[tid][0];
        a.part_ml[(part_idx * 8 + tid) * 2 + 1] = ml[tid][1];
    }
}

// Second stage: merge the key slices of one (sequence, head) in slice order.
template <int DH>
__global__ __launch_bounds__(DH) void attention_combine_kernel(AttnArgs a) {
    const int hh = blockIdx.x, seq = blockIdx.y, dd = threadIdx.x;
    const int H = a.H, M = a.M, NS = a.n_split;
    const size_t base = ((size_t)seq * H + hh) * NS;
    const int KS = H * DH / 32;
    for (int m = 0; m < M; ++m) {
        float mstar = -INFINITY;
        for (int s = 0; s < NS; ++s) mstar = fmaxf(mstar, a.part_ml[((base + s) * 8 + m) * 2]);
        float num = 0.f, den = 0.f;
        for (int s = 0; s < NS; ++s) {
            float ms = a.part_ml[((base + s) * 8 + m) * 2];
            float ls = a.part_ml[((base + s) * 8 + m) * 2 + 1];
            float wgt = (ms == -INFINITY) ? 0.f : expf(ms - mstar);
            den += wgt * ls;
            num += wgt * a.part_o[((base + s) * 8 + m) * DH + dd];
        }
        float val = num / den;
        uint16_t hi, lo;
        split_hi_lo(val, hi, lo);
        int row = seq * M + m, k = hh * DH + dd;
        ((uint16_t *)a.xout)[xpack_index(row, k, KS, 0)] = hi;
        ((uint16_t *)a.xout)[xpack_index(row, k, KS, 1)] = lo;
    }
}

hipError_t launch_attention(const AttnArgs &a, hipStream_t stream) {
    if (a.split_len < 1 || a.split_len > kSplitMax || a.M < 1 || a.M > 8) return hipErrorInvalidValue;
    dim3 grid(a.n_split, a.H, a.n_seqs);
    if (a.dh == 128) {
        hipLaunchKernelGGL(attention_partial_kernel<128>, grid, dim3(256), 0, stream, a);
        hipLaunchKernelGGL(attention_combine_kernel<128>, dim3(a.H, a.n_seqs), dim3(128), 0, stream, a);
    } else if (a.dh == 64) {
        hipLaunchKernelGGL(attention_partial_kernel<64>, grid, dim3(256), 0, stream, a);
        hipLaunchKernelGGL(attention_combine_kernel<64>, dim3(a.H, a.n_seqs), dim3(64), 0, stream, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace spd
