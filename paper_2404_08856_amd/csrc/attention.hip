// RoPE + KV-cache append + causal attention of M <= 8 new queries per sequence over
// the cached prefix (image rows + text + already accepted tokens), split over the
// key range ("split-KV") and merged by the last slice to finish, in a fixed order.
//
// Grid: (key slice, head, sequence).  Each workgroup
//   0. issues the 16-byte loads of ALL its cached keys and values first (a slice is at
//      most 128 keys, i.e. at most 8 + 8 loads per lane), so the whole kernel pays one
//      HBM latency;
//   1. rotates q and k of its head for the M new positions (half-split RoPE pairing,
//      table of cos/sin per position), rounds the new k, v to bf16 -- the cache
//      precision -- and, if it owns the position, appends them to the cache;
//   2. scores its slice (one key per 16 or 8 lanes, partial dot products reduced with
//      wavefront shuffles) plus the new keys that fall into it (causal among new rows);
//   3. softmax statistics of the slice (max, sum) with wavefront reductions;
//   4. weighted sum of its slice of V; writes (o, max, sum) of the slice;
//   5. bumps a per-(sequence, head) counter; the workgroup that arrives last merges all
//      slices in slice order (so the result does not depend on which one that is) and
//      writes the output as bf16 head + tail in B-operand order for the O projection.
#include "launch.h"

namespace spd {

constexpr int kSplitMax = 128;       // keys per workgroup (upper bound of split_len)

// Slice results travel between workgroups that may sit on different XCDs (each XCD has its
// own L2).  They are written and read with device-scope relaxed atomics, which the compiler
// turns into write-through stores / L2-bypassing loads; together with "wait until my stores
// are acknowledged" before the arrival counter is bumped this orders the hand-over without a
// whole-L2 write-back.
__device__ __forceinline__ void store_dev(float *p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_dev(const float *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int DH>
__global__ __launch_bounds__(256) void attention_kernel(AttnArgs a) {
    constexpr int LG = DH / 8;        // lanes that share one key row (16 B each)
    constexpr int PPW = 64 / LG;      // keys per wave per iteration
    constexpr int IT = kSplitMax / (4 * PPW);   // iterations that cover a full slice
    constexpr int HALF = DH / 2;
    const int sp = blockIdx.x, hh = blockIdx.y, seq = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int li = lane % LG, lg = lane / LG;
    const int M = a.M, H = a.H, NS = a.n_split;
    const int P = a.lens.len[seq];                  // cached positions before this call
    const int L = a.split_len;
    const int lo = sp * L;                          // this workgroup's key range [lo, hi)
    const int hi = min(lo + L, P + M);
    const int c1 = min(hi, P);                      // cached keys of the slice: [lo, c1)
    const size_t pair = (size_t)seq * H + hh;
    const size_t part_idx = pair * NS + sp;

    __shared__ float qs[8][DH];
    __shared__ float kf[8][DH];
    __shared__ float vf[8][DH];
    __shared__ float sc[8][kSplitMax];
    __shared__ float red_o[4][8][DH];
    __shared__ float ml[8][2];
    __shared__ float wgt[8][kMaxRows];              // merge weights, [m][slice] (n_split <= 64)
    __shared__ float lsum[8][kMaxRows];             // slice sums
    __shared__ int s_last;

    const size_t HD = (size_t)H * DH;
    uint16_t *Kc = (uint16_t *)a.k_cache + pair * a.max_positions * DH;
    uint16_t *Vc = (uint16_t *)a.v_cache + pair * a.max_positions * DH;

    // ---- 0. all cached K, V of the slice into registers ---------------------------------------
    uint4 kreg[IT], vreg[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        int p = lo + (it * 4 + w) * PPW + lg;
        if (p < c1) {
            kreg[it] = *reinterpret_cast<const uint4 *>(Kc + (size_t)p * DH + li * 8);
            vreg[it] = *reinterpret_cast<const uint4 *>(Vc + (size_t)p * DH + li * 8);
        } else {
            kreg[it] = uint4{0, 0, 0, 0};
            vreg[it] = uint4{0, 0, 0, 0};
        }
    }

    if (hi > lo) {
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
        {
            float qreg[8][8];
#pragma unroll
            for (int m = 0; m < 8; ++m)
#pragma unroll
                for (int e = 0; e < 8; ++e) qreg[m][e] = qs[m][li * 8 + e];
#pragma unroll
            for (int it = 0; it < IT; ++it) {
                int p = lo + (it * 4 + w) * PPW + lg;
                if (lo + (it * 4 + w) * PPW < c1) {     // wave-uniform: some lane group has a key
                    uint4 kv = kreg[it];
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
                    if (p < c1 && li < 8) {
                        // lane li of the group stores query li's score (all lanes hold all sums)
                        float mine = s[0];
#pragma unroll
                        for (int m = 1; m < 8; ++m) mine = (li == m) ? s[m] : mine;
                        sc[li][p - lo] = mine;
                    }
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
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            int p = lo + (it * 4 + w) * PPW + lg;
            if (p < c1) {
                uint4 vv = vreg[it];
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
            store_dev(&a.part_o[part_idx * 8 * DH + i], sum);
        }
        if (tid < 8) {
            store_dev(&a.part_ml[(part_idx * 8 + tid) * 2 + 0], ml[tid][0]);
            store_dev(&a.part_ml[(part_idx * 8 + tid) * 2 + 1], ml[tid][1]);
        }
    } else {
        // empty slice: neutral element of the merge
        for (int i = tid; i < 8 * DH; i += 256) store_dev(&a.part_o[part_idx * 8 * DH + i], 0.f);
        if (tid < 8) {
            store_dev(&a.part_ml[(part_idx * 8 + tid) * 2 + 0], -INFINITY);
            store_dev(&a.part_ml[(part_idx * 8 + tid) * 2 + 1], 0.f);
        }
    }

    // ---- 5. the last slice to arrive merges -----------------------------------------------------
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // this thread's write-through stores are acknowledged
    __syncthreads();
    if (tid == 0) {
        int prev = __hip_atomic_fetch_add(&a.counters[pair], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (prev == NS - 1) ? 1 : 0;
        if (prev == NS - 1) __hip_atomic_store(&a.counters[pair], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!s_last) return;

    const int KS = H * DH / 32;
    // merge weights exp(max_s - max*) and sums per (m, slice)
    {
        int m = tid >> 5, t = tid & 31;
        float ms0 = -INFINITY, ms1 = -INFINITY, l0 = 0.f, l1 = 0.f;      // slices t and t + 32
        if (t < NS) {
            ms0 = load_dev(&a.part_ml[((pair * NS + t) * 8 + m) * 2]);
            l0 = load_dev(&a.part_ml[((pair * NS + t) * 8 + m) * 2 + 1]);
        }
        if (t + 32 < NS) {
            ms1 = load_dev(&a.part_ml[((pair * NS + t + 32) * 8 + m) * 2]);
            l1 = load_dev(&a.part_ml[((pair * NS + t + 32) * 8 + m) * 2 + 1]);
        }
        float mstar = fmaxf(ms0, ms1);
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) mstar = fmaxf(mstar, __shfl_xor(mstar, o));
        if (t < NS) { wgt[m][t] = (ms0 == -INFINITY) ? 0.f : expf(ms0 - mstar); lsum[m][t] = l0; }
        if (t + 32 < NS) { wgt[m][t + 32] = (ms1 == -INFINITY) ? 0.f : expf(ms1 - mstar); lsum[m][t + 32] = l1; }
    }
    __syncthreads();
    // thread (m, q) merges 4 output dims; all its slice loads of a batch are issued before
    // the first is waited for (16-byte L2-bypassing loads), then summed in slice order
    constexpr int Q = DH / 4;
    if (tid < M * Q) {
        const int m = tid / Q, q = tid % Q;
        float num[4] = {0.f, 0.f, 0.f, 0.f}, den = 0.f;
        for (int sb = 0; sb < NS; sb += 16) {
            f32x4_t v[16];
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (sb + j < NS) {
                    const float *src = &a.part_o[((pair * NS + sb + j) * 8 + m) * DH + q * 4];
                    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v[j]) : "v"(src) : "memory");
                }
            asm volatile("s_waitcnt vmcnt(0)"
                         : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]),
                           "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]), "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15])
                         :
                         : "memory");
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (sb + j < NS) {
                    float wg = wgt[m][sb + j];
                    den += wg * lsum[m][sb + j];
#pragma unroll
                    for (int e = 0; e < 4; ++e) num[e] += wg * v[j][e];
                }
        }
        union { uint2 v; uint16_t h[4]; } h16, l16;
#pragma unroll
        for (int e = 0; e < 4; ++e) split_hi_lo(num[e] / den, h16.h[e], l16.h[e]);
        const int row = seq * M + m, k = hh * DH + q * 4;      // 4 consecutive k share a lane slot
        *reinterpret_cast<uint2 *>((uint16_t *)a.xout + xpack_index(row, k, KS, 0)) = h16.v;
        *reinterpret_cast<uint2 *>((uint16_t *)a.xout + xpack_index(row, k, KS, 1)) = l16.v;
    }
}

hipError_t launch_attention(const AttnArgs &a, hipStream_t stream) {
    if (a.split_len < 1 || a.split_len > kSplitMax || a.M < 1 || a.M > 8) return hipErrorInvalidValue;
    if (a.n_split < 1 || a.n_split > kMaxRows) return hipErrorInvalidValue;
    dim3 grid(a.n_split, a.H, a.n_seqs);
    if (a.dh == 128) {
        hipLaunchKernelGGL(attention_kernel<128>, grid, dim3(256), 0, stream, a);
    } else if (a.dh == 64) {
        hipLaunchKernelGGL(attention_kernel<64>, grid, dim3(256), 0, stream, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace spd
