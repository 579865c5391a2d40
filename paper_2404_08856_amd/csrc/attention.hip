// RoPE + KV-cache append + causal attention of M <= 8 new queries per sequence over the
// cached prefix (image rows + text + already accepted tokens), on the matrix cores.
//
// One workgroup (8 waves) per (sequence, head, half of the head dimension).  The cached
// keys are cut into units of 32; every wave owns a contiguous run of units and walks it
// 3 units (96 keys) at a time.  All loads of an iteration -- the K rows and the V columns of
// the wave's keys -- are issued before anything is computed, so for contexts up to 768 keys
// the whole kernel pays a single HBM round trip.  There is no cross-workgroup merge: the
// two workgroups of a head both score all keys (K is read twice, V once) and each produces
// its own half of the output dimensions.
//
//   scores  S[key, m] = sum_d K[key, d] q[m, d]     v_mfma_f32_16x16x32_bf16, A = 16 keys x 32 dims
//           of the bf16 cache as stored, B = q as bf16 head (columns 0..7) + bf16 tail
//           (columns 8..15), so S is exact up to float32 rounding of q.
//   softmax per wave with running max / sum ("online"), wavefront shuffles for the
//           reductions across the 4 lane groups.
//   output  O[d, m] = sum_key V[key, d] p[m, key]   A = 16 dims x 32 keys of the TRANSPOSED V
//           cache (keys contiguous), B = p as bf16 head + tail.
// The rows of the two score tiles of a unit are assigned to keys so that each lane ends up
// with the probabilities of 8 consecutive keys, which is exactly the B-operand slot of the
// second product: no data moves between lanes.
//
// The M new keys/values (this call's own rows, causal among themselves) are handled from
// LDS with plain float32 arithmetic as one more partial; the 8 + 1 partials are merged in a
// fixed order.  K (after RoPE) and V are rounded to bf16 -- the cache precision -- before
// they are used, appended to the cache, and the result is written as bf16 head + tail in
// B-operand order for the O projection.
#include "launch.h"

namespace spd {

constexpr int kAttnWaves = 8;
constexpr int kUnitsPerIter = 3;      // units of 32 keys per wave per iteration

__device__ __forceinline__ f32x4_t mfma16(const uint4 &a, const uint4 &b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack2(uint16_t lo, uint16_t hi) { return (uint32_t)lo | ((uint32_t)hi << 16); }

template <int DH, int DS>
__global__ __launch_bounds__(kAttnWaves * 64) void attention_kernel(AttnArgs a) {
    constexpr int HALF = DH / 2;
    constexpr int NC = DH / 32;                   // 32-dim chunks of a key row
    constexpr int DW = DH / DS;                   // output dims of this workgroup
    constexpr int NDT = DW / 16;                  // 16-dim tiles of this workgroup
    constexpr int UPI = kUnitsPerIter;
    const int ds = blockIdx.x, hh = blockIdx.y, seq = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;
    const int M = a.M, H = a.H;
    const int P = a.lens.len[seq];                // cached positions before this call
    const int dim0 = ds * DW;
    const size_t pair = (size_t)seq * H + hh;
    const size_t HD = (size_t)H * DH;
    const int VS = a.v_stride;                    // positions per row of the transposed V cache
    uint16_t *Kc = (uint16_t *)a.k_cache + pair * a.max_positions * DH;        // [pos][DH]
    uint16_t *Vt = (uint16_t *)a.v_cache + pair * (size_t)DH * VS;             // [DH][VS]

    __shared__ float qf[8][DH];
    __shared__ float kf[8][DH];
    __shared__ float vf[8][DH];
    __shared__ uint16_t qb[NC][64][8];            // q as matrix-core B operand (head | tail)
    __shared__ float pn[8][8];
    __shared__ float part_m[kAttnWaves + 1][8];
    __shared__ float part_l[kAttnWaves + 1][8];
    __shared__ float part_o[kAttnWaves + 1][8][DW];

    // ---- key units of this wave; first iteration's loads go out before anything else --------
    const int n_units = (P + 31) / 32;
    const int u_begin = (n_units * w) / kAttnWaves, u_end = (n_units * (w + 1)) / kAttnWaves;

    uint4 kreg[UPI][2][NC], vreg[UPI][NDT];
    auto issue_loads = [&](int u0) {
#pragma unroll
        for (int s = 0; s < UPI; ++s) {
            const int unit = u0 + s;
            if (unit < u_end) {                                        // wave-uniform
#pragma unroll
                for (int ab = 0; ab < 2; ++ab) {
                    int key = 32 * unit + 8 * (r >> 2) + 4 * ab + (r & 3);
                    key = min(key, P - 1);                             // stay inside the valid rows
                    const uint16_t *row = Kc + (size_t)key * DH + g * 8;
#pragma unroll
                    for (int c = 0; c < NC; ++c) kreg[s][ab][c] = *reinterpret_cast<const uint4 *>(row + c * 32);
                }
#pragma unroll
                for (int i = 0; i < NDT; ++i)
                    vreg[s][i] = *reinterpret_cast<const uint4 *>(Vt + (size_t)(dim0 + 16 * i + r) * VS + 32 * unit + 8 * g);
            }
        }
    };
    issue_loads(u_begin);

    // ---- RoPE on q, k of the new rows; bf16 rounding of new k, v; cache append ------------
    {
        const float scale = 1.0f / sqrtf((float)DH);
        for (int idx = tid; idx < 8 * HALF; idx += kAttnWaves * 64) {
            const int i = idx / HALF, j = idx % HALF;
            float qa = 0.f, qc = 0.f;
            if (i < M) {
                const int pos = P + i;
                const float *row = a.qkv + (size_t)(seq * M + i) * 3 * HD + (size_t)hh * DH;
                const float c = a.rope[((size_t)pos * HALF + j) * 2 + 0];
                const float s = a.rope[((size_t)pos * HALF + j) * 2 + 1];
                const float q1 = row[j], q2 = row[j + HALF];
                const float k1 = row[HD + j], k2 = row[HD + j + HALF];
                const float v1 = row[2 * HD + j], v2 = row[2 * HD + j + HALF];
                qa = (q1 * c - q2 * s) * scale;
                qc = (q2 * c + q1 * s) * scale;
                const uint16_t kb1 = f32_to_bf16_bits(k1 * c - k2 * s);
                const uint16_t kb2 = f32_to_bf16_bits(k2 * c + k1 * s);
                const uint16_t vb1 = f32_to_bf16_bits(v1), vb2 = f32_to_bf16_bits(v2);
                kf[i][j] = bf16_bits_to_f32(kb1);
                kf[i][j + HALF] = bf16_bits_to_f32(kb2);
                vf[i][j] = bf16_bits_to_f32(vb1);
                vf[i][j + HALF] = bf16_bits_to_f32(vb2);
                if (ds == 0) {                                         // one workgroup of the head appends
                    Kc[(size_t)pos * DH + j] = kb1;
                    Kc[(size_t)pos * DH + j + HALF] = kb2;
                    Vt[(size_t)j * VS + pos] = vb1;
                    Vt[(size_t)(j + HALF) * VS + pos] = vb2;
                }
            } else {
                kf[i][j] = 0.f; kf[i][j + HALF] = 0.f;
                vf[i][j] = 0.f; vf[i][j + HALF] = 0.f;
            }
            qf[i][j] = qa;
            qf[i][j + HALF] = qc;
            // B operand: column i holds the bf16 head of q_i, column i + 8 the bf16 tail
            uint16_t h1, l1, h2, l2;
            split_hi_lo(qa, h1, l1);
            split_hi_lo(qc, h2, l2);
            const int d1 = j, d2 = j + HALF;
            qb[d1 >> 5][i + 16 * ((d1 & 31) >> 3)][d1 & 7] = h1;
            qb[d1 >> 5][i + 8 + 16 * ((d1 & 31) >> 3)][d1 & 7] = l1;
            qb[d2 >> 5][i + 16 * ((d2 & 31) >> 3)][d2 & 7] = h2;
            qb[d2 >> 5][i + 8 + 16 * ((d2 & 31) >> 3)][d2 & 7] = l2;
        }
    }
    __syncthreads();

    // ---- cached keys on the matrix cores ----------------------------------------------------
    float m_run = -INFINITY, l_run = 0.f;         // per query column r & 7 (replicated over lane groups)
    f32x4_t acc_o[NDT];
#pragma unroll
    for (int i = 0; i < NDT; ++i) acc_o[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    uint4 qreg[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) qreg[c] = *reinterpret_cast<const uint4 *>(&qb[c][lane][0]);

    for (int u0 = u_begin; u0 < u_end; u0 += UPI) {
        if (u0 != u_begin) issue_loads(u0);
        float sv[UPI][2][4];
        float mx = -INFINITY;
#pragma unroll
        for (int s = 0; s < UPI; ++s) {
            const int unit = u0 + s;
#pragma unroll
            for (int ab = 0; ab < 2; ++ab) {
                f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
                if (unit < u_end) {
#pragma unroll
                    for (int c = 0; c < NC; ++c) acc = mfma16(kreg[s][ab][c], qreg[c], acc);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float x = acc[v];
                    x += __shfl_xor(x, 8);                             // head + tail columns
                    const int key = 32 * unit + 8 * g + 4 * ab + v;    // D row 4g + v of tile ab
                    x = (unit < u_end && key < P) ? x : -INFINITY;
                    sv[s][ab][v] = x;
                    mx = fmaxf(mx, x);
                }
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);                          // finite: the wave has >= 1 valid key
        const float rescale = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
        float lsum = 0.f;
        uint4 pb[UPI];
#pragma unroll
        for (int s = 0; s < UPI; ++s) {
            uint16_t hv[8];
#pragma unroll
            for (int ab = 0; ab < 2; ++ab)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float p = expf(sv[s][ab][v] - m_new);        // exp(-inf) = 0 for masked keys
                    lsum += p;
                    uint16_t hi, lo;
                    split_hi_lo(p, hi, lo);
                    hv[4 * ab + v] = (r < 8) ? hi : lo;                // columns 0..7 head, 8..15 tail
                }
            pb[s] = uint4{pack2(hv[0], hv[1]), pack2(hv[2], hv[3]), pack2(hv[4], hv[5]), pack2(hv[6], hv[7])};
        }
        lsum += __shfl_xor(lsum, 16);
        lsum += __shfl_xor(lsum, 32);
        l_run = l_run * rescale + lsum;
        m_run = m_new;
#pragma unroll
        for (int i = 0; i < NDT; ++i) {
#pragma unroll
            for (int v = 0; v < 4; ++v) acc_o[i][v] *= rescale;
        }
#pragma unroll
        for (int s = 0; s < UPI; ++s) {
            if (u0 + s < u_end) {
#pragma unroll
                for (int i = 0; i < NDT; ++i) acc_o[i] = mfma16(vreg[s][i], pb[s], acc_o[i]);
            }
        }
    }
    // partial of this wave: O[dim 16 i + 4 g + v][column r]; head + tail columns summed
#pragma unroll
    for (int i = 0; i < NDT; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float x = acc_o[i][v];
            x += __shfl_xor(x, 8);
            if (r < 8) part_o[w][r][16 * i + 4 * g + v] = x;
        }
    if (lane < 8) { part_m[w][lane] = m_run; part_l[w][lane] = l_run; }

    // ---- the M new keys (causal among the new rows), float32 from LDS -----------------------
    if (w == kAttnWaves - 1) {
        const int m = lane >> 3, j = lane & 7;
        float s = -INFINITY;
        if (m < M && j <= m) {
            s = 0.f;
            for (int e = 0; e < DH; ++e) s += qf[m][e] * kf[j][e];
        }
        float mx = s;
        mx = fmaxf(mx, __shfl_xor(mx, 1));
        mx = fmaxf(mx, __shfl_xor(mx, 2));
        mx = fmaxf(mx, __shfl_xor(mx, 4));
        const float p = (mx == -INFINITY) ? 0.f : expf(s - mx);        // rows m >= M: nothing visible
        float l = p;
        l += __shfl_xor(l, 1);
        l += __shfl_xor(l, 2);
        l += __shfl_xor(l, 4);
        pn[m][j] = p;
        if (j == 0) { part_m[kAttnWaves][m] = mx; part_l[kAttnWaves][m] = l; }
    }
    __syncthreads();
    if (w == kAttnWaves - 1) {
        const int m = lane >> 3, j = lane & 7;
        for (int dd = j; dd < DW; dd += 8) {
            float o = 0.f;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) o += pn[m][jj] * vf[jj][dim0 + dd];
            part_o[kAttnWaves][m][dd] = o;
        }
    }
    __syncthreads();

    // ---- merge the 8 + 1 partials in index order, write the B operand of the O projection ----
    const int KS = H * DH / 32;
    for (int idx = tid; idx < M * DW; idx += kAttnWaves * 64) {
        const int m = idx / DW, dd = idx % DW;
        float mstar = -INFINITY;
#pragma unroll
        for (int p = 0; p <= kAttnWaves; ++p) mstar = fmaxf(mstar, part_m[p][m]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int p = 0; p <= kAttnWaves; ++p) {
            const float pm = part_m[p][m];
            const float wg = (pm == -INFINITY) ? 0.f : expf(pm - mstar);
            den += wg * part_l[p][m];
            num += wg * part_o[p][m][dd];
        }
        uint16_t hi, lo;
        split_hi_lo(num / den, hi, lo);
        const int row = seq * M + m, k = hh * DH + dim0 + dd;
        ((uint16_t *)a.xout)[xpack_index(row, k, KS, 0)] = hi;
        ((uint16_t *)a.xout)[xpack_index(row, k, KS, 1)] = lo;
    }
}

hipError_t launch_attention(const AttnArgs &a, hipStream_t stream) {
    if (a.M < 1 || a.M > 8 || (a.v_stride % 32) != 0 || a.v_stride < a.max_positions) return hipErrorInvalidValue;
    if (a.dh == 128) {
        hipLaunchKernelGGL((attention_kernel<128, 2>), dim3(2, a.H, a.n_seqs), dim3(kAttnWaves * 64), 0, stream, a);
    } else if (a.dh == 64) {
        hipLaunchKernelGGL((attention_kernel<64, 1>), dim3(1, a.H, a.n_seqs), dim3(kAttnWaves * 64), 0, stream, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace spd
