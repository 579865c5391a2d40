// RoPE + KV-cache append + causal attention of up to 8 new queries per sequence and launch over
// the cached prefix (image rows + text + already accepted tokens), on the matrix cores.  The
// queries form groups of 5 (three bf16 terms each fill 15 of the 16 operand columns); 6..8
// queries are two groups multiplied with the same cached keys.  Longer runs of new rows (the
// prefill) take several launches: a later one sees the earlier ones' rows in the cache like any
// other prefix position.
//
// One workgroup (12 waves) per (sequence, head, slice of 16 or more output dimensions).  The cached keys are cut
// into units of 32; every wave owns a contiguous run of units and walks it 2 units (64 keys)
// at a time.  All loads of an iteration -- the K rows and the V columns of the wave's keys --
// are issued before anything is computed, so for contexts up to 768 keys the whole kernel pays
// a single round trip.  There is no cross-workgroup merge: every workgroup of a head scores
// all keys and produces its own slice of the output dimensions.  K is therefore read by all
// slices of a head; they are launched so that they share an XCD, whose L2 then serves the
// repeats (HBM sees K once), and V, the other half of the bytes, is read exactly once.
//
//   scores  S[key, m] = sum_d K[key, d] q[m, d]     v_mfma_f32_16x16x32_bf16, A = 16 keys x 32 dims
//           of the bf16 cache as stored, B = q as three bf16 terms (columns m, m + 5, m + 10 of
//           query m), so S is exact up to float32 rounding of q.
//   softmax per wave with running max / sum ("online"), wavefront shuffles for the
//           reductions across the 4 lane groups.
//   output  O[d, m] = sum_key V[key, d] p[m, key]   A = 16 dims x 32 keys of the TRANSPOSED V
//           cache (keys contiguous), B = p as three bf16 terms.
// The rows of the two score tiles of a unit are assigned to keys so that each lane ends up
// with the probabilities of 8 consecutive keys, which is exactly the B-operand slot of the
// second product: no data moves between lanes.
//
// The M new keys/values (this call's own rows, causal among themselves) are handled from
// LDS with plain float32 arithmetic as one more partial; the partials (one per wave + this one)
// are merged in a fixed order.  K (after RoPE) and V are rounded to bf16 -- the cache precision -- before
// they are used, appended to the cache, and the result is written as three bf16 terms in
// B-operand order for the O projection.
#pragma once
#include "launch.h"

namespace spd {

constexpr int kAttnWaves = 12;
constexpr int kUnitsPerIter = 2;      // units of 32 keys per wave per iteration

template <bool DEV>
__device__ __forceinline__ float ldf(const float *p) {
    if (DEV) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *p;
}

__device__ __forceinline__ f32x4_t mfma16(const uint4 &a, const uint4 &b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// x rounded to the nearest bf16 (ties to even), as a float
__device__ __forceinline__ float rne_bf16(float x) { return bf16_bits_to_f32(f32_to_bf16_bits(x)); }

__device__ __forceinline__ uint32_t pack2(uint16_t lo, uint16_t hi) { return (uint32_t)lo | ((uint32_t)hi << 16); }

// One (sequence, head, slice of the head dimension).  Must be called by all AW waves of the
// workgroup.  DEV: the float32 QKV rows were written by other workgroups of the same kernel and
// are read with device-scope loads.
// `rows_ready()` is called by every thread after the loads of the cached keys have been issued and
// before the new rows are read: the place to wait for their producer.
// QG: query groups of 5 handled by one launch (1: up to 5 new rows per sequence, 2: up to 8; the
// cached keys are then multiplied with both groups from the same registers).
template <int DH, int DS, int AW, int UPI, bool DEV, int QG, class ReadyFn>
__device__ __forceinline__ void attention_core(const AttnArgs &a, const int hh, const int ds, const int seq, ReadyFn rows_ready) {
    constexpr int HALF = DH / 2;
    constexpr int NC = DH / 32;                   // 32-dim chunks of a key row
    constexpr int DW = DH / DS;                   // output dims of this workgroup
    constexpr int NDT = DW / 16;                  // 16-dim tiles of this workgroup
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;
    const int M = a.Mq, H = a.H;                  // queries of this launch
    int P0 = a.d_lens ? a.d_lens[seq] : a.lens.len[seq];
    if (P0 < 0 || P0 + a.M > a.max_positions) {   // only possible with device-resident lengths
        if (a.d_error && threadIdx.x == 0) *a.d_error = 1;
        P0 = max(0, min(P0, a.max_positions - a.M));
    }
    const int P = P0 + a.m0;                      // cached positions before this launch's rows
    const int row_base = seq * a.M + a.m0;        // first row of this launch in qkv / xout
    const int dim0 = ds * DW;
    const size_t pair = (size_t)seq * H + hh;
    const size_t HD = (size_t)H * DH;
    const int VS = a.v_stride;                    // positions per row of the transposed V cache
    uint16_t *Kc = (uint16_t *)a.k_cache + pair * a.max_positions * DH;        // [pos][DH]
    uint16_t *Vt = (uint16_t *)a.v_cache + pair * (size_t)DH * VS;             // [VS / 32][DH][32]: see launch.h

    __shared__ float qf[8][DH];
    __shared__ float kf[8][DH];
    __shared__ float vf[8][DH];
    __shared__ uint16_t qb[QG][NC][64][8];        // q as matrix-core B operand (three bf16 terms), per query group
    __shared__ float pn[8][8];
    __shared__ float part_m[AW + 1][8];
    __shared__ float part_l[AW + 1][8];
    __shared__ float part_o[AW + 1][8][DW];

    // ---- key units of this wave; first iteration's loads go out before anything else --------
    const int n_units = (P + 31) / 32;
    const int u_begin = (n_units * w) / AW, u_end = (n_units * (w + 1)) / AW;

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
                    vreg[s][i] = *reinterpret_cast<const uint4 *>(Vt + ((size_t)unit * DH + dim0 + 16 * i + r) * 32 + 8 * g);
            }
        }
    };
    issue_loads(u_begin);
    rows_ready();

    // ---- RoPE on q, k of the new rows; bf16 rounding of new k, v; cache append ------------
    {
        const float scale = 1.0f / sqrtf((float)DH);
        for (int idx = tid; idx < (QG == 1 ? 8 : 10) * HALF; idx += AW * 64) {      // rows 8, 9: zero columns of group 1
            const int i = idx / HALF, j = idx % HALF;
            float qa = 0.f, qc = 0.f;
            if (i < M) {
                const int pos = P + i;
                const float *row = a.qkv + (size_t)(row_base + i) * 3 * HD + (size_t)hh * DH;
                const float c = a.rope[((size_t)pos * HALF + j) * 2 + 0];
                const float s = a.rope[((size_t)pos * HALF + j) * 2 + 1];
                const float q1 = ldf<DEV>(row + j), q2 = ldf<DEV>(row + j + HALF);
                const float k1 = ldf<DEV>(row + HD + j), k2 = ldf<DEV>(row + HD + j + HALF);
                const float v1 = ldf<DEV>(row + 2 * HD + j), v2 = ldf<DEV>(row + 2 * HD + j + HALF);
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
                    Vt[((size_t)(pos >> 5) * DH + j) * 32 + (pos & 31)] = vb1;
                    Vt[((size_t)(pos >> 5) * DH + j + HALF) * 32 + (pos & 31)] = vb2;
                }
            } else if (i < 8) {
                kf[i][j] = 0.f; kf[i][j + HALF] = 0.f;
                vf[i][j] = 0.f; vf[i][j + HALF] = 0.f;
            }
            if (i < 8) {
                qf[i][j] = qa;
                qf[i][j + HALF] = qc;
            }
            // B operand: column c + 5 t of group i / 5 holds bf16 term t of q_i, c = i % 5 (rows beyond M carry zeros)
            if (i < kGroupRows * QG) {
                uint16_t t1[kTerms], t2[kTerms];
                split3(qa, t1);
                split3(qc, t2);
                const int d1 = j, d2 = j + HALF, qg = i / kGroupRows, c5 = i % kGroupRows;
#pragma unroll
                for (int t = 0; t < kTerms; ++t) {
                    qb[qg][d1 >> 5][c5 + kGroupRows * t + 16 * ((d1 & 31) >> 3)][d1 & 7] = t1[t];
                    qb[qg][d2 >> 5][c5 + kGroupRows * t + 16 * ((d2 & 31) >> 3)][d2 & 7] = t2[t];
                }
            }
        }
        for (int idx = tid; idx < QG * DH; idx += AW * 64) {          // column 15 (unused): keep it finite
            const int qg = idx / DH, dd = idx % DH;
            qb[qg][dd >> 5][15 + 16 * ((dd & 31) >> 3)][dd & 7] = 0;
        }
    }
    __syncthreads();

    // ---- cached keys on the matrix cores ----------------------------------------------------
    float m_run[QG], l_run[QG];                   // of query 5 qg + r % 5 (replicated over lane groups and terms)
#pragma unroll
    for (int qg = 0; qg < QG; ++qg) { m_run[qg] = -INFINITY; l_run[qg] = 0.f; }
    const float sel0 = r < 5 ? 1.f : 0.f, sel1 = (r >= 5 && r < 10) ? 1.f : 0.f, sel2 = (r >= 10 && r < 15) ? 1.f : 0.f;
    f32x4_t acc_o[QG][NDT];
    uint4 qreg[QG][NC];
#pragma unroll
    for (int qg = 0; qg < QG; ++qg) {
#pragma unroll
        for (int i = 0; i < NDT; ++i) acc_o[qg][i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < NC; ++c) qreg[qg][c] = *reinterpret_cast<const uint4 *>(&qb[qg][c][lane][0]);
    }

    for (int u0 = u_begin; u0 < u_end; u0 += UPI) {
        if (u0 != u_begin) issue_loads(u0);
        // one online-softmax step per unit of 32 keys: its K registers die after the scores, its V
        // registers after the second product, so the units' temporaries never coexist
#pragma unroll
        for (int s = 0; s < UPI; ++s) {
            const int unit = u0 + s;
            if (unit >= u_end) break;                                  // wave-uniform
#pragma unroll
            for (int qg = 0; qg < QG; ++qg) {
                float sv[2][4];
                float mx = -INFINITY;
#pragma unroll
                for (int ab = 0; ab < 2; ++ab) {
                    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int c = 0; c < NC; ++c) acc = mfma16(kreg[s][ab][c], qreg[qg][c], acc);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float x = acc[v];                              // summed over the three term columns of this lane's query
                        x = sum_terms_all(x, r);
                        const int key = 32 * unit + 8 * g + 4 * ab + v;    // D row 4g + v of tile ab
                        x = key < P ? x : -INFINITY;
                        sv[ab][v] = x;
                        mx = fmaxf(mx, x);
                    }
                }
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run[qg], mx);              // finite: a unit has >= 1 valid key
                const float rescale = (m_run[qg] == -INFINITY) ? 0.f : expf(m_run[qg] - m_new);
                float lsum = 0.f;
                uint32_t hv[8];
#pragma unroll
                for (int ab = 0; ab < 2; ++ab)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float p = sv[ab][v] == -INFINITY ? 0.f : exp_neg(sv[ab][v] - m_new);   // masked keys: 0
                        lsum += p;
                        // this lane's column carries term r / 5 of query r % 5: p, p - t0 or p - t0 - t1
                        const float r1 = p - rne_bf16(p);
                        const float r2 = r1 - rne_bf16(r1);
                        hv[4 * ab + v] = f32_to_bf16_bits(sel0 * p + sel1 * r1 + sel2 * r2);
                    }
                const uint4 pb = uint4{hv[0] | (hv[1] << 16), hv[2] | (hv[3] << 16), hv[4] | (hv[5] << 16), hv[6] | (hv[7] << 16)};
                lsum += __shfl_xor(lsum, 16);
                lsum += __shfl_xor(lsum, 32);
                l_run[qg] = l_run[qg] * rescale + lsum;
                m_run[qg] = m_new;
#pragma unroll
                for (int i = 0; i < NDT; ++i) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc_o[qg][i][v] *= rescale;
                    acc_o[qg][i] = mfma16(vreg[s][i], pb, acc_o[qg][i]);
                }
            }
        }
    }
    // partial of this wave: O[dim 16 i + 4 g + v][column r]; the three term columns summed
#pragma unroll
    for (int qg = 0; qg < QG; ++qg) {
        const int m = qg * kGroupRows + r;            // query of this lane's column (rows beyond 7 do not exist)
#pragma unroll
        for (int i = 0; i < NDT; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float x = sum_terms(acc_o[qg][i][v]);
                if (r < kGroupRows && m < 8) part_o[w][m][16 * i + 4 * g + v] = x;
            }
        if (lane < kGroupRows && m < 8) { part_m[w][m] = m_run[qg]; part_l[w][m] = l_run[qg]; }
    }

    // ---- the M new keys (causal among the new rows), float32 from LDS -----------------------
    if (w == 0) {                                   // wave 0 owns the fewest key units
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
        if (j == 0) { part_m[AW][m] = mx; part_l[AW][m] = l; }
    }
    __syncthreads();
    if (w == 0) {                                   // wave 0 owns the fewest key units
        const int m = lane >> 3, j = lane & 7;
        for (int dd = j; dd < DW; dd += 8) {
            float o = 0.f;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) o += pn[m][jj] * vf[jj][dim0 + dd];
            part_o[AW][m][dd] = o;
        }
    }
    __syncthreads();

    // ---- merge the 8 + 1 partials in index order, write the B operand of the O projection ----
    const int KS = H * DH / 32;
    for (int idx = tid; idx < M * DW; idx += AW * 64) {
        const int m = idx / DW, dd = idx % DW;
        float mstar = -INFINITY;
#pragma unroll
        for (int p = 0; p <= AW; ++p) mstar = fmaxf(mstar, part_m[p][m]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int p = 0; p <= AW; ++p) {
            const float pm = part_m[p][m];
            const float wg = (pm == -INFINITY) ? 0.f : expf(pm - mstar);
            den += wg * part_l[p][m];
            num += wg * part_o[p][m][dd];
        }
        uint16_t t3[kTerms];
        split3(num / den, t3);
        const int row = row_base + m, k = hh * DH + dim0 + dd;
#pragma unroll
        for (int t = 0; t < kTerms; ++t) ((uint16_t *)a.xout)[xpack_index(row, k, KS, t)] = t3[t];
    }
}

}  // namespace spd
