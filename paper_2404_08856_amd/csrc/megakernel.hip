// One persistent kernel for a whole decoder forward over up to 5 rows = one row group (the
// verify step at gamma + 1 <= 5, a draft step, a prefill pass).
//
// Why: at 5 rows every projection is a 5-15 us stream over its weights, and a layer is five
// dependent stages (QKV, attention, O, gate|up, down).  As separate launches each stage pays
// its own ramp-up and drain (first loads in flight, last tile's reduction and stores), during
// which HBM idles.  Here one workgroup per CU stays resident for the whole forward; the
// stages are separated by a device-wide barrier, and -- because the weights do not depend on
// the activations -- every wave refills its register ring with the first blocks of the NEXT
// stage's weights while the current stage drains and the barrier is crossed.  The O
// projection's entire weight matrix streams in while attention runs.
//
// Data between stages lives in small float32 row-major arrays ([8][K], 5 rows used); a consumer
// rebuilds its matrix-core B operand (three bf16 terms, see common.h) from them in registers.
// Workgroups run on different XCDs, each with its own L2, so these arrays are written with
// device-scope (write-through) stores and read with device-scope (L2-bypassing) loads; a
// producer waits for its stores to be acknowledged before it arrives at the barrier.
#include "launch.h"

namespace spd {

constexpr int kMW = 8;            // waves per workgroup
constexpr int kRing = 16;         // 1 KiB weight blocks a wave keeps in flight

typedef __attribute__((ext_vector_type(4))) float fx4;

// ---- device-scope accesses ---------------------------------------------------------------
__device__ __forceinline__ void st_dev(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_dev(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
// 16 bytes as two 8-byte device-scope loads (relaxed atomics are tracked by the compiler like
// ordinary loads, so a batch of them is issued back to back and waited for at first use)
__device__ __forceinline__ fx4 ld_dev4(const float *p) {
    const unsigned long long *q = reinterpret_cast<const unsigned long long *>(p);
    unsigned long long a = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned long long b = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return fx4{__uint_as_float((unsigned)a), __uint_as_float((unsigned)(a >> 32)),
               __uint_as_float((unsigned)b), __uint_as_float((unsigned)(b >> 32))};
}
__device__ __forceinline__ void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ fx4 mfma_b(const uint4 &a, const uint4 &b, fx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
__device__ __forceinline__ uint4 ld_stream(const uint4 *p) {
    typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
    u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return uint4{v.x, v.y, v.z, v.w};
}
__device__ __forceinline__ uint32_t pk2(uint16_t lo, uint16_t hi) { return (uint32_t)lo | ((uint32_t)hi << 16); }

// ---- device-wide barrier -------------------------------------------------------------------
// All workgroups are resident (cooperative launch).  `target` is the value the arrival counter
// reaches when every workgroup has arrived; the counter only grows (the host passes the base).
// The spin is bounded: if the limit is hit the abort flag is raised and every later barrier
// falls through, so the grid always drains.
__device__ __forceinline__ void grid_barrier(unsigned *bar, unsigned target, int *abort_flag) {
    // Data that crosses the barrier is written with device-scope (write-through) stores and
    // read with device-scope loads, so no cache write-back or invalidate is needed here --
    // only that this wave's stores have been acknowledged.  (Full release/acquire fences at
    // this point were measured at roughly 50 us per barrier with 256 workgroups.)
    wait_all_loads();
    __syncthreads();
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (__hip_atomic_load(abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
            unsigned spins = 0;
            while ((int)(__hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
                __builtin_amdgcn_s_sleep(2);
                if (++spins > (1u << 22)) {
                    __hip_atomic_store(abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
            }
        }
    }
    __syncthreads();
}

// ---- B operand from a float32 activation array --------------------------------------------
// One K-step of the B operand is 8 rows x 32 floats = one 16-byte load per lane: lane l reads
// row l / 8, floats 4 (l % 8) .. +3.  conv = 1 KiB of LDS private to the wave, used to
// re-arrange the three bf16 terms into operand order (lane c + 16 g: column c, k = 8 g .. 8 g + 7).
__device__ __forceinline__ uint4 to_b_operand(fx4 raw, bool row_valid, uint2 *conv, int lane) {
    const int rho = lane >> 3, kap = lane & 7;
    union { uint2 v; uint16_t h[4]; } term[kTerms];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float x = row_valid ? raw[e] : 0.f;
        uint16_t t3[kTerms];
        split3(x, t3);
#pragma unroll
        for (int t = 0; t < kTerms; ++t) term[t].h[e] = t3[t];
    }
    const int g = kap >> 1, half = kap & 1;
    asm volatile("" ::: "memory");                      // keep the LDS accesses below in program order
    if (rho < kGroupRows) {                             // column rho + 5 t: bf16 term t of row rho
#pragma unroll
        for (int t = 0; t < kTerms; ++t) conv[(rho + kGroupRows * t + 16 * g) * 2 + half] = term[t].v;
    } else if (rho == kGroupRows) {                     // column 15 is unused: keep it zero
        conv[(15 + 16 * g) * 2 + half] = uint2{0u, 0u};
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // LDS ops of one wave complete in order
    uint2 a0 = conv[lane * 2], a1 = conv[lane * 2 + 1];
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    return uint4{a0.x, a0.y, a1.x, a1.y};
}

struct GemmStage {
    const uint4 *W; int KS, n_tiles;       // packed weights of this stage
    const float *X; int ldx;               // float32 activations [8][ldx], K = ldx
    int rows, epi;
    float *Y; int ldy;                     // STORE target, or h for RESIDUAL
    bool y_dev;                            // Y is consumed later in this kernel (device-scope stores)
    const float *ssq_in; int ssq_parts; float inv_d, eps;   // RMSNorm scale of the input rows (NULL: 1)
    float *Yg; const float *gain_next; float *ssq_out;      // RESIDUAL: gain-scaled copy + sums of squares
    float *Xf; int ldf;                    // SWIGLU output
    const uint4 *succ_W; int succ_KS, succ_tiles;           // next GEMM stage (ring prefetch), W = NULL: none
};

struct WaveSplit { int s0, ns; };
__device__ __forceinline__ WaveSplit wave_split(int KS, int w) {
    int s0 = (KS * w) / kMW, s1 = (KS * (w + 1)) / kMW;
    return WaveSplit{s0, s1 - s0};
}

// first blocks of tile `t` of matrix W into the ring
__device__ __forceinline__ void prime_ring(uint4 (&ring)[kRing], const uint4 *W, int KS, int t, int w, int lane) {
    WaveSplit sp = wave_split(KS, w);
#pragma unroll
    for (int u = 0; u < kRing; ++u)
        if (u < sp.ns) ring[u] = ld_stream(W + ((size_t)t * KS + sp.s0 + u) * 64 + lane);
}

// One GEMM stage.  Precondition: if this workgroup owns a tile (blockIdx.x < n_tiles) the ring
// holds positions 0 .. min(16, ns) - 1 of its first tile.  Postcondition: the same for the
// successor stage.  RESIDENT: the wave's whole activation slice fits 16 registers (ns <= 16).
template <bool RESIDENT>
__device__ __forceinline__ void gemm_stage(const GemmStage &st, uint4 (&ring)[kRing], float (*red)[kMW][16][8],
                                           float *inv_s, uint2 *conv, int lane, int w) {
    const int b = blockIdx.x, G = gridDim.x;
    const int KS = st.KS;
    const WaveSplit sp = wave_split(KS, w);
    const int s0 = sp.s0, ns = sp.ns;
    const WaveSplit ssp = wave_split(st.succ_W ? st.succ_KS : 0, w);
    const bool succ_mine = st.succ_W && b < st.succ_tiles;
    const uint4 *succ_base = succ_mine ? st.succ_W + ((size_t)b * st.succ_KS + ssp.s0) * 64 : st.W;
    const int succ_ns = succ_mine ? ssp.ns : 0;

    if (b >= st.n_tiles) {                              // idle in this stage: just get ready for the next
        if (succ_mine) prime_ring(ring, st.succ_W, st.succ_KS, b, w, lane);
        return;
    }

    // ---- activation slice (and the RMS statistics): one batch of device-scope loads ----------
    const int rho = lane >> 3, kap = lane & 7;
    const bool row_valid = rho < st.rows;
    const int en = lane & 15, em = (w & 1) * 4 + (lane >> 4);     // epilogue element of this thread
    const bool row_ok = em < st.rows;
    fx4 braw[kRing];                                    // raw float32 block, then (same registers) the B operand
    float sq[4];
    if (RESIDENT) {
#pragma unroll
        for (int i = 0; i < kRing; ++i)
            if (i < ns && row_valid) braw[i] = ld_dev4(st.X + (size_t)rho * st.ldx + 32 * (s0 + i) + 4 * kap);
    }
    if (st.ssq_in && w < st.rows) {                     // wave w sums the partials of row w
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (lane + 64 * j < st.ssq_parts) sq[j] = ld_dev(st.ssq_in + (size_t)(lane + 64 * j) * 8 + w);
    }
    if (st.ssq_in) {
        if (w < st.rows) {
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (lane + 64 * j < st.ssq_parts) sum += sq[j];
            }
            for (int p = lane + 256; p < st.ssq_parts; p += 64) sum += ld_dev(st.ssq_in + (size_t)p * 8 + w);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
            if (lane == 0) inv_s[w] = 1.0f / sqrtf(sum * st.inv_d + st.eps);
        }
        __syncthreads();
    }
    const float inv_row = (st.ssq_in && row_ok) ? inv_s[em] : 1.0f;
    if (RESIDENT) {
#pragma unroll
        for (int i = 0; i < kRing; ++i) {
            if (i < ns) braw[i] = __builtin_bit_cast(fx4, to_b_operand(braw[i], row_valid, conv + (i & 1) * 128, lane));
        }
    }

    int parity = 0, turn = 0;
    for (int t = b; t < st.n_tiles; t += G, parity ^= 1, turn = (turn + 2) % kMW) {
        const int tn = t + G;
        const bool has_next = tn < st.n_tiles;
        const bool my_turn = (w == turn) || (w == turn + 1);
        const bool e_active = my_turn && row_ok && (st.epi != EPI_SWIGLU || en < 8);
        float hold = 0.f;
        if (st.epi == EPI_RESIDUAL && e_active) hold = ld_dev(st.Y + (size_t)em * st.ldy + (size_t)t * 16 + en);

        // where the slot refills of this tile's last positions come from
        const uint4 *nbase = has_next ? st.W + ((size_t)tn * KS + s0) * 64 : succ_base;
        const int nns = has_next ? ns : succ_ns;

        fx4 acc = {0.f, 0.f, 0.f, 0.f};
        if (RESIDENT) {
#pragma unroll
            for (int i = 0; i < kRing; ++i) {
                if (i < ns) {
                    acc = mfma_b(ring[i], __builtin_bit_cast(uint4, braw[i]), acc);
                    // ns <= 16: the slot's next block is position i of the next tile / stage
                    ring[i] = ld_stream(nbase + (size_t)(i < nns ? i : 0) * 64 + lane);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            // streamed activations: raw float32 blocks ride in a second ring (this stage only)
            if (t == b) {
#pragma unroll
                for (int u = 0; u < kRing; ++u)
                    if (u < ns && row_valid) braw[u] = ld_dev4(st.X + (size_t)rho * st.ldx + 32 * (s0 + u) + 4 * kap);
            }
            for (int c = 0; c * kRing < ns; ++c) {
#pragma unroll
                for (int u = 0; u < kRing; ++u) {
                    const int i = c * kRing + u;
                    if (i < ns) {
                        uint4 bb = to_b_operand(braw[u], row_valid, conv + (u & 1) * 128, lane);
                        acc = mfma_b(ring[u], bb, acc);
                        const int i2 = i + kRing;
                        if (i2 < ns) {
                            ring[u] = ld_stream(st.W + ((size_t)t * KS + s0 + i2) * 64 + lane);
                            if (row_valid) braw[u] = ld_dev4(st.X + (size_t)rho * st.ldx + 32 * (s0 + i2) + 4 * kap);
                        } else {
                            ring[u] = ld_stream(nbase + (size_t)(u < nns ? u : 0) * 64 + lane);
                            if (has_next && row_valid) braw[u] = ld_dev4(st.X + (size_t)rho * st.ldx + 32 * (s0 + u) + 4 * kap);
                        }
                    }
                }
            }
        }

        // D[n = 4 (lane / 16) + v][c = lane % 16]; columns c and c + 8 are head and tail of row c
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float x = sum_terms(acc[v]);
            if ((lane & 15) < kGroupRows) red[parity][w][4 * (lane >> 4) + v][lane & 15] = x;
        }
        __syncthreads();
        if (!my_turn) continue;

        if (st.epi == EPI_SWIGLU) {
            if (e_active) {
                float gate = 0.f, up = 0.f;
#pragma unroll
                for (int ww = 0; ww < kMW; ++ww) { gate += red[parity][ww][en][em]; up += red[parity][ww][en + 8][em]; }
                gate *= inv_row;
                up *= inv_row;
                st_dev(st.Xf + (size_t)em * st.ldf + t * 8 + en, gate / (1.0f + expf(-gate)) * up);
            }
        } else {
            float sum = 0.f;
#pragma unroll
            for (int ww = 0; ww < kMW; ++ww) sum += red[parity][ww][en][em];
            sum *= inv_row;
            const int col = t * 16 + en;
            if (st.epi == EPI_STORE) {
                if (e_active) {
                    if (st.y_dev) st_dev(st.Y + (size_t)em * st.ldy + col, sum);
                    else st.Y[(size_t)em * st.ldy + col] = sum;
                }
            } else {
                float hnew = e_active ? hold + sum : 0.f;
                if (e_active) {
                    st_dev(st.Y + (size_t)em * st.ldy + col, hnew);
                    st_dev(st.Yg + (size_t)em * st.ldy + col, hnew * st.gain_next[col]);
                }
                float q = hnew * hnew;
#pragma unroll
                for (int o = 8; o > 0; o >>= 1) q += __shfl_xor(q, o);
                if (en == 0 && e_active) st_dev(st.ssq_out + (size_t)t * 8 + em, q);
            }
        }
    }
    // successor positions that this stage's (shorter) K range never cycled through
    if (succ_mine) {
#pragma unroll
        for (int i = 0; i < kRing; ++i)
            if (i >= ns && i < succ_ns) ring[i] = ld_stream(succ_base + (size_t)i * 64 + lane);
    }
}

// ---- attention item: one (sequence, head, slice of the head dimension) --------------------
// Same algorithm as the stand-alone attention kernel, 2 key units per wave per iteration to
// leave registers for the weight ring, float32 input/output arrays with device-scope access.
struct MegaAttn {
    const float *qkv;        // [rows][3 HD]
    const float *rope;
    uint16_t *k_cache, *v_cache;
    float *att;              // [rows][HD]
    int M, H, max_positions, v_stride;
};

template <int DH, int DS>
__device__ __forceinline__ void attention_item(const MegaAttn &a, int ds, int hh, int seq, int P, char *lds, int lane, int w) {
    constexpr int HALF = DH / 2, NC = DH / 32, DW = DH / DS, NDT = DW / 16, UPI = 2;
    const int tid = threadIdx.x;
    const int r = lane & 15, g = lane >> 4;
    const int M = a.M, H = a.H;
    const int dim0 = ds * DW;
    const size_t pair = (size_t)seq * H + hh;
    const size_t HD = (size_t)H * DH;
    const int VS = a.v_stride;
    uint16_t *Kc = a.k_cache + pair * a.max_positions * DH;
    uint16_t *Vt = a.v_cache + pair * (size_t)DH * VS;

    float (*qf)[DH] = reinterpret_cast<float (*)[DH]>(lds);
    float (*kf)[DH] = reinterpret_cast<float (*)[DH]>(lds + 8 * DH * 4);
    float (*vf)[DH] = reinterpret_cast<float (*)[DH]>(lds + 16 * DH * 4);
    uint16_t (*qb)[64][8] = reinterpret_cast<uint16_t (*)[64][8]>(lds + 24 * DH * 4);
    float (*pn)[8] = reinterpret_cast<float (*)[8]>(lds + 24 * DH * 4 + NC * 1024);
    float (*part_m)[8] = reinterpret_cast<float (*)[8]>(lds + 24 * DH * 4 + NC * 1024 + 256);
    float (*part_l)[8] = reinterpret_cast<float (*)[8]>(lds + 24 * DH * 4 + NC * 1024 + 256 + (kMW + 1) * 32);
    float (*part_o)[8][DW] = reinterpret_cast<float (*)[8][DW]>(lds + 24 * DH * 4 + NC * 1024 + 256 + (kMW + 1) * 64);

    const int n_units = (P + 31) / 32;
    const int u_begin = (n_units * w) / kMW, u_end = (n_units * (w + 1)) / kMW;

    uint4 kreg[UPI][2][NC], vreg[UPI][NDT];
    auto issue_loads = [&](int u0) {
#pragma unroll
        for (int s = 0; s < UPI; ++s) {
            const int unit = u0 + s;
            if (unit < u_end) {
#pragma unroll
                for (int ab = 0; ab < 2; ++ab) {
                    int key = 32 * unit + 8 * (r >> 2) + 4 * ab + (r & 3);
                    key = min(key, P - 1);
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

    // RoPE on q, k of the new rows; bf16 rounding of new k, v; cache append
    {
        const float scale = 1.0f / sqrtf((float)DH);
        for (int idx = tid; idx < 8 * HALF; idx += kMW * 64) {
            const int i = idx / HALF, j = idx % HALF;
            float qa = 0.f, qc = 0.f;
            if (i < M) {
                const int pos = P + i;
                const float *row = a.qkv + (size_t)(seq * M + i) * 3 * HD + (size_t)hh * DH;
                const float q1 = ld_dev(row + j), q2 = ld_dev(row + j + HALF);
                const float k1 = ld_dev(row + HD + j), k2 = ld_dev(row + HD + j + HALF);
                const float v1 = ld_dev(row + 2 * HD + j), v2 = ld_dev(row + 2 * HD + j + HALF);
                const float c = a.rope[((size_t)pos * HALF + j) * 2 + 0];
                const float s = a.rope[((size_t)pos * HALF + j) * 2 + 1];
                qa = (q1 * c - q2 * s) * scale;
                qc = (q2 * c + q1 * s) * scale;
                const uint16_t kb1 = f32_to_bf16_bits(k1 * c - k2 * s);
                const uint16_t kb2 = f32_to_bf16_bits(k2 * c + k1 * s);
                const uint16_t vb1 = f32_to_bf16_bits(v1), vb2 = f32_to_bf16_bits(v2);
                kf[i][j] = bf16_bits_to_f32(kb1);
                kf[i][j + HALF] = bf16_bits_to_f32(kb2);
                vf[i][j] = bf16_bits_to_f32(vb1);
                vf[i][j + HALF] = bf16_bits_to_f32(vb2);
                if (ds == 0) {
                    Kc[(size_t)pos * DH + j] = kb1;
                    Kc[(size_t)pos * DH + j + HALF] = kb2;
                    Vt[((size_t)(pos >> 5) * DH + j) * 32 + (pos & 31)] = vb1;
                    Vt[((size_t)(pos >> 5) * DH + j + HALF) * 32 + (pos & 31)] = vb2;
                }
            } else {
                kf[i][j] = 0.f; kf[i][j + HALF] = 0.f;
                vf[i][j] = 0.f; vf[i][j + HALF] = 0.f;
            }
            qf[i][j] = qa;
            qf[i][j + HALF] = qc;
            if (i < kGroupRows) {                     // column i + 5 t: bf16 term t of q_i
                uint16_t t1[kTerms], t2[kTerms];
                split3(qa, t1);
                split3(qc, t2);
                const int d1 = j, d2 = j + HALF;
#pragma unroll
                for (int t = 0; t < kTerms; ++t) {
                    qb[d1 >> 5][i + kGroupRows * t + 16 * ((d1 & 31) >> 3)][d1 & 7] = t1[t];
                    qb[d2 >> 5][i + kGroupRows * t + 16 * ((d2 & 31) >> 3)][d2 & 7] = t2[t];
                }
            } else if (i == kGroupRows) {             // column 15 (unused): keep it finite
                qb[j >> 5][15 + 16 * ((j & 31) >> 3)][j & 7] = 0;
                qb[(j + HALF) >> 5][15 + 16 * (((j + HALF) & 31) >> 3)][(j + HALF) & 7] = 0;
            }
        }
    }
    __syncthreads();

    float m_run = -INFINITY, l_run = 0.f;         // of query r % 5
    fx4 acc_o[NDT];
#pragma unroll
    for (int i = 0; i < NDT; ++i) acc_o[i] = fx4{0.f, 0.f, 0.f, 0.f};
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
                fx4 acc = {0.f, 0.f, 0.f, 0.f};
                if (unit < u_end) {
#pragma unroll
                    for (int c = 0; c < NC; ++c) acc = mfma_b(kreg[s][ab][c], qreg[c], acc);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float x = acc[v];
                    x = sum_terms_all(x, r);
                    const int key = 32 * unit + 8 * g + 4 * ab + v;
                    x = (unit < u_end && key < P) ? x : -INFINITY;
                    sv[s][ab][v] = x;
                    mx = fmaxf(mx, x);
                }
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
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
                    const float p = expf(sv[s][ab][v] - m_new);
                    lsum += p;
                    uint16_t t3[kTerms];
                    split3(p, t3);
                    hv[4 * ab + v] = r < 5 ? t3[0] : (r < 10 ? t3[1] : (r < 15 ? t3[2] : (uint16_t)0));
                }
            pb[s] = uint4{pk2(hv[0], hv[1]), pk2(hv[2], hv[3]), pk2(hv[4], hv[5]), pk2(hv[6], hv[7])};
        }
        lsum += __shfl_xor(lsum, 16);
        lsum += __shfl_xor(lsum, 32);
        l_run = l_run * rescale + lsum;
        m_run = m_new;
#pragma unroll
        for (int i = 0; i < NDT; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc_o[i][v] *= rescale;
#pragma unroll
        for (int s = 0; s < UPI; ++s)
            if (u0 + s < u_end) {
#pragma unroll
                for (int i = 0; i < NDT; ++i) acc_o[i] = mfma_b(vreg[s][i], pb[s], acc_o[i]);
            }
    }
#pragma unroll
    for (int i = 0; i < NDT; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float x = sum_terms(acc_o[i][v]);
            if (r < kGroupRows) part_o[w][r][16 * i + 4 * g + v] = x;
        }
    if (lane < kGroupRows) { part_m[w][lane] = m_run; part_l[w][lane] = l_run; }

    if (w == kMW - 1) {                                 // the M new keys, float32 from LDS
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
        const float p = (mx == -INFINITY) ? 0.f : expf(s - mx);
        float l = p;
        l += __shfl_xor(l, 1);
        l += __shfl_xor(l, 2);
        l += __shfl_xor(l, 4);
        pn[m][j] = p;
        if (j == 0) { part_m[kMW][m] = mx; part_l[kMW][m] = l; }
    }
    __syncthreads();
    if (w == kMW - 1) {
        const int m = lane >> 3, j = lane & 7;
        for (int dd = j; dd < DW; dd += 8) {
            float o = 0.f;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) o += pn[m][jj] * vf[jj][dim0 + dd];
            part_o[kMW][m][dd] = o;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < M * DW; idx += kMW * 64) {
        const int m = idx / DW, dd = idx % DW;
        float mstar = -INFINITY;
#pragma unroll
        for (int p = 0; p <= kMW; ++p) mstar = fmaxf(mstar, part_m[p][m]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int p = 0; p <= kMW; ++p) {
            const float pm = part_m[p][m];
            const float wg = (pm == -INFINITY) ? 0.f : expf(pm - mstar);
            den += wg * part_l[p][m];
            num += wg * part_o[p][m][dd];
        }
        st_dev(a.att + (size_t)(seq * M + m) * HD + hh * DH + dim0 + dd, num / den);
    }
    __syncthreads();                                    // LDS is reused by the next item / stage
}

// ---- the kernel ---------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(kMW * 64) void decoder_megakernel(MegaArgs a) {
    constexpr int DS = (DH == 128) ? 4 : 2;             // workgroups per head (slices of the head dimension)
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b = blockIdx.x;
    const unsigned G = gridDim.x;

    __shared__ float red[2][kMW][16][8];
    __shared__ uint2 conv_all[kMW][256];                // 2 KiB per wave (two 1 KiB slots)
    __shared__ float inv_s[8];
    __shared__ __attribute__((aligned(16))) char attn_lds[24 * DH * 4 + (DH / 32) * 1024 + 256 + (kMW + 1) * 64 + (kMW + 1) * 8 * (DH / DS) * 4];
    uint2 *conv = conv_all[w];

    const int d = a.d, HD = a.H * DH, F = a.F;
    const int T_qkv = 3 * HD / 16, T_d = d / 16, T_gu = 2 * F / 16, T_lm = a.V / 16;
    const int KS_d = d / 32, KS_hd = HD / 32, KS_f = (F + 31) / 32;
    auto Wm = [&](size_t off0, int l) { return reinterpret_cast<const uint4 *>(a.packed + off0 + (size_t)l * a.layer_stride); };
    auto Gn = [&](size_t off0, int l) { return reinterpret_cast<const float *>(a.packed + off0 + (size_t)l * a.layer_stride); };

    uint4 ring[kRing];
    if (b < T_qkv) prime_ring(ring, Wm(a.off_wqkv0, 0), KS_d, b, w, lane);

    unsigned bar_no = 0;
    // optional tracing: every workgroup records, per barrier, when it arrived and when it left
    // (100 MHz wall clock)
    const unsigned n_stamps = 2 * (2 + kMegaBarriersPerLayer * a.n_layers);
    auto stamp = [&](int slot) {
        if (a.stage_clock && threadIdx.x == 0) a.stage_clock[(size_t)b * n_stamps + 2 * bar_no + slot] = wall_clock64();
    };
    auto barrier = [&]() {
        stamp(0);
        ++bar_no;
        grid_barrier(a.bar, a.bar_base + bar_no * G, a.abort_flag);
        stamp(1);
    };
    stamp(1);

    // ---- input rows: h, gain-scaled copy, sum of squares (one part) --------------------------
    for (int row = b; row < a.rows; row += G) {
        const uint16_t *src_tok = nullptr;
        if (a.tokens) src_tok = reinterpret_cast<const uint16_t *>(a.packed + a.off_embed) + (size_t)min(max(a.tokens[row], 0), a.V - 1) * d;
        const float *gain = Gn(a.off_attn_norm0, 0);
        float ss = 0.f;
        for (int k = threadIdx.x; k < d; k += kMW * 64) {
            float x = src_tok ? bf16_bits_to_f32(src_tok[k]) : a.embeds[(size_t)row * d + k];
            st_dev(a.h + (size_t)row * d + k, x);
            st_dev(a.hg + (size_t)row * d + k, x * gain[k]);
            ss += x * x;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
        float *tmp = &red[0][0][0][0];
        if (lane == 0) tmp[w] = ss;
        __syncthreads();
        if (threadIdx.x == 0) {
            float tot = 0.f;
            for (int i = 0; i < kMW; ++i) tot += tmp[i];
            st_dev(a.ssq_b + row, tot);
        }
        __syncthreads();
    }
    barrier();

    MegaAttn at;
    at.qkv = a.qkv; at.rope = a.rope; at.att = a.att; at.M = a.M; at.H = a.H;
    at.max_positions = a.max_positions; at.v_stride = a.v_stride;

    // stages of the forward: per layer QKV, attention, O, gate|up, down; then the LM head
    const int n_stages = 5 * a.n_layers + (a.logits ? 1 : 0);
    for (int sidx = 0; sidx < n_stages; ++sidx) {
        const int l = sidx / 5, kind = (l < a.n_layers) ? sidx % 5 : 5;
        const bool last_layer = l + 1 == a.n_layers;
        if (kind == 1) {
            // attention (the O projection's first weight blocks are already in flight in the ring)
            char *kv_l = a.kv + (size_t)l * a.kv_layer_stride;
            at.k_cache = reinterpret_cast<uint16_t *>(kv_l) + (size_t)a.seq0 * a.H * a.max_positions * DH;
            at.v_cache = reinterpret_cast<uint16_t *>(kv_l + a.kv_v_offset) + (size_t)a.seq0 * a.H * DH * a.v_stride;
            const int items = a.n_seqs * a.H * DS;
            for (int it = b; it < items; it += G) {
                const int ds = it / (a.n_seqs * a.H), pr = it % (a.n_seqs * a.H);
                attention_item<DH, DS>(at, ds, pr % a.H, pr / a.H, a.lens.len[pr / a.H], attn_lds, lane, w);
            }
            barrier();
            continue;
        }
        GemmStage st{};
        st.rows = a.rows;
        if (kind == 0) {            // QKV projection (RMSNorm folded in)
            st.W = Wm(a.off_wqkv0, l); st.KS = KS_d; st.n_tiles = T_qkv; st.X = a.hg; st.ldx = d;
            st.epi = EPI_STORE; st.Y = a.qkv; st.ldy = 3 * HD; st.y_dev = true;
            st.ssq_in = a.ssq_b; st.ssq_parts = (l == 0) ? 1 : T_d; st.inv_d = 1.0f / d; st.eps = a.eps;
            st.succ_W = Wm(a.off_wo0, l); st.succ_KS = KS_hd; st.succ_tiles = T_d;
        } else if (kind == 2) {     // O projection + residual
            st.W = Wm(a.off_wo0, l); st.KS = KS_hd; st.n_tiles = T_d; st.X = a.att; st.ldx = HD;
            st.epi = EPI_RESIDUAL; st.Y = a.h; st.ldy = d; st.Yg = a.hg; st.gain_next = Gn(a.off_mlp_norm0, l); st.ssq_out = a.ssq_a;
            st.succ_W = Wm(a.off_wgu0, l); st.succ_KS = KS_d; st.succ_tiles = T_gu;
        } else if (kind == 3) {     // gate | up projection + SwiGLU
            st.W = Wm(a.off_wgu0, l); st.KS = KS_d; st.n_tiles = T_gu; st.X = a.hg; st.ldx = d;
            st.epi = EPI_SWIGLU; st.Xf = a.xf; st.ldf = KS_f * 32;
            st.ssq_in = a.ssq_a; st.ssq_parts = T_d; st.inv_d = 1.0f / d; st.eps = a.eps;
            st.succ_W = Wm(a.off_wdown0, l); st.succ_KS = KS_f; st.succ_tiles = T_d;
        } else if (kind == 4) {     // down projection + residual
            st.W = Wm(a.off_wdown0, l); st.KS = KS_f; st.n_tiles = T_d; st.X = a.xf; st.ldx = KS_f * 32;
            st.epi = EPI_RESIDUAL; st.Y = a.h; st.ldy = d; st.Yg = a.hg; st.ssq_out = a.ssq_b;
            st.gain_next = last_layer ? reinterpret_cast<const float *>(a.packed + a.off_final_norm) : Gn(a.off_attn_norm0, l + 1);
            if (!last_layer) { st.succ_W = Wm(a.off_wqkv0, l + 1); st.succ_KS = KS_d; st.succ_tiles = T_qkv; }
            else if (a.logits) { st.succ_W = reinterpret_cast<const uint4 *>(a.packed + a.off_lm_head); st.succ_KS = KS_d; st.succ_tiles = T_lm; }
        } else {                    // LM head (final RMSNorm folded in)
            st.W = reinterpret_cast<const uint4 *>(a.packed + a.off_lm_head); st.KS = KS_d; st.n_tiles = T_lm; st.X = a.hg; st.ldx = d;
            st.epi = EPI_STORE; st.Y = a.logits; st.ldy = a.V; st.y_dev = false;
            st.ssq_in = a.ssq_b; st.ssq_parts = T_d; st.inv_d = 1.0f / d; st.eps = a.eps;
        }
        if (st.KS <= kMW * kRing) gemm_stage<true>(st, ring, red, inv_s, conv, lane, w);
        else gemm_stage<false>(st, ring, red, inv_s, conv, lane, w);
        if (kind != 5) barrier();
    }
    stamp(0);
    wait_all_loads();
}

hipError_t launch_megakernel(const MegaArgs &a, int grid, hipStream_t stream) {
    MegaArgs args = a;
    void *params[] = {&args};
    if (a.dh == 128)
        return hipLaunchCooperativeKernel(reinterpret_cast<void *>(decoder_megakernel<128>), dim3(grid), dim3(kMW * 64), params, 0, stream);
    if (a.dh == 64)
        return hipLaunchCooperativeKernel(reinterpret_cast<void *>(decoder_megakernel<64>), dim3(grid), dim3(kMW * 64), params, 0, stream);
    return hipErrorInvalidValue;
}

int megakernel_max_grid(int dh) {
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    hipError_t e = (dh == 128)
        ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decoder_megakernel<128>, kMW * 64, 0)
        : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decoder_megakernel<64>, kMW * 64, 0);
    if (e != hipSuccess || per_cu < 1) return 0;
    return cus < kMegaMaxGrid ? cus : kMegaMaxGrid;     // one workgroup per CU
}

}  // namespace spd
