// QKV projection + RoPE + KV append + attention in one launch (see QkvAttnArgs in launch.h).
//
// Grid: H * (dh / 16) workgroups of 12 waves, head index fastest (the slices of a head share an
// XCD).  Waves 0..7 stream the workgroup's three weight tiles exactly like the stand-alone
// register-resident projection kernel (K split 8 ways, activation slice in registers, ring of
// 8 blocks); waves 8..11 only take part in the barriers.  The q/k/v slices are written with
// device-scope (write-through) stores, acknowledged, and counted on the head's arrival
// counter.  All 12 waves then run the attention of (head, slice): its cached-key loads go out
// first, then the counter is awaited (bounded spin), then the head's new rows are read with
// device-scope loads.  Every workgroup is resident at once (the grid is at most one workgroup
// per CU and the kernel's resources allow one per CU), so every awaited arrival does happen.
#include "attention_core.h"

namespace spd {

constexpr int kQaGemmWaves = 8, kQaNB = 16, kQaRing = 8;

__device__ __forceinline__ f32x4_t qa_mfma(const uint4 &a, const uint4 &b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
__device__ __forceinline__ uint4 qa_load_stream(const uint4 *p) {
    typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
    u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return uint4{v.x, v.y, v.z, v.w};
}

// NG = 1: up to 5 rows; 12 waves, 8 of which stream the projection.  NG = 2: 6..10 rows of one sequence
// (its attention then handles up to 8 of them as two query groups); 8 waves, all in both parts -- the
// second activation slice needs the registers that a wider workgroup would not leave.
template <int DH, int NG>
__global__ __launch_bounds__((NG == 1 ? kAttnWaves : kQaGemmWaves) * 64) void qkv_attention_kernel(QkvAttnArgs a) {
    constexpr int S = DH / 16, GW = kQaGemmWaves, NB = kQaNB, U = kQaRing, KS = GW * NB;
    constexpr int TW = NG == 1 ? kAttnWaves : kQaGemmWaves;      // waves of the workgroup
    const int H = a.at.H, HD = H * DH;
    const int hh = blockIdx.x % H, ds = blockIdx.x / H;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint4 *W = reinterpret_cast<const uint4 *>(a.W);
    const uint4 *X = reinterpret_cast<const uint4 *>(a.X);
    float *Y = const_cast<float *>(a.at.qkv);
    const int ldy = 3 * HD;

    __shared__ float red[2][GW][NG][16][8];

    // ---- projection: tiles q, k, v of (head, slice) ---------------------------------------
    const int tile0 = hh * S + ds, tstride = HD / 16;
    const int s0 = w * NB;
    uint4 av[U], bv[NG][NB];
    if (w < GW) {
#pragma unroll
        for (int u = 0; u < U; ++u) av[u] = qa_load_stream(W + ((size_t)tile0 * KS + s0 + u) * 64 + lane);
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int i = 0; i < NB; ++i) bv[g][i] = X[((size_t)g * KS + s0 + i) * 64 + lane];
    }
    // epilogue element of this thread: waves 2 NG j' .. 2 NG j' + 2 NG - 1 finish a tile, a pair per row group
    const int en = lane & 15, em = (w & 1) * 4 + (lane >> 4);
    const int eg = (w >> 1) % NG;                                      // row group of this wave's pair
    const int erow = eg * kGroupRows + em;
    const bool row_ok = em < kGroupRows && erow < a.rows;
    float inv_row = 1.0f;
    if (a.ssq_in && w < GW) {
        float sum = 0.f;
        if (row_ok) {
            const float *part = a.ssq_in + (size_t)erow * (KS * 2);
            if ((a.ssq_in_parts & 3) == 0) {
#pragma unroll 4
                for (int p = en; p < (a.ssq_in_parts >> 2); p += 16) {
                    const float4 q = reinterpret_cast<const float4 *>(part)[p];
                    sum += (q.x + q.y) + (q.z + q.w);
                }
            } else {
                for (int p = en; p < a.ssq_in_parts; p += 16) sum += part[p];
            }
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        inv_row = 1.0f / sqrtf(sum * (1.0f / (float)a.K) + a.eps);
    }

#pragma unroll
    for (int j = 0; j < 3; ++j) {
        const int t = tile0 + j * tstride;
        if (w < GW) {
            f32x4_t acc[NG];
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[g] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            const uint4 *wnext = (j < 2) ? W + ((size_t)(t + tstride) * KS + s0) * 64 : X;   // last tile: harmless re-read
#pragma unroll
            for (int i = 0; i < NB; ++i) {
#pragma unroll
                for (int g = 0; g < NG; ++g) acc[g] = qa_mfma(av[i % U], bv[g][i], acc[g]);
                if (i + U < NB) av[i % U] = qa_load_stream(W + ((size_t)t * KS + s0 + i + U) * 64 + lane);
                else av[i % U] = qa_load_stream(wnext + (size_t)(j < 2 ? (i + U - NB) : 0) * 64 + lane);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float x = sum_terms(acc[g][v]);
                    if ((lane & 15) < kGroupRows) red[j & 1][w][g][4 * (lane >> 4) + v][lane & 15] = x;
                }
        }
        __syncthreads();
        if (w < GW && (w / (2 * NG)) == (j % (GW / (2 * NG))) && row_ok) {   // 2 NG waves finish tile j
            float sum = 0.f;
#pragma unroll
            for (int ww = 0; ww < GW; ++ww) sum += red[j & 1][ww][eg][en][em];
            __hip_atomic_store(Y + (size_t)erow * ldy + (size_t)t * 16 + en, sum * inv_row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // the slices are written through to memory; once acknowledged, count this workgroup in
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_fetch_add(a.head_count + hh, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    // ---- attention of (head, slice) ------------------------------------------------------------
    const unsigned target = a.count_before + (unsigned)S;
    auto wait_head = [&] {
        if (threadIdx.x == 0 && __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
            unsigned spins = 0;
            while ((int)(__hip_atomic_load(a.head_count + hh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
                __builtin_amdgcn_s_sleep(1);
                if (++spins > (1u << 22)) {                 // never in a healthy run: let everything drain
                    __hip_atomic_store(a.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
            }
        }
        __syncthreads();
    };
    attention_core<DH, S, TW, kUnitsPerIter, true, NG>(a.at, hh, ds, 0, wait_head);
}

bool qkv_attention_supported(int K, int H, int dh, int rows, int n_seqs, int M) {
    if (K != 32 * kQaGemmWaves * kQaNB || dh != 128 || rows > 8 || n_seqs != 1 || M != rows) return false;
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return false;
    hipError_t e = rows <= kGroupRows
        ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, qkv_attention_kernel<128, 1>, kAttnWaves * 64, 0)
        : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, qkv_attention_kernel<128, 2>, kQaGemmWaves * 64, 0);
    return e == hipSuccess && per_cu >= 1 && H * (dh / 16) <= cus * per_cu;   // all workgroups resident at once
}

hipError_t launch_qkv_attention(const QkvAttnArgs &a, hipStream_t stream) {
    const AttnArgs &t = a.at;
    if (a.K != 32 * kQaGemmWaves * kQaNB || t.dh != 128 || a.rows < 1 || a.rows > 8 || t.n_seqs != 1 || t.M != a.rows ||
        t.m0 != 0 || t.Mq != t.M || (t.v_stride % 32) != 0 || t.v_stride < t.max_positions || t.M > t.max_positions)
        return hipErrorInvalidValue;
    if (a.rows <= kGroupRows) launch_kernel(qkv_attention_kernel<128, 1>, dim3(t.H * (t.dh / 16)), dim3(kAttnWaves * 64), stream, a);
    else launch_kernel(qkv_attention_kernel<128, 2>, dim3(t.H * (t.dh / 16)), dim3(kQaGemmWaves * 64), stream, a);
    return hipGetLastError();
}

}  // namespace spd
