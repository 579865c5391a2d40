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
//
// The arrival counters only grow, and what a workgroup waits for is derived on the device from
// its own arrival: launches on one model are stream-ordered and each adds exactly S = dh / 16 to
// every head's counter, so a counter is a multiple of S when a launch starts, the value the
// arriving workgroup's atomic add returns is S * epoch + (arrivals before it), and the head is
// complete at S * (epoch + 1).  Nothing about the count comes from the host, so a launch that
// is replayed from a captured graph, or follows a capture that ran nothing, waits correctly.
#include "attention_core.h"
#include "gemm_core.h"

namespace spd {

constexpr int kQaGemmWaves = 8, kQaNB = 16, kQaRing = 8;

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
        for (int u = 0; u < U; ++u) av[u] = load_stream(W + ((size_t)tile0 * KS + s0 + u) * 64 + lane);
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
    if (a.ssq_in && w < GW)
        inv_row = rms_inv_from_parts(a.ssq_in + (size_t)erow * (KS * 2), a.ssq_in_parts, en, row_ok, 1.0f / (float)a.K, a.eps);

#pragma unroll
    for (int j = 0; j < 3; ++j) {
        const int t = tile0 + j * tstride;
        if (w < GW) {
            f32x4_t acc[NG];
            const uint4 *wcur = W + ((size_t)t * KS + s0) * 64 + lane;
            const uint4 *wnext = ((j < 2) ? W + ((size_t)(t + tstride) * KS + s0) * 64 : X) + lane;   // last tile: harmless re-read
            regb_tile<NB, U, NG>(acc, av, bv, wcur, wnext, j < 2);
            store_partial<NG>(acc, red[j & 1][w], lane);
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
    // thread 0's ticket: counter value before this workgroup's arrival
    unsigned ticket = 0;
    if (threadIdx.x == 0) ticket = __hip_atomic_fetch_add(a.head_count + hh, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    // ---- attention of (head, slice) ------------------------------------------------------------
    auto wait_head = [&] {
        if (threadIdx.x == 0) {
            const unsigned target = (ticket / (unsigned)S + 1u) * (unsigned)S;     // this launch completes the head here
            // the last of the head's S workgroups to arrive need not look at the counter at all
            if (ticket + 1u != target && __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
                unsigned spins = 0;
                while ((int)(__hip_atomic_load(a.head_count + hh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
                    __builtin_amdgcn_s_sleep(1);
                    if (++spins > a.spin_limit) {               // never in a healthy run: let everything drain
                        __hip_atomic_store(a.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
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
