// Building blocks shared by every kernel that streams packed weights through the matrix cores:
// the matrix-core step, the streaming load, the RMSNorm scale from the producer's partial
// sums, and the tile body of the register-resident projection (used by the stand-alone
// projection kernel and by the first stage of the fused QKV + attention kernel).
#pragma once
#include "common.h"

namespace spd {

__device__ __forceinline__ f32x4_t mfma_bf16(const uint4 &a, const uint4 &b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

__device__ __forceinline__ uint4 load_stream(const uint4 *p) {
    // weights are read exactly once per step: non-temporal loads (measured: +15% on a pure read stream)
    typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
    u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return uint4{v.x, v.y, v.z, v.w};
}

// 1 / rms of one input row from the producer's partial sums of squares (`parts` of them, contiguous),
// computed by the 16 lanes that share `en16 = lane % 16`'s row: every lane of the 16 gets the result.
// Fixed summation order.  `active` = false lanes contribute nothing (and still take part in the shuffles).
__device__ __forceinline__ float rms_inv_from_parts(const float *part, int parts, int en16, bool active, float inv_d, float eps) {
    float sum = 0.f;
    if (active) {
        if ((parts & 3) == 0) {                           // 16 lanes read float4, all loads in flight at once
#pragma unroll 4
            for (int p = en16; p < (parts >> 2); p += 16) {
                const float4 q = reinterpret_cast<const float4 *>(part)[p];
                sum += (q.x + q.y) + (q.z + q.w);
            }
        } else {
            for (int p = en16; p < parts; p += 16) sum += part[p];
        }
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    return 1.0f / sqrtf(sum * inv_d + eps);
}

// One tile of the register-resident projection for one wave: NB matrix-core steps over the wave's
// K slice (activation blocks bv resident), each followed by the refill of its ring slot with the
// block U steps ahead -- of the same tile (`wcur` = block (tile, s0) + lane) or, past its end, of the
// next tile (`wnext` = block (next tile, s0) + lane; with has_next = false any readable address:
// the refill is then a harmless re-read of its first block).  Straight-line code: no branch between
// a step and its refill, so the compiler waits for exactly the oldest block.
template <int NB, int U, int NG>
__device__ __forceinline__ void regb_tile(f32x4_t (&acc)[NG], uint4 (&av)[U], const uint4 (&bv)[NG][NB],
                                          const uint4 *wcur, const uint4 *wnext, bool has_next) {
    static_assert(NB % U == 0, "ring must divide the per-wave K range");
#pragma unroll
    for (int g = 0; g < NG; ++g) acc[g] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < NB; ++i) {
#pragma unroll
        for (int g = 0; g < NG; ++g) acc[g] = mfma_bf16(av[i % U], bv[g][i], acc[g]);
        if (i + U < NB) av[i % U] = load_stream(wcur + (size_t)(i + U) * 64);
        else av[i % U] = load_stream(wnext + (size_t)(has_next ? (i + U - NB) : 0) * 64);
        __builtin_amdgcn_sched_barrier(0);                // keep "consume slot, refill slot" in program order
    }
}

// The wave's partial tile into the cross-wave reduction buffer: D[n = 4 (lane / 16) + v][c = lane % 16];
// columns c, c + 5, c + 10 are the three bf16 terms of activation row c.
template <int NG>
__device__ __forceinline__ void store_partial(const f32x4_t (&acc)[NG], float (*red)[16][8], int lane) {
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float x = sum_terms(acc[g][v]);
            if ((lane & 15) < kGroupRows) red[g][4 * (lane >> 4) + v][lane & 15] = x;
        }
}

}  // namespace spd
