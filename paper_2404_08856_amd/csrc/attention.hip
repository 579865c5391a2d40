// Stand-alone attention kernel: RoPE + KV-cache append + causal attention (see attention_core.h).
#include "attention_core.h"

namespace spd {

template <int DH, int DS, int AW, int QG>
__global__ __launch_bounds__(AW * 64) void attention_kernel(AttnArgs a) {
    // head index fastest: consecutive workgroups go to consecutive XCDs, so with a head count that is
    // a multiple of 8 all slices of one head share an XCD and its L2 holds that head's K once
    attention_core<DH, DS, AW, kUnitsPerIter, false, QG>(a, blockIdx.x, blockIdx.y, blockIdx.z, [] {});
}

hipError_t launch_attention(const AttnArgs &a, hipStream_t stream) {
    if (a.M < 1 || a.M > kMaxRows || (a.v_stride % 32) != 0 || a.v_stride < a.max_positions) return hipErrorInvalidValue;
    if (a.Mq < 1 || a.Mq > 8 || a.m0 < 0 || a.m0 + a.Mq > a.M || a.M > a.max_positions) return hipErrorInvalidValue;
    // Workgroups per head (slices of the head dimension).  One sequence: 16 output dimensions per
    // workgroup is fastest at the 7B shape (15.4 us per layer against 16.2 with 32 and 18.8 with 64).
    // More (sequence, head) pairs: every slice re-reads K, so slices beyond one workgroup per CU only
    // cost (8 sequences, context 2048: 73 us per layer unsliced, 76 with 2, 108 with 4, 160 with 8 slices;
    // context 640, 5 queries, 32 heads: 3 sequences 17.8 us with 2 slices against 24.2 with 4, 5 sequences
    // 22.3 unsliced against 28.9 with 2): the largest count that keeps pairs * slices within the 256 CUs.
    // a.slices (a tuning knob for tests and sweeps) overrides; 64-wide heads have at most 4 slices.
    int slices = a.slices;
    const int pairs = a.n_seqs * a.H;
    if (slices != 1 && slices != 2 && slices != 4 && slices != 8) slices = pairs > 128 ? 1 : (pairs > 64 ? 2 : (pairs > 32 ? 4 : 8));
    if (slices == 1 && a.Mq > kGroupRows) slices = 2;   // two query groups and a whole head do not fit the registers
    // up to 5 queries per sequence: one query group; 6..8: two groups share the cached keys' registers
#define SPD_ATTN(DH_, DS_, AW_)                                                                                              \
    do {                                                                                                                     \
        if (a.Mq <= kGroupRows)                                                                                              \
            hipLaunchKernelGGL((attention_kernel<DH_, DS_, AW_, 1>), dim3(a.H, DS_, a.n_seqs), dim3(AW_ * 64), 0, stream, a); \
        else                                                                                                                 \
            hipLaunchKernelGGL((attention_kernel<DH_, DS_, 8, 2>), dim3(a.H, DS_, a.n_seqs), dim3(8 * 64), 0, stream, a);    \
    } while (0)
    if (a.dh == 128 && slices == 1) {
        SPD_ATTN(128, 1, 8);
    } else if (a.dh == 128 && slices == 2) {
        SPD_ATTN(128, 2, kAttnWaves);
    } else if (a.dh == 128 && slices == 4) {
        SPD_ATTN(128, 4, kAttnWaves);
    } else if (a.dh == 128) {
        SPD_ATTN(128, 8, kAttnWaves);
    } else if (a.dh == 64 && slices >= 4) {
        SPD_ATTN(64, 4, kAttnWaves);
    } else if (a.dh == 64 && slices == 2) {
        SPD_ATTN(64, 2, kAttnWaves);
    } else if (a.dh == 64) {
        SPD_ATTN(64, 1, kAttnWaves);
    } else {
        return hipErrorInvalidValue;
    }
#undef SPD_ATTN
    return hipGetLastError();
}

}  // namespace spd
