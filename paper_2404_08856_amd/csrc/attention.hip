// Stand-alone attention kernel: RoPE + KV-cache append + causal attention (see attention_core.h).
#include <cstdlib>

#include "attention_core.h"

namespace spd {

template <int DH, int DS>
__global__ __launch_bounds__(kAttnWaves * 64) void attention_kernel(AttnArgs a) {
    // head index fastest: consecutive workgroups go to consecutive XCDs, so with a head count that is
    // a multiple of 8 all slices of one head share an XCD and its L2 holds that head's K once
    attention_core<DH, DS, kAttnWaves, kUnitsPerIter, false>(a, blockIdx.x, blockIdx.y, blockIdx.z, [] {});
}

hipError_t launch_attention(const AttnArgs &a, hipStream_t stream) {
    if (a.M < 1 || a.M > 8 || (a.v_stride % 32) != 0 || a.v_stride < a.max_positions) return hipErrorInvalidValue;
    if (a.Mq < 1 || a.Mq > kGroupRows || a.m0 < 0 || a.m0 + a.Mq > a.M || a.M > a.max_positions) return hipErrorInvalidValue;
    // Workgroups per head (slices of the head dimension).  One sequence: 16 output dimensions per
    // workgroup is fastest at the 7B shape (15.4 us per layer against 16.2 with 32 and 18.8 with 64).
    // Several sequences: a workgroup is latency-bound whatever its slice, so fewer, wider slices
    // that still fill the chip once (measured at 8 sequences: 83 us per layer with 8 slices).
    // SPD_ATTN_SLICES overrides for head_dim 128.
    static const int forced = [] { const char *e = getenv("SPD_ATTN_SLICES"); return e ? atoi(e) : 0; }();
    int slices = forced;
    if (slices != 2 && slices != 4 && slices != 8) slices = a.n_seqs * a.H >= 256 ? 2 : (a.n_seqs * a.H >= 64 ? 4 : 8);
    if (a.dh == 128 && slices == 2) {
        hipLaunchKernelGGL((attention_kernel<128, 2>), dim3(a.H, 2, a.n_seqs), dim3(kAttnWaves * 64), 0, stream, a);
    } else if (a.dh == 128 && slices == 4) {
        hipLaunchKernelGGL((attention_kernel<128, 4>), dim3(a.H, 4, a.n_seqs), dim3(kAttnWaves * 64), 0, stream, a);
    } else if (a.dh == 128) {
        hipLaunchKernelGGL((attention_kernel<128, 8>), dim3(a.H, 8, a.n_seqs), dim3(kAttnWaves * 64), 0, stream, a);
    } else if (a.dh == 64) {
        hipLaunchKernelGGL((attention_kernel<64, 4>), dim3(a.H, 4, a.n_seqs), dim3(kAttnWaves * 64), 0, stream, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace spd
