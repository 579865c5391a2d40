// Host-side launch wrappers of the HIP kernels (internal to libspd).
// Every wrapper only enqueues work on `stream` and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.h"

#include <hip/hip_ext.h>

namespace spd {

// ---- per-kernel timing (tracing) ---------------------------------------------------
// While *launch_timing() points at a pair of events, the single-kernel launch wrappers below hand
// them to the launch itself, so that they time the kernel alone (start of execution to completion,
// what a profiler reports) instead of the interval between two events recorded around the launch.
struct LaunchTiming { hipEvent_t start, stop; bool used; };
LaunchTiming *&launch_timing();                    // thread-local; NULL: plain launches

template <class Kernel, class... Args>
inline void launch_kernel(Kernel kernel, dim3 grid, dim3 block, hipStream_t stream, Args... args) {
    LaunchTiming *t = launch_timing();
    if (t && !t->used) {
        hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, t->start, t->stop, 0, args...);
        t->used = true;
    } else {
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, args...);
    }
}

// ---- weight re-tiling (model creation) ------------------------------------------
enum PackMode { PACK_PLAIN = 0, PACK_CONCAT3 = 1, PACK_GATE_UP = 2 };
// dst: packed blocks of a [N, K] matrix assembled from up to three row-major sources:
//   PLAIN     rows of src0
//   CONCAT3   rows of src0, then src1, then src2 (N/3 rows each)         -- fused QKV
//   GATE_UP   tile j = 8 rows of src0 (gate) then the same 8 rows of src1 (up)
hipError_t launch_pack_weight(const void *src0, const void *src1, const void *src2, int mode,
                              int N, int K, void *dst, hipStream_t stream);
size_t packed_matrix_bytes(int N, int K);

// ---- skinny weight-streaming GEMM -------------------------------------------------
enum Epilogue { EPI_STORE = 0, EPI_RESIDUAL = 1, EPI_SWIGLU = 2 };
constexpr int kBatchMaxTileGroups = 1024;    // arrival counters of the batched projection kernel (one per tile group)
struct GemmTuning { int waves; int grid_cap; int ring; int no_regb; int no_batch; int force_batch; };   // 0 = default for grid_cap / ring
struct GemmArgs {
    const void *W;        // packed weights [N, K]
    const void *X;        // packed activations (B operand blocks), K columns
    int N, K;             // logical sizes (N % 16 == 0)
    int rows;             // valid activation rows (<= 64)
    float *Y;             // STORE: Y[row, n] = s * acc ; RESIDUAL: Y[row, n] += acc   (ld = ldy)
    int ldy;
    // RMSNorm folded into the GEMM: X holds (h * gain) un-normalised; the row scale
    // s = 1 / sqrt(sum_sq / K + eps) is applied to the accumulator.  ssq_in[64][K / 16] holds
    // ssq_in_parts partial sums of squares per row (NULL: s = 1).
    const float *ssq_in;
    int ssq_in_parts;
    float eps;
    // RESIDUAL only: also emit what the next norm + GEMM needs from the new h (N % 32 == 0):
    const float *gain_next;   // gain of the following RMSNorm, or NULL
    void *Xnext;              // packed (h_new * gain_next), K = N
    float *ssq_out;           // [64][N / 16] per-tile sums of squares of h_new
    void *Xout;           // SWIGLU: packed activations with K_out = N / 2 columns
    int K_out;
    // more than 10 rows: scratch for the partial tiles of the K slices (gemm_batch_scratch_bytes) and the tile
    // groups' arrival counters (1024 entries, zero between launches); NULL: the kernels that need neither
    float *batch_partials;
    unsigned *batch_arrive;
    const void *batch_zero;   // 1 KiB of zeros that nobody writes
};
size_t gemm_batch_scratch_bytes(int N, int K);
hipError_t launch_gemm(const GemmArgs &a, int epilogue, GemmTuning tune, hipStream_t stream);

// ---- row-wise kernels -------------------------------------------------------------
// Input rows of a forward: h[row, :] = float(E[tokens[row], :]) (token ids clamped into
// [0, vocab)) or h[row, :] = embeds[row, :]; also writes the packed (h * gain) operand of
// the first QKV projection and the sum of squares of every row (ssq[row * (d / 16)], one part).
// tokens: ids of sequence s at tokens[s * token_stride + i], i < M (rows = n_seqs * M).
hipError_t launch_input_rows(const void *embed_bf16, const int32_t *tokens, int M, int token_stride,
                             const float *embeds, int rows, int d, int vocab, const float *gain, float *h,
                             void *xpack, float *ssq, hipStream_t stream);
// lens[i] += delta for i < n (KV lengths that live on the device)
hipError_t launch_lens_add(int32_t *lens, int n, int delta, hipStream_t stream);
// end of a speculative-decoding block, entirely on the device
struct CommitArgs {
    const int32_t *n_accepted, *next_token;   // [n_seqs] k and y of the accept step
    int32_t *verify_tokens;                   // [n_seqs][gamma + 1] in: t, d_1 .. d_gamma; out: slot 0 = y
    int32_t *draft_in;                        // [n_seqs][2] out: the draft's next inputs (token before y, y)
    int32_t *target_lens, *draft_lens;        // [n_seqs] device KV lengths, both reduced by gamma - k
    int32_t *out_tokens;                      // [n_seqs][out_capacity] emitted tokens, or NULL
    int32_t *n_out;                           // [n_seqs] tokens emitted so far
    int n_seqs, gamma, out_capacity;
};
hipError_t launch_block_commit(const CommitArgs &a, hipStream_t stream);
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t stream);
// K and V of positions pos0 .. pos0 + n - 1 of one (layer, sequence) as float32 [n][H][dh] (k_cache / v_cache: that pair's slices)
hipError_t launch_kv_export(const void *k_cache, const void *v_cache, int H, int dh, int max_positions, int pos0, int n,
                            float *k_out, float *v_out, hipStream_t stream);

// ---- attention ----------------------------------------------------------------------
struct AttnArgs {
    const float *qkv;        // [rows, 3 * H * dh] (q | k | v), before RoPE
    const float *rope;       // [max_positions, dh / 2, 2] (cos, sin)
    void *k_cache;           // this layer: bf16 [max_seqs, H, max_positions, dh]   (K after RoPE)
    void *v_cache;           // this layer: bf16 [max_seqs, H, v_stride / 32, dh, 32]: V transposed in blocks of 32
                             // positions, so that the dh x 32 tile one unit of 32 keys needs is 64 * dh contiguous bytes
    void *xout;              // packed activations, K = H * dh (attention output)
    int n_seqs, M, H, dh, max_positions, v_stride;
    int slices;              // stand-alone kernel: workgroups per head (1, 2, 4, 8 for head_dim 128), 0 = chosen by batch size
    int m0, Mq;              // this launch handles rows m0 .. m0 + Mq - 1 of every sequence (Mq <= 8); rows
                             // 0 .. m0 - 1 were appended to the cache by an earlier launch
    const int32_t *d_lens;   // KV lengths in device memory [n_seqs], or NULL: then `lens` below holds them
    int32_t *d_error;        // set to 1 if a device length does not leave room for M rows (the launch then
                             // works on a clamped length: wrong results, but every access stays in bounds)
    SeqLens lens;            // KV length of every sequence before this call
};
hipError_t launch_attention(const AttnArgs &a, hipStream_t stream);

// ---- QKV projection and attention in one kernel (one row group, one sequence, K = 4096, head_dim 128) ----
// One workgroup per (head, 16 output dimensions) computes the three 16-row tiles of the fused
// QKV matrix that hold its slice of q, k and v, announces them on the head's arrival counter,
// and -- once all slices of the head have arrived -- runs attention for its slice.  The
// dependency between the two stages is per head, so no device-wide barrier is needed; the
// loads of the cached keys and values are in flight while the counter is awaited.
struct QkvAttnArgs {
    const void *W;            // packed [3 * H * dh, K]
    const void *X;            // packed activations, one row group
    int K, rows;
    const float *ssq_in;      // as in GemmArgs
    int ssq_in_parts;
    float eps;
    AttnArgs at;              // at.qkv: float32 [rows][3 * H * dh] scratch filled by the projection part
    unsigned *head_count;     // [H] arrival counters (only grow); every launch adds dh / 16 to each
    unsigned spin_limit;      // polls of a counter before the wait gives up and raises abort_flag
    int *abort_flag;          // raised (and never cleared) if a wait hit its spin limit
};
bool qkv_attention_supported(int K, int H, int dh, int rows, int n_seqs, int M);
hipError_t launch_qkv_attention(const QkvAttnArgs &a, hipStream_t stream);

// ---- sampling ---------------------------------------------------------------------
struct AcceptArgs {
    const float *target, *draft;
    const int32_t *draft_tokens;
    const float *u;
    int n_seqs, gamma, vocab;
    float temperature;
    uint32_t flags;
    int32_t *n_accepted, *next_token;
    int token_stride;        // draft token j of sequence s at draft_tokens[s * token_stride + j]
    float *accept_prob;      // may be NULL
    float *stats;            // workspace: [n_seqs * (2 gamma + 1), 4]
};
hipError_t launch_accept(const AcceptArgs &a, hipStream_t stream);
size_t accept_workspace_bytes(int n_seqs, int gamma);

// softmax(logits[seq * ld_rows + ...]) -> probs row + one sample per sequence
// sequence s: logits + s * row_stride, u[s * u_stride], probs_out + s * probs_stride, token_out[s * token_stride]
hipError_t launch_softmax_sample(const float *logits, size_t row_stride, int n_seqs, int vocab,
                                 float temperature, const float *u, int u_stride, float *probs_out,
                                 size_t probs_stride, int32_t *token_out, int token_stride, hipStream_t stream);

}  // namespace spd
