/*
 * spd.h -- C ABI of the MI355X (gfx950) speculative-decoding hot path.
 *
 * The library implements the data-parallel part of speculative decoding (SPD)
 * for a LLaVA-style multimodal LLM, after "On Speculative Decoding for
 * Multimodal Large Language Models" (arXiv 2404.08856):
 *
 *   - the target verification step: ONE forward pass of a LLaMA-architecture
 *     decoder over the gamma+1 tokens [t, d_1..d_gamma] against a KV cache that
 *     already holds the image-embedding prefix V_1..V_m and the text prefix
 *     X_1..X_n (Section 2.1; Section 2.2, Eq. 1; Section 3);
 *   - the draft model's autoregressive steps (Section 2.1; text-only draft,
 *     Section 3) -- the same kernels at a smaller shape;
 *   - the accept/reject rule min{1, T/D} and the residual resample from
 *     max(0, T - D) (Section 2.1), plus the bonus token on full acceptance
 *     (implied by the maximum block efficiency gamma+1, Section 4 Metrics).
 *
 * Notation: T(x) = target probability, D(x) = draft probability (the paper
 * writes q and p; other texts swap the letters).
 *
 * Conventions
 *   - Every function returns an int32 status (SPD_OK = 0, negative = error) and
 *     never throws.  spd_last_error() returns a static description of the last
 *     error of the calling thread.
 *   - Pointers are DEVICE pointers unless the name starts with h_ (host).
 *   - All device work is enqueued on the caller's hipStream_t, passed as void*
 *     (NULL = the default stream).  No call synchronises the device, except the few
 *     whose comment says so (spd_kv_lens_to_device / _from_device, spd_device_status,
 *     spd_trace_read).
 *   - The library allocates no device memory: weights (packed), KV cache and
 *     workspace live in caller-owned buffers whose sizes spd_model_bytes()
 *     reports.  The model borrows them until spd_model_destroy().
 *   - Shapes: d_model % 32 == 0, head_dim in {64, 128}, (n_heads*head_dim) % 32
 *     == 0, d_ffn % 8 == 0, vocab % 16 == 0, max_seqs <= 64, rows per call
 *     (n_seqs * M) <= 64, M <= 8.  Violations return SPD_ERR_SHAPE before anything is launched.
 */
#ifndef SPD_H
#define SPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPD_OK               0
#define SPD_ERR_INVALID_ARG (-1)
#define SPD_ERR_SHAPE       (-2)
#define SPD_ERR_CAPACITY    (-3)   /* KV cache / workspace / row limit exceeded */
#define SPD_ERR_HIP         (-4)   /* a HIP runtime call failed; see spd_last_error() */

#define SPD_MAX_ROWS         64    /* rows (n_seqs * M) per forward call          */
#define SPD_MAX_M             8    /* new tokens per sequence per forward call    */

/* flags of spd_speculative_accept */
#define SPD_TARGET_IS_PROBS  1u    /* target rows are probabilities, not logits   */
#define SPD_DRAFT_IS_PROBS   2u    /* draft rows are probabilities, not logits    */

typedef struct spd_model spd_model;

/* Shape of a LLaMA-architecture decoder (Appendix A.1, Table 1) + capacities. */
typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    float   rms_eps;           /* RMSNorm epsilon (inside the square root)        */
    float   rope_theta;        /* RoPE base; pair (i, i+head_dim/2), freq theta^(-2i/head_dim) */
    int32_t tied_embeddings;   /* 1: LM head = embedding table                    */
    int32_t max_seqs;          /* sequences the KV cache holds                    */
    int32_t max_positions;     /* positions per sequence the KV cache holds       */
} spd_model_config;

/* Unpacked weights, device memory, row-major [out_features, in_features],
 * bfloat16 matrices and float32 norm gains.  The per-layer members are HOST
 * arrays of n_layers device pointers.  Only read during spd_model_create (and
 * the work it enqueues): once that work has finished the caller may free them. */
typedef struct {
    const void  *embed;              /* bf16 [vocab, d_model]                      */
    const void  *lm_head;            /* bf16 [vocab, d_model]; NULL if tied        */
    const float *final_norm;         /* f32  [d_model]                             */
    const float *const *attn_norm;   /* f32  [d_model] per layer                   */
    const void  *const *wq;          /* bf16 [n_heads*head_dim, d_model]           */
    const void  *const *wk;
    const void  *const *wv;
    const void  *const *wo;          /* bf16 [d_model, n_heads*head_dim]           */
    const float *const *mlp_norm;    /* f32  [d_model]                             */
    const void  *const *w_gate;      /* bf16 [d_ffn, d_model]                      */
    const void  *const *w_up;        /* bf16 [d_ffn, d_model]                      */
    const void  *const *w_down;      /* bf16 [d_model, d_ffn]                      */
} spd_weights;

/* Description of the last error on this thread ("" if none).  Host pointer,
 * valid until the next failing call on the same thread. */
const char *spd_last_error(void);

/* Sizes (bytes) of the three caller-owned device buffers of a model:
 * packed weights (matrices re-tiled for the matrix cores + gains + embedding
 * table), KV cache (bf16, K after RoPE and V, all layers) and workspace. */
int32_t spd_model_bytes(const spd_model_config *h_cfg, size_t *h_packed_bytes,
                        size_t *h_kv_bytes, size_t *h_workspace_bytes);

/* Builds a model (target or draft) over caller-owned buffers: enqueues the
 * re-tiling of every matrix of *h_weights into `packed`, the RoPE table and the
 * clearing of the workspace on `stream`.  All KV lengths start at 0.
 * Errors: SPD_ERR_SHAPE (unsupported shape), SPD_ERR_CAPACITY (a buffer is
 * smaller than spd_model_bytes says), SPD_ERR_INVALID_ARG (NULL/misaligned;
 * buffers must be 256-byte aligned), SPD_ERR_HIP. */
int32_t spd_model_create(const spd_model_config *h_cfg, const spd_weights *h_weights,
                         void *packed, size_t packed_bytes, void *kv_cache, size_t kv_bytes,
                         void *workspace, size_t workspace_bytes, void *stream,
                         spd_model **h_out);

int32_t spd_model_destroy(spd_model *model);

/* Kernel-selection knobs of a model, for tests and sweeps (not part of the method; production
 * code never needs this call: spd_model_create picks the measured defaults).  Zero-initialise the
 * struct for "all defaults".  Takes effect from the next forward; host-side only.
 * Projections are indexed qkv, o, gate_up, down, lm_head. */
#define SPD_N_PROJECTIONS 5
typedef struct {
    int32_t  separate_qkv_attention; /* 1: QKV projection and attention always as two kernels;
                                        0 = default: one kernel where the shape allows */
    int32_t  attention_slices;       /* workgroups per head of the stand-alone attention kernel at head_dim 128:
                                        1, 2, 4 or 8; 0 = chosen by batch size */
    int32_t  gemm_waves[SPD_N_PROJECTIONS];          /* waves per workgroup: 4, 8 or 16; 0 = default */
    int32_t  gemm_grid_cap[SPD_N_PROJECTIONS];       /* upper bound of the grid; 0 = default         */
    int32_t  gemm_general_kernel[SPD_N_PROJECTIONS]; /* 1: never the register-resident variant       */
    int32_t  gemm_ring[SPD_N_PROJECTIONS];           /* general kernel: weight blocks a wave keeps in flight, 8 or 16; 0 = default */
    int32_t  batch_kernel;           /* calls of more than 10 rows: 0 = the library chooses per projection between the
                                        tile-splitting batched kernel (one pass over the weights for up to 64 rows) and
                                        the K-splitting kernels (passes of 40 rows); 1 = always the former, 2 = always
                                        the latter */
    uint32_t wait_spin_limit;        /* polls before a wait between workgroups gives up and raises the flag that
                                        spd_device_status reports (0 = default, 2^22); a tiny value lets a test
                                        drive that error path from the host while every kernel still exits */
} spd_tuning;
int32_t spd_model_set_tuning(spd_model *model, const spd_tuning *h_tuning);

/* Sets the number of valid KV positions of sequences 0..n_seqs-1 (rollback
 * after a rejection, reset to 0, ...).  Host-side bookkeeping only: positions
 * >= the new length are simply overwritten by later calls.
 * Errors: SPD_ERR_CAPACITY if a length exceeds max_positions or n_seqs exceeds
 * max_seqs, SPD_ERR_INVALID_ARG on negative values. */
int32_t spd_kv_set_len(spd_model *model, const int32_t *h_len_per_seq, int32_t n_seqs);
int32_t spd_kv_get_len(const spd_model *model, int32_t *h_len_per_seq, int32_t n_seqs);

/* Inspection (tests, baselines; not part of the method): the cached keys (after RoPE) and values of
 * positions pos0 .. pos0+n-1 of one layer and sequence as float32 [n, n_heads, head_dim] each (the cache
 * itself is bfloat16 in layouts of the library's own).  Positions need not be below the current KV
 * length: whatever the cache holds there is returned.  Errors: SPD_ERR_INVALID_ARG, SPD_ERR_CAPACITY
 * (positions outside max_positions). */
int32_t spd_kv_export(spd_model *model, int32_t layer, int32_t seq, int32_t pos0, int32_t n,
                      float *k_out, float *v_out, void *stream);

/* Not hot: feeds n_rows input-embedding rows (float32 [n_rows, d_model],
 * e.g. [V_1..V_m ; E[X_1..X_n]] for the target, Section 2.2 Eq. 1) to sequence
 * `seq` starting at its current KV length, appending their K, V.  If
 * last_logits != NULL it receives the float32 logits [vocab] of the last row.
 * Runs the same kernels as a batched verify step, 40 rows per pass. */
int32_t spd_prefill(spd_model *model, int32_t seq, const float *embeds, int32_t n_rows,
                    float *last_logits, void *stream);

/* Same, from token ids (int32 [n_rows]); the text-only draft's prefill (Section 3). */
int32_t spd_prefill_tokens(spd_model *model, int32_t seq, const int32_t *tokens, int32_t n_rows,
                           float *last_logits, void *stream);

/* HOT.  One decoder forward over M new tokens for each of sequences
 * 0..n_seqs-1, starting at each sequence's current KV length: the single
 * target call that yields T_1..T_{gamma+1} when tokens = [t, d_1..d_gamma] and
 * M = gamma+1 (Section 2.1, Section 3); M = 1 is plain autoregressive decoding.
 * tokens: int32 [n_seqs, M].  logits_out: float32 [n_seqs, M, vocab]; row j is
 * the distribution of the token after input j.  Appends the M keys/values of
 * every sequence and advances its KV length by M (roll back with
 * spd_kv_set_len).  Errors: SPD_ERR_SHAPE (M > 8 or n_seqs*M > 64),
 * SPD_ERR_CAPACITY (KV overflow; nothing is launched). */
int32_t spd_verify_forward(spd_model *target, const int32_t *tokens, int32_t n_seqs, int32_t M,
                           float *logits_out, void *stream);

/* HOT.  One draft decode step (Section 2.1: d_j ~ D(. | X_1:n, d_1..d_{j-1});
 * Section 3: text-only conditioning): feeds n_in (1 or 2) tokens per sequence
 * -- 2 after a fully accepted block, when the draft has not yet consumed
 * d_gamma -- and from the logits of the last one writes
 *   D_row_out  float32 [n_seqs, vocab]  softmax(logits / temperature)
 *   token_out  int32   [n_seqs]         drawn from D_row with the fixed-point
 *                                        inverse-CDF sampler and u_draft[n_seqs];
 * temperature 0: D_row is one-hot at the argmax (lowest index on ties).
 * tokens_in: int32 [n_seqs, n_in].  Advances the draft's KV lengths by n_in. */
int32_t spd_draft_step(spd_model *draft, const int32_t *tokens_in, int32_t n_seqs, int32_t n_in,
                       float temperature, const float *u_draft, float *D_row_out,
                       int32_t *token_out, void *stream);

/* HOT.  Speculative sampling for n_seqs sequences x gamma drafted tokens
 * (Section 2.1; Section 3 for the multimodal conditioning of T).
 *   target        float32 [n_seqs, gamma+1, vocab]  logits, or probabilities with SPD_TARGET_IS_PROBS
 *   draft         float32 [n_seqs, gamma, vocab]    logits, or probabilities with SPD_DRAFT_IS_PROBS
 *   draft_tokens  int32   [n_seqs, gamma]
 *   u             float32 [n_seqs, gamma+1] on the grid j/2^24: u[:, :gamma] drive the
 *                 accept tests, u[:, gamma] the replacement / bonus draw
 * Per sequence: k = number of leading j with u_j * D_j(d_j) < T_j(d_j) (float32
 * multiply and compare: accept probability min{1, T/D}); then the next token y
 * is drawn from max(0, T_{k+1} - D_{k+1}) normalised if k < gamma, else from
 * T_{gamma+1}, with the fixed-point inverse-CDF sampler: w(x) = floor(r(x) 2^32),
 * threshold = floor(u 2^24 * sum w / 2^24), y = first x whose running sum
 * exceeds it (if the residual has no representable mass: same draw from T_{k+1}).
 * temperature scales logits (softmax(l / temperature)); temperature 0 = greedy
 * (one-hot rows, lowest index on ties); it is ignored for probability inputs.
 *   n_accepted_out  int32 [n_seqs]      k
 *   next_token_out  int32 [n_seqs]      y
 *   accept_prob_out float32 [n_seqs, gamma] or NULL: min{1, T_j(d_j)/D_j(d_j)}
 *   workspace       float32 scratch, >= spd_accept_workspace_bytes(...) bytes
 * Errors: SPD_ERR_INVALID_ARG (NULL, gamma < 1, temperature < 0),
 * SPD_ERR_CAPACITY (workspace too small). */
int32_t spd_accept_workspace_bytes(int32_t n_seqs, int32_t gamma, int32_t vocab, size_t *h_bytes);
int32_t spd_speculative_accept(const float *target, const float *draft, const int32_t *draft_tokens,
                               const float *u, int32_t n_seqs, int32_t gamma, int32_t vocab,
                               float temperature, uint32_t flags, int32_t *n_accepted_out,
                               int32_t *next_token_out, float *accept_prob_out,
                               void *workspace, size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): spd_speculative_accept with its scratch memory in
 * a fixed 64 KiB array inside the library (one copy per GPU, held until the process ends).  Same
 * arguments, results and errors as spd_speculative_accept, minus the workspace; calls nothing that
 * allocates.  Limit: n_seqs * (2 gamma + 1) <= SPD_STATIC_ACCEPT_MAX_ROWS, else SPD_ERR_CAPACITY and
 * nothing is launched.  All calls on one GPU share that GPU's array: calls that may overlap (different
 * streams, different threads) race on it -- order them, or use spd_speculative_accept with one
 * workspace per stream.  Nothing in the array has to survive between calls. */
#define SPD_STATIC_ACCEPT_MAX_ROWS 4096
int32_t spd_speculative_accept_static(const float *target, const float *draft, const int32_t *draft_tokens,
                                      const float *u, int32_t n_seqs, int32_t gamma, int32_t vocab,
                                      float temperature, uint32_t flags, int32_t *n_accepted_out,
                                      int32_t *next_token_out, float *accept_prob_out, void *stream);

/* ---- the block loop without the host (Section 2.1, one block = gamma draft steps, one
 * target call, accept / resample, commit) ---------------------------------------------
 *
 * With the calls above the host reads k after every block to roll both KV caches back.
 * The calls below keep the KV lengths in device memory, so that a whole block is a fixed
 * sequence of launches with fixed arguments: it can be enqueued back to back, or captured
 * once in a HIP graph and replayed, without a host round trip per block.
 *
 * spd_kv_lens_to_device copies the model's current KV lengths into its workspace and
 * switches the model to device lengths: from then on every forward reads them there and
 * advances them there.  The host copy becomes an upper bound, so KV overflow can no longer
 * be refused before the launch: a forward whose device length leaves no room for its rows
 * works on a clamped length (every access stays in bounds, the results are meaningless) and
 * raises a flag that spd_kv_lens_from_device reports as SPD_ERR_CAPACITY.  Both calls wait
 * for `stream` (they are the only ones besides spd_trace_* that block).  spd_kv_set_len is
 * refused while the lengths live on the device. */
int32_t spd_kv_lens_to_device(spd_model *model, void *stream);
int32_t spd_kv_lens_from_device(spd_model *model, void *stream);

/* spd_draft_step with explicit strides (in elements between consecutive sequences), so that
 * a draft step can read its input from, and write its token and its D row into, the buffers
 * the target call and the accept step use: sequence s reads tokens_in[s * in_stride + i]
 * (i < n_in) and u_draft[s * u_stride], writes D_row_out[s * D_stride + x] (x < vocab) and
 * token_out[s * token_stride]. */
int32_t spd_draft_step_strided(spd_model *draft, const int32_t *tokens_in, int32_t in_stride, int32_t n_seqs,
                               int32_t n_in, float temperature, const float *u_draft, int32_t u_stride,
                               float *D_row_out, size_t D_stride, int32_t *token_out, int32_t token_stride,
                               void *stream);

/* Accept / resample and commit of one block, all on the device.  Both models must be in
 * device-length mode.  Inputs: target_logits float32 [n_seqs, gamma+1, vocab] of the target
 * call over verify_tokens = [t, d_1..d_gamma] (int32 [n_seqs, gamma+1]); draft_probs float32
 * [n_seqs, gamma, vocab], the D rows of the draft steps; u as in spd_speculative_accept.
 * Computes k and y exactly as spd_speculative_accept (target logits, draft probabilities),
 * then per sequence:
 *   - appends d_1..d_k, y to out_tokens[s, n_out[s]..] (int32 [n_seqs, out_capacity], may be
 *     NULL) and adds k+1 to n_out[s] (tokens beyond out_capacity are dropped);
 *   - verify_tokens[s, 0] = y (the next block's t);
 *   - draft_in_out[s] = [token before y, y] (int32 [n_seqs, 2]): the next block's first
 *     draft step takes these two tokens, whether or not the block was fully accepted;
 *   - both models' KV lengths -= gamma - k.
 * Convention of the loop: at the start of a block the target's KV cache holds everything
 * before t and the draft's cache everything before the token that precedes t (so the
 * draft re-computes that one position each block, which makes every block the same shape);
 * the first draft step has n_in = 2, the other gamma-1 steps n_in = 1. */
int32_t spd_block_finish(spd_model *target, spd_model *draft, const float *target_logits, const float *draft_probs,
                         int32_t *verify_tokens, const float *u, int32_t n_seqs, int32_t gamma, float temperature,
                         int32_t *n_accepted_out, int32_t *next_token_out, int32_t *draft_in_out,
                         int32_t *out_tokens, int32_t out_capacity, int32_t *n_out,
                         void *workspace, size_t workspace_bytes, void *stream);

/* Waits for `stream` and reports conditions that kernels can only flag on the device:
 * SPD_ERR_HIP if a bounded wait between workgroups (fused QKV + attention kernel) ever ran
 * into its spin limit -- never in a healthy run; results since then are
 * invalid --, SPD_ERR_CAPACITY if a forward in device-length mode found no room for its rows,
 * else SPD_OK. */
int32_t spd_device_status(spd_model *model, void *stream);

/* Tracing aid (not part of the method).  While enabled, every kernel launch group of
 * this model's forward passes is timed with a pair of HIP events (host-side event
 * objects only: no device memory): a group that is a single kernel gets them as the
 * launch's own start / stop events (the kernel's execution time, as a profiler
 * reports it), a group of several launches is bracketed by events recorded on the
 * caller's stream.  Where QKV projection and attention run as one kernel, kind 0
 * covers both and kind 5 stays empty.  spd_trace_read WAITS for
 * the recorded events (the one call here that blocks the host), adds the elapsed
 * milliseconds and launch counts per kind into h_ms_sum[n_kinds] / h_count[n_kinds] and
 * forgets them.  Kinds: 0 QKV projection, 1 O projection, 2 gate|up projection + SwiGLU,
 * 3 down projection, 4 LM head, 5 RoPE + KV append + attention, 6 input rows (embedding
 * gather).  The events perturb the stream slightly: time whole steps with tracing off. */
#define SPD_TRACE_KINDS 7
int32_t spd_trace_enable(spd_model *model, int32_t enable);
int32_t spd_trace_read(spd_model *model, int32_t n_kinds, double *h_ms_sum, int32_t *h_count);

/* Measurement aid (not part of the method): launches n_stages plain streaming-read kernels back to back on
 * `stream`, stage i reading h_stage_bytes[i] bytes (multiples of 1024) of `buffer` (any readable device memory
 * of buffer_bytes >= the sum; consecutive repetitions read different windows of it), `reps` times, and reports
 * in microseconds each kernel's own execution time (mean over the repetitions) and the wall time of one chain
 * (events around all repetitions).  This is what a chain of kernels of the projections' sizes costs on the
 * device when the kernels do nothing but read.  `sink`: 4 KiB of device memory the kernels may write.  Blocks
 * the host.  Errors: SPD_ERR_INVALID_ARG, SPD_ERR_CAPACITY (buffer too small / misaligned), SPD_ERR_HIP. */
int32_t spd_probe_read_chain(const void *buffer, size_t buffer_bytes, const size_t *h_stage_bytes, int32_t n_stages,
                             int32_t reps, void *sink, double *h_kernel_us, double *h_chain_us_per_rep, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPD_H */
