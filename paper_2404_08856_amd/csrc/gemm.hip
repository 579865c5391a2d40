// Weight re-tiling and the skinny weight-streaming GEMM  Y[rows, N] = X[rows, K] W[N, K]^T
// (rows <= 64).  This is where ~97% of the bytes of a verify step are read: every
// projection of the decoder (QKV, O, gate|up, down, LM head) at gamma+1 rows is a
// stream over the weight matrix with ~5 flop per byte, so the kernel is organised
// around the HBM stream: weights are stored pre-tiled in matrix-core operand order
// (common.h), each wave reads 1 KiB blocks with one coalesced load per block and
// feeds them straight to v_mfma_f32_16x16x32_bf16; nothing goes through LDS except
// the final cross-wave reduction of a 16 x 8 output tile.
#include "gemm_core.h"
#include "launch.h"

namespace spd {

// ---------------------------------------------------------------------------------
// re-tiling
// ---------------------------------------------------------------------------------
__global__ void pack_weight_kernel(const uint16_t *__restrict__ src0, const uint16_t *__restrict__ src1,
                                   const uint16_t *__restrict__ src2, int mode, int N, int K, int KS,
                                   uint4 *__restrict__ dst, size_t n_lanes) {
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= n_lanes) return;
    int lane = (int)(gid & 63);
    size_t block = gid >> 6;
    int s = (int)(block % KS);
    int t = (int)(block / KS);
    int r = lane & 15, g = lane >> 4;
    int p = t * 16 + r;                       // packed row
    const uint16_t *src;
    int row;
    if (mode == PACK_PLAIN) {
        src = src0; row = p;
    } else if (mode == PACK_CONCAT3) {
        int third = N / 3;
        int which = p / third;
        src = which == 0 ? src0 : (which == 1 ? src1 : src2);
        row = p - which * third;
    } else {                                  // PACK_GATE_UP
        src = (r < 8) ? src0 : src1;
        row = t * 8 + (r & 7);
    }
    int k0 = s * 32 + g * 8;
    union { uint4 v; uint16_t h[8]; } out;
    const uint16_t *rp = src + (size_t)row * K + k0;
    if (k0 + 8 <= K) {
        out.v = *reinterpret_cast<const uint4 *>(rp);     // K % 8 == 0 and 16-byte aligned base
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) out.h[e] = (k0 + e < K) ? rp[e] : (uint16_t)0;
    }
    dst[gid] = out.v;
}

size_t packed_matrix_bytes(int N, int K) {
    size_t KS = (size_t)(K + 31) / 32;
    return (size_t)(N / 16) * KS * 1024;
}

hipError_t launch_pack_weight(const void *src0, const void *src1, const void *src2, int mode,
                              int N, int K, void *dst, hipStream_t stream) {
    int KS = (K + 31) / 32;
    size_t n_lanes = (size_t)(N / 16) * KS * 64;
    unsigned grid = (unsigned)((n_lanes + 255) / 256);
    hipLaunchKernelGGL(pack_weight_kernel, dim3(grid), dim3(256), 0, stream,
                       (const uint16_t *)src0, (const uint16_t *)src1, (const uint16_t *)src2, mode,
                       N, K, KS, (uint4 *)dst, n_lanes);
    return hipGetLastError();
}

LaunchTiming *&launch_timing() {
    static thread_local LaunchTiming *t = nullptr;
    return t;
}

// ---------------------------------------------------------------------------------
// GEMM
// ---------------------------------------------------------------------------------
struct GemmKernelArgs {
    const uint4 *W;
    const uint4 *X;
    int KS, n_tiles;
    int row0, rows;           // this launch covers rows row0 .. row0 + rows - 1 (row0 a multiple of 5)
    float *Y;
    int ldy;
    const float *ssq_in;      // [64][K / 16]: ssq_in_parts partial sums of squares per input row, or NULL
    int ssq_in_parts;
    float inv_d, eps;         // RMSNorm: 1 / sqrt(sum * inv_d + eps)
    const float *gain_next;   // RESIDUAL: gain of the norm that follows, or NULL
    uint16_t *Xnext;          // RESIDUAL: packed (h * gain_next), K = N
    float *ssq_out;           // RESIDUAL: [64][n_tiles] partial sums of squares of the new h, one per tile
    uint16_t *Xout;           // SWIGLU: packed activations, K = N / 2
    int KS_out;
};

// General one-row-group kernel (any K; used where the register-resident variant below does not
// apply, e.g. the down projection with K = 11008).  The NG parameter is kept at 1: several row
// groups go through gemm_multi_kernel.
// Persistent workgroups: workgroup b owns tiles b, b + gridDim.x, ...; its WAVES waves split
// the K range of every tile.  Each wave keeps a ring of U weight blocks (and the matching
// activation blocks) in flight: right after a block has been consumed by the matrix core its
// register slot is refilled with the block U steps ahead -- of the same tile or of the
// workgroup's next tile -- so the HBM stream never drains at a tile boundary, during the
// cross-wave reduction or during the epilogue.
template <int NG, int WAVES, int EPI, int U>
__global__ __launch_bounds__(WAVES * 64) void gemm_stream_kernel(GemmKernelArgs a) {
    static_assert(NG * 128 <= WAVES * 64, "one epilogue thread per (group, row slot, column)");
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index, known uniform
    const int KS = a.KS;
    const int s0 = (int)(((long)KS * w) / WAVES);
    const int s1 = (int)(((long)KS * (w + 1)) / WAVES);
    const int ns = s1 - s0;
    const int nfull = ns / U, rem = ns - nfull * U;
    const int G = gridDim.x;

    __shared__ float red[2][WAVES][NG][16][8];
    __shared__ float inv_s[kMaxRows];
    const int g0 = a.row0 / kGroupRows;                   // first row group of this launch (row0 % 5 == 0)

    uint4 av[U], bv[NG][U];
    int t = blockIdx.x;
    if (t < a.n_tiles) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (u < ns) {
                av[u] = load_stream(a.W + ((size_t)t * KS + s0 + u) * 64 + lane);
#pragma unroll
                for (int g = 0; g < NG; ++g) bv[g][u] = a.X[((size_t)(g0 + g) * KS + s0 + u) * 64 + lane];
            }
    }
    // 1 / rms of every input row from the producer's per-tile partial sums (fixed order)
    if (a.ssq_in) {
        for (int r = a.row0 + w; r < a.row0 + a.rows; r += WAVES) {
            float sum = 0.f;
            for (int p = lane; p < a.ssq_in_parts; p += 64) sum += a.ssq_in[(size_t)r * (KS * 2) + p];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
            if (lane == 0) inv_s[r] = 1.0f / sqrtf(sum * a.inv_d + a.eps);
        }
    } else {
        if (threadIdx.x < kMaxRows) inv_s[threadIdx.x] = 1.0f;
    }
    __syncthreads();

    int parity = 0;
    for (; t < a.n_tiles; t += G, parity ^= 1) {
        const int tn = t + G;
        // epilogue element of this thread (threads < NG * 128): fetch the old residual early
        const int e = threadIdx.x;
        const int en = e & 15, em = (e >> 4) & 7, eg = e >> 7;
        const int erow = a.row0 + eg * kGroupRows + em;               // absolute row of the call
        const bool e_in = e < NG * 128 && em < kGroupRows && erow < a.row0 + a.rows;
        const bool e_active = (EPI != EPI_SWIGLU) ? e_in : (e_in && en < 8);
        float hold = 0.f, gnext = 0.f;
        if (EPI == EPI_RESIDUAL && e_active) {
            hold = a.Y[(size_t)erow * a.ldy + (size_t)t * 16 + en];
            if (a.gain_next) gnext = a.gain_next[t * 16 + en];
        }

        f32x4_t acc[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) acc[g] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        // Steady state: straight-line code, no branch between a matrix-core step and the
        // refill of its slot, so that the compiler can wait for exactly the oldest block.
        // A slot whose next block lies beyond the workgroup's last tile re-reads an
        // activation block (cache hit, result unused) instead of branching.
        const bool has_next = tn < a.n_tiles;
        for (int c = 0; c < nfull; ++c) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int g = 0; g < NG; ++g) acc[g] = mfma_bf16(av[u], bv[g][u], acc[g]);
                const int i2 = c * U + u + U;
                const bool same = i2 < ns;
                const uint4 *wsrc = (same || has_next) ? a.W : a.X;
                const size_t woff = same ? ((size_t)t * KS + s0 + i2) : (has_next ? ((size_t)tn * KS + s0 + u) : (size_t)0);
                av[u] = load_stream(wsrc + woff * 64 + lane);
                const int xs = same ? s0 + i2 : s0 + u;
#pragma unroll
                for (int g = 0; g < NG; ++g) bv[g][u] = a.X[((size_t)(g0 + g) * KS + xs) * 64 + lane];
                __builtin_amdgcn_sched_barrier(0);        // keep "consume slot, refill slot" in program order
            }
        }
        if (rem) {                                        // ragged tail of this wave's K range
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (u < rem) {
#pragma unroll
                    for (int g = 0; g < NG; ++g) acc[g] = mfma_bf16(av[u], bv[g][u], acc[g]);
                    if (has_next) {
                        av[u] = load_stream(a.W + ((size_t)tn * KS + s0 + u) * 64 + lane);
#pragma unroll
                        for (int g = 0; g < NG; ++g) bv[g][u] = a.X[((size_t)(g0 + g) * KS + s0 + u) * 64 + lane];
                    }
                }
            }
        }
        // D[n = 4 (lane / 16) + v][c = lane % 16]; columns c, c + 5, c + 10 are the three terms of row c
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float x = sum_terms(acc[g][v]);
                if ((lane & 15) < kGroupRows) red[parity][w][g][4 * (lane >> 4) + v][lane & 15] = x;
            }
        __syncthreads();

        if (EPI == EPI_SWIGLU) {
            // rows 0..7 of a tile are gate features f0..f0+7, rows 8..15 the matching up features
            if (e_active) {
                float gate = 0.f, up = 0.f;
#pragma unroll
                for (int ww = 0; ww < WAVES; ++ww) {            // fixed order: deterministic
                    gate += red[parity][ww][eg][en][em];
                    up += red[parity][ww][eg][en + 8][em];
                }
                gate *= inv_s[erow];
                up *= inv_s[erow];
                float val = gate / (1.0f + expf(-gate)) * up;
                int f = t * 8 + en;
                uint16_t t3[kTerms];
                split3(val, t3);
#pragma unroll
                for (int q = 0; q < kTerms; ++q) a.Xout[xpack_index(erow, f, a.KS_out, q)] = t3[q];
            }
        } else if (e < NG * 128) {
            float sum = 0.f;
#pragma unroll
            for (int ww = 0; ww < WAVES; ++ww) sum += red[parity][ww][eg][en][em];
            sum *= inv_s[erow < kMaxRows ? erow : 0];
            if (EPI == EPI_STORE) {
                if (e_active) a.Y[(size_t)erow * a.ldy + (size_t)t * 16 + en] = sum;
            } else {
                float hnew = e_active ? hold + sum : 0.f;
                const int col = t * 16 + en;
                if (e_active) {
                    a.Y[(size_t)erow * a.ldy + col] = hnew;
                    if (a.gain_next) {
                        uint16_t t3[kTerms];
                        split3(hnew * gnext, t3);
                        const int KSn = a.n_tiles / 2;               // N / 32
#pragma unroll
                        for (int q = 0; q < kTerms; ++q) a.Xnext[xpack_index(erow, col, KSn, q)] = t3[q];
                    }
                }
                // sum of squares of the 16 new values of this row in this tile (lanes en = 0..15)
                float sq = hnew * hnew;
#pragma unroll
                for (int o = 8; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
                if (a.ssq_out && en == 0 && e_active) a.ssq_out[(size_t)erow * a.n_tiles + t] = sq;
            }
        }
        // no second barrier: the next tile writes the other half of `red`
    }
}

// More than one row group (6..64 rows): NG groups and TT weight tiles are in flight together.
// A weight block is used by all NG groups (NG matrix-core steps), an activation block by all
// TT tiles, so per streamed weight byte the workgroup reads (TT + NG) / TT bytes through its
// L1 instead of 1 + NG.  (Reading the activation blocks anew for every single tile, as the
// kernel above does, was measured at 2-3x the one-group time already for 2 groups: every
// workgroup of the chip asks the same L2 lines at the same moment.)  Persistent workgroups own
// groups of TT consecutive tiles (the last group may be ragged); 8 waves split K; two K-steps
// of loads are in flight per wave while the previous step is multiplied.
template <int NG, int TT, int EPI>
__global__ __launch_bounds__(512) void gemm_multi_kernel(GemmKernelArgs a) {
    constexpr int WAVES = 8;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KS = a.KS;
    const int s0 = (int)(((long)KS * w) / WAVES), s1 = (int)(((long)KS * (w + 1)) / WAVES);
    const int g0 = a.row0 / kGroupRows;
    const int n_groups_t = (a.n_tiles + TT - 1) / TT;     // tile groups
    const int ngv = (a.rows + kGroupRows - 1) / kGroupRows;   // row groups that hold rows of this pass (<= NG)

    __shared__ float red[WAVES][TT][NG][16][8];
    __shared__ float inv_s[kMaxRows];

    if (a.ssq_in) {
        for (int r = a.row0 + w; r < a.row0 + a.rows; r += WAVES) {
            float sum = 0.f;
            for (int p = lane; p < a.ssq_in_parts; p += 64) sum += a.ssq_in[(size_t)r * (KS * 2) + p];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
            if (lane == 0) inv_s[r] = 1.0f / sqrtf(sum * a.inv_d + a.eps);
        }
    } else if (threadIdx.x < kMaxRows) {
        inv_s[threadIdx.x] = 1.0f;
    }
    __syncthreads();

    for (int tg = blockIdx.x; tg < n_groups_t; tg += gridDim.x) {
        const int t0 = tg * TT;
        uint4 av[2][TT], bv[2][NG];
        auto load_step = [&](int buf, int s) {            // blocks of K-step s (tiles beyond the matrix: tile 0, unused)
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const int t = t0 + tt < a.n_tiles ? t0 + tt : 0;
                av[buf][tt] = load_stream(a.W + ((size_t)t * KS + s) * 64 + lane);
            }
#pragma unroll
            for (int g = 0; g < NG; ++g)                  // groups beyond this pass's rows: re-read the first one, result unused
                bv[buf][g] = a.X[((size_t)(g0 + (g < ngv ? g : 0)) * KS + s) * 64 + lane];
        };
        f32x4_t acc[TT][NG];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[tt][g] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (s0 < s1) load_step(0, s0);
        if (s0 + 1 < s1) load_step(1, s0 + 1);
        for (int s = s0; s < s1; s += 2) {
#pragma unroll
            for (int buf = 0; buf < 2; ++buf) {
                if (s + buf < s1) {                       // wave-uniform
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                        for (int g = 0; g < NG; ++g) acc[tt][g] = mfma_bf16(av[buf][tt], bv[buf][g], acc[tt][g]);
                    if (s + buf + 2 < s1) load_step(buf, s + buf + 2);
                }
            }
        }
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float x = sum_terms(acc[tt][g][v]);
                    if ((lane & 15) < kGroupRows) red[w][tt][g][4 * (lane >> 4) + v][lane & 15] = x;
                }
        __syncthreads();
        // epilogue: one element (tile tt, group g, row slot em, column en) per thread and round
        for (int e = threadIdx.x; e < TT * NG * 128; e += WAVES * 64) {
            const int en = e & 15, em = (e >> 4) & 7, g = (e >> 7) % NG, tt = (e >> 7) / NG;
            const int t = t0 + tt;
            const int erow = a.row0 + g * kGroupRows + em;
            const bool ok = em < kGroupRows && erow < a.row0 + a.rows && t < a.n_tiles;
            if (EPI == EPI_SWIGLU) {
                if (ok && en < 8) {
                    float gate = 0.f, up = 0.f;
#pragma unroll
                    for (int ww = 0; ww < WAVES; ++ww) { gate += red[ww][tt][g][en][em]; up += red[ww][tt][g][en + 8][em]; }
                    gate *= inv_s[erow];
                    up *= inv_s[erow];
                    uint16_t t3[kTerms];
                    split3(gate / (1.0f + expf(-gate)) * up, t3);
#pragma unroll
                    for (int q = 0; q < kTerms; ++q) a.Xout[xpack_index(erow, t * 8 + en, a.KS_out, q)] = t3[q];
                }
            } else {
                float sum = 0.f;
#pragma unroll
                for (int ww = 0; ww < WAVES; ++ww) sum += red[ww][tt][g][en][em];
                const int col = t * 16 + en;
                if (EPI == EPI_STORE) {
                    if (ok) a.Y[(size_t)erow * a.ldy + col] = sum * inv_s[erow];
                } else {
                    float hnew = 0.f;
                    if (ok) {
                        hnew = a.Y[(size_t)erow * a.ldy + col] + sum;
                        a.Y[(size_t)erow * a.ldy + col] = hnew;
                        if (a.gain_next) {
                            uint16_t t3[kTerms];
                            split3(hnew * a.gain_next[col], t3);
#pragma unroll
                            for (int q = 0; q < kTerms; ++q) a.Xnext[xpack_index(erow, col, a.n_tiles / 2, q)] = t3[q];
                        }
                    }
                    float sq = hnew * hnew;                // the 16 columns of a row slot sit in 16 neighbouring lanes
#pragma unroll
                    for (int o = 8; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
                    if (a.ssq_out && en == 0 && ok) a.ssq_out[(size_t)erow * a.n_tiles + t] = sq;
                }
            }
        }
        __syncthreads();                                  // `red` is rewritten by the next tile group
    }
}

template <int NG, int TT>
static hipError_t launch_multi(const GemmKernelArgs &k, int epilogue, int grid, hipStream_t stream) {
    dim3 g(grid), block(512);
    switch (epilogue) {
        case EPI_STORE: hipLaunchKernelGGL((gemm_multi_kernel<NG, TT, EPI_STORE>), g, block, 0, stream, k); break;
        case EPI_RESIDUAL: hipLaunchKernelGGL((gemm_multi_kernel<NG, TT, EPI_RESIDUAL>), g, block, 0, stream, k); break;
        case EPI_SWIGLU: hipLaunchKernelGGL((gemm_multi_kernel<NG, TT, EPI_SWIGLU>), g, block, 0, stream, k); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Batched rows (11..64 rows: several sequences' verify tokens, or a prefill pass)
// ---------------------------------------------------------------------------------
// With many row groups the activation operand is as large as a weight tile group (40 rows x K = 4096 x 3
// terms = 1 MiB), so a kernel whose waves split K re-reads it from L2 for every few tiles and is bound by
// that traffic, not by HBM.  Here the waves of a workgroup split TILES instead: all 8 waves walk the same
// K range, each with its own TT tiles, so an activation block is fetched once per workgroup (into LDS, CH
// K-steps at a time, several chunks ahead) and used by 8 * TT tiles.  No cross-wave reduction is needed.  To keep
// enough workgroups for the chip the K range is split ACROSS workgroups (J slices): every workgroup writes
// its partial tiles to a scratch buffer and counts itself in on its tile group's arrival counter; the one
// that arrives last (its ticket says so -- nobody ever waits) adds the J partials in slice order and runs
// the epilogue, then clears the counter for the next launch.  Fixed order => bit-reproducible.  The partials
// cross workgroups (and XCDs, each with its own L2) inside one launch: device-scope stores, acknowledged
// before the arrival is counted, and device-scope loads.
constexpr int kBatchWaves = 8, kBatchMaxJ = 8;
constexpr int kBatchCH = 4;      // K-steps per activation chunk: every LDS buffer holds NG * CH KiB
// chunks the weight ring runs ahead (registers: TT * RDC * CH * 4 for the ring next to TT * NG * 4 accumulators)
constexpr int batch_ring_chunks(int NG, int TT) { return (TT * NG * 4 + TT * 2 * kBatchCH * 4 <= 144) ? 2 : 1; }

struct BatchPlan { int TT, J, n_tgroups; };
// TT tiles per wave (accumulators = TT * NG * 4 VGPRs, weight ring = TT * CH blocks in flight per wave and ring
// chunk); J K-slices (at most 8: the last arriver reads J partials per output) so that there is about one
// workgroup per CU: the J in range with the shortest longest slice.
static BatchPlan batch_plan(int n_tiles, int KS, int NG, int tt = 0) {
    BatchPlan p;
    // Measured at the 7B shapes: one tile per wave beats two everywhere (40 rows: 5.31 against 5.45 ms per step, 20 rows:
    // 4.02 against 4.27) -- twice the workgroups, and the larger matrices then need no K slices at all.  Two tiles per
    // wave remain for matrices with more tile groups than arrival counters.
    p.TT = tt == 1 || tt == 2 ? tt : 1;
    p.n_tgroups = (n_tiles + kBatchWaves * p.TT - 1) / (kBatchWaves * p.TT);
    const int unit = batch_ring_chunks(NG, p.TT) * kBatchCH;
    const int n_units = (KS + unit - 1) / unit;
    int Jmax = 256 / p.n_tgroups;                             // at most one workgroup per CU: a single round
    if (Jmax > kBatchMaxJ) Jmax = kBatchMaxJ;
    if (Jmax > n_units) Jmax = n_units;
    if (Jmax < 1) Jmax = 1;
    int J = 1;
    for (int c = 2; c <= Jmax; ++c)                           // slices are whole units: the longest one has ceil(n_units / c)
        if ((n_units + c - 1) / c < (n_units + J - 1) / J) J = c;
    p.J = J;
    return p;
}
size_t gemm_batch_scratch_bytes(int N, int K) {
    const int n_tiles = N / 16, KS = (K + 31) / 32;
    size_t worst = 0;
    for (int NG : {4, 8, kMaxGroups})
        for (int tt : {1, 2}) {
            const BatchPlan p = batch_plan(n_tiles, KS, NG, tt);
            const size_t b = (size_t)p.J * p.n_tgroups * kBatchWaves * p.TT * NG * 80 * sizeof(float);
            worst = b > worst ? b : worst;
        }
    return worst;
}

struct BatchArgs { float *partials; unsigned *arrive; int J; const uint4 *zero_block; };

// Two loader waves next to the 8 multiplying waves bring the activation chunks into LDS with LDS-direct loads (no
// registers, asynchronous), NBUF - 1 chunks ahead of the products; a wave can have 63 loads outstanding, which
// bounds (NBUF - 1) * blocks per loader wave and chunk.
constexpr int kBatchLoaders = 2;
constexpr int batch_buffers(int NG) { return NG <= 8 ? 4 : 3; }

template <int NG, int TT, int EPI>
__global__ __launch_bounds__((kBatchWaves + kBatchLoaders) * 64) void gemm_batch_kernel(GemmKernelArgs a, BatchArgs b) {
    constexpr int WAVES = kBatchWaves, LW = kBatchLoaders, CH = kBatchCH, RDC = batch_ring_chunks(NG, TT), NBUF = batch_buffers(NG);
    constexpr int TPG = WAVES * TT;                        // tiles per workgroup
    constexpr int PB = (NG * CH + LW - 1) / LW;            // activation blocks per loader wave and chunk
    static_assert((NBUF - 1) * PB <= 63, "outstanding loads of a loader wave");
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KS = a.KS, J = b.J;
    const int j = blockIdx.x % J, tg = blockIdx.x / J;     // K slice fastest: the slices of a tile group start together
    // K slices are whole units of RDC chunks of CH K-steps; the last unit of the matrix may be ragged (its missing
    // K-steps get zero activations), so the loops below have no conditional parts and every wait counts exactly
    const int n_units = (KS + RDC * CH - 1) / (RDC * CH);
    const int c_begin = RDC * (int)(((long)n_units * j) / J), c_end = RDC * (int)(((long)n_units * (j + 1)) / J);
    const int g0 = a.row0 / kGroupRows;
    const int ngv = (a.rows + kGroupRows - 1) / kGroupRows;    // row groups that hold rows of this pass (<= NG)

    __shared__ uint4 Xs[NBUF][NG][CH][64];
    __shared__ float inv_s[kMaxRows];
    __shared__ int is_last;

    f32x4_t acc[TT][NG];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int g = 0; g < NG; ++g) acc[tt][g] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    if (w >= WAVES) {
        // ---- loader waves: chunk c + NBUF - 1 is requested while chunk c is multiplied; their loads wait in
        // their own queues, so the multiplying waves' weight rings are never held up by them ----
        auto issue_chunk = [&](int c) __attribute__((always_inline)) {
            const int cc = c < c_end ? c : c_begin;           // past the slice: a harmless re-read
            const int bufi = (c - c_begin) % NBUF;
#pragma unroll
            for (int r = 0; r < PB; ++r) {
                const int blk = (w - WAVES) + r * LW;         // wave-uniform
                const int bb = blk < NG * CH ? blk : 0;       // (an odd block count: the last one twice)
                const int k = bb % CH, g = bb / CH;
                const int s = cc * CH + k;
                // K-steps beyond the matrix read a block of zeros: they contribute nothing
                const uint4 *src = (s < KS ? a.X + ((size_t)(g0 + (g < ngv ? g : 0)) * KS + s) * 64 : b.zero_block) + lane;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                                 (__attribute__((address_space(3))) void *)&Xs[bufi][g][k][0], 16, 0, 0);
            }
        };
#pragma unroll
        for (int i = 0; i < NBUF - 1; ++i) issue_chunk(c_begin + i);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NBUF - 2) * PB) : "memory");   // chunk c_begin has landed (loads complete in order)
        __builtin_amdgcn_s_barrier();
        for (int c = c_begin; c < c_end; ++c) {
            issue_chunk(c + NBUF - 1);                        // into the buffer the products left one iteration ago
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NBUF - 2) * PB) : "memory");   // chunk c + 1 has landed
            __builtin_amdgcn_s_barrier();
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
        // ---- multiplying waves: TT tiles each, weight ring RDC chunks ahead; chunk c uses slots (c % RDC) * CH + k ----
        int tile[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int t = (tg * WAVES + w) * TT + tt;
            tile[tt] = t < a.n_tiles ? t : a.n_tiles - 1;     // beyond the matrix: a valid tile, result dropped
        }
        uint4 ring[TT][RDC * CH];
        auto refill = [&](int tt, int slot, int k, int c) __attribute__((always_inline)) {   // block (tile, K-step k of chunk c)
            int s = (c < c_end ? c : c_begin) * CH + k;       // past the slice: a harmless re-read
            s = s < KS ? s : KS - 1;
            ring[tt][slot] = load_stream(a.W + ((size_t)tile[tt] * KS + s) * 64 + lane);
        };
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int h = 0; h < RDC; ++h)
#pragma unroll
                for (int k = 0; k < CH; ++k) refill(tt, h * CH + k, k, c_begin + h);
        __syncthreads();
        int bufi = 0;
        for (int c0 = c_begin; c0 < c_end; c0 += RDC) {
#pragma unroll
            for (int h = 0; h < RDC; ++h) {
#pragma unroll
                for (int k = 0; k < CH; ++k) {
#pragma unroll
                    for (int g = 0; g < NG; ++g) {
                        const uint4 bq = Xs[bufi][g][k][lane];
#pragma unroll
                        for (int tt = 0; tt < TT; ++tt) acc[tt][g] = mfma_bf16(ring[tt][h * CH + k], bq, acc[tt][g]);
                    }
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) refill(tt, h * CH + k, k, c0 + h + RDC);
                    __builtin_amdgcn_sched_barrier(0);        // keep "multiply, refill the freed slots" in program order
                }
                bufi = bufi + 1 == NBUF ? 0 : bufi + 1;
                __syncthreads();
            }
        }
    }

    // ---- partial tiles of this K slice -> scratch: P[slice][tile][group][row slot c < 5][column n < 16] ----
    // Through LDS (the activation buffers are free now), so that the stores to memory are whole, contiguous lines:
    // device-scope stores are written through, and pieces of lines cost the memory a read-modify-write each.
    __syncthreads();                                      // the loaders' last (surplus) chunks have landed: the buffers are free
    float *stage = reinterpret_cast<float *>(&Xs[0][0][0][0]);
    static_assert(sizeof(Xs) >= (size_t)TPG * NG * 80 * sizeof(float), "staging area");
    const int r = lane & 15, grp = lane >> 4;
    if (w < WAVES) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int tl = w * TT + tt;                       // tile within the group
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                float4 v4;
                v4.x = sum_terms(acc[tt][g][0]); v4.y = sum_terms(acc[tt][g][1]);
                v4.z = sum_terms(acc[tt][g][2]); v4.w = sum_terms(acc[tt][g][3]);
                if (r < kGroupRows) *reinterpret_cast<float4 *>(stage + (((size_t)tl * NG + g) * kGroupRows + r) * 16 + 4 * grp) = v4;
            }
        }
    }
    __syncthreads();
    if (J > 1) {                                          // (a single slice finishes its tiles straight from the staging area)
        const unsigned long long *src = reinterpret_cast<const unsigned long long *>(stage);
        unsigned long long *dst = reinterpret_cast<unsigned long long *>(b.partials + (size_t)(tg * J + j) * TPG * NG * 80);
        for (int i = threadIdx.x; i < TPG * NG * 40; i += (WAVES + LW) * 64)
            __hip_atomic_store(dst + i, src[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // once the partials are acknowledged, count this workgroup in; the last one to arrive finishes the tiles
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0) {
            const unsigned ticket = __hip_atomic_fetch_add(b.arrive + tg, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            is_last = ticket == (unsigned)(J - 1);
        }
        __syncthreads();
        if (!is_last) return;
        if (threadIdx.x == 0) __hip_atomic_store(b.arrive + tg, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
    }

    // Four columns (tile, group, row slot c, columns 4 q .. 4 q + 3) per thread and item; q fastest: the 16
    // columns of a (row, tile) sit in 4 neighbouring lanes.  The other slices' partials were written through to
    // memory by workgroups on other XCDs: device-scope loads of 8 bytes.  All loads of up to four items are issued
    // before anything is used, and before the rows' 1 / rms is worked out, so the tail costs about two round trips.
    constexpr int NT = (WAVES + LW) * 64;
    constexpr int ITEMS = TPG * NG * kGroupRows * 4;
    // At most 16 partial quads in flight per thread: four items for up to 4 slices, two for up to 8.
    auto finish = [&](auto jc_, auto ipb_) __attribute__((always_inline)) {
    constexpr int JC = decltype(jc_)::value > 0 ? decltype(jc_)::value : 1, IPB = decltype(ipb_)::value;
    constexpr bool LOCAL = decltype(jc_)::value == 0;         // the only slice: its sums are still in the staging area
    for (int e0 = threadIdx.x; e0 - (int)threadIdx.x < ITEMS; e0 += NT * IPB) {
        unsigned long long lo[IPB][JC], hi[IPB][JC];
        float4 h4[IPB];
        bool ok[IPB];
#pragma unroll
        for (int i = 0; i < IPB; ++i) {
            const int e = e0 + i * NT;
            const int q = e & 3, c = (e >> 2) % kGroupRows, g = (e / (4 * kGroupRows)) % NG, tl = e / (4 * kGroupRows * NG);
            const int t = tg * TPG + tl;
            const int erow = a.row0 + g * kGroupRows + c;
            ok[i] = e < ITEMS && erow < a.row0 + a.rows && t < a.n_tiles;
            h4[i] = float4{0.f, 0.f, 0.f, 0.f};
            if (ok[i] && LOCAL) {
                const unsigned long long *src = reinterpret_cast<const unsigned long long *>(
                    stage + (((size_t)tl * NG + g) * kGroupRows + c) * 16 + 4 * q);
                lo[i][0] = src[0];
                hi[i][0] = src[1];
                if (EPI == EPI_RESIDUAL) h4[i] = *reinterpret_cast<const float4 *>(a.Y + (size_t)erow * a.ldy + t * 16 + 4 * q);
            } else if (ok[i]) {
                const unsigned long long *src = reinterpret_cast<const unsigned long long *>(
                    b.partials + ((((size_t)(tg * J) * TPG + tl) * NG + g) * kGroupRows + c) * 16 + 4 * q);
#pragma unroll
                for (int jj = 0; jj < JC; ++jj) {
                    if (jj < J) {                             // workgroup-uniform
                        const unsigned long long *pj = src + (size_t)jj * TPG * NG * kGroupRows * 8;
                        lo[i][jj] = __hip_atomic_load(pj, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        hi[i][jj] = __hip_atomic_load(pj + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
                if (EPI == EPI_RESIDUAL) h4[i] = *reinterpret_cast<const float4 *>(a.Y + (size_t)erow * a.ldy + t * 16 + 4 * q);
            }
        }
        if (e0 == (int)threadIdx.x) {
            // 1 / rms of every input row of this pass from the producer's partial sums: 16 lanes per row, fixed order
            if (a.ssq_in) {
                for (int row = a.row0 + (int)threadIdx.x / 16; row < a.row0 + kMaxRows; row += NT / 16) {
                    const bool in = row < a.row0 + a.rows;
                    const float inv = rms_inv_from_parts(a.ssq_in + (size_t)(in ? row : a.row0) * (KS * 2), a.ssq_in_parts, lane & 15, in, a.inv_d, a.eps);
                    if (in && (lane & 15) == 0) inv_s[row] = inv;
                }
            } else if (threadIdx.x < kMaxRows) {
                inv_s[threadIdx.x] = 1.0f;
            }
            __syncthreads();
        }
#pragma unroll
        for (int i = 0; i < IPB; ++i) {
            const int e = e0 + i * NT;
            const int q = e & 3, c = (e >> 2) % kGroupRows, g = (e / (4 * kGroupRows)) % NG, tl = e / (4 * kGroupRows * NG);
            const int t = tg * TPG + tl;
            const int erow = a.row0 + g * kGroupRows + c;
            float4 sum = float4{0.f, 0.f, 0.f, 0.f};
            if (ok[i]) {
#pragma unroll
                for (int jj = 0; jj < JC; ++jj) {             // slice order: the same sum in every run
                    if (jj < J) {
                        sum.x += __uint_as_float((unsigned)lo[i][jj]); sum.y += __uint_as_float((unsigned)(lo[i][jj] >> 32));
                        sum.z += __uint_as_float((unsigned)hi[i][jj]); sum.w += __uint_as_float((unsigned)(hi[i][jj] >> 32));
                    }
                }
                const float sc = inv_s[erow];
                sum.x *= sc; sum.y *= sc; sum.z *= sc; sum.w *= sc;
            }
            float v[4] = {sum.x, sum.y, sum.z, sum.w};
            if (EPI == EPI_SWIGLU) {
                // rows 0..7 of a tile are gate features (q = 0, 1), rows 8..15 the matching up features (q = 2, 3)
                float out4[4];
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const float up = __shfl_down(v[x], 2, 4);
                    out4[x] = v[x] / (1.0f + expf(-v[x])) * up;
                }
                if (ok[i] && q < 2) {
                    union { uint2 u; uint16_t h[4]; } term[kTerms];
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        uint16_t t3[kTerms];
                        split3(out4[x], t3);
#pragma unroll
                        for (int y = 0; y < kTerms; ++y) term[y].h[x] = t3[y];
                    }
#pragma unroll
                    for (int y = 0; y < kTerms; ++y)          // 4 consecutive features stay inside one 8-element lane slot
                        *reinterpret_cast<uint2 *>(a.Xout + xpack_index(erow, t * 8 + 4 * q, a.KS_out, y)) = term[y].u;
                }
            } else {
                const int col = t * 16 + 4 * q;
                if (EPI == EPI_STORE) {
                    if (ok[i]) *reinterpret_cast<float4 *>(a.Y + (size_t)erow * a.ldy + col) = sum;
                } else {
                    float sq = 0.f;
                    if (ok[i]) {
                        float4 hn = h4[i];
                        hn.x += v[0]; hn.y += v[1]; hn.z += v[2]; hn.w += v[3];
                        *reinterpret_cast<float4 *>(a.Y + (size_t)erow * a.ldy + col) = hn;
                        sq = (hn.x * hn.x + hn.y * hn.y) + (hn.z * hn.z + hn.w * hn.w);
                        if (a.gain_next) {
                            const float4 gn = *reinterpret_cast<const float4 *>(a.gain_next + col);
                            const float y4[4] = {hn.x * gn.x, hn.y * gn.y, hn.z * gn.z, hn.w * gn.w};
                            union { uint2 u; uint16_t h[4]; } term[kTerms];
#pragma unroll
                            for (int x = 0; x < 4; ++x) {
                                uint16_t t3[kTerms];
                                split3(y4[x], t3);
#pragma unroll
                                for (int y = 0; y < kTerms; ++y) term[y].h[x] = t3[y];
                            }
#pragma unroll
                            for (int y = 0; y < kTerms; ++y)
                                *reinterpret_cast<uint2 *>(a.Xnext + xpack_index(erow, col, a.n_tiles / 2, y)) = term[y].u;
                        }
                    }
                    sq += __shfl_xor(sq, 2);
                    sq += __shfl_xor(sq, 1);
                    if (a.ssq_out && q == 0 && ok[i]) a.ssq_out[(size_t)erow * a.n_tiles + t] = sq;
                }
            }
        }
    }
    };
    if (J == 1) finish(std::integral_constant<int, 0>{}, std::integral_constant<int, 4>{});
    else if (J <= 4) finish(std::integral_constant<int, 4>{}, std::integral_constant<int, 4>{});
    else finish(std::integral_constant<int, kBatchMaxJ>{}, std::integral_constant<int, 2>{});
}

template <int NG, int TT>
static hipError_t launch_batch(const GemmKernelArgs &k, const BatchArgs &b, int epilogue, int grid, hipStream_t stream) {
    dim3 g(grid), block((kBatchWaves + kBatchLoaders) * 64);
    switch (epilogue) {
        case EPI_STORE: hipLaunchKernelGGL((gemm_batch_kernel<NG, TT, EPI_STORE>), g, block, 0, stream, k, b); break;
        case EPI_RESIDUAL: hipLaunchKernelGGL((gemm_batch_kernel<NG, TT, EPI_RESIDUAL>), g, block, 0, stream, k, b); break;
        case EPI_SWIGLU: hipLaunchKernelGGL((gemm_batch_kernel<NG, TT, EPI_SWIGLU>), g, block, 0, stream, k, b); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Fast path for up to 8 rows (one row group) when every wave owns exactly NB K-steps of a
// tile (KS == WAVES * NB): the wave's slice of the activation operand stays in registers
// for the whole kernel -- it is the same for every tile -- so the only loads in the loop are
// the weight blocks.  (Measured on a read probe of the same shape: re-reading the
// activation blocks per tile from L2 costs 15-20% of the achieved HBM bandwidth.)
// The tile body is straight-line code: NB matrix-core steps, each followed by the refill
// of its register slot with the block U steps ahead (same tile, or the workgroup's next
// tile), so all of a wave's loads for the next tile are in flight while the tile is
// reduced across waves and written out.
// NG = 2: rows 6..10 (two row groups) with both groups' activation slices resident: every weight block
// feeds two matrix-core steps; the epilogue duty of a tile goes to four waves (a pair per group).
template <int WAVES, int EPI, int NB, int U, int NG = 1>
__global__ __launch_bounds__(WAVES * 64, (NG > 1 ? 1 : (NB <= 8 ? 4 : 2))) void gemm_regb_kernel(GemmKernelArgs a) {
    static_assert(NB % U == 0, "ring must divide the per-wave K range");
    static_assert(2 * NG <= WAVES && WAVES % (2 * NG) == 0, "a pair of epilogue waves per row group");
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KS = a.KS;                                  // == WAVES * NB
    const int s0 = w * NB;
    const int G = gridDim.x;

    __shared__ float red[2][WAVES][NG][16][8];

    int t = blockIdx.x;
    if (t >= a.n_tiles) return;

    uint4 av[U], bv[NG][NB];
#pragma unroll
    for (int u = 0; u < U; ++u) av[u] = load_stream(a.W + ((size_t)t * KS + s0 + u) * 64 + lane);
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int i = 0; i < NB; ++i) bv[g][i] = a.X[((size_t)g * KS + s0 + i) * 64 + lane];

    // Epilogue role of this thread: 2 NG consecutive waves take a tile (tile k starts at wave
    // 2 NG (k mod WAVES / (2 NG))), a pair per row group; a thread always handles row slot em
    // and column en, of the group its pair has in that tile.
    const int en = lane & 15, em = (w & 1) * 4 + (lane >> 4);
    float inv_row[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) inv_row[g] = 1.0f;
    if (a.ssq_in) {                                       // 1 / rms of rows em and 5 + em from the per-tile partial sums
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int row = g * kGroupRows + em;
            inv_row[g] = rms_inv_from_parts(a.ssq_in + (size_t)row * (KS * 2), a.ssq_in_parts, en,
                                            em < kGroupRows && row < a.rows, a.inv_d, a.eps);
        }
    }

    int parity = 0, turn = 0;
    for (; t < a.n_tiles; t += G, parity ^= 1, turn = (turn + 2 * NG) % WAVES) {
        const int tn = t + G;
        const bool has_next = tn < a.n_tiles;
        const int rel = w - turn;                         // 0 .. 2 NG - 1 for the waves on duty
        const bool my_turn = rel >= 0 && rel < 2 * NG;
        const int eg = my_turn ? (rel >> 1) : 0;          // row group of this wave's pair
        const int erow = eg * kGroupRows + em;
        const bool row_ok = em < kGroupRows && erow < a.rows;
        const bool e_active = my_turn && row_ok && (EPI != EPI_SWIGLU || en < 8);
        float inv = inv_row[0];
#pragma unroll
        for (int g = 1; g < NG; ++g) inv = (eg == g) ? inv_row[g] : inv;
        float hold = 0.f, gnext = 0.f;                    // the epilogue's operands, on their way before the tile's arithmetic
        if (EPI == EPI_RESIDUAL && e_active) {
            hold = a.Y[(size_t)erow * a.ldy + (size_t)t * 16 + en];
            if (a.gain_next) gnext = a.gain_next[t * 16 + en];
        }

        f32x4_t acc[NG];
        const uint4 *wcur = a.W + ((size_t)t * KS + s0) * 64 + lane;
        const uint4 *wnext = (has_next ? a.W + ((size_t)tn * KS + s0) * 64 : a.X) + lane;   // past the end: harmless re-read
        regb_tile<NB, U, NG>(acc, av, bv, wcur, wnext, has_next);
        store_partial<NG>(acc, red[parity][w], lane);
        __syncthreads();
        if (!my_turn) continue;

        if (EPI == EPI_SWIGLU) {
            if (e_active) {
                float gate = 0.f, up = 0.f;
#pragma unroll
                for (int ww = 0; ww < WAVES; ++ww) {
                    gate += red[parity][ww][eg][en][em];
                    up += red[parity][ww][eg][en + 8][em];
                }
                gate *= inv;
                up *= inv;
                float val = gate / (1.0f + expf(-gate)) * up;
                int f = t * 8 + en;
                uint16_t t3[kTerms];
                split3(val, t3);
#pragma unroll
                for (int q = 0; q < kTerms; ++q) a.Xout[xpack_index(erow, f, a.KS_out, q)] = t3[q];
            }
        } else {
            float sum = 0.f;
#pragma unroll
            for (int ww = 0; ww < WAVES; ++ww) sum += red[parity][ww][eg][en][em];
            sum *= inv;
            const int col = t * 16 + en;
            if (EPI == EPI_STORE) {
                if (e_active) a.Y[(size_t)erow * a.ldy + col] = sum;
            } else {
                float hnew = e_active ? hold + sum : 0.f;
                if (e_active) {
                    a.Y[(size_t)erow * a.ldy + col] = hnew;
                    if (a.gain_next) {
                        uint16_t t3[kTerms];
                        split3(hnew * gnext, t3);
                        const int KSn = a.n_tiles / 2;
#pragma unroll
                        for (int q = 0; q < kTerms; ++q) a.Xnext[xpack_index(erow, col, KSn, q)] = t3[q];
                    }
                }
                float sq = hnew * hnew;
#pragma unroll
                for (int o = 8; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
                if (a.ssq_out && en == 0 && e_active) a.ssq_out[(size_t)erow * a.n_tiles + t] = sq;
            }
        }
    }
}

template <int WAVES, int NB, int U, int NG = 1>
static hipError_t launch_regb(const GemmKernelArgs &k, int epilogue, int grid, hipStream_t stream) {
    dim3 g(grid), block(WAVES * 64);
    switch (epilogue) {
        case EPI_STORE:
            launch_kernel(gemm_regb_kernel<WAVES, EPI_STORE, NB, U, NG>, g, block, stream, k);
            break;
        case EPI_RESIDUAL:
            launch_kernel(gemm_regb_kernel<WAVES, EPI_RESIDUAL, NB, U, NG>, g, block, stream, k);
            break;
        case EPI_SWIGLU:
            launch_kernel(gemm_regb_kernel<WAVES, EPI_SWIGLU, NB, U, NG>, g, block, stream, k);
            break;
        default:
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int NG, int WAVES, int U>
static hipError_t launch_epi(const GemmKernelArgs &k, int epilogue, int grid, hipStream_t stream) {
    dim3 g(grid), block(WAVES * 64);
    switch (epilogue) {
        case EPI_STORE:
            launch_kernel(gemm_stream_kernel<NG, WAVES, EPI_STORE, U>, g, block, stream, k);
            break;
        case EPI_RESIDUAL:
            launch_kernel(gemm_stream_kernel<NG, WAVES, EPI_RESIDUAL, U>, g, block, stream, k);
            break;
        case EPI_SWIGLU:
            launch_kernel(gemm_stream_kernel<NG, WAVES, EPI_SWIGLU, U>, g, block, stream, k);
            break;
        default:
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Largest divisor of n_tiles that is <= cap (equal work per workgroup), at least cap / 2
// if one exists; otherwise cap itself (some workgroups then own one tile more).
static int pick_grid(int n_tiles, int cap) {
    if (n_tiles <= cap) return n_tiles;
    for (int g = cap; g >= cap / 2; --g)
        if (n_tiles % g == 0) return g;
    return cap;
}

hipError_t launch_gemm(const GemmArgs &a, int epilogue, GemmTuning tune, hipStream_t stream) {
    if (a.N % 16 != 0 || a.rows < 1 || a.rows > kMaxRows) return hipErrorInvalidValue;
    if (epilogue == EPI_RESIDUAL && a.gain_next && (a.N % 32 != 0)) return hipErrorInvalidValue;
    GemmKernelArgs k;
    k.W = (const uint4 *)a.W;
    k.X = (const uint4 *)a.X;
    k.KS = (a.K + 31) / 32;
    k.n_tiles = a.N / 16;
    k.row0 = 0;
    k.rows = a.rows;
    k.Y = a.Y;
    k.ldy = a.ldy;
    k.ssq_in = a.ssq_in;
    k.ssq_in_parts = a.ssq_in_parts;
    k.inv_d = a.K > 0 ? 1.0f / (float)a.K : 0.f;
    k.eps = a.eps;
    k.gain_next = a.gain_next;
    k.Xnext = (uint16_t *)a.Xnext;
    k.ssq_out = a.ssq_out;
    k.Xout = (uint16_t *)a.Xout;
    k.KS_out = (a.K_out + 31) / 32;
    const int groups = (a.rows + kGroupRows - 1) / kGroupRows;
    int waves = tune.waves;
    if (waves != 4 && waves != 8 && waves != 16) waves = 8;
    if (groups > 1 && waves == 16) waves = 8;            // 16 waves need <= 128 VGPRs: only the 1-group ring fits
    int cap = tune.grid_cap > 0 ? tune.grid_cap : (waves == 4 ? 1024 : (waves == 8 ? 512 : 256));
    const int grid = pick_grid(k.n_tiles, cap);
    if (groups == 1 && !tune.no_regb) {
        // register-resident activation slice: every wave owns exactly 8 or 16 K-steps.
        // Resident workgroups per CU follow from the register budget of each variant.
        auto grid_for = [&](int per_cu) { return pick_grid(k.n_tiles, tune.grid_cap > 0 ? tune.grid_cap : 256 * per_cu); };
        if (waves == 16 && k.KS == 16 * 8) return launch_regb<16, 8, 8>(k, epilogue, grid_for(1), stream);
        if (waves == 8 && k.KS == 8 * 16) return launch_regb<8, 16, 8>(k, epilogue, grid_for(1), stream);
        if (waves == 8 && k.KS == 8 * 8) return launch_regb<8, 8, 8>(k, epilogue, grid_for(2), stream);
        if (waves == 4 && k.KS == 4 * 8) return launch_regb<4, 8, 8>(k, epilogue, grid_for(4), stream);
        if (waves == 4 && k.KS == 4 * 16) return launch_regb<4, 16, 8>(k, epilogue, grid_for(2), stream);
    }
    if (groups == 2 && !tune.no_regb) {                 // rows 6..10: both activation slices register-resident
        const int g1 = pick_grid(k.n_tiles, tune.grid_cap > 0 ? tune.grid_cap : 256);
        if (waves == 16 && k.KS == 16 * 8) return launch_regb<16, 8, 8, 2>(k, epilogue, g1, stream);
        if (k.KS == 8 * 16) return launch_regb<8, 16, 8, 2>(k, epilogue, g1, stream);
        if (waves == 8 && k.KS == 8 * 8) return launch_regb<8, 8, 8, 2>(k, epilogue, g1, stream);
        if (waves == 4 && k.KS == 4 * 8) return launch_regb<4, 8, 8, 2>(k, epilogue, pick_grid(k.n_tiles, tune.grid_cap > 0 ? tune.grid_cap : 512), stream);
    }
#define SPD_GEMM_CASE(NG_, W_, U_) return launch_epi<NG_, W_, U_>(k, epilogue, grid, stream)
    if (groups == 1) {
        if (tune.ring == 16 && waves != 16) {
            if (waves == 4) SPD_GEMM_CASE(1, 4, 16);
            SPD_GEMM_CASE(1, 8, 16);
        }
        if (waves == 4) SPD_GEMM_CASE(1, 4, 8);
        if (waves == 8) SPD_GEMM_CASE(1, 8, 8);
        SPD_GEMM_CASE(1, 16, 8);
    }
    // rows 6..10 on a matrix with few tiles (the draft models' projections at 6..10 sequences): the general kernel with
    // both groups' activation blocks riding in the ring beats the K-splitting kernel below (d = 768: QKV 7.1 against
    // 8.6 us, O 6.5 / 8.8, down 9.3 / 12.0); from 256 tiles on it is the other way round (LM head 21.5 / 17.9)
    if (groups == 2 && k.n_tiles < 256) {
        if (waves == 4) SPD_GEMM_CASE(2, 4, 8);
        SPD_GEMM_CASE(2, 8, 8);
    }
#undef SPD_GEMM_CASE
    // More than 10 rows with a scratch buffer: the tile-splitting kernel makes one pass over the weights for up to 13
    // row groups (65 rows).  Measured at the 7B shapes against the K-splitting kernel (microseconds per launch), 20 rows:
    // gate|up 40 / 48, down 28 / 36, LM head 51 / 66, QKV 30 / 29, O 17 / 17; 40 rows: gate|up 51 / 67, down 34 / 52,
    // LM head 51 / 91, QKV 35 / 40, O 22 / 23; beyond 40 rows the K-splitting kernel needs a second pass.
    const bool batch_pays = groups > 2;
    if (a.batch_partials && a.batch_arrive && a.batch_zero && groups > 2 && !tune.no_batch && (batch_pays || tune.force_batch)) {
        const int NG = groups <= 4 ? 4 : (groups <= 8 ? 8 : kMaxGroups);
        BatchPlan p = batch_plan(k.n_tiles, k.KS, NG);
        if (p.n_tgroups > kBatchMaxTileGroups) p = batch_plan(k.n_tiles, k.KS, NG, 2);
        if (p.n_tgroups > kBatchMaxTileGroups) return hipErrorInvalidValue;     // more than 256 K output columns
        if (tune.grid_cap > 0 && tune.grid_cap / p.n_tgroups < p.J)          // a cap on the grid means fewer K slices here
            p.J = tune.grid_cap / p.n_tgroups > 0 ? tune.grid_cap / p.n_tgroups : 1;
        BatchArgs b{a.batch_partials, a.batch_arrive, p.J, (const uint4 *)a.batch_zero};
        const int bgrid = p.n_tgroups * p.J;
#define SPD_BATCH_CASE(NG_, TT_) if (NG == NG_ && p.TT == TT_) return launch_batch<NG_, TT_>(k, b, epilogue, bgrid, stream)
        SPD_BATCH_CASE(4, 1); SPD_BATCH_CASE(4, 2);
        SPD_BATCH_CASE(8, 1); SPD_BATCH_CASE(8, 2);
        SPD_BATCH_CASE(kMaxGroups, 1); SPD_BATCH_CASE(kMaxGroups, 2);
#undef SPD_BATCH_CASE
        return hipErrorInvalidValue;
    }
    // More than 5 rows: passes of up to 8 row groups (40 rows) over the weights.  Tiles are taken three at
    // a time where that still leaves a tile group for (almost) every CU, or where the matrix is too small to
    // fill the chip anyway.
    const bool wide = k.n_tiles >= 3 * 192 || k.n_tiles < 256;
    for (int g0 = 0; g0 < groups; g0 += 8) {
        const int ng = groups - g0 < 8 ? groups - g0 : 8;
        k.row0 = g0 * kGroupRows;
        k.rows = a.rows - k.row0 < ng * kGroupRows ? a.rows - k.row0 : ng * kGroupRows;
        const int tgroups = wide ? (k.n_tiles + 2) / 3 : k.n_tiles;
        const int mgrid = tgroups < 256 ? tgroups : 256;
        hipError_t e;
        if (ng <= 2) e = wide ? launch_multi<2, 3>(k, epilogue, mgrid, stream) : launch_multi<2, 1>(k, epilogue, mgrid, stream);
        else if (ng <= 4) e = wide ? launch_multi<4, 3>(k, epilogue, mgrid, stream) : launch_multi<4, 1>(k, epilogue, mgrid, stream);
        else e = wide ? launch_multi<8, 3>(k, epilogue, mgrid, stream) : launch_multi<8, 1>(k, epilogue, mgrid, stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace spd
