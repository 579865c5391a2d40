// Weight re-tiling and the skinny weight-streaming GEMM  Y[rows, N] = X[rows, K] W[N, K]^T
// (rows <= 64).  This is where ~97% of the bytes of a verify step are read: every
// projection of the decoder (QKV, O, gate|up, down, LM head) at gamma+1 rows is a
// stream over the weight matrix with ~5 flop per byte, so the kernel is organised
// around the HBM stream: weights are stored pre-tiled in matrix-core operand order
// (common.h), each wave reads 1 KiB blocks with one coalesced load per block and
// feeds them straight to v_mfma_f32_16x16x32_bf16; nothing goes through LDS except
// the final cross-wave reduction of a 16 x 8 output tile.
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

// ---------------------------------------------------------------------------------
// GEMM
// ---------------------------------------------------------------------------------
__device__ __forceinline__ f32x4_t mfma_bf16(const uint4 &a, const uint4 &b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

__device__ __forceinline__ uint4 load_stream(const uint4 *p) {
    // weights are read exactly once per step: mark the load non-temporal
    typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
    u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return uint4{v.x, v.y, v.z, v.w};
}

struct GemmKernelArgs {
    const uint4 *W;
    const uint4 *X;
    int KS, n_tiles, rows;
    float *Y;
    int ldy;
    uint16_t *Xout;
    int KS_out;
};

// One workgroup = R consecutive 16-row tiles of W; its WAVES waves split the K range.
template <int NG, int R, int WAVES, int EPI>
__global__ __launch_bounds__(WAVES * 64) void gemm_skinny_kernel(GemmKernelArgs a) {
    constexpr int U = (R * NG >= 4) ? 4 : 8;          // 1 KiB weight blocks in flight per tile
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int tile0 = blockIdx.x * R;
    const int KS = a.KS;
    const int s0 = (int)(((long)KS * w) / WAVES);
    const int s1 = (int)(((long)KS * (w + 1)) / WAVES);

    f32x4_t acc[R][NG];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int g = 0; g < NG; ++g) acc[r][g] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    const uint4 *wp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) wp[r] = a.W + (size_t)(tile0 + r) * KS * 64 + lane;
    const uint4 *xp = a.X + lane;

    int s = s0;
    for (; s + U <= s1; s += U) {
        uint4 av[R][U], bv[NG][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int r = 0; r < R; ++r) av[r][u] = load_stream(wp[r] + (size_t)(s + u) * 64);
#pragma unroll
            for (int g = 0; g < NG; ++g) bv[g][u] = xp[((size_t)g * KS + s + u) * 64];
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int g = 0; g < NG; ++g) acc[r][g] = mfma_bf16(av[r][u], bv[g][u], acc[r][g]);
    }
    for (; s < s1; ++s) {
        uint4 av[R], bv[NG];
#pragma unroll
        for (int r = 0; r < R; ++r) av[r] = load_stream(wp[r] + (size_t)s * 64);
#pragma unroll
        for (int g = 0; g < NG; ++g) bv[g] = xp[((size_t)g * KS + s) * 64];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[r][g] = mfma_bf16(av[r], bv[g], acc[r][g]);
    }

    // D[n = 4 (lane / 16) + v][c = lane % 16]; columns c and c + 8 are head and tail of row c.
    __shared__ float red[WAVES][R][NG][16][8];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float x = acc[r][g][v];
                float y = __shfl_xor(x, 8);
                if ((lane & 15) < 8) red[w][r][g][4 * (lane >> 4) + v][lane & 7] = x + y;
            }
    __syncthreads();

    if (EPI == EPI_SWIGLU) {
        // rows 0..7 of a tile are gate features f0..f0+7, rows 8..15 the matching up features
        for (int e = threadIdx.x; e < R * NG * 64; e += WAVES * 64) {
            int n = e & 7, m = (e >> 3) & 7, g = (e >> 6) % NG, r = e / (64 * NG);
            float gate = 0.f, up = 0.f;
#pragma unroll
            for (int ww = 0; ww < WAVES; ++ww) {      // fixed order: deterministic
                gate += red[ww][r][g][n][m];
                up += red[ww][r][g][n + 8][m];
            }
            int row = g * 8 + m;
            if (row < a.rows) {
                float val = gate / (1.0f + expf(-gate)) * up;
                int f = (tile0 + r) * 8 + n;
                uint16_t hi, lo;
                split_hi_lo(val, hi, lo);
                a.Xout[xpack_index(row, f, a.KS_out, 0)] = hi;
                a.Xout[xpack_index(row, f, a.KS_out, 1)] = lo;
            }
        }
    } else {
        for (int e = threadIdx.x; e < R * NG * 128; e += WAVES * 64) {
            int n = e & 15, m = (e >> 4) & 7, g = (e >> 7) % NG, r = e / (128 * NG);
            float sum = 0.f;
#pragma unroll
            for (int ww = 0; ww < WAVES; ++ww) sum += red[ww][r][g][n][m];
            int row = g * 8 + m;
            if (row < a.rows) {
                float *y = a.Y + (size_t)row * a.ldy + (size_t)(tile0 + r) * 16 + n;
                if (EPI == EPI_RESIDUAL) *y += sum; else *y = sum;
            }
        }
    }
}

template <int NG, int R, int WAVES>
static hipError_t launch_epi(const GemmKernelArgs &k, int epilogue, hipStream_t stream) {
    dim3 grid(k.n_tiles / R), block(WAVES * 64);
    switch (epilogue) {
        case EPI_STORE:
            hipLaunchKernelGGL((gemm_skinny_kernel<NG, R, WAVES, EPI_STORE>), grid, block, 0, stream, k);
            break;
        case EPI_RESIDUAL:
            hipLaunchKernelGGL((gemm_skinny_kernel<NG, R, WAVES, EPI_RESIDUAL>), grid, block, 0, stream, k);
            break;
        case EPI_SWIGLU:
            hipLaunchKernelGGL((gemm_skinny_kernel<NG, R, WAVES, EPI_SWIGLU>), grid, block, 0, stream, k);
            break;
        default:
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int NG>
static hipError_t launch_ng(const GemmKernelArgs &k, int epilogue, GemmTuning t, hipStream_t stream) {
    if (NG == 1) {
        if (t.tiles_per_wg == 2) {
            if (t.waves == 4) return launch_epi<NG, 2, 4>(k, epilogue, stream);
            if (t.waves == 8) return launch_epi<NG, 2, 8>(k, epilogue, stream);
            return launch_epi<NG, 2, 16>(k, epilogue, stream);
        }
        if (t.waves == 4) return launch_epi<NG, 1, 4>(k, epilogue, stream);
        if (t.waves == 8) return launch_epi<NG, 1, 8>(k, epilogue, stream);
        return launch_epi<NG, 1, 16>(k, epilogue, stream);
    }
    if (t.waves == 4) return launch_epi<NG, 1, 4>(k, epilogue, stream);
    return launch_epi<NG, 1, 8>(k, epilogue, stream);
}

hipError_t launch_gemm(const GemmArgs &a, int epilogue, GemmTuning tune, hipStream_t stream) {
    if (a.N % 16 != 0 || a.rows < 1 || a.rows > kMaxRows) return hipErrorInvalidValue;
    GemmKernelArgs k;
    k.W = (const uint4 *)a.W;
    k.X = (const uint4 *)a.X;
    k.KS = (a.K + 31) / 32;
    k.n_tiles = a.N / 16;
    k.rows = a.rows;
    k.Y = a.Y;
    k.ldy = a.ldy;
    k.Xout = (uint16_t *)a.Xout;
    k.KS_out = (a.K_out + 31) / 32;
    int groups = (a.rows + 7) / 8;
    // normalise the tuning to an instantiated variant
    if (tune.waves != 4 && tune.waves != 8 && tune.waves != 16) tune.waves = 8;
    if (groups > 1) {
        tune.tiles_per_wg = 1;
        if (tune.waves == 16) tune.waves = 8;
    }
    if (tune.tiles_per_wg != 2 || (k.n_tiles % 2) != 0) tune.tiles_per_wg = 1;
    if (groups == 1) return launch_ng<1>(k, epilogue, tune, stream);
    if (groups == 2) return launch_ng<2>(k, epilogue, tune, stream);
    if (groups <= 4) return launch_ng<4>(k, epilogue, tune, stream);
    return launch_ng<8>(k, epilogue, tune, stream);
}

}  // namespace spd
