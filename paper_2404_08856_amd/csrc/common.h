// Internal helpers shared by the HIP translation units of libspd (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int kWave = 64;
constexpr int kTileN = 16;     // weight rows per matrix-core tile
constexpr int kStepK = 32;     // contraction elements per matrix-core step
constexpr int kGroupRows = 5;  // activation rows per row group: 5 rows x 3 bf16 terms fill 15 of the 16 columns
constexpr int kTerms = 3;      // bf16 terms per activation value
constexpr int kMaxRows = 64;
constexpr int kMaxGroups = (kMaxRows + kGroupRows - 1) / kGroupRows;

// float32 -> bfloat16 bits, round to nearest even (NaN stays NaN): the conversion instruction of
// gfx950 (v_cvt_pk_bf16_f32; checked bit for bit against the integer formula
// (b + 0x7fff + ((b >> 16) & 1)) >> 16 on 2^24 random patterns, every exact tie, denormals and infinities).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}
// exp(x) for x <= 0 through the hardware base-2 exponential, with the rounding error of
// x * log2(e) carried along (about 2 ulp overall); arguments below -87 give (nearly) 0.
__device__ __forceinline__ float exp_neg(float x) {
    x = fmaxf(x, -87.0f);
    const float c1 = 1.44269502162933349609375f, c2 = 1.925963033500011e-8f;   // log2(e) = c1 + c2
    const float t = x * c1;
    const float lo = __builtin_fmaf(x, c1, -t) + x * c2;
    const float p = __builtin_amdgcn_exp2f(t);
    return __builtin_fmaf(p, lo * 0.693147180559945f, p);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t h) {
    return __uint_as_float(((uint32_t)h) << 16);
}
// two bf16 packed in a uint32 (element 0 in the low half)
__device__ __forceinline__ float bf16_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }

// Split x into three bf16 terms, x = t0 + t1 + t2 to float32 accuracy (each residual is exact
// in float32, three 8-bit significands cover the 24 bits).  Two terms (16 bits) are not
// enough: through 32 layers a 2^-17 perturbation of every projection input grows to a mean
// logit error of 3e-3 against a float64 reference, three terms give the same 1.5e-3 as
// float32 activations.
__device__ __forceinline__ void split3(float x, uint16_t (&t)[kTerms]) {
    t[0] = f32_to_bf16_bits(x);
    const float r1 = x - bf16_bits_to_f32(t[0]);
    t[1] = f32_to_bf16_bits(r1);
    t[2] = f32_to_bf16_bits(r1 - bf16_bits_to_f32(t[1]));
}
// Data-parallel-primitive moves inside a row of 16 lanes (no LDS traffic, no wait): lane i of a row
// receives the value of lane i + n (row_shl) or i - n (row_shr) of the same row, 0 beyond the row
// (lane semantics checked on the device).
template <int CTRL>
__device__ __forceinline__ float dpp_row(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
constexpr int kRowShl = 0x100, kRowShr = 0x110;

// Sum of the three term columns of an accumulator tile: on lanes with lane % 16 < 5 the result
// is D[.][c] + D[.][c + 5] + D[.][c + 10]; other lanes hold garbage (finite if the tile is).
__device__ __forceinline__ float sum_terms(float x) {
    return x + dpp_row<kRowShl + kGroupRows>(x) + dpp_row<kRowShl + 2 * kGroupRows>(x);
}
// The same sum on every lane of the three term columns: lane r < 15 of a row gets the sum of
// row r % 5; lane 15 gets a finite value nobody uses.
__device__ __forceinline__ float sum_terms_all(float x, int r) {
    const float y = sum_terms(x);
    const float y5 = dpp_row<kRowShr + kGroupRows>(y), y10 = dpp_row<kRowShr + 2 * kGroupRows>(y);
    return r < kGroupRows ? y : (r < 2 * kGroupRows ? y5 : y10);
}

// ---------------------------------------------------------------------------------
// Operand layouts for v_mfma_f32_16x16x32_bf16 (A: 16 x 32, B: 32 x 16, D: 16 x 16).
//
// Lane l = r + 16 g (r = l % 16, g = l / 16) holds
//     A[r][8g .. 8g+7]      B[8g .. 8g+7][r]      D[4g .. 4g+3][r]
//
// Weights W[N, K] are the A operand and are stored in HBM as a stream of 1 KiB
// blocks, block (tile t, step s) at index t * KS + s (KS = ceil(K / 32)); inside a
// block lane l's 8 bf16 sit at byte 16 l.  A wave reads one block with one fully
// coalesced 16-byte-per-lane load and feeds it to the matrix core unchanged.
//
// Activations X[rows, K] are the B operand.  Rows are taken in groups of 5; column
// c + 5 t (c < 5, t < 3) of the B operand is bf16 term t of row 5 grp + c (column 15 is
// unused), so one matrix-core step multiplies by all three terms at once and
// D[:, c] + D[:, c + 5] + D[:, c + 10] is the product with float32-accurate activations.
// Block (group grp, step s) sits at index grp * KS + s, lane layout as above.
// ---------------------------------------------------------------------------------
__host__ __device__ __forceinline__ size_t packed_elem_index(int row_in_tile, int k_in_step) {
    // element offset (bf16 units) inside one 512-element block
    int g = k_in_step >> 3, e = k_in_step & 7;
    return (size_t)((row_in_tile + 16 * g) * 8 + e);
}

// address (bf16 units) of activation element (row, k) in a packed activation buffer
__device__ __forceinline__ size_t xpack_index(int row, int k, int KS, int term) {
    int grp = row / kGroupRows, c = row % kGroupRows + kGroupRows * term;
    int s = k >> 5;
    return ((size_t)grp * KS + s) * 512 + packed_elem_index(c, k & 31);
}

struct SeqLens { int32_t len[kMaxRows]; };   // KV length of each sequence before the call

}  // namespace spd
