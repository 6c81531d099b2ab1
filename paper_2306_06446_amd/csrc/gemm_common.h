// Shared pieces of the two matrix-core kernels (int8 shift expert, fp16 Mult expert):
// the output-side epilogues and the accumulator-to-coordinate map of a 32x32 MFMA tile.
#pragma once

#include "common.h"

namespace sa {

enum EpiMode : int {
    kEpiInt32 = 0,     // y[m, n] = acc (+ bias[n])                              int32
    kEpiRequantLut,    // h[m, n] = lut[clamp(rne(float(acc) * rq)) + 128]        int8
    kEpiScatterI32,    // yf[rows[m], n] = gate[rows[m]] * (out_scale * float(acc))
    kEpiFloat,         // of[m, n] = acc                                          fp32
    kEpiGeluHalf,      // hh[m, n] = half(gelu(acc))                              fp16
    kEpiScatterF32,    // yf[rows[m], n] = gate[rows[m]] * acc
    kEpiLinearF32,     // parts[n / part_width][m, n % part_width] = fma(float(acc), lin_scale, residual[m, n])
    kEpiQkvCodes,      // column blocks 0 and 1 leave as sign codes (bit = acc >= 0) per head, block 2 as kEpiLinearF32
};

struct Epilogue {
    int32_t *y = nullptr;          // compact int32 out [max_rows, N]
    const int32_t *bias = nullptr;
    int8_t *h = nullptr;           // compact int8 out
    float rq = 1.0f;
    const int8_t *lut = nullptr;
    float *yf = nullptr;           // scattered fp32 out [T, N]
    const float *gate = nullptr;
    float out_scale = 1.0f;
    float *of = nullptr;           // compact fp32 out
    _Float16 *hh = nullptr;        // compact fp16 out
    bool accumulate = false;       // scattered fp32 out: add to what yf holds (fma(gate, value, old)) instead of overwriting
    float *parts[3] = {nullptr, nullptr, nullptr};   // kEpiLinearF32: column block p of width part_width goes to parts[p]
    int part_width = 0;
    const float *residual = nullptr;                 // kEpiLinearF32: [rows, N] or null
    float lin_scale = 1.0f;
    uint64_t *codes[2] = {nullptr, nullptr};         // kEpiQkvCodes: [B, H, tokens, head_dim / 64] each
    int head_dim = 0, tokens = 0, heads = 0;         // tokens per batch element
};

__device__ inline int8_t requant_code(float t) {
    // clamp(rne(t), -127, 127), NaN -> 0; t is the already rounded fp32 product
    t = __builtin_rintf(t);
    t = t < -127.0f ? -127.0f : t;
    t = t > 127.0f ? 127.0f : t;
    return (t != t) ? (int8_t)0 : (int8_t)t;
}

// The same code for an int32 accumulator and a finite scale, as the table index code + 128 (1..255),
// in five vector operations: clamp first (a finite product never is NaN), then add 1.5 * 2^23 + 128,
// which rounds to nearest even at unit spacing and leaves the index in the low byte of the sum.
// The host passes a finite scale (requant_scale_finite): the results are those of requant_code.
__device__ inline uint32_t requant_index(int32_t acc, float rq_finite) {
    const float t = __builtin_amdgcn_fmed3f((float)acc * rq_finite, -127.0f, 127.0f);
    return __builtin_bit_cast(uint32_t, t + 12583040.0f) & 0xFFu;
}

// requant_code as the byte of the int8 code, for a float that may be anything: clamp + magic add (three vector
// operations) and one select for NaN (a median with a NaN operand is not 0).
__device__ inline uint32_t requant_byte(float t) {
    const float c = __builtin_amdgcn_fmed3f(t, -127.0f, 127.0f);
    const uint32_t idx = __builtin_bit_cast(uint32_t, c + 12583040.0f) & 0xFFu;     // code + 128
    return (t != t) ? 0u : (idx ^ 0x80u);
}

// NaN -> 0 (every product is NaN -> code 0, as 0 * acc), +-Inf -> +-FLT_MAX (same clamped codes; 0 * acc = 0 -> code 0,
// where Inf * 0 = NaN -> code 0 as well).
inline float requant_scale_finite(float s) {
    if (s != s) return 0.0f;
    if (s > 3.402823466e38f) return 3.402823466e38f;
    if (s < -3.402823466e38f) return -3.402823466e38f;
    return s;
}

// Row of the 32x32 accumulator tile that register r of lane `lane` holds; the column is lane % 32.
__device__ inline int mfma32_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

}  // namespace sa
