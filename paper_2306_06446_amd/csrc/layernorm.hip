// LayerNorm of Eq. 2 fused with what its consumers read: the int8 codes of the shift Linears
// (static per-tensor scale), the fp16 rows of the Mult expert and the router logits (Sec. 4.2).
//
// One wavefront owns one row, held in registers (CH float4 per lane), so x is read once:
// mean, then the centred sum of squares (two passes over registers, no E[x^2] - mean^2
// cancellation), then the outputs.  HBM-bound: 4 B in and 1 (+2, +4) B out per element.
#include "common.h"
#include "gemm_common.h"

namespace {

using namespace sa;

typedef _Float16 v4h_t __attribute__((ext_vector_type(4)));

constexpr int kRowsPerBlock = 4;      // one wavefront each
constexpr int kMaxExperts = 8;

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

struct LnArgs {
    const float *x;
    long T;
    int E;
    const float *gamma, *beta;
    float eps, inv_scale;
    float *ln;          // optional outputs
    int8_t *q;
    _Float16 *xh;
    const float *wg;    // [E, n_exp] or null
    const float *bg;    // [n_exp]
    int n_exp;
    float *logits;      // [T, n_exp]
};

// ROUTE: the router has two experts and its weight columns live in registers next to gamma and
// beta (all three depend on the column only), so a wavefront that walks over several rows loads
// them once.  More experts take the weights from memory (the table is small and stays in cache).
template <int CH, bool ROUTE2>
__global__ __launch_bounds__(64 * kRowsPerBlock) void layernorm_kernel(LnArgs a, int rows_per_wave) {
    const int lane = threadIdx.x & 63;
    const int E = a.E;
    const long t0 = ((long)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6)) * rows_per_wave;
    if (t0 >= a.T) return;
    constexpr bool CACHE = CH <= 8;               // wider rows re-read gamma and beta per row (registers)
    constexpr int PC = CACHE ? CH : 1;
    float4 gm[PC], bt[PC], w0[PC], w1[PC];
#pragma unroll
    for (int c = 0; c < PC; ++c) {
        const int j = (c * 64 + lane) * 4;
        const bool in = j < E;
        gm[c] = in ? *reinterpret_cast<const float4 *>(a.gamma + j) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        bt[c] = in ? *reinterpret_cast<const float4 *>(a.beta + j) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (ROUTE2) {                             // wg rows j..j+3: (e0, e1) pairs
            w0[c] = in ? *reinterpret_cast<const float4 *>(a.wg + 2 * j) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            w1[c] = in ? *reinterpret_cast<const float4 *>(a.wg + 2 * j + 4) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
    }
    const long t_end = t0 + rows_per_wave < a.T ? t0 + rows_per_wave : a.T;
    for (long t = t0; t < t_end; ++t) {
        const float *row = a.x + (size_t)t * E;
        float4 v[CH];
        float s = 0.0f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int j = (c * 64 + lane) * 4;
            v[c] = j < E ? *reinterpret_cast<const float4 *>(row + j) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            s += (v[c].x + v[c].y) + (v[c].z + v[c].w);
        }
        const float mean = wave_sum(s) / (float)E;
        float ss = 0.0f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int j = (c * 64 + lane) * 4;
            if (j < E) {
                const float d0 = v[c].x - mean, d1 = v[c].y - mean, d2 = v[c].z - mean, d3 = v[c].w - mean;
                ss += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
            }
        }
        const float rstd = 1.0f / __builtin_sqrtf(wave_sum(ss) / (float)E + a.eps);
        float part[kMaxExperts];
#pragma unroll
        for (int e = 0; e < kMaxExperts; ++e) part[e] = 0.0f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int j = (c * 64 + lane) * 4;
            if (j >= E) continue;
            const float4 g = CACHE ? gm[CACHE ? c : 0] : *reinterpret_cast<const float4 *>(a.gamma + j);
            const float4 b = CACHE ? bt[CACHE ? c : 0] : *reinterpret_cast<const float4 *>(a.beta + j);
            float y[4];
            y[0] = (v[c].x - mean) * rstd * g.x + b.x;
            y[1] = (v[c].y - mean) * rstd * g.y + b.y;
            y[2] = (v[c].z - mean) * rstd * g.z + b.z;
            y[3] = (v[c].w - mean) * rstd * g.w + b.w;
            const size_t o = (size_t)t * E + j;
            if (a.ln) *reinterpret_cast<float4 *>(a.ln + o) = make_float4(y[0], y[1], y[2], y[3]);
            if (a.q) {
                uint32_t w = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) w |= (uint32_t)(uint8_t)requant_code(y[i] * a.inv_scale) << (8 * i);
                *reinterpret_cast<uint32_t *>(a.q + o) = w;
            }
            if (a.xh) {
                v4h_t h;
#pragma unroll
                for (int i = 0; i < 4; ++i) h[i] = (_Float16)y[i];
                *reinterpret_cast<v4h_t *>(a.xh + o) = h;
            }
            if (ROUTE2 && CACHE) {
                part[0] = __builtin_fmaf(y[0], w0[c].x, part[0]);
                part[1] = __builtin_fmaf(y[0], w0[c].y, part[1]);
                part[0] = __builtin_fmaf(y[1], w0[c].z, part[0]);
                part[1] = __builtin_fmaf(y[1], w0[c].w, part[1]);
                part[0] = __builtin_fmaf(y[2], w1[c].x, part[0]);
                part[1] = __builtin_fmaf(y[2], w1[c].y, part[1]);
                part[0] = __builtin_fmaf(y[3], w1[c].z, part[0]);
                part[1] = __builtin_fmaf(y[3], w1[c].w, part[1]);
            } else if (a.logits) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int e = 0; e < kMaxExperts; ++e)
                        if (e < a.n_exp) part[e] = __builtin_fmaf(y[i], a.wg[(size_t)(j + i) * a.n_exp + e], part[e]);
            }
        }
        if (a.logits) {
#pragma unroll
            for (int e = 0; e < kMaxExperts; ++e) {
                if (e >= a.n_exp) break;
                const float sum = wave_sum(part[e]);
                if (lane == 0) a.logits[(size_t)t * a.n_exp + e] = sum + a.bg[e];
            }
        }
    }
}

template <int CH>
int launch(const LnArgs &a, hipStream_t st) {
    // a few rows per wavefront amortise the per-column parameters; keep >= ~2000 wavefronts in flight
    int rows_per_wave = 1;
    while (rows_per_wave < 8 && a.T / (2 * rows_per_wave) >= 2048) rows_per_wave *= 2;
    const long waves = (a.T + rows_per_wave - 1) / rows_per_wave;
    const long blocks = (waves + kRowsPerBlock - 1) / kRowsPerBlock;
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_layernorm_quant: too many rows");
    const dim3 grid((unsigned)blocks), block(64 * kRowsPerBlock);
    if (a.logits && a.n_exp == 2 && CH <= 8)
        layernorm_kernel<CH, true><<<grid, block, 0, st>>>(a, rows_per_wave);
    else
        layernorm_kernel<CH, false><<<grid, block, 0, st>>>(a, rows_per_wave);
    return check_launch("sa_layernorm_quant");
}

}  // namespace

extern "C" int sa_layernorm_quant(const float *x, long T, int E, const float *gamma, const float *beta, float eps,
                                  float inv_scale, float *ln_or_null, int8_t *q_or_null, void *xh_or_null,
                                  const float *wg_or_null, const float *bg_or_null, int n_experts,
                                  float *logits_or_null, void *stream) {
    sa::clear_error();
    SA_REQUIRE(T >= 0 && E > 0, SA_ERR_INVALID, "sa_layernorm_quant: T < 0 or E <= 0");
    SA_REQUIRE(E % 4 == 0, SA_ERR_SHAPE, "sa_layernorm_quant: E (%d) must be a multiple of 4", E);
    SA_REQUIRE(E <= 8192, SA_ERR_UNSUPPORTED, "sa_layernorm_quant: rows of more than 8192 elements are not built");
    const bool route = logits_or_null != nullptr;
    if (route) {
        SA_REQUIRE(wg_or_null && bg_or_null, SA_ERR_INVALID, "sa_layernorm_quant: logits need wg and bg");
        SA_REQUIRE(n_experts >= 2 && n_experts <= kMaxExperts, SA_ERR_SHAPE,
                   "sa_layernorm_quant: 2 to 8 experts (got %d)", n_experts);
    }
    if (T == 0) return SA_OK;
    SA_REQUIRE(x && gamma && beta, SA_ERR_INVALID, "sa_layernorm_quant: NULL buffer");
    SA_REQUIRE(ln_or_null || q_or_null || xh_or_null || route, SA_ERR_INVALID, "sa_layernorm_quant: no output requested");
    SA_REQUIRE(sa::aligned16(x) && sa::aligned16(gamma) && sa::aligned16(beta) && sa::aligned16(ln_or_null) &&
                   sa::aligned16(q_or_null) && sa::aligned16(xh_or_null) && sa::aligned16(wg_or_null) &&
                   sa::aligned16(bg_or_null) && sa::aligned16(logits_or_null),
               SA_ERR_ALIGN, "sa_layernorm_quant: pointers must be 16-byte aligned");
    LnArgs a{x, T, E, gamma, beta, eps, inv_scale, ln_or_null, q_or_null, static_cast<_Float16 *>(xh_or_null),
             route ? wg_or_null : nullptr, route ? bg_or_null : nullptr, route ? n_experts : 0, logits_or_null};
    hipStream_t st = sa::as_stream(stream);
    const int ch = (E + 255) / 256;
    if (ch <= 1) return launch<1>(a, st);
    if (ch <= 2) return launch<2>(a, st);
    if (ch <= 3) return launch<3>(a, st);
    if (ch <= 4) return launch<4>(a, st);
    if (ch <= 8) return launch<8>(a, st);
    if (ch <= 16) return launch<16>(a, st);
    return launch<32>(a, st);
}
