/*
 * CPU oracle for the reparameterised transformer-block path of ShiftAddViT.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the path computes, as
 * plain loops in fp64 / int64, so that the GPU library can be compared with
 * it.  It shares no code with the GPU library, is never linked into it and is
 * never called by it.  Only the tests, the smoke check and the benchmark's
 * CPU-baseline leg may call it.
 *
 * Every function cites the passage of the paper it follows.  Where the paper
 * is silent the reading taken is stated next to the code.
 *
 * Conventions
 *   codes : uint64 [B, H, N, W], W = nbits / 64, bit j of a code lives in
 *           word j / 64 at position j % 64 (least significant bit = lowest j)
 *   sigma : bit 1 -> +1, bit 0 -> -1  (codes live in Hamming space, abstract;
 *           the Add layer of Eq. 3 accumulates the selected operand rows)
 *   x,Q,K : fp32 [B, N, H, d];  V, O : [B, N, H, dv];  KV : [B, H, nbits, dv]
 *
 * All floating-point outputs are fp64 computed from the fp32 / packed inputs,
 * except where a float decides an integer (hash bits, quantised codes): those
 * decisions are taken in fp32 with the single rounding sequence stated at the
 * function, so that the other side can take the same decision.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * against closed forms, dense +-1 matmuls, brute force and special cases.
 * The paper prints no worked numeric example for any of these operations.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline int code_bit(const uint64_t *code, int j) {
    return (int)((code[j >> 6] >> (j & 63)) & 1u);
}

/* ------------------------------------------------------------------------
 * Hashing Q / K to binary codes (Sec. 4.1, reparameterisation of attention:
 * binary quantisation of Q and K; appendix "scaling factor clarification":
 * vanilla layer-wise sign quantisation, or a set of hash functions).
 *
 * proj == NULL : bit_j = [x_j >= 0]                     (nbits == d)
 * proj != NULL : bit_j = [sum_k x_k * proj[k][j] >= 0]  (sign of a projection)
 *
 * The sum is DEFINED as the fp32 chain acc = fma(x_k, proj[k][j], acc) for
 * k = 0 .. d-1 starting from +0.0f: the sign of a float sum depends on the
 * order, so one order is part of the definition.  >= makes +-0 hash to 1 and
 * NaN to 0.
 * ------------------------------------------------------------------------ */
void oracle_binarize(const float *x, int B, int N, int H, int d,
                     const float *proj, int nbits, uint64_t *codes) {
    const int W = nbits / 64;
#pragma omp parallel for collapse(2)
    for (int b = 0; b < B; ++b)
        for (int n = 0; n < N; ++n)
            for (int h = 0; h < H; ++h) {
                const float *row = x + (((size_t)b * N + n) * H + h) * d;
                uint64_t *out = codes + (((size_t)b * H + h) * N + n) * W;
                for (int w = 0; w < W; ++w) out[w] = 0;
                for (int j = 0; j < nbits; ++j) {
                    float acc;
                    if (proj == NULL) {
                        acc = row[j];
                    } else {
                        acc = 0.0f;
                        for (int k = 0; k < d; ++k)
                            acc = fmaf(row[k], proj[(size_t)k * nbits + j], acc);
                    }
                    if (acc >= 0.0f) out[j >> 6] |= (uint64_t)1 << (j & 63);
                }
            }
}

/* ------------------------------------------------------------------------
 * K^T V as an Add layer (Eq. 3, O_Add; Sec. 4.1: order of the MatMuls
 * exchanged from (QK)V to Q(KV)).
 *   KV[b,h,j,c] = sum_n sigma(K[b,h,n,j]) * V[b,n,h,c]
 * ------------------------------------------------------------------------ */
void oracle_ktv(const uint64_t *k_codes, const float *v, int B, int H, int Nk,
                int nbits, int dv, double *kv) {
    const int W = nbits / 64;
#pragma omp parallel for collapse(2)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            double *KV = kv + ((size_t)b * H + h) * nbits * dv;
            for (size_t i = 0; i < (size_t)nbits * dv; ++i) KV[i] = 0.0;
            for (int n = 0; n < Nk; ++n) {
                const uint64_t *code = k_codes + (((size_t)b * H + h) * Nk + n) * W;
                const float *vr = v + (((size_t)b * Nk + n) * H + h) * dv;
                for (int j = 0; j < nbits; ++j) {
                    const double s = code_bit(code, j) ? 1.0 : -1.0;
                    for (int c = 0; c < dv; ++c) KV[(size_t)j * dv + c] += s * (double)vr[c];
                }
            }
        }
}

/* ------------------------------------------------------------------------
 * Q (K^T V) as an Add layer followed by the post-add scale (Eq. 3, O_Add;
 * appendix "scaling factor clarification": the layer-wise scale is multiplied
 * after the add operations).
 *   O[b,n,h,c] = scale * sum_j sigma(Q[b,h,n,j]) * KV[b,h,j,c]
 * ------------------------------------------------------------------------ */
void oracle_qkv(const uint64_t *q_codes, const double *kv, int B, int H, int Nq,
                int nbits, int dv, float scale, double *out) {
    const int W = nbits / 64;
#pragma omp parallel for collapse(2)
    for (int b = 0; b < B; ++b)
        for (int n = 0; n < Nq; ++n)
            for (int h = 0; h < H; ++h) {
                const uint64_t *code = q_codes + (((size_t)b * H + h) * Nq + n) * W;
                const double *KV = kv + ((size_t)b * H + h) * nbits * dv;
                double *o = out + (((size_t)b * Nq + n) * H + h) * dv;
                for (int c = 0; c < dv; ++c) {
                    double acc = 0.0;
                    for (int j = 0; j < nbits; ++j)
                        acc += (code_bit(code, j) ? 1.0 : -1.0) * KV[(size_t)j * dv + c];
                    o[c] = (double)scale * acc;
                }
            }
}

/* ------------------------------------------------------------------------
 * Hamming similarity of two codes: the dot product of their +-1 vectors,
 * written out bit by bit (abstract: Q and K mapped to binary codes in Hamming
 * space; Eq. 1 with both operands of Q K^T binarised).
 * ------------------------------------------------------------------------ */
static int sigma_dot(const uint64_t *a, const uint64_t *b, int nbits) {
    int s = 0;
    for (int j = 0; j < nbits; ++j) s += (code_bit(a, j) == code_bit(b, j)) ? 1 : -1;
    return s;
}

void oracle_hamming_scores(const uint64_t *q_codes, const uint64_t *k_codes, int B, int H,
                           int Nq, int Nk, int nbits, int16_t *scores) {
    const int W = nbits / 64;
#pragma omp parallel for collapse(2)
    for (int bh = 0; bh < B * H; ++bh)
        for (int i = 0; i < Nq; ++i) {
            const uint64_t *qc = q_codes + ((size_t)bh * Nq + i) * W;
            for (int j = 0; j < Nk; ++j) {
                const uint64_t *kc = k_codes + ((size_t)bh * Nk + j) * W;
                scores[((size_t)bh * Nq + i) * Nk + j] = (int16_t)sigma_dot(qc, kc, nbits);
            }
        }
}

/* ------------------------------------------------------------------------
 * Quadratic variant (Eq. 1 with the Q K^T MatMul replaced by the Hamming
 * similarity of the codes; V stays in high precision, Sec. 4.1):
 *   O[b,i,h,:] = sum_j softmax_j(scale * S[i,j]) * V[b,j,h,:]
 * Softmax with the row maximum subtracted, all in fp64.
 * ------------------------------------------------------------------------ */
void oracle_hamming_attention(const uint64_t *q_codes, const uint64_t *k_codes, const float *v,
                              int B, int H, int Nq, int Nk, int nbits, int dv, float scale,
                              double *out) {
    const int W = nbits / 64;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)Nk);
#pragma omp for collapse(2)
        for (int bh = 0; bh < B * H; ++bh)
            for (int i = 0; i < Nq; ++i) {
                const int b = bh / H, h = bh % H;
                const uint64_t *qc = q_codes + ((size_t)bh * Nq + i) * W;
                double mx = -INFINITY;
                for (int j = 0; j < Nk; ++j) {
                    const uint64_t *kc = k_codes + ((size_t)bh * Nk + j) * W;
                    p[j] = (double)scale * (double)sigma_dot(qc, kc, nbits);
                    if (p[j] > mx) mx = p[j];
                }
                double den = 0.0;
                for (int j = 0; j < Nk; ++j) { p[j] = exp(p[j] - mx); den += p[j]; }
                double *o = out + (((size_t)b * Nq + i) * H + h) * dv;
                for (int c = 0; c < dv; ++c) {
                    double acc = 0.0;
                    for (int j = 0; j < Nk; ++j)
                        acc += p[j] * (double)v[(((size_t)b * Nk + j) * H + h) * dv + c];
                    o[c] = acc / den;
                }
            }
        free(p);
    }
}

/* ------------------------------------------------------------------------
 * Shift layer (Eq. 3, O_Shift = sum X * s * 2^P with s in {-1,+1}).
 * Stored nibble = (neg << 3) | e, e = P + 7 in [0,7] (P in [-7,0]); on
 * integer activations the layer is evaluated as sum s * (x << e), the common
 * factor 2^-7 belongs to the de-quantisation scale.  int64 accumulation;
 * returns the number of outputs that do not fit int32 (0 in every test).
 * ------------------------------------------------------------------------ */
long oracle_shift_linear(const int8_t *x, const uint8_t *w4, const int32_t *bias, int32_t *y,
                         long M, int K, int N) {
    long overflow = 0;
#pragma omp parallel for reduction(+ : overflow)
    for (long m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            int64_t acc = bias ? (int64_t)bias[n] : 0;
            for (int k = 0; k < K; ++k) {
                const uint8_t byte = w4[(size_t)n * (K / 2) + (k >> 1)];
                const int nib = (k & 1) ? (byte >> 4) : (byte & 15);
                const int64_t mag = (int64_t)1 << (nib & 7);
                const int64_t wgt = (nib & 8) ? -mag : mag;
                acc += (int64_t)x[(size_t)m * K + k] * wgt;
            }
            if (acc > INT32_MAX || acc < INT32_MIN) ++overflow;
            y[(size_t)m * N + n] = (int32_t)acc;
        }
    return overflow;
}

/* ------------------------------------------------------------------------
 * Activation quantisation, per-tensor symmetric with a static scale that is
 * passed in (appendix "scaling factor clarification", integer-arithmetic
 * quantisation).  One fp32 multiply, one round-to-nearest-even, clamp:
 *   q = clamp(rne(x * inv_scale), -127, 127),   NaN -> 0
 * ------------------------------------------------------------------------ */
static inline int8_t clamp_rne_i8(float t) {
    if (t != t) return 0;
    t = nearbyintf(t);                 /* default rounding mode = to nearest even */
    if (t < -127.0f) t = -127.0f;
    if (t > 127.0f) t = 127.0f;
    return (int8_t)t;
}

void oracle_quantize_act(const float *x, long n, float inv_scale, int8_t *q) {
    for (long i = 0; i < n; ++i) {
        volatile float t = x[i] * inv_scale;   /* keep the fp32 product rounded once */
        q[i] = clamp_rne_i8(t);
    }
}

/* ------------------------------------------------------------------------
 * Between the two shift linears of the Shift expert: int32 accumulator ->
 * int8 by a static scale, then a 256-entry int8 -> int8 activation table
 * (the paper names no activation for the Shift expert; a table keeps the
 * expert integer-only and exact).
 *   h = lut[clamp(rne(float(y) * s), -127, 127) + 128]
 * ------------------------------------------------------------------------ */
void oracle_requant_lut(const int32_t *y, long n, float s, const int8_t *lut, int8_t *h) {
    for (long i = 0; i < n; ++i) {
        volatile float f = (float)y[i];
        volatile float t = f * s;
        h[i] = lut[(int)clamp_rne_i8(t) + 128];
    }
}

/* ------------------------------------------------------------------------
 * Top-1 routing between the Mult expert (0) and the Shift expert (1)
 * (Sec. 4.2: p = softmax(router logits); G(x) = p_i * 1{p_i >= p_j for all j}).
 * The decision is taken on the raw logits (softmax is monotone); a tie goes
 * to the lowest index.  gate = the winner's softmax probability.  No
 * capacity limit, no dropped token.  perm lists expert 0's tokens in
 * ascending order, then expert 1's, and so on.
 * ------------------------------------------------------------------------ */
void oracle_moe_dispatch(const float *logits, long T, int E, int32_t *perm, int32_t *expert_of,
                         int32_t *counts, double *gate) {
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (long t = 0; t < T; ++t) {
        const float *l = logits + (size_t)t * E;
        int best = 0;
        for (int e = 1; e < E; ++e)
            if (l[e] > l[best]) best = e;
        double den = 0.0;
        for (int e = 0; e < E; ++e) den += exp((double)l[e] - (double)l[best]);
        gate[t] = 1.0 / den;
        expert_of[t] = best;
        counts[best] += 1;
    }
    long pos = 0;
    for (int e = 0; e < E; ++e)
        for (long t = 0; t < T; ++t)
            if (expert_of[t] == e) perm[pos++] = (int32_t)t;
}

/* ---- fp16 rounding written out (IEEE binary16, round to nearest even) ---- */
static double round_to_half(double x) {
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int ex;
    frexp(fabs(x), &ex);               /* |x| = f * 2^ex, f in [0.5,1) */
    int e = ex - 1;                    /* |x| in [2^e, 2^(e+1)) */
    if (e < -14) e = -14;              /* subnormal spacing 2^-24 */
    const double ulp = ldexp(1.0, e - 10);
    double r = nearbyint(x / ulp) * ulp;
    if (fabs(r) > 65504.0) r = (x > 0) ? INFINITY : -INFINITY;
    return r;
}

void oracle_round_to_half(const double *x, long n, double *r) {
    for (long i = 0; i < n; ++i) r[i] = round_to_half(x[i]);
}

static double half_bits_to_double(uint16_t h) {
    const int sign = h >> 15, ex = (h >> 10) & 31, man = h & 1023;
    double v;
    if (ex == 0) v = ldexp((double)man, -24);
    else if (ex == 31) v = man ? NAN : INFINITY;
    else v = ldexp(1.0 + man / 1024.0, ex - 15);
    return sign ? -v : v;
}

/* ------------------------------------------------------------------------
 * Mult expert: an ordinary two-layer MLP with GELU (Sec. 4.2, the Mult.
 * expert; GELU is the ViT default, the paper names no other).  Operands are
 * fp16: the input rows and the hidden activation are rounded to fp16 where
 * the fp16 kernel rounds them; sums are fp64.
 *   y = W2 * half(gelu(W1 * half(x)))         W1 [hid,E], W2 [E,hid]
 * rows: indices of the input rows to process (NULL = 0..n_rows-1).
 * ------------------------------------------------------------------------ */
void oracle_mult_mlp(const float *x, const int32_t *rows, long n_rows, int E, int hid,
                     const uint16_t *w1_half, const uint16_t *w2_half, double *y) {
    double *W1 = (double *)malloc(sizeof(double) * (size_t)hid * E);
    double *W2 = (double *)malloc(sizeof(double) * (size_t)E * hid);
    for (size_t i = 0; i < (size_t)hid * E; ++i) W1[i] = half_bits_to_double(w1_half[i]);
    for (size_t i = 0; i < (size_t)E * hid; ++i) W2[i] = half_bits_to_double(w2_half[i]);
#pragma omp parallel
    {
        double *xh = (double *)malloc(sizeof(double) * (size_t)E);
        double *hh = (double *)malloc(sizeof(double) * (size_t)hid);
#pragma omp for
        for (long r = 0; r < n_rows; ++r) {
            const float *xr = x + (size_t)(rows ? rows[r] : r) * E;
            for (int k = 0; k < E; ++k) xh[k] = round_to_half((double)xr[k]);
            for (int j = 0; j < hid; ++j) {
                double acc = 0.0;
                for (int k = 0; k < E; ++k) acc += W1[(size_t)j * E + k] * xh[k];
                hh[j] = round_to_half(0.5 * acc * (1.0 + erf(acc / sqrt(2.0))));
            }
            for (int n = 0; n < E; ++n) {
                double acc = 0.0;
                for (int j = 0; j < hid; ++j) acc += W2[(size_t)n * hid + j] * hh[j];
                y[(size_t)r * E + n] = acc;
            }
        }
        free(xh);
        free(hh);
    }
    free(W1);
    free(W2);
}

/* ------------------------------------------------------------------------
 * Combine (Sec. 4.2: y = sum_i G(x) * E_i(x), one non-zero term per token).
 *   y[perm[i], :] = gate[perm[i]] * expert_out[i, :]
 * expert_out rows follow perm order (expert 0's rows first).
 * ------------------------------------------------------------------------ */
void oracle_combine(const double *expert_out, const int32_t *perm, const double *gate, long T,
                    int E, double *y) {
    for (long i = 0; i < T; ++i) {
        const long t = perm[i];
        for (int c = 0; c < E; ++c) y[(size_t)t * E + c] = gate[t] * expert_out[(size_t)i * E + c];
    }
}

/* ------------------------------------------------------------------------
 * The remaining pieces of the block of Eq. 2: LayerNorm, the four attention
 * Linears as shift layers (Sec. 4.1: the Linears of the attention module are
 * reparameterised with sign flips and power-of-two shifts), the residual sums
 * and the router G (Sec. 4.2).
 * ------------------------------------------------------------------------ */

/* LayerNorm over the last dimension (Eq. 2), fp64 from fp32 inputs:
 *   y = (x - mean) / sqrt(var + eps) * gamma + beta,  var = mean((x - mean)^2). */
void oracle_layernorm(const float *x, long T, int E, const float *gamma, const float *beta,
                      double eps, double *y) {
#pragma omp parallel for
    for (long t = 0; t < T; ++t) {
        const float *row = x + (size_t)t * E;
        double mean = 0.0, var = 0.0;
        for (int j = 0; j < E; ++j) mean += (double)row[j];
        mean /= (double)E;
        for (int j = 0; j < E; ++j) {
            const double c = (double)row[j] - mean;
            var += c * c;
        }
        var /= (double)E;
        const double rstd = 1.0 / sqrt(var + eps);
        for (int j = 0; j < E; ++j)
            y[(size_t)t * E + j] = ((double)row[j] - mean) * rstd * (double)gamma[j] + (double)beta[j];
    }
}

/* Output side of a shift Linear that feeds fp32 consumers (Q, K, V; the output
 * projection with its residual, Eq. 2).  The integer accumulator of Eq. 3 is
 * exact; its real value is acc * scale (the common power of two of the weights
 * and the activation scale folded into one factor).  The paper does not say
 * how the factor is applied; the reading taken is one fused multiply-add in
 * fp32 with the int32 converted round-to-nearest-even first:
 *   y = fmaf((float)acc, scale, residual)       (residual = 0 when absent)
 * which both sides can follow to the bit. */
void oracle_dequant_residual(const int32_t *acc, long n, float scale, const float *residual,
                             float *y) {
#pragma omp parallel for
    for (long i = 0; i < n; ++i)
        y[i] = fmaf((float)acc[i], scale, residual ? residual[i] : 0.0f);
}

/* Router (Sec. 4.2, the gate G over the experts): logits = z Wg + bg in fp64;
 * z [T, E] fp64, Wg [E, n_exp] fp32, bg [n_exp] fp32. */
void oracle_router_logits(const double *z, long T, int E, const float *wg, const float *bg,
                          int n_exp, double *logits) {
#pragma omp parallel for
    for (long t = 0; t < T; ++t)
        for (int e = 0; e < n_exp; ++e) {
            double s = 0.0;
            for (int j = 0; j < E; ++j) s += z[(size_t)t * E + j] * (double)wg[(size_t)j * n_exp + e];
            logits[(size_t)t * n_exp + e] = s + (double)bg[e];
        }
}

/* ------------------------------------------------------------------------
 * Dense weights -> shift weights (Sec. 4.1, below Eq. 3): s = sign(W) in
 * {-1, +1}, P = round(log2 |W|).  Stored as the nibble (neg << 3) | (P + 7)
 * with P clamped to [-7, 0] (weights in [-1, 1]); sign(0) = +1; W = 0 has
 * log2 = -inf and takes P = -7; NaN is treated as +1.0.  log2 |W| = n + 1/2
 * would need |W| = 2^n * sqrt(2), which no float is, so the rounding rule at
 * one half never applies and fp64 log2 decides every fp32 input correctly (the
 * nearest floats to 2^n * sqrt(2) are 1e-8 away in log2).
 * ------------------------------------------------------------------------ */
void oracle_shift_weights_from_float(const float *w, long N, int K, uint8_t *w4) {
#pragma omp parallel for
    for (long n = 0; n < N; ++n)
        for (int k = 0; k < K; k += 2) {
            uint8_t byte = 0;
            for (int i = 0; i < 2; ++i) {
                const double a = fabs((double)w[(size_t)n * K + k + i]);
                double p;
                if (a != a) p = 0.0;
                else if (a == 0.0) p = -7.0;
                else p = nearbyint(log2(a));
                if (p < -7.0) p = -7.0;
                if (p > 0.0) p = 0.0;
                const int neg = w[(size_t)n * K + k + i] < 0.0f;
                byte |= (uint8_t)(((neg << 3) | ((int)p + 7)) << (4 * i));
            }
            w4[(size_t)n * (K / 2) + k / 2] = byte;
        }
}

/* ------------------------------------------------------------------------
 * Linear attention on {0,1} codes with its row normaliser, and the depthwise
 * convolution on the V branch (Sec. 4.1: the Add layer of Eq. 3 accumulates
 * where the binary weight is non-zero and skips zeros; the attention is built
 * on kernel-based linear attention, Q(K^T V), with a light depthwise
 * convolution on V in parallel; Sec. 5 names the normalisation among the extra
 * operations of linear attention).  The paper prints neither formula; the
 * reading taken is the standard kernel-based form with the code bits c in
 * {0,1} as the feature map:
 *   KV[j,:]  = sum_n cK[n,j] * V[n,:]          ksum[j] = sum_n cK[n,j]
 *   O[n,:]   = (sum_j cQ[n,j] * KV[j,:]) / (sum_j cQ[n,j] * ksum[j] + eps)
 * The denominator is an integer count (plus eps), exact on both sides.
 * ------------------------------------------------------------------------ */
void oracle_ktv01(const uint64_t *k_codes, const float *v, int B, int H, int Nk, int nbits, int dv,
                  double *kv, int64_t *ksum) {
    const int W = nbits / 64;
#pragma omp parallel for collapse(2)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h)
            for (int j = 0; j < nbits; ++j) {
                double *row = kv + (((size_t)b * H + h) * nbits + j) * dv;
                for (int c = 0; c < dv; ++c) row[c] = 0.0;
                int64_t cnt = 0;
                for (int n = 0; n < Nk; ++n) {
                    const uint64_t *code = k_codes + (((size_t)b * H + h) * Nk + n) * W;
                    if (!code_bit(code, j)) continue;            /* zeros are skipped */
                    ++cnt;
                    const float *vr = v + (((size_t)b * Nk + n) * H + h) * dv;
                    for (int c = 0; c < dv; ++c) row[c] += (double)vr[c];
                }
                ksum[((size_t)b * H + h) * nbits + j] = cnt;
            }
}

void oracle_qkv01(const uint64_t *q_codes, const double *kv, const int64_t *ksum, int B, int H, int Nq,
                  int nbits, int dv, double eps, double *out, int64_t *den_out) {
    const int W = nbits / 64;
#pragma omp parallel for collapse(2)
    for (int b = 0; b < B; ++b)
        for (int n = 0; n < Nq; ++n)
            for (int h = 0; h < H; ++h) {
                const uint64_t *code = q_codes + (((size_t)b * H + h) * Nq + n) * W;
                double *o = out + (((size_t)b * Nq + n) * H + h) * dv;
                for (int c = 0; c < dv; ++c) o[c] = 0.0;
                int64_t den = 0;
                for (int j = 0; j < nbits; ++j) {
                    if (!code_bit(code, j)) continue;
                    den += ksum[((size_t)b * H + h) * nbits + j];
                    const double *row = kv + (((size_t)b * H + h) * nbits + j) * dv;
                    for (int c = 0; c < dv; ++c) o[c] += row[c];
                }
                for (int c = 0; c < dv; ++c) o[c] /= ((double)den + eps);
                if (den_out) den_out[((size_t)b * H + h) * Nq + n] = den;
            }
}

/* Depthwise 3x3 convolution over the token grid, stride 1, zero padding 1
 * (the "lightweight DWConv on the V branch", Sec. 4.1), added by the caller to
 * the attention output.  v, out: [B, gh, gw, E] (tokens row-major over the
 * grid, channels = heads x dv inner); w: [E, 3, 3] (w[c][dy+1][dx+1] applies to
 * the neighbour at (y+dy, x+dx)); bias: [E] or NULL. */
void oracle_dwconv3x3(const float *v, const float *w, const float *bias, int B, int gh, int gw, int E,
                      double *out) {
#pragma omp parallel for collapse(2)
    for (int b = 0; b < B; ++b)
        for (int y = 0; y < gh; ++y)
            for (int x = 0; x < gw; ++x)
                for (int c = 0; c < E; ++c) {
                    double s = bias ? (double)bias[c] : 0.0;
                    for (int dy = -1; dy <= 1; ++dy)
                        for (int dx = -1; dx <= 1; ++dx) {
                            const int yy = y + dy, xx = x + dx;
                            if (yy < 0 || yy >= gh || xx < 0 || xx >= gw) continue;
                            s += (double)w[(size_t)c * 9 + (dy + 1) * 3 + (dx + 1)] *
                                 (double)v[(((size_t)b * gh + yy) * gw + xx) * E + c];
                        }
                    out[(((size_t)b * gh + y) * gw + x) * E + c] = s;
                }
}

/* ------------------------------------------------------------------------
 * Forward value of the latency-aware load-balancing loss (Eq. 4):
 *   IMP_i  = alpha_i * sum_x p_i(x),     p = softmax(logits(x))
 *   LOAD_i = alpha_i * sum_x q_i(x),     q_i(x) = P(p_i(x) + eps >= p_j(x) for all j != i)
 *   L_IMP = SCV(IMP),  L_LOAD = SCV(LOAD),  SCV(u) = var(u) / mean(u)^2 over the experts
 * The paper calls eps a noise proxy and gives no distribution; the reading
 * taken is eps ~ N(0, noise_std^2) added to p_i alone, so
 *   q_i(x) = Phi((p_i(x) - max_{j != i} p_j(x)) / noise_std)
 * (Phi = standard normal distribution function), and the population variance
 * (divide by the number of experts) in SCV.  sums: [2 * E] = IMP then LOAD.
 * ------------------------------------------------------------------------ */
void oracle_moe_balance_loss(const float *logits, long T, int E, const float *alpha, double noise_std,
                             double *losses, double *sums) {
    for (int i = 0; i < 2 * E; ++i) sums[i] = 0.0;
    for (long t = 0; t < T; ++t) {
        const float *l = logits + (size_t)t * E;
        double p[64], mx = (double)l[0], den = 0.0;
        for (int e = 1; e < E; ++e) if ((double)l[e] > mx) mx = (double)l[e];
        for (int e = 0; e < E; ++e) { p[e] = exp((double)l[e] - mx); den += p[e]; }
        for (int e = 0; e < E; ++e) p[e] /= den;
        for (int e = 0; e < E; ++e) {
            double other = -1.0;
            for (int j = 0; j < E; ++j) if (j != e && p[j] > other) other = p[j];
            const double z = (p[e] - other) / noise_std;
            sums[e] += p[e];
            sums[E + e] += 0.5 * erfc(-z / sqrt(2.0));
        }
    }
    for (int k = 0; k < 2; ++k) {
        double mean = 0.0, var = 0.0;
        for (int e = 0; e < E; ++e) { sums[k * E + e] *= (double)alpha[e]; mean += sums[k * E + e]; }
        mean /= (double)E;
        for (int e = 0; e < E; ++e) { const double c = sums[k * E + e] - mean; var += c * c; }
        var /= (double)E;
        losses[k] = var / (mean * mean);
    }
}
