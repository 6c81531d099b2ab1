/* Runs every function of the CPU oracle on small, ragged inputs whose buffers are exactly as large as the
 * function's contract says, under AddressSanitizer and UndefinedBehaviorSanitizer (built by
 * tests/test_sanitizers.py).  A read or write past a buffer, a signed overflow or a misaligned access stops the
 * program with a report; a clean run prints "oracle driver ok".  Test infrastructure only. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void oracle_binarize(const float *, int, int, int, int, const float *, int, uint64_t *);
void oracle_ktv(const uint64_t *, const float *, int, int, int, int, int, double *);
void oracle_qkv(const uint64_t *, const double *, int, int, int, int, int, float, double *);
void oracle_hamming_scores(const uint64_t *, const uint64_t *, int, int, int, int, int, int16_t *);
void oracle_hamming_attention(const uint64_t *, const uint64_t *, const float *, int, int, int, int, int, int, float, double *);
long oracle_shift_linear(const int8_t *, const uint8_t *, const int32_t *, int32_t *, long, int, int);
void oracle_quantize_act(const float *, long, float, int8_t *);
void oracle_requant_lut(const int32_t *, long, float, const int8_t *, int8_t *);
void oracle_moe_dispatch(const float *, long, int, int32_t *, int32_t *, int32_t *, double *);
void oracle_round_to_half(const double *, long, double *);
void oracle_mult_mlp(const float *, const int32_t *, long, int, int, const uint16_t *, const uint16_t *, double *);
void oracle_combine(const double *, const int32_t *, const double *, long, int, double *);
void oracle_layernorm(const float *, long, int, const float *, const float *, double, double *);
void oracle_dequant_residual(const int32_t *, long, float, const float *, float *);
void oracle_router_logits(const double *, long, int, const float *, const float *, int, double *);
void oracle_shift_weights_from_float(const float *, long, int, uint8_t *);
void oracle_ktv01(const uint64_t *, const float *, int, int, int, int, int, double *, int64_t *);
void oracle_qkv01(const uint64_t *, const double *, const int64_t *, int, int, int, int, int, double, double *, int64_t *);
void oracle_dwconv3x3(const float *, const float *, const float *, int, int, int, int, double *);
void oracle_moe_balance_loss(const float *, long, int, const float *, double, double *, double *);

static uint32_t state = 2463534242u;
static uint32_t rnd(void) { state ^= state << 13; state ^= state >> 17; state ^= state << 5; return state; }
static float frand(void) { return (float)((int)(rnd() % 2001) - 1000) / 500.0f; }

/* exact-size heap buffers: the sanitizer sees every byte past the end */
static void *owned[256];
static int n_owned = 0;
static void *buf(size_t bytes) {
    void *p = malloc(bytes ? bytes : 1);
    if (!p || n_owned == 256) exit(2);
    memset(p, 0, bytes);
    owned[n_owned++] = p;
    return p;
}
static float *fbuf(size_t n) { float *p = buf(n * sizeof(float)); for (size_t i = 0; i < n; ++i) p[i] = frand(); return p; }

int main(void) {
    /* attention: B 2, N 5 queries / 7 keys, H 3, d 32 -> 128-bit codes, dv 8 */
    const int B = 2, H = 3, Nq = 5, Nk = 7, d = 32, nbits = 128, dv = 8, W = nbits / 64;
    float *q = fbuf((size_t)B * Nq * H * d), *k = fbuf((size_t)B * Nk * H * d), *proj = fbuf((size_t)d * nbits);
    float *v = fbuf((size_t)B * Nk * H * dv);
    uint64_t *qc = buf(sizeof(uint64_t) * B * H * Nq * W), *kc = buf(sizeof(uint64_t) * B * H * Nk * W);
    oracle_binarize(q, B, Nq, H, d, proj, nbits, qc);
    oracle_binarize(k, B, Nk, H, d, proj, nbits, kc);
    float *x64 = fbuf((size_t)1 * 3 * 2 * 64);
    x64[5] = -0.0f; x64[6] = NAN; x64[7] = INFINITY;
    uint64_t *c64 = buf(sizeof(uint64_t) * 1 * 2 * 3 * 1);
    oracle_binarize(x64, 1, 3, 2, 64, NULL, 64, c64);               /* sign hash, no projection */
    double *kv = buf(sizeof(double) * B * H * nbits * dv), *o = buf(sizeof(double) * B * Nq * H * dv);
    oracle_ktv(kc, v, B, H, Nk, nbits, dv, kv);
    oracle_qkv(qc, kv, B, H, Nq, nbits, dv, 0.125f, o);
    int16_t *sc = buf(sizeof(int16_t) * B * H * Nq * Nk);
    oracle_hamming_scores(qc, kc, B, H, Nq, Nk, nbits, sc);
    oracle_hamming_attention(qc, kc, v, B, H, Nq, Nk, nbits, dv, 0.09f, o);
    oracle_hamming_attention(qc, kc, v, B, H, Nq, 1, nbits, dv, -3.0f, o);        /* one key, negative scale */
    int64_t *ksum = buf(sizeof(int64_t) * B * H * nbits), *den = buf(sizeof(int64_t) * B * H * Nq);
    oracle_ktv01(kc, v, B, H, Nk, nbits, dv, kv, ksum);
    oracle_qkv01(qc, kv, ksum, B, H, Nq, nbits, dv, 1e-6, o, den);
    float *img = fbuf((size_t)2 * 3 * 4 * 6), *cw = fbuf(6 * 9), *cb = fbuf(6);
    double *co = buf(sizeof(double) * 2 * 3 * 4 * 6);
    oracle_dwconv3x3(img, cw, cb, 2, 3, 4, 6, co);
    oracle_dwconv3x3(img, cw, NULL, 2 * 3 * 4, 1, 1, 6, co);                     /* 1 x 1 grids */

    /* shift layers: M 5, K 34 (odd number of bytes per row), N 3, extremes included */
    const long M = 5; const int K = 34, N = 3;
    int8_t *x8 = buf((size_t)M * K);
    for (long i = 0; i < M * K; ++i) x8[i] = (int8_t)((int)(rnd() % 255) - 127);
    uint8_t *w4 = buf((size_t)N * K / 2);
    for (int i = 0; i < N * K / 2; ++i) w4[i] = (uint8_t)rnd();
    int32_t *bias = buf(sizeof(int32_t) * N), *y32 = buf(sizeof(int32_t) * M * N);
    bias[0] = 2147483000; bias[1] = -2147483000;                                  /* near the int32 ends: counted, not wrapped */
    long ovf = oracle_shift_linear(x8, w4, bias, y32, M, K, N);
    (void)ovf;
    oracle_shift_linear(x8, w4, NULL, y32, M, K, N);
    int8_t *big = buf(3072); memset(big, 127, 3072);
    uint8_t *wmax = buf(1536); memset(wmax, 0x77, 1536);
    if (oracle_shift_linear(big, wmax, NULL, y32, 1, 3072, 1) != 0 || y32[0] != 127 * 128 * 3072) return 3;
    float edge[8] = {0.5f, 1.5f, -2.5f, 1e30f, -1e30f, NAN, INFINITY, -INFINITY};
    int8_t q8[8];
    oracle_quantize_act(edge, 8, 1.0f, q8);
    int32_t acc[6] = {0, 1, -1, 2147483647, -2147483647 - 1, 123456};
    int8_t lut[256], h8[6];
    for (int i = 0; i < 256; ++i) lut[i] = (int8_t)(i - 128);
    oracle_requant_lut(acc, 6, 1.0f / 32.0f, lut, h8);
    oracle_requant_lut(acc, 6, INFINITY, lut, h8);
    float resid[6] = {1, 2, 3, 4, 5, 6}, yq[6];
    oracle_dequant_residual(acc, 6, 3.0e-5f, resid, yq);
    oracle_dequant_residual(acc, 6, 3.0e-5f, NULL, yq);
    float wf[2 * 8] = {0.0f, -0.0f, 1.0f, -1.0f, 1e-30f, 3.0f, NAN, INFINITY, 0.3f, -0.3f, 0.7f, 0.71f, 0.0078125f, 0.004f, -0.5f, 0.25f};
    uint8_t w4f[2 * 4];
    oracle_shift_weights_from_float(wf, 2, 8, w4f);

    /* routing and experts: T 9 tokens, E 3 experts with ties; Mult expert E 6 -> hid 10 */
    const long T = 9;
    float *lg = fbuf(T * 3);
    lg[3] = lg[4] = lg[5];                                                        /* a three-way tie */
    int32_t *perm = buf(sizeof(int32_t) * T), *eo = buf(sizeof(int32_t) * T), cnt[3];
    double *gate = buf(sizeof(double) * T);
    oracle_moe_dispatch(lg, T, 3, perm, eo, cnt, gate);
    float alpha[3] = {0.5f, 0.3f, 0.2f};
    double losses[2], sums[6];
    oracle_moe_balance_loss(lg, T, 3, alpha, 0.05, losses, sums);
    double hv[5] = {0.0, 65504.0, 65520.0, 1e-8, -1.0 / 3.0}, hr[5];
    oracle_round_to_half(hv, 5, hr);
    const int E = 6, hid = 10;
    float *xm = fbuf(T * E);
    uint16_t *mw1 = buf(sizeof(uint16_t) * hid * E), *mw2 = buf(sizeof(uint16_t) * E * hid);
    for (int i = 0; i < hid * E; ++i) { mw1[i] = (uint16_t)(0x3000 + rnd() % 0x800); mw2[i] = (uint16_t)(0xB000 + rnd() % 0x800); }
    int32_t rows[4] = {8, 0, 3, 3};
    double *ym = buf(sizeof(double) * 4 * E), *yall = buf(sizeof(double) * T * E), *yc = buf(sizeof(double) * T * E);
    oracle_mult_mlp(xm, rows, 4, E, hid, mw1, mw2, ym);
    oracle_mult_mlp(xm, NULL, T, E, hid, mw1, mw2, yall);
    oracle_combine(yall, perm, gate, T, E, yc);
    float *gamma = fbuf(E), *beta = fbuf(E);
    double *ln = buf(sizeof(double) * T * E), *rl = buf(sizeof(double) * T * 3);
    oracle_layernorm(xm, T, E, gamma, beta, 1e-6, ln);
    float *wg = fbuf(E * 3), bg[3] = {0.1f, -0.2f, 0.0f};
    oracle_router_logits(ln, T, E, wg, bg, 3, rl);
    for (long i = 0; i < T * E; ++i) if (!isfinite(yc[i]) || !isfinite(ln[i])) return 4;
    while (n_owned > 0) free(owned[--n_owned]);       /* what is still allocated now is a leak inside the oracle */
    puts("oracle driver ok");
    return 0;
}
