/*
 * libshiftadd - the reparameterised transformer block of ShiftAddViT
 * (arXiv 2306.06446) as hand-written HIP kernels for AMD gfx950 (MI355X).
 *
 * C ABI.  Every pointer named below is a DEVICE pointer unless it says
 * "host".  The caller owns every buffer; the library never allocates, frees
 * or keeps a pointer, and never synchronises: all work is enqueued on the
 * caller's stream (a hipStream_t passed as void*, NULL = the default stream).
 * Scratch memory comes from a caller-provided workspace whose size the
 * matching *_workspace_bytes query returns.  Arguments are validated on the
 * host before anything is launched, so error paths never touch the GPU.
 *
 * Every entry point returns SA_OK or a negative SA_ERR_* code; a text for the
 * most recent error of the calling thread is available from sa_last_error().
 * All device pointers must be 16-byte aligned (SA_ERR_ALIGN otherwise); row-id
 * lists need 4-byte alignment only.
 *
 * Storage formats
 *   code words  uint64 [B, H, N, W], W = nbits / 64; bit j of a code is bit
 *               (j % 64) of word (j / 64), least significant bit first.
 *               Bit 1 stands for +1, bit 0 for -1.
 *   activations fp32 [B, N, H, d] (token-major, heads inner), so that
 *               [B, N, H, dv] is also the [T, E] matrix of the MLP, T = B*N,
 *               E = H*dv.
 *   shift weight 4 bits: (neg << 3) | e, the weight is (neg ? -1 : +1) * 2^e,
 *               e = P + 7 for the paper's exponent P in [-7, 0]; row n of a
 *               layer holds K/2 bytes, even k in the low nibble.
 */
#ifndef SHIFTADD_H_
#define SHIFTADD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SA_OK 0
#define SA_ERR_INVALID (-1)     /* null pointer, negative size, bad enum value        */
#define SA_ERR_SHAPE (-2)       /* a size the operation is not defined for            */
#define SA_ERR_ALIGN (-3)       /* a pointer that is not 16-byte aligned              */
#define SA_ERR_WORKSPACE (-4)   /* workspace missing or smaller than the query says   */
#define SA_ERR_HIP (-5)         /* the HIP runtime refused a launch                   */
#define SA_ERR_UNSUPPORTED (-6) /* defined, but no kernel is built for this size      */

#define SA_VARIANT_VALU 0 /* shift-and-accumulate on the vector ALU                   */
#define SA_VARIANT_MFMA 1 /* 4-bit weights decoded to int8, int8 matrix cores         */
#define SA_VARIANT_AUTO 2 /* the faster of the two for the shape                      */
#define SA_VARIANT_MFMA_PREPARED 3 /* shift layers only: as MFMA, but the weight pointers
                                      hold planes made by sa_shift_planes_prepare         */

/*
 * Measurement helper, not a step of the path: a register-only loop of matrix instructions (no memory
 * traffic), 4 wavefronts per workgroup, 8 * iters instructions per wavefront, so that a caller can
 * read off the instruction rate and the shader clock the matrix cores sustain (the peaks the roofline
 * of this library is priced against are the published ones; this shows what part of them is reachable).
 *   kind      0 = int8 32x32x32 (65536 operations each), 1 = fp16 32x32x16, 2 = bf16 32x32x16 (32768)
 *   operands  0 = one non-zero element per register, 1 = random bits, 2 = (int8) random activations
 *             against powers of two and a plane that is 7/8 zeros, as in a Shift layer
 *   out       device memory, 3 x uint64, 16-byte aligned: [0] shader cycles and [1] ticks of the 100 MHz
 *             wall clock that the loop of workgroup 0 took ([2] is scratch)
 * The caller times the launch (events on `stream`) for the rate.
 */
int sa_probe_mfma(int kind, int operands, int workgroups, int iters, unsigned long long *out,
                  void *stream);

int sa_version(void);
/* Host string describing the last error returned on this thread ("" if none). */
const char *sa_last_error(void);

/*
 * Hash rows of Q or K to packed binary codes (Sec. 4.1, binary quantisation
 * of Q and K; appendix, "scaling factor clarification": vanilla sign
 * quantisation or a set of hash functions).
 *   proj == NULL : bit j = [x_j >= 0], requires nbits == d
 *   proj != NULL : bit j = [sum_k x_k * proj[k][j] >= 0], proj fp32 [d, nbits]
 * The sum is the fp32 chain acc = fma(x_k, proj[k][j], acc), k ascending from
 * +0.0f; results are bit-exact with that definition.
 *   x [B,N,H,d] fp32 in;  codes [B,H,N,nbits/64] uint64 out.
 * nbits % 64 == 0; with proj, d in {32, 64, 128}; without, d % 64 == 0.
 */
int sa_binarize(const float *x, int B, int N, int H, int d, const float *proj, int nbits,
                uint64_t *codes, void *stream);
/* The same with the kernel chosen by hand (both give the same bits):
 *   SA_VARIANT_VALU  every bit through the defining chain on the vector ALU
 *   SA_VARIANT_MFMA  matrix-core pre-pass; bits whose sign it cannot settle (a rigorous
 *                    margin test) are re-run through the defining chain
 *   SA_VARIANT_AUTO  what sa_binarize uses                                          */
int sa_binarize_ex(const float *x, int B, int N, int H, int d, const float *proj, int nbits,
                   uint64_t *codes, int variant, void *stream);
/* Q and K of one block: two tensors of the same shape through the same hash, in one launch
 * where the matrix-core kernel takes the shape (otherwise the same as two sa_binarize calls). */
int sa_binarize_pair(const float *q, const float *k, int B, int N, int H, int d, const float *proj,
                     int nbits, uint64_t *q_codes, uint64_t *k_codes, void *stream);

/*
 * Linear attention with both MatMuls as Add layers (Eq. 3, O_Add; Sec. 4.1,
 * order (QK)V -> Q(KV); appendix: the scale is applied after the adds).
 *   phase 1:  kv[b,h,j,:]  = sum_n sigma(k_codes[b,h,n,j]) * v[b,n,h,:]
 *   phase 2:  out[b,n,h,:] = scale * sum_j sigma(q_codes[b,h,n,j]) * kv[b,h,j,:]
 * phases: 1 = phase 1 only, 2 = phase 2 only (kv is an input), 3 = both.
 *   q_codes [B,H,Nq,W], k_codes [B,H,Nk,W], v [B,Nk,H,dv], out [B,Nq,H,dv],
 *   kv [B,H,nbits,dv] fp32.  dv in {32, 64, 128}.
 * Sums are fp32, in a fixed order (results are reproducible run to run).
 * Both phases run on the matrix cores (the +-1 operand against the three exact bf16 term
 * planes of the fp32 operand: the same sums); adding SA_ADDITIVE_VALU to `phases` runs the
 * sign-select-and-accumulate kernels on the vector ALU instead.
 */
#define SA_ADDITIVE_VALU 4
size_t sa_additive_attention_workspace_bytes(int B, int H, int Nk, int nbits, int dv);
int sa_additive_attention(const uint64_t *q_codes, const uint64_t *k_codes, const float *v,
                          float *out, int B, int H, int Nq, int Nk, int nbits, int dv,
                          float scale, float *kv, int phases, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * Linear attention on {0,1} codes with its row normaliser (Eq. 3: the Add
 * layer accumulates where the binary weight is non-zero and skips zeros;
 * Sec. 4.1: kernel-based linear attention in the order Q(K^T V)).  A set code
 * bit stands for 1, a clear bit for 0:
 *   phase 1:  kv[b,h,j,:] = sum_n cK[n,j] * v[b,n,h,:]      fp32 [B,H,nbits,dv]
 *             ksum[b,h,j] = sum_n cK[n,j]                   int32 [B,H,nbits]
 *   phase 2:  out[b,n,h,:] = (sum_j cQ[n,j] * kv[b,h,j,:]) / (sum_j cQ[n,j] * ksum[b,h,j] + eps)
 * phases 1, 2 or 3 (| SA_ADDITIVE_VALU as for sa_additive_attention); eps > 0
 * (a query whose set bits meet no key bit gives 0 / eps = 0).  The normaliser
 * is an exact integer; Nk * nbits < 2^31.  dv in {32, 64, 128}.
 */
size_t sa_linear_attention_01_workspace_bytes(int B, int H, int Nq, int Nk, int nbits, int dv);
int sa_linear_attention_01(const uint64_t *q_codes, const uint64_t *k_codes, const float *v, float *out,
                           int B, int H, int Nq, int Nk, int nbits, int dv, float eps, float *kv,
                           int32_t *ksum, int phases, void *workspace, size_t workspace_bytes,
                           void *stream);

/*
 * Depthwise 3x3 convolution over the token grid of the V branch (Sec. 4.1: a
 * light depthwise convolution on V in parallel to the attention), stride 1,
 * zero padding:  v, out fp32 [B, gh, gw, E] (tokens row-major over the grid,
 * E = H * dv channels inner, i.e. V's own [B,N,H,dv] with N = gh * gw),
 * w fp32 [E, 3, 3] (w[c][dy+1][dx+1] weighs the neighbour at (y+dy, x+dx)),
 * bias fp32 [E] or NULL.  accumulate != 0 adds the result to out (the sum with
 * the attention output), else out is overwritten.  E % 4 == 0; out != v.
 */
int sa_dwconv3x3(const float *v, const float *w, const float *bias_or_null, float *out, int accumulate,
                 int B, int gh, int gw, int E, void *stream);

/*
 * Quadratic attention on codes (Eq. 1 with Q K^T replaced by the Hamming
 * similarity S[i,j] = nbits - 2 * popcount(q_i xor k_j) of the codes):
 *   out[b,i,h,:] = sum_j softmax_j(scale * S[i,j]) * v[b,j,h,:]
 * scores_or_null: if not NULL, S is also written as int16 [B,H,Nq,Nk]
 * (bit-exact).  dv in {32, 64, 128}; fp32 softmax and accumulation.
 */
int sa_hamming_attention(const uint64_t *q_codes, const uint64_t *k_codes, const float *v,
                         float *out, int B, int H, int Nq, int Nk, int nbits, int dv,
                         float scale, int16_t *scores_or_null, void *stream);
/* The same, with the attention output also written in the two forms the MLP of the block
 * reads (Eq. 2 feeds the attention output to the MLP): xq_or_null int8 [B*Nq, H*dv], the
 * codes sa_quantize_act(out, act_inv_scale) would give, and xh_or_null fp16 [B*Nq, H*dv],
 * out rounded to nearest.  Either may be NULL, and so may `out` when one of them is given
 * (a consumer that reads only the quantised form saves the fp32 write).
 * variant: SA_VARIANT_VALU computes the scores by XOR + popcount on the vector ALU, one
 * (batch, head, 256 queries) unit per workgroup; SA_VARIANT_MFMA as the dot product of the
 * +-1 sign vectors on the matrix cores (the same integers, nbits <= 256); SA_VARIANT_AUTO
 * (what sa_hamming_attention uses) is the popcount form again, for dv <= 64, nbits <= 256 and
 * scales that need no per-row reference as a launch whose workgroups walk over several units
 * with the next chunk of V and key codes loading meanwhile (bit-identical to
 * SA_VARIANT_VALU), else as SA_VARIANT_VALU. */
int sa_hamming_attention_fused(const uint64_t *q_codes, const uint64_t *k_codes, const float *v,
                               float *out, int B, int H, int Nq, int Nk, int nbits, int dv,
                               float scale, int16_t *scores_or_null, int8_t *xq_or_null,
                               void *xh_or_null, float act_inv_scale, int variant, void *stream);

/*
 * Shift layer (Eq. 3, O_Shift = sum X * s * 2^P) on int8 activations with
 * int32 accumulation:  y[m,n] = bias[n] + sum_k s[n,k] * (x[m,k] << e[n,k]).
 *   x [M,K] int8, w4 [N,K/2] packed 4-bit, bias [N] int32 or NULL, y [M,N] int32.
 * K % 32 == 0 (16-byte weight rows), for both variants.
 * Both variants are bit-exact.  The MFMA variant decodes the weights to two
 * int8 planes in the workspace before the matrix-core pass (2*N*Kp bytes, Kp = K
 * rounded up to a multiple of 64: plane rows are padded with zeros to whole
 * 64-byte stages; the activation rows are read as they are).
 *
 * The planes depend on the weights only (s * 2^min(e,6) and s * 64 * [e == 7],
 * which sum to s * 2^e of Eq. 3), so a caller with fixed weights decodes them
 * once: sa_shift_planes_prepare writes them to `planes` (device memory of
 * sa_shift_planes_bytes(K, N) bytes, 16-byte aligned, owned by the caller;
 * layout [2, N, Kp] int8; K % 32 == 0).  With variant SA_VARIANT_MFMA_PREPARED the weight arguments of
 * sa_shift_linear, sa_shift_mlp and sa_block_forward (w4, w1, w2) point at such
 * planes instead of packed nibbles, and no decode runs.
 */
/*
 * Dense weights to shift weights (Sec. 4.1, below Eq. 3: s = sign(W),
 * P = round(log2 |W|)), in the 4-bit storage format of this library:
 *   w [N,K] fp32  ->  w4 [N,K/2],  nibble = (W < 0) << 3 | (clamp(P, -7, 0) + 7)
 * sign(0) = +1; W = 0 and every |W| < 2^-7.5 take P = -7, |W| > 2^-0.5 takes P = 0
 * (weights are expected in [-1, 1], as after the usual normalisation); NaN
 * counts as +1.0.  log2 |W| is never half-way for a float, so the rounding is
 * unambiguous; the result is bit-exact.  K % 8 == 0.
 */
int sa_shift_weights_from_float(const float *w, int N, int K, uint8_t *w4, void *stream);

size_t sa_shift_planes_bytes(int K, int N);
int sa_shift_planes_prepare(const uint8_t *w4, int K, int N, void *planes, size_t planes_bytes,
                            void *stream);
size_t sa_shift_linear_workspace_bytes(long M, int K, int N, int variant);
int sa_shift_linear(const int8_t *x, const uint8_t *w4, const int32_t *bias_or_null, int32_t *y,
                    long M, int K, int N, int variant, void *workspace, size_t workspace_bytes,
                    void *stream);

/*
 * A shift Linear whose consumers are fp32 (Sec. 4.1: the four Linears of the
 * attention module as shift layers; Eq. 2 for the residual):
 *   y[m, n] = fma(float(acc[m, n]), scale, residual[m, n]),  acc as in sa_shift_linear
 * (int32 accumulator converted round-to-nearest-even, one fused multiply-add;
 * residual_or_null == NULL stands for 0).  The N columns leave as `parts`
 * (1..3) column blocks of N / parts columns each, block p to y0 / y1 / y2 as a
 * dense [M, N / parts] matrix: a fused Q/K/V projection (weight rows = Wq, Wk,
 * Wv stacked) writes its three outputs in the layout the attention calls read.
 * N % (4 * parts) == 0; a residual [M, N] needs parts == 1 and may be y0 itself
 * (in place).  Variants, weights and workspace as for sa_shift_linear.
 */
int sa_shift_linear_f32(const int8_t *x, const uint8_t *w4, long M, int K, int N, int variant,
                        float scale, const float *residual_or_null, int parts, float *y0, float *y1,
                        float *y2, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The fused Q/K/V projection of the sign-hash variant (Sec. 4.1 with vanilla
 * sign quantisation of Q and K, nbits = head width): the shift Linear of
 * sa_shift_linear_f32 over the stacked [3E, E] weight, but Q and K never leave
 * as floats: their code bits are the signs of the accumulators,
 *   bit j of token n, head h = [acc[n, h * d + j] >= 0]     (= [scale * acc >= 0], scale > 0)
 * packed as sa_binarize would pack them ([B,H,N,d/64]), and only V is written
 * as fp32 [B*N, E] = fma(float(acc), scale, 0).  x int8 [B*N, E]; d = E / H in
 * {64, 128}; E % 128 == 0; matrix-core variants only.  Bit-identical to
 * sa_shift_linear_f32 followed by sa_binarize_pair without a projection.
 */
int sa_shift_linear_qkv_codes(const int8_t *x, const uint8_t *wqkv, int B, int N, int H, int E, int variant,
                              float scale, uint64_t *q_codes, uint64_t *k_codes, float *v, void *workspace,
                              size_t workspace_bytes, void *stream);

/*
 * Top-1 routing (Sec. 4.2: p = softmax(logits), G(x) = p_i * 1{p_i >= p_j}).
 * Expert 0 = Mult, expert 1 = Shift.  The decision compares raw logits; ties
 * go to the lowest index.  2 <= E <= 8.
 *   logits [T,E] fp32 in
 *   perm [T]      token ids, expert 0's in ascending order, then expert 1's, ...
 *   expert_of [T] chosen expert per token
 *   counts [E]    tokens per expert (device memory, like the others)
 *   gate [T]      softmax probability of the chosen expert, fp32
 * Up to 32768 tokens the call is one launch and needs no workspace (the query returns 0).
 */
size_t sa_moe_dispatch_workspace_bytes(long T, int E);
int sa_moe_dispatch(const float *logits, long T, int E, int32_t *perm, int32_t *expert_of,
                    int32_t *counts, float *gate, void *workspace, size_t workspace_bytes,
                    void *stream);
/*
 * sa_moe_dispatch for callers that cannot allocate device memory and so have no workspace
 * to pass: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and kernels; the scratch of the long-input path is an
 * array built into the library (256 KiB per GPU, held until the process ends) instead of
 * a workspace.  The call allocates nothing.  T <= sa_moe_dispatch_static_max_tokens()
 * (1048576), SA_ERR_UNSUPPORTED beyond.  All calls on one GPU share that array: two calls
 * that overlap in time on the same GPU (different streams) race; calls on one stream, or
 * on different GPUs, do not.
 */
long sa_moe_dispatch_static_max_tokens(void);
int sa_moe_dispatch_static(const float *logits, long T, int E, int32_t *perm, int32_t *expert_of,
                           int32_t *counts, float *gate, void *stream);

/*
 * The MoE form of one Linear layer (Sec. 4.1: the Linear layers of the attention module become
 * Shift layers or MoEs; Sec. 4.2: y = sum_i G(x) E_i(x), G = p_i * 1{p_i >= p_j}).  Top-1 routing
 * by logits [T,2] between expert 0 (Mult: w_f16 [N,K] fp16 times xh, the fp16 form of the
 * activations, fp32 accumulation) and expert 1 (Shift: w4 [N,K/2] packed 4-bit shift weights
 * times xq, the int8 codes of the same activations, int32 accumulation, times out_scale):
 *   y[t, :] = gate[t] * (xh[t, :] . W^T)                      t routed to expert 0
 *   y[t, :] = gate[t] * out_scale * (xq[t, :] . Wshift^T)     t routed to expert 1
 * xq [T,K] int8, xh [T,K] fp16, y [T,N] fp32, all device memory; every row of y is written once.
 * expert_of_or_null [T] int32 and gate_or_null [T] fp32 receive the routing when given.  K % 32 == 0.
 * variant as for sa_shift_linear (with SA_VARIANT_MFMA_PREPARED w4 points at prepared planes).
 * The Shift rows are bit-exact up to the fp32 product with gate and out_scale; the Mult rows carry
 * the rounding of fp32 accumulation.  Workspace (sa_moe_linear_workspace_bytes): routing lists and
 * the decoded weight planes; nothing in it needs to be initialised.
 */
size_t sa_moe_linear_workspace_bytes(long T, int K, int N, int variant);
int sa_moe_linear(const int8_t *xq, const void *xh, const float *logits, long T, int K, int N,
                  const uint8_t *w4, const void *w_f16, float out_scale, float *y,
                  int32_t *expert_of_or_null, float *gate_or_null, int variant, void *workspace,
                  size_t workspace_bytes, void *stream);

/*
 * Forward value of the latency-aware load-balancing loss (Eq. 4):
 *   IMP_i  = alpha_i * sum_x p_i(x),   LOAD_i = alpha_i * sum_x q_i(x),   p = softmax(logits)
 *   q_i(x) = Phi((p_i(x) - max_{j != i} p_j(x)) / noise_std)     (normal noise on p_i as the proxy)
 *   losses[0] = SCV(IMP), losses[1] = SCV(LOAD),  SCV(u) = var(u) / mean(u)^2 (population variance)
 * logits [T,E] fp32, alpha [E] fp32 (the latency coefficients Lat_i / sum Lat_j), all device
 * memory; losses fp32 [2]; sums_or_null fp32 [2,E] = IMP then LOAD.  2 <= E <= 8, T > 0,
 * noise_std > 0.  Token sums are taken per 256 tokens in fp32, then in fp64 in ascending order
 * (deterministic).
 */
size_t sa_moe_balance_loss_workspace_bytes(long T, int E);
int sa_moe_balance_loss(const float *logits, long T, int E, const float *alpha, float noise_std,
                        float *losses, float *sums_or_null, void *workspace, size_t workspace_bytes,
                        void *stream);

/*
 * Activation quantisation with a static per-tensor scale (appendix,
 * integer-arithmetic quantisation):  q = clamp(rne(x * inv_scale), -127, 127),
 * NaN -> 0.  One fp32 multiply and one round-to-nearest-even; bit-exact.
 */
int sa_quantize_act(const float *x, long n, float inv_scale, int8_t *q, void *stream);
/* The same pass also leaves x rounded to fp16 in xh_or_null ([n], 16-byte aligned) when it
 * is not NULL: the input form of the Mult expert (Sec. 4.2), so x is read once for both. */
int sa_quantize_act_half(const float *x, long n, float inv_scale, int8_t *q, void *xh_or_null,
                         void *stream);

/*
 * LayerNorm over the rows of x [T, E] (Eq. 2), fp32, biased variance:
 *   y = (x - mean) / sqrt(var + eps) * gamma + beta
 * fused with the forms its consumers read; each output is optional (NULL):
 *   ln_or_null     fp32 [T, E]   y itself
 *   q_or_null      int8 [T, E]   clamp(rne(y * inv_scale), -127, 127), the input of shift Linears
 *   xh_or_null     fp16 [T, E]   y rounded to half, the input of the Mult expert (Sec. 4.2)
 *   logits_or_null fp32 [T, n_experts] = y * wg + bg, the router G of Sec. 4.2;
 *                  wg fp32 [E, n_experts], bg fp32 [n_experts], 2 <= n_experts <= 8
 * E % 4 == 0 and E <= 8192.
 */
int sa_layernorm_quant(const float *x, long T, int E, const float *gamma, const float *beta, float eps,
                       float inv_scale, float *ln_or_null, int8_t *q_or_null, void *xh_or_null,
                       const float *wg_or_null, const float *bg_or_null, int n_experts,
                       float *logits_or_null, void *stream);

/*
 * Between the two shift linears of the Shift expert:
 *   h = lut[clamp(rne(float(y) * s), -127, 127) + 128],  lut int8 [256].
 */
int sa_requant_lut(const int32_t *y, long n, float s, const int8_t *lut, int8_t *h, void *stream);

/*
 * Row selection.  Several calls below work on a subset of the rows of a
 * [T, E] matrix.  rows_or_null lists the row ids (NULL = rows 0..max_rows-1).
 * If counts_or_null is not NULL the list is expert `expert`'s segment of a
 * dispatch result: rows = perm + sum(counts[0..expert-1]) and the number of
 * rows is counts[expert], both read on the device (no host round trip);
 * max_rows then only bounds the launch and the compact outputs.
 */
typedef struct sa_rows {
    const int32_t *rows_or_null;   /* [max_rows] row ids, or perm [T] with counts  */
    const int32_t *counts_or_null; /* [E] device, from sa_moe_dispatch             */
    int expert;                    /* which segment, with counts                   */
    long max_rows;                 /* upper bound on the rows processed            */
} sa_rows;

/*
 * Shift expert (Sec. 4.2, the Shift expert; Sec. 4.1, MLPs as shift layers):
 *   h  = lut[requant(shift_linear(xq[rows], w1), requant_scale)]
 *   y2 = shift_linear(h, w2)                                     (int32, exact)
 * Outputs, either or both:
 *   y2_or_null  int32 [max_rows, E], row i belongs to rows[i]
 *   y_or_null   fp32 [T, E]:  y[rows[i], :] = gate[rows[i]] * out_scale * y2[i, :]
 *               (gate_or_null == NULL stands for gate 1)
 *   xq [T,E] int8, w1 [hid, E/2], w2 [E, hid/2], lut int8 [256].
 * Workspace holds the int8 hidden rows.  E % 64 == 0 and hid % 64 == 0.
 * stages: 1 = first layer only (fills the workspace), 2 = second layer only
 * (reads the workspace a stage-1 call with the same rows filled), 3 = both.
 * stages | SA_MLP_ACCUMULATE: y_or_null is added to instead of overwritten,
 *   y[rows[i], :] = fma(gate, out_scale * y2[i, :], y[rows[i], :])
 * (the residual sum of Eq. 2 when y holds the block's input rows).
 */
#define SA_MLP_ACCUMULATE 4
size_t sa_shift_mlp_workspace_bytes(long max_rows, int E, int hid);
int sa_shift_mlp(const int8_t *xq, const sa_rows *rows, int E, int hid, const uint8_t *w1,
                 const uint8_t *w2, float requant_scale, const int8_t *lut, int32_t *y2_or_null,
                 float *y_or_null, const float *gate_or_null, float out_scale, int variant,
                 int stages, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Mult expert (Sec. 4.2): a dense two-layer MLP with erf-GELU in fp16 with
 * fp32 accumulation.  x rows and the hidden activation are rounded to fp16.
 *   out = W2 * half(gelu(W1 * half(x[rows])))      W1 [hid,E], W2 [E,hid] fp16
 * Outputs as for sa_shift_mlp: out_or_null fp32 [max_rows, E] and / or
 * y_or_null fp32 [T, E] with y[rows[i], :] = gate[rows[i]] * out[i, :].
 * E % 32 == 0 and hid % 32 == 0.  stages as for sa_shift_mlp (the workspace
 * holds the fp16 hidden rows).
 */
size_t sa_mult_mlp_workspace_bytes(long max_rows, int E, int hid);
int sa_mult_mlp_f16(const float *x, const sa_rows *rows, int E, int hid, const void *w1_f16,
                    const void *w2_f16, float *out_or_null, float *y_or_null,
                    const float *gate_or_null, int stages, void *workspace,
                    size_t workspace_bytes, void *stream);
/* The same expert on rows that already exist in fp16: xh_all is [T, E] fp16 (all tokens, as
 * sa_quantize_act_half or sa_hamming_attention_fused leave them) and the first layer picks
 * the rows of `rows` itself, so no gathered copy is made. */
int sa_mult_mlp_f16_half(const void *xh_all, const sa_rows *rows, int E, int hid,
                         const void *w1_f16, const void *w2_f16, float *out_or_null,
                         float *y_or_null, const float *gate_or_null, int stages,
                         void *workspace, size_t workspace_bytes, void *stream);

/* Plain row movement (Sec. 4.2, y = sum_i G(x) * E_i(x) with one non-zero term):
 *   gather : dst[i, :] = src[rows[i], :]                 (row_bytes % 16 == 0)
 *   combine: y[rows[i], :] = gate[rows[i]] * src[i, :]   (fp32, width E)      */
int sa_gather_rows(const void *src, size_t row_bytes, const sa_rows *rows, void *dst,
                   void *stream);
int sa_combine_rows(const float *src, const sa_rows *rows, const float *gate_or_null, int E,
                    float *y, void *stream);

/*
 * One pass of the block (Eq. 2 restricted to the reparameterised parts):
 *   codes = binarize(Q), binarize(K)
 *   O     = additive attention (linear) or Hamming attention (quadratic)
 *   y     = MoE{Mult, Shift}(O) with top-1 dispatch, or Shift MLP(O) if no router
 * Q, K, V enter as fp32 [B,N,H,d] / [B,N,H,dv]; O [B,N,H,dv] = [T,E] and
 * y [T,E] leave as fp32.  All kernels are enqueued on one stream.
 */
typedef struct sa_block_desc {
    int B, N, H, d, nbits, dv;
    int attention;          /* 0 = linear additive, 1 = quadratic Hamming            */
    int hid;                /* MLP hidden width; 0 = attention only                  */
    int moe;                /* 1 = router + two experts, 0 = Shift MLP for all rows  */
    int shift_variant;      /* SA_VARIANT_*                                          */
    float attn_scale, act_inv_scale, requant_scale, out_scale;
    const float *q, *k, *v; /* inputs                                                */
    const float *proj;      /* [d, nbits] or NULL                                    */
    const float *logits;    /* [T, 2] router logits (moe == 1)                       */
    const uint8_t *w1, *w2; /* Shift expert, packed 4-bit                            */
    const int8_t *lut;      /* [256]                                                 */
    const void *mw1, *mw2;  /* Mult expert fp16 (moe == 1)                           */
    float *o;               /* [T, E] attention output                               */
    float *y;               /* [T, E] block output (hid > 0)                         */
    void *workspace;
    size_t workspace_bytes;
} sa_block_desc;

size_t sa_block_workspace_bytes(const sa_block_desc *desc /* host */);
int sa_block_forward(const sa_block_desc *desc /* host */, void *stream);

/*
 * The complete block of Eq. 2 on tokens x [T, E] fp32, T = B * N:
 *   z1 = int8(LayerNorm1(x))                          sa_layernorm_quant
 *   Q, K, V = qkv_scale * ShiftLinear(z1, wqkv)       one launch, rows of wqkv = Wq, Wk, Wv stacked
 *   O = attention(binarize(Q), binarize(K), V)        heads are column blocks of width E / H
 *   x1 = fma(ShiftLinear(int8(O), wo), o_scale, x)    residual, Eq. 2 (left)
 *   z2 = LayerNorm2(x1): int8, fp16, router logits z2 * wg + bg
 *   y  = x1 + MoE{Mult, Shift}(z2)  or  x1 + ShiftMLP(z2)        Eq. 2 (right)
 * The four attention Linears are shift layers (Sec. 4.1); all scales are static
 * and passed in.  Weights follow shift_variant (packed 4-bit rows, or planes
 * from sa_shift_planes_prepare for SA_VARIANT_MFMA_PREPARED; wqkv as one
 * [3E, E] matrix).  E % 64 == 0, hid % 64 == 0, E / H in {32, 64, 128} for the
 * Hamming variant.  y must not overlap x.
 */
typedef struct sa_layer_desc {
    int B, N, H, nbits;
    int E, hid;
    int attention;          /* 0 = linear additive, 1 = quadratic Hamming            */
    int moe;                /* 1 = router + two experts, 0 = Shift MLP for all rows  */
    int shift_variant;      /* SA_VARIANT_*                                          */
    float eps;              /* both LayerNorms                                       */
    float ln_inv_scale;     /* LayerNorm output -> int8                              */
    float qkv_scale;        /* int32 accumulator -> fp32 Q, K, V                     */
    float attn_scale;
    float act_inv_scale;    /* attention output -> int8                              */
    float o_scale;          /* int32 accumulator of the output projection -> fp32    */
    float requant_scale, out_scale;              /* Shift expert                     */
    const float *x;         /* [T, E]                                                */
    const float *gamma1, *beta1, *gamma2, *beta2; /* [E] each                        */
    const uint8_t *wqkv;    /* [3E, E/2] packed (or planes of the [3E, E] matrix)    */
    const uint8_t *wo;      /* [E, E/2]                                              */
    const float *proj;      /* [E/H, nbits] or NULL (then nbits == E/H)              */
    const float *wg, *bg;   /* router [E, 2], [2] (moe == 1)                         */
    const uint8_t *w1, *w2; /* Shift expert                                          */
    const int8_t *lut;      /* [256]                                                 */
    const void *mw1, *mw2;  /* Mult expert fp16 (moe == 1)                           */
    float *y;               /* [T, E] block output                                   */
    void *workspace;
    size_t workspace_bytes;
} sa_layer_desc;

size_t sa_layer_workspace_bytes(const sa_layer_desc *desc /* host */);
int sa_layer_forward(const sa_layer_desc *desc /* host */, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SHIFTADD_H_ */
