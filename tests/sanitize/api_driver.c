/* Drives the host side of libshiftadd (argument validation, size queries, error text) under AddressSanitizer and
 * UndefinedBehaviorSanitizer: every entry point is called with arguments that its validation must refuse before
 * anything is launched, so no GPU is needed.  Built by tests/test_sanitizers.py against a build of the library
 * whose host code is instrumented.  A clean run prints "api driver ok". */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "shiftadd.h"

static int failures = 0;
#define EXPECT(call, code)                                                                   \
    do {                                                                                     \
        int rc_ = (call);                                                                    \
        if (rc_ != (code)) { printf("line %d: got %d, expected %d (%s)\n", __LINE__, rc_, (code), sa_last_error()); ++failures; } \
        else if ((code) != SA_OK && sa_last_error()[0] == '\0') { printf("line %d: no error text\n", __LINE__); ++failures; }     \
    } while (0)

int main(void) {
    void *fake = (void *)0x1000, *odd = (void *)0x1004;
    if (sa_version() <= 0) return 2;
    /* hash */
    EXPECT(sa_binarize(fake, 1, 1, 1, 64, fake, 65, fake, NULL), SA_ERR_SHAPE);
    EXPECT(sa_binarize(fake, 1, 1, 1, 64, NULL, 128, fake, NULL), SA_ERR_SHAPE);
    EXPECT(sa_binarize(odd, 1, 1, 1, 64, fake, 64, fake, NULL), SA_ERR_ALIGN);
    EXPECT(sa_binarize(fake, 1, 1, 1, 48, fake, 64, fake, NULL), SA_ERR_UNSUPPORTED);
    EXPECT(sa_binarize(NULL, 0, 5, 1, 64, NULL, 64, NULL, NULL), SA_OK);
    EXPECT(sa_binarize_ex(fake, 1, 1, 1, 64, fake, 64, fake, 9, NULL), SA_ERR_INVALID);
    EXPECT(sa_binarize_pair(fake, NULL, 1, 1, 1, 64, fake, 64, fake, fake, NULL), SA_ERR_INVALID);
    /* attention */
    EXPECT(sa_additive_attention(fake, fake, fake, fake, 1, 1, 4, 4, 64, 64, 1.0f, fake, 0, NULL, 0, NULL), SA_ERR_INVALID);
    EXPECT(sa_additive_attention(fake, fake, fake, fake, 1, 1, 4, 4, 64, 48, 1.0f, fake, 3, NULL, 0, NULL), SA_ERR_UNSUPPORTED);
    if (sa_additive_attention_workspace_bytes(8, 4, 16384, 256, 64) == 0) ++failures;
    if (sa_additive_attention_workspace_bytes(-1, 4, 16384, 256, 64) != 0) ++failures;
    EXPECT(sa_additive_attention(fake, fake, fake, fake, 8, 4, 16384, 16384, 256, 64, 1.0f, fake, 3, NULL, 0, NULL), SA_ERR_WORKSPACE);
    EXPECT(sa_linear_attention_01(fake, fake, fake, fake, 1, 1, 4, 4, 64, 64, 0.0f, fake, fake, 3, NULL, 0, NULL), SA_ERR_INVALID);
    EXPECT(sa_dwconv3x3(fake, fake, NULL, fake, 0, 1, 2, 2, 6, NULL), SA_ERR_SHAPE);
    EXPECT(sa_hamming_attention(fake, fake, fake, fake, 1, 1, 4, 0, 64, 64, 1.0f, NULL, NULL), SA_ERR_SHAPE);
    EXPECT(sa_hamming_attention(fake, fake, fake, fake, 1, 1, 4, 4, 64, 64, NAN, NULL, NULL), SA_ERR_INVALID);
    EXPECT(sa_hamming_attention_fused(fake, fake, fake, NULL, 1, 1, 4, 4, 64, 64, 1.0f, NULL, NULL, NULL, 1.0f, 2, NULL), SA_ERR_INVALID);
    /* shift layers */
    EXPECT(sa_shift_linear(fake, fake, NULL, fake, 4, 33, 8, 0, NULL, 0, NULL), SA_ERR_SHAPE);
    EXPECT(sa_shift_linear(fake, fake, NULL, fake, 4, 64, 8, 7, NULL, 0, NULL), SA_ERR_INVALID);
    EXPECT(sa_shift_linear(fake, fake, NULL, fake, 4, 48, 8, 1, NULL, 0, NULL), SA_ERR_SHAPE);
    EXPECT(sa_shift_linear(fake, fake, NULL, fake, 4, 96, 8, 1, NULL, 0, NULL), SA_ERR_WORKSPACE);
    EXPECT(sa_shift_linear(NULL, fake, NULL, fake, 4, 64, 8, 0, NULL, 0, NULL), SA_ERR_INVALID);
    EXPECT(sa_shift_linear(fake, fake, NULL, fake, 4, 64, 8, 1, NULL, 0, NULL), SA_ERR_WORKSPACE);
    EXPECT(sa_shift_linear(fake, fake, NULL, fake, 1L << 40, 64, 8, 0, NULL, 0, NULL), SA_ERR_SHAPE);
    EXPECT(sa_shift_linear(fake, fake, NULL, fake, 4, 262144, 8, 0, NULL, 0, NULL), SA_ERR_SHAPE);
    if (sa_shift_planes_bytes(64, 8) != 1024 || sa_shift_planes_bytes(96, 8) != 2048 || sa_shift_planes_bytes(48, 8) != 0) ++failures;
    EXPECT(sa_shift_planes_prepare(fake, 64, 8, fake, 16, NULL), SA_ERR_WORKSPACE);
    EXPECT(sa_shift_weights_from_float(fake, 4, 12, fake, NULL), SA_ERR_SHAPE);
    EXPECT(sa_shift_linear_f32(fake, fake, 4, 64, 12, 0, 1.0f, fake, 3, fake, fake, fake, NULL, 0, NULL), SA_ERR_INVALID);
    EXPECT(sa_shift_linear_f32(fake, fake, 4, 64, 10, 0, 1.0f, NULL, 1, fake, NULL, NULL, NULL, 0, NULL), SA_ERR_SHAPE);
    EXPECT(sa_shift_linear_qkv_codes(fake, fake, 1, 4, 3, 192, 0, 1.0f, fake, fake, fake, NULL, 0, NULL), SA_ERR_UNSUPPORTED);
    EXPECT(sa_shift_linear_qkv_codes(fake, fake, 1, 4, 2, 128, 1, -1.0f, fake, fake, fake, NULL, 0, NULL), SA_ERR_INVALID);
    EXPECT(sa_quantize_act(fake, -1, 1.0f, fake, NULL), SA_ERR_INVALID);
    EXPECT(sa_quantize_act_half(fake, 4, 1.0f, fake, odd, NULL), SA_ERR_ALIGN);
    EXPECT(sa_requant_lut(fake, 4, 1.0f, NULL, fake, NULL), SA_ERR_INVALID);
    EXPECT(sa_layernorm_quant(fake, 4, 66, fake, fake, 1e-6f, 1.0f, fake, NULL, NULL, NULL, NULL, 0, NULL, NULL), SA_ERR_SHAPE);
    /* routing */
    EXPECT(sa_moe_dispatch(fake, 100, 1, fake, fake, fake, fake, NULL, 0, NULL), SA_ERR_SHAPE);
    EXPECT(sa_moe_dispatch(fake, 100000, 2, fake, fake, fake, fake, NULL, 0, NULL), SA_ERR_WORKSPACE);
    EXPECT(sa_moe_dispatch(fake, 100, 2, fake, fake, NULL, fake, NULL, 0, NULL), SA_ERR_INVALID);
    EXPECT(sa_moe_dispatch_static(fake, sa_moe_dispatch_static_max_tokens() + 1, 2, fake, fake, fake, fake, NULL), SA_ERR_UNSUPPORTED);
    EXPECT(sa_moe_dispatch_static(fake, 100, 9, fake, fake, fake, fake, NULL), SA_ERR_SHAPE);
    EXPECT(sa_moe_balance_loss(fake, 0, 2, fake, 0.1f, fake, NULL, fake, 1024, NULL), SA_ERR_INVALID);
    EXPECT(sa_moe_balance_loss(fake, 10, 2, fake, -1.0f, fake, NULL, fake, 1024, NULL), SA_ERR_INVALID);
    /* the MoE form of a Linear layer */
    EXPECT(sa_moe_linear(fake, fake, fake, 10, 48, 8, fake, fake, 1.0f, fake, NULL, NULL, 1, fake, 1 << 20, NULL), SA_ERR_SHAPE);
    EXPECT(sa_moe_linear(fake, fake, NULL, 10, 64, 8, fake, fake, 1.0f, fake, NULL, NULL, 1, fake, 1 << 20, NULL), SA_ERR_INVALID);
    EXPECT(sa_moe_linear(fake, fake, fake, 10, 64, 8, fake, fake, 1.0f, fake, NULL, NULL, 1, fake, 16, NULL), SA_ERR_WORKSPACE);
    EXPECT(sa_moe_linear(fake, fake, fake, 10, 64, 8, fake, fake, 1.0f, fake, NULL, NULL, 9, fake, 1 << 20, NULL), SA_ERR_INVALID);
    EXPECT(sa_moe_linear(fake, fake, fake, 0, 64, 8, fake, fake, 1.0f, fake, NULL, NULL, 1, NULL, 0, NULL), SA_OK);
    if (sa_moe_linear_workspace_bytes(10, 48, 8, 1) != 0 || sa_moe_linear_workspace_bytes(10, 64, 8, 1) < 2 * 8 * 64) ++failures;
    /* experts and row movement */
    sa_rows rows = {NULL, fake, 0, 10};                      /* counts without a list */
    EXPECT(sa_shift_mlp(fake, &rows, 64, 64, fake, fake, 1.0f, fake, fake, NULL, NULL, 1.0f, 1, 3, fake, 1 << 20, NULL), SA_ERR_INVALID);
    sa_rows all = {NULL, NULL, 0, 10};
    EXPECT(sa_shift_mlp(fake, &all, 64, 96, fake, fake, 1.0f, fake, fake, NULL, NULL, 1.0f, 1, 3, fake, 1 << 20, NULL), SA_ERR_SHAPE);
    EXPECT(sa_shift_mlp(fake, &all, 64, 64, fake, fake, 1.0f, fake, NULL, NULL, NULL, 1.0f, 1, 3, fake, 1 << 20, NULL), SA_ERR_INVALID);
    EXPECT(sa_shift_mlp(fake, &all, 64, 64, fake, fake, 1.0f, fake, fake, NULL, NULL, 1.0f, 1, 3, fake, 16, NULL), SA_ERR_WORKSPACE);
    EXPECT(sa_shift_mlp(fake, NULL, 64, 64, fake, fake, 1.0f, fake, fake, NULL, NULL, 1.0f, 1, 3, fake, 16, NULL), SA_ERR_INVALID);
    EXPECT(sa_mult_mlp_f16(fake, &all, 48, 64, fake, fake, fake, NULL, NULL, 3, fake, 1 << 20, NULL), SA_ERR_SHAPE);
    EXPECT(sa_mult_mlp_f16_half(fake, &all, 64, 64, fake, fake, NULL, NULL, NULL, 3, fake, 1 << 20, NULL), SA_ERR_INVALID);
    EXPECT(sa_gather_rows(fake, 24, &all, fake, NULL), SA_ERR_SHAPE);
    EXPECT(sa_combine_rows(fake, &all, NULL, 6, fake, NULL), SA_ERR_SHAPE);
    /* block and layer descriptors */
    sa_block_desc bd;
    memset(&bd, 0, sizeof bd);
    EXPECT(sa_block_forward(&bd, NULL), SA_ERR_INVALID);
    EXPECT(sa_block_forward(NULL, NULL), SA_ERR_INVALID);
    bd.B = 1; bd.N = 4; bd.H = 1; bd.d = 64; bd.nbits = 96; bd.dv = 64;
    EXPECT(sa_block_forward(&bd, NULL), SA_ERR_SHAPE);
    bd.nbits = 64; bd.hid = 64; bd.moe = 1;
    if (sa_block_workspace_bytes(&bd) == 0) ++failures;
    bd.q = bd.k = bd.v = fake; bd.o = fake;
    EXPECT(sa_block_forward(&bd, NULL), SA_ERR_WORKSPACE);
    sa_layer_desc ld;
    memset(&ld, 0, sizeof ld);
    EXPECT(sa_layer_forward(&ld, NULL), SA_ERR_INVALID);
    ld.B = 1; ld.N = 4; ld.H = 3; ld.nbits = 64; ld.E = 200; ld.hid = 256;
    EXPECT(sa_layer_forward(&ld, NULL), SA_ERR_SHAPE);
    if (sa_layer_workspace_bytes(&ld) != 0) ++failures;
    if (failures) { printf("%d failures\n", failures); return 1; }
    puts("api driver ok");
    return 0;
}
