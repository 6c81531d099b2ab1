// sa_block_forward: one pass of the reparameterised block (Eq. 2 restricted to the
// attention MatMuls and the MLP): hash Q and K, additive or Hamming attention, then the
// Shift MLP or the two-expert MoE.  Pure composition of the library's own entry points;
// the expert row counts stay on the device (no host round trip).
#include "common.h"

namespace {

struct Layout {
    size_t qc, kc, kv, attn_ws, xq, xh, perm, expert_of, counts, gate, disp_ws, shift_ws, mult_ws, total;
    size_t attn_ws_bytes, disp_ws_bytes, shift_ws_bytes, mult_ws_bytes;
};

size_t up(size_t x) { return (x + 255) / 256 * 256; }

int plan(const sa_block_desc *d, Layout *L) {
    SA_REQUIRE(d != nullptr, SA_ERR_INVALID, "block: descriptor is NULL");
    SA_REQUIRE(d->B > 0 && d->N > 0 && d->H > 0 && d->d > 0 && d->nbits > 0 && d->dv > 0, SA_ERR_INVALID,
               "block: sizes must be positive");
    SA_REQUIRE(d->nbits % 64 == 0, SA_ERR_SHAPE, "block: nbits must be a multiple of 64");
    SA_REQUIRE(d->attention == 0 || d->attention == 1, SA_ERR_INVALID, "block: attention must be 0 or 1");
    SA_REQUIRE(d->hid >= 0, SA_ERR_INVALID, "block: hid < 0");
    const size_t T = (size_t)d->B * d->N, E = (size_t)d->H * d->dv;
    SA_REQUIRE(T < (1ull << 31), SA_ERR_SHAPE, "block: too many tokens");
    size_t off = 0;
    const size_t code_bytes = up((size_t)d->B * d->H * d->N * (d->nbits / 64) * 8);
    L->qc = off; off += code_bytes;
    L->kc = off; off += code_bytes;
    L->kv = off;
    L->attn_ws_bytes = 0;
    if (d->attention == 0) {
        off += up((size_t)d->B * d->H * d->nbits * d->dv * 4);
        L->attn_ws_bytes = sa_additive_attention_workspace_bytes(d->B, d->H, d->N, d->nbits, d->dv);
    }
    L->attn_ws = off; off += up(L->attn_ws_bytes);
    L->xq = L->xh = off;
    L->disp_ws_bytes = L->shift_ws_bytes = L->mult_ws_bytes = 0;
    L->perm = L->expert_of = L->counts = L->gate = L->disp_ws = L->shift_ws = L->mult_ws = off;
    if (d->hid > 0) {
        off += up(T * E);
        L->shift_ws_bytes = sa_shift_mlp_workspace_bytes((long)T, (int)E, d->hid);
        L->shift_ws = off; off += up(L->shift_ws_bytes);
        if (d->moe) {
            L->xh = off; off += up(T * E * 2);          // fp16 copy of the attention output for the Mult expert
            L->perm = off; off += up(T * 4);
            L->expert_of = off; off += up(T * 4);
            L->counts = off; off += 256;
            L->gate = off; off += up(T * 4);
            L->disp_ws_bytes = sa_moe_dispatch_workspace_bytes((long)T, 2);
            L->disp_ws = off; off += up(L->disp_ws_bytes);
            L->mult_ws_bytes = sa_mult_mlp_workspace_bytes((long)T, (int)E, d->hid);
            L->mult_ws = off; off += up(L->mult_ws_bytes);
        }
    }
    L->total = off;
    return SA_OK;
}

}  // namespace

extern "C" size_t sa_block_workspace_bytes(const sa_block_desc *desc) {
    Layout L;
    if (plan(desc, &L) != SA_OK) return 0;
    return L.total;
}

extern "C" int sa_block_forward(const sa_block_desc *d, void *stream) {
    sa::clear_error();
    Layout L;
    int rc = plan(d, &L);
    if (rc != SA_OK) return rc;
    SA_REQUIRE(d->q && d->k && d->v && d->o, SA_ERR_INVALID, "block: q, k, v and o are required");
    SA_REQUIRE(d->workspace != nullptr && d->workspace_bytes >= L.total, SA_ERR_WORKSPACE,
               "block: workspace of %zu bytes needed, %zu given", L.total, d->workspace_bytes);
    SA_REQUIRE(sa::aligned16(d->workspace), SA_ERR_ALIGN, "block: workspace must be 16-byte aligned");
    if (d->hid > 0) {
        SA_REQUIRE(d->w1 && d->w2 && d->lut && d->y, SA_ERR_INVALID, "block: w1, w2, lut and y are required");
        if (d->moe) SA_REQUIRE(d->logits && d->mw1 && d->mw2, SA_ERR_INVALID, "block: logits, mw1, mw2 are required");
    }
    uint8_t *ws = static_cast<uint8_t *>(d->workspace);
    uint64_t *qc = reinterpret_cast<uint64_t *>(ws + L.qc), *kc = reinterpret_cast<uint64_t *>(ws + L.kc);
    const long T = (long)d->B * d->N;
    const int E = d->H * d->dv;

    const bool moe = d->hid > 0 && d->moe;
    int32_t *perm = reinterpret_cast<int32_t *>(ws + L.perm);
    int32_t *expert_of = reinterpret_cast<int32_t *>(ws + L.expert_of);
    int32_t *counts = reinterpret_cast<int32_t *>(ws + L.counts);
    float *gate = reinterpret_cast<float *>(ws + L.gate);
    // Everything runs on the caller's stream, one kernel after the other.  The two experts are independent
    // once the routing lists exist (the paper's "experts run in parallel", Sec. 4.2), but each of their GEMMs
    // fills the chip on its own: running them on two streams was measured and gains nothing (247-252 us against
    // 248 us per step at the DeiT-Base shape), while a caller that keeps two batches in flight on two streams of
    // its own is 5 % faster without the library's extra stream and events in the way.
    if (moe) {
        rc = sa_moe_dispatch(d->logits, T, 2, perm, expert_of, counts, gate, ws + L.disp_ws, L.disp_ws_bytes, stream);
        if (rc != SA_OK) return rc;
    }

    rc = sa_binarize_pair(d->q, d->k, d->B, d->N, d->H, d->d, d->proj, d->nbits, qc, kc, stream);
    if (rc != SA_OK) return rc;
    // The attention output leaves in three forms: fp32 (the block's output o), the int8 codes the
    // Shift layers read, and (with a Mult expert) the fp16 rounding its first layer reads.  The
    // Hamming kernel writes all three from its accumulators; the linear path adds one pass over o.
    int8_t *xq = reinterpret_cast<int8_t *>(ws + L.xq);
    void *xh = moe ? static_cast<void *>(ws + L.xh) : nullptr;
    const bool mlp = d->hid > 0;
    if (d->attention == 0) {
        rc = sa_additive_attention(qc, kc, d->v, d->o, d->B, d->H, d->N, d->N, d->nbits, d->dv, d->attn_scale,
                                   reinterpret_cast<float *>(ws + L.kv), 3, ws + L.attn_ws, L.attn_ws_bytes, stream);
        if (rc == SA_OK && mlp) rc = sa_quantize_act_half(d->o, T * E, d->act_inv_scale, xq, xh, stream);
    } else {
        rc = sa_hamming_attention_fused(qc, kc, d->v, d->o, d->B, d->H, d->N, d->N, d->nbits, d->dv, d->attn_scale,
                                         nullptr, mlp ? xq : nullptr, xh, d->act_inv_scale, SA_VARIANT_AUTO, stream);
    }
    if (rc != SA_OK || !mlp) return rc;

    if (moe) {
        const sa_rows mult_rows{perm, counts, 0, T};
        rc = sa_mult_mlp_f16_half(xh, &mult_rows, E, d->hid, d->mw1, d->mw2, nullptr, d->y, gate, 3, ws + L.mult_ws,
                                  L.mult_ws_bytes, stream);
        if (rc != SA_OK) return rc;
    }

    if (!moe) {
        const sa_rows all{nullptr, nullptr, 0, T};
        return sa_shift_mlp(xq, &all, E, d->hid, d->w1, d->w2, d->requant_scale, d->lut, nullptr, d->y, nullptr,
                            d->out_scale, d->shift_variant, 3, ws + L.shift_ws, L.shift_ws_bytes, stream);
    }
    const sa_rows shift_rows{perm, counts, 1, T};
    return sa_shift_mlp(xq, &shift_rows, E, d->hid, d->w1, d->w2, d->requant_scale, d->lut, nullptr, d->y, gate,
                        d->out_scale, d->shift_variant, 3, ws + L.shift_ws, L.shift_ws_bytes, stream);
}

// ---------------------------------------------------------------------------------------
// sa_layer_forward: the complete block of Eq. 2.  LayerNorm -> int8 -> fused Q/K/V shift
// Linear -> hash -> attention -> int8 -> output shift Linear + residual -> LayerNorm (int8,
// fp16 and router logits in one pass) -> dispatch -> experts adding into the residual rows.
namespace {

struct LayerLayout {
    size_t codes8, q, k, v, qc, kc, kv, attn_ws, xh, logits, perm, expert_of, counts, gate, disp_ws, shift_ws,
        mult_ws, lin_ws, total;
    size_t attn_ws_bytes, disp_ws_bytes, shift_ws_bytes, mult_ws_bytes, lin_ws_bytes;
};

int plan_layer(const sa_layer_desc *d, LayerLayout *L) {
    SA_REQUIRE(d != nullptr, SA_ERR_INVALID, "layer: descriptor is NULL");
    SA_REQUIRE(d->B > 0 && d->N > 0 && d->H > 0 && d->nbits > 0 && d->E > 0 && d->hid > 0, SA_ERR_INVALID,
               "layer: sizes must be positive");
    SA_REQUIRE(d->E % d->H == 0, SA_ERR_SHAPE, "layer: E (%d) is not a multiple of H (%d)", d->E, d->H);
    SA_REQUIRE(d->E % 64 == 0 && d->hid % 64 == 0, SA_ERR_SHAPE, "layer: E and hid must be multiples of 64");
    SA_REQUIRE(d->nbits % 64 == 0, SA_ERR_SHAPE, "layer: nbits must be a multiple of 64");
    SA_REQUIRE(d->attention == 0 || d->attention == 1, SA_ERR_INVALID, "layer: attention must be 0 or 1");
    SA_REQUIRE(d->shift_variant >= 0 && d->shift_variant <= 3, SA_ERR_INVALID, "layer: unknown shift variant");
    const size_t T = (size_t)d->B * d->N, E = (size_t)d->E;
    const int dv = d->E / d->H;
    SA_REQUIRE(T < (size_t)65535 * 8, SA_ERR_SHAPE, "layer: too many tokens for one call");
    size_t off = 0;
    L->codes8 = off; off += up(T * E);
    L->q = off; off += up(T * E * 4);
    L->k = off; off += up(T * E * 4);
    L->v = off; off += up(T * E * 4);
    const size_t code_bytes = up(T * d->H * (d->nbits / 64) * 8);
    L->qc = off; off += code_bytes;
    L->kc = off; off += code_bytes;
    L->kv = off;
    L->attn_ws_bytes = 0;
    if (d->attention == 0) {
        off += up((size_t)d->B * d->H * d->nbits * dv * 4);
        L->attn_ws_bytes = sa_additive_attention_workspace_bytes(d->B, d->H, d->N, d->nbits, dv);
    }
    L->attn_ws = off; off += up(L->attn_ws_bytes);
    L->shift_ws_bytes = sa_shift_mlp_workspace_bytes((long)T, d->E, d->hid);
    L->shift_ws = off; off += up(L->shift_ws_bytes);
    const size_t lin_qkv = sa_shift_linear_workspace_bytes((long)T, d->E, 3 * d->E, d->shift_variant);
    const size_t lin_o = sa_shift_linear_workspace_bytes((long)T, d->E, d->E, d->shift_variant);
    L->lin_ws_bytes = lin_qkv > lin_o ? lin_qkv : lin_o;
    L->lin_ws = off; off += up(L->lin_ws_bytes);
    L->xh = L->logits = L->perm = L->expert_of = L->counts = L->gate = L->disp_ws = L->mult_ws = off;
    L->disp_ws_bytes = L->mult_ws_bytes = 0;
    if (d->moe) {
        L->xh = off; off += up(T * E * 2);
        L->logits = off; off += up(T * 2 * 4);
        L->perm = off; off += up(T * 4);
        L->expert_of = off; off += up(T * 4);
        L->counts = off; off += 256;
        L->gate = off; off += up(T * 4);
        L->disp_ws_bytes = sa_moe_dispatch_workspace_bytes((long)T, 2);
        L->disp_ws = off; off += up(L->disp_ws_bytes);
        L->mult_ws_bytes = sa_mult_mlp_workspace_bytes((long)T, d->E, d->hid);
        L->mult_ws = off; off += up(L->mult_ws_bytes);
    }
    L->total = off;
    return SA_OK;
}

}  // namespace

extern "C" size_t sa_layer_workspace_bytes(const sa_layer_desc *desc) {
    LayerLayout L;
    if (plan_layer(desc, &L) != SA_OK) return 0;
    return L.total;
}

extern "C" int sa_layer_forward(const sa_layer_desc *d, void *stream) {
    sa::clear_error();
    LayerLayout L;
    int rc = plan_layer(d, &L);
    if (rc != SA_OK) return rc;
    SA_REQUIRE(d->x && d->y && d->gamma1 && d->beta1 && d->gamma2 && d->beta2 && d->wqkv && d->wo && d->w1 && d->w2 &&
                   d->lut,
               SA_ERR_INVALID, "layer: x, y, the LayerNorm parameters, wqkv, wo, w1, w2 and lut are required");
    if (d->moe) SA_REQUIRE(d->wg && d->bg && d->mw1 && d->mw2, SA_ERR_INVALID, "layer: wg, bg, mw1, mw2 are required");
    SA_REQUIRE(d->workspace != nullptr && d->workspace_bytes >= L.total, SA_ERR_WORKSPACE,
               "layer: workspace of %zu bytes needed, %zu given", L.total, d->workspace_bytes);
    SA_REQUIRE(sa::aligned16(d->workspace), SA_ERR_ALIGN, "layer: workspace must be 16-byte aligned");
    uint8_t *ws = static_cast<uint8_t *>(d->workspace);
    const long T = (long)d->B * d->N;
    const int E = d->E, dv = d->E / d->H;
    int8_t *codes8 = reinterpret_cast<int8_t *>(ws + L.codes8);
    float *q = reinterpret_cast<float *>(ws + L.q), *k = reinterpret_cast<float *>(ws + L.k);
    float *v = reinterpret_cast<float *>(ws + L.v);
    float *o = q;                                 // Q is dead once it is hashed
    uint64_t *qc = reinterpret_cast<uint64_t *>(ws + L.qc), *kc = reinterpret_cast<uint64_t *>(ws + L.kc);

    // attention half: X_attn = Attn(LayerNorm(X)) + X, left in y
    rc = sa_layernorm_quant(d->x, T, E, d->gamma1, d->beta1, d->eps, d->ln_inv_scale, nullptr, codes8, nullptr, nullptr,
                            nullptr, 0, nullptr, stream);
    if (rc != SA_OK) return rc;
    // Sign hash (no projection): the code bits are the signs of the Q and K accumulators, taken in the epilogue of
    // the projection, so Q and K never exist as floats.  Otherwise Q, K, V leave as fp32 and Q, K are hashed.
    const bool fused_hash = d->proj == nullptr && d->nbits == dv && (dv == 64 || dv == 128) && E % 128 == 0 &&
                            d->shift_variant != SA_VARIANT_VALU && d->qkv_scale > 0.0f &&
                            d->qkv_scale - d->qkv_scale == 0.0f;
    if (fused_hash) {
        rc = sa_shift_linear_qkv_codes(codes8, d->wqkv, d->B, d->N, d->H, E, d->shift_variant, d->qkv_scale, qc, kc, v,
                                       ws + L.lin_ws, L.lin_ws_bytes, stream);
        if (rc != SA_OK) return rc;
    } else {
        rc = sa_shift_linear_f32(codes8, d->wqkv, T, E, 3 * E, d->shift_variant, d->qkv_scale, nullptr, 3, q, k, v,
                                 ws + L.lin_ws, L.lin_ws_bytes, stream);
        if (rc != SA_OK) return rc;
        rc = sa_binarize_pair(q, k, d->B, d->N, d->H, dv, d->proj, d->nbits, qc, kc, stream);
        if (rc != SA_OK) return rc;
    }
    if (d->attention == 0) {
        rc = sa_additive_attention(qc, kc, v, o, d->B, d->H, d->N, d->N, d->nbits, dv, d->attn_scale,
                                   reinterpret_cast<float *>(ws + L.kv), 3, ws + L.attn_ws, L.attn_ws_bytes, stream);
        if (rc == SA_OK) rc = sa_quantize_act(o, T * E, d->act_inv_scale, codes8, stream);
    } else {
        // only the int8 form of the attention output is read (by the output projection): no fp32 write
        rc = sa_hamming_attention_fused(qc, kc, v, nullptr, d->B, d->H, d->N, d->N, d->nbits, dv, d->attn_scale, nullptr,
                                         codes8, nullptr, d->act_inv_scale, SA_VARIANT_AUTO, stream);
    }
    if (rc != SA_OK) return rc;
    rc = sa_shift_linear_f32(codes8, d->wo, T, E, E, d->shift_variant, d->o_scale, d->x, 1, d->y, nullptr, nullptr,
                             ws + L.lin_ws, L.lin_ws_bytes, stream);
    if (rc != SA_OK) return rc;

    // MLP half: y += MLP(LayerNorm(y)); every row is read by the LayerNorm before an expert adds to it
    const bool moe = d->moe != 0;
    void *xh = moe ? static_cast<void *>(ws + L.xh) : nullptr;
    float *logits = moe ? reinterpret_cast<float *>(ws + L.logits) : nullptr;
    rc = sa_layernorm_quant(d->y, T, E, d->gamma2, d->beta2, d->eps, d->ln_inv_scale, nullptr, codes8, xh,
                            moe ? d->wg : nullptr, moe ? d->bg : nullptr, moe ? 2 : 0, logits, stream);
    if (rc != SA_OK) return rc;
    if (!moe) {
        const sa_rows all{nullptr, nullptr, 0, T};
        return sa_shift_mlp(codes8, &all, E, d->hid, d->w1, d->w2, d->requant_scale, d->lut, nullptr, d->y, nullptr,
                            d->out_scale, d->shift_variant, 3 | SA_MLP_ACCUMULATE, ws + L.shift_ws, L.shift_ws_bytes,
                            stream);
    }
    int32_t *perm = reinterpret_cast<int32_t *>(ws + L.perm);
    int32_t *expert_of = reinterpret_cast<int32_t *>(ws + L.expert_of);
    int32_t *counts = reinterpret_cast<int32_t *>(ws + L.counts);
    float *gate = reinterpret_cast<float *>(ws + L.gate);
    rc = sa_moe_dispatch(logits, T, 2, perm, expert_of, counts, gate, ws + L.disp_ws, L.disp_ws_bytes, stream);
    if (rc != SA_OK) return rc;
    // both experts on the caller's stream; they add to disjoint rows of y
    const sa_rows mult_rows{perm, counts, 0, T};
    rc = sa_mult_mlp_f16_half(xh, &mult_rows, E, d->hid, d->mw1, d->mw2, nullptr, d->y, gate, 3 | SA_MLP_ACCUMULATE,
                              ws + L.mult_ws, L.mult_ws_bytes, stream);
    if (rc != SA_OK) return rc;
    const sa_rows shift_rows{perm, counts, 1, T};
    return sa_shift_mlp(codes8, &shift_rows, E, d->hid, d->w1, d->w2, d->requant_scale, d->lut, nullptr, d->y, gate,
                        d->out_scale, d->shift_variant, 3 | SA_MLP_ACCUMULATE, ws + L.shift_ws, L.shift_ws_bytes, stream);
}
