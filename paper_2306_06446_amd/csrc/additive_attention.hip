// sa_additive_attention: K^T V and Q (K^T V) as Add layers (Eq. 3, O_Add; Sec. 4.1,
// MatMul order exchanged to Q(KV); appendix: the scale is multiplied after the adds).
//
// Both kernels are sign-select-and-accumulate on the vector ALU: the operand
// that every lane shares (a row of V, a row of K^T V) arrives through scalar
// loads and is consumed straight from scalar registers; the sign each lane
// applies comes from its own code bit.  acc = fma(+-1.0f, v, acc) is an exact
// add or subtract (the product never rounds) and issues at the rate of v_add.
//
//   K^T V   : lane j  <-> code bit j of one 64-bit word, accumulators = the dv
//             columns of row j; tokens stream by, split over wavefronts and
//             workgroups, partial sums meet in LDS and then in a second pass,
//             always in the same order.
//   Q(K^T V): lane n  <-> token n, accumulators = the dv outputs of the token.
#include "common.h"

namespace {

using sa::kWave;

constexpr int kKtvWaves = 4;   // wavefronts per workgroup that share one (b, h, word)

template <int DV, bool ZO>
__global__ __launch_bounds__(256) void ktv_kernel(const uint64_t *__restrict__ k_codes,
                                                  const float *__restrict__ v,
                                                  float *__restrict__ dst, int H, int Nk, int W,
                                                  int splits, int tokens_per_wave) {
    __shared__ float red[kWave * DV];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // blockIdx.x = (bh * W + w) * splits + split
    const int split = blockIdx.x % splits;
    const long bhw = blockIdx.x / splits;
    const int w = (int)(bhw % W);
    const long bh = bhw / W;
    const int b = (int)(bh / H), h = (int)(bh % H);

    float acc[DV];
#pragma unroll
    for (int c = 0; c < DV; ++c) acc[c] = 0.0f;

    const long first = ((long)split * kKtvWaves + wave) * tokens_per_wave;
    const long last = min((long)Nk, first + tokens_per_wave);
    for (long n = first; n < last; ++n) {
        const uint64_t word = k_codes[((size_t)bh * Nk + n) * W + w];           // uniform
        const float *vr = v + (((size_t)b * Nk + n) * H + h) * DV;              // uniform
        const float sig = ((word >> lane) & 1ull) ? 1.0f : (ZO ? 0.0f : -1.0f);
#pragma unroll
        for (int c = 0; c < DV; ++c) acc[c] = __builtin_fmaf(sig, vr[c], acc[c]);
    }

    // cross-wavefront reduction through LDS, fixed order ((w0 + w1) + w2) + w3
    for (int s = 1; s < kKtvWaves; ++s) {
        if (wave == s) {
#pragma unroll
            for (int c = 0; c < DV; ++c) red[c * kWave + lane] = acc[c];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int c = 0; c < DV; ++c) acc[c] += red[c * kWave + lane];
        }
        __syncthreads();
    }
    if (wave == 0) {
        // dst: [splits][BH][nbits][DV]; row = w*64 + lane
        const size_t BH_rows = (size_t)gridDim.x / splits * 64;   // BH * W * 64 = BH * nbits
        float *o = dst + ((size_t)split * BH_rows + (size_t)bhw * 64 + lane) * DV;
#pragma unroll
        for (int c = 0; c < DV; c += 4)
            *reinterpret_cast<float4 *>(o + c) = make_float4(acc[c], acc[c + 1], acc[c + 2], acc[c + 3]);
    }
}

// kv[i] = sum over splits of part[s][i], s ascending.
__global__ __launch_bounds__(256) void ktv_reduce_kernel(const float4 *__restrict__ part,
                                                         float4 *__restrict__ kv, long n4,
                                                         int splits) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    float4 a = part[i];
    for (int s = 1; s < splits; ++s) {
        const float4 p = part[(size_t)s * n4 + i];
        a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
    }
    kv[i] = a;
}

template <int DV, bool ZO>
__global__ __launch_bounds__(256) void qkv_kernel(const uint64_t *__restrict__ q_codes,
                                                  const float *__restrict__ kv,
                                                  float *__restrict__ out, int H, int Nq, int W,
                                                  int n_chunks, long n_tasks, float scale,
                                                  const int32_t *__restrict__ den, float eps) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long task = (long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (task >= n_tasks) return;
    const int chunk = (int)(task % n_chunks);
    const long bh = task / n_chunks;
    const int b = (int)(bh / H), h = (int)(bh % H);
    const int n = chunk * 64 + lane;
    const int n_ld = min(n, Nq - 1);

    float acc[DV];
#pragma unroll
    for (int c = 0; c < DV; ++c) acc[c] = 0.0f;

    const uint64_t *code = q_codes + ((size_t)bh * Nq + n_ld) * W;
    const float *kv_bh = kv + (size_t)bh * W * 64 * DV;
    for (int w = 0; w < W; ++w) {
        const uint64_t word = ~code[w];
        const uint32_t half[2] = {(uint32_t)word, (uint32_t)(word >> 32)};
#pragma unroll
        for (int j = 0; j < 64; ++j) {
            // bit 1 -> +1.0f, bit 0 -> -1.0f: move the inverted bit into the float sign
            // ({0,1} codes: bit 1 -> 1.0f, bit 0 -> 0.0f; `word` is the inverted code)
            const uint32_t s = ZO ? ((~half[j >> 5] >> (j & 31)) & 1u) * 0x3f800000u
                                  : ((half[j >> 5] << (31 - (j & 31))) & 0x80000000u) | 0x3f800000u;
            const float sig = __builtin_bit_cast(float, s);
            const float *row = kv_bh + (size_t)(w * 64 + j) * DV;                // uniform
#pragma unroll
            for (int c = 0; c < DV; ++c) acc[c] = __builtin_fmaf(sig, row[c], acc[c]);
        }
    }
    if (n < Nq) {
        float *o = out + (((size_t)b * Nq + n) * H + h) * DV;
        const float f = den ? 1.0f / ((float)den[(size_t)bh * Nq + n] + eps) : scale;
#pragma unroll
        for (int c = 0; c < DV; c += 4)
            *reinterpret_cast<float4 *>(o + c) = make_float4(f * acc[c], f * acc[c + 1], f * acc[c + 2], f * acc[c + 3]);
    }
}

// ksum[bh, j] += number of tokens of the block's range whose code bit j is set (lane <-> bit of one word).
// The code words are wave-uniform; eight are fetched before any is used so that their latencies overlap.
__global__ __launch_bounds__(256) void bit_count_kernel(const uint64_t *__restrict__ k_codes, int32_t *__restrict__ ksum,
                                                        int Nk, int W, int splits, int tokens_per_wave) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int split = blockIdx.x % splits;
    const long bhw = blockIdx.x / splits;
    const int w = (int)(bhw % W);
    const long bh = bhw / W;
    const long first = ((long)split * 4 + wave) * tokens_per_wave;
    const long last = min((long)Nk, first + tokens_per_wave);
    const uint64_t *base = k_codes + (size_t)bh * Nk * W + w;
    int32_t cnt = 0;
    long n = first;
    for (; n + 8 <= last; n += 8) {
        uint64_t wd[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) wd[t] = base[(size_t)(n + t) * W];             // uniform
#pragma unroll
        for (int t = 0; t < 8; ++t) cnt += (int32_t)((wd[t] >> lane) & 1ull);
    }
    for (; n < last; ++n) cnt += (int32_t)((base[(size_t)n * W] >> lane) & 1ull);
    if (cnt) atomicAdd(ksum + (size_t)bhw * 64 + lane, cnt);                        // integers: order-independent
}

// den[bh, n] = sum over the set bits j of query n's code of ksum[bh, j]  (thread <-> query).  The sums of every
// 4-bit group over its 16 possible nibbles are tabulated in LDS first (nbits / 4 groups x 16 entries), so a query
// costs one table read per nibble of its code.
__global__ __launch_bounds__(256) void den_kernel(const uint64_t *__restrict__ q_codes, const int32_t *__restrict__ ksum,
                                                  int32_t *__restrict__ den, int Nq, int W, int n_chunks) {
    extern __shared__ int32_t tab[];                 // [W * 16 groups][16]
    const long bh = blockIdx.x / n_chunks;
    const int chunk = blockIdx.x % n_chunks;
    const int n_entries = W * 16 * 16;
    for (int i = threadIdx.x; i < n_entries; i += blockDim.x) {
        const int g = i >> 4, nib = i & 15;
        const int32_t *k4 = ksum + (size_t)bh * W * 64 + g * 4;
        tab[i] = ((nib & 1) ? k4[0] : 0) + ((nib & 2) ? k4[1] : 0) + ((nib & 4) ? k4[2] : 0) + ((nib & 8) ? k4[3] : 0);
    }
    __syncthreads();
    const int n = chunk * 256 + threadIdx.x;
    if (n >= Nq) return;
    const uint64_t *code = q_codes + ((size_t)bh * Nq + n) * W;
    int32_t d = 0;
    for (int w = 0; w < W; ++w) {
        const uint64_t word = code[w];
        const uint32_t half[2] = {(uint32_t)word, (uint32_t)(word >> 32)};
#pragma unroll
        for (int g = 0; g < 16; ++g) d += tab[((w * 16 + g) << 4) + ((half[g >> 3] >> (4 * (g & 7))) & 15u)];
    }
    den[(size_t)bh * Nq + n] = d;
}

// Depthwise 3x3 over the token grid, zero padding; thread <-> four channels of one token, a few items per
// thread.  The weights pass through LDS transposed to [tap][channel] so that a lane reads its four channels' weights
// of a tap as one 16-byte word (their [channel][tap] layout in memory would make every lane touch another line).
constexpr int kDwMaxItems = 8;
constexpr int kDwMaxLdsE = 1024;      // 36 KB of weights in LDS; wider layers read them from memory

__global__ __launch_bounds__(256) void dwconv3x3_kernel(const float *__restrict__ v, const float *__restrict__ w,
                                                        const float *__restrict__ bias, float *__restrict__ out,
                                                        int accumulate, long n_tokens, int gh, int gw, int E4,
                                                        int items) {
    extern __shared__ float w_s[];                   // [9][E], or unused when E is too wide
    const int E = E4 * 4;
    const bool staged = E <= kDwMaxLdsE;
    if (staged) {
        for (int i = threadIdx.x; i < 9 * E; i += blockDim.x) w_s[(i % 9) * E + i / 9] = w[i];
        __syncthreads();
    }
    const long total = n_tokens * E4;
    for (int it = 0; it < items; ++it) {
        const long i = ((long)blockIdx.x * items + it) * blockDim.x + threadIdx.x;
        if (i >= total) return;
        const int c4 = (int)(i % E4);
        const long tok = i / E4;
        const int x = (int)(tok % gw), y = (int)((tok / gw) % gh);
        const int c = c4 * 4;
        float acc[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[q] = bias ? bias[c + q] : 0.0f;
#pragma unroll
        for (int dy = -1; dy <= 1; ++dy)
#pragma unroll
            for (int dx = -1; dx <= 1; ++dx) {
                const int yy = y + dy, xx = x + dx;
                if (yy < 0 || yy >= gh || xx < 0 || xx >= gw) continue;
                const float4 nv = *reinterpret_cast<const float4 *>(v + (size_t)(tok + (long)dy * gw + dx) * E + c);
                const int t = (dy + 1) * 3 + (dx + 1);
                float4 wt;
                if (staged)
                    wt = *reinterpret_cast<const float4 *>(w_s + t * E + c);
                else
                    wt = make_float4(w[(size_t)(c + 0) * 9 + t], w[(size_t)(c + 1) * 9 + t], w[(size_t)(c + 2) * 9 + t],
                                     w[(size_t)(c + 3) * 9 + t]);
                acc[0] = __builtin_fmaf(wt.x, nv.x, acc[0]);
                acc[1] = __builtin_fmaf(wt.y, nv.y, acc[1]);
                acc[2] = __builtin_fmaf(wt.z, nv.z, acc[2]);
                acc[3] = __builtin_fmaf(wt.w, nv.w, acc[3]);
            }
        float4 *o = reinterpret_cast<float4 *>(out + (size_t)tok * E + c);
        float4 r = make_float4(acc[0], acc[1], acc[2], acc[3]);
        if (accumulate) {
            const float4 old = *o;
            r.x += old.x; r.y += old.y; r.z += old.z; r.w += old.w;
        }
        *o = r;
    }
}

struct KtvPlan {
    int splits;            // workgroups per (b, h, word)
    int tokens_per_wave;
};

KtvPlan plan_ktv(int B, int H, int Nk, int nbits) {
    const long groups = (long)B * H * (nbits / 64);
    // aim at ~4096 wavefronts in flight, at least 64 tokens per wavefront
    long splits = (1024 + groups - 1) / groups;
    const long max_splits = ((long)Nk + 64 * kKtvWaves - 1) / (64 * kKtvWaves);
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    if (splits > 64) splits = 64;
    const long waves = splits * kKtvWaves;
    KtvPlan p;
    p.splits = (int)splits;
    p.tokens_per_wave = (int)(((long)Nk + waves - 1) / waves);
    if (p.tokens_per_wave < 1) p.tokens_per_wave = 1;
    return p;
}

bool dv_ok(int dv) { return dv == 32 || dv == 64 || dv == 128; }

}  // namespace

extern "C" size_t sa_additive_attention_workspace_bytes(int B, int H, int Nk, int nbits, int dv) {
    if (B <= 0 || H <= 0 || Nk <= 0 || nbits <= 0 || dv <= 0 || nbits % 64) return 0;
    // room for whichever variant runs: partial sums [splits][B*H][nbits][dv]
    const KtvPlan p = plan_ktv(B, H, Nk, nbits);
    int splits = p.splits;
    if (sa::additive_mfma_ktv_supported(nbits, dv)) {
        const sa::AdditiveMfmaPlan m = sa::plan_additive_mfma(B, H, Nk, nbits);
        if (m.splits > splits) splits = m.splits;
    }
    if (splits <= 1) return 0;
    return (size_t)splits * B * H * nbits * dv * sizeof(float);
}

namespace {

// The two Add layers.  zero_one: a clear code bit contributes nothing instead of -V; den (with zero_one) is the
// row normaliser int32 [B*H, Nq]: rows leave as acc / (den + eps) instead of scale * acc.
struct AddMode {
    bool zero_one = false;
    const int32_t *den = nullptr;
    float eps = 0.0f;
};

int run_additive(const uint64_t *q_codes, const uint64_t *k_codes, const float *v, float *out, int B, int H, int Nq,
                 int Nk, int nbits, int dv, float scale, float *kv, int phases, void *workspace,
                 size_t workspace_bytes, void *stream, const AddMode &mode) {
    SA_REQUIRE(phases >= 1 && phases <= 7 && (phases & 3) != 0, SA_ERR_INVALID,
               "sa_additive_attention: phases must be 1, 2 or 3, optionally + 4");
    const bool valu = (phases & SA_ADDITIVE_VALU) != 0;
    SA_REQUIRE(B >= 0 && H >= 0 && Nq >= 0 && Nk >= 0 && nbits > 0 && dv > 0, SA_ERR_INVALID,
               "sa_additive_attention: negative size");
    SA_REQUIRE(nbits % 64 == 0 && nbits <= 4096, SA_ERR_SHAPE,
               "sa_additive_attention: nbits %d must be a multiple of 64, at most 4096", nbits);
    SA_REQUIRE(dv_ok(dv), SA_ERR_UNSUPPORTED, "sa_additive_attention: dv must be 32, 64 or 128 (got %d)", dv);
    SA_REQUIRE((long)B * H < (1L << 20), SA_ERR_SHAPE, "sa_additive_attention: B*H too large");
    if ((long)B * H == 0) return SA_OK;
    SA_REQUIRE(kv != nullptr, SA_ERR_INVALID, "sa_additive_attention: kv is NULL");
    SA_REQUIRE(sa::aligned16(q_codes) && sa::aligned16(k_codes) && sa::aligned16(v) &&
                   sa::aligned16(out) && sa::aligned16(kv) && sa::aligned16(workspace),
               SA_ERR_ALIGN, "sa_additive_attention: pointers must be 16-byte aligned");
    hipStream_t st = sa::as_stream(stream);
    const int W = nbits / 64;
    const long BH = (long)B * H;

    if (phases & 1) {
        const size_t kv_elems = (size_t)BH * nbits * dv;
        if (Nk == 0) {
            int rc = sa::launch_zero(kv, kv_elems * sizeof(float), st);   // empty sum
            if (rc != SA_OK) return rc;
        } else {
            SA_REQUIRE(k_codes != nullptr && v != nullptr, SA_ERR_INVALID,
                       "sa_additive_attention: phase 1 needs k_codes and v");
            if (!valu && sa::additive_mfma_ktv_supported(nbits, dv)) {
                const sa::AdditiveMfmaPlan m = sa::plan_additive_mfma(B, H, Nk, nbits);
                float *dst = kv;
                if (m.splits > 1) {
                    const size_t need = (size_t)m.splits * kv_elems * sizeof(float);
                    SA_REQUIRE(workspace != nullptr && workspace_bytes >= need, SA_ERR_WORKSPACE,
                               "sa_additive_attention: workspace of %zu bytes needed, %zu given", need,
                               workspace_bytes);
                    dst = static_cast<float *>(workspace);
                }
                int rc = sa::launch_ktv_mfma(k_codes, v, dst, B, H, Nk, nbits, dv, m, mode.zero_one, st);
                if (rc != SA_OK) return rc;
                if (m.splits > 1) {
                    const long n4 = (long)(kv_elems / 4);
                    ktv_reduce_kernel<<<dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st>>>(
                        reinterpret_cast<const float4 *>(dst), reinterpret_cast<float4 *>(kv), n4, m.splits);
                    rc = sa::check_launch("sa_additive_attention(reduce)");
                    if (rc != SA_OK) return rc;
                }
            } else {
            const KtvPlan p = plan_ktv(B, H, Nk, nbits);
            float *dst = kv;
            if (p.splits > 1) {
                const size_t need = (size_t)p.splits * kv_elems * sizeof(float);
                SA_REQUIRE(workspace != nullptr && workspace_bytes >= need, SA_ERR_WORKSPACE,
                           "sa_additive_attention: workspace of %zu bytes needed, %zu given", need,
                           workspace_bytes);
                dst = static_cast<float *>(workspace);
            }
            const long blocks = BH * W * p.splits;
            SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_additive_attention: grid too large");
            const dim3 grid((unsigned)blocks), block(kKtvWaves * kWave);
#define SA_KTV(DV_, ZO_) ktv_kernel<DV_, ZO_><<<grid, block, 0, st>>>(k_codes, v, dst, H, Nk, W, p.splits, p.tokens_per_wave)
            switch (dv) {
                case 32: if (mode.zero_one) SA_KTV(32, true); else SA_KTV(32, false); break;
                case 64: if (mode.zero_one) SA_KTV(64, true); else SA_KTV(64, false); break;
                default: if (mode.zero_one) SA_KTV(128, true); else SA_KTV(128, false); break;
            }
#undef SA_KTV
            int rc = sa::check_launch("sa_additive_attention(K^T V)");
            if (rc != SA_OK) return rc;
            if (p.splits > 1) {
                const long n4 = (long)(kv_elems / 4);
                ktv_reduce_kernel<<<dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st>>>(
                    reinterpret_cast<const float4 *>(dst), reinterpret_cast<float4 *>(kv), n4, p.splits);
                rc = sa::check_launch("sa_additive_attention(reduce)");
                if (rc != SA_OK) return rc;
            }
            }
        }
    }
    if ((phases & 2) && Nq > 0) {
        SA_REQUIRE(q_codes != nullptr && out != nullptr, SA_ERR_INVALID,
                   "sa_additive_attention: phase 2 needs q_codes and out");
        if (!valu && sa::additive_mfma_qkv_supported(nbits, dv))
            return sa::launch_qkv_mfma(q_codes, kv, out, B, H, Nq, nbits, dv, scale, mode.zero_one, mode.den, mode.eps, st);
        const int n_chunks = (Nq + 63) / 64;
        const long n_tasks = BH * n_chunks;
        const long blocks = (n_tasks + 3) / 4;
        SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_additive_attention: grid too large");
        const dim3 grid((unsigned)blocks), block(256);
#define SA_QKV(DV_, ZO_) \
    qkv_kernel<DV_, ZO_><<<grid, block, 0, st>>>(q_codes, kv, out, H, Nq, W, n_chunks, n_tasks, scale, mode.den, mode.eps)
        switch (dv) {
            case 32: if (mode.zero_one) SA_QKV(32, true); else SA_QKV(32, false); break;
            case 64: if (mode.zero_one) SA_QKV(64, true); else SA_QKV(64, false); break;
            default: if (mode.zero_one) SA_QKV(128, true); else SA_QKV(128, false); break;
        }
#undef SA_QKV
        return sa::check_launch("sa_additive_attention(Q(K^T V))");
    }
    return SA_OK;
}

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

extern "C" int sa_additive_attention(const uint64_t *q_codes, const uint64_t *k_codes,
                                     const float *v, float *out, int B, int H, int Nq, int Nk,
                                     int nbits, int dv, float scale, float *kv, int phases,
                                     void *workspace, size_t workspace_bytes, void *stream) {
    sa::clear_error();
    return run_additive(q_codes, k_codes, v, out, B, H, Nq, Nk, nbits, dv, scale, kv, phases, workspace, workspace_bytes,
                        stream, AddMode{});
}

extern "C" size_t sa_linear_attention_01_workspace_bytes(int B, int H, int Nq, int Nk, int nbits, int dv) {
    if (B <= 0 || H <= 0 || Nq < 0 || Nk < 0 || nbits <= 0 || dv <= 0 || nbits % 64) return 0;
    const size_t a = up256(sa_additive_attention_workspace_bytes(B, H, Nk, nbits, dv));
    return a + up256((size_t)B * H * (Nq > 0 ? Nq : 1) * sizeof(int32_t));
}

extern "C" int sa_linear_attention_01(const uint64_t *q_codes, const uint64_t *k_codes, const float *v, float *out,
                                      int B, int H, int Nq, int Nk, int nbits, int dv, float eps, float *kv,
                                      int32_t *ksum, int phases, void *workspace, size_t workspace_bytes,
                                      void *stream) {
    sa::clear_error();
    SA_REQUIRE(phases >= 1 && phases <= 7 && (phases & 3) != 0, SA_ERR_INVALID,
               "sa_linear_attention_01: phases must be 1, 2 or 3, optionally + 4");
    SA_REQUIRE(B >= 0 && H >= 0 && Nq >= 0 && Nk >= 0 && nbits > 0 && dv > 0, SA_ERR_INVALID,
               "sa_linear_attention_01: negative size");
    SA_REQUIRE(nbits % 64 == 0 && nbits <= 4096, SA_ERR_SHAPE,
               "sa_linear_attention_01: nbits %d must be a multiple of 64, at most 4096", nbits);
    SA_REQUIRE((long)Nk * nbits < (1L << 31), SA_ERR_SHAPE, "sa_linear_attention_01: the normaliser does not fit int32");
    SA_REQUIRE(eps > 0.0f && eps - eps == 0.0f, SA_ERR_INVALID, "sa_linear_attention_01: eps must be positive and finite");
    SA_REQUIRE((long)B * H < (1L << 20), SA_ERR_SHAPE, "sa_linear_attention_01: B*H too large");
    if ((long)B * H == 0) return SA_OK;
    SA_REQUIRE(ksum != nullptr, SA_ERR_INVALID, "sa_linear_attention_01: ksum is NULL");
    SA_REQUIRE(sa::aligned16(ksum) && sa::aligned16(workspace) && sa::aligned16(q_codes) && sa::aligned16(k_codes),
               SA_ERR_ALIGN, "sa_linear_attention_01: pointers must be 16-byte aligned");
    const size_t need = sa_linear_attention_01_workspace_bytes(B, H, Nq, Nk, nbits, dv);
    SA_REQUIRE(workspace != nullptr && workspace_bytes >= need, SA_ERR_WORKSPACE,
               "sa_linear_attention_01: workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    const size_t add_ws = up256(sa_additive_attention_workspace_bytes(B, H, Nk, nbits, dv));
    int32_t *den = reinterpret_cast<int32_t *>(static_cast<uint8_t *>(workspace) + add_ws);
    hipStream_t st = sa::as_stream(stream);
    const int W = nbits / 64;
    const long BH = (long)B * H;
    AddMode mode;
    mode.zero_one = true;
    if (phases & 1) {
        int rc = run_additive(nullptr, k_codes, v, nullptr, B, H, 0, Nk, nbits, dv, 1.0f, kv, 1 | (phases & SA_ADDITIVE_VALU),
                              workspace, add_ws, stream, mode);
        if (rc != SA_OK) return rc;
        rc = sa::launch_zero(ksum, (size_t)BH * nbits * sizeof(int32_t), st);
        if (rc != SA_OK) return rc;
        if (Nk > 0) {
            SA_REQUIRE(k_codes != nullptr, SA_ERR_INVALID, "sa_linear_attention_01: phase 1 needs k_codes");
            // about 64 tokens per wavefront (eight batches of eight loads): short dependent chains, many wavefronts
            long splits = ((long)Nk + 255) / 256;
            if (splits > 1024) splits = 1024;
            const int tokens_per_wave = (int)(((long)Nk + splits * 4 - 1) / (splits * 4));
            const long blocks = BH * W * splits;
            SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_linear_attention_01: grid too large");
            bit_count_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(k_codes, ksum, Nk, W, (int)splits, tokens_per_wave);
            rc = sa::check_launch("sa_linear_attention_01(bit counts)");
            if (rc != SA_OK) return rc;
        }
    }
    if ((phases & 2) && Nq > 0) {
        SA_REQUIRE(q_codes != nullptr && out != nullptr, SA_ERR_INVALID, "sa_linear_attention_01: phase 2 needs q_codes and out");
        const int n_chunks = (Nq + 255) / 256;
        const long blocks = BH * n_chunks;
        SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_linear_attention_01: grid too large");
        den_kernel<<<dim3((unsigned)blocks), dim3(256), (size_t)nbits * 4 * sizeof(int32_t), st>>>(q_codes, ksum, den, Nq, W, n_chunks);
        int rc = sa::check_launch("sa_linear_attention_01(normaliser)");
        if (rc != SA_OK) return rc;
        mode.den = den;
        mode.eps = eps;
        return run_additive(q_codes, nullptr, nullptr, out, B, H, Nq, Nk, nbits, dv, 1.0f, kv, 2 | (phases & SA_ADDITIVE_VALU),
                            workspace, add_ws, stream, mode);
    }
    return SA_OK;
}

extern "C" int sa_dwconv3x3(const float *v, const float *w, const float *bias_or_null, float *out, int accumulate,
                            int B, int gh, int gw, int E, void *stream) {
    sa::clear_error();
    SA_REQUIRE(B >= 0 && gh >= 0 && gw >= 0 && E >= 0, SA_ERR_INVALID, "sa_dwconv3x3: negative size");
    SA_REQUIRE(E % 4 == 0, SA_ERR_SHAPE, "sa_dwconv3x3: E (%d) must be a multiple of 4", E);
    const long n_tokens = (long)B * gh * gw;
    if (n_tokens == 0 || E == 0) return SA_OK;
    SA_REQUIRE(v && w && out, SA_ERR_INVALID, "sa_dwconv3x3: NULL buffer");
    SA_REQUIRE(v != out, SA_ERR_INVALID, "sa_dwconv3x3: out must not be v (neighbours are read after they would be written)");
    SA_REQUIRE(sa::aligned16(v) && sa::aligned16(w) && sa::aligned16(bias_or_null) && sa::aligned16(out), SA_ERR_ALIGN,
               "sa_dwconv3x3: pointers must be 16-byte aligned");
    const long n = n_tokens * (E / 4);
    // several items per thread amortise the staging of the weights, as long as the grid still fills the chip
    int items = (int)(n / (256L * 2048));
    items = items < 1 ? 1 : (items > kDwMaxItems ? kDwMaxItems : items);
    const long per_block = 256L * items;
    const long blocks = (n + per_block - 1) / per_block;
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_dwconv3x3: too many elements");
    const size_t lds = E <= kDwMaxLdsE ? (size_t)9 * E * sizeof(float) : 0;
    dwconv3x3_kernel<<<dim3((unsigned)blocks), dim3(256), lds, sa::as_stream(stream)>>>(v, w, bias_or_null, out, accumulate,
                                                                                         n_tokens, gh, gw, E / 4, items);
    return sa::check_launch("sa_dwconv3x3");
}
