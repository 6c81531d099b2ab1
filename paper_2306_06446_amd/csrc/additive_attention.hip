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

template <int DV>
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
        const float sig = ((word >> lane) & 1ull) ? 1.0f : -1.0f;
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

template <int DV>
__global__ __launch_bounds__(256) void qkv_kernel(const uint64_t *__restrict__ q_codes,
                                                  const float *__restrict__ kv,
                                                  float *__restrict__ out, int H, int Nq, int W,
                                                  int n_chunks, long n_tasks, float scale) {
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
            const uint32_t s = ((half[j >> 5] << (31 - (j & 31))) & 0x80000000u) | 0x3f800000u;
            const float sig = __builtin_bit_cast(float, s);
            const float *row = kv_bh + (size_t)(w * 64 + j) * DV;                // uniform
#pragma unroll
            for (int c = 0; c < DV; ++c) acc[c] = __builtin_fmaf(sig, row[c], acc[c]);
        }
    }
    if (n < Nq) {
        float *o = out + (((size_t)b * Nq + n) * H + h) * DV;
#pragma unroll
        for (int c = 0; c < DV; c += 4)
            *reinterpret_cast<float4 *>(o + c) =
                make_float4(scale * acc[c], scale * acc[c + 1], scale * acc[c + 2], scale * acc[c + 3]);
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

extern "C" int sa_additive_attention(const uint64_t *q_codes, const uint64_t *k_codes,
                                     const float *v, float *out, int B, int H, int Nq, int Nk,
                                     int nbits, int dv, float scale, float *kv, int phases,
                                     void *workspace, size_t workspace_bytes, void *stream) {
    sa::clear_error();
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
                int rc = sa::launch_ktv_mfma(k_codes, v, dst, B, H, Nk, nbits, dv, m, st);
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
            switch (dv) {
                case 32: ktv_kernel<32><<<grid, block, 0, st>>>(k_codes, v, dst, H, Nk, W, p.splits, p.tokens_per_wave); break;
                case 64: ktv_kernel<64><<<grid, block, 0, st>>>(k_codes, v, dst, H, Nk, W, p.splits, p.tokens_per_wave); break;
                default: ktv_kernel<128><<<grid, block, 0, st>>>(k_codes, v, dst, H, Nk, W, p.splits, p.tokens_per_wave); break;
            }
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
            return sa::launch_qkv_mfma(q_codes, kv, out, B, H, Nq, nbits, dv, scale, st);
        const int n_chunks = (Nq + 63) / 64;
        const long n_tasks = BH * n_chunks;
        const long blocks = (n_tasks + 3) / 4;
        SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_additive_attention: grid too large");
        const dim3 grid((unsigned)blocks), block(256);
        switch (dv) {
            case 32: qkv_kernel<32><<<grid, block, 0, st>>>(q_codes, kv, out, H, Nq, W, n_chunks, n_tasks, scale); break;
            case 64: qkv_kernel<64><<<grid, block, 0, st>>>(q_codes, kv, out, H, Nq, W, n_chunks, n_tasks, scale); break;
            default: qkv_kernel<128><<<grid, block, 0, st>>>(q_codes, kv, out, H, Nq, W, n_chunks, n_tasks, scale); break;
        }
        return sa::check_launch("sa_additive_attention(Q(K^T V))");
    }
    return SA_OK;
}
