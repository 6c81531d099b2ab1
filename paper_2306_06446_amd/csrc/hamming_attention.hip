// sa_hamming_attention: quadratic attention on binary codes (Eq. 1 with Q K^T
// replaced by the Hamming similarity S = nbits - 2 * popcount(q xor k) of the
// codes; V stays fp32, Sec. 4.1).
//
// Lane i <-> query i.  Keys stream by: a key's code words and its V row are
// the same for every lane, so they arrive through scalar loads; each lane
// XORs the key code with its own query code, counts bits, turns the distance
// into an un-normalised softmax weight and accumulates weight * V row.  The
// score matrix never exists in memory (an optional second kernel dumps it).
//
// softmax(scale*S)_j = exp(-2*scale*(dist_j - dist_ref)) / sum, with dist_ref
// the distance of the largest score.  When scale >= 0 and the exponent range
// cannot underflow, dist_ref = 0 is used (no pass over the keys to find the
// row maximum); otherwise a first pass finds it per query.
#include "common.h"

namespace {

using sa::kWave;

template <int DV, int W, bool ROWREF>
__global__ __launch_bounds__(256) void hamming_kernel(const uint64_t *__restrict__ q_codes,
                                                      const uint64_t *__restrict__ k_codes,
                                                      const float *__restrict__ v,
                                                      float *__restrict__ out, int H, int Nq,
                                                      int Nk, int n_chunks, long n_tasks,
                                                      float c2 /* -2*scale*log2(e) */) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long task = (long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (task >= n_tasks) return;
    const int chunk = (int)(task % n_chunks);
    const long bh = task / n_chunks;
    const int b = (int)(bh / H), h = (int)(bh % H);
    const int i = chunk * 64 + lane;
    const int i_ld = min(i, Nq - 1);

    uint64_t q[W];
#pragma unroll
    for (int w = 0; w < W; ++w) q[w] = q_codes[((size_t)bh * Nq + i_ld) * W + w];

    const uint64_t *kc = k_codes + (size_t)bh * Nk * W;
    int dref = 0;
    if (ROWREF) {
        // the distance whose score scale*S is largest: smallest if scale >= 0 (c2 <= 0)
        int dmin = 1 << 30, dmax = -1;
        for (int j = 0; j < Nk; ++j) {
            int dist = 0;
#pragma unroll
            for (int w = 0; w < W; ++w) dist += __builtin_popcountll(q[w] ^ kc[(size_t)j * W + w]);
            dmin = min(dmin, dist);
            dmax = max(dmax, dist);
        }
        dref = (c2 <= 0.0f) ? dmin : dmax;
    }

    float acc[DV];
#pragma unroll
    for (int c = 0; c < DV; ++c) acc[c] = 0.0f;
    float den = 0.0f;
    for (int j = 0; j < Nk; ++j) {
        int dist = 0;
#pragma unroll
        for (int w = 0; w < W; ++w) dist += __builtin_popcountll(q[w] ^ kc[(size_t)j * W + w]);   // kc: uniform
        const float p = __builtin_amdgcn_exp2f(c2 * (float)(dist - dref));
        den += p;
        const float *vr = v + (((size_t)b * Nk + j) * H + h) * DV;                                // uniform
#pragma unroll
        for (int c = 0; c < DV; ++c) acc[c] = __builtin_fmaf(p, vr[c], acc[c]);
    }
    if (i < Nq) {
        const float inv = 1.0f / den;
        float *o = out + (((size_t)b * Nq + i) * H + h) * DV;
#pragma unroll
        for (int c = 0; c < DV; c += 4)
            *reinterpret_cast<float4 *>(o + c) =
                make_float4(acc[c] * inv, acc[c + 1] * inv, acc[c + 2] * inv, acc[c + 3] * inv);
    }
}

// Optional dump of the integer scores, one thread per (query, key) pair.
__global__ __launch_bounds__(256) void hamming_scores_kernel(const uint64_t *__restrict__ q_codes,
                                                             const uint64_t *__restrict__ k_codes,
                                                             int16_t *__restrict__ scores, int Nq,
                                                             int Nk, int W, long total) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int j = (int)(idx % Nk);
    const long t = idx / Nk;
    const int i = (int)(t % Nq);
    const long bh = t / Nq;
    const uint64_t *q = q_codes + ((size_t)bh * Nq + i) * W;
    const uint64_t *k = k_codes + ((size_t)bh * Nk + j) * W;
    int dist = 0;
    for (int w = 0; w < W; ++w) dist += __builtin_popcountll(q[w] ^ k[w]);
    scores[idx] = (int16_t)(W * 64 - 2 * dist);
}

template <int DV, int W>
void launch_hamming(bool rowref, dim3 grid, hipStream_t st, const uint64_t *q, const uint64_t *k,
                    const float *v, float *out, int H, int Nq, int Nk, int n_chunks, long n_tasks,
                    float c2) {
    if (rowref)
        hamming_kernel<DV, W, true><<<grid, dim3(256), 0, st>>>(q, k, v, out, H, Nq, Nk, n_chunks, n_tasks, c2);
    else
        hamming_kernel<DV, W, false><<<grid, dim3(256), 0, st>>>(q, k, v, out, H, Nq, Nk, n_chunks, n_tasks, c2);
}

template <int DV>
int dispatch_w(int W, bool rowref, dim3 grid, hipStream_t st, const uint64_t *q, const uint64_t *k,
               const float *v, float *out, int H, int Nq, int Nk, int n_chunks, long n_tasks, float c2) {
    switch (W) {
        case 1: launch_hamming<DV, 1>(rowref, grid, st, q, k, v, out, H, Nq, Nk, n_chunks, n_tasks, c2); break;
        case 2: launch_hamming<DV, 2>(rowref, grid, st, q, k, v, out, H, Nq, Nk, n_chunks, n_tasks, c2); break;
        case 4: launch_hamming<DV, 4>(rowref, grid, st, q, k, v, out, H, Nq, Nk, n_chunks, n_tasks, c2); break;
        case 8: launch_hamming<DV, 8>(rowref, grid, st, q, k, v, out, H, Nq, Nk, n_chunks, n_tasks, c2); break;
        default:
            return sa::fail(SA_ERR_UNSUPPORTED, "sa_hamming_attention: nbits must be 64, 128, 256 or 512");
    }
    return SA_OK;
}

}  // namespace

extern "C" int sa_hamming_attention(const uint64_t *q_codes, const uint64_t *k_codes, const float *v,
                                    float *out, int B, int H, int Nq, int Nk, int nbits, int dv,
                                    float scale, int16_t *scores_or_null, void *stream) {
    sa::clear_error();
    SA_REQUIRE(B >= 0 && H >= 0 && Nq >= 0 && Nk >= 0 && nbits > 0 && dv > 0, SA_ERR_INVALID,
               "sa_hamming_attention: negative size");
    SA_REQUIRE(nbits % 64 == 0, SA_ERR_SHAPE, "sa_hamming_attention: nbits %d is not a multiple of 64", nbits);
    SA_REQUIRE(nbits <= 16320, SA_ERR_SHAPE, "sa_hamming_attention: scores do not fit int16");
    SA_REQUIRE(dv == 32 || dv == 64 || dv == 128, SA_ERR_UNSUPPORTED,
               "sa_hamming_attention: dv must be 32, 64 or 128 (got %d)", dv);
    SA_REQUIRE(scale == scale && scale - scale == 0.0f, SA_ERR_INVALID, "sa_hamming_attention: scale is not finite");
    SA_REQUIRE((long)B * H < (1L << 20), SA_ERR_SHAPE, "sa_hamming_attention: B*H too large");
    if ((long)B * H == 0 || Nq == 0) return SA_OK;
    SA_REQUIRE(Nk > 0, SA_ERR_SHAPE, "sa_hamming_attention: softmax over zero keys is undefined");
    SA_REQUIRE(q_codes && k_codes && v && out, SA_ERR_INVALID, "sa_hamming_attention: NULL buffer");
    SA_REQUIRE(sa::aligned16(q_codes) && sa::aligned16(k_codes) && sa::aligned16(v) &&
                   sa::aligned16(out) && sa::aligned16(scores_or_null),
               SA_ERR_ALIGN, "sa_hamming_attention: pointers must be 16-byte aligned");
    hipStream_t st = sa::as_stream(stream);
    const int W = nbits / 64;
    const long BH = (long)B * H;
    const int n_chunks = (Nq + 63) / 64;
    const long n_tasks = BH * n_chunks;
    const long blocks = (n_tasks + 3) / 4;
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_hamming_attention: grid too large");
    const float c2 = -2.0f * scale * 1.4426950408889634f;
    // exp2 of c2*dist stays a normal float for every possible distance -> no row reference needed
    const bool rowref = !(scale >= 0.0f && -c2 * (float)nbits <= 100.0f);
    const dim3 grid((unsigned)blocks);
    int rc;
    switch (dv) {
        case 32: rc = dispatch_w<32>(W, rowref, grid, st, q_codes, k_codes, v, out, H, Nq, Nk, n_chunks, n_tasks, c2); break;
        case 64: rc = dispatch_w<64>(W, rowref, grid, st, q_codes, k_codes, v, out, H, Nq, Nk, n_chunks, n_tasks, c2); break;
        default: rc = dispatch_w<128>(W, rowref, grid, st, q_codes, k_codes, v, out, H, Nq, Nk, n_chunks, n_tasks, c2); break;
    }
    if (rc != SA_OK) return rc;
    rc = sa::check_launch("sa_hamming_attention");
    if (rc != SA_OK) return rc;
    if (scores_or_null != nullptr) {
        const long total = BH * Nq * Nk;
        const long sb = (total + 255) / 256;
        SA_REQUIRE(sb < (1L << 31), SA_ERR_SHAPE, "sa_hamming_attention: score dump too large");
        hamming_scores_kernel<<<dim3((unsigned)sb), dim3(256), 0, st>>>(q_codes, k_codes, scores_or_null,
                                                                         Nq, Nk, W, total);
        return sa::check_launch("sa_hamming_attention(scores)");
    }
    return SA_OK;
}
