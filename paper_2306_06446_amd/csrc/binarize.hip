// sa_binarize: rows of Q / K -> packed binary codes (Sec. 4.1, binary quantisation
// of Q and K; appendix, "scaling factor clarification").
//
// One wavefront owns 64 code bits (one uint64 word) of up to 64 consecutive
// tokens of one (batch, head): lane j holds column j of the hash matrix in
// registers, the token's row arrives through scalar loads (it is the same for
// every lane), each lane runs the defining fp32 fma chain for its own bit and
// a wavefront-wide ballot packs the 64 sign tests into the code word.  The
// ballots of the 64 tokens are parked one per lane and leave in one store.
#include "common.h"

namespace {

using sa::kWave;

template <int D>
__global__ __launch_bounds__(256) void binarize_proj_kernel(
    const float *__restrict__ x, const float *__restrict__ proj, uint64_t *__restrict__ codes,
    int N, int H, int nbits, int n_chunks, long n_tasks) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long task = (long)blockIdx.x * (blockDim.x >> 6) + wave_in_block;
    if (task >= n_tasks) return;
    const int W = nbits >> 6;
    const int w = (int)(task % W);
    const long t2 = task / W;
    const int chunk = (int)(t2 % n_chunks);
    const long bh = t2 / n_chunks;
    const int b = (int)(bh / H), h = (int)(bh % H);

    float r[D];
#pragma unroll
    for (int k = 0; k < D; ++k) r[k] = proj[(size_t)k * nbits + w * 64 + lane];

    const int n0 = chunk * 64;
    const int rows = min(64, N - n0);
    uint64_t mine = 0;
    for (int i = 0; i < rows; ++i) {
        const float *xr = x + (((size_t)b * N + (n0 + i)) * H + h) * D;   // wave-uniform
        float acc = 0.0f;
#pragma unroll
        for (int k = 0; k < D; ++k) acc = __builtin_fmaf(xr[k], r[k], acc);
        const uint64_t word = __ballot(acc >= 0.0f);
        if (lane == i) mine = word;
    }
    if (lane < rows) codes[((size_t)bh * N + n0 + lane) * W + w] = mine;
}

// proj == NULL: bit j = [x_j >= 0]; one wavefront per 64 features of a row.
__global__ __launch_bounds__(256) void binarize_sign_kernel(const float *__restrict__ x,
                                                            uint64_t *__restrict__ codes, int N,
                                                            int H, int d, long n_words) {
    const int lane = threadIdx.x & (kWave - 1);
    const long word_id = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (word_id >= n_words) return;
    const int W = d >> 6;
    const int w = (int)(word_id % W);
    const long row = word_id / W;              // (b * N + n) * H + h
    const int h = (int)(row % H);
    const long bn = row / H;
    const long n = bn % N, b = bn / N;
    const float v = x[(size_t)row * d + w * 64 + lane];
    const uint64_t word = __ballot(v >= 0.0f);
    if (lane == 0) codes[(((size_t)b * H + h) * N + n) * W + w] = word;
}

}  // namespace

extern "C" int sa_binarize(const float *x, int B, int N, int H, int d, const float *proj,
                           int nbits, uint64_t *codes, void *stream) {
    return sa_binarize_ex(x, B, N, H, d, proj, nbits, codes, SA_VARIANT_AUTO, stream);
}

extern "C" int sa_binarize_pair(const float *q, const float *k, int B, int N, int H, int d, const float *proj,
                                int nbits, uint64_t *q_codes, uint64_t *k_codes, void *stream) {
    sa::clear_error();
    const long rows = (long)B * N * H;
    // both tensors are checked before anything is launched for either
    if (rows > 0) {
        SA_REQUIRE(q && k && q_codes && k_codes, SA_ERR_INVALID, "sa_binarize_pair: NULL buffer");
        SA_REQUIRE(sa::aligned16(q) && sa::aligned16(k) && sa::aligned16(q_codes) && sa::aligned16(k_codes), SA_ERR_ALIGN,
                   "sa_binarize_pair: pointers must be 16-byte aligned");
    }
    // one launch when the matrix-core kernel takes the shape; otherwise simply one call per tensor
    if (proj != nullptr && B > 0 && N > 0 && H > 0 && rows < (1L << 31) && sa::binarize_mfma_supported(d, nbits) &&
        nbits <= 4096 && q && k && q_codes && k_codes && sa::aligned16(q) && sa::aligned16(k) && sa::aligned16(proj) &&
        sa::aligned16(q_codes) && sa::aligned16(k_codes))
        return sa::launch_binarize_mfma(q, k, proj, q_codes, k_codes, rows, N, H, d, nbits, sa::as_stream(stream));
    const int rc = sa_binarize_ex(q, B, N, H, d, proj, nbits, q_codes, SA_VARIANT_AUTO, stream);
    if (rc != SA_OK) return rc;
    return sa_binarize_ex(k, B, N, H, d, proj, nbits, k_codes, SA_VARIANT_AUTO, stream);
}

extern "C" int sa_binarize_ex(const float *x, int B, int N, int H, int d, const float *proj,
                              int nbits, uint64_t *codes, int variant, void *stream) {
    sa::clear_error();
    SA_REQUIRE(variant >= 0 && variant <= 2, SA_ERR_INVALID, "sa_binarize: unknown variant %d", variant);
    SA_REQUIRE(B >= 0 && N >= 0 && H >= 0 && d > 0 && nbits > 0, SA_ERR_INVALID,
               "sa_binarize: negative size");
    SA_REQUIRE(nbits % 64 == 0, SA_ERR_SHAPE, "sa_binarize: nbits %d is not a multiple of 64", nbits);
    SA_REQUIRE(nbits <= 4096, SA_ERR_SHAPE, "sa_binarize: nbits %d > 4096", nbits);
    if (proj == nullptr)
        SA_REQUIRE(nbits == d, SA_ERR_SHAPE, "sa_binarize: without proj nbits (%d) must equal d (%d)",
                   nbits, d);
    const long rows = (long)B * N * H;
    SA_REQUIRE(rows < (1L << 31), SA_ERR_SHAPE, "sa_binarize: B*N*H >= 2^31");
    if (rows == 0) return SA_OK;
    SA_REQUIRE(x != nullptr && codes != nullptr, SA_ERR_INVALID, "sa_binarize: NULL buffer");
    SA_REQUIRE(sa::aligned16(x) && sa::aligned16(codes) && sa::aligned16(proj), SA_ERR_ALIGN,
               "sa_binarize: pointers must be 16-byte aligned");
    hipStream_t st = sa::as_stream(stream);
    const int W = nbits / 64;
    if (proj == nullptr) {
        const long n_words = rows * W;
        const long blocks = (n_words + 3) / 4;
        SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_binarize: too many rows");
        binarize_sign_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(x, codes, N, H, d, n_words);
        return sa::check_launch("sa_binarize(sign)");
    }
    if (variant != SA_VARIANT_VALU && sa::binarize_mfma_supported(d, nbits))
        return sa::launch_binarize_mfma(x, nullptr, proj, codes, nullptr, rows, N, H, d, nbits, st);
    SA_REQUIRE(variant != SA_VARIANT_MFMA, SA_ERR_UNSUPPORTED,
               "sa_binarize: the matrix-core variant needs d in {32, 64, 128} (got %d)", d);
    const int n_chunks = (N + 63) / 64;
    const long n_tasks = (long)B * H * n_chunks * W;
    const long blocks = (n_tasks + 3) / 4;
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_binarize: too many rows");
    const dim3 grid((unsigned)blocks), block(256);
    switch (d) {
        case 32:
            binarize_proj_kernel<32><<<grid, block, 0, st>>>(x, proj, codes, N, H, nbits, n_chunks, n_tasks);
            break;
        case 64:
            binarize_proj_kernel<64><<<grid, block, 0, st>>>(x, proj, codes, N, H, nbits, n_chunks, n_tasks);
            break;
        case 128:
            binarize_proj_kernel<128><<<grid, block, 0, st>>>(x, proj, codes, N, H, nbits, n_chunks, n_tasks);
            break;
        default:
            return sa::fail(SA_ERR_UNSUPPORTED, "sa_binarize: with proj, d must be 32, 64 or 128 (got %d)", d);
    }
    return sa::check_launch("sa_binarize(proj)");
}
