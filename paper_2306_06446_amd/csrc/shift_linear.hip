// Shift layers (Eq. 3, O_Shift = sum X * s * 2^P) on int8 activations, int32 accumulation,
// 4-bit weights (neg << 3) | e with value (neg ? -1 : +1) << e.
//
// Two bit-exact variants:
//   VALU  : true shift-and-accumulate.  -(x << e) = ((~x) << e) + (1 << e), so a
//           negative weight is "xor the activation with all-ones, shift, add" and
//           the (1 << e) terms, which depend on the weights only, are summed once
//           per output column through a virtual all-zero activation row.
//   MFMA  : the 4-bit weights are decoded once per call to two int8 planes,
//           A = s * 2^min(e,6) and B = s * 64 * [e == 7] (+128 is not an int8),
//           and both planes go through v_mfma_i32_32x32x32_i8 into one accumulator.
// Both share the epilogues (plain int32, requantise + table, gated fp32 scatter).
#include "common.h"
#include "gemm_common.h"
#include "gemm_mfma.h"

namespace {

using namespace sa;

template <int MODE>
__device__ inline void epi_store(const Epilogue &e, long m, int n, int N, int32_t acc,
                                 const int32_t *rows) {
    if (MODE == kEpiInt32) {
        e.y[(size_t)m * N + n] = acc + (e.bias ? e.bias[n] : 0);
    } else if (MODE == kEpiRequantLut) {
        const float t = (float)acc * e.rq;
        e.h[(size_t)m * N + n] = e.lut[(int)requant_code(t) + 128];
    } else if (MODE == kEpiLinearF32) {
        const float res = e.residual ? e.residual[(size_t)m * N + n] : 0.0f;
        const int part = n / e.part_width;
        e.parts[part][(size_t)m * e.part_width + (n - part * e.part_width)] = __builtin_fmaf((float)acc, e.lin_scale, res);
    } else {
        const long t = rows ? rows[m] : m;
        const float g = e.gate ? e.gate[t] : 1.0f;
        const float val = e.out_scale * (float)acc;
        float *dst = e.yf + (size_t)t * N + n;
        *dst = e.accumulate ? __builtin_fmaf(g, val, *dst) : g * val;
    }
}

// ------------------------------------------------------------------ VALU variant ----
// thread <-> output column n; MT activation rows per workgroup pass, their bytes
// arrive through scalar loads (they are the same for every lane).
constexpr int kValuRows = 8;

template <int MODE>
__global__ __launch_bounds__(256) void shift_valu_kernel(const int8_t *__restrict__ x,
                                                         const uint8_t *__restrict__ w4,
                                                         RowSel sel, bool gather, int K, int N,
                                                         Epilogue epi) {
    const int32_t *rows;
    long n_rows;
    resolve_rows(sel, rows, n_rows);
    const long m0 = (long)blockIdx.y * kValuRows;
    if (m0 >= n_rows) return;
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    const int n_ld = min(n, N - 1);
    const uint4 *wrow = reinterpret_cast<const uint4 *>(w4 + (size_t)n_ld * (K / 2));

    const int8_t *xr[kValuRows];
#pragma unroll
    for (int i = 0; i < kValuRows; ++i) {
        const long m = min(m0 + i, n_rows - 1);
        const long src = (gather && rows) ? rows[m] : m;
        xr[i] = x + (size_t)src * K;                      // wave-uniform
    }
    uint32_t acc[kValuRows + 1];
#pragma unroll
    for (int i = 0; i <= kValuRows; ++i) acc[i] = 0u;

    const int k32 = K / 32;
    for (int kb = 0; kb < k32; ++kb) {
        const uint4 wv = wrow[kb];
        const uint32_t wd[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t e = (wd[q] >> (4 * i)) & 7u;
                const uint32_t msk = (uint32_t)((int32_t)(wd[q] << (28 - 4 * i)) >> 31);   // 0 or ~0
                const int k = kb * 32 + q * 8 + i;
#pragma unroll
                for (int r = 0; r < kValuRows; ++r) {
                    const uint32_t xv = (uint32_t)(int32_t)xr[r][k];
                    acc[r] += (xv ^ msk) << e;
                }
                acc[kValuRows] += msk << e;               // the virtual row x = 0
            }
        }
    }
    // K % 32 tail, one byte (two weights) at a time
    for (int k = k32 * 32; k < K; k += 2) {
        const uint32_t byte = w4[(size_t)n_ld * (K / 2) + (k >> 1)];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t nib = (byte >> (4 * i)) & 15u;
            const uint32_t e = nib & 7u;
            const uint32_t msk = (nib & 8u) ? ~0u : 0u;
#pragma unroll
            for (int r = 0; r < kValuRows; ++r) {
                const uint32_t xv = (uint32_t)(int32_t)xr[r][k + i];
                acc[r] += (xv ^ msk) << e;
            }
            acc[kValuRows] += msk << e;
        }
    }
    if (n < N) {
#pragma unroll
        for (int r = 0; r < kValuRows; ++r)
            if (m0 + r < n_rows)
                epi_store<MODE>(epi, m0 + r, n, N, (int32_t)(acc[r] - acc[kValuRows]), rows);
    }
}

// ------------------------------------------------------------------ MFMA variant ----
// Step 1: decode the 4-bit weights once per call into two int8 planes [N, K] in the
// workspace (they stay in the last-level cache); step 2: the shared tiled GEMM runs
// both planes into one int32 accumulator.
__device__ inline uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel) {
    return __builtin_amdgcn_perm(hi, lo, sel);
}

// 8 nibbles of `x` (k ascending from bit 0) -> 8 int8 of plane A and 8 of plane B, k order.
__device__ inline void decode8(uint32_t x, uint32_t outA[2], uint32_t outB[2]) {
    // magnitude tables indexed by e: bytes 0..3 in the low word, 4..7 in the high word
    constexpr uint32_t TA_LO = 0x08040201u, TA_HI = 0x40402010u;   // 1 2 4 8 | 16 32 64 64
    constexpr uint32_t TB_LO = 0x00000000u, TB_HI = 0x40000000u;   // 0 .. 0 64
    const uint32_t nibs[2] = {x & 0x0F0F0F0Fu, (x >> 4) & 0x0F0F0F0Fu};   // even k, odd k
    uint32_t a[2], b[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const uint32_t sel = nibs[p] & 0x07070707u;
        const uint32_t s1 = (nibs[p] >> 3) & 0x01010101u;          // 1 where negative
        const uint32_t m = s1 * 0xFFu;                             // 0xFF where negative
        const uint32_t pa = perm(TA_HI, TA_LO, sel);
        const uint32_t pb = perm(TB_HI, TB_LO, sel);
        a[p] = (pa ^ m) + s1;                 // per byte: ~pa + 1 = -pa (pa >= 1: no carry)
        b[p] = pb | (m & (pb << 1));          // 0x40 -> 0xC0 = -64 where negative
    }
    // interleave even / odd back into k order: k0 k1 k2 k3 | k4 k5 k6 k7
    outA[0] = perm(a[1], a[0], 0x05010400u);
    outA[1] = perm(a[1], a[0], 0x07030602u);
    outB[0] = perm(b[1], b[0], 0x05010400u);
    outB[1] = perm(b[1], b[0], 0x07030602u);
}

// One thread per 32 weights of a padded plane row (row_chunks of them, the first valid_chunks from 16 bytes of
// packed weights each, the others zero): 32 B out to each plane.
__global__ __launch_bounds__(256) void decode_w4_kernel(const uint4 *__restrict__ w4, long n_chunks,
                                                        uint4 *__restrict__ plane_a, uint4 *__restrict__ plane_b,
                                                        int valid_chunks, int row_chunks) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_chunks) return;
    uint4 wv;
    if (valid_chunks == row_chunks) {
        wv = w4[i];
    } else {
        const long n = i / row_chunks;
        const int kc = (int)(i - n * row_chunks);
        if (kc >= valid_chunks) {
            const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
            plane_a[2 * i] = plane_a[2 * i + 1] = plane_b[2 * i] = plane_b[2 * i + 1] = zero;
            return;
        }
        wv = w4[n * valid_chunks + kc];
    }
    const uint32_t wd[4] = {wv.x, wv.y, wv.z, wv.w};
    uint32_t oa[8], ob[8];
#pragma unroll
    for (int q = 0; q < 4; ++q) decode8(wd[q], oa + 2 * q, ob + 2 * q);
    plane_a[2 * i] = make_uint4(oa[0], oa[1], oa[2], oa[3]);
    plane_a[2 * i + 1] = make_uint4(oa[4], oa[5], oa[6], oa[7]);
    plane_b[2 * i] = make_uint4(ob[0], ob[1], ob[2], ob[3]);
    plane_b[2 * i + 1] = make_uint4(ob[4], ob[5], ob[6], ob[7]);
}

// The same for the two weight matrices of an MLP in one launch (threads past the first matrix's chunks take the second's).
__global__ __launch_bounds__(256) void decode_w4_pair_kernel(const uint4 *__restrict__ w4_0, long n0, uint4 *__restrict__ a0,
                                                             uint4 *__restrict__ b0, const uint4 *__restrict__ w4_1, long n1,
                                                             uint4 *__restrict__ a1, uint4 *__restrict__ b1) {
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const bool second = i >= n0;
    if (second) i -= n0;
    if (second && i >= n1) return;
    const uint4 wv = second ? w4_1[i] : w4_0[i];
    const uint32_t wd[4] = {wv.x, wv.y, wv.z, wv.w};
    uint32_t oa[8], ob[8];
#pragma unroll
    for (int q = 0; q < 4; ++q) decode8(wd[q], oa + 2 * q, ob + 2 * q);
    uint4 *pa = second ? a1 : a0, *pb = second ? b1 : b0;
    pa[2 * i] = make_uint4(oa[0], oa[1], oa[2], oa[3]);
    pa[2 * i + 1] = make_uint4(oa[4], oa[5], oa[6], oa[7]);
    pb[2 * i] = make_uint4(ob[0], ob[1], ob[2], ob[3]);
    pb[2 * i + 1] = make_uint4(ob[4], ob[5], ob[6], ob[7]);
}

inline Epilogue with_finite_scale(Epilogue e) {
    e.rq = requant_scale_finite(e.rq);
    return e;
}

template <int MODE>
struct ShiftStore {
    static constexpr int kBytes = (MODE == kEpiRequantLut) ? 1 : 4;
    static constexpr int kTableBytes = (MODE == kEpiRequantLut) ? 256 : 0;
    static constexpr bool kScatter = (MODE == kEpiScatterI32);
    static constexpr bool kLinear = (MODE == kEpiLinearF32 || MODE == kEpiQkvCodes);
    static constexpr bool kSignCodes = (MODE == kEpiQkvCodes);
    Epilogue e;
    void *out;             // int32 rows | int8 hidden rows | scattered fp32 rows
    const void *table;     // the 256-entry activation table
    const float *gate;
    bool accumulate;
    float *parts[3];       // kEpiLinearF32: column blocks, residual and scale
    int part_width;
    const float *residual;
    float scale;
    uint64_t *codes[2];    // kEpiQkvCodes: sign codes of column blocks 0 and 1
    int code_cols, head_dim, tokens, heads;
    explicit ShiftStore(const Epilogue &epi)     // epi.rq is made finite here: convert() relies on it
        : e(with_finite_scale(epi)),
          out(MODE == kEpiInt32 ? (void *)epi.y : MODE == kEpiRequantLut ? (void *)epi.h
              : MODE == kEpiLinearF32 ? (void *)epi.parts[0] : MODE == kEpiQkvCodes ? (void *)epi.parts[2] : (void *)epi.yf),
          table(epi.lut),
          gate(MODE == kEpiScatterI32 ? epi.gate : nullptr),
          accumulate(MODE == kEpiScatterI32 && epi.accumulate),
          parts{epi.parts[0], epi.parts[1], epi.parts[2]},
          part_width(epi.part_width > 0 ? epi.part_width : 4),
          residual(epi.residual),
          scale(epi.lin_scale),
          codes{epi.codes[0], epi.codes[1]},
          code_cols(MODE == kEpiQkvCodes ? 2 * epi.part_width : 0),
          head_dim(epi.head_dim > 0 ? epi.head_dim : 64),
          tokens(epi.tokens > 0 ? epi.tokens : 1),
          heads(epi.heads) {}
    __device__ inline uint32_t convert(int32_t acc, int n, const uint8_t *lds_table) const {
        if (MODE == kEpiInt32) return (uint32_t)(acc + (e.bias ? e.bias[n] : 0));
        if (MODE == kEpiRequantLut) return lds_table[requant_index(acc, e.rq)];
        if (MODE == kEpiLinearF32 || MODE == kEpiQkvCodes) return __builtin_bit_cast(uint32_t, (float)acc);   // scaled at the store
        return __builtin_bit_cast(uint32_t, e.out_scale * (float)acc);
    }
};

constexpr int kMfmaK = 32;   // K granularity of the MFMA variant (16 bytes of packed weights, 32 of activations)
// Plane rows are padded with zeros to whole 64-byte LDS stages.
int padded_k(int K) { return (K + 63) / 64 * 64; }
size_t planes_bytes(int K, int N) { return ((size_t)2 * N * padded_k(K) + 255) / 256 * 256; }

int decode_planes(const uint8_t *w4, int K, int N, void *planes, hipStream_t st) {
    const int Kp = padded_k(K);
    int8_t *pa = static_cast<int8_t *>(planes), *pb = pa + (size_t)N * Kp;
    const long n_chunks = (long)N * Kp / 32;
    decode_w4_kernel<<<dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, st>>>(
        reinterpret_cast<const uint4 *>(w4), n_chunks, reinterpret_cast<uint4 *>(pa), reinterpret_cast<uint4 *>(pb), K / 32,
        Kp / 32);
    return check_launch("shift layer (weight decode)");
}

// Both weight matrices of an MLP ([N0, K0] and [N1, K1]) to their planes in one launch.
int decode_planes_pair(const uint8_t *w4_0, int K0, int N0, void *planes0, const uint8_t *w4_1, int K1, int N1, void *planes1,
                       hipStream_t st) {
    int8_t *a0 = static_cast<int8_t *>(planes0), *b0 = a0 + (size_t)N0 * K0;
    int8_t *a1 = static_cast<int8_t *>(planes1), *b1 = a1 + (size_t)N1 * K1;
    const long n0 = (long)N0 * K0 / 32, n1 = (long)N1 * K1 / 32;
    decode_w4_pair_kernel<<<dim3((unsigned)((n0 + n1 + 255) / 256)), dim3(256), 0, st>>>(
        reinterpret_cast<const uint4 *>(w4_0), n0, reinterpret_cast<uint4 *>(a0), reinterpret_cast<uint4 *>(b0),
        reinterpret_cast<const uint4 *>(w4_1), n1, reinterpret_cast<uint4 *>(a1), reinterpret_cast<uint4 *>(b1));
    return check_launch("shift layers (weight decode)");
}

// planes: workspace of planes_bytes(K, N) for the MFMA variant (unused by the VALU and the
// prepared variant; for the latter w4 already points at decoded planes).
// decoded: the planes of w4 are already in `planes` (decoded earlier in this call).
template <int MODE>
int launch_shift(int variant, const int8_t *x, const uint8_t *w4, const RowSel &sel, bool gather, int K,
                 int N, const Epilogue &epi, void *planes, hipStream_t st, bool decoded = false) {
    if (sel.max_rows == 0 || N == 0) return SA_OK;
    if (variant == SA_VARIANT_AUTO) variant = (K % kMfmaK == 0) ? SA_VARIANT_MFMA : SA_VARIANT_VALU;
    if (variant == SA_VARIANT_MFMA || variant == SA_VARIANT_MFMA_PREPARED) {
        SA_REQUIRE(K % kMfmaK == 0, SA_ERR_SHAPE, "shift layer: the MFMA variant needs K %% 32 == 0 (K = %d)", K);
        const int Kp = padded_k(K);
        const int8_t *pa, *pb;
        if (variant == SA_VARIANT_MFMA_PREPARED) {
            pa = reinterpret_cast<const int8_t *>(w4);      // the caller decoded the weights beforehand
        } else {
            if (!decoded) {
                int rc = decode_planes(w4, K, N, planes, st);
                if (rc != SA_OK) return rc;
            }
            pa = static_cast<const int8_t *>(planes);
        }
        pb = pa + (size_t)N * Kp;
        GemmArgs g;
        g.a = x;
        g.b[0] = pa;
        g.b[1] = pb;
        g.sel = sel;
        g.gather_a = gather;
        g.K = Kp;           // the planes' rows are padded with zeros to whole stages; the activation rows are not
        g.a_ld = K;
        g.a_valid = K;
        g.N = N;
        ShiftStore<MODE> store(epi);
        return launch_gemm<I8Traits>(g, store, st, "shift layer (MFMA)");
    }
    const long gy = (sel.max_rows + kValuRows - 1) / kValuRows;
    SA_REQUIRE(gy < 65536, SA_ERR_SHAPE, "shift layer: too many rows for one launch");
    // narrow layers: a workgroup no wider than the columns need (whole wavefronts), so that lanes are not idle
    const int threads = N >= 256 ? 256 : (N + 63) / 64 * 64;
    const dim3 grid((N + threads - 1) / threads, (unsigned)gy);
    shift_valu_kernel<MODE><<<grid, dim3(threads), 0, st>>>(x, w4, sel, gather, K, N, epi);
    return check_launch("shift layer (VALU)");
}

typedef _Float16 v4h_t __attribute__((ext_vector_type(4)));

// q = int8 codes of x * inv_scale; xh (optional) = x rounded to fp16.  Four elements per thread.
__global__ __launch_bounds__(256) void quantize_kernel(const float *__restrict__ x, long n,
                                                       float inv_scale, int8_t *__restrict__ q,
                                                       _Float16 *__restrict__ xh) {
    const long i4 = ((long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i4 + 3 < n) {
        const float4 v = *reinterpret_cast<const float4 *>(x + i4);
        const uint32_t b0 = (uint8_t)requant_code(v.x * inv_scale), b1 = (uint8_t)requant_code(v.y * inv_scale);
        const uint32_t b2 = (uint8_t)requant_code(v.z * inv_scale), b3 = (uint8_t)requant_code(v.w * inv_scale);
        *reinterpret_cast<uint32_t *>(q + i4) = b0 | (b1 << 8) | (b2 << 16) | (b3 << 24);
        if (xh) {
            v4h_t h;
            h[0] = (_Float16)v.x; h[1] = (_Float16)v.y; h[2] = (_Float16)v.z; h[3] = (_Float16)v.w;
            *reinterpret_cast<v4h_t *>(xh + i4) = h;
        }
    } else {
        for (long i = i4; i < n; ++i) {
            q[i] = requant_code(x[i] * inv_scale);
            if (xh) xh[i] = (_Float16)x[i];
        }
    }
}

// One weight -> its 4-bit form (neg << 3) | e, e = clamp(round(log2 |w|), -7, 0) + 7.  log2 |w| is
// never half-way between two integers for a float (2^(n + 1/2) is irrational), so rounding is a
// comparison of the mantissa with that of sqrt(2): integer logic, no transcendental.  The fp32
// neighbours of sqrt(2) are 0x3FB504F3 < sqrt(2) < 0x3FB504F4.
__device__ inline uint32_t weight_nibble(float w) {
    const uint32_t bits = __builtin_bit_cast(uint32_t, w) & 0x7FFFFFFFu;
    int p = (int)(bits >> 23) - 127 + ((bits & 0x7FFFFFu) >= 0x3504F4u ? 1 : 0);   // zero, subnormals: <= -126
    p = p < -7 ? -7 : (p > 0 ? 0 : p);                                              // Inf, NaN: exponent 255 -> 0
    return (uint32_t)(p + 7) | (w < 0.0f ? 8u : 0u);                                // -0 and NaN count as positive
}

// Eight consecutive weights of a row per thread: two 16-byte loads, one 4-byte store.
__global__ __launch_bounds__(256) void pack_weights_kernel(const float *__restrict__ w, long n8,
                                                           uint32_t *__restrict__ w4) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n8) return;
    const float4 a = *reinterpret_cast<const float4 *>(w + 8 * i);
    const float4 b = *reinterpret_cast<const float4 *>(w + 8 * i + 4);
    const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    uint32_t word = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) word |= weight_nibble(v[k]) << (4 * k);      // even k = low nibble of byte k / 2
    w4[i] = word;
}

__global__ __launch_bounds__(256) void requant_lut_kernel(const int32_t *__restrict__ y, long n, float s,
                                                          const int8_t *__restrict__ lut,
                                                          int8_t *__restrict__ h) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) h[i] = lut[(int)requant_code((float)y[i] * s) + 128];
}

}  // namespace

extern "C" size_t sa_shift_planes_bytes(int K, int N) {
    if (K <= 0 || N <= 0 || K % kMfmaK != 0) return 0;
    return planes_bytes(K, N);
}

extern "C" int sa_shift_planes_prepare(const uint8_t *w4, int K, int N, void *planes, size_t planes_bytes_given,
                                       void *stream) {
    sa::clear_error();
    SA_REQUIRE(K > 0 && N > 0, SA_ERR_INVALID, "sa_shift_planes_prepare: K and N must be positive");
    SA_REQUIRE(K % kMfmaK == 0, SA_ERR_SHAPE, "sa_shift_planes_prepare: K (%d) must be a multiple of 32", K);
    SA_REQUIRE(w4 && planes, SA_ERR_INVALID, "sa_shift_planes_prepare: NULL buffer");
    SA_REQUIRE(sa::aligned16(w4) && sa::aligned16(planes), SA_ERR_ALIGN,
               "sa_shift_planes_prepare: pointers must be 16-byte aligned");
    SA_REQUIRE(planes_bytes_given >= planes_bytes(K, N), SA_ERR_WORKSPACE,
               "sa_shift_planes_prepare: %zu bytes needed, %zu given", planes_bytes(K, N), planes_bytes_given);
    return decode_planes(w4, K, N, planes, sa::as_stream(stream));
}

extern "C" int sa_shift_weights_from_float(const float *w, int N, int K, uint8_t *w4, void *stream) {
    sa::clear_error();
    SA_REQUIRE(N >= 0 && K >= 0, SA_ERR_INVALID, "sa_shift_weights_from_float: negative size");
    SA_REQUIRE(K % 8 == 0, SA_ERR_SHAPE, "sa_shift_weights_from_float: K (%d) must be a multiple of 8", K);
    if (N == 0 || K == 0) return SA_OK;
    SA_REQUIRE(w && w4, SA_ERR_INVALID, "sa_shift_weights_from_float: NULL buffer");
    SA_REQUIRE(sa::aligned16(w) && sa::aligned16(w4), SA_ERR_ALIGN,
               "sa_shift_weights_from_float: pointers must be 16-byte aligned");
    const long n8 = (long)N * K / 8;
    const long blocks = (n8 + 255) / 256;
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_shift_weights_from_float: too many weights");
    pack_weights_kernel<<<dim3((unsigned)blocks), dim3(256), 0, sa::as_stream(stream)>>>(
        w, n8, reinterpret_cast<uint32_t *>(w4));
    return sa::check_launch("sa_shift_weights_from_float");
}

extern "C" size_t sa_shift_linear_workspace_bytes(long M, int K, int N, int variant) {
    if (M <= 0 || K <= 0 || N <= 0 || variant == SA_VARIANT_VALU || variant == SA_VARIANT_MFMA_PREPARED) return 0;
    if (K % kMfmaK != 0) return 0;
    return planes_bytes(K, N);
}

extern "C" int sa_shift_linear(const int8_t *x, const uint8_t *w4, const int32_t *bias_or_null,
                               int32_t *y, long M, int K, int N, int variant, void *workspace,
                               size_t workspace_bytes, void *stream) {
    sa::clear_error();
    SA_REQUIRE(M >= 0 && K >= 0 && N >= 0, SA_ERR_INVALID, "sa_shift_linear: negative size");
    SA_REQUIRE(variant >= 0 && variant <= 3, SA_ERR_INVALID, "sa_shift_linear: unknown variant %d", variant);
    SA_REQUIRE(K % 2 == 0, SA_ERR_SHAPE, "sa_shift_linear: K (%d) must be even (two weights per byte)", K);
    SA_REQUIRE(K <= 131072, SA_ERR_SHAPE, "sa_shift_linear: K too large for int32 accumulation");
    SA_REQUIRE(M < (1L << 31), SA_ERR_SHAPE, "sa_shift_linear: M >= 2^31");
    if (M == 0 || N == 0) return SA_OK;
    SA_REQUIRE(x && w4 && y, SA_ERR_INVALID, "sa_shift_linear: NULL buffer");
    SA_REQUIRE(sa::aligned16(x) && sa::aligned16(w4) && sa::aligned16(y) && sa::aligned16(bias_or_null) &&
                   sa::aligned16(workspace),
               SA_ERR_ALIGN, "sa_shift_linear: pointers must be 16-byte aligned");
    SA_REQUIRE(K % 32 == 0, SA_ERR_SHAPE, "sa_shift_linear: K (%d) must be a multiple of 32 (16-byte weight rows)", K);
    if (variant == SA_VARIANT_MFMA || variant == SA_VARIANT_MFMA_PREPARED)
        SA_REQUIRE(K % kMfmaK == 0, SA_ERR_SHAPE, "sa_shift_linear: the MFMA variants need K %% 32 == 0 (K = %d)", K);
    const size_t need = sa_shift_linear_workspace_bytes(M, K, N, variant);
    SA_REQUIRE(need == 0 || (workspace != nullptr && workspace_bytes >= need), SA_ERR_WORKSPACE,
               "sa_shift_linear: workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    sa::Epilogue epi;
    epi.bias = bias_or_null;
    // at most 65535 row tiles per launch: very tall inputs go in slices
    const long rows_per_launch = 65535L * kValuRows;
    for (long m = 0; m < M; m += rows_per_launch) {
        sa::RowSel s2{nullptr, nullptr, 0, (M - m) < rows_per_launch ? (M - m) : rows_per_launch};
        sa::Epilogue e2 = epi;
        e2.y = y + (size_t)m * N;
        int rc = launch_shift<sa::kEpiInt32>(variant, x + (size_t)m * K, w4, s2, false, K, N, e2, workspace,
                                             sa::as_stream(stream));
        if (rc != SA_OK) return rc;
    }
    return SA_OK;
}

extern "C" int sa_shift_linear_f32(const int8_t *x, const uint8_t *w4, long M, int K, int N, int variant,
                                   float scale, const float *residual_or_null, int parts, float *y0, float *y1,
                                   float *y2, void *workspace, size_t workspace_bytes, void *stream) {
    sa::clear_error();
    SA_REQUIRE(M >= 0 && K >= 0 && N >= 0, SA_ERR_INVALID, "sa_shift_linear_f32: negative size");
    SA_REQUIRE(variant >= 0 && variant <= 3, SA_ERR_INVALID, "sa_shift_linear_f32: unknown variant %d", variant);
    SA_REQUIRE(parts >= 1 && parts <= 3, SA_ERR_INVALID, "sa_shift_linear_f32: parts must be 1, 2 or 3");
    SA_REQUIRE(K % 32 == 0, SA_ERR_SHAPE, "sa_shift_linear_f32: K (%d) must be a multiple of 32", K);
    SA_REQUIRE(K <= 131072, SA_ERR_SHAPE, "sa_shift_linear_f32: K too large for int32 accumulation");
    SA_REQUIRE(N % (4 * parts) == 0, SA_ERR_SHAPE,
               "sa_shift_linear_f32: N (%d) must split into %d column blocks of whole 16-byte chunks", N, parts);
    SA_REQUIRE(parts == 1 || residual_or_null == nullptr, SA_ERR_INVALID,
               "sa_shift_linear_f32: a residual needs parts == 1");
    SA_REQUIRE(M < 65535L * kValuRows, SA_ERR_SHAPE, "sa_shift_linear_f32: too many rows for one call");
    if (M == 0 || N == 0) return SA_OK;
    SA_REQUIRE(x && w4 && y0 && (parts < 2 || y1) && (parts < 3 || y2), SA_ERR_INVALID,
               "sa_shift_linear_f32: NULL buffer");
    SA_REQUIRE(sa::aligned16(x) && sa::aligned16(w4) && sa::aligned16(y0) && sa::aligned16(y1) && sa::aligned16(y2) &&
                   sa::aligned16(residual_or_null) && sa::aligned16(workspace),
               SA_ERR_ALIGN, "sa_shift_linear_f32: pointers must be 16-byte aligned");
    if (variant == SA_VARIANT_MFMA || variant == SA_VARIANT_MFMA_PREPARED)
        SA_REQUIRE(K % kMfmaK == 0, SA_ERR_SHAPE, "sa_shift_linear_f32: the MFMA variants need K %% 32 == 0 (K = %d)", K);
    const size_t need = sa_shift_linear_workspace_bytes(M, K, N, variant);
    SA_REQUIRE(need == 0 || (workspace != nullptr && workspace_bytes >= need), SA_ERR_WORKSPACE,
               "sa_shift_linear_f32: workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    sa::Epilogue epi;
    epi.parts[0] = y0;
    epi.parts[1] = parts > 1 ? y1 : y0;
    epi.parts[2] = parts > 2 ? y2 : y0;
    epi.part_width = N / parts;
    epi.residual = residual_or_null;
    epi.lin_scale = scale;
    sa::RowSel sel{nullptr, nullptr, 0, M};
    return launch_shift<sa::kEpiLinearF32>(variant, x, w4, sel, false, K, N, epi, workspace, sa::as_stream(stream));
}

extern "C" int sa_shift_linear_qkv_codes(const int8_t *x, const uint8_t *wqkv, int B, int N, int H, int E, int variant,
                                         float scale, uint64_t *q_codes, uint64_t *k_codes, float *v, void *workspace,
                                         size_t workspace_bytes, void *stream) {
    sa::clear_error();
    SA_REQUIRE(B >= 0 && N >= 0 && H > 0 && E > 0, SA_ERR_INVALID, "sa_shift_linear_qkv_codes: bad size");
    SA_REQUIRE(variant >= 1 && variant <= 3, SA_ERR_UNSUPPORTED,
               "sa_shift_linear_qkv_codes: matrix-core variants only (1, 2 or 3; got %d)", variant);
    SA_REQUIRE(E % H == 0 && (E / H == 64 || E / H == 128), SA_ERR_UNSUPPORTED,
               "sa_shift_linear_qkv_codes: head width E / H must be 64 or 128 (E = %d, H = %d)", E, H);
    SA_REQUIRE(E % 128 == 0, SA_ERR_UNSUPPORTED, "sa_shift_linear_qkv_codes: E (%d) must be a multiple of 128", E);
    SA_REQUIRE(scale > 0.0f && scale - scale == 0.0f, SA_ERR_INVALID,
               "sa_shift_linear_qkv_codes: the scale must be positive and finite (the sign of scale * acc is taken from acc)");
    const long M = (long)B * N;
    SA_REQUIRE(M < 65535L * kValuRows, SA_ERR_SHAPE, "sa_shift_linear_qkv_codes: too many rows for one call");
    if (M == 0) return SA_OK;
    SA_REQUIRE(x && wqkv && q_codes && k_codes && v, SA_ERR_INVALID, "sa_shift_linear_qkv_codes: NULL buffer");
    SA_REQUIRE(sa::aligned16(x) && sa::aligned16(wqkv) && sa::aligned16(q_codes) && sa::aligned16(k_codes) &&
                   sa::aligned16(v) && sa::aligned16(workspace),
               SA_ERR_ALIGN, "sa_shift_linear_qkv_codes: pointers must be 16-byte aligned");
    if (variant == SA_VARIANT_AUTO) variant = SA_VARIANT_MFMA;
    const size_t need = sa_shift_linear_workspace_bytes(M, E, 3 * E, variant);
    SA_REQUIRE(need == 0 || (workspace != nullptr && workspace_bytes >= need), SA_ERR_WORKSPACE,
               "sa_shift_linear_qkv_codes: workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    sa::Epilogue epi;
    epi.parts[0] = epi.parts[1] = epi.parts[2] = v;      // only column block 2 is written as fp32
    epi.part_width = E;
    epi.lin_scale = scale;
    epi.codes[0] = q_codes;
    epi.codes[1] = k_codes;
    epi.head_dim = E / H;
    epi.tokens = N;
    epi.heads = H;
    sa::RowSel sel{nullptr, nullptr, 0, M};
    return launch_shift<sa::kEpiQkvCodes>(variant, x, wqkv, sel, false, E, 3 * E, epi, workspace, sa::as_stream(stream));
}

extern "C" int sa_quantize_act(const float *x, long n, float inv_scale, int8_t *q, void *stream) {
    sa::clear_error();
    return sa_quantize_act_half(x, n, inv_scale, q, nullptr, stream);
}

extern "C" int sa_quantize_act_half(const float *x, long n, float inv_scale, int8_t *q, void *xh_or_null,
                                    void *stream) {
    sa::clear_error();
    SA_REQUIRE(n >= 0, SA_ERR_INVALID, "sa_quantize_act: n < 0");
    if (n == 0) return SA_OK;
    SA_REQUIRE(x && q, SA_ERR_INVALID, "sa_quantize_act: NULL buffer");
    SA_REQUIRE(sa::aligned16(x) && sa::aligned16(q) && sa::aligned16(xh_or_null), SA_ERR_ALIGN,
               "sa_quantize_act: pointers must be 16-byte aligned");
    const long blocks = ((n + 3) / 4 + 255) / 256;
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_quantize_act: n too large");
    quantize_kernel<<<dim3((unsigned)blocks), dim3(256), 0, sa::as_stream(stream)>>>(
        x, n, inv_scale, q, static_cast<_Float16 *>(xh_or_null));
    return sa::check_launch("sa_quantize_act");
}

extern "C" int sa_requant_lut(const int32_t *y, long n, float s, const int8_t *lut, int8_t *h, void *stream) {
    sa::clear_error();
    SA_REQUIRE(n >= 0, SA_ERR_INVALID, "sa_requant_lut: n < 0");
    if (n == 0) return SA_OK;
    SA_REQUIRE(y && lut && h, SA_ERR_INVALID, "sa_requant_lut: NULL buffer");
    SA_REQUIRE(sa::aligned16(y) && sa::aligned16(h) && sa::aligned16(lut), SA_ERR_ALIGN,
               "sa_requant_lut: pointers must be 16-byte aligned");
    const long blocks = (n + 255) / 256;
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_requant_lut: n too large");
    requant_lut_kernel<<<dim3((unsigned)blocks), dim3(256), 0, sa::as_stream(stream)>>>(y, n, s, lut, h);
    return sa::check_launch("sa_requant_lut");
}

// workspace layout of sa_shift_mlp: hidden int8 [max_rows, hid] | planes of w1 | planes of w2
size_t sa::shift_linear_rows_workspace_bytes(int K, int N, int variant) {
    return (variant == SA_VARIANT_VALU || variant == SA_VARIANT_MFMA_PREPARED) ? 0 : planes_bytes(K, N);
}

int sa::shift_linear_rows(const int8_t *xq_all, const RowSel &sel, int K, int N, const uint8_t *w4, float out_scale, float *y,
                          const float *gate, int variant, void *planes, hipStream_t st) {
    SA_REQUIRE((sel.max_rows + kValuRows - 1) / kValuRows < 65536 || variant != SA_VARIANT_VALU, SA_ERR_SHAPE,
               "sa_moe_linear: too many rows for the VALU variant in one call");
    sa::Epilogue e;
    e.yf = y;
    e.gate = gate;
    e.out_scale = out_scale;
    return launch_shift<sa::kEpiScatterI32>(variant, xq_all, w4, sel, true, K, N, e, planes, st);
}

extern "C" size_t sa_shift_mlp_workspace_bytes(long max_rows, int E, int hid) {
    if (max_rows <= 0 || hid <= 0 || E <= 0) return 0;
    const size_t hidden = (((size_t)max_rows * hid) + 255) / 256 * 256;
    return hidden + 2 * planes_bytes(E, hid);
}

extern "C" int sa_shift_mlp(const int8_t *xq, const sa_rows *rows, int E, int hid, const uint8_t *w1,
                            const uint8_t *w2, float requant_scale, const int8_t *lut,
                            int32_t *y2_or_null, float *y_or_null, const float *gate_or_null,
                            float out_scale, int variant, int stages, void *workspace,
                            size_t workspace_bytes, void *stream) {
    sa::clear_error();
    sa::RowSel sel;
    int rc = sa::validate_rows(rows, &sel);
    if (rc != SA_OK) return rc;
    SA_REQUIRE(E > 0 && hid > 0, SA_ERR_INVALID, "sa_shift_mlp: E and hid must be positive");
    SA_REQUIRE(variant >= 0 && variant <= 3, SA_ERR_INVALID, "sa_shift_mlp: unknown variant %d", variant);
    SA_REQUIRE(E % 64 == 0 && hid % 64 == 0, SA_ERR_SHAPE,
               "sa_shift_mlp: E (%d) and hid (%d) must be multiples of 64", E, hid);
    SA_REQUIRE(E <= 131072 && hid <= 131072, SA_ERR_SHAPE, "sa_shift_mlp: width too large");
    if (sel.max_rows == 0) return SA_OK;
    SA_REQUIRE(xq && w1 && w2 && lut, SA_ERR_INVALID, "sa_shift_mlp: NULL buffer");
    SA_REQUIRE((stages & 3) != 0 && (stages & ~(3 | SA_MLP_ACCUMULATE)) == 0, SA_ERR_INVALID,
               "sa_shift_mlp: stages must be 1, 2 or 3, optionally | SA_MLP_ACCUMULATE");
    SA_REQUIRE(!(stages & 2) || y2_or_null || y_or_null, SA_ERR_INVALID, "sa_shift_mlp: no output requested");
    SA_REQUIRE(sa::aligned16(xq) && sa::aligned16(w1) && sa::aligned16(w2) && sa::aligned16(lut) &&
                   sa::aligned16(y2_or_null) && sa::aligned16(y_or_null) && sa::aligned16(gate_or_null) &&
                   sa::aligned16(workspace) && sa::aligned4(sel.rows),
               SA_ERR_ALIGN, "sa_shift_mlp: pointers must be 16-byte aligned");
    const size_t need = sa_shift_mlp_workspace_bytes(sel.max_rows, E, hid);
    SA_REQUIRE(workspace != nullptr && workspace_bytes >= need, SA_ERR_WORKSPACE,
               "sa_shift_mlp: workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    SA_REQUIRE((sel.max_rows + kValuRows - 1) / kValuRows < 65536 || variant != SA_VARIANT_VALU, SA_ERR_SHAPE,
               "sa_shift_mlp: too many rows for the VALU variant in one call");
    hipStream_t st = sa::as_stream(stream);
    int8_t *hbuf = static_cast<int8_t *>(workspace);
    uint8_t *planes1 = static_cast<uint8_t *>(workspace) + (((size_t)sel.max_rows * hid) + 255) / 256 * 256;
    uint8_t *planes2 = planes1 + planes_bytes(E, hid);

    // both layers in this call on the matrix cores: their 4-bit weights are decoded by one launch
    const int v_eff = variant == SA_VARIANT_AUTO ? SA_VARIANT_MFMA : variant;      // E and hid are multiples of 64
    const bool pair = v_eff == SA_VARIANT_MFMA && (stages & 3) == 3;
    if (pair) {
        rc = decode_planes_pair(w1, E, hid, planes1, w2, hid, E, planes2, st);
        if (rc != SA_OK) return rc;
    }
    if (stages & 1) {
        sa::Epilogue e1;
        e1.h = hbuf;
        e1.rq = requant_scale;
        e1.lut = lut;
        rc = launch_shift<sa::kEpiRequantLut>(variant, xq, w1, sel, true, E, hid, e1, planes1, st, pair);
        if (rc != SA_OK) return rc;
    }
    if (!(stages & 2)) return SA_OK;

    if (y2_or_null) {
        sa::Epilogue e2;
        e2.y = y2_or_null;
        rc = launch_shift<sa::kEpiInt32>(variant, hbuf, w2, sel, false, hid, E, e2, planes2, st, pair);
        if (rc != SA_OK) return rc;
    }
    if (y_or_null) {
        sa::Epilogue e3;
        e3.yf = y_or_null;
        e3.gate = gate_or_null;
        e3.out_scale = out_scale;
        e3.accumulate = (stages & SA_MLP_ACCUMULATE) != 0;
        rc = launch_shift<sa::kEpiScatterI32>(variant, hbuf, w2, sel, false, hid, E, e3, planes2, st, pair || y2_or_null != nullptr);
        if (rc != SA_OK) return rc;
    }
    return SA_OK;
}
