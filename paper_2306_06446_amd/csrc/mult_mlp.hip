// sa_mult_mlp_f16: the Mult expert (Sec. 4.2), a dense two-layer MLP with erf-GELU,
// fp16 operands, fp32 accumulation on the matrix cores (v_mfma_f32_32x32x16_f16).
//   hidden = half(gelu(half(x[rows]) * W1^T)),   out = hidden * W2^T
// This is the one step of the block that the method keeps as a true dense
// multiplication, so it is a plain tiled MFMA GEMM: 128x128 workgroup tile,
// 4 wavefronts of 64x64, K staged through LDS 32 halves at a time.
#include "common.h"
#include "gemm_common.h"

namespace {

using namespace sa;

constexpr int BM = 128, BN = 128, BKB = 64;    // BKB: bytes of K per stage (32 halves)
constexpr int LDS_STRIDE = BKB + 16;

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

__device__ inline float gelu_erf(float a) { return 0.5f * a * (1.0f + erff(a * 0.70710678118654752f)); }

// A_F32: A rows are fp32 (converted to fp16 on the way into LDS) and may be gathered.
template <bool A_F32, int MODE>
__global__ __launch_bounds__(256) void mult_gemm_kernel(const void *__restrict__ a_ptr,
                                                        const _Float16 *__restrict__ w, RowSel sel,
                                                        int K, int N, Epilogue epi) {
    __shared__ __attribute__((aligned(16))) uint8_t As[BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) uint8_t Bs[BN * LDS_STRIDE];

    const int32_t *rows;
    long n_rows;
    resolve_rows(sel, rows, n_rows);
    const long m0 = (long)blockIdx.y * BM;
    if (m0 >= n_rows) return;
    const int n0 = blockIdx.x * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;

    // A staging: fp32 source: 128 rows x 8 chunks (4 floats); fp16 source: 128 rows x 4 chunks (8 halves)
    constexpr int A_CHUNKS = A_F32 ? 4 : 2;
    const uint8_t *a_src[A_CHUNKS];
    bool a_ok[A_CHUNKS];
    int a_dst[A_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
        const int c = tid + 256 * i;
        const int r = A_F32 ? (c >> 3) : (c >> 2);
        const int col = A_F32 ? (c & 7) : (c & 3);
        const long m = m0 + r;
        a_ok[i] = m < n_rows;
        long src = 0;
        if (a_ok[i]) src = (A_F32 && rows) ? (long)rows[m] : m;
        if (A_F32) {
            a_src[i] = static_cast<const uint8_t *>(a_ptr) + ((size_t)src * K + col * 4) * 4;
            a_dst[i] = r * LDS_STRIDE + col * 8;
        } else {
            a_src[i] = static_cast<const uint8_t *>(a_ptr) + ((size_t)src * K + col * 8) * 2;
            a_dst[i] = r * LDS_STRIDE + col * 16;
        }
    }
    const uint8_t *b_src[2];
    bool b_ok[2];
    int b_dst[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = tid + 256 * i;
        const int r = c >> 2, col = c & 3;
        b_ok[i] = (n0 + r) < N;
        b_src[i] = reinterpret_cast<const uint8_t *>(w) + ((size_t)(b_ok[i] ? n0 + r : 0) * K + col * 8) * 2;
        b_dst[i] = r * LDS_STRIDE + col * 16;
    }

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int frag_row = lane & 31, frag_k = (lane >> 5) * 16;
    const int k_stage = 32;   // halves per stage

    for (int k0 = 0; k0 < K; k0 += k_stage) {
        uint4 av[A_CHUNKS], bv[2];
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i)
            av[i] = a_ok[i] ? *reinterpret_cast<const uint4 *>(a_src[i] + (size_t)k0 * (A_F32 ? 4 : 2))
                            : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 2; ++i)
            bv[i] = b_ok[i] ? *reinterpret_cast<const uint4 *>(b_src[i] + (size_t)k0 * 2) : make_uint4(0, 0, 0, 0);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            if (A_F32) {
                const float4 f = __builtin_bit_cast(float4, av[i]);
                v4h hv;
                hv[0] = (_Float16)f.x; hv[1] = (_Float16)f.y; hv[2] = (_Float16)f.z; hv[3] = (_Float16)f.w;
                *reinterpret_cast<v4h *>(As + a_dst[i]) = hv;
            } else {
                *reinterpret_cast<uint4 *>(As + a_dst[i]) = av[i];
            }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<uint4 *>(Bs + b_dst[i]) = bv[i];
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BKB; kk += 32) {
            v8h af[2], bf[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                af[i] = *reinterpret_cast<const v8h *>(As + (wm + i * 32 + frag_row) * LDS_STRIDE + kk + frag_k);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                bf[j] = *reinterpret_cast<const v8h *>(Bs + (wn + j * 32 + frag_row) * LDS_STRIDE + kk + frag_k);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
    }

#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const long m = m0 + wm + i * 32 + mfma32_row(r, lane);
                if (m >= n_rows || n >= N) continue;
                const float a = acc[i][j][r];
                if (MODE == kEpiGeluHalf) {
                    epi.hh[(size_t)m * N + n] = (_Float16)gelu_erf(a);
                } else if (MODE == kEpiFloat) {
                    epi.of[(size_t)m * N + n] = a;
                } else {
                    const long t = rows ? rows[m] : m;
                    const float g = epi.gate ? epi.gate[t] : 1.0f;
                    epi.yf[(size_t)t * N + n] = g * a;
                }
            }
        }
}

}  // namespace

extern "C" size_t sa_mult_mlp_workspace_bytes(long max_rows, int E, int hid) {
    if (max_rows <= 0 || hid <= 0) return 0;
    return (((size_t)max_rows * hid * 2) + 255) / 256 * 256;
}

extern "C" int sa_mult_mlp_f16(const float *x, const sa_rows *rows, int E, int hid, const void *w1_f16,
                               const void *w2_f16, float *out_or_null, float *y_or_null,
                               const float *gate_or_null, int stages, void *workspace,
                               size_t workspace_bytes, void *stream) {
    sa::clear_error();
    sa::RowSel sel;
    int rc = sa::validate_rows(rows, &sel);
    if (rc != SA_OK) return rc;
    SA_REQUIRE(E > 0 && hid > 0, SA_ERR_INVALID, "sa_mult_mlp_f16: E and hid must be positive");
    SA_REQUIRE(E % 32 == 0 && hid % 32 == 0, SA_ERR_SHAPE,
               "sa_mult_mlp_f16: E (%d) and hid (%d) must be multiples of 32", E, hid);
    if (sel.max_rows == 0) return SA_OK;
    SA_REQUIRE(x && w1_f16 && w2_f16, SA_ERR_INVALID, "sa_mult_mlp_f16: NULL buffer");
    SA_REQUIRE(stages >= 1 && stages <= 3, SA_ERR_INVALID, "sa_mult_mlp_f16: stages must be 1, 2 or 3");
    SA_REQUIRE(!(stages & 2) || out_or_null || y_or_null, SA_ERR_INVALID, "sa_mult_mlp_f16: no output requested");
    SA_REQUIRE(sa::aligned16(x) && sa::aligned16(w1_f16) && sa::aligned16(w2_f16) && sa::aligned16(out_or_null) &&
                   sa::aligned16(y_or_null) && sa::aligned16(gate_or_null) && sa::aligned16(workspace) && sa::aligned4(sel.rows),
               SA_ERR_ALIGN, "sa_mult_mlp_f16: pointers must be 16-byte aligned");
    const size_t need = sa_mult_mlp_workspace_bytes(sel.max_rows, E, hid);
    SA_REQUIRE(workspace != nullptr && workspace_bytes >= need, SA_ERR_WORKSPACE,
               "sa_mult_mlp_f16: workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    const long gy = (sel.max_rows + BM - 1) / BM;
    SA_REQUIRE(gy < 65536, SA_ERR_SHAPE, "sa_mult_mlp_f16: too many rows");
    hipStream_t st = sa::as_stream(stream);
    _Float16 *hbuf = static_cast<_Float16 *>(workspace);
    const _Float16 *w1 = static_cast<const _Float16 *>(w1_f16), *w2 = static_cast<const _Float16 *>(w2_f16);

    if (stages & 1) {
        sa::Epilogue e1;
        e1.hh = hbuf;
        mult_gemm_kernel<true, sa::kEpiGeluHalf><<<dim3((hid + BN - 1) / BN, (unsigned)gy), dim3(256), 0, st>>>(
            x, w1, sel, E, hid, e1);
        rc = sa::check_launch("sa_mult_mlp_f16(fc1)");
        if (rc != SA_OK) return rc;
    }
    if (!(stages & 2)) return SA_OK;
    const dim3 grid2((E + BN - 1) / BN, (unsigned)gy);
    if (out_or_null) {
        sa::Epilogue e2;
        e2.of = out_or_null;
        mult_gemm_kernel<false, sa::kEpiFloat><<<grid2, dim3(256), 0, st>>>(hbuf, w2, sel, hid, E, e2);
        rc = sa::check_launch("sa_mult_mlp_f16(fc2)");
        if (rc != SA_OK) return rc;
    }
    if (y_or_null) {
        sa::Epilogue e3;
        e3.yf = y_or_null;
        e3.gate = gate_or_null;
        mult_gemm_kernel<false, sa::kEpiScatterF32><<<grid2, dim3(256), 0, st>>>(hbuf, w2, sel, hid, E, e3);
        rc = sa::check_launch("sa_mult_mlp_f16(fc2 scatter)");
        if (rc != SA_OK) return rc;
    }
    return SA_OK;
}
