// sa_mult_mlp_f16: the Mult expert (Sec. 4.2), a dense two-layer MLP with erf-GELU,
// fp16 operands, fp32 accumulation on the matrix cores (v_mfma_f32_32x32x16_f16).
//   hidden = half(gelu(half(x[rows]) * W1^T)),   out = hidden * W2^T
// This is the one step of the block that the method keeps as a true dense
// multiplication, so it runs on the shared tiled MFMA GEMM.  A small kernel first
// gathers the expert's fp32 rows and rounds them to fp16.
#include "common.h"
#include "gemm_common.h"
#include "gemm_mfma.h"

namespace {

using namespace sa;

__device__ inline float gelu_erf(float a) { return 0.5f * a * (1.0f + erff(a * 0.70710678118654752f)); }

typedef _Float16 v4h __attribute__((ext_vector_type(4)));

// xh[i, :] = half(x[rows[i], :]); one thread per 4 elements.
__global__ __launch_bounds__(256) void gather_half_kernel(const float4 *__restrict__ x, int E4, RowSel sel,
                                                          v4h *__restrict__ xh) {
    const int32_t *rows;
    long n_rows;
    resolve_rows(sel, rows, n_rows);
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long i = idx / E4;
    const int c = (int)(idx % E4);
    if (i >= n_rows) return;
    const long t = rows ? rows[i] : i;
    const float4 f = x[(size_t)t * E4 + c];
    v4h h;
    h[0] = (_Float16)f.x; h[1] = (_Float16)f.y; h[2] = (_Float16)f.z; h[3] = (_Float16)f.w;
    xh[(size_t)i * E4 + c] = h;
}

template <int MODE>
struct MultStore {
    static constexpr int kBytes = (MODE == kEpiGeluHalf) ? 2 : 4;
    static constexpr int kTableBytes = 0;
    static constexpr bool kScatter = (MODE == kEpiScatterF32);
    static constexpr bool kLinear = false;
    static constexpr bool kSignCodes = false;
    void *out;                      // compact fp32 rows | fp16 hidden rows | scattered fp32 rows
    const void *table = nullptr;
    const float *gate;
    bool accumulate;
    explicit MultStore(const Epilogue &epi)
        : out(MODE == kEpiFloat ? (void *)epi.of : MODE == kEpiGeluHalf ? (void *)epi.hh : (void *)epi.yf),
          gate(MODE == kEpiScatterF32 ? epi.gate : nullptr),
          accumulate(MODE == kEpiScatterF32 && epi.accumulate) {}
    __device__ inline uint32_t convert(float a, int, const uint8_t *) const {
        if (MODE == kEpiGeluHalf) return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)gelu_erf(a));
        return __builtin_bit_cast(uint32_t, a);
    }
};

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

// workspace: fp16 hidden rows [max_rows, hid] | fp16 input rows [max_rows, E]
extern "C" size_t sa_mult_mlp_workspace_bytes(long max_rows, int E, int hid) {
    if (max_rows <= 0 || hid <= 0 || E <= 0) return 0;
    return up256((size_t)max_rows * hid * 2) + up256((size_t)max_rows * E * 2);
}

namespace {

// Both layers.  Either x (fp32, gathered and rounded to fp16 by a small kernel first) or
// xh_all (fp16 rows of every token, picked by `sel` inside the GEMM) is given.
int mult_mlp_impl(const float *x, const _Float16 *xh_all, const sa::RowSel &sel, int E, int hid, const void *w1_f16,
                  const void *w2_f16, float *out_or_null, float *y_or_null, const float *gate_or_null, int stages,
                  void *workspace, hipStream_t st) {
    int rc;
    _Float16 *hbuf = static_cast<_Float16 *>(workspace);
    _Float16 *xh = reinterpret_cast<_Float16 *>(static_cast<uint8_t *>(workspace) +
                                                 up256((size_t)sel.max_rows * hid * 2));
    if (stages & 1) {
        sa::GemmArgs g;
        if (xh_all) {
            g.a = xh_all;
            g.gather_a = true;
        } else {
            const long total = sel.max_rows * (E / 4);
            const long blocks = (total + 255) / 256;
            SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_mult_mlp_f16: too many rows");
            gather_half_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(reinterpret_cast<const float4 *>(x),
                                                                             E / 4, sel, reinterpret_cast<v4h *>(xh));
            rc = sa::check_launch("sa_mult_mlp_f16(gather)");
            if (rc != SA_OK) return rc;
            g.a = xh;
            g.gather_a = false;
        }
        g.b[0] = w1_f16;
        g.b[1] = nullptr;
        g.sel = sel;
        g.K = E;
        g.N = hid;
        sa::Epilogue e1;
        e1.hh = hbuf;
        MultStore<sa::kEpiGeluHalf> s1(e1);
        rc = sa::launch_gemm<sa::F16Traits>(g, s1, st, "sa_mult_mlp_f16(fc1)");
        if (rc != SA_OK) return rc;
    }
    if (!(stages & 2)) return SA_OK;
    sa::GemmArgs g2;
    g2.a = hbuf;
    g2.b[0] = w2_f16;
    g2.b[1] = nullptr;
    g2.sel = sel;
    g2.gather_a = false;
    g2.K = hid;
    g2.N = E;
    if (out_or_null) {
        sa::Epilogue e2;
        e2.of = out_or_null;
        MultStore<sa::kEpiFloat> s2(e2);
        rc = sa::launch_gemm<sa::F16Traits>(g2, s2, st, "sa_mult_mlp_f16(fc2)");
        if (rc != SA_OK) return rc;
    }
    if (y_or_null) {
        sa::Epilogue e3;
        e3.yf = y_or_null;
        e3.gate = gate_or_null;
        e3.accumulate = (stages & SA_MLP_ACCUMULATE) != 0;
        MultStore<sa::kEpiScatterF32> s3(e3);
        rc = sa::launch_gemm<sa::F16Traits>(g2, s3, st, "sa_mult_mlp_f16(fc2 scatter)");
        if (rc != SA_OK) return rc;
    }
    return SA_OK;
}

int check_mult_args(const void *x, const sa_rows *rows, sa::RowSel *sel, int E, int hid, const void *w1_f16,
                    const void *w2_f16, float *out_or_null, float *y_or_null, const float *gate_or_null, int stages,
                    void *workspace, size_t workspace_bytes) {
    int rc = sa::validate_rows(rows, sel);
    if (rc != SA_OK) return rc;
    SA_REQUIRE(E > 0 && hid > 0, SA_ERR_INVALID, "sa_mult_mlp_f16: E and hid must be positive");
    SA_REQUIRE(E % 32 == 0 && hid % 32 == 0, SA_ERR_SHAPE,
               "sa_mult_mlp_f16: E (%d) and hid (%d) must be multiples of 32", E, hid);
    if (sel->max_rows == 0) return SA_OK;
    SA_REQUIRE(x && w1_f16 && w2_f16, SA_ERR_INVALID, "sa_mult_mlp_f16: NULL buffer");
    SA_REQUIRE((stages & 3) != 0 && (stages & ~(3 | SA_MLP_ACCUMULATE)) == 0, SA_ERR_INVALID,
               "sa_mult_mlp_f16: stages must be 1, 2 or 3, optionally | SA_MLP_ACCUMULATE");
    SA_REQUIRE(!(stages & 2) || out_or_null || y_or_null, SA_ERR_INVALID, "sa_mult_mlp_f16: no output requested");
    SA_REQUIRE(sa::aligned16(x) && sa::aligned16(w1_f16) && sa::aligned16(w2_f16) && sa::aligned16(out_or_null) &&
                   sa::aligned16(y_or_null) && sa::aligned16(gate_or_null) && sa::aligned16(workspace) &&
                   sa::aligned4(sel->rows),
               SA_ERR_ALIGN, "sa_mult_mlp_f16: pointers must be 16-byte aligned");
    const size_t need = sa_mult_mlp_workspace_bytes(sel->max_rows, E, hid);
    SA_REQUIRE(workspace != nullptr && workspace_bytes >= need, SA_ERR_WORKSPACE,
               "sa_mult_mlp_f16: workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    return SA_OK;
}

}  // namespace

int sa::mult_linear_rows(const void *xh_all, const RowSel &sel, int K, int N, const void *w_f16, float *y, const float *gate,
                         hipStream_t st) {
    sa::GemmArgs g;
    g.a = xh_all;
    g.gather_a = true;
    g.b[0] = w_f16;
    g.b[1] = nullptr;
    g.sel = sel;
    g.K = K;
    g.N = N;
    sa::Epilogue e;
    e.yf = y;
    e.gate = gate;
    MultStore<sa::kEpiScatterF32> store(e);
    return sa::launch_gemm<sa::F16Traits>(g, store, st, "sa_moe_linear(mult expert)");
}

extern "C" int sa_mult_mlp_f16(const float *x, const sa_rows *rows, int E, int hid, const void *w1_f16,
                               const void *w2_f16, float *out_or_null, float *y_or_null,
                               const float *gate_or_null, int stages, void *workspace,
                               size_t workspace_bytes, void *stream) {
    sa::clear_error();
    sa::RowSel sel;
    int rc = check_mult_args(x, rows, &sel, E, hid, w1_f16, w2_f16, out_or_null, y_or_null, gate_or_null, stages,
                             workspace, workspace_bytes);
    if (rc != SA_OK || sel.max_rows == 0) return rc;
    return mult_mlp_impl(x, nullptr, sel, E, hid, w1_f16, w2_f16, out_or_null, y_or_null, gate_or_null, stages,
                         workspace, sa::as_stream(stream));
}

extern "C" int sa_mult_mlp_f16_half(const void *xh_all, const sa_rows *rows, int E, int hid, const void *w1_f16,
                                    const void *w2_f16, float *out_or_null, float *y_or_null,
                                    const float *gate_or_null, int stages, void *workspace,
                                    size_t workspace_bytes, void *stream) {
    sa::clear_error();
    sa::RowSel sel;
    int rc = check_mult_args(xh_all, rows, &sel, E, hid, w1_f16, w2_f16, out_or_null, y_or_null, gate_or_null,
                             stages, workspace, workspace_bytes);
    if (rc != SA_OK || sel.max_rows == 0) return rc;
    return mult_mlp_impl(nullptr, static_cast<const _Float16 *>(xh_all), sel, E, hid, w1_f16, w2_f16, out_or_null,
                         y_or_null, gate_or_null, stages, workspace, sa::as_stream(stream));
}
