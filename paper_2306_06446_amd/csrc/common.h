// Internal helpers of libshiftadd (host-side validation, error text, launch checks).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "shiftadd.h"

namespace sa {

// Records a message for sa_last_error() and returns `code`.
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

// Turns the status of the launch just issued into an SA code.
int check_launch(const char *what);

// Zero-fills `bytes` (a multiple of 4) with a kernel (safe under graph capture).
int launch_zero(void *p, size_t bytes, hipStream_t st);

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

constexpr int kWave = 64;

// Resolves an sa_rows descriptor inside a kernel (all lanes get the same values).
struct RowSel {
    const int32_t *rows;    // may be null: identity
    const int32_t *counts;  // may be null: n_rows = max_rows
    int expert;
    long max_rows;
};

__device__ inline void resolve_rows(const RowSel &sel, const int32_t *&rows, long &n_rows) {
    rows = sel.rows;
    n_rows = sel.max_rows;
    if (sel.counts != nullptr) {
        long off = 0;
        for (int e = 0; e < sel.expert; ++e) off += sel.counts[e];
        long cnt = sel.counts[sel.expert];
        rows = sel.rows + off;
        n_rows = cnt < sel.max_rows ? cnt : sel.max_rows;
    }
}

int validate_rows(const sa_rows *rows, RowSel *out);

// One Linear layer on the rows an expert was given, gated and scattered (the two experts of sa_moe_linear):
//   y[rows[i], :] = gate[rows[i]] * (xh[rows[i], :] . W^T)                      fp16 operands   (mult_mlp.hip)
//   y[rows[i], :] = gate[rows[i]] * out_scale * (xq[rows[i], :] . Wshift^T)      int8 / 4-bit    (shift_linear.hip)
// Arguments are checked by the caller; `planes` is shift_linear_rows_workspace_bytes(K, N, variant) bytes.
int mult_linear_rows(const void *xh_all, const RowSel &sel, int K, int N, const void *w_f16, float *y, const float *gate,
                     hipStream_t st);
size_t shift_linear_rows_workspace_bytes(int K, int N, int variant);
int shift_linear_rows(const int8_t *xq_all, const RowSel &sel, int K, int N, const uint8_t *w4, float out_scale, float *y,
                      const float *gate, int variant, void *planes, hipStream_t st);
// The routing of sa_moe_dispatch without its argument checks (moe.hip).
size_t moe_dispatch_scratch_bytes(long T, int E);
int moe_dispatch_launch(const float *logits, long T, int E, int32_t *perm, int32_t *expert_of, int32_t *counts, float *gate,
                        void *scratch, hipStream_t st);

// Hash pre-pass on the matrix cores with exact fallback (binarize_mfma.hip).
bool binarize_mfma_supported(int d, int nbits);
int launch_binarize_mfma(const float *x0, const float *x1_or_null, const float *proj, uint64_t *codes0,
                         uint64_t *codes1_or_null, long rows, int N, int H, int d, int nbits, hipStream_t st);

// Additive attention on the matrix cores (additive_mfma.hip).
struct AdditiveMfmaPlan {
    int groups;             // groups of up to 4 code words
    int wb, ph;             // words per workgroup, token phases per word
    int splits;             // token ranges (partial K^T V each)
    int tokens_per_block;
};
bool additive_mfma_ktv_supported(int nbits, int dv);
bool additive_mfma_qkv_supported(int nbits, int dv);
AdditiveMfmaPlan plan_additive_mfma(int B, int H, int Nk, int nbits);
// zero_one: a clear code bit stands for 0 instead of -1; den (with zero_one): int32 [B*H, Nq] row normaliser, the
// output row is then acc / (den + eps) instead of scale * acc.
int launch_ktv_mfma(const uint64_t *k_codes, const float *v, float *dst, int B, int H, int Nk, int nbits, int dv,
                    const AdditiveMfmaPlan &p, bool zero_one, hipStream_t st);
int launch_qkv_mfma(const uint64_t *q_codes, const float *kv, float *out, int B, int H, int Nq, int nbits, int dv,
                    float scale, bool zero_one, const int32_t *den, float eps, hipStream_t st);

}  // namespace sa

#define SA_REQUIRE(cond, code, ...) \
    do {                            \
        if (!(cond)) return ::sa::fail((code), __VA_ARGS__); \
    } while (0)
